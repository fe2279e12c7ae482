// Refinement of a row permutation by proposed exchanges (arXiv 2302.06058 leaves permutations
// better than random ones to future work, Limitations; the objective is the eligible-block
// count of Sec. 3.3 / Alg. 1).  Proposal t exchanges the entries at two positions of P and is
// kept only if the count grows strictly; proposals are taken in order, each against the
// permutation the earlier ones left.
//
// An exchange between blocks A and B of M permuted rows changes the count of those two blocks
// only, so a proposal costs 2M mask rows, not the matrix, and two proposals that share no block
// commute.  One workgroup of 8 wavefronts owns the permutation (in LDS).  Each round takes up to
// 64 proposals in order: wavefront w evaluates up to 8 of them against the current permutation
// (lanes stride over the 32-column words of the 2M rows, add the M - 1 unchanged rows of each
// block bit-sliced, add either exchanged row on top, compare with N and pop-count the four
// eligibility words; a wavefront reduction gives the change of the count).  Then every wavefront
// decides the round the same way, in order: a proposal that shares a block with an earlier
// proposal of the round that was kept (its evaluation is stale) or deferred (it must not
// overtake it) is deferred; any other is kept if its change is positive and dropped otherwise.
// Deferred proposals open the next round, in their order, ahead of fresh ones.  Proposals that
// share a block therefore never change their relative order, the ones that do not commute, so the
// result equals taking the proposals one by one.  The first proposal of a round is always
// decided, so the loop ends.  Integer only: the result is bit-reproducible.
#include <atomic>

#include "common.hpp"

namespace bimask {
namespace {

constexpr int kRefineThreads = 512;
constexpr int kRefineWaves = kRefineThreads / 64;
constexpr int kRefineChunk = 1024;                       // proposals staged in LDS at a time

template <int M> struct RefinePlanes { static constexpr int L = M == 4 ? 3 : (M == 8 ? 4 : 5); };

// c += w, one counter per bit column, planes least significant first
template <int L>
__device__ __forceinline__ void add_word(uint32_t (&c)[L], uint32_t w) {
#pragma unroll
    for (int k = 0; k < L; ++k) {
        const uint32_t t = c[k] & w;
        c[k] ^= w;
        w = t;
    }
}

// bit columns of (c + w) that hold at most N
template <int L>
__device__ __forceinline__ uint32_t at_most(const uint32_t (&c)[L], uint32_t w, int N) {
    uint32_t s[L];
#pragma unroll
    for (int k = 0; k < L; ++k) s[k] = c[k];
    add_word<L>(s, w);
    uint32_t gt = 0u, eq = ~0u;
#pragma unroll
    for (int k = L - 1; k >= 0; --k) {
        const uint32_t nk = (N >> k) & 1 ? ~0u : 0u;
        gt |= eq & s[k] & ~nk;
        eq &= ~(s[k] ^ nk);
    }
    return ~gt;
}

// Change of the eligible-block count for the proposals wave * PPWX + p (p < PPWX) of a round of nb, evaluated
// against the permutation in sP; results to the round's LDS arrays.  The round's first npend proposals are the
// ones deferred by the round before (sPend), the others come from the staged stream (sSw, from `first`).
template <int M, int PPWX>
__device__ __forceinline__ void refine_evaluate(const uint32_t* __restrict__ Bm, int I, int words, int N,
                                                const int32_t* sP, const int32_t* sPend, int npend,
                                                const int32_t* sSw, int first, int nb, int wave, int lane,
                                                int* sDelta, int* sKa, int* sKb, int* sPa, int* sPb) {
    constexpr int L = RefinePlanes<M>::L;
    constexpr int SH = M == 4 ? 2 : (M == 8 ? 3 : 4);
    // proposals wave * PPWX + p; one that changes nothing (outside [0, I), both positions in one
    // block, beyond the round) is evaluated on positions 0 and 0 and its result dropped
    int a[PPWX], b[PPWX], ka[PPWX], kb[PPWX], d[PPWX];
    bool live[PPWX];
    uint32_t ra[PPWX][M], rb[PPWX][M];
#pragma unroll
    for (int p = 0; p < PPWX; ++p) {
        const int q = wave * PPWX + p;
        const int32_t* src = q < npend ? sPend + 2 * q : sSw + 2 * (first + q - npend);
        a[p] = q < nb ? src[0] : -1;
        b[p] = q < nb ? src[1] : -1;
        const bool valid = a[p] >= 0 && a[p] < I && b[p] >= 0 && b[p] < I;
        live[p] = valid && (a[p] >> SH) != (b[p] >> SH);
        const int ac = live[p] ? a[p] : 0, bc = live[p] ? b[p] : 0;
        ka[p] = ac >> SH;
        kb[p] = bc >> SH;
        // word offsets of the rows: I * words < 2^31 is checked on the host
#pragma unroll
        for (int m = 0; m < M; ++m) {
            ra[p][m] = static_cast<uint32_t>(sP[ka[p] * M + m]) * words;
            rb[p][m] = static_cast<uint32_t>(sP[kb[p] * M + m]) * words;
        }
        d[p] = 0;
    }
    for (int w0 = 0; w0 < words; w0 += 64) {     // uniform trip count
        const bool in = w0 + lane < words;
        const uint32_t w = in ? w0 + lane : 0;
        // all loads of the round first, then the arithmetic: a round costs one memory round trip
        uint32_t xa[PPWX][M], xb[PPWX][M];
#pragma unroll
        for (int p = 0; p < PPWX; ++p) {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                xa[p][m] = Bm[ra[p][m] + w];
                xb[p][m] = Bm[rb[p][m] + w];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int p = 0; p < PPWX; ++p) {
            const int ma = a[p] & (M - 1), mb = b[p] & (M - 1);
            uint32_t cA[L], cB[L], wa = 0u, wb = 0u;   // wa, wb: the two exchanged rows
#pragma unroll
            for (int k = 0; k < L; ++k) cA[k] = cB[k] = 0u;
#pragma unroll
            for (int m = 0; m < M; ++m) {
                add_word<L>(cA, m == ma ? 0u : xa[p][m]);
                add_word<L>(cB, m == mb ? 0u : xb[p][m]);
                wa |= m == ma ? xa[p][m] : 0u;
                wb |= m == mb ? xb[p][m] : 0u;
            }
            const int dd = __popc(at_most<L>(cA, wb, N)) + __popc(at_most<L>(cB, wa, N))
                         - __popc(at_most<L>(cA, wa, N)) - __popc(at_most<L>(cB, wb, N));
            d[p] += in ? dd : 0;
        }
    }
#pragma unroll
    for (int p = 0; p < PPWX; ++p) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) d[p] += __shfl_xor(d[p], off, 64);
        const int q = wave * PPWX + p;
        if (lane == 0 && q < nb) {
            sDelta[q] = live[p] ? d[p] : 0;
            sKa[q] = live[p] ? ka[p] : -1;       // changes nothing: never in anyone's way
            sKb[q] = live[p] ? kb[p] : -1;
            sPa[q] = a[p];
            sPb[q] = b[p];
        }
    }
}

// PPW proposals per wavefront and round, all their loads in flight together: 8 for M = 4, 4 for
// M = 8, 2 for M = 16 keeps the kernel within the 256 registers a 512-thread workgroup leaves per lane.
template <int M> struct RefineShape {
    static constexpr int PPW = M == 4 ? 8 : (M == 8 ? 4 : 2);
    static constexpr int ROUND = kRefineWaves * PPW;     // proposals per round, at most 64
};

template <int M>
__device__ __forceinline__ void
perm_refine_body(const uint32_t* __restrict__ Bm, int I, int words, int N, const int32_t* perm_in,
                 const int32_t* __restrict__ swaps, int64_t S, int32_t* perm_out, int32_t* __restrict__ result) {
    constexpr int PPW = RefineShape<M>::PPW, ROUND = RefineShape<M>::ROUND;
    extern __shared__ int32_t sP[];                      // the permutation, I entries
    __shared__ int32_t sSw[2 * kRefineChunk];
    __shared__ int sDelta[ROUND], sKa[ROUND], sKb[ROUND], sPa[ROUND], sPb[ROUND];
    __shared__ int32_t sPend[2 * ROUND];
    __shared__ uint2 sC[kRefineWaves][64];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;

    for (int r = tid; r < I; r += kRefineThreads) sP[r] = perm_in ? perm_in[r] : r;

    int gain = 0, kept = 0, npend = 0;                   // npend: proposals deferred by the round before
    int64_t base = 0, chunk0 = 0, chunk1 = 0;            // staged proposals: [chunk0, chunk1)
    while (base < S || npend > 0) {                      // uniform over the workgroup
        if (base + ROUND > chunk1 && chunk1 < S) {
            __syncthreads();                             // everyone is done with the old chunk
            chunk0 = base;
            chunk1 = base + kRefineChunk < S ? base + kRefineChunk : S;
            for (int64_t e = tid; e < 2 * (chunk1 - chunk0); e += kRefineThreads) sSw[e] = swaps[2 * chunk0 + e];
        }
        __syncthreads();                                 // permutation, deferred and staged proposals are in place
        const int room = ROUND - npend;
        const int nfresh = S - base < room ? static_cast<int>(S - base) : room;
        const int nb = npend + nfresh;                   // >= 1
        const int first = static_cast<int>(base - chunk0);
        if (wave * PPW < nb)
            refine_evaluate<M, PPW>(Bm, I, words, N, sP, sPend, npend, sSw, first, nb, wave, lane, sDelta, sKa, sKb,
                                    sPa, sPb);
        __syncthreads();
        // Every wavefront decides the round the same way, in registers.  Lane i: which earlier proposals of
        // the round share a block with proposal i.
        const int dL = lane < nb ? sDelta[lane] : 0;
        const int kaL = lane < nb ? sKa[lane] : -1;
        const int kbL = lane < nb ? sKb[lane] : -1;
        uint64_t keep = 0u, pend = 0u;
        if (__ballot(dL > 0) != 0ull) {                  // else nothing can be kept, so nothing is deferred either
            // the comparisons are split over the wavefronts (columns j of wavefront w: w * JW ..) and OR-ed via LDS
            constexpr int JW = ROUND / kRefineWaves;
            uint32_t clo = 0u, chi = 0u;
#pragma unroll
            for (int jj = 0; jj < JW; ++jj) {
                const int j = wave * JW + jj;            // wave-uniform
                if (j < nb) {
                    const int ja = __builtin_amdgcn_readlane(kaL, j), jb = __builtin_amdgcn_readlane(kbL, j);
                    const bool hit = j < lane && kaL >= 0 && ja >= 0 && (kaL == ja || kaL == jb || kbL == ja || kbL == jb);
                    if (j < 32) clo |= hit ? 1u << j : 0u;
                    else chi |= hit ? 1u << (j - 32) : 0u;
                }
            }
            sC[wave][lane] = make_uint2(clo, chi);
            __syncthreads();
            clo = chi = 0u;
#pragma unroll
            for (int w = 0; w < kRefineWaves; ++w) {
                const uint2 c = sC[w][lane];
                clo |= c.x;
                chi |= c.y;
            }
            // In order: a proposal that shares a block with an earlier one that was kept (its evaluation is
            // stale) or deferred (it must not overtake it) is deferred; any other is decided now.
            for (int i = 0; i < nb; ++i) {
                const uint64_t ci = (static_cast<uint64_t>(__builtin_amdgcn_readlane(chi, i)) << 32) |
                                    static_cast<uint32_t>(__builtin_amdgcn_readlane(clo, i));
                if (ci & (keep | pend)) {
                    pend |= 1ull << i;
                } else {
                    const int d = __builtin_amdgcn_readlane(dL, i);
                    if (d > 0) {
                        keep |= 1ull << i;
                        gain += d;
                        ++kept;
                    }
                }
            }
        }
        if (wave == 0 && lane < nb) {
            const int a = sPa[lane], b = sPb[lane];
            if ((keep >> lane) & 1ull) {                 // kept proposals touch disjoint blocks: disjoint positions
                const int32_t t = sP[a];
                sP[a] = sP[b];
                sP[b] = t;
            }
            if ((pend >> lane) & 1ull) {                 // deferred proposals open the next round, in order
                const int slot = __builtin_popcountll(pend & ((1ull << lane) - 1ull));
                sPend[2 * slot] = a;
                sPend[2 * slot + 1] = b;
            }
        }
        base += nfresh;
        npend = __builtin_popcountll(pend);              // < nb: the round's first proposal is always decided
    }
    __syncthreads();
    for (int r = tid; r < I; r += kRefineThreads) perm_out[r] = sP[r];
    if (tid == 0) {
        result[0] = gain;
        result[1] = kept;
    }
}

template <int M>
__global__ void __launch_bounds__(kRefineThreads)
k_perm_refine(const uint32_t* __restrict__ Bm, int I, int words, int N, const int32_t* perm_in,
              const int32_t* __restrict__ swaps, int64_t S, int32_t* perm_out, int32_t* __restrict__ result) {
    perm_refine_body<M>(Bm, I, words, N, perm_in, swaps, S, perm_out, result);
}

// Many layers at once: workgroup b refines layer b (in place), the argument table travels in the kernel arguments.
struct RefineEntry {
    const uint32_t* B;
    int32_t* perm;
    const int32_t* swaps;
    int32_t* result;
    int64_t S;
    int I, words;
};
constexpr int kRefineGroupCap = 64;
struct RefineGroup { RefineEntry e[kRefineGroupCap]; };
static_assert(sizeof(RefineGroup) <= 3840, "argument table must fit the kernel arguments");

template <int M>
__global__ void __launch_bounds__(kRefineThreads)
k_perm_refine_group(const RefineGroup g, int N) {
    const RefineEntry& e = g.e[blockIdx.x];
    perm_refine_body<M>(e.B, e.I, e.words, N, e.perm, e.swaps, e.S, e.perm, e.result);
}

template <int M>
int set_refine_lds(const void* kern, size_t lds, DeviceMemo& done) {
    const int dev = DeviceMemo::device();
    if (lds > 48 * 1024 && !done.get(dev)) {
        if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return BIMASK_ERR_HIP;
        }
        done.set(dev, 1);
    }
    return BIMASK_OK;
}

template <int M>
int run_refine_group(const bimask_group_layer* L, int n, int N, hipStream_t s) {
    static DeviceMemo attr_set;
    for (int first = 0; first < n; first += kRefineGroupCap) {
        const int cnt = n - first < kRefineGroupCap ? n - first : kRefineGroupCap;
        RefineGroup g;
        size_t lds = 0;
        for (int l = 0; l < cnt; ++l) {
            const bimask_group_layer& a = L[first + l];
            g.e[l] = RefineEntry{a.B_bits, a.best_perm, a.swaps, a.refine_result, a.n_swaps, static_cast<int>(a.I),
                                 static_cast<int>(ceil_div(a.J, 32))};
            lds = lds > static_cast<size_t>(a.I) * 4 ? lds : static_cast<size_t>(a.I) * 4;
        }
        if (int rc = set_refine_lds<M>(reinterpret_cast<const void*>(k_perm_refine_group<M>), lds, attr_set)) return rc;
        hipLaunchKernelGGL(k_perm_refine_group<M>, dim3(cnt), dim3(kRefineThreads), lds, s, g, N);
        if (int rc = check_launch()) return rc;
    }
    return BIMASK_OK;
}

template <int M>
int run_refine(const uint32_t* B_bits, int64_t I, int64_t J, int N, const int32_t* perm_in, const int32_t* swaps,
               int64_t S, int32_t* perm_out, int32_t* result, hipStream_t s) {
    static DeviceMemo attr_set;
    const size_t lds = static_cast<size_t>(I) * 4;
    if (int rc = set_refine_lds<M>(reinterpret_cast<const void*>(k_perm_refine<M>), lds, attr_set)) return rc;
    hipLaunchKernelGGL(k_perm_refine<M>, dim3(1), dim3(kRefineThreads), lds, s, B_bits, static_cast<int>(I),
                       static_cast<int>(ceil_div(J, 32)), N, perm_in, swaps, S, perm_out, result);
    return check_launch();
}

}  // namespace

int launch_perm_refine(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perm_in,
                       const int32_t* swaps, int64_t S, int32_t* perm_out, int32_t* result, hipStream_t s) {
    if (I > kRefineMaxRows || I * ceil_div(J, 32) > 0x7FFFFFFFll) return BIMASK_ERR_UNSUPPORTED;
    switch (M) {
        case 4: return run_refine<4>(B_bits, I, J, N, perm_in, swaps, S, perm_out, result, s);
        case 8: return run_refine<8>(B_bits, I, J, N, perm_in, swaps, S, perm_out, result, s);
        case 16: return run_refine<16>(B_bits, I, J, N, perm_in, swaps, S, perm_out, result, s);
        default: return BIMASK_ERR_NM;
    }
}

int launch_perm_refine_group(const bimask_group_layer* L, int n, int N, int M, hipStream_t s) {
    for (int l = 0; l < n; ++l)
        if (L[l].I > kRefineMaxRows || L[l].I * ceil_div(L[l].J, 32) > 0x7FFFFFFFll) return BIMASK_ERR_UNSUPPORTED;
    switch (M) {
        case 4: return run_refine_group<4>(L, n, N, s);
        case 8: return run_refine_group<8>(L, n, N, s);
        case 16: return run_refine_group<16>(L, n, N, s);
        default: return BIMASK_ERR_NM;
    }
}

}  // namespace bimask
