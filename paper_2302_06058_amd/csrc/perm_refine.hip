// Refinement of a row permutation by proposed exchanges (arXiv 2302.06058 leaves permutations
// better than random ones to future work, Limitations; the objective is the eligible-block
// count of Sec. 3.3 / Alg. 1).  Proposal t exchanges the entries at two positions of P and is
// kept only if the count grows strictly; proposals are taken in order, each against the
// permutation the earlier ones left.
//
// An exchange between blocks A and B of M permuted rows changes the count of those two blocks
// only, so a proposal costs 2M mask rows, not the matrix.  One workgroup of 8 wavefronts owns
// the permutation (in LDS).  Each round, wavefront w evaluates up to 8 proposals (base + 8w ..)
// against the current permutation: lanes stride over the 32-column words of the 2M rows, add the M - 1
// unchanged rows of each block bit-sliced, add either exchanged row on top, compare with N and
// pop-count the four eligibility words; a wavefront reduction gives the change of the count.
// Then every wavefront walks the round's results in proposal order: a proposal that shares a block
// with one kept earlier in the same round was evaluated against a stale permutation, so the
// round ends there and the next one starts at it; otherwise it is kept if its change is
// positive.  Kept proposals of a round touch disjoint blocks, so their exchanges commute and the
// result equals taking the proposals one by one.  Every round consumes at least its first
// proposal, so the loop ends.  Integer only: the result is bit-reproducible.
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

// PPW proposals per wavefront and round, all their loads in flight together: 8 for M = 4, 4 for
// M = 8, 2 for M = 16 keeps the kernel within the 256 registers a 512-thread workgroup leaves per lane.
template <int M> struct RefineShape {
    static constexpr int PPW = M == 4 ? 8 : (M == 8 ? 4 : 2);
    static constexpr int ROUND = kRefineWaves * PPW;     // proposals per round, at most 64
};

template <int M>
__global__ void __launch_bounds__(kRefineThreads)
k_perm_refine(const uint32_t* __restrict__ Bm, int I, int words, int N, const int32_t* __restrict__ perm_in,
              const int32_t* __restrict__ swaps, int64_t S, int32_t* __restrict__ perm_out,
              int32_t* __restrict__ result) {
    constexpr int L = RefinePlanes<M>::L;
    constexpr int SH = M == 4 ? 2 : (M == 8 ? 3 : 4);
    constexpr int PPW = RefineShape<M>::PPW, ROUND = RefineShape<M>::ROUND;
    extern __shared__ int32_t sP[];                      // the permutation, I entries
    __shared__ int32_t sSw[2 * kRefineChunk];
    __shared__ int sDelta[ROUND], sKa[ROUND], sKb[ROUND], sPa[ROUND], sPb[ROUND];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    for (int r = tid; r < I; r += kRefineThreads) sP[r] = perm_in ? perm_in[r] : r;

    int gain = 0, kept = 0;
    int64_t base = 0, chunk0 = 0, chunk1 = 0;            // staged proposals: [chunk0, chunk1)
    while (base < S) {                                   // uniform over the workgroup
        if (base + ROUND > chunk1 && chunk1 < S) {
            __syncthreads();                             // everyone is done with the old chunk
            chunk0 = base;
            chunk1 = base + kRefineChunk < S ? base + kRefineChunk : S;
            for (int64_t e = tid; e < 2 * (chunk1 - chunk0); e += kRefineThreads) sSw[e] = swaps[2 * chunk0 + e];
        }
        __syncthreads();                                 // permutation and proposals are in place
        const int nb = S - base < ROUND ? static_cast<int>(S - base) : ROUND;
        if (wave * PPW < nb) {
            // proposals wave * PPW + p; one that changes nothing (outside [0, I), both positions in one
            // block, beyond the round) is evaluated on positions 0 and 0 and its result dropped
            int a[PPW], b[PPW], ka[PPW], kb[PPW], d[PPW];
            bool live[PPW];
            uint32_t ra[PPW][M], rb[PPW][M];
#pragma unroll
            for (int p = 0; p < PPW; ++p) {
                const int q = wave * PPW + p;
                const int e = q < nb ? static_cast<int>(base - chunk0) + q : static_cast<int>(base - chunk0);
                a[p] = sSw[2 * e];
                b[p] = sSw[2 * e + 1];
                const bool valid = q < nb && a[p] >= 0 && a[p] < I && b[p] >= 0 && b[p] < I;
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
                uint32_t xa[PPW][M], xb[PPW][M];
#pragma unroll
                for (int p = 0; p < PPW; ++p) {
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        xa[p][m] = Bm[ra[p][m] + w];
                        xb[p][m] = Bm[rb[p][m] + w];
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int p = 0; p < PPW; ++p) {
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
            for (int p = 0; p < PPW; ++p) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) d[p] += __shfl_xor(d[p], off, 64);
                const int q = wave * PPW + p;
                if (lane == 0 && q < nb) {
                    sDelta[q] = live[p] ? d[p] : 0;
                    sKa[q] = live[p] ? ka[p] : -1;       // changes nothing: never in anyone's way
                    sKb[q] = live[p] ? kb[p] : -1;
                    sPa[q] = a[p];
                    sPb[q] = b[p];
                }
            }
        }
        __syncthreads();
        // every wavefront takes the same walk over the round's results, in scalar registers
        const int dL = lane < nb ? sDelta[lane] : 0;
        const int kaL = lane < nb ? sKa[lane] : -1;
        const int kbL = lane < nb ? sKb[lane] : -1;
        int stop = nb;
        uint64_t keep = 0u;
        for (int i = 0; i < nb; ++i) {
            const int ka = __builtin_amdgcn_readlane(kaL, i), kb = __builtin_amdgcn_readlane(kbL, i);
            bool stale = false;
            if (ka >= 0)
                for (uint64_t k = keep; k; k &= k - 1) {
                    const int j = __builtin_ctzll(k);
                    const int ja = __builtin_amdgcn_readlane(kaL, j), jb = __builtin_amdgcn_readlane(kbL, j);
                    stale |= ka == ja || ka == jb || kb == ja || kb == jb;
                }
            if (stale) { stop = i; break; }
            const int d = __builtin_amdgcn_readlane(dL, i);
            if (d > 0) {
                keep |= 1ull << i;
                gain += d;
                ++kept;
            }
        }
        if (wave == 0 && lane < nb && ((keep >> lane) & 1ull)) {   // disjoint blocks: disjoint positions
            const int a = sPa[lane], b = sPb[lane];
            const int32_t t = sP[a];
            sP[a] = sP[b];
            sP[b] = t;
        }
        base += stop;                                    // stop >= 1: the first proposal is never stale
    }
    __syncthreads();
    for (int r = tid; r < I; r += kRefineThreads) perm_out[r] = sP[r];
    if (tid == 0) {
        result[0] = gain;
        result[1] = kept;
    }
}

template <int M>
int run_refine(const uint32_t* B_bits, int64_t I, int64_t J, int N, const int32_t* perm_in, const int32_t* swaps,
               int64_t S, int32_t* perm_out, int32_t* result, hipStream_t s) {
    static std::atomic<bool> attr_set{false};
    const size_t lds = static_cast<size_t>(I) * 4;
    if (lds > 48 * 1024 && !attr_set.load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_perm_refine<M>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return BIMASK_ERR_HIP;
        }
        attr_set.store(true, std::memory_order_relaxed);
    }
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

}  // namespace bimask
