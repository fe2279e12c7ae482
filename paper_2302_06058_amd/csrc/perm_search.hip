// Row-permutation search (Sec. 3.3 / Alg. 1 of arXiv 2302.06058): score K candidate
// permutations by their number of eligible N:M column blocks and take the first best.
//
// The forward mask is cut into column slices of 1024 columns (128 bytes per row, one cache
// line; 4096 columns when rows do not start on line boundaries).  A wavefront scores one
// candidate on one slice over a range of row blocks: lane (b, q) = (l / CHL, l % CHL) handles
// row block b of the current step and 16 bytes of the slice, so one load instruction fetches
// whole contiguous row segments through the gather P, and the M rows of a block are added
// bit-sliced (one counter per column, 128 columns per lane at once), compared with N and the
// eligible columns pop-counted.  Workgroups are numbered so that each XCD works on one slice
// at a time: the slice then stays in that XCD's L2 for all K candidates and the mask is read
// from HBM about once.  Partial scores per (slice, row range, candidate) go to scratch; a
// second one-workgroup kernel sums them, takes the arg-max and copies the winning
// permutation.  Integer only, no atomics: the result is bit-reproducible.
#include <atomic>

#include "common.hpp"

namespace bimask {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int M> struct Planes { static constexpr int L = M == 4 ? 3 : (M == 8 ? 4 : 5); };

// VEC: rows of the mask start on 16-byte boundaries (whole 16-byte chunks exist or not).
// CHL: 16-byte chunks per row and slice (8 or 32).  U: row-block groups per step, all in
// flight at once.  N2OF4: the 2:4 case, where "more than two of four" is a 7-operation
// boolean formula instead of a bit-sliced adder.
template <int M, bool VEC, int CHL, int U, bool N2OF4>
__device__ __forceinline__ void
perm_score_body(const uint32_t* __restrict__ B_bits, int I, int64_t J, int wpr32,
                const int32_t* __restrict__ perms, int K, int N, int nseg, int sps, int64_t items,
                int32_t* __restrict__ partial, unsigned block, unsigned grid) {
    constexpr int L = Planes<M>::L;
    constexpr int BPS = 64 / CHL;                        // row blocks per load instruction
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // workgroup ids go round-robin over the 8 XCDs: XCD x takes a contiguous range of items
    const int64_t per_xcd = grid / 8;
    const int64_t item = ((block % 8) * per_xcd + block / 8) * (kThreads / 64) + wave;
    if (item >= items) return;
    const int seg = static_cast<int>(item % nseg);
    const int64_t sc = item / nseg;
    const int c = static_cast<int>(sc % K), slice = static_cast<int>(sc / K);
    const int bl = lane / CHL, ch = lane % CHL;
    const int word0 = (slice * CHL + ch) * 4;

    // columns at or beyond J never count; words beyond the row are not read (clamped address)
    uint32_t valid[4];
    int woff[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int64_t nv = J - static_cast<int64_t>(word0 + w) * 32;
        valid[w] = nv >= 32 ? 0xFFFFFFFFu : (nv <= 0 ? 0u : (1u << static_cast<int>(nv)) - 1u);
        woff[w] = word0 + w < wpr32 ? word0 + w : wpr32 - 1;
    }
    const uint32_t* Bs = B_bits + (VEC ? (word0 < wpr32 ? word0 : 0) : 0);

    const int nblk = I / M, steps = (nblk + BPS * U - 1) / (BPS * U);
    const int s_begin = seg * sps;
    const int s_end = s_begin + sps < steps ? s_begin + sps : steps;
    const int32_t* P = perms + static_cast<int64_t>(c) * I;

    int4 pe[U][M / 4];                                   // permutation entries of the next step
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int b = (s_begin * U + u) * BPS + bl;
        b = b < nblk ? b : nblk - 1;                     // clamped: loaded, counted as nothing
#pragma unroll
        for (int v = 0; v < M / 4; ++v) pe[u][v] = *reinterpret_cast<const int4*>(P + static_cast<int64_t>(b) * M + 4 * v);
    }
    int acc = 0;
    for (int s = s_begin; s < s_end; ++s) {
        u32x4 x[U][M];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int r = (m & 3) == 0 ? pe[u][m >> 2].x : ((m & 3) == 1 ? pe[u][m >> 2].y
                            : ((m & 3) == 2 ? pe[u][m >> 2].z : pe[u][m >> 2].w));
                const uint32_t* row = Bs + static_cast<int64_t>(r) * wpr32;
                if constexpr (VEC) {
                    x[u][m] = *reinterpret_cast<const u32x4*>(row);
                } else {
                    x[u][m].x = row[woff[0]]; x[u][m].y = row[woff[1]]; x[u][m].z = row[woff[2]]; x[u][m].w = row[woff[3]];
                }
            }
        const int sn = s + 1 < s_end ? s + 1 : s;        // the last step reloads its own entries
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int b = (sn * U + u) * BPS + bl;
            b = b < nblk ? b : nblk - 1;
#pragma unroll
            for (int v = 0; v < M / 4; ++v) pe[u][v] = *reinterpret_cast<const int4*>(P + static_cast<int64_t>(b) * M + 4 * v);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int cnt = 0;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t gt;                             // columns whose block holds more than N ones
                if constexpr (N2OF4) {
                    const uint32_t a = x[u][0][w], b = x[u][1][w], cc = x[u][2][w], d = x[u][3][w];
                    gt = (a & b & (cc | d)) | (cc & d & (a | b));
                } else {
                    uint32_t sp[L];
#pragma unroll
                    for (int p = 0; p < L; ++p) sp[p] = 0;
#pragma unroll
                    for (int m = 0; m < M; ++m) {        // bit-sliced add of one bit-row
                        uint32_t carry = x[u][m][w];
#pragma unroll
                        for (int p = 0; p < L; ++p) {
                            const uint32_t t = sp[p] & carry;
                            sp[p] ^= carry;
                            carry = t;
                        }
                    }
                    uint32_t eq = 0xFFFFFFFFu;
                    gt = 0;
#pragma unroll
                    for (int p = L - 1; p >= 0; --p) {
                        if ((N >> p) & 1) { eq &= sp[p]; }
                        else { gt |= eq & sp[p]; eq &= ~sp[p]; }
                    }
                }
                cnt += __popc(~gt & valid[w]);
            }
            acc += (s * U + u) * BPS + bl < nblk ? cnt : 0;   // a clamped (repeated) block counts nothing
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) partial[(static_cast<int64_t>(slice) * nseg + seg) * K + c] = acc;
}

template <int M, bool VEC, int CHL, int U, bool N2OF4>
__global__ void __launch_bounds__(kThreads)
k_perm_score(const uint32_t* __restrict__ B_bits, int I, int64_t J, int wpr32,
             const int32_t* __restrict__ perms, int K, int N, int nseg, int sps, int64_t items,
             int32_t* __restrict__ partial) {
    perm_score_body<M, VEC, CHL, U, N2OF4>(B_bits, I, J, wpr32, perms, K, N, nseg, sps, items, partial, blockIdx.x, gridDim.x);
}

// Grouped launch: the searches of several independent layers in one grid (first[l] = first
// workgroup of layer l, a multiple of 8 so that the XCD assignment of a layer's items holds).
struct ScoreGroupP {
    const uint32_t* B_bits;
    const int32_t* perms;
    int32_t* partial;
    int64_t J, items;
    int I, wpr32, nseg, sps;
};
constexpr int kSearchGroupCap = group_capacity(sizeof(ScoreGroupP));     // 56-byte entries: 63 layers
struct ScoreGroup {
    int n;
    unsigned first[kSearchGroupCap + 1];
    ScoreGroupP p[kSearchGroupCap];
};
template <int M, bool VEC, int CHL, int U, bool N2OF4>
__global__ void __launch_bounds__(kThreads)
k_perm_score_group(const ScoreGroup g, int K, int N) {
    int l = 0;
    while (l + 1 < g.n && blockIdx.x >= g.first[l + 1]) ++l;
    const ScoreGroupP& p = g.p[l];
    perm_score_body<M, VEC, CHL, U, N2OF4>(p.B_bits, p.I, p.J, p.wpr32, p.perms, K, N, p.nseg, p.sps, p.items, p.partial,
                                           blockIdx.x - g.first[l], g.first[l + 1] - g.first[l]);
}

// Sums the per-tile partial scores, takes the first arg-max and copies the winner.
// One workgroup of 1024 threads: 128 candidates x 8 tile groups at a time, so every
// thread issues its few independent loads at once instead of walking all tiles serially.
constexpr int kFinalThreads = 1024;
__device__ __forceinline__ void
perm_final_body(const int32_t* __restrict__ partial, int ntiles, int K, int64_t I,
                const int32_t* __restrict__ perms, int32_t* __restrict__ scores,
                int32_t* __restrict__ best, int32_t* __restrict__ best_perm) {
    __shared__ int psum[8][128];
    __shared__ long long red[128];
    const int cl = threadIdx.x & 127, part = threadIdx.x >> 7;
    long long mine = -1;
    for (int c0 = 0; c0 < K; c0 += 128) {
        const int c = c0 + cl;
        int s = 0;
        if (c < K) {
            // four independent loads per round: the partial sums are L2 latency, not bandwidth
            int t = part;
            for (; t + 24 < ntiles; t += 32) {
                const int a0 = partial[static_cast<int64_t>(t) * K + c], a1 = partial[static_cast<int64_t>(t + 8) * K + c];
                const int a2 = partial[static_cast<int64_t>(t + 16) * K + c], a3 = partial[static_cast<int64_t>(t + 24) * K + c];
                s += (a0 + a1) + (a2 + a3);
            }
            for (; t < ntiles; t += 8) s += partial[static_cast<int64_t>(t) * K + c];
        }
        psum[part][cl] = s;
        __syncthreads();
        if (part == 0 && c < K) {
            int tot = 0;
#pragma unroll
            for (int p = 0; p < 8; ++p) tot += psum[p][cl];
            scores[c] = tot;
            // larger score first, then the smaller candidate index
            const long long key = (static_cast<long long>(tot) << 32) | static_cast<uint32_t>(0x7FFFFFFF - c);
            mine = key > mine ? key : mine;
        }
        __syncthreads();
    }
    if (part == 0) red[cl] = mine;
    __syncthreads();
    for (int off = 64; off > 0; off >>= 1) {
        if (static_cast<int>(threadIdx.x) < off) {
            const long long o = red[threadIdx.x + off];
            if (o > red[threadIdx.x]) red[threadIdx.x] = o;
        }
        __syncthreads();
    }
    const int bc = 0x7FFFFFFF - static_cast<int>(red[0] & 0xFFFFFFFFll);
    if (threadIdx.x == 0) *best = bc;
    if (best_perm) {
        const int32_t* P = perms + static_cast<int64_t>(bc) * I;
        for (int64_t i = threadIdx.x; i < I; i += kFinalThreads) best_perm[i] = P[i];
    }
}

__global__ void __launch_bounds__(kFinalThreads)
k_perm_final(const int32_t* __restrict__ partial, int ntiles, int K, int64_t I,
             const int32_t* __restrict__ perms, int32_t* __restrict__ scores,
             int32_t* __restrict__ best, int32_t* __restrict__ best_perm) {
    perm_final_body(partial, ntiles, K, I, perms, scores, best, best_perm);
}

struct FinalGroupP {
    const int32_t* partial;
    const int32_t* perms;
    int32_t* scores;
    int32_t* best;
    int32_t* best_perm;
    int64_t I;
    int ntiles;
};
struct FinalGroup {
    FinalGroupP p[kSearchGroupCap];
};
// one workgroup per layer
__global__ void __launch_bounds__(kFinalThreads)
k_perm_final_group(const FinalGroup g, int K) {
    const FinalGroupP& p = g.p[blockIdx.x];
    perm_final_body(p.partial, p.ntiles, K, p.I, p.perms, p.scores, p.best, p.best_perm);
}

template <int M>
int run_score(const uint32_t* B_bits, int64_t I, int64_t J, int N, const int32_t* perms, int K,
              const PermPlan& pl, int32_t* partial, hipStream_t s) {
    constexpr int U = M == 16 ? 1 : 2;
    const int wpr32 = static_cast<int>(ceil_div(J, 32));
    const int64_t items = static_cast<int64_t>(pl.ntiles) * K;
    const unsigned grid = static_cast<unsigned>(round_up(ceil_div(items, kThreads / 64), 8));
    const bool vec = aligned16(B_bits) && wpr32 % 4 == 0;
#define BIMASK_SCORE(VEC, CHL)                                                                               \
    {                                                                                                        \
        if (M == 4 && N == 2)                                                                                \
            hipLaunchKernelGGL((k_perm_score<M, VEC, CHL, U, M == 4>), dim3(grid), dim3(kThreads), 0, s, B_bits, \
                               static_cast<int>(I), J, wpr32, perms, K, N, pl.nseg, pl.sps, items, partial); \
        else                                                                                                 \
            hipLaunchKernelGGL((k_perm_score<M, VEC, CHL, U, false>), dim3(grid), dim3(kThreads), 0, s, B_bits, \
                               static_cast<int>(I), J, wpr32, perms, K, N, pl.nseg, pl.sps, items, partial); \
    }
    if (pl.chunks == 32) { if (vec) BIMASK_SCORE(true, 32) else BIMASK_SCORE(false, 32) }
    else                 { if (vec) BIMASK_SCORE(true, 8)  else BIMASK_SCORE(false, 8) }
#undef BIMASK_SCORE
    return check_launch();
}

}  // namespace

PermPlan plan_perm_search(int64_t I, int64_t J, int K, int M) {
    PermPlan pl{};
    const int64_t pitch = ceil_div(J, 32) * 4;                   // bytes per mask row
    pl.chunks = (pitch % 128 != 0 && J >= 4096) ? 32 : 8;
    pl.nslices = static_cast<int>(ceil_div(J, pl.chunks * 128));
    const int U = M == 16 ? 1 : 2;
    const int64_t steps = ceil_div(I / M, (64 / pl.chunks) * U); // row blocks per wavefront step
    // about 32 wavefronts per CU, at least 2 steps each
    int64_t nseg = ceil_div(8192, static_cast<int64_t>(pl.nslices) * K);
    const int64_t nseg_max = steps / 2 > 1 ? steps / 2 : 1;
    nseg = nseg < 1 ? 1 : (nseg > nseg_max ? nseg_max : nseg);
    pl.sps = static_cast<int>(ceil_div(steps, nseg));
    pl.nseg = static_cast<int>(ceil_div(steps, pl.sps));
    pl.ntiles = pl.nslices * pl.nseg;
    pl.ws_bytes = static_cast<size_t>(pl.ntiles) * K * sizeof(int32_t);
    return pl;
}

namespace {

// score kernels of the layers that share one instantiation (row alignment, slice width)
template <int M>
int run_score_group(const bimask_group_layer* L, const int* which, int cnt, int N, int K, bool vec, int chunks,
                    hipStream_t s) {
    constexpr int U = M == 16 ? 1 : 2;
    ScoreGroup g{};
    g.n = cnt;
    unsigned blocks = 0;
    for (int l = 0; l < cnt; ++l) {
        const bimask_group_layer& a = L[which[l]];
        const PermPlan pl = plan_perm_search(a.I, a.J, K, M);
        ScoreGroupP& p = g.p[l];
        p.B_bits = a.B_bits; p.perms = a.perms; p.partial = static_cast<int32_t*>(a.workspace);
        p.J = a.J; p.I = static_cast<int>(a.I);
        p.wpr32 = static_cast<int>(ceil_div(a.J, 32));
        p.nseg = pl.nseg; p.sps = pl.sps;
        p.items = static_cast<int64_t>(pl.ntiles) * K;
        g.first[l] = blocks;
        blocks += static_cast<unsigned>(round_up(ceil_div(p.items, kThreads / 64), 8));
    }
    g.first[cnt] = blocks;
#define BIMASK_SCOREG(VEC, CHL)                                                                              \
    {                                                                                                        \
        if (M == 4 && N == 2)                                                                                \
            hipLaunchKernelGGL((k_perm_score_group<M, VEC, CHL, U, M == 4>), dim3(blocks), dim3(kThreads), 0, s, g, K, N); \
        else                                                                                                 \
            hipLaunchKernelGGL((k_perm_score_group<M, VEC, CHL, U, false>), dim3(blocks), dim3(kThreads), 0, s, g, K, N);  \
    }
    if (chunks == 32) { if (vec) BIMASK_SCOREG(true, 32) else BIMASK_SCOREG(false, 32) }
    else              { if (vec) BIMASK_SCOREG(true, 8)  else BIMASK_SCOREG(false, 8) }
#undef BIMASK_SCOREG
    return check_launch();
}

}  // namespace

// The searches of n independent layers (same N:M and number of candidates) in a few launches:
// one scoring launch per kernel instantiation in use, one finalising launch with a workgroup
// per layer.  Same results as n calls of launch_perm_search.
int launch_perm_search_group(const bimask_group_layer* L, int n, int N, int M, int K, hipStream_t s) {
    static_assert(sizeof(FinalGroup) <= 3840 && sizeof(ScoreGroup) <= 3840, "argument tables must fit the kernel arguments");
    for (int b = 0; b < n; b += kSearchGroupCap) {
        const int m = n - b < kSearchGroupCap ? n - b : kSearchGroupCap;
        for (int cls = 0; cls < 4; ++cls) {              // (rows 16-byte aligned?, 8 or 32 chunks per slice)
            const bool vec = cls & 1;
            const int chunks = (cls & 2) ? 32 : 8;
            int which[kSearchGroupCap], cnt = 0;
            for (int l = 0; l < m; ++l) {
                const bimask_group_layer& a = L[b + l];
                const bool v = aligned16(a.B_bits) && ceil_div(a.J, 32) % 4 == 0;
                if (v == vec && plan_perm_search(a.I, a.J, K, M).chunks == chunks) which[cnt++] = b + l;
            }
            if (cnt == 0) continue;
            int rc = BIMASK_ERR_NM;
            if (M == 4) rc = run_score_group<4>(L, which, cnt, N, K, vec, chunks, s);
            else if (M == 8) rc = run_score_group<8>(L, which, cnt, N, K, vec, chunks, s);
            else if (M == 16) rc = run_score_group<16>(L, which, cnt, N, K, vec, chunks, s);
            if (rc != BIMASK_OK) return rc;
        }
        FinalGroup f{};
        for (int l = 0; l < m; ++l) {
            const bimask_group_layer& a = L[b + l];
            FinalGroupP& p = f.p[l];
            p.partial = static_cast<const int32_t*>(a.workspace); p.perms = a.perms; p.scores = a.scores; p.best = a.best;
            p.best_perm = a.best_perm; p.I = a.I;
            p.ntiles = plan_perm_search(a.I, a.J, K, M).ntiles;
        }
        hipLaunchKernelGGL(k_perm_final_group, dim3(static_cast<unsigned>(m)), dim3(kFinalThreads), 0, s, f, K);
        if (int rc = check_launch()) return rc;
    }
    return BIMASK_OK;
}

int launch_perm_search(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                       int32_t* scores, int32_t* best, int32_t* best_perm, void* ws, hipStream_t s) {
    const PermPlan pl = plan_perm_search(I, J, K, M);
    int32_t* partial = static_cast<int32_t*>(ws);
    int rc = BIMASK_ERR_NM;
    if (M == 4) rc = run_score<4>(B_bits, I, J, N, perms, K, pl, partial, s);
    else if (M == 8) rc = run_score<8>(B_bits, I, J, N, perms, K, pl, partial, s);
    else if (M == 16) rc = run_score<16>(B_bits, I, J, N, perms, K, pl, partial, s);
    if (rc != BIMASK_OK) return rc;
    hipLaunchKernelGGL(k_perm_final, dim3(1), dim3(kFinalThreads), 0, s, partial, pl.ntiles, K, I, perms, scores, best,
                       best_perm);
    return check_launch();
}

// ---- the search for callers that cannot allocate: partial scores in a static device array --------
// One copy of the array exists per GPU the library runs on, for the life of the process.  In host
// code the array's name is only a handle for hipGetSymbolAddress: the address the kernels get is
// looked up once per device, with that device current, and remembered.
constexpr size_t kStaticScratchBytes = BIMASK_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t perm_search_static_capacity() { return kStaticScratchBytes; }

int launch_perm_search_static(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                              int32_t* scores, int32_t* best, int32_t* best_perm, hipStream_t s) {
    static std::atomic<void*> device_ptr[kMaxDevices];       // zero-initialised: not looked up yet
    if (plan_perm_search(I, J, K, M).ws_bytes > kStaticScratchBytes) return BIMASK_ERR_WORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BIMASK_ERR_HIP;
    void* ptr = device_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return BIMASK_ERR_HIP;
        }
        device_ptr[dev].store(ptr, std::memory_order_release);
    }
    // every partial score the second kernel reads is written by the first: nothing to clear
    return launch_perm_search(B_bits, I, J, N, M, perms, K, scores, best, best_perm, ptr, s);
}

namespace {

// Debug helper: is every candidate a permutation of 0 .. I-1?  One workgroup per candidate marks the
// values it meets in an LDS bitmap; a value out of range or met twice clears the candidate's flag.
__global__ void __launch_bounds__(kThreads)
k_check_perms(const int32_t* __restrict__ perms, int64_t I, int32_t* __restrict__ ok) {
    extern __shared__ uint32_t seen[];
    const int words = static_cast<int>((I + 31) >> 5);
    for (int w = threadIdx.x; w < words; w += kThreads) seen[w] = 0u;
    __syncthreads();
    const int32_t* P = perms + static_cast<int64_t>(blockIdx.x) * I;
    int bad = 0;
    for (int64_t r = threadIdx.x; r < I; r += kThreads) {
        const int32_t v = P[r];
        if (v < 0 || v >= I) {
            bad = 1;
        } else {
            const uint32_t bit = 1u << (v & 31);
            if (atomicOr(&seen[v >> 5], bit) & bit) bad = 1;
        }
    }
    bad = __syncthreads_or(bad);
    if (threadIdx.x == 0) ok[blockIdx.x] = bad ? 0 : 1;
}

}  // namespace

int launch_check_perms(const int32_t* perms, int K, int64_t I, int32_t* ok, hipStream_t s) {
    static DeviceMemo attr_set;
    if (I > kCheckPermsMaxRows) return BIMASK_ERR_UNSUPPORTED;
    const size_t lds = static_cast<size_t>((I + 31) >> 5) * 4;
    const int dev = DeviceMemo::device();
    if (lds > 48 * 1024 && !attr_set.get(dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_check_perms), hipFuncAttributeMaxDynamicSharedMemorySize,
                                128 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return BIMASK_ERR_HIP;
        }
        attr_set.set(dev, 1);
    }
    hipLaunchKernelGGL(k_check_perms, dim3(static_cast<unsigned>(K)), dim3(kThreads), lds, s, perms, I, ok);
    return check_launch();
}

}  // namespace bimask
