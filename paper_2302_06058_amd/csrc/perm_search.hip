// Row-permutation search (Sec. 3.3 / Alg. 1 of arXiv 2302.06058): score K candidate
// permutations by their number of eligible N:M column blocks and take the first best.
//
// A workgroup keeps a column tile of the forward mask -- all I rows x (ctw words) -- in
// LDS and scores a subset of the candidates on it: per block of M permuted rows the M
// bit-rows are gathered from LDS, added bit-sliced (one counter per column, all columns
// of a word at once), compared with N, and the eligible columns are pop-counted.
// Partial scores per (tile, candidate) go to scratch; a second one-workgroup kernel sums
// them, takes the arg-max and copies the winning permutation.  Integer only, no atomics:
// the result is bit-reproducible.
#include "common.hpp"

namespace bimask {
namespace {

constexpr size_t kLdsCap = 144 * 1024;     // of the 160 KB a workgroup may use
constexpr int kWantGroups = 512;           // enough workgroups for 256 CUs

template <int M> struct Planes { static constexpr int L = M == 4 ? 3 : (M == 8 ? 4 : 5); };

template <typename WordT, int M>
__global__ void __launch_bounds__(kThreads)
k_perm_score(const uint32_t* __restrict__ B_bits, int64_t I, int64_t J, int wpr32,
             const int32_t* __restrict__ perms, int K, int N, int kc, int ctw,
             int32_t* __restrict__ partial) {
    extern __shared__ uint4 smem_u4[];
    WordT* tile = reinterpret_cast<WordT*>(smem_u4);
    constexpr int WB = sizeof(WordT) * 8;
    constexpr int L = Planes<M>::L;
    const int tile_id = blockIdx.x / kc, chunk = blockIdx.x % kc;

    for (int64_t idx = threadIdx.x; idx < I * ctw; idx += kThreads) {
        const int64_t r = idx / ctw;
        const int w = static_cast<int>(idx - r * ctw);
        const int64_t gw = static_cast<int64_t>(tile_id) * ctw + w;
        WordT v = 0;
        if constexpr (sizeof(WordT) == 8) {
            const int64_t w32 = 2 * gw;
            const uint64_t lo = w32 < wpr32 ? B_bits[r * wpr32 + w32] : 0u;
            const uint64_t hi = w32 + 1 < wpr32 ? B_bits[r * wpr32 + w32 + 1] : 0u;
            v = lo | (hi << 32);
        } else {
            v = gw < wpr32 ? B_bits[r * wpr32 + gw] : 0u;
        }
        tile[idx] = v;
    }
    __syncthreads();

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t nblk = I / M;
    for (int c = chunk + kc * wave; c < K; c += kc * (kThreads / 64)) {
        const int32_t* P = perms + static_cast<int64_t>(c) * I;
        int acc = 0;
        for (int64_t kb = lane; kb < nblk; kb += 64) {
            int rows[M];
#pragma unroll
            for (int v = 0; v < M / 4; ++v) {
                const int4 q = *reinterpret_cast<const int4*>(P + kb * M + 4 * v);
                rows[4 * v] = q.x; rows[4 * v + 1] = q.y; rows[4 * v + 2] = q.z; rows[4 * v + 3] = q.w;
            }
            for (int w = 0; w < ctw; ++w) {
                WordT s[L];
#pragma unroll
                for (int p = 0; p < L; ++p) s[p] = 0;
#pragma unroll
                for (int m = 0; m < M; ++m) {                    // bit-sliced add of one bit-row
                    WordT carry = tile[static_cast<int64_t>(rows[m]) * ctw + w];
#pragma unroll
                    for (int p = 0; p < L; ++p) {
                        const WordT t = s[p] & carry;
                        s[p] ^= carry;
                        carry = t;
                    }
                }
                WordT gt = 0, eq = ~static_cast<WordT>(0);        // per-column count > N
#pragma unroll
                for (int p = L - 1; p >= 0; --p) {
                    if ((N >> p) & 1) { eq &= s[p]; }
                    else { gt |= eq & s[p]; eq &= ~s[p]; }
                }
                const int64_t col0 = (static_cast<int64_t>(tile_id) * ctw + w) * WB;
                const int64_t nvalid = J - col0;
                WordT valid = nvalid >= WB ? ~static_cast<WordT>(0)
                                           : (nvalid <= 0 ? 0 : ((static_cast<WordT>(1) << nvalid) - 1));
                const WordT ok = ~gt & valid;
                if constexpr (sizeof(WordT) == 8) acc += __popcll(ok);
                else acc += __popc(ok);
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
        if (lane == 0) partial[static_cast<int64_t>(tile_id) * K + c] = acc;
    }
}

// Sums the per-tile partial scores, takes the first arg-max and copies the winner.
// One workgroup of 1024 threads: 128 candidates x 8 tile groups at a time, so every
// thread issues its few independent loads at once instead of walking all tiles serially.
constexpr int kFinalThreads = 1024;
__global__ void __launch_bounds__(kFinalThreads)
k_perm_final(const int32_t* __restrict__ partial, int ntiles, int K, int64_t I,
             const int32_t* __restrict__ perms, int32_t* __restrict__ scores,
             int32_t* __restrict__ best, int32_t* __restrict__ best_perm) {
    __shared__ int psum[8][128];
    __shared__ long long red[128];
    const int cl = threadIdx.x & 127, part = threadIdx.x >> 7;
    long long mine = -1;
    for (int c0 = 0; c0 < K; c0 += 128) {
        const int c = c0 + cl;
        int s = 0;
        if (c < K)
            for (int t = part; t < ntiles; t += 8) s += partial[static_cast<int64_t>(t) * K + c];
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

template <typename WordT, int M>
int run_score(const uint32_t* B_bits, int64_t I, int64_t J, int N, const int32_t* perms, int K,
              const PermPlan& pl, int32_t* partial, hipStream_t s) {
    auto kern = k_perm_score<WordT, M>;
    if (pl.lds_bytes > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(pl.lds_bytes)) != hipSuccess) return BIMASK_ERR_HIP;
    }
    const int wpr32 = static_cast<int>(ceil_div(J, 32));
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(pl.ntiles * pl.kc)), dim3(kThreads), pl.lds_bytes, s,
                       B_bits, I, J, wpr32, perms, K, N, pl.kc, pl.ctw, partial);
    return check_launch();
}

}  // namespace

PermPlan plan_perm_search(int64_t I, int64_t J, int K) {
    PermPlan pl{};
    pl.ok = false;
    if (static_cast<size_t>(I) * 8 <= kLdsCap) pl.word_bytes = 8;
    else if (static_cast<size_t>(I) * 4 <= kLdsCap) pl.word_bytes = 4;
    else return pl;                                              // the mask column tile must fit in LDS
    const int64_t nw = ceil_div(J, pl.word_bytes * 8);           // column words per row
    pl.kc = K < 8 ? K : 8;                                       // candidate chunks; 8 = one per XCD
    const int64_t ctw_max = static_cast<int64_t>((64 * 1024) / (static_cast<size_t>(I) * pl.word_bytes));
    const int64_t tiles_wanted = ceil_div(kWantGroups, pl.kc);
    int64_t ctw = nw / tiles_wanted;
    if (ctw > ctw_max) ctw = ctw_max;
    if (ctw < 1) ctw = 1;
    pl.ctw = static_cast<int>(ctw);
    pl.ntiles = static_cast<int>(ceil_div(nw, ctw));
    pl.lds_bytes = static_cast<size_t>(I) * pl.ctw * pl.word_bytes;
    pl.ws_bytes = static_cast<size_t>(pl.ntiles) * K * sizeof(int32_t);
    pl.ok = true;
    return pl;
}

int launch_perm_search(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                       int32_t* scores, int32_t* best, int32_t* best_perm, void* ws, hipStream_t s) {
    const PermPlan pl = plan_perm_search(I, J, K);
    if (!pl.ok) return BIMASK_ERR_UNSUPPORTED;
    int32_t* partial = static_cast<int32_t*>(ws);
    int rc = BIMASK_ERR_NM;
#define BIMASK_SCORE(WT, MM) rc = run_score<WT, MM>(B_bits, I, J, N, perms, K, pl, partial, s)
    if (pl.word_bytes == 8) {
        if (M == 4) BIMASK_SCORE(uint64_t, 4);
        else if (M == 8) BIMASK_SCORE(uint64_t, 8);
        else if (M == 16) BIMASK_SCORE(uint64_t, 16);
    } else {
        if (M == 4) BIMASK_SCORE(uint32_t, 4);
        else if (M == 8) BIMASK_SCORE(uint32_t, 8);
        else if (M == 16) BIMASK_SCORE(uint32_t, 16);
    }
#undef BIMASK_SCORE
    if (rc != BIMASK_OK) return rc;
    hipLaunchKernelGGL(k_perm_final, dim3(1), dim3(kFinalThreads), 0, s, partial, pl.ntiles, K, I, perms, scores, best,
                       best_perm);
    return check_launch();
}

}  // namespace bimask
