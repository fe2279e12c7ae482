// N:M-sparse GEMMs of Bi-Mask (Eq. 3 and Eq. 10 of arXiv 2302.06058) on gfx950.
//
// Both directions are the same contraction   C[t][a] = sum_k Bm[t][k] * A[a][k]
//   forward : A = (B .* W)       (a = out feature i, k = in feature j),  Bm = X,      C = Y
//   backward: A = (Bbar.*W[P,:])^T (a = in feature j, k = permuted row r), Bm = dY[:,P], C = dX
// A is the weight operand: only the A side of a sparse matrix instruction may be 2:4
// compressed, so the weights sit on the A side and the product is formed transposed
// (rows of the accumulator tile are weight rows, columns are tokens).
//
// bf16, 2:4  : v_smfmac_f32_32x32x32_bf16 on the fragment-major compressed operand (gemm_sp24.hip)
// bf16, other: v_mfma_f32_32x32x16_bf16 on the dense masked weights (this file)
// fp32       : plain fp32 FMA kernel, small problems only (this file)
#include "common.hpp"

namespace bimask {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte register vector
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;                // dense k per pipeline stage
constexpr int kRowB = 144;            // LDS bytes per 64-k row (128 + 16 pad: conflict-free 16-byte reads)

// 8 consecutive bf16 of a row starting at element k (zero beyond kend).
__device__ __forceinline__ u32x4 load_granule(const uint16_t* row, int64_t k, int64_t kend, bool vec) {
    if (k + 8 <= kend) {
        if (vec) return *reinterpret_cast<const u32x4*>(row + k);
        const uint32_t* p = reinterpret_cast<const uint32_t*>(row + k);
        u32x4 r = {p[0], p[1], p[2], p[3]};
        return r;
    }
    u32x4 r = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (k + e < kend) r[e >> 1] |= static_cast<uint32_t>(row[k + e]) << (16 * (e & 1));
    return r;
}

template <int BM, int BN>
struct Smem {
    static constexpr int kA = BM * kRowB;
    static constexpr int kB = BN * kRowB;
    static constexpr int kStage = kA + kB;
    static constexpr int kCRow = BM * 2 + 16;
    static constexpr int kC = BN * kCRow;
    static constexpr int kTotal = (2 * kStage > kC) ? 2 * kStage : kC;
};

// Dense bf16 GEMM on masked weights (N:M ratios with N > 2), general fallback (any alignment, any
// contraction length).  Workgroup tile BM (weight rows a) x BN (tokens t); both operands go global ->
// registers -> padded LDS -> MFMA fragments, one stage prefetched in registers; the weight granules
// come from the fragment-major dense operand.
// FAST: K is a multiple of BK and all rows start 16-byte aligned: unconditional 16-byte loads.
template <bool FAST, int BM, int BN, int WAVES_M, int WAVES_N>
__global__ void __launch_bounds__(kThreads)
k_gemm_dense_bf16(const uint16_t* __restrict__ A, int64_t Adim, int64_t K, const uint16_t* __restrict__ Bm,
                  int64_t T, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc, int tiles_a, bool vecA,
                  bool vecB, bool vecC) {
    static_assert(WAVES_M * WAVES_N == kThreads / 64, "four wavefronts");
    using S = Smem<BM, BN>;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    extern __shared__ u32x4 smem_u4[];
    uint8_t* smem = reinterpret_cast<uint8_t*>(smem_u4);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const int l32 = lane & 31, h = lane >> 5;
    // Tile order as in the 2:4 kernel: workgroup ids are dealt round-robin to the 8 XCDs, so XCD x takes a
    // contiguous chunk of a sequence in which 8 token tiles x all weight tiles run side by side and share
    // that XCD's L2.
    constexpr int kGroupT = 8;
    const int64_t tiles_t = ceil_div(T, BN);
    const int64_t total = tiles_t * tiles_a;
    const int64_t per_xcd = ceil_div(total, 8);
    const int64_t n = static_cast<int64_t>(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (n >= total) return;
    const int64_t grp = n / (static_cast<int64_t>(kGroupT) * tiles_a);
    const int64_t first_t = grp * kGroupT;
    const int64_t gsz = (tiles_t - first_t) < kGroupT ? (tiles_t - first_t) : kGroupT;
    const int64_t within = n - grp * kGroupT * tiles_a;
    const int64_t a0 = (within / gsz) * BM;
    const int64_t t0 = (first_t + within % gsz) * BN;
    const int nk = static_cast<int>(ceil_div(K, BK));

    constexpr int NB_ = BN * 8 / kThreads, NA_ = BM * 8 / kThreads;   // 16-byte granules per thread
    u32x4 rb[NB_], ra[NA_];
    const uint16_t* pb[NB_];
    int64_t arow[NA_];                                   // weight row of each of this thread's granules (clamped)
#pragma unroll
    for (int it = 0; it < NB_; ++it) {
        int64_t t = t0 + ((tid + kThreads * it) >> 3);
        pb[it] = Bm + (t < T ? t : T - 1) * ldb;
    }
#pragma unroll
    for (int it = 0; it < NA_; ++it) {
        int64_t a = a0 + ((tid + kThreads * it) >> 3);
        arow[it] = a < Adim ? a : Adim - 1;
    }
    const int64_t ksA = ceil_div(K, 128);                // stages of the padded fragment-major weight operand
    const int g8 = (tid & 7) * 8;                        // this thread's k offset inside a stage

#define BIMASK_DENSE_LOAD(kt)                                                                     \
    {                                                                                             \
        const int64_t k = static_cast<int64_t>(kt) * BK + g8;                                     \
        _Pragma("unroll") for (int it = 0; it < NB_; ++it) {                                      \
            if constexpr (FAST) rb[it] = *reinterpret_cast<const u32x4*>(pb[it] + k);             \
            else rb[it] = load_granule(pb[it], k, K, vecB);                                       \
        }                                                                                         \
        /* the weight operand is padded to whole stages: every granule exists (zeros beyond K) */ \
        _Pragma("unroll") for (int it = 0; it < NA_; ++it)                                        \
            ra[it] = *reinterpret_cast<const u32x4*>(A + tiled_dense_off(arow[it], k, ksA));      \
    }
#define BIMASK_DENSE_STORE(buf)                                                                   \
    {                                                                                             \
        uint8_t* sA_ = smem + (buf) * S::kStage;                                                  \
        uint8_t* sB_ = sA_ + S::kA;                                                               \
        _Pragma("unroll") for (int it = 0; it < NB_; ++it)                                        \
            *reinterpret_cast<u32x4*>(sB_ + ((tid + kThreads * it) >> 3) * kRowB + (tid & 7) * 16) = rb[it]; \
        _Pragma("unroll") for (int it = 0; it < NA_; ++it)                                        \
            *reinterpret_cast<u32x4*>(sA_ + ((tid + kThreads * it) >> 3) * kRowB + (tid & 7) * 16) = ra[it]; \
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    BIMASK_DENSE_LOAD(0)
    BIMASK_DENSE_STORE(0)
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) BIMASK_DENSE_LOAD(kt + 1)
        const uint8_t* sA = smem + (kt & 1) * S::kStage;
        const uint8_t* sB = sA + S::kA;
#pragma unroll
        for (int c = 0; c < 4; ++c) {                    // four 16-k MFMA steps per stage
            bf16x8 af[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(sA + (wm * WM + i * 32 + l32) * kRowB + c * 32 + h * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const bf16x8 bf = *reinterpret_cast<const bf16x8*>(sB + (wn * WN + j * 32 + l32) * kRowB + c * 32 + h * 16);
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf, acc[i][j], 0, 0, 0);
            }
        }
        if (more) BIMASK_DENSE_STORE((kt + 1) & 1)
        __syncthreads();
    }
#undef BIMASK_DENSE_LOAD
#undef BIMASK_DENSE_STORE

    // Epilogue: accumulators -> bf16 tile [t][a] in LDS -> 16-byte row-contiguous stores.
    uint8_t* sC = smem;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int t = wn * WN + j * 32 + l32;
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const int a = wm * WM + i * 32 + 8 * qq + 4 * h;
                u32x2 v;
                v.x = pack_bf16(acc[i][j][4 * qq + 0], acc[i][j][4 * qq + 1]);
                v.y = pack_bf16(acc[i][j][4 * qq + 2], acc[i][j][4 * qq + 3]);
                *reinterpret_cast<u32x2*>(sC + t * S::kCRow + a * 2) = v;
            }
        }
    __syncthreads();
    constexpr int GPR = BM / 8;                          // 16-byte granules per output row
    for (int q = tid; q < BN * GPR; q += kThreads) {
        const int row = q / GPR, g = q % GPR;
        const int64_t t = t0 + row, a = a0 + 8 * g;
        if (t >= T || a >= Adim) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(sC + row * S::kCRow + g * 16);
        uint16_t* dst = C + t * ldc + a;
        if (vecC && a + 8 <= Adim) {
            *reinterpret_cast<u32x4*>(dst) = v;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (a + e < Adim) dst[e] = static_cast<uint16_t>(v[e >> 1] >> (16 * (e & 1)));
        }
    }
}

// ---------------------------------------------------------------------------------
// fp32: 64 x 64 tile, 16 x 16 threads, 4 x 4 outputs per thread, plain FMA.
// ---------------------------------------------------------------------------------
template <bool SPARSE>
__global__ void __launch_bounds__(kThreads)
k_gemm_f32(const float* __restrict__ A, const uint32_t* __restrict__ Ameta, int64_t Adim, int64_t K,
           const float* __restrict__ Bm, int64_t T, int64_t ldb, float* __restrict__ C, int64_t ldc) {
    constexpr int TS = 64, KS = 32;
    __shared__ float sA[TS][KS + 1];
    __shared__ float sB[TS][KS + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t a0 = static_cast<int64_t>(blockIdx.x) * TS, t0 = static_cast<int64_t>(blockIdx.y) * TS;
    const int64_t ks = ceil_div(K, 128);                 // stages of the fragment-major operand
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < K; k0 += KS) {
        for (int idx = threadIdx.x; idx < TS * KS; idx += kThreads) {
            const int r = idx / KS, k = idx % KS;
            const int64_t gk = k0 + k;
            float va = 0.f, vb = 0.f;
            if (gk < K) {
                const int64_t a = a0 + r, t = t0 + r;
                if (t < T) vb = Bm[t * ldb + gk];
                if (a < Adim) {
                    if constexpr (SPARSE) {
                        const int64_t g = gk >> 2;
                        const int pos = static_cast<int>(gk & 3);
                        const uint32_t nib = (Ameta[tiled_idx_word(a, g, ks)] >> (4 * (g & 7))) & 15u;
                        const int p0 = nib & 3, p1 = nib >> 2;
                        if (pos == p0) va = A[tiled_val_off(a, 2 * g, ks)];
                        else if (pos == p1) va = A[tiled_val_off(a, 2 * g + 1, ks)];
                    } else {
                        va = A[tiled_dense_off(a, gk, ks)];
                    }
                }
            }
            sA[r][k] = va;
            sB[r][k] = vb;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < KS; ++k) {
            float av[4], bv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { av[u] = sA[tx * 4 + u][k]; bv[u] = sB[ty * 4 + u][k]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(bv[u], av[v], acc[u][v]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t t = t0 + ty * 4 + u, a = a0 + tx * 4 + v;
            if (t < T && a < Adim) C[t * ldc + a] = acc[u][v];
        }
}

// out[t][r] = in[t][perm[r]]   (the column permutation of g(Y) in Eq. 10)
template <typename raw>
__global__ void __launch_bounds__(kThreads)
k_gather_cols(const raw* __restrict__ in, int64_t T, int64_t ld, const int32_t* __restrict__ perm, int64_t I,
              raw* __restrict__ out, bool vec) {
    constexpr int E = 16 / sizeof(raw);
    const int64_t chunks = ceil_div(I, E);
    const int64_t id = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (id >= T * chunks) return;
    const int64_t t = id / chunks, r0 = (id - t * chunks) * E;
    const raw* src = in + t * ld;
    raw v[E];
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = (r0 + e < I) ? src[perm[r0 + e]] : static_cast<raw>(0);
    raw* dst = out + t * I + r0;
    if (vec && r0 + E <= I) {
        uint4 pk;
        if constexpr (sizeof(raw) == 2) {
            pk.x = v[0] | (static_cast<uint32_t>(v[1]) << 16); pk.y = v[2] | (static_cast<uint32_t>(v[3]) << 16);
            pk.z = v[4] | (static_cast<uint32_t>(v[5]) << 16); pk.w = v[6] | (static_cast<uint32_t>(v[7]) << 16);
        } else {
            pk.x = v[0]; pk.y = v[1]; pk.z = v[2]; pk.w = v[3];
        }
        *reinterpret_cast<uint4*>(dst) = pk;
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e)
            if (r0 + e < I) dst[e] = v[e];
    }
}

// Same result, for rows that fit in LDS: a workgroup reads `rows` whole token rows with
// contiguous 16-byte lanes, keeps them in LDS, and every thread assembles 16-byte pieces of
// the permuted rows from 2- or 4-byte LDS reads.  Both global streams are fully coalesced.
// CPT > 0 (long rows): the grid is persistent, a thread owns the same CPT 16-byte output
// columns in every row tile and keeps their permutation entries in registers, so the
// permutation is read once per workgroup instead of once per row tile.
template <typename raw, int CPT>
__global__ void __launch_bounds__(kThreads)
k_gather_cols_lds(const raw* __restrict__ in, int64_t T, int64_t ld, const int32_t* __restrict__ perm, int64_t I,
                  raw* __restrict__ out, int rows, bool vec_in, bool vec_out) {
    constexpr int E = 16 / sizeof(raw);
    constexpr int NP = CPT > 0 ? CPT : 1;
    extern __shared__ uint4 gather_smem[];
    raw* buf = reinterpret_cast<raw*>(gather_smem);
    const int chunks = static_cast<int>(ceil_div(I, E));
    const int Ipad = chunks * E;
    const int64_t ntiles = ceil_div(T, rows);
    int p[NP][E];
    if constexpr (CPT > 0) {
#pragma unroll
        for (int k = 0; k < CPT; ++k) {
            const int c = threadIdx.x + kThreads * k;
#pragma unroll
            for (int e = 0; e < E; ++e) p[k][e] = (c * E + e < I) ? perm[c * E + e] : 0;
        }
    }
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t t0 = tile * rows;
        const int nrows = static_cast<int>((T - t0) < rows ? (T - t0) : rows);
        for (int idx = threadIdx.x; idx < nrows * chunks; idx += kThreads) {
            const int row = idx / chunks, c = idx - row * chunks;
            const raw* src = in + (t0 + row) * ld + static_cast<int64_t>(c) * E;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (vec_in && (c + 1) * E <= I) {
                v = *reinterpret_cast<const uint4*>(src);
            } else {
                uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (c * E + e < I) {
                        if constexpr (sizeof(raw) == 2) w[e >> 1] |= static_cast<uint32_t>(src[e]) << (16 * (e & 1));
                        else w[e] = src[e];
                    }
                v = make_uint4(w[0], w[1], w[2], w[3]);
            }
            *reinterpret_cast<uint4*>(buf + static_cast<int64_t>(row) * Ipad + c * E) = v;
        }
        __syncthreads();
        auto emit = [&](int c, const int (&pc)[E]) {
            for (int row = 0; row < nrows; ++row) {
                const raw* r = buf + static_cast<int64_t>(row) * Ipad;
                uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const uint32_t x = r[pc[e]];
                    if constexpr (sizeof(raw) == 2) w[e >> 1] |= x << (16 * (e & 1));
                    else w[e] = x;
                }
                raw* dst = out + (t0 + row) * I + static_cast<int64_t>(c) * E;
                if (vec_out && (c + 1) * E <= I) {
                    *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < E; ++e)
                        if (c * E + e < I) {
                            if constexpr (sizeof(raw) == 2) dst[e] = static_cast<raw>(w[e >> 1] >> (16 * (e & 1)));
                            else dst[e] = w[e];
                        }
                }
            }
        };
        if constexpr (CPT > 0) {
#pragma unroll
            for (int k = 0; k < CPT; ++k) {
                const int c = threadIdx.x + kThreads * k;
                if (c < chunks) emit(c, p[k]);
            }
        } else {
            for (int c = threadIdx.x; c < chunks; c += kThreads) {
#pragma unroll
                for (int e = 0; e < E; ++e) p[0][e] = (c * E + e < I) ? perm[c * E + e] : 0;
                emit(c, p[0]);
            }
        }
        __syncthreads();                                 // the tile buffer is reused by the next row tile
    }
}

// The same gather for bf16 rows that are 16-byte aligned and a multiple of 8 long, with R = 2, 4 or 8 token rows
// per tile INTERLEAVED in LDS: element (column c, row r) sits at 2 (c R + r), so one LDS read of 2 R bytes at
// a permuted column returns that column for all R rows (R times fewer LDS reads than row-major tiles).  A
// thread owns the same CPT chunks of 8 columns in every tile, for the load (R global 16-byte loads per chunk,
// an 8 x R transpose of half-words in registers, R contiguous 16-byte LDS writes) and for the emit (8 LDS
// reads, the transpose back, R 16-byte stores), and keeps the chunks' permutation entries in registers as
// LDS byte offsets.  Persistent grid; the loads of the next tile are in flight while a tile is emitted.
// Measured at 8192 tokens: 8 KB rows (R = 8) 29 us against 38 us row-major, 22 KB rows (R = 2) 87 us against
// 92 us; a plain device-to-device copy of the same arrays takes 24 / 64 us.
template <int R> struct GatherVec;
template <> struct GatherVec<2> { using type = uint32_t; };
template <> struct GatherVec<4> { using type = uint2; };
template <> struct GatherVec<8> { using type = uint4; };

template <int R, int CPT>
__global__ void __launch_bounds__(kThreads)
k_gather_cols_rows(const uint16_t* __restrict__ in, int64_t T, int64_t ld, const int32_t* __restrict__ perm, int I,
                   uint16_t* __restrict__ out) {
    using vec = typename GatherVec<R>::type;
    constexpr int W = R / 2;                             // dwords per column group
    extern __shared__ uint4 gather_smem[];
    uint8_t* buf = reinterpret_cast<uint8_t*>(gather_smem);
    const int chunks = I / 8;
    const int64_t ntiles = ceil_div(T, R);
    int p[CPT][8];
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
        const int c = threadIdx.x + kThreads * k;
#pragma unroll
        for (int e = 0; e < 8; ++e) p[k][e] = c < chunks ? perm[c * 8 + e] * (2 * R) : 0;
    }
    // the loads of a tile are issued before the previous tile is emitted: they are in flight during its LDS reads and stores
    uint4 v[CPT][R];
    auto load_tile = [&](int64_t tile) {
        const int64_t t0 = tile * R;
#pragma unroll
        for (int k = 0; k < CPT; ++k) {
            const int c = threadIdx.x + kThreads * k;
            if (c < chunks) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int64_t t = t0 + r < T ? t0 + r : T - 1;      // rows beyond T repeat the last row (never stored)
                    v[k][r] = *reinterpret_cast<const uint4*>(in + t * ld + c * 8);
                }
            }
        }
    };
    if (static_cast<int64_t>(blockIdx.x) < ntiles) load_tile(blockIdx.x);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t t0 = tile * R;
        __syncthreads();                                 // the previous tile has been emitted
#pragma unroll
        for (int k = 0; k < CPT; ++k) {
            const int c = threadIdx.x + kThreads * k;
            if (c < chunks) {
                // 8 columns x R rows: column e of the chunk -> R half-words (rows 0 .. R-1)
                uint32_t o[8][W];
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        const uint32_t a = reinterpret_cast<const uint32_t*>(&v[k][2 * w])[e >> 1];
                        const uint32_t b = reinterpret_cast<const uint32_t*>(&v[k][2 * w + 1])[e >> 1];
                        o[e][w] = (e & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
                    }
                uint32_t* dst = reinterpret_cast<uint32_t*>(buf + static_cast<size_t>(c) * (16 * R));
#pragma unroll
                for (int q = 0; q < 8 * W; ++q)          // R 16-byte writes: 8 columns x W dwords
                    if ((q & 3) == 0)
                        *reinterpret_cast<uint4*>(dst + q) = make_uint4(o[(q + 0) / W][(q + 0) % W], o[(q + 1) / W][(q + 1) % W],
                                                                        o[(q + 2) / W][(q + 2) % W], o[(q + 3) / W][(q + 3) % W]);
            }
        }
        __syncthreads();
        if (tile + gridDim.x < ntiles) load_tile(tile + gridDim.x);
#pragma unroll
        for (int k = 0; k < CPT; ++k) {
            const int c = threadIdx.x + kThreads * k;
            if (c < chunks) {
                uint32_t g[8][W];                        // permuted column e of the chunk, R rows
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const vec x = *reinterpret_cast<const vec*>(buf + p[k][e]);
#pragma unroll
                    for (int w = 0; w < W; ++w) g[e][w] = reinterpret_cast<const uint32_t*>(&x)[w];
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (t0 + r < T) {
                        uint32_t wd[4];
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const uint32_t a = g[2 * d][r >> 1], b = g[2 * d + 1][r >> 1];
                            wd[d] = (r & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
                        }
                        typedef unsigned int gv4 __attribute__((ext_vector_type(4)));
                        const gv4 pk = {wd[0], wd[1], wd[2], wd[3]};
                        __builtin_nontemporal_store(pk, reinterpret_cast<gv4*>(out + (t0 + r) * I + c * 8));
                    }
                }
            }
        }
    }
}

template <int R, int CPT>
int run_gather_rows(const void* dY, int64_t T, int64_t ld, const int32_t* perm, int64_t I, void* out, hipStream_t s) {
    auto kern = k_gather_cols_rows<R, CPT>;
    const size_t lds = static_cast<size_t>(I) * 2 * R;
    if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess) return BIMASK_ERR_HIP;
    const int64_t ntiles = ceil_div(T, R);
    const int64_t per_cu = static_cast<int64_t>(160 * 1024 / lds) < 4 ? static_cast<int64_t>(160 * 1024 / lds) : 4;
    const unsigned grid = static_cast<unsigned>(ntiles < 256 * per_cu ? ntiles : 256 * per_cu);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, static_cast<const uint16_t*>(dY), T, ld, perm,
                       static_cast<int>(I), static_cast<uint16_t*>(out));
    return check_launch();
}

template <typename raw, int CPT>
int run_gather_lds(const void* dY, int64_t T, int64_t ld, const int32_t* perm, int64_t I, void* out, int rows,
                   size_t lds, unsigned grid, bool vec_in, bool vec_out, hipStream_t s) {
    auto kern = k_gather_cols_lds<raw, CPT>;
    if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess) return BIMASK_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, static_cast<const raw*>(dY), T, ld, perm, I,
                       static_cast<raw*>(out), rows, vec_in, vec_out);
    return check_launch();
}

template <bool FAST, int BM, int BN, int WAVES_M, int WAVES_N>
int run_dense_t(const void* A, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb, void* C,
                int64_t ldc, hipStream_t s) {
    using S = Smem<BM, BN>;
    auto kern = k_gemm_dense_bf16<FAST, BM, BN, WAVES_M, WAVES_N>;
    if (S::kTotal > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                S::kTotal) != hipSuccess) return BIMASK_ERR_HIP;
    }
    const bool vecA = aligned16(A) && (K * 2) % 16 == 0;
    const bool vecB = aligned16(Bm) && (ldb * 2) % 16 == 0;
    const bool vecC = aligned16(C) && (ldc * 2) % 16 == 0;
    const int tiles_a = static_cast<int>(ceil_div(Adim, BM));
    const int64_t tiles_t = ceil_div(T, BN);
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(ceil_div(tiles_a * tiles_t, 8) * 8)), dim3(kThreads), S::kTotal, s,
                       static_cast<const uint16_t*>(A), Adim, K, static_cast<const uint16_t*>(Bm), T, ldb,
                       static_cast<uint16_t*>(C), ldc, tiles_a, vecA, vecB, vecC);
    return check_launch();
}

int run_dense(const void* A, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb, void* C,
              int64_t ldc, hipStream_t s) {
    const bool fast = K % BK == 0 && aligned16(A) && aligned16(Bm) && (ldb * 2) % 16 == 0;
    if (fast) return run_dense_t<true, 128, 128, 2, 2>(A, Adim, K, Bm, T, ldb, C, ldc, s);
    return run_dense_t<false, 128, 128, 2, 2>(A, Adim, K, Bm, T, ldb, C, ldc, s);
}

}  // namespace

int launch_gather_cols(const void* dY, int64_t T, int64_t ld, const int32_t* perm, int64_t I, int dtype,
                       void* out, hipStream_t s) {
    const size_t esz = dtype == BIMASK_BF16 ? 2 : 4;
    const int64_t E = 16 / static_cast<int64_t>(esz);
    const size_t row_bytes = static_cast<size_t>(round_up(I, E)) * esz;
    if (row_bytes <= 64 * 1024) {
        // rows kept in LDS: as many as fit in 64 KB, but enough workgroups to fill the chip
        int64_t rows = static_cast<int64_t>((64 * 1024) / row_bytes);
        if (rows > 32) rows = 32;
        while (rows > 1 && ceil_div(T, rows) < 1024) rows /= 2;
        const size_t lds = static_cast<size_t>(rows) * row_bytes;
        const bool vec_in = aligned16(dY) && (ld * esz) % 16 == 0;
        const bool vec_out = aligned16(out) && (I * esz) % 16 == 0;
        const int64_t ntiles = ceil_div(T, rows);
        const int64_t cpt = ceil_div(ceil_div(I, E), kThreads);      // 16-byte output columns per thread
        // long aligned bf16 rows with enough of them: row-interleaved tiles.  Rows of 4-8 KB (2 chunks of 8 columns
        // per thread) fit 8 to a tile, of 8-16 KB (3-4 chunks) 4, of 16-24 KB (5-6 chunks) 2.
        if (dtype == BIMASK_BF16 && vec_in && vec_out && I % 8 == 0 && cpt >= 2 && cpt <= 6 && T >= 2048) {
            if (cpt <= 2) return run_gather_rows<8, 2>(dY, T, ld, perm, I, out, s);
            if (cpt <= 4) return run_gather_rows<4, 4>(dY, T, ld, perm, I, out, s);
            return run_gather_rows<2, 6>(dY, T, ld, perm, I, out, s);
        }
        // long rows: persistent grid (3 workgroups per CU), permutation entries in registers
        const bool persistent = cpt >= 2 && cpt <= 8;
        const unsigned grid = static_cast<unsigned>(persistent && ntiles > 768 ? 768 : ntiles);
        const int r = static_cast<int>(rows);
#define BIMASK_GATHER(RAW)                                                                                       \
        {                                                                                                        \
            if (!persistent) return run_gather_lds<RAW, 0>(dY, T, ld, perm, I, out, r, lds, grid, vec_in, vec_out, s); \
            if (cpt <= 2) return run_gather_lds<RAW, 2>(dY, T, ld, perm, I, out, r, lds, grid, vec_in, vec_out, s);    \
            if (cpt <= 4) return run_gather_lds<RAW, 4>(dY, T, ld, perm, I, out, r, lds, grid, vec_in, vec_out, s);    \
            if (cpt <= 6) return run_gather_lds<RAW, 6>(dY, T, ld, perm, I, out, r, lds, grid, vec_in, vec_out, s);    \
            return run_gather_lds<RAW, 8>(dY, T, ld, perm, I, out, r, lds, grid, vec_in, vec_out, s);                  \
        }
        if (dtype == BIMASK_BF16) BIMASK_GATHER(uint16_t)
        BIMASK_GATHER(uint32_t)
#undef BIMASK_GATHER
    }
    if (dtype == BIMASK_BF16) {
        const int64_t total = T * ceil_div(I, 8);
        const bool vec = aligned16(out) && (I * 2) % 16 == 0;
        hipLaunchKernelGGL(k_gather_cols<uint16_t>, dim3(static_cast<unsigned>(ceil_div(total, kThreads))),
                           dim3(kThreads), 0, s, static_cast<const uint16_t*>(dY), T, ld, perm, I,
                           static_cast<uint16_t*>(out), vec);
    } else {
        const int64_t total = T * ceil_div(I, 4);
        const bool vec = aligned16(out) && (I * 4) % 16 == 0;
        hipLaunchKernelGGL(k_gather_cols<uint32_t>, dim3(static_cast<unsigned>(ceil_div(total, kThreads))),
                           dim3(kThreads), 0, s, static_cast<const uint32_t*>(dY), T, ld, perm, I,
                           static_cast<uint32_t*>(out), vec);
    }
    return check_launch();
}

bool gemm_bwd_needs_gather(int64_t I, int64_t J, int dtype, int N, int M) {
    if (dtype != BIMASK_BF16) return true;
    if (!uses_sp24(N, M)) return !gemm_dense_rowres_shape(J, I);
    return !(I <= 512 || gemm_sp24_rowres_shape(J, I));
}

int launch_gemm(const void* A_values, const uint32_t* A_index, int64_t Adim, int64_t K, bool sparse24,
                const void* Bm, int64_t T, int64_t ldb, void* C, int64_t ldc, int dtype, hipStream_t s) {
    if (dtype == BIMASK_F32) {
        dim3 grid(static_cast<unsigned>(ceil_div(Adim, 64)), static_cast<unsigned>(ceil_div(T, 64)));
        if (sparse24)
            hipLaunchKernelGGL(k_gemm_f32<true>, grid, dim3(kThreads), 0, s, static_cast<const float*>(A_values),
                               A_index, Adim, K, static_cast<const float*>(Bm), T, ldb, static_cast<float*>(C), ldc);
        else
            hipLaunchKernelGGL(k_gemm_f32<false>, grid, dim3(kThreads), 0, s, static_cast<const float*>(A_values),
                               A_index, Adim, K, static_cast<const float*>(Bm), T, ldb, static_cast<float*>(C), ldc);
        return check_launch();
    }
    if (sparse24) {
        if (K <= 512) {
            // narrow weights: wavefront-private tiles; short contractions (below 256, or below 384 with more
            // than 512 weight rows): token tile resident in LDS, reused by every weight tile; otherwise the
            // streaming kernel below (measured per layer shape: 128 x 512 forward 30 -> 20 us, 2048 x 512 14 -> 10 us)
            int rc = launch_gemm_sp24_narrow(A_values, A_index, Adim, K, Bm, ldb, nullptr, T, C, ldc, s);
            if (rc != BIMASK_ERR_UNSUPPORTED) return rc;
            if (K < 256 || (K < 384 && Adim > 512)) {
                rc = launch_gemm_sp24_resident(A_values, A_index, Adim, K, Bm, ldb, nullptr, T, C, ldc, s);
                if (rc != BIMASK_ERR_UNSUPPORTED) return rc;
            }
        }
        // the largest problems: 512 x 128 tiles, wavefronts of 64 x 128 (fewest L2 and LDS bytes per matrix instruction)
        if (gemm_sp24_big_shape(Adim, K, T)) {
            const int rc = launch_gemm_sp24_big(A_values, A_index, Adim, K, Bm, T, ldb, C, ldc, s);
            if (rc != BIMASK_ERR_UNSUPPORTED) return rc;
        }
        // large problems: 256 x 128 tiles on 8 wavefronts (half the weight traffic per token);
        // otherwise 256 x 64 tiles so that the grid still covers the chip; weight dimensions that
        // would leave a fifth or more of the 256-row tiles empty (384 = 1.5 tiles) take 128-row tiles
        const bool big = ceil_div(Adim, 256) * ceil_div(T, 128) >= 190;
        const int64_t w256 = round_up(Adim, 256), w128 = round_up(Adim, 128);
        const bool narrow = (w256 - w128) * 5 >= w256;
        // few tokens and few weight tiles: 256-row tiles would leave CUs idle
        const bool underfilled = ceil_div(Adim, 256) * ceil_div(T, 64) <= 128;
        const Sp24Tile tile = Adim <= 64 ? Sp24Tile::k64x64
                            : (narrow || underfilled ? Sp24Tile::k128x64 : (big ? Sp24Tile::k256x128 : Sp24Tile::k256x64));
        return launch_gemm_sp24(A_values, A_index, Adim, K, Bm, T, ldb, C, ldc, tile, s);
    }
    {   // dense masked weights: the streaming kernel on the fragment-major operand; else the general kernel
        const int rc = launch_gemm_dense_frag(A_values, Adim, K, Bm, T, ldb, C, ldc, s);
        if (rc != BIMASK_ERR_UNSUPPORTED) return rc;
    }
    return run_dense(A_values, Adim, K, Bm, T, ldb, C, ldc, s);
}

}  // namespace bimask
