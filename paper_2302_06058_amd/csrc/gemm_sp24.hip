// 2:4-sparse bf16 GEMM for gfx950, streaming variant:  C[t][a] = sum_k Bm[t][k] * A[a][k]
// with A given as compressed values + 2-bit indices (the operand of Eq. 3 / Eq. 10 of
// arXiv 2302.06058).
//
// Design (one stage = 128 dense k):
//   * the compressed weights never touch LDS: they are stored fragment-major (see
//     include/bimask.h), i.e. the 16 bytes of values lane l needs for instruction s of a
//     stage sit at [row tile][stage][s][l], so a wavefront fetches each A operand as one
//     fully contiguous 1 KB load (and its indices as one 512-byte load) straight into the
//     operand registers;
//   * the token operand is loaded 256 bytes per row with 16-byte lanes, staged through a
//     double-buffered XOR-swizzled LDS tile and read back as 16-byte fragments;
//   * PF stages of both operands are kept in flight in registers, so a workgroup has
//     PF * (BM*72 + BN*256) bytes outstanding to hide HBM latency;
//   * fp32 accumulators are rounded to bf16, regrouped by a swap between the two lane halves
//     and a pass through LDS, and written as whole row segments with streaming stores.
// Lane/operand mapping of v_smfmac_f32_32x32x32_bf16 (checked on the device): lane l holds
// weight row l%32; with h = l/32, compressed element e of the A register pairs with slot
// 8h + 4((e%4)/2) + idx_e of the B register of token lane half e/4, and idx_e sits in bits
// [2e+1:2e] of the 16-bit index set selected by ABID.
#include "common.hpp"

namespace bimask {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte register vector
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int SK = 128;                 // dense k per stage
constexpr int kRowBytes = SK * 2;       // LDS bytes per token row per stage (16 granules)

union BFrag { bf16x16 v; u32x4 q[2]; };
union AFrag { bf16x8 v; u32x4 q; };

template <int BM, int BN>
struct SpSmem {
    static constexpr int kStage = BN * kRowBytes;
    static constexpr int kTotal = 2 * kStage;
};

// 8 consecutive bf16 of a token row starting at element k, zero beyond kend; 4-byte loads
// only (rows that are not 16-byte aligned, or the ragged last stage).
__device__ __forceinline__ u32x4 load_guarded(const uint16_t* row, int64_t k, int64_t kend) {
    u32x4 r = {0u, 0u, 0u, 0u};
    if (k + 8 <= kend) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(row + k);
        r.x = p[0]; r.y = p[1]; r.z = p[2]; r.w = p[3];
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (k + e < kend) r[e >> 1] |= static_cast<uint32_t>(row[k + e]) << (16 * (e & 1));
    }
    return r;
}

// BGUARD: token rows are not 16-byte aligned or K is not a multiple of 128; every token
// load is then bounds-checked against K (the weight operand is zero-padded by its format).
// KTAIL (without BGUARD): rows are 16-byte aligned and K is a multiple of 8 but not of 128: 16-byte token loads as on
// the fast path, the granules of the last stage that lie beyond K are fetched from the row's start and zeroed.
// BHALF: only the first half of the wavefronts fetch the token tile (twice as much each).  The
// token rows come from HBM, the weights from L2; a wavefront's loads complete in order, so weight
// loads queued behind token loads inherit their latency -- with BHALF half of the wavefronts
// carry nothing but L2 hits.
// DENSE: the weight operand is the dense masked matrix of a ratio with N > 2 in its fragment-major layout
// (two 16-byte A fragments per sub-step instead of one compressed fragment plus index bits) and every
// sparse 32x32x32 instruction becomes two dense 32x32x16 ones on the same token fragment halves.
template <int BM, int BN, int WAVES_M, int WAVES_N, int PF, bool BGUARD, bool BHALF, bool KTAIL, bool DENSE>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
k_gemm_sp24(const uint16_t* __restrict__ A, const uint32_t* __restrict__ Ameta, int64_t Adim, int64_t K,
            const uint16_t* __restrict__ Bm, int64_t T, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc,
            int tiles_a, bool vecC) {
    constexpr int NT = 64 * WAVES_M * WAVES_N;          // threads per workgroup
    using S = SpSmem<BM, BN>;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int NBUF = PF + 1;
    constexpr int NTB = BHALF ? NT / 2 : NT;            // threads that fetch the token tile
    constexpr int NB_ = BN * 16 / NTB;                  // 16-byte granules of Bm per fetching thread per stage
    static_assert(NB_ >= 1 && (BN * 16) % NTB == 0, "token tile too small");
    extern __shared__ u32x4 smem_u4[];
    uint8_t* smem = reinterpret_cast<uint8_t*>(smem_u4);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const bool bfetch = !BHALF || __builtin_amdgcn_readfirstlane(wave) < WAVES_M * WAVES_N / 2;   // wave-uniform
    const int l32 = lane & 31, h = lane >> 5;
    // Tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so
    // XCD x takes the contiguous chunk [x*per_xcd, (x+1)*per_xcd) of a grouped tile sequence in
    // which 8 token tiles x consecutive weight tiles run side by side: the ~32 workgroups an
    // XCD holds at one time share 4 weight tiles and 8 token tiles through that XCD's L2.
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
    const int nk = static_cast<int>(ceil_div(K, SK));   // = stages of the padded weight operand
    const int64_t rt_last = ceil_div(Adim, 32) - 1;

    // per-lane source pointers (row tiles / rows clamped at the edges: loaded, never stored)
    const uint16_t* pa[TM];
    const uint32_t* pm[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int64_t rt = (a0 + wm * WM + i * 32) >> 5;
        rt = rt < rt_last ? rt : rt_last;
        pa[i] = A + (rt * nk * (DENSE ? 512 : 256) + lane) * 8;
        pm[i] = DENSE ? nullptr : Ameta + (rt * nk * 64 + lane) * 2;
    }
    const uint16_t* pb[NB_];
    int sb_off[NB_];
    const int g8 = 8 * (tid & 15);                      // first element of this thread's granule within a stage (NTB is a multiple of 16)
#pragma unroll
    for (int it = 0; it < NB_; ++it) {
        const int q = (BHALF ? tid & (NTB - 1) : tid) + NTB * it, row = q >> 4, g = q & 15;
        int64_t t = t0 + row;
        t = t < T ? t : T - 1;
        pb[it] = Bm + t * ldb + (BGUARD ? 0 : 8 * g);
        sb_off[it] = row * kRowBytes + ((g ^ (row & 15)) << 4);
    }

    constexpr int NA = DENSE ? 8 : 4;                   // 16-byte weight fragments per row tile and stage
    u32x4 ra[NBUF][TM][NA];
    u32x2 rmeta[NBUF][DENSE ? 1 : TM];
    u32x4 rb[NBUF][NB_];

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

#define BIMASK_LOAD_STAGE(slot, kt)                                                              \
    {                                                                                            \
        const int64_t kk = static_cast<int64_t>(kt) * SK;                                          \
        if (bfetch) _Pragma("unroll") for (int it = 0; it < NB_; ++it) {                        \
            if constexpr (BGUARD)                                                                \
                rb[slot][it] = load_guarded(pb[it], kk + 8 * ((tid + NTB * it) & 15), K);       \
            else if constexpr (KTAIL) {                                                          \
                const bool in = kk + g8 < K;                                                     \
                const u32x4 v = *reinterpret_cast<const u32x4*>(pb[it] + (in ? kk : -static_cast<int64_t>(g8))); \
                rb[slot][it] = in ? v : (u32x4){0u, 0u, 0u, 0u};                                 \
            } else                                                                               \
                rb[slot][it] = *reinterpret_cast<const u32x4*>(pb[it] + kk);                     \
        }                                                                                        \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            _Pragma("unroll") for (int g = 0; g < NA; ++g)                                       \
                ra[slot][i][g] = *reinterpret_cast<const u32x4*>(pa[i] + (kk * NA + g * SK) * 4); \
            if constexpr (!DENSE) rmeta[slot][i] = *reinterpret_cast<const u32x2*>(pm[i] + kk);  \
        }                                                                                        \
    }

#define BIMASK_READ_FRAGS(dst, s4v)                                                              \
    {                                                                                            \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                         \
            const int row = wn * WN + j * 32 + l32;                                              \
            const uint8_t* base = sB + row * kRowBytes;                                          \
            dst[j].q[0] = *reinterpret_cast<const u32x4*>(base + (((2 * (s4v) + h) ^ (row & 15)) << 4));     \
            dst[j].q[1] = *reinterpret_cast<const u32x4*>(base + (((8 + 2 * (s4v) + h) ^ (row & 15)) << 4)); \
        }                                                                                        \
    }

    // One pipeline step: stage kt leaves its registers for LDS / the matrix cores while stage
    // kt+PF is requested.  Kept free of control flow (loads past the end are clamped to the
    // last stage, never skipped) so that the outstanding-load bookkeeping stays exact and a
    // step only ever waits for the stage it consumes.
#define BIMASK_STEP(u, kt, DO_LOAD)                                                              \
    {                                                                                            \
        uint8_t* sB = smem + ((kt) & 1) * S::kStage;                                             \
        if (bfetch) _Pragma("unroll") for (int it = 0; it < NB_; ++it)                          \
            *reinterpret_cast<u32x4*>(sB + sb_off[it]) = rb[u][it];                              \
        if (DO_LOAD) {                                                                           \
            const int ktl = (kt) + PF < nk ? (kt) + PF : nk - 1;                                 \
            BIMASK_LOAD_STAGE(((u) + PF) % NBUF, ktl)                                            \
        }                                                                                        \
        __syncthreads();                                                                         \
        /* token fragments of instruction s4+1 are requested from LDS before the matrix       \
           instructions of s4 are issued, so LDS latency hides behind them */                 \
        BFrag bf[2][TN];                                                                         \
        BIMASK_READ_FRAGS(bf[0], 0)                                                              \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {                                       \
            if (s4 < 3) BIMASK_READ_FRAGS(bf[(s4 + 1) & 1], s4 + 1)                              \
            _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                     \
                if constexpr (DENSE) {                                                           \
                    _Pragma("unroll") for (int x = 0; x < 2; ++x) {                              \
                        AFrag af;                                                                \
                        af.q = ra[u][i][s4 * 2 + x];                                             \
                        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                         \
                            AFrag bh;                                                            \
                            bh.q = bf[s4 & 1][j].q[x];                                           \
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bh.v, acc[i][j], 0, 0, 0); \
                        }                                                                        \
                    }                                                                            \
                } else {                                                                         \
                    AFrag af;                                                                    \
                    af.q = ra[u][i][s4];                                                         \
                    const int idx = static_cast<int>(s4 < 2 ? rmeta[u][i].x : rmeta[u][i].y);    \
                    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                             \
                        if (s4 & 1)                                                              \
                            acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf[s4 & 1][j].v, acc[i][j], idx, 0, 1); \
                        else                                                                     \
                            acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf[s4 & 1][j].v, acc[i][j], idx, 0, 0); \
                    }                                                                            \
                }                                                                                \
            }                                                                                    \
        }                                                                                        \
    }

#pragma unroll
    for (int s = 0; s < PF; ++s) {
        const int ktl = s < nk ? s : nk - 1;
        BIMASK_LOAD_STAGE(s, ktl)
    }

    int kt0 = 0;
#pragma unroll 1
    for (; kt0 + NBUF <= nk; kt0 += NBUF) {
#pragma unroll
        for (int u = 0; u < NBUF; ++u) BIMASK_STEP(u, kt0 + u, true)
    }
    // fewer than NBUF stages remain: everything they need is already in flight
#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u) {
        if (kt0 + u < nk) BIMASK_STEP(u, kt0 + u, false)
    }
#undef BIMASK_STEP
#undef BIMASK_READ_FRAGS
#undef BIMASK_LOAD_STAGE

    // Epilogue: a lane holds 4 consecutive weight rows of one token per accumulator quad;
    // swapping quads between the two lane halves gives every lane 8 consecutive bf16
    // (16 bytes) of its token row.  The tile goes through LDS (the stage buffers are free now)
    // so that it leaves as whole 2*BM-byte row segments with streaming stores: full lines go
    // straight to memory and neither evict the operands from L2 nor wait there as dirty lines.
    static_assert(BN * BM * 2 <= S::kTotal, "output tile must fit the stage buffers");
    __syncthreads();                                     // every wavefront is done with the last stage
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int t = wn * WN + j * 32 + l32;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const uint32_t xlo = pack_bf16(acc[i][j][8 * p + 0], acc[i][j][8 * p + 1]);
                const uint32_t xhi = pack_bf16(acc[i][j][8 * p + 2], acc[i][j][8 * p + 3]);
                const uint32_t ylo = pack_bf16(acc[i][j][8 * p + 4], acc[i][j][8 * p + 5]);
                const uint32_t yhi = pack_bf16(acc[i][j][8 * p + 6], acc[i][j][8 * p + 7]);
                const auto slo = __builtin_amdgcn_permlane32_swap(xlo, ylo, false, false);
                const auto shi = __builtin_amdgcn_permlane32_swap(xhi, yhi, false, false);
                const u32x4 v = {slo[0], shi[0], slo[1], shi[1]};
                const int u = (wm * WM + i * 32 + 16 * p + 8 * h) >> 3;      // 16-byte unit of the row
                *reinterpret_cast<u32x4*>(smem + t * (BM * 2) + ((u ^ ((2 * t) & (BM / 8 - 1))) << 4)) = v;
            }
        }
    __syncthreads();
    constexpr int UPR = BM / 8;                          // 16-byte units per tile row
#pragma unroll
    for (int it = 0; it < BN * UPR / NT; ++it) {
        const int q = tid + NT * it, t = q / UPR, u = q % UPR;
        const u32x4 v = *reinterpret_cast<const u32x4*>(smem + t * (BM * 2) + ((u ^ ((2 * t) & (UPR - 1))) << 4));
        const int64_t a = a0 + 8 * u;
        if (t0 + t < T && a < Adim) {
            uint16_t* dst = C + (t0 + t) * ldc + a;
            if (vecC && a + 8 <= Adim) {
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
            } else if (a + 8 <= Adim) {
                // rows not 16-byte aligned: 4-byte stores (pointers and pitches are 4-byte aligned)
                uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
                d32[0] = v.x; d32[1] = v.y; d32[2] = v.z; d32[3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (a + e < Adim) dst[e] = static_cast<uint16_t>(v[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int PF, bool BGUARD, bool BHALF, bool KTAIL = false, bool DENSE = false>
int run_sp24_t(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb,
             void* C, int64_t ldc, hipStream_t s) {
    using S = SpSmem<BM, BN>;
    auto kern = k_gemm_sp24<BM, BN, WAVES_M, WAVES_N, PF, BGUARD, BHALF, KTAIL, DENSE>;
    if (S::kTotal > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                S::kTotal) != hipSuccess) return BIMASK_ERR_HIP;
    }
    const bool vecC = aligned16(C) && (ldc * 2) % 16 == 0;
    const int tiles_a = static_cast<int>(ceil_div(Adim, BM));
    const int64_t tiles_t = ceil_div(T, BN);
    const int64_t grid = ceil_div(tiles_a * tiles_t, 8) * 8;      // whole rounds over the 8 XCDs
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(64 * WAVES_M * WAVES_N), S::kTotal, s,
                       static_cast<const uint16_t*>(A), meta, Adim, K, static_cast<const uint16_t*>(Bm), T, ldb,
                       static_cast<uint16_t*>(C), ldc, tiles_a, vecC);
    return check_launch();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int PF, bool BHALF = false>
int run_sp24(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb,
             void* C, int64_t ldc, hipStream_t s) {
    const bool rows16 = aligned16(Bm) && (ldb * 2) % 16 == 0;
    if (rows16 && K % SK == 0) return run_sp24_t<BM, BN, WAVES_M, WAVES_N, PF, false, BHALF>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
    if (rows16 && K % 8 == 0) return run_sp24_t<BM, BN, WAVES_M, WAVES_N, PF, false, BHALF, true>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
    return run_sp24_t<BM, BN, WAVES_M, WAVES_N, 1, true, false>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
}

// dense masked weights: aligned token rows and a contraction that is a multiple of 8 only (the caller
// takes the general dense kernel otherwise)
template <int BM, int BN, int WAVES_M, int WAVES_N, int PF>
int run_dense_frag(const void* A, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb, void* C, int64_t ldc,
                   hipStream_t s) {
    if (K % SK == 0) return run_sp24_t<BM, BN, WAVES_M, WAVES_N, PF, false, false, false, true>(A, nullptr, Adim, K, Bm, T, ldb, C, ldc, s);
    return run_sp24_t<BM, BN, WAVES_M, WAVES_N, PF, false, false, true, true>(A, nullptr, Adim, K, Bm, T, ldb, C, ldc, s);
}

}  // namespace

// 2:4 GEMM on the fragment-major weight operand.
//   256 x 64, 4 wavefronts, 2 stages prefetched: mid-size problems (the grid covers the chip)
//   128 x 64, 4 wavefronts: weight dimensions that would leave 256-row tiles largely empty, or few tokens
//   256 x 128, 8 wavefronts, 1 stage prefetched: large problems (half the weight traffic per token)
//   64 x 64, 4 wavefronts of 32 x 32: at most 64 weight rows (no matrix work or fragment reads on padding rows)
int launch_gemm_sp24(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bm, int64_t T,
                     int64_t ldb, void* C, int64_t ldc, Sp24Tile tile, hipStream_t s) {
    if (!aligned16(A) || !aligned16(meta)) return BIMASK_ERR_ALIGN;
    switch (tile) {
        case Sp24Tile::k256x64: return run_sp24<256, 64, 4, 1, 2, true>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
        case Sp24Tile::k128x64: return run_sp24<128, 64, 4, 1, 2>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
        case Sp24Tile::k256x128: return run_sp24<256, 128, 8, 1, 1>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
        case Sp24Tile::k64x64: return run_sp24<64, 64, 2, 2, 2>(A, meta, Adim, K, Bm, T, ldb, C, ldc, s);
    }
    return BIMASK_ERR_UNSUPPORTED;
}

// The same streaming kernel on the dense masked operand of a ratio with N > 2 (dense 32x32x16 matrix
// instructions).  BIMASK_ERR_UNSUPPORTED when the token rows are not 16-byte aligned or the contraction is no
// multiple of 8: the caller then takes the general dense kernel.
//   128 x 64, 4 wavefronts, 2 stages prefetched; 256 x 128, 8 wavefronts, for large problems; 64 x 64 for at
//   most 64 weight rows.  (256 x 64 with two row tiles per wavefront would need 128 registers of weight
//   fragments per stage in flight.)
int launch_gemm_dense_frag(const void* A, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb, void* C,
                           int64_t ldc, hipStream_t s) {
    if (!aligned16(A) || !aligned16(Bm) || (ldb * 2) % 16 != 0 || K % 8 != 0) return BIMASK_ERR_UNSUPPORTED;
    if (Adim <= 64) return run_dense_frag<64, 64, 2, 2, 2>(A, Adim, K, Bm, T, ldb, C, ldc, s);
    const bool big = ceil_div(Adim, 256) * ceil_div(T, 128) >= 190;
    // weight dimensions that would leave a fifth or more of the 256-row tiles empty (384 = 1.5 tiles) take 128-row tiles
    const int64_t w256 = round_up(Adim, 256), w128 = round_up(Adim, 128);
    const bool wasteful = (w256 - w128) * 5 >= w256;
    if (big && !wasteful) return run_dense_frag<256, 128, 8, 1, 1>(A, Adim, K, Bm, T, ldb, C, ldc, s);
    return run_dense_frag<128, 64, 4, 1, 2>(A, Adim, K, Bm, T, ldb, C, ldc, s);
}

}  // namespace bimask
