// 2:4-sparse bf16 GEMM for gfx950, large-problem variant:  C[t][a] = sum_k Bm[t][k] * A[a][k]
// with A given as compressed values + 2-bit indices (the operand of Eq. 3 / Eq. 10 of
// arXiv 2302.06058), for shapes whose matrix work dominates (thousands of weight rows AND
// thousands of tokens: the MLP block of a transformer).
//
// What bounds such a shape on this chip is not the matrix pipe but the bytes every CU pulls from
// its L2 and from LDS per matrix instruction, so the tile is shaped to cut both:
//   * workgroup tile 512 weight rows x 128 tokens on 8 wavefronts; wavefront w owns weight rows
//     [64 w, 64 w + 64) -- two 32-row tiles -- against ALL 128 tokens: 8 accumulator tiles
//     (128 registers), every token fragment read from LDS feeds two matrix instructions, every
//     weight fragment (registers, straight from L2 in the fragment-major layout) feeds four;
//   * per 128-deep stage a workgroup pulls 72 KB of weights + 32 KB of tokens for 2 x 8.4 MFLOP
//     dense-equivalent (52 KB per 8.4 MFLOP; the 256 x 128 tile of the streaming kernel: 68 KB)
//     and reads 256 KB from LDS (streaming kernel: 256 KB for half the work);
//   * the weight fragments of a stage are not double-buffered as a whole: the registers of sub-step
//     s4 are re-loaded with the NEXT stage's fragment as soon as the sub-step's matrix instructions
//     have been issued (one stage of distance at 32 + 8 registers instead of 72);
//   * the token tile of the next stage goes from registers to the other LDS buffer in the middle of
//     the current stage's matrix instructions, so one barrier is all that separates two stages;
//   * token fragments are read three 32-token sub-tiles ahead of the matrix instructions that use them.
// Measured on the MLP block (11008 x 4096 and 4096 x 11008 weights, 8192 tokens): 1.75-2.0 PFLOP/s
// dense-equivalent against 1.5 with 256 x 128 tiles.  Timing-only ablations of this kernel: without the
// weight loads -15 %, with both load streams always hitting L2 -17 %, matrix instructions alone
// (no loads, no fragment reads) -30 %: what remains is the sustained rate of the matrix pipe itself plus
// the per-tile prologue / epilogue.  Half tiles (512 x 64) for the last, partial round over the chip were
// measured and dropped: the round they save costs less than their lower efficiency (436 vs 460 us).
#include "common.hpp"

namespace bimask {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBigThreads = 512;        // 8 wavefronts
constexpr int kBigRows = 512;           // weight rows per workgroup tile
constexpr int kBigTokens = 128;         // tokens per full tile
constexpr int kBigStage = kBigTokens * 256;          // LDS bytes of one token stage (128 k = 256 B per token)
constexpr int kBigSmem = 2 * kBigStage;              // 64 KB: two stages; the output passes reuse it

union BFragB { bf16x16 v; u32x4 q[2]; };
union AFragB { bf16x8 v; u32x4 q; };

// One workgroup tile: weight rows [a0, a0 + 512) x tokens [t0, t0 + 32 TN).
template <int TN>
__device__ __forceinline__ void
big_tile(const uint16_t* __restrict__ A, const uint32_t* __restrict__ Ameta, int64_t Adim, int nk,
         const uint16_t* __restrict__ Bm, int64_t T, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc,
         int64_t a0, int64_t t0, uint8_t* smem) {
    constexpr int NT = kBigThreads, BN = 32 * TN, TM = 2;
    constexpr int NB_ = BN * 16 / NT;                    // 16-byte token granules per thread and stage (4 or 2)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t rt_last = ceil_div(Adim, 32) - 1;

    // weight fragments: per-lane source pointers (row tiles clamped at the edge: loaded, never stored)
    // (32-bit element offsets from the operands' bases, which sit in scalar registers: the host checks the sizes)
    int pa[TM], pm[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int64_t rt = (a0 >> 5) + wave * TM + i;
        rt = rt < rt_last ? rt : rt_last;
        pa[i] = static_cast<int>((rt * nk * 256 + lane) * 8);
        pm[i] = static_cast<int>((rt * nk * 64 + lane) * 2);
    }
    // token tile: thread -> (row, granule) of a stage
    Bm += t0 * ldb;                                      // the tile's first token row
    int pb[NB_];
    int sb_off[NB_];
#pragma unroll
    for (int it = 0; it < NB_; ++it) {
        const int q = tid + NT * it, row = q >> 4, g = q & 15;
        const int64_t r = t0 + row < T ? row : T - 1 - t0;
        pb[it] = static_cast<int>(r * ldb + 8 * g);
        sb_off[it] = row * 256 + ((g ^ (row & 15)) << 4);
    }

    u32x4 ra[TM][4];                 // weight fragments of the current stage, re-loaded sub-step by sub-step
    u32x2 rmeta[2][TM];              // index words: current and next stage
    u32x4 rb[NB_];                   // token granules of the next stage
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    // prologue: stage 0 of everything
#pragma unroll
    for (int it = 0; it < NB_; ++it) rb[it] = *reinterpret_cast<const u32x4*>(Bm + pb[it]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) ra[i][s4] = *reinterpret_cast<const u32x4*>(A + (pa[i] + s4 * 512));
        rmeta[0][i] = *reinterpret_cast<const u32x2*>(Ameta + pm[i]);
    }

    // token fragment (32 tokens x 32 k of sub-step s4v, token sub-tile j) from the stage buffer sB
#define BIMASK_BIG_FRAG(dst, s4v, j)                                                             \
    {                                                                                            \
        const uint8_t* base = sB + ((j) * 32 + l32) * 256;                                       \
        dst.q[0] = *reinterpret_cast<const u32x4*>(base + (((2 * (s4v) + h) ^ (l32 & 15)) << 4));     \
        dst.q[1] = *reinterpret_cast<const u32x4*>(base + (((8 + 2 * (s4v) + h) ^ (l32 & 15)) << 4)); \
    }
#define BIMASK_BIG_MFMA(frag, s4v, j, MS)                                                        \
    {                                                                                            \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            AFragB af;                                                                           \
            af.q = ra[i][s4v];                                                                   \
            const int idx = static_cast<int>((s4v) < 2 ? rmeta[MS][i].x : rmeta[MS][i].y);       \
            if ((s4v) & 1)                                                                       \
                acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, frag.v, acc[i][j], idx, 0, 1); \
            else                                                                                 \
                acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, frag.v, acc[i][j], idx, 0, 0); \
        }                                                                                        \
    }
    // One stage.  MS = slot of this stage's index words.  The stage's token tile is already in LDS
    // (buffer kt & 1).  In the middle of the stage's matrix instructions the NEXT stage's token granules
    // (in registers since the middle of the previous stage) go to the other LDS buffer and the stage
    // after that is requested, so the only thing between two stages is one barrier.  Loads past the last
    // stage are clamped to it (never skipped): the number of loads in flight at every wait is the same
    // in every step.  Token fragments are read kDepth sub-tiles ahead of their matrix instructions.
    constexpr int kDepth = 3;
#define BIMASK_BIG_STEP(kt, MS)                                                                  \
    {                                                                                            \
        const uint8_t* sB = smem + ((kt) & 1) * kBigStage;                                       \
        uint8_t* sBw = smem + (((kt) + 1) & 1) * kBigStage;                                      \
        const int ktn = (kt) + 1 < nk ? (kt) + 1 : nk - 1;                                       \
        const int ktn2 = (kt) + 2 < nk ? (kt) + 2 : nk - 1;                                      \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
            rmeta[1 - (MS)][i] = *reinterpret_cast<const u32x2*>(Ameta + (pm[i] + ktn * 128));   \
        BFragB f[kDepth + 1];                                                                    \
        _Pragma("unroll") for (int d = 0; d < kDepth; ++d)                                       \
            BIMASK_BIG_FRAG(f[d], d / TN, d % TN)                                                \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {                                       \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                     \
                const int q = s4 * TN + j;                                                       \
                if (q + kDepth < 4 * TN)                                                         \
                    BIMASK_BIG_FRAG(f[(q + kDepth) % (kDepth + 1)], (q + kDepth) / TN, (q + kDepth) % TN) \
                BIMASK_BIG_MFMA(f[q % (kDepth + 1)], s4, j, MS)                                  \
            }                                                                                    \
            /* this sub-step's weight registers are free: fetch the next stage's fragment */     \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                       \
                ra[i][s4] = *reinterpret_cast<const u32x4*>(A + (pa[i] + (ktn * 4 + s4) * 512)); \
            if (s4 == 1) {                                                                       \
                _Pragma("unroll") for (int it = 0; it < NB_; ++it)                               \
                    *reinterpret_cast<u32x4*>(sBw + sb_off[it]) = rb[it];                        \
                _Pragma("unroll") for (int it = 0; it < NB_; ++it)                               \
                    rb[it] = *reinterpret_cast<const u32x4*>(Bm + (pb[it] + ktn2 * 128));        \
            }                                                                                    \
            __builtin_amdgcn_sched_barrier(0);   /* keep the loads where they are written: a stage ahead of their use */ \
        }                                                                                        \
        __syncthreads();                                                                         \
    }
    {   // stage 0 of the token tile into LDS buffer 0, stage 1 into the registers
#pragma unroll
        for (int it = 0; it < NB_; ++it) *reinterpret_cast<u32x4*>(smem + sb_off[it]) = rb[it];
        const int k1 = 1 < nk ? 1 : 0;
#pragma unroll
        for (int it = 0; it < NB_; ++it) rb[it] = *reinterpret_cast<const u32x4*>(Bm + (pb[it] + k1 * 128));
        __syncthreads();
    }

    int kt = 0;
#pragma unroll 1
    for (; kt + 2 <= nk; kt += 2) {
        BIMASK_BIG_STEP(kt, 0)
        BIMASK_BIG_STEP(kt + 1, 1)
    }
    if (kt < nk) BIMASK_BIG_STEP(kt, 0)
#undef BIMASK_BIG_STEP
#undef BIMASK_BIG_MFMA
#undef BIMASK_BIG_FRAG

    // Epilogue.  A lane holds 4 consecutive weight rows of one token per accumulator quad; a swap
    // between the two lane halves gives it 8 consecutive bf16 (16 bytes) of its token's output row.
    // The tile leaves through LDS in two passes of 256 weight rows (wavefronts 0-3, then 4-7) as whole
    // 512-byte row segments with streaming stores.
    constexpr int UPR = 32;                              // 16-byte units per 256-row segment
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        __syncthreads();                                 // the stage buffers / the previous pass are free
        if ((wave >> 2) == pass) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int t = j * 32 + l32;
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        const uint32_t xlo = pack_bf16(acc[i][j][8 * p + 0], acc[i][j][8 * p + 1]);
                        const uint32_t xhi = pack_bf16(acc[i][j][8 * p + 2], acc[i][j][8 * p + 3]);
                        const uint32_t ylo = pack_bf16(acc[i][j][8 * p + 4], acc[i][j][8 * p + 5]);
                        const uint32_t yhi = pack_bf16(acc[i][j][8 * p + 6], acc[i][j][8 * p + 7]);
                        const auto slo = __builtin_amdgcn_permlane32_swap(xlo, ylo, false, false);
                        const auto shi = __builtin_amdgcn_permlane32_swap(xhi, yhi, false, false);
                        const u32x4 v = {slo[0], shi[0], slo[1], shi[1]};
                        const int u = ((wave & 3) * 64 + i * 32 + 16 * p + 8 * h) >> 3;
                        *reinterpret_cast<u32x4*>(smem + t * 512 + ((u ^ ((2 * t) & (UPR - 1))) << 4)) = v;
                    }
                }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < BN * UPR / NT; ++it) {
            const int q = tid + NT * it, t = q / UPR, u = q % UPR;
            const u32x4 v = *reinterpret_cast<const u32x4*>(smem + t * 512 + ((u ^ ((2 * t) & (UPR - 1))) << 4));
            const int64_t a = a0 + pass * 256 + 8 * u;
            if (t0 + t < T && a < Adim) {
                uint16_t* dst = C + (t0 + t) * ldc + a;
                if (a + 8 <= Adim) {
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (a + e < Adim) dst[e] = static_cast<uint16_t>(v[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
    }
}

// Work order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2: XCD x owns the
// contiguous run of `tpx` token tiles starting at x * tpx, against all weight tiles.  Its workgroups start in
// the order of their position in the XCD's sequence, token tile fastest, so that the ~32 workgroups an XCD
// runs at one time share a few weight tiles and all of its token tiles through that XCD's L2.
__global__ void __launch_bounds__(kBigThreads)
k_gemm_sp24_big(const uint16_t* __restrict__ A, const uint32_t* __restrict__ Ameta, int64_t Adim, int nk,
                const uint16_t* __restrict__ Bm, int64_t T, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc,
                int tiles_a, int tiles_t, int tpx) {
    extern __shared__ u32x4 smem_u4[];
    uint8_t* smem = reinterpret_cast<uint8_t*>(smem_u4);
    const int x = blockIdx.x & 7, pos = blockIdx.x >> 3;
    const int t_begin = x * tpx < tiles_t ? x * tpx : tiles_t;
    const int nt = t_begin + tpx < tiles_t ? tpx : tiles_t - t_begin;
    if (pos >= nt * tiles_a) return;                     // whole workgroup, before any barrier
    const int ta = pos / nt, tt = pos - ta * nt;
    big_tile<4>(A, Ameta, Adim, nk, Bm, T, ldb, C, ldc, static_cast<int64_t>(ta) * kBigRows,
                static_cast<int64_t>(t_begin + tt) * kBigTokens, smem);
}

}  // namespace

// Shapes the large-problem kernel takes: whole stages, a contraction long enough (at least 8 stages) that a
// tile's matrix loop outweighs its prologue and epilogue, and enough tiles that the chip is covered twice over.
bool gemm_sp24_big_shape(int64_t Adim, int64_t K, int64_t T) {
    return K % 128 == 0 && K >= 1024 && Adim >= 1024 && Adim % 8 == 0 &&
           ceil_div(Adim, kBigRows) * ceil_div(T, kBigTokens) >= 512;
}

int launch_gemm_sp24_big(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bm, int64_t T,
                         int64_t ldb, void* C, int64_t ldc, hipStream_t s) {
    if (!gemm_sp24_big_shape(Adim, K, T)) return BIMASK_ERR_UNSUPPORTED;
    if (!aligned16(A) || !aligned16(meta) || !aligned16(Bm) || !aligned16(C) || ldb % 8 || ldc % 8) return BIMASK_ERR_UNSUPPORTED;
    // 32-bit offsets inside the operand and inside a token tile, 32-bit tile counts
    if (round_up(Adim, 32) * (K / 2) > 0x7FFFFFFFll || 128 * ldb + K > 0x7FFFFFFFll ||
        ceil_div(T, kBigTokens) * ceil_div(Adim, kBigRows) > 0x0FFFFFFFll) return BIMASK_ERR_UNSUPPORTED;
    static DeviceMemo attr_set;
    const int dev = DeviceMemo::device();
    auto kern = k_gemm_sp24_big;
    if (!attr_set.get(dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kBigSmem) != hipSuccess)
            return BIMASK_ERR_HIP;
        attr_set.set(dev, 1);
    }
    const int tiles_a = static_cast<int>(ceil_div(Adim, kBigRows));
    const int64_t tiles_t = ceil_div(T, kBigTokens);
    const int64_t tpx = ceil_div(tiles_t, 8);
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(tpx * tiles_a * 8)), dim3(kBigThreads), kBigSmem, s,
                       static_cast<const uint16_t*>(A), meta, Adim, static_cast<int>(K / 128),
                       static_cast<const uint16_t*>(Bm), T, ldb, static_cast<uint16_t*>(C), ldc, tiles_a,
                       static_cast<int>(tiles_t), static_cast<int>(tpx));
    return check_launch();
}

}  // namespace bimask
