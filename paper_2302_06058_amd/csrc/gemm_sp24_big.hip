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
// dense-equivalent against 1.5 with 256 x 128 tiles.  The kernel takes the same time with every matrix
// instruction replaced by one ALU operation: what bounds it is each CU's vector-memory path (104 KB per
// stage, every line an L1 miss by construction, ~53 lines in flight per CU at a mean L2 round trip of 250
// clocks: 27 B/clk/CU), and the tile already holds as many accumulators as the register file allows.
// Half tiles (512 x 64, and 256 x 128 inside the persistent loop) for the last, partial round over the
// chip were measured and dropped: the half round they save costs less than their lower efficiency and
// the second copy of the stage code.
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
constexpr int kBigOut = kBigTokens * 512;            // LDS bytes of the output staging area (one pass of 256 weight rows)
constexpr int kBigSmem = 2 * kBigStage + kBigOut;    // 128 KB: two token stages + output staging

union BFragB { bf16x16 v; u32x4 q[2]; };
union AFragB { bf16x8 v; u32x4 q; };

// Work order.  One workgroup per CU, persistent: 256 workgroups, dealt round-robin to the 8 XCDs (each with its own
// L2).  XCD x owns the contiguous run of `tpx` token tiles starting at x * tpx, against all weight tiles; the tiles
// of an XCD form a sequence, token tile fastest, and workgroup w of the XCD (w = 0 .. 31) works on tiles w, w + 32,
// w + 64, ... of it: the 32 workgroups of an XCD are always on 32 consecutive tiles, which share a few weight tiles
// and all of the XCD's token tiles through its L2.
//
// The stages of a workgroup's tiles form ONE sequence kk = 0, 1, 2, ...: the loads that run one and two stages
// ahead simply run into the next tile's first stages, so a tile's epilogue (accumulators -> LDS staging -> memory)
// is the only thing between the last matrix instruction of one tile and the first of the next; the next tile's
// operands are already in registers / LDS by then.
__global__ void __launch_bounds__(kBigThreads)
k_gemm_sp24_big(const uint16_t* __restrict__ A, const uint32_t* __restrict__ Ameta, int64_t Adim, int nk,
                const uint16_t* __restrict__ Bm, int64_t T, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc,
                int tiles_a, int tiles_t, int tpx) {
    constexpr int NT = kBigThreads, TN = 4, BN = 32 * TN, TM = 2;
    constexpr int NB_ = BN * 16 / NT;                    // 16-byte token granules per thread and stage
    extern __shared__ u32x4 smem_u4[];
    uint8_t* smem = reinterpret_cast<uint8_t*>(smem_u4);
    uint8_t* sOut = smem + 2 * kBigStage;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
    const int l32 = lane & 31, h = lane >> 5;
    const int rt_last = static_cast<int>(ceil_div(Adim, 32)) - 1;

    // this workgroup's tiles
    const int x = blockIdx.x & 7, w = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
    const int t_begin = x * tpx < tiles_t ? x * tpx : tiles_t;
    const int nt = t_begin + tpx < tiles_t ? tpx : tiles_t - t_begin;
    const int ntiles = nt * tiles_a;                     // tiles of this XCD
    if (w >= ntiles) return;                             // whole workgroup, before any barrier
    const int n_mine = (ntiles - w + per_xcd - 1) / per_xcd;

    // Load cursors.  The weight loads run one stage ahead of the matrix instructions and the token loads two; each
    // has a cursor (tile position in the XCD's sequence, stage inside the tile) that steps through the stages of
    // ALL of the workgroup's tiles, so the loads run over tile boundaries by themselves (after the last tile they
    // stay on it: loads that nobody uses).  Everything a cursor determines is uniform and lives in scalar
    // registers: the addresses are a scalar base plus one per-lane offset that never changes (weights, index
    // words) or is re-derived per stage from the thread's row (tokens: rows past T are clamped to the last one).
    struct Cursor { int pos, stage; };
    auto advance = [&](Cursor& c) {
        const bool wrap = c.stage + 1 == nk;
        c.stage = wrap ? 0 : c.stage + 1;
        c.pos = wrap && c.pos + per_xcd < ntiles ? c.pos + per_xcd : c.pos;
    };
    const uint32_t lane16 = lane * 16, lane8 = lane * 8;
    auto weight_base = [&](const Cursor& c, int i) -> const uint8_t* {       // fragment block (row tile, stage), bytes
        int rt = (c.pos / nt) * (kBigRows / 32) + wave * TM + i;
        rt = rt < rt_last ? rt : rt_last;                                     // clamped at the edge: loaded, never stored
        return reinterpret_cast<const uint8_t*>(A) + (static_cast<int64_t>(rt) * nk + c.stage) * 4096;
    };
    auto index_base = [&](const Cursor& c, int i) -> const uint8_t* {
        int rt = (c.pos / nt) * (kBigRows / 32) + wave * TM + i;
        rt = rt < rt_last ? rt : rt_last;
        return reinterpret_cast<const uint8_t*>(Ameta) + (static_cast<int64_t>(rt) * nk + c.stage) * 512;
    };
    const int row16 = tid >> 4;                          // this thread's token row inside each 32-row group
    const uint32_t g16 = (tid & 15) * 16;                // and its 16-byte granule of the 256-byte stage row
    u32x4 rb[NB_];                   // token granules of the next stage
    auto load_tokens = [&](const Cursor& c) {
        const int64_t t0 = static_cast<int64_t>(t_begin + c.pos % nt) * kBigTokens;
        const int last = static_cast<int>(T - t0 < kBigTokens ? T - t0 : kBigTokens) - 1;   // last valid row of the tile
        const uint8_t* base = reinterpret_cast<const uint8_t*>(Bm + (t0 * ldb + c.stage * 128));
        const uint32_t ldb2 = static_cast<uint32_t>(2 * ldb);
#pragma unroll
        for (int it = 0; it < NB_; ++it) {
            // row 32 it + row16, clamped to `last`: the group's first row goes into the (scalar) base, the rest
            // is min(row16, rows of the group that exist - 1); a group with no row at all reads row `last`
            const int s_it = last - 32 * it;
            const uint8_t* gb = base + static_cast<int64_t>(s_it >= 0 ? 32 * it : last) * ldb2;
            const int r = row16 < (s_it > 0 ? s_it : 0) ? row16 : (s_it > 0 ? s_it : 0);
            rb[it] = *reinterpret_cast<const u32x4*>(gb + (static_cast<uint32_t>(r) * ldb2 + g16));
        }
    };
    // LDS byte offsets, all toggled between the two stage buffers by one XOR per stage: where this thread writes
    // its token granules (the buffer NOT being read), and where this lane reads token fragments: fo[s4][c] is the
    // granule of k = 32 s4 + 8 h + 64 c .. + 8 in the row of token l32 (granules are XOR-swizzled by the row).
    int sb_off[NB_], fo[4][2];
#pragma unroll
    for (int it = 0; it < NB_; ++it) {
        const int q = tid + NT * it, row = q >> 4, g = q & 15;
        sb_off[it] = row * 256 + ((g ^ (row & 15)) << 4);
    }
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
        for (int c = 0; c < 2; ++c) fo[s4][c] = l32 * 256 + (((8 * c + 2 * s4 + h) ^ (l32 & 15)) << 4);

    u32x4 ra[TM][4];                 // weight fragments of the current stage, re-loaded sub-step by sub-step
    u32x2 rmeta[TM], rmeta_next[TM]; // index words: current and next stage
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    // prologue of the first tile: stage 0 of everything, token stage 0 into LDS buffer 0, token stage 1 requested
    Cursor cw{w, 0}, ct{w, 0};
    load_tokens(ct);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const uint8_t* wb = weight_base(cw, i);
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) ra[i][s4] = *reinterpret_cast<const u32x4*>(wb + lane16 + s4 * 1024);
        rmeta[i] = *reinterpret_cast<const u32x2*>(index_base(cw, i) + lane8);
    }
#pragma unroll
    for (int it = 0; it < NB_; ++it) {
        *reinterpret_cast<u32x4*>(smem + sb_off[it]) = rb[it];
        sb_off[it] ^= kBigStage;
    }
    advance(ct);
    load_tokens(ct);
    __syncthreads();

    // token fragment (32 tokens x 32 k of sub-step s4v, token sub-tile j) from the current stage buffer
#define BIMASK_BIG_FRAG(dst, s4v, j)                                                             \
    {                                                                                            \
        dst.q[0] = *reinterpret_cast<const u32x4*>(smem + (fo[s4v][0] + (j) * 8192));            \
        dst.q[1] = *reinterpret_cast<const u32x4*>(smem + (fo[s4v][1] + (j) * 8192));            \
    }
#define BIMASK_BIG_MFMA(frag, s4v, j)                                                            \
    {                                                                                            \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            AFragB af;                                                                           \
            af.q = ra[i][s4v];                                                                   \
            const int idx = static_cast<int>((s4v) < 2 ? rmeta[i].x : rmeta[i].y);               \
            if ((s4v) & 1)                                                                       \
                acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, frag.v, acc[i][j], idx, 0, 1); \
            else                                                                                 \
                acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, frag.v, acc[i][j], idx, 0, 0); \
        }                                                                                        \
    }

    // Epilogue of one tile.  A lane holds 4 consecutive weight rows of one token per accumulator quad; a swap
    // between the two lane halves gives it 8 consecutive bf16 (16 bytes) of its token's output row.  The tile
    // leaves through the LDS staging area in two passes of 256 weight rows (wavefronts 0-3, then 4-7) as whole
    // 512-byte row segments with streaming stores; the accumulators start the next tile at zero.
    constexpr int UPR = 32;                              // 16-byte units per 256-row segment
#define BIMASK_BIG_EPILOGUE()                                                                    \
    {                                                                                            \
        const int ta = pos / nt, tt = pos - ta * nt;                                             \
        const int64_t a0 = static_cast<int64_t>(ta) * kBigRows;                                  \
        const int64_t t0 = static_cast<int64_t>(t_begin + tt) * kBigTokens;                      \
        _Pragma("unroll 1") for (int pass = 0; pass < 2; ++pass) {                               \
            __syncthreads();                             /* the previous pass has been read */   \
            if ((wave >> 2) == pass) {                                                           \
                _Pragma("unroll") for (int i = 0; i < TM; ++i)                                   \
                    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                             \
                        const int t = j * 32 + l32;                                              \
                        _Pragma("unroll") for (int p = 0; p < 2; ++p) {                          \
                            const uint32_t xlo = pack_bf16(acc[i][j][8 * p + 0], acc[i][j][8 * p + 1]); \
                            const uint32_t xhi = pack_bf16(acc[i][j][8 * p + 2], acc[i][j][8 * p + 3]); \
                            const uint32_t ylo = pack_bf16(acc[i][j][8 * p + 4], acc[i][j][8 * p + 5]); \
                            const uint32_t yhi = pack_bf16(acc[i][j][8 * p + 6], acc[i][j][8 * p + 7]); \
                            const auto slo = __builtin_amdgcn_permlane32_swap(xlo, ylo, false, false); \
                            const auto shi = __builtin_amdgcn_permlane32_swap(xhi, yhi, false, false); \
                            const u32x4 v = {slo[0], shi[0], slo[1], shi[1]};                    \
                            const int u = ((wave & 3) * 64 + i * 32 + 16 * p + 8 * h) >> 3;      \
                            *reinterpret_cast<u32x4*>(sOut + t * 512 + ((u ^ ((2 * t) & (UPR - 1))) << 4)) = v; \
                        }                                                                        \
                    }                                                                            \
            }                                                                                    \
            __syncthreads();                                                                     \
            _Pragma("unroll") for (int it = 0; it < BN * UPR / NT; ++it) {                       \
                const int q = tid + NT * it, t = q / UPR, u = q % UPR;                           \
                const u32x4 v = *reinterpret_cast<const u32x4*>(sOut + t * 512 + ((u ^ ((2 * t) & (UPR - 1))) << 4)); \
                const int64_t a = a0 + pass * 256 + 8 * u;                                       \
                if (t0 + t < T && a < Adim)              /* Adim is a multiple of 8: whole 16-byte pieces */ \
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(C + (t0 + t) * ldc + a)); \
            }                                                                                    \
        }                                                                                        \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                       \
                _Pragma("unroll") for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;               \
    }

    // The stages of all of the workgroup's tiles, one after the other.  A stage's token tile is already in LDS.  In
    // the middle of the stage's matrix instructions the NEXT stage's token granules (in registers since the middle
    // of the previous stage) go to the other LDS buffer and the stage after that is requested; the weight registers
    // of sub-step s4 are re-loaded with the next stage's fragment as soon as the sub-step's matrix instructions have
    // been issued.  Token fragments are read kDepth sub-tiles ahead of their matrix instructions.  A stage has no
    // branch: the matrix instructions of one stage and the next are only separated by the barrier.
    constexpr int kDepth = 3;
    int pos = w, kin = 0, left = n_mine;                 // current tile, stage inside it, tiles still to finish
#pragma unroll 1
    for (;;) {
        advance(cw);
        // (re-defined per stage so that the per-lane offsets stay 32-bit next to the scalar bases)
        uint32_t l16 = lane16, l8 = lane8;
        asm volatile("" : "+v"(l16), "+v"(l8));
        const uint8_t* wb[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            wb[i] = weight_base(cw, i);
            rmeta_next[i] = *reinterpret_cast<const u32x2*>(index_base(cw, i) + l8);
        }
        BFragB f[kDepth + 1];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) BIMASK_BIG_FRAG(f[d], d / TN, d % TN)
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int q = s4 * TN + j;
                if (q + kDepth < 4 * TN) BIMASK_BIG_FRAG(f[(q + kDepth) % (kDepth + 1)], (q + kDepth) / TN, (q + kDepth) % TN)
                BIMASK_BIG_MFMA(f[q % (kDepth + 1)], s4, j)
                __builtin_amdgcn_sched_barrier(0);       // fragment reads stay kDepth sub-tiles ahead, in this order
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) ra[i][s4] = *reinterpret_cast<const u32x4*>(wb[i] + l16 + s4 * 1024);
            if (s4 == 1) {
#pragma unroll
                for (int it = 0; it < NB_; ++it) {
                    *reinterpret_cast<u32x4*>(smem + sb_off[it]) = rb[it];
                    sb_off[it] ^= kBigStage;
                }
                advance(ct);
                load_tokens(ct);
            }
            __builtin_amdgcn_sched_barrier(0);           // keep the loads where they are written: a stage ahead of their use
        }
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
            for (int c = 0; c < 2; ++c) fo[s4][c] ^= kBigStage;
#pragma unroll
        for (int i = 0; i < TM; ++i) rmeta[i] = rmeta_next[i];
        __syncthreads();
        if (++kin == nk) {
            BIMASK_BIG_EPILOGUE()
            if (--left == 0) break;
            pos += per_xcd;
            kin = 0;
        }
    }
#undef BIMASK_BIG_EPILOGUE
#undef BIMASK_BIG_MFMA
#undef BIMASK_BIG_FRAG
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
    const int tiles_a = static_cast<int>(ceil_div(Adim, kBigRows));
    const int64_t tiles_t = ceil_div(T, kBigTokens);
    const int64_t tpx = ceil_div(tiles_t, 8);
    // 32-bit element offsets inside the weight operand and inside the token matrix, 32-bit tile counts
    if (round_up(Adim, 32) * (K / 2) > 0x7FFFFFFFll || T * ldb + K > 0x7FFFFFFFll || tiles_t * tiles_a > 0x0FFFFFFFll)
        return BIMASK_ERR_UNSUPPORTED;
    static DeviceMemo attr_set;
    const int dev = DeviceMemo::device();
    auto kern = k_gemm_sp24_big;
    if (!attr_set.get(dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kBigSmem) != hipSuccess)
            return BIMASK_ERR_HIP;
        attr_set.set(dev, 1);
    }
    // 256 persistent workgroups: one per CU (128 KB of LDS and 256 registers per wavefront leave room for one)
    hipLaunchKernelGGL(kern, dim3(256), dim3(kBigThreads), kBigSmem, s,
                       static_cast<const uint16_t*>(A), meta, Adim, static_cast<int>(K / 128),
                       static_cast<const uint16_t*>(Bm), T, ldb, static_cast<uint16_t*>(C), ldc, tiles_a,
                       static_cast<int>(tiles_t), static_cast<int>(tpx));
    return check_launch();
}

}  // namespace bimask
