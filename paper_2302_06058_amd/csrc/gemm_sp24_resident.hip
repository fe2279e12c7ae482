// 2:4-sparse bf16 GEMM for short contractions (K <= 512), resident-token variant:
//     C[t][a] = sum_k Bsrc[t][perm[k]] * A[a][k]
// This is the backward product of Eq. (10) of arXiv 2302.06058 for layers with few output
// features: k runs over the permuted out-feature index r, Bsrc = g(Y), perm = P.
//
// A workgroup owns a tile of tokens.  It loads that tile of g(Y) ONCE, full rows (contiguous
// 16-byte lanes) into LDS and regroups it there through the permutation into an
// XOR-swizzled LDS tile, so the column permutation of Eq. (10) costs no extra pass over
// memory.  It then walks over ALL weight-row tiles: the fragment-major compressed weights
// stream from L2 straight into the sparse matrix instruction's A registers (prefetched one
// weight tile ahead), the token fragments come from the resident tile (registers when the
// contraction is at most 256 long, LDS otherwise), and every finished output strip
// leaves through a double-buffered LDS tile as whole 512-byte row segments written with
// streaming stores (one barrier per weight tile).
// Token tiles have a run-time height (<= BN) so that the grid can be cut to the CU count.
#include "common.hpp"

namespace bimask {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

union BFragR { bf16x16 v; u32x4 q[2]; };
union AFragR { bf16x8 v; u32x4 q; };

template <int BM, int BN, int NSTG, bool PERSIST>
struct ResSmem {
    static constexpr int kB = NSTG * BN * 256;          // resident token tile, 256 B per row and stage
    static constexpr int kPerm = NSTG * 128 * 2;        // permutation (int16)
    static constexpr int kOut = BN * BM * 2;            // one bf16 output tile (two of them: double buffer)
    // The permutation is only read while the token tile is filled: it sits behind the un-permuted
    // rows inside the output staging area and is re-written from a register for every tile.
    // (Two 256 x 64 workgroups with a 128-long contraction then fit one CU's 160 KB exactly.)
    static constexpr int kInv = 0;
    static constexpr int kFill = kB + kPerm;
    // output staging (two tiles); the un-permuted row tile of the fill phase shares this area
    static constexpr int kArea = 2 * kOut > kFill ? 2 * kOut : kFill;
    static constexpr int kTotal = kB + kInv + kArea;
};

// byte offset of element (t, r) of the resident tile
template <int BN>
__device__ __forceinline__ int resb_off(int t, int r) {
    return (r >> 7) * (BN * 256) + t * 256 + (((((r & 127) >> 3) ^ (t & 15))) << 4) + (r & 7) * 2;
}

// PERSIST: the grid is smaller than the number of token tiles; a workgroup walks over its
// tiles and requests the rows of the next one before it multiplies the current one, and the
// 16-bit copy of the permutation (and, with a single weight tile, the weight fragments) are set
// up once.
template <int BM, int BN, int WAVES_M, int NSTG, bool PERSIST>
__global__ void __launch_bounds__(64 * WAVES_M)
k_gemm_sp24_resident(const uint16_t* __restrict__ A, const uint32_t* __restrict__ Ameta, int64_t Adim, int64_t K,
                     const uint16_t* __restrict__ Bsrc, int64_t ldb, const int32_t* __restrict__ perm, int64_t T,
                     uint16_t* __restrict__ C, int64_t ldc, int rpt, bool vecB, bool vecC) {
    constexpr int NT = 64 * WAVES_M;
    using S = ResSmem<BM, BN, NSTG, PERSIST>;
    constexpr int WM = BM / WAVES_M, TM = WM / 32, TN = BN / 32;
    extern __shared__ u32x4 smem_u4[];
    uint8_t* sB = reinterpret_cast<uint8_t*>(smem_u4);
    uint8_t* lin = sB + S::kB + S::kInv;                               // un-permuted rows (shares the output staging area)
    int16_t* sP = reinterpret_cast<int16_t*>(lin + S::kB);             // the permutation, 16-bit

    const int tid = threadIdx.x, lane = tid & 63, wm = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t ntiles = ceil_div(T, rpt);
    int64_t tile = blockIdx.x;
    int64_t t0 = tile * rpt;
    int rows = static_cast<int>((T - t0) < rpt ? (T - t0) : rpt);
    // blockIdx.y selects a contiguous group of weight tiles (layers with few tokens: more workgroups)
    const int tiles_all = static_cast<int>(ceil_div(Adim, BM));
    const int tiles_per_group = (tiles_all + static_cast<int>(gridDim.y) - 1) / static_cast<int>(gridDim.y);
    const int at_begin = static_cast<int>(blockIdx.y) * tiles_per_group;
    const int tiles_a = at_begin + tiles_per_group < tiles_all ? at_begin + tiles_per_group : tiles_all;   // end of this group
    if (at_begin >= tiles_a) return;                     // whole workgroup, before any barrier
    const int64_t rt_last = ceil_div(Adim, 32) - 1;

    // ---- weight fragments of one weight tile: NSTG stages x TM row tiles
    u32x4 ra[2][NSTG][TM][4];
    u32x2 rmeta[2][NSTG][TM];
#define BIMASK_LOAD_WTILE(set, at)                                                               \
    {                                                                                            \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            int64_t rt = (static_cast<int64_t>(at) * BM + wm * WM + i * 32) >> 5;                \
            rt = rt < rt_last ? rt : rt_last;                                                    \
            const uint16_t* pa = A + (rt * NSTG * 256 + lane) * 8;                               \
            const uint32_t* pm = Ameta + (rt * NSTG * 64 + lane) * 2;                            \
            _Pragma("unroll") for (int st = 0; st < NSTG; ++st) {                                \
                _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                 \
                    ra[set][st][i][s4] = *reinterpret_cast<const u32x4*>(pa + (st * 4 + s4) * 512); \
                rmeta[set][st][i] = *reinterpret_cast<const u32x2*>(pm + st * 128);              \
            }                                                                                    \
        }                                                                                        \
    }
    BIMASK_LOAD_WTILE(0, at_begin)

    // ---- resident token tile.  The g(Y) rows are requested first (registers), then LDS is
    // zeroed and the permutation copied to LDS while they are in flight.
    const int G = static_cast<int>((K + 7) >> 3);        // 8-element granules per token row
    constexpr int NL = (BN * NSTG * 16 + NT - 1) / NT;
    u32x4 v[NL];
#define BIMASK_LOAD_ROWS(T0, ROWS)                                                               \
    _Pragma("unroll") for (int it = 0; it < NL; ++it) {                                          \
        const int q = tid + NT * it;                                                             \
        const int t = q / G, g = q - t * G;                                                      \
        v[it] = (u32x4){0u, 0u, 0u, 0u};                                                         \
        if (q < (ROWS) * G) {                                                                    \
            const uint16_t* src = Bsrc + ((T0) + t) * ldb + 8 * g;                               \
            if (8 * g + 8 <= K) {                                                                \
                if (vecB) v[it] = *reinterpret_cast<const u32x4*>(src);                          \
                else { const uint32_t* p = reinterpret_cast<const uint32_t*>(src); v[it].x = p[0]; v[it].y = p[1]; v[it].z = p[2]; v[it].w = p[3]; } \
            } else {                                                                             \
                _Pragma("unroll") for (int e = 0; e < 8; ++e)                                    \
                    if (8 * g + e < K) v[it][e >> 1] |= static_cast<uint32_t>(src[e]) << (16 * (e & 1)); \
            }                                                                                    \
        }                                                                                        \
    }
    BIMASK_LOAD_ROWS(t0, rows)
    for (int it = tid; it < S::kB / 16; it += NT) reinterpret_cast<u32x4*>(sB)[it] = (u32x4){0u, 0u, 0u, 0u};
    static_assert(NT >= NSTG * 128, "one permutation entry per thread");
    const int16_t pown = perm && tid < static_cast<int>(K) ? static_cast<int16_t>(perm[tid]) : static_cast<int16_t>(0);
    // k positions beyond K keep the zeros written above; rows beyond `rows` keep whatever an
    // earlier tile left (their outputs are never stored).
    for (;;) {
    __syncthreads();                                     // LDS set up / the previous tile is fully consumed
    if (perm) {
        // Eq. (10)'s column gather: the rows go to LDS as they are (16-byte stores), then each
        // thread assembles whole 16-byte granules of the permuted rows from 2-byte LDS reads
        if (tid < NSTG * 128) sP[tid] = pown;
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int q = tid + NT * it;
            const int t = q / G, g = q - t * G;
            if (q < rows * G) *reinterpret_cast<u32x4*>(lin + t * (NSTG * 256) + g * 16) = v[it];
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int q = tid + NT * it;
            const int t = q / G, g = q - t * G;
            if (q < rows * G) {
                const u32x4 pv = *reinterpret_cast<const u32x4*>(sP + 8 * g);   // P[8g .. 8g+7]
                const uint16_t* row = reinterpret_cast<const uint16_t*>(lin + t * (NSTG * 256));
                u32x4 o = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t src_col = (pv[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                    const uint32_t x = 8 * g + e < K ? row[src_col] : 0u;
                    o[e >> 1] |= x << (16 * (e & 1));
                }
                *reinterpret_cast<u32x4*>(sB + resb_off<BN>(t, 8 * g)) = o;
            }
        }
    } else {
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int q = tid + NT * it;
            const int t = q / G, g = q - t * G;
            if (q < rows * G) *reinterpret_cast<u32x4*>(sB + resb_off<BN>(t, 8 * g)) = v[it];
        }
    }
    const int64_t tile_next = tile + gridDim.x;
    int64_t t0_next = 0;
    int rows_next = 0;
    if constexpr (PERSIST) {
        if (tile_next < ntiles) {                        // rows of the next tile: in flight during this one
            t0_next = tile_next * rpt;
            rows_next = static_cast<int>((T - t0_next) < rpt ? (T - t0_next) : rpt);
            BIMASK_LOAD_ROWS(t0_next, rows_next)
        }
    }
    __syncthreads();

    // Short contractions: the token fragments are the same for every weight tile, so they are
    // read from LDS once and stay in registers (NSTG * 4 * TN * 8 VGPRs).
    constexpr bool REGB = NSTG <= 2;
    BFragR bfr[REGB ? NSTG : 1][4][TN];
    if constexpr (REGB) {
#pragma unroll
        for (int st = 0; st < NSTG; ++st)
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int row = j * 32 + l32;
                    const uint8_t* base = sB + st * (BN * 256) + row * 256;
                    bfr[st][s4][j].q[0] = *reinterpret_cast<const u32x4*>(base + (((2 * s4 + h) ^ (row & 15)) << 4));
                    bfr[st][s4][j].q[1] = *reinterpret_cast<const u32x4*>(base + (((8 + 2 * s4 + h) ^ (row & 15)) << 4));
                }
    }

    // ---- one weight tile: NSTG x 4 sparse matrix instructions per (row tile, token tile)
#define BIMASK_WTILE(set, at)                                                                    \
    {                                                                                            \
        f32x16 acc[TM][TN];                                                                      \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                       \
                _Pragma("unroll") for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;               \
        _Pragma("unroll") for (int st = 0; st < NSTG; ++st) {                                    \
            _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {                                   \
                BFragR bf[TN];                                                                   \
                _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                 \
                    if constexpr (REGB) {                                                        \
                        bf[j] = bfr[st][s4][j];                                                  \
                    } else {                                                                     \
                        const int row = j * 32 + l32;                                            \
                        const uint8_t* base = sB + st * (BN * 256) + row * 256;                  \
                        bf[j].q[0] = *reinterpret_cast<const u32x4*>(base + (((2 * s4 + h) ^ (row & 15)) << 4));     \
                        bf[j].q[1] = *reinterpret_cast<const u32x4*>(base + (((8 + 2 * s4 + h) ^ (row & 15)) << 4)); \
                    }                                                                            \
                }                                                                                \
                _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                 \
                    AFragR af;                                                                   \
                    af.q = ra[set][st][i][s4];                                                   \
                    const int idx = static_cast<int>(s4 < 2 ? rmeta[set][st][i].x : rmeta[set][st][i].y); \
                    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                             \
                        if (s4 & 1)                                                              \
                            acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf[j].v, acc[i][j], idx, 0, 1); \
                        else                                                                     \
                            acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf[j].v, acc[i][j], idx, 0, 0); \
                    }                                                                            \
                }                                                                                \
            }                                                                                    \
        }                                                                                        \
        /* Output.  A lane holds 4 consecutive weight rows of one token per accumulator quad;   \
           swapping quads between the two lane halves gives every lane 8 consecutive bf16       \
           (16 bytes) of its token row.  The tile is staged through LDS (double-buffered, one   \
           barrier per weight tile) so that it leaves as whole 512-byte row segments with        \
           streaming stores: full-line writes go straight to memory instead of piling up as      \
           dirty lines in L2 that the end of the kernel has to wait for. */                      \
        uint8_t* stg = sB + S::kB + S::kInv + ((at) & 1) * S::kOut;                              \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                     \
                const int t = j * 32 + l32;                                                      \
                _Pragma("unroll") for (int p = 0; p < 2; ++p) {                                  \
                    const uint32_t xlo = pack_bf16(acc[i][j][8 * p + 0], acc[i][j][8 * p + 1]);  \
                    const uint32_t xhi = pack_bf16(acc[i][j][8 * p + 2], acc[i][j][8 * p + 3]);  \
                    const uint32_t ylo = pack_bf16(acc[i][j][8 * p + 4], acc[i][j][8 * p + 5]);  \
                    const uint32_t yhi = pack_bf16(acc[i][j][8 * p + 6], acc[i][j][8 * p + 7]);  \
                    const auto slo = __builtin_amdgcn_permlane32_swap(xlo, ylo, false, false);   \
                    const auto shi = __builtin_amdgcn_permlane32_swap(xhi, yhi, false, false);   \
                    const u32x4 v = {slo[0], shi[0], slo[1], shi[1]};                            \
                    const int u = (wm * WM + i * 32 + 16 * p + 8 * h) >> 3;   /* 16-byte unit of the row */ \
                    *reinterpret_cast<u32x4*>(stg + t * (BM * 2) + ((u ^ ((2 * t) & (BM / 8 - 1))) << 4)) = v; \
                }                                                                                \
            }                                                                                    \
        __syncthreads();                                                                         \
        constexpr int UPR = BM / 8;                          /* 16-byte units per tile row */    \
        _Pragma("unroll") for (int it = 0; it < BN * UPR / NT; ++it) {                           \
            const int q = tid + NT * it, t = q / UPR, u = q % UPR;                               \
            const u32x4 v = *reinterpret_cast<const u32x4*>(stg + t * (BM * 2) + ((u ^ ((2 * t) & (BM / 8 - 1))) << 4)); \
            const int64_t a = static_cast<int64_t>(at) * BM + 8 * u;                             \
            if (t < rows && a < Adim) {                                                          \
                uint16_t* dst = C + (t0 + t) * ldc + a;                                          \
                if (vecC && a + 8 <= Adim) {                                                     \
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));               \
                } else if (a + 8 <= Adim) {      /* rows not 16-byte aligned: 4-byte stores */   \
                    uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);                            \
                    d32[0] = v.x; d32[1] = v.y; d32[2] = v.z; d32[3] = v.w;                      \
                } else {                                                                         \
                    _Pragma("unroll") for (int e = 0; e < 8; ++e)                                \
                        if (a + e < Adim) dst[e] = static_cast<uint16_t>(v[e >> 1] >> (16 * (e & 1))); \
                }                                                                                \
            }                                                                                    \
        }                                                                                        \
    }

    int at = at_begin;
#pragma unroll 1
    for (; at + 2 <= tiles_a; at += 2) {
        BIMASK_LOAD_WTILE(1, at + 1)
        BIMASK_WTILE(0, at)
        { const int nx = at + 2 < tiles_a ? at + 2 : tiles_a - 1; BIMASK_LOAD_WTILE(0, nx) }
        BIMASK_WTILE(1, at + 1)
    }
    if (at < tiles_a) BIMASK_WTILE(0, at)
    if constexpr (!PERSIST) break;
    if (tile_next >= ntiles) break;
    tile = tile_next; t0 = t0_next; rows = rows_next;
    if (tiles_a - at_begin > 1) BIMASK_LOAD_WTILE(0, at_begin)   // several weight tiles: set 0 starts over
    }
#undef BIMASK_WTILE
#undef BIMASK_LOAD_WTILE
#undef BIMASK_LOAD_ROWS
}

constexpr unsigned kPersistGrid = 768;     // persistent variant: three workgroups per CU

template <int BM, int BN, int WAVES_M, int NSTG, bool PERSIST = false>
int run_resident(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc, int64_t ldb,
                 const int32_t* perm, int64_t T, void* C, int64_t ldc, int rpt, hipStream_t s) {
    using S = ResSmem<BM, BN, NSTG, PERSIST>;
    auto kern = k_gemm_sp24_resident<BM, BN, WAVES_M, NSTG, PERSIST>;
    if (S::kTotal > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                S::kTotal) != hipSuccess) return BIMASK_ERR_HIP;
    }
    const bool vecB = aligned16(Bsrc) && (ldb * 2) % 16 == 0;
    const bool vecC = aligned16(C) && (ldc * 2) % 16 == 0;
    unsigned grid = static_cast<unsigned>(ceil_div(T, rpt));
    if (PERSIST) {
        unsigned cap = kPersistGrid;
        if (BM > 128) {                              // large tiles: as many workgroups as stay resident
            static DeviceMemo memo;                  // per instantiation (kernel and LDS size are fixed) and device
            const int dev = DeviceMemo::device();
            int occ = static_cast<int>(memo.get(dev));
            if (occ < 1) {
                if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, reinterpret_cast<const void*>(kern), 64 * WAVES_M,
                                                                 static_cast<size_t>(S::kTotal)) != hipSuccess || occ < 1)
                    return BIMASK_ERR_HIP;
                memo.set(dev, static_cast<uint64_t>(occ));
            }
            cap = 256u * static_cast<unsigned>(occ);
        }
        if (grid > cap) grid = cap;
    }
    // few token tiles: split the weight tiles over blockIdx.y, as far as one round of 256
    // workgroups goes (the kernel runs one workgroup per CU; a second round costs a full pass)
    const int64_t tiles_all = ceil_div(Adim, BM);
    int64_t groups = 256 / grid;
    if (groups < 1) groups = 1;
    if (groups > tiles_all) groups = tiles_all;
    hipLaunchKernelGGL(kern, dim3(grid, static_cast<unsigned>(groups)), dim3(64 * WAVES_M), S::kTotal, s,
                       static_cast<const uint16_t*>(A), meta,
                       Adim, K, static_cast<const uint16_t*>(Bsrc), ldb, perm, T, static_cast<uint16_t*>(C), ldc,
                       rpt, vecB, vecC);
    return check_launch();
}

}  // namespace

// Rows per token tile: as close to BN as possible while the grid is a whole number of
// waves of `cus` workgroups (every CU gets the same share of the output).
static int pick_rows_per_tile(int64_t T, int bn, int cus) {
    const int64_t tiles_min = ceil_div(T, bn);
    const int64_t tiles = ceil_div(tiles_min, cus) * cus;
    int64_t rpt = ceil_div(T, tiles);
    if (rpt < 32) rpt = T < 32 ? T : 32;                // do not starve the 32-wide matrix tiles
    if (rpt > bn) rpt = bn;
    return static_cast<int>(rpt);
}

// Short-contraction 2:4 GEMM with the token tile resident in LDS and an optional fused
// column gather.  Returns BIMASK_ERR_UNSUPPORTED when K is too long for this kernel.
int launch_gemm_sp24_resident(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc,
                              int64_t ldb, const int32_t* perm, int64_t T, void* C, int64_t ldc,
                              hipStream_t s) {
    if (K > 512) return BIMASK_ERR_UNSUPPORTED;
    if (!aligned16(A) || !aligned16(meta)) return BIMASK_ERR_ALIGN;
    {   // narrow weights: one wavefront per token tile, weights in registers
        const int rc = launch_gemm_sp24_narrow(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, s);
        if (rc != BIMASK_ERR_UNSUPPORTED) return rc;
    }
    if (perm && K > 128 && ceil_div(T, 32) >= 512) {
        // Eq. (10)'s gather with many tokens: whole rows of g(Y) in LDS, 16-32 rows per workgroup (512 x 128
        // backward at 50176 tokens 41 -> 29 us, 384 x 384 at 25216 tokens 22 -> 20 us; fewer tokens: 512 x 512
        // at 12544 was 15 -> 16.5 us, hence the bound); takes aligned operands only, else the kernels below
        const int rc = launch_gemm_sp24_rowres(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, s);
        if (rc != BIMASK_ERR_UNSUPPORTED) return rc;
    }
    const int nstg = static_cast<int>(ceil_div(K, 128));
    if (Adim <= 128 && nstg <= 2) {
        // one narrow weight tile: the workgroup is a latency chain (fill, multiply, store), so
        // small token tiles on 4 wavefronts with few registers let three of them share a CU
        const int rpt = pick_rows_per_tile(T, 32, 256);
        if (nstg == 1) return run_resident<128, 32, 4, 1, true>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, rpt, s);
        return run_resident<128, 32, 4, 2, true>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, rpt, s);
    }
    // few tokens: full 64-row tiles (the weight tiles are split over workgroups instead)
    const int rpt = ceil_div(T, 64) <= 128 ? 64 : pick_rows_per_tile(T, 64, 256);
#define BIMASK_RES(WAVES) \
    switch (nstg) { \
        case 1: return run_resident<256, 64, WAVES, 1>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, rpt, s); \
        case 2: return run_resident<256, 64, WAVES, 2>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, rpt, s); \
        case 3: return run_resident<256, 64, WAVES, 3>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, rpt, s); \
        default: return run_resident<256, 64, WAVES, 4>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, rpt, s); \
    }
    if (ceil_div(T, 64) >= 1024) {
        // many token tiles per CU: persistent workgroups fetch the next tile's rows during the current one
        switch (nstg) {
            case 1: return run_resident<256, 64, 8, 1, true>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, 64, s);
            case 2: return run_resident<256, 64, 8, 2, true>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, 64, s);
            default: break;
        }
    }
    BIMASK_RES(8)
#undef BIMASK_RES
}

}  // namespace bimask
