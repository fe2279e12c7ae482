// 2:4-sparse bf16 GEMM for narrow weights and short contractions, wavefront-private variant:
//     C[t][a] = sum_k Bsrc[t][perm[k]] * A[a][k],   a < Adim <= 256,  k < K <= 512
// (Eq. (3) / Eq. (10) of arXiv 2302.06058 for layers with few features on both sides of the
// weight matrix: the first convolutions of a ResNet, whose token count is in the hundreds of
// thousands.)  Such a layer is a pure stream: ~300 bytes in and ~130 bytes out per token and
// a handful of matrix instructions, so what matters is the instruction count per token.
//
// One wavefront owns one tile of 32 tokens at a time and shares nothing with other
// wavefronts: the compressed weights of ALL weight rows live in its registers for the whole
// kernel, the token rows travel global -> registers -> LDS as whole 16-byte pieces (requested
// one tile ahead), every token fragment is read from LDS exactly once, and the 32 x Adim
// output tile is regrouped through the same LDS area into whole rows that leave with
// streaming stores.  No workgroup barrier anywhere; LDS rows sit at a pitch whose dword
// stride is 2 x odd, which makes the 8-byte accesses of 32 lanes (one per token) hit 64
// distinct banks.  Rows whose byte length is no multiple of 16 (K or Adim = 8 m + 4) must be
// contiguous in memory; a 32-token tile is then one 16-byte-aligned block.
#include "common.hpp"

namespace bimask {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

union BFragN { bf16x16 v; u32x4 q[2]; };
union AFragN { bf16x8 v; u32x4 q; };

__device__ __forceinline__ void wave_lds_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

// LDS pitch of a row of `w` bf16: the row itself, plus 8 bytes when that is a multiple of 16
__host__ __device__ inline int narrow_pitch(int w) { return (w & 7) ? 2 * w : 2 * w + 8; }

// registers: TM * NSTG * 18 for the weights, TM * 16 accumulators, NSTG * 32 for the rows in flight;
// two wavefronts per SIMD (256 registers each) except for the longest contractions
constexpr int narrow_waves_per_simd(int tm, int nstg) { return nstg >= 4 || (nstg == 3 && tm >= 2) ? 1 : 2; }

template <int TM, int NSTG>
__global__ void __launch_bounds__(64, narrow_waves_per_simd(TM, NSTG))
k_gemm_sp24_narrow(const uint16_t* __restrict__ A_all, const uint32_t* __restrict__ Ameta_all, int Adim_all, int K,
                   const uint16_t* __restrict__ Bsrc, int ldb, const int32_t* __restrict__ perm, int64_t T,
                   uint16_t* __restrict__ C_all, int ldc, int nsplit, bool stream_out) {
    // Weight rows beyond TM * 32 are split over `nsplit` wavefronts that work on the same token
    // tile; workgroups 8 apart run on the same XCD, so the tile is fetched from memory once.
    const int split = (static_cast<int>(blockIdx.x) >> 3) % nsplit;
    const int64_t wave_id = ((static_cast<int64_t>(blockIdx.x) >> 3) / nsplit) * 8 + (blockIdx.x & 7);
    const int64_t nwaves = gridDim.x / nsplit;
    // row tiles of this split; the last split may own fewer than TM (7 row tiles over 2 x 4): its
    // surplus tiles re-read the operand's last row tile (loaded, never stored)
    const int rt_last = (Adim_all + 31) / 32 - 1;
    uint16_t* __restrict__ C = C_all + split * TM * 32;
    const int Adim = Adim_all - split * TM * 32 < TM * 32 ? Adim_all - split * TM * 32 : TM * 32;
    // q / G == (q * invG) >> 22 for q < 64, G <= 64
    const int invG_arg = (K & 7) ? 0 : ((1 << 22) + (K >> 3) - 1) / (K >> 3);
    const int invU_arg = (Adim & 7) ? 0 : ((1 << 22) + (Adim >> 3) - 1) / (Adim >> 3);
    const int dtB = (K & 7) ? 0 : 64 / (K >> 3), dgB = (K & 7) ? 0 : 64 % (K >> 3);
    const int dtC = (Adim & 7) ? 0 : 64 / (Adim >> 3), dgC = (Adim & 7) ? 0 : 64 % (Adim >> 3);
    extern __shared__ u32x4 smem_u4[];
    uint8_t* smem = reinterpret_cast<uint8_t*>(smem_u4);
    int32_t* sInv = reinterpret_cast<int32_t*>(smem);        // byte offset of column c inside a permuted row
    uint8_t* area = smem + NSTG * 512;                       // token rows, later the output rows

    // Everything below that depends only on the lane or on the shape is the same for every tile.
    // The values are re-derived per tile from copies the optimiser cannot see through: hoisted
    // out of the tile loop they would occupy a few hundred registers for the whole kernel.
#define BIMASK_NARROW_SHAPE(LANE_SRC, K_SRC, A_SRC)                                              \
    int lane = (LANE_SRC), Kq = (K_SRC), Aq = (A_SRC);                                           \
    asm volatile("" : "+v"(lane));                                                               \
    asm volatile("" : "+s"(Kq));                                                                 \
    asm volatile("" : "+s"(Aq));                                                                 \
    const int l32 = lane & 31, h = lane >> 5;                                                    \
    const bool packB = (Kq & 7) != 0, packC = (Aq & 7) != 0;                                     \
    const int pitchB = narrow_pitch(Kq), pitchC = narrow_pitch(Aq);                              \
    const int G = Kq >> 3, UPR = Aq >> 3;            /* 16-byte pieces per row (aligned rows) */ \
    /* 16-byte piece q = lane + 64 it of a tile is piece g of row t with q = t G + g; the walk from \
       one `it` to the next adds 64 = dt G + dg and carries when g passes G (no divisions) */    \
    const int tB0 = static_cast<int>(static_cast<uint32_t>(lane * invG_arg) >> 22), gB0 = lane - tB0 * G; \
    const int tC0 = static_cast<int>(static_cast<uint32_t>(lane * invU_arg) >> 22), gC0 = lane - tC0 * UPR; \
    const bool Kfull = Kq == NSTG * 128;                                                         \
    const bool Afull = Aq == TM * 32;                                                            \
    (void)l32; (void)h; (void)packC; (void)pitchC; (void)UPR; (void)Kfull; (void)Afull; (void)pitchB; (void)G; (void)packB; (void)tB0; (void)gB0; (void)tC0; (void)gC0;
    const int lane0 = threadIdx.x;
    constexpr int NLD = NSTG * 8;                            // 16-byte pieces of 32 token rows per lane, at most
    constexpr int NOUT = TM * 2;                             // the same for the output rows

    const int64_t ntiles = ceil_div(T, 32);
    int64_t tile = wave_id;
    if (tile >= ntiles) return;

    // ---- all weight fragments: NSTG stages x TM row tiles x 4 sub-steps, for the whole kernel
    u32x4 ra[NSTG][TM][4];
    u32x2 rmeta[NSTG][TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rt = split * TM + i < rt_last ? split * TM + i : rt_last;
        const uint16_t* pa = A_all + (static_cast<int64_t>(rt) * NSTG * 256 + lane0) * 8;
        const uint32_t* pm = Ameta_all + (static_cast<int64_t>(rt) * NSTG * 64 + lane0) * 2;
#pragma unroll
        for (int st = 0; st < NSTG; ++st) {
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
                ra[st][i][s4] = *reinterpret_cast<const u32x4*>(pa + (st * 4 + s4) * 512);
            rmeta[st][i] = *reinterpret_cast<const u32x2*>(pm + st * 128);
        }
    }

    // ---- token rows of one tile -> registers
    u32x4 v[NLD];
#define BIMASK_NARROW_LOAD(TILE)                                                                 \
    {                                                                                            \
        const int64_t t0_ = (TILE) * 32;                                                         \
        const int rows_ = static_cast<int>((T - t0_) < 32 ? (T - t0_) : 32);                     \
        if (packB) {                                                                             \
            const int nbytes = rows_ * Kq * 2;                                                    \
            const uint16_t* blk = Bsrc + t0_ * Kq;                                                \
            _Pragma("unroll") for (int it = 0; it < NLD; ++it) {                                 \
                const int q = lane + 64 * it;                                                    \
                v[it] = (u32x4){0u, 0u, 0u, 0u};                                                 \
                if (it * 1024 < nbytes) {                                                        \
                    if (q * 16 + 16 <= nbytes) v[it] = reinterpret_cast<const u32x4*>(blk)[q];   \
                    else if (q * 16 < nbytes) {      /* odd row count: the block ends in 8 bytes */ \
                        const u32x2 t2 = *reinterpret_cast<const u32x2*>(blk + q * 8);           \
                        v[it].x = t2.x; v[it].y = t2.y;                                          \
                    }                                                                            \
                }                                                                                \
            }                                                                                    \
        } else {                                                                                 \
            const uint16_t* base = Bsrc + t0_ * ldb;                                             \
            const int step = dtB * ldb + 8 * dgB, carry = ldb - 8 * G, end = rows_ * ldb;        \
            int g = gB0, ofs = tB0 * ldb + 8 * gB0;          /* element offset of the piece */   \
            _Pragma("unroll") for (int it = 0; it < NLD; ++it) {                                 \
                v[it] = (u32x4){0u, 0u, 0u, 0u};                                                 \
                if (it * 64 < 32 * G) {                                                          \
                    if (ofs < end) v[it] = *reinterpret_cast<const u32x4*>(base + ofs);          \
                    g += dgB; ofs += step;                                                       \
                    if (g >= G) { g -= G; ofs += carry; }                                        \
                }                                                                                \
            }                                                                                    \
        }                                                                                        \
    }
    {
        BIMASK_NARROW_SHAPE(lane0, K, Adim)
        BIMASK_NARROW_LOAD(tile)
    }

    if (perm) {             // Eq. (10) reads column P[k] at position k: column c = P[k] is stored at 2 k
        for (int r = lane0; r < K; r += 64) sInv[perm[r]] = 2 * r;
    }

    for (;;) {
        BIMASK_NARROW_SHAPE(lane0, K, Adim)
        const int64_t t0 = tile * 32;
        const int rows = static_cast<int>((T - t0) < 32 ? (T - t0) : 32);
        wave_lds_fence();                                    // the previous tile's output rows have been read
        // ---- registers -> LDS rows (rows beyond `rows` are zeros)
        if (packB) {
#pragma unroll
            for (int it = 0; it < NLD; ++it) {
                const int q = lane + 64 * it;
                if (it * 1024 < 32 * pitchB && q * 16 < 32 * pitchB) *reinterpret_cast<u32x4*>(area + q * 16) = v[it];
            }
        } else if (perm) {
            // the column gather of Eq. (10), done as a scatter on the way into LDS: 2-byte stores
            const int step = dtB * pitchB, end = 32 * pitchB;
            int g = gB0, rofs = tB0 * pitchB;                // byte offset of the piece's row
#pragma unroll
            for (int it = 0; it < NLD; ++it) {
                if (it * 64 < 32 * G) {
                    if (rofs < end) {
                        const u32x4 i0 = *reinterpret_cast<const u32x4*>(sInv + 8 * g);
                        const u32x4 i1 = *reinterpret_cast<const u32x4*>(sInv + 8 * g + 4);
                        uint8_t* row = area + rofs;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const uint32_t off = e < 4 ? i0[e] : i1[e - 4];
                            *reinterpret_cast<uint16_t*>(row + off) = static_cast<uint16_t>(v[it][e >> 1] >> (16 * (e & 1)));
                        }
                    }
                    g += dgB; rofs += step;
                    if (g >= G) { g -= G; rofs += pitchB; }
                }
            }
        } else {
            const int step = dtB * pitchB + 16 * dgB, carry = pitchB - 16 * G, end = 32 * pitchB;
            int g = gB0, ofs = tB0 * pitchB + 16 * gB0;      // byte offset of the piece in LDS
#pragma unroll
            for (int it = 0; it < NLD; ++it) {
                if (it * 64 < 32 * G) {
                    if (ofs < end) {
                        u32x2* d = reinterpret_cast<u32x2*>(area + ofs);
                        d[0] = (u32x2){v[it].x, v[it].y};
                        d[1] = (u32x2){v[it].z, v[it].w};
                    }
                    g += dgB; ofs += step;
                    if (g >= G) { g -= G; ofs += carry; }
                }
            }
        }
        wave_lds_fence();
        const int64_t next = tile + nwaves;
        if (next < ntiles) BIMASK_NARROW_LOAD(next)          // in flight during this tile's arithmetic

        // ---- NSTG x 4 sparse matrix instructions per weight-row tile
        f32x16 acc[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][q] = 0.f;
        const uint8_t* myrow = area + l32 * pitchB;
#pragma unroll
        for (int st = 0; st < NSTG; ++st) {
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                BFragN bf;
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    const int k0 = 8 * (st * 16 + 8 * x + 2 * s4 + h);      // this lane's 8 contraction indices
                    const u32x2* p = reinterpret_cast<const u32x2*>(myrow + 2 * k0);
                    const u32x2 lo = p[0], hi = p[1];
                    u32x4 o = {lo.x, lo.y, hi.x, hi.y};
                    if (!Kfull) {                            // beyond K: whatever LDS holds there
#pragma unroll
                        for (int d = 0; d < 4; ++d)
                            if (k0 + 2 * d + 2 > Kq) o[d] = 0u;
                    }
                    bf.q[x] = o;
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    AFragN af;
                    af.q = ra[st][i][s4];
                    const int idx = static_cast<int>(s4 < 2 ? rmeta[st][i].x : rmeta[st][i].y);
                    if (s4 & 1)
                        acc[i] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf.v, acc[i], idx, 0, 1);
                    else
                        acc[i] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf.v, acc[i], idx, 0, 0);
                }
            }
        }

        // ---- output.  A lane holds 4 consecutive weight rows of its token per accumulator quad;
        // swapping quads between the lane halves gives it 8 consecutive bf16 (16 bytes) of the
        // token's output row, which go to LDS at the output pitch.
        wave_lds_fence();                                    // all fragment reads precede the overwrite
        uint8_t* orow = area + l32 * pitchC;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const uint32_t xlo = pack_bf16(acc[i][8 * p + 0], acc[i][8 * p + 1]);
                const uint32_t xhi = pack_bf16(acc[i][8 * p + 2], acc[i][8 * p + 3]);
                const uint32_t ylo = pack_bf16(acc[i][8 * p + 4], acc[i][8 * p + 5]);
                const uint32_t yhi = pack_bf16(acc[i][8 * p + 6], acc[i][8 * p + 7]);
                const auto slo = __builtin_amdgcn_permlane32_swap(xlo, ylo, false, false);
                const auto shi = __builtin_amdgcn_permlane32_swap(xhi, yhi, false, false);
                const int a0 = i * 32 + 16 * p + 8 * h;      // first of this lane's 8 weight rows
                if (Afull || a0 + 8 <= Aq) {
                    u32x2* d = reinterpret_cast<u32x2*>(orow + 2 * a0);
                    d[0] = (u32x2){slo[0], shi[0]};
                    d[1] = (u32x2){slo[1], shi[1]};
                } else {
                    uint32_t* d = reinterpret_cast<uint32_t*>(orow + 2 * a0);
                    if (a0 + 2 <= Aq) d[0] = slo[0];
                    if (a0 + 4 <= Aq) d[1] = shi[0];
                    if (a0 + 6 <= Aq) d[2] = slo[1];
                }
            }
        wave_lds_fence();
        if (packC) {                                         // the tile is one aligned block of the output
            const int nbytes = rows * Aq * 2;
            uint16_t* blk = C + t0 * Aq;
#pragma unroll
            for (int it = 0; it < NOUT; ++it) {
                const int q = lane + 64 * it;
                if (it * 1024 < nbytes) {
                    if (q * 16 + 16 <= nbytes) {
                        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(area + q * 16), reinterpret_cast<u32x4*>(blk) + q);
                    } else if (q * 16 < nbytes) {            // odd row count: the block ends in 8 bytes
                        *reinterpret_cast<u32x2*>(blk + q * 8) = *reinterpret_cast<const u32x2*>(area + q * 16);
                    }
                }
            }
        } else {
            uint16_t* base = C + t0 * ldc;
            const int lstep = dtC * pitchC + 16 * dgC, lcarry = pitchC - 16 * UPR;
            const int gstep = dtC * ldc + 8 * dgC, gcarry = ldc - 8 * UPR, end = rows * ldc;
            int u = gC0, lofs = tC0 * pitchC + 16 * gC0, gofs = tC0 * ldc + 8 * gC0;
#pragma unroll
            for (int it = 0; it < NOUT; ++it) {
                if (it * 64 < 32 * UPR) {
                    if (gofs < end) {
                        const u32x2* p = reinterpret_cast<const u32x2*>(area + lofs);
                        const u32x2 lo = p[0], hi = p[1];
                        const u32x4 o = {lo.x, lo.y, hi.x, hi.y};
                        u32x4* dst = reinterpret_cast<u32x4*>(base + gofs);
                        if (stream_out) __builtin_nontemporal_store(o, dst);
                        else *dst = o;
                    }
                    u += dgC; lofs += lstep; gofs += gstep;
                    if (u >= UPR) { u -= UPR; lofs += lcarry; gofs += gcarry; }
                }
            }
        }
        if (next >= ntiles) break;
        tile = next;
    }
#undef BIMASK_NARROW_LOAD
#undef BIMASK_NARROW_SHAPE
}

template <int TM, int NSTG>
int run_narrow(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc, int64_t ldb,
               const int32_t* perm, int64_t T, void* C, int64_t ldc, hipStream_t s) {
    auto kern = k_gemm_sp24_narrow<TM, NSTG>;
    const int in_bytes = 32 * narrow_pitch(static_cast<int>(K)) + NSTG * 256;   // fragment reads may run past row 31
    const int out_bytes = 32 * narrow_pitch(static_cast<int>(Adim < TM * 32 ? Adim : TM * 32)) + 16;
    const int lds = NSTG * 512 + (((in_bytes > out_bytes ? in_bytes : out_bytes) + 15) & ~15);
    if (lds > 48 * 1024) return BIMASK_ERR_UNSUPPORTED;
    // wavefronts per CU by LDS and registers; the grid is a multiple of the CU count in which every
    // wavefront gets the same number of tiles (+-1)
    // (the answer depends on the kernel, the LDS size and the device: remembered per instantiation and device,
    // LDS size and answer in one word)
    static DeviceMemo memo;
    const int dev = DeviceMemo::device();
    const uint64_t known = memo.get(dev);
    int wpc = (known >> 32) == static_cast<uint64_t>(lds) ? static_cast<int>(known & 0xFFFFFFFFu) : 0;
    if (wpc < 1) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&wpc, reinterpret_cast<const void*>(kern), 64, static_cast<size_t>(lds)) != hipSuccess || wpc < 1)
            return BIMASK_ERR_HIP;
        memo.set(dev, (static_cast<uint64_t>(lds) << 32) | static_cast<uint32_t>(wpc));
    }
    if (wpc > 16) wpc = 16;
    const int nsplit = static_cast<int>(ceil_div(Adim, TM * 32));
    const int64_t ntiles = ceil_div(T, 32);
    const int64_t slots = 256 * wpc / nsplit;                                   // token tiles in flight on the chip
    const int64_t rounds = ceil_div(ntiles, slots);
    int64_t nwaves = ceil_div(ceil_div(ntiles, rounds), 256) * 256;
    if (nwaves > round_up(ntiles, 8)) nwaves = round_up(ntiles, 8);
    const unsigned grid = static_cast<unsigned>(nwaves * nsplit);
    // whole rows leave as full 128-byte lines when the output is contiguous or its row pieces are whole lines
    const bool stream_out = nsplit == 1
        ? (ldc == Adim || (Adim % 64 == 0 && ldc % 64 == 0 && (reinterpret_cast<uintptr_t>(C) & 127u) == 0))
        : ((TM * 32) % 64 == 0 && Adim % 64 == 0 && ldc % 64 == 0 && (reinterpret_cast<uintptr_t>(C) & 127u) == 0);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64), static_cast<size_t>(lds), s, static_cast<const uint16_t*>(A), meta,
                       static_cast<int>(Adim), static_cast<int>(K), static_cast<const uint16_t*>(Bsrc),
                       static_cast<int>(ldb), perm, T, static_cast<uint16_t*>(C), static_cast<int>(ldc), nsplit, stream_out);
    return check_launch();
}

}  // namespace

// Returns BIMASK_ERR_UNSUPPORTED when the shape, the alignment or the leading dimensions are
// outside what this kernel handles (the caller then takes the workgroup-tiled kernels).
int launch_gemm_sp24_narrow(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc,
                            int64_t ldb, const int32_t* perm, int64_t T, void* C, int64_t ldc, hipStream_t s) {
    if (T < 1 || K < 4 || Adim < 4 || K % 4 != 0 || Adim % 4 != 0) return BIMASK_ERR_UNSUPPORTED;
    if (!aligned16(A) || !aligned16(meta) || !aligned16(Bsrc) || !aligned16(C)) return BIMASK_ERR_UNSUPPORTED;
    if (ldb >= (1 << 20) || ldc >= (1 << 20)) return BIMASK_ERR_UNSUPPORTED;    // 32-bit offsets inside a tile
    if (K % 8 != 0 ? (ldb != K || perm) : ldb % 8 != 0) return BIMASK_ERR_UNSUPPORTED;
    if (Adim % 8 != 0 ? ldc != Adim : ldc % 8 != 0) return BIMASK_ERR_UNSUPPORTED;
    const int nstg = static_cast<int>(ceil_div(K, 128)), tm = static_cast<int>(ceil_div(Adim, 32));
#define BIMASK_NARROW(TM_, NSTG_) return run_narrow<TM_, NSTG_>(A, meta, Adim, K, Bsrc, ldb, perm, T, C, ldc, s);
    if (nstg == 1) {
        switch (tm) {
            case 1: BIMASK_NARROW(1, 1)
            case 2: BIMASK_NARROW(2, 1)
            case 3: BIMASK_NARROW(3, 1)
            case 4: BIMASK_NARROW(4, 1)
            case 5: BIMASK_NARROW(5, 1)
            default: break;
        }
        // up to 256 weight rows: two wavefronts per token tile, each with half of the rows (the
        // token rows are short, so fetching them twice from L2 is cheap next to the output)
        if (Adim % 8 == 0) {
            if (tm == 6) BIMASK_NARROW(3, 1)
            if (tm == 7 || tm == 8) BIMASK_NARROW(4, 1)
        }
    } else if (tm <= 2) {
        // longer contractions: at most 64 weight rows, all their fragments in registers.  (Splitting
        // more rows over sibling wavefronts does not pay here: every sibling re-reads the long rows.)
        switch (nstg) {
            case 2: if (tm == 1) BIMASK_NARROW(1, 2) else BIMASK_NARROW(2, 2)
            case 3: if (tm == 1) BIMASK_NARROW(1, 3) else BIMASK_NARROW(2, 3)
            case 4: if (tm == 1) BIMASK_NARROW(1, 4) else BIMASK_NARROW(2, 4)
            default: break;
        }
    }
#undef BIMASK_NARROW
    return BIMASK_ERR_UNSUPPORTED;
}

}  // namespace bimask
