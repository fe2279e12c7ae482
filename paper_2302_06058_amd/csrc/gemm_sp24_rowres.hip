// 2:4-sparse bf16 backward GEMM with the column gather of Eq. (10) fused, for out-feature
// counts too long for the resident-token kernel (512 < I <= 2048; with many tokens also
// 128 < I <= 512, where it is the faster of the two) and few in-features:
//     dX[t][j] = sum_r dY[t][P[r]] * Wb[j][r],   j < J <= 512,  r < I
// (arXiv 2302.06058, Eq. (10); the shapes are the 1x1 "expand" convolutions of a ResNet
// bottleneck, I = 4 J, and the wide linear layers of a transformer block seen from behind.)
//
// Without this kernel g(Y)[:, P] is materialised by a separate pass (read + write of T x I
// elements) and read a third time by the GEMM.  Here a workgroup keeps up to 32 WHOLE rows of
// g(Y) in LDS: they arrive as contiguous 16-byte pieces and are scattered to their permuted
// positions with 2-byte LDS stores (the inverse permutation sits in LDS), so the gather costs
// no memory traffic at all.  The four wavefronts then walk over the weight-row tiles (64
// rows per pass, at most two passes each), streaming the fragment-major compressed weights
// from L2 two stages ahead and reading every token fragment with two 8-byte LDS loads
// (row pitch = 2 I + 8 bytes: 32 lanes hit 64 distinct banks).  The output tile is regrouped
// through the same LDS area and leaves as whole rows.
#include "common.hpp"

namespace bimask {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

union BFragW { bf16x16 v; u32x4 q[2]; };
union AFragW { bf16x8 v; u32x4 q; };

constexpr int kRowResThreads = 256;

// TM weight-row tiles (32 rows each) per wavefront pass, NP passes per wavefront: 4 wavefronts cover
// 4 * NP * TM * 32 weight rows (256 / 384 / 512 for <2,1> / <3,1> / <2,2>)
// DENSE: the weight operand is the dense masked matrix of a ratio with N > 2 (fragment-major): two 16-byte
// fragments per sub-step and two dense 32x32x16 instructions instead of one sparse 32x32x32; one stage ahead.
template <int TM, int NP, bool DENSE>
__global__ void __launch_bounds__(kRowResThreads, 2)
k_gemm_sp24_rowres(const uint16_t* __restrict__ A, const uint32_t* __restrict__ Ameta, int Adim, int K,
                   const uint16_t* __restrict__ Bsrc, int64_t ldb, const int32_t* __restrict__ perm, int64_t T,
                   uint16_t* __restrict__ C, int64_t ldc, int rpt, bool stream_out) {
    constexpr int PF = DENSE ? 1 : 2, NBUF = PF + 1;     // weight stages in flight beyond the current one
    constexpr int NA = DENSE ? 8 : 4;                    // 16-byte weight fragments per row tile and stage
    extern __shared__ u32x4 smem_u4[];
    uint8_t* smem = reinterpret_cast<uint8_t*>(smem_u4);
    uint16_t* sInv = reinterpret_cast<uint16_t*>(smem);                  // position of column c in a permuted row
    uint8_t* rowsA = smem + ((2 * K + 15) & ~15);                        // rpt rows, later the output rows
    const int pitch = 2 * K + 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * rpt;
    const int rows = static_cast<int>((T - t0) < rpt ? (T - t0) : rpt);
    const int nks = (K + 127) >> 7;                                      // stages of the padded weight operand
    const bool Kfull = (K & 127) == 0;

    // ---- weight fragments of this wavefront's first pass: requested before anything else, they do
    // not depend on the token rows
    const int ntr = (Adim + 31) >> 5;                                    // 32-row tiles of the weight operand
    // With few token tiles the launcher splits the weight rows over blockIdx.y: this workgroup takes the row tiles
    // [rtb, rtb + 4 NP TM) and writes the matching columns of its output rows.
    const int rtb = blockIdx.y * (4 * NP * TM);
    const uint16_t* pa[TM];
    const uint32_t* pm[TM];
    u32x4 ra[NBUF][TM][NA];
    u32x2 rmeta[NBUF][DENSE ? 1 : TM];
#define BIMASK_RR_LOAD(slot, st)                                                                 \
    {                                                                                            \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            _Pragma("unroll") for (int g = 0; g < NA; ++g)                                       \
                ra[slot][i][g] = *reinterpret_cast<const u32x4*>(pa[i] + ((st) * NA + g) * 512); \
            if constexpr (!DENSE) rmeta[slot][i] = *reinterpret_cast<const u32x2*>(pm[i] + (st) * 128); \
        }                                                                                        \
    }
#define BIMASK_RR_SETUP(ps)                                                                      \
    {                                                                                            \
        const int rt0_ = rtb + (wave + 4 * (ps)) * TM;                                           \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            int rt = rt0_ + i < ntr ? rt0_ + i : ntr - 1;    /* clamped: computed, never stored */ \
            pa[i] = A + (static_cast<int64_t>(rt) * nks * (DENSE ? 512 : 256) + lane) * 8;       \
            pm[i] = DENSE ? nullptr : Ameta + (static_cast<int64_t>(rt) * nks * 64 + lane) * 2;  \
        }                                                                                        \
        _Pragma("unroll") for (int s = 0; s < PF; ++s) {                                         \
            const int stl = s < nks ? s : nks - 1;                                               \
            BIMASK_RR_LOAD(s, stl)                                                               \
        }                                                                                        \
    }
    BIMASK_RR_SETUP(0)

    // ---- rows of g(Y): contiguous 16-byte pieces from memory (first batch requested before the
    // inverse permutation is built), then a 2-byte scatter into LDS: column c = P[r] goes to position r
    {
        const int G = K >> 3;                                            // pieces per row (K is a multiple of 8)
        const int total = rows * G;
        constexpr int U = 16;                                            // pieces in flight per thread
        // piece c = tid + 256 n is piece g of row t; the walk from n to n + 1 adds 256 = dt G + dg
        const int dt = kRowResThreads / G, dg = kRowResThreads % G;
        int t = tid / G, g = tid - t * G;
        for (int c0 = 0; c0 < total; c0 += kRowResThreads * U) {
            u32x4 v[U];
            int rofs[U], gg[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + tid + kRowResThreads * u;
                rofs[u] = t * pitch;
                gg[u] = g;
                v[u] = (u32x4){0u, 0u, 0u, 0u};
                if (c < total) v[u] = *reinterpret_cast<const u32x4*>(Bsrc + (t0 + t) * ldb + 8 * g);
                t += dt; g += dg;
                if (g >= G) { g -= G; t += 1; }
            }
            if (c0 == 0) {                                               // uniform
                for (int r = tid; r < K; r += kRowResThreads) sInv[perm[r]] = static_cast<uint16_t>(r);
                __syncthreads();
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + tid + kRowResThreads * u;
                if (c < total) {
                    const u32x4 iv = *reinterpret_cast<const u32x4*>(sInv + 8 * gg[u]);      // 8 positions
                    uint8_t* row = rowsA + rofs[u];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t pos = (iv[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                        *reinterpret_cast<uint16_t*>(row + 2 * pos) = static_cast<uint16_t>(v[u][e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- 3. weight-row tiles: wavefront w takes pairs w, w + 4; fragments stream from L2
    const int lrow = l32 < rows ? l32 : rows - 1;                        // lanes beyond the tile re-read its last row
    const uint8_t* myrow = rowsA + lrow * pitch;
    f32x16 acc[NP][TM];
#pragma unroll
    for (int ps = 0; ps < NP; ++ps)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[ps][i][q] = 0.f;

#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
        const int rt0 = rtb + (wave + 4 * ps) * TM;                      // first row tile of this pass
        if (rt0 >= ntr) break;                                           // wave-uniform
        if (ps > 0) BIMASK_RR_SETUP(ps)
        // one stage = 128 contraction indices: 4 x TM sparse matrix instructions; loads past the
        // last stage are clamped to it (never skipped: the number in flight is known at every wait)
#define BIMASK_RR_STEP(u, st, DO_LOAD)                                                           \
        {                                                                                        \
            if (DO_LOAD) {                                                                       \
                const int stl = (st) + PF < nks ? (st) + PF : nks - 1;                           \
                BIMASK_RR_LOAD(((u) + PF) % NBUF, stl)                                           \
            }                                                                                    \
            _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {                                   \
                BFragW bf;                                                                       \
                _Pragma("unroll") for (int x = 0; x < 2; ++x) {                                  \
                    const int k0 = 8 * ((st) * 16 + 8 * x + 2 * s4 + h);                         \
                    const u32x2* p = reinterpret_cast<const u32x2*>(myrow + 2 * k0);             \
                    const u32x2 lo = p[0], hi = p[1];                                            \
                    u32x4 o = {lo.x, lo.y, hi.x, hi.y};                                          \
                    if (!Kfull) {                                                                \
                        _Pragma("unroll") for (int d = 0; d < 4; ++d)                            \
                            if (k0 + 2 * d + 2 > K) o[d] = 0u;                                   \
                    }                                                                            \
                    bf.q[x] = o;                                                                 \
                }                                                                                \
                _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                 \
                    if constexpr (DENSE) {                                                       \
                        _Pragma("unroll") for (int x = 0; x < 2; ++x) {                          \
                            AFragW af, bh;                                                       \
                            af.q = ra[u][i][s4 * 2 + x];                                         \
                            bh.q = bf.q[x];                                                      \
                            acc[ps][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bh.v, acc[ps][i], 0, 0, 0); \
                        }                                                                        \
                    } else {                                                                     \
                        AFragW af;                                                               \
                        af.q = ra[u][i][s4];                                                     \
                        const int idx = static_cast<int>(s4 < 2 ? rmeta[u][i].x : rmeta[u][i].y); \
                        if (s4 & 1)                                                              \
                            acc[ps][i] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf.v, acc[ps][i], idx, 0, 1); \
                        else                                                                     \
                            acc[ps][i] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af.v, bf.v, acc[ps][i], idx, 0, 0); \
                    }                                                                            \
                }                                                                                \
            }                                                                                    \
        }
        int st0 = 0;
#pragma unroll 1
        for (; st0 + NBUF <= nks; st0 += NBUF) {
#pragma unroll
            for (int u = 0; u < NBUF; ++u) BIMASK_RR_STEP(u, st0 + u, true)
        }
#pragma unroll
        for (int u = 0; u < NBUF - 1; ++u) {
            if (st0 + u < nks) BIMASK_RR_STEP(u, st0 + u, false)
        }
#undef BIMASK_RR_STEP
    }
#undef BIMASK_RR_SETUP
#undef BIMASK_RR_LOAD
    __syncthreads();                                     // every wavefront is done with the rows of g(Y)

    // ---- 4. output: a lane holds 4 consecutive weight rows of its token per accumulator quad; a swap
    // between the lane halves gives it 8 consecutive bf16 of the token's output row (16 bytes, two
    // 8-byte LDS stores); the tile then leaves as whole rows
    const int a_base = rtb * 32;                                         // first weight row (= output column) of this workgroup
    const int width = Adim - a_base < 4 * NP * TM * 32 ? Adim - a_base : 4 * NP * TM * 32;
    const int pitchC = 2 * width + 8;
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
        const int rt0 = rtb + (wave + 4 * ps) * TM;
        if (rt0 >= ntr) break;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const uint32_t xlo = pack_bf16(acc[ps][i][8 * p + 0], acc[ps][i][8 * p + 1]);
                const uint32_t xhi = pack_bf16(acc[ps][i][8 * p + 2], acc[ps][i][8 * p + 3]);
                const uint32_t ylo = pack_bf16(acc[ps][i][8 * p + 4], acc[ps][i][8 * p + 5]);
                const uint32_t yhi = pack_bf16(acc[ps][i][8 * p + 6], acc[ps][i][8 * p + 7]);
                const auto slo = __builtin_amdgcn_permlane32_swap(xlo, ylo, false, false);
                const auto shi = __builtin_amdgcn_permlane32_swap(xhi, yhi, false, false);
                const int a0 = (rt0 + i) * 32 + 16 * p + 8 * h;          // first of this lane's 8 weight rows
                if (l32 < rows && a0 + 8 <= Adim) {                      // Adim is a multiple of 8
                    u32x2* d = reinterpret_cast<u32x2*>(rowsA + l32 * pitchC + 2 * (a0 - a_base));
                    d[0] = (u32x2){slo[0], shi[0]};
                    d[1] = (u32x2){slo[1], shi[1]};
                }
            }
    }
    __syncthreads();
    {
        const int UPR = width >> 3;
        const int total = rows * UPR;
        for (int c = tid; c < total; c += kRowResThreads) {
            const int t = c / UPR, u = c - t * UPR;
            const u32x2* p = reinterpret_cast<const u32x2*>(rowsA + t * pitchC + 16 * u);
            const u32x2 lo = p[0], hi = p[1];
            const u32x4 o = {lo.x, lo.y, hi.x, hi.y};
            u32x4* dst = reinterpret_cast<u32x4*>(C + (t0 + t) * ldc + a_base + 8 * u);
            if (stream_out) __builtin_nontemporal_store(o, dst);
            else *dst = o;
        }
    }
}

}  // namespace

namespace {
// what the kernel itself takes; contractions up to 512 reach it through launch_gemm_sp24_resident
bool rowres_takes(int64_t Adim, int64_t K) {
    return K > 128 && K <= 2048 && K % 8 == 0 && Adim >= 8 && Adim <= 512 && Adim % 8 == 0 && Adim <= K;
}
}  // namespace

bool gemm_sp24_rowres_shape(int64_t Adim, int64_t K) { return K > 512 && rowres_takes(Adim, K); }
bool gemm_dense_rowres_shape(int64_t Adim, int64_t K) { return rowres_takes(Adim, K); }

// Returns BIMASK_ERR_UNSUPPORTED when the shape / alignment is outside this kernel (the caller then
// gathers g(Y)[:, P] into the workspace and runs the streaming kernel).
int launch_gemm_sp24_rowres(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc,
                            int64_t ldb, const int32_t* perm, int64_t T, void* C, int64_t ldc, hipStream_t s, bool dense) {
    if (!perm || T < 1) return BIMASK_ERR_UNSUPPORTED;
    if (!rowres_takes(Adim, K)) return BIMASK_ERR_UNSUPPORTED;
    if (!aligned16(A) || !aligned16(meta) || !aligned16(Bsrc) || !aligned16(C) || ldb % 8 != 0 || ldc % 8 != 0)
        return BIMASK_ERR_UNSUPPORTED;
    // rows per token tile (<= 32): the fewest sequential tile slots per CU, then the tallest tile
    const int pitch = static_cast<int>(2 * K + 8), inv_bytes = static_cast<int>((2 * K + 15) & ~15);
    int best_rpt = 0, best_cost = 1 << 30, best_occ = 0;
    size_t best_lds = 0;
    for (int rpt = 32; rpt >= 16; --rpt) {
        const size_t lds = static_cast<size_t>(inv_bytes) + static_cast<size_t>(rpt) * pitch;
        if (lds > 160 * 1024) continue;
        const int occ = 2 * lds <= 160 * 1024 ? 2 : 1;
        const int64_t tiles = ceil_div(T, rpt);
        const int cost = static_cast<int>(ceil_div(tiles, 256 * occ)) * occ;       // tile times per CU, L1-shared
        // ties go to two workgroups per CU: one fills its rows while the other multiplies
        if (cost < best_cost || (cost == best_cost && occ > best_occ)) { best_cost = cost; best_rpt = rpt; best_lds = lds; best_occ = occ; }
    }
    if (best_rpt == 0) return BIMASK_ERR_UNSUPPORTED;
    const bool stream_out = (Adim * 2) % 128 == 0 && ldc % 64 == 0 && (reinterpret_cast<uintptr_t>(C) & 127u) == 0;
    const unsigned grid = static_cast<unsigned>(ceil_div(T, best_rpt));
    // Few token tiles (less than half the CUs busy) and more than 256 weight rows: every workgroup would stream the
    // whole weight operand through one CU for its 32 tokens.  Split the rows over blockIdx.y in pieces of 256:
    // twice (or three, four times) the workgroups, each streaming a half (third, quarter) of the weights; the token
    // rows are gathered once per piece, from L2 after the first.
    const bool split = !dense && grid <= 128 && Adim > 256;
    const unsigned nsplit = split ? static_cast<unsigned>(ceil_div(Adim, 256)) : 1u;
#define BIMASK_ROWRES(TM_, NP_, DENSE_)                                                                      \
    {                                                                                                        \
        static DeviceMemo attr_set;                                                                          \
        const int dev = DeviceMemo::device();                                                                \
        auto kern = k_gemm_sp24_rowres<TM_, NP_, DENSE_>;                                                    \
        if (!attr_set.get(dev)) {                                                                            \
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    160 * 1024) != hipSuccess) return BIMASK_ERR_HIP;                        \
            attr_set.set(dev, 1);                                                                            \
        }                                                                                                    \
        hipLaunchKernelGGL(kern, dim3(grid, nsplit), dim3(kRowResThreads), best_lds, s, static_cast<const uint16_t*>(A), meta, \
                           static_cast<int>(Adim), static_cast<int>(K), static_cast<const uint16_t*>(Bsrc), ldb, perm, T, \
                           static_cast<uint16_t*>(C), ldc, best_rpt, stream_out);                            \
    }
    if (dense) {
        if (Adim <= 256) BIMASK_ROWRES(2, 1, true)
        else BIMASK_ROWRES(2, 2, true)
    } else if (Adim <= 256 || split) BIMASK_ROWRES(2, 1, false)
    else if (Adim <= 384) BIMASK_ROWRES(3, 1, false)
    else BIMASK_ROWRES(2, 2, false)
#undef BIMASK_ROWRES
    return check_launch();
}

}  // namespace bimask
