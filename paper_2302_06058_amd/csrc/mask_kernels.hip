// Forward / backward N:M mask selection and operand compression (Eq. 4, Eq. 9, Eq. 11
// of arXiv 2302.06058).  Pure integer work on bit patterns; bound by the HBM read of W.
#include "common.hpp"

namespace bimask {
namespace {

// ---------------------------------------------------------------------------------
// small register helpers
// ---------------------------------------------------------------------------------
template <typename DT> struct Pack;            // 8 consecutive elements in 32-bit words
template <> struct Pack<BF16> { static constexpr int kWords = 4; };
template <> struct Pack<F32> { static constexpr int kWords = 8; };

template <typename DT>
__device__ __forceinline__ uint32_t elem(const uint32_t* words, int q) {   // q is compile-time after unrolling
    if constexpr (sizeof(typename DT::raw) == 2) return (words[q >> 1] >> (16 * (q & 1))) & 0xFFFFu;
    else return words[q];
}

// Load 8 consecutive elements starting at column j0 of a row (guarded, zero-filled).
template <typename DT>
__device__ __forceinline__ void load8(const typename DT::raw* row, int64_t j0, int64_t J, bool vec, uint32_t* out) {
    using raw = typename DT::raw;
    constexpr int W = Pack<DT>::kWords;
    if (vec && j0 + 8 <= J) {
        const uint4* p = reinterpret_cast<const uint4*>(row + j0);
#pragma unroll
        for (int v = 0; v < W / 4; ++v) {
            const uint4 x = p[v];
            out[4 * v + 0] = x.x; out[4 * v + 1] = x.y; out[4 * v + 2] = x.z; out[4 * v + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int w = 0; w < W; ++w) out[w] = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t v = (j0 + q < J) ? static_cast<uint32_t>(row[j0 + q]) : 0u;
            if constexpr (sizeof(raw) == 2) out[q >> 1] |= v << (16 * (q & 1));
            else out[q] = v;
        }
    }
}

__device__ __forceinline__ uint32_t pick4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, int p) {
    uint32_t r = a0;
    r = p == 1 ? a1 : r;
    r = p == 2 ? a2 : r;
    r = p == 3 ? a3 : r;
    return r;
}

// ---------------------------------------------------------------------------------
// Forward direction: one thread owns CH consecutive columns of one row.
//   MODE 0: mask only   1: + 2:4 compressed values/index   2: + dense masked values
// mask_in != nullptr: the mask is read instead of selected (stand-alone compression).
// ---------------------------------------------------------------------------------
template <typename DT, int M, int CH>
__global__ void __launch_bounds__(kThreads)
k_forward(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
          const uint32_t* __restrict__ mask_in, uint32_t* __restrict__ B_bits,
          typename DT::raw* __restrict__ values, uint32_t* __restrict__ index, int mode,
          int wpr, int cpr, int64_t rows_pad, bool vec_in, bool vec_out) {
    using raw = typename DT::raw;
    constexpr int NV = CH / 8;                 // 8-element vectors per chunk
    constexpr int PW = Pack<DT>::kWords;
    const int64_t id = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (id >= rows_pad * cpr) return;
    const int64_t i = id / cpr;
    const int c = static_cast<int>(id - i * cpr);
    const int64_t j0 = static_cast<int64_t>(c) * CH;
    // mode 1 also covers the zero padding of the fragment-major operand (rows >= I, cols >= J)
    const bool in_row = i < I;
    const bool in_mask = in_row && c < wpr * (32 / CH);
    const raw* row = W + (in_row ? i : 0) * ldw;
    const int64_t Jr = in_row ? J : 0;         // padding rows read nothing

    uint32_t w[NV][PW];
#pragma unroll
    for (int v = 0; v < NV; ++v) load8<DT>(row, j0 + 8 * v, Jr, vec_in, w[v]);

    // mask bits of this chunk
    uint32_t bits = 0;
    if (mask_in) {
        if (in_mask) {
            if constexpr (CH == 8) bits = reinterpret_cast<const uint8_t*>(mask_in)[i * wpr * 4 + c];
            else bits = reinterpret_cast<const uint16_t*>(mask_in)[i * wpr * 2 + c];
        }
    } else {
#pragma unroll
        for (int g = 0; g < CH / M; ++g) {
            uint32_t key[M];
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int e = g * M + m;
                key[m] = elem<DT>(w[e / 8], e % 8) & DT::kAbs;
            }
            const uint32_t sel = (j0 + g * M < Jr) ? select_top_n<M>(key, N) : 0u;
            bits |= sel << (g * M);
        }
    }
    if (B_bits && in_mask) {
        if constexpr (CH == 8) reinterpret_cast<uint8_t*>(B_bits)[i * wpr * 4 + c] = static_cast<uint8_t>(bits);
        else reinterpret_cast<uint16_t*>(B_bits)[i * wpr * 2 + c] = static_cast<uint16_t>(bits);
    }

    if (mode == 1) {
        if constexpr (M == 4 && CH == 8) {
            raw out[4];
            uint32_t nibs = 0;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const uint32_t mb = (bits >> (4 * g)) & 15u;
                const uint32_t sel = complete_slots<4>(mb, 2);
                const int p0 = __builtin_ctz(sel), p1 = 31 - __builtin_clz(sel);
                const uint32_t e0 = elem<DT>(w[0], 4 * g + 0), e1 = elem<DT>(w[0], 4 * g + 1),
                               e2 = elem<DT>(w[0], 4 * g + 2), e3 = elem<DT>(w[0], 4 * g + 3);
                out[2 * g + 0] = static_cast<raw>(((mb >> p0) & 1u) ? pick4(e0, e1, e2, e3, p0) : 0u);
                out[2 * g + 1] = static_cast<raw>(((mb >> p1) & 1u) ? pick4(e0, e1, e2, e3, p1) : 0u);
                if (j0 + 4 * g < Jr) nibs |= static_cast<uint32_t>(p0 | (p1 << 2)) << (4 * g);
            }
            // four consecutive slots of one lane vector of the fragment-major layout
            const int64_t ks = static_cast<int64_t>(cpr) / 16;
            raw* dst = values + tiled_val_off(i, j0 / 2, ks);
            if (vec_out) {
                if constexpr (sizeof(raw) == 2) {
                    uint2 v; v.x = out[0] | (static_cast<uint32_t>(out[1]) << 16); v.y = out[2] | (static_cast<uint32_t>(out[3]) << 16);
                    *reinterpret_cast<uint2*>(dst) = v;
                } else {
                    uint4 v; v.x = out[0]; v.y = out[1]; v.z = out[2]; v.w = out[3];
                    *reinterpret_cast<uint4*>(dst) = v;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[e] = out[e];
            }
            const int64_t g0 = j0 / 4;
            reinterpret_cast<uint8_t*>(index)[tiled_idx_word(i, g0, ks) * 4 + ((g0 & 7) >> 1)] = static_cast<uint8_t>(nibs);
        }
    } else if (mode == 2) {
        raw* dst = values + i * J + j0;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            uint32_t o[PW];
#pragma unroll
            for (int pw = 0; pw < PW; ++pw) o[pw] = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t keep = (bits >> (8 * v + q)) & 1u;
                const uint32_t x = keep ? elem<DT>(w[v], q) : 0u;
                if constexpr (sizeof(raw) == 2) o[q >> 1] |= x << (16 * (q & 1));
                else o[q] = x;
            }
            if (vec_out && j0 + 8 * v + 8 <= J) {
                uint4* p = reinterpret_cast<uint4*>(dst + 8 * v);
#pragma unroll
                for (int u = 0; u < PW / 4; ++u) p[u] = make_uint4(o[4 * u], o[4 * u + 1], o[4 * u + 2], o[4 * u + 3]);
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (j0 + 8 * v + q < J) dst[8 * v + q] = static_cast<raw>(elem<DT>(o, q));
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Backward direction: a workgroup owns a tile of 128 permuted rows x TC columns (TC = 128,
// or 32 for small matrices so that enough workgroups exist); a thread owns one block of M
// permuted rows x 8 columns.  Rows of W are gathered through P, every row read is a
// contiguous 2*TC-byte (bf16) segment.  Transposed outputs go through LDS so
// that they leave as contiguous runs along the permuted-row axis.
//   MODE 0: Bbar only   1: + transposed 2:4 values/index   2: + transposed dense masked
// Bbar_in != nullptr: Bbar is read instead of selected (stand-alone compression).
// ---------------------------------------------------------------------------------
constexpr int kTR = 128;   // permuted rows per tile = one 128-deep stage of the transposed operand

// mode 1: fragment-major image of TC output rows x 64 slots (2048 elements per 32 output rows)
template <int TC> __host__ __device__ constexpr int img_elems() { return TC / 32 * 2048; }
template <typename DT> __host__ __device__ constexpr int lds_stride_m2() { return kTR + 16 / (int)sizeof(typename DT::raw); }

template <typename DT, int M, int TC>
__global__ void __launch_bounds__(kThreads)
k_backward(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
           const uint32_t* __restrict__ B_bits, const uint32_t* __restrict__ Bbar_in,
           const int32_t* __restrict__ perm, uint32_t* __restrict__ Bbar_bits,
           typename DT::raw* __restrict__ values, uint32_t* __restrict__ index, int mode,
           int wpr, bool vec_in, bool vec_out) {
    using raw = typename DT::raw;
    constexpr int PW = Pack<DT>::kWords;
    constexpr int NB = kTR / M;                         // row blocks per tile
    extern __shared__ uint4 lds_u4[];
    raw* lds_val = reinterpret_cast<raw*>(lds_u4);
    constexpr int S2 = lds_stride_m2<DT>();
    constexpr int CPT = TC / 8;                         // 8-column chunks per tile row
    uint8_t* lds_meta = reinterpret_cast<uint8_t*>(lds_val + img_elems<TC>());  // mode 1 only: [TC][32] nibbles

    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * kTR;
    const int64_t c0 = static_cast<int64_t>(blockIdx.x) * TC;
    const int ch = threadIdx.x % CPT;
    const int64_t j0 = c0 + ch * 8;

    if (mode == 1) {                                    // padding of the operand image is zero
        constexpr int kZeroWords = (img_elems<TC>() * (int)sizeof(raw) + TC * 32) / 16;
        for (int it = threadIdx.x; it < kZeroWords; it += kThreads) lds_u4[it] = make_uint4(0, 0, 0, 0);
        __syncthreads();
    }

    for (int kb = threadIdx.x / CPT; kb < NB; kb += kThreads / CPT) {
        const int64_t rb = r0 + static_cast<int64_t>(kb) * M;
        if (rb >= I) continue;
        if (j0 >= J) {                                   // pad bytes of the last mask word stay zero
            if (Bbar_bits && j0 < static_cast<int64_t>(wpr) * 32) {
#pragma unroll
                for (int m = 0; m < M; ++m)
                    reinterpret_cast<uint8_t*>(Bbar_bits)[(rb + m) * wpr * 4 + (j0 >> 3)] = 0;
            }
            continue;
        }
        uint32_t w[M][PW];
        uint32_t bb[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int64_t src = perm ? static_cast<int64_t>(perm[rb + m]) : rb + m;
            load8<DT>(W + src * ldw, j0, J, vec_in, w[m]);
            bb[m] = Bbar_in ? reinterpret_cast<const uint8_t*>(Bbar_in)[(rb + m) * wpr * 4 + (j0 >> 3)]
                            : reinterpret_cast<const uint8_t*>(B_bits)[src * wpr * 4 + (j0 >> 3)];
        }
        uint32_t ob[M];
#pragma unroll
        for (int m = 0; m < M; ++m) ob[m] = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint32_t colbits = 0;                       // mask bits of this column block
#pragma unroll
            for (int m = 0; m < M; ++m) colbits |= ((bb[m] >> q) & 1u) << m;
            uint32_t sel;
            if (Bbar_in) {
                sel = complete_slots<M>(colbits, N);
            } else {
                uint32_t key[M];
#pragma unroll
                for (int m = 0; m < M; ++m) key[m] = ((colbits >> m) & 1u) ? (elem<DT>(w[m], q) & DT::kAbs) : 0u;
                sel = select_top_n<M>(key, N);
            }
            const uint32_t keep = Bbar_in ? colbits : (sel & colbits);
#pragma unroll
            for (int m = 0; m < M; ++m) ob[m] |= ((keep >> m) & 1u) << q;
            const int col = ch * 8 + q;
            if (c0 + col >= J) continue;                 // ragged last chunk: not a row of the operand
            if (mode == 1) {
                if constexpr (M == 4) {
                    const int p0 = __builtin_ctz(sel), p1 = 31 - __builtin_clz(sel);
                    const uint32_t e0 = elem<DT>(w[0], q), e1 = elem<DT>(w[1], q), e2 = elem<DT>(w[2], q), e3 = elem<DT>(w[3], q);
                    const uint32_t v0 = ((keep >> p0) & 1u) ? pick4(e0, e1, e2, e3, p0) : 0u;
                    const uint32_t v1 = ((keep >> p1) & 1u) ? pick4(e0, e1, e2, e3, p1) : 0u;
                    // output row = this column, slots 2kb, 2kb+1 of the stage: lane half kb/16,
                    // instruction (kb%16)/4, elements 2(kb%4), 2(kb%4)+1
                    raw* d = lds_val + (((col >> 5) * 4 + ((kb & 15) >> 2)) * 64 + (col & 31) + 32 * (kb >> 4)) * 8 + 2 * (kb & 3);
                    if constexpr (sizeof(raw) == 2) *reinterpret_cast<uint32_t*>(d) = v0 | (v1 << 16);
                    else *reinterpret_cast<uint2*>(d) = make_uint2(v0, v1);
                    lds_meta[col * 32 + kb] = static_cast<uint8_t>(p0 | (p1 << 2));
                }
            } else if (mode == 2) {
#pragma unroll
                for (int m = 0; m < M; ++m)
                    lds_val[col * S2 + kb * M + m] = static_cast<raw>(((keep >> m) & 1u) ? elem<DT>(w[m], q) : 0u);
            }
        }
        if (Bbar_bits) {
#pragma unroll
            for (int m = 0; m < M; ++m)
                reinterpret_cast<uint8_t*>(Bbar_bits)[(rb + m) * wpr * 4 + (j0 >> 3)] = static_cast<uint8_t>(ob[m]);
        }
    }
    if (mode == 0) return;
    __syncthreads();

    const int64_t rows_valid = (I - r0) < kTR ? (I - r0) : kTR;       // multiple of M
    const int64_t cols_valid = (J - c0) < TC ? (J - c0) : TC;
    if (mode == 1) {
        // the tile is stage r0/128 of output row tiles c0/32 .. c0/32+3: 4 KB-contiguous images
        const int64_t ks = ceil_div(I, 128), stage = r0 / kTR;
        const int rts = static_cast<int>((cols_valid + 31) / 32);
        constexpr int VPT = 2048 * (int)sizeof(raw) / 16;              // 16-byte vectors per row tile
        for (int it = threadIdx.x; it < rts * VPT; it += kThreads) {
            const int rtl = it / VPT, v = it % VPT;
            raw* dst = values + ((c0 / 32 + rtl) * ks + stage) * 2048;
            reinterpret_cast<uint4*>(dst)[v] = reinterpret_cast<const uint4*>(lds_val + rtl * 2048)[v];
        }
        for (int it = threadIdx.x; it < rts * 128; it += kThreads) {
            const int rtl = it >> 7, lane = (it & 127) >> 1, wd = it & 1;
            const int col = rtl * 32 + (lane & 31);
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 8; ++b)
                word |= static_cast<uint32_t>(lds_meta[col * 32 + 16 * (lane >> 5) + 8 * wd + b]) << (4 * b);
            index[((c0 / 32 + rtl) * ks + stage) * 128 + lane * 2 + wd] = word;
        }
    } else {
        if (vec_out && rows_valid == kTR) {
            constexpr int EPG = 16 / sizeof(raw);
            constexpr int GPC = kTR / EPG;
            for (int it = threadIdx.x; it < TC * GPC; it += kThreads) {
                const int col = it / GPC, g = it % GPC;
                if (col >= cols_valid) continue;
                const uint4 v = *reinterpret_cast<const uint4*>(lds_val + col * S2 + g * EPG);
                *reinterpret_cast<uint4*>(values + (c0 + col) * I + r0 + g * EPG) = v;
            }
        } else {
            for (int64_t it = threadIdx.x; it < TC * rows_valid; it += kThreads) {
                const int col = static_cast<int>(it / rows_valid), e = static_cast<int>(it % rows_valid);
                if (col >= cols_valid) continue;
                values[(c0 + col) * I + r0 + e] = lds_val[col * S2 + e];
            }
        }
    }
}

template <typename DT, int M>
int run_forward(const void* W, int64_t I, int64_t J, int64_t ldw, int N, const uint32_t* mask_in,
                uint32_t* B_bits, void* values, uint32_t* index, int mode, hipStream_t s) {
    using raw = typename DT::raw;
    constexpr int CH = M == 16 ? 16 : 8;
    const int wpr = static_cast<int>(ceil_div(J, 32));
    // mode 1 walks the padded operand (rows to 32, columns to 128) so that its padding is zeroed
    const int cpr = mode == 1 ? static_cast<int>(round_up(J, 128) / CH) : wpr * 32 / CH;
    const int64_t rows_pad = mode == 1 ? round_up(I, 32) : I;
    if (mode == 1 && (!aligned16(values) || !aligned16(index))) return BIMASK_ERR_ALIGN;
    const bool vec_in = aligned16(W) && (ldw * sizeof(raw)) % 16 == 0;
    const bool vec_out = values && aligned16(values) && (mode == 1 || J % 8 == 0);
    const int64_t total = rows_pad * cpr;
    const unsigned grid = static_cast<unsigned>(ceil_div(total, kThreads));
    hipLaunchKernelGGL((k_forward<DT, M, CH>), dim3(grid), dim3(kThreads), 0, s,
                       static_cast<const raw*>(W), I, J, ldw, N, mask_in, B_bits, static_cast<raw*>(values),
                       index, mode, wpr, cpr, rows_pad, vec_in, vec_out);
    return check_launch();
}

template <typename DT, int M, int TC>
int run_backward_t(const void* W, int64_t I, int64_t J, int64_t ldw, int N, const uint32_t* B_bits,
                   const uint32_t* Bbar_in, const int32_t* perm, uint32_t* Bbar_bits, void* values,
                   uint32_t* index, int mode, hipStream_t s) {
    using raw = typename DT::raw;
    const int wpr = static_cast<int>(ceil_div(J, 32));
    const bool vec_in = aligned16(W) && (ldw * sizeof(raw)) % 16 == 0;
    bool vec_out = false;
    size_t lds = 0;
    if (mode == 1) {
        if (!aligned16(values) || !aligned16(index)) return BIMASK_ERR_ALIGN;
        lds = static_cast<size_t>(img_elems<TC>()) * sizeof(raw) + TC * 32;
    } else if (mode == 2) {
        vec_out = aligned16(values) && (I * sizeof(raw)) % 16 == 0;
        lds = static_cast<size_t>(TC) * lds_stride_m2<DT>() * sizeof(raw);
    }
    auto kern = k_backward<DT, M, TC>;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(lds)) != hipSuccess) return BIMASK_ERR_HIP;
    }
    dim3 grid(static_cast<unsigned>(ceil_div(J, TC)), static_cast<unsigned>(ceil_div(I, kTR)));
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, s, static_cast<const raw*>(W), I, J, ldw, N, B_bits,
                       Bbar_in, perm, Bbar_bits, static_cast<raw*>(values), index, mode, wpr, vec_in, vec_out);
    return check_launch();
}

template <typename DT, int M>
int run_backward(const void* W, int64_t I, int64_t J, int64_t ldw, int N, const uint32_t* B_bits,
                 const uint32_t* Bbar_in, const int32_t* perm, uint32_t* Bbar_bits, void* values,
                 uint32_t* index, int mode, hipStream_t s) {
    // small matrices: narrow tiles so that the grid still covers the chip
    if (ceil_div(J, 128) * ceil_div(I, kTR) < 256)
        return run_backward_t<DT, M, 32>(W, I, J, ldw, N, B_bits, Bbar_in, perm, Bbar_bits, values, index, mode, s);
    return run_backward_t<DT, M, 128>(W, I, J, ldw, N, B_bits, Bbar_in, perm, Bbar_bits, values, index, mode, s);
}

}  // namespace

int launch_forward(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                   const uint32_t* mask_in, uint32_t* B_bits, void* values, uint32_t* index,
                   bool want_values, hipStream_t s) {
    const int mode = !want_values ? 0 : ((N == 2 && M == 4) ? 1 : 2);
#define BIMASK_FWD(DT, MM) return run_forward<DT, MM>(W, I, J, ldw, N, mask_in, B_bits, values, index, mode, s)
    if (dtype == BIMASK_BF16) {
        if (M == 4) BIMASK_FWD(BF16, 4);
        if (M == 8) BIMASK_FWD(BF16, 8);
        if (M == 16) BIMASK_FWD(BF16, 16);
    } else {
        if (M == 4) BIMASK_FWD(F32, 4);
        if (M == 8) BIMASK_FWD(F32, 8);
        if (M == 16) BIMASK_FWD(F32, 16);
    }
#undef BIMASK_FWD
    return BIMASK_ERR_NM;
}

int launch_backward(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                    const uint32_t* B_bits, const uint32_t* Bbar_in, const int32_t* perm,
                    uint32_t* Bbar_bits, void* values, uint32_t* index, bool want_values, hipStream_t s) {
    const int mode = !want_values ? 0 : ((N == 2 && M == 4) ? 1 : 2);
#define BIMASK_BWD(DT, MM) return run_backward<DT, MM>(W, I, J, ldw, N, B_bits, Bbar_in, perm, Bbar_bits, values, index, mode, s)
    if (dtype == BIMASK_BF16) {
        if (M == 4) BIMASK_BWD(BF16, 4);
        if (M == 8) BIMASK_BWD(BF16, 8);
        if (M == 16) BIMASK_BWD(BF16, 16);
    } else {
        if (M == 4) BIMASK_BWD(F32, 4);
        if (M == 8) BIMASK_BWD(F32, 8);
        if (M == 16) BIMASK_BWD(F32, 16);
    }
#undef BIMASK_BWD
    return BIMASK_ERR_NM;
}

}  // namespace bimask
