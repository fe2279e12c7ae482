// Forward / backward N:M mask selection and operand compression (Eq. 4, Eq. 9, Eq. 11
// of arXiv 2302.06058).  Pure integer work on bit patterns; bound by the HBM read of W.
#include "common.hpp"

#include <type_traits>

namespace bimask {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte register vector

// Compressed operands up to this size are written with ordinary stores so that the GEMM that
// follows finds them in L2 (4 MB per XCD); larger ones are streamed to memory.
constexpr size_t kL2Keep = 2u << 20;

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

// Positions p0 < p1 of the two largest magnitudes among four bf16 values packed as
// w0 = (e1:e0), w1 = (e3:e2); equal magnitudes go to the lower index (Eq. 4 with N:M = 2:4).
// Each key is magnitude * 4 + (3 - position): the four keys differ, so the two largest keys
// are exactly the selection, and the second largest of four follows from a 2+2 network.
__device__ __forceinline__ void top2_of4_bf16(uint32_t w0, uint32_t w1, uint32_t& p0, uint32_t& p1) {
    const uint32_t k0 = ((w0 & 0x7FFFu) << 2) | 3u;
    const uint32_t k1 = (((w0 >> 16) & 0x7FFFu) << 2) | 2u;
    const uint32_t k2 = ((w1 & 0x7FFFu) << 2) | 1u;
    const uint32_t k3 = ((w1 >> 16) & 0x7FFFu) << 2;
    const uint32_t hi1 = max(k0, k1), lo1 = min(k0, k1), hi2 = max(k2, k3), lo2 = min(k2, k3);
    const uint32_t top = max(hi1, hi2);
    const uint32_t second = max(min(hi1, hi2), max(lo1, lo2));
    const uint32_t a = top & 3u, b = second & 3u;           // 3 - position
    p0 = 3u - max(a, b);
    p1 = 3u - min(a, b);
}

// One group of four bf16 weights (w0 = e1:e0, w1 = e3:e2): mask bits, index nibble and the two
// slot values (packed) for 2:4 (the two largest magnitudes) or 1:4 (the largest; the other slot
// is the lowest remaining position and carries zero).  Selector byte 0x0C of the byte-permute
// instruction yields 0x00.
__device__ __forceinline__ void select_compress4_bf16(uint32_t w0, uint32_t w1, int N, uint32_t& bits,
                                                      uint32_t& nib, uint32_t& vals) {
    if (N == 2) {
        uint32_t p0, p1;
        top2_of4_bf16(w0, w1, p0, p1);
        bits = (1u << p0) | (1u << p1);
        nib = p0 | (p1 << 2);
        // bytes (2 p0, 2 p0 + 1, 2 p1, 2 p1 + 1) of the 8-byte group
        vals = __builtin_amdgcn_perm(w1, w0, 0x01000100u + p0 * 0x0202u + p1 * 0x02020000u);
    } else {
        const uint32_t k0 = ((w0 & 0x7FFFu) << 2) | 3u;
        const uint32_t k1 = (((w0 >> 16) & 0x7FFFu) << 2) | 2u;
        const uint32_t k2 = ((w1 & 0x7FFFu) << 2) | 1u;
        const uint32_t k3 = ((w1 >> 16) & 0x7FFFu) << 2;
        const uint32_t p = 3u - (max(max(k0, k1), max(k2, k3)) & 3u);     // lowest index among equals
        bits = 1u << p;
        nib = p == 0 ? 4u : (p << 2);                                      // slots (0, 1) or (0, p)
        vals = __builtin_amdgcn_perm(w1, w0, p == 0 ? 0x0C0C0100u : (0x0C0Cu | ((0x0100u + p * 0x0202u) << 16)));
    }
}

// ---------------------------------------------------------------------------------
// Forward direction: one thread owns CH consecutive columns of one row.
//   MODE 0: mask only   2: + dense masked values   (2-of-4 compression: k_forward24 below)
// mask_in != nullptr: the mask is read instead of selected (stand-alone compression).
// ---------------------------------------------------------------------------------
template <typename DT, int M, int CH>
__global__ void __launch_bounds__(kThreads)
k_forward(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
          const uint32_t* __restrict__ mask_in, uint32_t* __restrict__ B_bits,
          typename DT::raw* __restrict__ values, uint32_t* __restrict__ index, int mode,
          int wpr, int cpr, int64_t rows_pad, bool vec_in, bool vec_out) {
    using raw = typename DT::raw;
    (void)vec_out;
    constexpr int NV = CH / 8;                 // 8-element vectors per chunk
    constexpr int PW = Pack<DT>::kWords;
    const int64_t id = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (id >= rows_pad * cpr) return;
    const int64_t i = id / cpr;
    const int c = static_cast<int>(id - i * cpr);
    const int64_t j0 = static_cast<int64_t>(c) * CH;
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

    if (mode == 2) {
        // dense masked operand, fragment-major: every 8-entry granule of the padded matrix is written whole
        // (rows >= I and columns >= J: zeros)
        const int64_t ks = static_cast<int64_t>(cpr) * CH / 128;
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
            uint4* p = reinterpret_cast<uint4*>(values + tiled_dense_off(i, j0 + 8 * v, ks));
#pragma unroll
            for (int u = 0; u < PW / 4; ++u) p[u] = make_uint4(o[4 * u], o[4 * u + 1], o[4 * u + 2], o[4 * u + 3]);
        }
    }
}

// ---------------------------------------------------------------------------------
// Forward direction, 2:4 with compression (the hot case).  A wavefront owns 8 rows x one
// 128-column stage: lane (r, q) = (l/8, l%8) reads the 16 weights [16q, 16q+16) of its row
// (8 lanes cover the row's stage contiguously) and produces exactly one 16-byte lane vector
// of the fragment-major operand -- the 8 lanes that share q write 128 contiguous bytes --
// plus 16 mask bits and 16 index bits, which neighbouring lanes merge into whole words.
// mask_in != nullptr: the mask is read instead of selected (stand-alone compression).
// ---------------------------------------------------------------------------------
template <typename DT, int M>
__device__ __forceinline__ void
forward24_body(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
               const uint32_t* __restrict__ mask_in, uint32_t* __restrict__ B_bits,
               typename DT::raw* __restrict__ values, uint32_t* __restrict__ index,
               int wpr, int ks, int64_t row_octets, bool vec_in, bool stream_out, int64_t block) {
    using raw = typename DT::raw;
    constexpr int PW = Pack<DT>::kWords;
    constexpr int U = 2;                               // stages per wavefront: 4 loads in flight per lane
    const int lane = threadIdx.x & 63;
    const int ksu = (ks + U - 1) / U;
    const int64_t unit = block * (kThreads / 64) + (threadIdx.x >> 6);
    if (unit >= row_octets * ksu) return;
    const int64_t r8 = unit / ksu;
    const int st0 = static_cast<int>(unit - r8 * ksu) * U;
    const int q = lane & 7;
    const int64_t i = r8 * 8 + (lane >> 3);
    const bool in_row = i < I;
    const int64_t Jr = in_row ? J : 0;                 // padding rows read nothing
    const raw* row = W + (in_row ? i : 0) * ldw;

    // Interior wavefronts of the bf16 select-and-compress case (8 rows and both stages inside
    // the matrix, aligned rows) run a straight-line path: all loads issued back to back, no
    // bounds checks, neighbour exchange by a DPP quad swap.  Everything else takes the guarded
    // path below.
    const bool fast = __builtin_amdgcn_readfirstlane(static_cast<int>(
        sizeof(raw) == 2 && M == 4 && N <= 2 && !mask_in && vec_in && r8 * 8 + 8 <= I && static_cast<int64_t>(st0 + U) * 128 <= J)) != 0;
    if constexpr (sizeof(raw) == 2) {
        if (fast) {
            u32x4 t[U][2];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v)
                    t[u][v] = *reinterpret_cast<const u32x4*>(row + static_cast<int64_t>(st0 + u) * 128 + 16 * q + 8 * v);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int st = st0 + u;
                uint32_t bits = 0, nibs = 0;
                u32x4 ov;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t w0 = t[u][g >> 1][(g & 1) * 2], w1 = t[u][g >> 1][(g & 1) * 2 + 1];
                    uint32_t b4, n4, v2;
                    select_compress4_bf16(w0, w1, N, b4, n4, v2);
                    bits |= b4 << (4 * g);
                    nibs |= n4 << (4 * g);
                    ov[g] = v2;
                }
                raw* dst = values + ((((i >> 5) * ks + st) * 4 + (q & 3)) * 64 + (i & 31) + 32 * (q >> 2)) * 8;
                if (stream_out) __builtin_nontemporal_store(ov, reinterpret_cast<u32x4*>(dst));
                else *reinterpret_cast<u32x4*>(dst) = ov;
                // lanes q and q^1 merge their 16 index / mask bits into one word (even lane writes)
                const uint32_t packed = bits | (nibs << 16);
                const uint32_t other = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(packed), 0xB1, 0xF, 0xF, true));
                if (!(q & 1)) {
                    index[(((i >> 5) * ks + st) * 64 + (i & 31) + 32 * (q >> 2)) * 2 + ((q >> 1) & 1)] = (packed >> 16) | (other & 0xFFFF0000u);
                    if (B_bits) B_bits[i * wpr + st * 4 + (q >> 1)] = (packed & 0xFFFFu) | (other << 16);
                }
            }
            return;
        }
    }
    uint32_t w[U][2][PW];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t j0 = static_cast<int64_t>(st0 + u) * 128 + 16 * q;
        load8<DT>(row, j0, Jr, vec_in, w[u][0]);
        load8<DT>(row, j0 + 8, Jr, vec_in, w[u][1]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int st = st0 + u;
        if (st >= ks) break;                           // wave-uniform
        const int64_t j0 = static_cast<int64_t>(st) * 128 + 16 * q;
        const bool in_mask = in_row && (j0 >> 4) < 2 * wpr;      // this lane's half-word exists in B
        uint32_t bits = 0, nibs = 0;
        // values: lane vector (row tile i/32, stage st, instruction q%4, lane i%32 + 32*(q/4))
        raw* dst = values + ((((i >> 5) * ks + st) * 4 + (q & 3)) * 64 + (i & 31) + 32 * (q >> 2)) * 8;
        bool done = false;
        if constexpr (sizeof(raw) == 2 && M == 4) {
            if (!mask_in && N <= 2) {                      // wave-uniform: select and compress in one go
                uint32_t ow[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t w0 = w[u][g >> 1][(g & 1) * 2], w1 = w[u][g >> 1][(g & 1) * 2 + 1];
                    uint32_t b4, n4;
                    select_compress4_bf16(w0, w1, N, b4, n4, ow[g]);
                    bits |= b4 << (4 * g);
                    nibs |= n4 << (4 * g);
                }
                // groups at or beyond the row end (zero padding): no mask bits, index 0
                const int64_t left = (Jr - j0) >> 2;
                const uint32_t vmask = left >= 4 ? 0xFFFFu : (left <= 0 ? 0u : (1u << (4 * static_cast<int>(left))) - 1u);
                bits &= vmask;
                nibs &= vmask;
                // whole 128-byte lines per 8 lanes; streamed past L2 when the operand is too large to
                // wait there for the GEMM anyway
                const u32x4 ov = {ow[0], ow[1], ow[2], ow[3]};
                if (stream_out) __builtin_nontemporal_store(ov, reinterpret_cast<u32x4*>(dst));
                else *reinterpret_cast<u32x4*>(dst) = ov;
                done = true;
            }
        }
        if (!done) {
            if (mask_in) {
                if (in_mask) bits = reinterpret_cast<const uint16_t*>(mask_in)[i * wpr * 2 + (j0 >> 4)];
            } else {
                // Eq. (4): top N of every M consecutive weights (16 / M groups in this lane's 16)
#pragma unroll
                for (int g = 0; g < 16 / M; ++g) {
                    uint32_t key[M];
#pragma unroll
                    for (int m = 0; m < M; ++m) key[m] = elem<DT>(w[u][(g * M + m) >> 3], (g * M + m) & 7) & DT::kAbs;
                    const uint32_t sel = (j0 + M * g < Jr) ? select_top_n<M>(key, N) : 0u;
                    bits |= sel << (M * g);
                }
            }
            uint32_t out[8];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t mb = (bits >> (4 * g)) & 15u;
                const uint32_t sel = complete_slots<4>(mb, 2);
                const int p0 = __builtin_ctz(sel), p1 = 31 - __builtin_clz(sel);
                const uint32_t e0 = elem<DT>(w[u][g >> 1], (g & 1) * 4 + 0), e1 = elem<DT>(w[u][g >> 1], (g & 1) * 4 + 1),
                               e2 = elem<DT>(w[u][g >> 1], (g & 1) * 4 + 2), e3 = elem<DT>(w[u][g >> 1], (g & 1) * 4 + 3);
                out[2 * g + 0] = ((mb >> p0) & 1u) ? pick4(e0, e1, e2, e3, p0) : 0u;
                out[2 * g + 1] = ((mb >> p1) & 1u) ? pick4(e0, e1, e2, e3, p1) : 0u;
                if (j0 + 4 * g < Jr) nibs |= static_cast<uint32_t>(p0 | (p1 << 2)) << (4 * g);
            }
            if constexpr (sizeof(raw) == 2) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(out[0] | (out[1] << 16), out[2] | (out[3] << 16),
                                                            out[4] | (out[5] << 16), out[6] | (out[7] << 16));
            } else {
                reinterpret_cast<uint4*>(dst)[0] = make_uint4(out[0], out[1], out[2], out[3]);
                reinterpret_cast<uint4*>(dst)[1] = make_uint4(out[4], out[5], out[6], out[7]);
            }
        }
        // index / mask: lanes q and q^1 merge their 16 bits into one word, written by the even lane
        const uint32_t nib_other = __shfl_xor(nibs, 1, 64), bit_other = __shfl_xor(bits, 1, 64);
        if (!(q & 1)) {
            const uint32_t iw = nibs | (nib_other << 16), bw = bits | (bit_other << 16);
            index[(((i >> 5) * ks + st) * 64 + (i & 31) + 32 * (q >> 2)) * 2 + ((q >> 1) & 1)] = iw;
            const int64_t word = (j0 >> 5);
            if (B_bits && in_row && word < wpr) B_bits[i * wpr + word] = bw;
        }
    }
}

template <typename DT, int M>
__global__ void __launch_bounds__(kThreads)
k_forward24(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
            const uint32_t* __restrict__ mask_in, uint32_t* __restrict__ B_bits,
            typename DT::raw* __restrict__ values, uint32_t* __restrict__ index,
            int wpr, int ks, int64_t row_octets, bool vec_in, bool stream_out) {
    forward24_body<DT, M>(W, I, J, ldw, N, mask_in, B_bits, values, index, wpr, ks, row_octets, vec_in, stream_out,
                          static_cast<int64_t>(blockIdx.x));
}

// Grouped launches: the workgroups of several independent layers in one grid.  The per-layer
// arguments travel as a table in the kernel arguments; first[l] is the first workgroup of
// layer l.  Small layers are launch-latency bound, a network has dozens of them.
template <typename P>
struct GroupTable {
    int n;
    static constexpr int kCap = group_capacity(sizeof(P));
    unsigned first[kCap + 1];
    P p[kCap];
};
template <typename P>
__device__ __forceinline__ int group_layer_of(const GroupTable<P>& g, unsigned block) {
    int l = 0;
    while (l + 1 < g.n && block >= g.first[l + 1]) ++l;
    return l;
}

struct FwdGroupP {
    const void* W;
    uint32_t* B_bits;
    void* values;
    uint32_t* index;
    int64_t I, J, ldw, row_octets;
    int wpr, ks, vec_in, stream_out;
};

template <typename DT, int M>
__global__ void __launch_bounds__(kThreads)
k_forward24_group(const GroupTable<FwdGroupP> g, int N) {
    using raw = typename DT::raw;
    const int l = group_layer_of(g, blockIdx.x);
    const FwdGroupP& p = g.p[l];
    forward24_body<DT, M>(static_cast<const raw*>(p.W), p.I, p.J, p.ldw, N, nullptr, p.B_bits, static_cast<raw*>(p.values),
                          p.index, p.wpr, p.ks, p.row_octets, p.vec_in != 0, p.stream_out != 0,
                          static_cast<int64_t>(blockIdx.x - g.first[l]));
}

// ---------------------------------------------------------------------------------
// Backward direction: a workgroup owns a tile of 128 permuted rows x TC columns (TC = 128,
// or 32 for small matrices so that enough workgroups exist); a thread owns one block of M
// permuted rows x 8 columns.  Rows of W are gathered through P, every row read is a
// contiguous 2*TC-byte (bf16) segment.  Transposed outputs go through LDS so
// that they leave as contiguous runs along the permuted-row axis.
//   MODE 0: Bbar only   1: + transposed 2-of-4 values/index (N <= 2)   2: + transposed dense masked
// Bbar_in != nullptr: Bbar is read instead of selected (stand-alone compression).
// ---------------------------------------------------------------------------------
constexpr int kTR = 128;   // permuted rows per tile = one 128-deep stage of the transposed operand

// mode 1: fragment-major image of TC output rows x 64 slots (2048 elements per 32 output rows)
template <int TC> __host__ __device__ constexpr int img_elems() { return TC / 32 * 2048; }
template <typename DT> __host__ __device__ constexpr int lds_stride_m2() { return kTR + 16 / (int)sizeof(typename DT::raw); }

template <typename DT, int M, int TC>
__device__ __forceinline__ void
backward_body(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
              const uint32_t* __restrict__ B_bits, const uint32_t* __restrict__ Bbar_in,
              const int32_t* __restrict__ perm, uint32_t* __restrict__ Bbar_bits,
              typename DT::raw* __restrict__ values, uint32_t* __restrict__ index, int mode,
              int wpr, bool vec_in, bool vec_out, unsigned block_x, unsigned block_y) {
    using raw = typename DT::raw;
    constexpr int PW = Pack<DT>::kWords;
    constexpr int NB = kTR / M;                         // row blocks per tile
    extern __shared__ uint4 lds_u4[];
    raw* lds_val = reinterpret_cast<raw*>(lds_u4);
    constexpr int S2 = lds_stride_m2<DT>();
    constexpr int CPT = TC / 8;                         // 8-column chunks per tile row
    uint8_t* lds_meta = reinterpret_cast<uint8_t*>(lds_val + img_elems<TC>());  // mode 1 only: [TC][32] nibbles

    const int64_t r0 = static_cast<int64_t>(block_y) * kTR;
    const int64_t c0 = static_cast<int64_t>(block_x) * TC;
    const int ch = threadIdx.x % CPT;
    const int64_t j0 = c0 + ch * 8;

    if (mode == 1) {                                    // padding of the operand image is zero
        constexpr int kZeroWords = (img_elems<TC>() * (int)sizeof(raw) + TC * 32) / 16;
        for (int it = threadIdx.x; it < kZeroWords; it += kThreads) lds_u4[it] = make_uint4(0, 0, 0, 0);
        __syncthreads();
    } else if (mode == 2) {                             // rows beyond I and columns beyond J of the tile: zeros
        constexpr int kZeroWords = TC * S2 * (int)sizeof(raw) / 16;
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
                // N <= 2: every aligned group of 4 permuted rows keeps at most two entries; its slots
                // are the kept positions completed with the lowest-index other positions
#pragma unroll
                for (int sg = 0; sg < M / 4; ++sg) {
                    const uint32_t k4 = (keep >> (4 * sg)) & 15u;
                    const uint32_t sl = complete_slots<4>(k4, 2);
                    const int p0 = __builtin_ctz(sl), p1 = 31 - __builtin_clz(sl);
                    const uint32_t e0 = elem<DT>(w[4 * sg + 0], q), e1 = elem<DT>(w[4 * sg + 1], q),
                                   e2 = elem<DT>(w[4 * sg + 2], q), e3 = elem<DT>(w[4 * sg + 3], q);
                    const uint32_t v0 = ((k4 >> p0) & 1u) ? pick4(e0, e1, e2, e3, p0) : 0u;
                    const uint32_t v1 = ((k4 >> p1) & 1u) ? pick4(e0, e1, e2, e3, p1) : 0u;
                    // output row = this column, group g4 of the stage's 32: lane half g4/16,
                    // instruction (g4%16)/4, elements 2(g4%4), 2(g4%4)+1
                    const int g4 = kb * (M / 4) + sg;
                    raw* d = lds_val + (((col >> 5) * 4 + ((g4 & 15) >> 2)) * 64 + (col & 31) + 32 * (g4 >> 4)) * 8 + 2 * (g4 & 3);
                    if constexpr (sizeof(raw) == 2) *reinterpret_cast<uint32_t*>(d) = v0 | (v1 << 16);
                    else *reinterpret_cast<uint2*>(d) = make_uint2(v0, v1);
                    lds_meta[col * 32 + g4] = static_cast<uint8_t>(p0 | (p1 << 2));
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

    (void)vec_out;
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
        // dense masked operand, fragment-major: the tile is stage r0 / 128 of the output rows c0 .. c0 + TC - 1;
        // whole 32-row tiles are written (output rows beyond J are zero padding), 8 entries at a time
        (void)rows_valid;
        const int64_t ks = ceil_div(I, 128);
        const int rows_out = static_cast<int>((cols_valid + 31) / 32) * 32;
        constexpr int V = 8 * (int)sizeof(raw) / 16;                  // 16-byte vectors per granule
        for (int it = threadIdx.x; it < rows_out * 16; it += kThreads) {
            const int g = it / rows_out, col = it - g * rows_out;     // consecutive threads: consecutive output rows
            const uint4* src = reinterpret_cast<const uint4*>(lds_val + col * S2 + g * 8);
            uint4* dst = reinterpret_cast<uint4*>(values + tiled_dense_off(c0 + col, r0 + 8 * g, ks));
#pragma unroll
            for (int u = 0; u < V; ++u) dst[u] = src[u];
        }
    }
}

template <typename DT, int M, int TC>
__global__ void __launch_bounds__(kThreads)
k_backward(const typename DT::raw* __restrict__ W, int64_t I, int64_t J, int64_t ldw, int N,
           const uint32_t* __restrict__ B_bits, const uint32_t* __restrict__ Bbar_in,
           const int32_t* __restrict__ perm, uint32_t* __restrict__ Bbar_bits,
           typename DT::raw* __restrict__ values, uint32_t* __restrict__ index, int mode,
           int wpr, bool vec_in, bool vec_out) {
    backward_body<DT, M, TC>(W, I, J, ldw, N, B_bits, Bbar_in, perm, Bbar_bits, values, index, mode, wpr, vec_in, vec_out,
                             blockIdx.x, blockIdx.y);
}

struct BwdGenGroupP {
    const void* W;
    const uint32_t* B_bits;
    const int32_t* perm;
    uint32_t* Bbar_bits;
    void* values;
    uint32_t* index;
    int64_t I, J, ldw;
    int wpr, vec_in, vec_out;
    unsigned gx;                                        // column tiles of the layer
};

// small layers of any dtype / ratio: 128 permuted rows x 32 columns per workgroup
template <typename DT, int M>
__global__ void __launch_bounds__(kThreads)
k_backward_group(const GroupTable<BwdGenGroupP> g, int N, int mode) {
    using raw = typename DT::raw;
    const int l = group_layer_of(g, blockIdx.x);
    const BwdGenGroupP& p = g.p[l];
    const unsigned local = blockIdx.x - g.first[l];
    backward_body<DT, M, 32>(static_cast<const raw*>(p.W), p.I, p.J, p.ldw, N, p.B_bits, nullptr, p.perm, p.Bbar_bits,
                             static_cast<raw*>(p.values), p.index, mode, p.wpr, p.vec_in != 0, p.vec_out != 0,
                             local % p.gx, local / p.gx);
}

// ---------------------------------------------------------------------------------
// Backward direction, bf16 2:4 with transposed compression (the hot case).  A wavefront owns
// 32 permuted rows x 64*NO columns and needs no other wavefront: lane (k, c) = (l/8, l%8)
// owns the block of 4 permuted rows 4k..4k+3 and the column octets c (and c + 8 for NO = 2).
// Rows of W are gathered through P as contiguous 128*NO-byte segments (8 lanes x 16 bytes).
// The mask words of B are loaded once per quad of lanes and redistributed with a 4x4 byte
// transpose inside the quad, so that each lane has the bits of its octet for its 4 rows;
// the same transpose in the other direction yields whole words of Bbar.  W is ANDed with
// the expanded mask (this is B (.) W of Eq. 9), each column's 4 values are brought into one
// register pair and selected like a forward group.  Transposed values go through a
// bank-swizzled LDS image of the wavefront's part of the fragment-major operand and leave
// as 512-byte contiguous runs; the 2-bit indices are transposed across the 8 row-block
// lanes in registers and stored as whole words.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t quad_transpose_bytes(uint32_t x, int lane) {
    // lane j of each quad ends with byte j of the four lanes (byte m from lane m); involution
    uint32_t p = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0xB1, 0xF, 0xF, true));
    x = __builtin_amdgcn_perm(p, x, (lane & 1) ? 0x03070105u : 0x06020400u);
    p = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x4E, 0xF, 0xF, true));
    x = __builtin_amdgcn_perm(p, x, (lane & 2) ? 0x03020706u : 0x05040100u);
    return x;
}

// 8x8 transpose of 4-bit fields across the 8 lanes that share lane % 8 (k = lane / 8):
// lane k ends with field k of every lane, field j coming from lane j.  Branch-free: the lane's
// side of each exchange is a select between two shifts and one bit-field insert.
__device__ __forceinline__ uint32_t nibble_transpose8(uint32_t x, int k) {
    uint32_t p = __shfl_xor(x, 32, 64);
    uint32_t keep = (k & 4) ? 0xFFFF0000u : 0x0000FFFFu;
    uint32_t ps = (k & 4) ? (p >> 16) : (p << 16);
    x = (x & keep) | (ps & ~keep);
    p = __shfl_xor(x, 16, 64);
    keep = (k & 2) ? 0xFF00FF00u : 0x00FF00FFu;
    ps = (k & 2) ? (p >> 8) : (p << 8);
    x = (x & keep) | (ps & ~keep);
    p = __shfl_xor(x, 8, 64);
    keep = (k & 1) ? 0xF0F0F0F0u : 0x0F0F0F0Fu;
    ps = (k & 1) ? (p >> 4) : (p << 4);
    x = (x & keep) | (ps & ~keep);
    return x;
}

// One wavefront's tile.  FAST: all 32 rows and all 64*NO columns lie inside the matrix and
// rows are 16-byte aligned, so every load and store is unconditional and the row loads are
// issued back to back; otherwise everything is bounds-checked.
template <int NO, bool FAST>
__device__ __forceinline__ void backward24_tile(
        const uint16_t* __restrict__ W, int64_t I, int64_t J, int64_t ldw, const uint32_t* __restrict__ B_bits,
        const int32_t* __restrict__ perm, uint32_t* __restrict__ Bbar_bits, uint16_t* __restrict__ values,
        uint32_t* __restrict__ index, int wpr, bool vec_in, bool vec_perm, bool stream_out, bool active,
        int64_t r0, int c0, uint4* lds_wave, int lane, int N) {
    const int c = lane & 7, k = lane >> 3;
    const int64_t rb = r0 + 4 * k;
    const bool row_ok = FAST || (active && rb < I);
    const int64_t Jr = row_ok ? J : 0;                   // rows beyond I (stage padding) read nothing

    int64_t src[4] = {0, 0, 0, 0};
    if (row_ok) {
        if (!perm) {
#pragma unroll
            for (int m = 0; m < 4; ++m) src[m] = rb + m;
        } else if (vec_perm) {
            const int4 pv = *reinterpret_cast<const int4*>(perm + rb);
            src[0] = pv.x; src[1] = pv.y; src[2] = pv.z; src[3] = pv.w;
        } else {
#pragma unroll
            for (int m = 0; m < 4; ++m) src[m] = perm[rb + m];
        }
    }
    uint32_t w[4][NO][4];
    if constexpr (FAST) {
        u32x4 t[4][NO];
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int o2 = 0; o2 < NO; ++o2)
                t[m][o2] = *reinterpret_cast<const u32x4*>(W + src[m] * ldw + c0 + 8 * (c + 8 * o2));
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int o2 = 0; o2 < NO; ++o2) {
                w[m][o2][0] = t[m][o2].x; w[m][o2][1] = t[m][o2].y; w[m][o2][2] = t[m][o2].z; w[m][o2][3] = t[m][o2].w;
            }
    } else {
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int o2 = 0; o2 < NO; ++o2)
                load8<BF16>(W + src[m] * ldw, c0 + 8 * (c + 8 * o2), Jr, vec_in, w[m][o2]);
    }

    // mask bits: lane (a, m) = (c / 4, c % 4) fetches word a (+ 2 for the second octet) of row m
    const int64_t src_m = (c & 2) ? ((c & 1) ? src[3] : src[2]) : ((c & 1) ? src[1] : src[0]);
    uint32_t X[NO];
#pragma unroll
    for (int o2 = 0; o2 < NO; ++o2) {
        const int word = c0 / 32 + 2 * o2 + (c >> 2);
        const uint32_t bw = (FAST || (row_ok && word < wpr)) ? B_bits[src_m * wpr + word] : 0u;
        X[o2] = quad_transpose_bytes(bw, lane);          // byte m = bits of row m for this lane's octet
    }

    uint32_t* lds32 = reinterpret_cast<uint32_t*>(lds_wave);
    // LDS word of (output row = column 8 (c + 8 o2) + q, row block k): unit ul, word k % 4
    const int ul0 = ((c >> 2) * 2 + (k >> 2)) * 32 + 8 * (c & 3);
    uint32_t nib[NO], R[NO];
#pragma unroll
    for (int o2 = 0; o2 < NO; ++o2) {
        // B (.) W
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // mask bit -> 0 / all ones by a signed one-bit field extract, the two halves merged by a bit-field insert
                const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_sbfe(static_cast<int>(X[o2]), 8 * m + 2 * j, 1));
                const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_sbfe(static_cast<int>(X[o2]), 8 * m + 2 * j + 1, 1));
                w[m][o2][j] &= (lo & 0x0000FFFFu) | (hi & ~0x0000FFFFu);
            }
        nib[o2] = 0;
        R[o2] = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int j = q >> 1;
            const uint32_t half = (q & 1) ? 0x07060302u : 0x05040100u;
            const uint32_t e01 = __builtin_amdgcn_perm(w[1][o2][j], w[0][o2][j], half);   // (row 1 : row 0)
            const uint32_t e23 = __builtin_amdgcn_perm(w[3][o2][j], w[2][o2][j], half);   // (row 3 : row 2)
            uint32_t b4, n4, ow;
            select_compress4_bf16(e01, e23, N, b4, n4, ow);              // top N of the column's 4 masked weights
            nib[o2] |= n4 << (4 * q);
            // byte m: columns that select row m
            // (bit m of b4 to bit 8 m: one 24-bit multiply spreads the four bits 7 apart, the mask keeps bit 0 of each byte)
            R[o2] |= (__umul24(b4, 0x00204081u) & 0x01010101u) << q;
            // output row = this column; slots 2kb, 2kb+1 of the stage (kb = row block in the stage)
            const int ul = ul0 + o2 * 128 + q;
            lds32[((ul ^ ((ul >> 4) & 7)) << 2) + (k & 3)] = ow;
        }
    }

    // position of this wavefront's 32 rows inside the 128-deep stage of the transposed operand
    const int64_t ks = ceil_div(I, 128), stage = r0 >> 7;
    const int kb0 = static_cast<int>(r0 & 127) >> 2;     // first row block: 0, 8, 16 or 24
    const int lane_half = kb0 >> 4, s4base = (kb0 & 15) >> 2, wd = (kb0 >> 3) & 1;

#pragma unroll
    for (int o2 = 0; o2 < NO; ++o2) {
        // Bbar = selection AND B, back to whole words per row
        const uint32_t back = quad_transpose_bytes(R[o2] & X[o2], lane);
        const int word = c0 / 32 + 2 * o2 + (c >> 2);
        if (Bbar_bits && (FAST || (row_ok && word < wpr))) Bbar_bits[(rb + (c & 3)) * wpr + word] = back;
        // indices: columns at or beyond J and padding rows carry index 0
        uint32_t vm = 0xFFFFFFFFu;
        if constexpr (!FAST) {
            const int64_t left = J - (c0 + 8 * (c + 8 * o2));
            vm = !row_ok || left <= 0 ? 0u : (left >= 8 ? 0xFFFFFFFFu : (1u << (4 * static_cast<int>(left))) - 1u);
        }
        const uint32_t iw = nibble_transpose8(nib[o2] & vm, k);          // column 8 (c + 8 o2) + k, row blocks kb0..kb0+7
        const int col = 8 * (c + 8 * o2) + k;
        if (FAST || (active && c0 + (col & ~31) < J))
            index[((c0 / 32 + (col >> 5)) * ks + stage) * 128 + ((col & 31) + 32 * lane_half) * 2 + wd] = iw;
    }
    // the image is written and read by this wavefront only; LDS operations of a wavefront
    // execute in order, the fence keeps the compiler from moving the reads up
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
    for (int it0 = 0; it0 < 2 * NO; ++it0) {
        const int it = lane + 64 * it0;                   // (row tile it0, slot it/32 % 2, lane it % 32)
        const u32x4 v = reinterpret_cast<const u32x4*>(lds_wave)[it ^ ((it >> 4) & 7)];
        if (FAST || (active && c0 + 32 * it0 < J)) {
            uint16_t* dst = values + ((((c0 / 32 + it0) * ks + stage) * 4 + s4base + ((it >> 5) & 1)) * 64 + (it & 31) + 32 * lane_half) * 8;
            // 512-byte runs, whole lines; streamed past L2 for operands too large to stay there
            if (stream_out) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
            else *reinterpret_cast<u32x4*>(dst) = v;
        }
    }
}

template <int NO>
__global__ void __launch_bounds__(kThreads)
k_backward24_bf16(const uint16_t* __restrict__ W, int64_t I, int64_t J, int64_t ldw,
                  const uint32_t* __restrict__ B_bits, const int32_t* __restrict__ perm,
                  uint32_t* __restrict__ Bbar_bits, uint16_t* __restrict__ values,
                  uint32_t* __restrict__ index, int wpr, int64_t col_tiles, int64_t units,
                  bool vec_in, bool vec_perm, bool stream_out, int N) {
    constexpr int TC = 64 * NO;
    // per wavefront: 2*NO output row tiles x 2 instruction slots x 32 lanes x 16 bytes
    __shared__ uint4 lds[kThreads / 64][NO * 128];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t unit = static_cast<int64_t>(blockIdx.x) * (blockDim.x >> 6) + wave;
    const bool active = unit < units;
    const int64_t rg = active ? unit / col_tiles : 0;
    const int c0 = static_cast<int>((active ? unit - rg * col_tiles : 0) * TC);
    const int64_t r0 = rg * 32;
    const bool fast = __builtin_amdgcn_readfirstlane(
        static_cast<int>(active && vec_in && r0 + 32 <= I && c0 + TC <= J)) != 0;
    if (fast)
        backward24_tile<NO, true>(W, I, J, ldw, B_bits, perm, Bbar_bits, values, index, wpr, vec_in, vec_perm,
                                  stream_out, active, r0, c0, lds[wave], lane, N);
    else
        backward24_tile<NO, false>(W, I, J, ldw, B_bits, perm, Bbar_bits, values, index, wpr, vec_in, vec_perm,
                                   stream_out, active, r0, c0, lds[wave], lane, N);
}

struct BwdGroupP {
    const uint16_t* W;
    const uint32_t* B_bits;
    const int32_t* perm;
    uint32_t* Bbar_bits;
    uint16_t* values;
    uint32_t* index;
    int64_t I, J, ldw, col_tiles, units;
    int wpr, vec_in, vec_perm, stream_out;
};

// small bf16 2:4 layers, one wavefront (= one 32 x 64 tile) per workgroup
__global__ void __launch_bounds__(64)
k_backward24_bf16_group(const GroupTable<BwdGroupP> g, int N) {
    __shared__ uint4 lds[128];
    const int l = group_layer_of(g, blockIdx.x);
    const BwdGroupP& p = g.p[l];
    const int lane = threadIdx.x & 63;
    const int64_t unit = static_cast<int64_t>(blockIdx.x - g.first[l]);
    const bool active = unit < p.units;
    const int64_t rg = active ? unit / p.col_tiles : 0;
    const int c0 = static_cast<int>((active ? unit - rg * p.col_tiles : 0) * 64);
    const int64_t r0 = rg * 32;
    const bool fast = __builtin_amdgcn_readfirstlane(
        static_cast<int>(active && p.vec_in != 0 && r0 + 32 <= p.I && c0 + 64 <= p.J)) != 0;
    if (fast)
        backward24_tile<1, true>(p.W, p.I, p.J, p.ldw, p.B_bits, p.perm, p.Bbar_bits, p.values, p.index, p.wpr, p.vec_in != 0,
                                 p.vec_perm != 0, p.stream_out != 0, active, r0, c0, lds, lane, N);
    else
        backward24_tile<1, false>(p.W, p.I, p.J, p.ldw, p.B_bits, p.perm, p.Bbar_bits, p.values, p.index, p.wpr, p.vec_in != 0,
                                  p.vec_perm != 0, p.stream_out != 0, active, r0, c0, lds, lane, N);
}

template <typename DT, int M>
int run_forward(const void* W, int64_t I, int64_t J, int64_t ldw, int N, const uint32_t* mask_in,
                uint32_t* B_bits, void* values, uint32_t* index, int mode, hipStream_t s) {
    using raw = typename DT::raw;
    constexpr int CH = M == 16 ? 16 : 8;
    const int wpr = static_cast<int>(ceil_div(J, 32));
    if (mode == 1) {                                   // N <= 2: the 2-of-4 operand format
        if (!aligned16(values) || !aligned16(index)) return BIMASK_ERR_ALIGN;
        const bool vec_in = aligned16(W) && (ldw * sizeof(raw)) % 16 == 0;
        const int ks = static_cast<int>(round_up(J, 128) / 128);
        const int64_t row_octets = round_up(I, 32) / 8;
        const int64_t units = row_octets * ((ks + 1) / 2);     // one wavefront each (two stages)
        hipLaunchKernelGGL((k_forward24<DT, M>), dim3(static_cast<unsigned>(ceil_div(units, kThreads / 64))),
                           dim3(kThreads), 0, s, static_cast<const raw*>(W), I, J, ldw, N, mask_in, B_bits,
                           static_cast<raw*>(values), index, wpr, ks, row_octets, vec_in,
                           static_cast<size_t>(I) * J * sizeof(raw) / 2 > kL2Keep);
        return check_launch();
    }
    // mask only: threads cover the mask words; dense operand: the padded matrix (rows to 32, columns to 128)
    const int cpr = mode == 2 ? static_cast<int>(round_up(J, 128) / CH) : wpr * 32 / CH;
    const int64_t rows_pad = mode == 2 ? round_up(I, 32) : I;
    if (mode == 2 && !aligned16(values)) return BIMASK_ERR_ALIGN;
    const bool vec_in = aligned16(W) && (ldw * sizeof(raw)) % 16 == 0;
    const bool vec_out = true;
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
        if (!aligned16(values)) return BIMASK_ERR_ALIGN;
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
    if constexpr (std::is_same<DT, BF16>::value && M == 4) {
        if (mode == 1 && !Bbar_in && N <= 2) {
            if (!aligned16(values) || !aligned16(index)) return BIMASK_ERR_ALIGN;
            const int wpr = static_cast<int>(ceil_div(J, 32));
            const bool vec_in = aligned16(W) && (ldw * 2) % 16 == 0;
            const bool vec_perm = perm && aligned16(perm);
            const int64_t row_groups = ceil_div(I, 128) * 4;            // 32-row groups of the padded stages
            const uint16_t* Wp = static_cast<const uint16_t*>(W);
            uint16_t* vp = static_cast<uint16_t*>(values);
            const bool stream_out = static_cast<size_t>(I) * J > kL2Keep;     // operand bytes = I*J*2/2
            // wide tiles when they still give every SIMD of the chip a wavefront
            if (row_groups * ceil_div(J, 128) >= 2048) {
                const int64_t ct = ceil_div(J, 128), units = row_groups * ct;
                hipLaunchKernelGGL((k_backward24_bf16<2>), dim3(static_cast<unsigned>(ceil_div(units, 4))), dim3(kThreads),
                                   0, s, Wp, I, J, ldw, B_bits, perm, Bbar_bits, vp, index, wpr, ct, units, vec_in, vec_perm, stream_out, N);
            } else {
                // small matrices: one wavefront per workgroup so that the tiles spread over all CUs
                const int64_t ct = ceil_div(J, 64), units = row_groups * ct;
                hipLaunchKernelGGL((k_backward24_bf16<1>), dim3(static_cast<unsigned>(units)), dim3(64),
                                   0, s, Wp, I, J, ldw, B_bits, perm, Bbar_bits, vp, index, wpr, ct, units, vec_in, vec_perm, stream_out, N);
            }
            return check_launch();
        }
    }
    // small matrices: narrow tiles so that the grid still covers the chip
    if (ceil_div(J, 128) * ceil_div(I, kTR) < 256)
        return run_backward_t<DT, M, 32>(W, I, J, ldw, N, B_bits, Bbar_in, perm, Bbar_bits, values, index, mode, s);
    return run_backward_t<DT, M, 128>(W, I, J, ldw, N, B_bits, Bbar_in, perm, Bbar_bits, values, index, mode, s);
}

}  // namespace

int launch_forward(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                   const uint32_t* mask_in, uint32_t* B_bits, void* values, uint32_t* index,
                   bool want_values, hipStream_t s) {
    const int mode = !want_values ? 0 : (uses_sp24(N, M) ? 1 : 2);
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

// ---- grouped launches ------------------------------------------------------------
namespace {

template <typename DT, int M>
int run_forward_group(const bimask_group_layer* L, int n, int N, hipStream_t s) {
    using raw = typename DT::raw;
    constexpr int kCap = GroupTable<FwdGroupP>::kCap;
    for (int b = 0; b < n; b += kCap) {
        GroupTable<FwdGroupP> g{};
        g.n = n - b < kCap ? n - b : kCap;
        unsigned blocks = 0;
        for (int l = 0; l < g.n; ++l) {
            const bimask_group_layer& a = L[b + l];
            FwdGroupP& p = g.p[l];
            p.W = a.W; p.B_bits = a.B_bits; p.values = a.Wf_values; p.index = a.Wf_index;
            p.I = a.I; p.J = a.J; p.ldw = a.ldw;
            p.wpr = static_cast<int>(ceil_div(a.J, 32));
            p.ks = static_cast<int>(round_up(a.J, 128) / 128);
            p.row_octets = round_up(a.I, 32) / 8;
            p.vec_in = aligned16(a.W) && (a.ldw * sizeof(raw)) % 16 == 0;
            p.stream_out = static_cast<size_t>(a.I) * a.J * sizeof(raw) / 2 > kL2Keep;
            g.first[l] = blocks;
            blocks += static_cast<unsigned>(ceil_div(p.row_octets * ((p.ks + 1) / 2), kThreads / 64));
        }
        g.first[g.n] = blocks;
        hipLaunchKernelGGL((k_forward24_group<DT, M>), dim3(blocks), dim3(kThreads), 0, s, g, N);
        if (int rc = check_launch()) return rc;
    }
    return BIMASK_OK;
}

}  // namespace

// Forward mask + compressed operand of n independent layers (same dtype and N:M).
int launch_forward_group(const bimask_group_layer* L, int n, int dtype, int N, int M, hipStream_t s) {
    if (uses_sp24(N, M)) {
#define BIMASK_FWDG(DT, MM) return run_forward_group<DT, MM>(L, n, N, s)
        if (dtype == BIMASK_BF16) {
            if (M == 4) BIMASK_FWDG(BF16, 4);
            if (M == 8) BIMASK_FWDG(BF16, 8);
            if (M == 16) BIMASK_FWDG(BF16, 16);
        } else {
            if (M == 4) BIMASK_FWDG(F32, 4);
            if (M == 8) BIMASK_FWDG(F32, 8);
            if (M == 16) BIMASK_FWDG(F32, 16);
        }
#undef BIMASK_FWDG
        return BIMASK_ERR_NM;
    }
    for (int l = 0; l < n; ++l)                           // dense masked operands: one launch per layer
        if (int rc = launch_forward(L[l].W, L[l].I, L[l].J, L[l].ldw, dtype, N, M, nullptr, L[l].B_bits, L[l].Wf_values,
                                    L[l].Wf_index, true, s)) return rc;
    return BIMASK_OK;
}

namespace {

// small layers on the general kernel (any dtype / ratio): 128 x 32 tiles
template <typename DT, int M>
int run_backward_group_general(const bimask_group_layer* L, const int* which, int cnt, int N, int mode, hipStream_t s) {
    using raw = typename DT::raw;
    constexpr int TC = 32;
    const size_t lds = mode == 1 ? static_cast<size_t>(img_elems<TC>()) * sizeof(raw) + TC * 32
                                 : static_cast<size_t>(TC) * lds_stride_m2<DT>() * sizeof(raw);
    constexpr int kCap = GroupTable<BwdGenGroupP>::kCap;
    for (int b = 0; b < cnt; b += kCap) {
        GroupTable<BwdGenGroupP> g{};
        g.n = cnt - b < kCap ? cnt - b : kCap;
        unsigned blocks = 0;
        for (int l = 0; l < g.n; ++l) {
            const bimask_group_layer& a = L[which[b + l]];
            BwdGenGroupP& p = g.p[l];
            p.W = a.W; p.B_bits = a.B_bits; p.perm = a.best_perm; p.Bbar_bits = a.Bbar_bits;
            p.values = a.Wb_values; p.index = a.Wb_index;
            p.I = a.I; p.J = a.J; p.ldw = a.ldw;
            p.wpr = static_cast<int>(ceil_div(a.J, 32));
            p.vec_in = aligned16(a.W) && (a.ldw * sizeof(raw)) % 16 == 0;
            p.vec_out = mode == 2 && aligned16(a.Wb_values) && (a.I * sizeof(raw)) % 16 == 0;
            p.gx = static_cast<unsigned>(ceil_div(a.J, TC));
            g.first[l] = blocks;
            blocks += p.gx * static_cast<unsigned>(ceil_div(a.I, kTR));
        }
        g.first[g.n] = blocks;
        hipLaunchKernelGGL((k_backward_group<DT, M>), dim3(blocks), dim3(kThreads), lds, s, g, N, mode);
        if (int rc = check_launch()) return rc;
    }
    return BIMASK_OK;
}

}  // namespace

// Backward mask + transposed compressed operand of n independent layers, each with its own
// permutation (best_perm).  Small layers share grouped launches (bf16 2:4: the wavefront-tile
// kernel; everything else: the general kernel); layers large enough to fill the chip on their
// own are launched one by one.
int launch_backward_group(const bimask_group_layer* L, int n, int dtype, int N, int M, hipStream_t s) {
    const bool fastpath = dtype == BIMASK_BF16 && N <= 2 && M == 4;
    const int mode = uses_sp24(N, M) ? 1 : 2;
    GroupTable<BwdGroupP> g{};
    unsigned blocks = 0;
    auto flush = [&]() -> int {
        if (g.n == 0) return BIMASK_OK;
        g.first[g.n] = blocks;
        hipLaunchKernelGGL(k_backward24_bf16_group, dim3(blocks), dim3(64), 0, s, g, N);
        g.n = 0;
        blocks = 0;
        return check_launch();
    };
    int general[1024], n_general = 0;
    for (int l = 0; l < n; ++l) {
        const bimask_group_layer& a = L[l];
        const int64_t row_groups = ceil_div(a.I, 128) * 4;
        const bool big = fastpath ? row_groups * ceil_div(a.J, 128) >= 2048 : ceil_div(a.J, 128) * ceil_div(a.I, kTR) >= 256;
        if (big || (!fastpath && n_general == 1024)) {
            if (int rc = launch_backward(a.W, a.I, a.J, a.ldw, dtype, N, M, a.B_bits, nullptr, a.best_perm, a.Bbar_bits,
                                         a.Wb_values, a.Wb_index, true, s)) return rc;
            continue;
        }
        if (!fastpath) {
            general[n_general++] = l;
            continue;
        }
        BwdGroupP& p = g.p[g.n];
        p.W = static_cast<const uint16_t*>(a.W); p.B_bits = a.B_bits; p.perm = a.best_perm; p.Bbar_bits = a.Bbar_bits;
        p.values = static_cast<uint16_t*>(a.Wb_values); p.index = a.Wb_index;
        p.I = a.I; p.J = a.J; p.ldw = a.ldw;
        p.col_tiles = ceil_div(a.J, 64);
        p.units = row_groups * p.col_tiles;
        p.wpr = static_cast<int>(ceil_div(a.J, 32));
        p.vec_in = aligned16(a.W) && (a.ldw * 2) % 16 == 0;
        p.vec_perm = a.best_perm && aligned16(a.best_perm);
        p.stream_out = static_cast<size_t>(a.I) * a.J > kL2Keep;
        g.first[g.n] = blocks;
        blocks += static_cast<unsigned>(p.units);
        if (++g.n == GroupTable<BwdGroupP>::kCap)
            if (int rc = flush()) return rc;
    }
    if (int rc = flush()) return rc;
    if (n_general > 0) {
#define BIMASK_BWDG(DT, MM) return run_backward_group_general<DT, MM>(L, general, n_general, N, mode, s)
        if (dtype == BIMASK_BF16) {
            if (M == 4) BIMASK_BWDG(BF16, 4);
            if (M == 8) BIMASK_BWDG(BF16, 8);
            if (M == 16) BIMASK_BWDG(BF16, 16);
        } else {
            if (M == 4) BIMASK_BWDG(F32, 4);
            if (M == 8) BIMASK_BWDG(F32, 8);
            if (M == 16) BIMASK_BWDG(F32, 16);
        }
#undef BIMASK_BWDG
        return BIMASK_ERR_NM;
    }
    return BIMASK_OK;
}

int launch_backward(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                    const uint32_t* B_bits, const uint32_t* Bbar_in, const int32_t* perm,
                    uint32_t* Bbar_bits, void* values, uint32_t* index, bool want_values, hipStream_t s) {
    const int mode = !want_values ? 0 : (uses_sp24(N, M) ? 1 : 2);
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
