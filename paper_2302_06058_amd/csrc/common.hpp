// Shared host/device helpers of the Bi-Mask HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>
#include "../../include/bimask.h"

namespace bimask {

constexpr int kThreads = 256;   // 4 wavefronts of 64 lanes per workgroup

// Storage types: weights travel as raw bit patterns, magnitudes are compared as
// unsigned integers with the sign bit cleared (total order, +0 == -0).
struct BF16 { using raw = uint16_t; static constexpr uint32_t kAbs = 0x7FFFu; };
struct F32  { using raw = uint32_t; static constexpr uint32_t kAbs = 0x7FFFFFFFu; };

__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ inline int ilog2(int m) { int b = 0; while ((1 << b) < m) ++b; return b; }

// N:M ratios with N <= 2 keep at most two entries in every aligned group of 4 (M is a multiple
// of 4), so their operands use the 2-of-4 format of the sparse matrix instruction.
__host__ __device__ inline bool uses_sp24(int N, int M) { return N <= 2 && M % 4 == 0; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

// Host-side memo of one small answer of the runtime per GPU (an occupancy figure, "this kernel's LDS limit
// has been raised"): such answers belong to a device, so they are remembered per device ordinal, each as ONE
// 64-bit word that is read and written atomically (0 = not known yet).  Objects of this type have static
// storage (zero-initialised).  No other host state is kept between calls.
constexpr int kMaxDevices = 64;
struct DeviceMemo {
    std::atomic<uint64_t> word[kMaxDevices];
    // ordinal of the current device, or -1 (then nothing is remembered and the runtime is asked every time)
    static int device() {
        int d = -1;
        return hipGetDevice(&d) == hipSuccess && d >= 0 && d < kMaxDevices ? d : -1;
    }
    uint64_t get(int d) const { return d < 0 ? 0 : word[d].load(std::memory_order_acquire); }
    void set(int d, uint64_t x) { if (d >= 0) word[d].store(x, std::memory_order_release); }
};

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? BIMASK_OK : BIMASK_ERR_HIP;
}

// Top-N of M by key; the lower position wins among equal keys.  Returns the
// selected positions as a bit set (exactly N bits).
template <int M>
__device__ __forceinline__ uint32_t select_top_n(const uint32_t (&key)[M], int N) {
    int rank[M];
#pragma unroll
    for (int m = 0; m < M; ++m) rank[m] = 0;
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = a + 1; b < M; ++b) {
            const int a_first = key[a] >= key[b];   // a has the lower index: it wins ties
            rank[b] += a_first;
            rank[a] += 1 - a_first;
        }
    uint32_t sel = 0;
#pragma unroll
    for (int m = 0; m < M; ++m) sel |= (rank[m] < N ? 1u : 0u) << m;
    return sel;
}

// Slot positions of a group given its mask bits: the ones (at most N are used, lowest
// first) completed with the lowest-index zeros up to N positions.
template <int M>
__device__ __forceinline__ uint32_t complete_slots(uint32_t bits, int N) {
    uint32_t sel = 0;
    int n = 0;
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const bool take = ((bits >> m) & 1u) && n < N;
        sel |= (take ? 1u : 0u) << m;
        n += take;
    }
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const bool take = !((bits >> m) & 1u) && n < N;
        sel |= (take ? 1u : 0u) << m;
        n += take;
    }
    return sel;
}

// Fragment-major layout of a 2:4 compressed operand (see include/bimask.h): element
// offsets of slot s / index word of group g of logical row r; ks = padded cols / 128.
__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
__host__ __device__ inline int64_t tiled_val_off(int64_t r, int64_t s, int64_t ks) {
    const int64_t st = s >> 6;
    const int c = static_cast<int>(s & 63);
    return ((((r >> 5) * ks + st) * 4 + ((c & 31) >> 3)) * 64 + (r & 31) + 32 * (c >> 5)) * 8 + (c & 7);
}
__host__ __device__ inline int64_t tiled_idx_word(int64_t r, int64_t g, int64_t ks) {
    const int64_t st = g >> 5;
    const int q = static_cast<int>(g & 31);
    return (((r >> 5) * ks + st) * 64 + (r & 31) + 32 * (q >> 4)) * 2 + ((q >> 3) & 1);
}

// Fragment-major layout of a DENSE masked operand (ratios with N > 2; see include/bimask.h): element offset of
// entry (r, k); ks = padded cols / 128.  The 8 entries k .. k+7 (k a multiple of 8) are contiguous, and the 64
// granules lane l = r % 32 + 32 ((k % 16) / 8) of one 32x32x16 matrix instruction's A operand follow each other.
__host__ __device__ inline int64_t tiled_dense_off(int64_t r, int64_t k, int64_t ks) {
    const int64_t st = k >> 7;
    const int kk = static_cast<int>(k & 127);
    return ((((((r >> 5) * ks + st) * 4 + ((kk & 63) >> 4)) * 2 + (kk >> 6)) * 64 + (r & 31) + 32 * ((kk & 15) >> 3)) << 3) + (kk & 7);
}

// Two fp32 accumulators -> packed bf16 (round to nearest even) with the gfx950 conversion
// instruction; the low half holds `lo`.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}

// launchers implemented in the .hip files -------------------------------------------
int launch_forward(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                   const uint32_t* mask_in, uint32_t* B_bits, void* values, uint32_t* index,
                   bool want_values, hipStream_t s);
int launch_backward(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                    const uint32_t* B_bits, const uint32_t* Bbar_in, const int32_t* perm,
                    uint32_t* Bbar_bits, void* values, uint32_t* index, bool want_values, hipStream_t s);

struct PermPlan {
    int chunks;          // 16-byte chunks per row and slice: 8 (1024 columns) or 32 (4096 columns)
    int nslices;         // column slices
    int nseg;            // row-block ranges per (slice, candidate)
    int sps;             // wavefront steps (8 row blocks each) per range
    int ntiles;          // nslices * nseg partial scores per candidate
    size_t ws_bytes;     // partial-score scratch
};
PermPlan plan_perm_search(int64_t I, int64_t J, int K, int M);
int launch_perm_search(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                       int32_t* scores, int32_t* best, int32_t* best_perm, void* ws, hipStream_t s);

// the same search with its partial scores in the library's static device array (no workspace argument)
size_t perm_search_static_capacity();
int launch_perm_search_static(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                              int32_t* scores, int32_t* best, int32_t* best_perm, hipStream_t s);

// grouped variants: n independent layers, few launches (see include/bimask.h); the per-layer argument
// tables travel in the kernel arguments (kept below 4 KB): this many layers per launch for an entry of
// `entry_bytes` plus a 4-byte first-workgroup index
constexpr int group_capacity(size_t entry_bytes) { return static_cast<int>((3840 - 16) / (entry_bytes + 4)); }
int launch_forward_group(const bimask_group_layer* L, int n, int dtype, int N, int M, hipStream_t s);
int launch_perm_search_group(const bimask_group_layer* L, int n, int N, int M, int K, hipStream_t s);
int launch_backward_group(const bimask_group_layer* L, int n, int dtype, int N, int M, hipStream_t s);

int launch_gather_cols(const void* dY, int64_t T, int64_t ld, const int32_t* perm, int64_t I, int dtype,
                       void* out, hipStream_t s);
// C[t][a] = sum_k Bm[t][k] * A[a][k];  A sparse 2:4 (values + index) or dense.
int launch_gemm(const void* A_values, const uint32_t* A_index, int64_t Adim, int64_t K, bool sparse24,
                const void* Bm, int64_t T, int64_t ldb, void* C, int64_t ldc, int dtype, hipStream_t s);

// workgroup tile (weight rows x tokens) of the streaming 2:4 kernel
enum class Sp24Tile { k256x64, k128x64, k256x128, k64x64 };
int launch_gemm_sp24(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bm, int64_t T,
                     int64_t ldb, void* C, int64_t ldc, Sp24Tile tile, hipStream_t s);

// dense masked weights (N > 2) on the streaming kernel; BIMASK_ERR_UNSUPPORTED for unaligned operands
int launch_gemm_dense_frag(const void* A, int64_t Adim, int64_t K, const void* Bm, int64_t T, int64_t ldb, void* C,
                           int64_t ldc, hipStream_t s);

// large problems (thousands of weight rows and tokens): 512 x 128 tiles; BIMASK_ERR_UNSUPPORTED otherwise
bool gemm_sp24_big_shape(int64_t Adim, int64_t K, int64_t T);
int launch_gemm_sp24_big(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bm, int64_t T,
                         int64_t ldb, void* C, int64_t ldc, hipStream_t s);

int launch_gemm_sp24_resident(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc,
                              int64_t ldb, const int32_t* perm, int64_t T, void* C, int64_t ldc,
                              hipStream_t s);
// wavefront-private variant for narrow weights (Adim <= 256 with K <= 128, Adim <= 64 with K <= 256); BIMASK_ERR_UNSUPPORTED otherwise
int launch_gemm_sp24_narrow(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc,
                            int64_t ldb, const int32_t* perm, int64_t T, void* C, int64_t ldc, hipStream_t s);
// backward GEMM with whole rows of g(Y) resident in LDS (512 < K <= 2048, Adim <= 512): gather fused;
// BIMASK_ERR_UNSUPPORTED otherwise
// (dense: the weight operand is the dense masked matrix of a ratio with N > 2, meta unused)
int launch_gemm_sp24_rowres(const void* A, const uint32_t* meta, int64_t Adim, int64_t K, const void* Bsrc,
                            int64_t ldb, const int32_t* perm, int64_t T, void* C, int64_t ldc, hipStream_t s,
                            bool dense = false);
// true when the backward GEMM needs the gathered copy of g(Y) in the workspace
// Debug helper: one flag per candidate, 1 = a permutation of 0 .. I-1 (bitmap of I bits in LDS).
constexpr int64_t kCheckPermsMaxRows = 1 << 20;
int launch_check_perms(const int32_t* perms, int K, int64_t I, int32_t* ok, hipStream_t s);
// Refinement of a permutation by proposed exchanges; the permutation lives in LDS.
constexpr int64_t kRefineMaxRows = 32768;
int launch_perm_refine(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perm_in,
                       const int32_t* swaps, int64_t S, int32_t* perm_out, int32_t* result, hipStream_t s);
int launch_perm_refine_group(const bimask_group_layer* L, int n, int N, int M, hipStream_t s);
bool gemm_bwd_needs_gather(int64_t I, int64_t J, int dtype, int N, int M);
// Shapes (output rows Adim, contraction K) the row-resident backward kernel takes.
bool gemm_sp24_rowres_shape(int64_t Adim, int64_t K);
// The same for dense masked weights (N > 2), which have no other fused path: 128 < K <= 2048, Adim <= min(K, 512).
bool gemm_dense_rowres_shape(int64_t Adim, int64_t K);

}  // namespace bimask
