// extern "C" boundary of the Bi-Mask library: argument validation on the host, then
// kernel launches on the caller's stream.  See include/bimask.h for the contract.
#include "common.hpp"
#include <cstdlib>

using namespace bimask;

namespace {

int check_nm(int N, int M) {
    if (!(M == 4 || M == 8 || M == 16)) return BIMASK_ERR_NM;
    if (N < 1 || N >= M) return BIMASK_ERR_NM;
    return BIMASK_OK;
}

int check_dtype(int dtype) { return (dtype == BIMASK_F32 || dtype == BIMASK_BF16) ? BIMASK_OK : BIMASK_ERR_DTYPE; }

size_t esize(int dtype) { return dtype == BIMASK_BF16 ? 2 : 4; }

int check_matrix(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M) {
    if (!W) return BIMASK_ERR_NULL;
    if (int rc = check_dtype(dtype)) return rc;
    if (int rc = check_nm(N, M)) return rc;
    if (I <= 0 || J <= 0 || ldw < J) return BIMASK_ERR_SHAPE;
    if (I % M != 0 || J % M != 0) return BIMASK_ERR_SHAPE;
    if (I > 0x7FFFFFFFll || J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(W) % esize(dtype)) return BIMASK_ERR_ALIGN;
    return BIMASK_OK;
}

inline hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// Operand checks shared by the two GEMM entry points.
int check_gemm(const void* act, int64_t T, int64_t ldact, int64_t kdim, const void* values, const uint32_t* index,
               int64_t I, int64_t J, int dtype, int N, int M, const void* out, int64_t ldout, int64_t outdim) {
    if (!act || !values || !out) return BIMASK_ERR_NULL;
    if (int rc = check_dtype(dtype)) return rc;
    if (int rc = check_nm(N, M)) return rc;
    if (T <= 0 || I <= 0 || J <= 0 || I % M || J % M || ldact < kdim || ldout < outdim) return BIMASK_ERR_SHAPE;
    if (uses_sp24(N, M) && !index) return BIMASK_ERR_NULL;
    if (!aligned16(values) || (uses_sp24(N, M) && !aligned16(index))) return BIMASK_ERR_ALIGN;
    if (dtype == BIMASK_BF16) {
        // rows are read in 4-byte units at least
        if (ldact % 2 || ldout % 2) return BIMASK_ERR_ALIGN;
        if (!aligned4(act) || !aligned4(values) || !aligned4(out)) return BIMASK_ERR_ALIGN;
    } else {
        if (!aligned4(act) || !aligned4(values) || !aligned4(out)) return BIMASK_ERR_ALIGN;
    }
    return BIMASK_OK;
}

}  // namespace

extern "C" {

int bimask_forward_mask(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                        uint32_t* B_bits, void* stream) {
    if (int rc = check_matrix(W, I, J, ldw, dtype, N, M)) return rc;
    if (!B_bits) return BIMASK_ERR_NULL;
    return launch_forward(W, I, J, ldw, dtype, N, M, nullptr, B_bits, nullptr, nullptr, false, as_stream(stream));
}

int bimask_forward_mask_compress(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                                 uint32_t* B_bits, void* values, uint32_t* index, void* stream) {
    if (int rc = check_matrix(W, I, J, ldw, dtype, N, M)) return rc;
    if (!B_bits || !values) return BIMASK_ERR_NULL;
    if (uses_sp24(N, M) && !index) return BIMASK_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(values) % esize(dtype)) return BIMASK_ERR_ALIGN;
    if (!aligned16(values) || (uses_sp24(N, M) && !aligned16(index))) return BIMASK_ERR_ALIGN;
    return launch_forward(W, I, J, ldw, dtype, N, M, nullptr, B_bits, values, index, true, as_stream(stream));
}

int bimask_perm_search(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                       int32_t* scores, int32_t* best, int32_t* best_perm, void* workspace, size_t workspace_bytes,
                       void* stream) {
    if (!B_bits || !perms || !scores || !best) return BIMASK_ERR_NULL;
    if (int rc = check_nm(N, M)) return rc;
    if (I <= 0 || J <= 0 || K <= 0 || I % M || J % M) return BIMASK_ERR_SHAPE;
    if (I > 0x7FFFFFFFll || J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
    if ((I / M) * J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;       // a score must fit int32
    if (!aligned16(perms)) return BIMASK_ERR_ALIGN;
    const PermPlan pl = plan_perm_search(I, J, K, M);
    if (!workspace || workspace_bytes < pl.ws_bytes) return BIMASK_ERR_WORKSPACE;
    return launch_perm_search(B_bits, I, J, N, M, perms, K, scores, best, best_perm, workspace, as_stream(stream));
}

int bimask_perm_search_static(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perms, int K,
                              int32_t* scores, int32_t* best, int32_t* best_perm, void* stream) {
    if (!B_bits || !perms || !scores || !best) return BIMASK_ERR_NULL;
    if (int rc = check_nm(N, M)) return rc;
    if (I <= 0 || J <= 0 || K <= 0 || I % M || J % M) return BIMASK_ERR_SHAPE;
    if (I > 0x7FFFFFFFll || J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
    if ((I / M) * J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;       // a score must fit int32
    if (!aligned16(perms)) return BIMASK_ERR_ALIGN;
    return launch_perm_search_static(B_bits, I, J, N, M, perms, K, scores, best, best_perm, as_stream(stream));
}

int bimask_check_perms(const int32_t* perms, int K, int64_t I, int32_t* ok, void* stream) {
    if (!perms || !ok) return BIMASK_ERR_NULL;
    if (K <= 0 || I <= 0) return BIMASK_ERR_SHAPE;
    if (!aligned4(perms) || !aligned4(ok)) return BIMASK_ERR_ALIGN;
    return launch_check_perms(perms, K, I, ok, as_stream(stream));
}

int bimask_perm_refine(const uint32_t* B_bits, int64_t I, int64_t J, int N, int M, const int32_t* perm_in,
                       const int32_t* swaps, int64_t S, int32_t* perm_out, int32_t* result, void* stream) {
    if (!B_bits || !perm_out || !result || (S > 0 && !swaps)) return BIMASK_ERR_NULL;
    if (int rc = check_nm(N, M)) return rc;
    if (I <= 0 || J <= 0 || S < 0 || I % M || J % M) return BIMASK_ERR_SHAPE;
    if (I > 0x7FFFFFFFll || J > 0x7FFFFFFFll || (I / M) * J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
    if (!aligned4(perm_in) || !aligned4(swaps) || !aligned4(perm_out) || !aligned4(result)) return BIMASK_ERR_ALIGN;
    return launch_perm_refine(B_bits, I, J, N, M, perm_in, swaps, S, perm_out, result, as_stream(stream));
}

int bimask_backward_mask(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                         const uint32_t* B_bits, const int32_t* perm, uint32_t* Bbar_bits, void* stream) {
    if (int rc = check_matrix(W, I, J, ldw, dtype, N, M)) return rc;
    if (!B_bits || !Bbar_bits) return BIMASK_ERR_NULL;
    return launch_backward(W, I, J, ldw, dtype, N, M, B_bits, nullptr, perm, Bbar_bits, nullptr, nullptr, false,
                           as_stream(stream));
}

int bimask_backward_mask_compress(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                                  const uint32_t* B_bits, const int32_t* perm, uint32_t* Bbar_bits, void* values,
                                  uint32_t* index, void* stream) {
    if (int rc = check_matrix(W, I, J, ldw, dtype, N, M)) return rc;
    if (!B_bits || !Bbar_bits || !values) return BIMASK_ERR_NULL;
    if (uses_sp24(N, M) && !index) return BIMASK_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(values) % esize(dtype)) return BIMASK_ERR_ALIGN;
    if (!aligned16(values) || (uses_sp24(N, M) && !aligned16(index))) return BIMASK_ERR_ALIGN;
    return launch_backward(W, I, J, ldw, dtype, N, M, B_bits, nullptr, perm, Bbar_bits, values, index, true,
                           as_stream(stream));
}

int bimask_compress_nm(const void* W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                       const uint32_t* mask_bits, const int32_t* perm, int transposed, void* values,
                       uint32_t* index, void* stream) {
    if (int rc = check_matrix(W, I, J, ldw, dtype, N, M)) return rc;
    if (!mask_bits || !values) return BIMASK_ERR_NULL;
    if (uses_sp24(N, M) && !index) return BIMASK_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(values) % esize(dtype)) return BIMASK_ERR_ALIGN;
    if (!aligned16(values) || (uses_sp24(N, M) && !aligned16(index))) return BIMASK_ERR_ALIGN;
    if (transposed != 0 && transposed != 1) return BIMASK_ERR_SHAPE;
    if (!transposed) {
        if (perm) return BIMASK_ERR_UNSUPPORTED;                     // rows of the forward operand are not permuted
        return launch_forward(W, I, J, ldw, dtype, N, M, mask_bits, nullptr, values, index, true, as_stream(stream));
    }
    return launch_backward(W, I, J, ldw, dtype, N, M, nullptr, mask_bits, perm, nullptr, values, index, true,
                           as_stream(stream));
}

int bimask_forward_mask_compress_group(const bimask_group_layer* layers, int n, int dtype, int N, int M,
                                       void* stream) {
    if (!layers) return BIMASK_ERR_NULL;
    if (n <= 0) return BIMASK_ERR_SHAPE;
    for (int l = 0; l < n; ++l) {
        const bimask_group_layer& a = layers[l];
        if (int rc = check_matrix(a.W, a.I, a.J, a.ldw, dtype, N, M)) return rc;
        if (!a.B_bits || !a.Wf_values) return BIMASK_ERR_NULL;
        if (uses_sp24(N, M) && !a.Wf_index) return BIMASK_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(a.Wf_values) % esize(dtype)) return BIMASK_ERR_ALIGN;
        if (!aligned16(a.Wf_values) || (uses_sp24(N, M) && !aligned16(a.Wf_index))) return BIMASK_ERR_ALIGN;
    }
    return launch_forward_group(layers, n, dtype, N, M, as_stream(stream));
}

int bimask_perm_search_group(const bimask_group_layer* layers, int n, int N, int M, int K, void* stream) {
    if (!layers) return BIMASK_ERR_NULL;
    if (n <= 0 || K <= 0) return BIMASK_ERR_SHAPE;
    if (int rc = check_nm(N, M)) return rc;
    for (int l = 0; l < n; ++l) {
        const bimask_group_layer& a = layers[l];
        if (!a.B_bits || !a.perms || !a.scores || !a.best) return BIMASK_ERR_NULL;
        if (a.I <= 0 || a.J <= 0 || a.I % M || a.J % M) return BIMASK_ERR_SHAPE;
        if (a.I > 0x7FFFFFFFll || a.J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
        if ((a.I / M) * a.J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
        if (!aligned16(a.perms)) return BIMASK_ERR_ALIGN;
        if (!a.workspace || a.workspace_bytes < plan_perm_search(a.I, a.J, K, M).ws_bytes) return BIMASK_ERR_WORKSPACE;
    }
    return launch_perm_search_group(layers, n, N, M, K, as_stream(stream));
}

int bimask_perm_refine_group(const bimask_group_layer* layers, int n, int N, int M, void* stream) {
    if (!layers) return BIMASK_ERR_NULL;
    if (n <= 0) return BIMASK_ERR_SHAPE;
    if (int rc = check_nm(N, M)) return rc;
    for (int l = 0; l < n; ++l) {
        const bimask_group_layer& a = layers[l];
        if (!a.B_bits || !a.best_perm || !a.refine_result || (a.n_swaps > 0 && !a.swaps)) return BIMASK_ERR_NULL;
        if (a.I <= 0 || a.J <= 0 || a.n_swaps < 0 || a.I % M || a.J % M) return BIMASK_ERR_SHAPE;
        if (a.I > 0x7FFFFFFFll || a.J > 0x7FFFFFFFll || (a.I / M) * a.J > 0x7FFFFFFFll) return BIMASK_ERR_SHAPE;
        if (!aligned4(a.best_perm) || !aligned4(a.swaps) || !aligned4(a.refine_result)) return BIMASK_ERR_ALIGN;
    }
    return launch_perm_refine_group(layers, n, N, M, as_stream(stream));
}

int bimask_backward_mask_compress_group(const bimask_group_layer* layers, int n, int dtype, int N, int M,
                                        void* stream) {
    if (!layers) return BIMASK_ERR_NULL;
    if (n <= 0) return BIMASK_ERR_SHAPE;
    for (int l = 0; l < n; ++l) {
        const bimask_group_layer& a = layers[l];
        if (int rc = check_matrix(a.W, a.I, a.J, a.ldw, dtype, N, M)) return rc;
        if (!a.B_bits || !a.Bbar_bits || !a.Wb_values) return BIMASK_ERR_NULL;
        if (uses_sp24(N, M) && !a.Wb_index) return BIMASK_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(a.Wb_values) % esize(dtype)) return BIMASK_ERR_ALIGN;
        if (!aligned16(a.Wb_values) || (uses_sp24(N, M) && !aligned16(a.Wb_index))) return BIMASK_ERR_ALIGN;
    }
    return launch_backward_group(layers, n, dtype, N, M, as_stream(stream));
}

int bimask_sparse_gemm_fwd(const void* X, int64_t T, int64_t ldx, const void* Wf_values, const uint32_t* Wf_index,
                           int64_t I, int64_t J, int dtype, int N, int M, void* Y, int64_t ldy, void* workspace,
                           size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (int rc = check_gemm(X, T, ldx, J, Wf_values, Wf_index, I, J, dtype, N, M, Y, ldy, I)) return rc;
    const bool sp = uses_sp24(N, M);
    return launch_gemm(Wf_values, Wf_index, I, J, sp, X, T, ldx, Y, ldy, dtype, as_stream(stream));
}

int bimask_sparse_gemm_bwd(const void* dY, int64_t T, int64_t lddy, const int32_t* perm, const void* Wb_values,
                           const uint32_t* Wb_index, int64_t I, int64_t J, int dtype, int N, int M, void* dX,
                           int64_t lddx, void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_gemm(dY, T, lddy, I, Wb_values, Wb_index, I, J, dtype, N, M, dX, lddx, J)) return rc;
    const bool sp = uses_sp24(N, M);
    const void* act = dY;
    int64_t ldact = lddy;
    if (perm && !gemm_bwd_needs_gather(I, J, dtype, N, M)) {
        if (sp && I <= 512)      // short contraction: the column gather is fused into the GEMM's token-tile load
            return launch_gemm_sp24_resident(Wb_values, Wb_index, J, I, dY, lddy, perm, T, dX, lddx, as_stream(stream));
        // rows of g(Y) that fit LDS whole: gather fused as well, rows move in 16-byte pieces
        if (!aligned16(dY) || !aligned16(dX) || lddy % 8 || lddx % 8) return BIMASK_ERR_ALIGN;
        return launch_gemm_sp24_rowres(Wb_values, Wb_index, J, I, dY, lddy, perm, T, dX, lddx, as_stream(stream), !sp);
    }
    if (perm) {
        const size_t need = bimask_workspace_bytes(BIMASK_WS_GEMM_BWD, I, J, T, 0, dtype, N, M);
        if (!workspace || workspace_bytes < need) return BIMASK_ERR_WORKSPACE;
        if (!aligned16(workspace)) return BIMASK_ERR_ALIGN;
        if (int rc = launch_gather_cols(dY, T, lddy, perm, I, dtype, workspace, as_stream(stream))) return rc;
        act = workspace;
        ldact = I;
    }
    return launch_gemm(Wb_values, Wb_index, J, I, sp, act, T, ldact, dX, lddx, dtype, as_stream(stream));
}

int64_t bimask_operand_elems(int64_t rows, int64_t cols, int N, int M) {
    if (rows <= 0 || cols <= 0) return 0;
    if (uses_sp24(N, M)) return round_up(rows, 32) * (round_up(cols, 128) / 2);
    return round_up(rows, 32) * round_up(cols, 128);
}

int64_t bimask_operand_index_words(int64_t rows, int64_t cols, int N, int M) {
    if (rows <= 0 || cols <= 0 || !uses_sp24(N, M)) return 0;
    return round_up(rows, 32) * (round_up(cols, 128) / 32);
}

size_t bimask_workspace_bytes(int kind, int64_t I, int64_t J, int64_t T, int K, int dtype, int N, int M) {
    (void)N; (void)M;
    if (I <= 0 || J <= 0) return 0;
    switch (kind) {
        case BIMASK_WS_PERM_SEARCH: {
            if (K <= 0) return 0;
            if (M != 4 && M != 8 && M != 16) return 0;
            return plan_perm_search(I, J, K, M).ws_bytes;
        }
        case BIMASK_WS_GEMM_FWD:
            return 0;
        case BIMASK_WS_GEMM_BWD:
            if (!gemm_bwd_needs_gather(I, J, dtype, N, M)) return 0;
            return T > 0 ? static_cast<size_t>(T) * static_cast<size_t>(I) * esize(dtype) : 0;
        default:
            return 0;
    }
}

const char* bimask_status_string(int status) {
    switch (status) {
        case BIMASK_OK: return "ok";
        case BIMASK_ERR_NULL: return "a required pointer is NULL";
        case BIMASK_ERR_SHAPE: return "bad shape: sizes must be positive, I and J multiples of M, ld >= columns";
        case BIMASK_ERR_NM: return "bad N:M: M must be 4, 8 or 16 and 1 <= N < M";
        case BIMASK_ERR_DTYPE: return "dtype must be BIMASK_F32 or BIMASK_BF16";
        case BIMASK_ERR_UNSUPPORTED: return "combination not supported by this build";
        case BIMASK_ERR_WORKSPACE: return "workspace missing or too small";
        case BIMASK_ERR_ALIGN: return "pointer or leading dimension breaks the stated alignment";
        case BIMASK_ERR_HIP: return "HIP runtime error at kernel launch";
        default: return "unknown status";
    }
}

}  // extern "C"
