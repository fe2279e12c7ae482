// Host sanitizer driver for the argument validation of include/bimask.h (test infrastructure).
//
// Built by tests/test_sanitizers.py against a build of the library whose host code is compiled with
// -fsanitize=address,undefined, and run as a plain executable on a machine without a GPU: every call
// below must be rejected on the host, with the stated status, before any HIP call is made.  The
// pointers handed in are small host allocations that validation must never dereference (a read or
// write through them past their 16 bytes would be reported).  Exit status 0 = clean.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "bimask.h"

static int failures = 0;
#define EXPECT(call, want)                                                                         \
    do {                                                                                           \
        const int got_ = (call);                                                                   \
        if (got_ != (want)) { std::fprintf(stderr, "line %d: %s -> %d, want %d\n", __LINE__, #call, got_, (want)); ++failures; } \
    } while (0)

int main() {
    alignas(16) static unsigned char buf[16];
    void* F = buf;                                  // aligned, never dereferenced
    uint32_t* U = reinterpret_cast<uint32_t*>(buf);
    int32_t* P = reinterpret_cast<int32_t*>(buf);
    void* odd = buf + 1;
    const int BF = BIMASK_BF16, F32 = BIMASK_F32;

    EXPECT(bimask_forward_mask(nullptr, 64, 128, 128, BF, 2, 4, U, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_forward_mask(F, 64, 128, 128, BF, 2, 4, nullptr, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_forward_mask(F, 64, 130, 130, BF, 2, 4, U, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_forward_mask(F, 62, 128, 128, BF, 2, 4, U, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_forward_mask(F, 64, 128, 100, BF, 2, 4, U, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_forward_mask(F, 0, 128, 128, BF, 2, 4, U, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_forward_mask(F, int64_t(1) << 40, 128, 128, BF, 2, 4, U, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_forward_mask(F, 64, 128, 128, BF, 4, 4, U, nullptr), BIMASK_ERR_NM);
    EXPECT(bimask_forward_mask(F, 60, 120, 120, BF, 2, 5, U, nullptr), BIMASK_ERR_NM);
    EXPECT(bimask_forward_mask(F, 64, 128, 128, 7, 2, 4, U, nullptr), BIMASK_ERR_DTYPE);
    EXPECT(bimask_forward_mask(odd, 64, 128, 128, BF, 2, 4, U, nullptr), BIMASK_ERR_ALIGN);
    EXPECT(bimask_forward_mask_compress(F, 64, 128, 128, BF, 2, 4, U, nullptr, U, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_forward_mask_compress(F, 64, 128, 128, BF, 2, 4, U, F, nullptr, nullptr), BIMASK_ERR_NULL);

    EXPECT(bimask_perm_search(U, 64, 128, 2, 4, nullptr, 4, P, P, nullptr, F, 1 << 20, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_perm_search(U, 64, 128, 2, 4, P, 0, P, P, nullptr, F, 1 << 20, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_perm_search(U, 64, 128, 2, 4, P, 4, P, P, nullptr, nullptr, 0, nullptr), BIMASK_ERR_WORKSPACE);
    EXPECT(bimask_perm_search(U, 64, 128, 2, 4, P, 4, P, P, nullptr, F, 8, nullptr), BIMASK_ERR_WORKSPACE);
    EXPECT(bimask_perm_search(U, 64, 128, 2, 4, reinterpret_cast<int32_t*>(buf + 4), 4, P, P, nullptr, F, 1 << 20, nullptr), BIMASK_ERR_ALIGN);
    EXPECT(bimask_perm_search(U, int64_t(1) << 30, int64_t(1) << 20, 2, 4, P, 4, P, P, nullptr, F, 1 << 20, nullptr), BIMASK_ERR_SHAPE);

    EXPECT(bimask_perm_search_static(U, 64, 128, 2, 4, nullptr, 4, P, P, nullptr, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_perm_search_static(U, 64, 128, 2, 5, P, 4, P, P, nullptr, nullptr), BIMASK_ERR_NM);
    EXPECT(bimask_perm_search_static(U, 8, int64_t(1) << 22, 2, 4, P, 100, P, P, nullptr, nullptr), BIMASK_ERR_WORKSPACE);

    EXPECT(bimask_check_perms(nullptr, 4, 64, P, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_check_perms(P, 0, 64, P, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_check_perms(P, 4, (1 << 20) + 1, P, nullptr), BIMASK_ERR_UNSUPPORTED);

    EXPECT(bimask_perm_refine(nullptr, 64, 128, 2, 4, nullptr, P, 10, P, P, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_perm_refine(U, 64, 128, 2, 4, nullptr, nullptr, 10, P, P, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_perm_refine(U, 62, 128, 2, 4, nullptr, P, 10, P, P, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_perm_refine(U, 64, 128, 2, 4, nullptr, P, -1, P, P, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_perm_refine(U, 32772, 128, 2, 4, nullptr, P, 10, P, P, nullptr), BIMASK_ERR_UNSUPPORTED);

    EXPECT(bimask_backward_mask(F, 64, 128, 128, F32, 2, 4, nullptr, nullptr, U, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_backward_mask_compress(F, 64, 128, 128, F32, 2, 4, U, nullptr, U, nullptr, U, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_compress_nm(F, 64, 128, 128, BF, 2, 4, U, nullptr, 2, F, U, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_compress_nm(F, 64, 128, 128, BF, 2, 4, U, P, 0, F, U, nullptr), BIMASK_ERR_UNSUPPORTED);

    EXPECT(bimask_sparse_gemm_fwd(nullptr, 32, 128, F, U, 64, 128, BF, 2, 4, F, 64, nullptr, 0, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_sparse_gemm_fwd(F, 32, 100, F, U, 64, 128, BF, 2, 4, F, 64, nullptr, 0, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_sparse_gemm_fwd(F, 32, 129, F, U, 64, 128, BF, 2, 4, F, 64, nullptr, 0, nullptr), BIMASK_ERR_ALIGN);
    EXPECT(bimask_sparse_gemm_bwd(F, 32, 4096, P, F, U, 4096, 128, BF, 2, 4, F, 128, nullptr, 0, nullptr), BIMASK_ERR_WORKSPACE);
    EXPECT(bimask_sparse_gemm_bwd(F, 32, 1028, P, F, U, 1024, 128, BF, 2, 4, F, 128, nullptr, 0, nullptr), BIMASK_ERR_ALIGN);

    // grouped calls: a host table of descriptors is read during the call; the second layer is the bad one
    std::vector<bimask_group_layer> L(2);
    for (auto& g : L) {
        std::memset(&g, 0, sizeof(g));
        g.W = F; g.I = 64; g.J = 128; g.ldw = 128; g.B_bits = U; g.Wf_values = F; g.Wf_index = U; g.perms = P;
        g.scores = P; g.best = P; g.best_perm = P; g.workspace = F; g.workspace_bytes = 1 << 20; g.Bbar_bits = U;
        g.Wb_values = F; g.Wb_index = U; g.swaps = P; g.n_swaps = 10; g.refine_result = P;
    }
    EXPECT(bimask_forward_mask_compress_group(nullptr, 2, BF, 2, 4, nullptr), BIMASK_ERR_NULL);
    EXPECT(bimask_forward_mask_compress_group(L.data(), 0, BF, 2, 4, nullptr), BIMASK_ERR_SHAPE);
    L[1].J = 130; L[1].ldw = 130;
    EXPECT(bimask_forward_mask_compress_group(L.data(), 2, BF, 2, 4, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_backward_mask_compress_group(L.data(), 2, BF, 2, 4, nullptr), BIMASK_ERR_SHAPE);
    EXPECT(bimask_perm_search_group(L.data(), 2, 2, 4, 100, nullptr), BIMASK_ERR_SHAPE);
    L[1].J = 128; L[1].ldw = 128; L[1].workspace_bytes = 8;
    EXPECT(bimask_perm_search_group(L.data(), 2, 2, 4, 100, nullptr), BIMASK_ERR_WORKSPACE);
    L[1].n_swaps = -1;
    EXPECT(bimask_perm_refine_group(L.data(), 2, 2, 4, nullptr), BIMASK_ERR_SHAPE);

    // size helpers and strings
    if (bimask_operand_elems(64, 128, 2, 4) != 64 * 64 || bimask_operand_index_words(64, 128, 2, 4) != 64 * 4) ++failures;
    if (bimask_operand_elems(0, 128, 2, 4) != 0 || bimask_workspace_bytes(99, 64, 128, 32, 4, BF, 2, 4) != 0) ++failures;
    for (int s = -1; s < 12; ++s)
        if (!bimask_status_string(s) || !bimask_status_string(s)[0]) ++failures;

    if (failures) { std::fprintf(stderr, "%d failures\n", failures); return 1; }
    std::puts("argument-validation sanitizer driver: clean");
    return 0;
}
