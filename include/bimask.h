/*
 * bimask.h -- C ABI of the Bi-Mask N:M sparse-training hot path for AMD MI355X (gfx950).
 *
 * Method: "Bi-directional Masks for Efficient N:M Sparse Training" (arXiv 2302.06058).
 * One training step of one linear / conv-as-GEMM layer (Alg. 1) maps onto the calls
 * below in this order:
 *
 *     bimask_forward_mask      B     = top-N-of-M along the rows of W            Eq. (4), Eq. (2)
 *     bimask_compress_nm       W_f   = compressed (B .* W)                       operand of Eq. (3)
 *     bimask_sparse_gemm_fwd   Y     = X * (B .* W)^T                            Eq. (3)
 *     bimask_perm_search       P     = best of K row permutations               Sec. 3.3, Alg. 1
 *     bimask_backward_mask     Bbar  = top-N-of-M along the columns of
 *                                      (B .* W)[P,:], AND-ed with B[P,:]         Eq. (11) / Eq. (9)
 *     bimask_compress_nm       W_b   = compressed (Bbar .* W[P,:])^T             operand of Eq. (10)
 *     bimask_sparse_gemm_bwd   dX    = dY[:,P] * (Bbar .* W[P,:])                Eq. (10) / Eq. (8)
 *
 * The weight gradient dW = dY^T * X stays dense (straight-through estimator, Sec. 3.1)
 * and is not part of this library.
 *
 * Shapes and layouts (all row-major, zero-based; "ld" = leading dimension in elements):
 *     W      I x J   weights, I = out features, J = in features          (Sec. 3.1)
 *     X      T x J   activations, T = tokens; the paper writes X as J x T and Y = W * X
 *     Y, dY  T x I   output and its gradient g(Y)
 *     dX     T x J   the approximate input gradient g-bar(X)
 *     B      I x J   forward mask bits, N:M along each row               (Eq. 2)
 *     Bbar   I x J   backward mask bits, N:M along each column, rows in PERMUTED order:
 *                    row r of Bbar belongs to row P[r] of W              (Eq. 7, Eq. 11)
 *     P      I       row permutation in gather form: (W[P,:])[r] = W[P[r]]
 *
 * Bit matrices: ceil(cols/32) uint32 words per row; entry j is bit (j % 32) of word
 * (j / 32); unused high bits of the last word of a row are written as zero.
 *
 * Compressed N:M operand (this library's format; the paper only names the sparse
 * tensor core as consumer).  Let the operand have `rows` x `cols` logical entries:
 *   transposed = 0: rows = I, cols = J (groups of M along J);
 *   transposed = 1: rows = J, cols = I (groups of M along the permuted row index r).
 *   for N <= 2 (2:4, 1:4, 2:8, 1:8, 2:16, 1:16): the 2-of-4 format of the 32x32x32 sparse
 *   matrix instruction, in a "fragment-major" layout in which one wavefront fetches its
 *   whole A operand with contiguous 16-byte lanes.  M is a multiple of 4, so a mask with at
 *   most N <= 2 ones per group of M holds at most two ones in every aligned group of 4
 *   positions; "group" below is such a group of 4, whatever M is.
 *   Rp = rows rounded up to 32, Cp = cols rounded up to 128, KS = Cp/128.
 *     Logical content per row: slot s = 2g + n (n = 0, 1) of group g holds the n-th slot
 *     value of that group, slots in ascending position order; the group's index nibble is
 *     p0 | (p1 << 2), p0 < p1.  The slot positions are the mask's ones; a group whose
 *     mask holds fewer than two ones is completed with its lowest-index zero positions,
 *     which carry value 0.  Rows >= rows and columns >= cols are zero padding.
 *     values  Rp * Cp/2 elements.  Slot s of row r: with st = s / 64, c = s % 64,
 *             element (((r/32 * KS + st) * 4 + (c%32)/8) * 64 + r%32 + 32*(c/32)) * 8 + c%8.
 *     index   Rp * Cp/32 uint32.  Group g of row r: with st = g / 32, q = g % 32, nibble
 *             q%8 (bits [4(q%8)+3 : 4(q%8)]) of word
 *             ((r/32 * KS + st) * 64 + r%32 + 32*(q/16)) * 2 + (q/8)%2.
 *     Both buffers must be 16-byte aligned.
 *   for N > 2 (4:8, ...): values is the dense masked matrix (zeros where the mask is 0), also
 *     fragment-major, for the dense 32x32x16 matrix instruction; index is not written (may be NULL).
 *     Rp * Cp elements; entry (r, k): with st = k / 128, kk = k % 128, element
 *     ((((( r/32 * KS + st) * 4 + (kk%64)/16) * 2 + kk/64) * 64 + r%32 + 32*((kk%16)/8)) * 8 + kk%8.
 *     Rows >= rows and columns >= cols are zero padding.  values must be 16-byte aligned.
 *   bimask_operand_elems / bimask_operand_index_words give the buffer sizes.
 *
 * Conventions:
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates
 *     nothing, keeps no device state between calls (on the host it only remembers, per device
 *     ordinal, answers of the runtime's occupancy query and which kernels had their LDS limit raised:
 *     several devices may be driven from one process), and never synchronises: every call only
 *     enqueues work on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Return value: BIMASK_OK or a bimask_status error.  Argument errors are detected on
 *     the host before anything is launched and leave all outputs untouched.  Nothing
 *     aborts or throws across this boundary.
 *   - I and J must be multiples of M; M is 4, 8 or 16; 1 <= N < M.  Callers pad ragged
 *     shapes with zero columns (a zero never displaces a real weight because the lowest
 *     index wins ties and padding sits at the highest indices).
 *   - Magnitudes are compared on the stored dtype's bit pattern with the sign cleared,
 *     so the order is total: ties keep the lowest index, +0 = -0, and inputs are assumed
 *     finite.  Exactly N entries are kept per forward group.
 *   - Permutations are not validated (each must hold every value of 0..I-1 once).
 */
#ifndef BIMASK_H
#define BIMASK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BIMASK_API __attribute__((visibility("default")))

typedef enum {
    BIMASK_OK = 0,
    BIMASK_ERR_NULL = 1,        /* a required pointer is NULL */
    BIMASK_ERR_SHAPE = 2,       /* size <= 0, I % M, J % M, ld < cols, K <= 0 */
    BIMASK_ERR_NM = 3,          /* M not in {4, 8, 16} or not 1 <= N < M */
    BIMASK_ERR_DTYPE = 4,       /* dtype is neither BIMASK_F32 nor BIMASK_BF16 */
    BIMASK_ERR_UNSUPPORTED = 5, /* a combination this build has no kernel for */
    BIMASK_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than bimask_workspace_bytes says */
    BIMASK_ERR_ALIGN = 7,       /* a pointer or leading dimension breaks a stated alignment */
    BIMASK_ERR_HIP = 8          /* the HIP runtime reported an error at launch */
} bimask_status;

typedef enum { BIMASK_F32 = 0, BIMASK_BF16 = 1 } bimask_dtype;

typedef enum {
    BIMASK_WS_PERM_SEARCH = 0,
    BIMASK_WS_GEMM_FWD = 1,
    BIMASK_WS_GEMM_BWD = 2
} bimask_ws_kind;

/* Forward mask, Eq. (4) under the constraint of Eq. (2): in every group of M consecutive
 * columns of every row keep the N largest magnitudes.
 *   W       in   I x J, leading dimension ldw >= J, dtype `dtype`
 *   B_bits  out  I x ceil(J/32) words                                                  */
BIMASK_API int bimask_forward_mask(const void *W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                        uint32_t *B_bits, void *stream);

/* Forward mask and the compressed forward operand in one pass over W (same results as
 * bimask_forward_mask followed by bimask_compress_nm(transposed = 0)).
 *   values  out  bimask_operand_elems(I, J, N, M) elements
 *   index   out  bimask_operand_index_words(I, J, N, M) words for N <= 2, else ignored      */
BIMASK_API int bimask_forward_mask_compress(const void *W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                                 uint32_t *B_bits, void *values, uint32_t *index, void *stream);

/* Row-permutation search, Sec. 3.3 and Alg. 1: scores[c] = number of (block, column)
 * pairs of (B .* W)[perms[c],:] -- a block being M consecutive permuted rows -- that hold
 * at most N ones of B ("eligible N:M blocks"); best = the lowest c with the highest score.
 *   B_bits     in   forward mask
 *   perms      in   K x I int32, candidate c at perms + c*I; 16-byte aligned
 *   scores     out  K int32 (fits: the maximum is (I/M)*J)
 *   best       out  1 int32
 *   best_perm  out  I int32, a copy of perms[best]; may be NULL
 *   workspace  scratch of bimask_workspace_bytes(BIMASK_WS_PERM_SEARCH, ...) bytes       */
BIMASK_API int bimask_perm_search(const uint32_t *B_bits, int64_t I, int64_t J, int N, int M,
                       const int32_t *perms, int K, int32_t *scores, int32_t *best, int32_t *best_perm,
                       void *workspace, size_t workspace_bytes, void *stream);

/* bimask_perm_search for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the
 * workspace) and bit-identical results; the partial scores live in a static device array of
 * BIMASK_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends).
 *   - bimask_workspace_bytes(BIMASK_WS_PERM_SEARCH, ...) above that size: BIMASK_ERR_WORKSPACE,
 *     nothing is launched.
 *   - Calls no hipMalloc / hipFree and no allocating routine; the array's address is looked up
 *     (hipGetSymbolAddress) at the first call on each device, so make that first call outside a
 *     graph capture.
 *   - All calls on one GPU share the array: two calls that overlap in time on one GPU (different
 *     streams, or graphs replayed concurrently) race.  Calls on one stream are ordered and safe.   */
#define BIMASK_STATIC_SCRATCH_BYTES (1u << 20)
BIMASK_API int bimask_perm_search_static(const uint32_t *B_bits, int64_t I, int64_t J, int N, int M,
                              const int32_t *perms, int K, int32_t *scores, int32_t *best, int32_t *best_perm,
                              void *stream);

/* Backward mask, Eq. (11); with perm = NULL (identity) it is Eq. (9).  For every column
 * and every block of M consecutive permuted rows: rank the magnitudes of
 * (B .* W)[P[r], l], select the top N (lowest r first among equals) and AND the selection
 * with B[P[r], l], so Bbar <= B[P,:] and every block holds at most N ones (Eq. 7).
 *   perm       in   I int32 or NULL
 *   Bbar_bits  out  I x ceil(J/32) words, rows in permuted order                        */
BIMASK_API int bimask_backward_mask(const void *W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                         const uint32_t *B_bits, const int32_t *perm, uint32_t *Bbar_bits, void *stream);

/* Backward mask and the transposed compressed backward operand in one pass (same results
 * as bimask_backward_mask followed by bimask_compress_nm(transposed = 1)).
 *   values  out  bimask_operand_elems(J, I, N, M) elements
 *   index   out  bimask_operand_index_words(J, I, N, M) words for N <= 2, else ignored      */
BIMASK_API int bimask_backward_mask_compress(const void *W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                                  const uint32_t *B_bits, const int32_t *perm, uint32_t *Bbar_bits,
                                  void *values, uint32_t *index, void *stream);

/* Compress a masked weight matrix into the operand format described at the top.
 *   transposed = 0: mask_bits = B (rows of W), perm must be NULL; output rows = I.
 *   transposed = 1: mask_bits = Bbar (permuted rows), perm = P or NULL; output row l is
 *                   column l of (Bbar .* W[P,:]); output rows = J.
 * The mask must hold at most N ones per group.                                          */
BIMASK_API int bimask_compress_nm(const void *W, int64_t I, int64_t J, int64_t ldw, int dtype, int N, int M,
                       const uint32_t *mask_bits, const int32_t *perm, int transposed,
                       void *values, uint32_t *index, void *stream);

/* Forward GEMM, Eq. (3):  Y[t][i] = sum_j X[t][j] * (B .* W)[i][j], with (B .* W) given in
 * compressed form (transposed = 0).  bf16: fp32 accumulation, bf16 output, N <= 2 on the
 * sparse matrix cores, other ratios on the dense matrix cores; f32: fp32 throughout.
 *   X  in  T x J (ldx >= J);   Y  out  T x I (ldy >= I);   same dtype as the values.
 *   Pointers at least 4-byte aligned and, for bf16, even leading dimensions (else
 *   BIMASK_ERR_ALIGN); 16-byte aligned pointers and row pitches take the fast path.     */
BIMASK_API int bimask_sparse_gemm_fwd(const void *X, int64_t T, int64_t ldx, const void *Wf_values, const uint32_t *Wf_index,
                           int64_t I, int64_t J, int dtype, int N, int M, void *Y, int64_t ldy,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Backward GEMM, Eq. (10):  dX[t][j] = sum_r dY[t][P[r]] * (Bbar .* W[P,:])[r][j], with the
 * weight operand given in transposed compressed form (transposed = 1); perm = NULL is Eq. (8).
 *   dY  in  T x I (lddy >= I);   dX  out  T x J (lddx >= J).
 *   workspace: bimask_workspace_bytes(BIMASK_WS_GEMM_BWD, ...) bytes (holds dY[:,P] when the
 *   gather is not fused into the GEMM; 0 = none needed).  bf16 with N <= 2 fuses it for
 *   I <= 512 and for 512 < I <= 2048 with J <= min(I, 512), I and J multiples of 8; bf16 with
 *   N > 2 for 128 < I <= 2048 with J <= min(I, 512), I and J multiples of 8.  Apart from the
 *   N <= 2, I <= 512 range these move rows in 16-byte pieces: dY, dX 16-byte aligned, lddy, lddx
 *   multiples of 8, else BIMASK_ERR_ALIGN.                                               */
BIMASK_API int bimask_sparse_gemm_bwd(const void *dY, int64_t T, int64_t lddy, const int32_t *perm,
                           const void *Wb_values, const uint32_t *Wb_index, int64_t I, int64_t J,
                           int dtype, int N, int M, void *dX, int64_t lddx,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Debug helper, off the hot path: the search, the backward mask, the backward GEMM and the
 * refinement trust that what they are given are permutations of 0 .. I-1 (Sec. 3.3: P is a row
 * permutation) and read rows through them unchecked.  This call checks K candidates:
 *   perms  in   K x I int32, device;   ok  out  int32[K], device: 1 = a permutation, 0 = a value
 *   out of range or repeated.   I <= 2^20 (a bitmap of I bits in LDS), else BIMASK_ERR_UNSUPPORTED. */
BIMASK_API int bimask_check_perms(const int32_t *perms, int K, int64_t I, int32_t *ok, void *stream);

/* Refinement of a permutation by proposed exchanges.  The paper's Limitations leave "a better
 * permutation than a random one" to future work; this is hill climbing on the objective its
 * search already uses (Sec. 3.3 / Alg. 1: the number of (block of M permuted rows, column)
 * pairs of B[P,:] holding at most N ones).  Proposal t exchanges P[swaps[2t]] and
 * P[swaps[2t+1]]; it is kept iff the count grows strictly.  Proposals are taken in order,
 * each against the permutation the earlier ones left; a proposal naming a position outside
 * [0, I) is skipped.  The library draws no random numbers: the caller supplies the proposals.
 *   B_bits    in   I x ceil(J/32) words (as written by bimask_forward_mask)
 *   perm_in   in   I int32, or NULL for the identity (may be the same buffer as perm_out)
 *   swaps     in   S x 2 int32 positions, device memory; S >= 0 (NULL allowed when S == 0)
 *   perm_out  out  I int32
 *   result    out  int32[2], device memory: gain in the count, number of proposals kept
 * One workgroup keeps the permutation in LDS: I <= 32768 and a mask below 2^31 words, else
 * BIMASK_ERR_UNSUPPORTED.  Cost per proposal: 2M mask rows, independent of I.              */
BIMASK_API int bimask_perm_refine(const uint32_t *B_bits, int64_t I, int64_t J, int N, int M,
                       const int32_t *perm_in, const int32_t *swaps, int64_t S,
                       int32_t *perm_out, int32_t *result, void *stream);

/* Grouped calls: the mask and search steps of n INDEPENDENT layers (all layers of a network,
 * say) in a few launches instead of 2-3 per layer.  Layers this small are bound by launch
 * latency, and Alg. 1 treats every layer separately, so a training step can issue them
 * together: all forward masks first, then all searches, then all backward masks.  Results are
 * identical to calling the per-layer functions in a loop; all layers of one call share dtype,
 * N:M and (for the search) the number of candidates K.
 *   layers   HOST array of n descriptors (read during the call only); the pointers inside
 *            are device pointers with the meaning, size and alignment rules of the per-layer
 *            calls:  forward  uses W, I, J, ldw -> B_bits, Wf_values, Wf_index
 *                    search   uses B_bits, I, J, perms -> scores, best, best_perm (may be
 *                             NULL), with workspace / workspace_bytes as in bimask_perm_search
 *                    backward uses W, I, J, ldw, B_bits, best_perm (the permutation; NULL =
 *                             identity) -> Bbar_bits, Wb_values, Wb_index
 *                    refine   uses B_bits, I, J, swaps, n_swaps -> best_perm (refined IN PLACE,
 *                             must not be NULL), refine_result; one workgroup per layer, all
 *                             layers at once (limits as bimask_perm_refine)
 * Errors: as the per-layer calls; the first failing layer's code is returned and nothing is
 * launched if any layer fails validation.                                                */
typedef struct bimask_group_layer {
    const void *W;
    int64_t I, J, ldw;
    uint32_t *B_bits;
    void *Wf_values;
    uint32_t *Wf_index;
    const int32_t *perms;
    int32_t *scores;
    int32_t *best;
    int32_t *best_perm;
    void *workspace;
    size_t workspace_bytes;
    uint32_t *Bbar_bits;
    void *Wb_values;
    uint32_t *Wb_index;
    const int32_t *swaps;       /* n_swaps x 2 proposed exchanges (bimask_perm_refine) */
    int64_t n_swaps;
    int32_t *refine_result;     /* int32[2]: gain, proposals kept */
} bimask_group_layer;

BIMASK_API int bimask_forward_mask_compress_group(const bimask_group_layer *layers, int n, int dtype, int N, int M,
                                       void *stream);
BIMASK_API int bimask_perm_search_group(const bimask_group_layer *layers, int n, int N, int M, int K, void *stream);
BIMASK_API int bimask_backward_mask_compress_group(const bimask_group_layer *layers, int n, int dtype, int N, int M,
                                        void *stream);
BIMASK_API int bimask_perm_refine_group(const bimask_group_layer *layers, int n, int N, int M, void *stream);

/* Buffer sizes of a compressed operand with `rows` x `cols` logical entries: number of
 * elements of `values` and of uint32 words of `index` (0 when no index is written).     */
BIMASK_API int64_t bimask_operand_elems(int64_t rows, int64_t cols, int N, int M);
BIMASK_API int64_t bimask_operand_index_words(int64_t rows, int64_t cols, int N, int M);

/* Scratch bytes a call needs (0 if none).  kind is a bimask_ws_kind.                     */
BIMASK_API size_t bimask_workspace_bytes(int kind, int64_t I, int64_t J, int64_t T, int K, int dtype, int N, int M);

/* Static, never NULL.                                                                    */
BIMASK_API const char *bimask_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* BIMASK_H */
