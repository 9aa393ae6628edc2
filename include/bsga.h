/*
 * bsga -- block-sparse global attention for MI355X (gfx950).  C ABI.
 *
 * The library implements the training-free block-sparse replacement for dense
 * global attention in multi-view geometry transformers:
 *   1. pool Q and K per block of b tokens                (Sec. 4.1, "Predicting Block Masks")
 *   2. block scores S = P^b(Q) P^b(K)^T, row softmax      (same paragraph)
 *   3. CDF-threshold (tau) + top-k floor (rho) selection  (Sec. 4.1, "Selecting Blocks")
 *   4. softmax attention over the kept key blocks only    (Sec. 4.1, Eq. (2))
 * plus the dense baseline of Eq. (1).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers unless marked "host".  The caller owns
 *     every buffer; the library allocates, frees and copies nothing, and only enqueues
 *     work on `stream` (a hipStream_t passed as void*; NULL = the null stream).  Calls
 *     return after enqueueing; they do not synchronise.  They record kernel launches only
 *     (no memset, copy or allocation), so they may be called on a stream that is being
 *     captured into a HIP graph (bsga_sparse_attn_noalloc: after one call outside a capture).
 *   - Tensors are contiguous row-major; Q, K, V, O are [heads, n_tokens, head_dim]
 *     (a batch dimension is folded into heads).  Pointers must be 16-byte aligned.
 *   - head_dim must be 64.  block must be 64 or 128.  dtype: BSGA_BF16 or BSGA_FP32
 *     (the fp32 path is a correctness path, not a tuned one).
 *   - Blocks: block I covers tokens I*block .. min((I+1)*block, n_tokens)-1;
 *     nb = ceil(n_tokens / block).  The last block may be ragged.
 *   - Return value: BSGA_OK or an error code; bsga_last_error() gives a message
 *     (thread-local).  Arguments are validated before anything is launched, so
 *     argument errors can be observed without a GPU.
 */
#ifndef BSGA_H
#define BSGA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BSGA_OK 0
#define BSGA_ERR_INVALID_ARG 1
#define BSGA_ERR_UNSUPPORTED 2
#define BSGA_ERR_WORKSPACE 3
#define BSGA_ERR_HIP 4

#define BSGA_BF16 0
#define BSGA_FP32 1

/* ABI version of this header (bumped on incompatible change). */
int bsga_version(void);

/* Message for the last error returned on this thread ("" if none). Host pointer, library-owned. */
const char* bsga_last_error(void);

/*
 * Block average pooling of Q and K  (Sec. 4.1, "Predicting Block Masks": P^b(Q), P^b(K)).
 *   q, k          [heads, n_tokens, 64], dtype as given
 *   q_pool,k_pool [heads, nb, 64] float64 out; block I is the mean over its valid tokens
 *                 (the ragged last block divides by its own token count).
 * Sums are accumulated in float64, so for bf16 inputs the block sums are exact.
 * Either of (q, q_pool) or (k, k_pool) may be NULL together to pool only one tensor.
 */
int bsga_pool_qk(const void* q, const void* k, int dtype, int heads, int64_t n_tokens, int head_dim,
                 int block, double* q_pool, double* k_pool, void* stream);

/*
 * Block average pooling when the sequence is split in two parts that are blocked separately
 * (Sec. 4.2: the patch tokens X_p and the special tokens X_s are kept apart, so that no pooled block
 * mixes the two kinds).  Tokens [0, n_first) form blocks 0 .. ceil(n_first/block)-1, tokens
 * [n_first, n_tokens) the blocks after them; the last block of EACH part may be ragged and is
 * averaged over its own tokens.  nb = ceil(n_first/block) + ceil((n_tokens-n_first)/block).
 * 0 <= n_first <= n_tokens; n_first = n_tokens (or 0) is bsga_pool_qk.  Otherwise as bsga_pool_qk.
 */
int bsga_pool_qk_split(const void* q, const void* k, int dtype, int heads, int64_t n_tokens,
                       int64_t n_first, int head_dim, int block, double* q_pool, double* k_pool,
                       void* stream);

/*
 * Bytes of device workspace bsga_select_blocks needs: the float64 block logits
 * [heads, nb_q, nb_k] (Sec. 4.1, the low-resolution score matrix S).  0 for invalid arguments.
 */
size_t bsga_select_workspace_bytes(int heads, int nb_q, int nb_k);

/*
 * Block scores, block softmax and block selection  (Sec. 4.1, "Predicting Block Masks" and
 * "Selecting Blocks").  For every head h and query block I:
 *   logits[J] = score_scale * <q_pool[h,I], k_pool[h,J]>,  p = softmax_J(logits)      (float64)
 *   rank key blocks by descending p, equal p by ascending J;
 *   n_cdf = length of the shortest ranked prefix whose summed p is >= tau
 *           (all nb_k blocks if tau >= 1 or the sum never gets there);
 *   k = floor(nb_k * (1 - rho)) evaluated in float64;  n = min(nb_k, max(n_cdf, k, 1));
 *   the first n ranked blocks are kept.
 * Then, if given (Sec. 4.2, everything that touches a special token stays dense):
 *   force_q[I] != 0 keeps the whole row I;
 *   force_k[J] == 1 keeps column J in every row (J is still ranked like any other block);
 *   force_k[J] == 2 keeps column J in every row and takes J OUT of the ranking: it gets no mass in
 *                   the block softmax and does not count towards B (nb_k above becomes the number
 *                   of ranked blocks).  This is the patch-only block map of Sec. 4.2.
 *   q_pool   [heads, nb_q, 64] float64      k_pool [heads, nb_k, 64] float64
 *   force_q  nullable [nb_q] uint8          force_k nullable [nb_k] uint8
 * Outputs (each nullable):
 *   mask_bits [heads, nb_q, ceil(nb_k/32)] uint32, bit (J%32) of word J/32 set iff (I,J) kept;
 *   kv_idx    [heads, nb_q, idx_stride] int32, the kept J in ascending order; entries past the
 *             count are left untouched;  idx_stride >= nb_k;
 *   kv_cnt    [heads, nb_q] int32, number of kept blocks.
 *   workspace, workspace_bytes: device scratch of at least bsga_select_workspace_bytes(...) bytes,
 *             16-byte aligned; holds the block logits between the two kernels of this call and is
 *             overwritten; calls sharing one workspace must be stream-ordered.
 * Limits: 1 <= nb_k <= 8192 (rows are held in registers; above 4096 key blocks the kernel spills and
 * is several times slower per row), 1 <= nb_q <= 2^18, heads <= 65535.  score_scale must be finite;
 * 0 <= tau; 0 <= rho <= 1.
 */
int bsga_select_blocks(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k,
                       int head_dim, double score_scale, double tau, double rho,
                       const uint8_t* force_q, const uint8_t* force_k, uint32_t* mask_bits,
                       int32_t* kv_idx, int32_t* kv_cnt, int idx_stride, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * Token gather  (Sec. 4.2: the tokens are split into patch tokens X_p and special tokens X_s).
 *   dst[h, i, :] = src[h, index[i], :]   for i in [0, n_dst)
 *   src   [heads, n_src, 64], dtype as given      dst [heads, n_dst, 64] same dtype, must not overlap src
 *   index [n_dst] int32 device array; values outside [0, n_src) are clamped into it
 * Used to make the patch tokens contiguous (so that no pooled block mixes the two kinds) and to
 * put the outputs back in the caller's token order (gather with the inverse permutation).
 */
int bsga_gather_tokens(const void* src, int dtype, int heads, int64_t n_src, int head_dim,
                       const int32_t* index, int64_t n_dst, void* dst, void* stream);

/*
 * Bytes of device workspace bsga_sparse_attn needs for this shape (bsga_dense_attn uses 16 bytes
 * of one and accepts NULL).  Q, K and V are read in place and all intermediates stay on chip; the
 * workspace holds the launch order of the (head, query block) rows, heaviest first, and the counter
 * through which the last rows of a large launch are handed out at run time (4 bytes per row, sized
 * for block 64 and a split sequence, plus 128 bytes per head and 16 bytes; 0 for fp32 and for invalid
 * arguments).
 */
size_t bsga_attn_workspace_bytes(int dtype, int heads, int64_t n_tokens, int head_dim);

/*
 * Block-sparse attention  (Sec. 4.1, Eq. (2), with masked entries excluded from the softmax).
 * For token i in query block I of head h:
 *   o_i = sum_j softmax_j(softmax_scale * <q_i, k_j>) v_j   over keys j < n_tokens that lie in
 *   the key blocks kv_idx[h, I, 0 .. kv_cnt[h,I]-1].
 *   q, k, v  [heads, n_tokens, 64], dtype as given;  out same shape and dtype
 *   kv_idx   [heads, nb, idx_stride] int32, each row's kept key blocks: distinct, in [0, nb);
 *   kv_cnt   [heads, nb] int32, 1 <= count <= nb (a row with count 0 yields zeros, lse = -inf)
 *   lse      nullable [heads, n_tokens] float32: natural-log sum-exp of each row's kept logits
 *   workspace, workspace_bytes: device scratch of at least bsga_attn_workspace_bytes(...) bytes;
 *            contents are overwritten; calls sharing one workspace must be stream-ordered.  May be
 *            NULL: the query blocks are then launched in index order instead of heaviest first,
 *            and every row is tied to the workgroup of its number (same results; a longer tail when
 *            row lengths differ a lot, and a few per cent slower on large shapes because the XCDs of
 *            a part do not run equally fast and cannot then share the last rows unevenly).
 * bf16: products on bf16 MFMA with fp32 accumulation, fp32 softmax weights.  softmax_scale > 0.
 * The index lists are trusted to be in range (they come from bsga_select_blocks); block
 * indices are clamped to [0, nb) before use so a corrupt list cannot read out of bounds.
 * Any order of a row's entries gives the same result up to rounding; the ascending order that
 * bsga_select_blocks writes is the fast one (a ragged block, which is always the last block of the
 * sequence or of its first part, should come last or nearly last in its row: the tiles after it
 * take a slower path).  K and V must be finite everywhere: rows of a tile that are not keys of a
 * listed block are multiplied by a weight of exactly zero, not skipped.
 */
int bsga_sparse_attn(const void* q, const void* k, const void* v, int dtype, int heads,
                     int64_t n_tokens, int head_dim, int block, float softmax_scale,
                     const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * bsga_sparse_attn for callers that cannot allocate or hand over device memory beyond the tensors
 * themselves: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and results as bsga_sparse_attn without the workspace: the launch order of the rows
 * lives in a buffer built into the library (bsga_noalloc_scratch_bytes() bytes of device memory per
 * GPU, held from the first call on that GPU until the process ends).  The call allocates and frees
 * nothing and clears nothing with a memset.  Shapes whose launch order does not fit, i.e.
 * bsga_attn_workspace_bytes(...) > bsga_noalloc_scratch_bytes(), return BSGA_ERR_UNSUPPORTED (the
 * buffer holds heads * (ceil(n_tokens/64) + 33) + 4 <= 524288 words: e.g. 16 heads x 2 million
 * tokens).  All calls on one GPU share the one buffer and each overwrites it: calls that overlap in
 * time on the same GPU (different streams, or different threads) race; order them on one stream.
 */
int bsga_sparse_attn_noalloc(const void* q, const void* k, const void* v, int dtype, int heads,
                             int64_t n_tokens, int head_dim, int block, float softmax_scale,
                             const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out,
                             float* lse, void* stream);

/* Size in bytes of the built-in buffer of bsga_sparse_attn_noalloc (a constant of the build). */
size_t bsga_noalloc_scratch_bytes(void);

/*
 * Block-sparse attention with separate query and key block sizes (the appendix's learned-projection
 * ablation predicts its maps with query blocks of 128 and key blocks of 64; Sec. 4.1 otherwise).
 * As bsga_sparse_attn, but query block I covers block_q tokens and the lists refer to key blocks of
 * block_k tokens: kv_idx [heads, ceil(n_tokens/block_q), idx_stride] with entries in
 * [0, ceil(n_tokens/block_k)), idx_stride >= ceil(n_tokens/block_k).
 * Supported: block_k == block_q (64 or 128), and block_q = 128 with block_k = 64 (bf16 only; pool Q
 * and K separately with bsga_pool_qk, select with nb_q != nb_k).  Other pairs: BSGA_ERR_UNSUPPORTED.
 */
int bsga_sparse_attn_qk(const void* q, const void* k, const void* v, int dtype, int heads,
                        int64_t n_tokens, int head_dim, int block_q, int block_k, float softmax_scale,
                        const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out,
                        float* lse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Block-sparse attention over a sequence split in two separately blocked parts (Sec. 4.2; Eq. (2) of
 * Sec. 4.1 on the blocks of bsga_pool_qk_split).  Query block I and key block J are the blocks
 * described at bsga_pool_qk_split, with block_q tokens per query block and block_k per key block
 * (the same pairs as bsga_sparse_attn_qk): a block never crosses n_first, and the last block of each
 * part may be ragged.  kv_idx [heads, nbq, idx_stride], kv_cnt [heads, nbq] with
 * nbq = ceil(n_first/block_q) + ceil((n_tokens-n_first)/block_q), entries in [0, nbk),
 * nbk = ceil(n_first/block_k) + ceil((n_tokens-n_first)/block_k), idx_stride >= nbk.
 * With the patch tokens first and the special tokens after them, every patch token lies in a block
 * of patch tokens only.  Everything else as bsga_sparse_attn.
 */
int bsga_sparse_attn_split(const void* q, const void* k, const void* v, int dtype, int heads,
                           int64_t n_tokens, int64_t n_first, int head_dim, int block_q, int block_k,
                           float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt,
                           int idx_stride, void* out, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * Dense attention baseline  (Sec. 4.1, Eq. (1)): softmax(softmax_scale * Q K^T) V per head.
 * Same tensors and numerics as bsga_sparse_attn, every key visible.  workspace: NULL, or at least
 * 16 bytes (16-byte aligned; a smaller or misaligned one is ignored) for the counter that hands out
 * the last rows of a large launch at run time; overwritten; stream-ordered like the others.
 */
int bsga_dense_attn(const void* q, const void* k, const void* v, int dtype, int heads,
                    int64_t n_tokens, int head_dim, float softmax_scale, void* out, float* lse,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aid, not part of the method: the rate the matrix pipes sustain on the MFMA instruction
 * the bf16 attention kernels use (32x32x16 bf16, the products of Eqs. (1)/(2)), with no memory traffic
 * at all, two workgroups of four waves per CU.  The part lowers its clock with the switching activity
 * of the data, so this rate on random operands, not the nominal peak, bounds any bf16 kernel.
 *   operands     0 = all-zero operands, 1 = pseudo-random roughly unit-normal bf16 values
 *   softmax_mix  0 = MFMAs only; 1 = beside every MFMA the softmax arithmetic attention needs per MFMA
 *                at head dim 64: two exp2, one pack to bf16, two fp32 adds for the row sum;
 *                2 = the same with the row sums taken the way the attention kernel takes them, by one
 *                16x16x32 MFMA per four products instead of the adds
 *   iters        rounds of 8 MFMAs per wave
 *   sink         device buffer of at least 2 * (number of CUs) * 1024 bytes, overwritten
 *   flops        nullable host pointer: receives the FLOPs of the launch (2 * 32*32*16 per MFMA)
 * The call only enqueues the kernel on `stream`; the caller times it.
 */
int bsga_probe_mfma(int operands, int softmax_mix, int iters, void* sink, size_t sink_bytes,
                    double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BSGA_H */
