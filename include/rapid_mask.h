/*
 * rapid_mask.h -- C ABI of the block-mask selection that turns a Sparse-Attention
 * level into the mask rapid_attn_block_sparse takes; exported by the same shared
 * library as rapid_attn.h.
 *
 * RAPID^3 (Sec. 3.2 "Level-3: Sparse-Attention", Sec. 3.3 (c)) lets the policy pick,
 * per step, one of N_sparse = 3 candidate settings of increasing sparsity for a
 * sparse attention that prunes the attention map per layer and head; the paper
 * takes that sparse attention from prior work and does not state its pruning
 * rule.  The rule here is this library's own, of the kind the paper describes
 * (a cheap per-head prediction of which blocks of the map matter):
 *
 *   for every (sample, head), with nb = N/block mask blocks, live blocks = those
 *   that start below kv_len:
 *   1. qbar_i, kbar_j = means of Q, K over the valid tokens of block i, j
 *   2. phat_i = softmax over the live j of scale * qbar_i . kbar_j
 *   3. row i keeps the fewest key-blocks, taken by decreasing phat_ij, whose mass
 *      reaches tau (blocks tying with the last one taken are kept as well);
 *      tau >= 1 keeps every live block
 *   4. always kept: the diagonal, and the rows and columns of text blocks (blocks
 *      holding a token at or after text_start) -- the paper's settings keep the
 *      text tokens dense
 *   5. rows and columns of blocks that are not live are 0
 *
 * Arithmetic: bf16 inputs, fp32 sums and softmax; the cut compares fp32 partial
 * sums, so a block whose inclusion decides whether the mass reaches tau to within
 * rounding may fall on either side.
 *
 * Memory: q, k, mask, workspace are DEVICE pointers owned by the caller; q, k are
 * bf16 [B,H,N,D] contiguous and read-only; mask is fully overwritten.  Nothing is
 * allocated, no state is kept, nothing synchronises; kernels go to `stream`.
 * Errors are found on the host before any launch (status codes of rapid_attn.h):
 * RAPID_ERR_NULL, RAPID_ERR_SHAPE (B,H,N <= 0, kv_len outside 1..N, N % block != 0,
 * text_start < 0, tau <= 0 or NaN), RAPID_ERR_UNSUPPORTED (D not 64/128, block not
 * 64/128, more than 2048 mask blocks), RAPID_ERR_ALIGN, RAPID_ERR_WORKSPACE,
 * RAPID_ERR_DEVICE.
 */
#ifndef RAPID_MASK_H
#define RAPID_MASK_H

#include <stddef.h>
#include "rapid_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 *   q, k        device, bf16 [B,H,N,D]
 *   block       mask tile edge, 64 or 128; N % block == 0; N/block <= 2048
 *   kv_len      valid tokens, 1..N
 *   text_start  first text token (tokens are image first, then text); a value
 *               >= kv_len means there are no text blocks
 *   tau         mass each row keeps, > 0; >= 1 keeps every live block
 *   scale       score scale; <= 0 selects 1/sqrt(D)
 *   mask        device, uint8 [B,H,N/block,N/block], written with 0/1
 *   workspace   device, at least rapid_mask_select_workspace_bytes(...) bytes,
 *               16-byte aligned: the fp32 block means of Q and K
 */
RAPID_API int rapid_mask_select(const void* q, const void* k, int B, int H, int N, int D,
                                int block, int kv_len, int text_start, float tau, float scale,
                                unsigned char* mask, void* workspace, size_t workspace_bytes,
                                void* stream);

/* Workspace bytes of rapid_mask_select; 0 if the shape is invalid or unsupported. */
RAPID_API size_t rapid_mask_select_workspace_bytes(int B, int H, int N, int D, int block);

/*
 * The same selection on Q and K as an MM-DiT block holds them (Sec. 3.1: image and text
 * stream are separate tensors, joined only for attention), so that the mask for
 * rapid_attn_joint comes from the very tensors that call reads, without a concatenated
 * copy.  Same rule, same kernels.
 *   segments     HOST array of n_segments (1 or 2) rapid_attn_segment descriptors, read
 *                during the call: q, k, n and in_stride_* are used, v and o are ignored
 *                (may be NULL).  Constraints as for rapid_attn_joint: pointers 16-byte
 *                aligned, strides multiples of 8 elements, D <= in_stride_n <= 2^23; with
 *                two segments segments[0].n is a multiple of 128 and in_stride_h,
 *                in_stride_n are the same in both.  N = sum of the n.
 *   block        64 or 128; nb = ceil(N/block) <= 2048, the last block ends at N
 *   kv_len       valid tokens of every sample, 1..N; 0 selects N
 *   kv_lens      device, int32 [B], or NULL: per-sample valid tokens, each clamped to 0..N;
 *                replaces kv_len when given.  Live blocks, block means and the text blocks
 *                (text_start < that sample's length) are taken per sample; a sample with
 *                0 valid tokens gets an all-zero mask.
 *   mask         device, uint8 [B,H,nb,nb]
 *   workspace    at least rapid_mask_select_joint_workspace_bytes(B,H,N,D,block) bytes
 *   other arguments, semantics and errors as rapid_mask_select.
 */
RAPID_API int rapid_mask_select_joint(const rapid_attn_segment* segments, int n_segments,
                                      int B, int H, int D, int block, int kv_len, const int* kv_lens,
                                      int text_start, float tau, float scale,
                                      unsigned char* mask, void* workspace, size_t workspace_bytes,
                                      void* stream);

/* Workspace bytes of rapid_mask_select_joint (N = total tokens, any positive count). */
RAPID_API size_t rapid_mask_select_joint_workspace_bytes(int B, int H, int N, int D, int block);

/*
 * Selection and attention of one layer in one call (Sec. 3.3 (c): the step's sparse action
 * drives the attention of every layer): what rapid_mask_select_joint followed by
 * rapid_attn_joint with that mask computes, but the selection writes the kept key-block
 * lists straight into the attention's workspace, so no byte mask is written, read back and
 * compacted in between.
 *   segments     as rapid_attn_joint (q, k, v, o and all strides are used)
 *   block, kv_len, kv_lens, text_start, tau   as rapid_mask_select_joint
 *   scale        of the attention and of the selection scores; <= 0 selects 1/sqrt(D)
 *   mask_out     device, uint8 [B,H,nb,nb], or NULL: the selected mask, if the caller wants
 *                to see it (written by the same kernel)
 *   workspace    at least rapid_attn_joint_select_workspace_bytes(B,H,N,D,block) bytes,
 *                16-byte aligned; same rules as the workspace of rapid_attn_block_sparse
 * Errors as rapid_attn_joint and rapid_mask_select_joint.
 */
RAPID_API int rapid_attn_joint_select(const rapid_attn_segment* segments, int n_segments,
                                      int B, int H, int D, int block, int kv_len, const int* kv_lens,
                                      int text_start, float tau, float scale, unsigned char* mask_out,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* Workspace bytes of rapid_attn_joint_select; 0 if the shape is invalid or unsupported. */
RAPID_API size_t rapid_attn_joint_select_workspace_bytes(int B, int H, int N, int D, int block);

/*
 * The library's default tau for a Sparse-Attention action (Sec. 3.3 (c)): action 0
 * (full attention) -> 1.0, actions 1, 2, 3 -> 0.98, 0.95, 0.90 (progressively
 * sparser; values of this library, not of the paper); anything else -> NaN.
 */
RAPID_API float rapid_mask_level_tau(int action);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_MASK_H */
