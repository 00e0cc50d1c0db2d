/*
 * rapid_attn.h -- C ABI of the MI355X (gfx950) MM-DiT joint-attention library.
 *
 * One call = the self-attention of ONE DiT layer over the joint image+text
 * token sequence, for all samples and heads (RAPID^3 Sec. 3.1, Eq. 1: F_SA),
 * either dense or with the attention map pruned to a per-(sample, head) set
 * of (query-block, key-block) tiles (Sec. 3.2 "Level-3: Sparse-Attention",
 * Eq. 4: F_SA_sparse, controlled per layer and per head).
 *
 * Mapping from the Sparse-Attention action of Sec. 3.3 (c):
 *   a = 0            -> rapid_attn_dense
 *   a in 1..N_sparse -> rapid_attn_block_sparse with that action's mask
 *   cache reused     -> no call (the policy is inactive on such a step)
 * A CFG pair (App. B: SD3 runs cond + null as a batch of two under one
 * action) passes the same mask for both samples.
 *
 * Semantics, for sample b, head h, query row r (M = 1 everywhere when dense):
 *   r >= kv_len                                   -> O[b,h,r,:] = 0
 *   A = { c < kv_len : M[b,h,r/block,c/block] != 0 }
 *   A empty                                       -> O[b,h,r,:] = 0
 *   else   O[b,h,r,:] = sum_{c in A} softmax_A(scale * Q[r].K[c]) V[c,:]
 * Pruned keys are removed before the softmax; K/V tiles of pruned blocks and
 * rows at or beyond kv_len are never multiplied in (NaN/Inf there are inert).
 * Arithmetic: bf16 inputs, bf16 MFMA with fp32 accumulation, fp32 online
 * softmax, probabilities rounded to bf16 before the PV product and the
 * normaliser taken as the fp32 sum of those rounded probabilities, bf16 output.
 *
 * Memory: every pointer except `stream` is a DEVICE pointer owned by the
 * caller.  Q, K, V, O are bf16 [B, H, N, D] contiguous, D fastest.  Q/K/V/mask
 * are read-only; O is fully overwritten ([B,H,N,D], padded rows included) and
 * must not overlap an input (checked for the contiguous entry points).  The library allocates nothing, keeps no state
 * between calls and never synchronises: kernels are enqueued on `stream`
 * (a hipStream_t; NULL = the default stream) and the call returns at once.
 *
 * Errors: every argument check happens on the host before any launch, so each
 * code below is reachable without a GPU.  On error nothing is launched.
 */
#ifndef RAPID_ATTN_H
#define RAPID_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RAPID_ATTN_VERSION 100

/* exported with default visibility; everything else in the library is hidden */
#define RAPID_API __attribute__((visibility("default")))

typedef enum {
    RAPID_OK              =  0,
    RAPID_ERR_NULL        = -1,  /* a required pointer is NULL                        */
    RAPID_ERR_SHAPE       = -2,  /* B,H,N <= 0; kv_len outside 1..N; N % block != 0;
                                    N > 2^22; B*H > 524287                            */
    RAPID_ERR_UNSUPPORTED = -3,  /* D not in {64,128}; block not in {64,128}          */
    RAPID_ERR_ALIGN       = -4,  /* q/k/v/o/workspace not 16-byte aligned             */
    RAPID_ERR_WORKSPACE   = -5,  /* workspace NULL or smaller than required           */
    RAPID_ERR_DEVICE      = -6,  /* the HIP runtime refused a launch                  */
    RAPID_ERR_ALIAS       = -7   /* o shares bytes with q, k or v (contiguous entries) */
} rapid_status;

/*
 * Dense joint attention (Sec. 3.1 Eq. 1; action 0 of Sec. 3.3 (c)).
 *   q,k,v   device, bf16 [B,H,N,D]           o   device, bf16 [B,H,N,D]
 *   N       tokens as allocated, 1 .. 2^22; B*H <= 524287
 *   D       head dimension, 64 or 128
 *   kv_len  valid tokens, 1..N, a prefix of the sequence: keys >= kv_len are
 *           ignored, query rows >= kv_len produce 0
 *   scale   softmax scale; <= 0 selects 1/sqrt(D)
 *   workspace, workspace_bytes   unused by the dense path; may be NULL / 0
 *   stream  hipStream_t, NULL = default stream
 * Returns RAPID_OK or a negative rapid_status.
 */
RAPID_API int rapid_attn_dense(const void* q, const void* k, const void* v, void* o,
                     int B, int H, int N, int D, int kv_len, float scale,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Block-sparse joint attention (Sec. 3.2 Level-3, Eq. 4; actions 1..N_sparse).
 *   block   square mask tile edge in tokens, 64 or 128; N % block == 0
 *   mask    device, uint8 [B,H,N/block,N/block], row-major (query-block,
 *           key-block); nonzero = keep the tile.  One mask per (sample, head),
 *           as the sparsity control is per layer and per head.
 *   workspace  device scratch of at least rapid_attn_workspace_bytes(...)
 *           bytes, 16-byte aligned.  Its contents on entry do not matter and
 *           nothing in it survives as state: every call first compacts the
 *           mask into it (kept key-blocks per query-block, blocks starting at
 *           or beyond kv_len dropped), lays out its launch plan there, and
 *           then runs attention over the kept tiles only; rows that keep many
 *           tiles may be cut into pieces whose partial results pass through it.
 *           One workspace must not serve two calls that can run concurrently
 *           (different streams): each call rewrites all of it.  Calls on one
 *           stream, and replays of a captured graph, may share it.
 *           What it holds after a call (for tests and tools; may change with
 *           RAPID_ATTN_VERSION).  nb = N/block, items = ceil(B*H/8)*nb, each
 *           array starting at the next 256-byte boundary after the previous:
 *             int32 counts [B*H*nb]      kept key-blocks of each query-block
 *             launch plan, 8 segments of `chunk` entries; segment x holds the
 *                                        work of the (b,h) pairs with
 *                                        (b*H+h) % 8 == x, then "none" entries
 *               block 64:  chunk = items; entry = int32 item id
 *                          b*H*nb + h*nb + i, none = -1
 *               block 128: chunk = items + pmax, pmax = min(256, items);
 *                          entry = 4 x int32 (item, first, n, w): n kept
 *                          key-blocks of the item starting at position `first`
 *                          of its list; none = (-1,0,0,-1); w = -1 for a whole
 *                          item, else (slot << 8) | (k << 4) | (P-1) for piece
 *                          k of P, slot = first of the item's P partial-result
 *                          slots.  The pieces of an item cover its list once,
 *                          in order of k.
 *             int32 index  [B*H*nb*nb]   ascending kept key-blocks, row-wise;
 *                                        entries past counts[] are undefined
 *             block 128 only: int32 arrived [8*pmax] (pieces of a cut item
 *                                        that have finished, at its first
 *                                        slot) and the partial-result slots
 *   N       as rapid_attn_dense, and a multiple of block
 *   limits  N <= 2^22 and B*H <= 524287 (RAPID_ERR_SHAPE beyond), for the
 *           dense call too
 *   other arguments as rapid_attn_dense.
 */
RAPID_API int rapid_attn_block_sparse(const void* q, const void* k, const void* v, void* o,
                            int B, int H, int N, int D, int block,
                            const unsigned char* mask, int kv_len, float scale,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * rapid_attn_block_sparse without a workspace argument, for callers that cannot
 * allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, semantics and kernels as
 * rapid_attn_block_sparse; the scratch is a fixed array of
 * RAPID_ATTN_STATIC_SCRATCH_BYTES inside the library's code object (one copy per
 * GPU, held until the process ends), and the call allocates and frees nothing.
 *   - A shape whose counts, lists and plan alone exceed the array returns
 *     RAPID_ERR_WORKSPACE.  When only the partial-result slots of split items do
 *     not all fit, fewer slots are used (fewer long rows are cut into pieces;
 *     results stay within the stated tolerances, and are bit-identical to
 *     rapid_attn_block_sparse whenever everything fits, e.g. B*H <= 24 at
 *     N <= 4608).
 *   - All calls on one GPU share that GPU's array: two calls that can run
 *     concurrently on one GPU (different streams, or different host threads on
 *     streams that are not ordered) race.  Calls on one stream are ordered.
 *   - The first call on a device looks the array's address up
 *     (hipGetSymbolAddress); make that call outside graph capture.
 */
#define RAPID_ATTN_STATIC_SCRATCH_BYTES (64u << 20)
RAPID_API int rapid_attn_block_sparse_static(const void* q, const void* k, const void* v, void* o,
                            int B, int H, int N, int D, int block,
                            const unsigned char* mask, int kv_len, float scale, void* stream);

/* Bytes of workspace rapid_attn_block_sparse needs for this shape; 0 if the
 * shape is invalid or unsupported.  Pure host arithmetic. */
RAPID_API size_t rapid_attn_workspace_bytes(int B, int H, int N, int D, int block);

/*
 * The same attention on tensors as an MM-DiT block holds them (Sec. 3.1: the text
 * and the image stream are separate tensors, joined only for attention): the
 * joint sequence is given as one or two token segments, each with its own
 * Q/K/V/O tensors and strides, so no concatenated or transposed copy is needed.
 * Token t of the joint sequence is row t of segment 0 if t < segments[0].n,
 * else row t - segments[0].n of segment 1; N = sum of the n.
 *   q,k,v,o      device, bf16; element (b, h, r, d) of a tensor lies at
 *                ptr + b*stride_b + h*stride_h + r*stride_n + d  (elements; the
 *                D elements of a row are contiguous).  in_stride_* address
 *                q, k and v, out_stride_* address o.  [B,n,H,D] tensors have
 *                stride_b = n*H*D, stride_h = D, stride_n = H*D; a fused
 *                [B,n,3,H,D] projection has in_stride_n = 3*H*D.
 *   constraints  pointers 16-byte aligned, strides multiples of 8 elements,
 *                D <= stride_n <= 2^23; with two segments segments[0].n is a
 *                multiple of 128 (no 64-key tile and no 128-query block lies in
 *                both tensors) and stride_h, stride_n are the same in both.
 *                The stride of a dimension of size 1 (stride_b when B == 1,
 *                stride_h when H == 1, stride_n of a one-token second segment)
 *                addresses nothing and is not looked at.
 */
typedef struct rapid_attn_segment {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    int n;                                            /* tokens in this segment */
    long long in_stride_b, in_stride_h, in_stride_n;  /* of q, k, v */
    long long out_stride_b, out_stride_h, out_stride_n;
} rapid_attn_segment;

/*
 * Joint attention over the segments (dense when mask is NULL, else block-sparse).
 *   segments     HOST array of n_segments (1 or 2) descriptors, read during the call
 *   block, mask  as rapid_attn_block_sparse, except that N need not be a multiple
 *                of block: nb = ceil(N/block) and the last block ends at N.
 *                mask NULL = dense (block ignored)
 *   kv_len       valid tokens for every sample, 1..N; 0 selects N
 *   kv_lens      device, int32 [B], or NULL: per-sample valid tokens (prompts of
 *                different length in one batch), each clamped to 0..N; replaces
 *                kv_len when given.  A sample with 0 valid tokens outputs zeros.
 *   workspace    sparse only: at least rapid_attn_joint_workspace_bytes(B,H,N,D,block)
 *   other arguments and all semantics as above.
 */
RAPID_API int rapid_attn_joint(const rapid_attn_segment* segments, int n_segments,
                     int B, int H, int D, int block, const unsigned char* mask,
                     int kv_len, const int* kv_lens, float scale,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Workspace bytes of the sparse form of rapid_attn_joint (N = total tokens, any
 * positive count); 0 if the shape is invalid or unsupported. */
RAPID_API size_t rapid_attn_joint_workspace_bytes(int B, int H, int N, int D, int block);

/* Static, NUL-terminated description of a status code.  Never NULL. */
RAPID_API const char* rapid_attn_status_string(int status);

/* RAPID_ATTN_VERSION the library was built from. */
RAPID_API int rapid_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_ATTN_H */
