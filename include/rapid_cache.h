/*
 * rapid_cache.h -- C ABI of the Cache-Reuse residual operations and of the cost
 * accounting of RAPID^3, exported by the same shared library as rapid_attn.h.
 *
 * Cache-Reuse (Sec. 3.2 "Level-2: Cache-Reuse", Eq. 3): a step that updates the
 * cache runs the generator and keeps the residual between its output and its
 * input, Delta = G(X) - X; a step that reuses the cache skips the generator and
 * outputs O = X + Delta.  The policy decides per image (Sec. 3.3 (b)), so both
 * operations take an optional per-sample flag.
 *
 * Tensors are bf16, contiguous, laid out [B, elems_per_sample]; the exact sum or
 * difference is rounded once to bf16, nearest-even (computed in fp32, which
 * holds it exactly or far from a bf16 tie).  NaN in gives NaN out.
 *
 * Memory: x, delta, out, gen_out, sample_flags are DEVICE pointers owned by the
 * caller; the library allocates nothing, keeps no state, never synchronises and
 * enqueues on `stream` (a hipStream_t; NULL = the default stream).  The output
 * may alias an input of the same call element for element (in-place update).
 *
 * Errors (all checked on the host before any launch; nothing is launched on
 * error): RAPID_ERR_NULL for a missing pointer, RAPID_ERR_SHAPE for B <= 0 or
 * elems_per_sample <= 0 or more than 2^40 elements in total, RAPID_ERR_ALIGN for
 * a tensor pointer that is not 2-byte aligned, RAPID_ERR_DEVICE if the runtime
 * refuses the launch.  Status codes are those of rapid_attn.h.
 */
#ifndef RAPID_CACHE_H
#define RAPID_CACHE_H

#include <stddef.h>
#include "rapid_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Cache update: delta[b, :] = gen_out[b, :] - x[b, :]  (Delta = G(X) - X, Sec. 3.2).
 *   gen_out, x   device, bf16 [B, elems_per_sample], read-only
 *   delta        device, bf16 [B, elems_per_sample]
 *   sample_flags device, uint8 [B], or NULL: a sample with flag 0 is left
 *                untouched (its cache is not updated); NULL = every sample
 */
RAPID_API int rapid_cache_store(const void* gen_out, const void* x, void* delta,
                                int B, size_t elems_per_sample,
                                const unsigned char* sample_flags, void* stream);

/*
 * Cache reuse: out[b, :] = x[b, :] + delta[b, :]  (Eq. 3, the "reuse cache" branch).
 *   x, delta     device, bf16 [B, elems_per_sample], read-only
 *   out          device, bf16 [B, elems_per_sample]
 *   sample_flags as above: a sample with flag 0 is left untouched (the caller
 *                runs the generator for it)
 */
RAPID_API int rapid_cache_reuse(const void* x, const void* delta, void* out,
                                int B, size_t elems_per_sample,
                                const unsigned char* sample_flags, void* stream);

/*
 * Equivalent steps (Sec. 3.3, reward paragraph): K = sum_k (1 - c_cache[k]) *
 * (1 - c_sparse[k]) over the n_steps steps actually taken; each c is the cost
 * reduction of that step in [0, 1] (the paper measures 0.95 for a cached step
 * and 0.05 / 0.07 / 0.10 for its three sparse candidates).  HOST pointers, pure
 * host arithmetic in double.  *k_exact (may be NULL) receives the sum; the
 * return value is K rounded to the nearest integer (ties away from zero), at
 * least 1, or a negative rapid_status (NULL arrays with n_steps > 0,
 * n_steps < 0, a reduction outside [0, 1]).
 */
RAPID_API int rapid_equivalent_steps(const double* c_cache, const double* c_sparse,
                                     int n_steps, double* k_exact);

/*
 * Reward of one image (same paragraph): (1/K) sum_{k=1..K} lambda^(K-k) *
 * (q + omega * d), with q the image-reward score and d the discriminator
 * score.  Host arithmetic in double, the sum written out.  K < 1 returns NaN.
 */
RAPID_API double rapid_reward(double q, double d, double omega, double lambda, int K);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_CACHE_H */
