// Calls between the translation units of librapid_attn.so (hidden symbols, not part of the C ABI).
#ifndef RAPID_INTERNAL_H
#define RAPID_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "rapid_attn.h"

namespace rapid_internal {

// The strides of a dimension of size 1 address nothing (frameworks leave arbitrary values there):
// the batch stride when B == 1, the head stride when H == 1, the token stride of a one-token second
// segment.  Returns the descriptor with those replaced by values that pass the checks and change
// no address (0 for batch and head; the first segment's token strides).
inline rapid_attn_segment normalised_segment(const rapid_attn_segment& g, int B, int H, const rapid_attn_segment* first)
{
    rapid_attn_segment r = g;
    if (B == 1) r.in_stride_b = r.out_stride_b = 0;
    if (H == 1) r.in_stride_h = r.out_stride_h = 0;
    if (first != nullptr && g.n == 1) { r.in_stride_n = first->in_stride_n; r.out_stride_n = first->out_stride_n; }
    return r;
}

// rapid_mask.hip.  The selection of include/rapid_mask.h on the Q, K of `segments` (validated as by
// rapid_mask_select_joint), written as the attention workspace holds a compacted mask: counts
// [B*H*nb] and ascending kept key-block lists index [B*H*nb, nb]; also as a byte mask when `mask`
// is not null.  `scratch` takes the block means (select_scratch_bytes).
size_t select_scratch_bytes(int B, int H, int nb, int D);
int select_to_lists(const rapid_attn_segment* segments, int n_segments, int B, int H, int D, int block,
                    int kv_len, const int* kv_lens, int text_start, float tau, float scale,
                    unsigned char* mask, int32_t* counts, int32_t* index, void* scratch, size_t scratch_bytes,
                    void* stream);

}  // namespace rapid_internal

#endif
