// Calls between the translation units of librapid_attn.so (hidden symbols, not part of the C ABI).
#ifndef RAPID_INTERNAL_H
#define RAPID_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "rapid_attn.h"

namespace rapid_internal {

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
