// Host-side segment table: cuts a ragged list of tensors into chunks of bounded size.
// Integer-only; needs no GPU.  The method clips per parameter tensor (Sec. 4.2, Eq. 3), so a
// chunk never spans two tensors and is cut relative to its tensor's own first element.

#include <stdint.h>

#include "adagc.h"

extern "C" int adagc_build_segment_table(const adagc_tensor_desc* descs, int64_t n_tensors,
                                         int64_t chunk_elems, int64_t* chunk_begin,
                                         uint32_t* chunk_tensor, uint32_t* chunk_index, int64_t capacity,
                                         int64_t* n_chunks)
{
    if (!descs || !chunk_begin || !n_chunks || n_tensors <= 0 || chunk_elems <= 0)
        return ADAGC_ERR_INVALID_ARG;
    if (n_tensors > (int64_t)UINT32_MAX) return ADAGC_ERR_TOO_LARGE;

    // Pass 1: validate and count (64-bit exclusive prefix sum of per-tensor chunk counts).
    int64_t total = 0;
    for (int64_t i = 0; i < n_tensors; ++i) {
        const adagc_tensor_desc& d = descs[i];
        if (d.numel <= 0 || d.flags != 0 || d.reserved != 0) return ADAGC_ERR_INVALID_ARG;
        const int64_t count = d.numel / chunk_elems + (d.numel % chunk_elems != 0 ? 1 : 0);
        if (count > (int64_t)UINT32_MAX || total > (int64_t)UINT32_MAX - count) return ADAGC_ERR_TOO_LARGE;
        total += count;
    }
    const bool fill = chunk_tensor != nullptr || chunk_index != nullptr;
    if (fill && capacity < total) return ADAGC_ERR_INVALID_ARG;

    // Pass 2: write.
    int64_t c = 0;
    for (int64_t i = 0; i < n_tensors; ++i) {
        chunk_begin[i] = c;
        const int64_t numel = descs[i].numel;
        const int64_t count = numel / chunk_elems + (numel % chunk_elems != 0 ? 1 : 0);
        if (fill) {
            for (int64_t k = 0; k < count; ++k) {
                if (chunk_tensor) chunk_tensor[c + k] = (uint32_t)i;
                if (chunk_index) chunk_index[c + k] = (uint32_t)k;
            }
        }
        c += count;
    }
    chunk_begin[n_tensors] = c;
    *n_chunks = c;
    return ADAGC_OK;
}
