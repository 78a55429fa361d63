// Host-side segment table: cuts a ragged list of tensors into chunks of bounded size.
// Integer-only; needs no GPU.  The method clips per parameter tensor (Sec. 4.2, Eq. 3), so a
// chunk never spans two tensors and is cut relative to its tensor's own first element.

#include <stdint.h>

#include <vector>

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

// Visiting order of the streaming kernels.  Workgroups are dealt to the 8 XCDs in turn, so position k of
// the order is worked on by XCD k mod 8.  With `parts` in {1, 2, 4, 8} the list is cut into that many
// contiguous parts, XCD x works in part x mod parts, and the 8/parts XCDs that share a part take runs of
// `run` consecutive chunks in turn.  Any other `parts` value deals position k to part k mod parts.
extern "C" int adagc_build_visiting_order(int64_t n_chunks, int32_t parts, int32_t run, uint32_t* order)
{
    if (!order || n_chunks <= 0 || parts <= 0 || run <= 0) return ADAGC_ERR_INVALID_ARG;
    if (n_chunks > (int64_t)UINT32_MAX) return ADAGC_ERR_TOO_LARGE;
    const uint64_t nc = (uint64_t)n_chunks, w = (uint64_t)parts, R = (uint64_t)run;
    if (w == 1 && R == 1) {
        for (uint64_t k = 0; k < nc; ++k) order[k] = (uint32_t)k;
        return ADAGC_OK;
    }
    if (w > nc) {                                     // more parts than chunks: list order
        for (uint64_t k = 0; k < nc; ++k) order[k] = (uint32_t)k;
        return ADAGC_OK;
    }
    const uint64_t base_len = nc / w, extra = nc % w;     // the first `extra` parts are one chunk longer
    auto part_start = [&](uint64_t p) { return p * base_len + (p < extra ? p : extra); };
    auto part_len = [&](uint64_t p) { return base_len + (p < extra ? 1 : 0); };
    if (8 % w != 0) {
        // position k -> part k mod w, at offset k / w inside it
        uint64_t k = 0;
        for (uint64_t row = 0; row <= base_len; ++row)
            for (uint64_t p = 0; p < w; ++p)
                if (row < part_len(p)) order[k++] = (uint32_t)(part_start(p) + row);
        return ADAGC_OK;
    }
    // One cursor per XCD: the XCD's share index among the `share` XCDs of its part, and its position
    // inside the current run.  Positions are handed out XCD by XCD; an XCD whose part is used up is
    // skipped (this only happens in the last few positions).
    const uint64_t share = 8 / w;
    uint64_t block[8] = {0, 0, 0, 0, 0, 0, 0, 0}, within[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint64_t k = 0;
    while (k < nc) {
        for (uint64_t x = 0; x < 8 && k < nc; ++x) {
            const uint64_t p = x % w, sidx = x / w, len = part_len(p);
            uint64_t off = (block[x] * share + sidx) * R + within[x];
            if (off >= len) continue;
            order[k++] = (uint32_t)(part_start(p) + off);
            if (++within[x] == R) { within[x] = 0; ++block[x]; }
        }
    }
    return ADAGC_OK;
}
