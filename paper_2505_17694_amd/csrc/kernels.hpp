// Launch interface of the gfx950 kernels (partial attention and partial-output reduction).
#pragma once

#include <cstdint>

#include "planner.hpp"

namespace codec {

struct PacParams {
    const void *q;                  // [B][h_q][128], 16-bit
    const void *k_pages;
    const void *v_pages;
    int64_t page_stride, token_stride, head_stride;     // elements
    const DevTask *slot_recs;       // slot s runs the records slot_recs[slot_off[s] .. slot_off[s+1])
    const int32_t *slot_off;
    const int32_t *node_q;
    const int32_t *page_ids;
    float *part_o;                  // [h_kv][part_rows][128] unnormalised partial outputs
    float *part_ml;                 // [h_kv][part_rows][2]   (max in log2 units, sum of exponentials)
    int32_t h_q, h_kv, group, page_shift, part_rows;    // page_shift = log2(tokens per page)
    float scale_log2e;              // scale * log2(e): scores are kept in log2 units
    // Run-time queue (queue_off == nullptr: static slot lists).  Entry e holds the records
    // queue_recs[queue_off[e] .. queue_off[e+1]); counters[2*head] counts the entries taken beyond the
    // first num_slots, counters[2*head + 1] the workgroups of the head that have finished.  The last
    // workgroup to finish puts both back to zero.
    const int32_t *queue_off;
    const DevTask *queue_recs;
    int32_t *counters;
    int32_t num_entries, num_slots;
};

struct MergeParams {
    const float *part_o;
    const float *part_ml;
    const int32_t *req_part_off;
    const int32_t *req_part;
    const int32_t *req_inline;      // [B][1 + kInlineParts]: count, then the first rows of the list
    void *out;                      // [B][h_q][128], 16-bit
    int32_t num_requests, h_q, group, part_rows;
};

// Both return a hipError_t value (0 = success) without synchronising.
// `max_rows_in_plan` selects the register-budget variant of the attention kernel.
int launch_pac(const PacParams &p, int dtype, int num_slots, int max_rows_in_plan, void *stream);
int launch_merge(const MergeParams &p, int dtype, void *stream);

}  // namespace codec
