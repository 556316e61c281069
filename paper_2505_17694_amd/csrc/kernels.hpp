// Launch interface of the gfx950 kernels (partial attention and partial-output reduction).
#pragma once

#include <cstddef>
#include <cstdint>

#include "planner.hpp"

namespace codec {

struct MergeParams {
    const float *part_o;
    const float *part_ml;
    const int32_t *req_part_off;
    const int32_t *req_part;
    const int32_t *req_inline;      // [B][1 + kInlineParts]: count, then the first rows of the list
    void *out;                      // [B][h_q][head_dim], 16-bit
    int32_t num_requests, h_q, group, part_rows;
};

struct PacParams {
    const void *q;                  // [B][h_q][head_dim], 16-bit
    const void *k_pages;
    const void *v_pages;
    int64_t page_stride, token_stride, head_stride;     // elements
    const DevTask *slot_recs;       // slot s runs the records slot_recs[slot_off[s] .. slot_off[s+1])
    const int32_t *slot_off;
    const int32_t *node_q;
    const int32_t *page_ids;
    float *part_o;                  // [h_kv][part_rows][head_dim] unnormalised partial outputs
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
    // Single-launch mode (arrive == nullptr: off).  arrive[head * num_requests + r] counts the partial
    // results of request r that tasks of KV head `head` have delivered in this launch; the workgroup
    // that delivers the last one (the count reaches the length of the request's reduction list) reduces
    // the request's rows of that head into merge.out and puts the counter back to zero.
    int32_t *arrive;
    MergeParams merge;
    // Visibility masks (nullptr: none).  nodeq_mask[e], e an index into node_q: first word in mask_words
    // of that request's mask over the node, or -1 (the node does not end the request, or no mask).
    const int32_t *nodeq_mask;
    const uint32_t *mask_words;
};


// Size of the library's own scratch array (one per GPU) behind codec_decode_attention_static.
constexpr size_t kStaticScratchBytes = size_t(64) << 20;

// Address of that array on the current device (looked up once per device); returns a hipError_t value.
int static_scratch_address(void **ptr);

// One-off kernel attributes for the current device (dynamic LDS size of the wide variant); a
// hipError_t value.  Not to be called under stream capture; launches need it to have run once.
int prepare_kernels();

// Read-only streaming kernel over `chunks` (a power of two) 4 KB chunks in the order c -> c * mult mod
// chunks (mult odd); `once` = nontemporal loads; `sink` holds one word per workgroup.
int launch_stream_read(const void *buf, uint64_t chunks, uint64_t mult, int once, int blocks, void *sink, void *stream);

// Both return a hipError_t value (0 = success) without synchronising.
// `max_rows_in_plan` selects the register-budget variant of the attention kernel.
// `head_dim`: 64, 128 or 256 (plans for 64 and 256 hold tasks of at most 16 rows).
int launch_pac(const PacParams &p, int dtype, int head_dim, int num_slots, int max_rows_in_plan, void *stream);
int launch_merge(const MergeParams &p, int dtype, int head_dim, void *stream);

}  // namespace codec
