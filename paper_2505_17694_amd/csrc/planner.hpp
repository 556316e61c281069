// Host-side workload balancer: forest indexing, cost estimation, KV division and
// slot scheduling (paper Sec. 4.1 indexes, Sec. 5 Eq. 3-7).  Pure C++, no HIP.
#pragma once

#include <cstdint>
#include <vector>

#include "codec.h"

namespace codec {

// Profiled cost table with integer bilinear interpolation (Sec. 5.2, Eq. 6).
struct CostTable {
    std::vector<int32_t> row_grid;
    std::vector<int32_t> len_grid;
    std::vector<int64_t> cost;          // [row][len]

    int validate() const;
    int64_t estimate(int64_t rows, int64_t len) const;
};

// A task of at most kSoloMaxRows rows and kSoloMaxLen tokens may be run by a single wave; the kernels
// take runs of such tasks in a slot's list one wave each (see solo_run below).
constexpr int32_t kSoloMaxRows = 16;
// Most rows of a task with `head_dim` channels: 256 in the dense task shape, which exists for 128 channels;
// otherwise what the stream shape holds, two row tiles of 16 with 64 channels and one with 256.
constexpr int32_t max_task_rows(int32_t head_dim) { return head_dim == 128 ? 256 : head_dim == 64 ? 32 : 16; }
constexpr int32_t kSoloMaxLen = 2048;
// Most short tasks in one entry of the run-time queue (measured on cfg3/cfg4: 2 costs fetches, 8 and
// more make the last entries long).
constexpr int32_t kQueueBundle = 4;
// schedule = 2 takes the run-time queue from this many entries per slot on.
constexpr int32_t kAutoQueueEntriesPerSlot = 6;
// fused = 2 reduces inside the attention launch when the estimated makespan (ns) is below this: where a
// second launch (about 5 us with the gap in front of it) is a large part of the step.
constexpr int64_t kAutoFusedMakespanNs = 40000;
// ... and when the batch has at most this many query rows per KV head (requests x group).
constexpr int64_t kAutoFusedMaxRows = 64;

// Task record as the kernels read it (32 bytes).  The device image holds the records twice: in the
// order of the slots' lists and in the order of the run-time queue, so that a workgroup reads record
// i of its list directly instead of through an index (a task's start is a chain of dependent reads,
// each of which costs microseconds when the memory system is busy).
struct DevTask {
    int32_t page_off;       // index into the device copy of page_ids of the slice's first page
    int32_t kv_len;         // tokens in the slice
    int32_t q_off;          // first request of the task in node_q
    int32_t n_req;          // requests in the task
    int32_t part_row_base;  // first partial row
    int32_t solo_run;       // number of consecutive single-wave tasks in the slot's list from this one on
    int32_t flags;          // kTaskReadOnce: no other task reads this KV slice (its node has a single row
                            // tile); kTaskMasked: some request of the task has a visibility mask over this node
    int32_t single_req;     // n_req == 1: the request itself (saves the read of node_q); else -1
};

enum : int32_t { kTaskReadOnce = 1, kTaskMasked = 2 };

// Per request, the reduction kernel reads one 64-byte line: the number of partial rows on the request's
// path and, if there are at most kInlineParts of them, the rows themselves; longer lists are read
// from the CSR arrays.  One dependent read less than offset -> list -> partial rows.
constexpr int32_t kInlineParts = 15;

// Byte offsets of the arrays inside the device metadata blob.
struct DevLayout {
    size_t slot_recs = 0, slot_off = 0, node_q = 0, page_ids = 0,
           req_part_off = 0, req_part = 0, req_inline = 0, queue_off = 0, queue_recs = 0, counters = 0,
           arrive = 0,      // [h_kv][num_requests] partial results arrived (single-launch mode), zero between launches
           nodeq_mask = 0,  // per entry of node_q: first word of that request's mask if the node ends the request, else -1
           mask_words = 0,
           total = 0;
};

struct PlanData {
    codec_head_config head{};
    int32_t group = 1;
    int32_t num_slots = 0, split_align = 0, max_rows = 0, share = 1, schedule = 0, fused = 0;
    int32_t num_nodes = 0, num_requests = 0;

    std::vector<int32_t> node_len, node_page_off, page_ids;
    std::vector<int32_t> node_q_off, node_q;
    std::vector<int32_t> req_node;                  // last node of every request
    std::vector<int32_t> req_mask_off;              // empty: no visibility masks
    std::vector<uint32_t> req_mask;
    std::vector<codec_item> items;
    std::vector<codec_task> tasks;
    std::vector<int32_t> slot_off, slot_tasks;
    std::vector<int32_t> queue_off, queue_tasks;    // run-time queue: entries in longest-first order
    std::vector<int32_t> req_part_off, req_part;
    int64_t cost_l = 0, makespan = 0;
    int32_t part_rows = 0;

    CostTable table;                    // the table the plan was estimated with (for refresh_plan)

    DevLayout layout;
    std::vector<unsigned char> blob;    // host image of the device metadata
};

const CostTable &builtin_cost_table(bool wide);

// Fills `plan` from the caller's forest; returns a CODEC_* status.
int build_plan(const codec_tree &tree, const codec_head_config &head,
               const codec_plan_options &opt, PlanData &plan);

// options.share == 2: builds the candidate plans named in codec.h and keeps the one with the lowest
// estimated makespan (ties: the earlier candidate).  Other values: build_plan.
int build_best_plan(const codec_tree &tree, const codec_head_config &head,
                    const codec_plan_options &opt, PlanData &plan);

// Carries `plan` over to new node lengths and page lists without dividing or scheduling again (the
// paper divides tasks only every few decoding steps: Implementation section, task division module):
// slices keep their boundaries, a node's last slice takes up the change in length, costs and the
// makespan are re-estimated, the device image is rebuilt.  On error `plan` is left as it was.
int refresh_plan(PlanData &plan, const int32_t *node_len, const int32_t *node_page_off, const int32_t *page_ids);

}  // namespace codec
