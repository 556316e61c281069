// C ABI of the library (include/codec.h): argument checks, plan ownership, launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "codec.h"
#include "kernels.hpp"
#include "planner.hpp"

struct codec_plan {
    codec::PlanData d;
    void *device_meta = nullptr;
    int32_t max_page_id = -1;
    int32_t max_task_rows = 0;
};

namespace {

thread_local char g_last_error[256] = "";

// Records which HIP call failed and why; returns CODEC_ERR_HIP.
int hip_failure(const char *what, int code)
{
    std::snprintf(g_last_error, sizeof g_last_error, "%s: %s (%d)", what,
                  hipGetErrorString(static_cast<hipError_t>(code)), code);
    (void)hipGetLastError();        // do not leave the error for the caller's next HIP call
    return CODEC_ERR_HIP;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t part_o_bytes(const codec::PlanData &d)
{
    return align_up(size_t(d.head.num_kv_heads) * size_t(d.part_rows) * size_t(d.head.head_dim) * sizeof(float), 256);
}

size_t part_ml_bytes(const codec::PlanData &d)
{
    return align_up(size_t(d.head.num_kv_heads) * size_t(d.part_rows) * 2 * sizeof(float), 256);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int codec_plan_create(const codec_tree *tree, const codec_head_config *head,
                      const codec_plan_options *options, codec_plan_t **out)
{
    if (!tree || !head || !out) return CODEC_ERR_INVALID_ARGUMENT;
    codec_plan_options opt{};
    opt.share = 1;
    if (options) opt = *options;
    codec_plan *p = new (std::nothrow) codec_plan;
    if (!p) return CODEC_ERR_OUT_OF_MEMORY;
    int st;
    try {
        st = codec::build_best_plan(*tree, *head, opt, p->d);
    } catch (const std::bad_alloc &) {
        st = CODEC_ERR_OUT_OF_MEMORY;
    }
    if (st != CODEC_OK) {
        delete p;
        return st;
    }
    for (int32_t id : p->d.page_ids) p->max_page_id = id > p->max_page_id ? id : p->max_page_id;
    for (const codec_task &t : p->d.tasks) {
        const int32_t rows = t.n_req * p->d.group;
        p->max_task_rows = rows > p->max_task_rows ? rows : p->max_task_rows;
    }
    *out = p;
    return CODEC_OK;
}

int codec_plan_destroy(codec_plan_t *plan)
{
    delete plan;
    return CODEC_OK;
}

int codec_plan_export(const codec_plan_t *plan, codec_plan_view *v)
{
    if (!plan || !v) return CODEC_ERR_INVALID_ARGUMENT;
    const codec::PlanData &d = plan->d;
    v->num_items = int32_t(d.items.size());
    v->items = d.items.data();
    v->num_tasks = int32_t(d.tasks.size());
    v->tasks = d.tasks.data();
    v->num_slots = d.num_slots;
    v->slot_off = d.slot_off.data();
    v->slot_tasks = d.slot_tasks.data();
    v->num_nodes = d.num_nodes;
    v->node_q_off = d.node_q_off.data();
    v->node_q = d.node_q.data();
    v->num_requests = d.num_requests;
    v->req_part_off = d.req_part_off.data();
    v->req_part = d.req_part.data();
    v->cost_l = d.cost_l;
    v->makespan = d.makespan;
    v->part_rows = d.part_rows;
    v->split_align = d.split_align;
    v->max_rows = d.max_rows;
    v->share = d.share;
    v->schedule = d.schedule;
    v->fused = d.fused;
    v->num_entries = int32_t(d.queue_off.size()) - 1;
    v->queue_off = d.queue_off.data();
    v->queue_tasks = d.queue_tasks.data();
    return CODEC_OK;
}

int codec_plan_refresh_lengths(codec_plan_t *plan, const int32_t *node_len,
                               const int32_t *node_page_off, const int32_t *page_ids)
{
    if (!plan) return CODEC_ERR_INVALID_ARGUMENT;
    int st;
    try {
        st = codec::refresh_plan(plan->d, node_len, node_page_off, page_ids);
    } catch (const std::bad_alloc &) {
        return CODEC_ERR_OUT_OF_MEMORY;
    }
    if (st != CODEC_OK) return st;
    plan->device_meta = nullptr;
    plan->max_page_id = -1;
    for (int32_t id : plan->d.page_ids) plan->max_page_id = id > plan->max_page_id ? id : plan->max_page_id;
    return CODEC_OK;
}

int64_t codec_cost_estimate(const codec_cost_table *table, int32_t rows, int32_t len)
{
    if (rows < 1 || len < 1) return CODEC_ERR_INVALID_ARGUMENT;
    if (!table) return codec::builtin_cost_table(rows > 16).estimate(rows, len);
    if (table->num_row_points < 1 || table->num_len_points < 1 || !table->row_grid || !table->len_grid || !table->cost)
        return CODEC_ERR_INVALID_ARGUMENT;
    codec::CostTable t;
    try {
        t.row_grid.assign(table->row_grid, table->row_grid + table->num_row_points);
        t.len_grid.assign(table->len_grid, table->len_grid + table->num_len_points);
        t.cost.assign(table->cost, table->cost + size_t(table->num_row_points) * table->num_len_points);
    } catch (const std::bad_alloc &) {
        return CODEC_ERR_OUT_OF_MEMORY;
    }
    if (int st = t.validate()) return st;
    return t.estimate(rows, len);
}

const codec_cost_table *codec_default_cost_table(int32_t wide)
{
    auto view_of = [](bool w) {
        const codec::CostTable &t = codec::builtin_cost_table(w);
        codec_cost_table v;
        v.num_row_points = int32_t(t.row_grid.size());
        v.num_len_points = int32_t(t.len_grid.size());
        v.row_grid = t.row_grid.data();
        v.len_grid = t.len_grid.data();
        v.cost = t.cost.data();
        return v;
    };
    static const codec_cost_table views[2] = {view_of(false), view_of(true)};   // built once, never rewritten
    return &views[wide != 0];
}

size_t codec_plan_device_bytes(const codec_plan_t *plan)
{
    return plan ? plan->d.layout.total : 0;
}

int codec_plan_upload(codec_plan_t *plan, void *device_meta, size_t device_meta_bytes, void *stream)
{
    if (!plan || !device_meta) return CODEC_ERR_INVALID_ARGUMENT;
    if (device_meta_bytes < plan->d.layout.total) return CODEC_ERR_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(device_meta) & 255u) return CODEC_ERR_INVALID_ARGUMENT;
    if (int e = codec::prepare_kernels()) return hip_failure("hipFuncSetAttribute(dynamic LDS size)", e);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipError_t e = hipMemcpyAsync(device_meta, plan->d.blob.data(), plan->d.layout.total, hipMemcpyHostToDevice, s))
        return hip_failure("hipMemcpyAsync(plan metadata)", int(e));
    // the source is pageable host memory owned by the plan: wait so that it may be freed any time after
    if (hipError_t e = hipStreamSynchronize(s)) return hip_failure("hipStreamSynchronize", int(e));
    plan->device_meta = device_meta;
    return CODEC_OK;
}

size_t codec_plan_workspace_bytes(const codec_plan_t *plan)
{
    if (!plan) return 0;
    const size_t n = part_o_bytes(plan->d) + part_ml_bytes(plan->d);
    return n ? n : 256;
}

}  // extern "C"

namespace {

codec::MergeParams merge_params(const codec_plan_t *plan, const void *workspace, void *out)
{
    const codec::PlanData &d = plan->d;
    const char *meta = static_cast<const char *>(plan->device_meta);
    const codec::DevLayout &L = d.layout;
    const char *ws = static_cast<const char *>(workspace);
    codec::MergeParams mp{};
    mp.part_o = reinterpret_cast<const float *>(ws);
    mp.part_ml = reinterpret_cast<const float *>(ws + part_o_bytes(d));
    mp.req_part_off = reinterpret_cast<const int32_t *>(meta + L.req_part_off);
    mp.req_part = reinterpret_cast<const int32_t *>(meta + L.req_part);
    mp.req_inline = reinterpret_cast<const int32_t *>(meta + L.req_inline);
    mp.out = out;
    mp.num_requests = d.num_requests;
    mp.h_q = d.head.num_q_heads;
    mp.group = d.group;
    mp.part_rows = d.part_rows;
    return mp;
}

// Partial attention over the plan's tasks; with `fused_out` the launch also reduces (single-launch mode).
int partial_attention(const codec_plan_t *plan, const void *q, const void *k_pages,
                      const void *v_pages, const codec_kv_layout *layout,
                      void *workspace, size_t workspace_bytes, void *fused_out, void *stream)
{
    if (!plan || !layout) return CODEC_ERR_INVALID_ARGUMENT;
    const codec::PlanData &d = plan->d;
    if (d.num_requests == 0) return CODEC_OK;               // nothing to compute
    if (!q || !k_pages || !v_pages || !workspace) return CODEC_ERR_INVALID_ARGUMENT;
    if (!plan->device_meta) return CODEC_ERR_NOT_UPLOADED;
    if (workspace_bytes < codec_plan_workspace_bytes(plan)) return CODEC_ERR_WORKSPACE_TOO_SMALL;
    if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages)) return CODEC_ERR_INVALID_ARGUMENT;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return CODEC_ERR_INVALID_ARGUMENT;
    if (layout->num_pages <= plan->max_page_id) return CODEC_ERR_INVALID_ARGUMENT;
    if (layout->page_stride < 1 || layout->token_stride < d.head.head_dim || layout->head_stride < d.head.head_dim ||
        layout->page_stride % 8 || layout->token_stride % 8 || layout->head_stride % 8)
        return CODEC_ERR_INVALID_ARGUMENT;
    // the kernels keep a page's size in bytes, and every byte offset of a token inside its page, in 32 bits
    if (layout->page_stride > (int64_t(1) << 30) || layout->token_stride > (int64_t(1) << 30) ||
        int64_t(d.head.page_size) * layout->token_stride * 2 >= (int64_t(1) << 32))
        return CODEC_ERR_INVALID_ARGUMENT;

    const char *meta = static_cast<const char *>(plan->device_meta);
    const codec::DevLayout &L = d.layout;
    char *ws = static_cast<char *>(workspace);

    codec::PacParams pp{};
    pp.q = q;
    pp.k_pages = k_pages;
    pp.v_pages = v_pages;
    pp.page_stride = layout->page_stride;
    pp.token_stride = layout->token_stride;
    pp.head_stride = layout->head_stride;
    pp.slot_recs = reinterpret_cast<const codec::DevTask *>(meta + L.slot_recs);
    pp.slot_off = reinterpret_cast<const int32_t *>(meta + L.slot_off);
    pp.node_q = reinterpret_cast<const int32_t *>(meta + L.node_q);
    pp.page_ids = reinterpret_cast<const int32_t *>(meta + L.page_ids);
    pp.part_o = reinterpret_cast<float *>(ws);
    pp.part_ml = reinterpret_cast<float *>(ws + part_o_bytes(d));
    pp.h_q = d.head.num_q_heads;
    pp.h_kv = d.head.num_kv_heads;
    pp.group = d.group;
    pp.page_shift = 0;
    while ((1 << pp.page_shift) < d.head.page_size) ++pp.page_shift;
    pp.part_rows = d.part_rows;
    pp.scale_log2e = d.head.scale * 1.4426950408889634f;
    pp.num_slots = d.num_slots;
    if (d.schedule == 1) {
        pp.queue_off = reinterpret_cast<const int32_t *>(meta + L.queue_off);
        pp.queue_recs = reinterpret_cast<const codec::DevTask *>(meta + L.queue_recs);
        pp.counters = reinterpret_cast<int32_t *>(const_cast<char *>(meta) + L.counters);
        pp.num_entries = int32_t(d.queue_off.size()) - 1;
    }
    if (!d.req_mask_off.empty()) {
        pp.nodeq_mask = reinterpret_cast<const int32_t *>(meta + L.nodeq_mask);
        pp.mask_words = reinterpret_cast<const uint32_t *>(meta + L.mask_words);
    }
    if (fused_out) {
        pp.merge = merge_params(plan, workspace, fused_out);
        pp.arrive = reinterpret_cast<int32_t *>(const_cast<char *>(meta) + L.arrive);
    }
    if (int e = codec::launch_pac(pp, d.head.dtype, d.head.head_dim, d.num_slots, plan->max_task_rows, stream))
        return hip_failure("partial attention launch", e);
    return CODEC_OK;
}

}  // namespace

extern "C" {

int codec_partial_attention(const codec_plan_t *plan, const void *q, const void *k_pages,
                            const void *v_pages, const codec_kv_layout *layout,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    return partial_attention(plan, q, k_pages, v_pages, layout, workspace, workspace_bytes, nullptr, stream);
}

int codec_partial_reduction(const codec_plan_t *plan, const void *workspace, size_t workspace_bytes,
                            void *out, void *stream)
{
    if (!plan) return CODEC_ERR_INVALID_ARGUMENT;
    const codec::PlanData &d = plan->d;
    if (d.num_requests == 0) return CODEC_OK;
    if (!workspace || !out) return CODEC_ERR_INVALID_ARGUMENT;
    if (!plan->device_meta) return CODEC_ERR_NOT_UPLOADED;
    if (workspace_bytes < codec_plan_workspace_bytes(plan)) return CODEC_ERR_WORKSPACE_TOO_SMALL;
    if (!aligned16(out) || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return CODEC_ERR_INVALID_ARGUMENT;

    const codec::MergeParams mp = merge_params(plan, workspace, out);
    if (int e = codec::launch_merge(mp, d.head.dtype, d.head.head_dim, stream)) return hip_failure("partial reduction launch", e);
    return CODEC_OK;
}

int codec_decode_attention(const codec_plan_t *plan, const void *q, const void *k_pages,
                           const void *v_pages, const codec_kv_layout *layout, void *out,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (plan && plan->d.num_requests == 0) return layout ? CODEC_OK : CODEC_ERR_INVALID_ARGUMENT;
    if (!out || !aligned16(out)) return CODEC_ERR_INVALID_ARGUMENT;
    if (plan && plan->d.fused)          // one launch: the last workgroup to arrive at a request reduces it
        return partial_attention(plan, q, k_pages, v_pages, layout, workspace, workspace_bytes, out, stream);
    if (int st = codec_partial_attention(plan, q, k_pages, v_pages, layout, workspace, workspace_bytes, stream))
        return st;
    return codec_partial_reduction(plan, workspace, workspace_bytes, out, stream);
}

int codec_decode_attention_static(const codec_plan_t *plan, const void *q, const void *k_pages,
                                  const void *v_pages, const codec_kv_layout *layout, void *out, void *stream)
{
    if (!plan) return CODEC_ERR_INVALID_ARGUMENT;
    if (plan->d.num_requests == 0) return layout ? CODEC_OK : CODEC_ERR_INVALID_ARGUMENT;
    if (!plan->device_meta) return CODEC_ERR_NOT_UPLOADED;      // before the first HIP call of this entry point
    const size_t need = codec_plan_workspace_bytes(plan);
    if (need > codec::kStaticScratchBytes) {
        std::snprintf(g_last_error, sizeof g_last_error,
                      "codec_decode_attention_static: the plan needs %zu bytes of scratch, the library holds %zu",
                      need, codec::kStaticScratchBytes);
        return CODEC_ERR_WORKSPACE_TOO_SMALL;
    }
    void *ws = nullptr;
    if (int e = codec::static_scratch_address(&ws)) return hip_failure("hipGetSymbolAddress(scratch)", e);
    return codec_decode_attention(plan, q, k_pages, v_pages, layout, out, ws, codec::kStaticScratchBytes, stream);
}

size_t codec_static_scratch_bytes(void) { return codec::kStaticScratchBytes; }

int codec_stream_read_probe(const void *buffer, size_t bytes, int32_t pattern, int32_t nontemporal,
                            int32_t workgroups, void *sink, void *stream)
{
    if (!buffer || !sink || workgroups < 1 || workgroups > (1 << 20)) return CODEC_ERR_INVALID_ARGUMENT;
    if (pattern != 0 && pattern != 1) return CODEC_ERR_INVALID_ARGUMENT;
    if (!aligned16(buffer)) return CODEC_ERR_INVALID_ARGUMENT;
    const uint64_t chunks = bytes / 4096;
    if (chunks < 1 || (chunks & (chunks - 1)) != 0 || chunks * 4096 != bytes) return CODEC_ERR_INVALID_ARGUMENT;
    // pattern 1: chunk c of the walk is chunk c * mult mod chunks, an odd multiplier near chunks / phi
    const uint64_t mult = pattern == 0 ? 1 : ((uint64_t(double(chunks) * 0.6180339887498949) | 1u));
    if (int e = codec::launch_stream_read(buffer, chunks, mult, nontemporal != 0, workgroups, sink, stream))
        return hip_failure("stream read launch", e);
    return CODEC_OK;
}

const char *codec_last_error_message(void) { return g_last_error; }

const char *codec_status_string(int status)
{
    switch (status) {
    case CODEC_OK: return "ok";
    case CODEC_ERR_INVALID_ARGUMENT: return "invalid argument";
    case CODEC_ERR_INVALID_TREE: return "invalid tree";
    case CODEC_ERR_UNSUPPORTED: return "unsupported configuration";
    case CODEC_ERR_WORKSPACE_TOO_SMALL: return "buffer too small";
    case CODEC_ERR_HIP: return "HIP runtime error";
    case CODEC_ERR_NOT_UPLOADED: return "plan metadata not uploaded";
    case CODEC_ERR_OUT_OF_MEMORY: return "out of host memory";
    default: return "unknown status";
    }
}

}  // extern "C"
