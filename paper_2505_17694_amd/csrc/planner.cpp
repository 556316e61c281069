// Host-side workload balancer (paper Sec. 5).  See planner.hpp.
//
// The paper states the solver in prose (Sec. 5.1): fix b_q = 1, find a lower
// bound cost_l of the makespan by binary search on the average-load inequality
// (Eq. 4), bound every node's slice count by ceil(C_est / cost_l) (Eq. 5), grid
// search the slice counts and schedule greedily.  Everything it leaves open is
// fixed here in integers so that the result can be re-derived bit for bit:
// integer costs, round-half-up bilinear interpolation, slices of equal length
// on aligned boundaries, one grid-search pass in order of decreasing node cost
// with ties to fewer slices, longest-first scheduling with ties to the lower
// slot id.  Two extensions of that solver (a slice of slack over Eq. 5, extra
// search points on the diagonal of the grid) are options, off unless asked for.
#include "planner.hpp"

#include <algorithm>
#include <cstring>
#include <queue>

namespace codec {

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Position of x on an ascending grid: neighbours i0, i1 and the weight num/den of i1.
struct Bracket {
    int i0, i1;
    int64_t num, den;
};

Bracket bracket(const std::vector<int32_t> &grid, int64_t x)
{
    const int k = static_cast<int>(grid.size());
    if (k == 1 || x <= grid[0]) return {0, 0, 0, 1};            // clamp below the grid
    if (x >= grid[k - 1])                                        // continue the last segment
        return {k - 2, k - 1, x - grid[k - 2], int64_t(grid[k - 1]) - grid[k - 2]};
    int i = static_cast<int>(std::upper_bound(grid.begin(), grid.end(), x) - grid.begin()) - 1;
    return {i, i + 1, x - grid[i], int64_t(grid[i + 1]) - grid[i]};
}

// A KV slice layout: `count` slices of `length` tokens, the last one `last` tokens.
struct Slicing {
    int32_t count, length, last;
};

Slicing slice_node(int64_t len, int64_t want, int64_t align)
{
    const int64_t length = align * ceil_div(ceil_div(len, want), align);
    const int64_t count = ceil_div(len, length);
    return {int32_t(count), int32_t(length), int32_t(len - (count - 1) * length)};
}

struct Sub {
    int64_t cost;
    int32_t item, chunk, begin, len;
};

struct Schedule {
    int64_t makespan = 0;
    std::vector<int32_t> slot_of;                   // per subtask
    std::vector<std::vector<int32_t>> lists;        // per slot, assignment order
};

// Longest-processing-time-first list scheduling onto m slots.
void schedule_lpt(const std::vector<Sub> &sub, int m, bool keep_lists, Schedule &out)
{
    std::vector<int32_t> order(sub.size());
    for (size_t i = 0; i < sub.size(); ++i) order[i] = int32_t(i);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (sub[a].cost != sub[b].cost) return sub[a].cost > sub[b].cost;
        if (sub[a].item != sub[b].item) return sub[a].item < sub[b].item;
        return sub[a].chunk < sub[b].chunk;
    });
    using Load = std::pair<int64_t, int32_t>;       // (load, slot): smallest load, then lowest slot
    std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
    for (int s = 0; s < m; ++s) heap.push({0, s});
    if (keep_lists) {
        out.slot_of.assign(sub.size(), 0);
        out.lists.assign(m, {});
    }
    int64_t makespan = 0;
    for (int32_t i : order) {
        Load l = heap.top();
        heap.pop();
        l.first += sub[i].cost;
        makespan = std::max(makespan, l.first);
        if (keep_lists) {
            out.slot_of[i] = l.second;
            out.lists[l.second].push_back(i);
        }
        heap.push(l);
    }
    out.makespan = makespan;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Host image of the device metadata: task records, slot lists, query lists, page table, partial lists.
void build_device_image(PlanData &p)
{
    const int32_t ps = p.head.page_size;
    DevLayout &L = p.layout;
    size_t off = 0;
    auto place = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    L.slot_recs = place(p.slot_tasks.size() * sizeof(DevTask));
    L.slot_off = place(p.slot_off.size() * 4);
    L.node_q = place(p.node_q.size() * 4);
    L.page_ids = place(p.page_ids.size() * 4);
    L.req_part_off = place(p.req_part_off.size() * 4);
    L.req_part = place(p.req_part.size() * 4);
    L.req_inline = place(size_t(p.num_requests) * (kInlineParts + 1) * 4);
    // Run-time queue.  Short tasks (the ones a single wave runs) are bundled, in order of decreasing
    // cost, into entries that a workgroup hands out one wave each, like a run of short tasks in a
    // slot's list; every other task is an entry of its own.  The bundle size is the smallest that lets
    // every entry have a workgroup of its own (then no entry is ever fetched at run time and the queue
    // costs nothing), at most kQueueBundle.  Entries are ordered by decreasing cost, a bundle counting
    // as the sum of its tasks, ties to the entry with the lower first task: the order in which the
    // greedy schedule would deal them.
    {
        std::vector<int32_t> order(p.tasks.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = int32_t(i);
        std::stable_sort(order.begin(), order.end(),
                         [&](int32_t a, int32_t b) { return p.tasks[a].cost > p.tasks[b].cost; });
        auto is_short = [&](int32_t i) {
            return p.tasks[i].n_req * p.group <= kSoloMaxRows && p.tasks[i].kv_len <= kSoloMaxLen;
        };
        int64_t n_short = 0;
        for (int32_t i : order) n_short += is_short(i);
        const int64_t n_long = int64_t(order.size()) - n_short;
        int64_t bundle = kQueueBundle;
        if (n_long < p.num_slots) bundle = std::min<int64_t>(kQueueBundle, std::max<int64_t>(1, ceil_div(n_short, p.num_slots - n_long)));
        struct Entry { int64_t cost; std::vector<int32_t> tasks; };
        std::vector<Entry> entries;
        int64_t open_bundle = -1;
        for (int32_t i : order) {
            if (is_short(i) && open_bundle >= 0 && int64_t(entries[open_bundle].tasks.size()) < bundle) {
                entries[open_bundle].tasks.push_back(i);
                entries[open_bundle].cost += p.tasks[i].cost;
                continue;
            }
            entries.push_back({p.tasks[i].cost, {i}});
            open_bundle = is_short(i) ? int64_t(entries.size()) - 1 : open_bundle;
            if (is_short(i) && bundle == 1) open_bundle = -1;
        }
        std::stable_sort(entries.begin(), entries.end(), [](const Entry &a, const Entry &b) { return a.cost > b.cost; });
        p.queue_off.assign(1, 0);
        p.queue_tasks.clear();
        for (const Entry &e : entries) {
            p.queue_tasks.insert(p.queue_tasks.end(), e.tasks.begin(), e.tasks.end());
            p.queue_off.push_back(int32_t(p.queue_tasks.size()));
        }
    }
    if (p.schedule == 2)
        p.schedule = int64_t(p.queue_off.size()) - 1 >= int64_t(kAutoQueueEntriesPerSlot) * p.num_slots ? 1 : 0;
    L.queue_off = place(p.queue_off.size() * 4);
    L.queue_recs = place(p.queue_tasks.size() * sizeof(DevTask));
    L.counters = place(size_t(p.head.num_kv_heads) * 2 * 4);               // zero: nothing taken, nobody done
    L.arrive = place(size_t(p.head.num_kv_heads) * size_t(p.num_requests) * 4);   // zero: nothing arrived
    const bool masks = !p.req_mask_off.empty();
    L.nodeq_mask = place(masks ? p.node_q.size() * 4 : 0);
    L.mask_words = place(masks ? p.req_mask.size() * 4 : 0);
    // one workgroup may end up last for every request: more query rows than a workgroup reduces in a
    // few rounds make the single launch slower than two (cfg2, 256 rows per KV head: 89 against 26 us)
    if (p.fused == 2)
        p.fused = p.makespan < kAutoFusedMakespanNs && int64_t(p.num_requests) * p.group <= kAutoFusedMaxRows ? 1 : 0;
    L.total = std::max<size_t>(off, 256);
    p.blob.assign(L.total, 0);
    // Streaming hint (kernels.hip): a task reads its slice with it when no other task reads that slice
    // (its node has one item: one row tile, or one request of a flat plan) and the plan as a whole reads
    // little twice (tokens read <= 1.25 x tokens held).  Measured on MI355X: plans that re-read a lot,
    // like the flat plan of a tree with shared prefixes, lose up to 15 % when their single-reader
    // slices carry the hint, plans that read everything about once gain up to 12 %.
    std::vector<int32_t> readers(size_t(p.num_nodes), 0);
    for (const codec_item &it : p.items) ++readers[it.node];
    int64_t tokens_read = 0, tokens_held = 0;
    for (const codec_task &t : p.tasks) tokens_read += t.kv_len;
    for (int32_t len : p.node_len) tokens_held += len;
    const bool streaming_plan = 4 * tokens_read <= 5 * tokens_held;
    // visibility masks: which (node, request) entries carry one (the node ends the request)
    std::vector<int32_t> nodeq_mask;
    if (masks) {
        nodeq_mask.assign(p.node_q.size(), -1);
        for (int32_t n = 0; n < p.num_nodes; ++n)
            for (int32_t e = p.node_q_off[n]; e < p.node_q_off[n + 1]; ++e) {
                const int32_t r = p.node_q[e];
                if (p.req_node[r] == n && p.req_mask_off[r + 1] > p.req_mask_off[r]) nodeq_mask[e] = p.req_mask_off[r];
            }
    }
    auto record = [&](int32_t i) {
        const codec_task &t = p.tasks[i];
        DevTask r{};
        r.page_off = p.node_page_off[t.node] + t.kv_begin / ps;
        r.kv_len = t.kv_len;
        r.q_off = t.q_off;
        r.n_req = t.n_req;
        r.part_row_base = t.part_row_base;
        r.solo_run = 0;
        r.flags = streaming_plan && readers[t.node] == 1 ? kTaskReadOnce : 0;
        if (masks)
            for (int32_t e = t.q_off; e < t.q_off + t.n_req; ++e)
                if (nodeq_mask[e] >= 0) r.flags |= kTaskMasked;
        r.single_req = t.n_req == 1 ? p.node_q[t.q_off] : -1;
        return r;
    };
    // A slot's records in the order the workgroup runs them: the tasks that need the whole workgroup
    // first, then the single-wave tasks as one run (both in the order of the slot's list, which is by
    // decreasing cost).  Every run ends with waves waiting for the last one; one run per slot pays that
    // once, at the end of the launch, where the short tasks also even out what the long ones left.
    DevTask *by_slot = reinterpret_cast<DevTask *>(p.blob.data() + L.slot_recs);
    auto is_short = [&](int32_t i) {
        return p.tasks[i].n_req * p.group <= kSoloMaxRows && p.tasks[i].kv_len <= kSoloMaxLen;
    };
    for (int32_t sl = 0; sl < p.num_slots; ++sl) {
        std::vector<int32_t> order(p.slot_tasks.begin() + p.slot_off[sl], p.slot_tasks.begin() + p.slot_off[sl + 1]);
        std::stable_partition(order.begin(), order.end(), [&](int32_t i) { return !is_short(i); });
        int32_t run = 0;
        for (int32_t k = int32_t(order.size()) - 1; k >= 0; --k) {       // runs of single-wave tasks, back to front
            DevTask &r = by_slot[p.slot_off[sl] + k];
            r = record(order[k]);
            run = is_short(order[k]) ? run + 1 : 0;
            r.solo_run = run;
        }
    }
    DevTask *by_entry = reinterpret_cast<DevTask *>(p.blob.data() + L.queue_recs);
    for (size_t i = 0; i < p.queue_tasks.size(); ++i) by_entry[i] = record(p.queue_tasks[i]);
    auto put = [&](size_t at, const std::vector<int32_t> &v) {
        if (!v.empty()) std::memcpy(p.blob.data() + at, v.data(), v.size() * 4);
    };
    put(L.slot_off, p.slot_off);
    put(L.node_q, p.node_q);
    put(L.page_ids, p.page_ids);
    put(L.req_part_off, p.req_part_off);
    put(L.req_part, p.req_part);
    {
        int32_t *line = reinterpret_cast<int32_t *>(p.blob.data() + L.req_inline);
        for (int32_t r = 0; r < p.num_requests; ++r, line += kInlineParts + 1) {
            const int32_t e0 = p.req_part_off[r], cnt = p.req_part_off[r + 1] - e0;
            line[0] = cnt;
            for (int32_t j = 0; j < kInlineParts; ++j) line[1 + j] = j < cnt ? p.req_part[e0 + j] : 0;
        }
    }
    put(L.queue_off, p.queue_off);
    if (masks) {
        put(L.nodeq_mask, nodeq_mask);
        if (!p.req_mask.empty()) std::memcpy(p.blob.data() + L.mask_words, p.req_mask.data(), p.req_mask.size() * 4);
    }
}

}  // namespace

int CostTable::validate() const
{
    if (row_grid.empty() || len_grid.empty()) return CODEC_ERR_INVALID_ARGUMENT;
    if (cost.size() != row_grid.size() * len_grid.size()) return CODEC_ERR_INVALID_ARGUMENT;
    for (size_t i = 0; i < row_grid.size(); ++i)
        if (row_grid[i] < 1 || (i && row_grid[i] <= row_grid[i - 1])) return CODEC_ERR_INVALID_ARGUMENT;
    for (size_t i = 0; i < len_grid.size(); ++i)
        if (len_grid[i] < 1 || (i && len_grid[i] <= len_grid[i - 1])) return CODEC_ERR_INVALID_ARGUMENT;
    for (int64_t c : cost)
        if (c < 1 || c > (int64_t(1) << 40)) return CODEC_ERR_INVALID_ARGUMENT;
    return CODEC_OK;
}

int64_t CostTable::estimate(int64_t rows, int64_t len) const
{
    const Bracket r = bracket(row_grid, rows), n = bracket(len_grid, len);
    const size_t nl = len_grid.size();
    auto c = [&](int ri, int ni) { return static_cast<__int128>(cost[ri * nl + ni]); };
    const __int128 wr1 = r.num, wr0 = r.den - r.num, wn1 = n.num, wn0 = n.den - n.num;
    const __int128 num = wr0 * wn0 * c(r.i0, n.i0) + wr1 * wn0 * c(r.i1, n.i0)
                       + wr0 * wn1 * c(r.i0, n.i1) + wr1 * wn1 * c(r.i1, n.i1);
    const __int128 den = static_cast<__int128>(r.den) * n.den;
    if (num <= 0) return 1;
    const __int128 v = (num + den / 2) / den;
    return v < 1 ? 1 : static_cast<int64_t>(v);
}

// Built-in tables: cost in ns of one task inside a busy persistent workgroup, measured on an MI355X
// with the profiler of the Python package (one launch with three tasks per slot minus one launch with
// one task per slot, halved; every slot and KV head busy, K/V cold).  The kernel has two launch
// variants with different workgroup shapes, hence two tables: `wide` for plans that hold a task of
// more than 16 rows, `narrow` for the others.  The numbers come straight from the profiler's output:
// the build writes cost_table_generated.inc from cost_table_mi355x.json.
const CostTable &builtin_cost_table(bool wide)
{
#include "cost_table_generated.inc"
    return wide ? wide_table : narrow_table;
}

int build_plan(const codec_tree &tree, const codec_head_config &head,
               const codec_plan_options &opt, PlanData &p)
{
    // ---- argument checks ------------------------------------------------------------
    if (tree.num_nodes < 0 || tree.num_requests < 0) return CODEC_ERR_INVALID_ARGUMENT;
    if (tree.num_requests > 0 && tree.num_nodes == 0) return CODEC_ERR_INVALID_TREE;
    if (tree.num_nodes > 0 && (!tree.parent || !tree.node_len || !tree.node_page_off))
        return CODEC_ERR_INVALID_ARGUMENT;
    if (tree.num_requests > 0 && !tree.req_node) return CODEC_ERR_INVALID_ARGUMENT;
    if (head.num_q_heads < 1 || head.num_kv_heads < 1) return CODEC_ERR_INVALID_ARGUMENT;
    if (head.num_q_heads % head.num_kv_heads != 0) return CODEC_ERR_INVALID_ARGUMENT;
    if (head.head_dim != 64 && head.head_dim != 128 && head.head_dim != 256) return CODEC_ERR_UNSUPPORTED;
    if (head.dtype != CODEC_DTYPE_FP16 && head.dtype != CODEC_DTYPE_BF16) return CODEC_ERR_UNSUPPORTED;
    if (head.page_size < 16 || head.page_size > 4096 || (head.page_size & (head.page_size - 1)) != 0)
        return CODEC_ERR_UNSUPPORTED;
    if (!(head.scale > 0.0f) || !(head.scale < 1e30f)) return CODEC_ERR_INVALID_ARGUMENT;
    const int32_t group = head.num_q_heads / head.num_kv_heads;
    if (group > 64) return CODEC_ERR_UNSUPPORTED;

    const int32_t align = opt.split_align > 0 ? opt.split_align : std::max(256, head.page_size);
    int32_t max_rows = opt.max_rows > 0 ? opt.max_rows : std::max(256, group);
    if (head.head_dim != 128) {
        // 64 and 256 channels run in the stream task shape only: row tiles of at most 32 and 16 rows
        if (group > kSoloMaxRows) return CODEC_ERR_UNSUPPORTED;
        const int32_t tile = max_task_rows(head.head_dim);
        max_rows = std::min(max_rows, std::max(group, tile / group * group));
    }
    if (opt.num_slots < 0 || opt.split_align < 0 || opt.max_rows < 0) return CODEC_ERR_INVALID_ARGUMENT;
    if (opt.num_slots > (1 << 20)) return CODEC_ERR_INVALID_ARGUMENT;
    if (align % 32 != 0 || align % head.page_size != 0) return CODEC_ERR_INVALID_ARGUMENT;
    if (max_rows > 256 || max_rows < group) return CODEC_ERR_INVALID_ARGUMENT;
    if (opt.share != 0 && opt.share != 1) return CODEC_ERR_INVALID_ARGUMENT;
    if (opt.fixed_slices < 0) return CODEC_ERR_INVALID_ARGUMENT;
    if (opt.schedule < 0 || opt.schedule > 2) return CODEC_ERR_INVALID_ARGUMENT;
    if (opt.fused < 0 || opt.fused > 2) return CODEC_ERR_INVALID_ARGUMENT;
    if (opt.extensions < 0 || opt.extensions > (CODEC_PLAN_EXT_SLACK | CODEC_PLAN_EXT_DIAGONAL))
        return CODEC_ERR_INVALID_ARGUMENT;
    const bool ext_slack = (opt.extensions & CODEC_PLAN_EXT_SLACK) != 0;
    const bool ext_diagonal = (opt.extensions & CODEC_PLAN_EXT_DIAGONAL) != 0;

    CostTable user;
    const CostTable *table = nullptr;           // nullptr: the built-in table of the kernel variant
    if (opt.cost) {
        const codec_cost_table &c = *opt.cost;
        if (c.num_row_points < 1 || c.num_len_points < 1 || !c.row_grid || !c.len_grid || !c.cost)
            return CODEC_ERR_INVALID_ARGUMENT;
        user.row_grid.assign(c.row_grid, c.row_grid + c.num_row_points);
        user.len_grid.assign(c.len_grid, c.len_grid + c.num_len_points);
        user.cost.assign(c.cost, c.cost + size_t(c.num_row_points) * c.num_len_points);
        if (int st = user.validate()) return st;
        table = &user;
    }

    const int32_t N = tree.num_nodes, B = tree.num_requests;

    // ---- forest checks --------------------------------------------------------------
    for (int32_t i = 0; i < N; ++i) {
        if (tree.parent[i] < -1 || tree.parent[i] >= N || tree.parent[i] == i) return CODEC_ERR_INVALID_TREE;
        if (tree.node_len[i] < 1) return CODEC_ERR_INVALID_TREE;
    }
    {   // cycles anywhere in the parent array: colour walk (0 new, 1 on the current walk, 2 cleared)
        std::vector<uint8_t> colour(N, 0);
        std::vector<int32_t> walk;
        for (int32_t s = 0; s < N; ++s) {
            walk.clear();
            int32_t n = s;
            while (n != -1 && colour[n] == 0) {
                colour[n] = 1;
                walk.push_back(n);
                n = tree.parent[n];
            }
            if (n != -1 && colour[n] == 1) return CODEC_ERR_INVALID_TREE;
            for (int32_t v : walk) colour[v] = 2;
        }
    }
    if (N > 0) {
        if (tree.node_page_off[0] < 0) return CODEC_ERR_INVALID_TREE;
        for (int32_t i = 0; i < N; ++i) {
            const int64_t have = int64_t(tree.node_page_off[i + 1]) - tree.node_page_off[i];
            if (have < ceil_div(tree.node_len[i], head.page_size)) return CODEC_ERR_INVALID_TREE;
        }
        if (tree.node_page_off[N] > 0 && !tree.page_ids) return CODEC_ERR_INVALID_ARGUMENT;
        for (int32_t i = tree.node_page_off[0]; i < tree.node_page_off[N]; ++i)
            if (tree.page_ids[i] < 0) return CODEC_ERR_INVALID_TREE;
    }
    for (int32_t r = 0; r < B; ++r)
        if (tree.req_node[r] < 0 || tree.req_node[r] >= N) return CODEC_ERR_INVALID_TREE;
    // visibility masks over the requests' last nodes (Sec. 4.1)
    std::vector<uint8_t> ends_masked(N, 0);         // the node is the last node of a masked request
    if (tree.req_mask_off) {
        if (group > kSoloMaxRows) return CODEC_ERR_UNSUPPORTED;
        if (tree.req_mask_off[0] != 0) return CODEC_ERR_INVALID_TREE;
        for (int32_t r = 0; r < B; ++r) {
            const int64_t words = int64_t(tree.req_mask_off[r + 1]) - tree.req_mask_off[r];
            if (words == 0) continue;
            const int32_t len = tree.node_len[tree.req_node[r]];
            if (words != ceil_div(len, 32) || !tree.req_mask) return CODEC_ERR_INVALID_TREE;
            bool sees = false;
            for (int32_t t = 0; t < len && !sees; ++t)
                sees = (tree.req_mask[tree.req_mask_off[r] + t / 32] >> (t % 32)) & 1u;
            if (!sees) return CODEC_ERR_INVALID_TREE;
            ends_masked[tree.req_node[r]] = 1;
        }
        p.req_mask_off.assign(tree.req_mask_off, tree.req_mask_off + B + 1);
        if (tree.req_mask_off[B] > 0) p.req_mask.assign(tree.req_mask, tree.req_mask + tree.req_mask_off[B]);
    }
    p.req_node.assign(tree.req_node, tree.req_node + B);

    p.head = head;
    p.group = group;
    p.split_align = align;
    p.max_rows = max_rows;
    p.share = opt.share;
    p.schedule = opt.schedule;
    p.fused = opt.fused;
    p.num_nodes = N;
    p.num_requests = B;
    p.node_len.assign(tree.node_len, tree.node_len + N);
    p.node_page_off.assign(tree.node_page_off, tree.node_page_off + (N ? N + 1 : 0));
    if (N) p.page_ids.assign(tree.page_ids, tree.page_ids + tree.node_page_off[N]);

    // ---- a1: prefix paths and per-node query sets (Sec. 4.1) ------------------------------
    std::vector<std::vector<int32_t>> paths(B);
    std::vector<int32_t> n_q(N, 0);
    for (int32_t r = 0; r < B; ++r) {
        for (int32_t n = tree.req_node[r]; n != -1; n = tree.parent[n]) paths[r].push_back(n);
        std::reverse(paths[r].begin(), paths[r].end());
        for (int32_t n : paths[r]) ++n_q[n];
    }
    p.node_q_off.assign(N + 1, 0);
    for (int32_t i = 0; i < N; ++i) p.node_q_off[i + 1] = p.node_q_off[i] + n_q[i];
    p.node_q.assign(p.node_q_off[N], 0);
    {
        std::vector<int32_t> fill(p.node_q_off.begin(), p.node_q_off.end() - 1);
        for (int32_t r = 0; r < B; ++r)           // ascending r keeps every list sorted
            for (int32_t n : paths[r]) p.node_q[fill[n]++] = r;
    }

    // ---- work items: a node with (a row tile of) its queries -------------------------------
    // requests per work item: row tiles of max_rows; a node that ends a masked request takes tiles of at
    // most 16 rows (the task shape that applies masks) and is not divided along KV
    std::vector<int32_t> qpt_of(N, p.share ? std::max(1, max_rows / group) : 1);
    for (int32_t n = 0; n < N; ++n)
        if (ends_masked[n]) qpt_of[n] = std::min(qpt_of[n], std::max(1, kSoloMaxRows / group));
    std::vector<int32_t> first_item(N, 0);
    for (int32_t n = 0; n < N; ++n) {
        first_item[n] = int32_t(p.items.size());
        const int32_t qpt = qpt_of[n];
        for (int32_t a = 0; a < n_q[n]; a += qpt) {
            codec_item it{};
            it.node = n;
            it.q_off = p.node_q_off[n] + a;
            it.n_req = std::min(qpt, n_q[n] - a);
            it.rows = it.n_req * group;
            it.len = p.node_len[n];
            p.items.push_back(it);
        }
    }
    const size_t J = p.items.size();
    // kernel variant: a task above 16 rows needs the wide one (one workgroup per CU, 256 CUs);
    // otherwise two narrow workgroups share a CU.  It fixes the default slot count and cost table.
    int32_t widest = 0;
    for (const codec_item &it : p.items) widest = std::max(widest, it.rows);
    const bool wide = widest > 16 && head.head_dim == 128;
    const int32_t m = opt.num_slots > 0 ? opt.num_slots : std::max(1, (wide ? 256 : 512) / head.num_kv_heads);
    p.num_slots = m;
    if (!table) table = &builtin_cost_table(wide);
    p.table = *table;
    for (codec_item &it : p.items) it.cost = table->estimate(it.rows, it.len);       // a2: Eq. 6
    std::vector<int64_t> max_b(J);
    for (size_t j = 0; j < J; ++j) max_b[j] = ends_masked[p.items[j].node] ? 1 : ceil_div(p.items[j].len, align);

    auto slices_at = [&](size_t j, int64_t T) {
        return std::min(ceil_div(p.items[j].cost, T), max_b[j]);
    };
    auto division_cost = [&](size_t j, int64_t want) {
        const Slicing s = slice_node(p.items[j].len, want, align);
        return int64_t(s.count - 1) * table->estimate(p.items[j].rows, s.length)
               + table->estimate(p.items[j].rows, s.last);
    };

    // ---- a3: lower bound cost_l (Eq. 4) by binary search, upper bounds (Eq. 5) ----------------
    p.cost_l = 0;
    if (J) {
        int64_t biggest = 0, sum = 0;
        for (const codec_item &it : p.items) {
            biggest = std::max(biggest, it.cost);
            sum += it.cost;
        }
        int64_t lo = 1, hi = std::max(biggest, ceil_div(sum, m));
        while (lo < hi) {
            const int64_t mid = lo + (hi - lo) / 2;
            __int128 total = 0;
            for (size_t j = 0; j < J; ++j) total += division_cost(j, slices_at(j, mid));
            if (total <= static_cast<__int128>(m) * mid) hi = mid; else lo = mid + 1;
        }
        p.cost_l = lo;
    }
    // Eq. 5 prunes the search (most nodes cost far less than the average load and stay whole).
    // Extension (CODEC_PLAN_EXT_SLACK, not in the paper): a node whose cost is at least a quarter of
    // cost_l may take one slice more than the quotient: without it a few nodes of 0.3 .. 1 average
    // loads cannot be packed evenly onto the slots.
    for (size_t j = 0; j < J; ++j) {
        int64_t want = slices_at(j, p.cost_l);
        if (ext_slack && 4 * p.items[j].cost >= p.cost_l) want = std::min(want + 1, max_b[j]);
        p.items[j].ub = slice_node(p.items[j].len, want, align).count;
        p.items[j].b = p.items[j].ub;
    }

    // ---- grid search over slice counts, evaluated by the greedy schedule ---------------------
    std::vector<Sub> sub;
    struct Sliced { int32_t b = -1; Slicing s{}; int64_t c_full = 0, c_last = 0; };
    std::vector<Sliced> sliced(J);          // the search changes one node at a time: keep the others' costs
    auto expand = [&]() {
        sub.clear();
        for (size_t j = 0; j < J; ++j) {
            const codec_item &it = p.items[j];
            Sliced &k = sliced[j];
            if (k.b != it.b) {
                k.b = it.b;
                k.s = slice_node(it.len, it.b, align);
                k.c_full = k.s.count > 1 ? table->estimate(it.rows, k.s.length) : 0;
                k.c_last = table->estimate(it.rows, k.s.last);
            }
            const Slicing &s = k.s;
            const int64_t c_full = k.c_full, c_last = k.c_last;
            for (int32_t c = 0; c < s.count; ++c) {
                const bool last = c == s.count - 1;
                sub.push_back({last ? c_last : c_full, int32_t(j), c, c * s.length, last ? s.last : s.length});
            }
        }
    };
    if (opt.fixed_slices > 0) {
        // the naive strategy of the granularity study: the same slice count for every node
        for (size_t j = 0; j < J; ++j)
            p.items[j].b = slice_node(p.items[j].len, std::min<int64_t>(opt.fixed_slices, max_b[j]), align).count;
    } else {
        std::vector<int32_t> order;
        for (size_t j = 0; j < J; ++j)
            if (p.items[j].ub > 1) order.push_back(int32_t(j));
        std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            if (p.items[a].cost != p.items[b].cost) return p.items[a].cost > p.items[b].cost;
            return a < b;
        });
        Schedule trial;
        for (int32_t j : order) {
            codec_item &it = p.items[j];
            int32_t best_b = 0, prev = 0;
            int64_t best_ms = 0;
            for (int32_t want = 1; want <= it.ub; ++want) {
                const int32_t count = slice_node(it.len, want, align).count;
                if (count == prev) continue;            // counts are non-decreasing in `want`
                prev = count;
                it.b = count;
                expand();
                schedule_lpt(sub, m, false, trial);
                if (best_b == 0 || trial.makespan < best_ms) {
                    best_b = count;
                    best_ms = trial.makespan;
                }
            }
            it.b = best_b;
        }
        // Extension (CODEC_PLAN_EXT_DIAGONAL, not in the paper).  The pass above moves one node at a
        // time and stops where no single move helps; equal nodes started at their bound can stay one
        // slice short of an even packing.  So the search also looks along the diagonal of the grid:
        // every node at its Eq. 5 quotient for one common target cost_l * (1 + k/8), k = 0 .. 8 (capped
        // by its bound), and keeps the best point seen.
        expand();
        schedule_lpt(sub, m, false, trial);
        int64_t best_ms = trial.makespan;
        std::vector<int32_t> best_b(J);
        for (size_t j = 0; j < J; ++j) best_b[j] = p.items[j].b;
        for (int k = 0; ext_diagonal && k <= 8; ++k) {
            const int64_t target = std::max<int64_t>(1, p.cost_l + p.cost_l * k / 8);
            for (size_t j = 0; j < J; ++j) {
                const int64_t want = std::min<int64_t>(p.items[j].ub, slices_at(j, target));
                p.items[j].b = slice_node(p.items[j].len, want, align).count;
            }
            expand();
            schedule_lpt(sub, m, false, trial);
            if (trial.makespan < best_ms) {
                best_ms = trial.makespan;
                for (size_t j = 0; j < J; ++j) best_b[j] = p.items[j].b;
            }
        }
        for (size_t j = 0; j < J; ++j) p.items[j].b = best_b[j];
    }

    // ---- a4: final schedule and emission --------------------------------------------------------
    expand();
    Schedule fin;
    schedule_lpt(sub, m, true, fin);
    p.makespan = fin.makespan;

    std::vector<int32_t> first_task(J, 0);
    p.tasks.resize(sub.size());
    int64_t base = 0;
    for (size_t i = 0; i < sub.size(); ++i) {
        const codec_item &it = p.items[sub[i].item];
        if (sub[i].chunk == 0) first_task[sub[i].item] = int32_t(i);
        codec_task &t = p.tasks[i];
        t.item = sub[i].item;
        t.node = it.node;
        t.kv_begin = sub[i].begin;
        t.kv_len = sub[i].len;
        t.q_off = it.q_off;
        t.n_req = it.n_req;
        t.part_row_base = int32_t(base);
        t.slot = fin.slot_of[i];
        t.cost = sub[i].cost;
        base += it.rows;
        if (base > INT32_MAX) return CODEC_ERR_UNSUPPORTED;
    }
    p.part_rows = int32_t(base);

    p.slot_off.assign(m + 1, 0);
    p.slot_tasks.clear();
    for (int32_t s = 0; s < m; ++s) {
        p.slot_tasks.insert(p.slot_tasks.end(), fin.lists[s].begin(), fin.lists[s].end());
        p.slot_off[s + 1] = int32_t(p.slot_tasks.size());
    }

    // per-request partial lists: path order, slices in order (Sec. 4.1 "Indexing of partial results")
    p.req_part_off.assign(B + 1, 0);
    p.req_part.clear();
    for (int32_t r = 0; r < B; ++r) {
        for (int32_t n : paths[r]) {
            const int32_t *lo = p.node_q.data() + p.node_q_off[n];
            const int32_t *hi = p.node_q.data() + p.node_q_off[n + 1];
            const int32_t qi = int32_t(std::lower_bound(lo, hi, r) - lo);
            const int32_t qpt = qpt_of[n];
            const int32_t j = first_item[n] + qi / qpt;
            for (int32_t c = 0; c < p.items[j].b; ++c)
                p.req_part.push_back(p.tasks[first_task[j] + c].part_row_base + (qi % qpt) * group);
        }
        p.req_part_off[r + 1] = int32_t(p.req_part.size());
    }

    build_device_image(p);
    return CODEC_OK;
}

int build_best_plan(const codec_tree &tree, const codec_head_config &head,
                    const codec_plan_options &opt, PlanData &plan)
{
    if (opt.share != 2) return build_plan(tree, head, opt, plan);
    if (head.num_kv_heads < 1 || head.num_q_heads < 1 || head.num_q_heads % head.num_kv_heads != 0)
        return CODEC_ERR_INVALID_ARGUMENT;
    const int32_t group = head.num_q_heads / head.num_kv_heads;
    codec_plan_options cand[4] = {opt, opt, opt, opt};
    int n = 0;
    cand[n].share = 1;                                          // row tiles of max_rows (default 256)
    ++n;
    const int32_t widest = opt.max_rows > 0 ? opt.max_rows : 256;
    const int32_t half = widest / 2 / group * group;            // row tiles of half that (still dense tasks)
    if (half > 16 && half >= group) {
        cand[n].share = 1;
        cand[n].max_rows = half;
        ++n;
    }
    const int32_t small = group <= 16 ? 16 / group * group : 0; // row tiles of at most 16 rows
    if (small >= group && (opt.max_rows == 0 || small < opt.max_rows)) {
        cand[n].share = 1;
        cand[n].max_rows = small;
        ++n;
    }
    cand[n].share = 0;                                          // flat
    ++n;
    bool have = false;
    for (int i = 0; i < n; ++i) {
        PlanData trial;
        const int st = build_plan(tree, head, cand[i], trial);
        if (st != CODEC_OK) return st;
        if (!have || trial.makespan < plan.makespan) {
            plan = std::move(trial);
            have = true;
        }
    }
    return CODEC_OK;
}

int refresh_plan(PlanData &p, const int32_t *node_len, const int32_t *node_page_off, const int32_t *page_ids)
{
    const int32_t N = p.num_nodes;
    if (N == 0) return CODEC_OK;
    if (!node_len || !node_page_off) return CODEC_ERR_INVALID_ARGUMENT;
    const int32_t ps = p.head.page_size;
    // ---- checks first: nothing is changed on error ----------------------------------------------
    if (node_page_off[0] < 0) return CODEC_ERR_INVALID_TREE;
    for (int32_t i = 0; i < N; ++i) {
        if (node_len[i] < 1) return CODEC_ERR_INVALID_TREE;
        const int64_t have = int64_t(node_page_off[i + 1]) - node_page_off[i];
        if (have < ceil_div(node_len[i], ps)) return CODEC_ERR_INVALID_TREE;
    }
    if (node_page_off[N] > 0 && !page_ids) return CODEC_ERR_INVALID_ARGUMENT;
    for (int32_t i = node_page_off[0]; i < node_page_off[N]; ++i)
        if (page_ids[i] < 0) return CODEC_ERR_INVALID_TREE;
    for (int32_t r = 0; r < p.num_requests && !p.req_mask_off.empty(); ++r)
        if (p.req_mask_off[r + 1] > p.req_mask_off[r] && node_len[p.req_node[r]] != p.node_len[p.req_node[r]])
            return CODEC_ERR_INVALID_ARGUMENT;          // a mask covers the tokens the node had at plan time
    std::vector<int32_t> first_task(p.items.size(), -1);
    for (size_t i = 0; i < p.tasks.size(); ++i)
        if (first_task[p.tasks[i].item] < 0) first_task[p.tasks[i].item] = int32_t(i);
    for (size_t j = 0; j < p.items.size(); ++j) {
        const codec_item &it = p.items[j];
        const codec_task &last = p.tasks[first_task[j] + it.b - 1];
        if (int64_t(node_len[it.node]) - last.kv_begin < 1) return CODEC_ERR_INVALID_ARGUMENT;
    }
    // ---- carry over ---------------------------------------------------------------------------------
    p.node_len.assign(node_len, node_len + N);
    p.node_page_off.assign(node_page_off, node_page_off + N + 1);
    p.page_ids.assign(page_ids, page_ids + node_page_off[N]);
    for (size_t j = 0; j < p.items.size(); ++j) {
        codec_item &it = p.items[j];
        it.len = p.node_len[it.node];
        it.cost = p.table.estimate(it.rows, it.len);
        codec_task &last = p.tasks[first_task[j] + it.b - 1];
        last.kv_len = it.len - last.kv_begin;
        last.cost = p.table.estimate(it.rows, last.kv_len);
    }
    int64_t makespan = 0;
    for (int32_t s = 0; s < p.num_slots; ++s) {
        int64_t load = 0;
        for (int32_t i = p.slot_off[s]; i < p.slot_off[s + 1]; ++i) load += p.tasks[p.slot_tasks[i]].cost;
        makespan = std::max(makespan, load);
    }
    p.makespan = makespan;
    build_device_image(p);
    return CODEC_OK;
}

}  // namespace codec
