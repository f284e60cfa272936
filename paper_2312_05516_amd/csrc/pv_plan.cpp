// Host-side auxiliary data of a batch: validation, prefix sums and the work lists.
//
// The paper computes the per-batch auxiliary arrays (cumulative sequence lengths, each request's
// region of the concatenated tokens) once on the CPU and reuses them in every layer (Section 6.4;
// Section 4.4.1).  This file is that step, extended with the decomposition of the batch into work
// items for the two attention kernels.  It is pure host code and touches no HIP API.
#include "pv_plan.h"

#include <algorithm>
#include <cmath>
#include <numeric>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_set>

namespace pv {

bool pool_desc_valid(const pv_pool_desc *p, pv_status *why)
{
    pv_status s = PV_OK;
    if (!p || p->num_pages <= 0 || p->num_kv_heads <= 0 || p->page_size <= 0 || p->head_dim <= 0)
        s = PV_ERR_INVALID_ARG;
    else if (p->page_size != 16 || (p->head_dim != 64 && p->head_dim != 128) ||
             (p->dtype != PV_F16 && p->dtype != PV_BF16))
        s = PV_ERR_UNSUPPORTED;
    if (why) *why = s;
    return s == PV_OK;
}

static int32_t env_int(const char *name, int32_t fallback)
{
    const char *v = std::getenv(name);
    if (!v || !*v) return fallback;
    char *end = nullptr;
    long x = std::strtol(v, &end, 10);
    if (end == v || x <= 0 || x > (1 << 24)) return fallback;
    return (int32_t)x;
}

Tuning default_tuning()
{
    Tuning t;
    t.split_target = env_int("PV_SPLIT_TARGET", 1024);
    t.min_split_keys = env_int("PV_MIN_SPLIT_KEYS", 256);
    t.wide_min_rows = env_int("PV_WIDE_MIN_ROWS", 33);
    t.xcds = env_int("PV_XCDS", 8);
    t.unify = env_int("PV_UNIFY", 1) == 1 ? 1 : 0;  // any other positive value switches it off
    t.unify_max_steps = env_int("PV_UNIFY_MAX_STEPS", 90000);
    {
        const char *v = std::getenv("PV_TILE_MIN_KEYS");
        t.tile_min_keys = (v && *v == '0' && !v[1]) ? 0 : env_int("PV_TILE_MIN_KEYS", 8192);
        t.tile_batch_min_keys = (v && *v) ? 0 : 1536;
    }
    return t;
}

// Whether the full 256-row tiles of a (request, KV head) unit go to the 256-row kernel: that
// kernel exists for head size 128 and pays off when an item streams many 32-key blocks.
static bool use_tile256(const pv_pool_desc *pool, const Tuning &tune, int64_t rows_total,
                        int64_t kv_len)
{
    return tune.tile_min_keys > 0 && pool->head_dim == 128 && rows_total >= kTileRows &&
           kv_len >= tune.tile_min_keys;
}

static int64_t item_cost(const WorkItem &w, int rows_per_step)
{
    const int64_t steps = (w.row_count + rows_per_step - 1) / rows_per_step;
    return (int64_t)(w.kv_end - w.kv_begin) * steps;
}

// Cut long items into parts of the KV range.  With `chunk` = the KV length that would give about
// split_target equal items (never below min_split_keys):
//  * a list too short to fill the GPU (fewer than split_target items) is cut everywhere, every
//    item longer than `chunk` into parts of about that length;
//  * in a longer list only the outliers are cut, items more than twice as long as `chunk`, because
//    one workgroup walking such an item alone would outlast everything else.
//  * whatever the list, no part is longer than max_len keys (0 = no such limit).
static void split_items(std::vector<WorkItem> &items, std::vector<CombineItem> &combine,
                        int64_t &slots, const Tuning &tune, int64_t max_len = 0)
{
    if (items.empty()) return;
    int64_t total_keys = 0;
    for (const WorkItem &w : items) total_keys += w.kv_end - w.kv_begin;
    int64_t chunk = (total_keys + tune.split_target - 1) / tune.split_target;
    chunk = std::max<int64_t>(chunk, tune.min_split_keys);
    chunk = (chunk + kKvBlock - 1) / kKvBlock * kKvBlock;
    const bool outliers_only = (int64_t)items.size() >= tune.split_target;
    auto too_long = [&](int64_t len) { return max_len > 0 && len > max_len; };
    auto wants_split = [&](const WorkItem &w) {
        const int64_t len = w.kv_end - w.kv_begin;
        return too_long(len) || (len > chunk && len >= 2 * (int64_t)tune.min_split_keys &&
                                 !(outliers_only && len <= 2 * chunk));
    };
    bool any = false;
    for (const WorkItem &w : items) any = any || wants_split(w);
    if (!any) return;  // the common case of a long list: nothing is copied
    std::vector<WorkItem> result;
    result.reserve(items.size() * 2);
    for (const WorkItem &w : items) {
        const int64_t len = w.kv_end - w.kv_begin;
        int64_t parts = (len + chunk - 1) / chunk;
        if (parts <= 1 || len < 2 * (int64_t)tune.min_split_keys ||
            (outliers_only && len <= 2 * chunk))
            parts = 1;
        if (too_long(len)) parts = std::max(parts, (len + max_len - 1) / max_len);
        if (parts <= 1) {
            result.push_back(w);
            continue;
        }
        int64_t part_len = (len + parts - 1) / parts;
        part_len = (part_len + kKvBlock - 1) / kKvBlock * kKvBlock;
        parts = (len + part_len - 1) / part_len;
        if (parts <= 1) {
            result.push_back(w);
            continue;
        }
        CombineItem c;
        c.req = w.req;
        c.kv_head = w.kv_head;
        c.row_begin = w.row_begin;
        c.row_count = w.row_count;
        c.partial_base = (int32_t)slots;
        c.split_count = (int32_t)parts;
        c.q_row0 = w.q_row0;
        c.reserved = 0;
        combine.push_back(c);
        for (int64_t s = 0; s < parts; ++s) {
            WorkItem part = w;
            part.kv_begin = (int32_t)(w.kv_begin + s * part_len);
            part.kv_end = (int32_t)std::min<int64_t>(w.kv_end, w.kv_begin + (s + 1) * part_len);
            part.split_index = (int32_t)s;
            part.split_count = (int32_t)parts;
            part.partial_base = (int32_t)(slots + s * w.row_count);
            result.push_back(part);
        }
        slots += parts * w.row_count;
    }
    items.swap(result);
}

// Order of the work list = order of workgroup dispatch.  Two goals:
//  * longest first, so that in-order dispatch approximates longest-processing-time scheduling;
//  * items that stream the same K/V (the row tiles of one (request, KV head, KV part)) should run
//    at the same time on the same XCD, so that the second and later tiles hit in that XCD's L2.
//    Workgroup i of a launch goes to XCD i % xcds, so a group's items are placed `xcds` positions
//    apart.  Groups are dealt to the XCDs greedily by accumulated cost (longest group first).
static void order_items(std::vector<WorkItem> &items, int rows_per_step, int xcds)
{
    if (items.empty()) return;
    if (xcds < 1) xcds = 1;
    const size_t n = items.size();
    // 1. group by (req, kv_head, split_index); items of a group keep their row order.  Sorted as
    //    (key, position) pairs: the 48-byte items themselves are moved only once, at the end.
    struct Keyed {
        int32_t req, kv_head, split_index;
        uint32_t pos;
        bool same_group(const Keyed &o) const
        {
            return req == o.req && kv_head == o.kv_head && split_index == o.split_index;
        }
    };
    std::vector<Keyed> keyed(n);
    for (size_t i = 0; i < n; ++i)
        keyed[i] = Keyed{items[i].req, items[i].kv_head, items[i].split_index, (uint32_t)i};
    auto before = [](const Keyed &a, const Keyed &b) {
        if (a.req != b.req) return a.req < b.req;
        if (a.kv_head != b.kv_head) return a.kv_head < b.kv_head;
        if (a.split_index != b.split_index) return a.split_index < b.split_index;
        return a.pos < b.pos;
    };
    if (!std::is_sorted(keyed.begin(), keyed.end(), before))
        std::sort(keyed.begin(), keyed.end(), before);
    struct Group { uint32_t begin, end; int64_t cost; };
    std::vector<Group> groups;
    groups.reserve(n);
    for (size_t i = 0; i < n;) {
        size_t j = i;
        int64_t cost = 0;
        while (j < n && keyed[j].same_group(keyed[i])) {
            cost += item_cost(items[keyed[j].pos], rows_per_step);
            ++j;
        }
        groups.push_back(Group{(uint32_t)i, (uint32_t)j, cost});
        i = j;
    }
    // 2. longest group first (per item, so that a long single item is not hidden behind a group of
    //    many short ones), dealt to the least loaded XCD
    std::stable_sort(groups.begin(), groups.end(), [&](const Group &a, const Group &b) {
        return a.cost * (int64_t)(b.end - b.begin) > b.cost * (int64_t)(a.end - a.begin);
    });
    std::vector<std::vector<uint32_t>> queue((size_t)xcds);
    for (auto &qv : queue) qv.reserve(n / (size_t)xcds + 16);
    std::vector<int64_t> load((size_t)xcds, 0);
    for (const Group &g : groups) {
        size_t best = 0;
        for (size_t x = 1; x < (size_t)xcds; ++x)
            if (load[x] < load[best]) best = x;
        for (uint32_t i = g.begin; i < g.end; ++i) queue[best].push_back(keyed[i].pos);
        load[best] += g.cost;
    }
    // 3. interleave: position k*xcds + x takes the k-th item of XCD x's queue; once a queue is
    //    empty its positions are filled from the queues that still have items
    std::vector<WorkItem> out;
    out.reserve(n);
    std::vector<size_t> at((size_t)xcds, 0);
    size_t x = 0;
    while (out.size() < n) {
        size_t pick = x;
        for (int tries = 0; tries < xcds && at[pick] >= queue[pick].size(); ++tries)
            pick = (pick + 1) % (size_t)xcds;
        out.push_back(items[queue[pick][at[pick]++]]);
        x = (x + 1) % (size_t)xcds;
    }
    items.swap(out);
}

// One contiguous host image of the arrays the kernels read, each part 256-byte aligned.
static void build_image(pv_plan *plan)
{
    struct Part { const void *src; size_t bytes; };
    const Part parts[9] = {
        {plan->ctx_lens.data(), plan->ctx_lens.size() * sizeof(int32_t)},
        {plan->q_lens.data(), plan->q_lens.size() * sizeof(int32_t)},
        {plan->q_start.data(), plan->q_start.size() * sizeof(int32_t)},
        {plan->combine_chunks.data(), plan->combine_chunks.size() * sizeof(CombineChunk)},
        {plan->narrow.data(), plan->narrow.size() * sizeof(WorkItem)},
        {plan->wide.data(), plan->wide.size() * sizeof(WorkItem)},
        {plan->tile256.data(), plan->tile256.size() * sizeof(WorkItem)},
        {plan->combine.data(), plan->combine.size() * sizeof(CombineItem)},
        {plan->append_groups.data(), plan->append_groups.size() * sizeof(AppendGroup)},
    };
    size_t total = 0;
    for (int i = 0; i < 9; ++i) {
        plan->image_off[i] = total;
        total += (parts[i].bytes + 255) / 256 * 256;
    }
    if (total == 0) total = 256;
    plan->image.assign(total, 0);
    for (int i = 0; i < 9; ++i)
        if (parts[i].bytes)
            std::memcpy(plan->image.data() + plan->image_off[i], parts[i].src, parts[i].bytes);
}

pv_status build_plan(const pv_pool_desc *pool, int32_t num_q_heads, const int32_t *ctx_lens,
                     const int32_t *q_lens, int32_t num_reqs, int32_t max_pages_per_req,
                     const Tuning &tune, pv_plan **out)
{
    if (!out) return PV_ERR_INVALID_ARG;
    *out = nullptr;
    pv_status why;
    if (!pool_desc_valid(pool, &why)) return why;
    if (num_q_heads <= 0 || num_q_heads % pool->num_kv_heads != 0) return PV_ERR_INVALID_ARG;
    if (num_reqs < 0 || max_pages_per_req < 0) return PV_ERR_INVALID_ARG;
    if (num_reqs > 0 && (!ctx_lens || !q_lens)) return PV_ERR_INVALID_ARG;
    const int32_t P = pool->page_size;
    const int32_t G = num_q_heads / pool->num_kv_heads;

    int64_t total_q = 0;
    for (int32_t r = 0; r < num_reqs; ++r) {
        if (ctx_lens[r] < 0 || q_lens[r] < 0) return PV_ERR_INVALID_ARG;
        const int64_t len = (int64_t)ctx_lens[r] + q_lens[r];
        if (len > INT32_MAX - 64) return PV_ERR_OUT_OF_RANGE;
        if (q_lens[r] > 0 && (len + P - 1) / P > max_pages_per_req) return PV_ERR_OUT_OF_RANGE;
        if ((int64_t)q_lens[r] * G > INT32_MAX / 2) return PV_ERR_OUT_OF_RANGE;
        total_q += q_lens[r];
    }
    // rows of q/out are indexed with 64-bit arithmetic in the kernels; the row count itself and
    // the workspace slot numbers stay 32-bit
    if (total_q > INT32_MAX / 2) return PV_ERR_OUT_OF_RANGE;

    pv_plan *plan = new (std::nothrow) pv_plan();
    if (!plan) return PV_ERR_INVALID_ARG;
    plan->pool = *pool;
    plan->num_q_heads = num_q_heads;
    plan->group = G;
    plan->num_reqs = num_reqs;
    plan->max_pages_per_req = max_pages_per_req;
    plan->total_q = (int32_t)total_q;
    plan->ctx_lens.assign(ctx_lens, ctx_lens + num_reqs);
    plan->q_lens.assign(q_lens, q_lens + num_reqs);
    plan->q_start.resize(num_reqs);
    plan->partial_slots = 0;
    plan->uploaded = false;
    plan->device = -1;
    plan->d_owned = nullptr;
    std::memset(&plan->dev, 0, sizeof plan->dev);
    plan->timing = false;
    for (void *&e : plan->events) e = nullptr;
    for (bool &u : plan->event_used) u = false;
    int32_t at = 0;
    for (int32_t r = 0; r < num_reqs; ++r) {
        plan->q_start[r] = at;
        at += q_lens[r];
    }

    // append: runs of new tokens that share an 8-slot group of a page
    for (int32_t r = 0; r < num_reqs; ++r) {
        const int64_t c = ctx_lens[r], end = (int64_t)ctx_lens[r] + q_lens[r];
        for (int64_t t = c; t < end;) {
            const int64_t group_end = (t / 8 + 1) * 8;
            const int64_t stop = std::min(end, group_end);
            AppendGroup g;
            g.req = r;
            g.t_begin = (int32_t)t;
            g.count = (int32_t)(stop - t);
            g.q_row = plan->q_start[r] + (int32_t)(t - c);
            plan->append_groups.push_back(g);
            t = stop;
        }
    }

    // One attention launch instead of two for a mixed batch.  Every launch has a fixed cost, the
    // two kernels cannot share a CU, and a short bandwidth-oriented launch never gets the GPU up to
    // speed, while its units fit well into the slots the long matrix-core items leave.  But an item
    // of the matrix-core kernel holds a workgroup slot for one step per 32 keys whatever its row
    // count, so when the small units (generation steps) are a large amount of work, the
    // bandwidth-oriented kernel is the better place for them.  Measured crossover on mixes of
    // 256-token prompts and generation steps over 2000-token contexts, MHA 40/40 and GQA 64/8 alike:
    // 80-100 K steps of 32 keys summed over the small units and KV heads (~1.5 GB of K/V).
    // The 256-row kernel runs one workgroup per CU and needs a launch of its own, so in a mixed
    // batch it only pays for long KV ranges (tile_min_keys).  A batch that is nearly all long
    // multi-token units of head size 128 is another matter: measured on batches of 256- to 512-token
    // requests it is ahead of the 128-row kernel from about 1.5 K keys up (+5 % there, +7-8 % with
    // mixed lengths of 1-3.5 K or a few generation steps in the batch, +11 % at 4.5 K).  The
    // lower limit applies when at least 90 % of the batch's (row, key) pairs are in full 256-row
    // tiles of units that qualify under it, and those tiles are many enough and even enough that
    // the plan will not cut them (a cut item writes fp32 partial results that a merge pass reads).
    Tuning tune_batch = tune;
    if (tune.tile_batch_min_keys > 0 && tune.tile_min_keys > tune.tile_batch_min_keys &&
        pool->head_dim == 128) {
        int64_t pairs_all = 0, pairs_tile = 0, items = 0, keys = 0, longest = 0;
        for (int32_t r = 0; r < num_reqs; ++r) {
            const int64_t n = q_lens[r], c = ctx_lens[r];
            if (n == 0) continue;
            const int64_t rows_total = n * G, kv = c + n;
            pairs_all += rows_total * kv;
            if (rows_total >= kTileRows && kv >= tune.tile_batch_min_keys) {
                const int64_t tiles = rows_total / kTileRows;
                pairs_tile += tiles * kTileRows * kv;
                items += tiles * pool->num_kv_heads;
                keys += tiles * pool->num_kv_heads * kv;
                longest = std::max(longest, kv);
            }
        }
        int64_t chunk = (keys + tune.split_target - 1) / std::max(tune.split_target, 1);
        chunk = std::max<int64_t>(chunk, tune.min_split_keys);
        if (items >= tune.split_target && pairs_tile * 10 >= pairs_all * 9 && longest <= 2 * chunk)
            tune_batch.tile_min_keys = tune.tile_batch_min_keys;
    }
    bool all_wide = false;
    if (tune.unify) {
        int64_t wide_steps = 0, small_steps = 0;
        for (int32_t r = 0; r < num_reqs; ++r) {
            const int64_t n = q_lens[r], c = ctx_lens[r];
            if (n == 0) continue;
            const int64_t rows_total = n * G;
            if (rows_total >= tune.wide_min_rows) {
                for (int64_t rb = 0; rb < rows_total; rb += kWideRows) {
                    const int64_t last = (std::min<int64_t>(rows_total, rb + kWideRows) - 1) / G;
                    wide_steps += (c + last + 1 + kKvBlock - 1) / kKvBlock;
                }
            } else {
                small_steps += (c + n + kKvBlock - 1) / kKvBlock;
            }
        }
        all_wide = wide_steps > 0 &&
                   small_steps * (int64_t)pool->num_kv_heads <= (int64_t)tune.unify_max_steps;
    }
    {
        // capacity for the item lists, so that filling them does not reallocate
        size_t n_narrow = 0, n_wide = 0;
        for (int32_t r = 0; r < num_reqs; ++r) {
            const int64_t rows_total = (int64_t)q_lens[r] * G;
            if (rows_total == 0) continue;
            const bool big = rows_total >= tune.wide_min_rows;
            const size_t tiles = (size_t)((rows_total + (big ? kWideRows : kNarrowRows) - 1) /
                                          (big ? kWideRows : kNarrowRows));
            (big || all_wide ? n_wide : n_narrow) += tiles * (size_t)pool->num_kv_heads;
        }
        plan->narrow.reserve(n_narrow);
        plan->wide.reserve(n_wide);
    }
    for (int32_t r = 0; r < num_reqs; ++r) {
        const int32_t n = q_lens[r], c = ctx_lens[r];
        if (n == 0) continue;
        const int32_t rows_total = n * G;
        for (int32_t hk = 0; hk < pool->num_kv_heads; ++hk) {
            WorkItem w;
            std::memset(&w, 0, sizeof w);
            w.req = r;
            w.kv_head = hk;
            w.kv_begin = 0;
            w.split_index = 0;
            w.split_count = 1;
            w.partial_base = -1;
            w.q_row0 = plan->q_start[r];
            w.ctx = c;
            const bool use_wide = rows_total >= tune.wide_min_rows || all_wide;
            const int32_t tile = use_wide ? kWideRows : kNarrowRows;
            // long units: their full 256-row tiles go to the 256-row kernel, the rest as usual
            int32_t rb = 0;
            if (use_tile256(pool, tune_batch, rows_total, (int64_t)c + n)) {
                for (; rb + kTileRows <= rows_total; rb += kTileRows) {
                    w.row_begin = rb;
                    w.row_count = kTileRows;
                    w.kv_end = c + (rb + kTileRows - 1) / G + 1;
                    plan->tile256.push_back(w);
                }
            }
            for (; rb < rows_total; rb += tile) {
                w.row_begin = rb;
                w.row_count = std::min(tile, rows_total - rb);
                const int32_t last_token = (rb + w.row_count - 1) / G;
                w.kv_end = c + last_token + 1;  // causal limit of the tile's last row
                (use_wide ? plan->wide : plan->narrow).push_back(w);
            }
        }
    }
    int64_t slots = 0;
    split_items(plan->narrow, plan->combine, slots, tune);
    split_items(plan->wide, plan->combine, slots, tune);
    split_items(plan->tile256, plan->combine, slots, tune,
                (int64_t)kTileMaxPages * pool->page_size - kKvBlock);
    if (slots > INT32_MAX / 2) {
        delete plan;
        return PV_ERR_OUT_OF_RANGE;
    }
    order_items(plan->narrow, kNarrowRows, tune.xcds);
    order_items(plan->wide, kWideRows, tune.xcds);
    order_items(plan->tile256, kTileRows, tune.xcds);
    plan->partial_slots = slots;
    for (size_t i = 0; i < plan->combine.size(); ++i)
        for (int32_t r0 = 0; r0 < plan->combine[i].row_count; r0 += 8)
            plan->combine_chunks.push_back(CombineChunk{(int32_t)i, r0});
    // workspace: fp32 partial outputs [slots][D], then (running max, running sum) [slots][2]
    plan->workspace_bytes = (size_t)slots * (size_t)(pool->head_dim + 2) * sizeof(float);
    build_image(plan);
    *out = plan;
    return PV_OK;
}

DeviceLists lists_at(const pv_plan *plan, const void *base)
{
    const unsigned char *b = static_cast<const unsigned char *>(base);
    DeviceLists d;
    d.ctx_lens = reinterpret_cast<const int32_t *>(b + plan->image_off[0]);
    d.q_lens = reinterpret_cast<const int32_t *>(b + plan->image_off[1]);
    d.q_start = reinterpret_cast<const int32_t *>(b + plan->image_off[2]);
    d.combine_chunks = reinterpret_cast<const CombineChunk *>(b + plan->image_off[3]);
    d.narrow = reinterpret_cast<const WorkItem *>(b + plan->image_off[4]);
    d.wide = reinterpret_cast<const WorkItem *>(b + plan->image_off[5]);
    d.tile256 = reinterpret_cast<const WorkItem *>(b + plan->image_off[6]);
    d.combine = reinterpret_cast<const CombineItem *>(b + plan->image_off[7]);
    d.append_groups = reinterpret_cast<const AppendGroup *>(b + plan->image_off[8]);
    return d;
}

}  // namespace pv

// ---------------------------------------------------------------------------------------------
// C ABI: the host-only entry points
// ---------------------------------------------------------------------------------------------
extern "C" {

const char *pv_status_string(pv_status s)
{
    switch (s) {
    case PV_OK: return "ok";
    case PV_ERR_INVALID_ARG: return "invalid argument";
    case PV_ERR_UNSUPPORTED: return "unsupported configuration";
    case PV_ERR_OUT_OF_RANGE: return "length or index out of range";
    case PV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case PV_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

size_t pv_pool_bytes(const pv_pool_desc *pool)
{
    if (!pv::pool_desc_valid(pool, nullptr)) return 0;
    return (size_t)pool->num_pages * pool->num_kv_heads * pool->page_size * pool->head_dim * 2u;
}

int64_t pv_pool_k_offset(const pv_pool_desc *pool, int32_t page, int32_t head, int32_t slot,
                         int32_t d)
{
    if (!pv::pool_desc_valid(pool, nullptr)) return -1;
    if (page < 0 || page >= pool->num_pages || head < 0 || head >= pool->num_kv_heads ||
        slot < 0 || slot >= pool->page_size || d < 0 || d >= pool->head_dim)
        return -1;
    const int64_t tile = (int64_t)page * pool->num_kv_heads + head;
    const int64_t chunks = pool->head_dim / 8;
    return ((tile * chunks + d / 8) * pool->page_size + slot) * 8 + d % 8;
}

int64_t pv_pool_v_offset(const pv_pool_desc *pool, int32_t page, int32_t head, int32_t slot,
                         int32_t d)
{
    if (!pv::pool_desc_valid(pool, nullptr)) return -1;
    if (page < 0 || page >= pool->num_pages || head < 0 || head >= pool->num_kv_heads ||
        slot < 0 || slot >= pool->page_size || d < 0 || d >= pool->head_dim)
        return -1;
    const int64_t tile = (int64_t)page * pool->num_kv_heads + head;
    const int64_t groups = pool->page_size / 8;
    return ((tile * groups + slot / 8) * pool->head_dim + d) * 8 + slot % 8;
}

pv_status pv_plan_create(const pv_pool_desc *pool, int32_t num_q_heads, const int32_t *ctx_lens,
                         const int32_t *q_lens, int32_t num_reqs, int32_t max_pages_per_req,
                         pv_plan **plan)
{
    return pv::build_plan(pool, num_q_heads, ctx_lens, q_lens, num_reqs, max_pages_per_req,
                          pv::default_tuning(), plan);
}

int32_t pv_plan_total_q(const pv_plan *plan) { return plan ? plan->total_q : -1; }

const int32_t *pv_plan_q_start(const pv_plan *plan)
{
    return plan ? plan->q_start.data() : nullptr;
}

size_t pv_plan_workspace_bytes(const pv_plan *plan) { return plan ? plan->workspace_bytes : 0; }

size_t pv_plan_device_bytes(const pv_plan *plan) { return plan ? plan->image.size() : 0; }

int32_t pv_plan_owns_device_memory(const pv_plan *plan)
{
    return plan ? (plan->d_owned != nullptr ? 1 : 0) : -1;
}

int32_t pv_plan_num_work_items(const pv_plan *plan, int32_t kind)
{
    if (!plan) return -1;
    switch (kind) {
    case 0: return (int32_t)plan->narrow.size();
    case 1: return (int32_t)plan->wide.size();
    case 2: return (int32_t)plan->combine.size();
    case 3: return (int32_t)plan->tile256.size();
    }
    return -1;
}

pv_status pv_plan_work_item(const pv_plan *plan, int32_t kind, int32_t index, int32_t out[8])
{
    if (!plan || !out || index < 0) return PV_ERR_INVALID_ARG;
    if (kind == 0 || kind == 1 || kind == 3) {
        const std::vector<pv::WorkItem> &v =
            kind == 0 ? plan->narrow : kind == 1 ? plan->wide : plan->tile256;
        if ((size_t)index >= v.size()) return PV_ERR_INVALID_ARG;
        const pv::WorkItem &w = v[index];
        const int32_t f[8] = {w.req, w.kv_head, w.row_begin, w.row_count,
                              w.kv_begin, w.kv_end, w.split_index, w.split_count};
        std::memcpy(out, f, sizeof f);
        return PV_OK;
    }
    if (kind == 2) {
        if ((size_t)index >= plan->combine.size()) return PV_ERR_INVALID_ARG;
        const pv::CombineItem &c = plan->combine[index];
        const int32_t f[8] = {c.req, c.kv_head, c.row_begin, c.row_count, 0, 0, 0, c.split_count};
        std::memcpy(out, f, sizeof f);
        return PV_OK;
    }
    return PV_ERR_INVALID_ARG;
}

pv_status pv_plan_check_page_table(const pv_plan *plan, const int32_t *page_table,
                                   int32_t check_append_unique)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (plan->num_reqs > 0 && !page_table) return PV_ERR_INVALID_ARG;
    const int32_t P = plan->pool.page_size;
    std::unordered_set<int64_t> seen;
    for (int32_t r = 0; r < plan->num_reqs; ++r) {
        const int32_t n = plan->q_lens[r], c = plan->ctx_lens[r];
        if (n == 0) continue;
        const int64_t pages = ((int64_t)c + n + P - 1) / P;
        const int32_t *row = page_table + (int64_t)r * plan->max_pages_per_req;
        for (int64_t lp = 0; lp < pages; ++lp)
            if (row[lp] < 0 || row[lp] >= plan->pool.num_pages) return PV_ERR_OUT_OF_RANGE;
        if (check_append_unique) {
            for (int32_t j = 0; j < n; ++j) {
                const int64_t t = (int64_t)c + j;
                const int64_t key = (int64_t)row[t / P] * P + t % P;
                if (!seen.insert(key).second) return PV_ERR_INVALID_ARG;
            }
        }
    }
    return PV_OK;
}

pv_status pv_rope_table(double base, int32_t head_dim, int32_t max_pos, float *table)
{
    if (!(base > 0.0) || head_dim <= 0 || head_dim % 2 != 0 || max_pos < 0 || !table)
        return PV_ERR_INVALID_ARG;
    const int32_t half = head_dim / 2;
    std::vector<double> theta((size_t)half);
    for (int32_t i = 0; i < half; ++i) theta[(size_t)i] = std::pow(base, -2.0 * i / head_dim);
    for (int64_t t = 0; t < max_pos; ++t) {
        float *row = table + t * head_dim;
        for (int32_t i = 0; i < half; ++i) {
            const double angle = (double)t * theta[(size_t)i];
            row[i] = (float)std::cos(angle);
            row[half + i] = (float)std::sin(angle);
        }
    }
    return PV_OK;
}

double pv_cost_model(const int32_t *ctx_points, const double *attn_cost, int32_t n, double c_other,
                     int32_t l)
{
    if (n <= 0) return c_other;
    if (!ctx_points || !attn_cost) return std::nan("");
    if (n == 1) return attn_cost[0] + c_other;
    // segment whose right end is the first profiled point >= l (clamped to the outer segments)
    const int32_t *hi = std::lower_bound(ctx_points + 1, ctx_points + n - 1, l);
    const int32_t k = (int32_t)(hi - ctx_points) - 1;
    const double t = ((double)l - ctx_points[k]) / ((double)ctx_points[k + 1] - ctx_points[k]);
    return attn_cost[k] + t * (attn_cost[k + 1] - attn_cost[k]) + c_other;
}

pv_status pv_retention_order(const double *cost, const double *idle_time, int32_t n,
                             int32_t *order_out)
{
    if (n < 0 || (n > 0 && (!cost || !idle_time || !order_out))) return PV_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (!(idle_time[i] > 0.0)) return PV_ERR_INVALID_ARG;
    std::iota(order_out, order_out + n, 0);
    std::stable_sort(order_out, order_out + n, [&](int32_t a, int32_t b) {
        return cost[a] / idle_time[a] < cost[b] / idle_time[b];
    });
    return PV_OK;
}

}  // extern "C"
