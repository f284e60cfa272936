// Internal: host-side batch plan shared by the API file and the kernel launchers.
#pragma once

#include <cstdint>
#include <vector>

#include "pv.h"

namespace pv {

// One unit of kernel work.  A "row" is a (new token, query head within the GQA group) pair of one
// (request, KV head): row = token * G + g, so the rows of one KV head that can share a K/V tile
// are contiguous and ordered by token (which keeps the causal limit monotone in the row index).
struct WorkItem {
    int32_t req;
    int32_t kv_head;
    int32_t row_begin;    // first row of the item
    int32_t row_count;    // rows in the item
    int32_t kv_begin;     // first logical KV position (multiple of 32 unless 0)
    int32_t kv_end;       // one past the last logical KV position any row of the item may see
    int32_t split_index;  // which part of the KV range this is
    int32_t split_count;  // 1 = writes `out` directly, >1 = writes a partial result
    int32_t partial_base; // first workspace row slot of this item (split_count > 1), else -1
    int32_t q_row0;       // q_start[req]
    int32_t ctx;          // ctx_lens[req]
    int32_t reserved;
};
static_assert(sizeof(WorkItem) == 48, "WorkItem is read by the kernels as 12 int32");

// Merge of the partial results of one split item.
struct CombineItem {
    int32_t req;
    int32_t kv_head;
    int32_t row_begin;
    int32_t row_count;
    int32_t partial_base; // slot of split 0, row 0; split s, row i lives at base + s*row_count + i
    int32_t split_count;
    int32_t q_row0;
    int32_t reserved;
};
static_assert(sizeof(CombineItem) == 32, "CombineItem is read by the kernels as 8 int32");

// Eight rows of one combine item: the unit of work of one merge workgroup.
struct CombineChunk {
    int32_t item;  // index into the combine list
    int32_t row0;  // first row (relative to the item) of the chunk
};
static_assert(sizeof(CombineChunk) == 8, "CombineChunk is read by the kernel as 2 int32");

// Up to 8 consecutive new tokens of one request that fall into the same 8-slot group of a page
// (the V pool keeps 8 consecutive slots of one head dimension in one 16-byte run).
struct AppendGroup {
    int32_t req;
    int32_t t_begin;  // logical position of the first token of the group
    int32_t count;    // 1..8 tokens
    int32_t q_row;    // row of that first token in k_new / v_new
};
static_assert(sizeof(AppendGroup) == 16, "AppendGroup is read by the kernel as 4 int32");

constexpr int kNarrowRows = 16;  // rows per item of the bandwidth-oriented kernel
constexpr int kWideRows = 128;   // rows per item of the matrix-core kernel (4 waves x 32 rows)
constexpr int kTileRows = 256;   // rows per item of the 256-row matrix-core kernel (4 waves x 64)
constexpr int kKvBlock = 32;     // keys per inner step (two pages)
constexpr int kTileMaxPages = 8192;  // page ids an item of the 256-row kernel may span (it keeps
                                     // them in LDS): its KV range is at most 16 times that

// Where the lists of a plan live on a device: pointers into one buffer laid out as the plan's
// host image (see pv_plan::image).  The launchers take the lists through this, so that the same
// plan can run from its own upload, from a buffer of the caller's, or from the library's static
// scratch array.
struct DeviceLists {
    const int32_t *ctx_lens, *q_lens, *q_start;
    const CombineChunk *combine_chunks;
    const WorkItem *narrow, *wide, *tile256;
    const CombineItem *combine;
    const AppendGroup *append_groups;
};

struct Tuning {
    int32_t split_target;    // aim for at least this many work items per kernel
    int32_t min_split_keys;  // never make a KV part shorter than this
    int32_t wide_min_rows;   // (request, KV head) units with n*G >= this use the matrix-core
                             // kernel; smaller ones are cut into 16-row items of the narrow kernel
    int32_t xcds;            // L2 domains the work list is interleaved over
    int32_t unify;           // 1: a batch with matrix-core work sends its small units to that
                             // kernel too (one attention launch, not two) unless they are many
    int32_t unify_max_steps; // "many": more than this many 32-key steps over all small units and
                             // KV heads (then the bandwidth-oriented kernel is worth its launch)
    int32_t tile_min_keys;   // (request, KV head) units with at least 256 rows and at least this
                             // many keys send their full 256-row tiles to the 256-row kernel
                             // (0 switches that kernel off)
    int32_t tile_batch_min_keys;  // the lower limit that applies instead when nearly all of a
                             // batch's work qualifies under it and its items need no splitting
                             // (0: no such rule; it is off when tile_min_keys is set by hand)
};

}  // namespace pv

struct pv_plan {
    pv_pool_desc pool;
    int32_t num_q_heads;
    int32_t group;  // G
    int32_t num_reqs;
    int32_t max_pages_per_req;
    int32_t total_q;
    std::vector<int32_t> ctx_lens, q_lens, q_start;
    std::vector<pv::WorkItem> narrow, wide, tile256;
    std::vector<pv::CombineItem> combine;
    std::vector<pv::AppendGroup> append_groups;
    std::vector<pv::CombineChunk> combine_chunks;
    int64_t partial_slots;  // workspace row slots
    size_t workspace_bytes;

    // Host image of everything the kernels read from the plan: the nine arrays above, each at a
    // 256-byte aligned offset (image_off, in the order of pv::DeviceLists).  Built with the plan,
    // copied to a device by pv_plan_upload / pv_plan_upload_to / the no-allocation launch.
    std::vector<unsigned char> image;
    size_t image_off[9];

    // device copy (set by pv_plan_upload or pv_plan_upload_to)
    bool uploaded;
    int device;
    void *d_owned;        // device memory the plan allocated itself (pv_plan_upload), else null
    pv::DeviceLists dev;  // valid while `uploaded`

    // optional per-kernel timing: events[2*kind], events[2*kind+1] bracket kernel `kind`
    bool timing;
    void *events[10];
    bool event_used[5];
};

namespace pv {
// the lists of a plan image that was copied to `base`
DeviceLists lists_at(const pv_plan *plan, const void *base);
bool pool_desc_valid(const pv_pool_desc *p, pv_status *why);
Tuning default_tuning();
pv_status build_plan(const pv_pool_desc *pool, int32_t num_q_heads, const int32_t *ctx_lens,
                     const int32_t *q_lens, int32_t num_reqs, int32_t max_pages_per_req,
                     const Tuning &tune, pv_plan **out);
}  // namespace pv
