// KV append: store the new K/V rows of a batch into the slots the page table assigns to them
// (paper Section 4.4.1: the newly generated KV-tokens are stored in their allocated slots before
// the attention runs).  Pure 16-bit moves, so the pool image is bit-exact.
//
// One workgroup of D threads handles one append group (up to 8 consecutive new tokens of a request
// inside one 8-slot group of a page, listed by the host plan) for one KV head.
//   K pool: 8 consecutive head dimensions of a token are one 16-byte run; thread t copies run
//           (token t / (D/8), chunk t % (D/8)).
//   V pool: 8 consecutive slots of one head dimension are one 16-byte run; thread d gathers its
//           dimension from the group's tokens and, when the group is full, writes the run with one
//           16-byte store (otherwise element by element, leaving the other slots untouched).
#include "pv_device.h"

namespace pv {

template <int D>
__global__ __launch_bounds__(D) void kv_append_kernel(
    const AppendGroup *__restrict__ groups, const uint16_t *__restrict__ k_new,
    const uint16_t *__restrict__ v_new, const int32_t *__restrict__ page_table, int32_t max_pages,
    int32_t num_kv_heads, uint16_t *__restrict__ k_pages, uint16_t *__restrict__ v_pages)
{
    constexpr int CH = D / 8;
    const AppendGroup g = groups[blockIdx.x];
    const int h = (int)blockIdx.y;
    const int t = (int)threadIdx.x;
    const int64_t page = page_table[(int64_t)g.req * max_pages + (g.t_begin >> 4)];
    const int slot0 = g.t_begin & 15;  // slot of the group's first token; the group stays in one
                                       // half (8 slots) of the page
    const int64_t tile = (page * num_kv_heads + h) * (int64_t)(16 * D);
    const int64_t row_stride = (int64_t)num_kv_heads * D;
    const uint16_t *ksrc = k_new + (int64_t)g.q_row * row_stride + (int64_t)h * D;
    const uint16_t *vsrc = v_new + (int64_t)g.q_row * row_stride + (int64_t)h * D;

    // K: thread -> (token j, chunk c8)
    {
        const int j = t / CH, c8 = t % CH;
        if (j < g.count) {
            const u32x4 kv = load16(ksrc + j * row_stride + 8 * c8);
            *reinterpret_cast<u32x4 *>(k_pages + tile + (c8 * 16 + slot0 + j) * 8) = kv;
        }
    }
    // V: thread -> head dimension d = t
    scatter_v_group<D>(vsrc, row_stride, g.count, slot0, t, v_pages + tile);
}

hipError_t launch_kv_append(const pv_plan *plan, const DeviceLists &dl, const void *k_new, const void *v_new,
                            const int32_t *page_table, void *k_pages, void *v_pages,
                            hipStream_t stream)
{
    const int D = plan->pool.head_dim;
    const size_t groups = plan->append_groups.size();
    if (groups == 0) return hipSuccess;
    const dim3 grid((unsigned)groups, (unsigned)plan->pool.num_kv_heads);
    if (D == 128)
        hipLaunchKernelGGL((kv_append_kernel<128>), grid, dim3(128), 0, stream,
                           dl.append_groups, (const uint16_t *)k_new, (const uint16_t *)v_new,
                           page_table, plan->max_pages_per_req, plan->pool.num_kv_heads,
                           (uint16_t *)k_pages, (uint16_t *)v_pages);
    else
        hipLaunchKernelGGL((kv_append_kernel<64>), grid, dim3(64), 0, stream,
                           dl.append_groups, (const uint16_t *)k_new, (const uint16_t *)v_new,
                           page_table, plan->max_pages_per_req, plan->pool.num_kv_heads,
                           (uint16_t *)k_pages, (uint16_t *)v_pages);
    return hipGetLastError();
}

}  // namespace pv
