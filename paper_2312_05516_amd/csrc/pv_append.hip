// KV append: store the new K/V rows of a batch into the slots the page table assigns to them
// (paper Section 4.4.1: the newly generated KV-tokens are stored in their allocated slots before
// the attention runs).  Pure 16-bit moves, so the pool image is bit-exact.
//
// One thread moves 8 consecutive head dimensions of one (token, KV head): in the K pool these are
// one 16-byte run; in the V pool they are 8 elements 16 bytes apart (the V pool keeps 8
// consecutive slots of one dimension together).
#include "pv_device.h"

namespace pv {

template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new,
    const int32_t *__restrict__ page_table, int32_t max_pages, const int32_t *__restrict__ tok_req,
    const int32_t *__restrict__ slot_offsets, const int32_t *__restrict__ q_start,
    int32_t num_kv_heads, int64_t total_chunks, uint16_t *__restrict__ k_pages,
    uint16_t *__restrict__ v_pages)
{
    constexpr int CH = D / 8;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total_chunks) return;
    const int c8 = (int)(idx % CH);
    const int64_t th = idx / CH;
    const int h = (int)(th % num_kv_heads);
    const int64_t tok = th / num_kv_heads;
    const int r = tok_req[tok];
    const int t = slot_offsets[r] + (int)(tok - q_start[r]);  // logical position
    const int64_t page = page_table[(int64_t)r * max_pages + (t >> 4)];
    const int slot = t & 15;
    const int64_t tile = (page * num_kv_heads + h) * (int64_t)(16 * D);
    const u32x4 kv = load16(k_new + (tok * num_kv_heads + h) * D + 8 * c8);
    *reinterpret_cast<u32x4 *>(k_pages + tile + (c8 * 16 + slot) * 8) = kv;
    const u32x4 vv = load16(v_new + (tok * num_kv_heads + h) * D + 8 * c8);
    uint16_t *vdst = v_pages + tile + ((int64_t)((slot >> 3) * D + 8 * c8) * 8) + (slot & 7);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        vdst[(2 * j) * 8] = (uint16_t)(vv[j] & 0xFFFFu);
        vdst[(2 * j + 1) * 8] = (uint16_t)(vv[j] >> 16);
    }
}

hipError_t launch_kv_append(const pv_plan *plan, const void *k_new, const void *v_new,
                            const int32_t *page_table, void *k_pages, void *v_pages,
                            hipStream_t stream)
{
    const int D = plan->pool.head_dim;
    const int64_t chunks = (int64_t)plan->total_q * plan->pool.num_kv_heads * (D / 8);
    if (chunks == 0) return hipSuccess;
    const int64_t blocks = (chunks + 255) / 256;
    if (D == 128)
        hipLaunchKernelGGL((kv_append_kernel<128>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, page_table,
                           plan->max_pages_per_req, plan->d_tok_req, plan->d_ctx_lens,
                           plan->d_q_start, plan->pool.num_kv_heads, chunks, (uint16_t *)k_pages,
                           (uint16_t *)v_pages);
    else
        hipLaunchKernelGGL((kv_append_kernel<64>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, page_table,
                           plan->max_pages_per_req, plan->d_tok_req, plan->d_ctx_lens,
                           plan->d_q_start, plan->pool.num_kv_heads, chunks, (uint16_t *)k_pages,
                           (uint16_t *)v_pages);
    return hipGetLastError();
}

}  // namespace pv
