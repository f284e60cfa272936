// Page gather / scatter for tier swapping: whole pages leave the GPU pools for a staging buffer
// (swap-out, paper Section 4.3.2) and come back into newly assigned pages (swap-in, Section 4.3.3).
// The staging buffer may be device memory or pinned host memory that the GPU can address; with the
// latter the copy crosses PCIe inside the kernel, with no intermediate device buffer.
//
// Staging layout: for the i-th listed page, its K image (num_kv_heads * 16 * D elements, exactly
// as in the pool) followed by its V image.  One workgroup moves one 4 KiB piece with 16 bytes per
// lane; pure copies, bit-exact.
#include "pv_device.h"

namespace pv {

// GATHER = true : pools -> staging;  false : staging -> pools
template <bool GATHER>
__global__ __launch_bounds__(256) void pages_copy_kernel(
    const int32_t *__restrict__ page_ids, int64_t page_bytes, int32_t pieces_per_page,
    unsigned char *__restrict__ k_pages, unsigned char *__restrict__ v_pages,
    unsigned char *__restrict__ staging)
{
    const int i = (int)blockIdx.x / (2 * pieces_per_page);      // listed page
    const int rem = (int)blockIdx.x % (2 * pieces_per_page);
    const int which = rem / pieces_per_page;                    // 0 = K, 1 = V
    const int64_t off = (int64_t)(rem % pieces_per_page) * 4096 + (int64_t)threadIdx.x * 16;
    if (off >= page_bytes) return;
    const int64_t page = page_ids[i];
    unsigned char *pool = (which ? v_pages : k_pages) + page * page_bytes + off;
    unsigned char *stage = staging + ((int64_t)2 * i + which) * page_bytes + off;
    if (GATHER)
        *reinterpret_cast<u32x4 *>(stage) = load16_stream(pool);
    else
        *reinterpret_cast<u32x4 *>(pool) = load16_stream(stage);
}

hipError_t launch_pages_copy(bool gather, const pv_pool_desc *pool, const int32_t *page_ids,
                             int32_t n, void *k_pages, void *v_pages, void *staging,
                             hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    const int64_t page_bytes = (int64_t)pool->num_kv_heads * pool->page_size * pool->head_dim * 2;
    const int32_t pieces = (int32_t)((page_bytes + 4095) / 4096);
    const int64_t blocks = (int64_t)n * 2 * pieces;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (gather)
        hipLaunchKernelGGL((pages_copy_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           page_ids, page_bytes, pieces, (unsigned char *)k_pages,
                           (unsigned char *)v_pages, (unsigned char *)staging);
    else
        hipLaunchKernelGGL((pages_copy_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           page_ids, page_bytes, pieces, (unsigned char *)k_pages,
                           (unsigned char *)v_pages, (unsigned char *)staging);
    return hipGetLastError();
}

}  // namespace pv
