// Matrix-core attention kernel: work items of up to 128 query rows (new-prompt tokens, times the
// query heads of a GQA group) that share one KV head's K/V stream.
//
// Computes paper Eq. 2-3 with the causal rule of Section 4.4 for the rows of one item over the
// item's KV range, reading K and V through the page table: the pair of matrix products with the
// fused causal mask that Section 4.4 describes, fused flash-style so that the score matrix is
// never materialised.
//
// Mapping to gfx950.  One workgroup = 4 wavefronts = one item; wavefront w owns rows 32w..32w+31.
// The K/V page tiles of a 32-key block (two pages) are copied from HBM straight into LDS
// (global_load_lds, 16 bytes per lane, fully coalesced because a (page, head) tile is contiguous
// in the pool; no register staging, no ds_write) into a ring of three stages, two blocks ahead of
// their use, and every wavefront reads its matrix-core operands from there, so a tile is fetched
// once for all 128 rows.  The pool keeps runs of 8 elements along the contracted dimension
// together, so the plain linear copy already puts the operands where 16 consecutive lanes read 256
// consecutive bytes (no bank conflicts, no padding, no transposes).  Scores are produced
// transposed, S^T = K Q^T (v_mfma_f32_32x32x16), so each lane owns one query row (softmax without
// cross-lane traffic except one exchange for the maximum) and the probabilities are already the B
// operand of O^T += V^T P^T.  About 160 VGPRs and 48 KiB of LDS let three workgroups share a CU, whose
// wavefronts overlap each other's matrix-core, vector-ALU and LDS phases.  One raw s_barrier per
// block, preceded by a wait that leaves only the newest loads in flight.  Blocks that touch the
// causal boundary or the end of the sequence take a separate, masked instantiation so the
// steady-state loop has no branches.  The running maximum is only moved when a new score exceeds
// it by more than 2^8 (softmax is shift-invariant), which makes rescaling the accumulator rare.
#include <type_traits>

#include "pv_device.h"

namespace pv {

template <typename T, int D>
__global__ __launch_bounds__(256, 3) void attn_wide_kernel(
    const WorkItem *__restrict__ items, const uint16_t *__restrict__ q,
    const uint16_t *__restrict__ k_pages, const uint16_t *__restrict__ v_pages,
    const int32_t *__restrict__ page_table, int32_t max_pages, int32_t num_q_heads,
    int32_t num_kv_heads, int32_t group, float scale_log2e, uint32_t q_sign,
    uint16_t *__restrict__ out, float *__restrict__ ws_o, float *__restrict__ ws_ml)
{
    constexpr int BK = 32;                      // keys per block
    constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T
    constexpr int NB = D / 32;                  // 32-wide blocks of d in O^T
    constexpr int TILE_BYTES = 16 * D * 2;      // one (page, head) tile
    constexpr int HALF_BYTES = 2 * TILE_BYTES;  // K (or V) part of a stage: two pages
    constexpr int PASSES = HALF_BYTES / 4096;   // 16-byte copies per lane for K (same for V)
    constexpr int STAGES = 3;
    typedef typename T::vec8 vec8;
    __shared__ __attribute__((aligned(16))) unsigned char smem[STAGES][2 * HALF_BYTES];

    const WorkItem it = items[blockIdx.x];
    const int lane = lane_id();
    const int w = wave_id();
    const int q32 = lane & 31;
    const int h = lane >> 5;

    const int row = it.row_begin + 32 * w + q32;
    const bool valid = 32 * w + q32 < it.row_count;
    const int tok = valid ? row / group : 0;
    const int hq = it.kv_head * group + (valid ? row % group : 0);
    const int vis_end = valid ? it.ctx + tok + 1 : it.kv_end;
    // wavefront-uniform limits: below unmasked_end nothing is masked for this wavefront's rows
    // (and no slot is past the end); at or beyond wave_end nothing is visible to them
    const int wave_rows = it.row_count - 32 * w;  // may be <= 0
    int unmasked_end = it.ctx + (it.row_begin + 32 * w) / group + 1;
    if (unmasked_end > it.kv_end) unmasked_end = it.kv_end;
    int wave_end = 0;
    if (wave_rows > 0) {
        const int last = it.row_begin + 32 * w + (wave_rows < 32 ? wave_rows : 32) - 1;
        wave_end = it.ctx + last / group + 1;
        if (wave_end > it.kv_end) wave_end = it.kv_end;
    }

    vec8 qf[KS];
    {
        const uint16_t *qrow = q + ((int64_t)(it.q_row0 + tok) * num_q_heads + hq) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (valid) raw = load16(qrow + 16 * ks + 8 * h);
            raw ^= q_sign;  // a negative scale is applied as |scale| on negated queries
            qf[ks] = as_vec8<T>(raw);
        }
    }

    // LDS byte offsets of this lane's operands inside a stage.  S^T row i of the K operand is fed
    // with key pi(i) (bits 2 and 3 of i swapped) so that the accumulator registers of S^T, taken in
    // order, are exactly the 8 consecutive keys the P^T operand of the second product needs.
    const int key = (q32 & 0x13) | ((q32 & 4) << 1) | ((q32 & 8) >> 1);
    const int k_lds = (key >> 4) * TILE_BYTES + (h * 16 + (key & 15)) * 16;  // + ks * 512
    const int v_lds = HALF_BYTES + (h * D + q32) * 16;  // + page * TILE_BYTES + blk * 512

    const int32_t *pt = page_table + (int64_t)it.req * max_pages;
    const int last_pg = (it.kv_end - 1) >> 4;
    const int pg0 = it.kv_begin >> 4;
    const int nblocks = (it.kv_end - it.kv_begin + BK - 1) / BK;
    const int64_t head_off = (int64_t)it.kv_head * (16 * D);
    const int64_t page_stride = (int64_t)num_kv_heads * (16 * D);

    const uint32_t lane_bytes = (uint32_t)lane * 16u;
    // page ids of a block (two pages; a page past the end is never used, so any valid id will do)
    auto page_ids = [&](int b, int &id0, int &id1) {
        const int pg = pg0 + 2 * b;
        id0 = pt[pg <= last_pg ? pg : last_pg];
        id1 = pt[pg + 1 <= last_pg ? pg + 1 : last_pg];
    };
    // asynchronous copy of block b into stage b % 3: wavefront w moves bytes [w*1024, w*1024+1024)
    // of every 4 KiB pass, lane l the 16 bytes at 16*l of those (scalar base + lane offset)
    auto dma_block = [&](int b, int id0, int id1) {
        unsigned char *stage = smem[b % STAGES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int off = p * 4096 + w * 1024;  // wavefront-uniform
            const int page = off / TILE_BYTES ? id1 : id0;
            const int64_t elem = (int64_t)page * page_stride + head_off + (off % TILE_BYTES) / 2;
            lds_dma16(k_pages + elem, lane_bytes, stage + off);
            lds_dma16(v_pages + elem, lane_bytes, stage + HALF_BYTES + off);
        }
    };

    f32x16 o[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[blk][v] = 0.f;
    float m_run = -INFINITY;  // reference maximum of the RAW scores (before scaling)
    float l_run = 0.f;        // this lane's share of the running sum
    float mc = 0.f;           // m_run in the exp2 domain (0 while there is no reference yet)

    auto compute_block = [&](const unsigned char *sb, int kb0, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 kf = *reinterpret_cast<const u32x4 *>(sb + k_lds + ks * 512);
            s = T::mfma32(as_vec8<T>(kf), qf[ks], s);
        }
        // register v = 8*page + j  <->  key kb0 + 16*page + 8*h + j
        bool vis[16];
        if constexpr (MASKED) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                vis[v] = kb0 + 16 * (v >> 3) + 8 * h + (v & 7) < vis_end;
                if (!vis[v]) s[v] = -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
        // Lazy rescale: the reference maximum of a row only moves when a new score exceeds it by
        // more than 2^kLazyLog2 in the scaled domain (exact, because softmax is shift-invariant; the
        // probabilities just range up to 2^kLazyLog2 instead of 1).  Each lane tests the 16 keys it
        // holds; only when some lane of the wavefront sees such a score (or has no reference yet)
        // do the two lanes of a row exchange their maxima and the accumulators get rescaled.
        const bool grow = m_run == -INFINITY || (mx - m_run) * scale_log2e > kLazyLog2;
        if (__any(grow)) {
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new =
                (m_run == -INFINITY || (mx - m_run) * scale_log2e > kLazyLog2) ? mx : m_run;
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha =
                m_run == -INFINITY ? 0.f : fast_exp2((m_run - m_safe) * scale_log2e);
            mc = m_safe * scale_log2e;
            m_run = m_new;
            l_run *= alpha;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int blk = 0; blk < NB; ++blk) o[blk] *= alpha;
            }
        }
        // page by page: the matrix-core work of page 0 is issued before the exponentials of page 1,
        // so that inside this wavefront the two have something to overlap with
        float psum = 0.f;
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            u32x4 praw;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                float p0 = fast_exp2(__builtin_fmaf(s[8 * pg + 2 * jj], scale_log2e, -mc));
                float p1 = fast_exp2(__builtin_fmaf(s[8 * pg + 2 * jj + 1], scale_log2e, -mc));
                if constexpr (MASKED) {
                    p0 = vis[8 * pg + 2 * jj] ? p0 : 0.f;
                    p1 = vis[8 * pg + 2 * jj + 1] ? p1 : 0.f;
                }
                praw[jj] = T::pack2(p0, p1);
                psum = T::add_pair(praw[jj], psum);  // the sum of what the matrix core will see
            }
            const vec8 pf = as_vec8<T>(praw);
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                u32x4 vf = *reinterpret_cast<const u32x4 *>(sb + v_lds + pg * TILE_BYTES + blk * 512);
                if constexpr (MASKED) {  // slots past the end may hold anything: zero those values
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int kk = kb0 + 16 * pg + 8 * h + 2 * jj;
                        uint32_t word = vf[jj];
                        if (kk >= it.kv_end) word &= 0xFFFF0000u;
                        if (kk + 1 >= it.kv_end) word &= 0x0000FFFFu;
                        vf[jj] = word;
                    }
                }
                o[blk] = T::mfma32(as_vec8<T>(vf), pf, o[blk]);
            }
        }
        l_run += psum;
    };

    // prologue: blocks 0 and 1 on their way, block 0 landed and visible to everyone; the page ids
    // of the block after next are always fetched one iteration early
    int id0, id1;
    page_ids(0, id0, id1);
    dma_block(0, id0, id1);
    if (nblocks > 1) {
        page_ids(1, id0, id1);
        dma_block(1, id0, id1);
    }
    page_ids(2, id0, id1);
    asm volatile("" ::: "memory");
    // the queries (loaded first) and block 0 must be there; block 1 may still be on its way
    if (nblocks > 1)
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * PASSES, 0));
    else
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    for (int b = 0; b < nblocks; ++b) {
        const bool more = b + 2 < nblocks;
        if (more) dma_block(b + 2, id0, id1);  // its stage held block b-1: everyone is done with it
        page_ids(b + 3, id0, id1);
        const int kb0 = it.kv_begin + BK * b;
        if (kb0 < wave_end) {
            if (kb0 + BK <= unmasked_end)
                compute_block(smem[b % STAGES], kb0, std::false_type{});
            else
                compute_block(smem[b % STAGES], kb0, std::true_type{});
        }
        // block b+1 (issued one iteration ago) must have landed before the barrier publishes it;
        // this iteration's own copies may stay in flight.  This wavefront's LDS reads of block b
        // must have returned too: after the barrier the others refill that stage.  The scheduling
        // barrier keeps the block's last matrix-core instructions (which consume those reads) in
        // front of the wait, so the wait itself costs nothing.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        if (more)
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * PASSES, 0));
        else
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

    // ---- finish: every lane owns one row; the two half-waves hold partial sums ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!valid) return;
    if (it.split_count == 1) {
        const float inv = 1.f / l_tot;
        uint16_t *dst = out + ((int64_t)(it.q_row0 + tok) * num_q_heads + hq) * D;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int d = 32 * blk + 8 * a + 4 * h;
                *reinterpret_cast<u32x2 *>(dst + d) =
                    u32x2{T::pack2(o[blk][4 * a] * inv, o[blk][4 * a + 1] * inv),
                          T::pack2(o[blk][4 * a + 2] * inv, o[blk][4 * a + 3] * inv)};
            }
    } else {
        const int64_t slot = (int64_t)it.partial_base + 32 * w + q32;
        float *po = ws_o + slot * D;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int d = 32 * blk + 8 * a + 4 * h;
                *reinterpret_cast<f32x4 *>(po + d) = f32x4{o[blk][4 * a], o[blk][4 * a + 1],
                                                           o[blk][4 * a + 2], o[blk][4 * a + 3]};
            }
        if (h == 0) {
            // the merge works in the log2 domain of the scaled scores
            ws_ml[2 * slot] = m_run == -INFINITY ? -INFINITY : m_run * scale_log2e;
            ws_ml[2 * slot + 1] = l_tot;
        }
    }
}

template <typename T, int D>
static hipError_t launch_wide_t(const pv_plan *plan, const DeviceLists &dl, const void *q, const void *k_pages,
                                const void *v_pages, const int32_t *page_table, float scale,
                                void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    const int n = (int)plan->wide.size();
    const float c = (scale < 0.f ? -scale : scale) * kLog2e;
    const uint32_t q_sign = scale < 0.f ? 0x80008000u : 0u;
    hipLaunchKernelGGL((attn_wide_kernel<T, D>), dim3(n), dim3(256), 0, stream, dl.wide,
                       (const uint16_t *)q, (const uint16_t *)k_pages, (const uint16_t *)v_pages,
                       page_table, plan->max_pages_per_req, plan->num_q_heads,
                       plan->pool.num_kv_heads, plan->group, c, q_sign, (uint16_t *)out, ws_o,
                       ws_ml);
    return hipGetLastError();
}

hipError_t launch_attn_wide(const pv_plan *plan, const DeviceLists &dl, const void *q, const void *k_pages,
                            const void *v_pages, const int32_t *page_table, float scale, void *out,
                            float *ws_o, float *ws_ml, hipStream_t stream)
{
    if (plan->wide.empty()) return hipSuccess;
    const bool f = plan->pool.dtype == PV_F16;
    if (plan->pool.head_dim == 128)
        return f ? launch_wide_t<F16, 128>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                           ws_ml, stream)
                 : launch_wide_t<BF16, 128>(plan, dl, q, k_pages, v_pages, page_table, scale, out,
                                            ws_o, ws_ml, stream);
    return f ? launch_wide_t<F16, 64>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                      ws_ml, stream)
             : launch_wide_t<BF16, 64>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                       ws_ml, stream);
}

}  // namespace pv
