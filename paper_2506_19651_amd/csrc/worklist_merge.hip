// Work-list builder kernels and the log-sum-exp merge of split-KV partials.
#include "common.h"

namespace pevlm {

// One thread per work item: locate the sequence in the chunk table, then evaluate the closed-form
// item (the same inline function the host enumeration uses).
__global__ __launch_bounds__(256) void build_prefill_items_kernel(SeqTable tab, int32_t tile_rows,
                                                                  pevlm_work_item *items, int32_t item_offset)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    int32_t total = tab.item_base[tab.num_seqs];
    if (i >= total) return;
    int32_t s = 0;
    while (s + 1 < tab.num_seqs && i >= tab.item_base[s + 1]) ++s;
    items[item_offset + i] = prefill_item_sel(tab.start[s], tab.sink[s], tab.block[s], tab.ctx[s], tile_rows, tab.sel_first[s],
                                              tab.sel_sink, i - tab.item_base[s], tab.seq_index0 + s);
}

__global__ __launch_bounds__(256) void build_query_items_kernel(SeqTable tab, int32_t tile_rows, int32_t num_splits,
                                                                int32_t total_q_rows, int32_t align,
                                                                pevlm_work_item *items, int32_t item_offset,
                                                                int32_t *qrow_of_compact)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    int32_t total = tab.item_base[tab.num_seqs];
    if (i < total) {
        int32_t s = 0;
        while (s + 1 < tab.num_seqs && i >= tab.item_base[s + 1]) ++s;
        items[item_offset + i] =
            tab.windowed ? query_item_window(tab.start[s], tab.sink[s], tab.ctx[s], tab.query[s], tile_rows, num_splits,
                                             i - tab.item_base[s], tab.seq_index0 + s, tab.qrow_base[s], total_q_rows, align,
                                             tab.win_start[s])
                         : query_item(tab.start[s], tab.sink[s], tab.ctx[s], tab.query[s], tile_rows, num_splits,
                                      i - tab.item_base[s], tab.seq_index0 + s, tab.qrow_base[s], total_q_rows, align);
    }
    // packed row of every compact question row of this chunk
    int32_t stride = gridDim.x * blockDim.x;
    for (int32_t s = 0; s < tab.num_seqs; ++s)
        for (int32_t r = i; r < tab.query[s]; r += stride)
            qrow_of_compact[tab.qrow_base[s] + r] = tab.start[s] + tab.sink[s] + tab.ctx[s] + r;
}

// Same for the stream items of the bf16 streaming block-prefill kernel (item_base counts stream items).
__global__ __launch_bounds__(256) void build_stream_items_kernel(SeqTable tab, int32_t G, int32_t Hkv, HeadTable heads,
                                                                 pevlm_stream_item *items, int32_t item_offset)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    int32_t total = tab.item_base[tab.num_seqs];
    if (i >= total) return;
    int32_t s = 0;
    while (s + 1 < tab.num_seqs && i >= tab.item_base[s + 1]) ++s;
    items[item_offset + i] = stream_item(tab.start[s], tab.sink[s], tab.block[s], tab.ctx[s], G, Hkv, tab.sel_first[s], tab.sel_sink,
                                         i - tab.item_base[s], tab.seq_index0 + s, heads.head_order);
}

hipError_t launch_build_stream_items(const SeqTable &tab, int32_t G, int32_t Hkv, const HeadTable &heads,
                                     pevlm_stream_item *items, int32_t item_offset, hipStream_t stream)
{
    int32_t total = tab.item_base[tab.num_seqs];
    hipLaunchKernelGGL(build_stream_items_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, tab, G, Hkv, heads, items,
                       item_offset);
    return hipGetLastError();
}

hipError_t launch_build_prefill_items(const SeqTable &tab, int32_t tile_rows, pevlm_work_item *items,
                                      int32_t item_offset, hipStream_t stream)
{
    int32_t total = tab.item_base[tab.num_seqs];
    hipLaunchKernelGGL(build_prefill_items_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, tab, tile_rows, items,
                       item_offset);
    return hipGetLastError();
}

hipError_t launch_build_query_items(const SeqTable &tab, int32_t tile_rows, int32_t num_splits, int32_t total_q_rows,
                                    int32_t align, pevlm_work_item *items, int32_t item_offset, int32_t *qrow_of_compact,
                                    hipStream_t stream)
{
    int32_t total = tab.item_base[tab.num_seqs];
    int32_t blocks = (total + 255) / 256;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(build_query_items_kernel, dim3(blocks), dim3(256), 0, stream, tab, tile_rows, num_splits,
                       total_q_rows, align, items, item_offset, qrow_of_compact);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Merge of split-KV partials.  For one (question row, head) with partial s holding the running
// max m_s of the raw scores, l_s = sum exp(scale (score - m_s)) and acc_s = sum exp(...) v:
//   M = max_s m_s,  w_s = exp(scale (m_s - M)),  out = sum_s w_s acc_s / sum_s w_s l_s,
//   lse = scale M + log(sum_s w_s l_s).           (exact identity of Eq. 1's softmax)
// One thread per 4 output elements.
// ------------------------------------------------------------------------------------------
__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__global__ __launch_bounds__(256) void merge_kernel(MergeParams p)
{
    int32_t D = p.head_dim;
    int32_t per_unit = D / 4;
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t unit = gid / per_unit;  // (compact row, head)
    int32_t d4 = (int32_t)(gid % per_unit) * 4;
    int64_t n_units = (int64_t)p.total_q_rows * p.n_q_heads;
    if (unit >= n_units) return;
    int64_t stride_units = n_units;  // units per split
    float M = -INFINITY;
    for (int32_t s = 0; s < p.num_splits; ++s) M = fmaxf(M, p.part_ml[(s * stride_units + unit) * 2]);
    float denom = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t s = 0; s < p.num_splits; ++s) {
        const float *ml = p.part_ml + (s * stride_units + unit) * 2;
        float m = ml[0], l = ml[1];
        if (m == -INFINITY) continue;  // this split saw no key of the row
        float w = expf((m - M) * p.scale);
        denom += w * l;
        float4 a = *reinterpret_cast<const float4 *>(p.part_acc + (s * stride_units + unit) * D + d4);
        acc.x += w * a.x; acc.y += w * a.y; acc.z += w * a.z; acc.w += w * a.w;
    }
    float inv = 1.f / denom;
    int32_t row = p.qrow_of_compact[unit / p.n_q_heads];
    int32_t h = (int32_t)(unit % p.n_q_heads);
    int64_t o = ((int64_t)row * p.n_q_heads + h) * D + d4;
    if (p.is_bf16) {
        ushort4 r;
        r.x = f32_to_bf16_rne(acc.x * inv); r.y = f32_to_bf16_rne(acc.y * inv);
        r.z = f32_to_bf16_rne(acc.z * inv); r.w = f32_to_bf16_rne(acc.w * inv);
        *reinterpret_cast<ushort4 *>((uint16_t *)p.out + o) = r;
    } else {
        *reinterpret_cast<float4 *>((float *)p.out + o) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
    }
    if (p.lse && d4 == 0) p.lse[(int64_t)row * p.n_q_heads + h] = M * p.scale + logf(denom);
}

hipError_t launch_merge(const MergeParams &p, hipStream_t stream)
{
    int64_t threads = (int64_t)p.total_q_rows * p.n_q_heads * (p.head_dim / 4);
    hipLaunchKernelGGL(merge_kernel, dim3((uint32_t)((threads + 255) / 256)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace pevlm
