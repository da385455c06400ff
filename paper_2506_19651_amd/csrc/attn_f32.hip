// fp32 attention kernels (plain FMA, no matrix cores): the numerical anchor of the library and the
// path taken for fp32 tensors.  One wavefront owns one query row of a work item; lanes run over
// keys for the scores and over head_dim for the weighted sum of values.
#include "common.h"

namespace pevlm {

__device__ inline float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

template <int D, bool PARTIAL>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnParams p)
{
    constexpr int NW = 4;
    constexpr int DV = D / 64;
    __shared__ float q_s[NW][D];
    __shared__ float p_s[NW][64];
    const pevlm_work_item it = p.items[blockIdx.x];
    const int32_t h = blockIdx.y;
    const int32_t g = p.heads.kv_of_q[h];
    const int32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int32_t Hq = p.n_q_heads, Hkv = p.n_kv_heads;
    const float *Q = (const float *)p.q, *K = (const float *)p.k, *V = (const float *)p.v;

    for (int32_t rr = wave; rr < it.q_rows; rr += NW) {
        const int32_t row = it.q_start + rr;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < DV; ++c) q_s[wave][lane + 64 * c] = Q[((int64_t)row * Hq + h) * D + lane + 64 * c];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float m = -INFINITY, l = 0.f, acc[DV];
#pragma unroll
        for (int c = 0; c < DV; ++c) acc[c] = 0.f;
        for (int seg = 0; seg < 2; ++seg) {
            const int32_t start = seg == 0 ? it.full_start : it.diag_start;
            int32_t n = seg == 0 ? it.full_len : it.diag_len;
            if (seg == 1 && row - start + 1 < n) n = row - start + 1;  // causal: keys <= row
            for (int32_t k0 = 0; k0 < n; k0 += 64) {
                const int32_t j = k0 + lane;
                float s = -INFINITY;
                if (j < n) {
                    const float4 *kp = reinterpret_cast<const float4 *>(K + ((int64_t)(start + j) * Hkv + g) * D);
                    float dot = 0.f;
#pragma unroll 8
                    for (int d = 0; d < D / 4; ++d) {
                        float4 kv = kp[d];
                        dot += q_s[wave][4 * d] * kv.x + q_s[wave][4 * d + 1] * kv.y + q_s[wave][4 * d + 2] * kv.z +
                               q_s[wave][4 * d + 3] * kv.w;
                    }
                    s = dot;
                }
                const float m_new = fmaxf(m, wave_max(s));  // finite: lane 0 always holds a key
                const float pj = j < n ? expf((s - m_new) * p.scale) : 0.f;
                const float alpha = expf((m - m_new) * p.scale);  // m = -inf gives 0
                l = l * alpha + wave_sum(pj);
#pragma unroll
                for (int c = 0; c < DV; ++c) acc[c] *= alpha;
                m = m_new;
                __builtin_amdgcn_wave_barrier();
                p_s[wave][lane] = pj;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int32_t cnt = n - k0 < 64 ? n - k0 : 64;
                for (int32_t jj = 0; jj < cnt; ++jj) {
                    const float w = p_s[wave][jj];
                    const float *vp = V + ((int64_t)(start + k0 + jj) * Hkv + g) * D;
#pragma unroll
                    for (int c = 0; c < DV; ++c) acc[c] += w * vp[lane + 64 * c];
                }
            }
        }
        if (PARTIAL) {
            const int64_t slot = (int64_t)it.reserved + rr;
#pragma unroll
            for (int c = 0; c < DV; ++c) p.part_acc[(slot * Hq + h) * D + lane + 64 * c] = acc[c];
            if (lane == 0) {
                p.part_ml[(slot * Hq + h) * 2] = m;
                p.part_ml[(slot * Hq + h) * 2 + 1] = l;
            }
        } else {
            const float inv = 1.f / l;
#pragma unroll
            for (int c = 0; c < DV; ++c) ((float *)p.out)[((int64_t)row * Hq + h) * D + lane + 64 * c] = acc[c] * inv;
            if (p.lse && lane == 0) p.lse[(int64_t)row * Hq + h] = m * p.scale + logf(l);
        }
    }
}

hipError_t launch_attn_f32(const AttnParams &p, int32_t D, bool partial, hipStream_t stream)
{
    dim3 grid(p.n_items, p.n_q_heads), block(256);
    if (D == 128) {
        if (partial) hipLaunchKernelGGL((attn_f32_kernel<128, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((attn_f32_kernel<128, false>), grid, block, 0, stream, p);
    } else {
        if (partial) hipLaunchKernelGGL((attn_f32_kernel<64, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((attn_f32_kernel<64, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace pevlm
