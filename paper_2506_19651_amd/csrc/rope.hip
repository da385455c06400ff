// Sequential rotary position embedding (Sec. "Position Encoding"): every token of a sequence is
// rotated at its index in the whole sequence; nothing restarts at a block boundary.
// HBM-bound: each element of q and k is read once and written once.
#include "common.h"
#include "rope_math.h"

namespace pevlm {

// A lane owns 8 consecutive pair indices i of one token: it loads x[i..i+8) and x[i+D/2..i+D/2+8)
// (16 bytes each in bf16), forms the 8 angles once in fp64, reduces them to [-pi, pi], and then
// walks over all query heads and key heads of that token.  D/16 lanes cover one token; a
// wavefront covers 64/(D/16) tokens, so every load instruction touches whole 128-byte lines.
//
// MROPE (three position axes: temporal, height, width; the scheme of the Qwen2.5-VL models of the
// paper's experiments): the token's three ids come from pos3 [3][T] in device memory and pair index
// i takes the id of the axis whose section holds i (sections are consecutive: [0, sec0),
// [sec0, sec01), [sec01, D/2)); `tab` is not used.
template <int D, bool BF16, bool MROPE>
__global__ __launch_bounds__(256) void rope_kernel(void *q, void *k, SeqTable tab, RopeFreq fr, int32_t Hq, int32_t Hkv,
                                                   int32_t row_begin, int32_t row_end, const int32_t *pos3, int64_t T,
                                                   int32_t sec0, int32_t sec01, float2 *table)
{
    constexpr int LANES_PER_TOKEN = D / 16;
    constexpr int TOKENS_PER_BLOCK = 256 / LANES_PER_TOKEN;
    int32_t tok = row_begin + blockIdx.x * TOKENS_PER_BLOCK + threadIdx.x / LANES_PER_TOKEN;
    if (tok >= row_end) return;
    int32_t i0 = (threadIdx.x % LANES_PER_TOKEN) * 8;
    // bf16: the first rows of the token are requested before the angles are formed, and each row is
    // requested four rows ahead of its use, so that the sine/cosine arithmetic and the rotation run
    // under the memory latency.  Rows of the token: its Hq query heads, then its Hkv key heads.
    constexpr int PF = 4;
    const int32_t nq = q ? Hq : 0, nrows = nq + (k ? Hkv : 0);
    uint16_t *const qrow = (uint16_t *)q + ((int64_t)tok * Hq) * D + i0;
    uint16_t *const krow = (uint16_t *)k + ((int64_t)tok * Hkv) * D + i0;
    uint4 plo[PF], phi[PF];
    if (BF16) {
#pragma unroll
        for (int j = 0; j < PF; ++j)
            if (j < nrows) {
                const uint16_t *x = j < nq ? qrow + (int64_t)j * D : krow + (int64_t)(j - nq) * D;
                plo[j] = *reinterpret_cast<const uint4 *>(x);
                phi[j] = *reinterpret_cast<const uint4 *>(x + D / 2);
            }
    }
    double pos = 0.0, pos_axis[3] = {0.0, 0.0, 0.0};
    if (MROPE) {
#pragma unroll
        for (int a = 0; a < 3; ++a) pos_axis[a] = (double)pos3[(int64_t)a * T + tok];
    } else {
        int32_t s = 0;
        while (s + 1 < tab.num_seqs && tok >= tab.start[s + 1]) ++s;
        pos = (double)(tok - tab.start[s] + tab.pos_offset[s]);
    }
    float cs[8], sn[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (MROPE) pos = i0 + j < sec0 ? pos_axis[0] : (i0 + j < sec01 ? pos_axis[1] : pos_axis[2]);
        rope_cos_sin<!BF16>(pos, fr.inv_freq[i0 + j], cs[j], sn[j]);
    }
    if (table) {  // by-product for the fused query rotation of the attention kernels: entry = packed row
        float2 *dst = table + (int64_t)tok * (D / 2) + i0;
#pragma unroll
        for (int j = 0; j < 8; j += 2) *reinterpret_cast<float4 *>(dst + j) = make_float4(cs[j], sn[j], cs[j + 1], sn[j + 1]);
    }
    if (BF16) {
        for (int32_t r0 = 0; r0 < nrows; r0 += PF) {
#pragma unroll
            for (int j = 0; j < PF; ++j) {
                const int32_t r = r0 + j;
                if (r >= nrows) break;
                uint16_t *x = r < nq ? qrow + (int64_t)r * D : krow + (int64_t)(r - nq) * D;
                const uint4 lo = plo[j], hi = phi[j];
                if (r + PF < nrows) {
                    const int32_t rn = r + PF;
                    const uint16_t *xn = rn < nq ? qrow + (int64_t)rn * D : krow + (int64_t)(rn - nq) * D;
                    plo[j] = *reinterpret_cast<const uint4 *>(xn);
                    phi[j] = *reinterpret_cast<const uint4 *>(xn + D / 2);
                }
                uint32_t l[4] = {lo.x, lo.y, lo.z, lo.w}, u[4] = {hi.x, hi.y, hi.z, hi.w};
                uint32_t ol[4], ou[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    float a0 = __uint_as_float(l[w] << 16), a1 = __uint_as_float(l[w] & 0xffff0000u);
                    float b0 = __uint_as_float(u[w] << 16), b1 = __uint_as_float(u[w] & 0xffff0000u);
                    float r0f, r1f, t0f, t1f;
                    rope_rotate(a0, b0, cs[2 * w], sn[2 * w], r0f, t0f);
                    rope_rotate(a1, b1, cs[2 * w + 1], sn[2 * w + 1], r1f, t1f);
                    ol[w] = rope_pack_bf16(r0f, r1f);
                    ou[w] = rope_pack_bf16(t0f, t1f);
                }
                *reinterpret_cast<uint4 *>(x) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
                *reinterpret_cast<uint4 *>(x + D / 2) = make_uint4(ou[0], ou[1], ou[2], ou[3]);
            }
        }
        return;
    }
    for (int pass = 0; pass < 2; ++pass) {
        void *base = pass == 0 ? q : k;
        int32_t H = pass == 0 ? Hq : Hkv;
        if (!base) continue;
        {
            float *x = (float *)base + ((int64_t)tok * H) * D + i0;
            for (int32_t h = 0; h < H; ++h, x += D) {
                float a[8], b[8];
                *reinterpret_cast<float4 *>(a) = *reinterpret_cast<const float4 *>(x);
                *reinterpret_cast<float4 *>(a + 4) = *reinterpret_cast<const float4 *>(x + 4);
                *reinterpret_cast<float4 *>(b) = *reinterpret_cast<const float4 *>(x + D / 2);
                *reinterpret_cast<float4 *>(b + 4) = *reinterpret_cast<const float4 *>(x + D / 2 + 4);
                float r[8], t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) rope_rotate(a[j], b[j], cs[j], sn[j], r[j], t[j]);
                *reinterpret_cast<float4 *>(x) = *reinterpret_cast<const float4 *>(r);
                *reinterpret_cast<float4 *>(x + 4) = *reinterpret_cast<const float4 *>(r + 4);
                *reinterpret_cast<float4 *>(x + D / 2) = *reinterpret_cast<const float4 *>(t);
                *reinterpret_cast<float4 *>(x + D / 2 + 4) = *reinterpret_cast<const float4 *>(t + 4);
            }
        }
    }
}

// cos/sin table for the query rotation fused into the bf16 attention kernel: entry e holds, for
// every pair index i, (cos, sin) of the angle of packed row row_of_entry[e] (e itself when
// row_of_entry is NULL).  Same arithmetic as rope_kernel, so a query rotated from the table gets the
// bits pevlm_rope_seq would have stored.  One thread per (entry, 8 pair indices).
template <int D>
__global__ __launch_bounds__(256) void rope_table_kernel(float2 *table, const int32_t *row_of_entry, SeqTable tab, RopeFreq fr,
                                                         int32_t entry_begin, int32_t entry_end, const int32_t *pos3, int64_t T,
                                                         int32_t sec0, int32_t sec01)
{
    constexpr int LANES_PER_ENTRY = D / 16;
    const int32_t e = entry_begin + (blockIdx.x * 256 + threadIdx.x) / LANES_PER_ENTRY;
    if (e >= entry_end) return;
    const int32_t i0 = (threadIdx.x % LANES_PER_ENTRY) * 8;
    const int32_t row = row_of_entry ? row_of_entry[e] : e;
    double pos_axis[3];
    if (pos3) {  // three position axes: pair index i takes the id of the axis whose section holds it
#pragma unroll
        for (int a = 0; a < 3; ++a) pos_axis[a] = (double)pos3[(int64_t)a * T + row];
    } else {
        int32_t s = 0;
        while (s + 1 < tab.num_seqs && row >= tab.start[s + 1]) ++s;
        pos_axis[0] = pos_axis[1] = pos_axis[2] = (double)(row - tab.start[s] + tab.pos_offset[s]);
        sec0 = sec01 = D;  // every pair index on axis 0
    }
    float2 *dst = table + (int64_t)e * (D / 2) + i0;
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        float c0, s0, c1, s1;
        const int32_t ia = i0 + j, ib = i0 + j + 1;
        rope_cos_sin<false>(ia < sec0 ? pos_axis[0] : (ia < sec01 ? pos_axis[1] : pos_axis[2]), fr.inv_freq[ia], c0, s0);
        rope_cos_sin<false>(ib < sec0 ? pos_axis[0] : (ib < sec01 ? pos_axis[1] : pos_axis[2]), fr.inv_freq[ib], c1, s1);
        *reinterpret_cast<float4 *>(dst + j) = make_float4(c0, s0, c1, s1);
    }
}

hipError_t launch_rope_table(float *table, const int32_t *row_of_entry, const SeqTable &tab, int32_t D, double rope_base,
                             int32_t entry_begin, int32_t entry_end, const int32_t *pos3, int64_t T, int32_t sec0, int32_t sec01,
                             hipStream_t stream)
{
    if (entry_end <= entry_begin) return hipSuccess;
    RopeFreq fr;
    for (int i = 0; i < 64; ++i) fr.inv_freq[i] = i < D / 2 ? pow(rope_base, -2.0 * (double)i / (double)D) : 0.0;
    const int32_t per_block = 256 / (D / 16);
    dim3 grid((entry_end - entry_begin + per_block - 1) / per_block);
    if (D == 128) hipLaunchKernelGGL((rope_table_kernel<128>), grid, dim3(256), 0, stream, (float2 *)table, row_of_entry, tab, fr, entry_begin, entry_end, pos3, T, sec0, sec01);
    else hipLaunchKernelGGL((rope_table_kernel<64>), grid, dim3(256), 0, stream, (float2 *)table, row_of_entry, tab, fr, entry_begin, entry_end, pos3, T, sec0, sec01);
    return hipGetLastError();
}

static void fill_freq(RopeFreq &fr, int32_t D, double rope_base)
{
    for (int i = 0; i < 64; ++i) fr.inv_freq[i] = i < D / 2 ? pow(rope_base, -2.0 * (double)i / (double)D) : 0.0;
}

template <bool MROPE>
static hipError_t launch_rope_any(void *q, void *k, const SeqTable &tab, int32_t Hq, int32_t Hkv, int32_t D, bool bf16,
                                  double rope_base, int32_t row_begin, int32_t row_end, const int32_t *pos3, int64_t T,
                                  int32_t sec0, int32_t sec01, float *table, hipStream_t stream)
{
    RopeFreq fr;
    fill_freq(fr, D, rope_base);
    if (row_end <= row_begin) return hipSuccess;
    int32_t tokens_per_block = 256 / (D / 16);
    dim3 grid((row_end - row_begin + tokens_per_block - 1) / tokens_per_block);
#define PEVLM_ROPE_LAUNCH(DD, BB) \
    hipLaunchKernelGGL((rope_kernel<DD, BB, MROPE>), grid, dim3(256), 0, stream, q, k, tab, fr, Hq, Hkv, row_begin, row_end, pos3, T, sec0, sec01, (float2 *)table)
    if (D == 128 && bf16) PEVLM_ROPE_LAUNCH(128, true);
    else if (D == 128) PEVLM_ROPE_LAUNCH(128, false);
    else if (bf16) PEVLM_ROPE_LAUNCH(64, true);
    else PEVLM_ROPE_LAUNCH(64, false);
#undef PEVLM_ROPE_LAUNCH
    return hipGetLastError();
}

hipError_t launch_rope(void *q, void *k, const SeqTable &tab, int32_t Hq, int32_t Hkv, int32_t D, bool bf16,
                       double rope_base, float *table, hipStream_t stream)
{
    int32_t n = tab.num_seqs;
    int32_t row_begin = tab.start[0];
    int32_t row_end = tab.start[n - 1] + tab.sink[n - 1] + tab.ctx[n - 1] + tab.query[n - 1];
    return launch_rope_any<false>(q, k, tab, Hq, Hkv, D, bf16, rope_base, row_begin, row_end, nullptr, 0, 0, 0, table, stream);
}

hipError_t launch_rope_mrope(void *q, void *k, int64_t T, int32_t Hq, int32_t Hkv, int32_t D, bool bf16, double rope_base,
                             const int32_t *pos3, int32_t sec0, int32_t sec01, float *table, hipStream_t stream)
{
    SeqTable tab = {};
    return launch_rope_any<true>(q, k, tab, Hq, Hkv, D, bf16, rope_base, 0, (int32_t)T, pos3, T, sec0, sec01, table, stream);
}

}  // namespace pevlm
