// Sequential rotary position embedding (Sec. "Position Encoding"): every token of a sequence is
// rotated at its index in the whole sequence; nothing restarts at a block boundary.
// HBM-bound: each element of q and k is read once and written once.
#include "common.h"

namespace pevlm {

struct RopeFreq {
    double inv_freq[64];  // rope_base^(-2i/D), i < D/2
};

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
                                                   int32_t sec0, int32_t sec01)
{
    constexpr int LANES_PER_TOKEN = D / 16;
    constexpr int TOKENS_PER_BLOCK = 256 / LANES_PER_TOKEN;
    int32_t tok = row_begin + blockIdx.x * TOKENS_PER_BLOCK + threadIdx.x / LANES_PER_TOKEN;
    if (tok >= row_end) return;
    int32_t i0 = (threadIdx.x % LANES_PER_TOKEN) * 8;
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
        double theta = pos * fr.inv_freq[i0 + j];
        const double two_pi = 6.283185307179586476925286766559;
        double r = theta - two_pi * rint(theta / two_pi);
        if (BF16) {
            sincosf((float)r, &sn[j], &cs[j]);
        } else {
            double sd, cd;
            sincos(r, &sd, &cd);
            sn[j] = (float)sd;
            cs[j] = (float)cd;
        }
    }
    for (int pass = 0; pass < 2; ++pass) {
        void *base = pass == 0 ? q : k;
        int32_t H = pass == 0 ? Hq : Hkv;
        if (!base) continue;
        if (BF16) {
            uint16_t *x = (uint16_t *)base + ((int64_t)tok * H) * D + i0;
#pragma unroll 4
            for (int32_t h = 0; h < H; ++h, x += D) {
                uint4 lo = *reinterpret_cast<const uint4 *>(x);
                uint4 hi = *reinterpret_cast<const uint4 *>(x + D / 2);
                uint32_t l[4] = {lo.x, lo.y, lo.z, lo.w}, u[4] = {hi.x, hi.y, hi.z, hi.w};
                uint32_t ol[4], ou[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    float a0 = __uint_as_float(l[w] << 16), a1 = __uint_as_float(l[w] & 0xffff0000u);
                    float b0 = __uint_as_float(u[w] << 16), b1 = __uint_as_float(u[w] & 0xffff0000u);
                    float r0 = a0 * cs[2 * w] - b0 * sn[2 * w], r1 = a1 * cs[2 * w + 1] - b1 * sn[2 * w + 1];
                    float t0 = b0 * cs[2 * w] + a0 * sn[2 * w], t1 = b1 * cs[2 * w + 1] + a1 * sn[2 * w + 1];
                    uint32_t x0 = __float_as_uint(r0), x1 = __float_as_uint(r1);
                    uint32_t y0 = __float_as_uint(t0), y1 = __float_as_uint(t1);
                    x0 += 0x7fffu + ((x0 >> 16) & 1u); x1 += 0x7fffu + ((x1 >> 16) & 1u);
                    y0 += 0x7fffu + ((y0 >> 16) & 1u); y1 += 0x7fffu + ((y1 >> 16) & 1u);
                    ol[w] = (x0 >> 16) | (x1 & 0xffff0000u);
                    ou[w] = (y0 >> 16) | (y1 & 0xffff0000u);
                }
                *reinterpret_cast<uint4 *>(x) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
                *reinterpret_cast<uint4 *>(x + D / 2) = make_uint4(ou[0], ou[1], ou[2], ou[3]);
            }
        } else {
            float *x = (float *)base + ((int64_t)tok * H) * D + i0;
            for (int32_t h = 0; h < H; ++h, x += D) {
                float a[8], b[8];
                *reinterpret_cast<float4 *>(a) = *reinterpret_cast<const float4 *>(x);
                *reinterpret_cast<float4 *>(a + 4) = *reinterpret_cast<const float4 *>(x + 4);
                *reinterpret_cast<float4 *>(b) = *reinterpret_cast<const float4 *>(x + D / 2);
                *reinterpret_cast<float4 *>(b + 4) = *reinterpret_cast<const float4 *>(x + D / 2 + 4);
                float r[8], t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    r[j] = a[j] * cs[j] - b[j] * sn[j];
                    t[j] = b[j] * cs[j] + a[j] * sn[j];
                }
                *reinterpret_cast<float4 *>(x) = *reinterpret_cast<const float4 *>(r);
                *reinterpret_cast<float4 *>(x + 4) = *reinterpret_cast<const float4 *>(r + 4);
                *reinterpret_cast<float4 *>(x + D / 2) = *reinterpret_cast<const float4 *>(t);
                *reinterpret_cast<float4 *>(x + D / 2 + 4) = *reinterpret_cast<const float4 *>(t + 4);
            }
        }
    }
}

static void fill_freq(RopeFreq &fr, int32_t D, double rope_base)
{
    for (int i = 0; i < 64; ++i) fr.inv_freq[i] = i < D / 2 ? pow(rope_base, -2.0 * (double)i / (double)D) : 0.0;
}

template <bool MROPE>
static hipError_t launch_rope_any(void *q, void *k, const SeqTable &tab, int32_t Hq, int32_t Hkv, int32_t D, bool bf16,
                                  double rope_base, int32_t row_begin, int32_t row_end, const int32_t *pos3, int64_t T,
                                  int32_t sec0, int32_t sec01, hipStream_t stream)
{
    RopeFreq fr;
    fill_freq(fr, D, rope_base);
    if (row_end <= row_begin) return hipSuccess;
    int32_t tokens_per_block = 256 / (D / 16);
    dim3 grid((row_end - row_begin + tokens_per_block - 1) / tokens_per_block);
#define PEVLM_ROPE_LAUNCH(DD, BB) \
    hipLaunchKernelGGL((rope_kernel<DD, BB, MROPE>), grid, dim3(256), 0, stream, q, k, tab, fr, Hq, Hkv, row_begin, row_end, pos3, T, sec0, sec01)
    if (D == 128 && bf16) PEVLM_ROPE_LAUNCH(128, true);
    else if (D == 128) PEVLM_ROPE_LAUNCH(128, false);
    else if (bf16) PEVLM_ROPE_LAUNCH(64, true);
    else PEVLM_ROPE_LAUNCH(64, false);
#undef PEVLM_ROPE_LAUNCH
    return hipGetLastError();
}

hipError_t launch_rope(void *q, void *k, const SeqTable &tab, int32_t Hq, int32_t Hkv, int32_t D, bool bf16,
                       double rope_base, hipStream_t stream)
{
    int32_t n = tab.num_seqs;
    int32_t row_begin = tab.start[0];
    int32_t row_end = tab.start[n - 1] + tab.sink[n - 1] + tab.ctx[n - 1] + tab.query[n - 1];
    return launch_rope_any<false>(q, k, tab, Hq, Hkv, D, bf16, rope_base, row_begin, row_end, nullptr, 0, 0, 0, stream);
}

hipError_t launch_rope_mrope(void *q, void *k, int64_t T, int32_t Hq, int32_t Hkv, int32_t D, bool bf16, double rope_base,
                             const int32_t *pos3, int32_t sec0, int32_t sec01, hipStream_t stream)
{
    SeqTable tab = {};
    return launch_rope_any<true>(q, k, tab, Hq, Hkv, D, bf16, rope_base, 0, (int32_t)T, pos3, T, sec0, sec01, stream);
}

}  // namespace pevlm
