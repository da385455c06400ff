// FP8 (OCP E4M3) variant of the block-prefill step for gfx950 (CDNA4): rows of the sink (Eq. 3) and of the
// context blocks (Eq. 4) with Q K^T and P V on v_mfma_f32_32x32x64_f8f6f4 (fp32 accumulation, fp32
// online softmax).  Two stages:
//
//   quantise   bf16 Q, K, V -> E4M3 codes times power-of-two scales (Q: one scale per token and query
//              head; K, V: one scale per KV head over all tokens).  K and V are written as the
//              64-key tiles the attention kernel stages, one run of tiles per region (sink, each
//              context block), zero padded, already in the byte order the tile has in LDS; V tiles
//              are transposed (head_dim major) with the keys in the order in which a lane of the
//              score MFMA holds them, so that the weights go from the score registers to the value
//              MFMA without any exchange between lanes.
//   attend     one workgroup (4 wavefronts x 32 rows) per 128 query rows of a region and query head;
//              a K tile and a V tile per step are copied into LDS (two stages each) by asynchronous
//              global->LDS loads issued one tile ahead.
//
// Scores.  Q is quantised after multiplication by c = softmax factor * log2(e); the power-of-two scales of
// the query row and of the K head enter the score MFMAs as their 8-bit block exponents, and the
// accumulators start from 7 - m (m: the row's reference maximum): the MFMAs deliver the exponents of the
// weights, and the vector ALU is left with exp2, the row sum, the row maximum and the conversion.
//
// Weights.  p = exp2(c s - m + 7) is rounded to E4M3; m is a reference maximum of the row that is
// raised to the running maximum whenever that has outgrown it by more than one octave, so the
// largest weight of a row lies in [2^7, 2^8] (E4M3 reaches 448) and weights down to 2^-16 of the
// largest keep at least one significant bit.  The row sum is taken over the unrounded weights.
#include <algorithm>

#include "attn_bf16_tile.h"

namespace pevlm {

namespace {

typedef __attribute__((ext_vector_type(8))) int32_t i32x8;
typedef __attribute__((ext_vector_type(4))) int32_t i32x4v;

constexpr int32_t kExpLimit = 100;
constexpr float kWeightShift = 7.f;  // log2 of the weight of a key whose score equals the reference maximum
constexpr float kWeightLag = 1.f;    // octaves the running maximum may exceed the reference

// smallest e with amax * 2^-e <= 448 (0 for amax == 0), within [-100, 100]
__device__ __forceinline__ int32_t scale_exponent(float amax)
{
    if (!(amax > 0.f)) return 0;
    int x;
    const float f = frexpf(amax, &x);  // amax = f 2^x, f in [0.5, 1); 448 = 0.875 * 2^9
    int32_t e = (f <= 0.875f) ? x - 9 : x - 8;
    e = e < -kExpLimit ? -kExpLimit : e;
    return e > kExpLimit ? kExpLimit : e;
}
__device__ __forceinline__ float pow2(int32_t e) { return __int_as_float((127 + e) << 23); }  // |e| <= 126

// two fp32 values -> two E4M3 codes in the low or high half of a 32-bit word (round to nearest even)
template <bool HIGH>
__device__ __forceinline__ int32_t pack2(float a, float b, int32_t old)
{
    return __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, HIGH);
}
__device__ __forceinline__ i32x4v quantise16(const float (&x)[16], float inv_scale)
{
    i32x4v r;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int32_t v = pack2<false>(x[4 * w] * inv_scale, x[4 * w + 1] * inv_scale, 0);
        r[w] = pack2<true>(x[4 * w + 2] * inv_scale, x[4 * w + 3] * inv_scale, v);
    }
    return r;
}
__device__ __forceinline__ void bf16x8_to_f32(const uint4 &raw, float *dst)
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        dst[2 * i] = __uint_as_float(w[i] << 16);
        dst[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// position of the 16-byte chunk c of row r inside a staged tile whose rows hold CPR chunks: rows that
// 16 consecutive lanes read together are spread over all LDS banks
template <int CPR>
__host__ __device__ __forceinline__ int32_t swizzled_chunk(int32_t r, int32_t c)
{
    return c ^ ((r / (16 / CPR)) % CPR);
}

}  // namespace

// ---------------------------------------------------------------- work list
__global__ __launch_bounds__(256) void build_fp8_items_kernel(SeqTable tab, Fp8TileBases bases, Fp8Item *items, int32_t item_offset)
{
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= tab.item_base[tab.num_seqs]) return;
    int32_t s = 0;
    while (s + 1 < tab.num_seqs && i >= tab.item_base[s + 1]) ++s;
    const int32_t S = tab.sink[s], B = tab.block[s];
    const pevlm_work_item w = prefill_item(tab.start[s], S, B, tab.ctx[s], kFp8TileRows, i - tab.item_base[s], tab.seq_index0 + s);
    Fp8Item it;
    it.q_start = w.q_start;
    it.q_rows = w.q_rows;
    it.full_start = w.full_start;
    it.full_len = w.full_len;
    it.full_tile0 = bases.base[s];  // the sink is the first region of the sequence
    it.diag_start = w.diag_start;
    it.diag_len = w.diag_len;
    const int32_t local = w.diag_start - tab.start[s];  // first position of the item's own region
    it.diag_tile0 = bases.base[s] + (local < S ? 0 : ceil_div(S, kKeyTile) + ((local - S) / B) * ceil_div(B, kKeyTile));
    items[item_offset + i] = it;
}

__global__ void zero_words_kernel(uint32_t *p, int32_t n)
{
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ---------------------------------------------------------------- quantise
// Largest magnitude per KV head of K (amax[g]) and V (amax[Hkv + g]): blockIdx.y = head, blockIdx.z = tensor.
// Bit patterns of non-negative floats order like the floats, so the reduction is an integer maximum.
template <int D>
__global__ __launch_bounds__(256) void amax_kv_kernel(const uint16_t *k, const uint16_t *v, int64_t T, int32_t Hkv, uint32_t *amax)
{
    constexpr int CPR = D / 8;          // 16-byte chunks of bf16 per row of one head
    constexpr int RPS = 256 / CPR;      // rows per step of the workgroup
    const int32_t g = blockIdx.y;
    const uint16_t *src = blockIdx.z ? v : k;
    const int32_t c = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
    float m = 0.f;
    const int64_t step = (int64_t)gridDim.x * RPS;
    int64_t r = (int64_t)blockIdx.x * RPS + r0;
    for (; r + 3 * step < T; r += 4 * step) {  // four rows in flight per lane
        uint4 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) raw[u] = *reinterpret_cast<const uint4 *>(src + ((r + u * step) * Hkv + g) * D + c * 8);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float x[8];
            bf16x8_to_f32(raw[u], x);
#pragma unroll
            for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
        }
    }
    for (; r < T; r += step) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(src + (r * Hkv + g) * D + c * 8);
        float x[8];
        bf16x8_to_f32(raw, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    // one atomic per workgroup: atomics on the same word are served one after the other
    __shared__ float wave_max[4];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0)
        atomicMax(amax + blockIdx.z * Hkv + g, __float_as_uint(fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]))));
}

// Q: one scale per (token, head); D/16 consecutive lanes share a row of one head.  What is quantised is
// q * factor (factor = softmax factor * log2(e), one fp32 multiplication per element), so that the score
// MFMAs deliver base-2 exponents.
template <int D>
__global__ __launch_bounds__(256) void quantise_q_kernel(const uint16_t *q, int64_t n_rows_heads, float factor, uint8_t *codes, float *scales)
{
    constexpr int LPR = D / 16;  // lanes per row of one head
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rh = t / LPR;
    const int32_t c = (int32_t)(t % LPR);
    const bool live = rh < n_rows_heads;
    float x[16];
    if (live) {
        const uint4 *src = reinterpret_cast<const uint4 *>(q + rh * D + c * 16);
        bf16x8_to_f32(src[0], x);
        bf16x8_to_f32(src[1], x + 8);
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = __fmul_rn(x[i], factor);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = 0.f;
    }
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(x[i]));
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    const int32_t e = scale_exponent(m);
    if (live) {
        *reinterpret_cast<i32x4v *>(codes + rh * D + c * 16) = quantise16(x, pow2(-e));
        if (c == 0) scales[rh] = pow2(e);
    }
}

// K and V tiles: blockIdx.x = key tile (64 rows of one region), blockIdx.y = KV head.
//   K tile image: 64 rows of D bytes, chunk c of row r at chunk position swizzled_chunk<D/16>(r, c).
//   V tile image: D rows (head_dim) of 64 bytes; byte j of a row is key
//       kappa(j) = ((j % 32) / 16) * 32 + ((j % 16) / 4) * 8 + (j / 32) * 4 + j % 4
//   of the tile (the order in which the two halves of a wavefront hold the keys of a score tile);
//   chunk c of row d at chunk position swizzled_chunk<4>(d, c).
template <int D>
__global__ __launch_bounds__(256) void quantise_kv_tiles_kernel(const uint16_t *k, const uint16_t *v, const pevlm_work_item *key_tiles,
                                                                int32_t Hkv, const uint32_t *amax, uint8_t *k_tiles, uint8_t *v_tiles)
{
    constexpr int CPR = D / 16, TILEB = kKeyTile * D;
    __shared__ uint16_t vt[kKeyTile][D + 2];
    const int32_t tile = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
    const pevlm_work_item it = key_tiles[tile];
    const float k_inv = pow2(-scale_exponent(__uint_as_float(amax[g])));
    const float v_inv = pow2(-scale_exponent(__uint_as_float(amax[Hkv + g])));
    uint8_t *kdst = k_tiles + ((int64_t)tile * Hkv + g) * TILEB;
    uint8_t *vdst = v_tiles + ((int64_t)tile * Hkv + g) * TILEB;
    // K: 16 values of one row per step; V rows into LDS
    for (int32_t u = tid; u < kKeyTile * CPR; u += 256) {
        const int32_t r = u / CPR, c = u % CPR;
        float x[16];
        uint4 v0 = {0, 0, 0, 0}, v1 = {0, 0, 0, 0};
        if (r < it.q_rows) {
            const int64_t row = ((int64_t)(it.q_start + r) * Hkv + g) * D + c * 16;
            const uint4 *ks = reinterpret_cast<const uint4 *>(k + row);
            bf16x8_to_f32(ks[0], x);
            bf16x8_to_f32(ks[1], x + 8);
            const uint4 *vs = reinterpret_cast<const uint4 *>(v + row);
            v0 = vs[0];
            v1 = vs[1];
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = 0.f;
        }
        *reinterpret_cast<i32x4v *>(kdst + r * D + swizzled_chunk<CPR>(r, c) * 16) = quantise16(x, k_inv);
        const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<uint32_t *>(&vt[r][c * 16 + 2 * i]) = w[i];
    }
    __syncthreads();
    for (int32_t u = tid; u < D * 4; u += 256) {
        const int32_t d = u / 4, c = u % 4;
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int32_t j = c * 16 + i;
            const int32_t key = ((j % 32) / 16) * 32 + ((j % 16) / 4) * 8 + (j / 32) * 4 + j % 4;
            x[i] = __uint_as_float((uint32_t)vt[key][d] << 16);
        }
        *reinterpret_cast<i32x4v *>(vdst + d * kKeyTile + swizzled_chunk<4>(d, c) * 16) = quantise16(x, v_inv);
    }
}

// ---------------------------------------------------------------- attend
// Three wavefronts per SIMD (the second launch bound): it keeps the kernel within 168 registers, all of
// them ordinary vector registers -- given more, the compiler parks the MFMA results in accumulation
// registers and copies them back and forth around every softmax step (measured 24 % slower) -- and
// lets the vector work of one wavefront run under the MFMAs of the others.
template <int D>
__global__ __launch_bounds__(256, 3) void attn_fp8_kernel(Fp8Params p)
{
    constexpr int KT = kKeyTile, CPR = D / 16, TILEB = KT * D;
    constexpr int KQ = D / 64;            // score MFMAs (64 values of head_dim each) per 32-key chunk
    constexpr int DBLK = D / 32;          // 32-wide blocks of head_dim in O^T
    constexpr int NLD = TILEB / (256 * 16);
    constexpr int ROWB = D * 2, CH = D / 8, RPI = 1024 / ROWB, NOL = 32 * ROWB / 1024;  // output rows through LDS
    static_assert(4 * TILEB == 4 * 32 * ROWB, "the output slices reuse the four tile stages");
    __shared__ __attribute__((aligned(1024))) uint8_t lds[4 * TILEB];  // K stage 0, 1, V stage 0, 1

    // consecutive (item, head) pairs on one XCD: workgroup b runs on XCD b % 8
    const int32_t n_work = p.n_items * p.n_q_heads;
    const int32_t per_xcd = (n_work + 7) >> 3;
    const int32_t work = (int32_t)(blockIdx.x & 7) * per_xcd + (int32_t)(blockIdx.x >> 3);
    if ((int32_t)(blockIdx.x >> 3) >= per_xcd || work >= n_work) return;
    const Fp8Item it = p.items[work / p.n_q_heads];
    const int32_t head = p.heads.head_order[work % p.n_q_heads];
    const int32_t g = p.heads.kv_of_q[head];
    const int32_t Hq = p.n_q_heads, Hkv = p.n_kv_heads;

    const int32_t tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int32_t l32 = lane & 31, g32 = lane >> 5;
    const int32_t n_full = ceil_div(it.full_len, KT), n_tiles = n_full + ceil_div(it.diag_len, KT);
    const int32_t w_rows = min(max(it.q_rows - wave * 32, 0), 32);
    const int32_t wr_lo = it.q_start + wave * 32, wr_hi = wr_lo + w_rows - 1;
    int32_t n_w = 0;  // tiles this wavefront computes: all of the sink, its own region up to its last row
    if (w_rows > 0) n_w = n_full + min((wr_hi - it.diag_start) / KT + 1, n_tiles - n_full);
    const int32_t my_row = w_rows > 0 ? wr_lo + (l32 < w_rows ? l32 : w_rows - 1) : it.q_start;  // always a row of the item

    const uint32_t lds_addr = (uint32_t)(size_t)LDS_PTR(void, lds);
    const uint8_t *const k_head = p.k_tiles + (int64_t)g * TILEB, *const v_head = p.v_tiles + (int64_t)g * TILEB;
    const int64_t tile_stride = (int64_t)Hkv * TILEB;
#define PEVLM_FP8_LOAD_TILE(t, stage)                                                                              \
    do {                                                                                                           \
        const int64_t ti_ = (t) < n_full ? it.full_tile0 + (t) : it.diag_tile0 + ((t) - n_full);                   \
        const uint8_t *ks_ = uniform_ptr(k_head + ti_ * tile_stride), *vs_ = uniform_ptr(v_head + ti_ * tile_stride); \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                                          \
            load_lds_16_base(ks_, (uint32_t)((j * 256 + tid) * 16), lds_addr + (stage) * TILEB + (j * 4 + wave) * 1024); \
            load_lds_16_base(vs_, (uint32_t)((j * 256 + tid) * 16), lds_addr + (2 + (stage)) * TILEB + (j * 4 + wave) * 1024); \
        }                                                                                                          \
    } while (0)

    PEVLM_FP8_LOAD_TILE(0, 0);

    // query fragments: lane (row l32, half g32) holds head_dim [64 kk + 32 g32, +32) of its row
    i32x8 qf[KQ];
    {
        const uint8_t *qrow = p.q_codes + ((int64_t)my_row * Hq + head) * D;
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) {
            const i32x4v a = *reinterpret_cast<const i32x4v *>(qrow + kk * 64 + g32 * 32);
            const i32x4v b = *reinterpret_cast<const i32x4v *>(qrow + kk * 64 + g32 * 32 + 16);
            qf[kk] = i32x8{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
        }
    }
    // The scales of K (per head) and of the query row (per lane: both halves of the wavefront hold the same
    // rows) go into the score MFMAs as 8-bit exponents; the accumulators start from kWeightShift minus the
    // row's reference maximum, so the MFMAs deliver the exponents of the weights directly.
    const int32_t k_exp8 = 127 + scale_exponent(__uint_as_float(p.kv_amax[g]));
    const int32_t q_exp8 = (__float_as_int(p.q_scales[(int64_t)my_row * Hq + head]) >> 23) & 0xff;
    const float v_scale = pow2(scale_exponent(__uint_as_float(p.kv_amax[Hkv + g])));

    f32x16 o[DBLK], s[2];
#pragma unroll
    for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[b][i] = 0.f;
    float m_ref = -INFINITY, l_run = 0.f;
    float shift = kWeightShift;  // kWeightShift - (reference maximum, 0 while the row has none)
    f32x16 start;                // the same in all 16 accumulator registers of the lane
#pragma unroll
    for (int i = 0; i < 16; ++i) start[i] = shift;

    for (int32_t t = 0; t < n_tiles; ++t) {
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's share of tile t has landed
        __builtin_amdgcn_s_barrier();        // ... everybody's has, and everybody has left tile t - 1
        asm volatile("" ::: "memory");
        if (t + 1 < n_tiles) PEVLM_FP8_LOAD_TILE(t + 1, (t + 1) & 1);
        if (t >= n_w) continue;
        const uint8_t *tk = lds + (t & 1) * TILEB, *tv = lds + (2 + (t & 1)) * TILEB;
        // ---- S^T = K Q^T: rows = keys of the chunk, columns = this wavefront's query rows
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const int32_t r = kc * 32 + l32;
#pragma unroll
            for (int kk = 0; kk < KQ; ++kk) {
                const int32_t c0 = kk * 4 + g32 * 2;
                const i32x4v a = *reinterpret_cast<const i32x4v *>(tk + r * D + swizzled_chunk<CPR>(r, c0) * 16);
                const i32x4v b = *reinterpret_cast<const i32x4v *>(tk + r * D + swizzled_chunk<CPR>(r, c0 + 1) * 16);
                const i32x8 kf = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
                s[kc] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[kk], kk == 0 ? start : s[kc], 0, 0, 0, k_exp8, 0, q_exp8);
            }
        }
        int32_t k0, kend;
        bool causal;
        if (t < n_full) {
            k0 = it.full_start + t * KT; kend = it.full_start + it.full_len; causal = false;
        } else {
            k0 = it.diag_start + (t - n_full) * KT; kend = it.diag_start + it.diag_len; causal = true;
        }
        if ((k0 + KT > kend) || (causal && (k0 + KT - 1 > wr_lo))) mask_tile(s, k0, kend, causal, my_row, g32);
        // ---- reference maximum: raised to the running maximum once that is more than kWeightLag above it
        const float mx = row_max(s) - shift;
        const bool raise = mx > m_ref + kWeightLag;
        if (__any(raise)) {
            const float m_new = raise ? mx : m_ref;
            const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // 1 where nothing changes, 0 for the first tile
            m_ref = m_new;
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < DBLK; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
            // the scores of this tile move to the new reference; later tiles start from it
            const float new_shift = kWeightShift - ((m_ref == -INFINITY) ? 0.f : m_ref);
            const float delta = new_shift - shift;
            shift = new_shift;
#pragma unroll
            for (int kc = 0; kc < 2; ++kc)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kc][i] += delta;
#pragma unroll
            for (int i = 0; i < 16; ++i) start[i] = shift;
        }
        // ---- weights: E4M3 codes in the order the value MFMA wants them (byte 16 kc + i of the lane)
        float psum = 0.f;
        i32x8 pf;
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float w0 = __builtin_amdgcn_exp2f(s[kc][4 * w]);
                const float w1 = __builtin_amdgcn_exp2f(s[kc][4 * w + 1]);
                const float w2 = __builtin_amdgcn_exp2f(s[kc][4 * w + 2]);
                const float w3 = __builtin_amdgcn_exp2f(s[kc][4 * w + 3]);
                psum += (w0 + w1) + (w2 + w3);
                pf[kc * 4 + w] = pack2<true>(w2, w3, pack2<false>(w0, w1, 0));
            }
        l_run += psum;
        // ---- O^T += V^T P^T
#pragma unroll
        for (int b = 0; b < DBLK; ++b) {
            const int32_t d = b * 32 + l32;
            const i32x4v a = *reinterpret_cast<const i32x4v *>(tv + d * KT + swizzled_chunk<4>(d, g32 * 2) * 16);
            const i32x4v c = *reinterpret_cast<const i32x4v *>(tv + d * KT + swizzled_chunk<4>(d, g32 * 2 + 1) * 16);
            const i32x8 vf = {a[0], a[1], a[2], a[3], c[0], c[1], c[2], c[3]};
            o[b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf, pf, o[b], 0, 0, 0, 0, 0, 0);
        }
    }
#undef PEVLM_FP8_LOAD_TILE

    // ---- output: normalise, undo the V scale, rows out through LDS as whole 2 D-byte rows
    __syncthreads();  // every wavefront has left the tile stages
    uint8_t *slice = lds + wave * 32 * ROWB;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = v_scale / l_tot;
#pragma unroll
    for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            bf16x4 v4;
            v4[0] = (__bf16)(o[b][i4 * 4] * inv);
            v4[1] = (__bf16)(o[b][i4 * 4 + 1] * inv);
            v4[2] = (__bf16)(o[b][i4 * 4 + 2] * inv);
            v4[3] = (__bf16)(o[b][i4 * 4 + 3] * inv);
            *reinterpret_cast<bf16x4 *>(slice + l32 * ROWB + (((b * 4 + i4) ^ (l32 & (CH - 1))) << 4) + g32 * 8) = v4;
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint16_t *const obase = (uint16_t *)p.out;
    const int32_t cp = lane % CH;
#pragma unroll
    for (int j = 0; j < NOL; ++j) {
        const int32_t rl = j * RPI + lane / CH;
        const uint4 val = *reinterpret_cast<const uint4 *>(slice + rl * ROWB + ((cp ^ (rl & (CH - 1))) << 4));
        if (rl < w_rows) *reinterpret_cast<uint4 *>(obase + ((int64_t)(wr_lo + rl) * Hq + head) * D + cp * 8) = val;
    }
    if (p.lse && g32 == 0 && l32 < w_rows)
        p.lse[(int64_t)(wr_lo + l32) * Hq + head] = (m_ref - kWeightShift + __log2f(l_tot)) * 0.69314718056f;
}

// ---------------------------------------------------------------- launchers
hipError_t launch_build_fp8_items(const SeqTable &tab, const Fp8TileBases &bases, Fp8Item *items, int32_t item_offset, hipStream_t stream)
{
    const int32_t total = tab.item_base[tab.num_seqs];
    hipLaunchKernelGGL(build_fp8_items_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, tab, bases, items, item_offset);
    return hipGetLastError();
}

hipError_t launch_fp8_quantise(const void *q, const void *k, const void *v, int64_t T, int32_t Hq, int32_t Hkv, int32_t D,
                               float q_factor, const pevlm_work_item *key_tiles, int32_t n_key_tiles, uint32_t *kv_amax, float *q_scales,
                               uint8_t *q_codes, uint8_t *k_tiles, uint8_t *v_tiles, int32_t compute_units, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(256), 0, stream, kv_amax, 2 * Hkv);
    const int32_t rows_per_step = 256 / (D / 8);
    int32_t bx = (int32_t)std::min<int64_t>((T + rows_per_step - 1) / rows_per_step, std::max(1, 8 * compute_units / std::max(1, 2 * Hkv)));
    const int64_t q_threads = T * Hq * (D / 16);
    const dim3 q_grid((uint32_t)((q_threads + 255) / 256));
    if (D == 128) {
        hipLaunchKernelGGL((amax_kv_kernel<128>), dim3(bx, Hkv, 2), dim3(256), 0, stream, (const uint16_t *)k, (const uint16_t *)v, T, Hkv, kv_amax);
        hipLaunchKernelGGL((quantise_q_kernel<128>), q_grid, dim3(256), 0, stream, (const uint16_t *)q, T * Hq, q_factor, q_codes, q_scales);
        hipLaunchKernelGGL((quantise_kv_tiles_kernel<128>), dim3(n_key_tiles, Hkv), dim3(256), 0, stream, (const uint16_t *)k,
                           (const uint16_t *)v, key_tiles, Hkv, kv_amax, k_tiles, v_tiles);
    } else {
        hipLaunchKernelGGL((amax_kv_kernel<64>), dim3(bx, Hkv, 2), dim3(256), 0, stream, (const uint16_t *)k, (const uint16_t *)v, T, Hkv, kv_amax);
        hipLaunchKernelGGL((quantise_q_kernel<64>), q_grid, dim3(256), 0, stream, (const uint16_t *)q, T * Hq, q_factor, q_codes, q_scales);
        hipLaunchKernelGGL((quantise_kv_tiles_kernel<64>), dim3(n_key_tiles, Hkv), dim3(256), 0, stream, (const uint16_t *)k,
                           (const uint16_t *)v, key_tiles, Hkv, kv_amax, k_tiles, v_tiles);
    }
    return hipGetLastError();
}

hipError_t launch_attn_fp8(const Fp8Params &p, int32_t D, hipStream_t stream)
{
    const int32_t n_work = p.n_items * p.n_q_heads;
    const dim3 grid(8 * ((n_work + 7) / 8)), block(256);
    if (D == 128) hipLaunchKernelGGL((attn_fp8_kernel<128>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((attn_fp8_kernel<64>), grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace pevlm
