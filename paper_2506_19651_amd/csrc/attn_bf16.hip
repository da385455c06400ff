// bf16 flash-style attention kernel for gfx950 (CDNA4): bf16 MFMA for Q K^T and P V with fp32
// accumulation, fp32 online softmax.  Serves the block-parallel prefill (sink rows, Eq. 3, and
// context-block rows, Eq. 4: a work item names a tile of query rows plus the sink key range and the
// own-block key range up to the diagonal, nothing else) and, in partial mode, the split-KV question
// attention (Eq. 5).
//
// Tiling.  A workgroup of 4 wavefronts owns one work item (<= 128 query rows of one head); wave w
// owns rows 32w..32w+31.  Keys are staged 64 at a time in LDS (K and V tiles, XOR-swizzled 16-byte
// chunks).  Scores are formed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: in the
// accumulator layout a lane then holds 16 keys of ONE query (column = lane % 32), so the softmax
// row reduction is 15 in-lane max/add operations and a single exchange with lane ^ 32.  The same
// registers, converted to bf16, are directly the B operand of O^T += V^T P^T; V^T fragments come
// from LDS through the transposing read ds_read_b64_tr_b16.
#include "common.h"

namespace pevlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

template <int D, bool PARTIAL>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnParams p, int32_t n_logical, int32_t heads_inner)
{
    constexpr int KT = kKeyTile;          // keys per staged tile
    constexpr int ROWB = D * 2;           // bytes per K/V row
    constexpr int CH = D / 8;             // 16-byte chunks per row
    constexpr int NLD = KT * CH / 256;    // chunks each thread moves per tensor per tile
    constexpr int KSTEPS = D / 16;        // MFMA k-steps of Q K^T
    constexpr int DBLK = D / 32;          // 32-wide blocks of head_dim in O^T
    constexpr int VSW = CH / 4 - 1;       // V swizzle mask (64-byte granules per row - 1)
    constexpr int TILEB = KT * ROWB;      // bytes of one staged K (or V) tile
    constexpr int RPI = 1024 / ROWB;      // rows one wavefront-wide 16-byte-per-lane load covers
    __shared__ __attribute__((aligned(1024))) uint8_t lds_k[2 * TILEB];
    __shared__ __attribute__((aligned(1024))) uint8_t lds_v[2 * TILEB];

    // Workgroup -> logical id.  Consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2); give every XCD one contiguous run of logical ids so that the heads of a GQA
    // group working on the same context block share that XCD's L2.
    const int32_t per_xcd = gridDim.x >> 3;
    const int32_t logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= n_logical) return;
    const int32_t inner = logical % heads_inner;
    const int32_t rest = logical / heads_inner;
    const int32_t item_idx = rest % p.n_items;
    const int32_t hs = (rest / p.n_items) * heads_inner + inner;
    const pevlm_work_item it = p.items[item_idx];
    const int32_t h = p.heads.head_order[hs];
    const int32_t g = p.heads.kv_of_q[h];
    const int32_t Hq = p.n_q_heads, Hkv = p.n_kv_heads;

    const int32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t l32 = lane & 31, g32 = lane >> 5;
    const uint16_t *Q = (const uint16_t *)p.q, *K = (const uint16_t *)p.k, *V = (const uint16_t *)p.v;

    // ---- this lane's query row, Q fragments (B operand of S^T = K Q^T) stay in registers ----
    const int32_t row_in_tile = wave * 32 + l32;
    const bool row_valid = row_in_tile < it.q_rows;
    const int32_t my_row = it.q_start + (row_valid ? row_in_tile : it.q_rows - 1);
    const bool wave_active = wave * 32 < it.q_rows;
    const int32_t wr_lo = it.q_start + wave * 32;
    const int32_t wr_hi = it.q_start + ((wave * 32 + 31 < it.q_rows) ? wave * 32 + 31 : it.q_rows - 1);
    bf16x8 qf[KSTEPS];
    {
        const uint16_t *qp = Q + ((int64_t)my_row * Hq + h) * D + g32 * 8;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + kk * 16);
    }

    const float c_log2 = p.scale * 1.4426950408889634f;
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o[DBLK];
#pragma unroll
    for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[b][i] = 0.f;

    const int32_t n_full_tiles = (it.full_len + KT - 1) / KT;
    const int32_t n_tiles = n_full_tiles + (it.diag_len + KT - 1) / KT;

    // ---- K/V tiles go straight from global memory into LDS (global_load_lds, 16 bytes per lane): a
    // wavefront instruction fills 1 KB of contiguous LDS, i.e. RPI whole rows; the XOR swizzle is
    // applied by choosing which 16-byte chunk of the row each lane fetches.  Two LDS stages: tile
    // t+1 streams in while tile t is consumed.  Rows past the key range repeat its last key (their
    // scores are masked, their values stay finite).
#define PEVLM_TILE_RANGE(t, k0, kend, causal)                 \
    do {                                                      \
        if ((t) < n_full_tiles) {                             \
            k0 = it.full_start + (t) * KT;                    \
            kend = it.full_start + it.full_len;               \
            causal = false;                                   \
        } else {                                              \
            k0 = it.diag_start + ((t) - n_full_tiles) * KT;   \
            kend = it.diag_start + it.diag_len;               \
            causal = true;                                    \
        }                                                     \
    } while (0)
#define PEVLM_ISSUE_TILE(t, stage)                                                                        \
    do {                                                                                                  \
        int32_t pk0, pkend;                                                                               \
        bool pcausal;                                                                                     \
        PEVLM_TILE_RANGE(t, pk0, pkend, pcausal);                                                         \
        (void)pcausal;                                                                                    \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                                 \
            const int32_t rbase = (j * 4 + wave) * RPI;                                                   \
            const int32_t row = rbase + lane / CH, cpos = lane % CH;                                      \
            int32_t key = pk0 + row;                                                                      \
            key = key < pkend ? key : pkend - 1;                                                          \
            const int64_t roff = ((int64_t)key * Hkv + g) * D;                                            \
            const uint16_t *ksrc = K + roff + ((cpos ^ (row & (CH - 1))) << 3);                           \
            const uint16_t *vsrc = V + roff + ((cpos ^ ((row & VSW) << 2)) << 3);                         \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)ksrc,        \
                                             LDS_PTR(void, lds_k + (stage) * TILEB + rbase * ROWB), 16, 0, 0); \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)vsrc,        \
                                             LDS_PTR(void, lds_v + (stage) * TILEB + rbase * ROWB), 16, 0, 0); \
        }                                                                                                 \
    } while (0)

    if (n_tiles > 0) PEVLM_ISSUE_TILE(0, 0);
    for (int32_t t = 0; t < n_tiles; ++t) {
        const int32_t stage = t & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's part of tile t has landed in LDS
        __syncthreads();                     // ... and everyone's; all waves are done with tile t-1
        if (t + 1 < n_tiles) PEVLM_ISSUE_TILE(t + 1, stage ^ 1);
        const uint8_t *tk = lds_k + stage * TILEB;
        const uint8_t *tv = lds_v + stage * TILEB;
        int32_t k0, kend;
        bool causal;
        PEVLM_TILE_RANGE(t, k0, kend, causal);

        // keys of this tile the wave needs, in 32-key chunks
        int32_t lim = kend - k0;
        if (causal && wr_hi - k0 + 1 < lim) lim = wr_hi - k0 + 1;
        const int32_t nkc = (!wave_active || lim <= 0) ? 0 : (lim > 32 ? 2 : 1);
        if (nkc == 0) continue;
        const bool need_mask = (k0 + nkc * 32 > kend) || (causal && (k0 + nkc * 32 - 1 > wr_lo));

        // ---- S^T = K Q^T ----
        f32x16 s[2];
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
#pragma unroll
            for (int i = 0; i < 16; ++i) s[kc][i] = 0.f;
            if (kc < nkc) {
                const int32_t row = kc * 32 + l32;
#pragma unroll
                for (int kk = 0; kk < KSTEPS; ++kk) {
                    const int32_t ch = kk * 2 + g32;
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(tk + row * ROWB + ((ch ^ (row & (CH - 1))) << 4));
                    s[kc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[kc], 0, 0, 0);
                }
            }
        }
        // ---- mask (only tiles that touch the diagonal or the end of the key range) ----
        if (need_mask) {
#pragma unroll
            for (int kc = 0; kc < 2; ++kc)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int32_t key = k0 + kc * 32 + (i >> 2) * 8 + g32 * 4 + (i & 3);
                    const bool ok = key < kend && (!causal || key <= my_row);
                    s[kc][i] = ok ? s[kc][i] : -INFINITY;
                }
        }
        // ---- online softmax: a lane holds 16 (or 32) keys of its own query ----
        float mx = -INFINITY;
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
            if (kc < nkc)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kc][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c_log2);
        const float mc = m_use * c_log2;
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
            if (kc < nkc) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float e = __builtin_amdgcn_exp2f(s[kc][i] * c_log2 - mc);
                    psum += e;
                    pf[kc * 2 + (i >> 3)][i & 7] = (__bf16)e;
                }
            }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.f)) {  // the running maximum of some row moved: rescale the accumulators
#pragma unroll
            for (int b = 0; b < DBLK; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
        }

        // ---- O^T += V^T P^T ----
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < nkc * 2) {
#pragma unroll
                for (int b = 0; b < DBLK; ++b) {
                    bf16x8 a;
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt) {
                        const int32_t row = ks * 16 + tt * 8 + g32 * 4 + ((lane & 15) >> 2);
                        const int32_t dcol = b * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
                        const int32_t ch = dcol >> 3;
                        const uint8_t *ptr = tv + row * ROWB + ((ch ^ ((row & VSW) << 2)) << 4) + (dcol & 7) * 2;
                        const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ptr));
                        const bf16x4 rb = __builtin_bit_cast(bf16x4, r);
                        a[tt * 4 + 0] = rb[0]; a[tt * 4 + 1] = rb[1]; a[tt * 4 + 2] = rb[2]; a[tt * 4 + 3] = rb[3];
                    }
                    o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[ks], o[b], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!row_valid) return;
    if (PARTIAL) {
        const int64_t slot = (int64_t)it.reserved + row_in_tile;
        float *acc = p.part_acc + (slot * Hq + h) * D;
#pragma unroll
        for (int b = 0; b < DBLK; ++b)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int32_t d = b * 32 + i4 * 8 + g32 * 4;
                f32x4 v4 = {o[b][i4 * 4], o[b][i4 * 4 + 1], o[b][i4 * 4 + 2], o[b][i4 * 4 + 3]};
                *reinterpret_cast<f32x4 *>(acc + d) = v4;
            }
        if (g32 == 0) {
            p.part_ml[(slot * Hq + h) * 2] = m_run;
            p.part_ml[(slot * Hq + h) * 2 + 1] = l_tot;
        }
    } else {
        const float inv = 1.f / l_tot;
        uint16_t *op = (uint16_t *)p.out + ((int64_t)my_row * Hq + h) * D;
#pragma unroll
        for (int b = 0; b < DBLK; ++b)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int32_t d = b * 32 + i4 * 8 + g32 * 4;
                bf16x4 v4;
                v4[0] = (__bf16)(o[b][i4 * 4] * inv);
                v4[1] = (__bf16)(o[b][i4 * 4 + 1] * inv);
                v4[2] = (__bf16)(o[b][i4 * 4 + 2] * inv);
                v4[3] = (__bf16)(o[b][i4 * 4 + 3] * inv);
                *reinterpret_cast<bf16x4 *>(op + d) = v4;
            }
        if (p.lse && g32 == 0) p.lse[(int64_t)my_row * Hq + h] = m_run * p.scale + __logf(l_tot);
    }
}

hipError_t launch_attn_bf16(const AttnParams &p, int32_t D, bool partial, hipStream_t stream)
{
    // heads that share a KV head are scheduled next to each other when the groups are uniform
    int32_t G = p.n_q_heads / p.n_kv_heads;
    bool uniform = true;
    for (int32_t i = 0; i < p.n_q_heads; ++i)
        if (p.heads.kv_of_q[p.heads.head_order[i]] != i / G) uniform = false;
    int32_t heads_inner = uniform ? G : p.n_q_heads;
    int32_t n_logical = p.n_items * p.n_q_heads;
    dim3 grid((n_logical + 7) / 8 * 8), block(256);
    if (D == 128) {
        if (partial) hipLaunchKernelGGL((attn_bf16_kernel<128, true>), grid, block, 0, stream, p, n_logical, heads_inner);
        else hipLaunchKernelGGL((attn_bf16_kernel<128, false>), grid, block, 0, stream, p, n_logical, heads_inner);
    } else {
        if (partial) hipLaunchKernelGGL((attn_bf16_kernel<64, true>), grid, block, 0, stream, p, n_logical, heads_inner);
        else hipLaunchKernelGGL((attn_bf16_kernel<64, false>), grid, block, 0, stream, p, n_logical, heads_inner);
    }
    return hipGetLastError();
}

}  // namespace pevlm
