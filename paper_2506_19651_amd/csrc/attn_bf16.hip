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

// 16-byte-per-lane load from global memory straight into LDS (no register staging).  The LDS
// destination of lane i is lds_addr + 16 i; lds_addr must be wavefront-uniform.  Issued through
// inline assembly so that the tile being consumed can be read while the next one is in flight: the
// wait for completion is the explicit vmcnt(0) at the top of the tile loop.
__device__ __forceinline__ void load_lds_16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n" ::"s"(lds_addr), "v"(gptr) : "memory");
}

__device__ __forceinline__ float max3f(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Same, with a wavefront-uniform 64-bit base address and a per-lane 32-bit byte offset.
__device__ __forceinline__ void load_lds_16_base(const void *sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

// Marks a pointer that is the same in every lane as wavefront-uniform (scalar registers).
template <typename T>
__device__ __forceinline__ const T *uniform_ptr(const T *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const T *)(((uint64_t)hi << 32) | lo);
}

template <int D>
struct TileCfg {
    static constexpr int KT = kKeyTile;        // keys per staged tile
    static constexpr int ROWB = D * 2;         // bytes per K/V row
    static constexpr int CH = D / 8;           // 16-byte chunks per row
    static constexpr int NLD = KT * CH / 256;  // 16-byte loads each wavefront issues per tensor per tile
    static constexpr int KSTEPS = D / 16;      // MFMA k-steps of Q K^T
    static constexpr int DBLK = D / 32;        // 32-wide blocks of head_dim in O^T
    static constexpr int VSW = CH / 4 - 1;     // V swizzle mask (64-byte granules per row - 1)
    static constexpr int TILEB = KT * ROWB;    // bytes of one staged K (or V) tile
    static constexpr int RPI = 1024 / ROWB;    // rows one wavefront-wide 16-byte-per-lane load covers
};

// One 64-key tile for one wavefront: S^T = K Q^T, online softmax, O^T += V^T P^T.
// masked = false: all 64 keys are visible to all 32 rows of the wave (the common case).
// masked = true : the tile touches the diagonal or the end of the key range; nkc (1 or 2) 32-key
//                 chunks are needed, entries are masked by key < kend and (causal) key <= row.
// Kept as ONE inlined instance with wavefront-uniform flags: two specialised copies would meet at
// a join that has to reconcile the 64 accumulator registers of O^T.
template <int D>
__device__ __forceinline__ void process_tile(const uint8_t *tk, const uint8_t *tv, const bf16x8 (&qf)[D / 16],
                                             f32x16 (&o)[D / 32], float &m_run, float &l_run, float c_log2,
                                             bool masked, int32_t nkc, int32_t k0, int32_t kend, bool causal,
                                             int32_t my_row, int32_t lane)
{
    using C = TileCfg<D>;
    const int32_t l32 = lane & 31, g32 = lane >> 5;
    // per-lane LDS offsets (the XOR swizzles depend on the lane only)
    const int32_t k_row_off = l32 * C::ROWB;
    const int32_t k_swz = l32 & (C::CH - 1);
    const int32_t v_row_off = (g32 * 4 + ((lane & 15) >> 2)) * C::ROWB + (lane & 1) * 8;
    const int32_t v_ch_lo = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    const int32_t v_swz = (lane >> 2) & C::VSW;

    f32x16 s[2];
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kc][i] = 0.f;

    // ---- S^T = K Q^T: A fragments (16 bytes per lane) are fetched one chunk ahead of the MFMAs ----
    // The two 32-key chunks form two independent accumulation chains that are issued alternately.
    bf16x8 a0[C::KSTEPS], a1[C::KSTEPS];
    constexpr int HK = C::KSTEPS / 2;
#pragma unroll
    for (int kk = 0; kk < HK; ++kk) {
        a0[kk] = *reinterpret_cast<const bf16x8 *>(tk + k_row_off + (((kk * 2 + g32) ^ k_swz) << 4));
        a1[kk] = *reinterpret_cast<const bf16x8 *>(tk + 32 * C::ROWB + k_row_off + (((kk * 2 + g32) ^ k_swz) << 4));
    }
    __builtin_amdgcn_sched_barrier(0);
    if (nkc > 1) {
#pragma unroll
        for (int kk = 0; kk < HK; ++kk) {
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], s[0], 0, 0, 0);
            a0[kk + HK] = *reinterpret_cast<const bf16x8 *>(tk + k_row_off + ((((kk + HK) * 2 + g32) ^ k_swz) << 4));
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[kk], qf[kk], s[1], 0, 0, 0);
            a1[kk + HK] = *reinterpret_cast<const bf16x8 *>(tk + 32 * C::ROWB + k_row_off + ((((kk + HK) * 2 + g32) ^ k_swz) << 4));
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = HK; kk < C::KSTEPS; ++kk) {
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[kk], qf[kk], s[1], 0, 0, 0);
        }
    } else {
#pragma unroll
        for (int kk = 0; kk < HK; ++kk) {
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], s[0], 0, 0, 0);
            a0[kk + HK] = *reinterpret_cast<const bf16x8 *>(tk + k_row_off + ((((kk + HK) * 2 + g32) ^ k_swz) << 4));
        }
#pragma unroll
        for (int kk = HK; kk < C::KSTEPS; ++kk) s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], s[0], 0, 0, 0);
    }

    // ---- V^T fragments of the first 16 keys: in flight during the softmax ----
    bf16x8 va[C::DBLK];
#define PEVLM_READ_V(dst, ks)                                                                                   \
    _Pragma("unroll") for (int b = 0; b < C::DBLK; ++b) {                                                       \
        _Pragma("unroll") for (int tt = 0; tt < 2; ++tt) {                                                      \
            const uint8_t *ptr = tv + ((ks) * 16 + tt * 8) * C::ROWB + v_row_off + (((b ^ v_swz) * 4 + v_ch_lo) << 4); \
            const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ptr));                       \
            const bf16x4 rb = __builtin_bit_cast(bf16x4, r);                                                    \
            dst[b][tt * 4 + 0] = rb[0]; dst[b][tt * 4 + 1] = rb[1];                                             \
            dst[b][tt * 4 + 2] = rb[2]; dst[b][tt * 4 + 3] = rb[3];                                             \
        }                                                                                                       \
    }
    PEVLM_READ_V(va, 0);

    // ---- mask ----
    if (masked) {
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int32_t key = k0 + kc * 32 + (i >> 2) * 8 + g32 * 4 + (i & 3);
                const bool ok = kc < nkc && key < kend && (!causal || key <= my_row);
                s[kc][i] = ok ? s[kc][i] : -INFINITY;
            }
    }
    // ---- online softmax: a lane holds 32 keys of its own query; its partner lane ^ 32 the others.
    // The reference maximum m_run is only moved when some row's maximum grew by more than
    // kRescaleStep (log2 units): weights are then at most 2^kRescaleStep, which fp32 sums and bf16
    // weights carry without loss, and the 64 accumulator multiplies are skipped on almost every
    // tile.  The result is unchanged in exact arithmetic: sum and values share one reference.
    float mx = max3f(s[0][0], s[0][1], s[0][2]);
#pragma unroll
    for (int i = 3; i < 31; i += 2) mx = max3f(mx, s[i >> 4][i & 15], s[(i + 1) >> 4][(i + 1) & 15]);
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        const auto sl = __builtin_amdgcn_permlane32_swap(__float_as_uint(s[1][15]), __float_as_uint(s[1][15]), false, false);
        mx = max3f(__uint_as_float(sw[0]), __uint_as_float(sw[1]), __uint_as_float(sl[0]));
        mx = max3f(mx, __uint_as_float(sl[1]), mx);
    }
    constexpr float kRescaleStep = 8.f;
    if (__any((mx - m_run) * c_log2 > kRescaleStep || m_run == -INFINITY)) {
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c_log2);  // m_run = -inf gives 0
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int b = 0; b < C::DBLK; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
    }
    const float mc = (m_run == -INFINITY) ? 0.f : m_run * c_log2;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float e = __builtin_amdgcn_exp2f(s[kc][i] * c_log2 - mc);
            psum += e;
            pf[kc * 2 + (i >> 3)][i & 7] = (__bf16)e;
        }
    l_run += psum;

    // ---- O^T += V^T P^T, V^T fragments one k-step ahead ----
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 vb[C::DBLK];
    const int32_t nks = nkc * 2;
#pragma unroll
    for (int ks = 0; ks < 4; ks += 2) {
        if (ks >= nks) break;
        PEVLM_READ_V(vb, ks + 1);
#pragma unroll
        for (int b = 0; b < C::DBLK; ++b) o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[b], pf[ks], o[b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (ks + 2 < 4 && ks + 2 < nks) PEVLM_READ_V(va, ks + 2);
#pragma unroll
        for (int b = 0; b < C::DBLK; ++b) o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[b], pf[ks + 1], o[b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
#undef PEVLM_READ_V
}

template <int D, bool PARTIAL>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnParams p, int32_t n_logical, int32_t heads_inner)
{
    using C = TileCfg<D>;
    constexpr int KT = C::KT, ROWB = C::ROWB, CH = C::CH, NLD = C::NLD, KSTEPS = C::KSTEPS, DBLK = C::DBLK;
    constexpr int VSW = C::VSW, TILEB = C::TILEB, RPI = C::RPI;
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

    const int32_t tid = threadIdx.x, lane = tid & 63;
    const int32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int32_t l32 = lane & 31, g32 = lane >> 5;
    const uint16_t *Q = (const uint16_t *)p.q, *K = (const uint16_t *)p.k, *V = (const uint16_t *)p.v;

    // ---- this lane's query row, Q fragments (B operand of S^T = K Q^T) stay in registers ----
    const int32_t row_in_tile = wave * 32 + l32;
    const bool row_valid = row_in_tile < it.q_rows;
    const int32_t my_row = it.q_start + (row_valid ? row_in_tile : it.q_rows - 1);
    const bool wave_active = wave * 32 < it.q_rows;
    const int32_t wr_lo = it.q_start + wave * 32;
    const int32_t wr_hi = it.q_start + ((wave * 32 + 31 < it.q_rows) ? wave * 32 + 31 : it.q_rows - 1);
    const uint32_t lds_k_addr = (uint32_t)(size_t)LDS_PTR(void, lds_k);
    const uint32_t lds_v_addr = (uint32_t)(size_t)LDS_PTR(void, lds_v);
    // Q rows of the wave are fetched with whole-row (coalesced) direct-to-LDS loads into a
    // wave-private slice of LDS stage 1 (unused until the first tile is being consumed), then read
    // back as MFMA B fragments.  Same 16-byte-chunk XOR swizzle as the K tile.
    constexpr int WSLICE = 32 * ROWB;  // bytes of 32 rows
    uint8_t *const wave_slice = (wave < 2 ? lds_k : lds_v) + TILEB + (wave & 1) * WSLICE;
    const uint32_t wave_slice_addr = (wave < 2 ? lds_k_addr : lds_v_addr) + TILEB + (wave & 1) * WSLICE;
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int j = 0; j < WSLICE / 1024; ++j) {
        const int32_t rl = j * RPI + lane / CH, cpos = lane % CH;
        int32_t r = wave * 32 + rl;
        r = r < it.q_rows ? r : it.q_rows - 1;
        load_lds_16(Q + ((int64_t)(it.q_start + r) * Hq + h) * D + ((cpos ^ (rl & (CH - 1))) << 3),
                    wave_slice_addr + j * 1024);
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

    // ---- K/V tiles go straight from global memory into LDS (16 bytes per lane): a wavefront
    // instruction fills 1 KB of contiguous LDS, i.e. RPI whole rows; the XOR swizzle is applied by
    // choosing which 16-byte chunk of the row each lane fetches.  Two LDS stages: tile t+1 streams
    // in while tile t is consumed.  Rows past the key range repeat its last key (their scores are
    // masked, their values stay finite).
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
    // Per-lane byte offsets of the NLD loads inside a tile are fixed (row within the tile, swizzled
    // chunk); a tile that lies wholly inside its key range only needs a new uniform base address.
    uint32_t koff[NLD], voff[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int32_t row = (j * 4 + wave) * RPI + lane / CH, cpos = lane % CH;
        koff[j] = (uint32_t)((row * Hkv * D + ((cpos ^ (row & (CH - 1))) << 3)) * 2);
        voff[j] = (uint32_t)((row * Hkv * D + ((cpos ^ ((row & VSW) << 2)) << 3)) * 2);
    }
#define PEVLM_ISSUE_TILE(t, stage)                                                                   \
    do {                                                                                             \
        int32_t pk0, pkend;                                                                          \
        bool pcausal;                                                                                \
        PEVLM_TILE_RANGE(t, pk0, pkend, pcausal);                                                    \
        (void)pcausal;                                                                               \
        if (pk0 + KT <= pkend) {                                                                     \
            const uint16_t *kb = uniform_ptr(K + ((int64_t)pk0 * Hkv + g) * D);                      \
            const uint16_t *vb = uniform_ptr(V + ((int64_t)pk0 * Hkv + g) * D);                      \
            _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                        \
                const uint32_t dst = (uint32_t)((stage) * TILEB + (j * 4 + wave) * RPI * ROWB);      \
                load_lds_16_base(kb, koff[j], lds_k_addr + dst);                                     \
                load_lds_16_base(vb, voff[j], lds_v_addr + dst);                                     \
            }                                                                                        \
        } else {                                                                                     \
            _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                        \
                const int32_t rbase = (j * 4 + wave) * RPI;                                          \
                const int32_t row = rbase + lane / CH, cpos = lane % CH;                             \
                int32_t key = pk0 + row;                                                             \
                key = key < pkend ? key : pkend - 1;                                                 \
                const int64_t roff = ((int64_t)key * Hkv + g) * D;                                   \
                const uint32_t dst = (uint32_t)((stage) * TILEB + rbase * ROWB);                     \
                load_lds_16(K + roff + ((cpos ^ (row & (CH - 1))) << 3), lds_k_addr + dst);          \
                load_lds_16(V + roff + ((cpos ^ ((row & VSW) << 2)) << 3), lds_v_addr + dst);        \
            }                                                                                        \
        }                                                                                            \
    } while (0)

    if (n_tiles > 0) {
        PEVLM_ISSUE_TILE(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * NLD));  // all but the tile-0 loads: Q has landed
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8 *>(wave_slice + l32 * ROWB + (((kk * 2 + g32) ^ (l32 & (CH - 1))) << 4));
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
        process_tile<D>(tk, tv, qf, o, m_run, l_run, c_log2, need_mask || nkc < 2, nkc, k0, kend, causal, my_row, lane);
    }

    // ---- epilogue ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (PARTIAL) {
        if (!row_valid) return;
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
        // O^T fragments -> wave-private LDS slice of the stage the last tile did not use (row-major
        // bf16, swizzled), then whole-row 16-byte stores.
        const float inv = 1.f / l_tot;
        const int32_t free_stage = n_tiles & 1;
        uint8_t *const oslice = (wave < 2 ? lds_k : lds_v) + free_stage * TILEB + (wave & 1) * WSLICE;
#pragma unroll
        for (int b = 0; b < DBLK; ++b)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                bf16x4 v4;
                v4[0] = (__bf16)(o[b][i4 * 4] * inv);
                v4[1] = (__bf16)(o[b][i4 * 4 + 1] * inv);
                v4[2] = (__bf16)(o[b][i4 * 4 + 2] * inv);
                v4[3] = (__bf16)(o[b][i4 * 4 + 3] * inv);
                *reinterpret_cast<bf16x4 *>(oslice + l32 * ROWB + (((b * 4 + i4) ^ (l32 & (CH - 1))) << 4) + g32 * 8) = v4;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint16_t *const obase = (uint16_t *)p.out;
#pragma unroll
        for (int j = 0; j < WSLICE / 1024; ++j) {
            const int32_t rl = j * RPI + lane / CH, cpos = lane % CH;
            const uint4 val = *reinterpret_cast<const uint4 *>(oslice + rl * ROWB + ((cpos ^ (rl & (CH - 1))) << 4));
            if (wave * 32 + rl < it.q_rows)
                *reinterpret_cast<uint4 *>(obase + ((int64_t)(it.q_start + wave * 32 + rl) * Hq + h) * D + cpos * 8) = val;
        }
        if (p.lse && g32 == 0 && row_valid) p.lse[(int64_t)my_row * Hq + h] = m_run * p.scale + __logf(l_tot);
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
