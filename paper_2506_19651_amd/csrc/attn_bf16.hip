// bf16 flash-style attention kernel for gfx950 (CDNA4): bf16 MFMA for Q K^T and P V with fp32
// accumulation, fp32 online softmax.  Serves the block-parallel prefill (sink rows, Eq. 3, and
// context-block rows, Eq. 4: a work item names a tile of query rows plus the sink key range and the
// own-block key range up to the diagonal, nothing else) and, in partial mode, the split-KV question
// attention (Eq. 5).
//
// Tiling.  A workgroup of 4 wavefronts owns one work item (<= 128 query rows of one head); wave w
// owns rows 32w..32w+31; two workgroups share a compute unit (two wavefronts per SIMD).  Keys are
// staged 64 at a time in LDS (K and V tiles, XOR-swizzled 16-byte chunks, direct global->LDS loads,
// two stages each).  Scores are formed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: in
// the accumulator layout a lane then holds 16 keys of ONE query (column = lane % 32), so the softmax
// row reduction is in-lane max3/add chains and a single exchange with lane ^ 32.  The same
// registers, converted to bf16, are directly the B operand of O^T += V^T P^T; V^T fragments come
// from LDS through the transposing read ds_read_b64_tr_b16.
//
// Schedule inside a wavefront (software pipeline over key tiles): the value MFMAs of tile t-1 are
// issued interleaved with the vector-ALU work that turns the scores of tile t into weights, so the
// matrix cores and the vector ALU of a SIMD overlap within one instruction stream as well as
// across the two resident wavefronts; the wavefront's share of the next K tile and of the current V
// tile is requested piecewise between those MFMAs.
//
// Softmax.  Weights of a tile are formed against the reference maximum the row already has; the
// row maximum is only computed (and the reference raised, accumulators rescaled) when a lane's sum
// of weights shows that one of them may have reached 2^8, or on the row's first tile.
//
// Variants: PARTIAL writes un-normalised fp32 partials (question attention, merged afterwards);
// ROPEQ rotates the query rows in registers from a (cos, sin) table instead of expecting rotated
// queries; items of <= 64 rows are taken for 2 or 4 heads of a KV group by one workgroup.
#include "attn_bf16_tile.h"
#include "rope_math.h"

namespace pevlm {

// ROPEQ: q holds un-rotated queries; each wavefront rotates its 32 rows once, right after loading
// them, from the (cos, sin) table of the call (the sequential positions of Sec. "Position Encoding").
// One work item for one head (or several heads of a KV group, see below): `logical` indexes
// (KV head group, item, head in group).
template <int D, bool PARTIAL, bool ROPEQ>
__device__ __forceinline__ void attn_item(const AttnParams &p, int32_t logical, int32_t heads_inner, int32_t pack_heads,
                                          int32_t identity_map, uint8_t *lds_k, uint8_t *lds_v)
{
    using C = TileCfg<D>;
    constexpr int KT = C::KT, ROWB = C::ROWB, CH = C::CH, NLD = C::NLD, KSTEPS = C::KSTEPS, DBLK = C::DBLK;
    constexpr int VSW = C::VSW, TILEB = C::TILEB, RPI = C::RPI;
    const int32_t inner = logical % heads_inner;
    const int32_t rest = logical / heads_inner;
    // last item first: within a context block the later tiles are the longer ones, and a launch that
    // ends on short items has a shorter tail
    const int32_t item_idx = p.n_items - 1 - rest % p.n_items;
    const int32_t hs = (rest / p.n_items) * heads_inner + inner;
    const pevlm_work_item it = p.items[item_idx];
    // With the default head map (query head h on KV head h / G, schedule order = head order) both
    // indices are plain arithmetic; the tables live in kernel-argument memory and looking them up
    // costs two dependent memory round trips before the first query row can be requested.
    const int32_t g = identity_map ? rest / p.n_items
                                   : __builtin_amdgcn_readfirstlane((int32_t)p.heads.kv_of_q[p.heads.head_order[hs]]);  // workgroup-uniform
    const int32_t Hq = p.n_q_heads, Hkv = p.n_kv_heads;

    const int32_t tid = threadIdx.x, lane = tid & 63;
    const int32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Short items (<= 64 rows: small question blocks, tails of context blocks) would leave
    // wavefronts idle.  When the query heads of a KV group are scheduled next to each other, such an
    // item is taken for 2 or 4 heads of the group at once (they need the same K/V tiles): wave w
    // then owns row group w % wph of head slot inner + w / wph, and the workgroups of the other head
    // slots leave at once.
    const int32_t groups32 = (it.q_rows + 31) >> 5;
    const int32_t wph = groups32 <= 1 ? 1 : (groups32 <= 2 ? 2 : 4);  // wavefronts per head
    const int32_t hpw = pack_heads ? 4 / wph : 1;                     // heads per workgroup
    if (hpw > 1 && (inner % hpw) != 0) return;
    const int32_t slot = hpw > 1 ? inner + wave / wph : inner;
    const bool head_ok = slot < heads_inner;
    const int32_t h = identity_map ? hs - inner + (head_ok ? slot : inner)
                                   : __builtin_amdgcn_readfirstlane((int32_t)p.heads.head_order[hs - inner + (head_ok ? slot : inner)]);  // wavefront-uniform
    const int32_t rg = hpw > 1 ? wave % wph : wave;  // this wave's group of 32 rows
    const int32_t l32 = lane & 31, g32 = lane >> 5;
    const uint16_t *Q = (const uint16_t *)p.q, *K = (const uint16_t *)p.k, *V = (const uint16_t *)p.v;

    LaneOff L;
    L.g32 = g32;
    L.k_row_off = l32 * ROWB;
    L.k_swz = l32 & (CH - 1);
    L.v_row_off = (g32 * 4 + ((lane & 15) >> 2)) * ROWB + (lane & 1) * 8;
    L.v_ch_lo = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    L.v_swz = (lane >> 2) & VSW;

    // ---- this lane's query row ----
    const int32_t row_in_tile = rg * 32 + l32;
    const bool row_valid = head_ok && row_in_tile < it.q_rows;
    const int32_t my_row = it.q_start + (row_in_tile < it.q_rows ? row_in_tile : it.q_rows - 1);
    const bool wave_active = head_ok && rg * 32 < it.q_rows;
    const int32_t wr_lo = it.q_start + rg * 32;
    const int32_t wr_hi = it.q_start + ((rg * 32 + 31 < it.q_rows) ? rg * 32 + 31 : it.q_rows - 1);

    // (cos, sin) of this lane's row for the fused query rotation: fetched first, so that the loads
    // are in flight together with the Q rows
    f32x4 rope_cs[ROPEQ ? KSTEPS / 2 : 1][4];
    if (ROPEQ) {
        int64_t entry = my_row;
        if (p.rope_compact_rows > 0)
            entry = it.reserved % p.rope_compact_rows + (row_in_tile < it.q_rows ? row_in_tile : it.q_rows - 1);
        const f32x4 *tab = reinterpret_cast<const f32x4 *>(p.rope_tab + entry * D) + g32 * 4;
#pragma unroll
        for (int kk = 0; kk < KSTEPS / 2; ++kk)
#pragma unroll
            for (int j = 0; j < 4; ++j) rope_cs[kk][j] = tab[kk * 8 + j];
    }
    const uint32_t lds_k_addr = (uint32_t)(size_t)LDS_PTR(void, lds_k);
    const uint32_t lds_v_addr = (uint32_t)(size_t)LDS_PTR(void, lds_v);
    // Q rows of the wave are fetched with whole-row (coalesced) direct-to-LDS loads into a
    // wave-private slice of LDS stage 1 (unused until the first tile is being consumed), then read
    // back as MFMA B fragments.  Same 16-byte-chunk XOR swizzle as the K tile.
    constexpr int WSLICE = 32 * ROWB;  // bytes of 32 rows
    uint8_t *const wave_slice = (wave < 2 ? lds_k : lds_v) + TILEB + (wave & 1) * WSLICE;
    const uint32_t wave_slice_addr = (wave < 2 ? lds_k_addr : lds_v_addr) + TILEB + (wave & 1) * WSLICE;

    const int32_t n_full_tiles = (it.full_len + KT - 1) / KT;
    const int32_t n_diag_tiles = (it.diag_len + KT - 1) / KT;
    const int32_t n_tiles = n_full_tiles + n_diag_tiles;
    // tiles this wave computes: all fully visible ones, and the causal ones that start at or before
    // its last row (the rest is masked for every row of the wave)
    int32_t n_w = 0;
    if (wave_active) {
        int32_t nd = wr_hi >= it.diag_start ? (wr_hi - it.diag_start) / KT + 1 : 0;
        n_w = n_full_tiles + (nd < n_diag_tiles ? nd : n_diag_tiles);
    }

    // ---- K/V tiles go straight from global memory into LDS (16 bytes per lane): a wavefront
    // instruction fills 1 KB of contiguous LDS, i.e. RPI whole rows; the XOR swizzle is applied by
    // choosing which 16-byte chunk of the row each lane fetches.  Two LDS stages per tensor: K(t+1)
    // and V(t) stream in while tile t's scores and tile t-1's values are computed.  Rows past the
    // key range repeat its last key (their scores are masked, their values stay finite).
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
#define PEVLM_ISSUE(T, toff, swz_expr, lds_base_addr, t, stage)                                       \
    do {                                                                                              \
        int32_t pk0, pkend;                                                                           \
        bool pcausal;                                                                                 \
        PEVLM_TILE_RANGE(t, pk0, pkend, pcausal);                                                     \
        (void)pcausal;                                                                                \
        if (pk0 + KT <= pkend) {                                                                      \
            const uint16_t *tb = uniform_ptr(T + ((int64_t)pk0 * Hkv + g) * D);                       \
            _Pragma("unroll") for (int j = 0; j < NLD; ++j)                                           \
                load_lds_16_base(tb, toff[j], lds_base_addr + (stage) * TILEB + (j * 4 + wave) * RPI * ROWB); \
        } else {                                                                                      \
            _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                         \
                const int32_t rbase = (j * 4 + wave) * RPI;                                           \
                const int32_t row = rbase + lane / CH, cpos = lane % CH;                              \
                int32_t key = pk0 + row;                                                              \
                key = key < pkend ? key : pkend - 1;                                                  \
                load_lds_16(T + ((int64_t)key * Hkv + g) * D + ((cpos ^ (swz_expr)) << 3),            \
                            lds_base_addr + (stage) * TILEB + rbase * ROWB);                          \
            }                                                                                         \
        }                                                                                             \
    } while (0)
#define PEVLM_ISSUE_K(t) PEVLM_ISSUE(K, koff, (row & (CH - 1)), lds_k_addr, t, (t) & 1)
#define PEVLM_ISSUE_V(t) PEVLM_ISSUE(V, voff, ((row & VSW) << 2), lds_v_addr, t, (t) & 1)
    // top of tile t: K(t) and V(t-1) have landed for everybody, everybody is done with K(t-1) and
    // V(t-2); then K(t+1) and V(t) are put in flight
#define PEVLM_TOP(t)                                                   \
    do {                                                               \
        __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0) */             \
        __syncthreads();                                               \
        if ((t) + 1 < n_tiles) PEVLM_ISSUE_K((t) + 1);                 \
        PEVLM_ISSUE_V(t);                                              \
    } while (0)

    // Inside the pipelined loop the loads of a tile are not issued in one burst behind the barrier
    // (the wavefront would sit in the memory-instruction queue while its MFMAs wait) but one at a
    // time between MFMAs.  PEVLM_SET_LOADS prepares them: base address of tile tl, LDS destination in
    // `stage`, and, for a tile that runs past the end of its key range, per-lane offsets clamped to
    // the last valid key (put back to the plain ones on the next use).
#define PEVLM_SET_LOADS(ld, T, toff, modified, swz_expr, lds_base_addr, tl, stage)                      \
    do {                                                                                              \
        int32_t pk0, pkend;                                                                           \
        bool pcausal;                                                                                 \
        PEVLM_TILE_RANGE(tl, pk0, pkend, pcausal);                                                    \
        (void)pcausal;                                                                                \
        const bool edge = pk0 + KT > pkend;                                                           \
        if (edge || modified) {                                                                       \
            const int32_t last = edge ? pkend - 1 - pk0 : KT - 1;                                     \
            _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                         \
                const int32_t row = (j * 4 + wave) * RPI + lane / CH, cpos = lane % CH;               \
                const int32_t key = row < last ? row : last;                                          \
                toff[j] = (uint32_t)((key * Hkv * D + ((cpos ^ (swz_expr)) << 3)) * 2);               \
            }                                                                                         \
            modified = edge;                                                                          \
        }                                                                                             \
        ld.base = uniform_ptr(T + ((int64_t)pk0 * Hkv + g) * D);                                      \
        ld.lds = lds_base_addr + (stage) * TILEB + wave * 1024;                                       \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) ld.off[j] = toff[j];                          \
    } while (0)

    // First the K and V tiles of tile 0 (stage 0; they usually come from L2), then the query rows
    // (first touch: from HBM), so that all three are in flight together.
    if (n_tiles > 0) {
        PEVLM_ISSUE_K(0);
        PEVLM_ISSUE_V(0);
    }
#pragma unroll
    for (int j = 0; j < WSLICE / 1024; ++j) {
        const int32_t rl = j * RPI + lane / CH, cpos = lane % CH;
        int32_t r = rg * 32 + rl;
        r = r < it.q_rows ? r : it.q_rows - 1;
        load_lds_16(Q + ((int64_t)(it.q_start + r) * Hq + h) * D + ((cpos ^ (rl & (CH - 1))) << 3),
                    wave_slice_addr + j * 1024);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");
    const float c_log2 = p.scale * 1.4426950408889634f;
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8 *>(wave_slice + l32 * ROWB + (((kk * 2 + g32) ^ (l32 & (CH - 1))) << 4));
    if (ROPEQ) {
        // this lane holds dims kk*16 + g32*8 + e of its row: pair index i < D/2 in qf[kk], its partner
        // i + D/2 in qf[kk + KSTEPS/2]
#pragma unroll
        for (int kk = 0; kk < KSTEPS / 2; ++kk) {
            const f32x4 *cs = rope_cs[kk];
            const u32x4 lo = __builtin_bit_cast(u32x4, qf[kk]), hi = __builtin_bit_cast(u32x4, qf[kk + KSTEPS / 2]);
            u32x4 rl, rh;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float a0 = __uint_as_float(lo[w] << 16), a1 = __uint_as_float(lo[w] & 0xffff0000u);
                const float b0 = __uint_as_float(hi[w] << 16), b1 = __uint_as_float(hi[w] & 0xffff0000u);
                float r0, r1, t0, t1;
                rope_rotate(a0, b0, cs[w][0], cs[w][1], r0, t0);
                rope_rotate(a1, b1, cs[w][2], cs[w][3], r1, t1);
                rl[w] = rope_pack_bf16(r0, r1);
                rh[w] = rope_pack_bf16(t0, t1);
            }
            qf[kk] = __builtin_bit_cast(bf16x8, rl);
            qf[kk + KSTEPS / 2] = __builtin_bit_cast(bf16x8, rh);
        }
    }

    // m_ref: reference maximum of this lane's row in base-2 units, c_log2 * score (-inf: none yet)
    float m_ref = -INFINITY, l_run = 0.f;
#define PEVLM_MREF ((m_ref == -INFINITY) ? 0.f : m_ref)
    f32x16 o[DBLK];
#pragma unroll
    for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[b][i] = 0.f;

    // scores of tile t -> s (masked where the tile touches the diagonal or the end of its range)
#define PEVLM_SCORES(t, LOADS)                                                            \
    do {                                                                                  \
        int32_t k0, kend;                                                                 \
        bool causal;                                                                      \
        PEVLM_TILE_RANGE(t, k0, kend, causal);                                            \
        qk_tile<D, LOADS>(lds_k + ((t) & 1) * TILEB, L, qf, s, ldk);                     \
        if ((k0 + KT > kend) || (causal && (k0 + KT - 1 > wr_lo)))                        \
            mask_tile(s, k0, kend, causal, my_row, g32);                                  \
    } while (0)
    // The weights of a tile are first formed against the reference maximum the row already has.
    // Only if a lane's weights may have reached 2^kRescaleStep (or a row has no reference yet) is the
    // row maximum of the tile computed, the reference raised, o and l scaled down and the tile's weights formed
    // again: weights stay below 2^kRescaleStep, which fp32 sums and bf16 weights carry without loss,
    // and on almost every tile the vector ALU only does exp2, convert and sum.
#define PEVLM_FIX_REFERENCE()                                                                         \
    do {                                                                                              \
        if (__any(sum_reached_step(psum) || m_ref == -INFINITY)) {                                    \
            const float mx = row_max(s) * c_log2;                                                     \
            const bool has = m_ref != -INFINITY;                                                      \
            const float m_new = fmaxf(m_ref, mx);                                                     \
            const float alpha = has ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.f;                    \
            m_ref = m_new;                                                                            \
            psum = 0.f;                                                                               \
            weights(s, c_log2, PEVLM_MREF, psum, pf_new);                                             \
            if (__any(has)) { /* rows without a reference have o = l = 0 */                          \
                l_run *= alpha;                                                                       \
                _Pragma("unroll") for (int b = 0; b < DBLK; ++b)                                      \
                    _Pragma("unroll") for (int i = 0; i < 16; ++i) o[b][i] *= alpha;                  \
            }                                                                                         \
        }                                                                                             \
    } while (0)

    f32x16 s[2];
    u32x4 pf_prev[4], pf_new[4];
    float psum;
    TileLoads<NLD> ldk, ldv;
    bool k_mod = false, v_mod = false;
    if (n_tiles > 0) {  // top of tile 0 for every wavefront
        __syncthreads();  // K(0), V(0) of every wavefront have landed; the query slices in stage 1 have been read
        if (1 < n_tiles) PEVLM_ISSUE_K(1);
    }
    if (n_w > 0) {
        PEVLM_SCORES(0, false);
        psum = 0.f;  // no row has a reference yet: the first tile always takes the exact path
        PEVLM_FIX_REFERENCE();
        l_run += psum;
#pragma unroll
        for (int j = 0; j < 4; ++j) pf_prev[j] = pf_new[j];
        for (int32_t t = 1; t < n_w; ++t) {
            // top of tile t as in PEVLM_TOP, but K(t+1) and V(t) are fetched piecewise between the
            // MFMAs below; after the last tile the K loads repeat that tile into the stage nobody
            // reads any more, which keeps the loop body free of branches
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            const int32_t tk = t + 1 < n_tiles ? t + 1 : n_tiles - 1;
            PEVLM_SET_LOADS(ldk, K, koff, k_mod, (row & (CH - 1)), lds_k_addr, tk, (t + 1) & 1);
            PEVLM_SET_LOADS(ldv, V, voff, v_mod, ((row & VSW) << 2), lds_v_addr, t, t & 1);
            PEVLM_SCORES(t, true);
            // values of tile t-1 (matrix cores) under the weights of tile t (vector ALU)
            psum = 0.f;
            pv_prev_weights_cur<D>(lds_v + ((t - 1) & 1) * TILEB, L, pf_prev, o, s, c_log2, PEVLM_MREF, psum, pf_new, ldv);
            PEVLM_FIX_REFERENCE();
            l_run += psum;
#pragma unroll
            for (int j = 0; j < 4; ++j) pf_prev[j] = pf_new[j];
        }
    }
    // the burst loads below use the plain per-lane offsets
    if (k_mod) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int32_t row = (j * 4 + wave) * RPI + lane / CH, cpos = lane % CH;
            koff[j] = (uint32_t)((row * Hkv * D + ((cpos ^ (row & (CH - 1))) << 3)) * 2);
        }
    }
    if (v_mod) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int32_t row = (j * 4 + wave) * RPI + lane / CH, cpos = lane % CH;
            voff[j] = (uint32_t)((row * Hkv * D + ((cpos ^ ((row & VSW) << 2)) << 3)) * 2);
        }
    }
    // Every wavefront passes the top of all n_tiles tiles and one final barrier.  The values of the
    // last tile a wave computed are added once their V tile is known to be in LDS.
    int32_t t_rest = n_w > 0 ? n_w : (n_tiles > 0 ? 1 : 0);  // the top of tile 0 is behind every wavefront
    bool synced = false;
    if (n_w > 0 && n_w < n_tiles) {
        PEVLM_TOP(n_w);
        t_rest = n_w + 1;
    } else if (n_w == n_tiles) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        synced = true;
    }
    if (n_w > 0) pv_tile<D>(lds_v + ((n_w - 1) & 1) * TILEB, L, pf_prev, o);
    for (int32_t t = t_rest; t < n_tiles; ++t) PEVLM_TOP(t);
    if (!synced) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
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
            p.part_ml[(slot * Hq + h) * 2] = m_ref / c_log2;  // back to raw score units (-inf stays)
            p.part_ml[(slot * Hq + h) * 2 + 1] = l_tot;
        }
    } else {
        // O^T fragments -> wave-private LDS slice (row-major bf16, swizzled), then whole-row 16-byte
        // stores.  The slice lies in the stage the last tile does not use: a wavefront may still be
        // adding the values of the last tile out of the other stage.
        const float inv = 1.f / l_tot;
        uint8_t *const oslice = (wave < 2 ? lds_k : lds_v) + (n_tiles & 1) * TILEB + (wave & 1) * WSLICE;
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
            if (head_ok && rg * 32 + rl < it.q_rows)
                *reinterpret_cast<uint4 *>(obase + ((int64_t)(it.q_start + rg * 32 + rl) * Hq + h) * D + cpos * 8) = val;
        }
        if (p.lse && g32 == 0 && row_valid) p.lse[(int64_t)my_row * Hq + h] = (m_ref + __log2f(l_tot)) * 0.69314718056f;
    }
}

// One workgroup per logical id.  Consecutive workgroup ids land on different XCDs (8 of them, each
// with its own L2); every XCD gets one contiguous run of logical ids so that the heads of a GQA
// group working on the same context block share that XCD's L2.
template <int D, bool PARTIAL, bool ROPEQ>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnParams p, int32_t n_logical, int32_t heads_inner, int32_t pack_heads,
                                                           int32_t identity_map)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds_k[2 * TileCfg<D>::TILEB];
    __shared__ __attribute__((aligned(1024))) uint8_t lds_v[2 * TileCfg<D>::TILEB];
    const int32_t per_xcd = gridDim.x >> 3;
    const int32_t logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= n_logical) return;
    attn_item<D, PARTIAL, ROPEQ>(p, logical, heads_inner, pack_heads, identity_map, lds_k, lds_v);
}

hipError_t launch_attn_bf16(const AttnParams &p, int32_t D, bool partial, hipStream_t stream)
{
    // heads that share a KV head are scheduled next to each other when the groups are uniform
    int32_t G = p.n_q_heads / p.n_kv_heads;
    bool uniform = true;
    for (int32_t i = 0; i < p.n_q_heads; ++i)
        if (p.heads.kv_of_q[p.heads.head_order[i]] != i / G) uniform = false;
    int32_t heads_inner = uniform ? G : p.n_q_heads;
    int32_t identity = uniform ? 1 : 0;  // query head h on KV head h / G, scheduled in head order
    for (int32_t i = 0; i < p.n_q_heads; ++i)
        if (p.heads.head_order[i] != i || p.heads.kv_of_q[i] != i / G) identity = 0;
    int32_t pack = (uniform && G > 1) ? 1 : 0;  // short items are taken for several heads of a KV group at once
    int32_t n_logical = p.n_items * p.n_q_heads;
    dim3 grid((n_logical + 7) / 8 * 8), block(256);
#define PEVLM_ATTN_LAUNCH(DD, PP, RR) \
    hipLaunchKernelGGL((attn_bf16_kernel<DD, PP, RR>), grid, block, 0, stream, p, n_logical, heads_inner, pack, identity)
    const bool rope = p.rope_tab != nullptr;
    if (D == 128) {
        if (partial) { if (rope) PEVLM_ATTN_LAUNCH(128, true, true); else PEVLM_ATTN_LAUNCH(128, true, false); }
        else { if (rope) PEVLM_ATTN_LAUNCH(128, false, true); else PEVLM_ATTN_LAUNCH(128, false, false); }
    } else {
        if (partial) { if (rope) PEVLM_ATTN_LAUNCH(64, true, true); else PEVLM_ATTN_LAUNCH(64, true, false); }
        else { if (rope) PEVLM_ATTN_LAUNCH(64, false, true); else PEVLM_ATTN_LAUNCH(64, false, false); }
    }
#undef PEVLM_ATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace pevlm
