// Streaming block-prefill kernel for gfx950 (CDNA4): rows of the sink (Eq. 3) and of the context blocks
// (Eq. 4), bf16 MFMA with fp32 accumulation and fp32 online softmax -- the same tile arithmetic as the
// one-item-per-workgroup kernel (attn_bf16_tile.h), under another execution model.
//
// One workgroup of 8 wavefronts per compute unit stays resident and walks a list of stream items.  An
// item is 8 slots of <= 32 query rows of one region whose heads share a KV head (wavefront w takes slot
// w), so all 8 wavefronts consume the same key tiles: a K/V tile is staged once per 8 x 32 rows.  The
// tiles of consecutive items form ONE stream: K and V tiles travel through rings of three LDS stages,
// K two tiles and V one tile ahead of the arithmetic, across item boundaries, so a new item finds its
// first tiles already in LDS.  The query rows of the next item are fetched into a wavefront-private
// LDS slice while the current item is computed, and the output rows of an item leave through the
// same slice (transposed back to whole 256-byte rows) after the next item's queries have moved to
// registers.  What is left per item outside the steady-state loop: the last value tile, the output
// conversion, and the first tile's exact softmax.
//
// Waits.  Loads into LDS are asynchronous and complete in issue order per wavefront, so the top of a
// tile waits with a count: the loads issued during the previous tile (and a query prefetch issued
// within the last two tiles) may still be in flight.  Stores are counted by the same counter and may
// complete out of order with loads, therefore the allowance never includes stores: a wait may cover
// more than needed, never less.
#include "attn_bf16_tile.h"

namespace pevlm {

namespace {

__device__ __forceinline__ int32_t sgpr(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Field `idx` (in 32-bit words) of a stream item, read through the constant address space: the address
// is wavefront-uniform, so this is a scalar load that stays out of the vector-memory counter the
// asynchronous tile loads are waited on.  (The list was written by an earlier kernel and is never
// written here.)
enum { F_FULL_START = 0, F_FULL_LEN, F_DIAG_START, F_DIAG_LEN, F_KV_HEAD, F_N_FULL, F_N_TILES, F_SEQ, F_SLOT0 };
enum { S_Q_START = 0, S_Q_ROWS, S_HEAD, S_WORDS = 4 };
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;
__device__ __forceinline__ int32_t item_word(const pevlm_stream_item *it, int32_t idx)
{
    return sgpr(((const_i32_ptr)(uintptr_t)it)[idx]);
}
static_assert(sizeof(pevlm_stream_item) == (F_SLOT0 + 8 * S_WORDS) * 4, "stream item layout");

#define PEVLM_WAIT_VM(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")
// the same with a compile-time count
template <int N>
__device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The lane id as an opaque value: address arithmetic derived from it is redone where it is used (a
// handful of instructions per item) instead of being kept in registers across the tile loop.
__device__ __forceinline__ int32_t opaque(int32_t v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// ---- loads through a buffer descriptor (base address + byte count in scalar registers).  A lane's
// address is base + scalar offset + its own byte offset; an address at or beyond the byte count reads
// as zero instead of touching memory.  A key range (or a slot's query rows) gets a descriptor whose
// byte count ends with its last row, so rows past the end arrive as zeros: masked scores, zero values.
// Per tile only scalar registers change; the per-lane offsets are constants of the kernel.
typedef __attribute__((ext_vector_type(4))) int32_t i32x4;
__device__ __forceinline__ i32x4 make_rsrc(uint64_t base, uint32_t bytes)
{
    i32x4 r;
    r[0] = sgpr((int32_t)(uint32_t)base);
    r[1] = sgpr((int32_t)((uint32_t)(base >> 32) & 0xffffu));  // stride 0: raw buffer
    r[2] = sgpr((int32_t)bytes);
    r[3] = 0x00020000;
    return r;
}
// 16 bytes per lane straight into LDS at lds_addr + 16 * lane (lds_addr wavefront-uniform)
__device__ __forceinline__ void load_lds_16_buf(const i32x4 &rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds\n" ::"s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// the loads of one tensor for one tile step: piece j of the wavefront lies `sstep` bytes further in
// memory (32 or 64 rows) and PSTEP bytes further in LDS
template <int PSTEP>
struct BufTileLoads {
    i32x4 rsrc;
    uint32_t voff, soff, sstep, lds;
    __device__ __forceinline__ void issue(int j) const { load_lds_16_buf(rsrc, voff, soff + j * sstep, lds + j * PSTEP); }
};

// position of the load stream: tile t of the workgroup's item number ord, with the two key ranges of
// that item as (byte address of the first K row of the KV head, bytes up to the end of the range)
struct TileCursor {
    int32_t ord, t;
    int32_t n_full, n_tiles;
    uint64_t base_full, base_diag;
    uint32_t bytes_full, bytes_diag;
};

}  // namespace

template <int D>
__global__ __launch_bounds__(512, 2) void attn_bf16_stream_kernel(StreamParams p)
{
    using C = TileCfg<D>;
    constexpr int KT = C::KT, ROWB = C::ROWB, CH = C::CH, KSTEPS = C::KSTEPS, DBLK = C::DBLK;
    constexpr int VSW = C::VSW, TILEB = C::TILEB, RPI = C::RPI;
    constexpr int NW = 8;                         // wavefronts per workgroup
    constexpr int NL = KT * CH / (64 * NW);       // 16-byte loads a wavefront issues per tensor per tile
    constexpr int TL = 2 * NL;                    // ... per tile step (K and V)
    constexpr int PSTEP = NW * 1024;              // LDS distance between a wavefront's pieces of a tile
    constexpr int NST = 3;                        // LDS stages per tensor
    constexpr int WSLICE = 32 * ROWB;             // a wavefront's query / output slice
    constexpr int NQL = WSLICE / 1024;            // loads per query slice
    static_assert(NL >= 1 && NL <= 2 && (NW * RPI) % 16 == 0, "tile loads per wavefront");
    __shared__ __attribute__((aligned(1024))) uint8_t lds[2 * NST * TILEB + NW * WSLICE];

    // ---- the items of this workgroup: every XCD takes one contiguous eighth of the list (its L2 then
    // holds the K/V of the few regions its workgroups are in), its workgroups take items round robin
    const int32_t xcd = blockIdx.x & 7, wg_in_xcd = blockIdx.x >> 3, wgs_per_xcd = gridDim.x >> 3;
    const int32_t per_xcd = (p.n_items + 7) >> 3;
    const int32_t lo = xcd * per_xcd;
    const int32_t hi = lo + per_xcd < p.n_items ? lo + per_xcd : p.n_items;
    const int32_t first = lo + wg_in_xcd;
    if (first >= hi) return;
    const int32_t n_mine = (hi - first + wgs_per_xcd - 1) / wgs_per_xcd;
#define PEVLM_ITEM(ord) (p.items + (first + (ord) * wgs_per_xcd))

    const int32_t tid = threadIdx.x, lane = tid & 63;
    const int32_t wave = sgpr(tid >> 6);
    const int32_t l32 = lane & 31, g32 = lane >> 5;
    const int32_t Hq = p.n_q_heads, Hkv = p.n_kv_heads;

    LaneOff L;
    L.g32 = g32;
    L.k_row_off = l32 * ROWB;
    L.k_swz = l32 & (CH - 1);
    L.v_row_off = (g32 * 4 + ((lane & 15) >> 2)) * ROWB + (lane & 1) * 8;
    L.v_ch_lo = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    L.v_swz = (lane >> 2) & VSW;

    uint8_t *const lds_k = lds, *const lds_v = lds + NST * TILEB;
    uint8_t *const slice = lds + 2 * NST * TILEB + wave * WSLICE;
    const uint32_t lds_k_addr = (uint32_t)(size_t)LDS_PTR(void, lds_k);
    const uint32_t lds_v_addr = (uint32_t)(size_t)LDS_PTR(void, lds_v);
    const uint32_t slice_addr = (uint32_t)(size_t)LDS_PTR(void, slice);

    // ---- K/V tile loads: a wavefront instruction fills 1 KB of LDS = RPI whole rows of the tile, piece
    // j of wavefront w being rows (j * NW + w) * RPI ...; which 16-byte chunk of the row a lane fetches
    // carries the XOR swizzle (K by row & 15, V by (row & 3) << 2), the same for every piece of a lane
    // (pieces are a multiple of 16 rows apart).
    const uint32_t kv_row_bytes = (uint32_t)(Hkv * D * 2);
    const uint32_t tile_bytes = KT * kv_row_bytes;
    const int64_t v_minus_k = (int64_t)((uint64_t)p.v - (uint64_t)p.k);
    BufTileLoads<PSTEP> ldk, ldv;
    {
        const int32_t row0 = wave * RPI + lane / CH, cpos = lane % CH;
        ldk.voff = (uint32_t)row0 * kv_row_bytes + (uint32_t)((cpos ^ (row0 & (CH - 1))) << 4);
        ldv.voff = (uint32_t)row0 * kv_row_bytes + (uint32_t)((cpos ^ ((row0 & VSW) << 2)) << 4);
        ldk.sstep = ldv.sstep = NW * RPI * kv_row_bytes;
    }

    // ---- load stream state.  kc is the tile whose K is loaded next; the V loads of a tile follow one
    // tile later and use the descriptor remembered in (v_base, v_bytes, v_soff).
    TileCursor kc;
#define PEVLM_CURSOR_SET(ord_)                                                                          \
    do {                                                                                                \
        const pevlm_stream_item *ci_ = PEVLM_ITEM(ord_);                                                \
        const int32_t g_ = item_word(ci_, F_KV_HEAD);                                                   \
        const int32_t fs_ = item_word(ci_, F_FULL_START), fl_ = item_word(ci_, F_FULL_LEN);             \
        const int32_t ds_ = item_word(ci_, F_DIAG_START), dl_ = item_word(ci_, F_DIAG_LEN);             \
        kc.n_full = item_word(ci_, F_N_FULL);                                                           \
        kc.n_tiles = item_word(ci_, F_N_TILES);                                                         \
        kc.ord = (ord_);                                                                                \
        kc.t = 0;                                                                                       \
        kc.base_full = (uint64_t)p.k + ((uint64_t)((int64_t)fs_ * Hkv + g_) * D) * 2;                   \
        kc.base_diag = (uint64_t)p.k + ((uint64_t)((int64_t)ds_ * Hkv + g_) * D) * 2;                   \
        kc.bytes_full = (uint32_t)fl_ * kv_row_bytes;                                                   \
        kc.bytes_diag = (uint32_t)dl_ * kv_row_bytes;                                                   \
    } while (0)
    PEVLM_CURSOR_SET(0);
    uint64_t v_base = 0;
    uint32_t v_bytes = 0, v_soff = 0;
    // advances kc by one tile (into the next item at the end of one; stays on the last tile of the last item)
#define PEVLM_CURSOR_ADVANCE()                                        \
    do {                                                              \
        if (kc.t + 1 < kc.n_tiles) {                                  \
            kc.t += 1;                                                \
        } else if (kc.ord + 1 < n_mine) {                             \
            const int32_t nord_ = kc.ord + 1;                         \
            PEVLM_CURSOR_SET(nord_);                                  \
        }                                                             \
    } while (0)
    // descriptors of the loads of one tile step: K of tile kc -> stage ks_ld, V of the tile before it ->
    // stage vs_ld; then kc moves on
#define PEVLM_TILE_LOADS_SETUP(ks_ld, vs_ld)                                                            \
    do {                                                                                                \
        const bool full_ = kc.t < kc.n_full;                                                            \
        const uint64_t kb_ = full_ ? kc.base_full : kc.base_diag;                                       \
        const uint32_t kn_ = full_ ? kc.bytes_full : kc.bytes_diag;                                     \
        const uint32_t so_ = (uint32_t)(full_ ? kc.t : kc.t - kc.n_full) * tile_bytes;                  \
        ldk.rsrc = make_rsrc(kb_, kn_);                                                                 \
        ldk.soff = so_;                                                                                 \
        ldv.rsrc = make_rsrc(v_base, v_bytes);                                                          \
        ldv.soff = v_soff;                                                                              \
        ldk.lds = lds_k_addr + (ks_ld) * TILEB + wave * 1024;                                           \
        ldv.lds = lds_v_addr + (vs_ld) * TILEB + wave * 1024;                                           \
        v_base = kb_ + (uint64_t)v_minus_k; v_bytes = kn_; v_soff = so_;                                \
        PEVLM_CURSOR_ADVANCE();                                                                         \
    } while (0)
#define PEVLM_TILE_LOADS_BURST()                                       \
    do {                                                               \
        _Pragma("unroll") for (int j = 0; j < NL; ++j) ldk.issue(j);   \
        _Pragma("unroll") for (int j = 0; j < NL; ++j) ldv.issue(j);   \
    } while (0)

    // ---- query slice loads: whole 256-byte rows of one head, chunk-swizzled like a K tile.  The
    // descriptor ends with the slot's last row: rows past it (and every row of an unused slot, or of a
    // prefetch past the last item: zero rows) arrive as zeros.
#define PEVLM_ISSUE_Q(q_start, q_rows, head)                                                            \
    do {                                                                                                \
        const uint32_t qrb_ = (uint32_t)(Hq * D * 2);                                                   \
        const i32x4 rq_ = make_rsrc((uint64_t)p.q + ((uint64_t)((int64_t)(q_start) * Hq + (head)) * D) * 2, (uint32_t)(q_rows) * qrb_); \
        const int32_t ln_ = opaque(lane);                                                               \
        _Pragma("unroll") for (int j = 0; j < NQL; ++j) {                                               \
            const int32_t rl = j * RPI + ln_ / CH;                                                      \
            load_lds_16_buf(rq_, (uint32_t)rl * qrb_ + (uint32_t)(((ln_ % CH) ^ (rl & (CH - 1))) << 4), 0u, slice_addr + j * 1024); \
        }                                                                                               \
    } while (0)
#define PEVLM_READ_QF()                                                                                 \
    do {                                                                                                \
        const int32_t ln_ = opaque(lane), r32_ = ln_ & 31, h32_ = ln_ >> 5;                             \
        _Pragma("unroll") for (int kk = 0; kk < KSTEPS; ++kk)                                           \
            qf[kk] = *reinterpret_cast<const bf16x8 *>(slice + r32_ * ROWB + (((kk * 2 + h32_) ^ (r32_ & (CH - 1))) << 4)); \
    } while (0)

    // ---- per-wavefront compute state
    bf16x8 qf[KSTEPS];
    f32x16 o[DBLK], s[2];
    u32x4 pf_prev[4], pf_new[4];
    float m_ref = -INFINITY, l_run = 0.f, psum = 0.f;
    const float c_log2 = p.scale * 1.4426950408889634f;
#define PEVLM_MREF ((m_ref == -INFINITY) ? 0.f : m_ref)
    // slot of the item being computed / of the item whose last value tile and output are pending
    int32_t q_start = 0, q_rows = 0, head = 0;
    int32_t pend = 0, pend_vs = 0, pend_q_start = 0, pend_q_rows = 0, pend_head = 0;
    int32_t q_age = 3;  // tiles since this wavefront last issued a query prefetch (>= 3: it has landed)

    // same check-after-the-fact reference maximum as the one-item kernel
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
            if (__any(has)) {                                                                         \
                l_run *= alpha;                                                                       \
                _Pragma("unroll") for (int b = 0; b < DBLK; ++b)                                      \
                    _Pragma("unroll") for (int i = 0; i < 16; ++i) o[b][i] *= alpha;                  \
            }                                                                                         \
        }                                                                                             \
    } while (0)

    // last value tile of a finished slot (V stage pend_vs), normalisation, rows out through the slice
#define PEVLM_FINISH_PENDING()                                                                        \
    do {                                                                                              \
        pv_tile<D>(lds_v + pend_vs * TILEB, L, pf_prev, o);                                           \
        const float l_tot = l_run + __shfl_xor(l_run, 32);                                            \
        const float inv = 1.f / l_tot;                                                                \
        const int32_t ln_ = opaque(lane), r32_ = ln_ & 31, h32_ = ln_ >> 5, cp_ = ln_ % CH;           \
        _Pragma("unroll") for (int b = 0; b < DBLK; ++b)                                              \
            _Pragma("unroll") for (int i4 = 0; i4 < 4; ++i4) {                                        \
                bf16x4 v4;                                                                            \
                v4[0] = (__bf16)(o[b][i4 * 4] * inv);                                                 \
                v4[1] = (__bf16)(o[b][i4 * 4 + 1] * inv);                                             \
                v4[2] = (__bf16)(o[b][i4 * 4 + 2] * inv);                                             \
                v4[3] = (__bf16)(o[b][i4 * 4 + 3] * inv);                                             \
                *reinterpret_cast<bf16x4 *>(slice + r32_ * ROWB + (((b * 4 + i4) ^ (r32_ & (CH - 1))) << 4) + h32_ * 8) = v4; \
            }                                                                                         \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                        \
        __builtin_amdgcn_wave_barrier();                                                              \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");                                        \
        uint16_t *const obase = (uint16_t *)p.out;                                                    \
        _Pragma("unroll") for (int j = 0; j < NQL; ++j) {                                             \
            const int32_t rl = j * RPI + ln_ / CH;                                                    \
            const uint4 val = *reinterpret_cast<const uint4 *>(slice + rl * ROWB + ((cp_ ^ (rl & (CH - 1))) << 4)); \
            if (rl < pend_q_rows)                                                                     \
                *reinterpret_cast<uint4 *>(obase + ((int64_t)(pend_q_start + rl) * Hq + pend_head) * D + cp_ * 8) = val; \
        }                                                                                             \
        if (p.lse && h32_ == 0 && r32_ < pend_q_rows)                                                 \
            p.lse[(int64_t)(pend_q_start + r32_) * Hq + pend_head] = (m_ref + __log2f(l_tot)) * 0.69314718056f; \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); /* the slice has been read: it may be refilled */ \
        pend = 0;                                                                                     \
    } while (0)

    // query rows of the item after next (the next item's are already in registers or in the slice); past
    // the last item, or for an unused slot, a descriptor of zero rows: zeros arrive, no memory is touched
#define PEVLM_PREFETCH_Q(ord_target)                                                                  \
    do {                                                                                              \
        int32_t ps_ = 0, pr_ = 0, ph_ = 0;                                                            \
        if ((ord_target) < n_mine) {                                                                  \
            const pevlm_stream_item *nx_ = PEVLM_ITEM(ord_target);                                    \
            ps_ = item_word(nx_, F_SLOT0 + wave * S_WORDS + S_Q_START);                               \
            pr_ = item_word(nx_, F_SLOT0 + wave * S_WORDS + S_Q_ROWS);                                \
            ph_ = item_word(nx_, F_SLOT0 + wave * S_WORDS + S_HEAD);                                  \
        }                                                                                             \
        PEVLM_ISSUE_Q(ps_, pr_, ph_);                                                                 \
        q_age = 0;                                                                                    \
    } while (0)

    // ================= prologue: first tiles and the first item's queries =================
    {
        // K(0) -> stage 0 (the V descriptor of this step is empty: zeros into V stage 2, which is rewritten
        // before it is read), then K(1) -> stage 1 and V(0) -> stage 0; kc then stands on tile 2
        PEVLM_TILE_LOADS_SETUP(0, 2);
        PEVLM_TILE_LOADS_BURST();
        PEVLM_TILE_LOADS_SETUP(1, 0);
        PEVLM_TILE_LOADS_BURST();
    }
    {
        const pevlm_stream_item *it0 = PEVLM_ITEM(0);
        q_start = item_word(it0, F_SLOT0 + wave * S_WORDS + S_Q_START);
        q_rows = item_word(it0, F_SLOT0 + wave * S_WORDS + S_Q_ROWS);
        head = item_word(it0, F_SLOT0 + wave * S_WORDS + S_HEAD);
        PEVLM_ISSUE_Q(q_start, q_rows, head);
        PEVLM_WAIT_VM(0);
        PEVLM_READ_QF();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        PEVLM_PREFETCH_Q(1);
        q_age = 1;  // issued before the loads of tile 0: as if in the tile before it
    }

    int32_t ks = 0;  // LDS stage of the current tile's K; V of the previous tile sits in stage (ks + 2) % 3
    // top of a tile: K(t) and V(t-1) of every wavefront have landed (the loads issued during the previous
    // tile, and a query prefetch issued within the last two tiles, may still be in flight), everybody has
    // left the previous tile; then the loads of this tile step are prepared (K(t+2) -> stage (ks+2)%3,
    // V(t+1) -> stage (ks+1)%3)
#define PEVLM_TOP()                                                                                   \
    do {                                                                                              \
        if (q_age <= 2) wait_vm<TL + NQL>(); else wait_vm<TL>();                                      \
        __builtin_amdgcn_s_barrier();                                                                 \
        asm volatile("" ::: "memory");                                                                \
        PEVLM_TILE_LOADS_SETUP((ks >= 1 ? ks - 1 : 2), (ks + 1 < NST ? ks + 1 : 0));                  \
    } while (0)
#define PEVLM_NEXT_TILE()                  \
    do {                                   \
        ks = ks + 1 < NST ? ks + 1 : 0;    \
        q_age += 1;                        \
    } while (0)
    // key range of tile t of the current item
#define PEVLM_TILE_RANGE(t, k0, kend, causal)                                                         \
    do {                                                                                              \
        if ((t) < n_full_tiles) {                                                                     \
            k0 = full_start + (t) * KT; kend = full_start + full_len; causal = false;                 \
        } else {                                                                                      \
            k0 = diag_start + ((t) - n_full_tiles) * KT; kend = diag_start + diag_len; causal = true; \
        }                                                                                             \
    } while (0)
    // end of this wavefront's arithmetic for the item (after its last computed tile, or in tile 0 for an
    // unused slot): the next item's queries move from the slice to registers; the last value tile and the
    // output wait for the next tile top.  The prefetched queries must have landed: a prefetch issued in
    // this very tile is the youngest load; otherwise only this tile's K/V loads may still be in flight.
#define PEVLM_END_OF_COMPUTE(ord)                                                                     \
    do {                                                                                              \
        if (q_age == 0) {                                                                             \
            PEVLM_WAIT_VM(0);                                                                         \
        } else if (q_age < 3) {                                                                       \
            wait_vm<TL>();                                                                            \
        }                                                                                             \
        asm volatile("" ::: "memory");                                                                \
        if ((ord) + 1 < n_mine) PEVLM_READ_QF();                                                      \
        if (n_w > 0) {                                                                                \
            pend = 1;                                                                                 \
            pend_vs = ks; /* V(t) goes to stage t % 3 = ks */                                         \
            pend_q_start = q_start;                                                                   \
            pend_q_rows = q_rows;                                                                     \
            pend_head = head;                                                                         \
        } else {                                                                                      \
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                        \
            PEVLM_PREFETCH_Q((ord) + 2);                                                              \
        }                                                                                             \
    } while (0)

    // ================= the item loop =================
    for (int32_t ord = 0; ord < n_mine; ++ord) {
        const pevlm_stream_item *it = PEVLM_ITEM(ord);
        const int32_t full_start = item_word(it, F_FULL_START), full_len = item_word(it, F_FULL_LEN);
        const int32_t diag_start = item_word(it, F_DIAG_START), diag_len = item_word(it, F_DIAG_LEN);
        const int32_t n_full_tiles = item_word(it, F_N_FULL), n_tiles = item_word(it, F_N_TILES);
        q_start = item_word(it, F_SLOT0 + wave * S_WORDS + S_Q_START);
        q_rows = item_word(it, F_SLOT0 + wave * S_WORDS + S_Q_ROWS);
        head = item_word(it, F_SLOT0 + wave * S_WORDS + S_HEAD);
        // tiles this wavefront computes: every fully visible one and the causal ones that start at or
        // before its last row
        const int32_t wr_lo = q_start, wr_hi = q_start + q_rows - 1;
        int32_t n_w = 0;
        if (q_rows > 0) {
            const int32_t nd = wr_hi >= diag_start ? (wr_hi - diag_start) / KT + 1 : 0;
            n_w = n_full_tiles + (nd < n_tiles - n_full_tiles ? nd : n_tiles - n_full_tiles);
        }
        const int32_t my_row = q_start + (l32 < q_rows ? l32 : (q_rows > 0 ? q_rows - 1 : 0));
        int32_t k0, kend;
        bool causal;

        // ---- tile 0: loads in one burst, the pending end of the previous item's slot, then the first
        // tile's exact softmax (no row has a reference maximum yet)
        PEVLM_TOP();
        PEVLM_TILE_LOADS_BURST();
        if (pend) {
            PEVLM_FINISH_PENDING();
            PEVLM_PREFETCH_Q(ord + 1);
        }
        if (n_w > 0) {
            m_ref = -INFINITY;
            l_run = 0.f;
#pragma unroll
            for (int b = 0; b < DBLK; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[b][i] = 0.f;
            PEVLM_TILE_RANGE(0, k0, kend, causal);
            qk_tile_ring<D, false, NL>(lds_k + ks * TILEB, L, qf, s, ldk);
            if ((k0 + KT > kend) || (causal && (k0 + KT - 1 > wr_lo))) mask_tile(s, k0, kend, causal, my_row, g32);
            psum = 0.f;
            PEVLM_FIX_REFERENCE();
            l_run += psum;
#pragma unroll
            for (int j = 0; j < 4; ++j) pf_prev[j] = pf_new[j];
        }
        if (n_w <= 1) PEVLM_END_OF_COMPUTE(ord);
        PEVLM_NEXT_TILE();

        // ---- steady state: scores of tile t with K(t+2) requested piecewise, then the values of tile t-1
        // under the weights of tile t with V(t+1) requested piecewise
        for (int32_t t = 1; t < n_w; ++t) {
            PEVLM_TOP();
            PEVLM_TILE_RANGE(t, k0, kend, causal);
            qk_tile_ring<D, true, NL>(lds_k + ks * TILEB, L, qf, s, ldk);
            if ((k0 + KT > kend) || (causal && (k0 + KT - 1 > wr_lo))) mask_tile(s, k0, kend, causal, my_row, g32);
            psum = 0.f;
            pv_prev_weights_cur_ring<D, NL>(lds_v + (ks >= 1 ? ks - 1 : 2) * TILEB, L, pf_prev, o, s, c_log2, PEVLM_MREF, psum, pf_new, ldv);
            PEVLM_FIX_REFERENCE();
            l_run += psum;
#pragma unroll
            for (int j = 0; j < 4; ++j) pf_prev[j] = pf_new[j];
            if (t == n_w - 1) PEVLM_END_OF_COMPUTE(ord);
            PEVLM_NEXT_TILE();
        }

        // ---- tiles this wavefront does not compute (causal tiles past its rows): its share of the
        // loads; in the first of them the slot's last value tile and output
        for (int32_t t = n_w > 1 ? n_w : 1; t < n_tiles; ++t) {
            PEVLM_TOP();
            PEVLM_TILE_LOADS_BURST();
            if (pend) {
                PEVLM_FINISH_PENDING();
                PEVLM_PREFETCH_Q(ord + 2);
            }
            PEVLM_NEXT_TILE();
        }
    }
    // ================= flush: the last item's last value tile and output =================
    PEVLM_WAIT_VM(0);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (pend) PEVLM_FINISH_PENDING();
#undef PEVLM_ITEM
}

hipError_t launch_attn_bf16_stream(const StreamParams &p, int32_t D, int32_t compute_units, hipStream_t stream)
{
    // one resident workgroup per compute unit, a multiple of 8 so that every XCD gets the same number
    int32_t per_xcd_items = (p.n_items + 7) / 8;
    int32_t wgs_per_xcd = compute_units / 8 > 0 ? compute_units / 8 : 1;
    if (wgs_per_xcd > per_xcd_items) wgs_per_xcd = per_xcd_items;
    dim3 grid(8 * wgs_per_xcd), block(512);
    if (D == 128) hipLaunchKernelGGL((attn_bf16_stream_kernel<128>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((attn_bf16_stream_kernel<64>), grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace pevlm
