// Host side of libpevlm: argument validation, workspace carving, work-list builders and launches.
// Entry points are documented in include/pevlm.h.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "common.h"

namespace pevlm {

static thread_local char g_err[512] = "no error";

static pevlm_status fail(pevlm_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

static pevlm_status hip_fail(hipError_t e, const char *what)
{
    return fail(PEVLM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static size_t align256(size_t n) { return (n + 255) & ~size_t(255); }

static pevlm_status check_layout(const pevlm_layout *lay)
{
    if (!lay) return fail(PEVLM_ERR_INVALID_ARG, "layout is NULL");
    if (lay->num_seqs < 1) return fail(PEVLM_ERR_INVALID_ARG, "num_seqs must be >= 1");
    if (!lay->cu_seqlens || !lay->sink_len || !lay->block_len || !lay->ctx_len || !lay->query_len)
        return fail(PEVLM_ERR_INVALID_ARG, "layout array is NULL");
    if (lay->cu_seqlens[0] != 0) return fail(PEVLM_ERR_INVALID_ARG, "cu_seqlens[0] must be 0");
    for (int32_t s = 0; s < lay->num_seqs; ++s) {
        int64_t len = (int64_t)lay->cu_seqlens[s + 1] - lay->cu_seqlens[s];
        if (len < 0) return fail(PEVLM_ERR_INVALID_ARG, "cu_seqlens decreases at sequence %d", s);
        if (lay->sink_len[s] < 0 || lay->ctx_len[s] < 0 || lay->query_len[s] < 0)
            return fail(PEVLM_ERR_INVALID_ARG, "negative region length in sequence %d", s);
        if (lay->ctx_len[s] > 0 && lay->block_len[s] < 1)
            return fail(PEVLM_ERR_INVALID_ARG, "block_len must be >= 1 in sequence %d", s);
        if ((int64_t)lay->sink_len[s] + lay->ctx_len[s] + lay->query_len[s] != len)
            return fail(PEVLM_ERR_INVALID_ARG, "sink+ctx+query != sequence length in sequence %d", s);
    }
    return PEVLM_OK;
}

static pevlm_status check_heads(const pevlm_heads *h, HeadTable *tab)
{
    if (!h) return fail(PEVLM_ERR_INVALID_ARG, "heads is NULL");
    if (h->n_q_heads < 1 || h->n_kv_heads < 1 || h->n_q_heads % h->n_kv_heads != 0)
        return fail(PEVLM_ERR_INVALID_ARG, "need n_q_heads %% n_kv_heads == 0 (got %d / %d)", h->n_q_heads,
                    h->n_kv_heads);
    if (h->n_q_heads > kMaxHeads) return fail(PEVLM_ERR_UNSUPPORTED, "more than %d query heads", kMaxHeads);
    if (h->dtype != PEVLM_F32 && h->dtype != PEVLM_BF16) return fail(PEVLM_ERR_UNSUPPORTED, "unknown dtype %d", (int)h->dtype);
    if (h->head_dim != 64 && h->head_dim != 128)
        return fail(PEVLM_ERR_UNSUPPORTED, "head_dim %d not in {64, 128}", h->head_dim);
    int32_t G = h->n_q_heads / h->n_kv_heads;
    for (int32_t i = 0; i < h->n_q_heads; ++i) {
        int32_t g = h->kv_head_of_q ? h->kv_head_of_q[i] : i / G;
        if (g < 0 || g >= h->n_kv_heads) return fail(PEVLM_ERR_INVALID_ARG, "kv_head_of_q[%d] = %d out of range", i, g);
        if (tab) tab->kv_of_q[i] = (uint8_t)g;
    }
    if (tab) {  // schedule order: heads grouped by KV head so neighbours share K/V in L2
        int32_t n = 0;
        for (int32_t g = 0; g < h->n_kv_heads; ++g)
            for (int32_t i = 0; i < h->n_q_heads; ++i)
                if (tab->kv_of_q[i] == g) tab->head_order[n++] = (uint8_t)i;
    }
    return PEVLM_OK;
}

static float scale_of(const pevlm_heads *h)
{
    return h->softmax_scale > 0.f ? h->softmax_scale : (float)(1.0 / sqrt((double)h->head_dim));
}

static int32_t tile_rows_of(const pevlm_heads *h, bool /*query*/)
{
    return h->dtype == PEVLM_BF16 ? kTileRowsBf16 : kTileRowsF32;
}

// Streaming restrictions of a call (host arrays of num_seqs entries, NULL = no restriction).
struct Restrict {
    const int32_t *first_block = nullptr, *num_blocks = nullptr;  // prefill: context blocks computed
    int32_t with_sink = 1;                                        // prefill: sink rows computed
    const int32_t *window_blocks = nullptr;                       // question: last W blocks visible (<0: all)
};

// Three-axis position ids for the calls with RoPE folded in (pos_ids == NULL: sequential positions).
struct Axes {
    const int32_t *pos_ids = nullptr;  // DEVICE [3][T]
    int32_t sec0 = 0, sec01 = 0;       // sections [0, sec0), [sec0, sec01), [sec01, D/2)
};

static pevlm_status check_axes(const pevlm_heads *heads, const int32_t *pos_ids, const int32_t *section, Axes *ax)
{
    if (!pos_ids || ((uintptr_t)pos_ids & 3)) return fail(PEVLM_ERR_INVALID_ARG, "pos_ids must be a 4-byte aligned device pointer");
    if (!section || section[0] < 0 || section[1] < 0 || section[2] < 0 ||
        (int64_t)section[0] + section[1] + section[2] != heads->head_dim / 2)
        return fail(PEVLM_ERR_INVALID_ARG, "section must hold three non-negative counts that add up to head_dim/2");
    ax->pos_ids = pos_ids;
    ax->sec0 = section[0];
    ax->sec01 = section[0] + section[1];
    return PEVLM_OK;
}

static int32_t blocks_of(const pevlm_layout *lay, int32_t s)
{
    return lay->ctx_len[s] > 0 ? (lay->ctx_len[s] + lay->block_len[s] - 1) / lay->block_len[s] : 0;
}

static pevlm_status check_restrict(const pevlm_layout *lay, const Restrict &r)
{
    if ((r.first_block == nullptr) != (r.num_blocks == nullptr))
        return fail(PEVLM_ERR_INVALID_ARG, "first_block and num_blocks must be given together");
    if (r.first_block)
        for (int32_t s = 0; s < lay->num_seqs; ++s)
            if (r.first_block[s] < 0 || r.num_blocks[s] < 0 || (int64_t)r.first_block[s] + r.num_blocks[s] > blocks_of(lay, s))
                return fail(PEVLM_ERR_INVALID_ARG, "block range [%d, %d + %d) outside the %d context blocks of sequence %d",
                            r.first_block[s], r.first_block[s], r.num_blocks[s], blocks_of(lay, s), s);
    return PEVLM_OK;
}

// Fills the chunk table for sequences [s0, s0 + n).
static void fill_table(const pevlm_layout *lay, int32_t s0, int32_t n, const int32_t *pos_offset, SeqTable *t,
                       const Restrict &r = Restrict())
{
    memset(t, 0, sizeof *t);
    t->num_seqs = n;
    t->seq_index0 = s0;
    t->sel_sink = r.with_sink ? 1 : 0;
    t->windowed = r.window_blocks ? 1 : 0;
    for (int32_t i = 0; i < n; ++i) {
        int32_t s = s0 + i;
        t->start[i] = lay->cu_seqlens[s];
        t->sink[i] = lay->sink_len[s];
        t->block[i] = lay->ctx_len[s] > 0 ? lay->block_len[s] : 1;
        t->ctx[i] = lay->ctx_len[s];
        t->query[i] = lay->query_len[s];
        t->pos_offset[i] = pos_offset ? pos_offset[s] : 0;
        t->sel_first[i] = r.first_block ? r.first_block[s] : 0;
        t->sel_count[i] = r.num_blocks ? r.num_blocks[s] : blocks_of(lay, s);
        int32_t hidden = 0;  // context blocks the question no longer sees
        if (r.window_blocks && r.window_blocks[s] >= 0) hidden = std::max(0, blocks_of(lay, s) - r.window_blocks[s]);
        t->win_start[i] = t->sink[i] + (int32_t)std::min<int64_t>((int64_t)hidden * t->block[i], t->ctx[i]);
    }
}

static int64_t count_prefill_items(const pevlm_layout *lay, int32_t tile_rows, const Restrict &r = Restrict())
{
    int64_t n = 0;
    for (int32_t s = 0; s < lay->num_seqs; ++s)
        n += prefill_items_of_seq_sel(lay->sink_len[s], lay->ctx_len[s] > 0 ? lay->block_len[s] : 1, lay->ctx_len[s], tile_rows,
                                      r.first_block ? r.first_block[s] : 0, r.num_blocks ? r.num_blocks[s] : blocks_of(lay, s),
                                      r.with_sink);
    return n;
}

static int64_t count_query_tiles(const pevlm_layout *lay, int32_t tile_rows)
{
    int64_t n = 0;
    for (int32_t s = 0; s < lay->num_seqs; ++s) n += query_tiles_of_seq(lay->query_len[s], tile_rows);
    return n;
}

static int64_t total_query_rows(const pevlm_layout *lay)
{
    int64_t n = 0;
    for (int32_t s = 0; s < lay->num_seqs; ++s) n += lay->query_len[s];
    return n;
}

// The streaming bf16 block-prefill kernel applies when every KV head serves the same number of query
// heads (it deals the heads of a KV head out over the wavefronts of a workgroup).
static bool equal_head_groups(const pevlm_heads *h)
{
    const int32_t G = h->n_q_heads / h->n_kv_heads;
    if (!h->kv_head_of_q) return true;
    int32_t count[kMaxHeads] = {0};
    for (int32_t i = 0; i < h->n_q_heads; ++i) count[h->kv_head_of_q[i]] += 1;
    for (int32_t g = 0; g < h->n_kv_heads; ++g)
        if (count[g] != G) return false;
    return true;
}

// Which kernel serves the block-prefill call on bf16 tensors: 0 = chosen per call (below), 1 = always the
// one-item-per-workgroup kernel, 2 = the streaming kernel whenever it applies.  Process-wide; starts
// from PEVLM_PREFILL_KERNEL=classic|stream in the environment (anything else: 0).
static std::atomic<int32_t> &prefill_kernel_mode()
{
    static std::atomic<int32_t> mode([] {
        const char *e = getenv("PEVLM_PREFILL_KERNEL");
        return e && strcmp(e, "classic") == 0 ? 1 : (e && strcmp(e, "stream") == 0 ? 2 : 0);
    }());
    return mode;
}

// The streaming kernel needs equal head groups and bf16 tensors, and addresses a key range through
// 32-bit byte offsets from the range's first row.
static bool stream_kernel_applies(const pevlm_layout *lay, const pevlm_heads *h)
{
    const int64_t T = lay->cu_seqlens[lay->num_seqs];
    return h->dtype == PEVLM_BF16 && equal_head_groups(h) && T * h->n_kv_heads * h->head_dim * 2 < ((int64_t)1 << 31);
}

// It deals whole items out to one resident workgroup per compute unit; with only a few items per
// workgroup the shares come out too uneven, and the one-item-per-workgroup kernel (two small workgroups
// per compute unit, dispatched as slots free up) finishes sooner.  So it does on regions far longer
// than any block the method uses (a dense causal attention written as one block: measured 8 % faster at
// 64K rows), where the key stream of an item no longer stays in the L2 of its XCD.
constexpr int32_t kMinStreamItemsPerWorkgroup = 12;
constexpr int32_t kMaxStreamRegionRows = 16384;

static bool regions_fit_stream_kernel(const pevlm_layout *lay)
{
    for (int32_t s = 0; s < lay->num_seqs; ++s)
        if (lay->sink_len[s] > kMaxStreamRegionRows || (lay->ctx_len[s] > 0 && std::min(lay->block_len[s], lay->ctx_len[s]) > kMaxStreamRegionRows))
            return false;
    return true;
}

static int64_t count_stream_items(const pevlm_layout *lay, const pevlm_heads *h, const Restrict &r = Restrict())
{
    const int32_t G = h->n_q_heads / h->n_kv_heads;
    int64_t n = 0;
    for (int32_t s = 0; s < lay->num_seqs; ++s)
        n += stream_items_of_seq(lay->sink_len[s], lay->ctx_len[s] > 0 ? lay->block_len[s] : 1, lay->ctx_len[s], G, h->n_kv_heads,
                                 r.first_block ? r.first_block[s] : 0, r.num_blocks ? r.num_blocks[s] : blocks_of(lay, s),
                                 r.with_sink);
    return n;
}

static int32_t compute_units();

// Stream items of the call if the streaming kernel is to run it, else 0.
static int64_t stream_items_if_chosen(const pevlm_layout *lay, const pevlm_heads *h, const Restrict &r, bool fuse_rope)
{
    const int32_t mode = prefill_kernel_mode().load(std::memory_order_relaxed);
    if (fuse_rope || mode == 1 || !stream_kernel_applies(lay, h)) return 0;
    const int64_t n = count_stream_items(lay, h, r);
    return (mode == 2 || (n >= (int64_t)kMinStreamItemsPerWorkgroup * compute_units() && regions_fit_stream_kernel(lay))) ? n : 0;
}

// Compute units of the current device (256 when it cannot be queried, e.g. no GPU present).
static int32_t compute_units()
{
    static std::atomic<int32_t> cached[16];  // zero-initialised; racing first calls store the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) { (void)hipGetLastError(); return 256; }
    int32_t have = cached[dev].load(std::memory_order_relaxed);
    if (have == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            n = 256;
        }
        have = n;
        cached[dev].store(have, std::memory_order_relaxed);
    }
    return have;
}

// Split count when the caller leaves it to the library: the split kernel keeps two workgroups per
// compute unit, so the number of workgroups (row tiles x heads x splits) is brought as close as
// possible to one or two full rounds of 2 x CUs from below, with no split of the longest sequence shorter than 768 keys (measured sweet spots: 18 splits at
// 64K tokens x 28 heads, 8 at 100K x 2 tiles x 32 heads).
static int32_t auto_splits(const pevlm_layout *lay, const pevlm_heads *h)
{
    const int32_t tile_rows = tile_rows_of(h, true);
    const int32_t G = h->n_q_heads / h->n_kv_heads;
    // workgroups per split: one per (row tile, head); the bf16 kernel takes tiles of <= 64 rows
    // for 2 or 4 heads of a KV group at once
    int64_t units = 0, max_len = 0, min_len = INT64_MAX;
    for (int32_t s = 0; s < lay->num_seqs; ++s) {
        if (lay->query_len[s] == 0) continue;
        max_len = std::max<int64_t>(max_len, (int64_t)lay->cu_seqlens[s + 1] - lay->cu_seqlens[s]);
        min_len = std::min<int64_t>(min_len, (int64_t)lay->cu_seqlens[s + 1] - lay->cu_seqlens[s]);
        for (int32_t r0 = 0; r0 < lay->query_len[s]; r0 += tile_rows) {
            int32_t rows = std::min(tile_rows, lay->query_len[s] - r0);
            int32_t hpw = 1;
            if (h->dtype == PEVLM_BF16 && G > 1 && !h->kv_head_of_q) hpw = rows <= 32 ? 4 : (rows <= 64 ? 2 : 1);
            units += (int64_t)h->n_kv_heads * ((G + hpw - 1) / hpw);
        }
    }
    if (units == 0) return 1;
    const int64_t slots = 2 * (int64_t)compute_units();
    int64_t want = slots / units;                      // one round
    if (want < 1) want = 1;
    // a badly filled round, or sequences of very different length (every sequence gets the same
    // number of splits, so the long ones set the pace): take two rounds of finer pieces
    if (want * units * 4 < slots * 3 || 2 * min_len < max_len) want = (2 * slots) / units;
    const int64_t cap = std::max<int64_t>(1, max_len / 768);
    return (int32_t)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, cap), PEVLM_MAX_SPLITS));
}

// bytes of the (cos, sin) table of the fused query rotation: head_dim/2 pairs of floats per entry
static size_t rope_table_bytes(int64_t entries, const pevlm_heads *h) { return align256((size_t)entries * h->head_dim * sizeof(float)); }

struct QueryPlan {
    int32_t num_splits, tile_rows;
    int64_t n_items, total_q;
    size_t off_items, off_qrow, off_ml, off_acc, off_rope, bytes;
};

static QueryPlan plan_query(const pevlm_layout *lay, const pevlm_heads *h, int32_t num_splits, bool fuse_rope = false,
                            bool windowed = false)
{
    QueryPlan p;
    p.tile_rows = tile_rows_of(h, true);
    p.num_splits = num_splits > 0 ? num_splits : auto_splits(lay, h);
    // with a window the sink is a split of its own, the rest of the keys takes at least one more
    if (windowed) p.num_splits = std::min(PEVLM_MAX_SPLITS, std::max(2, p.num_splits + (num_splits > 0 ? 0 : 1)));
    p.total_q = total_query_rows(lay);
    p.n_items = count_query_tiles(lay, p.tile_rows) * p.num_splits;
    size_t off = 0;
    p.off_items = off;
    off += align256((size_t)p.n_items * sizeof(pevlm_work_item));
    p.off_qrow = off;
    off += align256((size_t)p.total_q * sizeof(int32_t));
    p.off_ml = off;
    off += align256((size_t)p.num_splits * p.total_q * h->n_q_heads * 2 * sizeof(float));
    p.off_acc = off;
    off += align256((size_t)p.num_splits * p.total_q * h->n_q_heads * h->head_dim * sizeof(float));
    p.off_rope = off;
    if (fuse_rope) off += rope_table_bytes(p.total_q, h);  // one entry per compact question row
    p.bytes = off;
    return p;
}

// ------------------------------------------------------------------------------------------
// Library-owned scratch memory of pevlm_query_attn_static: one array per GPU, part of the code
// object, alive until the process ends.  Host code never uses the array's name as an address: the
// device address is looked up once per device and kept.
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PEVLM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call per device).
static pevlm_status scratch_of_current_device(void **ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(PEVLM_ERR_UNSUPPORTED, "device index %d not below %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return PEVLM_OK;
}

}  // namespace pevlm

using namespace pevlm;

extern "C" {

const char *pevlm_last_error(void) { return g_err; }
int32_t pevlm_version(void) { return 100; }
int32_t pevlm_prefill_tile_rows(const pevlm_heads *heads) { return check_heads(heads, nullptr) == PEVLM_OK ? tile_rows_of(heads, false) : -1; }
int32_t pevlm_query_tile_rows(const pevlm_heads *heads) { return check_heads(heads, nullptr) == PEVLM_OK ? tile_rows_of(heads, true) : -1; }

pevlm_status pevlm_rope_seq(void *q, void *k, const pevlm_layout *layout, const pevlm_heads *heads,
                            double rope_base, const int32_t *pos_offset, void *stream)
{
    pevlm_status st = check_layout(layout);
    if (st != PEVLM_OK) return st;
    st = check_heads(heads, nullptr);
    if (st != PEVLM_OK) return st;
    if (!(rope_base > 0.0)) return fail(PEVLM_ERR_INVALID_ARG, "rope_base must be positive");
    if ((q && !aligned16(q)) || (k && !aligned16(k))) return fail(PEVLM_ERR_INVALID_ARG, "q/k must be 16-byte aligned");
    if (layout->cu_seqlens[layout->num_seqs] == 0 || (!q && !k)) return PEVLM_OK;
    for (int32_t s0 = 0; s0 < layout->num_seqs; s0 += kMaxSeqsPerLaunch) {
        SeqTable tab;
        fill_table(layout, s0, std::min(kMaxSeqsPerLaunch, layout->num_seqs - s0), pos_offset, &tab);
        hipError_t e = launch_rope(q, k, tab, heads->n_q_heads, heads->n_kv_heads, heads->head_dim,
                                   heads->dtype == PEVLM_BF16, rope_base, nullptr, (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "rope launch");
    }
    return PEVLM_OK;
}

pevlm_status pevlm_rope_mrope(void *q, void *k, int64_t num_tokens, const pevlm_heads *heads, double rope_base,
                              const int32_t *pos_ids, const int32_t *section, void *stream)
{
    pevlm_status st = check_heads(heads, nullptr);
    if (st != PEVLM_OK) return st;
    if (!(rope_base > 0.0)) return fail(PEVLM_ERR_INVALID_ARG, "rope_base must be positive");
    if (num_tokens < 0 || num_tokens > 0x7fffffff) return fail(PEVLM_ERR_INVALID_ARG, "num_tokens out of range");
    if ((q && !aligned16(q)) || (k && !aligned16(k))) return fail(PEVLM_ERR_INVALID_ARG, "q/k must be 16-byte aligned");
    if (!section || section[0] < 0 || section[1] < 0 || section[2] < 0 ||
        (int64_t)section[0] + section[1] + section[2] != heads->head_dim / 2)
        return fail(PEVLM_ERR_INVALID_ARG, "section must hold three non-negative counts that add up to head_dim/2");
    if (num_tokens == 0 || (!q && !k)) return PEVLM_OK;
    if (!pos_ids || ((uintptr_t)pos_ids & 3)) return fail(PEVLM_ERR_INVALID_ARG, "pos_ids must be a 4-byte aligned device pointer");
    hipError_t e = launch_rope_mrope(q, k, num_tokens, heads->n_q_heads, heads->n_kv_heads, heads->head_dim,
                                     heads->dtype == PEVLM_BF16, rope_base, pos_ids, section[0], section[0] + section[1],
                                     nullptr, (hipStream_t)stream);
    return e == hipSuccess ? PEVLM_OK : hip_fail(e, "mrope launch");
}

static size_t prefill_workspace(const pevlm_layout *layout, const pevlm_heads *heads, bool fuse_rope)
{
    if (check_layout(layout) != PEVLM_OK || check_heads(heads, nullptr) != PEVLM_OK) return 0;
    size_t n = align256((size_t)count_prefill_items(layout, tile_rows_of(heads, false)) * sizeof(pevlm_work_item));
    if (fuse_rope) n += rope_table_bytes(layout->cu_seqlens[layout->num_seqs], heads);
    // the streaming kernel's list (plain calls on bf16 tensors) lives in the same workspace
    if (!fuse_rope && heads->dtype == PEVLM_BF16 && equal_head_groups(heads))
        n = std::max(n, align256((size_t)count_stream_items(layout, heads) * sizeof(pevlm_stream_item)));
    return n + 256;
}

size_t pevlm_block_prefill_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads)
{
    return prefill_workspace(layout, heads, false);
}

size_t pevlm_block_prefill_rope_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads)
{
    return prefill_workspace(layout, heads, true);
}

static pevlm_status prefill_impl(const void *q, const void *k, const void *v, void *out, float *lse,
                                 const pevlm_layout *layout, const pevlm_heads *heads, void *workspace,
                                 size_t workspace_bytes, void *stream, bool fuse_rope, double rope_base,
                                 const int32_t *pos_offset, bool rotate_k, const Restrict &sel = Restrict(),
                                 const Axes &ax = Axes())
{
    pevlm_status st = check_layout(layout);
    if (st != PEVLM_OK) return st;
    st = check_restrict(layout, sel);
    if (st != PEVLM_OK) return st;
    AttnParams p;
    memset(&p, 0, sizeof p);
    st = check_heads(heads, &p.heads);
    if (st != PEVLM_OK) return st;
    if (!q || !k || !v || !out) return fail(PEVLM_ERR_INVALID_ARG, "q, k, v and out must not be NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (lse && ((uintptr_t)lse & 3)))
        return fail(PEVLM_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (fuse_rope && heads->dtype != PEVLM_BF16)
        return fail(PEVLM_ERR_UNSUPPORTED, "the fused query rotation exists for bf16 tensors only");
    if (fuse_rope && !(rope_base > 0.0)) return fail(PEVLM_ERR_INVALID_ARG, "rope_base must be positive");
    int32_t tile_rows = tile_rows_of(heads, false);
    int64_t n_items = count_prefill_items(layout, tile_rows, sel);
    if (n_items == 0) {  // no sink or context rows: nothing to attend, but the keys are still rotated if asked
        if (fuse_rope && rotate_k && layout->cu_seqlens[layout->num_seqs] > 0) {
            if (!ax.pos_ids) return pevlm_rope_seq(nullptr, const_cast<void *>(k), layout, heads, rope_base, pos_offset, stream);
            hipError_t e = launch_rope_mrope(nullptr, const_cast<void *>(k), layout->cu_seqlens[layout->num_seqs], heads->n_q_heads,
                                             heads->n_kv_heads, heads->head_dim, true, rope_base, ax.pos_ids, ax.sec0, ax.sec01,
                                             nullptr, (hipStream_t)stream);
            return e == hipSuccess ? PEVLM_OK : hip_fail(e, "mrope launch");
        }
        return PEVLM_OK;
    }
    if (n_items * heads->n_q_heads > 0x3fffffff) return fail(PEVLM_ERR_UNSUPPORTED, "too many work items");
    const int64_t n_stream = stream_items_if_chosen(layout, heads, sel, fuse_rope);
    if (n_stream > 0) {
        // ---- streaming kernel: resident workgroups walk a list of stream items
        if (n_stream > 0x3fffffff) return fail(PEVLM_ERR_UNSUPPORTED, "too many work items");
        size_t need_s = prefill_workspace(layout, heads, false);
        if (!workspace || workspace_bytes < need_s || ((uintptr_t)workspace & 255))
            return fail(PEVLM_ERR_WORKSPACE_TOO_SMALL, "prefill workspace needs %zu bytes, 256-byte aligned (got %zu)", need_s,
                        workspace ? workspace_bytes : (size_t)0);
        hipStream_t hs = (hipStream_t)stream;
        pevlm_stream_item *sitems = (pevlm_stream_item *)workspace;
        const int32_t G = heads->n_q_heads / heads->n_kv_heads;
        int32_t offset = 0;
        for (int32_t s0 = 0; s0 < layout->num_seqs; s0 += kMaxSeqsPerLaunch) {
            SeqTable tab;
            int32_t n = std::min(kMaxSeqsPerLaunch, layout->num_seqs - s0);
            fill_table(layout, s0, n, pos_offset, &tab, sel);
            for (int32_t i = 0; i < n; ++i)
                tab.item_base[i + 1] = tab.item_base[i] + stream_items_of_seq(tab.sink[i], tab.block[i], tab.ctx[i], G, heads->n_kv_heads,
                                                                              tab.sel_first[i], tab.sel_count[i], tab.sel_sink);
            if (tab.item_base[n] > 0) {
                hipError_t e = launch_build_stream_items(tab, G, heads->n_kv_heads, p.heads, sitems, offset, hs);
                if (e != hipSuccess) return hip_fail(e, "stream-item builder launch");
            }
            offset += tab.item_base[n];
        }
        StreamParams sp;
        sp.q = q; sp.k = k; sp.v = v; sp.out = out; sp.lse = lse;
        sp.items = sitems;
        sp.n_items = (int32_t)n_stream;
        sp.n_q_heads = heads->n_q_heads;
        sp.n_kv_heads = heads->n_kv_heads;
        sp.scale = scale_of(heads);
        hipError_t e = launch_attn_bf16_stream(sp, heads->head_dim, compute_units(), hs);
        if (e != hipSuccess) return hip_fail(e, "block-prefill launch");
        return PEVLM_OK;
    }
    size_t need = prefill_workspace(layout, heads, fuse_rope);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))
        return fail(PEVLM_ERR_WORKSPACE_TOO_SMALL, "prefill workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
                    workspace ? workspace_bytes : (size_t)0);
    hipStream_t hs = (hipStream_t)stream;
    pevlm_work_item *items = (pevlm_work_item *)workspace;
    float *rope_tab = (float *)((char *)workspace + align256((size_t)n_items * sizeof(pevlm_work_item)));
    const int64_t T = layout->cu_seqlens[layout->num_seqs];
    if (fuse_rope && ax.pos_ids && rotate_k) {  // three-axis ids: one launch rotates K of all tokens and fills the table
        hipError_t e = launch_rope_mrope(nullptr, const_cast<void *>(k), T, heads->n_q_heads, heads->n_kv_heads, heads->head_dim,
                                         true, rope_base, ax.pos_ids, ax.sec0, ax.sec01, rope_tab, hs);
        if (e != hipSuccess) return hip_fail(e, "mrope launch");
    }
    int32_t offset = 0;
    for (int32_t s0 = 0; s0 < layout->num_seqs; s0 += kMaxSeqsPerLaunch) {
        SeqTable tab;
        int32_t n = std::min(kMaxSeqsPerLaunch, layout->num_seqs - s0);
        fill_table(layout, s0, n, pos_offset, &tab, sel);
        for (int32_t i = 0; i < n; ++i)
            tab.item_base[i + 1] = tab.item_base[i] + prefill_items_of_seq_sel(tab.sink[i], tab.block[i], tab.ctx[i], tile_rows,
                                                                               tab.sel_first[i], tab.sel_count[i], tab.sel_sink);
        if (tab.item_base[n] > 0) {
            hipError_t e = launch_build_prefill_items(tab, tile_rows, items, offset, hs);
            if (e != hipSuccess) return hip_fail(e, "work-list builder launch");
        }
        if (fuse_rope && !(ax.pos_ids && rotate_k)) {  // table entries = packed rows of this chunk's sequences
            hipError_t e = rotate_k ? launch_rope(nullptr, const_cast<void *>(k), tab, heads->n_q_heads, heads->n_kv_heads,
                                                  heads->head_dim, true, rope_base, rope_tab, hs)
                                    : launch_rope_table(rope_tab, nullptr, tab, heads->head_dim, rope_base,
                                                        layout->cu_seqlens[s0], layout->cu_seqlens[s0 + n], ax.pos_ids, T,
                                                        ax.sec0, ax.sec01, hs);
            if (e != hipSuccess) return hip_fail(e, "rope table launch");
        }
        offset += tab.item_base[n];
    }
    p.q = q; p.k = k; p.v = v; p.out = out; p.lse = lse;
    p.rope_tab = fuse_rope ? rope_tab : nullptr;
    p.rope_compact_rows = 0;
    p.items = items;
    p.n_items = (int32_t)n_items;
    p.n_q_heads = heads->n_q_heads;
    p.n_kv_heads = heads->n_kv_heads;
    p.scale = scale_of(heads);
    hipError_t e = heads->dtype == PEVLM_BF16 ? launch_attn_bf16(p, heads->head_dim, false, hs)
                                                : launch_attn_f32(p, heads->head_dim, false, hs);
    if (e != hipSuccess) return hip_fail(e, "block-prefill launch");
    return PEVLM_OK;
}

pevlm_status pevlm_block_prefill_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                                      const pevlm_layout *layout, const pevlm_heads *heads, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    return prefill_impl(q, k, v, out, lse, layout, heads, workspace, workspace_bytes, stream, false, 0.0, nullptr, false);
}

pevlm_status pevlm_block_prefill_attn_blocks(const void *q, const void *k, const void *v, void *out, float *lse,
                                             const pevlm_layout *layout, const pevlm_heads *heads, const int32_t *first_block,
                                             const int32_t *num_blocks, int32_t with_sink, void *workspace,
                                             size_t workspace_bytes, void *stream)
{
    if (!first_block || !num_blocks) return fail(PEVLM_ERR_INVALID_ARG, "first_block and num_blocks must not be NULL");
    Restrict sel;
    sel.first_block = first_block;
    sel.num_blocks = num_blocks;
    sel.with_sink = with_sink;
    return prefill_impl(q, k, v, out, lse, layout, heads, workspace, workspace_bytes, stream, false, 0.0, nullptr, false, sel);
}

pevlm_status pevlm_block_prefill_attn_rope(const void *q, void *k, const void *v, void *out, float *lse,
                                           const pevlm_layout *layout, const pevlm_heads *heads, double rope_base,
                                           const int32_t *pos_offset, int32_t k_is_rotated, void *workspace,
                                           size_t workspace_bytes, void *stream)
{
    return prefill_impl(q, k, v, out, lse, layout, heads, workspace, workspace_bytes, stream, true, rope_base, pos_offset,
                        k_is_rotated == 0);
}

// ---- fp8 variant of the block-prefill call
static pevlm_status fp8_plan(const pevlm_layout *layout, const pevlm_heads *heads, pevlm_fp8_plan *plan)
{
    pevlm_status st = check_layout(layout);
    if (st != PEVLM_OK) return st;
    st = check_heads(heads, nullptr);
    if (st != PEVLM_OK) return st;
    if (heads->dtype != PEVLM_BF16) return fail(PEVLM_ERR_UNSUPPORTED, "the fp8 variant takes bf16 tensors");
    const int64_t T = layout->cu_seqlens[layout->num_seqs];
    const int64_t n_items = count_prefill_items(layout, kFp8TileRows), n_key_tiles = count_prefill_items(layout, kKeyTile);
    if (n_items * heads->n_q_heads > 0x3fffffff || n_key_tiles > 0x3fffffff) return fail(PEVLM_ERR_UNSUPPORTED, "too many work items");
    const size_t tile_bytes = (size_t)kKeyTile * heads->head_dim;
    size_t off = 0;
    plan->n_items = n_items;
    plan->n_key_tiles = n_key_tiles;
    plan->items = off;     off += align256((size_t)n_items * sizeof(Fp8Item));
    plan->key_tiles = off; off += align256((size_t)n_key_tiles * sizeof(pevlm_work_item));
    plan->kv_amax = off;   off += align256((size_t)2 * heads->n_kv_heads * sizeof(uint32_t));
    plan->q_scales = off;  off += align256((size_t)T * heads->n_q_heads * sizeof(float));
    plan->q_codes = off;   off += align256((size_t)T * heads->n_q_heads * heads->head_dim);
    plan->k_tiles = off;   off += align256((size_t)n_key_tiles * heads->n_kv_heads * tile_bytes);
    plan->v_tiles = off;   off += align256((size_t)n_key_tiles * heads->n_kv_heads * tile_bytes);
    plan->total = off + 256;
    return PEVLM_OK;
}

pevlm_status pevlm_block_prefill_fp8_plan(const pevlm_layout *layout, const pevlm_heads *heads, pevlm_fp8_plan *plan)
{
    if (!plan) return fail(PEVLM_ERR_INVALID_ARG, "plan must not be NULL");
    return fp8_plan(layout, heads, plan);
}

size_t pevlm_block_prefill_fp8_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads)
{
    pevlm_fp8_plan plan;
    return fp8_plan(layout, heads, &plan) == PEVLM_OK ? plan.total : 0;
}

pevlm_status pevlm_block_prefill_attn_fp8(const void *q, const void *k, const void *v, void *out, float *lse,
                                          const pevlm_layout *layout, const pevlm_heads *heads, void *workspace,
                                          size_t workspace_bytes, int32_t stages, void *stream)
{
    pevlm_fp8_plan plan;
    pevlm_status st = fp8_plan(layout, heads, &plan);
    if (st != PEVLM_OK) return st;
    Fp8Params p;
    memset(&p, 0, sizeof p);
    st = check_heads(heads, &p.heads);
    if (st != PEVLM_OK) return st;
    if (stages == 0) stages = PEVLM_FP8_QUANTISE | PEVLM_FP8_ATTEND;
    if (stages & ~(PEVLM_FP8_QUANTISE | PEVLM_FP8_ATTEND)) return fail(PEVLM_ERR_INVALID_ARG, "unknown stage bits %d", stages);
    if (!q || !k || !v || !out) return fail(PEVLM_ERR_INVALID_ARG, "q, k, v and out must not be NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (lse && ((uintptr_t)lse & 3)))
        return fail(PEVLM_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (plan.n_items == 0) return PEVLM_OK;
    if (!workspace || workspace_bytes < plan.total - 256 || ((uintptr_t)workspace & 255))
        return fail(PEVLM_ERR_WORKSPACE_TOO_SMALL, "fp8 prefill workspace needs %zu bytes, 256-byte aligned (got %zu)", plan.total,
                    workspace ? workspace_bytes : (size_t)0);
    hipStream_t hs = (hipStream_t)stream;
    char *ws = (char *)workspace;
    Fp8Item *items = (Fp8Item *)(ws + plan.items);
    pevlm_work_item *key_tiles = (pevlm_work_item *)(ws + plan.key_tiles);
    const int64_t T = layout->cu_seqlens[layout->num_seqs];
    if (stages & PEVLM_FP8_QUANTISE) {
        // both lists (they depend on the layout only), then the codes
        int32_t item_offset = 0, tile_offset = 0;
        for (int32_t s0 = 0; s0 < layout->num_seqs; s0 += kMaxSeqsPerLaunch) {
            SeqTable tab;
            Fp8TileBases bases;
            const int32_t n = std::min(kMaxSeqsPerLaunch, layout->num_seqs - s0);
            fill_table(layout, s0, n, nullptr, &tab);
            bases.base[0] = tile_offset;
            for (int32_t i = 0; i < n; ++i) {
                tab.item_base[i + 1] = tab.item_base[i] + prefill_items_of_seq(tab.sink[i], tab.block[i], tab.ctx[i], kKeyTile);
                bases.base[i + 1] = tile_offset + tab.item_base[i + 1];
            }
            if (tab.item_base[n] > 0) {
                hipError_t e = launch_build_prefill_items(tab, kKeyTile, key_tiles, tile_offset, hs);
                if (e != hipSuccess) return hip_fail(e, "key-tile list launch");
            }
            tile_offset += tab.item_base[n];
            for (int32_t i = 0; i < n; ++i)
                tab.item_base[i + 1] = tab.item_base[i] + prefill_items_of_seq(tab.sink[i], tab.block[i], tab.ctx[i], kFp8TileRows);
            if (tab.item_base[n] > 0) {
                hipError_t e = launch_build_fp8_items(tab, bases, items, item_offset, hs);
                if (e != hipSuccess) return hip_fail(e, "fp8 work-list launch");
            }
            item_offset += tab.item_base[n];
        }
        hipError_t e = launch_fp8_quantise(q, k, v, T, heads->n_q_heads, heads->n_kv_heads, heads->head_dim,
                                           scale_of(heads) * 1.4426950408889634f, key_tiles,
                                           (int32_t)plan.n_key_tiles, (uint32_t *)(ws + plan.kv_amax), (float *)(ws + plan.q_scales),
                                           (uint8_t *)(ws + plan.q_codes), (uint8_t *)(ws + plan.k_tiles),
                                           (uint8_t *)(ws + plan.v_tiles), compute_units(), hs);
        if (e != hipSuccess) return hip_fail(e, "fp8 quantise launch");
    }
    if (stages & PEVLM_FP8_ATTEND) {
        p.q_codes = (const uint8_t *)(ws + plan.q_codes);
        p.q_scales = (const float *)(ws + plan.q_scales);
        p.k_tiles = (const uint8_t *)(ws + plan.k_tiles);
        p.v_tiles = (const uint8_t *)(ws + plan.v_tiles);
        p.kv_amax = (const uint32_t *)(ws + plan.kv_amax);
        p.out = out;
        p.lse = lse;
        p.items = items;
        p.n_items = (int32_t)plan.n_items;
        p.n_q_heads = heads->n_q_heads;
        p.n_kv_heads = heads->n_kv_heads;
        p.scale = scale_of(heads);
        hipError_t e = launch_attn_fp8(p, heads->head_dim, hs);
        if (e != hipSuccess) return hip_fail(e, "fp8 block-prefill launch");
    }
    return PEVLM_OK;
}

size_t pevlm_query_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits)
{
    if (check_layout(layout) != PEVLM_OK || check_heads(heads, nullptr) != PEVLM_OK) return 0;
    if (num_splits < 0 || num_splits > PEVLM_MAX_SPLITS) return 0;
    return plan_query(layout, heads, num_splits).bytes + 256;
}

size_t pevlm_query_rope_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits)
{
    if (check_layout(layout) != PEVLM_OK || check_heads(heads, nullptr) != PEVLM_OK) return 0;
    if (num_splits < 0 || num_splits > PEVLM_MAX_SPLITS) return 0;
    return plan_query(layout, heads, num_splits, true).bytes + 256;
}

static pevlm_status query_impl(const void *q, const void *k, const void *v, void *out, float *lse,
                               const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits,
                               void *workspace, size_t workspace_bytes, void *stream, bool fuse_rope, double rope_base,
                               const int32_t *pos_offset, const Restrict &sel = Restrict(), const Axes &ax = Axes())
{
    pevlm_status st = check_layout(layout);
    if (st != PEVLM_OK) return st;
    AttnParams p;
    memset(&p, 0, sizeof p);
    st = check_heads(heads, &p.heads);
    if (st != PEVLM_OK) return st;
    if (num_splits < 0 || num_splits > PEVLM_MAX_SPLITS)
        return fail(PEVLM_ERR_INVALID_ARG, "num_splits must be in [0, %d]", PEVLM_MAX_SPLITS);
    if (!q || !k || !v || !out) return fail(PEVLM_ERR_INVALID_ARG, "q, k, v and out must not be NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (lse && ((uintptr_t)lse & 3)))
        return fail(PEVLM_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (fuse_rope && heads->dtype != PEVLM_BF16)
        return fail(PEVLM_ERR_UNSUPPORTED, "the fused query rotation exists for bf16 tensors only");
    if (fuse_rope && !(rope_base > 0.0)) return fail(PEVLM_ERR_INVALID_ARG, "rope_base must be positive");
    QueryPlan plan = plan_query(layout, heads, num_splits, fuse_rope, sel.window_blocks != nullptr);
    if (plan.total_q == 0) return PEVLM_OK;
    if (plan.n_items * heads->n_q_heads > 0x3fffffff) return fail(PEVLM_ERR_UNSUPPORTED, "too many work items");
    if (!workspace || workspace_bytes < plan.bytes || ((uintptr_t)workspace & 255))
        return fail(PEVLM_ERR_WORKSPACE_TOO_SMALL, "query workspace needs %zu bytes, 256-byte aligned (got %zu)",
                    plan.bytes + 256, workspace ? workspace_bytes : (size_t)0);
    hipStream_t hs = (hipStream_t)stream;
    char *ws = (char *)workspace;
    pevlm_work_item *items = (pevlm_work_item *)(ws + plan.off_items);
    int32_t *qrow = (int32_t *)(ws + plan.off_qrow);
    float *ml = (float *)(ws + plan.off_ml);
    float *acc = (float *)(ws + plan.off_acc);
    float *rope_tab = (float *)(ws + plan.off_rope);
    int32_t item_offset = 0, qrow_base = 0;
    for (int32_t s0 = 0; s0 < layout->num_seqs; s0 += kMaxSeqsPerLaunch) {
        SeqTable tab;
        int32_t n = std::min(kMaxSeqsPerLaunch, layout->num_seqs - s0);
        fill_table(layout, s0, n, pos_offset, &tab, sel);
        const int32_t entry_begin = qrow_base;
        for (int32_t i = 0; i < n; ++i) {
            tab.item_base[i + 1] = tab.item_base[i] + query_tiles_of_seq(tab.query[i], plan.tile_rows) * plan.num_splits;
            tab.qrow_base[i] = qrow_base;
            qrow_base += tab.query[i];
        }
        if (tab.item_base[n] > 0) {
            hipError_t e = launch_build_query_items(tab, plan.tile_rows, plan.num_splits, (int32_t)plan.total_q,
                                                    kKeyTile, items, item_offset, qrow, hs);
            if (e != hipSuccess) return hip_fail(e, "query work-list builder launch");
            if (fuse_rope) {  // table entries = compact question rows of this chunk (mapped through qrow)
                e = launch_rope_table(rope_tab, qrow, tab, heads->head_dim, rope_base, entry_begin, qrow_base, ax.pos_ids,
                                      layout->cu_seqlens[layout->num_seqs], ax.sec0, ax.sec01, hs);
                if (e != hipSuccess) return hip_fail(e, "rope table launch");
            }
        }
        item_offset += tab.item_base[n];
    }
    p.q = q; p.k = k; p.v = v;
    p.rope_tab = fuse_rope ? rope_tab : nullptr;
    p.rope_compact_rows = fuse_rope ? (int32_t)plan.total_q : 0;
    p.part_acc = acc;
    p.part_ml = ml;
    p.items = items;
    p.n_items = (int32_t)plan.n_items;
    p.n_q_heads = heads->n_q_heads;
    p.n_kv_heads = heads->n_kv_heads;
    p.scale = scale_of(heads);
    hipError_t e = heads->dtype == PEVLM_BF16 ? launch_attn_bf16(p, heads->head_dim, true, hs)
                                              : launch_attn_f32(p, heads->head_dim, true, hs);
    if (e != hipSuccess) return hip_fail(e, "query split launch");
    MergeParams m;
    m.part_acc = acc; m.part_ml = ml; m.qrow_of_compact = qrow; m.out = out; m.lse = lse;
    m.total_q_rows = (int32_t)plan.total_q;
    m.num_splits = plan.num_splits;
    m.n_q_heads = heads->n_q_heads;
    m.head_dim = heads->head_dim;
    m.scale = p.scale;
    m.is_bf16 = heads->dtype == PEVLM_BF16;
    e = launch_merge(m, hs);
    if (e != hipSuccess) return hip_fail(e, "merge launch");
    return PEVLM_OK;
}

pevlm_status pevlm_query_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                              const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return query_impl(q, k, v, out, lse, layout, heads, num_splits, workspace, workspace_bytes, stream, false, 0.0, nullptr);
}

pevlm_status pevlm_query_attn_static(const void *q, const void *k, const void *v, void *out, float *lse,
                                     const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits, void *stream)
{
    // validate sizes before touching the device: the plan is what pevlm_query_attn would carve
    pevlm_status st = check_layout(layout);
    if (st != PEVLM_OK) return st;
    st = check_heads(heads, nullptr);
    if (st != PEVLM_OK) return st;
    if (num_splits < 0 || num_splits > PEVLM_MAX_SPLITS)
        return fail(PEVLM_ERR_INVALID_ARG, "num_splits must be in [0, %d]", PEVLM_MAX_SPLITS);
    const QueryPlan plan = plan_query(layout, heads, num_splits);
    if (plan.bytes > (size_t)PEVLM_STATIC_SCRATCH_BYTES)
        return fail(PEVLM_ERR_WORKSPACE_TOO_SMALL,
                    "pevlm_query_attn_static: this call needs %zu bytes of scratch, the built-in array holds %zu "
                    "(use pevlm_query_attn with a caller workspace, or fewer splits)",
                    plan.bytes, (size_t)PEVLM_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    st = scratch_of_current_device(&ws);
    if (st != PEVLM_OK) return st;
    // Every field of the scratch a launch reads (work list, row map, partials of every split, row
    // and head) is written earlier in the same call on the same stream, so nothing needs clearing.
    return query_impl(q, k, v, out, lse, layout, heads, num_splits, ws, PEVLM_STATIC_SCRATCH_BYTES, stream, false, 0.0, nullptr);
}

pevlm_status pevlm_block_prefill_attn_mrope(const void *q, void *k, const void *v, void *out, float *lse,
                                            const pevlm_layout *layout, const pevlm_heads *heads, double rope_base,
                                            const int32_t *pos_ids, const int32_t *section, int32_t k_is_rotated,
                                            void *workspace, size_t workspace_bytes, void *stream)
{
    pevlm_status st = check_heads(heads, nullptr);
    if (st != PEVLM_OK) return st;
    Axes ax;
    st = check_axes(heads, pos_ids, section, &ax);
    if (st != PEVLM_OK) return st;
    return prefill_impl(q, k, v, out, lse, layout, heads, workspace, workspace_bytes, stream, true, rope_base, nullptr,
                        k_is_rotated == 0, Restrict(), ax);
}

pevlm_status pevlm_query_attn_mrope(const void *q, const void *k, const void *v, void *out, float *lse,
                                    const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits, double rope_base,
                                    const int32_t *pos_ids, const int32_t *section, void *workspace, size_t workspace_bytes,
                                    void *stream)
{
    pevlm_status st = check_heads(heads, nullptr);
    if (st != PEVLM_OK) return st;
    Axes ax;
    st = check_axes(heads, pos_ids, section, &ax);
    if (st != PEVLM_OK) return st;
    return query_impl(q, k, v, out, lse, layout, heads, num_splits, workspace, workspace_bytes, stream, true, rope_base, nullptr,
                      Restrict(), ax);
}

size_t pevlm_query_window_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits)
{
    if (check_layout(layout) != PEVLM_OK || check_heads(heads, nullptr) != PEVLM_OK) return 0;
    if (num_splits < 0 || num_splits > PEVLM_MAX_SPLITS) return 0;
    return plan_query(layout, heads, num_splits, false, true).bytes + 256;
}

pevlm_status pevlm_query_attn_window(const void *q, const void *k, const void *v, void *out, float *lse,
                                     const pevlm_layout *layout, const pevlm_heads *heads, const int32_t *window_blocks,
                                     int32_t num_splits, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!window_blocks) return fail(PEVLM_ERR_INVALID_ARG, "window_blocks must not be NULL");
    Restrict sel;
    sel.window_blocks = window_blocks;
    return query_impl(q, k, v, out, lse, layout, heads, num_splits, workspace, workspace_bytes, stream, false, 0.0, nullptr, sel);
}

pevlm_status pevlm_query_attn_rope(const void *q, const void *k, const void *v, void *out, float *lse,
                                   const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits, double rope_base,
                                   const int32_t *pos_offset, void *workspace, size_t workspace_bytes, void *stream)
{
    return query_impl(q, k, v, out, lse, layout, heads, num_splits, workspace, workspace_bytes, stream, true, rope_base,
                      pos_offset);
}

int64_t pevlm_prefill_worklist_host(const pevlm_layout *layout, int32_t tile_rows, pevlm_work_item *items,
                                    int64_t capacity)
{
    if (check_layout(layout) != PEVLM_OK) return -1;
    if (tile_rows < 1) { fail(PEVLM_ERR_INVALID_ARG, "tile_rows must be >= 1"); return -1; }
    int64_t n = 0;
    for (int32_t s = 0; s < layout->num_seqs; ++s) {
        int32_t B = layout->ctx_len[s] > 0 ? layout->block_len[s] : 1;
        int32_t cnt = prefill_items_of_seq(layout->sink_len[s], B, layout->ctx_len[s], tile_rows);
        for (int32_t i = 0; i < cnt; ++i, ++n)
            if (items && n < capacity)
                items[n] = prefill_item(layout->cu_seqlens[s], layout->sink_len[s], B, layout->ctx_len[s], tile_rows, i, s);
    }
    return n;
}

int64_t pevlm_query_worklist_host(const pevlm_layout *layout, int32_t tile_rows, int32_t num_splits,
                                  pevlm_work_item *items, int64_t capacity)
{
    if (check_layout(layout) != PEVLM_OK) return -1;
    if (tile_rows < 1 || num_splits < 1) { fail(PEVLM_ERR_INVALID_ARG, "tile_rows and num_splits must be >= 1"); return -1; }
    int64_t total_q = total_query_rows(layout);
    int64_t n = 0;
    int32_t qrow_base = 0;
    for (int32_t s = 0; s < layout->num_seqs; ++s) {
        int32_t cnt = query_tiles_of_seq(layout->query_len[s], tile_rows) * num_splits;
        for (int32_t i = 0; i < cnt; ++i, ++n)
            if (items && n < capacity)
                items[n] = query_item(layout->cu_seqlens[s], layout->sink_len[s], layout->ctx_len[s], layout->query_len[s],
                                      tile_rows, num_splits, i, s, qrow_base, (int32_t)total_q, kKeyTile);
        qrow_base += layout->query_len[s];
    }
    return n;
}

int64_t pevlm_prefill_worklist_blocks_host(const pevlm_layout *layout, int32_t tile_rows, const int32_t *first_block,
                                           const int32_t *num_blocks, int32_t with_sink, pevlm_work_item *items,
                                           int64_t capacity)
{
    if (check_layout(layout) != PEVLM_OK) return -1;
    if (tile_rows < 1) { fail(PEVLM_ERR_INVALID_ARG, "tile_rows must be >= 1"); return -1; }
    Restrict sel;
    sel.first_block = first_block;
    sel.num_blocks = num_blocks;
    sel.with_sink = with_sink;
    if (!first_block || !num_blocks || check_restrict(layout, sel) != PEVLM_OK) {
        if (!first_block || !num_blocks) fail(PEVLM_ERR_INVALID_ARG, "first_block and num_blocks must not be NULL");
        return -1;
    }
    int64_t n = 0;
    for (int32_t s = 0; s < layout->num_seqs; ++s) {
        int32_t B = layout->ctx_len[s] > 0 ? layout->block_len[s] : 1;
        int32_t cnt = prefill_items_of_seq_sel(layout->sink_len[s], B, layout->ctx_len[s], tile_rows, first_block[s],
                                               num_blocks[s], with_sink);
        for (int32_t i = 0; i < cnt; ++i, ++n)
            if (items && n < capacity)
                items[n] = prefill_item_sel(layout->cu_seqlens[s], layout->sink_len[s], B, layout->ctx_len[s], tile_rows,
                                            first_block[s], with_sink, i, s);
    }
    return n;
}

int32_t pevlm_prefill_uses_stream_kernel(const pevlm_layout *layout, const pevlm_heads *heads)
{
    if (check_layout(layout) != PEVLM_OK || check_heads(heads, nullptr) != PEVLM_OK) return 0;
    return stream_items_if_chosen(layout, heads, Restrict(), false) > 0 ? 1 : 0;
}

int32_t pevlm_set_prefill_kernel(int32_t mode)
{
    if (mode < 0 || mode > 2) return -1;
    return prefill_kernel_mode().exchange(mode);
}

int64_t pevlm_prefill_stream_items_host(const pevlm_layout *layout, const pevlm_heads *heads, const int32_t *first_block,
                                        const int32_t *num_blocks, int32_t with_sink, pevlm_stream_item *items,
                                        int64_t capacity)
{
    if (check_layout(layout) != PEVLM_OK) return -1;
    HeadTable ht;
    if (check_heads(heads, &ht) != PEVLM_OK) return -1;
    if (!equal_head_groups(heads)) { fail(PEVLM_ERR_UNSUPPORTED, "query heads are not in equal groups per KV head"); return -1; }
    Restrict sel;
    sel.first_block = first_block;
    sel.num_blocks = num_blocks;
    sel.with_sink = first_block ? with_sink : 1;
    if (check_restrict(layout, sel) != PEVLM_OK) return -1;
    const int32_t G = heads->n_q_heads / heads->n_kv_heads;
    int64_t n = 0;
    for (int32_t s = 0; s < layout->num_seqs; ++s) {
        int32_t B = layout->ctx_len[s] > 0 ? layout->block_len[s] : 1;
        int32_t first = first_block ? first_block[s] : 0;
        int32_t cnt = stream_items_of_seq(layout->sink_len[s], B, layout->ctx_len[s], G, heads->n_kv_heads, first,
                                          num_blocks ? num_blocks[s] : blocks_of(layout, s), sel.with_sink);
        for (int32_t i = 0; i < cnt; ++i, ++n)
            if (items && n < capacity)
                items[n] = stream_item(layout->cu_seqlens[s], layout->sink_len[s], B, layout->ctx_len[s], G, heads->n_kv_heads, first,
                                       sel.with_sink, i, s, ht.head_order);
    }
    return n;
}

int64_t pevlm_query_worklist_window_host(const pevlm_layout *layout, int32_t tile_rows, int32_t num_splits,
                                         const int32_t *window_blocks, pevlm_work_item *items, int64_t capacity)
{
    if (check_layout(layout) != PEVLM_OK) return -1;
    if (tile_rows < 1 || num_splits < 2 || !window_blocks) {
        fail(PEVLM_ERR_INVALID_ARG, "tile_rows >= 1, num_splits >= 2 and window_blocks are required");
        return -1;
    }
    Restrict sel;
    sel.window_blocks = window_blocks;
    int64_t total_q = total_query_rows(layout);
    int64_t n = 0;
    int32_t qrow_base = 0;
    for (int32_t s = 0; s < layout->num_seqs; ++s) {
        SeqTable tab;
        fill_table(layout, s, 1, nullptr, &tab, sel);
        int32_t cnt = query_tiles_of_seq(layout->query_len[s], tile_rows) * num_splits;
        for (int32_t i = 0; i < cnt; ++i, ++n)
            if (items && n < capacity)
                items[n] = query_item_window(layout->cu_seqlens[s], layout->sink_len[s], layout->ctx_len[s],
                                             layout->query_len[s], tile_rows, num_splits, i, s, qrow_base, (int32_t)total_q,
                                             kKeyTile, tab.win_start[0]);
        qrow_base += layout->query_len[s];
    }
    return n;
}

pevlm_status pevlm_visible_pairs(const pevlm_layout *layout, int64_t *sink_pairs, int64_t *block_pairs,
                                 int64_t *question_pairs)
{
    pevlm_status st = check_layout(layout);
    if (st != PEVLM_OK) return st;
    int64_t ps = 0, pb = 0, pq = 0;
    for (int32_t s = 0; s < layout->num_seqs; ++s) {
        int64_t S = layout->sink_len[s], C = layout->ctx_len[s], Q = layout->query_len[s];
        int64_t B = C > 0 ? layout->block_len[s] : 1;
        ps += S * (S + 1) / 2;
        int64_t nfull = C / B, last = C % B;
        pb += nfull * (B * S + B * (B + 1) / 2) + (last ? last * S + last * (last + 1) / 2 : 0);
        pq += Q * (S + C) + Q * (Q + 1) / 2;
    }
    if (sink_pairs) *sink_pairs = ps;
    if (block_pairs) *block_pairs = pb;
    if (question_pairs) *question_pairs = pq;
    return PEVLM_OK;
}

pevlm_status pevlm_probe_mfma_bf16(void *scratch, int32_t workgroups, int32_t iters, double *flop_count, void *stream)
{
    if (!scratch || ((uintptr_t)scratch & 3)) return fail(PEVLM_ERR_INVALID_ARG, "pevlm_probe_mfma_bf16: scratch must be a 4-byte aligned device pointer");
    if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24))
        return fail(PEVLM_ERR_INVALID_ARG, "pevlm_probe_mfma_bf16: workgroups in [1, 2^20], iters in [1, 2^24]");
    if (flop_count) *flop_count = (double)workgroups * 4.0 * (double)iters * 4.0 * 32768.0;
    hipError_t e = launch_probe_mfma((float *)scratch, workgroups, iters, (hipStream_t)stream);
    return e == hipSuccess ? PEVLM_OK : hip_fail(e, "probe_mfma_kernel launch");
}

pevlm_status pevlm_probe_tile_loop_bf16(void *scratch, const void *kv, size_t kv_bytes, int32_t workgroups, int32_t iters,
                                        int32_t with_softmax, double *flop_count, void *stream)
{
    const size_t tile = (size_t)kKeyTile * 128 * 2;
    if (!scratch || !kv || !aligned16(kv) || kv_bytes < 4 * tile || kv_bytes / tile > 0x7fffffff || workgroups < 1 || iters < 1)
        return fail(PEVLM_ERR_INVALID_ARG, "tile-loop probe needs scratch, a 16-byte aligned buffer of at least 4 tiles of 16 KiB, workgroups >= 1, iters >= 1");
    if (flop_count) *flop_count = (double)workgroups * 4 * iters * 32 * 32768.0;
    hipError_t e = launch_probe_tile_loop((float *)scratch, kv, (int32_t)(kv_bytes / tile), workgroups, iters, with_softmax != 0,
                                          (hipStream_t)stream);
    return e == hipSuccess ? PEVLM_OK : hip_fail(e, "tile-loop probe launch");
}

pevlm_status pevlm_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15) || bytes == 0 || (bytes & 15) || bytes > ((size_t)1 << 40))
        return fail(PEVLM_ERR_INVALID_ARG, "pevlm_probe_copy: 16-byte aligned device pointers and a positive multiple of 16 bytes");
    hipError_t e = launch_probe_copy(dst, src, (int64_t)bytes, (hipStream_t)stream);
    return e == hipSuccess ? PEVLM_OK : hip_fail(e, "probe_copy_kernel launch");
}

}  // extern "C"
