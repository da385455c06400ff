// Internal declarations shared by the host entry points and the gfx950 kernels of libpevlm.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pevlm.h"

namespace pevlm {

// ------------------------------------------------------------------------------------------
// Sequence table handed to the work-list builder kernels by value (kernel argument memory), so
// that the caller's host arrays may be released as soon as the entry point returns.
// ------------------------------------------------------------------------------------------
constexpr int kMaxSeqsPerLaunch = 48;
constexpr int kMaxHeads = 256;

struct SeqTable {
    int32_t num_seqs;                          // sequences in this chunk
    int32_t seq_index0;                        // index of the chunk's first sequence in the batch
    int32_t start[kMaxSeqsPerLaunch];          // first packed row of the sequence
    int32_t sink[kMaxSeqsPerLaunch];           // S
    int32_t block[kMaxSeqsPerLaunch];          // B (>= 1)
    int32_t ctx[kMaxSeqsPerLaunch];            // C
    int32_t query[kMaxSeqsPerLaunch];          // Q
    int32_t item_base[kMaxSeqsPerLaunch + 1];  // first work item of the sequence (chunk-relative)
    int32_t qrow_base[kMaxSeqsPerLaunch];      // first compact question row of the sequence
    int32_t pos_offset[kMaxSeqsPerLaunch];     // added to every position of the sequence (RoPE)
    // streaming use: the prefill call may be restricted to context blocks [sel_first, sel_first +
    // sel_count) (plus the sink rows when sel_sink != 0); the question call may hide the context
    // before local position win_start (== S: nothing hidden) and then gives the sink its own split
    int32_t sel_first[kMaxSeqsPerLaunch];
    int32_t sel_count[kMaxSeqsPerLaunch];
    int32_t win_start[kMaxSeqsPerLaunch];
    int32_t sel_sink;
    int32_t windowed;
};

struct HeadTable {
    uint8_t kv_of_q[kMaxHeads];     // KV head of query head h
    uint8_t head_order[kMaxHeads];  // query heads sorted by KV head (stable): schedule order
};

// Work items of a region tiling (Sec. "Formulations": a query tile never leaves its region).
__host__ __device__ inline int32_t ceil_div(int32_t a, int32_t b) { return (a + b - 1) / b; }

__host__ __device__ inline int32_t prefill_items_of_seq(int32_t S, int32_t B, int32_t C, int32_t tile_rows)
{
    int32_t n = ceil_div(S, tile_rows);
    if (C > 0) {
        int32_t nb = ceil_div(C, B);
        int32_t last = C - (nb - 1) * B;
        n += (nb - 1) * ceil_div(B, tile_rows) + ceil_div(last, tile_rows);
    }
    return n;
}

// idx-th prefill item of a sequence that starts at packed row `start`.
__host__ __device__ inline pevlm_work_item prefill_item(int32_t start, int32_t S, int32_t B, int32_t C,
                                                        int32_t tile_rows, int32_t idx, int32_t seq)
{
    pevlm_work_item it;
    it.seq = seq;
    it.reserved = 0;
    int32_t sink_tiles = ceil_div(S, tile_rows);
    if (idx < sink_tiles) {  // Eq. 3: sink rows see sink keys up to themselves
        int32_t r0 = idx * tile_rows;
        it.q_start = start + r0;
        it.q_rows = (S - r0 < tile_rows) ? S - r0 : tile_rows;
        it.full_start = start;
        it.full_len = 0;
        it.diag_start = start;
        it.diag_len = r0 + it.q_rows;
        return it;
    }
    // Eq. 4: a context block sees the whole sink and itself up to the diagonal
    int32_t j = idx - sink_tiles;
    int32_t tiles_per_block = ceil_div(B, tile_rows);
    int32_t b = j / tiles_per_block, ti = j % tiles_per_block;
    int32_t b0 = S + b * B;                       // local position of the block's first token
    int32_t blen = (C - b * B < B) ? C - b * B : B;
    int32_t r0 = ti * tile_rows;
    it.q_start = start + b0 + r0;
    it.q_rows = (blen - r0 < tile_rows) ? blen - r0 : tile_rows;
    it.full_start = start;
    it.full_len = S;
    it.diag_start = start + b0;
    it.diag_len = r0 + it.q_rows;
    return it;
}

// Restriction of the prefill items of a sequence to its sink tiles (if with_sink) and the tiles of
// context blocks [first, first + count): what a streaming caller computes when new blocks arrive.
__host__ __device__ inline int32_t prefill_items_of_seq_sel(int32_t S, int32_t B, int32_t C, int32_t tile_rows,
                                                            int32_t first, int32_t count, int32_t with_sink)
{
    int32_t n = with_sink ? ceil_div(S, tile_rows) : 0;
    if (C > 0 && count > 0) {
        int32_t nb = ceil_div(C, B);
        int32_t last = C - (nb - 1) * B;
        int32_t full = (first + count == nb) ? count - 1 : count;  // selected blocks of B rows
        n += full * ceil_div(B, tile_rows);
        if (first + count == nb) n += ceil_div(last, tile_rows);
    }
    return n;
}

__host__ __device__ inline pevlm_work_item prefill_item_sel(int32_t start, int32_t S, int32_t B, int32_t C, int32_t tile_rows,
                                                            int32_t first, int32_t with_sink, int32_t idx, int32_t seq)
{
    int32_t sink_tiles = ceil_div(S, tile_rows);
    int32_t n_sink_sel = with_sink ? sink_tiles : 0;
    int32_t full_idx = idx < n_sink_sel ? idx : sink_tiles + first * ceil_div(B, tile_rows) + (idx - n_sink_sel);
    return prefill_item(start, S, B, C, tile_rows, full_idx, seq);
}

// ------------------------------------------------------------------------------------------
// Stream items of the block-prefill call (bf16 streaming kernel): a region of R rows is cut into
// ceil(R/32) row groups; the slots (row group, head of the KV group), head fastest, are dealt out 8 at
// a time.  Order inside a sequence: region (sink, then the selected blocks), then KV head, then item.
// ------------------------------------------------------------------------------------------
constexpr int32_t kSlotRows = 32;
constexpr int32_t kSlotsPerItem = 8;

__host__ __device__ inline int32_t stream_items_of_region(int32_t R, int32_t G)
{
    return R > 0 ? ceil_div(G * ceil_div(R, kSlotRows), kSlotsPerItem) : 0;
}

// Items of one sequence restricted to the sink (if with_sink) and context blocks [first, first + count).
__host__ __device__ inline int32_t stream_items_of_seq(int32_t S, int32_t B, int32_t C, int32_t G, int32_t Hkv, int32_t first,
                                                       int32_t count, int32_t with_sink)
{
    int32_t n = with_sink ? stream_items_of_region(S, G) : 0;
    if (C > 0 && count > 0) {
        int32_t nb = ceil_div(C, B);
        int32_t last = C - (nb - 1) * B;
        int32_t full = (first + count == nb) ? count - 1 : count;
        n += full * stream_items_of_region(B, G);
        if (first + count == nb) n += stream_items_of_region(last, G);
    }
    return n * Hkv;
}

// idx-th stream item of a sequence that starts at packed row `start`.  head_order (may be NULL =
// identity) lists the query heads grouped by KV head: heads of KV head g are entries g*G .. g*G+G-1.
__host__ __device__ inline pevlm_stream_item stream_item(int32_t start, int32_t S, int32_t B, int32_t C, int32_t G, int32_t Hkv,
                                                         int32_t first, int32_t with_sink, int32_t idx, int32_t seq,
                                                         const uint8_t *head_order)
{
    pevlm_stream_item it;
    int32_t sink_items = with_sink ? stream_items_of_region(S, G) * Hkv : 0;
    int32_t R, r_start, in_region;  // rows of the region, its first local position, item index inside it
    if (idx < sink_items) {  // Eq. 3
        R = S;
        r_start = 0;
        in_region = idx;
        it.full_start = start;
        it.full_len = 0;
    } else {  // Eq. 4: the whole sink plus the block itself up to the diagonal
        int32_t j = idx - sink_items;
        int32_t per_block = stream_items_of_region(B, G) * Hkv;
        int32_t nb = ceil_div(C, B);
        int32_t b = first + j / per_block;
        if (b >= nb) b = nb - 1;  // items of a short last block: fewer than per_block, all beyond the full blocks
        in_region = j - (b - first) * per_block;
        R = (C - b * B < B) ? C - b * B : B;
        r_start = S + b * B;
        it.full_start = start;
        it.full_len = S;
    }
    int32_t per_head = stream_items_of_region(R, G);
    int32_t g = in_region / per_head, jj = in_region % per_head;
    int32_t n_slots = G * ceil_div(R, kSlotRows);
    it.diag_start = start + r_start;
    it.kv_head = g;
    it.seq = seq;
    int32_t row_end = 0;
    for (int32_t w = 0; w < kSlotsPerItem; ++w) {
        int32_t k = jj * kSlotsPerItem + w;
        if (k < n_slots) {
            int32_t r0 = (k / G) * kSlotRows;
            int32_t rows = (R - r0 < kSlotRows) ? R - r0 : kSlotRows;
            int32_t hs = g * G + k % G;
            it.slot[w].q_start = start + r_start + r0;
            it.slot[w].q_rows = rows;
            it.slot[w].head = head_order ? (int32_t)head_order[hs] : hs;
            row_end = r0 + rows;
        } else {
            it.slot[w].q_start = start + r_start;
            it.slot[w].q_rows = 0;
            it.slot[w].head = 0;
        }
        it.slot[w].reserved = 0;
    }
    it.diag_len = row_end;
    it.n_full_tiles = ceil_div(it.full_len, 64);
    it.n_tiles = it.n_full_tiles + ceil_div(it.diag_len, 64);
    return it;
}

// Question items (Eq. 5): tiles of question rows x key splits.  The keys of a sequence
// [start, start + L) are cut into num_splits runs of split_len keys; everything before the
// question is visible to every question row, keys inside the question are causal.
__host__ __device__ inline int32_t query_tiles_of_seq(int32_t Q, int32_t tile_rows) { return ceil_div(Q, tile_rows); }

__host__ __device__ inline int32_t split_len_of_seq(int32_t L, int32_t num_splits, int32_t align)
{
    int32_t per = ceil_div(L, num_splits);
    per = ceil_div(per, align) * align;
    return per < align ? align : per;
}

__host__ __device__ inline pevlm_work_item query_item(int32_t start, int32_t S, int32_t C, int32_t Q,
                                                      int32_t tile_rows, int32_t num_splits, int32_t idx,
                                                      int32_t seq, int32_t qrow_base, int32_t total_q_rows,
                                                      int32_t align)
{
    // idx = tile * num_splits + split
    pevlm_work_item it;
    int32_t tile = idx / num_splits, split = idx % num_splits;
    int32_t L = S + C + Q;
    int32_t r0 = tile * tile_rows;
    it.seq = seq;
    it.q_start = start + S + C + r0;
    it.q_rows = (Q - r0 < tile_rows) ? Q - r0 : tile_rows;
    int32_t last_key = S + C + r0 + it.q_rows;  // exclusive local bound of keys any row of the tile sees
    int32_t sl = split_len_of_seq(L, num_splits, align);
    int32_t lo = split * sl, hi = lo + sl;
    if (hi > last_key) hi = last_key;
    if (lo > hi) lo = hi;
    int32_t qb = S + C;  // first local question position
    int32_t full_hi = hi < qb ? hi : qb;
    int32_t full_lo = lo < full_hi ? lo : full_hi;
    it.full_start = start + full_lo;
    it.full_len = full_hi - full_lo;
    int32_t diag_lo = lo > qb ? lo : qb;
    if (diag_lo > hi) diag_lo = hi;
    it.diag_start = start + diag_lo;
    it.diag_len = hi - diag_lo;
    it.reserved = split * total_q_rows + qrow_base + r0;  // row of this tile in the partial buffers
    return it;
}

// Question items when older context blocks are hidden from the question (sliding window): the
// visible keys of a tile are the sink [0, S) and [win_start, last key of the tile).  Split 0 is the
// sink (empty when S == 0); splits 1 .. num_splits-1 cut [win_start, L) into equal runs.
__host__ __device__ inline pevlm_work_item query_item_window(int32_t start, int32_t S, int32_t C, int32_t Q,
                                                             int32_t tile_rows, int32_t num_splits, int32_t idx,
                                                             int32_t seq, int32_t qrow_base, int32_t total_q_rows,
                                                             int32_t align, int32_t win_start)
{
    pevlm_work_item it;
    int32_t tile = idx / num_splits, split = idx % num_splits;
    int32_t L = S + C + Q;
    int32_t r0 = tile * tile_rows;
    it.seq = seq;
    it.q_start = start + S + C + r0;
    it.q_rows = (Q - r0 < tile_rows) ? Q - r0 : tile_rows;
    it.reserved = split * total_q_rows + qrow_base + r0;
    int32_t qb = S + C;
    if (split == 0) {  // the sink: visible to every question row
        it.full_start = start;
        it.full_len = S;
        it.diag_start = start + qb;
        it.diag_len = 0;
        return it;
    }
    int32_t last_key = qb + r0 + it.q_rows;
    int32_t sl = split_len_of_seq(L - win_start, num_splits - 1, align);
    int32_t lo = win_start + (split - 1) * sl, hi = lo + sl;
    if (hi > last_key) hi = last_key;
    if (lo > hi) lo = hi;
    int32_t full_hi = hi < qb ? hi : qb;
    int32_t full_lo = lo < full_hi ? lo : full_hi;
    it.full_start = start + full_lo;
    it.full_len = full_hi - full_lo;
    int32_t diag_lo = lo > qb ? lo : qb;
    if (diag_lo > hi) diag_lo = hi;
    it.diag_start = start + diag_lo;
    it.diag_len = hi - diag_lo;
    return it;
}

// ------------------------------------------------------------------------------------------
// Kernel parameter blocks
// ------------------------------------------------------------------------------------------
struct AttnParams {
    const void *q, *k, *v;
    void *out;                      // final mode: [T][Hq][D] storage type
    float *lse;                     // final mode: [T][Hq] or nullptr
    float *part_acc;                // partial mode: [slots][Hq][D] unnormalised weighted values
    float *part_ml;                 // partial mode: [slots][Hq][2] (running max of raw scores, sum)
    const pevlm_work_item *items;
    int32_t n_items;
    int32_t n_q_heads, n_kv_heads;
    float scale;                    // softmax scale
    // fused query rotation (bf16 kernels): q holds un-rotated queries and rope_tab (cos, sin) pairs
    // [entries][head_dim/2]; the entry of a row is its packed row (rope_compact_rows == 0) or its
    // compact question row (item.reserved % rope_compact_rows + row in tile).  NULL: q is rotated.
    const float *rope_tab;
    int32_t rope_compact_rows;
    HeadTable heads;
};

struct StreamParams {
    const void *q, *k, *v;
    void *out;     // [T][Hq][D] bf16
    float *lse;    // [T][Hq] or nullptr
    const pevlm_stream_item *items;
    int32_t n_items;
    int32_t n_q_heads, n_kv_heads;
    float scale;
};

// fp8 variant of the block-prefill call: 128 query rows of one region; its key tiles are tiles
// full_tile0 .. of the sink and diag_tile0 .. of its own region in the tiled E4M3 copies of K and V
struct Fp8Item {
    int32_t q_start, q_rows;
    int32_t full_start, full_len;
    int32_t diag_start, diag_len;
    int32_t full_tile0, diag_tile0;
};
struct Fp8TileBases {
    int32_t base[kMaxSeqsPerLaunch + 1];  // first key tile of each sequence of the chunk (batch-absolute)
};
struct Fp8Params {
    const uint8_t *q_codes;   // [T][Hq][D]
    const float *q_scales;    // [T][Hq]
    const uint8_t *k_tiles, *v_tiles;  // [key tile][Hkv][64 * D]
    const uint32_t *kv_amax;  // [2][Hkv] bit patterns of the largest magnitudes of K and V per head
    void *out;                // [T][Hq][D] bf16
    float *lse;
    const Fp8Item *items;
    int32_t n_items;
    int32_t n_q_heads, n_kv_heads;
    float scale;
    HeadTable heads;
};

struct MergeParams {
    const float *part_acc, *part_ml;
    const int32_t *qrow_of_compact;  // [total_q_rows] packed row of each compact question row
    void *out;
    float *lse;
    int32_t total_q_rows, num_splits, n_q_heads, head_dim;
    float scale;
    int32_t is_bf16;
};

// ------------------------------------------------------------------------------------------
// Launchers implemented in the kernel translation units (all enqueue on `stream`, never sync)
// ------------------------------------------------------------------------------------------
hipError_t launch_build_prefill_items(const SeqTable &tab, int32_t tile_rows, pevlm_work_item *items,
                                      int32_t item_offset, hipStream_t stream);
hipError_t launch_build_query_items(const SeqTable &tab, int32_t tile_rows, int32_t num_splits,
                                    int32_t total_q_rows, int32_t align, pevlm_work_item *items,
                                    int32_t item_offset, int32_t *qrow_of_compact, hipStream_t stream);
// table != NULL (bf16 only): also stores (cos, sin) [packed row][D/2] for the fused query rotation
hipError_t launch_rope(void *q, void *k, const SeqTable &tab, int32_t Hq, int32_t Hkv, int32_t D, bool bf16,
                       double rope_base, float *table, hipStream_t stream);
// pos3 != NULL: three-axis ids [3][T] (device) with sections [0, sec0), [sec0, sec01), [sec01, D/2)
hipError_t launch_rope_table(float *table, const int32_t *row_of_entry, const SeqTable &tab, int32_t D, double rope_base,
                             int32_t entry_begin, int32_t entry_end, const int32_t *pos3, int64_t T, int32_t sec0, int32_t sec01,
                             hipStream_t stream);
hipError_t launch_rope_mrope(void *q, void *k, int64_t T, int32_t Hq, int32_t Hkv, int32_t D, bool bf16, double rope_base,
                             const int32_t *pos3, int32_t sec0, int32_t sec01, float *table, hipStream_t stream);
hipError_t launch_build_stream_items(const SeqTable &tab, int32_t G, int32_t Hkv, const HeadTable &heads,
                                     pevlm_stream_item *items, int32_t item_offset, hipStream_t stream);
// block-prefill rows of bf16 tensors from a stream-item list; workgroups = compute units (8 wavefronts each)
hipError_t launch_attn_bf16_stream(const StreamParams &p, int32_t D, int32_t compute_units, hipStream_t stream);
hipError_t launch_build_fp8_items(const SeqTable &tab, const Fp8TileBases &bases, Fp8Item *items, int32_t item_offset, hipStream_t stream);
// bf16 Q, K, V -> E4M3 codes and scales (key_tiles: the prefill items of 64 rows, one per K/V tile)
hipError_t launch_fp8_quantise(const void *q, const void *k, const void *v, int64_t T, int32_t Hq, int32_t Hkv, int32_t D,
                               float q_factor, const pevlm_work_item *key_tiles, int32_t n_key_tiles, uint32_t *kv_amax, float *q_scales,
                               uint8_t *q_codes, uint8_t *k_tiles, uint8_t *v_tiles, int32_t compute_units, hipStream_t stream);
hipError_t launch_attn_fp8(const Fp8Params &p, int32_t D, hipStream_t stream);
hipError_t launch_attn_f32(const AttnParams &p, int32_t D, bool partial, hipStream_t stream);
hipError_t launch_attn_bf16(const AttnParams &p, int32_t D, bool partial, hipStream_t stream);  // p.rope_tab selects the fused variant
hipError_t launch_merge(const MergeParams &p, hipStream_t stream);
hipError_t launch_probe_mfma(float *sink, int32_t workgroups, int32_t iters, hipStream_t stream);
hipError_t launch_probe_copy(void *dst, const void *src, int64_t bytes, hipStream_t stream);
hipError_t launch_probe_tile_loop(float *sink, const void *kv, int32_t n_tiles, int32_t workgroups, int32_t iters, bool weights,
                                  hipStream_t stream);

constexpr int32_t kTileRowsF32 = 16;   // query rows per work item of the fp32 kernels
constexpr int32_t kTileRowsBf16 = 128; // query rows per work item of the bf16 MFMA kernels
constexpr int32_t kKeyTile = 64;       // keys staged per step by the bf16 and fp8 kernels
constexpr int32_t kFp8TileRows = 128;  // query rows per work item of the fp8 kernel

}  // namespace pevlm
