/*
 * libpevlm -- prefill attention of PEVLM (parallel encoding for vision-language models) for
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * The method (paper Sec. "Parallel Encoding"): a long video token sequence is split into a Sink
 * Block (prompt + first frames), frame-aligned Context Blocks and a trailing Question Block
 * (Sec. "Partitioning Strategy").  Every token is rotated at the position it has in the whole
 * sequence -- never re-based per block (Sec. "Position Encoding").  Attention is standard softmax
 * attention (Eq. 1) restricted as in Sec. "Formulations":
 *     Attn_s   = f(Q_s,   K_s,            V_s)               (Eq. 3)  sink rows
 *     Attn_c_i = f(Q_c_i, K_{s + c_i},    V_{s + c_i})       (Eq. 4)  block i sees sink + itself
 *     Attn_q   = f(Q_q,   K_{s+c_all+q},  V_{s+c_all+q})     (Eq. 5)  question sees everything
 * and is causal inside every region (key index <= query index).  Eq. 4 is taken with the key set
 * "sink plus the block itself", which is what the operation count OP_ContextBlock = 2HB(S+B)
 * (Eq. 8) and the O(L) complexity claim describe.
 *
 * Data layout (all tensors, DEVICE memory, caller-owned): token-major packed,
 *     q, out : [T][n_q_heads][head_dim]      k, v : [T][n_kv_heads][head_dim]
 * contiguous, element type given by pevlm_heads.dtype, base pointers 16-byte aligned.  Sequence s
 * owns packed rows cu_seqlens[s] .. cu_seqlens[s+1]-1 in the order
 *     [ sink (S) | block 0 | ... | block N-1 (context, C tokens in total) | question (Q) ].
 *
 * Conventions shared by every call:
 *   - Descriptor structs and the arrays they point to are HOST memory, read during the call only.
 *   - Work is enqueued on the caller's HIP stream (`stream` is a hipStream_t passed as void*;
 *     NULL = the default stream).  No call synchronises with the device, allocates or frees
 *     device memory, or keeps device state between calls.  Scratch memory is a caller-provided
 *     DEVICE workspace sized by the matching *_workspace_bytes query (256-byte aligned).
 *   - Every call returns a pevlm_status; on failure nothing has been enqueued unless the status is
 *     PEVLM_ERR_HIP, and pevlm_last_error() describes the failure.
 *   - Results are bitwise reproducible for fixed arguments (no atomics, fixed split counts).
 */
#ifndef PEVLM_H
#define PEVLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PEVLM_OK = 0,
    PEVLM_ERR_INVALID_ARG = 1,        /* null / misaligned pointer, inconsistent layout, bad head map */
    PEVLM_ERR_UNSUPPORTED = 2,        /* head_dim or dtype outside what the kernels cover          */
    PEVLM_ERR_WORKSPACE_TOO_SMALL = 3,
    PEVLM_ERR_HIP = 4                 /* a HIP runtime call failed (launch, device query)          */
} pevlm_status;

typedef enum {
    PEVLM_F32 = 0,  /* fp32 storage and arithmetic (plain FMA kernels; the numerical anchor)       */
    PEVLM_BF16 = 1  /* bf16 storage, bf16 MFMA with fp32 accumulation and fp32 softmax             */
} pevlm_dtype;

/* Partition of every packed sequence (Sec. "Partitioning Strategy").  num_blocks = ceil(C / B);
 * the last context block holds C - (num_blocks-1)*B tokens and may be shorter than B.  S, C and Q
 * may each be 0.  Required: S + C + Q == cu_seqlens[s+1] - cu_seqlens[s], cu_seqlens[0] == 0. */
typedef struct {
    int32_t num_seqs;           /* >= 1 */
    const int32_t *cu_seqlens;  /* [num_seqs + 1] */
    const int32_t *sink_len;    /* [num_seqs]  S >= 0 */
    const int32_t *block_len;   /* [num_seqs]  B >= 1 (ignored where C == 0) */
    const int32_t *ctx_len;     /* [num_seqs]  C >= 0 */
    const int32_t *query_len;   /* [num_seqs]  Q >= 0 */
} pevlm_layout;

typedef struct {
    int32_t n_q_heads;            /* Hq */
    int32_t n_kv_heads;           /* Hkv, Hq % Hkv == 0 */
    int32_t head_dim;             /* D: 64 or 128 */
    const int32_t *kv_head_of_q;  /* HOST [Hq] KV head of each query head, or NULL = h / (Hq/Hkv) */
    pevlm_dtype dtype;
    float softmax_scale;          /* <= 0 selects 1/sqrt(head_dim) (Eq. 1) */
} pevlm_heads;

/*
 * Sequential rotary position embedding (Sec. "Position Encoding"), in place on q [T][Hq][D] and
 * k [T][Hkv][D] (either may be NULL to skip it).  Token t of sequence s is rotated at
 * pos = t - cu_seqlens[s] + pos_offset[s] (pos_offset: HOST [num_seqs] or NULL = 0): positions run
 * through sink, every context block and the question without restarting.  Rotate-half pairing:
 * (x[i], x[i+D/2]) turns by pos * rope_base^(-2i/D).  Angles are formed in fp64 and reduced before
 * the fp32 sine/cosine; results are rounded once to the storage type.
 */
pevlm_status pevlm_rope_seq(void *q, void *k, const pevlm_layout *layout, const pevlm_heads *heads,
                            double rope_base, const int32_t *pos_offset, void *stream);

/*
 * Multimodal RoPE with three position axes (temporal, height, width): the position scheme of the
 * Qwen2.5-VL models the paper evaluates (Sec. "Experimental setup"; related work on 3D-MRoPE).  The
 * method's rule (Sec. "Position Encoding") is unchanged: the ids are those of the whole prompt and
 * are never re-based per block, so the caller passes them explicitly.
 *   pos_ids : DEVICE int32 [3][num_tokens] (axis-major), read by the kernel on `stream`
 *   section : HOST int32 [3], how many of the head_dim/2 pair indices each axis owns, in the order
 *             temporal, height, width; consecutive ranges; must add up to head_dim/2
 * Pair (x[i], x[i+D/2]) of token t turns by pos_ids[axis(i)][t] * rope_base^(-2i/D); in place on
 * q [num_tokens][Hq][D] and k [num_tokens][Hkv][D] (either may be NULL).  With three equal axes the
 * result is that of pevlm_rope_seq at those positions.  No layout is needed: sequences only matter
 * through the ids.
 */
pevlm_status pevlm_rope_mrope(void *q, void *k, int64_t num_tokens, const pevlm_heads *heads, double rope_base,
                              const int32_t *pos_ids, const int32_t *section, void *stream);

/*
 * Block-parallel prefill attention: rows of the sink (Eq. 3) and of every context block (Eq. 4).
 * q and k must already be rotated.  Writes out rows of the sink and context regions only;
 * question rows of `out` (and `lse`) are left untouched.  lse: DEVICE fp32 [T][Hq] natural-log
 * sum-exp of the scaled scores per written row, or NULL.  A tile work list that names only
 * (query tile, sink keys, own-block keys up to the diagonal) is built on the device into the
 * workspace; cross-block tiles are never enumerated.  A dense causal attention over a sequence is
 * the layout S = 0, C = L, B = L, Q = 0.
 */
size_t pevlm_block_prefill_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads);
pevlm_status pevlm_block_prefill_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                                      const pevlm_layout *layout, const pevlm_heads *heads,
                                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Question attention (Eq. 5): every question row attends to all earlier tokens of its sequence
 * (sink, all context blocks, earlier question tokens).  The key range is cut into num_splits
 * parts (0 = chosen from the layout; 1..PEVLM_MAX_SPLITS otherwise) that are processed by
 * different workgroups into fp32 partials (max, sum, weighted values) in the workspace and then
 * merged with the log-sum-exp identity.  Writes question rows of `out` (and `lse`) only.
 */
#define PEVLM_MAX_SPLITS 64
size_t pevlm_query_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits);
pevlm_status pevlm_query_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                              const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * pevlm_query_attn for callers that cannot hand over (or allocate) a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same kernels and
 * bit-identical results, but the scratch memory (work list, row map, fp32 partials) is an array of
 * PEVLM_STATIC_SCRATCH_BYTES that is part of the library's code object: every GPU the library runs
 * on holds one copy until the process ends.  The call allocates and frees nothing and does not
 * synchronise.  A call whose plan needs more than the array (what pevlm_query_workspace_bytes
 * reports, minus its 256 bytes of slack) returns PEVLM_ERR_WORKSPACE_TOO_SMALL with nothing enqueued.
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different
 * streams, different threads) race and must be serialised by the caller.  The first call on a
 * device looks up the array's device address (make that call outside a graph capture).
 */
#define PEVLM_STATIC_SCRATCH_BYTES (64u << 20)
pevlm_status pevlm_query_attn_static(const void *q, const void *k, const void *v, void *out, float *lse,
                                     const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits,
                                     void *stream);

/*
 * The two attention calls with the sequential RoPE step (Sec. "Position Encoding") folded in, so
 * that q is never read and re-written by a separate pass.  `q` holds UN-rotated queries and is not
 * modified: each workgroup rotates its query rows once, on the fly, at
 * pos = t - cu_seqlens[s] + pos_offset[s] (pos_offset: HOST [num_seqs] or NULL = 0) with the same
 * arithmetic and the same single rounding to bf16 as pevlm_rope_seq, so `out` and `lse` are bit for
 * bit those of the three-call path.  Keys:
 *   pevlm_block_prefill_attn_rope, k_is_rotated == 0: k holds un-rotated keys of ALL tokens of the
 *       layout and is rotated IN PLACE first (as pevlm_rope_seq(NULL, k, ...) would), by the kernel
 *       that also fills the (cos, sin) table the query rotation reads;
 *   k_is_rotated != 0: k is already rotated and only read.
 *   pevlm_query_attn_rope: k must already be rotated (by either of the above).
 * bf16 tensors only (PEVLM_ERR_UNSUPPORTED otherwise).  The workspace additionally holds the
 * (cos, sin) table: head_dim * 4 bytes per token (prefill) or per question row (question call).
 * Everything else is as for pevlm_block_prefill_attn / pevlm_query_attn.
 */
size_t pevlm_block_prefill_rope_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads);
pevlm_status pevlm_block_prefill_attn_rope(const void *q, void *k, const void *v, void *out, float *lse,
                                           const pevlm_layout *layout, const pevlm_heads *heads, double rope_base,
                                           const int32_t *pos_offset, int32_t k_is_rotated, void *workspace,
                                           size_t workspace_bytes, void *stream);
size_t pevlm_query_rope_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits);
pevlm_status pevlm_query_attn_rope(const void *q, const void *k, const void *v, void *out, float *lse,
                                   const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits,
                                   double rope_base, const int32_t *pos_offset, void *workspace, size_t workspace_bytes,
                                   void *stream);

/* The same two calls for three-axis position ids (see pevlm_rope_mrope for pos_ids and section;
 * pos_ids is DEVICE [3][T] with T = cu_seqlens[num_seqs]).  Workspace sizes are those of the _rope calls. */
pevlm_status pevlm_block_prefill_attn_mrope(const void *q, void *k, const void *v, void *out, float *lse,
                                            const pevlm_layout *layout, const pevlm_heads *heads, double rope_base,
                                            const int32_t *pos_ids, const int32_t *section, int32_t k_is_rotated,
                                            void *workspace, size_t workspace_bytes, void *stream);
pevlm_status pevlm_query_attn_mrope(const void *q, const void *k, const void *v, void *out, float *lse,
                                    const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits,
                                    double rope_base, const int32_t *pos_ids, const int32_t *section, void *workspace,
                                    size_t workspace_bytes, void *stream);

/*
 * Streaming use (the paper's outlook, Sec. "Conclusion": streaming video, a sliding window that
 * discards the oldest video blocks).  Both calls work on the ordinary packed layout; blocks that
 * are no longer referenced are simply never read, so the caller may recycle their storage.
 *
 * pevlm_block_prefill_attn_blocks: as pevlm_block_prefill_attn, restricted per sequence to the rows
 * of context blocks first_block[s] .. first_block[s] + num_blocks[s] - 1 (HOST arrays [num_seqs];
 * the range must lie inside the sequence's ceil(C/B) blocks, num_blocks[s] may be 0) and, if
 * with_sink != 0, the sink rows.  By Eq. 4 a block needs only the sink's and its own K/V, so
 * appending blocks to a prompt costs the new blocks' rows only.  Rows outside the selection are
 * not touched.  Workspace: pevlm_block_prefill_workspace_bytes.
 *
 * pevlm_query_attn_window: as pevlm_query_attn, but a question row of sequence s sees, besides the
 * sink and the question itself, only the last window_blocks[s] context blocks (HOST [num_seqs];
 * a negative entry = all blocks; 0 = none).  The sink is always processed as a split of its own and
 * the remaining keys are cut into num_splits - 1 runs, so at least 2 splits are used (num_splits == 1
 * is raised to 2; 0 = chosen by the library).  Workspace: pevlm_query_window_workspace_bytes.
 */
pevlm_status pevlm_block_prefill_attn_blocks(const void *q, const void *k, const void *v, void *out, float *lse,
                                             const pevlm_layout *layout, const pevlm_heads *heads,
                                             const int32_t *first_block, const int32_t *num_blocks, int32_t with_sink,
                                             void *workspace, size_t workspace_bytes, void *stream);
size_t pevlm_query_window_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads, int32_t num_splits);
pevlm_status pevlm_query_attn_window(const void *q, const void *k, const void *v, void *out, float *lse,
                                     const pevlm_layout *layout, const pevlm_heads *heads, const int32_t *window_blocks,
                                     int32_t num_splits, void *workspace, size_t workspace_bytes, void *stream);

/* Message of the last failure on the calling thread (static storage, never NULL). */
const char *pevlm_last_error(void);
/* Library version: major * 10000 + minor * 100 + patch. */
int32_t pevlm_version(void);

/* ---- host-side utilities (no device access; usable on a machine without a GPU) ---- */

/* One unit of work of the block-prefill kernel: a tile of at most tile_rows query rows that lie
 * in one region (the sink, or one context block) plus the two key ranges it needs.  Indices are
 * packed token rows.  Keys [full_start, full_start + full_len) are all visible to every row of
 * the tile (the sink, for a context tile); keys [diag_start, diag_start + diag_len) are visible to
 * row i iff key <= i (own region up to the tile's last row). */
typedef struct {
    int32_t q_start, q_rows;
    int32_t full_start, full_len;
    int32_t diag_start, diag_len;
    int32_t seq, reserved;
} pevlm_work_item;

/* One unit of work of the streaming bf16 block-prefill kernel (head_dim 128 or 64, query heads in
 * equal groups per KV head): up to 8 slots of at most 32 query rows of ONE region (the sink, or one
 * context block) whose heads share one KV head, so that all slots need the same key tiles: keys
 * [full_start, full_start + full_len) visible to every row (the sink, for a context block) and keys
 * [diag_start, diag_start + diag_len) visible to row i iff key <= i.  Slot w is taken by wavefront w
 * of the workgroup that processes the item; q_rows == 0 marks an unused slot.  Within a region the
 * slots run over (group of 32 rows, query head of the KV group) with the head index fastest, so the
 * 8 slots of an item lie within 64 rows of each other and need almost the same number of key tiles. */
typedef struct {
    int32_t full_start, full_len;
    int32_t diag_start, diag_len;
    int32_t kv_head, n_full_tiles, n_tiles, seq; /* tiles of 64 keys: full range first, then diagonal range */
    struct {
        int32_t q_start, q_rows; /* packed row of the slot's first query, rows (1..32, 0 = unused) */
        int32_t head, reserved;  /* query head */
    } slot[8];
} pevlm_stream_item;

/* 1 if pevlm_block_prefill_attn runs the streaming kernel for this layout and head descriptor on the
 * current device, else 0: then the one-item-per-workgroup kernel and the pevlm_work_item list are
 * used.  The streaming kernel needs bf16 tensors, every KV head serving the same number of query
 * heads, and fewer than 2 GiB per K (or V) tensor; left to itself the library takes it when the list
 * holds at least 12 stream items per compute unit and no sink or block is longer than 16384 rows. */
int32_t pevlm_prefill_uses_stream_kernel(const pevlm_layout *layout, const pevlm_heads *heads);
/* Process-wide choice of that kernel, for timing comparisons and tests: 0 = per call as described
 * above (the default; the environment variable PEVLM_PREFILL_KERNEL=classic|stream sets the start
 * value 1 or 2), 1 = always the one-item-per-workgroup kernel, 2 = the streaming kernel wherever it
 * applies.  Results are bit-identical either way.  Returns the previous value, or -1 for a bad mode. */
int32_t pevlm_set_prefill_kernel(int32_t mode);
/* Enumerates, on the host, exactly the stream-item list the device builder writes for
 * pevlm_block_prefill_attn_blocks (first_block == NULL: every block and the sink, as
 * pevlm_block_prefill_attn).  Returns the number of items, or -1 for invalid arguments. */
int64_t pevlm_prefill_stream_items_host(const pevlm_layout *layout, const pevlm_heads *heads, const int32_t *first_block,
                                        const int32_t *num_blocks, int32_t with_sink, pevlm_stream_item *items,
                                        int64_t capacity);

/* ---- fp8 variant of the block-prefill call (an extension of Eq. 3-4 to 8-bit operands; bf16 in, bf16 out)
 *
 * pevlm_block_prefill_attn_fp8 computes the same rows as pevlm_block_prefill_attn from E4M3 copies
 * of Q, K and V (OCP 8-bit floating point: 4 exponent bits with bias 7, 3 mantissa bits, largest
 * value 448, no infinities) on the fp8 matrix cores, with fp32 accumulation and fp32 softmax; the
 * attention weights are rounded to E4M3 as well.  It runs in two stages, selected by `stages`
 * (0 = both): PEVLM_FP8_QUANTISE writes the work lists and the codes into the workspace,
 * PEVLM_FP8_ATTEND computes `out` (and `lse`) from a workspace a QUANTISE stage has filled for the
 * same layout, heads and tensors (q, k, v are not read by it).
 *
 * A tensor is stored as codes times a power-of-two scale 2^e, e the smallest integer with
 * amax * 2^-e <= 448 (amax: the largest magnitude the scale covers; e = 0 if that is 0; e within
 * [-100, 100]); codes are rounded to nearest, ties to even.  Q has one scale per (token, query
 * head), K and V one per KV head over all tokens of the call.  What is quantised of Q is q * f with
 * f = softmax factor * log2(e) (both float32, one float32 rounding per product): the scores of the
 * quantised operands are then base-2 exponents.  Inputs must be finite.
 *
 * Workspace (DEVICE, 256-byte aligned, pevlm_block_prefill_fp8_workspace_bytes; byte offsets of its
 * parts from pevlm_block_prefill_fp8_plan):
 *   q_codes   [T][Hq][D] codes of q * f;  q_scales [T][Hq] fp32 scales (2^e)
 *   kv_amax   [2][Hkv] fp32: largest magnitude of K, then of V, per KV head
 *   key_tiles n_key_tiles pevlm_work_item: (q_start, q_rows) = the token rows of key tile i; the
 *             tiles are the 64-row tiles of pevlm_prefill_worklist_host(layout, 64, ...)
 *   k_tiles   [key tile][Hkv][64 rows][D] codes, rows past q_rows zero; the 16-byte chunk c of row r
 *             is stored at chunk position c ^ ((r / (256 / D)) % (D / 16)) of the row
 *   v_tiles   [key tile][Hkv][D rows][64] codes: row d, byte j holds key
 *             ((j % 32) / 16) * 32 + ((j % 16) / 4) * 8 + (j / 32) * 4 + j % 4 of the tile; the 16-byte
 *             chunk c of row d is stored at chunk position c ^ ((d / 4) % 4)
 * head_dim 64 or 128, dtype PEVLM_BF16 (else PEVLM_ERR_UNSUPPORTED).  Other arguments, ownership
 * and error behaviour as pevlm_block_prefill_attn. */
enum { PEVLM_FP8_QUANTISE = 1, PEVLM_FP8_ATTEND = 2 };
typedef struct {
    int64_t n_items, n_key_tiles;
    size_t items, key_tiles, kv_amax, q_scales, q_codes, k_tiles, v_tiles; /* byte offsets into the workspace */
    size_t total;                                                        /* = pevlm_block_prefill_fp8_workspace_bytes */
} pevlm_fp8_plan;
pevlm_status pevlm_block_prefill_fp8_plan(const pevlm_layout *layout, const pevlm_heads *heads, pevlm_fp8_plan *plan);
size_t pevlm_block_prefill_fp8_workspace_bytes(const pevlm_layout *layout, const pevlm_heads *heads);
pevlm_status pevlm_block_prefill_attn_fp8(const void *q, const void *k, const void *v, void *out, float *lse,
                                          const pevlm_layout *layout, const pevlm_heads *heads, void *workspace,
                                          size_t workspace_bytes, int32_t stages, void *stream);

/* Query rows per work item the kernels selected by `heads` use for the block-prefill call and for
 * the question call (-1 for an invalid descriptor). */
int32_t pevlm_prefill_tile_rows(const pevlm_heads *heads);
int32_t pevlm_query_tile_rows(const pevlm_heads *heads);
/* Enumerates, on the host, exactly the work list the device builder writes.  Returns the number
 * of items (also when items == NULL or capacity is too small: then nothing beyond capacity is
 * written), or -1 for an invalid layout. */
int64_t pevlm_prefill_worklist_host(const pevlm_layout *layout, int32_t tile_rows,
                                    pevlm_work_item *items, int64_t capacity);
/* Same for the question call: tiles of question rows x num_splits key runs; `reserved` holds the
 * first row of the item in the partial buffers. */
int64_t pevlm_query_worklist_host(const pevlm_layout *layout, int32_t tile_rows, int32_t num_splits,
                                  pevlm_work_item *items, int64_t capacity);
/* The same enumerations for the streaming calls: prefill items of the selected blocks (and the sink
 * if with_sink != 0); question items under a window (num_splits >= 2: split 0 is the sink). */
int64_t pevlm_prefill_worklist_blocks_host(const pevlm_layout *layout, int32_t tile_rows, const int32_t *first_block,
                                           const int32_t *num_blocks, int32_t with_sink, pevlm_work_item *items,
                                           int64_t capacity);
int64_t pevlm_query_worklist_window_host(const pevlm_layout *layout, int32_t tile_rows, int32_t num_splits,
                                         const int32_t *window_blocks, pevlm_work_item *items, int64_t capacity);
/* Visible (query, key) pairs per head implied by the layout, split by region; the causal closed
 * forms behind the paper's operation counts (Eq. 6-10).  Any output pointer may be NULL.
 * Returns PEVLM_OK or PEVLM_ERR_INVALID_ARG. */
pevlm_status pevlm_visible_pairs(const pevlm_layout *layout, int64_t *sink_pairs, int64_t *block_pairs,
                                 int64_t *question_pairs);

/* ---- roofline probes (measurement only; none of the method's arithmetic) ----
 * The block-prefill kernel is bound by the bf16 matrix cores and the RoPE / question kernels by
 * HBM (the operation counts of Eq. 6-10 against the bytes of Q, K, V, O).  These two calls let a
 * benchmark time, on the same device and clocks, what those resources sustain.
 *
 * pevlm_probe_mfma_bf16: `workgroups` workgroups of 4 wavefronts each issue 4*iters register-resident
 * v_mfma_f32_32x32x16_bf16 instructions; *flop_count (HOST, may be NULL) receives the floating-point
 * operations of the launch.  scratch: DEVICE, >= 4 bytes, never written in practice.
 * pevlm_probe_copy: streaming copy of `bytes` (multiple of 16) from src to dst (DEVICE, 16-byte
 * aligned, not overlapping): bytes read + bytes written = 2*bytes.
 * All probes enqueue one kernel on `stream` and return PEVLM_ERR_INVALID_ARG without launching on bad
 * arguments. */
pevlm_status pevlm_probe_mfma_bf16(void *scratch, int32_t workgroups, int32_t iters, double *flop_count, void *stream);
pevlm_status pevlm_probe_copy(void *dst, const void *src, size_t bytes, void *stream);
/* pevlm_probe_tile_loop_bf16: the steady-state tile step of the bf16 block-prefill kernels and nothing
 * else -- per step and wavefront 32 v_mfma_f32_32x32x16_bf16 (scores of a 32 x 64 x 128 tile and the
 * values of the previous one), their LDS fragment reads, the asynchronous global->LDS loads of the next
 * K and V tile, a workgroup barrier and, if with_softmax != 0, the vector arithmetic that turns the
 * scores into bf16 weights -- run `iters` times by `workgroups` workgroups of 4 wavefronts (2 fit a
 * compute unit).  No masks, no rescaling, no queries, no outputs: what this sustains is what the
 * kernels' instruction mix allows on the device.  kv: DEVICE, 16-byte aligned, kv_bytes >= 64 KiB of
 * finite bf16 data, read as 16 KiB tiles (first half as K tiles, second half as V tiles); scratch:
 * DEVICE, >= 4 bytes, never written in practice; *flop_count (HOST, may be NULL) receives the
 * floating-point operations of the MFMAs of the launch. */
pevlm_status pevlm_probe_tile_loop_bf16(void *scratch, const void *kv, size_t kv_bytes, int32_t workgroups, int32_t iters,
                                        int32_t with_softmax, double *flop_count, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PEVLM_H */
