/*
 * PEVLM parallel-encoding attention -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, fp64 statement of what the prefill attention path computes.
 * It exists so that tests, the smoke check and the benchmark's cpu_baseline leg can compare the
 * GPU library against it.  It is not part of the product path, shares no code with the HIP
 * library, and nothing in the product may call it.
 *
 * What it follows (paper sections / equations):
 *   - Standard softmax attention  O = Softmax(Q K^T / sqrt(d)) V            (Sec. "Standard
 *     Attention Mechanism", Eq. 1).
 *   - Partition of a sequence into Sink Block, Context Blocks, Question Block
 *     (Sec. "Partitioning Strategy").
 *   - Sequential position embedding: every token keeps the position it has in the whole
 *     sequence; positions are never re-based per block and the question continues after the
 *     video (Sec. "Position Encoding").
 *   - The three attention formulas Attn_s, Attn_ci, Attn_q (Sec. "Formulations", Eq. 3-5),
 *     with the reading that a context block's keys are the sink plus the block itself, as the
 *     operation count OP_ContextBlock = 2HB(S+B) (Eq. 8) and the O(L) claim require, and with
 *     causality (key index <= query index) inside every region, the models being decoder-only.
 *
 * The mask is built explicitly (0 or -inf per key) and added to the scores; nothing is tiled,
 * fused or reordered.  The only shortcut offered is `skip_masked`: a key whose mask entry is
 * -inf contributes exp(-inf) = 0 exactly, so it may be bypassed; the literal mode scores every
 * key of the packed batch.  Tests show both modes agree bit for bit.
 *
 * Parity pins (all under tests/, none of them calls back into this file for the expected value):
 * brute-force Python loops that evaluate Eq. 3, 4, 5 one by one on gathered keys; torch's CPU
 * scaled_dot_product_attention on the gathered causal pieces; the closed-form pair counts of
 * Eq. 6-10; convexity / constant-V / zero-Q closed forms; RoPE analytic identities; for the two
 * extensions (three-axis RoPE, sliding window for the question) a complex-multiplication brute
 * force / the rule written out entry by entry and library causal attention over the kept keys.
 * The paper prints no numeric worked example, so value-level parity with the authors' own
 * implementation is unpinned; every function here is pinned by the checks above instead.
 *
 * Layout of all tensors: token-major packed, x[T][H][D] contiguous; sequence s owns packed rows
 * cu_seqlens[s] .. cu_seqlens[s+1]-1 ordered [sink | block 0 | ... | block N-1 | question].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

typedef struct {
    int32_t num_seqs;
    const int32_t *cu_seqlens; /* [num_seqs+1] */
    const int32_t *sink_len;   /* S per sequence */
    const int32_t *block_len;  /* B per sequence */
    const int32_t *ctx_len;    /* C per sequence: total context tokens, last block may be short */
    const int32_t *query_len;  /* Q per sequence */
    /* Sliding window for the question (the paper's outlook, Sec. "Conclusion": discard the oldest
     * video blocks): NULL, or per sequence the number W of most recent context blocks a question
     * row still sees besides the sink and the question itself; W < 0 = all blocks. */
    const int32_t *window_blocks;
} oracle_layout;

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F64) return ((const double *)base)[idx];
    if (dtype == ORACLE_F32) return (double)((const float *)base)[idx];
    /* bf16: the upper 16 bits of an IEEE float */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Returns 0 when the layout is self-consistent, else a positive code naming the first defect. */
int pevlm_oracle_check_layout(const oracle_layout *lay)
{
    if (!lay || lay->num_seqs < 1) return 1;
    if (lay->cu_seqlens[0] != 0) return 2;
    for (int32_t s = 0; s < lay->num_seqs; ++s) {
        int64_t len = (int64_t)lay->cu_seqlens[s + 1] - lay->cu_seqlens[s];
        if (len < 0) return 3;
        if (lay->sink_len[s] < 0 || lay->ctx_len[s] < 0 || lay->query_len[s] < 0) return 4;
        if (lay->ctx_len[s] > 0 && lay->block_len[s] < 1) return 5;
        if ((int64_t)lay->sink_len[s] + lay->ctx_len[s] + lay->query_len[s] != len) return 6;
    }
    return 0;
}

/* Sequence that owns packed row t (-1 if none). */
static int32_t seq_of(const oracle_layout *lay, int64_t t)
{
    for (int32_t s = 0; s < lay->num_seqs; ++s)
        if (t >= lay->cu_seqlens[s] && t < lay->cu_seqlens[s + 1]) return s;
    return -1;
}

/*
 * Visibility of key j to query i, both positions local to one sequence with sink S, block
 * length B, context length C (Eq. 3-5):
 *   sink row      (i < S)         : sink keys up to itself                      (Eq. 3)
 *   context row   (S <= i < S+C)  : all sink keys + keys of its own block up to itself (Eq. 4)
 *   question row  (i >= S+C)      : every key up to itself                      (Eq. 5)
 */
int pevlm_oracle_visible(int64_t S, int64_t B, int64_t C, int64_t i, int64_t j)
{
    if (j > i) return 0;                    /* causal */
    if (i < S) return 1;                    /* sink row: j <= i < S */
    if (i >= S + C) return 1;               /* question row */
    if (j < S) return 1;                    /* context row, sink key */
    return ((i - S) / B) == ((j - S) / B);  /* context row, context key: same block only */
}

/* Same, with the causal condition dropped inside regions: the block-granular mask whose pair
 * count the paper's operation-count formulas (Eq. 6-10) describe. */
int pevlm_oracle_visible_blockwise(int64_t S, int64_t B, int64_t C, int64_t Q, int64_t i, int64_t j)
{
    (void)Q;
    if (i < S) return j < S;                                  /* OP_Sink  ~ S*S       */
    if (i >= S + C) return 1;                                 /* OP_Quest ~ Q*L       */
    if (j < S) return 1;                                      /* OP_ContextBlock ~ B*(S+B) */
    if (j >= S + C) return 0;
    return ((i - S) / B) == ((j - S) / B);
}

/* Explicit mask row for packed query row t over all T packed keys: vis[j] = 1 visible, 0 masked.
 * Tokens of different packed sequences never see each other. */
void pevlm_oracle_mask_row(const oracle_layout *lay, int64_t t, int causal, uint8_t *vis)
{
    int64_t T = lay->cu_seqlens[lay->num_seqs];
    memset(vis, 0, (size_t)T);
    int32_t s = seq_of(lay, t);
    if (s < 0) return;
    int64_t base = lay->cu_seqlens[s];
    int64_t L = lay->cu_seqlens[s + 1] - base;
    int64_t S = lay->sink_len[s], B = lay->block_len[s], C = lay->ctx_len[s], Q = lay->query_len[s];
    if (B < 1) B = 1;
    for (int64_t j = 0; j < L; ++j)
        vis[base + j] = (uint8_t)(causal ? pevlm_oracle_visible(S, B, C, t - base, j)
                                         : pevlm_oracle_visible_blockwise(S, B, C, Q, t - base, j));
    /* sliding window: a question row loses the context blocks older than the last W */
    if (lay->window_blocks && lay->window_blocks[s] >= 0 && t - base >= S + C) {
        int64_t n_blocks = (C + B - 1) / B;
        int64_t first_kept = n_blocks - lay->window_blocks[s];
        if (first_kept < 0) first_kept = 0;
        for (int64_t j = S; j < S + C; ++j)
            if ((j - S) / B < first_kept) vis[base + j] = 0;
    }
}

/* Sequential positions (Sec. "Position Encoding"): pos[t] = index of token t inside its own
 * sequence (+ a per-sequence constant offset, 0 when pos_offset is NULL).  Never re-based per
 * block; question tokens continue where the video ends. */
void pevlm_oracle_positions(const oracle_layout *lay, const int32_t *pos_offset, int32_t *pos)
{
    for (int32_t s = 0; s < lay->num_seqs; ++s)
        for (int64_t t = lay->cu_seqlens[s]; t < lay->cu_seqlens[s + 1]; ++t)
            pos[t] = (int32_t)(t - lay->cu_seqlens[s]) + (pos_offset ? pos_offset[s] : 0);
}

/*
 * Rotary position embedding in fp64, rotate-half pairing (i, i + D/2):
 *   theta_i = pos * base^(-2i/D),   x'[i]       = x[i] cos(theta_i) - x[i+D/2] sin(theta_i)
 *                                   x'[i + D/2] = x[i+D/2] cos(theta_i) + x[i] sin(theta_i)
 * x is [T][H][D] of `dtype`; rows (packed token indices, NULL = all T rows in order) selects
 * which tokens are rotated; out is [n_rows][H][D] fp64.
 */
void pevlm_oracle_rope(const void *x, int dtype, int64_t T, int32_t H, int32_t D,
                       const int32_t *pos, double rope_base,
                       const int64_t *rows, int64_t n_rows, double *out)
{
    if (!rows) n_rows = T;
    int32_t half = D / 2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t t = rows ? rows[r] : r;
        double p = (double)pos[t];
        for (int32_t h = 0; h < H; ++h) {
            int64_t in0 = (t * H + h) * (int64_t)D;
            double *o = out + (r * H + h) * (int64_t)D;
            for (int32_t i = 0; i < half; ++i) {
                double inv_freq = pow(rope_base, -2.0 * (double)i / (double)D);
                double theta = p * inv_freq;
                double c = cos(theta), sn = sin(theta);
                double x0 = widen(x, dtype, in0 + i), x1 = widen(x, dtype, in0 + i + half);
                o[i] = x0 * c - x1 * sn;
                o[i + half] = x1 * c + x0 * sn;
            }
        }
    }
}

/*
 * Multimodal rotary embedding with three position axes (the position scheme of the Qwen2.5-VL
 * models the paper evaluates, Sec. "Experimental setup" / related work on 3D-MRoPE; the paper's
 * rule is only that the original ids are kept, never re-based per block, Sec. "Position Encoding").
 * The D/2 pair indices are cut into three consecutive sections of section[0], section[1],
 * section[2] indices (temporal, height, width; they must add up to D/2); pair i of token t turns by
 *   theta_i = pos3[axis(i)][t] * base^(-2i/D)
 * with the same rotate-half pairing (i, i + D/2) as pevlm_oracle_rope.  pos3 is [3][T].
 * With the three axes equal this is pevlm_oracle_rope.
 */
void pevlm_oracle_rope_mrope(const void *x, int dtype, int64_t T, int32_t H, int32_t D,
                             const int32_t *pos3, const int32_t *section, double rope_base,
                             const int64_t *rows, int64_t n_rows, double *out)
{
    if (!rows) n_rows = T;
    int32_t half = D / 2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t t = rows ? rows[r] : r;
        for (int32_t h = 0; h < H; ++h) {
            int64_t in0 = (t * H + h) * (int64_t)D;
            double *o = out + (r * H + h) * (int64_t)D;
            for (int32_t i = 0; i < half; ++i) {
                int axis = i < section[0] ? 0 : (i < section[0] + section[1] ? 1 : 2);
                double p_axis = (double)pos3[(int64_t)axis * T + t];
                double angle = p_axis * pow(rope_base, -(2.0 * i) / D);
                double ca = cos(angle), sa = sin(angle);
                double lo = widen(x, dtype, in0 + i), hi = widen(x, dtype, in0 + half + i);
                o[i] = lo * ca - hi * sa;
                o[half + i] = hi * ca + lo * sa;
            }
        }
    }
}

/*
 * Masked softmax attention, Eq. 1 with the explicit PEVLM mask added to the scores:
 *   s_j = (q_i . k_j) / sqrt(D) + M[i][j],  w_j = exp(s_j - max_j s_j),  o_i = sum_j w_j v_j / sum_j w_j
 * for every selected packed row t = rows[r] and every query head h (KV head kv_head_of_q[h]).
 *   q_rot [n_rows][Hq][D] fp64  rotated queries of the selected rows
 *   k_rot [T][Hkv][D]     fp64  rotated keys of every token
 *   v     [T][Hkv][D]     v_dtype
 *   key_lo/key_hi: restrict the keys to packed range [key_lo, key_hi) on top of the mask
 *                  (0, T for the plain result); a row left with no key gets out = 0, lse = -inf.
 *   causal: 1 = the method; 0 = block-granular mask (only used to pin pair counts).
 *   skip_masked: 0 = literal (every key scored, -inf added), 1 = masked keys bypassed.
 *   softmax_scale <= 0 selects 1/sqrt(D).
 * out [n_rows][Hq][D], lse [n_rows][Hq] (natural-log sum-exp of the scaled scores).
 */
void pevlm_oracle_attn(const double *q_rot, const double *k_rot, const void *v, int v_dtype,
                       const oracle_layout *lay, int32_t Hq, int32_t Hkv, int32_t D,
                       const int32_t *kv_head_of_q, double softmax_scale,
                       const int64_t *rows, int64_t n_rows,
                       int64_t key_lo, int64_t key_hi, int causal, int skip_masked,
                       double *out, double *lse)
{
    int64_t T = lay->cu_seqlens[lay->num_seqs];
    int64_t n_work = n_rows * Hq;
#pragma omp parallel
    {
        uint8_t *vis = (uint8_t *)malloc((size_t)(T > 0 ? T : 1));
        double *sc = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
#pragma omp for schedule(dynamic, 4)
        for (int64_t w = 0; w < n_work; ++w) {
            int64_t r = w / Hq;
            int32_t h = (int32_t)(w % Hq);
            int32_t g = kv_head_of_q ? kv_head_of_q[h] : h / (Hq / Hkv);
            int64_t t = rows ? rows[r] : r;
            const double *q = q_rot + (r * Hq + h) * (int64_t)D;
            double *o = out + (r * Hq + h) * (int64_t)D;

            pevlm_oracle_mask_row(lay, t, causal, vis);
            for (int64_t j = 0; j < T; ++j)
                if (j < key_lo || j >= key_hi) vis[j] = 0;

            /* scores + mask */
            double m = -INFINITY;
            for (int64_t j = 0; j < T; ++j) {
                if (skip_masked && !vis[j]) { sc[j] = -INFINITY; continue; }
                const double *kj = k_rot + (j * Hkv + g) * (int64_t)D;
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d) dot += q[d] * kj[d];
                double s = softmax_scale > 0.0 ? dot * softmax_scale : dot / sqrt((double)D);
                s += vis[j] ? 0.0 : -INFINITY;
                sc[j] = s;
                if (s > m) m = s;
            }
            for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
            if (m == -INFINITY) { /* no key at all (only possible under a key range) */
                if (lse) lse[r * Hq + h] = -INFINITY;
                continue;
            }
            /* softmax weights and weighted sum of values */
            double l = 0.0;
            for (int64_t j = 0; j < T; ++j) {
                if (skip_masked && !vis[j]) continue;
                double wj = exp(sc[j] - m); /* exp(-inf) == 0 exactly for masked keys */
                l += wj;
                int64_t v0 = (j * Hkv + g) * (int64_t)D;
                for (int32_t d = 0; d < D; ++d) o[d] += wj * widen(v, v_dtype, v0 + d);
            }
            for (int32_t d = 0; d < D; ++d) o[d] /= l;
            if (lse) lse[r * Hq + h] = m + log(l);
        }
        free(vis);
        free(sc);
    }
}

/* Number of OpenMP threads the loops above will use. */
#ifdef _OPENMP
#include <omp.h>
int pevlm_oracle_threads(void) { return omp_get_max_threads(); }
#else
int pevlm_oracle_threads(void) { return 1; }
#endif
