/* Runs every exported routine of the CPU oracle on small ragged inputs.  Built by
 * tests/test_oracle_sanitizers.py together with oracle/pevlm_oracle.c under
 * -fsanitize=address,undefined: any out-of-bounds access, use of freed memory, signed overflow or
 * misaligned access in the oracle aborts the run.  It checks no values (the pins do that). */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int32_t num_seqs;
    const int32_t *cu_seqlens, *sink_len, *block_len, *ctx_len, *query_len, *window_blocks;
} oracle_layout;

int pevlm_oracle_check_layout(const oracle_layout *);
void pevlm_oracle_mask_row(const oracle_layout *, int64_t, int, uint8_t *);
void pevlm_oracle_positions(const oracle_layout *, const int32_t *, int32_t *);
void pevlm_oracle_rope(const void *, int, int64_t, int32_t, int32_t, const int32_t *, double, const int64_t *, int64_t, double *);
void pevlm_oracle_rope_mrope(const void *, int, int64_t, int32_t, int32_t, const int32_t *, const int32_t *, double,
                             const int64_t *, int64_t, double *);
void pevlm_oracle_attn(const double *, const double *, const void *, int, const oracle_layout *, int32_t, int32_t, int32_t,
                       const int32_t *, double, const int64_t *, int64_t, int64_t, int64_t, int, int, double *, double *);

static double rnd(uint32_t *st)
{
    *st = *st * 1664525u + 1013904223u;
    return ((double)(*st >> 8) / 8388608.0) - 1.0;
}

int main(void)
{
    /* three packed sequences: partial last block, no sink, no context */
    enum { NS = 3, HQ = 4, HKV = 2, D = 8 };
    const int32_t S[NS] = {3, 0, 4}, B[NS] = {5, 2, 1}, C[NS] = {13, 6, 0}, Q[NS] = {2, 1, 3}, W[NS] = {1, -1, 0};
    int32_t cu[NS + 1] = {0};
    for (int s = 0; s < NS; ++s) cu[s + 1] = cu[s] + S[s] + C[s] + Q[s];
    const int64_t T = cu[NS];
    oracle_layout lay = {NS, cu, S, B, C, Q, NULL}, layw = {NS, cu, S, B, C, Q, W};
    if (pevlm_oracle_check_layout(&lay) != 0) return 2;

    uint32_t st = 7;
    float *qf = malloc(sizeof(float) * T * HQ * D);
    uint16_t *kb = malloc(sizeof(uint16_t) * T * HKV * D);
    double *vd = malloc(sizeof(double) * T * HKV * D);
    for (int64_t i = 0; i < T * HQ * D; ++i) qf[i] = (float)rnd(&st);
    for (int64_t i = 0; i < T * HKV * D; ++i) {
        float f = (float)rnd(&st);
        uint32_t bits;
        __builtin_memcpy(&bits, &f, 4);
        kb[i] = (uint16_t)(bits >> 16);
        vd[i] = rnd(&st);
    }
    int32_t *pos = malloc(sizeof(int32_t) * T), *pos3 = malloc(sizeof(int32_t) * 3 * T);
    const int32_t off[NS] = {11, 0, 100000};
    pevlm_oracle_positions(&lay, NULL, pos);
    pevlm_oracle_positions(&lay, off, pos);
    for (int64_t t = 0; t < T; ++t) { pos3[t] = pos[t]; pos3[T + t] = pos[t] / 2; pos3[2 * T + t] = pos[t] % 3; }

    uint8_t *vis = malloc((size_t)T);
    for (int64_t t = 0; t < T; ++t) {
        pevlm_oracle_mask_row(&lay, t, 1, vis);
        pevlm_oracle_mask_row(&lay, t, 0, vis);
        pevlm_oracle_mask_row(&layw, t, 1, vis);
    }
    const int64_t rows[5] = {0, T - 1, 7, 19, 20};
    double *qr = malloc(sizeof(double) * 5 * HQ * D), *kr = malloc(sizeof(double) * T * HKV * D);
    double *q3 = malloc(sizeof(double) * T * HQ * D);
    const int32_t sec[3] = {1, 2, 1};
    pevlm_oracle_rope(qf, 0, T, HQ, D, pos, 1.0e6, rows, 5, qr);
    pevlm_oracle_rope(kb, 1, T, HKV, D, pos, 1.0e6, NULL, 0, kr);
    pevlm_oracle_rope_mrope(qf, 0, T, HQ, D, pos3, sec, 1.0e4, NULL, 0, q3);
    double *out = malloc(sizeof(double) * 5 * HQ * D), *lse = malloc(sizeof(double) * 5 * HQ);
    const int32_t map[HQ] = {1, 0, 0, 1};
    double acc = 0.0;
    for (int skip = 0; skip < 2; ++skip)
        for (int causal = 0; causal < 2; ++causal) {
            pevlm_oracle_attn(qr, kr, vd, 2, &lay, HQ, HKV, D, NULL, 0.0, rows, 5, 0, T, causal, skip, out, lse);
            pevlm_oracle_attn(qr, kr, kb, 1, &layw, HQ, HKV, D, map, 0.3, rows, 5, 2, T - 1, causal, skip, out, NULL);
            for (int i = 0; i < 5 * HQ * D; ++i) acc += out[i];
        }
    /* all rows in order (rows == NULL) */
    double *qall = malloc(sizeof(double) * T * HQ * D), *oall = malloc(sizeof(double) * T * HQ * D), *lall = malloc(sizeof(double) * T * HQ);
    pevlm_oracle_rope(qf, 0, T, HQ, D, pos, 1.0e6, NULL, 0, qall);
    pevlm_oracle_attn(qall, kr, vd, 2, &lay, HQ, HKV, D, NULL, 0.0, NULL, T, 0, T, 1, 1, oall, lall);
    for (int64_t i = 0; i < T * HQ * D; ++i) acc += oall[i];
    if (!isfinite(acc)) return 3;
    free(qf); free(kb); free(vd); free(pos); free(pos3); free(vis); free(qr); free(kr); free(q3); free(out); free(lse);
    free(qall); free(oall); free(lall);
    printf("oracle sanitizer driver ok %.6f\n", acc);
    return 0;
}
