/*
 * Sanitizer run of the CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Includes tensair_oracle.c and drives every exported function over small inputs that reach
 * its edges (stream start and end, a partial mini-batch, empty sources, ids at both ends of
 * the vocabulary, zero-count words, both table types, the variants).  Built by the CPU test
 * suite with gcc -fsanitize=address,undefined and run as a program of its own: an access
 * outside an allocation, a leak, a signed overflow or a misaligned access ends it with a
 * report and a non-zero status.  It checks memory behaviour, not values (the pins do that).
 */
#include "tensair_oracle.c"

#include <stdio.h>

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s >> 8; }

static int run(int dtype, int64_t V, int32_t D, int32_t stride, int64_t T, int32_t w, int32_t N)
{
    uint32_t seed = 12345u + (uint32_t)V + (uint32_t)D;
    int32_t *tok = malloc(sizeof(int32_t) * (size_t)T);
    uint64_t *counts = calloc((size_t)V, sizeof(uint64_t));
    for (int64_t i = 0; i < T; ++i) {
        uint32_t r = lcg(&seed) % (uint32_t)V, r2 = lcg(&seed) % (uint32_t)V;
        tok[i] = (int32_t)(r < r2 ? r : r2);            /* skewed towards small ids */
        if (V > 3 && tok[i] == 2) tok[i] = 1;            /* word 2 never occurs: a zero count */
        counts[tok[i]]++;
    }
    uint32_t *thr = malloc(sizeof(uint32_t) * (size_t)V);
    int32_t *alias = malloc(sizeof(int32_t) * (size_t)V);
    if (orc_alias_build(counts, V, thr, alias) != 0) return 1;
    const size_t esz = dtype == ORC_F32 ? 4 : (dtype == ORC_BF16 ? 2 : 8);
    void *W_in = calloc((size_t)V * (size_t)stride, esz), *W_out = calloc((size_t)V * (size_t)stride, esz);
    orc_init_tables(V, D, stride, dtype, 77u, W_in, W_out);
    /* mini-batches at the stream start, in the middle, and the partial one at the end */
    const int64_t begins[3] = {0, T / 2, T - 3};
    const int32_t counts_c[3] = {5, 7, 3};
    for (int b = 0; b < 3; ++b) {
        int64_t P = orc_pairs(T, w, begins[b], counts_c[b], NULL, NULL);
        int64_t *pos = malloc(sizeof(int64_t) * (size_t)(P + 1));
        int32_t *q = malloc(sizeof(int32_t) * (size_t)(P + 1));
        orc_pairs(T, w, begins[b], counts_c[b], pos, q);
        int32_t *neg = malloc(sizeof(int32_t) * (size_t)(P * N + 1));
        orc_sample_negatives(V, thr, alias, 99u, 3u, 1u, P, pos, q, N, neg);
        orc_sample_negatives_resampled(V, thr, alias, 99u, 3u, 1u, P, pos, q, N, tok, w, neg);
        for (int pass = 0; pass < 2; ++pass) {           /* drawn negatives, then given ones */
            orc_grad *G = orc_sgns_grad(tok, T, w, N, begins[b], counts_c[b], V, D, stride, dtype, W_in, W_out,
                                        thr, alias, 99u, 3u, 1u, pass ? neg : NULL);
            int64_t Pg, Ui, Uo;
            orc_grad_sizes(G, &Pg, &Ui, &Uo);
            if (Pg != P) return 2;
            int32_t *ii = malloc(sizeof(int32_t) * (size_t)(Ui + 1)), *io = malloc(sizeof(int32_t) * (size_t)(Uo + 1));
            float *ri = malloc(sizeof(float) * (size_t)(Ui * D + 1)), *ro = malloc(sizeof(float) * (size_t)(Uo * D + 1));
            double *di = malloc(sizeof(double) * (size_t)(Ui * D + 1)), *dq = malloc(sizeof(double) * (size_t)(Uo * D + 1));
            int64_t *si = malloc(sizeof(int64_t) * (size_t)(Ui + 1)), *so = malloc(sizeof(int64_t) * (size_t)(Uo + 1));
            int32_t *ng = malloc(sizeof(int32_t) * (size_t)(P * N + 1));
            orc_grad_export(G, ii, ri, di, si, io, ro, dq, so, ng);
            (void)orc_grad_loss(G);
            /* apply_gradient: the own gradient, an empty source, and one that lists the first and last word */
            int32_t edge_ids[2] = {0, (int32_t)(V - 1)};
            float *edge_rows = calloc((size_t)(2 * D), sizeof(float));
            for (int e = 0; e < 2 * D; ++e) edge_rows[e] = 0.25f * (float)(e % 5);
            const int64_t n_in[3] = {Ui, 0, V > 1 ? 2 : 1}, n_out[3] = {Uo, 0, V > 1 ? 2 : 1};
            const int32_t *ids_in[3] = {ii, NULL, edge_ids}, *ids_out[3] = {io, NULL, edge_ids};
            const float *rows_in[3] = {ri, NULL, edge_rows}, *rows_out[3] = {ro, NULL, edge_rows};
            orc_dasgd_apply_table(V, D, stride, dtype, W_in, 3, n_in, ids_in, rows_in, 0.025f);
            orc_dasgd_apply_table_sr(V, D, stride, dtype, W_out, 3, n_out, ids_out, rows_out, 0.025f, 5u, (uint32_t)b, 1u);
            free(edge_rows); free(ii); free(io); free(ri); free(ro); free(di); free(dq); free(si); free(so); free(ng);
            orc_grad_free(G);
        }
        free(pos); free(q); free(neg);
    }
    free(tok); free(counts); free(thr); free(alias); free(W_in); free(W_out);
    return 0;
}

int main(void)
{
    uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
    orc_philox4x32_10(ctr, key, out);
    (void)orc_double_to_bf16(1.00390625);
    int rc = 0;
    rc |= run(ORC_F32, 37, 8, 8, 200, 2, 3);
    rc |= run(ORC_BF16, 64, 12, 16, 150, 3, 2);          /* padded rows */
    rc |= run(ORC_F64, 5, 4, 4, 60, 1, 0);               /* no negatives */
    rc |= run(ORC_F32, 1, 4, 4, 20, 2, 2);               /* a one-word vocabulary */
    printf(rc ? "sanitize_check: FAILED %d\n" : "sanitize_check: ok\n", rc);
    return rc;
}
