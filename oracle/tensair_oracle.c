/*
 * CPU oracle for one DASGD worker step on a skip-gram/negative-sampling model.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, sequential, obviously
 * correct statement of what the step computes.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may build or call it; the product library
 * never does, and the two share no code.
 *
 * What it follows (TensAIR, arXiv 2211.10280):
 *   - Eq. 1                      theta_{t+1} = theta_t - alpha * grad L(X, theta_t)
 *   - Section 2.2                the split into gradient calculation (GC) and
 *                                gradient application (GA)
 *   - Algorithm 1, train()       own mini-batch: calculate_gradient then
 *                                apply_gradient; a peer's gradient message:
 *                                apply_gradient with the same alpha
 *   - Section 3.1                ordering: the own gradient is computed on the
 *                                model as it stands before the peer gradients of
 *                                the same step are applied
 *   - Section 4, "Sparse vs. Dense Models": only the rows a mini-batch touches
 *                                carry gradient, hence the {row_ids,row_grads} form
 * The paper names the model only as a default skip-gram word-embedding model;
 * the equations used here are the standard skip-gram with negative sampling
 * (logistic loss on <v_c, u_j>, no biases), mean over the pairs of the batch.
 *
 * All arithmetic is IEEE double; tables are stored in their own type (float,
 * bfloat16, or double for the finite-difference tests) and rounded once on
 * store, round-to-nearest-even.
 *
 * Pins (tests/test_oracle_*.py): Philox known answers, alias-table mass
 * invariant and chi-square, pair-count closed form and brute force, closed-form
 * losses with W_out = 0 and a hand-worked D = 2 example, central finite
 * differences, autograd of the same loss in a tensor library, dense brute-force
 * duplicate summation, Eq. 1 for K = 0, merged-vs-sequential apply, peer
 * permutation invariance, apply(g) then apply(-g), untouched rows bit-identical.
 * End-to-end trained values are "parity unpinned": the paper prints no numbers
 * for this model.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F64 = 2 };

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11).  Counter-based generator: 10 rounds of
 * two 32x32->64 multiplies with a Weyl-sequence key schedule.          */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------ */
/* Alias table (Vose) for the noise distribution count^0.75 / sum.
 * thr[i] is the acceptance threshold on a 32-bit uniform: a draw (b, r)
 * yields b if r < thr[b], else alias[b].  Returns 0, or -1 if no id has
 * a positive count.                                                    */
int orc_alias_build(const uint64_t *counts, int64_t V, uint32_t *thr, int32_t *alias)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    int64_t *small = (int64_t *)malloc(sizeof(int64_t) * (size_t)V);
    int64_t *large = (int64_t *)malloc(sizeof(int64_t) * (size_t)V);
    double total = 0.0;
    for (int64_t i = 0; i < V; ++i) {
        p[i] = pow((double)counts[i], 0.75);
        total += p[i];
    }
    if (!(total > 0.0)) { free(p); free(small); free(large); return -1; }
    int64_t ns = 0, nl = 0;
    for (int64_t i = 0; i < V; ++i) {
        p[i] = p[i] * (double)V / total;
        if (p[i] < 1.0) small[ns++] = i; else large[nl++] = i;
    }
    const double two32 = 4294967296.0;
    while (ns > 0 && nl > 0) {
        int64_t s = small[--ns];
        int64_t l = large[--nl];
        double t = floor(p[s] * two32);
        thr[s] = (t >= two32) ? 0xFFFFFFFFu : (uint32_t)t;
        alias[s] = (int32_t)l;
        p[l] = (p[l] + p[s]) - 1.0;
        if (p[l] < 1.0) small[ns++] = l; else large[nl++] = l;
    }
    while (nl > 0) { int64_t l = large[--nl]; thr[l] = 0xFFFFFFFFu; alias[l] = (int32_t)l; }
    while (ns > 0) { int64_t s = small[--ns]; thr[s] = 0xFFFFFFFFu; alias[s] = (int32_t)s; }
    free(p); free(small); free(large);
    return 0;
}

/* One negative: counter = (position low, position high, q*65536 + slot,
 * worker + 65536*epoch), key = seed.  Word 0 picks the bucket by
 * multiply-high, word 1 is compared with the threshold.                */
static void negative_words(uint64_t seed, uint32_t worker, uint32_t epoch,
                           int64_t pos, int32_t q, int32_t slot, uint32_t r[4])
{
    uint32_t ctr[4], key[2];
    ctr[0] = (uint32_t)((uint64_t)pos & 0xFFFFFFFFu);
    ctr[1] = (uint32_t)((uint64_t)pos >> 32);
    ctr[2] = (uint32_t)q * 65536u + (uint32_t)slot;
    ctr[3] = worker + 65536u * epoch;
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    orc_philox4x32_10(ctr, key, r);
}

static int32_t alias_pick(int64_t V, const uint32_t *thr, const int32_t *alias, uint32_t r_bucket, uint32_t r_accept)
{
    int64_t b = (int64_t)(((uint64_t)r_bucket * (uint64_t)V) >> 32);
    return (r_accept < thr[b]) ? (int32_t)b : alias[b];
}

static int32_t draw_negative(int64_t V, const uint32_t *thr, const int32_t *alias,
                             uint64_t seed, uint32_t worker, uint32_t epoch,
                             int64_t pos, int32_t q, int32_t slot)
{
    uint32_t r[4];
    negative_words(seed, worker, epoch, pos, q, slot, r);
    return alias_pick(V, thr, alias, r[0], r[1]);
}

/* ------------------------------------------------------------------ */
/* Pair enumeration: centers p = begin .. begin+n-1 ascending; for each,
 * offsets -w..-1 then +1..+w (index q = 0..2w-1), kept if inside [0,T). */
int64_t orc_pairs(int64_t T, int32_t w, int64_t begin, int32_t n,
                  int64_t *pos_out, int32_t *q_out)
{
    int64_t P = 0;
    for (int64_t p = begin; p < begin + n; ++p) {
        for (int32_t q = 0; q < 2 * w; ++q) {
            int64_t o = (q < w) ? (int64_t)q - w : (int64_t)q - w + 1;
            int64_t x = p + o;
            if (x < 0 || x >= T) continue;
            if (pos_out) pos_out[P] = p;
            if (q_out) q_out[P] = q;
            ++P;
        }
    }
    return P;
}

void orc_sample_negatives(int64_t V, const uint32_t *thr, const int32_t *alias,
                          uint64_t seed, uint32_t worker, uint32_t epoch,
                          int64_t P, const int64_t *pos, const int32_t *q,
                          int32_t N, int32_t *neg_out)
{
    for (int64_t i = 0; i < P; ++i)
        for (int32_t k = 0; k < N; ++k)
            neg_out[i * N + k] = draw_negative(V, thr, alias, seed, worker, epoch, pos[i], q[i], k);
}

/* A variant the paper leaves open (it does not say what happens when a negative
 * equals the pair's center or context word; the base reading keeps it): such a
 * negative is drawn again, once, from words 2 and 3 of the same Philox block, and
 * the second draw is kept whatever it is -- still a pure function of the counter,
 * with fixed shapes.  tok: the token stream; the pair (pos, q) has center tok[pos]
 * and context tok[pos + offset(q)].                                              */
void orc_sample_negatives_resampled(int64_t V, const uint32_t *thr, const int32_t *alias,
                                    uint64_t seed, uint32_t worker, uint32_t epoch,
                                    int64_t P, const int64_t *pos, const int32_t *q,
                                    int32_t N, const int32_t *tok, int32_t w, int32_t *neg_out)
{
    for (int64_t i = 0; i < P; ++i) {
        int64_t o = (q[i] < w) ? (int64_t)q[i] - w : (int64_t)q[i] - w + 1;
        int32_t center = tok[pos[i]], context = tok[pos[i] + o];
        for (int32_t k = 0; k < N; ++k) {
            uint32_t r[4];
            negative_words(seed, worker, epoch, pos[i], q[i], k, r);
            int32_t id = alias_pick(V, thr, alias, r[0], r[1]);
            if (id == center || id == context) id = alias_pick(V, thr, alias, r[2], r[3]);
            neg_out[i * N + k] = id;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Table element access.                                                */
static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bfloat16, one rounding, ties to even.  bfloat16 = sign, 8
 * exponent bits (bias 127), 7 fraction bits; subnormals step 2^-133.    */
static uint16_t double_to_bf16(double x)
{
    if (isnan(x)) return 0x7FC0u;
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    int e;
    (void)frexp(a, &e);              /* a = m * 2^e, m in [0.5,1) -> exponent of leading bit is e-1 */
    int lead = e - 1;
    if (lead < -126) lead = -126;    /* subnormal range shares the quantum of the lowest normal binade */
    double quantum = ldexp(1.0, lead - 7);
    double k = nearbyint(a / quantum);      /* exact scaling, RNE in the default rounding mode */
    double r = k * quantum;
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    float f = (float)r;              /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(sign | (uint16_t)(u >> 16));
}

static double tab_get(const void *W, int dtype, int64_t idx)
{
    if (dtype == ORC_F32) return (double)((const float *)W)[idx];
    if (dtype == ORC_BF16) return bf16_to_double(((const uint16_t *)W)[idx]);
    return ((const double *)W)[idx];
}

static void tab_set(void *W, int dtype, int64_t idx, double x)
{
    if (dtype == ORC_F32) ((float *)W)[idx] = (float)x;
    else if (dtype == ORC_BF16) ((uint16_t *)W)[idx] = double_to_bf16(x);
    else ((double *)W)[idx] = x;
}

uint16_t orc_double_to_bf16(double x) { return double_to_bf16(x); }

/* ------------------------------------------------------------------ */
/* Initialisation: W_in ~ U(-0.5/D, 0.5/D), W_out = 0.  Element i = row*D + col
 * takes word (i mod 4) of Philox(counter = (i/4 low, i/4 high, 0, 'INIT'), seed);
 * the 24 high bits make u in [0,1); the value is (u - 0.5) * (1/D) evaluated in
 * single precision (every operation is exactly rounded, so any conforming
 * implementation produces the same bits), then rounded to the table type.       */
void orc_init_tables(int64_t V, int32_t D, int32_t stride, int dtype, uint64_t seed,
                     void *w_in, void *w_out)
{
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    const float invD = 1.0f / (float)D;
    for (int64_t r = 0; r < V; ++r) {
        for (int32_t c = 0; c < stride; ++c) {
            int64_t at = r * (int64_t)stride + c;
            if (c >= D) { tab_set(w_in, dtype, at, 0.0); tab_set(w_out, dtype, at, 0.0); continue; }
            uint64_t i = (uint64_t)r * (uint64_t)D + (uint64_t)c;
            uint64_t blk = i >> 2;
            uint32_t ctr[4] = { (uint32_t)(blk & 0xFFFFFFFFu), (uint32_t)(blk >> 32), 0u, 0x494E4954u };
            uint32_t out[4];
            orc_philox4x32_10(ctr, key, out);
            float u = (float)(out[i & 3] >> 8) * 0x1p-24f;
            float val = (u - 0.5f) * invD;
            tab_set(w_in, dtype, at, (double)val);
            tab_set(w_out, dtype, at, 0.0);
        }
    }
}

/* ------------------------------------------------------------------ */
/* Sparse row accumulator: rows appear in first-touch order and are sorted
 * by id on export.                                                      */
typedef struct {
    int64_t V; int32_t D;
    int32_t *slot;      /* [V], -1 = untouched */
    int64_t *ids;       /* [n] */
    int64_t *occ;       /* [n] number of occurrences */
    double *rows;       /* [n][D] */
    int64_t n, cap;
} rowacc;

static void rowacc_init(rowacc *a, int64_t V, int32_t D)
{
    a->V = V; a->D = D; a->n = 0; a->cap = 1024;
    a->slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)V);
    for (int64_t i = 0; i < V; ++i) a->slot[i] = -1;
    a->ids = (int64_t *)malloc(sizeof(int64_t) * (size_t)a->cap);
    a->occ = (int64_t *)malloc(sizeof(int64_t) * (size_t)a->cap);
    a->rows = (double *)malloc(sizeof(double) * (size_t)a->cap * (size_t)D);
}

static double *rowacc_touch(rowacc *a, int64_t id)
{
    int32_t s = a->slot[id];
    if (s < 0) {
        if (a->n == a->cap) {
            a->cap *= 2;
            a->ids = (int64_t *)realloc(a->ids, sizeof(int64_t) * (size_t)a->cap);
            a->occ = (int64_t *)realloc(a->occ, sizeof(int64_t) * (size_t)a->cap);
            a->rows = (double *)realloc(a->rows, sizeof(double) * (size_t)a->cap * (size_t)a->D);
        }
        s = (int32_t)a->n++;
        a->slot[id] = s;
        a->ids[s] = id;
        a->occ[s] = 0;
        memset(a->rows + (size_t)s * a->D, 0, sizeof(double) * (size_t)a->D);
    }
    return a->rows + (size_t)s * a->D;
}

static void rowacc_free(rowacc *a)
{
    free(a->slot); free(a->ids); free(a->occ); free(a->rows);
}

static int cmp_i64(const void *x, const void *y)
{
    int64_t a = *(const int64_t *)x, b = *(const int64_t *)y;
    return (a > b) - (a < b);
}

/* ------------------------------------------------------------------ */
typedef struct {
    int64_t P;            /* pairs in the batch */
    int32_t N, D;
    double loss;          /* mean over the P pairs */
    int32_t *negatives;   /* [P][N] */
    rowacc in, out;
    int64_t *in_sorted, *out_sorted;   /* ids ascending */
} orc_grad;

/* Gradient calculation (GC) of one mini-batch: Algorithm 1, calculate_gradient.
 * Per pair (c, x) and j in {x, neg_0..neg_{N-1}}: s = <W_in[c], W_out[j]>,
 * sigma = 1/(1+exp(-s)), g = (sigma - label)/P, Gin[c] += g*W_out[j],
 * Gout[j] += g*W_in[c]; loss += softplus(-s) for the context, softplus(s) for a
 * negative, divided by P.  Every read uses the tables as given (theta_t).
 * neg_override, if not NULL, supplies the negatives [P][N] instead of drawing
 * them (used to hold them fixed under finite differences).                      */
orc_grad *orc_sgns_grad(const int32_t *tok, int64_t T, int32_t w, int32_t N,
                        int64_t begin, int32_t n_centers,
                        int64_t V, int32_t D, int32_t stride, int dtype,
                        const void *W_in, const void *W_out,
                        const uint32_t *thr, const int32_t *alias,
                        uint64_t seed, uint32_t worker, uint32_t epoch,
                        const int32_t *neg_override)
{
    orc_grad *G = (orc_grad *)calloc(1, sizeof(orc_grad));
    G->N = N; G->D = D;
    int64_t P = orc_pairs(T, w, begin, n_centers, NULL, NULL);
    G->P = P;
    int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)(P > 0 ? P : 1));
    int32_t *qq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    orc_pairs(T, w, begin, n_centers, pos, qq);
    G->negatives = (int32_t *)malloc(sizeof(int32_t) * (size_t)(P * N > 0 ? P * N : 1));
    if (neg_override) memcpy(G->negatives, neg_override, sizeof(int32_t) * (size_t)(P * N));
    else orc_sample_negatives(V, thr, alias, seed, worker, epoch, P, pos, qq, N, G->negatives);

    rowacc_init(&G->in, V, D);
    rowacc_init(&G->out, V, D);
    double *v = (double *)malloc(sizeof(double) * (size_t)D);
    double *u = (double *)malloc(sizeof(double) * (size_t)D);
    double loss = 0.0;
    for (int64_t i = 0; i < P; ++i) {
        int64_t p = pos[i];
        int32_t q = qq[i];
        int64_t o = (q < w) ? (int64_t)q - w : (int64_t)q - w + 1;
        int64_t c = tok[p], x = tok[p + o];
        for (int32_t d = 0; d < D; ++d) v[d] = tab_get(W_in, dtype, c * (int64_t)stride + d);
        double *gin = rowacc_touch(&G->in, c);
        G->in.occ[G->in.slot[c]] += 1;
        for (int32_t k = 0; k <= N; ++k) {
            int64_t j = (k == 0) ? x : (int64_t)G->negatives[i * N + (k - 1)];
            double label = (k == 0) ? 1.0 : 0.0;
            for (int32_t d = 0; d < D; ++d) u[d] = tab_get(W_out, dtype, j * (int64_t)stride + d);
            double s = 0.0;
            for (int32_t d = 0; d < D; ++d) s += v[d] * u[d];
            double sigma = 1.0 / (1.0 + exp(-s));
            double g = (sigma - label) / (double)P;
            double z = (k == 0) ? -s : s;                 /* loss term = softplus(z) */
            loss += (fmax(z, 0.0) + log1p(exp(-fabs(z)))) / (double)P;
            double *gout = rowacc_touch(&G->out, j);
            gin = G->in.rows + (size_t)G->in.slot[c] * D;  /* touch may not move 'in', but stay safe */
            G->out.occ[G->out.slot[j]] += 1;
            for (int32_t d = 0; d < D; ++d) { gin[d] += g * u[d]; gout[d] += g * v[d]; }
        }
    }
    G->loss = loss;
    G->in_sorted = (int64_t *)malloc(sizeof(int64_t) * (size_t)(G->in.n > 0 ? G->in.n : 1));
    G->out_sorted = (int64_t *)malloc(sizeof(int64_t) * (size_t)(G->out.n > 0 ? G->out.n : 1));
    memcpy(G->in_sorted, G->in.ids, sizeof(int64_t) * (size_t)G->in.n);
    memcpy(G->out_sorted, G->out.ids, sizeof(int64_t) * (size_t)G->out.n);
    qsort(G->in_sorted, (size_t)G->in.n, sizeof(int64_t), cmp_i64);
    qsort(G->out_sorted, (size_t)G->out.n, sizeof(int64_t), cmp_i64);
    free(pos); free(qq); free(v); free(u);
    return G;
}

void orc_grad_sizes(const orc_grad *G, int64_t *P, int64_t *U_in, int64_t *U_out)
{
    *P = G->P; *U_in = G->in.n; *U_out = G->out.n;
}

double orc_grad_loss(const orc_grad *G) { return G->loss; }

static void export_side(const rowacc *a, const int64_t *sorted, int32_t *ids, float *rows32,
                        double *rows64, int64_t *seg)
{
    int64_t run = 0;
    for (int64_t i = 0; i < a->n; ++i) {
        int64_t id = sorted[i];
        int32_t s = a->slot[id];
        if (ids) ids[i] = (int32_t)id;
        if (seg) seg[i] = run;
        run += a->occ[s];
        const double *src = a->rows + (size_t)s * a->D;
        if (rows32) for (int32_t d = 0; d < a->D; ++d) rows32[i * (int64_t)a->D + d] = (float)src[d];
        if (rows64) for (int32_t d = 0; d < a->D; ++d) rows64[i * (int64_t)a->D + d] = src[d];
    }
    if (seg) seg[a->n] = run;
}

/* Sparse form: ids ascending and unique; rows cast to float (the message
 * payload type) and, optionally, in double; seg[i] = number of occurrences with
 * id below ids[i] (in-side: one occurrence per pair; out-side: N+1 per pair),
 * seg[U] = total.  Any pointer may be NULL.                                     */
void orc_grad_export(const orc_grad *G,
                     int32_t *in_ids, float *in_rows, double *in_rows64, int64_t *in_seg,
                     int32_t *out_ids, float *out_rows, double *out_rows64, int64_t *out_seg,
                     int32_t *negatives)
{
    export_side(&G->in, G->in_sorted, in_ids, in_rows, in_rows64, in_seg);
    export_side(&G->out, G->out_sorted, out_ids, out_rows, out_rows64, out_seg);
    if (negatives) memcpy(negatives, G->negatives, sizeof(int32_t) * (size_t)(G->P * G->N));
}

void orc_grad_free(orc_grad *G)
{
    rowacc_free(&G->in); rowacc_free(&G->out);
    free(G->negatives); free(G->in_sorted); free(G->out_sorted); free(G);
}

/* ------------------------------------------------------------------ */
/* Gradient application (GA), Eq. 1, for one table and n_src sparse gradients
 * (source 0 = own, 1..K = peers; Algorithm 1 applies each with the same alpha,
 * so the sources are summed, not averaged).  Because the update is linear in
 * the gradients and all of them exist before the step, the K+1 applications
 * are merged: G[r] = sum_k g_k[r] in double, then one rounded store
 * W[r] = round(W[r] - alpha*G[r]).  Rows outside the union are not written.
 * alpha is a float on the interface; it enters as (double)(float)lr.            */
/* sr != 0: the variant with stochastic rounding of bfloat16 tables (the paper leaves the
 * rounding open; the base reading is round-to-nearest-even).  The new value is taken
 * to single precision (nearest even), 16 random bits are added to its bit pattern below
 * the bfloat16 mantissa and the result is truncated, so the value goes up with
 * probability (discarded bits)/2^16 and the expectation is the single-precision value.
 * The bits of element i = row*D + col are the low half of word (i mod 4) of
 * Philox(counter = (i/4 low, i/4 high, serial, 'SRND' + table), key = seed); serial
 * counts the model's table updates, table is 0 for W_in and 1 for W_out.  Infinities
 * and NaN are kept.                                                                  */
static uint16_t stochastic_bf16(double x, uint64_t seed, uint32_t serial, uint32_t table, uint64_t i)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u)
        return (uint16_t)((u >> 16) | ((u & 0xFFFFu) ? 0x40u : 0u));
    uint64_t blk = i >> 2;
    uint32_t ctr[4] = { (uint32_t)(blk & 0xFFFFFFFFu), (uint32_t)(blk >> 32), serial, 0x53524E44u + table };
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return (uint16_t)((u + (out[i & 3] & 0xFFFFu)) >> 16);
}

static void apply_table(int64_t V, int32_t D, int32_t stride, int dtype, void *W,
                        int32_t n_src, const int64_t *n_rows,
                        const int32_t *const *ids, const float *const *rows, float lr,
                        int sr, uint64_t seed, uint32_t serial, uint32_t table)
{
    rowacc acc;
    rowacc_init(&acc, V, D);
    for (int32_t k = 0; k < n_src; ++k) {
        for (int64_t i = 0; i < n_rows[k]; ++i) {
            double *dst = rowacc_touch(&acc, ids[k][i]);
            const float *src = rows[k] + i * (int64_t)D;
            for (int32_t d = 0; d < D; ++d) dst[d] += (double)src[d];
        }
    }
    const double alpha = (double)lr;
    for (int64_t s = 0; s < acc.n; ++s) {
        int64_t r = acc.ids[s];
        const double *g = acc.rows + (size_t)s * D;
        for (int32_t d = 0; d < D; ++d) {
            int64_t at = r * (int64_t)stride + d;
            double nv = tab_get(W, dtype, at) - alpha * g[d];
            if (sr && dtype == ORC_BF16)
                ((uint16_t *)W)[at] = stochastic_bf16(nv, seed, serial, table, (uint64_t)r * (uint64_t)D + (uint64_t)d);
            else
                tab_set(W, dtype, at, nv);
        }
    }
    rowacc_free(&acc);
}

void orc_dasgd_apply_table(int64_t V, int32_t D, int32_t stride, int dtype, void *W,
                           int32_t n_src, const int64_t *n_rows,
                           const int32_t *const *ids, const float *const *rows, float lr)
{
    apply_table(V, D, stride, dtype, W, n_src, n_rows, ids, rows, lr, 0, 0, 0, 0);
}

void orc_dasgd_apply_table_sr(int64_t V, int32_t D, int32_t stride, int dtype, void *W,
                              int32_t n_src, const int64_t *n_rows,
                              const int32_t *const *ids, const float *const *rows, float lr,
                              uint64_t seed, uint32_t serial, uint32_t table)
{
    apply_table(V, D, stride, dtype, W, n_src, n_rows, ids, rows, lr, 1, seed, serial, table);
}
