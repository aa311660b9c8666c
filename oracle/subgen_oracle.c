/*
 * SubGen CPU oracle — TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-stream, double-precision implementation of the
 * per-token decode step of SubGen (Algorithm 1 of the paper) in the
 * configuration the GPU library implements:
 *
 *   - UpdateSoftmaxNormalizer (Algorithm 1, procedure 1; Lemma 2): online
 *     threshold clustering of keys, one representative and one count per
 *     cluster.  With t = 0 ("representative mode") the per-cluster reservoir
 *     S_i is collapsed to the representative x_i, so the softmax normaliser
 *     is tau = sum_i n_i * exp(<q, x_i>).  With t >= 1 the procedure is the
 *     paper's: S_i holds t uniform samples of the cluster (each slot replaced
 *     with probability 1/n_i on a join, t copies on creation; Lemma 2 (5)) and
 *     tau = sum_i (n_i / t) sum_{k in S_i} exp(<q, k>).
 *   - UpdateMatrixProduct (Algorithm 1, procedure 2; Lemma 1): s independent
 *     slots, each overwritten with probability ||v||^2 / (mu + ||v||^2),
 *     followed by mu += ||v||^2 (main loop of Algorithm 1).
 *   - QueryStreamAttn (Algorithm 1, procedure 3): z / tau, with the exact
 *     contribution of a sliding window of the w most recent tokens
 *     (Section 3.2: recent tokens are retained, the rest is compressed).
 *
 * Only tests, the smoke check and the bench's cpu-baseline leg may use this
 * file.  It shares no code with the HIP library.  Inputs are float arrays
 * that already hold the rounded (bf16 or fp32) values; all arithmetic below
 * is double precision, in the plain order the formulas are written in.
 *
 * Parity pins (tests, no GPU): Philox known-answer vectors; delta = 0 gives
 * the exact partition function; Lemma 2 invariants; separated-groups center
 * count; Lemma 1 sampling frequencies; unbiasedness of the numerator;
 * closed forms (single token, n <= w equals textbook softmax attention).
 * Per-seed sampled indices are "parity unpinned" against the paper (it
 * fixes no random number generator); they are pinned distributionally.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------
 * Counter-based random numbers: Philox-4x32 with 10 rounds (Salmon, Moraes,
 * Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11).
 * Stands in for the "flip a coin" of Algorithm 1 (procedure 2).
 * ---------------------------------------------------------------------- */
static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {           /* Weyl sequence on the key */
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void sgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    philox4x32_10(ctr, key, out);
}

/* 24-bit uniform in [0,1) for (seed, stream, token, slot): slot j uses word
 * j mod 4 of the block whose counter is (j div 4, token lo, token hi, stream). */
float sgo_uniform24(uint64_t seed, uint32_t stream, uint64_t token, uint32_t slot)
{
    uint32_t ctr[4] = { slot / 4u, (uint32_t)token, (uint32_t)(token >> 32), stream };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    philox4x32_10(ctr, key, r);
    return (float)(r[slot % 4u] >> 8) * (1.0f / 16777216.0f);
}

/* Coins of the per-cluster reservoirs (UpdateSoftmaxNormalizer): same generator, a disjoint counter
 * domain (top bit of the third counter word set), slot j of the reservoir of the cluster the token joins. */
float sgo_uniform24_res(uint64_t seed, uint32_t stream, uint64_t token, uint32_t slot)
{
    uint32_t ctr[4] = { slot / 4u, (uint32_t)token, (uint32_t)(token >> 32) | 0x80000000u, stream };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    philox4x32_10(ctr, key, r);
    return (float)(r[slot % 4u] >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------------
 * State of one stream
 * ---------------------------------------------------------------------- */
typedef struct sgo_stream {
    int d, s, w;
    int t;                    /* reservoir slots per cluster; 0 = representative mode */
    int max_centers;          /* 0 = unbounded */
    double delta;
    uint64_t seed;
    uint32_t stream;

    int64_t n_seen;           /* tokens given to update() so far          */
    int64_t n_evicted;        /* tokens that left the window (compressed) */

    /* sliding window: slot (token mod w) holds that token while it is among the last w */
    float *win_k, *win_v;
    int64_t *win_idx;

    /* D = {(x_i, n_i)}: representatives and counts */
    float *X;
    int64_t *cnt;
    float *R;                 /* [cap][t][d]: per-cluster reservoirs S_i (t >= 1) */
    int m, cap;

    /* M: s sampled (k, v) pairs, the token each came from, its ||v||^2 */
    float *Mk, *Mv;
    int64_t *Midx;            /* -1 = null slot */
    float *Mvn;
    double mu;

    /* decision log, one entry per evicted token */
    int32_t *assign;          /* center index the token was assigned to      */
    uint8_t *created;         /* 1 if the token opened that center           */
    double *dist1;            /* squared distance to the nearest center (inf if none) */
    double *dist2;            /* squared distance to the runner-up (inf if none)      */
    int64_t log_cap;

    int overflowed;           /* a token was force-joined because max_centers was hit */
    int64_t dropped;          /* tokens with NaN/Inf that were dropped when they left the window */

    /* near-tie protocol of the parity harness: decisions forced from outside, sorted by token */
    int64_t *ov_token;
    int32_t *ov_decision;     /* >= 0: join that cluster; SGO_FORCE_NEW: open a new cluster */
    int64_t n_ov, ov_used;
} sgo_stream;

#define SGO_FORCE_NEW (-2)

sgo_stream *sgo_create(int d, double delta, int s, int w, uint64_t seed, uint32_t stream, int max_centers, int t)
{
    if (d < 1 || s < 1 || w < 0 || t < 0 || !(delta >= 0.0)) return NULL;
    sgo_stream *o = (sgo_stream *)calloc(1, sizeof(sgo_stream));
    if (!o) return NULL;
    o->d = d; o->s = s; o->w = w; o->t = t; o->max_centers = max_centers;
    o->delta = delta; o->seed = seed; o->stream = stream;
    o->win_k = (float *)calloc((size_t)(w > 0 ? w : 1) * d, sizeof(float));
    o->win_v = (float *)calloc((size_t)(w > 0 ? w : 1) * d, sizeof(float));
    o->win_idx = (int64_t *)calloc((size_t)(w > 0 ? w : 1), sizeof(int64_t));
    o->Mk = (float *)calloc((size_t)s * d, sizeof(float));
    o->Mv = (float *)calloc((size_t)s * d, sizeof(float));
    o->Midx = (int64_t *)malloc((size_t)s * sizeof(int64_t));
    o->Mvn = (float *)calloc((size_t)s, sizeof(float));
    for (int j = 0; j < s; ++j) o->Midx[j] = -1;
    return o;
}

void sgo_destroy(sgo_stream *o)
{
    if (!o) return;
    free(o->win_k); free(o->win_v); free(o->win_idx);
    free(o->X); free(o->cnt); free(o->R);
    free(o->Mk); free(o->Mv); free(o->Midx); free(o->Mvn);
    free(o->assign); free(o->created); free(o->dist1); free(o->dist2);
    free(o->ov_token); free(o->ov_decision);
    free(o);
}

/* The paper's algorithm is stated over the reals; in floating point a distance can sit so close to delta, or
 * two distances so close to each other, that two correct implementations decide differently.  A parity harness
 * that has checked that such a decision of the other implementation lies inside the near-tie margin can force
 * it here and replay the stream, so that everything after that token is still compared.  tokens[] must be
 * strictly increasing; decision >= 0 joins that (existing) cluster, SGO_FORCE_NEW opens a new one.  Must be
 * called before the first update.  Returns 0, or -1 on bad arguments. */
int sgo_set_overrides(sgo_stream *o, const int64_t *tokens, const int32_t *decisions, int64_t n)
{
    if (!o || n < 0 || o->n_seen != 0) return -1;
    for (int64_t i = 0; i < n; ++i) {
        if (tokens[i] < 0 || (i > 0 && tokens[i] <= tokens[i - 1])) return -1;
        if (decisions[i] < 0 && decisions[i] != SGO_FORCE_NEW) return -1;
    }
    free(o->ov_token); free(o->ov_decision);
    o->ov_token = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    o->ov_decision = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (n > 0) {
        memcpy(o->ov_token, tokens, (size_t)n * sizeof(int64_t));
        memcpy(o->ov_decision, decisions, (size_t)n * sizeof(int32_t));
    }
    o->n_ov = n; o->ov_used = 0;
    return 0;
}

int64_t sgo_overrides_used(const sgo_stream *o) { return o->ov_used; }

static void append_center(sgo_stream *o, const float *k)
{
    if (o->m == o->cap) {
        int ncap = o->cap ? 2 * o->cap : 64;
        o->X = (float *)realloc(o->X, (size_t)ncap * o->d * sizeof(float));
        o->cnt = (int64_t *)realloc(o->cnt, (size_t)ncap * sizeof(int64_t));
        if (o->t > 0) o->R = (float *)realloc(o->R, (size_t)ncap * o->t * o->d * sizeof(float));
        o->cap = ncap;
    }
    memcpy(o->X + (size_t)o->m * o->d, k, (size_t)o->d * sizeof(float));
    for (int j = 0; j < o->t; ++j)   /* a new cluster's reservoir is t copies of its first key */
        memcpy(o->R + ((size_t)o->m * o->t + j) * o->d, k, (size_t)o->d * sizeof(float));
    o->cnt[o->m] = 1;
    o->m += 1;
}

static void log_decision(sgo_stream *o, int32_t a, int is_new, double d1, double d2)
{
    if (o->n_evicted == o->log_cap) {
        int64_t ncap = o->log_cap ? 2 * o->log_cap : 1024;
        o->assign = (int32_t *)realloc(o->assign, (size_t)ncap * sizeof(int32_t));
        o->created = (uint8_t *)realloc(o->created, (size_t)ncap);
        o->dist1 = (double *)realloc(o->dist1, (size_t)ncap * sizeof(double));
        o->dist2 = (double *)realloc(o->dist2, (size_t)ncap * sizeof(double));
        o->log_cap = ncap;
    }
    o->assign[o->n_evicted] = a;
    o->created[o->n_evicted] = (uint8_t)is_new;
    o->dist1[o->n_evicted] = d1;
    o->dist2[o->n_evicted] = d2;
}

/* Algorithm 1, UpdateSoftmaxNormalizer, representative mode: nearest
 * representative (lowest index on ties), join iff ||k - x_i*||_2 <= delta
 * (tested on squared values), else open a new cluster whose representative
 * is k.  When a capacity is set and reached the token joins its nearest
 * cluster regardless of delta. */
/* On a join with t >= 1 every reservoir slot of that cluster is replaced by k with probability 1/n_i,
 * n_i being the count after the increment (reservoir sampling, Lemma 2 (5)). */
static void reservoir_update(sgo_stream *o, int i, int64_t token, const float *k)
{
    const float p = 1.0f / (float)o->cnt[i];
    for (int j = 0; j < o->t; ++j) {
        float u = sgo_uniform24_res(o->seed, o->stream, (uint64_t)token, (uint32_t)j);
        if (u < p) memcpy(o->R + ((size_t)i * o->t + j) * o->d, k, (size_t)o->d * sizeof(float));
    }
}

static void cluster_update(sgo_stream *o, int64_t token, const float *k)
{
    const int d = o->d;
    double best = INFINITY, second = INFINITY;
    int arg = -1;
    for (int i = 0; i < o->m; ++i) {
        const float *x = o->X + (size_t)i * d;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) {
            double df = (double)x[c] - (double)k[c];
            acc += df * df;
        }
        if (acc < best) { second = best; best = acc; arg = i; }
        else if (acc < second) { second = acc; }
    }
    const double thr = o->delta * o->delta;
    for (int64_t e = 0; e < o->n_ov; ++e) {          /* a decision forced by the parity harness (near-tie) */
        if (o->ov_token[e] != token) continue;
        const int32_t dec = o->ov_decision[e];
        o->ov_used += 1;
        if (dec == SGO_FORCE_NEW || dec >= o->m) {
            append_center(o, k);
            log_decision(o, o->m - 1, 1, best, second);
        } else {
            o->cnt[dec] += 1;
            reservoir_update(o, dec, token, k);
            log_decision(o, dec, 0, best, second);
        }
        return;
    }
    if (arg >= 0 && best <= thr) {
        o->cnt[arg] += 1;
        reservoir_update(o, arg, token, k);
        log_decision(o, arg, 0, best, second);
    } else if (arg >= 0 && o->max_centers > 0 && o->m >= o->max_centers) {
        o->cnt[arg] += 1;
        reservoir_update(o, arg, token, k);
        o->overflowed = 1;
        log_decision(o, arg, 0, best, second);
    } else {
        append_center(o, k);
        log_decision(o, o->m - 1, 1, best, second);
    }
}

/* Algorithm 1, UpdateMatrixProduct followed by the mu update of the main
 * loop: p uses the mu from before this token. */
static void sample_update(sgo_stream *o, int64_t token, const float *k, const float *v)
{
    const int d = o->d;
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += (double)v[c] * (double)v[c];
    const float vn = (float)acc;
    float p;
    if (o->mu == 0.0) p = 1.0f;
    else if (vn == 0.0f) p = 0.0f;
    else p = (float)((double)vn / (o->mu + (double)vn));
    for (int j = 0; j < o->s; ++j) {
        float u = sgo_uniform24(o->seed, o->stream, (uint64_t)token, (uint32_t)j);
        if (u < p) {
            memcpy(o->Mk + (size_t)j * d, k, (size_t)d * sizeof(float));
            memcpy(o->Mv + (size_t)j * d, v, (size_t)d * sizeof(float));
            o->Midx[j] = token;
            o->Mvn[j] = vn;
        }
    }
    o->mu += (double)vn;
}

/* The paper is silent on tokens that hold NaN or Inf.  Reading taken here:
 * a token whose squared key norm or squared value norm (double sums, then
 * rounded to fp32) is not finite is dropped at the moment it leaves the
 * window: it is neither clustered nor offered to the sampler, mu does not
 * move, and it is counted in `dropped`.  Its decision-log entry is -1. */
static void compress_token(sgo_stream *o, int64_t token, const float *k, const float *v)
{
    double kk = 0.0, vv = 0.0;
    for (int c = 0; c < o->d; ++c) {
        kk += (double)k[c] * (double)k[c];
        vv += (double)v[c] * (double)v[c];
    }
    if (!((float)kk < INFINITY) || !((float)vv < INFINITY)) {
        o->dropped += 1;
        log_decision(o, -1, 0, INFINITY, INFINITY);
        return;
    }
    cluster_update(o, token, k);
    sample_update(o, token, k, v);
}

/* One token arrives.  It enters the window; the token it pushes out (if
 * any) is the one that is clustered and offered to the sampler. */
void sgo_update(sgo_stream *o, const float *k, const float *v)
{
    const int d = o->d;
    const int64_t i = o->n_seen;
    o->n_seen += 1;
    if (o->w == 0) {
        compress_token(o, i, k, v);
        o->n_evicted += 1;
        return;
    }
    const int slot = (int)(i % o->w);
    if (i >= o->w) {
        const float *ek = o->win_k + (size_t)slot * d;
        const float *ev = o->win_v + (size_t)slot * d;
        const int64_t ei = o->win_idx[slot];
        compress_token(o, ei, ek, ev);
        o->n_evicted += 1;
    }
    memcpy(o->win_k + (size_t)slot * d, k, (size_t)d * sizeof(float));
    memcpy(o->win_v + (size_t)slot * d, v, (size_t)d * sizeof(float));
    o->win_idx[slot] = i;
}

static double dotd(const float *a, const float *b, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += (double)a[c] * (double)b[c];
    return acc;
}

/* QueryStreamAttn with the window:
 *   den = sum_{j in W} e^{<q,k_j>} + sum_i n_i e^{<q,x_i>}        (t = 0)
 *       = sum_{j in W} e^{<q,k_j>} + sum_i (n_i/t) sum_{k in S_i} e^{<q,k>}   (t >= 1)
 *   num = sum_{j in W} e^{<q,k_j>} v_j + sum_{j in [s]} mu/(s ||v_j||^2) e^{<q,k_j>} v_j
 * every exponent shifted by the largest score.  Returns 0, or -1 if no token
 * has been seen.  Optionally reports den*e^{mx} pieces for tests. */
int sgo_attend(const sgo_stream *o, const float *q, double *out, double *den_out, double *mx_out)
{
    const int d = o->d;
    if (o->n_seen == 0) return -1;
    const int wfill = (int)(o->n_seen < o->w ? o->n_seen : o->w);
    const int have_samples = o->n_evicted > 0;

    double mx = -INFINITY;
    for (int j = 0; j < wfill; ++j) {
        double a = dotd(q, o->win_k + (size_t)j * d, d);
        if (a > mx) mx = a;
    }
    if (o->t == 0) {
        for (int i = 0; i < o->m; ++i) {
            double b = dotd(q, o->X + (size_t)i * d, d);
            if (b > mx) mx = b;
        }
    } else {
        for (int r = 0; r < o->m * o->t; ++r) {
            double b = dotd(q, o->R + (size_t)r * d, d);
            if (b > mx) mx = b;
        }
    }
    if (have_samples)
        for (int j = 0; j < o->s; ++j) {
            double c = dotd(q, o->Mk + (size_t)j * d, d);
            if (c > mx) mx = c;
        }

    double den = 0.0;
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int j = 0; j < wfill; ++j) {
        double e = exp(dotd(q, o->win_k + (size_t)j * d, d) - mx);
        den += e;
        for (int c = 0; c < d; ++c) out[c] += e * (double)o->win_v[(size_t)j * d + c];
    }
    if (o->t == 0) {
        for (int i = 0; i < o->m; ++i)
            den += (double)o->cnt[i] * exp(dotd(q, o->X + (size_t)i * d, d) - mx);
    } else {   /* tau = sum_i (n_i / t) sum_{k in S_i} e^{<q,k>} */
        for (int i = 0; i < o->m; ++i) {
            double si = 0.0;
            for (int j = 0; j < o->t; ++j) si += exp(dotd(q, o->R + ((size_t)i * o->t + j) * d, d) - mx);
            den += (double)o->cnt[i] / (double)o->t * si;
        }
    }
    if (have_samples)
        for (int j = 0; j < o->s; ++j) {
            double vn = (double)o->Mvn[j];
            double wgt = vn > 0.0 ? o->mu / ((double)o->s * vn) : 0.0;
            double e = wgt * exp(dotd(q, o->Mk + (size_t)j * d, d) - mx);
            for (int c = 0; c < d; ++c) out[c] += e * (double)o->Mv[(size_t)j * d + c];
        }
    for (int c = 0; c < d; ++c) out[c] /= den;
    if (den_out) *den_out = den;
    if (mx_out) *mx_out = mx;
    return 0;
}

/* ------------------------------------------------------------------------
 * Batched conveniences (plain loops over tokens) and state read-out
 * ---------------------------------------------------------------------- */
void sgo_ingest(sgo_stream *o, const float *K, const float *V, int64_t n)
{
    for (int64_t t = 0; t < n; ++t)
        sgo_update(o, K + (size_t)t * o->d, V + (size_t)t * o->d);
}

/* n decode steps: update with (K[t], V[t]) then attend with each of the g
 * queries Q[t][0..g); out is [n, g, d] doubles. */
int sgo_decode(sgo_stream *o, const float *K, const float *V, const float *Q, int64_t n, int g, double *out)
{
    for (int64_t t = 0; t < n; ++t) {
        sgo_update(o, K + (size_t)t * o->d, V + (size_t)t * o->d);
        for (int h = 0; h < g; ++h) {
            int rc = sgo_attend(o, Q + ((size_t)t * g + h) * o->d, out + ((size_t)t * g + h) * o->d, NULL, NULL);
            if (rc) return rc;
        }
    }
    return 0;
}

int sgo_m(const sgo_stream *o) { return o->m; }
int64_t sgo_n_seen(const sgo_stream *o) { return o->n_seen; }
int64_t sgo_n_evicted(const sgo_stream *o) { return o->n_evicted; }
double sgo_mu(const sgo_stream *o) { return o->mu; }
int sgo_overflowed(const sgo_stream *o) { return o->overflowed; }
int64_t sgo_dropped(const sgo_stream *o) { return o->dropped; }
const float *sgo_centers(const sgo_stream *o) { return o->X; }
const float *sgo_reservoirs(const sgo_stream *o) { return o->R; }
const int64_t *sgo_counts(const sgo_stream *o) { return o->cnt; }
const float *sgo_sample_k(const sgo_stream *o) { return o->Mk; }
const float *sgo_sample_v(const sgo_stream *o) { return o->Mv; }
const int64_t *sgo_sample_idx(const sgo_stream *o) { return o->Midx; }
const float *sgo_sample_vn(const sgo_stream *o) { return o->Mvn; }
const float *sgo_window_k(const sgo_stream *o) { return o->win_k; }
const float *sgo_window_v(const sgo_stream *o) { return o->win_v; }
const int64_t *sgo_window_idx(const sgo_stream *o) { return o->win_idx; }
const int32_t *sgo_assign(const sgo_stream *o) { return o->assign; }
const uint8_t *sgo_created(const sgo_stream *o) { return o->created; }
const double *sgo_dist1(const sgo_stream *o) { return o->dist1; }
const double *sgo_dist2(const sgo_stream *o) { return o->dist2; }
