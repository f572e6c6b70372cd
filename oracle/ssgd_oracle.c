/*
 * CPU oracle for straggler-aware distributed SGD (K-sync, K-batch-sync, K-async,
 * K-batch-async, AdaSync) and for the Monte-Carlo estimate of the expected
 * runtime per iteration.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, sequential restatement of
 * the paper's update rules (Sec. 2.2, Eq. (2) "K-sync" and Eq. (3) "K-async"),
 * of its delay model (Sec. 3.1: one i.i.d. delay per worker and mini-batch) and
 * of AdaSync (Sec. 6, Algorithm 1; App. D).  It shares no code with the GPU
 * library, and only the tests, the smoke check and the CPU-baseline leg of the
 * benchmark may call it.
 *
 * Arithmetic: data and stored parameters are fp32; every gradient, loss and
 * aggregate is accumulated in fp64 and the parameter vector is rounded to fp32
 * once per update.  Delays are fp32 values produced by a fixed sequence of
 * IEEE-754 single-precision operations (no fused multiply-add, no libm), so that
 * any conforming implementation reproduces them bit for bit.  Simulated
 * wall-clock times are fp64.
 *
 * Parity unpinned (nothing outside this file fixes the values; the tests pin
 * everything else against closed forms, brute force, known-answer vectors or
 * textbook special cases): the long-horizon trajectory of the two-layer
 * network (pinned only through its per-step gradients, finite differences and
 * a scaled-down run).  The K-async inter-update times of orc_runtime_mc under
 * Pareto delays beyond the first update of a chain have no closed form; they
 * are pinned in law (renewal rate E[X]/P at K = 1, identity with K-sync at
 * K = P, and an independent vectorised simulation for every K).
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fPIC -shared
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers: Philox4x32 with 10 rounds (Salmon, Moraes,   */
/* Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11).         */
/* The paper only asks for i.i.d. delays (Sec. 3.1) and random mini-batches   */
/* (Sec. 1.1); the generator is this build's choice.                          */
/* ------------------------------------------------------------------------- */

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

enum { ORC_STREAM_DELAY = 1, ORC_STREAM_BATCH = 2, ORC_STREAM_INIT = 3, ORC_STREAM_MC = 4 };

/* One 128-bit block addressed by (seed, stream, aux, replica, worker, ordinal, version). */
static void draw_block(uint64_t seed, uint32_t stream, uint32_t aux, uint32_t replica,
                       uint32_t worker, uint32_t ordinal, uint32_t version, uint32_t out[4])
{
    uint32_t ctr[4], key[2];
    ctr[0] = version;
    ctr[1] = (worker & 0xFFFFu) | (ordinal << 16);
    ctr[2] = replica;
    ctr[3] = (stream & 0xFFu) | (aux << 8);
    key[0] = (uint32_t)seed;
    key[1] = (uint32_t)(seed >> 32);
    orc_philox4x32_10(ctr, key, out);
}

/* ------------------------------------------------------------------------- */
/* Uniform, logarithm and exponential as fixed fp32 operation sequences.      */
/* ------------------------------------------------------------------------- */

static float bits_to_float(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

/* u = (top 23 bits + 1/2) * 2^-23, strictly inside (0,1); every step is exact. */
float orc_uniform(uint32_t bits)
{
    float n = (float)(bits >> 9);
    float h = n + 0.5f;
    return h * 1.1920928955078125e-07f; /* 2^-23 */
}

/* E = -ln(u) for a normal float u in (0,1).  Mantissa is brought to
 * (sqrt(1/2), sqrt(2)], then ln m = 2 atanh((m-1)/(m+1)) by its odd series up
 * to the 9th power, and e*ln2 is added with ln2 split in a short high part and
 * a low part. */
float orc_neg_ln(float u)
{
    uint32_t b = float_to_bits(u);
    int32_t e = (int32_t)(b >> 23) - 127;
    float m = bits_to_float((b & 0x007FFFFFu) | 0x3F800000u);
    if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
    float a = m - 1.0f;
    float c = m + 1.0f;
    float s = a / c;
    float s2 = s * s;
    float p = 0.222222224f;            /* 2/9 */
    p = p * s2; p = p + 0.285714298f;  /* 2/7 */
    p = p * s2; p = p + 0.400000006f;  /* 2/5 */
    p = p * s2; p = p + 0.666666687f;  /* 2/3 */
    p = p * s2; p = p + 2.0f;
    float r = p * s;
    float ef = (float)e;
    float hi = ef * 0.693359375f;          /* exact product */
    float lo = ef * -2.12194440e-4f;
    float t = r + lo;
    float ln = hi + t;
    return -ln;
}

/* exp(y) for y >= 0: y = n ln2 + r, |r| <= ln2/2, degree-7 Taylor polynomial in
 * r, scaled by 2^n through the exponent field.  n > 127 gives +infinity. */
float orc_exp_pos(float y)
{
    float t = y * 1.44269502f;
    float th = t + 0.5f;
    if (!(th < 128.0f)) return INFINITY;
    int32_t n = (int32_t)th;
    float nf = (float)n;
    float r = y - nf * 0.693359375f;
    r = r - nf * -2.12194440e-4f;
    float p = 1.98412701e-4f;            /* 1/5040 */
    p = p * r; p = p + 1.38888892e-3f;   /* 1/720 */
    p = p * r; p = p + 8.33333377e-3f;   /* 1/120 */
    p = p * r; p = p + 4.16666679e-2f;   /* 1/24 */
    p = p * r; p = p + 0.166666672f;     /* 1/6 */
    p = p * r; p = p + 0.5f;
    p = p * r; p = p + 1.0f;
    p = p * r; p = p + 1.0f;
    float scale = bits_to_float((uint32_t)(n + 127) << 23);
    return p * scale;
}

/* ------------------------------------------------------------------------- */
/* Delay distributions (Sec. 3: Exp(mu) with mu a rate, E[X_{P:P}] = sum      */
/* 1/(i mu); Lemma 4: shifted exponential Delta + Exp(mu); Fig. 5 / Fig. 6:   */
/* Pareto(shape, scale)).  TABLE replays caller-supplied delays (tests).      */
/* ------------------------------------------------------------------------- */

enum { ORC_EXP = 0, ORC_SHIFTED_EXP = 1, ORC_PARETO = 2, ORC_TABLE = 3 };

typedef struct {
    int32_t kind;
    double shift, rate, alpha, scale;
    const float *table;
    int64_t table_len;
} orc_dist;

float orc_delay_from_bits(const orc_dist *dist, uint32_t bits)
{
    float E = orc_neg_ln(orc_uniform(bits));
    switch (dist->kind) {
    case ORC_EXP:
        return E / (float)dist->rate;
    case ORC_SHIFTED_EXP: {
        float q = E / (float)dist->rate;
        return (float)dist->shift + q;
    }
    case ORC_PARETO: {
        float q = E / (float)dist->alpha;
        return (float)dist->scale * orc_exp_pos(q);
    }
    default:
        return NAN;
    }
}

void orc_delays_from_bits(const orc_dist *dist, const uint32_t *bits, int64_t n, float *out)
{
    for (int64_t q = 0; q < n; ++q) out[q] = orc_delay_from_bits(dist, bits[q]);
}

/* Delay of the `ordinal`-th mini-batch that `worker` starts after reading
 * parameter version `version`.  `table_ord` is the number of ordinals a TABLE
 * distribution reserves per (version, worker). */
static float delay_of(const orc_dist *dist, uint64_t seed, uint32_t stream, uint32_t aux,
                      uint32_t replica, int32_t P, int32_t table_ord, uint32_t worker,
                      uint32_t ordinal, uint32_t version)
{
    if (dist->kind == ORC_TABLE) {
        int64_t idx = ((int64_t)version * P + worker) * table_ord + ordinal;
        return dist->table[idx % dist->table_len];
    }
    uint32_t blk[4];
    draw_block(seed, stream, aux, replica, worker, ordinal, version, blk);
    return orc_delay_from_bits(dist, blk[0]);
}

float orc_delay(const orc_dist *dist, uint64_t seed, uint32_t replica, int32_t P,
                int32_t table_ord, uint32_t worker, uint32_t ordinal, uint32_t version)
{
    return delay_of(dist, seed, ORC_STREAM_DELAY, 0, replica, P, table_ord, worker, ordinal, version);
}

/* Sample id of slot `slot` of a mini-batch: uniform on [0,N) with replacement. */
uint32_t orc_batch_index(uint64_t seed, uint32_t replica, uint32_t worker, uint32_t ordinal,
                         uint32_t version, uint32_t slot, uint32_t N)
{
    uint32_t blk[4];
    draw_block(seed, ORC_STREAM_BATCH, slot >> 2, replica, worker, ordinal, version, blk);
    return (uint32_t)(((uint64_t)blk[slot & 3u] * (uint64_t)N) >> 32);
}

/* ------------------------------------------------------------------------- */
/* Models.  The paper fixes only g(w, xi) = (1/m) sum grad f (Sec. 2.2); the  */
/* three losses are the benchmark's: least squares, softmax regression and a  */
/* two-layer ReLU network with a bf16 hidden contraction.                     */
/* Parameter layout:                                                          */
/*   LSQ      w[d]                                                            */
/*   SOFTMAX  W[C][d] row-major, then b[C]                                    */
/*   MLP2     W1[H][d], b1[H], W2[C][H], b2[C]                                */
/* ------------------------------------------------------------------------- */

enum { ORC_LSQ = 0, ORC_SOFTMAX = 1, ORC_MLP2 = 2 };
enum { ORC_K_SYNC = 0, ORC_K_BATCH_SYNC = 1, ORC_K_ASYNC = 2, ORC_K_BATCH_ASYNC = 3 };

typedef struct {
    int32_t kind, d, classes, hidden, bf16;
    const float *X;   /* N x d, row-major */
    const void *y;    /* float[N] (LSQ) or int32[N] */
    int64_t N;
} orc_model;

int64_t orc_param_count(const orc_model *M)
{
    switch (M->kind) {
    case ORC_LSQ: return M->d;
    case ORC_SOFTMAX: return (int64_t)M->classes * M->d + M->classes;
    case ORC_MLP2:
        return (int64_t)M->hidden * M->d + M->hidden + (int64_t)M->classes * M->hidden + M->classes;
    default: return -1;
    }
}

/* Round to bfloat16 (nearest, ties to even) and return the value as a float. */
float orc_round_bf16(float x)
{
    uint32_t b = float_to_bits(x);
    if ((b & 0x7F800000u) == 0x7F800000u) return x; /* inf / nan unchanged */
    uint32_t lsb = (b >> 16) & 1u;
    b += 0x7FFFu + lsb;
    b &= 0xFFFF0000u;
    return bits_to_float(b);
}

/* Mini-batch gradient and mean loss of one mini-batch `idx[0..m)` at parameters
 * w (fp32).  grad (fp64, |w| entries) is overwritten with (1/m) sum grad f. */
double orc_minibatch_grad(const orc_model *M, const float *w, const uint32_t *idx, int32_t m,
                          double *grad)
{
    const int32_t d = M->d;
    const int64_t nw = orc_param_count(M);
    for (int64_t q = 0; q < nw; ++q) grad[q] = 0.0;
    double loss = 0.0;

    if (M->kind == ORC_LSQ) {
        /* f = (1/2)(x.w - y)^2, grad f = (x.w - y) x */
        const float *y = (const float *)M->y;
        for (int32_t s = 0; s < m; ++s) {
            const float *x = M->X + (int64_t)idx[s] * d;
            double r = -(double)y[idx[s]];
            for (int32_t k = 0; k < d; ++k) r += (double)x[k] * (double)w[k];
            loss += 0.5 * r * r;
            for (int32_t k = 0; k < d; ++k) grad[k] += r * (double)x[k];
        }
    } else if (M->kind == ORC_SOFTMAX) {
        /* f = -log softmax(Wx + b)_y, grad_W = (p - e_y) x^T, grad_b = p - e_y */
        const int32_t C = M->classes;
        const int32_t *y = (const int32_t *)M->y;
        const float *W = w, *b = w + (int64_t)C * d;
        double *z = (double *)malloc(sizeof(double) * C);
        for (int32_t s = 0; s < m; ++s) {
            const float *x = M->X + (int64_t)idx[s] * d;
            double zmax = -INFINITY;
            for (int32_t c = 0; c < C; ++c) {
                double acc = (double)b[c];
                for (int32_t k = 0; k < d; ++k) acc += (double)W[(int64_t)c * d + k] * (double)x[k];
                z[c] = acc;
                if (acc > zmax) zmax = acc;
            }
            double den = 0.0;
            for (int32_t c = 0; c < C; ++c) den += exp(z[c] - zmax);
            int32_t lab = y[idx[s]];
            loss += -(z[lab] - zmax - log(den));
            for (int32_t c = 0; c < C; ++c) {
                double delta = exp(z[c] - zmax) / den - (c == lab ? 1.0 : 0.0);
                for (int32_t k = 0; k < d; ++k) grad[(int64_t)c * d + k] += delta * (double)x[k];
                grad[(int64_t)C * d + c] += delta;
            }
        }
        free(z);
    } else {
        /* z1 = W1 x + b1, h = relu(z1), z2 = W2 h + b2, p = softmax(z2).
         * With bf16 set, x and W1 are rounded to bf16 for the first contraction,
         * delta1 is rounded to bf16 for the W1 gradient contraction, and the
         * second layer uses the bf16-rounded values of W2; everything else is
         * unrounded. */
        const int32_t C = M->classes, H = M->hidden;
        const int32_t *y = (const int32_t *)M->y;
        const float *W1 = w, *b1 = W1 + (int64_t)H * d, *W2 = b1 + H, *b2 = W2 + (int64_t)C * H;
        double *gW1 = grad, *gb1 = gW1 + (int64_t)H * d, *gW2 = gb1 + H, *gb2 = gW2 + (int64_t)C * H;
        float *W1r = (float *)malloc(sizeof(float) * (size_t)H * d);
        float *W2r = (float *)malloc(sizeof(float) * (size_t)C * H);
        float *xr = (float *)malloc(sizeof(float) * d);
        double *z1 = (double *)malloc(sizeof(double) * H);
        double *h = (double *)malloc(sizeof(double) * H);
        double *z2 = (double *)malloc(sizeof(double) * C);
        double *d2 = (double *)malloc(sizeof(double) * C);
        for (int64_t q = 0; q < (int64_t)H * d; ++q) W1r[q] = M->bf16 ? orc_round_bf16(W1[q]) : W1[q];
        for (int64_t q = 0; q < (int64_t)C * H; ++q) W2r[q] = M->bf16 ? orc_round_bf16(W2[q]) : W2[q];
        for (int32_t s = 0; s < m; ++s) {
            const float *x = M->X + (int64_t)idx[s] * d;
            for (int32_t k = 0; k < d; ++k) xr[k] = M->bf16 ? orc_round_bf16(x[k]) : x[k];
            for (int32_t j = 0; j < H; ++j) {
                double acc = (double)b1[j];
                for (int32_t k = 0; k < d; ++k) acc += (double)W1r[(int64_t)j * d + k] * (double)xr[k];
                z1[j] = acc;
                h[j] = acc > 0.0 ? acc : 0.0;
            }
            double zmax = -INFINITY;
            for (int32_t c = 0; c < C; ++c) {
                double acc = (double)b2[c];
                for (int32_t j = 0; j < H; ++j) acc += (double)W2r[(int64_t)c * H + j] * h[j];
                z2[c] = acc;
                if (acc > zmax) zmax = acc;
            }
            double den = 0.0;
            for (int32_t c = 0; c < C; ++c) den += exp(z2[c] - zmax);
            int32_t lab = y[idx[s]];
            loss += -(z2[lab] - zmax - log(den));
            for (int32_t c = 0; c < C; ++c) {
                d2[c] = exp(z2[c] - zmax) / den - (c == lab ? 1.0 : 0.0);
                gb2[c] += d2[c];
                for (int32_t j = 0; j < H; ++j) gW2[(int64_t)c * H + j] += d2[c] * h[j];
            }
            for (int32_t j = 0; j < H; ++j) {
                double d1 = 0.0;
                if (z1[j] > 0.0)
                    for (int32_t c = 0; c < C; ++c) d1 += (double)W2r[(int64_t)c * H + j] * d2[c];
                gb1[j] += d1;
                /* the 1/m factor is applied before the bf16 rounding, as a
                 * device would round the scaled back-propagated error */
                double d1s = d1 / (double)m;
                double d1c = M->bf16 ? (double)orc_round_bf16((float)d1s) : d1s;
                if (d1c != 0.0)
                    for (int32_t k = 0; k < d; ++k) gW1[(int64_t)j * d + k] += d1c * (double)xr[k];
            }
        }
        /* gW1 already carries 1/m; scale the rest below */
        for (int64_t q = 0; q < (int64_t)H * d; ++q) gW1[q] *= (double)m;
        free(W1r); free(W2r); free(xr); free(z1); free(h); free(z2); free(d2);
    }
    for (int64_t q = 0; q < nw; ++q) grad[q] /= (double)m;
    return loss / (double)m;
}

/* Full-data objective F(w) = (1/N) sum f(w, xi_n) (Eq. (1)), fp64. */
double orc_full_loss(const orc_model *M, const float *w)
{
    /* evaluate through the mini-batch routine on consecutive blocks */
    const int64_t nw = orc_param_count(M);
    double *g = (double *)malloc(sizeof(double) * (size_t)nw);
    uint32_t idx[64];
    double total = 0.0;
    for (int64_t n0 = 0; n0 < M->N; n0 += 64) {
        int32_t cnt = (int32_t)((M->N - n0) < 64 ? (M->N - n0) : 64);
        for (int32_t s = 0; s < cnt; ++s) idx[s] = (uint32_t)(n0 + s);
        total += orc_minibatch_grad(M, w, idx, cnt, g) * cnt;
    }
    free(g);
    return total / (double)M->N;
}

/* Gradient of the full-data objective, grad F(w) = (1/N) sum_n grad f(w, xi_n)
 * (Eq. (1); the quantity the staleness bound, the fifth assumption of Sec. 4.1, is stated in), fp64:
 * the mini-batch gradients of consecutive blocks, weighted by their sizes. */
void orc_full_grad(const orc_model *M, const float *w, double *grad_out)
{
    const int64_t nw = orc_param_count(M);
    double *g = (double *)malloc(sizeof(double) * (size_t)nw);
    uint32_t idx[64];
    for (int64_t q = 0; q < nw; ++q) grad_out[q] = 0.0;
    for (int64_t n0 = 0; n0 < M->N; n0 += 64) {
        int32_t cnt = (int32_t)((M->N - n0) < 64 ? (M->N - n0) : 64);
        for (int32_t s = 0; s < cnt; ++s) idx[s] = (uint32_t)(n0 + s);
        (void)orc_minibatch_grad(M, w, idx, cnt, g);
        for (int64_t q = 0; q < nw; ++q) grad_out[q] += g[q] * cnt;
    }
    for (int64_t q = 0; q < nw; ++q) grad_out[q] /= (double)M->N;
    free(g);
}

/* ------------------------------------------------------------------------- */
/* The event process and the parameter-server loop.                           */
/* ------------------------------------------------------------------------- */

typedef struct {
    int32_t mode;   /* 0 fixed K; 1 double K when the windowed loss plateaus;
                       2 Algorithm 1 (square-root rule); 3 K-sync quadratic rule (App. D) */
    int32_t K0, Kmax, window;
    double rel_tol, interval_t;
} orc_adasync;

typedef struct { int64_t version; float *w; int32_t refs; } orc_snapshot;

typedef struct orc_ctx {
    orc_model M;
    int32_t P, K, m, variant;
    orc_dist dist;
    float *table_copy;
    double lr;
    uint64_t seed;
    uint32_t replica;
    orc_adasync ada;
    int64_t nw;

    int64_t j;      /* updates done */
    double t;       /* simulated wall-clock */
    float *w;       /* current parameters, fp32 storage */
    /* per worker */
    int64_t *tau;   /* version read */
    int32_t *ord;   /* ordinal of the mini-batch in flight (batch variants) */
    double *finish; /* absolute finish time (async) */
    int32_t *snap;  /* index of the snapshot the worker read (async) */
    orc_snapshot *snaps; int32_t nsnaps, capsnaps;

    /* AdaSync */
    double win_sum; int32_t win_cnt; double win_prev; int64_t win_index;
    double F0; int have_F0; double int_sum; int64_t int_cnt;

    /* trace */
    int64_t cap;
    double *tr_t; float *tr_loss; int32_t *tr_K; int32_t *tr_sel; int32_t *tr_stale; int32_t *tr_ord;
    int32_t Kcap;   /* row width of tr_sel / tr_stale */
    double *scratch_g, *scratch_sum;
    uint32_t *scratch_idx;
} orc_ctx;

static int32_t snap_acquire(orc_ctx *c, int64_t version)
{
    for (int32_t s = 0; s < c->nsnaps; ++s)
        if (c->snaps[s].refs > 0 && c->snaps[s].version == version) { c->snaps[s].refs++; return s; }
    int32_t s = -1;
    for (int32_t q = 0; q < c->nsnaps; ++q) if (c->snaps[q].refs == 0) { s = q; break; }
    if (s < 0) {
        if (c->nsnaps == c->capsnaps) {
            c->capsnaps = c->capsnaps ? 2 * c->capsnaps : 8;
            c->snaps = (orc_snapshot *)realloc(c->snaps, sizeof(orc_snapshot) * c->capsnaps);
        }
        s = c->nsnaps++;
        c->snaps[s].w = (float *)malloc(sizeof(float) * (size_t)c->nw);
    }
    c->snaps[s].version = version;
    c->snaps[s].refs = 1;
    memcpy(c->snaps[s].w, c->w, sizeof(float) * (size_t)c->nw);
    return s;
}

static int32_t table_ord_of(const orc_ctx *c)
{
    return (c->variant == ORC_K_BATCH_SYNC || c->variant == ORC_K_BATCH_ASYNC) ? c->Kcap + 1 : 1;
}

static float ctx_delay(const orc_ctx *c, int32_t worker, int32_t ordinal, int64_t version)
{
    return delay_of(&c->dist, c->seed, ORC_STREAM_DELAY, 0, c->replica, c->P, table_ord_of(c),
                    (uint32_t)worker, (uint32_t)ordinal, (uint32_t)version);
}

static void ctx_batch(const orc_ctx *c, int32_t worker, int32_t ordinal, int64_t version, uint32_t *idx)
{
    for (int32_t s = 0; s < c->m; ++s)
        idx[s] = orc_batch_index(c->seed, c->replica, (uint32_t)worker, (uint32_t)ordinal,
                                 (uint32_t)version, (uint32_t)s, (uint32_t)c->M.N);
}

/* Initial parameters: zeros for the linear models; for the MLP the two weight
 * matrices are uniform on (-1/sqrt(fan_in), +1/sqrt(fan_in)), biases zero. */
void orc_init_params(const orc_model *M, uint64_t seed, float *w)
{
    int64_t nw = orc_param_count(M);
    for (int64_t q = 0; q < nw; ++q) w[q] = 0.0f;
    if (M->kind != ORC_MLP2) return;
    const int32_t d = M->d, H = M->hidden, C = M->classes;
    float bound1 = (float)(1.0 / sqrt((double)d));
    float bound2 = (float)(1.0 / sqrt((double)H));
    int64_t off2 = (int64_t)H * d + H;
    for (int64_t q = 0; q < nw; ++q) {
        float bound;
        if (q < (int64_t)H * d) bound = bound1;
        else if (q >= off2 && q < off2 + (int64_t)C * H) bound = bound2;
        else continue;
        uint32_t blk[4];
        draw_block(seed, ORC_STREAM_INIT, (uint32_t)((q >> 2) >> 32), 0, 0, 0, (uint32_t)(q >> 2), blk);
        float u = orc_uniform(blk[q & 3]);
        float v = u + u;
        v = v - 1.0f;
        w[q] = v * bound;
    }
}

orc_ctx *orc_create(const orc_model *M, int32_t P, int32_t K, int32_t m, int32_t variant,
                    const orc_dist *dist, double lr, uint64_t seed, uint32_t replica,
                    const orc_adasync *ada)
{
    if (!M || !dist || P < 1 || K < 1 || m < 1 || M->N < 1) return NULL;
    int32_t Kcap = K;
    if (ada && ada->mode != 0) { if (ada->Kmax > Kcap) Kcap = ada->Kmax; }
    if (variant == ORC_K_SYNC || variant == ORC_K_ASYNC) { if (Kcap > P) return NULL; }
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->M = *M; c->P = P; c->K = K; c->m = m; c->variant = variant; c->dist = *dist;
    if (dist->kind == ORC_TABLE) {
        c->table_copy = (float *)malloc(sizeof(float) * (size_t)dist->table_len);
        memcpy(c->table_copy, dist->table, sizeof(float) * (size_t)dist->table_len);
        c->dist.table = c->table_copy;
    }
    c->lr = lr; c->seed = seed; c->replica = replica;
    if (ada) c->ada = *ada; else memset(&c->ada, 0, sizeof(c->ada));
    c->Kcap = Kcap;
    c->nw = orc_param_count(M);
    c->w = (float *)malloc(sizeof(float) * (size_t)c->nw);
    orc_init_params(M, seed, c->w);
    c->tau = (int64_t *)calloc(P, sizeof(int64_t));
    c->ord = (int32_t *)calloc(P, sizeof(int32_t));
    c->finish = (double *)calloc(P, sizeof(double));
    c->snap = (int32_t *)calloc(P, sizeof(int32_t));
    c->scratch_g = (double *)malloc(sizeof(double) * (size_t)c->nw);
    c->scratch_sum = (double *)malloc(sizeof(double) * (size_t)c->nw);
    c->scratch_idx = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)m);
    if (variant == ORC_K_ASYNC || variant == ORC_K_BATCH_ASYNC) {
        /* all workers are launched afresh with w_0 (proof of Lemma 4) */
        for (int32_t i = 0; i < P; ++i) {
            c->tau[i] = 0; c->ord[i] = 0;
            c->finish[i] = (double)ctx_delay(c, i, 0, 0);
            c->snap[i] = snap_acquire(c, 0);
        }
    }
    return c;
}

void orc_destroy(orc_ctx *c)
{
    if (!c) return;
    for (int32_t s = 0; s < c->nsnaps; ++s) free(c->snaps[s].w);
    free(c->snaps); free(c->table_copy); free(c->w); free(c->tau); free(c->ord); free(c->finish);
    free(c->snap); free(c->scratch_g); free(c->scratch_sum); free(c->scratch_idx);
    free(c->tr_t); free(c->tr_loss); free(c->tr_K); free(c->tr_sel); free(c->tr_stale); free(c->tr_ord);
    free(c);
}

static void trace_reserve(orc_ctx *c, int64_t need)
{
    if (need <= c->cap) return;
    int64_t cap = c->cap ? c->cap : 256;
    while (cap < need) cap *= 2;
    c->tr_t = (double *)realloc(c->tr_t, sizeof(double) * cap);
    c->tr_loss = (float *)realloc(c->tr_loss, sizeof(float) * cap);
    c->tr_K = (int32_t *)realloc(c->tr_K, sizeof(int32_t) * cap);
    c->tr_sel = (int32_t *)realloc(c->tr_sel, sizeof(int32_t) * cap * c->Kcap);
    c->tr_stale = (int32_t *)realloc(c->tr_stale, sizeof(int32_t) * cap * c->Kcap);
    c->tr_ord = (int32_t *)realloc(c->tr_ord, sizeof(int32_t) * cap * c->Kcap);
    c->cap = cap;
}

/* index of the smallest (key, id) among entries not yet taken */
static int32_t argmin_free(const double *key, const char *taken, int32_t P)
{
    int32_t best = -1;
    for (int32_t i = 0; i < P; ++i) {
        if (taken && taken[i]) continue;
        if (best < 0 || key[i] < key[best]) best = i; /* strict: lower id wins ties */
    }
    return best;
}

/* AdaSync controller, called after update j has been recorded (Sec. 6). */
static void adasync_after_update(orc_ctx *c, double loss_j, double t_prev, double t_new)
{
    orc_adasync *a = &c->ada;
    if (a->mode == 0) return;
    if (!c->have_F0) { c->F0 = loss_j; c->have_F0 = 1; }
    if (a->mode == 1) {
        c->win_sum += loss_j; c->win_cnt++;
        if (c->win_cnt == a->window) {
            double mean = c->win_sum / (double)a->window;
            if (c->win_index >= 1 && mean > (1.0 - a->rel_tol) * c->win_prev) {
                int32_t K2 = 2 * c->K; if (K2 > a->Kmax) K2 = a->Kmax;
                c->K = K2;
            }
            c->win_prev = mean; c->win_index++;
            c->win_sum = 0.0; c->win_cnt = 0;
        }
        return;
    }
    /* modes 2 and 3: every time the clock crosses a multiple of interval_t */
    c->int_sum += loss_j; c->int_cnt++;
    if (floor(t_new / a->interval_t) > floor(t_prev / a->interval_t)) {
        double Fstart = c->int_sum / (double)c->int_cnt;
        c->int_sum = 0.0; c->int_cnt = 0;
        if (c->K < a->Kmax && Fstart > 0.0) {
            double ratio = c->F0 / Fstart, Knew;
            if (a->mode == 2) {
                Knew = (double)a->K0 * sqrt(ratio);              /* Algorithm 1 */
            } else {
                /* K^2/(P-K) = K0^2/(P-K0) * F(w0)/F(w_start)  (App. D, K-sync) */
                double q = (double)a->K0 * a->K0 / (double)(c->P - a->K0) * ratio;
                Knew = 0.5 * (-q + sqrt(q * q + 4.0 * q * (double)c->P));
            }
            int32_t Ki = (int32_t)floor(Knew + 0.5);
            if (Ki < c->K) Ki = c->K;
            if (Ki > a->Kmax) Ki = a->Kmax;
            c->K = Ki;
        }
    }
}

/* One parameter-server update.  agg (nullable, fp64, |w|) receives
 * (1/K) sum_l g_l, the averaged gradient that the update applies. */
int orc_step(orc_ctx *c, double *agg)
{
    const int32_t P = c->P, K = c->K;
    const int64_t j = c->j;
    trace_reserve(c, j + 1);
    int32_t *sel = c->tr_sel + j * c->Kcap, *stale = c->tr_stale + j * c->Kcap,
            *ords = c->tr_ord + j * c->Kcap;
    for (int32_t l = 0; l < c->Kcap; ++l) { sel[l] = -1; stale[l] = -1; ords[l] = -1; }
    for (int64_t q = 0; q < c->nw; ++q) c->scratch_sum[q] = 0.0;
    double loss = 0.0, t_new = c->t;

    if (c->variant == ORC_K_SYNC) {
        /* all P start at t_j with w_j; the first K to finish contribute (Eq. (2)) */
        double *x = (double *)malloc(sizeof(double) * P);
        char *taken = (char *)calloc(P, 1);
        for (int32_t i = 0; i < P; ++i) x[i] = (double)ctx_delay(c, i, 0, j);
        double last = 0.0;
        for (int32_t l = 0; l < K; ++l) {
            int32_t i = argmin_free(x, taken, P);
            taken[i] = 1; last = x[i];
            sel[l] = i; stale[l] = 0; ords[l] = 0;
            ctx_batch(c, i, 0, j, c->scratch_idx);
            loss += orc_minibatch_grad(&c->M, c->w, c->scratch_idx, c->m, c->scratch_g);
            for (int64_t q = 0; q < c->nw; ++q) c->scratch_sum[q] += c->scratch_g[q];
        }
        t_new = c->t + last;
        free(x); free(taken);
    } else if (c->variant == ORC_K_BATCH_SYNC) {
        /* a finished worker starts another mini-batch at the same w_j; the first
         * K mini-batches to finish contribute (Sec. 2.2) */
        double *cmp = (double *)malloc(sizeof(double) * P);
        int32_t *r = (int32_t *)calloc(P, sizeof(int32_t));
        for (int32_t i = 0; i < P; ++i) cmp[i] = (double)ctx_delay(c, i, 0, j);
        double last = 0.0;
        for (int32_t l = 0; l < K; ++l) {
            int32_t i = argmin_free(cmp, NULL, P);
            last = cmp[i];
            sel[l] = i; stale[l] = 0; ords[l] = r[i];
            ctx_batch(c, i, r[i], j, c->scratch_idx);
            loss += orc_minibatch_grad(&c->M, c->w, c->scratch_idx, c->m, c->scratch_g);
            for (int64_t q = 0; q < c->nw; ++q) c->scratch_sum[q] += c->scratch_g[q];
            r[i] += 1;
            if (l + 1 < K) cmp[i] = cmp[i] + (double)ctx_delay(c, i, r[i], j);
        }
        t_new = c->t + last;
        free(cmp); free(r);
    } else if (c->variant == ORC_K_ASYNC) {
        /* the K earliest finishers contribute gradients taken at the version
         * each of them read; nobody is cancelled (Eq. (3)) */
        char *taken = (char *)calloc(P, 1);
        for (int32_t l = 0; l < K; ++l) {
            int32_t i = argmin_free(c->finish, taken, P);
            taken[i] = 1; t_new = c->finish[i];
            sel[l] = i; stale[l] = (int32_t)(j - c->tau[i]); ords[l] = 0;
            ctx_batch(c, i, 0, c->tau[i], c->scratch_idx);
            loss += orc_minibatch_grad(&c->M, c->snaps[c->snap[i]].w, c->scratch_idx, c->m, c->scratch_g);
            for (int64_t q = 0; q < c->nw; ++q) c->scratch_sum[q] += c->scratch_g[q];
        }
        free(taken);
    } else {
        /* K-batch-async: every finished mini-batch is pushed, the worker re-reads
         * the current parameters (still w_j until K pushes have arrived) and
         * starts its next mini-batch at once (Sec. 2.2) */
        for (int32_t l = 0; l < K; ++l) {
            int32_t i = argmin_free(c->finish, NULL, P);
            t_new = c->finish[i];
            sel[l] = i; stale[l] = (int32_t)(j - c->tau[i]); ords[l] = c->ord[i];
            ctx_batch(c, i, c->ord[i], c->tau[i], c->scratch_idx);
            loss += orc_minibatch_grad(&c->M, c->snaps[c->snap[i]].w, c->scratch_idx, c->m, c->scratch_g);
            for (int64_t q = 0; q < c->nw; ++q) c->scratch_sum[q] += c->scratch_g[q];
            c->snaps[c->snap[i]].refs--;
            c->snap[i] = -1;
            if (l + 1 < K) {
                /* restart at its own finish time, reading version j */
                if (c->tau[i] == j) c->ord[i] += 1; else { c->tau[i] = j; c->ord[i] = 0; }
                c->snap[i] = snap_acquire(c, j);
                c->finish[i] = c->finish[i] + (double)ctx_delay(c, i, c->ord[i], j);
            }
            /* the K-th push triggers the update; that worker reads w_{j+1} below */
        }
    }

    /* w_{j+1} = w_j - (eta/K) sum_l g_l, stored in fp32 */
    for (int64_t q = 0; q < c->nw; ++q) {
        double mean = c->scratch_sum[q] / (double)K;
        if (agg) agg[q] = mean;
        c->w[q] = (float)((double)c->w[q] - c->lr * mean);
    }
    loss /= (double)K;

    if (c->variant == ORC_K_BATCH_ASYNC) {
        int32_t i = sel[K - 1];
        c->tau[i] = j + 1; c->ord[i] = 0;
        c->snap[i] = snap_acquire(c, j + 1);
        c->finish[i] = t_new + (double)ctx_delay(c, i, 0, j + 1);
    }
    if (c->variant == ORC_K_ASYNC) {
        /* only the contributors fetch w_{j+1} and start a new mini-batch at t_{j+1} */
        for (int32_t l = 0; l < K; ++l) c->snaps[c->snap[sel[l]]].refs--;
        for (int32_t l = 0; l < K; ++l) {
            int32_t i = sel[l];
            c->tau[i] = j + 1;
            c->snap[i] = snap_acquire(c, j + 1);
            c->finish[i] = t_new + (double)ctx_delay(c, i, 0, j + 1);
        }
    }

    c->tr_t[j] = t_new; c->tr_loss[j] = (float)loss; c->tr_K[j] = K;
    double t_prev = c->t;
    c->t = t_new; c->j = j + 1;
    adasync_after_update(c, (double)(float)loss, t_prev, t_new);
    return 0;
}

int orc_run(orc_ctx *c, int64_t J)
{
    for (int64_t q = 0; q < J; ++q) { int rc = orc_step(c, NULL); if (rc) return rc; }
    return 0;
}

int64_t orc_updates_done(const orc_ctx *c) { return c->j; }
int32_t orc_current_K(const orc_ctx *c) { return c->K; }
int32_t orc_trace_width(const orc_ctx *c) { return c->Kcap; }
double orc_clock(const orc_ctx *c) { return c->t; }
void orc_get_params(const orc_ctx *c, float *out) { memcpy(out, c->w, sizeof(float) * (size_t)c->nw); }
void orc_set_params(orc_ctx *c, const float *in) { memcpy(c->w, in, sizeof(float) * (size_t)c->nw); }
void orc_force_K(orc_ctx *c, int32_t K) { if (K >= 1 && K <= c->Kcap) c->K = K; }

int orc_get_trace(const orc_ctx *c, int64_t from, int64_t n, double *t, float *loss, int32_t *K,
                  int32_t *sel, int32_t *stale, int32_t *ord)
{
    if (from < 0 || n < 0 || from + n > c->j) return 1;
    if (t) memcpy(t, c->tr_t + from, sizeof(double) * n);
    if (loss) memcpy(loss, c->tr_loss + from, sizeof(float) * n);
    if (K) memcpy(K, c->tr_K + from, sizeof(int32_t) * n);
    if (sel) memcpy(sel, c->tr_sel + from * c->Kcap, sizeof(int32_t) * n * c->Kcap);
    if (stale) memcpy(stale, c->tr_stale + from * c->Kcap, sizeof(int32_t) * n * c->Kcap);
    if (ord) memcpy(ord, c->tr_ord + from * c->Kcap, sizeof(int32_t) * n * c->Kcap);
    return 0;
}

/* Per-worker view of the event state (async variants): version read and finish time. */
void orc_get_workers(const orc_ctx *c, int64_t *tau, double *finish)
{
    for (int32_t i = 0; i < c->P; ++i) { if (tau) tau[i] = c->tau[i]; if (finish) finish[i] = c->finish[i]; }
}

/* ------------------------------------------------------------------------- */
/* Monte-Carlo runtime estimator (what Fig. 6 simulates; Lemmas 1-3).         */
/* Trial r: P fresh delays X(r,i).  For every K in [Kmin, Kmax] the chosen    */
/* variant's event process is run for chain_len updates from that fresh start */
/* and T_l = t_l - t_{l-1} is recorded.  The first delays of a trial are      */
/* shared by all K; later ones are keyed by K as well, and by the rank of the */
/* finisher they replace (delays are i.i.d., so T_l depends on the multiset   */
/* of finish times only, not on which worker holds which).                    */
/*   K-sync        every update is a fresh start: T_l = K-th smallest of P    */
/*   K-batch-sync  every update is a fresh start with immediate re-draws      */
/*   K-async       contributors restart at t_l, the rest keep running         */
/*   K-batch-async every push restarts its worker at once: one push sequence  */
/*                 for all K, update l at push l*K (Lemma 5)                  */
/* sum / sumsq: [(Kmax-Kmin+1) x chain_len] fp64 accumulators, added to.      */
/* per_trial (nullable): [ntrials x nK x chain_len] fp64.                     */
/* ------------------------------------------------------------------------- */

static float mc_delay(const orc_dist *dist, uint64_t seed, uint32_t trial, int32_t P, uint32_t aux,
                      uint32_t worker, uint32_t ordinal, uint32_t version)
{
    return delay_of(dist, seed, ORC_STREAM_MC, aux, trial, P, 1, worker, ordinal, version);
}

int orc_runtime_mc(int32_t variant, int32_t P, int32_t Kmin, int32_t Kmax, const orc_dist *dist,
                   int64_t trial0, int64_t ntrials, int32_t chain_len, uint64_t seed,
                   double *sum, double *sumsq, double *per_trial)
{
    if (P < 1 || Kmin < 1 || Kmax < Kmin || chain_len < 1 || ntrials < 0) return 1;
    if (variant != ORC_K_BATCH_SYNC && variant != ORC_K_BATCH_ASYNC && Kmax > P) return 1;
    const int32_t nK = Kmax - Kmin + 1;
    double *first = (double *)malloc(sizeof(double) * P);
    double *f = (double *)malloc(sizeof(double) * P);
    int32_t *r = (int32_t *)malloc(sizeof(int32_t) * P);
    char *taken = (char *)malloc(P);
    int32_t *who = (int32_t *)malloc(sizeof(int32_t) * (Kmax > P ? Kmax : P));
    for (int64_t q = 0; q < ntrials; ++q) {
        uint32_t trial = (uint32_t)(trial0 + q);
        for (int32_t i = 0; i < P; ++i) first[i] = (double)mc_delay(dist, seed, trial, P, 0, i, 0, 0);
        if (variant == ORC_K_BATCH_ASYNC) {
            /* No worker ever waits: each pushes mini-batch after mini-batch, whatever K is (the
             * K-th pusher of an update restarts at its own finish time, which is the update time).
             * The pushes of all workers, merged in time order, are one sequence p_1 <= p_2 <= ...
             * shared by every K, and update l of K-batch-async happens at push l*K (the
             * superposition of renewal processes in the proof of Lemma 5):
             * T_l = p_{lK} - p_{(l-1)K}.  Worker i's n-th delay is keyed by (worker i, version n). */
            const int64_t npush = (int64_t)chain_len * Kmax;
            double *push = (double *)malloc(sizeof(double) * (size_t)(npush + 1));
            push[0] = 0.0;
            for (int32_t i = 0; i < P; ++i) { f[i] = first[i]; r[i] = 0; }
            for (int64_t n = 1; n <= npush; ++n) {
                int32_t i = argmin_free(f, NULL, P);
                push[n] = f[i];
                r[i] += 1;
                f[i] = f[i] + (double)mc_delay(dist, seed, trial, P, 0, i, 0, (uint32_t)r[i]);
            }
            for (int32_t K = Kmin; K <= Kmax; ++K)
                for (int32_t l = 0; l < chain_len; ++l) {
                    double T = push[(int64_t)(l + 1) * K] - push[(int64_t)l * K];
                    int64_t cell = (int64_t)(K - Kmin) * chain_len + l;
                    if (sum) sum[cell] += T;
                    if (sumsq) sumsq[cell] += T * T;
                    if (per_trial) per_trial[(q * nK + (K - Kmin)) * chain_len + l] = T;
                }
            free(push);
            continue;
        }
        for (int32_t K = Kmin; K <= Kmax; ++K) {
            double t = 0.0;
            for (int32_t i = 0; i < P; ++i) f[i] = first[i];
            for (int32_t l = 0; l < chain_len; ++l) {
                double t_new = t;
                if (variant == ORC_K_ASYNC) {
                    memset(taken, 0, P);
                    for (int32_t a = 0; a < K; ++a) {
                        int32_t i = argmin_free(f, taken, P);
                        taken[i] = 1; who[a] = i; t_new = f[i];
                    }
                    /* the a-th earliest finisher takes the a-th fresh delay of this update:
                     * the process only depends on the multiset of finish times */
                    for (int32_t a = 0; a < K; ++a)
                        f[who[a]] = t_new + (double)mc_delay(dist, seed, trial, P, (uint32_t)K, a, 0, l + 1);
                } else {
                    if (l > 0)
                        for (int32_t i = 0; i < P; ++i)
                            f[i] = (double)mc_delay(dist, seed, trial, P, (uint32_t)K, i, 0, l);
                    if (variant == ORC_K_SYNC) {
                        memset(taken, 0, P);
                        double last = 0.0;
                        for (int32_t a = 0; a < K; ++a) {
                            int32_t i = argmin_free(f, taken, P);
                            taken[i] = 1; last = f[i];
                        }
                        t_new = t + last;
                    } else {
                        for (int32_t i = 0; i < P; ++i) r[i] = 0;
                        double last = 0.0;
                        for (int32_t a = 0; a < K; ++a) {
                            int32_t i = argmin_free(f, NULL, P);
                            last = f[i];
                            r[i] += 1;
                            /* the a-th finished mini-batch is followed by the a-th re-draw
                             * (ordinal 1 keeps these apart from the fresh delays) */
                            if (a + 1 < K)
                                f[i] = f[i] + (double)mc_delay(dist, seed, trial, P, (uint32_t)K, a, 1, l);
                        }
                        t_new = t + last;
                    }
                }
                double T = t_new - t;
                t = t_new;
                int64_t cell = (int64_t)(K - Kmin) * chain_len + l;
                if (sum) sum[cell] += T;
                if (sumsq) sumsq[cell] += T * T;
                if (per_trial) per_trial[(q * nK + (K - Kmin)) * chain_len + l] = T;
            }
        }
    }
    free(first); free(f); free(r); free(taken); free(who);
    return 0;
}
