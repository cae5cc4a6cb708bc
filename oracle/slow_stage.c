/*
 * Oracle, scalar-loop tier: forward and backward of a middle pipeline stage
 * (a slice of GPT pre-LN causal or BERT post-LN bidirectional blocks) written
 * as plain loops over scalars in double precision -- no library routine but
 * libm's erf, exp and sqrt, no blocking, no vectorisation by hand.
 *
 * TEST INFRASTRUCTURE ONLY. It exists to check the numpy tier of the oracle
 * (oracle/stage.py) against a second, independently written implementation of
 * the same textbook definitions, and to be timed as the slowest CPU baseline.
 * The model family is the paper's (Section 4.1, Table 2: 12 h^2 + 13 h
 * parameters per layer); the versioned backward follows Section 3.1: saved
 * activations are the forward's, parameters are whatever vector is handed in.
 *
 * Flat parameters per layer, in order: g1[D] b1[D] Wqkv[D][3D] bqkv[3D]
 * Wo[D][D] bo[D] g2[D] b2[D] W1[D][F] bf1[F] W2[F][D] bf2[D]; y = x W + b.
 * Activations are token-major [N][.], N = b*s, row = sequence*s + position.
 *
 * Saved activations per layer (doubles, in this order): block input [N][D],
 * xhat1 [N][D], rstd1 [N], attention input [N][D], qkv [N][3D], probabilities
 * [b][H][s][s], attention output [N][D], y1 [N][D], xhat2 [N][D], rstd2 [N],
 * MLP input [N][D], u [N][F], h [N][F].
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int kind, L, D, H, F, s, b;   /* kind 0: GPT pre-LN causal, 1: BERT post-LN bidirectional */
    double eps;
} shape_t;

static long layer_params(const shape_t* c) {
    long D = c->D, F = c->F;
    return 4 * D + 3 * D * D + 3 * D + D * D + D + D * F + F + F * D + D;
}

long slow_saved_doubles_per_layer(int D, int H, int F, int s, int b) {
    long N = (long)s * b;
    return N * D + N * D + N + N * D + N * 3 * D + (long)b * H * s * s + N * D + N * D + N * D + N + N * D + N * F + N * F;
}

typedef struct {
    const double *g1, *b1, *wqkv, *bqkv, *wo, *bo, *g2, *b2, *w1, *bf1, *w2, *bf2;
} lparams_t;
typedef struct {
    double *g1, *b1, *wqkv, *bqkv, *wo, *bo, *g2, *b2, *w1, *bf1, *w2, *bf2;
} lgrads_t;

static void split_params(const shape_t* c, const double* p, lparams_t* o) {
    long D = c->D, F = c->F;
    o->g1 = p; p += D; o->b1 = p; p += D; o->wqkv = p; p += 3 * D * D; o->bqkv = p; p += 3 * D;
    o->wo = p; p += D * D; o->bo = p; p += D; o->g2 = p; p += D; o->b2 = p; p += D;
    o->w1 = p; p += D * F; o->bf1 = p; p += F; o->w2 = p; p += F * D; o->bf2 = p;
}
static void split_grads(const shape_t* c, double* p, lgrads_t* o) {
    long D = c->D, F = c->F;
    o->g1 = p; p += D; o->b1 = p; p += D; o->wqkv = p; p += 3 * D * D; o->bqkv = p; p += 3 * D;
    o->wo = p; p += D * D; o->bo = p; p += D; o->g2 = p; p += D; o->b2 = p; p += D;
    o->w1 = p; p += D * F; o->bf1 = p; p += F; o->w2 = p; p += F * D; o->bf2 = p;
}

typedef struct {
    double *xin, *xhat1, *rstd1, *ain, *qkv, *prob, *o, *y1, *xhat2, *rstd2, *cin, *u, *h;
} saved_t;
static void split_saved(const shape_t* c, double* p, saved_t* o) {
    long N = (long)c->s * c->b, D = c->D, F = c->F;
    o->xin = p; p += N * D; o->xhat1 = p; p += N * D; o->rstd1 = p; p += N; o->ain = p; p += N * D;
    o->qkv = p; p += N * 3 * D; o->prob = p; p += (long)c->b * c->H * c->s * c->s; o->o = p; p += N * D;
    o->y1 = p; p += N * D; o->xhat2 = p; p += N * D; o->rstd2 = p; p += N; o->cin = p; p += N * D;
    o->u = p; p += N * F; o->h = p;
}

/* ---- primitives ---------------------------------------------------------- */
static void ln_fwd(const double* x, const double* g, const double* be, double eps, long N, long D, double* y,
                   double* xhat, double* rstd) {
    for (long n = 0; n < N; ++n) {
        double mu = 0.0, var = 0.0;
        for (long d = 0; d < D; ++d) mu += x[n * D + d];
        mu /= (double)D;
        for (long d = 0; d < D; ++d) { double t = x[n * D + d] - mu; var += t * t; }
        var /= (double)D;                                   /* biased */
        rstd[n] = 1.0 / sqrt(var + eps);
        for (long d = 0; d < D; ++d) {
            xhat[n * D + d] = (x[n * D + d] - mu) * rstd[n];
            y[n * D + d] = xhat[n * D + d] * g[d] + be[d];
        }
    }
}
/* dx (written), dgamma, dbeta (written) */
static void ln_bwd(const double* dy, const double* xhat, const double* rstd, const double* g, long N, long D, double* dx,
                   double* dg, double* db) {
    for (long d = 0; d < D; ++d) { dg[d] = 0.0; db[d] = 0.0; }
    for (long n = 0; n < N; ++n) {
        double m1 = 0.0, m2 = 0.0;
        for (long d = 0; d < D; ++d) {
            double dxh = dy[n * D + d] * g[d];
            m1 += dxh;
            m2 += dxh * xhat[n * D + d];
            dg[d] += dy[n * D + d] * xhat[n * D + d];
            db[d] += dy[n * D + d];
        }
        m1 /= (double)D; m2 /= (double)D;
        for (long d = 0; d < D; ++d)
            dx[n * D + d] = rstd[n] * (dy[n * D + d] * g[d] - m1 - xhat[n * D + d] * m2);
    }
}
/* y[N][O] = x[N][I] W[I][O] + bias[O] */
static void lin_fwd(const double* x, const double* W, const double* bias, long N, long I, long O, double* y) {
    for (long n = 0; n < N; ++n)
        for (long o = 0; o < O; ++o) {
            double acc = bias[o];
            for (long i = 0; i < I; ++i) acc += x[n * I + i] * W[i * O + o];
            y[n * O + o] = acc;
        }
}
/* dW[I][O] = x^T dy, db[O] = column sums of dy, dx[N][I] = dy W^T (W may be another version) */
static void lin_bwd(const double* dy, const double* x, const double* W, long N, long I, long O, double* dx, double* dW,
                    double* db) {
    for (long i = 0; i < I; ++i)
        for (long o = 0; o < O; ++o) {
            double acc = 0.0;
            for (long n = 0; n < N; ++n) acc += x[n * I + i] * dy[n * O + o];
            dW[i * O + o] = acc;
        }
    for (long o = 0; o < O; ++o) {
        double acc = 0.0;
        for (long n = 0; n < N; ++n) acc += dy[n * O + o];
        db[o] = acc;
    }
    for (long n = 0; n < N; ++n)
        for (long i = 0; i < I; ++i) {
            double acc = 0.0;
            for (long o = 0; o < O; ++o) acc += dy[n * O + o] * W[i * O + o];
            dx[n * I + i] = acc;
        }
}
static double gelu(double u) { return 0.5 * u * (1.0 + erf(u / sqrt(2.0))); }
static double gelu_grad(double u) {
    return 0.5 * (1.0 + erf(u / sqrt(2.0))) + u * exp(-0.5 * u * u) / sqrt(2.0 * M_PI);
}
static int hidden(const shape_t* c, int q, int k, int valid) { return c->kind == 0 ? k > q : k >= valid; }

static void attn_fwd(const shape_t* c, const double* qkv, const int* valid_len, double* prob, double* out) {
    const long D = c->D, s = c->s, dh = D / c->H;
    const double scale = 1.0 / sqrt((double)dh);
    for (int seq = 0; seq < c->b; ++seq)
        for (int h = 0; h < c->H; ++h) {
            double* P = prob + ((long)seq * c->H + h) * s * s;
            const int valid = valid_len ? valid_len[seq] : (int)s;
            for (long q = 0; q < s; ++q) {
                const double* Q = qkv + (seq * s + q) * 3 * D + h * dh;
                double mx = -INFINITY;
                for (long k = 0; k < s; ++k) {
                    if (hidden(c, (int)q, (int)k, valid)) { P[q * s + k] = -INFINITY; continue; }
                    const double* K = qkv + (seq * s + k) * 3 * D + D + h * dh;
                    double sc = 0.0;
                    for (long d = 0; d < dh; ++d) sc += Q[d] * K[d];
                    P[q * s + k] = sc * scale;
                    if (P[q * s + k] > mx) mx = P[q * s + k];
                }
                double sum = 0.0;
                for (long k = 0; k < s; ++k) {
                    P[q * s + k] = isinf(P[q * s + k]) ? 0.0 : exp(P[q * s + k] - mx);
                    sum += P[q * s + k];
                }
                for (long k = 0; k < s; ++k) P[q * s + k] /= sum;
                for (long d = 0; d < dh; ++d) {
                    double acc = 0.0;
                    for (long k = 0; k < s; ++k) acc += P[q * s + k] * qkv[(seq * s + k) * 3 * D + 2 * D + h * dh + d];
                    out[(seq * s + q) * D + h * dh + d] = acc;
                }
            }
        }
}
static void attn_bwd(const shape_t* c, const double* dout, const double* qkv, const double* prob, double* dqkv,
                     double* ds_row) {
    const long D = c->D, s = c->s, dh = D / c->H, N = s * c->b;
    const double scale = 1.0 / sqrt((double)dh);
    for (long i = 0; i < N * 3 * D; ++i) dqkv[i] = 0.0;
    for (int seq = 0; seq < c->b; ++seq)
        for (int h = 0; h < c->H; ++h) {
            const double* P = prob + ((long)seq * c->H + h) * s * s;
            for (long q = 0; q < s; ++q) {
                const double* dO = dout + (seq * s + q) * D + h * dh;
                double dot = 0.0;
                for (long k = 0; k < s; ++k) {           /* dP[q][k] = dO[q] . V[k] */
                    const double* V = qkv + (seq * s + k) * 3 * D + 2 * D + h * dh;
                    double dp = 0.0;
                    for (long d = 0; d < dh; ++d) dp += dO[d] * V[d];
                    ds_row[k] = dp;
                    dot += dp * P[q * s + k];
                }
                for (long k = 0; k < s; ++k) {
                    const double ds = P[q * s + k] * (ds_row[k] - dot) * scale;
                    const double* K = qkv + (seq * s + k) * 3 * D + D + h * dh;
                    const double* Q = qkv + (seq * s + q) * 3 * D + h * dh;
                    for (long d = 0; d < dh; ++d) {
                        dqkv[(seq * s + q) * 3 * D + h * dh + d] += ds * K[d];               /* dQ */
                        dqkv[(seq * s + k) * 3 * D + D + h * dh + d] += ds * Q[d];           /* dK */
                        dqkv[(seq * s + k) * 3 * D + 2 * D + h * dh + d] += P[q * s + k] * dO[d]; /* dV */
                    }
                }
            }
        }
}

/* ---- stage ----------------------------------------------------------------- */
/* theta: L * layer_params doubles; x [N][D]; valid_len [b] or NULL (GPT); y [N][D];
 * saved: L * slow_saved_doubles_per_layer doubles. Returns 0, or -1 out of memory. */
int slow_stage_forward(int kind, int L, int D, int H, int F, int s, int b, double eps, const double* theta,
                       const double* x, const int* valid_len, double* y, double* saved) {
    shape_t c = {kind, L, D, H, F, s, b, eps};
    const long N = (long)s * b, per = slow_saved_doubles_per_layer(D, H, F, s, b);
    double* cur = (double*)malloc(sizeof(double) * N * D);
    double* t1 = (double*)malloc(sizeof(double) * N * D);
    double* t2 = (double*)malloc(sizeof(double) * N * D);
    if (!cur || !t1 || !t2) { free(cur); free(t1); free(t2); return -1; }
    memcpy(cur, x, sizeof(double) * N * D);
    for (int l = 0; l < L; ++l) {
        lparams_t p; saved_t sv;
        split_params(&c, theta + l * layer_params(&c), &p);
        split_saved(&c, saved + l * per, &sv);
        memcpy(sv.xin, cur, sizeof(double) * N * D);
        if (kind == 0) {
            ln_fwd(cur, p.g1, p.b1, eps, N, D, sv.ain, sv.xhat1, sv.rstd1);              /* a = LN1(x) */
            lin_fwd(sv.ain, p.wqkv, p.bqkv, N, D, 3 * D, sv.qkv);
            attn_fwd(&c, sv.qkv, NULL, sv.prob, sv.o);
            lin_fwd(sv.o, p.wo, p.bo, N, D, D, t1);
            for (long i = 0; i < N * D; ++i) sv.y1[i] = cur[i] + t1[i];                  /* y1 = x + Attn */
            ln_fwd(sv.y1, p.g2, p.b2, eps, N, D, sv.cin, sv.xhat2, sv.rstd2);            /* c = LN2(y1) */
            lin_fwd(sv.cin, p.w1, p.bf1, N, D, F, sv.u);
            for (long i = 0; i < N * F; ++i) sv.h[i] = gelu(sv.u[i]);
            lin_fwd(sv.h, p.w2, p.bf2, N, F, D, t2);
            for (long i = 0; i < N * D; ++i) cur[i] = sv.y1[i] + t2[i];
        } else {
            memcpy(sv.ain, cur, sizeof(double) * N * D);
            lin_fwd(sv.ain, p.wqkv, p.bqkv, N, D, 3 * D, sv.qkv);
            attn_fwd(&c, sv.qkv, valid_len, sv.prob, sv.o);
            lin_fwd(sv.o, p.wo, p.bo, N, D, D, t1);
            for (long i = 0; i < N * D; ++i) t1[i] += cur[i];                            /* r1 = x + Attn */
            ln_fwd(t1, p.g1, p.b1, eps, N, D, sv.y1, sv.xhat1, sv.rstd1);                /* y1 = LN1(r1) */
            memcpy(sv.cin, sv.y1, sizeof(double) * N * D);
            lin_fwd(sv.cin, p.w1, p.bf1, N, D, F, sv.u);
            for (long i = 0; i < N * F; ++i) sv.h[i] = gelu(sv.u[i]);
            lin_fwd(sv.h, p.w2, p.bf2, N, F, D, t2);
            for (long i = 0; i < N * D; ++i) t2[i] += sv.y1[i];                          /* r2 = y1 + MLP */
            ln_fwd(t2, p.g2, p.b2, eps, N, D, cur, sv.xhat2, sv.rstd2);                  /* y = LN2(r2) */
        }
    }
    memcpy(y, cur, sizeof(double) * N * D);
    free(cur); free(t1); free(t2);
    return 0;
}

/* theta may be another version than the forward's. dy [N][D]; dx [N][D]; grad: L * layer_params. */
int slow_stage_backward(int kind, int L, int D, int H, int F, int s, int b, double eps, const double* theta,
                        const double* saved, const double* dy, double* dx, double* grad) {
    shape_t c = {kind, L, D, H, F, s, b, eps};
    const long N = (long)s * b, per = slow_saved_doubles_per_layer(D, H, F, s, b);
    double* d = (double*)malloc(sizeof(double) * N * D);
    double* dh = (double*)malloc(sizeof(double) * N * F);
    double* t1 = (double*)malloc(sizeof(double) * N * D);
    double* t2 = (double*)malloc(sizeof(double) * N * D);
    double* dqkv = (double*)malloc(sizeof(double) * N * 3 * D);
    double* row = (double*)malloc(sizeof(double) * s);
    if (!d || !dh || !t1 || !t2 || !dqkv || !row) { free(d); free(dh); free(t1); free(t2); free(dqkv); free(row); return -1; }
    memcpy(d, dy, sizeof(double) * N * D);
    for (int l = L - 1; l >= 0; --l) {
        lparams_t p; lgrads_t g; saved_t sv;
        split_params(&c, theta + l * layer_params(&c), &p);
        split_grads(&c, grad + l * layer_params(&c), &g);
        split_saved(&c, (double*)saved + l * per, &sv);
        if (kind == 0) {
            /* y = y1 + W2 gelu(W1 LN2(y1)) */
            lin_bwd(d, sv.h, p.w2, N, F, D, dh, g.w2, g.bf2);
            for (long i = 0; i < N * F; ++i) dh[i] *= gelu_grad(sv.u[i]);
            lin_bwd(dh, sv.cin, p.w1, N, D, F, t1, g.w1, g.bf1);                        /* t1 = dc */
            ln_bwd(t1, sv.xhat2, sv.rstd2, p.g2, N, D, t2, g.g2, g.b2);
            for (long i = 0; i < N * D; ++i) d[i] += t2[i];                              /* d = dy1 */
            /* y1 = x + Wo Attn(Wqkv LN1(x)) */
            lin_bwd(d, sv.o, p.wo, N, D, D, t1, g.wo, g.bo);                             /* t1 = dO */
            attn_bwd(&c, t1, sv.qkv, sv.prob, dqkv, row);
            lin_bwd(dqkv, sv.ain, p.wqkv, N, D, 3 * D, t1, g.wqkv, g.bqkv);              /* t1 = da */
            ln_bwd(t1, sv.xhat1, sv.rstd1, p.g1, N, D, t2, g.g1, g.b1);
            for (long i = 0; i < N * D; ++i) d[i] += t2[i];
        } else {
            /* y = LN2(r2), r2 = y1 + MLP(y1) */
            ln_bwd(d, sv.xhat2, sv.rstd2, p.g2, N, D, t1, g.g2, g.b2);                   /* t1 = dr2 */
            lin_bwd(t1, sv.h, p.w2, N, F, D, dh, g.w2, g.bf2);
            for (long i = 0; i < N * F; ++i) dh[i] *= gelu_grad(sv.u[i]);
            lin_bwd(dh, sv.cin, p.w1, N, D, F, t2, g.w1, g.bf1);
            for (long i = 0; i < N * D; ++i) t1[i] += t2[i];                             /* t1 = dy1 */
            /* y1 = LN1(r1), r1 = x + Attn(x) */
            ln_bwd(t1, sv.xhat1, sv.rstd1, p.g1, N, D, d, g.g1, g.b1);                   /* d = dr1 */
            lin_bwd(d, sv.o, p.wo, N, D, D, t1, g.wo, g.bo);
            attn_bwd(&c, t1, sv.qkv, sv.prob, dqkv, row);
            lin_bwd(dqkv, sv.ain, p.wqkv, N, D, 3 * D, t2, g.wqkv, g.bqkv);
            for (long i = 0; i < N * D; ++i) d[i] += t2[i];
        }
    }
    memcpy(dx, d, sizeof(double) * N * D);
    free(d); free(dh); free(t1); free(t2); free(dqkv); free(row);
    return 0;
}
