/*
 * CPU oracle for the batch-1 decoder forward (TEST INFRASTRUCTURE, not product).
 *
 * This file is the plain, slow definition of what the GPU library computes:
 * the two-phase execution of the paper's Section 3.5 (Eq. 3: KV <- Prefill(x_1:T);
 * Eq. 4: y_t <- DecodeStep(y_{t-1}, KV), KV <- UpdateKV(KV, y_t)) for the
 * pre-norm GQA / SwiGLU decoder whose operators the paper lists in Section 3.4
 * (QKV, RoPE, KV-cache write, attention, OProj, GateUp, DownProj,
 * normalisation, activation, greedy sampling as in Section 4.2).
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
 * it.  It shares no code with the HIP path.
 *
 * Arithmetic: every value and every accumulator is `real` (double unless the
 * file is compiled with -DORACLE_REAL=float, a variant kept only to measure
 * how much fp32 evaluation order matters).  Stored 16-bit tensors (weights,
 * embeddings, KV cache) are upcast exactly.  Each dot product is one
 * sequential accumulation in index order.  The only parallelism is an OpenMP
 * loop over independent outputs; it never changes the arithmetic.
 *
 * A block of n new positions is evaluated layer by layer (position t of a
 * layer needs only the cache rows 0..p0+t of that layer), so prefill is a
 * block of T positions and a decode step is a block of one position; both run
 * the same code and both read K/V back from the (rounded) cache.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

#define ORACLE_F16 1
#define ORACLE_BF16 2
#define ORACLE_FP8 3 /* e4m3, no infinities, largest finite value 448: KV-cache storage only; code in the low byte */

typedef struct {
    uint32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab;
    uint32_t max_seq_len;
    double rms_eps, rope_theta;
    uint32_t weight_dtype, kv_dtype;  /* weights: ORACLE_F16 / ORACLE_BF16; cache: those or ORACLE_FP8 */
    uint32_t tie_embeddings, qkv_bias;
    uint32_t kv_round; /* 1: cache holds values rounded to kv_dtype (the method); 0: unrounded (diagnostic) */
} oracle_config;

typedef struct {
    const uint16_t *embed, *lm_head, *final_norm;
    const uint16_t *const *attn_norm, *const *wqkv, *const *bqkv, *const *wo;
    const uint16_t *const *mlp_norm, *const *w_gate_up, *const *w_down;
} oracle_weights;

typedef struct {
    oracle_config c;
    oracle_weights w; /* borrowed: the caller keeps the arrays alive */
    const uint16_t **ptrs;
    real *kcache, *vcache; /* [L][n_kv][max_seq][d] */
    uint32_t kv_len;
} oracle_model;

/* ------------------------------------------------------------------ */
/* 16-bit storage formats                                              */
/* ------------------------------------------------------------------ */
static double bits_to_double(uint16_t b, uint32_t dtype) {
    if (dtype == ORACLE_BF16) {
        uint32_t u = (uint32_t)b << 16;
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
    /* IEEE binary16 */
    int sign = (b >> 15) & 1, e = (b >> 10) & 31, m = b & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

/* Cache storage codes: the 16-bit formats above, or 8-bit e4m3 (code in the low byte): sign, 4 exponent bits
 * (bias 7), 3 mantissa bits; exponent 15 with mantissa 7 is NaN, there are no infinities.  Kept apart from
 * bits_to_double, which sits in the innermost loop of every matrix product. */
static double cache_bits_to_double(uint16_t b, uint32_t dtype) {
    if (dtype != ORACLE_FP8) return bits_to_double(b, dtype);
    int s8 = (b >> 7) & 1, e8 = (b >> 3) & 15, m8 = b & 7;
    double v8;
    if (e8 == 15 && m8 == 7) v8 = NAN;
    else if (e8 == 0) v8 = ldexp((double)m8, -9);
    else v8 = ldexp((double)(8 + m8), e8 - 10);
    return s8 ? -v8 : v8;
}

/* Round to nearest, ties to even, onto a binary format with `p` significand
 * bits (implicit one included), minimum normal exponent emin, maximum finite
 * value maxv.  Result returned as a double that is exactly representable. */
static double round_to_format(double x, int p, int emin, double maxv) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e); /* |x| = f * 2^e, f in [0.5,1) -> leading bit has weight 2^(e-1) */
    int lead = e - 1;
    if (lead < emin) lead = emin;              /* subnormal range: fixed quantum */
    int q = lead - (p - 1);                    /* weight of the last kept bit */
    double r = ldexp(nearbyint(ldexp(x, -q)), q); /* default rounding mode = ties-to-even */
    if (fabs(r) > maxv) r = x > 0 ? INFINITY : -INFINITY;
    return r;
}

double oracle_round_kv(double x, uint32_t dtype) {
    if (dtype == ORACLE_BF16) return round_to_format(x, 8, -126, 3.3895313892515355e38);
    if (dtype == ORACLE_FP8) { /* the format has no infinity: what rounds beyond 448 stays at 448 */
        double r = round_to_format(x, 4, -6, 448.0);
        return isinf(r) ? (r > 0 ? 448.0 : -448.0) : r;
    }
    return round_to_format(x, 11, -14, 65504.0);
}

double oracle_upcast(uint16_t bits, uint32_t dtype) { return cache_bits_to_double(bits, dtype); }

/* ------------------------------------------------------------------ */
/* Operators (Section 3.4 names them; the formulas are the standard    */
/* ones for this decoder family)                                       */
/* ------------------------------------------------------------------ */

/* RMSNorm: y_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i. */
void oracle_rmsnorm(const real *x, const uint16_t *gain, uint32_t dtype, uint32_t n, double eps, real *y) {
    real ss = 0;
    for (uint32_t i = 0; i < n; ++i) ss += x[i] * x[i];
    real inv = (real)1 / (real)sqrt((double)(ss / (real)n) + eps);
    for (uint32_t i = 0; i < n; ++i) y[i] = x[i] * inv * (real)bits_to_double(gain[i], dtype);
}

/* y[r] = sum_k W[r][k] a[k] (+ b[r]), W row-major [rows, cols] in 16-bit storage. */
void oracle_matvec(const uint16_t *W, const uint16_t *bias, uint32_t dtype, uint32_t rows, uint32_t cols,
                   const real *a, real *y) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < (int64_t)rows; ++r) {
        const uint16_t *w = W + (size_t)r * cols;
        real acc = 0;
        for (uint32_t k = 0; k < cols; ++k) acc += (real)bits_to_double(w[k], dtype) * a[k];
        if (bias) acc += (real)bits_to_double(bias[r], dtype);
        y[r] = acc;
    }
}

/* Y[t][r] = sum_k W[r][k] A[t][k] (+ b[r]) for t < n: the same definition for a
 * block of positions.  At is A transposed ([cols][n]) so that the k-loop can
 * update all n sums side by side; every sum is still accumulated sequentially
 * in k order. */
static void matmul_block(const uint16_t *W, const uint16_t *bias, uint32_t dtype, uint32_t rows, uint32_t cols,
                         const real *A, uint32_t n, real *Y /* [n][rows] */) {
    if (n == 1) {
        oracle_matvec(W, bias, dtype, rows, cols, A, Y);
        return;
    }
    real *At = (real *)malloc(sizeof(real) * (size_t)cols * n);
    for (uint32_t t = 0; t < n; ++t)
        for (uint32_t k = 0; k < cols; ++k) At[(size_t)k * n + t] = A[(size_t)t * cols + k];
#pragma omp parallel
    {
        real *acc = (real *)malloc(sizeof(real) * n);
#pragma omp for schedule(static)
        for (int64_t r = 0; r < (int64_t)rows; ++r) {
            const uint16_t *w = W + (size_t)r * cols;
            for (uint32_t t = 0; t < n; ++t) acc[t] = 0;
            for (uint32_t k = 0; k < cols; ++k) {
                const real wk = (real)bits_to_double(w[k], dtype);
                const real *restrict a = At + (size_t)k * n;
                real *restrict s = acc;
                for (uint32_t t = 0; t < n; ++t) s[t] += wk * a[t]; /* n independent sums, each in k order */
            }
            real b = bias ? (real)bits_to_double(bias[r], dtype) : (real)0;
            for (uint32_t t = 0; t < n; ++t) Y[(size_t)t * rows + r] = acc[t] + b;
        }
        free(acc);
    }
    free(At);
}

/* Rotary embedding of one head at absolute position pos (0-based), in the
 * slice / negate / concat form of Appendix B.3:
 *   y = x * cos + concat(-x[d/2:], x[:d/2]) * sin,  angle_i = pos * theta^(-2i/d)
 * for i in [0, d/2), the same angle for elements i and i + d/2.
 * Angles and their cos/sin are evaluated in double. */
void oracle_rope(const real *x, uint32_t d, uint32_t pos, double theta, real *y) {
    uint32_t half = d / 2;
    for (uint32_t i = 0; i < half; ++i) {
        double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)d);
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = x[i], b = x[i + half];
        y[i] = a * c - b * s;
        y[i + half] = b * c + a * s;
    }
}

/* Single-query attention over cache rows 0..n_keys-1 of one KV head:
 * s_j = q.K_j / sqrt(d); a = softmax(s); o = sum_j a_j V_j.  Causality is the
 * loop bound (no mask constant, cf. Appendix B.3 item 3).  K, V: [n_keys][d]
 * with row stride `stride`.  probs (optional) receives a_j. */
void oracle_attend(const real *q, const real *K, const real *V, uint32_t n_keys, uint32_t d, size_t stride,
                   real *o, real *probs) {
    real *s = (real *)malloc(sizeof(real) * n_keys);
    real scale = (real)(1.0 / sqrt((double)d));
    real mx = 0;
    for (uint32_t j = 0; j < n_keys; ++j) {
        real acc = 0;
        const real *k = K + (size_t)j * stride;
        for (uint32_t i = 0; i < d; ++i) acc += q[i] * k[i];
        s[j] = acc * scale;
        if (j == 0 || s[j] > mx) mx = s[j];
    }
    real den = 0;
    for (uint32_t j = 0; j < n_keys; ++j) {
        s[j] = (real)exp((double)(s[j] - mx));
        den += s[j];
    }
    for (uint32_t i = 0; i < d; ++i) o[i] = 0;
    for (uint32_t j = 0; j < n_keys; ++j) {
        real a = s[j] / den;
        if (probs) probs[j] = a;
        const real *v = V + (size_t)j * stride;
        for (uint32_t i = 0; i < d; ++i) o[i] += a * v[i];
    }
    free(s);
}

/* SwiGLU: h_j = silu(g_j) * u_j, silu(z) = z / (1 + exp(-z)). */
void oracle_swiglu(const real *gate, const real *up, uint32_t n, real *h) {
    for (uint32_t j = 0; j < n; ++j) h[j] = gate[j] / ((real)1 + (real)exp(-(double)gate[j])) * up[j];
}

/* Greedy sampling: index of the maximum, lowest index on ties. */
int32_t oracle_argmax(const real *x, uint32_t n) {
    uint32_t best = 0;
    for (uint32_t i = 1; i < n; ++i)
        if (x[i] > x[best]) best = i;
    return (int32_t)best;
}

/* ------------------------------------------------------------------ */
/* Model object                                                        */
/* ------------------------------------------------------------------ */
static size_t cache_elems(const oracle_config *c) {
    return (size_t)c->n_layers * c->n_kv_heads * c->max_seq_len * c->head_dim;
}
static real *cache_row(real *base, const oracle_config *c, uint32_t layer, uint32_t kvh, uint32_t pos) {
    return base + (((size_t)layer * c->n_kv_heads + kvh) * c->max_seq_len + pos) * c->head_dim;
}

oracle_model *oracle_create(const oracle_config *cfg, const oracle_weights *w) {
    if (!cfg || !w || cfg->n_layers == 0 || cfg->n_kv_heads == 0 || cfg->n_q_heads % cfg->n_kv_heads ||
        cfg->head_dim % 2 || cfg->head_dim > 512)
        return NULL;
    oracle_model *m = (oracle_model *)calloc(1, sizeof(oracle_model));
    m->c = *cfg;
    uint32_t L = cfg->n_layers;
    /* copy the per-layer pointer tables so the caller's tables may go away */
    m->ptrs = (const uint16_t **)malloc(sizeof(void *) * 7 * L);
    const uint16_t *const *src[7] = {w->attn_norm, w->wqkv, w->bqkv, w->wo, w->mlp_norm, w->w_gate_up, w->w_down};
    for (int a = 0; a < 7; ++a)
        for (uint32_t l = 0; l < L; ++l) m->ptrs[a * L + l] = src[a] ? src[a][l] : NULL;
    m->w = *w;
    m->w.attn_norm = m->ptrs + 0 * L;
    m->w.wqkv = m->ptrs + 1 * L;
    m->w.bqkv = m->ptrs + 2 * L;
    m->w.wo = m->ptrs + 3 * L;
    m->w.mlp_norm = m->ptrs + 4 * L;
    m->w.w_gate_up = m->ptrs + 5 * L;
    m->w.w_down = m->ptrs + 6 * L;
    m->kcache = (real *)calloc(cache_elems(cfg), sizeof(real));
    m->vcache = (real *)calloc(cache_elems(cfg), sizeof(real));
    if (!m->kcache || !m->vcache) {
        free(m->kcache); free(m->vcache); free(m->ptrs); free(m);
        return NULL;
    }
    return m;
}

void oracle_destroy(oracle_model *m) {
    if (!m) return;
    free(m->kcache); free(m->vcache); free(m->ptrs); free(m);
}

uint32_t oracle_kv_len(const oracle_model *m) { return m->kv_len; }

/* Section 3.7 "release or recycle": keep the first keep_len positions (Eq. 5 prefix reuse), drop the rest. */
int oracle_kv_reset(oracle_model *m, uint32_t keep_len) {
    if (keep_len > m->kv_len) return -1;
    m->kv_len = keep_len;
    return 0;
}

/* Read one cache position of one layer: k, v are [n_kv*d]. */
int oracle_kv_read(const oracle_model *m, uint32_t layer, uint32_t pos, real *k, real *v) {
    const oracle_config *c = &m->c;
    if (layer >= c->n_layers || pos >= c->max_seq_len) return -1;
    for (uint32_t h = 0; h < c->n_kv_heads; ++h) {
        memcpy(k + (size_t)h * c->head_dim, cache_row(m->kcache, c, layer, h, pos), sizeof(real) * c->head_dim);
        memcpy(v + (size_t)h * c->head_dim, cache_row(m->vcache, c, layer, h, pos), sizeof(real) * c->head_dim);
    }
    return 0;
}

/* Inject n_pos cache rows (kv dtype bits, [n_pos][n_kv*d]) at positions 0.. of one layer. */
int oracle_kv_write(oracle_model *m, uint32_t layer, uint32_t n_pos, const uint16_t *k, const uint16_t *v) {
    const oracle_config *c = &m->c;
    if (layer >= c->n_layers || n_pos > c->max_seq_len) return -1;
    for (uint32_t p = 0; p < n_pos; ++p)
        for (uint32_t h = 0; h < c->n_kv_heads; ++h) {
            real *kr = cache_row(m->kcache, c, layer, h, p), *vr = cache_row(m->vcache, c, layer, h, p);
            for (uint32_t i = 0; i < c->head_dim; ++i) {
                size_t s = ((size_t)p * c->n_kv_heads + h) * c->head_dim + i;
                kr[i] = (real)cache_bits_to_double(k[s], c->kv_dtype);
                vr[i] = (real)cache_bits_to_double(v[s], c->kv_dtype);
            }
        }
    return 0;
}

/* Declare the first n positions valid (after oracle_kv_write on every layer). */
int oracle_kv_set_len(oracle_model *m, uint32_t n) {
    if (n > m->c.max_seq_len) return -1;
    m->kv_len = n;
    return 0;
}

/*
 * Evaluate n = n_embeds + n_tokens new positions p0 .. p0+n-1 (p0 = kv_len):
 * the caller's embedding rows first, then the token ids.
 *   hidden_out : NULL or [n][hidden], final-norm output of every new position
 *   logits_mode: 0 none, 1 last position only ([vocab]), 2 every position ([n][vocab])
 *   next_out   : NULL or argmax of each logits row produced
 * Returns 0, or a negative code: -1 bad argument, -2 context overflow, -3 bad token id.
 */
int oracle_forward(oracle_model *m, const uint16_t *embeds, uint32_t n_embeds, const int32_t *tokens,
                   uint32_t n_tokens, real *hidden_out, int logits_mode, real *logits_out, int32_t *next_out) {
    const oracle_config *c = &m->c;
    const uint32_t H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, I = c->intermediate;
    const uint32_t g = nq / nkv, qd = nq * d, kvd = nkv * d, R = qd + 2 * kvd, wd = c->weight_dtype;
    const uint32_t n = n_embeds + n_tokens, p0 = m->kv_len;
    if (n == 0 || (logits_mode == 2 && !logits_out)) return -1;
    if ((uint64_t)p0 + n > c->max_seq_len) return -2;
    for (uint32_t t = 0; t < n_tokens; ++t)
        if (tokens[t] < 0 || (uint32_t)tokens[t] >= c->vocab) return -3;

    real *x = (real *)malloc(sizeof(real) * (size_t)n * H);      /* residual stream */
    real *a = (real *)malloc(sizeof(real) * (size_t)n * H);      /* normed input   */
    real *qkv = (real *)malloc(sizeof(real) * (size_t)n * R);
    real *att = (real *)malloc(sizeof(real) * (size_t)n * qd);
    real *proj = (real *)malloc(sizeof(real) * (size_t)n * H);
    real *gu = (real *)malloc(sizeof(real) * (size_t)n * 2 * I);
    real *hh = (real *)malloc(sizeof(real) * (size_t)n * I);

    /* 1. embeddings */
    for (uint32_t t = 0; t < n; ++t) {
        const uint16_t *row = t < n_embeds ? embeds + (size_t)t * H
                                           : m->w.embed + (size_t)tokens[t - n_embeds] * H;
        for (uint32_t i = 0; i < H; ++i) x[(size_t)t * H + i] = (real)bits_to_double(row[i], wd);
    }

    for (uint32_t l = 0; l < c->n_layers; ++l) {
        /* 2. attention RMSNorm, 3. fused QKV projection (rows Q | K | V) */
        for (uint32_t t = 0; t < n; ++t)
            oracle_rmsnorm(x + (size_t)t * H, m->w.attn_norm[l], wd, H, c->rms_eps, a + (size_t)t * H);
        matmul_block(m->w.wqkv[l], c->qkv_bias ? m->w.bqkv[l] : NULL, wd, R, H, a, n, qkv);

        /* 4. RoPE on q and k heads, 5. cache write (rounded to the cache dtype) */
        for (uint32_t t = 0; t < n; ++t) {
            real *row = qkv + (size_t)t * R;
            real tmp[512];
            for (uint32_t h = 0; h < nq + nkv; ++h) {
                oracle_rope(row + (size_t)h * d, d, p0 + t, c->rope_theta, tmp);
                memcpy(row + (size_t)h * d, tmp, sizeof(real) * d);
            }
            for (uint32_t h = 0; h < nkv; ++h) {
                real *kr = cache_row(m->kcache, c, l, h, p0 + t), *vr = cache_row(m->vcache, c, l, h, p0 + t);
                const real *ks = row + qd + (size_t)h * d, *vs = row + qd + kvd + (size_t)h * d;
                for (uint32_t i = 0; i < d; ++i) {
                    kr[i] = c->kv_round ? (real)oracle_round_kv((double)ks[i], c->kv_dtype) : ks[i];
                    vr[i] = c->kv_round ? (real)oracle_round_kv((double)vs[i], c->kv_dtype) : vs[i];
                }
            }
        }

        /* 6. causal GQA attention: query head h reads KV head h / g, keys 0 .. p0+t */
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
        for (int64_t t = 0; t < (int64_t)n; ++t)
            for (int64_t h = 0; h < (int64_t)nq; ++h) {
                uint32_t kvh = (uint32_t)h / g;
                oracle_attend(qkv + (size_t)t * R + (size_t)h * d, cache_row(m->kcache, c, l, kvh, 0),
                              cache_row(m->vcache, c, l, kvh, 0), p0 + (uint32_t)t + 1, d, d,
                              att + (size_t)t * qd + (size_t)h * d, NULL);
            }

        /* 7. output projection + residual */
        matmul_block(m->w.wo[l], NULL, wd, H, qd, att, n, proj);
        for (size_t i = 0; i < (size_t)n * H; ++i) x[i] += proj[i];

        /* 8. MLP RMSNorm, gate/up projection (rows gate | up), SwiGLU, down projection + residual */
        for (uint32_t t = 0; t < n; ++t)
            oracle_rmsnorm(x + (size_t)t * H, m->w.mlp_norm[l], wd, H, c->rms_eps, a + (size_t)t * H);
        matmul_block(m->w.w_gate_up[l], NULL, wd, 2 * I, H, a, n, gu);
        for (uint32_t t = 0; t < n; ++t)
            oracle_swiglu(gu + (size_t)t * 2 * I, gu + (size_t)t * 2 * I + I, I, hh + (size_t)t * I);
        matmul_block(m->w.w_down[l], NULL, wd, H, I, hh, n, proj);
        for (size_t i = 0; i < (size_t)n * H; ++i) x[i] += proj[i];
    }
    m->kv_len = p0 + n;

    /* 9. final RMSNorm, lm_head (the embedding matrix when tied), greedy argmax */
    for (uint32_t t = 0; t < n; ++t)
        oracle_rmsnorm(x + (size_t)t * H, m->w.final_norm, wd, H, c->rms_eps, a + (size_t)t * H);
    if (hidden_out) memcpy(hidden_out, a, sizeof(real) * (size_t)n * H);
    const uint16_t *lm = c->tie_embeddings ? m->w.embed : m->w.lm_head;
    if (logits_mode == 1) {
        real *lg = logits_out ? logits_out : (real *)malloc(sizeof(real) * c->vocab);
        oracle_matvec(lm, NULL, wd, c->vocab, H, a + (size_t)(n - 1) * H, lg);
        if (next_out) next_out[0] = oracle_argmax(lg, c->vocab);
        if (!logits_out) free(lg);
    } else if (logits_mode == 2) {
        matmul_block(lm, NULL, wd, c->vocab, H, a, n, logits_out);
        if (next_out)
            for (uint32_t t = 0; t < n; ++t) next_out[t] = oracle_argmax(logits_out + (size_t)t * c->vocab, c->vocab);
    }
    free(x); free(a); free(qkv); free(att); free(proj); free(gu); free(hh);
    return 0;
}

int oracle_real_bytes(void) { return (int)sizeof(real); }

/* threads the OpenMP loops will use */
int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
