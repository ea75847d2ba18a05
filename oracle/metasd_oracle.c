/*
 * MetaSD reference oracle (CPU, plain C).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * MetaSD hot path computes.  It is called from tests/, from __graft_entry__.smoke() and from
 * the cpu_baseline leg of bench.py, and from nowhere else.  It shares no code, header, table
 * or constant with the HIP library.
 *
 * What is implemented, and the passage of the paper each part follows:
 *   om_forward      - the "M_p(x | x_1..x_l, ...)" / "M_q(...)" of Alg. 3 (speculative sampling):
 *                     a Llama-style decoder (Sec. 4 "Experimental setup": Llama architecture, SiLU)
 *                     run over a block of m positions against a KV cache.
 *   om_forward_rows - the same decoder over rows that form a token tree rather than a chain (tree attention,
 *                     Sec. 4 "Number of drafts"): per-row cache slot, position and set of visible slots.
 *   om_sample       - "x ~ M_q(...)" (Alg. 3, drafting loop) by inverse CDF, or argmax for T=0.
 *   om_accept       - Alg. 3, the accept / residual-resample / bonus-token part, plus the
 *                     per-position 1 - d_TV(p, q) terms of the block-divergence reward (Def. 2).
 *   om_ucb_*        - Alg. 2 (MetaSD-UCB): initial sweep over the arms, UCB index, mean update.
 *   om_philox / om_uniform - counter-based uniforms (Philox4x32-10, Salmon et al. 2011) so the
 *                     GPU library can draw the same numbers from its own implementation.
 *
 * Precision: values are stored as float; every reduction (dot products, softmax sums, CDFs,
 * bandit means) accumulates in double.  For dtype == 1 ("bf16 model") the weights and the KV
 * cache are bf16 (K and V are rounded to nearest-even when they are written to the cache);
 * activations, the residual stream and logits are float.  The paper does not fix an
 * activation precision (it mentions float16 only for the memory footprint); rounding every GEMM
 * operand to bf16 as well would make any two implementations diverge by about one bf16 ulp per
 * element after a few layers (a single flipped rounding perturbs all later roundings), which
 * leaves nothing tight to compare.
 *
 * Parity pins: see the header of oracle/__init__.py for which test pins which function.
 *   om_philox: pinned word for word against rocRAND's Philox4x32-10 host generator (an implementation
 *   neither side of this repository wrote) for counters (c0, c1, 0, 0) under several keys
 *   (tests/test_gpu_philox_pin.py; it needs a machine with a GPU because rocRAND's host generator
 *   allocates through the HIP runtime), and by structural and statistical tests on the CPU.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n_layers;   /* layers that are run */
    int32_t d_model;
    int32_t n_heads;
    int32_t n_kv_heads;
    int32_t d_ffn;
    int32_t vocab;
    int32_t act;        /* 0 = GELU (erf) two-matrix FFN, 1 = SwiGLU three-matrix FFN */
    int32_t dtype;      /* 0 = fp32 model, 1 = bf16 model */
    float rms_eps;
    float rope_theta;
} om_desc;

/* Weight table order: embed, then per layer
 *   attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down   (w_gate unused for GELU)
 * then final_norm, lm_head.  Matrices are [out_features][in_features] row-major. */
#define OM_PER_LAYER 9

typedef struct {
    om_desc d;
    const void **w;
    int32_t max_ctx;
    int32_t hd;
    float *kc; /* [layer][kv_head][max_ctx][hd] */
    float *vc;
    int borrowed; /* kc / vc belong to another model (early-exit drafter reading the target's cache) */
} om_model;

/* ---------------------------------------------------------------- helpers */

static float bf16_bits_to_float(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even to bf16, returned widened to float */
static float round_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return f; /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

float om_round_bf16(float f) { return round_bf16(f); }

static inline float rnd(const om_desc *d, double v) {
    float f = (float)v;
    return d->dtype == 1 ? round_bf16(f) : f;
}

static inline double wget(const om_desc *d, const void *w, size_t i) {
    if (d->dtype == 1) return (double)bf16_bits_to_float(((const uint16_t *)w)[i]);
    return (double)((const float *)w)[i];
}

/* y[m][n] = sum_k x[m][k] * W[n][k]   (double accumulation, float result) */
static void matmul(const om_desc *d, const float *x, int m, int K, const void *W, int N, float *y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int r = 0; r < m; ++r) {
            double acc = 0.0;
            const float *xr = x + (size_t)r * K;
            if (d->dtype == 1) {
                const uint16_t *wr = (const uint16_t *)W + (size_t)n * K;
                for (int k = 0; k < K; ++k) acc += (double)xr[k] * (double)bf16_bits_to_float(wr[k]);
            } else {
                const float *wr = (const float *)W + (size_t)n * K;
                for (int k = 0; k < K; ++k) acc += (double)xr[k] * (double)wr[k];
            }
            y[(size_t)r * N + n] = (float)acc;
        }
    }
}

/* out[r][:] = h[r][:] / sqrt(mean(h[r]^2) + eps) * g[:] */
static void rmsnorm(const om_desc *d, const float *h, int m, int D, const void *g, float *out) {
    for (int r = 0; r < m; ++r) {
        double ss = 0.0;
        for (int i = 0; i < D; ++i) ss += (double)h[(size_t)r * D + i] * (double)h[(size_t)r * D + i];
        double inv = 1.0 / sqrt(ss / (double)D + (double)d->rms_eps);
        for (int i = 0; i < D; ++i)
            out[(size_t)r * D + i] = (float)((double)h[(size_t)r * D + i] * inv * wget(d, g, (size_t)i));
    }
}

/* Rotary embedding, rotate-half pairing (i, i + hd/2), angle = pos * theta^(-2i/hd). In place. */
void om_rope(float *v, int hd, int pos, float theta) {
    int half = hd / 2;
    for (int i = 0; i < half; ++i) {
        double freq = pow((double)theta, -2.0 * (double)i / (double)hd);
        double ang = (double)pos * freq;
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = (float)(a * c - b * s);
        v[i + half] = (float)(a * s + b * c);
    }
}

static double gelu_erf(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }
static double silu(double x) { return x / (1.0 + exp(-x)); }

/* ---------------------------------------------------------------- model */

om_model *om_model_create(const om_desc *d, const void *const *weights, int32_t max_ctx) {
    om_model *m = (om_model *)calloc(1, sizeof(om_model));
    if (!m) return NULL;
    m->d = *d;
    int nw = 1 + OM_PER_LAYER * d->n_layers + 2;
    m->w = (const void **)malloc(sizeof(void *) * (size_t)nw);
    memcpy(m->w, weights, sizeof(void *) * (size_t)nw);
    m->max_ctx = max_ctx;
    m->hd = d->d_model / d->n_heads;
    size_t n = (size_t)d->n_layers * d->n_kv_heads * (size_t)max_ctx * m->hd;
    m->kc = (float *)calloc(n, sizeof(float));
    m->vc = (float *)calloc(n, sizeof(float));
    if (!m->kc || !m->vc) { free(m->kc); free(m->vc); free(m->w); free(m); return NULL; }
    return m;
}

/* An early-exit drafter that keeps no cache of its own (the paper's appendix on switching costs / efficient KV-cache
 * strategies: avoid recomputing K/V when a drafter is switched in).  Its layers are the owner's first d->n_layers
 * layers, so K/V of those layers at any position are the owner's by definition; the cache is layer-major, so the
 * owner's arrays serve as they are.  The caller passes the same weight arrays for those layers. */
om_model *om_model_create_shared(const om_desc *d, const void *const *weights, om_model *owner) {
    if (!owner || d->n_layers > owner->d.n_layers || d->d_model != owner->d.d_model || d->n_heads != owner->d.n_heads ||
        d->n_kv_heads != owner->d.n_kv_heads || d->dtype != owner->d.dtype)
        return NULL;
    om_model *m = (om_model *)calloc(1, sizeof(om_model));
    if (!m) return NULL;
    m->d = *d;
    int nw = 1 + OM_PER_LAYER * d->n_layers + 2;
    m->w = (const void **)malloc(sizeof(void *) * (size_t)nw);
    memcpy(m->w, weights, sizeof(void *) * (size_t)nw);
    m->max_ctx = owner->max_ctx;
    m->hd = owner->hd;
    m->kc = owner->kc;
    m->vc = owner->vc;
    m->borrowed = 1;
    return m;
}

void om_model_free(om_model *m) {
    if (!m) return;
    if (!m->borrowed) { free(m->kc); free(m->vc); }
    free((void *)m->w); free(m);
}

/* which: 0 = K cache, 1 = V cache; layout [layer][kv_head][max_ctx][hd] */
float *om_model_kv(om_model *m, int which) { return which ? m->vc : m->kc; }

/*
 * Block forward over m tokens placed at positions pos0 .. pos0+m-1.  Positions < pos0 are taken
 * from the KV cache; K/V of the block are written to the cache.  Row r attends to positions
 * 0 .. pos0+r (causal).  logits: NULL (none), or [m][V] when last_only == 0, or [V] holding the
 * last row's logits when last_only != 0.  Returns 0, or -1 on bad arguments.
 */
/*
 * om_forward_ex: om_forward with two optional additions used by drafters that run on the target's hidden states (the
 * white-box drafters of Sec. 4, "Eagle"; the paper gives no formulas for them - the reading is stated in oracle/loop.py):
 *   hidden_out [m][D]: the residual stream after the last layer of every row (the "feature" of that position);
 *   fc, feat_in [m][D]: the rows do not start from the token embedding alone but from
 *       h = W_fc . [embedding(token) ; feat_in[r]],   W_fc [D][2 D] row-major (no bias).
 * With fc == NULL and hidden_out == NULL it is om_forward, step for step.
 */
int om_forward_ex(om_model *M, const int32_t *tokens, int m, int pos0, float *logits, int last_only,
                  const void *fc, const float *feat_in, float *hidden_out);

int om_forward(om_model *M, const int32_t *tokens, int m, int pos0, float *logits, int last_only) {
    return om_forward_ex(M, tokens, m, pos0, logits, last_only, NULL, NULL, NULL);
}

int om_forward_ex(om_model *M, const int32_t *tokens, int m, int pos0, float *logits, int last_only,
                  const void *fc, const float *feat_in, float *hidden_out) {
    const om_desc *d = &M->d;
    const int D = d->d_model, H = d->n_heads, KH = d->n_kv_heads, hd = M->hd, F = d->d_ffn, V = d->vocab;
    const int DQ = H * hd, DKV = KH * hd;
    if (m <= 0 || pos0 < 0 || pos0 + m > M->max_ctx) return -1;
    for (int r = 0; r < m; ++r)
        if (tokens[r] < 0 || tokens[r] >= V) return -1;

    float *h = (float *)malloc(sizeof(float) * (size_t)m * D);
    float *a = (float *)malloc(sizeof(float) * (size_t)m * D);
    float *q = (float *)malloc(sizeof(float) * (size_t)m * DQ);
    float *k = (float *)malloc(sizeof(float) * (size_t)m * DKV);
    float *v = (float *)malloc(sizeof(float) * (size_t)m * DKV);
    float *o = (float *)malloc(sizeof(float) * (size_t)m * DQ);
    float *y = (float *)malloc(sizeof(float) * (size_t)m * D);
    float *g = (float *)malloc(sizeof(float) * (size_t)m * F);
    float *u = (float *)malloc(sizeof(float) * (size_t)m * F);

    const void *embed = M->w[0];
    for (int r = 0; r < m; ++r)
        for (int i = 0; i < D; ++i) h[(size_t)r * D + i] = (float)wget(d, embed, (size_t)tokens[r] * D + i);
    if (fc) {
        /* h = W_fc . [embedding ; feature] */
        float *cat = (float *)malloc(sizeof(float) * (size_t)m * 2 * D);
        for (int r = 0; r < m; ++r) {
            memcpy(cat + (size_t)r * 2 * D, h + (size_t)r * D, sizeof(float) * (size_t)D);
            memcpy(cat + (size_t)r * 2 * D + D, feat_in + (size_t)r * D, sizeof(float) * (size_t)D);
        }
        matmul(d, cat, m, 2 * D, fc, D, h);
        free(cat);
    }

    for (int L = 0; L < d->n_layers; ++L) {
        const void *const *w = M->w + 1 + OM_PER_LAYER * L;
        rmsnorm(d, h, m, D, w[0], a);
        matmul(d, a, m, D, w[1], DQ, q);
        matmul(d, a, m, D, w[2], DKV, k);
        matmul(d, a, m, D, w[3], DKV, v);
        for (int r = 0; r < m; ++r) {
            for (int hh = 0; hh < H; ++hh) {
                float *qv = q + (size_t)r * DQ + (size_t)hh * hd;
                om_rope(qv, hd, pos0 + r, d->rope_theta);
            }
            for (int kh = 0; kh < KH; ++kh) {
                float *kv = k + (size_t)r * DKV + (size_t)kh * hd;
                om_rope(kv, hd, pos0 + r, d->rope_theta);
                size_t base = (((size_t)L * KH + kh) * M->max_ctx + (size_t)(pos0 + r)) * hd;
                for (int i = 0; i < hd; ++i) {
                    M->kc[base + i] = rnd(d, kv[i]);
                    M->vc[base + i] = rnd(d, v[(size_t)r * DKV + (size_t)kh * hd + i]);
                }
            }
        }
        /* attention: query head hh uses KV head hh / (H / KH) */
        const double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
        for (int hh = 0; hh < H; ++hh) {
            int kh = hh / (H / KH);
            const float *Kc = M->kc + ((size_t)L * KH + kh) * (size_t)M->max_ctx * hd;
            const float *Vc = M->vc + ((size_t)L * KH + kh) * (size_t)M->max_ctx * hd;
            double *s = (double *)malloc(sizeof(double) * (size_t)(pos0 + m));
            double *acc = (double *)malloc(sizeof(double) * (size_t)hd);
            for (int r = 0; r < m; ++r) {
                const float *qv = q + (size_t)r * DQ + (size_t)hh * hd;
                int n = pos0 + r + 1;
                double mx = -INFINITY;
                for (int p = 0; p < n; ++p) {
                    double dot = 0.0;
                    for (int i = 0; i < hd; ++i) dot += (double)qv[i] * (double)Kc[(size_t)p * hd + i];
                    s[p] = dot * scale;
                    if (s[p] > mx) mx = s[p];
                }
                double Z = 0.0;
                for (int p = 0; p < n; ++p) { s[p] = exp(s[p] - mx); Z += s[p]; }
                for (int i = 0; i < hd; ++i) acc[i] = 0.0;
                for (int p = 0; p < n; ++p) {
                    double pw = s[p] / Z;
                    for (int i = 0; i < hd; ++i) acc[i] += pw * (double)Vc[(size_t)p * hd + i];
                }
                for (int i = 0; i < hd; ++i) o[(size_t)r * DQ + (size_t)hh * hd + i] = (float)acc[i];
            }
            free(s); free(acc);
        }
        matmul(d, o, m, DQ, w[4], D, y);
        for (size_t i = 0; i < (size_t)m * D; ++i) h[i] = (float)((double)h[i] + (double)y[i]);

        rmsnorm(d, h, m, D, w[5], a);
        matmul(d, a, m, D, w[7], F, u);
        if (d->act == 1) {
            matmul(d, a, m, D, w[6], F, g);
            for (size_t i = 0; i < (size_t)m * F; ++i) u[i] = (float)(silu((double)g[i]) * (double)u[i]);
        } else {
            for (size_t i = 0; i < (size_t)m * F; ++i) u[i] = (float)gelu_erf((double)u[i]);
        }
        matmul(d, u, m, F, w[8], D, y);
        for (size_t i = 0; i < (size_t)m * D; ++i) h[i] = (float)((double)h[i] + (double)y[i]);
    }

    if (hidden_out) memcpy(hidden_out, h, sizeof(float) * (size_t)m * D);
    if (logits) {
        const void *fn = M->w[1 + OM_PER_LAYER * d->n_layers];
        const void *head = M->w[2 + OM_PER_LAYER * d->n_layers];
        if (last_only) {
            rmsnorm(d, h + (size_t)(m - 1) * D, 1, D, fn, a);
            matmul(d, a, 1, D, head, V, logits);
        } else {
            rmsnorm(d, h, m, D, fn, a);
            matmul(d, a, m, D, head, V, logits);
        }
    }
    free(h); free(a); free(q); free(k); free(v); free(o); free(y); free(g); free(u);
    return 0;
}

/*
 * Forward over m rows that need not form a chain: tree attention (Sec. 4, "Number of drafts": multi-draft methods
 * verify a token tree with a tree-attention mechanism).  Row r carries token tokens[r]; its K/V are written to cache
 * slot slot[r]; its q and k are rotated for position pos[r]; it attends to exactly the cache slots p with
 * allow[r * max_ctx + p] != 0 (the caller lists them: the committed positions, the row's ancestors in the tree, the
 * row itself).  All rows' K/V are written before any row attends, so a row may attend to slots written by other rows
 * of the same call.  Everything else is om_forward's arithmetic, step for step; logits [m][V] (or NULL).
 * With slot[r] = pos[r] = pos0 + r and allow = (p <= pos0 + r) this IS om_forward.
 */
int om_forward_rows_ex(om_model *M, const int32_t *tokens, int m, const int32_t *slot, const int32_t *pos,
                       const uint8_t *allow, float *logits, const void *fc, const float *feat_in, float *hidden_out);

int om_forward_rows(om_model *M, const int32_t *tokens, int m, const int32_t *slot, const int32_t *pos,
                    const uint8_t *allow, float *logits) {
    return om_forward_rows_ex(M, tokens, m, slot, pos, allow, logits, NULL, NULL, NULL);
}

/* om_forward_rows with om_forward_ex's two optional additions (a drafter head's rows start from
 * W_fc . [embedding ; feat_in[r]]; hidden_out receives the residual stream after the last layer of every row). */
int om_forward_rows_ex(om_model *M, const int32_t *tokens, int m, const int32_t *slot, const int32_t *pos,
                       const uint8_t *allow, float *logits, const void *fc, const float *feat_in, float *hidden_out) {
    const om_desc *d = &M->d;
    const int D = d->d_model, H = d->n_heads, KH = d->n_kv_heads, hd = M->hd, F = d->d_ffn, V = d->vocab;
    const int DQ = H * hd, DKV = KH * hd;
    if (m <= 0) return -1;
    for (int r = 0; r < m; ++r)
        if (tokens[r] < 0 || tokens[r] >= V || slot[r] < 0 || slot[r] >= M->max_ctx || pos[r] < 0) return -1;

    float *h = (float *)malloc(sizeof(float) * (size_t)m * D);
    float *a = (float *)malloc(sizeof(float) * (size_t)m * D);
    float *q = (float *)malloc(sizeof(float) * (size_t)m * DQ);
    float *k = (float *)malloc(sizeof(float) * (size_t)m * DKV);
    float *v = (float *)malloc(sizeof(float) * (size_t)m * DKV);
    float *o = (float *)malloc(sizeof(float) * (size_t)m * DQ);
    float *y = (float *)malloc(sizeof(float) * (size_t)m * D);
    float *g = (float *)malloc(sizeof(float) * (size_t)m * F);
    float *u = (float *)malloc(sizeof(float) * (size_t)m * F);

    const void *embed = M->w[0];
    for (int r = 0; r < m; ++r)
        for (int i = 0; i < D; ++i) h[(size_t)r * D + i] = (float)wget(d, embed, (size_t)tokens[r] * D + i);
    if (fc) {
        /* h = W_fc . [embedding ; feature] */
        float *cat = (float *)malloc(sizeof(float) * (size_t)m * 2 * D);
        for (int r = 0; r < m; ++r) {
            memcpy(cat + (size_t)r * 2 * D, h + (size_t)r * D, sizeof(float) * (size_t)D);
            memcpy(cat + (size_t)r * 2 * D + D, feat_in + (size_t)r * D, sizeof(float) * (size_t)D);
        }
        matmul(d, cat, m, 2 * D, fc, D, h);
        free(cat);
    }

    for (int L = 0; L < d->n_layers; ++L) {
        const void *const *w = M->w + 1 + OM_PER_LAYER * L;
        rmsnorm(d, h, m, D, w[0], a);
        matmul(d, a, m, D, w[1], DQ, q);
        matmul(d, a, m, D, w[2], DKV, k);
        matmul(d, a, m, D, w[3], DKV, v);
        for (int r = 0; r < m; ++r) {
            for (int hh = 0; hh < H; ++hh) om_rope(q + (size_t)r * DQ + (size_t)hh * hd, hd, pos[r], d->rope_theta);
            for (int kh = 0; kh < KH; ++kh) {
                float *kv = k + (size_t)r * DKV + (size_t)kh * hd;
                om_rope(kv, hd, pos[r], d->rope_theta);
                size_t base = (((size_t)L * KH + kh) * M->max_ctx + (size_t)slot[r]) * hd;
                for (int i = 0; i < hd; ++i) {
                    M->kc[base + i] = rnd(d, kv[i]);
                    M->vc[base + i] = rnd(d, v[(size_t)r * DKV + (size_t)kh * hd + i]);
                }
            }
        }
        const double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
        for (int hh = 0; hh < H; ++hh) {
            int kh = hh / (H / KH);
            const float *Kc = M->kc + ((size_t)L * KH + kh) * (size_t)M->max_ctx * hd;
            const float *Vc = M->vc + ((size_t)L * KH + kh) * (size_t)M->max_ctx * hd;
            double *s = (double *)malloc(sizeof(double) * (size_t)M->max_ctx);
            double *acc = (double *)malloc(sizeof(double) * (size_t)hd);
            for (int r = 0; r < m; ++r) {
                const float *qv = q + (size_t)r * DQ + (size_t)hh * hd;
                const uint8_t *al = allow + (size_t)r * M->max_ctx;
                double mx = -INFINITY;
                for (int p = 0; p < M->max_ctx; ++p) {
                    if (!al[p]) continue;
                    double dot = 0.0;
                    for (int i = 0; i < hd; ++i) dot += (double)qv[i] * (double)Kc[(size_t)p * hd + i];
                    s[p] = dot * scale;
                    if (s[p] > mx) mx = s[p];
                }
                double Z = 0.0;
                for (int p = 0; p < M->max_ctx; ++p)
                    if (al[p]) { s[p] = exp(s[p] - mx); Z += s[p]; }
                for (int i = 0; i < hd; ++i) acc[i] = 0.0;
                for (int p = 0; p < M->max_ctx; ++p) {
                    if (!al[p]) continue;
                    double pw = s[p] / Z;
                    for (int i = 0; i < hd; ++i) acc[i] += pw * (double)Vc[(size_t)p * hd + i];
                }
                for (int i = 0; i < hd; ++i) o[(size_t)r * DQ + (size_t)hh * hd + i] = (float)acc[i];
            }
            free(s); free(acc);
        }
        matmul(d, o, m, DQ, w[4], D, y);
        for (size_t i = 0; i < (size_t)m * D; ++i) h[i] = (float)((double)h[i] + (double)y[i]);

        rmsnorm(d, h, m, D, w[5], a);
        matmul(d, a, m, D, w[7], F, u);
        if (d->act == 1) {
            matmul(d, a, m, D, w[6], F, g);
            for (size_t i = 0; i < (size_t)m * F; ++i) u[i] = (float)(silu((double)g[i]) * (double)u[i]);
        } else {
            for (size_t i = 0; i < (size_t)m * F; ++i) u[i] = (float)gelu_erf((double)u[i]);
        }
        matmul(d, u, m, F, w[8], D, y);
        for (size_t i = 0; i < (size_t)m * D; ++i) h[i] = (float)((double)h[i] + (double)y[i]);
    }
    if (hidden_out) memcpy(hidden_out, h, sizeof(float) * (size_t)m * D);
    if (logits) {
        rmsnorm(d, h, m, D, M->w[1 + OM_PER_LAYER * d->n_layers], a);
        matmul(d, a, m, D, M->w[2 + OM_PER_LAYER * d->n_layers], V, logits);
    }
    free(h); free(a); free(q); free(k); free(v); free(o); free(y); free(g); free(u);
    return 0;
}

/* ---------------------------------------------------------------- Philox4x32-10 */

static inline void mulhilo(uint32_t a, uint32_t b, uint32_t *hi, uint32_t *lo) {
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

/* Ten rounds of the Philox-4x32 bijection with the Weyl key schedule (Salmon et al., SC'11). */
void om_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t *out) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int r = 0; r < 10; ++r) {
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo(0xD2511F53u, c0, &hi0, &lo0);
        mulhilo(0xCD9E8D57u, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* u in [0,1): top 24 bits of output word 0 at counter (seq, round, pos, stream).
 * stream 0 = accept test, 1 = residual / bonus sample, 2 = draft sampling. */
float om_uniform(uint64_t seed, uint32_t seq, uint32_t round, uint32_t pos, uint32_t stream) {
    uint32_t o[4];
    om_philox(seed, seq, round, pos, stream, o);
    return (float)(o[0] >> 8) * (1.0f / 16777216.0f);
}

/* out[i] = om_uniform(seed, seq0 + i, round, pos, stream), i < n */
void om_uniform_batch(uint64_t seed, uint32_t seq0, int n, uint32_t round, uint32_t pos, uint32_t stream, float *out) {
    for (int i = 0; i < n; ++i) out[i] = om_uniform(seed, seq0 + (uint32_t)i, round, pos, stream);
}

/* ---------------------------------------------------------------- sampling */

/* p = softmax(logits / T), T > 0, in double. Returns nothing; out has V entries. */
void om_softmax(const float *logits, int V, float T, double *out) {
    double mx = -INFINITY;
    for (int i = 0; i < V; ++i) {
        double z = (double)logits[i] / (double)T;
        if (z > mx) mx = z;
    }
    double Z = 0.0;
    for (int i = 0; i < V; ++i) { out[i] = exp((double)logits[i] / (double)T - mx); Z += out[i]; }
    for (int i = 0; i < V; ++i) out[i] /= Z;
}

int om_argmax(const float *x, int V) {
    int best = 0;
    for (int i = 1; i < V; ++i)
        if (x[i] > x[best]) best = i; /* strict: lowest index wins ties */
    return best;
}

/* Inverse CDF over unnormalised non-negative weights in ascending index order: the smallest v
 * with sum_{w<=v} r_w > u * Z.  margin (optional) = distance from u*Z to the nearest CDF step
 * bounding the chosen cell, divided by Z (how close the draw was to picking a neighbour). */
static int inv_cdf(const double *r, int V, double u, double *margin) {
    double Z = 0.0;
    for (int i = 0; i < V; ++i) Z += r[i];
    double target = u * Z, c = 0.0;
    int pick = -1;
    double lo = 0.0, hi = 0.0;
    for (int i = 0; i < V; ++i) {
        double prev = c;
        c += r[i];
        if (c > target) { pick = i; lo = prev; hi = c; break; }
    }
    if (pick < 0) { /* only by rounding at the top end: take the last index with weight */
        for (int i = V - 1; i >= 0; --i)
            if (r[i] > 0.0) { pick = i; break; }
        if (pick < 0) pick = V - 1;
        lo = hi = Z;
    }
    if (margin) {
        double a = target - lo, b = hi - target;
        /* the lower edge at 0 and the upper edge at Z are not decision boundaries */
        if (lo <= 0.0) a = INFINITY;
        if (hi >= Z) b = INFINITY;
        double mm = a < b ? a : b;
        *margin = (Z > 0.0) ? mm / Z : INFINITY;
    }
    return pick;
}

/* Draft-token draw (Alg. 3, drafting loop): T == 0 -> argmax, else inverse CDF of softmax(logits/T). */
int om_sample(const float *logits, int V, float T, float u, double *margin) {
    if (T <= 0.0f) { if (margin) *margin = INFINITY; return om_argmax(logits, V); }
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    om_softmax(logits, V, T, p);
    int t = inv_cdf(p, V, (double)u, margin);
    free(p);
    return t;
}

/* Rows of om_sample: logits [rows][V], u [rows] -> tok [rows], margin [rows] (optional). */
void om_sample_batch(const float *logits, int rows, int V, float T, const float *u, int32_t *tok, double *margin) {
#pragma omp parallel for schedule(static)
    for (int b = 0; b < rows; ++b)
        tok[b] = om_sample(logits + (size_t)b * V, V, T, u[b], margin ? margin + b : NULL);
}

/*
 * Accept step of Alg. 3 for one sequence.
 *   P [gamma+1][V] target logits, Q [gamma][V] drafter logits, d [gamma] draft tokens,
 *   u_acc [gamma] uniforms of the accept tests, u_res the uniform of the residual / bonus draw.
 * Outputs:
 *   mask [gamma]   raw per-position test u_j < min(1, p_j(d_j)/q_j(d_j))  (every j, no prefix AND)
 *   n_acc          index of the first failed test, or gamma
 *   token          n_acc < gamma: draw from norm(max(0, p_n - q_n)); else draw from p_gamma
 *   bd [gamma]     sum_v min(p_j(v), q_j(v)) = 1 - d_TV(p_j, q_j)   (terms of Def. 2)
 *   ratio [gamma]  p_j(d_j)/q_j(d_j)  (+inf if q is 0)      - for near-tie logging
 *   margin         inverse-CDF margin of the draw that produced token - for near-tie logging
 * T == 0 (greedy): mask_j = [d_j == argmax P_j], token = argmax P_n, bd_j = mask_j, ratio_j = mask_j.
 */
void om_accept(const float *P, const float *Q, const int32_t *d, int gamma, int V, float T,
               const float *u_acc, float u_res,
               int32_t *mask, int32_t *n_acc, int32_t *token, double *bd, double *ratio, double *margin) {
    int n = gamma;
    if (T <= 0.0f) {
        for (int j = 0; j < gamma; ++j) {
            int am = om_argmax(P + (size_t)j * V, V);
            mask[j] = (d[j] == am);
            if (bd) bd[j] = (double)mask[j];
            if (ratio) ratio[j] = (double)mask[j];
            if (!mask[j] && n == gamma) n = j;
        }
        *n_acc = n;
        *token = om_argmax(P + (size_t)n * V, V);
        if (margin) *margin = INFINITY;
        return;
    }
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    for (int j = 0; j < gamma; ++j) {
        om_softmax(P + (size_t)j * V, V, T, p);
        om_softmax(Q + (size_t)j * V, V, T, q);
        double pd = p[d[j]], qd = q[d[j]];
        double rt = qd > 0.0 ? pd / qd : INFINITY;
        double thr = rt < 1.0 ? rt : 1.0;
        mask[j] = ((double)u_acc[j] < thr);
        if (ratio) ratio[j] = rt;
        if (bd) {
            double s = 0.0;
            for (int i = 0; i < V; ++i) s += p[i] < q[i] ? p[i] : q[i];
            bd[j] = s;
        }
        if (!mask[j] && n == gamma) n = j;
    }
    *n_acc = n;
    om_softmax(P + (size_t)n * V, V, T, p);
    if (n < gamma) {
        om_softmax(Q + (size_t)n * V, V, T, q);
        double Z = 0.0;
        for (int i = 0; i < V; ++i) { q[i] = p[i] > q[i] ? p[i] - q[i] : 0.0; Z += q[i]; }
        if (Z > 0.0) *token = inv_cdf(q, V, (double)u_res, margin);
        else *token = inv_cdf(p, V, (double)u_res, margin); /* p == q: rejection has probability 0 */
    } else {
        *token = inv_cdf(p, V, (double)u_res, margin);
    }
    free(p); free(q);
}

/* Rows of om_accept: row b uses P + b*(gamma+1)*V, Q + b*gamma*V, d + b*gamma, u_acc + b*gamma,
 * u_res[b]; outputs are laid out the same way. */
void om_accept_batch(const float *P, const float *Q, const int32_t *d, int rows, int gamma, int V, float T,
                     const float *u_acc, const float *u_res,
                     int32_t *mask, int32_t *n_acc, int32_t *token, double *bd, double *ratio, double *margin) {
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < rows; ++b) {
        om_accept(P + (size_t)b * (gamma + 1) * V, Q + (size_t)b * gamma * V, d + (size_t)b * gamma, gamma, V, T,
                  u_acc + (size_t)b * gamma, u_res[b],
                  mask + (size_t)b * gamma, n_acc + b, token + b,
                  bd ? bd + (size_t)b * gamma : NULL, ratio ? ratio + (size_t)b * gamma : NULL,
                  margin ? margin + b : NULL);
    }
}

/* ---------------------------------------------------------------- MetaSD-UCB (Alg. 2) */

typedef struct {
    int32_t K;
    int32_t t;       /* completed rounds */
    double beta;
    double mu[64];
    int32_t n[64];
} om_ucb;

void om_ucb_init(om_ucb *b, int K, double beta) {
    memset(b, 0, sizeof(*b));
    b->K = K;
    b->beta = beta;
}

/* Arms 0..K-1 once each in index order, then argmax of mu_i + beta*sqrt(2 ln t / n_i), lowest
 * index on ties.  scores (optional, K doubles) receives the indices (NaN during the sweep). */
int om_ucb_select(const om_ucb *b, double *scores) {
    if (b->t < b->K) {
        if (scores) for (int i = 0; i < b->K; ++i) scores[i] = NAN;
        return b->t;
    }
    int best = 0;
    double bs = -INFINITY;
    for (int i = 0; i < b->K; ++i) {
        double s = b->mu[i] + b->beta * sqrt(2.0 * log((double)b->t) / (double)b->n[i]);
        if (scores) scores[i] = s;
        if (s > bs) { bs = s; best = i; }
    }
    return best;
}

/* mu_a <- (mu_a * n_a + r) / (n_a + 1); n_a += 1; t += 1 */
void om_ucb_update(om_ucb *b, int arm, double reward) {
    b->mu[arm] = (b->mu[arm] * (double)b->n[arm] + reward) / (double)(b->n[arm] + 1);
    b->n[arm] += 1;
    b->t += 1;
}

/* Block-efficiency reward: N_acc / N_max. */
double om_reward_be(int n_acc, int gamma) { return (double)n_acc / (double)gamma; }

/* Block-divergence reward (Def. 2): mean over the block of 1 - d_TV(p_j, q_j). */
double om_reward_bd(const double *bd, int gamma) {
    double s = 0.0;
    for (int j = 0; j < gamma; ++j) s += bd[j];
    return s / (double)gamma;
}

int om_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
