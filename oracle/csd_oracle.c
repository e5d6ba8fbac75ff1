/*
 * csd_oracle.c — plain CPU oracle for the verify step of Cascade Speculative Drafting.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition the
 * HIP library is checked against.  It shares no code, header, table or helper with the
 * HIP path; only tests, the smoke check and the benchmark's CPU-baseline leg call it.
 *
 * What it follows in the paper:
 *   - review of a drafted block by one forward of the reviewing model, giving one
 *     probability vector per position                                   (Section 2)
 *   - accept / reject / resample / extra token of speculative sampling  (Section 2)
 *   - lenience in sampling and in greedy review                         (Section 3.1)
 *   - Max-Gram matching with a bigram fallback                  (Section 3.3, App. A)
 * The paper names model families only (Section 5.1); the decoders here are the two the
 * benchmark configurations spell out.  arch 0, LLaMA-style: RMSNorm, rotary position
 * embedding (half-split pairing), causal attention scaled by 1/sqrt(head_dim), SwiGLU, no
 * biases, untied LM head.  arch 1, T5-style decoder (the FLAN-T5 reviewers of Section 5.1):
 * RMS layer norm, no rotary embedding, unscaled causal self-attention with the bucketed
 * relative-position bias of the T5 paper (32 buckets, maximum distance 128, one table for all
 * layers), unmasked cross-attention over a fixed encoder output, gated tanh-GELU FFN, untied
 * LM head.
 *
 * Arithmetic: every floating-point step of the forward is fp64 on the stored values.
 * Stored values are the weights and the KV-cache rows, both in the configuration's storage
 * type: bf16 configurations keep K and V in the cache rounded to bf16 (round-to-nearest-even,
 * straight from the fp64 value), exactly as the weights are bf16; attention reads every row,
 * the block's own included, back from the cache.  fp32 configurations store the fp64 value.
 * The accept test and the residual are fp32, one rounded operation at a time, because they
 * decide integers and both sides must take that decision in the same precision; sampling is
 * exact integer arithmetic on 40-bit fixed-point weights.
 *
 * Parity pins (tests/test_oracle_*.py): library attention / norm / activation routines,
 * closed forms for degenerate weights, block-vs-incremental and cache-vs-no-cache
 * invariants, exact enumeration and chi-square of the emitted-token law, the Theorem 4.1
 * length law, Appendix A's worked Max-Gram cases and brute force on tiny alphabets.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t arch;      /* 0: LLaMA-style, 1: T5-style decoder with cross-attention */
    int32_t dtype;     /* 0: fp32 weights, 1: bf16 weights */
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t max_batch, max_seq, max_block, enc_len;
    float rms_eps, rope_theta;
} csdo_cfg;

typedef struct {
    csdo_cfg c;
    const void **w;      /* canonical order; borrowed host pointers */
    int32_t n_w;
    double *trace;       /* optional [n_layers+1][m][d] residual stream dump (one sequence) */
} csdo_model;

enum { W_EMBED = 0, W_FINAL_NORM_FROM_END = 2, W_LM_HEAD_FROM_END = 1 };
enum { L_ATTN_NORM = 0, L_WQ, L_WK, L_WV, L_WO, L_FFN_NORM, L_WGATE, L_WUP, L_WDOWN, L_COUNT };
/* arch 1: 14 tensors per layer; after the LM head comes the relative-position bias table fp32 [32][H] */
enum { T_SELF_NORM = 0, T_WQ, T_WK, T_WV, T_WO, T_CROSS_NORM, T_CQ, T_CK, T_CV, T_CO, T_FFN_NORM, T_W0, T_W1, T_WOUT, T_COUNT };
enum { REL_BUCKETS = 32, REL_MAX_DISTANCE = 128 };

int32_t csdo_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int32_t csdo_model_create(const csdo_cfg *cfg, const void *const *weights, int32_t n_w, csdo_model **out) {
    if (!cfg || !weights || !out) return -1;
    if (cfg->arch != 0 && cfg->arch != 1) return -2;
    if (cfg->arch == 0 && n_w != 3 + L_COUNT * cfg->n_layers) return -2;
    if (cfg->arch == 1 && (n_w != 4 + T_COUNT * cfg->n_layers || cfg->enc_len < 1)) return -2;
    if (cfg->head_dim % 2) return -2;
    csdo_model *m = (csdo_model *)calloc(1, sizeof *m);
    m->c = *cfg;
    m->w = (const void **)malloc(sizeof(void *) * (size_t)n_w);
    memcpy(m->w, weights, sizeof(void *) * (size_t)n_w);
    m->n_w = n_w;
    *out = m;
    return 0;
}

int32_t csdo_model_destroy(csdo_model *m) {
    if (!m) return -1;
    free(m->w);
    free(m);
    return 0;
}

void csdo_set_trace(csdo_model *m, double *trace) { m->trace = trace; }

/* cache: double K[L][B][max_seq][H*dh] followed by V of the same shape; arch 1 appends the
 * cross-attention keys and values Kc[L][B][enc_len][H*dh], Vc[...] (filled by csdo_cross_kv_init) */
static size_t self_kv_elems(const csdo_cfg *c) {
    return (size_t)2 * c->n_layers * c->max_batch * c->max_seq * c->n_heads * c->head_dim;
}
size_t csdo_kv_bytes(const csdo_model *m) {
    const csdo_cfg *c = &m->c;
    size_t n = self_kv_elems(c);
    if (c->arch == 1) n += (size_t)2 * c->n_layers * c->max_batch * c->enc_len * c->n_heads * c->head_dim;
    return n * sizeof(double);
}

static double *cross_row(const csdo_model *m, double *kv, int which, int l, int b, int pos) {
    const csdo_cfg *c = &m->c;
    size_t hd = (size_t)c->n_heads * c->head_dim;
    size_t per = (size_t)c->n_layers * c->max_batch * c->enc_len * hd;
    return kv + self_kv_elems(c) + which * per + (((size_t)l * c->max_batch + b) * c->enc_len + pos) * hd;
}

static double *kv_row(const csdo_model *m, double *kv, int which, int l, int b, int pos) {
    const csdo_cfg *c = &m->c;
    size_t hd = (size_t)c->n_heads * c->head_dim;
    size_t per = (size_t)c->n_layers * c->max_batch * c->max_seq * hd;
    return kv + which * per + (((size_t)l * c->max_batch + b) * c->max_seq + pos) * hd;
}

/* nearest bf16 (ties to even) of an fp64 value, returned as fp64 */
static double round_bf16(double x) {
    if (x == 0.0 || !isfinite(x)) return x;
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lo = u & 0xFFFF0000u;      /* neighbour towards zero (or f itself) */
    uint32_t hi = lo + 0x10000u;        /* next bf16 away from zero */
    float flo, fhi;
    memcpy(&flo, &lo, 4);
    memcpy(&fhi, &hi, 4);
    double dlo = fabs(x - (double)flo), dhi = fabs((double)fhi - x);
    if (dlo < dhi) return (double)flo;
    if (dhi < dlo) return (double)fhi;
    return ((lo >> 16) & 1u) ? (double)fhi : (double)flo;
}

static double to_cache(const csdo_model *m, double x) { return m->c.dtype == 1 ? round_bf16(x) : x; }

/* copy rows in/out of the cache (fp32 at the interface; rounded to the cache type on write) */
int32_t csdo_kv_write(const csdo_model *m, double *kv, int32_t l, int32_t b, int32_t pos0, int32_t n,
                      const float *K, const float *V) {
    size_t hd = (size_t)m->c.n_heads * m->c.head_dim;
    if (pos0 < 0 || pos0 + n > m->c.max_seq) return -2;
    for (int i = 0; i < n; i++)
        for (size_t x = 0; x < hd; x++) {
            kv_row(m, kv, 0, l, b, pos0 + i)[x] = to_cache(m, K[i * hd + x]);
            kv_row(m, kv, 1, l, b, pos0 + i)[x] = to_cache(m, V[i * hd + x]);
        }
    return 0;
}

int32_t csdo_kv_read(const csdo_model *m, double *kv, int32_t l, int32_t b, int32_t pos0, int32_t n,
                     double *K, double *V) {
    size_t hd = (size_t)m->c.n_heads * m->c.head_dim;
    if (pos0 < 0 || pos0 + n > m->c.max_seq) return -2;
    for (int i = 0; i < n; i++)
        for (size_t x = 0; x < hd; x++) {
            K[i * hd + x] = kv_row(m, kv, 0, l, b, pos0 + i)[x];
            V[i * hd + x] = kv_row(m, kv, 1, l, b, pos0 + i)[x];
        }
    return 0;
}

static inline double wval(const void *w, int dtype, size_t i) {
    if (dtype == 0) return (double)((const float *)w)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)w)[i] << 16;   /* bf16 = top half of an fp32 */
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* out[r][n] = sum_k in[r][k] * W[k][n], W row-major [K][N]; threads own column ranges */
static void matmul(const double *in, int m, int K, const void *W, int dtype, int N, double *out) {
#pragma omp parallel
    {
#ifdef _OPENMP
        int nt = omp_get_num_threads(), id = omp_get_thread_num();
#else
        int nt = 1, id = 0;
#endif
        int n_lo = (int)((int64_t)N * id / nt), n_hi = (int)((int64_t)N * (id + 1) / nt);
        for (int r = 0; r < m; r++)
            for (int n = n_lo; n < n_hi; n++) out[(size_t)r * N + n] = 0.0;
        for (int k = 0; k < K; k++)
            for (int r = 0; r < m; r++) {
                double x = in[(size_t)r * K + k];
                double *o = out + (size_t)r * N;
                if (dtype == 0) {
                    const float *wr = (const float *)W + (size_t)k * N;
                    for (int n = n_lo; n < n_hi; n++) o[n] += x * (double)wr[n];
                } else {
                    const uint16_t *wr = (const uint16_t *)W + (size_t)k * N;
                    for (int n = n_lo; n < n_hi; n++) {
                        uint32_t bits = (uint32_t)wr[n] << 16;
                        float f;
                        memcpy(&f, &bits, 4);
                        o[n] += x * (double)f;
                    }
                }
            }
    }
}

/* y = x * g / sqrt(mean(x^2) + eps) */
void csdo_rmsnorm(const double *x, const float *g, int d, double eps, double *y) {
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; i++) y[i] = x[i] * r * (double)g[i];
}

/* rotary embedding on one head vector, half-split pairing (j, j + dh/2), angle pos * theta^(-2j/dh) */
void csdo_rope(double *x, int dh, int pos, double theta) {
    int half = dh / 2;
    for (int j = 0; j < half; j++) {
        double ang = (double)pos * pow(theta, -2.0 * j / dh);
        double c = cos(ang), s = sin(ang);
        double a = x[j], b = x[j + half];
        x[j] = a * c - b * s;
        x[j + half] = a * s + b * c;
    }
}

static double silu(double z) { return z / (1.0 + exp(-z)); }

/* tanh form of GELU: 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) */
static double gelu_tanh(double z) {
    return 0.5 * z * (1.0 + tanh(0.79788456080286535588 * (z + 0.044715 * z * z * z)));
}

/*
 * Bucket of the T5 relative-position bias for a decoder (a query only looks back):
 * distance n = query position - key position >= 0.  The first half of the buckets holds the
 * distances 0 .. 15 exactly; the second half spaces the distances 16 .. 127 logarithmically,
 * bucket 16 + floor(16 * ln(n/16) / ln(128/16)); anything farther shares the last bucket.
 */
int32_t csdo_rel_bucket(int32_t n) {
    const int half = REL_BUCKETS / 2;
    if (n < 0) n = 0;
    if (n < half) return n;
    int32_t b = half + (int32_t)(log((double)n / half) / log((double)REL_MAX_DISTANCE / half) * (REL_BUCKETS - half));
    return b < REL_BUCKETS - 1 ? b : REL_BUCKETS - 1;
}

/* arch 1, once per prompt: project the encoder output [B][enc_len][d] (fp32 at the interface) to the
 * cross-attention keys and values of every layer and store them in the cache's storage type */
int32_t csdo_cross_kv_init(const csdo_model *mod, double *kv, const float *enc_out, int32_t B) {
    const csdo_cfg *c = &mod->c;
    if (c->arch != 1 || B < 1 || B > c->max_batch) return -2;
    const int d = c->d_model, hd = c->n_heads * c->head_dim, E = c->enc_len;
    double *x = (double *)malloc(sizeof(double) * (size_t)E * d);
    double *y = (double *)malloc(sizeof(double) * (size_t)E * hd);
    for (int b = 0; b < B; b++) {
        for (size_t i = 0; i < (size_t)E * d; i++) x[i] = (double)enc_out[(size_t)b * E * d + i];
        for (int l = 0; l < c->n_layers; l++) {
            const void **lw = mod->w + 1 + (size_t)l * T_COUNT;
            for (int which = 0; which < 2; which++) {
                matmul(x, E, d, lw[which == 0 ? T_CK : T_CV], c->dtype, hd, y);
                for (int j = 0; j < E; j++)
                    for (int z = 0; z < hd; z++) cross_row(mod, kv, which, l, b, j)[z] = to_cache(mod, y[(size_t)j * hd + z]);
            }
        }
    }
    free(x); free(y);
    return 0;
}

/* numerically plain softmax with max subtraction */
void csdo_softmax(const double *logits, int n, double inv_temperature, double *p) {
    double mx = -INFINITY;
    for (int i = 0; i < n; i++) if (logits[i] * inv_temperature > mx) mx = logits[i] * inv_temperature;
    double s = 0.0;
    for (int i = 0; i < n; i++) { p[i] = exp(logits[i] * inv_temperature - mx); s += p[i]; }
    for (int i = 0; i < n; i++) p[i] /= s;
}

/* softmax(scores) . V over rows 0 .. nk-1 given by an accessor; scores already complete in sc[] */
static void weighted_sum(const double *sc_exp, double z, int nk, int dh, int hh, const csdo_model *mod, double *kv, int cross,
                         int l, int b, double *oi) {
    for (int x = 0; x < dh; x++) oi[x] = 0.0;
    for (int j = 0; j < nk; j++) {
        const double *vj = (cross ? cross_row(mod, kv, 1, l, b, j) : kv_row(mod, kv, 1, l, b, j)) + hh * dh;
        double p = sc_exp[j] / z;
        for (int x = 0; x < dh; x++) oi[x] += p * vj[x];
    }
}

/*
 * arch 1: T5-style decoder layer stack over the block rows of one sequence.
 *   h += SelfAttn(norm(h))   causal over cache rows 0 .. t+i, scores q.k + bias[bucket(i_pos - j_pos)][head], no scaling
 *   h += CrossAttn(norm(h))  over all enc_len projected encoder rows, no mask, no bias, no scaling
 *   h += (gelu_tanh(norm(h) W0) * (norm(h) W1)) Wout
 */
static int32_t verify_block_t5(csdo_model *mod, double *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B,
                               int32_t m, double temperature, double *logits, double *probs) {
    const csdo_cfg *c = &mod->c;
    const int d = c->d_model, H = c->n_heads, dh = c->head_dim, F = c->d_ffn, V = c->vocab, L = c->n_layers, E = c->enc_len;
    const int hd = H * dh, dt = c->dtype;
    const void **w = mod->w;
    const float *rel = (const float *)w[mod->n_w - 1];          /* [REL_BUCKETS][H] */
    const int wide = d > hd ? d : hd;
    double *h = (double *)malloc(sizeof(double) * (size_t)m * d);
    double *a = (double *)malloc(sizeof(double) * (size_t)m * wide);
    double *q = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *kk = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *vv = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *o = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *t1 = (double *)malloc(sizeof(double) * (size_t)m * (F > d ? F : d));
    double *t2 = (double *)malloc(sizeof(double) * (size_t)m * (F > d ? F : d));
    const int scn = c->max_seq > E ? c->max_seq : E;
    double *sc = (double *)malloc(sizeof(double) * (size_t)scn);
    for (int b = 0; b < B; b++) {
        const int t = cache_len[b];
        for (int i = 0; i < m; i++)
            for (int x = 0; x < d; x++)
                h[(size_t)i * d + x] = wval(w[W_EMBED], dt, (size_t)tokens[b * m + i] * d + x);
        if (mod->trace && b == 0) memcpy(mod->trace, h, sizeof(double) * (size_t)m * d);
        for (int l = 0; l < L; l++) {
            const void **lw = w + 1 + (size_t)l * T_COUNT;
            /* self-attention */
            for (int i = 0; i < m; i++)
                csdo_rmsnorm(h + (size_t)i * d, (const float *)lw[T_SELF_NORM], d, c->rms_eps, a + (size_t)i * d);
            matmul(a, m, d, lw[T_WQ], dt, hd, q);
            matmul(a, m, d, lw[T_WK], dt, hd, kk);
            matmul(a, m, d, lw[T_WV], dt, hd, vv);
            for (int i = 0; i < m; i++)
                for (int x = 0; x < hd; x++) {
                    kv_row(mod, kv, 0, l, b, t + i)[x] = to_cache(mod, kk[(size_t)i * hd + x]);
                    kv_row(mod, kv, 1, l, b, t + i)[x] = to_cache(mod, vv[(size_t)i * hd + x]);
                }
            for (int i = 0; i < m; i++)
                for (int hh = 0; hh < H; hh++) {
                    const double *qi = q + (size_t)i * hd + hh * dh;
                    const int nk = t + i + 1;
                    double mx = -INFINITY;
                    for (int j = 0; j < nk; j++) {
                        const double *kj = kv_row(mod, kv, 0, l, b, j) + hh * dh;
                        double s = 0.0;
                        for (int x = 0; x < dh; x++) s += qi[x] * kj[x];
                        sc[j] = s + (double)rel[(size_t)csdo_rel_bucket(t + i - j) * H + hh];
                        if (sc[j] > mx) mx = sc[j];
                    }
                    double z = 0.0;
                    for (int j = 0; j < nk; j++) { sc[j] = exp(sc[j] - mx); z += sc[j]; }
                    weighted_sum(sc, z, nk, dh, hh, mod, kv, 0, l, b, o + (size_t)i * hd + hh * dh);
                }
            matmul(o, m, hd, lw[T_WO], dt, d, t1);
            for (size_t x = 0; x < (size_t)m * d; x++) h[x] += t1[x];
            /* cross-attention over the projected encoder rows */
            for (int i = 0; i < m; i++)
                csdo_rmsnorm(h + (size_t)i * d, (const float *)lw[T_CROSS_NORM], d, c->rms_eps, a + (size_t)i * d);
            matmul(a, m, d, lw[T_CQ], dt, hd, q);
            for (int i = 0; i < m; i++)
                for (int hh = 0; hh < H; hh++) {
                    const double *qi = q + (size_t)i * hd + hh * dh;
                    double mx = -INFINITY;
                    for (int j = 0; j < E; j++) {
                        const double *kj = cross_row(mod, kv, 0, l, b, j) + hh * dh;
                        double s = 0.0;
                        for (int x = 0; x < dh; x++) s += qi[x] * kj[x];
                        sc[j] = s;
                        if (s > mx) mx = s;
                    }
                    double z = 0.0;
                    for (int j = 0; j < E; j++) { sc[j] = exp(sc[j] - mx); z += sc[j]; }
                    weighted_sum(sc, z, E, dh, hh, mod, kv, 1, l, b, o + (size_t)i * hd + hh * dh);
                }
            matmul(o, m, hd, lw[T_CO], dt, d, t1);
            for (size_t x = 0; x < (size_t)m * d; x++) h[x] += t1[x];
            /* gated tanh-GELU feed-forward */
            for (int i = 0; i < m; i++)
                csdo_rmsnorm(h + (size_t)i * d, (const float *)lw[T_FFN_NORM], d, c->rms_eps, a + (size_t)i * d);
            matmul(a, m, d, lw[T_W0], dt, F, t1);
            matmul(a, m, d, lw[T_W1], dt, F, t2);
            for (size_t x = 0; x < (size_t)m * F; x++) t1[x] = gelu_tanh(t1[x]) * t2[x];
            matmul(t1, m, F, lw[T_WOUT], dt, d, t2);
            for (size_t x = 0; x < (size_t)m * d; x++) h[x] += t2[x];
            if (mod->trace && b == 0)
                memcpy(mod->trace + (size_t)(l + 1) * m * d, h, sizeof(double) * (size_t)m * d);
        }
        for (int i = 0; i < m; i++)
            csdo_rmsnorm(h + (size_t)i * d, (const float *)w[mod->n_w - 3], d, c->rms_eps, a + (size_t)i * d);
        double *lg = logits + (size_t)b * m * V;
        matmul(a, m, d, w[mod->n_w - 2], dt, V, lg);
        if (probs)
            for (int i = 0; i < m; i++)
                csdo_softmax(lg + (size_t)i * V, V, 1.0 / temperature, probs + ((size_t)b * m + i) * V);
    }
    free(h); free(a); free(q); free(kk); free(vv); free(o); free(t1); free(t2); free(sc);
    return 0;
}

/*
 * Review forward (Section 2: the reviewing model runs once over the whole drafted block and
 * yields a distribution per position).  Row i of sequence b sits at absolute position
 * cache_len[b] + i, attends cache rows 0 .. cache_len[b] + i, and its K/V are written to
 * the cache at that position.  logits: [B][m][V] fp64; probs: optional softmax(logits / T).
 */
static int32_t verify_rows(csdo_model *mod, double *kv, const int32_t *tokens, const int32_t *parent,
                           const int32_t *cache_len, int32_t B, int32_t m, double temperature, double *logits,
                           double *probs) {
    const csdo_cfg *c = &mod->c;
    if (B < 1 || B > c->max_batch || m < 1) return -2;
    if (parent && c->arch != 0) return -2;
    const int d = c->d_model, H = c->n_heads, dh = c->head_dim, F = c->d_ffn, V = c->vocab, L = c->n_layers;
    const int hd = H * dh, dt = c->dtype;
    for (int b = 0; b < B; b++) {
        if (cache_len[b] < 0 || cache_len[b] + m > c->max_seq) return -2;
        for (int i = 0; i < m; i++)
            if (tokens[b * m + i] < 0 || tokens[b * m + i] >= V) return -2;
    }
    if (probs && !(temperature > 0.0)) return -2;
    if (c->arch == 1) return verify_block_t5(mod, kv, tokens, cache_len, B, m, temperature, logits, probs);
    double *h = (double *)malloc(sizeof(double) * (size_t)m * d);
    double *a = (double *)malloc(sizeof(double) * (size_t)m * (d > hd ? d : hd));
    double *q = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *kk = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *vv = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *o = (double *)malloc(sizeof(double) * (size_t)m * hd);
    double *t1 = (double *)malloc(sizeof(double) * (size_t)m * (F > d ? F : d));
    double *t2 = (double *)malloc(sizeof(double) * (size_t)m * F);
    double *sc = (double *)malloc(sizeof(double) * (size_t)c->max_seq);
    int *depth = (int *)malloc(sizeof(int) * (size_t)m);
    unsigned char *sees = (unsigned char *)malloc((size_t)m * m);   /* sees[i*m + j]: block row j is row i or above it */
    const void **w = mod->w;
    for (int b = 0; b < B; b++) {
        const int t = cache_len[b];
        /* a plain block is the chain 0 <- 1 <- 2 ...; a tree block names every row's parent (row 0 is the root) */
        for (int i = 0; i < m; i++) {
            const int par = parent ? parent[b * m + i] : i - 1;
            if ((i == 0 && par != -1) || (i > 0 && (par < 0 || par >= i))) {
                free(h); free(a); free(q); free(kk); free(vv); free(o); free(t1); free(t2); free(sc); free(depth); free(sees);
                return -2;
            }
            depth[i] = i == 0 ? 0 : depth[par] + 1;
            for (int j = 0; j < m; j++) sees[i * m + j] = (j == i) || (i > 0 && j <= par && sees[par * m + j]);
        }
        for (int i = 0; i < m; i++)
            for (int x = 0; x < d; x++)
                h[(size_t)i * d + x] = wval(w[W_EMBED], dt, (size_t)tokens[b * m + i] * d + x);
        if (mod->trace && b == 0) memcpy(mod->trace, h, sizeof(double) * (size_t)m * d);
        for (int l = 0; l < L; l++) {
            const void **lw = w + 1 + (size_t)l * L_COUNT;
            for (int i = 0; i < m; i++)
                csdo_rmsnorm(h + (size_t)i * d, (const float *)lw[L_ATTN_NORM], d, c->rms_eps, a + (size_t)i * d);
            matmul(a, m, d, lw[L_WQ], dt, hd, q);
            matmul(a, m, d, lw[L_WK], dt, hd, kk);
            matmul(a, m, d, lw[L_WV], dt, hd, vv);
            for (int i = 0; i < m; i++) {
                for (int hh = 0; hh < H; hh++) {
                    /* the position of a row is how far it is from the root, not where it is stored */
                    csdo_rope(q + (size_t)i * hd + hh * dh, dh, t + depth[i], c->rope_theta);
                    csdo_rope(kk + (size_t)i * hd + hh * dh, dh, t + depth[i], c->rope_theta);
                }
                for (int x = 0; x < hd; x++) {      /* the cache holds the configuration's storage type */
                    kv_row(mod, kv, 0, l, b, t + i)[x] = to_cache(mod, kk[(size_t)i * hd + x]);
                    kv_row(mod, kv, 1, l, b, t + i)[x] = to_cache(mod, vv[(size_t)i * hd + x]);
                }
            }
            /* causal attention: row i sees the cached rows 0 .. t-1 and, of the block (stored at t .. t+i), itself
             * and the rows above it -- in a plain block that is every row 0 .. t+i */
            for (int i = 0; i < m; i++)
                for (int hh = 0; hh < H; hh++) {
                    const double *qi = q + (size_t)i * hd + hh * dh;
                    int nk = t + i + 1;
                    double mx = -INFINITY;
                    for (int j = 0; j < nk; j++) {
                        if (j >= t && !sees[i * m + (j - t)]) continue;
                        const double *kj = kv_row(mod, kv, 0, l, b, j) + hh * dh;
                        double s = 0.0;
                        for (int x = 0; x < dh; x++) s += qi[x] * kj[x];
                        sc[j] = s / sqrt((double)dh);
                        if (sc[j] > mx) mx = sc[j];
                    }
                    double z = 0.0;
                    for (int j = 0; j < nk; j++) {
                        if (j >= t && !sees[i * m + (j - t)]) { sc[j] = 0.0; continue; }
                        sc[j] = exp(sc[j] - mx);
                        z += sc[j];
                    }
                    double *oi = o + (size_t)i * hd + hh * dh;
                    for (int x = 0; x < dh; x++) oi[x] = 0.0;
                    for (int j = 0; j < nk; j++) {
                        if (j >= t && !sees[i * m + (j - t)]) continue;
                        const double *vj = kv_row(mod, kv, 1, l, b, j) + hh * dh;
                        double p = sc[j] / z;
                        for (int x = 0; x < dh; x++) oi[x] += p * vj[x];
                    }
                }
            matmul(o, m, hd, lw[L_WO], dt, d, t1);
            for (size_t x = 0; x < (size_t)m * d; x++) h[x] += t1[x];
            for (int i = 0; i < m; i++)
                csdo_rmsnorm(h + (size_t)i * d, (const float *)lw[L_FFN_NORM], d, c->rms_eps, a + (size_t)i * d);
            matmul(a, m, d, lw[L_WGATE], dt, F, t1);
            matmul(a, m, d, lw[L_WUP], dt, F, t2);
            for (size_t x = 0; x < (size_t)m * F; x++) t1[x] = silu(t1[x]) * t2[x];
            matmul(t1, m, F, lw[L_WDOWN], dt, d, t2);
            for (size_t x = 0; x < (size_t)m * d; x++) h[x] += t2[x];
            if (mod->trace && b == 0)
                memcpy(mod->trace + (size_t)(l + 1) * m * d, h, sizeof(double) * (size_t)m * d);
        }
        for (int i = 0; i < m; i++)
            csdo_rmsnorm(h + (size_t)i * d, (const float *)w[mod->n_w - 2], d, c->rms_eps, a + (size_t)i * d);
        double *lg = logits + (size_t)b * m * V;
        matmul(a, m, d, w[mod->n_w - 1], dt, V, lg);
        if (probs) {
            if (!(temperature > 0.0)) return -2;
            for (int i = 0; i < m; i++)
                csdo_softmax(lg + (size_t)i * V, V, 1.0 / temperature, probs + ((size_t)b * m + i) * V);
        }
    }
    free(h); free(a); free(q); free(kk); free(vv); free(o); free(t1); free(t2); free(sc); free(depth); free(sees);
    return 0;
}

int32_t csdo_verify_block(csdo_model *mod, double *kv, const int32_t *tokens, const int32_t *cache_len,
                          int32_t B, int32_t m, double temperature, double *logits, double *probs) {
    return verify_rows(mod, kv, tokens, NULL, cache_len, B, m, temperature, logits, probs);
}

/*
 * Review forward over a tree of drafts (Section 5.1 combines the cascade with tree attention; Appendix B gives
 * the lead node eight children).  Row 0 is the last kept token; parent[b][i] < i names the row that row i
 * continues (parent[b][0] = -1).  A row's position is cache_len + its distance from row 0, it attends the cached
 * rows, the rows above it in the tree and itself, and its K/V are stored at cache row cache_len + i: every
 * root-to-node path sees exactly what a plain block holding that path would see.  arch 0 only.
 */
int32_t csdo_verify_tree(csdo_model *mod, double *kv, const int32_t *tokens, const int32_t *parent,
                         const int32_t *cache_len, int32_t B, int32_t m, double temperature, double *logits,
                         double *probs) {
    if (!parent) return -2;
    return verify_rows(mod, kv, tokens, parent, cache_len, B, m, temperature, logits, probs);
}

/*
 * After a tree review kept the rows path[0 .. n) (a chain below row 0): move their K/V to cache rows
 * cache_len + 1 .. cache_len + n, where a plain block would have put them, so that the cache again holds one
 * sequence.  path is increasing and path[j] >= j + 1, so moving in order overwrites nothing still needed.
 */
int32_t csdo_tree_commit(const csdo_model *mod, double *kv, int32_t b, int32_t cache_len, const int32_t *path, int32_t n) {
    const csdo_cfg *c = &mod->c;
    const int hd = c->n_heads * c->head_dim;
    if (b < 0 || b >= c->max_batch || cache_len < 0 || n < 0) return -2;
    for (int j = 0; j < n; j++)
        if (path[j] < j + 1 || (j > 0 && path[j] <= path[j - 1]) || cache_len + path[j] >= c->max_seq) return -2;
    for (int l = 0; l < c->n_layers; l++)
        for (int j = 0; j < n; j++)
            for (int which = 0; which < 2; which++)
                memmove(kv_row(mod, kv, which, l, b, cache_len + 1 + j), kv_row(mod, kv, which, l, b, cache_len + path[j]),
                        sizeof(double) * (size_t)hd);
    return 0;
}

/* ------------------------------------------------------------------ statistical draft */

/*
 * Bigram table fit: next[a] = the successor b with the highest count of (a, b) in the
 * stream; among equal counts the pair whose last occurrence is latest wins; tokens that
 * never appear before another token keep the caller's pre-filled default.
 * (Section 3.3 uses a bigram model as the fallback of Max-Gram; Section 5.2 says it has
 * one parameter per vocabulary entry.)
 */
int32_t csdo_bigram_fit(const int32_t *s, int32_t n, int32_t vocab, int32_t *next_table) {
    if (n < 0 || vocab < 1) return -2;
    int32_t *best = (int32_t *)calloc((size_t)vocab, sizeof(int32_t));
    for (int i = 0; i + 1 < n; i++) {
        int32_t a = s[i], b = s[i + 1];
        if (a < 0 || a >= vocab || b < 0 || b >= vocab) { free(best); return -2; }
        int32_t cnt = 0;
        for (int j = 0; j + 1 < n; j++) cnt += (s[j] == a && s[j + 1] == b);
        if (cnt >= best[a]) { best[a] = cnt; next_table[a] = b; }   /* ascending i: later wins ties */
    }
    free(best);
    return 0;
}

/*
 * Max-Gram draft (Section 3.3, Appendix A).  For a decoder-only model the haystack is the
 * sequence itself.  A candidate match ends at e in [0, len-2] (the trivial match of the
 * sequence with itself, ending at len-1, is excluded so a continuation exists) and has
 * length mlen(e) = max r with s[e-r+1 .. e] == s[len-r .. len-1] (optionally capped).
 * The left-most e of maximal length is taken, as the appendix takes the first set index.
 * The k tokens after it are read from the sequence extended by the draft itself, so the
 * result always has k tokens.  No match at all: chain the bigram table from the last token.
 */
int32_t csdo_bigram_draft(const int32_t *ctx, const int32_t *ctx_len, int32_t B, int32_t ctx_stride,
                          const int32_t *next_table, int32_t vocab, int32_t k, int32_t max_match,
                          int32_t *out_tokens, int32_t *out_match_len) {
    if (B < 0 || k < 0 || vocab < 1) return -2;
    for (int b = 0; b < B; b++) {
        const int32_t *s = ctx + (size_t)b * ctx_stride;
        int len = ctx_len[b];
        if (len < 1 || len > ctx_stride) return -2;
        int best_len = 0, best_e = -1;
        for (int e = 0; e <= len - 2; e++) {
            int r = 0;
            while (r <= e && (max_match <= 0 || r < max_match) && s[e - r] == s[len - 1 - r]) r++;
            if (r > best_len) { best_len = r; best_e = e; }       /* strict: keeps the left-most */
        }
        int32_t *out = out_tokens + (size_t)b * k;
        if (best_len == 0) {
            int32_t cur = s[len - 1];
            for (int j = 0; j < k; j++) {
                if (cur < 0 || cur >= vocab) return -2;
                cur = next_table[cur];
                out[j] = cur;
            }
        } else {
            for (int j = 0; j < k; j++) {
                int idx = best_e + 1 + j;                          /* index into s ++ out */
                out[j] = idx < len ? s[idx] : out[idx - len];
            }
        }
        if (out_match_len) out_match_len[b] = best_len;
    }
    return 0;
}

/* Max-Gram with a separate haystack (Appendix A's signature; Section 3.3).  The longest suffix of the needle
 * that ends at a haystack position, the left-most such position; the continuation is copied while the
 * haystack lasts (n_copied tokens: Appendix A's return value), the rest chains the bigram table. */
int32_t csdo_maxgram_draft(const int32_t *hay, const int32_t *hay_len, int32_t hay_stride, const int32_t *needle,
                           const int32_t *needle_len, int32_t needle_stride, int32_t B, const int32_t *next_table,
                           int32_t vocab, int32_t k, int32_t max_match, int32_t *out_tokens, int32_t *out_match_len,
                           int32_t *out_n_copied) {
    if (B < 0 || k < 0 || vocab < 1) return -2;
    for (int b = 0; b < B; b++) {
        const int32_t *h = hay + (size_t)b * hay_stride, *s = needle + (size_t)b * needle_stride;
        const int hl = hay_len[b], len = needle_len[b];
        if (len < 1 || len > needle_stride || hl < 0 || hl > hay_stride) return -2;
        int best_len = 0, best_e = -1;
        for (int e = 0; e < hl; e++) {
            int r = 0;
            while (r <= e && r < len && (max_match <= 0 || r < max_match) && h[e - r] == s[len - 1 - r]) r++;
            if (r > best_len) { best_len = r; best_e = e; }       /* strict: keeps the left-most */
        }
        int32_t *out = out_tokens + (size_t)b * k;
        int n_copied = 0;
        if (best_len > 0)
            for (int j = 0; j < k && best_e + 1 + j < hl; j++) out[n_copied++] = h[best_e + 1 + j];
        int32_t cur = n_copied > 0 ? out[n_copied - 1] : s[len - 1];
        for (int j = n_copied; j < k; j++) {
            if (cur < 0 || cur >= vocab) return -2;
            cur = next_table[cur];
            out[j] = cur;
        }
        if (out_match_len) out_match_len[b] = best_len;
        if (out_n_copied) out_n_copied[b] = n_copied;
    }
    return 0;
}

/* ------------------------------------------------------------------ accept / resample */

static int32_t sample_fixed_point(const float *r, int V, float u) {
    /* weights w_v = floor(r_v * 2^40): exact (r_v is an fp32 scaled by a power of two) */
    unsigned __int128 Z = 0;
    for (int v = 0; v < V; v++) Z += (uint64_t)ldexp((double)r[v], 40);
    if (Z == 0) return -1;
    uint64_t u24 = (uint64_t)ldexp((double)u, 24);               /* floor(u * 2^24) */
    uint64_t T = (uint64_t)(((unsigned __int128)u24 * Z) >> 24);
    uint64_t cum = 0;
    for (int v = 0; v < V; v++) {
        cum += (uint64_t)ldexp((double)r[v], 40);
        if (cum > T) return v;
    }
    return V - 1;   /* unreachable: T < Z */
}

static int32_t argmax_first(const float *x, int V) {
    int best = 0;
    for (int v = 1; v < V; v++) if (x[v] > x[best]) best = v;     /* ties: smallest index */
    return best;
}

/*
 * Speculative-sampling review of k drafted tokens per sequence (Section 2), with lenience
 * l >= 1 (Section 3.1).  p: [B][k+1][V] reviewer distributions (row i scores draft i, the
 * last row is the extra token); q: [B][k][V] draft distributions, or NULL / q_onehot[i]!=0
 * when the draft at that position was deterministic (Max-Gram / bigram), i.e. one-hot.
 *   sampling (mode 0): accept draft i  iff  fl32(u_i * q_i(x_i)) < fl32(l * p_i(x_i));
 *     at the first rejection resample from norm(max(0, l*p_i - q_i)) and stop; with no
 *     rejection sample the extra token from p_{k+1}.  An all-zero residual falls back to p_i.
 *   greedy (mode 1): p may hold logits; accept iff x_i is the arg-max of row i (ties: the
 *     smallest id) or, when l > 1 and p holds probabilities, q_i(x_i) <= fl32(l * p_i(x_i));
 *     the emitted token is the arg-max of the row after the accepted ones.
 */
int32_t csdo_accept(const float *p, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                    const float *u_acc, const float *u_samp, int32_t B, int32_t k, int32_t V,
                    float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token) {
    if (B < 0 || k < 0 || V < 1 || !(lenience >= 1.0f) || (mode != 0 && mode != 1)) return -2;
    float *r = (float *)malloc(sizeof(float) * (size_t)V);
    for (int b = 0; b < B; b++) {
        const float *pb = p + (size_t)b * (k + 1) * V;
        const float *qb = q ? q + (size_t)b * k * V : NULL;
        int n = 0;
        for (; n < k; n++) {
            int32_t x = draft[b * k + n];
            if (x < 0 || x >= V) { free(r); return -2; }
            const float *pi = pb + (size_t)n * V;
            int dense = qb && !(q_onehot && q_onehot[n]);
            float qx = dense ? qb[(size_t)n * V + x] : 1.0f;
            int ok;
            if (mode == 1) {
                ok = (argmax_first(pi, V) == x);
                if (!ok && lenience > 1.0f) {
                    volatile float rhs = lenience * pi[x];
                    ok = (qx <= rhs);
                }
            } else {
                volatile float lhs = u_acc[b * k + n] * qx;
                volatile float rhs = lenience * pi[x];
                ok = (lhs < rhs);
            }
            if (!ok) break;
        }
        n_accepted[b] = n;
        const float *pn = pb + (size_t)n * V;
        if (mode == 1) {
            next_token[b] = argmax_first(pn, V);
            continue;
        }
        int32_t tok = -1;
        if (n < k) {                                   /* rejected at draft n: residual */
            int32_t x = draft[b * k + n];
            int dense = qb && !(q_onehot && q_onehot[n]);
            for (int v = 0; v < V; v++) {
                volatile float lp = lenience * pn[v];
                float qv = dense ? qb[(size_t)n * V + v] : (v == x ? 1.0f : 0.0f);
                volatile float df = lp - qv;
                r[v] = df > 0.0f ? df : 0.0f;
            }
            tok = sample_fixed_point(r, V, u_samp[b]);
        }
        if (tok < 0) tok = sample_fixed_point(pn, V, u_samp[b]);
        if (tok < 0) { free(r); return -3; }           /* p row sums to zero: not a distribution */
        next_token[b] = tok;
    }
    free(r);
    return 0;
}

/*
 * Review of a tree of deterministic candidates (the children of a node are tokens the draft side proposes for the
 * position after it; Section 5.1, Appendix B).  Walk down from row 0: take the reviewer's own token for the position
 * after the current row -- drawn from its distribution with the walk's next uniform (the same fixed-point inverse
 * CDF as the review of a chain), or its arg-max in greedy mode -- and if a child of the current row carries that
 * token, keep the child and go on from it; otherwise that token is what the review emits and the walk ends.
 * Every emitted token is the reviewer's own draw given what was kept before it, so the output law is the
 * reviewer's whatever the tree holds.  p [B][m][V] (probabilities; logits will do in greedy mode), tokens,
 * parent [B][m], u [B][m] (the j-th draw of sequence b uses u[b][j]).  path [B][m] receives the kept rows.
 * Among children with the same token the lowest row wins.
 */
int32_t csdo_tree_accept(const float *p, const int32_t *tokens, const int32_t *parent, const float *u, int32_t B,
                         int32_t m, int32_t V, int32_t mode, int32_t *n_accepted, int32_t *path, int32_t *next_token) {
    if (B < 0 || m < 1 || V < 1 || (mode != 0 && mode != 1)) return -2;
    for (int b = 0; b < B; b++) {
        const int32_t *par = parent + (size_t)b * m, *tok = tokens + (size_t)b * m;
        if (par[0] != -1) return -2;
        for (int i = 1; i < m; i++)
            if (par[i] < 0 || par[i] >= i) return -2;
        int node = 0, n = 0;
        for (;;) {
            const float *row = p + ((size_t)b * m + node) * V;
            const int32_t t = mode == 1 ? argmax_first(row, V) : sample_fixed_point(row, V, u[(size_t)b * m + n]);
            if (t < 0) return -3;                      /* the row sums to zero: not a distribution */
            int child = -1;
            for (int j = node + 1; j < m && child < 0; j++)
                if (par[j] == node && tok[j] == t) child = j;
            if (child < 0) { next_token[b] = t; break; }
            path[(size_t)b * m + n++] = child;
            node = child;
        }
        n_accepted[b] = n;
    }
    return 0;
}

/* fp32 softmax rows from fp64 logits, for feeding csdo_accept in end-to-end checks */
void csdo_probs_f32(const double *logits, int32_t rows, int32_t V, double temperature, float *p) {
    double *tmp = (double *)malloc(sizeof(double) * (size_t)V);
    for (int i = 0; i < rows; i++) {
        csdo_softmax(logits + (size_t)i * V, V, 1.0 / temperature, tmp);
        for (int v = 0; v < V; v++) p[(size_t)i * V + v] = (float)tmp[v];
    }
    free(tmp);
}
