/*
 * CPU oracle for one decode step of a Qwen2/Qwen3-style decoder.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, sequential definition of
 * what the GPU megakernel must compute; it shares no code, header, table or
 * constant with the HIP path and must never be linked into, imported by or
 * called from the product library.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may use it.
 *
 * What it follows.  The paper (Sec. 3, Phase I; Sec. 4.2.3) names the fused
 * computation -- "Transformer Decoder and LM Head": RMSNorm, QKV projection,
 * K/V cache, attention, SwiGLU with Up/Gate paths -- but does not define the
 * arithmetic; the megakernel only reorders and fuses it (Sec. 1, Sec. 2.1:
 * fusion removes launches and HBM round trips, results are unchanged).  The
 * oracle is therefore the public Qwen2/Qwen3 decoder definition, written out
 * op by op with no tiling, fusion or reordering.
 *
 * Precision.  Weights and the KV cache are bf16 (converted exactly to fp32 on
 * read, rounded to nearest-even on append).  Every activation is stored as
 * fp32; every sum (dot products, mean of squares, softmax denominator,
 * weighted sum of V) is accumulated in fp64 and rounded once to fp32.  RoPE
 * angles, cos and sin are computed in fp64 and rounded to fp32 before use.
 *
 * Layouts.  All matrices are row-major [out][in] bf16.  KV cache:
 * [layer][2 (0=K,1=V)][max_batch][n_kv_heads][max_context][head_dim] bf16.
 *
 * W4A16 (paper Sec. 4.3.2 "MegaKernel Quantization Implementation", Sec. 5.1:
 * the measured models are GPTQ-W4A16).  The paper fixes neither the code
 * layout nor the zero point; the reading taken here is symmetric group
 * quantisation of the seven decoder projections (embedding and LM head stay
 * bf16, as in GPTQ checkpoints): w[r][k] = (q[r][k] - 8) * s[r][k / G] with
 * q an unsigned 4-bit code, s a bf16 scale, G the group size along K.  Codes
 * are packed two per byte, row-major [out][in/2]: byte j of a row holds
 * k = 2j in its low nibble and k = 2j + 1 in its high nibble.  Scales are
 * row-major [out][in/G].  Activations stay fp32 ("A16" or wider).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_config {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab;
    int32_t qkv_bias, qk_norm, tie_embeddings;
    float rope_theta, rms_eps;
    int32_t max_batch, max_context;
} orc_config;

/* Host pointers.  Per-layer entries are arrays of n_layers pointers.  A NULL
 * bias / qk-norm array is allowed when the corresponding flag is 0; lm_head
 * may be NULL when tie_embeddings is 1 (embed is used). */
typedef struct orc_weights {
    const uint16_t *embed;      /* [vocab][hidden] */
    const uint16_t *lm_head;    /* [vocab][hidden] */
    const uint16_t *final_norm; /* [hidden] */
    const uint16_t *const *attn_norm; /* [hidden] */
    const uint16_t *const *wq;  /* [nq*d][hidden] */
    const uint16_t *const *wk;  /* [nkv*d][hidden] */
    const uint16_t *const *wv;  /* [nkv*d][hidden] */
    const uint16_t *const *bq;  /* [nq*d] */
    const uint16_t *const *bk;  /* [nkv*d] */
    const uint16_t *const *bv;  /* [nkv*d] */
    const uint16_t *const *q_norm; /* [d] */
    const uint16_t *const *k_norm; /* [d] */
    const uint16_t *const *wo;  /* [hidden][nq*d] */
    const uint16_t *const *mlp_norm; /* [hidden] */
    const uint16_t *const *w_gate; /* [inter][hidden] */
    const uint16_t *const *w_up;   /* [inter][hidden] */
    const uint16_t *const *w_down; /* [hidden][inter] */
} orc_weights;

/* W4A16 form of the seven decoder projections (host pointers, per-layer
 * arrays).  The matching bf16 matrix pointers of orc_weights are ignored. */
typedef struct orc_w4 {
    int32_t group;              /* group size along K; divides hidden, nq*d and intermediate */
    const uint8_t *const *wq, *const *wk, *const *wv, *const *wo, *const *w_gate, *const *w_up, *const *w_down;
    const uint16_t *const *sq, *const *sk, *const *sv, *const *so, *const *s_gate, *const *s_up, *const *s_down;
} orc_w4;

/* ---- bf16 <-> fp32 ------------------------------------------------------ */

/* bf16 is the upper 16 bits of an IEEE fp32: widening is exact. */
float orc_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Round to nearest, ties to even; denormals kept; NaN stays a quiet NaN. */
uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* ---- elementary operators ---------------------------------------------- */

/* y_i = x_i * (1/sqrt(mean_j x_j^2 + eps)) * g_i */
void orc_rmsnorm(const float *x, const uint16_t *g, int n, float eps, float *y)
{
    double ss = 0.0;
    for (int j = 0; j < n; ++j) ss += (double)x[j] * (double)x[j];
    double inv = 1.0 / sqrt(ss / (double)n + (double)eps);
    for (int i = 0; i < n; ++i)
        y[i] = (float)((double)x[i] * inv * (double)orc_bf16_to_f32(g[i]));
}

/* y = W x (+ bias); W is [n_out][n_in] row-major bf16. */
void orc_gemv(const uint16_t *W, int n_out, int n_in, const float *x,
              const uint16_t *bias, float *y)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < n_out; ++r) {
        const uint16_t *row = W + (size_t)r * (size_t)n_in;
        double acc = 0.0;
        for (int k = 0; k < n_in; ++k) acc += (double)orc_bf16_to_f32(row[k]) * (double)x[k];
        if (bias) acc += (double)orc_bf16_to_f32(bias[r]);
        y[r] = (float)acc;
    }
}

/* y = W x (+ bias) for a W4 matrix: codes [n_out][n_in/2] bytes, scales
 * [n_out][n_in/group] bf16, w = (q - 8) * s (see the file header). */
void orc_gemv_w4(const uint8_t *codes, const uint16_t *scales, int n_out, int n_in, int group,
                 const float *x, const uint16_t *bias, float *y)
{
    const int n_groups = n_in / group;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < n_out; ++r) {
        const uint8_t *row = codes + (size_t)r * (size_t)(n_in / 2);
        double acc = 0.0;
        for (int k = 0; k < n_in; ++k) {
            const int q = (k & 1) ? (row[k >> 1] >> 4) : (row[k >> 1] & 15);
            const double s = (double)orc_bf16_to_f32(scales[(size_t)r * n_groups + k / group]);
            acc += (double)(q - 8) * s * (double)x[k];
        }
        if (bias) acc += (double)orc_bf16_to_f32(bias[r]);
        y[r] = (float)acc;
    }
}

/* Rotary embedding of one head vector u[d] at position pos, half-split
 * pairing (i, i + d/2), angle pos * theta^(-2i/d). */
void orc_rope(float *u, int d, int pos, float theta)
{
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double phi = (double)pos * pow((double)theta, -2.0 * (double)i / (double)d);
        float c = (float)cos(phi), s = (float)sin(phi);
        double a = u[i], b = u[i + half];
        u[i] = (float)(a * (double)c - b * (double)s);
        u[i + half] = (float)(b * (double)c + a * (double)s);
    }
}

float orc_silu(float z)
{
    return (float)((double)z / (1.0 + exp(-(double)z)));
}

/* Numerically stable softmax over s[0..n). */
void orc_softmax(const float *s, int n, float *w)
{
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) if ((double)s[j] > m) m = s[j];
    double den = 0.0;
    for (int j = 0; j < n; ++j) den += exp((double)s[j] - m);
    for (int j = 0; j < n; ++j) w[j] = (float)(exp((double)s[j] - m) / den);
}

/* One query head against T cached positions.  K and V point at position 0 of
 * the head's cache rows ([t][d], contiguous).  o[d] = softmax(qK^T/sqrt(d)) V. */
void orc_attend(const float *q, const uint16_t *K, const uint16_t *V, int T, int d, float *o)
{
    float *s = (float *)malloc(sizeof(float) * (size_t)T);
    float *w = (float *)malloc(sizeof(float) * (size_t)T);
    double scale = 1.0 / sqrt((double)d);
    for (int t = 0; t < T; ++t) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
            acc += (double)q[i] * (double)orc_bf16_to_f32(K[(size_t)t * d + i]);
        s[t] = (float)(acc * scale);
    }
    orc_softmax(s, T, w);
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int t = 0; t < T; ++t)
            acc += (double)w[t] * (double)orc_bf16_to_f32(V[(size_t)t * d + i]);
        o[i] = (float)acc;
    }
    free(s);
    free(w);
}

/* Lowest index wins on ties. */
int32_t orc_argmax(const float *v, int n)
{
    int32_t best = 0;
    for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

/* ---- the decoder step --------------------------------------------------- */

static size_t kv_index(const orc_config *c, int layer, int which, int b, int g, int t)
{
    size_t i = (size_t)layer;
    i = i * 2 + (size_t)which;
    i = i * (size_t)c->max_batch + (size_t)b;
    i = i * (size_t)c->n_kv_heads + (size_t)g;
    i = i * (size_t)c->max_context + (size_t)t;
    return i * (size_t)c->head_dim;
}

/* Decode one token per sequence.  For sequence b: embeds tokens[b], appends
 * its K/V at slot positions[b] of kv_cache, attends over slots 0..positions[b],
 * and writes logits[b][vocab] unless logits is NULL (then the LM head is
 * skipped -- used for prefill).  Returns 0, or -1 on a bad argument. */
int orc_decode_step_q(const orc_config *c, const orc_weights *w, const orc_w4 *q4, int batch,
                      const int32_t *tokens, const int32_t *positions,
                      uint16_t *kv_cache, float *logits);

int orc_decode_step(const orc_config *c, const orc_weights *w, int batch,
                    const int32_t *tokens, const int32_t *positions,
                    uint16_t *kv_cache, float *logits)
{
    return orc_decode_step_q(c, w, NULL, batch, tokens, positions, kv_cache, logits);
}

/* One projection of the decoder: the bf16 matrix, or its W4 form when q4 is given. */
static void proj(const uint16_t *W, const uint8_t *codes, const uint16_t *scales, int group,
                 int n_out, int n_in, const float *x, const uint16_t *bias, float *y)
{
    if (codes) orc_gemv_w4(codes, scales, n_out, n_in, group, x, bias, y);
    else orc_gemv(W, n_out, n_in, x, bias, y);
}

/* The same step with the seven decoder projections taken from q4 (W4A16) when q4 != NULL. */
int orc_decode_step_q(const orc_config *c, const orc_weights *w, const orc_w4 *q4, int batch,
                      const int32_t *tokens, const int32_t *positions,
                      uint16_t *kv_cache, float *logits)
{
    const int H = c->hidden, nq = c->n_q_heads, nkv = c->n_kv_heads, d = c->head_dim;
    const int I = c->intermediate, V = c->vocab;
    const int qd = nq * d, kvd = nkv * d, group = nq / nkv;
    if (batch < 1 || batch > c->max_batch || nq % nkv != 0 || (d & 1)) return -1;
    const int G = q4 ? q4->group : 0;
    if (q4 && (G < 2 || (G & 1) || H % G || qd % G || I % G)) return -1;
#define Q4(field) (q4 ? q4->field[l] : NULL)
    for (int b = 0; b < batch; ++b)
        if (tokens[b] < 0 || tokens[b] >= V || positions[b] < 0 || positions[b] >= c->max_context)
            return -1;

    float *x = (float *)malloc(sizeof(float) * (size_t)H);
    float *h = (float *)malloc(sizeof(float) * (size_t)H);
    float *q = (float *)malloc(sizeof(float) * (size_t)qd);
    float *k = (float *)malloc(sizeof(float) * (size_t)kvd);
    float *v = (float *)malloc(sizeof(float) * (size_t)kvd);
    float *o = (float *)malloc(sizeof(float) * (size_t)qd);
    float *t1 = (float *)malloc(sizeof(float) * (size_t)(I > H ? I : H));
    float *t2 = (float *)malloc(sizeof(float) * (size_t)I);

    for (int b = 0; b < batch; ++b) {
        const int p = positions[b];
        for (int i = 0; i < H; ++i)
            x[i] = orc_bf16_to_f32(w->embed[(size_t)tokens[b] * H + i]);

        for (int l = 0; l < c->n_layers; ++l) {
            /* attention block */
            orc_rmsnorm(x, w->attn_norm[l], H, c->rms_eps, h);
            proj(q4 ? NULL : w->wq[l], Q4(wq), Q4(sq), G, qd, H, h, c->qkv_bias ? w->bq[l] : NULL, q);
            proj(q4 ? NULL : w->wk[l], Q4(wk), Q4(sk), G, kvd, H, h, c->qkv_bias ? w->bk[l] : NULL, k);
            proj(q4 ? NULL : w->wv[l], Q4(wv), Q4(sv), G, kvd, H, h, c->qkv_bias ? w->bv[l] : NULL, v);
            if (c->qk_norm) {
                for (int hh = 0; hh < nq; ++hh)
                    orc_rmsnorm(q + hh * d, w->q_norm[l], d, c->rms_eps, q + hh * d);
                for (int g = 0; g < nkv; ++g)
                    orc_rmsnorm(k + g * d, w->k_norm[l], d, c->rms_eps, k + g * d);
            }
            for (int hh = 0; hh < nq; ++hh) orc_rope(q + hh * d, d, p, c->rope_theta);
            for (int g = 0; g < nkv; ++g) orc_rope(k + g * d, d, p, c->rope_theta);
            for (int g = 0; g < nkv; ++g) {
                uint16_t *kc = kv_cache + kv_index(c, l, 0, b, g, p);
                uint16_t *vc = kv_cache + kv_index(c, l, 1, b, g, p);
                for (int i = 0; i < d; ++i) {
                    kc[i] = orc_f32_to_bf16(k[g * d + i]);
                    vc[i] = orc_f32_to_bf16(v[g * d + i]);
                }
            }
            for (int hh = 0; hh < nq; ++hh) {
                int g = hh / group;
                orc_attend(q + hh * d, kv_cache + kv_index(c, l, 0, b, g, 0),
                           kv_cache + kv_index(c, l, 1, b, g, 0), p + 1, d, o + hh * d);
            }
            proj(q4 ? NULL : w->wo[l], Q4(wo), Q4(so), G, H, qd, o, NULL, t1);
            for (int i = 0; i < H; ++i) x[i] += t1[i];

            /* SwiGLU MLP block */
            orc_rmsnorm(x, w->mlp_norm[l], H, c->rms_eps, h);
            proj(q4 ? NULL : w->w_gate[l], Q4(w_gate), Q4(s_gate), G, I, H, h, NULL, t1);
            proj(q4 ? NULL : w->w_up[l], Q4(w_up), Q4(s_up), G, I, H, h, NULL, t2);
            for (int i = 0; i < I; ++i) t1[i] = orc_silu(t1[i]) * t2[i];
            proj(q4 ? NULL : w->w_down[l], Q4(w_down), Q4(s_down), G, H, I, t1, NULL, h);
            for (int i = 0; i < H; ++i) x[i] += h[i];
        }

        if (logits) {
            const uint16_t *head = (c->tie_embeddings || !w->lm_head) ? w->embed : w->lm_head;
            orc_rmsnorm(x, w->final_norm, H, c->rms_eps, h);
            orc_gemv(head, V, H, h, NULL, logits + (size_t)b * V);
        }
    }
#undef Q4
    free(x); free(h); free(q); free(k); free(v); free(o); free(t1); free(t2);
    return 0;
}

/* ---- shared-memory page budget (paper Sec. 4.1.1, Eq. 1 and Eq. 2) ------- */

/* Eq. 1: pages left after each pipeline stage's fixed overhead (instruction
 * buffer + semaphores + scratch) is taken out of the on-chip memory; floor. */
int64_t orc_pages_available(int64_t smem_max, int64_t n_stage, int64_t instr_buf,
                            int64_t semaphores, int64_t scratch, int64_t page_size)
{
    int64_t left = smem_max - n_stage * (instr_buf + semaphores + scratch);
    if (left < 0) return 0;
    return left / page_size;
}

/* Eq. 2: pipeline depth that the pages not pinned by weights, scales and
 * activations can sustain; floor. */
int64_t orc_pipeline_stages(int64_t pages_total, int64_t pages_weight, int64_t pages_scale,
                            int64_t pages_act, int64_t pages_per_stage)
{
    int64_t left = pages_total - pages_weight - pages_scale - pages_act;
    if (left < 0) return 0;
    return left / pages_per_stage;
}
