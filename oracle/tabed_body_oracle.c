/*
 * Draft-model body in front of the LM head -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT (see tabed_oracle.c).  One decode step of the
 * shared draft model M_q for every row of the batch of drafting methods
 * (Sec. 5.1, "Ensemble learning via Batched Inference": all m drafting methods
 * share the parameters of M_q and run as one batch; Sec. 4.1, "Target and Draft
 * Models": LLaMA-style draft models of 68M / 160M parameters).  The paper gives
 * the model family, not its equations; the LLaMA decoder block is public and is
 * written out here: token embedding, then per layer
 *     h   = RMSNorm(x) * g_attn
 *     q,k,v = h Wqkv^T, rotary position embedding on q and k at the row's position
 *     (pairs (i, i + head_dim/2) rotated by pos * theta^(-2i/head_dim)), k and v
 *     appended to the row's cache
 *     a   = softmax(q K^T / sqrt(head_dim)) V  over the row's own cache (causal)
 *     x  += a Wo^T
 *     h2  = RMSNorm(x) * g_mlp
 *     x  += (silu(h2 Wgate^T) * (h2 Wup^T)) Wdown^T
 * and H = RMSNorm(x) * g_final, the hidden state the LM head consumes.
 *
 * reading (precision, none is stated): weights, the caches and every activation
 * that feeds a matrix product are stored in bf16; the residual stream x and the
 * products' results are fp32.  The oracle computes in fp64 and rounds at
 * exactly those storage points (round to nearest even), so that the HIP path,
 * which accumulates in fp32, differs from it only by accumulation noise and the
 * occasional flip of a bf16 rounding.
 *
 * Pin: tests compare this file with an independent fp64 implementation made of
 * library operators (embedding, linear, rms_norm, scaled_dot_product_attention,
 * silu, complex multiplication for the rotation).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_f64(uint16_t b)
{
    uint32_t bits = (uint32_t)b << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static uint16_t f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t bias = ((u >> 16) & 1u) + 0x7FFFu;
    return (uint16_t)((u + bias) >> 16);
}

/* value as stored in bf16 */
static double round_bf16(double x) { return bf16_to_f64(f32_to_bf16((float)x)); }
/* value as stored in fp32 */
static double round_f32(double x) { return (double)(float)x; }

/* y[N] = W[N,K] (bf16) . x[K], fp64 accumulation in k order, result stored as fp32 */
static void linear(const uint16_t* W, int N, int K, const double* x, double* y)
{
    for (int o = 0; o < N; ++o) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k) acc += x[k] * bf16_to_f64(W[(size_t)o * K + k]);
        y[o] = round_f32(acc);
    }
}

/* h = x / sqrt(mean(x^2) + eps) * g, stored as bf16 */
static void rmsnorm_bf16(const double* x, const float* g, int d, double eps, double* h)
{
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    double inv = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; ++i) h[i] = round_bf16(x[i] * inv * (double)g[i]);
}

/*
 * One decode step for M rows.
 *   tokens [M]                 token fed to every row
 *   ctx_len [M]                tokens already in the row's cache = position of this token
 *   embed [V,d] bf16; per layer l: g_attn[l] [d] fp32, wqkv[l] [3d,d], wo[l] [d,d], g_mlp[l] [d] fp32,
 *   wgu[l] [2*d_ff,d] (gate rows, then up rows), wdown[l] [d,d_ff]; g_final [d] fp32
 *   kcache, vcache [layers,M,max_ctx,d] bf16, entry ctx_len[r] of every row is written
 *   H [M,d] bf16 out
 * ctx_len is not changed.
 */
void oracle_body_step(int layers, int d, int heads, int d_ff, int V, int max_ctx, double rope_theta, double rms_eps,
                      int M, const int32_t* tokens, const int32_t* ctx_len,
                      const uint16_t* embed, const float* const* g_attn, const uint16_t* const* wqkv,
                      const uint16_t* const* wo, const float* const* g_mlp, const uint16_t* const* wgu,
                      const uint16_t* const* wdown, const float* g_final,
                      uint16_t* kcache, uint16_t* vcache, uint16_t* H)
{
    const int hd = d / heads;
    (void)V;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < M; ++r) {
        double* x = (double*)malloc((size_t)d * sizeof(double));
        double* h = (double*)malloc((size_t)d * sizeof(double));
        double* qkv = (double*)malloc((size_t)3 * d * sizeof(double));
        double* att = (double*)malloc((size_t)d * sizeof(double));
        double* proj = (double*)malloc((size_t)d * sizeof(double));
        double* gu = (double*)malloc((size_t)2 * d_ff * sizeof(double));
        double* act = (double*)malloc((size_t)d_ff * sizeof(double));
        double* sc = (double*)malloc((size_t)max_ctx * sizeof(double));
        const int pos = ctx_len[r];
        for (int i = 0; i < d; ++i) x[i] = bf16_to_f64(embed[(size_t)tokens[r] * d + i]);
        for (int l = 0; l < layers; ++l) {
            rmsnorm_bf16(x, g_attn[l], d, rms_eps, h);
            linear(wqkv[l], 3 * d, d, h, qkv);
            uint16_t* Kr = kcache + (((size_t)l * M + r) * max_ctx) * d;
            uint16_t* Vr = vcache + (((size_t)l * M + r) * max_ctx) * d;
            for (int hh = 0; hh < heads; ++hh) {
                double* q = qkv + hh * hd;
                double* k = qkv + d + hh * hd;
                double* v = qkv + 2 * d + hh * hd;
                for (int i = 0; i < hd / 2; ++i) {      /* rotary embedding: pairs (i, i + hd/2) */
                    double ang = (double)pos * pow(rope_theta, -2.0 * i / hd);
                    double c = cos(ang), s = sin(ang);
                    double q0 = q[i], q1 = q[i + hd / 2], k0 = k[i], k1 = k[i + hd / 2];
                    q[i] = round_f32(q0 * c - q1 * s); q[i + hd / 2] = round_f32(q1 * c + q0 * s);
                    k[i] = k0 * c - k1 * s;            k[i + hd / 2] = k1 * c + k0 * s;
                }
                for (int i = 0; i < hd; ++i) {
                    Kr[(size_t)pos * d + hh * hd + i] = f32_to_bf16((float)k[i]);
                    Vr[(size_t)pos * d + hh * hd + i] = f32_to_bf16((float)v[i]);
                }
                double mx = -INFINITY;
                for (int t = 0; t <= pos; ++t) {
                    double acc = 0.0;
                    for (int i = 0; i < hd; ++i) acc += q[i] * bf16_to_f64(Kr[(size_t)t * d + hh * hd + i]);
                    sc[t] = acc / sqrt((double)hd);
                    if (sc[t] > mx) mx = sc[t];
                }
                double Z = 0.0;
                for (int t = 0; t <= pos; ++t) { sc[t] = exp(sc[t] - mx); Z += sc[t]; }
                for (int i = 0; i < hd; ++i) {
                    double acc = 0.0;
                    for (int t = 0; t <= pos; ++t) acc += sc[t] * bf16_to_f64(Vr[(size_t)t * d + hh * hd + i]);
                    att[hh * hd + i] = round_bf16(acc / Z);
                }
            }
            linear(wo[l], d, d, att, proj);
            for (int i = 0; i < d; ++i) x[i] = round_f32(x[i] + proj[i]);
            rmsnorm_bf16(x, g_mlp[l], d, rms_eps, h);
            linear(wgu[l], 2 * d_ff, d, h, gu);
            for (int f = 0; f < d_ff; ++f) act[f] = round_bf16(gu[f] / (1.0 + exp(-gu[f])) * gu[d_ff + f]);
            linear(wdown[l], d, d_ff, act, proj);
            for (int i = 0; i < d; ++i) x[i] = round_f32(x[i] + proj[i]);
        }
        rmsnorm_bf16(x, g_final, d, rms_eps, h);
        for (int i = 0; i < d; ++i) H[(size_t)r * d + i] = f32_to_bf16((float)h[i]);
        free(x); free(h); free(qkv); free(att); free(proj); free(gu); free(act); free(sc);
    }
}
