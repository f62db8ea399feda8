// Draft-model body in front of the LM head (Sec. 5.1 "Ensemble learning via Batched Inference", Sec. 4.1 "Target and
// Draft Models"): one decode step of a LLaMA-style decoder for the n*B rows of the batch of drafting methods, each
// with its own key / value cache.  At 64 rows every projection streams its weights once (a few megabytes) and is
// launch-bound: they run through the LM head's W-streaming kernels (any [rows,K] x [N,K]^T -> fp32).  What is new
// here are the small kernels between them: embedding + RMSNorm, rotary embedding + cache append + attention over
// the row's own cache, residual + RMSNorm, SwiGLU.  Storage points: bf16 for weights, caches and everything that
// feeds a projection; fp32 for the residual stream and the projections' results.
#include <hip/hip_bf16.h>

#include "device_utils.h"
#include "internal.h"

namespace tabed {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4b;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {            // round to nearest even
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + (((u >> 16) & 1u) + 0x7FFFu)) >> 16);
}

__device__ __forceinline__ float block_sum_f32(float v, float* lds4) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    const float r = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
    __syncthreads();
    return r;
}

// ---------------------------------------------------------------- embedding + first RMSNorm
__global__ __launch_bounds__(kBlock) void k_body_embed_norm(int d, int V, float eps, const int32_t* __restrict__ token_src,
                                                            int token_stride, int rows_per_token,
                                                            const uint16_t* __restrict__ embed, const float* __restrict__ g,
                                                            float* __restrict__ x, uint16_t* __restrict__ hb) {
    __shared__ float s_red[kWavesPerBlock];
    const int r = blockIdx.x;
    int tok = token_src[(size_t)(r / rows_per_token) * token_stride];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    const uint16_t* e = embed + (size_t)tok * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += kBlock) {
        const float v = bf16_bits_to_f32(e[i]);
        x[(size_t)r * d + i] = v;
        ss += v * v;
    }
    const float inv = 1.f / sqrtf(block_sum_f32(ss, s_red) / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += kBlock)
        hb[(size_t)r * d + i] = f32_to_bf16_bits(bf16_bits_to_f32(e[i]) * inv * g[i]);
}

// ---------------------------------------------------------------- residual + RMSNorm (+ position advance at the end of a step)
__global__ __launch_bounds__(kBlock) void k_body_add_norm(int d, int ldy, float eps, float* __restrict__ x,
                                                          const float* __restrict__ y, const float* __restrict__ g,
                                                          uint16_t* __restrict__ out, int32_t* ctx_len_advance) {
    __shared__ float s_red[kWavesPerBlock];
    const int r = blockIdx.x;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += kBlock) {
        const float v = x[(size_t)r * d + i] + y[(size_t)r * ldy + i];
        x[(size_t)r * d + i] = v;
        ss += v * v;
    }
    const float inv = 1.f / sqrtf(block_sum_f32(ss, s_red) / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += kBlock)
        out[(size_t)r * d + i] = f32_to_bf16_bits(x[(size_t)r * d + i] * inv * g[i]);
    if (ctx_len_advance != nullptr && threadIdx.x == 0) ctx_len_advance[r] += 1;
}

// ---------------------------------------------------------------- SwiGLU: silu(gate) * up
__global__ __launch_bounds__(kBlock) void k_body_silu_mul(int rows, int d_ff, const float* __restrict__ gu,
                                                          uint16_t* __restrict__ act) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= (size_t)rows * d_ff) return;
    const size_t r = i / d_ff, f = i % d_ff;
    const float gte = gu[r * 2 * d_ff + f], up = gu[r * 2 * d_ff + d_ff + f];
    act[i] = f32_to_bf16_bits(gte / (1.f + __expf(-gte)) * up);
}

// ---------------------------------------------------------------- rotary embedding + cache append + attention
// Grid (head, row), four waves.  The rotation is done in fp64 (a position times a tiny frequency loses digits in
// fp32).  Scores: one thread per cached key (its head slice is hd contiguous bf16); softmax over the workgroup;
// values: lanes over the head's dimensions, waves over the keys, so a wave reads a key's slice coalesced.  The
// token's own key and value (just written to the cache) are taken from LDS.
__global__ __launch_bounds__(kBlock) void k_body_rope_attn(int d, int hd, int max_ctx, double theta, int rows,
                                                           const float* __restrict__ qkv /* [rows,3d] */,
                                                           const int32_t* __restrict__ ctx_len,
                                                           uint16_t* __restrict__ kc /* [rows,max_ctx,d] of this layer */,
                                                           uint16_t* __restrict__ vc, uint16_t* __restrict__ att /* [rows,d] */) {
    extern __shared__ __attribute__((aligned(16))) float s_sc[];          // [max_ctx] scores, then probabilities
    __shared__ float s_q[128], s_knew[128], s_vnew[128], s_part[kWavesPerBlock][128];
    __shared__ float s_redf[kWavesPerBlock];
    const int hh = blockIdx.x, r = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int pos = ctx_len[r];
    pos = pos < 0 ? 0 : (pos >= max_ctx ? max_ctx - 1 : pos);            // the host checks the range; never write outside
    const float* q = qkv + (size_t)r * 3 * d + hh * hd;
    const float* k = q + d;
    const float* v = q + 2 * d;
    uint16_t* Kr = kc + (size_t)r * max_ctx * d + hh * hd;                // row t of this head: Kr + t * d
    uint16_t* Vr = vc + (size_t)r * max_ctx * d + hh * hd;
    if (tid < hd / 2) {
        const int i = tid;
        const double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
        double sn, cs;
        sincos(ang, &sn, &cs);
        const double q0 = (double)q[i], q1 = (double)q[i + hd / 2], k0 = (double)k[i], k1 = (double)k[i + hd / 2];
        s_q[i] = (float)(q0 * cs - q1 * sn);
        s_q[i + hd / 2] = (float)(q1 * cs + q0 * sn);
        const uint16_t kb0 = f32_to_bf16_bits((float)(k0 * cs - k1 * sn)), kb1 = f32_to_bf16_bits((float)(k1 * cs + k0 * sn));
        Kr[(size_t)pos * d + i] = kb0;
        Kr[(size_t)pos * d + i + hd / 2] = kb1;
        s_knew[i] = bf16_bits_to_f32(kb0);
        s_knew[i + hd / 2] = bf16_bits_to_f32(kb1);
    }
    if (tid >= 128 && tid < 128 + hd) {
        const int i = tid - 128;
        const uint16_t vb = f32_to_bf16_bits(v[i]);
        Vr[(size_t)pos * d + i] = vb;
        s_vnew[i] = bf16_bits_to_f32(vb);
    }
    __syncthreads();
    const float scale = 1.f / sqrtf((float)hd);
    float mx = -INFINITY;
    for (int t = tid; t <= pos; t += kBlock) {
        float acc = 0.f;
        if (t == pos) {
            for (int i = 0; i < hd; ++i) acc += s_q[i] * s_knew[i];
        } else {
            const u32x4b* row = reinterpret_cast<const u32x4b*>(Kr + (size_t)t * d);
            for (int c8 = 0; c8 < hd / 8; ++c8) {
                const u32x4b w4 = row[c8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t w = w4[e];
                    acc += s_q[c8 * 8 + 2 * e] * __builtin_bit_cast(float, w << 16);
                    acc += s_q[c8 * 8 + 2 * e + 1] * __builtin_bit_cast(float, w & 0xffff0000u);
                }
            }
        }
        acc *= scale;
        s_sc[t] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = block_max(mx, s_redf);
    float zs = 0.f;
    for (int t = tid; t <= pos; t += kBlock) {
        const float p = __expf(s_sc[t] - mx);
        s_sc[t] = p;
        zs += p;
    }
    const float Z = block_sum_f32(zs, s_redf);                            // its barriers also publish s_sc
    for (int dd = lane; dd < hd; dd += kWave) {
        float acc = 0.f;
        for (int t = wave; t < pos; t += kWavesPerBlock) acc += s_sc[t] * bf16_bits_to_f32(Vr[(size_t)t * d + dd]);
        if (wave == (pos % kWavesPerBlock)) acc += s_sc[pos] * s_vnew[dd];
        s_part[wave][dd] = acc;
    }
    __syncthreads();
    if (tid < hd) {
        const float o = ((s_part[0][tid] + s_part[1][tid]) + (s_part[2][tid] + s_part[3][tid])) / Z;
        att[(size_t)r * d + hh * hd + tid] = f32_to_bf16_bits(o);
    }
}

__global__ void k_body_fill_ones(float* p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 1.f;
}

__global__ void k_body_rollback(int rows, int rows_per_seq, int gamma, const int32_t* __restrict__ ctx_base,
                                const int32_t* __restrict__ accept_len, int32_t* __restrict__ ctx_len) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const int k = accept_len[r / rows_per_seq];
    const int kept = (k + 1 < gamma) ? k + 1 : gamma;
    ctx_len[r] = ctx_base[r] + (kept < 0 ? 0 : kept);
}

// ---------------------------------------------------------------- host side
static size_t al256(size_t x) { return (x + 255) / 256 * 256; }

// A projection [rows,K] x [N,K]^T runs as an LM head with vocabulary N, hidden size K, one draft and `rows` sequences.
static tabed_cfg gemm_cfg(int rows, int K, int N) {
    tabed_cfg c{};
    c.V = N; c.d = K; c.n = 1; c.B = rows; c.gamma = 1; c.h = 1; c.w_dtype = 1; c.distance = 0; c.policy = 0;
    c.tau_w = 1.f; c.eps = 1e-6f; c.seed = 0;
    return c;
}

BodyLayout body_layout(const tabed_body_cfg& c, int rows) {
    BodyLayout L;
    const int wide = (3 * c.d > 2 * c.d_ff) ? 3 * c.d : 2 * c.d_ff;
    const int act = (c.d > c.d_ff) ? c.d : c.d_ff;
    size_t off = 0;
    L.off_ones = off; off = al256(off + sizeof(float) * (size_t)rows);
    L.off_x = off;    off = al256(off + sizeof(float) * (size_t)rows * c.d);
    L.off_y = off;    off = al256(off + sizeof(float) * (size_t)rows * wide);
    L.off_hb = off;   off = al256(off + sizeof(uint16_t) * (size_t)rows * act);
    size_t g = 0;
    for (int N : {3 * c.d, c.d, 2 * c.d_ff}) {
        const size_t t = ws_layout(gemm_cfg(rows, c.d, N)).total;
        g = t > g ? t : g;
    }
    const size_t t = ws_layout(gemm_cfg(rows, c.d_ff, c.d)).total;
    g = t > g ? t : g;
    L.off_gemm = off; off = al256(off + g);
    L.total = off;
    return L;
}

int validate_body_cfg(const tabed_body_cfg* c, int rows) {
    if (c == nullptr) return TABED_ENULL;
    if (c->layers < 1 || c->layers > TABED_BODY_MAX_LAYERS) return TABED_ERANGE;
    if (c->d < 8 || c->d % 8 != 0 || c->d_ff < 8 || c->d_ff % 8 != 0 || c->heads < 1 || c->d % c->heads != 0) return TABED_EINVAL;
    const int hd = c->d / c->heads;
    if (hd < 8 || hd > 128 || hd % 8 != 0) return TABED_EINVAL;
    if (c->V < 1 || c->max_ctx < 1 || c->max_ctx > 8192) return TABED_ERANGE;
    if (!(c->rope_theta > 0.f) || !(c->rms_eps > 0.f)) return TABED_EINVAL;
    if (rows < 1 || rows > 65535) return TABED_ERANGE;
    if (3 * c->d > 262144 || 2 * c->d_ff > 262144) return TABED_ERANGE;
    return TABED_OK;
}

hipError_t launch_body_init(const tabed_body_cfg& c, int rows, char* ws, hipStream_t s) {
    const BodyLayout L = body_layout(c, rows);
    launch(nullptr, k_body_fill_ones, dim3((rows + 255) / 256), dim3(256), 0, s, reinterpret_cast<float*>(ws + L.off_ones), rows);
    return hipGetLastError();
}

static hipError_t projection(int rows, int K, int N, char* gemm_ws, const void* W, const uint16_t* in, const float* ones,
                             float* out, hipStream_t s) {
    const tabed_cfg gc = gemm_cfg(rows, K, N);
    return launch_lmhead(gc, ws_layout(gc), gemm_ws, W, in, ones, out, s, TABED_K_BODY);
}

hipError_t launch_body_step(const tabed_body_cfg& c, const tabed_body_weights& w, char* ws, int rows,
                            const int32_t* token_src, int token_stride, int rows_per_token, int32_t* ctx_len,
                            uint16_t* kcache, uint16_t* vcache, uint16_t* H, hipStream_t s) {
    const BodyLayout L = body_layout(c, rows);
    const float* ones = reinterpret_cast<const float*>(ws + L.off_ones);
    float* x = reinterpret_cast<float*>(ws + L.off_x);
    float* y = reinterpret_cast<float*>(ws + L.off_y);
    uint16_t* hb = reinterpret_cast<uint16_t*>(ws + L.off_hb);
    char* gws = ws + L.off_gemm;
    const int d = c.d, hd = c.d / c.heads;
    hipError_t e;
#define TABED_BODY_CHECK()            \
    e = hipGetLastError();            \
    if (e != hipSuccess) return e
    {
        ProfScope prof(TABED_K_BODY, s);
        launch(&prof, k_body_embed_norm, dim3(rows), dim3(kBlock), 0, s, d, c.V, c.rms_eps, token_src, token_stride,
               rows_per_token, static_cast<const uint16_t*>(w.embed), w.g_attn[0], x, hb);
        TABED_BODY_CHECK();
    }
    for (int l = 0; l < c.layers; ++l) {
        e = projection(rows, d, 3 * d, gws, w.wqkv[l], hb, ones, y, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            const size_t layer_off = (size_t)l * rows * c.max_ctx * d;
            launch(&prof, k_body_rope_attn, dim3(c.heads, rows), dim3(kBlock), sizeof(float) * (size_t)c.max_ctx, s, d, hd,
                   c.max_ctx, (double)c.rope_theta, rows, y, ctx_len, kcache + layer_off, vcache + layer_off, hb);
            TABED_BODY_CHECK();
        }
        e = projection(rows, d, d, gws, w.wo[l], hb, ones, y, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            launch(&prof, k_body_add_norm, dim3(rows), dim3(kBlock), 0, s, d, d, c.rms_eps, x, y, w.g_mlp[l], hb,
                   static_cast<int32_t*>(nullptr));
            TABED_BODY_CHECK();
        }
        e = projection(rows, d, 2 * c.d_ff, gws, w.wgu[l], hb, ones, y, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            const size_t count = (size_t)rows * c.d_ff;
            launch(&prof, k_body_silu_mul, dim3((unsigned)((count + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, rows, c.d_ff, y, hb);
            TABED_BODY_CHECK();
        }
        e = projection(rows, c.d_ff, d, gws, w.wdown[l], hb, ones, y, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            const bool last = (l + 1 == c.layers);
            launch(&prof, k_body_add_norm, dim3(rows), dim3(kBlock), 0, s, d, d, c.rms_eps, x, y,
                   last ? w.g_final : w.g_attn[l + 1], last ? H : hb, last ? ctx_len : static_cast<int32_t*>(nullptr));
            TABED_BODY_CHECK();
        }
    }
#undef TABED_BODY_CHECK
    return hipSuccess;
}

hipError_t launch_body_rollback(int rows, int rows_per_seq, int gamma, const int32_t* ctx_base, const int32_t* accept_len,
                                int32_t* ctx_len, hipStream_t s) {
    launch(nullptr, k_body_rollback, dim3((rows + 255) / 256), dim3(256), 0, s, rows, rows_per_seq, gamma, ctx_base, accept_len,
           ctx_len);
    return hipGetLastError();
}

}  // namespace tabed
