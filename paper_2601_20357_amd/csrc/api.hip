// C ABI of the TABED hot path (see include/tabed.h): argument validation on the host, workspace
// layout, launch sequencing, optional per-kernel event timing.  No allocation, no synchronisation,
// except inside the tabed_prof_* calls.
#include <atomic>
#include <mutex>
#include <vector>

#include "internal.h"

namespace tabed {

static thread_local int g_last_hip_error = 0;

static size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int validate_cfg(const tabed_cfg* c) {
    if (c == nullptr) return TABED_ENULL;
    if (c->V < 1 || c->d < 1 || c->B < 1 || c->h < 0 || c->n < 1 || c->gamma < 1) return TABED_EINVAL;
    if (c->n > TABED_MAX_N || c->gamma > TABED_MAX_GAMMA) return TABED_ERANGE;
    if (c->w_dtype != 0 && c->w_dtype != 1) return TABED_EINVAL;
    if (c->w_dtype == 1 && (c->d % 8) != 0) return TABED_EINVAL;
    if (c->distance < 0 || c->distance > 2) return TABED_EINVAL;
    if (c->policy < 0 || c->policy > 3) return TABED_EINVAL;
    if (c->policy == 2 && c->n != 2) return TABED_EINVAL;
    if (!(c->tau_w > 0.f) || !(c->eps > 0.f)) return TABED_EINVAL;
    if (c->B > 65535 || (long long)c->B * c->n > (1ll << 24)) return TABED_ERANGE;   // B is a grid dimension
    if (c->V > kTileV * kBlock * 32) return TABED_ERANGE;      // 262144: largest vocabulary the sampler tiles
    return TABED_OK;
}

WsLayout ws_layout(const tabed_cfg& c) {
    WsLayout L;
    L.M = c.n * c.B;
    L.NT = (c.V + kTileV - 1) / kTileV;
    L.C2 = (c.V + kChunkV - 1) / kChunkV;
    if (L.C2 > kMaxGreedyChunks) L.C2 = kMaxGreedyChunks;
    L.C3max = (c.V + kBlock * 4 - 1) / (kBlock * 4);
    L.NSEG = (c.V + kSegV - 1) / kSegV;
    L.C5 = (c.V + kResidChunkV - 1) / kResidChunkV;
    L.RS = kStatHdr + ((c.policy == 2 && TABED_GRID_CANDIDATES > c.n) ? TABED_GRID_CANDIDATES : c.n);   // A sums: per draft, or per mixture
    L.DW = (c.policy == 2) ? TABED_GRID_CANDIDATES : c.n;
    L.Cd = (c.V + kChunkV - 1) / kChunkV;
    size_t off = 0;
    L.off_tickets = off; off = align_up(off + sizeof(uint32_t) * 5 * (size_t)c.B);
    L.off_pm = off;      off = align_up(off + sizeof(float) * (size_t)L.M * L.NT);
    L.off_ps = off;      off = align_up(off + sizeof(float) * (size_t)L.M * L.NT);
    L.off_cand = off;    off = align_up(off + sizeof(Top2Rec) * (size_t)c.B * L.C2);
    L.off_stats = off;   off = align_up(off + sizeof(double) * (size_t)c.B * (c.gamma + 1) * L.C3max * L.RS);
    L.off_seg = off;     off = align_up(off + sizeof(double) * 2 * (size_t)c.B * L.NSEG);
    L.off_wstage = off;  off = align_up(off + sizeof(float) * (size_t)c.B * c.n);
    L.off_dist = off;    off = align_up(off + sizeof(double) * 2 * (size_t)c.B * c.gamma * L.DW * L.Cd);
    L.off_tstate = off;  off = align_up(off + sizeof(double) * kTsSlots * (size_t)c.B);
    L.off_tseg = off;    off = align_up(off + sizeof(double) * 2 * (size_t)c.B * L.NSEG);
    L.total = off;
    return L;
}

// ---------------------------------------------------------------- event timing
struct ProfRec {
    int id;
    hipEvent_t start, stop;
};
static std::mutex g_prof_mu;
static std::atomic<bool> g_prof_on{false};
static std::vector<ProfRec> g_prof_pending;
static double g_prof_ms[TABED_K_COUNT];
static int64_t g_prof_n[TABED_K_COUNT];

bool prof_on() { return g_prof_on.load(std::memory_order_relaxed); }
void prof_push(int id, hipEvent_t start, hipEvent_t stop) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_pending.push_back(ProfRec{id, start, stop});
}
static void prof_drain() {
    for (ProfRec& r : g_prof_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            g_prof_ms[r.id] += (double)ms;
            g_prof_n[r.id] += 1;
        }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_prof_pending.clear();
}

static int fail_hip(hipError_t e) {
    g_last_hip_error = (int)e;
    return TABED_EHIP;
}
static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// ---------------------------------------------------------------- built-in scratch of tabed_draft_step_static
// One array per GPU, part of the loaded code object, so no call ever allocates it.  `scratch` is only a
// host-side handle: the array's device address on the current GPU comes from hipGetSymbolAddress, looked up once
// per device, and that pointer is what kernels and launchers receive.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[TABED_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];

static int static_scratch(char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e);
    if (dev < 0 || dev >= kMaxDevices) return TABED_ERANGE;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return fail_hip(e);
        if (p == nullptr) return fail_hip(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char*>(g_scratch_ptr[dev]);
    return TABED_OK;
}

}  // namespace tabed

using namespace tabed;

extern "C" {

int32_t tabed_dev_width(const tabed_cfg* cfg) {
    if (validate_cfg(cfg) != TABED_OK) return 0;
    return ws_layout(*cfg).DW;
}

size_t tabed_workspace_bytes(const tabed_cfg* cfg) {
    if (validate_cfg(cfg) != TABED_OK) return 0;
    return ws_layout(*cfg).total;
}

int tabed_workspace_init(const tabed_cfg* cfg, void* ws, void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (ws == nullptr) return TABED_ENULL;
    if (misaligned(ws)) return TABED_EALIGN;
    const hipError_t e = launch_ws_init(*cfg, ws_layout(*cfg), static_cast<char*>(ws), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

const char* tabed_strerror(int code) {
    switch (code) {
        case TABED_OK: return "ok";
        case TABED_ENULL: return "a required pointer is NULL";
        case TABED_EINVAL: return "a configuration field is out of range";
        case TABED_ERANGE: return "an index or count exceeds the supported range";
        case TABED_EALIGN: return "a base pointer is not 16-byte aligned";
        case TABED_EUNSUPPORTED: return "valid request that this build does not implement";
        case TABED_EHIP: return "a kernel launch failed";
        case TABED_ETOOBIG: return "the configuration needs more scratch than the built-in buffer holds";
        default: return "unknown error code";
    }
}

int tabed_last_hip_error(void) { return g_last_hip_error; }

int tabed_draft_step(const tabed_cfg* cfg, void* ws, uint64_t round, int32_t pos, const void* W, const void* H,
                     const float* weights, const float* temperature, const float* u_draft, float* draft_logits,
                     double* draft_lse, int32_t* draft_tokens, float* draft_q, uint8_t* flags, void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (!ws || !W || !H || !weights || !temperature || !draft_logits || !draft_lse || !draft_tokens || !draft_q || !flags)
        return TABED_ENULL;
    if (pos < 0 || pos >= cfg->gamma) return TABED_ERANGE;
    if (misaligned(ws) || misaligned(W) || misaligned(H) || misaligned(draft_logits) || misaligned(draft_lse))
        return TABED_EALIGN;
    const WsLayout L = ws_layout(*cfg);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* slot = draft_logits + (size_t)pos * L.M * cfg->V;
    hipError_t e = launch_lmhead(*cfg, L, static_cast<char*>(ws), W, H, temperature, slot, s);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_sample(*cfg, L, static_cast<char*>(ws), round, pos, slot, weights, temperature, u_draft, draft_lse,
                      draft_tokens, draft_q, flags, s);
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_draft_step_static(const tabed_cfg* cfg, uint64_t round, int32_t pos, const void* W, const void* H,
                            const float* weights, const float* temperature, const float* u_draft,
                            float* draft_logits, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                            uint8_t* flags, void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (!W || !H || !weights || !temperature || !draft_logits || !draft_lse || !draft_tokens || !draft_q || !flags)
        return TABED_ENULL;
    if (pos < 0 || pos >= cfg->gamma) return TABED_ERANGE;
    if (misaligned(W) || misaligned(H) || misaligned(draft_logits) || misaligned(draft_lse)) return TABED_EALIGN;
    const WsLayout L = ws_layout(*cfg);
    if (L.total > (size_t)TABED_STATIC_SCRATCH_BYTES) return TABED_ETOOBIG;
    char* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != TABED_OK) return rs;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the array keeps whatever the last call (of any configuration) left: the arrival counters start at zero
    hipError_t e = launch_ws_init(*cfg, L, ws, s);
    if (e != hipSuccess) return fail_hip(e);
    float* slot = draft_logits + (size_t)pos * L.M * cfg->V;
    e = launch_lmhead(*cfg, L, ws, W, H, temperature, slot, s);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_sample(*cfg, L, ws, round, pos, slot, weights, temperature, u_draft, draft_lse, draft_tokens, draft_q,
                      flags, s);
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_verify(const tabed_cfg* cfg, void* ws, uint64_t round, const float* target_logits,
                 const float* draft_logits, const double* draft_lse, const int32_t* draft_tokens,
                 const float* draft_q, const float* weights, const float* temperature, const float* u_acc,
                 const float* u_res, int32_t* accept_len, int32_t* out_tokens, float* dev, int32_t* n_valid,
                 uint8_t* flags, float* ring, int32_t* ring_head, int32_t* ring_count, float* next_weights,
                 void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (!ws || !target_logits || !draft_logits || !draft_lse || !draft_tokens || !draft_q || !weights ||
        !temperature || !accept_len || !out_tokens || !dev || !n_valid || !flags)
        return TABED_ENULL;
    if (misaligned(ws) || misaligned(target_logits) || misaligned(draft_logits) || misaligned(draft_lse))
        return TABED_EALIGN;
    const int nwin = (ring != nullptr) + (ring_head != nullptr) + (ring_count != nullptr) + (next_weights != nullptr);
    if (nwin != 0 && nwin != 4) return TABED_ENULL;        // the fused window update takes all four or none
    const WsLayout L = ws_layout(*cfg);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = launch_verify(*cfg, L, static_cast<char*>(ws), round, target_logits, draft_logits, draft_lse,
                                       draft_tokens, draft_q, weights, temperature, u_acc, u_res, accept_len,
                                       out_tokens, dev, n_valid, flags, ring, ring_head, ring_count, next_weights,
                                       /*tree=*/false, s);
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_draft_siblings(const tabed_cfg* cfg, void* ws, uint64_t round, int32_t pos, int32_t tree_width,
                         const float* draft_logits, const int32_t* draft_tokens, const float* weights,
                         const float* temperature, const float* u_sib, int32_t* sib_tokens, float* sib_q,
                         uint8_t* sib_flags, void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (tree_width < 1 || tree_width > TABED_MAX_TREE_WIDTH) return TABED_ERANGE;
    if (pos < 0 || pos >= cfg->gamma) return TABED_ERANGE;
    if (tree_width == 1) return TABED_OK;                   // a chain has no siblings
    if (!ws || !draft_logits || !draft_tokens || !weights || !temperature || !sib_tokens || !sib_q || !sib_flags)
        return TABED_ENULL;
    if (misaligned(ws) || misaligned(draft_logits)) return TABED_EALIGN;
    const WsLayout L = ws_layout(*cfg);
    const float* slot = draft_logits + (size_t)pos * L.M * cfg->V;
    const hipError_t e = launch_siblings(*cfg, L, static_cast<char*>(ws), round, pos, tree_width, slot, draft_tokens, weights,
                                         temperature, u_sib, sib_tokens, sib_q, sib_flags, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_verify_tree(const tabed_cfg* cfg, void* ws, uint64_t round, int32_t tree_width, const float* target_logits,
                      const float* leaf_logits, const float* draft_logits, const double* draft_lse,
                      const int32_t* draft_tokens, const float* draft_q, const int32_t* sib_tokens, const float* sib_q,
                      const float* weights, const float* temperature, const float* u_acc, const float* u_res,
                      const float* u_acc_sib, int32_t* accept_len, int32_t* out_tokens, float* dev, int32_t* n_valid,
                      uint8_t* flags, int32_t* leaf, int32_t* n_out, float* ring, int32_t* ring_head,
                      int32_t* ring_count, float* next_weights, void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (tree_width < 1 || tree_width > TABED_MAX_TREE_WIDTH) return TABED_ERANGE;
    if (cfg->distance == 2) return TABED_EUNSUPPORTED;      // hard labels are defined for the chain only
    if (!ws || !target_logits || !draft_logits || !draft_lse || !draft_tokens || !draft_q || !weights ||
        !temperature || !accept_len || !out_tokens || !dev || !n_valid || !flags || !leaf || !n_out)
        return TABED_ENULL;
    if (tree_width > 1 && (!leaf_logits || !sib_tokens || !sib_q)) return TABED_ENULL;
    if (misaligned(ws) || misaligned(target_logits) || misaligned(draft_logits) || misaligned(draft_lse) ||
        (tree_width > 1 && misaligned(leaf_logits)))
        return TABED_EALIGN;
    const int nwin = (ring != nullptr) + (ring_head != nullptr) + (ring_count != nullptr) + (next_weights != nullptr);
    if (nwin != 0 && nwin != 4) return TABED_ENULL;
    if (next_weights == weights) return TABED_EINVAL;       // the tree passes still read this block's weights
    const WsLayout L = ws_layout(*cfg);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_verify(*cfg, L, static_cast<char*>(ws), round, target_logits, draft_logits, draft_lse,
                                 draft_tokens, draft_q, weights, temperature, u_acc, u_res, accept_len, out_tokens, dev,
                                 n_valid, flags, ring, ring_head, ring_count, next_weights, /*tree=*/true, s);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_verify_tree(*cfg, L, static_cast<char*>(ws), round, tree_width, target_logits, leaf_logits, draft_logits,
                           draft_lse, sib_tokens, sib_q, weights, temperature, u_res, u_acc_sib, out_tokens, flags, leaf,
                           n_out, s);
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_update_weights(const tabed_cfg* cfg, void* ws, uint64_t round, const float* dev, const int32_t* n_valid, float* ring,
                         int32_t* ring_head, int32_t* ring_count, float* weights, void* stream) {
    (void)ws;
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (!ring || !ring_head || !ring_count || !weights) return TABED_ENULL;
    if ((dev == nullptr) != (n_valid == nullptr)) return TABED_ENULL;
    const hipError_t e = launch_weights(*cfg, round, dev, n_valid, ring, ring_head, ring_count, weights,
                                        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

size_t tabed_body_workspace_bytes(const tabed_body_cfg* cfg, int32_t rows) {
    if (validate_body_cfg(cfg, rows) != TABED_OK) return 0;
    return body_layout(*cfg, rows).total;
}

int tabed_body_workspace_init(const tabed_body_cfg* cfg, int32_t rows, void* ws, void* stream) {
    const int rc = validate_body_cfg(cfg, rows);
    if (rc != TABED_OK) return rc;
    if (ws == nullptr) return TABED_ENULL;
    if (misaligned(ws)) return TABED_EALIGN;
    const hipError_t e = launch_body_init(*cfg, rows, static_cast<char*>(ws), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_draft_body_step(const tabed_body_cfg* cfg, const tabed_body_weights* weights, void* ws, int32_t rows,
                          const int32_t* token_src, int32_t token_stride, int32_t rows_per_token, int32_t* ctx_len,
                          void* kcache, void* vcache, void* H, void* stream) {
    const int rc = validate_body_cfg(cfg, rows);
    if (rc != TABED_OK) return rc;
    if (!weights || !ws || !token_src || !ctx_len || !kcache || !vcache || !H) return TABED_ENULL;
    if (rows_per_token < 1 || token_stride < 0) return TABED_ERANGE;
    if (!weights->embed || !weights->g_final) return TABED_ENULL;
    for (int l = 0; l < cfg->layers; ++l) {
        if (!weights->g_attn[l] || !weights->wqkv[l] || !weights->wo[l] || !weights->g_mlp[l] || !weights->wgu[l] ||
            !weights->wdown[l])
            return TABED_ENULL;
        if (misaligned(weights->wqkv[l]) || misaligned(weights->wo[l]) || misaligned(weights->wgu[l]) ||
            misaligned(weights->wdown[l]) || misaligned(weights->g_attn[l]) || misaligned(weights->g_mlp[l]))
            return TABED_EALIGN;
    }
    if (misaligned(ws) || misaligned(kcache) || misaligned(vcache) || misaligned(H) || misaligned(weights->embed) ||
        misaligned(weights->g_final))
        return TABED_EALIGN;
    const hipError_t e = launch_body_step(*cfg, *weights, static_cast<char*>(ws), rows, token_src, token_stride, rows_per_token,
                                          ctx_len, static_cast<uint16_t*>(kcache), static_cast<uint16_t*>(vcache),
                                          static_cast<uint16_t*>(H), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_draft_body_rollback(int32_t rows, int32_t rows_per_seq, int32_t gamma, const int32_t* ctx_base,
                              const int32_t* accept_len, int32_t* ctx_len, void* stream) {
    if (!ctx_base || !accept_len || !ctx_len) return TABED_ENULL;
    if (rows < 1 || rows_per_seq < 1 || gamma < 1) return TABED_ERANGE;
    const hipError_t e = launch_body_rollback(rows, rows_per_seq, gamma, ctx_base, accept_len, ctx_len,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_philox_uniforms(const tabed_cfg* cfg, uint64_t round, float* out, void* stream) {
    const int rc = validate_cfg(cfg);
    if (rc != TABED_OK) return rc;
    if (!out) return TABED_ENULL;
    const hipError_t e = launch_philox(*cfg, round, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

int tabed_prof_enable(int on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on.store(on != 0, std::memory_order_relaxed);
    return TABED_OK;
}

int tabed_prof_read(int id, double* total_ms, int64_t* launches) {
    if (id < 0 || id >= TABED_K_COUNT) return TABED_ERANGE;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    prof_drain();
    if (total_ms) *total_ms = g_prof_ms[id];
    if (launches) *launches = g_prof_n[id];
    return TABED_OK;
}

int tabed_prof_reset(void) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    prof_drain();
    for (int i = 0; i < TABED_K_COUNT; ++i) { g_prof_ms[i] = 0.0; g_prof_n[i] = 0; }
    return TABED_OK;
}

int tabed_prof_null(void* stream) {
    const hipError_t e = launch_null(static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TABED_OK : fail_hip(e);
}

const char* tabed_kernel_name(int id) {
    switch (id) {
        case TABED_K_LMHEAD: return "lmhead";
        case TABED_K_SAMPLE: return "sample";
        case TABED_K_STATS: return "stats";
        case TABED_K_RESID: return "resid";
        case TABED_K_WEIGHTS: return "weights";
        case TABED_K_DIST: return "dist";
        case TABED_K_TREE: return "tree";
        case TABED_K_BODY: return "body";
        case TABED_K_NULL: return "null";
        default: return "?";
    }
}

}  // extern "C"
