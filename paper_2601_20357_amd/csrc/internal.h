// Host-side plumbing shared by the TABED translation units: workspace layout, launcher prototypes,
// per-kernel event timing.  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/tabed.h"

namespace tabed {

constexpr int kWave = 64;
constexpr int kBlock = 256;     // every vocab-pass kernel runs 4 waves per workgroup
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kTileV = 32;      // width of one softmax-partial tile written by the LM-head epilogue
constexpr int kSegV = 256;      // width of one CDF segment of the corrected/bonus sampler (one wave x float4)
constexpr int kChunkV = 4096;   // vocabulary span of one workgroup in the greedy arg-max pass (256 threads x 4 float4)
constexpr int kMaxGreedyChunks = 8;  // workgroups per greedy row in the draft arg-max pass
constexpr int kResidChunkV = 2048;  // vocabulary span of one workgroup in the corrected/bonus sampler (2 segments per wave)
constexpr int kStatHdr = 4;     // doubles before the per-draft sums in a chunk record: max, Z, argmax value, argmax index

struct Top2Rec {                // chunk candidate of the greedy draft arg-max
    float v1;
    int i1;
    float v2;
    int pad;
};

// Where everything lives inside the caller's workspace (byte offsets, 256-byte aligned).
struct WsLayout {
    int M, NT, C2, C3max, NSEG, C5, RS;
    int DW;              // width of one distance vector: n, or 11 candidate mixtures (policy 2)
    int Cd;              // vocabulary chunks of the second-pass distance kernel
    size_t off_tickets;  // uint32 [5][B]: arrival counters (0: greedy draft arg-max, 2: corrected/bonus sampler,
                         // 3: token-tree residual level, 4: token-tree bonus after a leaf)
    size_t off_pm;       // float  [M][NT] tile maxima of scaled logits
    size_t off_ps;       // float  [M][NT] tile sums of exp(scaled logit - tile max)
    size_t off_cand;     // Top2Rec [B][C2]
    size_t off_stats;    // double [B][gamma+1][C3max][RS]: header + one KL sum per draft (or per grid candidate)
    size_t off_seg;      // double [B][2][NSEG] segment masses: residual, target
    size_t off_wstage;   // float [B][n] next weights staged by the fused window update
    size_t off_dist;     // double [B][gamma][DW][Cd][2] chunk sums, or chunk arg-maxes (value, index), of the second pass
    size_t off_tstate;   // double [B][8] token-tree walk of every sequence (see TreeState)
    size_t off_tseg;     // double [B][2][NSEG] token-tree passes: segment masses, segment maxima
    size_t total;
};
WsLayout ws_layout(const tabed_cfg& c);
int validate_cfg(const tabed_cfg* c);

// ---------------------------------------------------------------- launchers (each enqueues on `s`)
hipError_t launch_ws_init(const tabed_cfg& c, const WsLayout& L, char* ws, hipStream_t s);

// prof_id: the timing bucket of the launch (the draft body runs its projections through the same kernels).
hipError_t launch_lmhead(const tabed_cfg& c, const WsLayout& L, char* ws, const void* W, const void* H,
                         const float* temperature, float* logits /* slot pos: [M,V] */, hipStream_t s,
                         int prof_id = TABED_K_LMHEAD);

hipError_t launch_sample(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int pos,
                         const float* logits /* slot pos */, const float* weights, const float* temperature,
                         const float* u_draft, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                         uint8_t* flags, hipStream_t s);

// Token tree.  Slots of a sequence's record in the workspace (doubles):
enum TreeState { kTsStatus = 0, kTsIndex = 1, kTsK = 2, kTsRowMax = 3, kTsRowZ = 4, kTsZ1 = 5, kTsZ2 = 6, kTsArgmax = 7, kTsSlots = 8 };
constexpr int kTreeDone = 0, kTreePending = 1, kTreeLeaf = 2;   // kTsStatus; kTsIndex = next level / accepted sibling
constexpr uint32_t kSiblingStride = 65536u;                     // Philox counter word 3 of sibling s: pos + s * 65536

hipError_t launch_siblings(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int pos, int width,
                           const float* logits /* slot pos */, const int32_t* draft_tokens, const float* weights,
                           const float* temperature, const float* u_sib, int32_t* sib_tokens, float* sib_q,
                           uint8_t* sib_flags, hipStream_t s);

hipError_t launch_verify_tree(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int width,
                              const float* target_logits, const float* leaf_logits, const float* draft_logits,
                              const double* draft_lse, const int32_t* sib_tokens, const float* sib_q,
                              const float* weights, const float* temperature, const float* u_res,
                              const float* u_acc_sib, int32_t* out_tokens, uint8_t* flags, int32_t* leaf,
                              int32_t* n_out, hipStream_t s);

hipError_t launch_verify(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round,
                         const float* target_logits, const float* draft_logits, const double* draft_lse,
                         const int32_t* draft_tokens, const float* draft_q, const float* weights,
                         const float* temperature, const float* u_acc, const float* u_res, int32_t* accept_len,
                         int32_t* out_tokens, float* dev, int32_t* n_valid, uint8_t* flags, float* ring,
                         int32_t* ring_head, int32_t* ring_count, float* next_weights, bool tree, hipStream_t s);

hipError_t launch_weights(const tabed_cfg& c, uint64_t round, const float* dev, const int32_t* n_valid, float* ring,
                          int32_t* ring_head, int32_t* ring_count, float* weights, hipStream_t s);

hipError_t launch_null(hipStream_t s);

hipError_t launch_philox(const tabed_cfg& c, uint64_t round, float* out, hipStream_t s);

// ---------------------------------------------------------------- draft-model body
struct BodyLayout {
    size_t off_ones;   // float [rows]: the "temperature" the projection launches divide by
    size_t off_x;      // float [rows,d] residual stream
    size_t off_y;      // float [rows, max(3d, 2 d_ff)] result of the current projection
    size_t off_hb;     // bf16 [rows, max(d, d_ff)] input of the next projection
    size_t off_gemm;   // scratch of the projection launches (softmax partials nobody reads)
    size_t total;
};
BodyLayout body_layout(const tabed_body_cfg& c, int rows);
int validate_body_cfg(const tabed_body_cfg* c, int rows);
hipError_t launch_body_init(const tabed_body_cfg& c, int rows, char* ws, hipStream_t s);
hipError_t launch_body_step(const tabed_body_cfg& c, const tabed_body_weights& w, char* ws, int rows,
                            const int32_t* token_src, int token_stride, int rows_per_token, int32_t* ctx_len,
                            uint16_t* kcache, uint16_t* vcache, uint16_t* H, hipStream_t s);
hipError_t launch_body_rollback(int rows, int rows_per_seq, int gamma, const int32_t* ctx_base, const int32_t* accept_len,
                                int32_t* ctx_len, hipStream_t s);

// ---------------------------------------------------------------- event timing
// While timing is enabled a launch goes through hipExtLaunchKernelGGL, which attaches a start and a stop
// event to the dispatch itself: the pair measures the kernel's own begin-to-end time (what a kernel trace
// reports), not the dispatch gaps around it.
bool prof_on();
void prof_push(int id, hipEvent_t start, hipEvent_t stop);
struct ProfScope {
    int id;
    bool on;
    hipEvent_t start = nullptr, stop = nullptr;
    ProfScope(int id_, hipStream_t) : id(id_), on(prof_on()) {
        if (on && (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess)) on = false;
    }
    ~ProfScope() { if (on) prof_push(id, start, stop); }
    ProfScope(const ProfScope&) = delete;
    ProfScope& operator=(const ProfScope&) = delete;
};

}  // namespace tabed

#if defined(__HIPCC__)
#include <hip/hip_ext.h>
namespace tabed {
template <typename K, typename... Args>
inline void launch(const ProfScope* prof, K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, Args... args) {
    if (prof != nullptr && prof->on)
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, s, prof->start, prof->stop, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}
}  // namespace tabed
#endif
