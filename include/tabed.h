/*
 * tabed.h -- C ABI of the TABED per-round hot path on one MI355X (gfx950).
 *
 * TABED (Test-time Adaptive Batched Ensemble Drafting) runs n drafting methods
 * as one batch through a shared draft model, mixes their next-token
 * distributions with test-time-adaptive weights, and has the target model
 * verify gamma drafted tokens by speculative sampling.  This library is the
 * part of one such round that sits behind the two models' transformer bodies:
 *
 *   tabed_update_weights   Alg. 1 (weight-selection step) with the many-draft policy of
 *                          App. B.2 (w = softmax(1/e; tau)), incl. the window.
 *   tabed_draft_step       Alg. 1 (loop body: draft forward, W-Avg, Sample) for one in-block position: LM head
 *                          of the n drafts as one batched GEMM, per-draft
 *                          softmax, weighted-average ensemble, next token.
 *   tabed_verify           Sec. 3 items 2-3: accept each drafted token with
 *                          probability min(1, p/q), resample the first rejected
 *                          one from norm(max(0, p - q)); plus the per-position
 *                          distances D(p, q^(j)) of Sec. 5.1 that feed the
 *                          next tabed_update_weights.
 *
 * Around that path:
 *
 *   tabed_draft_siblings,  Sec. 6.1 "Verification: Integrating Token Tree" (App. D): sibling candidates of a
 *   tabed_verify_tree      position and their verification by multi-round rejection sampling.
 *   tabed_draft_body_step, Sec. 5.1 "Ensemble learning via Batched Inference", Sec. 4.1 "Target and Draft
 *   tabed_draft_body_rollback   Models": one decode step of the shared LLaMA-style draft model for the n * B rows.
 *   tabed_draft_step_static     tabed_draft_step for callers that cannot allocate device memory.
 *
 * Notation: n = number of drafting methods (the paper's m), B independent
 * sequences, V vocabulary size, d draft hidden size, gamma block length,
 * h observation window (in verified positions).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller; `cfg` is a
 *     HOST pointer.  The library allocates, frees and synchronises nothing:
 *     kernels are enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns at once.
 *   - Row-major, innermost index last.  Base pointers 16-byte aligned.
 *   - Return value: TABED_OK or a negative TABED_E* code.  Argument errors are
 *     detected on the host before anything is enqueued.
 *   - `ws` is scratch memory of tabed_workspace_bytes(cfg) bytes.  It must be
 *     prepared once with tabed_workspace_init() and may then be reused by any
 *     number of calls with the same cfg on the same stream.  Calls that share
 *     a workspace must not overlap.
 *   - A temperature of 0 marks a greedy row: token decisions are arg-max
 *     (lowest index on ties) and its distributions are the untempered softmax.
 *   - Uniform random numbers come from Philox4x32-10 with key = cfg->seed and
 *     counter = (round, b, pos): word 0 at pos < gamma drives the draft sample,
 *     word 1 the accept test; word 0 at pos = gamma drives the corrected /
 *     bonus sample; u = (x >> 8) * 2^-24.  Each call also takes optional
 *     arrays of explicit uniforms that replace them (NULL = Philox).
 *   - flag bits: TABED_FLAG_* below.  A flagged decision had a margin below
 *     1e-6 relative and may legitimately differ from a higher-precision
 *     evaluation.
 */
#ifndef TABED_H
#define TABED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TABED_MAX_N 16     /* drafting methods                      */
#define TABED_MAX_TREE_WIDTH 3 /* candidates per position of a token tree (1 = chain) */
#define TABED_MAX_GAMMA 32 /* block length                          */

#define TABED_OK 0
#define TABED_ENULL (-1)        /* a required pointer is NULL                         */
#define TABED_EINVAL (-2)       /* a cfg field is out of range                        */
#define TABED_ERANGE (-3)       /* pos >= gamma, n > TABED_MAX_N, ...                 */
#define TABED_EALIGN (-4)       /* a base pointer is not 16-byte aligned              */
#define TABED_EUNSUPPORTED (-5) /* valid request this build does not implement        */
#define TABED_EHIP (-6)         /* a kernel launch failed (see tabed_last_hip_error)  */
#define TABED_ETOOBIG (-7)      /* cfg needs more scratch than tabed_draft_step_static's built-in buffer */

#define TABED_FLAG_ACCEPT_MARGIN 1u /* accept test u*q < p closer than 1e-6 relative          */
#define TABED_FLAG_SAMPLE_MARGIN 2u /* CDF crossing / arg-max runner-up closer than 1e-6      */
#define TABED_FLAG_DEGENERATE 4u    /* empty residual, CDF never crossed, or token out of range */

typedef struct tabed_cfg {
    int32_t V;        /* vocabulary size, 1..262144                                        */
    int32_t d;        /* draft hidden size, >= 1 (multiple of 8 when w_dtype = 1)          */
    int32_t n;        /* drafting methods batched through the draft model, 1..TABED_MAX_N  */
    int32_t B;        /* independent sequences, 1..65535                                   */
    int32_t gamma;    /* draft block length, 1..TABED_MAX_GAMMA                            */
    int32_t h;        /* observation window length in verified positions, >= 1; 0 = ALL    */
                      /* positions since the start (the paper's default, App. B.1)         */
    int32_t w_dtype;  /* storage type of W and H: 0 = fp32, 1 = bf16                       */
    int32_t distance; /* D of Alg. 1: 0 = KL(p || q) (Sec. 5.1); 1 = total variation;      */
                      /* 2 = hard labels: 1 where the candidate's arg-max token differs    */
                      /*     from the token emitted at the position, else 0                */
    int32_t policy;   /* 0 = softmax(1/e; tau_w) (App. B.2); 1 = static equal weights;     */
                      /* 2 = two-draft grid (App. B.2): arg-min over w^c = [1-c/10, c/10], */
                      /*     c = 0..10, of the window sum of D(p, mixture); needs n = 2;   */
                      /* 3 = random weights, uniform on the simplex, fresh for every block */
                      /*     (the random-weights ablation of Sec. 6.2)                       */
    float tau_w;      /* temperature of the weight softmax, > 0 (paper default 1)          */
    float eps;        /* e is clamped to >= eps before 1/e, > 0                            */
    uint64_t seed;    /* Philox key                                                        */
} tabed_cfg;

#define TABED_GRID_CANDIDATES 11

/* Width DW of one distance vector (last dimension of `dev` and `ring`): n per-draft distances, or
 * TABED_GRID_CANDIDATES mixture distances when policy = 2; 0 if cfg is invalid. */
int32_t tabed_dev_width(const tabed_cfg* cfg);

/* Bytes of scratch the calls below need for this cfg; 0 if cfg is invalid. */
size_t tabed_workspace_bytes(const tabed_cfg* cfg);

/* Zeroes the arrival counters inside `ws` (a small fill kernel on `stream`).
 * Call once after allocating `ws`, before the first draft/verify call. */
int tabed_workspace_init(const tabed_cfg* cfg, void* ws, void* stream);

/* Static text for an error code. */
const char* tabed_strerror(int code);

/* hipError_t value of the most recent failed launch on this host thread (0 if none). */
int tabed_last_hip_error(void);

/*
 * Alg. 1 (loop body: draft forward, W-Avg, Sample) at in-block position `pos` (0 <= pos < gamma) for all B
 * sequences:  L = H W^T for the n*B rows, q^(j) = softmax(L_j / T),
 * q = sum_j w_j q^(j), y ~ Sample(q) (arg-max for greedy rows).
 *
 *   W            [V,d]            in   LM-head matrix shared by all drafts (w_dtype)
 *   H            [B,n,d]          in   last hidden state of every draft (w_dtype)
 *   weights      [B,n]     fp32   in   w*_t, constant over the block (Sec. 5.1)
 *   temperature  [B]       fp32   in   0 => greedy row
 *   u_draft      [B,gamma] fp32   in   optional explicit uniforms, column pos is read; NULL => Philox
 *   draft_logits [gamma,B,n,V] fp32 out slot pos is written
 *   draft_lse    [gamma,B,n] fp64 out  log-sum-exp of L_j / T, slot pos is written
 *   draft_tokens [B,gamma] int32  out  column pos is written
 *   draft_q      [B,gamma] fp32   out  q(y), column pos is written
 *   flags        [B,gamma] uint8  out  column pos is written
 */
int tabed_draft_step(const tabed_cfg* cfg, void* ws, uint64_t round, int32_t pos,
                     const void* W, const void* H, const float* weights, const float* temperature,
                     const float* u_draft,
                     float* draft_logits, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                     uint8_t* flags, void* stream);

/*
 * tabed_draft_step without a workspace argument, for callers that cannot allocate device memory at all: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; the scratch memory is a buffer of TABED_STATIC_SCRATCH_BYTES built into the
 * library's code object (every GPU the library runs on holds one copy until the process ends), so the call
 * neither allocates nor frees anything, directly or through a library.
 *   - returns TABED_ETOOBIG when tabed_workspace_bytes(cfg) exceeds TABED_STATIC_SCRATCH_BYTES (e.g. the
 *     512-row stress shape); nothing is enqueued then.
 *   - every call on a GPU uses that GPU's one buffer, which keeps the previous call's contents; the call
 *     clears what must start at zero itself (a fill kernel on `stream`).  Calls that overlap on one GPU
 *     (different streams, or threads) race on it: serialise them, or use tabed_draft_step with one
 *     workspace per stream.
 *   - the buffer's device address is looked up on the first call on each device (with that device current);
 *     make that first call outside graph capture.
 */
#define TABED_STATIC_SCRATCH_BYTES (8u << 20)
int tabed_draft_step_static(const tabed_cfg* cfg, uint64_t round, int32_t pos,
                            const void* W, const void* H, const float* weights, const float* temperature,
                            const float* u_draft,
                            float* draft_logits, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                            uint8_t* flags, void* stream);

/*
 * Sec. 3 items 2-3 for all B sequences, given the target's logits at the
 * gamma drafted positions and one position beyond; plus D(p_i, q_i^(j)) for
 * every drafted position i and draft j (Sec. 5.1).
 *
 *   target_logits [B,gamma+1,V] fp32 in
 *   draft_logits, draft_lse, draft_tokens, draft_q, weights, temperature: as written by / passed to
 *                 the gamma tabed_draft_step calls of this round
 *   u_acc         [B,gamma] fp32  in   optional explicit accept-test uniforms; NULL => Philox
 *   u_res         [B]       fp32  in   optional explicit uniform of the corrected/bonus sample
 *   accept_len    [B]       int32 out  k = number of accepted draft tokens, 0..gamma
 *   out_tokens    [B,gamma+1] int32 out k accepted tokens, then one corrected (k < gamma) or bonus
 *                 (k = gamma) token, then -1
 *   dev           [B,gamma,DW] fp32 out D(p_i, q_i^(j)) for every draft j (DW = n), or with policy = 2
 *                 D(p_i, (1-c/10) q_i^(1) + (c/10) q_i^(2)) for c = 0..10 (DW = 11); meaningful for i < n_valid[b]
 *   n_valid       [B]       int32 out  min(k+1, gamma): positions whose distances enter the window
 *   flags         [B,gamma+1] uint8 out flags of the accept test at i and of the sample emitted at i
 *                 (hard labels with the two-draft grid: TABED_FLAG_SAMPLE_MARGIN at a labelled position i <= k also
 *                 when the two largest entries of a candidate mixture there are closer than 1e-6 relative)
 *   ring, ring_head, ring_count, next_weights: optional, all four or all NULL.  When given, the call also
 *                 performs the tabed_update_weights() that would open round + 1 (same arguments, same
 *                 result: the window takes the n_valid verified positions and next_weights [B,n] receives the
 *                 weights of the next block), saving that call's launch.  next_weights may alias weights.
 * A drafted token outside [0,V) is rejected and flagged TABED_FLAG_DEGENERATE.
 */
int tabed_verify(const tabed_cfg* cfg, void* ws, uint64_t round,
                 const float* target_logits, const float* draft_logits, const double* draft_lse,
                 const int32_t* draft_tokens, const float* draft_q, const float* weights,
                 const float* temperature, const float* u_acc, const float* u_res,
                 int32_t* accept_len, int32_t* out_tokens, float* dev, int32_t* n_valid,
                 uint8_t* flags, float* ring, int32_t* ring_head, int32_t* ring_count, float* next_weights,
                 void* stream);

/*
 * Token tree (Sec. 6.1, paragraph "Verification: Integrating Token Tree"; results in App. D for widths 2 and 3).
 * The paper names the tree width and nothing else; the construction taken here: at every in-block position the
 * draft proposes tree_width sibling candidates for the same prefix, all from that position's ensembled
 * distribution q_i.  Candidate 0 is the token tabed_draft_step samples (the trunk: the only candidate the draft
 * model extends), candidates 1..tree_width-1 are leaves: a sampling row draws them independently from q_i, a
 * greedy row takes the next-largest entries of q_i.  tree_width = 1 is the chain.
 *
 * tabed_draft_siblings draws the siblings of position pos.  Call it after tabed_draft_step(pos) and before
 * tabed_draft_step(pos + 1): it works from the softmax partials that call left in `ws`.
 *   draft_logits [gamma,B,n,V], draft_tokens [B,gamma]: as written by tabed_draft_step (slot / column pos)
 *   u_sib        [B,gamma,tree_width-1] fp32 in   optional explicit uniforms; NULL => Philox block of counter
 *                (round, b, pos + s * 65536) for sibling s >= 1: word 0 draws it, word 1 is its accept uniform
 *   sib_tokens, sib_q, sib_flags [B,gamma,tree_width-1] out  entries (b, pos, :) are written: token, q_i(token), flags
 */
int tabed_draft_siblings(const tabed_cfg* cfg, void* ws, uint64_t round, int32_t pos, int32_t tree_width,
                         const float* draft_logits, const int32_t* draft_tokens, const float* weights,
                         const float* temperature, const float* u_sib,
                         int32_t* sib_tokens, float* sib_q, uint8_t* sib_flags, void* stream);

/*
 * Verification of the token tree.  The trunk is verified exactly as tabed_verify does (same arguments, same
 * results for accept_len = k, dev, n_valid, the window update).  At the position k where the trunk token is
 * rejected the siblings are tried in order by multi-round rejection sampling, the lossless rule for several
 * candidates from one proposal: with f_0 = p_k, Z_0 = 1 and f_c = max(0, f_{c-1} / Z_{c-1} - q_k), Z_c = sum f_c,
 * sibling c is accepted iff u_c q_k(y_c) Z_c < f_c(y_c).  An accepted sibling is emitted and followed by one
 * bonus token from the target's distribution after it (leaf_logits); if every candidate is rejected the
 * corrected token is drawn from f_width / Z_width.  Greedy rows: a candidate is accepted iff it equals
 * arg-max p_k.  The round's one final draw uses u_res, as in the chain.
 *   leaf_logits  [B,gamma,tree_width-1,V] fp32 in  target logits after sibling s of position i
 *   sib_tokens, sib_q [B,gamma,tree_width-1]   in  as written by tabed_draft_siblings
 *   u_acc_sib    [B,gamma,tree_width-1] fp32   in  optional explicit accept uniforms of the siblings
 *   out_tokens   [B,gamma+1]  k trunk tokens, then the accepted sibling and its bonus token, or the corrected /
 *                bonus token of the chain, then -1
 *   leaf         [B] int32 out  0, or the index s of the accepted sibling
 *   n_out        [B] int32 out  tokens emitted: k + 1, or k + 2 after a leaf
 *   flags        [B,gamma+1]    column k also carries the sibling tests' margin bits, column k + 1 the draw after a leaf
 * next_weights must not alias weights here (the tree passes read this block's weights after the window update).
 * cfg->distance = 2 (hard labels) is not defined for trees: TABED_EUNSUPPORTED.
 */
int tabed_verify_tree(const tabed_cfg* cfg, void* ws, uint64_t round, int32_t tree_width,
                      const float* target_logits, const float* leaf_logits, const float* draft_logits,
                      const double* draft_lse, const int32_t* draft_tokens, const float* draft_q,
                      const int32_t* sib_tokens, const float* sib_q, const float* weights, const float* temperature,
                      const float* u_acc, const float* u_res, const float* u_acc_sib,
                      int32_t* accept_len, int32_t* out_tokens, float* dev, int32_t* n_valid, uint8_t* flags,
                      int32_t* leaf, int32_t* n_out,
                      float* ring, int32_t* ring_head, int32_t* ring_count, float* next_weights, void* stream);

/*
 * Alg. 1 (weight-selection step) with the policy of App. B.2: push the distances of the
 * n_valid[b] verified positions of the finished block into the window, then
 * w = softmax((1 / max(e_j, eps)) / tau_w) with e_j the window sum (policy 0), or the candidate
 * [1-c/10, c/10] with the smallest window sum, lowest c on ties (policy 2).  An empty
 * window, or policy 1, gives equal weights.  Policy 3 ignores the window (but maintains it):
 * w_j = E_j / sum E with E_j = -ln U_j, U_j = (x + 0.5) 2^-24 from word j % 4 of the Philox block
 * (cfg->seed; round, b, gamma + 1 + j / 4).
 *
 *   round      the round (block) the weights are for: only policy 3 reads it
 *   dev        [B,gamma,DW] fp32 in     may be NULL together with n_valid (nothing to push)
 *   n_valid    [B]         int32 in
 *   ring       [B,h,DW]    fp32  in/out caller-owned window state (zero-initialised); with h = 0 it is
 *                                       [B,1,DW]: the running fp32 sum of all verified positions
 *   ring_head  [B]         int32 in/out next slot to overwrite
 *   ring_count [B]         int32 in/out live slots, <= h (h = 0: positions summed so far)
 *   weights    [B,n]       fp32  out
 */
int tabed_update_weights(const tabed_cfg* cfg, void* ws, uint64_t round, const float* dev, const int32_t* n_valid,
                         float* ring, int32_t* ring_head, int32_t* ring_count, float* weights,
                         void* stream);

/*
 * Draft-model body in front of the LM head (Sec. 5.1, "Ensemble learning via Batched Inference": the m drafting
 * methods share the parameters of the draft model and run as one batch; Sec. 4.1, "Target and Draft Models":
 * LLaMA-style drafts of 68M / 160M parameters).  One decode step for `rows` = n * B rows, each with its own
 * context: token embedding, then per layer RMSNorm, q/k/v projection, rotary position embedding (pairs
 * (i, i + head_dim/2)), attention over the row's own key / value cache, output projection, RMSNorm, SwiGLU MLP;
 * final RMSNorm.  The result H [rows,d] is what tabed_draft_step takes.  Weights, caches and every activation
 * that feeds a projection are bf16; the residual stream and the projections' results are fp32.  No trained
 * weights exist here: the body is exercised with random weights (parity with the oracle, and latency).
 *
 *   cfg, weights   HOST structs; the pointers inside `weights` are device pointers
 *   rows           <= 65535; row r = b * n + j as everywhere
 *   token_src, token_stride, rows_per_token: row r is fed token_src[(r / rows_per_token) * token_stride]
 *                  (in-block position i > 0: token_src = draft_tokens + i - 1, stride gamma, rows_per_token n;
 *                  a token outside [0,V) is clamped)
 *   ctx_len        [rows] int32 in/out  tokens already in the row's cache = position of the token fed now;
 *                  incremented by the call; must stay below cfg->max_ctx
 *   kcache, vcache [layers,rows,max_ctx,d] bf16 in/out  entry ctx_len[r] of every row and layer is written
 *   H              [rows,d] bf16 out
 * `ws` is scratch of tabed_body_workspace_bytes(cfg, rows) bytes prepared once by tabed_body_workspace_init.
 * Every pointer is 16-byte aligned (TABED_EALIGN otherwise); a ctx_len entry outside [0, max_ctx) is clamped into
 * the range, so nothing is written outside a row's cache.
 */
#define TABED_BODY_MAX_LAYERS 16
typedef struct tabed_body_cfg {
    int32_t layers;   /* 1..TABED_BODY_MAX_LAYERS                                   */
    int32_t d;        /* hidden size, multiple of 8, at most 8192                   */
    int32_t heads;    /* d / heads = head_dim, one of 8, 16, 32, 64, 128            */
    int32_t d_ff;     /* MLP width, multiple of 8                                   */
    int32_t V;        /* vocabulary of the embedding table                          */
    int32_t max_ctx;  /* cache length per row, 1..8192                              */
    float rope_theta; /* rotary base (10000)                                        */
    float rms_eps;    /* RMSNorm epsilon                                            */
} tabed_body_cfg;

typedef struct tabed_body_weights {
    const void* embed;                          /* [V,d] bf16                        */
    const float* g_final;                       /* [d]                               */
    const float* g_attn[TABED_BODY_MAX_LAYERS]; /* [d]                               */
    const void* wqkv[TABED_BODY_MAX_LAYERS];    /* [3d,d] bf16: q rows, k rows, v rows */
    const void* wo[TABED_BODY_MAX_LAYERS];      /* [d,d] bf16                        */
    const float* g_mlp[TABED_BODY_MAX_LAYERS];  /* [d]                               */
    const void* wgu[TABED_BODY_MAX_LAYERS];     /* [2*d_ff,d] bf16: gate rows, up rows */
    const void* wdown[TABED_BODY_MAX_LAYERS];   /* [d,d_ff] bf16                     */
} tabed_body_weights;

size_t tabed_body_workspace_bytes(const tabed_body_cfg* cfg, int32_t rows);   /* 0 if cfg is invalid */
int tabed_body_workspace_init(const tabed_body_cfg* cfg, int32_t rows, void* ws, void* stream);
int tabed_draft_body_step(const tabed_body_cfg* cfg, const tabed_body_weights* weights, void* ws, int32_t rows,
                          const int32_t* token_src, int32_t token_stride, int32_t rows_per_token,
                          int32_t* ctx_len, void* kcache, void* vcache, void* H, void* stream);
/*
 * After verification: the caches keep the fed tokens that were kept.  A round fed the round's first token and the
 * drafted tokens y_0 .. y_{gamma-2}; with k accepted, min(k + 1, gamma) of them stay:
 * ctx_len[r] = ctx_base[r] + min(accept_len[r / rows_per_seq] + 1, gamma).  (With k = gamma the last drafted
 * token has not been fed yet; the caller feeds it with one more tabed_draft_body_step.)
 */
int tabed_draft_body_rollback(int32_t rows, int32_t rows_per_seq, int32_t gamma, const int32_t* ctx_base,
                              const int32_t* accept_len, int32_t* ctx_len, void* stream);

/*
 * The uniforms the two calls above would draw: out[b,pos,word] for b < B,
 * pos <= gamma, word in {0,1}.  out is [B,gamma+1,2] fp32.
 */
int tabed_philox_uniforms(const tabed_cfg* cfg, uint64_t round, float* out, void* stream);

/*
 * Per-kernel timing.  While enabled, every kernel is launched with a start and a stop HIP event attached to
 * its dispatch (hipExtLaunchKernelGGL), so the pair brackets the kernel's own execution on the launch
 * stream; tabed_prof_read() waits for them and returns accumulated milliseconds and launch count of kernel
 * `id` (TABED_K_*), and keeps the totals until tabed_prof_reset().  Off by default; these calls create and
 * destroy events and synchronise, unlike the rest of the library.
 */
#define TABED_K_LMHEAD 0  /* LM-head GEMM + softmax partials    */
#define TABED_K_SAMPLE 1  /* ensemble + draft token             */
#define TABED_K_STATS 2   /* target statistics + distances + accept chain */
#define TABED_K_RESID 3   /* corrected / bonus token            */
#define TABED_K_WEIGHTS 4 /* window + weights                   */
#define TABED_K_DIST 5    /* second-pass distances (total variation, hard labels, grid mixtures) */
#define TABED_K_TREE 6    /* token tree: sibling 1's test (the later tree passes are not timed) */
#define TABED_K_BODY 7    /* draft-model body: every kernel of tabed_draft_body_step */
#define TABED_K_NULL 8    /* empty kernel, see tabed_prof_null  */
#define TABED_K_COUNT 9
int tabed_prof_enable(int on);
int tabed_prof_read(int id, double* total_ms, int64_t* launches);
int tabed_prof_reset(void);
const char* tabed_kernel_name(int id);
/* Launches an empty kernel on `stream`, timed like the others when timing is enabled: what
 * tabed_prof_read(TABED_K_NULL, ...) then reports is the floor of the method. */
int tabed_prof_null(void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TABED_H */
