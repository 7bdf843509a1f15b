/* skippipe.h - C boundary of the MI355X library for path-routed LLaMa stage training.
 *
 * The method (SkipPipe, sections "System Setting", "Partial pipeline schedule" and
 * "Guideline for Partial Pipelining Scheduler"): a model of L layers is cut into
 * s equal stages of consecutive layers; every microbatch of an iteration carries
 * a path, an ordered list of stage indices that opens with stage 0, and runs the
 * forward pass through exactly those stages, in that order.  A stage that is not
 * on the path is never applied, so the residual stream passes it unchanged.  The
 * loss is taken after the last stage of the path, the backward pass walks the
 * same stages in reverse, and the gradients of all microbatches are summed
 * before any update.
 *
 * Conventions
 *   - Every function returns 0 (SP_OK) or a negative sp_status; no exceptions and
 *     no C++ types cross this boundary.  sp_strerror() names a code; after
 *     SP_EHIP it also carries the HIP runtime's message.
 *   - Pointers are DEVICE pointers unless the parameter is marked "host".
 *   - All device work is enqueued on the HIP stream given to sp_create(); only
 *     sp_run_paths() waits for it (to hand back the loss).
 *   - The caller owns parameters, tokens, activation pools and gradients.  The
 *     library owns only what sp_create() allocated and frees it in sp_destroy().
 *   - Tensors are row-major, tokens-by-features.  A microbatch is seqs_per_mb
 *     sequences of seq_len tokens: N_mb = seqs_per_mb * seq_len rows.
 *   - dtype SP_F32: parameters and activations are float.  dtype SP_BF16:
 *     parameters and activations are bfloat16 (the caller's rounding of its
 *     float master copy); matrix products accumulate in float; norm statistics,
 *     softmax, log-sum-exp and the loss are float.  Gradients of parameters are
 *     float in both modes, in the parameter layout.
 *
 * Parameter layout (flat, element offsets from sp_param_layout):
 *   [embed vocab x dim]                                      if has_embed
 *   for each local stage, for each of its layers:
 *     g1 (dim) | wqkv ((dim + 2*dkv) x dim) | wo (dim x dim) |
 *     g2 (dim) | wgu (2*hidden x dim)       | wd (dim x hidden)
 *   [gf (dim)] [whead vocab x dim]                           if has_head
 *   Matrices are [out_features x in_features].  wqkv stacks query, key, value
 *   rows; wgu stacks gate rows then up rows.  dkv = n_kv_heads * (dim / n_heads).
 *   Query head a reads kv head a / (n_heads / n_kv_heads).  The rotary embedding
 *   turns the pair (2i, 2i+1) of every query and key head at position p of its
 *   sequence by p * rope_theta^(-2i/head_dim).
 */
#ifndef SKIPPIPE_H
#define SKIPPIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sp_status {
  SP_OK = 0,
  SP_EINVAL = -1, /* bad configuration, shape, index or null pointer */
  SP_EPATH = -2,  /* a path violates the constraints in force */
  SP_ENOMEM = -3, /* workspace exhausted or allocation failed */
  SP_EHIP = -4,   /* a HIP runtime call failed */
  SP_ESTATE = -5  /* call order: backward without the matching forward */
} sp_status;

enum { SP_F32 = 0, SP_BF16 = 1 };

/* path_flags */
enum {
  SP_STRICT_CC = 0,      /* stage 0 first, increasing order with at most one exchange of two
                            neighbouring entries whose stage indices differ by one */
  SP_SWAP_ANY_GAP = 1,   /* the two exchanged neighbours may be any two stages */
  SP_ALLOW_ANY_ORDER = 2 /* only: stage 0 first, no stage twice */
};

typedef struct sp_cfg {
  int32_t dim, n_heads, n_kv_heads, hidden, vocab;
  int32_t n_stages, layers_per_stage; /* equal stages of consecutive layers ("System Setting") */
  int32_t seq_len, seqs_per_mb;
  float rms_eps, rope_theta;
  int32_t dtype;                                /* SP_F32 | SP_BF16 */
  int32_t local_stage_begin, local_stage_count; /* stages whose weights this node holds */
  int32_t has_embed, has_head;                  /* token embedding / final norm + output head + loss held here */
  int32_t path_flags;
} sp_cfg;

typedef struct sp_tensor_desc {
  char name[32];        /* "embed", "s<stage>.l<layer>.wqkv", "gf", "whead", ... */
  int32_t stage, layer; /* -1 for tensors outside the stages */
  int64_t offset;       /* in elements from the start of the flat buffer */
  int64_t rows, cols;   /* vectors: rows = 1 */
} sp_tensor_desc;

typedef struct sp_ctx sp_ctx;

/* ---- host-only helpers (no GPU needed) ---------------------------------------------------------- */

/* Number of elements of the flat parameter (and gradient) buffer; negative sp_status on a bad cfg. */
int64_t sp_param_count(const sp_cfg* cfg);

/* Fills out[0..*n) with the tensors of the layout, in storage order.  cap = capacity of out (host);
 * if cap is too small only *n is set and SP_EINVAL is returned. */
int sp_param_layout(const sp_cfg* cfg, sp_tensor_desc* out, int cap, int* n);

/* Device bytes sp_create(cfg, ., n_mb_max, n_visits_max, .) will allocate. */
int64_t sp_workspace_bytes(const sp_cfg* cfg, int n_mb_max, int n_visits_max);

/* Seeded paths honouring the convergence constraints CC1-CC3 of "Guideline for Partial
 * Pipelining Scheduler" for a skip ratio k = skip_num / skip_den of the n_stages stages (stage 0
 * counts in the denominator and is never skipped; section "Allocating Nodes to Stages", Eq. 1).
 * Each path skips floor(s*k) or ceil(s*k) stages so that the total is round(n_mb*s*k); every stage
 * i >= 1 is skipped by the same number of paths up to one.  allow_swap: a path may get one
 * exchange of two neighbouring entries (strict form).  paths: host int32 [n_mb][n_stages], padded
 * with -1; len: host int32 [n_mb].  Returns SP_EINVAL if k leaves no stage besides stage 0. */
int sp_make_paths(int n_stages, int n_mb, int skip_num, int skip_den, int allow_swap, uint64_t seed,
                  int32_t* paths, int32_t* len);

/* Checks caller paths (host arrays as above) against the convergence constraints of "Guideline for
 * Partial Pipelining Scheduler" in the form cfg->path_flags selects: CC1 stage 0 first; CC2 the order rule
 * (increasing, at most one exchange of two neighbouring entries; the printed |i_j - i_j+1| <= 1 cannot hold
 * on a path with a skip and is read this way); plus what a path is by definition ("Partial and Reordered
 * Pipelining"): no stage twice, indices in range, length in [1, n_stages].  CC3 (every later stage skipped equally
 * often) is a property of a path set that sp_make_paths guarantees and this check does not demand of caller
 * paths.  SP_EPATH names the first violation through sp_strerror. */
int sp_check_paths(const sp_cfg* cfg, const int32_t* paths, const int32_t* len, int n_mb);

/* Route plan (section "Partial and Reordered Pipelining": several microbatches may share a path, and a
 * stage serves whoever arrives): for every path position pos and stage st, the microbatches with
 * paths[mb][pos]==st, restricted to local stages.  Groups are emitted by increasing pos, then stage; the forward pass
 * runs them in this order, the backward pass in reverse.  group_pos/group_stage/group_begin: host
 * int32 [cap_groups] (+1 for group_begin); group_mb: host int32 [n_mb*n_stages]. */
int sp_route_plan(const sp_cfg* cfg, const int32_t* paths, const int32_t* len, int n_mb, int32_t* group_pos,
                  int32_t* group_stage, int32_t* group_begin, int32_t* group_mb, int cap_groups, int* n_groups);

/* Nodes per stage by the node distribution rule (section "Allocating Nodes to Stages", Eq. 1): later stages
 * see only a share 1 - s/(s-1) k of the microbatches, so |S_i| = |S_0| (1 - s/(s-1) k) for i >= 1.  sizes: host
 * int32 [n_stages]; every node is used; the later stages get the nearest whole number, stage 0 the rest.
 * SP_EINVAL if fewer nodes than stages or the ratio leaves the later stages nothing. */
int sp_stage_sizes(int n_nodes, int n_stages, int skip_num, int skip_den, int32_t* sizes);

typedef struct sp_sched_problem {
  int32_t n_stages, n_nodes, n_agents;
  int32_t mem_limit;   /* m of TC1 */
  int32_t strict_swap; /* CC2: exchanged stages must be consecutive */
  int32_t no_swap;     /* != 0: stages strictly in increasing order (no exchange at all) */
  int32_t n_solutions, max_expansions;
  float delta;
  float focal_slack;   /* second phase: among solutions within this fraction of the cheapest, the one with the
                          fewest collisions is expanded next; 0 = strictly cheapest first (the paper); < 0 = 0.5 */
  const int32_t* node_stage;
  const float* compute_fwd;
  const float* compute_bwd;
  const float* comm;
  const int32_t* start_node;
  const int32_t* n_keep;
} sp_sched_problem;
/* Path scheduler (sections "Partial and Reordered Pipelining" and "Path finding", appendix "Detailed Path
 * Selection Algorithm"): for the first wave of microbatches (agents), which node of which stage each visits
 * and when, so that the slowest agent's end-to-end latency is small under the paper's constraints:
 *   CC1 an agent starts (and ends: the loss is taken there) on its node of stage 0;
 *   CC2 stages in increasing order with at most one exchange of two neighbouring stages (strict_swap != 0:
 *       the exchanged stages are consecutive stages of the model);
 *   CC3 every stage but the first is left out by the same number of agents, up to one;
 *   TC1 at most mem_limit paths through a node;  TC2 no two agents on one node at the same time (forward
 *       stays; links are full duplex and never conflict).
 * Conflict-based search: a best-first search per agent over (node, visited stages) with time as cost, and
 * a tree of per-agent "may not occupy node n during [t0, t1)" constraints above it, with the paper's greedy
 * rules (HR1: n_solutions solutions that honour CC1-CC3 are collected first, 32 if n_solutions <= 0; HR2: the
 * slowest quarter of the agents, and the slowest path through an over-full node, are never constrained; HR3:
 * of two colliding agents the faster one waits; if their latencies differ by less than delta both choices
 * are tried).  It is a
 * heuristic: the result is valid, not provably optimal.
 * All arrays are host arrays.  node_stage [n_nodes]; compute_fwd / compute_bwd [n_nodes]: seconds for one
 * microbatch; comm [n_nodes][n_nodes]: seconds to move one microbatch's activations from row to column node;
 * start_node [n_agents] (nodes of stage 0); n_keep [n_agents]: stages on the agent's path, stage 0 included
 * (s * (1 - k), rounded by the caller).  An agent's latency: forward stays and transfers, return to the
 * start node, then the backward pass along the reversed path without waiting (only the first forward pass
 * is scheduled, as in the paper).
 * Outputs (host): path_nodes, path_stages [n_agents][n_stages] padded with -1 (path_stages feeds
 * sp_run_paths / sp_check_paths); len [n_agents]; arrive [n_agents][n_stages] (start of each forward stay,
 * may be null); e2e [n_agents] and max_e2e (may be null).  SP_EPATH: no conflict-free solution found within
 * max_expansions (20000 if <= 0) constraint-tree expansions; SP_EINVAL: bad sizes, a start node outside
 * stage 0, a stage without nodes, negative times. */
int sp_schedule_paths(const sp_sched_problem* problem, int32_t* path_nodes, int32_t* path_stages, int32_t* len,
                      float* arrive, float* e2e, float* max_e2e);

const char* sp_strerror(int status);

/* ---- device ------------------------------------------------------------------------------------ */

/* Allocates the workspace on the current device: scratch for one group of up to n_mb_max
 * microbatches, saved activations for up to n_visits_max (stage, microbatch) visits alive at once,
 * and for a node holding embedding and head the two residual-stream pools sp_run_paths uses.
 * hip_stream: a hipStream_t (0 = the null stream).  Nothing else is allocated later. */
int sp_create(const sp_cfg* cfg, void* hip_stream, int n_mb_max, int n_visits_max, sp_ctx** out);
int sp_destroy(sp_ctx* ctx);

/* sp_stage_bwd (and sp_run_paths through it) runs the four weight-gradient products of a layer on a second
 * stream owned by the context, beside the chain that carries the activation gradient down the layers, and
 * joins that stream back into the caller's before it returns: for the caller all work is still ordered on
 * its own stream.  enabled = 1 (the default) does so for the groups it pays for: those whose R x d products
 * have fewer than 640 tiles of 256 x 256 (about 2.5 rounds of the 256 CUs), where the second stream fills
 * partly idle rounds; larger groups run in line, where two long products at once only disturb each other.
 * enabled = 2 uses the second stream for every group; enabled = 0 keeps everything in line on the caller's
 * stream (the per-launch timings of sp_prof_begin/end are then not inflated by kernels that share the GPU).
 * SP_EINVAL for other values.  Results differ between the settings only in the order of float additions. */
int sp_set_side_stream(sp_ctx* ctx, int enabled);

/* Forgets every saved forward (e.g. after an aborted iteration). */
int sp_reset(sp_ctx* ctx);

/* Token ids must lie in [0, vocab) and targets in [-1, vocab) (-1 = ignored).  The kernels check this on
 * the device and never read or write outside the caller's buffers: a row with a bad token id is embedded as
 * zeros and adds nothing to the embedding gradient, a bad target counts as ignored, and a flag inside ctx is
 * raised.  sp_run_paths and sp_eval_paths return SP_EINVAL when the flag is up at their end (their outputs
 * are then those of the inputs so repaired); after the asynchronous calls (sp_embed_fwd/bwd,
 * sp_head_fwd_bwd) sp_input_status() waits for the stream and reports the same way.  Reading the flag clears it. */
int sp_input_status(sp_ctx* ctx);

/* x[row, :] = embed[token[row], :] for n_mb microbatches (the front of stage 0, which every path opens
 * with: constraint CC1 of "Guideline for Partial Pipelining Scheduler").
 * tokens: int32 [n_mb * N_mb]; act_pool: [n_mb][N_mb][dim] in cfg->dtype. */
int sp_embed_fwd(sp_ctx* ctx, const void* params, const int32_t* tokens, int n_mb, void* act_pool);
/* grads[embed][token[row], :] += dact[row, :]. */
int sp_embed_bwd(sp_ctx* ctx, const int32_t* tokens, const void* dact_pool, int n_mb, float* grads);

/* Section "Partial pipeline schedule": a microbatch runs only the stages on its path; a stage is a run of
 * consecutive LLaMa decoder layers ("System Setting"; appendix "Model Configurations").
 * Forward of local stage `stage` (global index) for the group of microbatches mb_idx[0..n_group)
 * (host int32, distinct slot numbers of act_pool), in place on their slots; every other slot is
 * untouched (that is the skip).  The layers' intermediate results are kept inside ctx, keyed by
 * (stage, group), until the matching sp_stage_bwd. */
int sp_stage_fwd(sp_ctx* ctx, int stage, const void* params, void* act_pool, const int32_t* mb_idx, int n_group);

/* The backward pass visits the same stages in reverse ("Partial pipeline schedule"); gradients of all
 * microbatches are summed before any update ("System Setting").
 * Backward of the same group (same stage, same mb_idx in the same order; SP_ESTATE otherwise):
 * dact_pool slots hold dL/d(output) on entry and dL/d(input) on return; parameter gradients are
 * added into grads (float, parameter layout) with float atomics. */
int sp_stage_bwd(sp_ctx* ctx, int stage, const void* params, void* dact_pool, const int32_t* mb_idx, int n_group,
                 float* grads);

/* The loss is taken where the path closes, on stage 0's node ("Allocating Nodes to Stages": closed loop).
 * Final norm, output head and next-token cross-entropy for all n_mb microbatches, forward and
 * backward at once: loss_mb[mb] = mean over the targets >= 0 of microbatch mb; the iteration loss
 * is their mean, so dact_pool receives d(mean)/d(act) = d(loss_mb)/d(act) / n_mb.  targets: int32
 * [n_mb * N_mb], -1 = ignored.  loss_mb: device float [n_mb].  grads: += for gf and whead. */
int sp_head_fwd_bwd(sp_ctx* ctx, const void* params, const void* act_pool, const int32_t* targets, int n_mb,
                    float* loss_mb, void* dact_pool, float* grads);

/* One iteration of partial pipelining with every stage on this node ("Partial pipeline schedule").
 * Whole model on this node (all stages local, embedding and head held): embeds, walks the route
 * plan of the given paths (host arrays, checked against cfg->path_flags), takes the loss, walks
 * the plan backwards, and returns the iteration loss.  grads is zeroed by the call.  loss_host:
 * host float[1]; loss_mb_host: host float [n_mb] or NULL.  Waits for the stream. */
int sp_run_paths(sp_ctx* ctx, const void* params, const int32_t* tokens, const int32_t* targets,
                 const int32_t* paths, const int32_t* len, int n_mb, float* loss_host, float* loss_mb_host,
                 float* grads);

/* Matrix products used by the stages (the projections of the decoder layer and their gradients), exposed
 * for unit tests and roofline measurement.
 *   op 0: C[M,N]  = A[M,K] * B[N,K]^T  (+ R[M,N] if R != NULL)      C, R in cfg dtype
 *   op 1: C[M,N]  = A[M,K] * B[K,N]                                  C in cfg dtype
 *   op 2: C[M,N] += A[K,M]^T * B[K,N]                                C float
 * A, B in dtype (SP_F32 / SP_BF16), row-major, dense leading dimensions. */
int sp_gemm(void* hip_stream, int dtype, int op, int M, int N, int K, const void* A, const void* B, void* C,
            const void* R);

/* The two feed-forward steps whose pointwise part rides in a matrix product's epilogue (the SwiGLU block of the
 * decoder layer: act = silu(gate) * up with [gate | up] = hn wgu^T, and its gradient), exposed for unit tests.
 *   sp_ffn_up_fwd:   gu[R, 2h] = hn[R, d] * wgu[2h, d]^T  and  act[R, h] = silu(gu[:, :h]) * gu[:, h:]
 *   sp_ffn_down_bwd: dgu[R, 2h] = d(gate) | d(up) for d(act) = dy[R, d] * wd[d, h] and the saved gu;
 *                    da_scratch [R, h] is used only where the fused kernel does not apply (float, odd shapes)
 * All tensors in dtype, row-major, dense. */
int sp_ffn_up_fwd(void* hip_stream, int dtype, int R, int h, int d, const void* hn, const void* wgu, void* gu, void* act);
int sp_ffn_down_bwd(void* hip_stream, int dtype, int R, int h, int d, const void* dy, const void* wd, const void* gu,
                    void* dgu, void* da_scratch);

/* Causal softmax attention with grouped kv heads as used by the stages (per sequence and head:
 * softmax(q k^T / sqrt(hd) + causal mask) v, and its gradients), exposed for unit tests and roofline
 * measurement.
 * qkv: [B*T][(H + 2*Hkv)*hd] rows of query|key|value; o: [B*T][H*hd]; lse: float [B][H][T].
 * Backward: do_ like o; dqkv like qkv (overwritten). */
int sp_attention_fwd(void* hip_stream, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o,
                     float* lse);
int sp_attention_bwd(void* hip_stream, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv,
                     const void* o, const float* lse, const void* do_, void* dqkv, float* delta_scratch);

/* Forward-only evaluation under stage drops (section "Fault Tolerant Inference"): every microbatch (sample)
 * runs the stages of its path, stage 0 always among them; the number of stages may differ between samples.
 * half_stage (host, int32[n_mb], may be null; entries -1 = none): the one stage of a sample's path that
 * executes only the first layers_per_stage / 2 of its layers (the paper's partial stage skip for skip ratios
 * that do not divide the stage count; "the first half" of an odd count is read as rounded down).  It must be
 * on the path, must not be stage 0, and needs layers_per_stage >= 2 (SP_EPATH otherwise).  Paths are checked
 * as in sp_check_paths except for equal lengths.  Needs the whole model on this node.  Nothing is kept for a
 * backward pass.  loss_host (host, 1 float): mean over microbatches of the mean loss over non-ignored
 * targets; loss_mb_host (host, n_mb floats, may be null): each microbatch's own; perplexity is exp(loss).
 * Waits for the stream. */
int sp_eval_paths(sp_ctx* ctx, const void* params, const int32_t* tokens, const int32_t* targets, const int32_t* paths,
                  const int32_t* len, const int32_t* half_stage, int n_mb, float* loss_host, float* loss_mb_host);

/* The update that closes an iteration (appendix "Test Configurations": learning rate 3e-4, gradient norms
 * clipped to 1.0; the paper does not name the optimiser, this library's reading is AdamW):
 *   g <- g * min(1, clip_norm / (||g||_2 + 1e-6))      one norm over all n gradients; clip_norm 0 = off
 *   m <- beta1 m + (1 - beta1) g ;  v <- beta2 v + (1 - beta2) g^2
 *   p <- p (1 - lr weight_decay) - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * master, m, v (float, n elements, updated in place) and grads (float, read only; e.g. what sp_run_paths or
 * sp_stage_bwd accumulated) are device pointers, 16-byte aligned, owned by the caller.  params_out, if not
 * null (16-byte aligned), receives the new parameters rounded to out_dtype (SP_BF16 or SP_F32): the copy the next iteration's
 * kernels read.  workspace: sp_optim_workspace_bytes() bytes of device memory, 16-byte aligned, contents
 * irrelevant before and after.  grad_norm (device, 1 float, may be null) receives the norm before clipping.
 * step counts from 1.  Work is enqueued on hip_stream and not waited for.  The sum of squares is formed in
 * a fixed order in double, so the result is reproducible.  SP_EINVAL: null or misaligned pointers, step < 1,
 * hyper-parameters out of range (lr, eps, weight_decay, clip_norm < 0; beta outside [0, 1)). */
typedef struct sp_adamw {
  float lr, beta1, beta2, eps, weight_decay, clip_norm;
} sp_adamw;
int64_t sp_optim_workspace_bytes(void);
int sp_optim_step(void* hip_stream, const sp_adamw* hyper, int64_t n, int step, float* master, const float* grads,
                  float* m, float* v, void* params_out, int out_dtype, void* workspace, float* grad_norm);

/* sp_optim_step for callers that cannot allocate or pass a workspace: code under HIP graph capture, tight
 * serving / training loops, harnesses that forbid hipMalloc.  Same arguments without `workspace`, same kernels,
 * same results bit for bit.  The norm partials and clip factor (16 640 bytes) live in a static device array of
 * the library instead; every GPU the library runs on holds its own copy until the process ends.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine); the array's address on the
 * current device is looked up on the first call on that device.  Nothing in the array has to start at zero
 * (every partial that is read was written by the same call).  All calls on one GPU share the array: two calls
 * that overlap in time on one GPU (different streams, different threads) race and give wrong norms; calls on one
 * stream, or otherwise ordered, are fine.  SP_EINVAL also if n exceeds 2^32 elements. */
int sp_optim_step_noalloc(void* hip_stream, const sp_adamw* hyper, int64_t n, int step, float* master,
                          const float* grads, float* m, float* v, void* params_out, int out_dtype, float* grad_norm);

/* Gradient accumulation across the replicas of an iteration (section "Throughput": gradients of all
 * microbatches are accumulated before the update; with several nodes per stage each node holds the sum over
 * the microbatches it served): out[i] = scale * sum_r replica_grads[r][i], added in replica order.
 * replica_grads: host array of n_replicas (1..64) device pointers to float buffers of n elements; out: device
 * float [n] (may be one of the replica buffers); all 16-byte aligned.  scale: e.g. 1 / n_mb when every
 * head call took one microbatch's loss alone.  Enqueued on hip_stream, not waited for. */
int sp_grad_reduce(void* hip_stream, const float* const* replica_grads, int n_replicas, int64_t n, float scale,
                   float* out);

/* Measurement aid: between sp_prof_begin() and sp_prof_end() every matrix-product and attention
 * launch of this process is bracketed by HIP events on its stream.  sp_prof_end waits for them and
 * fills, per kernel class c < n_classes, the summed duration (ms), the summed algorithmic flops
 * and the launch count (host arrays).  Classes: 0 C=A B^T, 1 C=A B, 2 C+=A^T B (MFMA kernels),
 * 3 attention forward, 4 attention delta (see below), 5 attention dQ, 6 attention dK/dV, 7 plain matrix
 * product, 8 plain attention; and the bandwidth-bound kernels, whose "flops" entry holds algorithmic
 * BYTES instead: 4 attention delta (rows of o and dO read, one float per row and head written), 9 RMSNorm
 * forward, 10 RMSNorm backward, 11 cross-entropy, 12 slot gather / scatter, 13 SwiGLU as a pass of its own
 * (float mode, odd shapes). */
int sp_prof_begin(void);
int sp_prof_end(int n_classes, double* ms, double* flops, int64_t* launches);

/* Measurement aid: what the matrix cores sustain with nothing else going on.  Launches n_blocks (1..65536)
 * workgroups of 8 waves; every wave loads the 24 bf16 operand fragments of one 256 x 256 x 64 k-step of the
 * product kernels from src (device, 16-byte aligned, src_bytes >= 16 bytes of bf16 values of the caller's
 * choice, read modulo its size) and repeats that step's 64 v_mfma_f32_16x16x32_bf16 `iters` times with the
 * fragments held in registers.  sink: device float [n_blocks * 512], overwritten.  *flops (host) receives
 * the multiply-add flops of the launch; the caller times the launch on hip_stream.  Enqueued, not waited for.
 * Used to separate the chip's clock / power ceiling for a given operand content from what a kernel loses to
 * memory traffic and epilogues. */
int sp_probe_mfma_rate(void* hip_stream, const void* src, int64_t src_bytes, int n_blocks, int iters, float* sink,
                       double* flops);

#ifdef __cplusplus
}
#endif
#endif /* SKIPPIPE_H */
