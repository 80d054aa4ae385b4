/*
 * umas.h - C ABI of libumas: the model-local worker step of UnityMAS-O on one gfx950 GPU.
 *
 * Four calls follow the paper's statement of the problem (logical roles V, the
 * agent-to-model map phi: V -> M, trajectories with reward signals at role, turn and
 * trajectory level, model-local buffers B_i and PPO-style per-model updates):
 *
 *   umas_assign_token_rewards  reward composition, routing through phi, placement on tokens
 *   umas_advantages            GAE as a masked, segmented reverse scan
 *   umas_policy_logprobs       LM-head scoring: log-prob of the taken token, logsumexp, entropy
 *   umas_ppo_loss_fwd_bwd      scoring + clipped surrogate + backward to hidden states and weights
 *
 * Conventions
 *   - THIN metadata (graph, reward scalars) are HOST pointers, caller-owned, read during the
 *     call only (the paper's controller keeps exactly this: role ids, routing ids, reward
 *     metadata).  FAT tensors (masks, rewards per token, hidden states, weights, outputs,
 *     workspace) are DEVICE pointers, caller-allocated; the library owns no device memory
 *     besides the static scratch of umas_policy_logprobs_static.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default
 *     stream).  No call waits for the stream.  umas_assign_token_rewards and umas_ready_batch
 *     gather their thin host arrays in a block of pinned host memory that the library keeps (a
 *     ring of four blocks, each as large as the largest graph it has seen) and enqueue one
 *     asynchronous copy of it: the caller may free or overwrite its arrays on return, and the
 *     host can queue the next step while this one runs.  The one wait there is: a block is
 *     reused four such calls later, after the copy that was issued from it has run.  Results,
 *     including loss statistics, stay on the device.  Every other call only launches kernels
 *     (memory is cleared by fill kernels, never by memset nodes), so it may be recorded into a
 *     HIP graph as long as profiling (umas_profile_enable) is off.
 *   - Every call returns a umas_status.  Argument errors are found on the host before any
 *     launch, leave outputs untouched and set a thread-local message (umas_last_error).
 *     What the host can see is checked: scalars, host arrays, pointers and their alignment.
 *     The contents of DEVICE arrays are the caller's responsibility: a token id outside [0,V)
 *     is tolerated (counted, the row contributes nothing) and so is a role outside
 *     [0, n_roles) (the row or token joins no per-role statistic), but an entry of a row
 *     selection outside [0, n_rows), or streams that do not come from
 *     umas_assign_token_rewards, make kernels read or write out of bounds.
 *   - Workspace sizes come from the umas_*_workspace_bytes queries; workspace must be
 *     256-byte aligned.  Passing less than the required size returns UMAS_EWORKSPACE.
 *   - One GPU, one process; calls on different streams may run concurrently only with
 *     disjoint outputs and workspaces.  Some kernels of umas_assign_token_rewards,
 *     umas_ready_batch and umas_advantages have workgroups that wait for words published by
 *     their other workgroups; their grids are at most half of what the device holds at once (a
 *     quarter with four models or fewer), so two such calls fit side by side (three or four with
 *     four models or fewer).  Do not run more of them concurrently when each carries more than
 *     65536 trajectories (or segments of more than 16384 tokens).
 */
#ifndef UMAS_H
#define UMAS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  UMAS_OK = 0,
  UMAS_EINVAL = -1,     /* NULL required pointer, value out of range, malformed graph */
  UMAS_ESHAPE = -2,     /* size not supported (d not a multiple of 8 for bf16, too many models, ...) */
  UMAS_EDTYPE = -3,     /* unknown umas_dtype */
  UMAS_EWORKSPACE = -4, /* workspace NULL, misaligned or too small */
  UMAS_EHIP = -5        /* a HIP runtime call failed (message carries hipGetErrorString) */
} umas_status;

typedef enum { UMAS_F32 = 0, UMAS_BF16 = 1 } umas_dtype;

enum { UMAS_PLACE_LAST = 0, UMAS_PLACE_ALL = 1 };
enum { UMAS_SEG_TURN = 0, UMAS_SEG_TRAJ = 1 };
enum { UMAS_MAX_MODELS = 8, UMAS_MAX_ROLES = 64 };

/* Message of the last failing call on this thread; static storage, never freed by the caller. */
const char* umas_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Thin inputs (HOST pointers).
 * The executed workflow of every trajectory in its linearised view (s_0,k_1,a_1,...,k_T,a_T)
 * (Section "Workflow Graphs and Execution"): turn = one role invocation, turns of a trajectory
 * are consecutive and in linearised order, tokens of a turn are consecutive in the global
 * token order.  The predecessor CSR carries the control-flow record C of the trajectory; it is
 * validated (same trajectory, earlier turn) and not used by the arithmetic, which follows the
 * linearised order as the paper's objective does.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n_roles;              /* |V| <= UMAS_MAX_ROLES */
  int32_t n_models;             /* |M| <= UMAS_MAX_MODELS */
  int32_t n_traj;
  int32_t n_turns;
  int64_t n_tokens;
  const int32_t* role_to_model; /* [n_roles]    phi (Section "Agent--LLM Mapping") */
  const int32_t* traj_turn_off; /* [n_traj+1]   CSR: turns of trajectory b */
  const int32_t* turn_role;     /* [n_turns]    active role k_t of each turn */
  const int64_t* turn_tok_off;  /* [n_turns+1]  CSR: tokens of turn u in the global token order */
  const int32_t* turn_pred_off; /* [n_turns+1]  CSR of predecessor turns, or NULL = chain */
  const int32_t* turn_pred;     /* [turn_pred_off[n_turns]] global turn ids, or NULL */
  const int32_t* traj_group;    /* [n_traj] group id >= 0 for reward normalisation, or NULL = none */
} umas_graph;

/* Reward scalars at the three levels of the reward interface and the optional weights of
 * r_v = lam_node r_node + lam_turn r_turn + lam_traj r_traj (Section "Agent-Specific Reward
 * Interface").  NULL level = 0, NULL weight = 1.  With traj_group the trajectory-level
 * reward is z-scored inside each group first: (R - mean) / (population std + norm_eps). */
typedef struct {
  const float* role_reward;     /* [n_traj*n_roles] one scalar per (trajectory, role), or NULL */
  const float* turn_reward;     /* [n_turns]        one scalar per invocation, or NULL */
  const float* traj_reward;     /* [n_traj]         one scalar per trajectory, or NULL */
  const float* w_role;          /* [n_roles] or NULL */
  const float* w_turn;          /* [n_roles] or NULL */
  const float* w_traj;          /* [n_roles] or NULL */
  int32_t place_mode;           /* UMAS_PLACE_LAST: last mask=1 token of the turn; UMAS_PLACE_ALL: every mask=1 token */
  float norm_eps;               /* > 0 */
} umas_rewards;

/* ------------------------------------------------------------------------------------------
 * Model-local streams (DEVICE pointers, caller-allocated, all written by
 * umas_assign_token_rewards).  Stream m is the buffer B_m of the model-local worker group
 * (Section "Model-Local Buffers"): tokens of all turns with phi(role) = m, turns in ascending
 * global id, streams stored back to back.  "model-local order" below means this order.
 * The arrays of n_tokens entries must be 16-byte aligned (rowsel 4-byte); a stream holds at most
 * 2^31 - 1 tokens (UMAS_ESHAPE otherwise), n_tokens as a whole may be larger.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int64_t* model_tok_off;     /* [n_models+1]  stream m = positions [off[m], off[m+1]) */
  int64_t* perm;              /* [n_tokens]    model-local position -> global token index */
  int32_t* tok_turn;          /* [n_tokens]    global turn id of each token */
  int32_t* tok_role;          /* [n_tokens]    role id (kept under sharing for role-level reporting) */
  uint8_t* tok_mask;          /* [n_tokens]    mask gathered into model-local order */
  float*   tok_reward;        /* [n_tokens]    reward placed on tokens */
  int64_t* turn_seg_off;      /* [n_turns+1]   token offsets of the turn segments, grouped by model */
  int32_t* seg_turn;          /* [n_turns]     global turn id of turn segment s */
  int32_t* model_turn_off;    /* [n_models+1]  turn segments of model m */
  int64_t* traj_seg_off;      /* [n_turns+1]   token offsets of trajectory runs (maximal runs of one
                                               trajectory inside a stream); entries past the count are n_tokens */
  int32_t* model_trajrun_off; /* [n_models+1]  trajectory runs of model m; [n_models] = their number */
  int32_t* rowsel;            /* [n_tokens]    per model, ascending stream-relative positions with mask=1 */
  int64_t* model_rowsel_off;  /* [n_models+1]  rowsel of model m = [off[m], off[m+1]) */
  float*   turn_scalar;       /* [n_turns]     composed reward of each turn, global turn order */
  int32_t* turn_step;         /* [n_turns]     1-based position of the turn inside its trajectory */
  uint8_t* tok_flags;         /* [n_tokens]    bit 0 = mask, bit 1 = last token of its turn segment,
                                               bit 2 = last token of its trajectory run; on a turn's last token that
                                               does not end the run, bits 3-7 = steps from this turn to the run's next
                                               turn with tokens (31 = more than 30: take the difference of turn_step);
                                               read by umas_advantages */
} umas_streams;

/* Bytes of workspace umas_assign_token_rewards needs for this graph. */
size_t umas_assign_workspace_bytes(const umas_graph* graph);

/* Steps a1-a3: compose per-turn rewards, normalise, route through phi, place on tokens
 * (Sections "Agent-Specific Reward Interface", "Model-Local Buffers", paragraphs "Reward
 * assembly and commitment" and "Batch construction").
 *   tok_mask_global  DEVICE uint8 [n_tokens], global token order, 1 = action token
 *   out              HOST struct of DEVICE pointers, all non-NULL
 * Errors (nothing launched): NULL pointers, non-monotone CSR, role or phi out of range,
 * predecessor outside the trajectory or not earlier, negative group id, bad place_mode. */
umas_status umas_assign_token_rewards(const umas_graph* graph, const umas_rewards* rewards,
                                      const uint8_t* tok_mask_global, const umas_streams* out,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

size_t umas_advantages_workspace_bytes(int64_t n_tokens);

/* Step a4: A_t = sum_l (gamma lam)^l delta_{t+l}, delta_t = r_t + gamma V(s_{t+1}) - V(s_t)
 * (paragraph "Advantage computation and policy evaluation") as a masked, segmented reverse
 * scan over the model-local streams.  Segments: turns (UMAS_SEG_TURN) or trajectory runs
 * (UMAS_SEG_TRAJ); V and A past a segment end are 0; mask=0 tokens are skipped by the
 * recurrence and output 0.  In UMAS_SEG_TRAJ the carried state is multiplied by
 * gamma_turn^(step difference) when the scan crosses a turn boundary, which reproduces the
 * objective's gamma^(t-1) discount over role invocations.
 *   value  DEVICE float [n_tokens] in model-local order, or NULL (= 0)
 *   adv, ret  DEVICE float [n_tokens]; ret = adv + value at mask=1 tokens */
umas_status umas_advantages(const umas_streams* streams, int64_t n_tokens, int32_t n_turns,
                            const float* value, float gamma, float lam, float gamma_turn,
                            int32_t seg_mode, float* adv, float* ret,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

size_t umas_policy_logprobs_workspace_bytes(int64_t n_sel, int32_t d, int32_t V, umas_dtype dtype);

/* Step a5: for each selected row i, z = W h_i (float accumulate), lse = log sum_v exp z_v,
 * logp = z[ids[i]] - lse, entropy = lse - sum_v softmax(z)_v z_v ("old log probabilities",
 * paragraph "Advantage computation and policy evaluation").  Logits are never written out.
 *   H       DEVICE [n_rows, d] row-major, dtype;  W  DEVICE [V, d] row-major, dtype
 *   ids     DEVICE int32 [n_rows]; a row whose id is outside [0,V) gets logp = entropy = 0
 *   rowsel  DEVICE int32 [n_sel] rows to score, distinct, each in [0, n_rows), in any order (ascending as
 *           umas_assign_token_rewards writes them, or a part of a ready batch); NULL with n_sel = n_rows = all
 *   logp, lse, entropy  DEVICE float [n_rows]; rows not selected are set to 0; entropy may be NULL
 * bf16 needs d % 8 == 0. */
umas_status umas_policy_logprobs(const void* H, const void* W, umas_dtype dtype, int64_t n_rows,
                                 int32_t d, int32_t V, const int32_t* ids, const int32_t* rowsel,
                                 int64_t n_sel, float* logp, float* lse, float* entropy,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same scoring for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  No workspace argument and no allocation of any kind inside the call
 * (no hipMalloc, no hipFree, no host allocation): the per-tile partials that umas_policy_logprobs keeps in
 * its workspace go to a device array of UMAS_STATIC_SCRATCH_BYTES that is part of the library's code object;
 * each GPU the library runs on holds its own copy until the process ends.  Same arguments, outputs, kernels
 * and results as umas_policy_logprobs.
 *   limit   umas_policy_logprobs_workspace_bytes(n_sel, d, V, dtype) <= UMAS_STATIC_SCRATCH_BYTES, i.e. for bf16
 *           ceil(V / 256) * roundup(n_sel, 256) * 16 bytes: 3328 selected rows per call at V = 151936;
 *           float32 needs no scratch.  More returns UMAS_EWORKSPACE, nothing launched.
 *   sharing every call on one GPU uses that GPU's one array: calls that overlap on a GPU (two streams, two
 *           threads) race; calls on one stream are ordered and safe.  Nothing in the array carries over
 *           between calls (each call overwrites what it reads).
 *   set-up  the first call on a device (with that device current) looks the array's address up once; make that
 *           call outside graph capture. */
#define UMAS_STATIC_SCRATCH_BYTES (32u << 20)
umas_status umas_policy_logprobs_static(const void* H, const void* W, umas_dtype dtype, int64_t n_rows,
                                        int32_t d, int32_t V, const int32_t* ids, const int32_t* rowsel,
                                        int64_t n_sel, float* logp, float* lse, float* entropy, void* hip_stream);

/* Row 0: the model's totals; rows 1..n_roles: the same numbers over the rows of one role. */
typedef struct {
  float loss;              /* mean over scored rows of max(-A ratio, -A clip(ratio, 1-eps, 1+eps)) */
  float clip_frac;         /* share of scored rows whose clipped term is strictly larger */
  float entropy_mean;
  float approx_kl;         /* mean of logp_old - logp */
  int64_t n_scored;        /* rows in the mean (selected rows; rows with invalid ids add 0 to the sums) */
  int64_t n_invalid_ids;   /* selected rows whose token id is outside [0,V) */
} umas_loss_stats;

/* Smallest workspace the call accepts and the size at which it runs in the fewest passes.  For bf16 the
 * workspace holds, per chunk of selected rows, the bf16 operand of the two gradient products
 * [rows, V] (rounded up to multiples of 256) and a scaled bf16 copy of the chunk's rows of H; the
 * smallest size runs in chunks of 256 rows, the full size in chunks of up to 131072 rows. */
size_t umas_ppo_loss_workspace_bytes_min(int64_t n_sel, int32_t d, int32_t V, umas_dtype dtype, int32_t n_roles);
size_t umas_ppo_loss_workspace_bytes(int64_t n_sel, int32_t d, int32_t V, umas_dtype dtype, int32_t n_roles);

/* Steps a5-a7 for one model's stream (each worker group updates its own model, paragraph
 * "Model-specific updates and synchronization"): scoring as above, then the single-clip PPO
 * surrogate (PPO-style loop after Schulman et al. 2017) with the token mean over the n_sel
 * selected rows as loss, then the backward through the LM head:
 *   ratio = exp(logp - logp_old); L = max(-A ratio, -A clip(ratio, 1-eps, 1+eps))
 *   g = dloss/dlogp;  dz_iv = g_i (1[v = ids[i]] - softmax(z_i)_v);  dH = dz W;  dW = dz^T H
 *   logp_old, adv  DEVICE float [n_rows]; logp_old = NULL: the update is on-policy, logp_old is taken to be the
 *                  log-probs this call computes (ratio 1 on every row: L = -A, g = -A / n_sel, approx_kl = 0), which
 *                  saves the separate umas_policy_logprobs pass of the first update after a rollout
 *   tok_role       DEVICE int32 [n_rows] or NULL with n_roles = 0
 *   stats          DEVICE umas_loss_stats [1 + n_roles]
 *   logp_new       DEVICE float [n_rows] or NULL
 *   dH             DEVICE [n_rows, d] in the dtype of H; rows not selected are set to 0
 *   dW             DEVICE float [V, d]; accumulate_dW = 0 overwrites, 1 adds
 * clip_eps must lie in (0,1).
 * Optional terms (stabilisers of the PPO family; all off at 0):
 *   dual_clip c > 1: for A < 0 the row's term is capped at -A c, with no gradient where the cap binds;
 *   entropy_coef k >= 0: the loss becomes L_clip - k mean entropy (stats.loss includes it) and
 *     dz_iv gains (k / n_sel) p_iv (log p_iv + entropy_i), p = softmax(z_i).
 *   kl_coef b >= 0 with logp_ref DEVICE float [n_rows] (NULL when b = 0): the loss gains b times the mean over the
 *     scored rows of e^x - x - 1, x = logp_ref - logp (the non-negative estimate of KL(pi || pi_ref) whose mean over
 *     tokens drawn from pi is that divergence), and g gains b (1 - e^x) / n_sel.  The penalty may instead be folded into
 *     the rewards (umas_kl_rewards).  With b > 0 every scored row has a gradient.
 * norm_rows: 0, or the number of rows the token mean is taken over when the call is one micro-batch of a
 *   minibatch of norm_rows >= n_sel scored rows (gradient accumulation over the parts of a ready batch, paragraph
 *   "Model-specific updates and synchronization"): g, the entropy term and stats[0].loss are divided by it in
 *   place of n_sel, so that the micro-batches' dW (accumulate_dW = 1), dH rows and losses add up to those of one
 *   call on the whole minibatch.  The roles' rows of stats and the other fields stay means over the call's rows.
 * What the bf16 update keeps in memory, stated plainly: for every chunk of selected rows it WRITES one bf16 number
 * per (row, vocabulary entry) pair to the workspace and the two gradient products read that [rows, V] matrix back
 * (2 * rows * V bytes: 11.9 GB for 39 224 rows against V = 151 936 in one chunk).  With entropy_coef = 0 the
 * matrix holds the softmax numerators exp(z - z_y), written by the scoring pass itself, so the logits are computed
 * once; with an entropy bonus it holds dz, written by a second pass over the logits.  The float32 logits are
 * never stored, but a [rows, V] operand does pass through HBM; only umas_policy_logprobs keeps everything of that
 * shape on chip.  The workspace bounds it: the call works in chunks of as many rows as the workspace holds (256
 * at the least), at the price of one more pass over W per chunk.  The float32 path stores float32 dz per chunk. */
umas_status umas_ppo_loss_fwd_bwd(const void* H, const void* W, umas_dtype dtype, int64_t n_rows,
                                  int32_t d, int32_t V, const int32_t* ids, const int32_t* rowsel,
                                  int64_t n_sel, const float* logp_old, const float* adv,
                                  const int32_t* tok_role, int32_t n_roles, float clip_eps,
                                  float entropy_coef, float dual_clip, int32_t accumulate_dW, int64_t norm_rows,
                                  const float* logp_ref, float kl_coef, umas_loss_stats* stats,
                                  float* logp_new, void* dH, float* dW,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Critic.  The worker groups compute "value estimates" next to the log-probs and update "actor and
 * critic parameters" from the ready batch (Section "PPO-Style Training Loop", paragraphs "Advantage
 * computation and policy evaluation" and "Model-specific updates and synchronization").  The paper
 * prints no value loss; the clipped form that goes with PPO is taken:
 *   V_i = w . h_i + bias
 *   Vc = clip(V, V_old - eps, V_old + eps);  L = 1/2 max((V - R)^2, (Vc - R)^2);  loss = mean L
 *   g = dloss/dV = (V - R) / n_sel where the unclipped term is the larger one (ties included), else 0
 *   dH_i = g_i w;  dw = sum_i g_i h_i;  db = sum_i g_i
 * H [n_rows, d] and w [d] are DEVICE arrays of `dtype`, 16-byte aligned; d is a multiple of 8 (bf16) or
 * 4 (float32) and at most 8192 (bf16) or 4096 (float32); rowsel / n_sel select rows as in umas_policy_logprobs. */
typedef struct umas_value_stats {
  float loss;         /* mean over the rows of 1/2 max((V-R)^2, (Vc-R)^2) */
  float clip_frac;    /* rows whose clipped term is strictly larger */
  float value_mean;   /* mean V */
  float reserved;
  int64_t n_scored;   /* rows in the means */
} umas_value_stats;

/* value DEVICE float [n_rows]: V on the selected rows, 0 elsewhere.  Needs no workspace. */
umas_status umas_values(const void* H, const void* w, float bias, umas_dtype dtype, int64_t n_rows, int32_t d,
                        const int32_t* rowsel, int64_t n_sel, float* value, void* hip_stream);

size_t umas_value_workspace_bytes(int64_t n_sel, int32_t d, umas_dtype dtype, int32_t n_roles);

/* One pass over the selected rows of H: value head, clipped value loss, backward.
 *   value_old, ret  DEVICE float [n_rows] (the returns are umas_advantages' `ret`)
 *   tok_role        DEVICE int32 [n_rows] or NULL with n_roles = 0
 *   stats           DEVICE umas_value_stats [1 + n_roles]: the model, then each role
 *   value_new       DEVICE float [n_rows] or NULL
 *   dH              DEVICE [n_rows, d] in the dtype of H; accumulate_dH = 0 writes g_i w on the selected rows
 *                   and 0 elsewhere, 1 adds g_i w to the selected rows and leaves the others alone (a trunk
 *                   shared with the policy head)
 *   dw, db          DEVICE float [d], [1] (db may be NULL); accumulate_dw = 0 overwrites, 1 adds
 *   norm_rows       0, or the row count the mean is taken over (>= n_sel), as in umas_ppo_loss_fwd_bwd
 * clip_eps_v must be positive.  The result does not depend on scheduling: partial sums are reduced in a
 * fixed order. */
umas_status umas_value_loss_fwd_bwd(const void* H, const void* w, float bias, umas_dtype dtype, int64_t n_rows,
                                    int32_t d, const int32_t* rowsel, int64_t n_sel, const float* value_old,
                                    const float* ret, const int32_t* tok_role, int32_t n_roles, float clip_eps_v,
                                    int32_t accumulate_dH, int32_t accumulate_dw, int64_t norm_rows, umas_value_stats* stats,
                                    float* value_new, void* dH, float* dw, float* db, void* workspace,
                                    size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Reference-policy KL folded into the token rewards.  The worker groups compute "reference-policy
 * log probabilities" with the quantities of PPO-style optimisation (Section "PPO-Style Training
 * Loop", paragraph "Advantage computation and policy evaluation"); logp_ref comes from
 * umas_policy_logprobs with the reference head.  The paper prints no penalty; the per-token estimate
 * is taken:  r'_t = r_t - beta (logp_t - logp_ref_t) on mask=1 tokens, r_t elsewhere.
 *   tok_reward, logp, logp_ref  DEVICE float [n_tokens], 16-byte aligned;  tok_mask DEVICE uint8 [n_tokens]
 *   tok_reward_out              DEVICE float [n_tokens]; may be tok_reward itself
 *   kl_mean                     DEVICE float [1]: mean of logp - logp_ref over the mask=1 tokens (0 if none) */
size_t umas_kl_rewards_workspace_bytes(int64_t n_tokens);
umas_status umas_kl_rewards(const float* tok_reward, const float* logp, const float* logp_ref,
                            const uint8_t* tok_mask, int64_t n_tokens, float beta, float* tok_reward_out,
                            float* kl_mean, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Advantage whitening over the mask=1 tokens of each model's stream (UMAS_WHITEN_MODEL) or of each role
 * inside it (UMAS_WHITEN_MODEL_ROLE; role identity is kept under sharing, Section "Parameter Sharing in
 * the System"):  A'_t = (A_t - mu) / sqrt(var + eps), population variance, 0 on masked tokens; a group
 * without tokens is left alone; a token whose role is outside [0, n_roles) joins no group and gets 0.
 *   adv, adv_out    DEVICE float [n_tokens], 16-byte aligned; adv_out may be adv itself
 *   tok_role        DEVICE int32 [n_tokens] (may be NULL for UMAS_WHITEN_MODEL)
 *   model_tok_off   HOST int64 [n_models + 1]: the streams' token offsets, from 0 to n_tokens */
typedef enum umas_whiten_scope { UMAS_WHITEN_MODEL = 0, UMAS_WHITEN_MODEL_ROLE = 1 } umas_whiten_scope;
size_t umas_whiten_workspace_bytes(int64_t n_tokens, int32_t n_models, int32_t n_roles);
umas_status umas_whiten_advantages(const float* adv, const uint8_t* tok_mask, const int32_t* tok_role,
                                   const int64_t* model_tok_off, int32_t n_models, int32_t n_roles,
                                   int64_t n_tokens, int32_t scope, float eps, float* adv_out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Ready-batch construction, B_i -> D_i^ready (Section "Model-Local Buffers": filtering incomplete
 * trajectories, shuffling, matching the worker group's data-parallel configuration; the rewards were
 * aligned with the tokens by umas_assign_token_rewards).  The kept trajectories, in the order of the
 * shuffle, are cut into n_minibatch contiguous parts whose sizes differ by at most one: the q-th of
 * n_kept goes to part q * n_minibatch / n_kept.  For model m and minibatch k the scored rows of the
 * minibatch's trajectories are listed trajectory by trajectory in shuffled order, rows of one trajectory
 * in stream order (stream-relative positions, as in rowsel), ready to be passed as the row selection of
 * umas_policy_logprobs / umas_ppo_loss_fwd_bwd / umas_value_loss_fwd_bwd (accumulate_dW = 1 adds the
 * gradients of successive micro-batches).
 *   streams        the arrays written by umas_assign_token_rewards (DEVICE)
 *   traj_turn_off  HOST int32 [n_traj+1], as in umas_graph
 *   traj_keep      HOST uint8 [n_traj], 0 = drop the trajectory; NULL = keep all
 *   traj_order     HOST int32 [n_traj], a permutation of the trajectories (the shuffle); NULL = identity
 *   mb_rowsel      DEVICE int32, at least as many entries as rowsel
 *   mb_off         DEVICE int64 [n_models * (n_minibatch + 1)]: minibatch k of model m is
 *                  mb_rowsel[mb_off[m*(n_minibatch+1) + k] .. mb_off[m*(n_minibatch+1) + k + 1])
 * The host arrays are read inside the call (through the library's pinned staging memory); the call does not wait
 * for the stream. */
size_t umas_ready_batch_workspace_bytes(int32_t n_traj, int32_t n_models);
umas_status umas_ready_batch(const umas_streams* streams, int32_t n_models, int32_t n_turns,
                             const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                             const int32_t* traj_order, int32_t n_minibatch, int32_t* mb_rowsel,
                             int64_t* mb_off, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same with the parts cut by scored rows instead of by trajectories, per model, for worker groups whose
 * micro-batches should carry equal work (Section "Model-Local Buffers": batches are built per model, and
 * "different worker groups can receive different amounts of data"): listing model m's kept rows trajectory by
 * trajectory in shuffled order, T_m rows in all, the trajectory whose first row is the r-th (from 0) goes to part
 * r * n_minibatch / T_m; every part then holds T_m / n_minibatch rows give or take one trajectory.  mb_rowsel is
 * the same list as umas_ready_batch writes; only mb_off differs, and the cuts of different models fall between
 * different trajectories.  Same arguments, workspace and errors. */
umas_status umas_ready_batch_balanced(const umas_streams* streams, int32_t n_models, int32_t n_turns,
                                      const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                                      const int32_t* traj_order, int32_t n_minibatch, int32_t* mb_rowsel,
                                      int64_t* mb_off, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same list of rows cut into micro-batches under a budget of scored rows: sequence packing, i.e. whole sequences
 * laid end to end in a flat batch until it is full (Section "Model-Local Buffers": a ready batch is matched to the worker
 * group's configuration; the paper prints no rule).  Per model, going through the kept trajectories in shuffled order, a
 * trajectory's rows join the open part unless that part already holds rows and would then hold more than max_rows;
 * then the part is closed and the trajectory opens the next one.  Trajectories are never split: one with more than
 * max_rows rows has a part to itself.  No part is empty; a model without kept rows has no part.
 *   max_rows  >= 1 (UMAS_EINVAL otherwise)
 *   mb_off    DEVICE int64 [n_models * (n_traj + 1)]: part k < n_parts[m] of model m is
 *             mb_rowsel[mb_off[m*(n_traj+1) + k] .. mb_off[m*(n_traj+1) + k + 1]); entries past n_parts[m] repeat the end
 *   n_parts   DEVICE int32 [n_models]
 * Other arguments, workspace and errors as umas_ready_batch.  The cuts are found part after part by one wavefront
 * per model (one search per part): meant for budgets that give tens to thousands of parts, not one per trajectory. */
umas_status umas_ready_batch_packed(const umas_streams* streams, int32_t n_models, int32_t n_turns,
                                    const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                                    const int32_t* traj_order, int64_t max_rows, int32_t* mb_rowsel,
                                    int64_t* mb_off, int32_t* n_parts, void* workspace, size_t workspace_bytes,
                                    void* hip_stream);

/* Kernel timing aid for benchmarks (not part of the method).  While enabled, every kernel launch
 * of the library is followed by a HIP event on its stream and the time between consecutive events
 * of one call is booked to the kernel launched in between.  umas_profile_enable(on) discards earlier
 * records.  umas_profile_read waits for the recorded events and returns, per kernel name in order of
 * first launch, the summed milliseconds and the number of launches: names is HOST char [cap][32],
 * total_ms HOST float [cap], launches HOST int32 [cap]; returns the number of names or -1 on a HIP
 * error.  Not thread-safe; meant for a single benchmarking thread. */
umas_status umas_profile_enable(int32_t on);
int32_t umas_profile_read(char* names, float* total_ms, int32_t* launches, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* UMAS_H */
