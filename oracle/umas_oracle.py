"""CPU oracle for the model-local worker step of UnityMAS-O.  TEST INFRASTRUCTURE ONLY.

A plain, slow, sequential statement in float64 of what the GPU library computes:
reward composition and placement, routing through the agent-to-model map, GAE
scans, LM-head scoring, the clipped surrogate and its backward; then the steps around
it: the critic's value head and clipped value loss, the reference-policy KL folded into
the rewards, advantage whitening, and the dual-clip / entropy-bonus variants of the
surrogate.  It shares no
code with the HIP path and imports nothing from it; only tests, the smoke check
and the benchmark's CPU-baseline leg may call it.  The product path never does.

Each function names the passage of the paper it follows.  Where the paper leaves
the arithmetic open (it names PPO but prints no loss; it does not say which
token carries a delayed reward) the reading taken is stated in the docstring.

Parity pins (tests/test_oracle_pins.py, tests/test_oracle_pins_next.py): every function below is pinned against
hand-worked workflow examples, closed forms, invariants or brute force.  The
end-to-end composition of all steps is pinned by one closed form (a uniform
policy, on-policy, gamma = lam = 1) and is otherwise "parity unpinned" beyond the
composition of its pinned parts (the paper prints no end-to-end numbers).
"""
from __future__ import annotations

import numpy as np

PLACE_LAST = 0
PLACE_ALL = 1
SEG_TURN = 0
SEG_TRAJ = 1


# --------------------------------------------------------------------------------------
# Rewards: normalisation, composition  (Section "Agent-Specific Reward Interface")
# --------------------------------------------------------------------------------------
def group_normalise(traj_reward, traj_group, eps=1e-6):
    """z-score trajectory rewards inside each group of trajectories.

    The paper does not require grouped normalisation (its comparison with grouped
    methods says so); the pipeline-shaped workload asks for it.  Reading: population
    mean and standard deviation (divide by the group size), R~ = (R - mu) / (sigma + eps).
    Without groups the rewards pass through unchanged.
    """
    R = np.asarray(traj_reward, dtype=np.float64)
    if traj_group is None:
        return R.copy()
    g = np.asarray(traj_group)
    out = np.empty_like(R)
    for gid in np.unique(g):
        idx = np.nonzero(g == gid)[0]
        mu = R[idx].sum() / len(idx)
        sigma = np.sqrt(((R[idx] - mu) ** 2).sum() / len(idx))
        out[idx] = (R[idx] - mu) / (sigma + eps)
    return out


def compose_rewards(traj_turn_off, turn_role, n_roles, role_reward=None, turn_reward=None,
                    traj_reward=None, w_role=None, w_turn=None, w_traj=None):
    """Per-invocation reward r_v = lam_node r_node + lam_turn r_turn + lam_traj r_traj.

    Follows the additive combination of node-, turn- and trajectory-level rewards
    (equation for r_v with the lambda_v weights).  Reading of the three levels: the
    node/role-level term is one scalar per (trajectory, role) applied to every
    invocation of that role in that trajectory (a format penalty), the turn-level term
    one scalar per invocation (a score delta), the trajectory-level term one scalar per
    trajectory (a shared final score).  Missing levels count 0, missing weights 1.
    Evaluated in float32 in the association (node + turn) + traj so that a float32
    implementation can match it bit for bit.  Returns float32 [n_turns].
    """
    n_traj = len(traj_turn_off) - 1
    n_turns = int(traj_turn_off[-1])
    f32 = np.float32
    rho = np.zeros(n_turns, dtype=np.float32)
    for b in range(n_traj):
        for u in range(int(traj_turn_off[b]), int(traj_turn_off[b + 1])):
            v = int(turn_role[u])
            wr = f32(1) if w_role is None else f32(w_role[v])
            wt = f32(1) if w_turn is None else f32(w_turn[v])
            wj = f32(1) if w_traj is None else f32(w_traj[v])
            rr = f32(0) if role_reward is None else f32(role_reward[b * n_roles + v])
            rt = f32(0) if turn_reward is None else f32(turn_reward[u])
            rj = f32(0) if traj_reward is None else f32(traj_reward[b])
            rho[u] = f32(f32(f32(wr * rr) + f32(wt * rt)) + f32(wj * rj))
    return rho


# --------------------------------------------------------------------------------------
# Routing through phi and reward placement  (Sections "Agent--LLM Mapping",
# "Model-Local Buffers", paragraph "Batch construction")
# --------------------------------------------------------------------------------------
def route(n_models, role_to_model, traj_turn_off, turn_role, turn_tok_off, tok_mask):
    """Commit every invocation to the buffer of the model phi(role) that generated it.

    Model-local stream m holds the tokens of all turns u with phi(turn_role[u]) = m,
    turns in ascending global id (trajectory-major, linearised order inside a
    trajectory, as in the linearised trajectory view), tokens in order inside a turn.
    Streams are stored one after another (model 0 first).  Role identities travel with
    the tokens (the paper keeps them under sharing for role-level reporting).
    A "trajectory run" is the maximal run of one trajectory's turns inside one stream.
    rowsel lists, per model, the stream-relative positions of tokens with mask = 1.
    """
    n_traj = len(traj_turn_off) - 1
    n_turns = int(traj_turn_off[-1])
    turn_traj = np.zeros(n_turns, dtype=np.int64)
    for b in range(n_traj):
        turn_traj[int(traj_turn_off[b]):int(traj_turn_off[b + 1])] = b
    perm, tok_turn, tok_role = [], [], []
    model_tok_off, model_turn_off, model_trajrun_off = [0], [0], [0]
    turn_seg_off, seg_turn, traj_seg_off = [0], [], [0]
    rowsel, model_rowsel_off = [], [0]
    for m in range(n_models):
        stream_start = len(perm)
        last_traj = -1
        for u in range(n_turns):
            if int(role_to_model[int(turn_role[u])]) != m:
                continue
            if last_traj != -1 and turn_traj[u] != last_traj:
                traj_seg_off.append(len(perm))
            last_traj = turn_traj[u]
            for t in range(int(turn_tok_off[u]), int(turn_tok_off[u + 1])):
                if tok_mask[t]:
                    rowsel.append(len(perm) - stream_start)
                perm.append(t)
                tok_turn.append(u)
                tok_role.append(int(turn_role[u]))
            seg_turn.append(u)
            turn_seg_off.append(len(perm))
        if last_traj != -1:
            traj_seg_off.append(len(perm))
        model_tok_off.append(len(perm))
        model_turn_off.append(len(seg_turn))
        model_trajrun_off.append(len(traj_seg_off) - 1)
        model_rowsel_off.append(len(rowsel))
    perm = np.array(perm, dtype=np.int64)
    return {
        "model_tok_off": np.array(model_tok_off, np.int64),
        "perm": perm,
        "tok_turn": np.array(tok_turn, np.int32),
        "tok_role": np.array(tok_role, np.int32),
        "tok_mask": np.asarray(tok_mask, np.uint8)[perm] if len(perm) else np.zeros(0, np.uint8),
        "turn_seg_off": np.array(turn_seg_off, np.int64),
        "seg_turn": np.array(seg_turn, np.int32),
        "model_turn_off": np.array(model_turn_off, np.int32),
        "traj_seg_off": np.array(traj_seg_off, np.int64),
        "model_trajrun_off": np.array(model_trajrun_off, np.int32),
        "rowsel": np.array(rowsel, np.int32),
        "model_rowsel_off": np.array(model_rowsel_off, np.int64),
    }


def place_rewards(streams, rho, place_mode=PLACE_LAST):
    """Align each invocation's reward with its token sequence (paragraph "Batch construction").

    Reading: LAST puts rho_u on the highest-index token of turn u with mask = 1 (the
    terminal-reward convention GAE expects); ALL puts it on every mask = 1 token.
    A turn without any mask = 1 token receives nothing.  Pure copies, float32.
    """
    n = len(streams["perm"])
    out = np.zeros(n, dtype=np.float32)
    off, seg_turn, mask = streams["turn_seg_off"], streams["seg_turn"], streams["tok_mask"]
    for s in range(len(seg_turn)):
        a, e = int(off[s]), int(off[s + 1])
        r = np.float32(rho[int(seg_turn[s])])
        if place_mode == PLACE_ALL:
            for p in range(a, e):
                if mask[p]:
                    out[p] = r
        else:
            for p in range(e - 1, a - 1, -1):
                if mask[p]:
                    out[p] = r
                    break
    return out


# --------------------------------------------------------------------------------------
# Advantages and returns  (paragraph "Advantage computation and policy evaluation")
# --------------------------------------------------------------------------------------
def advantages(streams, traj_turn_off, tok_reward, value, gamma, lam, gamma_turn=1.0, seg_mode=SEG_TURN):
    """Generalised advantage estimation A_t = sum_l (gamma lam)^l delta_{t+l},
    delta_t = r_t + gamma V(s_{t+1}) - V(s_t), by its backward recurrence, per segment.

    Readings where the paper is silent.  Segments: every turn is its own episode
    (SEG_TURN) or every trajectory run inside a model stream is (SEG_TRAJ).  V and A
    beyond the end of a segment are 0.  Tokens with mask = 0 (padding, tool output) are
    not actions: the recurrence skips them, the carried state passes through and their
    outputs are 0.  In SEG_TRAJ the objective's per-step discount gamma^(t-1) over role
    invocations is honoured by multiplying the carried state by
    gamma_turn^(step(later turn) - step(earlier turn)) when the scan crosses from a turn
    to the previous turn of the run (step = 1-based position in the trajectory).
    Returns (adv, ret) in float64, ret = adv + V at valid tokens.
    """
    n = len(streams["perm"])
    r = np.asarray(tok_reward, dtype=np.float64)
    V = np.zeros(n) if value is None else np.asarray(value, dtype=np.float64)
    mask, tok_turn = streams["tok_mask"], streams["tok_turn"]
    n_turns = int(traj_turn_off[-1])
    step = np.zeros(n_turns, dtype=np.int64)
    for b in range(len(traj_turn_off) - 1):
        for k, u in enumerate(range(int(traj_turn_off[b]), int(traj_turn_off[b + 1]))):
            step[u] = k + 1
    seg_off = streams["turn_seg_off"] if seg_mode == SEG_TURN else streams["traj_seg_off"]
    adv, ret = np.zeros(n), np.zeros(n)
    for s in range(len(seg_off) - 1):
        G, NV = 0.0, 0.0
        for t in range(int(seg_off[s + 1]) - 1, int(seg_off[s]) - 1, -1):
            if t + 1 < int(seg_off[s + 1]) and tok_turn[t + 1] != tok_turn[t]:
                c = gamma_turn ** int(step[tok_turn[t + 1]] - step[tok_turn[t]])
                G *= c
                NV *= c
            if mask[t]:
                delta = r[t] + gamma * NV - V[t]
                G = delta + gamma * lam * G
                adv[t] = G
                ret[t] = G + V[t]
                NV = V[t]
    return adv, ret


# --------------------------------------------------------------------------------------
# LM-head scoring  ("old log probabilities" in the policy-evaluation paragraph)
# --------------------------------------------------------------------------------------
def score(H, W, ids, rowsel=None, chunk=256):
    """Per scored row i: z = W h_i, lse = log sum_v exp z_v, logp = z[y_i] - lse,
    entropy = -sum_v p_v log p_v = lse - sum_v p_v z_v with p = softmax(z).

    Natural log, temperature 1, no bias.  Rows outside rowsel are not scored and
    return 0.  Inputs are upcast exactly to float64 (bf16 or float32 values are both
    representable); the product z = H W^T is a library matmul in float64.
    Returns (logp, lse, entropy), float64 [n_rows].
    """
    n = H.shape[0]
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    W64 = np.asarray(W, dtype=np.float64)
    logp, lse, ent = np.zeros(n), np.zeros(n), np.zeros(n)
    for c0 in range(0, len(rows), chunk):
        rr = rows[c0:c0 + chunk]
        z = np.asarray(H[rr], dtype=np.float64) @ W64.T
        zmax = z.max(axis=1, keepdims=True)
        e = np.exp(z - zmax)
        ssum = e.sum(axis=1)
        l = zmax[:, 0] + np.log(ssum)
        p = e / ssum[:, None]
        lse[rr] = l
        logp[rr] = z[np.arange(len(rr)), np.asarray(ids)[rr]] - l
        ent[rr] = l - (p * z).sum(axis=1)
    return logp, lse, ent


# --------------------------------------------------------------------------------------
# Clipped surrogate  (PPO, named in "PPO-Style Training Loop"; formula from Schulman et al. 2017)
# --------------------------------------------------------------------------------------
def ppo_loss(logp, logp_old, adv, entropy, rowsel, tok_role, n_roles, clip_eps):
    """Single-clip PPO surrogate over the scored rows of one model.

    ratio = exp(logp - logp_old); L = max(-A ratio, -A clip(ratio, 1-eps, 1+eps));
    loss = sum_scored L / S (token mean over this model's scored rows, S = 0 gives 0).
    g = d loss / d logp = -A ratio / S on the unclipped branch (taken when
    -A ratio >= -A clip(ratio), ties included), 0 on the clipped branch.
    Statistics: clip fraction (#rows with clipped term strictly larger) / S, mean
    entropy, approx-KL = mean(logp_old - logp); each also restricted to the rows of one
    role (divided by that role's row count), since role identity is preserved for
    role-level reporting under parameter sharing.
    Returns (stats, g) with stats float64 [1+n_roles, 5] = (loss, clip_frac,
    entropy_mean, approx_kl, n_scored) for the model, then per role; g float64 [n_rows].
    """
    n = len(logp)
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    S = len(rows)
    g = np.zeros(n)
    stats = np.zeros((1 + n_roles, 5))
    if S == 0:
        return stats, g
    lp = np.asarray(logp, np.float64)[rows]
    lo = np.asarray(logp_old, np.float64)[rows]
    A = np.asarray(adv, np.float64)[rows]
    H = np.asarray(entropy, np.float64)[rows]
    ratio = np.exp(lp - lo)
    u = -A * ratio
    c = -A * np.minimum(np.maximum(ratio, 1.0 - clip_eps), 1.0 + clip_eps)
    L = np.maximum(u, c)
    unclipped = u >= c
    g[rows] = np.where(unclipped, -A * ratio, 0.0) / S
    role = np.asarray(tok_role)[rows]
    for k in range(1 + n_roles):
        sel = np.ones(S, bool) if k == 0 else (role == k - 1)
        cnt = int(sel.sum())
        if cnt == 0:
            continue
        stats[k] = (L[sel].sum() / cnt, (~unclipped[sel]).sum() / cnt, H[sel].sum() / cnt,
                    (lo[sel] - lp[sel]).sum() / cnt, cnt)
    return stats, g


# --------------------------------------------------------------------------------------
# Backward through the LM head  (paragraph "Model-specific updates and synchronization")
# --------------------------------------------------------------------------------------
def lm_head_backward(H, W, ids, lse, g, rowsel=None, chunk=256):
    """dz_iv = g_i (1[v = y_i] - softmax(z_i)_v); dH_i = sum_v dz_iv W_v; dW_v = sum_i dz_iv h_i.

    The chain rule through logp_i = z_i[y_i] - lse_i.  Unscored rows get dH = 0 and add
    nothing to dW.  Returns (dH [n_rows, d], dW [V, d]) in float64.
    """
    n, d = H.shape
    V = W.shape[0]
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    W64 = np.asarray(W, dtype=np.float64)
    dH, dW = np.zeros((n, d)), np.zeros((V, d))
    for c0 in range(0, len(rows), chunk):
        rr = rows[c0:c0 + chunk]
        Hc = np.asarray(H[rr], dtype=np.float64)
        z = Hc @ W64.T
        p = np.exp(z - np.asarray(lse, np.float64)[rr][:, None])
        dz = -p
        dz[np.arange(len(rr)), np.asarray(ids)[rr]] += 1.0
        dz *= np.asarray(g, np.float64)[rr][:, None]
        dH[rr] = dz @ W64
        dW += dz.T @ Hc
    return dH, dW


# --------------------------------------------------------------------------------------
# Critic  ("value estimates", "actor and critic parameters" in "PPO-Style Training Loop";
# the paper prints no value loss: the clipped form of Schulman et al. 2017 / common PPO
# implementations is the reading taken)
# --------------------------------------------------------------------------------------
def value_head(H, w, b=0.0, rowsel=None):
    """V_i = w . h_i + b for the selected rows, 0 elsewhere.  float64 [n_rows]."""
    n = H.shape[0]
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    V = np.zeros(n)
    w64 = np.asarray(w, dtype=np.float64)
    for i in rows:
        V[i] = float(np.dot(np.asarray(H[i], dtype=np.float64), w64)) + float(b)
    return V


def value_loss(V, V_old, ret, rowsel, tok_role, n_roles, clip_eps_v):
    """Clipped value loss over the selected rows.

    Vc = clip(V, V_old - eps, V_old + eps) (V itself inside the range); L = 1/2 max((V - R)^2, (Vc - R)^2);
    loss = sum L / S.  g = d loss / d V = (V - R) / S where the unclipped term is the
    larger one (ties included), 0 where the clipped term is strictly larger (Vc is then
    a constant).  Statistics per model and per role, float64 [1+n_roles, 4] =
    (loss, clip_frac, mean V, n); g float64 [n_rows].
    """
    n = len(V)
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    S = len(rows)
    g = np.zeros(n)
    stats = np.zeros((1 + n_roles, 4))
    if S == 0:
        return stats, g
    v = np.asarray(V, np.float64)[rows]
    vo = np.asarray(V_old, np.float64)[rows]
    R = np.asarray(ret, np.float64)[rows]
    vc = np.minimum(np.maximum(v, vo - clip_eps_v), vo + clip_eps_v)
    lu = (v - R) ** 2
    lc = (vc - R) ** 2
    unclipped = lu >= lc
    L = 0.5 * np.maximum(lu, lc)
    g[rows] = np.where(unclipped, v - R, 0.0) / S
    role = np.asarray(tok_role)[rows]
    for k in range(1 + n_roles):
        sel = np.ones(S, bool) if k == 0 else (role == k - 1)
        cnt = int(sel.sum())
        if cnt:
            stats[k] = (L[sel].sum() / cnt, (~unclipped[sel]).sum() / cnt, v[sel].sum() / cnt, cnt)
    return stats, g


def value_head_backward(H, w, g, rowsel=None):
    """dH_i = g_i w, dw = sum_i g_i h_i, db = sum_i g_i over the selected rows (float64)."""
    n, d = H.shape
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    w64 = np.asarray(w, dtype=np.float64)
    dH, dw, db = np.zeros((n, d)), np.zeros(d), 0.0
    for i in rows:
        dH[i] = g[i] * w64
        dw += g[i] * np.asarray(H[i], dtype=np.float64)
        db += g[i]
    return dH, dw, db


# --------------------------------------------------------------------------------------
# Reference-policy KL folded into the token rewards  ("reference-policy log probabilities"
# in "PPO-Style Training Loop"; the paper prints no penalty: the per-token estimate
# log pi - log pi_ref scaled by beta and subtracted from the reward is the reading taken)
# --------------------------------------------------------------------------------------
def kl_penalised_rewards(tok_reward, logp, logp_ref, tok_mask, beta):
    """r'_t = r_t - beta (logp_t - logp_ref_t) on mask=1 tokens, r_t elsewhere.
    Also returns the mean of (logp - logp_ref) over the mask=1 tokens (0 if there are none)."""
    r = np.asarray(tok_reward, dtype=np.float64).copy()
    m = np.asarray(tok_mask) != 0
    kl = np.asarray(logp, np.float64) - np.asarray(logp_ref, np.float64)
    r[m] -= beta * kl[m]
    return r, (float(kl[m].mean()) if m.any() else 0.0)


# --------------------------------------------------------------------------------------
# Advantage whitening per model or per (model, role)  (agent-wise normalisation is the
# stabiliser the related work the paper cites centres on; role identity is kept under sharing)
# --------------------------------------------------------------------------------------
WHITEN_MODEL = 0
WHITEN_MODEL_ROLE = 1


def whiten_advantages(adv, tok_mask, tok_role, model_tok_off, n_roles, scope, eps=1e-8):
    """A'_t = (A_t - mu) / sqrt(var + eps) over the mask=1 tokens of each group, where a group is a
    model's stream (scope MODEL) or the tokens of one role inside it (scope MODEL_ROLE); population
    variance; masked tokens keep 0; an empty group is left alone.  float64 [n_tokens]."""
    A = np.asarray(adv, dtype=np.float64)
    out = np.zeros_like(A)
    m = np.asarray(tok_mask) != 0
    role = np.asarray(tok_role)
    for k in range(len(model_tok_off) - 1):
        a, e = int(model_tok_off[k]), int(model_tok_off[k + 1])
        groups = [np.arange(a, e)[m[a:e]]] if scope == WHITEN_MODEL else \
            [np.arange(a, e)[m[a:e] & (role[a:e] == v)] for v in range(n_roles)]
        for idx in groups:
            if len(idx) == 0:
                continue
            mu = A[idx].mean()
            var = ((A[idx] - mu) ** 2).mean()
            out[idx] = (A[idx] - mu) / np.sqrt(var + eps)
    return out


# --------------------------------------------------------------------------------------
# Surrogate variants: dual clip and entropy bonus
# --------------------------------------------------------------------------------------
def ppo_loss_variants(logp, logp_old, adv, entropy, rowsel, tok_role, n_roles, clip_eps, dual_clip=0.0,
                      entropy_coef=0.0, kl_coef=0.0, logp_ref=None):
    """The clipped surrogate with its optional terms.

    dual_clip c > 1: for A < 0 the per-row term max(-A ratio, -A clip(ratio)) is capped at -A c
    (the gradient vanishes where the cap is strictly smaller).  entropy_coef > 0: the loss
    becomes L_clip - entropy_coef * mean entropy; its gradient reaches the logits directly
    (lm_head_backward_entropy), g stays d L_clip / d logp.  The clip fraction counts rows whose
    active term is not the unclipped one.  kl_coef > 0: the reference-policy log-probs (listed with
    the quantities of the update in "Advantage computation and policy evaluation"; the paper prints
    no penalty) enter the loss as kl_coef * mean(e^x - x - 1), x = logp_ref - logp: each term is
    non-negative and its expectation over tokens drawn from the policy is KL(policy || reference);
    d/dlogp of a term is 1 - e^x, which is added to g (divided by S).
    Returns (stats [1+n_roles, 5], g) like ppo_loss; stats[:, 0] includes the entropy and KL terms.
    """
    n = len(logp)
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    S = len(rows)
    g = np.zeros(n)
    stats = np.zeros((1 + n_roles, 5))
    if S == 0:
        return stats, g
    lp = np.asarray(logp, np.float64)[rows]
    lo = np.asarray(logp_old, np.float64)[rows]
    A = np.asarray(adv, np.float64)[rows]
    Hh = np.asarray(entropy, np.float64)[rows]
    ratio = np.exp(lp - lo)
    u = -A * ratio
    c = -A * np.minimum(np.maximum(ratio, 1.0 - clip_eps), 1.0 + clip_eps)
    L = np.maximum(u, c)
    active_unclipped = u >= c
    if dual_clip > 0.0:
        cap = -A * dual_clip
        capped = (A < 0) & (cap < L)
        L = np.where(capped, cap, L)
        active_unclipped &= ~capped
    g[rows] = np.where(active_unclipped, -A * ratio, 0.0) / S
    if kl_coef > 0.0:
        x = np.asarray(logp_ref, np.float64)[rows] - lp
        L = L + kl_coef * (np.exp(x) - x - 1.0)
        g[rows] += kl_coef * (1.0 - np.exp(x)) / S
    role = np.asarray(tok_role)[rows]
    for k in range(1 + n_roles):
        sel = np.ones(S, bool) if k == 0 else (role == k - 1)
        cnt = int(sel.sum())
        if cnt:
            stats[k] = (L[sel].sum() / cnt - entropy_coef * Hh[sel].sum() / cnt, (~active_unclipped[sel]).sum() / cnt,
                        Hh[sel].sum() / cnt, (lo[sel] - lp[sel]).sum() / cnt, cnt)
    return stats, g


def lm_head_backward_entropy(H, W, ids, lse, entropy, g, entropy_coef, n_scored, rowsel=None, chunk=256):
    """Backward of L_clip - entropy_coef * mean entropy through the LM head.

    d entropy_i / d z_iv = -p_iv (log p_iv + entropy_i), so
    dz_iv = g_i (1[v = y_i] - p_iv) + (entropy_coef / n_scored) p_iv (log p_iv + entropy_i);
    dH and dW follow as in lm_head_backward.  Returns (dH, dW) in float64.
    """
    n, d = H.shape
    V = W.shape[0]
    rows = np.arange(n) if rowsel is None else np.asarray(rowsel, dtype=np.int64)
    W64 = np.asarray(W, dtype=np.float64)
    dH, dW = np.zeros((n, d)), np.zeros((V, d))
    for c0 in range(0, len(rows), chunk):
        rr = rows[c0:c0 + chunk]
        Hc = np.asarray(H[rr], dtype=np.float64)
        z = Hc @ W64.T
        logp_all = z - np.asarray(lse, np.float64)[rr][:, None]
        p = np.exp(logp_all)
        dz = -p * np.asarray(g, np.float64)[rr][:, None]
        dz[np.arange(len(rr)), np.asarray(ids)[rr]] += np.asarray(g, np.float64)[rr]
        dz += (entropy_coef / n_scored) * p * (logp_all + np.asarray(entropy, np.float64)[rr][:, None])
        dH[rr] = dz @ W64
        dW += dz.T @ Hc
    return dH, dW


# --------------------------------------------------------------------------------------
# Ready-batch construction  (Section "Model-Local Buffers": a buffer becomes a ready batch by
# filtering incomplete trajectories, shuffling and matching the worker group's data-parallel
# configuration; rewards were aligned with the tokens by place_rewards)
# --------------------------------------------------------------------------------------
def ready_batch(streams, traj_turn_off, traj_keep, traj_order, n_minibatch, balance_rows=False):
    """Split every model's scored rows into minibatches of whole trajectories.

    traj_keep[b] = 0 drops trajectory b (incomplete).  traj_order is the shuffle: a permutation of
    the trajectories, supplied by the caller.  The kept trajectories, in shuffled order, are cut into
    n_minibatch contiguous parts whose sizes differ by at most one: the q-th of n_kept goes to part
    q * n_minibatch // n_kept.  For model m and minibatch k the rows are those of the minibatch's
    trajectories, trajectory by trajectory in shuffled order, each trajectory's scored rows in stream
    order (stream-relative positions, as in rowsel).
    With balance_rows the parts are cut by scored rows instead of by trajectories, per model (worker groups
    "can receive different amounts of data"; what is matched to the data-parallel configuration is the work):
    listing a model's rows trajectory by trajectory in shuffled order, T rows in all, the trajectory whose
    first row is the r-th (from 0) goes to part r * n_minibatch // T, so that every part holds T / n_minibatch
    rows give or take one trajectory.
    Returns (mb_rowsel int32 [kept scored rows], mb_off int64 [n_models, n_minibatch + 1]):
    minibatch k of model m is mb_rowsel[mb_off[m, k] : mb_off[m, k + 1]].
    """
    n_traj = len(traj_turn_off) - 1
    n_models = len(streams["model_tok_off"]) - 1
    turn_traj = {}
    for b in range(n_traj):
        for u in range(int(traj_turn_off[b]), int(traj_turn_off[b + 1])):
            turn_traj[u] = b
    kept = [int(b) for b in traj_order if traj_keep[int(b)]]
    part = {b: (q * n_minibatch) // len(kept) for q, b in enumerate(kept)}
    out, off = [], np.zeros((n_models, n_minibatch + 1), dtype=np.int64)
    for m in range(n_models):
        a = int(streams["model_tok_off"][m])
        ra, re = int(streams["model_rowsel_off"][m]), int(streams["model_rowsel_off"][m + 1])
        rows_of = {}
        for row in streams["rowsel"][ra:re]:
            b = turn_traj[int(streams["tok_turn"][a + int(row)])]
            rows_of.setdefault(b, []).append(int(row))
        part_m = part
        if balance_rows:
            total = sum(len(rows_of.get(b, [])) for b in kept)
            part_m, first_row = {}, 0
            for b in kept:
                part_m[b] = (first_row * n_minibatch) // total if total else 0
                first_row += len(rows_of.get(b, []))
        for k in range(n_minibatch):
            off[m, k] = len(out)
            for b in kept:
                if part_m[b] == k:
                    out.extend(rows_of.get(b, []))
        off[m, n_minibatch] = len(out)
    return np.array(out, dtype=np.int32), off


def ready_batch_packed(streams, traj_turn_off, traj_keep, traj_order, max_rows):
    """The ready batch cut into micro-batches under a budget of scored rows (sequence packing: whole sequences
    laid end to end in a flat batch until it is full; the paper says only that batches are matched to the worker
    group's configuration).  Per model, going through the kept trajectories in shuffled order: a trajectory's rows
    join the open part unless that part already holds rows and would then hold more than max_rows, in which case
    the part is closed and the trajectory opens the next one.  Trajectories are never split, so a trajectory with
    more than max_rows rows has a part to itself; trajectories without rows in the model open or close nothing,
    so no part is empty.  The rows and their order are those of ready_batch.
    Returns (mb_rowsel int32, mb_off int64 [n_models, n_traj + 1], n_parts int32 [n_models]): part k < n_parts[m]
    of model m is mb_rowsel[mb_off[m, k] : mb_off[m, k + 1]]; the entries past n_parts[m] repeat the model's end."""
    n_traj = len(traj_turn_off) - 1
    n_models = len(streams["model_tok_off"]) - 1
    turn_traj = {}
    for b in range(n_traj):
        for u in range(int(traj_turn_off[b]), int(traj_turn_off[b + 1])):
            turn_traj[u] = b
    kept = [int(b) for b in traj_order if traj_keep[int(b)]]
    out = []
    off = np.zeros((n_models, n_traj + 1), dtype=np.int64)
    n_parts = np.zeros(n_models, dtype=np.int32)
    for m in range(n_models):
        a = int(streams["model_tok_off"][m])
        ra, re = int(streams["model_rowsel_off"][m]), int(streams["model_rowsel_off"][m + 1])
        rows_of = {}
        for row in streams["rowsel"][ra:re]:
            rows_of.setdefault(turn_traj[int(streams["tok_turn"][a + int(row)])], []).append(int(row))
        starts, in_part = [len(out)], 0
        for b in kept:
            mine = rows_of.get(b, [])
            if not mine:
                continue
            if in_part > 0 and in_part + len(mine) > max_rows:
                starts.append(len(out))
                in_part = 0
            out.extend(mine)
            in_part += len(mine)
        k = len(starts) if in_part > 0 else 0          # no rows at all: no part
        n_parts[m] = k
        off[m, :] = len(out)
        off[m, :len(starts)] = starts
    return np.array(out, dtype=np.int32), off, n_parts
