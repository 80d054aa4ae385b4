"""Steps a1-a4 (reward composition, routing, placement, flags, the advantage recurrence) restated array-wise in numpy,
for instances far beyond what the sequential oracle can walk.  Test infrastructure: written from the same definitions
as the oracle but sharing no code with it (sorting, prefix sums and gathers in place of its loops);
tests/test_oracle_pins.py holds the two against each other on seeded random graphs, the GPU tests use this one at
sizes of tens of millions of tokens."""
import numpy as np

import workloads as wl


def turn_steps(w):
    """1-based position of every turn inside its trajectory, and the trajectory of every turn."""
    n_t = np.diff(w.traj_turn_off).astype(np.int64)
    traj = np.repeat(np.arange(w.n_traj, dtype=np.int64), n_t)
    step = np.arange(w.n_turns, dtype=np.int64) - np.repeat(w.traj_turn_off[:-1].astype(np.int64), n_t) + 1
    return step, traj


def composed_rewards(w):
    """r_v = lam_node r_node + lam_turn r_turn + lam_traj r_traj per turn (Section "Agent-Specific Reward Interface"),
    float32 with every product and sum rounded on its own, (node + turn) + traj; the trajectory level z-scored inside
    its group in float64 first (population deviation + eps)."""
    f32 = np.float32
    _, traj = turn_steps(w)
    rj = np.zeros(w.n_traj, f32)
    if w.traj_reward is not None:
        rj = w.traj_reward.astype(f32)
        if w.traj_group is not None:
            R = w.traj_reward.astype(np.float64)
            _, inv, cnt = np.unique(w.traj_group, return_inverse=True, return_counts=True)
            mu = np.bincount(inv, weights=R) / cnt
            var = np.bincount(inv, weights=(R - mu[inv]) ** 2) / cnt
            rj = ((R - mu[inv]) / (np.sqrt(var)[inv] + w.norm_eps)).astype(f32)
    one = np.ones(w.n_roles, f32)
    wr, wt, wj = (one if x is None else np.asarray(x, f32) for x in (w.w_role, w.w_turn, w.w_traj))
    v = w.turn_role
    rr = np.zeros(w.n_turns, f32) if w.role_reward is None else w.role_reward.astype(f32)[traj * w.n_roles + v]
    rt = np.zeros(w.n_turns, f32) if w.turn_reward is None else w.turn_reward.astype(f32)
    return ((wr[v] * rr + wt[v] * rt) + wj[v] * rj[traj]).astype(f32) if w.n_turns else np.zeros(0, f32)


def streams(w):
    """The model-local streams (Sections "Agent--LLM Mapping", "Model-Local Buffers"): turns stably sorted by the model
    of their role, tokens of a turn kept together and in order."""
    K, U, N = w.n_models, w.n_turns, w.n_tokens
    step, traj = turn_steps(w)
    model_of_turn = w.role_to_model[w.turn_role].astype(np.int64) if U else np.zeros(0, np.int64)
    order = np.argsort(model_of_turn, kind="stable")
    lens = np.diff(w.turn_tok_off)[order]
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    model_turn_off = np.searchsorted(model_of_turn[order], np.arange(K + 1), side="left").astype(np.int32)
    model_tok_off = seg_off[model_turn_off]
    perm = np.repeat(w.turn_tok_off[:-1][order] - seg_off[:-1], lens) + np.arange(N, dtype=np.int64)
    tok_slot = np.repeat(np.arange(U, dtype=np.int64), lens)
    tok_turn = order[tok_slot].astype(np.int32)
    mask = (w.tok_mask[perm] != 0).astype(np.uint8)
    scored = np.flatnonzero(mask)
    model_of_scored = np.searchsorted(model_tok_off, scored, side="right") - 1
    rowsel = (scored - model_tok_off[model_of_scored]).astype(np.int32)
    model_rowsel_off = np.searchsorted(scored, model_tok_off, side="left").astype(np.int64)
    # trajectory runs: maximal runs of one trajectory's turns inside one stream (turns without tokens included)
    t_o, m_o = traj[order], model_of_turn[order]
    new_run = np.ones(U, bool)
    new_run[1:] = (t_o[1:] != t_o[:-1]) | (m_o[1:] != m_o[:-1])
    run_of_slot = np.cumsum(new_run) - 1
    n_runs = int(new_run.sum())
    traj_seg_off = np.concatenate([seg_off[:-1][new_run], [N]]).astype(np.int64)
    model_trajrun_off = np.concatenate([[0], np.cumsum(np.bincount(m_o[new_run], minlength=K))]).astype(np.int32)
    # the last token of every turn that has tokens: turn end; run end, else the steps to the run's next turn with tokens
    flags = mask.copy()
    filled = np.flatnonzero(lens > 0)
    if len(filled):
        last = seg_off[filled + 1] - 1
        same_run = np.zeros(len(filled), bool)
        same_run[:-1] = run_of_slot[filled[1:]] == run_of_slot[filled[:-1]]
        ds = np.zeros(len(filled), np.int64)
        ds[:-1] = step[order[filled[1:]]] - step[order[filled[:-1]]]
        flags[last] |= np.where(same_run, 2 | (np.minimum(ds, 31) << 3), 2 | 4).astype(np.uint8)
    return dict(model_tok_off=model_tok_off, perm=perm, tok_turn=tok_turn, tok_role=w.turn_role[tok_turn].astype(np.int32),
                tok_mask=mask, turn_seg_off=seg_off, seg_turn=order.astype(np.int32), model_turn_off=model_turn_off,
                traj_seg_off=traj_seg_off, model_trajrun_off=model_trajrun_off, rowsel=rowsel,
                model_rowsel_off=model_rowsel_off, tok_flags=flags, turn_step=step.astype(np.int32),
                tok_slot=tok_slot, run_of_slot=run_of_slot, n_runs=n_runs)


def placed_rewards(st, rho, place_mode):
    """The turn's reward on its last mask=1 token (LAST) or on every mask=1 token (ALL), copies of rho (paragraph
    "Batch construction")."""
    N = len(st["perm"])
    mask = st["tok_mask"] != 0
    r = np.zeros(N, np.float32)
    if place_mode == wl.PLACE_ALL:
        r[mask] = rho[st["tok_turn"][mask]]
        return r
    off = st["turn_seg_off"]
    filled = np.flatnonzero(np.diff(off) > 0)
    if len(filled):
        pos = np.where(mask, np.arange(N), -1)
        last = np.maximum.reduceat(pos, off[filled])     # consecutive filled turns tile [0, N)
        has = last >= 0
        r[last[has]] = rho[st["seg_turn"][filled[has]]]
    return r


def recurrence_check(st, r, value, adv, ret, gamma, lam, gamma_turn, seg_mode, tol=1e-5):
    """A_t = delta_t + gamma lam A_next with delta_t = r_t + gamma V_next - V_t (paragraph "Advantage computation and
    policy evaluation"), next = the next mask=1 token of the same segment (0 beyond it), what is carried across a turn
    boundary multiplied by gamma_turn^(step difference); every scored token against its successor's GIVEN advantage,
    so no error hides behind an accumulated one.  Returns the largest residual relative to its allowance."""
    N = len(st["perm"])
    a, rt = np.asarray(adv, np.float64), np.asarray(ret, np.float64)
    mask = st["tok_mask"] != 0
    assert not a[~mask].any() and not rt[~mask].any(), "mask=0 tokens must output 0"
    V = np.zeros(N) if value is None else np.asarray(value, np.float64)
    scored = np.flatnonzero(mask)
    if len(scored) == 0:
        return 0.0
    slot = st["tok_slot"]
    seg = slot if seg_mode == wl.SEG_TURN else st["run_of_slot"][slot]
    step = st["turn_step"].astype(np.int64)[st["tok_turn"]]
    cur, nxt = scored[:-1], scored[1:]
    same = seg[nxt] == seg[cur]
    c = np.where(slot[nxt] != slot[cur], np.float64(gamma_turn) ** (step[nxt] - step[cur]), 1.0)
    tail_v, tail_a = np.zeros(len(scored)), np.zeros(len(scored))
    tail_v[:-1] = np.where(same, c * gamma * V[nxt], 0.0)
    tail_a[:-1] = np.where(same, c * gamma * lam * a[nxt], 0.0)
    rs = np.asarray(r, np.float64)[scored]
    want = rs - V[scored] + tail_v + tail_a
    rms = max(float(np.sqrt(np.mean(want * want))), 1e-30)
    allow = tol * np.maximum(np.abs(want), rms) + 8 * 2.0 ** -24 * (np.abs(rs) + np.abs(V[scored]) + np.abs(tail_v) + np.abs(tail_a))
    worst = float((np.abs(a[scored] - want) / allow).max())
    worst_ret = float((np.abs(rt[scored] - (a[scored] + V[scored])) / (2.0 ** -22 * (np.abs(a[scored]) + np.abs(V[scored])) + 1e-30)).max())
    return max(worst, worst_ret)


def ready_batch(w, st, keep, order, M, balanced):
    """The ready batch (Section "Model-Local Buffers", B_i -> D_i^ready) with sorts and prefix sums: a model's rows are
    those of its kept trajectories one after the other in shuffled order, stream order inside a trajectory; the q-th
    of n kept trajectories belongs to part q M // n, or, cut by rows, the trajectory whose first row is the r-th of
    the model's T rows to part r M // T.  Parts ascend along the shuffled order, so a part ends where the next one's
    first trajectory begins.  Returns (rows, off [n_models, M + 1])."""
    K, B = w.n_models, w.n_traj
    _, traj_of_turn = turn_steps(w)
    scored = np.flatnonzero(st["tok_mask"])
    model_of = np.searchsorted(st["model_tok_off"], scored, side="right") - 1
    traj_of = traj_of_turn[st["tok_turn"][scored]]
    order = np.arange(B) if order is None else np.asarray(order, np.int64)
    kept = order if keep is None else order[np.asarray(keep)[order] != 0]
    rank = np.full(B, -1, np.int64)
    rank[kept] = np.arange(len(kept))
    sel = rank[traj_of] >= 0 if len(scored) else np.zeros(0, bool)
    key = model_of[sel] * (B + 1) + rank[traj_of[sel]]
    rows = st["rowsel"][sel][np.argsort(key, kind="stable")]
    cnt = np.zeros((K, len(kept)), np.int64)
    np.add.at(cnt, (model_of[sel], rank[traj_of[sel]]), 1)
    off = np.zeros((K, M + 1), np.int64)
    base = 0
    for m in range(K):
        first_row = np.cumsum(cnt[m]) - cnt[m]
        total = int(cnt[m].sum())
        if balanced:
            part = first_row * M // total if total else np.zeros(len(kept), np.int64)
        else:
            part = np.arange(len(kept), dtype=np.int64) * M // max(len(kept), 1)
        # trailing trajectories without rows may fall behind the last part when cut by rows: they add nothing
        per_part = np.bincount(np.minimum(part, M - 1), weights=cnt[m], minlength=M).astype(np.int64)
        off[m] = base + np.concatenate([[0], np.cumsum(per_part)])
        base += total
    return rows, off


def ready_batch_packed(w, st, keep, order, max_rows):
    """Micro-batches under a budget of scored rows: the rows of ready_batch; per model, from the prefix sums of the
    kept trajectories' row counts, a part ends at the last trajectory boundary within max_rows rows of its start, or
    behind the trajectory at its start when that one alone is over the budget (a search per part).
    Returns (rows, off [n_models, n_traj + 1], n_parts)."""
    K, B = w.n_models, w.n_traj
    rows, off1 = ready_batch(w, st, keep, order, 1, False)
    _, traj_of_turn = turn_steps(w)
    scored = np.flatnonzero(st["tok_mask"])
    model_of = np.searchsorted(st["model_tok_off"], scored, side="right") - 1
    traj_of = traj_of_turn[st["tok_turn"][scored]]
    order = np.arange(B) if order is None else np.asarray(order, np.int64)
    kept = order if keep is None else order[np.asarray(keep)[order] != 0]
    rank = np.full(B, -1, np.int64)
    rank[kept] = np.arange(len(kept))
    sel = rank[traj_of] >= 0 if len(scored) else np.zeros(0, bool)
    cnt = np.zeros((K, len(kept)), np.int64)
    np.add.at(cnt, (model_of[sel], rank[traj_of[sel]]), 1)
    off = np.zeros((K, B + 1), np.int64)
    n_parts = np.zeros(K, np.int32)
    for m in range(K):
        bounds = np.concatenate([[0], np.cumsum(cnt[m])])        # row boundaries between the kept trajectories
        bounds = np.unique(bounds)                                # trajectories without rows add no boundary
        total, at, cuts = int(bounds[-1]), 0, [0]
        while at < total:
            j = int(np.searchsorted(bounds, at + max_rows, side="right")) - 1
            end = int(bounds[j])
            if end == at:
                end = int(bounds[j + 1])
            cuts.append(end)
            at = end
        n_parts[m] = len(cuts) - 1
        off[m, :] = off1[m, 0] + total
        off[m, :len(cuts)] = off1[m, 0] + np.array(cuts)
    return rows, off, n_parts
