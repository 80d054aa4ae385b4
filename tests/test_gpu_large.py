"""Routing, placement and the scans at sizes far beyond what the sequential oracle can walk: the instances of
configurations 1 and 4 that the bandwidth figures are measured on, 84 and 101 million tokens (tens of thousands of token blocks, hundreds of groups of
blocks, scan ranges by the thousand), checked through properties that hold at any size and that numpy can
evaluate array-wise: with one model the stable partition is the identity, every per-token array is a gather of
per-turn data, the scored positions are the non-zero mask entries, the reward sits on each turn's last scored
token, and the advantages satisfy the printed recurrence token by token (each against its successor, so that no
error can hide behind an accumulated one)."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2605_26646_amd as umas
from tests import parity as P

pytestmark = pytest.mark.gpu


def composed_rewards(w):
    """The additive per-turn reward, array-wise, in the association and float32 rounding of the definition; the
    z-score of the trajectory rewards inside groups of consecutive trajectories in float64."""
    f32 = np.float32
    traj_of_turn = np.repeat(np.arange(w.n_traj), np.diff(w.traj_turn_off))
    rj = np.zeros(w.n_traj, f32)
    if w.traj_reward is not None:
        rj = w.traj_reward.astype(f32)
        if w.traj_group is not None:
            size = int(np.bincount(w.traj_group).max())
            assert w.n_traj % size == 0 and np.array_equal(w.traj_group, np.arange(w.n_traj) // size)
            R = w.traj_reward.astype(np.float64).reshape(-1, size)
            mu, sd = R.mean(axis=1, keepdims=True), R.std(axis=1, keepdims=True)
            rj = ((R - mu) / (sd + w.norm_eps)).reshape(-1).astype(f32)
    one = np.ones(w.n_roles, f32)
    wr, wt, wj = (one if x is None else x.astype(f32) for x in (w.w_role, w.w_turn, w.w_traj))
    rr = np.zeros(w.n_turns, f32) if w.role_reward is None else w.role_reward.astype(f32)[traj_of_turn * w.n_roles + w.turn_role]
    rt = np.zeros(w.n_turns, f32) if w.turn_reward is None else w.turn_reward.astype(f32)
    v = w.turn_role
    return (wr[v] * rr + wt[v] * rt) + wj[v] * rj[traj_of_turn]


@pytest.mark.parametrize("cfg,n_traj,seg_mode,gamma_turn", [(1, 131072, 0, 1.0), (4, 8192, 0, 1.0), (4, 8192, 1, 0.97)])
def test_front_end_properties_at_bandwidth_sizes(cfg, n_traj, seg_mode, gamma_turn):
    w = wl.make_workload(cfg, n_traj=n_traj)
    assert w.n_models == 1 and w.n_tokens > 16_000_000
    N, U, B = w.n_tokens, w.n_turns, w.n_traj
    s, adv, ret = P.gpu_front(w, seg_mode=seg_mode, gamma_turn=gamma_turn)
    lens = np.diff(w.turn_tok_off)
    assert (lens > 0).all()
    get = lambda t: t.cpu().numpy()
    # one model: the stable partition is the identity
    assert np.array_equal(get(s.model_tok_off), [0, N]) and np.array_equal(get(s.model_turn_off), [0, U])
    assert np.array_equal(get(s.perm), np.arange(N))
    assert np.array_equal(get(s.turn_seg_off), w.turn_tok_off) and np.array_equal(get(s.seg_turn), np.arange(U))
    assert np.array_equal(get(s.model_trajrun_off), [0, B])
    runs = get(s.traj_seg_off)
    assert np.array_equal(runs[:B + 1], w.turn_tok_off[w.traj_turn_off])
    tok_turn = np.repeat(np.arange(U, dtype=np.int32), lens)
    assert np.array_equal(get(s.tok_turn), tok_turn)
    assert np.array_equal(get(s.tok_role), w.turn_role[tok_turn])
    mask = w.tok_mask != 0
    assert np.array_equal(get(s.tok_mask), mask.astype(np.uint8))
    scored = np.flatnonzero(mask)
    assert np.array_equal(get(s.model_rowsel_off), [0, len(scored)])
    assert np.array_equal(get(s.rowsel)[:len(scored)], scored)
    step = (np.arange(U) - np.repeat(w.traj_turn_off[:-1], np.diff(w.traj_turn_off)) + 1).astype(np.int32)
    assert np.array_equal(get(s.turn_step), step)
    # flags: mask, turn ends, run (= trajectory) ends, one step to the next turn of the run
    flags = mask.astype(np.uint8)
    turn_last = w.turn_tok_off[1:] - 1
    traj_last = w.turn_tok_off[w.traj_turn_off[1:]] - 1
    flags[turn_last] |= 2 | (1 << 3)
    flags[traj_last] = (flags[traj_last] & 3) | 4
    assert np.array_equal(get(s.tok_flags), flags)
    # composed rewards, and their place: the last scored token of every turn
    rho = composed_rewards(w)
    ts = get(s.turn_scalar)
    if w.traj_group is None:
        assert np.array_equal(ts.view(np.uint32), rho.view(np.uint32))
    else:
        P.close(ts, rho, 1e-5, "turn_scalar")
    pos = np.where(mask, np.arange(N), -1)
    last_scored = np.maximum.reduceat(pos, w.turn_tok_off[:-1])
    r = np.zeros(N, np.float32)
    if w.place_mode == wl.PLACE_LAST:
        has = last_scored >= 0
        r[last_scored[has]] = ts[has]
    else:
        r[mask] = ts[tok_turn][mask]
    tr = get(s.tok_reward)
    assert np.array_equal(tr.view(np.uint32), r.view(np.uint32)), "placed rewards differ"
    # advantages: every scored token against its successor inside the segment
    a, rt = get(adv).astype(np.float64), get(ret).astype(np.float64)
    assert not a[~mask].any() and not rt[~mask].any()
    V = np.zeros(N) if w.value is None else w.value.astype(np.float64)
    seg = tok_turn if seg_mode == 0 else np.repeat(np.arange(B), np.diff(w.turn_tok_off[w.traj_turn_off]))
    nxt = scored[1:]
    same = seg[nxt] == seg[scored[:-1]]
    c = np.where(tok_turn[nxt] != tok_turn[scored[:-1]], gamma_turn ** (step[tok_turn[nxt]] - step[tok_turn[scored[:-1]]]).astype(np.float64), 1.0)
    tail = np.zeros(len(scored))
    tail[:-1] = np.where(same, c * (w.gamma * V[nxt] + w.gamma * w.lam * a[nxt]), 0.0)
    want = r[scored].astype(np.float64) - V[scored] + tail
    scale = max(float(np.sqrt(np.mean(want * want))), 1e-30)
    err = np.abs(a[scored] - want)
    assert (err <= 1e-5 * np.maximum(np.abs(want), scale) + 4 * 2.0 ** -24 * (np.abs(r[scored]) + np.abs(V[scored]) + np.abs(tail))).all(), \
        f"recurrence residual {float((err / np.maximum(np.abs(want), scale)).max()):.3g}"
    assert np.abs(rt[scored] - (a[scored] + V[scored])).max() <= 1e-6 * max(1.0, float(np.abs(rt).max()))
    # the ready batch on the same streams: keep everything, identity order, one part = the selection itself
    rows, off = umas.umas_ready_batch(s, w.traj_turn_off, 1)
    assert np.array_equal(get(off), [[0, len(scored)]]) and np.array_equal(get(rows)[:len(scored)], scored)


def test_shaping_and_ready_batch_at_bandwidth_sizes():
    """The steps around the advantage step on the 101-million-token instance of configuration 1: KL-penalised rewards
    and whitening per (model, role) against the oracle's own array-wise definitions; the ready batch (a tenth of
    the trajectories dropped, a seeded shuffle, eight parts, both cuts) against its definition written with prefix
    sums: the parts are ascending along the shuffled order, so the rows are those of the kept trajectories one
    after the other and a part's end is the number of rows of the trajectories before the next part's first."""
    from oracle import umas_oracle as orc
    w = wl.make_workload(1, n_traj=131072)
    N, B, M = w.n_tokens, w.n_traj, 8
    s, adv, _ = P.gpu_front(w)
    mask = w.tok_mask != 0
    rng = np.random.default_rng(77)
    logp = rng.uniform(-3.0, 0.0, N).astype(np.float32)
    logp_ref = (logp + 0.1 * rng.standard_normal(N, dtype=np.float32)).astype(np.float32)
    r_in = s.tok_reward.cpu().numpy()
    r_g, kl_g = umas.umas_kl_rewards(s.tok_reward, P.to_dev(logp), P.to_dev(logp_ref), s.tok_mask, 0.05)
    r_o, kl_o = orc.kl_penalised_rewards(r_in, logp, logp_ref, w.tok_mask, 0.05)
    r_g = r_g.cpu().numpy()
    assert np.array_equal(r_g[~mask].view(np.uint32), r_in[~mask].view(np.uint32))
    # r - beta * kl in float32: the product and the difference round once each
    assert (np.abs(r_g - r_o) <= 2.0 ** -23 * (np.abs(r_in) + 0.05 * np.abs(logp.astype(np.float64) - logp_ref)) + 1e-30).all()
    assert abs(float(kl_g.cpu()[0]) - kl_o) <= 1e-5 * max(abs(kl_o), 1e-3)
    a_in = adv.cpu().numpy()
    role = np.repeat(w.turn_role, np.diff(w.turn_tok_off))
    off = np.array([0, N], np.int64)
    wh_o = orc.whiten_advantages(a_in, w.tok_mask, role, off, w.n_roles, orc.WHITEN_MODEL_ROLE)
    wh = umas.umas_whiten_advantages(adv, s.tok_mask, s.tok_role, off, w.n_roles, umas.WHITEN_MODEL_ROLE).cpu().numpy()
    bound = P.whiten_bounds(a_in, w.tok_mask, role, off, w.n_roles, True)
    P.close_bounded(wh, wh_o, bound + 1e-30, 1e-5, "whitened advantages")
    del wh_o, bound, r_o, logp, logp_ref
    # ready batch
    order = np.random.default_rng(7).permutation(B).astype(np.int32)
    keep = (np.random.default_rng(8).random(B) < 0.9).astype(np.uint8)
    scored = np.flatnonzero(mask)
    cum = np.concatenate([[0], np.cumsum(mask, dtype=np.int64)])
    t0, t1 = w.turn_tok_off[w.traj_turn_off[:-1]], w.turn_tok_off[w.traj_turn_off[1:]]
    kept = order[keep[order] != 0]
    c = (cum[t1] - cum[t0])[kept]
    first_row = np.cumsum(c) - c
    total = int(c.sum())
    want_rows = scored[np.repeat(cum[t0][kept] - first_row, c) + np.arange(total)]
    for balanced, part in ((False, np.arange(len(kept), dtype=np.int64) * M // len(kept)), (True, first_row * M // total)):
        assert (np.diff(part) >= 0).all()
        want_off = np.concatenate([[0], np.cumsum(np.bincount(part, weights=c, minlength=M).astype(np.int64))])
        rows, mb_off = umas.umas_ready_batch(s, w.traj_turn_off, M, keep, order, balance_rows=balanced)
        assert np.array_equal(mb_off.cpu().numpy(), want_off[None, :]), f"part offsets, balanced={balanced}"
        assert np.array_equal(rows.cpu().numpy()[:total], want_rows), f"rows, balanced={balanced}"
