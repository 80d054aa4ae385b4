"""Routing, placement and the scans at sizes far beyond what the sequential oracle can walk: the instances of
configurations 1 and 4 that the bandwidth figures are measured on (84 and 101 million tokens: tens of thousands of
token blocks, hundreds of groups of blocks, scan ranges by the thousand) and seeded random multi-model graphs of
about 25 million tokens (turns and trajectories without tokens, turns without a scored token, streams that start
anywhere inside a block).  Expected values come from tests/arraywise.py, the array-wise restatement of steps a1-a4
that tests/test_oracle_pins.py holds against the sequential oracle: streams, flags and placed rewards bit for bit,
the advantages through the recurrence token by token (each against its successor, so that no error can hide behind
an accumulated one)."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2605_26646_amd as umas
from tests import arraywise as aw
from tests import parity as P

pytestmark = pytest.mark.gpu


def check_front_arraywise(w, s, adv, ret, place_mode, seg_mode, gamma, lam, gamma_turn):
    get = lambda t: t.cpu().numpy()
    sa = aw.streams(w)
    U, N = w.n_turns, w.n_tokens
    for f in ("model_tok_off", "perm", "tok_turn", "tok_role", "tok_mask", "turn_seg_off", "model_turn_off",
              "model_trajrun_off", "model_rowsel_off", "tok_flags"):
        assert np.array_equal(get(getattr(s, f)), sa[f]), f
    assert np.array_equal(get(s.seg_turn)[:U], sa["seg_turn"]) and np.array_equal(get(s.turn_step)[:U], sa["turn_step"])
    runs = get(s.traj_seg_off)
    assert np.array_equal(runs[:sa["n_runs"] + 1], sa["traj_seg_off"]) and (runs[sa["n_runs"] + 1:] == N).all()
    assert np.array_equal(get(s.rowsel)[:len(sa["rowsel"])], sa["rowsel"])
    rho = aw.composed_rewards(w)
    ts = get(s.turn_scalar)[:U]
    if w.traj_group is None:
        assert np.array_equal(ts.view(np.uint32), rho.view(np.uint32))
    else:
        P.close(ts, rho, 1e-5, "turn_scalar")
    r = aw.placed_rewards(sa, ts, place_mode)            # copies of the composed rewards as the device holds them
    assert np.array_equal(get(s.tok_reward).view(np.uint32), r.view(np.uint32)), "placed rewards differ"
    worst = aw.recurrence_check(sa, r, w.value, get(adv), get(ret), gamma, lam, gamma_turn, seg_mode)
    assert worst <= 1.0, f"recurrence residual {worst:.3g} x its allowance"
    return sa


@pytest.mark.parametrize("cfg,n_traj,seg_mode,gamma_turn", [(1, 131072, 0, 1.0), (4, 8192, 0, 1.0), (4, 8192, 1, 0.97)])
def test_front_end_at_bandwidth_sizes(cfg, n_traj, seg_mode, gamma_turn):
    w = wl.make_workload(cfg, n_traj=n_traj)
    assert w.n_tokens > 80_000_000
    s, adv, ret = P.gpu_front(w, seg_mode=seg_mode, gamma_turn=gamma_turn)
    sa = check_front_arraywise(w, s, adv, ret, w.place_mode, seg_mode, w.gamma, w.lam, gamma_turn)
    assert np.array_equal(sa["perm"], np.arange(w.n_tokens))      # one model: the stable partition is the identity


def big_random_graph(seed, n_traj, n_models, n_roles):
    """A seeded random workflow graph of millions of tokens: 0-6 turns per trajectory, turn lengths from 0 to 5000
    around the tile edges, per-turn mask densities from none to all, all three reward levels with weights,
    normalisation groups of four, critic values."""
    rng = np.random.default_rng([4242, seed])
    w = wl.make_workload(0)
    turns = rng.integers(0, 7, n_traj)
    U = int(turns.sum())
    lens = rng.choice(np.array([0, 1, 5, 63, 64, 65, 300, 1024, 2049, 5000], np.int64), U)
    w.n_traj, w.n_turns, w.n_roles, w.n_models = n_traj, U, n_roles, n_models
    w.traj_turn_off = np.concatenate([[0], np.cumsum(turns)]).astype(np.int32)
    w.turn_role = rng.integers(0, n_roles, U).astype(np.int32)
    w.role_to_model = rng.integers(0, n_models, n_roles).astype(np.int32)
    w.turn_tok_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    w.n_tokens = int(w.turn_tok_off[-1])
    w.turn_pred_off, w.turn_pred = None, None
    density = rng.choice(np.array([0.0, 0.02, 0.3, 0.9, 1.0], np.float32), U)
    w.tok_mask = (rng.random(w.n_tokens, dtype=np.float32) < np.repeat(density, lens)).astype(np.uint8)
    w.traj_reward = rng.normal(size=n_traj).astype(np.float32)
    w.traj_group = (np.arange(n_traj) // 4).astype(np.int32)
    w.role_reward = rng.normal(size=n_traj * n_roles).astype(np.float32)
    w.turn_reward = rng.normal(size=U).astype(np.float32)
    w.w_role, w.w_turn, w.w_traj = (rng.random(n_roles).astype(np.float32) for _ in range(3))
    w.value = rng.normal(size=w.n_tokens).astype(np.float32)
    return w


@pytest.mark.parametrize("seed,n_models,n_roles,place_mode,seg_mode,gamma,lam,gamma_turn", [
    (0, 3, 5, wl.PLACE_LAST, wl.SEG_TRAJ, 0.99, 0.95, 0.9),
    (1, 8, 13, wl.PLACE_ALL, wl.SEG_TURN, 1.0, 0.9, 1.0),
    (2, 2, 2, wl.PLACE_LAST, wl.SEG_TURN, 1.0, 1.0, 1.0),
])
def test_front_end_on_big_random_multi_model_graphs(seed, n_models, n_roles, place_mode, seg_mode, gamma, lam, gamma_turn):
    w = big_random_graph(seed, 10000, n_models, n_roles)
    assert w.n_tokens > 20_000_000
    s, adv, ret = P.gpu_front(w, place_mode=place_mode, seg_mode=seg_mode, gamma=gamma, lam=lam, gamma_turn=gamma_turn)
    check_front_arraywise(w, s, adv, ret, place_mode, seg_mode, gamma, lam, gamma_turn)
    # the ready batch on the same streams, both cuts: every part holds whole trajectories in shuffled order
    rng = np.random.default_rng(seed)
    order = rng.permutation(w.n_traj).astype(np.int32)
    keep = (rng.random(w.n_traj) < 0.9).astype(np.uint8)
    check_ready_batch_arraywise(w, s, aw.streams(w), keep, order, 8)


def test_front_end_on_many_random_graphs():
    """400 small random workflow graphs (workloads.random_graph) and 40 of up to 700 trajectories on up to 8 models
    and 19 roles: streams, flags, rewards, advantages and both cuts of the ready batch against the array-wise
    restatement.  (The same loop has been run over 60 000 and 1500 of them.)"""
    for seed in range(50000, 50400):
        w, kw = wl.random_graph(seed)
        s, adv, ret = P.gpu_front(w, **kw)
        sa = check_front_arraywise(w, s, adv, ret, kw["place_mode"], kw["seg_mode"], kw["gamma"], kw["lam"], kw["gamma_turn"])
        rng = np.random.default_rng(seed)
        check_ready_batch_arraywise(w, s, sa, (rng.random(w.n_traj) < 0.8).astype(np.uint8), rng.permutation(w.n_traj).astype(np.int32),
                                    int(rng.integers(1, 6)))
    for seed in range(40):
        rng = np.random.default_rng([77, seed])
        K, R = int(rng.integers(1, 9)), int(rng.integers(1, 20))
        w = big_random_graph(1000 + seed, int(rng.integers(1, 700)), K, R)
        if rng.random() < 0.3:
            w.traj_group = None
        if rng.random() < 0.3:
            w.value = None
        kw = dict(seg_mode=int(rng.integers(0, 2)), gamma_turn=float(rng.choice([1.0, 0.8])), place_mode=int(rng.integers(0, 2)),
                  gamma=float(rng.choice([1.0, 0.97])), lam=float(rng.choice([1.0, 0.9])))
        s, adv, ret = P.gpu_front(w, **kw)
        sa = check_front_arraywise(w, s, adv, ret, kw["place_mode"], kw["seg_mode"], kw["gamma"], kw["lam"], kw["gamma_turn"])
        check_ready_batch_arraywise(w, s, sa, (rng.random(w.n_traj) < 0.8).astype(np.uint8), rng.permutation(w.n_traj).astype(np.int32),
                                    int(rng.integers(1, 9)))


def check_ready_batch_arraywise(w, s, sa, keep, order, M):
    for balanced in (False, True):
        want_rows, want_off = aw.ready_batch(w, sa, keep, order, M, balanced)
        rows, mb_off = umas.umas_ready_batch(s, w.traj_turn_off, M, keep, order, balance_rows=balanced)
        assert np.array_equal(mb_off.cpu().numpy(), want_off), f"part offsets, balanced={balanced}"
        assert np.array_equal(rows.cpu().numpy()[:len(want_rows)], want_rows), f"rows, balanced={balanced}"
    # packed under a budget of rows: a budget that gives about 3 M parts per model
    total = int(sa["model_rowsel_off"][-1])
    budget = max(total // (3 * M * w.n_models), 1)
    want_rows, want_off, want_n = aw.ready_batch_packed(w, sa, keep, order, budget)
    rows, mb_off, n_parts = umas.umas_ready_batch_packed(s, w.traj_turn_off, budget, keep, order)
    assert np.array_equal(n_parts.cpu().numpy(), want_n), f"numbers of parts, budget {budget}"
    assert np.array_equal(mb_off.cpu().numpy(), want_off), f"part offsets, budget {budget}"
    assert np.array_equal(rows.cpu().numpy()[:len(want_rows)], want_rows), f"rows, budget {budget}"


def test_shaping_and_ready_batch_at_bandwidth_sizes():
    """The steps around the advantage step on the 101-million-token instance of configuration 1: KL-penalised rewards
    and whitening per (model, role) against the oracle's own array-wise definitions; the ready batch (a tenth of
    the trajectories dropped, a seeded shuffle, eight parts, both cuts) against its array-wise restatement."""
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
    check_ready_batch_arraywise(w, s, aw.streams(w), keep, order, M)
