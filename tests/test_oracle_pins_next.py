"""Pins of the oracle's critic, KL-penalty, whitening and surrogate-variant functions: hand-worked
examples, closed forms, invariants and finite differences (none of them retypes the oracle's formula)."""
import math

import numpy as np
import pytest

from oracle import umas_oracle as orc


# ------------------------------------------------------------------ critic
def test_value_head_brute_force_and_selection():
    rng = np.random.default_rng(3)
    H = rng.normal(size=(5, 4))
    w = rng.normal(size=4)
    V = orc.value_head(H, w, 0.25, np.array([0, 2, 4]))
    for i in range(5):
        want = sum(H[i, j] * w[j] for j in range(4)) + 0.25 if i in (0, 2, 4) else 0.0
        assert abs(V[i] - want) < 1e-14


def test_value_loss_worked_example():
    # row 0: V moved 0.2 from V_old, clip 0.1 -> Vc = 0.9; (1-1.5)^2 = .25 < (0.9-1.5)^2 = .36: clipped, L = .18, g = 0
    # row 1: Vc = 2.5 - 0.1 = 2.4; (2-2)^2 = 0 < .16: clipped, L = .08, g = 0
    # row 2: V = V_old: tie, unclipped, L = .125, g = (0.5-1)/3
    V, Vo, R = np.array([1.0, 2.0, 0.5]), np.array([0.8, 2.5, 0.5]), np.array([1.5, 2.0, 1.0])
    stats, g = orc.value_loss(V, Vo, R, None, np.array([0, 1, 0]), 2, 0.1)
    assert abs(stats[0, 0] - (0.18 + 0.08 + 0.125) / 3) < 1e-15
    assert abs(stats[0, 1] - 2 / 3) < 1e-15 and abs(stats[0, 2] - 3.5 / 3) < 1e-15 and stats[0, 3] == 3
    assert np.allclose(g, [0.0, 0.0, -0.5 / 3], atol=1e-16)
    # per role: role 0 holds rows 0 and 2, role 1 row 1
    assert abs(stats[1, 0] - (0.18 + 0.125) / 2) < 1e-15 and stats[1, 3] == 2
    assert abs(stats[2, 0] - 0.08) < 1e-15 and stats[2, 1] == 1.0


def test_value_loss_without_movement_is_half_mse_and_rowsel():
    rng = np.random.default_rng(5)
    V, R = rng.normal(size=8), rng.normal(size=8)
    rows = np.array([1, 2, 5, 7])
    stats, g = orc.value_loss(V, V.copy(), R, rows, np.zeros(8, np.int32), 1, 0.2)
    assert abs(stats[0, 0] - 0.5 * np.mean((V[rows] - R[rows]) ** 2)) < 1e-15
    assert stats[0, 1] == 0.0
    want = np.zeros(8)
    want[rows] = (V[rows] - R[rows]) / 4
    assert np.allclose(g, want, atol=1e-16)
    # a huge clip range never clips either
    stats2, g2 = orc.value_loss(V, V + rng.normal(size=8), R, rows, np.zeros(8, np.int32), 1, 1e9)
    assert abs(stats2[0, 0] - stats[0, 0]) < 1e-15 and np.allclose(g2, g)


def critic_scalar(H, w, b, Vo, R, rows, eps):
    V = orc.value_head(H, w, b, rows)
    return orc.value_loss(V, Vo, R, rows, np.zeros(len(V), np.int32), 1, eps)[0][0, 0]


def test_critic_backward_matches_finite_differences():
    rng = np.random.default_rng(11)
    n, d = 7, 5
    H, w, b = rng.normal(size=(n, d)), rng.normal(size=d), 0.1
    rows = np.array([0, 1, 3, 4, 6])
    V = orc.value_head(H, w, b, rows)
    Vo = V + rng.normal(size=n) * 0.3
    R = rng.normal(size=n)
    stats, g = orc.value_loss(V, Vo, R, rows, np.zeros(n, np.int32), 1, 0.2)
    assert 0 < stats[0, 1] < 1                       # both branches occur
    dH, dw, db = orc.value_head_backward(H, w, g, rows)
    h = 1e-6
    for j in range(d):
        keep = w[j]
        w[j] = keep + h; fp = critic_scalar(H, w, b, Vo, R, rows, 0.2)
        w[j] = keep - h; fm = critic_scalar(H, w, b, Vo, R, rows, 0.2)
        w[j] = keep
        assert abs((fp - fm) / (2 * h) - dw[j]) < 1e-8
    for idx in [(0, 0), (1, 2), (2, 1), (4, 4), (6, 3)]:
        keep = H[idx]
        H[idx] = keep + h; fp = critic_scalar(H, w, b, Vo, R, rows, 0.2)
        H[idx] = keep - h; fm = critic_scalar(H, w, b, Vo, R, rows, 0.2)
        H[idx] = keep
        assert abs((fp - fm) / (2 * h) - dH[idx]) < 1e-8
    fp = critic_scalar(H, w, b + h, Vo, R, rows, 0.2)
    fm = critic_scalar(H, w, b - h, Vo, R, rows, 0.2)
    assert abs((fp - fm) / (2 * h) - db) < 1e-8
    assert not dH[2].any() and not dH[5].any()      # unselected rows


# ------------------------------------------------------------------ KL-penalised rewards
def test_kl_rewards_by_hand_and_identities():
    r = np.array([0.0, 1.0, 0.0, 0.5], np.float32)
    lp, ref = np.array([-1.0, -2.0, -3.0, -0.5]), np.array([-1.5, -1.0, -3.0, -9.0])
    mask = np.array([1, 1, 1, 0], np.uint8)
    out, kl = orc.kl_penalised_rewards(r, lp, ref, mask, 0.1)
    assert np.allclose(out, [0.0 - 0.1 * 0.5, 1.0 - 0.1 * (-1.0), 0.0, 0.5], atol=1e-15)
    assert abs(kl - (0.5 - 1.0 + 0.0) / 3) < 1e-15
    assert np.array_equal(orc.kl_penalised_rewards(r, lp, ref, mask, 0.0)[0], r.astype(np.float64))
    assert np.array_equal(orc.kl_penalised_rewards(r, lp, lp, mask, 0.7)[0], r.astype(np.float64))
    assert orc.kl_penalised_rewards(r, lp, ref, np.zeros(4, np.uint8), 0.7)[1] == 0.0


# ------------------------------------------------------------------ whitening
def test_whitening_moments_invariance_and_scopes():
    rng = np.random.default_rng(17)
    n = 400
    mask = (rng.random(n) < 0.7).astype(np.uint8)
    role = rng.integers(0, 3, size=n).astype(np.int32)
    off = np.array([0, 250, 400])
    A = rng.normal(size=n) * 3 + 1 + role            # every role has its own level
    A[mask == 0] = 0
    Wm = orc.whiten_advantages(A, mask, role, off, 3, orc.WHITEN_MODEL)
    for k in range(2):
        sel = np.arange(off[k], off[k + 1])[mask[off[k]:off[k + 1]] == 1]
        assert abs(Wm[sel].mean()) < 1e-12 and abs(Wm[sel].std() - 1) < 1e-6
        # second opinion: numpy's own mean/std on the group
        assert np.allclose(Wm[sel], (A[sel] - A[sel].mean()) / np.sqrt(A[sel].var() + 1e-8), atol=1e-12)
    assert not Wm[mask == 0].any()
    # positive affine maps of the advantages change nothing (up to the eps in the denominator)
    assert np.allclose(orc.whiten_advantages(np.where(mask, 5 * A - 2, 0), mask, role, off, 3, orc.WHITEN_MODEL), Wm, atol=1e-7)
    Wr = orc.whiten_advantages(A, mask, role, off, 3, orc.WHITEN_MODEL_ROLE)
    for k in range(2):
        for v in range(3):
            sel = np.arange(off[k], off[k + 1])
            sel = sel[(mask[sel] == 1) & (role[sel] == v)]
            assert abs(Wr[sel].mean()) < 1e-12 and abs(Wr[sel].std() - 1) < 1e-6
    assert np.abs(Wr - Wm).max() > 0.1                # the scopes differ on this input
    # one-role input: both scopes agree; an empty group is left alone
    assert np.array_equal(orc.whiten_advantages(A, mask, np.zeros(n, np.int32), off, 3, orc.WHITEN_MODEL_ROLE),
                          orc.whiten_advantages(A, mask, np.zeros(n, np.int32), off, 3, orc.WHITEN_MODEL))
    assert not orc.whiten_advantages(A, np.zeros(n, np.uint8), role, off, 3, orc.WHITEN_MODEL).any()


# ------------------------------------------------------------------ surrogate variants
def test_variants_reduce_to_the_plain_surrogate():
    rng = np.random.default_rng(19)
    n = 50
    lp, lo = -rng.random(n) * 3, -rng.random(n) * 3
    A, ent = rng.normal(size=n), rng.random(n)
    rows = np.sort(rng.choice(n, 37, replace=False))
    role = rng.integers(0, 2, size=n)
    s0, g0 = orc.ppo_loss(lp, lo, A, ent, rows, role, 2, 0.2)
    s1, g1 = orc.ppo_loss_variants(lp, lo, A, ent, rows, role, 2, 0.2)
    assert np.array_equal(s0, s1) and np.array_equal(g0, g1)
    # a dual-clip constant so large that it never binds changes nothing either
    s2, g2 = orc.ppo_loss_variants(lp, lo, A, ent, rows, role, 2, 0.2, dual_clip=1e9)
    assert np.array_equal(s0, s2) and np.array_equal(g0, g2)


def test_dual_clip_by_hand():
    # A = -1: ratio 5 -> max(5, 1.2) = 5, capped at 3, no gradient; ratio 2 -> 2 < 3, gradient -A ratio / S
    # A = +1: ratio 5 -> max(-5, -1.2) = -1.2 (clipped), never capped
    lo = np.zeros(3)
    lp = np.log(np.array([5.0, 2.0, 5.0]))
    A = np.array([-1.0, -1.0, 1.0])
    stats, g = orc.ppo_loss_variants(lp, lo, A, np.zeros(3), None, np.zeros(3, np.int32), 1, 0.2, dual_clip=3.0)
    assert abs(stats[0, 0] - (3.0 + 2.0 - 1.2) / 3) < 1e-14
    assert np.allclose(g, [0.0, 2.0 / 3, 0.0], atol=1e-15)
    assert abs(stats[0, 1] - 2 / 3) < 1e-15


def total_loss(H, W, ids, logp_old, A, rows, eps, c_ent):
    logp, lse, ent = orc.score(H, W, ids, rows)
    return orc.ppo_loss_variants(logp, logp_old, A, ent, rows, np.zeros(len(ids), np.int32), 1, eps, 0.0, c_ent)[0][0, 0]


def test_entropy_bonus_backward_matches_finite_differences():
    rng = np.random.default_rng(29)
    n, d, V = 8, 5, 11
    H, W = rng.normal(size=(n, d)), rng.normal(size=(V, d)) * 0.6
    ids = rng.integers(0, V, size=n).astype(np.int32)
    rows = np.array([0, 1, 2, 4, 6, 7], np.int32)
    logp, lse, ent = orc.score(H, W, ids, rows)
    logp_old = logp + rng.normal(size=n) * 0.3
    A = rng.normal(size=n)
    c_ent = 0.05
    stats, g = orc.ppo_loss_variants(logp, logp_old, A, ent, rows, np.zeros(n, np.int32), 1, 0.2, 0.0, c_ent)
    plain, _ = orc.ppo_loss(logp, logp_old, A, ent, rows, np.zeros(n, np.int32), 1, 0.2)
    assert abs(stats[0, 0] - (plain[0, 0] - c_ent * plain[0, 2])) < 1e-15
    dH, dW = orc.lm_head_backward_entropy(H, W, ids, lse, ent, g, c_ent, len(rows), rows)
    h = 1e-6
    for (arr, grad) in ((H, dH), (W, dW)):
        for idx in [(0, 0), (1, 3), (2, 4), (4, 1), (7, 2), (6, 0), (5, 1)]:
            keep = arr[idx]
            arr[idx] = keep + h; fp = total_loss(H, W, ids, logp_old, A, rows, 0.2, c_ent)
            arr[idx] = keep - h; fm = total_loss(H, W, ids, logp_old, A, rows, 0.2, c_ent)
            arr[idx] = keep
            assert abs((fp - fm) / (2 * h) - grad[idx]) < 1e-8
    # with coefficient 0 it is the plain backward
    dH0, dW0 = orc.lm_head_backward_entropy(H, W, ids, lse, ent, g, 0.0, len(rows), rows)
    dH1, dW1 = orc.lm_head_backward(H, W, ids, lse, g, rows)
    assert np.allclose(dH0, dH1, atol=1e-15) and np.allclose(dW0, dW1, atol=1e-15)
    # W = 0: uniform softmax, entropy log V is a maximum, so the entropy term has no gradient
    Wz = np.zeros((V, d))
    lz, lsez, entz = orc.score(H, Wz, ids, rows)
    assert np.allclose(entz[rows], math.log(V))
    dHz, dWz = orc.lm_head_backward_entropy(H, Wz, ids, lsez, entz, np.zeros(n), c_ent, len(rows), rows)
    assert np.abs(dHz).max() < 1e-15 and np.abs(dWz).max() < 1e-15


def test_kl_loss_term_by_hand_expectation_and_finite_differences():
    n = 3
    z3 = np.zeros(n, np.int32)
    # by hand: A = 0 leaves only the penalty; x = ln 2 -> e^x - x - 1 = 1 - ln 2, x = 0 -> 0, x = -ln 2 -> ln 2 - 1/2
    lp = np.zeros(n)
    ref = np.array([math.log(2.0), 0.0, -math.log(2.0)])
    stats, g = orc.ppo_loss_variants(lp, lp, np.zeros(n), np.zeros(n), None, z3, 1, 0.2, kl_coef=0.5, logp_ref=ref)
    assert abs(stats[0, 0] - 0.5 * ((1 - math.log(2.0)) + 0.0 + (math.log(2.0) - 0.5)) / 3) < 1e-15
    assert np.allclose(g, 0.5 * np.array([1 - 2.0, 0.0, 1 - 0.5]) / 3, atol=1e-16)
    # every term is non-negative and vanishes only where the two policies agree on the token
    rng = np.random.default_rng(41)
    x = rng.normal(size=1000)
    assert (np.exp(x) - x - 1 >= 0).all()
    # its mean over tokens drawn from the policy is KL(policy || reference): exact enumeration of a small distribution
    p = rng.random(7); p /= p.sum()
    q = rng.random(7); q /= q.sum()
    st7, _ = orc.ppo_loss_variants(np.log(p), np.log(p), np.zeros(7), np.zeros(7), None, np.zeros(7, np.int32), 1, 0.2,
                                   kl_coef=1.0, logp_ref=np.log(q))
    per_token = np.exp(np.log(q) - np.log(p)) - (np.log(q) - np.log(p)) - 1
    assert abs(float((p * per_token).sum()) - float((p * np.log(p / q)).sum())) < 1e-14       # the identity itself
    assert abs(st7[0, 0] - per_token.mean()) < 1e-15                                          # and what the oracle averages
    # gradient with respect to logp by central differences, with the surrogate active and a row selection
    n = 9
    lp, lo, ref = -rng.random(n) * 2, -rng.random(n) * 2, -rng.random(n) * 2
    A, ent = rng.normal(size=n), rng.random(n)
    rows = np.array([0, 2, 3, 5, 8], np.int32)
    role = np.zeros(n, np.int32)
    f = lambda v: orc.ppo_loss_variants(v, lo, A, ent, rows, role, 1, 0.2, kl_coef=0.3, logp_ref=ref)[0][0, 0]
    _, g = orc.ppo_loss_variants(lp, lo, A, ent, rows, role, 1, 0.2, kl_coef=0.3, logp_ref=ref)
    h = 1e-6
    for i in range(n):
        e = np.zeros(n); e[i] = h
        assert abs((f(lp + e) - f(lp - e)) / (2 * h) - g[i]) < 1e-8
    assert not g[[1, 4, 6, 7]].any()
    # coefficient 0 is the plain surrogate
    s0, g0 = orc.ppo_loss(lp, lo, A, ent, rows, role, 1, 0.2)
    s1, g1 = orc.ppo_loss_variants(lp, lo, A, ent, rows, role, 1, 0.2, kl_coef=0.0, logp_ref=ref)
    assert np.array_equal(s0, s1) and np.array_equal(g0, g1)


# ------------------------------------------------------------------ ready batch
def _routed(seed, n_traj=7, phi=(0, 1, 0)):
    rng = np.random.default_rng(seed)
    roles, lens = [], []
    for b in range(n_traj):
        k = int(rng.integers(1, 5))
        roles.append([int(rng.integers(0, len(phi))) for _ in range(k)])
        lens.append([int(rng.integers(0, 6)) for _ in range(k)])
    tto = np.concatenate([[0], np.cumsum([len(r) for r in roles])])
    role = np.array([v for r in roles for v in r], np.int32)
    tok_off = np.concatenate([[0], np.cumsum([l for ls in lens for l in ls])])
    mask = (rng.random(int(tok_off[-1])) < 0.7).astype(np.uint8)
    st = orc.route(max(phi) + 1, np.array(phi), tto, role, tok_off, mask)
    turn_traj = np.repeat(np.arange(n_traj), np.diff(tto))
    return st, tto, turn_traj


def test_ready_batch_hand_example():
    # 3 trajectories of one turn each (lengths 2, 3, 2), one model, all tokens valid; shuffle (2, 0, 1), drop none,
    # two minibatches: kept order 2,0,1 -> parts 0,0,1 -> minibatch 0 = rows of traj 2 then traj 0, minibatch 1 = traj 1
    st = orc.route(1, np.array([0]), np.array([0, 1, 2, 3]), np.zeros(3, np.int32), np.array([0, 2, 5, 7]), np.ones(7, np.uint8))
    rows, off = orc.ready_batch(st, np.array([0, 1, 2, 3]), np.ones(3), np.array([2, 0, 1]), 2)
    assert rows.tolist() == [5, 6, 0, 1, 2, 3, 4] and off.tolist() == [[0, 4, 7]]
    # dropping trajectory 0: kept order 2,1 -> one each
    rows, off = orc.ready_batch(st, np.array([0, 1, 2, 3]), np.array([0, 1, 1]), np.array([2, 0, 1]), 2)
    assert rows.tolist() == [5, 6, 2, 3, 4] and off.tolist() == [[0, 2, 5]]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_ready_batch_partition_properties(seed):
    st, tto, turn_traj = _routed(seed)
    n_traj = len(tto) - 1
    rng = np.random.default_rng(100 + seed)
    keep = (rng.random(n_traj) < 0.75).astype(np.uint8)
    keep[int(rng.integers(0, n_traj))] = 1
    order = rng.permutation(n_traj)
    M = 3
    rows, off = orc.ready_batch(st, tto, keep, order, M)
    kept = [b for b in order if keep[b]]
    sizes = [sum(1 for q in range(len(kept)) if q * M // len(kept) == k) for k in range(M)]
    assert max(sizes) - min(sizes) <= 1
    for m in range(len(st["model_tok_off"]) - 1):
        a = int(st["model_tok_off"][m])
        ra, re = int(st["model_rowsel_off"][m]), int(st["model_rowsel_off"][m + 1])
        want_all = [int(r) for r in st["rowsel"][ra:re] if keep[turn_traj[st["tok_turn"][a + r]]]]
        got_all = rows[off[m, 0]:off[m, M]].tolist()
        assert sorted(got_all) == want_all and len(set(got_all)) == len(got_all)
        q0 = 0
        for k in range(M):
            trajs = kept[q0:q0 + sizes[k]]
            q0 += sizes[k]
            got = rows[off[m, k]:off[m, k + 1]]
            got_traj = [int(turn_traj[st["tok_turn"][a + r]]) for r in got]
            assert set(got_traj) <= set(trajs)
            # trajectory by trajectory in shuffled order, rows ascending inside a trajectory
            seen = [b for i, b in enumerate(got_traj) if i == 0 or got_traj[i - 1] != b]
            assert seen == [b for b in trajs if b in set(got_traj)]
            for b in set(got_traj):
                rb = [int(r) for r, t in zip(got, got_traj) if t == b]
                assert rb == sorted(rb)
    # everything kept, identity order, one minibatch: the selection itself
    rows1, off1 = orc.ready_batch(st, tto, np.ones(n_traj), np.arange(n_traj), 1)
    assert np.array_equal(rows1, st["rowsel"]) and np.array_equal(off1[:, 0], st["model_rowsel_off"][:-1])


def test_ready_batch_balanced_by_rows_hand_example():
    # 4 trajectories of one turn each with 6, 1, 1, 4 valid tokens, one model, identity order, two parts.
    # By trajectories: {0, 1} | {2, 3} = 7 + 5 rows.  By rows (T = 12, first rows 0, 6, 7, 8 -> parts 0, 1, 1, 1): {0} | {1, 2, 3}.
    st = orc.route(1, np.array([0]), np.arange(5), np.zeros(4, np.int32), np.array([0, 6, 7, 8, 12]), np.ones(12, np.uint8))
    rows, off = orc.ready_batch(st, np.arange(5), np.ones(4), np.arange(4), 2)
    assert off.tolist() == [[0, 7, 12]]
    rows_b, off_b = orc.ready_batch(st, np.arange(5), np.ones(4), np.arange(4), 2, balance_rows=True)
    assert off_b.tolist() == [[0, 6, 12]] and rows_b.tolist() == rows.tolist()
    # three parts: thresholds ceil(12 k / 3) = 4, 8: first rows 0 | 6, 7 | 8 -> {0} | {1, 2} | {3}
    _, off_3 = orc.ready_batch(st, np.arange(5), np.ones(4), np.arange(4), 3, balance_rows=True)
    assert off_3.tolist() == [[0, 6, 8, 12]]
    # shuffled and filtered: order 3, 1, 0, 2 without trajectory 1 -> rows 4, 6, 1 -> T = 11, first rows 0, 4, 10 -> parts 0, 0, 1
    rows_s, off_s = orc.ready_batch(st, np.arange(5), np.array([1, 0, 1, 1]), np.array([3, 1, 0, 2]), 2, balance_rows=True)
    assert off_s.tolist() == [[0, 10, 11]] and rows_s.tolist() == [8, 9, 10, 11, 0, 1, 2, 3, 4, 5, 7]


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_ready_batch_balanced_by_rows_properties(seed):
    """The same rows in the same order as the split by trajectories; cuts only between trajectories; part k starts
    at the first trajectory whose first row is at or behind ceil(k T / M) (the rule stated from the cut's side);
    every part holds T / M rows give or take the rows of one trajectory."""
    st, tto, turn_traj = _routed(seed)
    n_traj = len(tto) - 1
    rng = np.random.default_rng(200 + seed)
    keep = (rng.random(n_traj) < 0.8).astype(np.uint8)
    keep[int(rng.integers(0, n_traj))] = 1
    order = rng.permutation(n_traj)
    M = int(rng.integers(2, 6))
    rows, off = orc.ready_batch(st, tto, keep, order, M)
    rows_b, off_b = orc.ready_batch(st, tto, keep, order, M, balance_rows=True)
    assert np.array_equal(rows, rows_b) and np.array_equal(off[:, [0, M]], off_b[:, [0, M]])
    kept = [b for b in order if keep[b]]
    for m in range(len(st["model_tok_off"]) - 1):
        a = int(st["model_tok_off"][m])
        got = rows_b[off_b[m, 0]:off_b[m, M]]
        got_traj = [int(turn_traj[st["tok_turn"][a + r]]) for r in got]
        n_rows = {b: got_traj.count(b) for b in kept}
        first = np.concatenate([[0], np.cumsum([n_rows[b] for b in kept])])       # first row of every kept trajectory, then T
        T = int(first[-1])
        for k in range(M + 1):
            thr = -(-k * T // M)
            start = int(np.argmax(first >= thr))                                   # first trajectory at or behind the threshold
            assert off_b[m, k] - off_b[m, 0] == first[start]
        if T:
            sizes = np.diff(off_b[m])
            biggest = max(n_rows.values())
            assert sizes.max() <= -(-T // M) + biggest and sizes.min() >= T // M - biggest


def test_ready_batch_packed_hand_example():
    # 5 trajectories of one turn each with 3, 2, 4, 1, 2 valid tokens, one model, identity order, budget 5:
    # 3 + 2 = 5 fits | 4 + 1 = 5 fits | 2 -> parts of 5, 5, 2 rows.  Budget 4: 3 | 2 | 4 | 1 + 2.  Budget 3: 3 | 2 | 4 alone
    # (more than the budget, never split) | 1 + 2.
    tto = np.arange(6)
    st = orc.route(1, np.array([0]), tto, np.zeros(5, np.int32), np.array([0, 3, 5, 9, 10, 12]), np.ones(12, np.uint8))
    rows, off, n = orc.ready_batch_packed(st, tto, np.ones(5), np.arange(5), 5)
    assert rows.tolist() == list(range(12)) and n.tolist() == [3] and off.tolist() == [[0, 5, 10, 12, 12, 12]]
    _, off, n = orc.ready_batch_packed(st, tto, np.ones(5), np.arange(5), 4)
    assert n.tolist() == [4] and off.tolist() == [[0, 3, 5, 9, 12, 12]]
    _, off, n = orc.ready_batch_packed(st, tto, np.ones(5), np.arange(5), 3)
    assert n.tolist() == [4] and off.tolist() == [[0, 3, 5, 9, 12, 12]]
    # a budget of one row: every trajectory with rows by itself; a budget of everything: one part
    _, off, n = orc.ready_batch_packed(st, tto, np.ones(5), np.arange(5), 1)
    assert n.tolist() == [5] and off.tolist() == [[0, 3, 5, 9, 10, 12]]
    _, off, n = orc.ready_batch_packed(st, tto, np.ones(5), np.arange(5), 12)
    assert n.tolist() == [1] and off.tolist() == [[0, 12, 12, 12, 12, 12]]
    # shuffled and filtered: order 4, 2, 0, 3, 1 without trajectory 3 -> rows 2, 4, 3, 2; budget 6: 2 + 4 | 3 + 2
    rows, off, n = orc.ready_batch_packed(st, tto, np.array([1, 1, 1, 0, 1]), np.array([4, 2, 0, 3, 1]), 6)
    assert rows.tolist() == [10, 11, 5, 6, 7, 8, 0, 1, 2, 3, 4] and n.tolist() == [2] and off.tolist() == [[0, 6, 11, 11, 11, 11]]
    # nothing kept: no part
    rows, off, n = orc.ready_batch_packed(st, tto, np.zeros(5), np.arange(5), 6)
    assert len(rows) == 0 and n.tolist() == [0] and not off.any()


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6])
def test_ready_batch_packed_properties(seed):
    """What fixes a next-fit packing: the rows and their order are those of the plain ready batch; cuts lie between
    trajectories; no part is empty; a part is over the budget only if it is one trajectory; and no cut could have come
    later (a part together with the first trajectory of the next one is over the budget).  With trajectory sizes that
    all fit, the number of parts is at least ceil(T / budget) and less than 2 T / budget + 1 (two neighbouring parts
    together always exceed the budget)."""
    st, tto, turn_traj = _routed(seed, n_traj=11)
    n_traj = len(tto) - 1
    rng = np.random.default_rng(300 + seed)
    keep = (rng.random(n_traj) < 0.85).astype(np.uint8)
    order = rng.permutation(n_traj)
    budget = int(rng.integers(1, 12))
    rows, off, n_parts = orc.ready_batch_packed(st, tto, keep, order, budget)
    rows1, off1 = orc.ready_batch(st, tto, keep, order, 1)
    assert np.array_equal(rows, rows1)
    for m in range(len(st["model_tok_off"]) - 1):
        a = int(st["model_tok_off"][m])
        k = int(n_parts[m])
        assert off[m, 0] == off1[m, 0] and (off[m, k:] == off1[m, 1]).all()
        sizes = np.diff(off[m, :k + 1])
        assert (sizes > 0).all()
        base = int(off[m, 0])
        traj_of = [int(turn_traj[st["tok_turn"][a + r]]) for r in rows[base:int(off1[m, 1])]]   # of the model's rows
        for p in range(k):
            lo, hi = int(off[m, p]) - base, int(off[m, p + 1]) - base
            trajs = traj_of[lo:hi]
            if p + 1 < k:
                assert trajs[-1] != traj_of[hi]                                    # the cut lies between two trajectories
                first_next = traj_of[hi]
                size_next = sum(1 for t in traj_of[hi:int(off[m, p + 2]) - base] if t == first_next)
                assert sizes[p] + size_next > budget                             # the next trajectory did not fit
            if sizes[p] > budget:
                assert len(set(trajs)) == 1
        T = len(traj_of)
        assert T == int(off[m, k] - off[m, 0])
        biggest = max([traj_of.count(t) for t in set(traj_of)], default=0)
        if T and biggest <= budget:
            assert -(-T // budget) <= k < 2 * T / budget + 1
