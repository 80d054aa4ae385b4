"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only).

Nothing here compares the oracle with itself: expectations are hand-worked workflow
examples (tests/golden/), closed forms, invariants, brute force in pure Python and
second-opinion library routines.
"""
import math
import os

import numpy as np
import pytest

from oracle import umas_oracle as orc
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    rows, kv = [], {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            try:
                kv[parts[0]] = [float(x) for x in parts[1:]]
            except ValueError:
                rows.append(parts)
            else:
                rows.append(parts)
    return rows, kv


def chain_graph(turn_roles_per_traj, lens_per_traj):
    """Thin graph arrays of trajectories given as lists of role ids and turn lengths."""
    turn_role = np.array([r for t in turn_roles_per_traj for r in t], np.int32)
    traj_turn_off = np.concatenate([[0], np.cumsum([len(t) for t in turn_roles_per_traj])]).astype(np.int32)
    lens = np.array([l for t in lens_per_traj for l in t], np.int64)
    turn_tok_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    return traj_turn_off, turn_role, turn_tok_off


# ------------------------------------------------------------------ O1 composition
def test_compose_workflow_ab_rule():
    # r_v = F1 + r_v^fmt for every trainable node (Workflows A and B): F1 = 0.5 shared
    # at trajectory level, format penalties (0, -0.25, 0) at role level.
    tto, role, _ = chain_graph([[0, 1, 2]], [[4, 4, 4]])
    rho = orc.compose_rewards(tto, role, 3, role_reward=np.array([0, -0.25, 0], np.float32),
                              traj_reward=np.array([0.5], np.float32))
    assert rho.dtype == np.float32
    assert rho.tolist() == [0.5, 0.25, 0.5]


def test_compose_weights_and_levels_by_hand():
    # two trajectories, roles (0,1) and (1,0,1); every level and weight distinct so that a
    # swapped index or dropped term changes the result.
    tto, role, _ = chain_graph([[0, 1], [1, 0, 1]], [[1, 1], [1, 1, 1]])
    Rr = np.array([1, 2, 4, 8], np.float32)            # [traj, role]
    Rt = np.array([0.5, 0.25, 0.125, 16, 32], np.float32)
    Rj = np.array([64, 128], np.float32)
    wr, wt, wj = (np.array(x, np.float32) for x in ([1, 2], [4, 8], [0.5, 0.25]))
    rho = orc.compose_rewards(tto, role, 2, Rr, Rt, Rj, wr, wt, wj)
    want = [1 * 1 + 4 * 0.5 + 0.5 * 64,      # traj 0, role 0
            2 * 2 + 8 * 0.25 + 0.25 * 64,    # traj 0, role 1
            2 * 8 + 8 * 0.125 + 0.25 * 128,  # traj 1, role 1
            1 * 4 + 4 * 16 + 0.5 * 128,      # traj 1, role 0
            2 * 8 + 8 * 32 + 0.25 * 128]     # traj 1, role 1
    assert rho.tolist() == want


# ------------------------------------------------------------------ O2 group normalisation
def test_group_norm_closed_form_bernoulli():
    eps = 1e-6
    for k in range(1, 8):
        R = np.array([1.0] * k + [0.0] * (8 - k))
        out = orc.group_normalise(R, np.zeros(8, np.int32), eps)
        p = k / 8
        sigma = math.sqrt(p * (1 - p))
        assert np.allclose(out[:k], (1 - p) / (sigma + eps), rtol=0, atol=1e-14)
        assert np.allclose(out[k:], -p / (sigma + eps), rtol=0, atol=1e-14)
        # up to eps these are +sqrt((8-k)/k) and -sqrt(k/(8-k))
        assert abs(out[0] - math.sqrt((8 - k) / k)) < 1e-5
        assert abs(out[-1] + math.sqrt(k / (8 - k))) < 1e-5


def test_group_norm_invariants_and_constant_group():
    rng = np.random.default_rng(1)
    R = rng.normal(size=24)
    g = np.array([0] * 8 + [2] * 8 + [1] * 8, np.int32)[rng.permutation(24)]
    eps = 1e-6
    out = orc.group_normalise(R, g, eps)
    for gid in (0, 1, 2):
        sel = g == gid
        sigma = R[sel].std()  # numpy's population std: a library second opinion
        assert abs(out[sel].sum()) < 1e-12
        assert abs((out[sel] ** 2).sum() - 8 * sigma ** 2 / (sigma + eps) ** 2) < 1e-10
    assert orc.group_normalise(np.full(8, 0.7), np.zeros(8, np.int32)).tolist() == [0.0] * 8
    assert orc.group_normalise(R, None).tolist() == R.tolist()


# ------------------------------------------------------------------ O3 routing
def brute_route(n_models, phi, tto, role, tok_off):
    """Independent statement with comprehensions: stream m = tokens of turns mapped to m."""
    streams = []
    for m in range(n_models):
        streams.append([(t, u) for u in range(len(role)) if phi[role[u]] == m
                        for t in range(tok_off[u], tok_off[u + 1])])
    return streams


@pytest.mark.parametrize("phi", [[0, 0, 0], [0, 1, 2], [1, 0, 1], [2, 2, 0]])
def test_route_against_brute_force(phi):
    rng = np.random.default_rng(7)
    trajs = [[0, 1, 2, 1], [2], [1, 1, 0], [0, 2, 2, 1, 0]]
    lens = [[int(rng.integers(1, 6)) for _ in t] for t in trajs]
    tto, role, tok_off = chain_graph(trajs, lens)
    N = int(tok_off[-1])
    mask = (rng.random(N) < 0.6).astype(np.uint8)
    K = 3
    st = orc.route(K, np.array(phi, np.int32), tto, role, tok_off, mask)
    want = brute_route(K, phi, tto, role, tok_off)
    flat = [x for s in want for x in s]
    assert st["perm"].tolist() == [t for t, _ in flat]
    assert st["tok_turn"].tolist() == [u for _, u in flat]
    assert st["tok_role"].tolist() == [int(role[u]) for _, u in flat]
    assert st["model_tok_off"].tolist() == np.concatenate([[0], np.cumsum([len(s) for s in want])]).tolist()
    assert sorted(st["perm"].tolist()) == list(range(N))          # a permutation: disjoint, complete
    assert st["tok_mask"].tolist() == mask[st["perm"]].tolist()
    # rowsel: stream-relative positions with mask = 1
    for m in range(K):
        a, e = st["model_tok_off"][m], st["model_tok_off"][m + 1]
        rs = st["rowsel"][st["model_rowsel_off"][m]:st["model_rowsel_off"][m + 1]]
        assert rs.tolist() == [p - a for p in range(a, e) if mask[st["perm"][p]]]
    # turn segments tile each stream in order; trajectory runs are unions of them
    assert st["turn_seg_off"][-1] == N and st["traj_seg_off"][-1] == N
    turn_traj = np.repeat(np.arange(len(trajs)), np.diff(tto))
    for s in range(len(st["seg_turn"])):
        u = st["seg_turn"][s]
        assert st["turn_seg_off"][s + 1] - st["turn_seg_off"][s] == tok_off[u + 1] - tok_off[u]
    runs = []
    for m in range(K):
        last = None
        for u in range(len(role)):
            if phi[role[u]] == m:
                if last != (m, turn_traj[u]):
                    runs.append(0)
                    last = (m, turn_traj[u])
                runs[-1] += int(tok_off[u + 1] - tok_off[u])
    assert np.diff(st["traj_seg_off"]).tolist() == runs
    assert st["model_trajrun_off"][-1] == len(runs)


def test_route_full_sharing_is_identity_and_full_separation_is_by_role():
    tto, role, tok_off = chain_graph([[0, 1, 2], [2, 1, 0]], [[2, 3, 1], [1, 2, 2]])
    N = int(tok_off[-1])
    mask = np.ones(N, np.uint8)
    shared = orc.route(1, np.array([0, 0, 0], np.int32), tto, role, tok_off, mask)
    assert shared["perm"].tolist() == list(range(N))
    sep = orc.route(3, np.array([0, 1, 2], np.int32), tto, role, tok_off, mask)
    for v in range(3):
        a, e = sep["model_tok_off"][v], sep["model_tok_off"][v + 1]
        assert set(sep["tok_role"][a:e].tolist()) == {v}
    # role identities are preserved regardless of phi
    assert sorted(zip(shared["perm"], shared["tok_role"])) == sorted(zip(sep["perm"], sep["tok_role"]))


# ------------------------------------------------------------------ O4 placement
def workflow_d(lens=3, phi=(0, 0, 0), mask=None):
    rows, kv = read_golden("workflow_d_rewards.txt")
    turns = [r for r in rows if len(r) == 4 and r[0][0] in "PCR"]
    roles = [int(r[1]) for r in turns]
    rew = np.array([float(r[3]) for r in turns], np.float32)
    steps = [int(r[2]) for r in turns]
    tto, role, tok_off = chain_graph([roles], [[lens] * len(roles)])
    N = int(tok_off[-1])
    mask = np.ones(N, np.uint8) if mask is None else mask
    K = max(phi) + 1
    st = orc.route(K, np.array(phi, np.int32), tto, role, tok_off, mask)
    rho = orc.compose_rewards(tto, role, 3, turn_reward=rew)
    return st, rho, tto, role, tok_off, rew, steps, kv


def test_place_workflow_d_last_token():
    st, rho, tto, role, tok_off, rew, steps, _ = workflow_d(lens=3)
    assert steps == list(range(1, 9))
    assert rho.tolist() == rew.tolist() == [0.25, 0.25, 0.25, 0.25, 0.25, 0.5, 0.5, 0.5]
    r = orc.place_rewards(st, rho, orc.PLACE_LAST)
    want = np.zeros(24, np.float32)
    want[2::3] = rew
    assert r.tolist() == want.tolist()
    r_all = orc.place_rewards(st, rho, orc.PLACE_ALL)
    assert r_all.tolist() == np.repeat(rew, 3).tolist()


def test_place_respects_mask_and_empty_turns():
    mask = np.ones(24, np.uint8)
    mask[2] = 0              # last token of P0 masked -> reward moves to token 1
    mask[3:6] = 0            # C0 entirely masked -> nothing placed
    mask[7] = 0              # interior masked token of R0: no effect in LAST mode
    st, rho, *_ = workflow_d(lens=3, mask=mask)
    r = orc.place_rewards(st, rho, orc.PLACE_LAST)
    want = np.zeros(24, np.float32)
    want[1] = 0.25
    want[8] = 0.25
    want[11], want[14], want[17], want[20], want[23] = 0.25, 0.25, 0.5, 0.5, 0.5
    assert r.tolist() == want.tolist()
    r_all = orc.place_rewards(st, rho, orc.PLACE_ALL)
    assert r_all.tolist() == (np.repeat(rho, 3) * mask).tolist()


def test_token_rewards_do_not_depend_on_phi():
    per_phi = []
    for phi in [(0, 0, 0), (0, 1, 2), (1, 0, 1)]:
        st, rho, *_ = workflow_d(lens=2, phi=phi)
        r = orc.place_rewards(st, rho, orc.PLACE_LAST)
        glob = np.zeros_like(r)
        glob[st["perm"]] = r
        per_phi.append(glob.tolist())
    assert per_phi[0] == per_phi[1] == per_phi[2]


# ------------------------------------------------------------------ O5 scan
def gae_double_sum(r, V, gamma, lam):
    """The printed closed form on one unmasked segment, V beyond the end = 0."""
    T = len(r)
    Vn = list(V) + [0.0]
    delta = [r[t] + gamma * Vn[t + 1] - Vn[t] for t in range(T)]
    return [sum((gamma * lam) ** l * delta[t + l] for l in range(T - t)) for t in range(T)]


def single_stream(lens, mask=None):
    tto, role, tok_off = chain_graph([[0] * len(lens)], [lens])
    N = int(tok_off[-1])
    mask = np.ones(N, np.uint8) if mask is None else np.asarray(mask, np.uint8)
    st = orc.route(1, np.array([0], np.int32), tto, role, tok_off, mask)
    return st, tto


def test_gae_worked_example_and_mask_insertion():
    _, kv = read_golden("gae_worked_example.txt")
    st, tto = single_stream([3])
    adv, ret = orc.advantages(st, tto, kv["r"], kv["V"], kv["gamma"][0], kv["lam"][0])
    assert np.allclose(adv, kv["adv"], atol=1e-15) and np.allclose(ret, kv["ret"], atol=1e-15)
    # masked tokens anywhere leave the valid tokens' results unchanged and output 0
    mask = [0, 1, 0, 0, 1, 1, 0]
    r = [9, kv["r"][0], 9, 9, kv["r"][1], kv["r"][2], 9]
    V = [9, kv["V"][0], 9, 9, kv["V"][1], kv["V"][2], 9]
    st, tto = single_stream([7], mask)
    adv, ret = orc.advantages(st, tto, r, V, kv["gamma"][0], kv["lam"][0])
    assert np.allclose(adv[[1, 4, 5]], kv["adv"], atol=1e-15)
    assert np.allclose(ret[[1, 4, 5]], kv["ret"], atol=1e-15)
    assert adv[[0, 2, 3, 6]].tolist() == [0, 0, 0, 0] and ret[[0, 2, 3, 6]].tolist() == [0, 0, 0, 0]


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.99, 0.95), (0.9, 0.0), (1.0, 1.0), (0.7, 0.3)])
def test_gae_equals_printed_double_sum(gamma, lam):
    rng = np.random.default_rng(3)
    lens = [5, 1, 9, 3]
    st, tto = single_stream(lens)
    N = sum(lens)
    r, V = rng.normal(size=N), rng.normal(size=N)
    adv, ret = orc.advantages(st, tto, r, V, gamma, lam, seg_mode=orc.SEG_TURN)
    a = 0
    for L in lens:
        want = gae_double_sum(r[a:a + L], V[a:a + L], gamma, lam)
        assert np.allclose(adv[a:a + L], want, rtol=0, atol=1e-12)
        a += L
    assert np.allclose(ret - adv, V, atol=1e-12)
    if lam == 0.0:  # one-step TD residual
        Vn = np.concatenate([V[1:], [0]])
        ends = np.cumsum(lens) - 1
        Vn[ends] = 0
        assert np.allclose(adv, r + gamma * Vn - V, atol=1e-12)


def test_gae_gamma_lam_one_is_masked_suffix_sum_and_modes_agree():
    rng = np.random.default_rng(5)
    lens = [6, 4, 7]
    N = sum(lens)
    mask = (rng.random(N) < 0.7).astype(np.uint8)
    mask[[5, 9]] = 1
    st, tto = single_stream(lens, mask)
    r = rng.normal(size=N) * mask
    adv, _ = orc.advantages(st, tto, r, None, 1.0, 1.0)
    a = 0
    for L in lens:
        seg = r[a:a + L]
        want = np.cumsum(seg[::-1])[::-1] * mask[a:a + L]   # textbook reverse cumulative sum
        assert np.allclose(adv[a:a + L], want, atol=1e-13)
        a += L
    # with gamma = lam = 1 and V = 0, placing a turn reward on the last valid token or
    # on ... the suffix sum at the last valid token equals the reward itself
    rho = np.array([0.5, -1.0, 2.0], np.float32)
    r_last = orc.place_rewards(st, rho, orc.PLACE_LAST)
    adv_last, _ = orc.advantages(st, tto, r_last, None, 1.0, 1.0)
    assert np.allclose(adv_last, np.repeat(rho, lens) * mask, atol=0)


def test_traj_mode_workflow_d_coder_stream_telescopes():
    st, rho, tto, role, tok_off, rew, steps, kv = workflow_d(lens=3, phi=(0, 1, 2))
    r = orc.place_rewards(st, rho, orc.PLACE_LAST)
    a, e = st["model_tok_off"][1], st["model_tok_off"][2]       # the coder's model
    for key, gt in (("coder_adv_gamma_turn_1", 1.0), ("coder_adv_gamma_turn_half", 0.5)):
        adv, _ = orc.advantages(st, tto, r, None, 1.0, 1.0, gamma_turn=gt, seg_mode=orc.SEG_TRAJ)
        assert adv[a:e].tolist() == np.repeat(kv[key], 3).tolist()
    # reflector stream: s_2 - s_0
    a, e = st["model_tok_off"][2], st["model_tok_off"][3]
    adv, _ = orc.advantages(st, tto, r, None, 1.0, 1.0, seg_mode=orc.SEG_TRAJ)
    assert adv[a] == 0.75


def gae_double_sum_varying_discount(r, V, disc, lam):
    """A_t = sum_l (prod_{j<l} disc_{t+j} lam) delta_{t+l}, delta_t = r_t + disc_t V_{t+1} - V_t: the printed closed
    form with the discount of the transition t -> t+1 given per transition, V beyond the end = 0."""
    T = len(r)
    Vn = list(V) + [0.0]
    delta = [r[t] + disc[t] * Vn[t + 1] - Vn[t] for t in range(T)]
    out = []
    for t in range(T):
        acc, w = 0.0, 1.0
        for l in range(T - t):
            acc += w * delta[t + l]
            w *= disc[t + l] * lam
        out.append(acc)
    return out


def test_traj_mode_with_values_worked_example():
    # two turns of one trajectory at steps 1 and 3 inside one model stream, value estimates given
    _, kv = read_golden("gae_traj_value_worked_example.txt")
    tto, role, tok_off = chain_graph([[0, 1, 0]], [[2, 5, 1]])
    st = orc.route(2, np.array([0, 1], np.int32), tto, role, tok_off, np.ones(8, np.uint8))
    a, e = int(st["model_tok_off"][0]), int(st["model_tok_off"][1])
    assert e - a == 3 and st["traj_seg_off"][:2].tolist() == [0, 3]
    r, V = np.zeros(8), np.zeros(8)
    r[a:e], V[a:e] = kv["r"], kv["V"]
    adv, ret = orc.advantages(st, tto, r, V, kv["gamma"][0], kv["lam"][0], gamma_turn=kv["gamma_turn"][0],
                              seg_mode=orc.SEG_TRAJ)
    assert adv[a:e].tolist() == kv["adv"] and ret[a:e].tolist() == kv["ret"]


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.99, 0.95), (0.9, 0.0), (0.7, 0.3)])
def test_traj_mode_with_values_equals_printed_double_sum_on_the_concatenated_run(gamma, lam):
    # gamma_turn = 1: a trajectory run is one episode, so the printed closed form holds on the concatenation of
    # its turns, value estimates included (the next token's value crosses turn boundaries unchanged)
    rng = np.random.default_rng(17)
    trajs, lens = [[0, 0, 0, 0], [0, 0, 0]], [[4, 1, 6, 3], [2, 5, 2]]
    tto, role, tok_off = chain_graph(trajs, lens)
    N = int(tok_off[-1])
    st = orc.route(1, np.array([0], np.int32), tto, role, tok_off, np.ones(N, np.uint8))
    r, V = rng.normal(size=N), rng.normal(size=N)
    adv, ret = orc.advantages(st, tto, r, V, gamma, lam, gamma_turn=1.0, seg_mode=orc.SEG_TRAJ)
    a = 0
    for L in (sum(lens[0]), sum(lens[1])):
        want = gae_double_sum(r[a:a + L], V[a:a + L], gamma, lam)
        assert np.allclose(adv[a:a + L], want, rtol=0, atol=1e-12)
        a += L
    assert np.allclose(ret - adv, V, atol=1e-12)
    # and it differs from treating every turn as an episode: the boundary terms matter
    adv_turn, _ = orc.advantages(st, tto, r, V, gamma, lam, seg_mode=orc.SEG_TURN)
    assert np.abs(adv_turn - adv).max() > 1e-3


@pytest.mark.parametrize("gamma,lam,gamma_turn", [(1.0, 0.95, 0.5), (0.99, 0.9, 0.8), (0.9, 0.0, 0.7), (1.0, 1.0, 0.9)])
def test_traj_mode_with_values_and_step_discount_against_closed_form(gamma, lam, gamma_turn):
    # partial sharing: roles 0 and 2 share model 0, role 1 has model 1, so model 0's run of a trajectory skips
    # steps.  Crossing from the turn at step s to the turn at step s' > s discounts the transition by
    # gamma * gamma_turn^(s' - s) in place of gamma: GAE with a per-transition discount, whose closed form is
    # written out above.  Masked tokens are no actions and drop out of the episode.
    rng = np.random.default_rng(19)
    trajs = [[0, 1, 1, 2, 0, 1, 2], [2, 1, 0]]
    lens = [[3, 2, 4, 2, 1, 3, 4], [2, 2, 3]]
    tto, role, tok_off = chain_graph(trajs, lens)
    N = int(tok_off[-1])
    mask = np.ones(N, np.uint8)
    mask[[1, 12, 20]] = 0                      # a token inside a turn, a whole one-token turn (step 5), a last token
    st = orc.route(2, np.array([0, 1, 0], np.int32), tto, role, tok_off, mask)
    r, V = rng.normal(size=N), rng.normal(size=N)
    adv, ret = orc.advantages(st, tto, r, V, gamma, lam, gamma_turn=gamma_turn, seg_mode=orc.SEG_TRAJ)
    step = np.concatenate([np.arange(1, len(t) + 1) for t in trajs])
    seg = st["traj_seg_off"]
    checked = 0
    for s in range(len(seg) - 1):
        pos = [p for p in range(int(seg[s]), int(seg[s + 1])) if st["tok_mask"][p]]
        if not pos:
            continue
        steps = [int(step[st["tok_turn"][p]]) for p in pos]
        disc = [gamma * gamma_turn ** (steps[i + 1] - steps[i]) for i in range(len(pos) - 1)] + [gamma]
        want = gae_double_sum_varying_discount(r[pos], V[pos], disc, lam)
        assert np.allclose(adv[pos], want, rtol=0, atol=1e-12)
        assert np.allclose(ret[pos] - adv[pos], V[pos], atol=1e-12)
        checked += len(pos)
    assert checked == int(mask.sum())
    assert np.all(adv[st["tok_mask"] == 0] == 0) and np.all(ret[st["tok_mask"] == 0] == 0)


def test_traj_mode_reproduces_discounted_objective():
    # the objective discounts role invocations by gamma^(t-1); with token gamma = lam = 1,
    # V = 0 and gamma_turn = gamma the advantage on a token of step k is
    # sum_{t >= k} gamma^(t-k) r_t = gamma^-(k-1) * tail of sum_t gamma^(t-1) r_t
    rng = np.random.default_rng(11)
    T, gam = 7, 0.9
    lens = [int(x) for x in rng.integers(1, 5, size=T)]
    st, tto = single_stream(lens)
    rho = rng.normal(size=T).astype(np.float32)
    r = orc.place_rewards(st, rho, orc.PLACE_LAST)
    adv, _ = orc.advantages(st, tto, r, None, 1.0, 1.0, gamma_turn=gam, seg_mode=orc.SEG_TRAJ)
    terms = [gam ** (t - 1) * float(rho[t - 1]) for t in range(1, T + 1)]
    a = 0
    for k in range(1, T + 1):
        want = sum(terms[k - 1:]) / gam ** (k - 1)
        assert np.allclose(adv[a:a + lens[k - 1]], want, rtol=1e-13, atol=1e-13)
        a += lens[k - 1]


def test_workflow_c_turn_deltas_telescope():
    # r_iter^(t) = F1(a_t) - F1(a_{t-1}): the search agent's stream, gamma = lam = 1, V = 0,
    # trajectory segments: advantage at its first loop turn = F1(a_T) - F1(a_0).
    f1 = [0.125, 0.375, 0.25, 0.75]
    roles = [0] + [1, 2] * 3          # planner, then (search, answer) x 3
    turn_rew = np.array([f1[0]] + [x for t in range(1, 4) for x in (f1[t] - f1[t - 1], f1[t])], np.float32)
    tto, role, tok_off = chain_graph([roles], [[2] * 7])
    st = orc.route(3, np.array([0, 1, 2], np.int32), tto, role, tok_off, np.ones(14, np.uint8))
    rho = orc.compose_rewards(tto, role, 3, turn_reward=turn_rew)
    r = orc.place_rewards(st, rho)
    adv, _ = orc.advantages(st, tto, r, None, 1.0, 1.0, seg_mode=orc.SEG_TRAJ)
    assert adv[st["model_tok_off"][1]] == f1[3] - f1[0]


def test_scan_commutes_with_compaction():
    rng = np.random.default_rng(13)
    lens = [8, 5]
    N = 13
    mask = (rng.random(N) < 0.6).astype(np.uint8)
    r, V = rng.normal(size=N), rng.normal(size=N)
    st, tto = single_stream(lens, mask)
    adv, ret = orc.advantages(st, tto, r, V, 0.97, 0.9)
    a = 0
    for L in lens:
        sel = np.nonzero(mask[a:a + L])[0] + a
        if len(sel):
            st2, tto2 = single_stream([len(sel)])
            adv2, ret2 = orc.advantages(st2, tto2, r[sel], V[sel], 0.97, 0.9)
            assert np.allclose(adv[sel], adv2, atol=1e-14) and np.allclose(ret[sel], ret2, atol=1e-14)
        a += L


# ------------------------------------------------------------------ O6 scoring
def brute_score_row(h, W, y):
    z = [sum(float(a) * float(b) for a, b in zip(h, w)) for w in W]
    m = max(z)
    s = sum(math.exp(x - m) for x in z)
    lse = m + math.log(s)
    p = [math.exp(x - lse) for x in z]
    return z[y] - lse, lse, -sum(q * math.log(q) for q in p if q > 0)


def test_score_against_pure_python_brute_force():
    rng = np.random.default_rng(17)
    n, d, V = 6, 5, 11
    H = rng.normal(size=(n, d)).astype(np.float32)
    W = rng.normal(size=(V, d)).astype(np.float32)
    ids = rng.integers(0, V, size=n).astype(np.int32)
    rowsel = np.array([0, 2, 3, 5], np.int32)
    logp, lse, ent = orc.score(H, W, ids, rowsel, chunk=3)
    for i in range(n):
        if i in rowsel:
            want = brute_score_row(H[i], W, ids[i])
            assert np.allclose([logp[i], lse[i], ent[i]], want, rtol=0, atol=1e-13)
        else:
            assert (logp[i], lse[i], ent[i]) == (0, 0, 0)


def test_score_closed_forms():
    V, d = 37, 8
    H = np.random.default_rng(0).normal(size=(4, d)).astype(np.float32)
    ids = np.array([0, 5, 36, 7], np.int32)
    logp, lse, ent = orc.score(H, np.zeros((V, d), np.float32), ids)
    assert np.allclose(logp, -math.log(V), atol=1e-15) and np.allclose(ent, math.log(V), atol=1e-14)
    # one dominant logit: entropy -> 0, logp of that token -> 0
    W = np.zeros((V, d), np.float32)
    W[5] = 50 * H[1] / np.dot(H[1], H[1])
    logp, lse, ent = orc.score(H[1:2], W, np.array([5], np.int32))
    assert abs(logp[0]) < 1e-18 * 1e3 + 1e-12 and ent[0] < 1e-18 * 1e3 + 1e-9
    # transposed-operand check: swapping the roles of two weight rows swaps their log-probs
    W = np.random.default_rng(1).normal(size=(V, d)).astype(np.float32)
    la, _, _ = orc.score(H, W, np.array([3] * 4, np.int32))
    W2 = W.copy()
    W2[[3, 9]] = W2[[9, 3]]
    lb, _, _ = orc.score(H, W2, np.array([9] * 4, np.int32))
    assert np.allclose(la, lb, atol=1e-14)


def test_score_second_opinion_torch_and_statistics():
    torch = pytest.importorskip("torch")
    w = wl.make_workload(0)
    t = w.model_tensors(0)
    logp, lse, ent = orc.score(t["H"], t["W"], t["ids"])
    z = torch.from_numpy(t["H"]).double() @ torch.from_numpy(t["W"]).double().T
    ls = torch.log_softmax(z, dim=1)
    want_logp = ls[torch.arange(z.shape[0]), torch.from_numpy(t["ids"]).long()]
    want_ent = torch.distributions.Categorical(logits=z).entropy()
    assert np.allclose(logp, want_logp.numpy(), atol=1e-12)
    assert np.allclose(lse, torch.logsumexp(z, 1).numpy(), atol=1e-12)
    assert np.allclose(ent, want_ent.numpy(), atol=1e-12)
    # logits ~ N(0, d*0.02^2): E[lse] ~ ln V + sigma^2/2 for the random-init head
    sigma2 = 64 * 0.02 ** 2
    assert abs(lse.mean() - (math.log(512) + sigma2 / 2)) < 0.01


# ------------------------------------------------------------------ O7 loss
def test_ppo_worked_example():
    _, kv = read_golden("ppo_clip_worked_example.txt")
    A, ratio = np.array(kv["A"]), np.array(kv["ratio"])
    logp_old = np.array([-1.0, -2.0, -0.5, -3.0])
    logp = logp_old + np.log(ratio)
    role = np.array([0, 1, 0, 1], np.int32)
    stats, g = orc.ppo_loss(logp, logp_old, A, np.array([1.0, 2.0, 3.0, 4.0]), None, role, 2, kv["eps"][0])
    assert np.allclose(stats[0], [kv["loss"][0], kv["clip_frac"][0], 2.5, -np.log(ratio).mean(), 4], atol=1e-15)
    assert np.allclose(g, kv["g"], atol=1e-15)
    # per role: role 0 holds rows 0 and 2, role 1 rows 1 and 3
    L = kv["L"]
    assert np.allclose(stats[1], [(L[0] + L[2]) / 2, 0.5, 2.0, -(math.log(1.5) + math.log(0.5)) / 2, 2], atol=1e-15)
    assert np.allclose(stats[2], [(L[1] + L[3]) / 2, 0.5, 3.0, -(math.log(1.5) + math.log(0.5)) / 2, 2], atol=1e-15)


def test_ppo_ratio_one_identity_and_rowsel():
    rng = np.random.default_rng(19)
    n = 50
    logp = -rng.random(n) * 5
    A = rng.normal(size=n)
    rowsel = np.sort(rng.choice(n, size=31, replace=False)).astype(np.int32)
    mask = np.zeros(n)
    mask[rowsel] = 1
    stats, g = orc.ppo_loss(logp, logp, A, np.zeros(n), rowsel, np.zeros(n, np.int32), 1, 0.2)
    assert abs(stats[0, 0] + (A * mask).sum() / mask.sum()) < 1e-15     # loss = -mean(A * mask)
    assert stats[0, 1] == 0 and stats[0, 3] == 0 and stats[0, 4] == 31
    assert np.allclose(g, -A * mask / 31, atol=1e-16)
    stats0, g0 = orc.ppo_loss(logp, logp, np.zeros(n), np.zeros(n), rowsel, np.zeros(n, np.int32), 1, 0.2)
    assert not stats0[0, :4].any() and not g0.any()
    stats_e, g_e = orc.ppo_loss(logp, logp, A, np.zeros(n), np.zeros(0, np.int32), np.zeros(n, np.int32), 1, 0.2)
    assert not stats_e.any() and not g_e.any()


# ------------------------------------------------------------------ O8 backward
def scalar_loss(H, W, ids, logp_old, A, rowsel, eps):
    logp, lse, ent = orc.score(H, W, ids, rowsel)
    stats, _ = orc.ppo_loss(logp, logp_old, A, ent, rowsel, np.zeros(len(ids), np.int32), 1, eps)
    return stats[0, 0]


def test_backward_matches_finite_differences_and_identities():
    rng = np.random.default_rng(23)
    n, d, V = 9, 6, 13
    H = rng.normal(size=(n, d))
    W = rng.normal(size=(V, d)) * 0.5
    ids = rng.integers(0, V, size=n).astype(np.int32)
    rowsel = np.array([0, 1, 2, 4, 5, 7, 8], np.int32)
    logp, lse, ent = orc.score(H, W, ids, rowsel)
    logp_old = logp + rng.normal(size=n) * 0.3        # some rows end up clipped
    A = rng.normal(size=n)
    stats, g = orc.ppo_loss(logp, logp_old, A, ent, rowsel, np.zeros(n, np.int32), 1, 0.2)
    assert 0 < stats[0, 1] < 1
    dH, dW = orc.lm_head_backward(H, W, ids, lse, g, rowsel)
    h = 1e-6
    for (arr, grad) in ((H, dH), (W, dW)):
        for idx in [(0, 0), (1, 3), (2, 5), (4, 1), (8, 2), (3, 3), (6, 0)]:
            if idx[0] >= arr.shape[0]:
                continue
            keep = arr[idx]
            arr[idx] = keep + h
            fp = scalar_loss(H, W, ids, logp_old, A, rowsel, 0.2)
            arr[idx] = keep - h
            fm = scalar_loss(H, W, ids, logp_old, A, rowsel, 0.2)
            arr[idx] = keep
            assert abs((fp - fm) / (2 * h) - grad[idx]) < 1e-8
    # unscored and clipped rows: no gradient
    assert not dH[[3, 6]].any()
    clipped = [i for i in rowsel if g[i] == 0]
    assert len(clipped) > 0 and not dH[clipped].any()
    # sum_v dz_iv = 0  =>  the vocabulary-axis sum of dW vanishes
    assert np.abs(dW.sum(axis=0)).max() < 1e-14
    # ratio = 1: dH_i = -(A_i/S) (W[y_i] - sum_v p_iv W_v)
    stats1, g1 = orc.ppo_loss(logp, logp, A, ent, rowsel, np.zeros(n, np.int32), 1, 0.2)
    dH1, dW1 = orc.lm_head_backward(H, W, ids, lse, g1, rowsel)
    for i in rowsel:
        p = np.exp(H[i] @ W.T - lse[i])
        assert np.allclose(dH1[i], -(A[i] / len(rowsel)) * (W[ids[i]] - p @ W), atol=1e-14)
    # dW by its definition, element by element, for one vocabulary row
    v = int(ids[0])
    want = np.zeros(d)
    for i in rowsel:
        p_v = math.exp(float(H[i] @ W[v]) - lse[i])
        want += g1[i] * ((1.0 if ids[i] == v else 0.0) - p_v) * H[i]
    assert np.allclose(dW1[v], want, atol=1e-14)


# ------------------------------------------------------------------ workloads sanity
def test_workload_shapes_follow_the_configurations():
    w0 = wl.make_workload(0)
    assert (w0.n_traj, w0.n_turns, w0.n_tokens) == (4, 24, 768)
    w1 = wl.make_workload(1)
    assert (w1.n_turns, w1.n_tokens) == (192, 49152) and 0.75 < w1.tok_mask.mean() < 0.85
    w2 = wl.make_workload(2)
    assert 64 <= w2.n_turns <= 192 and 0.6 < w2.tok_mask.mean() < 0.8
    w3 = wl.make_workload(3)
    assert w3.model_ntok == [73728, 49152]
    w4 = wl.make_workload(4)
    assert (w4.n_turns, w4.n_tokens) == (64, 163840)
    t = wl.make_workload(1, n_traj=2, models=[(64, 300, "bf16")]).model_tensors(0)
    assert np.array_equal(wl.round_to_bf16(t["H"]), t["H"]) and t["ids"].max() < 300
    assert np.allclose((t["H"].astype(np.float64) ** 2).mean(axis=1), 1.0, atol=2e-2)


def test_array_wise_restatement_agrees_with_the_sequential_oracle_on_random_graphs():
    """tests/arraywise.py states steps a1-a4 with sorts, prefix sums and gathers; the oracle walks turns and tokens
    one by one.  Two implementations written separately from the same definitions: on seeded random workflow graphs
    (empty turns and trajectories, models that receive nothing, every mask density, all reward levels) every stream,
    the flags, the composed and the placed rewards must be identical, and the oracle's advantages must satisfy the
    recurrence token by token."""
    from tests import arraywise as aw
    from tests import parity as P
    done = 0
    for seed in range(400):
        w, kw = wl.random_graph(seed)
        if w.n_tokens > 20000:
            continue
        done += 1
        rho, st, r, adv_o, ret_o = P.oracle_front(w, **kw)
        sa = aw.streams(w)
        n_runs = int(st["model_trajrun_off"][-1])
        assert sa["n_runs"] == n_runs
        for f in ("model_tok_off", "perm", "tok_turn", "tok_role", "tok_mask", "turn_seg_off", "seg_turn", "model_turn_off",
                  "model_trajrun_off", "rowsel", "model_rowsel_off", "traj_seg_off"):
            assert np.array_equal(sa[f], st[f]), f"seed {seed}: {f}"
        if w.n_turns:
            assert np.array_equal(sa["tok_flags"], P.expected_flags(w, st, sa["turn_step"])), f"seed {seed}: flags"
        rho_a = aw.composed_rewards(w)
        if w.traj_group is None:
            assert np.array_equal(rho_a.view(np.uint32), rho.view(np.uint32)), f"seed {seed}: rho"
        else:
            assert np.allclose(rho_a, rho, rtol=1e-6, atol=1e-7), f"seed {seed}: rho"
        r_a = aw.placed_rewards(sa, rho, kw["place_mode"])
        assert np.array_equal(r_a.view(np.uint32), r.view(np.uint32)), f"seed {seed}: placed rewards"
        value = w.value
        worst = aw.recurrence_check(sa, r, value, adv_o, ret_o, kw["gamma"], kw["lam"], kw["gamma_turn"], kw["seg_mode"], tol=1e-12)
        assert worst <= 1.0, f"seed {seed}: recurrence residual {worst:.3g} x its allowance"
        # a wrong carry must not pass: the same check with another discount fails wherever something is carried
        if n_runs and kw["lam"] > 0 and np.abs(adv_o).max() > 0:
            cur = np.flatnonzero(st["tok_mask"])
            seg = sa["tok_slot"] if kw["seg_mode"] == wl.SEG_TURN else sa["run_of_slot"][sa["tok_slot"]]
            carried = (seg[cur[1:]] == seg[cur[:-1]]) & (adv_o[cur[1:]] != 0)
            if carried.any():
                assert aw.recurrence_check(sa, r, value, adv_o, ret_o, kw["gamma"], 0.5 * kw["lam"], kw["gamma_turn"], kw["seg_mode"], tol=1e-12) > 1.0
        # the ready batch, both cuts
        rng = np.random.default_rng(seed)
        order = rng.permutation(w.n_traj).astype(np.int32) if rng.random() < 0.8 else None
        keep = (rng.random(w.n_traj) < 0.8).astype(np.uint8) if rng.random() < 0.8 else None
        M = int(rng.integers(1, 6))
        for balanced in (False, True):
            rows_o, off_o = orc.ready_batch(st, w.traj_turn_off, np.ones(w.n_traj, np.uint8) if keep is None else keep,
                                            np.arange(w.n_traj) if order is None else order, M, balance_rows=balanced)
            rows_a, off_a = aw.ready_batch(w, sa, keep, order, M, balanced)
            assert np.array_equal(rows_a, rows_o) and np.array_equal(off_a, off_o), f"seed {seed}: ready batch, balanced={balanced}"
        budget = int(rng.choice([1, 2, 9, 70, 2000, 10 ** 7]))
        rows_o, off_o, n_o = orc.ready_batch_packed(st, w.traj_turn_off, np.ones(w.n_traj, np.uint8) if keep is None else keep,
                                                    np.arange(w.n_traj) if order is None else order, budget)
        rows_a, off_a, n_a = aw.ready_batch_packed(w, sa, keep, order, budget)
        assert np.array_equal(rows_a, rows_o) and np.array_equal(off_a, off_o) and np.array_equal(n_a, n_o), f"seed {seed}: packed, budget {budget}"
    assert done >= 150


def end_to_end_closed_form(w, H, ids, V):
    """What the whole path must give for a policy with W = 0 (uniform over the vocabulary), ratio 1, gamma = lam = 1,
    no critic, turn segments and the reward on a turn's last valid token - written from the inputs alone:
    every valid token of a turn carries the turn's composed reward as its advantage (the suffix sum of a single
    reward), log-prob = -ln V, loss = -mean A, g = -A / S, dH = 0 (every row of W is the same), and
    dW[v] = sum_i g_i (1[v = y_i] - 1/V) h_i.  One model holding all roles: stream order = global order."""
    f64 = np.float64
    traj = np.repeat(np.arange(w.n_traj), np.diff(w.traj_turn_off))
    rho = np.zeros(w.n_turns)
    if w.role_reward is not None:
        rho += w.role_reward.astype(f64)[traj * w.n_roles + w.turn_role]
    if w.turn_reward is not None:
        rho += w.turn_reward.astype(f64)
    if w.traj_reward is not None:
        rho += w.traj_reward.astype(f64)[traj]
    tok_turn = np.repeat(np.arange(w.n_turns), np.diff(w.turn_tok_off))
    valid = w.tok_mask != 0
    A = np.where(valid, rho[tok_turn], 0.0)
    S = int(valid.sum())
    g = np.where(valid, -A / S, 0.0)
    gh = g[:, None] * H.astype(f64)
    dW = np.zeros((V, H.shape[1]))
    np.add.at(dW, ids[valid], gh[valid])
    dW -= gh.sum(axis=0)[None, :] / V
    return A, -A[valid].mean(), g, dW


def test_end_to_end_closed_form_for_a_uniform_policy():
    """The composition of all steps (rewards -> routing -> placement -> scan -> scoring -> surrogate -> backward) against
    a closed form that uses none of the oracle's functions: a plausible mistake in how the steps are joined (advantages
    in the wrong order, the mean over the wrong count, a gradient with the wrong sign) changes the loss or dW."""
    from tests import parity as P
    w = wl.make_workload(0)
    rng = np.random.default_rng(5)
    w.tok_mask = (rng.random(w.n_tokens) < 0.7).astype(np.uint8)
    w.tok_mask[:40] = 0                                           # a turn without any valid token
    w.turn_reward = rng.normal(size=w.n_turns).astype(np.float32)
    w.value = None
    t = w.model_tensors(0)
    V, d = w.models[0].V, w.models[0].d
    W0 = np.zeros((V, d), np.float32)
    rho, st, r, adv, ret = P.oracle_front(w, gamma=1.0, lam=1.0, seg_mode=wl.SEG_TURN, place_mode=wl.PLACE_LAST)
    assert np.array_equal(st["perm"], np.arange(w.n_tokens))
    A, loss, g, dW = end_to_end_closed_form(w, t["H"], t["ids"], V)
    assert np.allclose(adv, A, rtol=1e-6, atol=1e-7) and np.allclose(ret, A, rtol=1e-6, atol=1e-7)
    rows = st["rowsel"]
    logp, lse, ent = orc.score(t["H"], W0, t["ids"], rows)
    assert np.allclose(logp[rows], -math.log(V), atol=1e-12) and np.allclose(ent[rows], math.log(V), atol=1e-12)
    stats, g_o = orc.ppo_loss(logp, logp, adv, ent, rows, st["tok_role"], w.n_roles, 0.2)
    assert abs(stats[0, 0] - loss) <= 1e-6 * abs(loss) and stats[0, 1] == 0 and stats[0, 4] == len(rows)   # composed rewards are float32
    assert np.allclose(g_o, g, rtol=1e-6, atol=1e-12)
    dH_o, dW_o = orc.lm_head_backward(t["H"], W0, t["ids"], lse, g_o, rows)
    assert not np.abs(dH_o).max() > 1e-15
    assert np.allclose(dW_o, dW, rtol=1e-6, atol=1e-9)
