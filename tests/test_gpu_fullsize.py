"""GPU parity at the configurations' full sizes, in the launch configuration the benchmark times.

The CPU oracle cannot score 10^5 rows against a 152k-entry vocabulary inside a test, so its
log-probs, logsumexps and entropies come from files under tests/golden/ that
tests/golden/make_fullsize_golden.py wrote by calling the oracle alone (every scored row of every model of
configurations 1 to 4; the code also takes files that hold a seeded row sample).  Everything else the oracle
computes here, live: routing, rewards and advantages on the whole batch, the surrogate statistics and
per-row gradients, and dH / dW on sampled rows and vocabulary entries, which depend on one row or one
vocabulary entry at a time once the stored logsumexp is given.
"""
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import umas_oracle as orc
import paper_2605_26646_amd as umas
from tests import parity as P

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL_LOGP, TOL = 2e-2, 1e-2          # bf16: absolute on log-probs, relative on loss and gradients
N_DH_ROWS, N_DW_ROWS = 128, 320        # sampled rows of dH; sampled vocabulary entries of dW (at least 256 after merging)


def fingerprint(t):
    return np.array([float(t["H"][:64].astype(np.float64).sum()), float(t["W"][:64].astype(np.float64).sum()),
                     float(t["ids"].astype(np.int64).sum()), float(t["noise"].astype(np.float64).sum())])


def spread(idx, n, seed):
    """n entries of idx: both ends (first and last tiles) and a seeded draw in between."""
    if len(idx) <= n:
        return np.asarray(idx)
    e = n // 4
    mid = idx[e:len(idx) - e]
    pick = np.random.default_rng([seed, 31]).choice(len(mid), size=n - 2 * e, replace=False)
    return np.sort(np.concatenate([idx[:e], mid[pick], idx[len(idx) - e:]]))


def run_fullsize(cfg, fixed_rounds=None):
    path = os.path.join(GOLDEN, f"fullsize_cfg{cfg}.npz" if fixed_rounds is None else f"fullsize_cfg{cfg}r{fixed_rounds}.npz")
    if not os.path.exists(path):
        pytest.skip(f"{os.path.basename(path)} has not been generated")
    gold = np.load(path)
    w = wl.make_workload(cfg) if fixed_rounds is None else wl.make_workload(cfg, fixed_rounds=fixed_rounds)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    P.check_front(w, s, adv, ret, rho, st, r, adv_o, ret_o)
    for m in range(w.n_models):
        spec = w.models[m]
        assert spec.dtype == "bf16"
        t = w.model_tensors(m)
        assert np.array_equal(fingerprint(t), gold[f"fingerprint_{m}"]), "stored values belong to other inputs"
        a, e = int(st["model_tok_off"][m]), int(st["model_tok_off"][m + 1])
        ra, re = int(st["model_rowsel_off"][m]), int(st["model_rowsel_off"][m + 1])
        rowsel_o = st["rowsel"][ra:re]
        n_sel = re - ra
        full = f"rows_{m}" not in gold.files
        known = rowsel_o if full else gold[f"rows_{m}"]
        assert np.isin(known, rowsel_o).all()
        logp_o, lse_o, ent_o = (gold[f"{k}_{m}"].astype(np.float64) for k in ("logp", "lse", "entropy"))

        H = P.to_dev(t["H"], torch.bfloat16)
        W = P.to_dev(t["W"], torch.bfloat16)
        ids = P.to_dev(t["ids"])
        rowsel = s.rowsel[ra:re]
        # scoring
        logp, lse, ent = umas.umas_policy_logprobs(H, W, ids, rowsel)
        for name, x, o in (("logp", logp, logp_o), ("lse", lse, lse_o), ("entropy", ent, ent_o)):
            err = np.abs(x.cpu().numpy().astype(np.float64)[known] - o[known]).max()
            assert err <= TOL_LOGP, f"cfg {cfg} model {m} {name}: max abs error {err:.3g}"
        unscored = np.setdiff1d(np.arange(e - a), rowsel_o)
        assert not logp.cpu().numpy()[unscored].any(), "unscored rows must read 0"
        # old log-probs are an input of both sides: oracle log-prob + generator noise where the oracle's
        # value is stored, a typical value (about -log V) + noise elsewhere
        logp_old = (-12.0 + t["noise"].astype(np.float64))
        logp_old[known] = logp_o[known] + t["noise"][known]
        logp_old32 = logp_old.astype(np.float32)
        role_o = st["tok_role"][a:e]
        stats_o, g_known = orc.ppo_loss(logp_o, logp_old32, adv_o[a:e], ent_o, known, role_o, w.n_roles, w.clip_eps)
        g_o = g_known * (len(known) / n_sel)           # the oracle divided by the rows it was given
        # loss + backward exactly as the benchmark launches it
        ws = torch.empty(umas.ppo_workspace_bytes(n_sel, spec.d, spec.V, torch.bfloat16, w.n_roles),
                         dtype=torch.uint8, device="cuda")
        dW = torch.empty((spec.V, spec.d), dtype=torch.float32, device="cuda")
        dH = torch.empty_like(H)
        logp_new = torch.empty(e - a, dtype=torch.float32, device="cuda")
        stats = torch.empty((1 + w.n_roles) * 32, dtype=torch.uint8, device="cuda")
        umas.umas_ppo_loss_fwd_bwd(H, W, ids, rowsel, P.to_dev(logp_old32), adv[a:e].contiguous(),
                                   s.tok_role[a:e].contiguous(), w.n_roles, w.clip_eps, dW=dW, dH=dH,
                                   logp_new=logp_new, stats=stats, workspace=ws)
        torch.cuda.synchronize()
        sg = umas.read_stats(stats)
        assert np.abs(logp_new.cpu().numpy()[known] - logp_o[known]).max() <= TOL_LOGP
        for k in range(1 + w.n_roles):
            cnt = n_sel if k == 0 else int((role_o[rowsel_o] == k - 1).sum())
            assert int(sg["n_scored"][k]) == cnt and int(sg["n_invalid_ids"][k]) == 0
            if not full:
                continue
            for j, name in enumerate(("loss", "clip_frac", "entropy_mean", "approx_kl")):
                o = stats_o[k, j]
                lim = TOL * max(abs(o), abs(stats_o[0, j]), 1e-3)
                if name == "clip_frac":
                    lim = max(lim, 2.0 / max(cnt, 1))
                if name == "approx_kl":
                    lim = TOL_LOGP
                assert abs(float(sg[name][k]) - o) <= lim, f"cfg {cfg} model {m} {name}[{k}]: {float(sg[name][k])} vs {o}"
        # dH on sampled rows: row i of dH depends on row i alone
        rows_h = spread(known, N_DH_ROWS, 10 * cfg + m)
        dH_o, _ = orc.lm_head_backward(t["H"], t["W"], t["ids"], lse_o, g_o, rows_h)
        rel_h = P.close(dH[torch.from_numpy(rows_h).cuda()].float().cpu().numpy(), dH_o[rows_h], TOL, "dH sample")
        dH_host = dH.float().cpu().numpy()
        assert not dH_host[unscored].any(), "unscored rows must get a zero gradient"
        rel_w = None
        dW_host = dW.cpu().numpy()
        if full:
            # dW on sampled vocabulary entries: with lse given, column v of dz needs only W[v].  The oracle
            # runs on the restricted head; labels outside the sample point at an extra all-zero entry
            # whose gradient is discarded.
            labels = np.unique(t["ids"][rowsel_o])
            vs = np.unique(np.concatenate([spread(labels, N_DW_ROWS // 2, cfg), [0, 255, 256, spec.V - 1],
                                           spread(np.arange(spec.V), N_DW_ROWS // 2, cfg + 50)]))
            pos = np.full(spec.V, len(vs), dtype=np.int64)
            pos[vs] = np.arange(len(vs))
            W_sub = np.concatenate([t["W"][vs], np.zeros((1, spec.d), t["W"].dtype)])
            _, dW_sub = orc.lm_head_backward(t["H"], W_sub, pos[t["ids"]], lse_o, g_o, rowsel_o, chunk=4096)
            assert len(vs) >= 256
            rel_w = P.close(dW_host[vs], dW_sub[:len(vs)], TOL, "dW sample")
        # every row of dz sums to zero over the vocabulary, so dW summed over the vocabulary vanishes
        col = dW_host.sum(axis=0, dtype=np.float64)
        mag = np.abs(dW_host).sum(axis=0, dtype=np.float64)
        assert (np.abs(col) <= TOL * mag + 1e-12).all(), "dW does not sum to zero over the vocabulary"
        print(f"  cfg {cfg} model {m}: scored={n_sel} oracle rows={len(known)} loss={float(sg['loss'][0]):+.6f} "
              f"(oracle {stats_o[0, 0]:+.6f}) dH rel {rel_h:.2e} dW rel {rel_w}", flush=True)
        del H, W, dW, dH, ws
        torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size(cfg):
    run_fullsize(cfg)


def test_full_size_cfg4_with_three_fixed_rounds():
    """The other reading of configuration 4 (every trajectory runs all three rounds: 245 760 tokens, two chunks of the
    backward at the recommended workspace): routing, rewards and advantages on the whole batch, log-probs, logsumexps
    and entropies on a stored sample of 4096 rows, dH on 128 of them, dW summing to zero over the vocabulary."""
    run_fullsize(4, fixed_rounds=3)


def test_full_size_single_pass_backward_agrees_with_recomputing_backward():
    """Without an entropy bonus the update keeps the softmax numerators of its scoring pass and never computes a
    logit twice; with one it recomputes them tile by tile.  An entropy coefficient too small to change any
    float32 result selects the second path: both must give the same loss and the same gradients, everywhere,
    at the benchmark's size (the oracle covers sampled entries only there)."""
    w = wl.make_workload(1)
    s, adv, ret = P.gpu_front(w)
    spec = w.models[0]
    t = w.model_tensors(0)
    n_sel = int(s.model_rowsel_off[-1].item())           # rowsel is allocated for every token; only the scored ones are written
    assert n_sel == int(w.tok_mask.sum())
    rowsel = s.rowsel[:n_sel]
    H, W, ids = P.to_dev(t["H"], torch.bfloat16), P.to_dev(t["W"], torch.bfloat16), P.to_dev(t["ids"])
    logp, _, _ = umas.umas_policy_logprobs(H, W, ids, rowsel)
    logp_old = logp + P.to_dev(t["noise"].astype(np.float32))
    ws = torch.empty(umas.ppo_workspace_bytes(n_sel, spec.d, spec.V, torch.bfloat16, w.n_roles), dtype=torch.uint8, device="cuda")
    out = []
    for coef in (0.0, 1e-30):
        stats, logp_new, dH, dW = umas.umas_ppo_loss_fwd_bwd(H, W, ids, rowsel, logp_old, adv, s.tok_role, w.n_roles,
                                                            w.clip_eps, entropy_coef=coef, workspace=ws)
        torch.cuda.synchronize()
        out.append((umas.read_stats(stats), logp_new.cpu().numpy(), dH.float().cpu().numpy(), dW.cpu().numpy()))
        del dH, dW
    # the same update in three chunks of selected rows (a workspace a third of the size): dW is accumulated
    # over the chunks, everything else is per row
    part = umas.ppo_workspace_bytes((n_sel + 2) // 3, spec.d, spec.V, torch.bfloat16, w.n_roles)
    assert umas.ppo_workspace_bytes(n_sel, spec.d, spec.V, torch.bfloat16, w.n_roles, minimum=True) < part < ws.numel() // 2
    stats, logp_new, dH, dW = umas.umas_ppo_loss_fwd_bwd(H, W, ids, rowsel, logp_old, adv, s.tok_role, w.n_roles,
                                                        w.clip_eps, workspace=ws[:part])
    torch.cuda.synchronize()
    sc_, lc, dHc, dWc = umas.read_stats(stats), logp_new.cpu().numpy(), dH.float().cpu().numpy(), dW.cpu().numpy()
    del dH, dW
    assert np.array_equal(lc, out[0][1]) and np.array_equal(dHc, out[0][2])
    assert float(sc_["loss"][0]) == float(out[0][0]["loss"][0])
    # the same products summed in float32 in another grouping (three partial sums) and one-hot rows added by atomics in
    # another order: a few 2^-24 of the sum of the terms' magnitudes, which is up to a hundred times an entry that
    # cancels; a tenth of the gradient bar
    P.close(dWc, out[0][3], 1e-3, "dW, three chunks against one")
    (sa, la, dHa, dWa), (sb, lb, dHb, dWb) = out
    assert np.abs(la - lb).max() <= 1e-4
    assert abs(float(sa["loss"][0]) - float(sb["loss"][0])) <= 1e-5 * max(abs(float(sb["loss"][0])), 1e-3)
    P.close(dHa, dHb, TOL, "dH, kept numerators against recomputed logits")
    P.close(dWa, dWb, TOL, "dW, kept numerators against recomputed logits")


@pytest.mark.parametrize("cfg", [1, 4])
def test_full_size_critic(cfg):
    """The critic's fused pass at the configurations' real row counts and hidden sizes; the oracle's per-row
    dot products are cheap enough to run live."""
    from tests.test_gpu_next import critic_case
    w = wl.make_workload(cfg)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    for m in range(w.n_models):
        critic_case(w, m, st, ret_o, s, ret)
