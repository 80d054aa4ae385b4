"""GPU parity of the steps around the policy update (critic, KL-penalised rewards, whitening,
surrogate variants) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import umas_oracle as orc
import paper_2605_26646_amd as umas
from tests import parity as P

pytestmark = pytest.mark.gpu


def critic_case(w, m, st, ret_o, s, ret_gpu, accumulate=False):
    """Value head, clipped value loss and backward of model m on the returns of each side."""
    spec = w.models[m]
    tdt = torch.float32 if spec.dtype == "f32" else torch.bfloat16
    tol_v, tol = (1e-5, 1e-5) if spec.dtype == "f32" else (2e-2, 1e-2)
    t = w.model_tensors(m)
    c = w.critic_tensors(m)
    a, e = int(st["model_tok_off"][m]), int(st["model_tok_off"][m + 1])
    ra, re = int(st["model_rowsel_off"][m]), int(st["model_rowsel_off"][m + 1])
    rows_o = st["rowsel"][ra:re]
    role_o = st["tok_role"][a:e]
    H, wv = P.to_dev(t["H"], tdt), P.to_dev(c["w"], tdt)
    rowsel = s.rowsel[ra:re]
    bias = float(c["bias"])
    # forward
    V = umas.umas_values(H, wv, bias, rowsel)
    V_o = orc.value_head(t["H"], c["w"], bias, rows_o)
    lim = tol_v * (max(1.0, np.abs(V_o).max()) if spec.dtype == "f32" else 1.0)
    assert np.abs(V.cpu().numpy() - V_o).max(initial=0) <= lim
    # old values are an input of both sides: oracle values + generator noise; clip range 0.1 so both branches occur
    V_old = (V_o + c["v_noise"]).astype(np.float32)
    stats_o, g_o = orc.value_loss(V_o, V_old, ret_o[a:e], rows_o, role_o, w.n_roles, 0.1)
    dH_o, dw_o, db_o = orc.value_head_backward(t["H"], c["w"], g_o, rows_o)
    dH0 = dw0 = db0 = None
    if accumulate:
        g = torch.Generator(device="cpu").manual_seed(5)
        dH0 = torch.randn(t["H"].shape, generator=g).mul_(1e-4).to(tdt).cuda()
        dw0 = torch.randn(spec.d, generator=g).mul_(1e-3).cuda()
        db0 = torch.full((1,), 0.25, device="cuda")
    stats, V_new, dH, dw, db = umas.umas_value_loss_fwd_bwd(
        H, wv, bias, rowsel, P.to_dev(V_old), ret_gpu[a:e].contiguous(), s.tok_role[a:e].contiguous(), w.n_roles, 0.1,
        accumulate_dH=accumulate, accumulate_dw=accumulate, dH=None if dH0 is None else dH0.clone(),
        dw=None if dw0 is None else dw0.clone(), db=None if db0 is None else db0.clone())
    torch.cuda.synchronize()
    sg = umas.read_value_stats(stats)
    assert np.abs(V_new.cpu().numpy() - V_o).max(initial=0) <= lim
    assert 0 < stats_o[0, 1] < 1, "the case must exercise both branches"
    for k in range(1 + w.n_roles):
        assert int(sg["n_scored"][k]) == int(stats_o[k, 3])
        for j, name in enumerate(("loss", "clip_frac", "value_mean")):
            o = stats_o[k, j]
            lim_s = tol * max(abs(o), abs(stats_o[0, j]), 1e-3)
            if name == "clip_frac":       # a row on the clip boundary may fall either way
                lim_s = max(lim_s, 2.0 / max(stats_o[k, 3], 1))
            if name == "value_mean":
                lim_s = lim
            assert abs(float(sg[name][k]) - o) <= lim_s, f"{name}[{k}]: {float(sg[name][k])} vs {o}"
    # g_i = (V_i - R_i) / S inherits the absolute error of V_i, whatever is left of V_i - R_i after cancellation
    row_abs = lim / max(len(rows_o), 1) * float(np.linalg.norm(c["w"].astype(np.float64)))
    if accumulate:
        dH_o = dH_o + dH0.float().cpu().numpy().astype(np.float64)
        dw_o = dw_o + dw0.cpu().numpy().astype(np.float64)
        db_o = db_o + 0.25
        # accumulated rows are rounded to the storage type once more
        P.close(dH.float().cpu().numpy(), dH_o, tol, "dH (accumulated)", row_abs=row_abs)
    else:
        P.close(dH.float().cpu().numpy(), dH_o, tol, "dH", row_abs=row_abs)
        unsel = np.setdiff1d(np.arange(e - a), rows_o)
        assert not dH.float().cpu().numpy()[unsel].any()
    P.close(dw.cpu().numpy(), dw_o, tol, "dw")
    assert abs(float(db.item()) - db_o) <= tol * max(abs(db_o), np.abs(g_o).sum() * 1e-2 + 1e-12)


def run_critic(cfg, **kw):
    w = wl.make_workload(cfg, **kw)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    for m in range(w.n_models):
        critic_case(w, m, st, ret_o, s, ret)
    return w, st, ret_o, s, ret


def test_critic_cfg0_fp32():
    w, st, ret_o, s, ret = run_critic(0)
    critic_case(w, 0, st, ret_o, s, ret, accumulate=True)


def test_critic_scaled_bf16_configs():
    run_critic(2, n_traj=8, tokens_per_turn=48, models=[(200, 1000, "bf16")])        # interior masks, d % 64 != 0
    w, st, ret_o, s, ret = run_critic(3, n_traj=6, tokens_per_turn=40, models=[(128, 700, "bf16"), (200, 1000, "bf16")])
    critic_case(w, 1, st, ret_o, s, ret, accumulate=True)


def test_critic_full_width_rows():
    # real hidden sizes (2048 and 3584: 4 and 7 column vectors per thread, 16 and 9 rows per chunk), few rows
    run_critic(3, n_traj=3, tokens_per_turn=37, models=[(2048, 512, "bf16"), (3584, 512, "bf16")])


def test_critic_widest_rows():
    # the widest rows the value head takes: 8192 (bf16, 16 column vectors per lane) and 4096 (float32)
    run_critic(3, n_traj=2, tokens_per_turn=23, models=[(8192, 256, "bf16"), (4096, 256, "f32")])
    H = torch.zeros((4, 8200), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(umas.UmasError):
        umas.umas_values(H, torch.zeros(8200, dtype=torch.bfloat16, device="cuda"))


def test_critic_empty_selection_and_errors():
    H = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    wv = torch.ones(64, dtype=torch.bfloat16, device="cuda")
    z = torch.zeros(8, device="cuda")
    sel = torch.zeros(0, dtype=torch.int32, device="cuda")
    stats, V_new, dH, dw, db = umas.umas_value_loss_fwd_bwd(H, wv, 0.0, sel, z, z, None, 0, 0.2)
    torch.cuda.synchronize()
    sg = umas.read_value_stats(stats)
    assert int(sg["n_scored"][0]) == 0 and float(sg["loss"][0]) == 0.0
    assert not dw.cpu().numpy().any() and not dH.float().cpu().numpy().any() and float(db.item()) == 0.0
    with pytest.raises(umas.UmasError):
        umas.umas_values(torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda"), torch.zeros(12, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(umas.UmasError):
        umas.umas_value_loss_fwd_bwd(H, wv, 0.0, None, z, z, None, 0, -1.0)


def shaping_case(cfg, **kw):
    """KL-penalised rewards feed the scan with dense rewards; whitening on the resulting advantages."""
    w = wl.make_workload(cfg, **kw)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    n = w.n_tokens
    rng = np.random.default_rng(1234 + cfg)
    logp = (-3.0 * rng.random(n)).astype(np.float32)
    logp_ref = (logp + rng.normal(size=n).astype(np.float32) * 0.1).astype(np.float32)
    beta = 0.05
    r_o, kl_o = orc.kl_penalised_rewards(r, logp, logp_ref, st["tok_mask"], beta)
    r_g, kl_g = umas.umas_kl_rewards(s.tok_reward, P.to_dev(logp), P.to_dev(logp_ref), s.tok_mask, beta)
    P.close(r_g.cpu().numpy(), r_o, 1e-5, "penalised rewards")
    assert abs(float(kl_g.item()) - kl_o) <= 1e-5 * max(abs(kl_o), np.abs(logp - logp_ref).mean())
    masked = st["tok_mask"] == 0
    assert np.array_equal(r_g.cpu().numpy()[masked].view(np.uint32), r[masked].view(np.uint32)), "masked tokens keep their reward"
    # dense rewards through the scan on both sides
    value = None if w.value is None else w.value
    adv2_o, ret2_o = orc.advantages(st, w.traj_turn_off, r_o.astype(np.float32), value, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
    s.tok_reward = r_g
    adv2, ret2 = umas.umas_advantages(s, None if value is None else P.to_dev(value), w.gamma, w.lam, w.gamma_turn, w.seg_mode)
    P.close(adv2.cpu().numpy(), adv2_o, 1e-5, "advantages on dense rewards")
    P.close(ret2.cpu().numpy(), ret2_o, 1e-5, "returns on dense rewards")
    # in place
    r_in = s.tok_reward.clone()
    umas.umas_kl_rewards(r_in, P.to_dev(logp), P.to_dev(logp_ref), s.tok_mask, beta, out=r_in)
    r_twice, _ = orc.kl_penalised_rewards(r_o, logp, logp_ref, st["tok_mask"], beta)
    P.close(r_in.cpu().numpy(), r_twice, 1e-5, "in-place penalty")
    for scope, oscope in ((umas.WHITEN_MODEL, orc.WHITEN_MODEL), (umas.WHITEN_MODEL_ROLE, orc.WHITEN_MODEL_ROLE)):
        # both sides whiten the same float32 input: the oracle's advantages, rounded once
        a_in = adv2_o.astype(np.float32)
        wh_o = orc.whiten_advantages(a_in, st["tok_mask"], st["tok_role"], st["model_tok_off"], w.n_roles, oscope)
        wh = umas.umas_whiten_advantages(P.to_dev(a_in), s.tok_mask, s.tok_role, st["model_tok_off"], w.n_roles, scope)
        bound = P.whiten_bounds(a_in, st["tok_mask"], st["tok_role"], st["model_tok_off"], w.n_roles, oscope == orc.WHITEN_MODEL_ROLE)
        P.close_bounded(wh.cpu().numpy(), wh_o, bound + 1e-30, 1e-5, f"whitened advantages, scope {scope}")
        assert not wh.cpu().numpy()[masked].any()
    buf = adv2.clone()
    umas.umas_whiten_advantages(buf, s.tok_mask, s.tok_role, st["model_tok_off"], w.n_roles, umas.WHITEN_MODEL, out=buf)
    assert np.array_equal(buf.cpu().numpy(), umas.umas_whiten_advantages(adv2, s.tok_mask, s.tok_role, st["model_tok_off"], w.n_roles).cpu().numpy())


def test_kl_rewards_and_whitening_small_and_full_sizes():
    shaping_case(0)
    shaping_case(2)                                    # interior masks, values, gamma < 1
    shaping_case(3)                                    # two models, five roles
    shaping_case(4, n_traj=64)                         # long segments, several blocks


def test_shaping_empty_and_errors():
    z = torch.zeros(0, device="cuda")
    zm = torch.zeros(0, dtype=torch.uint8, device="cuda")
    out, kl = umas.umas_kl_rewards(z, z, z, zm, 0.1)
    assert out.numel() == 0 and float(kl.item()) == 0.0
    a = torch.ones(8, device="cuda")
    m = torch.ones(8, dtype=torch.uint8, device="cuda")
    with pytest.raises(umas.UmasError):
        umas.umas_whiten_advantages(a, m, None, np.array([0, 5]), 1)          # offsets do not end at n_tokens
    with pytest.raises(umas.UmasError):
        umas.umas_whiten_advantages(a, m, None, np.array([0, 8]), 1, scope=umas.WHITEN_MODEL_ROLE)   # roles needed
    # a group of equal values: (A - mu) is exactly 0 whatever eps does
    out = umas.umas_whiten_advantages(a * 0.3, m, None, np.array([0, 8]), 1)
    assert not out.cpu().numpy().any()


def variants_case(cfg, entropy_coef, dual_clip, noise_scale, kl_coef=0.0, zero_adv=False, **kw):
    """Dual clip, entropy bonus and KL term of the surrogate and its backward, per model."""
    w = wl.make_workload(cfg, **kw)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    if zero_adv:                                     # only the KL term is left: every row still has a gradient
        adv_o = np.zeros_like(adv_o)
        adv = torch.zeros_like(adv)
    for m in range(w.n_models):
        spec = w.models[m]
        tdt = torch.float32 if spec.dtype == "f32" else torch.bfloat16
        tol_logp, tol = (1e-5, 1e-5) if spec.dtype == "f32" else (2e-2, 1e-2)
        t = w.model_tensors(m)
        a, e = int(st["model_tok_off"][m]), int(st["model_tok_off"][m + 1])
        ra, re = int(st["model_rowsel_off"][m]), int(st["model_rowsel_off"][m + 1])
        rows_o = st["rowsel"][ra:re]
        role_o = st["tok_role"][a:e]
        logp_o, lse_o, ent_o = orc.score(t["H"], t["W"], t["ids"], rows_o)
        logp_old = (logp_o + noise_scale * t["noise"]).astype(np.float32)
        logp_ref = (logp_o + w.critic_tensors(m)["ref_noise"]).astype(np.float32) if kl_coef > 0 else None
        stats_o, g_o = orc.ppo_loss_variants(logp_o, logp_old, adv_o[a:e], ent_o, rows_o, role_o, w.n_roles, w.clip_eps,
                                             dual_clip, entropy_coef, kl_coef, logp_ref)
        plain_o, g_plain = orc.ppo_loss(logp_o, logp_old, adv_o[a:e], ent_o, rows_o, role_o, w.n_roles, w.clip_eps)
        if dual_clip > 0:
            assert np.abs(g_o - g_plain).max() > 0, "the case must make the dual clip bind"
        dH_o, dW_o = orc.lm_head_backward_entropy(t["H"], t["W"], t["ids"], lse_o, ent_o, g_o, entropy_coef, len(rows_o), rows_o)
        H, W, ids = P.to_dev(t["H"], tdt), P.to_dev(t["W"], tdt), P.to_dev(t["ids"])
        stats, logp_new, dH, dW = umas.umas_ppo_loss_fwd_bwd(
            H, W, ids, s.rowsel[ra:re], P.to_dev(logp_old), adv[a:e].contiguous(), s.tok_role[a:e].contiguous(), w.n_roles,
            w.clip_eps, entropy_coef=entropy_coef, dual_clip=dual_clip, kl_coef=kl_coef,
            logp_ref=None if logp_ref is None else P.to_dev(logp_ref))
        torch.cuda.synchronize()
        sg = umas.read_stats(stats)
        if zero_adv:
            assert np.abs(dH_o[rows_o]).max(axis=1).min() > 0, "every scored row must have a gradient"
        for k in range(1 + w.n_roles):
            assert int(sg["n_scored"][k]) == int(stats_o[k, 4])
            o = stats_o[k, 0]
            # the loss is a mean of terms of size |A| ratio and of coef * entropy
            # (a KL term is a mean of non-negative terms: its own size)
            assert abs(float(sg["loss"][k]) - o) <= tol * max(abs(o), abs(stats_o[0, 0]), entropy_coef * abs(stats_o[k, 2]), 1e-3)
            assert abs(float(sg["clip_frac"][k]) - stats_o[k, 1]) <= max(tol * stats_o[k, 1], 2.0 / max(stats_o[k, 4], 1))
        # The KL part of g, b (1 - e^x) / S with x = logp_ref - logp, carries the absolute error of logp itself (a few
        # units in the last place of a float32 |logp| of about 6), whatever is left of 1 - e^x for a small x: an absolute
        # allowance per row of that error times the largest possible norm of d logp / d h.
        lp_err = 4e-6 if spec.dtype == "f32" else 1e-4
        row_abs = kl_coef * lp_err / max(len(rows_o), 1) * 2.0 * float(np.linalg.norm(t["W"].astype(np.float64), axis=1).max())
        P.close(dH.float().cpu().numpy(), dH_o, tol, "dH", row_abs=row_abs)
        P.close(dW.cpu().numpy(), dW_o, tol, "dW")


def test_surrogate_variants():
    variants_case(0, 0.01, 0.0, 1.0)                                           # entropy bonus alone, float32
    variants_case(0, 0.0, 3.0, 14.0)                                           # dual clip alone (noise std 0.7: ratios beyond 3)
    variants_case(0, 0.02, 2.0, 14.0)
    variants_case(2, 0.01, 3.0, 14.0, n_traj=8, tokens_per_turn=48, models=[(200, 1000, "bf16")])
    variants_case(3, 0.05, 0.0, 1.0, n_traj=6, tokens_per_turn=40, models=[(128, 700, "bf16"), (200, 1000, "bf16")])


def test_kl_loss_term():
    variants_case(0, 0.0, 0.0, 1.0, kl_coef=0.1)                                # float32
    variants_case(2, 0.0, 0.0, 1.0, kl_coef=0.1, n_traj=8, tokens_per_turn=48, models=[(200, 1000, "bf16")])   # single pass
    variants_case(1, 0.0, 0.0, 1.0, kl_coef=0.2, zero_adv=True, n_traj=16, tokens_per_turn=40, models=[(200, 1000, "bf16")])
    variants_case(3, 0.02, 3.0, 14.0, kl_coef=0.05, n_traj=6, tokens_per_turn=40, models=[(128, 700, "bf16"), (200, 1000, "bf16")])


def ready_case(cfg, n_minibatch, seed, drop=0.25, **kw):
    """Both cuts of the ready batch (by trajectories, by scored rows) against the oracle, bit for bit."""
    w = wl.make_workload(cfg, **kw)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    rng = np.random.default_rng(seed)
    keep = (rng.random(w.n_traj) >= drop).astype(np.uint8)
    keep[int(rng.integers(0, w.n_traj))] = 1
    order = rng.permutation(w.n_traj).astype(np.int32)
    rows_o, off_o = orc.ready_batch(st, w.traj_turn_off, keep, order, n_minibatch)
    rows, off = umas.umas_ready_batch(s, w.traj_turn_off, n_minibatch, keep, order)
    assert np.array_equal(off.cpu().numpy(), off_o), "minibatch offsets differ"
    assert np.array_equal(rows.cpu().numpy()[:len(rows_o)], rows_o), "minibatch rows differ"
    rows_bo, off_bo = orc.ready_batch(st, w.traj_turn_off, keep, order, n_minibatch, balance_rows=True)
    rows_b, off_b = umas.umas_ready_batch(s, w.traj_turn_off, n_minibatch, keep, order, balance_rows=True)
    assert np.array_equal(off_b.cpu().numpy(), off_bo), "minibatch offsets differ (cut by rows)"
    assert np.array_equal(rows_b.cpu().numpy()[:len(rows_bo)], rows_bo), "minibatch rows differ (cut by rows)"
    biggest = int(np.diff(off_o[:, [0, -1]]).max())
    for budget in (1, 7, max(biggest // 9, 1), max(biggest // 2, 1), biggest + 5):
        check_packed(w, st, s, keep, order, budget)
    return w, st, s, adv_o, adv, rows, off, off_o, rows_o


def check_packed(w, st, s, keep, order, budget):
    """The ready batch packed under a budget of scored rows against the oracle, bit for bit."""
    rows_o, off_o, n_o = orc.ready_batch_packed(st, w.traj_turn_off, np.ones(w.n_traj, np.uint8) if keep is None else keep,
                                                np.arange(w.n_traj) if order is None else order, budget)
    rows, off, n = umas.umas_ready_batch_packed(s, w.traj_turn_off, budget, keep, order)
    assert np.array_equal(n.cpu().numpy(), n_o), f"numbers of parts differ, budget {budget}"
    assert np.array_equal(off.cpu().numpy(), off_o), f"part offsets differ, budget {budget}"
    assert np.array_equal(rows.cpu().numpy()[:len(rows_o)], rows_o), f"packed rows differ, budget {budget}"


def test_ready_batch_index_work_is_exact():
    ready_case(0, 2, 1)
    ready_case(1, 4, 2)                                            # padding masks, 64 trajectories
    ready_case(2, 3, 3)                                            # variable turns, interior masks
    ready_case(3, 5, 4)                                            # two models
    ready_case(4, 3, 5)                                            # long turns, 16 trajectories
    ready_case(1, 7, 6, n_traj=1000)
    ready_case(1, 13, 8, n_traj=9000, tokens_per_turn=6)          # five scan tiles of trajectories, their sums handed over
    ready_case(3, 6, 9, n_traj=5000, tokens_per_turn=4, models=[(128, 700, "bf16"), (200, 1000, "bf16")])   # the same with two models
    ready_case(2, 40, 7, drop=0.9)                                 # more minibatches than kept trajectories
    # defaults: keep all, identity order, one minibatch = the selection itself
    w = wl.make_workload(3)
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    rows, off = umas.umas_ready_batch(s, w.traj_turn_off, 1)
    n = int(st["model_rowsel_off"][-1])
    assert np.array_equal(rows.cpu().numpy()[:n], st["rowsel"])
    assert np.array_equal(off.cpu().numpy()[:, 0], st["model_rowsel_off"][:-1])
    with pytest.raises(umas.UmasError):
        umas.umas_ready_batch(s, w.traj_turn_off, 2, None, np.zeros(w.n_traj, np.int32))   # not a permutation
    check_packed(w, st, s, None, None, 3000)                       # defaults: keep all, identity order
    with pytest.raises(umas.UmasError):
        umas.umas_ready_batch_packed(s, w.traj_turn_off, 0)


def test_minibatch_gradients_accumulate():
    """The update over a ready batch: one call per minibatch, gradients of the LM head accumulated."""
    w, st, s, adv_o, adv, rows, off, off_o, rows_o = ready_case(2, 3, 11, n_traj=8, tokens_per_turn=48, models=[(200, 1000, "bf16")])
    t = w.model_tensors(0)
    H, W, ids = P.to_dev(t["H"], torch.bfloat16), P.to_dev(t["W"], torch.bfloat16), P.to_dev(t["ids"])
    n = w.model_ntok[0]
    role_o = st["tok_role"][:n]
    dW = torch.empty((1000, 200), dtype=torch.float32, device="cuda")
    dW_o = np.zeros((1000, 200))
    for k in range(3):
        a, e = int(off_o[0, k]), int(off_o[0, k + 1])
        rr_o = rows_o[a:e]
        logp_o, lse_o, ent_o = orc.score(t["H"], t["W"], t["ids"], rr_o)
        logp_old = (logp_o + t["noise"]).astype(np.float32)
        stats_o, g_o = orc.ppo_loss(logp_o, logp_old, adv_o[:n], ent_o, rr_o, role_o, w.n_roles, w.clip_eps)
        dH_o, dWk = orc.lm_head_backward(t["H"], t["W"], t["ids"], lse_o, g_o, rr_o)
        dW_o += dWk
        stats, logp_new, dH, _ = umas.umas_ppo_loss_fwd_bwd(H, W, ids, rows[a:e], P.to_dev(logp_old), adv[:n].contiguous(),
                                                            s.tok_role[:n].contiguous(), w.n_roles, w.clip_eps,
                                                            accumulate_dW=(k > 0), dW=dW)
        torch.cuda.synchronize()
        sg = umas.read_stats(stats)
        assert int(sg["n_scored"][0]) == e - a
        assert abs(float(sg["loss"][0]) - stats_o[0, 0]) <= 1e-2 * max(abs(stats_o[0, 0]), 1e-3)
        P.close(dH.float().cpu().numpy(), dH_o, 1e-2, f"dH of minibatch {k}")
    P.close(dW.cpu().numpy(), dW_o, 1e-2, "accumulated dW")


@pytest.mark.parametrize("dtype,entropy_coef", [("bf16", 0.0), ("bf16", 0.02), ("f32", 0.0)])
def test_micro_batches_add_up_to_the_minibatch(dtype, entropy_coef):
    """One minibatch cut into three micro-batches of unequal size, each call normalised by the minibatch's
    row count: loss, dH and the accumulated dW equal the oracle's on the whole minibatch."""
    if dtype == "f32":      # the float32 configuration (its logits are small enough for the 1e-5 bar): 4 trajectories in 3 parts
        w, st, s, adv_o, adv, rows, off, off_o, rows_o = ready_case(0, 3, 17, drop=0.0)
    else:
        w, st, s, adv_o, adv, rows, off, off_o, rows_o = ready_case(2, 3, 17, n_traj=7, tokens_per_turn=48, models=[(200, 1000, dtype)])
    d, V = w.models[0].d, w.models[0].V
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    tol = 1e-5 if dtype == "f32" else 1e-2
    t = w.model_tensors(0)
    H, W, ids = P.to_dev(t["H"], tdt), P.to_dev(t["W"], tdt), P.to_dev(t["ids"])
    n = w.model_ntok[0]
    role_o = st["tok_role"][:n]
    rr_all = rows_o[int(off_o[0, 0]):int(off_o[0, 3])]
    S = len(rr_all)
    sizes = [int(off_o[0, k + 1] - off_o[0, k]) for k in range(3)]
    assert len(set(sizes)) > 1, "the micro-batches must differ in size"
    logp_o, lse_o, ent_o = orc.score(t["H"], t["W"], t["ids"], rr_all)
    logp_old = (logp_o + t["noise"]).astype(np.float32)
    stats_o, g_o = orc.ppo_loss_variants(logp_o, logp_old, adv_o[:n], ent_o, rr_all, role_o, w.n_roles, w.clip_eps,
                                         entropy_coef=entropy_coef)
    dH_o, dW_o = orc.lm_head_backward_entropy(t["H"], t["W"], t["ids"], lse_o, ent_o, g_o, entropy_coef, S, rr_all)
    dW = torch.empty((V, d), dtype=torch.float32, device="cuda")
    dH_sum = np.zeros(t["H"].shape)
    loss_sum, n_sum = 0.0, 0
    for k in range(3):
        a, e = int(off_o[0, k]), int(off_o[0, k + 1])
        stats, logp_new, dH, _ = umas.umas_ppo_loss_fwd_bwd(H, W, ids, rows[a:e], P.to_dev(logp_old), adv[:n].contiguous(),
                                                            s.tok_role[:n].contiguous(), w.n_roles, w.clip_eps,
                                                            entropy_coef=entropy_coef, accumulate_dW=(k > 0), norm_rows=S, dW=dW)
        torch.cuda.synchronize()
        sg = umas.read_stats(stats)
        loss_sum += float(sg["loss"][0])
        n_sum += int(sg["n_scored"][0])
        dH_k = dH.float().cpu().numpy().astype(np.float64)
        assert not dH_k[np.setdiff1d(np.arange(n), rows_o[a:e])].any()
        dH_sum += dH_k
    assert n_sum == S
    assert abs(loss_sum - stats_o[0, 0]) <= tol * max(abs(stats_o[0, 0]), 1e-3)
    P.close(dH_sum, dH_o, tol, "dH over the micro-batches")
    P.close(dW.cpu().numpy(), dW_o, tol, "dW accumulated over the micro-batches")
    with pytest.raises(umas.UmasError):
        umas.umas_ppo_loss_fwd_bwd(H, W, ids, rows[:sizes[0]], P.to_dev(logp_old), adv[:n].contiguous(),
                                   s.tok_role[:n].contiguous(), w.n_roles, w.clip_eps, norm_rows=sizes[0] - 1)


def test_packed_micro_batches_add_up_to_the_batch():
    """A ready batch packed under a row budget: as many micro-batches as the device says, each call normalised by the
    batch's row count, offsets and counts read back from the device; loss, dH and the accumulated dW equal the oracle's
    on all kept rows."""
    w, st, s, adv_o, adv, rows_g, off_g, off_o, rows_o = ready_case(2, 1, 23, n_traj=9, tokens_per_turn=48, models=[(200, 1000, "bf16")])
    rng = np.random.default_rng(23)                      # the same keep and order as ready_case drew
    keep = (rng.random(w.n_traj) >= 0.25).astype(np.uint8)
    keep[int(rng.integers(0, w.n_traj))] = 1
    order = rng.permutation(w.n_traj).astype(np.int32)
    S = int(off_o[0, 1] - off_o[0, 0])
    budget = S // 4
    rows, off, n_parts = umas.umas_ready_batch_packed(s, w.traj_turn_off, budget, keep, order)
    k_parts = int(n_parts[0].item())
    off = off.cpu().numpy()[0]
    assert k_parts >= 4 and off[0] == 0 and off[k_parts] == S
    assert np.array_equal(rows.cpu().numpy()[:S], rows_o[:S])
    t = w.model_tensors(0)
    H, W, ids = P.to_dev(t["H"], torch.bfloat16), P.to_dev(t["W"], torch.bfloat16), P.to_dev(t["ids"])
    n = w.model_ntok[0]
    rr_all = rows_o[:S]
    logp_o, lse_o, ent_o = orc.score(t["H"], t["W"], t["ids"], rr_all)
    logp_old = (logp_o + t["noise"]).astype(np.float32)
    stats_o, g_o = orc.ppo_loss(logp_o, logp_old, adv_o[:n], ent_o, rr_all, st["tok_role"][:n], w.n_roles, w.clip_eps)
    dH_o, dW_o = orc.lm_head_backward(t["H"], t["W"], t["ids"], lse_o, g_o, rr_all)
    dW = torch.empty((1000, 200), dtype=torch.float32, device="cuda")
    dH_sum, loss_sum = np.zeros(t["H"].shape), 0.0
    for k in range(k_parts):
        a, e = int(off[k]), int(off[k + 1])
        assert 0 < e - a
        stats, _, dH, _ = umas.umas_ppo_loss_fwd_bwd(H, W, ids, rows[a:e], P.to_dev(logp_old), adv[:n].contiguous(),
                                                     s.tok_role[:n].contiguous(), w.n_roles, w.clip_eps,
                                                     accumulate_dW=(k > 0), norm_rows=S, dW=dW)
        loss_sum += float(umas.read_stats(stats)["loss"][0])
        dH_sum += dH.float().cpu().numpy().astype(np.float64)
    assert abs(loss_sum - stats_o[0, 0]) <= 1e-2 * max(abs(stats_o[0, 0]), 1e-3)
    P.close(dH_sum, dH_o, 1e-2, "dH over the packed micro-batches")
    P.close(dW.cpu().numpy(), dW_o, 1e-2, "dW accumulated over the packed micro-batches")


def test_critic_micro_batches_add_up_to_the_minibatch():
    w, st, s, adv_o, adv, rows, off, off_o, rows_o = ready_case(2, 3, 19, n_traj=7, tokens_per_turn=48, models=[(200, 1000, "bf16")])
    rho, st2, r, adv2, ret_o = P.oracle_front(w)
    _, _, ret = P.gpu_front(w)
    t, c = w.model_tensors(0), w.critic_tensors(0)
    n = w.model_ntok[0]
    rr_all = rows_o[int(off_o[0, 0]):int(off_o[0, 3])]
    S = len(rr_all)
    bias = float(c["bias"])
    V_o = orc.value_head(t["H"], c["w"], bias, rr_all)
    V_old = (V_o + c["v_noise"]).astype(np.float32)
    stats_o, g_o = orc.value_loss(V_o, V_old, ret_o[:n], rr_all, st["tok_role"][:n], w.n_roles, 0.1)
    dH_o, dw_o, db_o = orc.value_head_backward(t["H"], c["w"], g_o, rr_all)
    H, wv = P.to_dev(t["H"], torch.bfloat16), P.to_dev(c["w"], torch.bfloat16)
    dw = torch.empty(200, dtype=torch.float32, device="cuda")
    db = torch.empty(1, dtype=torch.float32, device="cuda")
    dH = torch.zeros_like(H)
    loss_sum = 0.0
    for k in range(3):
        a, e = int(off_o[0, k]), int(off_o[0, k + 1])
        stats, _, _, _, _ = umas.umas_value_loss_fwd_bwd(H, wv, bias, rows[a:e], P.to_dev(V_old), ret[:n].contiguous(),
                                                         s.tok_role[:n].contiguous(), w.n_roles, 0.1, accumulate_dH=True,
                                                         accumulate_dw=(k > 0), norm_rows=S, dH=dH, dw=dw, db=db)
        torch.cuda.synchronize()
        loss_sum += float(umas.read_value_stats(stats)["loss"][0])
    assert abs(loss_sum - stats_o[0, 0]) <= 1e-2 * max(abs(stats_o[0, 0]), 1e-3)
    row_abs = 2e-2 / S * float(np.linalg.norm(c["w"].astype(np.float64)))
    P.close(dH.float().cpu().numpy(), dH_o, 1e-2, "dH over the micro-batches", row_abs=row_abs)
    P.close(dw.cpu().numpy(), dw_o, 1e-2, "dw accumulated over the micro-batches")
    assert abs(float(db.item()) - db_o) <= 1e-2 * max(abs(db_o), np.abs(g_o).sum() * 1e-2 + 1e-12)


@pytest.mark.parametrize("seed", list(range(24)) + [443, 8022, 8396])
def test_random_shapes_with_optional_terms(seed):
    """Seeded random shapes around the tile edges with random combinations of the optional terms (entropy bonus, dual
    clip, KL term, the caller's normaliser, roles, the smallest workspace).  Peaked logits as in
    test_random_small_shapes: every entry within the error bound that follows from the kernels' arithmetic, arrays
    1 %.  Seed 443 (five vocabulary entries, 169 of 1100 rows selected, chunked) once sat exactly on an ad hoc 4 %
    per-entry limit; in 8022 and 8396 a row without an advantage has log p_y within 4e-5 of the reference's, so that its
    whole gradient is the KL term's and moves by percents with the float32 rounding of log p_y."""
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([8, 64, 72, 200, 264, 320]))
    V = int(rng.choice([5, 255, 257, 700, 1030]))
    n = int(rng.choice([1, 17, 256, 257, 600, 1100]))
    H = wl.round_to_bf16((rng.normal(size=(n, d)) / np.sqrt(d) * 2).astype(np.float32))
    W = wl.round_to_bf16(rng.normal(size=(V, d)).astype(np.float32))
    ids = rng.integers(0, V, size=n).astype(np.int32)
    n_sel = int(rng.integers(1, n + 1))
    rowsel = np.sort(rng.choice(n, size=n_sel, replace=False)).astype(np.int32) if rng.random() < 0.7 else None
    sel = rowsel if rowsel is not None else np.arange(n, dtype=np.int32)
    adv = rng.normal(size=n).astype(np.float32)
    adv[rng.random(n) < 0.2] = 0.0
    if len(sel) > 300 and rng.random() < 0.7:
        adv[sel[256:512]] = 0.0                           # a block of selected rows without an advantage
    ent_c = float(rng.choice([0.0, 0.0, 0.02]))
    dual = float(rng.choice([0.0, 0.0, 2.5]))
    kl_c = float(rng.choice([0.0, 0.1, 0.3]))
    S = len(sel)
    norm = int(S + rng.integers(0, 50)) if rng.random() < 0.5 else 0
    Sn = norm if norm else S
    n_roles = int(rng.choice([0, 3]))
    role = rng.integers(0, max(n_roles, 1), size=n).astype(np.int32)
    logp_o, lse_o, ent_o = orc.score(H, W, ids, sel)
    logp_old = (logp_o + 0.3 * rng.normal(size=n)).astype(np.float32)
    logp_ref = (logp_o + 0.2 * rng.normal(size=n)).astype(np.float32)
    st_o, g_o = orc.ppo_loss_variants(logp_o, logp_old, adv, ent_o, sel, role, n_roles, 0.2, dual, ent_c, kl_c, logp_ref)
    g_o = g_o * S / Sn                                    # the oracle divides by S; the call by the caller's normaliser
    dH_o, dW_o = orc.lm_head_backward_entropy(H, W, ids, lse_o, ent_o, g_o, ent_c, Sn, sel)
    loss_o = st_o[0, 0] * S / Sn
    ws = None
    if rng.random() < 0.5:
        ws = torch.empty(umas.ppo_workspace_bytes(S, d, V, torch.bfloat16, n_roles, minimum=True), dtype=torch.uint8, device="cuda")
    what = (f"seed {seed}: d={d} V={V} n={n} sel={S} entropy={ent_c} dual={dual} kl={kl_c} norm={norm} roles={n_roles} "
            f"chunked={ws is not None}")
    stats, lp, dH, dW = umas.umas_ppo_loss_fwd_bwd(
        P.to_dev(H, torch.bfloat16), P.to_dev(W, torch.bfloat16), P.to_dev(ids), None if rowsel is None else P.to_dev(rowsel),
        P.to_dev(logp_old), P.to_dev(adv), P.to_dev(role) if n_roles else None, n_roles, 0.2, entropy_coef=ent_c, dual_clip=dual,
        kl_coef=kl_c, logp_ref=P.to_dev(logp_ref) if kl_c else None, norm_rows=norm, workspace=ws)
    torch.cuda.synchronize()
    sg = umas.read_stats(stats)
    term = float(np.abs(adv[sel]).mean())                 # the size of the terms the losses are means of
    assert abs(float(sg["loss"][0]) - loss_o) <= 1e-2 * max(abs(loss_o), term * S / Sn, 1e-3), what
    for k in range(1, 1 + n_roles):
        assert int(sg["n_scored"][k]) == int(st_o[k, 4]), what
        assert abs(float(sg["loss"][k]) - st_o[k, 0]) <= 1e-2 * max(abs(st_o[k, 0]), term, 1e-3), what
    dz = P.oracle_dz(H, W, ids, lse_o, g_o, sel, ent_o, ent_c / Sn)
    # the taken token's entry also carries the entropy term k p_y (log p_y + entropy): its slope in log p_y adds to |g|
    coef = np.abs(g_o) + abs(ent_c / Sn) * (1.0 + np.abs(ent_o) + np.abs(logp_o))
    # the KL term kl (1 - e^x) / S has the slope kl e^x / S in log p_y, however small the term itself is
    g_slope = kl_c / Sn * np.exp(logp_ref.astype(np.float64) - logp_o)
    bound_h, bound_w = P.bf16_gradient_bounds(H, W, dz, dH_o, dW_o, sel, ids, lse_o, coef, g_slope)
    P.close_bounded(dH.float().cpu().numpy(), dH_o, bound_h, 1e-2, "dH, " + what)
    P.close_bounded(dW.cpu().numpy(), dW_o, bound_w, 1e-2, "dW, " + what)


@pytest.mark.parametrize("seed", list(range(12)) + [33, 101, 333, 356, 1081, 1353, 1387])
def test_random_critic_shapes(seed):
    """Seeded random shapes of the critic's fused pass in both dtypes: hidden sizes around the vector width, row counts
    around a workgroup's share, random selections, roles, a caller's normaliser.  Seeds 33, 101, 333 and 356 are
    float32 cases with d = 4096 whose dH once missed 1e-5 by a factor of up to two, when the value head summed its
    float32 products in float32; the float32 path now carries its sums in float64.  In 1081 and 1387 (5000 rows of
    bf16) one row's clipped and unclipped terms are equal to within the float32 rounding of its value, and the device
    and the oracle took different branches; 1353 is a float32 row whose V - R cancels."""
    rng = np.random.default_rng(31000 + seed)
    bf = rng.random() < 0.7
    d = int(rng.choice([8, 16, 64, 72, 200, 512, 520, 2048, 3584, 8192])) if bf else int(rng.choice([4, 12, 64, 100, 1024, 4096]))
    n = int(rng.choice([1, 3, 8, 9, 64, 257, 1000, 5000]))
    H = rng.normal(size=(n, d)).astype(np.float32)
    w_ = (rng.normal(size=d) * 0.05).astype(np.float32)
    if bf:
        H, w_ = wl.round_to_bf16(H), wl.round_to_bf16(w_)
    tdt = torch.bfloat16 if bf else torch.float32
    n_sel = int(rng.integers(0, n + 1))
    rowsel = np.sort(rng.choice(n, size=n_sel, replace=False)).astype(np.int32) if rng.random() < 0.7 else None
    sel = rowsel if rowsel is not None else np.arange(n, dtype=np.int32)
    S = len(sel)
    n_roles = int(rng.choice([0, 4]))
    role = rng.integers(0, max(n_roles, 1), size=n).astype(np.int32)
    bias = float(rng.normal() * 0.1)
    V_o = orc.value_head(H, w_, bias, sel)
    V_old = (V_o + 0.1 * rng.normal(size=n)).astype(np.float32)
    ret = (V_o + 0.3 * rng.normal(size=n)).astype(np.float32)
    norm = int(S + rng.integers(0, 9)) if (rng.random() < 0.5 and S > 0) else 0
    Sn = norm if norm else max(S, 1)
    st_o, g_o = orc.value_loss(V_o, V_old, ret, sel, role, n_roles, 0.1)
    g_o = g_o * max(S, 1) / Sn
    dH_o, dw_o, db_o = orc.value_head_backward(H, w_, g_o, sel)
    what = f"seed {seed}: bf16={bf} d={d} n={n} sel={S} rowsel={rowsel is not None} roles={n_roles} norm={norm}"
    tol = 1e-2 if bf else 1e-5
    lim = 2e-2 if bf else 1e-5 * max(1.0, np.abs(V_o).max(initial=0))            # the value itself: absolute / relative to its scale
    stats, V_new, dH, dw, db = umas.umas_value_loss_fwd_bwd(
        P.to_dev(H, tdt), P.to_dev(w_, tdt), bias, None if rowsel is None else P.to_dev(rowsel), P.to_dev(V_old), P.to_dev(ret),
        P.to_dev(role) if n_roles else None, n_roles, 0.1, norm_rows=norm)
    torch.cuda.synchronize()
    sg = umas.read_value_stats(stats)
    assert int(sg["n_scored"][0]) == S, what
    assert np.abs(V_new.cpu().numpy() - V_o).max(initial=0) <= lim, what
    if S:
        assert abs(float(sg["loss"][0]) - st_o[0, 0] * S / Sn) <= tol * max(abs(st_o[0, 0]) * S / Sn, 1e-3) + lim * 0.5, what
    if S == 0:
        assert not dH.float().cpu().numpy().any() and not dw.cpu().numpy().any(), what
        return
    # The value is a float32 number on the device: dV bounds its distance from the oracle's (bf16 path: float32 sums of
    # d / 64 products per lane and a tree over the lanes; float32 path: float64 sums, one rounding; then the bias).
    H64, w64 = H.astype(np.float64), w_.astype(np.float64)
    dV = np.zeros(n)
    dV[sel] = 2.0 ** -24 * (((d / 64 + 8) * (np.abs(H64[sel]) @ np.abs(w64)) if bf else 0.0) + 2 * np.abs(V_o[sel]) + abs(bias))
    # g_i = (V_i - R_i) / S inherits the absolute error of V_i, whatever is left of V_i - R_i after cancellation; and a
    # row whose two loss terms are equal to within that error may take either branch (gradient (V - R) / S or 0): such
    # rows are checked against the branch the device took, and the sums over rows are formed with that branch.
    _, g_hi = orc.value_loss(V_o + dV, V_old, ret, sel, role, n_roles, 0.1)
    _, g_lo = orc.value_loss(V_o - dV, V_old, ret, sel, role, n_roles, 0.1)
    either = (g_hi == 0) != (g_lo == 0)
    dH_g = dH.float().cpu().numpy().astype(np.float64)
    g_use = g_o.copy()
    for i in np.nonzero(either)[0]:
        took_zero = not dH_g[i].any()
        g_use[i] = 0.0 if took_zero else (V_o[i] - float(ret[i])) / Sn
    dH_o, dw_o, db_o = orc.value_head_backward(H, w_, g_use, sel)
    rms = float(np.sqrt(np.mean(dH_o * dH_o)))
    bound_h = tol * np.maximum(np.abs(dH_o), rms) + (dV / Sn)[:, None] * np.abs(w64)[None, :] + 1e-30
    P.close_bounded(dH_g, dH_o, bound_h, tol, "dH, " + what)
    rms_w = float(np.sqrt(np.mean(dw_o * dw_o)))
    bound_w = tol * np.maximum(np.abs(dw_o), rms_w) + (dV[sel] / Sn) @ np.abs(H64[sel]) + 1e-30
    P.close_bounded(dw.cpu().numpy(), dw_o, bound_w, tol + float(np.linalg.norm((dV[sel] / Sn) @ np.abs(H64[sel])) / max(np.linalg.norm(dw_o), 1e-300)),
                    "dw, " + what)


@pytest.mark.parametrize("seed", range(30))
def test_random_graphs_around_the_update(seed):
    """Ready batch (bit-exact), KL-penalised rewards and both whitening scopes on seeded random workflow graphs."""
    w, kw = wl.random_graph(seed)
    rho, st, r, adv_o, ret_o = P.oracle_front(w, **kw)
    s, adv, ret = P.gpu_front(w, **kw)
    rng = np.random.default_rng(777 + seed)
    n = w.n_tokens
    keep = (rng.random(w.n_traj) >= 0.3).astype(np.uint8)
    order = rng.permutation(w.n_traj).astype(np.int32)
    n_parts = int(rng.integers(1, 9))
    rows_o, off_o = orc.ready_batch(st, w.traj_turn_off, keep, order, n_parts)
    rows, off = umas.umas_ready_batch(s, w.traj_turn_off, n_parts, keep, order)
    assert np.array_equal(off.cpu().numpy(), off_o), "minibatch offsets differ"
    assert np.array_equal(rows.cpu().numpy()[:len(rows_o)], rows_o), "minibatch rows differ"
    _, off_bo = orc.ready_batch(st, w.traj_turn_off, keep, order, n_parts, balance_rows=True)
    _, off_b = umas.umas_ready_batch(s, w.traj_turn_off, n_parts, keep, order, balance_rows=True)
    assert np.array_equal(off_b.cpu().numpy(), off_bo), "minibatch offsets differ (cut by rows)"
    check_packed(w, st, s, keep, order, int(rng.choice([1, 3, 40, 700, 10 ** 6])))
    logp = (-3.0 * rng.random(n)).astype(np.float32)
    logp_ref = (logp + 0.1 * rng.normal(size=n)).astype(np.float32)
    r_o, kl_o = orc.kl_penalised_rewards(r, logp, logp_ref, st["tok_mask"], 0.05)
    r_g, kl_g = umas.umas_kl_rewards(s.tok_reward, P.to_dev(logp), P.to_dev(logp_ref), s.tok_mask, 0.05)
    P.close(r_g.cpu().numpy(), r_o, 1e-5, "penalised rewards")
    assert abs(float(kl_g.item()) - kl_o) <= 1e-5 * max(abs(kl_o), float(np.abs(logp - logp_ref).mean()) if n else 0.0) + 1e-30
    a_in = (rng.normal(size=n) * 3 + 1).astype(np.float32)
    for scope, oscope in ((umas.WHITEN_MODEL, orc.WHITEN_MODEL), (umas.WHITEN_MODEL_ROLE, orc.WHITEN_MODEL_ROLE)):
        wh_o = orc.whiten_advantages(a_in, st["tok_mask"], st["tok_role"], st["model_tok_off"], w.n_roles, oscope)
        wh = umas.umas_whiten_advantages(P.to_dev(a_in), s.tok_mask, s.tok_role, st["model_tok_off"], w.n_roles, scope)
        # groups of a few tokens: the whitened values are differences from a mean, on the scale of 1, and inherit the
        # float32 rounding of the values and of the mean divided by the group's deviation
        bound = P.whiten_bounds(a_in, st["tok_mask"], st["tok_role"], st["model_tok_off"], w.n_roles, oscope == orc.WHITEN_MODEL_ROLE)
        P.close_bounded(wh.cpu().numpy(), wh_o, bound + 1e-30, 1e-5, f"whitened advantages, scope {scope}")


def test_roles_outside_the_range_join_no_per_role_statistic():
    """Role ids are device data the host cannot check: a row or token whose role lies outside [0, n_roles) still counts
    in the model's totals and gradients and joins no role's statistics, in the policy update, the value update and
    the per-role whitening (where it keeps 0).  The oracle's per-role selections leave such rows out by themselves."""
    w = wl.make_workload(1, n_traj=6, tokens_per_turn=40, models=[(64, 300, "bf16")])
    t = w.model_tensors(0)
    n, R = len(t["ids"]), 3
    rng = np.random.default_rng(41)
    role = rng.integers(0, R, n).astype(np.int32)
    stray = rng.choice(n, 40, replace=False)
    role[stray] = rng.choice(np.array([-1, -7, R, R + 5, 10 ** 6], np.int32), len(stray))
    rows = np.arange(n, dtype=np.int32)
    logp_o, lse_o, ent_o = orc.score(t["H"], t["W"], t["ids"], rows)
    logp_old = (logp_o + t["noise"]).astype(np.float32)
    adv = rng.normal(size=n).astype(np.float32)
    st_o, g_o = orc.ppo_loss(logp_o, logp_old, adv, ent_o, rows, role, R, 0.2)
    assert st_o[1:, 4].sum() == n - len(stray)
    H, W = P.to_dev(t["H"], torch.bfloat16), P.to_dev(t["W"], torch.bfloat16)
    stats, logp_new, dH, dW = umas.umas_ppo_loss_fwd_bwd(H, W, P.to_dev(t["ids"]), None, P.to_dev(logp_old), P.to_dev(adv),
                                                        P.to_dev(role), R, 0.2)
    sg = umas.read_stats(stats)
    for k in range(1 + R):
        assert int(sg["n_scored"][k]) == int(st_o[k, 4])
        assert abs(float(sg["loss"][k]) - st_o[k, 0]) <= 1e-2 * max(abs(st_o[k, 0]), float(np.abs(adv).mean()))
        assert abs(float(sg["entropy_mean"][k]) - st_o[k, 2]) <= 2e-2 and abs(float(sg["approx_kl"][k]) - st_o[k, 3]) <= 2e-2
    dH_o, dW_o = orc.lm_head_backward(t["H"], t["W"], t["ids"], lse_o, g_o, rows)
    P.close(dH.float().cpu().numpy(), dH_o, 1e-2, "dH")
    P.close(dW.cpu().numpy(), dW_o, 1e-2, "dW")
    # value head
    wv = (rng.normal(size=64) * 0.1).astype(np.float32)
    wv_b = torch.from_numpy(wv).bfloat16()
    V_o = orc.value_head(t["H"], wv_b.float().numpy(), 0.1, rows)
    v_old = (V_o + 0.05 * rng.normal(size=n)).astype(np.float32)
    ret = rng.normal(size=n).astype(np.float32)
    sv_o, gv_o = orc.value_loss(V_o, v_old, ret, rows, role, R, 0.2)
    stats_v, V_new, dHv, dw, db = umas.umas_value_loss_fwd_bwd(H, wv_b.cuda(), 0.1, None, P.to_dev(v_old), P.to_dev(ret),
                                                             P.to_dev(role), R, 0.2)
    sv = umas.read_value_stats(stats_v)
    for k in range(1 + R):
        assert int(sv["n_scored"][k]) == int(sv_o[k, 3])
        assert abs(float(sv["loss"][k]) - sv_o[k, 0]) <= 1e-2 * max(abs(sv_o[k, 0]), 1e-3)
        assert abs(float(sv["value_mean"][k]) - sv_o[k, 2]) <= 1e-2 * max(abs(sv_o[k, 2]), float(np.abs(V_o).mean()))
    # whitening per (model, role): the stray tokens keep 0 on both sides
    mask = (rng.random(n) < 0.8).astype(np.uint8)
    a_in = rng.normal(size=n).astype(np.float32)
    off = np.array([0, n], np.int64)
    wh_o = orc.whiten_advantages(a_in, mask, role, off, R, orc.WHITEN_MODEL_ROLE)
    wh = umas.umas_whiten_advantages(P.to_dev(a_in), P.to_dev(mask), P.to_dev(role), off, R, umas.WHITEN_MODEL_ROLE).cpu().numpy()
    assert not wh[stray].any() and not wh_o[stray].any()
    P.close(wh, wh_o, 1e-5, "whitened advantages")
