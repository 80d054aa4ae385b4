"""The update calls launch kernels only (no memset nodes, no copies, no host waits), so a caller can record
them into a HIP graph.  The graph is replayed several times with the advantages changed in place and eager
library work and synchronisations between the replays; every replay is checked against the CPU oracle and
against the eager call on the same inputs."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import umas_oracle as orc
import paper_2605_26646_amd as umas
from paper_2605_26646_amd import binding
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("entropy_coef", [0.0, 0.02])
def test_update_calls_replay_from_a_hip_graph(entropy_coef):
    w = wl.make_workload(2, n_traj=8, tokens_per_turn=48, models=[(200, 1000, "bf16")])
    rho, st, r, adv_o, ret_o = P.oracle_front(w)
    s, adv, ret = P.gpu_front(w)
    t, c = w.model_tensors(0), w.critic_tensors(0)
    n = w.model_ntok[0]
    S = int(st["model_rowsel_off"][1])
    rows_o, role_o = st["rowsel"][:S], st["tok_role"][:n]
    H, W, ids = P.to_dev(t["H"], torch.bfloat16), P.to_dev(t["W"], torch.bfloat16), P.to_dev(t["ids"])
    wv, bias = P.to_dev(c["w"], torch.bfloat16), float(c["bias"])
    rowsel, role = s.rowsel[:S].contiguous(), s.tok_role[:n].contiguous()
    logp_o, lse_o, ent_o = orc.score(t["H"], t["W"], t["ids"], rows_o)
    logp_old = P.to_dev((logp_o + t["noise"]).astype(np.float32))
    V_o = orc.value_head(t["H"], c["w"], bias, rows_o)
    V_old = P.to_dev((V_o + c["v_noise"]).astype(np.float32))

    # static buffers of the graph
    adv_s, ret_s = adv[:n].clone(), ret[:n].clone()
    dW = torch.empty((1000, 200), dtype=torch.float32, device="cuda")
    dH = torch.empty_like(H)
    logp_new = torch.empty(n, dtype=torch.float32, device="cuda")
    stats = torch.empty((1 + w.n_roles) * binding.STATS_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
    ws = torch.empty(umas.ppo_workspace_bytes(S, 200, 1000, torch.bfloat16, w.n_roles), dtype=torch.uint8, device="cuda")
    dHv = torch.empty_like(H)
    dwv = torch.empty(200, dtype=torch.float32, device="cuda")
    dbv = torch.empty(1, dtype=torch.float32, device="cuda")
    v_new = torch.empty(n, dtype=torch.float32, device="cuda")
    vstats = torch.empty((1 + w.n_roles) * binding.VALUE_STATS_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
    vws = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")

    def update(out):
        dW_, dH_, lp_, st_, dHv_, dwv_, dbv_, vn_, vst_ = out
        umas.umas_ppo_loss_fwd_bwd(H, W, ids, rowsel, logp_old, adv_s, role, w.n_roles, w.clip_eps,
                                   entropy_coef=entropy_coef, dW=dW_, dH=dH_, logp_new=lp_, stats=st_, workspace=ws)
        umas.umas_value_loss_fwd_bwd(H, wv, bias, rowsel, V_old, ret_s, role, w.n_roles, 0.1, dH=dHv_, dw=dwv_, db=dbv_,
                                     value_new=vn_, stats=vst_, workspace=vws)

    outs = (dW, dH, logp_new, stats, dHv, dwv, dbv, v_new, vstats)
    update(outs)                                     # once eagerly: the library is loaded and has run
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        update(outs)
    torch.cuda.synchronize()

    for k, factor in enumerate((1.0, -0.5, 2.0)):
        adv_k = (adv_o[:n] * factor).astype(np.float32)
        ret_k = (ret_o[:n] * (1.0 + 0.1 * k)).astype(np.float32)
        adv_s.copy_(P.to_dev(adv_k))
        ret_s.copy_(P.to_dev(ret_k))
        for o in outs:                               # nothing of an earlier replay may pass for this one's result
            o.view(torch.uint8).fill_(0xFF) if o.dtype != torch.uint8 else o.fill_(0xFF)
        umas.umas_policy_logprobs(H, W, ids, rowsel)   # eager work of the library between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        eager = tuple(torch.empty_like(o) for o in outs)
        update(eager)
        torch.cuda.synchronize()
        # against the eager call: same kernels, same inputs (dW adds its one-hot rows with float atomics)
        for name, a, b in zip(("dW", "dH", "logp_new", "stats", "dH_v", "dw_v", "db_v", "value_new", "stats_v"), got, eager):
            if a.dtype == torch.uint8:
                assert torch.equal(a, b), f"replay {k}: {name} differs from the eager call"
            else:
                a64, b64 = a.double(), b.double()
                lim = 1e-5 * float(b64.abs().max()) + 1e-30
                assert float((a64 - b64).abs().max()) <= lim, f"replay {k}: {name} differs from the eager call"
        # against the oracle
        stats_o, g_o = orc.ppo_loss_variants(logp_o, logp_old.cpu().numpy(), adv_k, ent_o, rows_o, role_o, w.n_roles,
                                             w.clip_eps, entropy_coef=entropy_coef)
        dH_o, dW_o = orc.lm_head_backward_entropy(t["H"], t["W"], t["ids"], lse_o, ent_o, g_o, entropy_coef, S, rows_o)
        sg = umas.read_stats(got[3])
        assert abs(float(sg["loss"][0]) - stats_o[0, 0]) <= 1e-2 * max(abs(stats_o[0, 0]), 1e-3)
        P.close(got[1].float().cpu().numpy(), dH_o, 1e-2, f"replay {k}: dH")
        P.close(got[0].cpu().numpy(), dW_o, 1e-2, f"replay {k}: dW")
        vstats_o, gv_o = orc.value_loss(V_o, V_old.cpu().numpy(), ret_k, rows_o, role_o, w.n_roles, 0.1)
        dHv_o, dwv_o, dbv_o = orc.value_head_backward(t["H"], c["w"], gv_o, rows_o)
        P.close(got[5].cpu().numpy(), dwv_o, 1e-2, f"replay {k}: dw of the value head")
        vg = umas.read_value_stats(got[8])
        assert abs(float(vg["loss"][0]) - vstats_o[0, 0]) <= 1e-2 * max(abs(vstats_o[0, 0]), 1e-3)


def test_scan_and_shaping_calls_replay_from_a_hip_graph():
    """umas_advantages (with a segment long enough to be cut inside, so that the kernel whose workgroups hand their
    state over through published maps is part of the graph), umas_kl_rewards and umas_whiten_advantages recorded once
    and replayed with the values and log-probs changed in place."""
    w = wl.make_workload(0)
    rng = np.random.default_rng(77)
    lens = np.array([40000, 7, 300, 2500, 0, 64], np.int64)
    w.n_traj, w.n_turns, w.n_roles, w.n_models = 2, len(lens), 2, 1
    w.traj_turn_off = np.array([0, 3, 6], np.int32)
    w.turn_role = np.array([0, 1, 0, 1, 1, 0], np.int32)
    w.role_to_model = np.zeros(2, np.int32)
    w.turn_tok_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    w.n_tokens = int(w.turn_tok_off[-1])
    w.turn_pred_off, w.turn_pred, w.traj_group = None, None, None
    w.tok_mask = (rng.random(w.n_tokens) < 0.8).astype(np.uint8)
    w.traj_reward = rng.normal(size=2).astype(np.float32)
    w.turn_reward = rng.normal(size=w.n_turns).astype(np.float32)
    w.role_reward = None
    n = w.n_tokens
    kw = dict(seg_mode=1, gamma_turn=0.9, place_mode=wl.PLACE_ALL, gamma=1.0, lam=0.97)
    w.value = np.zeros(n, np.float32)
    rho, st, r, _, _ = P.oracle_front(w, **kw)
    s, _, _ = P.gpu_front(w, **kw)
    value_s = torch.zeros(n, dtype=torch.float32, device="cuda")
    logp_s = torch.zeros(n, dtype=torch.float32, device="cuda")
    logp_ref_s = torch.zeros(n, dtype=torch.float32, device="cuda")
    off = s.model_tok_off.cpu().numpy()

    def calls():
        adv, ret = umas.umas_advantages(s, value_s, 1.0, 0.97, 0.9, 1)
        r2, kl = umas.umas_kl_rewards(s.tok_reward, logp_s, logp_ref_s, s.tok_mask, 0.05)
        a2 = umas.umas_whiten_advantages(adv, s.tok_mask, s.tok_role, off, w.n_roles, umas.WHITEN_MODEL_ROLE)
        return adv, ret, r2, kl, a2

    calls()                                          # once eagerly
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs = calls()
    torch.cuda.synchronize()
    for k in range(3):
        value = (0.1 * rng.normal(size=n)).astype(np.float32)
        logp = (-3.0 * rng.random(n)).astype(np.float32)
        logp_ref = (logp + 0.1 * rng.normal(size=n)).astype(np.float32)
        value_s.copy_(P.to_dev(value)); logp_s.copy_(P.to_dev(logp)); logp_ref_s.copy_(P.to_dev(logp_ref))
        for o in outs:
            o.fill_(float("nan"))
        P.gpu_front(w, **kw)                         # eager work of the library between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        eager = calls()
        torch.cuda.synchronize()
        for name, a, b in zip(("adv", "ret", "penalised rewards", "mean kl", "whitened"), got, eager):
            assert torch.equal(a, b), f"replay {k}: {name} differs from the eager call"
        adv_o, ret_o = orc.advantages(st, w.traj_turn_off, r, value, 1.0, 0.97, 0.9, 1)
        P.close(got[0].cpu().numpy(), adv_o, 1e-5, f"replay {k}: advantages")
        r_o, kl_o = orc.kl_penalised_rewards(r, logp, logp_ref, st["tok_mask"], 0.05)
        P.close(got[2].cpu().numpy(), r_o, 1e-5, f"replay {k}: penalised rewards")
