"""Benchmark of the model-local worker step on one MI355X.

A step is one pass of the whole hot path over one batch of the Qwen2.5-3B-shaped pipeline
workload (configuration 1: d=2048, V=151936, 64 trajectories x 3 roles x 256 tokens, bf16):
umas_assign_token_rewards -> umas_advantages -> umas_ppo_loss_fwd_bwd (scoring, clipped
surrogate, backward to hidden states and LM-head weights).  All inputs are resident in HBM
before the timed region.  Prints one JSON line.

Besides the headline the line carries: the same update with every row given a gradient, the update at
three workspace sizes, one step each of the other bf16 configurations (medians of event-timed
iterations), the reward / scan / shaping kernels on batch-replicated instances against the HBM
roofline, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0


def cpu_baseline(w, t, sample_rows):
    """The oracle's scoring + surrogate + backward on the first `sample_rows` rows, host cores only."""
    from oracle import umas_oracle as orc
    n = sample_rows
    H, ids = t["H"][:n], t["ids"][:n]
    t0 = time.perf_counter()
    logp, lse, ent = orc.score(H, t["W"], ids)
    logp_old = (logp + t["noise"][:n]).astype(np.float32)
    adv = np.ones(n)
    stats, g = orc.ppo_loss(logp, logp_old, adv, ent, None, np.zeros(n, np.int32), 0, w.clip_eps)
    orc.lm_head_backward(H, t["W"], ids, lse, g)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": n / dt, "unit": "scored tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n} rows of the same workload (same W), scoring+loss+backward in float64, {dt:.1f} s"}


def kernel_source_hash():
    """sha256 over the MFMA kernels' sources with comments and white space removed: a change of the code
    invalidates the stored counters, a change of a comment does not."""
    import hashlib, re
    h = hashlib.sha256()
    for fn in ("umas_score.hip", "umas_mfma.h", "umas_common.h"):
        text = open(os.path.join(ROOT, "paper_2605_26646_amd", "csrc", fn)).read()
        text = re.sub(r"//[^\n]*", "", text)
        h.update(re.sub(r"\s+", "", text).encode())
    return h.hexdigest()


def stored_traffic(kernel):
    """HBM-side bytes per launch of `kernel` from the committed counter summary (FETCH_SIZE + WRITE_SIZE,
    scaled by what the same counters read for a plain copy); None when the kernel sources have changed
    since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "bench_cfg1_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    k = rec["kernels"].get(kernel)
    if kernel_source_hash() != rec.get("kernel_sources_sha256") or k is None:
        return None
    return k["read_bytes"] + k["written_bytes"]


def event_times_ms(torch, fn, iters, warmup):
    """Per-iteration durations of fn() between events on the current stream (the one the library launches on)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    evs[0].record()
    for i in range(iters):
        fn()
        evs[i + 1].record()
    torch.cuda.synchronize()
    return [evs[i].elapsed_time(evs[i + 1]) for i in range(iters)]


def assign_kwargs(w, mask):
    return dict(n_roles=w.n_roles, n_models=w.n_models, role_to_model=w.role_to_model, traj_turn_off=w.traj_turn_off,
                turn_role=w.turn_role, turn_tok_off=w.turn_tok_off, tok_mask_global=mask, turn_pred_off=w.turn_pred_off,
                turn_pred=w.turn_pred, traj_group=w.traj_group, role_reward=w.role_reward, turn_reward=w.turn_reward,
                traj_reward=w.traj_reward, place_mode=w.place_mode)


def config_step(umas, wl, torch, cfg, iters, **overrides):
    """One whole step (routing + advantages + the update of every model) of another configuration at its full size:
    median of `iters` event-timed iterations after 2 warm-ups.  Old log-probs are the scoring pass's own plus the
    generator's noise; every zero advantage is replaced by a small number so that no row is left out."""
    dev = torch.device("cuda:0")
    w = wl.make_workload(cfg, **overrides)
    mask = torch.from_numpy(w.tok_mask).to(dev)
    value = None if w.value is None else torch.from_numpy(w.value).to(dev)
    kw = assign_kwargs(w, mask)
    s = umas.umas_assign_token_rewards(**kw)
    torch.cuda.synchronize()
    tok_off = s.model_tok_off.cpu().numpy()
    sel_off = s.model_rowsel_off.cpu().numpy()
    models = []
    flop = 0.0
    for m, spec in enumerate(w.models):
        t = w.model_tensors(m)
        H = torch.from_numpy(t["H"]).to(dev).bfloat16()
        W = torch.from_numpy(t["W"]).to(dev).bfloat16()
        ids = torch.from_numpy(t["ids"]).to(dev)
        noise = torch.from_numpy(t["noise"]).to(dev)
        del t
        a, e = int(tok_off[m]), int(tok_off[m + 1])
        ra, re = int(sel_off[m]), int(sel_off[m + 1])
        n_sel = re - ra
        logp, _, _ = umas.umas_policy_logprobs(H, W, ids, s.rowsel[ra:re])
        ws = torch.empty(umas.ppo_workspace_bytes(n_sel, spec.d, spec.V, torch.bfloat16, w.n_roles), dtype=torch.uint8, device=dev)
        models.append(dict(H=H, W=W, ids=ids, logp_old=logp + noise, a=a, e=e, ra=ra, re=re, ws=ws,
                           dW=torch.empty((spec.V, spec.d), dtype=torch.float32, device=dev), dH=torch.empty_like(H),
                           logp_new=torch.empty(e - a, dtype=torch.float32, device=dev),
                           stats=torch.empty((1 + w.n_roles) * 32, dtype=torch.uint8, device=dev)))
        flop += 6.0 * spec.V * spec.d * n_sel

    def step():
        st = umas.umas_assign_token_rewards(**kw)
        adv, _ = umas.umas_advantages(st, value, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
        adv = torch.where(adv == 0, torch.full_like(adv, 1e-3), adv)
        for M in models:
            umas.umas_ppo_loss_fwd_bwd(M["H"], M["W"], M["ids"], st.rowsel[M["ra"]:M["re"]], M["logp_old"],
                                       adv[M["a"]:M["e"]].contiguous(), st.tok_role[M["a"]:M["e"]].contiguous(), w.n_roles,
                                       w.clip_eps, dW=M["dW"], dH=M["dH"], logp_new=M["logp_new"], stats=M["stats"],
                                       workspace=M["ws"])

    ms = event_times_ms(torch, step, iters, 2)
    med = statistics.median(ms)
    n_scored = int(sel_off[-1])
    out = {"workload": w.name, "tokens": w.n_tokens, "scored_tokens": n_scored,
           "models": [{"d": sp.d, "V": sp.V, "scored": int(sel_off[m + 1] - sel_off[m])} for m, sp in enumerate(w.models)],
           "iterations": iters, "median_ms_per_step": med, "min_ms": min(ms), "max_ms": max(ms),
           "scored_tokens_per_s": n_scored / (med * 1e-3), "every_row_given_a_gradient": True,
           "frac_of_bf16_peak_6Vd": flop / (med * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "losses": [float(umas.read_stats(M["stats"])["loss"][0]) for M in models]}
    del models
    torch.cuda.empty_cache()
    return out


def hbm_kernels(umas, wl, torch, cfg, n_traj, iters=5, shaping=False, traj_scan=False):
    """Reward/routing and scan kernels on a batch-replicated instance: achieved GB/s on algorithmic bytes."""
    w = wl.make_workload(cfg, n_traj=n_traj)
    mask = torch.from_numpy(w.tok_mask).cuda()
    value = None if w.value is None else torch.from_numpy(w.value).cuda()
    kw = dict(n_roles=w.n_roles, n_models=w.n_models, role_to_model=w.role_to_model, traj_turn_off=w.traj_turn_off,
              turn_role=w.turn_role, turn_tok_off=w.turn_tok_off, tok_mask_global=mask, traj_group=w.traj_group,
              role_reward=w.role_reward, turn_reward=w.turn_reward, traj_reward=w.traj_reward, place_mode=w.place_mode)
    for _ in range(2):
        s = umas.umas_assign_token_rewards(**kw)
        umas.umas_advantages(s, value, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
    torch.cuda.synchronize()
    umas.profile_enable(True)
    for _ in range(iters):
        s = umas.umas_assign_token_rewards(**kw)
        umas.umas_advantages(s, value, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
    torch.cuda.synchronize()
    prof = umas.profile_read()
    umas.profile_enable(False)
    N = w.n_tokens
    scored = int(w.tok_mask.sum())
    scan_ms = sum(prof[k][0] for k in prof if k.startswith("k_gae_scan")) / iters
    route_names = [k for k in prof if not k.startswith("k_gae_scan")]
    route_ms = sum(prof[k][0] for k in route_names) / iters
    scan_bytes = (17 if value is not None else 13) * N
    # global mask read; perm, turn, role, mask, flags, reward written per token; rowsel per scored token
    route_bytes = (1 + 8 + 4 + 4 + 1 + 1 + 4) * N + 4 * scored

    def entry(t, nbytes):
        return {"ms": t, "algorithmic_bytes": nbytes, "GBps": nbytes / t / 1e6, "frac_of_hbm_peak": nbytes / t / 1e6 / PEAK_HBM_GBPS}
    extra = {}
    if traj_scan:
        # the same scan over trajectory runs (one episode per trajectory and model: segments of 5120 to 15360 tokens here)
        for gt, name in ((1.0, "scan_traj_segments"), (0.97, "scan_traj_segments_with_step_discount")):
            umas.umas_advantages(s, value, w.gamma, w.lam, gt, 1)
            torch.cuda.synchronize()
            umas.profile_enable(True)
            for _ in range(iters):
                umas.umas_advantages(s, value, w.gamma, w.lam, gt, 1)
            torch.cuda.synchronize()
            p3 = umas.profile_read()
            umas.profile_enable(False)
            t = sum(p3[k][0] for k in p3) / iters
            extra[name] = entry(t, scan_bytes)
            extra[name]["kernels_ms"] = {k: v[0] / iters for k, v in p3.items()}
    # the steps around the advantage step on the same instance: KL-penalised rewards, whitening, ready batch
    if shaping:
        logp = torch.empty(N, dtype=torch.float32, device="cuda").uniform_(-3.0, 0.0)
        logp_ref = logp + 0.1 * torch.randn(N, device="cuda")
        adv, _ = umas.umas_advantages(s, value, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
        order = np.random.default_rng(7).permutation(w.n_traj).astype(np.int32)
        keep = (np.random.default_rng(8).random(w.n_traj) < 0.9).astype(np.uint8)

        def run_extra():
            umas.umas_kl_rewards(s.tok_reward, logp, logp_ref, s.tok_mask, 0.05)
            umas.umas_whiten_advantages(adv, s.tok_mask, s.tok_role, w_off, w.n_roles, umas.WHITEN_MODEL_ROLE)
            umas.umas_ready_batch(s, w.traj_turn_off, 8, keep, order)
        w_off = s.model_tok_off.cpu().numpy()
        run_extra()
        torch.cuda.synchronize()
        umas.profile_enable(True)
        for _ in range(iters):
            run_extra()
        torch.cuda.synchronize()
        p2 = umas.profile_read()
        umas.profile_enable(False)
        kept_scored = scored * float(keep.mean())
        groups = (("kl_rewards", ("k_kl_",), 17 * N), ("whiten_advantages", ("k_whiten_",), 22 * N))
        used = set()
        for name, prefixes, nbytes in groups:
            ks = [k for k in p2 if k.startswith(prefixes)]
            used.update(ks)
            extra[name] = entry(sum(p2[k][0] for k in ks) / iters, nbytes)
        rb = [k for k in p2 if k not in used]
        extra["ready_batch"] = entry(sum(p2[k][0] for k in rb) / iters, 8 * kept_scored)
        extra["ready_batch"]["kernels_ms"] = {k: p2[k][0] / iters for k in rb}
        # the same rows cut under a budget of scored rows that gives about 64 micro-batches
        budget = max(int(kept_scored) // 64, 1)
        umas.umas_ready_batch_packed(s, w.traj_turn_off, budget, keep, order)
        torch.cuda.synchronize()
        umas.profile_enable(True)
        for _ in range(iters):
            _, _, n_parts = umas.umas_ready_batch_packed(s, w.traj_turn_off, budget, keep, order)
        torch.cuda.synchronize()
        p4 = umas.profile_read()
        umas.profile_enable(False)
        extra["ready_batch_packed"] = {"max_rows": budget, "parts": int(n_parts[0].item()), "ms": sum(v[0] for v in p4.values()) / iters,
                                       "kernels_ms": {k: v[0] / iters for k, v in p4.items()}}
    return {"workload": f"{w.name} x{n_traj} trajectories", "tokens": N, **extra,
            "scan": entry(scan_ms, scan_bytes), "route_place": entry(route_ms, route_bytes),
            "kernels_ms": {k: v[0] / iters for k, v in prof.items()}}


def critic_kernel(umas, torch, H, n_sel, d, rep=8, iters=5):
    """The critic's fused pass (value head, clipped value loss, backward) on the benchmark's hidden states
    repeated `rep` times, so that the rows exceed the caches: bytes = read H once + write dH once."""
    Hr = H.repeat(rep, 1)
    n = Hr.shape[0]
    g = torch.Generator(device="cuda").manual_seed(3)
    wv = (0.02 * torch.randn(d, device="cuda", generator=g)).to(H.dtype)
    v_old = 0.1 * torch.randn(n, device="cuda", generator=g)
    ret = 0.5 * torch.randn(n, device="cuda", generator=g)
    dH = torch.empty_like(Hr)
    for _ in range(2):
        umas.umas_value_loss_fwd_bwd(Hr, wv, 0.0, None, v_old, ret, None, 0, 0.2, dH=dH)
    torch.cuda.synchronize()
    umas.profile_enable(True)
    for _ in range(iters):
        umas.umas_value_loss_fwd_bwd(Hr, wv, 0.0, None, v_old, ret, None, 0, 0.2, dH=dH)
    torch.cuda.synchronize()
    prof = umas.profile_read()
    umas.profile_enable(False)
    t = prof["k_value_rows"][0] / iters
    nbytes = 2 * n * d * H.element_size()
    return {"rows": n, "d": d, "kernel": "k_value_rows", "ms": t, "algorithmic_bytes": nbytes, "GBps": nbytes / t / 1e6,
            "frac_of_hbm_peak": nbytes / t / 1e6 / PEAK_HBM_GBPS,
            "all_kernels_ms": {k: v[0] / iters for k, v in prof.items()}}


def power_probe(umas, torch, H, W, ids, rowsel, iters=3):
    """The scoring kernel on the benchmark's operands and on all-zero operands of the same shape: the
    instruction stream is identical, so a faster run on zeros shows that the shader clock under random
    data is held down by the power limit rather than by the kernel's schedule."""
    out = {}
    for tag, h, w_ in (("random", H, W), ("zeros", torch.zeros_like(H), torch.zeros_like(W))):
        umas.umas_policy_logprobs(h, w_, ids, rowsel)
        torch.cuda.synchronize()
        umas.profile_enable(True)
        for _ in range(iters):
            umas.umas_policy_logprobs(h, w_, ids, rowsel)
        torch.cuda.synchronize()
        prof = umas.profile_read()
        umas.profile_enable(False)
        out[tag + "_ms"] = prof["k_score_tiles"][0] / iters
    flop = 2.0 * W.shape[0] * W.shape[1] * (H.shape[0] if rowsel is None else rowsel.numel())
    out["random_tflops"] = flop / out["random_ms"] / 1e9
    out["zeros_tflops"] = flop / out["zeros_ms"] / 1e9
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the CPU-oracle baseline sample (0 = skip)")
    ap.add_argument("--no-hbm", action="store_true", help="skip the batch-replicated reward/scan measurement")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline only: skip the all-rows-live update, the workspace sizes and the other configurations "
                         "(their launches would mix into the per-kernel averages of a profile of this command)")
    ap.add_argument("--config-iters", type=int, default=20, help="event-timed iterations per other configuration")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (reference for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no collectives or sharding; run with --gpus 1")

    import torch
    import workloads as wl
    import paper_2605_26646_amd as umas
    umas.load_library()          # fails loudly when the HIP library is missing
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dev = torch.device("cuda:0")

    w = wl.make_workload(1)
    spec = w.models[0]
    t = w.model_tensors(0)
    H = torch.from_numpy(t["H"]).to(dev).bfloat16()
    W = torch.from_numpy(t["W"]).to(dev).bfloat16()
    ids = torch.from_numpy(t["ids"]).to(dev)
    mask = torch.from_numpy(w.tok_mask).to(dev)
    noise = torch.from_numpy(t["noise"]).to(dev)
    kw = assign_kwargs(w, mask)

    # set-up outside the timed region: routing once to learn the selection size, old log-probs, buffers
    s = umas.umas_assign_token_rewards(**kw)
    torch.cuda.synchronize()
    n_sel = int(s.model_rowsel_off[1].item())
    rowsel = s.rowsel[:n_sel]
    logp, _, _ = umas.umas_policy_logprobs(H, W, ids, rowsel)
    logprobs_ms = statistics.median(event_times_ms(torch, lambda: umas.umas_policy_logprobs(H, W, ids, rowsel), 5, 1))
    logp_old = logp + noise * mask.float()
    ws_full = umas.ppo_workspace_bytes(n_sel, spec.d, spec.V, torch.bfloat16, w.n_roles)
    ws = torch.empty(ws_full, dtype=torch.uint8, device=dev)
    dW = torch.empty((spec.V, spec.d), dtype=torch.float32, device=dev)
    dH = torch.empty_like(H)
    logp_new = torch.empty(w.n_tokens, dtype=torch.float32, device=dev)
    stats = torch.empty((1 + w.n_roles) * 32, dtype=torch.uint8, device=dev)

    def step():
        st = umas.umas_assign_token_rewards(**kw)
        adv, _ = umas.umas_advantages(st, None, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
        umas.umas_ppo_loss_fwd_bwd(H, W, ids, st.rowsel[:n_sel], logp_old, adv, st.tok_role, w.n_roles, w.clip_eps,
                                   dW=dW, dH=dH, logp_new=logp_new, stats=stats, workspace=ws)

    # The timed region: W warm-ups, then exactly K steps between synchronisations; per-kernel events of the library and
    # one event per step on the launch stream are recorded inside it (the step's median comes from the latter).
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    umas.profile_enable(True)
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    step_ev[0].record()
    for i in range(args.steps):
        step()
        step_ev[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = umas.profile_read()
    umas.profile_enable(False)
    ms_per_step = elapsed * 1e3 / args.steps
    step_ms = [step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(args.steps)]
    loss = float(umas.read_stats(stats)["loss"][0])

    # Rows whose advantage is 0 have no gradient; the backward packs the blocks of 256 selected rows that have one
    # and does no work for the others (group-normalised outcome rewards zero out whole trajectory groups).  The
    # flop counts below follow that: scoring covers every selected row, dH and dW the rows they work on.
    st0 = umas.umas_assign_token_rewards(**kw)
    adv0, _ = umas.umas_advantages(st0, None, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
    nz = (adv0[st0.rowsel[:n_sel].long()] != 0).cpu().numpy()
    rows_with_gradient = int(nz.sum())
    rows_in_live_blocks = int(sum(min(256, n_sel - i) for i in range(0, n_sel, 256) if nz[i:i + 256].any()))

    # dominant kernel: the one with the largest summed time; a vocabulary-sized GEMM does 2*V*d flop per row
    per_launch = {k: v[0] / v[1] for k, v in prof.items()}
    per_step = {k: v[0] / args.steps for k, v in prof.items()}
    dom = max(per_step, key=per_step.get)
    launches_per_step = prof[dom][1] / args.steps
    passes = {"k_gemm_dh_dw": 2}          # GEMMs of 2*V*d flop per row inside one launch
    rows_of = {"k_gemm_dh_dw": rows_in_live_blocks}          # rows a kernel works on per step (default: all selected rows)
    rows_needed = {"k_gemm_dh_dw": rows_with_gradient}       # rows it has to work on: the algorithmic count
    rows_per_launch = rows_needed.get(dom, n_sel) / launches_per_step
    flop_per_launch = 2.0 * spec.V * spec.d * rows_per_launch * passes.get(dom, 1)
    achieved = flop_per_launch / (per_launch[dom] * 1e-3) / 1e12
    algorithmic = 2.0 * spec.V * spec.d * (n_sel + 2 * rows_with_gradient)
    gemms = [k for k in ("k_score_tiles", "k_score_keep_tiles", "k_dz_tiles", "k_gemm_dh_dw") if k in per_step]
    n_gemms = sum(passes.get(k, 1) for k in gemms)
    executed = 2.0 * spec.V * spec.d * sum(passes.get(k, 1) * rows_of.get(k, n_sel) for k in gemms)
    nominal = 6.0 * spec.V * spec.d * n_sel
    out = {
        "metric": "scored tokens/sec, PPO loss fwd+bwd (3B-shape, V=151936) + % bf16 MFMA peak",
        "value": n_sel / (ms_per_step * 1e-3), "unit": "scored tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg1 Qwen2.5-3B-shaped pipeline: d=2048 V=151936, 64 traj x 3 roles x 256 tokens",
                   "tokens": w.n_tokens, "scored_tokens": n_sel, "scored_tokens_with_gradient": rows_with_gradient,
                   "rows_in_blocks_with_gradient": rows_in_live_blocks,
                   "step": "assign_token_rewards + advantages + ppo_loss_fwd_bwd"},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": stored_traffic(dom),
                     "flop_per_launch": flop_per_launch, "ms_per_launch": per_launch[dom]},
        "step_ms_events": {"median": statistics.median(step_ms), "min": min(step_ms), "max": max(step_ms), "iterations": args.steps},
        # algorithmic: 2*V*d per scored row for the logits + 4*V*d per row that has a gradient; executed: what the
        # kernels did (whole blocks of 256 rows); nominal: 6*V*d for every scored row, gradient or not
        "whole_step": {"algorithmic_tflops": algorithmic / (ms_per_step * 1e-3) / 1e12,
                       "frac_of_bf16_peak_algorithmic": algorithmic / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                       "executed_gemm_passes": n_gemms,
                       "frac_of_bf16_peak_executed": executed / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                       "frac_of_bf16_peak_nominal_6Vd_all_rows": nominal / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "kernels_ms_per_step": per_step,
        "policy_logprobs_ms": logprobs_ms,
        "loss": loss,
    }

    if not args.no_extras:
        # the same step with every row given a gradient (advantage 0 replaced by a small number): all of 6*V*d is work
        adv_all = torch.where(adv0 == 0, torch.full_like(adv0, 1e-3), adv0)

        def step_all_live():
            st = umas.umas_assign_token_rewards(**kw)
            umas.umas_advantages(st, None, w.gamma, w.lam, w.gamma_turn, w.seg_mode)
            umas.umas_ppo_loss_fwd_bwd(H, W, ids, st.rowsel[:n_sel], logp_old, adv_all, st.tok_role, w.n_roles, w.clip_eps,
                                       dW=dW, dH=dH, logp_new=logp_new, stats=stats, workspace=ws)
        ms = event_times_ms(torch, step_all_live, args.config_iters, 2)
        med = statistics.median(ms)
        out["step_every_row_given_a_gradient"] = {
            "iterations": len(ms), "median_ms_per_step": med, "min_ms": min(ms), "max_ms": max(ms),
            "scored_tokens_per_s": n_sel / (med * 1e-3), "frac_of_bf16_peak_6Vd": nominal / (med * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}

        # the update call alone (all rows live) at three workspace sizes: the [rows, V] operand of the backward is cut
        # into chunks of as many rows as the workspace holds, at the price of one more pass over W per chunk
        ws_min = umas.ppo_workspace_bytes(n_sel, spec.d, spec.V, torch.bfloat16, w.n_roles, minimum=True)
        sizes = []
        for label, nbytes in (("minimum (256-row chunks)", ws_min), ("about 2 GB", max(ws_min, 2 << 30)), ("full (one chunk)", ws_full)):
            view = ws[:nbytes]
            ms = event_times_ms(torch, lambda: umas.umas_ppo_loss_fwd_bwd(
                H, W, ids, st0.rowsel[:n_sel], logp_old, adv_all, st0.tok_role, w.n_roles, w.clip_eps, dW=dW, dH=dH,
                logp_new=logp_new, stats=stats, workspace=view), 5 if nbytes == ws_min else 10, 1)
            # the same call on the path that recomputes the logits in the backward instead of keeping the numerators
            # (an entropy coefficient too small to change a bit of the result selects it): the trade in numbers
            if nbytes == ws_min:
                rec = None                       # minutes at 256-row chunks: left out
            else:
                rec = statistics.median(event_times_ms(torch, lambda: umas.umas_ppo_loss_fwd_bwd(
                    H, W, ids, st0.rowsel[:n_sel], logp_old, adv_all, st0.tok_role, w.n_roles, w.clip_eps, dW=dW, dH=dH,
                    logp_new=logp_new, stats=stats, workspace=view, entropy_coef=1e-30), 5, 1))
            sizes.append({"workspace": label, "bytes": int(nbytes), "median_ms": statistics.median(ms), "recomputing_path_median_ms": rec})
        out["update_call_ms_by_workspace"] = sizes
    out["power_probe"] = power_probe(umas, torch, H, W, ids, rowsel)
    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "copies": 3}
        del src, dst
    critic = None
    if not args.no_hbm:
        critic = critic_kernel(umas, torch, H, n_sel, spec.d)
    del ws, dW, dH, H, W
    torch.cuda.empty_cache()
    if not args.no_extras:
        out["other_configs"] = [config_step(umas, wl, torch, 2, args.config_iters),
                                config_step(umas, wl, torch, 3, args.config_iters),
                                config_step(umas, wl, torch, 4, args.config_iters),
                                config_step(umas, wl, torch, 4, max(5, args.config_iters // 2), fixed_rounds=3)]
    if not args.no_hbm:
        out["hbm_kernels"] = [hbm_kernels(umas, wl, torch, 4, 8192, traj_scan=True),
                              hbm_kernels(umas, wl, torch, 1, 131072, shaping=True)]
        out["critic"] = critic
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(w, t, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
