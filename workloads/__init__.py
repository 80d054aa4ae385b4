"""Seeded synthetic workloads shaped like the paper's four workflow families.

This module only *draws inputs*: trajectory graphs (roles, turns, the
agent-to-model map), masks, reward scalars, critic values, hidden states,
LM-head weights, token ids and old-log-prob noise.  It holds none of the
method's arithmetic (no reward composition, routing, scans, scoring or loss),
so both the CPU oracle's tests and the GPU path's tests may feed from it.

Shapes follow the paper's workflow table (Section "Workflows and Rewards"):
a retrieve/filter/answer pipeline (Workflow B), an iterative search loop with a
variable number of turns (Workflow C), partial parameter sharing over five roles
(Section "Agent--LLM Mapping") and the reflective coder/critic loop with early
termination (Workflow D).  Every draw comes from numpy's PCG64 streams seeded
with ``26646000 + cfg`` (graph-level data) and child streams for the per-model
tensors, so a workload is a pure function of (cfg, overrides).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 26646000

PLACE_LAST = 0
PLACE_ALL = 1
SEG_TURN = 0
SEG_TRAJ = 1


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), keep float32 storage."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


@dataclass
class ModelSpec:
    d: int
    V: int
    dtype: str  # "f32" or "bf16"


@dataclass
class Workload:
    name: str
    cfg: int
    seed: int
    # graph (thin, host side)
    n_roles: int
    n_models: int
    n_traj: int
    n_turns: int
    n_tokens: int
    role_to_model: np.ndarray      # int32 [n_roles]
    traj_turn_off: np.ndarray      # int32 [n_traj+1]
    turn_role: np.ndarray          # int32 [n_turns]
    turn_tok_off: np.ndarray       # int64 [n_turns+1]
    turn_pred_off: np.ndarray      # int32 [n_turns+1]
    turn_pred: np.ndarray          # int32 [n_pred]
    traj_group: Optional[np.ndarray]   # int32 [n_traj] or None
    # rewards (thin)
    role_reward: Optional[np.ndarray]  # float32 [n_traj*n_roles]
    turn_reward: Optional[np.ndarray]  # float32 [n_turns]
    traj_reward: Optional[np.ndarray]  # float32 [n_traj]
    w_role: Optional[np.ndarray]
    w_turn: Optional[np.ndarray]
    w_traj: Optional[np.ndarray]
    place_mode: int
    norm_eps: float
    # token-level inputs
    tok_mask: np.ndarray           # uint8 [n_tokens], global token order
    value: Optional[np.ndarray]    # float32 [n_tokens], model-local order, or None
    # scan and loss parameters
    gamma: float
    lam: float
    gamma_turn: float
    seg_mode: int
    clip_eps: float
    noise_std: float
    # per model
    models: List[ModelSpec] = field(default_factory=list)
    model_ntok: List[int] = field(default_factory=list)

    def model_tensors(self, m: int, rows: Optional[int] = None) -> dict:
        """Hidden states H [n,d], LM-head weights W [V,d], token ids and log-prob noise of model m.

        H rows are N(0,1) scaled to unit RMS in float32, W is N(0, std 0.02); both are then
        rounded to the model's dtype (kept in float32 storage).  Token ids follow a
        truncated Zipf(1.1) law over [0, V); noise is N(0, noise_std).  ``rows`` limits
        the stream to its first rows (an N-truncated replica with the same W).
        """
        spec = self.models[m]
        n = self.model_ntok[m] if rows is None else min(rows, self.model_ntok[m])
        rng_i = np.random.default_rng([self.seed, 3000 + m])
        rng_n = np.random.default_rng([self.seed, 4000 + m])
        bf16 = spec.dtype == "bf16"

        def h_block(out, blk, r0, r1):
            g = np.random.default_rng([self.seed, 1000 + m, blk])
            x = g.standard_normal((r1 - r0, spec.d), dtype=np.float32)
            rms = np.sqrt(np.mean(x * x, axis=1, dtype=np.float32), dtype=np.float32)
            x /= rms[:, None]
            out[r0:r1] = round_to_bf16(x) if bf16 else x

        def w_block(out, blk, r0, r1):
            g = np.random.default_rng([self.seed, 2000 + m, blk])
            x = g.standard_normal((r1 - r0, spec.d), dtype=np.float32)
            x *= np.float32(0.02)
            out[r0:r1] = round_to_bf16(x) if bf16 else x

        H = _fill_blocks(n, spec.d, h_block)
        W = _fill_blocks(spec.V, spec.d, w_block)
        k = np.arange(1, spec.V + 1, dtype=np.float64)
        cdf = np.cumsum(k ** -1.1)
        cdf /= cdf[-1]
        ids = np.searchsorted(cdf, rng_i.random(n), side="left")
        ids = np.minimum(ids, spec.V - 1).astype(np.int32)
        noise = (rng_n.standard_normal(n) * self.noise_std).astype(np.float32)
        return {"H": H, "W": W, "ids": ids, "noise": noise}

    def critic_tensors(self, m: int) -> dict:
        """Inputs of model m's critic and of the steps around the policy update, from streams of their own:
        value-head weights w ~ N(0, std 0.02) in the model's dtype and a bias, noise for the old value
        estimates N(0, 0.1), reference log-prob offsets N(0, 0.1) and a second LM head W_ref = W + N(0, 0.002)
        is left to the caller (it only needs another seed offset)."""
        spec = self.models[m]
        n = self.model_ntok[m]
        g = np.random.default_rng([self.seed, 7000 + m])
        w = (g.standard_normal(spec.d) * 0.02).astype(np.float32)
        if spec.dtype == "bf16":
            w = round_to_bf16(w)
        return {"w": w, "bias": np.float32(0.05), "v_noise": (g.standard_normal(n) * 0.1).astype(np.float32),
                "ref_noise": (g.standard_normal(n) * 0.1).astype(np.float32)}


def _fill_blocks(n_rows: int, n_cols: int, fill) -> np.ndarray:
    """Float32 [n_rows, n_cols] filled block by block; every block of rows draws from a stream of
    its own, so the result does not depend on how many threads fill it."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    out = np.empty((n_rows, n_cols), dtype=np.float32)
    step = max(1, (1 << 22) // max(n_cols, 1))
    jobs = [(b, r0, min(n_rows, r0 + step)) for b, r0 in enumerate(range(0, n_rows, step))]
    workers = max(1, min(16, os.cpu_count() or 1, len(jobs)))
    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(lambda j: fill(out, *j), jobs))
    return out


def _chain_preds(traj_turn_off: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Predecessor CSR of a chain: every turn but the first of a trajectory points at the one before."""
    n_turns = int(traj_turn_off[-1])
    is_first = np.zeros(n_turns, dtype=bool)
    is_first[traj_turn_off[:-1][traj_turn_off[:-1] < n_turns]] = True
    cnt = (~is_first).astype(np.int32)
    off = np.zeros(n_turns + 1, dtype=np.int32)
    np.cumsum(cnt, out=off[1:])
    pred = (np.nonzero(~is_first)[0] - 1).astype(np.int32)
    return off, pred


def _alternating_mask(rng, n_turns: int, length: int, mean_valid: float, mean_masked: float) -> np.ndarray:
    """Per turn: runs of valid tokens (geometric, mean mean_valid) alternate with masked runs, valid first."""
    mask = np.zeros((n_turns, length), dtype=np.uint8)
    for u in range(n_turns):
        pos, valid = 0, True
        while pos < length:
            run = int(rng.geometric(1.0 / (mean_valid if valid else mean_masked)))
            if valid:
                mask[u, pos:pos + run] = 1
            pos += run
            valid = not valid
    return mask.reshape(-1)


def make_workload(cfg: int, *, n_traj: Optional[int] = None, tokens_per_turn: Optional[int] = None,
                  models: Optional[Sequence[Tuple[int, int, str]]] = None,
                  noise_std: float = 0.05, seed_offset: int = 0, fixed_rounds: Optional[int] = None) -> Workload:
    """Build workload ``cfg`` (0..4).  Overrides shrink or replicate it while keeping its structure.

    n_traj           number of trajectories (default: the configuration's own)
    tokens_per_turn  scales every turn length so the base turn has this many tokens
    models           list of (d, V, dtype) replacing the configuration's model shapes
    noise_std        std of the old-log-prob noise (0.05 nominal, 0.25 for the clip-stress variant)
    fixed_rounds     configuration 4 only: every trajectory runs this many coder -> critic rounds (no early
                     termination; 3 gives the 16 x 3 x 5120 = 245 760 tokens of the configuration read literally)
    """
    seed = BASE_SEED + cfg + 1000 * seed_offset
    rng = np.random.default_rng(seed)
    gamma_turn, seg_mode, clip_eps, norm_eps = 1.0, SEG_TURN, 0.2, 1e-6
    traj_group = role_reward = turn_reward = traj_reward = None
    value_std = 0.1

    if cfg == 0:
        B = n_traj or 4
        L = tokens_per_turn or 32
        roles_per_traj = [0, 1, 2, 0, 1, 2]
        turn_role = np.tile(np.array(roles_per_traj, np.int32), B)
        traj_turn_off = (np.arange(B + 1) * 6).astype(np.int32)
        turn_len = np.full(6 * B, L, np.int64)
        n_roles, phi = 3, [0, 0, 0]
        mdl = [(64, 512, "f32")]
        gamma, lam = 1.0, 0.95
        name = "cfg0_tiny_fp32"
    elif cfg == 1:
        B = n_traj or 64
        L = tokens_per_turn or 256
        turn_role = np.tile(np.array([0, 1, 2], np.int32), B)
        traj_turn_off = (np.arange(B + 1) * 3).astype(np.int32)
        turn_len = np.full(3 * B, L, np.int64)
        n_roles, phi = 3, [0, 0, 0]
        mdl = [(2048, 151936, "bf16")]
        gamma, lam = 1.0, 1.0
        value_std = None
        traj_group = (np.arange(B) // 8).astype(np.int32)
        name = "cfg1_qwen3b_pipeline"
    elif cfg == 2:
        B = n_traj or 32
        L = tokens_per_turn or 384
        n_t = rng.integers(2, 7, size=B)
        cyc = [0, 1, 2, 1, 2, 1]
        turn_role = np.concatenate([np.array(cyc[:t], np.int32) for t in n_t])
        traj_turn_off = np.concatenate([[0], np.cumsum(n_t)]).astype(np.int32)
        turn_len = np.full(int(n_t.sum()), L, np.int64)
        n_roles, phi = 3, [0, 0, 0]
        mdl = [(2048, 151936, "bf16")]
        gamma, lam = 0.99, 0.95
        name = "cfg2_iterative_search"
    elif cfg == 3:
        B = n_traj or 48
        L = tokens_per_turn or 512
        turn_role = np.tile(np.arange(5, dtype=np.int32), B)
        traj_turn_off = (np.arange(B + 1) * 5).astype(np.int32)
        turn_len = np.full(5 * B, L, np.int64)
        n_roles, phi = 5, [0, 0, 1, 0, 1]
        mdl = [(2048, 151936, "bf16"), (3584, 152064, "bf16")]
        gamma, lam = 1.0, 0.95
        name = "cfg3_partial_sharing"
    elif cfg == 4:
        B = n_traj or 16
        Lc = tokens_per_turn or 4096
        Lr = max(1, Lc // 4)
        rounds = np.array([[1, 2, 3, 2][b % 4] if fixed_rounds is None else fixed_rounds for b in range(B)])
        turn_role = np.concatenate([np.tile(np.array([0, 1], np.int32), r) for r in rounds])
        traj_turn_off = np.concatenate([[0], np.cumsum(2 * rounds)]).astype(np.int32)
        turn_len = np.where(turn_role == 0, Lc, Lr).astype(np.int64)
        n_roles, phi = 2, [0, 0]
        mdl = [(3584, 152064, "bf16")]
        gamma, lam = 1.0, 0.95
        name = "cfg4_reflective_code" if fixed_rounds is None else f"cfg4_reflective_code_{fixed_rounds}_rounds"
    else:
        raise ValueError("cfg must be 0..4")

    if models is not None:
        mdl = list(models)
    n_models = max(phi) + 1
    if len(mdl) != n_models:
        raise ValueError("need one model shape per physical model")
    n_turns = int(turn_role.shape[0])
    turn_tok_off = np.concatenate([[0], np.cumsum(turn_len)]).astype(np.int64)
    n_tokens = int(turn_tok_off[-1])
    turn_pred_off, turn_pred = _chain_preds(traj_turn_off)
    turn_traj = np.repeat(np.arange(B), np.diff(traj_turn_off))

    # masks (global token order)
    if cfg == 1:
        L = int(turn_len[0])
        lo = max(1, int(round(0.6 * L)))
        valid_len = rng.integers(lo, L + 1, size=n_turns)
        tok_mask = (np.arange(L)[None, :] < valid_len[:, None]).astype(np.uint8).reshape(-1)
    elif cfg == 2:
        tok_mask = _alternating_mask(rng, n_turns, int(turn_len[0]), 56.0, 24.0)
    else:
        tok_mask = np.ones(n_tokens, np.uint8)

    # rewards
    if cfg in (0, 3):
        traj_reward = (rng.random(B) < 0.3).astype(np.float32)
        role_reward = (rng.random(B * n_roles) < 0.5).astype(np.float32)
    elif cfg == 1:
        traj_reward = (rng.random(B) < 0.4).astype(np.float32)
    elif cfg == 2:
        turn_reward = rng.uniform(-0.25, 0.25, size=n_turns).astype(np.float32)
        traj_reward = rng.uniform(0.0, 1.0, size=B).astype(np.float32)
    elif cfg == 4:
        traj_reward = (rng.random(B) < 0.15).astype(np.float32)
        turn_reward = np.where(turn_role == 1, rng.uniform(0.0, 1.0, size=n_turns), 0.0).astype(np.float32)

    value = None
    if value_std is not None:
        value = (rng.standard_normal(n_tokens) * value_std).astype(np.float32)

    phi_arr = np.array(phi, np.int32)
    turn_model = phi_arr[turn_role]
    model_ntok = [int(turn_len[turn_model == m].sum()) for m in range(n_models)]
    del turn_traj

    return Workload(
        name=name, cfg=cfg, seed=seed, n_roles=n_roles, n_models=n_models, n_traj=B, n_turns=n_turns,
        n_tokens=n_tokens, role_to_model=phi_arr, traj_turn_off=traj_turn_off, turn_role=turn_role,
        turn_tok_off=turn_tok_off, turn_pred_off=turn_pred_off, turn_pred=turn_pred, traj_group=traj_group,
        role_reward=role_reward, turn_reward=turn_reward, traj_reward=traj_reward,
        w_role=None, w_turn=None, w_traj=None, place_mode=PLACE_LAST, norm_eps=norm_eps,
        tok_mask=tok_mask, value=value, gamma=gamma, lam=lam, gamma_turn=gamma_turn, seg_mode=seg_mode,
        clip_eps=clip_eps, noise_std=noise_std,
        models=[ModelSpec(int(d), int(V), str(t)) for d, V, t in mdl], model_ntok=model_ntok)


def random_graph(seed: int):
    """A seeded random workflow graph for robustness tests: 1-39 trajectories of 0-6 turns, 1-5 roles on 1-3 models,
    turn lengths from 0 to 9000 tokens around the tile edges, mask densities from none to all, any subset of the three
    reward levels and their weights, normalisation groups of 1-4.  Returns (workload, dict of scan and placement
    parameters).  The model tensors of the returned workload are not meant to be used."""
    rng = np.random.default_rng(9000 + seed)
    w = make_workload(0)
    B, R, K = int(rng.integers(1, 40)), int(rng.integers(1, 6)), int(rng.integers(1, 4))
    turns = [int(rng.integers(0, 7)) for _ in range(B)]
    U = sum(turns)
    big = rng.random() < 0.3
    lens = np.array([int(rng.choice([0, 1, 2, 5, 63, 64, 65, 300, 2049 if big else 17, 9000 if big else 30])) for _ in range(U)],
                    np.int64)
    w.n_traj, w.n_turns, w.n_roles, w.n_models = B, U, R, K
    w.traj_turn_off = np.concatenate([[0], np.cumsum(turns)]).astype(np.int32)
    w.turn_role = rng.integers(0, R, size=U).astype(np.int32)
    w.role_to_model = rng.integers(0, K, size=R).astype(np.int32)
    w.turn_tok_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    w.n_tokens = int(w.turn_tok_off[-1])
    w.turn_pred_off, w.turn_pred = None, None
    w.tok_mask = (rng.random(w.n_tokens) < float(rng.choice([0.0, 0.3, 0.9, 1.0]))).astype(np.uint8)
    w.traj_reward = rng.normal(size=B).astype(np.float32) if rng.random() < 0.8 else None
    grouped = w.traj_reward is not None and rng.random() < 0.5
    w.traj_group = (np.arange(B) // int(rng.integers(1, 5))).astype(np.int32) if grouped else None
    w.role_reward = rng.normal(size=B * R).astype(np.float32) if rng.random() < 0.6 else None
    w.turn_reward = rng.normal(size=U).astype(np.float32) if rng.random() < 0.6 else None
    w.w_role = rng.random(R).astype(np.float32) if rng.random() < 0.5 else None
    w.w_turn = rng.random(R).astype(np.float32) if rng.random() < 0.5 else None
    w.w_traj = rng.random(R).astype(np.float32) if rng.random() < 0.5 else None
    w.value = rng.normal(size=w.n_tokens).astype(np.float32) if rng.random() < 0.6 else None
    kw = dict(seg_mode=int(rng.choice([SEG_TURN, SEG_TRAJ])), gamma_turn=float(rng.choice([1.0, 0.8])),
              place_mode=int(rng.choice([PLACE_LAST, PLACE_ALL])), gamma=float(rng.choice([1.0, 0.97])),
              lam=float(rng.choice([1.0, 0.9])))
    return w, kw
