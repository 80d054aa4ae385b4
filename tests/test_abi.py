"""The C-ABI library loads, exports every declared symbol, and rejects bad arguments on the host (no GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2605_26646_amd as umas
    if not os.path.exists(umas.lib_path()):
        import __graft_entry__ as g
        g.build()
    return umas.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "umas.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(umas_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"umas_assign_token_rewards", "umas_advantages", "umas_policy_logprobs",
            "umas_ppo_loss_fwd_bwd", "umas_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layouts_match_the_header():
    from paper_2605_26646_amd import binding as b
    assert C.sizeof(b._Graph) == 4 * 4 + 8 + 7 * 8
    assert C.sizeof(b._Rewards) == 6 * 8 + 8
    assert C.sizeof(b._Streams) == 16 * 8
    assert b.STATS_DTYPE.itemsize == 32


def test_workspace_queries(lib):
    assert lib.umas_advantages_workspace_bytes(0) > 0
    small = lib.umas_ppo_loss_workspace_bytes_min(39000, 2048, 151936, 1, 3)
    full = lib.umas_ppo_loss_workspace_bytes(39000, 2048, 151936, 1, 3)
    assert 0 < small < full
    assert lib.umas_policy_logprobs_workspace_bytes(1000, 64, 512, 0) > 0


def graph(**kw):
    from paper_2605_26646_amd import binding as b
    base = dict(n_roles=2, n_models=2, role_to_model=[0, 1], traj_turn_off=[0, 2], turn_role=[0, 1],
                turn_tok_off=[0, 3, 5], turn_pred_off=None, turn_pred=None, traj_group=None)
    base.update(kw)
    keep = []

    def h(a, dt):
        if a is None:
            return None
        arr = np.ascontiguousarray(a, dtype=dt)
        keep.append(arr)
        return arr.ctypes.data

    g = b._Graph(base["n_roles"], base["n_models"], len(base["traj_turn_off"]) - 1, len(base["turn_tok_off"]) - 1,
                 int(base["turn_tok_off"][-1]), h(base["role_to_model"], np.int32), h(base["traj_turn_off"], np.int32),
                 h(base["turn_role"], np.int32), h(base["turn_tok_off"], np.int64), h(base["turn_pred_off"], np.int32),
                 h(base["turn_pred"], np.int32), h(base["traj_group"], np.int32))
    return g, keep


@pytest.mark.parametrize("kw,code,needle", [
    (dict(role_to_model=[0, 2]), -1, "role_to_model"),
    (dict(turn_role=[0, 5]), -1, "turn_role"),
    (dict(turn_tok_off=[0, 4, 3]), -1, "turn_tok_off"),
    (dict(traj_turn_off=[0, 1]), -1, "traj_turn_off"),
    (dict(n_models=9, role_to_model=[0, 1]), -2, "n_models"),
    (dict(turn_pred_off=[0, 0, 1], turn_pred=[1]), -1, "predecessor"),
    (dict(traj_group=[-1]), -1, "traj_group"),
    (dict(turn_tok_off=[0, 2 ** 31 + 5, 2 ** 31 + 9]), -2, "stream of model 0"),
    (dict(), -1, "16-byte aligned"),          # a well-formed graph: the dummy output pointers (address 1) are what is refused
])
def test_malformed_graphs_are_rejected_before_any_launch(lib, kw, code, needle):
    from paper_2605_26646_amd import binding as b
    g, keep = graph(**kw)
    r = b._Rewards(None, None, None, None, None, None, 0, 1e-6)
    s = b._Streams(*([1] * 16))          # non-NULL dummies: validation fails before they are used
    status = lib.umas_assign_token_rewards(C.addressof(g), C.addressof(r), 1, C.addressof(s), 256, 1 << 20, None)
    assert status == code
    assert needle in lib.umas_last_error().decode()


def test_bad_scalar_arguments(lib):
    assert lib.umas_policy_logprobs(256, 256, 7, 4, 8, 8, 256, None, 4, 256, 256, None, 256, 1 << 20, None) == -3
    assert lib.umas_policy_logprobs(256, 256, 1, 4, 12, 8, 256, None, 4, 256, 256, None, 256, 1 << 20, None) == -2
    assert "d % 8" in lib.umas_last_error().decode()
    # bf16 H of 4 GiB or more is refused (32-bit buffer offsets); one row less gets as far as the workspace check
    assert lib.umas_policy_logprobs(256, 256, 1, 1 << 28, 8, 8, 256, None, 1 << 28, 256, 256, None, 256, 1 << 20, None) == -2
    assert "4 GiB" in lib.umas_last_error().decode()
    assert lib.umas_policy_logprobs(256, 256, 1, (1 << 28) - 1, 8, 8, 256, None, (1 << 28) - 1, 256, 256, None, 256, 1 << 20, None) == -4
    # clip_eps outside (0,1)
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 1.5, 0.0, 0.0, 0, 0, None, 0.0, 256, None,
                                   256, 256, 256, 1 << 30, None)
    assert st == -1 and "clip_eps" in lib.umas_last_error().decode()
    # workspace too small
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 0.2, 0.0, 0.0, 0, 0, None, 0.0, 256, None,
                                   256, 256, 256, 16, None)
    assert st == -4
    # dual clip constants in (0, 1] and a negative entropy coefficient are refused
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 0.2, 0.0, 0.5, 0, 0, None, 0.0, 256, None,
                                   256, 256, 256, 1 << 30, None)
    assert st == -1 and "dual_clip" in lib.umas_last_error().decode()
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 0.2, -0.1, 0.0, 0, 0, None, 0.0, 256, None,
                                   256, 256, 256, 1 << 30, None)
    assert st == -1 and "entropy_coef" in lib.umas_last_error().decode()
    # a normaliser smaller than the call's own row count is refused
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 0.2, 0.0, 0.0, 0, 3, None, 0.0, 256, None,
                                   256, 256, 256, 1 << 30, None)
    assert st == -1 and "norm_rows" in lib.umas_last_error().decode()
    # a KL coefficient without reference log-probs, and a negative one
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 0.2, 0.0, 0.0, 0, 0, None, 0.1, 256, None,
                                   256, 256, 256, 1 << 30, None)
    assert st == -1 and "logp_ref" in lib.umas_last_error().decode()
    st = lib.umas_ppo_loss_fwd_bwd(256, 256, 0, 4, 8, 8, 256, None, 4, 256, 256, None, 0, 0.2, 0.0, 0.0, 0, 0, 256, -0.1, 256, None,
                                   256, 256, 256, 1 << 30, None)
    assert st == -1 and "kl_coef" in lib.umas_last_error().decode()
    from paper_2605_26646_amd import binding as b
    s = b._Streams(*([1] * 16))
    assert lib.umas_advantages(C.addressof(s), 10, 1, None, 1.0, 1.0, 1.0, 3, 256, 256, 256, 1 << 20, None) == -1


def test_entry_points_around_the_update_reject_bad_arguments(lib):
    """Host-side validation of the critic, shaping and ready-batch calls: every refusal happens before any launch."""
    from paper_2605_26646_amd import binding as b
    assert b.VALUE_STATS_DTYPE.itemsize == 24
    f32, i64 = C.c_float, C.c_int64
    # critic: d must be a multiple of 8 for bf16 and at most 8192; clip range positive
    lib.umas_values.restype = C.c_int
    lib.umas_values.argtypes = [C.c_void_p, C.c_void_p, f32, C.c_int, i64, C.c_int32, C.c_void_p, i64, C.c_void_p, C.c_void_p]
    assert lib.umas_values(256, 256, 0.0, 1, 4, 12, None, 4, 256, None) == -2
    assert lib.umas_values(256, 256, 0.0, 1, 4, 16384, None, 4, 256, None) == -2
    assert lib.umas_values(256, 256, 0.0, 0, 4, 8192, None, 4, 256, None) == -2          # float32: at most 4096
    assert lib.umas_values(256, 256, 0.0, 1, 4, 64, None, 3, 256, None) == -1            # NULL selection but n_sel != n_rows
    lib.umas_value_workspace_bytes.restype = C.c_size_t
    lib.umas_value_workspace_bytes.argtypes = [i64, C.c_int32, C.c_int, C.c_int32]
    assert lib.umas_value_workspace_bytes(1000, 2048, 1, 3) > 0
    lib.umas_value_loss_fwd_bwd.restype = C.c_int
    lib.umas_value_loss_fwd_bwd.argtypes = [C.c_void_p, C.c_void_p, f32, C.c_int, i64, C.c_int32, C.c_void_p, i64, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_int32, f32, C.c_int32, C.c_int32, i64, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    st = lib.umas_value_loss_fwd_bwd(256, 256, 0.0, 1, 4, 64, None, 4, 256, 256, None, 0, 0.0, 0, 0, 0, 256, None, 256, 256,
                                     None, 256, 1 << 20, None)
    assert st == -1 and "clip_eps_v" in lib.umas_last_error().decode()
    st = lib.umas_value_loss_fwd_bwd(256, 256, 0.0, 1, 4, 64, None, 4, 256, 256, None, 0, 0.2, 0, 0, 0, 256, None, 256, 256,
                                     None, 256, 16, None)
    assert st == -4
    # KL-penalised rewards: alignment and workspace
    lib.umas_kl_rewards.restype = C.c_int
    lib.umas_kl_rewards.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, i64, f32, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.umas_kl_rewards(260, 256, 256, 256, 8, 0.1, 256, 256, 256, 1 << 20, None) == -1
    assert lib.umas_kl_rewards(256, 256, 256, 256, 8, 0.1, 256, 256, 256, 0, None) == -4
    # whitening: offsets must run from 0 to n_tokens without decreasing; the per-role scope needs roles
    lib.umas_whiten_advantages.restype = C.c_int
    lib.umas_whiten_advantages.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, i64,
                                           C.c_int32, f32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    for off, code in (([0, 5], -1), ([0, 9, 8], -1)):
        a = np.array(off, np.int64)
        assert lib.umas_whiten_advantages(256, 256, 256, a.ctypes.data, len(off) - 1, 2, 8, 0, 1e-8, 256, 256, 1 << 20, None) == code
    a = np.array([0, 8], np.int64)
    assert lib.umas_whiten_advantages(256, 256, None, a.ctypes.data, 1, 2, 8, 1, 1e-8, 256, 256, 1 << 20, None) == -1
    assert lib.umas_whiten_advantages(256, 256, 256, a.ctypes.data, 1, 2, 8, 7, 1e-8, 256, 256, 1 << 20, None) == -1
    assert lib.umas_whiten_advantages(256, 256, 256, a.ctypes.data, 1, 2, 8, 0, 0.0, 256, 256, 1 << 20, None) == -1
    # ready batch: the shuffle must be a permutation, at least one minibatch
    lib.umas_ready_batch.restype = C.c_int
    lib.umas_ready_batch.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    s = b._Streams(*([256] * 16))
    tto = np.array([0, 1, 2], np.int32)
    bad = np.array([1, 1], np.int32)
    st = lib.umas_ready_batch(C.addressof(s), 1, 2, tto.ctypes.data, 2, None, bad.ctypes.data, 2, 256, 256, 256, 1 << 20, None)
    assert st == -1 and "permutation" in lib.umas_last_error().decode()
    assert lib.umas_ready_batch(C.addressof(s), 1, 2, tto.ctypes.data, 2, None, None, 0, 256, 256, 256, 1 << 20, None) == -1
    assert lib.umas_ready_batch(C.addressof(s), 1, 3, tto.ctypes.data, 2, None, None, 1, 256, 256, 256, 1 << 20, None) == -1
    lib.umas_ready_batch_packed.restype = C.c_int
    lib.umas_ready_batch_packed.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                            C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.umas_ready_batch_packed(C.addressof(s), 1, 2, tto.ctypes.data, 2, None, None, 0, 256, 256, 256, 256, 1 << 20, None) == -1
    assert "max_rows" in lib.umas_last_error().decode()
    assert lib.umas_ready_batch_packed(C.addressof(s), 1, 2, tto.ctypes.data, 2, None, None, 5, 256, 256, None, 256, 1 << 20, None) == -1


def test_benchmark_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
