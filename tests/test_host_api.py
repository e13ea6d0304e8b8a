"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, and its host-side
entry points (schedule, bubble ratio, argument validation) behave.  No kernel runs here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle.schedule import blockwise_schedule as oracle_schedule
from oracle.schedule import bubble_ratio_reverse, bubble_ratio_sequential

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    lib = os.path.join(ROOT, "paper_2505_21070_amd", "libdualparal.so")
    if not os.path.exists(lib):
        from paper_2505_21070_amd import build
        build.build()
    from paper_2505_21070_amd import binding
    return binding


def test_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "dualparal.h")).read()
    names = set(re.findall(r"\b(dp_[a-z_]+)\s*\(", header))
    assert {"dp_stage_init", "dp_cache_update", "dp_stage_forward", "dp_blockwise_schedule"} <= names
    for n in sorted(names):
        assert hasattr(B._lib, n), n


@pytest.mark.parametrize("args", [(8, 8, 4, 4, 0), (50, 4, 8, 8, 0), (4, 3, 4, 2, 5), (3, 1, 4, 4, 0), (5, 7, 4, 0, 0)])
@pytest.mark.parametrize("order", ["reverse", "sequential"])
@pytest.mark.parametrize("variant", ["block", "extended", "nocache"])
def test_schedule_matches_oracle(B, args, order, variant):
    got = B.blockwise_schedule(*args, 1000.0, order, variant)
    ref = oracle_schedule(args[0], args[1], args[2], args[3], args[4] or None, 1000.0, order, variant)
    assert len(got) == len(ref) == args[0] * args[1]
    for g, r in zip(got, ref):
        for k, v in r.items():
            assert g[k] == (np.float32(v) if k == "timestep" else v), (k, g, r)


def test_schedule_capacity_and_bad_input(B):
    cfg = B.SchedConfig(4, 3, 4, 4, 0, 0, 1000.0)
    n = C.c_int64()
    arr = (B.SchedEntry * 5)()
    assert B._lib.dp_blockwise_schedule(C.byref(cfg), arr, 5, C.byref(n)) == B.DP_ENOMEM and n.value == 12
    assert "capacity" in B.last_error()
    bad = B.SchedConfig(0, 3, 4, 4, 0, 0, 1000.0)
    assert B._lib.dp_blockwise_schedule(C.byref(bad), arr, 5, C.byref(n)) == B.DP_EINVAL
    bad = B.SchedConfig(4, 3, 4, 4, 0, 0, 1000.0, 3)                       # unknown input variant
    assert B._lib.dp_blockwise_schedule(C.byref(bad), arr, 5, C.byref(n)) == B.DP_EINVAL
    assert B._lib.dp_blockwise_schedule(None, arr, 5, C.byref(n)) == B.DP_EINVAL
    bad = B.SchedConfig(4, 3, 2, 6, 0, 0, 1000.0)                          # num_c / 2 > num_b: outside Sec. 3.2
    assert B._lib.dp_blockwise_schedule(C.byref(bad), arr, 5, C.byref(n)) == B.DP_EINVAL
    assert "num_c" in B.last_error()
    with pytest.raises(AssertionError):
        oracle_schedule(4, 3, 2, 6)


def test_bubble_ratio_matches_oracle_and_paper(B):
    assert B.bubble_ratio(4, 50, 4) == pytest.approx(11 / 211)
    for N, T, Bn in [(4, 50, 4), (8, 50, 64), (4, 50, 3), (2, 8, 8)]:
        assert B.bubble_ratio(N, T, Bn) == pytest.approx(bubble_ratio_reverse(N, T, Bn))
        assert B.bubble_ratio(N, T, Bn, "sequential") == pytest.approx(bubble_ratio_sequential(N, T, Bn))
    assert B.bubble_ratio(0, 50, 4) == -1.0


def test_config_validation_without_gpu(B):
    from paper_2505_21070_amd import synth
    good = B.make_config(synth.stage_config("wan1p3b_stage"))
    nbytes = B.workspace_bytes(good)
    assert 1 << 28 < nbytes < 1 << 32                     # a few hundred MB .. GBs for 4 Wan-1.3B layers
    for field, value in [("head_dim", 96), ("n_heads", 11), ("dtype", 7), ("freq_dim", 255), ("tok_w", 51)]:
        c = B.make_config(synth.stage_config("wan1p3b_stage"))
        setattr(c, field, value)
        assert B.workspace_bytes(c) == 0, field
        assert B.last_error()
    h = C.c_void_p(1)
    assert B._lib.dp_stage_init(C.byref(good), None, None, None, 0, None, C.byref(h)) == B.DP_EINVAL
    assert not h.value
    assert B._lib.dp_stage_forward(None, None, None, 1, 0, 0.0, None) == B.DP_EINVAL
    assert B._lib.dp_cache_update(None, 0, 1, None) == B.DP_EINVAL
    B._lib.dp_stage_free(None)


@pytest.mark.parametrize("block_num,num_b,num_c", [(8, 4, 4), (5, 4, 2), (6, 8, 8), (7, 3, 6), (4, 5, 0), (4, 1, 2), (1, 4, 4)])
@pytest.mark.parametrize("seed", [0, 3])
def test_noise_assignment_matches_oracle(B, block_num, num_b, num_c, seed):
    from oracle.noise import noise_assignment
    from paper_2505_21070_amd import synth
    words = synth.shuffle_words((block_num - 1) * (num_b - 1) + 2, seed)
    assert B.noise_assign(block_num, num_b, num_c, words) == noise_assignment(block_num, num_b, num_c, words)


def test_noise_assignment_bad_input(B):
    import ctypes as C
    cfg = B.NoiseConfig(3, 4, 4)
    n = C.c_int64()
    words = (C.c_uint32 * 6)(*range(6))
    assert B._lib.dp_noise_assign(C.byref(cfg), words, 6, None, 0, C.byref(n)) == B.DP_ENOMEM and n.value == 6 + 2 * 4
    assert B._lib.dp_noise_assign(C.byref(cfg), words, 5, None, 0, C.byref(n)) == B.DP_EINVAL      # too few words
    assert B._lib.dp_noise_assign(None, words, 6, None, 0, C.byref(n)) == B.DP_EINVAL
    bad = B.NoiseConfig(0, 4, 4)
    assert B._lib.dp_noise_assign(C.byref(bad), words, 6, None, 0, C.byref(n)) == B.DP_EINVAL
    assert b"dp_noise_assign" in B._lib.dp_last_error()
    bad = B.NoiseConfig(3, 2, 6)                                           # num_c / 2 > num_b: outside Sec. 3.3
    assert B._lib.dp_noise_assign(C.byref(bad), words, 6, None, 0, C.byref(n)) == B.DP_EINVAL
    assert b"num_c" in B._lib.dp_last_error()
    from oracle.noise import noise_assignment
    with pytest.raises(AssertionError):
        noise_assignment(3, 2, 6, list(range(6)))


def test_pipeline_simulation_matches_oracle(B):
    import ctypes as C
    from oracle.pipeline import simulate_pipeline
    for order in ("reverse", "sequential"):
        for N, T, Bn in [(1, 3, 2), (2, 2, 2), (4, 50, 4), (4, 50, 3), (4, 50, 8), (8, 50, 64), (5, 3, 7), (3, 9, 1)]:
            r = simulate_pipeline(N, T, Bn, order)
            assert B.pipeline_simulate(N, T, Bn, order) == (r["makespan"], r["bubble_per_device"])
    mk, bub = C.c_int64(), C.c_int64()
    assert B._lib.dp_pipeline_simulate(0, 5, 5, 0, C.byref(mk), C.byref(bub)) == B.DP_EINVAL
    assert B._lib.dp_pipeline_simulate(2, 5, 5, 7, C.byref(mk), C.byref(bub)) == B.DP_EINVAL
    assert B._lib.dp_pipeline_simulate(2, 5, 5, 0, None, C.byref(bub)) == B.DP_EINVAL


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_product_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing under the package imports, loads or runs it, and bench.py only
    does so inside its cpu_baseline leg."""
    pkg = os.path.join(ROOT, "paper_2505_21070_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", os.path.join(dirpath, f)
    synth_src = open(os.path.join(pkg, "synth.py")).read()
    assert "import oracle" not in synth_src and "from oracle" not in synth_src
    bench = open(os.path.join(ROOT, "bench.py")).read()
    head, _, rest = bench.partition("def cpu_baseline(")
    body, _, tail = rest.partition("\ndef ")
    assert "oracle" in body                                   # the baseline leg is where it is used ...
    assert "from oracle" not in head and "import oracle" not in head
    assert "from oracle" not in tail and "import oracle" not in tail      # ... and nowhere else


@pytest.mark.parametrize("name", ["wan1p3b_stage", "wan1p3b_full", "wan14b_stage", "tiny"])
def test_key_value_memory_is_the_papers_bound(B, name):
    """Table 1 / appendix memory analysis: a device's K/V memory is (Num_B + Num_C) * KV per layer, KV = one
    frame's keys and values.  The library's per-layer key/value buffer (cached range + current block) is exactly
    that many frame positions plus at most 127 positions of alignment padding, and the workspace grows by at
    least that much per layer."""
    from paper_2505_21070_amd import synth
    cfg = synth.stage_config(name)
    conf = B.make_config(cfg)
    num_b, num_c = cfg["block_frames"], 2 * cfg["cache_frames"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    frame_kv = 2 * cfg["tok_h"] * cfg["tok_w"] * cfg["dim"] * esz          # keys + values of one frame, one layer
    bound = (num_b + num_c) * frame_kv
    got = B.kv_bytes_per_layer(conf)
    assert bound <= got <= bound + 2 * 127 * cfg["dim"] * esz, (got, bound)
    more = B.make_config(dict(cfg, n_layers=cfg["n_layers"] + 1))
    assert B.workspace_bytes(more) - B.workspace_bytes(conf) >= got


def test_out_in_weight_layout_validation_and_workspace(B):
    """DP_WEIGHTS_OUT_IN: bf16 only, dim and ffn_dim multiples of 256 (no padding rows exist in the caller's
    memory); the workspace then holds no weight matrix: with it, a device keeps its model chunk once (Sec. 2,
    Table 1) and the per-layer growth of the workspace is K/V, text keys/values and vectors only."""
    from paper_2505_21070_amd import synth
    cfg = synth.stage_config("wan1p3b_stage")
    io, oi = B.make_config(cfg), B.make_config(cfg, weight_layout="out_in")
    D, F, L = cfg["dim"], cfg["ffn_dim"], cfg["n_layers"]
    matrices = L * (6 * D * D + 2 * D * F) * 2
    saved = B.workspace_bytes(io) - B.workspace_bytes(oi)
    assert B.workspace_bytes(oi) > 0
    assert matrices <= saved <= matrices + (1 << 20) + max(D, cfg["text_dim"]) * D * 2       # + the transposition buffer
    per_layer = B.workspace_bytes(B.make_config(dict(cfg, n_layers=L + 1), weight_layout="out_in")) - B.workspace_bytes(oi)
    assert per_layer < B.kv_bytes_per_layer(oi) + 4 * 512 * D * 2 + (1 << 20)                # K/V + text K/V (+ gains)
    for bad in (dict(cfg, dtype="f32"), dict(cfg, ffn_dim=8960 + 64), synth.stage_config("small_bf16"),
                synth.stage_config("tile192_bf16")):
        assert B.workspace_bytes(B.make_config(bad, weight_layout="out_in")) == 0
        assert B.last_error()
    c = B.make_config(cfg)
    c.weight_layout = 2
    assert B.workspace_bytes(c) == 0 and "weight_layout" in B.last_error()


def test_schedule_random_parameter_sweep_matches_oracle(B):
    """Integer work, bit-exact: 300 seeded random queues (T, block count, Num_B, Num_C <= 2 Num_B, optional longer
    first block; both orders, all three input variants) against the oracle's schedule (Sec. 3.1 - 3.3)."""
    rng = np.random.default_rng(20250521)
    for _ in range(300):
        T, nb = int(rng.integers(1, 13)), int(rng.integers(1, 10))
        num_b = int(rng.integers(1, 9))
        num_c = 2 * int(rng.integers(0, num_b + 1))
        first = int(rng.integers(num_b, num_b + 4)) if rng.random() < 0.3 else 0
        order = ("reverse", "sequential")[int(rng.integers(2))]
        variant = ("block", "extended", "nocache")[int(rng.integers(3))]
        got = B.blockwise_schedule(T, nb, num_b, num_c, first, 1000.0, order, variant)
        ref = oracle_schedule(T, nb, num_b, num_c, first or None, 1000.0, order, variant)
        assert len(got) == len(ref) == T * nb
        for g, r in zip(got, ref):
            for k, v in r.items():
                assert g[k] == (np.float32(v) if k == "timestep" else v), ((T, nb, num_b, num_c, first, order, variant), k, g, r)


def test_noise_assignment_random_parameter_sweep_matches_oracle(B):
    """300 seeded random (block count, Num_B, Num_C <= 2 Num_B) cases of the coordinated noise initialisation
    (Sec. 3.3) against the oracle, index for index."""
    from oracle.noise import noise_assignment
    from paper_2505_21070_amd import synth
    rng = np.random.default_rng(33)
    for i in range(300):
        nb, num_b = int(rng.integers(1, 12)), int(rng.integers(1, 10))
        num_c = 2 * int(rng.integers(0, num_b + 1))
        words = synth.shuffle_words((nb - 1) * max(num_b - 1, 0) + 2 * num_b + 2, 1000 + i)
        assert B.noise_assign(nb, num_b, num_c, words) == noise_assignment(nb, num_b, num_c, words), (nb, num_b, num_c)
