"""Shared helpers of the GPU parity tests: build the HIP stage and the CPU oracle from one synthetic
case and compare them at the tolerances the build states."""
import numpy as np
import torch

from oracle.stage import OracleStage
from paper_2505_21070_amd import synth

FP32_TOL = 1e-4      # |gpu - ref| <= 1e-4 * max(1, |ref|), every element
BF16_REL_L2 = 2e-2   # ||gpu - ref||_2 / ||ref||_2


def gpu_stage(cfg, weights, text, **kw):
    from paper_2505_21070_amd import binding as B
    conf = B.make_config(cfg, **kw)
    wd = B.weights_to_device(weights, cfg["dtype"])
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    return B.Stage(conf, wd, text.to(device="cuda", dtype=td).contiguous())


def oracle_stage(cfg, weights, text):
    return OracleStage(cfg, synth.to_numpy(weights), text.numpy())


def to_dev(x, cfg):
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    return x.to(device="cuda", dtype=td).contiguous()


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def check(name, got, ref, dtype, report=None):
    """Asserts the build's tolerance; returns the error figures."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    err = np.abs(got - ref)
    max_abs = float(err.max()) if err.size else 0.0
    max_rel = float((err / np.maximum(np.abs(ref), 1e-30)).max()) if err.size else 0.0
    rel_l2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))
    if report is not None:
        report[name] = dict(max_abs=max_abs, max_rel=max_rel, rel_l2=rel_l2)
    if dtype == "f32":
        bad = err > FP32_TOL * np.maximum(1.0, np.abs(ref))
        assert not bad.any(), f"{name}: {int(bad.sum())} elements beyond 1e-4 (max_abs {max_abs:.3e}, max_rel {max_rel:.3e})"
    else:
        assert rel_l2 <= BF16_REL_L2, f"{name}: relative L2 {rel_l2:.3e} > 2e-2 (max_abs {max_abs:.3e})"
    return max_abs, max_rel, rel_l2
