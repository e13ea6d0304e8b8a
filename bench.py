#!/usr/bin/env python3
"""Benchmark of the block-wise denoising stage on one MI355X.

A step is one pass of the whole hot path over one synthetic frame block: dp_stage_forward (timestep
modulation, then for every layer LayerNorm+modulate, QKV projection, q/k RMSNorm + 3D RoPE,
self-attention over [cached K/V ; block], output projection, cross-attention, FFN) followed by
dp_cache_update (feature-cache hand-over).  Inputs, weights and the primed cache are resident in HBM
before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_FP32_TFLOPS = 157.3      # fp32 vector
PEAK_HBM_GBS = 8000.0         # HBM3E, published

# HBM-side bytes per launch of the dominant kernel from two `rocprofv3 --pmc` runs of this command (FETCH_SIZE,
# then WRITE_SIZE, each scaled by what the same counter reads for the LayerNorm dispatches, streaming kernels of
# known size); figures and commands in profiles/bench_<workload>.md.  An entry is only valid for the kernel source
# it was measured on: `src` names the source file and `sha` the first 16 hex digits of its SHA-256 at the time of
# the profile.  With any other source (or no entry) the bench prints null instead of a stale figure.
MEASURED_TRAFFIC = {
    ("wan14b_stage", "self_attn"): {"bytes": 1.5602e+09, "src": "attn_bf16.hip", "sha": "870a6262f55fc09c"},
    ("wan1p3b_stage", "self_attn"): {"bytes": 2.2954e+08, "src": "attn_bf16.hip", "sha": "870a6262f55fc09c"},
}


def measured_traffic(workload, kernel):
    import hashlib
    ent = MEASURED_TRAFFIC.get((workload, kernel))
    if not ent:
        return None
    path = os.path.join(ROOT, "paper_2505_21070_amd", "csrc", ent["src"])
    try:
        with open(path, "rb") as f:
            sha = hashlib.sha256(f.read()).hexdigest()[:16]
    except OSError:
        return None
    return ent["bytes"] if sha == ent["sha"] else None


def class_work(cfg, S, Nc):
    """Algorithmic work per launch of each kernel class: (flops, bytes).  bytes only for the HBM-bound ones."""
    D, F, Lt = cfg["dim"], cfg["ffn_dim"], cfg["text_len"]
    E = 2 if cfg["dtype"] == "bf16" else 4
    return {
        "self_attn": (4.0 * S * (S + Nc) * D, None),
        "cross_attn": (4.0 * S * Lt * D, None),
        "qkv_gemm": (2.0 * S * D * 3 * D, None),
        "oproj_gemm": (2.0 * S * D * D, None),
        "cross_q_gemm": (2.0 * S * D * D, None),
        "cross_o_gemm": (2.0 * S * D * D, None),
        "ffn1_gemm": (2.0 * S * D * F, None),
        "ffn2_gemm": (2.0 * S * F * D, None),
        "ln": (None, S * D * (4 + E)),                       # fp32 residual in, storage type out
        "cache_copy": (None, 2 * (2 * Nc * D) * E),          # K and V of the retained frames, read + write
        "norm_rope": (None, None), "modulation": (None, None), "convert": (None, None),
    }


def cpu_baseline(cfg, weights, text, x_block, budget_s=24.0):
    """The CPU oracle (its fp32 build, the plain fp32 CPU implementation) timed on a bounded sample of the same
    workload: layer 0 of the stage; keys/values for `n_kv` of the block's S tokens, the rest of the layer for
    `n_rows` sampled query rows, each attending over S + Nc keys (the keys the sample did not compute are
    synthetic, like the cache).  A small calibration run gives the oracle's rate on this host, which sizes the
    sample to the time budget; the sample's time is scaled to the whole step by algorithmic flops (keys/values
    for S tokens + the rest of the layer for S rows, times the number of layers)."""
    import numpy as np
    from oracle.stage import OracleStage, token_positions
    cores = int(os.environ.get("OMP_NUM_THREADS") or os.cpu_count())
    one = dict(cfg, n_layers=1)
    host = {"stage": {k: v.numpy() for k, v in weights["stage"].items()},
            "layers": [{k: v.numpy() for k, v in weights["layers"][0].items()}]}
    t0 = time.perf_counter()
    st = OracleStage(one, host, text.numpy(), real="f32")
    t_init = time.perf_counter() - t0
    nf, tok, D, F, Lt = cfg["block_frames"], cfg["tok_h"] * cfg["tok_w"], cfg["dim"], cfg["ffn_dim"], cfg["text_len"]
    S, Nc = nf * tok, cfg["cache_frames"] * tok
    f_kv = 2.0 * D * 2 * D                                             # K and V projections of one token
    f_row = 2.0 * D * 4 * D + 4.0 * (S + Nc) * D + 4.0 * Lt * D + 4.0 * D * F   # q, o, cross q, cross o; attention; FFN
    x = x_block.numpy()
    e0 = st.modulation(500.0)
    pos = token_positions(nf, 0, cfg["tok_h"], cfg["tok_w"])
    base = np.random.default_rng(0).standard_normal((1024, D)).astype(np.float32)

    def run(n_kv, n_rows):
        fill = Nc + S - n_kv                               # synthetic keys/values so that S + Nc keys are attended
        kv = np.tile(base, ((fill + 1023) // 1024, 1))[:fill]
        t0 = time.perf_counter()
        st.layer(0, x[:n_kv], e0, tuple(p[:n_kv] for p in pos), (kv, kv), rows=np.arange(n_rows))
        return time.perf_counter() - t0

    n_kv, n_rows = 8 * cores, 2 * cores                    # calibration: a few rows per thread
    t_cal = run(n_kv, n_rows)
    rate = (n_kv * f_kv + n_rows * f_row) / t_cal
    n_kv = int(min(S, max(n_kv, 0.5 * budget_s * rate / f_kv)))
    n_rows = int(min(n_kv, max(n_rows, 0.5 * budget_s * rate / f_row)))
    t_big = run(n_kv, n_rows)
    t_stage = t_big * S * (f_kv + f_row) / (n_kv * f_kv + n_rows * f_row) * cfg["n_layers"]
    return {"value": S / t_stage, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"fp32 build of the oracle, layer 0 of {cfg['n_layers']}: K/V for {n_kv} of {S} tokens + {n_rows} sampled "
                      f"query rows over {S + Nc} keys took {t_big:.1f} s ({t_cal:.1f} s calibration and {t_init:.1f} s text side "
                      f"before it); scaled by algorithmic flops to {S} tokens x {cfg['n_layers']} layers = {t_stage:.0f} s per step"}


def build_stage(B, cfg, weights, text, **kw):
    """The stage as a deployment holds it: on the bf16 path the weight matrices are handed over [out, in], the
    layout the GEMMs read, so the library multiplies by them in place and the device keeps its model chunk once
    (geometries whose dim or ffn_dim is no multiple of 256 take the [in, out] hand-over and the library's copies).
    Uploaded layer by layer so that the transposition never holds more than one layer twice."""
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    oi = cfg["dtype"] == "bf16" and cfg["dim"] % 256 == 0 and cfg["ffn_dim"] % 256 == 0
    fix = B.weights_out_in if oi else (lambda w: w)
    wd = fix(B.weights_to_device({"stage": weights["stage"], "layers": []}, cfg["dtype"]))
    for lw in weights["layers"]:
        wd["layers"].append(fix(B.weights_to_device({"stage": {}, "layers": [lw]}, cfg["dtype"]))["layers"][0])
    conf = B.make_config(cfg, weight_layout="out_in" if oi else "in_out", **kw)
    return conf, B.Stage(conf, wd, text.to("cuda", td).contiguous())


def cache_ablation(args):
    """Informational: the shape of the paper's feature-cache ablation (Table 4, with / without cache) on one
    stage.  Num_B = Num_C = 8 latent frames as in the paper's experiments: with the cache a pass feeds
    [B_{i-1} tail ; B_i] = 12 frames and attends to 4 cached frames; without it the pass feeds
    [B_{i-1} tail ; B_i ; B_{i+1} head] = 16 frames."""
    from paper_2505_21070_amd import binding as B
    from paper_2505_21070_amd import synth
    torch.cuda.set_device(0)
    num_b, num_c = 8, 8
    cfg, weights, text, _ = synth.make_case("wan1p3b_stage", seed=0, n_blocks=0)
    tok = cfg["tok_h"] * cfg["tok_w"]
    td = torch.bfloat16
    conf, stage = build_stage(B, cfg, weights, text, max_block_frames=num_b + num_c, max_cache_frames=num_c // 2, max_abs_frames=64)
    gen = torch.Generator().manual_seed(3)
    video = synth.round_to(torch.randn((24 * tok, cfg["dim"]), generator=gen, dtype=torch.float32), "bf16").to("cuda", td)
    half = num_c // 2
    x_prev = video[8 * tok: 20 * tok].contiguous()        # the pass of B_{i+1}: [B_i tail ; B_{i+1}], frames 8..19
    x_ext = video[0: 12 * tok].contiguous()               # [B_{i-1} tail ; B_i], frames 0..11
    x_all = video[0: 16 * tok].contiguous()               # [B_{i-1} tail ; B_i ; B_{i+1} head], frames 0..15
    out12, out16 = torch.empty_like(x_ext), torch.empty_like(x_all)

    def with_cache():
        stage.forward(x_ext, num_b + half, 0, 500.0, out=out12)

    def without_cache():
        stage.forward(x_all, num_b + num_c, 0, 500.0, out=out16)

    def timed(fn, prep):
        prep()
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    def prime():                                          # B_{i+1}'s pass leaves its first 4 frames' K/V behind
        stage.forward(x_prev, num_b + half, 8, 625.0, out=out12)
        stage.cache_update(half, half)

    ms_c = timed(with_cache, prime)
    ms_n = timed(without_cache, lambda: stage.cache_update(0, 0))
    assert torch.isfinite(out12.float()).all() and torch.isfinite(out16.float()).all()
    res = {"metric": "latent tokens/sec per DiT stage (cached block); attn+FFN TFLOP/s vs bf16 MFMA peak",
           "value": num_b * tok / (ms_c * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_c, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": "wan1p3b_ablation (informational: one pass of an 8-frame block with 8 context frames)",
                      "layers": cfg["n_layers"], "fed_tokens_with_cache": 12 * tok, "cached_tokens": 4 * tok,
                      "fed_tokens_without_cache": 16 * tok},
           "ablation": {"ms_with_cache": ms_c, "ms_without_cache": ms_n, "speedup_from_cache": ms_n / ms_c,
                        "paper_speedup_end_to_end": 182.71 / 142.62}}
    print(json.dumps(res))


def latent_step(args):
    """Informational: one block pass in latent space on one stage that holds both ends of the model:
    patch embedding -> 4 layers (+ cache hand-over) -> output head -> Euler update."""
    from paper_2505_21070_amd import binding as B
    from paper_2505_21070_amd import synth
    torch.cuda.set_device(0)
    C = 16
    cfg, weights, text, blocks = synth.make_case("wan1p3b_stage", seed=0, n_blocks=1)
    nf, nc, tok = cfg["block_frames"], cfg["cache_frames"], cfg["tok_h"] * cfg["tok_w"]
    td = torch.bfloat16
    _conf, stage = build_stage(B, cfg, weights, text, max_abs_frames=64)
    ew = synth.make_end_weights(cfg, C, 0)
    dev = {k: v.to("cuda", td).contiguous() for k, v in ew.items()}
    dev.update({k: weights["stage"][k].to("cuda", td).contiguous() for k in ("wt1", "bt1", "wt2", "bt2")})
    ends = B.Ends(cfg, dev, C, nf)
    gen = torch.Generator().manual_seed(1)
    lat = synth.make_latent(cfg, nf, C, gen).cuda()
    stage.forward(blocks[0].to("cuda", td).contiguous(), nf, nf, 625.0)
    stage.cache_update(0, nc)
    out = torch.empty((nf * tok, cfg["dim"]), dtype=td, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]

    def step(timed=False):
        if timed: ev[0].record()
        x = ends.embed(lat)
        if timed: ev[1].record()
        stage.forward(x, nf, 0, 500.0, out=out)
        stage.cache_update(0, nc)
        if timed: ev[2].record()
        v = ends.head(out, 500.0, nf)
        B.euler_step(lat, v, 0.5, 0.48)
        if timed: ev[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    step(timed=True)
    torch.cuda.synchronize()
    parts = {"embed_ms": ev[0].elapsed_time(ev[1]), "stage_ms": ev[1].elapsed_time(ev[2]), "head_euler_ms": ev[2].elapsed_time(ev[3])}
    assert torch.isfinite(lat).all()
    print(json.dumps({"metric": "latent tokens/sec per DiT stage (cached block); attn+FFN TFLOP/s vs bf16 MFMA peak",
                      "value": nf * tok / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
                      "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "wan1p3b_latent (informational: patch embedding + 4 layers + head + Euler step)",
                                 "layers": cfg["n_layers"], "block_tokens": nf * tok, "latent": [nf, 2 * cfg["tok_h"], 2 * cfg["tok_w"], C]},
                      "parts": parts}))


def long_sweep(args):
    """Informational: the long-video configuration end to end in latent space on one GPU that holds all 30 layers:
    257 latent frames as one 5-frame block + 63 blocks of 4 (the first block is the longer one, Sec. 3.3), T noise
    levels, the whole block queue from the first push to the last pop (T * 64 block passes).  Every pass is
    patch embedding -> 30 layers with the neighbour's cached K/V -> cache hand-over -> output head -> Euler
    update of the block's latent frames.  Reports sustained tokens/s over the whole run and peak device memory."""
    from paper_2505_21070_amd import binding as B
    from paper_2505_21070_amd import synth
    torch.cuda.set_device(0)
    C, frames, nf, nc, first, block_num, T = 16, 257, 4, 2, 5, 64, args.levels
    cfg, weights, text, _ = synth.make_case("wan1p3b_full", seed=0, n_blocks=0)
    tok, td = cfg["tok_h"] * cfg["tok_w"], torch.bfloat16
    torch.cuda.reset_peak_memory_stats()
    free0, _total = torch.cuda.mem_get_info()
    _conf, stage = build_stage(B, cfg, weights, text, max_block_frames=first, max_cache_frames=nc, max_abs_frames=frames + 7)
    dev = {k: v.to("cuda", td).contiguous() for k, v in synth.make_end_weights(cfg, C, 0).items()}
    dev.update({k: weights["stage"][k].to("cuda", td).contiguous() for k in ("wt1", "bt1", "wt2", "bt2")})
    ends = B.Ends(cfg, dev, C, first)
    # coordinated noise initialisation: every block's frames come from one pool of num_b + num_c/2 noise frames;
    # block 1 is one frame shorter here than the pool (257 = 5 + 63 * 4), so it takes the pool's last 5 frames
    gen = torch.Generator().manual_seed(1)
    pool = synth.make_latent(cfg, nf + nc, C, gen).cuda()
    idx = B.noise_assign(block_num, nf, 2 * nc, synth.shuffle_words((block_num - 1) * (nf - 1), 2))
    idx[0] = idx[0][-first:]
    flat = torch.tensor([i for blk in idx for i in blk], dtype=torch.int32, device="cuda")
    assert flat.numel() == frames
    sched = B.blockwise_schedule(T, block_num, nf, 2 * nc, first, 1000.0, "reverse")
    assert len(sched) == T * block_num and sched[-1]["frame0"] + sched[-1]["n_frames"] <= frames
    assert max(e["frame0"] + e["n_frames"] for e in sched) == frames
    out = torch.empty((first * tok, cfg["dim"]), dtype=td, device="cuda")

    def run():
        lat = B.noise_gather(pool, flat)                  # [257, 60, 104, 16] fp32, the video's latent frames
        for e in sched:
            n, f0, k = e["n_frames"], e["frame0"], e["level"]
            if e["cache_block"] == 0:
                stage.cache_update(0, 0)
            blk = lat[f0:f0 + n]
            y = out[:n * tok]
            stage.forward(ends.embed(blk), n, f0, e["timestep"], out=y)
            stage.cache_update(0, nc)
            B.euler_step(blk, ends.head(y, e["timestep"], n), k / T, (k - 1) / T)
        return lat

    for e in sched[:2]:                                   # warm-up: two passes
        stage.forward(ends.embed(pool[:e["n_frames"]].contiguous()), e["n_frames"], e["frame0"], e["timestep"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    lat = run()
    torch.cuda.synchronize()
    sec = time.perf_counter() - t0
    assert torch.isfinite(lat).all()
    free1, _ = torch.cuda.mem_get_info()
    tokens = sum(e["n_frames"] for e in sched) * tok
    print(json.dumps({"metric": "latent tokens/sec per DiT stage (cached block); attn+FFN TFLOP/s vs bf16 MFMA peak",
                      "value": tokens / sec, "unit": "tokens/s", "n_gpus": 1, "steps": len(sched), "warmup": 2,
                      "ms_per_step": sec * 1e3 / len(sched), "higher_is_better": True, "scaling": "weak",
                      "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"wan1p3b_long (informational: 257 latent frames, 64 blocks, T = {T} levels, "
                                             "30 layers + both ends + Euler in latent space; one step = one block pass)",
                                 "layers": cfg["n_layers"], "latent_frames": frames, "blocks": block_num, "levels": T,
                                 "block_passes": len(sched), "tokens_processed": tokens},
                      "run_seconds": sec,
                      "peak_hbm_bytes": {"torch_max_allocated": torch.cuda.max_memory_allocated(),
                                         "device_in_use_delta": free0 - free1}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="wan14b_stage",
                    help="wan14b_stage (default: the largest single-GPU stage configuration), wan1p3b_stage, or an "
                         "informational one: wan1p3b_queue, wan1p3b_long, wan1p3b_latent, wan1p3b_ablation")
    ap.add_argument("--levels", type=int, default=8, help="noise levels T of the wan1p3b_long workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="print the per-class time table to stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the stage has no CPU path", file=sys.stderr)
        sys.exit(3)
    from paper_2505_21070_amd import build as lib_build
    lib_build.ensure_built()                # loads what is built; builds only if nothing is
    if args.workload == "wan1p3b_ablation":
        return cache_ablation(args)
    if args.workload == "wan1p3b_latent":
        return latent_step(args)
    if args.workload == "wan1p3b_long":
        return long_sweep(args)
    from paper_2505_21070_amd import binding as B
    from paper_2505_21070_amd import synth

    torch.cuda.set_device(0)
    # "wan1p3b_queue": all 30 layers, a full queue of 8 blocks at timesteps 1000..125; one step = one sweep
    # of the queue tail to head (8 block passes, each reading the cache of the pass before it)
    queue = args.workload == "wan1p3b_queue"
    cfg, weights, text, blocks = synth.make_case("wan1p3b_full" if queue else args.workload, seed=0,
                                                 n_blocks=2)
    nf, nc, tok = cfg["block_frames"], cfg["cache_frames"], cfg["tok_h"] * cfg["tok_w"]
    S, Nc = nf * tok, nc * tok
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    conf, stage = build_stage(B, cfg, weights, text, max_abs_frames=64)
    x_nb, x_cur = (b.to("cuda", td).contiguous() for b in blocks[:2])
    out = torch.empty_like(x_cur)
    # prime the cache the way the queue does: the neighbour (later, noisier) block runs first and hands
    # its first cache_frames frames over
    stage.forward(x_nb, nf, nf, 625.0, out=out)
    stage.cache_update(0, nc)
    torch.cuda.synchronize()

    if queue:
        # 9 blocks initialised from the shared noise pool (coordinated noise initialisation: block 1 is the
        # whole pool of nf + nc frames); the sweep timed is diffusion step 9 of T = 8, when blocks 9..2, all
        # nf frames long, fill the queue
        gen = torch.Generator().manual_seed(1)
        pool = synth.noise_pool(cfg, nf + nc, gen).to("cuda", td).contiguous()
        idx = B.noise_assign(9, nf, 2 * nc, synth.shuffle_words(8 * (nf - 1), 2))
        xq = [B.noise_gather(pool, torch.tensor(i, dtype=torch.int32, device="cuda")).reshape(-1, cfg["dim"]) for i in idx]
        sweep = [e for e in B.blockwise_schedule(8, 9, nf, 2 * nc, nf + nc, 1000.0, "reverse") if e["step"] == 9]
        assert len(sweep) == 8 and all(e["n_frames"] == nf for e in sweep)

        def step():
            for e in sweep:
                if e["cache_block"] == 0:
                    stage.cache_update(0, 0)
                stage.forward(xq[e["block"] - 1], nf, e["frame0"], e["timestep"], out=out)
                stage.cache_update(0, nc)
    else:
        def step():
            stage.forward(x_cur, nf, 0, 500.0, out=out)
            stage.cache_update(0, nc)
    tokens_per_step = S * (8 if queue else 1)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # per-class breakdown (outside the timed region) to find the dominant kernel
    work = class_work(cfg, S, Nc)
    stage.profile_begin("all")
    nb = max(2, min(5, args.steps))
    for _ in range(nb):
        step()
    prof = stage.profile_end()
    total_ms = sum(v[0] for v in prof.values())
    dominant = max(prof, key=lambda k: prof[k][0])
    breakdown = {}
    for k, (ms, n) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
        fl, by = work[k]
        ent = {"ms_per_launch": ms / n, "share": ms / total_ms}
        if fl:
            ent["tflops"] = fl / (ms / n * 1e-3) / 1e12
        if by:
            ent["gbs"] = by / (ms / n * 1e-3) / 1e9
        breakdown[k] = ent
    if args.breakdown:
        for k, e in breakdown.items():
            print(f"  {k:14s} {e['ms_per_launch']*1e3:9.1f} us/launch  {100*e['share']:5.1f} %"
                  + (f"  {e['tflops']:8.1f} TFLOP/s" if "tflops" in e else "")
                  + (f"  {e['gbs']:8.1f} GB/s" if "gbs" in e else ""), file=sys.stderr)
    mf_classes = ("self_attn", "cross_attn", "ffn1_gemm", "ffn2_gemm")
    mf_flops = sum(work[k][0] * prof[k][1] for k in mf_classes if k in prof)
    mf_ms = sum(prof[k][0] for k in mf_classes if k in prof)
    gemm_classes = [k for k in prof if work[k][0]]
    all_flops = sum(work[k][0] * prof[k][1] for k in gemm_classes)
    all_ms = sum(prof[k][0] for k in gemm_classes)

    # timed region: K steps, HIP events only around the dominant kernel's launches
    stage.profile_begin([dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms, dom_n = stage.profile_end()[dominant]
    assert torch.isfinite(out.float()).all()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    fl, by = work[dominant]
    if fl:
        peak = PEAK_BF16_TFLOPS if cfg["dtype"] == "bf16" else PEAK_FP32_TFLOPS
        achieved = fl / (dom_ms / dom_n * 1e-3) / 1e12
        roof = {"kernel": dominant, "bound": "mfma" if cfg["dtype"] == "bf16" else "alu", "achieved": achieved,
                "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                "traffic": measured_traffic(args.workload, dominant),
                "avg_launch_ms": dom_ms / dom_n, "launches": dom_n}
    else:
        achieved = by / (dom_ms / dom_n * 1e-3) / 1e9
        roof = {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": None, "avg_launch_ms": dom_ms / dom_n, "launches": dom_n}
    res = {
        "metric": "latent tokens/sec per DiT stage (cached block); attn+FFN TFLOP/s vs bf16 MFMA peak",
        "value": tokens_per_step / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload + (" (informational: one step = one 8-block queue sweep)" if queue else ""), "layers": cfg["n_layers"], "dim": cfg["dim"], "heads": cfg["n_heads"],
                   "head_dim": cfg["head_dim"], "ffn_dim": cfg["ffn_dim"], "block_tokens": S, "cached_tokens": Nc,
                   "text_tokens": cfg["text_len"], "step": "dp_stage_forward + dp_cache_update",
                   "weight_layout": "out_in" if conf.weight_layout else "in_out", "workspace_bytes": B.workspace_bytes(conf)},
        "roofline": roof,
        "attn_ffn_tflops": mf_flops / (mf_ms * 1e-3) / 1e12 if mf_ms else None,
        "attn_ffn_frac_of_bf16_peak": mf_flops / (mf_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS if mf_ms else None,
        "all_gemm_attn_tflops": all_flops / (all_ms * 1e-3) / 1e12 if all_ms else None,
        "breakdown": breakdown,
    }
    if cfg["dtype"] == "bf16":
        # what the matrix cores sustain on this machine with nothing else running: zero vs pseudo-random operand bits
        res["mfma_issue_ceiling_tflops"] = {"zeros": B.probe_mfma_bf16("zeros"), "random": B.probe_mfma_bf16("random")}
        # what a plain streaming pass of the LayerNorm's traffic shape and size (fp32 in, bf16 out) reaches
        res["stream_copy_gbs_same_bytes_as_ln"] = B.probe_stream_f32_bf16(S * cfg["dim"])
    if not args.no_cpu_baseline and not queue:
        res["cpu_baseline"] = cpu_baseline(cfg, weights, text, blocks[1])
    print(json.dumps(res))


if __name__ == "__main__":
    main()
