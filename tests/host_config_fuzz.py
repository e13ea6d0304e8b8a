"""Child process of test_host_ubsan_configs.py: calls dp_stage_workspace_bytes and dp_ends_workspace_bytes of a
library whose host code was built with trapping UndefinedBehaviorSanitizer checks, over configurations with
extreme field values.  Every call must return (0 with an error, or a size); an overflow, a bad shift or an
exception ends the process with a signal.  usage: host_config_fuzz.py <path to the .so>"""
import ctypes as C
import random
import sys

lib = C.CDLL(sys.argv[1])
I32 = C.c_int32


class StageConfig(C.Structure):
    _fields_ = [(n, I32) for n in ("n_layers", "dim", "n_heads", "head_dim", "ffn_dim", "text_len", "text_dim",
                                   "tok_h", "tok_w", "max_block_frames", "max_cache_frames", "max_abs_frames",
                                   "dtype", "freq_dim")] + \
               [("rope_theta", C.c_float), ("eps", C.c_float), ("debug_taps", I32), ("weight_layout", I32)]


class EndsConfig(C.Structure):
    _fields_ = [(n, I32) for n in ("dim", "tok_h", "tok_w", "channels", "max_frames", "dtype", "freq_dim")] + \
               [("eps", C.c_float)]


lib.dp_stage_workspace_bytes.restype = C.c_size_t
lib.dp_stage_workspace_bytes.argtypes = [C.POINTER(StageConfig)]
lib.dp_ends_workspace_bytes.restype = C.c_size_t
lib.dp_ends_workspace_bytes.argtypes = [C.POINTER(EndsConfig)]

base = dict(n_layers=4, dim=1536, n_heads=12, head_dim=128, ffn_dim=8960, text_len=512, text_dim=4096, tok_h=30,
            tok_w=52, max_block_frames=4, max_cache_frames=2, max_abs_frames=300, dtype=1, freq_dim=256,
            rope_theta=1e4, eps=1e-6, debug_taps=0)
IMAX = 2 ** 31 - 1
wild = [-IMAX - 1, -1, 0, 1, 8, 64, 4096, 2 ** 20, 2 ** 24, 2 ** 30, IMAX - 1, IMAX]
calls = nonzero = 0


def stage(c):
    global calls, nonzero
    print("stage", c, flush=True)          # names the case if the call below ends the process
    r = lib.dp_stage_workspace_bytes(C.byref(StageConfig(**c)))
    calls += 1
    nonzero += r != 0
    assert 0 <= r < 2 ** 62
    return r


assert stage(base) > 0
int_fields = [k for k in base if k not in ("rope_theta", "eps")]
for dt in (0, 1):
    for f in int_fields:
        for v in wild:
            c = dict(base, dtype=dt)
            c[f] = v
            if f == "dim" and v > 0:
                c["n_heads"] = max(1, v // 128)
            stage(c)
rng = random.Random(1)
mix = [k for k in int_fields if k not in ("dtype", "head_dim")]
for _ in range(3000):
    c = dict(base, dtype=rng.choice((0, 1)))
    for f in rng.sample(mix, 3):
        c[f] = rng.choice(wild)
    if rng.random() < 0.5 and c["dim"] > 0:
        c["n_heads"] = max(1, c["dim"] // c["head_dim"])
    stage(c)
# the largest sizes validation lets through, all at once
stage(dict(base, n_layers=1024, dim=8192, n_heads=64, ffn_dim=1 << 17, text_len=1 << 20, text_dim=1 << 16, tok_h=4096,
           tok_w=4096, max_block_frames=1, max_cache_frames=1, max_abs_frames=1 << 24, freq_dim=1 << 16, debug_taps=1))

eb = dict(dim=1536, tok_h=30, tok_w=52, channels=16, max_frames=8, dtype=1, freq_dim=256, eps=1e-6)
for dt in (0, 1):
    for f in [k for k in eb if k != "eps"]:
        for v in wild:
            c = dict(eb, dtype=dt)
            c[f] = v
            print("ends", c, flush=True)
            r = lib.dp_ends_workspace_bytes(C.byref(EndsConfig(**c)))
            calls += 1
            assert 0 <= r < 2 ** 62
print("ok", calls, "calls,", nonzero, "accepted")
