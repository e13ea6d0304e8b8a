"""Thin ctypes binding of libdualparal.so: argument marshalling only.

Every step of the stage runs in the library's HIP kernels; torch is used for
device memory (weights, workspace, activations) and for the stream handle.
There is no fallback: if the library has not been built, importing fails.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdualparal.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_21070_amd.build` "
                      "(hipcc, gfx950); there is no fallback path")
_lib = C.CDLL(LIB_PATH)

DP_OK, DP_EINVAL, DP_ENOMEM, DP_ESTATE, DP_EHIP = 0, -1, -2, -3, -4
DP_F32, DP_BF16 = 0, 1
WEIGHT_LAYOUT = {"in_out": 0, "out_in": 1}
ORDER = {"reverse": 0, "sequential": 1}
PEEK = dict(k=0, v=1, cache_k=2, cache_v=3, q=4, attn=5, cross_attn=6, x_self=7, x_cross=8, mod=9,
            text_k=10, text_v=11, x_res=12)

LAYER_FIELDS = ("mod", "wq", "bq", "wk", "bk", "wv", "bv", "gq", "gk", "wo", "bo", "ln3_g", "ln3_b",
                "cwq", "cbq", "cgq", "cwk", "cbk", "cgk", "cwv", "cbv", "cwo", "cbo", "w1", "b1", "w2", "b2")
STAGE_FIELDS = ("wt1", "bt1", "wt2", "bt2", "wm", "bm", "wx1", "bx1", "wx2", "bx2")


class StageConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "dim", "n_heads", "head_dim", "ffn_dim", "text_len",
                                         "text_dim", "tok_h", "tok_w", "max_block_frames", "max_cache_frames",
                                         "max_abs_frames", "dtype", "freq_dim")] + \
               [("rope_theta", C.c_float), ("eps", C.c_float), ("debug_taps", C.c_int32), ("weight_layout", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class StageWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in STAGE_FIELDS] + [("layers", C.POINTER(LayerWeights))]


class SchedConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("T", "block_num", "num_b", "num_c", "first_block_frames", "order")] + \
               [("t_max", C.c_float), ("input", C.c_int32)]


class SchedEntry(C.Structure):
    _fields_ = [("step", C.c_int32), ("block", C.c_int32), ("level", C.c_int32), ("timestep", C.c_float),
                ("frame0", C.c_int32), ("n_frames", C.c_int32), ("cache_block", C.c_int32),
                ("cache_first", C.c_int32), ("cache_frames", C.c_int32), ("in_frame0", C.c_int32),
                ("in_frames", C.c_int32), ("keep_first", C.c_int32)]


_lib.dp_stage_workspace_bytes.restype = C.c_size_t
_lib.dp_stage_workspace_bytes.argtypes = [C.POINTER(StageConfig)]
_lib.dp_stage_kv_bytes.restype = C.c_size_t
_lib.dp_stage_kv_bytes.argtypes = [C.POINTER(StageConfig)]
_lib.dp_stage_init.restype = C.c_int
_lib.dp_stage_init.argtypes = [C.POINTER(StageConfig), C.POINTER(StageWeights), C.c_void_p, C.c_void_p, C.c_size_t,
                               C.c_void_p, C.POINTER(C.c_void_p)]
_lib.dp_stage_forward.restype = C.c_int
_lib.dp_stage_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p]
_lib.dp_cache_update.restype = C.c_int
_lib.dp_cache_update.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
_lib.dp_blockwise_schedule.restype = C.c_int
_lib.dp_blockwise_schedule.argtypes = [C.POINTER(SchedConfig), C.POINTER(SchedEntry), C.c_int64, C.POINTER(C.c_int64)]
_lib.dp_bubble_ratio.restype = C.c_double
_lib.dp_bubble_ratio.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
_lib.dp_stage_peek.restype = C.c_int
_lib.dp_stage_peek.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.POINTER(C.c_int64), C.c_void_p]
PROF = ("ln", "qkv_gemm", "norm_rope", "self_attn", "oproj_gemm", "cross_q_gemm", "cross_attn", "cross_o_gemm",
        "ffn1_gemm", "ffn2_gemm", "cache_copy", "modulation", "convert")
_lib.dp_stage_profile_begin.restype = C.c_int
_lib.dp_stage_profile_begin.argtypes = [C.c_void_p, C.c_uint32]
_lib.dp_stage_profile_end.restype = C.c_int
_lib.dp_stage_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
_lib.dp_stage_free.restype = None
class NoiseConfig(C.Structure):
    _fields_ = [("block_num", C.c_int32), ("num_b", C.c_int32), ("num_c", C.c_int32)]


_lib.dp_noise_assign.restype = C.c_int
_lib.dp_noise_assign.argtypes = [C.POINTER(NoiseConfig), C.POINTER(C.c_uint32), C.c_int64, C.POINTER(C.c_int32),
                                 C.c_int64, C.POINTER(C.c_int64)]
_lib.dp_noise_gather.restype = C.c_int
_lib.dp_noise_gather.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
class EndsConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dim", "tok_h", "tok_w", "channels", "max_frames", "dtype", "freq_dim")] + \
               [("eps", C.c_float)]


ENDS_FIELDS = ("w_pe", "b_pe", "m_head", "w_head", "b_head", "wt1", "bt1", "wt2", "bt2")


class EndsWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ENDS_FIELDS]


_lib.dp_ends_workspace_bytes.restype = C.c_size_t
_lib.dp_ends_workspace_bytes.argtypes = [C.POINTER(EndsConfig)]
_lib.dp_ends_init.restype = C.c_int
_lib.dp_ends_init.argtypes = [C.POINTER(EndsConfig), C.POINTER(EndsWeights), C.c_void_p, C.c_size_t, C.c_void_p,
                              C.POINTER(C.c_void_p)]
_lib.dp_embed_forward.restype = C.c_int
_lib.dp_embed_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
_lib.dp_head_forward.restype = C.c_int
_lib.dp_head_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_int32, C.c_void_p]
_lib.dp_head_forward_static.restype = C.c_int
_lib.dp_head_forward_static.argtypes = [C.POINTER(EndsConfig), C.POINTER(EndsWeights), C.c_void_p, C.c_float, C.c_void_p,
                                        C.c_int32, C.c_void_p]
_lib.dp_euler_step.restype = C.c_int
_lib.dp_euler_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_float, C.c_void_p]
_lib.dp_ends_free.restype = None
_lib.dp_ends_free.argtypes = [C.c_void_p]
_lib.dp_pipeline_simulate.restype = C.c_int
_lib.dp_pipeline_simulate.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
_lib.dp_probe_mfma_bf16.restype = C.c_int
_lib.dp_probe_mfma_bf16.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(C.c_double)]
_lib.dp_probe_stream_f32_bf16.restype = C.c_int
_lib.dp_probe_stream_f32_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
_lib.dp_stage_free.argtypes = [C.c_void_p]
_lib.dp_last_error.restype = C.c_char_p
_lib.dp_last_error.argtypes = []


class DualParalError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where} failed with status {code}: {_lib.dp_last_error().decode()}")


def last_error():
    return _lib.dp_last_error().decode()


def _check(code, where):
    if code != DP_OK:
        raise DualParalError(code, where)


def make_config(cfg, max_block_frames=None, max_cache_frames=None, max_abs_frames=4096, debug_taps=0,
                weight_layout="in_out"):
    """cfg: dict as produced by synth.stage_config."""
    c = StageConfig()
    for n in ("n_layers", "dim", "n_heads", "head_dim", "ffn_dim", "text_len", "text_dim", "tok_h", "tok_w", "freq_dim"):
        setattr(c, n, int(cfg[n]))
    c.max_block_frames = int(max_block_frames if max_block_frames is not None else cfg["block_frames"])
    c.max_cache_frames = int(max_cache_frames if max_cache_frames is not None else cfg["cache_frames"])
    c.max_abs_frames = int(max_abs_frames)
    c.dtype = DP_BF16 if cfg["dtype"] == "bf16" else DP_F32
    c.rope_theta = float(cfg["rope_theta"])
    c.eps = float(cfg["eps"])
    c.debug_taps = int(debug_taps)
    c.weight_layout = WEIGHT_LAYOUT[weight_layout]
    return c


def workspace_bytes(config):
    return int(_lib.dp_stage_workspace_bytes(C.byref(config)))


def kv_bytes_per_layer(config):
    return int(_lib.dp_stage_kv_bytes(C.byref(config)))


def _stream_handle(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


class Stage:
    """One pipeline stage on the current device.  weights: {"stage": {...}, "layers": [{...}]} of device
    tensors in the stage's dtype (contiguous; matrices [in, out], or as weights_out_in returns them when the
    config says "out_in"); text: device [text_len, text_dim]."""

    def __init__(self, config, weights, text, stream=None):
        self.config = config
        self.torch_dtype = torch.bfloat16 if config.dtype == DP_BF16 else torch.float32
        dev = text.device
        assert dev.type == "cuda", "the stage runs on the GPU only"
        self._keep = [weights, text]            # the library borrows this memory for the handle's life

        def ptr(t, shape):
            assert t.is_cuda and t.dtype == self.torch_dtype and t.is_contiguous() and tuple(t.shape) == tuple(shape), \
                (tuple(t.shape), shape, t.dtype)
            return t.data_ptr()

        D, F, Td, fd = config.dim, config.ffn_dim, config.text_dim, config.freq_dim
        oi = config.weight_layout == WEIGHT_LAYOUT["out_in"]
        sw = StageWeights()
        shapes = dict(wt1=(fd, D), bt1=(D,), wt2=(D, D), bt2=(D,), wm=(D, 6 * D), bm=(6 * D,),
                      wx1=(D, Td) if oi else (Td, D), bx1=(D,), wx2=(D, D), bx2=(D,))
        for n in STAGE_FIELDS:
            if n in weights["stage"]:
                setattr(sw, n, ptr(weights["stage"][n], shapes[n]))
        arr = (LayerWeights * config.n_layers)()
        for i, lw in enumerate(weights["layers"]):
            for n in LAYER_FIELDS:
                shape = (6, D) if n == "mod" else ((F, D) if oi else (D, F)) if n == "w1" else (F,) if n == "b1" \
                    else ((D, F) if oi else (F, D)) if n == "w2" \
                    else (D, D) if n in ("wq", "wk", "wv", "wo", "cwq", "cwk", "cwv", "cwo") else (D,)
                setattr(arr[i], n, ptr(lw[n], shape))
        sw.layers = arr
        assert tuple(text.shape) == (config.text_len, Td) and text.dtype == self.torch_dtype and text.is_contiguous()
        nbytes = workspace_bytes(config)
        if nbytes == 0:
            raise DualParalError(DP_EINVAL, "dp_stage_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        h = C.c_void_p()
        self._h = None
        _check(_lib.dp_stage_init(C.byref(config), C.byref(sw), text.data_ptr(), self.workspace.data_ptr(), nbytes,
                                  _stream_handle(stream), C.byref(h)), "dp_stage_init")
        self._h = h
        self.tok = config.tok_h * config.tok_w

    def forward(self, x_in, n_frames, frame0, timestep, out=None, stream=None):
        assert x_in.is_cuda and x_in.dtype == self.torch_dtype and x_in.is_contiguous()
        assert tuple(x_in.shape) == (n_frames * self.tok, self.config.dim), tuple(x_in.shape)
        if out is None:
            out = torch.empty_like(x_in)
        assert out.shape == x_in.shape and out.dtype == x_in.dtype and out.is_contiguous() and out.is_cuda
        _check(_lib.dp_stage_forward(self._h, x_in.data_ptr(), out.data_ptr(), n_frames, frame0, float(timestep),
                                     _stream_handle(stream)), "dp_stage_forward")
        return out

    def cache_update(self, first_frame, n_frames, stream=None):
        _check(_lib.dp_cache_update(self._h, first_frame, n_frames, _stream_handle(stream)), "dp_cache_update")

    def peek(self, what, layer=0, stream=None):
        max_rows = max(self.config.max_block_frames * self.tok, self.config.text_len, 6)
        buf = torch.empty((max_rows, self.config.dim), dtype=torch.float32, device=self.workspace.device)
        rows = C.c_int64()
        _check(_lib.dp_stage_peek(self._h, PEEK[what], layer, buf.data_ptr(), buf.numel(), C.byref(rows),
                                  _stream_handle(stream)), "dp_stage_peek")
        return buf[: rows.value]

    def profile_begin(self, classes):
        """classes: iterable of names from PROF (or "all")."""
        names = PROF if classes == "all" else classes
        mask = 0
        for n in names:
            mask |= 1 << PROF.index(n)
        _check(_lib.dp_stage_profile_begin(self._h, mask), "dp_stage_profile_begin")

    def profile_end(self):
        """{class: (total_ms, launches)} for the classes that were launched."""
        ms = (C.c_double * len(PROF))()
        n = (C.c_int64 * len(PROF))()
        _check(_lib.dp_stage_profile_end(self._h, ms, n), "dp_stage_profile_end")
        return {PROF[i]: (ms[i], n[i]) for i in range(len(PROF)) if n[i] > 0}

    def close(self):
        if self._h is not None:
            _lib.dp_stage_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


INPUT = {"block": 0, "extended": 1, "nocache": 2}


def blockwise_schedule(T, block_num, num_b, num_c, first_block_frames=0, t_max=1000.0, order="reverse", variant="block"):
    cfg = SchedConfig(T, block_num, num_b, num_c, first_block_frames, ORDER[order], t_max, INPUT[variant])
    n = C.c_int64()
    rc = _lib.dp_blockwise_schedule(C.byref(cfg), None, 0, C.byref(n))
    if rc not in (DP_OK, DP_ENOMEM):
        raise DualParalError(rc, "dp_blockwise_schedule")
    arr = (SchedEntry * n.value)()
    _check(_lib.dp_blockwise_schedule(C.byref(cfg), arr, n.value, C.byref(n)), "dp_blockwise_schedule")
    return [{f: getattr(e, f) for f, _ in SchedEntry._fields_} for e in arr]


def bubble_ratio(n_devices, T, block_num, order="reverse"):
    return float(_lib.dp_bubble_ratio(n_devices, T, block_num, ORDER[order]))


class Ends:
    """Patch embedding and output head of the model on the current device.  weights: dict of device tensors in
    the storage dtype with ENDS_FIELDS (the timestep MLP arrays are the stage's)."""

    def __init__(self, cfg, weights, channels, max_frames, stream=None):
        dt = DP_BF16 if cfg["dtype"] == "bf16" else DP_F32
        self.config = EndsConfig(cfg["dim"], cfg["tok_h"], cfg["tok_w"], channels, max_frames, dt, cfg["freq_dim"], cfg["eps"])
        self.torch_dtype = torch.bfloat16 if dt == DP_BF16 else torch.float32
        self.tok, self.dim, self.channels = cfg["tok_h"] * cfg["tok_w"], cfg["dim"], channels
        self.frame_shape = (2 * cfg["tok_h"], 2 * cfg["tok_w"], channels)
        D, P, fd = cfg["dim"], 4 * channels, cfg["freq_dim"]
        shapes = dict(w_pe=(P, D), b_pe=(D,), m_head=(2, D), w_head=(D, P), b_head=(P,), wt1=(fd, D), bt1=(D,),
                      wt2=(D, D), bt2=(D,))
        ew = EndsWeights()
        for n in ENDS_FIELDS:
            t = weights[n]
            assert t.is_cuda and t.dtype == self.torch_dtype and t.is_contiguous() and tuple(t.shape) == shapes[n], n
            setattr(ew, n, t.data_ptr())
        self._keep = weights
        nbytes = _lib.dp_ends_workspace_bytes(C.byref(self.config))
        if nbytes == 0:
            raise DualParalError(DP_EINVAL, "dp_ends_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        self._h = None
        _check(_lib.dp_ends_init(C.byref(self.config), C.byref(ew), self.workspace.data_ptr(), nbytes,
                                 _stream_handle(stream), C.byref(h)), "dp_ends_init")
        self._h = h

    def embed(self, latent, stream=None):
        n = latent.shape[0]
        assert latent.is_cuda and latent.dtype == torch.float32 and latent.is_contiguous() and tuple(latent.shape[1:]) == self.frame_shape
        out = torch.empty((n * self.tok, self.dim), dtype=self.torch_dtype, device=latent.device)
        _check(_lib.dp_embed_forward(self._h, latent.data_ptr(), out.data_ptr(), n, _stream_handle(stream)), "dp_embed_forward")
        return out

    def head(self, x, timestep, n_frames, stream=None):
        assert x.is_cuda and x.dtype == self.torch_dtype and x.is_contiguous() and tuple(x.shape) == (n_frames * self.tok, self.dim)
        v = torch.empty((n_frames,) + self.frame_shape, dtype=torch.float32, device=x.device)
        _check(_lib.dp_head_forward(self._h, x.data_ptr(), float(timestep), v.data_ptr(), n_frames, _stream_handle(stream)),
               "dp_head_forward")
        return v

    def close(self):
        if self._h is not None:
            _lib.dp_ends_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def head_forward_static(cfg, weights, channels, x, timestep, n_frames, out, stream=None):
    """dp_head_forward_static: the output head without handle or workspace.  `out` is the caller's float32
    [n_frames, 2*tok_h, 2*tok_w, channels] device tensor (the call itself allocates nothing)."""
    dt = DP_BF16 if cfg["dtype"] == "bf16" else DP_F32
    td = torch.bfloat16 if dt == DP_BF16 else torch.float32
    conf = EndsConfig(cfg["dim"], cfg["tok_h"], cfg["tok_w"], channels, n_frames, dt, cfg["freq_dim"], cfg["eps"])
    ew = EndsWeights()
    for n in ENDS_FIELDS:
        t = weights[n]
        assert t.is_cuda and t.dtype == td and t.is_contiguous(), n
        setattr(ew, n, t.data_ptr())
    tok = cfg["tok_h"] * cfg["tok_w"]
    assert x.is_cuda and x.dtype == td and x.is_contiguous() and tuple(x.shape) == (n_frames * tok, cfg["dim"])
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
    assert tuple(out.shape) == (n_frames, 2 * cfg["tok_h"], 2 * cfg["tok_w"], channels)
    _check(_lib.dp_head_forward_static(C.byref(conf), C.byref(ew), x.data_ptr(), float(timestep), out.data_ptr(), n_frames,
                                       _stream_handle(stream)), "dp_head_forward_static")
    return out


def euler_step(x, v, sigma, sigma_next, stream=None):
    """In place: x += (sigma_next - sigma) * v (float32 device tensors of equal size)."""
    assert x.is_cuda and v.is_cuda and x.dtype == v.dtype == torch.float32 and x.is_contiguous() and v.is_contiguous()
    assert x.numel() == v.numel()
    _check(_lib.dp_euler_step(x.data_ptr(), v.data_ptr(), x.numel(), float(sigma), float(sigma_next), _stream_handle(stream)),
           "dp_euler_step")
    return x


def pipeline_simulate(n_devices, T, block_num, order="reverse"):
    """(makespan, idle slots per device) of the N-device pipeline running the block queue."""
    mk, bub = C.c_int64(), C.c_int64()
    _check(_lib.dp_pipeline_simulate(n_devices, T, block_num, ORDER[order], C.byref(mk), C.byref(bub)), "dp_pipeline_simulate")
    return mk.value, bub.value


def noise_assign(block_num, num_b, num_c, words):
    """Pool-frame indices of every block (list of lists), from the caller's uint32 random words."""
    cfg = NoiseConfig(block_num, num_b, num_c)
    w = (C.c_uint32 * max(len(words), 1))(*[int(v) for v in words])
    n = C.c_int64()
    rc = _lib.dp_noise_assign(C.byref(cfg), w, len(words), None, 0, C.byref(n))
    if rc not in (DP_OK, DP_ENOMEM):
        raise DualParalError(rc, "dp_noise_assign")
    arr = (C.c_int32 * n.value)()
    _check(_lib.dp_noise_assign(C.byref(cfg), w, len(words), arr, n.value, C.byref(n)), "dp_noise_assign")
    flat, first = list(arr), num_b + num_c // 2
    return [flat[:first]] + [flat[first + i * num_b: first + (i + 1) * num_b] for i in range(block_num - 1)]


def noise_gather(pool, index, out=None):
    """out[f] = pool[index[f]] on the device; pool is [pool_frames, ...], index an int32 device tensor."""
    assert pool.is_cuda and pool.is_contiguous() and index.is_cuda and index.dtype == torch.int32
    n = int(index.numel())
    if out is None:
        out = torch.empty((n,) + tuple(pool.shape[1:]), dtype=pool.dtype, device=pool.device)
    frame_bytes = pool[0].numel() * pool.element_size()
    stream = torch.cuda.current_stream().cuda_stream
    _check(_lib.dp_noise_gather(pool.data_ptr(), pool.shape[0], frame_bytes, index.data_ptr(), n, out.data_ptr(), stream),
           "dp_noise_gather")
    return out


def probe_mfma_bf16(operands="random", iters=20000, device="cuda"):
    """Rate (TFLOP/s) of back-to-back bf16 MFMAs with all-zero or pseudo-random operand bits."""
    scratch = torch.empty(131072, dtype=torch.float32, device=device)
    out = C.c_double()
    stream = torch.cuda.current_stream().cuda_stream
    _check(_lib.dp_probe_mfma_bf16({"zeros": 0, "random": 1}[operands], iters, scratch.data_ptr(), scratch.numel(),
                                   stream, C.byref(out)), "dp_probe_mfma_bf16")
    return out.value


def probe_stream_f32_bf16(n, iters=20, device="cuda"):
    """Rate (GB/s) of a plain fp32 -> bf16 streaming pass over n elements (the LayerNorm's traffic shape)."""
    src = torch.ones(n, dtype=torch.float32, device=device)
    dst = torch.empty(n, dtype=torch.bfloat16, device=device)
    out = C.c_double()
    stream = torch.cuda.current_stream().cuda_stream
    _check(_lib.dp_probe_stream_f32_bf16(src.data_ptr(), dst.data_ptr(), n, iters, stream, C.byref(out)),
           "dp_probe_stream_f32_bf16")
    return out.value


def weights_out_in(weights):
    """Device weights with [in, out] matrices -> the same weights as the "out_in" layout wants them: every matrix
    the GEMMs multiply by transposed to [out, in], q | k | v in one [3 * dim, dim] tensor (the three entries
    are views of it).  The timestep MLP and the modulation head stay [in, out]."""
    def t(m):
        return m.t().contiguous()
    st = dict(weights["stage"])
    for n in ("wx1", "wx2"):
        if n in st:
            st[n] = t(st[n])
    layers = []
    for lw in weights["layers"]:
        o = dict(lw)
        D = lw["wq"].shape[0]
        qkv = torch.cat([lw["wq"].t(), lw["wk"].t(), lw["wv"].t()], dim=0).contiguous()
        o["wq"], o["wk"], o["wv"] = qkv[:D], qkv[D:2 * D], qkv[2 * D:]
        for n in ("wo", "cwq", "cwk", "cwv", "cwo", "w1", "w2"):
            o[n] = t(lw[n])
        layers.append(o)
    return {"stage": st, "layers": layers}


def weights_to_device(weights, dtype, device="cuda"):
    """synth weights (fp32 CPU tensors holding values representable in `dtype`) -> device tensors of `dtype`."""
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    return {"stage": {k: v.to(device=device, dtype=td).contiguous() for k, v in weights["stage"].items()},
            "layers": [{k: v.to(device=device, dtype=td).contiguous() for k, v in lw.items()} for lw in weights["layers"]]}
