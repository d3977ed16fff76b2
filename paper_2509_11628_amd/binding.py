"""ctypes binding of libspeca.so: argument marshalling only.  Every step of the
sampling path runs inside the library's HIP kernels; torch is used here for device
memory and the current stream.  Names mirror include/speca.h."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspeca.so")

OK, EINVAL, ENOMEM, ESTATE, EHIP, EUNSUPPORTED = range(6)
F32, BF16 = 0, 1
MODEL_NONE, MODEL_DIT, MODEL_MMDIT = 0, 1, 2
COEF_TAYLOR, COEF_NEWTON, COEF_ADAMS_BASHFORTH = 0, 1, 2
SOLVER_DDIM, SOLVER_FLOW, SOLVER_DDPM = 0, 1, 2
CACHE_DIFFERENCES, CACHE_RING = 0, 1
KIND_FULL, KIND_SPEC, KIND_REJECT = 0, 1, 2
METRIC_L2, METRIC_L1, METRIC_LINF, METRIC_COSINE = 0, 1, 2, 3
MAX_ORDER = 4
MAX_LAUNCH_ROWS = 64


class SpecaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"speca status {code}: {msg}")
        self.code = code
        self.msg = msg


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "kind", "dtype", "depth", "depth_single", "hidden", "heads", "mlp_hidden", "in_channels",
        "latent_t", "latent_h", "latent_w", "patch", "num_classes", "freq_dim", "txt_tokens",
        "txt_dim", "vec_dim", "n_slots", "tokens")]


class Weights(C.Structure):
    _fields_ = [("count", C.c_int32), ("names", C.POINTER(C.c_char_p)),
                ("ptrs", C.POINTER(C.c_void_p)), ("numel", C.POINTER(C.c_int64))]


class Cfg(C.Structure):
    _fields_ = [("order", C.c_int32), ("interval", C.c_int32), ("verify_block", C.c_int32),
                ("coef_mode", C.c_int32), ("eps", C.c_float), ("warmup_full", C.c_int32),
                ("metric", C.c_int32), ("layout", C.c_int32)]


class Cond(C.Structure):
    _fields_ = [("labels", C.POINTER(C.c_int32)), ("txt", C.c_void_p), ("pooled", C.c_void_p),
                ("timestep", C.c_float)]


class Solver(C.Structure):
    _fields_ = [("kind", C.c_int32), ("steps", C.c_int32), ("timesteps", C.POINTER(C.c_float)),
                ("table", C.POINTER(C.c_float)), ("cfg_scale", C.c_float), ("noise", C.c_void_p)]


class Trace(C.Structure):
    _fields_ = [("kind", C.POINTER(C.c_int8)), ("err", C.POINTER(C.c_float)),
                ("n_full", C.c_int32), ("n_spec", C.c_int32), ("n_reject", C.c_int32)]


class Profile(C.Structure):
    _fields_ = [("launches", C.c_int64 * 6), ("ms", C.c_double * 6), ("flops", C.c_double * 6), ("bytes", C.c_double * 6)]


PROF_CLASSES = ["gemm", "attention", "forecast", "verify", "refresh", "other"]

_lib = None


def load_library() -> C.CDLL:
    """Load libspeca.so (built in-tree by paper_2509_11628_amd.build).  torch is imported
    first so that the library binds to the HIP runtime torch already loaded.  There is no
    fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads libamdhip64 with the soname libspeca.so needs)
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2509_11628_amd.build` "
                          "(there is no CPU fallback for the HIP path)")
    lib = C.CDLL(LIB_PATH)
    i32p, f32p, u8p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_uint8), C.c_void_p
    sig = {
        "speca_create": [C.POINTER(vp), C.POINTER(ModelDesc), C.POINTER(Weights), vp],
        "speca_destroy": [vp],
        "speca_init_cache": [vp, C.POINTER(Cfg), C.c_int],
        "speca_refresh": [vp, C.c_int, i32p, C.c_int, vp],
        "speca_full_step": [vp, vp, C.POINTER(Cond), C.c_int, i32p, C.c_int, vp],
        "speca_forecast": [vp, C.c_int, i32p, C.c_int, vp],
        "speca_verify": [vp, vp, vp, C.c_int, C.c_int64, C.c_int, f32p, C.c_float, f32p, u8p],
        "speca_verify_static": [vp, vp, vp, C.c_int, C.c_int64, C.c_int, vp, C.c_float, vp, vp],
        "speca_spec_step": [vp, vp, C.POINTER(Cond), C.c_int, i32p, C.c_int, f32p, C.c_int, f32p, u8p, vp],
        "speca_sample": [vp, vp, C.c_int, C.POINTER(Cond), C.POINTER(Solver), f32p, C.POINTER(Trace)],
        "speca_linear": [vp, C.c_int, vp, C.c_int, C.c_int, vp, C.c_int, vp, C.c_int, vp],
        "speca_attention": [vp, C.c_int, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int],
        "speca_set_lanes": [vp, C.c_int, C.c_int],
        "speca_profile_begin": [vp],
        "speca_profile_end": [vp, C.POINTER(Profile)],
        "speca_tau_geometric": [C.c_float, C.c_float, C.c_int, f32p],
        "speca_tau_linear": [C.c_float, C.c_float, C.c_int, f32p],
        "speca_coefficients": [C.c_int, C.c_int, i32p, C.c_int, C.c_int, f32p],
        "speca_divisors": [C.c_int, C.c_int, i32p, C.c_int, C.c_int, f32p],
        "speca_ring_weights": [C.c_int, C.c_int, i32p, C.c_int, C.c_int, f32p, i32p, C.POINTER(C.c_int)],
        "speca_sched_create": [C.POINTER(vp), C.c_int, C.POINTER(Cfg)],
        "speca_sched_destroy": [vp],
        "speca_sched_plan": [vp, C.c_int, C.c_float, i32p, C.POINTER(C.c_int), i32p, C.POINTER(C.c_int)],
        "speca_sched_commit": [vp, C.c_int, u8p, C.POINTER(C.c_int8)],
        "speca_sched_refs": [vp, C.c_int, i32p, C.POINTER(C.c_int)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.speca_last_error.argtypes = [vp]
    lib.speca_last_error.restype = C.c_char_p
    _lib = lib
    return lib


EXPORTED = ["speca_create", "speca_destroy", "speca_last_error", "speca_init_cache", "speca_refresh",
            "speca_full_step", "speca_forecast", "speca_verify", "speca_verify_static", "speca_spec_step", "speca_sample",
            "speca_linear", "speca_attention", "speca_set_lanes", "speca_profile_begin", "speca_profile_end",
            "speca_tau_geometric", "speca_tau_linear", "speca_coefficients", "speca_divisors",
            "speca_ring_weights", "speca_sched_create", "speca_sched_destroy", "speca_sched_plan", "speca_sched_commit",
            "speca_sched_refs"]


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def make_cfg(order=2, interval=5, verify_block=-1, coef_mode=COEF_TAYLOR, eps=1e-8, warmup_full=1,
             metric=METRIC_L2, layout=CACHE_DIFFERENCES) -> Cfg:
    return Cfg(order, interval, verify_block, coef_mode, eps, warmup_full, metric, layout)


# ---- host-only helpers ------------------------------------------------------------------


def tau_geometric(tau0: float, beta: float, steps: int) -> np.ndarray:
    out = np.empty(steps, np.float32)
    _check(None, load_library().speca_tau_geometric(tau0, beta, steps, _p(out, C.c_float)))
    return out


def tau_linear(a: float, b: float, steps: int) -> np.ndarray:
    out = np.empty(steps, np.float32)
    _check(None, load_library().speca_tau_linear(a, b, steps, _p(out, C.c_float)))
    return out


def coefficients(mode: int, step: int, refs: Sequence[int], order: int) -> np.ndarray:
    r = _i32(refs)
    out = np.zeros(order + 1, np.float32)
    _check(None, load_library().speca_coefficients(mode, step, _p(r, C.c_int32), len(r), order, _p(out, C.c_float)))
    return out


def ring_weights(mode: int, order: int, full_steps: Sequence[int], step: int):
    """-> (weights by age [n], planes by age [n]) of the ring layout after the given full steps."""
    r = _i32(full_steps)
    w = np.zeros(order + 1, np.float32); pl = np.zeros(order + 1, np.int32); n = C.c_int(0)
    _check(None, load_library().speca_ring_weights(mode, order, _p(r, C.c_int32), len(r), step, _p(w, C.c_float), _p(pl, C.c_int32),
                                                   C.byref(n)))
    return w[:n.value], pl[:n.value]


def divisors(mode: int, step: int, refs: Sequence[int], order: int) -> np.ndarray:
    r = _i32(refs)
    out = np.zeros(max(order, 1), np.float32)
    _check(None, load_library().speca_divisors(mode, step, _p(r, C.c_int32), len(r), order, _p(out, C.c_float)))
    return out[:order]


def _check(ctx, code: int):
    if code != OK:
        msg = load_library().speca_last_error(ctx).decode() if ctx is not None else ""
        raise SpecaError(code, msg)


def linear(a, w, bias=None, act: int = 0, out=None):
    """speca_linear on torch device tensors: a [M,K], w [N,K] -> [M,N]."""
    import torch
    lib = load_library()
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K and a.is_contiguous() and w.is_contiguous() and a.dtype == w.dtype
    if out is None:
        out = torch.empty((M, N), dtype=a.dtype, device=a.device)
    dt = BF16 if a.dtype == torch.bfloat16 else F32
    code = lib.speca_linear(C.c_void_p(torch.cuda.current_stream().cuda_stream), dt, C.c_void_p(a.data_ptr()), M, K,
                            C.c_void_p(w.data_ptr()), N, C.c_void_p(bias.data_ptr()) if bias is not None else None, act,
                            C.c_void_p(out.data_ptr()))
    if code != OK:
        raise SpecaError(code, lib.speca_last_error(None).decode())
    return out


def attention(qkv, heads: int, out=None):
    """speca_attention on a torch device tensor qkv [rows, T, 3*H*hd] -> [rows, T, H*hd]."""
    import torch
    lib = load_library()
    rows, T, D3 = qkv.shape
    D = D3 // 3
    assert qkv.is_contiguous() and D % heads == 0
    if out is None:
        out = torch.empty((rows, T, D), dtype=qkv.dtype, device=qkv.device)
    dt = BF16 if qkv.dtype == torch.bfloat16 else F32
    code = lib.speca_attention(C.c_void_p(torch.cuda.current_stream().cuda_stream), dt, C.c_void_p(qkv.data_ptr()),
                               C.c_void_p(out.data_ptr()), rows, T, heads, D // heads)
    if code != OK:
        raise SpecaError(code, lib.speca_last_error(None).decode())
    return out


class Scheduler:
    """speca_sched_*: the per-sample full/speculative state machine (host only)."""

    def __init__(self, batch: int, cfg: Cfg):
        self.lib = load_library()
        self.h = C.c_void_p()
        self.batch = batch
        code = self.lib.speca_sched_create(C.byref(self.h), batch, C.byref(cfg))
        if code != OK:
            raise SpecaError(code, "speca_sched_create")

    def plan(self, step: int, tau_s: float):
        spec = np.zeros(self.batch, np.int32); full = np.zeros(self.batch, np.int32)
        ns, nf = C.c_int(0), C.c_int(0)
        code = self.lib.speca_sched_plan(self.h, step, tau_s, _p(spec, C.c_int32), C.byref(ns), _p(full, C.c_int32), C.byref(nf))
        if code != OK:
            raise SpecaError(code, "speca_sched_plan")
        return spec[:ns.value].tolist(), full[:nf.value].tolist()

    def commit(self, step: int, accept: Sequence[int]):
        acc = np.ascontiguousarray(accept, dtype=np.uint8)
        kinds = np.zeros(self.batch, np.int8)
        code = self.lib.speca_sched_commit(self.h, step, _p(acc, C.c_uint8) if len(acc) else None, _p(kinds, C.c_int8))
        if code != OK:
            raise SpecaError(code, "speca_sched_commit")
        return kinds

    def refs(self, sample: int):
        r = np.zeros(MAX_ORDER + 1, np.int32); n = C.c_int(0)
        code = self.lib.speca_sched_refs(self.h, sample, _p(r, C.c_int32), C.byref(n))
        if code != OK:
            raise SpecaError(code, "speca_sched_refs")
        return r[:n.value].tolist()

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.speca_sched_destroy(self.h)
            self.h = None


# ---- device contexts ------------------------------------------------------------------------


def _torch_dtype(dtype: int):
    import torch
    return torch.bfloat16 if dtype == BF16 else torch.float32


class Context:
    """speca_ctx wrapper.  Tensors are torch CUDA(HIP) tensors; only their data_ptr()
    crosses the boundary."""

    def __init__(self, desc: ModelDesc, weights: Optional[Dict[str, "object"]] = None, stream=None):
        import torch
        self.lib = load_library()
        self.desc = desc
        self.h = C.c_void_p()
        self._keep = []
        wptr = None
        if weights is not None:
            names = list(weights.keys())
            n = len(names)
            arr_names = (C.c_char_p * n)(*[s.encode() for s in names])
            arr_ptrs = (C.c_void_p * n)(*[weights[k].data_ptr() for k in names])
            arr_numel = (C.c_int64 * n)(*[weights[k].numel() for k in names])
            w = Weights(n, arr_names, arr_ptrs, arr_numel)
            self._keep += [weights, arr_names, arr_ptrs, arr_numel, w]
            wptr = C.byref(w)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        code = self.lib.speca_create(C.byref(self.h), C.byref(desc), wptr, C.c_void_p(self.stream.cuda_stream))
        if code != OK:
            raise SpecaError(code, self.lib.speca_last_error(None).decode())
        self.batch_rows = 0
        self.cfg = None

    def close(self):
        if getattr(self, "h", None):
            self.lib.speca_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def _ck(self, code):
        if code != OK:
            raise SpecaError(code, self.lib.speca_last_error(self.h).decode())

    def init_cache(self, cfg: Cfg, batch_rows: int):
        self._ck(self.lib.speca_init_cache(self.h, C.byref(cfg), batch_rows))
        self.cfg, self.batch_rows = cfg, batch_rows

    def refresh(self, step: int, rows, features):
        r = _i32(rows)
        self._ck(self.lib.speca_refresh(self.h, step, _p(r, C.c_int32), len(r), C.c_void_p(features.data_ptr())))

    def forecast(self, step: int, rows, out):
        r = _i32(rows)
        self._ck(self.lib.speca_forecast(self.h, step, _p(r, C.c_int32), len(r), C.c_void_p(out.data_ptr())))

    def verify(self, pred, truth, tau=None, eps: float = 1e-8):
        n_rows = pred.shape[0]
        E = pred.numel() // n_rows
        import torch
        dtype = BF16 if pred.dtype == torch.bfloat16 else F32
        assert pred.dtype == truth.dtype and pred.is_contiguous() and truth.is_contiguous()
        err = np.zeros(n_rows, np.float32); acc = np.zeros(n_rows, np.uint8)
        t = _f32(np.broadcast_to(tau, (n_rows,))) if tau is not None else None
        self._ck(self.lib.speca_verify(self.h, C.c_void_p(pred.data_ptr()), C.c_void_p(truth.data_ptr()), n_rows, E, dtype,
                                       _p(t, C.c_float) if t is not None else None, eps, _p(err, C.c_float), _p(acc, C.c_uint8)))
        return err, (acc.astype(bool) if t is not None else None)

    def verify_static(self, pred, truth, err_out, tau=None, accept_out=None, eps: float = 1e-8):
        """speca_verify_static: tau / err_out / accept_out are device tensors (fp32, fp32, uint8) of n_rows;
        nothing is allocated or synchronised by the library."""
        import torch
        n_rows = pred.shape[0]
        E = pred.numel() // n_rows
        dtype = BF16 if pred.dtype == torch.bfloat16 else F32
        assert pred.dtype == truth.dtype and pred.is_contiguous() and truth.is_contiguous()
        assert err_out.dtype == torch.float32 and err_out.numel() >= n_rows
        assert tau is None or tau.dtype == torch.float32
        assert accept_out is None or accept_out.dtype == torch.uint8
        self._ck(self.lib.speca_verify_static(self.h, C.c_void_p(pred.data_ptr()), C.c_void_p(truth.data_ptr()), n_rows, E, dtype,
                                              C.c_void_p(tau.data_ptr()) if tau is not None else None, eps,
                                              C.c_void_p(err_out.data_ptr()),
                                              C.c_void_p(accept_out.data_ptr()) if accept_out is not None else None))

    def set_lanes(self, lanes: int, profile_keeps_lanes: bool = False):
        """Row groups of a step that run side by side on streams of the library (1 = serial)."""
        self._ck(self.lib.speca_set_lanes(self.h, int(lanes), int(bool(profile_keeps_lanes))))

    def profile_begin(self):
        self._ck(self.lib.speca_profile_begin(self.h))

    def profile_end(self) -> Dict[str, dict]:
        p = Profile()
        self._ck(self.lib.speca_profile_end(self.h, C.byref(p)))
        return {name: {"launches": int(p.launches[i]), "ms": float(p.ms[i]), "flops": float(p.flops[i]), "bytes": float(p.bytes[i])}
                for i, name in enumerate(PROF_CLASSES)}

    def _cond(self, labels=None, timestep: float = 0.0, txt=None, pooled=None):
        lab = _i32(labels) if labels is not None else None
        c = Cond(_p(lab, C.c_int32) if lab is not None else None,
                 C.c_void_p(txt.data_ptr()) if txt is not None else None,
                 C.c_void_p(pooled.data_ptr()) if pooled is not None else None, float(timestep))
        return c, lab

    def full_step(self, x, step: int, rows, model_out, labels=None, timestep: float = 0.0, txt=None, pooled=None):
        r = _i32(rows)
        c, keep = self._cond(labels, timestep, txt, pooled)
        self._ck(self.lib.speca_full_step(self.h, C.c_void_p(x.data_ptr()), C.byref(c), step, _p(r, C.c_int32), len(r),
                                          C.c_void_p(model_out.data_ptr())))

    def spec_step(self, x, step: int, rows, tau, model_out, labels=None, timestep: float = 0.0, pair_stride: int = 0,
                  txt=None, pooled=None):
        r = _i32(rows)
        c, keep = self._cond(labels, timestep, txt, pooled)
        t = _f32(np.broadcast_to(tau, (len(r),)))
        err = np.zeros(len(r), np.float32); acc = np.zeros(len(r), np.uint8)
        self._ck(self.lib.speca_spec_step(self.h, C.c_void_p(x.data_ptr()), C.byref(c), step, _p(r, C.c_int32), len(r),
                                          _p(t, C.c_float), pair_stride, _p(err, C.c_float), _p(acc, C.c_uint8),
                                          C.c_void_p(model_out.data_ptr())))
        return err, acc.astype(bool)

    def sample(self, latents, timesteps, table, tau, solver_kind=SOLVER_DDIM, cfg_scale: float = 0.0, labels=None,
               txt=None, pooled=None, want_trace: bool = True, noise=None):
        """latents: fp32 device tensor [B, ...], updated in place.  noise: fp32 device tensor [S, B, ...]
        (SOLVER_DDPM).  -> dict trace."""
        B = latents.shape[0]
        ts, tb, ta = _f32(timesteps), _f32(table), _f32(tau)
        S = len(ts)
        assert len(tb) == S + 1 and len(ta) == S
        if noise is not None:
            assert noise.is_contiguous() and tuple(noise.shape) == (S,) + tuple(latents.shape) and noise.dtype == latents.dtype
        sol = Solver(solver_kind, S, _p(ts, C.c_float), _p(tb, C.c_float), float(cfg_scale),
                     C.c_void_p(noise.data_ptr()) if noise is not None else None)
        c, keep = self._cond(labels, 0.0, txt, pooled)
        kind = np.zeros((B, S), np.int8); err = np.full((B, S, 2), np.nan, np.float32)
        tr = Trace(_p(kind, C.c_int8), _p(err, C.c_float), 0, 0, 0)
        self._ck(self.lib.speca_sample(self.h, C.c_void_p(latents.data_ptr()), B, C.byref(c), C.byref(sol), _p(ta, C.c_float),
                                       C.byref(tr) if want_trace else None))
        return {"kind": kind, "err": err, "n_full": tr.n_full, "n_spec": tr.n_spec, "n_reject": tr.n_reject}


def cache_only_desc(n_slots: int, tokens: int, hidden: int, dtype: int) -> ModelDesc:
    d = ModelDesc()
    d.kind, d.dtype, d.n_slots, d.tokens, d.hidden = MODEL_NONE, dtype, n_slots, tokens, hidden
    return d


def dit_desc(shape, dtype: Optional[int] = None) -> ModelDesc:
    """shape: an object with the fields of speca_inputs.DiTShape."""
    d = ModelDesc()
    d.kind = MODEL_DIT
    d.dtype = dtype if dtype is not None else (BF16 if shape.dtype == "bf16" else F32)
    d.depth, d.depth_single = shape.depth, 0
    d.hidden, d.heads, d.mlp_hidden = shape.hidden, shape.heads, shape.mlp_hidden
    d.in_channels, d.latent_t, d.latent_h, d.latent_w, d.patch = shape.in_channels, 1, shape.latent_hw, shape.latent_hw, shape.patch
    d.num_classes, d.freq_dim = shape.num_classes, shape.freq_dim
    return d


FP32_TABLES = ("rope_cos", "rope_sin")     # tables the library reads as float32 whatever the model dtype


def to_device(arrays: Dict[str, np.ndarray], dtype: int, device="cuda") -> Dict[str, "object"]:
    """NumPy float32 arrays -> contiguous device tensors of the model dtype (exact when the
    values are already representable); the rotary tables stay float32."""
    import torch
    td = _torch_dtype(dtype)
    return {k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(device=device, dtype=torch.float32 if k in FP32_TABLES else td).contiguous()
            for k, v in arrays.items()}


def mmdit_desc(shape, dtype: Optional[int] = None) -> ModelDesc:
    """shape: an object with the fields of speca_inputs.MMDiTShape."""
    d = ModelDesc()
    d.kind = MODEL_MMDIT
    d.dtype = dtype if dtype is not None else (BF16 if shape.dtype == "bf16" else F32)
    d.depth, d.depth_single = shape.depth_dual, shape.depth_single
    d.hidden, d.heads, d.mlp_hidden = shape.hidden, shape.heads, shape.mlp_hidden
    d.in_channels, d.latent_t, d.latent_h, d.latent_w, d.patch = shape.in_channels, shape.latent_t, shape.latent_h, shape.latent_w, shape.patch
    d.freq_dim, d.txt_tokens, d.txt_dim, d.vec_dim = shape.freq_dim, shape.txt_tokens, shape.txt_dim, shape.vec_dim
    return d
