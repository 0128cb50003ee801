"""Python binding of libwildcat (argument marshalling only).

Every step of CompressKV and WtdAttn runs in the HIP kernels of ``libwildcat.so``; this module turns
torch tensors into raw device pointers, fills the C structs of ``include/wildcat.h`` and allocates
outputs and the workspace with torch.  There is no CPU fallback: if the shared library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwildcat.so")

WILDCAT_F32, WILDCAT_BF16 = 0, 1
EXPORTS = ("wildcat_version", "wildcat_strerror", "wildcat_workspace_bytes", "wildcat_draw_uniforms",
           "wildcat_query_radius", "wildcat_compress_kv", "wildcat_wtd_attn", "wildcat_pack_values",
           "wildcat_rpnys_single_launch", "wildcat_loop_plan", "wildcat_query_radius_static")


class WildcatError(RuntimeError):
    pass


class _Opts(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("q_heads", ctypes.c_int32), ("kv_heads", ctypes.c_int32),
        ("m", ctypes.c_int64), ("dv", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("beta", ctypes.c_double), ("rank_tol", ctypes.c_double),
        ("r_q", ctypes.c_void_p), ("uniforms", ctypes.c_void_p),
        ("bins", ctypes.c_int32), ("tau_length", ctypes.c_int32),
        ("history", ctypes.c_int32), ("loop_driver", ctypes.c_int32),
        ("stream", ctypes.c_void_p), ("ev_loop_begin", ctypes.c_void_p), ("ev_loop_end", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("wait_limit", ctypes.c_int64),
    ]


class _Coreset(ctypes.Structure):
    _fields_ = [
        ("idx", ctypes.c_void_p), ("r_eff", ctypes.c_void_p), ("k_s", ctypes.c_void_p),
        ("v_s", ctypes.c_void_p), ("w", ctypes.c_void_p), ("v_min", ctypes.c_void_p),
        ("v_max", ctypes.c_void_p), ("tau", ctypes.c_void_p), ("v_t", ctypes.c_void_p),
        ("v_scale", ctypes.c_void_p), ("W", ctypes.c_void_p),
    ]


_lib = None


def load_library(force: bool = False):
    """Loads libwildcat.so (built in-tree by ``__graft_entry__.build()``) and declares its signatures."""
    global _lib
    if _lib is not None and not force:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise WildcatError(f"{LIB_PATH} not found: build it first (python __graft_entry__.py)")
    # torch first: it ships its own HIP runtime, and the library must bind to the runtime that owns the tensors'
    # memory and streams.  Loaded before torch, the library would pull in the system's runtime as a second one
    # in the process, and its launches would fail there (no device).
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    for name in EXPORTS:
        if not hasattr(lib, name):
            raise WildcatError(f"libwildcat.so does not export {name}")
    lib.wildcat_version.restype = ctypes.c_int
    lib.wildcat_strerror.restype = ctypes.c_char_p
    lib.wildcat_strerror.argtypes = [ctypes.c_int]
    lib.wildcat_workspace_bytes.restype = ctypes.c_size_t
    lib.wildcat_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_Opts)]
    lib.wildcat_draw_uniforms.restype = ctypes.c_int
    lib.wildcat_draw_uniforms.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_void_p]
    lib.wildcat_query_radius.restype = ctypes.c_int
    lib.wildcat_query_radius.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(_Opts),
                                         ctypes.c_void_p]
    lib.wildcat_query_radius_static.restype = ctypes.c_int
    lib.wildcat_query_radius_static.argtypes = lib.wildcat_query_radius.argtypes
    lib.wildcat_compress_kv.restype = ctypes.c_int
    lib.wildcat_compress_kv.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_uint64, ctypes.POINTER(_Opts),
                                        ctypes.POINTER(_Coreset)]
    lib.wildcat_wtd_attn.restype = ctypes.c_int
    lib.wildcat_wtd_attn.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Coreset), ctypes.c_void_p, ctypes.c_int64,
                                     ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_Opts)]
    lib.wildcat_rpnys_single_launch.restype = ctypes.c_int
    lib.wildcat_rpnys_single_launch.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_Opts)]
    lib.wildcat_loop_plan.restype = ctypes.c_int
    lib.wildcat_loop_plan.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_Opts),
                                      ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    lib.wildcat_pack_values.restype = ctypes.c_int
    lib.wildcat_pack_values.argtypes = [ctypes.POINTER(_Coreset), ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_Opts)]
    _lib = lib
    return lib


def _check(rc, what):
    if rc != 0:
        raise WildcatError(f"{what} failed: {load_library().wildcat_strerror(rc).decode()} ({rc})")


def version():
    return load_library().wildcat_version()


def draw_uniforms(seed: int, count: int):
    """The library's host-side uniform stream for `seed` (numpy float64 [count])."""
    import numpy as np
    out = np.empty(count, dtype=np.float64)
    _check(load_library().wildcat_draw_uniforms(seed, count, out.ctypes.data), "wildcat_draw_uniforms")
    return out


@dataclass
class Coreset:
    """Device buffers of the compressed cache (see wildcat_coreset in include/wildcat.h)."""
    idx: "torch.Tensor"     # [B, Hkv, r] int32
    r_eff: "torch.Tensor"   # [B, Hkv] int32
    k_s: "torch.Tensor"     # [B, Hkv, r, d] storage dtype
    v_s: "torch.Tensor"     # [B, Hkv, r, dv] float32
    w: "torch.Tensor"       # [B, Hkv, r] float32
    v_min: "torch.Tensor"   # [B, Hkv, dv] float32
    v_max: "torch.Tensor"   # [B, Hkv, dv] float32
    tau: "torch.Tensor"     # [B, Hkv] float64
    v_t: "torch.Tensor" = None      # [B, Hkv, dv, r64] float16 (bf16 storage only): v_s^T / v_scale, MFMA operand
    v_scale: "torch.Tensor" = None  # [B, Hkv] float32 power of two
    bins: int = 1                   # B of Alg. 2; r_eff and tau are [B, Hkv, bins] when bins > 1
    W: "torch.Tensor" = None        # [B, Hkv, bins, r/bins, n/bins] float64: debug output of compress_kv(weights=True)

    def c_struct(self):
        return _Coreset(self.idx.data_ptr(), self.r_eff.data_ptr() if self.r_eff is not None else None,
                        self.k_s.data_ptr(), self.v_s.data_ptr(), self.w.data_ptr(), self.v_min.data_ptr(),
                        self.v_max.data_ptr(), self.tau.data_ptr() if self.tau is not None else None,
                        self.v_t.data_ptr() if self.v_t is not None else None,
                        self.v_scale.data_ptr() if self.v_scale is not None else None,
                        self.W.data_ptr() if self.W is not None else None)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return WILDCAT_F32
    if t.dtype == torch.bfloat16:
        return WILDCAT_BF16
    raise WildcatError(f"unsupported storage dtype {t.dtype}")


def _need(t, name, ndim):
    if not t.is_cuda or not t.is_contiguous() or t.dim() != ndim:
        raise WildcatError(f"{name} must be a contiguous CUDA tensor with {ndim} dims")


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _opts(batch, q_heads, kv_heads, m, dv, dtype, beta, rank_tol=0.0, r_q=None, uniforms=None, workspace=None):
    o = _Opts()
    o.batch, o.q_heads, o.kv_heads, o.m, o.dv, o.dtype = batch, q_heads, kv_heads, m, dv, dtype
    o.beta = 0.0 if beta is None else float(beta)
    o.rank_tol = float(rank_tol)
    o.r_q = r_q.data_ptr() if r_q is not None else None
    o.uniforms = uniforms.data_ptr() if uniforms is not None else None
    o.stream = _stream()
    if workspace is not None:
        o.workspace, o.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    return o


def _history_code(history):
    if history not in ("f64", "f32"):
        raise WildcatError("history is 'f64' or 'f32'")
    return int(history == "f32")


_LOOPS = {"auto": 0, "steps": 1, "wave": 2}


def _loop_code(loop):
    if loop not in _LOOPS:
        raise WildcatError("loop is 'auto', 'steps' or 'wave'")
    return _LOOPS[loop]


def _shape_opts(batch, kv_heads, dv, dtype, bins, history, loop):
    o = _Opts()
    o.batch, o.kv_heads, o.dv, o.dtype, o.bins = batch, kv_heads, dv, dtype, bins
    o.history, o.loop_driver = _history_code(history), _loop_code(loop)
    return o


def workspace_bytes(n, d, r, batch=1, kv_heads=1, dv=0, dtype=WILDCAT_BF16, bins=1, history="f64"):
    o = _shape_opts(batch, kv_heads, dv, dtype, bins, history, "auto")
    return load_library().wildcat_workspace_bytes(n, d, r, ctypes.byref(o))


def rpnys_single_launch(n, d, r, batch=1, kv_heads=1, dv=0, dtype=WILDCAT_BF16, bins=1, history="f64", loop="auto"):
    """True if compress_kv runs the selection loop of this shape with all steps inside a launch (needs a GPU)."""
    o = _shape_opts(batch, kv_heads, dv, dtype, bins, history, loop)
    rc = load_library().wildcat_rpnys_single_launch(n, d, r, ctypes.byref(o))
    if rc < 0:
        _check(rc, "wildcat_rpnys_single_launch")
    return bool(rc)


LOOP_PLAN_FIELDS = ("driver", "keys_per_thread", "slabs", "problems_per_launch", "launches", "keys_in_registers",
                    "workgroups_per_cu", "reserved")


def loop_plan(n, d, r, batch=1, kv_heads=1, dv=0, dtype=WILDCAT_BF16, bins=1, history="f64", loop="auto",
              compute_units=0, occ_resident_keys=0, occ_streamed_keys=0):
    """wildcat_loop_plan as a dict (see include/wildcat.h).  compute_units = 0: the current device (needs a GPU);
    > 0: pure host logic for a device with the given capacities."""
    o = _shape_opts(batch, kv_heads, dv, dtype, bins, history, loop)
    out = (ctypes.c_int32 * 8)()
    _check(load_library().wildcat_loop_plan(n, d, r, ctypes.byref(o), compute_units, occ_resident_keys,
                                            occ_streamed_keys, out), "wildcat_loop_plan")
    return dict(zip(LOOP_PLAN_FIELDS, (int(x) for x in out)))


def query_radius(Q, kv_heads=None, workspace=None):
    """R_Q of Alg. 4 per (batch, kv_head): float64 tensor [B, Hkv].  Q: [B, Hq, m, d].  `workspace`: optional
    uint8 device tensor used as scratch (any later call on the stream may overwrite it)."""
    import torch
    _need(Q, "Q", 4)
    B, Hq, m, d = Q.shape
    kv_heads = kv_heads or Hq
    out = torch.empty((B, kv_heads), dtype=torch.float64, device=Q.device)
    o = _opts(B, Hq, kv_heads, m, 0, _dtype_code(Q), None, workspace=workspace)
    _check(load_library().wildcat_query_radius(Q.data_ptr(), m, d, ctypes.byref(o), out.data_ptr()),
           "wildcat_query_radius")
    return out


def query_radius_static(Q, kv_heads=None, out=None):
    """wildcat_query_radius_static: R_Q with the library's own scratch (no workspace; see include/wildcat.h).  `out`:
    optional float64 [B, Hkv] device tensor to write into (then nothing at all is allocated here either)."""
    import torch
    _need(Q, "Q", 4)
    B, Hq, m, d = Q.shape
    kv_heads = kv_heads or Hq
    if out is None:
        out = torch.empty((B, kv_heads), dtype=torch.float64, device=Q.device)
    o = _opts(B, Hq, kv_heads, m, 0, _dtype_code(Q), None)
    _check(load_library().wildcat_query_radius_static(Q.data_ptr(), m, d, ctypes.byref(o), out.data_ptr()),
           "wildcat_query_radius_static")
    return out


def compress_kv(K, V, r, r_q, seed=0, uniforms=None, beta=None, rank_tol=0.0, workspace=None, loop_events=None,
                bins=1, temperature_n="bin", history="f64", loop="auto", wait_limit=0, weights=False):
    """CompressKV (Alg. 2).  K: [B, Hkv, n, d], V: [B, Hkv, n, dv]; r_q: float64 [B, Hkv] on the device;
    uniforms: optional float64 [B*Hkv, r] on the device (else drawn from `seed`); loop_events: optional pair
    of raw hipEvent_t handles recorded around the RPNys loop; bins: B of Alg. 2 (must divide n and r);
    temperature_n: "bin" (length n/B in the temperature) or "full" (n); history: "f64" (pivots identical to a
    float64 reference) or "f32" (fast mode, see wildcat_history in include/wildcat.h); loop: "auto", "steps" or
    "wave" (wildcat_loop); wait_limit: see wildcat_opts; weights: also return the Nystrom weights W per bin in
    Coreset.W (debug output, see wildcat_coreset.W).  Returns a Coreset."""
    import torch
    _need(K, "K", 4)
    _need(V, "V", 4)
    B, H, n, d = K.shape
    dv = V.shape[3]
    if V.shape[:3] != K.shape[:3] or V.dtype != K.dtype:
        raise WildcatError("K and V must agree in batch, heads, length and dtype")
    if r_q.dtype != torch.float64 or r_q.numel() != B * H or not r_q.is_cuda:
        raise WildcatError("r_q must be a float64 CUDA tensor with batch*kv_heads entries")
    if uniforms is not None and (uniforms.dtype != torch.float64 or uniforms.numel() != B * H * r
                                 or not uniforms.is_cuda or not uniforms.is_contiguous()):
        raise WildcatError("uniforms must be a contiguous float64 CUDA tensor with batch*kv_heads*r entries")
    code = _dtype_code(K)
    dev = K.device
    if temperature_n not in ("bin", "full"):
        raise WildcatError("temperature_n is 'bin' or 'full'")
    bins = max(int(bins), 1)
    need = workspace_bytes(n, d, r, B, H, dv, code, bins, history)
    if need == 0:
        raise WildcatError("wildcat_workspace_bytes rejected the shape")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    cs = Coreset(
        idx=torch.empty((B, H, r), dtype=torch.int32, device=dev),
        r_eff=torch.empty((B, H) if bins == 1 else (B, H, bins), dtype=torch.int32, device=dev),
        k_s=torch.empty((B, H, r, d), dtype=K.dtype, device=dev),
        v_s=torch.empty((B, H, r, dv), dtype=torch.float32, device=dev),
        w=torch.empty((B, H, r), dtype=torch.float32, device=dev),
        v_min=torch.empty((B, H, dv), dtype=torch.float32, device=dev),
        v_max=torch.empty((B, H, dv), dtype=torch.float32, device=dev),
        tau=torch.empty((B, H) if bins == 1 else (B, H, bins), dtype=torch.float64, device=dev),
        v_t=(torch.empty((B, H, dv, (r + 63) // 64 * 64), dtype=torch.float16, device=dev)
             if code == WILDCAT_BF16 else None),
        v_scale=torch.empty((B, H), dtype=torch.float32, device=dev) if code == WILDCAT_BF16 else None,
        bins=bins,
        W=torch.empty((B, H, bins, r // bins, n // bins), dtype=torch.float64, device=dev) if weights else None,
    )
    o = _opts(B, H, H, n, dv, code, beta, rank_tol, r_q.contiguous(), uniforms, workspace)
    o.bins, o.tau_length, o.history = bins, int(temperature_n == "full"), _history_code(history)
    o.loop_driver, o.wait_limit = _loop_code(loop), int(wait_limit)
    if loop_events is not None:
        o.ev_loop_begin, o.ev_loop_end = loop_events
    c = cs.c_struct()
    _check(load_library().wildcat_compress_kv(K.data_ptr(), V.data_ptr(), n, d, r, seed, ctypes.byref(o),
                                              ctypes.byref(c)), "wildcat_compress_kv")
    return cs


def pack_values(cs: Coreset):
    """Allocates (if needed) and fills cs.v_t, cs.v_scale from cs.v_s: for coresets assembled by hand (bf16 storage)."""
    import torch
    B, H, r, dv = cs.v_s.shape
    if cs.v_t is None:
        cs.v_t = torch.empty((B, H, dv, (r + 63) // 64 * 64), dtype=torch.float16, device=cs.v_s.device)
    if cs.v_scale is None:
        cs.v_scale = torch.empty((B, H), dtype=torch.float32, device=cs.v_s.device)
    o = _opts(B, H, H, 0, dv, WILDCAT_BF16, None)
    c = cs.c_struct()
    _check(load_library().wildcat_pack_values(ctypes.byref(c), r, dv, ctypes.byref(o)), "wildcat_pack_values")
    return cs


def wtd_attn(Q, cs: Coreset, beta=None, out=None):
    """WtdAttn (Alg. 3).  Q: [B, Hq, m, d]; returns [B, Hq, m, dv] in Q's dtype."""
    import torch
    _need(Q, "Q", 4)
    B, Hq, m, d = Q.shape
    Hkv, r, dv = cs.k_s.shape[1], cs.k_s.shape[2], cs.v_s.shape[3]
    if cs.k_s.dtype != Q.dtype or cs.k_s.shape[0] != B or cs.k_s.shape[3] != d:
        raise WildcatError("coreset does not match Q")
    if out is None:
        out = torch.empty((B, Hq, m, dv), dtype=Q.dtype, device=Q.device)
    o = _opts(B, Hq, Hkv, m, dv, _dtype_code(Q), beta)
    o.bins = cs.bins
    c = cs.c_struct()
    _check(load_library().wildcat_wtd_attn(Q.data_ptr(), ctypes.byref(c), out.data_ptr(), m, d, r, ctypes.byref(o)),
           "wildcat_wtd_attn")
    return out


def wildcat(Q, K, V, r, seed=0, uniforms=None, beta=None, rank_tol=0.0, workspace=None, return_coreset=False,
            bins=1, temperature_n="bin", history="f64", loop="auto", wait_limit=0):
    """WildCat (Alg. 4): query radius, CompressKV, WtdAttn."""
    if workspace is None:
        import torch
        bins_ = max(int(bins), 1)
        need = workspace_bytes(K.shape[2], K.shape[3], r, K.shape[0], K.shape[1], V.shape[3], _dtype_code(K), bins_,
                               history)
        if need == 0:
            raise WildcatError("wildcat_workspace_bytes rejected the shape")
        workspace = torch.empty(need, dtype=torch.uint8, device=K.device)
    r_q = query_radius(Q, K.shape[1], workspace=workspace)
    cs = compress_kv(K, V, r, r_q, seed=seed, uniforms=uniforms, beta=beta, rank_tol=rank_tol, workspace=workspace,
                     bins=bins, temperature_n=temperature_n, history=history, loop=loop, wait_limit=wait_limit)
    out = wtd_attn(Q, cs, beta=beta)
    return (out, cs) if return_coreset else out
