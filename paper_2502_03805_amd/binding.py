"""Thin ctypes binding of libcriticalkv.so.

Argument marshalling only: tensors are PyTorch-ROCm device buffers, every step of the
pass runs inside the library's gfx950 kernels.  There is no CPU fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

PKG = os.path.dirname(os.path.abspath(__file__))
# CRITICALKV_LIB overrides the library file (to compare two builds in one process-per-build run)
LIB_PATH = os.environ.get("CRITICALKV_LIB") or os.path.join(PKG, "libcriticalkv.so")

CKV_BF16, CKV_F32 = 0, 1
CKV_NORM_L1, CKV_NORM_L2 = 1, 2
CKV_MEAN, CKV_SUM = 0, 1
CKV_WO_OUT_IN, CKV_NO_MFMA, CKV_WO_IS_GRAM, CKV_CAUSAL_TAIL, CKV_PROTECT_WINDOW, CKV_ATTN_ONLY = 1, 2, 4, 8, 16, 32
CKV_OK, CKV_E_INVALID_ARG, CKV_E_UNSUPPORTED, CKV_E_WORKSPACE, CKV_E_HIP, CKV_E_STATIC_LIMIT = 0, -1, -2, -3, -4, -5
CKV_STATIC_SCRATCH_BYTES = 12 << 20

EXPORTS = ("criticalkv_workspace_bytes", "criticalkv_score", "criticalkv_score_profiled", "criticalkv_select",
           "criticalkv_compact", "criticalkv_strerror", "criticalkv_gram_bytes", "criticalkv_prepare_gram",
           "criticalkv_allocate", "criticalkv_diagnostics", "criticalkv_select_noalloc", "criticalkv_prepared_wo_bytes",
           "criticalkv_prepare_wo", "criticalkv_probe_mfma_bf16", "criticalkv_probe_hbm_read")
STAGES = ("wo_layout", "attn_stats", "attn_colsum", "vproj", "combine")


class LayerDesc(ctypes.Structure):
    """Mirror of ckv_layer_desc in include/criticalkv.h."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_ctx", ctypes.c_int32),
        ("window", ctypes.c_int32), ("pool_kernel", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("norm", ctypes.c_int32), ("window_reduce", ctypes.c_int32), ("flags", ctypes.c_uint32),
        ("softmax_scale", ctypes.c_float), ("eps", ctypes.c_float),
        ("k_stride", ctypes.c_int64 * 3), ("v_stride", ctypes.c_int64 * 3),
    ]


class CriticalKVError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} (code {code})")


_lib = None
_hip = None


def hip_runtime() -> ctypes.CDLL:
    """The process's single HIP runtime, made visible to libcriticalkv.so.

    libcriticalkv.so is linked without a HIP dependency so that it binds to the runtime PyTorch
    already uses: device pointers, streams and events then belong to one runtime.  PyTorch ships its
    own copy (torch/lib/libamdhip64.so); it is opened again here with RTLD_GLOBAL, which returns the
    loaded instance and exposes its symbols."""
    global _hip
    if _hip is None:
        import torch  # device memory and streams come from PyTorch; importing it first loads its HIP runtime
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        if not os.path.exists(path):
            raise ImportError(f"PyTorch-ROCm's HIP runtime not found at {path}")
        _hip = ctypes.CDLL(path, mode=ctypes.RTLD_GLOBAL)
    return _hip


def load() -> ctypes.CDLL:
    """Load the built library.  Raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2502_03805_amd.build` "
                              "(or __graft_entry__.build()) first")
        hip_runtime()
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        dp = ctypes.POINTER(LayerDesc)
        lib.criticalkv_workspace_bytes.restype = ctypes.c_size_t
        lib.criticalkv_workspace_bytes.argtypes = [dp, i32]
        lib.criticalkv_score.restype = ctypes.c_int
        lib.criticalkv_score.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.criticalkv_score_profiled.restype = ctypes.c_int
        lib.criticalkv_score_profiled.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp,
                                                  ctypes.POINTER(ctypes.c_void_p)]
        lib.criticalkv_gram_bytes.restype = ctypes.c_size_t
        lib.criticalkv_gram_bytes.argtypes = [dp]
        lib.criticalkv_prepare_gram.restype = ctypes.c_int
        lib.criticalkv_prepare_gram.argtypes = [dp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.criticalkv_select.restype = ctypes.c_int
        lib.criticalkv_select.argtypes = [dp, vp, vp, vp, f32, i32, vp, vp, vp, ctypes.c_size_t, vp]
        lib.criticalkv_select_noalloc.restype = ctypes.c_int
        lib.criticalkv_select_noalloc.argtypes = [dp, vp, vp, vp, f32, i32, vp, vp, vp]
        lib.criticalkv_prepared_wo_bytes.restype = ctypes.c_size_t
        lib.criticalkv_prepared_wo_bytes.argtypes = [dp]
        lib.criticalkv_prepare_wo.restype = ctypes.c_int
        lib.criticalkv_prepare_wo.argtypes = [dp, vp, vp, vp]
        lib.criticalkv_probe_mfma_bf16.restype = ctypes.c_int
        lib.criticalkv_probe_mfma_bf16.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), vp, vp]
        lib.criticalkv_probe_hbm_read.restype = ctypes.c_int
        lib.criticalkv_probe_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.criticalkv_allocate.restype = ctypes.c_int
        lib.criticalkv_allocate.argtypes = [dp, vp, i32, f32, vp, vp, ctypes.c_size_t, vp]
        lib.criticalkv_diagnostics.restype = ctypes.c_int
        lib.criticalkv_diagnostics.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, vp, ctypes.c_size_t, vp]
        lib.criticalkv_compact.restype = ctypes.c_int
        lib.criticalkv_compact.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp]
        lib.criticalkv_strerror.restype = ctypes.c_char_p
        lib.criticalkv_strerror.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load().criticalkv_strerror(int(code)).decode()


def make_desc(*, batch, n_q_heads, n_kv_heads, head_dim, d_model, n_ctx, window, pool_kernel, dtype,
              norm=CKV_NORM_L1, window_reduce=CKV_MEAN, flags=0, softmax_scale=0.0, eps=1e-4,
              k_stride=(0, 0, 0), v_stride=(0, 0, 0)) -> LayerDesc:
    d = LayerDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim, d.d_model = batch, n_q_heads, n_kv_heads, head_dim, d_model
    d.n_ctx, d.window, d.pool_kernel, d.dtype, d.norm = n_ctx, window, pool_kernel, dtype, norm
    d.window_reduce, d.flags, d.softmax_scale, d.eps = window_reduce, flags, softmax_scale, eps
    d.k_stride = (ctypes.c_int64 * 3)(*k_stride)
    d.v_stride = (ctypes.c_int64 * 3)(*v_stride)
    return d


def workspace_bytes(desc: LayerDesc, max_budget: int) -> int:
    return int(load().criticalkv_workspace_bytes(ctypes.byref(desc), int(max_budget)))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def criticalkv_score(desc: LayerDesc, q_win, k, v, w_o, attn, crit, vnorm=None, *, workspace, stream=None) -> None:
    rc = load().criticalkv_score(ctypes.byref(desc), _ptr(q_win), _ptr(k), _ptr(v), _ptr(w_o), _ptr(attn), _ptr(crit),
                                 _ptr(vnorm), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_score")


def gram_bytes(desc: LayerDesc) -> int:
    return int(load().criticalkv_gram_bytes(ctypes.byref(desc)))


def criticalkv_prepare_gram(desc: LayerDesc, w_o, gram_out, *, workspace, stream=None) -> None:
    rc = load().criticalkv_prepare_gram(ctypes.byref(desc), _ptr(w_o), _ptr(gram_out), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_prepare_gram")


def criticalkv_score_profiled(desc: LayerDesc, q_win, k, v, w_o, attn, crit, vnorm=None, *, workspace, stage_events,
                              stream=None) -> None:
    """stage_events: ctypes array (c_void_p * (2 * len(STAGES))) of hipEvent_t handles, NULL = skip."""
    rc = load().criticalkv_score_profiled(ctypes.byref(desc), _ptr(q_win), _ptr(k), _ptr(v), _ptr(w_o), _ptr(attn),
                                          _ptr(crit), _ptr(vnorm), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream), stage_events)
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_score_profiled")


def criticalkv_select(desc: LayerDesc, attn, crit, budget, alpha: float, max_budget: int, idx, count, *, workspace,
                      stream=None) -> None:
    rc = load().criticalkv_select(ctypes.byref(desc), _ptr(attn), _ptr(crit), _ptr(budget), float(alpha),
                                  int(max_budget), _ptr(idx), _ptr(count), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_select")


def criticalkv_select_noalloc(desc: LayerDesc, attn, crit, budget, alpha: float, max_budget: int, idx, count, *,
                              stream=None) -> None:
    rc = load().criticalkv_select_noalloc(ctypes.byref(desc), _ptr(attn), _ptr(crit), _ptr(budget), float(alpha),
                                          int(max_budget), _ptr(idx), _ptr(count), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_select_noalloc")


def prepared_wo_bytes(desc: LayerDesc) -> int:
    return int(load().criticalkv_prepared_wo_bytes(ctypes.byref(desc)))


def criticalkv_prepare_wo(desc: LayerDesc, w_o, w_out, *, stream=None) -> None:
    rc = load().criticalkv_prepare_wo(ctypes.byref(desc), _ptr(w_o), _ptr(w_out), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_prepare_wo")


def criticalkv_allocate(desc: LayerDesc, attn, total_budget: int, floor_frac: float, budget, *, workspace,
                        stream=None) -> None:
    rc = load().criticalkv_allocate(ctypes.byref(desc), _ptr(attn), int(total_budget), float(floor_frac), _ptr(budget),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_allocate")


def criticalkv_probe_mfma_bf16(operands, iters: int, sink, *, stream=None) -> float:
    """Enqueues the register-only bf16 MFMA loop; returns the launch's floating-point operation count."""
    flop = ctypes.c_double()
    rc = load().criticalkv_probe_mfma_bf16(_ptr(operands), int(iters), ctypes.byref(flop), _ptr(sink), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_probe_mfma_bf16")
    return float(flop.value)


def criticalkv_probe_hbm_read(buf, nbytes: int, sink, *, stream=None) -> None:
    rc = load().criticalkv_probe_hbm_read(_ptr(buf), int(nbytes), _ptr(sink), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_probe_hbm_read")


DIAG_FIELDS = ("sigma", "s", "C", "theta", "theta_hat", "theta_relax", "L", "M")


def criticalkv_diagnostics(desc: LayerDesc, v, w_o, vnorm_opt, idx, count, max_budget: int, out, *, workspace,
                           stream=None) -> None:
    rc = load().criticalkv_diagnostics(ctypes.byref(desc), _ptr(v), _ptr(w_o), _ptr(vnorm_opt), _ptr(idx), _ptr(count),
                                       int(max_budget), _ptr(out), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_diagnostics")


def criticalkv_compact(desc: LayerDesc, k, v, idx, count, max_budget: int, k_out, v_out, *, stream=None) -> None:
    rc = load().criticalkv_compact(ctypes.byref(desc), _ptr(k), _ptr(v), _ptr(idx), _ptr(count), int(max_budget),
                                   _ptr(k_out), _ptr(v_out), _stream(stream))
    if rc != CKV_OK:
        raise CriticalKVError(rc, "criticalkv_compact")
