"""ctypes binding over libcoreinfer.so -- argument marshalling only.

Function names mirror the C ABI (include/coreinfer.h).  Tensors are torch
tensors on the GPU; torch supplies device memory and the current stream,
every step of the path runs in the library's own HIP kernels.  There is no
fallback: if the library is missing, importing this module raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported first so that the HIP runtime torch ships is the one the library binds to

from .build import LIB_PATH

CI_OK = 0
CI_ERR_INVALID_ARG = -1
CI_ERR_BAD_DTYPE = -2
CI_ERR_BAD_LAYOUT = -3
CI_ERR_WORKSPACE = -4
CI_ERR_HIP = -5
CI_ERR_UNSUPPORTED = -6

CI_F32, CI_F16, CI_BF16 = 0, 1, 2
CI_ACT_RELU, CI_ACT_SWIGLU = 0, 1
CI_DOWN_OUT_MAJOR, CI_DOWN_NEURON_MAJOR = 0, 1

DTYPE_CODE = {torch.float32: CI_F32, torch.float16: CI_F16, torch.bfloat16: CI_BF16}
ACT_CODE = {"relu": CI_ACT_RELU, "swiglu": CI_ACT_SWIGLU}
LAYOUT_CODE = {"out_major": CI_DOWN_OUT_MAJOR, "neuron_major": CI_DOWN_NEURON_MAJOR}

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built; run `python -m paper_2410_18311_amd.build` "
        "(there is no CPU or PyTorch fallback for the CoreInfer kernels)")

_lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _int, _dbl, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_size_t


class ci_ffn_weights(ctypes.Structure):
    _fields_ = [("w_up", _vp), ("w_gate", _vp), ("b_up", _vp), ("w_down", _vp), ("b_down", _vp),
                ("core_idx", _vp), ("K", _i64), ("d", _i64), ("N", _i64), ("ld_down", _i64),
                ("down_layout", ctypes.c_int32)]


_SIGNATURES = {
    "coreinfer_strerror": (ctypes.c_char_p, [_int]),
    "coreinfer_version": (_int, []),
    "coreinfer_keep_count": (_int, [_dbl, _i64, ctypes.POINTER(_i64)]),
    "coreinfer_select_workspace_size": (_int, [_i64, _i64, ctypes.POINTER(_sz)]),
    "coreinfer_select": (_int, [_vp, _i64, _i64, _i64, _dbl, _dbl, _vp, _vp, _vp, _sz, _vp]),
    "coreinfer_select_batch_workspace_size": (_int, [_i64, _i64, _i64, ctypes.POINTER(_sz)]),
    "coreinfer_select_batch": (_int, [_vp, _i64, _i64, _i64, _i64, _dbl, _dbl, _vp, _vp, _vp, _sz, _vp]),
    "coreinfer_select_hidden": (_int, [_vp, _int, _int, _i64, _i64, _i64, _dbl, _dbl, _vp, _vp, _vp, _sz, _vp]),
    "coreinfer_count_tokens": (_int, [_vp, _i64, _i64, _i64, _dbl, _vp, _int, _vp, _sz, _vp]),
    "coreinfer_count_select": (_int, [_vp, _i64, _i64, _dbl, _vp, _vp, _sz, _vp]),
    "coreinfer_group_select": (_int, [_vp, _i64, _i64, _i64, _dbl, _vp, _vp, _vp, _sz, _vp]),
    "coreinfer_core_similarity": (_int, [_vp, _i64, _vp, _i64, _vp, _vp]),
    "coreinfer_assign_group": (_int, [_vp, _i64, _vp, _i64, _i64, _vp, _vp, _vp]),
    "coreinfer_assign_centroid_workspace_size": (_int, [_i64, ctypes.POINTER(_sz)]),
    "coreinfer_assign_centroid": (_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp, _sz, _vp]),
    "coreinfer_compact_down_ld": (_int, [_i64, _int, ctypes.POINTER(_i64)]),
    "coreinfer_compact_preferred_layout": (_int, [_i64, _i64, _int, _int, ctypes.POINTER(_int)]),
    "coreinfer_compact": (_int, [_vp, _vp, _vp, _vp, _int, _int, _int, _i64, _i64, _vp, _i64,
                                 _vp, _vp, _vp, _vp, _int, _vp, _vp]),
    "coreinfer_compact_update_workspace_size": (_int, [_i64, _i64, ctypes.POINTER(_sz)]),
    "coreinfer_compact_update": (_int, [_vp, _vp, _vp, _vp, _int, _int, _int, _i64, _i64, _vp, _i64, _vp,
                                        _vp, _vp, _vp, _vp, _int, _vp, _vp, _sz, _vp]),
    "coreinfer_ffn_decode_workspace_size": (_int, [_i64, _i64, _i64, ctypes.POINTER(_sz)]),
    "coreinfer_ffn_decode": (_int, [_vp, _i64, ctypes.POINTER(ci_ffn_weights), _int, _int, _vp,
                                    _vp, _sz, _vp]),
    "coreinfer_ffn_decode_status": (_int, [_vp, _vp, _vp]),
    "coreinfer_ffn_decode_static": (_int, [_vp, _i64, ctypes.POINTER(ci_ffn_weights), _int, _int, _vp, _vp, _vp]),
    "coreinfer_union_workspace_size": (_int, [_i64, ctypes.POINTER(_sz)]),
    "coreinfer_union_build": (_int, [_vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]),
    "coreinfer_ffn_decode_union_workspace_size": (_int, [_i64, _i64, _i64, _int, _int, ctypes.POINTER(_sz)]),
    "coreinfer_ffn_decode_union": (_int, [_vp, _i64, ctypes.POINTER(ci_ffn_weights), _vp, _vp, _vp, _i64,
                                          _int, _int, _vp, _vp, _sz, _vp]),
    "coreinfer_ffn_dense_hidden_workspace_size": (_int, [_i64, _i64, _i64, _int, ctypes.POINTER(_sz)]),
    "coreinfer_ffn_dense_hidden": (_int, [_vp, _i64, _vp, _vp, _vp, _vp, _vp, _int, _int, _int, _i64, _i64, _vp, _vp,
                                          _vp, _sz, _vp]),
    "coreinfer_ffn_dense_workspace_size": (_int, [_i64, _i64, _i64, _int, ctypes.POINTER(_sz)]),
    "coreinfer_ffn_dense": (_int, [_vp, _i64, _vp, _vp, _vp, _vp, _vp, _int, _int, _int, _i64, _i64,
                                   _vp, _vp, _vp, _sz, _vp]),
}
for _name, (_res, _args) in _SIGNATURES.items():
    _f = getattr(_lib, _name)
    _f.restype, _f.argtypes = _res, _args

EXPORTS = tuple(_SIGNATURES)
raw = _lib  # the bare C entry points, for tests of the error paths

# development hook (csrc/coreinfer_dev.h): launch-shape parameters for sweeps, not part of the interface
_lib.coreinfer_dev_set_param.restype = _int
_lib.coreinfer_dev_set_param.argtypes = [ctypes.c_char_p, _int]
_lib.coreinfer_dev_fused_plan.restype = _int
_lib.coreinfer_dev_fused_plan.argtypes = [_i64, _i64, _int, _int, ctypes.POINTER(_int)]
_lib.coreinfer_dev_stream_probe.restype = _int
_lib.coreinfer_dev_stream_probe.argtypes = [_vp, _i64, _i64, _int, _int, _int, _int, _int, _vp, _vp]
_lib.coreinfer_dev_tile_probe.restype = _int
_lib.coreinfer_dev_tile_probe.argtypes = [_vp, _i64, _i64, _int, _int, _int, _int, _int, _vp, _vp]


class CoreInferError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


def _check(status: int, where: str):
    if status != CI_OK:
        raise CoreInferError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream(t: torch.Tensor):
    return torch.cuda.current_stream(t.device).cuda_stream if t.is_cuda else None


def _workspace(nbytes: int, like: torch.Tensor) -> torch.Tensor:
    return torch.empty(nbytes, dtype=torch.uint8, device=like.device)


def strerror(status: int) -> str:
    return _lib.coreinfer_strerror(status).decode()


def version() -> int:
    return _lib.coreinfer_version()


def dev_set_param(name: str, value: int) -> None:
    _check(_lib.coreinfer_dev_set_param(name.encode(), int(value)), "coreinfer_dev_set_param")


def dev_fused_plan(K: int, d: int, dtype: torch.dtype, act: str) -> dict:
    """Launch shape of the single-launch decode under the current development settings."""
    out = (_int * 5)()
    _check(_lib.coreinfer_dev_fused_plan(K, d, DTYPE_CODE[dtype], ACT_CODE[act], out), "coreinfer_dev_fused_plan")
    return dict(zip(("chunks", "chunk_neurons", "compute_waves", "loads_per_row", "workgroups"), list(out)))


def dev_stream_probe(buf: torch.Tensor, window_bytes: int, per_workgroup: bool, workgroups: int, threads: int,
                     depth: int, iters: int, out: torch.Tensor) -> None:
    """Measurement aid: streams 16-byte loads over windows of `buf` (see csrc/coreinfer_dev.h)."""
    _check(_lib.coreinfer_dev_stream_probe(_ptr(buf), buf.numel() * buf.element_size(), int(window_bytes),
                                           int(bool(per_workgroup)), int(workgroups), int(threads), int(depth),
                                           int(iters), _ptr(out), _stream(buf)), "coreinfer_dev_stream_probe")


def dev_tile_probe(buf: torch.Tensor, pitch_bytes: int, shared: bool, workgroups: int, depth: int, ksteps: int,
                   iters: int, out: torch.Tensor) -> None:
    """Measurement aid: the load stream of a GEMM operand tile (see csrc/coreinfer_dev.h)."""
    _check(_lib.coreinfer_dev_tile_probe(_ptr(buf), buf.numel() * buf.element_size(), int(pitch_bytes),
                                         int(bool(shared)), int(workgroups), int(depth), int(ksteps), int(iters),
                                         _ptr(out), _stream(buf)), "coreinfer_dev_tile_probe")


def keep_count(frac: float, n: int) -> int:
    k = _i64(0)
    _check(_lib.coreinfer_keep_count(float(frac), int(n), ctypes.byref(k)), "coreinfer_keep_count")
    return k.value


def select_workspace_size(M: int, N: int) -> int:
    b = _sz(0)
    _check(_lib.coreinfer_select_workspace_size(M, N, ctypes.byref(b)), "coreinfer_select_workspace_size")
    return b.value


def select(act: torch.Tensor, alpha: float, beta: float, core_idx: Optional[torch.Tensor] = None,
           counts: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """coreinfer_select on A [M, N] fp32 (device).  Returns (core_idx, counts)."""
    assert act.dim() == 2 and act.dtype == torch.float32 and act.stride(1) == 1
    M, N = act.shape
    K = keep_count(beta, N)
    if core_idx is None:
        core_idx = torch.empty(K, dtype=torch.int32, device=act.device)
    if counts is None:
        counts = torch.empty(N, dtype=torch.int32, device=act.device)
    if ws is None:
        ws = _workspace(select_workspace_size(M, N), act)
    _check(_lib.coreinfer_select(_ptr(act), M, N, act.stride(0), float(alpha), float(beta),
                                 _ptr(core_idx), _ptr(counts), _ptr(ws), ws.numel(), _stream(act)),
           "coreinfer_select")
    return core_idx, counts


def select_batch_workspace_size(B: int, M: int, N: int) -> int:
    b = _sz(0)
    _check(_lib.coreinfer_select_batch_workspace_size(B, M, N, ctypes.byref(b)), "coreinfer_select_batch_workspace_size")
    return b.value


def select_batch(act: torch.Tensor, B: int, alpha: float, beta: float, core_idx: Optional[torch.Tensor] = None,
                 counts: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """coreinfer_select_batch on act [B * M, N] (fp32): returns (core_idx [B, K], counts [B, N])."""
    BM, N = act.shape
    M = BM // B
    assert M * B == BM
    K = keep_count(beta, N)
    if core_idx is None:
        core_idx = torch.empty((B, K), dtype=torch.int32, device=act.device)
    if counts is None:
        counts = torch.empty((B, N), dtype=torch.int32, device=act.device)
    if ws is None:
        ws = _workspace(select_batch_workspace_size(B, M, N), act)
    _check(_lib.coreinfer_select_batch(_ptr(act), B, M, N, act.stride(0), float(alpha), float(beta), _ptr(core_idx),
                                       _ptr(counts), _ptr(ws), ws.numel(), _stream(act)), "coreinfer_select_batch")
    return core_idx, counts


def select_hidden(hidden: torch.Tensor, act: str, alpha: float, beta: float,
                  core_idx: Optional[torch.Tensor] = None, counts: Optional[torch.Tensor] = None,
                  ws: Optional[torch.Tensor] = None):
    """coreinfer_select_hidden on H [M, N] of the layer's element type.  Returns (core_idx, counts)."""
    assert hidden.dim() == 2 and hidden.stride(1) == 1
    M, N = hidden.shape
    K = keep_count(beta, N)
    if core_idx is None:
        core_idx = torch.empty(K, dtype=torch.int32, device=hidden.device)
    if counts is None:
        counts = torch.empty(N, dtype=torch.int32, device=hidden.device)
    if ws is None:
        ws = _workspace(select_workspace_size(M, N), hidden)
    _check(_lib.coreinfer_select_hidden(_ptr(hidden), DTYPE_CODE[hidden.dtype], ACT_CODE[act], M, N,
                                        hidden.stride(0), float(alpha), float(beta), _ptr(core_idx),
                                        _ptr(counts), _ptr(ws), ws.numel(), _stream(hidden)),
           "coreinfer_select_hidden")
    return core_idx, counts


def count_tokens(act: torch.Tensor, alpha: float, counts: Optional[torch.Tensor] = None,
                 accumulate: bool = False, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_count_tokens: Eq. 3 over the rows of act, optionally added to existing counts."""
    assert act.dim() == 2 and act.dtype == torch.float32 and act.stride(1) == 1
    M, N = act.shape
    if counts is None:
        assert not accumulate
        counts = torch.empty(N, dtype=torch.int32, device=act.device)
    if ws is None:
        ws = _workspace(select_workspace_size(M, N), act)
    _check(_lib.coreinfer_count_tokens(_ptr(act), M, N, act.stride(0), float(alpha), _ptr(counts),
                                       1 if accumulate else 0, _ptr(ws), ws.numel(), _stream(act)),
           "coreinfer_count_tokens")
    return counts


def count_select(counts: torch.Tensor, max_count: int, beta: float,
                 core_idx: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_count_select: Def. 2 on given counts."""
    N = counts.numel()
    if core_idx is None:
        core_idx = torch.empty(keep_count(beta, N), dtype=torch.int32, device=counts.device)
    if ws is None:
        ws = _workspace(256, counts)
    _check(_lib.coreinfer_count_select(_ptr(counts), N, int(max_count), float(beta), _ptr(core_idx),
                                       _ptr(ws), ws.numel(), _stream(counts)), "coreinfer_count_select")
    return core_idx


def group_select(core_sets: torch.Tensor, N: int, gamma: float, core_idx: Optional[torch.Tensor] = None,
                 counts: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """coreinfer_group_select on core_sets [G, K] int32.  Returns (core_idx, counts)."""
    assert core_sets.dim() == 2 and core_sets.dtype == torch.int32 and core_sets.is_contiguous()
    G, K = core_sets.shape
    if core_idx is None:
        core_idx = torch.empty(keep_count(gamma, N), dtype=torch.int32, device=core_sets.device)
    if counts is None:
        counts = torch.empty(N, dtype=torch.int32, device=core_sets.device)
    if ws is None:
        ws = _workspace(select_workspace_size(G, N), core_sets)
    _check(_lib.coreinfer_group_select(_ptr(core_sets), G, K, N, float(gamma), _ptr(core_idx), _ptr(counts),
                                       _ptr(ws), ws.numel(), _stream(core_sets)), "coreinfer_group_select")
    return core_idx, counts


def core_similarity(set_a: torch.Tensor, set_b: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_core_similarity.  Returns the device tensor [identical, involved]."""
    if out is None:
        out = torch.empty(2, dtype=torch.int32, device=set_a.device)
    _check(_lib.coreinfer_core_similarity(_ptr(set_a), set_a.numel(), _ptr(set_b), set_b.numel(), _ptr(out),
                                          _stream(set_a)), "coreinfer_core_similarity")
    return out


def assign_group(prompt_set: torch.Tensor, group_sets: torch.Tensor):
    """coreinfer_assign_group.  Returns (best [1] int32, inter_union [G, 2] int32) on the device."""
    G, Kg = group_sets.shape
    best = torch.empty(1, dtype=torch.int32, device=group_sets.device)
    iu = torch.empty((G, 2), dtype=torch.int32, device=group_sets.device)
    _check(_lib.coreinfer_assign_group(_ptr(prompt_set), prompt_set.numel(), _ptr(group_sets), G, Kg,
                                       _ptr(best), _ptr(iu), _stream(group_sets)), "coreinfer_assign_group")
    return best, iu


def assign_centroid(act: torch.Tensor, centroids: torch.Tensor, ws: Optional[torch.Tensor] = None):
    """coreinfer_assign_centroid on A [M, N] fp32 and centroids [G, N] fp32 (device).
    Returns (best [1] int32, dist [G] fp32, feature [N] fp32 = a view of the workspace)."""
    M, N = act.shape
    G = centroids.shape[0]
    if ws is None:
        b = _sz(0)
        _check(_lib.coreinfer_assign_centroid_workspace_size(N, ctypes.byref(b)),
               "coreinfer_assign_centroid_workspace_size")
        ws = torch.empty(b.value, dtype=torch.uint8, device=act.device)
    best = torch.empty(1, dtype=torch.int32, device=act.device)
    dist = torch.empty(G, dtype=torch.float32, device=act.device)
    _check(_lib.coreinfer_assign_centroid(_ptr(act), M, N, act.stride(0), _ptr(centroids), G, _ptr(best),
                                          _ptr(dist), _ptr(ws), ws.numel(), _stream(act)),
           "coreinfer_assign_centroid")
    return best, dist, ws[:N * 4].view(torch.float32)


def compact_down_ld(K: int, dtype: torch.dtype) -> int:
    ld = _i64(0)
    _check(_lib.coreinfer_compact_down_ld(int(K), DTYPE_CODE[dtype], ctypes.byref(ld)), "coreinfer_compact_down_ld")
    return ld.value


def compact_preferred_layout(K: int, d: int, dtype: torch.dtype, act: str) -> str:
    out = _int(0)
    _check(_lib.coreinfer_compact_preferred_layout(int(K), int(d), DTYPE_CODE[dtype], ACT_CODE[act], ctypes.byref(out)),
           "coreinfer_compact_preferred_layout")
    return "out_major" if out.value == CI_DOWN_OUT_MAJOR else "neuron_major"


def compact_buffers(K: int, d: int, dtype: torch.dtype, device, gate: bool, bias: bool,
                    down_c_layout: str = "neuron_major") -> dict:
    """Uninitialised compact buffers for coreinfer_compact; `down_c_layout` is recorded in the dict."""
    ld = compact_down_ld(K, dtype)
    down_shape = (K, d) if down_c_layout == "neuron_major" else (d, ld)
    # with an output-major down matrix the bias buffer is padded to whole 16-byte vectors as well
    nb = K if down_c_layout == "neuron_major" else ld
    return {"w_up_c": torch.empty((K, d), dtype=dtype, device=device),
            "w_gate_c": torch.empty((K, d), dtype=dtype, device=device) if gate else None,
            "b_up_c": torch.zeros((nb,), dtype=dtype, device=device) if bias else None,
            "w_down_c": torch.empty(down_shape, dtype=dtype, device=device),
            "down_c_layout": down_c_layout}


def compact(w_up, w_gate, b_up, w_down, down_layout: str, act: str, core_idx: torch.Tensor,
            out: Optional[dict] = None, status: Optional[torch.Tensor] = None,
            down_c_layout: Optional[str] = None) -> dict:
    """coreinfer_compact.  Returns the dict of compact buffers (allocated when `out` is not
    given): w_up_c, w_gate_c, b_up_c [K, ...] and w_down_c, [K, d] ("neuron_major", the
    default) or [d, ld] ("out_major"); the dict also records "down_c_layout"."""
    N, d = w_up.shape
    K = core_idx.numel()
    if out is None:
        out = compact_buffers(K, d, w_up.dtype, w_up.device, w_gate is not None, b_up is not None,
                              down_c_layout or "neuron_major")
    layout_c = out.get("down_c_layout", "neuron_major")
    assert down_c_layout is None or down_c_layout == layout_c
    _check(_lib.coreinfer_compact(_ptr(w_up), _ptr(w_gate), _ptr(b_up), _ptr(w_down),
                                  LAYOUT_CODE[down_layout], DTYPE_CODE[w_up.dtype], ACT_CODE[act],
                                  d, N, _ptr(core_idx), K, _ptr(out["w_up_c"]), _ptr(out["w_gate_c"]),
                                  _ptr(out["b_up_c"]), _ptr(out["w_down_c"]), LAYOUT_CODE[layout_c],
                                  _ptr(status), _stream(w_up)),
           "coreinfer_compact")
    return out


def compact_update(w_up, w_gate, b_up, w_down, down_layout: str, act: str, new_idx: torch.Tensor,
                   slot_idx: torch.Tensor, bufs: dict, changed: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_compact_update: `bufs` (from compact) and `slot_idx` are changed in place.
    Returns the device int32 [1] holding the number of rows rewritten."""
    N, d = w_up.shape
    K = new_idx.numel()
    if changed is None:
        changed = torch.zeros(1, dtype=torch.int32, device=w_up.device)
    b = _sz(0)
    _check(_lib.coreinfer_compact_update_workspace_size(N, K, ctypes.byref(b)),
           "coreinfer_compact_update_workspace_size")
    ws = _workspace(b.value, w_up)
    _check(_lib.coreinfer_compact_update(_ptr(w_up), _ptr(w_gate), _ptr(b_up), _ptr(w_down),
                                         LAYOUT_CODE[down_layout], DTYPE_CODE[w_up.dtype], ACT_CODE[act],
                                         d, N, _ptr(new_idx), K, _ptr(slot_idx), _ptr(bufs["w_up_c"]),
                                         _ptr(bufs["w_gate_c"]), _ptr(bufs["b_up_c"]), _ptr(bufs["w_down_c"]),
                                         LAYOUT_CODE[bufs.get("down_c_layout", "neuron_major")],
                                         _ptr(changed), _ptr(ws), ws.numel(), _stream(w_up)),
           "coreinfer_compact_update")
    return changed


def ffn_decode_workspace_size(B: int, K: int, d: int) -> int:
    b = _sz(0)
    _check(_lib.coreinfer_ffn_decode_workspace_size(B, K, d, ctypes.byref(b)),
           "coreinfer_ffn_decode_workspace_size")
    return b.value


def make_weights(w_up, w_gate, b_up, w_down, b_down, core_idx=None, K: Optional[int] = None,
                 down_layout: str = "neuron_major") -> ci_ffn_weights:
    """Fills the ci_ffn_weights descriptor.  Compacted: pass the [K, d] buffers and, for an
    output-major compact down matrix [d, ld], down_layout="out_major".  Gathered: pass the
    resident neuron-major [N, d] weights and core_idx [B, K]."""
    rows, d = w_up.shape
    if core_idx is None:
        K = rows if K is None else K
    else:
        K = core_idx.shape[-1]
    ld = w_down.shape[1] if (w_down is not None and down_layout == "out_major") else 0
    return ci_ffn_weights(_ptr(w_up), _ptr(w_gate), _ptr(b_up), _ptr(w_down), _ptr(b_down),
                          _ptr(core_idx), K, d, rows, ld, LAYOUT_CODE[down_layout])


def make_compact_weights(bufs: dict, b_down) -> ci_ffn_weights:
    """Descriptor over the buffers coreinfer_compact wrote (either layout of w_down_c)."""
    return make_weights(bufs["w_up_c"], bufs["w_gate_c"], bufs["b_up_c"], bufs["w_down_c"], b_down,
                        down_layout=bufs.get("down_c_layout", "neuron_major"))


def decode_workspace(B: int, K: int, d: int, device) -> torch.Tensor:
    """A zeroed workspace for coreinfer_ffn_decode (the single-launch path needs it zeroed once)."""
    return torch.zeros(ffn_decode_workspace_size(B, K, d), dtype=torch.uint8, device=device)


def ffn_decode_status(ws: torch.Tensor) -> int:
    """coreinfer_ffn_decode_status, synchronised: 0, or 1 if a single-launch decode gave up waiting."""
    out = torch.zeros(1, dtype=torch.int32, device=ws.device)
    _check(_lib.coreinfer_ffn_decode_status(_ptr(ws), _ptr(out), _stream(ws)), "coreinfer_ffn_decode_status")
    return int(out.item())


def ffn_decode(x: torch.Tensor, weights: ci_ffn_weights, act: str, y: Optional[torch.Tensor] = None,
               ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_ffn_decode on x [B, d] (or [d])."""
    x2 = x if x.dim() == 2 else x.unsqueeze(0)
    B, d = x2.shape
    if y is None:
        y = torch.empty_like(x2)
    if ws is None:
        ws = decode_workspace(B, weights.K, d, x.device)
    _check(_lib.coreinfer_ffn_decode(_ptr(x2), B, ctypes.byref(weights), DTYPE_CODE[x.dtype],
                                     ACT_CODE[act], _ptr(y), _ptr(ws), ws.numel(), _stream(x)),
           "coreinfer_ffn_decode")
    return y if x.dim() == 2 else y.squeeze(0)


def ffn_decode_static(x: torch.Tensor, weights: ci_ffn_weights, act: str, y: Optional[torch.Tensor] = None,
                      status: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_ffn_decode_static on x [B, d] (or [d]): the library's own scratch, no allocation in the call
    (pass y to keep this wrapper from allocating the output)."""
    x2 = x if x.dim() == 2 else x.unsqueeze(0)
    B, d = x2.shape
    if y is None:
        y = torch.empty_like(x2)
    _check(_lib.coreinfer_ffn_decode_static(_ptr(x2), B, ctypes.byref(weights), DTYPE_CODE[x.dtype],
                                            ACT_CODE[act], _ptr(y), _ptr(status), _stream(x)),
           "coreinfer_ffn_decode_static")
    return y if x.dim() == 2 else y.squeeze(0)


def union_build(core_idx: torch.Tensor, N: int, max_rows: Optional[int] = None):
    """coreinfer_union_build on core_idx [B, K] int32.  Returns (union_idx [max_rows] int32,
    union_mask [max_rows] int32 holding the uint32 bits, union_count [1] int32), all on the device."""
    B, K = core_idx.shape
    if max_rows is None:
        max_rows = max(1, min(N, B * K))
    dev = core_idx.device
    union_idx = torch.empty(max_rows, dtype=torch.int32, device=dev)
    union_mask = torch.empty(max_rows, dtype=torch.int32, device=dev)
    union_count = torch.empty(1, dtype=torch.int32, device=dev)
    b = _sz(0)
    _check(_lib.coreinfer_union_workspace_size(N, ctypes.byref(b)), "coreinfer_union_workspace_size")
    ws = _workspace(b.value, core_idx)
    _check(_lib.coreinfer_union_build(_ptr(core_idx), B, K, N, max_rows, _ptr(union_idx), _ptr(union_mask),
                                      _ptr(union_count), _ptr(ws), ws.numel(), _stream(core_idx)),
           "coreinfer_union_build")
    return union_idx, union_mask, union_count


def ffn_decode_union_workspace_size(B: int, max_rows: int, d: int, dtype: torch.dtype, act: str) -> int:
    b = _sz(0)
    _check(_lib.coreinfer_ffn_decode_union_workspace_size(B, max_rows, d, DTYPE_CODE[dtype], ACT_CODE[act],
                                                          ctypes.byref(b)),
           "coreinfer_ffn_decode_union_workspace_size")
    return b.value


def ffn_decode_union(x: torch.Tensor, weights: ci_ffn_weights, union_idx: torch.Tensor,
                     union_mask: torch.Tensor, union_count: torch.Tensor, act: str,
                     y: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """coreinfer_ffn_decode_union on x [B, d]; weights = the resident neuron-major matrices."""
    B, d = x.shape
    max_rows = union_idx.numel()
    if y is None:
        y = torch.empty_like(x)
    if ws is None:
        ws = _workspace(ffn_decode_union_workspace_size(B, max_rows, d, x.dtype, act), x)
    _check(_lib.coreinfer_ffn_decode_union(_ptr(x), B, ctypes.byref(weights), _ptr(union_idx), _ptr(union_mask),
                                           _ptr(union_count), max_rows, DTYPE_CODE[x.dtype], ACT_CODE[act],
                                           _ptr(y), _ptr(ws), ws.numel(), _stream(x)),
           "coreinfer_ffn_decode_union")
    return y


def ffn_dense_workspace_size(M: int, d: int, N: int, dtype: torch.dtype) -> int:
    b = _sz(0)
    _check(_lib.coreinfer_ffn_dense_workspace_size(M, d, N, DTYPE_CODE[dtype], ctypes.byref(b)),
           "coreinfer_ffn_dense_workspace_size")
    return b.value


def ffn_dense(X: torch.Tensor, w_up, w_gate, b_up, w_down, b_down, down_layout: str, act: str,
              want_y: bool = True, want_a: bool = False, Y=None, A=None, ws=None):
    """coreinfer_ffn_dense on X [M, d].  Returns (Y or None, A or None)."""
    M, d = X.shape
    N = w_up.shape[0]
    if want_y and Y is None:
        Y = torch.empty((M, d), dtype=X.dtype, device=X.device)
    if want_a and A is None:
        A = torch.empty((M, N), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _workspace(ffn_dense_workspace_size(M, d, N, X.dtype), X)
    _check(_lib.coreinfer_ffn_dense(_ptr(X), M, _ptr(w_up), _ptr(w_gate), _ptr(b_up), _ptr(w_down),
                                    _ptr(b_down), LAYOUT_CODE[down_layout], DTYPE_CODE[X.dtype],
                                    ACT_CODE[act], d, N, _ptr(Y), _ptr(A), _ptr(ws), ws.numel(),
                                    _stream(X)),
           "coreinfer_ffn_dense")
    return Y, A


def ffn_dense_hidden(X: torch.Tensor, w_up, w_gate, b_up, w_down, b_down, down_layout: str, act: str,
                     want_y: bool = True, Y=None, H=None, ws=None):
    """coreinfer_ffn_dense_hidden on X [M, d].  Returns (Y or None, H [M, N] of X's dtype)."""
    M, d = X.shape
    N = w_up.shape[0]
    if want_y and Y is None:
        Y = torch.empty((M, d), dtype=X.dtype, device=X.device)
    if H is None:
        H = torch.empty((M, N), dtype=X.dtype, device=X.device)
    if ws is None:
        b = _sz(0)
        _check(_lib.coreinfer_ffn_dense_hidden_workspace_size(M, d, N, DTYPE_CODE[X.dtype], ctypes.byref(b)),
               "coreinfer_ffn_dense_hidden_workspace_size")
        ws = _workspace(b.value, X)
    _check(_lib.coreinfer_ffn_dense_hidden(_ptr(X), M, _ptr(w_up), _ptr(w_gate), _ptr(b_up), _ptr(w_down),
                                           _ptr(b_down), LAYOUT_CODE[down_layout], DTYPE_CODE[X.dtype],
                                           ACT_CODE[act], d, N, _ptr(Y), _ptr(H), _ptr(ws), ws.numel(),
                                           _stream(X)),
           "coreinfer_ffn_dense_hidden")
    return Y, H
