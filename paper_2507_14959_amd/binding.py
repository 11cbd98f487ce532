"""ctypes binding of libpoly (argument marshalling only; every step runs in the HIP kernels).

PyTorch provides device memory and streams.  The functions mirror include/poly.h:
``poly_select``, ``poly_forward``, ``poly_forward_workspace_bytes``, ``poly_lora_linear``.
There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np
import torch

POLY_OK, POLY_EINVAL, POLY_ERANGE, POLY_ECAP, POLY_EHIP = 0, -1, -2, -3, -4
POLY_F32, POLY_BF16 = 0, 1
TARGETS = ("qkv", "proj", "fc1", "fc2")

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpoly.so")

EXPORTS = ("poly_status_string", "poly_select_state_bytes", "poly_select", "poly_forward_workspace_bytes",
           "poly_forward", "poly_stream_step_workspace_bytes", "poly_stream_step", "poly_lora_linear_workspace_bytes",
           "poly_lora_linear", "poly_lora_linear_static", "poly_build_contexts", "poly_intra_coherence", "poly_stream_metrics",
           "poly_profile_begin", "poly_profile_end")
STATIC_SCRATCH_BYTES = 4 * 1024 * 1024
STAGES = ("select", "gemm", "shrink", "attention", "layernorm", "other")


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("H", "W", "patch", "D", "heads", "L", "Dm", "L0", "targets", "r",
                                         "n_adapters", "C", "dtype")] + \
               [("lora_scale", C.c_float), ("ln_eps", C.c_float), ("compose", C.c_int32)]


class BaseWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("patch_w", "patch_b", "cls", "pos", "ln1_g", "ln1_b", "qkv_w", "qkv_b",
                                          "proj_w", "proj_b", "ln2_g", "ln2_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b",
                                          "lnf_g", "lnf_b")]


class LoraWeights(C.Structure):
    _fields_ = [("At", C.c_void_p * 4), ("Bt", C.c_void_p * 4)]


class Heads(C.Structure):
    _fields_ = [("head_w", C.c_void_p), ("head_b", C.c_void_p), ("class_map", C.c_void_p)]


class SelectOpts(C.Structure):
    _fields_ = [("theta", C.c_float), ("context_copy", C.c_int32), ("acc", C.c_void_p), ("tau", C.c_float)]


class Stream(C.Structure):
    _fields_ = [("base_w", C.c_void_p), ("base_b", C.c_void_p), ("K", C.c_int32), ("M", C.c_int32),
                ("group_membership", C.c_void_p), ("opts", SelectOpts), ("state", C.c_void_p), ("carry", C.c_void_p)]


class Profile(C.Structure):
    _fields_ = [("launches", C.c_int32 * 6), ("ms", C.c_float * 6), ("dropped", C.c_int32)]


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_14959_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.poly_status_string.restype = C.c_char_p
        L.poly_status_string.argtypes = [C.c_int]
        L.poly_select_state_bytes.restype = C.c_size_t
        L.poly_select_state_bytes.argtypes = [C.c_int]
        L.poly_select.restype = C.c_int
        L.poly_select.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.POINTER(SelectOpts), C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.poly_forward_workspace_bytes.restype = C.c_size_t
        L.poly_forward_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_int]
        L.poly_forward.restype = C.c_int
        L.poly_forward.argtypes = [C.POINTER(ModelDesc), C.POINTER(BaseWeights), C.POINTER(LoraWeights), C.POINTER(Heads),
                                   C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.poly_stream_step_workspace_bytes.restype = C.c_size_t
        L.poly_stream_step_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_int, C.c_int]
        L.poly_stream_step.restype = C.c_int
        L.poly_stream_step.argtypes = [C.POINTER(ModelDesc), C.POINTER(BaseWeights), C.POINTER(LoraWeights), C.POINTER(Heads),
                                       C.POINTER(Stream), C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                       C.c_void_p]
        L.poly_lora_linear_workspace_bytes.restype = C.c_size_t
        L.poly_lora_linear_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
        L.poly_lora_linear.restype = C.c_int
        L.poly_lora_linear.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                       C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p,
                                       C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.poly_lora_linear_static.restype = C.c_int
        L.poly_lora_linear_static.argtypes = L.poly_lora_linear.argtypes[:18] + [C.c_void_p]
        L.poly_build_contexts.restype = C.c_int
        L.poly_build_contexts.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int32)]
        L.poly_intra_coherence.restype = C.c_int
        L.poly_intra_coherence.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_void_p, C.c_int, C.POINTER(C.c_double)]
        L.poly_stream_metrics.restype = C.c_int
        L.poly_stream_metrics.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.poly_profile_begin.restype = C.c_int
        L.poly_profile_begin.argtypes = [C.c_int]
        L.poly_profile_end.restype = C.c_int
        L.poly_profile_end.argtypes = [C.POINTER(Profile)]
        _lib = L
    return _lib


def status_string(rc: int) -> str:
    return lib().poly_status_string(rc).decode()


class PolyError(RuntimeError):
    def __init__(self, rc: int, where: str):
        super().__init__(f"{where}: {status_string(rc)} ({rc})")
        self.rc = rc


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _elt(dtype: int):
    return torch.bfloat16 if dtype == POLY_BF16 else torch.float32


# --------------------------------------------------------------------------- weights

class DeviceModel:
    """Device copies of a weight set in the library's layout (contraction index fastest).

    `w` is a dict in the paper's orientation (W[D_in, D_out], A[D_in, r], B[r, D_out], stacked
    over layers); this only transposes, slices the LoRA stacks to layers [L0, L), converts the
    matrices to the element type and uploads.
    """

    def __init__(self, cfg, w: Dict[str, np.ndarray], L0: Optional[int] = None, device="cuda", compose: str = "branch"):
        assert compose in ("branch", "sum")
        self.cfg = cfg
        self.L0 = cfg.L0 if L0 is None else L0
        elt = _elt(cfg.dtype)
        self.t: Dict[str, torch.Tensor] = {}

        def mat(name, a):   # [..., D_in, D_out] -> [..., D_out, D_in]
            self.t[name] = torch.from_numpy(np.ascontiguousarray(np.swapaxes(a, -1, -2))).to(device=device, dtype=elt).contiguous()

        def vec(name, a):
            self.t[name] = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)

        for n in ("patch_w", "qkv_w", "proj_w", "fc1_w", "fc2_w", "head_w"):
            mat(n, w[n])
        for n in ("patch_b", "cls", "pos", "ln1_g", "ln1_b", "qkv_b", "proj_b", "ln2_g", "ln2_b", "fc1_b", "fc2_b",
                  "lnf_g", "lnf_b", "head_b"):
            vec(n, w[n])
        for i, n in enumerate(TARGETS):
            if cfg.targets & (1 << i) and self.L0 < cfg.L:
                mat(f"At_{n}", w[f"A_{n}"][self.L0:])
                mat(f"Bt_{n}", w[f"B_{n}"][self.L0:])
        if w.get("class_map") is not None:
            self.t["class_map"] = torch.from_numpy(np.ascontiguousarray(w["class_map"], dtype=np.int32)).to(device)

        self.desc = ModelDesc(cfg.H, cfg.W, cfg.patch, cfg.D, cfg.heads, cfg.L, cfg.Dm, self.L0, cfg.targets, cfg.r,
                              cfg.n_adapters, cfg.C, cfg.dtype, float(cfg.lora_scale), float(cfg.ln_eps),
                              1 if compose == "sum" else 0)
        self.base = BaseWeights(**{n: self.t[n].data_ptr() for n, _ in BaseWeights._fields_})
        self.lora = LoraWeights()
        for i, n in enumerate(TARGETS):
            if f"At_{n}" in self.t:
                self.lora.At[i] = self.t[f"At_{n}"].data_ptr()
                self.lora.Bt[i] = self.t[f"Bt_{n}"].data_ptr()
        self.heads = Heads(self.t["head_w"].data_ptr(), self.t["head_b"].data_ptr(),
                           self.t["class_map"].data_ptr() if "class_map" in self.t else None)

    def frames_to_device(self, frames: np.ndarray, device="cuda") -> torch.Tensor:
        return torch.from_numpy(np.ascontiguousarray(frames, dtype=np.float32)).to(device=device, dtype=_elt(self.cfg.dtype)).contiguous()


# --------------------------------------------------------------------------- entry points

def poly_select_state_bytes(K: int) -> int:
    return int(lib().poly_select_state_bytes(K))


def poly_select(label_scores: torch.Tensor, group_membership: torch.Tensor, row_offsets: torch.Tensor,
                adapter_ids: torch.Tensor, counters: torch.Tensor, theta: float = 0.5, context_copy: bool = False,
                acc: Optional[torch.Tensor] = None, tau: float = 0.0, state: Optional[torch.Tensor] = None,
                stream=None, check: bool = True) -> int:
    """Alg. 2 on the device.  All tensors are caller-allocated device tensors (see poly.h)."""
    F, K = label_scores.shape
    M = group_membership.shape[0]
    assert label_scores.dtype == torch.float32 and group_membership.dtype == torch.uint8
    assert row_offsets.dtype == torch.int32 and adapter_ids.dtype == torch.int32 and counters.dtype == torch.int32
    assert row_offsets.numel() >= F + 1 and counters.numel() >= 2
    opts = SelectOpts(theta, int(context_copy), acc.data_ptr() if acc is not None else None, tau)
    rc = lib().poly_select(_ptr(label_scores), F, K, _ptr(group_membership), M, C.byref(opts), _ptr(state),
                           _ptr(row_offsets), _ptr(adapter_ids), adapter_ids.numel(), _ptr(counters), _stream(stream))
    if check and rc != POLY_OK:
        raise PolyError(rc, "poly_select")
    return rc


def poly_forward_workspace_bytes(model: DeviceModel, F: int, R: int) -> int:
    return int(lib().poly_forward_workspace_bytes(C.byref(model.desc), F, R))


def poly_forward(model: DeviceModel, frames: torch.Tensor, row_offsets: torch.Tensor, adapter_ids: torch.Tensor, R: int,
                 out_scores: torch.Tensor, workspace: torch.Tensor, out_logits: Optional[torch.Tensor] = None,
                 out_merged: Optional[torch.Tensor] = None, dev_status: Optional[torch.Tensor] = None, stream=None,
                 check: bool = True) -> int:
    """Forward of every (frame, adapter) row-block; outputs land in the caller's tensors."""
    F = frames.shape[0]
    K = out_merged.shape[1] if out_merged is not None else 0
    rc = lib().poly_forward(C.byref(model.desc), C.byref(model.base), C.byref(model.lora), C.byref(model.heads),
                            _ptr(frames), F, _ptr(row_offsets), _ptr(adapter_ids), R, _ptr(out_logits), _ptr(out_scores),
                            _ptr(out_merged), K, _ptr(dev_status), _ptr(workspace), workspace.numel() * workspace.element_size(),
                            _stream(stream))
    if check and rc != POLY_OK:
        raise PolyError(rc, "poly_forward")
    return rc


class DeviceStream:
    """Device side of the lagged loop: base head [D, K] / [K] (paper orientation; transposed and converted here), context
    membership [M, K], selection state and the carried scores (zeros = no previous frame)."""

    def __init__(self, model: DeviceModel, base_w: np.ndarray, base_b: np.ndarray, membership: np.ndarray, theta: float = 0.5,
                 context_copy: bool = False, device="cuda"):
        K = base_w.shape[1]
        self.K, self.M = K, membership.shape[0]
        self.base_w = torch.from_numpy(np.ascontiguousarray(base_w.T)).to(device=device, dtype=_elt(model.cfg.dtype)).contiguous()
        self.base_b = torch.from_numpy(np.ascontiguousarray(base_b, dtype=np.float32)).to(device)
        self.membership = torch.from_numpy(np.ascontiguousarray(membership, dtype=np.uint8)).to(device)
        self.state = torch.zeros(poly_select_state_bytes(K), dtype=torch.uint8, device=device)
        self.carry = torch.zeros(K, dtype=torch.float32, device=device)
        self.c = Stream(self.base_w.data_ptr(), self.base_b.data_ptr(), K, self.M, self.membership.data_ptr(),
                        SelectOpts(theta, int(context_copy), None, 0.0), self.state.data_ptr(), self.carry.data_ptr())


def poly_stream_step_workspace_bytes(model: DeviceModel, F: int, R: int, K: int) -> int:
    return int(lib().poly_stream_step_workspace_bytes(C.byref(model.desc), F, R, K))


def poly_stream_step(model: DeviceModel, s: DeviceStream, frames: torch.Tensor, R: int, row_offsets: torch.Tensor,
                     adapter_ids: torch.Tensor, counters: torch.Tensor, out_scores: torch.Tensor, workspace: torch.Tensor,
                     out_base_scores: Optional[torch.Tensor] = None, out_logits: Optional[torch.Tensor] = None,
                     out_merged: Optional[torch.Tensor] = None, dev_status: Optional[torch.Tensor] = None, stream=None,
                     check: bool = True) -> int:
    """One call of the lagged loop (base head -> Alg. 2 -> adapted layers) on consecutive frames of one stream."""
    rc = lib().poly_stream_step(C.byref(model.desc), C.byref(model.base), C.byref(model.lora), C.byref(model.heads), C.byref(s.c),
                                _ptr(frames), frames.shape[0], R, _ptr(row_offsets), _ptr(adapter_ids), _ptr(counters),
                                _ptr(out_base_scores), _ptr(out_logits), _ptr(out_scores), _ptr(out_merged), _ptr(dev_status),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != POLY_OK:
        raise PolyError(rc, "poly_stream_step")
    return rc


def poly_lora_linear_workspace_bytes(n_xblocks: int, T: int, r: int, R: int, dtype: int) -> int:
    return int(lib().poly_lora_linear_workspace_bytes(n_xblocks, T, r, R, dtype))


def poly_lora_linear(X: torch.Tensor, Wt: torch.Tensor, bias: Optional[torch.Tensor], At: torch.Tensor, Bt: torch.Tensor,
                     scale: float, row_offsets: torch.Tensor, adapter_ids: torch.Tensor, R: int, Y: torch.Tensor,
                     workspace: torch.Tensor, dev_status: Optional[torch.Tensor] = None, stream=None, check: bool = True) -> int:
    """Y[b] = X[f] Wt^T + bias + scale (X[f] At_k^T) Bt_k^T for every row-block b = (f, k)."""
    n_xblocks, T, Kdim = X.shape
    Ndim = Wt.shape[0]
    n_adapters, r = At.shape[0], At.shape[1]
    dtype = POLY_BF16 if X.dtype == torch.bfloat16 else POLY_F32
    rc = lib().poly_lora_linear(_ptr(X), n_xblocks, T, Kdim, _ptr(Wt), _ptr(bias), Ndim, _ptr(At), _ptr(Bt), n_adapters, r,
                                scale, _ptr(row_offsets), _ptr(adapter_ids), R, _ptr(Y), dtype, _ptr(dev_status),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != POLY_OK:
        raise PolyError(rc, "poly_lora_linear")
    return rc


def poly_lora_linear_static(X: torch.Tensor, Wt: torch.Tensor, bias: Optional[torch.Tensor], At: torch.Tensor, Bt: torch.Tensor,
                            scale: float, row_offsets: torch.Tensor, adapter_ids: torch.Tensor, R: int, Y: torch.Tensor,
                            dev_status: Optional[torch.Tensor] = None, stream=None, check: bool = True) -> int:
    """poly_lora_linear on the library's own static scratch array: no workspace argument, nothing allocated."""
    n_xblocks, T, Kdim = X.shape
    Ndim = Wt.shape[0]
    n_adapters, r = At.shape[0], At.shape[1]
    dtype = POLY_BF16 if X.dtype == torch.bfloat16 else POLY_F32
    rc = lib().poly_lora_linear_static(_ptr(X), n_xblocks, T, Kdim, _ptr(Wt), _ptr(bias), Ndim, _ptr(At), _ptr(Bt), n_adapters, r,
                                       scale, _ptr(row_offsets), _ptr(adapter_ids), R, _ptr(Y), dtype, _ptr(dev_status),
                                       _stream(stream))
    if check and rc != POLY_OK:
        raise PolyError(rc, "poly_lora_linear_static")
    return rc


# ---- offline half of the selector (host arrays)

def poly_build_contexts(cooc: np.ndarray, B: int, M_max: int, allow_overlap: bool = False, check: bool = True):
    """Alg. 1 on a host co-occurrence matrix [K, K].  Returns (membership uint8 [M, K], n_unplaced)."""
    cooc = np.ascontiguousarray(cooc, dtype=np.float32)
    K = cooc.shape[0]
    mem = np.zeros((max(M_max, 1), K), dtype=np.uint8)
    n_ctx, n_unplaced = C.c_int32(0), C.c_int32(0)
    rc = lib().poly_build_contexts(cooc.ctypes.data, K, B, M_max, int(allow_overlap), mem.ctypes.data, C.byref(n_ctx), C.byref(n_unplaced))
    if rc != POLY_OK:
        if check:
            raise PolyError(rc, "poly_build_contexts")
        return rc
    return mem[:n_ctx.value].copy(), int(n_unplaced.value)


def poly_intra_coherence(cooc: np.ndarray, membership: np.ndarray, norm: float = 1.0) -> float:
    cooc = np.ascontiguousarray(cooc, dtype=np.float32)
    mem = np.ascontiguousarray(membership, dtype=np.uint8)
    out = C.c_double(0.0)
    rc = lib().poly_intra_coherence(cooc.ctypes.data, cooc.shape[0], float(norm), mem.ctypes.data, mem.shape[0], C.byref(out))
    if rc != POLY_OK:
        raise PolyError(rc, "poly_intra_coherence")
    return float(out.value)


def poly_stream_metrics(row_offsets: np.ndarray, adapter_ids: np.ndarray, M: int):
    """(AvgCoverage, SwitchPenalty) of host CSR arrays."""
    off = np.ascontiguousarray(row_offsets, dtype=np.int32)
    ids = np.ascontiguousarray(adapter_ids, dtype=np.int32)
    cov, sw = C.c_double(0.0), C.c_int64(0)
    rc = lib().poly_stream_metrics(off.ctypes.data, ids.ctypes.data if ids.size else None, len(off) - 1, M, C.byref(cov), C.byref(sw))
    if rc != POLY_OK:
        raise PolyError(rc, "poly_stream_metrics")
    return float(cov.value), int(sw.value)


def poly_profile_begin(max_launches: int) -> None:
    rc = lib().poly_profile_begin(max_launches)
    if rc != POLY_OK:
        raise PolyError(rc, "poly_profile_begin")


def poly_profile_end() -> Dict[str, Dict[str, float]]:
    """Per-stage launch counts and summed kernel execution time (ms) since poly_profile_begin."""
    p = Profile()
    rc = lib().poly_profile_end(C.byref(p))
    if rc != POLY_OK:
        raise PolyError(rc, "poly_profile_end")
    return {n: dict(launches=int(p.launches[i]), ms=float(p.ms[i])) for i, n in enumerate(STAGES)}


# --------------------------------------------------------------------------- conveniences for tests and the bench

def run_forward(model: "DeviceModel", frames_np: np.ndarray, row_offsets_np, adapter_ids_np, K: int = 0, R_cap: Optional[int] = None):
    """Allocate buffers, call poly_forward once, synchronise and return host arrays."""
    dev = "cuda"
    F = frames_np.shape[0]
    R = int(row_offsets_np[-1]) if R_cap is None else R_cap
    frames = model.frames_to_device(frames_np)
    off = torch.from_numpy(np.ascontiguousarray(row_offsets_np, dtype=np.int32)).to(dev)
    ids = torch.from_numpy(np.ascontiguousarray(adapter_ids_np, dtype=np.int32)).to(dev) if len(adapter_ids_np) else torch.zeros(1, dtype=torch.int32, device=dev)
    Cc = model.cfg.C
    logits = torch.full((max(R, 1), Cc), float("nan"), device=dev)
    scores = torch.full((max(R, 1), Cc), float("nan"), device=dev)
    merged = torch.full((F, K), float("nan"), device=dev) if K else None
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(max(poly_forward_workspace_bytes(model, F, R), 256), dtype=torch.uint8, device=dev)
    poly_forward(model, frames, off, ids, R, scores, ws, out_logits=logits, out_merged=merged, dev_status=status)
    torch.cuda.synchronize()
    return dict(logits=logits.cpu().numpy()[:R], scores=scores.cpu().numpy()[:R],
                merged=merged.cpu().numpy() if K else None, status=int(status.item()))
