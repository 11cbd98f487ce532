"""CPU checker for the Polymorph hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``polymorph_oracle.c`` (plain C, double precision)
plus shape accounting that reproduces the paper's Table 2.  Only the tests,
the smoke check and the bench's CPU-baseline leg may import this package; the
HIP library and its Python binding never do, and nothing here imports them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "polymorph_oracle.c")
_LIB = os.path.join(_HERE, "libpolymorph_oracle.so")

TARGETS = ("qkv", "proj", "fc1", "fc2")


def build(force: bool = False) -> str:
    """Compile the C checker with gcc (a few seconds)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("H", "W", "patch", "D", "heads", "L", "Dm", "L0", "targets", "r", "n_adapters", "C")] + \
               [("lora_scale", C.c_double), ("ln_eps", C.c_double)]


_FP = C.POINTER(C.c_float)


class _Weights(C.Structure):
    _fields_ = [(n, _FP) for n in
                ("patch_w", "patch_b", "cls", "pos", "ln1_g", "ln1_b", "qkv_w", "qkv_b", "proj_w", "proj_b",
                 "ln2_g", "ln2_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b", "lnf_g", "lnf_b")] + \
               [("A", _FP * 4), ("B", _FP * 4), ("head_w", _FP), ("head_b", _FP),
                ("class_map", C.POINTER(C.c_int32))]


class _SelState(C.Structure):
    _fields_ = [("valid", C.c_int32), ("prev_labels", C.POINTER(C.c_uint8)),
                ("prev_set", C.POINTER(C.c_int32)), ("prev_count", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_FP)


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


# ------------------------------------------------------------------- stages

def linear(x, W, b=None):
    x, xp = _f64(x); W, Wp = _f32(W)
    rows, din = x.shape; dout = W.shape[1]
    bp = None
    if b is not None:
        b, bp = _f32(b)
    y = np.empty((rows, dout)); _, yp = _f64(y)
    lib().ora_linear(xp, rows, din, Wp, bp, dout, y.ctypes.data_as(C.POINTER(C.c_double)))
    return y


def lora_add(x, A, B, s, y):
    x, xp = _f64(x); A, Ap = _f32(A); B, Bp = _f32(B)
    y = np.array(y, dtype=np.float64, order="C", copy=True)
    lib().ora_lora_add(xp, x.shape[0], x.shape[1], Ap, A.shape[1], Bp, B.shape[1], C.c_double(s),
                       y.ctypes.data_as(C.POINTER(C.c_double)))
    return y


def layernorm(x, g, b, eps):
    x, xp = _f64(x); g, gp = _f32(g); b, bp = _f32(b)
    y = np.empty_like(x)
    lib().ora_layernorm(xp, x.shape[0], x.shape[1], gp, bp, C.c_double(eps), y.ctypes.data_as(C.POINTER(C.c_double)))
    return y


def gelu(x):
    y = np.array(x, dtype=np.float64, order="C", copy=True)
    lib().ora_gelu(y.ctypes.data_as(C.POINTER(C.c_double)), C.c_size_t(y.size))
    return y


def attention(qkv, heads):
    qkv, qp = _f64(qkv)
    T, D3 = qkv.shape
    out = np.empty((T, D3 // 3))
    lib().ora_attention(qp, T, D3 // 3, heads, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def patch_embed(frame, cfg, w):
    frame, fp = _f32(frame)
    keep = [_f32(w[n]) for n in ("patch_w", "patch_b", "cls", "pos")]
    x = np.empty((cfg.T, cfg.D))
    lib().ora_patch_embed(fp, cfg.H, cfg.W, cfg.patch, cfg.D, *[p for _, p in keep],
                          x.ctypes.data_as(C.POINTER(C.c_double)))
    return x


# ------------------------------------------------------------ whole forward

def _pack(cfg, w: Dict[str, np.ndarray], L0: int):
    """ctypes views of a weight dict; LoRA stacks are sliced to layers [L0, L)."""
    m = _Model(cfg.H, cfg.W, cfg.patch, cfg.D, cfg.heads, cfg.L, cfg.Dm, L0, cfg.targets, cfg.r,
               cfg.n_adapters, cfg.C, float(cfg.lora_scale), float(cfg.ln_eps))
    keep = []
    ws = _Weights()
    for name in ("patch_w", "patch_b", "cls", "pos", "ln1_g", "ln1_b", "qkv_w", "qkv_b", "proj_w", "proj_b",
                 "ln2_g", "ln2_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b", "lnf_g", "lnf_b", "head_w", "head_b"):
        a, p = _f32(w[name]); keep.append(a); setattr(ws, name, p)
    for t, name in enumerate(TARGETS):
        if cfg.targets & (1 << t) and L0 < cfg.L:
            a, p = _f32(w[f"A_{name}"][L0:]); keep.append(a); ws.A[t] = p
            a, p = _f32(w[f"B_{name}"][L0:]); keep.append(a); ws.B[t] = p
    if w.get("class_map") is not None:
        a, p = _i32(w["class_map"]); keep.append(a); ws.class_map = p
    return m, ws, keep


def forward(cfg, w, frames, row_offsets, adapter_ids, L0: Optional[int] = None, merged: bool = False,
            K: int = 0, want_x: bool = False, compose: str = "branch"):
    """Scores of every (frame, adapter) row-block.  Returns dict(logits, scores, merged, x).

    compose = "branch": every (frame, adapter) pair is its own branch with that adapter alone (x is [R, T, D]);
    compose = "sum": one hidden state per frame with all of its adapters summed on top of the shared weights, then
    every active adapter's head on that state (x is [F, T, D]).
    """
    assert compose in ("branch", "sum")
    L0 = cfg.L0 if L0 is None else L0
    m, ws, keep = _pack(cfg, w, L0)
    frames, fp = _f32(frames)
    F = frames.shape[0]
    off, offp = _i32(row_offsets); ids, idsp = _i32(adapter_ids)
    R = int(off[F])
    logits = np.zeros((R, cfg.C)); scores = np.zeros((R, cfg.C))
    mo = np.zeros((F, K)) if K else None
    xf = np.zeros((R if compose == "branch" else F, cfg.T, cfg.D)) if want_x else None
    dp = C.POINTER(C.c_double)
    fn = lib().ora_forward if compose == "branch" else lib().ora_forward_sum
    rc = fn(C.byref(m), C.byref(ws), fp, F, offp, idsp, int(merged),
                           logits.ctypes.data_as(dp), scores.ctypes.data_as(dp),
                           mo.ctypes.data_as(dp) if K else None, K,
                           xf.ctypes.data_as(dp) if want_x else None)
    if rc != 0:
        raise ValueError("ora_forward: adapter id out of range or offsets not monotone")
    return dict(logits=logits, scores=scores, merged=mo, x=xf)


def lora_linear(case, s: float = 1.0, b_begin: int = 0, b_end: Optional[int] = None):
    """Y[b_begin:b_end] of the isolated multi-LoRA linear (double)."""
    X, Xp = _f32(case["X"]); W, Wp = _f32(case["W"]); A, Ap = _f32(case["A"]); B, Bp = _f32(case["B"])
    bp = None
    if case.get("bias") is not None:
        bias, bp = _f32(case["bias"])
    off, offp = _i32(case["row_offsets"]); ids, idsp = _i32(case["adapter_ids"])
    F, T, Kd = X.shape; Nd = W.shape[1]
    R = int(off[F]); b_end = R if b_end is None else b_end
    Y = np.zeros((b_end - b_begin, T, Nd))
    rc = lib().ora_lora_linear(Xp, F, T, Kd, Wp, bp, Nd, Ap, Bp, A.shape[0], A.shape[2], C.c_double(s),
                               offp, idsp, b_begin, b_end, Y.ctypes.data_as(C.POINTER(C.c_double)))
    if rc != 0:
        raise ValueError("ora_lora_linear: bad row range or adapter id")
    return Y


# ---------------------------------------------------------------- selection

class SelectState:
    """(Y_{t-1}, S_{t-1}) carried between calls of `select` on one stream (Alg. 2)."""

    def __init__(self, K: int, M: int):
        self.labels = np.zeros(K, dtype=np.uint8)
        self.set = np.zeros(M, dtype=np.int32)
        self.c = _SelState(0, self.labels.ctypes.data_as(C.POINTER(C.c_uint8)),
                           self.set.ctypes.data_as(C.POINTER(C.c_int32)), 0)


def select(scores, membership, theta: float = 0.5, context_copy: bool = False, acc=None, tau: float = 0.0,
           state: Optional[SelectState] = None, cap: Optional[int] = None):
    """Alg. 2 on a stream.  Returns (row_offsets, adapter_ids, n_uncovered)."""
    scores, sp = _f32(scores)
    mem = np.ascontiguousarray(membership, dtype=np.uint8)
    F, K = scores.shape; M = mem.shape[0]
    assert mem.shape[1] == K
    accp = None
    if acc is not None:
        acc, accp = _f32(acc)
    cap = F * M if cap is None else cap
    off = np.zeros(F + 1, dtype=np.int32); ids = np.zeros(max(cap, 1), dtype=np.int32)
    n_rows = C.c_int32(0); n_unc = C.c_int32(0)
    rc = lib().ora_select(sp, F, K, mem.ctypes.data_as(C.POINTER(C.c_uint8)), M, C.c_float(theta),
                          int(context_copy), accp, C.c_float(tau), C.byref(state.c) if state else None,
                          off.ctypes.data_as(C.POINTER(C.c_int32)), ids.ctypes.data_as(C.POINTER(C.c_int32)),
                          cap, C.byref(n_rows), C.byref(n_unc))
    if rc != 0:
        raise OverflowError(f"ora_select: cap {cap} < needed {n_rows.value}")
    return off, ids[:n_rows.value].copy(), int(n_unc.value)


# ------------------------------------- base head and the lagged loop (Fig. 3b)

def trunk(cfg, w, frames, L0: Optional[int] = None):
    """Residual stream of every frame after the shared layers [0, L0), which no adapter touches: [F, T, D].

    The stages above applied in the order of the pre-LayerNorm block, one frame at a time.
    """
    L0 = cfg.L0 if L0 is None else L0
    out = np.empty((len(frames), cfg.T, cfg.D))
    for f, frame in enumerate(frames):
        x = patch_embed(frame, cfg, w)
        for l in range(L0):
            u = layernorm(x, w["ln1_g"][l], w["ln1_b"][l], cfg.ln_eps)
            o = attention(linear(u, w["qkv_w"][l], w["qkv_b"][l]), cfg.heads)
            x = x + linear(o, w["proj_w"][l], w["proj_b"][l])
            u = layernorm(x, w["ln2_g"][l], w["ln2_b"][l], cfg.ln_eps)
            x = x + linear(gelu(linear(u, w["fc1_w"][l], w["fc1_b"][l])), w["fc2_w"][l], w["fc2_b"][l])
        out[f] = x
    return out


def base_head(cfg, w, frames, base_w, base_b, L0: Optional[int] = None):
    """Label scores of the base model's own head on the class token of the shared layers' output (the monitor
    that drives the selection, Sec. 3.2 / Fig. 3b): sigmoid(LN_f(x[0]) base_w + base_b), [F, K]."""
    x = trunk(cfg, w, frames, L0)[:, 0, :]
    z = layernorm(x, w["lnf_g"], w["lnf_b"], cfg.ln_eps)
    return 1.0 / (1.0 + np.exp(-linear(z, base_w, base_b)))


def stream_step(cfg, w, frames, base_w, base_b, membership, carry, state: Optional[SelectState] = None,
                L0: Optional[int] = None, theta: float = 0.5, context_copy: bool = False, acc=None, tau: float = 0.0,
                K_merged: int = 0):
    """One call of the lagged loop on consecutive frames of one stream: frame t runs with the adapters selected
    (Alg. 2) from the base scores of frame t - 1; the first frame of the call uses `carry` (the base scores of the
    last frame of the previous call; zeros = no previous frame, hence no labels and no adapters).

    Returns dict(base_scores [F,K], carry [K], row_offsets, adapter_ids, n_uncovered, logits, scores, merged).
    """
    bs = base_head(cfg, w, frames, base_w, base_b, L0)
    lagged = np.concatenate([np.asarray(carry, dtype=np.float64)[None, :], bs[:-1]], axis=0)
    # the selection sees the scores in single precision, as the kernel that thresholds them does
    off, ids, n_unc = select(lagged.astype(np.float32), membership, theta=theta, context_copy=context_copy, acc=acc, tau=tau,
                             state=state)
    out = forward(cfg, w, frames, off, ids, L0=L0, K=K_merged)
    out.update(base_scores=bs, carry=bs[-1].copy(), row_offsets=off, adapter_ids=ids, n_uncovered=n_unc)
    return out


# ------------------------------------- context construction (Alg. 1) and its metrics

def build_contexts(cooc, B: int, M_max: int, allow_overlap: bool = False):
    """Alg. 1 on a [K, K] co-occurrence matrix.  Returns (membership uint8 [M, K], n_unplaced)."""
    cooc, cp = _f32(cooc)
    K = cooc.shape[0]
    assert cooc.shape == (K, K)
    mem = np.zeros((max(M_max, 1), K), dtype=np.uint8)
    unplaced = C.c_int32(0)
    M = lib().ora_build_contexts(cp, K, B, M_max, int(allow_overlap), mem.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(unplaced))
    return mem[:M].copy(), int(unplaced.value)


def intra_coherence(cooc, membership, norm: float = 1.0) -> float:
    """Eq. 6 with co(i, j) = cooc[i, j] / norm."""
    cooc, cp = _f32(cooc)
    mem = np.ascontiguousarray(membership, dtype=np.uint8)
    f = lib().ora_intra_coherence
    f.restype = C.c_double
    return float(f(cp, cooc.shape[0], C.c_double(norm), mem.ctypes.data_as(C.POINTER(C.c_uint8)), mem.shape[0]))


def stream_metrics(row_offsets, adapter_ids, M: int):
    """(AvgCoverage, SwitchPenalty) of a stream of context sets given as CSR arrays (Sec. 3.4)."""
    off, offp = _i32(row_offsets)
    ids, idsp = _i32(adapter_ids if len(adapter_ids) else np.zeros(1, dtype=np.int32))
    cov = C.c_double(0.0); sw = C.c_int64(0)
    lib().ora_stream_metrics(offp, idsp, len(off) - 1, M, C.byref(cov), C.byref(sw))
    return float(cov.value), int(sw.value)


# ------------------------------------------------- shape accounting (Table 2)

def count_params(cfg, n_classes_base_head: int = 0) -> int:
    """Parameters of the backbone exactly as `forward` consumes them (+ an optional all-class head)."""
    D, L, Dm, T = cfg.D, cfg.L, cfg.Dm, cfg.T
    per_layer = 2 * D + (D * 3 * D + 3 * D) + (D * D + D) + 2 * D + (D * Dm + Dm) + (Dm * D + D)
    n = cfg.patch_dim * D + D + D + T * D + L * per_layer + 2 * D
    if n_classes_base_head:
        n += D * n_classes_base_head + n_classes_base_head
    return n


def count_adapter_params(n_layers: int, linears: Tuple[Tuple[int, int], ...], r: int, D: int, C_: int) -> int:
    """One adapter: (A, B) on each (D_in, D_out) linear of each adapted layer + its head."""
    return n_layers * sum(din * r + r * dout for din, dout in linears) + D * C_ + C_


def count_lora_macs(T: int, n_layers: int, linears: Tuple[Tuple[int, int], ...], r: int) -> int:
    """Multiply-accumulates of the low-rank branch x A B of one adapter over a T-token frame."""
    return T * n_layers * sum(din * r + r * dout for din, dout in linears)


def count_linear_macs(cfg) -> int:
    """MACs of patch embedding and the four linears per layer (attention products excluded)."""
    D, Dm, T = cfg.D, cfg.Dm, cfg.T
    return (T - 1) * cfg.patch_dim * D + cfg.L * T * (D * 3 * D + D * D + 2 * D * Dm)
