"""Pins of the CPU checker's stages against fp64 library routines and closed forms.

Each stage of oracle/polymorph_oracle.c is a hand-written loop; here it meets
an independent implementation (numpy / torch library kernels in float64) on
random inputs, so a dropped term, a wrong index or a transposed operand in
the loops shows up.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2507_14959_amd import synth

TOL = 1e-11


def test_linear_matches_matmul():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 13)); W = rng.standard_normal((13, 5)).astype(np.float32)
    b = rng.standard_normal(5).astype(np.float32)
    assert np.abs(oracle.linear(x, W, b) - (x @ W.astype(np.float64) + b)).max() < TOL
    assert np.abs(oracle.linear(x, W) - x @ W.astype(np.float64)).max() < TOL


def test_linear_is_not_symmetric_in_its_operands():
    # a transposed W must not pass: use a non-square, non-symmetric case with a known answer
    x = np.array([[1.0, 2.0]]); W = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    assert np.array_equal(oracle.linear(x, W), np.array([[9.0, 12.0, 15.0]]))


def test_lora_add_matches_definition():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((6, 11)); A = rng.standard_normal((11, 3)).astype(np.float32)
    B = rng.standard_normal((3, 9)).astype(np.float32); y0 = rng.standard_normal((6, 9))
    want = y0 + 1.75 * (x @ A.astype(np.float64)) @ B.astype(np.float64)
    assert np.abs(oracle.lora_add(x, A, B, 1.75, y0) - want).max() < TOL


def test_layernorm_matches_torch():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 24)) * 3 + 1; g = rng.standard_normal(24).astype(np.float32)
    b = rng.standard_normal(24).astype(np.float32)
    want = F.layer_norm(torch.from_numpy(x), (24,), torch.from_numpy(g).double(), torch.from_numpy(b).double(), 1e-6)
    assert np.abs(oracle.layernorm(x, g, b, 1e-6) - want.numpy()).max() < TOL
    # eps matters: a constant row has zero variance and must map to the shift alone
    y = oracle.layernorm(np.full((1, 24), 2.5), g, b, 1e-6)
    assert np.abs(y - b).max() < 1e-12


def test_gelu_is_x_times_normal_cdf():
    x = np.linspace(-6, 6, 97)
    want = F.gelu(torch.from_numpy(x)).numpy()
    got = oracle.gelu(x)
    assert np.abs(got - want).max() < 1e-14
    assert got[48] == 0.0
    # Phi(1) = 0.8413447460685429 (standard normal table)
    assert abs(oracle.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    assert abs(oracle.gelu(np.array([-1.0]))[0] + (1 - 0.8413447460685429)) < 1e-15


@pytest.mark.parametrize("T,heads", [(5, 1), (17, 3), (33, 2)])
def test_attention_matches_sdpa(T, heads):
    rng = np.random.default_rng(4 + T)
    d = 64; D = heads * d
    qkv = rng.standard_normal((T, 3 * D))
    q, k, v = (torch.from_numpy(qkv[:, i * D:(i + 1) * D]).reshape(T, heads, d).transpose(0, 1) for i in range(3))
    want = F.scaled_dot_product_attention(q, k, v).transpose(0, 1).reshape(T, D).numpy()
    got = oracle.attention(qkv, heads)
    assert np.abs(got - want).max() < 1e-12


def test_attention_rows_are_convex_combinations():
    # all values equal to one vector -> output is that vector whatever the scores are
    rng = np.random.default_rng(9)
    T, D = 9, 64
    qkv = rng.standard_normal((T, 3 * D)); v = rng.standard_normal(D)
    qkv[:, 2 * D:] = v
    assert np.abs(oracle.attention(qkv, 1) - v).max() < 1e-13


def test_patch_embed_matches_strided_convolution():
    cfg, w, frames, _, _ = synth.make_small_case(5, F=1, hw=32, patch=8, D=128, heads=2)
    p, D = cfg.patch, cfg.D
    # conv weight [D, 3, p, p] from W_pe[(i*p + j)*3 + c, D]
    cw = torch.from_numpy(w["patch_w"].astype(np.float64)).reshape(p, p, 3, D).permute(3, 2, 0, 1)
    img = torch.from_numpy(frames[0].astype(np.float64)).permute(2, 0, 1)[None]
    tok = F.conv2d(img, cw, torch.from_numpy(w["patch_b"]).double(), stride=p)[0].flatten(1).T  # [196, D] row-major patches
    want = np.concatenate([w["cls"][None].astype(np.float64), tok.numpy()]) + w["pos"]
    got = oracle.patch_embed(frames[0], cfg, w)
    assert got.shape == (cfg.T, D)
    assert np.abs(got - want).max() < 1e-12


def _torch_forward(cfg, w, frame, k, L0, head=None):
    """Whole forward of one (frame, adapter) branch from library routines, merged weights W + s A B.  `k` may be a list of
    adapters: then all of them are merged into the weights (W + s sum_k A_k B_k) and `head` names the adapter whose head reads
    the result."""
    ks = list(k) if isinstance(k, (list, tuple)) else [k]
    k = ks[0] if head is None else head
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    p, D, h = cfg.patch, cfg.D, cfg.heads
    cw = t(w["patch_w"]).reshape(p, p, 3, D).permute(3, 2, 0, 1)
    x = F.conv2d(t(frame).permute(2, 0, 1)[None], cw, t(w["patch_b"]), stride=p)[0].flatten(1).T
    x = torch.cat([t(w["cls"])[None], x]) + t(w["pos"])

    def W_of(name, l):
        W = t(w[f"{name}_w"][l])
        bit = dict(qkv=1, proj=2, fc1=4, fc2=8)[name]
        if l >= L0 and cfg.targets & bit:
            for ka in ks:
                W = W + cfg.lora_scale * t(w[f"A_{name}"][l, ka]) @ t(w[f"B_{name}"][l, ka])
        return W

    for l in range(cfg.L):
        u = F.layer_norm(x, (D,), t(w["ln1_g"][l]), t(w["ln1_b"][l]), cfg.ln_eps)
        qkv = u @ W_of("qkv", l) + t(w["qkv_b"][l])
        q, kk, v = (qkv[:, i * D:(i + 1) * D].reshape(-1, h, D // h).transpose(0, 1) for i in range(3))
        o = F.scaled_dot_product_attention(q, kk, v).transpose(0, 1).reshape(-1, D)
        x = x + o @ W_of("proj", l) + t(w["proj_b"][l])
        u = F.layer_norm(x, (D,), t(w["ln2_g"][l]), t(w["ln2_b"][l]), cfg.ln_eps)
        x = x + F.gelu(u @ W_of("fc1", l) + t(w["fc1_b"][l])) @ W_of("fc2", l) + t(w["fc2_b"][l])
    z = F.layer_norm(x[0], (D,), t(w["lnf_g"]), t(w["lnf_b"]), cfg.ln_eps)
    logits = z @ t(w["head_w"][k]) + t(w["head_b"][k])
    return logits.numpy(), torch.sigmoid(logits).numpy(), x.numpy()


@pytest.mark.parametrize("targets,L0", [(15, 0), (3, 0), (15, 1), (5, 2)])
def test_whole_forward_matches_library_composition(targets, L0):
    cfg, w, frames, off, ids = synth.make_small_case(11 + targets, targets=targets, L=3, F=3, max_set=2)
    # larger B so the low-rank branch is far above the tolerance
    for n in list(w):
        if n.startswith("B_"):
            w[n] = w[n] * 10
    out = oracle.forward(cfg, w, frames, off, ids, L0=L0, want_x=True)
    assert off[-1] > 0
    for f in range(len(off) - 1):
        for b in range(off[f], off[f + 1]):
            lg, sc, x = _torch_forward(cfg, w, frames[f], int(ids[b]), L0)
            assert np.abs(out["x"][b] - x).max() < 1e-9
            assert np.abs(out["logits"][b] - lg).max() < 1e-10
            assert np.abs(out["scores"][b] - sc).max() < 1e-12


def test_config1_forward_matches_library_composition():
    cfg, w, frames, off, ids = synth.make_forward_case(1)
    out = oracle.forward(cfg, w, frames, off, ids)
    for f in range(4):
        for b in range(off[f], off[f + 1]):
            lg, sc, _ = _torch_forward(cfg, w, frames[f], int(ids[b]), 0)
            assert np.abs(out["logits"][b] - lg).max() < 1e-10


@pytest.mark.parametrize("targets,L0", [(15, 0), (3, 1), (9, 2)])
def test_sum_composition_matches_library_composition_with_summed_weights(targets, L0):
    """Sec. 3.1, several adapters "summed on top": one state per frame equal to the forward whose weights are
    W + s sum_k A_k B_k over the frame's set, read by each active adapter's own head."""
    cfg, w, frames, _, _ = synth.make_small_case(70 + targets, targets=targets, L=3, F=3, n_adapters=4)
    for n in list(w):
        if n.startswith("B_"):
            w[n] = w[n] * 10
    off, ids = synth.sets_to_csr([[2, 0, 3], [], [1, 3]])
    out = oracle.forward(cfg, w, frames, off, ids, L0=L0, want_x=True, compose="sum")
    assert out["x"].shape[0] == 3
    for f in range(3):
        ks = [int(k) for k in ids[off[f]:off[f + 1]]]
        for b in range(off[f], off[f + 1]):
            lg, sc, x = _torch_forward(cfg, w, frames[f], ks, L0, head=int(ids[b]))
            assert np.abs(out["x"][f] - x).max() < 1e-9
            assert np.abs(out["logits"][b] - lg).max() < 1e-10
            assert np.abs(out["scores"][b] - sc).max() < 1e-12
