"""The base head and the lagged loop of the CPU checker, pinned against what does not depend on them."""
import numpy as np
import torch
import torch.nn.functional as F

import oracle
from paper_2507_14959_amd import synth


def _torch_trunk(cfg, w, frame, L0):
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    p, D, h = cfg.patch, cfg.D, cfg.heads
    cw = t(w["patch_w"]).reshape(p, p, 3, D).permute(3, 2, 0, 1)
    x = F.conv2d(t(frame).permute(2, 0, 1)[None], cw, t(w["patch_b"]), stride=p)[0].flatten(1).T
    x = torch.cat([t(w["cls"])[None], x]) + t(w["pos"])
    for l in range(L0):
        u = F.layer_norm(x, (D,), t(w["ln1_g"][l]), t(w["ln1_b"][l]), cfg.ln_eps)
        qkv = u @ t(w["qkv_w"][l]) + t(w["qkv_b"][l])
        q, kk, v = (qkv[:, i * D:(i + 1) * D].reshape(-1, h, D // h).transpose(0, 1) for i in range(3))
        o = F.scaled_dot_product_attention(q, kk, v).transpose(0, 1).reshape(-1, D)
        x = x + o @ t(w["proj_w"][l]) + t(w["proj_b"][l])
        u = F.layer_norm(x, (D,), t(w["ln2_g"][l]), t(w["ln2_b"][l]), cfg.ln_eps)
        x = x + F.gelu(u @ t(w["fc1_w"][l]) + t(w["fc1_b"][l])) @ t(w["fc2_w"][l]) + t(w["fc2_b"][l])
    return x


def test_trunk_matches_library_composition():
    cfg, w, frames, _, _ = synth.make_small_case(5, L=3, F=2)
    for L0 in (0, 1, 3):
        x = oracle.trunk(cfg, w, frames, L0)
        for f in range(2):
            assert np.abs(x[f] - _torch_trunk(cfg, w, frames[f], L0).numpy()).max() < 1e-9


def test_base_head_on_the_whole_backbone_is_an_adapter_head_without_adapter():
    """With L0 = L no layer is adapted: a row-block's scores are its adapter's head on the shared output, which is
    what the base head computes when it is given that head's weights (whole-forward path in C against the stages)."""
    cfg, w, frames, off, ids = synth.make_small_case(6, L=2, F=3, max_set=2)
    out = oracle.forward(cfg, w, frames, off, ids, L0=cfg.L)
    assert off[-1] > 0
    for f in range(3):
        for b in range(off[f], off[f + 1]):
            k = int(ids[b])
            bs = oracle.base_head(cfg, w, frames[f:f + 1], w["head_w"][k], w["head_b"][k], L0=cfg.L)
            assert np.abs(bs[0] - out["scores"][b]).max() < 1e-12


def test_base_head_closed_forms():
    cfg, w, frames, _, _ = synth.make_small_case(7, L=2, F=2)
    K = 6
    b = np.linspace(-2, 2, K).astype(np.float32)
    bs = oracle.base_head(cfg, w, frames, np.zeros((cfg.D, K), np.float32), b, L0=1)
    assert np.abs(bs - 1 / (1 + np.exp(-b.astype(np.float64)))[None]).max() < 1e-15      # zero weights: sigmoid(bias)
    # a head that reads one coordinate of the normalised class token
    W = np.zeros((cfg.D, K), np.float32); W[3, 0] = 1.0
    bs = oracle.base_head(cfg, w, frames, W, np.zeros(K, np.float32), L0=1)
    z = oracle.layernorm(oracle.trunk(cfg, w, frames, 1)[:, 0, :], w["lnf_g"], w["lnf_b"], cfg.ln_eps)
    assert np.abs(bs[:, 0] - 1 / (1 + np.exp(-z[:, 3]))).max() < 1e-15
    assert np.abs(bs[:, 1:] - 0.5).max() == 0


def test_stream_step_lags_by_one_frame_and_carries_over():
    cfg, w, frames, _, _ = synth.make_small_case(8, L=2, F=6, n_adapters=4)
    K = 8
    mem = synth.make_group_membership(4, 2)
    bw, bb = synth.make_base_head(cfg, K, 3)
    whole = oracle.stream_step(cfg, w, frames, bw, bb, mem, np.zeros(K), oracle.SelectState(K, 4), L0=1)
    bs = oracle.base_head(cfg, w, frames, bw, bb, L0=1)
    assert np.array_equal(whole["base_scores"], bs)
    # frame 0 has no previous frame: no adapters; frame t has exactly the sets that Alg. 2 gives for frame t - 1's labels
    assert whole["row_offsets"][1] == 0
    for t in range(1, 6):
        off, ids, _ = oracle.select(bs[t - 1:t].astype(np.float32), mem)
        got = whole["adapter_ids"][whole["row_offsets"][t]:whole["row_offsets"][t + 1]]
        assert list(got) == list(ids)
    assert whole["row_offsets"][-1] > 0
    # two calls of three frames with the carry and the state handed on = one call of six
    st = oracle.SelectState(K, 4)
    a = oracle.stream_step(cfg, w, frames[:3], bw, bb, mem, np.zeros(K), st, L0=1)
    b = oracle.stream_step(cfg, w, frames[3:], bw, bb, mem, a["carry"], st, L0=1)
    ids2 = np.concatenate([a["adapter_ids"], b["adapter_ids"]])
    off2 = np.concatenate([a["row_offsets"], b["row_offsets"][1:] + a["row_offsets"][-1]])
    assert np.array_equal(off2, whole["row_offsets"]) and np.array_equal(ids2, whole["adapter_ids"])
    assert np.array_equal(np.concatenate([a["scores"], b["scores"]]), whole["scores"])
