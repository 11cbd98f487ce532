"""Invariants the method fixes for the forward (Sec. 3.1) and the paper's Table 2 counts."""
import os

import numpy as np
import pytest

import oracle
from paper_2507_14959_amd import synth


def _case(seed=21, **kw):
    cfg, w, frames, off, ids = synth.make_small_case(seed, **kw)
    return cfg, w, frames, off, ids


def test_zero_B_reproduces_bare_backbone():
    cfg, w, frames, off, ids = _case(F=3, max_set=2, L=2)
    wz = {k: (np.zeros_like(v) if k.startswith("B_") else v) for k, v in w.items()}
    a = oracle.forward(cfg, wz, frames, off, ids, L0=0, want_x=True)
    bare = oracle.forward(cfg, w, frames, off, ids, L0=cfg.L, want_x=True)   # no layer adapted
    assert off[-1] > 0
    assert np.array_equal(a["x"], bare["x"])
    assert np.array_equal(a["logits"], bare["logits"])
    # and the adapters do matter when B is not zero
    full = oracle.forward(cfg, w, frames, off, ids, L0=0, want_x=True)
    assert np.abs(full["x"] - bare["x"]).max() > 1e-3


@pytest.mark.parametrize("which", ["small", "cfg1", "cfg2-slice"])
def test_unmerged_equals_merged(which):
    if which == "small":
        cfg, w, frames, off, ids = _case(22, F=2, L=2)
    elif which == "cfg1":
        cfg, w, frames, off, ids = synth.make_forward_case(1)
    else:
        cfg, w, frames, off, ids = synth.make_forward_case(2, F=2)
        cfg = cfg.with_L0(10)          # two adapted layers keeps the merged path short
    a = oracle.forward(cfg, w, frames, off, ids)
    b = oracle.forward(cfg, w, frames, off, ids, merged=True)
    assert np.abs(a["logits"] - b["logits"]).max() < 1e-6
    assert np.abs(a["logits"] - b["logits"]).max() > 0      # two different evaluation orders


def test_row_output_depends_only_on_frame_and_adapter():
    cfg, w, frames, _, _ = _case(23, F=2, n_adapters=4)
    fr = np.stack([frames[0], frames[1], frames[0], frames[0]])
    off, ids = synth.sets_to_csr([[0, 2], [1], [2], [3, 2, 0]])
    out = oracle.forward(cfg, w, fr, off, ids, want_x=True)
    # (frame0, adapter2) appears as rows 1, 3, 5; (frame0, adapter0) as rows 0 and 6
    assert np.array_equal(out["x"][1], out["x"][3]) and np.array_equal(out["x"][1], out["x"][5])
    assert np.array_equal(out["logits"][0], out["logits"][6])
    assert not np.array_equal(out["logits"][0], out["logits"][1])


def test_L0_consistency():
    cfg, w, frames, off, ids = _case(24, F=2, L=3)
    w0 = dict(w)
    for n in w:
        if n.startswith("B_"):
            z = w[n].copy(); z[:2] = 0; w0[n] = z            # adapters silent in layers 0, 1
    a = oracle.forward(cfg, w0, frames, off, ids, L0=0)
    b = oracle.forward(cfg, w, frames, off, ids, L0=2)
    assert np.array_equal(a["logits"], b["logits"])


def test_scores_are_sigmoid_and_merge_takes_max():
    cfg, w, frames, _, _ = _case(25, F=3, n_adapters=3, C=3)
    w = dict(w)
    w["class_map"] = np.array([[0, 1, 2], [2, 3, 4], [5, 6, 7]], dtype=np.int32)   # adapters 0, 1 overlap on class 2
    off, ids = synth.sets_to_csr([[0, 1], [], [2]])
    out = oracle.forward(cfg, w, frames, off, ids, K=9)
    s, m = out["scores"], out["merged"]
    assert np.all((s > 0) & (s < 1))
    assert np.abs(s - 1 / (1 + np.exp(-out["logits"]))).max() < 1e-15
    assert np.array_equal(m[1], np.zeros(9))                       # frame without adapters
    assert m[0, 2] == max(s[0, 2], s[1, 0]) and m[0, 0] == s[0, 0] and m[0, 4] == s[1, 2]
    assert np.array_equal(m[0, 5:], np.zeros(4)) and np.array_equal(m[2, 5:8], s[2]) and m[2, 8] == 0


def test_bad_ids_are_rejected():
    cfg, w, frames, off, ids = _case(26, F=2, max_set=1)
    off, ids = synth.sets_to_csr([[0], [cfg.n_adapters]])
    with pytest.raises(ValueError):
        oracle.forward(cfg, w, frames, off, ids)


def test_lora_linear_matches_library_and_forward_linear():
    case = synth.make_lora_linear_case(n_xblocks=3, T=5, Kdim=24, Ndim=16, n_adapters=4, r=4, per_block=2, seed=7,
                                       dtype=synth.DT_F32)
    Y = oracle.lora_linear(case, s=2.0)
    off, ids = case["row_offsets"], case["adapter_ids"]
    X, W, A, B = (case[k].astype(np.float64) for k in "XWAB")
    for f in range(3):
        for b in range(off[f], off[f + 1]):
            k = ids[b]
            want = X[f] @ W + case["bias"] + 2.0 * (X[f] @ A[k]) @ B[k]
            assert np.abs(Y[b] - want).max() < 1e-12
    assert np.array_equal(oracle.lora_linear(case, s=2.0, b_begin=2, b_end=5), Y[2:5])


# ------------------------------------------------- several adapters summed on one hidden state (Sec. 3.1)

def test_sum_composition_with_one_adapter_per_frame_is_the_branch_reading():
    cfg, w, frames, _, _ = _case(27, F=3, n_adapters=4, L=2)
    off, ids = synth.sets_to_csr([[2], [], [0]])
    a = oracle.forward(cfg, w, frames, off, ids, want_x=True, K=12)
    b = oracle.forward(cfg, w, frames, off, ids, want_x=True, K=12, compose="sum")
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["merged"], b["merged"])
    assert np.array_equal(a["x"][0], b["x"][0]) and np.array_equal(a["x"][1], b["x"][2])


def test_sum_composition_equals_the_forward_with_all_deltas_merged():
    cfg, w, frames, _, _ = _case(28, F=2, n_adapters=4, L=2)
    off, ids = synth.sets_to_csr([[3, 1, 0], [2, 1]])
    a = oracle.forward(cfg, w, frames, off, ids, compose="sum")
    b = oracle.forward(cfg, w, frames, off, ids, compose="sum", merged=True)
    assert 0 < np.abs(a["logits"] - b["logits"]).max() < 1e-6          # two different evaluation orders of the same sum
    # and it is not the branch reading: the other adapters of the frame change a row
    c = oracle.forward(cfg, w, frames, off, ids)
    assert np.abs(a["logits"] - c["logits"]).max() > 1e-4


def test_sum_composition_rows_share_the_frame_state_and_ignore_the_order_of_the_set():
    cfg, w, frames, _, _ = _case(29, F=2, n_adapters=4, L=2, C=3)
    off, ids = synth.sets_to_csr([[0, 2, 3], [1]])
    a = oracle.forward(cfg, w, frames, off, ids, compose="sum", K=12)
    off2, ids2 = synth.sets_to_csr([[3, 0, 2], [1]])
    b = oracle.forward(cfg, w, frames, off2, ids2, compose="sum", K=12)
    # same sets: the rows move with their adapters; sums of doubles in another order agree to rounding
    assert np.abs(a["logits"][[0, 1, 2]] - b["logits"][[1, 2, 0]]).max() < 1e-12
    assert np.abs(a["merged"] - b["merged"]).max() < 1e-12
    # zero B: every row is the bare backbone read by its adapter's head
    wz = {k: (np.zeros_like(v) if k.startswith("B_") else v) for k, v in w.items()}
    z = oracle.forward(cfg, wz, frames, off, ids, compose="sum")
    bare = oracle.forward(cfg, w, frames, off, ids, L0=cfg.L)
    assert np.array_equal(z["logits"], bare["logits"])


# ---------------------------------------------------------------- Table 2

def _table2():
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table2.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                name, p, mem, macs = line.split()
                rows[name] = (float(p), float(mem), float(macs))
    return rows


def test_table2_parameter_and_mac_counts():
    """The checker's shape accounting reproduces Table 2 as printed (two decimals)."""
    t2 = _table2()
    tiny, base = synth.CFG2, synth.CFG3
    MiB = 4 / 2 ** 20

    n_base = oracle.count_params(tiny, 80)
    assert round(n_base / 1e6, 2) == t2["Base"][0]
    assert abs(n_base * MiB - t2["Base"][1]) < 0.015
    n_large = oracle.count_params(base, 80)
    assert round(n_large / 1e6, 2) == t2["Larger"][0]
    assert abs(n_large * MiB - t2["Larger"][1]) < 0.015

    # Sec. 4: rank 16 on query and value (192 -> 192 each), last 20 % of 12 layers, 5-class head, 11 contexts
    n_layers = tiny.L - tiny.polymorph_L0()
    assert n_layers == 2
    qv = ((192, 192), (192, 192))
    n_ad = 11 * oracle.count_adapter_params(n_layers, qv, 16, 192, 5)
    assert round((n_base + n_ad) / 1e6, 2) == t2["Polymorph"][0]
    assert abs((n_base + n_ad) * MiB - t2["Polymorph"][1]) < 0.015
    # MACs: the low-rank branch of one active adapter is the printed difference Polymorph - Base
    lora_macs = oracle.count_lora_macs(tiny.T, n_layers, qv, 16)
    assert round(lora_macs / 1e6, 2) == round(t2["Polymorph"][2] - t2["Base"][2], 2)
    # linears + patch embedding alone stay below the printed total (which also counts attention products)
    assert oracle.count_linear_macs(tiny) / 1e6 < t2["Base"][2]
    assert oracle.count_linear_macs(tiny) / 1e6 > 0.99 * t2["Base"][2]


def test_accounting_agrees_with_generated_weights():
    for cfg in (synth.CFG1, synth.CFG2):
        w = synth.make_weights(cfg, np.random.default_rng(0))
        n = sum(v.size for k, v in w.items()
                if not k.startswith(("A_", "B_", "head_", "class_map")))
        assert n == oracle.count_params(cfg)
