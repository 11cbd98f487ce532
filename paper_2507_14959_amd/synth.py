"""Seeded synthetic inputs: model shapes, weights, frames, adapter sets, label streams.

This module only draws random numbers and lays arrays out.  It holds none of
the method's arithmetic (no linear, no attention, no cover search), so both
the CPU checker and the HIP library can be fed from it without sharing code.

All floating-point arrays are float32 in the paper's orientation: a linear is
``y = x W + b`` with ``W[D_in, D_out]``, a LoRA pair is ``A[D_in, r]``,
``B[r, D_out]`` (Sec. 3.1).  For the bf16 workloads every parameter and every
pixel is rounded once to the nearest bf16 value (ties to even) and stored as
that value in float32.

The inputs stand in for COCO-trained weights and TAO video frames, which are
not available offline.  The shapes follow the paper's workload: 80 classes,
at most 3 active labels per frame, label groups of 5, sticky label sets.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

# target bit mask of the linears that carry LoRA adapters
TGT_QKV, TGT_PROJ, TGT_FC1, TGT_FC2 = 1, 2, 4, 8
TARGET_NAMES = (("qkv", TGT_QKV), ("proj", TGT_PROJ), ("fc1", TGT_FC1), ("fc2", TGT_FC2))

DT_F32, DT_BF16 = 0, 1


@dataclass(frozen=True)
class ModelCfg:
    """Shape of the shared ViT backbone and of its adapters."""
    name: str
    H: int
    W: int
    patch: int
    D: int
    heads: int
    L: int
    Dm: int
    n_adapters: int
    r: int
    targets: int
    C: int
    dtype: int            # DT_F32 or DT_BF16: storage type of matrices and frames
    L0: int = 0           # first layer that carries LoRA; layers [0, L0) are shared
    lora_scale: float = 1.0
    ln_eps: float = 1e-6

    @property
    def T(self) -> int:
        return 1 + (self.H // self.patch) * (self.W // self.patch)

    @property
    def patch_dim(self) -> int:
        return 3 * self.patch * self.patch

    def target_dims(self) -> Dict[str, Tuple[int, int]]:
        d = {"qkv": (self.D, 3 * self.D), "proj": (self.D, self.D),
             "fc1": (self.D, self.Dm), "fc2": (self.Dm, self.D)}
        return {n: d[n] for n, bit in TARGET_NAMES if self.targets & bit}

    def with_L0(self, L0: int) -> "ModelCfg":
        return replace(self, L0=L0)

    def polymorph_L0(self) -> int:
        """Adapters on the final 20 % of the layers only (Sec. 3.1)."""
        return self.L - max(1, (self.L * 20) // 100)


CFG1 = ModelCfg("tiny-fp32", 64, 64, 16, 192, 3, 2, 768, 4, 4, TGT_QKV | TGT_PROJ, 5, DT_F32)
CFG2 = ModelCfg("deit-tiny-bf16", 224, 224, 16, 192, 3, 12, 768, 16, 8, TGT_QKV | TGT_PROJ, 5, DT_BF16)
CFG3 = ModelCfg("vit-base-bf16", 224, 224, 16, 768, 12, 12, 3072, 32, 16,
                TGT_QKV | TGT_PROJ | TGT_FC1 | TGT_FC2, 8, DT_BF16)
CFG4 = replace(CFG2, name="deit-tiny-stream-bf16")

N_FRAMES = {1: 4, 2: 32, 3: 64, 4: 64}


def seed_of(config_index: int) -> int:
    return 1000 + config_index


# ----------------------------------------------------------------------------
# bf16 helpers (storage only)
# ----------------------------------------------------------------------------

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bf16 value of each float32 (ties to even), returned as float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array that already holds bf16-valued float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "array is not bf16-valued"
    return (u >> np.uint32(16)).astype(np.uint16).reshape(a.shape)


# ----------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------

def _n(rng, shape, std, mean=0.0):
    return (mean + std * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)


def make_weights(cfg: ModelCfg, rng: np.random.Generator) -> Dict[str, np.ndarray]:
    """Base, LoRA and head parameters.

    Matrices, cls, pos and heads ~ N(0, 0.02) (0.02 is the standard deviation);
    biases and LayerNorm shifts ~ N(0, 0.02); LayerNorm gains = 1 + N(0, 0.02);
    LoRA A ~ N(0, 1/r), B ~ N(0, 0.02).  LoRA stacks cover all L layers so one
    set of weights serves every choice of L0 (callers slice ``[L0:]``).
    """
    D, L, Dm, T = cfg.D, cfg.L, cfg.Dm, cfg.T
    w: Dict[str, np.ndarray] = {}
    w["patch_w"] = _n(rng, (cfg.patch_dim, D), 0.02)
    w["patch_b"] = _n(rng, (D,), 0.02)
    w["cls"] = _n(rng, (D,), 0.02)
    w["pos"] = _n(rng, (T, D), 0.02)
    w["ln1_g"] = _n(rng, (L, D), 0.02, 1.0)
    w["ln1_b"] = _n(rng, (L, D), 0.02)
    w["qkv_w"] = _n(rng, (L, D, 3 * D), 0.02)
    w["qkv_b"] = _n(rng, (L, 3 * D), 0.02)
    w["proj_w"] = _n(rng, (L, D, D), 0.02)
    w["proj_b"] = _n(rng, (L, D), 0.02)
    w["ln2_g"] = _n(rng, (L, D), 0.02, 1.0)
    w["ln2_b"] = _n(rng, (L, D), 0.02)
    w["fc1_w"] = _n(rng, (L, D, Dm), 0.02)
    w["fc1_b"] = _n(rng, (L, Dm), 0.02)
    w["fc2_w"] = _n(rng, (L, Dm, D), 0.02)
    w["fc2_b"] = _n(rng, (L, D), 0.02)
    w["lnf_g"] = _n(rng, (D,), 0.02, 1.0)
    w["lnf_b"] = _n(rng, (D,), 0.02)
    for name, (din, dout) in cfg.target_dims().items():
        w[f"A_{name}"] = _n(rng, (L, cfg.n_adapters, din, cfg.r), 1.0 / cfg.r)
        w[f"B_{name}"] = _n(rng, (L, cfg.n_adapters, cfg.r, dout), 0.02)
    w["head_w"] = _n(rng, (cfg.n_adapters, D, cfg.C), 0.02)
    w["head_b"] = _n(rng, (cfg.n_adapters, cfg.C), 0.02)
    if cfg.dtype == DT_BF16:
        w = {k: round_to_bf16(v) for k, v in w.items()}
    # adapter k reports classes k*C .. k*C+C-1 of the merged label space
    w["class_map"] = (np.arange(cfg.n_adapters, dtype=np.int32)[:, None] * cfg.C
                      + np.arange(cfg.C, dtype=np.int32)[None, :]).astype(np.int32)
    return w


def make_frames(cfg: ModelCfg, F: int, rng: np.random.Generator) -> np.ndarray:
    """F frames of uniform [0,1) pixels, NHWC float32 (bf16-valued if cfg is bf16)."""
    x = rng.random((F, cfg.H, cfg.W, 3), dtype=np.float32)
    return round_to_bf16(x) if cfg.dtype == DT_BF16 else x


# ----------------------------------------------------------------------------
# adapter sets
# ----------------------------------------------------------------------------

def _draw_ids(rng, n_adapters: int, count: int, zipf_s: float | None) -> List[int]:
    """`count` distinct adapter ids; uniform, or Zipf P(k) ~ (k+1)^-s renormalised after each draw."""
    if zipf_s is None:
        p = np.ones(n_adapters)
    else:
        p = (np.arange(n_adapters) + 1.0) ** (-zipf_s)
    ids: List[int] = []
    for _ in range(count):
        q = p / p.sum()
        k = int(rng.choice(n_adapters, p=q))
        ids.append(k)
        p[k] = 0.0
    return sorted(ids)


def sets_to_csr(sets: List[List[int]]) -> Tuple[np.ndarray, np.ndarray]:
    off = np.zeros(len(sets) + 1, dtype=np.int32)
    for f, s in enumerate(sets):
        off[f + 1] = off[f] + len(s)
    ids = np.array([k for s in sets for k in s], dtype=np.int32).reshape(-1)
    return off, ids


def make_adapter_sets(config_index: int, cfg: ModelCfg, F: int, rng) -> Tuple[np.ndarray, np.ndarray]:
    """Per-frame adapter sets as CSR (row_offsets[F+1], adapter_ids[R]), ids ascending in a frame."""
    sets = []
    for _ in range(F):
        if config_index == 1:
            cnt, s = int(rng.integers(1, 3)), None
        elif config_index == 2:
            cnt, s = 1 + int(rng.binomial(2, 0.4)), None
        elif config_index == 3:
            cnt, s = int(rng.integers(1, 4)), 1.1
        else:
            raise ValueError(config_index)
        sets.append(_draw_ids(rng, cfg.n_adapters, cnt, s))
    return sets_to_csr(sets)


# ----------------------------------------------------------------------------
# whole workloads
# ----------------------------------------------------------------------------

def make_forward_case(config_index: int, F: int | None = None, cfg: ModelCfg | None = None):
    """(cfg, weights, frames, row_offsets, adapter_ids) of forward configs 1-3."""
    cfg = cfg or {1: CFG1, 2: CFG2, 3: CFG3}[config_index]
    F = F or N_FRAMES[config_index]
    rng = np.random.default_rng(seed_of(config_index))
    w = make_weights(cfg, rng)
    frames = make_frames(cfg, F, rng)
    off, ids = make_adapter_sets(config_index, cfg, F, rng)
    return cfg, w, frames, off, ids


def make_small_case(seed: int, dtype: int = DT_F32, F: int = 3, targets: int = 15,
                    L: int = 2, r: int = 4, n_adapters: int = 3, D: int = 128, heads: int = 2,
                    Dm: int = 256, hw: int = 32, patch: int = 8, C: int = 3, max_set: int = 2):
    """A small model for fast tests (head dim stays 64)."""
    cfg = ModelCfg(f"small-{seed}", hw, hw, patch, D, heads, L, Dm, n_adapters, r, targets, C, dtype)
    rng = np.random.default_rng(seed)
    w = make_weights(cfg, rng)
    frames = make_frames(cfg, F, rng)
    sets = [_draw_ids(rng, n_adapters, int(rng.integers(0, max_set + 1)), None) for _ in range(F)]
    off, ids = sets_to_csr(sets)
    return cfg, w, frames, off, ids


def make_lora_linear_case(n_xblocks: int = 256, T: int = 197, Kdim: int = 768, Ndim: int = 2304,
                          n_adapters: int = 64, r: int = 16, per_block: int = 2,
                          dtype: int = DT_BF16, seed: int = seed_of(5), x_std: float = 1.0):
    """Isolated multi-LoRA linear (config 5): X blocks, base W, adapter stacks, CSR adapter sets.

    Every X block holds `per_block` distinct adapters drawn Zipf(1.1); with
    per_block=1 and n_xblocks=512 it is the deep-layer variant where no two
    row-blocks share an input.
    """
    rng = np.random.default_rng(seed)
    X = _n(rng, (n_xblocks, T, Kdim), x_std)
    W = _n(rng, (Kdim, Ndim), 0.02)
    bias = _n(rng, (Ndim,), 0.02)
    A = _n(rng, (n_adapters, Kdim, r), 1.0 / r)
    B = _n(rng, (n_adapters, r, Ndim), 0.02)
    if dtype == DT_BF16:
        X, W, bias, A, B = (round_to_bf16(t) for t in (X, W, bias, A, B))
    sets = [_draw_ids(rng, n_adapters, per_block, 1.1) for _ in range(n_xblocks)]
    off, ids = sets_to_csr(sets)
    return dict(X=X, W=W, bias=bias, A=A, B=B, row_offsets=off, adapter_ids=ids,
                T=T, Kdim=Kdim, Ndim=Ndim, n_adapters=n_adapters, r=r, dtype=dtype)


def make_paper_preset(F: int = 32, seed: int = 1006, adapters_per_frame: int | None = None):
    """The setting the paper trains (Sec. 4): DeiT-tiny, 11 contexts with 5-class heads, rank 16 with scaling factor 32
    (s = 32 / 16 = 2) on the query and value projections only, adapters on the last 20 % of the layers.

    On the fused qkv linear D -> 3D a query + value adapter is ONE adapter of rank 32: A = [A_q | A_v] and
    B = [[B_q, 0, 0], [0, 0, B_v]] (the key columns and the cross blocks of B are zero).  Returns (cfg, weights, frames,
    row_offsets, adapter_ids) with 1 + Binomial(2, 0.4) adapters per frame (or exactly `adapters_per_frame`).
    """
    D, r = 192, 16
    cfg = ModelCfg("deit-tiny-paper-preset", 224, 224, 16, D, 3, 12, 768, 11, 2 * r, TGT_QKV, 5, DT_BF16, L0=10, lora_scale=2.0)
    rng = np.random.default_rng(seed)
    w = make_weights(cfg, rng)
    B = np.zeros_like(w["B_qkv"])                       # [L, N_ad, 2r, 3D]
    B[:, :, :r, :D] = w["B_qkv"][:, :, :r, :D]          # query ranks write query columns
    B[:, :, r:, 2 * D:] = w["B_qkv"][:, :, r:, 2 * D:]  # value ranks write value columns
    w["B_qkv"] = B
    frames = make_frames(cfg, F, rng)
    sets = [_draw_ids(rng, cfg.n_adapters, adapters_per_frame or 1 + int(rng.binomial(2, 0.4)), None) for _ in range(F)]
    off, ids = sets_to_csr(sets)
    return cfg, w, frames, off, ids


# ----------------------------------------------------------------------------
# label stream (config 4)
# ----------------------------------------------------------------------------

def make_base_head(cfg: ModelCfg, K: int, seed: int, logit_std: float = 3.0, bias_mean: float = -1.0) -> Tuple[np.ndarray, np.ndarray]:
    """Weights [D, K] and bias [K] of a base head over K labels.  The LayerNorm output it reads has unit variance per
    element, so weights ~ N(0, logit_std^2 / D) give logits of about that spread around bias_mean: a few labels per
    frame are active (bias_mean = -5 with 80 labels: about four, close to the paper's streams) and the active set
    changes from frame to frame."""
    rng = np.random.default_rng(seed)
    W = _n(rng, (cfg.D, K), logit_std / np.sqrt(cfg.D))
    b = _n(rng, (K,), 0.5, bias_mean)
    if cfg.dtype == DT_BF16:
        W, b = round_to_bf16(W), round_to_bf16(b)
    return W, b


def make_group_membership(n_groups: int = 16, group_size: int = 5) -> np.ndarray:
    """membership[m, l] = 1 iff label l belongs to context m; group m = labels 5m..5m+4."""
    K = n_groups * group_size
    mem = np.zeros((n_groups, K), dtype=np.uint8)
    for m in range(n_groups):
        mem[m, m * group_size:(m + 1) * group_size] = 1
    return mem


def make_label_stream(n_frames: int = 1024, n_groups: int = 16, group_size: int = 5,
                      p_stay: float = 0.9, max_labels: int = 3, mu: float = 3.0,
                      seed: int = seed_of(4)):
    """Sticky label process and its noisy per-class scores.

    State = ordered active label list.  Each step every active label survives
    independently with probability p_stay; when at least one is dropped a new
    group is picked uniformly and 1-3 of its labels join the survivors, the
    list being cut to `max_labels`.  Scores are sigmoid(mu*(2*[active]-1)+N(0,1)).
    Returns (scores float32 [n_frames, K], true_sets list of label lists).
    """
    rng = np.random.default_rng(seed)
    K = n_groups * group_size

    def fresh():
        g = int(rng.integers(0, n_groups))
        n = int(rng.integers(1, 4))
        return [g * group_size + int(i) for i in rng.choice(group_size, size=n, replace=False)]

    active = fresh()[:max_labels]
    truth = []
    for _ in range(n_frames):
        truth.append(list(active))
        keep = [l for l in active if rng.random() < p_stay]
        if len(keep) != len(active):
            nxt = list(keep)
            for l in fresh():
                if l not in nxt:
                    nxt.append(l)
            active = nxt[:max_labels]
    truth = truth[:n_frames]
    sign = -np.ones((n_frames, K), dtype=np.float32)
    for t, ls in enumerate(truth):
        sign[t, ls] = 1.0
    z = mu * sign + rng.standard_normal((n_frames, K), dtype=np.float32)
    scores = (1.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)
    return scores, truth


def make_cover_instance(seed: int, K: int, M: int, max_size: int, partition: bool = False,
                        with_acc: bool = False):
    """Small random contexts (possibly overlapping) for cover tests: (membership, acc or None)."""
    rng = np.random.default_rng(seed)
    mem = np.zeros((M, K), dtype=np.uint8)
    if partition:
        perm = rng.permutation(K)
        cuts = np.sort(rng.choice(np.arange(1, K), size=M - 1, replace=False)) if M > 1 else []
        for m, part in enumerate(np.split(perm, cuts)):
            mem[m, part] = 1
    else:
        for m in range(M):
            n = int(rng.integers(1, max_size + 1))
            mem[m, rng.choice(K, size=n, replace=False)] = 1
    acc = rng.random((M, K), dtype=np.float32) if with_acc else None
    return mem, acc


# ----------------------------------------------------------------------------
# co-occurrence matrix and accuracy table (context construction, overlapping contexts)
# ----------------------------------------------------------------------------

def make_cooccurrence(n_groups: int = 16, group_size: int = 5, n_images: int = 20000, p_partner: float = 0.0,
                      p_extra: float = 0.15, seed: int = 2001, shuffle: bool = True):
    """Counts of a synthetic training set with planted label groups, in place of the COCO co-occurrence matrix.

    Every image shows 1-3 labels of one planted group (groups have a Zipf-like popularity); each shown label brings its
    fixed partner label from another group along with probability p_partner (cross-group structure: with it the
    neighbourhoods of the labels of one group differ, which is what makes overlapping contexts distinct); with
    probability p_extra one label from anywhere is added.  cooc[i, j] (i != j) = images showing both, cooc[l, l] =
    images showing l.  Returns (cooc float32 [K, K], planted list of label lists, n_images).  With `shuffle` the
    label ids are permuted so that the planted groups are not runs of consecutive ids.
    """
    rng = np.random.default_rng(seed)
    K = n_groups * group_size
    perm = rng.permutation(K) if shuffle else np.arange(K)
    planted = [[int(perm[g * group_size + i]) for i in range(group_size)] for g in range(n_groups)]
    group_of = np.zeros(K, dtype=np.int64)
    for g, ls in enumerate(planted):
        group_of[ls] = g
    partner = np.zeros(K, dtype=np.int64)
    for l in range(K):
        while True:
            c = int(rng.integers(0, K))
            if group_of[c] != group_of[l]:
                partner[l] = c
                break
    pop = (np.arange(n_groups) + 1.0) ** -0.7
    pop /= pop.sum()
    cooc = np.zeros((K, K), dtype=np.float64)
    groups = rng.choice(n_groups, size=n_images, p=pop)
    counts = rng.integers(1, 4, size=n_images)
    extra = rng.random(n_images) < p_extra
    extra_label = rng.integers(0, K, size=n_images)
    for g, n, e, el in zip(groups, counts, extra, extra_label):
        shown = [int(x) for x in rng.choice(planted[g], size=int(n), replace=False)]
        labels = set(shown)
        for l in shown:
            if p_partner > 0.0 and rng.random() < p_partner:
                labels.add(int(partner[l]))
        if e:
            labels.add(int(el))
        labels = sorted(labels)
        for a in labels:
            for b in labels:
                cooc[a, b] += 1.0
    return cooc.astype(np.float32), planted, n_images


def make_accuracy_table(membership: np.ndarray, seed: int = 2002, lo: float = 0.05, hi: float = 1.0) -> np.ndarray:
    """A synthetic a_{C,l} table [M, K]: uniform in [lo, hi) where label l is in context C, 0 elsewhere (in place of the
    per-class validation accuracies of trained adapters)."""
    rng = np.random.default_rng(seed)
    acc = (lo + (hi - lo) * rng.random(membership.shape, dtype=np.float32)).astype(np.float32)
    return np.where(membership != 0, acc, np.float32(0.0)).astype(np.float32)
