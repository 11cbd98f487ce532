"""The library's host-side entry points for context construction (Alg. 1) and the cluster metrics of Sec. 3.4 against the
checker, element for element.  No GPU needed: all of this is host code."""
import numpy as np
import pytest

import oracle
from paper_2507_14959_amd import binding, synth


@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("overlap", [False, True])
def test_library_build_contexts_matches_checker(seed, overlap):
    rng = np.random.default_rng(300 + seed)
    K = int(rng.integers(3, 90))
    B = int(rng.integers(1, 8))
    M_max = int(rng.integers(1, 65))
    c = rng.integers(0, 5, size=(K, K)).astype(np.float32)
    c = np.minimum(c, c.T)
    c[np.diag_indices(K)] = rng.integers(0, 12, size=K)
    c[rng.integers(0, K), :] = 0
    want, want_unplaced = oracle.build_contexts(c, B, M_max, overlap)
    got, unplaced = binding.poly_build_contexts(c, B, M_max, overlap)
    assert np.array_equal(got, want) and unplaced == want_unplaced
    if len(want):
        assert binding.poly_intra_coherence(c, got, norm=7.0) == pytest.approx(oracle.intra_coherence(c, want, norm=7.0), rel=1e-12)


@pytest.mark.parametrize("p_partner,M_max,overlap", [(0.0, 16, False), (0.5, 11, False), (0.5, 45, True), (0.5, 50, True), (0.7, 64, True)])
def test_library_on_the_synthetic_training_set(p_partner, M_max, overlap):
    cooc, _, n_images = synth.make_cooccurrence(p_partner=p_partner, seed=2003)
    want, want_unplaced = oracle.build_contexts(cooc, 5, M_max, overlap)
    got, unplaced = binding.poly_build_contexts(cooc, 5, M_max, overlap)
    assert np.array_equal(got, want) and unplaced == want_unplaced
    assert binding.poly_intra_coherence(cooc, got, norm=n_images) == pytest.approx(oracle.intra_coherence(cooc, want, norm=n_images), rel=1e-12)


def test_library_stream_metrics_and_argument_checks():
    rng = np.random.default_rng(11)
    sets = [rng.permutation(rng.choice(45, size=int(rng.integers(0, 4)), replace=False)).tolist() for _ in range(500)]
    off, ids = synth.sets_to_csr(sets)
    assert binding.poly_stream_metrics(off, ids, 45) == oracle.stream_metrics(off, ids, 45)
    off0, ids0 = synth.sets_to_csr([[], [], []])
    assert binding.poly_stream_metrics(off0, ids0, 4) == (0.0, 0)
    with pytest.raises(binding.PolyError):
        binding.poly_stream_metrics(off, ids, 10)             # ids up to 44 with M = 10
    assert binding.poly_build_contexts(np.zeros((4, 4), dtype=np.float32), 0, 4, check=False) == binding.POLY_EINVAL
    assert binding.poly_build_contexts(np.zeros((4, 4), dtype=np.float32), 2, 65, check=False) == binding.POLY_EINVAL
    mem, unplaced = binding.poly_build_contexts(np.zeros((4, 4), dtype=np.float32), 2, 4)   # no valid label: no context
    assert mem.shape == (0, 4) and unplaced == 0
