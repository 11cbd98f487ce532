"""Pins of the checker's context construction (Alg. 1, Sec. 3.4) and cluster metrics (Eq. 6, AvgCoverage, SwitchPenalty)."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2507_14959_amd import synth

# A 4-label matrix worked by hand.  Frequencies 10, 8, 6, 5: labels are visited in the order 0, 1, 2, 3.
HAND = np.array([[10, 4, 1, 0],
                 [4, 8, 2, 0],
                 [1, 2, 6, 3],
                 [0, 0, 3, 5]], dtype=np.float32)


def sets_of(mem):
    return [sorted(np.flatnonzero(r).tolist()) for r in mem]


def test_hand_worked_example_without_overlap():
    # 0 takes its strongest neighbour 1 (4 > 1); 1 is assigned; 2 takes the strongest free neighbour 3 (1 is taken); 3 is assigned
    mem, unplaced = oracle.build_contexts(HAND, B=2, M_max=4, allow_overlap=False)
    assert sets_of(mem) == [[0, 1], [2, 3]] and unplaced == 0


def test_hand_worked_example_with_overlap():
    # B = 3: 0 -> {0,1,2}; 1 -> {1,0,2}, a duplicate; 2 -> {2,3,1} (3 > 2 > 1); 3 -> {3,2}: its only positive neighbour
    mem, unplaced = oracle.build_contexts(HAND, B=3, M_max=4, allow_overlap=True)
    assert sets_of(mem) == [[0, 1, 2], [1, 2, 3], [2, 3]] and unplaced == 0
    # B = 2: the clusters of 1 and 3 repeat those of 0 and 2
    mem, _ = oracle.build_contexts(HAND, B=2, M_max=4, allow_overlap=True)
    assert sets_of(mem) == [[0, 1], [2, 3]]


def test_hand_worked_example_leftover_labels_go_to_the_best_fitting_context_with_room():
    # M_max = 1, B = 3: only {0,1,2} is kept; label 3 is uncovered and the context is full -> unplaced
    mem, unplaced = oracle.build_contexts(HAND, B=3, M_max=1, allow_overlap=False)
    assert sets_of(mem) == [[0, 1, 2]] and unplaced == 1
    # six labels, B = 3, M_max = 2: 0 -> {0,1} (its only neighbour); 2 -> {2,3}; 4 and 5 have no free neighbour left and
    # their singletons are refused (two contexts exist); 4 fits {2,3} (0 + 2 against 0 + 1 for {0,1}) and fills it, 5 then
    # goes to the only context with room although it has no tie to it
    c = np.zeros((6, 6), dtype=np.float32)
    for i, f in enumerate([9, 8, 7, 6, 5, 4]):
        c[i, i] = f
    def link(a, b, v): c[a, b] = c[b, a] = v
    link(0, 1, 5); link(2, 3, 4); link(4, 3, 2); link(4, 1, 1); link(5, 3, 2)
    mem, unplaced = oracle.build_contexts(c, B=3, M_max=2, allow_overlap=False)
    assert sets_of(mem) == [[0, 1, 5], [2, 3, 4]] and unplaced == 0


def test_intra_coherence_hand_worked_and_closed_forms():
    mem = np.array([[1, 1, 0, 0], [0, 0, 1, 1]], dtype=np.uint8)
    # ((4 + 4) / 2 + (3 + 3) / 2) / 2 = 3.5
    assert oracle.intra_coherence(HAND, mem) == pytest.approx(3.5, abs=1e-12)
    assert oracle.intra_coherence(HAND, mem, norm=2.0) == pytest.approx(1.75, abs=1e-12)
    # {0,1,2}: pairs 4,1,4,2,1,2 -> 14 / 6; the singleton contributes 0 but counts as a context
    mem2 = np.array([[1, 1, 1, 0], [0, 0, 0, 1]], dtype=np.uint8)
    assert oracle.intra_coherence(HAND, mem2) == pytest.approx(14 / 6 / 2, abs=1e-12)
    # every pair co-occurs once: the metric is 1 whatever the contexts are
    ones = np.ones((9, 9), dtype=np.float32)
    rnd = synth.make_cover_instance(3, 9, 4, max_size=5)[0]
    rnd[rnd.sum(1) < 2, :2] = 1
    assert oracle.intra_coherence(ones, rnd) == pytest.approx(1.0, abs=1e-12)


@pytest.mark.parametrize("seed", range(5))
def test_intra_coherence_is_the_quadratic_form_of_the_membership_rows(seed):
    rng = np.random.default_rng(seed)
    K, M = 30, 7
    c = rng.integers(0, 50, size=(K, K)).astype(np.float32)
    mem, _ = synth.make_cover_instance(seed, K, M, max_size=6)
    want = 0.0
    for m in mem.astype(np.float64):
        n = m.sum()
        if n >= 2:
            want += (m @ c.astype(np.float64) @ m - (np.diag(c) * m).sum()) / (n * (n - 1))
    assert oracle.intra_coherence(c, mem, norm=3.0) == pytest.approx(want / M / 3.0, rel=1e-12)


def test_planted_groups_are_recovered_as_a_partition():
    cooc, planted, _ = synth.make_cooccurrence()             # 16 groups of 5 with shuffled ids, 15 % stray labels
    for overlap in (False, True):
        mem, unplaced = oracle.build_contexts(cooc, B=5, M_max=16, allow_overlap=overlap)
        assert sorted(sets_of(mem)) == sorted(sorted(p) for p in planted) and unplaced == 0


def py_build(cooc, B, M_max, overlap):
    """A second writing of Alg. 1 with Python sets and sorted()."""
    K = len(cooc)
    valid = [l for l in range(K) if np.any(cooc[l] != 0)]
    visit = sorted(valid, key=lambda l: (-cooc[l, l], l))
    contexts, assigned = [], set()
    for l in visit:
        if not overlap and l in assigned:
            continue
        cand = [j for j in range(K) if j != l and cooc[l, j] > 0 and (overlap or j not in assigned)]
        cand.sort(key=lambda j: (-cooc[l, j], j))
        cluster = {l} | set(cand[:B - 1])
        if cluster not in contexts and len(contexts) < M_max:
            contexts.append(cluster)
            if not overlap:
                assigned |= cluster
    unplaced = 0
    for l in visit:
        if any(l in c for c in contexts):
            continue
        room = [i for i, c in enumerate(contexts) if len(c) < B]
        if not room:
            unplaced += 1
            continue
        best = max(room, key=lambda i: (sum(float(cooc[l, j]) for j in sorted(contexts[i])), -i))
        contexts[best].add(l)
    return [sorted(c) for c in contexts], unplaced


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("overlap", [False, True])
def test_invariants_and_second_writing_on_random_matrices(seed, overlap):
    rng = np.random.default_rng(100 + seed)
    K = int(rng.integers(6, 40))
    B = int(rng.integers(1, 7))
    M_max = int(rng.integers(1, 20))
    c = rng.integers(0, 6, size=(K, K)).astype(np.float32)   # small integers: many ties
    c = np.minimum(c, c.T)
    c[np.diag_indices(K)] = rng.integers(0, 30, size=K)
    dead = rng.choice(K, size=2, replace=False)              # labels that never occur
    c[dead, :] = 0; c[:, dead] = 0
    mem, unplaced = oracle.build_contexts(c, B, M_max, overlap)
    got = sets_of(mem)
    want, want_unplaced = py_build(c, B, M_max, overlap)
    assert got == want and unplaced == want_unplaced
    assert len(got) <= M_max and all(1 <= len(s) <= B for s in got)
    assert not mem[:, dead].any()                            # invalid labels are in no context
    covered = mem.sum(0)
    if not overlap:
        assert covered.max() <= 1                            # contexts are disjoint
    valid = np.array([np.any(c[l] != 0) for l in range(K)])
    assert int((valid & (covered == 0)).sum()) == unplaced   # every valid label is in a context or counted
    if unplaced:
        assert all(len(s) == B for s in got)                 # a label stays out only when no context has room


@pytest.mark.parametrize("seed", range(6))
def test_cluster_around_a_label_maximises_the_co_occurrence_with_it(seed):
    """Brute force: with M_max = 1 the only context is the cluster around the most frequent label, and among all label sets of
    at most B labels that contain it, it has the largest total co-occurrence with that label (strictly: the draws are distinct)."""
    rng = np.random.default_rng(200 + seed)
    K, B = 8, int(rng.integers(2, 5))
    c = rng.permutation(K * K).reshape(K, K).astype(np.float32) + 1.0
    c = np.maximum(c, c.T)
    c[np.diag_indices(K)] = rng.permutation(K) + 100.0
    mem, _ = oracle.build_contexts(c, B, 1, True)
    l = int(np.argmax(np.diag(c)))
    best = max((s for n in range(B) for s in itertools.combinations([j for j in range(K) if j != l], n)),
               key=lambda s: sum(c[l, j] for j in s))
    # (the leftover labels are then inserted into it while it has room; with n = B - 1 neighbours it is full)
    assert sets_of(mem)[0] == sorted((l,) + best)


def test_stream_metrics_closed_forms_and_recount():
    off, ids = synth.sets_to_csr([[1, 2]] * 10)
    assert oracle.stream_metrics(off, ids, 4) == (2.0, 0)
    off, ids = synth.sets_to_csr([[0], [1]] * 5)
    assert oracle.stream_metrics(off, ids, 4) == (1.0, 9)
    off, ids = synth.sets_to_csr([[2, 0], [0, 2], [], [], [3]])          # the same set in another order is no switch
    assert oracle.stream_metrics(off, ids, 4) == (1.0, 2)
    rng = np.random.default_rng(7)
    sets = [sorted(rng.choice(6, size=int(rng.integers(0, 4)), replace=False).tolist()) for _ in range(200)]
    off, ids = synth.sets_to_csr(sets)
    cov, sw = oracle.stream_metrics(off, ids, 6)
    assert cov == pytest.approx(np.mean([len(s) for s in sets])) and sw == sum(a != b for a, b in zip(sets, sets[1:]))
