"""Pins for the routing-statistics oracle (oracle/routing_stats.py): each test checks it against something
other than itself - a hand-worked example, closed forms, invariants, brute force over tiny inputs."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import routing_stats as rs
from paper_2603_06626_amd import workloads as wl


def _golden(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "routing_stats_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, *vals = line.split()
            out[name] = [float(v) for v in vals]
    return out


def test_hand_worked_example(golden_dir):
    g = _golden(golden_dir)
    idx = np.array(g["ids"], dtype=np.int32).reshape(1, 4, 2)
    counts = rs.affinity_counts(idx, 4)
    assert counts.tolist() == [[int(v) for v in g["counts"]]]
    assert np.allclose(rs.affinity(idx, 4)[0], g["phi"], rtol=0, atol=1e-15)
    assert abs(rs.entropy_bits(counts)[0] - g["entropy_bits"][0]) < 1e-14
    assert abs(rs.maxvio(rs.expert_loads(counts)) - g["maxvio"][0]) < 1e-15
    comm, best = rs.placement(idx, [[0, 3], [1, 2]], 4)
    assert comm.tolist() == [[int(v) for v in g["placement_a_comm"]]] and best.tolist() == [int(g["placement_a_best"][0])]
    comm, best = rs.placement(idx, [[1], [2, 3]], 4)
    assert comm.tolist() == [[int(v) for v in g["placement_b_comm"]]] and best.tolist() == [int(g["placement_b_best"][0])]
    P = rs.coactivation(idx.reshape(-1, 2), 4)
    assert P.reshape(-1).tolist() == [int(v) for v in g["coactivation"]]
    grp = rs.fold_groups(P, 2)
    assert grp.tolist() == [int(v) for v in g["fold_group_of"]]
    W = np.array(g["fold_weights_in"], dtype=np.float32).reshape(1, 4)
    assert rs.fold_weights(W, grp, 2).tolist() == [g["fold_weights_out"]]


def test_affinity_closed_forms():
    E, k, L = 16, 4, 64
    # token t takes experts (t*k + j) mod E: every expert is chosen by exactly L*k/E tokens
    idx = ((np.arange(L)[:, None] * k + np.arange(k)[None, :]) % E).astype(np.int32)[None]
    c = rs.affinity_counts(idx, E)
    assert (c == L * k // E).all()
    assert np.allclose(rs.affinity(idx, E), k / E)
    assert abs(rs.entropy_bits(c)[0] - math.log2(E)) < 1e-12          # uniform distribution: log2 E bits
    assert rs.maxvio(rs.expert_loads(c)) == 0.0
    # every token picks the same k experts: phi = 1 on those, entropy = log2 k
    idx = np.tile(np.array([3, 7, 8, 15], dtype=np.int32), (1, L, 1))
    c = rs.affinity_counts(idx, E)
    assert c[0, [3, 7, 8, 15]].tolist() == [L] * 4 and c.sum() == 4 * L
    assert abs(rs.entropy_bits(c)[0] - 2.0) < 1e-12
    # everything on one expert, k = 1: MaxVio = (T - T/E)/(T/E) = E - 1, entropy 0
    idx = np.full((1, L, 1), 5, dtype=np.int32)
    c = rs.affinity_counts(idx, E)
    assert rs.entropy_bits(c)[0] == 0.0
    assert abs(rs.maxvio(rs.expert_loads(c)) - (E - 1)) < 1e-12
    # an empty sample
    assert rs.entropy_bits(np.zeros((1, E), dtype=np.int32))[0] == 0.0


def test_affinity_against_python_loops_and_bincount():
    rng = np.random.default_rng(5)
    S, L, E, k = 5, 37, 11, 3
    idx = rng.integers(0, E, size=(S, L, k)).astype(np.int32)        # duplicates inside tokens do occur
    c = rs.affinity_counts(idx, E)
    for s in range(S):
        ref = [0] * E
        for t in range(L):
            for e in set(int(v) for v in idx[s, t]):
                ref[e] += 1
        assert c[s].tolist() == ref
    # distinct ids: membership counts equal a plain histogram of the slots
    d = wl.draw_sequence_routing(4, 200, 32, 4, seed=3)
    c = rs.affinity_counts(d, 32)
    for s in range(4):
        assert (c[s] == np.bincount(d[s].reshape(-1), minlength=32)).all()
    assert (c.sum(axis=1) == 200 * 4).all()
    # entropy against scipy's definition
    from scipy.stats import entropy
    H = rs.entropy_bits(c)
    for s in range(4):
        assert abs(H[s] - entropy(c[s].astype(np.float64), base=2)) < 1e-12


def test_maxvio_of_the_generator_configs():
    # the zipf configs were specified to have a hottest expert ~10x the mean: (max - mean)/mean in [7.5, 9.7]
    idx, _ = wl.make_routing(2)
    c = rs.affinity_counts(idx[None], 64)
    v = rs.maxvio(rs.expert_loads(c))
    assert 7.5 < v < 64 / 6 - 1
    loads = np.bincount(idx.reshape(-1), minlength=64)
    assert abs(v - (loads.max() / loads.mean() - 1)) < 1e-12


def test_placement_properties_and_brute_force():
    rng = np.random.default_rng(11)
    S, L, E, k, N = 6, 50, 12, 3, 4
    idx = np.stack([np.stack([rng.permutation(E)[:k] for _ in range(L)]) for _ in range(S)]).astype(np.int32)
    nodes = [list(range(n, E, N)) for n in range(N)]
    comm, best = rs.placement(idx, nodes, E)
    for s in range(S):
        for n in range(N):
            ref = sum(1 for t in range(L) if set(int(v) for v in idx[s, t]) & set(nodes[n]))
            assert comm[s, n] == ref
        assert best[s] == min(n for n in range(N) if comm[s, n] == comm[s].max())
    # one node holding every expert sees every token
    comm, best = rs.placement(idx, [list(range(E))], E)
    assert (comm == L).all() and (best == 0).all()
    # k = 1 and a partition of the experts: every token is local to exactly one node
    idx1 = idx[:, :, :1]
    comm, _ = rs.placement(idx1, nodes, E)
    assert (comm.sum(axis=1) == L).all()
    node_of = np.zeros(E, dtype=np.int64)
    for n, m in enumerate(nodes):
        node_of[m] = n
    for s in range(S):
        assert (comm[s] == np.bincount(node_of[idx1[s, :, 0]], minlength=N)).all()
    # overlapping expert sets and an empty node are legal
    comm, best = rs.placement(idx, [[0, 1, 2], [], [2, 3]], E)
    assert (comm[:, 1] == 0).all()
    # inclusion-exclusion with k = 2 over a partition: sum_n comm = 2L - (tokens with both experts on one node)
    idx2 = idx[:, :, :2]
    comm, _ = rs.placement(idx2, nodes, E)
    same = (node_of[idx2[..., 0]] == node_of[idx2[..., 1]]).sum(axis=1)
    assert (comm.sum(axis=1) == 2 * L - same).all()


def test_placement_prefers_the_node_that_holds_the_topic():
    c = dict(S=12, L=512, E=32, k=4, n_topics=4)
    idx = wl.draw_sequence_routing(c["S"], c["L"], c["E"], c["k"], c["n_topics"], seed=2)
    nodes = wl.draw_expert_placement(c["E"], 4, seed=2, aligned=True)
    comm, best = rs.placement(idx, nodes, c["E"])
    # a sequence's best node is the one whose experts have the largest total affinity count there
    counts = rs.affinity_counts(idx, c["E"])
    mass = np.stack([counts[:, m].sum(axis=1) for m in nodes], axis=1)
    agree = (mass.argmax(axis=1) == best).mean()
    assert agree >= 0.75


def test_coactivation_properties_and_brute_force():
    rng = np.random.default_rng(21)
    T, E, k = 300, 9, 3
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)           # with duplicates
    P = rs.coactivation(idx, E, block=64)                            # several blocks
    ref = np.zeros((E, E), dtype=np.int64)
    for t in range(T):
        members = set(int(v) for v in idx[t])
        for i, j in itertools.product(members, members):
            ref[i, j] += 1
    assert (P == ref).all()
    assert (P == P.T).all()
    # distinct ids: diagonal = histogram, off-diagonal row sums = (k-1) * diagonal, total = T*k*k
    d = wl.draw_routing(500, 16, 4, "zipf", seed=4, zipf_s=1.0)
    P = rs.coactivation(d, 16)
    assert (np.diag(P) == np.bincount(d.reshape(-1), minlength=16)).all()
    assert ((P.sum(axis=1) - np.diag(P)) == 3 * np.diag(P)).all()
    assert P.sum() == 500 * 16
    # k = 1: diagonal only
    P1 = rs.coactivation(d[:, :1], 16)
    assert (P1 == np.diag(np.diag(P1))).all()


def test_fold_groups_sizes_partition_and_greedy_rule():
    rng = np.random.default_rng(8)
    for E_S, E_T in [(10, 3), (12, 4), (7, 7), (9, 1), (16, 5)]:
        A = rng.integers(0, 50, size=(E_S, E_S))
        P = (A + A.T).astype(np.int64)
        grp = rs.fold_groups(P, E_T)
        sizes = np.bincount(grp, minlength=E_T)
        g_avg, n_extra = divmod(E_S, E_T)
        assert sizes.tolist() == [g_avg + 1] * n_extra + [g_avg] * (E_T - n_extra)
        assert grp.min() >= 0 and grp.max() == E_T - 1
    # E_T = E_S: each expert alone, numbered in order; E_T = 1: one group
    assert P.shape == (16, 16)
    assert rs.fold_groups(P, 16).tolist() == list(range(16))
    assert (rs.fold_groups(P, 1) == 0).all()
    # block-diagonal co-activation: the blocks are recovered whatever the numbering
    E_S, E_T = 12, 3
    perm = rng.permutation(E_S)
    block = perm % E_T                                                # hidden block of each expert
    P = np.where(block[:, None] == block[None, :], 100, 1).astype(np.int64)
    grp = rs.fold_groups(P, E_T)
    for g in range(E_T):
        assert len(set(block[grp == g])) == 1
    # ties go to the lowest expert number: all-equal P gives consecutive runs
    assert rs.fold_groups(np.ones((6, 6), dtype=np.int64), 3).tolist() == [0, 0, 1, 1, 2, 2]
    # a hand-checked greedy trace where the second pick depends on the sum over both members
    P = np.array([[0, 5, 4, 0, 0, 0],
                  [5, 0, 0, 1, 0, 3],
                  [4, 0, 0, 3, 0, 0],
                  [0, 1, 3, 0, 0, 0],
                  [0, 0, 0, 0, 0, 9],
                  [0, 3, 0, 0, 9, 0]], dtype=np.int64)
    # group 0: start 0, take 1 (5 > 4), then scores 2:4+0=4, 3:0+1=1, 4:0, 5:0+3=3 -> take 2; group 1 = {3,4,5}
    assert rs.fold_groups(P, 2).tolist() == [0, 0, 0, 1, 1, 1]


def test_fold_weights_properties():
    rng = np.random.default_rng(9)
    d, E_S, E_T = 7, 10, 4
    W = rng.standard_normal((d, E_S)).astype(np.float32)
    grp = rng.integers(0, E_T, size=E_S).astype(np.int32)
    F = rs.fold_weights(W, grp, E_T)
    assert F.shape == (d, E_T)
    assert np.allclose(F.sum(axis=1), W.astype(np.float64).sum(axis=1), atol=1e-12)   # M's rows each hold a single 1
    for g in range(E_T):
        assert np.allclose(F[:, g], W[:, grp == g].astype(np.float64).sum(axis=1), atol=1e-12)
    # identity grouping keeps W, a permutation grouping permutes its columns
    assert (rs.fold_weights(W, np.arange(E_S), E_S) == W.astype(np.float64)).all()
    p = rng.permutation(E_S)
    assert (rs.fold_weights(W, p, E_S)[:, p] == W.astype(np.float64)).all()
    # folding scores commutes with folding weights: (h W) M == h (W M)
    h = rng.standard_normal(d)
    M = np.zeros((E_S, E_T))
    M[np.arange(E_S), grp] = 1
    assert np.allclose((h @ W.astype(np.float64)) @ M, h @ F, atol=1e-12)


def test_corpus_generator_structure():
    c = wl.CORPUS
    idx = wl.draw_sequence_routing(16, 1024, c["E"], c["k"], c["n_topics"], seed=0)
    assert idx.dtype == np.uint8 and idx.shape == (16, 1024, c["k"])
    srt = np.sort(idx, axis=-1)
    assert (srt[..., 1:] != srt[..., :-1]).all()                      # k distinct experts per token
    H = rs.entropy_bits(rs.affinity_counts(idx, c["E"]))
    assert H.max() <= math.log2(c["E"]) and H.min() > math.log2(c["k"])
    assert H.max() - H.min() > 0.5                                    # flat and peaked sequences both occur
    nodes = wl.draw_expert_placement(c["E"], c["n_nodes"])
    allm = np.sort(np.concatenate(nodes))
    assert (allm == np.arange(c["E"])).all()
