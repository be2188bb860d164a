"""Pins of the CPU oracle against things other than itself.

Each test fixes the oracle to a closed form, a library routine (numpy matmul / stable argsort, torch
autograd on the dense form of Eq. 1), an invariant, or brute force, so that a dropped term, a wrong
sign or index, or a transposed operand in the oracle fails at least one of them.
"""
import os

import numpy as np
import pytest

import oracle
from tests.helpers import expert_subproblem, rel_max_err, token_subproblem


def _rand_problem(seed, T, d, f, E, k, distinct=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    W1 = rng.standard_normal((E, d, f)) / np.sqrt(d)
    W3 = rng.standard_normal((E, d, f)) / np.sqrt(d)
    W2 = rng.standard_normal((E, f, d)) / np.sqrt(f)
    if distinct:
        idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    else:
        idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    w = rng.random((T, k)) + 0.1
    dY = rng.standard_normal((T, d))
    return x, w, idx, W1, W3, W2, dY


def _silu(g):
    return g / (1.0 + np.exp(-g))


def _dense_swiglu(x, W1, W3, W2):
    return (_silu(x @ W1) * (x @ W3)) @ W2


# ---------------------------------------------------------------- closed form (tests/golden)
def test_scalar_worked_example(golden_dir):
    gold = {}
    with open(os.path.join(golden_dir, "scalar_swiglu_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, val = line.split()
            gold[name] = float(val)
    one = lambda v: np.array([[v]], dtype=np.float64)
    x, w, idx = one(1.0), one(0.5), np.array([[0]], dtype=np.int32)
    W1, W3, W2 = one(1.0)[None], one(2.0)[None], one(3.0)[None]
    y = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    dX, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, one(1.0))
    assert abs(y.item() - gold["y"]) < 1e-14
    assert abs(dX.item() - gold["dX"]) < 1e-14
    assert abs(dW1.item() - gold["dW1"]) < 1e-14
    assert abs(dW3.item() - gold["dW3"]) < 1e-14
    assert abs(dW2.item() - gold["dW2"]) < 1e-14
    y32 = oracle.moe_fwd(x, w, idx, W1, W3, W2, dtype=np.float32)
    assert abs(float(y32.item()) - gold["y"]) < 1e-6


def test_silu_special_values():
    # silu(0) = 0 and silu'(0) = 1/2: with W1 = 0 the gate branch is 0 => y = 0, dW3 = 0, dX = 0 + via-gate term
    x, w, idx, W1, W3, W2, dY = _rand_problem(1, 6, 4, 5, 3, 2)
    y = oracle.moe_fwd(x, w, idx, np.zeros_like(W1), W3, W2)
    assert np.all(y == 0.0)
    dX, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, np.zeros_like(W1), W3, W2, dY)
    assert np.all(dW3 == 0.0) and np.all(dW2 == 0.0) and np.all(dX == 0.0)
    # d silu(g)/dg at 0 is 1/2:  dW1_e = sum_slots x (x) (dh * u * 1/2)
    k = idx.shape[1]
    ref = np.zeros_like(W1)
    for t in range(x.shape[0]):
        for j in range(k):
            e = idx[t, j]
            dh = W2[e] @ (w[t, j] * dY[t])
            ref[e] += np.outer(x[t], dh * (x[t] @ W3[e]) * 0.5)
    assert rel_max_err(dW1, ref) < 1e-13
    # zero input => zero output
    assert np.all(oracle.moe_fwd(np.zeros_like(x), w, idx, W1, W3, W2) == 0.0)


# ---------------------------------------------------------------- special cases = library routines
def test_top1_weight1_equals_per_expert_dense_ffn():
    T, d, f, E = 37, 12, 20, 5
    x, _, _, W1, W3, W2, _ = _rand_problem(2, T, d, f, E, 1)
    idx = np.random.default_rng(3).integers(0, E, size=(T, 1)).astype(np.int32)
    w = np.ones((T, 1))
    y = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    ref = np.zeros((T, d))
    for e in range(E):
        m = idx[:, 0] == e
        ref[m] = _dense_swiglu(x[m], W1[e], W3[e], W2[e])
    assert rel_max_err(y, ref) < 1e-13


def test_all_to_one_expert_equals_single_dense_swiglu():
    T, d, f, E = 29, 16, 24, 4
    x, _, _, W1, W3, W2, _ = _rand_problem(4, T, d, f, E, 1)
    idx = np.full((T, 1), 2, dtype=np.int32)
    y = oracle.moe_fwd(x, np.ones((T, 1)), idx, W1, W3, W2)
    assert rel_max_err(y, _dense_swiglu(x, W1[2], W3[2], W2[2])) < 1e-13
    y32 = oracle.moe_fwd(x, np.ones((T, 1)), idx, W1, W3, W2, dtype=np.float32)
    assert rel_max_err(y32, _dense_swiglu(x, W1[2], W3[2], W2[2])) < 1e-5


def test_forward_equals_dense_sum_over_all_experts():
    # Eq. 1 literally: y = sum_{i=1..E} r_i f_i(x) with r the E-vector that is zero off the top-k.
    T, d, f, E, k = 23, 10, 14, 6, 3
    x, w, idx, W1, W3, W2, _ = _rand_problem(5, T, d, f, E, k)
    R = np.zeros((T, E))
    for t in range(T):
        for j in range(k):
            R[t, idx[t, j]] += w[t, j]
    ref = sum(R[:, e:e + 1] * _dense_swiglu(x, W1[e], W3[e], W2[e]) for e in range(E))
    assert rel_max_err(oracle.moe_fwd(x, w, idx, W1, W3, W2), ref) < 1e-13


def test_backward_equals_autograd_of_dense_form():
    torch = pytest.importorskip("torch")
    T, d, f, E, k = 19, 9, 13, 5, 2
    x, w, idx, W1, W3, W2, dY = _rand_problem(6, T, d, f, E, k)
    R = np.zeros((T, E))
    for t in range(T):
        for j in range(k):
            R[t, idx[t, j]] += w[t, j]
    tx, tW1, tW3, tW2 = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, W1, W3, W2))
    tR = torch.tensor(R)
    y = 0
    for e in range(E):
        y = y + tR[:, e:e + 1] * ((torch.nn.functional.silu(tx @ tW1[e]) * (tx @ tW3[e])) @ tW2[e])
    (y * torch.tensor(dY)).sum().backward()
    dX, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    assert rel_max_err(dX, tx.grad.numpy()) < 1e-12
    assert rel_max_err(dW1, tW1.grad.numpy()) < 1e-12
    assert rel_max_err(dW3, tW3.grad.numpy()) < 1e-12
    assert rel_max_err(dW2, tW2.grad.numpy()) < 1e-12


# ---------------------------------------------------------------- brute-force finite differences
def test_gradients_match_central_finite_differences():
    T, d, f, E, k = 5, 3, 4, 3, 2
    x, w, idx, W1, W3, W2, dY = _rand_problem(7, T, d, f, E, k)
    dX, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    loss = lambda x_, W1_, W3_, W2_: float(np.sum(oracle.moe_fwd(x_, w, idx, W1_, W3_, W2_) * dY))
    eps = 1e-5
    args = [x, W1, W3, W2]
    for which, grad in enumerate((dX, dW1, dW3, dW2)):
        fd = np.zeros_like(grad)
        base = args[which]
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            plus = [a.copy() for a in args]
            minus = [a.copy() for a in args]
            plus[which][mi] += eps
            minus[which][mi] -= eps
            fd[mi] = (loss(*plus) - loss(*minus)) / (2 * eps)
        assert rel_max_err(grad, fd) < 1e-6, which


def test_empty_expert_gets_zero_weight_gradient():
    T, d, f, E, k = 11, 4, 6, 5, 2
    x, w, idx, W1, W3, W2, dY = _rand_problem(8, T, d, f, E, k)
    idx[idx == 3] = 0  # expert 3 receives nothing (duplicates inside a token are legal)
    _, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    assert np.all(dW1[3] == 0) and np.all(dW3[3] == 0) and np.all(dW2[3] == 0)
    assert np.any(dW1[0] != 0)


# ---------------------------------------------------------------- symmetries and linearity
def test_token_permutation_equivariance_and_expert_relabelling():
    T, d, f, E, k = 17, 6, 8, 4, 2
    x, w, idx, W1, W3, W2, dY = _rand_problem(9, T, d, f, E, k)
    y = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    dX, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    perm = np.random.default_rng(10).permutation(T)
    y_p = oracle.moe_fwd(x[perm], w[perm], idx[perm], W1, W3, W2)
    g_p = oracle.moe_bwd(x[perm], w[perm], idx[perm], W1, W3, W2, dY[perm])
    assert np.array_equal(y_p, y[perm]) and np.array_equal(g_p[0], dX[perm])
    assert rel_max_err(g_p[1], dW1) < 1e-13 and rel_max_err(g_p[3], dW2) < 1e-13
    rel = np.random.default_rng(11).permutation(E)  # new id of old expert e is rel[e]
    inv = np.argsort(rel)
    y_r = oracle.moe_fwd(x, w, rel[idx].astype(np.int32), W1[inv], W3[inv], W2[inv])
    g_r = oracle.moe_bwd(x, w, rel[idx].astype(np.int32), W1[inv], W3[inv], W2[inv], dY)
    assert np.array_equal(y_r, y) and np.array_equal(g_r[0], dX)
    assert np.array_equal(g_r[1][rel], dW1) and np.array_equal(g_r[2][rel], dW3) and np.array_equal(g_r[3][rel], dW2)


def test_linearity_in_gates_and_upstream_gradient():
    x, w, idx, W1, W3, W2, dY = _rand_problem(12, 13, 5, 7, 4, 2)
    y = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    assert rel_max_err(oracle.moe_fwd(x, 4.0 * w, idx, W1, W3, W2), 4.0 * y) < 1e-14
    g1 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    g2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, -2.0 * dY)
    for a, b in zip(g1, g2):
        assert rel_max_err(b, -2.0 * a) < 1e-14


def test_duplicate_expert_in_one_token_contributes_twice():
    x, w, _, W1, W3, W2, _ = _rand_problem(13, 4, 5, 6, 3, 2)
    idx = np.array([[1, 1], [0, 2], [2, 2], [1, 0]], dtype=np.int32)
    y = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    assert rel_max_err(y[0], (w[0, 0] + w[0, 1]) * _dense_swiglu(x[0:1], W1[1], W3[1], W2[1])[0]) < 1e-13


def test_f32_instance_tracks_f64_instance():
    x, w, idx, W1, W3, W2, dY = _rand_problem(14, 64, 96, 80, 6, 2)
    f = lambda a: a.astype(np.float32)
    y64 = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    y32 = oracle.moe_fwd(f(x), f(w), idx, f(W1), f(W3), f(W2), dtype=np.float32)
    assert y32.dtype == np.float32 and rel_max_err(y32, y64) < 1e-5
    g64 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    g32 = oracle.moe_bwd(f(x), f(w), idx, f(W1), f(W3), f(W2), f(dY), dtype=np.float32)
    for a, b in zip(g32, g64):
        assert rel_max_err(a, b) < 1e-5


# ---------------------------------------------------------------- plan
def _check_plan_invariants(idx, E, counts, offsets, r2s, s2r):
    flat = idx.reshape(-1)
    N = flat.size
    assert counts.sum() == N
    assert offsets[0] == 0 and offsets[E] == N and np.all(np.diff(offsets) == counts)
    assert np.array_equal(np.sort(r2s), np.arange(N))
    assert np.array_equal(s2r[r2s], np.arange(N))
    assert np.all(np.diff(flat[r2s]) >= 0)
    for e in range(E):
        seg = r2s[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


@pytest.mark.parametrize("T,E,k,seed", [(1, 1, 1, 0), (7, 3, 2, 1), (256, 8, 2, 2), (1000, 256, 8, 3), (513, 17, 5, 4)])
def test_plan_is_the_stable_sort(T, E, k, seed):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    counts, offsets, r2s, s2r = oracle.plan(idx, E)
    _check_plan_invariants(idx, E, counts, offsets, r2s, s2r)
    flat = idx.reshape(-1)
    assert np.array_equal(r2s, np.argsort(flat, kind="stable"))          # library routine
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    if flat.size <= 2000:                                                 # brute-force rank count
        for i in range(flat.size):
            rank = int(np.sum(flat < flat[i]) + np.sum(flat[:i] == flat[i]))
            assert s2r[i] == rank


def test_plan_edge_cases():
    counts, offsets, r2s, s2r = oracle.plan(np.full((50, 1), 3, dtype=np.int32), 6)  # all to one, others empty
    assert counts.tolist() == [0, 0, 0, 50, 0, 0] and offsets.tolist() == [0, 0, 0, 0, 50, 50, 50]
    assert np.array_equal(r2s, np.arange(50)) and np.array_equal(s2r, np.arange(50))
    counts, offsets, r2s, s2r = oracle.plan(np.array([[255, 0], [0, 255]], dtype=np.int32), 256)  # uint8 range end
    assert counts[255] == 2 and counts[0] == 2 and r2s.tolist() == [1, 2, 0, 3]
    with pytest.raises(ValueError):
        oracle.plan(np.array([[0, 4]], dtype=np.int32), 4)
    with pytest.raises(ValueError):
        oracle.plan(np.array([[-1, 0]], dtype=np.int32), 4)


def test_permute_then_unpermute_is_identity():
    # k = 1, gate 1, experts that act as the identity on a 1-hot-free construction are not available for
    # SwiGLU, so check the index algebra itself: gathering by row_to_src then reading through src_to_row
    # returns every slot's own token.
    rng = np.random.default_rng(5)
    T, E, k = 300, 9, 3
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    _, _, r2s, s2r = oracle.plan(idx, E)
    x = rng.standard_normal((T, 4))
    xp = x[r2s // k]                     # permute
    back = xp[s2r].reshape(T, k, 4)      # un-permute, one copy per slot
    assert np.array_equal(back, np.repeat(x[:, None, :], k, axis=1))


# ---------------------------------------------------------------- sub-problem helpers used at full size
def test_subproblems_reproduce_full_problem_rows():
    x, w, idx, W1, W3, W2, dY = _rand_problem(15, 40, 8, 10, 6, 3)
    y = oracle.moe_fwd(x, w, idx, W1, W3, W2)
    dX, dW1, dW3, dW2 = oracle.moe_bwd(x, w, idx, W1, W3, W2, dY)
    sel = [3, 17, 39, 0]
    sp = token_subproblem(sel, x, w, idx, W1, W3, W2, dY)
    assert np.array_equal(oracle.moe_fwd(sp["x"], sp["w"], sp["idx"], sp["W1"], sp["W3"], sp["W2"]), y[sel])
    assert np.array_equal(oracle.moe_bwd(sp["x"], sp["w"], sp["idx"], sp["W1"], sp["W3"], sp["W2"], sp["dY"])[0], dX[sel])
    for e in (0, 4):
        ep = expert_subproblem(e, x, w, idx, W1, W3, W2, dY)
        g = oracle.moe_bwd(ep["x"], ep["w"], ep["idx"], ep["W1"], ep["W3"], ep["W2"], ep["dY"])
        assert np.array_equal(g[1][0], dW1[e]) and np.array_equal(g[2][0], dW3[e]) and np.array_equal(g[3][0], dW2[e])
