"""GPU parity of the routing-statistics entry points against oracle/routing_stats.py.

Integer outputs (affinity counts, loads, comm, best node, co-activation, groups) must match bit for bit.
Float outputs: entropy and MaxVio are fp64 on both sides and differ only by summation order and the log2
routine, tolerance 1e-12 absolute; folded weights are fp32 sums of fp32 inputs against an fp64 oracle,
tolerance 1e-6 * max|oracle| (at most E_S additions of relative error 2^-24 each)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import routing_stats as rs                      # noqa: E402
from paper_2603_06626_amd import binding as b               # noqa: E402
from paper_2603_06626_amd import workloads as wl            # noqa: E402

DEV = "cuda:0"


def node_bits(nodes, E):
    bits = np.zeros(E, dtype=np.uint64)
    for n, members in enumerate(nodes):
        for e in members:
            bits[int(e)] |= np.uint64(1) << np.uint64(n)
    return torch.from_numpy(bits.view(np.int64)).to(DEV)


def run_affinity(idx_t, E):
    S = idx_t.shape[0]
    counts = torch.full((S, E), -7, dtype=torch.int32, device=DEV)
    ent = torch.full((S,), -1.0, dtype=torch.float64, device=DEV)
    loads = torch.full((E,), -5, dtype=torch.int64, device=DEV)
    mv = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    b.grouter_affinity(idx_t, E, counts, ent, loads, mv)
    torch.cuda.synchronize()
    return counts.cpu().numpy(), ent.cpu().numpy(), loads.cpu().numpy(), float(mv.cpu()[0])


def run_placement(idx_t, E, nodes):
    S = idx_t.shape[0]
    comm = torch.full((S, len(nodes)), -7, dtype=torch.int32, device=DEV)
    best = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    b.grouter_sample_placement(idx_t, E, node_bits(nodes, E), len(nodes), comm, best)
    torch.cuda.synchronize()
    return comm.cpu().numpy(), best.cpu().numpy()


def run_coact(idx_t, E):
    P = torch.full((E, E), -3, dtype=torch.int64, device=DEV)
    b.grouter_coactivation(idx_t, E, P)
    torch.cuda.synchronize()
    return P


def check_all(idx_np, E, nodes, E_T_list=(), label=""):
    print(f"routing stats case {label}: idx {idx_np.shape} {idx_np.dtype} E={E} nodes={len(nodes)}", flush=True)
    idx_t = torch.from_numpy(idx_np).to(DEV)
    counts, ent, loads, mv = run_affinity(idx_t, E)
    o_counts = rs.affinity_counts(idx_np, E)
    assert (counts == o_counts).all()
    assert (loads == rs.expert_loads(o_counts)).all()
    assert np.abs(ent - rs.entropy_bits(o_counts)).max() <= 1e-12
    assert abs(mv - rs.maxvio(rs.expert_loads(o_counts))) <= 1e-12
    comm, best = run_placement(idx_t, E, nodes)
    o_comm, o_best = rs.placement(idx_np, nodes, E)
    assert (comm == o_comm).all() and (best == o_best).all()
    # the fused call (one pass over the ids) must give the same eight outputs
    S = idx_np.shape[0]
    f_counts = torch.full((S, E), -7, dtype=torch.int32, device=DEV)
    f_ent = torch.full((S,), -1.0, dtype=torch.float64, device=DEV)
    f_loads = torch.full((E,), -5, dtype=torch.int64, device=DEV)
    f_mv = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    f_comm = torch.full((S, len(nodes)), -7, dtype=torch.int32, device=DEV)
    f_best = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    b.grouter_sample_stats(idx_t, E, f_counts, f_ent, f_loads, f_mv, node_bits(nodes, E), len(nodes), f_comm, f_best)
    torch.cuda.synchronize()
    assert (f_counts.cpu().numpy() == counts).all() and (f_loads.cpu().numpy() == loads).all()
    assert (f_ent.cpu().numpy() == ent).all() and float(f_mv.cpu()[0]) == mv
    assert (f_comm.cpu().numpy() == comm).all() and (f_best.cpu().numpy() == best).all()
    flat = idx_np.reshape(-1, idx_np.shape[-1])
    P = run_coact(idx_t.reshape(-1, idx_np.shape[-1]), E)
    o_P = rs.coactivation(flat, E)
    assert (P.cpu().numpy() == o_P).all()
    for E_T in E_T_list:
        grp = torch.full((E,), -1, dtype=torch.int32, device=DEV)
        b.grouter_fold_groups(P, E_T, grp)
        torch.cuda.synchronize()
        o_grp = rs.fold_groups(o_P, E_T)
        assert (grp.cpu().numpy() == o_grp).all()
        W = wl.draw_score_weights(96, E, seed=E_T)
        out = torch.full((96, E_T), float("nan"), dtype=torch.float32, device=DEV)
        b.grouter_fold_weights(torch.from_numpy(W).to(DEV), grp, E_T, out)
        torch.cuda.synchronize()
        o_out = rs.fold_weights(W, o_grp, E_T)
        assert np.abs(out.cpu().numpy().astype(np.float64) - o_out).max() <= 1e-6 * np.abs(o_out).max()
    return ent


def test_hand_worked_example_on_gpu():
    idx = np.array([[[0, 1], [0, 2], [0, 1], [3, 3]]], dtype=np.int32)
    ent = check_all(idx, 4, [[0, 3], [1, 2]], E_T_list=(2, 4, 1), label="hand-worked")
    assert abs(ent[0] - 1.842370993177108) < 1e-12
    check_all(idx, 4, [[1], [2, 3]], label="hand-worked, tie between nodes")


@pytest.mark.parametrize("dtype", ["uint8", "int32"])
def test_corpus_shape_small(dtype):
    # several staging passes per sample (4096 tokens, 2048 per pass for uint8 k=8), 4 topic nodes
    c = wl.CORPUS
    idx = wl.draw_sequence_routing(24, c["L"], c["E"], c["k"], c["n_topics"], seed=1, dtype=dtype)
    nodes = wl.draw_expert_placement(c["E"], c["n_nodes"], seed=1)
    ent = check_all(idx, c["E"], nodes, E_T_list=(32, 48), label=f"corpus {dtype}")
    assert (ent > 6.85).any() and (ent <= 6.85).any()         # the paper's filter threshold splits this mix


def test_ragged_shapes_duplicates_and_invalid_ids():
    rng = np.random.default_rng(3)
    # L and k chosen so that sample boundaries are not 16-byte aligned and the last staging pass is ragged
    for (S, L, E, k, dt) in [(7, 333, 37, 3, np.uint8), (5, 2500, 200, 7, np.uint8), (3, 1111, 300, 5, np.int32),
                             (2, 50, 1024, 64, np.int32), (9, 1, 5, 1, np.uint8)]:
        idx = rng.integers(0, E, size=(S, L, k)).astype(dt)       # duplicates inside tokens occur
        n_nodes = min(64, E)
        perm = rng.permutation(E)
        nodes = [perm[n::n_nodes] for n in range(n_nodes)]
        if E <= 256:
            check_all(idx, E, nodes, E_T_list=(max(1, E // 3),), label=f"ragged {S}x{L}x{k} E={E}")
        else:
            idx_t = torch.from_numpy(idx).to(DEV)
            counts, ent, loads, mv = run_affinity(idx_t, E)
            o = rs.affinity_counts(idx, E)
            assert (counts == o).all() and np.abs(ent - rs.entropy_bits(o)).max() <= 1e-12
            comm, best = run_placement(idx_t, E, nodes)
            oc, ob = rs.placement(idx, nodes, E)
            assert (comm == oc).all() and (best == ob).all()
    # ids outside [0,E) are ignored: same result as the oracle on the tokens with those slots removed
    E, k = 16, 4
    idx = rng.integers(0, E, size=(3, 100, k)).astype(np.int32)
    bad = idx.copy()
    bad[:, ::7, 1] = E + 5
    bad[:, ::11, 2] = -1
    idx_t = torch.from_numpy(bad).to(DEV)
    counts, _, _, _ = run_affinity(idx_t, E)
    ref = np.zeros((3, E), dtype=np.int64)
    for s in range(3):
        for t in range(100):
            for e in set(int(v) for v in bad[s, t] if 0 <= v < E):
                ref[s, e] += 1
    assert (counts == ref).all()
    # overlapping node sets and an empty node
    comm, best = run_placement(torch.from_numpy(idx).to(DEV), E, [[0, 1, 2], [], [2, 3], list(range(E))])
    oc, ob = rs.placement(idx, [[0, 1, 2], [], [2, 3], list(range(E))], E)
    assert (comm == oc).all() and (best == ob).all()


def test_placement_result_grouped_into_per_node_sample_lists():
    """The assignment sets of the placement algorithm (node -> its samples) are the stable grouping of best_node,
    which is what the plan builder computes: samples of node n are row_to_src[offsets[n]:offsets[n+1]], ascending."""
    c = wl.CORPUS
    S = 300
    idx = wl.draw_sequence_routing(S, 256, c["E"], c["k"], c["n_topics"], seed=5)
    nodes = wl.draw_expert_placement(c["E"], c["n_nodes"], seed=5)
    idx_t = torch.from_numpy(idx).to(DEV)
    comm = torch.empty((S, len(nodes)), dtype=torch.int32, device=DEV)
    best = torch.empty((S,), dtype=torch.int32, device=DEV)
    b.grouter_sample_placement(idx_t, c["E"], node_bits(nodes, c["E"]), len(nodes), comm, best)
    plan = torch.empty(b.grouter_plan_bytes(S, 1, len(nodes)), dtype=torch.uint8, device=DEV)
    b.grouter_plan_build(best.view(S, 1), len(nodes), plan)
    b.grouter_plan_status(plan)
    counts, offsets, row_to_src, _ = (v.cpu().numpy() for v in b.grouter_plan_views(plan, S, 1, len(nodes)))
    _, o_best = rs.placement(idx, nodes, c["E"])
    for n in range(len(nodes)):
        mine = row_to_src[offsets[n]:offsets[n + 1]]
        assert np.array_equal(mine, np.flatnonzero(o_best == n)) and counts[n] == mine.size


def test_coactivation_flushes_its_16_bit_counters():
    # every token activates the same pair: one workgroup sees far more than 2^16 tokens of it
    T, E = 1 << 19, 8
    idx = np.zeros((T, 2), dtype=np.uint8)
    idx[:, 1] = 5
    P = run_coact(torch.from_numpy(idx).to(DEV), E).cpu().numpy()
    ref = np.zeros((E, E), dtype=np.int64)
    ref[0, 0] = ref[5, 5] = ref[0, 5] = ref[5, 0] = T
    assert (P == ref).all()


def test_full_corpus_size_in_the_benchmark_configuration():
    # the shape bench.py times (2048 x 4096 tokens, E = 128, k = 8, uint8), ids drawn on the device
    c = wl.CORPUS
    idx_t = wl.draw_sequence_routing(c["S"], c["L"], c["E"], c["k"], c["n_topics"], seed=0, device=DEV)
    nodes = wl.draw_expert_placement(c["E"], c["n_nodes"], seed=0)
    print("full corpus: affinity", flush=True)
    counts, ent, loads, mv = run_affinity(idx_t, c["E"])
    comm, best = run_placement(idx_t, c["E"], nodes)
    print("full corpus: co-activation", flush=True)
    P = run_coact(idx_t.reshape(-1, c["k"]), c["E"]).cpu().numpy()
    idx = idx_t.cpu().numpy()
    # sampled samples against the oracle one by one
    pick = np.random.default_rng(0).choice(c["S"], size=48, replace=False)
    o_counts = rs.affinity_counts(idx[pick], c["E"])
    assert (counts[pick] == o_counts).all()
    assert np.abs(ent[pick] - rs.entropy_bits(o_counts)).max() <= 1e-12
    o_comm, o_best = rs.placement(idx[pick], nodes, c["E"])
    assert (comm[pick] == o_comm).all() and (best[pick] == o_best).all()
    # properties that hold at any size
    assert (counts.sum(axis=1) == c["L"] * c["k"]).all()                       # ids are distinct per token
    assert (loads == counts.astype(np.int64).sum(axis=0)).all()
    assert abs(mv - (loads.max() / loads.mean() - 1.0)) <= 1e-12
    assert (best == comm.argmax(axis=1)).all() and comm.max() <= c["L"]
    assert (P == P.T).all() and (np.diag(P) == loads).all()
    assert ((P.sum(axis=1) - np.diag(P)) == (c["k"] - 1) * np.diag(P)).all()
    # and the whole co-activation matrix against the oracle (an indicator-matrix product, a few seconds)
    print("full corpus: oracle co-activation", flush=True)
    assert (P == rs.coactivation(idx.reshape(-1, c["k"]), c["E"])).all()
