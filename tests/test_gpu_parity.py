"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: plan arrays bit-exact; every float tensor max|gpu - oracle| <= 1e-2 * max|oracle| over the whole
tensor (bf16 storage, fp32 accumulation), no NaN/Inf.  This file holds the small and medium shapes, compared
element by element; the named full-size configurations live in test_gpu_full_size.py.
"""
import numpy as np
import pytest

import oracle
from paper_2603_06626_amd import workloads as wl
from tests.helpers import rel_max_err

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-2


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util

    return gpu_util


def _widen(bits):
    return oracle.bf16_bits_to_f32(bits)


# -------------------------------------------------------------------------------------------- plan
def _plan_case(gpu, idx, E, dtype=np.int32):
    T, k = idx.shape
    layer = gpu.Layer(T, k, E, 8, 8)
    layer.build_plan(torch.from_numpy(idx.astype(dtype)).to(gpu.DEV))
    got = layer.plan_views()
    ref = oracle.plan(idx.astype(np.int32), E)
    for name, g, r in zip(("counts", "offsets", "row_to_src", "src_to_row"), got, ref):
        assert np.array_equal(g, r), name


@pytest.mark.parametrize("cfg", [0, 1, 2, 4])
def test_plan_named_configs_bit_exact(gpu, cfg):
    idx, _ = wl.make_routing(cfg)
    _plan_case(gpu, idx, wl.CONFIGS[cfg]["E"])


def test_plan_adversarial_inputs(gpu):
    rng = np.random.default_rng(0)
    _plan_case(gpu, np.full((1000, 1), 5, dtype=np.int32), 9)                       # all to one, empty experts
    _plan_case(gpu, np.zeros((1, 1), dtype=np.int32), 1)                            # smallest problem
    _plan_case(gpu, rng.integers(0, 256, size=(777, 3)).astype(np.int32), 256, np.uint8)   # uint8 ids up to 255
    _plan_case(gpu, rng.integers(0, 1024, size=(333, 7)).astype(np.int32), 1024)    # widest E, ragged N
    _plan_case(gpu, rng.integers(0, 3, size=(513, 1)).astype(np.int32), 3)          # one slot past a chunk
    _plan_case(gpu, rng.integers(0, 17, size=(4099, 5)).astype(np.int32), 17)
    relabel = rng.permutation(64).astype(np.int32)                                   # hottest expert is not id 0
    idx, _ = wl.make_routing(2)
    _plan_case(gpu, relabel[idx], 64)


def test_plan_reports_bad_ids_and_host_checks(gpu):
    from paper_2603_06626_amd import binding as b

    idx = np.array([[0, 1], [7, 2]], dtype=np.int32)
    layer = gpu.Layer(2, 2, 4, 8, 8)
    b.grouter_plan_build(torch.from_numpy(idx).to(gpu.DEV), 4, layer.plan)
    with pytest.raises(b.GrouterError) as ei:
        b.grouter_plan_status(layer.plan)
    assert ei.value.code == b.ERR_INDEX_OUT_OF_RANGE
    with pytest.raises(b.GrouterError) as ei:
        b.grouter_plan_build(torch.zeros((4, 2), dtype=torch.int32, device=gpu.DEV), 4, layer.plan[:256])
    assert ei.value.code == b.ERR_WORKSPACE_TOO_SMALL


def test_calls_with_other_dimensions_than_the_plan_write_nothing(gpu):
    """The build records (N, k, E) in the plan; kernels handed a plan together with other dimensions leave at once."""
    from paper_2603_06626_amd import binding as b

    T, d, f, E, k = 64, 16, 16, 4, 2
    idx, gates, t = wl.make_custom(T, d, f, E, k, routing="uniform", seed=3, stream=510)
    layer = gpu.Layer(T, k, E, d, f)
    layer.build_plan(idx)
    g = {n: gpu.to_dev(v) for n, v in t.items()}
    big = torch.empty(b.grouter_plan_bytes(T, k, 2 * E), dtype=torch.uint8, device=gpu.DEV)
    big[:layer.plan.numel()] = layer.plan                    # the plan of E experts, presented as one of 2E experts
    W = {n: torch.cat([g[n], g[n]]) for n in ("W1", "W3", "W2")}
    y = torch.full((T, d), 7.0, dtype=torch.bfloat16, device=gpu.DEV)
    ctx = torch.empty(b.grouter_ctx_bytes(T, k, d, f), dtype=torch.uint8, device=gpu.DEV)
    b.grouter_moe_fwd(big, g["x"], gpu.to_dev(gates), W["W1"], W["W3"], W["W2"], y, ctx)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())


# -------------------------------------------------------------------------------------------- permute / combine
def test_permute_then_combine_is_identity_bit_exact(gpu):
    from paper_2603_06626_amd import binding as b

    T, E, d = 3001, 11, 264
    idx = wl.draw_routing(T, E, 1, "zipf", seed=3, stream=7, zipf_s=1.1)
    x = wl.draw_normal_bf16((T, d), 1.0, 3, 7, "x")
    layer = gpu.Layer(T, 1, E, d, 8)
    layer.build_plan(idx)
    xd = gpu.to_dev(x)
    xp = torch.empty((T, d), dtype=torch.bfloat16, device=gpu.DEV)
    back = torch.empty_like(xd)
    b.grouter_permute(layer.plan, T, 1, E, xd, None, xp)
    _, _, r2s, _ = oracle.plan(idx, E)
    assert np.array_equal(gpu.to_bits(xp), x[r2s])                 # gather is a pure copy
    b.grouter_combine(layer.plan, T, 1, E, xp, None, back)
    assert np.array_equal(gpu.to_bits(back), x)                    # k = 1, weight 1: exact identity


def test_permute_scaled_and_combine_weighted_match_definition(gpu):
    from paper_2603_06626_amd import binding as b

    T, E, k, d = 1237, 13, 4, 136
    idx = wl.draw_routing(T, E, k, "uniform", seed=4, stream=8)
    gates = wl.draw_gates(T, k, seed=4, stream=8)
    x = wl.draw_normal_bf16((T, d), 1.0, 4, 8, "x")
    layer = gpu.Layer(T, k, E, d, 8)
    layer.build_plan(idx)
    _, _, r2s, s2r = oracle.plan(idx, E)
    xf, gf = _widen(x).astype(np.float64), _widen(gates).astype(np.float64)
    xd, gd = gpu.to_dev(x), gpu.to_dev(gates)
    out = torch.empty((T * k, d), dtype=torch.bfloat16, device=gpu.DEV)
    b.grouter_permute(layer.plan, T, k, E, xd, gd, out)            # gate-weighted: w * row
    ref = gf.reshape(-1)[r2s][:, None] * xf[r2s // k]
    assert rel_max_err(gpu.to_f64(out), ref) <= 2.0 ** -8
    rows = wl.draw_normal_bf16((T * k, d), 1.0, 4, 8, "dY")
    y = torch.empty((T, d), dtype=torch.bfloat16, device=gpu.DEV)
    b.grouter_combine(layer.plan, T, k, E, gpu.to_dev(rows), gd, y)
    rf = _widen(rows).astype(np.float64)
    ref = np.einsum("tk,tkd->td", gf, rf[s2r].reshape(T, k, d))
    assert rel_max_err(gpu.to_f64(y), ref) <= 2.0 ** -8


# -------------------------------------------------------------------------------------------- full layer
def _run_and_compare(gpu, idx, gates, t, E, dtype, bwd=True):
    T, k = idx.shape
    d, f = t["x"].shape[1], t["W1"].shape[2]
    layer = gpu.Layer(T, k, E, d, f)
    layer.build_plan(idx)
    g = {n: gpu.to_dev(v) for n, v in t.items()}
    gw = gpu.to_dev(gates)
    y = layer.fwd(g["x"], gw, g["W1"], g["W3"], g["W2"])
    w = lambda a: _widen(a).astype(dtype)
    ref_y = oracle.moe_fwd(w(t["x"]), w(gates), idx, w(t["W1"]), w(t["W3"]), w(t["W2"]), dtype=dtype)
    errs = {"y": rel_max_err(gpu.to_f64(y), ref_y)}
    # the forward-only entry point (rows gathered inside the gate/up GEMM, no saved context) must agree bit for bit
    y_only = layer.fwd_only(g["x"], gw, g["W1"], g["W3"], g["W2"])
    assert np.array_equal(gpu.to_bits(y_only), gpu.to_bits(y)), "forward-only y differs from the training forward"
    if bwd:
        got = layer.bwd(g["x"], gw, g["W1"], g["W3"], g["W2"], g["dY"])
        ref = oracle.moe_bwd(w(t["x"]), w(gates), idx, w(t["W1"]), w(t["W3"]), w(t["W2"]), w(t["dY"]), dtype=dtype)
        for name, a, r in zip(("dX", "dW1", "dW3", "dW2"), got, ref):
            errs[name] = rel_max_err(gpu.to_f64(a), r)
            counts = np.bincount(idx.reshape(-1), minlength=E)
            if name != "dX":
                a64 = gpu.to_f64(a)
                for e in np.flatnonzero(counts == 0):
                    assert np.all(a64[e] == 0.0), f"{name}[{e}] of an empty expert must be zero"
                # per-expert error, reported so a broken cold expert cannot hide behind the hot one's scale
                worst = max((rel_max_err(a64[e], r[e]) for e in np.flatnonzero(counts > 0)), default=0.0)
                print(f"  {name}: whole-tensor {errs[name]:.3e}, worst per-expert {worst:.3e}")
    print("  rel max err:", {n: f"{v:.3e}" for n, v in errs.items()})
    for n, v in errs.items():
        assert v <= TOL, (n, v)
    return layer


def test_config0_fwd_bwd_every_element(gpu):
    idx, gates = wl.make_routing(0)
    _run_and_compare(gpu, idx, gates, wl.make_tensors(0), wl.CONFIGS[0]["E"], np.float64)


@pytest.mark.parametrize("T,d,f,E,k,routing,s", [
    (777, 200, 328, 5, 3, "zipf", 1.0),      # nothing a multiple of the tile sizes: ragged rows, K and N tails
    (64, 8, 8, 4, 2, "uniform", 0.0),        # the narrowest widths the ABI accepts
    (1500, 320, 136, 12, 1, "zipf", 1.5),    # top-1, heavy skew, experts with very few rows
    (2048, 512, 768, 16, 4, "zipf", 1.2),    # several 256-row tiles per expert, several column tiles
])
def test_medium_shapes_every_element(gpu, T, d, f, E, k, routing, s):
    idx, gates, t = wl.make_custom(T, d, f, E, k, routing=routing, zipf_s=s, seed=1, stream=200 + T)
    _run_and_compare(gpu, idx, gates, t, E, np.float32)


def test_seeded_sweep_of_small_shapes(gpu):
    """Ten seeded shapes with every dimension drawn independently (d, f any multiple of 8; k up to E)."""
    rng = np.random.default_rng(2026)
    for case in range(10):
        E = int(rng.integers(1, 20))
        k = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.integers(1, 700))
        d = 8 * int(rng.integers(1, 40))
        f = 8 * int(rng.integers(1, 40))
        routing = ["uniform", "zipf"][case % 2]
        print(f" sweep case {case}: T={T} d={d} f={f} E={E} k={k} {routing}", flush=True)
        idx, gates, t = wl.make_custom(T, d, f, E, k, routing=routing, zipf_s=1.3, seed=7, stream=700 + case)
        _run_and_compare(gpu, idx, gates, t, E, np.float32)


def test_seeded_sweep_around_tile_edges(gpu):
    """Sixteen seeded shapes whose widths sit on and next to the kernels' 128- and 256-column tile edges (the last
    column tile of a GEMM is then full, a few columns wide, just over or just under half: each takes another path
    through the fragment skipping and the epilogue masks), with ragged token counts and skewed routing."""
    rng = np.random.default_rng(4242)
    edges = [8, 24, 120, 128, 136, 248, 256, 264, 376, 384, 392, 504, 512, 520, 640, 776]
    for case in range(16):
        E = int(rng.integers(1, 24))
        k = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.integers(1, 1400))
        d = int(rng.choice(edges))
        f = edges[case]                       # every edge once as the hidden width
        routing = ["uniform", "zipf"][case % 2]
        print(f" edge case {case}: T={T} d={d} f={f} E={E} k={k} {routing}", flush=True)
        idx, gates, t = wl.make_custom(T, d, f, E, k, routing=routing, zipf_s=1.2, seed=9, stream=1200 + case)
        _run_and_compare(gpu, idx, gates, t, E, np.float32)


def test_degenerate_layers(gpu):
    from paper_2603_06626_amd import binding as b

    # one token, one expert, the narrowest widths
    idx, gates, t = wl.make_custom(1, 8, 8, 1, 1, routing="uniform", seed=3, stream=500)
    _run_and_compare(gpu, idx, gates, t, 1, np.float64)
    # every token goes to every expert (k = E)
    idx, gates, t = wl.make_custom(37, 16, 24, 4, 4, routing="uniform", seed=3, stream=501)
    _run_and_compare(gpu, idx, gates, t, 4, np.float64)
    # all tokens to one of many experts: one long run of rows, every other expert empty
    idx, gates, t = wl.make_custom(700, 72, 40, 9, 1, routing="uniform", seed=3, stream=502)
    idx = np.full_like(idx, 6)
    _run_and_compare(gpu, idx, gates, t, 9, np.float32)
    # the largest expert count the ABI accepts, most experts with a handful of rows, many with none
    idx, gates, t = wl.make_custom(900, 16, 24, 1024, 4, routing="zipf", zipf_s=1.1, seed=3, stream=504)
    _run_and_compare(gpu, idx, gates, t, 1024, np.float32)
    # the plan flags an id outside [0,E) and the layer still runs inside its workspaces (the id is handled as expert 0)
    idx, gates, t = wl.make_custom(64, 16, 16, 4, 2, routing="uniform", seed=3, stream=503)
    bad = idx.copy()
    bad[5, 1] = 9
    layer = gpu.Layer(64, 2, 4, 16, 16)
    b.grouter_plan_build(torch.from_numpy(bad).to(gpu.DEV), 4, layer.plan)
    with pytest.raises(b.GrouterError):
        b.grouter_plan_status(layer.plan)
    g = {n: gpu.to_dev(v) for n, v in t.items()}
    y = layer.fwd(g["x"], gpu.to_dev(gates), g["W1"], g["W3"], g["W2"])
    fixed = bad.copy()
    fixed[5, 1] = 0
    w = lambda a: _widen(a).astype(np.float64)
    ref = oracle.moe_fwd(w(t["x"]), w(gates), fixed, w(t["W1"]), w(t["W3"]), w(t["W2"]), dtype=np.float64)
    assert rel_max_err(gpu.to_f64(y), ref) <= TOL


def test_empty_experts_and_duplicate_ids(gpu):
    T, d, f, E, k = 300, 128, 192, 10, 2
    idx, gates, t = wl.make_custom(T, d, f, E, k, routing="uniform", seed=2, stream=300)
    idx = idx.copy()
    idx[idx >= 7] = 1              # experts 7..9 receive nothing; some tokens now hold expert 1 twice
    _run_and_compare(gpu, idx, gates, t, E, np.float64)


def test_expert_relabelling_does_not_change_results(gpu):
    T, d, f, E, k = 512, 128, 256, 8, 2
    idx, gates, t = wl.make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.3, seed=5, stream=400)
    rel = np.random.default_rng(9).permutation(E)       # new id of expert e is rel[e]; hottest is no longer id 0
    inv = np.argsort(rel)
    t2 = dict(t, W1=t["W1"][inv], W3=t["W3"][inv], W2=t["W2"][inv])
    a = _run_and_compare(gpu, idx, gates, t, E, np.float64)
    b_ = _run_and_compare(gpu, rel[idx].astype(np.int32), gates, t2, E, np.float64)
    del a, b_


def test_plan_reuse_and_rerun_is_bit_reproducible(gpu):
    idx, gates = wl.make_routing(0)
    t = wl.make_tensors(0)
    c = wl.CONFIGS[0]
    layer = gpu.Layer(c["T"], c["k"], c["E"], c["d"], c["f"])
    layer.build_plan(idx)
    g = {n: gpu.to_dev(v) for n, v in t.items()}
    gw = gpu.to_dev(gates)
    runs = []
    for _ in range(2):
        y = layer.fwd(g["x"], gw, g["W1"], g["W3"], g["W2"])
        grads = layer.bwd(g["x"], gw, g["W1"], g["W3"], g["W2"], g["dY"])
        runs.append([gpu.to_bits(a) for a in (y, *grads)])
    for a, b_ in zip(*runs):
        assert np.array_equal(a, b_)


def test_gates_attached_to_the_plan_give_the_same_bits(gpu):
    """grouter_plan_set_gates lays the gate weights out in the plan once; the layer called with gate_w = NULL must
    then reproduce, bit for bit, what it computes from an explicit gate_w argument."""
    from paper_2603_06626_amd import binding as b

    T, d, f, E, k = 777, 200, 328, 5, 3
    idx, gates, t = wl.make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.0, seed=1, stream=920)
    layer = gpu.Layer(T, k, E, d, f)
    layer.build_plan(idx)
    g = {n: gpu.to_dev(v) for n, v in t.items()}
    gw = gpu.to_dev(gates)
    y = layer.fwd(g["x"], gw, g["W1"], g["W3"], g["W2"])
    grads = layer.bwd(g["x"], gw, g["W1"], g["W3"], g["W2"], g["dY"])
    ref = [gpu.to_bits(a).copy() for a in (y, *grads)]
    b.grouter_plan_set_gates(layer.plan, E, gw)
    layer.ctx.fill_(0xFF)
    y2 = torch.empty_like(y)
    b.grouter_moe_fwd(layer.plan, g["x"], None, g["W1"], g["W3"], g["W2"], y2, layer.ctx, k=k)
    out = [torch.empty_like(a) for a in grads]
    b.grouter_moe_bwd(layer.plan, g["x"], None, g["W1"], g["W3"], g["W2"], g["dY"], layer.ctx, *out, layer.scratch, k=k)
    y3 = torch.empty_like(y)
    ws = torch.empty(b.grouter_fwd_only_bytes(T, k, d, f), dtype=torch.uint8, device=gpu.DEV)
    b.grouter_moe_fwd_only(layer.plan, g["x"], None, g["W1"], g["W3"], g["W2"], y3, ws, k=k)
    for name, a, r in zip(("y", "dX", "dW1", "dW3", "dW2"), (y2, *out), ref):
        assert np.array_equal(gpu.to_bits(a), r), name
    assert np.array_equal(gpu.to_bits(y3), ref[0])


def test_rerun_is_bit_reproducible_with_long_reductions(gpu):
    """The weight-gradient kernels reduce over an expert's rows 32 at a time; with thousands of rows per
    expert the pipeline runs for dozens of steps per tile (its LDS rings wrap many times).  Two runs on the
    same inputs must agree bit for bit, and a run into poisoned buffers must not depend on their contents."""
    T, d, f, E, k = 2048, 512, 768, 16, 4
    idx, gates, t = wl.make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.2, seed=11, stream=900)
    assert np.bincount(idx.reshape(-1), minlength=E).max() >= 32 * 32      # >= 32 reduction steps in one expert
    layer = gpu.Layer(T, k, E, d, f)
    layer.build_plan(idx)
    g = {n: gpu.to_dev(v) for n, v in t.items()}
    gw = gpu.to_dev(gates)
    runs = []
    for rep in range(3):
        if rep == 2:                                     # same plan, workspaces filled with NaN patterns first
            layer.ctx.fill_(0xFF)
            layer.scratch.fill_(0xFF)
        y = layer.fwd(g["x"], gw, g["W1"], g["W3"], g["W2"])
        grads = layer.bwd(g["x"], gw, g["W1"], g["W3"], g["W2"], g["dY"])
        runs.append([gpu.to_bits(a) for a in (y, *grads)])
    for other in runs[1:]:
        for name, a, b_ in zip(("y", "dX", "dW1", "dW3", "dW2"), runs[0], other):
            assert np.array_equal(a, b_), name


def test_step_replays_from_a_hip_graph(gpu):
    """Plan build + forward + backward enqueue kernels only (no allocation, no synchronisation, nothing that an
    earlier launch must have cleared), so the whole step can be captured once and replayed on new inputs."""
    from paper_2603_06626_amd import binding as b

    T, d, f, E, k = 300, 72, 136, 6, 2
    layer = gpu.Layer(T, k, E, d, f)
    scratch = torch.empty(b.grouter_bwd_scratch_bytes(T, k, d, f), dtype=torch.uint8, device=gpu.DEV)
    problems = [wl.make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.0, seed=s_, stream=600) for s_ in (1, 2, 3)]
    # static buffers the captured graph reads and writes
    idx0, gates0, t0 = problems[0]
    idx_d = torch.from_numpy(idx0).to(gpu.DEV)
    gw = gpu.to_dev(gates0)
    g = {n: gpu.to_dev(v) for n, v in t0.items()}
    y = torch.empty((T, d), dtype=torch.bfloat16, device=gpu.DEV)
    dX = torch.empty_like(y)
    dW1, dW3, dW2 = torch.empty_like(g["W1"]), torch.empty_like(g["W3"]), torch.empty_like(g["W2"])

    def step():
        b.grouter_plan_build(idx_d, E, layer.plan)
        b.grouter_moe_fwd(layer.plan, g["x"], gw, g["W1"], g["W3"], g["W2"], y, layer.ctx)
        b.grouter_moe_bwd(layer.plan, g["x"], gw, g["W1"], g["W3"], g["W2"], g["dY"], layer.ctx, dX, dW1, dW3, dW2, scratch)

    def load(problem):
        idx, gates, t = problem
        idx_d.copy_(torch.from_numpy(idx))
        gw.copy_(gpu.to_dev(gates))
        for n, v in t.items():
            g[n].copy_(gpu.to_dev(v))

    def outputs():
        torch.cuda.synchronize()
        return [gpu.to_bits(a).copy() for a in (y, dX, dW1, dW3, dW2)]

    eager = []
    for pr in problems:
        load(pr)
        step()
        eager.append(outputs())
    load(problems[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in (0, 1, 2, 1, 0):                  # replays on changing inputs, eager work in between
        load(problems[rep])
        for a in (y, dX, dW1, dW3, dW2):
            a.fill_(float("nan"))
        graph.replay()
        got = outputs()
        for name, a, r in zip(("y", "dX", "dW1", "dW3", "dW2"), got, eager[rep]):
            assert np.array_equal(a, r), f"replay on problem {rep}: {name} differs from the eager result"
        b.grouter_plan_status(layer.plan)


def test_next_plan_built_on_a_side_stream_while_a_layer_runs(gpu):
    """Plan streaming: every call takes a stream and a plan is a caller-owned buffer, so the plan of the next
    micro-batch can be built on a side stream while the current one computes.  Results must not change."""
    from paper_2603_06626_amd import binding as b

    T, d, f, E, k = 2048, 256, 384, 16, 4
    batches = [wl.make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.2, seed=s_, stream=800) for s_ in (1, 2, 3)]
    W = {n: gpu.to_dev(batches[0][2][n]) for n in ("W1", "W3", "W2")}
    dev = [(torch.from_numpy(i).to(gpu.DEV), gpu.to_dev(g), gpu.to_dev(t["x"])) for i, g, t in batches]
    plans = [torch.empty(b.grouter_plan_bytes(T, k, E), dtype=torch.uint8, device=gpu.DEV) for _ in range(2)]
    ws = torch.empty(b.grouter_fwd_only_bytes(T, k, d, f), dtype=torch.uint8, device=gpu.DEV)

    def forward(plan, gw, x):
        y = torch.empty((T, d), dtype=torch.bfloat16, device=gpu.DEV)
        b.grouter_moe_fwd_only(plan, x, gw, W["W1"], W["W3"], W["W2"], y, ws)
        return y

    # reference: everything in order on one stream
    ref = []
    for idx_d, gw, x in dev:
        b.grouter_plan_build(idx_d, E, plans[0])
        ref.append(gpu.to_bits(forward(plans[0], gw, x)).copy())
    torch.cuda.synchronize()
    # pipelined: while batch n runs on the main stream, batch n+1's plan is built on the side stream
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    built = [torch.cuda.Event() for _ in dev]
    used = [torch.cuda.Event() for _ in dev]
    b.grouter_plan_build(dev[0][0], E, plans[0])
    built[0].record(main)
    got = []
    for n, (idx_d, gw, x) in enumerate(dev):
        if n + 1 < len(dev):
            with torch.cuda.stream(side):
                if n >= 1:
                    side.wait_event(used[n - 1])         # the buffer being overwritten was last read by batch n-1
                b.grouter_plan_build(dev[n + 1][0], E, plans[(n + 1) % 2], stream=side)
                built[n + 1].record(side)
        main.wait_event(built[n])
        got.append(forward(plans[n % 2], gw, x))
        used[n].record(main)
    torch.cuda.synchronize()
    for n, y in enumerate(got):
        assert np.array_equal(gpu.to_bits(y), ref[n]), f"batch {n}"
    for p_ in plans:
        b.grouter_plan_status(p_)


def test_matrix_core_probe_runs_in_every_mode(gpu):
    """The measurement aid: every mode launches, finishes and reports the FLOP count the header states."""
    b = gpu.b
    sink = torch.empty(16 * 256, dtype=torch.float32, device=gpu.DEV)
    for mode in range(8):
        flop = b.grouter_mfma_probe(mode, 64, 16, sink)
        torch.cuda.synchronize()
        assert flop == 16 * 4 * 64 * 8 * 32768
        assert torch.isfinite(sink).all()
    with pytest.raises(b.GrouterError):
        b.grouter_mfma_probe(0, 64, 32, sink)      # sink holds 16 workgroups only

