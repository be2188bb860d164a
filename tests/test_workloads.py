"""The synthetic routing has the structure the configurations name (load skew, distinct ids, gate sums)."""
import numpy as np
import pytest

import oracle
from paper_2603_06626_amd import workloads as wl
from tests.helpers import bf16_to_f64


def _max_vio(idx, E):
    # MaxVio_Global (App. "Maximal Violation"): (max_i L_i - mean L) / mean L
    load = np.bincount(idx.reshape(-1), minlength=E).astype(np.float64)
    return (load.max() - load.mean()) / load.mean()


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_routing_structure(cfg):
    c = wl.CONFIGS[cfg]
    idx, gates = wl.make_routing(cfg, seed=0)
    T, E, k = c["T"], c["E"], c["k"]
    assert idx.shape == (T, k) and idx.dtype == np.int32 and gates.shape == (T, k) and gates.dtype == np.uint16
    assert idx.min() >= 0 and idx.max() < E
    srt = np.sort(idx, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1])                      # k distinct experts per token
    counts, offsets, _, _ = oracle.plan(idx, E)
    assert counts.sum() == T * k                                   # expert counts sum to T*k
    g = bf16_to_f64(gates)
    assert np.all(g > 0) and np.max(np.abs(g.sum(axis=1) - 1.0)) <= 2.0 ** -7 * 1.01
    mv = _max_vio(idx, E)
    if cfg in (2, 3):
        assert 8.0 <= mv + 1.0 <= E / k + 1e-9                     # hottest expert ~10x the mean load
        assert np.argmax(counts) == 0
    elif cfg == 1:
        assert mv < 0.2
    elif cfg == 4:
        assert 1.5 <= counts[0] / counts.mean() <= 1.9             # 5% of tokens forced onto expert 0
        assert _max_vio(idx[:, 1:], E) < 0.3
    elif cfg == 0:
        assert 1.8 <= mv + 1.0 <= 3.2


def test_config3_reuses_config2_tensors():
    a, ga = wl.make_routing(2)
    b, gb = wl.make_routing(3)
    assert np.array_equal(a, b) and np.array_equal(ga, gb)


def test_bf16_rounding_is_nearest_even():
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0, 3.0e38],
                    dtype=np.float32)
    bits = wl.f32_to_bf16_bits(vals)
    back = bf16_to_f64(bits)
    assert back[0] == 1.0 and back[1] == 1.0                       # tie -> even mantissa
    assert back[2] == 1.0 + 2.0 ** -7                              # just above the tie -> up
    assert back[3] == 1.0 + 2.0 ** -6                              # tie -> even (up)
    assert back[4] == -2.5 and back[5] == 0.0
    torch = pytest.importorskip("torch")
    r = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    tb = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(r), tb)


def test_tensors_config0_moments_and_determinism():
    t = wl.make_tensors(0, seed=0)
    t2 = wl.make_tensors(0, seed=0)
    for name in ("x", "W1", "W3", "W2", "dY"):
        assert np.array_equal(t[name], t2[name])
    c = wl.CONFIGS[0]
    assert abs(bf16_to_f64(t["x"]).std() - 1.0) < 0.02
    assert abs(bf16_to_f64(t["W1"]).std() * np.sqrt(c["d"]) - 1.0) < 0.02
    assert abs(bf16_to_f64(t["W2"]).std() * np.sqrt(c["f"]) - 1.0) < 0.02
    assert not np.array_equal(t["W1"], t["W3"])
    assert not np.array_equal(wl.make_tensors(0, seed=1)["x"], t["x"])


def test_flop_convention():
    # forward 6*T*k*d*f, backward twice the forward (App. M: C_fwd = 2NP, C_bwd = 4NP)
    c = wl.CONFIGS[3]
    assert wl.flops(c["T"], c["d"], c["f"], c["k"], bwd=True) == pytest.approx(2551.2e9, rel=1e-4)
    assert wl.flops(c["T"], c["d"], c["f"], c["k"], bwd=False) == pytest.approx(850.40e9, rel=1e-4)
