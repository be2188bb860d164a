"""The forward entry point that allocates nothing (its workspace is a static device array inside the library)
against grouter_moe_fwd_only on the same inputs: y must agree bit for bit, on two calls in a row that share the
array, the second on a smaller problem."""
import numpy as np
import pytest

from paper_2603_06626_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_static_workspace_forward_matches_fwd_only():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_06626_amd import binding as b
    from tests import gpu_util as gpu

    limit = b.grouter_static_ws_bytes()
    assert limit == 64 << 20
    for T, d, f, E, k, stream in ((2048, 512, 768, 16, 4, 910), (300, 72, 136, 6, 2, 911)):   # large first, then small
        assert b.grouter_fwd_only_bytes(T, k, d, f) <= limit
        idx, gates, t = wl.make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.2, seed=13, stream=stream)
        layer = gpu.Layer(T, k, E, d, f)
        layer.build_plan(idx)
        g = {n: gpu.to_dev(v) for n, v in t.items()}
        gw = gpu.to_dev(gates)
        ref = layer.fwd_only(g["x"], gw, g["W1"], g["W3"], g["W2"])
        y = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=gpu.DEV)
        b.grouter_moe_fwd_only_static(layer.plan, g["x"], gw, g["W1"], g["W3"], g["W2"], y)
        torch.cuda.synchronize()
        assert np.array_equal(gpu.to_bits(y), gpu.to_bits(ref)), (T, d, f, E, k)
    # a problem whose workspace exceeds the array is refused on the host
    c = wl.CONFIGS[3]
    assert b.grouter_fwd_only_bytes(c["T"], c["k"], c["d"], c["f"]) > limit
    fake = torch.empty(256, dtype=torch.bfloat16, device=gpu.DEV)
    rc = b.lib().grouter_moe_fwd_only_static(fake.data_ptr(), c["T"], c["k"], c["E"], c["d"], c["f"], fake.data_ptr(),
                                             fake.data_ptr(), fake.data_ptr(), fake.data_ptr(), fake.data_ptr(),
                                             fake.data_ptr(), None)
    assert rc == b.ERR_WORKSPACE_TOO_SMALL
