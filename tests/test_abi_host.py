"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol,
sizes are consistent, and argument errors are caught before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    from paper_2603_06626_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_06626_amd.build import build_library

        build_library()
    return binding


def test_every_declared_symbol_is_exported(b):
    hdr = open(os.path.join(ROOT, "include", "grouter.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(grouter_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(b.EXPORTS)
    L = b.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_workspace_sizes(b):
    assert b.grouter_plan_bytes(0, 1, 1) == 0 and b.grouter_plan_bytes(4, 3, 2) == 0      # k > E
    assert b.grouter_plan_bytes(4, 1, 2000) == 0                                           # E too large
    assert b.grouter_plan_bytes(1 << 31, 2, 4) == 0                                        # T*k overflows int32
    small, big = b.grouter_plan_bytes(256, 2, 8), b.grouter_plan_bytes(16384, 8, 128)
    assert 0 < small < big and small % 256 == 0
    N, d, f = 8192 * 6, 2048, 1408
    assert b.grouter_ctx_bytes(8192, 6, d, f) >= N * d * 2 + 3 * N * f * 2
    assert b.grouter_bwd_scratch_bytes(8192, 6, d, f) >= N * d * 2 + 2 * N * f * 2
    assert b.grouter_ctx_bytes(8192, 6, 2050, f) == 0                                      # d not a multiple of 8
    assert b.grouter_ctx_bytes(1 << 16, 8, 4096, 1536) == 0                                # activation matrix of 2^32 bytes
    assert b.grouter_ctx_bytes(64, 2, 1 << 15, 1 << 15) == 0                               # weight slab of 2^31 bytes
    assert b.grouter_ctx_bytes(16384, 8, 4096, 1536) > 0                                   # the largest configured shape fits
    assert 0 < b.grouter_fwd_only_bytes(8192, 6, d, f) < b.grouter_ctx_bytes(8192, 6, d, f)
    assert b.grouter_fwd_only_bytes(8192, 6, d, f) >= N * f * 2 + N * d * 2


def test_argument_errors_are_reported_on_the_host(b):
    L = b.lib()
    fake = ctypes.c_void_p(256 * 1024)        # never dereferenced: every call below must fail first
    assert L.grouter_plan_build(None, 0, 4, 2, 4, fake, 1 << 20, None) == b.ERR_INVALID_ARG
    assert L.grouter_plan_build(fake, 0, 4, 5, 4, fake, 1 << 20, None) == b.ERR_INVALID_ARG       # k > E
    assert L.grouter_plan_build(fake, 1, 4, 2, 300, fake, 1 << 20, None) == b.ERR_INVALID_ARG     # uint8 ids, E > 256
    assert L.grouter_plan_build(fake, 7, 4, 2, 4, fake, 1 << 20, None) == b.ERR_INVALID_ARG       # unknown dtype
    assert L.grouter_plan_build(fake, 0, 4, 2, 4, fake, 16, None) == b.ERR_WORKSPACE_TOO_SMALL
    assert L.grouter_plan_build(fake, 0, 4, 2, 4, ctypes.c_void_p(264), 1 << 20, None) == b.ERR_INVALID_ARG  # alignment
    args = [fake, 4, 2, 4, 64, 64, fake, fake, fake, fake, fake, fake, fake]
    assert L.grouter_moe_fwd(*args, 16, None) == b.ERR_WORKSPACE_TOO_SMALL
    args[4] = 60                                                                                     # d % 8 != 0
    assert L.grouter_moe_fwd(*args, 1 << 30, None) == b.ERR_INVALID_ARG
    assert L.grouter_permute(fake, 4, 2, 4, 64, None, None, fake, None) == b.ERR_INVALID_ARG
    args[4] = 64
    assert L.grouter_moe_fwd_only(*args, 16, None) == b.ERR_WORKSPACE_TOO_SMALL
    args[5] = 60                                                                                     # f % 8 != 0
    assert L.grouter_moe_fwd_only(*args, 1 << 30, None) == b.ERR_INVALID_ARG
    assert b.lib().grouter_strerror(b.ERR_INDEX_OUT_OF_RANGE).decode() == "expert index out of range"
    assert b.lib().grouter_phase_name(2).decode() == "gateup"
    # routing statistics
    assert L.grouter_affinity(fake, 1, 4, 16, 2, 8, None, fake, fake, fake, None) == b.ERR_INVALID_ARG        # null output
    assert L.grouter_affinity(fake, 1, 4, 16, 2, 300, fake, fake, fake, fake, None) == b.ERR_INVALID_ARG      # uint8, E > 256
    assert L.grouter_affinity(fake, 0, 4, 16, 65, 128, fake, fake, fake, fake, None) == b.ERR_INVALID_ARG     # k > 64
    assert L.grouter_affinity(fake, 0, 0, 16, 2, 8, fake, fake, fake, fake, None) == b.ERR_INVALID_ARG        # no samples
    assert L.grouter_sample_placement(fake, 0, 4, 16, 2, 8, fake, 65, fake, fake, None) == b.ERR_INVALID_ARG  # > 64 nodes
    assert L.grouter_sample_placement(fake, 0, 4, 0, 2, 8, fake, 4, fake, fake, None) == b.ERR_INVALID_ARG    # empty samples
    assert L.grouter_coactivation(fake, 0, 100, 2, 257, fake, None) == b.ERR_INVALID_ARG                     # E > 256
    assert L.grouter_fold_groups(fake, 8, 9, fake, None) == b.ERR_INVALID_ARG                                # E_T > E_S
    assert L.grouter_fold_groups(fake, 2000, 4, fake, None) == b.ERR_INVALID_ARG                             # E_S too large
    assert L.grouter_fold_weights(fake, fake, 0, 8, 4, fake, None) == b.ERR_INVALID_ARG                      # d = 0
    assert b.lib().grouter_phase_name(13).decode() == "coactivation"
    # plan-side gates and the measurement aids
    assert L.grouter_plan_set_gates(fake, 4, 2, 4, None, None) == b.ERR_INVALID_ARG                          # no gates
    assert L.grouter_plan_set_gates(fake, 4, 5, 4, fake, None) == b.ERR_INVALID_ARG                          # k > E
    assert L.grouter_mfma_probe(8, 4, 8, fake, 8 * 256, None) == b.ERR_INVALID_ARG                           # unknown mode
    assert L.grouter_mfma_probe(0, 6, 8, fake, 8 * 256, None) == b.ERR_INVALID_ARG                           # iters % 4 != 0
    assert L.grouter_mfma_probe(0, 4, 8, fake, 8 * 256 - 1, None) == b.ERR_WORKSPACE_TOO_SMALL               # sink too small
    assert L.grouter_mfma_probe(0, 4, 8, None, 8 * 256, None) == b.ERR_INVALID_ARG


def test_missing_library_fails_loudly(b, monkeypatch):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError):
        b.lib()
