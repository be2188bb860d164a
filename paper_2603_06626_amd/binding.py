"""Thin ctypes binding over libgrouter.so: argument marshalling only.

Every function mirrors the C entry point of the same name in include/grouter.h and takes torch tensors
that already live on the GPU (PyTorch is used for device memory and streams, nothing else).  There is
no fallback: if the HIP library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgrouter.so")
_lib = None

OK, ERR_INVALID_ARG, ERR_WORKSPACE_TOO_SMALL, ERR_INDEX_OUT_OF_RANGE, ERR_HIP = 0, -1, -2, -3, -4
IDX_INT32, IDX_UINT8 = 0, 1
PHASES = ("plan", "permute", "gateup", "down", "combine", "dO", "dH", "dW2", "dW13", "dXp", "dX_reduce", "affinity",
          "placement", "coactivation", "fold", "sample_stats")

EXPORTS = (
    "grouter_strerror", "grouter_last_hip_error", "grouter_plan_bytes", "grouter_ctx_bytes",
    "grouter_bwd_scratch_bytes", "grouter_plan_build", "grouter_plan_views", "grouter_plan_status",
    "grouter_permute", "grouter_combine", "grouter_moe_fwd", "grouter_moe_bwd", "grouter_timing_enable",
    "grouter_timing_read", "grouter_phase_name", "grouter_fwd_only_bytes", "grouter_moe_fwd_only", "grouter_affinity", "grouter_sample_placement",
    "grouter_coactivation", "grouter_fold_groups", "grouter_fold_weights", "grouter_static_ws_bytes",
    "grouter_moe_fwd_only_static", "grouter_sample_stats", "grouter_plan_set_gates", "grouter_mfma_probe",
)


class GrouterError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().grouter_strerror(code).decode()
        if code == ERR_HIP:
            msg += f" (hipError_t {lib().grouter_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


def lib():
    """Load libgrouter.so (built in-tree by paper_2603_06626_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no non-HIP fallback)")
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.grouter_strerror.argtypes = [i32]
        L.grouter_strerror.restype = ctypes.c_char_p
        L.grouter_phase_name.argtypes = [i32]
        L.grouter_phase_name.restype = ctypes.c_char_p
        L.grouter_last_hip_error.restype = i32
        L.grouter_plan_bytes.argtypes = [i64, i32, i32]
        L.grouter_plan_bytes.restype = sz
        L.grouter_ctx_bytes.argtypes = [i64, i32, i32, i32]
        L.grouter_ctx_bytes.restype = sz
        L.grouter_bwd_scratch_bytes.argtypes = [i64, i32, i32, i32]
        L.grouter_bwd_scratch_bytes.restype = sz
        L.grouter_plan_build.argtypes = [vp, i32, i64, i32, i32, vp, sz, vp]
        L.grouter_plan_set_gates.argtypes = [vp, i64, i32, i32, vp, vp]
        L.grouter_plan_set_gates.restype = i32
        L.grouter_plan_views.argtypes = [vp, i64, i32, i32] + [ctypes.POINTER(vp)] * 4
        L.grouter_plan_status.argtypes = [vp, vp]
        L.grouter_permute.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp]
        L.grouter_combine.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp]
        L.grouter_moe_fwd.argtypes = [vp, i64, i32, i32, i32, i32] + [vp] * 7 + [sz, vp]
        L.grouter_fwd_only_bytes.argtypes = [i64, i32, i32, i32]
        L.grouter_fwd_only_bytes.restype = sz
        L.grouter_moe_fwd_only.argtypes = [vp, i64, i32, i32, i32, i32] + [vp] * 7 + [sz, vp]
        L.grouter_moe_fwd_only.restype = i32
        L.grouter_static_ws_bytes.argtypes = []
        L.grouter_static_ws_bytes.restype = sz
        L.grouter_moe_fwd_only_static.argtypes = [vp, i64, i32, i32, i32, i32] + [vp] * 6 + [vp]
        L.grouter_moe_fwd_only_static.restype = i32
        L.grouter_moe_bwd.argtypes = [vp, i64, i32, i32, i32, i32] + [vp] * 7 + [sz] + [vp] * 5 + [sz, vp]
        L.grouter_timing_enable.argtypes = [i32]
        L.grouter_timing_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.grouter_affinity.argtypes = [vp, i32, i64, i32, i32, i32, vp, vp, vp, vp, vp]
        L.grouter_sample_placement.argtypes = [vp, i32, i64, i32, i32, i32, vp, i32, vp, vp, vp]
        L.grouter_sample_stats.argtypes = [vp, i32, i64, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp]
        L.grouter_sample_stats.restype = i32
        L.grouter_coactivation.argtypes = [vp, i32, i64, i32, i32, vp, vp]
        L.grouter_fold_groups.argtypes = [vp, i32, i32, vp, vp]
        L.grouter_mfma_probe.argtypes = [i32, i32, i32, vp, sz, vp]
        L.grouter_fold_weights.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        for name in ("grouter_plan_build", "grouter_plan_views", "grouter_plan_status", "grouter_permute",
                     "grouter_combine", "grouter_moe_fwd", "grouter_moe_bwd", "grouter_timing_enable",
                     "grouter_timing_read", "grouter_affinity", "grouter_sample_placement", "grouter_coactivation",
                     "grouter_fold_groups", "grouter_fold_weights"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _check(code: int, where: str):
    if code != OK:
        raise GrouterError(code, where)


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t, name, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}")
    return t


def grouter_plan_bytes(T, k, E) -> int:
    return int(lib().grouter_plan_bytes(T, k, E))


def grouter_ctx_bytes(T, k, d, f) -> int:
    return int(lib().grouter_ctx_bytes(T, k, d, f))


def grouter_bwd_scratch_bytes(T, k, d, f) -> int:
    return int(lib().grouter_bwd_scratch_bytes(T, k, d, f))


def grouter_plan_build(topk_idx, E, plan_ws, stream=None):
    """topk_idx: [T,k] int32 or uint8 GPU tensor; plan_ws: uint8 GPU tensor of >= grouter_plan_bytes."""
    import torch

    _dev(topk_idx, "topk_idx")
    if topk_idx.dtype == torch.int32:
        dt = IDX_INT32
    elif topk_idx.dtype == torch.uint8:
        dt = IDX_UINT8
    else:
        raise ValueError("topk_idx must be int32 or uint8")
    T, k = topk_idx.shape
    _check(lib().grouter_plan_build(_p(topk_idx), dt, T, k, E, _p(_dev(plan_ws, "plan_ws")), plan_ws.numel(),
                                    _stream(stream)), "grouter_plan_build")


def grouter_plan_set_gates(plan_ws, E, gate_w, stream=None):
    """Lay the gate weights [T,k] (bf16) out in the plan; the layer calls then take gate_w=None and k."""
    import torch

    T, k = gate_w.shape
    _dev(gate_w, "gate_w", torch.bfloat16)
    _check(lib().grouter_plan_set_gates(_p(_dev(plan_ws, "plan_ws")), T, k, E, _p(gate_w), _stream(stream)),
           "grouter_plan_set_gates")


def grouter_plan_views(plan_ws, T, k, E):
    """(counts[E], offsets[E+1], row_to_src[N], src_to_row[N]) as int32 GPU tensors aliasing plan_ws."""
    import torch

    ptrs = [ctypes.c_void_p() for _ in range(4)]
    _check(lib().grouter_plan_views(_p(plan_ws), T, k, E, *[ctypes.byref(p) for p in ptrs]), "grouter_plan_views")
    base = plan_ws.data_ptr()
    as_i32 = plan_ws.view(torch.int32)
    out = []
    for p, n in zip(ptrs, (E, E + 1, T * k, T * k)):
        off = (p.value - base) // 4
        out.append(as_i32[off:off + n])
    return tuple(out)


def grouter_plan_status(plan_ws, stream=None):
    _check(lib().grouter_plan_status(_p(plan_ws), _stream(stream)), "grouter_plan_status")


def grouter_permute(plan_ws, T, k, E, inp, gate_w, out, stream=None):
    d = inp.shape[1]
    _check(lib().grouter_permute(_p(plan_ws), T, k, E, d, _p(_dev(inp, "in")), _p(gate_w), _p(_dev(out, "out")),
                                 _stream(stream)), "grouter_permute")


def grouter_combine(plan_ws, T, k, E, inp, gate_w, out, stream=None):
    d = inp.shape[1]
    _check(lib().grouter_combine(_p(plan_ws), T, k, E, d, _p(_dev(inp, "in")), _p(gate_w), _p(_dev(out, "out")),
                                 _stream(stream)), "grouter_combine")


def grouter_moe_fwd(plan_ws, x, gate_w, W1, W3, W2, y, ctx_ws, stream=None, k=None):
    """gate_w=None: use the gates attached to the plan with grouter_plan_set_gates (k must then be given)."""
    import torch

    bf = torch.bfloat16
    T, d = x.shape
    k = gate_w.shape[1] if gate_w is not None else int(k)
    E, d1, f = W1.shape
    if d1 != d or tuple(W3.shape) != (E, d, f) or tuple(W2.shape) != (E, f, d) or tuple(y.shape) != (T, d):
        raise ValueError("shape mismatch")
    for t, n in ((x, "x"), (gate_w, "gate_w"), (W1, "W1"), (W3, "W3"), (W2, "W2"), (y, "y")):
        if t is not None:
            _dev(t, n, bf)
    _check(lib().grouter_moe_fwd(_p(plan_ws), T, k, E, d, f, _p(x), _p(gate_w), _p(W1), _p(W3), _p(W2), _p(y),
                                 _p(_dev(ctx_ws, "ctx_ws")), ctx_ws.numel(), _stream(stream)), "grouter_moe_fwd")


def grouter_fwd_only_bytes(T, k, d, f) -> int:
    return int(lib().grouter_fwd_only_bytes(T, k, d, f))


def grouter_moe_fwd_only(plan_ws, x, gate_w, W1, W3, W2, y, ws, stream=None, k=None):
    import torch

    bf = torch.bfloat16
    T, d = x.shape
    k = gate_w.shape[1] if gate_w is not None else int(k)
    E, d1, f = W1.shape
    if d1 != d or tuple(W3.shape) != (E, d, f) or tuple(W2.shape) != (E, f, d) or tuple(y.shape) != (T, d):
        raise ValueError("shape mismatch")
    for t, n in ((x, "x"), (gate_w, "gate_w"), (W1, "W1"), (W3, "W3"), (W2, "W2"), (y, "y")):
        if t is not None:
            _dev(t, n, bf)
    _check(lib().grouter_moe_fwd_only(_p(plan_ws), T, k, E, d, f, _p(x), _p(gate_w), _p(W1), _p(W3), _p(W2), _p(y),
                                      _p(_dev(ws, "ws")), ws.numel(), _stream(stream)), "grouter_moe_fwd_only")


def grouter_static_ws_bytes() -> int:
    return int(lib().grouter_static_ws_bytes())


def grouter_moe_fwd_only_static(plan_ws, x, gate_w, W1, W3, W2, y, stream=None, k=None):
    """grouter_moe_fwd_only with the library's static device array as workspace (allocates nothing)."""
    import torch

    bf = torch.bfloat16
    T, d = x.shape
    k = gate_w.shape[1] if gate_w is not None else int(k)
    E, d1, f = W1.shape
    if d1 != d or tuple(W3.shape) != (E, d, f) or tuple(W2.shape) != (E, f, d) or tuple(y.shape) != (T, d):
        raise ValueError("shape mismatch")
    for t, n in ((x, "x"), (gate_w, "gate_w"), (W1, "W1"), (W3, "W3"), (W2, "W2"), (y, "y")):
        if t is not None:
            _dev(t, n, bf)
    _check(lib().grouter_moe_fwd_only_static(_p(plan_ws), T, k, E, d, f, _p(x), _p(gate_w), _p(W1), _p(W3), _p(W2),
                                             _p(y), _stream(stream)), "grouter_moe_fwd_only_static")


def grouter_moe_bwd(plan_ws, x, gate_w, W1, W3, W2, dY, ctx_ws, dX, dW1, dW3, dW2, scratch_ws, stream=None, k=None):
    import torch

    bf = torch.bfloat16
    T, d = x.shape
    k = gate_w.shape[1] if gate_w is not None else int(k)
    E, _, f = W1.shape
    if (tuple(dY.shape) != (T, d) or tuple(dX.shape) != (T, d) or tuple(dW1.shape) != (E, d, f)
            or tuple(dW3.shape) != (E, d, f) or tuple(dW2.shape) != (E, f, d)):
        raise ValueError("shape mismatch")
    for t, n in ((x, "x"), (gate_w, "gate_w"), (W1, "W1"), (W3, "W3"), (W2, "W2"), (dY, "dY"), (dX, "dX"),
                 (dW1, "dW1"), (dW3, "dW3"), (dW2, "dW2")):
        if t is not None:
            _dev(t, n, bf)
    _check(lib().grouter_moe_bwd(_p(plan_ws), T, k, E, d, f, _p(x), _p(gate_w), _p(W1), _p(W3), _p(W2), _p(dY),
                                 _p(_dev(ctx_ws, "ctx_ws")), ctx_ws.numel(), _p(dX), _p(dW1), _p(dW3), _p(dW2),
                                 _p(_dev(scratch_ws, "scratch_ws")), scratch_ws.numel(), _stream(stream)),
           "grouter_moe_bwd")


def _idx_dtype(t):
    import torch

    if t.dtype == torch.int32:
        return IDX_INT32
    if t.dtype == torch.uint8:
        return IDX_UINT8
    raise ValueError("topk_idx must be int32 or uint8")


def grouter_affinity(topk_idx, E, counts, entropy_bits, loads, maxvio, stream=None):
    """topk_idx [S,L,k]; counts int32 [S,E]; entropy_bits float64 [S]; loads int64 [E]; maxvio float64 [1]."""
    import torch

    S, L, k = topk_idx.shape
    _dev(topk_idx, "topk_idx")
    _dev(counts, "counts", torch.int32)
    _dev(entropy_bits, "entropy_bits", torch.float64)
    _dev(loads, "loads", torch.int64)
    _dev(maxvio, "maxvio", torch.float64)
    if tuple(counts.shape) != (S, E) or entropy_bits.numel() != S or loads.numel() != E or maxvio.numel() != 1:
        raise ValueError("shape mismatch")
    _check(lib().grouter_affinity(_p(topk_idx), _idx_dtype(topk_idx), S, L, k, E, _p(counts), _p(entropy_bits),
                                  _p(loads), _p(maxvio), _stream(stream)), "grouter_affinity")


def grouter_sample_placement(topk_idx, E, expert_nodes, n_nodes, comm, best_node, stream=None):
    """topk_idx [S,L,k]; expert_nodes int64 [E] (bit n = expert on node n); comm int32 [S,n_nodes]; best_node int32 [S]."""
    import torch

    S, L, k = topk_idx.shape
    _dev(topk_idx, "topk_idx")
    _dev(expert_nodes, "expert_nodes", torch.int64)
    _dev(comm, "comm", torch.int32)
    _dev(best_node, "best_node", torch.int32)
    if expert_nodes.numel() != E or tuple(comm.shape) != (S, n_nodes) or best_node.numel() != S:
        raise ValueError("shape mismatch")
    _check(lib().grouter_sample_placement(_p(topk_idx), _idx_dtype(topk_idx), S, L, k, E, _p(expert_nodes), n_nodes,
                                          _p(comm), _p(best_node), _stream(stream)), "grouter_sample_placement")


def grouter_sample_stats(topk_idx, E, counts, entropy_bits, loads, maxvio, expert_nodes, n_nodes, comm, best_node,
                         stream=None):
    """grouter_affinity and grouter_sample_placement in one pass over topk_idx [S,L,k]."""
    import torch

    S, L, k = topk_idx.shape
    _dev(topk_idx, "topk_idx")
    _dev(counts, "counts", torch.int32)
    _dev(entropy_bits, "entropy_bits", torch.float64)
    _dev(loads, "loads", torch.int64)
    _dev(maxvio, "maxvio", torch.float64)
    _dev(expert_nodes, "expert_nodes", torch.int64)
    _dev(comm, "comm", torch.int32)
    _dev(best_node, "best_node", torch.int32)
    if (tuple(counts.shape) != (S, E) or entropy_bits.numel() != S or loads.numel() != E or maxvio.numel() != 1
            or expert_nodes.numel() != E or tuple(comm.shape) != (S, n_nodes) or best_node.numel() != S):
        raise ValueError("shape mismatch")
    _check(lib().grouter_sample_stats(_p(topk_idx), _idx_dtype(topk_idx), S, L, k, E, _p(counts), _p(entropy_bits),
                                      _p(loads), _p(maxvio), _p(expert_nodes), n_nodes, _p(comm), _p(best_node),
                                      _stream(stream)), "grouter_sample_stats")


def grouter_coactivation(topk_idx, E, P, stream=None):
    """topk_idx [T,k]; P int64 [E,E]."""
    import torch

    T, k = topk_idx.shape
    _dev(topk_idx, "topk_idx")
    _dev(P, "P", torch.int64)
    if tuple(P.shape) != (E, E):
        raise ValueError("shape mismatch")
    _check(lib().grouter_coactivation(_p(topk_idx), _idx_dtype(topk_idx), T, k, E, _p(P), _stream(stream)),
           "grouter_coactivation")


def grouter_fold_groups(P, E_T, group_of, stream=None):
    """P int64 [E_S,E_S]; group_of int32 [E_S]."""
    import torch

    E_S = P.shape[0]
    _dev(P, "P", torch.int64)
    _dev(group_of, "group_of", torch.int32)
    if tuple(P.shape) != (E_S, E_S) or group_of.numel() != E_S:
        raise ValueError("shape mismatch")
    _check(lib().grouter_fold_groups(_p(P), E_S, E_T, _p(group_of), _stream(stream)), "grouter_fold_groups")


def grouter_mfma_probe(mode, iters, workgroups, out, stream=None):
    """out float32, at least workgroups*256 elements (a checksum only); returns the FLOP count of the launch."""
    import torch

    _dev(out, "out", torch.float32)
    _check(lib().grouter_mfma_probe(mode, iters, workgroups, _p(out), out.numel(), _stream(stream)), "grouter_mfma_probe")
    return workgroups * 4 * iters * 8 * 32768


def grouter_fold_weights(W_s, group_of, E_T, out, stream=None):
    """W_s float32 [d,E_S]; group_of int32 [E_S]; out float32 [d,E_T]."""
    import torch

    d, E_S = W_s.shape
    _dev(W_s, "W_s", torch.float32)
    _dev(group_of, "group_of", torch.int32)
    _dev(out, "out", torch.float32)
    if group_of.numel() != E_S or tuple(out.shape) != (d, E_T):
        raise ValueError("shape mismatch")
    _check(lib().grouter_fold_weights(_p(W_s), _p(group_of), d, E_S, E_T, _p(out), _stream(stream)),
           "grouter_fold_weights")


def grouter_timing_enable(on: bool):
    _check(lib().grouter_timing_enable(1 if on else 0), "grouter_timing_enable")


def grouter_timing_read():
    """{phase: (milliseconds, launches)} accumulated since the previous read; waits for the recorded events."""
    n = len(PHASES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(lib().grouter_timing_read(ms, cnt), "grouter_timing_read")
    return {PHASES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}
