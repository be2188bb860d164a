"""Seeded synthetic inputs for the fixed-routing expert layer.

This module only *draws inputs*: routing ids, gate weights, activations, expert weights and the
upstream gradient, in the storage formats the layer consumes (int32 / uint8 expert ids, bfloat16 bit
patterns).  It holds none of the layer's arithmetic and is the one module that both the HIP path's
callers and the CPU checker may import.

The workloads stand in for the paper's cached routing (Sec. 3.3.1, "Decoupling Preemptive Routing":
per token k expert ids stored as uint8 and k scores stored as bfloat16) on Qwen3 / DeepSeek-V2-Lite
style MoE shapes (App. "Model Configuration" table).  The five named configurations are:

  id  T      d     f     E    k  routing                          pass
  0   256    128   256   8    2  Zipf(1.0), distinct per token    fwd+bwd
  1   4096   1024  512   64   8  uniform, distinct                fwd
  2   8192   2048  1408  64   6  Zipf(1.2), distinct              fwd
  3   8192   2048  1408  64   6  same tensors as 2, plus dY       fwd+bwd
  4   16384  4096  1536  128  8  uniform + 5% tokens -> expert 0  4 x (fwd+bwd), one plan

Recipes
  * activations x, dY ~ N(0,1); W1 (gate), W3 (up) ~ N(0, 1/d); W2 (down) ~ N(0, 1/f)  (variance =
    1/fan_in); everything rounded to bfloat16, round-to-nearest-even.
  * Zipf(s): p_r ~ r^-s over ranks r = 1..E, rank r is expert id r-1; each token draws k *distinct*
    experts sequentially without replacement (implemented as Gumbel-top-k on log p, which has the same
    law); ids are kept in draw order.
  * gate weights: k iid N(0,1) logits per token, softmax over those k in fp32, rounded to bfloat16
    (so a token's gates sum to 1 only up to that rounding; nothing downstream renormalises).
  * config 4: uniform distinct draw; then floor(0.05*T) tokens picked by a seeded permutation get
    expert 0 written into slot 0 unless they already hold it.
  * independent sub-streams per (seed, config tensors, tensor name, layer) via numpy SeedSequence.
"""
from __future__ import annotations

import numpy as np

CONFIGS = {
    0: dict(T=256, d=128, f=256, E=8, k=2, routing="zipf", zipf_s=1.0, bwd=True, layers=1, tensors_of=0),
    1: dict(T=4096, d=1024, f=512, E=64, k=8, routing="uniform", bwd=False, layers=1, tensors_of=1),
    2: dict(T=8192, d=2048, f=1408, E=64, k=6, routing="zipf", zipf_s=1.2, bwd=False, layers=1, tensors_of=2),
    3: dict(T=8192, d=2048, f=1408, E=64, k=6, routing="zipf", zipf_s=1.2, bwd=True, layers=1, tensors_of=2),
    4: dict(T=16384, d=4096, f=1536, E=128, k=8, routing="uniform_hot", hot_frac=0.05, bwd=True, layers=4,
            tensors_of=4),
}

_TAGS = {"routing": 1, "gates": 2, "x": 3, "dY": 4, "W1": 5, "W3": 6, "W2": 7, "hot": 8, "topics": 9, "placement": 10,
         "score_w": 11}

# Corpus-statistics workload: cached routing of packed training sequences (App. "Efficiency Experiment Detail":
# fixed-length packed sequences, uint8 ids; Qwen3-style E = 128, k = 8, 4096-token sequences, 4 expert groups).
CORPUS = dict(S=2048, L=4096, E=128, k=8, n_topics=4, n_nodes=4)


def _seedseq(seed: int, stream: int, tag: str, layer: int = 0) -> np.random.SeedSequence:
    return np.random.SeedSequence([int(seed), int(stream), _TAGS[tag], int(layer)])


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def draw_routing(T: int, E: int, k: int, kind: str, seed: int = 0, stream: int = 0, zipf_s: float = 1.0,
                 hot_frac: float = 0.05) -> np.ndarray:
    """Expert ids [T,k] int32, k distinct experts per token, in draw order."""
    if not (0 < k <= E):
        raise ValueError("need 0 < k <= E")
    rng = np.random.default_rng(_seedseq(seed, stream, "routing"))
    if kind == "zipf":
        logp = -float(zipf_s) * np.log(np.arange(1, E + 1, dtype=np.float64))
    elif kind in ("uniform", "uniform_hot"):
        logp = np.zeros(E, dtype=np.float64)
    else:
        raise ValueError(f"unknown routing kind {kind!r}")
    u = rng.random((T, E))
    u = np.clip(u, 1e-300, 1.0 - 1e-16)
    keys = logp[None, :] - np.log(-np.log(u))
    order = np.argsort(-keys, axis=1, kind="stable")
    idx = np.ascontiguousarray(order[:, :k]).astype(np.int32)
    if kind == "uniform_hot":
        n_hot = int(np.floor(hot_frac * T))
        hot_rng = np.random.default_rng(_seedseq(seed, stream, "hot"))
        chosen = hot_rng.permutation(T)[:n_hot]
        for t in chosen:
            if not np.any(idx[t] == 0):
                idx[t, 0] = 0
    return idx


def draw_gates(T: int, k: int, seed: int = 0, stream: int = 0) -> np.ndarray:
    """Gate weights [T,k] as bfloat16 bit patterns: softmax over k iid N(0,1) logits."""
    rng = np.random.default_rng(_seedseq(seed, stream, "gates"))
    logits = rng.standard_normal((T, k), dtype=np.float32)
    z = np.exp(logits - logits.max(axis=1, keepdims=True))
    p = (z / z.sum(axis=1, keepdims=True)).astype(np.float32)
    return f32_to_bf16_bits(p)


def draw_normal_bf16(shape, sigma: float, seed: int, stream: int, tag: str, layer: int = 0, device=None):
    """N(0, sigma^2) rounded to bfloat16.

    device=None: numpy uint16 bit patterns on the host.  Otherwise a torch.bfloat16 tensor drawn with
    torch's generator on that device (a different stream of numbers than the numpy path; callers that
    need the host copy read it back from the tensor).
    """
    ss = _seedseq(seed, stream, tag, layer)
    if device is None:
        rng = np.random.default_rng(ss)
        out = np.empty(shape, dtype=np.uint16)
        flat = out.reshape(-1)
        n = flat.size
        step = 1 << 24
        for s in range(0, n, step):
            e = min(n, s + step)
            flat[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32) * np.float32(sigma))
        return out
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(_device_seed(ss))
    shape = tuple(int(s) for s in shape)
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    # draw in pieces so the fp32 temporary stays small next to multi-GB weight tensors
    step = 1 << 26
    for s0 in range(0, flat.numel(), step):
        n = min(step, flat.numel() - s0)
        flat[s0:s0 + n] = torch.randn(n, generator=g, device=device, dtype=torch.float32).mul_(float(sigma)).to(
            torch.bfloat16)
    return out


def _device_seed(ss: np.random.SeedSequence) -> int:
    return int(ss.generate_state(2, dtype=np.uint32).astype(np.uint64) @ np.array([1, 1 << 31], dtype=np.uint64))


def draw_sequence_routing(S: int, L: int, E: int, k: int, n_topics: int = 4, seed: int = 0, stream: int = 50,
                          device=None, dtype="uint8"):
    """Cached routing of S packed sequences of L tokens: expert ids [S,L,k], k distinct per token.

    Structure (stands in for routing a frozen router produces on real text): experts are split by a seeded
    permutation into n_topics equal groups; expert e has a global popularity z_e ~ N(0, 0.25^2); sequence s
    has a topic g_s (uniform) and a sharpness b_s ~ U(0, 3); token logits are z_e + b_s*[e in group g_s] and
    each token draws k distinct experts by Gumbel-top-k.  Sequences with small b_s have near-uniform
    affinity vectors (the ones an entropy filter drops); the others prefer one group.

    device=None: numpy on the host.  Otherwise drawn with torch's generator on that device (a different
    stream of numbers) and returned as a torch tensor there.
    """
    if not (0 < k <= E):
        raise ValueError("need 0 < k <= E")
    if dtype == "uint8" and E > 256:
        raise ValueError("uint8 ids need E <= 256")
    rng = np.random.default_rng(_seedseq(seed, stream, "topics"))
    group_of_expert = rng.permutation(E) % n_topics
    z = rng.normal(0.0, 0.25, size=E)
    topic = rng.integers(0, n_topics, size=S)
    sharp = rng.uniform(0.0, 3.0, size=S)
    logits = z[None, :] + sharp[:, None] * (group_of_expert[None, :] == topic[:, None])   # [S,E]
    np_dtype = np.uint8 if dtype == "uint8" else np.int32
    if device is None:
        draw = np.random.default_rng(_seedseq(seed, stream, "routing"))
        out = np.empty((S, L, k), dtype=np_dtype)
        for s in range(S):
            u = np.clip(draw.random((L, E)), 1e-300, 1.0 - 1e-16)
            keys = logits[s][None, :] - np.log(-np.log(u))
            out[s] = np.argsort(-keys, axis=1, kind="stable")[:, :k]
        return out
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(_device_seed(_seedseq(seed, stream, "routing")))
    t_dtype = torch.uint8 if dtype == "uint8" else torch.int32
    out = torch.empty((S, L, k), dtype=t_dtype, device=device)
    lg = torch.tensor(logits, dtype=torch.float32, device=device)
    step = max(1, (1 << 25) // (L * E))          # sequences per piece: keep the [piece*L, E] temporaries small
    for s0 in range(0, S, step):
        s1 = min(S, s0 + step)
        u = torch.rand((s1 - s0, L, E), generator=g, device=device, dtype=torch.float32).clamp_(1e-30, 1.0 - 1e-7)
        keys = lg[s0:s1, None, :] - torch.log(-torch.log(u))
        out[s0:s1] = torch.topk(keys, k, dim=2).indices.to(t_dtype)
    return out


def draw_expert_placement(E: int, n_nodes: int, seed: int = 0, stream: int = 50, aligned: bool = True):
    """A seeded partition of the experts over n_nodes nodes, sizes as equal as possible: list of int arrays.

    aligned=True reuses the permutation that defines the topic groups of draw_sequence_routing (with
    n_topics == n_nodes each node then holds exactly one topic's experts - the outcome the paper's expert
    grouping aims for); aligned=False draws an unrelated partition.
    """
    rng = np.random.default_rng(_seedseq(seed, stream, "topics" if aligned else "placement"))
    node_of = rng.permutation(E) % n_nodes
    return [np.flatnonzero(node_of == n).astype(np.int32) for n in range(n_nodes)]


def draw_score_weights(d: int, E: int, seed: int = 0, stream: int = 50) -> np.ndarray:
    """Final score layer of a router, [d,E] float32 ~ N(0, 1/d)."""
    rng = np.random.default_rng(_seedseq(seed, stream, "score_w"))
    return (rng.standard_normal((d, E), dtype=np.float32) / np.float32(np.sqrt(d))).astype(np.float32)


def make_routing(cfg_id: int, seed: int = 0):
    """(idx int32 [T,k], gates uint16 bf16-bits [T,k]) of a named configuration."""
    c = CONFIGS[cfg_id]
    st = c["tensors_of"]
    idx = draw_routing(c["T"], c["E"], c["k"], c["routing"], seed=seed, stream=st, zipf_s=c.get("zipf_s", 1.0),
                       hot_frac=c.get("hot_frac", 0.05))
    gates = draw_gates(c["T"], c["k"], seed=seed, stream=st)
    return idx, gates


def make_tensors(cfg_id: int, seed: int = 0, layer: int = 0, device=None, need_bwd=None):
    """x, W1, W3, W2 (and dY when the configuration has a backward pass) of a named configuration."""
    c = CONFIGS[cfg_id]
    st = c["tensors_of"]
    T, d, f, E = c["T"], c["d"], c["f"], c["E"]
    need_bwd = c["bwd"] if need_bwd is None else need_bwd
    out = {
        "x": draw_normal_bf16((T, d), 1.0, seed, st, "x", 0, device),
        "W1": draw_normal_bf16((E, d, f), d ** -0.5, seed, st, "W1", layer, device),
        "W3": draw_normal_bf16((E, d, f), d ** -0.5, seed, st, "W3", layer, device),
        "W2": draw_normal_bf16((E, f, d), f ** -0.5, seed, st, "W2", layer, device),
    }
    if need_bwd:
        out["dY"] = draw_normal_bf16((T, d), 1.0, seed, st, "dY", 0, device)
    return out


def make_custom(T, d, f, E, k, routing="zipf", zipf_s=1.0, seed=0, stream=100, device=None):
    """A free-form problem with the same recipes (used for parity cases between the named sizes)."""
    idx = draw_routing(T, E, k, routing, seed=seed, stream=stream, zipf_s=zipf_s)
    gates = draw_gates(T, k, seed=seed, stream=stream)
    t = {
        "x": draw_normal_bf16((T, d), 1.0, seed, stream, "x", 0, device),
        "W1": draw_normal_bf16((E, d, f), d ** -0.5, seed, stream, "W1", 0, device),
        "W3": draw_normal_bf16((E, d, f), d ** -0.5, seed, stream, "W3", 0, device),
        "W2": draw_normal_bf16((E, f, d), f ** -0.5, seed, stream, "W2", 0, device),
        "dY": draw_normal_bf16((T, d), 1.0, seed, stream, "dY", 0, device),
    }
    return idx, gates, t


def flops(T, d, f, k, bwd: bool) -> float:
    """Algorithmic FLOP of one pass: forward 6*T*k*d*f, backward twice that (App. M's 2:4 convention)."""
    fwd = 6.0 * T * k * d * f
    return fwd * 3.0 if bwd else fwd
