"""CPU oracle of the routing statistics that feed the offline optimisers - TEST INFRASTRUCTURE ONLY.

Plain numpy / Python definitions, fp64 wherever a float appears; shares nothing with the HIP path and is
imported only by the tests, the smoke check and the benchmark's cpu_baseline leg.

Covered (each function cites the passage it follows):
  * routing affinity vector of a sample (Sec. 3.3.2, first equation: per expert, the fraction of the
    sample's tokens whose top-k set contains it), its entropy in bits (App. "Efficiency Experiment
    Detail", expert grouping: samples whose affinity entropy exceeds a threshold are dropped), the expert
    loads and the global maximal violation (App. "Maximal Violation");
  * sample placement (App. "Efficiency Experiment Detail", Alg. "Optimize Sample-to-Node Assignment");
  * expert folding (Sec. 3.2.1: co-activation matrix P, greedy affinity grouping, folded score weights
    W_s M).

Readings taken where the text leaves a choice (the GPU side takes the same ones):
  * membership is an indicator per token, so an expert id repeated inside one token counts once;
  * entropy is the Shannon entropy, base 2, of the affinity vector normalised to sum 1; terms with zero
    probability contribute 0; a sample with no tokens has entropy 0;
  * loads L_e are the column sums of the per-sample token counts, mean load = sum(L)/E;
  * placement: comm(n, s) = number of tokens of s that find at least one of their experts on node n; the
    best node is the first (lowest n) that attains the maximum, as the strict comparison in the algorithm
    implies.  (The section's prose speaks of minimising a cost; the tokens that stay local are the
    complement of the tokens that must travel, so maximising comm is that minimisation.)
  * P_ij (i != j) = number of tokens whose top-k set contains both i and j; P_ii = number of tokens whose
    set contains i;
  * folding: groups are filled one after the other; the first E_S mod E_T groups get floor(E_S/E_T)+1
    members, the others floor(E_S/E_T); a group is started by the lowest-numbered unassigned expert; each
    further member is the unassigned expert with the largest summed co-activation with the current
    members, the lowest number winning ties; folded weights are W_s M with W_s stored [d][E_S].
"""
from __future__ import annotations

import numpy as np


def _indicator(ids: np.ndarray, E: int) -> np.ndarray:
    """[L,k] expert ids -> [L,E] bool: does token t's top-k set contain expert e."""
    ids = np.asarray(ids).astype(np.int64)
    L = ids.shape[0]
    ind = np.zeros((L, E), dtype=bool)
    if L:
        ind[np.arange(L)[:, None], ids] = True
    return ind


def affinity_counts(idx: np.ndarray, E: int) -> np.ndarray:
    """idx [S,L,k] -> counts [S,E] int32: tokens of sample s whose top-k set contains expert e.

    The affinity vector of Sec. 3.3.2 is counts / L.
    """
    idx = np.asarray(idx)
    S = idx.shape[0]
    out = np.zeros((S, E), dtype=np.int32)
    for s in range(S):
        out[s] = _indicator(idx[s], E).sum(axis=0)
    return out


def affinity(idx: np.ndarray, E: int) -> np.ndarray:
    """phi(X)_i for every sample: [S,E] float64."""
    idx = np.asarray(idx)
    L = idx.shape[1]
    return affinity_counts(idx, E).astype(np.float64) / max(L, 1)


def entropy_bits(counts: np.ndarray) -> np.ndarray:
    """Shannon entropy (base 2) of each row of counts normalised to a distribution: [S] float64."""
    c = np.asarray(counts).astype(np.float64)
    out = np.zeros(c.shape[0], dtype=np.float64)
    for s in range(c.shape[0]):
        tot = c[s].sum()
        if tot <= 0:
            continue
        p = c[s][c[s] > 0] / tot
        out[s] = -(p * np.log2(p)).sum()
    return out


def expert_loads(counts: np.ndarray) -> np.ndarray:
    """L_e: tokens given to expert e over all samples, int64 [E]."""
    return np.asarray(counts).astype(np.int64).sum(axis=0)


def maxvio(loads: np.ndarray) -> float:
    """(max_e L_e - mean L) / mean L, App. "Maximal Violation"; 0 when nothing was routed."""
    l = np.asarray(loads).astype(np.float64)
    mean = l.sum() / l.shape[0]
    return float((l.max() - mean) / mean) if mean > 0 else 0.0


def placement(idx: np.ndarray, node_experts, E: int):
    """idx [S,L,k]; node_experts: one iterable of expert ids per node.

    Returns comm [S,N] int32 (tokens of s with at least one expert on node n) and best_node [S] int32.
    """
    idx = np.asarray(idx)
    S = idx.shape[0]
    N = len(node_experts)
    comm = np.zeros((S, N), dtype=np.int32)
    best = np.zeros(S, dtype=np.int32)
    on_node = np.zeros((N, E), dtype=bool)
    for n, members in enumerate(node_experts):
        for e in members:
            on_node[n, int(e)] = True
    for s in range(S):
        ids = idx[s].astype(np.int64)
        best_node, max_comm = 0, -1
        for n in range(N):
            local = on_node[n][ids].any(axis=1) if ids.shape[0] else np.zeros(0, dtype=bool)
            c = int(local.sum())
            comm[s, n] = c
            if c > max_comm:
                max_comm, best_node = c, n
        best[s] = best_node
    return comm, best


def coactivation(idx: np.ndarray, E: int, block: int = 1 << 16) -> np.ndarray:
    """idx [T,k] -> P [E,E] int64 (Sec. 3.2.1): tokens whose top-k set contains both i and j.

    Indicator-matrix product; the product runs in float64, which is exact for counts below 2^53.
    """
    idx = np.asarray(idx).reshape(-1, np.asarray(idx).shape[-1])
    P = np.zeros((E, E), dtype=np.int64)
    for t0 in range(0, idx.shape[0], block):
        ind = _indicator(idx[t0:t0 + block], E).astype(np.float64)
        P += np.rint(ind.T @ ind).astype(np.int64)
    return P


def fold_groups(P: np.ndarray, E_T: int) -> np.ndarray:
    """Greedy affinity grouping of Sec. 3.2.1: returns group_of [E_S] int32 (target expert of each source)."""
    P = np.asarray(P).astype(np.int64)
    E_S = P.shape[0]
    g_avg, n_extra = E_S // E_T, E_S % E_T
    group_of = np.full(E_S, -1, dtype=np.int32)
    for g in range(E_T):
        size = g_avg + (1 if g < n_extra else 0)
        members = []
        for _ in range(size):
            free = [e for e in range(E_S) if group_of[e] < 0]
            if not members:
                pick = free[0]
            else:
                pick, best = -1, None
                for e in free:
                    score = int(sum(P[m, e] for m in members))
                    if best is None or score > best:
                        pick, best = e, score
            group_of[pick] = g
            members.append(pick)
    return group_of


def fold_weights(W_s: np.ndarray, group_of: np.ndarray, E_T: int) -> np.ndarray:
    """W_s [d,E_S] times the binary map M [E_S,E_T] (M[i, group_of[i]] = 1), float64."""
    W = np.asarray(W_s, dtype=np.float64)
    E_S = W.shape[1]
    M = np.zeros((E_S, E_T), dtype=np.float64)
    M[np.arange(E_S), np.asarray(group_of).astype(np.int64)] = 1.0
    return W @ M
