"""Plumbing for the GPU parity tests: host<->device copies and one call sequence through the C ABI."""
import numpy as np
import torch

from paper_2603_06626_amd import binding as b

DEV = torch.device("cuda:0")


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def to_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 GPU tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class Layer:
    """Owns the workspaces of one (T,k,E,d,f) problem and runs plan / fwd / bwd through the binding."""

    def __init__(self, T, k, E, d, f):
        self.T, self.k, self.E, self.d, self.f = T, k, E, d, f
        self.plan = torch.empty(b.grouter_plan_bytes(T, k, E), dtype=torch.uint8, device=DEV)
        self.ctx = torch.empty(b.grouter_ctx_bytes(T, k, d, f), dtype=torch.uint8, device=DEV)
        self.scratch = None

    def build_plan(self, idx):
        if isinstance(idx, np.ndarray):
            idx = torch.from_numpy(idx).to(DEV)
        b.grouter_plan_build(idx, self.E, self.plan)
        b.grouter_plan_status(self.plan)

    def plan_views(self):
        return [v.cpu().numpy() for v in b.grouter_plan_views(self.plan, self.T, self.k, self.E)]

    def fwd(self, x, gw, W1, W3, W2):
        y = torch.empty((self.T, self.d), dtype=torch.bfloat16, device=DEV)
        b.grouter_moe_fwd(self.plan, x, gw, W1, W3, W2, y, self.ctx)
        return y

    def fwd_only(self, x, gw, W1, W3, W2):
        """The forward-only entry point with its own (smaller) workspace."""
        ws = torch.empty(b.grouter_fwd_only_bytes(self.T, self.k, self.d, self.f), dtype=torch.uint8, device=DEV)
        y = torch.empty((self.T, self.d), dtype=torch.bfloat16, device=DEV)
        b.grouter_moe_fwd_only(self.plan, x, gw, W1, W3, W2, y, ws)
        return y

    def bwd(self, x, gw, W1, W3, W2, dY):
        if self.scratch is None:
            self.scratch = torch.empty(b.grouter_bwd_scratch_bytes(self.T, self.k, self.d, self.f), dtype=torch.uint8,
                                       device=DEV)
        dX = torch.empty((self.T, self.d), dtype=torch.bfloat16, device=DEV)
        dW1 = torch.empty_like(W1)
        dW3 = torch.empty_like(W3)
        dW2 = torch.empty_like(W2)
        b.grouter_moe_bwd(self.plan, x, gw, W1, W3, W2, dY, self.ctx, dX, dW1, dW3, dW2, self.scratch)
        return dX, dW1, dW3, dW2

