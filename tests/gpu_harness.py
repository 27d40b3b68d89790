"""GPU-side test driver: device buffers through torch, every computation through the C-ABI binding."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from paper_2505_14371_amd import qoda, workloads


def dev():
    return torch.device("cuda:0")


class GpuModel:
    """Buffers for one model on the GPU: K nodes' gradients (one flat buffer per node, layers 256-byte aligned),
    two message buffers per node, and the solver state."""

    def __init__(self, sizes: Sequence[int], layer_type: Sequence[int], type_points: Sequence[int], K: int, seed: int,
                 norm_scope: int = 0, norm_kind: int = 2):
        self.sizes = [int(s) for s in sizes]
        self.L, self.K = len(self.sizes), K
        self.ctx = qoda.Context(self.sizes, layer_type, type_points, K, seed, norm_scope=norm_scope, norm_kind=norm_kind)
        self.off, self.flat_len = workloads.padded_offsets(self.sizes)
        self.grad_flat = [torch.zeros(self.flat_len, dtype=torch.float32, device=dev()) for _ in range(K)]
        self.mbytes = self.ctx.message_bytes()
        self.msg = [[torch.zeros(self.mbytes, dtype=torch.uint8, device=dev()) for _ in range(K)] for _ in range(2)]
        self.cur = 0
        self.have_prev = False
        self.x1 = torch.zeros(self.flat_len, dtype=torch.float32, device=dev())
        self.y = torch.zeros_like(self.x1)
        self.x_half = torch.zeros_like(self.x1)
        self.x_next = torch.zeros_like(self.x1)
        self.mean = torch.zeros_like(self.x1)
        self.acc = torch.zeros(1, dtype=torch.float64, device=dev())
        self.eta = torch.ones(2, dtype=torch.float32, device=dev())
        self.alt_sums = torch.zeros(2, dtype=torch.float64, device=dev())      # lambda, mu of eq. (Alt)

    # ---- views
    def layer_ptrs(self, flat: torch.Tensor) -> List[int]:
        base = flat.data_ptr()
        return [base + 4 * int(o) for o in self.off]

    def grad_ptrs(self) -> List[int]:
        return [p for k in range(self.K) for p in self.layer_ptrs(self.grad_flat[k])]

    def layers(self, flat: torch.Tensor) -> List[np.ndarray]:
        h = flat.cpu().numpy()
        return [h[int(o): int(o) + s].copy() for o, s in zip(self.off, self.sizes)]

    def set_layers(self, flat: torch.Tensor, arrs: Sequence[np.ndarray]):
        h = np.zeros(self.flat_len, dtype=np.float32)
        for o, s, a in zip(self.off, self.sizes, arrs):
            h[int(o): int(o) + s] = a
        flat.copy_(torch.from_numpy(h))

    def set_grads(self, grads: Sequence[Sequence[np.ndarray]]):
        for k in range(self.K):
            self.set_layers(self.grad_flat[k], grads[k])

    # ---- the calls
    def fit(self, round_: int):
        self.ctx.fit_levels(self.grad_ptrs(), round_)

    def quantize_all(self, round_: int):
        prev = self.msg[1 - self.cur] if self.have_prev else None
        self.ctx.quantize_all(self.grad_ptrs(), round_, self.msg[self.cur], prev)

    def quantize_each(self, round_: int):
        for k in range(self.K):
            prev = self.msg[1 - self.cur][k] if self.have_prev else None
            self.ctx.quantize(k, self.layer_ptrs(self.grad_flat[k]), round_, self.msg[self.cur][k], prev)

    def step(self, want_next: bool = True):
        self.ctx.step(self.msg[self.cur], self.layer_ptrs(self.x1), self.layer_ptrs(self.y),
                      self.layer_ptrs(self.x_half), self.acc, self.layer_ptrs(self.x_next) if want_next else None,
                      self.eta)
        self.cur = 1 - self.cur
        self.have_prev = True

    def quantize_all_alt(self, round_: int):
        """eq. (Alt): the per-node term is ||Vhat_k||^2, i.e. the distance to an all-zero previous message."""
        self.ctx.quantize_all(self.grad_ptrs(), round_, self.msg[self.cur], None)

    def step_alt(self, q_hat: float, want_next: bool = True):
        self.ctx.step_alt(self.msg[self.cur], self.layer_ptrs(self.x1), self.layer_ptrs(self.y),
                          self.layer_ptrs(self.x_half), self.alt_sums, self.eta, q_hat,
                          self.layer_ptrs(self.x_next) if want_next else None)
        self.cur = 1 - self.cur
        self.have_prev = True

    def aggregate(self):
        self.ctx.dequant_aggregate(self.msg[self.cur], self.layer_ptrs(self.mean))

    def messages(self, which: Optional[int] = None) -> List[np.ndarray]:
        w = self.cur if which is None else which
        return [m.cpu().numpy() for m in self.msg[w]]

    def sync(self):
        torch.cuda.synchronize()
