"""Alg. 1 as a loop a caller can drive from torch: buffer management and argument marshalling around the library.

    opt = QODA(params, num_nodes=K, points=8)       # params: fp32 CUDA tensors; they hold the query point X_{t+1/2}
    for t in range(T):
        grads = [operator(k, params) for k in range(K)]   # the caller's A_k(X_{t+1/2}) + U_k, one list per node
        opt.step(grads)                             # levels (at update steps), ENCODE, exchange, DECODE, eq. (ODA)

Nothing here computes: every step of the path runs in the HIP library (qoda.Context).  The K nodes are K lists of
gradient tensors on one GPU.  The parameter tensors themselves are the X_{t+1/2} buffer of the fused update, so
after step() the model sits at the next query point (Alg. 1 line 10); X_1 and Y_t live in tensors owned by this
object; ``state_point()`` returns X_{t+1} when asked for.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import qoda


class QODA:
    def __init__(self, params: Sequence[torch.Tensor], num_nodes: int, points: int = 8,
                 layer_types: Optional[Sequence[int]] = None, type_points: Optional[Sequence[int]] = None, seed: int = 0,
                 norm_scope: int = qoda.SCOPE_LAYER, norm_kind: int = qoda.NORM_L2, fit_every: int = 0,
                 q_hat: Optional[float] = None, keep_next: bool = False):
        """layer_types[l] in [0, M): which level sequence tensor l uses (default: one type for tensors with two or more
        dimensions, one for vectors); type_points[m]: grid points of type m (default: ``points`` for all).
        fit_every = n > 0: the levels are refitted at rounds 1, 1+n, 1+2n, ... (the set U of Alg. 1) from the
        gradients of that round; 0: the initial uniform levels stay.  q_hat: use the step sizes of eq. (Alt) with this
        exponent instead of eq. (general_stepsize).  keep_next: also materialise X_{t+1}."""
        self.params = list(params)
        if not self.params:
            raise ValueError("QODA: no parameters")
        for p in self.params:
            if not (p.is_cuda and p.dtype == torch.float32 and p.is_contiguous()):
                raise ValueError("QODA: parameters must be contiguous fp32 CUDA tensors")
            if p.data_ptr() % 16 != 0:
                raise ValueError("QODA: parameter storage must be 16-byte aligned")
        self.K = int(num_nodes)
        if layer_types is None:
            layer_types = [0 if p.dim() >= 2 else 1 for p in self.params]
            if 1 not in layer_types:
                layer_types = [0] * len(self.params)
            elif 0 not in layer_types:
                layer_types = [0] * len(self.params)
        M = max(layer_types) + 1
        if type_points is None:
            type_points = [points] * M
        dev = self.params[0].device
        self.ctx = qoda.Context([p.numel() for p in self.params], list(layer_types), list(type_points), self.K, seed,
                                norm_scope=norm_scope, norm_kind=norm_kind)
        self.norm_scope = norm_scope
        self.fit_every = int(fit_every)
        self.q_hat = q_hat
        mb = self.ctx.message_bytes()
        self._msg = [[torch.zeros(mb, dtype=torch.uint8, device=dev) for _ in range(self.K)] for _ in range(2)]
        self._x1 = [p.detach().clone() for p in self.params]                    # X_1
        self._y = [torch.zeros_like(p) for p in self.params]                    # Y_1 = 0
        self._xn = [torch.zeros_like(p) for p in self.params] if keep_next else None
        self._acc = torch.zeros(1, dtype=torch.float64, device=dev)            # eq. (general_stepsize)
        self._sums = torch.zeros(2, dtype=torch.float64, device=dev)           # eq. (Alt): lambda, mu
        self.rates = torch.ones(2, dtype=torch.float32, device=dev)            # eta_{t+1}, gamma_{t+1} after a step
        # pointer sets that never change: marshalled once
        self._p_msg = [qoda.pointer_array(m) for m in self._msg]
        self._p_xh = qoda.pointer_array(self.params)
        self._p_x1 = qoda.pointer_array(self._x1)
        self._p_y = qoda.pointer_array(self._y)
        self._p_xn = None if self._xn is None else qoda.pointer_array(self._xn)
        self.t = 0

    def _check_grads(self, node_grads) -> List[int]:
        if len(node_grads) != self.K:
            raise ValueError(f"QODA.step: {len(node_grads)} gradient lists for {self.K} nodes")
        ptrs = []
        for g in node_grads:
            if len(g) != len(self.params):
                raise ValueError("QODA.step: a node's gradient list does not match the parameters")
            for t, p in zip(g, self.params):
                if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == p.numel()):
                    raise ValueError("QODA.step: gradients must be contiguous fp32 CUDA tensors shaped like the parameters")
                ptrs.append(t.data_ptr())
        return ptrs

    def step(self, node_grads: Sequence[Sequence[torch.Tensor]], stream=None) -> None:
        """One round of Alg. 1 given the K nodes' dual vectors at the current query point (the parameters)."""
        gp = qoda.pointer_array(self._check_grads(node_grads))
        self.t += 1
        t, cur = self.t, self.t & 1
        if self.fit_every > 0 and (t - 1) % self.fit_every == 0:
            # bucket scope after the first fit: from the statistics the previous quantize pass gathered
            if self.norm_scope == qoda.SCOPE_BUCKET and t > 1:
                self.ctx.fit_levels(None, t, stream=stream)
            else:                                    # the round's own vectors, quantized unchanged right below
                self.ctx.fit_levels_keep_norms(gp, t, stream=stream)
        alt = self.q_hat is not None
        prev = self._p_msg[1 - cur] if (t > 1 and not alt) else None
        self.ctx.quantize_all(gp, t, self._p_msg[cur], prev, stream=stream)
        if alt:
            self.ctx.step_alt(self._p_msg[cur], self._p_x1, self._p_y, self._p_xh, self._sums, self.rates, self.q_hat,
                              self._p_xn, stream=stream)
        else:
            self.ctx.step(self._p_msg[cur], self._p_x1, self._p_y, self._p_xh, self._acc, self._p_xn, self.rates,
                          stream=stream)

    def state_point(self) -> List[torch.Tensor]:
        """X_{t+1} (the dual-averaging iterate; the parameters hold X_{t+3/2}); needs keep_next=True."""
        if self._xn is None:
            raise RuntimeError("QODA: constructed without keep_next")
        return self._xn

    def status(self) -> int:
        return self.ctx.status()

    def close(self) -> None:
        self.ctx.close()
