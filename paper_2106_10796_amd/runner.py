"""Device-side layout and driving of one workload (harness, not part of the library).

Lays the layer list of a synth.Config out in flat HBM arenas, plays the N-1
other workers on the same device (their gradients come from seeds, their packed
streams from cdsgd_quantize_pack with their own residuals) and calls the
library for the observed worker, either as one fused launch per step
(cdsgd_step_fused) or as the three single-tensor calls per tensor.

HBM layout: one arena per kind of buffer (w_global, w_local, residual, grad,
agg_full: fp32; packed streams: 32-bit words).  Tensor i starts at element
offset off[i], a multiple of 1024 elements (4 KiB), and its packed stream at
word offset off[i] / 16 (256 B aligned); gaps are zero.  With that, one flat
cdsgd_quantize_pack call over a whole arena yields every tensor's packed stream
in place (gap elements quantise to code 0), which is how the peers are played.
"""
from typing import List, Optional

import torch

from . import binding, synth

ALIGN_ELEMS = 1024


def default_arena(numel, dtype, device):
    """One arena = one zeroed device allocation of its own."""
    return torch.zeros(numel, dtype=dtype, device=device)


# how a Workload gets its arenas: (numel, dtype, device) -> zeroed 1-D tensor
arena_allocator = default_arena


class Workload:
    def __init__(self, cfg: synth.Config, device="cuda", dense: bool = False, self_rank: int = 0,
                 peer_residuals: bool = True, full_grads: bool = False, grad_dtype=torch.float32,
                 sparse_peers: bool = False):
        self.cfg = cfg
        self.device = torch.device(device)
        self.dense = dense
        self.self_rank = int(self_rank)
        self.N = cfg.num_workers
        assert 0 <= self.self_rank < self.N
        self.off: List[int] = []
        o = 0
        for n in cfg.sizes:
            self.off.append(o)
            o += (n + ALIGN_ELEMS - 1) // ALIGN_ELEMS * ALIGN_ELEMS
        self.total = o
        f32 = dict(dtype=torch.float32, device=self.device)
        i32 = dict(dtype=binding.PACKED_DTYPE, device=self.device)
        alloc = arena_allocator
        self.w_global = alloc(self.total, torch.float32, self.device)
        self.w_local = alloc(self.total, torch.float32, self.device)
        self.residual = alloc(self.total, torch.float32, self.device)
        # gradients may be held in bf16 / fp16 (the library widens them on load); everything else is fp32
        self.grad_dtype = grad_dtype
        self.grad = alloc(self.total, grad_dtype, self.device)
        self.agg_full = alloc(self.total, torch.float32, self.device)
        self.packed_self = alloc(self.total // 16, binding.PACKED_DTYPE, self.device)
        self.peer_packed: List[Optional[torch.Tensor]] = [
            None if j == self.self_rank else alloc(self.total // 16, binding.PACKED_DTYPE, self.device)
            for j in range(self.N)]
        self.peer_residual: List[Optional[torch.Tensor]] = [
            None if (j == self.self_rank or not peer_residuals) else torch.zeros(self.total, **f32)
            for j in range(self.N)]
        # sparse_peers: the observed worker reads the peers' streams in the library's sparse form; every
        # peer's packed stream (made by cdsgd_quantize_pack as before) is re-encoded tensor by tensor
        self.sparse_peers = sparse_peers
        self.soff: List[int] = []
        so = 0
        for n in cfg.sizes:
            self.soff.append(so)
            so += binding.sparse_words(n) if sparse_peers else 0
        self.peer_sparse: List[Optional[torch.Tensor]] = [
            None if (j == self.self_rank or not sparse_peers) else alloc(so, binding.PACKED_DTYPE, self.device)
            for j in range(self.N)]
        self._scratch = torch.zeros(self.total, **f32)   # a peer's gradient, one worker at a time
        # full_grads: every peer's 32-bit gradient stays resident (what the server side would hold on a
        # correction or warm-up pass) and those passes sum in the kernel instead of reading agg_full
        self.peer_grad: List[Optional[torch.Tensor]] = [
            None if (j == self.self_rank or not full_grads)
            else torch.zeros(self.total, dtype=grad_dtype, device=self.device) for j in range(self.N)]
        self.full_grads = full_grads
        self._agg = None                                 # decoded aggregate of the unfused path
        for i in range(cfg.num_tensors):
            synth.fill_weight(self.view(self.w_global, i), cfg, i)
        self.w_local.copy_(self.w_global)
        self.thresholds = None
        self.plan = binding.Plan(self._plan_tensors(), self._plan_peers(), self.N, self.self_rank,
                                 grad_dtype=grad_dtype, peers_sparse=sparse_peers)
        if full_grads and self.N > 1:
            self.plan.bind_full_grads([None if j == self.self_rank else
                                       [self.view(self.peer_grad[j], i) for i in range(cfg.num_tensors)]
                                       for j in range(self.N)])

    def set_thresholds(self, thresholds):
        """One threshold per tensor for the observed worker and the played peers (None: the config's)."""
        self.thresholds = list(thresholds) if thresholds is not None else None
        self.plan.set_thresholds(self.thresholds)

    # -- views ------------------------------------------------------------
    def view(self, arena: torch.Tensor, i: int) -> torch.Tensor:
        return arena[self.off[i]: self.off[i] + self.cfg.sizes[i]]

    def pview(self, arena: torch.Tensor, i: int) -> torch.Tensor:
        o = self.off[i] // 16
        return arena[o: o + binding.packed_words(self.cfg.sizes[i])]

    def _plan_tensors(self):
        return [dict(w_global=self.view(self.w_global, i), w_local=self.view(self.w_local, i),
                     residual=self.view(self.residual, i), grad=self.view(self.grad, i),
                     packed_self=self.pview(self.packed_self, i), agg_full=self.view(self.agg_full, i))
                for i in range(self.cfg.num_tensors)]

    def sview(self, arena: torch.Tensor, i: int) -> torch.Tensor:
        return arena[self.soff[i]: self.soff[i] + binding.sparse_words(self.cfg.sizes[i])]

    def _plan_peers(self):
        if self.N == 1:
            return None
        if self.sparse_peers:
            return [None if j == self.self_rank else [self.sview(self.peer_sparse[j], i)
                                                      for i in range(self.cfg.num_tensors)]
                    for j in range(self.N)]
        return [None if j == self.self_rank else [self.pview(self.peer_packed[j], i)
                                                  for i in range(self.cfg.num_tensors)]
                for j in range(self.N)]

    # -- inputs of a step ---------------------------------------------------
    def compressed(self, step: int) -> bool:
        return step % self.cfg.k != 0

    def gen_grad(self, worker: int, step: int, tensor: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Worker `worker`'s gradient of one tensor (same bits every time it is asked for)."""
        if out is None:
            out = torch.empty(self.cfg.sizes[tensor], dtype=torch.float32, device=self.device)
        return synth.fill_grad(out, self.cfg, worker, step, tensor, dense=self.dense)

    def _fill_arena(self, arena: torch.Tensor, worker: int, step: int):
        for i in range(self.cfg.num_tensors):
            self.gen_grad(worker, step, i, out=self.view(arena, i))

    def prepare_step(self, step: int, capture=None, compressed=None):
        """Everything the observed worker's step consumes: its own gradient, and either the
        peers' packed streams (compressed step) or the fp32 sum of all gradients and, with
        full_grads, the peers' gradients themselves (correction or warm-up pass).

        `step` seeds the gradients; `compressed` overrides the step % k rule (a trainer with
        warm-up passes numbers its iterations differently).
        capture: optional list of (tensor, start, length); the matching slices of every
        worker's gradient are returned as host arrays, out[worker][slice] (for checkers)."""
        comp = self.compressed(step) if compressed is None else bool(compressed)
        t = self.cfg.threshold
        if not comp:
            self.agg_full.zero_()
        captured = []
        if self._scratch is None:
            self._scratch = torch.zeros(self.total, dtype=torch.float32, device=self.device)
        g = self._scratch
        for j in range(self.N):
            self._fill_arena(g, j, step)
            if self.grad_dtype != torch.float32:
                g.copy_(g.to(self.grad_dtype))      # round once: every worker's values are representable
            if j == self.self_rank:
                self.grad.copy_(g)
            else:
                if self.full_grads:
                    self.peer_grad[j].copy_(g)
                if comp:
                    if self.peer_residual[j] is None:
                        raise RuntimeError("this workload was built without peer residuals")
                    if self.thresholds is None:
                        binding.cdsgd_quantize_pack(g, self.peer_residual[j], self.peer_packed[j], t)
                    else:
                        for i in range(self.cfg.num_tensors):
                            binding.cdsgd_quantize_pack(self.view(g, i), self.view(self.peer_residual[j], i),
                                                        self.pview(self.peer_packed[j], i), self.thresholds[i])
                    if self.sparse_peers:
                        for i, n in enumerate(self.cfg.sizes):
                            binding.cdsgd_sparse_encode(self.pview(self.peer_packed[j], i), n,
                                                        self.sview(self.peer_sparse[j], i))
            if not comp:
                self.agg_full.add_(g)   # worker order 0..N-1, fp32, from +0
            if capture is not None:
                captured.append([self.view(g, i)[a: a + ln].cpu().numpy() for (i, a, ln) in capture])
        return captured if capture is not None else None

    # -- the step itself ------------------------------------------------------
    def fused_step(self, step: int):
        c = self.cfg
        self.plan.step(step, c.k, c.threshold, c.lr, c.lr)

    def unfused_step(self, step: int):
        c = self.cfg
        if self._agg is None:
            self._agg = torch.zeros(self.total, dtype=torch.float32, device=self.device)
        for i in range(c.num_tensors):
            wg, wl = self.view(self.w_global, i), self.view(self.w_local, i)
            g = self.view(self.grad, i)
            assert self.grad_dtype == torch.float32, "the three single-tensor calls take fp32 gradients"
            if self.compressed(step):
                binding.cdsgd_quantize_pack(g, self.view(self.residual, i), self.pview(self.packed_self, i),
                                            c.threshold)
                streams = [self.pview(self.packed_self if j == self.self_rank else self.peer_packed[j], i)
                           for j in range(self.N)]
                agg = self.view(self._agg, i)
                binding.cdsgd_decode_sum(streams, agg, c.threshold)
            else:
                agg = self.view(self.agg_full, i)
            binding.cdsgd_update(wg, wl, g, agg, c.lr, c.lr, self.N)

    def destroy(self):
        self.plan.destroy()
