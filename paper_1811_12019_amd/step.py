"""Whole-network K-FAC step on one GPU: owns the device buffers of every layer and enqueues the C-ABI
calls in the order of Algorithm 1 (stages 1, 2, 4, 5) for all layers locally.

No arithmetic happens here: every number is produced by the HIP library.  torch is used for device
memory, seeded synthetic inputs and the stream.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as kb
from .synth import LayerShape, SIGMA_GOUT, SIGMA_GRADW


def device_inputs(shape: LayerShape, seed: int, layer_idx: int, step: int, dtype: int, device="cuda"):
    """Seeded synthetic (act, gout, gradW) generated on the device, NHWC memory order.

    act/gout are returned as (N, H, W, C) tensors of the requested dtype; the logical (n, c, y, x) tensor
    the definitions refer to is ``t.permute(0, 3, 1, 2)``.
    """
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + layer_idx) * 1000003 + step)
    tdt = kb._TORCH_DTYPE[dtype]
    act = torch.randn((shape.N, shape.H, shape.W, shape.C_in), generator=g, device=device, dtype=torch.float32)
    if shape.relu_input:
        act.clamp_(min=0)
    gout = torch.randn((shape.N, shape.H_out, shape.W_out, shape.C_out), generator=g, device=device,
                       dtype=torch.float32) * SIGMA_GOUT
    gradw = torch.randn((shape.d_G, shape.d_A), generator=g, device=device, dtype=torch.float32) * SIGMA_GRADW
    return act.to(tdt).contiguous(), gout.to(tdt).contiguous(), gradw.contiguous()


class LayerState:
    def __init__(self, shape: LayerShape, idx: int, dtype: int, order: int, seed: int, device):
        self.shape = shape
        self.desc = kb.make_desc(shape, kb.KFAC_NHWC, dtype, order)
        self.act, self.gout, self.gradW = device_inputs(shape, seed, idx, 0, dtype, device)
        dA, dG = shape.d_A, shape.d_G
        f32 = dict(dtype=torch.float32, device=device)
        self.A_new, self.G_new = torch.empty((dA, dA), **f32), torch.empty((dG, dG), **f32)
        self.A_run, self.G_run = torch.eye(dA, **f32), torch.eye(dG, **f32)      # running averages start at I
        self.A_inv, self.G_inv = torch.empty((dA, dA), **f32), torch.empty((dG, dG), **f32)
        self.P = torch.empty((dG, dA), **f32)


class KfacNetworkStep:
    """All layers of a network resident on one GPU; step() = factor builds, running averages,
    damped inverses (optionally skipped: stale inverses) and preconditioning for every layer."""

    def __init__(self, layers: Sequence[LayerShape], dtype: int = kb.KFAC_BF16, order: int = kb.KFAC_ORDER_KH_KW_C,
                 decay: Optional[float] = 0.95, gamma: float = 1e-3, seed: int = 0, device="cuda",
                 inverse_streams: int = 3):
        self.decay = decay
        self.damping = float(gamma) ** 0.5           # sqrt(gamma) on each factor
        self.layers: List[LayerState] = [LayerState(s, i, dtype, order, seed, device) for i, s in enumerate(layers)]
        builds = []
        for l in self.layers:
            builds.append((kb.KFAC_OP_FACTOR_A, l.desc, l.act, l.A_new, 0.0))
            builds.append((kb.KFAC_OP_FACTOR_G, l.desc, l.gout, l.G_new, 0.0))
        self.factor_batch = kb.FactorBatch(builds, device=device)
        self.pre_batch = kb.PrecondBatch([l.G_inv for l in self.layers], [l.A_inv for l in self.layers],
                                         [l.gradW for l in self.layers], [l.P for l in self.layers], device=device)
        self.ema_batch = kb.EmaBatch([t for l in self.layers for t in (l.A_run, l.G_run)],
                                     [t for l in self.layers for t in (l.A_new, l.G_new)])
        src = []
        for l in self.layers:
            src += [l.A_run if decay is not None else l.A_new, l.G_run if decay is not None else l.G_new]
        dst = []
        for l in self.layers:
            dst += [l.A_inv, l.G_inv]
        # The inversions are independent, so they are dealt (largest first, to the least loaded group, by d^3) into a
        # few groups that run on streams of their own: the latency-bound pivot/panel kernels of one group then overlap
        # with the throughput-bound rank-128 updates of the others.
        n_groups = max(1, min(inverse_streams, len(src)))
        order_by_size = sorted(range(len(src)), key=lambda i: -src[i].shape[0])
        groups, load = [[] for _ in range(n_groups)], [0.0] * n_groups
        for i in order_by_size:
            g = load.index(min(load))
            groups[g].append(i)
            load[g] += float(src[i].shape[0]) ** 3
        self.inv_batches = [kb.InverseBatch([src[i] for i in grp], [dst[i] for i in grp], [self.damping] * len(grp),
                                            device=device)
                            for grp in groups if grp]
        self.inv_streams = [torch.cuda.Stream(device=device) for _ in self.inv_batches[1:]]
        self.overlap_inversions = True      # False: run the groups one after the other on the caller's stream

    # -- stages ------------------------------------------------------------------------------
    def build_factors(self, stream=None):
        kb.kfac_factor_batched(self.factor_batch, stream)

    def update_running(self, stream=None):
        if self.decay is None:
            return
        kb.kfac_ema_batched(self.ema_batch, self.decay, stream)

    def invert(self, stream=None):
        main = torch.cuda.current_stream() if stream is None else stream
        if len(self.inv_batches) == 1 or not self.overlap_inversions:
            for batch in self.inv_batches:
                kb.kfac_damped_inverse_batched(batch, main)
            return
        fork = torch.cuda.Event()
        fork.record(main)
        joins = []
        for batch, side in zip(self.inv_batches[1:], self.inv_streams):
            side.wait_event(fork)
            kb.kfac_damped_inverse_batched(batch, side)
            done = torch.cuda.Event()
            done.record(side)
            joins.append(done)
        kb.kfac_damped_inverse_batched(self.inv_batches[0], main)
        for done in joins:
            main.wait_event(done)

    def inverse_info(self) -> torch.Tensor:
        """Status words of all inversions (0 = positive definite)."""
        return torch.cat([b.info for b in self.inv_batches])

    def precondition(self, stream=None):
        kb.kfac_precondition_batched(self.pre_batch, stream)

    def step(self, refresh_inverse: bool = True, stream=None):
        self.build_factors(stream)
        self.update_running(stream)
        if refresh_inverse:
            self.invert(stream)
        self.precondition(stream)

    def reset_running(self):
        for l in self.layers:
            l.A_run.copy_(torch.eye(l.shape.d_A, device=l.A_run.device))
            l.G_run.copy_(torch.eye(l.shape.d_G, device=l.G_run.device))


def refresh_interval(epoch: int) -> int:
    """Iterations between refreshes of the statistics in epoch e (Sec. 5.4, first heuristic): min(20, 5 floor(e/5) + 1)."""
    return min(20, 5 * (int(epoch) // 5) + 1)


def refresh_interval_late(epoch: int) -> int:
    """Second heuristic of Sec. 5.4: every iteration before epoch 13, every 20th afterwards."""
    return 1 if int(epoch) < 13 else 20


def learning_rate(epoch: float, eta0: float, e_start: float, e_end: float, p_decay: float) -> float:
    """Polynomial decay of Sec. 4.3 (eta0 before e_start, 0 after e_end)."""
    if epoch <= e_start:
        return float(eta0)
    if epoch >= e_end:
        return 0.0
    return float(eta0) * (1.0 - (epoch - e_start) / (e_end - e_start)) ** p_decay


def momentum_rate(eta: float, eta0: float, m0: float) -> float:
    """m(e) = m0 / eta0 * eta(e) (Sec. 4.3)."""
    return float(m0) / float(eta0) * float(eta)


# Algorithmic work, for rooflines (2 flops per multiply-add; symmetric outputs counted as a triangle).
def factor_flops(rows: int, dim: int) -> float:
    return float(rows) * dim * (dim + 1)


def inverse_flops(dim: int) -> float:
    return float(dim) ** 3


def precondition_flops(dG: int, dA: int) -> float:
    return 2.0 * dG * dG * dA + 2.0 * dG * dA * dA


INVERSE_BLOCK = 128     # elimination block of the library's blocked sweep


def inverse_update_flops_split(dim: int):
    """Flops of the rank-b updates of the blocked sweep (triangle of the part outside each pivot block):
    (all steps but the matrix's last, the last step)."""
    if dim <= INVERSE_BLOCK:
        return 0.0, 0.0
    mid, last, k0 = 0.0, 0.0, 0
    while k0 < dim:
        b = min(INVERSE_BLOCK, dim - k0)
        rest = dim - b
        work = float(rest) * (rest + 1) * b
        if k0 + b >= dim:
            last += work
        else:
            mid += work
        k0 += b
    return mid, last


def inverse_update_flops(dim: int) -> float:
    return sum(inverse_update_flops_split(dim))


def inverse_pivot_flops(dim: int) -> float:
    """Flops of the pivot-block inversions of the blocked sweep (b^3 per b x b block)."""
    total, k0 = 0.0, 0
    while k0 < dim:
        b = min(INVERSE_BLOCK, dim - k0)
        total += float(b) ** 3
        k0 += b
    return total


def inverse_first_pivot_flops(dim: int) -> float:
    """The first pivot block's share of inverse_pivot_flops: the only one inverted by a launch of its own (the later
    ones are inverted inside the update launch of the step before)."""
    return float(min(INVERSE_BLOCK, dim)) ** 3


def inverse_panel_flops(dim: int) -> float:
    """Flops of the panel products T = W_:k P of the blocked sweep (every row outside the pivot block)."""
    if dim <= INVERSE_BLOCK:
        return 0.0
    total, k0 = 0.0, 0
    while k0 < dim:
        b = min(INVERSE_BLOCK, dim - k0)
        total += 2.0 * (dim - b) * b * b
        k0 += b
    return total
