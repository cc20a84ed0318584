"""Whole-network K-FAC step on one GPU: owns the device buffers of every layer and enqueues the C-ABI
calls in the order of Algorithm 1 (stages 1, 2, 4, 5) for all layers locally.

No arithmetic of the method happens here: every number is produced by the HIP library (the schedules of Sec. 4.2 and
5.4 are host functions of the library too: binding.kfac_warmup_damping_*, binding.kfac_refresh_interval).  torch is used for device
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
        # scratch of the batched calls, owned here so that the call tables of the stage-wise schedule and of the two
        # waves (which never run at the same time) share it
        self.factor_ws = [kb.alloc_workspace(kb.kfac_factor_workspace_bytes(op, self.desc), device)
                          for op in (kb.KFAC_OP_FACTOR_A, kb.KFAC_OP_FACTOR_G)]
        self.inverse_ws = [kb.alloc_workspace(kb.kfac_inverse_workspace_bytes(d), device) for d in (dA, dG)]
        # the inverses a second time, as the fp16 piece planes the preconditioning products multiply from (written by the
        # inversions, kept with the inverses while these are stale)
        self.A_planes, self.G_planes = (kb.alloc_workspace(kb.kfac_inverse_planes_bytes(d), device) for d in (dA, dG))
        self.pre_ws = kb.alloc_workspace(kb.kfac_precondition_workspace_bytes(dG, dA), device)


INVERSE_BLOCK = 128     # elimination block of the library's blocked sweep

_SIDE_STREAMS = {}


def _side_streams(device, n: int):
    """The n side streams of a device, created once and shared by every network object: which hardware queue a stream
    lands on depends on the order in which the process creates its streams, and a step whose streams share a hardware
    queue (there are four) runs up to 30 % slower, so every object gets the same, first-created ones."""
    key = str(torch.device(device))
    pool = _SIDE_STREAMS.setdefault(key, [])
    while len(pool) < n:
        pool.append(torch.cuda.Stream(device=device))
    return pool[:n]


class _Wave:
    """A subset of the layers with batched-call tables of its own."""

    def __init__(self, layers: List[LayerState], decay, damping: float, n_groups: int, device, pi_split: bool = False,
                 fused_ema: bool = False):
        self.layers = layers
        builds = []
        for l in layers:
            builds.append((kb.KFAC_OP_FACTOR_A, l.desc, l.act, l.A_new, 0.0))
            builds.append((kb.KFAC_OP_FACTOR_G, l.desc, l.gout, l.G_new, 0.0))
        # fused: every build folds its result into the running average in its own epilogue (no fresh factor is stored)
        self.fused_ema = bool(fused_ema and decay is not None)
        fws = [w for l in layers for w in l.factor_ws]
        self.factor_batch = (kb.FactorBatch(builds, device=device, running=[t for l in layers for t in (l.A_run, l.G_run)],
                                            decay=decay, ws=fws) if self.fused_ema
                             else kb.FactorBatch(builds, device=device, ws=fws))
        self.pre_batch = kb.PrecondBatch([l.G_inv for l in layers], [l.A_inv for l in layers],
                                         [l.gradW for l in layers], [l.P for l in layers], device=device,
                                         ws=[l.pre_ws for l in layers], Ginv_planes=[l.G_planes for l in layers],
                                         Ainv_planes=[l.A_planes for l in layers])
        self.ema_batch = kb.EmaBatch([t for l in layers for t in (l.A_run, l.G_run)],
                                     [t for l in layers for t in (l.A_new, l.G_new)])
        src, dst, iws, planes = [], [], [], []
        for l in layers:
            src += [l.A_run if decay is not None else l.A_new, l.G_run if decay is not None else l.G_new]
            dst += [l.A_inv, l.G_inv]
            iws += l.inverse_ws
            planes += [l.A_planes, l.G_planes]
        # trace-ratio split of the damping between a layer's factors: computed on the device before the inversions,
        # which read their damping from there
        self.pi_batch = kb.PiBatch(src[0::2], src[1::2], device=device) if pi_split else None
        lam_dev = ([self.pi_batch.address(i // 2, i % 2) for i in range(len(src))] if pi_split else None)
        # The inversions are independent, so they are dealt (largest first, to the least loaded group, by d^3) into a
        # few groups that run on streams of their own: the latency-bound pivot / panel kernels of one group then
        # overlap with the throughput-bound updates of the others.  (Grouping by block count instead, so that a
        # group's launches are all equally long, measured 2 % slower.)
        n_groups = max(1, min(n_groups, len(src)))
        order_by_size = sorted(range(len(src)), key=lambda i: -src[i].shape[0])
        groups, load = [[] for _ in range(n_groups)], [0.0] * n_groups
        for i in order_by_size:
            g = load.index(min(load))
            groups[g].append(i)
            load[g] += float(src[i].shape[0]) ** 3
        self.inv_batches = [kb.InverseBatch([src[i] for i in grp], [dst[i] for i in grp], [damping] * len(grp),
                                            device=device, ws=[iws[i] for i in grp], planes=[planes[i] for i in grp],
                                            dampings_dev=None if lam_dev is None else [lam_dev[i] for i in grp])
                            for grp in groups if grp]


class KfacNetworkStep:
    """All layers of a network resident on one GPU; step() = factor builds, running averages,
    damped inverses (optionally skipped: stale inverses) and preconditioning for every layer.

    The stage methods (build_factors, update_running, invert, precondition) run one stage for the whole network.
    step() strings them together when pipelined is False.  By default it works in two waves instead: the inversion of
    a 4609-wide factor is a chain of ~110 small dependent launches that takes about half of the whole step and leaves
    most of the GPU idle, so the factors of the layers with a factor of long_dim or more are built first and their
    inversions started on the side streams at once; the other layers' stages run on the launch stream beside them,
    and each wave is preconditioned when its inverses are done."""

    def __init__(self, layers: Sequence[LayerShape], dtype: int = kb.KFAC_BF16, order: int = kb.KFAC_ORDER_KH_KW_C,
                 decay: Optional[float] = 0.95, gamma: float = 1e-3, seed: int = 0, device="cuda",
                 inverse_streams: int = 3, long_dim: int = 2048, pi_split: bool = False, fused_ema: bool = True):
        self.decay = decay
        self.gamma = float(gamma)
        self.pi_split = pi_split                     # False: sqrt(gamma) on each factor; True: the trace-ratio split
        self.damping = float(gamma) ** 0.5           # sqrt(gamma) on each factor
        self.layers: List[LayerState] = [LayerState(s, i, dtype, order, seed, device) for i, s in enumerate(layers)]
        self.fused_ema = bool(fused_ema and decay is not None)   # running averages formed by the builders themselves
        self.all = _Wave(self.layers, decay, self.damping, inverse_streams, device, pi_split, fused_ema)
        long_ = [l for l in self.layers if max(l.shape.d_A, l.shape.d_G) >= long_dim]
        short = [l for l in self.layers if max(l.shape.d_A, l.shape.d_G) < long_dim]
        self.waves = ([_Wave(long_, decay, self.damping, inverse_streams, device, pi_split, fused_ema),
                       _Wave(short, decay, self.damping, 1, device, pi_split, fused_ema)] if long_ and short else [])
        self.inv_streams = _side_streams(device, max(1, inverse_streams))
        self.overlap_inversions = True      # False: run the groups one after the other on the caller's stream
        self.pipelined = True               # False: step() runs stage after stage

    # -- stages ------------------------------------------------------------------------------
    def build_factors(self, stream=None):
        kb.kfac_factor_batched(self.all.factor_batch, stream)

    def update_running(self, stream=None):
        if self.decay is None or self.fused_ema:
            return
        kb.kfac_ema_batched(self.all.ema_batch, self.decay, stream)

    def _split_damping(self, wave, stream):
        if wave.pi_batch is not None:
            kb.kfac_pi_damping_batched(wave.pi_batch, self.gamma, stream)

    @staticmethod
    def _fork(batches, sides, main):
        """batches[i] on sides[i], after what `main` holds now; returns the events to join on."""
        fork = torch.cuda.Event()
        fork.record(main)
        joins = []
        for batch, side in zip(batches, sides):
            side.wait_event(fork)
            kb.kfac_damped_inverse_batched(batch, side)
            done = torch.cuda.Event()
            done.record(side)
            joins.append(done)
        return joins

    def invert(self, stream=None):
        main = torch.cuda.current_stream() if stream is None else stream
        batches = self.all.inv_batches
        self._split_damping(self.all, main)
        if not self.overlap_inversions or len(batches) == 1:
            for batch in batches:
                kb.kfac_damped_inverse_batched(batch, main)
            return
        joins = self._fork(batches, self.inv_streams, main)
        for done in joins:
            main.wait_event(done)

    def inverse_info(self) -> torch.Tensor:
        """Status words of all inversions (0 = positive definite)."""
        sets = self.waves if self._use_waves(True) else [self.all]
        return torch.cat([b.info for w in sets for b in w.inv_batches])

    def precondition(self, stream=None):
        kb.kfac_precondition_batched(self.all.pre_batch, stream)

    def _use_waves(self, refresh_inverse: bool) -> bool:
        return bool(self.pipelined and self.overlap_inversions and refresh_inverse and self.waves)

    def step(self, refresh_inverse: bool = True, stream=None):
        if not self._use_waves(refresh_inverse):
            self.build_factors(stream)
            self.update_running(stream)
            if refresh_inverse:
                self.invert(stream)
            self.precondition(stream)
            return
        main = torch.cuda.current_stream() if stream is None else stream
        lw, sw = self.waves
        kb.kfac_factor_batched(lw.factor_batch, main)
        if self.decay is not None and not self.fused_ema:
            kb.kfac_ema_batched(lw.ema_batch, self.decay, main)
        self._split_damping(lw, main)
        joins = self._fork(lw.inv_batches, self.inv_streams, main)
        kb.kfac_factor_batched(sw.factor_batch, main)
        if self.decay is not None and not self.fused_ema:
            kb.kfac_ema_batched(sw.ema_batch, self.decay, main)
        self._split_damping(sw, main)
        for batch in sw.inv_batches:
            kb.kfac_damped_inverse_batched(batch, main)
        kb.kfac_precondition_batched(sw.pre_batch, main)
        for done in joins:
            main.wait_event(done)
        kb.kfac_precondition_batched(lw.pre_batch, main)

    def reset_running(self):
        for l in self.layers:
            l.A_run.copy_(torch.eye(l.shape.d_A, device=l.A_run.device))
            l.G_run.copy_(torch.eye(l.shape.d_G, device=l.G_run.device))


# Algorithmic work, for rooflines (2 flops per multiply-add; symmetric outputs counted as a triangle).
def factor_flops(rows: int, dim: int) -> float:
    return float(rows) * dim * (dim + 1)


def inverse_flops(dim: int) -> float:
    return float(dim) ** 3


def precondition_flops(dG: int, dA: int) -> float:
    return 2.0 * dG * dG * dA + 2.0 * dG * dA * dA



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
