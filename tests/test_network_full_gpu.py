"""GPU parity at the target configuration: one K-FAC step of all 54 conv/fc layers of ResNet-50 at per-GPU batch 32,
in the launch configuration the benchmark times (KfacNetworkStep's default two-wave schedule, batched entry points
only), every stage of every layer against the float64 oracle (Sec. 3.2 Eq. 5-7; Algorithm 1 stages 1, 2, 4, 5).

Each stage is checked against the oracle fed the GPU stage's own fp32 input ("identical rounded inputs"), with the
relative Frobenius bars of the target (factors 1e-2 -- the kernels meet FACTOR_TOL --, inverse and preconditioned
gradient 1e-4) and, beside every norm, an element-wise bound max|got - ref| <= c max|ref| so that a single misplaced
entry cannot hide inside a norm.  This is also the only place where the batched inverse sees more matrices than one
launch's argument block describes (76 in the second wave) and where preconditioning runs at d_A = 4609.
"""
import numpy as np
import pytest
import torch

from oracle import kfac_oracle as ko
from paper_1811_12019_amd import binding as kb
from paper_1811_12019_amd import synth

pytestmark = pytest.mark.gpu

# The fresh factor is not stored in this schedule; the one implied by the running average, (S - rho I) / (1 - rho), carries
# the fp32 rounding of S (half an ulp of ~1, 3e-8) divided by 1 - rho = 0.05 and by the factor's own size (1e-2 for the G
# factors): up to 1e-4 of its largest entry.  The stated bar is 1e-2; the builders alone are held to 2e-5 in
# test_parity_gpu.py, on the same full-size layers.
FACTOR_TOL = 5e-4
FACTOR_MAX_TOL = 5e-4
EMA_TOL = 1e-6          # relative Frobenius, running average (mostly the identity it started from)
EMA_MAX_TOL = 2e-7      # element-wise, relative to the largest entry (one fp32 multiply-add per element)
INV_TOL = 1e-4          # relative Frobenius (the stated bar)
INV_MAX_TOL = 1e-4      # element-wise, relative to the largest entry of the inverse
PRE_TOL = 1e-4
PRE_MAX_TOL = 1e-4
DECAY, GAMMA = 0.95, 1e-3
LAYERS = synth.resnet50_layers(32)
WORST = {}


def rel_fro(got, want):
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def rel_max(got, want):
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-300))


def note(stage, name, fro, mx):
    w = WORST.setdefault(stage, [0.0, "", 0.0, ""])
    if fro > w[0]:
        w[0], w[1] = fro, name
    if mx > w[2]:
        w[2], w[3] = mx, name


@pytest.fixture(scope="module")
def net():
    from paper_1811_12019_amd import step as kstep
    n = kstep.KfacNetworkStep(LAYERS, dtype=kb.KFAC_BF16, order=kb.KFAC_ORDER_KH_KW_C, decay=DECAY, gamma=GAMMA,
                              seed=0, device="cuda")
    assert n.pipelined and len(n.waves) == 2 and n.fused_ema         # the schedule the benchmark times
    assert max(b.count for w in n.waves for b in w.inv_batches) > 64  # more matrices than one launch group holds
    for l in n.layers:                                                # poison every output: nothing may be left unwritten
        for t in (l.A_inv, l.G_inv, l.P):
            t.fill_(float("nan"))
    n.step()
    torch.cuda.synchronize()
    assert int(n.inverse_info().abs().max()) == 0
    yield n
    del n
    torch.cuda.empty_cache()


def f64(t):
    return t.detach().cpu().numpy().astype(np.float64)


def nchw(t):
    return t.float().permute(0, 3, 1, 2).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("idx", range(len(LAYERS)), ids=[s.name for s in LAYERS])
def test_resnet50_batch32_step_layer(net, idx):
    l = net.layers[idx]
    s = l.shape
    lam = float(np.float32(ko.factor_damping(GAMMA)))
    A_run, G_run = f64(l.A_run), f64(l.G_run)
    A_inv, G_inv = f64(l.A_inv), f64(l.G_inv)
    P = f64(l.P)
    for m in (A_run, G_run, A_inv, G_inv, P):
        assert np.isfinite(m).all(), s.name
    # stages 1, 2 and the running average from identity, formed in the builders' epilogues (the fresh factor is never
    # stored): against the oracle's factor of the bf16 tensors the GPU read, folded into I by the oracle.  The fresh
    # factor implied by the result, (S - rho I) / (1 - rho), meets the factor tolerance too.
    for tag, got, ref in (("A", A_run, ko.factor_A(nchw(l.act), s.kh, s.kw, s.stride, s.pad, True, ko.ORDER_KH_KW_C)),
                          ("G", G_run, ko.factor_G(nchw(l.gout)))):
        want = ko.ema(np.eye(ref.shape[0]), ref, DECAY)
        fro, mx = rel_fro(got, want), rel_max(got, want)
        note("ema_" + tag, s.name, fro, mx)
        assert fro < EMA_TOL and mx < EMA_MAX_TOL, (s.name, tag, fro, mx)
        np.testing.assert_array_equal(got, got.T)
        implied = (got - DECAY * np.eye(ref.shape[0])) / (1.0 - DECAY)
        fro, mx = rel_fro(implied, ref), rel_max(implied, ref)
        note("factor_" + tag, s.name, fro, mx)
        assert fro < FACTOR_TOL and mx < FACTOR_MAX_TOL, (s.name, tag, fro, mx)
    assert A_run[-1, -1] == pytest.approx(1.0, rel=1e-6)
    # stage 4: damped inverse of the GPU's own running average
    for tag, got, run in (("A", A_inv, A_run), ("G", G_inv, G_run)):
        ref = ko.damped_inverse(run, lam)
        fro, mx = rel_fro(got, ref), rel_max(got, ref)
        note("inverse_" + tag, s.name, fro, mx)
        assert fro < INV_TOL and mx < INV_MAX_TOL, (s.name, tag, fro, mx)
        np.testing.assert_array_equal(got, got.T)
    # stage 5: preconditioned gradient from the GPU's own inverses
    ref = ko.precondition(G_inv, f64(l.gradW), A_inv)
    fro, mx = rel_fro(P, ref), rel_max(P, ref)
    note("precondition", s.name, fro, mx)
    assert fro < PRE_TOL and mx < PRE_MAX_TOL, (s.name, fro, mx)


def test_resnet50_batch32_step_worst_errors(net):
    """Prints the worst error of every stage over the 54 layers (run with -s to see it)."""
    assert len(WORST) == 7
    for stage, (fro, n1, mx, n2) in sorted(WORST.items()):
        print(f"full-network parity: {stage:14s} worst rel. Frobenius {fro:.2e} ({n1}), worst max-entry {mx:.2e} ({n2})")
