"""GPU parity: every C-ABI entry point against the float64 oracle on the same seeded inputs.

Tolerances (relative Frobenius error):
  * factors built from bf16 / fp16 / fp32 inputs, oracle fed the identical rounded inputs: 1e-2 allowed by the
    target; the kernels accumulate in fp32, so FACTOR_TOL below is much tighter;
  * fp32 inverse and preconditioned gradient, oracle run on the GPU stage's own fp32 input: 1e-4.
"""
import numpy as np
import pytest
import torch

from oracle import kfac_oracle as ko
from paper_1811_12019_amd import binding as kb
from paper_1811_12019_amd import synth

pytestmark = pytest.mark.gpu

FACTOR_TOL = 2e-5      # fp32 accumulation of exactly representable products; the stated bar is 1e-2
INV_TOL = 1e-4
PRE_TOL = 1e-4
DEV = "cuda"

_NP_ROUND = {kb.KFAC_F32: lambda x: x.astype(np.float32),
             kb.KFAC_BF16: synth.round_to_bf16,
             kb.KFAC_F16: lambda x: x.astype(np.float16).astype(np.float32)}


def rel_fro(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def rel_max(got, want):
    """Largest entry-wise error relative to the largest entry: a single misplaced entry cannot hide in it."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-300))


def gpu_factor(op, shape, x_rounded, layout, dtype, order, scale=0.0):
    desc = kb.make_desc(shape, layout, dtype, order)
    xt = kb.to_device_tensor(x_rounded, layout, dtype, DEV)
    d = shape.d_A if op == kb.KFAC_OP_FACTOR_A else shape.d_G
    out = torch.full((d, d), float("nan"), dtype=torch.float32, device=DEV)
    ws = kb.alloc_workspace(kb.kfac_factor_workspace_bytes(op, desc), DEV)
    fn = kb.kfac_factor_A if op == kb.KFAC_OP_FACTOR_A else kb.kfac_factor_G
    fn(desc, xt, scale, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check_factor_pair(shape, layout, dtype, order, seed=0):
    rnd = _NP_ROUND[dtype]
    act = rnd(synth.make_act(shape, seed))
    gout = rnd(synth.make_gout(shape, seed))
    A = gpu_factor(kb.KFAC_OP_FACTOR_A, shape, act, layout, dtype, order)
    G = gpu_factor(kb.KFAC_OP_FACTOR_G, shape, gout, layout, dtype, order)
    A_ref = ko.factor_A(act, shape.kh, shape.kw, shape.stride, shape.pad, shape.has_bias, order)
    G_ref = ko.factor_G(gout)
    assert A.shape == A_ref.shape and G.shape == G_ref.shape
    assert np.isfinite(A).all() and np.isfinite(G).all()
    assert rel_fro(A, A_ref) < FACTOR_TOL, rel_fro(A, A_ref)
    assert rel_fro(G, G_ref) < FACTOR_TOL, rel_fro(G, G_ref)
    assert rel_max(A, A_ref) < FACTOR_TOL, rel_max(A, A_ref)
    assert rel_max(G, G_ref) < FACTOR_TOL, rel_max(G, G_ref)
    np.testing.assert_array_equal(A, A.T)
    np.testing.assert_array_equal(G, G.T)
    if shape.has_bias:
        assert A[-1, -1] == pytest.approx(1.0, rel=1e-6)
    return A, G


# ----------------------------------------------------------------------------------------------
# factors
# ----------------------------------------------------------------------------------------------
def test_factors_config0_fp32_nchw():
    shp = synth.config0()
    for order in (kb.KFAC_ORDER_C_KH_KW, kb.KFAC_ORDER_KH_KW_C):
        A, G = check_factor_pair(shp, kb.KFAC_NCHW, kb.KFAC_F32, order)
        assert A.shape == (145, 145) and G.shape == (16, 16)


SMALL_SHAPES = [
    # name, N, C_in, H, W, C_out, kh, kw, stride, pad  -- several tiles and a ragged tail in every dimension
    synth.LayerShape("s3x3", 3, 40, 9, 9, 70, 3, 3, 1, 1),
    synth.LayerShape("s3x3s2", 2, 24, 11, 11, 130, 3, 3, 2, 1),
    synth.LayerShape("s7x7s2", 2, 3, 37, 37, 64, 7, 7, 2, 3, relu_input=False),
    synth.LayerShape("s1x1", 5, 136, 7, 7, 72, 1, 1, 1, 0),
    synth.LayerShape("s1x1s2", 3, 64, 10, 10, 200, 1, 1, 2, 0),
    synth.LayerShape("fc", 32, 300, 1, 1, 100, 1, 1, 1, 0),
    synth.LayerShape("nobias", 2, 16, 6, 6, 8, 3, 3, 1, 1, has_bias=False),
    synth.LayerShape("rect", 2, 5, 6, 9, 7, 2, 3, 1, 1),
]


@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("layout,dtype,order", [
    (kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C),
    (kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_C_KH_KW),
    (kb.KFAC_NCHW, kb.KFAC_F32, kb.KFAC_ORDER_C_KH_KW),
    (kb.KFAC_NCHW, kb.KFAC_F16, kb.KFAC_ORDER_KH_KW_C),
    (kb.KFAC_NHWC, kb.KFAC_F32, kb.KFAC_ORDER_KH_KW_C),
    (kb.KFAC_NHWC, kb.KFAC_F16, kb.KFAC_ORDER_KH_KW_C),
])
def test_factors_small_shapes(shape, layout, dtype, order):
    check_factor_pair(shape, layout, dtype, order, seed=1)


@pytest.mark.parametrize("name", ["layer1.0.conv2", "layer2.0.downsample", "layer3.1.conv2", "layer4.0.conv1", "fc"])
def test_factors_resnet_layers_full_size(name):
    """Full-size ResNet-50 layers at batch 32 in the benchmark's launch configuration (NHWC bf16, (kh,kw,c) order):
    3x3 with 100,352 rows (split over rows), strided 1x1 shortcut, 2305-dim 3x3, 1025-dim 1x1, fc."""
    shp = {l.name: l for l in synth.resnet50_layers(32)}[name]
    check_factor_pair(shp, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C, seed=5)


GATHER_SHAPES = [
    # narrow layers (channels not a multiple of 8) with thousands of rows: the gather-based matrix-core kernel
    synth.LayerShape("g7x7s2", 4, 3, 70, 70, 16, 7, 7, 2, 3, relu_input=False),      # 4,900 rows, 148 columns
    synth.LayerShape("g3x3c5", 3, 5, 48, 50, 8, 3, 3, 1, 1),                         # 7,200 rows, 46 columns
    synth.LayerShape("g1x1c17", 2, 17, 50, 47, 8, 1, 1, 1, 0),                       # 4,700 rows, 18 columns
    synth.LayerShape("g5x5nobias", 2, 6, 52, 52, 8, 5, 5, 1, 2, has_bias=False),     # 5,408 rows, 150 columns
]


@pytest.mark.parametrize("shape", GATHER_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("dtype", [kb.KFAC_BF16, kb.KFAC_F16])
def test_factors_narrow_layers(shape, dtype):
    check_factor_pair(shape, kb.KFAC_NHWC, dtype, kb.KFAC_ORDER_KH_KW_C, seed=3)


def test_factor_image_too_wide_for_the_packed_patch_origin():
    """An image wider than the matrix-core kernel's 16-bit patch coordinates allow is served by another kernel."""
    shp = synth.LayerShape("wide", 1, 8, 3, 17000, 8, 3, 3, 1, 1)
    check_factor_pair(shp, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)


def test_factor_batched_matches_single_calls():
    """A mixed batch (1x1, 3x3, strided, fc, a layer only the generic kernel serves) equals the single calls bit for bit."""
    shapes = [SMALL_SHAPES[0], SMALL_SHAPES[1], SMALL_SHAPES[3], SMALL_SHAPES[4], SMALL_SHAPES[5], SMALL_SHAPES[2]]
    builds, keep, singles = [], [], []
    for i, shp in enumerate(shapes):
        desc = kb.make_desc(shp, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
        act = synth.round_to_bf16(synth.make_act(shp, 7 + i))
        gout = synth.round_to_bf16(synth.make_gout(shp, 7 + i))
        at = kb.to_device_tensor(act, kb.KFAC_NHWC, kb.KFAC_BF16, DEV)
        gt = kb.to_device_tensor(gout, kb.KFAC_NHWC, kb.KFAC_BF16, DEV)
        A = torch.full((shp.d_A, shp.d_A), float("nan"), device=DEV)
        G = torch.full((shp.d_G, shp.d_G), float("nan"), device=DEV)
        builds += [(kb.KFAC_OP_FACTOR_A, desc, at, A, 0.0), (kb.KFAC_OP_FACTOR_G, desc, gt, G, 0.0)]
        keep.append((shp, act, gout, A, G))
    batch = kb.FactorBatch(builds, device=DEV)
    kb.kfac_factor_batched(batch)
    torch.cuda.synchronize()
    for shp, act, gout, A, G in keep:
        A_ref = ko.factor_A(act, shp.kh, shp.kw, shp.stride, shp.pad, True, ko.ORDER_KH_KW_C)
        assert rel_fro(A.cpu().numpy(), A_ref) < FACTOR_TOL
        assert rel_fro(G.cpu().numpy(), ko.factor_G(gout)) < FACTOR_TOL
        np.testing.assert_array_equal(A.cpu().numpy(), gpu_factor(kb.KFAC_OP_FACTOR_A, shp, act, kb.KFAC_NHWC,
                                                                  kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C))
        np.testing.assert_array_equal(G.cpu().numpy(), gpu_factor(kb.KFAC_OP_FACTOR_G, shp, gout, kb.KFAC_NHWC,
                                                                  kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C))


def test_factor_batched_many_builds_use_coarser_row_splits():
    """With 16 or more matrix-core builds in one call the library splits each build over fewer, longer row ranges
    than it does for a build on its own (fewer partial sums through HBM): same factors to rounding, not bit for bit.
    Shapes with enough rows for the two plans to differ: 12,800 and 9,248 unfolded rows."""
    shapes = [synth.LayerShape("b3x3", 8, 48, 40, 40, 72, 3, 3, 1, 1),
              synth.LayerShape("b1x1", 8, 136, 34, 34, 200, 1, 1, 1, 0)]
    builds, keep = [], []
    for rep in range(5):
        for i, shp in enumerate(shapes):
            desc = kb.make_desc(shp, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
            act = synth.round_to_bf16(synth.make_act(shp, 20 + 2 * rep + i))
            gout = synth.round_to_bf16(synth.make_gout(shp, 20 + 2 * rep + i))
            at = kb.to_device_tensor(act, kb.KFAC_NHWC, kb.KFAC_BF16, DEV)
            gt = kb.to_device_tensor(gout, kb.KFAC_NHWC, kb.KFAC_BF16, DEV)
            A = torch.full((shp.d_A, shp.d_A), float("nan"), device=DEV)
            G = torch.full((shp.d_G, shp.d_G), float("nan"), device=DEV)
            builds += [(kb.KFAC_OP_FACTOR_A, desc, at, A, 0.0), (kb.KFAC_OP_FACTOR_G, desc, gt, G, 0.0)]
            keep.append((shp, act, gout, A, G))
    assert len(builds) == 20
    kb.kfac_factor_batched(kb.FactorBatch(builds, device=DEV))
    torch.cuda.synchronize()
    for n, (shp, act, gout, A, G) in enumerate(keep):
        A, G = A.cpu().numpy(), G.cpu().numpy()
        np.testing.assert_array_equal(A, A.T)
        np.testing.assert_array_equal(G, G.T)
        if n < 4:      # the oracle on the first of each kind (and their repeats with other seeds against single calls)
            assert rel_fro(A, ko.factor_A(act, shp.kh, shp.kw, shp.stride, shp.pad, True, ko.ORDER_KH_KW_C)) < FACTOR_TOL
            assert rel_fro(G, ko.factor_G(gout)) < FACTOR_TOL
        A1 = gpu_factor(kb.KFAC_OP_FACTOR_A, shp, act, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
        G1 = gpu_factor(kb.KFAC_OP_FACTOR_G, shp, gout, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
        assert rel_fro(A, A1) < 1e-5 and rel_fro(G, G1) < 1e-5       # fp32 summation order only


def test_factor_scale_argument():
    shp = SMALL_SHAPES[0]
    act = synth.round_to_bf16(synth.make_act(shp, 2))
    A = gpu_factor(kb.KFAC_OP_FACTOR_A, shp, act, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C, scale=0.5)
    ref = ko.factor_A(act, 3, 3, 1, 1, True, ko.ORDER_KH_KW_C, scale=0.5)
    assert rel_fro(A, ref) < FACTOR_TOL


def test_factors_config1_full_size():
    """Stage-5 3x3 convolution at per-GPU batch 32: d_A = 4609 from 1568 rows, d_G = 512."""
    shp = synth.config1()
    A, G = check_factor_pair(shp, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
    assert A.shape == (4609, 4609) and G.shape == (512, 512)


def test_factors_config2_full_size():
    """First convolution at batch 32: 401,408 unfolded rows, d_A = 148, d_G = 64 (tall-skinny, split over rows)."""
    shp = synth.config2()
    A, G = check_factor_pair(shp, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
    assert A.shape == (148, 148) and G.shape == (64, 64)


def _fused_and_packed_case(shapes, dtype=None):
    dtype = kb.KFAC_BF16 if dtype is None else dtype
    layout = kb.KFAC_NHWC if dtype != kb.KFAC_F32 else kb.KFAC_NCHW
    rnd = _NP_ROUND[dtype]
    builds, refs = [], []
    for i, shp in enumerate(shapes):
        desc = kb.make_desc(shp, layout, dtype, kb.KFAC_ORDER_KH_KW_C)
        act, gout = rnd(synth.make_act(shp, 5, i)), rnd(synth.make_gout(shp, 5, i))
        builds.append((kb.KFAC_OP_FACTOR_A, desc, kb.to_device_tensor(act, layout, dtype, DEV), shp.d_A))
        refs.append(ko.factor_A(act, shp.kh, shp.kw, shp.stride, shp.pad, True, ko.ORDER_KH_KW_C))
        builds.append((kb.KFAC_OP_FACTOR_G, desc, kb.to_device_tensor(gout, layout, dtype, DEV), shp.d_G))
        refs.append(ko.factor_G(gout))
    return builds, refs


FUSED_SHAPES = [
    synth.LayerShape("f.3x3", 3, 40, 9, 9, 70, 3, 3, 1, 1),                 # several tiles, ragged edges, one row split
    synth.LayerShape("f.1x1long", 4, 64, 40, 40, 136, 1, 1, 1, 0),          # 6,400 rows: split over workgroups, reduced
    synth.LayerShape("f.conv1", 2, 3, 70, 70, 16, 7, 7, 2, 3, relu_input=False),   # 3 channels: the narrow-layer kernel
    synth.LayerShape("f.wide", 2, 160, 5, 5, 300, 3, 3, 1, 1),              # d_A = 1441: many whole tiles
]


def test_factor_batched_running_average_in_the_epilogue():
    """Builds that fold their result into the running average themselves (Sec. 3.4 saves the traffic of a stored fresh
    factor; the running average is this build's reading 5): S <- rho S + (1 - rho) X against the oracle, element-wise,
    and bit for bit against building X and calling kfac_ema."""
    decay = 0.95
    builds, refs = _fused_and_packed_case(FUSED_SHAPES)
    rng = np.random.default_rng(9)
    S0 = []
    for op, desc, x, d in builds:
        m = rng.standard_normal((d, d)).astype(np.float32)
        S0.append((m + m.T) * np.float32(0.5))
    run_fused = [torch.from_numpy(s).to(DEV) for s in S0]
    run_plain = [torch.from_numpy(s).to(DEV) for s in S0]
    fresh = [torch.full((d, d), float("nan"), dtype=torch.float32, device=DEV) for _, _, _, d in builds]
    items = [(op, desc, x, f, 0.0) for (op, desc, x, d), f in zip(builds, fresh)]
    kb.kfac_factor_batched(kb.FactorBatch(items, device=DEV, running=run_fused, decay=decay))
    kb.kfac_factor_batched(kb.FactorBatch(items, device=DEV))
    kb.kfac_ema_batched(kb.EmaBatch(run_plain, fresh), decay)
    torch.cuda.synchronize()
    for s0, ref, got, plain in zip(S0, refs, run_fused, run_plain):
        want = ko.ema(s0, ref, decay)
        g = got.cpu().numpy()
        assert rel_max(g, want) < 1e-6, rel_max(g, want)
        np.testing.assert_array_equal(g, g.T)
        np.testing.assert_array_equal(g, plain.cpu().numpy())


def test_factor_batched_packed_upper_triangle_output():
    """Builds that deliver the packed upper triangle (Sec. 3.4, symmetry-aware communication): against the oracle's
    packing of the oracle's factor, and bit for bit against packing the full build."""
    builds, refs = _fused_and_packed_case(FUSED_SHAPES)
    packed = [torch.full((kb.packed_elems(d),), float("nan"), dtype=torch.float32, device=DEV) for _, _, _, d in builds]
    full = [torch.empty((d, d), dtype=torch.float32, device=DEV) for _, _, _, d in builds]
    kb.kfac_factor_batched(kb.FactorBatch([(op, desc, x, p, 0.0) for (op, desc, x, d), p in zip(builds, packed)],
                                          device=DEV, packed=True))
    kb.kfac_factor_batched(kb.FactorBatch([(op, desc, x, f, 0.0) for (op, desc, x, d), f in zip(builds, full)], device=DEV))
    torch.cuda.synchronize()
    for ref, p, f in zip(refs, packed, full):
        got = p.cpu().numpy()
        want = ko.pack_upper(ref)
        assert np.isfinite(got).all()
        assert rel_fro(got, want) < FACTOR_TOL and rel_max(got, want) < FACTOR_TOL
        np.testing.assert_array_equal(got, ko.pack_upper(f.cpu().numpy()).astype(np.float32))


# ----------------------------------------------------------------------------------------------
# running average
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dim", [1, 7, 145, 512, 1025])
def test_ema(dim):
    rng = np.random.default_rng(dim)
    S = rng.standard_normal((dim, dim)).astype(np.float32)
    X = rng.standard_normal((dim, dim)).astype(np.float32)
    St, Xt = torch.from_numpy(S).to(DEV), torch.from_numpy(X).to(DEV)
    kb.kfac_ema(St, Xt, dim, 0.95)
    torch.cuda.synchronize()
    want = ko.ema(S, X, np.float32(0.95))
    np.testing.assert_allclose(St.cpu().numpy(), want, rtol=0, atol=2e-7 * np.abs(want).max())
    # from the identity, constant fresh factor: closed form after k steps
    St = torch.eye(dim, device=DEV)
    for _ in range(5):
        kb.kfac_ema(St, Xt, dim, 0.95)
    torch.cuda.synchronize()
    want = 0.95 ** 5 * np.eye(dim) + (1 - 0.95 ** 5) * X.astype(np.float64)
    np.testing.assert_allclose(St.cpu().numpy(), want, rtol=0, atol=1e-6 * np.abs(want).max())


@pytest.mark.gpu
def test_ema_batched_mixed_sizes():
    """One launch over many matrices: chunk boundaries (4096 elements), ragged tails, a 1 x 1 matrix, more
    matrices than one launch carries (128)."""
    dims = [1, 3, 64, 65, 127, 128, 577, 1025] + [5 + (i % 7) for i in range(130)]
    rng = np.random.default_rng(11)
    S = [rng.standard_normal((d, d)).astype(np.float32) for d in dims]
    X = [rng.standard_normal((d, d)).astype(np.float32) for d in dims]
    St = [torch.from_numpy(a).to(DEV) for a in S]
    Xt = [torch.from_numpy(a).to(DEV) for a in X]
    kb.kfac_ema_batched(kb.EmaBatch(St, Xt), 0.95)
    torch.cuda.synchronize()
    for s, x, st, xt in zip(S, X, St, Xt):
        want = ko.ema(s, x, np.float32(0.95))
        np.testing.assert_allclose(st.cpu().numpy(), want, rtol=0, atol=2e-7 * max(np.abs(want).max(), 1.0))
        np.testing.assert_array_equal(xt.cpu().numpy(), x)          # the fresh factor is only read
    kb.kfac_ema_batched(kb.EmaBatch([], []), 0.95)                   # empty batch: nothing to do


# ----------------------------------------------------------------------------------------------
# packed upper triangles and the running average fed from a packed factor
# ----------------------------------------------------------------------------------------------
PACK_DIMS = [1, 2, 63, 64, 65, 128, 130, 577, 1025] + [3 + (i % 5) for i in range(125)]     # > 128 matrices: two launches


def test_pack_upper_batched_bit_exact():
    rng = np.random.default_rng(21)
    full = [rng.standard_normal((d, d)).astype(np.float32) for d in PACK_DIMS]          # not symmetric on purpose:
    ft = [torch.from_numpy(a).to(DEV) for a in full]                                    # only the upper triangle is read
    pt = [torch.full((kb.packed_elems(d),), float("nan"), device=DEV) for d in PACK_DIMS]
    kb.kfac_pack_upper_batched(kb.PackBatch(ft, pt))
    torch.cuda.synchronize()
    for a, p, f in zip(full, pt, ft):
        np.testing.assert_array_equal(p.cpu().numpy(), ko.pack_upper(a).astype(np.float32))    # copies: bit exact
        np.testing.assert_array_equal(f.cpu().numpy(), a)                                      # source untouched
    kb.kfac_pack_upper_batched(kb.PackBatch([], []))                                           # empty batch


def test_ema_packed_batched():
    rng = np.random.default_rng(22)
    run, packed = [], []
    for d in PACK_DIMS:
        B = rng.standard_normal((d, d)).astype(np.float32)
        run.append((B + B.T).astype(np.float32))
        C = rng.standard_normal((d, d)).astype(np.float32)
        packed.append(ko.pack_upper(C + C.T).astype(np.float32))
    rt = [torch.from_numpy(a.copy()).to(DEV) for a in run]
    for r in rt:                                                     # poison the lower triangles: they must not be read
        r.copy_(torch.triu(r) + torch.tril(torch.full_like(r, 1e30), diagonal=-1))
    pk = [torch.from_numpy(a).to(DEV) for a in packed]
    kb.kfac_ema_packed_batched(kb.PackBatch(rt, pk), 0.95)
    torch.cuda.synchronize()
    for a, p, r in zip(run, packed, rt):
        want = ko.ema_packed(a, p, np.float32(0.95))
        got = r.cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=0, atol=2e-7 * max(np.abs(want).max(), 1.0))
        np.testing.assert_array_equal(got, got.T)                   # mirrored, not recomputed


def test_pack_then_ema_packed_equals_plain_ema():
    """pack on the sender, running average from the packed factor on the owner = running average of the full factor."""
    d = 300
    rng = np.random.default_rng(23)
    B = rng.standard_normal((d, d)).astype(np.float32)
    X = (B @ B.T / d).astype(np.float32)
    X = np.triu(X) + np.triu(X, 1).T
    Xt = torch.from_numpy(X).to(DEV)
    pk = torch.empty(kb.packed_elems(d), device=DEV)
    kb.kfac_pack_upper_batched(kb.PackBatch([Xt], [pk]))
    R1, R2 = torch.eye(d, device=DEV), torch.eye(d, device=DEV)
    kb.kfac_ema_packed_batched(kb.PackBatch([R1], [pk]), 0.95)
    kb.kfac_ema(R2, Xt, d, 0.95)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(R1.cpu().numpy(), R2.cpu().numpy())


# ----------------------------------------------------------------------------------------------
# change rate between two refreshes (staleness)
# ----------------------------------------------------------------------------------------------
def test_factor_diff_batched():
    dims = [1, 2, 90, 91, 128, 577, 1025] + [4 + (i % 6) for i in range(126)]        # chunk tails; two launches
    rng = np.random.default_rng(31)
    Xp = [rng.standard_normal((d, d)).astype(np.float32) for d in dims]
    X = [(a + 0.05 * rng.standard_normal(a.shape)).astype(np.float32) for a in Xp]
    X[3] = Xp[3].copy()                                                             # unchanged statistic: exactly 0
    X[4] = (2.0 * Xp[4]).astype(np.float32)                                         # doubled: exactly 1
    xt = [torch.from_numpy(a).to(DEV) for a in X]
    pt = [torch.from_numpy(a).to(DEV) for a in Xp]
    batch = kb.DiffBatch(xt, pt, device=DEV)
    got = kb.kfac_factor_diff_batched(batch).cpu().numpy()
    torch.cuda.synchronize()
    want = np.array([ko.factor_diff(a, b) if a.size <= 8192 else np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b.astype(np.float64))
                     for a, b in zip(X, Xp)])
    # the big matrices use the library norm (the oracle's element loop takes minutes there); cross-check the two once
    assert ko.factor_diff(X[2], Xp[2]) == pytest.approx(np.linalg.norm(X[2].astype(np.float64) - Xp[2]) / np.linalg.norm(Xp[2].astype(np.float64)), rel=1e-12)
    np.testing.assert_allclose(got, want, rtol=2e-6, atol=0)
    assert got[3] == 0.0 and got[4] == pytest.approx(1.0, rel=1e-6)
    again = kb.kfac_factor_diff_batched(batch).cpu().numpy()
    np.testing.assert_array_equal(got, again)                                       # deterministic


# ----------------------------------------------------------------------------------------------
# optimizer tail: weight update with momentum, then rescaling
# ----------------------------------------------------------------------------------------------
def test_weight_update_batched():
    shapes = [(1, 1), (16, 145), (64, 148), (64, 577), (130, 129), (1000, 2049)] + [(3 + i % 4, 5 + i % 7) for i in range(125)]
    rng = np.random.default_rng(41)
    W = [rng.standard_normal(sh).astype(np.float32) for sh in shapes]
    Wp = [(w + 0.01 * rng.standard_normal(w.shape)).astype(np.float32) for w in W]
    P = [rng.standard_normal(sh).astype(np.float32) for sh in shapes]
    wt, wpt, pt = ([torch.from_numpy(a.copy()).to(DEV) for a in L] for L in (W, Wp, P))
    eta, mom = 0.02, 0.9 * 0.02 / 8.18e-3
    kb.kfac_weight_update_batched(kb.UpdateBatch(wt, wpt, pt, device=DEV), eta, mom)
    torch.cuda.synchronize()
    for w, wp, p, a, b, c in zip(W, Wp, P, wt, wpt, pt):
        want = ko.rescale_weights(ko.weight_update(w, wp, p, np.float32(eta), np.float32(mom)), w.shape[0])
        got = a.cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=0, atol=3e-6 * np.abs(want).max())
        assert np.linalg.norm(got.astype(np.float64)) == pytest.approx(np.sqrt(2.0 * w.shape[0]), rel=1e-5)
        np.testing.assert_array_equal(b.cpu().numpy(), w)            # w_prev <- old w, bit for bit
        np.testing.assert_array_equal(c.cpu().numpy(), p)            # the preconditioned gradient is only read
    kb.kfac_weight_update_batched(kb.UpdateBatch([], [], [], device=DEV), eta, mom)


# ----------------------------------------------------------------------------------------------
# Batch Normalization layers: per-sample gradients, diagonal and full Fisher matrix
# ----------------------------------------------------------------------------------------------
def _bn_inputs(N, C, H, W, dtype, seed):
    rng = np.random.default_rng([seed, N, C, H, W])
    rnd = _NP_ROUND[dtype]
    xhat = rnd(rng.standard_normal((N, C, H, W)))                   # a normalised activation: N(0, 1)
    gout = rnd(synth.SIGMA_GOUT * rng.standard_normal((N, C, H, W)))
    td = kb._TORCH_DTYPE[dtype]
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 3, 1))).to(DEV).to(td).contiguous()
    return xhat, gout, to_dev(xhat), to_dev(gout)


@pytest.mark.parametrize("N,C,H,W,dtype", [
    (4, 64, 23, 24, kb.KFAC_BF16),        # 552 positions: two chunks, 32 position lanes
    (3, 192, 9, 9, kb.KFAC_F16),          # 24 vectors per position: idle threads
    (2, 2048, 7, 7, kb.KFAC_BF16),        # widest ResNet-50 BN layer
    (2, 2056, 3, 3, kb.KFAC_BF16),        # more than 256 vectors per position, ragged
    (3, 5, 6, 7, kb.KFAC_BF16),           # channels not a multiple of 8: general kernel
    (2, 16, 5, 5, kb.KFAC_F32),
])
def test_bn_sample_grads(N, C, H, W, dtype):
    xhat, gout, xt, gt = _bn_inputs(N, C, H, W, dtype, 51)
    g = kb.kfac_bn_sample_grads(xt, gt, dtype)
    torch.cuda.synchronize()
    want = ko.bn_sample_grads(xhat, gout)
    assert g.shape == (N, 2 * C)
    np.testing.assert_allclose(g.cpu().numpy(), want, rtol=0, atol=2e-6 * np.abs(want).max())


def test_bn_sample_grads_batched_mixed_layers():
    cases = [(4, 64, 23, 24, kb.KFAC_BF16), (2, 2048, 7, 7, kb.KFAC_BF16), (3, 192, 9, 9, kb.KFAC_F16), (3, 5, 6, 7, kb.KFAC_BF16),
             (2, 16, 33, 32, kb.KFAC_F32), (5, 256, 14, 14, kb.KFAC_BF16), (2, 1032, 2, 3, kb.KFAC_F16)]
    ins = [_bn_inputs(*c, 54 + i) for i, c in enumerate(cases)]
    batch = kb.BnBatch([t[2] for t in ins], [t[3] for t in ins], [c[4] for c in cases], DEV)
    for rep in range(2):                                             # the scratch is reused: a second call gives the same
        gs = kb.kfac_bn_sample_grads_batched(batch)
        torch.cuda.synchronize()
        for (xhat, gout, _, _), g in zip(ins, gs):
            want = ko.bn_sample_grads(xhat, gout)
            np.testing.assert_allclose(g.cpu().numpy(), want, rtol=0, atol=2e-6 * np.abs(want).max())


def test_bn_diag_and_full_fisher_preconditioning():
    N, C, H, W = 32, 64, 14, 14
    xhat, gout, xt, gt = _bn_inputs(N, C, H, W, kb.KFAC_BF16, 52)
    g = kb.kfac_bn_sample_grads(xt, gt, kb.KFAC_BF16)
    rng = np.random.default_rng(53)
    grad = rng.standard_normal(2 * C).astype(np.float32)
    gradt = torch.from_numpy(grad).to(DEV)
    damping = 10.0 * 1e-3                                            # rho_BN * gamma
    fd, out = torch.empty(2 * C, device=DEV), torch.empty(2 * C, device=DEV)
    kb.kfac_bn_diag_precondition(g, gradt, damping, fd, out)
    torch.cuda.synchronize()
    g64 = g.cpu().numpy().astype(np.float64)                         # each stage against the oracle on the GPU stage's input
    np.testing.assert_allclose(fd.cpu().numpy(), ko.bn_fisher_diag(g64), rtol=2e-6)
    np.testing.assert_allclose(out.cpu().numpy(), ko.bn_precondition_diag(ko.bn_fisher_diag(g64), grad, np.float32(damping)), rtol=1e-5)
    # full 2C x 2C Fisher matrix through the generic entry points: factor of the (N x 2C) gradient matrix, damped
    # inverse, product with the gradient as a 1 x 2C matrix
    shp = synth.LayerShape("bn.full", N, 1, 1, 1, 2 * C, 1, 1, 1, 0)
    desc = kb.make_desc(shp, kb.KFAC_NHWC, kb.KFAC_F32, kb.KFAC_ORDER_KH_KW_C)
    F = torch.empty((2 * C, 2 * C), device=DEV)
    kb.kfac_factor_G(desc, g, 0.0, F, kb.alloc_workspace(kb.kfac_factor_workspace_bytes(kb.KFAC_OP_FACTOR_G, desc), DEV))
    Finv = torch.empty_like(F)
    info = torch.zeros(1, dtype=torch.int32, device=DEV)
    kb.kfac_damped_inverse(F, 2 * C, damping, Finv, info, kb.alloc_workspace(kb.kfac_inverse_workspace_bytes(2 * C)))
    one = torch.ones((1, 1), device=DEV)
    P = torch.empty((1, 2 * C), device=DEV)
    kb.kfac_precondition(one, Finv, gradt.view(1, -1), 1, 2 * C, P, kb.alloc_workspace(kb.kfac_precondition_workspace_bytes(1, 2 * C)))
    torch.cuda.synchronize()
    assert int(info) == 0
    assert rel_fro(F.cpu().numpy(), ko.bn_fisher(g64)) < FACTOR_TOL
    want = ko.bn_precondition_full(F.cpu().numpy().astype(np.float64), grad, float(np.float32(damping)))
    assert rel_fro(P.cpu().numpy().ravel(), want) < PRE_TOL
    np.testing.assert_allclose(np.diag(F.cpu().numpy()), fd.cpu().numpy(), rtol=1e-5)      # the diagonal form is its diagonal


# ----------------------------------------------------------------------------------------------
# damped inverse
# ----------------------------------------------------------------------------------------------
def gpu_inverse(S, damping):
    dim = S.shape[0]
    St = torch.from_numpy(S).to(DEV)
    out = torch.full((dim, dim), float("nan"), dtype=torch.float32, device=DEV)
    info = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    ws = kb.alloc_workspace(kb.kfac_inverse_workspace_bytes(dim), DEV)
    kb.kfac_damped_inverse(St, dim, damping, out, info, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), int(info.item())


# (block counts 1 .. 13: every length of a matrix's last group of steps, after one, two and three full groups; ragged and
# full last blocks)
@pytest.mark.parametrize("dim", [1, 2, 16, 64, 65, 128, 129, 148, 256, 257, 300, 384, 512, 513, 640, 700, 769, 897, 1153,
                                 1290, 1500, 1601])
def test_damped_inverse_random_spd(dim):
    S = synth.random_spd(dim, seed=3, eig_lo=1e-3, eig_hi=10.0, n_zero=dim // 3)
    lam = float(np.float32(np.sqrt(1e-3)))
    Minv, info = gpu_inverse(S, lam)
    assert info == 0
    ref = ko.damped_inverse(S, lam)
    assert rel_fro(Minv, ref) < INV_TOL, rel_fro(Minv, ref)
    assert rel_max(Minv, ref) < INV_TOL, rel_max(Minv, ref)
    np.testing.assert_array_equal(Minv, Minv.T)
    M = S.astype(np.float64) + lam * np.eye(dim)
    assert np.linalg.norm(M @ Minv - np.eye(dim)) / np.sqrt(dim) < 1e-3


@pytest.mark.parametrize("scale", [1e-6, 1e-3, 1e3, 1e6])
def test_damped_inverse_magnitudes(scale):
    """Factors far from unit magnitude (the update's fp16 operand pieces rely on per-slab power-of-two scales): the
    inverse of c (S + lambda I) is (1/c) times the inverse of S + lambda I, to the same relative accuracy."""
    dim = 641
    S = (synth.random_spd(dim, seed=11, eig_lo=1e-2, eig_hi=5.0) * scale).astype(np.float32)
    lam = np.float32(0.05 * scale)
    Minv, info = gpu_inverse(S, lam)
    assert info == 0
    ref = ko.damped_inverse(S, lam)
    assert np.isfinite(Minv).all()
    assert rel_fro(Minv, ref) < INV_TOL, rel_fro(Minv, ref)


def test_damped_inverse_reads_lower_triangle_only():
    S = synth.random_spd(200, seed=4)
    junk = S.copy()
    junk[np.triu_indices(200, 1)] = 1e9
    a, ia = gpu_inverse(S, 0.05)
    b, ib = gpu_inverse(junk, 0.05)
    assert ia == 0 and ib == 0
    np.testing.assert_array_equal(a, b)


def test_damped_inverse_diagonal_and_identity():
    d = np.diag(np.arange(1, 201, dtype=np.float32))
    Minv, info = gpu_inverse(d, 0.5)
    assert info == 0
    np.testing.assert_allclose(Minv, np.diag(1 / (np.arange(1, 201) + 0.5)), rtol=0, atol=1e-7)


@pytest.mark.parametrize("dim", [40, 300, 700, 1100])
def test_damped_inverse_reports_not_positive_definite(dim):
    S = np.eye(dim, dtype=np.float32)
    S[dim // 2, dim // 2] = -2.0
    _, info = gpu_inverse(S, 0.1)
    assert info == dim // 2 + 1          # first leading minor that fails
    _, info = gpu_inverse(np.eye(dim, dtype=np.float32), -3.0)
    assert info == 1


def test_damped_inverse_config1_full_size():
    """The 4609-dim stage-5 factor without running average: the worst-conditioned case (kappa ~ 1.7e4)."""
    shp = synth.config1()
    act = synth.round_to_bf16(synth.make_act(shp, 0))
    S = gpu_factor(kb.KFAC_OP_FACTOR_A, shp, act, kb.KFAC_NHWC, kb.KFAC_BF16, kb.KFAC_ORDER_KH_KW_C)
    lam = float(np.float32(np.sqrt(1e-3)))
    Minv, info = gpu_inverse(S, lam)
    assert info == 0
    ref = ko.damped_inverse(S, lam)
    err = rel_fro(Minv, ref)
    print(f"config1 inverse rel. Frobenius error {err:.3e}, largest entry-wise error / largest entry {rel_max(Minv, ref):.3e}")
    assert err < INV_TOL
    assert rel_max(Minv, ref) < INV_TOL
    np.testing.assert_array_equal(Minv, Minv.T)


def test_damped_inverse_batched_mixed_sizes():
    dims = [64, 513, 128, 300, 65, 148, 1, 257]
    Ss = [synth.random_spd(d, seed=10 + i, n_zero=d // 4) for i, d in enumerate(dims)]
    lams = [0.03 + 0.01 * i for i in range(len(dims))]
    St = [torch.from_numpy(s).to(DEV) for s in Ss]
    Mt = [torch.full((d, d), float("nan"), dtype=torch.float32, device=DEV) for d in dims]
    batch = kb.InverseBatch(St, Mt, lams, device=DEV)
    kb.kfac_damped_inverse_batched(batch)
    torch.cuda.synchronize()
    assert batch.info.cpu().tolist() == [0] * len(dims)
    for S, lam, M in zip(Ss, lams, Mt):
        got = M.cpu().numpy()
        assert rel_fro(got, ko.damped_inverse(S, np.float32(lam))) < INV_TOL
        assert rel_max(got, ko.damped_inverse(S, np.float32(lam))) < INV_TOL
        np.testing.assert_array_equal(got, got.T)
    # same answer as one-at-a-time calls, bit for bit
    for S, lam, M in zip(Ss, lams, Mt):
        single, _ = gpu_inverse(S, lam)
        np.testing.assert_array_equal(single, M.cpu().numpy())


def test_damped_inverse_batched_more_matrices_than_one_launch_group():
    """150 small matrices of mixed size in one call: more than one launch's argument block describes (64 for the kernels
    that read the input, 112 for the sweep's per-step launches), so the call deals them into groups and sub-batches;
    every one against the oracle, and bit for bit against the single call."""
    dims = [1 + (37 * i) % 300 for i in range(146)] + [385, 257, 129, 128]
    Ss = [synth.random_spd(d, seed=100 + i, n_zero=d // 5) for i, d in enumerate(dims)]
    lams = [0.02 + 0.001 * i for i in range(len(dims))]
    St = [torch.from_numpy(s).to(DEV) for s in Ss]
    Mt = [torch.full((d, d), float("nan"), dtype=torch.float32, device=DEV) for d in dims]
    batch = kb.InverseBatch(St, Mt, lams, device=DEV)
    assert batch.count == 150
    kb.kfac_damped_inverse_batched(batch)
    torch.cuda.synchronize()
    assert batch.info.cpu().tolist() == [0] * len(dims)
    for i, (S, lam, M) in enumerate(zip(Ss, lams, Mt)):
        got = M.cpu().numpy()
        ref = ko.damped_inverse(S, np.float32(lam))
        assert rel_fro(got, ref) < INV_TOL, (i, dims[i])
        assert rel_max(got, ref) < INV_TOL, (i, dims[i])
        np.testing.assert_array_equal(got, got.T)
        if i % 7 == 0:
            single, _ = gpu_inverse(S, lam)
            np.testing.assert_array_equal(single, got)


def test_pi_damping_split_and_device_side_damping():
    """Trace-ratio split of the damping on the device (Sec. 4.2), and inversions that read their damping from there."""
    dims = [(145, 16), (577, 64), (64, 300), (1, 1)]
    rng = np.random.default_rng(31)
    As = [synth.random_spd(a, seed=40 + i) * np.float32(10.0 ** (i - 1)) for i, (a, g) in enumerate(dims)]
    Gs = [synth.random_spd(g, seed=50 + i) * np.float32(0.01) for i, (a, g) in enumerate(dims)]
    At = [torch.from_numpy(x).to(DEV) for x in As]
    Gt = [torch.from_numpy(x).to(DEV) for x in Gs]
    gamma = 1e-3
    pi = kb.PiBatch(At, Gt, device=DEV)
    lam = kb.kfac_pi_damping_batched(pi, gamma)
    torch.cuda.synchronize()
    lam = lam.cpu().numpy()
    for i in range(len(dims)):
        la, lg = ko.factor_damping_pi(As[i], Gs[i], gamma)
        assert lam[2 * i] == pytest.approx(la, rel=2e-6) and lam[2 * i + 1] == pytest.approx(lg, rel=2e-6)
    # the inversions read lambda from the device array (the host value, deliberately wrong, must be ignored)
    S = At + Gt
    Mt = [torch.full_like(x, float("nan")) for x in S]
    addr = [pi.address(i, 0) for i in range(len(dims))] + [pi.address(i, 1) for i in range(len(dims))]
    batch = kb.InverseBatch(S, Mt, [123.0] * len(S), device=DEV, dampings_dev=addr)
    kb.kfac_damped_inverse_batched(batch)
    torch.cuda.synchronize()
    assert batch.info.cpu().tolist() == [0] * len(S)
    lams = [lam[2 * i] for i in range(len(dims))] + [lam[2 * i + 1] for i in range(len(dims))]
    for x, l, m in zip(As + Gs, lams, Mt):
        ref = ko.damped_inverse(x, float(l))
        assert rel_fro(m.cpu().numpy(), ref) < INV_TOL and rel_max(m.cpu().numpy(), ref) < INV_TOL


# ----------------------------------------------------------------------------------------------
# preconditioning
# ----------------------------------------------------------------------------------------------
def gpu_precondition(Ginv, Ainv, gradW):
    dG, dA = gradW.shape
    out = torch.full((dG, dA), float("nan"), dtype=torch.float32, device=DEV)
    ws = kb.alloc_workspace(kb.kfac_precondition_workspace_bytes(dG, dA), DEV)
    kb.kfac_precondition(torch.from_numpy(Ginv).to(DEV), torch.from_numpy(Ainv).to(DEV),
                         torch.from_numpy(gradW).to(DEV), dG, dA, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("dG,dA", [(1, 1), (16, 145), (64, 148), (130, 129), (200, 577), (512, 1153), (1000, 2049)])
def test_precondition(dG, dA):
    rng = np.random.default_rng([dG, dA])
    Ginv = ko.damped_inverse(synth.random_spd(dG, 5), 0.03).astype(np.float32)
    Ainv = ko.damped_inverse(synth.random_spd(dA, 6), 0.03).astype(np.float32)
    gradW = (rng.standard_normal((dG, dA)) * synth.SIGMA_GRADW).astype(np.float32)
    P = gpu_precondition(Ginv, Ainv, gradW)
    ref = ko.precondition(Ginv, gradW, Ainv)
    assert rel_fro(P, ref) < PRE_TOL, rel_fro(P, ref)
    assert rel_max(P, ref) < PRE_TOL, rel_max(P, ref)


def test_precondition_batched_matches_single_calls():
    shapes = [(64, 65), (256, 577), (130, 129), (512, 1153), (16, 145)]
    rng = np.random.default_rng(12)
    Gi = [ko.damped_inverse(synth.random_spd(g, 20 + i), 0.05).astype(np.float32) for i, (g, a) in enumerate(shapes)]
    Ai = [ko.damped_inverse(synth.random_spd(a, 30 + i), 0.05).astype(np.float32) for i, (g, a) in enumerate(shapes)]
    Ws = [(rng.standard_normal(s) * synth.SIGMA_GRADW).astype(np.float32) for s in shapes]
    dev = lambda xs: [torch.from_numpy(x).to(DEV) for x in xs]
    Gt, At, Wt = dev(Gi), dev(Ai), dev(Ws)
    Pt = [torch.full(s, float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
    batch = kb.PrecondBatch(Gt, At, Wt, Pt, device=DEV)
    kb.kfac_precondition_batched(batch)
    torch.cuda.synchronize()
    for g, a, w, p in zip(Gi, Ai, Ws, Pt):
        assert rel_fro(p.cpu().numpy(), ko.precondition(g, w, a)) < PRE_TOL
        np.testing.assert_array_equal(p.cpu().numpy(), gpu_precondition(g, a, w))


def test_precondition_from_the_planes_the_inversion_wrote():
    """kfac_inverse_item.planes -> kfac_precond_item.Ginv_planes / Ainv_planes: the inverse delivered a second time as fp16
    piece planes, and the preconditioning products multiplying from them, against the oracle and against the same call
    splitting the fp32 inverses itself.  Sizes: one block, a multiple of the block, ragged, a last block of one row
    (Eq. 6, Eq. 7)."""
    shapes = [(64, 65), (256, 577), (130, 129), (128, 1153), (512, 1025), (1, 384)]
    lam = 0.03
    rng = np.random.default_rng(21)
    Sg = [synth.random_spd(g, 40 + i).astype(np.float32) for i, (g, a) in enumerate(shapes)]
    Sa = [synth.random_spd(a, 60 + i).astype(np.float32) for i, (g, a) in enumerate(shapes)]
    Ws = [(rng.standard_normal(s) * synth.SIGMA_GRADW).astype(np.float32) for s in shapes]
    dev = lambda xs: [torch.from_numpy(x).to(DEV) for x in xs]
    S = dev(Sg) + dev(Sa)
    Minv = [torch.full_like(x, float("nan")) for x in S]
    planes = [kb.alloc_workspace(kb.kfac_inverse_planes_bytes(x.shape[0]), DEV) for x in S]
    for pl in planes:
        pl.fill_(0x7f)                                    # (fp16 0x7f7f is a huge number: nothing may be left unwritten)
    inv = kb.InverseBatch(S, Minv, [lam] * len(S), device=DEV, planes=planes)
    kb.kfac_damped_inverse_batched(inv)
    torch.cuda.synchronize()
    assert int(inv.info.abs().max()) == 0
    n = len(shapes)
    Gt, At, Wt = Minv[:n], Minv[n:], dev(Ws)
    P_planes = [torch.full(s, float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
    P_self = [torch.full(s, float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
    kb.kfac_precondition_batched(kb.PrecondBatch(Gt, At, Wt, P_planes, device=DEV, Ginv_planes=planes[:n],
                                                 Ainv_planes=planes[n:]))
    kb.kfac_precondition_batched(kb.PrecondBatch(Gt, At, Wt, P_self, device=DEV))
    P_mixed = [torch.full(s, float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
    kb.kfac_precondition_batched(kb.PrecondBatch(Gt, At, Wt, P_mixed, device=DEV, Ainv_planes=planes[n:]))   # G split by the call
    torch.cuda.synchronize()
    for i, (g, a) in enumerate(shapes):
        assert rel_fro(P_mixed[i].cpu().numpy(), P_planes[i].cpu().numpy()) < 1e-5, shapes[i]
        gi, ai = Gt[i].cpu().numpy().astype(np.float64), At[i].cpu().numpy().astype(np.float64)
        assert rel_fro(gi, ko.damped_inverse(Sg[i], lam)) < INV_TOL
        ref = ko.precondition(gi, Ws[i], ai)
        got = P_planes[i].cpu().numpy()
        assert np.isfinite(got).all(), shapes[i]
        assert rel_fro(got, ref) < 1e-5 and rel_max(got, ref) < 1e-5, (shapes[i], rel_fro(got, ref), rel_max(got, ref))
        assert rel_fro(got, P_self[i].cpu().numpy()) < 1e-5, shapes[i]


def test_precondition_operand_roles():
    """Non-symmetric stand-ins for the inverses would expose a swapped or transposed operand; the ABI takes
    symmetric ones, so use distinct symmetric matrices and a rectangular gradient."""
    rng = np.random.default_rng(7)
    Gi = rng.standard_normal((70, 70)); Gi = (Gi + Gi.T).astype(np.float32)
    Ai = rng.standard_normal((150, 150)); Ai = (Ai + Ai.T).astype(np.float32)
    W = rng.standard_normal((70, 150)).astype(np.float32)
    assert rel_fro(gpu_precondition(Gi, Ai, W), ko.precondition(Gi, W, Ai)) < 1e-5


# ----------------------------------------------------------------------------------------------
# whole layer step
# ----------------------------------------------------------------------------------------------
def test_layer_step_config0_end_to_end():
    shp = synth.config0()
    order = kb.KFAC_ORDER_C_KH_KW
    act, gout, gradW = synth.make_act(shp), synth.make_gout(shp), synth.make_gradw(shp)
    ref = ko.kfac_layer_step(act, gout, gradW, np.eye(shp.d_A), np.eye(shp.d_G), kh=3, kw=3, stride=1, pad=1,
                             decay=0.95, gamma=1e-3)
    desc = kb.make_desc(shp, kb.KFAC_NCHW, kb.KFAC_F32, order)
    dA, dG = shp.d_A, shp.d_G
    A_new = torch.empty((dA, dA), device=DEV)
    G_new = torch.empty((dG, dG), device=DEV)
    wsA = kb.alloc_workspace(kb.kfac_factor_workspace_bytes(kb.KFAC_OP_FACTOR_A, desc), DEV)
    wsG = kb.alloc_workspace(kb.kfac_factor_workspace_bytes(kb.KFAC_OP_FACTOR_G, desc), DEV)
    kb.kfac_factor_A(desc, kb.to_device_tensor(act, kb.KFAC_NCHW, kb.KFAC_F32), 0.0, A_new, wsA)
    kb.kfac_factor_G(desc, kb.to_device_tensor(gout, kb.KFAC_NCHW, kb.KFAC_F32), 0.0, G_new, wsG)
    A_run, G_run = torch.eye(dA, device=DEV), torch.eye(dG, device=DEV)
    kb.kfac_ema(A_run, A_new, dA, 0.95)
    kb.kfac_ema(G_run, G_new, dG, 0.95)
    lam = float(np.sqrt(np.float32(1e-3)))
    A_inv, G_inv = torch.empty_like(A_run), torch.empty_like(G_run)
    info = torch.zeros(2, dtype=torch.int32, device=DEV)
    kb.kfac_damped_inverse(A_run, dA, lam, A_inv, info[0:1], kb.alloc_workspace(kb.kfac_inverse_workspace_bytes(dA)))
    kb.kfac_damped_inverse(G_run, dG, lam, G_inv, info[1:2], kb.alloc_workspace(kb.kfac_inverse_workspace_bytes(dG)))
    P = torch.empty((dG, dA), device=DEV)
    kb.kfac_precondition(G_inv, A_inv, torch.from_numpy(gradW).to(DEV), dG, dA, P,
                         kb.alloc_workspace(kb.kfac_precondition_workspace_bytes(dG, dA)))
    torch.cuda.synchronize()
    assert info.cpu().tolist() == [0, 0]
    assert rel_fro(A_new.cpu().numpy(), ref["A_new"]) < FACTOR_TOL
    assert rel_fro(G_new.cpu().numpy(), ref["G_new"]) < FACTOR_TOL
    assert rel_fro(A_run.cpu().numpy(), ref["A_run"]) < FACTOR_TOL
    assert rel_fro(A_inv.cpu().numpy(), ref["A_inv"]) < INV_TOL
    assert rel_fro(G_inv.cpu().numpy(), ref["G_inv"]) < INV_TOL
    assert rel_fro(P.cpu().numpy(), ref["P"]) < PRE_TOL


# ----------------------------------------------------------------------------------------------
# whole-network step (the object bench.py times), with a stale-inverse schedule
# ----------------------------------------------------------------------------------------------
NET_LAYERS = [
    synth.LayerShape("n.conv1", 4, 3, 70, 70, 16, 7, 7, 2, 3, relu_input=False),    # narrow-layer kernel, 4,900 rows
    synth.LayerShape("n.3x3", 4, 16, 14, 14, 24, 3, 3, 1, 1),
    synth.LayerShape("n.1x1", 4, 24, 14, 14, 40, 1, 1, 1, 0),
    synth.LayerShape("n.3x3s2", 4, 40, 14, 14, 48, 3, 3, 2, 1),                     # d_A = 361: three 128-blocks
    synth.LayerShape("n.1x1wide", 4, 48, 7, 7, 136, 1, 1, 1, 0),                    # d_G = 136: two blocks
    synth.LayerShape("n.fc", 4, 200, 1, 1, 10, 1, 1, 1, 0),
]
# End to end the fp32 inverse inherits the fp32 rounding of the factors it is given, amplified by at most the
# condition number of the damped factor (here <= (trace + lambda) / lambda ~ 2e3 on errors ~1e-6 measured
# stage-wise): 2e-3 bounds the preconditioned gradient against the all-float64 chain.  Stage by stage, each against
# the oracle fed the GPU stage's own input, the bars are the usual ones.
END_TO_END_TOL = 2e-3


@pytest.mark.parametrize("long_dim", [2048, 140])
def test_network_step_with_trace_ratio_damping(long_dim):
    """One step of the small network with the damping split by the trace ratio of each layer's factors (computed on the
    device between the running averages and the inversions), in both schedules."""
    from paper_1811_12019_amd import step as kstep
    gamma = 1e-3
    net = kstep.KfacNetworkStep(NET_LAYERS, dtype=kb.KFAC_BF16, order=kb.KFAC_ORDER_KH_KW_C, decay=0.95, gamma=gamma,
                                seed=5, device=DEV, inverse_streams=2, long_dim=long_dim, pi_split=True)
    net.step()
    torch.cuda.synchronize()
    assert int(net.inverse_info().abs().max()) == 0
    f64 = lambda t: t.detach().cpu().numpy().astype(np.float64)
    for l in net.layers:
        la, lg = ko.factor_damping_pi(f64(l.A_run), f64(l.G_run), gamma)
        assert rel_fro(f64(l.A_inv), ko.damped_inverse(f64(l.A_run), float(np.float32(la)))) < INV_TOL, l.shape.name
        assert rel_fro(f64(l.G_inv), ko.damped_inverse(f64(l.G_run), float(np.float32(lg)))) < INV_TOL, l.shape.name
        assert rel_fro(f64(l.P), ko.precondition(f64(l.G_inv), f64(l.gradW), f64(l.A_inv))) < PRE_TOL


@pytest.mark.parametrize("long_dim", [2048, 140])
def test_network_step_with_stale_inverses(long_dim):
    """KfacNetworkStep (batched entry points only) over three steps, inverses refreshed on steps 0 and 2 only:
    every stage of every layer against the oracle, stale inverses untouched on step 1.  long_dim = 140 makes two
    waves (the four layers with a factor of 145 to 361, the two others); the first is inverted on side streams beside
    the second's stages: the schedule the benchmark times.  The default threshold leaves this small
    network in one wave, stage after stage."""
    from paper_1811_12019_amd import step as kstep
    decay, gamma = 0.95, 1e-3
    lam = ko.factor_damping(gamma)
    net = kstep.KfacNetworkStep(NET_LAYERS, dtype=kb.KFAC_BF16, order=kb.KFAC_ORDER_KH_KW_C, decay=decay, gamma=gamma,
                                seed=3, device=DEV, inverse_streams=2, long_dim=long_dim, fused_ema=False)
    assert len(net.waves) == (2 if long_dim == 140 else 0)
    f64 = lambda t: t.detach().cpu().numpy().astype(np.float64)
    nchw = lambda t: t.float().permute(0, 3, 1, 2).cpu().numpy().astype(np.float64)
    chain = [dict(A_run=np.eye(l.shape.d_A), G_run=np.eye(l.shape.d_G)) for l in net.layers]     # all-float64 chain
    prev_run = [(f64(l.A_run), f64(l.G_run)) for l in net.layers]
    prev_inv = None
    for step_no, refresh in enumerate([True, False, True]):
        for l in net.layers:
            l.gradW.mul_(1.5)                                         # a different gradient every step
        net.step(refresh_inverse=refresh)
        torch.cuda.synchronize()
        assert int(net.inverse_info().abs().max()) == 0
        for i, l in enumerate(net.layers):
            s = l.shape
            A_new = ko.factor_A(nchw(l.act), s.kh, s.kw, s.stride, s.pad, True, ko.ORDER_KH_KW_C)
            G_new = ko.factor_G(nchw(l.gout))
            assert rel_fro(f64(l.A_new), A_new) < FACTOR_TOL, (step_no, s.name)
            assert rel_fro(f64(l.G_new), G_new) < FACTOR_TOL, (step_no, s.name)
            # running average from the GPU's own previous value and fresh factor
            assert rel_fro(f64(l.A_run), ko.ema(prev_run[i][0], f64(l.A_new), decay)) < 1e-6
            assert rel_fro(f64(l.G_run), ko.ema(prev_run[i][1], f64(l.G_new), decay)) < 1e-6
            if refresh:
                assert rel_fro(f64(l.A_inv), ko.damped_inverse(f64(l.A_run), float(np.float32(lam)))) < INV_TOL
                assert rel_fro(f64(l.G_inv), ko.damped_inverse(f64(l.G_run), float(np.float32(lam)))) < INV_TOL
            else:
                np.testing.assert_array_equal(f64(l.A_inv), prev_inv[i][0])
                np.testing.assert_array_equal(f64(l.G_inv), prev_inv[i][1])
            assert rel_fro(f64(l.P), ko.precondition(f64(l.G_inv), f64(l.gradW), f64(l.A_inv))) < PRE_TOL
            # the all-float64 chain
            c = chain[i]
            c["A_run"], c["G_run"] = ko.ema(c["A_run"], A_new, decay), ko.ema(c["G_run"], G_new, decay)
            if refresh:
                c["A_inv"], c["G_inv"] = ko.damped_inverse(c["A_run"], lam), ko.damped_inverse(c["G_run"], lam)
            assert rel_fro(f64(l.P), ko.precondition(c["G_inv"], f64(l.gradW), c["A_inv"])) < END_TO_END_TOL
        prev_run = [(f64(l.A_run), f64(l.G_run)) for l in net.layers]
        prev_inv = [(f64(l.A_inv), f64(l.G_inv)) for l in net.layers]
