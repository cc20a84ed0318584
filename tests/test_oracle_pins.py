"""Pins for the float64 oracle: each oracle function is checked against something other than itself.

Brute-force loops, torch's own unfold / autograd, closed forms, an explicitly formed Kronecker
product, and the storage totals the paper prints.  All CPU, all small.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import kfac_oracle as ko
from paper_1811_12019_amd import synth


# ----------------------------------------------------------------------------------------------
# unfold
# ----------------------------------------------------------------------------------------------
def brute_unfold(act, kh, kw, stride, pad, order):
    """Seven nested loops straight from the definition of a zero-padded convolution's input patch."""
    N, C, H, W = act.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    X = np.zeros((N * Ho * Wo, C * kh * kw))
    for n in range(N):
        for yo in range(Ho):
            for xo in range(Wo):
                r = (n * Ho + yo) * Wo + xo
                for c in range(C):
                    for i in range(kh):
                        for j in range(kw):
                            y, x = yo * stride + i - pad, xo * stride + j - pad
                            v = act[n, c, y, x] if (0 <= y < H and 0 <= x < W) else 0.0
                            col = (c * kh + i) * kw + j if order == ko.ORDER_C_KH_KW else (i * kw + j) * C + c
                            X[r, col] = v
    return X


UNFOLD_CASES = [
    # N, C, H, W, kh, kw, stride, pad
    (2, 3, 5, 5, 3, 3, 1, 1),
    (2, 3, 9, 9, 7, 7, 2, 3),     # the first-convolution geometry, shrunk
    (1, 2, 6, 7, 2, 3, 1, 0),     # non-square kernel and image
    (2, 4, 6, 6, 1, 1, 2, 0),     # strided 1x1 projection shortcut
    (1, 2, 5, 5, 3, 3, 2, 1),
]


@pytest.mark.parametrize("case", UNFOLD_CASES)
@pytest.mark.parametrize("order", [ko.ORDER_C_KH_KW, ko.ORDER_KH_KW_C])
def test_unfold_matches_bruteforce(case, order):
    N, C, H, W, kh, kw, s, p = case
    act = np.random.default_rng(1).standard_normal((N, C, H, W))
    np.testing.assert_array_equal(ko.unfold(act, kh, kw, s, p, order), brute_unfold(act, kh, kw, s, p, order))


@pytest.mark.parametrize("case", UNFOLD_CASES)
def test_unfold_matches_torch_unfold(case):
    N, C, H, W, kh, kw, s, p = case
    act = np.random.default_rng(2).standard_normal((N, C, H, W))
    t = torch.nn.functional.unfold(torch.from_numpy(act), (kh, kw), padding=p, stride=s)   # N, C*kh*kw, L
    want = t.permute(0, 2, 1).reshape(-1, C * kh * kw).numpy()
    np.testing.assert_array_equal(ko.unfold(act, kh, kw, s, p, ko.ORDER_C_KH_KW), want)


def test_unfold_1x1_is_a_reshape():
    act = np.random.default_rng(3).standard_normal((3, 5, 4, 4))
    want = act.transpose(0, 2, 3, 1).reshape(-1, 5)
    for order in (ko.ORDER_C_KH_KW, ko.ORDER_KH_KW_C):
        np.testing.assert_array_equal(ko.unfold(act, 1, 1, 1, 0, order), want)


def test_orders_are_a_column_permutation():
    C, kh, kw = 3, 2, 3
    act = np.random.default_rng(4).standard_normal((2, C, 5, 6))
    Xc = ko.unfold(act, kh, kw, 1, 1, ko.ORDER_C_KH_KW)
    Xk = ko.unfold(act, kh, kw, 1, 1, ko.ORDER_KH_KW_C)
    perm = [(c * kh + i) * kw + j for i in range(kh) for j in range(kw) for c in range(C)]
    np.testing.assert_array_equal(Xk, Xc[:, perm])


# ----------------------------------------------------------------------------------------------
# unfolded rows vs the convolution they belong to (pins column order, padding, stride, bias column)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", UNFOLD_CASES)
def test_unfold_reproduces_conv_forward_and_weight_gradient(case):
    N, C, H, W, kh, kw, s, p = case
    Co = 4
    rng = np.random.default_rng(5)
    act = torch.from_numpy(rng.standard_normal((N, C, H, W)))
    w = torch.from_numpy(rng.standard_normal((Co, C, kh, kw))).requires_grad_()
    b = torch.from_numpy(rng.standard_normal(Co)).requires_grad_()
    out = torch.nn.functional.conv2d(act, w, b, stride=s, padding=p)
    gout = torch.from_numpy(rng.standard_normal(tuple(out.shape)))
    (out * gout).sum().backward()

    X = ko.unfold(act.numpy(), kh, kw, s, p, ko.ORDER_C_KH_KW)
    Xbar = np.concatenate([X, np.ones((X.shape[0], 1))], axis=1)
    Wbar = np.concatenate([w.detach().numpy().reshape(Co, -1), b.detach().numpy()[:, None]], axis=1)
    Gamma = gout.numpy().transpose(0, 2, 3, 1).reshape(-1, Co)
    # forward: out[(n,y,x), o] = Xbar . Wbar^T
    np.testing.assert_allclose(Xbar @ Wbar.T, out.detach().numpy().transpose(0, 2, 3, 1).reshape(-1, Co), atol=1e-12)
    # backward: dL/dWbar = Gamma^T Xbar, in weight.reshape(C_out, -1) order, bias gradient last
    want = np.concatenate([w.grad.numpy().reshape(Co, -1), b.grad.numpy()[:, None]], axis=1)
    np.testing.assert_allclose(Gamma.T @ Xbar, want, atol=1e-11)
    # and the same cross moment is what factor_A / factor_G are the second moments of
    R = X.shape[0]
    A = ko.factor_A(act.numpy(), kh, kw, s, p, True, ko.ORDER_C_KH_KW)
    G = ko.factor_G(gout.numpy())
    np.testing.assert_allclose(A, Xbar.T @ Xbar / R, atol=1e-12)
    np.testing.assert_allclose(G, Gamma.T @ Gamma / R, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# factor A
# ----------------------------------------------------------------------------------------------
def coverage_count(H, W, kh, kw, stride, pad):
    """m[y, x] = number of (output position, kernel tap) pairs that read input pixel (y, x)."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    m = np.zeros((H, W))
    for yo, xo, i, j in itertools.product(range(Ho), range(Wo), range(kh), range(kw)):
        y, x = yo * stride + i - pad, xo * stride + j - pad
        if 0 <= y < H and 0 <= x < W:
            m[y, x] += 1
    return m


@pytest.mark.parametrize("case", UNFOLD_CASES)
@pytest.mark.parametrize("order", [ko.ORDER_C_KH_KW, ko.ORDER_KH_KW_C])
def test_factor_A_invariants(case, order):
    N, C, H, W, kh, kw, s, p = case
    act = np.maximum(np.random.default_rng(6).standard_normal((N, C, H, W)), 0)
    A = ko.factor_A(act, kh, kw, s, p, True, order)
    d = C * kh * kw + 1
    assert A.shape == (d, d)
    np.testing.assert_allclose(A, A.T, atol=1e-14)
    assert np.linalg.eigvalsh(A).min() >= -1e-12 * np.trace(A)
    assert A[-1, -1] == pytest.approx(1.0, abs=1e-14)
    X = brute_unfold(act, kh, kw, s, p, order)
    np.testing.assert_allclose(A[:-1, -1], X.mean(axis=0), atol=1e-13)     # bias column = column means
    # trace without unfolding: every pixel contributes its square once per patch that reads it
    R = X.shape[0]
    m = coverage_count(H, W, kh, kw, s, p)
    assert np.trace(A) == pytest.approx(1.0 + (act ** 2 * m).sum() / R, rel=1e-12)
    # mean squared norm of the rows of [X | 1]
    assert np.trace(A) == pytest.approx(((X ** 2).sum(axis=1) + 1).mean(), rel=1e-12)


def test_factor_A_without_bias_and_scale():
    act = np.random.default_rng(7).standard_normal((2, 3, 5, 5))
    X = brute_unfold(act, 3, 3, 1, 1, ko.ORDER_C_KH_KW)
    np.testing.assert_allclose(ko.factor_A(act, 3, 3, 1, 1, False), X.T @ X / X.shape[0], atol=1e-13)
    np.testing.assert_allclose(ko.factor_A(act, 3, 3, 1, 1, False, scale=1.0), X.T @ X, atol=1e-12)


def test_factor_A_fc_is_second_moment():
    a = np.random.default_rng(8).standard_normal((50, 7))
    A = ko.factor_A(a.reshape(50, 7, 1, 1), 1, 1, 1, 0, True)
    mu = a.mean(axis=0)
    want = np.cov(a, rowvar=False, bias=True) + np.outer(mu, mu)
    np.testing.assert_allclose(A[:-1, :-1], want, atol=1e-13)
    np.testing.assert_allclose(A[-1, :-1], mu, atol=1e-14)


def test_factor_A_config0_expected_trace():
    """ReLU'd N(0,1) input, 8x8, 3x3 pad 1: E[trace A] = 1 + C * 1/2 * (sum of coverage)/(H*W) = 61.5."""
    shp = synth.config0()
    m = coverage_count(8, 8, 3, 3, 1, 1)
    expected = 1 + shp.C_in * 0.5 * m.sum() / 64
    assert expected == pytest.approx(61.5)
    act = synth.make_act(shp, seed=0)
    A = ko.factor_A(act, 3, 3, 1, 1, True)
    assert A.shape == (145, 145)
    assert np.trace(A) == pytest.approx(61.5, rel=0.08)          # ~2.5 % sampling s.d.
    # interior off-diagonal entries between different channels: E = E[relu]^2 * coverage = cov/(2 pi)
    centre = 4            # tap (1, 1)
    vals = [A[c * 9 + centre, c2 * 9 + centre] for c in range(16) for c2 in range(c)]
    assert np.mean(vals) == pytest.approx(1 / (2 * np.pi), rel=0.08)


# ----------------------------------------------------------------------------------------------
# factor G
# ----------------------------------------------------------------------------------------------
def test_factor_G_invariants_and_bruteforce():
    rng = np.random.default_rng(9)
    gout = rng.standard_normal((3, 4, 5, 6)) * 0.1
    G = ko.factor_G(gout)
    want = np.zeros((4, 4))
    for n, y, x in itertools.product(range(3), range(5), range(6)):
        g = gout[n, :, y, x]
        want += np.outer(g, g)
    want /= 3 * 5 * 6
    np.testing.assert_allclose(G, want, atol=1e-15)
    np.testing.assert_allclose(G, G.T, atol=1e-16)
    assert np.linalg.eigvalsh(G).min() >= -1e-14
    assert np.trace(G) == pytest.approx((gout ** 2).sum() / 90, rel=1e-12)
    np.testing.assert_allclose(ko.factor_G(gout, scale=1.0), want * 90, atol=1e-13)


def test_factor_G_expected_value():
    shp = synth.config0()
    G = ko.factor_G(synth.make_gout(shp, seed=0))
    assert G.shape == (16, 16)
    assert np.trace(G) / 16 == pytest.approx(1e-2, rel=0.05)
    assert np.abs(G - np.diag(np.diag(G))).max() < 3e-3          # off-diagonals ~ sigma^2 / sqrt(R) = 4.4e-4


# ----------------------------------------------------------------------------------------------
# running average, damping, inverse
# ----------------------------------------------------------------------------------------------
def test_ema_closed_form():
    rng = np.random.default_rng(10)
    X = rng.standard_normal((6, 6))
    S = np.eye(6)
    np.testing.assert_allclose(ko.ema(S, X, 0.95), 0.95 * np.eye(6) + 0.05 * X, atol=1e-16)
    for k in range(1, 8):
        S = ko.ema(S, X, 0.95)
        np.testing.assert_allclose(S, 0.95 ** k * np.eye(6) + (1 - 0.95 ** k) * X, atol=1e-14)
    np.testing.assert_array_equal(ko.ema(np.eye(6), X, 1.0), np.eye(6))
    np.testing.assert_array_equal(ko.ema(np.eye(6), X, 0.0), X)


def test_damping_split():
    lam = ko.factor_damping(1e-3)
    assert lam == pytest.approx(0.0316227766, rel=1e-9)
    assert lam * lam == pytest.approx(1e-3, rel=1e-14)


def test_damped_inverse_pins():
    S = synth.random_spd(60, seed=1, n_zero=20).astype(np.float64)
    lam = 0.03
    Minv = ko.damped_inverse(S, lam)
    M = S + lam * np.eye(60)
    assert np.linalg.norm(M @ Minv - np.eye(60)) / np.sqrt(60) < 1e-10
    assert np.linalg.norm(Minv @ M - np.eye(60)) / np.sqrt(60) < 1e-10
    # eigenvalues of the inverse are 1 / (eig + lam); the null space of S maps to exactly 1/lam
    w = np.linalg.eigvalsh(S)
    np.testing.assert_allclose(np.sort(np.linalg.eigvalsh(Minv)), np.sort(1 / (w + lam)), rtol=1e-9)
    # independent route: Cholesky solve
    import scipy.linalg
    want = scipy.linalg.cho_solve(scipy.linalg.cho_factor(M), np.eye(60))
    np.testing.assert_allclose(Minv, want, rtol=0, atol=1e-9 * np.abs(want).max())
    # diagonal closed form
    d = np.arange(1.0, 6.0)
    np.testing.assert_allclose(ko.damped_inverse(np.diag(d), 0.5), np.diag(1 / (d + 0.5)), atol=1e-15)
    # zero damping on a 2x2 with a hand-computed inverse
    np.testing.assert_allclose(ko.damped_inverse(np.array([[2.0, 1.0], [1.0, 1.0]]), 0.0),
                               np.array([[1.0, -1.0], [-1.0, 2.0]]), atol=1e-15)


# ----------------------------------------------------------------------------------------------
# preconditioning: the Kronecker identity with an explicitly formed Kronecker product
# ----------------------------------------------------------------------------------------------
def test_precondition_explicit_kronecker_full_config0():
    shp = synth.config0()
    act, gout, gradW = synth.make_act(shp), synth.make_gout(shp), synth.make_gradw(shp)
    out = ko.kfac_layer_step(act, gout, gradW, np.eye(shp.d_A), np.eye(shp.d_G),
                             kh=3, kw=3, stride=1, pad=1, decay=0.95, gamma=1e-3)
    lam = np.sqrt(1e-3)
    # rebuild the damped factors by hand from the closed-form running average
    X = brute_unfold(act.astype(np.float64), 3, 3, 1, 1, ko.ORDER_C_KH_KW)
    Xb = np.concatenate([X, np.ones((X.shape[0], 1))], axis=1)
    A_d = 0.95 * np.eye(145) + 0.05 * (Xb.T @ Xb) / 512 + lam * np.eye(145)
    Gm = gout.astype(np.float64).transpose(0, 2, 3, 1).reshape(-1, 16)
    G_d = 0.95 * np.eye(16) + 0.05 * (Gm.T @ Gm) / 512 + lam * np.eye(16)
    # F = G (x) A acts on the row-major vec of the d_G x d_A gradient (Eq. 5-7)
    F = np.kron(G_d, A_d)                                     # 2320 x 2320
    assert F.shape == (2320, 2320)
    want = np.linalg.solve(F, gradW.astype(np.float64).reshape(-1)).reshape(16, 145)
    np.testing.assert_allclose(out["P"], want, rtol=0, atol=1e-10 * np.abs(want).max())
    # column-major vec convention: (A (x) G)^-1 vec(gradW) = vec(G^-1 gradW A^-1)
    F2 = np.kron(A_d, G_d)
    want2 = np.linalg.solve(F2, gradW.astype(np.float64).reshape(-1, order="F")).reshape(16, 145, order="F")
    np.testing.assert_allclose(out["P"], want2, rtol=0, atol=1e-10 * np.abs(want2).max())


def test_precondition_small_cases():
    rng = np.random.default_rng(11)
    W = rng.standard_normal((3, 5))
    np.testing.assert_array_equal(ko.precondition(np.eye(3), W, np.eye(5)), W)
    # non-symmetric stand-ins expose a transposed or swapped operand
    Gi, Ai = rng.standard_normal((3, 3)), rng.standard_normal((5, 5))
    want = np.zeros((3, 5))
    for i, j, k, l in itertools.product(range(3), range(5), range(3), range(5)):
        want[i, j] += Gi[i, k] * W[k, l] * Ai[l, j]
    np.testing.assert_allclose(ko.precondition(Gi, W, Ai), want, atol=1e-13)
    # identity factors and damping lam on both: gradient shrinks by 1/(1+lam)^2
    lam = 0.1
    P = ko.precondition(ko.damped_inverse(np.eye(3), lam), W, ko.damped_inverse(np.eye(5), lam))
    np.testing.assert_allclose(P, W / (1 + lam) ** 2, atol=1e-14)


def test_layer_step_without_running_average():
    shp = synth.LayerShape("t", 2, 3, 5, 5, 4, 3, 3, 2, 1)
    act, gout, gradW = synth.make_act(shp, 3), synth.make_gout(shp, 3), synth.make_gradw(shp, 3)
    out = ko.kfac_layer_step(act, gout, gradW, None, None, kh=3, kw=3, stride=2, pad=1, decay=None, gamma=1e-2)
    lam = 0.1
    F = np.kron(out["G_new"] + lam * np.eye(4), out["A_new"] + lam * np.eye(28))
    want = np.linalg.solve(F, gradW.astype(np.float64).reshape(-1)).reshape(4, 28)
    np.testing.assert_allclose(out["P"], want, rtol=0, atol=1e-10 * np.abs(want).max())


# ----------------------------------------------------------------------------------------------
# the ResNet-50 layer table against the totals the paper prints
# ----------------------------------------------------------------------------------------------
MiB = 2.0 ** 20


def test_resnet50_layer_table_matches_paper_totals(paper_values):
    layers = synth.resnet50_layers(32)
    bn = synth.resnet50_bn_channels()
    assert len(layers) == 54 and len(bn) == 53
    assert len(layers) + len(bn) == paper_values["layers_total"]
    assert layers[0].N == paper_values["images_per_gpu"]
    kron = ko.factor_bytes(layers, 4)
    assert round(kron / MiB) == paper_values["fim_memory_diag_bn"]                 # 587 MiB
    full_bn = sum((2 * c) ** 2 * 4 for c in bn)
    assert round((kron + full_bn) / MiB) == pytest.approx(paper_values["fim_memory_full_bn"], abs=1)   # 1017 MiB
    tri = sum(ko.packed_triangle_elems(l.d_A) + ko.packed_triangle_elems(l.d_G) for l in layers) * 4
    grads = sum(l.d_A * l.d_G for l in layers) * 4
    assert round((tri + grads) / MiB) == paper_values["packed_message"]             # 391 MiB
    assert round(100 * (1 - (tri + grads) / (kron + grads))) == paper_values["packed_reduction"]   # 43 %


def test_resnet50_layer_table_shapes():
    layers = synth.resnet50_layers(32)
    by_name = {l.name: l for l in layers}
    c1 = by_name["conv1"]
    assert (c1.d_A, c1.d_G, c1.R) == (148, 64, 401408)
    s5 = by_name["layer4.1.conv2"]
    assert (s5.d_A, s5.d_G, s5.R) == (4609, 512, 1568)
    assert s5 == synth.config1().__class__(**{**synth.config1().__dict__, "name": s5.name})
    fc = by_name["fc"]
    assert (fc.d_A, fc.d_G, fc.R) == (2049, 1000, 32)
    dims = sorted([l.d_A for l in layers] + [l.d_G for l in layers])
    assert dims[0] == 64 and dims[-1] == 4609 and dims.count(4609) == 3 and dims.count(2305) == 6
    # spatial sizes chain: each layer's input size equals some earlier output size
    assert by_name["layer2.0.conv2"].H_out == 28 and by_name["layer4.0.downsample"].H_out == 7
    assert packed_ok()


def packed_ok():
    return ko.packed_triangle_elems(4) == 10 and ko.packed_triangle_elems(1) == 1


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -3.14159, 1e-30, 65504.0], dtype=np.float32)
    got = synth.round_to_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got, want)
    assert synth.bf16_bits(got).dtype == np.uint16


# ---------------------------------------------------------------------------------------------------
# packed upper triangles (Sec. 3.4, symmetry-aware communication)
# ---------------------------------------------------------------------------------------------------
def test_pack_upper_matches_library_triangle_indexing_and_counts():
    rng = np.random.default_rng(5)
    for n in (1, 2, 5, 33):
        B = rng.standard_normal((n, n))
        S = B + B.T
        p = ko.pack_upper(S)
        assert p.shape == (ko.packed_triangle_elems(n),) == (n * (n + 1) // 2,)
        np.testing.assert_array_equal(p, S[np.triu_indices(n)])            # numpy's own row-major upper-triangle order
        np.testing.assert_array_equal(ko.unpack_upper(p, n), S)             # round trip rebuilds both triangles
    # hand-written 3 x 3: rows (1 2 3), (. 4 5), (. . 6)
    S3 = np.array([[1., 2., 3.], [2., 4., 5.], [3., 5., 6.]])
    np.testing.assert_array_equal(ko.pack_upper(S3), [1., 2., 3., 4., 5., 6.])
    np.testing.assert_array_equal(ko.unpack_upper([1., 2., 3., 4., 5., 6.], 3), S3)


def test_pack_upper_reads_only_the_upper_triangle():
    S = np.array([[1., 2.], [99., 4.]])                                     # lower entry must not leak into the result
    np.testing.assert_array_equal(ko.pack_upper(S), [1., 2., 4.])


def test_ema_packed_equals_ema_of_the_full_matrix():
    rng = np.random.default_rng(6)
    n = 7
    B = rng.standard_normal((n, n)); X = B @ B.T
    R = np.eye(n)
    np.testing.assert_allclose(ko.ema_packed(R, X[np.triu_indices(n)], 0.95), 0.95 * R + 0.05 * X, rtol=0, atol=1e-15)


# ---------------------------------------------------------------------------------------------------
# staleness: change rate and refresh intervals (Sec. 5.4)
# ---------------------------------------------------------------------------------------------------
def test_factor_diff_closed_forms():
    rng = np.random.default_rng(8)
    P = rng.standard_normal((6, 6))
    assert ko.factor_diff(P, P) == 0.0
    assert ko.factor_diff(2.0 * P, P) == pytest.approx(1.0, rel=1e-14)             # ||P|| / ||P||
    assert ko.factor_diff(0.0 * P, P) == pytest.approx(1.0, rel=1e-14)
    assert ko.factor_diff(3.0 * P, 3.0 * 0.5 * P) == pytest.approx(1.0, rel=1e-14)  # scale invariant
    # 3-4-5: X_prev = (3, 0), X = (3, 4): ||X - X_prev|| = 4, ||X_prev|| = 3
    assert ko.factor_diff(np.array([[3.0, 4.0]]), np.array([[3.0, 0.0]])) == pytest.approx(4.0 / 3.0, rel=1e-15)
    # library norm as an independent routine; not symmetric in its arguments (the OLD value normalises)
    Q = rng.standard_normal((6, 6))
    assert ko.factor_diff(Q, P) == pytest.approx(np.linalg.norm(Q - P) / np.linalg.norm(P), rel=1e-13)
    assert ko.factor_diff(Q, P) != pytest.approx(ko.factor_diff(P, Q), rel=1e-3)


def test_refresh_intervals_worked_values():
    # min(20, 5 floor(e/5) + 1): 1 for epochs 0-4, 6 for 5-9, 11 for 10-14, 16 for 15-19, capped at 20 from epoch 20 on
    assert [ko.refresh_interval(e) for e in (0, 4, 5, 9, 10, 14, 15, 19, 20, 44)] == [1, 1, 6, 6, 11, 11, 16, 16, 20, 20]
    assert [ko.refresh_interval_late(e) for e in (0, 12, 13, 44)] == [1, 1, 20, 20]


# ---------------------------------------------------------------------------------------------------
# optimizer tail: learning rate, momentum, update, rescaling (Sec. 4.3, 4.4)
# ---------------------------------------------------------------------------------------------------
def test_learning_rate_and_momentum_schedule_values():
    # end points and a linear / quadratic midpoint, worked by hand: eta0 = 8, start 1, end 5
    assert ko.learning_rate(1, 8.0, 1, 5, 2.0) == 8.0
    assert ko.learning_rate(5, 8.0, 1, 5, 2.0) == 0.0
    assert ko.learning_rate(3, 8.0, 1, 5, 1.0) == pytest.approx(4.0)          # half way, p = 1
    assert ko.learning_rate(3, 8.0, 1, 5, 2.0) == pytest.approx(2.0)          # half way, p = 2: 8 * 0.25
    assert ko.learning_rate(4, 8.0, 1, 5, 3.0) == pytest.approx(8.0 / 64)     # (1/4)^3
    assert ko.learning_rate(0, 8.0, 1, 5, 2.0) == 8.0
    # momentum keeps its ratio to the learning rate
    for e in (1.0, 2.5, 4.0):
        eta = ko.learning_rate(e, 8.0, 1, 5, 2.0)
        assert ko.momentum_rate(eta, 8.0, 0.9) / eta == pytest.approx(0.9 / 8.0)
    assert ko.momentum_rate(8.0, 8.0, 0.9) == pytest.approx(0.9)


def test_weight_update_special_cases():
    rng = np.random.default_rng(9)
    w, wp, g = rng.standard_normal((3, 5)), rng.standard_normal((3, 5)), rng.standard_normal((3, 5))
    np.testing.assert_allclose(ko.weight_update(w, wp, g, 0.1, 0.0), w - 0.1 * g)                 # no momentum: plain step
    np.testing.assert_allclose(ko.weight_update(w, wp, 0 * g, 0.1, 0.5), w + 0.5 * (w - wp))      # no gradient: coasting
    np.testing.assert_allclose(ko.weight_update(w, w, g, 0.1, 0.9), w - 0.1 * g)                  # no previous motion
    # scalar case by hand: w = 2, w_prev = 1, G = 4, eta = 0.5, m = 0.25 -> 2 - 2 + 0.25 = 0.25
    assert ko.weight_update([2.0], [1.0], [4.0], 0.5, 0.25)[0] == pytest.approx(0.25)


def test_rescale_weights_norm_and_direction():
    rng = np.random.default_rng(10)
    w = rng.standard_normal((64, 577))
    r = ko.rescale_weights(w, 64)
    assert np.linalg.norm(r) == pytest.approx(np.sqrt(128.0), rel=1e-9)                          # sqrt(2 d_out)
    np.testing.assert_allclose(r / np.linalg.norm(r), w / np.linalg.norm(w), atol=1e-15)         # direction kept
    np.testing.assert_allclose(ko.rescale_weights(7.0 * w, 64), r, rtol=1e-9)                    # scale of w is forgotten
    assert np.all(ko.rescale_weights(np.zeros((2, 2)), 2) == 0.0)                                # eps keeps 0 / 0 away
    # 3-4-5 by hand: ||(3, 4)|| = 5, d_out = 2 -> sqrt(4) * (3, 4) / 5
    np.testing.assert_allclose(ko.rescale_weights([3.0, 4.0], 2), [1.2, 1.6], rtol=1e-9)


# ---------------------------------------------------------------------------------------------------
# Batch Normalization layers: per-sample gradients, full / diagonal Fisher matrix (Sec. 5.4)
# ---------------------------------------------------------------------------------------------------
def test_bn_sample_grads_match_autograd_per_sample():
    torch.manual_seed(0)
    N, C, H, W = 3, 4, 5, 2
    xhat = torch.randn(N, C, H, W, dtype=torch.float64)
    gout = torch.randn(N, C, H, W, dtype=torch.float64)
    got = ko.bn_sample_grads(xhat.numpy(), gout.numpy())
    assert got.shape == (N, 2 * C)
    for n in range(N):
        scale = torch.ones(C, dtype=torch.float64, requires_grad=True)
        shift = torch.zeros(C, dtype=torch.float64, requires_grad=True)
        y = scale.view(1, C, 1, 1) * xhat[n:n + 1] + shift.view(1, C, 1, 1)
        (y * gout[n:n + 1]).sum().backward()                      # dL/dy = gout
        np.testing.assert_allclose(got[n, :C], scale.grad.numpy(), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(got[n, C:], shift.grad.numpy(), rtol=1e-13, atol=1e-13)


def test_bn_fisher_brute_force_and_diagonal():
    rng = np.random.default_rng(12)
    g = rng.standard_normal((5, 6))
    F = np.zeros((6, 6))
    for n in range(5):
        for i in range(6):
            for j in range(6):
                F[i, j] += g[n, i] * g[n, j] / 5
    np.testing.assert_allclose(ko.bn_fisher(g), F, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(ko.bn_fisher_diag(g), np.diag(F), rtol=1e-14)
    # ResNet-50: full BN blocks (2C)^2 floats add up to the paper's 1017 - 587 MiB
    total = sum((2 * c) ** 2 * 4 for c in synth.resnet50_bn_channels())
    assert total / 2 ** 20 == pytest.approx(1017 - 587, abs=1.0)


def test_bn_precondition_diag_and_full():
    rng = np.random.default_rng(13)
    g = rng.standard_normal((40, 8))
    F, grad = ko.bn_fisher(g), rng.standard_normal(8)
    full = ko.bn_precondition_full(F, grad, 0.1)
    np.testing.assert_allclose((F + 0.1 * np.eye(8)) @ full, grad, rtol=1e-12, atol=1e-13)
    # a diagonal Fisher matrix: both forms agree; by hand: diag (1, 3), grad (2, 2), damping 1 -> (1, 0.5)
    np.testing.assert_allclose(ko.bn_precondition_diag([1.0, 3.0], [2.0, 2.0], 1.0), [1.0, 0.5])
    np.testing.assert_allclose(ko.bn_precondition_full(np.diag([1.0, 3.0]), [2.0, 2.0], 1.0), [1.0, 0.5])


# ---------------------------------------------------------------------------------------------------
# damping: trace-ratio split between the factors, warm-up schedule (Sec. 4.2)
# ---------------------------------------------------------------------------------------------------
def test_pi_corrected_damping_split():
    # by hand: mean eigenvalue of A = 4, of G = 1 -> pi = 2 -> (2 sqrt(gamma), sqrt(gamma) / 2)
    A, G = np.diag([4.0, 4.0]), np.diag([1.0, 1.0, 1.0])
    assert ko.pi_correction(A, G) == pytest.approx(2.0)
    la, lg = ko.factor_damping_pi(A, G, 1e-2)
    assert la == pytest.approx(0.2) and lg == pytest.approx(0.05)
    # equal scales: the even split of factor_damping
    la, lg = ko.factor_damping_pi(np.eye(5), np.eye(3), 1e-3)
    assert la == pytest.approx(ko.factor_damping(1e-3)) and lg == pytest.approx(ko.factor_damping(1e-3))
    # general factors: the two shifts multiply to gamma, and the two cross terms of
    # (A + la I) (x) (G + lg I) - A (x) G - gamma I, namely lg (A (x) I) and la (I (x) G), have equal traces per dimension
    rng = np.random.default_rng(21)
    X, Y = rng.standard_normal((30, 7)), 0.1 * rng.standard_normal((30, 4))
    A, G = X.T @ X / 30, Y.T @ Y / 30
    la, lg = ko.factor_damping_pi(A, G, 3e-4)
    assert la * lg == pytest.approx(3e-4, rel=1e-12)
    full = np.kron(A + la * np.eye(7), G + lg * np.eye(4)) - np.kron(A, G) - 3e-4 * np.eye(28)
    np.testing.assert_allclose(full, lg * np.kron(A, np.eye(4)) + la * np.kron(np.eye(7), G), atol=1e-15)
    assert np.trace(lg * np.kron(A, np.eye(4))) == pytest.approx(np.trace(la * np.kron(np.eye(7), G)), rel=1e-12)
    # scaling A by c^2 scales pi by c
    assert ko.pi_correction(9.0 * A, G) == pytest.approx(3.0 * ko.pi_correction(A, G), rel=1e-12)


def test_warmup_damping_schedule(paper_values):
    g0, gt = paper_values["warmup_gamma0_bs4096"], paper_values["warmup_gamma_target_bs4096"]
    tw = paper_values["warmup_steps_bs4096"]
    alpha = ko.warmup_damping_alpha(g0, gt, tw)
    assert alpha == pytest.approx(4.0 / 313.0, rel=1e-12)            # log10(100) = 2, by hand
    assert ko.warmup_damping_alpha(2.0e-2, 2.0e-4, paper_values["warmup_steps_bs32768"]) == pytest.approx(4.0 / 59.0)
    # one step by hand: 0.025 (1 - 4/313) + 0.00025 (4/313)
    assert ko.warmup_damping_next(g0, gt, alpha) == pytest.approx(0.025 - 0.02475 * 4.0 / 313.0, rel=1e-12)
    # closed form of the recurrence: gamma(t) - gamma_target = (1 - alpha)^t (gamma(0) - gamma_target)
    g = g0
    for t in range(1, 401):
        g = ko.warmup_damping_next(g, gt, alpha)
        assert g == pytest.approx(gt + (1.0 - alpha) ** t * (g0 - gt), rel=1e-10)
        assert gt < g < g0                                           # decreasing towards the target, never below it
    assert ko.warmup_damping_next(gt, gt, alpha) == pytest.approx(gt)    # the target is the fixed point
    assert ko.bn_damping(2.5e-4, paper_values["warmup_rho_bn_bs4096"]) == pytest.approx(4.0e-3)
