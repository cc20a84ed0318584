"""Float64 CPU oracle for one K-FAC step of one layer.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP library is checked against.  It is plain numpy in float64,
written directly from the definitions, with no blocking, fusion or reordering, and it shares no
code with the GPU path.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product never does.

What the path computes (every output is a unique real matrix, so the oracle is the definition
itself, not an iteration):

  * Kronecker factors of a layer's Fisher block, F ~ G (x) A (Sec. 3.2 "K-FAC", Eq. 5): A is the
    mini-batch mean (Sec. 3.1, E[.] = mean over the mini-batch samples) of a a^T over the layer's
    input vectors a, G the mean of g g^T over the gradients g of the loss w.r.t. the layer's
    output.  For a convolution the "samples" are the unfolded input patches, one per image and
    output position (the paper defers the conv case to Grosse & Martens 2016); a constant 1 is
    appended to a when the layer has a bias.
  * running average S <- rho S + (1 - rho) X of a factor (not in the paper; the usual K-FAC
    convention, rho multiplies the old value);
  * damping, Sec. 4.2 "Warmup damping" (its first equation): a multiple of the identity is
    added before inverting.  For the Kronecker-factored block the damping gamma is split as
    sqrt(gamma) on each factor;
  * inverse of each damped factor, Eq. 6: (G (x) A)^-1 = G^-1 (x) A^-1;
  * preconditioned gradient, Eq. 7: (G^-1 (x) A^-1) grad  ==  G^-1 . gradW . A^-1 for the weight
    gradient gradW stored as a d_G x d_A matrix (rows = output channels).

Parity pins (tests/test_oracle_pins.py) check every function against something other than
itself: a brute-force loop unfold, torch's own unfold and autograd weight gradient, closed forms
(trace identity, constant-input EMA, diagonal inverse), an explicitly formed Kronecker product, and
the factor-memory totals the paper prints (Sec. 5.4, Fig. 4).  No function here is unpinned.
"""
from __future__ import annotations

import numpy as np

ORDER_C_KH_KW = 0   # column (c, i, j) -> c*kh*kw + i*kw + j : matches weight.reshape(C_out, -1)
ORDER_KH_KW_C = 1   # column (i, j, c) -> (i*kw + j)*C + c   : matches a channels-last weight


def out_size(H: int, k: int, stride: int, pad: int) -> int:
    return (H + 2 * pad - k) // stride + 1


def unfold(act, kh: int, kw: int, stride: int, pad: int, order: int = ORDER_C_KH_KW) -> np.ndarray:
    """Explicit patch matrix X (R x C*kh*kw) of a zero-padded input act[n, c, y, x].

    Row r = (n*H_o + yo)*W_o + xo holds the patch read by output position (yo, xo) of image n:
    entry (c, i, j) is act[n, c, yo*stride + i - pad, xo*stride + j - pad], 0 outside the image.
    """
    act = np.asarray(act, dtype=np.float64)
    N, C, H, W = act.shape
    Ho, Wo = out_size(H, kh, stride, pad), out_size(W, kw, stride, pad)
    padded = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    padded[:, :, pad:pad + H, pad:pad + W] = act
    X = np.empty((N, Ho, Wo, C, kh, kw), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            window = padded[:, :, i:i + (Ho - 1) * stride + 1:stride, j:j + (Wo - 1) * stride + 1:stride]
            X[:, :, :, :, i, j] = window.transpose(0, 2, 3, 1)
    if order == ORDER_C_KH_KW:
        return X.reshape(N * Ho * Wo, C * kh * kw)
    if order == ORDER_KH_KW_C:
        return X.transpose(0, 1, 2, 4, 5, 3).reshape(N * Ho * Wo, kh * kw * C)
    raise ValueError("unknown column order")


def factor_A(act, kh: int, kw: int, stride: int, pad: int, has_bias: bool = True,
             order: int = ORDER_C_KH_KW, scale: float | None = None) -> np.ndarray:
    """A = scale * Xbar^T Xbar, Xbar = [unfold(act) | 1]; scale defaults to 1/R (mean over rows)."""
    X = unfold(act, kh, kw, stride, pad, order)
    if has_bias:
        X = np.concatenate([X, np.ones((X.shape[0], 1))], axis=1)
    s = 1.0 / X.shape[0] if scale is None else float(scale)
    return (X.T @ X) * s


def factor_G(gout, scale: float | None = None) -> np.ndarray:
    """G = scale * Gamma^T Gamma, Gamma[(n, y, x), o] = gout[n, o, y, x]; scale defaults to 1/R."""
    gout = np.asarray(gout, dtype=np.float64)
    N, Co, Ho, Wo = gout.shape
    Gamma = gout.transpose(0, 2, 3, 1).reshape(N * Ho * Wo, Co)
    s = 1.0 / Gamma.shape[0] if scale is None else float(scale)
    return (Gamma.T @ Gamma) * s


def ema(running, fresh, decay: float) -> np.ndarray:
    """S_new = decay * S_old + (1 - decay) * X."""
    return float(decay) * np.asarray(running, dtype=np.float64) + (1.0 - float(decay)) * np.asarray(fresh, dtype=np.float64)


def factor_damping(gamma: float) -> float:
    """Per-factor diagonal shift for a block damping gamma: sqrt(gamma) on A and on G."""
    return float(np.sqrt(gamma))


def pi_correction(A, G) -> float:
    """Trace-ratio factor pi of the factored Tikhonov damping of Martens & Grosse (2015), the technique Sec. 4.2 names for
    the Kronecker-factored block: pi = sqrt((tr A / d_A) / (tr G / d_G)), the ratio of the factors' mean eigenvalues.
    (The paper cites the technique without a formula; this is the cited paper's.)"""
    A = np.asarray(A, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    mean_a = np.trace(A) / A.shape[0]
    mean_g = np.trace(G) / G.shape[0]
    return float(np.sqrt(mean_a / mean_g))


def factor_damping_pi(A, G, gamma: float):
    """Per-factor diagonal shifts (lambda_A, lambda_G) = (pi sqrt(gamma), sqrt(gamma) / pi): the block damping gamma
    split between the factors in proportion to their scale, so that (A + lambda_A I) (x) (G + lambda_G I) differs from
    A (x) G + gamma I by cross terms of equal average size.  pi = 1 gives factor_damping's even split."""
    pi = pi_correction(A, G)
    root = float(np.sqrt(gamma))
    return pi * root, root / pi


def warmup_damping_alpha(gamma0: float, gamma_target: float, t_warmup: float) -> float:
    """alpha = 2 log10(gamma0 / gamma_target) / t_warmup (Sec. 4.2, warm-up damping)."""
    return 2.0 * float(np.log10(gamma0 / gamma_target)) / float(t_warmup)


def warmup_damping_next(gamma: float, gamma_target: float, alpha: float) -> float:
    """gamma(t+1) = (1 - alpha) gamma(t) + alpha gamma_target (Sec. 4.2)."""
    return (1.0 - alpha) * gamma + alpha * gamma_target


def bn_damping(gamma: float, rho_bn: float) -> float:
    """Damping of the Batch Normalization layers, rho_BN times the current gamma (Sec. 4.2)."""
    return float(rho_bn) * float(gamma)


def damped_inverse(S, damping: float) -> np.ndarray:
    """(S + damping * I)^-1 for symmetric S."""
    S = np.asarray(S, dtype=np.float64)
    M = S + float(damping) * np.eye(S.shape[0])
    return np.linalg.inv(M)


def precondition(Ginv, gradW, Ainv) -> np.ndarray:
    """P = Ginv . gradW . Ainv for a d_G x d_A weight gradient."""
    return np.asarray(Ginv, dtype=np.float64) @ np.asarray(gradW, dtype=np.float64) @ np.asarray(Ainv, dtype=np.float64)


def kfac_layer_step(act, gout, gradW, A_run, G_run, *, kh, kw, stride, pad, has_bias=True,
                    order=ORDER_C_KH_KW, decay: float | None = 0.95, gamma: float = 1e-3):
    """One K-FAC step of one layer, start to end.  decay=None skips the running average.

    Returns a dict with every intermediate so that a test can compare stage by stage.
    """
    A_new = factor_A(act, kh, kw, stride, pad, has_bias, order)
    G_new = factor_G(gout)
    if decay is None:
        A_s, G_s = A_new, G_new
    else:
        A_s, G_s = ema(A_run, A_new, decay), ema(G_run, G_new, decay)
    lam = factor_damping(gamma)
    A_inv = damped_inverse(A_s, lam)
    G_inv = damped_inverse(G_s, lam)
    P = precondition(G_inv, gradW, A_inv)
    return dict(A_new=A_new, G_new=G_new, A_run=A_s, G_run=G_s, A_inv=A_inv, G_inv=G_inv, P=P)


def factor_bytes(layers, bytes_per_el: int = 4) -> int:
    """Bytes needed to hold every layer's A and G as full dense squares."""
    return sum((l.d_A ** 2 + l.d_G ** 2) * bytes_per_el for l in layers)


def pack_upper(S) -> np.ndarray:
    """Upper triangle of a symmetric n x n matrix, row by row: row i contributes S[i, i], S[i, i+1], ..., S[i, n-1]
    (Sec. 3.4, symmetry-aware communication: only the upper triangular part of a factor is sent)."""
    S = np.asarray(S, dtype=np.float64)
    n = S.shape[0]
    out = []
    for i in range(n):
        out.append(S[i, i:])
    return np.concatenate(out) if out else np.zeros(0)


def unpack_upper(packed, n: int) -> np.ndarray:
    """The symmetric n x n matrix whose upper triangle, row by row, is `packed` (inverse of pack_upper)."""
    packed = np.asarray(packed, dtype=np.float64)
    S = np.zeros((n, n))
    pos = 0
    for i in range(n):
        row = packed[pos:pos + n - i]
        S[i, i:] = row
        S[i:, i] = row
        pos += n - i
    return S


def ema_packed(running, packed_fresh, decay: float) -> np.ndarray:
    """Running average of a full symmetric factor from a fresh factor that arrives as a packed upper triangle (what a
    layer's owner does with the reduced, packed statistics: Sec. 3.3 stage 3 -> 4 with the packing of Sec. 3.4)."""
    running = np.asarray(running, dtype=np.float64)
    return ema(running, unpack_upper(packed_fresh, running.shape[0]), decay)


def factor_diff(X, X_prev) -> float:
    """Change rate of a statistic between two refreshes, ||X - X_prev||_F / ||X_prev||_F (Sec. 5.4, "Staleness of
    Fisher information")."""
    X = np.asarray(X, dtype=np.float64)
    X_prev = np.asarray(X_prev, dtype=np.float64)
    num = 0.0
    den = 0.0
    for a, b in zip(X.ravel(), X_prev.ravel()):
        num += (a - b) * (a - b)
        den += b * b
    return float(np.sqrt(num) / np.sqrt(den))


def refresh_interval(epoch: int) -> int:
    """Iterations between refreshes of the statistics in epoch e: min(20, 5 * floor(e / 5) + 1) (Sec. 5.4, "Training with
    stale Fisher information", first heuristic)."""
    return min(20, 5 * (int(epoch) // 5) + 1)


def refresh_interval_late(epoch: int) -> int:
    """The second heuristic of Sec. 5.4: every iteration before epoch 13, every 20th from then on."""
    return 1 if int(epoch) < 13 else 20


# ---- Batch Normalization layers (Sec. 5.4: their Fisher matrix is not factorised; full or diagonal) -----------------
# The paper gives no formula.  Reading: a BN layer with C channels has parameters theta = (scale_1..scale_C,
# shift_1..shift_C); with xhat the normalised input and gout the gradient w.r.t. the layer's output, the gradient of
# sample n is  d/d scale_c = sum_{y,x} gout[n,c,y,x] xhat[n,c,y,x],  d/d shift_c = sum_{y,x} gout[n,c,y,x];  the
# Fisher matrix is the mini-batch mean of the outer products of these per-sample gradients (the same empirical
# estimate the conv factors are built from), 2C x 2C, or only its diagonal.
def bn_sample_grads(xhat, gout) -> np.ndarray:
    """Per-sample gradients of a BN layer's (scale, shift): (N, C, H, W) x 2 -> (N, 2C)."""
    xhat = np.asarray(xhat, dtype=np.float64)
    gout = np.asarray(gout, dtype=np.float64)
    d_scale = (gout * xhat).sum(axis=(2, 3))
    d_shift = gout.sum(axis=(2, 3))
    return np.concatenate([d_scale, d_shift], axis=1)


def bn_fisher(sample_grads) -> np.ndarray:
    """F = (1/N) sum_n g_n g_n^T, 2C x 2C ("no approx" in Sec. 5.4)."""
    g = np.asarray(sample_grads, dtype=np.float64)
    return g.T @ g / g.shape[0]


def bn_fisher_diag(sample_grads) -> np.ndarray:
    """diag(F): (1/N) sum_n g_n,i^2 (the diagonal approximation of Sec. 5.4)."""
    g = np.asarray(sample_grads, dtype=np.float64)
    return (g * g).sum(axis=0) / g.shape[0]


def bn_precondition_diag(fisher_diag, grad, damping: float) -> np.ndarray:
    """(diag(F) + damping I)^-1 grad, element-wise; damping = rho_BN * gamma (Sec. 4.2)."""
    return np.asarray(grad, dtype=np.float64) / (np.asarray(fisher_diag, dtype=np.float64) + float(damping))


def bn_precondition_full(fisher, grad, damping: float) -> np.ndarray:
    """(F + damping I)^-1 grad."""
    F = np.asarray(fisher, dtype=np.float64)
    return np.linalg.solve(F + float(damping) * np.eye(F.shape[0]), np.asarray(grad, dtype=np.float64))


def learning_rate(epoch: float, eta0: float, e_start: float, e_end: float, p_decay: float) -> float:
    """Polynomial decay of Sec. 4.3: eta0 * (1 - (e - e_start) / (e_end - e_start)) ** p_decay.  The paper defines
    it between e_start and e_end; before e_start this keeps eta0 and after e_end 0 (reading: the decay has not begun /
    has finished)."""
    if epoch <= e_start:
        return float(eta0)
    if epoch >= e_end:
        return 0.0
    return float(eta0) * (1.0 - (epoch - e_start) / (e_end - e_start)) ** p_decay


def momentum_rate(eta: float, eta0: float, m0: float) -> float:
    """m(e) = m0 / eta0 * eta(e): the ratio momentum / learning rate stays fixed (Sec. 4.3)."""
    return float(m0) / float(eta0) * float(eta)


def weight_update(w, w_prev, precond_grad, eta: float, m: float) -> np.ndarray:
    """w_next = w - eta * G + m * (w - w_prev), G the preconditioned gradient (Sec. 4.3, the update equation)."""
    w = np.asarray(w, dtype=np.float64)
    return w - float(eta) * np.asarray(precond_grad, dtype=np.float64) + float(m) * (w - np.asarray(w_prev, dtype=np.float64))


def rescale_weights(w, d_out: int, eps: float = 1e-9) -> np.ndarray:
    """w <- sqrt(2 d_out) * w / (||w|| + eps), eps = 1e-9 (Sec. 4.4, weights rescaling); ||.|| is the 2-norm of all
    of the layer's weights."""
    w = np.asarray(w, dtype=np.float64)
    return np.sqrt(2.0 * d_out) * w / (np.sqrt(np.sum(w * w)) + eps)


def packed_triangle_elems(n: int) -> int:
    """Entries of the upper triangle of an n x n symmetric matrix (Sec. 3.4, symmetry-aware communication)."""
    return n * (n + 1) // 2
