"""Pins for the CPU oracle: each test checks it against something other than itself.

The paper prints no worked numeric example, so the oracle is pinned by what the
definitions and the mathematics fix: an independently written gather-form brute
force, library routines (numpy matmul, scipy correlate2d, torch conv2d and its
autograd), closed forms, the adjoint identities, and the two duality statements
of the section "Backward propagation implementation".
"""
import itertools

import numpy as np
import pytest

import oracle

TINY = [
    # N, C, K, H, W, R, S, stride, pad
    (1, 1, 1, 3, 3, 1, 1, 1, 0),
    (2, 2, 3, 5, 4, 3, 2, 1, 1),
    (1, 3, 2, 7, 6, 3, 3, 2, 1),
    (2, 2, 2, 6, 7, 2, 3, 3, 2),
    (1, 2, 1, 5, 5, 1, 1, 2, 0),
    (1, 1, 2, 4, 6, 3, 3, 1, 0),
    (2, 3, 3, 7, 7, 7, 7, 2, 3),
    (1, 2, 2, 3, 5, 3, 1, 1, 2),
]


def _rand(rng, *shape):
    return rng.uniform(-1.0, 1.0, size=shape)


# ---------------------------------------------------------------- P1 brute force
def gather_fwd(I, Wt, stride, pad):
    """Per output element: walk the input window, look the tap up from the position."""
    N, C, H, W = I.shape
    K, _, R, S = Wt.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    O = np.zeros((N, K, P, Q))
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        tot = 0.0
        for c in range(C):
            for ih in range(H):
                for iw in range(W):
                    r = ih - (p * stride - pad)
                    s = iw - (q * stride - pad)
                    if 0 <= r < R and 0 <= s < S:
                        tot += I[n, c, ih, iw] * Wt[k, c, r, s]
        O[n, k, p, q] = tot
    return O


def gather_bwd(dO, Wt, H, W, stride, pad):
    """Per dI element: solve stride*oj - pad + r = ih for oj, tap by tap."""
    N, K, P, Q = dO.shape
    _, C, R, S = Wt.shape
    dI = np.zeros((N, C, H, W))
    for n, c, ih, iw in itertools.product(range(N), range(C), range(H), range(W)):
        tot = 0.0
        for r in range(R):
            tj = ih + pad - r
            if tj % stride or not (0 <= tj // stride < P):
                continue
            for s in range(S):
                ti = iw + pad - s
                if ti % stride or not (0 <= ti // stride < Q):
                    continue
                for k in range(K):
                    tot += dO[n, k, tj // stride, ti // stride] * Wt[k, c, r, s]
        dI[n, c, ih, iw] = tot
    return dI


def gather_upd(I, dO, R, S, stride, pad):
    """Per dW element: dot product of a strided window of the padded input with dO."""
    N, C, H, W = I.shape
    _, K, P, Q = dO.shape
    Ip = np.zeros((N, C, H + 2 * pad + stride * P, W + 2 * pad + stride * Q))
    Ip[:, :, pad:pad + H, pad:pad + W] = I
    dW = np.zeros((K, C, R, S))
    for k, c, r, s in itertools.product(range(K), range(C), range(R), range(S)):
        win = Ip[:, c, r:r + stride * P:stride, s:s + stride * Q:stride]
        dW[k, c, r, s] = float(np.sum(win * dO[:, k]))
    return dW


@pytest.mark.parametrize("shape", TINY)
def test_brute_force_tiny(shape, rng):
    N, C, K, H, W, R, S, stride, pad = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    assert P == (H + 2 * pad - R) // stride + 1 and Q == (W + 2 * pad - S) // stride + 1
    I, Wt, dO = _rand(rng, N, C, H, W), _rand(rng, K, C, R, S), _rand(rng, N, K, P, Q)
    np.testing.assert_allclose(oracle.fwd(I, Wt, stride, pad), gather_fwd(I, Wt, stride, pad),
                               rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.bwd_data(dO, Wt, H, W, stride, pad),
                               gather_bwd(dO, Wt, H, W, stride, pad), rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.upd(I, dO, R, S, stride, pad),
                               gather_upd(I, dO, R, S, stride, pad), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- P2 1x1 == GEMM
@pytest.mark.parametrize("stride", [1, 2, 3])
def test_1x1_is_gemm(stride, rng):
    """With R = S = 1 the contraction is a matrix product M=k, N=pixels, K=c
    (section "Code generation for convolution microkernel")."""
    N, C, K, H, W = 2, 5, 4, 7, 6
    P, Q = oracle.out_hw(H, W, 1, 1, stride, 0)
    I, Wt, dO = _rand(rng, N, C, H, W), _rand(rng, K, C, 1, 1), _rand(rng, N, K, P, Q)
    Wm = Wt[:, :, 0, 0]
    Is = I[:, :, ::stride, ::stride]
    assert Is.shape[2:] == (P, Q)
    O_ref = np.stack([(Wm @ Is[n].reshape(C, -1)).reshape(K, P, Q) for n in range(N)])
    np.testing.assert_allclose(oracle.fwd(I, Wt, stride, 0), O_ref, atol=1e-13)
    dI_ref = np.zeros((N, C, H, W))
    for n in range(N):
        dI_ref[n, :, ::stride, ::stride] = (Wm.T @ dO[n].reshape(K, -1)).reshape(C, P, Q)
    np.testing.assert_allclose(oracle.bwd_data(dO, Wt, H, W, stride, 0), dI_ref, atol=1e-13)
    dW_ref = sum(dO[n].reshape(K, -1) @ Is[n].reshape(C, -1).T for n in range(N))
    np.testing.assert_allclose(oracle.upd(I, dO, 1, 1, stride, 0)[:, :, 0, 0], dW_ref, atol=1e-13)


# ---------------------------------------------------------------- P3 delta filters
@pytest.mark.parametrize("r0,s0", [(0, 0), (1, 1), (2, 0), (0, 2), (2, 2)])
def test_delta_filter_is_shift(r0, s0, rng):
    """W[k,c,r0,s0] = delta_kc: forward shifts by (r0-pad, s0-pad) with zero fill
    (no filter flip: cross-correlation); backward shifts the other way."""
    N, C, H, W, R, S, pad = 2, 3, 6, 5, 3, 3, 1
    I = _rand(rng, N, C, H, W)
    Wt = np.zeros((C, C, R, S))
    for c in range(C):
        Wt[c, c, r0, s0] = 1.0
    O = oracle.fwd(I, Wt, 1, pad)
    dy, dx = r0 - pad, s0 - pad
    ref = np.zeros_like(I)
    for y in range(H):
        for x in range(W):
            if 0 <= y + dy < H and 0 <= x + dx < W:
                ref[:, :, y, x] = I[:, :, y + dy, x + dx]
    np.testing.assert_array_equal(O, ref)
    dO = _rand(rng, N, C, H, W)
    dI = oracle.bwd_data(dO, Wt, H, W, 1, pad)
    refb = np.zeros_like(dO)
    for y in range(H):
        for x in range(W):
            if 0 <= y - dy < H and 0 <= x - dx < W:
                refb[:, :, y, x] = dO[:, :, y - dy, x - dx]
    np.testing.assert_array_equal(dI, refb)


# ---------------------------------------------------------------- P4 adjoints
@pytest.mark.parametrize("shape", TINY + [(3, 4, 5, 9, 8, 3, 3, 2, 1), (2, 6, 4, 8, 8, 1, 1, 2, 0)])
def test_adjoint_identities(shape, rng):
    """<y, fwd(x,w)> = <bwd_data(y,w), x> = <upd(x,y), w> for every stride and pad."""
    N, C, K, H, W, R, S, stride, pad = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    x, w, y = _rand(rng, N, C, H, W), _rand(rng, K, C, R, S), _rand(rng, N, K, P, Q)
    a = np.vdot(y, oracle.fwd(x, w, stride, pad))
    b = np.vdot(oracle.bwd_data(y, w, H, W, stride, pad), x)
    c = np.vdot(oracle.upd(x, y, R, S, stride, pad), w)
    scale = max(1.0, abs(a))
    assert abs(a - b) < 1e-12 * scale
    assert abs(a - c) < 1e-12 * scale


# ---------------------------------------------------------------- P5 dualities
@pytest.mark.parametrize("R,S,pad", [(3, 3, 1), (3, 3, 0), (2, 2, 1), (5, 5, 2), (1, 1, 0), (7, 7, 3)])
def test_duality_stride1(R, S, pad, rng):
    """stride 1: bwd_data(dO, W; pad) == fwd(dO, W'; R-1-pad) with
    W'[c][k][r'][s'] = W[k][c][R-1-r'][S-1-s'] (scenario 1 of the duality section;
    square filters, so that the single-pad geometry can express the dual problem)."""
    N, C, K, H, W = 2, 3, 4, 7, 6
    P, Q = oracle.out_hw(H, W, R, S, 1, pad)
    dO, Wt = _rand(rng, N, K, P, Q), _rand(rng, K, C, R, S)
    Wp = np.ascontiguousarray(Wt.transpose(1, 0, 2, 3)[:, :, ::-1, ::-1])
    via_fwd = oracle.fwd(dO, Wp, 1, R - 1 - pad)
    assert via_fwd.shape == (N, C, H, W)
    np.testing.assert_allclose(oracle.bwd_data(dO, Wt, H, W, 1, pad), via_fwd, atol=1e-13)


@pytest.mark.parametrize("stride,H,W", [(2, 8, 8), (2, 7, 9), (3, 8, 7)])
def test_duality_1x1_strided(stride, H, W, rng):
    """R = S = 1: dI at positions that are multiples of the stride is W^T dO,
    every other position is zero (scenario 2 of the duality section)."""
    N, C, K = 2, 3, 4
    P, Q = oracle.out_hw(H, W, 1, 1, stride, 0)
    dO, Wt = _rand(rng, N, K, P, Q), _rand(rng, K, C, 1, 1)
    dI = oracle.bwd_data(dO, Wt, H, W, stride, 0)
    dense = np.einsum("kc,nkpq->ncpq", Wt[:, :, 0, 0], dO)
    mask = np.zeros((H, W), dtype=bool)
    mask[::stride, ::stride] = True
    np.testing.assert_allclose(dI[:, :, ::stride, ::stride], dense, atol=1e-13)
    assert np.all(dI[:, :, ~mask] == 0.0)


# ---------------------------------------------------------------- P6 all-ones
@pytest.mark.parametrize("shape", [(2, 3, 2, 6, 7, 3, 3, 1, 1), (1, 2, 3, 9, 8, 3, 3, 2, 1),
                                   (2, 3, 2, 11, 11, 7, 7, 2, 3)])
def test_all_ones_counts_valid_taps(shape):
    N, C, K, H, W, R, S, stride, pad = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    O = oracle.fwd(np.ones((N, C, H, W)), np.ones((K, C, R, S)), stride, pad)
    rows = np.array([sum(0 <= stride * p - pad + r < H for r in range(R)) for p in range(P)])
    cols = np.array([sum(0 <= stride * q - pad + s < W for s in range(S)) for q in range(Q)])
    np.testing.assert_array_equal(O, np.broadcast_to(C * np.outer(rows, cols), O.shape))
    dW = oracle.upd(np.ones((N, C, H, W)), np.ones((N, K, P, Q)), R, S, stride, pad)
    rcount = np.array([sum(0 <= stride * p - pad + r < H for p in range(P)) for r in range(R)])
    scount = np.array([sum(0 <= stride * q - pad + s < W for q in range(Q)) for s in range(S)])
    np.testing.assert_array_equal(dW, np.broadcast_to(N * np.outer(rcount, scount), dW.shape))


# ---------------------------------------------------------------- P7 additivity
def test_upd_is_additive_over_images(rng):
    N, C, K, H, W, R, S, stride, pad = 5, 3, 4, 8, 7, 3, 3, 2, 1
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    I, dO = _rand(rng, N, C, H, W), _rand(rng, N, K, P, Q)
    whole = oracle.upd(I, dO, R, S, stride, pad)
    parts = oracle.upd(I[:2], dO[:2], R, S, stride, pad) + oracle.upd(I[2:], dO[2:], R, S, stride, pad)
    np.testing.assert_allclose(whole, parts, atol=1e-12)
    O = oracle.fwd(I, _rand(rng, K, C, R, S), stride, pad)
    assert O.shape == (N, K, P, Q)


def test_fwd_images_independent(rng):
    N, C, K, H, W, R, S, stride, pad = 3, 2, 3, 6, 6, 3, 3, 1, 1
    I, Wt = _rand(rng, N, C, H, W), _rand(rng, K, C, R, S)
    O = oracle.fwd(I, Wt, stride, pad)
    for n in range(N):
        np.testing.assert_array_equal(O[n:n + 1], oracle.fwd(I[n:n + 1], Wt, stride, pad))


# ---------------------------------------------------------------- P8 library routines
def test_separable_matches_scipy_correlate2d(rng):
    """W = b[k] a[c] g[r,s]  =>  O[n,k] = b[k] * correlate2d(sum_c a[c] I[n,c] (padded), g, 'valid')."""
    from scipy.signal import correlate2d
    N, C, K, H, W, R, S, pad = 2, 4, 3, 9, 8, 3, 3, 1
    a, b, g = rng.normal(size=C), rng.normal(size=K), rng.normal(size=(R, S))
    I = _rand(rng, N, C, H, W)
    Wt = np.einsum("k,c,rs->kcrs", b, a, g)
    for stride in (1, 2):
        O = oracle.fwd(I, Wt, stride, pad)
        for n in range(N):
            m = np.pad(np.tensordot(a, I[n], axes=1), pad)
            full = correlate2d(m, g, mode="valid")[::stride, ::stride]
            for k in range(K):
                np.testing.assert_allclose(O[n, k], b[k] * full, atol=1e-12)
    # update pass with rank-1 activations: dW[k,c,r,s] = a[c] b[k] T[r,s],
    # T = sum_n correlate2d(pad(u_n), v_n, 'valid')  (stride 1).
    u, v = _rand(rng, N, H, W), _rand(rng, N, H, W)
    I1 = np.einsum("c,nhw->nchw", a, u)
    dO1 = np.einsum("k,npq->nkpq", b, v)
    T = sum(correlate2d(np.pad(u[n], pad), v[n], mode="valid") for n in range(N))
    assert T.shape == (R, S)
    dW = oracle.upd(I1, dO1, R, S, 1, pad)
    np.testing.assert_allclose(dW, np.einsum("k,c,rs->kcrs", b, a, T), atol=1e-12)


@pytest.mark.parametrize("shape", [(2, 4, 6, 9, 10, 3, 3, 1, 1), (2, 3, 5, 12, 11, 7, 7, 2, 3),
                                   (3, 8, 4, 8, 8, 1, 1, 2, 0), (2, 5, 3, 9, 9, 3, 3, 2, 1),
                                   (1, 2, 2, 10, 7, 5, 3, 3, 2)])
def test_against_torch_conv2d_and_autograd(shape, rng):
    """torch's fp64 CPU conv2d is the library routine for the forward pass; its
    autograd gradients are the library's backward-by-data and weight update."""
    import torch
    N, C, K, H, W, R, S, stride, pad = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    I, Wt, dO = _rand(rng, N, C, H, W), _rand(rng, K, C, R, S), _rand(rng, N, K, P, Q)
    x = torch.tensor(I, dtype=torch.float64, requires_grad=True)
    w = torch.tensor(Wt, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.conv2d(x, w, stride=stride, padding=pad)
    assert tuple(y.shape) == (N, K, P, Q)
    y.backward(torch.tensor(dO, dtype=torch.float64))
    np.testing.assert_allclose(oracle.fwd(I, Wt, stride, pad), y.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.bwd_data(dO, Wt, H, W, stride, pad), x.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.upd(I, dO, R, S, stride, pad), w.grad.numpy(), atol=1e-12)


def test_upd_entries_match_full(rng):
    N, C, K, H, W, R, S, stride, pad = 3, 4, 5, 9, 8, 3, 3, 2, 1
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    I, dO = _rand(rng, N, C, H, W), _rand(rng, N, K, P, Q)
    full = gather_upd(I, dO, R, S, stride, pad)
    ent = np.array(list(itertools.product(range(K), range(C), range(R), range(S))))[::7]
    got = oracle.upd_entries(I, dO, R, S, stride, pad, ent)
    np.testing.assert_allclose(got, full[ent[:, 0], ent[:, 1], ent[:, 2], ent[:, 3]], atol=1e-13)


def test_thread_count_does_not_change_result(rng):
    """Threads split only loops with disjoint outputs, so results are bitwise stable."""
    import os
    import subprocess
    import sys
    code = ("import numpy as np, oracle, hashlib;"
            "r=np.random.default_rng(5);I=r.normal(size=(4,3,9,9));W=r.normal(size=(5,3,3,3));"
            "dO=r.normal(size=(4,5,5,5));"
            "h=hashlib.sha1();"
            "h.update(oracle.fwd(I,W,2,1).tobytes());h.update(oracle.bwd_data(dO,W,9,9,2,1).tobytes());"
            "h.update(oracle.upd(I,dO,3,3,2,1).tobytes());print(h.hexdigest())")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    outs = set()
    for t in ("1", "3"):
        env = dict(os.environ, OMP_NUM_THREADS=t, PYTHONPATH=root)
        outs.add(subprocess.check_output([sys.executable, "-c", code], env=env, cwd=root).strip())
    assert len(outs) == 1


def test_fused_forward_reduces_to_its_parts():
    """Algorithm 4's L(): with zero weights the result is relu(bias + residual); with no
    operator it is the plain forward pass; ReLU only clamps; bias shifts channel k alone."""
    rng = np.random.default_rng(11)
    N, C, K, H, W, R, S = 2, 3, 4, 5, 6, 3, 3
    I = rng.standard_normal((N, C, H, W))
    Wt = rng.standard_normal((K, C, R, S))
    b = rng.standard_normal(K)
    plain = oracle.fwd(I, Wt, 1, 1)
    res = rng.standard_normal(plain.shape)
    assert np.array_equal(oracle.fwd_fused(I, Wt, 1, 1), plain)
    z = oracle.fwd_fused(I, np.zeros_like(Wt), 1, 1, bias=b, residual=res, relu=True)
    assert np.array_equal(z, np.maximum(b[None, :, None, None] + res, 0.0))
    full = oracle.fwd_fused(I, Wt, 1, 1, bias=b, residual=res, relu=True)
    lin = oracle.fwd_fused(I, Wt, 1, 1, bias=b, residual=res, relu=False)
    assert np.array_equal(full, np.maximum(lin, 0.0))
    assert full.min() == 0.0 and (lin < 0).any()
    only_b = oracle.fwd_fused(I, Wt, 1, 1, bias=b)
    for k in range(K):
        assert np.allclose(only_b[:, k] - plain[:, k], b[k], rtol=0, atol=1e-12)
    # the per-channel scale is a rescaling of the filters of channel k (the convolution is
    # linear in them): scale folded into the weights gives the same result
    g = rng.uniform(0.5, 2.0, size=K) * np.array([1, -1, 1, -1])
    scaled = oracle.fwd_fused(I, Wt, 1, 1, scale=g)
    assert np.allclose(scaled, oracle.fwd(I, Wt * g[:, None, None, None], 1, 1), rtol=1e-13, atol=1e-13)
    allops = oracle.fwd_fused(I, Wt, 1, 1, scale=g, bias=b, residual=res, relu=True)
    assert np.allclose(allops, np.maximum(scaled + b[None, :, None, None] + res, 0.0), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- per-axis padding
# N, C, K, H, W, R, S, stride, pad_h, pad_w: rectangular filters padded along their long side
# only (the 1x7 / 7x1 / 1x3 / 3x1 shapes of Inception-style layers), and unequal pads in general.
RECT = [(2, 3, 4, 7, 9, 1, 7, 1, 0, 3), (2, 2, 3, 9, 7, 7, 1, 1, 3, 0), (1, 3, 2, 8, 8, 1, 3, 1, 0, 1),
        (2, 2, 2, 6, 7, 3, 1, 2, 1, 0), (1, 2, 3, 9, 9, 5, 5, 1, 2, 2), (2, 2, 2, 8, 10, 3, 5, 2, 0, 2),
        (1, 2, 2, 7, 6, 3, 3, 1, 2, 0)]


def _padded(I, ph, pw):
    return np.pad(I, ((0, 0), (0, 0), (ph, ph), (pw, pw)))


def window_fwd(I, Wt, stride, ph, pw):
    """Explicitly padded input, then the pad-free window sum per output element."""
    Ip = _padded(I, ph, pw)
    K, _, R, S = Wt.shape
    P = (Ip.shape[2] - R) // stride + 1
    Q = (Ip.shape[3] - S) // stride + 1
    O = np.zeros((I.shape[0], K, P, Q))
    for n, k, p, q in itertools.product(range(I.shape[0]), range(K), range(P), range(Q)):
        O[n, k, p, q] = np.sum(Ip[n, :, p * stride:p * stride + R, q * stride:q * stride + S] * Wt[k])
    return O


def window_bwd(dO, Wt, H, W, stride, ph, pw):
    """Scatter every output gradient over its window of a padded dI, then crop the padding."""
    N, K, P, Q = dO.shape
    _, C, R, S = Wt.shape
    dIp = np.zeros((N, C, H + 2 * ph + stride, W + 2 * pw + stride))
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        dIp[n, :, p * stride:p * stride + R, q * stride:q * stride + S] += dO[n, k, p, q] * Wt[k]
    return dIp[:, :, ph:ph + H, pw:pw + W]


def window_upd(I, dO, R, S, stride, ph, pw):
    Ip = _padded(I, ph, pw)
    N, K, P, Q = dO.shape
    dW = np.zeros((K, I.shape[1], R, S))
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        dW[k] += dO[n, k, p, q] * Ip[n, :, p * stride:p * stride + R, q * stride:q * stride + S]
    return dW


@pytest.mark.parametrize("shape", RECT)
def test_per_axis_padding_against_explicitly_padded_windows(shape, rng):
    N, C, K, H, W, R, S, stride, ph, pw = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, (ph, pw))
    assert P == (H + 2 * ph - R) // stride + 1 and Q == (W + 2 * pw - S) // stride + 1
    I, Wt, dO = _rand(rng, N, C, H, W), _rand(rng, K, C, R, S), _rand(rng, N, K, P, Q)
    np.testing.assert_allclose(oracle.fwd(I, Wt, stride, (ph, pw)), window_fwd(I, Wt, stride, ph, pw),
                               rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.bwd_data(dO, Wt, H, W, stride, (ph, pw)),
                               window_bwd(dO, Wt, H, W, stride, ph, pw), rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.upd(I, dO, R, S, stride, (ph, pw)),
                               window_upd(I, dO, R, S, stride, ph, pw), rtol=0, atol=1e-13)
    ent = np.array(list(itertools.product(range(K), range(C), range(R), range(S))))[::3]
    np.testing.assert_allclose(oracle.upd_entries(I, dO, R, S, stride, (ph, pw), ent),
                               window_upd(I, dO, R, S, stride, ph, pw)[ent[:, 0], ent[:, 1], ent[:, 2], ent[:, 3]],
                               atol=1e-13)


@pytest.mark.parametrize("shape", RECT)
def test_per_axis_padding_against_torch_and_adjoints(shape, rng):
    import torch
    N, C, K, H, W, R, S, stride, ph, pw = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, (ph, pw))
    I, Wt, dO = _rand(rng, N, C, H, W), _rand(rng, K, C, R, S), _rand(rng, N, K, P, Q)
    x = torch.tensor(I, dtype=torch.float64, requires_grad=True)
    w = torch.tensor(Wt, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.conv2d(x, w, stride=stride, padding=(ph, pw))
    assert tuple(y.shape) == (N, K, P, Q)
    y.backward(torch.tensor(dO, dtype=torch.float64))
    O = oracle.fwd(I, Wt, stride, (ph, pw))
    dI = oracle.bwd_data(dO, Wt, H, W, stride, (ph, pw))
    dW = oracle.upd(I, dO, R, S, stride, (ph, pw))
    np.testing.assert_allclose(O, y.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dI, x.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dW, w.grad.numpy(), atol=1e-12)
    a = np.vdot(dO, O)
    assert abs(a - np.vdot(dI, I)) < 1e-12 * max(1.0, abs(a))
    assert abs(a - np.vdot(dW, Wt)) < 1e-12 * max(1.0, abs(a))


def test_equal_pads_as_pair_or_scalar_agree(rng):
    I, Wt = _rand(rng, 2, 3, 7, 8), _rand(rng, 4, 3, 3, 3)
    np.testing.assert_array_equal(oracle.fwd(I, Wt, 2, 1), oracle.fwd(I, Wt, 2, (1, 1)))
