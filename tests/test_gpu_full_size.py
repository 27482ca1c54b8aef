"""Parity at the benchmark's full sizes (N = 256, the launch configuration
bench.py times).  A full fp64 oracle pass is too slow there, so:
  * forward / backward: images are independent -- the oracle computes every
    output of a seeded subset of images (always the first and the last);
  * update: the oracle computes a seeded subset of dW entries, each one a full
    N*P*Q-long fp64 dot product (always including the corner taps/channels).
"""
import numpy as np
import pytest

import oracle
from paper_1808_05567_amd import conv, inputs

from gpu_util import assert_close, run_pass

pytestmark = pytest.mark.gpu

N = 256
# every layer of Table I in both types: each layer has its own tile, split and kernel variant
# (layer-major order, so that the two types of a layer share one set of generated inputs)
CASES = [(l.id, dt) for l in inputs.TABLE_I for dt in (conv.CONV_F32, conv.CONV_BF16)]
_generated = {}


def _inputs_of(l, lid):
    """Seeded fp32 operands of a layer at N = 256, kept for the next case of the same layer."""
    if lid not in _generated:
        _generated.clear()
        _generated[lid] = (inputs.gen_input(N, l.C, l.H, l.W, lid),
                           inputs.gen_weights(l.K, l.C, l.R, l.S, lid),
                           inputs.gen_outgrad(N, l.K, l.P, l.Q, lid))
    return _generated[lid]


def _entries(rng, K, C, R, S, count):
    e = np.stack([rng.integers(0, K, count), rng.integers(0, C, count),
                  rng.integers(0, R, count), rng.integers(0, S, count)], axis=1)
    corners = [(k, c, r, s) for k in (0, K - 1) for c in (0, C - 1)
               for r in (0, R - 1) for s in (0, S - 1)]
    return np.concatenate([np.array(corners), e]).astype(np.int32)


# Inception-v3 shapes (ids of inputs.INCEPTION_V3): the first layer (299 wide, stride 2,
# unpadded), a 147-wide 3x3 (update in column strips), 5x5, unpadded stride-2 3x3, 1x7 / 7x1
# at 160 and 192 channels, 1x3 / 3x1
V3_CASES = [(1, conv.CONV_F32), (1, conv.CONV_BF16), (3, conv.CONV_F32), (13, conv.CONV_F32), (16, conv.CONV_F32),
            (29, conv.CONV_F32), (30, conv.CONV_F32), (41, conv.CONV_F32), (42, conv.CONV_F32),
            (2, conv.CONV_BF16), (13, conv.CONV_BF16), (25, conv.CONV_BF16), (26, conv.CONV_BF16),
            (42, conv.CONV_BF16),
            # 32-row tiles of the 32-channel stem, 128-row tiles of a 17-pixel-wide grid reduction
            (2, conv.CONV_F32), (16, conv.CONV_BF16)]


@pytest.mark.parametrize("lid,dtype", CASES,
                         ids=["L%d-%s" % (l, "bf16" if d else "f32") for l, d in CASES])
def test_table1_layer_at_n256(lid, dtype):
    _layer_at_n256(inputs.layer(lid), lid, dtype)


@pytest.mark.parametrize("lid,dtype", V3_CASES,
                         ids=["V3L%d-%s" % (l, "bf16" if d else "f32") for l, d in V3_CASES])
def test_inception_v3_layer_at_n256(lid, dtype):
    _layer_at_n256(inputs.layer(lid, "inception_v3"), 100 + lid, dtype)


def _layer_at_n256(l, lid, dtype):
    print("layer", lid, "dtype", dtype, flush=True)
    I, Wt, dO = _inputs_of(l, lid)
    if dtype == conv.CONV_BF16:
        I, Wt, dO = (inputs.round_to_bf16(x) for x in (I, Wt, dO))
    rng = np.random.default_rng(1000 + lid)
    imgs = sorted({0, N - 1, *rng.integers(1, N - 1, 2).tolist()})
    L = conv.ConvLayer(N, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad, dtype=dtype)
    try:
        got = run_pass(L, "fwd", I=I, Wt=Wt)
        ref = oracle.fwd(I[imgs], Wt, l.stride, l.pad)
        assert_close(got[imgs], ref, dtype, "fwd")
        assert np.isfinite(got).all()
        got = run_pass(L, "bwd", dO=dO, Wt=Wt)
        ref = oracle.bwd_data(dO[imgs], Wt, l.H, l.W, l.stride, l.pad)
        assert_close(got[imgs], ref, dtype, "bwd")
        assert np.isfinite(got).all()
        got = run_pass(L, "upd", I=I, dO=dO)
        ent = _entries(rng, l.K, l.C, l.R, l.S, 512 if l.H > 200 else 2048)
        ref = oracle.upd_entries(I.astype(np.float64), dO.astype(np.float64), l.R, l.S,
                                 l.stride, l.pad, ent)
        assert_close(got[ent[:, 0], ent[:, 1], ent[:, 2], ent[:, 3]], ref, conv.CONV_F32, "upd")
        assert np.isfinite(got).all()
    finally:
        L.close()


SEP_CASES = [(4, conv.CONV_F32), (18, conv.CONV_F32), (6, conv.CONV_F32), (1, conv.CONV_F32),
             (13, conv.CONV_BF16), (2, conv.CONV_BF16), (1, conv.CONV_BF16)]


@pytest.mark.parametrize("lid,dtype", SEP_CASES,
                         ids=["L%d-%s" % (l, "bf16" if d else "f32") for l, d in SEP_CASES])
def test_full_tensor_at_n256_separable_integers(lid, dtype):
    """Every output of every image at N = 256, exactly.  With rank-1 weights
    W[k,c,r,s] = b[k] a[c] g[r,s] the passes collapse to single-channel convolutions:
        fwd:  O[n,k]  = b[k] * conv1(sum_c a[c] I[n,c], g)
        bwd:  dI[n,c] = a[c] * conv1_bwd(sum_k b[k] dO[n,k], g)
        upd:  I = a[c] u[n], dO = b[k] v[n]  =>  dW[k,c,r,s] = a[c] b[k] * conv1_upd(u, v)[r,s]
    and the oracle computes the single-channel problems in full.  All values are small
    integers, so every product and partial sum is exact in fp32 (|sum| < 2^24) whatever the
    summation order: the result must match bit for bit (bf16 outputs: the exact value
    rounded once to bf16).  Distinct a[c], b[k] catch channel permutations."""
    l = inputs.layer(lid)
    rng = np.random.default_rng(4242 + lid)
    a = rng.choice([-2, -1, 1, 2], size=l.C).astype(np.float32)
    b = rng.choice([-2, -1, 1, 2], size=l.K).astype(np.float32)
    g = rng.integers(-1, 2, size=(l.R, l.S)).astype(np.float32)
    Wt = b[:, None, None, None] * a[None, :, None, None] * g[None, None]
    g1 = g[None, None].astype(np.float64)
    out_round = inputs.round_to_bf16 if dtype == conv.CONV_BF16 else (lambda x: x)
    L = conv.ConvLayer(N, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad, dtype=dtype)
    try:
        I = rng.integers(-1, 2, size=(N, l.C, l.H, l.W)).astype(np.float32)
        J = np.einsum("c,nchw->nhw", a.astype(np.float64), I)[:, None]
        ref = b[None, :, None, None] * oracle.fwd(J, g1, l.stride, l.pad)
        got = run_pass(L, "fwd", I=I, Wt=Wt)
        assert np.array_equal(got, out_round(ref.astype(np.float32)))
        del J, ref, got

        dO = rng.integers(-1, 2, size=(N, l.K, l.P, l.Q)).astype(np.float32)
        G = np.einsum("k,nkpq->npq", b.astype(np.float64), dO)[:, None]
        ref = a[None, :, None, None] * oracle.bwd_data(G, g1, l.H, l.W, l.stride, l.pad)
        got = run_pass(L, "bwd", dO=dO, Wt=Wt)
        assert np.array_equal(got, out_round(ref.astype(np.float32)))
        del G, ref, got, I, dO

        u = rng.integers(-1, 2, size=(N, 1, l.H, l.W)).astype(np.float32)
        v = rng.integers(-1, 2, size=(N, 1, l.P, l.Q)).astype(np.float32)
        T = oracle.upd(u.astype(np.float64), v.astype(np.float64), l.R, l.S, l.stride, l.pad)[0, 0]
        assert np.abs(T).max() * 4 < 2 ** 24
        ref = b[:, None, None, None] * a[None, :, None, None] * T[None, None]
        got = run_pass(L, "upd", I=a[None, :, None, None] * u, dO=b[None, :, None, None] * v)
        assert np.array_equal(got, ref.astype(np.float32))
    finally:
        L.close()


# (the 3-channel first layer is an fp32 workload only)
N1_CASES = [(lid, dt) for lid in (4, 8, 13, 18, 1, 6, 20) for dt in (conv.CONV_F32, conv.CONV_BF16)
            if not (lid == 1 and dt == conv.CONV_BF16)]


@pytest.mark.parametrize("lid,dtype", N1_CASES,
                         ids=["L%d-%s" % (l, "bf16" if d else "f32") for l, d in N1_CASES])
def test_single_image_inference_forward(lid, dtype):
    """N = 1 forward (latency-bound, few tiles): full-tensor oracle comparison."""
    l = inputs.layer(lid)
    I = inputs.gen_input(1, l.C, l.H, l.W, lid)
    Wt = inputs.gen_weights(l.K, l.C, l.R, l.S, lid)
    if dtype == conv.CONV_BF16:
        I, Wt = inputs.round_to_bf16(I), inputs.round_to_bf16(Wt)
    L = conv.ConvLayer(1, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad, dtype=dtype)
    try:
        got = run_pass(L, "fwd", I=I, Wt=Wt)
        assert_close(got, oracle.fwd(I, Wt, l.stride, l.pad), dtype, "fwd")
    finally:
        L.close()
