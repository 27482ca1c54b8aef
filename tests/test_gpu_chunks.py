"""The minibatch in chunks (conv_create_chunked, and conv_create by itself for tensors of
4 GB and more): every pass runs once per chunk on that chunk's slice of the tensors, and
the result must be the whole minibatch's, against the oracle."""
import numpy as np
import pytest

import oracle
from paper_1808_05567_amd import conv, inputs

from gpu_util import assert_close, make_inputs, run_pass

pytestmark = pytest.mark.gpu

DTYPES = [pytest.param(conv.CONV_F32, id="f32"), pytest.param(conv.CONV_BF16, id="bf16")]

# (N, C, K, H, W, R, S, stride, pad), images per chunk
CHUNKED = [
    ((10, 64, 64, 14, 14, 3, 3, 1, 1), 4),           # chunks of 4, 4, 2
    ((9, 64, 64, 14, 14, 3, 3, 1, 1), 3),            # three equal chunks
    ((7, 32, 160, 9, 9, 1, 1, 2, 0), 3),             # 3, 3, 1: the last chunk is one image
    ((5, 3, 64, 32, 32, 7, 7, 2, 3), 2),             # first-layer kernels
    ((4, 48, 40, 8, 8, 1, 3, 1, (0, 1)), 1),         # one image per launch
    ((6, 20, 24, 9, 11, 1, 5, 1, (0, 2)), 4),        # chunks that run on the direct kernels
    ((5, 24, 32, 13, 13, 3, 3, 2, 0), 2),            # strided backward: several launches per chunk
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape,max_images", CHUNKED,
                         ids=["x".join(map(str, s)).replace(" ", "") + "-by%d" % m for s, m in CHUNKED])
def test_chunked_passes_match_oracle(shape, max_images, dtype):
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=23)
    L = conv.ConvLayer(*shape, dtype=dtype, max_images=max_images)
    try:
        n_chunks = -(-N // max_images)
        for which in (conv.PASS_FWD, conv.PASS_BWD_DATA, conv.PASS_UPD):
            assert conv.conv_describe(L.h, which).startswith("chunks=%d images=%d: " % (n_chunks, max_images))
        assert L.info.upd_splits == n_chunks
        got = run_pass(L, "fwd", I=I, Wt=Wt)
        assert_close(got, oracle.fwd(I, Wt, stride, pad), dtype, "fwd")
        got = run_pass(L, "bwd", dO=dO, Wt=Wt)
        assert_close(got, oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype, "bwd")
        got = run_pass(L, "upd", I=I, dO=dO)
        assert_close(got, oracle.upd(I, dO, R, S, stride, pad), conv.CONV_F32, "upd")
    finally:
        L.close()


@pytest.mark.parametrize("dtype", DTYPES)
def test_chunked_fused_forward_takes_the_residual_slice(dtype):
    """Each chunk adds its own slice of the residual; scale and bias are per channel."""
    import torch
    shape, max_images = (7, 40, 72, 10, 10, 3, 3, 1, 1), 3
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, _ = make_inputs(shape, dtype, layer_id=29)
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    rng = np.random.default_rng(11)
    bias = rng.standard_normal(K).astype(np.float32)
    scale = rng.uniform(0.5, 1.5, size=K).astype(np.float32)
    res = rng.uniform(-1, 1, size=(N, K, P, Q)).astype(np.float32)
    if dtype == conv.CONV_BF16:
        res = inputs.round_to_bf16(res)
    L = conv.ConvLayer(*shape, dtype=dtype, max_images=max_images)
    try:
        bias_dev = torch.zeros(L.info.Kp, dtype=torch.float32, device="cuda")
        bias_dev[:K] = torch.from_numpy(bias)
        scale_dev = torch.ones(L.info.Kp, dtype=torch.float32, device="cuda")
        scale_dev[:K] = torch.from_numpy(scale)
        L.set_outgrad(res)
        res_blk = L.out_blk.clone()
        L.set_input(I)
        L.set_weights(Wt)
        L.out_blk.fill_(float("nan"))
        L.fwd_fused(bias=bias_dev, residual=res_blk, relu=True, scale=scale_dev)
        torch.cuda.synchronize()
        got = L.get_output().float().cpu().numpy()
        ref = oracle.fwd_fused(I, Wt, stride, pad, bias=bias, residual=res, relu=True, scale=scale)
        assert_close(got, ref, dtype, "fused chunks")
    finally:
        L.close()


def test_chunked_update_repeats_bit_for_bit():
    shape = (10, 64, 64, 14, 14, 3, 3, 1, 1)
    I, Wt, dO = make_inputs(shape, conv.CONV_F32, layer_id=31)
    L = conv.ConvLayer(*shape, dtype=conv.CONV_F32, max_images=4)
    try:
        first = run_pass(L, "upd", I=I, dO=dO)
        for _ in range(3):
            assert np.array_equal(first, run_pass(L, "upd", I=I, dO=dO))
    finally:
        L.close()


def _sampled_parity(shape, dtype, seed, chunked):
    """All three passes of a large problem: the oracle computes every output of the first and
    last image and of the two images in the middle (either side of a chunk boundary where there
    is one), and a seeded subset of dW entries, each a full N*P*Q-long dot product (summed over
    the two halves of the minibatch to bound the fp64 copies)."""
    import torch
    N, C, K, H, W, R, S, stride, pad = shape
    print("shape", shape, "dtype", dtype, flush=True)
    L = conv.ConvLayer(*shape, dtype=dtype)
    try:
        P, Q = L.info.P, L.info.Q
        for which in (conv.PASS_FWD, conv.PASS_BWD_DATA):
            assert conv.conv_describe(L.h, which).startswith("chunks=2 ") == chunked
            assert " igemm " in " " + conv.conv_describe(L.h, which)
        I = inputs.gen_input(N, C, H, W, seed)
        Wt = inputs.gen_weights(K, C, R, S, seed)
        dO = inputs.gen_outgrad(N, K, P, Q, seed)
        if dtype == conv.CONV_BF16:
            I, Wt, dO = (inputs.round_to_bf16(x) for x in (I, Wt, dO))
        imgs = [0, N // 2 - 1, N // 2, N - 1]
        L.set_input(I)
        L.set_weights(Wt)
        L.out_blk.fill_(float("nan"))
        L.fwd()
        out = L.get_output()
        torch.cuda.synchronize()
        got = out[imgs].float().cpu().numpy()
        assert bool(torch.isfinite(out).all())
        del out
        assert_close(got, oracle.fwd(I[imgs], Wt, stride, pad), dtype, "fwd")
        print("fwd done", flush=True)

        L.set_outgrad(dO)
        L.in_blk.fill_(float("nan"))
        L.bwd_data()
        din = L.get_input()
        torch.cuda.synchronize()
        got = din[imgs].float().cpu().numpy()
        assert bool(torch.isfinite(din).all())
        del din
        assert_close(got, oracle.bwd_data(dO[imgs], Wt, H, W, stride, pad), dtype, "bwd")
        print("bwd done", flush=True)

        L.set_input(I)   # (the backward pass wrote dI over the blocked input)
        L.dwt_blk.fill_(float("nan"))
        L.upd()
        torch.cuda.synchronize()
        got = L.get_dweights().cpu().numpy()
        assert np.isfinite(got).all()
        rng = np.random.default_rng(seed)
        ent = np.stack([rng.integers(0, K, 24), rng.integers(0, C, 24), rng.integers(0, R, 24),
                        rng.integers(0, S, 24)], axis=1).astype(np.int32)
        ent = np.concatenate([np.array([[0, 0, 0, 0], [K - 1, C - 1, R - 1, S - 1]], dtype=np.int32), ent])
        ref = sum(oracle.upd_entries(I[a:b], dO[a:b], R, S, stride, pad, ent)
                  for a, b in ((0, N // 2), (N // 2, N)))
        assert_close(got[ent[:, 0], ent[:, 1], ent[:, 2], ent[:, 3]], ref, conv.CONV_F32, "upd entries")
    finally:
        L.close()


def test_output_tensor_beyond_4gb_runs_in_chunks():
    """An output tensor of 4.5 GB (fp32): forward and backward run as two chunks of 176
    images on the tiled kernels, the update in one piece on a kernel with 64-bit addressing."""
    shape = (352, 8, 64, 224, 224, 3, 3, 1, 1)
    _sampled_parity(shape, conv.CONV_F32, 37, chunked=True)


@pytest.mark.parametrize("shape", [(4000, 64, 64, 56, 56, 3, 3, 1, 1), (1200, 256, 64, 56, 56, 1, 1, 1, 0)],
                         ids=["3x3-3.2GB", "1x1-3.9GB"])
def test_tensors_between_2gb_and_4gb_in_one_launch(shape):
    """Byte offsets past 2^31 (a signed 32-bit offset would wrap) in single launches of the
    forward / backward kernel and of the fp32 band and flat update kernels."""
    _sampled_parity(shape, conv.CONV_F32, 41, chunked=False)
