"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU
oracle on the same seeded inputs.  Bars: rel-L2 <= 1e-5 (fp32), <= 1e-2 (bf16
inputs, fp32 accumulation); integer-valued inputs must match exactly."""
import numpy as np
import pytest

import oracle
from paper_1808_05567_amd import conv, inputs

from gpu_util import assert_close, make_inputs, run_pass

pytestmark = pytest.mark.gpu

DTYPES = [pytest.param(conv.CONV_F32, id="f32"), pytest.param(conv.CONV_BF16, id="bf16")]

# N, C, K, H, W, R, S, stride, pad -- small enough for a full-tensor oracle run,
# large enough to span several tiles, ragged tails and every kernel variant.
SMALL = [
    (2, 64, 64, 14, 14, 3, 3, 1, 1),      # benchmark config 1
    (3, 8, 12, 9, 11, 3, 3, 1, 1),        # rectangular image, K below a tile
    (2, 16, 136, 7, 7, 3, 3, 1, 1),       # ragged channel tile, bands cross images
    (5, 128, 128, 28, 28, 3, 3, 1, 1),    # several row tiles with a ragged last one
    (2, 20, 24, 8, 8, 3, 3, 1, 1),        # odd number of channel blocks
    (2, 24, 40, 12, 10, 3, 3, 1, 0),      # no padding
    (2, 64, 64, 14, 14, 1, 1, 1, 0),
    (3, 64, 256, 56, 56, 1, 1, 1, 0),
    (2, 32, 160, 9, 9, 1, 1, 2, 0),       # stride 2, odd image
    (3, 256, 128, 16, 16, 1, 1, 2, 0),
    (2, 4, 8, 8, 8, 1, 1, 1, 0),          # a single channel block
    (1, 16, 16, 5, 5, 3, 3, 1, 1),        # one tiny image (inference shape)
    (9, 72, 80, 7, 9, 3, 3, 1, 1),        # odd width, ragged channel tiles both ways, many bands
    (2, 64, 64, 14, 14, 3, 3, 2, 1),      # 3x3 stride 2: backward = four residue-class launches
    (3, 32, 48, 15, 13, 3, 3, 2, 1),      # ... odd extents: classes of different sizes
    # 1x1 with at least 256 channels on one side (fp32: the eight-wave update kernel)
    (2, 264, 72, 9, 9, 1, 1, 1, 0),       # ragged channel blocks on both sides, in x out
    (2, 100, 320, 7, 5, 1, 1, 1, 0),      # out x in, 128-channel narrow side, bands cross images
    (1, 512, 256, 6, 6, 1, 1, 2, 0),      # 256 x 256 tile, stride 2
    (2, 256, 36, 5, 5, 1, 1, 1, 0),       # narrow side below 64 channels, a single ragged band
    (2, 16, 24, 3, 37, 1, 1, 1, 0),       # one odd row per flat band: staged with a zero pixel
    # at most 32 channels on a side, odd rows (fp32 update: 32 x 64 and 32 x 32 blocks of dW,
    # four and eight pixel groups)
    (2, 32, 64, 9, 9, 3, 3, 1, 1),
    (3, 32, 32, 11, 15, 3, 3, 1, 1),
    (1, 8, 16, 5, 147, 3, 3, 1, 1),       # ... in strips of 49 columns
    (3, 40, 72, 10, 13, 7, 7, 2, 3),      # 7x7 stride 2 over many channels (fp32 forward: direct kernel)
    # enough 256 x 256 / 128 x 512 tiles for the bf16 eight-wave variants (ragged last pixel tile)
    (25, 128, 512, 28, 28, 1, 1, 1, 0),   # 1x1 forward: 2 channel tiles x 78 pixel tiles, two steps
    (32, 512, 128, 56, 56, 1, 1, 2, 0),   # 1x1 stride 2 backward: scatter with zero fill from eight waves
    (50, 32, 256, 28, 28, 3, 3, 1, 1),    # 3x3 forward: two wave groups staging one halo tile
    (52, 256, 32, 27, 29, 3, 3, 1, 1),    # 3x3 backward, odd extents
]


# few input channels (the first layer of an image network)
FEW_CHANNELS = [
    (2, 3, 64, 32, 32, 7, 7, 2, 3),       # conv1 geometry: 7x7, stride 2, pad 3
    (3, 3, 40, 21, 19, 7, 7, 2, 3),       # odd extents, ragged channel tile
    (2, 3, 32, 19, 21, 7, 7, 2, 3),       # an odd number of stride cells per row (backward pairs them)
    (1, 4, 16, 8, 6, 7, 7, 2, 3),         # ... three cells per row, fewer rows than the filter
    (2, 3, 16, 12, 12, 3, 3, 1, 1),
    (2, 4, 72, 9, 9, 3, 3, 1, 1),
    (2, 1, 32, 20, 18, 7, 7, 2, 3),       # one and two channels: the update's (tap, channel)
    (2, 2, 48, 18, 20, 7, 7, 2, 3),       # columns fill two and four accumulator tiles
    (3, 1, 24, 10, 10, 3, 3, 2, 1),
]

# rectangular filters and padding given per axis (pad_h, pad_w): the factorised 7x7 and 3x3
# filters and the 5x5 filter of Inception-style networks
RECT = [
    (2, 32, 48, 17, 17, 1, 7, 1, (0, 3)),
    (2, 32, 48, 17, 17, 7, 1, 1, (3, 0)),
    (3, 48, 40, 8, 8, 1, 3, 1, (0, 1)),
    (3, 48, 40, 8, 8, 3, 1, 1, (1, 0)),
    (2, 48, 64, 12, 12, 5, 5, 1, 2),
    (2, 160, 192, 17, 17, 1, 7, 1, (0, 3)),   # ragged 128-row channel tiles, several channel steps
    (2, 192, 160, 17, 17, 7, 1, 1, (3, 0)),
    (2, 20, 24, 9, 11, 1, 7, 1, (0, 3)),      # odd numbers of channel blocks
    (2, 20, 24, 11, 9, 7, 1, 1, (3, 0)),
    (2, 16, 24, 10, 9, 3, 3, 1, (2, 0)),      # 3x3 with unequal pads (the dual pads are 0 and 2)
    (2, 16, 24, 10, 9, 3, 3, 1, (0, 1)),
    (2, 24, 16, 9, 11, 3, 3, 2, (1, 0)),      # ... strided: residue classes with per-axis pads
    (2, 24, 32, 13, 13, 3, 3, 2, 0),          # unpadded stride-2 3x3 (grid-reduction layers)
    (2, 12, 16, 9, 9, 1, 7, 1, 0),            # rectangular, unpadded: the output narrows
    (2, 12, 16, 9, 9, 7, 1, 1, (0, 2)),       # padding along the short side only
    # rows wider than one band of the general update kernels: strips of output columns
    (1, 8, 16, 5, 150, 3, 3, 1, 1),
    (1, 16, 24, 4, 75, 1, 1, 1, 0),           # flat bands, a narrower last strip
    (1, 8, 8, 6, 140, 1, 7, 1, (0, 3)),
    (1, 8, 16, 7, 141, 3, 3, 2, 0),
    (2, 3, 32, 37, 301, 3, 3, 2, 0),          # first layer of a 299-wide network, widened
    # unpadded stride 2 on an even extent: a residue class of the backward pass is one
    # row / column larger than dO (its 1x1 sub-filter must not take the sampled staging)
    (2, 20, 16, 32, 22, 3, 3, 2, 0),
    (3, 264, 48, 8, 14, 3, 3, 2, (0, 1)),
    (2, 48, 256, 29, 10, 3, 3, 2, (1, 0)),
    # forward reduction split over workgroups with one channel block per step: fp32 partial
    # results through 16-byte buffer stores (wait states behind the store)
    (1, 264, 256, 23, 39, 1, 1, 1, 0),
    (4, 130, 256, 11, 134, 1, 3, 1, 0),
]

# descriptors outside the tiled kernels' tables: these run (in at least one pass) on the
# untiled direct kernels, which take any filter, stride and per-axis pad
DIRECT = [
    (2, 64, 32, 12, 12, 7, 7, 1, 3),          # 7x7 over many channels
    (2, 20, 24, 9, 11, 1, 5, 1, (0, 2)),
    (2, 24, 16, 11, 9, 5, 1, 2, (2, 0)),
    (2, 8, 16, 10, 10, 2, 2, 2, 0),           # non-overlapping 2x2 windows
    (2, 12, 20, 9, 9, 4, 4, 1, 1),            # even filter
    (1, 12, 8, 9, 8, 4, 3, 3, (1, 2)),        # stride 3, unequal pads
    (1, 16, 16, 8, 120, 7, 1, 1, (3, 0)),     # tall filter over rows wider than a staged tile
    (2, 8, 8, 6, 6, 6, 6, 1, 0),              # filter as large as the image: one output pixel
    (300, 8, 8, 5, 5, 2, 2, 1, 1),            # more pixels than one pass of the update's 256 threads
]


def _layer(shape, dtype):
    return conv.ConvLayer(*shape, dtype=dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", DIRECT, ids=lambda s: "x".join(map(str, s)).replace(" ", ""))
def test_direct_kernels_match_oracle(shape, dtype):
    """Algorithms 1, 6 and 8 as plain loop nests over the blocked layouts, for descriptors no
    tiled kernel fits: every pass has a kernel and matches the oracle."""
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=41)
    L = _layer(shape, dtype)
    try:
        kinds = [conv.conv_describe(L.h, w).split()[0] for w in
                 (conv.PASS_FWD, conv.PASS_BWD_DATA, conv.PASS_UPD)]
        assert "direct" in kinds, kinds
        got = run_pass(L, "fwd", I=I, Wt=Wt)
        assert_close(got, oracle.fwd(I, Wt, stride, pad), dtype, "fwd")
        got = run_pass(L, "bwd", dO=dO, Wt=Wt)
        assert_close(got, oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype, "bwd")
        got = run_pass(L, "upd", I=I, dO=dO)
        assert_close(got, oracle.upd(I, dO, R, S, stride, pad), conv.CONV_F32, "upd")
    finally:
        L.close()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "x".join(map(str, s)))
def test_three_passes_match_oracle(shape, dtype):
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=len(str(shape)))
    L = _layer(shape, dtype)
    try:
        got = run_pass(L, "fwd", I=I, Wt=Wt)
        assert_close(got, oracle.fwd(I, Wt, stride, pad), dtype, "fwd")
        got = run_pass(L, "bwd", dO=dO, Wt=Wt)
        assert_close(got, oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype, "bwd")
        got = run_pass(L, "upd", I=I, dO=dO)
        # weight gradients are fp32 for both dtypes; bf16 products are exact in fp32
        assert_close(got, oracle.upd(I, dO, R, S, stride, pad), conv.CONV_F32, "upd")
    finally:
        L.close()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", RECT, ids=lambda s: "x".join(map(str, s)).replace(" ", ""))
def test_rectangular_filters_match_oracle(shape, dtype):
    """1xS, Rx1 and 5x5 filters, padding per axis: forward, backward by data through the
    flipped filter with the dual pads (R-1-pad_h, S-1-pad_w), weight update one filter
    row per launch."""
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=30 + R + 2 * S)
    L = _layer(shape, dtype)
    try:
        assert_close(run_pass(L, "fwd", I=I, Wt=Wt), oracle.fwd(I, Wt, stride, pad), dtype, "fwd")
        assert_close(run_pass(L, "bwd", dO=dO, Wt=Wt),
                     oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype, "bwd")
        assert_close(run_pass(L, "upd", I=I, dO=dO), oracle.upd(I, dO, R, S, stride, pad), conv.CONV_F32, "upd")
    finally:
        L.close()


def _sweep_shapes():
    rng = np.random.default_rng(5567)
    out = []
    filters = [(1, 7), (7, 1), (1, 3), (3, 1), (5, 5), (3, 3), (1, 1)]
    while len(out) < 35:
        R, S = filters[len(out) % len(filters)]
        stride = int(rng.choice([1, 1, 2])) if R == S else 1
        ph, pw = int(rng.integers(0, R // 2 + 1)), int(rng.integers(0, S // 2 + 1))
        H = int(rng.integers(max(R, 3), 22))
        W = int(rng.integers(max(S, 3), 90 if len(out) % 4 == 0 else 22))
        C = int(rng.choice([3, 8, 20, 48, 72]))
        K = int(rng.choice([8, 24, 40, 96]))
        N = int(rng.integers(1, 4))
        out.append((N, C, K, H, W, R, S, stride, (ph, pw)))
    # a second batch with wider channel counts and images (long reductions at small N: split
    # forward reductions; wide rows: column strips; 7x7)
    filters = filters + [(7, 7), (3, 3), (1, 1)]
    while len(out) < 70:
        R, S = filters[int(rng.integers(0, len(filters)))]
        stride = int(rng.choice([1, 1, 2])) if R == S else 1
        ph, pw = int(rng.integers(0, R // 2 + 1)), int(rng.integers(0, S // 2 + 1))
        H = int(rng.integers(max(R, 3), 40))
        W = int(rng.integers(max(S, 3), 160 if len(out) % 3 == 0 else 40))
        C = int(rng.choice([3, 4, 8, 20, 32, 48, 72, 80, 96, 130, 264]))
        if R == 7 and S == 7:
            C = 3 + int(C % 2)  # (7x7 kernels exist for first layers only)
        K = int(rng.choice([8, 24, 32, 40, 64, 96, 136, 256]))
        N = int(rng.integers(1, 5))
        if N * C * H * W > 3e6 or N * K * H * W > 3e6:
            N = 1
        out.append((N, C, K, H, W, R, S, stride, (ph, pw)))
    return out


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", _sweep_shapes(), ids=lambda s: "x".join(map(str, s)).replace(" ", ""))
def test_seeded_descriptor_sweep_matches_oracle(shape, dtype):
    """Seeded descriptors over the filter shapes, strides and per-axis pads the library
    accepts: every pass matches the oracle, on a tiled kernel or on the direct one."""
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=77)
    L = _layer(shape, dtype)
    ran = 0
    try:
        for which, ref, kind in (
                ("fwd", lambda: oracle.fwd(I, Wt, stride, pad), dtype),
                ("bwd", lambda: oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype),
                ("upd", lambda: oracle.upd(I, dO, R, S, stride, pad), conv.CONV_F32)):
            got = run_pass(L, which, I=I, Wt=Wt, dO=dO)
            assert_close(got, ref(), kind, which)
            ran += 1
    finally:
        L.close()
    assert ran == 3


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", FEW_CHANNELS, ids=lambda s: "x".join(map(str, s)))
def test_few_channel_layers_match_oracle(shape, dtype):
    """C below the channel block: padded slots, tap pairing in the forward kernel,
    residue-class decomposition of the strided backward pass, (tap, channel) columns of the update
    (bf16 tensors are widened on their way into LDS there)."""
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=1)
    L = _layer(shape, dtype)
    try:
        assert_close(run_pass(L, "fwd", I=I, Wt=Wt), oracle.fwd(I, Wt, stride, pad), dtype, "fwd")
        assert_close(run_pass(L, "bwd", dO=dO, Wt=Wt),
                     oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype, "bwd")
        assert_close(run_pass(L, "upd", I=I, dO=dO), oracle.upd(I, dO, R, S, stride, pad), conv.CONV_F32, "upd")
    finally:
        L.close()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("wgs", [1, 2])
def test_first_layer_forward_resident_filter(dtype, wgs, monkeypatch):
    """Forward pass of a first layer on the kernel that keeps the filter in LDS and walks
    several tiles per workgroup, the next tile's input prefetched: with at most `wgs`
    workgroups per XCD a workgroup here walks up to five tiles (ragged last tile, an XCD
    with fewer tiles than the others).  Against the oracle, and bit for bit against the general
    kernel (same tiles, same order of the sum)."""
    shape = (5, 3, 64, 60, 220, 7, 7, 2, 3)
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, _ = make_inputs(shape, dtype, layer_id=1)
    ref = oracle.fwd(I, Wt, stride, pad)
    monkeypatch.setenv("CONVMI_STEM_WG", str(wgs))
    L = _layer(shape, dtype)
    try:
        desc = conv.conv_describe(L.h, 0)
        assert "resident_filter_lds" in desc, desc
        tiles = int(desc.split("tiles=")[1].split()[0])
        assert tiles > 8 * wgs, desc  # (several tiles per workgroup)
        got = run_pass(L, "fwd", I=I, Wt=Wt)
    finally:
        L.close()
    assert_close(got, ref, dtype, "fwd (resident filter)")
    monkeypatch.setenv("CONVMI_STEM", "0")
    L = _layer(shape, dtype)
    try:
        assert "resident_filter_lds" not in conv.conv_describe(L.h, 0)
        plain = run_pass(L, "fwd", I=I, Wt=Wt)
    finally:
        L.close()
    assert np.array_equal(got, plain)


@pytest.mark.parametrize("shape", [FEW_CHANNELS[0], (3, 3, 48, 21, 19, 7, 7, 2, 3)],
                         ids=lambda s: "x".join(map(str, s)))
def test_first_layer_backward_bf16(shape):
    """bf16 backward by data of the strided first layer: all stride-parity classes in one
    launch, 8 channel slots per class, interleaving store (odd extents drop the last cell row)."""
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, conv.CONV_BF16, layer_id=1)
    L = _layer(shape, conv.CONV_BF16)
    try:
        assert_close(run_pass(L, "bwd", dO=dO, Wt=Wt),
                     oracle.bwd_data(dO, Wt, H, W, stride, pad), conv.CONV_BF16, "bwd")
    finally:
        L.close()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(3, 32, 48, 14, 14, 3, 3, 1, 1), (2, 64, 32, 12, 12, 1, 1, 2, 0),
                                   (2, 288, 96, 10, 10, 1, 1, 2, 0), (2, 8, 8, 6, 6, 6, 6, 1, 0),
                                   (2, 12, 20, 9, 9, 4, 4, 2, 1)],
                         ids=["3x3", "1x1s2", "1x1s2wide", "6x6direct", "4x4s2direct"])
def test_integer_inputs_are_exact(shape, dtype):
    """Small integers: every product and partial sum is exact in fp32 (and the
    values are exact in bf16), so any summation order gives the oracle's bits; a bf16
    output is that exact value rounded once (to nearest even), in both the forward and the
    backward pass."""
    N, C, K, H, W, R, S, stride, pad = shape
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    I = inputs.gen_small_ints((N, C, H, W), -2, 2, which=3)
    Wt = inputs.gen_small_ints((K, C, R, S), -2, 2, which=4)
    dO = inputs.gen_small_ints((N, K, P, Q), -2, 2, which=5)
    L = _layer(shape, dtype)
    try:
        got = run_pass(L, "upd", I=I, dO=dO)
        assert np.array_equal(got, oracle.upd(I, dO, R, S, stride, pad))
        # (all sums stay far below 2^24, so the fp32 accumulator holds the oracle's value exactly;
        # a bf16 store keeps 8 significant bits of it)
        out_type = inputs.round_to_bf16 if dtype == conv.CONV_BF16 else (lambda x: x)
        ref = oracle.fwd(I, Wt, stride, pad)
        assert np.abs(ref).max() < 2 ** 24
        assert np.array_equal(run_pass(L, "fwd", I=I, Wt=Wt), out_type(ref.astype(np.float32)))
        ref = oracle.bwd_data(dO, Wt, H, W, stride, pad)
        assert np.abs(ref).max() < 2 ** 24
        assert np.array_equal(run_pass(L, "bwd", dO=dO, Wt=Wt), out_type(ref.astype(np.float32)))
    finally:
        L.close()


def test_pack_unpack_roundtrip_and_padding():
    import torch
    shape = (2, 10, 6, 5, 7, 3, 3, 1, 1)  # C, K not multiples of the block
    for dtype in (conv.CONV_F32, conv.CONV_BF16):
        I, Wt, dO = make_inputs(shape, dtype)
        L = _layer(shape, dtype)
        try:
            L.in_blk.fill_(float("nan")); L.wt_blk.fill_(float("nan")); L.out_blk.fill_(float("nan"))
            L.set_input(I); L.set_weights(Wt); L.set_outgrad(dO)
            assert np.array_equal(L.get_input().float().cpu().numpy(), I)
            assert np.array_equal(L.get_weights().float().cpu().numpy(), Wt)
            assert np.array_equal(L.get_output().float().cpu().numpy(), dO)
            v = L.info.vlen
            blk = L.in_blk.float().view(2, L.info.Cb, 5, 7, v).cpu().numpy()
            assert np.all(blk[:, -1, :, :, 10 % v:] == 0)          # padded channel slots are zero
            assert np.array_equal(blk[:, 1, :, :, 0], I[:, v])      # channel v sits in block 1, slot 0
            w = L.wt_blk.float().view(L.info.Cb, 3, 3, L.info.Kp, v).cpu().numpy()
            assert np.array_equal(w[0, 1, 2, 5, 3], Wt[5, 3, 1, 2])
            assert np.all(w[:, :, :, 6:, :] == 0)
        finally:
            L.close()
        torch.cuda.synchronize()


def test_upd_is_bitwise_deterministic():
    shape = (4, 64, 64, 28, 28, 3, 3, 1, 1)
    I, Wt, dO = make_inputs(shape, conv.CONV_F32)
    L = _layer(shape, conv.CONV_F32)
    try:
        a = run_pass(L, "upd", I=I, dO=dO)
        b = run_pass(L, "upd", I=I, dO=dO)
        assert np.array_equal(a, b)
        assert L.info.upd_splits > 1
    finally:
        L.close()


REPEAT = [
    (1, 264, 256, 23, 39, 1, 1, 1, 0),    # split forward reduction, 16-byte partial stores
    (4, 130, 256, 11, 134, 1, 3, 1, 0),
    (16, 64, 64, 28, 28, 3, 3, 1, 1),
    (8, 256, 128, 14, 14, 1, 1, 2, 0),
    (4, 32, 64, 35, 35, 3, 3, 1, 1),      # four pixel groups folded through LDS
    (2, 3, 64, 64, 64, 7, 7, 2, 3),
    (4, 96, 96, 17, 17, 7, 1, 1, (3, 0)),
    (300, 8, 8, 5, 5, 2, 2, 1, 1),        # the untiled direct kernels: update ...
    (8, 20, 24, 9, 11, 1, 5, 1, (0, 2)),  # ... forward and backward
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", REPEAT, ids=lambda s: "x".join(map(str, s)).replace(" ", ""))
def test_every_pass_repeats_bit_for_bit(shape, dtype):
    """No result may depend on timing: fixed-order reductions everywhere, and no store whose
    data a later instruction can overtake.  Four runs of each pass give identical bits."""
    I, Wt, dO = make_inputs(shape, dtype, layer_id=9)
    L = _layer(shape, dtype)
    try:
        for which in ("fwd", "bwd", "upd"):
            first = run_pass(L, which, I=I, Wt=Wt, dO=dO)
            assert np.isfinite(first).all(), which
            for _ in range(3):
                assert np.array_equal(first, run_pass(L, which, I=I, Wt=Wt, dO=dO)), which
    finally:
        L.close()


FUSED = [
    (2, 64, 64, 14, 14, 3, 3, 1, 1),      # reduction split over workgroups: operators in the reduce
    (5, 128, 128, 28, 28, 3, 3, 1, 1),    # many tiles: operators in the convolution's store
    (3, 64, 256, 56, 56, 1, 1, 1, 0),
    (2, 20, 24, 8, 8, 3, 3, 1, 1),        # padded channel slots stay zero
    (2, 48, 72, 17, 17, 1, 7, 1, (0, 3)),  # rectangular filter, padding along one axis
    (2, 32, 40, 13, 13, 3, 3, 2, 0),       # unpadded stride 2
    (2, 20, 24, 9, 11, 1, 5, 1, (0, 2)),   # a filter only the direct kernel serves
    (3, 3, 64, 40, 44, 7, 7, 2, 3),        # a first layer: operators in the resident-filter kernel's store
    (2, 3, 40, 21, 19, 7, 7, 2, 3),        # ... with a ragged channel tile
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", FUSED, ids=lambda s: "x".join(map(str, s)).replace(" ", ""))
def test_fused_forward_matches_oracle(shape, dtype):
    """Section II-G / Algorithm 4: bias, residual and ReLU applied before the result is stored."""
    import torch
    from paper_1808_05567_amd import inputs
    N, C, K, H, W, R, S, stride, pad = shape
    I, Wt, dO = make_inputs(shape, dtype, layer_id=7)
    P, Q = oracle.out_hw(H, W, R, S, stride, pad)
    rng = np.random.default_rng(5)
    bias = rng.standard_normal(K).astype(np.float32)
    res = rng.uniform(-1, 1, size=(N, K, P, Q)).astype(np.float32)
    if dtype == conv.CONV_BF16:
        res = inputs.round_to_bf16(res)
    L = _layer(shape, dtype)
    try:
        info = conv.conv_query(L.h)
        if C <= 4 and R == 7 and S == 7:
            # (the first-layer cases are there for the resident-filter kernel's fused store, which
            # fp32 uses; a fused bf16 pass of such a layer runs on the general kernel)
            assert "resident_filter_lds" in conv.conv_describe(L.h, 0)
        bias_dev = torch.zeros(info.Kp, dtype=torch.float32, device="cuda")
        bias_dev[:K] = torch.from_numpy(bias)
        scale = rng.uniform(0.5, 1.5, size=K).astype(np.float32) * rng.choice([-1.0, 1.0], size=K).astype(np.float32)
        scale_dev = torch.ones(info.Kp, dtype=torch.float32, device="cuda")
        scale_dev[:K] = torch.from_numpy(scale)
        L.set_outgrad(res)                 # blocked tensor of the output's shape ...
        res_blk = L.out_blk.clone()        # ... used as the residual
        L.set_input(I)
        L.set_weights(Wt)
        for kw in (dict(bias=bias_dev), dict(residual=res_blk, relu=True),
                   dict(bias=bias_dev, residual=res_blk, relu=True), dict(scale=scale_dev),
                   dict(scale=scale_dev, bias=bias_dev, residual=res_blk, relu=True)):
            L.out_blk.fill_(float("nan"))
            L.fwd_fused(**kw)
            torch.cuda.synchronize()
            got = L.get_output().float().cpu().numpy()
            ref = oracle.fwd_fused(I, Wt, stride, pad, bias=bias if "bias" in kw else None,
                                   residual=res if "residual" in kw else None,
                                   relu=kw.get("relu", False), scale=scale if "scale" in kw else None)
            assert_close(got, ref, dtype, "fused %s" % sorted(kw))
            if kw.get("relu"):
                assert got.min() >= 0.0
        # in place: the residual is the output buffer itself
        L.out_blk.copy_(res_blk)
        L.fwd_fused(bias=bias_dev, residual=L.out_blk, relu=True)
        torch.cuda.synchronize()
        got = L.get_output().float().cpu().numpy()
        ref = oracle.fwd_fused(I, Wt, stride, pad, bias=bias, residual=res, relu=True)
        assert_close(got, ref, dtype, "fused in place")
    finally:
        L.close()


@pytest.mark.gpu
def test_shader_clock_sampler_waits_out_its_window_and_reports_a_plausible_clock():
    """One sleeping wave per XCD counts shader cycles against the 100 MHz clock: the window it
    reports is the one asked for (within a sleep quantum), and the clock lies between the
    idle floor and the 2.4 GHz the peaks are quoted at (plus measurement slack)."""
    import torch
    ticks = torch.zeros(16, dtype=torch.int64, device="cuda")
    conv.conv_ceiling_shader_clock(8, 2000, ticks)
    torch.cuda.synchronize()
    t = ticks.cpu().view(8, 2)
    assert (t[:, 1] >= 2000 * 100).all() and (t[:, 1] < 2100 * 100).all()
    mhz = t[:, 0].double() / (t[:, 1].double() / 100.0)
    assert (mhz > 50).all() and (mhz < 2600).all()
