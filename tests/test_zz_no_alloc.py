"""The entry point that allocates nothing (conv_bwd_data_noalloc: scratch in a static device
array) against the existing conv_bwd_data on the same inputs, two calls in a row, the second
on a smaller problem; and the size check that precedes any launch."""
import numpy as np
import pytest

import oracle
from paper_1808_05567_amd import conv

from gpu_util import assert_close, make_inputs


def test_scratch_limit_is_checked_on_the_host_before_any_launch():
    lib = conv.load()
    assert lib.conv_noalloc_scratch_bytes() == 16 << 20
    # 1x1, 2048 -> 4096 channels in fp32: 32 MiB of transformed weights
    h = conv.conv_create(2, 2048, 4096, 7, 7, 1, 1, 1, 0, conv.CONV_F32)
    try:
        assert lib.conv_bwd_data_noalloc(h, 16, 16, 16, None) == conv.CONV_ESCRATCH
        assert lib.conv_bwd_data_noalloc(h, None, 16, 16, None) == conv.CONV_EINVAL
        assert "scratch" in conv.status_str(conv.CONV_ESCRATCH)
    finally:
        conv.conv_destroy(h)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [conv.CONV_F32, conv.CONV_BF16], ids=["f32", "bf16"])
def test_noalloc_backward_matches_the_workspace_entry_point(dtype):
    import torch
    # the larger problem first (3x3, 9 taps of 128 x 128 weights), then a smaller one whose
    # transformed weights cover only the head of the array the first call filled; then a
    # strided 3x3 (four residue-class transforms side by side in the scratch)
    shapes = [(4, 128, 128, 14, 14, 3, 3, 1, 1), (3, 24, 40, 9, 11, 1, 1, 1, 0),
              (2, 64, 64, 14, 14, 3, 3, 2, 1)]
    for shape in shapes:
        N, C, K, H, W, R, S, stride, pad = shape
        I, Wt, dO = make_inputs(shape, dtype, layer_id=55)
        L = conv.ConvLayer(*shape, dtype=dtype)
        try:
            L.set_outgrad(dO)
            L.set_weights(Wt)
            L.in_blk.fill_(float("nan"))
            conv.conv_bwd_data(L.h, L.out_blk, L.wt_blk, L.in_blk, L.ws)
            torch.cuda.synchronize()
            want = L.get_input().float().cpu().numpy()
            L.in_blk.fill_(float("nan"))
            conv.conv_bwd_data_noalloc(L.h, L.out_blk, L.wt_blk, L.in_blk)
            torch.cuda.synchronize()
            got = L.get_input().float().cpu().numpy()
        finally:
            L.close()
        # the same kernels on the same data: identical bits, and both within the parity bar
        assert np.array_equal(got, want), shape
        assert_close(got, oracle.bwd_data(dO, Wt, H, W, stride, pad), dtype, "bwd noalloc %s" % (shape,))
