"""Host-side checks of the planner (no GPU): every plan it hands out must fit the
machine (LDS per workgroup, a non-empty grid, a workspace that covers the partial
results), for the benchmark layers and for a seeded sweep of other descriptors, and
the kernel families must be chosen where they apply."""
import re

import numpy as np
import pytest

from paper_1808_05567_amd import conv, inputs

LDS_PER_CU = 160 * 1024


def _plans(shape, dt):
    h = conv.conv_create(*shape, dt)
    out = {}
    try:
        info = conv.conv_query(h)
        for which in (conv.PASS_FWD, conv.PASS_BWD_DATA, conv.PASS_UPD):
            # (every pass has a plan: a tiled kernel, or the untiled direct one)
            out[which] = conv.conv_describe(h, which)
    finally:
        conv.conv_destroy(h)
    return info, out


def _field(text, name):
    m = re.search(r"\b%s=(\d+)" % name, text)
    assert m, (name, text)
    return int(m.group(1))


def _tiled(text):
    return not text.startswith("direct ")


def _check(info, plans):
    for which, text in plans.items():
        if _tiled(text):
            assert 0 < _field(text, "lds") <= LDS_PER_CU, text
        else:
            assert _field(text, "lds") <= 64 * 1024, text  # static LDS only
        assert 1 <= _field(text, "grid") < 2 ** 31, text
    assert info.upd_splits >= 1
    if _tiled(plans[conv.PASS_UPD]):
        # every partial copy of dW the update kernel writes fits the workspace
        assert info.workspace_bytes >= info.upd_splits * info.dwt_bytes
    else:
        assert info.upd_splits == 1  # the direct kernel writes dW itself
    if _tiled(plans[conv.PASS_BWD_DATA]):
        # the transformed weights of the backward pass live in the workspace
        assert info.workspace_bytes >= 16


@pytest.mark.parametrize("dt", [conv.CONV_F32, conv.CONV_BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 256])
def test_inception_v3_plans_fit_the_machine(N, dt):
    """Every shape of the second workload has a tiled kernel in all three passes (rectangular filters, per-axis
    padding, unpadded stride 2, rows wider than an update band)."""
    assert len(inputs.INCEPTION_V3) == 43
    for l in inputs.INCEPTION_V3:
        info, plans = _plans((N, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad), dt)
        _check(info, plans)
        assert all(_tiled(p) for p in plans.values()), (l.id, plans)
        assert (info.P, info.Q) == (l.P, l.Q)


def test_update_of_tall_filters_and_wide_rows():
    def upd(shape, dt=conv.CONV_F32):
        return _plans(shape, dt)[1][conv.PASS_UPD]
    # 7x1 and 1x7: one launch; 5x5: one launch per filter row
    assert "RS=7x1" in upd((4, 64, 64, 17, 17, 7, 1, 1, (3, 0))) and "launches=1" in upd((4, 64, 64, 17, 17, 7, 1, 1, (3, 0)))
    assert "launches=1" in upd((4, 64, 64, 17, 17, 1, 7, 1, (0, 3)))
    assert "RS=1x5" in upd((4, 48, 64, 35, 35, 5, 5, 1, 2)) and "launches=5" in upd((4, 48, 64, 35, 35, 5, 5, 1, 2))
    # 147-wide rows: strips of output columns, one launch each
    assert "launches=3" in upd((2, 32, 64, 147, 147, 3, 3, 1, 1))
    assert "launches=2" in upd((2, 32, 64, 147, 147, 3, 3, 1, 1), conv.CONV_BF16)


@pytest.mark.parametrize("dt", [conv.CONV_F32, conv.CONV_BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 2, 256])
def test_table1_plans_fit_the_machine(N, dt):
    for l in inputs.TABLE_I:
        info, plans = _plans((N, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad), dt)
        _check(info, plans)
        assert all(_tiled(p) for p in plans.values()), (l.id, plans)


def test_seeded_descriptor_sweep_plans_fit_the_machine():
    rng = np.random.default_rng(180805567)
    planned = 0
    for _ in range(400):
        R = int(rng.choice([1, 1, 3, 3, 7]))
        stride = int(rng.choice([1, 1, 2, 3]))
        pad = int(rng.integers(0, R // 2 + 1))
        H = int(rng.integers(max(R, 1), 70))
        W = int(rng.integers(max(R, 1), 70))
        C = int(rng.choice([1, 3, 4, 8, 20, 64, 100, 128, 256, 264, 512, 1030]))
        K = int(rng.choice([1, 8, 12, 64, 72, 128, 256, 320, 1024, 2048]))
        N = int(rng.choice([1, 2, 3, 16, 64]))
        for dt in (conv.CONV_F32, conv.CONV_BF16):
            info, plans = _plans((N, C, K, H, W, R, R, stride, pad), dt)
            _check(info, plans)
            planned += sum(_tiled(p) for p in plans.values())
    assert planned > 1500  # most passes have a tiled kernel


def test_seeded_rectangular_sweep_plans_fit_the_machine():
    """Rectangular filters, padding per axis, images up to 300 wide (column strips)."""
    rng = np.random.default_rng(1808055670)
    planned = 0
    for _ in range(300):
        R, S = [(1, 7), (7, 1), (1, 3), (3, 1), (5, 5), (3, 3), (1, 5), (5, 1), (3, 7)][int(rng.integers(0, 9))]
        stride = int(rng.choice([1, 1, 1, 2]))
        ph, pw = int(rng.integers(0, R // 2 + 2)), int(rng.integers(0, S // 2 + 2))
        H = int(rng.integers(R, 40))
        W = int(rng.integers(S, 300 if rng.integers(0, 4) == 0 else 40))
        C = int(rng.choice([3, 8, 32, 48, 160, 192, 384]))
        K = int(rng.choice([8, 32, 64, 96, 160, 192, 448]))
        N = int(rng.choice([1, 2, 32]))
        for dt in (conv.CONV_F32, conv.CONV_BF16):
            info, plans = _plans((N, C, K, H, W, R, S, stride, (ph, pw)), dt)
            _check(info, plans)
            assert (info.P, info.Q) == ((H + 2 * ph - R) // stride + 1, (W + 2 * pw - S) // stride + 1)
            planned += sum(_tiled(p) for p in plans.values())
    assert planned > 1000  # (tiled kernels; the rest run on the direct ones)


def test_kernel_families_are_chosen_where_they_apply():
    # fp32 1x1 with 256 channels on one side: eight-wave kernel on the flat pixel list
    _, p = _plans((256, 256, 1024, 14, 14, 1, 1, 1, 0), conv.CONV_F32)
    assert p[conv.PASS_UPD].startswith("upd_1x1 dt=0") and "in x out" in p[conv.PASS_UPD]
    _, p = _plans((256, 64, 256, 56, 56, 1, 1, 1, 0), conv.CONV_F32)
    assert p[conv.PASS_UPD].startswith("upd_1x1 dt=0") and "out x in" in p[conv.PASS_UPD]
    # ... below that, the four-wave kernel
    _, p = _plans((256, 64, 64, 56, 56, 1, 1, 1, 0), conv.CONV_F32)
    assert p[conv.PASS_UPD].startswith("upd dt=0")
    # bf16 1x1: flat pixel list at every width
    for C, K in ((64, 64), (64, 256), (1024, 2048)):
        _, p = _plans((256, C, K, 14, 14, 1, 1, 1, 0), conv.CONV_BF16)
        assert p[conv.PASS_UPD].startswith("upd_1x1 dt=1")
    # 3x3 stride 1: band kernel (fp32), row kernel (bf16)
    _, p = _plans((256, 256, 256, 14, 14, 3, 3, 1, 1), conv.CONV_F32)
    assert p[conv.PASS_UPD].startswith("upd_bands")
    _, p = _plans((256, 256, 256, 14, 14, 3, 3, 1, 1), conv.CONV_BF16)
    assert p[conv.PASS_UPD].startswith("upd_rows")
    # one input channel block, fp32: filter-row kernel; backward: all classes in one launch
    _, p = _plans((256, 3, 64, 224, 224, 7, 7, 2, 3), conv.CONV_F32)
    assert p[conv.PASS_UPD].startswith("upd_c4")
    assert "launches=1" in p[conv.PASS_BWD_DATA]
    # 3x3 stride 2 backward: one launch per residue class
    _, p = _plans((4, 64, 64, 14, 14, 3, 3, 2, 1), conv.CONV_F32)
    assert "launches=4" in p[conv.PASS_BWD_DATA]
    # small minibatch, long reduction: the forward reduction is split
    _, p = _plans((1, 512, 512, 7, 7, 3, 3, 1, 1), conv.CONV_F32)
    assert _field(p[conv.PASS_FWD], "ksplit") > 1


def _describe_all(h):
    return [conv.conv_describe(h, w) for w in (conv.PASS_FWD, conv.PASS_BWD_DATA, conv.PASS_UPD)]


def test_minibatch_chunks_on_request():
    shape = (10, 64, 64, 14, 14, 3, 3, 1, 1)
    h = conv.conv_create_chunked(*shape, 4)
    try:
        info = conv.conv_query(h)
        assert all(t.startswith("chunks=3 images=4: ") for t in _describe_all(h))
        # one dW per chunk behind the chunks' own workspace
        assert info.upd_splits == 3 and info.workspace_bytes >= 3 * info.dwt_bytes
    finally:
        conv.conv_destroy(h)
    # a bound the minibatch already meets changes nothing
    h, g = conv.conv_create_chunked(*shape, 10), conv.conv_create(*shape)
    try:
        assert _describe_all(h) == _describe_all(g)
    finally:
        conv.conv_destroy(h)
        conv.conv_destroy(g)
    with pytest.raises(conv.ConvError) as e:
        conv.conv_create_chunked(*shape, 0)
    assert e.value.status == conv.CONV_EINVAL


@pytest.mark.parametrize("dt", [conv.CONV_F32, conv.CONV_BF16], ids=["f32", "bf16"])
def test_tensors_beyond_32bit_offsets_run_in_chunks_on_tiled_kernels(dt):
    """4 GB and more in one tensor, or more linear rows than the kernels' exact divisions
    reach: the planner splits the minibatch so that every pass keeps its tiled kernel."""
    for shape in ((1024 if dt == conv.CONV_BF16 else 512, 64, 64, 224, 224, 3, 3, 1, 1),
                  (8192 if dt == conv.CONV_BF16 else 4096, 64, 256, 56, 56, 1, 1, 1, 0),
                  (300000, 8, 8, 14, 14, 3, 3, 1, 1)):
        info, plans = _plans(shape, dt)
        _check(info, plans)
        assert all(_tiled(p) for p in plans.values()), (shape, plans)
        assert plans[conv.PASS_FWD].startswith("chunks=") and plans[conv.PASS_BWD_DATA].startswith("chunks=")
    # the benchmark's own sizes are never chunked
    for l in inputs.TABLE_I:
        _, plans = _plans((256, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad), dt)
        assert not any(p.startswith("chunks=") for p in plans.values())


def test_extreme_descriptors_plan_quickly_and_within_bounds():
    """Very tall images, millions of images, thousands of channels under a large filter:
    planning time must not grow with N*P, and the update's partial copies must not dwarf
    the tensors (such plans are left to the direct kernel, which needs no workspace)."""
    import time
    for shape, dt in (((77948, 3, 4, 16060, 9, 7, 7, 3, (2, 5)), conv.CONV_F32),
                      ((2000000, 8, 8, 9, 9, 3, 3, 1, 1), conv.CONV_BF16),
                      ((2, 5585, 5431, 330, 2214, 7, 7, 3, (6, 1)), conv.CONV_F32),
                      ((19, 5746, 6495, 325, 972, 7, 1, 1, (6, 0)), conv.CONV_F32)):
        t0 = time.time()
        info, plans = _plans(shape, dt)
        assert time.time() - t0 < 20.0, shape
        _check(info, plans)
        assert info.workspace_bytes <= max(2 * (info.in_bytes + info.out_bytes), 8e9) + 64 * info.dwt_bytes


@pytest.mark.parametrize("bad", [dict(C=2 ** 31 - 1), dict(K=2 ** 31 - 1), dict(W=2 ** 31 - 1),
                                 dict(H=2 ** 31 - 1), dict(N=2 ** 31 - 1), dict(stride=2 ** 31 - 1),
                                 dict(R=2 ** 20, H=2 ** 21), dict(pad=2 ** 30),
                                 dict(N=2 ** 24, C=2 ** 12, H=2 ** 12, W=2 ** 12)],
                         ids=lambda b: ",".join("%s=%d" % kv for kv in b.items()))
def test_extents_beyond_the_size_limits_are_refused_not_miscomputed(bad):
    """Extents near INT32_MAX once left the planner's int arithmetic (a garbage plan, a division
    by zero, half a minute inside conv_create): they are bounded in 64-bit before any planning."""
    import time
    d = dict(N=2, C=8, K=8, H=8, W=8, R=3, S=3, stride=1, pad=1, dtype=0)
    d.update(bad)
    t0 = time.time()
    with pytest.raises(conv.ConvError) as e:
        conv.conv_create(**d)
    assert e.value.status == conv.CONV_EUNSUPPORTED
    assert time.time() - t0 < 1.0


def test_large_but_legal_extents_plan_within_bounds():
    """Just inside the limits: a plan comes back at once, every figure positive."""
    import time
    for shape in ((1, 2 ** 20, 8, 1, 1, 1, 1, 1, 0), (2 ** 24, 4, 4, 1, 1, 1, 1, 1, 0),
                  (1, 4, 4, 2 ** 18, 2 ** 18, 3, 3, 1, 1), (1, 8, 8, 70000, 9, 5, 3, 60000, (0, 1)),
                  (3, 8, 8, 9, 40000, 3, 3, 1, 1)):
        t0 = time.time()
        info, plans = _plans(shape, conv.CONV_F32)
        assert time.time() - t0 < 5.0, shape
        _check(info, plans)
        assert info.P >= 1 and info.Q >= 1 and info.in_bytes > 0 and info.out_bytes > 0


def test_checked_workspace_entry_points_refuse_a_short_buffer():
    """conv_*_ws return CONV_EWORKSPACE before anything is launched (host only here: the
    pointers are never dereferenced because the size check comes first)."""
    lib = conv.load()
    h = conv.conv_create(4, 64, 64, 14, 14, 3, 3, 1, 1, 0)
    try:
        need = conv.conv_query(h).workspace_bytes
        assert need > 0
        assert lib.conv_bwd_data_ws(h, 16, 16, 16, 16, 0, None) == conv.CONV_EWORKSPACE
        assert lib.conv_upd_ws(h, 16, 16, 16, 16, need // 2, None) == conv.CONV_EWORKSPACE
        assert lib.conv_upd_ws(None, 16, 16, 16, 16, need, None) == conv.CONV_EINVAL
    finally:
        conv.conv_destroy(h)
