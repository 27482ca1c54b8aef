"""Host-side checks of the C-ABI library: it loads, exports every symbol the
public header declares, plans on a machine without a GPU, and rejects bad
arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_1808_05567_amd import conv, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "conv_mi355x.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = conv.load()
    names = declared_symbols()
    assert set(names) == set(conv.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_query_sizes_and_output_extent():
    for l in inputs.TABLE_I:
        for dt, es, v in ((conv.CONV_F32, 4, 4), (conv.CONV_BF16, 2, 8)):
            h = conv.conv_create(256, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad, dt)
            i = conv.conv_query(h)
            assert (i.P, i.Q, i.vlen) == (l.P, l.Q, v)
            Cp, Kp = -(-l.C // v) * v, -(-l.K // v) * v
            assert (i.Cp, i.Kp, i.Cb, i.Kb) == (Cp, Kp, Cp // v, Kp // v)
            assert i.in_bytes == 256 * Cp * l.H * l.W * es
            assert i.out_bytes == 256 * Kp * l.P * l.Q * es
            assert i.wt_bytes == Cp * Kp * l.R * l.S * es
            assert i.dwt_bytes == Cp * Kp * l.R * l.S * 4
            conv.conv_destroy(h)


@pytest.mark.parametrize("bad", [
    dict(N=0), dict(C=0), dict(K=-1), dict(H=0), dict(R=0), dict(stride=0), dict(pad=-1),
    dict(dtype=7), dict(H=2, W=2, R=5, S=5, pad=1),
])
def test_bad_descriptors_are_rejected(bad):
    d = dict(N=2, C=8, K=8, H=8, W=8, R=3, S=3, stride=1, pad=1, dtype=0)
    d.update(bad)
    with pytest.raises(conv.ConvError) as e:
        conv.conv_create(**d)
    assert e.value.status == conv.CONV_EINVAL


def test_null_and_misaligned_pointers_are_rejected_without_launch():
    lib = conv.load()
    h = conv.conv_create(2, 8, 8, 8, 8, 3, 3, 1, 1, 0)
    assert lib.conv_fwd(h, None, None, None, None, None) == conv.CONV_EINVAL
    assert lib.conv_fwd(None, 16, 16, 16, None, None) == conv.CONV_EINVAL
    assert lib.conv_fwd(h, 16, 16, 24, None, None) == conv.CONV_EINVAL  # 24 is not 16-aligned
    assert lib.conv_bwd_data(h, 16, 16, 16, None, None) == conv.CONV_EWORKSPACE
    assert lib.conv_upd(h, 16, 16, 16, None, None) == conv.CONV_EWORKSPACE
    assert lib.conv_pack_in(h, None, 16, None) == conv.CONV_EINVAL
    assert lib.conv_query(h, None) == conv.CONV_EINVAL
    assert lib.conv_create(None, None) == conv.CONV_EINVAL
    assert conv.status_str(conv.CONV_EUNSUPPORTED) == "unsupported problem"
    buf = ctypes.create_string_buffer(256)
    assert lib.conv_describe(h, 9, buf, 256) == conv.CONV_EINVAL
    conv.conv_destroy(h)
    # the shader-clock sampler: bounded workgroup count and duration, checked before any launch
    assert lib.conv_ceiling_shader_clock(8, 100, None, None) == conv.CONV_EINVAL
    assert lib.conv_ceiling_shader_clock(0, 100, 16, None) == conv.CONV_EINVAL
    assert lib.conv_ceiling_shader_clock(257, 100, 16, None) == conv.CONV_EINVAL
    assert lib.conv_ceiling_shader_clock(8, 0, 16, None) == conv.CONV_EINVAL
    assert lib.conv_ceiling_shader_clock(8, 1000001, 16, None) == conv.CONV_EINVAL


def test_every_table1_layer_is_planned():
    """Planning is host-only: all passes of the benchmark layers must have a kernel."""
    for l in inputs.TABLE_I:
        for dt in (conv.CONV_F32, conv.CONV_BF16):
            h = conv.conv_create(256, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad, dt)
            for which in (conv.PASS_FWD, conv.PASS_BWD_DATA, conv.PASS_UPD):
                assert conv.conv_describe(h, which)
            conv.conv_destroy(h)
