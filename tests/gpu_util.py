"""Helpers shared by the GPU parity tests: run one pass through the C ABI and
return the logical result; norms used for the comparison with the oracle."""
import numpy as np

from paper_1808_05567_amd import conv, inputs

TOL = {conv.CONV_F32: 1e-5, conv.CONV_BF16: 1e-2}  # rel-L2 bars of the parity target

# Per-element bars, |got - ref| <= rtol * |ref| + atol * rms(ref), beside the rel-L2 bar (which
# alone would let a handful of wrong elements hide in a million right ones).
#  fp32 results (fwd / bwd_data of fp32 layers, dW of both types): the inputs are exact, the only
#    error is fp32 accumulation.  A sum of n terms carries a rounding error of about
#    2^-24 * sqrt(n) * rms(partial sums); the longest chains here (4608 products per output,
#    at most 2^15 pixels per update chain before the fixed-order second stage) give a standard
#    deviation of at most 1e-6 * rms(ref) (measured rel-L2: 1e-7 ... 6e-7), so 1e-5 * rms(ref) is
#    more than ten standard deviations, and 1e-4 * |ref| covers elements far above the rms.
#  bf16 results: the fp32 sum c is within that fp32 bar of ref and is then rounded once to 8
#    significant bits, |round(c) - c| <= 2^-8 |c|: together 2^-8 |ref| + 2^-14 rms(ref).
ELEM = {conv.CONV_F32: (1e-4, 1e-5), conv.CONV_BF16: (2.0 ** -8, 2.0 ** -14)}


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    den = float(np.linalg.norm(ref))
    return float(np.linalg.norm(got - ref)) / (den if den > 0 else 1.0)


def error_norms(got, ref):
    """The error norms the paper's layer benchmark prints (Artifact Description, evaluation):
    Linf abs, L2 abs, Linf rel, L2 rel."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = np.abs(got - ref)
    nz = np.abs(ref) > 0
    return {"linf_abs": float(d.max()) if d.size else 0.0,
            "l2_abs": float(np.linalg.norm(d)),
            "linf_rel": float((d[nz] / np.abs(ref[nz])).max()) if nz.any() else 0.0,
            "l2_rel": rel_l2(got, ref)}


def assert_close(got, ref, dtype, what=""):
    """Both bars: rel-L2 over the tensor and the per-element bound, for a result of type
    `dtype` (CONV_F32 for every fp32 result, so also for the dW of a bf16 layer)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if got.size == 0:
        return
    rtol, atol = ELEM[dtype]
    rms = float(np.sqrt(np.mean(ref * ref)))
    d = np.abs(got - ref)
    bad = ~(d <= rtol * np.abs(ref) + atol * rms)      # (NaN counts as bad)
    r = rel_l2(got, ref)
    if r <= TOL[dtype] and not bad.any():
        return
    idx = np.unravel_index(int(np.argmax(np.where(np.isnan(d), np.inf, d))), d.shape)
    raise AssertionError(
        "%s: rel-L2 %.3e (bar %.0e); %d of %d elements beyond %.3g*|ref| + %.3g*rms (rms %.3e); "
        "norms %s; worst at %s: got %r ref %r" % (
            what, r, TOL[dtype], int(bad.sum()), bad.size, rtol, atol, rms,
            error_norms(got, ref), idx, float(got[idx]), float(ref[idx])))


def make_inputs(shape, dtype, layer_id=0, seed=0):
    N, C, K, H, W, R, S, stride, pad = shape
    ph, pw = pad if isinstance(pad, (tuple, list)) else (pad, pad)
    P = (H + 2 * ph - R) // stride + 1
    Q = (W + 2 * pw - S) // stride + 1
    I = inputs.gen_input(N, C, H, W, layer_id, seed)
    Wt = inputs.gen_weights(K, C, R, S, layer_id, seed)
    dO = inputs.gen_outgrad(N, K, P, Q, layer_id, seed)
    if dtype == conv.CONV_BF16:
        I, Wt, dO = (inputs.round_to_bf16(x) for x in (I, Wt, dO))
    return I, Wt, dO


def run_pass(L, which, I=None, Wt=None, dO=None):
    """Upload the logical operands of one pass, poison the output, run, unpack."""
    import torch
    # (the workspace too: a pass that left part of a partial copy unwritten must not pass by
    # what the allocator happened to hold there; all-ones bytes are NaN in both types)
    L.ws.fill_(0xFF)
    if which == "fwd":
        L.set_input(I)
        L.set_weights(Wt)
        L.out_blk.fill_(float("nan"))
        L.fwd()
        out = L.get_output()
    elif which == "bwd":
        L.set_outgrad(dO)
        L.set_weights(Wt)
        L.in_blk.fill_(float("nan"))
        L.bwd_data()
        out = L.get_input()
    else:
        L.set_input(I)
        L.set_outgrad(dO)
        L.dwt_blk.fill_(float("nan"))
        L.upd()
        out = L.get_dweights()
    torch.cuda.synchronize()
    return out.float().cpu().numpy()
