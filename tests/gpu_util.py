"""Helpers shared by the GPU parity tests: run one pass through the C ABI and
return the logical result; norms used for the comparison with the oracle."""
import numpy as np

from paper_1808_05567_amd import conv, inputs

TOL = {conv.CONV_F32: 1e-5, conv.CONV_BF16: 1e-2}  # rel-L2 bars of the parity target


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    den = float(np.linalg.norm(ref))
    return float(np.linalg.norm(got - ref)) / (den if den > 0 else 1.0)


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
