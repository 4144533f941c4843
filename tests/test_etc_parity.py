"""GPU parity of the ETC construction (Sec. 2: extra global tokens in front of the sequence)
served by the existing entry points at b = 64.

A number of global tokens that is a multiple of 64 is the blocked pattern with that many leading
global blocks (BB_GLOBAL_LEADING), r = 0.  Any other number (App. E uses 230, 320, 430) is padded
by the caller to the next multiple of 64 with a key-padding mask over the unused slots; queries
in those slots are computed and ignored, and their dO is zero.  (Blocks of 84 or 169 tokens, as
in App. E, are not supported: BB_ERR_UNSUPPORTED.)
Tolerance: 2e-2 (bf16), outputs and gradients.
"""
import numpy as np
import pytest

import bigbird_inputs as inp
import oracle
import paper_2007_14062_amd as bb
from gpu_util import to_host

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _padded(x, n_global, pad, fill=0.0):
    """Insert `pad` rows after the first n_global rows of the sequence axis."""
    if pad == 0:
        return x
    shape = list(x.shape)
    shape[2] = pad
    return np.concatenate([x[:, :, :n_global], np.full(shape, fill, dtype=x.dtype), x[:, :, n_global:]], axis=2)


@pytest.mark.parametrize("n_global", [256, 230, 70])
def test_etc_forward_and_backward_through_the_blocked_entry_points(n_global):
    import torch
    assert torch.cuda.is_available()
    B, H, N, w, scale = 2, 2, 1536, 3, 0.125
    g = (n_global + 63) // 64
    pad = g * 64 - n_global
    n_etc = n_global + N
    t = inp.make_tensors(B, H, n_etc, 64, 900 + n_global, "bf16", with_dO=True)
    ref_O, ref_L = oracle.attn_fwd_etc(t["Q"], t["K"], t["V"], None, 64, w, n_global, scale)
    ref_g = oracle.attn_bwd_etc(t["Q"], t["K"], t["V"], t["dO"], None, 64, w, n_global, scale)

    dev = {}
    for name in ("Q", "K", "V", "dO"):
        x = _padded(t[name].astype(np.float32), n_global, pad)
        dev[name] = torch.from_numpy(x).to("cuda:0").to(torch.bfloat16)      # values are bf16 already: exact
    km = None
    if pad:
        m = np.ones((B, g * 64 + N), dtype=np.uint8)
        m[:, n_global:g * 64] = 0
        km = torch.from_numpy(m).to("cuda:0")
    empty = torch.zeros((H, (g * 64 + N) // 64, 0), dtype=torch.int32, device="cuda:0")
    O, LSE = bb.bigbird_attn_fwd(dev["Q"], dev["K"], dev["V"], empty, g=g, w=w, scale=scale,
                                 key_padding_mask=km, global_mode=bb.BB_GLOBAL_LEADING)
    dQ, dK, dV = bb.bigbird_attn_bwd(dev["Q"], dev["K"], dev["V"], O, LSE, dev["dO"], empty, g=g, w=w, scale=scale,
                                     key_padding_mask=km, global_mode=bb.BB_GLOBAL_LEADING)
    torch.cuda.synchronize()
    keep = np.r_[0:n_global, g * 64:g * 64 + N]       # the slots that hold tokens
    errs = {"O": np.abs(to_host(O)[:, :, keep] - ref_O).max(), "LSE": np.abs(to_host(LSE)[:, :, keep] - ref_L).max()}
    for name, got, want in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref_g):
        errs[name] = np.abs(to_host(got)[:, :, keep] - want).max()
    print(f"ETC n_global={n_global} (g={g} blocks, {pad} padded slots): " + " ".join(f"{k} {v:.3e}" for k, v in errs.items()))
    assert max(errs.values()) <= TOL, errs
    if pad:   # padded slots: no gradient reaches their keys
        assert (to_host(dK)[:, :, n_global:g * 64] == 0).all() and (to_host(dV)[:, :, n_global:g * 64] == 0).all()
