"""GPU parity of the BB_SKIP_PADDED_QUERY_BLOCKS option (query blocks without a valid position
are not computed: O = 0, LSE = -inf, no gradient through them) against the oracle's
skip_padded_query_blocks reading, through the C ABI.  Tolerances as without the option."""
import numpy as np
import pytest

import bigbird_inputs as inp
import oracle
import paper_2007_14062_amd as bb
from gpu_util import device_qkv, device_tensor, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def check(t, ridx_h, b, g, w, scale, dtype, key_mask, mode=0, tag="", drop=None):
    torch = torch_mod()
    Q, K, V = device_qkv(t, dtype)
    dO = device_tensor(t, "dO", dtype)
    ridx = torch.from_numpy(np.ascontiguousarray(ridx_h)).to("cuda:0")
    km = torch.from_numpy(key_mask).to("cuda:0")
    flags = mode | bb.BB_SKIP_PADDED_QUERY_BLOCKS
    kw = dict(g=g, w=w, scale=scale, key_padding_mask=km, global_mode=flags)
    # O and LSE start from garbage: skipped rows must be written, not left alone
    O = torch.full_like(Q, 7.0)
    LSE = torch.full((Q.shape[0], Q.shape[1], Q.shape[2]), 3.0, dtype=torch.float32, device="cuda:0")
    if drop is None:
        bb.bigbird_attn_fwd(Q, K, V, ridx, O=O, LSE=LSE, **kw)
        grads = bb.bigbird_attn_bwd(Q, K, V, O, LSE, dO, ridx, **kw)
        Oo, Lo = oracle.attn_fwd(t["Q"], t["K"], t["V"], ridx_h, b, g, w, scale, key_mask=key_mask,
                                 global_mode=mode, skip_padded_query_blocks=True)
        ref = oracle.attn_bwd(t["Q"], t["K"], t["V"], t["dO"], ridx_h, b, g, w, scale, key_mask=key_mask,
                              global_mode=mode, skip_padded_query_blocks=True)
    else:
        p, seed = drop
        bb.bigbird_attn_fwd_dropout(Q, K, V, ridx, O=O, LSE=LSE, p_drop=p, seed=seed, **kw)
        grads = bb.bigbird_attn_bwd_dropout(Q, K, V, O, LSE, dO, ridx, p_drop=p, seed=seed, **kw)
        Oo, Lo = oracle.attn_fwd_dropout(t["Q"], t["K"], t["V"], ridx_h, b, g, w, scale, p, seed,
                                         key_mask=key_mask, global_mode=mode, skip_padded_query_blocks=True)
        ref = oracle.attn_bwd_dropout(t["Q"], t["K"], t["V"], t["dO"], ridx_h, b, g, w, scale, p, seed,
                                      key_mask=key_mask, global_mode=mode, skip_padded_query_blocks=True)
    torch.cuda.synchronize()
    fin = np.isfinite(Lo)
    Lh = to_host(LSE)
    assert (Lh[~fin] == -np.inf).all(), tag
    assert (to_host(O)[~fin] == 0).all(), tag
    err_o = np.abs(to_host(O) - Oo).max()
    err_l = np.abs(Lh[fin] - Lo[fin]).max()
    errs = [np.abs(to_host(x) - r_).max() for x, r_ in zip(grads, ref)]
    print(f"{tag}: rows skipped or empty {int((~fin).sum())}; max|dO|={err_o:.3e} max|dLSE|={err_l:.3e} grads {errs}")
    assert err_o <= TOL[dtype] and err_l <= TOL[dtype], tag
    assert all(np.isfinite(to_host(x)).all() for x in grads), tag
    assert max(errs) <= TOL[dtype], (tag, errs)
    assert (to_host(grads[0])[~fin] == 0).all(), tag   # dQ of rows that were not computed


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_suffix_padding_and_holes(dtype):
    """Aligned and unaligned valid lengths, a hole that covers whole blocks, a padded last global
    block; several batch entries so that skipped and computed items mix inside every wave."""
    B, H, n = 4, 3, 2048
    t = inp.make_tensors(B, H, n, 64, 401, dtype, with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 5)
    km = inp.lengths_to_key_mask(np.array([n, 1024, 1000, 192]), n)
    km[0, 640:832] = 0        # blocks 10..12 of the unpadded entry
    check(t, ridx, 64, 2, 3, 0.125, dtype, km, tag=f"skip {dtype}")


def test_leading_globals_wide_pattern_bf16():
    """Non-global rows of more than 16 key blocks (partial results + merge) and leading global
    blocks, one of which is fully padded in one batch entry."""
    B, H, n, g, w, r = 2, 2, 2048, 3, 15, 4
    t = inp.make_tensors(B, H, n, 64, 402, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 6, bb.BB_GLOBAL_LEADING)
    km = inp.lengths_to_key_mask(np.array([1500, n]), n)
    km[1, 64:128] = 0         # the second global block of entry 1
    check(t, ridx, 64, g, w, 0.125, "bf16", km, mode=bb.BB_GLOBAL_LEADING, tag="skip wide")


def test_with_dropout_bf16():
    B, H, n = 2, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 403, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 7)
    km = inp.lengths_to_key_mask(np.array([700, 320]), n)
    check(t, ridx, 64, 2, 3, 0.125, "bf16", km, tag="skip + dropout", drop=(0.1, 99))


def test_flag_without_mask_is_the_plain_call():
    torch = torch_mod()
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 404, "bf16")
    ridx_h = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 3)
    Q, K, V = device_qkv(t, "bf16")
    ridx = torch.from_numpy(ridx_h).to("cuda:0")
    O0, L0 = bb.bigbird_attn_fwd(Q, K, V, ridx, g=2, w=3, scale=0.125)
    O1, L1 = bb.bigbird_attn_fwd(Q, K, V, ridx, g=2, w=3, scale=0.125, global_mode=bb.BB_SKIP_PADDED_QUERY_BLOCKS)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(L0, L1)


def test_cfg3_shape_per_batch_entry():
    """The key-padding workload (B=8, H=12, n=4096) with the option: every batch entry, one head
    each, all rows, against the oracle."""
    torch = torch_mod()
    wl = inp.WORKLOADS["cfg3_key_padding"]
    t = inp.workload_tensors(wl)
    ridx_h = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    Q, K, V = device_qkv(t, "bf16")
    km = torch.from_numpy(t["key_mask"]).to("cuda:0")
    ridx = torch.from_numpy(ridx_h).to("cuda:0")
    O, LSE = bb.bigbird_attn_fwd(Q, K, V, ridx, g=wl.g, w=wl.w, scale=wl.scale, key_padding_mask=km,
                                 global_mode=bb.BB_SKIP_PADDED_QUERY_BLOCKS)
    torch.cuda.synchronize()
    worst_o = worst_l = 0.0
    for bi in range(wl.B):
        h = (5 * bi + 3) % wl.H
        sub = {k: t[k][bi:bi + 1, h:h + 1] for k in ("Q", "K", "V")}
        Oo, Lo = oracle.attn_fwd(sub["Q"], sub["K"], sub["V"], ridx_h[h:h + 1], wl.b, wl.g, wl.w, wl.scale,
                                 key_mask=t["key_mask"][bi:bi + 1], skip_padded_query_blocks=True)
        fin = np.isfinite(Lo[0, 0])
        Oh, Lh = to_host(O[bi, h]), to_host(LSE[bi, h])
        assert (Lh[~fin] == -np.inf).all() and (Oh[~fin] == 0).all()
        worst_o = max(worst_o, np.abs(Oh - Oo[0, 0]).max())
        worst_l = max(worst_l, np.abs(Lh[fin] - Lo[0, 0][fin]).max())
    print(f"cfg3 with skipped query blocks: max|dO|={worst_o:.3e} max|dLSE|={worst_l:.3e}")
    assert worst_o <= TOL["bf16"] and worst_l <= TOL["bf16"]
