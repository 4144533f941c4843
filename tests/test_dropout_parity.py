"""GPU parity of attention dropout (bigbird_attn_fwd_dropout / bigbird_attn_bwd_dropout) against
the fp64 oracle of oracle/dropout.py, through the C ABI.

The keep mask is integer work (a counter-based generator both sides implement): it is compared
bit for bit on the CPU in tests/test_dropout_host.py; here a wrong mask in any kernel shows as an
error of the size of the outputs themselves.  Tolerances are those of the undropped passes:
fp32 1e-4 (outputs and gradients), bf16 2e-2.
"""
import numpy as np
import pytest

import bigbird_inputs as inp
import oracle
import paper_2007_14062_amd as bb
from gpu_util import device_qkv, device_tensor, sample_rows, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def run(t, ridx_h, g, w, scale, p, seed, dtype, key_mask=None, mode=0, backward=True):
    torch = torch_mod()
    Q, K, V = device_qkv(t, dtype)
    ridx = torch.from_numpy(np.ascontiguousarray(ridx_h)).to("cuda:0")
    km = None if key_mask is None else torch.from_numpy(key_mask).to("cuda:0")
    O, LSE = bb.bigbird_attn_fwd_dropout(Q, K, V, ridx, g=g, w=w, scale=scale, p_drop=p, seed=seed,
                                         key_padding_mask=km, global_mode=mode)
    grads = None
    if backward:
        dO = device_tensor(t, "dO", dtype)
        grads = bb.bigbird_attn_bwd_dropout(Q, K, V, O, LSE, dO, ridx, g=g, w=w, scale=scale, p_drop=p,
                                            seed=seed, key_padding_mask=km, global_mode=mode)
    torch.cuda.synchronize()
    return O, LSE, grads


def check(t, ridx_h, b, g, w, scale, p, seed, dtype, key_mask=None, mode=0, tag="", backward=True):
    O, LSE, grads = run(t, ridx_h, g, w, scale, p, seed, dtype, key_mask, mode, backward)
    Oo, Lo = oracle.attn_fwd_dropout(t["Q"], t["K"], t["V"], ridx_h, b, g, w, scale, p, seed,
                                     key_mask=key_mask, global_mode=mode)
    fin = np.isfinite(Lo)
    err_o = np.abs(to_host(O) - Oo).max()
    err_l = np.abs(to_host(LSE)[fin] - Lo[fin]).max() if fin.any() else 0.0
    assert (to_host(LSE)[~fin] == -np.inf).all()
    msg = f"{tag}: max|dO|={err_o:.3e} max|dLSE|={err_l:.3e}"
    assert err_o <= TOL[dtype] and err_l <= TOL[dtype], msg
    if backward:
        ref = oracle.attn_bwd_dropout(t["Q"], t["K"], t["V"], t["dO"], ridx_h, b, g, w, scale, p, seed,
                                      key_mask=key_mask, global_mode=mode)
        errs = [np.abs(to_host(x) - r).max() for x, r in zip(grads, ref)]
        msg += f" max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} max|ddV|={errs[2]:.3e}"
        assert all(np.isfinite(to_host(x)).all() for x in grads), tag
        assert max(errs) <= TOL[dtype], msg
    print(msg)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_base_pattern(dtype):
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 301, dtype, with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 3)
    check(t, ridx, 64, 2, 3, 0.125, 0.1, 0x1234_5678_9ABC_DEF0, dtype, tag=f"dropout base {dtype}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_padding_inside_blocks_and_leading_globals(dtype):
    """Two batch entries, unaligned valid lengths (partly padded blocks, fully padded blocks, a
    global block without a valid key), three leading global blocks, window 5."""
    B, H, n, g, w, r = 2, 3, 640, 3, 5, 2
    t = inp.make_tensors(B, H, n, 64, 302, dtype, with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 9, bb.BB_GLOBAL_LEADING)
    km = inp.lengths_to_key_mask(np.array([n - 200, 100]), n)
    check(t, ridx, 64, g, w, 0.2, 0.25, 7, dtype, key_mask=km, mode=bb.BB_GLOBAL_LEADING,
          tag=f"dropout padding {dtype}")


def test_long_rows_and_wide_patterns_bf16():
    """Rows that are cut into slices whose partial results are merged afterwards: global rows of
    more than 64 key blocks, and non-global rows of more than 16 (the dropout scale is applied by
    the merge); global key columns cut into slices in the backward."""
    B, H, n = 1, 1, 8192
    t = inp.make_tensors(B, H, n, 64, 303, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 11)
    check(t, ridx, 64, 2, 3, 0.125, 0.1, 42, "bf16", tag="dropout n=8192")
    B, H, n, g, w, r = 1, 2, 2048, 2, 15, 4
    t = inp.make_tensors(B, H, n, 64, 304, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 12)
    check(t, ridx, 64, g, w, 0.125, 0.5, 43, "bf16", tag="dropout wide pattern")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rate_zero_is_the_plain_call_bit_for_bit(dtype):
    torch = torch_mod()
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 305, dtype, with_dO=True)
    ridx_h = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 3)
    O0, L0, G0 = run(t, ridx_h, 2, 3, 0.125, 0.0, 5, dtype)
    Q, K, V = device_qkv(t, dtype)
    ridx = torch.from_numpy(ridx_h).to("cuda:0")
    O1, L1 = bb.bigbird_attn_fwd(Q, K, V, ridx, g=2, w=3, scale=0.125)
    G1 = bb.bigbird_attn_bwd(Q, K, V, O1, L1, device_tensor(t, "dO", dtype), ridx, g=2, w=3, scale=0.125)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(L0, L1)
    assert all(torch.equal(a, c) for a, c in zip(G0, G1))


def test_same_seed_same_result_other_seed_other_mask():
    torch = torch_mod()
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 306, "bf16", with_dO=True)
    ridx_h = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 3)
    a = run(t, ridx_h, 2, 3, 0.125, 0.1, 1, "bf16")
    b_ = run(t, ridx_h, 2, 3, 0.125, 0.1, 1, "bf16")
    c = run(t, ridx_h, 2, 3, 0.125, 0.1, 2, "bf16")
    assert torch.equal(a[0], b_[0]) and all(torch.equal(x, y) for x, y in zip(a[2], b_[2]))
    assert torch.equal(a[1], c[1])                      # LSE does not see the mask
    assert not torch.equal(a[0], c[0])


def test_training_shape_sampled_rows_and_gradient_properties():
    """The forward + backward workload (B=2, H=12, n=4096) with dropout 0.1: sampled output rows of
    several slices against the oracle; gradients of one whole slice against the oracle."""
    torch = torch_mod()
    wl = inp.WORKLOADS["cfg4_fwd_bwd"]
    t = inp.workload_tensors(wl)
    ridx_h = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    p, seed = 0.1, 20200728
    O, LSE, grads = run(t, ridx_h, wl.g, wl.w, wl.scale, p, seed, "bf16")
    rng = np.random.default_rng(5)
    worst = 0.0
    for bi, h in ((0, 0), (1, 11), (0, 7)):
        rows = sample_rows(wl.n // wl.b, wl.b, rng)
        Or, Lr = oracle.attn_fwd_dropout_rows(t["Q"], t["K"], t["V"], ridx_h, wl.b, wl.g, wl.w, wl.scale,
                                              p, seed, bi, h, rows)
        worst = max(worst, np.abs(to_host(O[bi, h])[rows] - Or).max(), np.abs(to_host(LSE[bi, h])[rows] - Lr).max())
    assert worst <= TOL["bf16"], worst
    # one slice in full: the oracle on a one-slice problem whose slice number is the same
    bi, h = 1, 5
    sub = {k: v[bi:bi + 1, h:h + 1] for k, v in t.items() if not k.endswith("_bits")}
    bh = bi * wl.H + h
    from oracle.dropout import keep_mask, dropout_scale
    M = np.where(keep_mask(seed, bh, wl.n, p), dropout_scale(p), 0.0)
    A = oracle.dense_mask(ridx_h[h], wl.n, wl.b, wl.g, wl.w)
    Qf, Kf, Vf, dOf = (np.asarray(sub[x][0, 0], dtype=np.float64) for x in ("Q", "K", "V", "dO"))
    S = np.where(A, wl.scale * (Qf @ Kf.T), -np.inf)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    dP = M * (dOf @ Vf.T)
    dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
    ref = (wl.scale * dS @ Kf, wl.scale * dS.T @ Qf, (P * M).T @ dOf)
    errs = [np.abs(to_host(x[bi, h]) - r).max() for x, r in zip(grads, ref)]
    print(f"dropout cfg4: forward rows {worst:.3e}; slice ({bi},{h}) gradients {errs}")
    assert max(errs) <= TOL["bf16"], errs
