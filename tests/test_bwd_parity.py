"""GPU parity of bigbird_attn_bwd (bf16 storage, fp32 gradients) against the fp64 oracle.

The backward consumes the GPU forward's own O and LSE, as a training step would.
Tolerance: max abs error of dQ, dK, dV <= 2e-2.
"""
import numpy as np
import pytest

import bigbird_inputs as inp
import oracle
import paper_2007_14062_amd as bb
from gpu_util import device_qkv, device_tensor, to_host

pytestmark = pytest.mark.gpu

TOL = 2e-2


def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def run_fwd_bwd(t, rand_idx, g, w, scale, key_mask=None, mode=0):
    torch = torch_mod()
    Q, K, V = device_qkv(t, "bf16")
    dO = device_tensor(t, "dO", "bf16")
    ridx = torch.from_numpy(np.ascontiguousarray(rand_idx)).to("cuda:0")
    km = None if key_mask is None else torch.from_numpy(key_mask).to("cuda:0")
    O, LSE = bb.bigbird_attn_fwd(Q, K, V, ridx, g=g, w=w, scale=scale, key_padding_mask=km,
                                 global_mode=mode)
    dQ, dK, dV = bb.bigbird_attn_bwd(Q, K, V, O, LSE, dO, ridx, g=g, w=w, scale=scale,
                                     key_padding_mask=km, global_mode=mode)
    torch.cuda.synchronize()
    return dQ, dK, dV


def check_full(t, rand_idx, b, g, w, scale, key_mask=None, mode=0, tag=""):
    dQ, dK, dV = run_fwd_bwd(t, rand_idx, g, w, scale, key_mask, mode)
    rQ, rK, rV = oracle.attn_bwd(t["Q"], t["K"], t["V"], t["dO"], rand_idx, b, g, w, scale,
                                 key_mask=key_mask, global_mode=mode)
    errs = [np.abs(to_host(x) - r).max() for x, r in ((dQ, rQ), (dK, rK), (dV, rV))]
    print(f"{tag}: max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} max|ddV|={errs[2]:.3e} "
          f"(|dQ|max={np.abs(rQ).max():.2f} |dK|max={np.abs(rK).max():.2f} |dV|max={np.abs(rV).max():.2f})")
    assert all(np.isfinite(to_host(x)).all() for x in (dQ, dK, dV)), tag
    assert max(errs) <= TOL, (tag, errs)
    return dQ, dK, dV


def test_small_full_parity():
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 103, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 3)
    check_full(t, ridx, 64, 2, 3, 0.125, tag="bwd n=1024")


def test_ragged_shapes_leading_globals():
    B, H, n, g, w, r = 2, 3, 640, 3, 5, 2
    t = inp.make_tensors(B, H, n, 64, 17, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 9, bb.BB_GLOBAL_LEADING)
    check_full(t, ridx, 64, g, w, 0.2, mode=bb.BB_GLOBAL_LEADING, tag="bwd ragged")


def test_full_coverage_long_lists():
    """Window over every block: every row and every column is attended by all blocks."""
    B, H, n = 1, 2, 1280
    nb = n // 64
    t = inp.make_tensors(B, H, n, 64, 18, "bf16", with_dO=True)
    empty = np.full((H, nb, 0), -1, dtype=np.int32)
    check_full(t, empty, 64, 0, 2 * nb - 1, 0.125, tag="bwd full coverage (window)")
    check_full(t, empty, 64, nb, 1, 0.125, tag="bwd full coverage (all global)")


@pytest.mark.parametrize("g,w,r", [(0, 1, 0), (1, 1, 0), (0, 3, 2), (2, 3, 0), (1, 7, 4)])
def test_degenerate_patterns(g, w, r):
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 19, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 3)
    check_full(t, ridx, 64, g, w, 0.125, tag=f"bwd g{g} w{w} r{r}")


def test_summarisation_encoder_length_3072():
    """nb = 48 (not a power of two; six slices per global row and column), B*H = 10."""
    B, H, n, g, w, r = 1, 10, 3072, 2, 3, 3
    t = inp.make_tensors(B, H, n, 64, 57, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 13)
    dQ, dK, dV = run_fwd_bwd(t, ridx, g, w, 0.125)
    for h in (0, 9):
        sub = {k: v[:, h:h + 1] for k, v in t.items() if k in ("Q", "K", "V", "dO")}
        rQ, rK, rV = oracle.attn_bwd(sub["Q"], sub["K"], sub["V"], sub["dO"], ridx[h:h + 1], 64, g, w, 0.125)
        errs = [np.abs(to_host(x)[:, h:h + 1] - r_).max() for x, r_ in ((dQ, rQ), (dK, rK), (dV, rV))]
        print(f"bwd n=3072 head {h}: max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} max|ddV|={errs[2]:.3e}")
        assert max(errs) <= TOL, (h, errs)


def test_long_sequence_one_head_in_full():
    """n = 8192 (nb = 128): sixteen slices per global row and per global key column go through
    the fixed-order reduction; one of the three heads is compared in full."""
    B, H, n, g, w, r = 1, 3, 8192, 2, 3, 3
    t = inp.make_tensors(B, H, n, 64, 91, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 19)
    dQ, dK, dV = run_fwd_bwd(t, ridx, g, w, 0.125)
    h = 2
    sub = {k: v[:, h:h + 1] for k, v in t.items() if k in ("Q", "K", "V", "dO")}
    rQ, rK, rV = oracle.attn_bwd(sub["Q"], sub["K"], sub["V"], sub["dO"], ridx[h:h + 1], 64, g, w, 0.125)
    errs = [np.abs(to_host(x)[:, h:h + 1] - r_).max() for x, r_ in ((dQ, rQ), (dK, rK), (dV, rV))]
    print(f"bwd n=8192 head {h}: max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} max|ddV|={errs[2]:.3e}")
    assert max(errs) <= TOL, errs


def test_single_block_sequence():
    t = inp.make_tensors(2, 1, 64, 64, 20, "bf16", with_dO=True)
    empty = np.full((1, 1, 0), -1, dtype=np.int32)
    check_full(t, empty, 64, 1, 1, 0.125, tag="bwd nb=1 global")
    check_full(t, empty, 64, 0, 1, 0.125, tag="bwd nb=1 window")


def test_table_with_duplicates_and_negative_entries():
    B, H, n, g, w, r = 1, 2, 1024, 2, 3, 4
    t = inp.make_tensors(B, H, n, 64, 21, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 5)
    ridx[0, 5] = [-1, 9, 9, 12]
    ridx[0, 6] = [6, 0, 7, 3]
    ridx[1, 8] = [-1, -1, -1, -1]
    ridx[1, 9] = [15, 2, 2, 2]
    check_full(t, ridx, 64, g, w, 0.125, tag="bwd dirty table")


def test_key_padding_gradients():
    B, H, n, g, w, r = 3, 2, 1024, 2, 3, 3
    t = inp.make_tensors(B, H, n, 64, 22, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 6)
    km = np.ones((B, n), dtype=np.uint8)
    km[0, 700:] = 0
    km[1, :64] = 0
    km[1, 300:309] = 0
    km[1, 640:768] = 0
    km[2, :] = 0
    dQ, dK, dV = check_full(t, ridx, 64, g, w, 0.125, key_mask=km, tag="bwd padding")
    dKh, dVh, dQh = to_host(dK), to_host(dV), to_host(dQ)
    pad = km == 0
    for bi in range(B):
        assert (dKh[bi][:, pad[bi]] == 0).all() and (dVh[bi][:, pad[bi]] == 0).all()
    assert (dQh[2] == 0).all()


def test_runs_are_bit_reproducible():
    torch = torch_mod()
    t = inp.make_tensors(2, 3, 2048, 64, 23, "bf16", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(3, 2048, 64, 2, 3, 3, 2)
    a = run_fwd_bwd(t, ridx, 2, 3, 0.125)
    b_ = run_fwd_bwd(t, ridx, 2, 3, 0.125)
    for x, y in zip(a, b_):
        assert torch.equal(x, y)


def test_cfg4_sampled_heads():
    """Full-size forward+backward workload; the oracle is run on three (batch, head) slices."""
    wl = inp.WORKLOADS["cfg4_fwd_bwd"]
    t = inp.workload_tensors(wl)
    ridx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    assert (ridx == oracle.make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)).all()
    dQ, dK, dV = run_fwd_bwd(t, ridx, wl.g, wl.w, wl.scale)
    hQ, hK, hV = to_host(dQ), to_host(dK), to_host(dV)
    assert np.isfinite(hQ).all() and np.isfinite(hK).all() and np.isfinite(hV).all()
    worst = 0.0
    for (bi, h) in [(0, 0), (1, 11), (0, 5)]:
        sl = (slice(bi, bi + 1), slice(h, h + 1))
        rQ, rK, rV = oracle.attn_bwd(t["Q"][sl], t["K"][sl], t["V"][sl], t["dO"][sl], ridx[h:h + 1],
                                     wl.b, wl.g, wl.w, wl.scale)
        errs = [np.abs(hQ[sl] - rQ).max(), np.abs(hK[sl] - rK).max(), np.abs(hV[sl] - rV).max()]
        print(f"cfg4 (b={bi}, h={h}): max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} max|ddV|={errs[2]:.3e}")
        worst = max(worst, *errs)
    assert worst <= TOL
    # properties that hold at any size (rows of P sum to 1, rows of dS sum to 0)
    dOh = t["dO"].astype(np.float64)
    assert np.abs(hV.sum(axis=2) - dOh.sum(axis=2)).max() <= 0.5       # sums of 4096 bf16-rounded terms
    assert np.abs(hK.sum(axis=2)).max() <= 0.5
    # dQ = scale dS K and dK = scale dS^T Q give sum(Q o dQ) = sum(K o dK) = sum(dS o S) per head
    qdq = (t["Q"].astype(np.float64) * hQ).sum(axis=(2, 3))
    kdk = (t["K"].astype(np.float64) * hK).sum(axis=(2, 3))
    print("cfg4 sum(Q o dQ) vs sum(K o dK): max diff", np.abs(qdq - kdk).max(), "of", np.abs(qdq).max())
    assert np.abs(qdq - kdk).max() <= 1e-3 * max(1.0, np.abs(qdq).max()) + 0.5


def test_cfg3_shape_backward_with_padding_sampled_heads():
    """The key-padding workload (B = 8, lengths 1024..4096) through forward + backward; the
    oracle is run on three (batch, head) slices, among them the shortest and the longest row."""
    wl = inp.WORKLOADS["cfg3_key_padding"]
    t = inp.make_tensors(wl.B, wl.H, wl.n, wl.d, wl.data_seed, "bf16", with_dO=True)
    km = inp.lengths_to_key_mask(inp.make_valid_lengths(wl.B, wl.n, wl.b, wl.length_seed), wl.n)
    ridx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    dQ, dK, dV = run_fwd_bwd(t, ridx, wl.g, wl.w, wl.scale, key_mask=km)
    hQ, hK, hV = to_host(dQ), to_host(dK), to_host(dV)
    assert np.isfinite(hQ).all() and np.isfinite(hK).all() and np.isfinite(hV).all()
    lens = km.sum(axis=1)
    worst = 0.0
    for (bi, h) in [(int(lens.argmin()), 0), (int(lens.argmax()), 7), (3, 11)]:
        sl = (slice(bi, bi + 1), slice(h, h + 1))
        rQ, rK, rV = oracle.attn_bwd(t["Q"][sl], t["K"][sl], t["V"][sl], t["dO"][sl], ridx[h:h + 1],
                                     wl.b, wl.g, wl.w, wl.scale, key_mask=km[bi:bi + 1])
        errs = [np.abs(hQ[sl] - rQ).max(), np.abs(hK[sl] - rK).max(), np.abs(hV[sl] - rV).max()]
        print(f"cfg3 bwd (b={bi}, len={int(lens[bi])}, h={h}): max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} "
              f"max|ddV|={errs[2]:.3e}")
        worst = max(worst, *errs)
    assert worst <= TOL
    pad = km == 0
    for bi in range(wl.B):   # gradients of padded keys are exactly zero
        assert (hK[bi][:, pad[bi]] == 0).all() and (hV[bi][:, pad[bi]] == 0).all()


TOL_F32 = 1e-4


def check_full_f32(t, rand_idx, b, g, w, scale, key_mask=None, mode=0, tag=""):
    """fp32 tensors through forward + backward; max abs error of the gradients <= 1e-4."""
    torch = torch_mod()
    Q, K, V = device_qkv(t, "f32")
    dO = device_tensor(t, "dO", "f32")
    ridx = torch.from_numpy(np.ascontiguousarray(rand_idx)).to("cuda:0")
    km = None if key_mask is None else torch.from_numpy(key_mask).to("cuda:0")
    O, LSE = bb.bigbird_attn_fwd(Q, K, V, ridx, g=g, w=w, scale=scale, key_padding_mask=km, global_mode=mode)
    dQ, dK, dV = bb.bigbird_attn_bwd(Q, K, V, O, LSE, dO, ridx, g=g, w=w, scale=scale,
                                     key_padding_mask=km, global_mode=mode)
    torch.cuda.synchronize()
    ref = oracle.attn_bwd(t["Q"], t["K"], t["V"], t["dO"], rand_idx, b, g, w, scale,
                          key_mask=key_mask, global_mode=mode)
    errs = [np.abs(to_host(x) - r).max() for x, r in zip((dQ, dK, dV), ref)]
    print(f"{tag}: max|ddQ|={errs[0]:.3e} max|ddK|={errs[1]:.3e} max|ddV|={errs[2]:.3e}")
    assert all(np.isfinite(to_host(x)).all() for x in (dQ, dK, dV)), tag
    assert max(errs) <= TOL_F32, (tag, errs)
    return dQ, dK, dV


def test_fp32_backward_cfg1_shape():
    wl = inp.WORKLOADS["cfg1_fp32_small"]
    t = inp.make_tensors(wl.B, wl.H, wl.n, wl.d, wl.data_seed, "f32", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    check_full_f32(t, ridx, wl.b, wl.g, wl.w, wl.scale, tag="fp32 bwd cfg1 shape")


def test_fp32_backward_ragged_padding_and_long_lists():
    # leading globals, ragged shape
    B, H, n, g, w, r = 2, 3, 640, 3, 5, 2
    t = inp.make_tensors(B, H, n, 64, 17, "f32", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 9, bb.BB_GLOBAL_LEADING)
    check_full_f32(t, ridx, 64, g, w, 0.2, mode=bb.BB_GLOBAL_LEADING, tag="fp32 bwd ragged")
    # padding: unaligned lengths, a hole, one sequence without any valid key
    B, H, n, g, w, r = 3, 2, 1024, 2, 3, 3
    t = inp.make_tensors(B, H, n, 64, 31, "f32", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 4)
    km = np.ones((B, n), dtype=np.uint8)
    km[0, 700:] = 0
    km[0, 130:150] = 0
    km[1, :] = 0
    dQ, dK, dV = check_full_f32(t, ridx, 64, g, w, 0.125, key_mask=km, tag="fp32 bwd padding")
    assert (to_host(dK)[0][:, 700:] == 0).all() and (to_host(dV)[1] == 0).all() and (to_host(dQ)[1] == 0).all()
    # every row and every column attended by all 80 blocks (lists longer than one chunk of 64)
    B, H, n = 1, 1, 5120
    nb = n // 64
    t = inp.make_tensors(B, H, n, 64, 18, "f32", with_dO=True)
    empty = np.full((H, nb, 0), -1, dtype=np.int32)
    check_full_f32(t, empty, 64, nb, 1, 0.125, tag="fp32 bwd full coverage (all global, 80 blocks)")


@pytest.mark.parametrize("g,w,r", [(0, 1, 0), (1, 1, 0), (0, 3, 2), (2, 3, 0), (1, 7, 4)])
def test_fp32_backward_degenerate_patterns(g, w, r):
    B, H, n = 1, 2, 1024
    t = inp.make_tensors(B, H, n, 64, 19, "f32", with_dO=True)
    ridx = bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 3)
    check_full_f32(t, ridx, 64, g, w, 0.125, tag=f"fp32 bwd g{g} w{w} r{r}")


def test_seeded_sweep_of_small_configurations():
    """Twenty-five seeded combinations of batch, heads, length, pattern, placement and padding."""
    rng = np.random.default_rng(20261)
    done = 0
    while done < 25:
        nb = int(rng.integers(1, 17))
        g = int(rng.integers(0, min(nb, 3) + 1))
        w = int(rng.choice([1, 3, 5, 7]))
        r = int(rng.integers(0, 5))
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        mode = int(rng.integers(0, 2))
        n = nb * 64
        try:
            ridx = oracle.make_rand_idx(H, n, 64, g, w, r, int(rng.integers(0, 1000)), mode)
        except ValueError:
            continue
        t = inp.make_tensors(B, H, n, 64, int(rng.integers(0, 10000)), "bf16", with_dO=True)
        km = None
        if rng.random() < 0.5:
            km = np.ones((B, n), dtype=np.uint8)
            for bi in range(B):
                km[bi, int(rng.integers(0, n + 1)):] = 0
                if rng.random() < 0.3:
                    a = int(rng.integers(0, n)); km[bi, a:a + int(rng.integers(1, 130))] = 0
        check_full(t, ridx, 64, g, w, 0.125, key_mask=km, mode=mode,
                   tag=f"bwd sweep {done}: B{B} H{H} nb{nb} g{g} w{w} r{r} mode{mode} pad{km is not None}")
        done += 1
