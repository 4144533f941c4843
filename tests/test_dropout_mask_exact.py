"""GPU test: the keep mask inside the bf16 kernels, bit by bit.

The parity tolerance of the bf16 path (2e-2) is wider than what one wrong mask bit changes in an
output of an ordinary problem, so the parity tests alone could not see a sparse mask error in the
bf16 kernels (the fp32 kernels, held to 1e-4, have their own mask code).  Here the inputs are
chosen so that every output element counts kept keys (or queries) of one residue class modulo 64:
with Q = 0 or K = 0 the softmax is uniform, and one-hot V, K, Q or dO rows route each attended
pair into one output column.  One flipped mask bit then moves an output by a whole step
(rs / |N(i)|, times scale for dQ and dK), the rounding of the bf16 path stays below a tenth of a
step, and the comparison with the oracle uses a quarter of the smallest step as its tolerance:
forward (O), dK/dV kernel (dV, dK) and dQ kernel (dQ) each see every mask bit of the pattern.
"""
import numpy as np
import pytest

import bigbird_inputs as inp
import oracle
import paper_2007_14062_amd as bb
from gpu_util import to_host

pytestmark = pytest.mark.gpu

B, H, n, b, g, w, r = 1, 2, 1024, 64, 2, 3, 3
SCALE, P_DROP, SEED = 0.125, 0.1, 0xC0FFEE1234


def _dev(x):
    import torch
    _, bits = inp.round_to_bf16(np.ascontiguousarray(x, dtype=np.float32))
    return torch.from_numpy(bits.view(np.int16)).to("cuda:0").view(torch.bfloat16)


def _onehot():
    x = np.zeros((B, H, n, 64), dtype=np.float32)
    x[:, :, np.arange(n), np.arange(n) % 64] = 1.0
    return x


def _run(Q, K, V, dO, ridx_h):
    import torch
    ridx = torch.from_numpy(ridx_h).to("cuda:0")
    dQ_, dK_, dV_, ddO = _dev(Q), _dev(K), _dev(V), _dev(dO)
    O, LSE = bb.bigbird_attn_fwd_dropout(dQ_, dK_, dV_, ridx, g=g, w=w, scale=SCALE, p_drop=P_DROP, seed=SEED)
    grads = bb.bigbird_attn_bwd_dropout(dQ_, dK_, dV_, O, LSE, ddO, ridx, g=g, w=w, scale=SCALE,
                                        p_drop=P_DROP, seed=SEED)
    torch.cuda.synchronize()
    Oo, _ = oracle.attn_fwd_dropout(Q, K, V, ridx_h, b, g, w, SCALE, P_DROP, SEED)
    ref = oracle.attn_bwd_dropout(Q, K, V, dO, ridx_h, b, g, w, SCALE, P_DROP, SEED)
    return to_host(O), [to_host(x) for x in grads], Oo, ref


def test_every_mask_bit_shows_in_the_outputs():
    import torch
    assert torch.cuda.is_available()
    ridx_h = bb.bigbird_make_rand_idx(H, n, b, g, w, r, 21)
    rs = oracle.dropout_scale(P_DROP)
    step = rs / n                 # the smallest step: a global row attends all n keys
    rng = np.random.default_rng(3)
    zeros = np.zeros((B, H, n, 64), dtype=np.float32)
    ones = np.ones((B, H, n, 64), dtype=np.float32)
    rnd = rng.standard_normal((B, H, n, 64)).astype(np.float32)

    # forward and dV: Q = 0; V and dO one-hot by position modulo 64
    O, G, Oo, ref = _run(zeros, rnd, _onehot(), _onehot(), ridx_h)
    assert np.abs(O - Oo).max() < 0.25 * step, np.abs(O - Oo).max() / step
    assert np.abs(G[2] - ref[2]).max() < 0.25 * step, np.abs(G[2] - ref[2]).max() / step
    # the steps are really there: the oracle without dropout differs by many of them
    O_plain, _ = oracle.attn_fwd(zeros, rnd, _onehot(), ridx_h, b, g, w, SCALE)
    assert np.abs(Oo - O_plain * rs).max() > 2 * step

    # dQ: Q = 0, K one-hot, dO . V = 1 for every pair
    O, G, Oo, ref = _run(zeros, _onehot(), ones, ones / 64.0, ridx_h)
    assert np.abs(G[0] - ref[0]).max() < 0.25 * SCALE * step, np.abs(G[0] - ref[0]).max() / (SCALE * step)

    # dK: K = 0, Q one-hot, dO . V = 1 for every pair
    O, G, Oo, ref = _run(_onehot(), zeros, ones, ones / 64.0, ridx_h)
    assert np.abs(G[1] - ref[1]).max() < 0.25 * SCALE * step, np.abs(G[1] - ref[1]).max() / (SCALE * step)
