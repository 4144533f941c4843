"""CPU-side tests of the C ABI: symbols, host pattern functions, error paths (no GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2007_14062_amd as bb
from paper_2007_14062_amd.binding import load_library

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bigbird.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bigbird_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = load_library()
    names = declared_functions()
    assert len(names) >= 7
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(bb.EXPORTED_SYMBOLS) == names


def test_status_strings():
    assert bb.bigbird_status_string(0) == "ok"
    for code in range(-7, 0):
        assert bb.bigbird_status_string(code) not in ("ok", "unknown status")
    assert bb.bigbird_status_string(-99) == "unknown status"


@pytest.mark.parametrize("H,n,b,g,w,r,seed,mode", [
    (2, 1024, 64, 2, 3, 3, 0, 0),
    (12, 4096, 64, 2, 3, 3, 1, 0),
    (3, 16384, 64, 2, 3, 3, 4, 0),
    (1, 12, 2, 1, 3, 1, 7, 0),
    (3, 640, 64, 3, 5, 2, 9, 1),
    (2, 2048, 64, 0, 1, 5, 123456789012345, 0),
    (2, 512, 64, 2, 3, 0, 5, 0),
])
def test_rand_idx_is_bit_exact_with_the_oracle_generator(H, n, b, g, w, r, seed, mode):
    got = bb.bigbird_make_rand_idx(H, n, b, g, w, r, seed, mode)
    want = oracle.make_rand_idx(H, n, b, g, w, r, seed, mode)
    assert got.dtype == np.int32 and got.shape == want.shape
    assert (got == want).all()
    assert bb.bigbird_validate_rand_idx(got, H, n, b, g, w, r, mode) == 0


def test_rand_idx_matches_golden_file(golden_dir):
    with open(os.path.join(golden_dir, "rand_idx_cfg2_seed1.txt")) as f:
        H, nb, r, seed, g, w, mode = (int(x) for x in f.readline().split())
        want = np.array([[int(x) for x in line.split()] for line in f], dtype=np.int32)
    got = bb.bigbird_make_rand_idx(H, nb * 64, 64, g, w, r, seed, mode)
    assert (got.reshape(-1, r) == want).all()


def test_validate_rejects_bad_tables():
    H, n, b, g, w, r = 2, 1024, 64, 2, 3, 3
    t = bb.bigbird_make_rand_idx(H, n, b, g, w, r, 0)
    for (h, j, i, val) in [(0, 5, 0, 5), (0, 5, 1, 4), (1, 3, 2, 0), (1, 3, 2, 15), (0, 7, 0, 16),
                           (0, 7, 0, -1)]:
        bad = t.copy()
        bad[h, j, i] = val
        assert bb.bigbird_validate_rand_idx(bad, H, n, b, g, w, r) == -3
        assert not oracle.validate_rand_idx(bad, H, n, b, g, w, r)
    bad = t.copy()
    bad[0, 6, 1] = bad[0, 6, 0]
    assert bb.bigbird_validate_rand_idx(bad, H, n, b, g, w, r) == -3
    # rows of global query blocks are ignored
    ok = t.copy()
    ok[0, 0, :] = 7
    assert bb.bigbird_validate_rand_idx(ok, H, n, b, g, w, r) == 0


def test_make_rand_idx_error_paths():
    lib = load_library()
    buf = np.zeros(1024, dtype=np.int32)
    p = buf.ctypes.data
    assert lib.bigbird_make_rand_idx(None, 1, 1024, 64, 2, 3, 3, 0, 0) == -1
    assert lib.bigbird_make_rand_idx(p, 1, 1000, 64, 2, 3, 3, 0, 0) == -2      # n % b
    assert lib.bigbird_make_rand_idx(p, 1, 1024, 64, 2, 4, 3, 0, 0) == -2      # w even
    assert lib.bigbird_make_rand_idx(p, 1, 1024, 64, 17, 3, 3, 0, 0) == -2     # g > nb
    assert lib.bigbird_make_rand_idx(p, 1, 1024, 64, 2, 3, 3, 0, 5) == -2      # global mode
    assert lib.bigbird_make_rand_idx(p, 1, 320, 64, 2, 3, 3, 0, 0) == -3       # too few candidates
    with pytest.raises(bb.BigBirdError):
        bb.bigbird_make_rand_idx(1, 320, 64, 2, 3, 3, 0)


def test_count_block_pairs_matches_oracle_and_closed_form():
    for (B, H, n, seed) in [(1, 2, 1024, 0), (2, 3, 4096, 1)]:
        t = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, seed)
        nb = n // 64
        got = bb.bigbird_count_block_pairs(t, None, B, H, n, 64, 2, 3, 3)
        assert got == B * H * (10 * nb - 18)
        assert got == B * oracle.count_block_pairs(t, n, 64, 2, 3)
    # with a key-padding mask: pairs whose key block is fully padded are not counted
    B, H, n = 2, 2, 2048
    t = bb.bigbird_make_rand_idx(H, n, 64, 2, 3, 3, 2)
    km = np.ones((B, n), dtype=np.uint8)
    km[0, 1000:] = 0
    km[1, 1536:] = 0
    got = bb.bigbird_count_block_pairs(t, km, B, H, n, 64, 2, 3, 3)
    want = 0
    for bi in range(B):
        valid = km[bi].reshape(-1, 64).any(axis=1)
        want += oracle.count_block_pairs(t, n, 64, 2, 3, key_block_valid=valid)
    assert got == want


def test_workspace_bytes():
    assert bb.bigbird_attn_workspace_bytes(4, 12, 4096, 64, 64, 2, 3, 3) > 0
    assert bb.bigbird_attn_workspace_bytes(4, 12, 4096, 32, 64, 2, 3, 3) == 0     # d unsupported
    assert bb.bigbird_attn_workspace_bytes(4, 12, 4100, 64, 64, 2, 3, 3) == 0     # n % b
    small = bb.bigbird_attn_workspace_bytes(1, 1, 512, 64, 64, 2, 3, 3)           # nb = 8: nothing split
    assert small == 0
    assert (bb.bigbird_attn_workspace_bytes(4, 12, 4096, 64, 64, 2, 3, 3, True)
            >= bb.bigbird_attn_workspace_bytes(4, 12, 4096, 64, 64, 2, 3, 3, False))


def test_attn_fwd_host_checks_fire_before_any_launch():
    """Every error below is found on the host: no GPU is touched, so this runs anywhere."""
    lib = load_library()
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: the checks fail first
    odd = ctypes.c_void_p(0x1004)

    def call(Q=fake, K=fake, V=fake, O=fake, LSE=fake, rand=fake, km=None, B=1, H=2, n=1024, d=64,
             b=64, g=2, w=3, r=3, scale=0.125, dtype=1, mode=0, ws=fake, ws_bytes=1 << 30):
        return lib.bigbird_attn_fwd(Q, K, V, O, LSE, rand, km, B, H, n, d, b, g, w, r, scale,
                                    dtype, mode, ws, ws_bytes, None)

    assert call(Q=None) == -1
    assert call(LSE=None) == -1
    assert call(rand=None) == -1
    assert call(n=1000) == -2
    assert call(w=4) == -2
    assert call(g=-1) == -2
    assert call(B=-1) == -2
    assert call(K=odd) == -2                       # misaligned pointer
    assert call(d=128) == -6
    assert call(b=32, n=1024) == -6
    assert call(scale=0.0) == -6
    assert call(scale=float("nan")) == -6
    assert call(dtype=7) == -4
    assert call(ws=None) == -5
    assert call(ws_bytes=16) == -5
    assert call(ws=odd) == -5
    assert call(B=0) == 0                          # empty problem
    assert call(H=0) == 0


def test_attn_bwd_host_checks_fire_before_any_launch():
    lib = load_library()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)

    def call(Q=fake, K=fake, V=fake, O=fake, LSE=fake, dO=fake, dQ=fake, dK=fake, dV=fake, rand=fake,
             km=None, B=1, H=2, n=1024, d=64, b=64, g=2, w=3, r=3, scale=0.125, dtype=1, mode=0,
             ws=fake, ws_bytes=1 << 30):
        return lib.bigbird_attn_bwd(Q, K, V, O, LSE, dO, dQ, dK, dV, rand, km, B, H, n, d, b, g, w, r,
                                    scale, dtype, mode, ws, ws_bytes, None)

    assert call(dO=None) == -1
    assert call(dV=None) == -1
    assert call(rand=None) == -1
    assert call(n=1000) == -2
    assert call(w=2) == -2
    assert call(dK=odd) == -2
    assert call(d=32) == -6
    assert call(dtype=0, ws=None) == -5            # the fp32 backward goes through the same checks
    assert call(dtype=9) == -4
    assert call(scale=-1.0) == -6
    assert call(n=64 * 257) == -6                  # more key blocks than the backward's list holds (256)
    assert call(ws=None) == -5
    assert call(ws_bytes=1024) == -5
    assert call(B=0) == 0
    need_fwd = bb.bigbird_attn_workspace_bytes(1, 2, 1024, 64, 64, 2, 3, 3, False)
    need_bwd = bb.bigbird_attn_workspace_bytes(1, 2, 1024, 64, 64, 2, 3, 3, True)
    assert need_bwd > need_fwd
    assert call(ws_bytes=need_fwd) == -5           # a forward-sized workspace is too small


def test_binding_refuses_cpu_tensors():
    import torch
    Q = torch.zeros(1, 1, 64, 64)
    t = torch.zeros(1, 1, 0, dtype=torch.int32)
    with pytest.raises(ValueError):
        bb.bigbird_attn_fwd(Q, Q, Q, t, g=1, w=1, scale=1.0)


def test_binding_validator_refuses_wrong_dtypes_and_shapes():
    """The C side reads tensors through raw pointers: the one validator shared by the forward,
    backward and prepare_* wrappers must refuse what would be misread (checked on CPU tensors: the
    validator looks at shapes and dtypes only)."""
    import torch
    from paper_2007_14062_amd.binding import _check_attn_args as chk
    B, H, n, d, b, r = 2, 3, 256, 64, 64, 2
    Q = torch.zeros((B, H, n, d), dtype=torch.bfloat16)
    ridx = torch.zeros((H, n // b, r), dtype=torch.int32)
    km = torch.ones((B, n), dtype=torch.uint8)
    lse = torch.zeros((B, H, n), dtype=torch.float32)
    g32 = torch.zeros((B, H, n, d), dtype=torch.float32)
    assert chk(Q, Q, Q, ridx, km, b, O=Q, LSE=lse, dO=Q, grads=(g32, g32, g32)) == (B, H, n, d, r)
    assert chk(Q, Q, Q, None, None, b) == (B, H, n, d, 0)
    bad = [
        dict(K=Q.float()),                                   # K of another dtype
        dict(V=Q[:, :, :128]),                               # V of another shape
        dict(rand_idx=ridx.long()),                          # int64 table
        dict(rand_idx=ridx[:, :2]),                          # table with too few rows
        dict(key_padding_mask=km.bool()),                    # mask not uint8
        dict(key_padding_mask=km[:, :128]),                  # mask of another length
        dict(LSE=lse.double()),                              # float64 LSE
        dict(LSE=lse[:, :, :128]),
        dict(O=Q.float()),
        dict(dO=Q.float()),
        dict(grads=(g32.double(), g32, g32)),                # float64 gradient buffer
        dict(grads=(g32, g32[:, :1], g32)),
    ]
    for kw in bad:
        args = dict(Q=Q, K=Q, V=Q, rand_idx=ridx, key_padding_mask=km, b=b, O=Q, LSE=lse, dO=Q, grads=(g32, g32, g32))
        args.update(kw)
        with pytest.raises(ValueError):
            chk(**args)
    with pytest.raises(ValueError):
        chk(Q[0], Q[0], Q[0], ridx, km, b)                   # Q not [B, H, n, d]


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; any other --gpus value exits with a message and status 2."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
