"""GPU test: the forward under HIP graph capture.  A captured call must record kernels only (the
library clears its item counters with a small kernel, not a memset node) and every replay must
give what the eager call gives for the inputs then in the buffers -- checked on several replays
with eager work and synchronisations between them, on the plain path and on the path that claims
items from counters (padding mask + BB_SKIP_PADDED_QUERY_BLOCKS)."""
import numpy as np
import pytest

import bigbird_inputs as inp
import paper_2007_14062_amd as bb
from gpu_util import device_qkv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("masked", [False, True])
def test_replays_equal_eager_calls(masked):
    import torch
    assert torch.cuda.is_available()
    B, H, n, g, w, r = 2, 3, 2048, 2, 3, 3
    sets = [device_qkv(inp.make_tensors(B, H, n, 64, 500 + i, "bf16"), "bf16") for i in range(3)]
    ridx = torch.from_numpy(bb.bigbird_make_rand_idx(H, n, 64, g, w, r, 8)).to("cuda:0")
    km = None
    flags = 0
    if masked:
        km = torch.from_numpy(inp.lengths_to_key_mask(np.array([1300, 700]), n)).to("cuda:0")
        flags = bb.BB_SKIP_PADDED_QUERY_BLOCKS
    kw = dict(g=g, w=w, scale=0.125, key_padding_mask=km, global_mode=flags)
    Q, K, V = (x.clone() for x in sets[0])
    O = torch.empty_like(Q)
    L = torch.empty((B, H, n), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(bb.bigbird_attn_workspace_bytes(B, H, n, 64, 64, g, w, r, False), dtype=torch.uint8,
                     device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        bb.bigbird_attn_fwd(Q, K, V, ridx, O=O, LSE=L, workspace=ws, stream=torch.cuda.current_stream(), **kw)
    torch.cuda.synchronize()
    for rep in range(5):
        src = sets[rep % 3]
        for dst, s in zip((Q, K, V), src):
            dst.copy_(s)
        O.fill_(float("nan"))
        ws.fill_(0xAB)                       # whatever the previous replay left must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        O_ref, L_ref = bb.bigbird_attn_fwd(*src, ridx, **kw)    # eager, own buffers
        torch.cuda.synchronize()
        assert torch.equal(O, O_ref), (masked, rep)
        assert torch.equal(L, L_ref), (masked, rep)
