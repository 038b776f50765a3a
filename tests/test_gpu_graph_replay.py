"""HIP-graph capture and replay of the entry points (a serving loop would capture its launches):
the library allocates nothing, never synchronises and launches on the caller's stream, so its
calls can be recorded into a graph once the kernels' one-time set-up (raising the LDS limit)
has happened in an eager warm-up call.  Every replay is compared bit for bit with the eager
result on the same inputs, with eager work and synchronisations between the replays.
"""
import pytest
import torch

import synthetic_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    import paper_2505_09326_amd as p
    p.load_library()
    return p


def _capture(fn):
    """Warm up eagerly on a side stream (torch's rule for capture), then capture `fn`."""
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def test_graph_replay_forward_splitkv_and_backward(pkg):
    print("case graph replay bf16", flush=True)
    B, H, N, d = 1, 2, 700, 128
    q, k, v = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "bf16", seed=1))
    dO = torch.randn(B, H, N, d, device=DEV).to(torch.bfloat16)
    out, out_s = torch.empty_like(v), torch.empty_like(v)
    Z = torch.empty(B, H, N, dtype=torch.float32, device=DEV)
    dQ, dK, dV = (torch.empty_like(q) for _ in range(3))
    delta = torch.empty(2, B, H, N, dtype=torch.float32, device=DEV)
    ws = torch.empty(pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, 4), dtype=torch.uint8, device=DEV)

    def step():
        pkg.sphattn_fwd_z(q, k, v, out, Z, dtype="bf16")
        pkg.sphattn_splitkv_fwd(q, k, v, ws, O=out_s, n_splits=4, dtype="bf16")
        pkg.sphattn_bwd(q, k, v, out, dO, Z, dQ, dK, dV, delta, dtype="bf16")

    g = _capture(step)
    for rep in range(3):
        q2, k2, v2 = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "bf16", seed=10 + rep))
        q.copy_(q2); k.copy_(k2); v.copy_(v2)
        for t in (out, out_s, dQ, dK, dV):
            t.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, out_s, Z, dQ, dK, dV)]
        for t in (out, out_s, dQ, dK, dV):
            t.zero_()
        step()                                   # eager, same inputs
        torch.cuda.synchronize()
        for a, b in zip(got, (out, out_s, Z, dQ, dK, dV)):
            assert torch.equal(a, b)
        assert torch.isfinite(out.float()).all() and out.float().abs().max() > 0


def test_graph_replay_all_e4m3_forward(pkg):
    print("case graph replay fp8", flush=True)
    B, H, N, d = 1, 2, 520, 128
    q, k, v = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "fp8", seed=2))
    out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=DEV)

    def step():
        pkg.sphattn_fp8_fwd(q, k, v, ws, O=out)

    g = _capture(step)
    for rep in range(3):
        q2, k2, v2 = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "fp8", seed=20 + rep, factor=2.0 ** rep))
        q.view(torch.uint8).copy_(q2.view(torch.uint8))
        k.view(torch.uint8).copy_(k2.view(torch.uint8))
        v.view(torch.uint8).copy_(v2.view(torch.uint8))
        out.zero_()
        ws.fill_(0xFF)                           # the call clears what it needs itself
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, out)
        assert torch.isfinite(out.float()).all() and out.float().abs().max() > 0
