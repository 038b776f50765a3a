"""sphattn_splitkv_fwd_noalloc (the entry point for callers that cannot allocate) against
sphattn_splitkv_fwd, through the C ABI: same kernels and the same slice plan, so the outputs
must be equal bit for bit.  Two calls in a row share the library's one scratch array, the
second on a smaller input (stale partials of the first call lie behind it); then a call that
needs more scratch than the array holds must be refused without enqueueing anything.  The
allocator's counters must not move across the calls."""
import re
import os

import numpy as np
import pytest
import torch

import synthetic_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_2505_09326_amd as p
    p.load_library()
    return p


def _reference(pkg, q, k, v, mult, n_splits, dtype):
    B, H, N, d = q.shape
    used = n_splits if n_splits else pkg.sphattn_splitkv_heuristic(B, H, N, d, dtype)
    ws = torch.empty(pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, max(used, 1)), dtype=torch.uint8, device=DEV)
    Z = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    O = pkg.sphattn_splitkv_fwd(q, k, v, ws, mult=mult, Z=Z, n_splits=n_splits, dtype=dtype)
    return O, Z


def test_header_and_binding_agree_on_the_limit(pkg):
    text = open(os.path.join(ROOT, "include", "sphattn.h")).read()
    m = re.search(r"#define SPHATTN_NOALLOC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == pkg.NOALLOC_SCRATCH_BYTES


def test_noalloc_matches_workspace_call_twice_in_a_row(pkg, oracle):
    cases = [  # first a larger problem, then a smaller one in the same scratch array
        dict(B=1, H=2, H_kv=1, N=3000, d=128, n_splits=6, dtype="bf16", mult=True, seed=71),
        dict(B=1, H=1, H_kv=1, N=700, d=64, n_splits=3, dtype="bf16", mult=False, seed=72),
        dict(B=1, H=1, H_kv=1, N=1200, d=128, n_splits=0, dtype="f16", mult=False, seed=73),
    ]
    prepared = []
    for c in cases:
        q, _, _ = si.make_qkv(c["B"], c["H"], c["N"], c["d"], c["dtype"], seed=c["seed"])
        _, k, v = si.make_qkv(c["B"], c["H_kv"], c["N"], c["d"], c["dtype"], seed=c["seed"] + 100)
        mult = None
        if c["mult"]:
            g = torch.Generator(device="cpu").manual_seed(c["seed"])
            mult = torch.poisson(torch.full((c["B"], c["N"]), 1.5), generator=g).to(torch.float32)
        dev = [t.to(DEV) if t is not None else None for t in (q, k, v, mult)]
        O = torch.empty(q.shape, dtype=q.dtype, device=DEV)
        Z = torch.empty(q.shape[:3], dtype=torch.float32, device=DEV)
        prepared.append((c, (q, k, v, mult), dev, O, Z))
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    for c, _, (qd, kd, vd, md), O, Z in prepared:
        print(f"case noalloc {c}", flush=True)
        pkg.sphattn_splitkv_fwd_noalloc(qd, kd, vd, O, mult=md, Z=Z, n_splits=c["n_splits"], dtype=c["dtype"])
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == before   # torch's allocator was not asked
    for c, (q, k, v, mult), (qd, kd, vd, md), O, Z in prepared:
        O_ref, Z_ref = _reference(pkg, qd, kd, vd, md, c["n_splits"], c["dtype"])
        torch.cuda.synchronize()
        assert torch.equal(O.view(torch.int16), O_ref.view(torch.int16))
        assert torch.equal(Z, Z_ref)
        # and the pair is right, not just equal: against the oracle at the path's tolerance
        bits = [si.storage_bits(t)[0] for t in (q, k, v)]
        kind = si.storage_bits(q)[1]
        ref = oracle.grn_attention(*bits, mult.numpy() if mult is not None else None, kinds=(kind,) * 3)
        err = np.abs(O.cpu().double().numpy() - ref).max() / np.sqrt((ref ** 2).mean())
        print(f"noalloc vs oracle max|err|/rms={err:.3e}", flush=True)
        assert err <= (2e-2 if c["dtype"] == "bf16" else 5e-3)


def test_noalloc_refuses_what_does_not_fit(pkg):
    # 2 slices of B*H*N*(d+1)*4 bytes = 2 * 135 MB: more than the array
    B, H, N, d = 1, 8, 32768, 128
    assert pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, 2) > pkg.NOALLOC_SCRATCH_BYTES
    q = torch.zeros((B, H, N, d), dtype=torch.bfloat16, device=DEV)
    O = torch.full_like(q, 3.0)
    with pytest.raises(pkg.SphattnError) as e:
        pkg.sphattn_splitkv_fwd_noalloc(q, q, q, O, n_splits=2)
    assert e.value.code == -10
    torch.cuda.synchronize()
    assert torch.all(O == 3.0)                   # nothing was enqueued


def test_one_slice_is_the_unsplit_launch_without_scratch(pkg):
    """One slice: both split entry points run the plain forward (bit-equal to sphattn_fwd_z),
    and the no-allocation one has no size limit then: 2 x 16 x 8192 x 128 in one slice would
    need 135 MB of partial pairs."""
    B, H, N, d = 2, 16, 8192, 128
    assert pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, 1) > pkg.NOALLOC_SCRATCH_BYTES
    assert pkg.sphattn_splitkv_heuristic(B, H, N, d, "bf16") == 1
    q, k, v = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "bf16", seed=5))
    want, zw = pkg.sphattn_fwd_z(q, k, v, dtype="bf16")
    O = torch.empty_like(q)
    Z = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    for n_splits in (0, 1):
        O.zero_()
        Z.zero_()
        pkg.sphattn_splitkv_fwd_noalloc(q, k, v, O, Z=Z, n_splits=n_splits, dtype="bf16")
        torch.cuda.synchronize()
        assert torch.equal(O, want) and torch.equal(Z, zw)
