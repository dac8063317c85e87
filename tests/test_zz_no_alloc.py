"""scmoe_dispatch_static (the entry point that allocates nothing: its scratch is a static
device array) against scmoe_dispatch with a caller workspace: every output array bit for bit,
on two calls in a row, the second one smaller, so that what the first left in the shared
scratch is there when the second runs."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2404_05019_amd import binding as B
    from gpu_util import DEV


def _both(T, E, k, C_, d, seed):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.full(E, 0.6))
    idx_h = rng.choice(E, size=T * k, p=p).astype(np.int32)
    idx_h[rng.integers(0, T * k, 50)] = -1                       # indices outside [0, E) are dropped items
    idx = torch.from_numpy(idx_h).to(DEV)
    x = torch.randn((T, d), dtype=torch.float32, device=DEV).to(torch.bfloat16)
    rows = min(T * k, E * C_)
    out = []
    for static in (False, True):
        counts = torch.full((E,), -5, dtype=torch.int32, device=DEV)
        offsets = torch.full((E + 1,), -5, dtype=torch.int32, device=DEV)
        dst_row = torch.full((T * k,), -5, dtype=torch.int32, device=DEV)
        src_token = torch.full((rows,), -5, dtype=torch.int32, device=DEV)
        x_perm = torch.zeros((rows, d), dtype=torch.bfloat16, device=DEV)
        if static:
            B.scmoe_dispatch_static(x, idx, E, k, C_, counts, offsets, dst_row, src_token, x_perm)
        else:
            ws = torch.empty(max(B.scmoe_dispatch_workspace_bytes(T, E, k), 16), dtype=torch.uint8, device=DEV)
            B.scmoe_dispatch(x, idx, E, k, C_, counts, offsets, dst_row, src_token, x_perm, ws)
        torch.cuda.synchronize()
        out.append((counts, offsets, dst_row, src_token, x_perm))
    for a, b in zip(*out):
        assert torch.equal(a, b)
    K = int(out[0][1][E].item())
    assert 0 < K <= rows and int((out[0][2] >= 0).sum().item()) == K
    return K


def test_static_scratch_dispatch_matches_the_workspace_form_twice():
    print("case: scmoe_dispatch_static T=300000 E=16 k=1, then T=70001 E=5 k=2", flush=True)
    assert B.scmoe_dispatch_workspace_bytes(300000, 16, 1) <= B.scmoe_dispatch_static_max_bytes()
    k1 = _both(300000, 16, 1, 20000, 8, seed=11)      # capacity binds for the popular experts
    k2 = _both(70001, 5, 2, 30000, 16, seed=12)       # smaller, ragged, two choices per token
    assert k1 < 300000 and k2 < 140002


def test_static_scratch_dispatch_rejects_sizes_beyond_its_scratch():
    T, E, k = 1 << 21, 64, 4
    assert B.scmoe_dispatch_workspace_bytes(T, E, k) > B.scmoe_dispatch_static_max_bytes()
    x = torch.empty((T, 8), dtype=torch.bfloat16, device=DEV)
    i32 = lambda n: torch.empty(n, dtype=torch.int32, device=DEV)
    with pytest.raises(B.ScmoeError) as e:
        B.scmoe_dispatch_static(x, i32(T * k), E, k, T, i32(E), i32(E + 1), i32(T * k), i32(T * k), None)
    assert e.value.status == 4
    torch.cuda.synchronize()
