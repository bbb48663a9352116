"""The entry point that allocates nothing (fobq_sensitivity_static) against the entry point it is a
variant of (fobq_sensitivity), through the C ABI: same kernels, scratch in the library's static
device array instead of context-owned allocations.  Named so that pytest collects it last."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _inputs(r, d, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((r, d)) * np.sqrt(2.0 / d)).astype(np.float32)
    A = rng.standard_normal((d, d + 8))
    Hinv = A @ A.T / (d + 8) + 0.1 * np.eye(d)          # any SPD matrix serves: only its diagonal is read
    return torch.from_numpy(W).cuda(), torch.from_numpy(Hinv).cuda()


def test_static_entry_point_matches_the_allocating_one_on_two_calls_in_a_row():
    import paper_2509_05576_amd as f
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (no CPU fallback exists)")
    f.load_library()
    ctx = f.Ctx(0)
    ref_ctx = f.Ctx(0)
    try:
        # second call smaller than the first: whatever the first left in the static array must not leak in
        cases = [(300, 1100, 4, 100, f.ORDER_SENSI_DESC), (70, 130, 3, 0, f.ORDER_ERR_ASC)]
        for r, d, bits, group, order in cases:
            _say(f"static sensitivity r={r} d={d} bits={bits} group={group} order={order}")
            W, Hinv = _inputs(r, d, 7 * r + d)
            S = torch.full((d,), -1.0, dtype=torch.float64, device="cuda")
            perm = torch.full((d,), -1, dtype=torch.int32, device="cuda")
            S_ref, perm_ref = f.fobq_sensitivity(ref_ctx.handle, W, Hinv, bits=bits, group=group, order=order)
            torch.cuda.synchronize()
            free_before, _ = torch.cuda.mem_get_info()
            f.fobq_sensitivity_static(ctx.handle, W, Hinv, bits=bits, group=group, order=order, S=S, perm=perm)
            free_after, _ = torch.cuda.mem_get_info()
            assert free_after >= free_before, "device memory was allocated during the call"
            # the same kernels in the same order on the same inputs: the fp64 scores agree to the
            # parity bar of S (1e-12 relative; in fact bit for bit) and the order is identical
            assert torch.allclose(S, S_ref, rtol=1e-12, atol=0.0)
            assert torch.equal(S, S_ref)
            assert torch.equal(perm, perm_ref)
            assert sorted(perm.cpu().tolist()) == list(range(d))
        # custom order: a bad permutation is reported by the static variant as well, and the array's
        # status words are cleared again by the next call
        W, Hinv = _inputs(16, 40, 3)
        bad = torch.zeros(40, dtype=torch.int32, device="cuda")
        with pytest.raises(f.FobqError) as ei:
            f.fobq_sensitivity_static(ctx.handle, W, Hinv, order=f.ORDER_CUSTOM, perm_in=bad)
        assert ei.value.code == f.EINVAL
        good = torch.arange(39, -1, -1, dtype=torch.int32, device="cuda")
        _, p = f.fobq_sensitivity_static(ctx.handle, W, Hinv, order=f.ORDER_CUSTOM, perm_in=good)
        assert torch.equal(p, good)
        # beyond the static limits: a clear error, nothing launched
        Wb = torch.zeros((4, 8200), dtype=torch.float32, device="cuda")
        Hb = torch.zeros((1, 1), dtype=torch.float64, device="cuda")     # never read: the call fails on the shape
        with pytest.raises(f.FobqError) as ei:
            f.fobq_sensitivity_static(ctx.handle, Wb, Hb)
        assert ei.value.code == f.EINVAL and "static scratch" in str(ei.value)
    finally:
        ctx.close()
        ref_ctx.close()
