"""The entry point that allocates nothing (lwp_eliminate_node_noalloc) against lwp_eliminate_node.

Two calls in a row through the C ABI, the second with a smaller input, so that anything the first
call left in the library's fixed scratch array would show; outputs must equal those of the
allocating entry point bit for bit (and the oracle's)."""
import ctypes

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def draw(rng, batch, Ci, Cj, Ck, hi):
    A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    w += (1000 * np.arange(batch, dtype=np.int32))[:, None]       # a different cost level per product
    return A, w, B


def run_both(ctx, A, w, B, want_argmin=True):
    import torch
    from paper_1802_04924_amd import binding
    d_A, d_w, d_B = dev(A), dev(w), dev(B)
    batch, Ci, _ = A.shape
    Ck = B.shape[2]
    ref_out, ref_arg = ctx.eliminate_node(d_A, d_w, d_B, want_argmin=want_argmin)
    ctx.synchronize()
    out = torch.full((batch, Ci, Ck), -7, dtype=torch.int32, device="cuda")
    arg = torch.full((batch, Ci, Ck), -7, dtype=torch.int32, device="cuda") if want_argmin else None
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    lib = binding.load()
    st = torch.cuda.current_stream().cuda_stream
    rc = lib.lwp_eliminate_node_noalloc(ctypes.c_void_p(st), batch, Ci, A.shape[2], Ck, d_A.data_ptr(), d_w.data_ptr(),
                                        d_B.data_ptr(), out.data_ptr(), arg.data_ptr() if want_argmin else None,
                                        status.data_ptr())
    assert rc == 0
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert torch.equal(out, ref_out)
    if want_argmin:
        assert torch.equal(arg, ref_arg)
    for b in range(0, batch, max(1, batch // 5)):
        ro, ra = oracle.minplus_argmin(A[b], w[b], B[b])
        assert np.array_equal(out[b].cpu().numpy(), ro)
        if want_argmin:
            assert np.array_equal(arg[b].cpu().numpy(), ra)


def test_no_alloc_entry_point_matches_the_allocating_one():
    from paper_1802_04924_amd import Context
    rng = np.random.default_rng(7)
    with Context(0) as ctx:
        # split tiles (few tiles, long c range), then a smaller input of another shape
        run_both(ctx, *draw(rng, 3, 130, 2100, 140, 1 << 20))
        run_both(ctx, *draw(rng, 2, 70, 300, 65, 1 << 20))
        # a batch of many tiles, then fewer and smaller products, heavy ties
        run_both(ctx, *draw(rng, 40, 256, 256, 256, 3))
        run_both(ctx, *draw(rng, 5, 100, 64, 200, 3))
        # values too wide for packed keys (compare/select variant), and the minimum-only variant
        run_both(ctx, *draw(rng, 2, 90, 500, 77, (1 << 29) - 1))
        run_both(ctx, *draw(rng, 3, 130, 2100, 140, 1 << 20), want_argmin=False)
        run_both(ctx, *draw(rng, 1, 64, 100, 64, 1 << 20), want_argmin=False)


def test_no_alloc_entry_point_limits_and_status():
    import torch
    from paper_1802_04924_amd import binding
    lib = binding.load()
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    p = t.data_ptr()
    too_many = binding.NOALLOC_MAX_BATCH + 1
    assert lib.lwp_eliminate_node_noalloc(None, too_many, 1, 1, 1, p, p, p, p, p, None) == binding.E_TOO_LARGE
    assert b"capacity" in lib.lwp_status_string(binding.E_TOO_LARGE)
    assert lib.lwp_eliminate_node_noalloc(None, 1, 4, 4, 4, None, p, p, p, p, None) == binding.E_INVAL
    assert lib.lwp_eliminate_node_noalloc(None, 1, 4, 1 << 17, 4, p, p, p, p, p, None) == binding.E_INVAL
    # a sum that leaves int32 sets bit 0 of the caller's status word
    big = torch.full((1, 4, 4), (1 << 31) - 1, dtype=torch.int32, device="cuda")
    one = torch.ones((1, 4), dtype=torch.int32, device="cuda")
    zero = torch.zeros((1, 4, 4), dtype=torch.int32, device="cuda")
    out = torch.empty((1, 4, 4), dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    binding.eliminate_node_noalloc(big, one, zero, out, argmin=torch.empty_like(out), status=status)
    torch.cuda.synchronize()
    assert int(status.item()) & 1
