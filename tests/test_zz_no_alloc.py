"""The entry point that allocates nothing: pac_mask_from_nonzero_noalloc against pac_mask_from_nonzero,
through the C ABI, bit for bit, on two calls in a row, the second with a smaller input (the static
scratch array keeps the first call's contents)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def _values(n, dtype, seed, dev):
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    v = torch.randn(n, device=dev, generator=gen)
    v[torch.rand(n, device=dev, generator=gen) < 0.6] = 0.0       # pruned positions
    v[::97] = -0.0
    return v.to(dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_noalloc_mask_matches_the_context_entry_point_twice(dtype):
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(0)
    sizes = [(1 << 25) + 12345, 70001]       # several scan tiles and a ragged tail, then much smaller
    ctx = pac.PacContext(max_elems=max(sizes), device=0)
    try:
        for call, n in enumerate(sizes):
            v = _values(n, dtype, 1000 + call, dev)
            words = (n + 63) // 64
            # every output is allocated before the call under test
            mask = torch.full((words,), -1, dtype=torch.int64, device=dev)
            prefix = torch.full((words,), -1, dtype=torch.int32, device=dev)
            nnz = torch.full((1,), -1, dtype=torch.int64, device=dev)
            flags = torch.full((1,), -1, dtype=torch.int32, device=dev)
            torch.cuda.synchronize()
            pac.pac_mask_from_nonzero_noalloc(v, mask, prefix, nnz, flags)
            torch.cuda.synchronize()
            want_mask, want_prefix, want_nnz = ctx.mask_from_nonzero(v)
            torch.cuda.synchronize()
            assert torch.equal(mask, want_mask), f"call {call}: mask differs"
            assert torch.equal(prefix, want_prefix), f"call {call}: prefix differs"
            assert int(nnz.item()) == int(want_nnz.item()) == int((v != 0).sum().item()), f"call {call}: count differs"
            assert int(flags.item()) == 0
    finally:
        ctx.close()


def test_noalloc_rejects_what_it_cannot_take_and_accepts_empty():
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(0)
    lib = pac.load_library()
    nnz = torch.full((1,), -1, dtype=torch.int64, device=dev)
    flags = torch.full((1,), -1, dtype=torch.int32, device=dev)
    st = lib.pac_mask_from_nonzero_noalloc(nnz.data_ptr(), 0, 1 << 32, nnz.data_ptr(), nnz.data_ptr(), 0, 0, 0)
    assert st == -3 and "2^32" in pac.pac_last_error(None)
    st = lib.pac_mask_from_nonzero_noalloc(nnz.data_ptr(), 7, 10, nnz.data_ptr(), nnz.data_ptr(), 0, 0, 0)
    assert st == -1
    st = lib.pac_mask_from_nonzero_noalloc(0, 0, 0, 0, 0, nnz.data_ptr(), flags.data_ptr(), 0)
    torch.cuda.synchronize()
    assert st == 0 and int(nnz.item()) == 0 and int(flags.item()) == 0
