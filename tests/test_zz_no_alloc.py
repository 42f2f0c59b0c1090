"""s2r_decode_noalloc (the decode that takes no workspace and allocates nothing: its
scratch is a static device array of the library) against s2r_decode on the same
inputs, through the C ABI: two calls in a row on one GPU, the second on a smaller
input, so that what the first call left in the shared scratch is still there.
Both calls take the same kernels (bucket reads by gathers), so every output is
compared bit for bit, which is inside the bar the parity tests hold s2r_decode to.
"""

import numpy as np
import pytest
import torch

from paper_2110_02140_amd import binding, pipeline, workloads

pytestmark = pytest.mark.gpu


def _aggregate(wl):
    """Encode and merge on the device; returns the buffers (aggregated sketch and bitmap inside)."""
    b = pipeline.buffers_for(wl, dense_out=True)
    b.encode_all()
    b.merge()
    torch.cuda.synchronize()
    return b


def _decode_both_ways(b, wl, what):
    print(f"[case] {what}: {wl.name} W={wl.W} n={wl.n} d={wl.d} w={wl.w}", flush=True)
    dev = b.device
    cap = b.out_idx.numel()
    # the existing entry point, gather route (the route the new one takes)
    binding.set_decode_strategy(binding.S2R_DECODE_GATHER)
    try:
        b.decode()
    finally:
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)
    torch.cuda.synchronize()
    want_cnt = int(b.out_count.cpu()[0])
    want_idx = b.out_idx[:want_cnt].cpu().numpy().copy()
    want_val = b.out_val[:want_cnt].cpu().numpy().copy()
    want_dense = b.dense_out.cpu().numpy().copy()

    idx = torch.full((cap,), -1, dtype=torch.int32, device=dev)
    val = torch.full((cap,), float("nan"), dtype=torch.float32, device=dev)
    cnt = torch.full((1,), -1, dtype=torch.int64, device=dev)
    dense = torch.full((wl.n,), float("nan"), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    binding.decode_noalloc(b.sketch_sum, b.bitmap_or, wl.n, wl.d, wl.w, wl.seed, idx, val, cnt, dense)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the device's free memory"
    got_cnt = int(cnt.cpu()[0])
    assert got_cnt == want_cnt, f"{what}: count {got_cnt} != {want_cnt}"
    assert np.array_equal(idx[:got_cnt].cpu().numpy(), want_idx), f"{what}: indices"
    assert np.array_equal(val[:got_cnt].cpu().numpy().view(np.uint32), want_val.view(np.uint32)), f"{what}: values"
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), want_dense.view(np.uint32)), f"{what}: dense output"
    assert np.all(idx[got_cnt:].cpu().numpy() == -1), f"{what}: wrote beyond the count"
    return got_cnt


def test_decode_noalloc_equals_decode_on_two_calls_the_second_smaller():
    big = workloads.make_small(4)              # several tiles, dense pockets (whole embedding rows), ragged n
    small = workloads.make_small(1)
    assert small.n < big.n
    bb, bs = _aggregate(big), _aggregate(small)
    c1 = _decode_both_ways(bb, big, "first call")
    c2 = _decode_both_ways(bs, small, "second call, smaller input")
    assert c1 > 0 and c2 > 0
    # and once more on the larger input: the scratch now holds the smaller call's leftovers
    _decode_both_ways(bb, big, "third call, larger again")


def test_decode_noalloc_counts_only_and_rejects_oversize():
    wl = workloads.make_small(3)
    b = _aggregate(wl)
    cnt = torch.full((1,), -1, dtype=torch.int64, device=b.device)
    binding.decode_noalloc(b.sketch_sum, b.bitmap_or, wl.n, wl.d, wl.w, wl.seed, None, None, cnt, None)
    b.decode()
    torch.cuda.synchronize()
    assert int(cnt.cpu()[0]) == int(b.out_count.cpu()[0])
    lib = binding.load()
    too_long = binding.S2R_DECODE_NOALLOC_MAX_N + 1
    st = lib.s2r_decode_noalloc(b.sketch_sum.data_ptr(), b.bitmap_or.data_ptr(), too_long, wl.d, wl.w, wl.seed,
                                None, None, 0, cnt.data_ptr(), None, None)
    assert st == binding.S2R_ERR_SIZE
