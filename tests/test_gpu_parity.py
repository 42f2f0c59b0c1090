"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.

Bar (from the oracle's arithmetic): bitmaps, index lists and counts bit-exact;
every sketch cell within 1e-5 * M of the float64 oracle, where M is the sum of
|contributions| to that cell (float32 accumulation of k terms in any order errs
by at most (k-1) 2^-24 M; a dropped or doubled term errs by ~M/k); every decoded
value within 1e-5 * max_j M[j, h_j(i)] (the median moves by at most the largest
per-row perturbation).  A slack of a few float32 denormals is added because the
hardware float32 atomic add may flush denormals.
"""

import json
import os

import numpy as np
import pytest
import torch

from oracle import s2r_oracle as orc
from paper_2110_02140_amd import binding, pipeline, workloads

pytestmark = pytest.mark.gpu

STRATEGIES = {"auto": binding.S2R_INSERT_AUTO, "atomic": binding.S2R_INSERT_ATOMIC, "slice": binding.S2R_INSERT_SLICE}


@pytest.fixture(params=["atomic", "slice"])
def strategy(request):
    """Run the test once per way of forming the sketch in s2r_encode."""
    binding.set_insert_strategy(STRATEGIES[request.param])
    yield request.param
    binding.set_insert_strategy(binding.S2R_INSERT_AUTO)

DECODES = {"gather": binding.S2R_DECODE_GATHER, "slice": binding.S2R_DECODE_SLICE, "rows": binding.S2R_DECODE_ROWS}


@pytest.fixture(params=["gather", "slice", "rows"])
def decode_strategy(request):
    """Run the test once per way of reading the buckets in s2r_decode."""
    binding.set_decode_strategy(DECODES[request.param])
    yield request.param
    binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


REL = 1e-5
DENORM_SLACK = 64 * float(np.finfo(np.float32).tiny)


def _oracle_for(wl):
    enc = [orc.encode_sparse(wl.idx[k], wl.val[k], wl.n, wl.d, wl.w, wl.seed) for k in range(wl.W)]
    S, C = orc.merge([e["S"] for e in enc], [e["bitmap"] for e in enc])
    M = np.sum([e["M"] for e in enc], axis=0)
    dec = orc.decode(S, C, wl.n, wl.seed)
    return enc, S, C, M, dec


def _report_strict_errors(what, got, ref):
    """Reported, not gated: how far inside the tolerance the kernels run.  Strict relative error
    |got - ref| / |ref| over the entries whose reference is not zero: its maximum, its 99.9th
    percentile, the share of entries above 1e-5, and the normwise error.  One JSON line per call is
    appended to the file named by S2R_R11_REPORT, if that is set."""
    path = os.environ.get("S2R_R11_REPORT")
    if not path:
        return
    got, ref = np.asarray(got, dtype=np.float64).ravel(), np.asarray(ref, dtype=np.float64).ravel()
    nz = ref != 0
    if not nz.any():
        return
    rel = np.abs(got[nz] - ref[nz]) / np.abs(ref[nz])
    line = dict(what, entries=int(nz.sum()), max_rel=float(rel.max()), p999_rel=float(np.quantile(rel, 0.999)),
                share_above_1e5=float(np.mean(rel > 1e-5)),
                normwise=float(np.linalg.norm(got - ref) / np.linalg.norm(ref)))
    with open(path, "a") as f:
        f.write(json.dumps(line) + "\n")


def _insert_name():
    return {binding.S2R_INSERT_ATOMIC: "atomic", binding.S2R_INSERT_SLICE: "slice"}.get(binding.defaults.insert_strategy, "auto")


def _check_sketch(got, S, M, what):
    got = got.astype(np.float64).reshape(S.shape)
    err = np.abs(got - S)
    bad = err > REL * M + DENORM_SLACK
    assert not bad.any(), f"{what}: {bad.sum()} cells off, worst {err.max():.3e} (M there {M[np.unravel_index(err.argmax(), err.shape)]:.3e})"
    assert np.all(got[M == 0] == 0.0), f"{what}: untouched cells must be zero"


def _run_and_check(wl, dense_out=False, batched=True, slack=0, sort_cap=None):
    print(f"[case] {wl.name} W={wl.W} n={wl.n} d={wl.d} w={wl.w} batched={batched} slack={slack} sort_cap={sort_cap}", flush=True)
    enc, S, C, M, dec = _oracle_for(wl)
    b = pipeline.buffers_for(wl, dense_out=dense_out, slack=slack, sort_cap=sort_cap)
    b.step(batched=batched, fused_merge_decode=batched)   # (per-worker encodes go with separate merge and decode calls)
    torch.cuda.synchronize()
    nnz = b.nnz.cpu().numpy()
    for k in range(wl.W):
        assert nnz[k] == len(enc[k]["idx"]), f"worker {k} nnz"
        assert np.array_equal(pipeline.u64(b.bitmap[k]), enc[k]["bitmap"]), f"worker {k} bitmap"
        assert np.array_equal(b.nz_idx[k][: nnz[k]].cpu().numpy().view(np.uint32), enc[k]["idx"]), f"worker {k} idx"
        assert np.array_equal(b.nz_val[k][: nnz[k]].cpu().numpy(), enc[k]["val"]), f"worker {k} val"
        _check_sketch(b.sketch[k].cpu().numpy(), enc[k]["S"], enc[k]["M"], f"worker {k} sketch")
    assert np.array_equal(pipeline.u64(b.bitmap_or), C), "merged bitmap"
    _check_sketch(b.sketch_sum.cpu().numpy(), S, M, "merged sketch")
    _report_strict_errors({"workload": wl.name, "n": wl.n, "insert": _insert_name(), "of": "merged sketch cells"},
                          b.sketch_sum.cpu().numpy(), S)
    cnt = int(b.out_count.cpu().numpy()[0])
    assert cnt == len(dec["idx"]), "union count"
    assert np.array_equal(b.out_idx[:cnt].cpu().numpy().view(np.uint32), dec["idx"]), "union indices"
    tol = REL * orc.decode_tolerance_mass(M, dec["idx"], wl.seed) + DENORM_SLACK
    got = b.out_val[:cnt].cpu().numpy().astype(np.float64)
    err = np.abs(got - dec["val"])
    assert np.all(err <= tol), f"decoded values: worst {err.max():.3e}"
    _report_strict_errors({"workload": wl.name, "n": wl.n, "insert": _insert_name(), "of": "decoded values"}, got, dec["val"])
    if dense_out:
        dense = b.dense_out.cpu().numpy()
        ref = np.zeros(wl.n)
        ref[dec["idx"]] = dec["val"]
        assert np.array_equal(dense[dec["idx"]], b.out_val[:cnt].cpu().numpy()), "dense output at set bits"
        mask = np.ones(wl.n, dtype=bool)
        mask[dec["idx"]] = False
        assert not dense[mask].any() and not np.signbit(dense[mask]).any(), "dense output must be +0 at unset bits"
    return b, dec


@pytest.mark.parametrize("batched", [True, False], ids=["batch", "per_worker"])
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_small_recipes_match_oracle(cfg, strategy, batched):
    _run_and_check(workloads.make_small(cfg), dense_out=True, batched=batched)


def test_recipe1_full_size(strategy):
    _run_and_check(workloads.make(1), dense_out=True)


@pytest.mark.parametrize("case", range(36))
def test_seeded_random_problems(case):
    """Thirty-six problems drawn from a seeded generator: lengths from one word to a few tiles (ragged),
    1 to 16 rows, 2^6 to 2^16 columns, 1 to 5 workers, isolated non-zeros, runs and fully dense stretches mixed,
    list capacities from exact to generous, each of the insertion strategies and decode routes asked for in
    turn (the library falls back where one does not apply), with and without a dense output."""
    rng = np.random.default_rng(9000 + case)
    n = int(rng.choice([rng.integers(1, 200), rng.integers(200, 70000), rng.integers(70000, 400000)]))
    d = int(rng.integers(1, 17))
    w = 1 << int(rng.integers(6, 17))
    W = int(rng.integers(1, 6))
    idx, val = [], []
    for k in range(W):
        kind = rng.integers(0, 3)
        if kind == 0:                                      # isolated
            m = int(rng.integers(0, max(1, n // 20) + 1))
            i = rng.choice(n, size=min(m, n), replace=False)
        elif kind == 1:                                    # runs of consecutive indices
            starts = rng.choice(n, size=min(n, int(rng.integers(1, 12))), replace=False)
            i = np.concatenate([np.arange(s0, min(n, s0 + int(rng.integers(1, 5000)))) for s0 in starts])
        else:                                              # a dense stretch (tiles with more than 2048 set bits)
            a = int(rng.integers(0, n))
            i = np.arange(a, min(n, a + int(rng.integers(1, 40000))))
        i = np.unique(i).astype(np.uint32)
        idx.append(i)
        v = rng.normal(0, 1, len(i)).astype(np.float32)
        v[v == 0] = 1.0
        val.append(v)
    wl = _custom(n, idx, val, d=d, w=w, W=W, seed=int(rng.integers(0, 2**31)))
    binding.set_insert_strategy([binding.S2R_INSERT_AUTO, binding.S2R_INSERT_ATOMIC, binding.S2R_INSERT_SLICE][case % 3])
    binding.set_decode_strategy([binding.S2R_DECODE_AUTO, binding.S2R_DECODE_GATHER, binding.S2R_DECODE_SLICE,
                                 binding.S2R_DECODE_ROWS][case % 4])
    try:
        _run_and_check(wl, dense_out=bool(case % 5 == 0), batched=bool(case % 2), slack=int(rng.choice([0, 1, 1000])))
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


def test_recipe1_with_lds_sized_sketch(strategy, decode_strategy):
    """Recipe 1 with a 96 KB sketch (w = 2^13): the size at which the sketch is
    two LDS slices; heavy collisions (41 000 union items in 8192 columns)."""
    _run_and_check(workloads.make_cfg1_lds(), dense_out=False)


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_full_size_recipes_match_oracle(cfg, strategy):
    _run_and_check(workloads.make(cfg), batched=(cfg != 3))


def _custom(n, idx, val, d=3, w=64, W=1, seed=0):
    wl = workloads.Workload("custom", 0, W, n, d, w, seed)
    for k in range(W):
        wl.idx.append(np.asarray(idx[k], dtype=np.uint32))
        wl.val.append(np.asarray(val[k], dtype=np.float32))
    return wl


@pytest.mark.parametrize("d,w", [(3, 1 << 14), (3, 1 << 20), (5, 1 << 17)], ids=["one_slice_per_row", "64_slices", "8_slices"])
def test_long_lists_take_several_passes_per_bin(d, w, decode_strategy):
    """Lists of 1.7 million entries per worker: 206 chunks of 8192, more than the lane groups of a slice
    workgroup's waves take in one pass, so every bin is read in several passes; with one slice per row a
    chunk's segment is the whole chunk (the loop over the rest of a long segment), with 64 slices it is
    128 records."""
    n = 1 << 23
    rng = np.random.default_rng(77)
    idx, val = [], []
    for k in range(2):
        i = np.flatnonzero(rng.random(n) < 0.2).astype(np.uint32)
        idx.append(i)
        val.append(rng.normal(0, 1, len(i)).astype(np.float32) + np.float32(2.0))
    binding.set_insert_strategy(binding.S2R_INSERT_SLICE)
    binding.want_report(True)
    try:
        _run_and_check(_custom(n, idx, val, d=d, w=w, W=2, seed=5))
        assert binding.last_insert_strategy() == binding.S2R_INSERT_SLICE
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
        binding.want_report(False)


@pytest.mark.parametrize("n", [1, 63, 64, 65, 2047, 2048, 2049, 4096 + 64, 32768, 32769, 100003])
def test_ragged_lengths_dense_gradient(n, strategy):
    """Every element non-zero: maximal counts, every tile boundary crossed."""
    rng = np.random.default_rng(n)
    idx = [np.arange(n)]
    val = [rng.normal(0, 1, n).astype(np.float32) + 3.0]
    _run_and_check(_custom(n, idx, val, d=3, w=1 << 8), dense_out=True)


@pytest.mark.parametrize("n,dense", [(1, True), (63, False), (2049, True), (32768, False), (32769, True), (100003, False),
                                     (16 * 32768 + 5, True)])
def test_merge_decode_is_merge_then_decode_bit_for_bit(n, dense, decode_strategy):
    """s2r_merge_decode (the merge kernel counts the aggregated bitmap) against s2r_merge followed by
    s2r_decode (which counts it itself) on the same encoded workers: every output identical, also for
    lengths whose last piece, tile or word is ragged, for empty tiles in the middle, for a dense output."""
    rng = np.random.default_rng(1000 + n)
    W = 3
    idx, val = [], []
    for k in range(W):
        m = min(n, max(1, n // (k + 2)))
        i = np.sort(rng.choice(n, m, replace=False))
        if n > 5 * 32768:                                  # leave tiles 2 and 3 empty
            i = i[(i < 2 * 32768) | (i >= 4 * 32768)]
        idx.append(i)
        val.append(rng.normal(0, 1, len(i)).astype(np.float32) + 2.0)
    wl = _custom(n, idx, val, d=3, w=1 << 9, W=W)
    b = pipeline.buffers_for(wl, dense_out=dense)
    names = ("sketch_sum", "bitmap_or", "out_idx", "out_val", "out_count") + (("dense_out",) if dense else ())
    b.encode_all()                                         # (atomic insertions differ from run to run: encode once)
    _same_outputs_from_both_call_sequences(b, names)
    assert int(b.out_count.cpu()[0]) == len(np.unique(np.concatenate(idx)))


def _same_outputs_from_both_call_sequences(b, names):
    def run(call):
        for name in names:
            getattr(b, name).fill_(0)
        call()
        torch.cuda.synchronize()
        return {name: getattr(b, name).cpu().numpy().copy() for name in names}
    two_calls = run(lambda: (b.merge(), b.decode()))
    one_call = run(b.merge_decode)
    for name in names:
        assert np.array_equal(two_calls[name].view(np.uint8), one_call[name].view(np.uint8)), name


@pytest.mark.parametrize("n,B", [(1000, 7), (70000, 650), (200001, 64), (3 * 32768 * 16 + 11, 16)])
def test_merge_decode_blocks_is_merge_then_decode_blocks_bit_for_bit(n, B, decode_strategy):
    rng = np.random.default_rng(n + B)
    W = 2
    idx = [np.sort(rng.choice(n, max(1, n // 50), replace=False)) for _ in range(W)]
    val = [rng.normal(0, 1, len(i)).astype(np.float32) + 2.0 for i in idx]
    wl = _custom(n, idx, val, d=3, w=1 << 9, W=W)
    b = pipeline.block_buffers_for(wl, B)
    b.encode_all()
    _same_outputs_from_both_call_sequences(b, ("sketch_sum", "bitmap_or", "out_blk", "out_val", "out_count"))


@pytest.mark.parametrize("dense_out", [False, True], ids=["lists", "lists+dense"])
def test_tiles_around_the_expansion_group_size(strategy, dense_out):
    """Tiles (32768 elements) holding 0, 1, 2047, 2048, 2049, 4096, 4097 and 32768
    non-zeros, the last tile ragged: every boundary of the 2048-position groups into
    which the expansion kernels cut a dense tile, with and without the dense output
    (which makes decode launch the tiles' first groups and the further ones apart)."""
    tile = 32768
    counts = [2049, 0, 32768, 1, 2048, 4097, 2047, 4096, 32768, 700]
    n = tile * (len(counts) - 1) + 1000
    rng = np.random.default_rng(77)
    idx, val = [], []
    for k in range(2):
        parts = []
        for t, c in enumerate(counts):
            span = min(tile, n - t * tile)
            pick = np.arange(span) if c >= span else np.sort(rng.choice(span, size=c, replace=False))
            parts.append(t * tile + pick)
        i = np.concatenate(parts).astype(np.uint32)
        idx.append(i)
        val.append((rng.normal(0, 1, len(i)) + 2.5).astype(np.float32))
    _run_and_check(_custom(n, idx, val, d=3, w=1 << 10, W=2), dense_out=dense_out)


def test_dense_tiles_with_an_estimate_far_too_small(strategy, decode_strategy):
    """Every element set (sixteen further groups per tile) while the caller expects one non-zero: the few
    workgroups launched for the dense-tile list walk all of its entries."""
    n = 20 * 32768 + 77
    rng = np.random.default_rng(5)
    idx = [np.arange(n)] * 2
    val = [(rng.normal(0, 1, n) + 3.0).astype(np.float32) for _ in range(2)]
    binding.set_expected_nnz(1, 1)
    try:
        _run_and_check(_custom(n, idx, val, d=3, w=1 << 10, W=2))
    finally:
        binding.set_expected_nnz(0, 0)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_small_recipes_both_decodes(cfg, decode_strategy):
    """Without a dense output the decode may take either route; with one (the
    tests above) it gathers."""
    b, _ = _run_and_check(workloads.make_small(cfg))
    assert binding.last_decode_strategy() == DECODES[decode_strategy]


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_full_size_recipes_both_decodes(cfg, decode_strategy):
    _run_and_check(workloads.make(cfg))
    assert binding.last_decode_strategy() == DECODES[decode_strategy]


@pytest.mark.parametrize("n", [1, 65, 8191, 8192, 8193, 3 * 8192 + 5, 100003])
def test_decode_by_slices_dense_gradient_chunk_boundaries(n):
    """Every element set: list chunks (8192 positions) full, ragged and single."""
    binding.set_decode_strategy(binding.S2R_DECODE_SLICE)
    try:
        rng = np.random.default_rng(n)
        wl = _custom(n, [np.arange(n)] * 2, [rng.normal(0, 1, n).astype(np.float32) + 3.0 for _ in range(2)],
                     d=5, w=1 << 9, W=2)
        _run_and_check(wl)
        assert binding.last_decode_strategy() == binding.S2R_DECODE_SLICE
    finally:
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


@pytest.mark.parametrize("d,w", [(1, 1), (2, 4), (4, 1 << 14), (6, 1 << 15), (7, 1 << 3), (8, 1 << 16), (9, 1 << 6)])
def test_decode_by_slices_rows_and_widths(d, w):
    """Even and odd d up to the route's limit of 8 rows (d = 9 must gather), widths
    below, at and above one LDS slice."""
    binding.set_decode_strategy(binding.S2R_DECODE_SLICE)
    try:
        rng = np.random.default_rng(100 * d + 7)
        n = 70001
        idx = [np.sort(rng.choice(n, 9000, replace=False)) for _ in range(3)]
        val = [rng.normal(0, 1, 9000).astype(np.float32) for _ in range(3)]
        _run_and_check(_custom(n, idx, val, d=d, w=w, W=3))
        want = binding.S2R_DECODE_SLICE if d <= 8 else binding.S2R_DECODE_GATHER
        assert binding.last_decode_strategy() == want
    finally:
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


def test_decode_by_slices_respects_capacity():
    """Union of 30000 indices, lists of 20000: the first 20000 entries, the true
    count, nothing beyond the lists."""
    binding.set_decode_strategy(binding.S2R_DECODE_SLICE)
    try:
        rng = np.random.default_rng(3)
        n, cap = 200000, 20000
        idx = np.sort(rng.choice(n, 30000, replace=False)).astype(np.uint32)
        val = rng.normal(0, 1, 30000).astype(np.float32)
        wl = _custom(n, [idx], [val], d=3, w=1 << 12)
        b = pipeline.buffers_for(wl)
        b.out_idx = torch.full((cap + 16,), -1, dtype=torch.int32, device="cuda")[:cap]
        b.out_val = torch.full((cap + 16,), -7.0, dtype=torch.float32, device="cuda")[:cap]
        b.step()
        torch.cuda.synchronize()
        assert binding.last_decode_strategy() == binding.S2R_DECODE_SLICE
        assert int(b.out_count.cpu()[0]) == 30000
        assert np.array_equal(b.out_idx.cpu().numpy().view(np.uint32), idx[:cap])
        assert (b.out_idx._base[cap:].cpu().numpy() == -1).all() and (b.out_val._base[cap:].cpu().numpy() == -7.0).all()
        enc = orc.encode_sparse(idx, val, n, 3, 1 << 12, 0)
        dec = orc.decode(enc["S"], enc["bitmap"], n, 0)
        tol = REL * orc.decode_tolerance_mass(enc["M"], dec["idx"][:cap], 0) + DENORM_SLACK
        assert np.all(np.abs(b.out_val.cpu().numpy().astype(np.float64) - dec["val"][:cap]) <= tol)
    finally:
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


def test_both_decodes_return_identical_values():
    """The two routes read the same cells and take the same median: bit-identical."""
    wl = workloads.make_small(4)
    b = pipeline.buffers_for(wl)
    b.encode_all()
    b.merge()
    got = {}
    for name, st in DECODES.items():
        binding.set_decode_strategy(st)
        b.out_val.fill_(0)
        b.decode()
        torch.cuda.synchronize()
        cnt = int(b.out_count.cpu()[0])
        got[name] = (b.out_idx[:cnt].cpu().numpy().copy(), b.out_val[:cnt].cpu().numpy().copy())
    binding.set_decode_strategy(binding.S2R_DECODE_AUTO)
    assert np.array_equal(got["gather"][0], got["slice"][0])
    assert np.array_equal(got["gather"][1].view(np.uint32), got["slice"][1].view(np.uint32))


def test_all_zero_gradient(strategy):
    wl = _custom(5000, [np.empty(0, dtype=np.uint32)] * 2, [np.empty(0, dtype=np.float32)] * 2, W=2)
    b, dec = _run_and_check(wl, dense_out=True)
    assert int(b.out_count.cpu()[0]) == 0 and not b.sketch_sum.cpu().numpy().any()


def test_special_values_follow_the_bit_pattern_rule():
    n = 300
    g = np.zeros(n, dtype=np.float32)
    g[5] = -0.0                      # zero
    g[6] = 1e-42                     # denormal: counted as non-zero
    g[70] = -1e-45
    g[129] = 2.5
    g[299] = -7.0
    wl = _custom(n, [np.flatnonzero(orc.nonzero_mask(g))], [g[orc.nonzero_mask(g)]], d=3, w=1 << 10)
    b = pipeline.buffers_for(wl)
    b.grads[0] = torch.from_numpy(g).cuda()       # keeps the -0.0 in the dense input
    b.step()
    torch.cuda.synchronize()
    enc = orc.encode(g, wl.d, wl.w, wl.seed)
    assert int(b.nnz.cpu()[0]) == 4
    assert np.array_equal(pipeline.u64(b.bitmap[0]), enc["bitmap"])
    assert b.nz_idx[0][:4].cpu().numpy().tolist() == [6, 70, 129, 299]
    assert np.array_equal(b.nz_val[0][:4].cpu().numpy(), g[[6, 70, 129, 299]])


@pytest.mark.parametrize("d", [1, 2, 3, 4, 5])
def test_nan_and_infinities_poison_what_the_oracle_says_they_poison(d, strategy, decode_strategy):
    """A NaN, a +Inf and a -Inf among the gradient values are non-zero entries like any other: they
    are listed and inserted, their buckets become non-finite, and the median takes them in the total
    order of a sort (NaN last), so every decoded value is non-finite exactly where the oracle's is,
    with the same class (NaN, +Inf, -Inf), and within the tolerance elsewhere."""
    rng = np.random.default_rng(31 + d)
    n, W, w = 30000, 2, 256                       # narrow rows: the poisoned buckets are shared with many indices
    idx = [np.sort(rng.choice(n, 2000, replace=False)).astype(np.uint32) for _ in range(W)]
    val = [rng.normal(0, 1, 2000).astype(np.float32) + 3.0 for _ in range(W)]
    val[0][10], val[0][500], val[0][900] = np.nan, np.inf, -np.inf
    val[1][700], val[1][1300] = np.inf, -np.inf
    wl = _custom(n, idx, val, d=d, w=w, W=W, seed=5)
    enc, S, C, M, dec = _oracle_for(wl)
    b = pipeline.buffers_for(wl)
    b.step()
    torch.cuda.synchronize()
    for k in range(W):
        cnt = int(b.nnz.cpu()[k])
        assert cnt == len(idx[k])
        assert np.array_equal(b.nz_idx[k][:cnt].cpu().numpy().view(np.uint32), idx[k])
        assert np.array_equal(b.nz_val[k][:cnt].cpu().numpy().view(np.uint32), val[k].view(np.uint32))
    assert np.array_equal(pipeline.u64(b.bitmap_or), C)

    def same_class(got, ref, M_of, what):
        got, ref = np.asarray(got, dtype=np.float64).ravel(), np.asarray(ref, dtype=np.float64).ravel()
        fin = np.isfinite(ref)
        assert np.array_equal(np.isnan(got), np.isnan(ref)), f"{what}: NaN positions"
        assert np.array_equal(np.isposinf(got), np.isposinf(ref)) and np.array_equal(np.isneginf(got), np.isneginf(ref)), \
            f"{what}: infinities"
        # (an entry that reads a poisoned bucket besides its finite ones is judged against the largest finite mass)
        m = np.where(np.isfinite(M_of), M_of, np.max(M[np.isfinite(M)]))
        with np.errstate(invalid="ignore"):
            assert np.all(np.abs(got[fin] - ref[fin]) <= REL * m.ravel()[fin] + DENORM_SLACK), f"{what}: finite entries"
        return int((~fin).sum())

    bad_cells = same_class(b.sketch_sum.cpu().numpy(), S, M, "merged sketch")
    cnt = int(b.out_count.cpu()[0])
    assert cnt == len(dec["idx"]) and np.array_equal(b.out_idx[:cnt].cpu().numpy().view(np.uint32), dec["idx"])
    bad_vals = same_class(b.out_val[:cnt].cpu().numpy(), dec["val"], orc.decode_tolerance_mass(M, dec["idx"], wl.seed),
                          "decoded values")
    assert bad_cells >= d and bad_vals > 0, "the case must poison something"


@pytest.mark.parametrize("d,w", [(1, 1), (1, 64), (2, 2), (4, 128), (5, 1 << 12), (6, 32), (7, 64), (8, 64), (16, 16)])
def test_rows_and_widths(d, w, strategy):
    rng = np.random.default_rng(d * 1000 + w)
    n, W = 20011, 3
    idx = [np.sort(rng.choice(n, 700, replace=False)) for _ in range(W)]
    val = [rng.normal(0, 0.01, 700).astype(np.float32) for _ in range(W)]
    _run_and_check(_custom(n, idx, val, d=d, w=w, W=W, seed=d), dense_out=True)


def test_capacity_overflow_reports_true_count_and_keeps_prefix(strategy):
    rng = np.random.default_rng(77)
    n = 50000
    idx = np.sort(rng.choice(n, 3000, replace=False))
    val = rng.normal(0, 1, 3000).astype(np.float32)
    wl = _custom(n, [idx], [val], d=3, w=1 << 10)
    b = pipeline.buffers_for(wl)
    b.nz_idx[0] = torch.full((1000 + 16,), -1, dtype=torch.int32, device="cuda")[:1000]
    b.nz_val[0] = torch.zeros(1000, dtype=torch.float32, device="cuda")
    guard = b.nz_idx[0]._base[1000:]
    b.encode(0)
    torch.cuda.synchronize()
    assert int(b.nnz.cpu()[0]) == 3000
    assert np.array_equal(b.nz_idx[0].cpu().numpy().view(np.uint32), idx[:1000].astype(np.uint32))
    assert (guard.cpu().numpy() == -1).all(), "nothing written past cap"
    enc = orc.encode_sparse(idx, val, n, 3, 1 << 10, 0)
    _check_sketch(b.sketch[0].cpu().numpy(), enc["S"], enc["M"], "sketch is complete despite the short list")


def test_capacity_inside_a_dense_tile(strategy):
    """A fully dense gradient of three tiles with list capacities that end inside
    a later 2048-position group of the second tile: encode and decode write exactly
    the first cap entries, report the true counts, and the sketch stays complete."""
    rng = np.random.default_rng(5)
    n, cap = 3 * 32768 - 100, 32768 + 5000
    idx = np.arange(n, dtype=np.uint32)
    val = (rng.normal(0, 1, n) + 3.0).astype(np.float32)
    wl = _custom(n, [idx], [val], d=3, w=1 << 12)
    b = pipeline.buffers_for(wl)
    b.nz_idx[0] = torch.full((cap + 16,), -1, dtype=torch.int32, device="cuda")[:cap]
    b.nz_val[0] = torch.zeros(cap, dtype=torch.float32, device="cuda")
    b.out_idx = torch.full((cap + 16,), -1, dtype=torch.int32, device="cuda")[:cap]
    b.out_val = torch.zeros(cap, dtype=torch.float32, device="cuda")
    b.step()
    torch.cuda.synchronize()
    assert int(b.nnz.cpu()[0]) == n and int(b.out_count.cpu()[0]) == n
    assert np.array_equal(b.nz_idx[0].cpu().numpy().view(np.uint32), idx[:cap])
    assert np.array_equal(b.nz_val[0].cpu().numpy(), val[:cap])
    assert (b.nz_idx[0]._base[cap:].cpu().numpy() == -1).all(), "encode wrote past cap"
    assert np.array_equal(b.out_idx.cpu().numpy().view(np.uint32), idx[:cap])
    assert (b.out_idx._base[cap:].cpu().numpy() == -1).all(), "decode wrote past cap"
    enc = orc.encode_sparse(idx, val, n, 3, 1 << 12, 0)
    _check_sketch(b.sketch[0].cpu().numpy(), enc["S"], enc["M"], "sketch is complete despite the short list")
    dec = orc.decode(enc["S"], enc["bitmap"], n, 0)
    tol = REL * orc.decode_tolerance_mass(enc["M"], dec["idx"][:cap], 0) + DENORM_SLACK
    assert np.all(np.abs(b.out_val.cpu().numpy().astype(np.float64) - dec["val"][:cap]) <= tol)


def test_null_lists_and_in_place_merge():
    wl = workloads.make_small(3)
    enc, S, C, M, dec = _oracle_for(wl)
    b = pipeline.buffers_for(wl)
    for k in range(wl.W):
        binding.encode(b.grads[k], wl.d, wl.w, wl.seed, b.sketch[k], b.bitmap[k], None, None, b.nnz[k:k + 1],
                       b.workspace)
    binding.merge(b.sketch, b.bitmap, wl.n, wl.d, wl.w, wl.seed, b.sketch[0], b.bitmap[0])   # in place
    binding.decode(b.sketch[0], b.bitmap[0], wl.n, wl.d, wl.w, wl.seed, None, None, b.out_count, None, b.workspace)
    torch.cuda.synchronize()
    assert b.nnz.cpu().numpy().tolist() == [len(e["idx"]) for e in enc]
    assert np.array_equal(pipeline.u64(b.bitmap[0]), C)
    _check_sketch(b.sketch[0].cpu().numpy(), S, M, "in-place merged sketch")
    assert int(b.out_count.cpu()[0]) == len(dec["idx"])


@pytest.mark.parametrize("cfg", [1, 3])
def test_merge_with_bitmaps_at_8_byte_offsets_and_odd_word_counts(cfg):
    """Bitmaps need 8-byte alignment only: s2r_merge on views that start 8 bytes into their
    allocations, with an odd and an even number of words, writes exactly the words it owns."""
    wl = workloads.make_small(cfg)
    enc, S, C, M, dec = _oracle_for(wl)
    nw = pipeline.words_of(wl.n)
    b = pipeline.buffers_for(wl)
    b.encode_all()
    for shift in (0, 1):                                   # shift 1: views that start 8 bytes into an allocation
        hold = [torch.zeros(nw + 2, dtype=torch.int64, device="cuda") for _ in range(wl.W + 1)]
        views = [h[shift:shift + nw] for h in hold]
        for k in range(wl.W):
            views[k].copy_(b.bitmap[k])
        assert all((v.data_ptr() % 16 == 8) == bool(shift) for v in views)
        binding.merge(b.sketch, views[:wl.W], wl.n, wl.d, wl.w, wl.seed, b.sketch_sum, views[wl.W])
        torch.cuda.synchronize()
        assert np.array_equal(pipeline.u64(views[wl.W].contiguous()), C), f"shift {shift}, {nw} words"
        for h in hold:                                     # nothing outside the nw words is written
            assert int(h[:shift].abs().sum()) == 0 and int(h[shift + nw:].abs().sum()) == 0


def test_linearity_on_device(strategy):
    """Sum of the workers' sketches == sketch of the summed gradient."""
    wl = workloads.make_small(2)
    b = pipeline.buffers_for(wl)
    b.step()
    total = torch.zeros(wl.n, dtype=torch.float64, device="cuda")
    for g in b.grads:
        total += g.double()
    gsum = total.float()
    b2 = pipeline.Buffers(1, wl.n, wl.d, wl.w, wl.seed, wl.n, wl.n)
    b2.grads.append(gsum)
    b2.encode(0)
    torch.cuda.synchronize()
    _, S, _, M, _ = _oracle_for(wl)
    diff = np.abs(b.sketch_sum.cpu().numpy().astype(np.float64) - b2.sketch[0].cpu().numpy().astype(np.float64))
    # the float32 cast of the summed gradient adds up to 2^-24 relative per element
    assert np.all(diff.reshape(M.shape) <= 2 * REL * M + DENORM_SLACK)


def test_runs_are_repeatable_bit_exact_in_the_integer_outputs():
    wl = workloads.make_small(4)
    b = pipeline.buffers_for(wl)
    b.step()
    torch.cuda.synchronize()
    first = (b.out_idx.clone(), b.out_count.clone(), [x.clone() for x in b.bitmap], [x.clone() for x in b.nz_idx])
    for _ in range(3):
        b.step()
    torch.cuda.synchronize()
    cnt = int(first[1][0])
    assert torch.equal(first[1], b.out_count) and torch.equal(first[0][:cnt], b.out_idx[:cnt])
    for a, c in zip(first[2], b.bitmap):
        assert torch.equal(a, c)
    for k, (a, c) in enumerate(zip(first[3], b.nz_idx)):
        m = int(b.nnz[k])
        assert torch.equal(a[:m], c[:m])


@pytest.mark.parametrize("expected", [0, 1, 3000, 10**9])
def test_capacity_far_above_the_count_and_estimates_that_are_wrong(strategy, decode_strategy, expected):
    """Lists eleven times longer than the non-zero count, and estimates of the count (which only size
    launches) from absent over far too small to far too large: every output as always."""
    wl = workloads.make_small(4)
    binding.set_expected_nnz(expected, expected)
    try:
        _run_and_check(wl, slack=10 * max(len(i) for i in wl.idx))
        assert binding.last_insert_strategy() == STRATEGIES[strategy]
        assert binding.last_decode_strategy() == DECODES[decode_strategy]
    finally:
        binding.set_expected_nnz(0, 0)


@pytest.mark.parametrize("asked", ["auto", "slice"])
@pytest.mark.parametrize("cfg", [2, 4, 5])
def test_lists_as_long_as_the_gradient_with_a_workspace_for_the_expected_count(cfg, asked):
    """A caller who cannot bound its non-zeros passes lists of n entries, says how many it expects, and sizes
    the workspace for that: the slice strategy is still there to be taken (its sort takes what the workspace
    holds; anything beyond would be inserted with atomics), and the library's own choice gives the same
    outputs."""
    wl = workloads.make_small(cfg)
    most = max(len(i) for i in wl.idx)
    binding.set_expected_nnz(most, 0)
    binding.set_insert_strategy(STRATEGIES[asked])
    binding.want_report(True)
    try:
        _run_and_check(wl, slack=wl.n - most, sort_cap=most + most // 4)
        if asked == "slice":
            assert binding.last_insert_strategy() == binding.S2R_INSERT_SLICE
    finally:
        binding.set_expected_nnz(0, 0)
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
        binding.want_report(False)


@pytest.mark.parametrize("fraction", [0.001, 0.3, 0.999])
def test_slice_strategy_with_a_workspace_for_a_part_of_the_lists(fraction):
    """The slice strategy asked for, with a workspace whose record area holds only a part of the listed
    non-zeros: the sort takes what fits, the rest is inserted with atomics after the slices are stored;
    lists and sketches are as always."""
    wl = workloads.make_small(4)
    most = max(len(i) for i in wl.idx)
    binding.set_insert_strategy(binding.S2R_INSERT_SLICE)
    try:
        _run_and_check(wl, sort_cap=max(1, int(fraction * most)))
        assert binding.last_insert_strategy() == binding.S2R_INSERT_SLICE
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)


def test_auto_strategy_matches_oracle_on_every_small_recipe():
    binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
    for cfg in (1, 2, 3, 4, 5):
        _run_and_check(workloads.make_small(cfg))


def test_strategy_argument_check():
    with pytest.raises(binding.S2RError):
        binding.set_insert_strategy(7)
    binding.set_insert_strategy(binding.S2R_INSERT_AUTO)


@pytest.mark.parametrize("asked", ["auto", "atomic"])
def test_recipe5_full_size_in_the_benchmarked_configuration(asked, request):
    """The workload bench.py times (W=16, n=1e9, 64 GB of dense input), with the
    library's own choice of strategy (the benchmarked one) and with atomics: every
    worker's count, bitmap, index list and sketch; the merged bitmap and sketch;
    every decoded index and value."""
    binding.set_insert_strategy(STRATEGIES[asked])
    request.addfinalizer(lambda: binding.set_insert_strategy(binding.S2R_INSERT_AUTO))
    wl = workloads.make(5)
    print(f"[case] {wl.name} full size", flush=True)
    b = pipeline.buffers_for(wl)
    b.step()
    torch.cuda.synchronize()
    nnz = b.nnz.cpu().numpy()
    S = np.zeros((wl.d, wl.w))
    M = np.zeros((wl.d, wl.w))
    C = np.zeros((wl.n + 63) // 64, dtype=np.uint64)
    for k in range(wl.W):
        e = orc.encode_sparse(wl.idx[k], wl.val[k], wl.n, wl.d, wl.w, wl.seed)
        assert nnz[k] == len(e["idx"]), f"worker {k} nnz"
        assert np.array_equal(pipeline.u64(b.bitmap[k]), e["bitmap"]), f"worker {k} bitmap"
        assert np.array_equal(b.nz_idx[k][: nnz[k]].cpu().numpy().view(np.uint32), e["idx"]), f"worker {k} idx"
        assert np.array_equal(b.nz_val[k][: nnz[k]].cpu().numpy(), e["val"]), f"worker {k} val"
        _check_sketch(b.sketch[k].cpu().numpy(), e["S"], e["M"], f"worker {k} sketch")
        S += e["S"]
        M += e["M"]
        C |= e["bitmap"]
        print(f"  worker {k} ok", flush=True)
    assert np.array_equal(pipeline.u64(b.bitmap_or), C), "merged bitmap"
    _check_sketch(b.sketch_sum.cpu().numpy(), S, M, "merged sketch")
    _report_strict_errors({"workload": wl.name, "n": wl.n, "insert": _insert_name(), "of": "merged sketch cells"},
                          b.sketch_sum.cpu().numpy(), S)
    dec = orc.decode(S, C, wl.n, wl.seed)
    cnt = int(b.out_count.cpu()[0])
    assert cnt == len(dec["idx"])
    assert np.array_equal(b.out_idx[:cnt].cpu().numpy().view(np.uint32), dec["idx"])
    tol = REL * orc.decode_tolerance_mass(M, dec["idx"], wl.seed) + DENORM_SLACK
    err = np.abs(b.out_val[:cnt].cpu().numpy().astype(np.float64) - dec["val"])
    assert np.all(err <= tol), f"decoded values: worst {err.max():.3e}"
    _report_strict_errors({"workload": wl.name, "n": wl.n, "insert": _insert_name(), "of": "decoded values"},
                          b.out_val[:cnt].cpu().numpy(), dec["val"])


def test_batch_with_null_lists_and_argument_checks():
    wl = workloads.make_small(1)
    enc, S, C, M, dec = _oracle_for(wl)
    b = pipeline.buffers_for(wl)
    binding.encode_batch(b.grads, wl.n, wl.d, wl.w, wl.seed, b.sketch, b.bitmap, None, None, b.nnz, b.workspace)
    torch.cuda.synchronize()
    assert b.nnz.cpu().numpy().tolist() == [len(e["idx"]) for e in enc]
    for k in range(wl.W):
        assert np.array_equal(pipeline.u64(b.bitmap[k]), enc[k]["bitmap"])
        _check_sketch(b.sketch[k].cpu().numpy(), enc[k]["S"], enc[k]["M"], f"worker {k} sketch")
    small = b.workspace[: binding.workspace_bytes(wl.n, wl.d, wl.w)]        # enough for one worker only
    with pytest.raises(binding.S2RError) as ei:
        binding.encode_batch(b.grads, wl.n, wl.d, wl.w, wl.seed, b.sketch, b.bitmap, None, None, b.nnz, small)
    assert ei.value.status == binding.S2R_ERR_WORKSPACE


def test_large_gradients_are_scanned_worker_by_worker():
    """n*4 >= 1 GiB with atomics: the batch is zeroed and scanned one worker per
    launch (first_worker advances), everything else in single launches."""
    binding.set_insert_strategy(binding.S2R_INSERT_ATOMIC)
    try:
        rng = np.random.default_rng(5)
        n, W, d, w = (1 << 28) + 77, 3, 3, 1 << 12
        idx = [np.sort(rng.choice(n, 2000, replace=False)) for _ in range(W)]
        val = [rng.normal(0, 0.01, 2000).astype(np.float32) for _ in range(W)]
        _run_and_check(_custom(n, idx, val, d=d, w=w, W=W, seed=3))
        assert binding.scan_launch_workers() == 1
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)


def test_estimation_quality_matches_oracle_and_improves_with_sketch_size():
    """The relative error of the decoded sum (quality.py) equals the oracle's on the
    same inputs, falls as the sketch grows, and is smaller with 3 rows than with 1
    at equal width (median of independent estimates, Section 3.1)."""
    from paper_2110_02140_amd import quality
    errs = {}
    for d in (1, 3):
        for L in (10, 13, 16):
            wl = workloads.cfg1(W=3, n=1 << 18, density=0.01, d=d, w=1 << L)
            r = quality.relative_error(wl)
            ref = orc.reduce_workers([wl.dense(k) for k in range(wl.W)], d, 1 << L, wl.seed)
            union, total = quality.true_sum(wl)
            assert np.array_equal(ref["idx"], union)
            ref_err = np.linalg.norm(ref["val"] - total) / np.linalg.norm(total)
            assert abs(r["rel_error"] - ref_err) <= 1e-4 * max(ref_err, 1e-3), (d, L, r["rel_error"], ref_err)
            errs[(d, L)] = r["rel_error"]
    for d in (1, 3):
        assert errs[(d, 10)] > errs[(d, 13)] > errs[(d, 16)]
    assert errs[(3, 13)] < errs[(1, 13)] and errs[(3, 16)] < errs[(1, 16)]


# ---------------------------------------------------------------- block-granular codec
def _oracle_blocks(wl, B):
    """The block oracle from the workload's sparse form (dense buffers only for small n)."""
    gs = [wl.dense(k) for k in range(wl.W)]
    return orc.reduce_workers_blocks(gs, B, wl.d, wl.w, wl.seed)


def _run_blocks_and_check(wl, B, batched=True):
    print(f"[case] blocks {wl.name} W={wl.W} n={wl.n} B={B} d={wl.d} w={wl.w} batched={batched}", flush=True)
    ref = _oracle_blocks(wl, B)
    b = pipeline.block_buffers_for(wl, B)
    b.step(batched=batched, fused_merge_decode=batched)   # (per-worker encodes go with separate merge and decode calls)
    torch.cuda.synchronize()
    nblk = b.nblk.cpu().numpy()
    for k in range(wl.W):
        e = ref["workers"][k]
        assert nblk[k] == len(e["blocks"]), f"worker {k} block count"
        assert np.array_equal(pipeline.u64(b.bitmap[k]), e["bitmap"]), f"worker {k} block bitmap"
        assert np.array_equal(b.blk_idx[k][: nblk[k]].cpu().numpy().view(np.uint32), e["blocks"]), f"worker {k} block list"
        _check_sketch(b.sketch[k].cpu().numpy(), e["S"], e["M"], f"worker {k} sketch")
    assert np.array_equal(pipeline.u64(b.bitmap_or), ref["bitmap"]), "merged block bitmap"
    _check_sketch(b.sketch_sum.cpu().numpy(), ref["S"], ref["M"], "merged sketch")
    cnt = int(b.out_count.cpu()[0])
    assert cnt == len(ref["blocks"]), "set blocks"
    assert np.array_equal(b.out_blk[:cnt].cpu().numpy().view(np.uint32), ref["blocks"])
    got = b.out_val[: cnt * B].cpu().numpy().astype(np.float64)
    want = ref["val"].reshape(-1)
    elems = (ref["blocks"].astype(np.int64)[:, None] * B + np.arange(B)[None, :]).reshape(-1)
    inside = elems < wl.n
    tol = np.zeros(len(elems))
    tol[inside] = REL * orc.decode_tolerance_mass(ref["M"], elems[inside].astype(np.uint32), wl.seed) + DENORM_SLACK
    assert np.all(np.abs(got - want) <= tol), f"block values: worst {np.abs(got - want).max():.3e}"
    assert not got[~inside].any(), "positions beyond the gradient must hold 0"
    return b, ref


@pytest.mark.parametrize("batched", [True, False], ids=["batch", "per_worker"])
@pytest.mark.parametrize("cfg,B", [(1, 1), (1, 37), (2, 25), (3, 64), (3, 256), (4, 96), (5, 1000)])
def test_small_recipes_block_codec(cfg, B, strategy, decode_strategy, batched):
    _run_blocks_and_check(workloads.make_small(cfg), B, batched=batched)


@pytest.mark.parametrize("cfg,B", [(2, 650), (3, 256)])
def test_full_size_recipes_block_codec(cfg, B):
    """Configs 2 and 3 with their natural blocks (embedding rows of 650, blocks of 256),
    in the library's own choice of strategies."""
    _run_blocks_and_check(workloads.make(cfg), B)


@pytest.mark.parametrize("case", range(24))
def test_block_codec_seeded_random_problems(case):
    """Two dozen seeded problems for the block-granular codec: block sizes from 1 to beyond the gradient,
    ragged last blocks, isolated non-zeros and runs, every strategy and route asked for in turn."""
    rng = np.random.default_rng(7000 + case)
    n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 60000), rng.integers(60000, 300000)]))
    B = int(rng.choice([1, 2, 7, 64, 100, 256, 650, 1000, 4096, n + 5]))
    d = int(rng.integers(1, 9))
    w = 1 << int(rng.integers(6, 15))
    W = int(rng.integers(1, 5))
    idx, val = [], []
    for k in range(W):
        if rng.integers(0, 2) == 0:
            i = rng.choice(n, size=min(n, int(rng.integers(0, max(1, n // 30) + 1))), replace=False)
        else:
            starts = rng.choice(n, size=min(n, int(rng.integers(1, 8))), replace=False)
            i = np.concatenate([np.arange(s0, min(n, s0 + int(rng.integers(1, 3000)))) for s0 in starts])
        i = np.unique(i).astype(np.uint32)
        idx.append(i)
        v = rng.normal(0, 1, len(i)).astype(np.float32)
        v[v == 0] = 1.0
        val.append(v)
    wl = _custom(n, idx, val, d=d, w=w, W=W, seed=int(rng.integers(0, 2**31)))
    binding.set_insert_strategy([binding.S2R_INSERT_AUTO, binding.S2R_INSERT_ATOMIC, binding.S2R_INSERT_SLICE][case % 3])
    binding.set_decode_strategy([binding.S2R_DECODE_AUTO, binding.S2R_DECODE_GATHER, binding.S2R_DECODE_SLICE,
                                 binding.S2R_DECODE_ROWS][case % 4])
    try:
        _run_blocks_and_check(wl, B, batched=bool(case % 2))
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


@pytest.mark.parametrize("n,B", [(1, 1), (63, 64), (64, 64), (65, 64), (1000, 7), (70000, 650), (200001, 4096), (5000, 9000)])
def test_block_codec_dense_gradient_ragged(n, B, strategy, decode_strategy):
    """Every element set, lengths that are not multiples of the block, one block larger than n."""
    rng = np.random.default_rng(n + B)
    wl = _custom(n, [np.arange(n)] * 2, [rng.normal(0, 1, n).astype(np.float32) + 3.0 for _ in range(2)],
                 d=3, w=1 << 9, W=2)
    _run_blocks_and_check(wl, B)


def test_block_codec_zero_and_special_values(strategy):
    """All-zero gradients give empty bitmaps; -0.0 does not set a block, denormals do."""
    n, B = 5000, 50
    wl = _custom(n, [np.empty(0, dtype=np.uint32)] * 2, [np.empty(0, dtype=np.float32)] * 2, W=2)
    b, _ = _run_blocks_and_check(wl, B)
    assert int(b.out_count.cpu()[0]) == 0
    g = np.zeros(n, dtype=np.float32)
    g[120] = -0.0
    g[777] = np.float32(1e-42)          # denormal
    g[2049] = 1.5
    b = pipeline.block_buffers_for(_custom(n, [np.array([777, 2049])], [g[[777, 2049]]]), B)
    b.grads[0][120] = -0.0
    b.encode(0)
    torch.cuda.synchronize()
    assert b.blk_idx[0][: int(b.nblk.cpu()[0])].cpu().numpy().tolist() == [777 // B, 2049 // B]


def test_block_codec_capacity(strategy, decode_strategy):
    """More set blocks than the lists hold: true counts, the first blk_cap entries,
    nothing beyond them, and a complete sketch."""
    rng = np.random.default_rng(9)
    n, B, cap = 64000, 32, 100
    blocks = np.sort(rng.choice(n // B, 300, replace=False))
    idx = (blocks[:, None] * B + np.arange(B)[None, :]).reshape(-1).astype(np.uint32)
    val = (rng.normal(0, 1, len(idx)) + 2.0).astype(np.float32)
    wl = _custom(n, [idx], [val], d=3, w=1 << 11)
    ref = _oracle_blocks(wl, B)
    b = pipeline.block_buffers_for(wl, B)
    b.blk_idx[0] = torch.full((cap + 8,), -1, dtype=torch.int32, device="cuda")[:cap]
    b.out_blk = torch.full((cap + 8,), -1, dtype=torch.int32, device="cuda")[:cap]
    b.out_val = torch.full((cap * B + 8,), -7.0, dtype=torch.float32, device="cuda")[: cap * B]
    b.step()
    torch.cuda.synchronize()
    assert int(b.nblk.cpu()[0]) == 300 and int(b.out_count.cpu()[0]) == 300
    assert np.array_equal(b.blk_idx[0].cpu().numpy().view(np.uint32), blocks[:cap])
    assert (b.blk_idx[0]._base[cap:].cpu().numpy() == -1).all()
    assert np.array_equal(b.out_blk.cpu().numpy().view(np.uint32), blocks[:cap])
    assert (b.out_blk._base[cap:].cpu().numpy() == -1).all() and (b.out_val._base[cap * B:].cpu().numpy() == -7.0).all()
    _check_sketch(b.sketch[0].cpu().numpy(), ref["S"], ref["M"], "sketch is complete despite the short list")
    want = ref["val"][:cap].reshape(-1)
    elems = (blocks[:cap, None] * B + np.arange(B)[None, :]).reshape(-1)
    tol = REL * orc.decode_tolerance_mass(ref["M"], elems.astype(np.uint32), 0) + DENORM_SLACK
    assert np.all(np.abs(b.out_val.cpu().numpy().astype(np.float64) - want) <= tol)


# ---------------------------------------------------------------- block Top-K with error feedback
def _topk_check(gs, es, B, K, in_place=False):
    """Runs s2r_topk_blocks_batch and checks it against oracle.topk_blocks.  The kept set must
    be the oracle's unless two scores around the threshold are within one float32 rounding of
    each other (the float64 sums may be formed in another order); sparse and residual must be
    bit-exact for the set the library kept."""
    W, n = len(gs), len(gs[0])
    nb = (n + B - 1) // B
    dev = "cuda"
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = None if es is None else [torch.from_numpy(e).to(dev) for e in es]
    sparse = grads if in_place else [torch.full((n,), 7.0, dtype=torch.float32, device=dev) for _ in range(W)]
    kept = [torch.full(((nb + 63) // 64,), -1, dtype=torch.int64, device=dev) for _ in range(W)]
    ws = torch.empty(binding.topk_workspace_bytes(n, B) * W, dtype=torch.uint8, device=dev)
    binding.topk_blocks_batch(grads, resid, n, B, K, sparse, kept, ws)
    torch.cuda.synchronize()
    for k in range(W):
        ref = orc.topk_blocks(gs[k], None if es is None else es[k], B, K)
        mask = orc.unpack_bitmap(pipeline.u64(kept[k]), nb)
        assert int(mask.sum()) == min(K, nb), f"worker {k}: kept {int(mask.sum())} blocks"
        got = np.flatnonzero(mask)
        if not np.array_equal(got, ref["blocks"]):
            sc = ref["score"].astype(np.float64)
            lo, hi = sc[mask].min(), sc[~mask].max()
            assert hi <= lo * (1 + 2.0 ** -22), f"worker {k}: a kept block scores {lo}, a dropped one {hi}"
        elem = np.repeat(mask, B)[:n]
        acc = ref["acc"]
        want_s = np.where(elem, acc, np.float32(0.0)).astype(np.float32)
        want_e = np.where(elem, np.float32(0.0), acc).astype(np.float32)
        assert np.array_equal(sparse[k].cpu().numpy().view(np.uint32), want_s.view(np.uint32)), f"worker {k} sparse"
        if es is not None:
            assert np.array_equal(resid[k].cpu().numpy().view(np.uint32), want_e.view(np.uint32)), f"worker {k} residual"


@pytest.mark.parametrize("n,B,K", [(1, 1, 1), (1000, 1, 37), (1000, 7, 20), (4096, 32, 5), (70001, 256, 50),
                                   (70001, 650, 3), (200000, 31, 1000), (200000, 33, 1000), (50000, 60000, 1),
                                   (300000, 4096, 10), (65536, 64, 0), (65536, 64, 1024), (65536, 64, 5000)])
def test_topk_blocks_match_oracle(n, B, K):
    rng = np.random.default_rng(n + 31 * B + K)
    gs = [(rng.normal(0, 1, n) * rng.gamma(0.5, 1.0, n)).astype(np.float32) for _ in range(3)]
    es = [(rng.normal(0, 0.2, n) * (rng.random(n) < 0.3)).astype(np.float32) for _ in range(3)]
    _topk_check(gs, es, B, K)


def test_topk_without_residual_in_place_and_ties():
    rng = np.random.default_rng(5)
    n, B = 40000, 100
    g = rng.normal(0, 1, n).astype(np.float32)
    _topk_check([g.copy(), g.copy()], None, B, 40, in_place=True)
    tied = np.tile(rng.normal(0, 1, B).astype(np.float32), n // B)      # every block identical: the lowest indices win
    _topk_check([tied], [np.zeros(n, dtype=np.float32)], B, 17)
    sparse = np.zeros(n, dtype=np.float32)
    sparse[:5 * B] = 1.0                                                # five non-zero blocks, K larger: zero blocks by index
    _topk_check([sparse], [np.zeros(n, dtype=np.float32)], B, 9)


def test_topk_error_feedback_over_steps_feeds_the_codec():
    """Three steps of gradient -> Top-K (+ residual) -> block codec on two workers: at
    every step the decoded blocks are the union of the kept blocks, and what the workers
    have sent plus their residuals is what they were given."""
    rng = np.random.default_rng(8)
    n, B, K, W, d, w = 32768, 64, 20, 2, 3, 1 << 14
    nb = n // B
    dev = "cuda"
    resid = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(W)]
    sent = [np.zeros(n) for _ in range(W)]
    given = [np.zeros(n) for _ in range(W)]
    ws = torch.empty(binding.topk_workspace_bytes(n, B) * W, dtype=torch.uint8, device=dev)
    wl = _custom(n, [np.empty(0, dtype=np.uint32)] * W, [np.empty(0, dtype=np.float32)] * W, d=d, w=w, W=W)
    bb = pipeline.BlockBuffers(W, n, B, d, w, 0, K, W * K)
    for step in range(3):
        gs = [rng.normal(0, 1, n).astype(np.float32) for _ in range(W)]
        grads = [torch.from_numpy(g).to(dev) for g in gs]
        kept = [torch.zeros((nb + 63) // 64, dtype=torch.int64, device=dev) for _ in range(W)]
        binding.topk_blocks_batch(grads, resid, n, B, K, grads, kept, ws)          # sparse gradient in place
        bb.grads = grads
        bb.step()
        torch.cuda.synchronize()
        union = np.zeros(nb, dtype=bool)
        for k in range(W):
            union |= orc.unpack_bitmap(pipeline.u64(kept[k]), nb)
            sent[k] += grads[k].cpu().numpy()
            given[k] += gs[k]
            assert np.allclose(sent[k] + resid[k].cpu().numpy(), given[k], rtol=0, atol=1e-4)
        cnt = int(bb.out_count.cpu()[0])
        assert np.array_equal(bb.out_blk[:cnt].cpu().numpy(), np.flatnonzero(union))


def _check_fused_worker(k, g, e, B, K, d, w, seed, bitmap, blk, cap, nblk, sketch, resid):
    """One worker's outputs of s2r_topk_encode_blocks_batch against the oracle (see _fused_topk_check)."""
    n = len(g)
    nb = (n + B - 1) // B
    ref = orc.topk_encode_blocks(g, e, B, K, d, w, seed)
    mask = orc.unpack_bitmap(pipeline.u64(bitmap), nb)
    assert int(mask.sum()) == min(K, nb) == nblk, f"worker {k}: kept {int(mask.sum())} blocks"
    got = np.flatnonzero(mask)
    if np.array_equal(got, ref["blocks"]):
        S, M, want_e = ref["S"], ref["M"], ref["residual"]
        assert np.array_equal(pipeline.u64(bitmap), ref["bitmap"])
    else:
        acc = g if e is None else (g + e).astype(np.float32)
        sc = orc.block_scores(acc, B).astype(np.float64)
        lo, hi = sc[mask].min(), sc[~mask].max()
        assert hi <= lo * (1 + 2.0 ** -22), f"worker {k}: a kept block scores {lo}, a dropped one {hi}"
        elem = np.repeat(mask, B)[:n]
        S, M = orc.insert(*orc.sparse_of(np.where(elem, acc, np.float32(0.0)).astype(np.float32)), d, w, seed)
        want_e = np.where(elem, np.float32(0.0), acc).astype(np.float32)
    if blk is not None:
        m = min(cap, len(got))
        assert np.array_equal(blk[:m].cpu().numpy().view(np.uint32), got[:m].astype(np.uint32)), f"worker {k} list"
        assert (blk[m:].cpu().numpy() == -1).all(), "entries beyond the count are not written"
    _check_sketch(sketch.cpu().numpy(), S, M, f"worker {k} sketch")
    if e is not None:
        assert np.array_equal(resid.cpu().numpy().view(np.uint32), want_e.view(np.uint32)), f"worker {k} residual"


def _fused_topk_check(gs, es, B, K, d, w, seed=0, cap=None, lists=True):
    """Runs s2r_topk_encode_blocks_batch and checks bitmap, block list, sketch and residual
    against the oracle's pieces for the set of blocks the library kept (which must be the
    oracle's set up to scores within one float32 rounding, as for s2r_topk_blocks)."""
    W, n = len(gs), len(gs[0])
    nb = (n + B - 1) // B
    cap = min(K, nb) if cap is None else cap
    dev = "cuda"
    print(f"[case] fused top-k W={W} n={n} B={B} K={K} d={d} w={w} cap={cap} lists={lists} residual={es is not None}", flush=True)
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = None if es is None else [torch.from_numpy(e).to(dev) for e in es]
    sketch = [torch.full((d * w,), 3.0, dtype=torch.float32, device=dev) for _ in range(W)]
    bitmap = [torch.full(((nb + 63) // 64,), -1, dtype=torch.int64, device=dev) for _ in range(W)]
    blk = [torch.full((max(cap, 1),), -1, dtype=torch.int32, device=dev) for _ in range(W)] if lists else None
    nblk = torch.zeros(W, dtype=torch.int64, device=dev)
    ws = torch.empty(binding.topk_encode_blocks_workspace_bytes(n, B, d, w, max(cap, 1) if lists else 0) * W, dtype=torch.uint8,
                     device=dev)
    binding.topk_encode_blocks_batch(grads, resid, n, B, K, d, w, seed, sketch, bitmap, blk, nblk, ws)
    torch.cuda.synchronize()
    for k in range(W):
        _check_fused_worker(k, gs[k], None if es is None else es[k], B, K, d, w, seed, bitmap[k], blk[k] if lists else None,
                            cap, int(nblk[k].cpu()), sketch[k], None if es is None else resid[k])
        assert np.array_equal(grads[k].cpu().numpy().view(np.uint32), gs[k].view(np.uint32)), "the gradient is an input"


@pytest.mark.parametrize("n,B,K,d,w", [(1, 1, 1, 1, 1), (1000, 1, 37, 3, 256), (1000, 7, 20, 3, 64), (4096, 32, 5, 5, 1 << 10),
                                       (70001, 256, 50, 3, 1 << 14), (70001, 650, 3, 4, 1 << 12),
                                       (200000, 31, 1000, 3, 1 << 15), (200000, 33, 1000, 5, 1 << 16),
                                       (50000, 60000, 1, 3, 1 << 13), (300000, 4096, 10, 3, 1 << 17),
                                       (65536, 64, 0, 3, 1 << 12), (65536, 64, 1024, 2, 1 << 18), (65536, 64, 5000, 3, 1 << 14)])
def test_fused_topk_encode_blocks_match_oracle(n, B, K, d, w, strategy):
    rng = np.random.default_rng(n + 31 * B + K)
    gs = [(rng.normal(0, 1, n) * rng.gamma(0.5, 1.0, n)).astype(np.float32) for _ in range(3)]
    es = [(rng.normal(0, 0.2, n) * (rng.random(n) < 0.3)).astype(np.float32) for _ in range(3)]
    _fused_topk_check(gs, es, B, K, d, w, seed=n % 7)


def test_fused_topk_short_lists_no_lists_no_residual_and_zero_blocks(strategy):
    rng = np.random.default_rng(15)
    n, B = 90000 + 13, 128
    gs = [rng.normal(0, 1, n).astype(np.float32) for _ in range(2)]
    es = [rng.normal(0, 0.3, n).astype(np.float32) for _ in range(2)]
    _fused_topk_check(gs, es, B, 300, 3, 1 << 14, cap=100)                 # 200 kept blocks beyond the lists
    _fused_topk_check(gs, es, B, 300, 3, 1 << 14, lists=False)             # no lists: every block by atomics
    _fused_topk_check(gs, None, B, 300, 5, 1 << 13)                        # plain Top-K: nothing but the outputs written
    sparse = np.zeros(n, dtype=np.float32)
    sparse[B * 40: B * 43] = rng.normal(0, 1, 3 * B).astype(np.float32)
    sparse[B * 41 + 5] = 0.0                                               # a zero inside a kept block is not inserted
    _fused_topk_check([sparse], [np.zeros(n, dtype=np.float32)], B, 9, 3, 1 << 12)   # six all-zero blocks kept and marked


def test_fused_topk_full_size_in_the_benchmarked_configuration():
    """The shape bench.py --workload cfg3 --block 256 --topk-frac 0.01 --fused-topk times
    (W = 8 dense gradients of 25.6e6 elements, 1000 of 100000 blocks kept), second step
    (residuals in place): every worker against the oracle."""
    W, n, B, K, d, w, seed = 8, 25_600_000, 256, 1000, 3, 1 << 20, 0
    nb = n // B
    dev = "cuda"
    gen = torch.Generator(device=dev).manual_seed(3998)
    grads = [torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 0.01, generator=gen) for _ in range(W)]
    resid = [torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 0.004, generator=gen) for _ in range(W)]
    check = tuple(range(W))
    gs = {k: grads[k].cpu().numpy() for k in check}
    es = {k: resid[k].cpu().numpy().copy() for k in check}
    bb = pipeline.BlockBuffers(W, n, B, d, w, seed, K, W * K)
    for t in bb.blk_idx:
        t.fill_(-1)
    print(f"[case] fused top-k full size W={W} n={n} B={B} K={K}", flush=True)
    bb.topk_encode_all(grads, resid, K)
    torch.cuda.synchronize()
    assert (bb.nblk.cpu().numpy() == K).all()
    for k in check:
        _check_fused_worker(k, gs[k], es[k], B, K, d, w, seed, bb.bitmap[k], bb.blk_idx[k], K, int(bb.nblk[k].cpu()),
                            bb.sketch[k], resid[k])


def test_fused_topk_equals_the_two_calls():
    """Same inputs through s2r_topk_blocks_batch + s2r_encode_blocks_batch and through the
    fused call: bitmaps, lists and residuals identical, sketches equal up to summation order."""
    rng = np.random.default_rng(23)
    W, n, B, K, d, w = 4, 1 << 20, 256, 200, 3, 1 << 16
    nb = n // B
    dev = "cuda"
    gs = [torch.from_numpy(rng.normal(0, 1, n).astype(np.float32)).to(dev) for _ in range(W)]
    e1 = [torch.from_numpy(rng.normal(0, 0.5, n).astype(np.float32)).to(dev) for _ in range(W)]
    e2 = [e.clone() for e in e1]
    mk = lambda: dict(sketch=[torch.empty(d * w, dtype=torch.float32, device=dev) for _ in range(W)],
                      bitmap=[torch.zeros(nb // 64, dtype=torch.int64, device=dev) for _ in range(W)],
                      blk=[torch.full((K,), -1, dtype=torch.int32, device=dev) for _ in range(W)],
                      nblk=torch.zeros(W, dtype=torch.int64, device=dev))
    a, f = mk(), mk()
    sparse = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(W)]
    ws1 = torch.empty(binding.topk_workspace_bytes(n, B) * W, dtype=torch.uint8, device=dev)
    ws2 = torch.empty(binding.encode_blocks_workspace_bytes(n, B, d, w, K) * W, dtype=torch.uint8, device=dev)
    binding.topk_blocks_batch(gs, e1, n, B, K, sparse, None, ws1)
    binding.encode_blocks_batch(sparse, n, B, d, w, 0, a["sketch"], a["bitmap"], a["blk"], a["nblk"], ws2)
    ws3 = torch.empty(binding.topk_encode_blocks_workspace_bytes(n, B, d, w, K) * W, dtype=torch.uint8, device=dev)
    binding.topk_encode_blocks_batch(gs, e2, n, B, K, d, w, 0, f["sketch"], f["bitmap"], f["blk"], f["nblk"], ws3)
    torch.cuda.synchronize()
    assert torch.equal(a["nblk"], f["nblk"])
    for k in range(W):
        assert torch.equal(a["bitmap"][k], f["bitmap"][k]) and torch.equal(a["blk"][k], f["blk"][k])
        assert torch.equal(e1[k].view(torch.int32), e2[k].view(torch.int32)), "residuals"
        sa, sf = a["sketch"][k].double(), f["sketch"][k].double()
        assert float((sa - sf).abs().max()) <= 2e-5 * float(sa.abs().max())


def _block_update_check(gs, B, d, w, seed, scale):
    W, n = len(gs), len(gs[0])
    nb = (n + B - 1) // B
    dev = "cuda"
    print(f"[case] block update W={W} n={n} B={B} d={d} w={w}", flush=True)
    res = orc.reduce_workers_blocks(gs, B, d, w, seed)
    S = torch.from_numpy(res["S"].astype(np.float32).reshape(-1)).to(dev)          # the oracle's merged sketch, rounded
    C = torch.from_numpy(res["bitmap"].view(np.int64)).to(dev)
    rng = np.random.default_rng(n + B)
    params0 = rng.normal(0, 1, n).astype(np.float32)
    params = torch.from_numpy(params0.copy()).to(dev)
    nblk = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = torch.empty(binding.decode_blocks_update_workspace_bytes(n, B, d, w), dtype=torch.uint8, device=dev)
    binding.decode_blocks_update(S, C, n, B, d, w, seed, params, scale, nblk, ws)
    torch.cuda.synchronize()
    blocks = orc.bitmap_indices(res["bitmap"], nb)
    assert int(nblk.cpu()[0]) == len(blocks)
    S32 = res["S"].astype(np.float32).astype(np.float64)
    want = orc.decode_blocks_update(S32, res["bitmap"], n, B, seed, params0, scale).astype(np.float64)
    elems = orc.block_elements(blocks, B, n)
    got = params.cpu().numpy()
    untouched = np.ones(n, dtype=bool)
    untouched[elems] = False
    assert np.array_equal(got[untouched], params0[untouched]), "entries outside the set blocks changed"
    tol = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
    tol[elems] += abs(scale) * (REL * orc.decode_tolerance_mass(res["M"], elems.astype(np.uint32), seed) + DENORM_SLACK)
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= tol), f"worst {err.max():.3e}"


@pytest.mark.parametrize("cfg,B", [(2, 650), (3, 256), (4, 768), (1, 1), (5, 31)])
def test_decode_blocks_update_matches_oracle(cfg, B):
    wl = workloads.make_small(cfg)
    _block_update_check([wl.dense(k) for k in range(wl.W)], B, wl.d, wl.w, wl.seed, -0.05 / wl.W)


def test_decode_blocks_update_reaches_every_block_of_a_dense_gradient():
    """Every block set, more list positions than one pass of the kernel's workgroups
    covers (8192 workgroups x 1024 positions), a ragged last block."""
    rng = np.random.default_rng(77)
    n = 9_000_000 + 77
    g = rng.normal(0, 1, n).astype(np.float32)
    _block_update_check([g], 256, 2, 1 << 16, 3, 0.125)


# ---------------------------------------------------------------- sizes at the limits, random shapes
def test_maximum_length_gradient():
    """n = 2^32 (the limit: indices are uint32), non-zeros at both ends, across the 2^31
    boundary and scattered: counts, index lists and decoded values against the oracle's
    building blocks (the oracle's dense bitmap unpacking is skipped: 2^32 flags)."""
    n, d, w, seed = 1 << 32, 3, 1 << 16, 7
    rng = np.random.default_rng(42)
    special = np.array([0, 1, 63, 64, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, n - 65, n - 64, n - 2, n - 1], dtype=np.int64)
    idx = np.unique(np.concatenate([special, rng.integers(0, n, 20000), (3 << 30) + np.arange(5000)])).astype(np.uint32)
    val = (rng.normal(0, 1, len(idx)) + 3.0).astype(np.float32)
    print(f"[case] maximum length n={n} nnz={len(idx)}", flush=True)
    g = torch.zeros(n, dtype=torch.float32, device="cuda")
    g[torch.from_numpy(idx.astype(np.int64)).cuda()] = torch.from_numpy(val).cuda()
    b = pipeline.Buffers(1, n, d, w, seed, len(idx) + 7, len(idx) + 7)
    b.grads = [g]
    for strategy in ("atomic", "slice"):
        for route in ("gather", "slice"):
            binding.set_insert_strategy(STRATEGIES[strategy])
            binding.set_decode_strategy(DECODES[route])
            try:
                b.nz_idx[0].fill_(-1)
                b.out_idx.fill_(-1)
                b.step()
                torch.cuda.synchronize()
            finally:
                binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
                binding.set_decode_strategy(binding.S2R_DECODE_AUTO)
            assert int(b.nnz.cpu()[0]) == len(idx) and int(b.out_count.cpu()[0]) == len(idx)
            assert np.array_equal(b.nz_idx[0][: len(idx)].cpu().numpy().view(np.uint32), idx)
            assert np.array_equal(b.nz_val[0][: len(idx)].cpu().numpy(), val)
            assert np.array_equal(b.out_idx[: len(idx)].cpu().numpy().view(np.uint32), idx)
            words = pipeline.u64(b.bitmap[0])
            assert int(np.unpackbits(words.view(np.uint8)).sum()) == len(idx)
            bit = (words[(idx >> np.uint32(6)).astype(np.int64)] >> (idx & np.uint32(63)).astype(np.uint64)) & np.uint64(1)
            assert bit.all(), "a listed index has no bit"
            S, M = orc.insert(idx, val, d, w, seed)
            _check_sketch(b.sketch[0].cpu().numpy(), S, M, f"sketch ({strategy})")
            want = orc.median_rows(orc.estimates(S, idx, seed))
            tol = REL * orc.decode_tolerance_mass(M, idx, seed) + DENORM_SLACK
            got = b.out_val[: len(idx)].cpu().numpy().astype(np.float64)
            assert np.all(np.abs(got - want) <= tol), f"decoded values ({strategy}, {route})"


@pytest.mark.parametrize("case", range(24))
def test_random_shapes(case):
    """Seeded random problems: length, rows, width, workers, density, clustering, both
    insertion strategies and both decode routes, element and block codec."""
    rng = np.random.default_rng(9000 + case)
    n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 70000), rng.integers(70000, 400000)]))
    d = int(rng.integers(1, 9))
    w = 1 << int(rng.integers(0, 18))
    W = int(rng.integers(1, 6))
    density = float(rng.choice([0.0005, 0.01, 0.2, 1.0]))
    run = int(rng.choice([1, 1, 17, 256]))
    idx, val = [], []
    for k in range(W):
        starts = np.flatnonzero(rng.random((n + run - 1) // run) < density) * run
        i = (starts[:, None] + np.arange(run)[None, :]).reshape(-1)
        i = np.unique(i[i < n]).astype(np.uint32)
        idx.append(i)
        val.append((rng.normal(0, 1, len(i)) + np.where(rng.random(len(i)) < 0.5, 2.0, -2.0)).astype(np.float32))
    wl = _custom(n, idx, val, d=d, w=w, W=W, seed=int(rng.integers(0, 1 << 40)))
    binding.set_insert_strategy(STRATEGIES[["atomic", "slice"][case % 2]])
    binding.set_decode_strategy(DECODES[["gather", "slice"][(case // 2) % 2]])
    try:
        if case % 3 == 2:
            _run_blocks_and_check(wl, int(rng.choice([1, 3, 64, 100, 1000])), batched=bool(case % 4 < 2))
        else:
            _run_and_check(wl, dense_out=(case % 3 == 0), batched=bool(case % 4 < 2))
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
        binding.set_decode_strategy(binding.S2R_DECODE_AUTO)


@pytest.mark.parametrize("case", range(16))
def test_random_shapes_sparsify_compress_update(case):
    """Seeded random problems through the one-call sparsifier + compress step and the
    block-granular update: length, block size (multiples of 4 and not, below and above a
    wave), kept fraction, rows, width, workers, with and without residuals and lists, gradients
    with many exact zeros."""
    rng = np.random.default_rng(12000 + case)
    n = int(rng.choice([rng.integers(1, 500), rng.integers(500, 60000), rng.integers(60000, 300000)]))
    B = int(rng.choice([1, 3, 4, 31, 32, 36, 64, 100, 256, 1000, 4096]))
    nb = (n + B - 1) // B
    K = int(rng.choice([0, 1, max(1, nb // 50), max(1, nb // 4), nb, nb + 5]))
    d = int(rng.integers(1, 9))
    w = 1 << int(rng.integers(0, 17))
    W = int(rng.integers(1, 5))
    zeros = float(rng.choice([0.0, 0.5, 0.98]))
    gs = [(rng.normal(0, 1, n) * (rng.random(n) >= zeros)).astype(np.float32) for _ in range(W)]
    es = None if case % 4 == 3 else [(rng.normal(0, 0.3, n) * (rng.random(n) >= zeros)).astype(np.float32) for _ in range(W)]
    seed = int(rng.integers(0, 1 << 40))
    binding.set_insert_strategy(STRATEGIES[["atomic", "slice"][case % 2]])
    try:
        kept = min(K, nb)
        _fused_topk_check(gs, es, B, K, d, w, seed=seed, cap=[None, max(kept // 2, 1)][(case // 2) % 2], lists=(case % 5 != 4))
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)
    _block_update_check(gs, B, d, w, seed, -0.01 * (1 + case % 3))


def test_very_sparse_gradient_with_dense_pockets(strategy):
    """Forty tiles with a handful of non-zeros per 2048-element piece, one piece of exactly
    8, one of 9 and one full piece, a ragged last tile, and a list capacity that ends inside
    a sparse tile."""
    rng = np.random.default_rng(123)
    n = 32768 * 40 + 1234
    parts = [np.sort(rng.choice(n, 2500, replace=False))]
    parts.append(32768 * 3 + 2048 * 5 + np.arange(8) * 7)              # a piece with exactly 8
    parts.append(32768 * 7 + 2048 * 2 + np.arange(9) * 5)              # a piece with 9: its tile expands the bitmap
    parts.append(32768 * 11 + 2048 * 9 + np.arange(2048))              # a full piece
    idx = np.unique(np.concatenate(parts)).astype(np.uint32)
    val = (rng.normal(0, 1, len(idx)) + 2.0).astype(np.float32)
    assert len(idx) + 5 < n // 256
    wl = _custom(n, [idx, idx[::3]], [val, val[::3]], d=3, w=1 << 12, W=2)
    _run_and_check(wl)
    b = pipeline.buffers_for(wl)
    cap = 1000
    b.nz_idx[0] = torch.full((cap + 16,), -1, dtype=torch.int32, device="cuda")[:cap]
    b.nz_val[0] = torch.zeros(cap, dtype=torch.float32, device="cuda")
    b.encode(0)
    torch.cuda.synchronize()
    assert int(b.nnz.cpu()[0]) == len(idx)
    assert np.array_equal(b.nz_idx[0].cpu().numpy().view(np.uint32), idx[:cap])
    assert np.array_equal(b.nz_val[0].cpu().numpy(), val[:cap])
    assert (b.nz_idx[0]._base[cap:].cpu().numpy() == -1).all()


def test_step_replays_from_a_captured_graph():
    """The library only enqueues kernels (no allocation, no memset, no host wait), so a
    caller can capture encode + merge + decode into a HIP graph.  The graph is replayed
    three times over gradients that change between the replays, with eager work and
    synchronisations in between; every replay must equal the eager result on the same
    gradients (bit-exact for bitmaps and lists; the slice routes make the values
    reproducible too)."""
    wl = workloads.make_small(3)
    b = pipeline.buffers_for(wl)
    binding.set_insert_strategy(binding.S2R_INSERT_SLICE)
    try:
        b.step()                                           # warm-up: raises the LDS limits outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            b.step(torch.cuda.current_stream())
        rng = np.random.default_rng(3)
        for replay in range(3):
            for k in range(wl.W):                          # new gradients: scale, and move a few non-zeros
                b.grads[k].mul_(1.5 + replay)
                pos = torch.from_numpy(rng.integers(0, wl.n, 50)).cuda()
                b.grads[k][pos] = float(replay + 1)
            torch.cuda.synchronize()
            b.step()                                       # eager reference on the same gradients
            torch.cuda.synchronize()
            want = (pipeline.u64(b.bitmap_or).copy(), int(b.out_count.cpu()[0]), b.out_idx.cpu().numpy().copy(),
                    b.out_val.cpu().numpy().copy(), b.sketch_sum.cpu().numpy().copy())
            b.out_val.zero_(); b.out_idx.zero_(); b.sketch_sum.zero_(); b.bitmap_or.zero_(); b.out_count.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            cnt = int(b.out_count.cpu()[0])
            assert cnt == want[1] and np.array_equal(pipeline.u64(b.bitmap_or), want[0]), f"replay {replay}"
            assert np.array_equal(b.out_idx.cpu().numpy()[:cnt], want[2][:cnt])
            assert np.allclose(b.sketch_sum.cpu().numpy(), want[4], rtol=1e-5, atol=1e-30)
            assert np.allclose(b.out_val.cpu().numpy()[:cnt], want[3][:cnt], rtol=1e-4, atol=1e-6)
    finally:
        binding.set_insert_strategy(binding.S2R_INSERT_AUTO)


@pytest.mark.parametrize("lists", [True, False], ids=["with_lists", "update_only"])
def test_decode_update_matches_oracle(lists):
    """params += scale * decoded sum, against the oracle, with lists shorter than the
    union (the update must still reach every union index) and without lists."""
    wl = workloads.make_small(4)
    enc, S, C, M, dec = _oracle_for(wl)
    b = pipeline.buffers_for(wl)
    b.encode_all()
    b.merge()
    rng = np.random.default_rng(17)
    params0 = rng.normal(0, 1, wl.n).astype(np.float32)
    params = torch.from_numpy(params0.copy()).cuda()
    scale = -0.05 / wl.W
    cap = len(dec["idx"]) // 3
    idx_out = torch.full((cap,), -1, dtype=torch.int32, device="cuda") if lists else None
    val_out = torch.zeros(cap, dtype=torch.float32, device="cuda") if lists else None
    binding.decode_update(b.sketch_sum, b.bitmap_or, wl.n, wl.d, wl.w, wl.seed, params, scale, idx_out, val_out,
                          b.out_count, b.workspace)
    torch.cuda.synchronize()
    assert int(b.out_count.cpu()[0]) == len(dec["idx"])
    want = orc.decode_update(S, C, wl.n, wl.seed, params0, scale).astype(np.float64)
    got = params.cpu().numpy().astype(np.float64)
    tol = np.zeros(wl.n)
    tol[dec["idx"]] = abs(scale) * (REL * orc.decode_tolerance_mass(M, dec["idx"], wl.seed) + DENORM_SLACK)
    tol += np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
    untouched = np.ones(wl.n, dtype=bool)
    untouched[dec["idx"]] = False
    assert np.array_equal(params.cpu().numpy()[untouched], params0[untouched]), "entries outside the union changed"
    assert np.all(np.abs(got - want) <= tol), f"worst {np.abs(got - want).max():.3e}"
    if lists:
        assert np.array_equal(idx_out.cpu().numpy().view(np.uint32), dec["idx"][:cap])
