"""CPU-only checks of the C-ABI library: it loads, exports every symbol that
include/s2r.h and include/s2r_bench.h declare, and its host-only entry points and argument checks
behave as documented.  No kernel is launched here."""

import ctypes
import os
import re

import numpy as np
import pytest

from oracle import s2r_oracle as orc
from paper_2110_02140_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in ("s2r.h", "s2r_bench.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(s2r_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = b.load()
    names = _declared_symbols()
    assert {"s2r_encode", "s2r_merge", "s2r_decode", "s2r_workspace_bytes"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(b.SIGNATURES), "binding and header disagree on the symbol list"


def test_version_and_status_strings():
    assert b.version() >= 100
    seen = set()
    for st in range(0, -7, -1):
        s = b.status_string(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 7
    assert b.status_string(-99) == "unknown status"


@pytest.mark.parametrize("seed", [0, 1, 12345, 2**64 - 1])
def test_host_hash_params_equal_oracle(seed):
    assert b.hash_params(seed, 16) == orc.hash_params(seed, 16)


def test_workspace_bytes_limits():
    assert b.workspace_bytes(0, 3, 16) == 0
    assert b.workspace_bytes(2**32 + 1, 3, 16) == 0
    assert b.workspace_bytes(100, 0, 16) == 0
    assert b.workspace_bytes(100, 17, 16) == 0
    assert b.workspace_bytes(100, 3, 12) == 0          # not a power of two
    assert b.workspace_bytes(100, 16, 1 << 29) == 0    # d*w > 2^32
    small = b.workspace_bytes(1, 1, 1)
    big = b.workspace_bytes(2**32, 5, 1 << 22)
    assert small >= 256 + 8 and small % 256 == 0
    assert big > small and big % 256 == 0


def _call_encode(**kw):
    lib = b.load()
    a = dict(grad=0x1000, n=1000, d=3, w=64, seed=0, sketch=0x2000, bitmap=0x3000, idx=0x4000, val=0x5000,
             cap=10, nnz=0x6000, ws=0x10000, wsb=1 << 20, stream=None)
    a.update(kw)
    return lib.s2r_encode(a["grad"], a["n"], a["d"], a["w"], a["seed"], a["sketch"], a["bitmap"], a["idx"],
                          a["val"], a["cap"], a["nnz"], a["ws"], a["wsb"], a["stream"])


def test_encode_rejects_bad_arguments_before_touching_the_device():
    # (pointers are never dereferenced: every case below fails validation first)
    assert _call_encode(grad=None) == b.S2R_ERR_NULL
    assert _call_encode(sketch=None) == b.S2R_ERR_NULL
    assert _call_encode(bitmap=None) == b.S2R_ERR_NULL
    assert _call_encode(nnz=None) == b.S2R_ERR_NULL
    assert _call_encode(idx=None) == b.S2R_ERR_NULL            # idx without val
    assert _call_encode(n=0) == b.S2R_ERR_SIZE
    assert _call_encode(n=2**32 + 1) == b.S2R_ERR_SIZE
    assert _call_encode(d=0) == b.S2R_ERR_SIZE
    assert _call_encode(d=17) == b.S2R_ERR_SIZE
    assert _call_encode(w=0) == b.S2R_ERR_SIZE
    assert _call_encode(w=48) == b.S2R_ERR_WIDTH
    assert _call_encode(ws=None) == b.S2R_ERR_WORKSPACE
    assert _call_encode(ws=0x10010) == b.S2R_ERR_WORKSPACE      # not 256-byte aligned
    assert _call_encode(wsb=8) == b.S2R_ERR_WORKSPACE
    assert _call_encode(sketch=0x2004) == b.S2R_ERR_ALIGN
    assert _call_encode(grad=0x1002) == b.S2R_ERR_ALIGN


def test_merge_and_decode_reject_bad_arguments():
    lib = b.load()
    two = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    one_null = (ctypes.c_void_p * 2)(0x1000, None)
    assert lib.s2r_merge(None, two, 2, 100, 3, 64, 0, 0x3000, 0x4000, None) == b.S2R_ERR_NULL
    assert lib.s2r_merge(two, two, 0, 100, 3, 64, 0, 0x3000, 0x4000, None) == b.S2R_ERR_SIZE
    assert lib.s2r_merge(two, two, 65, 100, 3, 64, 0, 0x3000, 0x4000, None) == b.S2R_ERR_SIZE
    assert lib.s2r_merge(one_null, two, 2, 100, 3, 64, 0, 0x3000, 0x4000, None) == b.S2R_ERR_NULL
    assert lib.s2r_merge(two, two, 2, 100, 3, 65, 0, 0x3000, 0x4000, None) == b.S2R_ERR_WIDTH
    assert lib.s2r_merge(two, two, 2, 100, 3, 64, 0, 0x3004, 0x4000, None) == b.S2R_ERR_ALIGN
    dec = lambda **k: lib.s2r_decode(k.get("S", 0x1000), k.get("C", 0x2000), k.get("n", 100), k.get("d", 3),
                                     k.get("w", 64), 0, k.get("idx", 0x3000), k.get("val", 0x4000), 10,
                                     k.get("cnt", 0x5000), None, k.get("ws", 0x10000), k.get("wsb", 1 << 20), None)
    assert dec(S=None) == b.S2R_ERR_NULL
    assert dec(cnt=None) == b.S2R_ERR_NULL
    assert dec(val=None) == b.S2R_ERR_NULL
    assert dec(n=0) == b.S2R_ERR_SIZE
    assert dec(w=3) == b.S2R_ERR_WIDTH
    assert dec(wsb=0) == b.S2R_ERR_WORKSPACE


def test_merge_decode_checks_both_halves_before_it_launches():
    """Every bad argument of either half is an error return (no GPU here: nothing may be enqueued)."""
    lib = b.load()
    two = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    one_null = (ctypes.c_void_p * 2)(0x1000, None)
    md = lambda **k: lib.s2r_merge_decode(k.get("S", two), k.get("C", two), k.get("W", 2), k.get("n", 100), k.get("d", 3),
                                          k.get("w", 64), 0, k.get("So", 0x3000), k.get("Co", 0x4000),
                                          k.get("idx", 0x5000), k.get("val", 0x6000), 10, k.get("cnt", 0x7000), None,
                                          k.get("ws", 0x10000), k.get("wsb", 1 << 20), None)
    assert md(S=None) == b.S2R_ERR_NULL
    assert md(C=one_null) == b.S2R_ERR_NULL
    assert md(W=0) == b.S2R_ERR_SIZE
    assert md(W=65) == b.S2R_ERR_SIZE
    assert md(So=None) == b.S2R_ERR_NULL
    assert md(So=0x3004) == b.S2R_ERR_ALIGN
    assert md(w=65) == b.S2R_ERR_WIDTH
    assert md(n=0) == b.S2R_ERR_SIZE
    assert md(cnt=None) == b.S2R_ERR_NULL               # the decode half
    assert md(val=None) == b.S2R_ERR_NULL
    assert md(wsb=0) == b.S2R_ERR_WORKSPACE
    assert md(ws=0x10010) == b.S2R_ERR_WORKSPACE
    bad = _options(decode_strategy=9)
    assert lib.s2r_merge_decode_ex(two, two, 2, 100, 3, 64, 0, 0x3000, 0x4000, 0x5000, 0x6000, 10, 0x7000, None,
                                   0x10000, 1 << 20, None, ctypes.byref(bad)) == b.S2R_ERR_SIZE
    mdb = lambda **k: lib.s2r_merge_decode_blocks(two, two, 2, k.get("n", 1000), k.get("B", 10), 3, 64, 0, 0x3000,
                                                  0x4000, 0x5000, k.get("val", 0x6000), 10, k.get("cnt", 0x7000),
                                                  0x10000, k.get("wsb", 1 << 20), None)
    assert mdb(B=0) == b.S2R_ERR_SIZE
    assert mdb(cnt=None) == b.S2R_ERR_NULL
    assert mdb(val=None) == b.S2R_ERR_NULL
    assert mdb(wsb=16) == b.S2R_ERR_WORKSPACE


def test_encode_batch_rejects_bad_arguments():
    lib = b.load()
    two = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    sk = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    one_null = (ctypes.c_void_p * 2)(0x1000, None)
    call = lambda **k: lib.s2r_encode_batch(k.get("g", two), k.get("W", 2), k.get("n", 1000), 3, k.get("w", 64), 0,
                                            k.get("S", sk), k.get("C", two), k.get("idx", None), k.get("val", None),
                                            10, k.get("nnz", 0x6000), k.get("ws", 0x100000), k.get("wsb", 1 << 20), None)
    assert call(g=None) == b.S2R_ERR_NULL
    assert call(g=one_null) == b.S2R_ERR_NULL
    assert call(nnz=None) == b.S2R_ERR_NULL
    assert call(idx=two) == b.S2R_ERR_NULL                  # idx without val
    assert call(idx=one_null, val=two) == b.S2R_ERR_NULL    # lists for some workers only
    assert call(W=0) == b.S2R_ERR_SIZE
    assert call(W=65) == b.S2R_ERR_SIZE
    assert call(w=100) == b.S2R_ERR_WIDTH
    assert call(wsb=300) == b.S2R_ERR_WORKSPACE
    assert call(ws=0x100010) == b.S2R_ERR_WORKSPACE
    assert call(S=(ctypes.c_void_p * 2)(0x10000, 0x20004)) == b.S2R_ERR_ALIGN


def _options(**kw):
    o = b.Options()
    o.struct_bytes = ctypes.sizeof(b.Options)
    for k, v in kw.items():
        setattr(o, k, v)
    return o


def _call_encode_ex(opt, **kw):
    lib = b.load()
    a = dict(grad=0x1000, n=1000, d=3, w=64, seed=0, sketch=0x2000, bitmap=0x3000, idx=0x4000, val=0x5000,
             cap=10, nnz=0x6000, ws=None, wsb=1 << 20, stream=None)
    a.update(kw)
    return lib.s2r_encode_ex(a["grad"], a["n"], a["d"], a["w"], a["seed"], a["sketch"], a["bitmap"], a["idx"],
                             a["val"], a["cap"], a["nnz"], a["ws"], a["wsb"], a["stream"],
                             None if opt is None else ctypes.byref(opt))


def test_options_are_checked_before_anything_else():
    # (every call below fails on its options, or, with good options, on the NULL workspace: nothing is enqueued)
    assert ctypes.sizeof(b.Options) == 40 and ctypes.sizeof(b.Report) == 16
    assert _call_encode_ex(None) == b.S2R_ERR_WORKSPACE
    assert _call_encode_ex(_options()) == b.S2R_ERR_WORKSPACE
    for st in (b.S2R_INSERT_SLICE, b.S2R_INSERT_ATOMIC, b.S2R_INSERT_AUTO):
        assert _call_encode_ex(_options(insert_strategy=st)) == b.S2R_ERR_WORKSPACE
    assert _call_encode_ex(_options(insert_strategy=3)) == b.S2R_ERR_SIZE
    assert _call_encode_ex(_options(insert_strategy=-1)) == b.S2R_ERR_SIZE
    assert _call_encode_ex(_options(decode_strategy=5)) == b.S2R_ERR_SIZE
    assert _call_encode_ex(_options(flags=1)) == b.S2R_ERR_SIZE
    assert _call_encode_ex(_options(struct_bytes=48)) == b.S2R_ERR_SIZE
    tr = b.Trace()
    tr.begin[b.S2R_KERNEL_ENCODE_SCAN] = 0x40                                         # begin without end
    assert _call_encode_ex(_options(trace=ctypes.pointer(tr))) == b.S2R_ERR_NULL
    tr.end[b.S2R_KERNEL_ENCODE_SCAN] = 0x50
    assert _call_encode_ex(_options(trace=ctypes.pointer(tr))) == b.S2R_ERR_WORKSPACE
    rep = b.Report(7, 7, 7, 7)
    assert _call_encode_ex(_options(report=ctypes.pointer(rep))) == b.S2R_ERR_WORKSPACE
    assert (rep.insert_strategy, rep.decode_strategy, rep.scan_launch_workers, rep.reserved) == (0, 0, 0, 0)
    lib = b.load()
    bad = _options(decode_strategy=9)
    assert lib.s2r_decode_ex(0x1000, 0x2000, 1000, 3, 64, 0, None, None, 0, 0x3000, None, None, 0, None,
                             ctypes.byref(bad)) == b.S2R_ERR_SIZE
    assert lib.s2r_decode_blocks_ex(0x1000, 0x2000, 1000, 10, 3, 64, 0, None, None, 0, 0x3000, None, 0, None,
                                    ctypes.byref(bad)) == b.S2R_ERR_SIZE
    one = lambda v: (ctypes.c_void_p * 1)(v)
    assert lib.s2r_encode_blocks_batch_ex(one(0x1000), 1, 1000, 10, 3, 64, 0, one(0x2000), one(0x3000), None, 0,
                                          0x4000, None, 0, None, ctypes.byref(bad)) == b.S2R_ERR_SIZE
    assert lib.s2r_topk_encode_blocks_batch_ex(one(0x1000), None, 1, 1000, 10, 5, 3, 64, 0, one(0x2000), one(0x3000),
                                               None, 0, 0x4000, None, 0, None, ctypes.byref(bad)) == b.S2R_ERR_SIZE


def test_binding_side_defaults_are_checked():
    with pytest.raises(b.S2RError):
        b.set_insert_strategy(7)
    with pytest.raises(b.S2RError):
        b.set_decode_strategy(5)
    with pytest.raises(b.S2RError):
        b.set_kernel_events(b.S2R_KERNEL_SLOTS, None, None)
    b.set_insert_strategy(b.S2R_INSERT_AUTO)
    b.set_decode_strategy(b.S2R_DECODE_AUTO)


def test_probe_read_argument_checks():
    lib = b.load()
    assert lib.s2r_probe_read(None, 1024, 0x100, None) == b.S2R_ERR_NULL
    assert lib.s2r_probe_read(0x1000, 1024, None, None) == b.S2R_ERR_NULL
    assert lib.s2r_probe_read(0x1000, 8, 0x100, None) == b.S2R_ERR_SIZE
    assert lib.s2r_probe_read(0x1004, 1024, 0x100, None) == b.S2R_ERR_ALIGN
    assert lib.s2r_probe_read(0x1000, 1024, 0x104, None) == b.S2R_ERR_ALIGN


def test_decode_strategy_and_workspace_argument_checks():
    base = b.workspace_bytes(1 << 20, 3, 1 << 14)
    assert b.decode_workspace_bytes(1 << 20, 3, 1 << 14, 50000) >= base + 8 * 3 * 50000
    assert b.decode_workspace_bytes(1 << 20, 9, 1 << 14, 50000) == base        # more than 8 rows: gather only
    assert b.decode_workspace_bytes(1 << 20, 3, 1 << 14, (1 << 20) + 1) == 0    # cap > n
    assert b.decode_workspace_bytes(0, 3, 1 << 14, 0) == 0


def test_block_codec_argument_checks():
    lib = b.load()
    n, d, w = 1 << 20, 3, 1 << 14
    assert b.blocks_workspace_bytes(n, 0, d, w) == 0
    assert b.blocks_workspace_bytes(n, 256, d, w) > 0
    assert b.blocks_workspace_bytes(n, 256, d, w) <= b.workspace_bytes(n, d, w)
    assert b.encode_blocks_workspace_bytes(n, 256, d, w, 4097) == 0            # more blocks than the gradient has
    assert b.encode_blocks_workspace_bytes(n, 256, d, w, 100) >= b.blocks_workspace_bytes(n, 256, d, w) + 8 * d * 100 * 256
    assert b.decode_blocks_workspace_bytes(n, 256, d, w, 100) >= b.blocks_workspace_bytes(n, 256, d, w) + 8 * d * 100 * 256
    assert lib.s2r_encode_blocks(0x1000, n, 0, d, w, 0, 0x2000, 0x3000, None, 0, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_SIZE
    assert lib.s2r_encode_blocks(None, n, 256, d, w, 0, 0x2000, 0x3000, None, 0, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_NULL
    assert lib.s2r_encode_blocks(0x1000, n, 256, d, w, 0, 0x2000, 0x3000, None, 0, 0x4000, None, 1 << 20, None) == b.S2R_ERR_WORKSPACE
    assert lib.s2r_decode_blocks(0x1000, 0x2000, n, 0, d, w, 0, None, None, 0, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_SIZE
    assert lib.s2r_decode_blocks(0x1000, 0x2000, n, 256, d, w, 0, 0x3000, None, 10, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_NULL
    assert lib.s2r_decode_blocks(0x1000, 0x2000, n, 256, d, w + 1, 0, None, None, 0, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_WIDTH


def test_topk_argument_checks():
    lib = b.load()
    assert b.topk_workspace_bytes(1 << 20, 0) == 0 and b.topk_workspace_bytes(0, 256) == 0
    assert b.topk_workspace_bytes(1 << 20, 256) >= 8 * 4096 + 4 * 2048
    assert lib.s2r_topk_blocks(None, None, 1000, 10, 5, 0x2000, None, 0x4000, 1 << 20, None) == b.S2R_ERR_NULL
    assert lib.s2r_topk_blocks(0x1000, None, 1000, 0, 5, 0x2000, None, 0x4000, 1 << 20, None) == b.S2R_ERR_SIZE
    assert lib.s2r_topk_blocks(0x1004, None, 1000, 10, 5, 0x2000, None, 0x4000, 1 << 20, None) == b.S2R_ERR_ALIGN
    assert lib.s2r_topk_blocks(0x1000, None, 1000, 10, 5, 0x2000, None, 0x4000, 64, None) == b.S2R_ERR_WORKSPACE


def test_topk_encode_blocks_argument_checks():
    import ctypes
    lib = b.load()
    n, B, d, w, cap = 1 << 20, 256, 3, 1 << 14, 40
    each = b.topk_encode_blocks_workspace_bytes(n, B, d, w, cap)
    assert each == b.topk_workspace_bytes(n, B) + b.encode_blocks_workspace_bytes(n, B, d, w, cap) and each % 256 == 0
    assert b.topk_encode_blocks_workspace_bytes(n, 0, d, w, cap) == 0
    assert b.topk_encode_blocks_workspace_bytes(n, B, d, 1000, cap) == 0
    one = lambda v: (ctypes.c_void_p * 1)(v)
    call = lambda grads, bitmaps, ws, ws_bytes, block=B, sketches=one(0x3000): lib.s2r_topk_encode_blocks_batch(
        grads, None, 1, n, block, 40, d, w, 0, sketches, bitmaps, None, 0, 0x6000, ws, ws_bytes, None)
    assert call(one(0x1000), None, 0x10000, 1 << 30) == b.S2R_ERR_NULL
    assert call(None, one(0x5000), 0x10000, 1 << 30) == b.S2R_ERR_NULL
    assert call(one(0x1000), one(0x5000), 0x10000, 1 << 30, block=0) == b.S2R_ERR_SIZE
    assert call(one(0x1004), one(0x5000), 0x10000, 1 << 30) == b.S2R_ERR_ALIGN
    assert call(one(0x1000), one(0x5000), 0x10000, 4096) == b.S2R_ERR_WORKSPACE
    assert call(one(0x1000), one(0x5000), None, 1 << 30) == b.S2R_ERR_WORKSPACE


def test_decode_blocks_update_argument_checks():
    lib = b.load()
    n, B, d, w = 1 << 20, 256, 3, 1 << 14
    need = b.decode_blocks_update_workspace_bytes(n, B, d, w)
    assert need >= b.blocks_workspace_bytes(n, B, d, w) + 4 * (n // B) and need % 256 == 0
    assert b.decode_blocks_update_workspace_bytes(n, 0, d, w) == 0
    args = (0x1000, 0x2000, n, B, d, w, 0)
    assert lib.s2r_decode_blocks_update(*args, None, 1.0, 0x4000, 0x10000, need, None) == b.S2R_ERR_NULL
    assert lib.s2r_decode_blocks_update(*args, 0x3002, 1.0, 0x4000, 0x10000, need, None) == b.S2R_ERR_ALIGN
    assert lib.s2r_decode_blocks_update(*args, 0x3000, 1.0, 0x4000, 0x10000, need - 256, None) == b.S2R_ERR_WORKSPACE
    assert lib.s2r_decode_blocks_update(0x1000, 0x2000, n, 0, d, w, 0, 0x3000, 1.0, 0x4000, 0x10000, need, None) == b.S2R_ERR_SIZE
    assert lib.s2r_decode_blocks_update(0x1000, 0x2000, n, B, d, 1000, 0, 0x3000, 1.0, 0x4000, 0x10000, need, None) == b.S2R_ERR_WIDTH


def test_decode_update_argument_checks():
    lib = b.load()
    args = (0x1000, 0x2000, 1 << 20, 3, 1 << 14, 0)
    assert lib.s2r_decode_update(*args, None, 1.0, None, None, 0, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_NULL
    assert lib.s2r_decode_update(*args, 0x3002, 1.0, None, None, 0, 0x4000, 0x5000, 1 << 20, None) == b.S2R_ERR_ALIGN
    assert lib.s2r_decode_update(*args, 0x3000, 1.0, None, None, 0, 0x4000, None, 1 << 20, None) == b.S2R_ERR_WORKSPACE
