"""Thin ctypes binding of libs2r.so (the C ABI declared in include/s2r.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch tensors supply device memory and the stream handle; nothing is
computed with torch ops here.  There is no CPU fallback: if the shared library
has not been built, loading raises.
"""

from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_int32, c_size_t, c_uint32, c_uint64, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("S2R_LIBRARY") or os.path.join(HERE, "libs2r.so")

S2R_OK = 0
S2R_ERR_NULL = -1
S2R_ERR_SIZE = -2
S2R_ERR_WIDTH = -3
S2R_ERR_WORKSPACE = -4
S2R_ERR_LAUNCH = -5
S2R_ERR_ALIGN = -6
S2R_MAX_ROWS = 16
S2R_MAX_WORKERS = 64
S2R_KERNEL_ENCODE_SCAN = 0
S2R_KERNEL_DECODE = 1
S2R_KERNEL_ENCODE_SLICE = 2
S2R_KERNEL_TOPK_SCORES = 3
S2R_KERNEL_MERGE = 4
S2R_KERNEL_SLOTS = 5
S2R_INSERT_AUTO = 0
S2R_INSERT_ATOMIC = 1
S2R_INSERT_SLICE = 2
S2R_DECODE_AUTO = 0
S2R_DECODE_GATHER = 1
S2R_DECODE_SLICE = 2
S2R_DECODE_ROWS = 3



class Report(ctypes.Structure):
    """s2r_report"""
    _fields_ = [("insert_strategy", c_int32), ("decode_strategy", c_int32),
                ("scan_launch_workers", c_uint32), ("reserved", c_uint32)]


class Trace(ctypes.Structure):
    """struct s2r_trace (include/s2r_bench.h)"""
    _fields_ = [("begin", c_void_p * S2R_KERNEL_SLOTS), ("end", c_void_p * S2R_KERNEL_SLOTS)]


class Options(ctypes.Structure):
    """s2r_options"""
    _fields_ = [("struct_bytes", c_uint32), ("insert_strategy", c_int32), ("decode_strategy", c_int32),
                ("flags", c_uint32), ("expected_nnz", c_uint64), ("report", ctypes.POINTER(Report)),
                ("trace", ctypes.POINTER(Trace))]


_OPT = ctypes.POINTER(Options)
_ENCODE_ARGS = [c_void_p, c_uint64, c_uint32, c_uint32, c_uint64,
                c_void_p, c_void_p, c_void_p, c_void_p, c_uint64,
                c_void_p, c_void_p, c_size_t, c_void_p]
_ENCODE_BATCH_ARGS = [ctypes.POINTER(c_void_p), c_uint32, c_uint64, c_uint32, c_uint32, c_uint64,
                      ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p),
                      ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p), c_uint64,
                      c_void_p, c_void_p, c_size_t, c_void_p]
_DECODE_ARGS = [c_void_p, c_void_p, c_uint64, c_uint32, c_uint32, c_uint64,
                c_void_p, c_void_p, c_uint64, c_void_p, c_void_p,
                c_void_p, c_size_t, c_void_p]
_MERGE_HEAD = [ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p), c_uint32]
_MERGE_DECODE_ARGS = _MERGE_HEAD + [c_uint64, c_uint32, c_uint32, c_uint64, c_void_p, c_void_p,
                                    c_void_p, c_void_p, c_uint64, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
_MERGE_DECODE_BLOCKS_ARGS = _MERGE_HEAD + [c_uint64, c_uint32, c_uint32, c_uint32, c_uint64, c_void_p, c_void_p,
                                           c_void_p, c_void_p, c_uint64, c_void_p, c_void_p, c_size_t, c_void_p]
_ENCODE_BLOCKS_ARGS = [c_void_p, c_uint64, c_uint32, c_uint32, c_uint32, c_uint64,
                       c_void_p, c_void_p, c_void_p, c_uint64, c_void_p, c_void_p, c_size_t, c_void_p]
_ENCODE_BLOCKS_BATCH_ARGS = [ctypes.POINTER(c_void_p), c_uint32, c_uint64, c_uint32, c_uint32, c_uint32,
                             c_uint64, ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p),
                             ctypes.POINTER(c_void_p), c_uint64, c_void_p, c_void_p, c_size_t, c_void_p]
_DECODE_BLOCKS_ARGS = [c_void_p, c_void_p, c_uint64, c_uint32, c_uint32, c_uint32, c_uint64,
                       c_void_p, c_void_p, c_uint64, c_void_p, c_void_p, c_size_t, c_void_p]
_TOPK_ENCODE_ARGS = [ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p), c_uint32, c_uint64,
                     c_uint32, c_uint64, c_uint32, c_uint32, c_uint64,
                     ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p),
                     ctypes.POINTER(c_void_p), c_uint64, c_void_p, c_void_p, c_size_t,
                     c_void_p]

# every symbol include/s2r.h and include/s2r_bench.h declare: name -> (restype, argtypes)
SIGNATURES = {
    "s2r_version": (c_int32, []),
    "s2r_status_string": (c_char_p, [c_int32]),
    "s2r_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32]),
    "s2r_encode_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint64]),
    "s2r_hash_params": (c_int32, [c_uint64, c_uint32, ctypes.POINTER(c_uint64)]),
    "s2r_encode": (c_int32, _ENCODE_ARGS),
    "s2r_encode_ex": (c_int32, _ENCODE_ARGS + [_OPT]),
    "s2r_encode_batch": (c_int32, _ENCODE_BATCH_ARGS),
    "s2r_encode_batch_ex": (c_int32, _ENCODE_BATCH_ARGS + [_OPT]),
    "s2r_merge": (c_int32, [ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p),
                            c_uint32, c_uint64, c_uint32, c_uint32, c_uint64,
                            c_void_p, c_void_p, c_void_p]),
    "s2r_decode": (c_int32, _DECODE_ARGS),
    "s2r_decode_ex": (c_int32, _DECODE_ARGS + [_OPT]),
    "s2r_merge_decode": (c_int32, _MERGE_DECODE_ARGS),
    "s2r_merge_decode_ex": (c_int32, _MERGE_DECODE_ARGS + [_OPT]),
    "s2r_merge_decode_blocks": (c_int32, _MERGE_DECODE_BLOCKS_ARGS),
    "s2r_merge_decode_blocks_ex": (c_int32, _MERGE_DECODE_BLOCKS_ARGS + [_OPT]),
    "s2r_decode_noalloc": (c_int32, [c_void_p, c_void_p, c_uint64, c_uint32, c_uint32, c_uint64,
                                     c_void_p, c_void_p, c_uint64, c_void_p, c_void_p, c_void_p]),
    "s2r_decode_update": (c_int32, [c_void_p, c_void_p, c_uint64, c_uint32, c_uint32, c_uint64, c_void_p, ctypes.c_float,
                                    c_void_p, c_void_p, c_uint64, c_void_p, c_void_p, c_size_t, c_void_p]),
    "s2r_probe_read": (c_int32, [c_void_p, c_size_t, c_void_p, c_void_p]),
    "s2r_decode_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint64]),
    "s2r_blocks_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint32]),
    "s2r_encode_blocks_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint32, c_uint64]),
    "s2r_decode_blocks_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint32, c_uint64]),
    "s2r_encode_blocks": (c_int32, _ENCODE_BLOCKS_ARGS),
    "s2r_encode_blocks_ex": (c_int32, _ENCODE_BLOCKS_ARGS + [_OPT]),
    "s2r_encode_blocks_batch": (c_int32, _ENCODE_BLOCKS_BATCH_ARGS),
    "s2r_encode_blocks_batch_ex": (c_int32, _ENCODE_BLOCKS_BATCH_ARGS + [_OPT]),
    "s2r_topk_workspace_bytes": (c_size_t, [c_uint64, c_uint32]),
    "s2r_topk_blocks": (c_int32, [c_void_p, c_void_p, c_uint64, c_uint32, c_uint64, c_void_p, c_void_p,
                                  c_void_p, c_size_t, c_void_p]),
    "s2r_topk_blocks_batch": (c_int32, [ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p), c_uint32, c_uint64, c_uint32,
                                        c_uint64, ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p),
                                        c_void_p, c_size_t, c_void_p]),
    "s2r_topk_encode_blocks_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint32, c_uint64]),
    "s2r_topk_encode_blocks_batch": (c_int32, _TOPK_ENCODE_ARGS),
    "s2r_topk_encode_blocks_batch_ex": (c_int32, _TOPK_ENCODE_ARGS + [_OPT]),
    "s2r_decode_blocks_update_workspace_bytes": (c_size_t, [c_uint64, c_uint32, c_uint32, c_uint32]),
    "s2r_decode_blocks_update": (c_int32, [c_void_p, c_void_p, c_uint64, c_uint32, c_uint32, c_uint32, c_uint64,
                                           c_void_p, ctypes.c_float, c_void_p, c_void_p, c_size_t, c_void_p]),
    "s2r_decode_blocks": (c_int32, _DECODE_BLOCKS_ARGS),
    "s2r_decode_blocks_ex": (c_int32, _DECODE_BLOCKS_ARGS + [_OPT]),
}

_lib = None


class S2RError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load():
    """Load libs2r.so (once).  Raises if it is not built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2110_02140_amd.build` "
                "(the codec has no CPU fallback)")
        # torch ships its own HIP runtime (same SONAME as the system one): import it
        # first so that libs2r.so binds to the runtime that owns torch's memory and
        # streams instead of loading a second copy.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().s2r_status_string(status).decode()


def version() -> int:
    return load().s2r_version()


def workspace_bytes(n: int, d: int, w: int) -> int:
    return load().s2r_workspace_bytes(n, d, w)


def encode_workspace_bytes(n: int, d: int, w: int, cap: int) -> int:
    return load().s2r_encode_workspace_bytes(n, d, w, cap)


def hash_params(seed: int, d: int) -> list[tuple[int, int, int, int]]:
    buf = (c_uint64 * (4 * d))()
    st = load().s2r_hash_params(seed, d, buf)
    if st != S2R_OK:
        raise S2RError(st, "s2r_hash_params")
    return [tuple(int(buf[4 * j + q]) for q in range(4)) for j in range(d)]


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return getattr(stream, "cuda_stream", stream)


# ---------------------------------------------------------------- per-call options
# The library keeps no state: what steers a call travels in its s2r_options.  The
# defaults below are this module's (Python-side) and are marshalled into every call
# that has an _ex sibling; with nothing set the plain entry point is called.
class CallDefaults:
    def __init__(self):
        self.insert_strategy = S2R_INSERT_AUTO
        self.decode_strategy = S2R_DECODE_AUTO
        self.expected_nnz = 0          # encode calls: per worker; decode calls: union (see set_expected_nnz)
        self.expected_union = 0
        self.trace = {}                # slot -> (begin handle, end handle)
        self.want_report = False


defaults = CallDefaults()
_last_report = {"insert_strategy": S2R_INSERT_AUTO, "decode_strategy": S2R_DECODE_AUTO,
                "scan_launch_workers": 0}


def _check_strategy(value, allowed, what):
    if value not in allowed:
        raise S2RError(S2R_ERR_SIZE, what)


def set_insert_strategy(strategy: int):
    """S2R_INSERT_AUTO / _ATOMIC / _SLICE for this module's following encode calls."""
    _check_strategy(strategy, (S2R_INSERT_AUTO, S2R_INSERT_ATOMIC, S2R_INSERT_SLICE), "set_insert_strategy")
    defaults.insert_strategy = strategy


def set_decode_strategy(strategy: int):
    """S2R_DECODE_AUTO / _GATHER / _SLICE / _ROWS for this module's following decode calls."""
    _check_strategy(strategy, (S2R_DECODE_AUTO, S2R_DECODE_GATHER, S2R_DECODE_SLICE, S2R_DECODE_ROWS),
                    "set_decode_strategy")
    defaults.decode_strategy = strategy


def set_expected_nnz(per_worker: int = 0, union: int = 0):
    """The caller's estimates for the following calls (0: none; the lists' capacity stands in)."""
    defaults.expected_nnz, defaults.expected_union = int(per_worker), int(union)


def set_kernel_events(slot: int, ev_begin, ev_end):
    """Install (or, with None, remove) raw hipEvent_t handles around a kernel (s2r_trace slot)."""
    if not 0 <= slot < S2R_KERNEL_SLOTS:
        raise S2RError(S2R_ERR_SIZE, "set_kernel_events")
    if ev_begin is None and ev_end is None:
        defaults.trace.pop(slot, None)
    else:
        defaults.trace[slot] = (ev_begin, ev_end)


def want_report(flag: bool = True):
    """Ask every following call for its s2r_report (last_insert_strategy() and friends read it)."""
    defaults.want_report = bool(flag)


def last_insert_strategy() -> int:
    return _last_report["insert_strategy"]


def last_decode_strategy() -> int:
    return _last_report["decode_strategy"]


def scan_launch_workers() -> int:
    return _last_report["scan_launch_workers"]


def _handle(ev):
    return getattr(ev, "handle", ev)


def _call(name: str, args, decode: bool = False):
    """Call s2r_<name> with this module's defaults: the plain symbol when nothing is set,
    else its _ex sibling with an s2r_options built for this one call."""
    lib = load()
    d = defaults
    strategy_set = d.decode_strategy != S2R_DECODE_AUTO if decode else d.insert_strategy != S2R_INSERT_AUTO
    expect = d.expected_union if decode else d.expected_nnz
    if not (strategy_set or expect or d.trace or d.want_report):
        st = getattr(lib, name)(*args)
        if st != S2R_OK:
            raise S2RError(st, name)
        return
    opt = Options()
    opt.struct_bytes = ctypes.sizeof(Options)
    opt.insert_strategy = d.insert_strategy
    opt.decode_strategy = d.decode_strategy
    opt.expected_nnz = expect
    rep = Report()
    opt.report = ctypes.pointer(rep)
    if d.trace:
        tr = Trace()
        for slot, (b, e) in d.trace.items():
            tr.begin[slot], tr.end[slot] = _handle(b), _handle(e)
        opt.trace = ctypes.pointer(tr)
    st = getattr(lib, name + "_ex")(*args, ctypes.byref(opt))
    if st != S2R_OK:
        raise S2RError(st, name + "_ex")
    if decode:
        _last_report["decode_strategy"] = rep.decode_strategy
    else:
        _last_report.update(insert_strategy=rep.insert_strategy, scan_launch_workers=rep.scan_launch_workers)


def encode(grad, d, w, seed, sketch, bitmap, nz_idx, nz_val, nnz_out, workspace, stream=None, n=None):
    """s2r_encode on torch device tensors.  grad float32[n]; sketch float32[d*w];
    bitmap int64/uint64[ceil(n/64)]; nz_idx int32[cap] / nz_val float32[cap] or
    both None; nnz_out int64[1]; workspace uint8[>= workspace_bytes]."""
    n = grad.numel() if n is None else n
    cap = 0 if nz_idx is None else nz_idx.numel()
    _call("s2r_encode", (_ptr(grad), n, d, w, seed, _ptr(sketch), _ptr(bitmap), _ptr(nz_idx), _ptr(nz_val),
                           cap, _ptr(nnz_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                           _stream(stream)))


def _ptr_array(tensors):
    return (c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def encode_batch(grads, n, d, w, seed, sketches, bitmaps, nz_idx, nz_val, nnz_out, workspace, stream=None):
    """s2r_encode_batch: lists of W device tensors; nz_idx / nz_val lists or both
    None; nnz_out int64[W]; workspace uint8[>= W * workspace bytes]."""
    W = len(grads)
    cap = 0 if nz_idx is None else min(t.numel() for t in nz_idx)
    _call("s2r_encode_batch", (_ptr_array(grads), W, n, d, w, seed, _ptr_array(sketches), _ptr_array(bitmaps),
                                 None if nz_idx is None else _ptr_array(nz_idx),
                                 None if nz_val is None else _ptr_array(nz_val), cap, _ptr(nnz_out),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def merge(sketches, bitmaps, n, d, w, seed, sketch_out, bitmap_out, stream=None):
    """s2r_merge: sketches / bitmaps are lists of W device tensors."""
    W = len(sketches)
    sp = (c_void_p * W)(*[t.data_ptr() for t in sketches])
    bp = (c_void_p * W)(*[t.data_ptr() for t in bitmaps])
    st = load().s2r_merge(sp, bp, W, n, d, w, seed, _ptr(sketch_out), _ptr(bitmap_out), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_merge")


def decode(sketch, bitmap, n, d, w, seed, idx_out, val_out, count_out, dense_out, workspace, stream=None):
    """s2r_decode on torch device tensors (idx_out/val_out both None or both
    given; dense_out None or float32[n])."""
    cap = 0 if idx_out is None else idx_out.numel()
    _call("s2r_decode", (_ptr(sketch), _ptr(bitmap), n, d, w, seed, _ptr(idx_out), _ptr(val_out), cap,
                           _ptr(count_out), _ptr(dense_out), _ptr(workspace),
                           workspace.numel() * workspace.element_size(), _stream(stream)), decode=True)


def merge_decode(sketches, bitmaps, n, d, w, seed, sketch_out, bitmap_out, idx_out, val_out, count_out, dense_out,
                 workspace, stream=None):
    """s2r_merge_decode: s2r_merge and s2r_decode of its outputs in one call."""
    W = len(sketches)
    cap = 0 if idx_out is None else idx_out.numel()
    _call("s2r_merge_decode", (_ptr_array(sketches), _ptr_array(bitmaps), W, n, d, w, seed, _ptr(sketch_out),
                                 _ptr(bitmap_out), _ptr(idx_out), _ptr(val_out), cap, _ptr(count_out), _ptr(dense_out),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
          decode=True)


def merge_decode_blocks(sketches, block_bitmaps, n, block, d, w, seed, sketch_out, bitmap_out, blk_idx_out, val_out,
                        nblk_out, workspace, stream=None):
    """s2r_merge_decode_blocks: s2r_merge and s2r_decode_blocks of its outputs in one call."""
    W = len(sketches)
    cap = 0 if blk_idx_out is None else blk_idx_out.numel()
    _call("s2r_merge_decode_blocks", (_ptr_array(sketches), _ptr_array(block_bitmaps), W, n, block, d, w, seed,
                                        _ptr(sketch_out), _ptr(bitmap_out), _ptr(blk_idx_out), _ptr(val_out), cap,
                                        _ptr(nblk_out), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)), decode=True)


S2R_DECODE_NOALLOC_MAX_N = 1 << 27


def decode_noalloc(sketch, bitmap, n, d, w, seed, idx_out, val_out, count_out, dense_out, stream=None):
    """s2r_decode_noalloc: s2r_decode without a workspace (the library's static device scratch)."""
    cap = 0 if idx_out is None else idx_out.numel()
    st = load().s2r_decode_noalloc(_ptr(sketch), _ptr(bitmap), n, d, w, seed, _ptr(idx_out), _ptr(val_out), cap,
                                   _ptr(count_out), _ptr(dense_out), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_decode_noalloc")


def blocks_workspace_bytes(n: int, block: int, d: int, w: int) -> int:
    return load().s2r_blocks_workspace_bytes(n, block, d, w)


def encode_blocks_workspace_bytes(n: int, block: int, d: int, w: int, blk_cap: int) -> int:
    return load().s2r_encode_blocks_workspace_bytes(n, block, d, w, blk_cap)


def decode_blocks_workspace_bytes(n: int, block: int, d: int, w: int, blk_cap: int) -> int:
    return load().s2r_decode_blocks_workspace_bytes(n, block, d, w, blk_cap)


def encode_blocks(grad, block, d, w, seed, sketch, block_bitmap, blk_idx, nblk_out, workspace, stream=None, n=None):
    """s2r_encode_blocks on torch device tensors; blk_idx int32[blk_cap] or None."""
    n = grad.numel() if n is None else n
    cap = 0 if blk_idx is None else blk_idx.numel()
    _call("s2r_encode_blocks", (_ptr(grad), n, block, d, w, seed, _ptr(sketch), _ptr(block_bitmap), _ptr(blk_idx), cap,
                                  _ptr(nblk_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  _stream(stream)))


def encode_blocks_batch(grads, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, nblk_out, workspace, stream=None):
    """s2r_encode_blocks_batch: lists of W device tensors; blk_idx a list or None; nblk_out int64[W]."""
    cap = 0 if blk_idx is None else min(t.numel() for t in blk_idx)
    _call("s2r_encode_blocks_batch", (_ptr_array(grads), len(grads), n, block, d, w, seed, _ptr_array(sketches),
                                        _ptr_array(block_bitmaps), None if blk_idx is None else _ptr_array(blk_idx),
                                        cap, _ptr(nblk_out), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)))


def decode_blocks(sketch, block_bitmap, n, block, d, w, seed, blk_idx_out, val_out, nblk_out, workspace, stream=None):
    """s2r_decode_blocks; blk_idx_out int32[blk_cap] and val_out float32[blk_cap * block], or both None."""
    cap = 0 if blk_idx_out is None else blk_idx_out.numel()
    _call("s2r_decode_blocks", (_ptr(sketch), _ptr(block_bitmap), n, block, d, w, seed, _ptr(blk_idx_out),
                                  _ptr(val_out), cap, _ptr(nblk_out), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)), decode=True)


def topk_workspace_bytes(n: int, block: int) -> int:
    return load().s2r_topk_workspace_bytes(n, block)


def topk_blocks_batch(grads, residuals, n, block, K, sparse_out, kept_bitmaps, workspace, stream=None):
    """s2r_topk_blocks_batch: lists of W device tensors; residuals / kept_bitmaps lists or None."""
    st = load().s2r_topk_blocks_batch(_ptr_array(grads), None if residuals is None else _ptr_array(residuals),
                                      len(grads), n, block, K, _ptr_array(sparse_out),
                                      None if kept_bitmaps is None else _ptr_array(kept_bitmaps), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_topk_blocks_batch")


def topk_encode_blocks_workspace_bytes(n: int, block: int, d: int, w: int, blk_cap: int) -> int:
    return load().s2r_topk_encode_blocks_workspace_bytes(n, block, d, w, blk_cap)


def topk_encode_blocks_batch(grads, residuals, n, block, K, d, w, seed, sketches, block_bitmaps, blk_idx, nblk_out,
                             workspace, stream=None):
    """s2r_topk_encode_blocks_batch: lists of W device tensors; residuals / blk_idx lists or None."""
    cap = 0 if blk_idx is None else min(t.numel() for t in blk_idx)
    _call("s2r_topk_encode_blocks_batch", (_ptr_array(grads), None if residuals is None else _ptr_array(residuals),
                                             len(grads), n, block, K, d, w, seed, _ptr_array(sketches),
                                             _ptr_array(block_bitmaps), None if blk_idx is None else _ptr_array(blk_idx),
                                             cap, _ptr(nblk_out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)))


def topk_blocks(grad, residual, block, K, sparse_out, kept_bitmap, workspace, stream=None, n=None):
    """s2r_topk_blocks on torch device tensors (residual / kept_bitmap may be None)."""
    n = grad.numel() if n is None else n
    st = load().s2r_topk_blocks(_ptr(grad), _ptr(residual), n, block, K, _ptr(sparse_out), _ptr(kept_bitmap),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_topk_blocks")


def decode_update(sketch, bitmap, n, d, w, seed, params, scale, idx_out, val_out, count_out, workspace, stream=None):
    """s2r_decode_update: params float32[n] updated in place; idx_out / val_out may both be None."""
    cap = 0 if idx_out is None else idx_out.numel()
    st = load().s2r_decode_update(_ptr(sketch), _ptr(bitmap), n, d, w, seed, _ptr(params), float(scale), _ptr(idx_out),
                                  _ptr(val_out), cap, _ptr(count_out), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_decode_update")


def decode_blocks_update_workspace_bytes(n: int, block: int, d: int, w: int) -> int:
    return load().s2r_decode_blocks_update_workspace_bytes(n, block, d, w)


def decode_blocks_update(sketch, block_bitmap, n, block, d, w, seed, params, scale, nblk_out, workspace, stream=None):
    """s2r_decode_blocks_update: params float32[n] updated in place at every element of every set block."""
    st = load().s2r_decode_blocks_update(_ptr(sketch), _ptr(block_bitmap), n, block, d, w, seed, _ptr(params),
                                         float(scale), _ptr(nblk_out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_decode_blocks_update")


def decode_workspace_bytes(n: int, d: int, w: int, cap: int) -> int:
    return load().s2r_decode_workspace_bytes(n, d, w, cap)


def probe_read(src, sink, stream=None, nbytes=None):
    """s2r_probe_read over a device tensor (all of it unless nbytes is given); sink int64[1]."""
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    st = load().s2r_probe_read(_ptr(src), nbytes, _ptr(sink), _stream(stream))
    if st != S2R_OK:
        raise S2RError(st, "s2r_probe_read")


# ---------------------------------------------------------------- raw HIP events
_hip = None


def _hiprt():
    global _hip
    if _hip is None:
        load()
        _hip = ctypes.CDLL("libamdhip64.so.7")      # already loaded: same runtime as libs2r.so
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(c_void_p)]
        _hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(c_void_p), ctypes.c_uint]
        _hip.hipEventDestroy.argtypes = [c_void_p]
        _hip.hipEventSynchronize.argtypes = [c_void_p]
        _hip.hipEventRecord.argtypes = [c_void_p, c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), c_void_p, c_void_p]
    return _hip


class HipEvent:
    """A raw hipEvent_t, usable with set_kernel_events."""

    def __init__(self, timing: bool = True):
        self.handle = c_void_p()
        rc = (_hiprt().hipEventCreate(ctypes.byref(self.handle)) if timing else
              _hiprt().hipEventCreateWithFlags(ctypes.byref(self.handle), 0x2))      # hipEventDisableTiming
        if rc != 0:
            raise RuntimeError("hipEventCreate failed")

    def record(self, stream=None):
        if _hiprt().hipEventRecord(self.handle, _stream(stream)) != 0:
            raise RuntimeError("hipEventRecord failed")

    def synchronize(self):
        if _hiprt().hipEventSynchronize(self.handle) != 0:
            raise RuntimeError("hipEventSynchronize failed")

    def elapsed_ms(self, end: "HipEvent") -> float:
        ms = ctypes.c_float()
        if _hiprt().hipEventElapsedTime(ctypes.byref(ms), self.handle, end.handle) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def __del__(self):
        try:
            _hiprt().hipEventDestroy(self.handle)
        except Exception:
            pass
