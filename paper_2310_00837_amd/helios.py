"""Thin Python binding of libhelios.so (argument marshalling only).

Every step of the path runs in the library's HIP kernels; torch is used for
device memory and streams.  There is no fallback: if the library is missing,
importing this module raises.
"""
from __future__ import annotations

import atexit
import ctypes as C
import os
import weakref
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libhelios.so")

OK, EINVAL, ECAPACITY, EHIP, ESTATE, EDATA, EINTERNAL = 0, -1, -2, -3, -4, -5, -6
MAX_HOPS, MAX_FANOUT = 8, 1024
DEDUP_NOALLOC_MAX_IDS = 262144
PARAM_HBM_GATHER_BLOCKS, PARAM_HOST_GATHER_BLOCKS, PARAM_SPLIT_COPIES = 1, 2, 3
PARAM_MISSQ_TIMEOUT_US, PARAM_MISSQ_WAVES, PARAM_SERVE_MISSES = 4, 5, 6
_NAMES = {0: "HELIOS_OK", -1: "HELIOS_EINVAL", -2: "HELIOS_ECAPACITY", -3: "HELIOS_EHIP", -4: "HELIOS_ESTATE",
          -5: "HELIOS_EDATA", -6: "HELIOS_EINTERNAL"}

# every symbol include/helios.h declares
EXPORTS = ["helios_create", "helios_destroy", "helios_last_error", "helios_reserve", "helios_sync",
           "helios_csr_load", "helios_cache_build", "helios_cache_fill", "helios_sample", "helios_dedup", "helios_dedup_noalloc",
           "helios_gather", "helios_gather_miss", "helios_prepare_batch", "helios_host_alloc", "helios_host_free", "helios_calibration_copy", "helios_make_blocks",
           "helios_hotness_add", "helios_hotness_order", "helios_plan_create", "helios_plan_launch", "helios_plan_wait", "helios_plan_make_blocks", "helios_plan_destroy",
           "helios_gang_create", "helios_gang_launch", "helios_gang_wait", "helios_gang_make_blocks", "helios_gang_destroy", "helios_set_param", "helios_set_timing",
           "helios_gather_times", "helios_batch_ticks", "helios_missq_create", "helios_missq_submit", "helios_missq_complete",
           "helios_missq_attach", "helios_missq_faulted", "helios_missq_counters", "helios_missq_destroy"]


class HopOut(C.Structure):
    _fields_ = [("frontier", C.c_void_p), ("frontier_cap", C.c_int64), ("indptr", C.c_void_p),
                ("flat", C.c_void_p), ("flat_cap", C.c_int64)]


class BlockOut(C.Structure):
    _fields_ = [("row_local", C.c_void_p), ("col_local", C.c_void_p)]


class BatchBuffersC(C.Structure):
    _fields_ = [("hops", C.POINTER(HopOut)), ("sizes", C.c_void_p), ("unique", C.c_void_p), ("unique_cap", C.c_int64),
                ("inverse", C.c_void_p), ("n_unique", C.c_void_p), ("out", C.c_void_p), ("miss_pos", C.c_void_p),
                ("miss_id", C.c_void_p), ("miss_slot", C.c_void_p), ("miss_cap", C.c_int64), ("stats", C.c_void_p)]


MAX_GANG = 4


class RoleTicks(C.Structure):
    _fields_ = [("kind", C.c_int32), ("stage", C.c_int32), ("workgroups", C.c_int64), ("start", C.c_uint64),
                ("end", C.c_uint64)]


ROLE_SAMPLE, ROLE_COMPACT_HOP, ROLE_COMPACT_LOOKUP, ROLE_COPY_HOST, ROLE_COPY_HBM, ROLE_INVERSE, ROLE_COPY_STANDIN = 1, 2, 3, 4, 5, 6, 7


class HeliosError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_NAMES.get(code, code)}: {msg}")
        self.code = code


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2310_00837_amd.build`")
    lib = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        getattr(lib, name)                      # raises AttributeError if a symbol is missing
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    lib.helios_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.helios_destroy.argtypes = [vp]
    lib.helios_last_error.argtypes = [vp]
    lib.helios_last_error.restype = C.c_char_p
    lib.helios_reserve.argtypes = [vp, i64]
    lib.helios_sync.argtypes = [vp]
    lib.helios_csr_load.argtypes = [vp, i64, i64, vp, vp]
    lib.helios_cache_build.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp]
    lib.helios_cache_fill.argtypes = [vp, vp, vp, i64, i64, i32, vp]
    lib.helios_sample.argtypes = [vp, vp, i64, C.POINTER(i32), i32, C.c_uint64, C.POINTER(HopOut), vp]
    lib.helios_dedup.argtypes = [vp, vp, i64, vp, i64, vp, vp]
    lib.helios_dedup_noalloc.argtypes = [vp, vp, i64, vp, i64, vp, vp]
    lib.helios_gather.argtypes = [vp, vp, i64, vp, vp, vp, vp, i64, vp]
    lib.helios_gather_miss.argtypes = [vp, vp, vp, i64, vp, vp, i64]
    lib.helios_prepare_batch.argtypes = [vp, vp, i64, C.POINTER(i32), i32, C.c_uint64, C.POINTER(HopOut), vp,
                                         vp, i64, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.helios_calibration_copy.argtypes = [vp, vp, vp, i64]
    lib.helios_make_blocks.argtypes = [vp, C.POINTER(HopOut), i32, C.POINTER(BlockOut)]
    lib.helios_hotness_add.argtypes = [vp, vp, i64, vp, vp]
    lib.helios_hotness_order.argtypes = [vp, vp, vp]
    lib.helios_plan_create.argtypes = [vp, i64, C.POINTER(i32), i32, C.POINTER(HopOut), vp, vp, i64, vp, vp, vp, vp, vp,
                                       vp, i64, vp, C.POINTER(vp)]
    lib.helios_plan_launch.argtypes = [vp, vp, C.c_uint64]
    lib.helios_plan_wait.argtypes = [vp]
    lib.helios_plan_make_blocks.argtypes = [vp, C.POINTER(BlockOut)]
    lib.helios_plan_destroy.argtypes = [vp]
    lib.helios_gang_create.argtypes = [C.POINTER(vp), i32, i64, C.POINTER(i32), i32, C.POINTER(BatchBuffersC), C.POINTER(vp)]
    lib.helios_gang_launch.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_uint64)]
    lib.helios_gang_wait.argtypes = [vp, C.POINTER(i32)]
    lib.helios_gang_make_blocks.argtypes = [vp, i32, C.POINTER(BlockOut)]
    lib.helios_gang_destroy.argtypes = [vp]
    lib.helios_host_alloc.argtypes = [i64]
    lib.helios_host_alloc.restype = vp
    lib.helios_host_free.argtypes = [vp]
    lib.helios_set_param.argtypes = [vp, C.c_int, i64]
    lib.helios_set_timing.argtypes = [vp, C.c_int]
    lib.helios_gather_times.argtypes = [vp] + [C.POINTER(C.c_float)] * 4
    lib.helios_batch_ticks.argtypes = [vp, C.POINTER(RoleTicks), i32, C.POINTER(i32), C.POINTER(C.c_double)]
    lib.helios_missq_create.argtypes = [vp, i32, i32, i32, C.POINTER(vp)]
    lib.helios_missq_submit.argtypes = [vp, vp, vp, i64, vp, i64]
    lib.helios_missq_complete.argtypes = [vp, vp]
    lib.helios_missq_attach.argtypes = [vp, vp]
    lib.helios_missq_faulted.argtypes = [vp]
    lib.helios_missq_counters.argtypes = [vp, C.POINTER(i64)]
    lib.helios_missq_destroy.argtypes = [vp]
    return lib


_lib = load_library()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous()
    return t.data_ptr()


def _is_pinned(t: torch.Tensor) -> bool:
    try:
        return bool(t.is_pinned())
    except RuntimeError:
        return False


def _dev(t: torch.Tensor, dtype: torch.dtype, what: str) -> torch.Tensor:
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{what}: expected a contiguous {dtype} tensor on the GPU")
    return t


def _dev_accessible(t: torch.Tensor, dtype: torch.dtype, what: str) -> torch.Tensor:
    if t.dtype != dtype or not t.is_contiguous() or not (t.is_cuda or _is_pinned(t)):
        raise TypeError(f"{what}: expected a contiguous {dtype} tensor on the GPU or in pinned host memory")
    return t


class PinnedBuffer:
    """Pinned, GPU-mapped host memory from helios_host_alloc, seen as a torch tensor.
    Unlike torch's pinned allocator it takes exactly the bytes asked for and gives them
    back on free().  Keep the object alive while `tensor` (or a view of it) is in use."""

    def __init__(self, shape, dtype: torch.dtype):
        n = 1
        for d in shape:
            n *= int(d)
        self.nbytes = max(n, 1) * torch.empty((), dtype=dtype).element_size()
        self.ptr = _lib.helios_host_alloc(self.nbytes)
        if not self.ptr:
            raise MemoryError(f"helios_host_alloc({self.nbytes}) failed")
        self._raw = (C.c_uint8 * self.nbytes).from_address(self.ptr)
        flat = torch.frombuffer(self._raw, dtype=dtype)
        self.tensor = flat[:n].reshape(tuple(int(d) for d in shape)) if n else flat[:0].reshape(tuple(shape))

    def free(self) -> None:
        if self.ptr:
            self.tensor = None
            self._raw = None
            _lib.helios_host_free(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pinned_empty(shape, dtype: torch.dtype) -> PinnedBuffer:
    return PinnedBuffer(shape, dtype)


@dataclass
class HopBuffers:
    """Caller-owned device outputs of one hop."""
    frontier: torch.Tensor     # int32[frontier_cap]
    indptr: torch.Tensor       # int64[frontier_cap + 1]
    flat: torch.Tensor         # int32[flat_cap]


def alloc_hops(n_seeds: int, fanouts: Sequence[int], device) -> List[HopBuffers]:
    """Worst-case buffers: frontier_cap(0) = n_seeds, flat_cap(h) = frontier_cap(h) * fanouts[h]."""
    hops, cap = [], n_seeds
    for f in fanouts:
        fr = torch.empty(max(cap, 1), dtype=torch.int32, device=device)
        ip = torch.empty(cap + 1, dtype=torch.int64, device=device)
        cap = cap * f
        fl = torch.empty(max(cap, 1), dtype=torch.int32, device=device)
        hops.append(HopBuffers(fr, ip, fl))
    return hops


class Plan:
    """A recorded batch (see helios_plan_create).  launch(seeds, rng_seed) enqueues one mini-batch."""

    def __init__(self, ctx: "Helios", handle, n_seeds: int, keep):
        self._ctx, self._p, self.n_seeds, self._keep = ctx, handle, n_seeds, keep
        ctx._children.append(self)

    def launch(self, seeds: torch.Tensor, rng_seed: int) -> None:
        _dev(seeds, torch.int32, "seeds")
        assert seeds.numel() == self.n_seeds
        self._ctx._check(_lib.helios_plan_launch(self._p, _ptr(seeds), C.c_uint64(rng_seed)))

    def wait(self) -> None:
        """Waits for this plan's last launch only; raises on the device-side errors of this plan's batches."""
        self._ctx._check(_lib.helios_plan_wait(self._p))

    def make_blocks(self, row_local: Sequence[torch.Tensor], col_local: Sequence[torch.Tensor]) -> None:
        """The hops of the plan's last launch in local numbering (see helios_plan_make_blocks)."""
        hops = self._keep[0]
        arr = (BlockOut * len(hops))()
        for i, hb in enumerate(hops):
            _dev(row_local[i], torch.int32, "row_local"), _dev(col_local[i], torch.int32, "col_local")
            assert row_local[i].numel() >= min(hb.frontier.numel(), hb.indptr.numel() - 1)
            assert col_local[i].numel() >= hb.flat.numel()
            arr[i] = BlockOut(row_local[i].data_ptr(), col_local[i].data_ptr())
        self._ctx._check(_lib.helios_plan_make_blocks(self._p, arr))

    def destroy(self) -> None:
        if self._p is not None and self._p.value:
            _lib.helios_plan_destroy(self._p)
            self._p = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


@dataclass
class BatchBuffers:
    """The caller-owned outputs of one whole-path batch (the buffer arguments of helios_prepare_batch)."""
    hops: Sequence["HopBuffers"]
    sizes: torch.Tensor
    unique: torch.Tensor
    inverse: Optional[torch.Tensor]
    n_unique: torch.Tensor
    out: torch.Tensor
    miss_pos: torch.Tensor
    miss_id: torch.Tensor
    miss_slot: torch.Tensor
    stats: torch.Tensor


class Gang:
    """The mini-batches of several contexts recorded into the same launches (see helios_gang_create).
    launch(seeds, rng_seeds) enqueues one mini-batch per member on the contexts' shared stream."""

    def __init__(self, ctxs: Sequence["Helios"], n_seeds: int, fanouts: Sequence[int], buffers: Sequence[BatchBuffers]):
        assert len(ctxs) == len(buffers) and len(ctxs) >= 1
        self._ctxs, self.n_seeds, self._keep = list(ctxs), n_seeds, list(buffers)
        self._g = C.c_void_p()
        n = len(ctxs)
        handles = (C.c_void_p * n)(*[c._h for c in ctxs])
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        arr = (BatchBuffersC * n)()
        self._hop_arrays = []
        for m, (c, b) in enumerate(zip(ctxs, buffers)):
            assert len(b.hops) == len(fanouts)
            _dev(b.unique, torch.int32, "unique")
            _dev_accessible(b.sizes, torch.int64, "sizes"), _dev_accessible(b.n_unique, torch.int64, "n_unique")
            _dev_accessible(b.stats, torch.int64, "stats")
            if b.inverse is not None:
                _dev(b.inverse, torch.int32, "inverse")
                assert b.inverse.numel() >= n_seeds + sum(h.flat.numel() for h in b.hops)
            if not b.out.is_cuda or b.out.numel() * b.out.element_size() < b.unique.numel() * c.row_bytes:
                raise TypeError("out must be a GPU tensor with room for unique_cap rows")
            for t in (b.miss_pos, b.miss_id, b.miss_slot):
                _dev(t, torch.int32, "miss list")
            hop_arr = c._hop_array(b.hops)
            self._hop_arrays.append(hop_arr)
            arr[m] = BatchBuffersC(hop_arr, _ptr(b.sizes), _ptr(b.unique), b.unique.numel(), _ptr(b.inverse), _ptr(b.n_unique),
                                   _ptr(b.out), _ptr(b.miss_pos), _ptr(b.miss_id), _ptr(b.miss_slot),
                                   min(b.miss_pos.numel(), b.miss_id.numel(), b.miss_slot.numel()), _ptr(b.stats))
        ctxs[0]._check(_lib.helios_gang_create(handles, n, n_seeds, fan, len(fanouts), arr, C.byref(self._g)))
        for c in ctxs:
            c._children.append(self)

    def launch(self, seeds: Sequence[torch.Tensor], rng_seeds: Sequence[int]) -> None:
        n = len(self._ctxs)
        assert len(seeds) == n and len(rng_seeds) == n
        for t in seeds:
            _dev(t, torch.int32, "seeds")
            assert t.numel() == self.n_seeds
        ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in seeds])
        rs = (C.c_uint64 * n)(*[int(r) for r in rng_seeds])
        self._ctxs[0]._check(_lib.helios_gang_launch(self._g, ptrs, rs))

    def wait(self, raise_on_error: bool = True) -> List[int]:
        """Waits for the gang's last launch; returns every member's own device-side error code."""
        st = (C.c_int32 * len(self._ctxs))()
        rc = _lib.helios_gang_wait(self._g, st)
        if rc != OK and raise_on_error:
            self._ctxs[0]._check(rc)
        return list(st)

    def make_blocks(self, member: int, row_local: Sequence[torch.Tensor], col_local: Sequence[torch.Tensor]) -> None:
        hops = self._keep[member].hops
        arr = (BlockOut * len(hops))()
        for i, hb in enumerate(hops):
            _dev(row_local[i], torch.int32, "row_local"), _dev(col_local[i], torch.int32, "col_local")
            assert row_local[i].numel() >= min(hb.frontier.numel(), hb.indptr.numel() - 1)
            assert col_local[i].numel() >= hb.flat.numel()
            arr[i] = BlockOut(row_local[i].data_ptr(), col_local[i].data_ptr())
        self._ctxs[member]._check(_lib.helios_gang_make_blocks(self._g, member, arr))

    def destroy(self) -> None:
        if self._g is not None and self._g.value:
            _lib.helios_gang_destroy(self._g)
            self._g = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class MissQueue:
    """An asynchronous miss queue of a context (see helios_missq_create): submit() and complete()
    alternate; attach() makes every batch of the context submit its own misses."""

    def __init__(self, ctx: "Helios", n_queues: int, queue_depth: int, n_service_threads: int):
        self._ctx, self._q = ctx, C.c_void_p()
        ctx._check(_lib.helios_missq_create(ctx._h, n_queues, queue_depth, n_service_threads, C.byref(self._q)))
        ctx._children.append(self)

    def submit(self, miss_pos: torch.Tensor, miss_slot: torch.Tensor, n_miss_max: int,
               n_miss_dev: Optional[torch.Tensor], out_rows: int) -> None:
        _dev(miss_pos, torch.int32, "miss_pos"), _dev(miss_slot, torch.int32, "miss_slot")
        assert n_miss_max <= min(miss_pos.numel(), miss_slot.numel())
        if n_miss_dev is not None:
            _dev_accessible(n_miss_dev, torch.int64, "n_miss_dev")
        self._ctx._check(_lib.helios_missq_submit(self._q, _ptr(miss_pos), _ptr(miss_slot), n_miss_max, _ptr(n_miss_dev),
                                                  out_rows))

    def complete(self, out: torch.Tensor) -> None:
        if not out.is_cuda or not out.is_contiguous():
            raise TypeError("out must be a contiguous GPU tensor")
        self._ctx._check(_lib.helios_missq_complete(self._q, _ptr(out)))

    def attach(self) -> None:
        self._ctx._check(_lib.helios_missq_attach(self._ctx._h, self._q))

    def detach(self) -> None:
        self._ctx._check(_lib.helios_missq_attach(self._ctx._h, None))

    def faulted(self) -> bool:
        return bool(_lib.helios_missq_faulted(self._q))

    def counters(self):
        """(rounds opened, rounds the service threads have finished, commands served)"""
        v = (C.c_int64 * 3)()
        self._ctx._check(_lib.helios_missq_counters(self._q, v))
        return tuple(v)

    def destroy(self) -> None:
        if self._q is not None and self._q.value:
            _lib.helios_missq_destroy(self._q)
            self._q = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_live_contexts = weakref.WeakSet()


@atexit.register
def _close_all() -> None:
    """Miss queues own host threads: stop them (and free every context) before the interpreter and the
    HIP runtime shut down."""
    for ctx in list(_live_contexts):
        try:
            ctx.close()
        except Exception:
            pass


class Helios:
    """One library context on one device and stream."""

    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None):
        self._h = C.c_void_p()
        self._keep = {}
        self._children = []          # plans and miss queues: destroyed before the context
        s = stream.cuda_stream if stream is not None else torch.cuda.current_stream(device).cuda_stream
        self._stream_ptr = s
        rc = _lib.helios_create(C.byref(self._h), device, C.c_void_p(s))
        if rc != OK:
            self._h = C.c_void_p()
            raise HeliosError(rc, "helios_create failed")
        self.device = torch.device("cuda", device)
        self.row_bytes = 0
        _live_contexts.add(self)

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            for child in self._children:
                child.destroy()
            self._children = []
            _lib.helios_destroy(self._h)
            self._h = C.c_void_p()
            self._keep.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int) -> None:
        if rc != OK:
            raise HeliosError(rc, _lib.helios_last_error(self._h).decode())

    # ---- plumbing
    def reserve(self, max_ids: int) -> None:
        self._check(_lib.helios_reserve(self._h, max_ids))

    def sync(self) -> None:
        self._check(_lib.helios_sync(self._h))

    def calibration_copy(self, src: torch.Tensor, dst: torch.Tensor) -> None:
        nbytes = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() == nbytes and nbytes % 16 == 0
        self._check(_lib.helios_calibration_copy(self._h, _ptr(src), _ptr(dst), nbytes))

    def set_param(self, param: int, value: int) -> None:
        self._check(_lib.helios_set_param(self._h, param, value))

    def set_timing(self, level: int) -> None:
        """0 off, 1 device clock per role, 2 HIP events on the two copy kernels (split copies, direct launches)."""
        self._check(_lib.helios_set_timing(self._h, int(level)))

    def gather_times(self):
        """(hbm_ms, host_ms, hbm_event_ms, host_event_ms) of the last gather."""
        v = [C.c_float() for _ in range(4)]
        self._check(_lib.helios_gather_times(self._h, *[C.byref(x) for x in v]))
        return tuple(x.value for x in v)

    def batch_ticks(self):
        """([(kind, stage, workgroups, start, end), ...] of the timed roles of the last batch, ticks per microsecond)"""
        buf, n, rate = (RoleTicks * 48)(), C.c_int32(), C.c_double()
        self._check(_lib.helios_batch_ticks(self._h, buf, 48, C.byref(n), C.byref(rate)))
        return [(r.kind, r.stage, r.workgroups, r.start, r.end) for r in buf[:n.value]], rate.value

    # ---- S0
    def csr_load(self, offsets: torch.Tensor, indices: torch.Tensor) -> None:
        _dev_accessible(offsets, torch.int64, "offsets")
        _dev_accessible(indices, torch.int32, "indices")
        self._keep["csr"] = (offsets, indices)
        self.n_nodes = offsets.numel() - 1
        self._check(_lib.helios_csr_load(self._h, self.n_nodes, indices.numel(), _ptr(offsets), _ptr(indices)))

    def cache_build(self, order: torch.Tensor, hbm_rows: int, host_rows: int, row_bytes: int,
                    hbm_table: Optional[torch.Tensor], host_table: Optional[torch.Tensor],
                    standin_table: Optional[torch.Tensor]) -> None:
        _dev(order, torch.int32, "order")
        if hbm_table is not None and not hbm_table.is_cuda:
            raise TypeError("hbm_table must be on the GPU")
        for t, w in ((host_table, "host_table"), (standin_table, "standin_table")):
            if t is not None and not (_is_pinned(t) or t.is_cuda):
                raise TypeError(f"{w} must be pinned host memory")
        self._keep["cache"] = (order, hbm_table, host_table, standin_table)
        self.row_bytes = row_bytes
        self._check(_lib.helios_cache_build(self._h, _ptr(order), hbm_rows, host_rows, row_bytes, _ptr(hbm_table),
                                            _ptr(host_table), _ptr(standin_table)))

    def cache_fill(self, src_table: torch.Tensor, order: torch.Tensor, first_rank: int, n_rows: int,
                   dst: torch.Tensor) -> None:
        row_bytes = src_table.shape[1] * src_table.element_size()
        assert dst.shape[1] * dst.element_size() == row_bytes and dst.shape[0] >= n_rows
        assert first_rank + n_rows <= order.numel()
        _dev(order, torch.int32, "order")
        self._check(_lib.helios_cache_fill(self._h, _ptr(src_table), _ptr(order), first_rank, n_rows, row_bytes,
                                           _ptr(dst)))

    # ---- S1
    def _hop_array(self, hops: Sequence[HopBuffers]):
        arr = (HopOut * len(hops))()
        for i, h in enumerate(hops):
            _dev(h.frontier, torch.int32, "frontier"), _dev(h.indptr, torch.int64, "indptr"), _dev(h.flat, torch.int32, "flat")
            arr[i] = HopOut(h.frontier.data_ptr(), min(h.frontier.numel(), h.indptr.numel() - 1), h.indptr.data_ptr(),
                            h.flat.data_ptr(), h.flat.numel())
        return arr

    def sample(self, seeds: torch.Tensor, fanouts: Sequence[int], rng_seed: int, hops: Sequence[HopBuffers],
               sizes: torch.Tensor) -> None:
        _dev(seeds, torch.int32, "seeds")
        _dev_accessible(sizes, torch.int64, "sizes")
        assert sizes.numel() >= 2 * len(fanouts) and len(hops) == len(fanouts)
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        self._check(_lib.helios_sample(self._h, _ptr(seeds), seeds.numel(), fan, len(fanouts),
                                       C.c_uint64(rng_seed), self._hop_array(hops), _ptr(sizes)))

    # ---- S2
    def dedup(self, ids: torch.Tensor, unique: torch.Tensor, inverse: Optional[torch.Tensor],
              n_unique: torch.Tensor, n_ids: Optional[int] = None) -> None:
        _dev(ids, torch.int32, "ids"), _dev(unique, torch.int32, "unique")
        _dev_accessible(n_unique, torch.int64, "n_unique")
        n = ids.numel() if n_ids is None else n_ids
        if inverse is not None:
            _dev(inverse, torch.int32, "inverse")
            assert inverse.numel() >= n
        self._check(_lib.helios_dedup(self._h, _ptr(ids), n, _ptr(unique), unique.numel(), _ptr(inverse),
                                      _ptr(n_unique)))

    def dedup_noalloc(self, ids: torch.Tensor, unique: torch.Tensor, inverse: Optional[torch.Tensor],
                      n_unique: torch.Tensor, n_ids: Optional[int] = None) -> None:
        """helios_dedup on the library's fixed scratch array: allocates nothing (at most DEDUP_NOALLOC_MAX_IDS IDs)."""
        _dev(ids, torch.int32, "ids"), _dev(unique, torch.int32, "unique")
        _dev_accessible(n_unique, torch.int64, "n_unique")
        n = ids.numel() if n_ids is None else n_ids
        if inverse is not None:
            _dev(inverse, torch.int32, "inverse")
            assert inverse.numel() >= n
        self._check(_lib.helios_dedup_noalloc(self._h, _ptr(ids), n, _ptr(unique), unique.numel(), _ptr(inverse),
                                              _ptr(n_unique)))

    # ---- S3 + S4 + S5
    def gather(self, ids: torch.Tensor, out: torch.Tensor, miss_pos: torch.Tensor, miss_id: torch.Tensor,
               miss_slot: torch.Tensor, stats: torch.Tensor, n_ids: Optional[int] = None) -> None:
        _dev(ids, torch.int32, "ids")
        n = ids.numel() if n_ids is None else n_ids
        if not out.is_cuda or not out.is_contiguous() or out.numel() * out.element_size() < n * self.row_bytes:
            raise TypeError("out must be a contiguous GPU tensor of n_ids x row_bytes")
        for t in (miss_pos, miss_id, miss_slot):
            _dev(t, torch.int32, "miss list")
        _dev_accessible(stats, torch.int64, "stats")
        assert stats.numel() >= 4
        cap = min(miss_pos.numel(), miss_id.numel(), miss_slot.numel())
        self._check(_lib.helios_gather(self._h, _ptr(ids), n, _ptr(out), _ptr(miss_pos), _ptr(miss_id),
                                       _ptr(miss_slot), cap, _ptr(stats)))

    # ---- S6
    def gather_miss(self, miss_pos: torch.Tensor, miss_slot: torch.Tensor, n_miss_max: int,
                    n_miss_dev: Optional[torch.Tensor], out: torch.Tensor, out_rows: Optional[int] = None) -> None:
        _dev(miss_pos, torch.int32, "miss_pos"), _dev(miss_slot, torch.int32, "miss_slot")
        assert n_miss_max <= min(miss_pos.numel(), miss_slot.numel())
        if n_miss_dev is not None:
            _dev_accessible(n_miss_dev, torch.int64, "n_miss_dev")
        if not out.is_cuda or not out.is_contiguous():
            raise TypeError("out must be a contiguous GPU tensor")
        rows = out.numel() * out.element_size() // max(self.row_bytes, 1) if out_rows is None else out_rows
        self._check(_lib.helios_gather_miss(self._h, _ptr(miss_pos), _ptr(miss_slot), n_miss_max, _ptr(n_miss_dev),
                                            _ptr(out), rows))

    # ---- recorded batch (HIP graph)
    def plan_create(self, n_seeds: int, fanouts: Sequence[int], hops: Sequence[HopBuffers], sizes: torch.Tensor,
                    unique: torch.Tensor, inverse: Optional[torch.Tensor], n_unique: torch.Tensor, out: torch.Tensor,
                    miss_pos: torch.Tensor, miss_id: torch.Tensor, miss_slot: torch.Tensor,
                    stats: torch.Tensor) -> "Plan":
        _dev(unique, torch.int32, "unique")
        _dev_accessible(sizes, torch.int64, "sizes"), _dev_accessible(n_unique, torch.int64, "n_unique")
        _dev_accessible(stats, torch.int64, "stats")
        if inverse is not None:
            _dev(inverse, torch.int32, "inverse")
            assert inverse.numel() >= n_seeds + sum(h.flat.numel() for h in hops)
        if not out.is_cuda or out.numel() * out.element_size() < unique.numel() * self.row_bytes:
            raise TypeError("out must be a GPU tensor with room for unique_cap rows")
        cap = min(miss_pos.numel(), miss_id.numel(), miss_slot.numel())
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        handle = C.c_void_p()
        self._check(_lib.helios_plan_create(
            self._h, n_seeds, fan, len(fanouts), self._hop_array(hops), _ptr(sizes), _ptr(unique), unique.numel(),
            _ptr(inverse), _ptr(n_unique), _ptr(out), _ptr(miss_pos), _ptr(miss_id), _ptr(miss_slot), cap, _ptr(stats),
            C.byref(handle)))
        keep = (hops, sizes, unique, inverse, n_unique, out, miss_pos, miss_id, miss_slot, stats)
        return Plan(self, handle, n_seeds, keep)

    # ---- batch generation, pre-sampling hotness
    def make_blocks(self, hops: Sequence[HopBuffers], row_local: Sequence[torch.Tensor],
                    col_local: Sequence[torch.Tensor]) -> None:
        arr = (BlockOut * len(hops))()
        for i, hb in enumerate(hops):
            _dev(row_local[i], torch.int32, "row_local"), _dev(col_local[i], torch.int32, "col_local")
            assert row_local[i].numel() >= min(hb.frontier.numel(), hb.indptr.numel() - 1)
            assert col_local[i].numel() >= hb.flat.numel()
            arr[i] = BlockOut(row_local[i].data_ptr(), col_local[i].data_ptr())
        self._check(_lib.helios_make_blocks(self._h, self._hop_array(hops), len(hops), arr))

    def hotness_add(self, ids: torch.Tensor, n_max: int, n_dev: Optional[torch.Tensor], counts: torch.Tensor) -> None:
        _dev(ids, torch.int32, "ids"), _dev(counts, torch.int32, "counts")
        assert n_max <= ids.numel() and counts.numel() >= self.n_nodes
        if n_dev is not None:
            _dev_accessible(n_dev, torch.int64, "n_dev")
        self._check(_lib.helios_hotness_add(self._h, _ptr(ids), n_max, _ptr(n_dev), _ptr(counts)))

    def hotness_order(self, counts: torch.Tensor, order: torch.Tensor) -> None:
        _dev(counts, torch.int32, "counts"), _dev(order, torch.int32, "order")
        assert counts.numel() >= self.n_nodes and order.numel() >= self.n_nodes
        self._check(_lib.helios_hotness_order(self._h, _ptr(counts), _ptr(order)))

    # ---- whole path
    def prepare_batch(self, seeds: torch.Tensor, fanouts: Sequence[int], rng_seed: int, hops: Sequence[HopBuffers],
                      sizes: torch.Tensor, unique: torch.Tensor, inverse: Optional[torch.Tensor],
                      n_unique: torch.Tensor, out: torch.Tensor, miss_pos: torch.Tensor, miss_id: torch.Tensor,
                      miss_slot: torch.Tensor, stats: torch.Tensor) -> None:
        _dev(seeds, torch.int32, "seeds"), _dev(unique, torch.int32, "unique")
        _dev_accessible(sizes, torch.int64, "sizes"), _dev_accessible(n_unique, torch.int64, "n_unique")
        _dev_accessible(stats, torch.int64, "stats")
        if inverse is not None:
            _dev(inverse, torch.int32, "inverse")
            assert inverse.numel() >= seeds.numel() + sum(h.flat.numel() for h in hops)
        if not out.is_cuda or out.numel() * out.element_size() < unique.numel() * self.row_bytes:
            raise TypeError("out must be a GPU tensor with room for unique_cap rows")
        cap = min(miss_pos.numel(), miss_id.numel(), miss_slot.numel())
        fan = (C.c_int32 * len(fanouts))(*fanouts)
        self._check(_lib.helios_prepare_batch(
            self._h, _ptr(seeds), seeds.numel(), fan, len(fanouts), C.c_uint64(rng_seed), self._hop_array(hops),
            _ptr(sizes), _ptr(unique), unique.numel(), _ptr(inverse), _ptr(n_unique), _ptr(out), _ptr(miss_pos),
            _ptr(miss_id), _ptr(miss_slot), cap, _ptr(stats)))
