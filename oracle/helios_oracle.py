"""ctypes front end of the CPU oracle (oracle/helios_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
Inputs and outputs are numpy arrays; nothing here does arithmetic of its own.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhelios_oracle.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        _lib = C.CDLL(_LIB_PATH)
        L = _lib
        L.orc_draw.restype = C.c_uint64
        L.orc_draw.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_uint32]
        L.orc_bounded.restype = C.c_uint64
        L.orc_bounded.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_sample_node.restype = C.c_int64
        L.orc_dedup.restype = C.c_int64
        L.orc_sample.restype = C.c_int
        L.orc_sample_hop.restype = C.c_int
        L.orc_rank_build.restype = C.c_int
        L.orc_num_threads.restype = C.c_int
        L.orc_local_ids.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def philox4x32_10(ctr, key):
    ctr = _arr(ctr, np.uint32)
    key = _arr(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def draw(rng_seed, node, hop, k):
    return int(lib().orc_draw(C.c_uint64(rng_seed), int(node), int(hop), int(k)))


def bounded(x, n):
    return int(lib().orc_bounded(C.c_uint64(x), C.c_uint64(n)))


def floyd_positions(d, f, draws):
    draws = _arr(draws, np.uint64)
    assert draws.size >= f
    s = np.zeros(max(f, 1), np.int64)
    lib().orc_floyd_positions(C.c_int64(d), C.c_int32(f), _p(draws), _p(s))
    return s[:f]


def sample_node(offsets, indices, v, hop, f, rng_seed):
    offsets = _arr(offsets, np.int64)
    indices = _arr(indices, np.int32)
    out = np.zeros(max(f, 1), np.int32)
    n = lib().orc_sample_node(C.c_int64(offsets.size - 1), _p(offsets), _p(indices), C.c_int32(v),
                              C.c_int32(hop), C.c_int32(f), C.c_uint64(rng_seed), _p(out))
    if n < 0:
        raise ValueError("node id out of range")
    return out[:n]


def sample(offsets, indices, seeds, fanouts, rng_seed):
    """Returns a list of (frontier, indptr, flat) per hop."""
    offsets = _arr(offsets, np.int64)
    indices = _arr(indices, np.int32)
    seeds = _arr(seeds, np.int32)
    fan = _arr(fanouts, np.int32)
    K = fan.size
    cap = int(seeds.size)
    fr, ip, fl = [], [], []
    for h in range(K):
        fr.append(np.zeros(max(cap, 1), np.int32))
        ip.append(np.zeros(cap + 1, np.int64))
        cap = cap * max(int(fan[h]), 0)
        fl.append(np.zeros(max(cap, 1), np.int32))
    PP = C.c_void_p * max(K, 1)
    sizes = np.zeros(2 * max(K, 1), np.int64)
    rc = lib().orc_sample(C.c_int64(offsets.size - 1), _p(offsets), _p(indices), _p(seeds),
                          C.c_int64(seeds.size), _p(fan), C.c_int32(K), C.c_uint64(rng_seed),
                          PP(*[a.ctypes.data for a in fr]), PP(*[a.ctypes.data for a in ip]),
                          PP(*[a.ctypes.data for a in fl]), _p(sizes))
    if rc != 0:
        raise ValueError("node id out of range")
    out = []
    for h in range(K):
        nf, nflat = int(sizes[2 * h]), int(sizes[2 * h + 1])
        out.append((fr[h][:nf].copy(), ip[h][:nf + 1].copy(), fl[h][:nflat].copy()))
    return out


def dedup(n_nodes, ids, want_inverse=True):
    ids = _arr(ids, np.int32)
    uniq = np.zeros(max(ids.size, 1), np.int32)
    inv = np.zeros(max(ids.size, 1), np.int32) if want_inverse else None
    u = lib().orc_dedup(C.c_int64(n_nodes), _p(ids), C.c_int64(ids.size), _p(uniq),
                        _p(inv) if want_inverse else None)
    if u < 0:
        raise ValueError("id out of range")
    return uniq[:u].copy(), (inv[:ids.size].copy() if want_inverse else None)


def rank_build(order):
    order = _arr(order, np.int32)
    rank = np.zeros(max(order.size, 1), np.int32)
    rc = lib().orc_rank_build(_p(order), C.c_int64(order.size), _p(rank))
    if rc != 0:
        raise ValueError("order is not a permutation")
    return rank[:order.size]


def lookup(ids, rank, n_hbm, n_host):
    ids = _arr(ids, np.int32)
    rank = _arr(rank, np.int32)
    tier = np.zeros(max(ids.size, 1), np.int8)
    slot = np.zeros(max(ids.size, 1), np.int32)
    lib().orc_lookup(_p(ids), C.c_int64(ids.size), _p(rank), C.c_int64(n_hbm), C.c_int64(n_host),
                     _p(tier), _p(slot))
    return tier[:ids.size], slot[:ids.size]


def gather(ids, rank, n_hbm, n_host, hbm_table, host_table, out):
    """hbm_table/host_table/out: 2-D uint8 arrays [rows, row_bytes]; out is modified in place.
    Returns (miss_pos, miss_id, miss_slot, stats[4])."""
    ids = _arr(ids, np.int32)
    rank = _arr(rank, np.int32)
    assert out.dtype == np.uint8 and out.flags.c_contiguous and out.shape[0] >= ids.size
    row_bytes = out.shape[1]
    for t in (hbm_table, host_table):
        assert t.dtype == np.uint8 and t.flags.c_contiguous and (t.shape[0] == 0 or t.shape[1] == row_bytes)
    mp = np.zeros(max(ids.size, 1), np.int32)
    mi = np.zeros(max(ids.size, 1), np.int32)
    ms = np.zeros(max(ids.size, 1), np.int32)
    stats = np.zeros(4, np.int64)
    lib().orc_gather(_p(ids), C.c_int64(ids.size), _p(rank), C.c_int64(n_hbm), C.c_int64(n_host),
                     C.c_int32(row_bytes), _p(hbm_table), _p(host_table), _p(out), _p(mp), _p(mi),
                     _p(ms), _p(stats))
    n = int(stats[3])
    return mp[:n].copy(), mi[:n].copy(), ms[:n].copy(), stats


def gather_miss(miss_pos, miss_slot, standin_table, out):
    miss_pos = _arr(miss_pos, np.int32)
    miss_slot = _arr(miss_slot, np.int32)
    assert standin_table.dtype == np.uint8 and standin_table.flags.c_contiguous
    lib().orc_gather_miss(_p(miss_pos), _p(miss_slot), C.c_int64(miss_pos.size),
                          C.c_int32(out.shape[1]), _p(standin_table), _p(out))


def hotness_add(unique, counts):
    """counts (int32[N]) is modified in place."""
    unique = _arr(unique, np.int32)
    assert counts.dtype == np.int32 and counts.flags.c_contiguous
    lib().orc_hotness_add(_p(unique), C.c_int64(unique.size), _p(counts))


def hotness_order(counts):
    counts = _arr(counts, np.int32)
    order = np.zeros(max(counts.size, 1), np.int32)
    lib().orc_hotness_order(_p(counts), C.c_int64(counts.size), _p(order))
    return order[:counts.size]


def local_ids(n_nodes, unique, ids):
    unique = _arr(unique, np.int32)
    ids = _arr(ids, np.int32)
    out = np.zeros(max(ids.size, 1), np.int32)
    rc = lib().orc_local_ids(C.c_int64(n_nodes), _p(unique), C.c_int64(unique.size), _p(ids),
                             C.c_int64(ids.size), _p(out))
    if rc != 0:
        raise ValueError("an id is not in the unique list")
    return out[:ids.size]


def num_threads():
    return int(lib().orc_num_threads())


def set_num_threads(n):
    lib().orc_set_num_threads(C.c_int(n))
