"""Why the de-duplication's hash table is not staged through LDS: measurements on a synthetic workload.

    python -m paper_2310_00837_amd.dedup_probe --config 1 [--batches 20]

For the batch ID lists [seeds | flat_0 | ...] of a workload it prints (one JSON line)
  * the share of list entries that repeat an earlier entry at all, and the share that repeat an
    earlier entry of the same tile of 1 Ki / 4 Ki / 16 Ki consecutive entries: only the latter could
    be absorbed by a table that a workgroup keeps in LDS for the entries it handles;
  * the span of every sampling pass with and without the inserts into the batch's table
    (helios_prepare_batch against helios_sample, device clock), i.e. what all those inserts cost.
The table of the cache placement plays no part, so the cache is built with every node a miss.
"""
import argparse
import json
import sys

import numpy as np
import torch

from . import helios, workload as W


def tile_repeat_share(ids: np.ndarray, tile: int) -> float:
    """Share of entries whose value occurred earlier within the same tile of `tile` consecutive entries."""
    n, rep = ids.size, 0
    for t0 in range(0, n, tile):
        part = ids[t0:t0 + tile]
        rep += part.size - np.unique(part).size
    return rep / max(n, 1)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--batches", type=int, default=20)
    ap.add_argument("--seed", type=int, default=1234)
    args = ap.parse_args()
    dev = torch.device("cuda", 0)
    sp = W.spec(args.config)
    g = W.make_graph(sp, args.seed, dev if sp.n_nodes > 5_000_000 else "cpu")
    off, idx, order = g.offsets.to(dev), g.indices.to(dev), g.order.to(dev)
    g.offsets, g.indices, g.order, g.perm_seed = off, idx, order, g.perm_seed.to(dev)
    h = helios.Helios(0)
    h.csr_load(off, idx)
    h.cache_build(order, 0, 0, sp.row_bytes, None, None, None)
    B = sp.batch
    hops = helios.alloc_hops(B, sp.fanouts, dev)
    cap = B + sum(hb.flat.numel() for hb in hops)
    unique = torch.empty(cap, dtype=torch.int32, device=dev)
    inverse = torch.empty(cap, dtype=torch.int32, device=dev)
    out = torch.empty((cap, sp.row_bytes), dtype=torch.uint8, device=dev)
    mp, mi, ms = (torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(3))
    sizes = torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory()
    nu = torch.zeros(1, dtype=torch.int64).pin_memory()
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    h.set_timing(1)
    K = len(sp.fanouts)
    acc = {"any": 0.0, 1024: 0.0, 4096: 0.0, 16384: 0.0}
    span = {"with_batch_table": [0.0] * K, "hop_table_only": [0.0] * K}
    n_cat = 0
    for b in range(args.batches + 2):
        seeds = W.seed_batch(sp, g, b).to(dev)
        rs = W.batch_rng_seed(args.seed, b)
        for mode in ("with_batch_table", "hop_table_only"):
            if mode == "with_batch_table":
                h.prepare_batch(seeds, sp.fanouts, rs, hops, sizes, unique, inverse, nu, out, mp, mi, ms, stats)
            else:
                h.sample(seeds, sp.fanouts, rs, hops, sizes)
            h.sync()
            roles, per_us = h.batch_ticks()
            if b >= 2:
                for kind, stage, _, a, z in roles:
                    if kind == helios.ROLE_SAMPLE and z > a:
                        span[mode][stage] += (z - a) / per_us / args.batches
        if b < 2:
            continue
        cat = np.concatenate([seeds.cpu().numpy()] + [hops[k].flat[:int(sizes[2 * k + 1])].cpu().numpy() for k in range(K)])
        n_cat += cat.size
        acc["any"] += (cat.size - np.unique(cat).size) / cat.size / args.batches
        for t in (1024, 4096, 16384):
            acc[t] += tile_repeat_share(cat, t) / args.batches
    h.close()
    print(json.dumps({"workload": f"configs[{args.config}] {sp.name}", "batches": args.batches,
                      "list_entries_per_batch": n_cat / args.batches,
                      "share_repeating_an_earlier_entry": acc["any"],
                      "share_repeating_within_a_tile_of": {"1024": acc[1024], "4096": acc[4096], "16384": acc[16384]},
                      "sampling_pass_span_us_by_hop": span}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
