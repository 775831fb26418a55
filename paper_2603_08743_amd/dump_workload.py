"""Write the tables of one benchmark workload to a binary file for ``zp_prof_driver``.

    python -m paper_2603_08743_amd.dump_workload --config 2 --out /tmp/cfg2.tables [--batch B] [--compress-frac F]

The file holds the shape, the seed, block tables, block counts, query slots, per-head keep counts and, for the
prefix-sharing workload, the target tables the host planner produces.  The driver regenerates the pool values from the
seed with the same integer hash as ``workloads.py``, so counter runs see the input ``bench.py`` times.  No GPU needed.
"""
from __future__ import annotations

import argparse

import numpy as np

from . import binding, workloads

MAGIC = 0x5A505754


def dump(cfg: int, path: str, batch=None, compress_frac: float = 1.0) -> None:
    if cfg == 3:
        w = workloads.config(3, B=batch, compress_frac=compress_frac)
    elif batch is None:
        w = workloads.config(cfg)
    else:
        N_max = workloads.config(cfg, B=1, L=1, N_total=2048).N_max
        w = workloads.config(cfg, B=batch, N_total=batch * N_max + 64)
    assert w.dtype == "bf16", "the driver handles bf16 pools"
    dst = None
    if cfg == 3:
        dst = binding.zp_plan(w.block_table, w.num_blocks, w.N_max, w.refcnt.copy(), w.free_list)["dst_table"]
    head = np.array([MAGIC, cfg, w.seed, w.B, w.max_blocks, w.N_max, w.L, w.h_kv, w.h_q, w.d, w.b, w.w, w.N_total, w.M,
                     int(w.keep is not None), int(dst is not None)], dtype=np.int32)
    with open(path, "wb") as f:
        f.write(head.tobytes())
        for a in (w.block_table, w.num_blocks, w.q_slot, w.keep, dst):
            if a is not None:
                f.write(np.ascontiguousarray(a, dtype=np.int32).tobytes())
    print("%s: %s B=%d L=%d N_total=%d" % (path, w.name, w.B, w.L, w.N_total))


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--out", required=True)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--compress-frac", type=float, default=1.0)
    a = ap.parse_args()
    dump(a.config, a.out, a.batch, a.compress_frac)
