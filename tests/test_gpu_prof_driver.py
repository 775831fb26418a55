"""The stand-alone counter driver must measure the kernel on the input bench.py times: its on-device fill is pinned to
workloads.py bit for bit, and its run of zp_compress must succeed on a reduced batch of the default workload."""
import os
import subprocess

import numpy as np
import pytest
import torch

from paper_2603_08743_amd import dump_workload, workloads
from paper_2603_08743_amd.workloads import to_host_bits

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "paper_2603_08743_amd", "zp_prof_driver")


@pytest.mark.parametrize("cfg", [2, 1])
def test_driver_pools_equal_the_workload_generator(cfg, tmp_path):
    assert os.path.exists(DRIVER), "zp_prof_driver not built: run `python -m paper_2603_08743_amd.build`"
    tables, sample = str(tmp_path / "t.tables"), str(tmp_path / "sample.bin")
    dump_workload.dump(cfg, tables, batch=2)
    r = subprocess.run([DRIVER, tables, "1", "1", "0", "0", "1", sample], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "zp_compress" in r.stdout
    N_max = workloads.config(cfg, B=1, L=1, N_total=2048).N_max
    w = workloads.config(cfg, B=2, N_total=2 * N_max + 64)
    K, V, Q = w.pools("cuda", 0, 1)
    got = np.fromfile(sample, dtype=np.uint16)
    off = 0
    for name, t in (("K", K), ("V", V), ("Q", Q)):
        n = min(t.numel(), 1 << 20)
        want = to_host_bits(t).reshape(-1)[:n]
        assert np.array_equal(got[off:off + n], want), "%s differs from workloads.py" % name
        off += n
    assert off == got.size
