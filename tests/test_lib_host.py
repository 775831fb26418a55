"""CPU-side checks of the C-ABI library: it loads, exports what include/zp.h declares, fails loudly
without a GPU, and its host planner agrees with the oracle's independent one."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import oracle
from paper_2603_08743_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "zp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the no-GPU failure mode")
def test_fails_loudly_without_a_gpu():
    lib = binding.load_library()
    h = ctypes.c_void_p()
    assert lib.zp_create(ctypes.byref(h)) == binding.ZP_EHIP and not h.value
    assert b"zp_create" in lib.zp_last_error(None)
    with pytest.raises(RuntimeError):
        binding.Context()


def test_package_has_no_cpu_fallback():
    # the product never reaches for the oracle
    pkg = os.path.join(ROOT, "paper_2603_08743_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "zp_oracle" not in text, f


def random_plan_case(seed):
    rng = np.random.default_rng(seed)
    N_max, N_total, B = int(rng.integers(2, 7)), 400, int(rng.integers(1, 9))
    perm = rng.permutation(N_total)
    n_prefix = int(rng.integers(0, 8))
    prefix, pos = perm[:n_prefix], n_prefix
    refcnt = np.zeros(N_total, dtype=np.int32)
    rows, nbs = [], []
    width = N_max + 8
    for n in range(B):
        N = int(rng.integers(N_max, N_max + 6))
        share = min(int(rng.integers(0, n_prefix + 1)), N - 1) if rng.random() < 0.6 else 0
        row = list(prefix[:share]) + list(perm[pos:pos + N - share])
        pos += N - share
        refcnt[row] += 1
        rows.append(row + [-1] * (width - N))
        nbs.append(N)
    if rng.random() < 0.5 and n_prefix:
        refcnt[prefix] += 1
    free = perm[pos:pos + int(rng.integers(0, 40))]
    return np.array(rows, dtype=np.int32), np.array(nbs, dtype=np.int32), N_max, refcnt, free.astype(np.int32)


@pytest.mark.parametrize("seed", range(40))
def test_planner_matches_oracle(seed):
    tbl, nb, N_max, refcnt, free = random_plan_case(seed)
    mine = refcnt.copy()
    try:
        want = oracle.plan(tbl, nb, N_max, refcnt, free)
    except MemoryError:
        with pytest.raises(binding.ZpError) as e:
            binding.zp_plan(tbl, nb, N_max, mine, free)
        assert e.value.status == binding.ZP_ENOMEM and np.array_equal(mine, refcnt)   # nothing modified
        return
    got = binding.zp_plan(tbl, nb, N_max, mine, free)
    assert np.array_equal(got["dst_table"], want["dst_table"]) and np.array_equal(got["new_table"], want["new_table"])
    assert np.array_equal(got["freed"], want["freed"]) and got["n_free_used"] == want["n_free_used"]
    assert np.array_equal(mine, want["refcnt"])


def test_planner_rejects_bad_input_without_side_effects():
    refcnt = np.array([1, 1, 1, 1, 0, 0], dtype=np.int32)
    before = refcnt.copy()
    for tbl, nb in [([[0, 1, 2, 9]], [4]), ([[0, 1, 2, 3]], [3]), ([[0, 1, 2, 4]], [4]), ([[0, 1, 1, 3]], [4])]:
        with pytest.raises(binding.ZpError) as e:
            binding.zp_plan(np.array(tbl, dtype=np.int32), np.array(nb, dtype=np.int32), 4, refcnt, np.array([5], dtype=np.int32))
        assert e.value.status == binding.ZP_EINVAL and np.array_equal(refcnt, before)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_traffic_figure_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    """bench.py quotes the profiled HBM traffic only while the kernel sources hash to what the profile was taken on."""
    import json
    import bench
    from paper_2603_08743_amd import profile_summary
    sha = profile_summary.source_sha()
    entry = dict(name="x", config=2, B=256, slab_layers=8, traffic_bytes=123.0, source_sha=sha, summary="profiles/x.md", date="d", head="h")
    f = tmp_path / "traffic.json"
    monkeypatch.setattr(profile_summary, "TRAFFIC_JSON", str(f))
    f.write_text(json.dumps([entry]))
    value, src = bench.profiled_traffic(2, 256, 8)
    assert value == 123.0 and src["kernel_sources_unchanged"] is True
    assert bench.profiled_traffic(2, 128, 8) == (None, None)                 # another launch shape: nothing to quote
    f.write_text(json.dumps([dict(entry, source_sha="0" * 16)]))            # profile taken on other sources
    value, src = bench.profiled_traffic(2, 256, 8)
    assert value is None and src["kernel_sources_unchanged"] is False
    f.unlink()
    assert bench.profiled_traffic(2, 256, 8) == (None, None)


def test_committed_traffic_profiles_match_the_committed_kernel_sources():
    """The figures under profiles/ are the ones of the sources in the tree (a kernel change without a new profile fails here)."""
    import json
    from paper_2603_08743_amd import profile_summary
    entries = json.load(open(profile_summary.TRAFFIC_JSON))
    assert entries, "profiles/traffic.json is empty"
    sha = profile_summary.source_sha()
    stale = [e["name"] for e in entries if e["source_sha"] != sha]
    assert not stale, "profiles taken on other kernel sources: %s" % stale
