"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the measured-traffic table it quotes."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_traffic_table_covers_the_reported_kernel_of_both_profiled_workloads():
    bench = _bench_module()
    for workload in ("large_sage", "large_gcn_bf16"):
        t, current = bench.measured_traffic(workload, "agg_fwd")
        assert t is not None and t > 1e8, workload
        assert current in (True, False)              # whether the counters were collected on this tree's kernel sources
    assert bench.measured_traffic("large_sage", "no_such_kernel") == (None, None)


def test_kernel_sources_hash_follows_the_sources(tmp_path, monkeypatch):
    from paper_2406_17611_amd import profile_summary as ps
    h = ps.kernel_sources_hash()
    assert len(h) == 64 and h == ps.kernel_sources_hash()
    import shutil
    pkg = tmp_path / "pkg"
    shutil.copytree(os.path.join(ROOT, "paper_2406_17611_amd", "csrc"), pkg / "csrc")
    os.makedirs(tmp_path / "include")
    shutil.copy(os.path.join(ROOT, "include", "varco.h"), tmp_path / "include" / "varco.h")
    monkeypatch.setattr(ps, "HERE", str(pkg))
    monkeypatch.setattr(ps, "ROOT", str(tmp_path))
    assert ps.kernel_sources_hash() == h
    with open(pkg / "csrc" / "elem.h", "a") as f:
        f.write("// changed\n")
    assert ps.kernel_sources_hash() != h


def test_source_row_reuse_counts_match_a_direct_count():
    """The reuse count's totals against a plain loop over one partition's rows of the smallest workload."""
    import numpy as np
    from paper_2406_17611_amd import source_row_reuse, synth

    w = synth.make_workload("tiny")
    width, ratio, p = 16, 4, 0
    g, part = w.graph, np.asarray(w.part)
    per_entry, entries, local_entries = 0, 0, 0
    seen = {}
    for i in np.nonzero(part == p)[0]:
        for c in g.colidx[g.rowptr[i]:g.rowptr[i + 1]]:
            b = (width if part[c] == p else width // ratio) * 4
            per_entry += b
            entries += 1
            local_entries += int(part[c] == p)
            seen[int(c)] = b
    c = source_row_reuse.reuse_counts(w, p, width, ratio, 4)
    assert (c["entries"], c["local_entries"]) == (entries, local_entries) and entries > 0
    assert c["per_entry_bytes"] == per_entry and c["per_row_bytes"] == sum(seen.values())
    assert len(c["refs"]) == len(seen) and int(c["refs"].sum()) == entries
    lines = source_row_reuse.reuse_table(w, p, width, ratio, 4)
    assert f"distinct source rows {len(seen)} " in lines[1]
    shares = [float(l.split()[-1]) for l in lines[6:]]
    assert shares == sorted(shares) and all(0.0 <= s <= 1.0 for s in shares)
