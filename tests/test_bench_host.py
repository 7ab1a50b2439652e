"""Host-side logic of bench.py that needs no GPU: the one-GPU rule, the static shapes it offers, the table behind its
labelled projection."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_static_shapes_offered_by_the_bench_are_valid_trees():
    import bench
    from oracle.static_tree import StaticShape
    import workload as wl
    for name, nodes, depth in (("chain5", 6, 5), ("chain1", 2, 1), ("tree26", 26, 5)):
        parent, rank = bench.static_shape(name)
        st = StaticShape(np.asarray(parent), np.asarray(rank))          # validates order, ranks and widths
        assert len(parent) == nodes and nodes <= wl.LLAMA2_7B.tree_total
        d = [0] * nodes
        for i in range(1, nodes):
            d[i] = d[parent[i]] + 1
        assert max(d) == depth and depth <= wl.LLAMA2_7B.tree_depth


def test_projection_table_covers_the_benchmark_shapes_with_the_papers_range():
    import bench
    import workload as wl
    for sh in wl.CONFIGS[1:]:
        for t in (0, 1):
            tau = bench.PAPER_TAU[(sh.name, t)]
            assert 4.0 < tau < 6.0                                      # Table 1's HASS rows
        assert bench.PAPER_TAU[(sh.name, 0)] > bench.PAPER_TAU[(sh.name, 1)]
