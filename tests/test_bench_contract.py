"""Host-side checks of bench.py that need no GPU: the one-GPU rule, the byte accounting behind the
roofline fraction, and the bookkeeping of measured traffic."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from synth import workloads as wl  # noqa: E402
from synth.layout import COPY, SUM, FORWARD_ONLY, NO_FORWARD  # noqa: E402


@pytest.mark.parametrize("argv,env", [(["--gpus", "2"], {}), ([], {"WORLD_SIZE": "4"})])
def test_more_than_one_gpu_is_refused_with_a_message(argv, env):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + argv, capture_output=True, text=True,
                       env={**os.environ, **env}, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_byte_model_of_a_call_matches_the_workload_generator():
    """bench.call_stats re-derives unique chunks, payload and algorithmic bytes from a record list;
    the generator computes them from the logical stream.  Both follow the single-pass model:
    reduce+forward 4 C, reduce 3 C, copy+forward 3 C, copy 2 C, relay 3 C, 36 B per arrival."""
    for relay in (False, True):
        w = wl.config2(seed=3, M=8 << 20, relay=relay)
        for ph in w.phases:
            assert bench.call_stats(ph.descs, ph.op) == (ph.n_unique, ph.payload_bytes, ph.algo_bytes), (relay, ph.name)
    w = wl.config3(seed=3, M=16 << 20)
    assert bench.call_stats(w.phases[0].descs, SUM) == (w.phases[0].n_unique, w.phases[0].payload_bytes, w.phases[0].algo_bytes)
    w = wl.config4(seed=3)
    ph = w.phases[0]
    assert bench.call_stats(ph.descs, COPY) == (ph.n_unique, ph.payload_bytes, ph.algo_bytes)


def test_byte_model_by_hand():
    from synth.layout import DESC
    C = 4096
    d = np.zeros(5, dtype=DESC)
    d["len"] = C
    d["seq"] = [0, 1, 1, 2, 3]                                   # one duplicate arrival
    d["out_off"] = [0, C, C, NO_FORWARD, np.uint64(2 * C) | FORWARD_ONLY]
    # SUM: seq 0 and 1 reduce + forward (4 C each), seq 2 reduce only (3 C), seq 3 relay (3 C), duplicate 0
    assert bench.call_stats(d, SUM) == (4, 4 * C, (4 + 4 + 3 + 3) * C + 36 * 5)
    # COPY: copy + forward 3 C, copy only 2 C, relayed copy 2 C
    assert bench.call_stats(d, COPY) == (4, 4 * C, (3 + 3 + 2 + 2) * C + 36 * 5)


def test_measured_traffic_is_keyed_by_the_kernel_source():
    h = bench.source_hash()
    assert len(h) == 16
    for (workload, key), nbytes in bench.MEASURED_TRAFFIC.items():
        assert workload in bench.WORKLOADS and len(key) == 16 and nbytes > 0
    # a figure measured on another source must not be reported for this one
    assert bench.MEASURED_TRAFFIC.get(("config2", "0" * 16)) is None


def test_bench_is_one_program():
    """Every top-level name of bench.py is defined once (a second definition would silently
    shadow the first, and an edit to the shadowed copy would do nothing) and every top-level
    function is reachable from main()."""
    import ast
    import collections
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    defs = [n for n in tree.body if isinstance(n, (ast.FunctionDef, ast.ClassDef))]
    twice = [name for name, k in collections.Counter(n.name for n in defs).items() if k > 1]
    assert not twice, f"defined more than once: {twice}"
    assigned = collections.Counter(t.id for n in tree.body if isinstance(n, ast.Assign)
                                   for t in n.targets if isinstance(t, ast.Name))
    assert not [k for k, v in assigned.items() if v > 1]
    used = {n.id for n in ast.walk(tree) if isinstance(n, ast.Name)} | \
           {n.attr for n in ast.walk(tree) if isinstance(n, ast.Attribute)}
    unused = [n.name for n in defs if n.name not in used]
    assert not unused, f"never referenced: {unused}"
    assert len(src.splitlines()) < 950
