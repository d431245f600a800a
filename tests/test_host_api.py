"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host-only logic (network / rollout validation, tableau levels, inference factor, pattern count)
agrees with the oracle.  No compute call is made; nothing here needs a GPU."""
import ctypes
import os
import random
import re

import pytest

import paper_1806_04965_amd as sr
from paper_1806_04965_amd import binding
from oracle import theory as th
import workloads as W
from workloads.graphs import Edge

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "sr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sr_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sr.load_library()
    names = header_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def edges_of(pairs, bits=None):
    bits = bits or [1] * len(pairs)
    return [Edge(s, t, "conv", 3, 3, 1, 1, 1, b) for (s, t), b in zip(pairs, bits)]


def test_analyze_matches_printed_factors():
    pairs = [(0, 1), (1, 2), (2, 3), (1, 3), (1, 1)]          # skip+recurrent example net
    assert sr.analyze(4, edges_of(pairs, [0, 0, 0, 0, 1])) == ([0, 1, 2, 3], 3)
    assert sr.analyze(4, edges_of(pairs))[1] == 1
    assert sr.count_valid_patterns(4, edges_of(pairs)) == 16
    assert sr.count_valid_patterns(4, edges_of([(0, 1), (1, 2), (2, 3), (3, 1)])) == 14


def test_analyze_agrees_with_oracle_on_random_graphs():
    rng = random.Random(5)
    checked = 0
    for _ in range(200):
        n = rng.randint(2, 7)
        pairs = list({(rng.randrange(n), rng.randrange(n)) for _ in range(rng.randint(1, 2 * n))})
        R = [rng.randint(0, 1) for _ in pairs]
        try:
            th.check_network(n, pairs)
            net_ok = True
        except th.GraphError:
            net_ok = False
        if not net_ok:
            with pytest.raises(sr.SrError) as ei:
                sr.analyze(n, edges_of(pairs, R))
            assert ei.value.name == "SR_ERR_GRAPH"
            continue
        if not th.is_valid(n, pairs, R):
            with pytest.raises(sr.SrError) as ei:
                sr.analyze(n, edges_of(pairs, R))
            assert ei.value.name == "SR_ERR_ROLLOUT"
            continue
        lv, f = sr.analyze(n, edges_of(pairs, R))
        assert lv == th.levels(n, pairs, R) and f == th.inference_factor(n, pairs, R)
        if len(pairs) <= 8:
            assert sr.count_valid_patterns(n, edges_of(pairs)) == len(th.all_valid_patterns(n, pairs))
        checked += 1
    assert checked > 30


def test_tableau_bounds_and_model_parallel_classes_match_paper_and_oracle():
    # skip+recurrent example net (Sec. 4): sequential tableau of the size-1 window is 0,1,2,3;
    # Lemma 1: 16 = 2^4 = 2^(5-1) patterns.  3-cycle fed by an input: bounds 2, 7 and 16 around 14.
    pairs = [(0, 1), (1, 2), (2, 3), (1, 3), (1, 1)]
    assert sr.tableau(4, edges_of(pairs, [0, 0, 0, 0, 1]), 1) == [[0, 0, 0, 0], [0, 1, 2, 3]]
    assert sr.tableau(4, edges_of(pairs), 3) == [[0, 0, 0, 0], [0, 1, 1, 1], [0, 2, 2, 2], [0, 3, 3, 3]]
    assert sr.pattern_count_bounds(4, edges_of(pairs)) == (16, 1, 16)
    assert sr.pattern_count_bounds(4, edges_of([(0, 1), (1, 2), (2, 3), (3, 1)])) == (2, 7, 16)
    seq, stream = [0, 0, 0, 0, 1], [1, 1, 1, 1, 1]
    assert not sr.equally_model_parallel(4, edges_of(pairs), seq, stream)
    assert sr.equally_model_parallel(4, edges_of(pairs), [0, 1, 1, 1, 1], stream)   # differs on the input edge only
    rng = random.Random(9)
    checked = 0
    for _ in range(150):
        n = rng.randint(2, 6)
        pairs = list({(rng.randrange(n), rng.randrange(n)) for _ in range(rng.randint(1, 2 * n))})
        try:
            th.check_network(n, pairs)
        except th.GraphError:
            continue
        R = [rng.randint(0, 1) for _ in pairs]
        R2 = [rng.randint(0, 1) for _ in pairs]
        assert sr.equally_model_parallel(n, edges_of(pairs), R, R2) == th.equally_model_parallel(n, pairs, R, R2)
        lo_f, lo_c, up = sr.pattern_count_bounds(n, edges_of(pairs))
        assert (lo_f, lo_c, up) == th.lemma1_bounds(n, pairs)
        if len(pairs) <= 8:
            cnt = sr.count_valid_patterns(n, edges_of(pairs))
            assert lo_f <= cnt <= up and lo_c <= cnt
        if th.is_valid(n, pairs, R):
            W_ = rng.randint(1, 4)
            t = sr.tableau(n, edges_of(pairs, R), W_)
            assert t == th.tableau_longest_path(n, pairs, R, W_) == th.tableau_update_steps(n, pairs, R, W_)
            checked += 1
    assert checked > 20


def test_analysis_calls_report_errors_as_status_codes():
    pairs = [(0, 1), (1, 2), (2, 1)]
    ok = edges_of(pairs)
    for bad, name in ((lambda: sr.tableau(3, ok, 0), "SR_ERR_ARG"),                       # W < 1
                      (lambda: sr.tableau(3, edges_of(pairs, [1, 0, 0]), 2), "SR_ERR_ROLLOUT"),   # R=0 cycle
                      (lambda: sr.tableau(3, edges_of([(1, 2), (2, 1)]), 1), "SR_ERR_GRAPH"),     # no input node
                      (lambda: sr.equally_model_parallel(3, ok, [1, 1, 2], [1, 1, 1]), "SR_ERR_ARG"),
                      (lambda: sr.pattern_count_bounds(3, edges_of([(0, 5)])), "SR_ERR_GRAPH"),
                      (lambda: sr.pattern_count_bounds(26, edges_of([(i, i + 1) for i in range(25)])), "SR_ERR_ARG")):
        with pytest.raises(sr.SrError) as ei:
            bad()
        assert ei.value.name == name
    # invalid patterns may still be compared for model-parallel equality
    assert sr.equally_model_parallel(3, ok, [1, 0, 0], [0, 0, 0])


def test_benchmark_graph_levels():
    for name, f in W.BENCH_CONFIGS.items():
        g = f()
        for bits in (W.streaming_pattern(g), W.sequential_pattern(g), W.hybrid_pattern(g)):
            gg = g.with_pattern(bits)
            pairs = [(e.src, e.dst) for e in gg.edges]
            lv, fac = sr.analyze(len(gg.nodes), gg.edges)
            assert lv == th.levels(len(gg.nodes), pairs, bits) and fac == th.inference_factor(len(gg.nodes), pairs, bits)


def create(nodes, edges, batch=1, dtype=0):
    lib = sr.load_library()
    na = (binding.NodeDesc * len(nodes))(*[binding.NodeDesc(*n) for n in nodes])
    h = ctypes.c_void_p()
    st = lib.sr_graph_create(na, len(nodes), binding._edge_array(edges), len(edges), batch, dtype, None, ctypes.byref(h))
    name = lib.sr_status_str(st).decode()
    if st == 0:
        lib.sr_graph_destroy(h)
    return name


def test_create_rejects_bad_graphs_before_touching_a_device():
    n3 = [(4, 8, 8, 0), (4, 8, 8, 1), (4, 8, 8, 1)]
    assert create(n3, []) == "SR_ERR_GRAPH"
    assert create(n3, edges_of([(0, 1), (2, 2)])) == "SR_ERR_GRAPH"                    # node 2 only feeds itself
    assert create([(4, 8, 8, 1)] * 4, edges_of([(0, 1), (1, 3), (3, 2), (2, 0)])) == "SR_ERR_GRAPH"   # cycle, no input
    assert create(n3, edges_of([(0, 1), (1, 2), (1, 1)], [1, 1, 0])) == "SR_ERR_ROLLOUT"   # self-edge must bridge
    assert create(n3, edges_of([(0, 1), (1, 2), (2, 1)], [0, 0, 0])) == "SR_ERR_ROLLOUT"
    assert create(n3, [Edge(0, 1), Edge(1, 2, stride=2)]) == "SR_ERR_SHAPE"
    assert create(n3, [Edge(0, 1), Edge(1, 2, bridge=2)]) == "SR_ERR_ARG"
    assert create(n3, edges_of([(0, 1), (1, 2)]), batch=0) == "SR_ERR_ARG"
    assert create([(4, 8, 8, 7)] * 3, edges_of([(0, 1), (1, 2)])) == "SR_ERR_ARG"
    lib = sr.load_library()
    assert lib.sr_graph_create(None, 0, None, 0, 1, 0, None, None) == 1
    assert b"SR_ERR_SHAPE" == lib.sr_status_str(4)


def test_null_handles_are_errors_not_crashes():
    lib = sr.load_library()
    assert lib.sr_reset(None, None) == 1
    assert lib.sr_frame_step(None, None) == 1
    assert lib.sr_rollout(None, None, 1, 0, None) == 1
    assert lib.sr_get_state(None, 0, None, 0) == 1
    assert lib.sr_graph_info(None, None, None, None) == 1
    assert lib.sr_graph_tile_kernel(None, None) == 1
    assert lib.sr_graph_node_kernels(None, None) == 1
    assert lib.sr_graph_health(None, None, None) == 1
    assert lib.sr_graph_traffic_model(None, None) == 1
    assert lib.sr_frame_step_static(None, None) == 1
    assert lib.sr_window_gradients(None, 1, None, None, None, 0, None, None, None) == 1
    assert lib.sr_rmsprop_step(None, 1e-3, 0.9, 1e-7, None, None) == 1
    assert lib.sr_graph_get_weights(None, 0, None, 0) == 1
    assert lib.sr_graph_get_bias(None, 0, None, 0) == 1
    lib.sr_graph_destroy(None)


def test_bench_rejects_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
