"""Pins for the oracle's rollout theory (Sec. 3, App. A1) against what the paper
prints and proves."""
import random

import pytest

from oracle import theory as th
import workloads as W


def sr_net():
    # Fig. 1: I -> H1 -> H2 -> O, skip H1 -> O, self-recurrent H1 -> H1
    return 4, [(0, 1), (1, 2), (2, 3), (1, 3), (1, 1)]


def three_cycle():
    # input-fed 3-cycle (second network of Fig. 2): in -> a -> b -> c -> a
    return 4, [(0, 1), (1, 2), (2, 3), (3, 1)]


def acyclic_r0(n, edges, R):
    """Independent validity test: the sub-graph of non-bridging edges has no cycle (DFS colouring)."""
    adj = {v: [] for v in range(n)}
    for (s, t), r in zip(edges, R):
        if r == 0:
            adj[s].append(t)
    colour = [0] * n

    def dfs(v):
        colour[v] = 1
        for t in adj[v]:
            if colour[t] == 1 or (colour[t] == 0 and not dfs(t)):
                return False
        colour[v] = 2
        return True

    return all(colour[v] != 0 or dfs(v) for v in range(n))


def random_network(rng, n_max=6):
    while True:
        n = rng.randint(2, n_max)
        m = rng.randint(1, 2 * n)
        edges = list({(rng.randrange(n), rng.randrange(n)) for _ in range(m)})
        try:
            th.check_network(n, edges)
        except th.GraphError:
            continue
        return n, edges


def test_printed_inference_factors_sr_net():
    # Sec. 4: F(R^seq) = 3 and F(R^str) = 1 for the skip+recurrent net
    n, e = sr_net()
    assert th.inference_factor(n, e, [0, 0, 0, 0, 1]) == 3
    assert th.inference_factor(n, e, [1, 1, 1, 1, 1]) == 1
    # streaming responds one update step earlier: shortest path I-H1-O (2) vs longest (3)
    assert th.shortest_path_length(n, e, 3) == 2
    assert th.levels(n, e, [0, 0, 0, 0, 1])[3] == 3


def test_three_most_sequential_patterns_of_the_3_cycle():
    # Fig. 2 caption: either of the three cycle edges could be unrolled -> 3 patterns
    n, e = three_cycle()
    valid = th.all_valid_patterns(n, e)
    most_zeros = max(R.count(0) for R in valid)
    best = [R for R in valid if R.count(0) == most_zeros]
    assert most_zeros == 3 and len(best) == 3
    assert all(R[0] == 0 and sum(R[1:]) == 1 for R in best)


def test_all_zero_pattern_invalid_with_cycles_and_self_edge_must_bridge():
    n, e = three_cycle()
    assert not th.is_valid(n, e, [0, 0, 0, 0])
    n, e = sr_net()
    assert not th.is_valid(n, e, [1, 1, 1, 1, 0])
    assert th.is_valid(n, e, [0, 0, 0, 0, 1])
    with pytest.raises(th.RolloutError):
        th.check_rollout(n, e, [0, 0, 0, 0, 0])


def test_streaming_always_valid_and_validity_is_window_independent():
    rng = random.Random(1)
    for _ in range(40):
        n, e = random_network(rng)
        assert th.is_valid(n, e, [1] * len(e), 1)
        R = [rng.randint(0, 1) for _ in e]
        v1 = th.is_valid(n, e, R, 1)
        assert v1 == th.is_valid(n, e, R, 3)
        assert v1 == acyclic_r0(n, e, R)


def test_lemma1_bounds_sr_net_count_is_16():
    n, e = sr_net()
    lo_fwd, lo_cyc, hi = th.lemma1_bounds(n, e)
    assert (lo_fwd, hi) == (16, 16)
    assert len(th.all_valid_patterns(n, e)) == 16
    assert lo_cyc == 1      # a self-edge gives 2^1 - 1 = 1


def test_lemma1_bounds_random():
    rng = random.Random(7)
    for _ in range(25):
        n, e = random_network(rng, 5)
        if len(e) > 9:
            continue
        count = len(th.all_valid_patterns(n, e))
        lo_fwd, lo_cyc, hi = th.lemma1_bounds(n, e)
        assert 1 <= lo_fwd <= count <= hi
        assert 1 <= lo_cyc <= count


def test_lemma1_3cycle():
    n, e = three_cycle()
    lo_fwd, lo_cyc, hi = th.lemma1_bounds(n, e)
    assert lo_fwd == 2 and lo_cyc == 7 and hi == 16
    assert len(th.all_valid_patterns(n, e)) == 14      # 2 * (2^3 - 1)


def test_tableau_two_definitions_agree():
    rng = random.Random(3)
    checked = 0
    for _ in range(60):
        n, e = random_network(rng)
        R = [rng.randint(0, 1) for _ in e]
        if not th.is_valid(n, e, R):
            continue
        for Wd in (1, 2, 4):
            assert th.tableau_longest_path(n, e, R, Wd) == th.tableau_update_steps(n, e, R, Wd)
        checked += 1
    assert checked > 15


def test_theorem1_equivalences():
    rng = random.Random(11)
    seen_true = seen_false = 0
    for _ in range(80):
        n, e = random_network(rng, 5)
        if len(e) > 8:
            continue
        valid = th.all_valid_patterns(n, e)
        Wd = 3
        tabs = {R: th.tableau_longest_path(n, e, R, Wd) for R in valid}
        tmin = [[min(tabs[R][i][v] for R in valid) for v in range(n)] for i in range(Wd + 1)]
        stream = tuple([1] * len(e))
        for R in valid:
            a = th.equally_model_parallel(n, e, R, stream)
            b = th.inference_factor(n, e, R) == 1
            c = all(tabs[R][i][v] <= i for i in range(Wd + 1) for v in range(n))
            d = tabs[R] == tmin
            assert a == b == c == d, (n, e, R, a, b, c, d)
            seen_true += a
            seen_false += (not a)
    assert seen_true > 10 and seen_false > 10


def test_window_edge_count_is_W_times_E():
    # Sec. 3: a window of size W holds W*|E| edges that are used for updates
    n, e = sr_net()
    for R in ([1] * 5, [0, 0, 0, 0, 1], [1, 0, 1, 0, 1]):
        for Wd in (1, 2, 5):
            used = [x for x in th.window_edges(n, e, R, Wd) if x[1][0] != 0]
            assert len(used) == Wd * len(e)


def test_rejections():
    with pytest.raises(th.GraphError):
        th.check_network(4, [(0, 1), (1, 3), (3, 2), (2, 0)])      # Fig. A1: cycle without input
    with pytest.raises(th.GraphError):
        th.check_network(3, [])
    with pytest.raises(th.GraphError):
        th.check_network(3, [(0, 1), (2, 2)])                      # node 2 only feeds itself
    with pytest.raises(th.GraphError):
        th.check_network(2, [(0, 5)])
    th.check_network(5, [(4, 0), (4, 2), (0, 1), (1, 3), (3, 2), (2, 0)])   # Fig. A1, last example


def test_dsr_family_path_lengths():
    # App. A2: shortest path always 4; the longest grows by one per network from 4;
    # Sec. 4: DSR2 has shortest 4 and longest 6 -> streaming answers 2 steps earlier
    for k in range(7):
        g = W.dsr_net(k)
        n = len(g.nodes)
        e = [(x.src, x.dst) for x in g.edges]
        seq = W.sequential_pattern(g)
        assert th.is_valid(n, e, seq)
        assert th.shortest_path_length(n, e, g.out_node) == 4
        assert th.inference_factor(n, e, seq) == 4 + k
        assert th.levels(n, e, seq)[g.out_node] == 4 + k
        assert th.inference_factor(n, e, W.streaming_pattern(g)) == 1
    g = W.dsr_net(2)
    e = [(x.src, x.dst) for x in g.edges]
    assert th.inference_factor(len(g.nodes), e, W.sequential_pattern(g)) - \
        th.shortest_path_length(len(g.nodes), e, g.out_node) == 2


def test_benchmark_graphs_are_networks_with_expected_factors():
    for name, f in W.BENCH_CONFIGS.items():
        g = f()
        n = len(g.nodes)
        e = [(x.src, x.dst) for x in g.edges]
        th.check_network(n, e)
        assert th.inference_factor(n, e, W.streaming_pattern(g)) == 1
        assert th.is_valid(n, e, W.sequential_pattern(g))
        assert th.is_valid(n, e, W.hybrid_pattern(g))
    g = W.cifar_sr()
    e = [(x.src, x.dst) for x in g.edges]
    assert th.inference_factor(len(g.nodes), e, W.sequential_pattern(g)) == 7
    assert len(W.tiny_sr().edges) == 6 and len(g.edges) == 14
    assert len(W.gtsrb_sr().edges) == 32 and len(W.hires_sr().edges) == 35
