"""Routing decision (host only, no GPU): the library against the plain-Python oracle, and the oracle against what
the paper fixes (section 3 score, section 5 algorithm, appendix discretisation, and the regime it reports)."""
import numpy as np
import pytest

import paper_2603_13358_amd as ppd
from oracle import routing

# nine workload types as input/output ratios: four decode-heavy, two balanced, three prefill-heavy; the two
# examples the paper gives are 32/512 and 1024/32
CENTERS = [32 / 512, 64 / 512, 64 / 256, 128 / 256, 1.0, 2.0, 512 / 64, 1024 / 64, 1024 / 32]


def _pins(routing):
    """What the paper fixes about the decision (and, where marked, the reading taken of what it leaves open)."""
    # turn 1 always uses the prefill-node path, whatever the table says
    assert routing.decide([1] * 270, CENTERS, 1, 100, 100, 0, 4.0) == 0
    # the regime the paper reports for the prefill-heavy slice: 94-96 % TTFT reduction at 7-12 % TPOT degradation
    for dt in (0.94, 0.96):
        for dp in (0.07, 0.12):
            assert routing.score(1.0, 1.0, dt, dp) > 0                       # equal weights: run locally
            flip = dt / dp                                                    # weight ratio where the sign turns
            assert routing.score(1.0, flip * 1.01, dt, dp) < 0 < routing.score(1.0, flip * 0.99, dt, dp)
    # traditional PD is the special case of a table of zeros
    assert routing.decide([0] * 270, CENTERS, 3, 1024, 32, 5000, 8.0) == 0
    # discretisation: context classes small <= 512 < large <= 4096 < huge
    c = lambda n_ctx: routing.cell(CENTERS, 100, 100, n_ctx, 1.0) // 90
    assert [c(0), c(512), c(513), c(4096), c(4097)] == [0, 0, 1, 1, 2]
    # the paper's two example settings land in the extreme workload types
    r = lambda a, b: (routing.cell(CENTERS, a, b, 100, 1.0) // 10) % 9
    assert r(32, 512) == 0 and r(1024, 32) == 8 and r(300, 300) == 4
    # QPS snaps to the nearest benchmark level
    q = lambda x: routing.cell(CENTERS, 100, 100, 100, x) % 10
    assert [q(0.1), q(0.8), q(5.1), q(11.2), q(19), q(500)] == [0, 1, 4, 7, 9, 9]
    # the score is a difference, and the decision is its strict sign: a tie stays on the prefill-node path
    assert routing.score(2.0, 3.0, 0.5, 0.25) == 2.0 * 0.5 - 3.0 * 0.25
    assert routing.build_table([0.5, 0.1, 0.2], [0.1, 0.5, 0.2], 1.0, 1.0) == [1, 0, 0]
    # a later turn takes what the table says, cell by cell
    one_hot = [0] * 270
    one_hot[routing.cell(CENTERS, 1024, 32, 5000, 8.0)] = 1
    assert routing.decide(one_hot, CENTERS, 2, 1024, 32, 5000, 8.0) == 1
    assert routing.decide(one_hot, CENTERS, 2, 1024, 32, 500, 8.0) == 0
    # reading: the nearest workload type is taken on a logarithmic ratio scale -- 0.09 lies above the geometric mean
    # of the two lowest centres (0.0884) and below their arithmetic mean (0.0938)
    assert r(90, 1000) == 1 and r(88, 1000) == 0


def test_oracle_pins_from_the_paper():
    _pins(routing)


ROUTING_MUTANTS = [
    ("small_class_excludes_512", "n_ctx <= 512", "n_ctx < 512"),
    ("large_class_excludes_4096", "n_ctx <= 4096", "n_ctx < 4096"),
    ("linear_ratio_distance", "abs(math.log(ratio) - math.log(ratio_centers[i]))", "abs(ratio - ratio_centers[i])"),
    ("turn_one_rule_dropped", "if turn == 1:", "if turn == 0:"),
    ("score_sign_of_tpot_term", "w_ttft * delta_ttft - w_tpot * delta_tpot", "w_ttft * delta_ttft + w_tpot * delta_tpot"),
    ("tie_goes_local", "a, b) > 0 else 0", "a, b) >= 0 else 0"),
    ("ratio_inverted", "ratio = n_in / n_out", "ratio = n_out / n_in"),
    ("qps_floor_instead_of_nearest", "key=lambda i: abs(QPS_LEVELS[i] - qps))", "key=lambda i: abs(QPS_LEVELS[i] - qps) if QPS_LEVELS[i] <= qps else 1e9)"),
    ("axes_swapped_in_cell_index", "(ctx * 9 + r) * 10 + q", "(r * 3 + ctx) * 10 + q"),
]


def test_the_unmodified_routing_oracle_source_passes_its_pins():
    import types
    mod = types.ModuleType("routing_copy")
    exec(compile(open(routing.__file__).read(), "routing_copy", "exec"), mod.__dict__)
    _pins(mod)


@pytest.mark.parametrize("name,old,new", ROUTING_MUTANTS, ids=[m[0] for m in ROUTING_MUTANTS])
def test_planted_routing_mistake_fails_a_pin(name, old, new):
    """One plausible slip at a time in a copy of the routing oracle's source: the pins must notice."""
    import types
    src = open(routing.__file__).read()
    assert src.count(old) == 1, "the routing oracle's source no longer contains %r exactly once" % old
    mod = types.ModuleType("routing_mutant")
    exec(compile(src.replace(old, new), name, "exec"), mod.__dict__)
    with pytest.raises(AssertionError):
        _pins(mod)


def test_library_matches_oracle():
    rng = np.random.default_rng(0)
    dt = rng.uniform(-0.2, 1.0, 270)
    dp = rng.uniform(0.0, 0.6, 270)
    for w in [(1.0, 1.0), (1.0, 0.0), (0.0, 1.0), (1.0, 4.0), (2.5, 0.3)]:
        table = ppd.ppd_route_table_build(dt, dp, *w)
        assert table.tolist() == routing.build_table(dt, dp, *w)
        for _ in range(300):
            turn = int(rng.integers(1, 6))
            n_in, n_out = int(rng.integers(1, 3000)), int(rng.integers(1, 3000))
            n_ctx = int(rng.choice([0, 100, 512, 513, 4096, 4097, 30000]))
            qps = float(rng.uniform(0.1, 30))
            assert ppd.ppd_route_cell(CENTERS, n_in, n_out, n_ctx, qps) == routing.cell(CENTERS, n_in, n_out, n_ctx, qps)
            assert ppd.ppd_route_decide(table, CENTERS, turn, n_in, n_out, n_ctx, qps) == \
                routing.decide(table.tolist(), CENTERS, turn, n_in, n_out, n_ctx, qps)
    assert ppd.ppd_route_score(1.0, 2.0, 0.5, 0.1) == routing.score(1.0, 2.0, 0.5, 0.1)
    # invalid arguments
    assert ppd.ppd_route_decide(table, CENTERS, 0, 10, 10, 10, 1.0) == -1
    assert ppd.ppd_route_decide(table, CENTERS, 2, 0, 10, 10, 1.0) == -1
    assert ppd.ppd_route_cell(CENTERS, 10, 10, 10, 0.0) == -1
    with pytest.raises(ppd.PPDError):
        ppd.ppd_route_table_build(dt, dp, -1.0, 1.0)


def test_decision_is_fast():
    """The paper bounds the online lookup by 1 ms.  The C function is timed with the loop inside one library call
    (ppd_route_decide_batch), so that the figure is the lookup's and not the Python marshalling's."""
    import time
    rng = np.random.default_rng(1)
    table = ppd.ppd_route_table_build(rng.uniform(-0.2, 1.0, 270), rng.uniform(0, 0.6, 270), 1.0, 1.0)
    count = 200_000
    turn = rng.integers(1, 6, count)
    n_in, n_out = rng.integers(1, 3000, count), rng.integers(1, 3000, count)
    n_ctx, qps = rng.integers(0, 30000, count), rng.uniform(0.1, 30, count)
    ppd.ppd_route_decide_batch(table, CENTERS, turn[:10], n_in[:10], n_out[:10], n_ctx[:10], qps[:10])
    t0 = time.perf_counter()
    x = ppd.ppd_route_decide_batch(table, CENTERS, turn, n_in, n_out, n_ctx, qps)
    per_call = (time.perf_counter() - t0) / count
    print("ppd_route_decide: %.0f ns per decision" % (per_call * 1e9))
    assert per_call < 1e-5            # 100 x below the paper's 1 ms bound
    for i in range(0, count, 9973):   # and the batch call is the single call, element by element
        assert x[i] == ppd.ppd_route_decide(table, CENTERS, int(turn[i]), int(n_in[i]), int(n_out[i]), int(n_ctx[i]),
                                            float(qps[i]))
