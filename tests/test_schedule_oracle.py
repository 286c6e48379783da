"""Pins for the brute-force schedule oracle: hand-derived schedules (CPU only).

Derived by hand from Section 3.1 (SCCs -> recurrent nodes; delayed connections first, then
the per-step DAG in topological order) and from the Fig. 1 caption (the LSTM's memory block
forms one non-singleton SCC), plus Section 4's remark that the language-model LSTM has no
connection from the block output back to the block input."""
import numpy as np

import workloads as wl
from oracle import schedule_oracle as so

B, SD, S0 = so.BATCHED, so.STEP_DELAYED, so.STEP_DELAY0


def names(spec):
    return [n["name"] for n in spec.nodes]


def by_name(spec, arr):
    return {n["name"]: arr[k] for k, n in enumerate(spec.nodes)}


def edge_classes_by_name(spec, cls):
    nm = names(spec)
    return {(nm[e["src"]], nm[e["dst"]], e["delay"]): cls[m] for m, e in enumerate(spec.edges)}


def test_s1_fig1_lstm():
    spec = wl.lstm_net(8, [16], 4)
    s = so.schedule(spec.nodes, spec.edges)
    assert s["n_comps"] == 3
    comp = by_name(spec, s["node_comp"])
    assert comp["x"] == 0 and comp["out"] == 2
    assert all(comp[f"L1.{v}"] == 1 for v in ("i", "f", "g", "m_ig", "m_fc", "c", "o", "tc", "h"))
    rec = by_name(spec, s["comp_recurrent"])
    assert rec["x"] == 0 and rec["out"] == 0 and rec["L1.c"] == 1 and rec["L1.h"] == 1
    lvl = by_name(spec, s["node_level"])
    expect = {"x": 0, "out": 0, "L1.i": 0, "L1.f": 0, "L1.g": 0, "L1.m_ig": 1, "L1.m_fc": 1,
              "L1.c": 2, "L1.o": 3, "L1.tc": 3, "L1.h": 4}
    assert lvl == expect
    assert by_name(spec, s["comp_level"]) == {**{k: 1 for k in expect}, "x": 0, "out": 2}
    ec = edge_classes_by_name(spec, s["edge_class"])
    for gate in "ifgo":
        assert ec[("x", f"L1.{gate}", 0)] == B
        assert ec[("L1.h", f"L1.{gate}", 1)] == SD
    assert ec[("L1.h", "out", 0)] == B
    assert ec[("L1.c", "L1.i", 1)] == SD and ec[("L1.c", "L1.f", 1)] == SD and ec[("L1.c", "L1.m_fc", 1)] == SD
    assert sum(1 for c in s["edge_class"] if c == SD) == 7
    assert sum(1 for c in s["edge_class"] if c == S0) == 9
    assert sum(1 for c in s["edge_class"] if c == B) == 5


def test_s2_lstm_without_output_recurrence():
    """Without h -> gate edges the loop shrinks to {i, f, m_ig, m_fc, c}; g comes before it, o, tc, h after."""
    spec = wl.lstm_net(8, [16], 4, output_recurrence=False)
    s = so.schedule(spec.nodes, spec.edges)
    comp = by_name(spec, s["node_comp"]); rec = by_name(spec, s["comp_recurrent"])
    clv = by_name(spec, s["comp_level"]); lvl = by_name(spec, s["node_level"])
    loop = ["L1.i", "L1.f", "L1.m_ig", "L1.m_fc", "L1.c"]
    assert len({comp[v] for v in loop}) == 1
    assert all(rec[v] == 1 for v in loop)
    for v in ("x", "L1.g", "L1.o", "L1.tc", "L1.h", "out"):
        assert rec[v] == 0 and lvl[v] == 0
        assert comp[v] != comp["L1.c"]
    assert s["n_comps"] == 7
    assert clv == {"x": 0, "L1.g": 1, "L1.i": 2, "L1.f": 2, "L1.m_ig": 2, "L1.m_fc": 2, "L1.c": 2,
                   "L1.o": 3, "L1.tc": 3, "L1.h": 4, "out": 5}
    # numbering by (level, smallest node id): x, g, loop, o, tc, h, out
    assert [comp[v] for v in ("x", "L1.g", "L1.c", "L1.o", "L1.tc", "L1.h", "out")] == [0, 1, 2, 3, 4, 5, 6]
    assert {v: lvl[v] for v in loop} == {"L1.i": 0, "L1.f": 0, "L1.m_ig": 1, "L1.m_fc": 1, "L1.c": 2}
    ec = edge_classes_by_name(spec, s["edge_class"])
    assert ec[("L1.g", "L1.m_ig", 0)] == B and ec[("L1.c", "L1.o", 0)] == B and ec[("L1.c", "L1.tc", 0)] == B
    assert ec[("L1.c", "L1.i", 1)] == SD and ec[("L1.i", "L1.m_ig", 0)] == S0


def test_s3_generalized_condensation():
    spec = wl.generalized_net(6, 4, 3, 5)
    assert len(spec.nodes) == 33 and len(spec.edges) == 70
    s = so.schedule(spec.nodes, spec.edges)
    assert s["n_comps"] == 9
    clv = by_name(spec, s["comp_level"]); comp = by_name(spec, s["node_comp"]); rec = by_name(spec, s["comp_recurrent"])
    expect = {"x": 0, "L1.h": 1, "q1": 2, "p1": 3, "L2.h": 4, "q2": 5, "p2": 6, "L3.h": 7, "out": 8}
    for v, l in expect.items():
        assert clv[v] == l and comp[v] == l
    assert [rec[v] for v in expect] == [0, 1, 0, 0, 1, 0, 0, 1, 0]
    ec = edge_classes_by_name(spec, s["edge_class"])
    assert ec[("L2.h", "L2.i", 2)] == SD and ec[("L1.h", "q1", 0)] == B and ec[("p1", "L2.i", 0)] == B


def test_elman_self_loop_is_recurrent_singleton():
    spec = wl.elman_net(3, 4, 2)
    s = so.schedule(spec.nodes, spec.edges)
    assert s["node_comp"] == [0, 1, 2] and s["comp_recurrent"] == [0, 1, 0]
    assert s["edge_class"] == [B, SD, B] and s["node_level"] == [0, 0, 0]


def test_delayed_edge_between_components_is_batched_and_delay0_full_edge_inside_scc():
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 3); a = g.add_node(wl.ADD, wl.TANH, 4)
    b = g.add_node(wl.ADD, wl.TANH, 2); out = g.add_node(wl.ADD, wl.SOFTMAX, 2, True, True)
    g.add_edge(x, a, wl.FULL, 2); g.add_edge(a, b, wl.FULL, 0); g.add_edge(b, a, wl.FULL, 1); g.add_edge(b, out, wl.FULL, 3)
    s = so.schedule(g.nodes, g.edges)
    assert s["edge_class"] == [B, S0, SD, B]
    assert s["node_level"] == [0, 0, 1, 0] and s["comp_recurrent"] == [0, 1, 1, 0]


def test_levels_invariant_under_relabelling():
    rng = np.random.default_rng(3)
    spec = wl.generalized_net(3, 4, 2, 3)
    s = so.schedule(spec.nodes, spec.edges)
    K, M = len(spec.nodes), len(spec.edges)
    pn, pe = rng.permutation(K), rng.permutation(M)
    s2 = so.schedule(*(lambda g: (g.nodes, g.edges))(spec.permuted(pn, pe)))
    for k in range(K):
        assert s2["node_level"][int(pn[k])] == s["node_level"][k]
        assert s2["comp_level"][int(pn[k])] == s["comp_level"][k]
        assert s2["comp_recurrent"][int(pn[k])] == s["comp_recurrent"][k]
    for m in range(M):
        assert s2["edge_class"][int(pe[m])] == s["edge_class"][m]
