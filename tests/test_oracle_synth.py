"""Pins for oracle.synth (Sec. 4: Hoare-triple semantics of Fig. "semantics", search space of Fig. "a*", cost model Sec. 3.2)."""
import numpy as np
import pytest

from oracle import rounding, synth as S

NET = dict(latency=1e-5, bandwidth=1e10, elem_bytes=4)


def example_graph():
    """The single-device program of Fig. "a*_example": e1 = Placeholder(), e2 = Parameter(), e3 = MatMul(e1, e2), loss = Sum(e3)."""
    return [S.node("placeholder", rows=64, cols=128), S.node("parameter", rows=128, cols=256), S.node("matmul", 0, 1, 64, 256), S.node("sum", 2)]


def mlp_graph(b=12, h=8, f=10):
    return [S.node("placeholder", rows=b, cols=h), S.node("parameter", rows=h, cols=f), S.node("matmul", 0, 1, b, f), S.node("unary", 2, rows=b, cols=f),
            S.node("parameter", rows=f, cols=h), S.node("matmul", 3, 4, b, h), S.node("sum", 5)]


def test_worked_example_of_the_search_figure():
    """With the example's restrictions (input sharded on dimension 0 only, never replicated; parameter whole or sharded on
    dimension 1; no communication optimisations) the only complete program without communication is the one the text
    arrives at as program 7: Placeholder-Shard(0), Parameter, MatMul, Sum, with property loss | All-Reduce."""
    t, ties, count = S.best_program(example_graph(), [0.5, 0.5], [1e12, 1e12], NET, placeholder_dims=(0,), parameter_dims=(1,),
                                    grouped_broadcast=False, replicated_matmul=False, placeholder_replicated=False)
    assert ties == [[("placeholder-shard", 0, 0), ("parameter", 1), ("matmul", 2, "ag0", "id"), ("sum", 3, "ag0")]]
    assert t == pytest.approx((2 * 64 * 128 * 256 + 64 * 256) * 0.5 / 1e12, rel=1e-12)


def test_program_time_hand_worked():
    """Two devices, B = (0.75, 0.25), speeds (2, 1) flop/s; a program with one All-Gather: stage 1 = sharded MatMul, then the
    collective, stage 2 = replicated Sum."""
    g = [S.node("placeholder", rows=4, cols=2), S.node("parameter", rows=2, cols=6), S.node("matmul", 0, 1, 4, 6), S.node("sum", 2)]
    net = dict(latency=0.5, bandwidth=8.0, elem_bytes=2)
    prog = [("placeholder-shard", 0, 0), ("parameter", 1), ("matmul", 2, "ag0", "id"), ("all-gather", 2, 0), ("sum", 3, "id")]
    # matmul: 2*4*2*6 = 96 flops -> device 0: 72/2 = 36 s, device 1: 24/1 = 24 s -> 36;  all-gather of 4x6x2 = 48 bytes in 2 slots of
    # the largest shard: 0.5 + 2*0.75*48/8 = 9.5;  sum over 24 elements replicated: 24/2 = 12, 24/1 = 24 -> 24
    assert S.program_time(g, prog, [0.75, 0.25], [2.0, 1.0], net) == pytest.approx(36 + 9.5 + 24)
    assert S.comm_time(g, ("grouped-broadcast", 2, 0), [0.75, 0.25], net) == pytest.approx(2 * 0.5 + 48 / 8)
    assert S.comm_time(g, ("all-reduce", 2), [0.75, 0.25], net) == pytest.approx(0.5 + 2 * 48 / 8)


_THEORY = {}


def theory_of(graph):
    key = id(graph)
    if key not in _THEORY:
        _THEORY[key] = {t[1]: t for t in S.theory(graph)}
    return _THEORY[key]


def _run_distributed(graph, program, B, rng):
    """Executes a distributed program on m simulated devices with uneven integer shards and returns (sum of the devices'
    loss instances, single-device loss): the semantic constraint loss | All-Reduce says the two are equal."""
    m = len(B)
    ref = {}
    for e, n in enumerate(graph):
        if n["op"] in ("placeholder", "parameter"):
            ref[e] = rng.standard_normal((n["rows"], n["cols"]))
        elif n["op"] == "matmul":
            ref[e] = ref[n["a"]] @ ref[n["b"]]
        elif n["op"] == "unary":
            ref[e] = np.tanh(ref[n["a"]])
        elif n["op"] == "add":
            ref[e] = ref[n["a"]] + ref[n["b"]]
        elif n["op"] == "transpose":
            ref[e] = ref[n["a"]].T
        elif n["op"] == "sum":
            ref[e] = ref[n["a"]].sum()

    def cut(t, d):
        _, offs = rounding.round_shards(B, t.shape[d], 1)
        return [t[offs[j]:offs[j + 1], :] if d == 0 else t[:, offs[j]:offs[j + 1]] for j in range(m)]
    inst = {}                      # (reference tensor, form) -> the distributed tensor's instances, one per device
    T = theory_of(graph)
    for ins in program:
        name, e = ins[0], ins[1]
        n = graph[e]
        (out_prop,) = T[ins][2]
        assert T[ins][0] <= set(inst), "precondition not established"
        if name in ("placeholder", "parameter"):
            val = [ref[e]] * m
        elif name in ("placeholder-shard", "parameter-shard"):
            val = cut(ref[e], ins[2])
        elif name == "matmul":
            val = [inst[(n["a"], ins[2])][j] @ inst[(n["b"], ins[3])][j] for j in range(m)]
        elif name == "unary":
            val = [np.tanh(x) for x in inst[(n["a"], ins[2])]]
        elif name == "add":
            val = [inst[(n["a"], ins[2])][j] + inst[(n["b"], ins[2])][j] for j in range(m)]
        elif name == "transpose":
            val = [x.T for x in inst[(n["a"], ins[2])]]
        elif name == "sum":
            val = [x.sum() for x in inst[(n["a"], ins[2])]]
        elif name == "all-reduce":
            val = [sum(inst[(e, "ar")])] * m
        elif name == "reduce-scatter":
            val = cut(sum(inst[(e, "ar")]), ins[2])
        elif name in ("all-gather", "grouped-broadcast"):
            val = [np.concatenate(inst[(e, S.AG(ins[2]))], axis=ins[2])] * m
        elif name == "all-to-all":
            val = cut(np.concatenate(inst[(e, S.AG(ins[2]))], axis=ins[2]), ins[3])
        else:
            raise ValueError(name)
        inst[out_prop] = val
        # what the property claims: applying its collective to the instances gives the reference tensor
        form = out_prop[1]
        whole = val[0] if form == "id" else (sum(val) if form == "ar" else np.concatenate(val, axis=int(form[2])))
        np.testing.assert_allclose(whole, ref[e], rtol=1e-9, atol=1e-9)
    loss = len(graph) - 1
    return sum(inst[(loss, "ar")]), ref[loss]


def test_every_complete_program_computes_the_single_device_loss():
    """The theory is sound: each program it admits - all sharding forms, all collectives, uneven shards with an empty one -
    reproduces the single-device loss when executed.  This pins every Hoare triple against the mathematics."""
    rng = np.random.default_rng(0)
    g = mlp_graph()
    B = [0.5, 0.3, 0.2, 0.0]
    progs = list(S.all_programs(g))
    assert len(progs) > 100
    names = set()
    for prog in progs:
        got, want = _run_distributed(g, prog, B, rng)
        assert got == pytest.approx(want, rel=1e-10, abs=1e-10), prog
        names |= {ins[0] for ins in prog}
    assert {"all-reduce", "reduce-scatter", "all-gather", "grouped-broadcast", "all-to-all", "placeholder-shard", "parameter-shard"} <= names
    # a graph with transpose and add: loss = sum(x w + ((x w)^T)^T); every 7th of its ~29k programs
    g2 = [S.node("placeholder", rows=6, cols=5), S.node("parameter", rows=5, cols=4), S.node("matmul", 0, 1, 6, 4), S.node("transpose", 2, rows=4, cols=6),
          S.node("transpose", 3, rows=6, cols=4), S.node("add", 2, 4, 6, 4), S.node("sum", 5)]
    n2 = 0
    for i, prog in enumerate(S.all_programs(g2, grouped_broadcast=False)):
        if i % 7:
            continue
        got, want = _run_distributed(g2, prog, [0.6, 0.4], rng)
        assert got == pytest.approx(want, rel=1e-10, abs=1e-10), prog
        n2 += 1
    assert n2 > 1000


def test_more_rules_never_hurt_and_bandwidth_decides():
    g = mlp_graph(b=64, h=256, f=1024)
    B, speed = [0.6, 0.4], [1.5e12, 1e12]
    t_all, _, n_all = S.best_program(g, B, speed, NET)
    t_few, _, n_few = S.best_program(g, B, speed, NET, grouped_broadcast=False, replicated_matmul=False)
    assert n_all > n_few and t_all <= t_few * (1 + 1e-12)
    # input sharded on the batch only, parameters whole or sharded: with a fast network nothing changes (no collective is needed
    # at all: batch-parallel or the feature/reduction pair); the optimum never contains a communication instruction here
    _, ties, _ = S.best_program(g, B, speed, NET)
    assert all(ins[0] not in S.COMM for prog in ties for ins in prog)
