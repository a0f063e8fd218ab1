"""Distributed program synthesis on small graphs (Sec. 4: syntax Fig. "syntax", semantics Fig. "semantics",
search Fig. "a*"; Sec. 4.4 / 4.5 rules for Grouped-Broadcast and the replicated MatMul; cost model Sec. 3.2).

This oracle does NOT run A*: it enumerates every instruction sequence the theory allows (depth-first, no cost
pruning, no dominance pruning) and returns the cheapest complete program, so a search that prunes can be checked
against it.  Everything is written out plainly:

  graph      list of nodes (op, inputs, rows, cols); a node's output is reference tensor e = its index.
             ops: "placeholder", "parameter", "matmul" (e = a b), "unary" (elementwise, non-linear), "add", "transpose",
             "sum" (all elements -> scalar; the loss)
  property   (e, form): what has to be done to the distributed tensor to obtain e on every device -
             "id" (nothing: replicated), ("ag", d) (All-Gather along d: sharded on d), "ar" (All-Reduce: partial sums)
  theory     Hoare triples (precondition set, instruction, postcondition set) matched on the graph
  complete   (loss, "ar") in P(Q)            (the semantic constraint of Sec. 4.2)
  cost       t(Q, B) of Sec. 3.2: a communication instruction synchronises the devices and starts a stage; a stage
             costs its communication time plus the slowest device's computation time

Restrictions (the paper's search-time optimisations of Sec. 4.5, or added here and named as such): every reference
tensor is communicated at most once and outputs of placeholder / parameter are not communicated (Sec. 4.5, second
optimisation); added here: every reference tensor is computed once, and computations appear in the graph's
(topological) order, so only the forms and the places of the collectives vary; loading instructions cost nothing.
"""
from __future__ import annotations

ID, AR = "id", "ar"


def AG(d):
    return "ag%d" % d


def node(op, a=-1, b=-1, rows=1, cols=1):
    return dict(op=op, a=a, b=b, rows=rows, cols=cols)


def theory(graph, placeholder_dims=(0, 1), parameter_dims=(0, 1), grouped_broadcast=True, replicated_matmul=True,
           placeholder_replicated=True):
    """All Hoare triples of the graph.  An instruction is (name, e, args...).  The keyword switches narrow the rule set
    (the worked example of Fig. "a*_example" shards the input on dimension 0 only and the parameter on dimension 1 only)."""
    T = []
    for e, n in enumerate(graph):
        op, a, b = n["op"], n["a"], n["b"]
        if op == "placeholder":
            if placeholder_replicated:
                T.append((frozenset(), ("placeholder", e), frozenset({(e, ID)})))
            for d in placeholder_dims:
                T.append((frozenset(), ("placeholder-shard", e, d), frozenset({(e, AG(d))})))
        elif op == "parameter":
            T.append((frozenset(), ("parameter", e), frozenset({(e, ID)})))
            for d in parameter_dims:
                T.append((frozenset(), ("parameter-shard", e, d), frozenset({(e, AG(d))})))
        elif op == "matmul":
            rules = [((AG(0), ID), AG(0)), ((ID, AG(1)), AG(1)), ((AG(1), AG(0)), AR)]       # Fig. "semantics"
            if replicated_matmul:
                rules.append(((ID, ID), ID))                                                   # Sec. 4.4, the SFB rule
            for (fa, fb), fo in rules:
                T.append((frozenset({(a, fa), (b, fb)}), ("matmul", e, fa, fb), frozenset({(e, fo)})))
        elif op == "unary":
            for f in (ID, AG(0), AG(1)):
                T.append((frozenset({(a, f)}), ("unary", e, f), frozenset({(e, f)})))
        elif op == "add":
            for f in (ID, AG(0), AG(1), AR):
                T.append((frozenset({(a, f), (b, f)}), ("add", e, f), frozenset({(e, f)})))
        elif op == "transpose":
            for f, g in ((ID, ID), (AG(0), AG(1)), (AG(1), AG(0)), (AR, AR)):
                T.append((frozenset({(a, f)}), ("transpose", e, f), frozenset({(e, g)})))
        elif op == "sum":
            for f in (AG(0), AG(1), AR):                                # partial sums of a sharded or partial tensor
                T.append((frozenset({(a, f)}), ("sum", e, f), frozenset({(e, AR)})))
            T.append((frozenset({(a, ID)}), ("sum", e, ID), frozenset({(e, ID)})))
        else:
            raise ValueError(op)
        if op not in ("placeholder", "parameter", "sum"):               # collectives on computed, non-scalar tensors
            T.append((frozenset({(e, AR)}), ("all-reduce", e), frozenset({(e, ID)})))
            for d in (0, 1):
                T.append((frozenset({(e, AR)}), ("reduce-scatter", e, d), frozenset({(e, AG(d))})))
                T.append((frozenset({(e, AG(d))}), ("all-gather", e, d), frozenset({(e, ID)})))
                if grouped_broadcast:
                    T.append((frozenset({(e, AG(d))}), ("grouped-broadcast", e, d), frozenset({(e, ID)})))
                T.append((frozenset({(e, AG(d))}), ("all-to-all", e, d, 1 - d), frozenset({(e, AG(1 - d))})))
    return T


COMM = ("all-reduce", "reduce-scatter", "all-gather", "grouped-broadcast", "all-to-all")
SOURCE = ("placeholder", "placeholder-shard", "parameter", "parameter-shard")


def flops(graph, ins, Bj):
    """Flops device j spends on a computation instruction when its ratio is Bj (Sec. 3.2: proportional to the ratio if a
    sharded dimension takes part, unchanged otherwise)."""
    name, e = ins[0], ins[1]
    n = graph[e]
    if name in SOURCE:
        return 0.0
    if name == "matmul":
        full = 2.0 * graph[n["a"]]["rows"] * graph[n["a"]]["cols"] * n["cols"]
        return full if (ins[2], ins[3]) == (ID, ID) else full * Bj
    src = graph[n["a"]] if name in ("sum", "transpose", "unary") else n
    full = float(src["rows"] * src["cols"])
    form = ins[2]
    return full * Bj if (form != ID and form != AR) else full


def comm_time(graph, ins, B, net):
    """Linear latency + size / bandwidth model on the largest shard (Sec. 3.2, Sec. 5.1); net = dict(latency, bandwidth,
    elem_bytes).  Padded All-Gather / Reduce-Scatter / All-To-All move m equal slots of the largest shard's size; the
    All-Reduce moves the whole tensor twice (reduce-scatter + all-gather of even pieces); the grouped Broadcast moves
    every shard at its own size (the whole tensor once) but pays one latency per device."""
    name, e = ins[0], ins[1]
    m = len(B)
    size = graph[e]["rows"] * graph[e]["cols"] * net["elem_bytes"]
    lat, bw = net["latency"], net["bandwidth"]
    if name == "all-reduce":
        return lat + 2.0 * size / bw
    if name == "grouped-broadcast":
        return m * lat + size / bw
    return lat + m * max(B) * size / bw


def program_time(graph, program, B, speed, net):
    """t(Q, B): stages end at communication instructions (Sec. 3.2)."""
    total = 0.0
    busy = [0.0] * len(B)
    for ins in program:
        if ins[0] in COMM:
            total += max(busy) + comm_time(graph, ins, B, net)
            busy = [0.0] * len(B)
        else:
            for j in range(len(B)):
                busy[j] += flops(graph, ins, B[j]) / speed[j]
    return total + max(busy)


def all_programs(graph, **rules):
    """Every complete program the theory allows under the restrictions above (a generator of instruction lists)."""
    T = theory(graph, **rules)
    loss = len(graph) - 1

    def rec(program, props, next_node, communicated):
        if (loss, AR) in props:
            yield list(program)
            return
        for pre, ins, post in T:
            e = ins[1]
            if not pre <= props or post <= props:
                continue
            if ins[0] in COMM:
                if e not in communicated:
                    yield from rec(program + [ins], props | post, next_node, communicated | {e})
            elif e == next_node:
                yield from rec(program + [ins], props | post, next_node + 1, communicated)

    yield from rec([], frozenset(), 0, frozenset())


def best_program(graph, B, speed, net, **rules):
    """Cheapest complete program by exhaustive enumeration.  Returns (time, the optimal programs (all ties), how many
    complete programs exist)."""
    best, ties, count = float("inf"), [], 0
    for prog in all_programs(graph, **rules):
        count += 1
        t = program_time(graph, prog, B, speed, net)
        if t < best * (1 - 1e-12):
            best, ties = t, [prog]
        elif t <= best * (1 + 1e-12):
            ties.append(prog)
    return best, ties, count


def program_stages(graph, program, m, net):
    """The program's stages as (F, G, a, c) tuples for the load balancer (Sec. 5.1): F flops that scale with the ratio,
    G flops that do not, a + c * max_j B_j the time of the collective that opens the stage."""
    stages = [[0.0, 0.0, 0.0, 0.0]]
    for ins in program:
        if ins[0] in COMM:
            a = comm_time(graph, ins, [0.0] * m, net)
            c = comm_time(graph, ins, [1.0] + [0.0] * (m - 1), net) - a
            stages.append([0.0, 0.0, a, c])
        else:
            f1, f0 = flops(graph, ins, 1.0), flops(graph, ins, 0.0)
            stages[-1][0] += f1 - f0
            stages[-1][1] += f0
    return [tuple(s) for s in stages]


def optimize(graph, speed, net, max_steps=10, **rules):
    """The alternating optimisation of Sec. 3.1 with exhaustive synthesis and the LP oracle: returns the sequence of
    (t(Q(s), B(s-1)), t(Q(s), B(s))) per step and the best time seen."""
    from . import lp
    m = len(speed)
    B = [s / sum(speed) for s in speed]
    history, best, prev = [], float("inf"), float("inf")
    for _ in range(max_steps):
        tq, ties, _ = best_program(graph, B, speed, net, **rules)
        # among equally cheap programs the load balancer may do better with one than another: take the best of them
        cand = [lp.shard_ratios(speed, program_stages(graph, p, m, net)) for p in ties]
        Bn, tb = min(cand, key=lambda x: x[1])
        history.append((tq, tb))
        best = min(best, tq, tb)
        B = list(Bn)
        if not tb < prev * (1 - 1e-12):
            break
        prev = tb
    return history, best
