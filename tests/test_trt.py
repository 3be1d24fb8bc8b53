"""Scheduling layer: the plain-Python oracle (oracle/trt.py) against what the paper and the
mathematics fix, then the library's host implementation against the oracle, bit for bit.
All CPU."""
import itertools

import numpy as np
import pytest

from oracle import trt as O
from paper_2603_16104_amd import workloads as wl


def calls_of(w):
    return [O.Call(t, lo, wk) for t, lo, wk in zip(w.templates, w.len_out, w.worker)]


def sym_weight(syms, len_out):
    return sum(1 if s >= 0 else len_out[-(s + 1)] for s in syms)


def lcp(a, b):
    k = 0
    while k < len(a) and k < len(b) and a[k] == b[k]:
        k += 1
    return k


SEEDS = list(range(12))


# ------------------------------------------------------------------ oracle pins: the tree

@pytest.mark.parametrize("seed", SEEDS)
def test_oracle_tree_is_a_radix_tree_of_the_templates(seed):
    """Structure fixed by the definition of a radix tree: every call's root-to-parent path spells its
    template; siblings start with different symbols; no internal node has a single internal child
    and nothing else (it would have been one segment); weights follow the symbols."""
    w = wl.random_workflow(seed, n_calls=14)
    t = O.build_trt(calls_of(w))
    assert t.parent[0] == -1 and all(0 <= t.parent[v] < v for v in range(1, t.n_nodes))   # parent-first numbering
    for c in range(w.n_calls):
        leaf = t.leaf_of_call[c]
        assert t.call[leaf] == c and t.weight[leaf] == 0 and t.seg_len[leaf] == 0
        spelled = []
        for v in t.path(leaf):
            spelled += t.syms[t.seg_begin[v]: t.seg_begin[v] + t.seg_len[v]]
        assert spelled == w.templates[c]
    for v in range(t.n_nodes):
        kids = t.children(v)
        firsts = [t.syms[t.seg_begin[k]] for k in kids if t.call[k] < 0]
        assert len(firsts) == len(set(firsts))
        if t.call[v] < 0:
            assert t.weight[v] == sym_weight(t.syms[t.seg_begin[v]: t.seg_begin[v] + t.seg_len[v]], w.len_out)
            if v > 0:
                assert t.seg_len[v] > 0
                assert len(kids) >= 2 or (len(kids) == 1 and t.call[kids[0]] >= 0)
        else:
            assert kids == []
    assert sum(1 for v in range(t.n_nodes) if t.call[v] >= 0) == w.n_calls


@pytest.mark.parametrize("seed", SEEDS)
def test_oracle_prefill_usage_equals_unshared_suffix_of_the_token_strings(seed):
    """u_p needs no tree at all: it is the weight of the call's template minus the weight of the
    longest common prefix with the previous call's template (Section 5, "Token usage")."""
    w = wl.random_workflow(seed, n_calls=14)
    t = O.build_trt(calls_of(w))
    rng = np.random.default_rng(seed)
    order = rng.permutation(w.n_calls).tolist()
    for j, c in enumerate(order):
        full = sym_weight(w.templates[c], w.len_out)
        if j == 0:
            assert O.prefill_usage(t, -1, c) == full
        else:
            k = lcp(w.templates[order[j - 1]], w.templates[c])
            assert O.prefill_usage(t, order[j - 1], c) == full - sym_weight(w.templates[c][:k], w.len_out)


def test_oracle_tree_insertion_order_is_topological():
    """A call whose template is a prefix of a later one, inserted after it, still yields the same
    set of segments (the radix tree of a set of strings is unique up to child order)."""
    a = [O.Call([1, 2, 3, 4], 1), O.Call([1, 2], 1), O.Call([1, 2, 3, 9], 1)]
    b = [a[1], a[2], a[0]]
    segs = lambda t: sorted(tuple(t.syms[t.seg_begin[v]: t.seg_begin[v] + t.seg_len[v]]) for v in range(t.n_nodes)
                            if t.call[v] < 0 and v > 0)
    assert segs(O.build_trt(a)) == segs(O.build_trt(b)) == [(1, 2), (3,), (4,), (9,)]
    with pytest.raises(ValueError):
        O.build_trt([O.Call([-2], 1), O.Call([-1], 1)])       # cycle
    with pytest.raises(ValueError):
        O.build_trt([O.Call([-5], 1)])                        # missing call


# ------------------------------------------------------------------ oracle pins: the cost model

def longest_path_T(w, sigma, capacity):
    """Independent evaluation: T is the longest path in the graph whose arcs are 'next on the same
    worker' (length U of the tail call) and 'dependency' (length U + M * len_out of the tail call),
    plus the head call's own U; U from the token strings as above."""
    n = w.n_calls
    U, arcs = [0] * n, [[] for _ in range(n)]
    for seq in sigma:
        for j, c in enumerate(seq):
            full = sym_weight(w.templates[c], w.len_out)
            shared = 0 if j == 0 else sym_weight(w.templates[c][:lcp(w.templates[seq[j - 1]], w.templates[c])], w.len_out)
            U[c] = w.len_out[c] * (full - shared) + w.len_out[c] * (w.len_out[c] + 1) // 2
    for seq in sigma:
        for j in range(1, len(seq)):
            arcs[seq[j]].append((seq[j - 1], 0))
    for c in range(n):
        for x in {-(s + 1) for s in w.templates[c] if s < 0}:
            arcs[c].append((x, capacity * w.len_out[x]))
    memo = {}

    def finish(c):            # completion of c = U[c] + max over incoming arcs (finish(tail) + extra)
        if c not in memo:
            memo[c] = U[c] + max((finish(x) + extra for x, extra in arcs[c]), default=0)
        return memo[c]
    return max((finish(c) for c in range(n)), default=0)


@pytest.mark.parametrize("seed", SEEDS)
def test_oracle_evaluate_matches_longest_path(seed):
    w = wl.random_workflow(seed, n_calls=10, n_workers=2)
    t = O.build_trt(calls_of(w))
    order = O.topological_order(calls_of(w))
    sigma = [[c for c in order if w.worker[c] == i] for i in range(2)]
    B, C, T = O.evaluate_schedule(t, sigma, 50)
    assert T == longest_path_T(w, sigma, 50)
    for c in range(w.n_calls):
        for x in t.deps[c]:
            assert B[c] >= C[x] + 50 * w.len_out[x]


def test_oracle_cost_model_closed_forms():
    """One call: T = len_out * |prompt| + len_out (len_out + 1) / 2.  Two independent calls sharing a
    prefix of p tokens: the second pays only for its own tail.  A dependent call starts no earlier
    than M * len_out after its source completes (precedence delay)."""
    t = O.build_trt([O.Call(list(range(10)), 4)])
    assert O.evaluate_schedule(t, [[0]], 100)[2] == 4 * 10 + 10
    t = O.build_trt([O.Call(list(range(10)), 2), O.Call(list(range(6)) + [77, 78], 3)])
    B, C, T = O.evaluate_schedule(t, [[0, 1]], 100)
    assert C[0] == 2 * 10 + 3 and C[1] == C[0] + 3 * 2 + 6 and T == C[1]
    B, C, T = O.evaluate_schedule(t, [[1, 0]], 100)
    assert C[1] == 3 * 8 + 6 and C[0] == C[1] + 2 * 4 + 3
    t = O.build_trt([O.Call([1, 2], 5), O.Call([3, -1], 1)])
    B, C, T = O.evaluate_schedule(t, [[0, 1]], 100)
    assert B[1] == C[0] + 100 * 5 and C[1] == B[1] + 1 * (1 + 5) + 1
    with pytest.raises(ValueError):
        O.evaluate_schedule(t, [[1, 0]], 100)     # the dependent call first on the only worker: can never run


def paper_example():
    """The paper's two-agent example (Section 5, figure of the templated radix tree): (1) agent 1
    answers, (2) agent 2 answers the same question, (3) agent 2 comments on agent 1's answer."""
    a1, a2, q, f = list(range(100, 132)), list(range(200, 248)), list(range(300, 316)), list(range(400, 408))
    return [O.Call(a1 + q, 20), O.Call(a2 + q, 20), O.Call(a2 + q + [-1] + f, 10)]


def test_oracle_paper_example_order():
    """The paper states that 1 -> 2 -> 3 beats 2 -> 1 -> 3 (agent 2's prompt stays cached between 2
    and 3) and that the scheduler finds it."""
    t = O.build_trt(paper_example())
    T123 = O.evaluate_schedule(t, [[0, 1, 2]], 4096)[2]
    T213 = O.evaluate_schedule(t, [[1, 0, 2]], 4096)[2]
    assert T123 < T213
    # in 2 -> 1 -> 3 call 1 completes later by the whole of call 2 (20 * 64 + 210 token steps), and with it the
    # precedence delay that call 3 waits for; call 3 then re-prefills agent 2's prompt and the question (64 tokens)
    assert T213 - T123 == (20 * 64 + 210) + 10 * 64
    sigma, B, C, T = O.cache_aware_schedule(t, 1, 4096)
    assert sigma == [[0, 1, 2]] and T == T123


@pytest.mark.parametrize("seed", SEEDS)
def test_oracle_schedule_is_valid_and_consistent(seed):
    w = wl.random_workflow(seed, n_calls=12, n_workers=2)
    t = O.build_trt(calls_of(w))
    sigma, B, C, T = O.cache_aware_schedule(t, 2, 40)
    assert sorted(c for s in sigma for c in s) == list(range(w.n_calls))
    assert all(w.worker[c] == i for i, s in enumerate(sigma) for c in s)
    B2, C2, T2 = O.evaluate_schedule(t, sigma, 40)
    # the scheduler never starts a call earlier than the evaluator allows, and its times are feasible;
    # since it places every call at its earliest start, both agree exactly
    assert (B, C, T) == (B2, C2, T2)
    assert O.cache_aware_schedule(t, 2, 40)[0] == sigma           # deterministic


@pytest.mark.parametrize("seed", range(6))
def test_oracle_schedule_against_brute_force(seed):
    """Tiny single-worker instances: the optimum over all feasible permutations bounds the
    heuristic from below, the worst one from above."""
    w = wl.random_workflow(seed, n_calls=6, max_len=6)
    t = O.build_trt(calls_of(w))
    Ts = []
    for perm in itertools.permutations(range(w.n_calls)):
        try:
            Ts.append(O.evaluate_schedule(t, [list(perm)], 30)[2])
        except ValueError:
            pass
    T = O.cache_aware_schedule(t, 1, 30)[3]
    assert min(Ts) <= T <= max(Ts)


def test_oracle_schedule_groups_shared_prefixes():
    """Map-reduce shape with independent queries: once a query's context is in the cache the
    scheduler finishes that query's mappers before moving on (depth-first over the tree), so the
    total prefill usage is far below the operator-by-operator order."""
    w = wl.workflow_map_reduce(n_queries=4, n_mappers=3)
    t = O.build_trt(calls_of(w))
    sigma, _, _, T = O.cache_aware_schedule(t, 1, 8192)
    up = lambda seq: sum(O.prefill_usage(t, seq[j - 1] if j else -1, c) for j, c in enumerate(seq))
    opwise = [q * 4 + m for m in range(4) for q in range(4)]
    assert up(sigma[0]) <= up(opwise)
    assert T <= O.evaluate_schedule(t, [opwise], 8192)[2]


# ------------------------------------------------------------------ oracle pins: partition, nested sequences, soft execution

def two_operator_example(n_queries=3, sys_len=32, q_len=16, len_out=8):
    """The paper's tree figure: operators 2 and 3 start with the same static system prompt, followed by a
    question prompt that is unique to each query of the batch; operator 3 also reads the output of operator 1,
    which has a system prompt of its own."""
    w = wl.Workflow("two_operators")
    sys_a, sys_b = w.fresh_tokens(sys_len), w.fresh_tokens(sys_len)
    ids = []
    for q in range(n_queries):
        question = w.fresh_tokens(q_len)
        o1 = w.add(sys_a + question, len_out)
        o2 = w.add(sys_b + question, len_out)
        o3 = w.add(sys_b + question + [wl.Workflow.out(o1)], len_out)
        ids.append((o1, o2, o3))
    return w, ids


@pytest.mark.parametrize("make", [lambda: wl.workflow_map_reduce(6, 3), lambda: wl.workflow_debate(5, 3, 2), lambda: wl.workflow_reflect(7),
                                  lambda: wl.workflow_iterative(5, 4), lambda: wl.workflow_parallel(4, 3, 2),
                                  lambda: wl.random_workflow(3, n_calls=30), lambda: wl.random_workflow(8, n_calls=30, p_placeholder=0.05)])
@pytest.mark.parametrize("n_workers", [1, 2, 3])
def test_oracle_partition_invariants(make, n_workers):
    """What any reading of PartitionWorkflow must give: every call on exactly one worker, no dependency between
    workers (a query's calls stay together, so its prefixes are cached where they are used), and the greedy
    guarantee: no worker carries more than the mean load plus one group."""
    w = make()
    calls = calls_of(w)
    worker = O.partition_workflow(calls, n_workers)
    assert len(worker) == len(calls) and all(0 <= x < n_workers for x in worker)
    for c, call in enumerate(calls):
        assert all(worker[x] == worker[c] for x in call.deps())
    lo = [c.len_out for c in calls]
    cost = [c.len_out * sym_weight(c.template, lo) + c.len_out * (c.len_out + 1) // 2 for c in calls]
    # groups by brute force: flood fill over the undirected dependency graph
    adj = {c: set() for c in range(len(calls))}
    for c, call in enumerate(calls):
        for x in call.deps():
            adj[c].add(x)
            adj[x].add(c)
    seen, groups = set(), []
    for c in range(len(calls)):
        if c in seen:
            continue
        todo, g = [c], []
        while todo:
            v = todo.pop()
            if v in seen:
                continue
            seen.add(v)
            g.append(v)
            todo.extend(adj[v])
        groups.append(g)
    assert all(len({worker[c] for c in g}) == 1 for g in groups)
    load = [sum(cost[c] for c in range(len(calls)) if worker[c] == i) for i in range(n_workers)]
    biggest = max((sum(cost[c] for c in g) for g in groups), default=0)
    assert max(load) <= sum(cost) / n_workers + biggest
    assert O.partition_workflow(calls, n_workers) == worker
    assert set(O.partition_workflow(calls, 1)) <= {0}


def test_oracle_partition_closed_forms():
    """Equal groups go round the workers in turn; one heavy group and many light ones: the heavy one sits alone
    until the others have caught up (the textbook behaviour of largest-first list scheduling)."""
    w = wl.workflow_reflect(n_queries=6)
    worker = O.partition_workflow(calls_of(w), 3)
    assert [worker[3 * q] for q in range(6)] == [0, 1, 2, 0, 1, 2]
    h = wl.Workflow("one_heavy")
    big = h.add(h.fresh_tokens(1000), 10)                 # cost 10 * 1000 + 55
    small = [h.add(h.fresh_tokens(100), 10) for _ in range(8)]      # cost 1055 each
    worker = O.partition_workflow(calls_of(h), 2)
    assert worker[big] == 0 and all(worker[c] == 1 for c in small)
    with pytest.raises(ValueError):
        O.partition_workflow(calls_of(h), 0)


def test_oracle_nested_sequences_paper_figure():
    """The paragraph below the scheduling algorithm: operators that share a static system prompt form one
    inner sequence, inside which the calls run query by query (the question prompt stays cached between
    operator 2 and operator 3 of a query); an operator-by-operator order alternates between the queries'
    question prompts and prefills each of them once more.  Closed forms of the prefill usage of both orders."""
    n_q, sys_len, q_len, len_out = 4, 32, 16, 8
    w, ids = two_operator_example(n_q, sys_len, q_len, len_out)
    t = O.build_trt(calls_of(w))
    sigma, _, _, _ = O.cache_aware_schedule(t, 1, 1)      # short precedence delays: operator 1's outputs arrive in time
    nested = O.nested_sequences(t, sigma)
    fam_a = [i[0] for i in ids]
    fam_b = [c for i in ids for c in (i[1], i[2])]
    assert nested == [[fam_a, fam_b]], nested            # operator by operator across, query by query within
    up = lambda seq: sum(O.prefill_usage(t, seq[j - 1] if j else -1, c) for j, c in enumerate(seq))
    flat = fam_a + fam_b
    opwise = [i[k] for k in range(3) for i in ids]
    # family A: the system prompt once, a question per query; family B: the same plus operator 1's output
    # (len_out tokens) per query, operator 3 of a query reusing the question operator 2 has just prefilled
    assert up(flat) == (sys_len + n_q * q_len) + (sys_len + n_q * (q_len + len_out))
    # operator by operator every operator-3 call follows another query's call and prefills its question again
    assert up(opwise) == up(flat) + n_q * q_len


@pytest.mark.parametrize("seed", SEEDS)
def test_oracle_nested_sequences_invariants(seed):
    """A regrouping of each worker's order: every call once, on its worker; an inner sequence holds calls of one
    static prompt only, each static prompt of a worker appears in exactly one inner sequence, calls keep their
    relative order inside it, and sequences are released in the order of their last call."""
    w = wl.random_workflow(seed, n_calls=24, n_workers=2)
    t = O.build_trt(calls_of(w))
    sigma, _, _, _ = O.cache_aware_schedule(t, 2, 50)
    nested = O.nested_sequences(t, sigma)
    assert len(nested) == 2
    for i, (seq, inner) in enumerate(zip(sigma, nested)):
        assert sorted(c for s_ in inner for c in s_) == sorted(seq)
        fams = [{O.static_prompt_node(t, c) for c in s_} for s_ in inner]
        assert all(len(f) == 1 for f in fams)
        assert len({next(iter(f)) for f in fams}) == len(inner)
        pos = {c: j for j, c in enumerate(seq)}
        for s_ in inner:
            assert [pos[c] for c in s_] == sorted(pos[c] for c in s_)
        last = [max(pos[c] for c in s_) for s_ in inner]
        assert last == sorted(last)
    # the static prompt is the first node below the root: the common prefix of a family is at least that node's segment
    for c in range(w.n_calls):
        v = O.static_prompt_node(t, c)
        assert t.parent[v] == 0 and v in ([t.leaf_of_call[c]] + t.path(t.leaf_of_call[c]))


@pytest.mark.parametrize("seed", SEEDS)
def test_oracle_soft_execution_equals_the_evaluator_on_feasible_orders(seed):
    """Where the priority order respects the dependencies, best-effort execution runs it as it stands, and the
    evaluator (pinned above against longest paths) gives the same times."""
    w = wl.random_workflow(seed, n_calls=14, n_workers=2)
    t = O.build_trt(calls_of(w))
    sigma, B, C, T = O.cache_aware_schedule(t, 2, 40)
    assert O.run_soft_schedule(t, sigma, 40) == (sigma, B, C, T)


@pytest.mark.parametrize("make", [lambda: wl.workflow_debate(3, 3, 2), lambda: wl.workflow_debate(4, 2, 3, n_workers=2),
                                  lambda: wl.workflow_iterative(3, 4), lambda: wl.workflow_parallel(2, 3, 2),
                                  lambda: wl.random_workflow(5, n_calls=20, n_workers=2)])
def test_oracle_soft_execution_repairs_orders_the_dependencies_contradict(make):
    """Debate: agent A's second round needs B's first and the other way round, so inner sequences per agent
    cannot run back to back; the flattened nested order is infeasible as it stands (the evaluator rejects it or
    not), best-effort execution still runs every call once, on its worker, never before its inputs are there,
    one call at a time per worker, and what it reports agrees with the evaluator on the order it realised."""
    w = make()
    t = O.build_trt(calls_of(w))
    n_workers = max(w.worker) + 1
    sigma, _, _, _ = O.cache_aware_schedule(t, n_workers, 64)
    nested = O.nested_sequences(t, sigma)
    prio = [[c for seq in inner for c in seq] for inner in nested]
    real, B, C, T = O.run_soft_schedule(t, prio, 64)
    assert [sorted(s_) for s_ in real] == [sorted(s_) for s_ in prio]
    for c in range(w.n_calls):
        for x in t.deps[c]:
            assert B[c] >= C[x] + 64 * t.len_out[x]
    for seq in real:
        for a, b in zip(seq, seq[1:]):
            assert B[b] >= C[a]
    assert (B, C, T) == O.evaluate_schedule(t, real, 64)
    # a call is overtaken only by calls that could run: whenever a call ran before an earlier one of the
    # priority order, that earlier one still missed an input at that moment
    for i, seq in enumerate(real):
        pos = {c: j for j, c in enumerate(prio[i])}
        for j, c in enumerate(seq):
            for d in seq[j + 1:]:
                if pos[d] < pos[c]:
                    assert any(x not in seq[:j] and w.worker[x] == i or w.worker[x] != i for x in t.deps[d])


def test_oracle_soft_execution_worked_example():
    """Two calls A, B and a third that reads both, priority order [third, A, B] on one worker: the third waits;
    A and B run in order, then the third.  Times by hand (M = 10): A: 5 tokens, 2 out; B: 3 tokens, 1 out."""
    calls = [O.Call([-2, -3], 1), O.Call([1, 2, 3, 4, 5], 2), O.Call([7, 8, 9], 1)]
    t = O.build_trt(calls)
    real, B, C, T = O.run_soft_schedule(t, [[0, 1, 2]], 10)
    assert real == [[1, 2, 0]]
    # A: U = 2 * 5 + 3 = 13 -> [0, 13]; B: U = 1 * 3 + 1 = 4 -> [13, 17]; third: inputs at 13 + 20 and 17 + 10,
    # prompt = the two outputs (2 + 1 tokens), nothing shared with B: U = 1 * 3 + 1 = 4 -> [33, 37]
    assert (B[1], C[1], B[2], C[2], B[0], C[0], T) == (0, 13, 13, 17, 33, 37, 37)


# ------------------------------------------------------------------ library against the oracle

@pytest.fixture(scope="module")
def hkv():
    from paper_2603_16104_amd import binding
    binding.lib()
    return binding


def build_both(hkv, w):
    t = O.build_trt(calls_of(w))
    h = hkv.trt_build(w.templates, w.len_out, w.worker)
    return t, h


def workflows():
    ws = [wl.random_workflow(s, n_calls=16, n_workers=3) for s in range(10)]
    ws += [wl.random_workflow(100 + s, n_calls=40, vocab=3, max_len=14, n_workers=2) for s in range(4)]
    ws += [wl.workflow_map_reduce(n_workers=2), wl.workflow_debate(n_workers=2), wl.workflow_reflect(n_workers=1)]
    ws += [wl.workflow_debate(n_queries=5, n_agents=4, rounds=3, n_workers=3)]
    ws += [wl.workflow_iterative(n_workers=2), wl.workflow_parallel(n_workers=2), wl.workflow_parallel(5, 7, 6, n_workers=3)]
    e = wl.Workflow("empty")
    ws.append(e)
    one = wl.Workflow("one_empty_template")
    one.add([], 3)
    ws.append(one)
    return ws


@pytest.mark.parametrize("w", workflows(), ids=lambda w: w.name)
def test_library_tree_usage_evaluate_schedule_bit_exact(hkv, w):
    t, h = build_both(hkv, w)
    try:
        nd = hkv.trt_nodes(h)
        assert nd["parent"].tolist() == t.parent and nd["weight"].tolist() == t.weight
        assert nd["call"].tolist() == t.call and nd["leaf_of_call"].tolist() == t.leaf_of_call
        assert nd["seg_begin"].tolist() == t.seg_begin and nd["seg_len"].tolist() == t.seg_len
        assert nd["syms"].tolist() == t.syms
        n_workers = max(w.worker, default=0) + 1
        rng = np.random.default_rng(5)
        order = rng.permutation(w.n_calls).tolist()
        exp = [O.prefill_usage(t, order[j - 1] if j else -1, c) for j, c in enumerate(order)]
        assert hkv.trt_prefill_usage(h, order).tolist() == exp
        topo = O.topological_order(calls_of(w))
        sigma = [[c for c in topo if w.worker[c] == i] for i in range(n_workers)]
        for cap in (1, 37, 4096):
            B, C, T = O.evaluate_schedule(t, sigma, cap)
            gB, gC, gT = hkv.trt_evaluate(h, sigma, cap)
            assert (gB.tolist(), gC.tolist(), gT) == ([b for b in B], [c for c in C], T)
            s, B, C, T = O.cache_aware_schedule(t, n_workers, cap)
            gs, gB, gC, gT = hkv.trt_schedule(h, n_workers, cap)
            assert gs == s and gB.tolist() == B and gC.tolist() == C and gT == T
            # the nested form of that schedule and its best-effort execution
            nested = O.nested_sequences(t, s)
            assert hkv.trt_nested(h, s) == nested
            prio = [[c for seq in inner for c in seq] for inner in nested]
            rs, B, C, T = O.run_soft_schedule(t, prio, cap)
            gs, gB, gC, gT = hkv.trt_run_soft(h, prio, cap)
            assert gs == rs and gB.tolist() == B and gC.tolist() == C and gT == T
        # a priority order that ignores the dependencies altogether
        back = [[c for c in reversed(topo) if w.worker[c] == i] for i in range(n_workers)]
        rs, B, C, T = O.run_soft_schedule(t, back, 9)
        gs, gB, gC, gT = hkv.trt_run_soft(h, back, 9)
        assert gs == rs and gB.tolist() == B and gC.tolist() == C and gT == T
        for m in (1, 2, 3, 5):
            assert hkv.trt_partition(w.templates, w.len_out, m).tolist() == O.partition_workflow(calls_of(w), m)
    finally:
        hkv.trt_destroy(h)


def test_library_partition_then_schedule_end_to_end(hkv):
    """The whole procedure of the scheduling algorithm through the library: partition, tree, recursion, nested
    sequences, best-effort execution; two workers halve the total token step of a batch of independent queries
    (up to the imbalance of one query)."""
    w = wl.workflow_parallel(n_queries=6, n_experts=3, n_chunks=2)
    T = {}
    for m in (1, 2):
        worker = hkv.trt_partition(w.templates, w.len_out, m)
        h = hkv.trt_build(w.templates, w.len_out, worker)
        sigma, _, _, _ = hkv.trt_schedule(h, m, 64)
        prio = [[c for seq in inner for c in seq] for inner in hkv.trt_nested(h, sigma)]
        real, B, C, T[m] = hkv.trt_run_soft(h, prio, 64)
        assert sorted(c for s_ in real for c in s_) == list(range(w.n_calls))
        hkv.trt_destroy(h)
    assert T[2] < 0.62 * T[1]


def test_library_scheduling_errors(hkv):
    with pytest.raises(hkv.HkvError) as e:
        hkv.trt_build([[-2], [-1]], [1, 1])
    assert e.value.code == -4                                    # ETREE: cycle
    with pytest.raises(hkv.HkvError) as e:
        hkv.trt_build([[-5]], [1])
    assert e.value.code == -4                                    # ETREE: missing call
    with pytest.raises(hkv.HkvError) as e:
        hkv.trt_build([[1]], [-1])
    assert e.value.code == -2                                    # ERANGE
    with pytest.raises(hkv.HkvError) as e:
        hkv.trt_partition([[1], [-9]], [1, 1], 2)
    assert e.value.code == -2                                    # ERANGE: output of a call outside the batch
    with pytest.raises(hkv.HkvError) as e:
        hkv.trt_partition([[1]], [1], 0)
    assert e.value.code == -1
    h = hkv.trt_build([[1, 2], [3, -1]], [5, 1])
    try:
        assert hkv.trt_run_soft(h, [[1, 0]], 10)[0] == [[0, 1]]      # the order is repaired, not rejected
        for bad in ([[0]], [[0, 0]], [[0, 5]]):
            with pytest.raises(hkv.HkvError):
                hkv.trt_nested(h, bad)
            with pytest.raises(hkv.HkvError):
                hkv.trt_run_soft(h, bad, 10)
        with pytest.raises(hkv.HkvError) as e:
            hkv.trt_evaluate(h, [[1, 0]], 10)
        assert e.value.code == -4                                # contradicts the dependencies
        with pytest.raises(hkv.HkvError) as e:
            hkv.trt_evaluate(h, [[0, 0]], 10)
        assert e.value.code == -2                                # no partition
        with pytest.raises(hkv.HkvError) as e:
            hkv.trt_prefill_usage(h, [2])
        assert e.value.code == -2
    finally:
        hkv.trt_destroy(h)
