"""Plain-Python oracle for the templated radix tree, the token-step cost model and the
cache-aware scheduling heuristic.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and by nothing in the product package).  Slow and
obvious on purpose: lists, dicts, recursion; integers only.

What follows the paper
  * Section 5, "Modeling Prompt Structure with a Templated Radix Tree": T = (V, E, E'), internal
    nodes carry sequences of tokens and placeholders, each leaf is one LLM call whose prompt is the
    path from the root to its parent, E' are the dependencies among the leaves.
  * Appendix "Templated Radix Tree Construction" (the construction algorithm): calls are taken in
    topological order; each call's prefix template is inserted by standard radix-tree insertion
    (longest common prefix, node split where the template leaves an existing path); the call
    becomes a new leaf; its dependencies become edges to the leaves of the calls it reads.
  * Section 5, "Token usage" / "Precedence delay" / problem formulation: u_p, u_d, u, d, b, c, T.
  * Section 5, the scheduling algorithm (Schedule / Recurse) and the paragraph below it.

Readings taken where the paper is silent (the same ones the library takes)
  R1  A template is a list of integer symbols: s >= 0 is a static token id, s < 0 is a placeholder
      for the output of call -(s + 1).  omega(v) = number of static tokens of v's segment plus, for
      every placeholder, the estimated output length len_out of the call it stands for.
  R2  Workers are identical (alpha_i = 1 / M, one capacity M for all).  All times are kept as
      integers scaled by M:  U = len_out * u_p + u_d  (= M * u),  D = M * len_out  (= M * d).
  R3  A worker runs its calls one after another in schedule order: b(i, j) >= c(i, j - 1).
  R4  Node numbering of a finished tree: depth-first preorder from the root, children in order of
      creation (a node created by a split takes the place of the node it was split from).
  R5  The heuristic details of the scheduling algorithm (SelectChildren, CanSchedule, UpdateState)
      are only described in prose; the reading is written out at `cache_aware_schedule`.
      PARITY UNPINNED for those choices: the tests pin validity, determinism, agreement of the
      reported times with the evaluator, and the paper's three-call example, not optimality.
  R6  PartitionWorkflow (named in the algorithm, described in one sentence: operators are partitioned
      across the workers and replicated per assignment to balance load).  Reading: the calls of a batch
      fall into groups that share data (connected through dependencies: one group per input query of
      the batch); a group goes to one worker as a whole, so an operator is replicated on every worker
      that received one of its queries; groups are placed largest estimated token usage first, each on
      the worker with the least usage so far (ties: lower number).  Estimated usage of a call =
      len_out * omega(its whole prompt) + u_d (no sharing assumed).  Written out at `partition_workflow`.
      PARITY UNPINNED for the placement rule; the tests pin what any reading must satisfy (a partition,
      no dependency across workers, the greedy bound on the imbalance, closed forms).
  R7  Nested sequences (the paragraph below the algorithm): a worker's final schedule is a sequence of
      inner sequences; an inner sequence holds the calls of that worker that share their static prompt
      (the first node below the root on their path: the system prompt of an operator family), in the
      order in which the recursion emitted them (query by query, as the depth-first walk leaves them).
      The intermediate buffer collects emitted calls per static prompt and releases a family as one
      inner sequence when its last call on that worker has been emitted.  Written out at `nested_sequences`.
  R8  Soft schedule, best-effort execution: a worker that falls free issues the first call of its
      nested order whose inputs have all been issued (it may wait for them to arrive, but does not
      overtake within what can run), so an order that the dependencies contradict is repaired at run time
      instead of being rejected.  Written out at `run_soft_schedule`; on orders the dependencies allow
      it equals `evaluate_schedule`.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

INF = 1 << 62


class Call:
    """One LLM call: prefix template (R1), estimated output length, worker."""

    def __init__(self, template: Sequence[int], len_out: int, worker: int = 0):
        self.template = [int(s) for s in template]
        self.len_out = int(len_out)
        self.worker = int(worker)

    def deps(self) -> List[int]:
        """Calls whose output this call's prompt contains (direct dependencies, ascending, unique)."""
        return sorted({-(s + 1) for s in self.template if s < 0})


class Node:
    def __init__(self, syms: List[int], parent: Optional["Node"]):
        self.syms = syms            # segment of the template (empty for the root and for leaves)
        self.parent = parent
        self.children: List["Node"] = []
        self.call = -1              # leaf: index of its call
        self.idx = -1               # final number (R4)


class TRT:
    """Finished tree in flat form.  Node 0 is the root."""

    def __init__(self):
        self.parent: List[int] = []
        self.weight: List[int] = []       # omega
        self.call: List[int] = []         # call of a leaf, -1 otherwise
        self.seg_begin: List[int] = []    # segment = syms[seg_begin : seg_begin + seg_len]
        self.seg_len: List[int] = []
        self.syms: List[int] = []
        self.leaf_of_call: List[int] = []
        self.deps: List[List[int]] = []   # per call: direct dependencies (calls)
        self.len_out: List[int] = []
        self.worker: List[int] = []

    @property
    def n_nodes(self) -> int:
        return len(self.parent)

    @property
    def n_calls(self) -> int:
        return len(self.leaf_of_call)

    def children(self, v: int) -> List[int]:
        return [c for c in range(self.n_nodes) if self.parent[c] == v]

    def path(self, v: int) -> List[int]:
        """Nodes from the root (exclusive) to v (inclusive)."""
        out = []
        while v > 0:
            out.append(v)
            v = self.parent[v]
        return out[::-1]


def topological_order(calls: Sequence[Call]) -> List[int]:
    """Dependencies before dependents; among the ready calls the smallest index first."""
    n = len(calls)
    deps = [c.deps() for c in calls]
    for i, d in enumerate(deps):
        for x in d:
            if x < 0 or x >= n or x == i:
                raise ValueError(f"call {i} reads call {x}")
    done, order = [False] * n, []
    while len(order) < n:
        for i in range(n):
            if not done[i] and all(done[x] for x in deps[i]):
                done[i] = True
                order.append(i)
                break
        else:
            raise ValueError("dependency cycle")
    return order


def build_trt(calls: Sequence[Call]) -> TRT:
    """Radix-tree insertion of every call's template, in topological order."""
    root = Node([], None)
    leaves: Dict[int, Node] = {}
    for ci in topological_order(calls):
        tmpl = calls[ci].template
        node, pos = root, 0
        while pos < len(tmpl):
            nxt = None
            for ch in node.children:
                if ch.call < 0 and ch.syms[0] == tmpl[pos]:
                    nxt = ch
                    break
            if nxt is None:                       # nothing shares the next symbol: new branch with the rest
                nxt = Node(list(tmpl[pos:]), node)
                node.children.append(nxt)
                node, pos = nxt, len(tmpl)
                break
            k = 0                                 # common prefix of the remaining template and nxt's segment
            while k < len(nxt.syms) and pos + k < len(tmpl) and nxt.syms[k] == tmpl[pos + k]:
                k += 1
            if k < len(nxt.syms):                 # the template leaves the path inside nxt: split it
                upper = Node(nxt.syms[:k], node)
                node.children[node.children.index(nxt)] = upper
                nxt.syms = nxt.syms[k:]
                nxt.parent = upper
                upper.children.append(nxt)
                nxt = upper
            node, pos = nxt, pos + k
        leaf = Node([], node)
        leaf.call = ci
        node.children.append(leaf)
        leaves[ci] = leaf

    t = TRT()
    stack = [root]
    while stack:                                   # preorder, children in creation order (R4)
        v = stack.pop()
        v.idx = len(t.parent)
        t.parent.append(v.parent.idx if v.parent else -1)
        w = 0
        for s in v.syms:
            w += 1 if s >= 0 else calls[-(s + 1)].len_out
        t.weight.append(w)
        t.call.append(v.call)
        t.seg_begin.append(len(t.syms))
        t.seg_len.append(len(v.syms))
        t.syms.extend(v.syms)
        stack.extend(reversed(v.children))
    t.leaf_of_call = [leaves[i].idx for i in range(len(calls))]
    t.deps = [c.deps() for c in calls]
    t.len_out = [c.len_out for c in calls]
    t.worker = [c.worker for c in calls]
    return t


# ---------------------------------------------------------------------------------------------
# cost model


def prefill_usage(t: TRT, prev_call: int, call: int) -> int:
    """u_p: omega over path(r, l) for a worker's first call (prev_call < 0), else over the path from
    the lowest common ancestor of the two leaves (exclusive) down to the call's leaf."""
    p = t.path(t.leaf_of_call[call])
    if prev_call < 0:
        return sum(t.weight[v] for v in p)
    q = set(t.path(t.leaf_of_call[prev_call]))
    return sum(t.weight[v] for v in p if v not in q)


def decode_usage(len_out: int) -> int:
    """u_d = len_out (len_out + 1) / 2."""
    return len_out * (len_out + 1) // 2


def evaluate_schedule(t: TRT, sigma: Sequence[Sequence[int]], capacity: int):
    """Earliest start and completion of every call under the schedule sigma (one sequence of calls
    per worker) and the total token step, all scaled by M = capacity (R2):
        U = len_out * u_p + u_d,  C = B + U,  B >= C' + M * len_out' for every dependency,  (R3).
    Returns (B, C, T) with B, C indexed by call; raises if sigma is no partition of the calls or
    contradicts the dependencies."""
    n = t.n_calls
    seen = sorted(c for seq in sigma for c in seq)
    if seen != list(range(n)):
        raise ValueError("sigma is not a partition of the calls")
    B, Cc = [None] * n, [None] * n
    pos = [0] * len(sigma)
    free = [0] * len(sigma)
    remaining = n
    while remaining:
        progressed = False
        for i, seq in enumerate(sigma):
            while pos[i] < len(seq):
                c = seq[pos[i]]
                if any(Cc[x] is None for x in t.deps[c]):
                    break
                b = free[i]
                for x in t.deps[c]:
                    b = max(b, Cc[x] + capacity * t.len_out[x])
                prev = seq[pos[i] - 1] if pos[i] else -1
                U = t.len_out[c] * prefill_usage(t, prev, c) + decode_usage(t.len_out[c])
                B[c], Cc[c] = b, b + U
                free[i] = Cc[c]
                pos[i] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise ValueError("sigma contradicts the dependencies")
    return B, Cc, max(Cc) if n else 0


# ---------------------------------------------------------------------------------------------
# scheduling heuristic (R5)


def cache_aware_schedule(t: TRT, n_workers: int, capacity: int):
    """The Schedule / Recurse procedure on the call-level tree.

    State: per worker the sequence so far and the token step at which it falls free; per call
    whether it is scheduled and its completion.  A call is READY when all its dependencies are
    scheduled; its earliest start est is the larger of its worker's free step and, over its
    dependencies, completion + precedence delay.
      CanSchedule(leaf, force)  READY and (force or est == the worker's free step), i.e. without
                                force a call is only placed where it opens no idle gap.
      ScheduleNode(leaf)        append to its worker at est; U uses u_p against that worker's
                                previous call.
      SelectChildren(node, f)   the node's remaining children ordered by
                                  without force: greatest aggregated dependency depth first, then
                                                 earliest schedulable step, then node number;
                                  with force:    earliest schedulable step first, then depth, then
                                                 number (the blocked call with the earliest start
                                                 goes first).
                                Aggregated dependency depth of a subtree = the largest, over its
                                unscheduled leaves, of the number of calls on the longest chain of
                                dependents hanging off the leaf (critical-path length in G).
                                Earliest schedulable step = the smallest est among its READY
                                unscheduled leaves (infinite if none).
      UpdateState               the two keys are recomputed from the current state each time a
                                node's children are ordered (nothing is cached).
    The order of a node's children is fixed when the node is entered; `force` applies to the first
    child only.  Returns (sigma, B, C, T)."""
    n = t.n_calls
    kids = [t.children(v) for v in range(t.n_nodes)]
    dependents = [[] for _ in range(n)]
    for c in range(n):
        for x in t.deps[c]:
            dependents[x].append(c)
    chain = [0] * n                                  # calls on the longest chain of dependents below c
    for c in reversed(topological_order_of_deps(t.deps)):
        chain[c] = 1 + max((chain[y] for y in dependents[c]), default=0)

    done = [False] * n
    B, Cc = [0] * n, [0] * n
    sigma: List[List[int]] = [[] for _ in range(n_workers)]
    free = [0] * n_workers
    removed = [False] * t.n_nodes

    def ready(c):
        return not done[c] and all(done[x] for x in t.deps[c])

    def est(c):
        b = free[t.worker[c]]
        for x in t.deps[c]:
            b = max(b, Cc[x] + capacity * t.len_out[x])
        return b

    def leaves_below(v):
        if t.call[v] >= 0:
            return [] if removed[v] else [t.call[v]]
        out = []
        for ch in kids[v]:
            if not removed[ch]:
                out.extend(leaves_below(ch))
        return out

    def keys(v):
        ls = leaves_below(v)
        depth = max((chain[c] for c in ls), default=0)
        early = min((est(c) for c in ls if ready(c)), default=INF)
        return depth, early

    def recurse(v, force):
        if t.call[v] >= 0:
            c = t.call[v]
            if ready(c) and (force or est(c) == free[t.worker[c]]):
                w = t.worker[c]
                prev = sigma[w][-1] if sigma[w] else -1
                B[c] = est(c)
                Cc[c] = B[c] + t.len_out[c] * prefill_usage(t, prev, c) + decode_usage(t.len_out[c])
                free[w] = Cc[c]
                sigma[w].append(c)
                done[c] = True
                return True
            return False
        live = [ch for ch in kids[v] if not removed[ch]]
        if force:
            live.sort(key=lambda ch: (keys(ch)[1], -keys(ch)[0], ch))
        else:
            live.sort(key=lambda ch: (-keys(ch)[0], keys(ch)[1], ch))
        for ch in live:
            if recurse(ch, force):
                removed[ch] = True
            force = False
        return all(removed[ch] for ch in kids[v])

    while not recurse(0, False):
        recurse(0, True)
    return sigma, B, Cc, (max(Cc) if n else 0)


def topological_order_of_deps(deps: Sequence[Sequence[int]]) -> List[int]:
    n = len(deps)
    done, order = [False] * n, []
    while len(order) < n:
        for i in range(n):
            if not done[i] and all(done[x] for x in deps[i]):
                done[i] = True
                order.append(i)
                break
        else:
            raise ValueError("dependency cycle")
    return order


# ---------------------------------------------------------------------------------------------
# PartitionWorkflow (R6), nested sequences (R7), best-effort execution of a soft schedule (R8)


def partition_workflow(calls: Sequence[Call], n_workers: int) -> List[int]:
    """Worker of every call.  Groups = connected components of the dependency graph; cost of a group =
    sum over its calls of len_out * omega(prompt) + u_d with omega as in R1; groups in order of
    decreasing cost (ties: smaller first call) each go to the worker with the least cost so far
    (ties: lower number)."""
    n = len(calls)
    if n_workers < 1:
        raise ValueError("n_workers")
    comp = list(range(n))

    def find(x):
        while comp[x] != x:
            x = comp[x]
        return x

    for c in range(n):
        for x in calls[c].deps():
            if not 0 <= x < n:
                raise ValueError("dependency outside the batch")
            a, b = find(c), find(x)
            if a != b:
                comp[max(a, b)] = min(a, b)
    cost = [0] * n
    for c in range(n):
        omega = sum(1 if sym >= 0 else calls[-(sym + 1)].len_out for sym in calls[c].template)
        cost[c] = calls[c].len_out * omega + decode_usage(calls[c].len_out)
    groups: Dict[int, List[int]] = {}
    for c in range(n):
        groups.setdefault(find(c), []).append(c)
    order = sorted(groups, key=lambda g: (-sum(cost[c] for c in groups[g]), g))
    load = [0] * n_workers
    worker = [0] * n
    for g in order:
        w = min(range(n_workers), key=lambda i: (load[i], i))
        for c in groups[g]:
            worker[c] = w
        load[w] += sum(cost[c] for c in groups[g])
    return worker


def static_prompt_node(t: TRT, call: int) -> int:
    """The first node below the root on the call's path (its leaf itself for an empty prompt)."""
    v = t.leaf_of_call[call]
    while t.parent[v] > 0:
        v = t.parent[v]
    return v


def nested_sequences(t: TRT, sigma: Sequence[Sequence[int]]) -> List[List[List[int]]]:
    """Per worker the inner sequences in the order in which the buffer releases them (R7)."""
    out: List[List[List[int]]] = []
    for seq in sigma:
        total: Dict[int, int] = {}
        for c in seq:
            g = static_prompt_node(t, c)
            total[g] = total.get(g, 0) + 1
        buffer: Dict[int, List[int]] = {}
        released: List[List[int]] = []
        for c in seq:
            g = static_prompt_node(t, c)
            buffer.setdefault(g, []).append(c)
            if len(buffer[g]) == total[g]:
                released.append(buffer.pop(g))
        out.append(released)
    return out


def run_soft_schedule(t: TRT, order: Sequence[Sequence[int]], capacity: int):
    """Best-effort execution of per-worker priority orders (the flattened nested sequences) under the cost
    model (R8).  Repeatedly: every worker with calls left names the first call of its order whose
    dependencies have all been issued; its start would be the larger of the worker's free step and, over the
    dependencies, completion + precedence delay; the worker whose candidate starts earliest (ties: lower
    number) issues it.  Returns (sigma, B, C, T): the order in which each worker ran its calls, start and
    completion per call, total token step (scaled by M as in evaluate_schedule)."""
    n = t.n_calls
    if sorted(c for seq in order for c in seq) != list(range(n)):
        raise ValueError("the orders are no partition of the calls")
    issued = [False] * n
    B, Cc = [0] * n, [0] * n
    left = [list(seq) for seq in order]
    sigma: List[List[int]] = [[] for _ in order]
    free = [0] * len(order)
    for _ in range(n):
        best = None
        for w, seq in enumerate(left):
            cand = next((c for c in seq if all(issued[x] for x in t.deps[c])), None)
            if cand is None:
                continue
            b = free[w]
            for x in t.deps[cand]:
                b = max(b, Cc[x] + capacity * t.len_out[x])
            if best is None or b < best[0]:
                best = (b, w, cand)
        if best is None:
            raise ValueError("dependency cycle")
        b, w, c = best
        prev = sigma[w][-1] if sigma[w] else -1
        B[c] = b
        Cc[c] = b + t.len_out[c] * prefill_usage(t, prev, c) + decode_usage(t.len_out[c])
        free[w] = Cc[c]
        issued[c] = True
        sigma[w].append(c)
        left[w].remove(c)
    return sigma, B, Cc, (max(Cc) if n else 0)
