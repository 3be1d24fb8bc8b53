// Host side of the scheduling layer: templated radix tree over prompt templates, the token-step
// cost model and the cache-aware scheduling procedure (Section 5: "Modeling Prompt Structure with
// a Templated Radix Tree", "Scheduling Problem Formulation", "Solver by Cache-Aware Scheduling";
// appendix "Templated Radix Tree Construction").  Integer arithmetic only; nothing here touches
// the device.  The tree it produces is the prefix forest the attention entry points consume: an
// internal node's omega is its n_tokens, a scheduled call sequence says which suffix each prefill
// call has to process (u_p).
#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/heliumkv.h"

namespace hkv {
int fail(int code, const char *fmt, ...);  // api.cpp: records the thread-local message, returns code
}
using hkv::fail;

struct hkv_trt {
    // flat tree, node 0 = root, numbered in depth-first preorder, children in order of creation
    std::vector<int32_t> parent, call, seg_begin, seg_len, syms, depth;
    std::vector<int64_t> weight;
    std::vector<std::vector<int32_t>> kids;
    // calls
    std::vector<int32_t> leaf_of_call, len_out, worker;
    std::vector<std::vector<int32_t>> deps, dependents;
    std::vector<int32_t> topo;   // dependencies first, smallest index first among the ready ones
    std::vector<int32_t> chain;  // calls on the longest chain of dependents starting at the call
};

namespace {

constexpr int64_t kInf = (int64_t)1 << 62;

struct BuildNode {
    std::vector<int32_t> syms;
    int32_t parent = -1;
    std::vector<int32_t> kids;
    int32_t call = -1;
};

// dependencies before dependents; among the ready calls the smallest index first
bool topological(const std::vector<std::vector<int32_t>> &deps, std::vector<int32_t> &order) {
    const int n = (int)deps.size();
    std::vector<char> done(n, 0);
    order.clear();
    while ((int)order.size() < n) {
        int pick = -1;
        for (int i = 0; i < n && pick < 0; ++i) {
            if (done[i]) continue;
            bool ok = true;
            for (int x : deps[i]) ok = ok && done[x];
            if (ok) pick = i;
        }
        if (pick < 0) return false;
        done[pick] = 1;
        order.push_back(pick);
    }
    return true;
}

// omega over the nodes of path(root, leaf of `call`) that are not on path(root, leaf of `prev`)
int64_t usage_between(const hkv_trt &t, int32_t prev, int32_t call) {
    int a = t.leaf_of_call[call];
    int b = prev >= 0 ? t.leaf_of_call[prev] : 0;
    // lift the deeper one, then both: the meeting point is the lowest common ancestor (root if prev < 0)
    int x = a, y = b;
    while (t.depth[x] > t.depth[y]) x = t.parent[x];
    while (t.depth[y] > t.depth[x]) y = t.parent[y];
    while (x != y) {
        x = t.parent[x];
        y = t.parent[y];
    }
    int64_t s = 0;
    for (int v = a; v != x; v = t.parent[v]) s += t.weight[v];
    return s;
}

int64_t call_usage(const hkv_trt &t, int32_t prev, int32_t c) {
    const int64_t lo = t.len_out[c];
    return lo * usage_between(t, prev, c) + lo * (lo + 1) / 2;
}

}  // namespace

extern "C" int trt_build(const int32_t *tmpl_indptr, const int32_t *tmpl_syms, const int32_t *len_out,
                         const int32_t *worker, int32_t n_calls, hkv_trt **out) {
    if (!out) return fail(HKV_EINVAL, "trt_build: null out");
    *out = nullptr;
    if (n_calls < 0 || (n_calls > 0 && (!tmpl_indptr || !len_out))) return fail(HKV_EINVAL, "trt_build: null argument");
    if (n_calls > 0 && tmpl_indptr[0] != 0) return fail(HKV_EINVAL, "trt_build: tmpl_indptr[0] must be 0");
    for (int i = 0; i < n_calls; ++i) {
        if (tmpl_indptr[i + 1] < tmpl_indptr[i]) return fail(HKV_EINVAL, "trt_build: tmpl_indptr decreases at call %d", i);
        if (len_out[i] < 0) return fail(HKV_ERANGE, "trt_build: call %d has negative output length", i);
        if (worker && worker[i] < 0) return fail(HKV_ERANGE, "trt_build: call %d has negative worker", i);
    }
    if (n_calls > 0 && tmpl_indptr[n_calls] > 0 && !tmpl_syms) return fail(HKV_EINVAL, "trt_build: null tmpl_syms");
    hkv_trt *t = new (std::nothrow) hkv_trt;
    if (!t) return fail(HKV_ENOMEM, "trt_build: out of host memory");
    t->len_out.assign(len_out, len_out + n_calls);
    t->worker.assign(n_calls, 0);
    if (worker) t->worker.assign(worker, worker + n_calls);
    t->deps.resize(n_calls);
    t->dependents.resize(n_calls);
    for (int i = 0; i < n_calls; ++i) {
        for (int p = tmpl_indptr[i]; p < tmpl_indptr[i + 1]; ++p) {
            const int32_t s = tmpl_syms[p];
            if (s >= 0) continue;
            const int64_t src = -((int64_t)s + 1);
            if (src >= n_calls || src == i) {
                delete t;
                return fail(HKV_ETREE, "trt_build: call %d reads the output of call %lld", i, (long long)src);
            }
            t->deps[i].push_back((int32_t)src);
        }
        std::sort(t->deps[i].begin(), t->deps[i].end());
        t->deps[i].erase(std::unique(t->deps[i].begin(), t->deps[i].end()), t->deps[i].end());
    }
    if (!topological(t->deps, t->topo)) {
        delete t;
        return fail(HKV_ETREE, "trt_build: the calls' dependencies form a cycle");
    }
    for (int i = 0; i < n_calls; ++i)
        for (int x : t->deps[i]) t->dependents[x].push_back(i);
    t->chain.assign(n_calls, 0);
    for (int k = n_calls - 1; k >= 0; --k) {
        const int c = t->topo[k];
        int best = 0;
        for (int y : t->dependents[c]) best = std::max(best, t->chain[y]);
        t->chain[c] = 1 + best;
    }

    // radix insertion in topological order
    std::vector<BuildNode> nodes(1);
    std::vector<int32_t> leaf(n_calls, -1);
    for (int ci : t->topo) {
        const int32_t *tm = tmpl_syms + tmpl_indptr[ci];
        const int len = tmpl_indptr[ci + 1] - tmpl_indptr[ci];
        int node = 0, pos = 0;
        while (pos < len) {
            int nxt = -1;
            for (int ch : nodes[node].kids)
                if (nodes[ch].call < 0 && nodes[ch].syms[0] == tm[pos]) {
                    nxt = ch;
                    break;
                }
            if (nxt < 0) {  // nothing shares the next symbol: one new node with the rest
                BuildNode b;
                b.syms.assign(tm + pos, tm + len);
                b.parent = node;
                nodes.push_back(b);
                nxt = (int)nodes.size() - 1;
                nodes[node].kids.push_back(nxt);
                node = nxt;
                pos = len;
                break;
            }
            int k = 0;
            const int seg = (int)nodes[nxt].syms.size();
            while (k < seg && pos + k < len && nodes[nxt].syms[k] == tm[pos + k]) ++k;
            if (k < seg) {  // the template leaves the path inside nxt: split, the upper part takes nxt's place
                BuildNode up;
                up.syms.assign(nodes[nxt].syms.begin(), nodes[nxt].syms.begin() + k);
                up.parent = node;
                up.kids.push_back(nxt);
                nodes.push_back(up);
                const int upi = (int)nodes.size() - 1;
                *std::find(nodes[node].kids.begin(), nodes[node].kids.end(), nxt) = upi;
                nodes[nxt].syms.erase(nodes[nxt].syms.begin(), nodes[nxt].syms.begin() + k);
                nodes[nxt].parent = upi;
                nxt = upi;
            }
            node = nxt;
            pos += k;
        }
        BuildNode lf;
        lf.parent = node;
        lf.call = ci;
        nodes.push_back(lf);
        leaf[ci] = (int)nodes.size() - 1;
        nodes[node].kids.push_back(leaf[ci]);
    }

    // flatten: preorder, children in creation order
    const int n_nodes = (int)nodes.size();
    std::vector<int32_t> number(n_nodes, -1), stack{0};
    t->leaf_of_call.assign(n_calls, -1);
    while (!stack.empty()) {
        const int v = stack.back();
        stack.pop_back();
        const int id = (int)t->parent.size();
        number[v] = id;
        const int par = nodes[v].parent >= 0 ? number[nodes[v].parent] : -1;
        t->parent.push_back(par);
        t->depth.push_back(par >= 0 ? t->depth[par] + 1 : 0);
        int64_t w = 0;
        for (int32_t s : nodes[v].syms) w += s >= 0 ? 1 : t->len_out[-((int64_t)s + 1)];
        t->weight.push_back(w);
        t->call.push_back(nodes[v].call);
        t->seg_begin.push_back((int32_t)t->syms.size());
        t->seg_len.push_back((int32_t)nodes[v].syms.size());
        t->syms.insert(t->syms.end(), nodes[v].syms.begin(), nodes[v].syms.end());
        if (nodes[v].call >= 0) t->leaf_of_call[nodes[v].call] = id;
        for (auto it = nodes[v].kids.rbegin(); it != nodes[v].kids.rend(); ++it) stack.push_back(*it);
    }
    t->kids.resize(n_nodes);
    for (int v = 1; v < n_nodes; ++v) t->kids[t->parent[v]].push_back(v);  // ascending = creation order in preorder
    *out = t;
    return HKV_OK;
}

extern "C" int trt_destroy(hkv_trt *t) {
    delete t;
    return HKV_OK;
}

extern "C" int32_t trt_num_nodes(const hkv_trt *t) { return t ? (int32_t)t->parent.size() : fail(HKV_EINVAL, "null tree"); }
extern "C" int32_t trt_num_syms(const hkv_trt *t) { return t ? (int32_t)t->syms.size() : fail(HKV_EINVAL, "null tree"); }
extern "C" int32_t trt_num_calls(const hkv_trt *t) { return t ? (int32_t)t->len_out.size() : fail(HKV_EINVAL, "null tree"); }

extern "C" int trt_nodes(const hkv_trt *t, int32_t *parent, int64_t *weight, int32_t *call, int32_t *seg_begin,
                         int32_t *seg_len, int32_t *syms, int32_t *leaf_of_call) {
    if (!t) return fail(HKV_EINVAL, "trt_nodes: null tree");
    const size_t n = t->parent.size();
    if (parent) memcpy(parent, t->parent.data(), n * sizeof(int32_t));
    if (weight) memcpy(weight, t->weight.data(), n * sizeof(int64_t));
    if (call) memcpy(call, t->call.data(), n * sizeof(int32_t));
    if (seg_begin) memcpy(seg_begin, t->seg_begin.data(), n * sizeof(int32_t));
    if (seg_len) memcpy(seg_len, t->seg_len.data(), n * sizeof(int32_t));
    if (syms && !t->syms.empty()) memcpy(syms, t->syms.data(), t->syms.size() * sizeof(int32_t));
    if (leaf_of_call && !t->leaf_of_call.empty())
        memcpy(leaf_of_call, t->leaf_of_call.data(), t->leaf_of_call.size() * sizeof(int32_t));
    return HKV_OK;
}

extern "C" int trt_prefill_usage(const hkv_trt *t, const int32_t *calls, int32_t n, int64_t *u_p) {
    if (!t || (n > 0 && (!calls || !u_p))) return fail(HKV_EINVAL, "trt_prefill_usage: null argument");
    const int nc = (int)t->len_out.size();
    for (int j = 0; j < n; ++j) {
        if (calls[j] < 0 || calls[j] >= nc) return fail(HKV_ERANGE, "trt_prefill_usage: calls[%d] = %d", j, calls[j]);
        u_p[j] = usage_between(*t, j ? calls[j - 1] : -1, calls[j]);
    }
    return HKV_OK;
}

extern "C" int trt_evaluate(const hkv_trt *t, const int32_t *sigma_indptr, const int32_t *sigma, int32_t n_workers,
                            int64_t capacity, int64_t *B, int64_t *C, int64_t *T) {
    if (!t || !sigma_indptr || !T || n_workers < 1 || capacity < 1) return fail(HKV_EINVAL, "trt_evaluate: bad argument");
    const int n = (int)t->len_out.size();
    if (sigma_indptr[0] != 0 || sigma_indptr[n_workers] != n) return fail(HKV_EINVAL, "trt_evaluate: sigma does not hold %d calls", n);
    if (n > 0 && !sigma) return fail(HKV_EINVAL, "trt_evaluate: null sigma");
    std::vector<char> seen(n, 0);
    for (int i = 0; i < n_workers; ++i)
        if (sigma_indptr[i + 1] < sigma_indptr[i]) return fail(HKV_EINVAL, "trt_evaluate: sigma_indptr decreases");
    for (int k = 0; k < n; ++k) {
        if (sigma[k] < 0 || sigma[k] >= n || seen[sigma[k]]) return fail(HKV_ERANGE, "trt_evaluate: sigma is no partition of the calls (entry %d)", k);
        seen[sigma[k]] = 1;
    }
    std::vector<int64_t> b(n, -1), c(n, -1), free_at(n_workers, 0);
    std::vector<int32_t> pos(sigma_indptr, sigma_indptr + n_workers);
    int remaining = n;
    while (remaining) {
        bool progressed = false;
        for (int i = 0; i < n_workers; ++i) {
            while (pos[i] < sigma_indptr[i + 1]) {
                const int cl = sigma[pos[i]];
                bool ok = true;
                for (int x : t->deps[cl]) ok = ok && c[x] >= 0;
                if (!ok) break;
                int64_t st = free_at[i];
                for (int x : t->deps[cl]) st = std::max(st, c[x] + capacity * t->len_out[x]);
                const int prev = pos[i] > sigma_indptr[i] ? sigma[pos[i] - 1] : -1;
                b[cl] = st;
                c[cl] = st + call_usage(*t, prev, cl);
                free_at[i] = c[cl];
                ++pos[i];
                --remaining;
                progressed = true;
            }
        }
        if (!progressed) return fail(HKV_ETREE, "trt_evaluate: the schedule contradicts the dependencies");
    }
    int64_t mx = 0;
    for (int k = 0; k < n; ++k) mx = std::max(mx, c[k]);
    if (B && n) memcpy(B, b.data(), n * sizeof(int64_t));
    if (C && n) memcpy(C, c.data(), n * sizeof(int64_t));
    *T = mx;
    return HKV_OK;
}

namespace {

struct Scheduler {
    const hkv_trt &t;
    int64_t capacity;
    std::vector<char> done, removed;
    std::vector<int64_t> B, C, free_at;
    std::vector<std::vector<int32_t>> sigma;

    bool ready(int c) const {
        if (done[c]) return false;
        for (int x : t.deps[c])
            if (!done[x]) return false;
        return true;
    }
    int64_t est(int c) const {
        int64_t b = free_at[t.worker[c]];
        for (int x : t.deps[c]) b = std::max(b, C[x] + capacity * t.len_out[x]);
        return b;
    }
    // (aggregated dependency depth, earliest schedulable step) of the unscheduled leaves below v
    void keys(int v, int &depth, int64_t &early) const {
        if (t.call[v] >= 0) {
            if (removed[v]) return;
            const int c = t.call[v];
            depth = std::max(depth, t.chain[c]);
            if (ready(c)) early = std::min(early, est(c));
            return;
        }
        for (int ch : t.kids[v])
            if (!removed[ch]) keys(ch, depth, early);
    }
    bool recurse(int v, bool force) {
        if (t.call[v] >= 0) {
            const int c = t.call[v];
            if (ready(c) && (force || est(c) == free_at[t.worker[c]])) {
                const int w = t.worker[c];
                const int prev = sigma[w].empty() ? -1 : sigma[w].back();
                B[c] = est(c);
                C[c] = B[c] + call_usage(t, prev, c);
                free_at[w] = C[c];
                sigma[w].push_back(c);
                done[c] = 1;
                return true;
            }
            return false;
        }
        struct Key {
            int depth;
            int64_t early;
            int node;
        };
        std::vector<Key> live;
        for (int ch : t.kids[v]) {
            if (removed[ch]) continue;
            Key k{0, kInf, ch};
            keys(ch, k.depth, k.early);
            live.push_back(k);
        }
        if (force)
            std::sort(live.begin(), live.end(), [](const Key &a, const Key &b) {
                if (a.early != b.early) return a.early < b.early;
                if (a.depth != b.depth) return a.depth > b.depth;
                return a.node < b.node;
            });
        else
            std::sort(live.begin(), live.end(), [](const Key &a, const Key &b) {
                if (a.depth != b.depth) return a.depth > b.depth;
                if (a.early != b.early) return a.early < b.early;
                return a.node < b.node;
            });
        for (const Key &k : live) {
            if (recurse(k.node, force)) removed[k.node] = 1;
            force = false;
        }
        for (int ch : t.kids[v])
            if (!removed[ch]) return false;
        return true;
    }
};

}  // namespace

extern "C" int trt_schedule(const hkv_trt *t, int32_t n_workers, int64_t capacity, int32_t *sigma_indptr,
                            int32_t *sigma, int64_t *B, int64_t *C, int64_t *T) {
    if (!t || !sigma_indptr || !T || n_workers < 1 || capacity < 1) return fail(HKV_EINVAL, "trt_schedule: bad argument");
    const int n = (int)t->len_out.size();
    if (n > 0 && !sigma) return fail(HKV_EINVAL, "trt_schedule: null sigma");
    for (int c = 0; c < n; ++c)
        if (t->worker[c] >= n_workers) return fail(HKV_ERANGE, "trt_schedule: call %d sits on worker %d of %d", c, t->worker[c], n_workers);
    Scheduler s{*t, capacity, std::vector<char>(n, 0), std::vector<char>(t->parent.size(), 0), std::vector<int64_t>(n, 0),
                std::vector<int64_t>(n, 0), std::vector<int64_t>(n_workers, 0), std::vector<std::vector<int32_t>>(n_workers)};
    while (!s.recurse(0, false)) s.recurse(0, true);
    int64_t mx = 0;
    sigma_indptr[0] = 0;
    for (int i = 0; i < n_workers; ++i) {
        if (!s.sigma[i].empty()) memcpy(sigma + sigma_indptr[i], s.sigma[i].data(), s.sigma[i].size() * sizeof(int32_t));
        sigma_indptr[i + 1] = sigma_indptr[i] + (int32_t)s.sigma[i].size();
    }
    for (int c = 0; c < n; ++c) mx = std::max(mx, s.C[c]);
    if (B && n) memcpy(B, s.B.data(), n * sizeof(int64_t));
    if (C && n) memcpy(C, s.C.data(), n * sizeof(int64_t));
    *T = mx;
    return HKV_OK;
}

// ---------------------------------------------------------------------------------------------
// PartitionWorkflow, nested sequences, best-effort execution of a soft schedule (Section 5, the
// scheduling algorithm and the paragraph below it; the paper names these steps and describes them in
// prose, the rules taken here are stated at each function)

// Groups of calls connected by dependencies (one per input query of a batch) go to one worker as a whole,
// largest estimated token usage first, each to the worker with the least usage so far (ties: lower number).
// Estimated usage of a call: len_out * omega(prompt) + len_out (len_out + 1) / 2, omega counting a static
// token as 1 and a placeholder as the output length of the call it stands for.
extern "C" int trt_partition(const int32_t *tmpl_indptr, const int32_t *tmpl_syms, const int32_t *len_out, int32_t n_calls,
                             int32_t n_workers, int32_t *worker) {
    if (n_calls < 0 || n_workers < 1 || (n_calls > 0 && (!tmpl_indptr || !len_out || !worker)))
        return fail(HKV_EINVAL, "trt_partition: bad argument");
    if (n_calls > 0 && tmpl_indptr[0] != 0) return fail(HKV_EINVAL, "trt_partition: tmpl_indptr[0] must be 0");
    const int n = n_calls;
    std::vector<int32_t> comp(n);
    for (int c = 0; c < n; ++c) comp[c] = c;
    auto find = [&](int x) {
        while (comp[x] != x) x = comp[x];
        return x;
    };
    std::vector<int64_t> cost(n, 0);
    for (int c = 0; c < n; ++c) {
        if (tmpl_indptr[c + 1] < tmpl_indptr[c]) return fail(HKV_EINVAL, "trt_partition: tmpl_indptr decreases at call %d", c);
        if (len_out[c] < 0) return fail(HKV_ERANGE, "trt_partition: call %d has negative output length", c);
        if (tmpl_indptr[c + 1] > tmpl_indptr[c] && !tmpl_syms) return fail(HKV_EINVAL, "trt_partition: null tmpl_syms");
    }
    for (int c = 0; c < n; ++c) {
        int64_t omega = 0;
        for (int k = tmpl_indptr[c]; k < tmpl_indptr[c + 1]; ++k) {
            const int32_t s = tmpl_syms[k];
            if (s >= 0) {
                ++omega;
                continue;
            }
            const int64_t x = -((int64_t)s + 1);
            if (x >= n) return fail(HKV_ERANGE, "trt_partition: call %d reads the output of call %lld (of %d)", c, (long long)x, n);
            omega += len_out[x];
            const int a = find(c), b = find((int)x);
            if (a != b) comp[std::max(a, b)] = std::min(a, b);
        }
        cost[c] = (int64_t)len_out[c] * omega + (int64_t)len_out[c] * (len_out[c] + 1) / 2;
    }
    std::vector<int64_t> group_cost(n, 0);
    std::vector<int32_t> roots;
    for (int c = 0; c < n; ++c) {
        const int g = find(c);
        if (g == c) roots.push_back(c);
        group_cost[g] += cost[c];
    }
    std::stable_sort(roots.begin(), roots.end(), [&](int a, int b) { return group_cost[a] > group_cost[b]; });  // ties: smaller first call
    std::vector<int64_t> load(n_workers, 0);
    std::vector<int32_t> of_group(n, 0);
    for (int g : roots) {
        int w = 0;
        for (int i = 1; i < n_workers; ++i)
            if (load[i] < load[w]) w = i;
        of_group[g] = w;
        load[w] += group_cost[g];
    }
    for (int c = 0; c < n; ++c) worker[c] = of_group[find(c)];
    return HKV_OK;
}

namespace {

// first node below the root on the call's path (its leaf for an empty prompt): the static prompt its operator
// family shares
int static_prompt_node(const hkv_trt &t, int c) {
    int v = t.leaf_of_call[c];
    while (t.parent[v] > 0) v = t.parent[v];
    return v;
}

int check_orders(const hkv_trt *t, const int32_t *indptr, const int32_t *calls, int32_t n_workers, const char *who) {
    if (!t || !indptr || n_workers < 1) return fail(HKV_EINVAL, "%s: bad argument", who);
    const int n = (int)t->len_out.size();
    if (indptr[0] != 0 || indptr[n_workers] != n) return fail(HKV_EINVAL, "%s: the orders do not hold %d calls", who, n);
    if (n > 0 && !calls) return fail(HKV_EINVAL, "%s: null order", who);
    for (int i = 0; i < n_workers; ++i)
        if (indptr[i + 1] < indptr[i]) return fail(HKV_EINVAL, "%s: indptr decreases", who);
    std::vector<char> seen(n, 0);
    for (int k = 0; k < n; ++k) {
        if (calls[k] < 0 || calls[k] >= n || seen[calls[k]]) return fail(HKV_ERANGE, "%s: the orders are no partition of the calls (entry %d)", who, k);
        seen[calls[k]] = 1;
    }
    return HKV_OK;
}

}  // namespace

// A worker's final schedule as inner sequences: the calls under one static prompt, in the order of sigma,
// released (appended to the worker's list) when the last of them has been emitted.
extern "C" int trt_nested(const hkv_trt *t, const int32_t *sigma_indptr, const int32_t *sigma, int32_t n_workers,
                          int32_t *seq_indptr, int32_t *seq_begin, int32_t *nested) {
    if (int rc = check_orders(t, sigma_indptr, sigma, n_workers, "trt_nested")) return rc;
    if (!seq_indptr || !seq_begin) return fail(HKV_EINVAL, "trt_nested: null output");
    const int n = (int)t->len_out.size();
    if (n > 0 && !nested) return fail(HKV_EINVAL, "trt_nested: null output");
    const int n_nodes = (int)t->parent.size();
    std::vector<int32_t> total(n_nodes), have(n_nodes);
    std::vector<std::vector<int32_t>> buffer(n_nodes);
    int n_seq = 0, pos = 0;
    seq_indptr[0] = 0;
    for (int i = 0; i < n_workers; ++i) {
        std::fill(total.begin(), total.end(), 0);
        for (int k = sigma_indptr[i]; k < sigma_indptr[i + 1]; ++k) ++total[static_prompt_node(*t, sigma[k])];
        for (int k = sigma_indptr[i]; k < sigma_indptr[i + 1]; ++k) {
            const int g = static_prompt_node(*t, sigma[k]);
            buffer[g].push_back(sigma[k]);
            if ((int)buffer[g].size() == total[g]) {  // the family is complete on this worker: release it
                seq_begin[n_seq++] = pos;
                for (int32_t c : buffer[g]) nested[pos++] = c;
                buffer[g].clear();
            }
        }
        seq_indptr[i + 1] = n_seq;
    }
    seq_begin[n_seq] = pos;
    return HKV_OK;
}

// Best-effort execution of per-worker priority orders under the cost model: every worker with calls left
// names the first call of its order whose dependencies have all been issued; the worker whose candidate can
// start earliest (ties: lower number) issues it.
extern "C" int trt_run_soft(const hkv_trt *t, const int32_t *order_indptr, const int32_t *order, int32_t n_workers,
                            int64_t capacity, int32_t *sigma, int64_t *B, int64_t *C, int64_t *T) {
    if (int rc = check_orders(t, order_indptr, order, n_workers, "trt_run_soft")) return rc;
    if (!T || capacity < 1) return fail(HKV_EINVAL, "trt_run_soft: bad argument");
    const int n = (int)t->len_out.size();
    if (n > 0 && !sigma) return fail(HKV_EINVAL, "trt_run_soft: null sigma");
    std::vector<char> issued(n, 0);
    std::vector<int64_t> b(n, 0), cc(n, 0), free_at(n_workers, 0);
    std::vector<std::vector<int32_t>> left(n_workers);
    std::vector<int32_t> n_run(n_workers, 0), last(n_workers, -1);
    for (int i = 0; i < n_workers; ++i) left[i].assign(order + order_indptr[i], order + order_indptr[i + 1]);
    for (int step = 0; step < n; ++step) {
        int best_w = -1, best_c = -1, best_k = -1;
        int64_t best_b = 0;
        for (int i = 0; i < n_workers; ++i) {
            int cand = -1, at = -1;
            for (int k = 0; k < (int)left[i].size() && cand < 0; ++k) {
                bool ok = true;
                for (int x : t->deps[left[i][k]]) ok = ok && issued[x];
                if (ok) {
                    cand = left[i][k];
                    at = k;
                }
            }
            if (cand < 0) continue;
            int64_t start = free_at[i];
            for (int x : t->deps[cand]) start = std::max(start, cc[x] + capacity * t->len_out[x]);
            if (best_w < 0 || start < best_b) {
                best_w = i;
                best_c = cand;
                best_k = at;
                best_b = start;
            }
        }
        if (best_w < 0) return fail(HKV_ETREE, "trt_run_soft: dependency cycle");
        b[best_c] = best_b;
        cc[best_c] = best_b + call_usage(*t, last[best_w], best_c);
        free_at[best_w] = cc[best_c];
        issued[best_c] = 1;
        sigma[order_indptr[best_w] + n_run[best_w]++] = best_c;
        last[best_w] = best_c;
        left[best_w].erase(left[best_w].begin() + best_k);
    }
    int64_t mx = 0;
    for (int c = 0; c < n; ++c) mx = std::max(mx, cc[c]);
    if (B && n) memcpy(B, b.data(), n * sizeof(int64_t));
    if (C && n) memcpy(C, cc.data(), n * sizeof(int64_t));
    *T = mx;
    return HKV_OK;
}
