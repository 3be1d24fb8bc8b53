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
