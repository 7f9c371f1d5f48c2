// cp_context_index: host-side context index behind the C ABI of cp_context_index.h
// (paper, Sections 4 and 5 and the appendix algorithms for construction, search, alignment and
// scheduling).  Plain C++; no GPU call.
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <deque>
#include <limits>
#include <map>
#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "cp_context_index.h"

namespace {

typedef std::vector<int32_t> Ids;

struct Node {
    Ids docs;
    std::vector<int32_t> children;
    int32_t parent = -1;
    bool leaf = false;
    int32_t freq = 0;
    double created_at = 0.0;
};

bool contains(const Ids &v, int32_t x) { return std::find(v.begin(), v.end(), x) != v.end(); }

int shared_count(const Ids &a, const Ids &b)
{
    int s = 0;
    for (int32_t x : a) s += contains(b, x) ? 1 : 0;
    return s;
}

// Eq. 1 in double precision; positions are 0-based ranks.
double context_distance(const Ids &ci, const Ids &cj, double alpha)
{
    if (ci.empty() && cj.empty()) return 0.0;
    int shared = 0;
    long gaps = 0;
    for (size_t p = 0; p < ci.size(); ++p)
        for (size_t q = 0; q < cj.size(); ++q)
            if (ci[p] == cj[q]) {
                ++shared;
                gaps += std::labs((long)p - (long)q);
            }
    double d = 1.0 - (double)shared / (double)std::max(ci.size(), cj.size());
    if (shared > 0) d += alpha * (double)gaps / (double)shared;
    return d;
}

// prefix followed by the rest of docs in their own order
Ids align_to(const Ids &prefix, const Ids &docs)
{
    Ids out(prefix);
    for (int32_t b : docs)
        if (!contains(prefix, b)) out.push_back(b);
    return out;
}

struct Merge {
    int32_t a, b; // cluster ids, a < b
    double d;
};

// Average-linkage clustering of m points.  Each step merges the active pair with the smallest
// (distance, lower id, higher id).  D is consumed.
std::vector<Merge> linkage(std::vector<double> &D, int32_t m)
{
    std::vector<Merge> merges;
    if (m < 2) return merges;
    struct Key {
        double d;
        int32_t lo, hi;
        bool operator<(const Key &o) const
        {
            if (d != o.d) return d < o.d;
            if (lo != o.lo) return lo < o.lo;
            return hi < o.hi;
        }
    };
    const Key none = {std::numeric_limits<double>::infinity(), INT32_MAX, INT32_MAX};
    std::vector<int32_t> id(m), size(m, 1), best(m, -1);
    std::vector<char> active(m, 1);
    std::vector<Key> best_key(m, none);
    for (int32_t i = 0; i < m; ++i) id[i] = i;
    auto key_of = [&](int32_t i, int32_t j) {
        return Key{D[(size_t)i * m + j], std::min(id[i], id[j]), std::max(id[i], id[j])};
    };
    auto rescan = [&](int32_t i) {
        best[i] = -1;
        best_key[i] = none;
        for (int32_t j = 0; j < m; ++j)
            if (j != i && active[j]) {
                const Key k = key_of(i, j);
                if (k < best_key[i]) {
                    best_key[i] = k;
                    best[i] = j;
                }
            }
    };
    for (int32_t i = 0; i < m; ++i) rescan(i);
    for (int32_t step = 0; step + 1 < m; ++step) {
        int32_t r = -1;
        for (int32_t i = 0; i < m; ++i)
            if (active[i] && (r < 0 || best_key[i] < best_key[r])) r = i;
        int32_t a = r, b = best[r];
        if (id[a] > id[b]) std::swap(a, b);
        merges.push_back({id[a], id[b], best_key[r].d});
        // the merged cluster lives in slot a
        const double sa = (double)size[a], sb = (double)size[b];
        for (int32_t k = 0; k < m; ++k)
            if (active[k] && k != a && k != b) {
                const double v = (sa * D[(size_t)a * m + k] + sb * D[(size_t)b * m + k]) / (sa + sb);
                D[(size_t)a * m + k] = v;
                D[(size_t)k * m + a] = v;
            }
        active[b] = 0;
        size[a] += size[b];
        id[a] = m + step;
        rescan(a);
        for (int32_t k = 0; k < m; ++k)
            if (active[k] && k != a) {
                if (best[k] == a || best[k] == b) {
                    rescan(k);
                } else {
                    const Key kk = key_of(k, a);
                    if (kk < best_key[k]) {
                        best_key[k] = kk;
                        best[k] = a;
                    }
                }
            }
    }
    return merges;
}

} // namespace

struct cp_index {
    double alpha = 0.0;
    std::vector<Node> nodes;      // handle = position; 0 is the root
    std::vector<int32_t> leaf_of; // stored context -> leaf handle

    int32_t leaves_below(int32_t v) const
    {
        if (nodes[v].leaf) return 1;
        int32_t s = 0;
        for (int32_t c : nodes[v].children) s += leaves_below(c);
        return s;
    }
    std::vector<int32_t> path_of(int32_t v) const
    {
        std::vector<int32_t> p;
        while (nodes[v].parent >= 0) {
            const std::vector<int32_t> &sib = nodes[nodes[v].parent].children;
            p.push_back((int32_t)(std::find(sib.begin(), sib.end(), v) - sib.begin()));
            v = nodes[v].parent;
        }
        std::reverse(p.begin(), p.end());
        return p;
    }
    // empty virtual nodes give their place to their children
    void remove_empty(int32_t v)
    {
        bool changed = true;
        while (changed) {
            changed = false;
            std::vector<int32_t> kids;
            for (int32_t c : nodes[v].children) {
                if (!nodes[c].leaf && nodes[c].docs.empty()) {
                    kids.insert(kids.end(), nodes[c].children.begin(), nodes[c].children.end());
                    changed = true;
                } else {
                    kids.push_back(c);
                }
            }
            nodes[v].children = kids;
            for (int32_t c : kids) nodes[c].parent = v;
        }
        for (size_t i = 0; i < nodes[v].children.size(); ++i) {
            const int32_t c = nodes[v].children[i];
            if (!nodes[c].leaf) remove_empty(c);
        }
    }
    // greedy descent; returns the matched node, fills path
    int32_t search(const Ids &C, std::vector<int32_t> &path) const
    {
        int32_t cur = 0;
        path.clear();
        while (!nodes[cur].children.empty()) {
            int32_t best = -1;
            double best_d = 0.0;
            for (size_t i = 0; i < nodes[cur].children.size(); ++i) {
                const Node &ch = nodes[nodes[cur].children[i]];
                if (shared_count(C, ch.docs) == 0) continue;
                const double d = context_distance(C, ch.docs, alpha);
                if (best < 0 || d < best_d) {
                    best = (int32_t)i;
                    best_d = d;
                }
            }
            if (best < 0) break;
            const int32_t c = nodes[cur].children[best];
            const int in_child = shared_count(C, nodes[c].docs);
            if (in_child <= shared_count(C, nodes[cur].docs)) break;
            path.push_back(best);
            if (nodes[c].leaf || in_child < (int)nodes[c].docs.size()) return c;
            cur = c;
        }
        return cur;
    }
};

namespace {

bool read_context(const int32_t *contexts, const int32_t *lens, int32_t i, int32_t stride, Ids &out)
{
    if (lens[i] < 0 || lens[i] > stride) return false;
    out.assign(contexts + (size_t)i * stride, contexts + (size_t)i * stride + lens[i]);
    for (size_t p = 0; p < out.size(); ++p) {
        if (out[p] < 0) return false;
        for (size_t q = 0; q < p; ++q)
            if (out[q] == out[p]) return false;
    }
    return true;
}

struct IdsHash {
    size_t operator()(const Ids &v) const
    {
        size_t h = 1469598103934665603ull ^ v.size();
        for (int32_t x : v) h = (h ^ (size_t)(uint32_t)x) * 1099511628211ull;
        return h;
    }
};

// distinct contexts in order of first appearance; member[i] = rank of row i's context
int distinct(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride, std::vector<Ids> &uniq,
             std::vector<int32_t> &member)
{
    std::unordered_map<Ids, int32_t, IdsHash> where;
    Ids c;
    member.resize(n);
    for (int32_t i = 0; i < n; ++i) {
        if (!read_context(contexts, lens, i, stride, c)) return -2;
        auto it = where.find(c);
        if (it == where.end()) {
            it = where.emplace(c, (int32_t)uniq.size()).first;
            uniq.push_back(c);
        }
        member[i] = it->second;
    }
    return 0;
}

int copy_out(const std::vector<int32_t> &v, int32_t *dst, int32_t cap, int32_t *len)
{
    if (len) *len = (int32_t)v.size();
    if ((int32_t)v.size() > cap) return -2;
    if (!v.empty() && !dst) return -1;
    std::copy(v.begin(), v.end(), dst);
    return 0;
}

} // namespace

extern "C" int cp_index_distinct(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride,
                                 int32_t *first_of, int32_t *m)
{
    if (n < 0 || stride < 1) return -2;
    if (!m || (n > 0 && (!contexts || !lens || !first_of))) return -1;
    std::vector<Ids> uniq;
    std::vector<int32_t> member;
    const int st = distinct(contexts, lens, n, stride, uniq, member);
    if (st) return st;
    std::copy(member.begin(), member.end(), first_of);
    *m = (int32_t)uniq.size();
    return 0;
}

extern "C" int cp_index_build(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride, double alpha,
                              const float *dist, int32_t m, cp_index **out)
{
    if (!out) return -1;
    *out = nullptr;
    if (n < 0 || stride < 1 || !(alpha >= 0.0) || !std::isfinite(alpha)) return -2;
    if (n > 0 && (!contexts || !lens)) return -1;
    std::vector<Ids> uniq;
    std::vector<int32_t> member;
    int st = distinct(contexts, lens, n, stride, uniq, member);
    if (st) return st;
    const int32_t mu = (int32_t)uniq.size();
    if (dist && m != mu) return -2;

    cp_index *idx = new (std::nothrow) cp_index();
    if (!idx) return -2;
    idx->alpha = alpha;
    std::vector<Node> &nodes = idx->nodes;
    nodes.emplace_back(); // root, empty context
    // cluster id c (0 .. 2 mu - 2) -> node handle 1 + c
    for (int32_t u = 0; u < mu; ++u) {
        Node leaf;
        leaf.docs = uniq[u];
        leaf.leaf = true;
        nodes.push_back(leaf);
    }
    for (int32_t i = 0; i < n; ++i) nodes[1 + member[i]].freq += 1;

    std::vector<double> D((size_t)mu * mu, 0.0);
    for (int32_t i = 0; i < mu; ++i)
        for (int32_t j = 0; j < mu; ++j)
            if (i != j)
                D[(size_t)i * mu + j] = dist ? (double)dist[(size_t)i * mu + j] : context_distance(uniq[i], uniq[j], alpha);
    std::vector<std::unordered_set<int32_t>> content(mu);
    for (int32_t u = 0; u < mu; ++u) content[u].insert(uniq[u].begin(), uniq[u].end());
    std::vector<int32_t> leaves(mu, 1);
    for (const Merge &mg : linkage(D, mu)) {
        Node v;
        std::unordered_set<int32_t> inter;
        for (int32_t x : content[mg.a])
            if (content[mg.b].count(x)) inter.insert(x);
        v.docs.assign(inter.begin(), inter.end());
        std::sort(v.docs.begin(), v.docs.end());
        v.created_at = mg.d;
        int32_t first = mg.a, second = mg.b; // larger subtree first, equal sizes in id order
        if (leaves[mg.b] > leaves[mg.a]) std::swap(first, second);
        const int32_t handle = (int32_t)nodes.size();
        v.children = {1 + first, 1 + second};
        nodes[1 + first].parent = handle;
        nodes[1 + second].parent = handle;
        nodes.push_back(v);
        content.push_back(inter);
        leaves.push_back(leaves[mg.a] + leaves[mg.b]);
    }
    if (mu > 0) {
        const int32_t top = (int32_t)nodes.size() - 1;
        nodes[0].children.push_back(top);
        nodes[top].parent = 0;
    }
    idx->remove_empty(0);
    // top-down prefix alignment, breadth first
    std::deque<int32_t> queue(nodes[0].children.begin(), nodes[0].children.end());
    while (!queue.empty()) {
        const int32_t v = queue.front();
        queue.pop_front();
        const int32_t par = nodes[v].parent;
        if (par != 0 && !nodes[par].docs.empty()) nodes[v].docs = align_to(nodes[par].docs, nodes[v].docs);
        queue.insert(queue.end(), nodes[v].children.begin(), nodes[v].children.end());
    }
    idx->leaf_of.resize(n);
    for (int32_t i = 0; i < n; ++i) idx->leaf_of[i] = 1 + member[i];
    *out = idx;
    return 0;
}

extern "C" void cp_index_free(cp_index *index) { delete index; }

extern "C" int32_t cp_index_num_contexts(const cp_index *index) { return index ? (int32_t)index->leaf_of.size() : -1; }
extern "C" int32_t cp_index_num_nodes(const cp_index *index) { return index ? (int32_t)index->nodes.size() : -1; }

extern "C" int cp_index_aligned(const cp_index *index, int32_t i, int32_t *ids, int32_t cap, int32_t *len)
{
    if (!index) return -1;
    if (i < 0 || i >= (int32_t)index->leaf_of.size()) return -2;
    return copy_out(index->nodes[index->leaf_of[i]].docs, ids, cap, len);
}

extern "C" int cp_index_path(const cp_index *index, int32_t i, int32_t *path, int32_t cap, int32_t *len)
{
    if (!index) return -1;
    if (i < 0 || i >= (int32_t)index->leaf_of.size()) return -2;
    return copy_out(index->path_of(index->leaf_of[i]), path, cap, len);
}

extern "C" int cp_index_leaf(const cp_index *index, int32_t i, int32_t *node)
{
    if (!index || !node) return -1;
    if (i < 0 || i >= (int32_t)index->leaf_of.size()) return -2;
    *node = index->leaf_of[i];
    return 0;
}

extern "C" int cp_index_node(const cp_index *index, int32_t node, int32_t *parent, int32_t *is_leaf, int32_t *freq,
                             double *created_at, int32_t *num_children, int32_t *ids, int32_t cap, int32_t *len)
{
    if (!index) return -1;
    if (node < 0 || node >= (int32_t)index->nodes.size()) return -2;
    const Node &v = index->nodes[node];
    if (parent) *parent = v.parent;
    if (is_leaf) *is_leaf = v.leaf ? 1 : 0;
    if (freq) *freq = v.freq;
    if (created_at) *created_at = v.created_at;
    if (num_children) *num_children = (int32_t)v.children.size();
    return copy_out(v.docs, ids, cap, len);
}

extern "C" int cp_index_children(const cp_index *index, int32_t node, int32_t *children, int32_t cap, int32_t *len)
{
    if (!index) return -1;
    if (node < 0 || node >= (int32_t)index->nodes.size()) return -2;
    return copy_out(index->nodes[node].children, children, cap, len);
}

namespace {
bool read_query(const int32_t *ids, int32_t len, Ids &C)
{
    C.assign(ids, ids + len);
    for (size_t p = 0; p < C.size(); ++p) {
        if (C[p] < 0) return false;
        for (size_t q = 0; q < p; ++q)
            if (C[q] == C[p]) return false;
    }
    return true;
}
} // namespace

extern "C" int cp_index_search(const cp_index *index, const int32_t *ids, int32_t len, int32_t *path, int32_t cap,
                               int32_t *path_len, int32_t *node)
{
    if (!index || (len > 0 && !ids)) return -1;
    if (len < 0) return -2;
    Ids C;
    if (!read_query(ids, len, C)) return -2;
    std::vector<int32_t> p;
    const int32_t v = index->search(C, p);
    if (node) *node = v;
    return copy_out(p, path, cap, path_len);
}

extern "C" int cp_index_insert(cp_index *index, const int32_t *ids, int32_t len, int32_t *aligned, int32_t *path,
                               int32_t cap, int32_t *path_len)
{
    if (!index || (len > 0 && (!ids || !aligned))) return -1;
    if (len < 0) return -2;
    Ids C;
    if (!read_query(ids, len, C)) return -2;
    std::vector<Node> &nodes = index->nodes;
    std::vector<int32_t> p;
    int32_t node = index->search(C, p);
    // Nothing is changed before the outputs are known to fit: the stored leaf ends up at most
    // one level below the matched node, so its path has at most p.size() + 1 entries.  A caller
    // that gets -2 can come back with a larger buffer and finds the index as it was.
    if (path_len) *path_len = (int32_t)p.size() + 1;
    if ((int64_t)p.size() + 1 > (int64_t)cap) return -2;
    if (!path) return -1;
    int32_t leaf = -1;
    if (nodes[node].leaf && nodes[node].docs == align_to(nodes[nodes[node].parent].docs, C)) {
        leaf = node; // identical context
    } else {
        if (nodes[node].leaf || shared_count(C, nodes[node].docs) < (int)nodes[node].docs.size()) {
            // a new virtual node takes the matched node's place
            Node v;
            for (int32_t b : nodes[node].docs)
                if (contains(C, b)) v.docs.push_back(b);
            v.created_at = context_distance(C, nodes[node].docs, index->alpha);
            v.parent = nodes[node].parent;
            v.children = {node};
            const int32_t handle = (int32_t)nodes.size();
            std::vector<int32_t> &sib = nodes[v.parent].children;
            *std::find(sib.begin(), sib.end(), node) = handle;
            nodes.push_back(v);
            nodes[node].parent = handle;
            node = handle;
        }
        const Ids a = align_to(nodes[node].docs, C);
        for (int32_t c : nodes[node].children)
            if (leaf < 0 && nodes[c].leaf && nodes[c].docs == a) leaf = c;
        if (leaf < 0) {
            Node l;
            l.docs = a;
            l.leaf = true;
            l.parent = node;
            leaf = (int32_t)nodes.size();
            nodes.push_back(l);
            nodes[node].children.push_back(leaf);
        }
    }
    nodes[leaf].freq += 1;
    index->leaf_of.push_back(leaf);
    std::copy(nodes[leaf].docs.begin(), nodes[leaf].docs.end(), aligned);
    return copy_out(index->path_of(leaf), path, cap, path_len);
}

extern "C" int cp_index_schedule(const int32_t *paths, const int32_t *path_lens, int32_t n, int32_t stride,
                                 int32_t *order)
{
    if (n < 0 || stride < 1) return -2;
    if (n > 0 && (!paths || !path_lens || !order)) return -1;
    // groups in order of first appearance of their key (first path element; -1 for an empty path)
    std::vector<std::vector<int32_t>> groups;
    std::map<int32_t, size_t> where;
    for (int32_t i = 0; i < n; ++i) {
        if (path_lens[i] < 0 || path_lens[i] > stride) return -2;
        const int32_t key = path_lens[i] > 0 ? paths[(size_t)i * stride] : -1;
        auto it = where.find(key);
        if (it == where.end()) {
            it = where.emplace(key, groups.size()).first;
            groups.emplace_back();
        }
        groups[it->second].push_back(i);
    }
    for (auto &g : groups)
        std::stable_sort(g.begin(), g.end(), [&](int32_t x, int32_t y) { return path_lens[x] > path_lens[y]; });
    std::stable_sort(groups.begin(), groups.end(),
                     [](const std::vector<int32_t> &x, const std::vector<int32_t> &y) { return x.size() > y.size(); });
    int32_t at = 0;
    for (const auto &g : groups)
        for (int32_t i : g) order[at++] = i;
    return 0;
}
