// Host side adaptive peer selection (Alg. 1 line 2 and Alg. 3 of the paper); declared in
// include/saps_select.h.  Pure C++17, no GPU calls.
#include "../../include/saps_select.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

namespace {

constexpr int64_t NEVER = std::numeric_limits<int64_t>::min();

// Small counter-seeded generator (splitmix64 stream) for the shuffles of RandomlyMaxMatch.
struct Shuffler {
    uint64_t s;
    explicit Shuffler(uint64_t seed) : s(seed) {}
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    // unbiased enough for shuffling small arrays: multiply-shift on the high word
    uint32_t below(uint32_t bound) { return (uint32_t)(((next() >> 32) * (uint64_t)bound) >> 32); }
    template <class T> void shuffle(std::vector<T>& v) {
        for (size_t k = v.size(); k > 1; --k) std::swap(v[k - 1], v[below((uint32_t)k)]);
    }
};

// Maximum-cardinality matching in a general graph (Edmonds 1965): repeated breadth-first
// searches for an augmenting path from every free vertex; an odd cycle met during the search
// (a blossom) is shrunk by giving all its vertices a common base.
class Blossom {
public:
    Blossom(int n, const std::vector<std::vector<int>>& adj)
        : n_(n), adj_(adj), mate_(n, -1), parent_(n), base_(n), in_tree_(n), in_blossom_(n), seen_(n) {}

    // roots are tried in the given order; returns the number of matched pairs
    int run(const std::vector<int>& order) {
        int pairs = 0;
        for (int r : order) {
            if (mate_[r] != -1) continue;
            const int leaf = search(r);
            if (leaf == -1) continue;
            // flip the alternating path leaf -> root
            for (int v = leaf; v != -1;) {
                const int pv = parent_[v], next = mate_[pv];
                mate_[v] = pv;
                mate_[pv] = v;
                v = next;
            }
            ++pairs;
        }
        return pairs;
    }
    const std::vector<int>& mate() const { return mate_; }

private:
    int common_base(int a, int b) {
        std::fill(seen_.begin(), seen_.end(), 0);
        for (;;) {                                   // climb from a to the root, marking bases
            a = base_[a];
            seen_[a] = 1;
            if (mate_[a] == -1) break;
            a = parent_[mate_[a]];
        }
        for (;;) {                                   // first marked base on b's way up
            b = base_[b];
            if (seen_[b]) return b;
            b = parent_[mate_[b]];
        }
    }

    void mark_to_base(int v, int stem, int child) {
        while (base_[v] != stem) {
            in_blossom_[base_[v]] = 1;
            in_blossom_[base_[mate_[v]]] = 1;
            parent_[v] = child;
            child = mate_[v];
            v = parent_[mate_[v]];
        }
    }

    int search(int root) {
        std::fill(in_tree_.begin(), in_tree_.end(), 0);
        std::fill(parent_.begin(), parent_.end(), -1);
        std::iota(base_.begin(), base_.end(), 0);
        queue_.clear();
        queue_.push_back(root);
        in_tree_[root] = 1;
        for (size_t head = 0; head < queue_.size(); ++head) {
            const int v = queue_[head];
            for (int to : adj_[v]) {
                if (base_[v] == base_[to] || mate_[v] == to) continue;
                if (to == root || (mate_[to] != -1 && parent_[mate_[to]] != -1)) {
                    // edge between two outer vertices: shrink the odd cycle
                    const int stem = common_base(v, to);
                    std::fill(in_blossom_.begin(), in_blossom_.end(), 0);
                    mark_to_base(v, stem, to);
                    mark_to_base(to, stem, v);
                    for (int u = 0; u < n_; ++u) {
                        if (!in_blossom_[base_[u]]) continue;
                        base_[u] = stem;
                        if (!in_tree_[u]) { in_tree_[u] = 1; queue_.push_back(u); }
                    }
                } else if (parent_[to] == -1) {
                    parent_[to] = v;
                    if (mate_[to] == -1) return to;  // free vertex reached: augmenting path
                    in_tree_[mate_[to]] = 1;
                    queue_.push_back(mate_[to]);
                }
            }
        }
        return -1;
    }

    int n_;
    const std::vector<std::vector<int>>& adj_;
    std::vector<int> mate_, parent_, base_;
    std::vector<char> in_tree_, in_blossom_, seen_;
    std::vector<int> queue_;
};

// RandomlyMaxMatch: shuffled neighbour lists and shuffled root order.
int randomly_max_match(int n, const std::vector<uint8_t>& E, uint64_t seed, std::vector<int>& mate) {
    Shuffler rng(seed);
    std::vector<std::vector<int>> adj(n);
    for (int i = 0; i < n; ++i)
        for (int j = i + 1; j < n; ++j)
            if (E[(size_t)i * n + j] || E[(size_t)j * n + i]) { adj[i].push_back(j); adj[j].push_back(i); }
    for (auto& a : adj) rng.shuffle(a);
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    rng.shuffle(order);
    Blossom bl(n, adj);
    const int pairs = bl.run(order);
    mate = bl.mate();
    return pairs;
}

// Connected components of the graph with adjacency predicate Q (dense n x n).
int components(int n, const std::vector<uint8_t>& Q, std::vector<int>& comp) {
    comp.assign(n, -1);
    int count = 0;
    std::vector<int> stack;
    for (int s = 0; s < n; ++s) {
        if (comp[s] != -1) continue;
        comp[s] = count;
        stack.push_back(s);
        while (!stack.empty()) {
            const int v = stack.back();
            stack.pop_back();
            for (int u = 0; u < n; ++u)
                if (comp[u] == -1 && Q[(size_t)v * n + u]) { comp[u] = count; stack.push_back(u); }
        }
        ++count;
    }
    return count;
}

uint64_t mix_seed(uint64_t seed, uint64_t t, uint64_t pass) {
    Shuffler a(seed ^ (t * 0xD1342543DE82EF95ull) ^ (pass << 56));
    return a.next();
}

}  // namespace

struct saps_selector {
    int n = 0;
    double B_thres = 0.0;
    int64_t T_thres = 1;
    uint64_t seed = 0;
    std::vector<double> B;        // symmetrised
    std::vector<uint8_t> Bstar;   // GetNewConnectedGraph: B_ij >= B_thres
    std::vector<int64_t> R;       // last round in which (i, j) exchanged
};

extern "C" {

int32_t saps_selector_create(saps_selector** out, int32_t n, const double* B, double B_thres, int64_t T_thres,
                             uint64_t seed) {
    if (!out) return 1;
    *out = nullptr;
    if (!B || n < 1 || T_thres < 1 || std::isnan(B_thres)) return 1;
    for (int64_t k = 0; k < (int64_t)n * n; ++k)
        if (std::isnan(B[k])) return 1;
    saps_selector* s = new (std::nothrow) saps_selector;
    if (!s) return 1;
    s->n = n; s->B_thres = B_thres; s->T_thres = T_thres; s->seed = seed;
    s->B.assign((size_t)n * n, 0.0);
    s->Bstar.assign((size_t)n * n, 0);
    s->R.assign((size_t)n * n, NEVER);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            if (i == j) continue;
            const double b = std::min(B[(size_t)i * n + j], B[(size_t)j * n + i]);   // the slower direction decides
            s->B[(size_t)i * n + j] = b;
            s->Bstar[(size_t)i * n + j] = b >= B_thres ? 1 : 0;
        }
    *out = s;
    return 0;
}

int32_t saps_selector_destroy(saps_selector* s) {
    if (!s) return 1;
    delete s;
    return 0;
}

int32_t saps_selector_get_R(const saps_selector* s, int64_t* R_out) {
    if (!s || !R_out) return 1;
    std::copy(s->R.begin(), s->R.end(), R_out);
    return 0;
}

int32_t saps_selector_next(saps_selector* s, int64_t t, int32_t* peer_out, saps_select_info* info) {
    if (!s || !peer_out) return 1;
    const int n = s->n;
    // IfConnected: graph of recently connected edges, R_ij > t - T_thres
    std::vector<uint8_t> Q((size_t)n * n, 0);
    for (size_t k = 0; k < Q.size(); ++k)
        Q[k] = (s->R[k] != NEVER && s->R[k] > t - s->T_thres) ? 1 : 0;
    std::vector<int> comp;
    const int ncomp = components(n, Q, comp);
    const bool connected = ncomp == 1;
    // candidate edges: B* when connected, else every pair that joins two different components
    std::vector<uint8_t> E;
    if (connected) {
        E = s->Bstar;
    } else {
        E.assign((size_t)n * n, 0);
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                if (i != j && comp[i] != comp[j]) E[(size_t)i * n + j] = 1;
    }
    std::vector<int> mate;
    const int first = randomly_max_match(n, E, mix_seed(s->seed, (uint64_t)t, 0), mate);
    int second = 0;
    if (first != n / 2) {
        // GetUnmatch: match the leftovers among themselves, bandwidth ignored
        std::vector<int> rest;
        for (int i = 0; i < n; ++i)
            if (mate[i] == -1) rest.push_back(i);
        const int m = (int)rest.size();
        std::vector<uint8_t> E2((size_t)m * m, 1);
        std::vector<int> mate2;
        second = randomly_max_match(m, E2, mix_seed(s->seed, (uint64_t)t, 1), mate2);
        for (int a = 0; a < m; ++a)
            if (mate2[a] != -1) mate[rest[a]] = rest[mate2[a]];
    }
    double bmin = std::numeric_limits<double>::infinity(), bsum = 0.0;
    int pairs = 0;
    for (int i = 0; i < n; ++i) {
        const int p = mate[i];
        peer_out[i] = p == -1 ? i : p;
        if (p > i) {
            const double b = s->B[(size_t)i * n + p];
            bmin = std::min(bmin, b);
            bsum += b;
            ++pairs;
            s->R[(size_t)i * n + p] = t;
            s->R[(size_t)p * n + i] = t;
        }
    }
    if (info) {
        info->rc_connected = connected ? 1 : 0;
        info->rc_components = ncomp;
        info->first_pairs = first;
        info->second_pairs = second;
        info->min_bandwidth = pairs ? bmin : 0.0;
        info->mean_bandwidth = pairs ? bsum / pairs : 0.0;
    }
    return 0;
}

int32_t saps_max_matching(int32_t n, const uint8_t* E, uint64_t seed, int32_t* peer_out) {
    if (n < 0 || (n > 0 && (!E || !peer_out))) return -1;
    std::vector<uint8_t> Ev(E, E + (size_t)n * n);
    std::vector<int> mate;
    const int pairs = randomly_max_match(n, Ev, seed, mate);
    for (int i = 0; i < n; ++i) peer_out[i] = mate[i] == -1 ? i : mate[i];
    return pairs;
}

}  // extern "C"
