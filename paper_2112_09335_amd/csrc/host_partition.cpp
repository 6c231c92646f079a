// Deterministic multilevel partitioner: size-capped synchronous label propagation until it rests, contraction of
// the clusters to the nodes of the next level, greedy merging on the last level along the heaviest connection,
// and propagation on the finest graph at the end until it rests again.
// The paper leaves the partition to METIS (Section 2); this is the library's own stand-in, every tie broken
// by node or cluster number so that the result depends on nothing but the input.
#include "host_partition.h"

#include <algorithm>
#include <map>
#include <queue>
#include <thread>
#include <tuple>
#include <vector>

namespace cadmm {

namespace {

template <class F>
void parallel_nodes(int64_t n, F f) {
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<int64_t>(std::max(1u, std::min(hw, 16u)), std::max<int64_t>(1, n / 8192));
    if (nt <= 1) { f(0, n); return; }
    std::vector<std::thread> th;
    const int64_t per = (n + nt - 1) / nt;
    for (int t = 0; t < nt; ++t) {
        const int64_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        th.emplace_back([=] { f(lo, hi); });
    }
    for (auto& x : th) x.join();
}

// Weighted graph of one level: neighbours of a node ascending, no repeats, no self.
struct Level {
    int64_t n = 0;
    std::vector<int64_t> ptr;      // [n+1]
    std::vector<int32_t> col;
    std::vector<int64_t> ew;       // edge weights, parallel to col
    std::vector<int64_t> nw;       // [n] node weights
};

Level finest_level(int64_t N, int64_t n_edges, const int32_t* src, const int32_t* dst) {
    std::vector<int64_t> start(N + 1, 0);
    for (int64_t e = 0; e < n_edges; ++e)
        if (src[e] != dst[e]) { start[src[e] + 1]++; start[dst[e] + 1]++; }
    for (int64_t i = 0; i < N; ++i) start[i + 1] += start[i];
    std::vector<int32_t> raw((size_t)start[N]);
    {
        std::vector<int64_t> cur(start.begin(), start.end() - 1);
        for (int64_t e = 0; e < n_edges; ++e)
            if (src[e] != dst[e]) {
                raw[(size_t)cur[src[e]]++] = dst[e];
                raw[(size_t)cur[dst[e]]++] = src[e];
            }
    }
    std::vector<int64_t> len(N);
    parallel_nodes(N, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i) {
            int32_t* b = raw.data() + start[i];
            int32_t* e = raw.data() + start[i + 1];
            std::sort(b, e);
            len[i] = std::unique(b, e) - b;
        }
    });
    Level g;
    g.n = N;
    g.ptr.assign(N + 1, 0);
    for (int64_t i = 0; i < N; ++i) g.ptr[i + 1] = g.ptr[i] + len[i];
    g.col.resize((size_t)g.ptr[N]);
    parallel_nodes(N, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i)
            std::copy(raw.data() + start[i], raw.data() + start[i] + len[i], g.col.data() + g.ptr[i]);
    });
    g.ew.assign(g.col.size(), 1);
    g.nw.assign(N, 1);
    return g;
}

inline bool takes_part(uint64_t v, uint64_t r) {
    return (((v * 2654435761ull + r * 40503ull) >> 16) & 1ull) == 0;     // arithmetic modulo 2^64
}

// One synchronous round.  label[v] in [0, size.size()); size[c] = weight of the nodes with label c.
// Returns the number of moves.
int64_t propagation_round(const Level& g, std::vector<int32_t>& label, std::vector<int64_t>& size, int64_t cap, int r,
                          std::vector<int32_t>& want, std::vector<int64_t>& granted) {
    const int64_t n = g.n;
    parallel_nodes(n, [&](int64_t lo, int64_t hi) {
        std::vector<std::pair<int32_t, int64_t>> seen;
        for (int64_t v = lo; v < hi; ++v) {
            want[v] = -1;
            const int64_t b = g.ptr[v], e = g.ptr[v + 1];
            if (b == e || !takes_part((uint64_t)v, (uint64_t)r)) continue;
            seen.resize((size_t)(e - b));
            for (int64_t k = b; k < e; ++k) seen[(size_t)(k - b)] = {label[g.col[(size_t)k]], g.ew[(size_t)k]};
            std::sort(seen.begin(), seen.end());
            int32_t best = -1;
            int64_t best_w = 0, own_w = 0;
            for (size_t i = 0; i < seen.size();) {
                int64_t w = 0;
                size_t j = i;
                while (j < seen.size() && seen[j].first == seen[i].first) w += seen[j++].second;
                if (w > best_w) { best_w = w; best = seen[i].first; }    // ascending labels: the first maximum stays
                if (seen[i].first == label[v]) own_w = w;
                i = j;
            }
            if (best_w > own_w) want[v] = best;
        }
    });
    // granted[c] = weight let into c so far; size[] still holds the weights at the start of the round
    for (int64_t v = 0; v < n; ++v)
        if (want[v] >= 0) granted[want[v]] = 0;
    int64_t moves = 0;
    for (int64_t v = 0; v < n; ++v) {
        const int32_t c = want[v];
        if (c < 0) continue;
        if (g.nw[v] <= cap - size[c] - granted[c]) { granted[c] += g.nw[v]; ++moves; }
        else want[v] = -1;
    }
    for (int64_t v = 0; v < n; ++v) {
        const int32_t c = want[v];
        if (c < 0) continue;
        size[label[v]] -= g.nw[v];
        size[c] += g.nw[v];
        label[v] = c;
    }
    return moves;
}

// Clusters numbered in increasing order of their label become the nodes of the next level.
Level contract(const Level& g, const std::vector<int32_t>& label, std::vector<int32_t>& member_of) {
    const int64_t n = g.n;
    std::vector<int32_t> number(n, -1);
    for (int64_t v = 0; v < n; ++v) number[label[v]] = 0;
    int32_t K = 0;
    for (int64_t c = 0; c < n; ++c)
        if (number[c] == 0) number[c] = K++;
    member_of.resize(n);
    Level h;
    h.n = K;
    h.nw.assign(K, 0);
    for (int64_t v = 0; v < n; ++v) { member_of[v] = number[label[v]]; h.nw[member_of[v]] += g.nw[v]; }
    // (a, b, w) of every edge that leaves its cluster, sorted by (a, b), equal pairs added up
    std::vector<std::tuple<int32_t, int32_t, int64_t>> out;
    for (int64_t v = 0; v < n; ++v)
        for (int64_t k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
            const int32_t a = member_of[v], b = member_of[g.col[(size_t)k]];
            if (a != b) out.emplace_back(a, b, g.ew[(size_t)k]);
        }
    std::sort(out.begin(), out.end());
    h.ptr.assign(K + 1, 0);
    for (size_t i = 0; i < out.size();) {
        size_t j = i;
        int64_t w = 0;
        while (j < out.size() && std::get<0>(out[j]) == std::get<0>(out[i]) && std::get<1>(out[j]) == std::get<1>(out[i]))
            w += std::get<2>(out[j++]);
        h.col.push_back(std::get<1>(out[i]));
        h.ew.push_back(w);
        h.ptr[std::get<0>(out[i]) + 1]++;
        i = j;
    }
    for (int32_t c = 0; c < K; ++c) h.ptr[c + 1] += h.ptr[c];
    return h;
}

// Community of every node of the last level: merge along the heaviest admissible connection, then the lightest
// nodes regardless of the cap, until at most M are left.
std::vector<int32_t> merge_down_to(const Level& g, int32_t M, int64_t cap) {
    const int32_t K = (int32_t)g.n;
    std::vector<std::map<int32_t, int64_t>> adj(K);
    using Entry = std::tuple<int64_t, int32_t, int32_t>;        // (-weight, a, b): the smallest entry is the wanted pair
    std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
    for (int32_t a = 0; a < K; ++a)
        for (int64_t k = g.ptr[a]; k < g.ptr[a + 1]; ++k) {
            adj[a][g.col[(size_t)k]] = g.ew[(size_t)k];
            if (a < g.col[(size_t)k]) heap.emplace(-g.ew[(size_t)k], a, g.col[(size_t)k]);
        }
    std::vector<int64_t> weight(g.nw);
    std::vector<char> alive(K, 1);
    std::vector<int32_t> into(K);
    for (int32_t c = 0; c < K; ++c) into[c] = c;
    int32_t n_alive = K;
    auto absorb = [&](int32_t a, int32_t b) {                   // b disappears into a (a < b)
        weight[a] += weight[b];
        weight[b] = 0;
        alive[b] = 0;
        into[b] = a;
        --n_alive;
    };
    // Weights of a pair only change by a merge, which pushes the new value; weights of nodes only grow, so a pair
    // that once did not fit never fits later.  An entry is current if both ends live and the weight is the stored one.
    while (n_alive > M && !heap.empty()) {
        const Entry top = heap.top();
        heap.pop();
        const int32_t a = std::get<1>(top), b = std::get<2>(top);
        if (!alive[a] || !alive[b]) continue;
        auto it = adj[a].find(b);
        if (it == adj[a].end() || it->second != -std::get<0>(top)) continue;
        if (weight[a] + weight[b] > cap) continue;
        for (const auto& kv : adj[b]) {
            const int32_t x = kv.first;
            if (x == a) continue;
            const int64_t w = (adj[a][x] += kv.second);
            adj[x].erase(b);
            adj[x][a] = w;
            heap.emplace(-w, std::min(a, x), std::max(a, x));
        }
        adj[a].erase(b);
        adj[b].clear();
        absorb(a, b);
    }
    while (n_alive > M) {
        int32_t s0 = -1, s1 = -1;                               // lightest and second lightest by (weight, number)
        for (int32_t c = 0; c < K; ++c) {
            if (!alive[c]) continue;
            if (s0 < 0 || weight[c] < weight[s0]) { s1 = s0; s0 = c; }
            else if (s1 < 0 || weight[c] < weight[s1]) s1 = c;
        }
        absorb(std::min(s0, s1), std::max(s0, s1));
    }
    std::vector<int32_t> community(K, -1);
    int32_t n_comm = 0;
    for (int32_t c = 0; c < K; ++c)
        if (alive[c]) community[c] = n_comm++;
    std::vector<int32_t> out(K);
    for (int32_t c = 0; c < K; ++c) {
        int32_t r = c;
        while (into[r] != r) r = into[r];
        out[c] = community[r];
    }
    return out;
}

}  // namespace

std::string partition_graph(int64_t N, int64_t n_edges, const int32_t* src, const int32_t* dst, int32_t M,
                            int32_t* comm) {
    if (N < 1 || N > INT32_MAX) return "N must be in [1, 2^31)";
    if (M < 1) return "M must be positive";
    if (n_edges < 0) return "n_edges must be non-negative";
    if (n_edges > 0 && (!src || !dst)) return "src/dst are null";
    if (!comm) return "comm is null";
    for (int64_t e = 0; e < n_edges; ++e)
        if (src[e] < 0 || src[e] >= N || dst[e] < 0 || dst[e] >= N) return "edge endpoint out of range";
    const Level finest = finest_level(N, n_edges, src, dst);
    const int64_t cap = (N + M - 1) / M + (N / M) / 20 + 1;

    // levels: propagate until at rest, contract
    std::vector<std::vector<int32_t>> chain;      // chain[i][v] = node of level i+1 that node v of level i went into
    Level coarse;                                 // the current level once it is no longer the finest
    const Level* g = &finest;
    std::vector<int32_t> label, want;
    std::vector<int64_t> size, granted;
    while (g->n > M) {
        const int64_t n = g->n;
        label.resize(n);
        want.resize(n);
        granted.assign(n, 0);
        size = g->nw;
        for (int64_t v = 0; v < n; ++v) label[v] = (int32_t)v;
        int quiet = 0;
        for (int r = 0; r < kPartitionMaxRounds && quiet < 2; ++r)
            quiet = propagation_round(*g, label, size, cap, r, want, granted) == 0 ? quiet + 1 : 0;
        chain.emplace_back();
        Level next = contract(*g, label, chain.back());
        const bool stalled = 20 * next.n > 19 * n;
        coarse = std::move(next);
        g = &coarse;
        if (stalled) break;
    }
    const std::vector<int32_t> top = merge_down_to(*g, M, cap);

    // back to the finest graph, then polish the borders
    label.resize(N);
    for (int64_t v = 0; v < N; ++v) {
        int32_t c = (int32_t)v;
        for (const auto& member_of : chain) c = member_of[c];
        label[v] = top[c];
    }
    want.resize(N);
    size.assign(M, 0);
    granted.assign(M, 0);
    for (int64_t v = 0; v < N; ++v) size[label[v]]++;
    int quiet = 0;
    for (int r = 0; r < kPartitionMaxRounds && quiet < 2; ++r)
        quiet = propagation_round(finest, label, size, cap, r, want, granted) == 0 ? quiet + 1 : 0;
    for (int64_t v = 0; v < N; ++v) comm[v] = label[v];
    return std::string();
}

}  // namespace cadmm
