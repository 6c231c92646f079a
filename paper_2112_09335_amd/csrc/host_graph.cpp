// Graph construction on the host: symmetric simple graph -> community-contiguous numbering ->
// CSR of the normalised adjacency -> per-row community segments (paper, Section 2).
#include "host_graph.h"

#include <algorithm>
#include <cmath>
#include <thread>

namespace cadmm {

namespace {

template <class F>
void parallel_rows(int64_t n, F f) {
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<int64_t>(std::max(1u, std::min(hw, 16u)), std::max<int64_t>(1, n / 4096));
    if (nt <= 1) { f(0, n); return; }
    std::vector<std::thread> th;
    int64_t per = (n + nt - 1) / nt;
    for (int t = 0; t < nt; ++t) {
        int64_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        th.emplace_back([=] { f(lo, hi); });
    }
    for (auto& x : th) x.join();
}

void split_long(LongRows& lr, const int64_t* lo, const int64_t* hi, int64_t nrows) {
    lr = LongRows();
    lr.long_part_ptr.push_back(0);
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t len = hi[r] - lo[r];
        if (len <= kSplitThreshold) continue;
        for (int64_t p = lo[r]; p < hi[r]; p += kSplitPart) {
            lr.part_lo.push_back(p);
            lr.part_hi.push_back(p + kSplitPart < hi[r] ? p + kSplitPart : hi[r]);
        }
        lr.long_row.push_back((int32_t)r);
        lr.long_part_ptr.push_back((int32_t)lr.part_lo.size());
    }
}

}  // namespace

std::string build_host_graph(HostGraph& g, int64_t N, int64_t n_edges, const int32_t* src,
                             const int32_t* dst, int32_t M, const int32_t* comm, int chunk_rows) {
    if (N < 1 || N > INT32_MAX) return "N must be in [1, 2^31)";
    if (M < 1) return "M must be positive";
    if (n_edges < 0) return "n_edges must be non-negative";
    if (n_edges > 0 && (!src || !dst)) return "src/dst are null";
    for (int64_t e = 0; e < n_edges; ++e)
        if (src[e] < 0 || src[e] >= N || dst[e] < 0 || dst[e] >= N) return "edge endpoint out of range";
    g = HostGraph();
    g.N = N;
    g.M = M;

    // community of every caller node
    std::vector<int32_t> cm(N);
    if (comm) {
        for (int64_t i = 0; i < N; ++i) {
            if (comm[i] < 0 || comm[i] >= M) return "community id out of range";
            cm[i] = comm[i];
        }
    } else {
        int64_t chunk = (N + M - 1) / M;
        for (int64_t i = 0; i < N; ++i) cm[i] = (int32_t)(i / chunk);
    }

    // stable counting sort by community: internal numbering
    g.comm_row_ptr.assign(M + 1, 0);
    for (int64_t i = 0; i < N; ++i) g.comm_row_ptr[cm[i] + 1]++;
    for (int32_t m = 0; m < M; ++m) g.comm_row_ptr[m + 1] += g.comm_row_ptr[m];
    g.perm.resize(N);
    g.inv_perm.resize(N);
    {
        std::vector<int64_t> cur(g.comm_row_ptr.begin(), g.comm_row_ptr.end() - 1);
        for (int64_t i = 0; i < N; ++i) {
            int64_t r = cur[cm[i]]++;
            g.perm[r] = (int32_t)i;
            g.inv_perm[i] = (int32_t)r;
        }
    }
    g.row_comm.resize(N);
    for (int64_t r = 0; r < N; ++r) g.row_comm[r] = cm[g.perm[r]];

    // bucket both orientations by row (with repeats), then sort + unique inside every row
    std::vector<int64_t> cnt(N + 1, 0);
    for (int64_t e = 0; e < n_edges; ++e) {
        if (src[e] == dst[e]) continue;
        cnt[g.inv_perm[src[e]] + 1]++;
        cnt[g.inv_perm[dst[e]] + 1]++;
    }
    for (int64_t i = 0; i < N; ++i) cnt[i + 1] += cnt[i];
    std::vector<int32_t> raw((size_t)cnt[N]);
    {
        std::vector<int64_t> cur(cnt.begin(), cnt.end() - 1);
        for (int64_t e = 0; e < n_edges; ++e) {
            if (src[e] == dst[e]) continue;
            int32_t a = g.inv_perm[src[e]], b = g.inv_perm[dst[e]];
            raw[(size_t)cur[a]++] = b;
            raw[(size_t)cur[b]++] = a;
        }
    }
    std::vector<int32_t> deg(N);   // distinct neighbours
    parallel_rows(N, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i) {
            int32_t* b = raw.data() + cnt[i];
            int32_t* e = raw.data() + cnt[i + 1];
            std::sort(b, e);
            deg[i] = (int32_t)(std::unique(b, e) - b);
        }
    });
    g.row_ptr.assign(N + 1, 0);
    for (int64_t i = 0; i < N; ++i) g.row_ptr[i + 1] = g.row_ptr[i] + deg[i] + 1;   // + self loop
    g.nnz = g.row_ptr[N];
    g.E = (g.nnz - N) / 2;
    g.col.resize((size_t)g.nnz);
    g.val.resize((size_t)g.nnz);
    parallel_rows(N, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i) {
            const int32_t* b = raw.data() + cnt[i];
            int64_t o = g.row_ptr[i];
            bool self_done = false;
            for (int32_t k = 0; k < deg[i]; ++k) {
                if (!self_done && b[k] > i) { g.col[(size_t)o++] = (int32_t)i; self_done = true; }
                g.col[(size_t)o++] = b[k];
            }
            if (!self_done) g.col[(size_t)o++] = (int32_t)i;
            double di = (double)(deg[i] + 1);
            for (int64_t p = g.row_ptr[i]; p < g.row_ptr[i + 1]; ++p) {
                double dj = (double)(deg[g.col[(size_t)p]] + 1);
                g.val[(size_t)p] = (float)(1.0 / std::sqrt(di * dj));
            }
        }
    });
    std::vector<int32_t>().swap(raw);

    // segments in (row, community) order
    g.neighbour.assign((size_t)M * M, 0);
    std::vector<int64_t> seg_cnt(N + 1, 0);
    std::vector<uint8_t> halo(N, 0);
    parallel_rows(N, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i) {
            int32_t prev = -1;
            int64_t c = 0;
            for (int64_t p = g.row_ptr[i]; p < g.row_ptr[i + 1]; ++p) {
                int32_t cc = g.row_comm[g.col[(size_t)p]];
                if (cc != prev) { ++c; prev = cc; }
                if (cc != g.row_comm[i]) halo[i] = 1;
            }
            seg_cnt[i + 1] = c;
        }
    });
    for (int64_t i = 0; i < N; ++i) {
        seg_cnt[i + 1] += seg_cnt[i];
        g.n_halo_rows += halo[i];
    }
    g.n_seg = seg_cnt[N];
    if (g.n_seg > INT32_MAX) return "too many (row, community) segments";
    g.seg_ptr.resize((size_t)g.n_seg + 1);
    g.seg_row.resize((size_t)g.n_seg);
    g.seg_comm.resize((size_t)g.n_seg);
    for (int64_t i = 0; i < N; ++i) {
        int32_t prev = -1;
        int64_t s = seg_cnt[i] - 1;
        for (int64_t p = g.row_ptr[i]; p < g.row_ptr[i + 1]; ++p) {
            int32_t cc = g.row_comm[g.col[(size_t)p]];
            if (cc != prev) {
                ++s;
                g.seg_ptr[(size_t)s] = p;
                g.seg_row[(size_t)s] = (int32_t)i;
                g.seg_comm[(size_t)s] = cc;
                prev = cc;
                if (cc != g.row_comm[i]) g.neighbour[(size_t)g.row_comm[i] * M + cc] = 1;
            }
        }
    }
    g.seg_ptr[(size_t)g.n_seg] = g.nnz;

    // segments in (community, row) order: stable counting sort on the community
    g.segc_comm_ptr.assign(M + 1, 0);
    for (int64_t s = 0; s < g.n_seg; ++s) g.segc_comm_ptr[g.seg_comm[(size_t)s] + 1]++;
    for (int32_t m = 0; m < M; ++m) g.segc_comm_ptr[m + 1] += g.segc_comm_ptr[m];
    g.segc_order.resize((size_t)g.n_seg);
    g.segc_row.resize((size_t)g.n_seg);
    {
        std::vector<int64_t> cur(g.segc_comm_ptr.begin(), g.segc_comm_ptr.end() - 1);
        for (int64_t s = 0; s < g.n_seg; ++s) {
            int64_t j = cur[g.seg_comm[(size_t)s]]++;
            g.segc_order[(size_t)j] = s;
            g.segc_row[(size_t)j] = g.seg_row[(size_t)s];
        }
    }
    // The entries once more, in this order: a pass over the segments of a community then reads its column
    // indices and values front to back instead of one short piece out of every row.
    g.segc_ptr.assign((size_t)g.n_seg + 1, 0);
    for (int64_t j = 0; j < g.n_seg; ++j) {
        const int64_t s = g.segc_order[(size_t)j];
        g.segc_ptr[(size_t)j + 1] = g.segc_ptr[(size_t)j] + (g.seg_ptr[(size_t)s + 1] - g.seg_ptr[(size_t)s]);
    }
    g.segc_col.resize((size_t)g.nnz);
    g.segc_val.resize((size_t)g.nnz);
    parallel_rows(g.n_seg, [&](int64_t j0, int64_t j1) {
        for (int64_t j = j0; j < j1; ++j) {
            const int64_t s = g.segc_order[(size_t)j];
            const int64_t from = g.seg_ptr[(size_t)s], n = g.seg_ptr[(size_t)s + 1] - from, to = g.segc_ptr[(size_t)j];
            for (int64_t k = 0; k < n; ++k) {
                g.segc_col[(size_t)(to + k)] = g.col[(size_t)(from + k)];
                g.segc_val[(size_t)(to + k)] = g.val[(size_t)(from + k)];
            }
        }
    });

    g.row_seg_ptr.assign(seg_cnt.begin(), seg_cnt.end());
    g.seg_pos.resize((size_t)g.n_seg);
    for (int64_t j = 0; j < g.n_seg; ++j) g.seg_pos[(size_t)g.segc_order[(size_t)j]] = (int32_t)j;

    split_long(g.long_rows, g.row_ptr.data(), g.row_ptr.data() + 1, N);
    for (int64_t j = 0; j < g.n_seg; ++j) {
        const int64_t lo = g.segc_ptr[(size_t)j], hi = g.segc_ptr[(size_t)j + 1];
        if (hi - lo == 1) {
            g.seg1_pos.push_back((int32_t)j);
            g.seg1_col.push_back(g.segc_col[(size_t)lo]);
            g.seg1_val.push_back(g.segc_val[(size_t)lo]);
        } else {
            g.segm_ptr.push_back(lo);
            g.segm_end.push_back(hi);
            g.segm_pos.push_back((int32_t)j);
        }
    }
    split_long(g.long_segs, g.segm_ptr.data(), g.segm_end.data(), (int64_t)g.segm_ptr.size());
    for (auto& r : g.long_segs.long_row) r = g.segm_pos[(size_t)r];

    // reduction chunks: for every community its own rows, then its segments
    g.unit_chunk_ptr.assign(M + 1, 0);
    for (int32_t m = 0; m < M; ++m) {
        for (int64_t b = g.comm_row_ptr[m]; b < g.comm_row_ptr[m + 1]; b += chunk_rows)
            g.chunks.push_back({m, 0, (int32_t)b, (int32_t)std::min<int64_t>(b + chunk_rows, g.comm_row_ptr[m + 1])});
        for (int64_t b = g.segc_comm_ptr[m]; b < g.segc_comm_ptr[m + 1]; b += chunk_rows)
            g.chunks.push_back({m, 1, (int32_t)b, (int32_t)std::min<int64_t>(b + chunk_rows, g.segc_comm_ptr[m + 1])});
        g.unit_chunk_ptr[m + 1] = (int32_t)g.chunks.size();
    }
    return "";
}

}  // namespace cadmm
