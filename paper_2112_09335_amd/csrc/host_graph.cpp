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

// Stored class of a row with len entries (see RowSchedule): -1 = split.
int stored_class(int64_t len) {
    if (len > kSplitThreshold) return -1;
    int k = 0;
    while (k < kLengthClasses - 1 && (int64_t)(4 << k) < len) ++k;     // smallest k with 4 * 2^k >= len, at most 7
    return kLengthClasses - 1 - k;
}

// Row r of the list has the entries [lo[r], hi[r]) of col / val and goes to output row out[r] (r if out is null).
void make_schedule(RowSchedule& rs, int64_t nrows, const int64_t* lo, const int64_t* hi, const int32_t* out,
                   const int32_t* col, const float* val) {
    rs = RowSchedule();
    int64_t count[kLengthClasses + 1] = {};
    int64_t n_long = 0, total = 0;
    for (int64_t r = 0; r < nrows; ++r) {
        const int j = stored_class(hi[r] - lo[r]);
        if (j < 0) ++n_long; else ++count[j + 1];
        total += hi[r] - lo[r];
    }
    for (int j = 0; j < kLengthClasses; ++j) count[j + 1] += count[j];
    for (int j = 0; j <= kLengthClasses; ++j) rs.class_start[j] = count[j];
    const int64_t n_sched = nrows - n_long;
    std::vector<int64_t> src((size_t)n_sched);                 // list row of scheduled row i
    std::vector<int64_t> long_src;
    {
        int64_t cur[kLengthClasses];
        for (int j = 0; j < kLengthClasses; ++j) cur[j] = count[j];
        for (int64_t r = 0; r < nrows; ++r) {
            const int j = stored_class(hi[r] - lo[r]);
            if (j < 0) long_src.push_back(r); else src[(size_t)cur[j]++] = r;
        }
    }
    rs.ptr.assign((size_t)n_sched + 1, 0);
    rs.out.resize((size_t)n_sched);
    for (int64_t i = 0; i < n_sched; ++i) {
        const int64_t r = src[(size_t)i];
        rs.ptr[(size_t)i + 1] = rs.ptr[(size_t)i] + (hi[r] - lo[r]);
        rs.out[(size_t)i] = out ? out[r] : (int32_t)r;
    }
    rs.col.resize((size_t)total);
    rs.val.resize((size_t)total);
    parallel_rows(n_sched, [&](int64_t i0, int64_t i1) {
        for (int64_t i = i0; i < i1; ++i) {
            const int64_t r = src[(size_t)i], to = rs.ptr[(size_t)i], n = hi[r] - lo[r];
            for (int64_t k = 0; k < n; ++k) {
                rs.col[(size_t)(to + k)] = col[lo[r] + k];
                rs.val[(size_t)(to + k)] = val[lo[r] + k];
            }
        }
    });
    int64_t to = rs.ptr[(size_t)n_sched];
    rs.longs.long_part_ptr.push_back(0);
    for (int64_t r : long_src) {
        const int64_t n = hi[r] - lo[r];
        for (int64_t k = 0; k < n; ++k) {
            rs.col[(size_t)(to + k)] = col[lo[r] + k];
            rs.val[(size_t)(to + k)] = val[lo[r] + k];
        }
        for (int64_t p = to; p < to + n; p += kSplitPart) {
            rs.longs.part_lo.push_back(p);
            rs.longs.part_hi.push_back(p + kSplitPart < to + n ? p + kSplitPart : to + n);
        }
        rs.longs.long_row.push_back(out ? out[r] : (int32_t)r);
        rs.longs.long_part_ptr.push_back((int32_t)rs.longs.part_lo.size());
        to += n;
    }
}

// What the aggregation kernel relies on: every scheduled row and every part is an in-range, non-negative entry
// range, a row sits in the class that bounds its length, outputs are in range.
bool schedule_ok(const RowSchedule& rs, int64_t n_out) {
    const int64_t n = rs.n_rows(), total = (int64_t)rs.col.size();
    if ((int64_t)rs.ptr.size() != n + 1 || rs.val.size() != rs.col.size()) return false;
    if (rs.class_start[0] != 0 || rs.class_start[kLengthClasses] != n) return false;
    for (int j = 0; j < kLengthClasses; ++j) {
        if (rs.class_start[j] > rs.class_start[j + 1]) return false;
        const int64_t cap = j == 0 ? kSplitThreshold : (int64_t)(4 << (kLengthClasses - 1 - j));
        for (int64_t i = rs.class_start[j]; i < rs.class_start[j + 1]; ++i) {
            const int64_t len = rs.ptr[(size_t)i + 1] - rs.ptr[(size_t)i];
            if (len < 0 || len > cap) return false;
        }
    }
    if (n > 0 && (rs.ptr[0] != 0 || rs.ptr[(size_t)n] > total)) return false;
    for (int64_t i = 0; i < n; ++i)
        if (rs.out[(size_t)i] < 0 || rs.out[(size_t)i] >= n_out) return false;
    const LongRows& lr = rs.longs;
    if (lr.part_lo.size() != lr.part_hi.size() || lr.long_part_ptr.size() != lr.long_row.size() + 1) return false;
    for (size_t p = 0; p < lr.part_lo.size(); ++p)
        if (lr.part_lo[p] < 0 || lr.part_lo[p] >= lr.part_hi[p] || lr.part_hi[p] > total ||
            lr.part_hi[p] - lr.part_lo[p] > kSplitPart) return false;
    for (size_t i = 0; i < lr.long_row.size(); ++i)
        if (lr.long_row[i] < 0 || lr.long_row[i] >= n_out || lr.long_part_ptr[i] >= lr.long_part_ptr[i + 1] ||
            lr.long_part_ptr[i + 1] > (int32_t)lr.part_lo.size()) return false;
    return true;
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
    g.row_seg_ptr.assign(seg_cnt.begin(), seg_cnt.end());
    g.seg_pos.resize((size_t)g.n_seg);
    for (int64_t j = 0; j < g.n_seg; ++j) g.seg_pos[(size_t)g.segc_order[(size_t)j]] = (int32_t)j;

    make_schedule(g.row_sched, N, g.row_ptr.data(), g.row_ptr.data() + 1, nullptr, g.col.data(), g.val.data());
    {
        std::vector<int64_t> mlo, mhi;
        std::vector<int32_t> mpos;
        for (int64_t j = 0; j < g.n_seg; ++j) {
            const int64_t s = g.segc_order[(size_t)j];
            const int64_t lo = g.seg_ptr[(size_t)s], hi = g.seg_ptr[(size_t)s + 1];
            if (hi - lo == 1) {
                g.seg1_pos.push_back((int32_t)j);
                g.seg1_col.push_back(g.col[(size_t)lo]);
                g.seg1_val.push_back(g.val[(size_t)lo]);
            } else {
                mlo.push_back(lo);
                mhi.push_back(hi);
                mpos.push_back((int32_t)j);
            }
        }
        make_schedule(g.seg_sched, (int64_t)mpos.size(), mlo.data(), mhi.data(), mpos.data(), g.col.data(), g.val.data());
    }

    if (!schedule_ok(g.row_sched, N) || !schedule_ok(g.seg_sched, g.n_seg)) return "internal error: row schedule";

    // reduction chunks: for every community its own rows, then its segments
    g.unit_chunk_ptr.assign(M + 1, 0);
    for (int32_t m = 0; m < M; ++m) {
        for (int64_t b = g.comm_row_ptr[m]; b < g.comm_row_ptr[m + 1]; b += chunk_rows)
            g.chunks.push_back({m, 0, (int32_t)b, (int32_t)std::min<int64_t>(b + chunk_rows, g.comm_row_ptr[m + 1])});
        // a segment carries a row of the next, usually much narrower layer: eight times as many per chunk, so that a
        // chunk's fixed costs (unit state, block reductions) do not outweigh its pass over memory
        const int64_t chunk_segs = (int64_t)chunk_rows * 8;
        for (int64_t b = g.segc_comm_ptr[m]; b < g.segc_comm_ptr[m + 1]; b += chunk_segs)
            g.chunks.push_back({m, 1, (int32_t)b, (int32_t)std::min<int64_t>(b + chunk_segs, g.segc_comm_ptr[m + 1])});
        g.unit_chunk_ptr[m + 1] = (int32_t)g.chunks.size();
    }
    return "";
}

}  // namespace cadmm
