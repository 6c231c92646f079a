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

// Row r of the list has the entries [lo[r], hi[r]) of col / val, belongs to group grp[r] (n_groups groups) and goes
// to output row out[r] (r if out is null).
void make_schedule(RowSchedule& rs, int64_t nrows, const int64_t* lo, const int64_t* hi, const int32_t* out,
                   const int32_t* grp, int32_t n_groups, const int32_t* col, const float* val) {
    rs = RowSchedule();
    // counting sort on (group, class)
    const size_t nkeys = (size_t)n_groups * kLengthClasses;
    std::vector<int64_t> count(nkeys + 1, 0);
    int64_t n_long = 0;
    for (int64_t r = 0; r < nrows; ++r) {
        const int j = stored_class(hi[r] - lo[r]);
        if (j < 0) ++n_long; else ++count[(size_t)grp[r] * kLengthClasses + j + 1];
    }
    for (size_t k = 0; k < nkeys; ++k) count[k + 1] += count[k];
    for (size_t k = 0; k < nkeys; ++k)
        if (count[k + 1] > count[k])
            rs.runs.push_back({count[k], count[k + 1], (int32_t)(k % kLengthClasses), (int32_t)(k / kLengthClasses)});
    const int64_t n_sched = nrows - n_long;
    rs.n_sched = n_sched;
    std::vector<int64_t> src((size_t)n_sched);                 // list row of scheduled row i
    std::vector<int64_t> long_src;
    {
        std::vector<int64_t> cur(count.begin(), count.end() - 1);
        for (int64_t r = 0; r < nrows; ++r) {
            const int j = stored_class(hi[r] - lo[r]);
            if (j < 0) long_src.push_back(r); else src[(size_t)cur[(size_t)grp[r] * kLengthClasses + j]++] = r;
        }
    }
    // records and chunk ranges: chunk 0 is the padding chunk, then the scheduled rows, then the parts of split rows
    auto chunks_of = [](int64_t len) { return (len + kChunkEntries - 1) / kChunkEntries; };
    int64_t n_parts = 0;
    for (int64_t r : long_src) n_parts += (hi[r] - lo[r] + kSplitPart - 1) / kSplitPart;
    rs.rec.resize((size_t)(n_sched + n_parts));
    int64_t at = 1;
    for (int64_t i = 0; i < n_sched; ++i) {
        const int64_t r = src[(size_t)i];
        const int64_t nc = chunks_of(hi[r] - lo[r]);
        rs.rec[(size_t)i] = {(int32_t)at, (int32_t)(at + nc), out ? out[r] : (int32_t)r, 0};
        at += nc;
    }
    std::vector<int64_t> part_lo, part_hi;                     // entry ranges of the parts in col / val
    rs.long_part_ptr.push_back(0);
    for (int64_t r : long_src) {
        for (int64_t p = lo[r]; p < hi[r]; p += kSplitPart) {
            const int64_t p1 = p + kSplitPart < hi[r] ? p + kSplitPart : hi[r];
            const int64_t nc = chunks_of(p1 - p);
            const int64_t k = (int64_t)part_lo.size();
            rs.rec[(size_t)(n_sched + k)] = {(int32_t)at, (int32_t)(at + nc), (int32_t)k, 0};
            part_lo.push_back(p);
            part_hi.push_back(p1);
            at += nc;
        }
        rs.long_row.push_back(out ? out[r] : (int32_t)r);
        rs.long_part_ptr.push_back((int32_t)part_lo.size());
    }
    rs.ent.assign((size_t)at * kChunkEntries, EntryPair{0, 0.f});
    auto fill = [&](const RowRecord& rec, int64_t p0, int64_t p1) {
        EntryPair* e = rs.ent.data() + (size_t)rec.chunk0 * kChunkEntries;
        const int64_t n = p1 - p0, padded = (int64_t)(rec.chunk1 - rec.chunk0) * kChunkEntries;
        for (int64_t k = 0; k < n; ++k) e[k] = {col[p0 + k], val[p0 + k]};
        for (int64_t k = n; k < padded; ++k) e[k] = {n > 0 ? col[p0] : 0, 0.f};
    };
    parallel_rows(n_sched, [&](int64_t i0, int64_t i1) {
        for (int64_t i = i0; i < i1; ++i) fill(rs.rec[(size_t)i], lo[src[(size_t)i]], hi[src[(size_t)i]]);
    });
    for (int64_t k = 0; k < n_parts; ++k) fill(rs.rec[(size_t)(n_sched + k)], part_lo[(size_t)k], part_hi[(size_t)k]);
}

// What the aggregation kernels rely on: every record names an in-range, non-empty chunk range past the padding chunk,
// the chunk ranges tile the entry array in order, the runs tile the scheduled rows and a row sits in a run whose
// class bounds its length, a part is no longer than kSplitPart, output rows are in range, every column is in range.
bool schedule_ok(const RowSchedule& rs, int64_t n_out, int64_t n_cols) {
    const int64_t n = rs.n_rows(), np = rs.n_parts(), nchunks = rs.n_chunks();
    if (n < 0 || np < 0 || nchunks < 1 || nchunks > INT32_MAX || rs.ent.size() % kChunkEntries != 0) return false;
    int64_t at = 1;
    for (int64_t i = 0; i < n + np; ++i) {
        const RowRecord& r = rs.rec[(size_t)i];
        if (r.chunk0 != at || r.chunk1 <= r.chunk0 || r.chunk1 > nchunks) return false;
        if (r.out < 0 || r.out >= (i < n ? n_out : np)) return false;
        if (i >= n && (int64_t)(r.chunk1 - r.chunk0) * kChunkEntries > kSplitPart) return false;
        at = r.chunk1;
    }
    if (at != nchunks) return false;
    for (const EntryPair& e : rs.ent)
        if (e.col < 0 || e.col >= n_cols) return false;
    int64_t row = 0;
    for (const ScheduleRun& run : rs.runs) {
        if (run.row0 != row || run.row1 <= run.row0 || run.cls < 0 || run.cls >= kLengthClasses) return false;
        const int64_t cap = run.cls == 0 ? kSplitThreshold : (int64_t)(4 << (kLengthClasses - 1 - run.cls));
        const int64_t cap_chunks = (cap + kChunkEntries - 1) / kChunkEntries;
        for (int64_t i = run.row0; i < run.row1; ++i)
            if (rs.rec[(size_t)i].chunk1 - rs.rec[(size_t)i].chunk0 > cap_chunks) return false;
        row = run.row1;
    }
    if (row != n) return false;
    if (rs.long_part_ptr.size() != rs.long_row.size() + 1) return false;
    for (size_t i = 0; i < rs.long_row.size(); ++i)
        if (rs.long_row[i] < 0 || rs.long_row[i] >= n_out || rs.long_part_ptr[i] >= rs.long_part_ptr[i + 1] ||
            rs.long_part_ptr[i + 1] > (int32_t)np) return false;
    if (!rs.long_part_ptr.empty() && rs.long_part_ptr.back() != (int32_t)np) return false;
    return true;
}

// lane groups per row (log2) for the rows of stored class cls when a gathered row takes 2^lpr_log2 lanes
int groups_log2(int cls, int lpr_log2) {
    const int g_max = 6 - lpr_log2;
    if (cls == 0) return g_max;
    int g = 0;
    while (g < g_max && (kChunkEntries << g) < (4 << (kLengthClasses - 1 - cls))) ++g;
    return g;
}

}  // namespace

int64_t count_blocks(const RowSchedule& rs, int lpr_log2) {
    int64_t n = (rs.n_parts() + 3) / 4;                 // a part takes a whole wavefront, four per workgroup
    for (const ScheduleRun& run : rs.runs) {
        const int64_t per = 4LL << (6 - lpr_log2 - groups_log2(run.cls, lpr_log2));
        n += (run.row1 - run.row0 + per - 1) / per;
    }
    return n;
}

void build_block_table(const RowSchedule& rs, int lpr_log2, BlockTable& out) {
    const int64_t n_rows = rs.n_rows(), n_parts = rs.n_parts();
    const int g_max = 6 - lpr_log2;
    auto chunks = [&](int64_t i) { return (int64_t)(rs.rec[(size_t)i].chunk1 - rs.rec[(size_t)i].chunk0); };
    auto trips_for = [](int64_t longest_chunks, int g) { return (int32_t)std::max<int64_t>(1, (longest_chunks + (1LL << g) - 1) >> g); };
    auto block_of = [&](int64_t r, int64_t r1, int g, double& cost) {
        int64_t longest = 0, total = 0;
        for (int64_t i = r; i < r1; ++i) { longest = std::max(longest, chunks(i)); total += chunks(i); }
        cost = (double)(total * kChunkEntries) + 8.0 * (double)(r1 - r);     // its entries, plus a fixed share per row
        return BlockRows{(int32_t)r, (int32_t)r1, g, trips_for(longest, g)};
    };
    // the parts of split rows, dealt round-robin to the XCDs; they come first in every slice, so that the longest
    // pieces of work do not form the tail of a launch
    std::vector<BlockRows> parts[8];
    double part_cost[8] = {}, total = 0.0, c = 0.0;
    for (int64_t p = 0, b = 0; p < n_parts; p += 4, ++b) {
        parts[b & 7].push_back(block_of(n_rows + p, n_rows + std::min(p + 4, n_parts), g_max, c));
        part_cost[b & 7] += c;
        total += c;
    }
    // the scheduled rows in run order
    std::vector<BlockRows> rows;
    std::vector<double> cost;
    rows.reserve((size_t)count_blocks(rs, lpr_log2));
    cost.reserve(rows.capacity());
    for (const ScheduleRun& run : rs.runs) {
        const int g = groups_log2(run.cls, lpr_log2);
        const int64_t per = 4LL << (6 - lpr_log2 - g);
        for (int64_t r = run.row0; r < run.row1; r += per) {
            rows.push_back(block_of(r, std::min(r + per, run.row1), g, c));
            cost.push_back(c);
            total += c;
        }
    }
    // slice k: its parts, then consecutive row workgroups until it holds an eighth of the work
    out.blocks.clear();
    out.blocks.reserve(rows.size() + (size_t)((n_parts + 3) / 4));
    const int64_t nb = (int64_t)rows.size();
    int64_t b = 0;
    double done = 0.0;                    // work handed out so far, parts included
    for (int k = 0; k < 8; ++k) {
        out.xcd_start[k] = (int64_t)out.blocks.size();
        out.blocks.insert(out.blocks.end(), parts[k].begin(), parts[k].end());
        done += part_cost[k];
        const double want = total * (k + 1) / 8.0;
        while (b < nb && (k == 7 || done + 0.5 * cost[(size_t)b] < want)) {
            out.blocks.push_back(rows[(size_t)b]);
            done += cost[(size_t)b++];
        }
    }
    out.xcd_start[8] = (int64_t)out.blocks.size();
}

// What the kernels' row mapping relies on: every scheduled row and every part is in exactly one workgroup, no
// workgroup mixes the two or holds more rows than four wavefronts cover with its lane groups, its trip count covers
// its longest row, and the XCD slices tile the table.
bool block_table_ok(const RowSchedule& rs, int lpr_log2, const BlockTable& bt) {
    const int64_t n_rows = rs.n_rows(), n_parts = rs.n_parts();
    if (n_rows + n_parts > INT32_MAX) return false;
    std::vector<BlockRows> sorted(bt.blocks);
    std::sort(sorted.begin(), sorted.end(), [](const BlockRows& a, const BlockRows& b) { return a.row0 < b.row0; });
    int64_t at = 0;
    for (const BlockRows& b : sorted) {
        if (b.row0 != at || b.row1 <= b.row0 || b.g < 0 || lpr_log2 + b.g > 6 || b.trips < 1) return false;
        if ((int64_t)b.row1 - b.row0 > (4LL << (6 - lpr_log2 - b.g))) return false;
        if (b.row0 < n_rows && b.row1 > n_rows) return false;
        for (int64_t i = b.row0; i < b.row1; ++i)
            if ((int64_t)(rs.rec[(size_t)i].chunk1 - rs.rec[(size_t)i].chunk0) > ((int64_t)b.trips << b.g)) return false;
        at = b.row1;
    }
    if (at != n_rows + n_parts) return false;
    if (bt.xcd_start[0] != 0 || bt.xcd_start[8] != (int64_t)bt.blocks.size()) return false;
    for (int k = 0; k < 8; ++k)
        if (bt.xcd_start[k] > bt.xcd_start[k + 1]) return false;
    return true;
}

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

    make_schedule(g.row_sched, N, g.row_ptr.data(), g.row_ptr.data() + 1, nullptr, g.row_comm.data(), M, g.col.data(),
                  g.val.data());
    {
        std::vector<int64_t> mlo, mhi;
        std::vector<int32_t> mpos, mgrp;
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
                mgrp.push_back(g.seg_comm[(size_t)s]);
            }
        }
        make_schedule(g.seg_sched, (int64_t)mpos.size(), mlo.data(), mhi.data(), mpos.data(), mgrp.data(), M, g.col.data(),
                      g.val.data());
    }

    if (!schedule_ok(g.row_sched, N, N) || !schedule_ok(g.seg_sched, g.n_seg, N)) return "internal error: row schedule";
    for (int l = 0; l < 7; ++l) {
        BlockTable bt;
        for (const RowSchedule* rs : {&g.row_sched, &g.seg_sched}) {
            build_block_table(*rs, l, bt);
            if (!block_table_ok(*rs, l, bt) || (int64_t)bt.blocks.size() != count_blocks(*rs, l))
                return "internal error: workgroup table of the aggregation";
        }
    }

    // reduction chunks: for every community its own rows, then its segments.  A segment carries a row of the next
    // layer: where that layer is narrow, eight times as many segments as rows go into a chunk, so that a chunk's fixed
    // costs (unit state, block reductions) do not outweigh its pass over memory; where it is wide, as many as rows, or
    // the few heavy chunks of a community are what the launch waits for.
    auto build_chunks = [&](int64_t chunk_segs, std::vector<Chunk>& chunks, std::vector<int32_t>& ptr) {
        chunks.clear();
        ptr.assign(M + 1, 0);
        for (int32_t m = 0; m < M; ++m) {
            for (int64_t b = g.comm_row_ptr[m]; b < g.comm_row_ptr[m + 1]; b += chunk_rows)
                chunks.push_back({m, 0, (int32_t)b, (int32_t)std::min<int64_t>(b + chunk_rows, g.comm_row_ptr[m + 1])});
            for (int64_t b = g.segc_comm_ptr[m]; b < g.segc_comm_ptr[m + 1]; b += chunk_segs)
                chunks.push_back({m, 1, (int32_t)b, (int32_t)std::min<int64_t>(b + chunk_segs, g.segc_comm_ptr[m + 1])});
            ptr[m + 1] = (int32_t)chunks.size();
        }
    };
    build_chunks((int64_t)chunk_rows * 8, g.chunks, g.unit_chunk_ptr);
    build_chunks((int64_t)chunk_rows, g.chunks_wide, g.unit_chunk_ptr_wide);
    return "";
}

}  // namespace cadmm
