// Host-side graph structures of the community-blocked ADMM library (integer work, done once).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace cadmm {

// Work unit of the per-community reductions of the Z step-size search: a run of rows of one
// community (kind 0) or a run of that community's segments in (community,row) order (kind 1).
struct Chunk {
    int32_t unit;    // community
    int32_t kind;    // 0 = own rows, 1 = segments
    int32_t begin;   // first row / first segment (index into the (community,row)-sorted list)
    int32_t end;     // one past the last
};

constexpr int kSplitThreshold = 384;   // rows with more entries are split ...
constexpr int kSplitPart = 256;        // ... into parts of at most this many entries
constexpr int kChunkEntries = 8;       // entries per chunk = gathers a lane group keeps in flight

// A row list laid out for the aggregation kernels.
// Entries: (column, value) pairs of 8 bytes, in chunks of kChunkEntries pairs (64 bytes, what a lane group gathers in
// one trip): a row's entries fill consecutive chunks, the last one padded with (the row's first column, 0.0f), so
// that a kernel never has to mask an entry.  Chunk 0 holds only padding and stands in for chunks past a row's end.
// Rows: one record (first chunk, one past the last chunk, output row, 0) per scheduled row.  The rows that are not
// split are sorted by (group, length class): the group is the community whose rows of the gathered matrix the list
// row reads most (its own community for a CSR row, the neighbour community for a (row, community) segment), and
// inside a group the longest class comes first; stored class j holds the rows with at most
// 4 * 2^(kLengthClasses-1-j) entries that fit no later class (stored class 0: everything longer, up to the split
// threshold).  A maximal stretch of one (group, class) is a run.  A launch walks the runs in order, one group after
// the other, so that the part of the gathered matrix a group reads (a few MB at narrow widths) is fetched into an
// XCD's L2 once and not once per class, and gives every run as many lanes per row as rows of its class can use.
// Rows longer than the split threshold (power-law hubs) are cut into parts of kSplitPart entries; a part is listed
// after the scheduled rows, as record n_rows + part index with the part index as its output row (a row of a side
// buffer), and a split row's parts are added in order by a combine kernel: deterministic, no atomics.
constexpr int kLengthClasses = 8;
struct ScheduleRun {
    int64_t row0, row1;      // scheduled rows [row0, row1)
    int32_t cls;             // stored length class
    int32_t group;
};
struct RowRecord { int32_t chunk0, chunk1, out, pad; };     // 16 bytes: one load per row
struct EntryPair { int32_t col; float val; };
struct RowSchedule {
    std::vector<RowRecord> rec;                  // [n_rows + n_parts]
    std::vector<EntryPair> ent;                  // [n_chunks * kChunkEntries]
    std::vector<ScheduleRun> runs;               // in order; they tile [0, n_rows)
    int64_t n_sched = 0;                         // scheduled (unsplit) rows
    std::vector<int32_t> long_row;               // [n_long] output row of a split row
    std::vector<int32_t> long_part_ptr;          // [n_long+1] its parts (indices into the side buffer)
    int64_t n_rows() const { return n_sched; }
    int64_t n_parts() const { return (int64_t)rec.size() - n_sched; }
    int64_t n_long() const { return (int64_t)long_row.size(); }
    int64_t n_chunks() const { return (int64_t)(ent.size() / kChunkEntries); }
};

// Which scheduled rows a workgroup of the aggregation kernel takes, for one lane count per gathered row
// (2^lpr_log2 lanes).  A workgroup is four wavefronts; with 2^g lane groups per row it covers 4 * 64 >> (lpr_log2 + g)
// consecutive rows of one run.  g is the smallest count whose chunks (one per group and trip) cover the longest row
// of the run's class in one trip, at most what a wavefront holds.  The workgroups are listed in run order and
// cut into eight consecutive slices of about equal work, one per XCD (a launch gives workgroup b of XCD b mod 8 the
// (b / 8)-th workgroup of that XCD's slice), so that an XCD walks whole groups one after the other.  trips: how many
// times the lane groups of a row must each take one chunk to cover the longest row of the workgroup (group j of a
// row takes its chunks j, j + 2^g, ...).  The parts of split rows, a wavefront each, stand at the head of every slice.
struct BlockRows { int32_t row0, row1, g, trips; };   // 16 bytes: one scalar load per workgroup
struct BlockTable {
    std::vector<BlockRows> blocks;
    int64_t xcd_start[9] = {};                   // slice k: blocks [xcd_start[k], xcd_start[k+1])
};
void build_block_table(const RowSchedule& rs, int lpr_log2, BlockTable& out);
int64_t count_blocks(const RowSchedule& rs, int lpr_log2);
bool block_table_ok(const RowSchedule& rs, int lpr_log2, const BlockTable& bt);

struct HostGraph {
    int64_t N = 0, E = 0, nnz = 0, n_seg = 0, n_halo_rows = 0;
    int32_t M = 0;
    std::vector<int32_t> perm;          // [N] internal row -> caller id
    std::vector<int32_t> inv_perm;      // [N] caller id -> internal row
    std::vector<int64_t> comm_row_ptr;  // [M+1]
    std::vector<int32_t> row_comm;      // [N] community of an internal row
    std::vector<int64_t> row_ptr;       // [N+1]
    std::vector<int32_t> col;           // [nnz]
    std::vector<float>   val;           // [nnz]
    // segments, (row, community) order
    std::vector<int64_t> seg_ptr;       // [n_seg+1]
    std::vector<int32_t> seg_row;       // [n_seg]
    std::vector<int32_t> seg_comm;      // [n_seg]
    std::vector<uint8_t> neighbour;     // [M*M]
    // segments, (community, row) order
    std::vector<int64_t> segc_order;    // [n_seg] index into the (row, community) order
    std::vector<int32_t> segc_row;      // [n_seg]
    std::vector<int64_t> segc_comm_ptr; // [M+1]
    std::vector<int64_t> row_seg_ptr;   // [N+1] segments of a row in the (row, community) order
    std::vector<int32_t> seg_pos;       // [n_seg] position of that segment in the (community, row) order
    // the same segments by length: one with a single entry is a scaled copy of one gathered row (listed in the
    // (community, row) order); the others are aggregated like rows (seg_sched)
    std::vector<int32_t> seg1_pos;      // [n_seg1] position of the segment in the (community, row) order
    std::vector<int32_t> seg1_col;      // [n_seg1] its entry
    std::vector<float>   seg1_val;      // [n_seg1]
    RowSchedule row_sched;              // the CSR rows; output row = the row, group = its community
    RowSchedule seg_sched;              // the segments with several entries; output row = position in the (community, row) order,
                                        // group = the segment's community
    // reduction chunks for the Z search, grouped by community: many segments per chunk for a narrow next layer ...
    std::vector<Chunk>   chunks;
    std::vector<int32_t> unit_chunk_ptr; // [M+1]
    // ... and the same with as many segments as rows per chunk, for a wide one
    std::vector<Chunk>   chunks_wide;
    std::vector<int32_t> unit_chunk_ptr_wide;
};

// Returns an empty string on success, an error text otherwise.
std::string build_host_graph(HostGraph& g, int64_t N, int64_t n_edges, const int32_t* src,
                             const int32_t* dst, int32_t M, const int32_t* comm, int chunk_rows);

}  // namespace cadmm
