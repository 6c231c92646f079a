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

// Rows of a row list (CSR rows, or segments) that are too long for one lane group are cut into parts;
// each part is aggregated like an ordinary row into a side buffer and the parts of a row are then
// added in order (deterministic, no atomics).
struct LongRows {
    std::vector<int64_t> part_lo, part_hi;   // [n_parts] entry range of a part
    std::vector<int32_t> long_row;           // [n_long] index of the split row in its row list
    std::vector<int32_t> long_part_ptr;      // [n_long+1] parts of a split row
    int64_t n_parts() const { return (int64_t)part_lo.size(); }
    int64_t n_long() const { return (int64_t)long_row.size(); }
};

constexpr int kSplitThreshold = 384;   // rows with more entries are split ...
constexpr int kSplitPart = 256;        // ... into parts of at most this many entries

// A row list laid out for the aggregation kernel.  The rows that are not split are grouped into kLengthClasses
// length classes, the longest class first, in the list's order inside a class: stored class j holds the rows
// with at most 4 * 2^(kLengthClasses-1-j) entries that fit no later class (stored class 0: everything longer, up to
// the split threshold).  A launch can then give every class as many lanes per row as its rows can use, so that
// few lanes of a gather instruction stay idle.  The entries are copied in the same order, those of the split
// rows after them, so that a launch reads col and val front to back.
constexpr int kLengthClasses = 8;
struct RowSchedule {
    std::vector<int64_t> ptr;                    // [n_rows+1] entries of scheduled row i: [ptr[i], ptr[i+1])
    std::vector<int32_t> out;                    // [n_rows] output row of scheduled row i
    std::vector<int32_t> col;                    // [entries of the list]
    std::vector<float>   val;
    int64_t class_start[kLengthClasses + 1] = {};   // scheduled rows of stored class j: [class_start[j], class_start[j+1])
    LongRows longs;                              // split rows: part ranges in col / val, long_row = the output row
    int64_t n_rows() const { return (int64_t)out.size(); }
};

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
    RowSchedule row_sched;              // the CSR rows; output row = the row
    RowSchedule seg_sched;              // the segments with several entries; output row = position in the (community, row) order
    // reduction chunks for the Z search, grouped by community
    std::vector<Chunk>   chunks;
    std::vector<int32_t> unit_chunk_ptr; // [M+1]
};

// Returns an empty string on success, an error text otherwise.
std::string build_host_graph(HostGraph& g, int64_t N, int64_t n_edges, const int32_t* src,
                             const int32_t* dst, int32_t M, const int32_t* comm, int chunk_rows);

}  // namespace cadmm
