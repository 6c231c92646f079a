// Built-in community partitioner (host side, integer work, done once before the graph is built).
#pragma once
#include <cstdint>
#include <string>

namespace cadmm {

constexpr int kPartitionMaxRounds = 100;    // propagation rounds per level and in the final refinement, unless two
                                            // rounds in a row move nothing before that

// Cuts the simple undirected graph of the edge list into at most M communities of about equal size
// (the paper uses METIS for this, Section 2).  Writes the community of every node to comm[N].
// Returns an empty string on success, an error text otherwise.
std::string partition_graph(int64_t N, int64_t n_edges, const int32_t* src, const int32_t* dst, int32_t M,
                            int32_t* comm);

}  // namespace cadmm
