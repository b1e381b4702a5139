// Extraction step of operator fusion (paper Section 4.1): dataflow DAG -> post-dominator
// tree -> fusion groups.  Host code; nothing here touches the GPU.
#pragma once
#include <cstdint>
#include <vector>

namespace relay {

enum : int32_t { PAT_OPAQUE = 0, PAT_ELEMWISE = 1, PAT_CONTRACTION = 2 };
constexpr int32_t kExit = -1;  // the virtual node every output of the graph flows into

// Operators are numbered in dataflow order (an operator only reads earlier ones); the inputs
// of operator i are in_nodes[in_offsets[i] .. in_offsets[i+1]).
// ipdom[i]: immediate post-dominator of i, or kExit.  group[i]: smallest operator of i's group.
void fuse_extract(int32_t n, const int32_t* pattern, const int32_t* in_offsets, const int32_t* in_nodes,
                  std::vector<int32_t>& ipdom, std::vector<int32_t>& group);

}  // namespace relay
