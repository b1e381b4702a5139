/*
 * relay_fusion.h -- C ABI of the extraction step of operator fusion (host code, no GPU).
 *
 * The paper's fusion pass (Section 4.1, "Extraction") builds the dataflow DAG between
 * operators, builds its post-dominator tree, groups operators by their immediate
 * post-dominator and turns every group into one primitive function; the entry points of
 * relay_fused.h are the compiled forms of such functions.  This call computes the groups.
 *
 * The paper does not say which operators may share a group.  Rule used here: an operator
 * joins the group of its immediate post-dominator, taking the operators on the paths between
 * them along, when all of those (the post-dominator included) are elementwise/broadcast and
 * the united group keeps at most one contraction; opaque operators stay alone; operators are
 * visited in dataflow order and a merge that would break the rule is skipped.
 */
#ifndef RELAY_FUSION_H_
#define RELAY_FUSION_H_

#include <stdint.h>

#include "relay_fused.h"

#ifdef __cplusplus
extern "C" {
#endif

/* how an operator may be fused */
typedef enum {
  RELAY_PATTERN_OPAQUE = 0,      /* never fused (graph inputs, pooling, ...) */
  RELAY_PATTERN_ELEMWISE = 1,    /* elementwise or broadcast: bias add, scale/shift, add, relu */
  RELAY_PATTERN_CONTRACTION = 2  /* conv2d, depthwise conv2d, dense: may take elementwise operators behind it */
} relay_op_pattern;

/*
 * The extraction step of operator fusion (paper Section 4.1, "Extraction").
 * All pointers are HOST pointers owned by the caller; nothing is retained.
 *   n_ops        number of operators, numbered in dataflow order: operator i reads only
 *                operators j < i.  1 <= n_ops <= 2^20.
 *   pattern      [n_ops] relay_op_pattern of each operator.
 *   in_offsets   [n_ops + 1] non-decreasing, in_offsets[0] == 0.
 *   in_nodes     [in_offsets[n_ops]] the operators that operator i reads are
 *                in_nodes[in_offsets[i] .. in_offsets[i+1]); duplicates are allowed.
 *   ipdom        [n_ops] out, may be NULL: immediate post-dominator of each operator in the
 *                DAG with a virtual exit behind every unread operator; -1 = that exit.
 *   group        [n_ops] out: the smallest operator index of the operator's fusion group.
 *                The operator with the largest index of a group is the only one read from
 *                outside the group (its result); groups ordered by that operator can be
 *                executed one after another.
 * Returns RELAY_ERR_NULL, RELAY_ERR_SHAPE (bad counts, offsets, an input that is not an
 * earlier operator) or RELAY_ERR_UNSUPPORTED (unknown pattern) without writing any output.
 */
relay_status relay_fuse_extract(int32_t n_ops, const int32_t* pattern, const int32_t* in_offsets,
                                const int32_t* in_nodes, int32_t* ipdom, int32_t* group);

#ifdef __cplusplus
}
#endif
#endif /* RELAY_FUSION_H_ */
