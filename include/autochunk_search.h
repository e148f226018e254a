/*
 * Chunk search on a small op graph: which runs of nodes can be executed segment by segment,
 * and along which dimension (AutoChunk, section 3.3: chunk flow, the four rules, the
 * bottom-up breadth-first search with its local window and first-stage filter).
 *
 * Also: the activation memory of such a graph with and without chunks, the selection cost
 * of section 3.4, and the loop of passes of section 3.2 that chunks a graph until it fits
 * a budget.
 *
 * Host code only: no device memory, no HIP call.  Same library and status codes as
 * autochunk_rt.h.  The executor of autochunk_rt.h works on fixed region kinds; this pass is
 * the general form of its legality table (a region kind and a chunk dimension the executor
 * accepts is a legal chunk of the corresponding graph here).
 */
#ifndef AUTOCHUNK_SEARCH_H
#define AUTOCHUNK_SEARCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AC_GRAPH_MAX_RANK 6
#define AC_GRAPH_MAX_INPUTS 3

/*
 * Op kinds and how a chunk flow passes them (output dimension c -> dimension of each input;
 * "whole": the input has no such dimension and is used whole by every segment; "interrupted":
 * the dimension is computed over, so no flow passes).
 *   INPUT, PARAM       leaves (activations from outside, parameters); never inside a region
 *   LINEAR             x [.., K], w [N, K], optional bias [N] -> [.., N].  c < last: x in c, w and
 *                      bias whole.  c = last: x whole, w and bias in dim 0.
 *   MATMUL_NT / _NN    a [.., M, K], b [.., N, K] / [.., K, N] -> [.., M, N].  Leading dims: both
 *                      in c.  M: a in c, b whole.  N: a whole, b in its N dim.
 *   ELEMENTWISE        any arity, trailing dims aligned, size-1 dims broadcast: an input is in
 *                      the aligned dim, or whole where it lacks or broadcasts it
 *   NORM_LAST, SOFTMAX_LAST   over the last dim: interrupted there, otherwise input 0 in c;
 *                      inputs 1, 2 (gain, shift) whole
 *   TRANSPOSE          attr = permutation: input in attr[c]
 *   SPLIT_DIM          attr = {p, outer}: [.., A*B, ..] -> [.., A, B, ..].  c = p (outer factor):
 *                      input in p; c = p + 1 (inner factor): interrupted; others shift
 *   MERGE_DIMS         attr = {p, inner}: [.., A, B, ..] -> [.., A*B, ..].  c = p: input in p,
 *                      chunk lengths must be multiples of B (the candidate's granule)
 *   SLICE_LAST         attr = {first, past}: a fixed range of the last dim; interrupted along
 *                      it, otherwise input in c
 *   CONTRACT_IKC_JKC   a [I, K, C], b [J, K, C] -> [I, J, C] (the triangle update): c = 0: a in
 *                      0, b whole; c = 1: a whole, b in 0; c = 2: both in 2
 *   CONV2D             x [B, Ci, H, W], w [Co, Ci, kh, kw] (kh, kw odd), optional bias [Co] ->
 *                      [B, Co, H, W], stride 1, same padding.  c = 0: x in 0, w and bias whole;
 *                      c = 1: x whole, w and bias in 0; c = 2, 3: x in c where the window has
 *                      one element along it, else interrupted (a wider window reads across any cut)
 *   GROUP_NORM         attr = {groups}: x [B, C, H, W] normalised over (C / groups, H, W); gain,
 *                      shift [C] whole.  c = 0: x in 0; otherwise interrupted (cuts of the
 *                      channels in whole groups would be legal; they are not expressed)
 */
typedef enum ac_graph_op {
  AC_OP_INPUT = 0, AC_OP_PARAM = 1, AC_OP_LINEAR = 2, AC_OP_MATMUL_NT = 3, AC_OP_MATMUL_NN = 4,
  AC_OP_ELEMENTWISE = 5, AC_OP_NORM_LAST = 6, AC_OP_SOFTMAX_LAST = 7, AC_OP_TRANSPOSE = 8,
  AC_OP_SPLIT_DIM = 9, AC_OP_MERGE_DIMS = 10, AC_OP_SLICE_LAST = 11, AC_OP_CONTRACT_IKC_JKC = 12,
  AC_OP_CONV2D = 13, AC_OP_GROUP_NORM = 14, AC_OP_KINDS = 15
} ac_graph_op;

/* Nodes are listed in a topological order: inputs[] hold indices of earlier nodes.  rank is
 * 1..AC_GRAPH_MAX_RANK, every extent at least 1, and a tensor has at most 2^40 elements (so
 * that byte and operation counts stay within 64 bits); shapes must fit the op kind.  A graph
 * that breaks any of this is refused with AC_ERR_ARG by every call below. */
typedef struct ac_graph_node {
  int32_t op;
  int32_t n_inputs;
  int32_t inputs[AC_GRAPH_MAX_INPUTS];
  int32_t rank;
  int64_t shape[AC_GRAPH_MAX_RANK];
  int64_t attr[AC_GRAPH_MAX_RANK];
} ac_graph_node;

typedef struct ac_chunk_candidate {
  int32_t start, end;   /* the region: nodes start .. end of the list */
  int32_t out_dim;      /* dimension of node `end` the segments are concatenated along */
  int32_t granule;      /* chunk lengths must be multiples of this */
} ac_chunk_candidate;

/*
 * Traces the chunk flow that leaves region [start, end] in dimension out_dim of node `end`
 * (section 3.3, rules 1 to 4): the region's only value used outside must be node `end`'s; the
 * flow must pass every node of the region, each in one dimension only (so no node of the
 * region may be read whole by another), meet no interrupted dimension, and reach at least
 * one input of the region.  An input may be cut for one operand and read whole by another.
 *
 * hoist = 1 applies the graph optimisation of section 3.3 first: nodes of the region that the
 * flow does not pass, or that another node reads whole, are taken out of it together with
 * everything inside the region they depend on; they are computed whole, once, ahead of the
 * segments and count as inputs of what remains, which must then satisfy the rules.  The
 * region's first and last node must remain.  hoist = 0: such a region is illegal.
 *
 * *legal = 1 or 0.  node_dims (n_nodes entries, caller's) receives, for a legal chunk, the
 * chunk dimension of every node that runs per segment and, for every input (a node outside
 * the region, or a moved one) that is cut, the dimension in which it is cut; -1 otherwise.
 * node_moved (n_nodes bytes, may be NULL) receives 1 for the moved nodes.
 * Returns AC_OK, or AC_ERR_ARG for a malformed graph or region (then *legal is 0).
 */
int ac_chunk_trace(const ac_graph_node* nodes, int n_nodes, int start, int end, int out_dim, int hoist,
                   int32_t* node_dims, uint8_t* node_moved, int* legal);

/*
 * All legal chunks whose region holds node `peak` and spans at most `window` nodes (the
 * local window of section 3.3, "complexity optimization").  A (region, dimension) pair is
 * traced in full only if some uninterrupted flow leads from that dimension to an input of the
 * region at all (first stage: no rule checked, stopped at the first input reached).  With
 * hoist = 1 a chunk that would move `peak` itself out of the region is not reported.
 * Candidates are written in order of start, end, out_dim; out (max_out entries), node_dims
 * and node_moved (max_out * n_nodes entries each, one ac_chunk_trace row per candidate;
 * node_moved may be NULL) are the caller's; out and node_dims may be NULL with max_out = 0
 * to count only.  *n_found counts all legal chunks even beyond max_out; n_tried / n_passed
 * (may be NULL) count the pairs tried and those that passed the first stage.
 */
int ac_chunk_search(const ac_graph_node* nodes, int n_nodes, int peak, int window, int hoist,
                    ac_chunk_candidate* out, int32_t* node_dims, uint8_t* node_moved, int max_out,
                    int* n_found, int* n_tried, int* n_passed);

/* One chosen chunk: region [start, end], cut along out_dim of node `end` in segments of
 * chunk_len (the last may be shorter); hoist as in ac_chunk_trace (the moved nodes follow
 * from the region and are not stored). */
typedef struct ac_graph_chunk {
  int32_t start, end, out_dim, hoist;
  int64_t chunk_len;
} ac_graph_chunk;

/*
 * Activation bytes live at every node of the graph run with the given chunks (sections 2.1
 * and 2.2, memory estimation of section 3.4).  Every node's result is a tensor of elem_bytes
 * per element with storage of its own; parameters are not activations.  A tensor is live
 * from its node (a graph input: from the start) to its last reader (none: to the end); the
 * bytes at a node are all tensors live while it runs, M = mem(X) + mem(Y) + mem(A).  Inside
 * a chunked region, M = mem(X) + mem(Y) + mem(A) / n: the region's result is held whole,
 * everything live at the region's entry stays live to its end, and the region's own tensors
 * have chunk_len / extent of their size.  Moved nodes (hoist) run first, in order and whole;
 * those the segments read stay live to the region's end and count with X.
 * chunks: legal (else AC_ERR_ILLEGAL_CHUNK_DIM), apart from each other, chunk_len a multiple
 * of the chunk's granule in 1..extent (else AC_ERR_ARG).  node_bytes (n_nodes entries, may
 * be NULL) receives the bytes per node, 0 for inputs and parameters; *peak_node is the
 * first node that reaches *peak_bytes.
 */
int ac_graph_estimate(const ac_graph_node* nodes, int n_nodes, int elem_bytes,
                      const ac_graph_chunk* chunks, int n_chunks, uint64_t* node_bytes,
                      uint64_t* peak_bytes, int* peak_node);

/*
 * Selection cost of a chunk (section 3.4): L = L_macro + L_micro with
 * L_macro = weights[0] N_node + weights[1] N_flop, L_micro = weights[2] N_density +
 * weights[3] N_stride.  N_node: nodes of the region that run per segment (all of them, or
 * those not moved when hoist = 1; the chunk must then be legal, else
 * AC_ERR_ILLEGAL_CHUNK_DIM); N_flop: their operations (2 per multiply-add of LINEAR, MATMUL,
 * CONTRACT and CONV2D; 1 per element of ELEMENTWISE, 5 of SOFTMAX_LAST, 8 of NORM_LAST and
 * GROUP_NORM; none for the reshaping ops); N_density = N_flop / N_node; N_stride: elements between neighbours along
 * out_dim in the contiguous result of `end`.  The paper tunes the four weights and prints
 * no values: they are the caller's.
 */
int ac_graph_chunk_cost(const ac_graph_node* nodes, int n_nodes, int start, int end, int out_dim, int hoist,
                        const double* weights, double* cost);

/*
 * Chunks the graph pass by pass until its estimated peak is at most budget_bytes (section
 * 3.2: estimate, search around the peak node, select; repeated), looking for the strategy
 * S = [s_1 .. s_l] of least summed cost (section 3.4).  One pass extends a strategy by one
 * chunk: the legal chunks of ac_chunk_search(peak node, window, hoist) that touch no region
 * chosen before get the longest chunk_len (multiple of the granule, below the extent) at
 * which their region fits the budget; those with none are dropped.  An extended strategy that
 * fits competes for the answer (least summed cost; ties: fewer segments in all, then the order
 * they were made in) and takes no place in the beam; of those that do not fit yet the `beam`
 * cheapest go on to the next pass; the call ends when none is left and returns the cheapest
 * strategy that fitted.  beam = 1: follow the cheapest candidate that does not fit yet.
 * out (max_out entries, caller's) receives the chunks in the order chosen, *n_out their
 * number, *peak_bytes the estimate with them.  AC_ERR_BUDGET_INFEASIBLE when no strategy in
 * the beam can be extended (*n_out = 0, *peak_bytes = the unchunked peak); AC_ERR_ARG when
 * the strategy has more than max_out chunks.
 */
int ac_graph_plan(const ac_graph_node* nodes, int n_nodes, int elem_bytes, uint64_t budget_bytes,
                  int window, const double* weights, int beam, int hoist, ac_graph_chunk* out,
                  int max_out, int* n_out, uint64_t* peak_bytes);

/*
 * What ties a node of a model's op graph to the executor of autochunk_rt.h: the region kind
 * whose kernels compute the node (AC_REGION_*, -1: none), the layer or block it belongs to, and
 * for every dim of its result the executor's chunk dim it is (AC_DIM_* of the workload, -1: the
 * executor has no such dim) with the number of executor units one index of the graph dim
 * stands for (a head of a [batch, heads, seq, head_dim] tensor is head_dim features).
 */
typedef struct ac_node_tag {
  int32_t region_kind, group;
  int32_t dim[AC_GRAPH_MAX_RANK];
  int64_t unit[AC_GRAPH_MAX_RANK];
} ac_node_tag;

/*
 * From chunks chosen on a graph (ac_graph_plan) to the chunk settings ac_plan_create takes
 * (section 3.2: the plan found by the passes is what the runtime executes; section 3.3, rule 4:
 * one setting per region).  A chunk goes to the region kind that holds all its nodes, within one
 * group; the executor cuts a kind in every layer alike, so a kind takes the shortest length
 * asked for in any group.  out (max_out entries, caller's) receives one ac_region_desc per kind,
 * ordered by kind; *n_out their number.  AC_ERR_ARG: a chunk's nodes lie in no single kind or
 * group, groups disagree on a kind's dim, bad indices, more kinds than max_out;
 * AC_ERR_UNSUPPORTED: a chunk is cut along a dim the executor has no chunk dim for.  Whether
 * the executor accepts the settings (legality, granules) is ac_plan_create's to say.
 */
struct ac_region_desc;
int ac_graph_chunks_to_regions(const ac_node_tag* tags, int n_nodes, const ac_graph_chunk* chunks, int n_chunks,
                               struct ac_region_desc* out, int max_out, int* n_out);

#ifdef __cplusplus
}
#endif
#endif
