// Chunk search on an op graph (AutoChunk, section 3.3).  Host code only.
//
// A chunk is a run [start, end] of the node list plus one dimension of node `end`.  The
// flow of that dimension is followed from `end` towards the region's inputs: each op kind
// says in which dimension of each operand the cut continues (a value >= 0), that the
// operand is not cut (kWhole), or that the op computes over the dimension (kCut).
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/autochunk_search.h"
#include "common.h"

namespace {

constexpr int kWhole = -1;  // operand used whole by every segment
constexpr int kCut = -2;    // the op reduces, contracts or strides over the dimension

inline bool is_leaf(const ac_graph_node& n) { return n.op == AC_OP_INPUT || n.op == AC_OP_PARAM; }

// Dimension of operand `k` that dimension `c` of n's output is cut along.
int step(const ac_graph_node* g, const ac_graph_node& n, int c, int k) {
  const ac_graph_node& x = g[n.inputs[k]];
  const int last = n.rank - 1;
  switch (n.op) {
    case AC_OP_ELEMENTWISE: {
      const int d = c - (n.rank - x.rank);
      if (d < 0) return kWhole;
      return (x.shape[d] == 1 && n.shape[c] != 1) ? kWhole : d;
    }
    case AC_OP_NORM_LAST:
    case AC_OP_SOFTMAX_LAST:
      if (k != 0) return kWhole;
      return c == last ? kCut : c;
    case AC_OP_LINEAR:
      if (c == last) return k == 0 ? kWhole : 0;
      return k == 0 ? c : kWhole;
    case AC_OP_MATMUL_NT:
    case AC_OP_MATMUL_NN:
      if (c < last - 1) return c;
      if (c == last - 1) return k == 0 ? c : kWhole;
      if (k == 0) return kWhole;
      return n.op == AC_OP_MATMUL_NT ? x.rank - 2 : x.rank - 1;
    case AC_OP_TRANSPOSE:
      return (int)n.attr[c];
    case AC_OP_SPLIT_DIM: {
      const int p = (int)n.attr[0];
      if (c <= p) return c;
      return c == p + 1 ? kCut : c - 1;
    }
    case AC_OP_MERGE_DIMS: {
      const int p = (int)n.attr[0];
      return c <= p ? c : c + 1;
    }
    case AC_OP_SLICE_LAST:
      return c == last ? kCut : c;
    case AC_OP_CONTRACT_IKC_JKC:
      if (c == 2) return 2;
      return (c == 0) == (k == 0) ? 0 : kWhole;
    default:
      return kCut;
  }
}

bool same_shape_but(const ac_graph_node& a, const ac_graph_node& b, int n_lead) {
  for (int i = 0; i < n_lead; ++i)
    if (a.shape[i] != b.shape[i]) return false;
  return true;
}

// Structural checks, so that step() indexes nothing out of range.
bool graph_ok(const ac_graph_node* g, int n_nodes) {
  if (!g || n_nodes <= 0) return false;
  for (int i = 0; i < n_nodes; ++i) {
    const ac_graph_node& n = g[i];
    if (n.op < 0 || n.op >= AC_OP_KINDS) return false;
    if (n.rank < 1 || n.rank > AC_GRAPH_MAX_RANK) return false;
    for (int d = 0; d < n.rank; ++d)
      if (n.shape[d] < 1) return false;
    if (n.n_inputs < 0 || n.n_inputs > AC_GRAPH_MAX_INPUTS) return false;
    for (int k = 0; k < n.n_inputs; ++k)
      if (n.inputs[k] < 0 || n.inputs[k] >= i) return false;
    const ac_graph_node* x = n.n_inputs > 0 ? &g[n.inputs[0]] : nullptr;
    const ac_graph_node* y = n.n_inputs > 1 ? &g[n.inputs[1]] : nullptr;
    switch (n.op) {
      case AC_OP_INPUT:
      case AC_OP_PARAM:
        if (n.n_inputs != 0) return false;
        break;
      case AC_OP_LINEAR:
        if (n.n_inputs < 2 || x->rank != n.rank || y->rank != 2) return false;
        if (y->shape[1] != x->shape[x->rank - 1] || y->shape[0] != n.shape[n.rank - 1]) return false;
        if (!same_shape_but(n, *x, n.rank - 1)) return false;
        if (n.n_inputs == 3 && (g[n.inputs[2]].rank != 1 || g[n.inputs[2]].shape[0] != y->shape[0])) return false;
        break;
      case AC_OP_MATMUL_NT:
      case AC_OP_MATMUL_NN: {
        if (n.n_inputs != 2 || n.rank < 2 || x->rank != n.rank || y->rank != n.rank) return false;
        if (!same_shape_but(n, *x, n.rank - 1) || !same_shape_but(n, *y, n.rank - 2)) return false;
        const int r = n.rank;
        const int64_t kk = x->shape[r - 1];
        const int64_t yn = n.op == AC_OP_MATMUL_NT ? y->shape[r - 2] : y->shape[r - 1];
        const int64_t yk = n.op == AC_OP_MATMUL_NT ? y->shape[r - 1] : y->shape[r - 2];
        if (yk != kk || yn != n.shape[r - 1]) return false;
        break;
      }
      case AC_OP_ELEMENTWISE:
        if (n.n_inputs < 1) return false;
        for (int k = 0; k < n.n_inputs; ++k) {
          const ac_graph_node& in = g[n.inputs[k]];
          if (in.rank > n.rank) return false;
          for (int d = 0; d < in.rank; ++d) {
            const int64_t e = in.shape[d], o = n.shape[d + n.rank - in.rank];
            if (e != o && e != 1) return false;
          }
        }
        break;
      case AC_OP_NORM_LAST:
      case AC_OP_SOFTMAX_LAST:
        if (n.n_inputs < 1 || x->rank != n.rank || !same_shape_but(n, *x, n.rank)) return false;
        for (int k = 1; k < n.n_inputs; ++k)
          if (g[n.inputs[k]].rank != 1 || g[n.inputs[k]].shape[0] != n.shape[n.rank - 1]) return false;
        break;
      case AC_OP_TRANSPOSE: {
        if (n.n_inputs != 1 || x->rank != n.rank) return false;
        unsigned seen = 0;
        for (int d = 0; d < n.rank; ++d) {
          const int64_t a = n.attr[d];
          if (a < 0 || a >= n.rank || (seen >> a & 1u) || x->shape[a] != n.shape[d]) return false;
          seen |= 1u << a;
        }
        break;
      }
      case AC_OP_SPLIT_DIM: {
        const int64_t p = n.attr[0], outer = n.attr[1];
        if (n.n_inputs != 1 || x->rank + 1 != n.rank || p < 0 || p >= x->rank) return false;
        if (outer < 1 || n.shape[p] != outer || n.shape[p] * n.shape[p + 1] != x->shape[p]) return false;
        for (int d = 0; d < x->rank; ++d)
          if (d != p && x->shape[d] != n.shape[d < p ? d : d + 1]) return false;
        break;
      }
      case AC_OP_MERGE_DIMS: {
        const int64_t p = n.attr[0], inner = n.attr[1];
        if (n.n_inputs != 1 || x->rank != n.rank + 1 || p < 0 || p >= n.rank) return false;
        if (x->shape[p + 1] != inner || x->shape[p] * inner != n.shape[p]) return false;
        for (int d = 0; d < n.rank; ++d)
          if (d != p && n.shape[d] != x->shape[d < p ? d : d + 1]) return false;
        break;
      }
      case AC_OP_SLICE_LAST: {
        if (n.n_inputs != 1 || x->rank != n.rank || !same_shape_but(n, *x, n.rank - 1)) return false;
        const int64_t a = n.attr[0], b = n.attr[1];
        if (a < 0 || b <= a || b > x->shape[n.rank - 1] || n.shape[n.rank - 1] != b - a) return false;
        break;
      }
      case AC_OP_CONTRACT_IKC_JKC:
        if (n.n_inputs != 2 || n.rank != 3 || x->rank != 3 || y->rank != 3) return false;
        if (x->shape[1] != y->shape[1] || x->shape[2] != y->shape[2]) return false;
        if (n.shape[0] != x->shape[0] || n.shape[1] != y->shape[0] || n.shape[2] != x->shape[2]) return false;
        break;
    }
  }
  return true;
}

struct Tracer {
  const ac_graph_node* g;
  int n_nodes;
  std::vector<int> last_use;   // highest index of a node that reads node i, -1 if none
  std::vector<int> leaves_upto;  // number of INPUT/PARAM nodes among 0..i-1
  std::vector<int> queue;
  std::vector<uint8_t> seen;

  Tracer(const ac_graph_node* nodes, int n) : g(nodes), n_nodes(n), last_use(n, -1), leaves_upto(n + 1, 0), seen(n, 0) {
    for (int i = 0; i < n; ++i) {
      for (int k = 0; k < g[i].n_inputs; ++k) last_use[g[i].inputs[k]] = i;
      leaves_upto[i + 1] = leaves_upto[i] + (is_leaf(g[i]) ? 1 : 0);
    }
    queue.reserve((size_t)n * AC_GRAPH_MAX_RANK);
  }

  bool holds_leaf(int start, int end) const { return leaves_upto[end + 1] != leaves_upto[start]; }

  // Rules 1 to 4 for one candidate; fills row (n_nodes entries) and the granule.
  bool trace(int start, int end, int out_dim, int32_t* row, int64_t* granule) {
    // Form Y^c = F(X^c, X^nc): no intermediate of the region is read after `end`.
    for (int i = start; i < end; ++i)
      if (last_use[i] > end) return false;
    for (int i = 0; i < n_nodes; ++i) row[i] = -1;
    row[end] = out_dim;
    queue.clear();
    queue.push_back(end);
    const int64_t ext_out = g[end].shape[out_dim];
    int64_t gran = 1;
    int reached_inputs = 0, passed = 1;
    for (size_t head = 0; head < queue.size(); ++head) {
      const ac_graph_node& n = g[queue[head]];
      const int c = row[queue[head]];
      for (int k = 0; k < n.n_inputs; ++k) {
        const int d = step(g, n, c, k);
        if (d == kCut) return false;   // the flow is interrupted
        const int s = n.inputs[k];
        if (d == kWhole) {
          if (s >= start) return false;  // a node of the region read whole: every segment would compute all of it
          continue;
        }
        if (row[s] >= 0) {
          if (row[s] != d) return false;  // one node (or input), two chunk dimensions
          continue;
        }
        row[s] = d;
        // a segment of len elements of the output covers len * ext / ext_out elements here
        const int64_t ext = g[s].shape[d];
        gran = std::lcm(gran, ext_out / std::gcd(ext_out, ext));
        if (s >= start) {
          queue.push_back(s);
          ++passed;
        } else {
          ++reached_inputs;
        }
      }
    }
    if (passed != end - start + 1) return false;  // some node is on no flow
    if (reached_inputs == 0) return false;        // no input can be cut
    *granule = gran;
    return true;
  }

  // First stage of the two-stage search: does any uninterrupted flow lead from the output
  // dimension to an input of the region?  Nothing else is checked, and the walk stops at the
  // first input it reaches.  seen[i] holds one bit per dimension of node i already expanded.
  bool reaches_an_input(int start, int end, int out_dim) {
    for (int i = start; i <= end; ++i) seen[i] = 0;
    queue.clear();
    queue.push_back(end * AC_GRAPH_MAX_RANK + out_dim);
    seen[end] = (uint8_t)(1u << out_dim);
    while (!queue.empty()) {
      const int item = queue.back();
      queue.pop_back();
      const ac_graph_node& n = g[item / AC_GRAPH_MAX_RANK];
      const int c = item % AC_GRAPH_MAX_RANK;
      for (int k = 0; k < n.n_inputs; ++k) {
        const int d = step(g, n, c, k);
        if (d < 0) continue;
        const int s = n.inputs[k];
        if (s < start) return true;
        if (seen[s] >> d & 1u) continue;
        seen[s] |= (uint8_t)(1u << d);
        queue.push_back(s * AC_GRAPH_MAX_RANK + d);
      }
    }
    return false;
  }
};

template <class... A>
int bad(const char* fmt, A... a) {
  ac::set_error(fmt, a...);
  return AC_ERR_ARG;
}

}  // namespace

extern "C" int ac_chunk_trace(const ac_graph_node* nodes, int n_nodes, int start, int end, int out_dim,
                              int32_t* node_dims, int* legal) {
  if (legal) *legal = 0;
  if (!legal || !node_dims) return bad("ac_chunk_trace: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_chunk_trace: malformed graph");
  if (start < 0 || end < start || end >= n_nodes) return bad("ac_chunk_trace: region [%d, %d] outside the graph", start, end);
  if (out_dim < 0 || out_dim >= nodes[end].rank) return bad("ac_chunk_trace: node %d has no dim %d", end, out_dim);
  Tracer t(nodes, n_nodes);
  if (t.holds_leaf(start, end)) return bad("ac_chunk_trace: region [%d, %d] holds an input or parameter node", start, end);
  int64_t gran = 1;
  if (t.trace(start, end, out_dim, node_dims, &gran)) {
    *legal = 1;
  } else {
    for (int i = 0; i < n_nodes; ++i) node_dims[i] = -1;
  }
  return AC_OK;
}

extern "C" int ac_chunk_search(const ac_graph_node* nodes, int n_nodes, int peak, int window,
                               ac_chunk_candidate* out, int32_t* node_dims, int max_out,
                               int* n_found, int* n_tried, int* n_passed) {
  if (n_found) *n_found = 0;
  if (n_tried) *n_tried = 0;
  if (n_passed) *n_passed = 0;
  if (!n_found) return bad("ac_chunk_search: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_chunk_search: malformed graph");
  if (peak < 0 || peak >= n_nodes || window < 1 || max_out < 0)
    return bad("ac_chunk_search: peak %d, window %d or max_out %d out of range", peak, window, max_out);
  if (max_out > 0 && (!out || !node_dims)) return bad("ac_chunk_search: null output with max_out %d", max_out);
  Tracer t(nodes, n_nodes);
  std::vector<int32_t> row(n_nodes);
  int found = 0, tried = 0, passed = 0;
  const int first = peak - window + 1 > 0 ? peak - window + 1 : 0;
  for (int start = first; start <= peak; ++start) {
    const int past = start + window < n_nodes ? start + window : n_nodes;
    for (int end = peak; end < past; ++end) {
      if (t.holds_leaf(start, end)) break;  // longer regions hold it too
      for (int d = 0; d < nodes[end].rank; ++d) {
        ++tried;
        if (!t.reaches_an_input(start, end, d)) continue;
        ++passed;
        int64_t gran = 1;
        if (!t.trace(start, end, d, row.data(), &gran)) continue;
        if (found < max_out) {
          out[found].start = start;
          out[found].end = end;
          out[found].out_dim = d;
          out[found].granule = (int32_t)gran;
          for (int i = 0; i < n_nodes; ++i) node_dims[(size_t)found * n_nodes + i] = row[i];
        }
        ++found;
      }
    }
  }
  *n_found = found;
  if (n_tried) *n_tried = tried;
  if (n_passed) *n_passed = passed;
  return AC_OK;
}
