// The passes that decide a chunk plan, on an op graph (AutoChunk sections 3.2 to 3.4): chunk
// flow and the four rules, the graph optimisation, the windowed two-stage search, activation
// memory with and without chunks, the selection cost, and the loop of passes with a beam.
// Host code only.
//
// A chunk is a run [start, end] of the node list plus one dimension of node `end`.  The
// flow of that dimension is followed from `end` towards the region's inputs: each op kind
// says in which dimension of each operand the cut continues (a value >= 0), that the
// operand is not cut (kWhole), or that the op computes over the dimension (kCut).
#include <algorithm>
#include <array>
#include <cstdint>
#include <numeric>
#include <set>
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
    case AC_OP_CONV2D:
      if (c == 0) return k == 0 ? 0 : kWhole;
      if (c == 1) return k == 0 ? kWhole : 0;
      if (g[n.inputs[1]].shape[c] != 1) return kCut;  // a window wider than one element reads across any cut
      return k == 0 ? c : kWhole;
    case AC_OP_GROUP_NORM:
      if (k != 0) return kWhole;
      return c == 0 ? 0 : kCut;
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
    // element and byte counts are kept in 64 bits: cap a tensor at 2^40 elements so that the sum
    // over a graph of up to 2^20 such tensors of 8-byte elements cannot wrap
    int64_t elems = 1;
    for (int d = 0; d < n.rank; ++d) {
      if (n.shape[d] < 1 || n.shape[d] > (int64_t(1) << 40) / elems) return false;
      elems *= n.shape[d];
    }
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
      case AC_OP_CONV2D: {
        if (n.n_inputs < 2 || n.rank != 4 || x->rank != 4 || y->rank != 4) return false;
        if (y->shape[1] != x->shape[1] || y->shape[0] != n.shape[1] || y->shape[2] % 2 != 1 || y->shape[3] % 2 != 1) return false;
        if (n.shape[0] != x->shape[0] || n.shape[2] != x->shape[2] || n.shape[3] != x->shape[3]) return false;
        if (n.n_inputs == 3 && (g[n.inputs[2]].rank != 1 || g[n.inputs[2]].shape[0] != n.shape[1])) return false;
        break;
      }
      case AC_OP_GROUP_NORM:
        if (n.n_inputs < 1 || n.rank != 4 || x->rank != 4 || !same_shape_but(n, *x, 4)) return false;
        if (n.attr[0] < 1 || n.shape[1] % n.attr[0] != 0) return false;
        for (int k = 1; k < n.n_inputs; ++k)
          if (g[n.inputs[k]].rank != 1 || g[n.inputs[k]].shape[0] != n.shape[1]) return false;
        break;
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
  std::vector<uint8_t> seen, read_whole;

  Tracer(const ac_graph_node* nodes, int n) : g(nodes), n_nodes(n), last_use(n, -1), leaves_upto(n + 1, 0), seen(n, 0), read_whole(n, 0) {
    for (int i = 0; i < n; ++i) {
      for (int k = 0; k < g[i].n_inputs; ++k) last_use[g[i].inputs[k]] = i;
      leaves_upto[i + 1] = leaves_upto[i] + (is_leaf(g[i]) ? 1 : 0);
    }
    queue.reserve((size_t)n * AC_GRAPH_MAX_RANK);
  }

  bool holds_leaf(int start, int end) const { return leaves_upto[end + 1] != leaves_upto[start]; }

  // Rules 1 to 4 for one candidate; fills row (n_nodes entries: chunk dim of every node of the
  // region and of every input that is cut, else -1) and the granule.
  //
  // With hoist (the graph optimisation of section 3.3) nodes of the region that the flow does
  // not pass, or that another node reads whole, do not make the chunk illegal: they are marked
  // in moved[] together with everything inside the region they depend on (to be computed whole,
  // once, ahead of the segments) and the rest is traced again with them as inputs, until
  // nothing more has to move.  The first and the last node must stay.
  bool trace(int start, int end, int out_dim, bool hoist, int32_t* row, uint8_t* moved, int64_t* granule) {
    // Form Y^c = F(X^c, X^nc): no intermediate of the region is read after `end`.
    for (int i = start; i < end; ++i)
      if (last_use[i] > end) return false;
    for (int i = start; i <= end; ++i) moved[i] = 0;
    const int64_t ext_out = g[end].shape[out_dim];
    for (;;) {
      for (int i = 0; i < n_nodes; ++i) row[i] = -1;
      for (int i = start; i <= end; ++i) read_whole[i] = 0;
      row[end] = out_dim;
      queue.clear();
      queue.push_back(end);
      int64_t gran = 1;
      int reached_inputs = 0;
      for (size_t head = 0; head < queue.size(); ++head) {
        const ac_graph_node& n = g[queue[head]];
        const int c = row[queue[head]];
        for (int k = 0; k < n.n_inputs; ++k) {
          const int d = step(g, n, c, k);
          if (d == kCut) return false;   // the flow is interrupted
          const int s = n.inputs[k];
          const bool in_rest = s >= start && !moved[s];
          if (d == kWhole) {
            // a node of the region read whole: every segment would compute all of it
            if (in_rest) {
              if (!hoist) return false;
              read_whole[s] = 1;
            }
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
          if (in_rest) queue.push_back(s);
          else ++reached_inputs;
        }
      }
      // nodes on no flow, or read whole: illegal, or (hoist) moved with their ancestors in the region
      bool grew = false;
      for (int i = end; i >= start; --i) {
        if (moved[i]) continue;
        bool go = row[i] < 0 || read_whole[i];
        if (go && !hoist) return false;
        if (go) {
          if (i == start || i == end) return false;
          moved[i] = 1;
          grew = true;
          // descending order: inputs of a moved node are visited later in this loop
          for (int k = 0; k < g[i].n_inputs; ++k)
            if (g[i].inputs[k] >= start) read_whole[g[i].inputs[k]] = 1;
        }
      }
      if (grew) continue;
      if (reached_inputs == 0) return false;        // no input can be cut
      *granule = gran;
      return true;
    }
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

  // Every legal chunk whose region holds `peak` and spans at most `window` nodes, in order of
  // start, end, dimension (the local window and the two stages of section 3.3).
  template <class F>
  void candidates(int peak, int window, bool hoist, int* tried, int* passed, F&& on_chunk) {
    std::vector<int32_t> row(n_nodes);
    std::vector<uint8_t> moved(n_nodes, 0);
    const int first = peak - window + 1 > 0 ? peak - window + 1 : 0;
    for (int start = first; start <= peak; ++start) {
      const int past = start + window < n_nodes ? start + window : n_nodes;
      for (int end = peak; end < past; ++end) {
        if (holds_leaf(start, end)) break;  // longer regions hold it too
        for (int d = 0; d < g[end].rank; ++d) {
          ++*tried;
          if (!reaches_an_input(start, end, d)) continue;
          ++*passed;
          int64_t gran = 1;
          // a chunk that moves the peak node out of the region does nothing for the peak
          if (trace(start, end, d, hoist, row.data(), moved.data(), &gran) && !moved[peak])
            on_chunk(start, end, d, gran, row.data(), moved.data());
        }
      }
    }
  }
};

// -----------------------------------------------------------------------------------------
// Activation memory of the graph (sections 2.1, 2.2) and the selection cost (section 3.4).
//
// Every node's result has storage of its own; parameters are not counted.  A tensor is live
// from its node (a graph input: from the start) to its last reader (none: to the end).  The
// bytes at a node are all tensors live while it runs.  Inside a chunked region the region's
// result is held whole, tensors of the region shrink to chunk_len / extent of their size, and
// everything live at the region's entry stays so until its last segment is done:
// M = X + Y + A / n.
// -----------------------------------------------------------------------------------------
typedef unsigned __int128 u128;

struct Memory {
  const Tracer& t;
  int n;
  std::vector<uint64_t> size;   // bytes of each node's result (0 for parameters)
  std::vector<int> dies;        // last reader; n - 1 for results nobody reads; -1 for unread leaves
  std::vector<uint64_t> whole;  // live bytes at each node of the unchunked graph
  mutable std::vector<uint8_t> keep_scratch;

  Memory(const Tracer& tr, int elem_bytes) : t(tr), n(tr.n_nodes), size(n), dies(n), whole(n, 0) {
    const ac_graph_node* g = t.g;
    std::vector<int64_t> delta(n + 1, 0);
    for (int i = 0; i < n; ++i) {
      uint64_t elems = 1;
      for (int d = 0; d < g[i].rank; ++d) elems *= (uint64_t)g[i].shape[d];
      size[i] = g[i].op == AC_OP_PARAM ? 0 : elems * (uint64_t)elem_bytes;
      dies[i] = t.last_use[i] >= 0 ? t.last_use[i] : (is_leaf(g[i]) ? -1 : n - 1);
      if (dies[i] < 0) continue;
      delta[is_leaf(g[i]) ? 0 : i] += (int64_t)size[i];
      delta[dies[i] + 1] -= (int64_t)size[i];
    }
    int64_t live = 0;
    for (int i = 0; i < n; ++i) {
      live += delta[i];
      whole[i] = is_leaf(g[i]) ? 0 : (uint64_t)live;
    }
  }

  // Bytes live at every node of a chunked region, as fixed part + part that scales with the
  // segment length: bytes(i) = fixed[i] + scaled[i] * len / extent.  moved[] marks the nodes
  // computed whole ahead of the segments: they run first, in order, with ordinary lifetimes,
  // except that those the segments read stay live to the region's end.
  void region(int start, int end, const uint8_t* moved, std::vector<uint64_t>& fixed,
              std::vector<uint64_t>& scaled) const {
    const ac_graph_node* g = t.g;
    const int count = end - start + 1;
    fixed.assign(count, 0);
    scaled.assign(count, 0);
    const uint64_t entry = whole[start] - size[start];   // X and everything else alive at the region's entry
    // moved nodes the segments read, and moved results that outlive the region
    uint64_t kept = 0;
    std::vector<uint8_t>& keep = keep_scratch;
    keep.assign(count, 0);
    for (int i = start; i <= end; ++i) {
      if (moved[i]) continue;
      for (int k = 0; k < g[i].n_inputs; ++k) {
        const int s = g[i].inputs[k];
        if (s >= start && moved[s]) keep[s - start] = 1;
      }
    }
    for (int h = start; h <= end; ++h)
      if (moved[h] && (keep[h - start] || t.last_use[h] < 0 || t.last_use[h] > end)) {
        keep[h - start] = 1;
        kept += size[h];
      }
    // ahead of the segments: the moved nodes in order
    for (int i = start; i <= end; ++i) {
      if (!moved[i]) continue;
      uint64_t live = entry;
      for (int h = start; h <= i; ++h)
        if (moved[h] && (keep[h - start] || t.last_use[h] >= i)) live += size[h];
      fixed[i - start] = live;
    }
    // the segments: Y whole, the region's own tensors at their segment's share
    uint64_t cur = 0;
    for (int i = start; i <= end; ++i) {
      if (moved[i]) continue;
      if (i != end) cur += size[i];
      fixed[i - start] = entry + kept + size[end];
      scaled[i - start] = cur;
      for (int k = 0; k < g[i].n_inputs; ++k) {
        const int s = g[i].inputs[k];
        bool counted = false;
        for (int q = 0; q < k; ++q) counted |= g[i].inputs[q] == s;
        if (!counted && s >= start && !moved[s] && t.last_use[s] == i) cur -= size[s];
      }
    }
  }

  // Longest chunk length (multiple of granule, below the extent) at which the region fits, or 0.
  int64_t longest_len(int start, int end, const uint8_t* moved, int64_t extent, int64_t granule, uint64_t budget,
                      std::vector<uint64_t>& fixed, std::vector<uint64_t>& scaled) const {
    region(start, end, moved, fixed, scaled);
    int64_t len = (extent - 1) / granule * granule;
    for (size_t i = 0; i < fixed.size(); ++i) {
      if (fixed[i] > budget) return 0;
      if (scaled[i] == 0) continue;
      const u128 fit = (u128)(budget - fixed[i]) * (u128)extent / scaled[i];
      if (fit < (u128)len) len = (int64_t)fit / granule * granule;
    }
    return len;
  }
};

// Operations of one node (128 bits: 2^40 elements times a contraction length can pass 2^64).
u128 node_flops(const ac_graph_node* g, const ac_graph_node& n) {
  u128 out = 1;
  for (int d = 0; d < n.rank; ++d) out *= (u128)n.shape[d];
  switch (n.op) {
    case AC_OP_LINEAR:
    case AC_OP_MATMUL_NT:
    case AC_OP_MATMUL_NN: {
      const ac_graph_node& x = g[n.inputs[0]];
      return 2 * out * (u128)x.shape[x.rank - 1];
    }
    case AC_OP_CONTRACT_IKC_JKC:
      return 2 * out * (u128)g[n.inputs[0]].shape[1];
    case AC_OP_ELEMENTWISE:
      return out;
    case AC_OP_SOFTMAX_LAST:
      return 5 * out;  // max, subtract, exponential, sum, divide
    case AC_OP_NORM_LAST:
    case AC_OP_GROUP_NORM:
      return 8 * out;  // mean; centre, square, sum; scale by the deviation; gain, shift
    case AC_OP_CONV2D: {
      const ac_graph_node& w = g[n.inputs[1]];
      return 2 * out * (u128)w.shape[1] * (u128)w.shape[2] * (u128)w.shape[3];
    }
    default:
      return 0;
  }
}

// L = (alpha N_node + beta N_flop) + (gamma N_density + lambda N_stride), over the nodes that
// run once per segment (moved may be null: all of the region).
double chunk_cost(const ac_graph_node* g, int start, int end, int out_dim, const uint8_t* moved, const double* w) {
  u128 flops = 0;
  int count = 0;
  for (int i = start; i <= end; ++i) {
    if (moved && moved[i]) continue;
    flops += node_flops(g, g[i]);
    ++count;
  }
  uint64_t stride = 1;
  for (int d = out_dim + 1; d < g[end].rank; ++d) stride *= (uint64_t)g[end].shape[d];
  const double n_node = (double)count, n_flop = (double)flops;
  const double n_density = n_flop / n_node, n_stride = (double)stride;
  const double macro = w[0] * n_node + w[1] * n_flop;
  const double micro = w[2] * n_density + w[3] * n_stride;
  return macro + micro;
}

// Checks a caller's chunk list (legal, lengths on the granule, regions apart), fills
// region_of[i] = index of the chunk that holds node i, or -1, and moved[c] = the nodes chunk c
// computes ahead of its segments (all zero without hoist).
int check_chunks(Tracer& t, const ac_graph_chunk* chunks, int n_chunks, std::vector<int>& region_of,
                 std::vector<std::vector<uint8_t>>& moved) {
  const int n = t.n_nodes;
  region_of.assign(n, -1);
  moved.assign(n_chunks, std::vector<uint8_t>(n, 0));
  std::vector<int32_t> row(n);
  for (int c = 0; c < n_chunks; ++c) {
    const ac_graph_chunk& ch = chunks[c];
    if (ch.start < 0 || ch.end < ch.start || ch.end >= n || t.holds_leaf(ch.start, ch.end) || ch.out_dim < 0 ||
        ch.out_dim >= t.g[ch.end].rank || (ch.hoist != 0 && ch.hoist != 1)) {
      ac::set_error("chunk %d: region [%d, %d], dim %d or hoist %d not valid for the graph", c, ch.start, ch.end,
                    ch.out_dim, ch.hoist);
      return AC_ERR_ARG;
    }
    int64_t gran = 1;
    if (!t.trace(ch.start, ch.end, ch.out_dim, ch.hoist != 0, row.data(), moved[c].data(), &gran)) {
      ac::set_error("chunk %d: region [%d, %d] cannot be cut along dim %d", c, ch.start, ch.end, ch.out_dim);
      return AC_ERR_ILLEGAL_CHUNK_DIM;
    }
    const int64_t extent = t.g[ch.end].shape[ch.out_dim];
    if (ch.chunk_len < 1 || ch.chunk_len > extent || ch.chunk_len % gran != 0) {
      ac::set_error("chunk %d: chunk_len %lld is not a multiple of %lld within 1..%lld", c, (long long)ch.chunk_len,
                    (long long)gran, (long long)extent);
      return AC_ERR_ARG;
    }
    for (int i = ch.start; i <= ch.end; ++i) {
      if (region_of[i] >= 0) {
        ac::set_error("chunks %d and %d overlap at node %d", region_of[i], c, i);
        return AC_ERR_ARG;
      }
      region_of[i] = c;
    }
  }
  return AC_OK;
}

// Live bytes at every node under the chunk list; returns the peak and its first node.
uint64_t estimate(const Memory& m, const ac_graph_chunk* chunks, const std::vector<std::vector<uint8_t>>& moved,
                  const std::vector<int>& region_of, std::vector<uint64_t>& bytes, int* peak_node) {
  const int n = m.n;
  bytes.assign(n, 0);
  std::vector<uint64_t> fixed, scaled;
  for (int i = 0; i < n;) {
    if (region_of[i] < 0) {
      bytes[i] = m.whole[i];
      ++i;
      continue;
    }
    const int c = region_of[i];
    const ac_graph_chunk& ch = chunks[c];
    const uint64_t extent = (uint64_t)m.t.g[ch.end].shape[ch.out_dim];
    m.region(ch.start, ch.end, moved[c].data(), fixed, scaled);
    for (int k = ch.start; k <= ch.end; ++k)
      bytes[k] = fixed[k - ch.start] + (uint64_t)((u128)scaled[k - ch.start] * (u128)ch.chunk_len / extent);
    i = ch.end + 1;
  }
  uint64_t peak = 0;
  *peak_node = 0;
  for (int i = 0; i < n; ++i)
    if (bytes[i] > peak) {
      peak = bytes[i];
      *peak_node = i;
    }
  return peak;
}

template <class... A>
int bad(const char* fmt, A... a) {
  ac::set_error(fmt, a...);
  return AC_ERR_ARG;
}

}  // namespace

extern "C" int ac_chunk_trace(const ac_graph_node* nodes, int n_nodes, int start, int end, int out_dim, int hoist,
                              int32_t* node_dims, uint8_t* node_moved, int* legal) {
  if (legal) *legal = 0;
  if (!legal || !node_dims) return bad("ac_chunk_trace: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_chunk_trace: malformed graph");
  if (start < 0 || end < start || end >= n_nodes) return bad("ac_chunk_trace: region [%d, %d] outside the graph", start, end);
  if (out_dim < 0 || out_dim >= nodes[end].rank) return bad("ac_chunk_trace: node %d has no dim %d", end, out_dim);
  if (hoist != 0 && hoist != 1) return bad("ac_chunk_trace: hoist must be 0 or 1");
  Tracer t(nodes, n_nodes);
  if (t.holds_leaf(start, end)) return bad("ac_chunk_trace: region [%d, %d] holds an input or parameter node", start, end);
  int64_t gran = 1;
  std::vector<uint8_t> moved(n_nodes, 0);
  if (t.trace(start, end, out_dim, hoist != 0, node_dims, moved.data(), &gran)) {
    *legal = 1;
  } else {
    for (int i = 0; i < n_nodes; ++i) node_dims[i] = -1;
    moved.assign(n_nodes, 0);
  }
  if (node_moved)
    for (int i = 0; i < n_nodes; ++i) node_moved[i] = moved[i];
  return AC_OK;
}

extern "C" int ac_chunk_search(const ac_graph_node* nodes, int n_nodes, int peak, int window, int hoist,
                               ac_chunk_candidate* out, int32_t* node_dims, uint8_t* node_moved, int max_out,
                               int* n_found, int* n_tried, int* n_passed) {
  if (n_found) *n_found = 0;
  if (n_tried) *n_tried = 0;
  if (n_passed) *n_passed = 0;
  if (!n_found) return bad("ac_chunk_search: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_chunk_search: malformed graph");
  if (peak < 0 || peak >= n_nodes || window < 1 || max_out < 0 || (hoist != 0 && hoist != 1))
    return bad("ac_chunk_search: peak %d, window %d, hoist %d or max_out %d out of range", peak, window, hoist, max_out);
  if (max_out > 0 && (!out || !node_dims)) return bad("ac_chunk_search: null output with max_out %d", max_out);
  Tracer t(nodes, n_nodes);
  int found = 0, tried = 0, passed = 0;
  t.candidates(peak, window, hoist != 0, &tried, &passed,
               [&](int start, int end, int d, int64_t gran, const int32_t* row, const uint8_t* moved) {
    if (found < max_out) {
      out[found].start = start;
      out[found].end = end;
      out[found].out_dim = d;
      out[found].granule = (int32_t)gran;
      for (int i = 0; i < n_nodes; ++i) node_dims[(size_t)found * n_nodes + i] = row[i];
      if (node_moved)
        for (int i = 0; i < n_nodes; ++i) node_moved[(size_t)found * n_nodes + i] = (i >= start && i <= end) ? moved[i] : 0;
    }
    ++found;
  });
  *n_found = found;
  if (n_tried) *n_tried = tried;
  if (n_passed) *n_passed = passed;
  return AC_OK;
}

extern "C" int ac_graph_estimate(const ac_graph_node* nodes, int n_nodes, int elem_bytes,
                                 const ac_graph_chunk* chunks, int n_chunks, uint64_t* node_bytes,
                                 uint64_t* peak_bytes, int* peak_node) {
  if (!peak_bytes || !peak_node || (n_chunks > 0 && !chunks)) return bad("ac_graph_estimate: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_graph_estimate: malformed graph");
  if (elem_bytes < 1 || n_chunks < 0) return bad("ac_graph_estimate: elem_bytes %d or n_chunks %d out of range", elem_bytes, n_chunks);
  Tracer t(nodes, n_nodes);
  std::vector<int> region_of;
  std::vector<std::vector<uint8_t>> moved;
  const int st = check_chunks(t, chunks, n_chunks, region_of, moved);
  if (st != AC_OK) return st;
  Memory m(t, elem_bytes);
  std::vector<uint64_t> bytes;
  *peak_bytes = estimate(m, chunks, moved, region_of, bytes, peak_node);
  if (node_bytes)
    for (int i = 0; i < n_nodes; ++i) node_bytes[i] = bytes[i];
  return AC_OK;
}

extern "C" int ac_graph_chunk_cost(const ac_graph_node* nodes, int n_nodes, int start, int end, int out_dim, int hoist,
                                   const double* weights, double* cost) {
  if (!weights || !cost) return bad("ac_graph_chunk_cost: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_graph_chunk_cost: malformed graph");
  if (start < 0 || end < start || end >= n_nodes || out_dim < 0 || out_dim >= nodes[end].rank || (hoist != 0 && hoist != 1))
    return bad("ac_graph_chunk_cost: region [%d, %d], dim %d or hoist %d not valid for the graph", start, end, out_dim, hoist);
  if (!hoist) {
    *cost = chunk_cost(nodes, start, end, out_dim, nullptr, weights);
    return AC_OK;
  }
  Tracer t(nodes, n_nodes);
  if (t.holds_leaf(start, end)) return bad("ac_graph_chunk_cost: region [%d, %d] holds an input or parameter node", start, end);
  std::vector<int32_t> row(n_nodes);
  std::vector<uint8_t> moved(n_nodes, 0);
  int64_t gran = 1;
  if (!t.trace(start, end, out_dim, true, row.data(), moved.data(), &gran)) {
    ac::set_error("ac_graph_chunk_cost: region [%d, %d] cannot be cut along dim %d", start, end, out_dim);
    return AC_ERR_ILLEGAL_CHUNK_DIM;
  }
  *cost = chunk_cost(nodes, start, end, out_dim, moved.data(), weights);
  return AC_OK;
}

namespace {

// One chunk strategy of the beam: its chunks in the order chosen (each with the nodes it
// moves ahead of its segments), the sum of their costs and of their segment counts.
struct Strategy {
  double total = 0;
  int64_t segments = 0;
  std::vector<ac_graph_chunk> chunks;
  std::vector<std::vector<uint8_t>> moved;
};

typedef std::vector<std::array<int64_t, 5>> StrategyKey;  // the chunks, sorted: order of choice does not matter

StrategyKey key_of(const std::vector<ac_graph_chunk>& chunks) {
  StrategyKey k;
  for (const ac_graph_chunk& c : chunks) k.push_back({c.start, c.end, c.out_dim, c.chunk_len, c.hoist});
  std::sort(k.begin(), k.end());
  return k;
}

}  // namespace

extern "C" int ac_graph_plan(const ac_graph_node* nodes, int n_nodes, int elem_bytes, uint64_t budget_bytes,
                             int window, const double* weights, int beam, int hoist, ac_graph_chunk* out, int max_out,
                             int* n_out, uint64_t* peak_bytes) {
  if (n_out) *n_out = 0;
  if (!weights || !out || !n_out || !peak_bytes) return bad("ac_graph_plan: null argument");
  if (!graph_ok(nodes, n_nodes)) return bad("ac_graph_plan: malformed graph");
  if (elem_bytes < 1 || window < 1 || beam < 1 || max_out < 1 || (hoist != 0 && hoist != 1))
    return bad("ac_graph_plan: elem_bytes %d, window %d, beam %d, hoist %d or max_out %d out of range", elem_bytes, window,
               beam, hoist, max_out);
  Tracer t(nodes, n_nodes);
  Memory m(t, elem_bytes);
  std::vector<int> region_of(n_nodes);
  std::vector<uint64_t> bytes, fixed, scaled;
  auto estimate_of = [&](const Strategy& st, int* peak_node) {
    region_of.assign(n_nodes, -1);
    for (size_t c = 0; c < st.chunks.size(); ++c)
      for (int i = st.chunks[c].start; i <= st.chunks[c].end; ++i) region_of[i] = (int)c;
    return estimate(m, st.chunks.data(), st.moved, region_of, bytes, peak_node);
  };
  int peak_node = 0;
  std::vector<Strategy> states(1);
  *peak_bytes = estimate_of(states[0], &peak_node);
  // Section 3.4: least summed cost among the strategies whose peak is within the budget.  A
  // strategy that fits competes for the answer and takes no place in the beam; of those that
  // do not fit yet the `beam` cheapest go on to the next pass; the search ends with the beam.
  Strategy incumbent;
  bool have = *peak_bytes <= budget_bytes;   // nothing to chunk: the empty strategy
  auto better = [](const Strategy& a, const Strategy& b) {
    return a.total < b.total || (a.total == b.total && a.segments < b.segments);
  };
  while (!have || !states.empty()) {
    if (states.empty()) break;
    if (have && states.size() == 1 && states[0].chunks.empty()) break;   // the unchunked graph fits
    std::vector<Strategy> grown;
    std::set<StrategyKey> known;
    for (const Strategy& st : states) {
      estimate_of(st, &peak_node);  // leaves region_of set for st
      if (region_of[peak_node] >= 0) continue;  // the peak lies in a region already chunked: a dead end
      const std::vector<int> region_of_st = region_of;
      int tried = 0, passed = 0;
      t.candidates(peak_node, window, hoist != 0, &tried, &passed,
                   [&](int start, int end, int d, int64_t gran, const int32_t*, const uint8_t* moved) {
        for (int i = start; i <= end; ++i)
          if (region_of_st[i] >= 0) return;
        const int64_t extent = nodes[end].shape[d];
        const int64_t len = m.longest_len(start, end, moved, extent, gran, budget_bytes, fixed, scaled);
        if (len < gran) return;
        Strategy next = st;
        next.chunks.push_back(ac_graph_chunk{start, end, d, hoist, len});
        if (!known.insert(key_of(next.chunks)).second) return;  // the same chunks, chosen in another order
        next.moved.emplace_back(moved, moved + n_nodes);
        for (int i = 0; i < n_nodes; ++i)
          if (i < start || i > end) next.moved.back()[i] = 0;
        next.total = st.total + chunk_cost(nodes, start, end, d, moved, weights);
        next.segments = st.segments + (extent + len - 1) / len;
        int pn = 0;
        if (estimate_of(next, &pn) <= budget_bytes) {
          if (!have || better(next, incumbent)) { incumbent = std::move(next); have = true; }
        } else {
          grown.push_back(std::move(next));
        }
      });
    }
    std::stable_sort(grown.begin(), grown.end(), better);
    if ((int)grown.size() > beam) grown.resize(beam);
    states.swap(grown);
  }
  if (!have) {
    ac::set_error("ac_graph_plan: no chunk strategy brings the peak of %llu bytes within %llu",
                  (unsigned long long)*peak_bytes, (unsigned long long)budget_bytes);
    return AC_ERR_BUDGET_INFEASIBLE;
  }
  const Strategy& best = incumbent;
  if ((int)best.chunks.size() > max_out) return bad("ac_graph_plan: %d chunks needed, max_out is %d", (int)best.chunks.size(), max_out);
  for (size_t c = 0; c < best.chunks.size(); ++c) out[c] = best.chunks[c];
  *n_out = (int)best.chunks.size();
  *peak_bytes = estimate_of(best, &peak_node);
  return AC_OK;
}

extern "C" int ac_graph_chunks_to_regions(const ac_node_tag* tags, int n_nodes, const ac_graph_chunk* chunks, int n_chunks,
                                          ac_region_desc* out, int max_out, int* n_out) {
  if (n_out) *n_out = 0;
  if (!tags || !n_out || n_nodes < 1 || n_chunks < 0 || max_out < 0 || (n_chunks > 0 && (!chunks || !out)))
    return bad("ac_graph_chunks_to_regions: null or negative argument");
  struct Kind { bool set = false; int dim = 0, group = 0; int64_t len = 0; };
  Kind kinds[AC_REGION_KINDS];
  for (int c = 0; c < n_chunks; ++c) {
    const ac_graph_chunk& ch = chunks[c];
    if (ch.start < 0 || ch.end < ch.start || ch.end >= n_nodes || ch.out_dim < 0 || ch.out_dim >= AC_GRAPH_MAX_RANK || ch.chunk_len < 1)
      return bad("ac_graph_chunks_to_regions: chunk %d: bad region [%d, %d], dim %d or length", c, ch.start, ch.end, ch.out_dim);
    const ac_node_tag& last = tags[ch.end];
    if (last.region_kind < 0 || last.region_kind >= AC_REGION_KINDS)
      return bad("ac_graph_chunks_to_regions: chunk %d ends at node %d, which no region kind of the executor computes", c, ch.end);
    for (int i = ch.start; i <= ch.end; ++i)
      if (tags[i].region_kind != last.region_kind || tags[i].group != last.group)
        return bad("ac_graph_chunks_to_regions: chunk [%d, %d] lies in no single region kind of one layer (node %d)", ch.start, ch.end, i);
    const int dim = last.dim[ch.out_dim];
    const int64_t unit = last.unit[ch.out_dim];
    if (dim < 0 || unit < 1) {
      ac::set_error("ac_graph_chunks_to_regions: chunk [%d, %d] is cut along dim %d of node %d: the executor has no such chunk dim",
                    ch.start, ch.end, ch.out_dim, ch.end);
      return AC_ERR_UNSUPPORTED;
    }
    Kind& k = kinds[last.region_kind];
    const int64_t len = ch.chunk_len * unit;
    if (k.set && k.dim != dim)
      return bad("ac_graph_chunks_to_regions: layers %d and %d disagree on the chunk dim of region kind %d", k.group, last.group, last.region_kind);
    k.len = k.set ? std::min(k.len, len) : len;
    k.set = true; k.dim = dim; k.group = last.group;
  }
  int n = 0;
  for (int kind = 0; kind < AC_REGION_KINDS; ++kind) {
    if (!kinds[kind].set) continue;
    if (n >= max_out) return bad("ac_graph_chunks_to_regions: more than %d region kinds", max_out);
    out[n].kind = kind; out[n].chunk_dim = kinds[kind].dim; out[n].chunk_len = kinds[kind].len;
    ++n;
  }
  *n_out = n;
  return AC_OK;
}
