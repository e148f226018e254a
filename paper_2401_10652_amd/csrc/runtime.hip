// Host side of the library: chunk plan, workspace arena, segment loop, C-ABI.
//
// AutoChunk section 2.2 / 3.1: a region Y^c = F(X^c, X^nc) is run one segment of its
// chunk dimension after another; only the intermediates of ONE segment are alive at a
// time.  The arena below makes that literal: whole tensors (layer input/output, keys and
// values, the second triangle operand) are pushed once, per-segment intermediates are
// pushed at the start of a segment and released at its end, and the high-water mark of
// the arena is the activation memory the plan needs.  Planning is a dry run of the very
// same walk with launches switched off, so planned and measured peaks agree by
// construction.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "common.h"

namespace ac {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline bool aligned256(const void* p) { return ((uintptr_t)p & 255u) == 0; }

enum KClass { K_GEMM = 0, K_ATTN = 1, K_LN = 2, K_ELEM = 3, K_TRI = 4, K_CLASSES = 5 };
static const char* const kClassName[K_CLASSES] = {"gemm", "attention", "layernorm", "elementwise", "trimul"};

struct Arena {
  uint8_t* base = nullptr;   // null during planning
  uint64_t top = 0, high = 0;
  uint64_t* watch = nullptr;   // high-water mark of the region being walked (planning)
  void* push(uint64_t bytes) {
    const uint64_t off = align_up(top, 256);
    top = off + bytes;
    high = std::max(high, top);
    if (watch) *watch = std::max(*watch, top);
    // during planning the "pointer" is only an offset and is never dereferenced
    return base ? (void*)(base + off) : (void*)(uintptr_t)(off + 256);
  }
  uint64_t mark() const { return top; }
  void release(uint64_t m) { top = m; }
};

struct Setting {   // chunk setting of one region kind (section 3.3, rule 4: one per region)
  bool present = false;
  int chunk_dim = 0;
  int64_t chunk_len = 0;   // resolved: 1..extent
  int64_t extent = 0;
  bool sized_by_budget = false;
};

struct WeightSlot { std::string name; int64_t rows, cols; };

struct ProfRec { int cls; hipEvent_t start, stop; double flops, bytes; };

}  // namespace ac

using namespace ac;

struct ac_plan {
  ac_model_desc m;
  Setting set[AC_REGION_KINDS];
  uint64_t budget = 0;
  std::vector<WeightSlot> weights;
  std::vector<const void*> wptr;
  bool bound = false;
  ac_plan_info info;
  // profiling
  bool profiling = false;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  size_t pool_used = 0;
  // second lane (AC_FLAG_TWO_SEGMENTS_IN_FLIGHT): a stream of default priority and untimed events
  hipStream_t aux_stream = nullptr;
  std::vector<hipEvent_t> sync_pool;
  size_t sync_used = 0;
  int sync_needed = 0;
  int64_t region_launches[AC_REGION_KINDS] = {};   // launches per layer of a region whose segments share launches (0: one per segment)
};

namespace ac {

static int elem_bytes(int dtype) { return dtype == AC_BF16 ? 2 : 4; }

static uint64_t attention_split_bytes(int64_t rows, int64_t batch, int heads, int head_dim, int ns);

// A run [i0, i0 + ni) of rows (or columns) of a pair tensor.
struct RowSeg { int64_t i0, ni; };

// One walk of the plan: either a dry run (planning) or the real thing.
struct Walk {
  ac_plan* p;
  bool dry;
  bool unchunked;          // planning variant: one segment per region
  hipStream_t stream;      // the stream the next kernel goes to (the caller's, or the second lane's)
  Arena arena;
  double flops = 0;
  hipError_t err = hipSuccess;
  const char* err_where = "";
  // Two segments in flight (AC_FLAG_TWO_SEGMENTS_IN_FLIGHT): segments of a region alternate
  // between the caller's stream and a second stream of the plan, each lane with its own
  // per-segment workspace; the lanes are joined at the end of every segment loop.
  int lanes = 1;
  hipStream_t lane_stream[2] = {nullptr, nullptr};
  bool measuring = false;  // sizing pass of a segment loop: pushes only, no launches, no counts
  // highest arena offset reached while each region kind was being walked: a region's own peak,
  // which depends on its own chunk length only (the whole tensors around it are fixed)
  uint64_t region_high[AC_REGION_KINDS] = {};
  void enter(int kind) { arena.watch = &region_high[kind]; }

  int sync_events = 0;     // planning: events one execute needs for its forks and joins
  int64_t region_launches[AC_REGION_KINDS] = {};   // launches per layer of a region whose segments share launches
  void fork() {
    if (dry && lanes == 2) ++sync_events;
    if (dry || lanes != 2 || !ok()) return;
    hipEvent_t e = next_sync_event();
    if (!e) return;
    if (hipEventRecord(e, lane_stream[0]) != hipSuccess || hipStreamWaitEvent(lane_stream[1], e, 0) != hipSuccess) {
      err = hipGetLastError(); err_where = "fork";
    }
  }
  void join() {
    stream = lane_stream[0];
    if (dry && lanes == 2) ++sync_events;
    if (dry || lanes != 2 || !ok()) return;
    hipEvent_t e = next_sync_event();
    if (!e) return;
    if (hipEventRecord(e, lane_stream[1]) != hipSuccess || hipStreamWaitEvent(lane_stream[0], e, 0) != hipSuccess) {
      err = hipGetLastError(); err_where = "join";
    }
  }
  hipEvent_t next_sync_event();

  // Runs body(segment) for every segment of a region.  One lane: each segment's pushes start at
  // the same arena offset.  Two lanes: a sizing pass finds the largest segment's extent
  // (transient pushes included), lane 1 works that far above lane 0, segments alternate.
  template <typename S, typename F>
  void seg_loop(const std::vector<S>& segs, F&& body) {
    const uint64_t base = arena.mark();
    uint64_t extent = 0;
    if (lanes == 2 && segs.size() > 1) {
      const bool was = measuring;
      const uint64_t high0 = arena.high;
      measuring = true;
      for (const S& sg : segs) {
        arena.release(base);
        arena.high = base;
        body(sg);
        extent = std::max(extent, arena.high - base);
      }
      arena.high = high0;
      measuring = was;
      extent = align_up(extent, 256);
    }
    const bool two = lanes == 2 && segs.size() > 1 && !measuring;
    if (two) fork();
    int i = 0;
    for (const S& sg : segs) {
      const int lane = two ? (i & 1) : 0;
      arena.release(base + (uint64_t)lane * extent);
      if (two) stream = lane_stream[lane];
      body(sg);
      ++i;
    }
    if (two) join();
    arena.release(base);
  }

  int eb() const { return elem_bytes(p->m.dtype); }
  const void* w(int layer, int slot, int per_layer) const {
    return dry ? nullptr : p->wptr[(size_t)layer * per_layer + slot];
  }

  bool ok() const { return err == hipSuccess; }

  template <typename F>
  void run(int cls, double fl, double by, const char* where, F&& launch) {
    if (measuring) return;
    flops += fl;
    if (dry || !ok()) return;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (p->profiling) {
      if (p->pool_used + 2 > p->pool.size()) {
        for (int i = 0; i < 64; ++i) {
          hipEvent_t e;
          if (hipEventCreate(&e) != hipSuccess) { err = hipGetLastError(); err_where = "hipEventCreate"; return; }
          p->pool.push_back(e);
        }
      }
      e0 = p->pool[p->pool_used++];
      e1 = p->pool[p->pool_used++];
      (void)hipEventRecord(e0, stream);
    }
    hipError_t e = launch();
    if (e != hipSuccess) { err = e; err_where = where; return; }
    if (p->profiling) {
      (void)hipEventRecord(e1, stream);
      p->recs.push_back(ProfRec{cls, e0, e1, fl, by});
    }
  }

  void ln(const void* x, int64_t ldx, const void* g, const void* b, void* y, int64_t ldy, int64_t rows,
          int64_t cols) {
    const int dt = p->m.dtype;
    const float eps = p->m.ln_eps;
    run(K_LN, 8.0 * rows * cols, 2.0 * rows * cols * eb(), "layernorm",
        [&] { return launch_layernorm(x, ldx, g, b, y, ldy, rows, cols, eps, dt, stream); });
  }
  void linear(LinearArgs g) {
    g.dtype = p->m.dtype;
    double by = ((double)g.m * (g.conv_c > 0 ? g.conv_c : g.k) + (double)g.n * g.k + (double)g.m * g.n) * eb();
    if (g.mul) by += (double)g.m * g.n * eb();
    if (g.resid) by += (double)g.m * g.n * eb();
    run(K_GEMM, 2.0 * g.m * g.n * g.k, by, "linear", [&] { return launch_linear(g, stream); });
  }
  // max_split_bytes caps the fp32 partial results of the launch's key splits (fewer splits if needed)
  void attention(AttnArgs a, uint64_t max_split_bytes = UINT64_MAX) {
    a.dtype = p->m.dtype;
    double pairs;   // visible (query, key) pairs per head and problem
    if (a.causal) {
      pairs = 0;
      // rows r see min(sk, q_offset + r + 1) keys
      const int64_t full_from = std::max<int64_t>(0, a.sk - 1 - a.q_offset);   // first r seeing all keys
      const int64_t tri = std::min<int64_t>(a.sq, full_from);
      pairs += (double)tri * (a.q_offset + 1) + (double)tri * (tri - 1) / 2.0;
      pairs += (double)(a.sq - tri) * a.sk;
    } else {
      pairs = (double)a.sq * a.sk;
    }
    const double fl = 4.0 * pairs * a.head_dim * a.heads * a.batch;
    // q and ctx rows of the segment, k and v rows any of them sees (causal: keys up to the last row)
    const int64_t keys_seen = a.causal ? std::min<int64_t>(a.sk, a.q_offset + a.sq) : a.sk;
    double by = ((double)a.sq * 2 + (double)keys_seen * 2) * a.heads * a.head_dim * a.batch * eb();
    if (a.gate) by += (double)a.sq * a.heads * a.head_dim * a.batch * eb();
    if (a.bias) by += (double)a.sq * a.sk * a.heads * eb();
    // few query rows: cut the keys into runs so that every CU gets blocks; the fp32 partial
    // results live in the arena for the duration of this call
    const uint64_t mk = arena.mark();
    // (a causal segment sees keys up to its last row only: early segments need fewer runs or none)
    a.n_splits = attention_key_splits(a.sq, keys_seen, a.heads, a.batch, a.head_dim, a.dtype, a.v_transposed);
    while (a.n_splits > 1 && attention_split_bytes(a.sq, a.batch, a.heads, a.head_dim, a.n_splits) > max_split_bytes)
      --a.n_splits;
    if (a.n_splits > 1) {
      const uint64_t rh = (uint64_t)a.n_splits * a.batch * a.sq * a.heads;
      a.part_o = arena.push(rh * a.head_dim * 4);
      a.part_ml = arena.push(rh * 2 * 4);
    }
    run(K_ATTN, fl, by, "attention", [&] { return launch_attention(a, stream); });
    arena.release(mk);
  }
  // The attention core as an unfused graph holds it (AC_FLAG_MATERIALIZED_SCORES): per problem
  // scores[h] = q_h k_h^T and probabilities[h] = softmax(scores[h] / sqrt(d_h)) are stored
  // tensors of the segment, then ctx_h = probabilities[h] v_h.  v is given transposed.
  void attention_materialized(const AttnArgs& a) {
    const int dt = p->m.dtype;
    const int e = eb();
    const int64_t c = a.sq, S = a.sk, H = a.heads, dh = a.head_dim;
    const uint64_t mk = arena.mark();
    uint8_t* scores = (uint8_t*)arena.push((uint64_t)a.batch * H * c * S * e);
    uint8_t* probs = (uint8_t*)arena.push((uint64_t)a.batch * H * c * S * e);
    const float scale = 1.0f / sqrtf((float)dh);
    for (int64_t b = 0; b < a.batch && ok(); ++b) {
      const uint64_t off = (uint64_t)b * H * c * S * e;
      LinearArgs g1{};
      g1.a = (const uint8_t*)a.q + b * a.sq_b * e; g1.lda = a.ldq; g1.sa_b = dh;
      g1.w = (const uint8_t*)a.k + b * a.sk_b * e; g1.ldw = a.ldk; g1.sw_b = dh;
      g1.out = dry ? nullptr : scores + off; g1.ldo = S; g1.so_b = c * S;
      g1.m = c; g1.n = S; g1.k = dh; g1.n_split = S; g1.batch = H; g1.act = AC_ACT_NONE; g1.dtype = dt;
      run(K_GEMM, 2.0 * c * S * dh * H, ((double)c * dh + (double)S * dh + (double)c * S) * H * e, "scores",
          [&] { return launch_linear(g1, stream); });
      const void* sp = dry ? nullptr : scores + off;
      void* pp = dry ? nullptr : probs + off;
      const int causal = a.causal;
      const int64_t qo = a.q_offset;
      hipStream_t st = stream;
      run(K_ELEM, 5.0 * c * S * H, 4.0 * c * S * H * e, "softmax",
          [&] { return launch_softmax_rows(sp, S, pp, S, H * c, S, scale, causal, qo, c, dt, st); });
      LinearArgs g2{};
      g2.a = pp; g2.lda = S; g2.sa_b = c * S;
      g2.w = (const uint8_t*)a.v + b * a.sv_b * e; g2.ldw = a.ldv; g2.sw_b = dh * a.ldv;
      g2.out = (uint8_t*)a.ctx + b * a.sc_b * e; g2.ldo = a.ldc; g2.so_b = dh;
      g2.m = c; g2.n = dh; g2.k = S; g2.n_split = dh; g2.batch = H; g2.act = AC_ACT_NONE; g2.dtype = dt;
      run(K_GEMM, 2.0 * c * S * dh * H, ((double)c * S + (double)S * dh + (double)c * dh) * H * e, "context",
          [&] { return launch_linear(g2, stream); });
    }
    arena.release(mk);
  }
  void bias_act(const void* x, int64_t ldx, const void* bias, void* y, int64_t ldy, int64_t rows, int64_t cols,
                int act) {
    const int dt = p->m.dtype;
    run(K_ELEM, 2.0 * rows * cols, 2.0 * rows * cols * eb(), "bias_act",
        [&] { return launch_bias_act(x, ldx, bias, y, ldy, rows, cols, act, dt, stream); });
  }
  void binary(const void* a, int64_t lda, const void* b, int64_t ldb, void* y, int64_t ldy, int64_t rows,
              int64_t cols, int op) {
    const int dt = p->m.dtype;
    run(K_ELEM, 1.0 * rows * cols, 3.0 * rows * cols * eb(), "binary",
        [&] { return launch_binary(a, lda, b, ldb, y, ldy, rows, cols, op, dt, stream); });
  }

  // out = act(a w^T + bias) [+ resid], fused in the GEMM epilogue or as standalone passes.
  void proj(const void* a, int64_t lda, const void* wmat, int64_t kdim, const void* bias, int act,
            const void* resid, int64_t ldr, void* out, int64_t ldo, int64_t rows, int64_t ncols) {
    LinearArgs g{};
    g.a = a; g.lda = lda; g.w = wmat; g.ldw = kdim; g.m = rows; g.n = ncols; g.k = kdim;
    g.n_split = ncols;
    const bool unfused = (p->m.flags & AC_FLAG_UNFUSED_ELEMENTWISE) != 0;
    if (!unfused) {
      g.bias = bias; g.act = act; g.resid = resid; g.ldr = ldr; g.out = out; g.ldo = ldo;
      linear(g);
      return;
    }
    if (resid) {
      const uint64_t mk = arena.mark();
      void* tmp = arena.push((uint64_t)rows * ncols * eb());
      g.out = tmp; g.ldo = ncols; g.act = AC_ACT_NONE;
      linear(g);
      bias_act(tmp, ncols, bias, tmp, ncols, rows, ncols, act);
      binary(tmp, ncols, resid, ldr, out, ldo, rows, ncols, 0);
      arena.release(mk);
    } else {
      g.out = out; g.ldo = ldo; g.act = AC_ACT_NONE;
      linear(g);
      bias_act(out, ldo, bias, out, ldo, rows, ncols, act);
    }
  }

  void transpose_inplace(void* data, int64_t ld, int64_t stride_b, int64_t n, int64_t batch) {
    const int dt = p->m.dtype;
    run(K_ELEM, 0.0, 2.0 * n * n * batch * eb(), "transpose",
        [&] { return launch_transpose_square_inplace(data, ld, stride_b, n, batch, dt, stream); });
  }
  void ln_channel_major(const void* src, int64_t stride_c, const void* g, const void* b, void* dst, int64_t ldd,
                        int64_t positions, int64_t channels) {
    const int dt = p->m.dtype;
    const float eps = p->m.ln_eps;
    run(K_LN, 8.0 * positions * channels, 2.0 * positions * channels * eb(), "layernorm_channel_major", [&] {
      return launch_layernorm_channel_major(src, stride_c, g, b, dst, ldd, positions, channels, eps, dt, stream);
    });
  }
  // out_c[c][i][j] = sum_k a_t[c][i][k] * b_t[c][j][k]: one NT product per channel.
  void contract(const void* a_t, int64_t lda, int64_t sa_c, const void* b_t, int64_t ldb, int64_t sb_c, void* out_c,
                int64_t ldo, int64_t so_c, int64_t ni, int64_t nj, int64_t nk, int64_t channels, bool descending = false) {
    LinearArgs g{};
    g.batch_descending = descending;
    g.a = a_t; g.lda = lda; g.sa_b = sa_c; g.w = b_t; g.ldw = ldb; g.sw_b = sb_c; g.out = out_c; g.ldo = ldo;
    g.so_b = so_c; g.m = ni; g.n = nj; g.k = nk; g.n_split = nj; g.batch = channels; g.dtype = p->m.dtype;
    const double by = ((double)ni * nk + (double)nj * nk + (double)ni * nj) * channels * eb();
    run(K_TRI, 2.0 * ni * nj * nk * channels, by, "triangle_contract", [&] { return launch_linear(g, stream); });
  }

  // LayerNorm of `rows` rows of width k and every projection of `parts` in one kernel (the
  // normalised rows never reach memory).  Callers ask fuses_ln_proj first; planning and
  // execution take the same answer from the shapes alone.
  bool fuses_ln_proj(int64_t k, std::initializer_list<int64_t> ns) const {
    if (p->m.flags & AC_FLAG_UNFUSED_ELEMENTWISE) return false;
    std::vector<int64_t> v(ns);
    return ln_proj_shapes_ok(p->m.dtype, k, v.data(), (int)v.size());
  }
  void ln_proj(const void* x, int64_t ldx, const void* g, const void* b, int64_t rows, int64_t k,
               std::initializer_list<ProjPart> parts) {
    LnProjArgs a{};
    a.x = x; a.ldx = ldx; a.gain = g; a.shift = b; a.eps = p->m.ln_eps; a.rows = rows; a.k = k;
    double fl = 8.0 * rows * k, by = (double)rows * k * eb();
    for (const ProjPart& pp : parts) {
      a.part[a.n_parts++] = pp;
      const double mult = pp.gated ? 2.0 : 1.0;
      fl += 2.0 * rows * k * pp.n * mult;
      by += ((double)rows * pp.n + (double)pp.n * k * mult) * eb();
    }
    run(K_GEMM, fl, by, "ln_proj", [&] { return launch_ln_proj(a, stream); });
  }

  int64_t seg_len(int kind) const { return unchunked ? p->set[kind].extent : p->set[kind].chunk_len; }

  void transformer(const void* x, void* y);
  void pair(const void* x, void* y);
  void res_stack(const void* x, void* y);
  const void* pair_segment(const void* zin, const RowSeg& sg, bool col);
  void pair_store(LinearArgs& o, void* zout, const RowSeg& sg, bool col);
  void tri_mul(int kind, const void* const* W, const void* zin, void* zout);
  void tri_att(int kind, const void* const* W, const void* zin, void* zout);
  void transition(const void* const* W, const void* zin, void* zout);
};

// Events of the forks and joins: all created when the weights are bound (the dry run counted them).
hipEvent_t Walk::next_sync_event() {
  if (p->sync_used == p->sync_pool.size()) {
    err = hipErrorInvalidResourceHandle; err_where = "fork/join event pool";
    return nullptr;
  }
  return p->sync_pool[p->sync_used++];
}

static const char* const kLayerTensor[12] = {"ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                                             "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2"};
enum { W_LN1G, W_LN1B, W_QKV, W_BQKV, W_O, W_BO, W_LN2G, W_LN2B, W_1, W_B1, W_2, W_B2 };

// Rows [r0, r1) of the flattened [batch * seq] token axis that form one segment.
struct Seg { int64_t b0, nb, s0, ns; };

static std::vector<Seg> token_segments(const ac_model_desc& m, int chunk_dim, int64_t len) {
  std::vector<Seg> v;
  if (chunk_dim == AC_DIM_BATCH) {
    for (int64_t b = 0; b < m.batch; b += len) v.push_back(Seg{b, std::min<int64_t>(len, m.batch - b), 0, m.seq});
  } else {
    for (int64_t b = 0; b < m.batch; ++b)
      for (int64_t s = 0; s < m.seq; s += len) v.push_back(Seg{b, 1, s, std::min<int64_t>(len, m.seq - s)});
  }
  return v;
}

// Bytes of fp32 partial results an attention launch with ns key splits keeps in the arena,
// exactly as Walk::attention pushes them.
static uint64_t attention_split_bytes(int64_t rows, int64_t batch, int heads, int head_dim, int ns) {
  if (ns <= 1) return 0;
  const uint64_t rh = (uint64_t)ns * batch * rows * heads;
  return align_up(rh * head_dim * 4, 256) + align_up(rh * 2 * 4, 256);
}
// ... of the launch the plan's own segment g would be, with the split count the launch shape calls for
static uint64_t attention_launch_bytes(const ac_model_desc& m, const Seg& g) {
  const int64_t keys_seen = m.causal ? std::min<int64_t>(m.seq, g.s0 + g.ns) : m.seq;
  const int ns = attention_key_splits(g.ns, keys_seen, m.heads, g.nb, m.head_dim, m.dtype, m.dtype == AC_BF16 ? 1 : 0);
  return attention_split_bytes(g.ns, g.nb, m.heads, m.head_dim, ns);
}

// Runs of consecutive segments (rows of one sequence, then whole sequences of consecutive batch
// elements) as single segments: the launches of a region whose segments hold no tensor of their own.
static std::vector<Seg> merged_segments(const ac_model_desc& m, const std::vector<Seg>& segs) {
  std::vector<Seg> rows;
  for (const Seg& sg : segs) {
    if (!rows.empty() && rows.back().nb == 1 && sg.nb == 1 && rows.back().b0 == sg.b0 &&
        sg.s0 == rows.back().s0 + rows.back().ns)
      rows.back().ns += sg.ns;
    else
      rows.push_back(sg);
  }
  std::vector<Seg> out;
  for (const Seg& sg : rows) {
    if (!out.empty() && out.back().s0 == 0 && sg.s0 == 0 && out.back().ns == m.seq && sg.ns == m.seq &&
        sg.b0 == out.back().b0 + out.back().nb)
      out.back().nb += sg.nb;
    else
      out.push_back(sg);
  }
  return out;
}
// The fused attention keeps no intermediate of a segment in memory (the scores live in
// registers), so consecutive segments of its region may share a launch without raising the
// bytes the plan needs: runs of consecutive segments (rows of one sequence, then whole
// sequences of consecutive batch elements) become one launch, whose key splits are capped so
// that their partial results stay within `bound`, the bytes of the region's largest single
// segment.  The segments are still computed block by block in order; what is saved is the fixed
// cost of a launch and its under-filled tail per segment (section 3.4's computation-density
// term).  A pure function of the shapes: planning and execution agree.
static std::vector<Seg> attention_launch_groups(const ac_model_desc& m, const std::vector<Seg>& segs, uint64_t& bound) {
  bound = 0;
  for (const Seg& sg : segs) bound = std::max(bound, attention_launch_bytes(m, sg));
  return merged_segments(m, segs);
}

void Walk::transformer(const void* x, void* y) {
  const ac_model_desc& m = p->m;
  const int64_t T = (int64_t)m.batch * m.seq, S = m.seq, d = m.d_model, F = m.d_ffn;
  const int e = eb();
  const bool bf = m.dtype == AC_BF16;
  auto at = [&](const void* base, int64_t elems) { return (const void*)((const uint8_t*)base + elems * e); };
  auto atw = [&](void* base, int64_t elems) { return (void*)((uint8_t*)base + elems * e); };

  // Whole tensors of a layer.  bf16: q,k row-major [T, 2d] and v transposed per batch
  // element [d, S]; fp32: q,k,v row-major [T, 3d].
  void* qk = arena.push((uint64_t)T * (bf ? 2 : 3) * d * e);
  const bool stored_scores = (m.flags & AC_FLAG_MATERIALIZED_SCORES) != 0;
  // v transposed: written by the projection's strided store (bf16), or, for the stored-scores
  // attention of an fp32 model, by a transpose after the projection region
  void* vt = (bf || stored_scores) ? arena.push((uint64_t)T * d * e) : nullptr;
  const int64_t ldqk = (bf ? 2 : 3) * d;
  void* ctx_all = arena.push((uint64_t)T * d * e);   // whole context: output of the attention region
  void* hbuf = arena.push((uint64_t)T * d * e);
  void* tbuf = m.layers > 1 ? arena.push((uint64_t)T * d * e) : nullptr;

  for (int l = 0; l < m.layers && ok(); ++l) {
    const void* in = l == 0 ? x : (const void*)tbuf;
    void* out = l == m.layers - 1 ? y : tbuf;
    auto W = [&](int slot) { return w(l, slot, 12); };

    // ---- region 1: LayerNorm 1 + packed projection, writes whole q, k, v
    // The normalised rows go to the context buffer, which holds nothing between the output projection of
    // the layer before and this layer's attention.  The region then has no tensor of a segment's own, and
    // (as for the attention core below) consecutive segments share a launch: the plan's segments bound
    // memory, and where they bound nothing they cost nothing.
    enter(AC_REGION_QKV);
    const std::vector<Seg> qkv_segs = merged_segments(m, token_segments(m, p->set[AC_REGION_QKV].chunk_dim, seg_len(AC_REGION_QKV)));
    region_launches[AC_REGION_QKV] = (int64_t)qkv_segs.size();
    seg_loop(qkv_segs, [&](const Seg& sg) {
      const int64_t r0 = sg.b0 * S + sg.s0, rows = sg.nb * sg.ns;
      void* u = atw(ctx_all, r0 * d);
      ln(at(in, r0 * d), d, W(W_LN1G), W(W_LN1B), u, d, rows, d);
      LinearArgs g{};
      g.a = u; g.lda = d; g.w = W(W_QKV); g.ldw = d; g.m = rows; g.n = 3 * d; g.k = d;
      g.out = atw(qk, r0 * ldqk); g.ldo = ldqk; g.n_split = 3 * d;
      if (bf) {
        g.n_split = 2 * d;
        g.out_t = atw(vt, sg.b0 * d * S + sg.s0);
        g.t_period = sg.ns; g.t_s1 = d * S; g.t_s2 = 1; g.t_s3 = S;
      }
      const bool unfused = (m.flags & AC_FLAG_UNFUSED_ELEMENTWISE) != 0;
      if (!unfused || bf) {   // the strided store of v only exists as a GEMM epilogue
        g.bias = W(W_BQKV);
        linear(g);
      } else {
        linear(g);
        bias_act(g.out, ldqk, W(W_BQKV), g.out, ldqk, rows, 3 * d, AC_ACT_NONE);
      }
    });

    if (stored_scores && !bf) {
      for (int64_t b = 0; b < m.batch && ok(); ++b) {
        const void* src = at(qk, b * S * ldqk + 2 * d);
        void* dst = atw(vt, b * d * S);
        hipStream_t st = stream;
        run(K_ELEM, 0.0, 2.0 * S * d * e, "transpose v", [&] { return launch_transpose(src, ldqk, dst, S, S, d, AC_F32, st); });
      }
    }
    // ---- region 2: attention of a query segment over whole k, v; writes its rows of the context
    enter(AC_REGION_ATTENTION);
    // A feature chunk is a run of whole heads over all rows.
    const bool by_heads = p->set[AC_REGION_ATTENTION].chunk_dim == AC_DIM_FEATURE;
    const int heads_per_seg = by_heads ? (int)(seg_len(AC_REGION_ATTENTION) / m.head_dim) : m.heads;
    std::vector<Seg> attn_segs = by_heads ? std::vector<Seg>{Seg{0, m.batch, 0, S}}
                                          : token_segments(m, p->set[AC_REGION_ATTENTION].chunk_dim, seg_len(AC_REGION_ATTENTION));
    uint64_t split_bound = UINT64_MAX;
    if (!stored_scores) attn_segs = attention_launch_groups(m, attn_segs, split_bound);
    struct HeadSeg { Seg t; int h0, hc; };
    std::vector<HeadSeg> head_segs;
    for (const Seg& sg : attn_segs) {
      // the fused kernel holds nothing per head either: only the stored-scores form runs head group by head group
      const int step = stored_scores ? heads_per_seg : m.heads;
      for (int h0 = 0; h0 < m.heads; h0 += step) head_segs.push_back(HeadSeg{sg, h0, std::min(step, m.heads - h0)});
    }
    region_launches[AC_REGION_ATTENTION] = (int64_t)head_segs.size();
    seg_loop(head_segs, [&](const HeadSeg& hs) {
      const Seg& sg = hs.t;
      const int64_t r0 = sg.b0 * S + sg.s0, c0 = (int64_t)hs.h0 * m.head_dim;
      AttnArgs a{};
      a.q = at(qk, r0 * ldqk + c0); a.ldq = ldqk; a.sq_b = S * ldqk;
      a.k = at(qk, sg.b0 * S * ldqk + d + c0); a.ldk = ldqk; a.sk_b = S * ldqk;
      if (bf) { a.v = at(vt, sg.b0 * d * S + c0 * S); a.ldv = S; a.sv_b = d * S; a.v_transposed = 1; }
      else { a.v = at(qk, sg.b0 * S * ldqk + 2 * d + c0); a.ldv = ldqk; a.sv_b = S * ldqk; a.v_transposed = 0; }
      a.ctx = atw(ctx_all, r0 * d + c0); a.ldc = d; a.sc_b = S * d;
      a.batch = sg.nb; a.sq = sg.ns; a.sk = S; a.heads = hs.hc; a.head_dim = m.head_dim;
      a.causal = m.causal; a.q_offset = sg.s0;
      if (stored_scores) {
        a.v = at(vt, sg.b0 * d * S + c0 * S); a.ldv = S; a.sv_b = d * S; a.v_transposed = 1;
        attention_materialized(a);
      } else {
        attention(a, split_bound);
      }
    });

    // ---- region 2b: output projection + residual
    enter(AC_REGION_OUT_PROJ);
    // (a feature chunk is a block of output columns over all rows: rows of w_o, entries of its bias)
    const bool by_cols = p->set[AC_REGION_OUT_PROJ].chunk_dim == AC_DIM_FEATURE;
    const bool out_fused = !(m.flags & AC_FLAG_UNFUSED_ELEMENTWISE);   // bias and residual in the epilogue: no tensor per segment
    std::vector<Seg> out_segs = by_cols ? std::vector<Seg>{Seg{0, m.batch, 0, S}}
                                        : token_segments(m, p->set[AC_REGION_OUT_PROJ].chunk_dim, seg_len(AC_REGION_OUT_PROJ));
    if (out_fused) out_segs = merged_segments(m, out_segs);
    struct ColSeg { Seg t; int64_t n0, nc; };
    std::vector<ColSeg> col_segs;
    for (const Seg& sg : out_segs) {
      const int64_t step = by_cols && !out_fused ? seg_len(AC_REGION_OUT_PROJ) : d;
      for (int64_t n0 = 0; n0 < d; n0 += step) col_segs.push_back(ColSeg{sg, n0, std::min<int64_t>(step, d - n0)});
    }
    region_launches[AC_REGION_OUT_PROJ] = (int64_t)col_segs.size();
    seg_loop(col_segs, [&](const ColSeg& cs) {
      const Seg& sg = cs.t;
      const int64_t r0 = sg.b0 * S + sg.s0, rows = sg.nb * sg.ns;
      proj(at(ctx_all, r0 * d), d, at(W(W_O), cs.n0 * d), d, at(W(W_BO), cs.n0), AC_ACT_NONE, at(in, r0 * d + cs.n0), d,
           atw(hbuf, r0 * d + cs.n0), d, rows, cs.nc);
    });

    // ---- region 3: LayerNorm 2 + feed-forward + residual
    // LayerNorm 2 writes into the context buffer as well (the output projection has consumed it), for all
    // rows at once; what a segment of this region holds is its hidden tensor.
    enter(AC_REGION_FFN);
    const std::vector<Seg> ffn_segs = token_segments(m, p->set[AC_REGION_FFN].chunk_dim, seg_len(AC_REGION_FFN));
    for (const Seg& sg : merged_segments(m, ffn_segs)) {
      const int64_t r0 = sg.b0 * S + sg.s0, rows = sg.nb * sg.ns;
      ln(at(hbuf, r0 * d), d, W(W_LN2G), W(W_LN2B), atw(ctx_all, r0 * d), d, rows, d);
    }
    seg_loop(ffn_segs, [&](const Seg& sg) {
      const int64_t r0 = sg.b0 * S + sg.s0, rows = sg.nb * sg.ns;
      const void* u = at(ctx_all, r0 * d);
      void* hid = arena.push((uint64_t)rows * F * e);
      proj(u, d, W(W_1), d, W(W_B1), m.activation, nullptr, 0, hid, F, rows, F);
      proj(hid, F, W(W_2), F, W(W_B2), AC_ACT_NONE, at(hbuf, r0 * d), d, atw(out, r0 * d), d, rows, d);
    });
  }
}

// ---------------------------------------------------------------------------------------
// Pair stack.  z is [N, N, c_z]; "rows" are the N*N positions, a segment is a run of output
// rows i (ni * N positions).  Whole operands of a module (the non-chunkable inputs of its
// chunked part) are built first, segment by segment, then the chunked part runs.
// ---------------------------------------------------------------------------------------
enum { TM_LN_IN_G, TM_LN_IN_B, TM_W_AP, TM_B_AP, TM_W_AG, TM_B_AG, TM_W_BP, TM_B_BP, TM_W_BG, TM_B_BG,
       TM_W_G, TM_B_G, TM_LN_OUT_G, TM_LN_OUT_B, TM_W_O, TM_B_O, TM_COUNT };
enum { TA_LN_G, TA_LN_B, TA_W_Q, TA_W_K, TA_W_V, TA_W_BIAS, TA_W_G, TA_B_G, TA_W_O, TA_B_O, TA_COUNT };
enum { PT_LN_G, PT_LN_B, PT_W_1, PT_B_1, PT_W_2, PT_B_2, PT_COUNT };
constexpr int kPairWeights = 2 * TM_COUNT + 2 * TA_COUNT + PT_COUNT;

static const char* const kTmName[TM_COUNT] = {"ln_in_g", "ln_in_b", "w_ap", "b_ap", "w_ag", "b_ag", "w_bp", "b_bp",
                                              "w_bg", "b_bg", "w_g", "b_g", "ln_out_g", "ln_out_b", "w_o", "b_o"};
static const char* const kTaName[TA_COUNT] = {"ln_g", "ln_b", "w_q", "w_k", "w_v", "w_bias", "w_g", "b_g", "w_o", "b_o"};
static const char* const kPtName[PT_COUNT] = {"ln_g", "ln_b", "w_1", "b_1", "w_2", "b_2"};

static std::vector<RowSeg> row_segments(int64_t n, int64_t len) {
  std::vector<RowSeg> v;
  for (int64_t i = 0; i < n; i += len) v.push_back(RowSeg{i, std::min<int64_t>(len, n - i)});
  return v;
}

// Input positions of one segment as a compact [ns * N, c_z] block.  A row chunk is a contiguous
// run of rows of z already.  A column chunk (section 3.3 makes both legal; section 3.4 charges the
// smaller stride) is gathered with the position indices swapped, (jj, i) <- z[i, j0 + jj]: from
// there on the segment is a row segment of the transposed tensor, every module below runs its
// transposed form on it, and the result rows (jj, i) are stored back to z'[i, j0 + jj].
const void* Walk::pair_segment(const void* zin, const RowSeg& sg, bool col) {
  const ac_model_desc& m = p->m;
  const int64_t N = m.n_res, cz = m.c_z;
  if (!col) return (const uint8_t*)zin + sg.i0 * N * cz * eb();
  void* zc = arena.push((uint64_t)sg.ni * N * cz * eb());
  const int dt = m.dtype;
  run(K_ELEM, 0.0, 2.0 * sg.ni * N * cz * eb(), "gather_columns",
      [&] { return launch_gather_columns(zin, zc, N, cz, sg.i0, sg.ni, dt, stream); });
  return zc;
}

// Where the rows of a segment's result go: rows of z' (row chunk), or, for a column chunk whose
// rows are (jj, i), position (i, j0 + jj).
void Walk::pair_store(LinearArgs& o, void* zout, const RowSeg& sg, bool col) {
  const ac_model_desc& m = p->m;
  const int64_t N = m.n_res, cz = m.c_z;
  if (!col) {
    o.out = (uint8_t*)zout + sg.i0 * N * cz * eb(); o.ldo = cz;
  } else {
    o.out = (uint8_t*)zout + sg.i0 * cz * eb(); o.ldo = cz;
    o.o_period = N; o.o_s1 = cz; o.o_s2 = N * cz;     // row jj * N + i -> (i * N + j0 + jj) * c_z
  }
}

void Walk::tri_mul(int kind, const void* const* W, const void* zin, void* zout) {
  const ac_model_desc& m = p->m;
  const int64_t N = m.n_res, cz = m.c_z, ch = m.c_hidden, R = N * N;
  const int e = eb();
  const bool incoming = kind == AC_REGION_TRIMUL_IN;
  const bool col = p->set[kind].chunk_dim == AC_DIM_COL;
  auto at = [&](const void* base, int64_t elems) { return (const void*)((const uint8_t*)base + elems * e); };
  auto atw = [&](void* base, int64_t elems) { return (void*)((uint8_t*)base + elems * e); };
  const uint64_t mk0 = arena.mark();
  enter(kind);
  void* a_t = arena.push((uint64_t)ch * R * e);   // [c][i][k]
  void* b_t = arena.push((uint64_t)ch * R * e);   // [c][j][k]
  const std::vector<RowSeg> segs = row_segments(N, seg_len(kind));
  // ---- whole operands: a and b of every position, channel-major.  Row r = (i, k) of z lands
  // at [c][r]; for the incoming form r = (k, i), and the per-channel matrices are transposed
  // in place afterwards.  (Built in runs of rows of the segment length whatever the chunk dim.)
  // The fused kernel keeps nothing of a run of rows in memory, so it takes them all in one launch.
  const bool fuse_ab = fuses_ln_proj(cz, {ch, ch}), fuse_g = fuses_ln_proj(cz, {cz});
  const std::vector<RowSeg> all_rows{RowSeg{0, N}};
  seg_loop(fuse_ab ? all_rows : segs, [&](const RowSeg& sg) {
    const int64_t r0 = sg.i0 * N, rows = sg.ni * N;
    if (fuse_ab) {   // LayerNorm and the four projections in one kernel; the gates stay in registers
      ProjPart pa{}, pb{};
      pa.w = W[TM_W_AP]; pa.bias = W[TM_B_AP]; pa.w_gate = W[TM_W_AG]; pa.bias_gate = W[TM_B_AG]; pa.gated = 1;
      pa.n = ch; pa.out_t = atw(a_t, r0); pa.t_s2 = 1; pa.t_s3 = R;
      pb.w = W[TM_W_BP]; pb.bias = W[TM_B_BP]; pb.w_gate = W[TM_W_BG]; pb.bias_gate = W[TM_B_BG]; pb.gated = 1;
      pb.n = ch; pb.out_t = atw(b_t, r0); pb.t_s2 = 1; pb.t_s3 = R;
      ln_proj(at(zin, r0 * cz), cz, W[TM_LN_IN_G], W[TM_LN_IN_B], rows, cz, {pa, pb});
      return;
    }
    void* t = arena.push((uint64_t)rows * cz * e);
    void* gate = arena.push((uint64_t)rows * ch * e);
    ln(at(zin, r0 * cz), cz, W[TM_LN_IN_G], W[TM_LN_IN_B], t, cz, rows, cz);
    for (int which = 0; which < 2; ++which) {
      LinearArgs g{};
      g.a = t; g.lda = cz; g.w = W[which ? TM_W_BG : TM_W_AG]; g.ldw = cz; g.bias = W[which ? TM_B_BG : TM_B_AG];
      g.act = AC_ACT_SIGMOID; g.out = gate; g.ldo = ch; g.m = rows; g.n = ch; g.k = cz; g.n_split = ch;
      linear(g);
      LinearArgs v{};
      v.a = t; v.lda = cz; v.w = W[which ? TM_W_BP : TM_W_AP]; v.ldw = cz; v.bias = W[which ? TM_B_BP : TM_B_AP];
      v.mul = gate; v.ldmul = ch; v.m = rows; v.n = ch; v.k = cz;
      v.out_t = atw(which ? b_t : a_t, r0); v.n_split = 0; v.t_period = 0; v.t_s2 = 1; v.t_s3 = R;
      linear(v);
    }
  });
  if (incoming) {
    transpose_inplace(a_t, N, R, N, ch);
    transpose_inplace(b_t, N, R, N, ch);
  }
  // ---- chunked part: rows i (or columns j) of the output.  For columns the contraction runs
  // with the operands exchanged, out^T[j, i] = sum_k b[j, k] a[i, k], on the gathered segment.
  seg_loop(segs, [&](const RowSeg& sg) {
    const int64_t rows = sg.ni * N;
    const void* zs = pair_segment(zin, sg, col);
    void* t = fuse_g ? nullptr : arena.push((uint64_t)rows * cz * e);
    void* gate = arena.push((uint64_t)rows * cz * e);
    void* o_c = arena.push((uint64_t)ch * rows * e);   // [c][segment index][other index]
    void* lo = arena.push((uint64_t)rows * ch * e);
    if (fuse_g) {
      ProjPart pg{};
      pg.w = W[TM_W_G]; pg.bias = W[TM_B_G]; pg.act = AC_ACT_SIGMOID; pg.n = cz; pg.out = gate; pg.ldo = cz;
      ln_proj(zs, cz, W[TM_LN_IN_G], W[TM_LN_IN_B], rows, cz, {pg});
    } else {
      ln(zs, cz, W[TM_LN_IN_G], W[TM_LN_IN_B], t, cz, rows, cz);
      LinearArgs g{};
      g.a = t; g.lda = cz; g.w = W[TM_W_G]; g.ldw = cz; g.bias = W[TM_B_G]; g.act = AC_ACT_SIGMOID;
      g.out = gate; g.ldo = cz; g.m = rows; g.n = cz; g.k = cz; g.n_split = cz;
      linear(g);
    }
    // every segment reads the whole second operand, which is about the size of the memory-side cache: odd
    // segments walk the channels backwards, so a segment starts on the channels the one before ended on
    contract(at(col ? b_t : a_t, sg.i0 * N), N, R, col ? a_t : b_t, N, R, o_c, N, rows, sg.ni, N, N, ch,
             (sg.i0 / seg_len(kind)) % 2 == 1);
    ln_channel_major(o_c, rows, W[TM_LN_OUT_G], W[TM_LN_OUT_B], lo, ch, rows, ch);
    LinearArgs o{};
    o.a = lo; o.lda = ch; o.w = W[TM_W_O]; o.ldw = ch; o.bias = W[TM_B_O]; o.mul = gate; o.ldmul = cz;
    o.resid = zs; o.ldr = cz; o.m = rows; o.n = cz; o.k = ch; o.n_split = cz;
    pair_store(o, zout, sg, col);
    linear(o);
  });
  arena.release(mk0);
}

// Triangle attention.  Two forms of the per-segment work, named after the node whose row chunks
// they serve: the STARTING form (one problem per row of the segment: queries along the row, keys
// and values from the same row, i.e. from the segment itself; bias[h][query][key] whole) and
// the ENDING form (one problem per column: queries are the segment's rows, keys and values
// come from every row, so they are whole operands; bias rows of the segment).  Because
// ending(z) = starting(z^T)^T, a column chunk of either node is the other node's form applied
// to the gathered (transposed) segment.
void Walk::tri_att(int kind, const void* const* W, const void* zin, void* zout) {
  const ac_model_desc& m = p->m;
  const int64_t N = m.n_res, cz = m.c_z, H = m.tri_heads, dh = m.tri_head_dim, hd = H * dh, R = N * N;
  const int e = eb();
  const bool ending = kind == AC_REGION_TRIATT_END;
  const bool col = p->set[kind].chunk_dim == AC_DIM_COL;
  const bool ending_form = ending != col;
  auto at = [&](const void* base, int64_t elems) { return (const void*)((const uint8_t*)base + elems * e); };
  auto atw = [&](void* base, int64_t elems) { return (void*)((uint8_t*)base + elems * e); };
  const uint64_t mk0 = arena.mark();
  enter(kind);
  const std::vector<RowSeg> segs = row_segments(N, seg_len(kind));
  // ---- whole operands, built from runs of rows of z.  The pair bias [h][q][k]: the projection at
  // position (q, k) for the starting node, at (k, q) for the ending node (transposed in place
  // per head afterwards).  For the ENDING form also all keys as [(problem, key)][h*d] and all
  // values channel-major [h*d][problem][key]: for the ending node's row chunks the problem is the
  // column j and the key index the row k of z, so the projection stores the row of position
  // (k, j) at (j, k), 256 contiguous bytes at a time, and the values are transposed in place per
  // channel; for the starting node's column chunks problem and key are (i, k) as z has them.
  void* bias = arena.push((uint64_t)H * R * e);
  void* k_all = ending_form ? arena.push((uint64_t)R * hd * e) : nullptr;
  void* v_all = ending_form ? arena.push((uint64_t)hd * R * e) : nullptr;
  const bool fuse_a = ending_form ? fuses_ln_proj(cz, {H, hd, hd}) : fuses_ln_proj(cz, {H});
  const bool fuse_b = ending_form ? fuses_ln_proj(cz, {hd, hd}) : fuses_ln_proj(cz, {hd, hd, hd, hd});
  const std::vector<RowSeg> all_rows{RowSeg{0, N}};   // the fused kernel holds nothing per run of rows: one launch
  seg_loop(fuse_a ? all_rows : segs, [&](const RowSeg& sg) {
    const int64_t r0 = sg.i0 * N, rows = sg.ni * N;
    // keys of the whole tensor: regrouped by column for the ending node, as they are otherwise
    void* k_dst = !k_all ? nullptr : (ending ? atw(k_all, sg.i0 * hd) : atw(k_all, r0 * hd));
    if (fuse_a) {
      ProjPart pb{}, pk{}, pv{};
      pb.w = W[TA_W_BIAS]; pb.n = H; pb.out_t = atw(bias, r0); pb.t_s2 = 1; pb.t_s3 = R;
      pk.w = W[TA_W_K]; pk.n = hd; pk.out = k_dst; pk.ldo = hd;
      if (ending) { pk.o_period = N; pk.o_s1 = hd; pk.o_s2 = N * hd; }     // row (k - i0, j) -> (j, k)
      pv.w = W[TA_W_V]; pv.n = hd; pv.out_t = v_all ? atw(v_all, r0) : nullptr; pv.t_s2 = 1; pv.t_s3 = R;
      if (ending_form) ln_proj(at(zin, r0 * cz), cz, W[TA_LN_G], W[TA_LN_B], rows, cz, {pb, pk, pv});
      else ln_proj(at(zin, r0 * cz), cz, W[TA_LN_G], W[TA_LN_B], rows, cz, {pb});
      return;
    }
    void* t = arena.push((uint64_t)rows * cz * e);
    ln(at(zin, r0 * cz), cz, W[TA_LN_G], W[TA_LN_B], t, cz, rows, cz);
    LinearArgs b{};
    b.a = t; b.lda = cz; b.w = W[TA_W_BIAS]; b.ldw = cz; b.m = rows; b.n = H; b.k = cz;
    b.out_t = atw(bias, r0); b.n_split = 0; b.t_s2 = 1; b.t_s3 = R;
    linear(b);
    if (ending_form) {
      LinearArgs kk{};
      kk.a = t; kk.lda = cz; kk.w = W[TA_W_K]; kk.ldw = cz; kk.m = rows; kk.n = hd; kk.k = cz;
      kk.out = k_dst; kk.ldo = hd; kk.n_split = hd;
      if (ending) { kk.o_period = N; kk.o_s1 = hd; kk.o_s2 = N * hd; }
      linear(kk);
      LinearArgs vv{};
      vv.a = t; vv.lda = cz; vv.w = W[TA_W_V]; vv.ldw = cz; vv.m = rows; vv.n = hd; vv.k = cz;
      vv.out_t = atw(v_all, r0); vv.n_split = 0; vv.t_s2 = 1; vv.t_s3 = R;
      linear(vv);
    }
  });
  if (ending) {
    transpose_inplace(bias, N, R, N, H);
    if (ending_form) transpose_inplace(v_all, N, R, N, hd);
  }
  // ---- chunked part
  seg_loop(segs, [&](const RowSeg& sg) {
    const int64_t rows = sg.ni * N;
    const void* zs = pair_segment(zin, sg, col);
    void* t = fuse_b ? nullptr : arena.push((uint64_t)rows * cz * e);
    void* q = arena.push((uint64_t)rows * hd * e);
    void* gate = arena.push((uint64_t)rows * hd * e);
    void* ctx = arena.push((uint64_t)rows * hd * e);
    void* k_seg = ending_form ? nullptr : arena.push((uint64_t)rows * hd * e);
    void* v_seg = ending_form ? nullptr : arena.push((uint64_t)rows * hd * e);   // [segment row][h*d][key]
    LinearArgs lq{};
    lq.a = t; lq.lda = cz; lq.w = W[TA_W_Q]; lq.ldw = cz; lq.m = rows; lq.n = hd; lq.k = cz;
    lq.out = q; lq.ldo = hd; lq.n_split = hd;
    if (fuse_b) {   // LayerNorm, q, gate (and k, v of the segment for the starting form) in one kernel
      ProjPart pq{}, pg{}, pk{}, pv{};
      pq.w = W[TA_W_Q]; pq.n = hd; pq.out = q; pq.ldo = hd;
      pg.w = W[TA_W_G]; pg.bias = W[TA_B_G]; pg.act = AC_ACT_SIGMOID; pg.n = hd; pg.out = gate; pg.ldo = hd;
      pk.w = W[TA_W_K]; pk.n = hd; pk.out = k_seg; pk.ldo = hd;
      pv.w = W[TA_W_V]; pv.n = hd; pv.out_t = v_seg; pv.t_period = N; pv.t_s1 = hd * N; pv.t_s2 = 1; pv.t_s3 = N;
      if (ending_form) ln_proj(zs, cz, W[TA_LN_G], W[TA_LN_B], rows, cz, {pq, pg});
      else ln_proj(zs, cz, W[TA_LN_G], W[TA_LN_B], rows, cz, {pq, pg, pk, pv});
    } else {
      ln(zs, cz, W[TA_LN_G], W[TA_LN_B], t, cz, rows, cz);
      linear(lq);
      LinearArgs lg = lq;
      lg.w = W[TA_W_G]; lg.bias = W[TA_B_G]; lg.act = AC_ACT_SIGMOID; lg.out = gate;
      linear(lg);
    }
    AttnArgs a{};
    a.heads = (int)H; a.head_dim = (int)dh; a.causal = 0; a.q_offset = 0; a.v_transposed = 1; a.sk = N;
    a.q = q; a.gate = gate; a.ctx = ctx;
    if (!ending_form) {
      if (!fuse_b) {
        LinearArgs lk = lq;
        lk.w = W[TA_W_K]; lk.out = k_seg;
        linear(lk);
        LinearArgs lv{};
        lv.a = t; lv.lda = cz; lv.w = W[TA_W_V]; lv.ldw = cz; lv.m = rows; lv.n = hd; lv.k = cz;
        lv.out_t = v_seg; lv.n_split = 0; lv.t_period = N; lv.t_s1 = hd * N; lv.t_s2 = 1; lv.t_s3 = N;
        linear(lv);
      }
      // one problem per row of the segment: queries and keys along that row
      a.batch = sg.ni; a.sq = N;
      a.ldq = hd; a.sq_b = N * hd; a.ldg = hd; a.sg_b = N * hd; a.ldc = hd; a.sc_b = N * hd;
      a.k = k_seg; a.ldk = hd; a.sk_b = N * hd;
      a.v = v_seg; a.ldv = N; a.sv_b = hd * N;
      a.bias = bias; a.ld_bias = N; a.s_bias_h = R;
    } else {
      // one problem per column: queries are the segment's rows, keys every row of that column
      a.batch = N; a.sq = sg.ni;
      a.ldq = N * hd; a.sq_b = hd; a.ldg = N * hd; a.sg_b = hd; a.ldc = N * hd; a.sc_b = hd;
      a.k = k_all; a.ldk = hd; a.sk_b = N * hd;
      a.v = v_all; a.ldv = R; a.sv_b = N;
      a.bias = at(bias, sg.i0 * N); a.ld_bias = N; a.s_bias_h = R;
    }
    attention(a);
    LinearArgs o{};
    o.a = ctx; o.lda = hd; o.w = W[TA_W_O]; o.ldw = hd; o.bias = W[TA_B_O]; o.resid = zs; o.ldr = cz;
    o.m = rows; o.n = cz; o.k = hd; o.n_split = cz;
    pair_store(o, zout, sg, col);
    linear(o);
  });
  arena.release(mk0);
}

void Walk::transition(const void* const* W, const void* zin, void* zout) {
  const ac_model_desc& m = p->m;
  const int64_t N = m.n_res, cz = m.c_z, F = (int64_t)m.transition_factor * cz;
  const int e = eb();
  const bool col = p->set[AC_REGION_PAIR_TRANSITION].chunk_dim == AC_DIM_COL;
  enter(AC_REGION_PAIR_TRANSITION);
  seg_loop(row_segments(N, seg_len(AC_REGION_PAIR_TRANSITION)), [&](const RowSeg& sg) {
    const int64_t rows = sg.ni * N;
    const void* zs = pair_segment(zin, sg, col);
    const bool fuse_up = fuses_ln_proj(cz, {F});
    void* u = fuse_up ? nullptr : arena.push((uint64_t)rows * cz * e);
    void* hid = arena.push((uint64_t)rows * F * e);
    if (fuse_up) {
      ProjPart pu{};
      pu.w = W[PT_W_1]; pu.bias = W[PT_B_1]; pu.act = m.activation; pu.n = F; pu.out = hid; pu.ldo = F;
      ln_proj(zs, cz, W[PT_LN_G], W[PT_LN_B], rows, cz, {pu});
    } else {
      ln(zs, cz, W[PT_LN_G], W[PT_LN_B], u, cz, rows, cz);
      proj(u, cz, W[PT_W_1], cz, W[PT_B_1], m.activation, nullptr, 0, hid, F, rows, F);
    }
    if (m.flags & AC_FLAG_UNFUSED_ELEMENTWISE) {   // standalone passes (row chunks only, checked at plan creation)
      proj(hid, F, W[PT_W_2], F, W[PT_B_2], AC_ACT_NONE, zs, cz, (uint8_t*)zout + sg.i0 * N * cz * e, cz, rows, cz);
      return;
    }
    LinearArgs o{};
    o.a = hid; o.lda = F; o.w = W[PT_W_2]; o.ldw = F; o.bias = W[PT_B_2]; o.resid = zs; o.ldr = cz;
    o.m = rows; o.n = cz; o.k = F; o.n_split = cz;
    pair_store(o, zout, sg, col);
    linear(o);
  });
}

void Walk::pair(const void* x, void* y) {
  const ac_model_desc& m = p->m;
  const uint64_t zbytes = (uint64_t)m.n_res * m.n_res * m.c_z * eb();
  // the modules that run: all five per block, or only the listed kinds
  std::vector<int> seq;
  for (int l = 0; l < m.layers; ++l)
    for (int k = 0; k < 5; ++k)
      if (!(m.flags & AC_FLAG_LISTED_REGIONS_ONLY) || p->set[AC_REGION_TRIMUL_OUT + k].present) seq.push_back(l * 5 + k);
  const int modules = (int)seq.size();
  void* tbuf[2] = {nullptr, nullptr};
  if (modules > 1) tbuf[0] = arena.push(zbytes);
  if (modules > 2) tbuf[1] = arena.push(zbytes);
  std::vector<const void*> nullw(kPairWeights, nullptr);
  for (int idx = 0; idx < modules && ok(); ++idx) {
    const int g = seq[idx];
    const void* zin = idx == 0 ? x : (const void*)tbuf[(idx - 1) % 2];
    void* zout = idx == modules - 1 ? y : tbuf[idx % 2];
    const void* const* base = dry ? nullw.data() : p->wptr.data() + (size_t)(g / 5) * kPairWeights;
    switch (g % 5) {
      case 0: tri_mul(AC_REGION_TRIMUL_OUT, base, zin, zout); break;
      case 1: tri_mul(AC_REGION_TRIMUL_IN, base + TM_COUNT, zin, zout); break;
      case 2: tri_att(AC_REGION_TRIATT_START, base + 2 * TM_COUNT, zin, zout); break;
      case 3: tri_att(AC_REGION_TRIATT_END, base + 2 * TM_COUNT + TA_COUNT, zin, zout); break;
      default: transition(base + 2 * TM_COUNT + 2 * TA_COUNT, zin, zout); break;
    }
  }
}

// ---------------------------------------------------------------------------------------
// UNet residual stack: x [B, H, W, C] channels-last.  Per block and per segment of images:
//   a = SiLU(GroupNorm(x));  t = conv3x3(a, w1) + (b1 + temb[image]);  a = SiLU(GroupNorm(t));
//   y = x + conv3x3(a, w2) + b2
// with the bias and the time embedding (one vector per image), and the skip, in the convolutions'
// epilogues.  A segment holds a and t; whole: the [B, C] bias-plus-embedding table, the GroupNorm
// partial statistics, one inter-block buffer.
//
// With heads > 0 an attention block follows every residual block; the positions of an image are its tokens:
//   t = GroupNorm(x) W_in^T + b_in;  t += attention(LN1(t)) W_o^T + b_o;
//   [with a context c of the image: t += attention(q = LNc(t) W_qc^T; k, v = c W_kvc^T) W_oc^T + b_oc;]
//   t += act(LN2(t) W_1^T + b_1) W_2^T + b_2   [gated: (value half) * act(gate half) of a 2F-wide first layer];
//   y = x + t W_out^T + b_out
// Per segment of images it holds the normalised rows (GroupNorm, then either LayerNorm), t (updated in place
// by the two residual epilogues), q | k and the transposed v, the context and the feed-forward's hidden rows.
// ---------------------------------------------------------------------------------------
enum { RB_GN1_G, RB_GN1_B, RB_W1, RB_B1, RB_GN2_G, RB_GN2_B, RB_W2, RB_B2, RB_TEMB, RB_COUNT };
static const char* const kRbName[RB_COUNT] = {"gn1_g", "gn1_b", "w1", "b1", "gn2_g", "gn2_b", "w2", "b2", "temb"};
// (the seven tensors of the cross-attention, AB_LNC_G .. AB_CONTEXT, are only there with a context)
enum { AB_GN_G, AB_GN_B, AB_W_IN, AB_B_IN, AB_LN1_G, AB_LN1_B, AB_W_QKV, AB_B_QKV, AB_W_O, AB_B_O,
       AB_LNC_G, AB_LNC_B, AB_W_QC, AB_W_KVC, AB_W_OC, AB_B_OC, AB_CONTEXT,
       AB_LN2_G, AB_LN2_B, AB_W_1, AB_B_1, AB_W_2, AB_B_2, AB_W_OUT, AB_B_OUT, AB_COUNT };
static const char* const kAbName[AB_COUNT] = {"gn_g", "gn_b", "w_in", "b_in", "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                                              "lnc_g", "lnc_b", "w_qc", "w_kvc", "w_oc", "b_oc", "context",
                                              "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2", "w_out", "b_out"};
constexpr int kAbCross = AB_CONTEXT - AB_LNC_G + 1;
static int ab_tensors(const ac_model_desc& m) { return m.heads <= 0 ? 0 : AB_COUNT - (m.seq > 0 ? 0 : kAbCross); }
// position of attention-block tensor `slot` among the block's bound tensors
static int ab_index(const ac_model_desc& m, int slot) { return slot - (slot > AB_CONTEXT && m.seq <= 0 ? kAbCross : 0); }

void Walk::res_stack(const void* x, void* y) {
  const ac_model_desc& m = p->m;
  const int64_t HW = (int64_t)m.img_h * m.img_w, C = m.channels;
  const int e = eb();
  auto at = [&](const void* base, int64_t elems) { return (const void*)((const uint8_t*)base + elems * e); };
  auto atw = [&](void* base, int64_t elems) { return (void*)((uint8_t*)base + elems * e); };
  const uint64_t img_bytes = (uint64_t)HW * C * e;
  const bool with_attn = m.heads > 0;
  const int per_layer = RB_COUNT + ab_tensors(m);
  const int modules = m.layers * (with_attn ? 2 : 1);          // each maps [B, H, W, C] to the same shape
  void* tbuf[2] = {nullptr, nullptr};
  if (modules > 1) tbuf[0] = arena.push((uint64_t)m.batch * img_bytes);
  if (modules > 2) tbuf[1] = arena.push((uint64_t)m.batch * img_bytes);
  void* bt = arena.push((uint64_t)m.batch * C * e);                                  // b1 + temb, per image
  void* stats = arena.push(group_norm_workspace_bytes(m.batch, m.groups));
  auto image_segments = [&](int kind) {
    std::vector<RowSeg> segs;
    for (int64_t b = 0; b < m.batch; b += seg_len(kind)) segs.push_back(RowSeg{b, std::min<int64_t>(seg_len(kind), m.batch - b)});
    return segs;
  };
  const int dt = m.dtype;
  for (int idx = 0; idx < modules && ok(); ++idx) {
    const int l = with_attn ? idx / 2 : idx;
    const bool attn = with_attn && idx % 2 == 1;
    const void* in = idx == 0 ? x : (const void*)tbuf[(idx - 1) % 2];
    void* out = idx == modules - 1 ? y : tbuf[idx % 2];
    auto W = [&](int slot) { return w(l, attn ? RB_COUNT + ab_index(m, slot) : slot, per_layer); };
    // GroupNorm of a segment's images; their partial statistics sit at the images' own place in the table,
    // so two segments in flight do not share any of it
    auto gn = [&](const RowSeg& sg, const void* src, int gslot, int bslot, void* dst, int act) {
      const void* gg = W(gslot); const void* bb = W(bslot);
      void* st = dry ? nullptr : (void*)((uint8_t*)stats + group_norm_workspace_bytes(sg.i0, m.groups));
      const int64_t nb = sg.ni;
      hipStream_t s_ = stream;
      run(K_LN, 8.0 * nb * HW * C, 3.0 * nb * HW * C * e, "group norm",
          [&] { return launch_group_norm(src, gg, bb, dst, st, nb, HW, (int)C, m.groups, m.ln_eps, act, dt, s_); });
    };
    if (!attn) {
      enter(AC_REGION_RES_BLOCK);
      bias_act(W(RB_TEMB), C, W(RB_B1), bt, C, m.batch, C, AC_ACT_NONE);
      seg_loop(image_segments(AC_REGION_RES_BLOCK), [&](const RowSeg& sg) {
        const int64_t nb = sg.ni, px = nb * HW;
        const void* xs = at(in, sg.i0 * HW * C);
        void* a = arena.push((uint64_t)nb * img_bytes);
        void* t = arena.push((uint64_t)nb * img_bytes);
        auto conv = [&](const void* src, int wslot, const void* bias, int64_t bias_period, const void* resid, void* dst) {
          LinearArgs g{};
          g.a = src; g.lda = C; g.w = W(wslot); g.ldw = 9 * C; g.bias = bias; g.bias_period = bias_period;
          g.resid = resid; g.ldr = C; g.out = dst; g.ldo = C; g.m = px; g.n = C; g.k = 9 * C; g.n_split = C;
          g.conv_h = m.img_h; g.conv_w = m.img_w; g.conv_c = (int)C;
          linear(g);
        };
        gn(sg, xs, RB_GN1_G, RB_GN1_B, a, AC_ACT_SILU);
        conv(a, RB_W1, at(bt, sg.i0 * C), HW, nullptr, t);
        gn(sg, t, RB_GN2_G, RB_GN2_B, a, AC_ACT_SILU);
        conv(a, RB_W2, W(RB_B2), 0, xs, atw(out, sg.i0 * HW * C));
      });
      continue;
    }
    enter(AC_REGION_UNET_ATTN);
    const int64_t F = m.d_ffn, dh = C / m.heads;
    const bool gated = (m.flags & AC_FLAG_GATED_FFN) != 0;
    const int64_t Tc = m.seq, D = m.d_model, Tcp = (Tc + 7) / 8 * 8;   // context tokens, width; padded row of its v^T
    seg_loop(image_segments(AC_REGION_UNET_ATTN), [&](const RowSeg& sg) {
      const int64_t nb = sg.ni, T = nb * HW;
      const void* xs = at(in, sg.i0 * HW * C);
      void* u = arena.push((uint64_t)T * C * e);        // normalised rows: GroupNorm, then LayerNorm 1, then LayerNorm 2
      void* t = arena.push((uint64_t)T * C * e);        // the block's stream, updated in place by the residual epilogues
      void* qk = arena.push((uint64_t)T * 2 * C * e);   // q | k row-major
      void* vt = arena.push((uint64_t)T * C * e);       // v transposed per image: [image][C][HW]
      void* ctx = arena.push((uint64_t)T * C * e);
      void* hid = arena.push((uint64_t)T * (gated ? 2 : 1) * F * e);
      void* act = gated ? arena.push((uint64_t)T * F * e) : hid;
      void* kc = Tc > 0 ? arena.push((uint64_t)nb * Tc * C * e) : nullptr;     // keys of the contexts, row-major
      void* vct = Tc > 0 ? arena.push((uint64_t)nb * C * Tcp * e) : nullptr;   // their values, transposed per image
      gn(sg, xs, AB_GN_G, AB_GN_B, u, AC_ACT_NONE);
      proj(u, C, W(AB_W_IN), C, W(AB_B_IN), AC_ACT_NONE, nullptr, 0, t, C, T, C);
      ln(t, C, W(AB_LN1_G), W(AB_LN1_B), u, C, T, C);
      LinearArgs g{};
      g.a = u; g.lda = C; g.w = W(AB_W_QKV); g.ldw = C; g.bias = W(AB_B_QKV); g.m = T; g.n = 3 * C; g.k = C;
      g.out = qk; g.ldo = 2 * C; g.n_split = 2 * C;
      g.out_t = vt; g.t_period = HW; g.t_s1 = C * HW; g.t_s2 = 1; g.t_s3 = HW;
      linear(g);
      AttnArgs a{};
      a.q = qk; a.ldq = 2 * C; a.sq_b = HW * 2 * C;
      a.k = at(qk, C); a.ldk = 2 * C; a.sk_b = HW * 2 * C;
      a.v = vt; a.ldv = HW; a.sv_b = C * HW; a.v_transposed = 1;
      a.ctx = ctx; a.ldc = C; a.sc_b = HW * C;
      a.batch = nb; a.sq = HW; a.sk = HW; a.heads = m.heads; a.head_dim = (int)dh; a.causal = 0; a.q_offset = 0;
      attention(a);
      proj(ctx, C, W(AB_W_O), C, W(AB_B_O), AC_ACT_NONE, t, C, t, C, T, C);
      if (Tc > 0) {
        // queries go where q | k of the self-attention were; keys and values of the segment's contexts are projected
        // once (a context is a whole input of its image: every position reads all of it)
        ln(t, C, W(AB_LNC_G), W(AB_LNC_B), u, C, T, C);
        proj(u, C, W(AB_W_QC), C, nullptr, AC_ACT_NONE, nullptr, 0, qk, C, T, C);
        LinearArgs kv{};
        kv.a = at(W(AB_CONTEXT), sg.i0 * Tc * D); kv.lda = D; kv.w = W(AB_W_KVC); kv.ldw = D; kv.m = nb * Tc; kv.n = 2 * C; kv.k = D;
        kv.out = kc; kv.ldo = C; kv.n_split = C;
        kv.out_t = vct; kv.t_period = Tc; kv.t_s1 = C * Tcp; kv.t_s2 = 1; kv.t_s3 = Tcp;
        linear(kv);
        AttnArgs c{};
        c.q = qk; c.ldq = C; c.sq_b = HW * C;
        c.k = kc; c.ldk = C; c.sk_b = Tc * C;
        c.v = vct; c.ldv = Tcp; c.sv_b = C * Tcp; c.v_transposed = 1;
        c.ctx = ctx; c.ldc = C; c.sc_b = HW * C;
        c.batch = nb; c.sq = HW; c.sk = Tc; c.heads = m.heads; c.head_dim = (int)dh; c.causal = 0; c.q_offset = 0;
        attention(c);
        proj(ctx, C, W(AB_W_OC), C, W(AB_B_OC), AC_ACT_NONE, t, C, t, C, T, C);
      }
      ln(t, C, W(AB_LN2_G), W(AB_LN2_B), u, C, T, C);
      if (gated) {
        proj(u, C, W(AB_W_1), C, W(AB_B_1), AC_ACT_NONE, nullptr, 0, hid, 2 * F, T, 2 * F);
        void* gate = atw(hid, F);
        bias_act(gate, 2 * F, nullptr, gate, 2 * F, T, F, m.activation);
        binary(hid, 2 * F, gate, 2 * F, act, F, T, F, 1);
      } else {
        proj(u, C, W(AB_W_1), C, W(AB_B_1), m.activation, nullptr, 0, hid, F, T, F);
      }
      proj(act, F, W(AB_W_2), F, W(AB_B_2), AC_ACT_NONE, t, C, t, C, T, C);
      proj(t, C, W(AB_W_OUT), C, W(AB_B_OUT), AC_ACT_NONE, xs, C, atw(out, sg.i0 * HW * C), C, T, C);
    });
  }
}

// ---------------------------------------------------------------------------------------
// Paper-style byte counts of the regions (section 2: M = X + Y + A, chunked M = X + Y + A/n
// with every op output a tensor of its own), used to size chunk lengths from a budget.
// ---------------------------------------------------------------------------------------
static uint64_t model_bytes(const ac_model_desc& m, int kind, int64_t c) {
  const uint64_t b = elem_bytes(m.dtype);
  if (m.workload == AC_TRANSFORMER_STACK) {
    // the token axis is [batch, seq]; c counts sequence rows or batch elements
    const uint64_t T = (uint64_t)m.batch * m.seq, d = m.d_model, F = m.d_ffn, H = m.heads, S = m.seq;
    switch (kind) {
      case AC_REGION_QKV: return T * d * b + 3 * T * d * b + (uint64_t)c * d * b;
      case AC_REGION_ATTENTION: return T * d * b + 3 * T * d * b + T * d * b + 2 * H * (uint64_t)c * S * b;
      case AC_REGION_OUT_PROJ: return 3 * T * d * b + (uint64_t)c * d * b;   // x, ctx, h whole; projection before the residual
      case AC_REGION_FFN: return 2 * T * d * b + (uint64_t)c * d * b + 2 * (uint64_t)c * F * b;
      default: return 0;
    }
  }
  if (m.workload == AC_UNET_RES_STACK) {
    // x and y whole; per segment of c images the seven intermediates of the unfused block
    // (two normalised, two activated, two convolved tensors and the sum with the embedding)
    const uint64_t img = (uint64_t)m.img_h * m.img_w * m.channels * b;
    if (kind == AC_REGION_UNET_ATTN) {
      // per image of a segment, every op output a tensor: the normalised image, t, LayerNorm 1, q, k, v, the
      // context, its projection, the sum, LayerNorm 2, the down projection, the sum, the output projection
      // (13 images' worth), the hidden rows before and after the activation, scores and probabilities
      // with a context: its LayerNorm, queries, context, projection and sum (5 images' worth), keys and values of
      // the context, scores and probabilities against it; gated: first layer twice as wide, activation, product
      const uint64_t hw = (uint64_t)m.img_h * m.img_w, tc = m.seq > 0 ? m.seq : 0;
      const uint64_t ffn = ((m.flags & AC_FLAG_GATED_FFN) ? 4 : 2) * hw * m.d_ffn * b;
      const uint64_t cross = tc ? 5 * img + 2 * tc * m.channels * b + 2 * (uint64_t)m.heads * hw * tc * b : 0;
      return 2 * (uint64_t)m.batch * img + (uint64_t)c * (13 * img + ffn + 2 * (uint64_t)m.heads * hw * hw * b + cross);
    }
    return 2 * (uint64_t)m.batch * img + 7 * (uint64_t)c * img;
  }
  const uint64_t n = m.n_res, cz = m.c_z, ch = m.c_hidden, hd = (uint64_t)m.tri_heads * m.tri_head_dim;
  const uint64_t H = m.tri_heads, cc = (uint64_t)c;
  switch (kind) {
    case AC_REGION_TRIMUL_OUT:
    case AC_REGION_TRIMUL_IN:
      return 2 * n * n * cz * b + 2 * n * n * ch * b + 2 * cc * n * cz * b + 2 * cc * n * ch * b;
    case AC_REGION_TRIATT_START:
    case AC_REGION_TRIATT_END:
      return 2 * n * n * cz * b + 2 * n * n * hd * b + H * n * n * b + cc * n * cz * b + 3 * cc * n * hd * b +
             cc * H * n * n * b;
    case AC_REGION_PAIR_TRANSITION:
      return 2 * n * n * cz * b + cc * n * cz * b + 2 * cc * n * m.transition_factor * cz * b;
    default: return 0;
  }
}

// For a token-axis chunk the model counts rows of ONE segment: seq chunk -> c rows of one
// batch element; batch chunk -> c * seq rows.
static int64_t model_rows(const ac_model_desc& m, const Setting& s, int64_t len) {
  if (m.workload == AC_TRANSFORMER_STACK && s.chunk_dim == AC_DIM_BATCH) return len * m.seq;
  // a feature chunk holds the fraction len / d_model of the region's intermediates: the rows that do the same
  if (m.workload == AC_TRANSFORMER_STACK && s.chunk_dim == AC_DIM_FEATURE)
    return ((int64_t)m.batch * m.seq * len + m.d_model - 1) / m.d_model;
  return len;
}

static void region_kinds(const ac_model_desc& m, int& first, int& count) {
  if (m.workload == AC_TRANSFORMER_STACK) { first = AC_REGION_QKV; count = 4; }
  else if (m.workload == AC_UNET_RES_STACK) { first = AC_REGION_RES_BLOCK; count = m.heads > 0 ? 2 : 1; }
  else { first = AC_REGION_TRIMUL_OUT; count = 5; }
}

static bool dim_legal(const ac_model_desc& m, int kind, int dim, bool& known) {
  known = true;
  if (m.workload == AC_TRANSFORMER_STACK) {
    if (dim == AC_DIM_BATCH || dim == AC_DIM_SEQ) return true;
    // The feature dim of the context (whole heads) and of the output projection (blocks of output
    // columns) can be cut: no node of those regions reduces over it.  The LayerNorms of the other two do.
    if (dim == AC_DIM_FEATURE) return kind == AC_REGION_ATTENTION || kind == AC_REGION_OUT_PROJ;
    if (dim == AC_DIM_HEAD_DIM || dim == AC_DIM_KEY) return false;
  } else if (m.workload == AC_UNET_RES_STACK) {
    // images are independent; positions and channels are reduced over by the GroupNorms and the windows
    if (dim == AC_DIM_BATCH) return true;
    if (dim == AC_DIM_SEQ || dim == AC_DIM_FEATURE) return false;
  } else {
    if (dim == AC_DIM_ROW || dim == AC_DIM_COL) return true;
    if (dim == AC_DIM_CHANNEL || dim == AC_DIM_CONTRACT) return false;
  }
  known = false;
  return false;
}

static void dry_run(ac_plan* p, bool unchunked, uint64_t& arena_bytes, double& flops,
                    uint64_t* region_high = nullptr) {
  Walk wk{p, true, unchunked, nullptr};
  wk.lanes = (p->m.flags & AC_FLAG_TWO_SEGMENTS_IN_FLIGHT) ? 2 : 1;
  if (p->m.workload == AC_TRANSFORMER_STACK) wk.transformer(nullptr, nullptr);
  else if (p->m.workload == AC_UNET_RES_STACK) wk.res_stack(nullptr, nullptr);
  else wk.pair(nullptr, nullptr);
  arena_bytes = wk.arena.high;
  flops = wk.flops;
  if (region_high) memcpy(region_high, wk.region_high, sizeof(wk.region_high));
  if (!unchunked) { p->sync_needed = wk.sync_events; memcpy(p->region_launches, wk.region_launches, sizeof(wk.region_launches)); }
}

static uint64_t io_bytes(const ac_model_desc& m) {
  if (m.workload == AC_TRANSFORMER_STACK) return 2ull * m.batch * m.seq * m.d_model * elem_bytes(m.dtype);
  if (m.workload == AC_UNET_RES_STACK) return 2ull * m.batch * m.img_h * m.img_w * m.channels * elem_bytes(m.dtype);
  return 2ull * m.n_res * m.n_res * m.c_z * elem_bytes(m.dtype);
}

}  // namespace ac

// =========================================================================================
// C-ABI
// =========================================================================================
extern "C" {

const char* ac_status_string(int s) {
  switch (s) {
    case AC_OK: return "ok";
    case AC_ERR_ARG: return "invalid argument";
    case AC_ERR_ILLEGAL_CHUNK_DIM: return "illegal chunk dimension";
    case AC_ERR_BUDGET_INFEASIBLE: return "activation budget infeasible";
    case AC_ERR_WORKSPACE: return "workspace too small";
    case AC_ERR_ALIGN: return "device pointer not 256-byte aligned";
    case AC_ERR_HIP: return "HIP error";
    case AC_ERR_STATE: return "invalid state";
    case AC_ERR_UNSUPPORTED: return "unsupported";
    default: return "unknown status";
  }
}

const char* ac_last_error(void) { return g_err; }

int ac_plan_create(const ac_model_desc* model, const ac_region_desc* regions, int n_regions,
                   uint64_t act_budget_bytes, ac_plan** out) {
  if (!model || !out || n_regions < 0 || (n_regions > 0 && !regions))
    return fail(AC_ERR_ARG, "ac_plan_create: null argument");
  *out = nullptr;
  const ac_model_desc& m = *model;
  if (m.dtype != AC_F32 && m.dtype != AC_BF16) return fail(AC_ERR_ARG, "dtype %d unknown", m.dtype);
  if (m.layers < 1) return fail(AC_ERR_ARG, "layers must be >= 1");
  if (!(m.ln_eps > 0.f)) return fail(AC_ERR_ARG, "ln_eps must be > 0");
  if (m.workload == AC_TRANSFORMER_STACK) {
    if (m.batch < 1 || m.seq < 1 || m.d_model < 1 || m.heads < 1 || m.head_dim < 1 || m.d_ffn < 1)
      return fail(AC_ERR_ARG, "transformer sizes must be positive");
    if ((int64_t)m.heads * m.head_dim != m.d_model)
      return fail(AC_ERR_ARG, "heads * head_dim (%d * %d) != d_model (%d)", m.heads, m.head_dim, m.d_model);
    if (m.activation != AC_ACT_GELU_ERF && m.activation != AC_ACT_GELU_TANH && m.activation != AC_ACT_RELU)
      return fail(AC_ERR_ARG, "activation %d not valid for a feed-forward", m.activation);
    const int hd = m.head_dim;
    if (hd != 8 && hd != 16 && hd != 32 && hd != 64 && hd != 128)
      return fail(AC_ERR_UNSUPPORTED, "head_dim %d has no attention kernel (8, 16, 32, 64, 128)", hd);
    if (m.dtype == AC_BF16 && (m.seq % 8 != 0 || m.d_model % 8 != 0 || m.d_ffn % 8 != 0))
      return fail(AC_ERR_UNSUPPORTED, "bf16 needs seq, d_model and d_ffn to be multiples of 8");
  } else if (m.workload == AC_PAIR_STACK) {
    if (m.n_res < 1 || m.c_z < 1 || m.c_hidden < 1 || m.tri_heads < 1 || m.tri_head_dim < 1 || m.transition_factor < 1)
      return fail(AC_ERR_ARG, "pair-stack sizes must be positive");
    if (m.activation != AC_ACT_GELU_ERF && m.activation != AC_ACT_GELU_TANH && m.activation != AC_ACT_RELU)
      return fail(AC_ERR_ARG, "activation %d not valid for the pair transition", m.activation);
    const int hd = m.tri_head_dim;
    if (hd != 8 && hd != 16 && hd != 32 && hd != 64 && hd != 128)
      return fail(AC_ERR_UNSUPPORTED, "tri_head_dim %d has no attention kernel (8, 16, 32, 64, 128)", hd);
    if (m.n_res % 8 != 0 || m.c_z % 8 != 0 || m.c_hidden % 8 != 0)
      return fail(AC_ERR_UNSUPPORTED, "n_res, c_z and c_hidden must be multiples of 8");
    if ((int64_t)64 * (m.c_hidden + 1) * 4 > 64 * 1024)
      return fail(AC_ERR_UNSUPPORTED, "c_hidden %d too wide for the channel-major LayerNorm tile", m.c_hidden);
    if (m.c_hidden > 65535 || (int64_t)m.tri_heads * m.tri_head_dim > 65535)
      return fail(AC_ERR_UNSUPPORTED, "too many channels for one launch");
  } else if (m.workload == AC_UNET_RES_STACK) {
    if (m.batch < 1 || m.img_h < 1 || m.img_w < 1 || m.channels < 1 || m.groups < 1)
      return fail(AC_ERR_ARG, "residual-stack sizes must be positive");
    if (m.channels % m.groups != 0) return fail(AC_ERR_ARG, "channels (%d) must be a multiple of groups (%d)", m.channels, m.groups);
    if (m.dtype != AC_BF16 || m.channels % 64 != 0 || m.groups > 128 || m.batch > 65535 ||
        (int64_t)m.batch * m.img_h * m.img_w >= (1ll << 31))
      return fail(AC_ERR_UNSUPPORTED, "the 3x3 convolution kernel takes bf16 images with channels in multiples of 64, "
                                      "at most 128 groups and fewer than 2^31 pixels");
    if (m.flags & (AC_FLAG_UNFUSED_ELEMENTWISE | AC_FLAG_BUDGET_PAPER_MODEL))
      return fail(AC_ERR_UNSUPPORTED, "flags %d do not apply to the residual stack", m.flags);
    if (m.heads < 0) return fail(AC_ERR_ARG, "heads must be >= 0");
    if (m.heads > 0) {
      if (m.channels % m.heads != 0) return fail(AC_ERR_ARG, "channels (%d) must be a multiple of heads (%d)", m.channels, m.heads);
      const int dh = m.channels / m.heads;
      if ((dh != 32 && dh != 64 && dh != 128) || m.d_ffn < 64 || m.d_ffn % 64 != 0 || (int64_t)m.img_h * m.img_w % 64 != 0)
        return fail(AC_ERR_UNSUPPORTED, "the attention block takes heads of 32, 64 or 128 channels, a feed-forward width in "
                                        "multiples of 64 and images of a multiple of 64 positions");
      if (m.seq < 0 || (m.seq > 0 && m.d_model < 1)) return fail(AC_ERR_ARG, "context tokens and width must be positive");
      if (m.seq > 0 && m.d_model % 8 != 0) return fail(AC_ERR_UNSUPPORTED, "the context's width must be a multiple of 8");
    } else if (m.seq != 0 || (m.flags & AC_FLAG_GATED_FFN)) {
      return fail(AC_ERR_ARG, "a context or a gated feed-forward needs the attention block (heads > 0)");
    }
  } else {
    return fail(AC_ERR_ARG, "workload %d unknown", m.workload);
  }

  if ((m.flags & AC_FLAG_GATED_FFN) && m.workload != AC_UNET_RES_STACK)
    return fail(AC_ERR_ARG, "AC_FLAG_GATED_FFN applies to the UNet attention block only");
  if ((m.flags & AC_FLAG_MATERIALIZED_SCORES) && m.workload != AC_TRANSFORMER_STACK)
    return fail(AC_ERR_UNSUPPORTED, "AC_FLAG_MATERIALIZED_SCORES applies to the transformer stack only");
  if (m.flags & AC_FLAG_LISTED_REGIONS_ONLY) {
    if (m.workload != AC_PAIR_STACK) return fail(AC_ERR_ARG, "AC_FLAG_LISTED_REGIONS_ONLY applies to the pair stack only");
    if (n_regions < 1) return fail(AC_ERR_ARG, "AC_FLAG_LISTED_REGIONS_ONLY needs at least one region");
  }
  ac_plan* p = new (std::nothrow) ac_plan();
  if (!p) return fail(AC_ERR_ARG, "out of host memory");
  p->m = m;
  p->budget = act_budget_bytes;
  int first, count;
  region_kinds(m, first, count);
  for (int k = first; k < first + count; ++k) {
    Setting& s = p->set[k];
    s.chunk_dim = m.workload == AC_TRANSFORMER_STACK ? AC_DIM_SEQ : m.workload == AC_UNET_RES_STACK ? AC_DIM_BATCH : AC_DIM_ROW;
    s.extent = m.workload == AC_TRANSFORMER_STACK ? m.seq : m.workload == AC_UNET_RES_STACK ? m.batch : m.n_res;
    s.chunk_len = s.extent;
  }
  for (int i = 0; i < n_regions; ++i) {
    const ac_region_desc& r = regions[i];
    if (r.kind < first || r.kind >= first + count) {
      delete p;
      return fail(AC_ERR_ARG, "region kind %d does not belong to this workload", r.kind);
    }
    Setting& s = p->set[r.kind];
    if (s.present) { delete p; return fail(AC_ERR_ARG, "region kind %d listed twice (one chunk setting per region)", r.kind); }
    bool known;
    if (!dim_legal(m, r.kind, r.chunk_dim, known)) {
      delete p;
      if (!known) return fail(AC_ERR_ARG, "chunk_dim %d unknown", r.chunk_dim);
      return fail(AC_ERR_ILLEGAL_CHUNK_DIM,
                  "region %d reduces over dim %d: its segments would not concatenate to the unchunked output",
                  r.kind, r.chunk_dim);
    }
    if (m.workload == AC_PAIR_STACK && r.chunk_dim == AC_DIM_COL && (m.flags & AC_FLAG_UNFUSED_ELEMENTWISE)) {
      delete p;
      return fail(AC_ERR_UNSUPPORTED, "column chunks store through the GEMM epilogue: not with AC_FLAG_UNFUSED_ELEMENTWISE");
    }
    if (r.chunk_len < 0) { delete p; return fail(AC_ERR_ARG, "chunk_len must be >= 0"); }
    s.present = true;
    s.chunk_dim = r.chunk_dim;
    s.extent = m.workload == AC_TRANSFORMER_STACK ? (r.chunk_dim == AC_DIM_BATCH ? m.batch : r.chunk_dim == AC_DIM_FEATURE ? m.d_model : m.seq)
               : m.workload == AC_UNET_RES_STACK ? m.batch : m.n_res;
    if (m.workload == AC_TRANSFORMER_STACK && r.chunk_dim == AC_DIM_FEATURE) {
      // a segment of the context is a run of whole heads; a block of output columns starts on a 16-byte boundary
      const int64_t g = r.kind == AC_REGION_ATTENTION ? m.head_dim : 8;
      if (r.chunk_len % g != 0) {
        delete p;
        return fail(AC_ERR_ARG, "feature chunk of region %d must be a multiple of %lld", r.kind, (long long)g);
      }
    }
    if (r.chunk_len == 0) {
      s.sized_by_budget = act_budget_bytes > 0;
      s.chunk_len = s.extent;
    } else {
      s.chunk_len = std::min<int64_t>(r.chunk_len, s.extent);
    }
  }

  // ---- paper-style model bytes as an additional bound (AC_FLAG_BUDGET_PAPER_MODEL): largest
  // length (the extent itself, or a multiple of the region's granule below it) whose unfused
  // region bytes fit; explicit lengths are checked against the same bound.
  const int64_t row_granule = m.workload != AC_TRANSFORMER_STACK ? 1 : (m.dtype == AC_BF16 ? 128 : 64);
  auto granule_of = [&](const Setting& s) -> int64_t {
    if (m.workload == AC_TRANSFORMER_STACK && s.chunk_dim == AC_DIM_FEATURE) return &s == &p->set[AC_REGION_ATTENTION] ? m.head_dim : 8;
    return (m.workload == AC_TRANSFORMER_STACK && s.chunk_dim == AC_DIM_BATCH) ? 1 : row_granule;
  };
  auto rows_of = [&](const Setting& s, int64_t len) { return model_rows(m, s, len); };
  if (act_budget_bytes > 0 && (m.flags & AC_FLAG_BUDGET_PAPER_MODEL)) {
    for (int k = first; k < first + count; ++k) {
      Setting& s = p->set[k];
      if (s.sized_by_budget) {
        int64_t c = s.extent;
        const int64_t g = granule_of(s);
        if (model_bytes(m, k, rows_of(s, c)) > act_budget_bytes) {
          c = (s.extent - 1) / g * g;
          while (c >= g && model_bytes(m, k, rows_of(s, c)) > act_budget_bytes) c -= g;
          if (c < g) {
            const uint64_t floor_b = model_bytes(m, k, rows_of(s, g));
            delete p;
            return fail(AC_ERR_BUDGET_INFEASIBLE,
                        "region %d needs %llu bytes even at chunk_len %lld; budget is %llu", k,
                        (unsigned long long)floor_b, (long long)g, (unsigned long long)act_budget_bytes);
          }
        }
        s.chunk_len = c;
      } else if (model_bytes(m, k, rows_of(s, s.chunk_len)) > act_budget_bytes) {
        const uint64_t need = model_bytes(m, k, rows_of(s, s.chunk_len));
        const long long len = (long long)s.chunk_len;
        delete p;
        return fail(AC_ERR_BUDGET_INFEASIBLE, "region %d at chunk_len %lld needs %llu bytes; budget is %llu", k,
                    len, (unsigned long long)need, (unsigned long long)act_budget_bytes);
      }
    }
  }

  // ---- weights
  if (m.workload == AC_TRANSFORMER_STACK) {
    const int64_t d = m.d_model, F = m.d_ffn;
    const int64_t shp[12][2] = {{1, d}, {1, d}, {3 * d, d}, {1, 3 * d}, {d, d}, {1, d},
                                {1, d}, {1, d}, {F, d}, {1, F}, {d, F}, {1, d}};
    for (int l = 0; l < m.layers; ++l)
      for (int t = 0; t < 12; ++t) {
        char nm[48];
        snprintf(nm, sizeof(nm), "L%d.%s", l, kLayerTensor[t]);
        p->weights.push_back(WeightSlot{nm, shp[t][0], shp[t][1]});
      }
  }
  if (m.workload == AC_UNET_RES_STACK) {
    const int64_t C = m.channels;
    const int64_t shp[RB_COUNT][2] = {{1, C}, {1, C}, {C, 9 * C}, {1, C}, {1, C}, {1, C}, {C, 9 * C}, {1, C}, {m.batch, C}};
    const int64_t F = m.d_ffn;
    const int64_t F1 = ((m.flags & AC_FLAG_GATED_FFN) ? 2 : 1) * F, D = m.d_model;
    const int64_t ashp[AB_COUNT][2] = {{1, C}, {1, C}, {C, C}, {1, C}, {1, C}, {1, C}, {3 * C, C}, {1, 3 * C}, {C, C}, {1, C},
                                       {1, C}, {1, C}, {C, C}, {2 * C, D}, {C, C}, {1, C}, {(int64_t)m.batch * m.seq, D},
                                       {1, C}, {1, C}, {F1, C}, {1, F1}, {C, F}, {1, C}, {C, C}, {1, C}};
    for (int l = 0; l < m.layers; ++l) {
      char nm[48];
      for (int t = 0; t < RB_COUNT; ++t) {
        snprintf(nm, sizeof(nm), "R%d.%s", l, kRbName[t]);
        p->weights.push_back(WeightSlot{nm, shp[t][0], shp[t][1]});
      }
      for (int t = 0; m.heads > 0 && t < AB_COUNT; ++t) {
        if (m.seq <= 0 && t >= AB_LNC_G && t <= AB_CONTEXT) continue;
        snprintf(nm, sizeof(nm), "A%d.%s", l, kAbName[t]);
        p->weights.push_back(WeightSlot{nm, ashp[t][0], ashp[t][1]});
      }
    }
  }
  if (m.workload == AC_PAIR_STACK) {
    const int64_t cz = m.c_z, ch = m.c_hidden, hd = (int64_t)m.tri_heads * m.tri_head_dim, H = m.tri_heads;
    const int64_t ft = (int64_t)m.transition_factor * cz;
    const int64_t tm[TM_COUNT][2] = {{1, cz}, {1, cz}, {ch, cz}, {1, ch}, {ch, cz}, {1, ch}, {ch, cz}, {1, ch},
                                     {ch, cz}, {1, ch}, {cz, cz}, {1, cz}, {1, ch}, {1, ch}, {cz, ch}, {1, cz}};
    const int64_t ta[TA_COUNT][2] = {{1, cz}, {1, cz}, {hd, cz}, {hd, cz}, {hd, cz}, {H, cz}, {hd, cz}, {1, hd},
                                     {cz, hd}, {1, cz}};
    const int64_t pt[PT_COUNT][2] = {{1, cz}, {1, cz}, {ft, cz}, {1, ft}, {cz, ft}, {1, cz}};
    for (int l = 0; l < m.layers; ++l) {
      char nm[48];
      const char* pre = "";
      char lbuf[16] = "";
      if (m.layers > 1) { snprintf(lbuf, sizeof(lbuf), "B%d.", l); pre = lbuf; }
      for (int mod = 0; mod < 2; ++mod)
        for (int t = 0; t < TM_COUNT; ++t) {
          snprintf(nm, sizeof(nm), "%s%s.%s", pre, mod ? "tmi" : "tmo", kTmName[t]);
          p->weights.push_back(WeightSlot{nm, tm[t][0], tm[t][1]});
        }
      for (int mod = 0; mod < 2; ++mod)
        for (int t = 0; t < TA_COUNT; ++t) {
          snprintf(nm, sizeof(nm), "%s%s.%s", pre, mod ? "tae" : "tas", kTaName[t]);
          p->weights.push_back(WeightSlot{nm, ta[t][0], ta[t][1]});
        }
      for (int t = 0; t < PT_COUNT; ++t) {
        snprintf(nm, sizeof(nm), "%spt.%s", pre, kPtName[t]);
        p->weights.push_back(WeightSlot{nm, pt[t][0], pt[t][1]});
      }
    }
  }
  p->wptr.assign(p->weights.size(), nullptr);

  // ---- plan = dry run of the walk.  The budget bounds the executor's own bytes, mem(X) + mem(Y)
  // + the arena's high-water mark.  A region's own peak (the highest arena offset reached while
  // it is walked) depends on its own chunk length only, so every region left open is sized on
  // its own: the largest length, the extent or a multiple of its granule, whose peak fits.
  ac_plan_info& inf = p->info;
  memset(&inf, 0, sizeof(inf));
  uint64_t arena = 0;
  double flops = 0;
  uint64_t rhigh[AC_REGION_KINDS];
  const uint64_t io = io_bytes(m);
  dry_run(p, false, arena, flops, rhigh);
  if (act_budget_bytes > 0 && io + arena > act_budget_bytes) {
    for (int k = first; k < first + count; ++k) {
      Setting& s = p->set[k];
      if (!s.sized_by_budget || io + rhigh[k] <= act_budget_bytes) continue;
      const int64_t g = granule_of(s);
      auto fits = [&](int64_t len) {
        s.chunk_len = len;
        dry_run(p, false, arena, flops, rhigh);
        return io + rhigh[k] <= act_budget_bytes;
      };
      // lengths tried: g, 2g, ... below the current one (an upper bound already set by the
      // paper-style model, or the extent); bisection, then a downward walk in case the peak is
      // not monotone in the length (attention key splits grow as the segment shrinks)
      int64_t hi = (s.chunk_len - 1) / g, lo = 1;   // in granules
      if (hi < 1 || !fits(g)) {
        const uint64_t need = io + rhigh[k];
        delete p;
        return fail(AC_ERR_BUDGET_INFEASIBLE, "region %d needs %llu bytes even at chunk_len %lld; budget is %llu", k,
                    (unsigned long long)need, (long long)g, (unsigned long long)act_budget_bytes);
      }
      while (lo < hi) {
        const int64_t mid = (lo + hi + 1) / 2;
        if (fits(mid * g)) lo = mid; else hi = mid - 1;
      }
      while (lo > 1 && !fits(lo * g)) --lo;
      s.chunk_len = lo * g;
    }
    dry_run(p, false, arena, flops, rhigh);
    if (io + arena > act_budget_bytes) {
      delete p;
      return fail(AC_ERR_BUDGET_INFEASIBLE, "executor needs %llu bytes; budget is %llu",
                  (unsigned long long)(io + arena), (unsigned long long)act_budget_bytes);
    }
  }
  inf.workspace_bytes = arena;
  inf.io_bytes = io_bytes(m);
  inf.peak_bytes_planned = inf.io_bytes + arena;
  inf.flops_per_execute = flops;
  uint64_t arena1 = 0;
  double f1 = 0;
  dry_run(p, true, arena1, f1);
  inf.peak_bytes_unchunked_planned = inf.io_bytes + arena1;
  inf.n_regions = count;
  for (int k = first; k < first + count; ++k) {
    const Setting& s = p->set[k];
    ac_region_info& ri = inf.regions[k - first];
    ri.kind = k;
    ri.chunk_dim = s.chunk_dim;
    ri.extent = s.extent;
    ri.chunk_len = s.chunk_len;
    ri.n_segments = ceil_div(s.extent, s.chunk_len);
    ri.launches = p->region_launches[k] > 0 ? p->region_launches[k] : ri.n_segments;
    ri.model_bytes = model_bytes(m, k, rows_of(s, s.chunk_len));
    ri.model_bytes_unchunked = model_bytes(m, k, rows_of(s, s.extent));
    inf.peak_bytes_model = std::max(inf.peak_bytes_model, ri.model_bytes);
    inf.peak_bytes_model_unchunked = std::max(inf.peak_bytes_model_unchunked, ri.model_bytes_unchunked);
  }
  inf.n_weights = (int32_t)p->weights.size();
  for (const WeightSlot& ws : p->weights) inf.weight_bytes += (uint64_t)ws.rows * ws.cols * elem_bytes(m.dtype);
  *out = p;
  return AC_OK;
}

int ac_plan_query(const ac_plan* plan, ac_plan_info* out) {
  if (!plan || !out) return fail(AC_ERR_ARG, "ac_plan_query: null argument");
  *out = plan->info;
  return AC_OK;
}

int ac_plan_weight_info(const ac_plan* plan, int index, ac_weight_info* out) {
  if (!plan || !out) return fail(AC_ERR_ARG, "ac_plan_weight_info: null argument");
  if (index < 0 || index >= (int)plan->weights.size()) return fail(AC_ERR_ARG, "weight index %d out of range", index);
  const WeightSlot& ws = plan->weights[index];
  memset(out, 0, sizeof(*out));
  snprintf(out->name, sizeof(out->name), "%s", ws.name.c_str());
  out->rows = ws.rows;
  out->cols = ws.cols;
  out->dtype = plan->m.dtype;
  out->index = index;
  return AC_OK;
}

int ac_plan_bind_weights(ac_plan* plan, const void* const* dev_ptrs, int n_ptrs) {
  if (!plan || !dev_ptrs) return fail(AC_ERR_ARG, "ac_plan_bind_weights: null argument");
  if (n_ptrs != (int)plan->weights.size())
    return fail(AC_ERR_ARG, "expected %d weight pointers, got %d", (int)plan->weights.size(), n_ptrs);
  for (int i = 0; i < n_ptrs; ++i) {
    if (!dev_ptrs[i]) return fail(AC_ERR_ARG, "weight %d (%s) is null", i, plan->weights[i].name.c_str());
    if (!aligned256(dev_ptrs[i])) return fail(AC_ERR_ALIGN, "weight %d (%s) is not 256-byte aligned", i, plan->weights[i].name.c_str());
  }
  if ((plan->m.flags & AC_FLAG_TWO_SEGMENTS_IN_FLIGHT) && !plan->aux_stream &&
      hipStreamCreateWithFlags(&plan->aux_stream, hipStreamNonBlocking) != hipSuccess)
    return fail(AC_ERR_HIP, "hipStreamCreate: %s", hipGetErrorString(hipGetLastError()));
  while ((int)plan->sync_pool.size() < plan->sync_needed) {
    hipEvent_t e;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess)
      return fail(AC_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(hipGetLastError()));
    plan->sync_pool.push_back(e);
  }
  plan->wptr.assign(dev_ptrs, dev_ptrs + n_ptrs);
  plan->bound = true;
  return AC_OK;
}

int ac_execute(ac_plan* plan, const void* x_dev, void* y_dev, void* workspace_dev, uint64_t workspace_bytes,
               void* stream, uint64_t* measured_peak_bytes) {
  if (!plan || !x_dev || !y_dev) return fail(AC_ERR_ARG, "ac_execute: null argument");
  if (!plan->bound) return fail(AC_ERR_STATE, "weights are not bound");
  if (workspace_bytes < plan->info.workspace_bytes || (plan->info.workspace_bytes > 0 && !workspace_dev))
    return fail(AC_ERR_WORKSPACE, "workspace has %llu bytes, plan needs %llu", (unsigned long long)workspace_bytes,
                (unsigned long long)plan->info.workspace_bytes);
  if (!aligned256(x_dev) || !aligned256(y_dev) || !aligned256(workspace_dev))
    return fail(AC_ERR_ALIGN, "x, y and workspace must be 256-byte aligned");
  const uint64_t half = plan->info.io_bytes / 2;
  const uint8_t* xb = (const uint8_t*)x_dev;
  const uint8_t* yb = (const uint8_t*)y_dev;
  if (xb < yb + half && yb < xb + half) return fail(AC_ERR_ARG, "x and y overlap");
  Walk wk{plan, false, false, (hipStream_t)stream};
  wk.arena.base = (uint8_t*)workspace_dev;
  wk.lane_stream[0] = (hipStream_t)stream;
  if (plan->m.flags & AC_FLAG_TWO_SEGMENTS_IN_FLIGHT) {
    if (!plan->aux_stream) return fail(AC_ERR_STATE, "the plan's second stream does not exist");
    wk.lanes = 2;
    wk.lane_stream[1] = plan->aux_stream;
    plan->sync_used = 0;
  }
  if (plan->m.workload == AC_TRANSFORMER_STACK) wk.transformer(x_dev, y_dev);
  else if (plan->m.workload == AC_UNET_RES_STACK) wk.res_stack(x_dev, y_dev);
  else wk.pair(x_dev, y_dev);
  if (measured_peak_bytes) *measured_peak_bytes = plan->info.io_bytes + wk.arena.high;
  if (!wk.ok()) return fail(AC_ERR_HIP, "%s: %s", wk.err_where, hipGetErrorString(wk.err));
  return AC_OK;
}

void ac_plan_destroy(ac_plan* plan) {
  if (!plan) return;
  for (hipEvent_t e : plan->pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : plan->sync_pool) (void)hipEventDestroy(e);
  if (plan->aux_stream) (void)hipStreamDestroy(plan->aux_stream);
  delete plan;
}

int ac_plan_set_profiling(ac_plan* plan, int enabled) {
  if (!plan) return fail(AC_ERR_ARG, "ac_plan_set_profiling: null plan");
  plan->profiling = enabled != 0;
  plan->recs.clear();
  plan->pool_used = 0;
  return AC_OK;
}

int ac_plan_read_profile(ac_plan* plan, ac_kernel_stat* out, int max_stats, int* n_out) {
  if (!plan || !out || !n_out || max_stats < 1) return fail(AC_ERR_ARG, "ac_plan_read_profile: bad argument");
  if (!plan->profiling) return fail(AC_ERR_STATE, "profiling is not enabled");
  ac_kernel_stat acc[K_CLASSES];
  memset(acc, 0, sizeof(acc));
  for (int c = 0; c < K_CLASSES; ++c) snprintf(acc[c].name, sizeof(acc[c].name), "%s", kClassName[c]);
  for (const ProfRec& r : plan->recs) {
    hipError_t e = hipEventSynchronize(r.stop);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e != hipSuccess) return fail(AC_ERR_HIP, "event timing: %s", hipGetErrorString(e));
    acc[r.cls].launches += 1;
    acc[r.cls].total_ms += ms;
    acc[r.cls].flops += r.flops;
    acc[r.cls].bytes += r.bytes;
  }
  int n = 0;
  for (int c = 0; c < K_CLASSES && n < max_stats; ++c)
    if (acc[c].launches > 0) out[n++] = acc[c];
  *n_out = n;
  plan->recs.clear();
  plan->pool_used = 0;
  return AC_OK;
}

// ---- single kernels ---------------------------------------------------------------------

static int hip_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return AC_OK;
  if (e == hipErrorNotSupported) return fail(AC_ERR_UNSUPPORTED, "%s: no kernel covers this shape", what);
  return fail(AC_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}
static bool dtype_ok(int dt) { return dt == AC_F32 || dt == AC_BF16; }

int ac_op_layernorm(const void* x, int64_t ldx, const void* gain, const void* shift, void* y, int64_t ldy,
                    int64_t rows, int64_t cols, float eps, int dtype, void* stream) {
  if (!x || !gain || !shift || !y || rows < 0 || cols < 1 || ldx < cols || ldy < cols || !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_layernorm: bad argument");
  return hip_status(launch_layernorm(x, ldx, gain, shift, y, ldy, rows, cols, eps, dtype, (hipStream_t)stream),
                    "layernorm");
}

int ac_op_ln_linear(const void* x, int64_t ldx, const void* gain, const void* shift, float eps, int64_t rows,
                    int64_t k, const ac_proj_part* parts, int n_parts, int dtype, void* stream) {
  if (!x || !gain || !shift || !parts || rows < 0 || k < 1 || ldx < k || n_parts < 1 || !(eps > 0.f) || !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_ln_linear: bad argument");
  if (n_parts > kMaxProjParts) return fail(AC_ERR_UNSUPPORTED, "ac_op_ln_linear: at most %d parts", kMaxProjParts);
  LnProjArgs a{};
  a.x = x; a.ldx = ldx; a.gain = gain; a.shift = shift; a.eps = eps; a.rows = rows; a.k = k; a.n_parts = n_parts;
  int64_t ns[kMaxProjParts];
  for (int i = 0; i < n_parts; ++i) {
    const ac_proj_part& s = parts[i];
    if (!s.w || s.n < 1 || (s.gated && !s.w_gate) || (!s.out && !s.out_t) || s.activation < 0 ||
        s.activation > AC_ACT_SIGMOID || (s.out && !s.out_t && s.o_period <= 0 && s.ldo < s.n))
      return fail(AC_ERR_ARG, "ac_op_ln_linear: bad part %d", i);
    ProjPart& d = a.part[i];
    d.w = s.w; d.bias = s.bias; d.w_gate = s.w_gate; d.bias_gate = s.bias_gate; d.gated = s.gated != 0;
    d.act = s.activation; d.n = s.n; d.out = s.out; d.ldo = s.ldo; d.o_period = s.o_period; d.o_s1 = s.o_s1;
    d.o_s2 = s.o_s2; d.out_t = s.out_t; d.t_period = s.t_period; d.t_s1 = s.t_s1; d.t_s2 = s.t_s2; d.t_s3 = s.t_s3;
    ns[i] = s.n;
  }
  if (!ln_proj_shapes_ok(dtype, k, ns, n_parts))
    return fail(AC_ERR_UNSUPPORTED, "ac_op_ln_linear: bf16, k = 64 or 128 and n %% 4 == 0 only");
  return hip_status(launch_ln_proj(a, (hipStream_t)stream), "ln_linear");
}

int ac_op_linear(const void* a, int64_t lda, const void* w, int64_t ldw, const void* bias, const void* mul,
                 int64_t ldmul, const void* residual, int64_t ldr, void* out, int64_t ldo, void* out_t,
                 int64_t n_split, int64_t t_period, int64_t t_s1, int64_t t_s2, int64_t t_s3, int64_t m,
                 int64_t n, int64_t k, int activation, int dtype, void* stream) {
  if (!a || !w || m < 0 || n < 0 || k < 1 || lda < k || ldw < k || !dtype_ok(dtype) || activation < 0 ||
      activation > AC_ACT_SIGMOID)
    return fail(AC_ERR_ARG, "ac_op_linear: bad argument");
  if (!out_t) n_split = n;
  if (n_split < 0 || n_split > n || (n_split > 0 && (!out || ldo < n_split)))
    return fail(AC_ERR_ARG, "ac_op_linear: bad output description");
  LinearArgs g{};
  g.a = a; g.lda = lda; g.w = w; g.ldw = ldw; g.bias = bias; g.mul = mul; g.ldmul = ldmul;
  g.resid = residual; g.ldr = ldr; g.out = out; g.ldo = ldo; g.out_t = out_t; g.n_split = n_split;
  g.t_period = t_period; g.t_s1 = t_s1; g.t_s2 = t_s2; g.t_s3 = t_s3; g.m = m; g.n = n; g.k = k;
  g.act = activation; g.dtype = dtype;
  return hip_status(launch_linear(g, (hipStream_t)stream), "linear");
}

int ac_op_attention(const void* q, int64_t ldq, int64_t stride_q_batch, const void* k, int64_t ldk,
                    int64_t stride_k_batch, const void* v, int64_t ldv, int64_t stride_v_batch, int v_transposed,
                    const void* bias, int64_t ld_bias, int64_t stride_bias_head, const void* gate, int64_t ldg,
                    int64_t stride_g_batch, void* ctx, int64_t ldc, int64_t stride_c_batch, int64_t batch,
                    int64_t sq, int64_t sk, int heads, int head_dim, int causal, int64_t q_offset, int n_splits,
                    void* split_workspace, uint64_t split_workspace_bytes, int dtype, void* stream) {
  if (!q || !k || !v || !ctx || batch < 0 || sq < 0 || sk < 1 || heads < 1 || head_dim < 1 || q_offset < 0 ||
      !dtype_ok(dtype) || n_splits < 0 || n_splits > 16)
    return fail(AC_ERR_ARG, "ac_op_attention: bad argument");
  if (n_splits > 1) {
    const uint64_t need = attention_split_workspace_bytes(sq, heads, batch, head_dim, n_splits);
    if (!split_workspace || split_workspace_bytes < need)
      return fail(AC_ERR_WORKSPACE, "ac_op_attention: %d key splits need %llu workspace bytes", n_splits,
                  (unsigned long long)need);
    if (((uintptr_t)split_workspace & 15u) != 0) return fail(AC_ERR_ALIGN, "split workspace must be 16-byte aligned");
  }
  AttnArgs a{};
  a.q = q; a.ldq = ldq; a.sq_b = stride_q_batch; a.k = k; a.ldk = ldk; a.sk_b = stride_k_batch;
  a.v = v; a.ldv = ldv; a.sv_b = stride_v_batch; a.v_transposed = v_transposed != 0;
  a.bias = bias; a.ld_bias = ld_bias; a.s_bias_h = stride_bias_head;
  a.gate = gate; a.ldg = ldg; a.sg_b = stride_g_batch; a.ctx = ctx; a.ldc = ldc; a.sc_b = stride_c_batch;
  a.batch = batch; a.sq = sq; a.sk = sk; a.heads = heads; a.head_dim = head_dim; a.causal = causal != 0;
  a.q_offset = q_offset; a.dtype = dtype;
  if (n_splits > 1) {
    a.n_splits = n_splits;
    a.part_o = split_workspace;
    a.part_ml = (uint8_t*)split_workspace + (uint64_t)n_splits * batch * sq * heads * head_dim * 4;
  }
  return hip_status(launch_attention(a, (hipStream_t)stream), "attention");
}

// ---- attention whose key-split partials live in a static device array ----------------------
// For callers that cannot allocate.  `scratch` is a file-scope device array: its name is only a
// host-side stand-in here, so its device address is asked for once per device (with that device
// current) and only that address is ever handed to kernels.
namespace {
constexpr uint64_t kStaticScratchBytes = 64ull << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_addr[kMaxDevices];   // per device: the address of that device's copy of `scratch`
std::mutex g_scratch_mu;

int static_scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(AC_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(AC_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_addr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(AC_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_addr[dev] = ptr;
  }
  *out = g_scratch_addr[dev];
  return AC_OK;
}
}  // namespace

uint64_t ac_static_scratch_bytes(void) { return kStaticScratchBytes; }

int ac_op_attention_static_scratch(const void* q, int64_t ldq, int64_t stride_q_batch, const void* k, int64_t ldk,
                                   int64_t stride_k_batch, const void* v, int64_t ldv, int64_t stride_v_batch,
                                   int v_transposed, const void* bias, int64_t ld_bias, int64_t stride_bias_head,
                                   const void* gate, int64_t ldg, int64_t stride_g_batch, void* ctx, int64_t ldc,
                                   int64_t stride_c_batch, int64_t batch, int64_t sq, int64_t sk, int heads,
                                   int head_dim, int causal, int64_t q_offset, int n_splits, int dtype, void* stream) {
  if (!q || !k || !v || !ctx || batch < 0 || sq < 0 || sk < 1 || heads < 1 || head_dim < 1 || q_offset < 0 ||
      !dtype_ok(dtype) || n_splits < 0 || n_splits > 16)
    return fail(AC_ERR_ARG, "ac_op_attention_static_scratch: bad argument");
  if (n_splits == 0) n_splits = attention_key_splits(sq, sk, heads, batch, head_dim, dtype, v_transposed != 0);
  AttnArgs a{};
  a.q = q; a.ldq = ldq; a.sq_b = stride_q_batch; a.k = k; a.ldk = ldk; a.sk_b = stride_k_batch;
  a.v = v; a.ldv = ldv; a.sv_b = stride_v_batch; a.v_transposed = v_transposed != 0;
  a.bias = bias; a.ld_bias = ld_bias; a.s_bias_h = stride_bias_head;
  a.gate = gate; a.ldg = ldg; a.sg_b = stride_g_batch; a.ctx = ctx; a.ldc = ldc; a.sc_b = stride_c_batch;
  a.batch = batch; a.sq = sq; a.sk = sk; a.heads = heads; a.head_dim = head_dim; a.causal = causal != 0;
  a.q_offset = q_offset; a.dtype = dtype;
  if (n_splits > 1) {
    const uint64_t need = attention_split_workspace_bytes(sq, heads, batch, head_dim, n_splits);
    if (need > kStaticScratchBytes)
      return fail(AC_ERR_WORKSPACE,
                  "ac_op_attention_static_scratch: %d key splits of this launch need %llu bytes of partial results; "
                  "the static scratch holds %llu (use fewer splits or fewer query rows, or ac_op_attention)",
                  n_splits, (unsigned long long)need, (unsigned long long)kStaticScratchBytes);
    void* base = nullptr;
    const int st = static_scratch_of_current_device(&base);
    if (st != AC_OK) return st;
    // every element of the partial results that the merge reads is written by the attention
    // kernel of this call first, so nothing of the array has to be cleared between calls
    a.n_splits = n_splits;
    a.part_o = base;
    a.part_ml = (uint8_t*)base + (uint64_t)n_splits * batch * sq * heads * head_dim * 4;
  }
  return hip_status(launch_attention(a, (hipStream_t)stream), "attention");
}

int ac_attention_key_splits(int64_t sq, int64_t sk, int heads, int64_t batch, int head_dim, int dtype,
                            int v_transposed) {
  return attention_key_splits(sq, sk, heads, batch, head_dim, dtype, v_transposed);
}

uint64_t ac_attention_split_workspace_bytes(int64_t sq, int heads, int64_t batch, int head_dim, int n_splits) {
  return attention_split_workspace_bytes(sq, heads, batch, head_dim, n_splits);
}

int ac_op_bias_act(const void* x, int64_t ldx, const void* bias, void* y, int64_t ldy, int64_t rows, int64_t cols,
                   int activation, int dtype, void* stream) {
  if (!x || !y || rows < 0 || cols < 1 || ldx < cols || ldy < cols || !dtype_ok(dtype) || activation < 0 ||
      activation > AC_ACT_SIGMOID)
    return fail(AC_ERR_ARG, "ac_op_bias_act: bad argument");
  return hip_status(launch_bias_act(x, ldx, bias, y, ldy, rows, cols, activation, dtype, (hipStream_t)stream),
                    "bias_act");
}

int ac_op_binary(const void* a, int64_t lda, const void* b, int64_t ldb, void* y, int64_t ldy, int64_t rows,
                 int64_t cols, int op, int dtype, void* stream) {
  if (!a || !b || !y || rows < 0 || cols < 1 || lda < cols || ldb < cols || ldy < cols || !dtype_ok(dtype) ||
      (op != 0 && op != 1))
    return fail(AC_ERR_ARG, "ac_op_binary: bad argument");
  return hip_status(launch_binary(a, lda, b, ldb, y, ldy, rows, cols, op, dtype, (hipStream_t)stream), "binary");
}

int ac_op_softmax_rows(const void* s, int64_t lds, void* p, int64_t ldp, int64_t rows, int64_t cols, float scale,
                       int causal, int64_t q_offset, int64_t period, int dtype, void* stream) {
  if (!s || !p || rows < 0 || cols < 1 || lds < cols || ldp < cols || !(scale > 0.f) || q_offset < 0 || period < 1 ||
      !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_softmax_rows: bad argument");
  return hip_status(launch_softmax_rows(s, lds, p, ldp, rows, cols, scale, causal != 0, q_offset, period, dtype,
                                        (hipStream_t)stream), "softmax_rows");
}

int ac_op_transpose(const void* src, int64_t lds, void* dst, int64_t ldd, int64_t rows, int64_t cols, int dtype,
                    void* stream) {
  if (!src || !dst || rows < 0 || cols < 0 || lds < cols || ldd < rows || !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_transpose: bad argument");
  return hip_status(launch_transpose(src, lds, dst, ldd, rows, cols, dtype, (hipStream_t)stream), "transpose");
}

int ac_op_triangle_contract(const void* a_t, int64_t lda, int64_t stride_a_c, const void* b_t, int64_t ldb,
                            int64_t stride_b_c, void* out_c, int64_t ldo, int64_t stride_o_c, int64_t ni,
                            int64_t nj, int64_t nk, int channels, int dtype, void* stream) {
  if (!a_t || !b_t || !out_c || ni < 0 || nj < 0 || nk < 1 || channels < 1 || lda < nk || ldb < nk || ldo < nj ||
      !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_triangle_contract: bad argument");
  LinearArgs g{};
  g.a = a_t; g.lda = lda; g.sa_b = stride_a_c; g.w = b_t; g.ldw = ldb; g.sw_b = stride_b_c; g.out = out_c;
  g.ldo = ldo; g.so_b = stride_o_c; g.m = ni; g.n = nj; g.k = nk; g.n_split = nj; g.batch = channels;
  g.dtype = dtype;
  return hip_status(launch_linear(g, (hipStream_t)stream), "triangle_contract");
}

int ac_op_transpose_square_inplace(void* data, int64_t ld, int64_t stride_batch, int64_t n, int64_t batch, int dtype,
                                   void* stream) {
  if (!data || n < 0 || batch < 0 || ld < n || !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_transpose_square_inplace: bad argument");
  return hip_status(launch_transpose_square_inplace(data, ld, stride_batch, n, batch, dtype, (hipStream_t)stream),
                    "transpose_square_inplace");
}

int ac_op_layernorm_channel_major(const void* src, int64_t stride_c, const void* gain, const void* shift, void* dst,
                                  int64_t ldd, int64_t positions, int64_t channels, float eps, int dtype,
                                  void* stream) {
  if (!src || !gain || !shift || !dst || positions < 0 || channels < 1 || stride_c < positions || ldd < channels ||
      !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_layernorm_channel_major: bad argument");
  return hip_status(launch_layernorm_channel_major(src, stride_c, gain, shift, dst, ldd, positions, channels, eps,
                                                   dtype, (hipStream_t)stream),
                    "layernorm_channel_major");
}

uint64_t ac_group_norm_workspace_bytes(int64_t images, int groups) {
  return images > 0 && groups > 0 ? group_norm_workspace_bytes(images, groups) : 0;
}

int ac_op_group_norm(const void* x, const void* gain, const void* shift, void* y, void* workspace, uint64_t workspace_bytes,
                     int64_t images, int64_t positions, int channels, int groups, float eps, int activation, int dtype,
                     void* stream) {
  if (!x || !gain || !shift || !y || images < 0 || positions < 0 || channels < 1 || groups < 1 || groups > 128 ||
      channels % groups != 0 || channels % (dtype == AC_BF16 ? 8 : 4) != 0 || images > 65535 || !dtype_ok(dtype) ||
      (activation != AC_ACT_NONE && activation != AC_ACT_SILU) || !(eps > 0.f))
    return fail(AC_ERR_ARG, "ac_op_group_norm: bad argument");
  if (!workspace || workspace_bytes < group_norm_workspace_bytes(images, groups))
    return fail(AC_ERR_WORKSPACE, "ac_op_group_norm: workspace of %llu bytes, %llu needed", (unsigned long long)workspace_bytes,
                (unsigned long long)group_norm_workspace_bytes(images, groups));
  return hip_status(launch_group_norm(x, gain, shift, y, workspace, images, positions, channels, groups, eps, activation, dtype,
                                      (hipStream_t)stream), "group_norm");
}

int ac_op_conv3x3(const void* x, const void* weight, const void* bias, int bias_per_image, const void* residual, void* out,
                  int64_t images, int height, int width, int c_in, int c_out, int dtype, void* stream) {
  if (!x || !weight || !out || images < 0 || height < 1 || width < 1 || c_in < 1 || c_out < 1 || !dtype_ok(dtype))
    return fail(AC_ERR_ARG, "ac_op_conv3x3: bad argument");
  if (dtype != AC_BF16 || c_in % 64 != 0 || c_out % 8 != 0 || images * height * width >= (1ll << 31))
    return fail(AC_ERR_UNSUPPORTED, "ac_op_conv3x3: bf16 images with c_in a multiple of 64, c_out of 8 and fewer than 2^31 pixels");
  if (images == 0) return AC_OK;
  LinearArgs g{};
  g.a = x; g.lda = c_in; g.w = weight; g.ldw = 9 * (int64_t)c_in; g.bias = bias;
  g.bias_period = bias && bias_per_image ? (int64_t)height * width : 0;
  g.resid = residual; g.ldr = c_out; g.out = out; g.ldo = c_out; g.m = images * height * width; g.n = c_out;
  g.k = 9 * (int64_t)c_in; g.n_split = c_out; g.conv_h = height; g.conv_w = width; g.conv_c = c_in; g.dtype = dtype;
  return hip_status(launch_linear(g, (hipStream_t)stream), "conv3x3");
}

}  // extern "C"
