// Shared device helpers and the internal launch interface of the kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/autochunk_rt.h"

namespace ac {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf2f(bf16_t v) { return static_cast<float>(v); }
__device__ __forceinline__ bf16_t f2bf(float v) { return static_cast<bf16_t>(v); }  // nearest-even

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;  // elements per 16-byte access
  __device__ static __forceinline__ float ld(const float* p) { return *p; }
  __device__ static __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
  __device__ static __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }
};

// 16-byte vector load / store of kVec elements, widened to fp32.
__device__ __forceinline__ void load_vec(const float* p, float (&v)[4]) {
  f32x4 t = *reinterpret_cast<const f32x4*>(p);
  v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
__device__ __forceinline__ void load_vec(const bf16_t* p, float (&v)[8]) {
  bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = bf2f(t[i]);
}
__device__ __forceinline__ void store_vec(float* p, const float (&v)[4]) {
  f32x4 t = {v[0], v[1], v[2], v[3]};
  *reinterpret_cast<f32x4*>(p) = t;
}
__device__ __forceinline__ void store_vec(bf16_t* p, const float (&v)[8]) {
  bf16x8 t;
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = f2bf(v[i]);
  *reinterpret_cast<bf16x8*>(p) = t;
}

// erf by the rational-exponential form of Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7):
// two quarter-rate ops (reciprocal, exp2) and a degree-5 Horner chain, about half the
// instructions of the library erff, which matters in a GEMM epilogue run on every element.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  p *= t;
  const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);
  return copysignf(fmaf(-p, e, 1.0f), x);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erf_as(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_tanh(float x) {
  float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
  return 0.5f * x * (1.0f + tanhf(u));
}
__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + __expf(-x)); }

template <int ACT> __device__ __forceinline__ float apply_act(float x) {
  if (ACT == AC_ACT_GELU_ERF) return gelu_erf(x);
  if (ACT == AC_ACT_GELU_TANH) return gelu_tanh(x);
  if (ACT == AC_ACT_RELU) return fmaxf(x, 0.0f);
  if (ACT == AC_ACT_SIGMOID) return sigmoidf(x);
  if (ACT == AC_ACT_SILU) return x * sigmoidf(x);
  return x;
}
__device__ __forceinline__ float apply_act_rt(float x, int act) {
  switch (act) {
    case AC_ACT_GELU_ERF: return gelu_erf(x);
    case AC_ACT_GELU_TANH: return gelu_tanh(x);
    case AC_ACT_RELU: return fmaxf(x, 0.0f);
    case AC_ACT_SIGMOID: return sigmoidf(x);
    case AC_ACT_SILU: return x * sigmoidf(x);
    default: return x;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over groups of G consecutive lanes (G a power of two <= 64).
template <int G> __device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ---------------------------------------------------------------------------------------
// Launch interface used by the executor and by the ac_op_* entry points.
// ---------------------------------------------------------------------------------------

struct LinearArgs {
  const void* a; int64_t lda;        // [m, k]
  const void* w; int64_t ldw;        // [n, k]
  const void* bias;                  // [n] or null
  const void* mul; int64_t ldmul;    // [m, n] or null
  const void* resid; int64_t ldr;    // [m, n] or null
  void* out; int64_t ldo;            // columns [0, n_split): out[m * ldo + n], or, with o_period > 0,
                                     // out[(m / o_period) * o_s1 + (m % o_period) * o_s2 + n]: rows regrouped
                                     // on the way out (e.g. positions (k, j) of a pair tensor stored as (j, k))
  int64_t o_period, o_s1, o_s2;
  // columns [n_split, n): out_t[(m / t_period) * t_s1 + (m % t_period) * t_s2 + (n - n_split) * t_s3]
  void* out_t; int64_t n_split; int64_t t_period, t_s1, t_s2, t_s3;
  int64_t m, n, k;
  int act;
  int dtype;
  // batch > 1: `batch` independent products; a, w and out advance by these strides (elements).
  // bias / mul / resid / out_t must be null then.
  int64_t batch, sa_b, sw_b, so_b;
  // batch > 1: nonzero = blocks take the products last to first.  Results are the same; a caller that runs
  // the same operands launch after launch alternates the direction so that each launch starts with the
  // products whose operands the one before touched last (they are the ones still in the memory-side cache).
  int batch_descending;
  // conv_c > 0: a is a stack of channels-last images [m / (conv_h * conv_w)][conv_h][conv_w][conv_c] and the
  // product is their 3x3 convolution (stride 1, zero padding 1): row m is a pixel, k = 9 * conv_c runs over
  // (window row, window column, input channel), w is [n][3][3][conv_c].  lda is ignored (= conv_c).
  int conv_h, conv_w, conv_c;
  // bias_period > 0: row m takes bias row m / bias_period (bias is [m / bias_period][n]): one bias vector per image
  int64_t bias_period;
};

struct AttnArgs {
  const void* q; int64_t ldq, sq_b;
  const void* k; int64_t ldk, sk_b;
  // v_transposed: v is vt[(h * head_dim + d) * ldv + key]; else row-major v[key * ldv + h * head_dim + d].
  const void* v; int64_t ldv, sv_b; int v_transposed;
  const void* bias; int64_t ld_bias, s_bias_h;   // bias[h * s_bias_h + (row) * ld_bias + key]
  const void* gate; int64_t ldg, sg_b;
  void* ctx; int64_t ldc, sc_b;
  int64_t batch, sq, sk;
  int heads, head_dim, causal;
  int64_t q_offset;
  int dtype;
  // n_splits > 1: the keys each query block sees are cut into n_splits runs handled by
  // separate blocks; partial results go to part_o [split][b][row][head][d] (fp32) and
  // part_ml [split][b][row][head][2] (running max, sum) and are merged by a second kernel.
  int n_splits;
  void* part_o;
  void* part_ml;
  int head_major;   // block order (head, problem, query block) instead of (problem, head, query block); set by launch_attention
};

// LayerNorm of short rows followed by several projections of the normalised rows, in one
// kernel: t = LN(x) stays on chip and every part computes act(t w^T + bias) or, for a gated
// pair, sigmoid(t w_gate^T + bias_gate) * (t w^T + bias), each with its own output layout.
constexpr int kMaxProjParts = 5;
constexpr int kMaxProjTiles = 48;
struct ProjPart {
  const void* w; const void* bias;             // [n, K], [n] or null
  const void* w_gate; const void* bias_gate;   // of a gated pair
  int gated;                                   // 1: out = sigmoid(t w_gate^T + bias_gate) * (t w^T + bias)
  int act;                                     // of a plain part
  int64_t n;
  void* out; int64_t ldo, o_period, o_s1, o_s2;            // row-major store (rows regrouped if o_period > 0), or
  void* out_t; int64_t t_period, t_s1, t_s2, t_s3;          // strided store of the whole part (see LinearArgs)
};
struct LnProjArgs {
  const void* x; int64_t ldx;      // [rows, K]
  const void* gain; const void* shift; float eps;
  int64_t rows; int64_t k;
  int n_parts;
  ProjPart part[kMaxProjParts];
};
// Shapes the kernel covers (bf16, K = 64 or 128, every n a multiple of 4); a pure function of the
// shapes so that planning and execution take the same path.
bool ln_proj_shapes_ok(int dtype, int64_t k, const int64_t* n, int n_parts);
hipError_t launch_ln_proj(const LnProjArgs& p, hipStream_t s);

hipError_t launch_layernorm(const void* x, int64_t ldx, const void* gain, const void* shift, void* y,
                            int64_t ldy, int64_t rows, int64_t cols, float eps, int dtype,
                            hipStream_t s);
hipError_t launch_bias_act(const void* x, int64_t ldx, const void* bias, void* y, int64_t ldy,
                           int64_t rows, int64_t cols, int act, int dtype, hipStream_t s);
hipError_t launch_binary(const void* a, int64_t lda, const void* b, int64_t ldb, void* y, int64_t ldy,
                         int64_t rows, int64_t cols, int op, int dtype, hipStream_t s);
hipError_t launch_linear(const LinearArgs& g, hipStream_t s);
// GroupNorm (+ SiLU) of channels-last images [images, positions, channels]; partials: group_norm_workspace_bytes()
uint64_t group_norm_workspace_bytes(int64_t images, int groups);
hipError_t launch_group_norm(const void* x, const void* gain, const void* shift, void* y, void* partials, int64_t images,
                             int64_t positions, int channels, int groups, float eps, int act, int dtype, hipStream_t s);
// p = softmax(scale * s [causal]) over stored rows; row r is query r mod period at position
// q_offset + (r mod period).
hipError_t launch_softmax_rows(const void* src, int64_t lds, void* dst, int64_t ldd, int64_t rows, int64_t cols,
                               float scale, int causal, int64_t q_offset, int64_t period, int dtype, hipStream_t s);
hipError_t launch_attention(const AttnArgs& a, hipStream_t s);
int attention_key_splits(int64_t sq, int64_t sk, int heads, int64_t batch, int head_dim, int dtype, int v_transposed);
uint64_t attention_split_workspace_bytes(int64_t sq, int heads, int64_t batch, int head_dim, int n_splits);
// Row-major value matrix [keys, cols] -> transposed copy [cols, keys] (bf16), for callers
// of the attention entry point that hold v row-major.
hipError_t launch_transpose(const void* src, int64_t lds, void* dst, int64_t ldd, int64_t rows,
                            int64_t cols, int dtype, hipStream_t s);
// In-place transpose of `batch` square [n, n] matrices (row stride ld, `stride_b` apart).
hipError_t launch_transpose_square_inplace(void* data, int64_t ld, int64_t stride_b, int64_t n,
                                           int64_t batch, int dtype, hipStream_t s);
// dst[jj][i][:] = z[i][j0 + jj][:] for a pair tensor z[n][n][c] (the copy behind a column chunk).
hipError_t launch_gather_columns(const void* src, void* dst, int64_t n, int64_t c, int64_t j0, int64_t nj, int dtype,
                                 hipStream_t s);
// LayerNorm over channels of a channel-major tensor: src[c * stride_c + p] -> dst[p * ldd + c].
hipError_t launch_layernorm_channel_major(const void* src, int64_t stride_c, const void* gain,
                                          const void* shift, void* dst, int64_t ldd, int64_t positions,
                                          int64_t channels, float eps, int dtype, hipStream_t s);

// hipErrorInvalidValue-style refusal with a message for ac_last_error().
void set_error(const char* fmt, ...);

}  // namespace ac
