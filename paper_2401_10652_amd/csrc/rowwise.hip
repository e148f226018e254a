// Row-wise HBM-bound passes over one segment: LayerNorm, bias + activation, add / multiply,
// and a tiled transpose.  Each element is read once and written once with 16-byte accesses;
// statistics are fp32.  (AutoChunk section 2.2: these are the per-segment elementwise and
// normalisation steps of a chunked region.)
#include "common.h"

namespace ac {

// ------------------------------------------------------------------------------------
// LayerNorm.  A group of G lanes owns one row and keeps it in registers (NV 16-byte
// vectors per lane): mean, then the centred second moment, then the affine output.
// cols == G * NV * kVec exactly; other widths take the generic kernel below.
// ------------------------------------------------------------------------------------
template <typename T, int G, int NV, int RPG>
__global__ void __launch_bounds__(256)
layernorm_rows(const T* __restrict__ x, int64_t ldx, const T* __restrict__ gain,
               const T* __restrict__ shift, T* __restrict__ y, int64_t ldy, int64_t rows, float eps) {
  // RPG rows per group at once: their loads are all issued before the first reduction, so
  // a thread has RPG * NV 16-byte loads in flight (one row of 128 columns alone is too little
  // to cover HBM latency).
  constexpr int V = Elem<T>::kVec;
  constexpr int COLS = G * NV * V;
  constexpr int ROWS_PER_BLOCK = 256 / G * RPG;
  const int lane_in_group = threadIdx.x % G;
  const int64_t row0 = (int64_t)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x / G) * RPG;
  float v[RPG][NV][V];
#pragma unroll
  for (int r = 0; r < RPG; ++r) {
    const int64_t rr = row0 + r < rows ? row0 + r : rows - 1;   // dead rows shadow the last row, store nothing
#pragma unroll
    for (int i = 0; i < NV; ++i) load_vec(x + rr * ldx + (i * G + lane_in_group) * V, v[r][i]);
  }
  float g[NV][V], b[NV][V];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    load_vec(gain + (i * G + lane_in_group) * V, g[i]);
    load_vec(shift + (i * G + lane_in_group) * V, b[i]);
  }
#pragma unroll
  for (int r = 0; r < RPG; ++r) {
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int j = 0; j < V; ++j) sum += v[r][i][j];
    const float mean = group_sum<G>(sum) * (1.0f / COLS);
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int j = 0; j < V; ++j) { float d = v[r][i][j] - mean; sq += d * d; }
    const float rstd = rsqrtf(group_sum<G>(sq) * (1.0f / COLS) + eps);
    if (row0 + r >= rows) continue;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float o[V];
#pragma unroll
      for (int j = 0; j < V; ++j) o[j] = (v[r][i][j] - mean) * rstd * g[i][j] + b[i][j];
      store_vec(y + (row0 + r) * ldy + (i * G + lane_in_group) * V, o);
    }
  }
}

// Any width: one wave per row, three passes over the row (it stays in L2).
template <typename T>
__global__ void __launch_bounds__(256)
layernorm_rows_generic(const T* __restrict__ x, int64_t ldx, const T* __restrict__ gain,
                       const T* __restrict__ shift, T* __restrict__ y, int64_t ldy, int64_t rows,
                       int64_t cols, float eps) {
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
  if (row >= rows) return;
  const T* xr = x + row * ldx;
  float sum = 0.f;
  for (int64_t c = lane; c < cols; c += kWave) sum += Elem<T>::ld(xr + c);
  const float mean = wave_sum(sum) / (float)cols;
  float sq = 0.f;
  for (int64_t c = lane; c < cols; c += kWave) { float d = Elem<T>::ld(xr + c) - mean; sq += d * d; }
  const float rstd = rsqrtf(wave_sum(sq) / (float)cols + eps);
  for (int64_t c = lane; c < cols; c += kWave)
    Elem<T>::st(y + row * ldy + c,
                (Elem<T>::ld(xr + c) - mean) * rstd * Elem<T>::ld(gain + c) + Elem<T>::ld(shift + c));
}

template <typename T, int G, int NV>
static hipError_t ln_launch(const void* x, int64_t ldx, const void* g, const void* b, void* y, int64_t ldy,
                            int64_t rows, float eps, hipStream_t s) {
  constexpr int RPG = NV >= 4 ? 1 : (NV >= 2 ? 2 : 4);   // about four vector loads in flight per thread
  const int rpb = 256 / G * RPG;
  dim3 grid((unsigned)((rows + rpb - 1) / rpb));
  hipLaunchKernelGGL((layernorm_rows<T, G, NV, RPG>), grid, dim3(256), 0, s, (const T*)x, ldx, (const T*)g,
                     (const T*)b, (T*)y, ldy, rows, eps);
  return hipGetLastError();
}

template <typename T>
static hipError_t ln_dispatch(const void* x, int64_t ldx, const void* g, const void* b, void* y, int64_t ldy,
                              int64_t rows, int64_t cols, float eps, hipStream_t s) {
  constexpr int V = Elem<T>::kVec;
  const bool vec_ok = (ldx % V == 0) && (ldy % V == 0) && (cols % V == 0);
  if (vec_ok) {
    const int64_t nvec = cols / V;   // 16-byte vectors per row
    switch (nvec) {
      case 8:   return ln_launch<T, 8, 1>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 16:  return ln_launch<T, 16, 1>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 32:  return ln_launch<T, 32, 1>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 64:  return ln_launch<T, 64, 1>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 40:  return ln_launch<T, 8, 5>(x, ldx, g, b, y, ldy, rows, eps, s);     // 320 bf16 channels (UNet stages:
      case 80:  return ln_launch<T, 16, 5>(x, ldx, g, b, y, ldy, rows, eps, s);    //  320, 640, 1280)
      case 96:  return ln_launch<T, 32, 3>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 160: return ln_launch<T, 32, 5>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 128: return ln_launch<T, 64, 2>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 192: return ln_launch<T, 64, 3>(x, ldx, g, b, y, ldy, rows, eps, s);
      case 256: return ln_launch<T, 64, 4>(x, ldx, g, b, y, ldy, rows, eps, s);
      default: break;
    }
  }
  dim3 grid((unsigned)((rows + 3) / 4));
  hipLaunchKernelGGL((layernorm_rows_generic<T>), grid, dim3(256), 0, s, (const T*)x, ldx, (const T*)g,
                     (const T*)b, (T*)y, ldy, rows, cols, eps);
  return hipGetLastError();
}

hipError_t launch_layernorm(const void* x, int64_t ldx, const void* gain, const void* shift, void* y,
                            int64_t ldy, int64_t rows, int64_t cols, float eps, int dtype, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (dtype == AC_BF16) return ln_dispatch<bf16_t>(x, ldx, gain, shift, y, ldy, rows, cols, eps, s);
  return ln_dispatch<float>(x, ldx, gain, shift, y, ldy, rows, cols, eps, s);
}

// ------------------------------------------------------------------------------------
// y = act(x + bias[col]);  y = a (+|*) b.   Grid-stride over 16-byte vectors of a
// [rows, cols] view with row strides; cols % kVec == 0 takes the vector path.
// ------------------------------------------------------------------------------------
// x and y may be the same buffer (the executor applies bias + activation in place), so the
// pointers carry no restrict qualifier.
template <typename T>
__global__ void __launch_bounds__(256)
bias_act_vec(const T* x, int64_t ldx, const T* bias, T* y,
             int64_t ldy, int64_t rows, int64_t vec_per_row, int act) {
  constexpr int V = Elem<T>::kVec;
  const int64_t total = rows * vec_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / vec_per_row, c = (i % vec_per_row) * V;
    float v[V], b[V];
    load_vec(x + r * ldx + c, v);
    if (bias) {
      load_vec(bias + c, b);
#pragma unroll
      for (int j = 0; j < V; ++j) v[j] += b[j];
    }
#pragma unroll
    for (int j = 0; j < V; ++j) v[j] = apply_act_rt(v[j], act);
    store_vec(y + r * ldy + c, v);
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
bias_act_scalar(const T* x, int64_t ldx, const T* bias, T* y,
                int64_t ldy, int64_t rows, int64_t cols, int act) {
  const int64_t total = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols, c = i % cols;
    float v = Elem<T>::ld(x + r * ldx + c);
    if (bias) v += Elem<T>::ld(bias + c);
    Elem<T>::st(y + r * ldy + c, apply_act_rt(v, act));
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
binary_vec(const T* __restrict__ a, int64_t lda, const T* __restrict__ b, int64_t ldb, T* __restrict__ y,
           int64_t ldy, int64_t rows, int64_t vec_per_row, int op) {
  constexpr int V = Elem<T>::kVec;
  const int64_t total = rows * vec_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / vec_per_row, c = (i % vec_per_row) * V;
    float u[V], v[V];
    load_vec(a + r * lda + c, u);
    load_vec(b + r * ldb + c, v);
#pragma unroll
    for (int j = 0; j < V; ++j) u[j] = op == 0 ? u[j] + v[j] : u[j] * v[j];
    store_vec(y + r * ldy + c, u);
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
binary_scalar(const T* __restrict__ a, int64_t lda, const T* __restrict__ b, int64_t ldb, T* __restrict__ y,
              int64_t ldy, int64_t rows, int64_t cols, int op) {
  const int64_t total = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols, c = i % cols;
    const float u = Elem<T>::ld(a + r * lda + c), v = Elem<T>::ld(b + r * ldb + c);
    Elem<T>::st(y + r * ldy + c, op == 0 ? u + v : u * v);
  }
}

static unsigned stream_grid(int64_t items) {
  int64_t blocks = (items + 255) / 256;
  const int64_t cap = 256 * 16;   // 256 CUs, enough waves each to cover HBM latency
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

template <typename T>
static hipError_t bias_act_dispatch(const void* x, int64_t ldx, const void* bias, void* y, int64_t ldy,
                                    int64_t rows, int64_t cols, int act, hipStream_t s) {
  constexpr int V = Elem<T>::kVec;
  if (cols % V == 0 && ldx % V == 0 && ldy % V == 0) {
    const int64_t vpr = cols / V;
    hipLaunchKernelGGL((bias_act_vec<T>), dim3(stream_grid(rows * vpr)), dim3(256), 0, s, (const T*)x, ldx,
                       (const T*)bias, (T*)y, ldy, rows, vpr, act);
  } else {
    hipLaunchKernelGGL((bias_act_scalar<T>), dim3(stream_grid(rows * cols)), dim3(256), 0, s, (const T*)x,
                       ldx, (const T*)bias, (T*)y, ldy, rows, cols, act);
  }
  return hipGetLastError();
}

hipError_t launch_bias_act(const void* x, int64_t ldx, const void* bias, void* y, int64_t ldy, int64_t rows,
                           int64_t cols, int act, int dtype, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (dtype == AC_BF16) return bias_act_dispatch<bf16_t>(x, ldx, bias, y, ldy, rows, cols, act, s);
  return bias_act_dispatch<float>(x, ldx, bias, y, ldy, rows, cols, act, s);
}

template <typename T>
static hipError_t binary_dispatch(const void* a, int64_t lda, const void* b, int64_t ldb, void* y, int64_t ldy,
                                  int64_t rows, int64_t cols, int op, hipStream_t s) {
  constexpr int V = Elem<T>::kVec;
  if (cols % V == 0 && lda % V == 0 && ldb % V == 0 && ldy % V == 0) {
    const int64_t vpr = cols / V;
    hipLaunchKernelGGL((binary_vec<T>), dim3(stream_grid(rows * vpr)), dim3(256), 0, s, (const T*)a, lda,
                       (const T*)b, ldb, (T*)y, ldy, rows, vpr, op);
  } else {
    hipLaunchKernelGGL((binary_scalar<T>), dim3(stream_grid(rows * cols)), dim3(256), 0, s, (const T*)a, lda,
                       (const T*)b, ldb, (T*)y, ldy, rows, cols, op);
  }
  return hipGetLastError();
}

hipError_t launch_binary(const void* a, int64_t lda, const void* b, int64_t ldb, void* y, int64_t ldy,
                         int64_t rows, int64_t cols, int op, int dtype, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (dtype == AC_BF16) return binary_dispatch<bf16_t>(a, lda, b, ldb, y, ldy, rows, cols, op, s);
  return binary_dispatch<float>(a, lda, b, ldb, y, ldy, rows, cols, op, s);
}

// ------------------------------------------------------------------------------------
// dst[c * ldd + r] = src[r * lds + c] through a padded 64x64 LDS tile.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
transpose_tiles(const T* __restrict__ src, int64_t lds_, T* __restrict__ dst, int64_t ldd, int64_t rows,
                int64_t cols) {
  __shared__ T tile[64][65];
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  for (int i = ty; i < 64; i += 4) {
    const int64_t r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = src[r * lds_ + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int64_t c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) dst[c * ldd + r] = tile[tx][i];
  }
}

hipError_t launch_transpose(const void* src, int64_t lds_, void* dst, int64_t ldd, int64_t rows, int64_t cols,
                            int dtype, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
  if (dtype == AC_BF16)
    hipLaunchKernelGGL((transpose_tiles<bf16_t>), grid, dim3(256), 0, s, (const bf16_t*)src, lds_, (bf16_t*)dst,
                       ldd, rows, cols);
  else
    hipLaunchKernelGGL((transpose_tiles<float>), grid, dim3(256), 0, s, (const float*)src, lds_, (float*)dst,
                       ldd, rows, cols);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Columns [j0, j0 + nj) of a pair tensor z[n][n][c], gathered with the two position indices
// swapped: dst[jj][i][:] = z[i][j0 + jj][:].  This is the copy a chunk along the second
// dimension pays for (AutoChunk section 3.4 counts such "continuous operation" copies as
// activation memory and penalises chunk dimensions with a small stride): after it the segment
// is a contiguous block of rows of the transposed tensor.  16-byte accesses; a position's c
// channels are contiguous on both sides.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
gather_columns(const T* src, T* dst, int64_t n, int64_t j0, int64_t nj, int64_t vec_per_pos, int64_t c) {
  constexpr int V = Elem<T>::kVec;
  const int64_t total = n * nj * vec_per_pos;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int64_t v = idx % vec_per_pos, pos = idx / vec_per_pos;
    const int64_t jj = pos % nj, i = pos / nj;            // source order: runs of nj positions are contiguous
    float t[V];
    load_vec(src + ((i * n + j0 + jj) * c + v * V), t);
    store_vec(dst + ((jj * n + i) * c + v * V), t);
  }
}

hipError_t launch_gather_columns(const void* src, void* dst, int64_t n, int64_t c, int64_t j0, int64_t nj, int dtype,
                                 hipStream_t s) {
  if (n <= 0 || nj <= 0 || c <= 0) return hipSuccess;
  const int V = dtype == AC_BF16 ? 8 : 4;
  if (c % V != 0) return hipErrorNotSupported;
  const int64_t items = n * nj * (c / V);
  if (dtype == AC_BF16)
    hipLaunchKernelGGL((gather_columns<bf16_t>), dim3(stream_grid(items)), dim3(256), 0, s, (const bf16_t*)src,
                       (bf16_t*)dst, n, j0, nj, c / V, c);
  else
    hipLaunchKernelGGL((gather_columns<float>), dim3(stream_grid(items)), dim3(256), 0, s, (const float*)src,
                       (float*)dst, n, j0, nj, c / V, c);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// In-place transpose of square matrices, by pairs of 64x64 tiles (bi <= bj): both tiles go
// to LDS, each is written transposed into the other's place.  grid.x enumerates the tile
// pairs of the upper triangle, grid.y the matrices.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
transpose_square_inplace(T* __restrict__ data, int64_t ld, int64_t stride_b, int64_t n, int tiles) {
  __shared__ T ta[64][65];
  __shared__ T tb[64][65];
  // pair index -> (bi, bj), bi <= bj, rows of the upper triangle laid end to end
  int p = blockIdx.x, bi = 0;
  while (p >= tiles - bi) { p -= tiles - bi; ++bi; }
  const int bj = bi + p;
  T* mat = data + (int64_t)blockIdx.y * stride_b;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  const int64_t r0 = (int64_t)bi * 64, c0 = (int64_t)bj * 64;
  for (int i = ty; i < 64; i += 4) {
    if (r0 + i < n && c0 + tx < n) ta[i][tx] = mat[(r0 + i) * ld + c0 + tx];
    if (bi != bj && c0 + i < n && r0 + tx < n) tb[i][tx] = mat[(c0 + i) * ld + r0 + tx];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    // tile (bj, bi) receives ta transposed; tile (bi, bj) receives tb transposed
    if (c0 + i < n && r0 + tx < n) mat[(c0 + i) * ld + r0 + tx] = ta[tx][i];
    if (bi != bj && r0 + i < n && c0 + tx < n) mat[(r0 + i) * ld + c0 + tx] = tb[tx][i];
  }
}

// The same with 16-byte global accesses (n, ld, stride_b multiples of the vector and a 16-byte aligned base):
// a thread moves runs of V elements of a row; the transposition happens in LDS, element by element.
template <typename T>
__global__ void __launch_bounds__(256)
transpose_square_inplace_vec(T* __restrict__ data, int64_t ld, int64_t stride_b, int64_t n, int tiles) {
  constexpr int V = Elem<T>::kVec, CPR = 64 / V;      // 16-byte runs per tile row
  __shared__ float ta[64][65];
  __shared__ float tb[64][65];
  int p = blockIdx.x, bi = 0;
  while (p >= tiles - bi) { p -= tiles - bi; ++bi; }
  const int bj = bi + p;
  T* mat = data + (int64_t)blockIdx.y * stride_b;
  const int64_t r0 = (int64_t)bi * 64, c0 = (int64_t)bj * 64;
  const int tid = threadIdx.x;
  // all loads of the thread first (both tiles), so that they are in flight together
  constexpr int RUNS = 64 * CPR / 256;                // runs per thread and tile: 2 (bf16) or 4 (fp32)
  float va[RUNS][V], vb[RUNS][V];
#pragma unroll
  for (int k = 0; k < RUNS; ++k) {
    const int q = tid + 256 * k, row = q / CPR, col = (q % CPR) * V;
    const bool ina = r0 + row < n && c0 + col < n, inb = bi != bj && c0 + row < n && r0 + col < n;
    load_vec(mat + (ina ? (r0 + row) * ld + c0 + col : 0), va[k]);
    load_vec(mat + (inb ? (c0 + row) * ld + r0 + col : 0), vb[k]);
  }
#pragma unroll
  for (int k = 0; k < RUNS; ++k) {
    const int q = tid + 256 * k, row = q / CPR, col = (q % CPR) * V;
#pragma unroll
    for (int e = 0; e < V; ++e) { ta[col + e][row] = va[k][e]; tb[col + e][row] = vb[k][e]; }   // stored transposed
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < RUNS; ++k) {
    const int q = tid + 256 * k, row = q / CPR, col = (q % CPR) * V;
    float oa[V], ob[V];
#pragma unroll
    for (int e = 0; e < V; ++e) { oa[e] = ta[row][col + e]; ob[e] = tb[row][col + e]; }
    // tile (bj, bi) receives ta transposed; tile (bi, bj) receives tb transposed
    if (c0 + row < n && r0 + col < n) store_vec(mat + (c0 + row) * ld + r0 + col, oa);
    if (bi != bj && r0 + row < n && c0 + col < n) store_vec(mat + (r0 + row) * ld + c0 + col, ob);
  }
}

hipError_t launch_transpose_square_inplace(void* data, int64_t ld, int64_t stride_b, int64_t n, int64_t batch,
                                           int dtype, hipStream_t s) {
  if (n <= 0 || batch <= 0) return hipSuccess;
  if (batch > 65535) return hipErrorInvalidValue;
  const int tiles = (int)((n + 63) / 64);
  dim3 grid((unsigned)(tiles * (tiles + 1) / 2), (unsigned)batch);
  const int64_t vec = dtype == AC_BF16 ? 8 : 4;
  if (n % vec == 0 && ld % vec == 0 && stride_b % vec == 0 && ((uintptr_t)data % 16) == 0) {
    if (dtype == AC_BF16)
      hipLaunchKernelGGL((transpose_square_inplace_vec<bf16_t>), grid, dim3(256), 0, s, (bf16_t*)data, ld, stride_b, n, tiles);
    else
      hipLaunchKernelGGL((transpose_square_inplace_vec<float>), grid, dim3(256), 0, s, (float*)data, ld, stride_b, n, tiles);
    return hipGetLastError();
  }
  if (dtype == AC_BF16)
    hipLaunchKernelGGL((transpose_square_inplace<bf16_t>), grid, dim3(256), 0, s, (bf16_t*)data, ld, stride_b, n, tiles);
  else
    hipLaunchKernelGGL((transpose_square_inplace<float>), grid, dim3(256), 0, s, (float*)data, ld, stride_b, n, tiles);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// LayerNorm over the channels of a channel-major tensor src[c][p], written position-major
// dst[p][c].  A block takes 64 consecutive positions: coalesced reads along p for every
// channel into an LDS tile [64][C], then one 16-lane group per position normalises its row
// and stores it with 16-byte accesses.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
layernorm_channel_major(const T* __restrict__ src, int64_t stride_c, const T* __restrict__ gain,
                        const T* __restrict__ shift, T* __restrict__ dst, int64_t ldd, int64_t positions,
                        int channels, float eps) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* tile = reinterpret_cast<float*>(smem_raw);   // [64][channels + 1]
  const int ldt = channels + 1;
  const int64_t p0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  for (int c = ty; c < channels; c += 4) {
    const int64_t p = p0 + tx;
    tile[tx * ldt + c] = p < positions ? Elem<T>::ld(src + (int64_t)c * stride_c + p) : 0.f;
  }
  __syncthreads();
  // 16 groups of 16 lanes; group g handles positions g, g + 16, g + 32, g + 48
  const int grp = threadIdx.x / 16, lane = threadIdx.x % 16;
  for (int pp = grp; pp < 64; pp += 16) {
    const int64_t p = p0 + pp;
    const float* row = tile + pp * ldt;
    float sum = 0.f;
    for (int c = lane; c < channels; c += 16) sum += row[c];
    const float mean = group_sum<16>(sum) / (float)channels;
    float sq = 0.f;
    for (int c = lane; c < channels; c += 16) { const float d = row[c] - mean; sq += d * d; }
    const float rstd = rsqrtf(group_sum<16>(sq) / (float)channels + eps);
    if (p < positions)
      for (int c = lane; c < channels; c += 16)
        Elem<T>::st(dst + p * ldd + c, (row[c] - mean) * rstd * Elem<T>::ld(gain + c) + Elem<T>::ld(shift + c));
  }
}

// The same with 16-byte global accesses on both sides (positions, stride_c and ldd multiples of the vector,
// channels a multiple of 16 vectors, 16-byte aligned bases): a thread reads runs of V positions of one channel,
// and each of the 16 lanes of a position's group owns channels / 16 consecutive channels.
template <typename T>
__global__ void __launch_bounds__(256)
layernorm_channel_major_vec(const T* __restrict__ src, int64_t stride_c, const T* __restrict__ gain,
                            const T* __restrict__ shift, T* __restrict__ dst, int64_t ldd, int64_t positions,
                            int channels, float eps) {
  constexpr int V = Elem<T>::kVec, PR = 64 / V;        // 16-byte runs of positions per channel and block
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* tile = reinterpret_cast<float*>(smem_raw);   // [64][channels + 1]
  const int ldt = channels + 1;
  const int64_t p0 = (int64_t)blockIdx.x * 64;
  const int tid = threadIdx.x;
  constexpr int B = 4;                                 // runs in flight per thread
  for (int q0 = tid; q0 < channels * PR; q0 += 256 * B) {
    float v[B][V];
#pragma unroll
    for (int k = 0; k < B; ++k) {
      const int q = q0 + 256 * k, c = q / PR, pr = (q % PR) * V;
      const bool in = q < channels * PR && p0 + pr < positions;
      load_vec(src + (in ? (int64_t)c * stride_c + p0 + pr : 0), v[k]);
    }
#pragma unroll
    for (int k = 0; k < B; ++k) {
      const int q = q0 + 256 * k, c = q / PR, pr = (q % PR) * V;
      if (q >= channels * PR) break;
      const bool in = p0 + pr < positions;
#pragma unroll
      for (int e = 0; e < V; ++e) tile[(pr + e) * ldt + c] = in ? v[k][e] : 0.f;
    }
  }
  __syncthreads();
  const int grp = tid / 16, lane = tid % 16;
  const int cpl = channels / 16;                        // consecutive channels per lane (a multiple of V)
  for (int pp = grp; pp < 64; pp += 16) {
    const int64_t p = p0 + pp;
    const float* row = tile + pp * ldt + lane * cpl;
    float sum = 0.f;
    for (int c = 0; c < cpl; ++c) sum += row[c];
    const float mean = group_sum<16>(sum) / (float)channels;
    float sq = 0.f;
    for (int c = 0; c < cpl; ++c) { const float d = row[c] - mean; sq += d * d; }
    const float rstd = rsqrtf(group_sum<16>(sq) / (float)channels + eps);
    if (p < positions)
      for (int c = 0; c < cpl; c += V) {
        float g[V], b[V], o[V];
        load_vec(gain + lane * cpl + c, g);
        load_vec(shift + lane * cpl + c, b);
#pragma unroll
        for (int e = 0; e < V; ++e) o[e] = (row[c + e] - mean) * rstd * g[e] + b[e];
        store_vec(dst + p * ldd + lane * cpl + c, o);
      }
  }
}

hipError_t launch_layernorm_channel_major(const void* src, int64_t stride_c, const void* gain, const void* shift,
                                          void* dst, int64_t ldd, int64_t positions, int64_t channels, float eps,
                                          int dtype, hipStream_t s) {
  if (positions <= 0 || channels <= 0) return hipSuccess;
  const size_t lds = (size_t)64 * (channels + 1) * sizeof(float);
  if (lds > 64 * 1024) return hipErrorNotSupported;
  dim3 grid((unsigned)((positions + 63) / 64));
  const int64_t vec = dtype == AC_BF16 ? 8 : 4;
  auto al16 = [](const void* p) { return ((uintptr_t)p % 16) == 0; };
  if (positions % vec == 0 && stride_c % vec == 0 && ldd % vec == 0 && channels % (16 * vec) == 0 && al16(src) && al16(dst) &&
      al16(gain) && al16(shift)) {
    if (dtype == AC_BF16)
      hipLaunchKernelGGL((layernorm_channel_major_vec<bf16_t>), grid, dim3(256), lds, s, (const bf16_t*)src, stride_c,
                         (const bf16_t*)gain, (const bf16_t*)shift, (bf16_t*)dst, ldd, positions, (int)channels, eps);
    else
      hipLaunchKernelGGL((layernorm_channel_major_vec<float>), grid, dim3(256), lds, s, (const float*)src, stride_c,
                         (const float*)gain, (const float*)shift, (float*)dst, ldd, positions, (int)channels, eps);
    return hipGetLastError();
  }
  if (dtype == AC_BF16)
    hipLaunchKernelGGL((layernorm_channel_major<bf16_t>), grid, dim3(256), lds, s, (const bf16_t*)src, stride_c,
                       (const bf16_t*)gain, (const bf16_t*)shift, (bf16_t*)dst, ldd, positions, (int)channels, eps);
  else
    hipLaunchKernelGGL((layernorm_channel_major<float>), grid, dim3(256), lds, s, (const float*)src, stride_c,
                       (const float*)gain, (const float*)shift, (float*)dst, ldd, positions, (int)channels, eps);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Row softmax of a stored score matrix: p = softmax(scale * s [causal]).  One block per row;
// the row is read three times (maximum, sum, write), which is what an unfused graph does
// (AutoChunk section 2.1: the scores and the probabilities are separate activation tensors).
// Row r is query i = r mod period, standing at position q_offset + i; with the causal mask it
// sees keys j <= q_offset + i and the rest get probability exactly 0.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
softmax_rows(const T* src, int64_t lds_, T* dst, int64_t ldd, int64_t cols, float scale,
             int causal, int64_t q_offset, int64_t period) {
  __shared__ float red[4];
  const int64_t r = blockIdx.x;
  const T* in = src + r * lds_;
  T* out = dst + r * ldd;
  int64_t vis = cols;
  if (causal) {
    const int64_t last = q_offset + r % period;
    if (last + 1 < vis) vis = last + 1;
  }
  const int tid = threadIdx.x;
  float m = -INFINITY;
  for (int64_t j = tid; j < vis; j += 256) m = fmaxf(m, Elem<T>::ld(in + j));
  m = wave_max(m);
  if (tid % 64 == 0) red[tid / 64] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) * scale;      // scale > 0
  __syncthreads();
  float l = 0.f;
  for (int64_t j = tid; j < vis; j += 256) l += __expf(Elem<T>::ld(in + j) * scale - m);
  l = wave_sum(l);
  if (tid % 64 == 0) red[tid / 64] = l;
  __syncthreads();
  const float inv = 1.0f / (red[0] + red[1] + red[2] + red[3]);
  for (int64_t j = tid; j < cols; j += 256)
    Elem<T>::st(out + j, j < vis ? __expf(Elem<T>::ld(in + j) * scale - m) * inv : 0.f);
}

// The same with 16-byte accesses (cols and both row strides multiples of the vector, aligned bases).  NV > 0: the
// row (at most 256 * NV vectors) stays in registers between the three steps, so it is read once; NV = 0: any
// length, three passes as above.
template <typename T, int NV>
__global__ void __launch_bounds__(256)
softmax_rows_vec(const T* src, int64_t lds_, T* dst, int64_t ldd, int64_t cols, float scale,
                 int causal, int64_t q_offset, int64_t period) {
  constexpr int V = Elem<T>::kVec;
  constexpr int R = NV > 0 ? NV : 1;
  __shared__ float red[4];
  const int64_t r = blockIdx.x;
  const T* in = src + r * lds_;
  T* out = dst + r * ldd;
  int64_t vis = cols;
  if (causal) {
    const int64_t last = q_offset + r % period;
    if (last + 1 < vis) vis = last + 1;
  }
  const int tid = threadIdx.x;
  const int64_t nvec = cols / V;
  float v[R][V];
  float m = -INFINITY;
  if (NV > 0) {
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const int64_t i = tid + 256 * k;
      if (i * V < vis) load_vec(in + i * V, v[k]);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        if (!(i * V + e < vis)) v[k][e] = -INFINITY;
        m = fmaxf(m, v[k][e]);
      }
    }
  } else {
    for (int64_t i = tid; i * V < vis; i += 256) {
      load_vec(in + i * V, v[0]);
#pragma unroll
      for (int e = 0; e < V; ++e) if (i * V + e < vis) m = fmaxf(m, v[0][e]);
    }
  }
  m = wave_max(m);
  if (tid % 64 == 0) red[tid / 64] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) * scale;      // scale > 0
  __syncthreads();
  float l = 0.f;
  if (NV > 0) {
#pragma unroll
    for (int k = 0; k < R; ++k)
#pragma unroll
      for (int e = 0; e < V; ++e) { v[k][e] = __expf(v[k][e] * scale - m); l += v[k][e]; }    // exp(-inf) = 0
  } else {
    for (int64_t i = tid; i * V < vis; i += 256) {
      load_vec(in + i * V, v[0]);
#pragma unroll
      for (int e = 0; e < V; ++e) if (i * V + e < vis) l += __expf(v[0][e] * scale - m);
    }
  }
  l = wave_sum(l);
  if (tid % 64 == 0) red[tid / 64] = l;
  __syncthreads();
  const float inv = 1.0f / (red[0] + red[1] + red[2] + red[3]);
  if (NV > 0) {
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const int64_t i = tid + 256 * k;
      if (i >= nvec) continue;
#pragma unroll
      for (int e = 0; e < V; ++e) v[k][e] *= inv;
      store_vec(out + i * V, v[k]);
    }
  } else {
    for (int64_t i = tid; i < nvec; i += 256) {
      if (i * V < vis) load_vec(in + i * V, v[0]);
#pragma unroll
      for (int e = 0; e < V; ++e) v[0][e] = i * V + e < vis ? __expf(v[0][e] * scale - m) * inv : 0.f;
      store_vec(out + i * V, v[0]);
    }
  }
}

template <typename T>
static hipError_t softmax_rows_vec_launch(const void* src, int64_t lds_, void* dst, int64_t ldd, int64_t rows, int64_t cols,
                                          float scale, int causal, int64_t q_offset, int64_t period, hipStream_t s) {
  const int64_t nvec = cols / Elem<T>::kVec;
  const dim3 grid((unsigned)rows);
#define AC_SOFTMAX_VEC(NV)                                                                                        \
  hipLaunchKernelGGL((softmax_rows_vec<T, NV>), grid, dim3(256), 0, s, (const T*)src, lds_, (T*)dst, ldd, cols, scale, \
                     causal, q_offset, period)
  if (nvec <= 256) AC_SOFTMAX_VEC(1);
  else if (nvec <= 512) AC_SOFTMAX_VEC(2);
  else if (nvec <= 1024) AC_SOFTMAX_VEC(4);
  else if (nvec <= 2048) AC_SOFTMAX_VEC(8);
  else AC_SOFTMAX_VEC(0);
#undef AC_SOFTMAX_VEC
  return hipGetLastError();
}

hipError_t launch_softmax_rows(const void* src, int64_t lds_, void* dst, int64_t ldd, int64_t rows, int64_t cols,
                               float scale, int causal, int64_t q_offset, int64_t period, int dtype, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (period <= 0 || !(scale > 0.f) || rows > 0x7fffffffLL) return hipErrorInvalidValue;
  const int64_t vec = dtype == AC_BF16 ? 8 : 4;
  if (cols % vec == 0 && lds_ % vec == 0 && ldd % vec == 0 && ((uintptr_t)src % 16) == 0 && ((uintptr_t)dst % 16) == 0) {
    if (dtype == AC_BF16) return softmax_rows_vec_launch<bf16_t>(src, lds_, dst, ldd, rows, cols, scale, causal, q_offset, period, s);
    return softmax_rows_vec_launch<float>(src, lds_, dst, ldd, rows, cols, scale, causal, q_offset, period, s);
  }
  if (dtype == AC_BF16)
    hipLaunchKernelGGL((softmax_rows<bf16_t>), dim3((unsigned)rows), dim3(256), 0, s, (const bf16_t*)src, lds_,
                       (bf16_t*)dst, ldd, cols, scale, causal, q_offset, period);
  else
    hipLaunchKernelGGL((softmax_rows<float>), dim3((unsigned)rows), dim3(256), 0, s, (const float*)src, lds_,
                       (float*)dst, ldd, cols, scale, causal, q_offset, period);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// GroupNorm (+ SiLU) of channels-last images x [images, positions, C]: the C channels of an image
// in `groups` runs of C / groups consecutive channels, mean and biased variance over a run's
// channels and all positions.  Two kernels, both HBM-bound passes over the images:
//   group_norm_partials_rows: block (image, part) reads whole rows of its share of the positions once (a lane
//     keeps one 16-byte run of channels and accumulates, per channel, the sum and the sum of squares of the
//     deviations from one value per group), one thread per group adds up its channels' sums in fixed order and
//     writes (count, mean, sum of squared deviations) per (image, group, part).  Rows wider than 256 such runs take group_norm_partials, one block per (image, group,
//     part), which reads only its group's channels of every row: with 10-channel groups every cache line is
//     then fetched by six blocks on different XCDs, twice (measured: 12 times the image per launch);
//   group_norm_apply: every block first merges the partials of its image (a tree of the parallel-variance
//     formula per group, one partial per lane; fixed shape, so the result does not depend on timing), then
//     normalises 16-byte runs of channels with a gain and a shift per channel and applies the activation.
// Statistics and arithmetic in fp32.
// ------------------------------------------------------------------------------------
constexpr int kGnParts = 64;          // position shares per (image, group): enough blocks to fill the chip at 2 images
constexpr int kGnApplyChunks = 4;     // 16-byte runs per thread of the apply kernel (amortises the merge of the partials)
constexpr int kGnMaxGroups = 128;

template <typename T>
__global__ void __launch_bounds__(256)
group_norm_partials(const T* x, float* part, int64_t positions, int channels, int groups) {
  __shared__ float red[4];
  const int cg = channels / groups;
  const int64_t bg = blockIdx.x;                  // image * groups + group
  const int64_t image = bg / groups;
  const int g = (int)(bg % groups);
  const int part_i = blockIdx.y;
  const int64_t per = (positions + kGnParts - 1) / kGnParts;
  const int64_t p0 = part_i * per, p1 = p0 + per < positions ? p0 + per : positions;
  const T* base = x + image * positions * channels + g * cg;
  const int tid = threadIdx.x;
  const int64_t count = p1 > p0 ? (p1 - p0) * cg : 0;
  float sum = 0.f;
  for (int64_t i = tid; i < count; i += 256) sum += Elem<T>::ld(base + (p0 + i / cg) * channels + i % cg);
  sum = wave_sum(sum);
  if (tid % 64 == 0) red[tid / 64] = sum;
  __syncthreads();
  const float mean = count > 0 ? (red[0] + red[1] + red[2] + red[3]) / (float)count : 0.f;
  __syncthreads();
  float m2 = 0.f;
  for (int64_t i = tid; i < count; i += 256) {
    const float d = Elem<T>::ld(base + (p0 + i / cg) * channels + i % cg) - mean;
    m2 += d * d;
  }
  m2 = wave_sum(m2);
  if (tid % 64 == 0) red[tid / 64] = m2;
  __syncthreads();
  if (tid == 0) {
    float* o = part + (bg * kGnParts + part_i) * 3;
    o[0] = (float)count; o[1] = mean; o[2] = red[0] + red[1] + red[2] + red[3];
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
group_norm_partials_rows(const T* x, float* part, int64_t positions, int channels, int groups) {
  constexpr int V = Elem<T>::kVec;
  __shared__ float s_s1[256][V + 1], s_s2[256][V + 1];   // (padded: a thread's row starts in its own bank)
  const int vpr = channels / V;                    // 16-byte runs per row (<= 256)
  const int rpp = 256 / vpr;                       // rows per pass of the block
  const int cg = channels / groups;
  const int64_t image = blockIdx.x;
  const int part_i = blockIdx.y;
  const int64_t per = (positions + kGnParts - 1) / kGnParts;
  const int64_t p0 = part_i * per, p1 = p0 + per < positions ? p0 + per : positions;
  const int tid = threadIdx.x, v = tid % vpr, r = tid / vpr;
  const T* img = x + image * positions * channels;
  // Sums of the deviations from one value per group, the group's first channel at the share's first position
  // (the shifted-data form: the sums stay small whatever the mean is, and merging lanes is plain addition).
  float k[V], s1[V], s2[V];
#pragma unroll
  for (int j = 0; j < V; ++j) { k[j] = 0.f; s1[j] = 0.f; s2[j] = 0.f; }
  if (r < rpp && p0 + r < p1) {
#pragma unroll
    for (int j = 0; j < V; ++j) k[j] = Elem<T>::ld(img + p0 * channels + (v * V + j) / cg * cg);
    const T* col = img + v * V;
    constexpr int B = 8;     // rows in flight per thread: the rows were written by the kernel before and come from memory
    for (int64_t base = p0 + r; base < p1; base += (int64_t)B * rpp) {
      float val[B][V];
#pragma unroll
      for (int i = 0; i < B; ++i) {
        const int64_t pos = base + (int64_t)i * rpp;
        load_vec(col + (pos < p1 ? pos : p1 - 1) * channels, val[i]);    // past the end: a valid row, not counted
      }
#pragma unroll
      for (int i = 0; i < B; ++i) {
        const float live = base + (int64_t)i * rpp < p1 ? 1.f : 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j) { const float d = (val[i][j] - k[j]) * live; s1[j] += d; s2[j] += d * d; }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < V; ++j) { s_s1[tid][j] = s1[j]; s_s2[tid][j] = s2[j]; }
  __syncthreads();
  for (int g = tid; g < groups; g += 256) {
    float a1 = 0.f, a2 = 0.f;
    for (int c = g * cg; c < (g + 1) * cg; ++c)
      for (int rr = 0; rr < rpp; ++rr) {             // fixed order: the result does not depend on timing
        a1 += s_s1[rr * vpr + c / V][c % V];
        a2 += s_s2[rr * vpr + c / V][c % V];
      }
    const float cnt = p1 > p0 ? (float)((p1 - p0) * cg) : 0.f;
    const float kg = p1 > p0 ? Elem<T>::ld(img + p0 * channels + g * cg) : 0.f;
    float* o = part + ((image * groups + g) * kGnParts + part_i) * 3;
    o[0] = cnt;
    o[1] = cnt > 0.f ? kg + a1 / cnt : 0.f;
    o[2] = cnt > 0.f ? fmaxf(a2 - a1 * a1 / cnt, 0.f) : 0.f;
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
group_norm_apply(const T* x, const float* part, const T* gain, const T* shift, T* y, int64_t positions, int channels,
                 int groups, float eps, int act) {
  __shared__ float s_mean[kGnMaxGroups], s_rstd[kGnMaxGroups];
  const int64_t image = blockIdx.y;
  const int tid = threadIdx.x;
  // a wave merges the 64 partials of a group as a tree (lane l holds part l; fixed shape, so the result does
  // not depend on timing): a thread that walked them one after the other cost more than the pass itself
  static_assert(kGnParts == kWave, "one partial per lane");
  constexpr int GB = 8;                            // groups whose partials a wave has in flight at a time
  for (int g0 = tid / kWave; g0 < groups; g0 += GB * (256 / kWave)) {
    float n[GB], mean[GB], m2[GB];
#pragma unroll
    for (int i = 0; i < GB; ++i) {
      const int g = g0 + i * (256 / kWave);
      const float* pp = part + ((image * groups + (g < groups ? g : groups - 1)) * kGnParts + tid % kWave) * 3;
      n[i] = pp[0]; mean[i] = pp[1]; m2[i] = pp[2];
    }
#pragma unroll
    for (int off = kWave / 2; off >= 1; off /= 2) {
#pragma unroll
      for (int i = 0; i < GB; ++i) {                 // (the groups' chains are independent: their exchanges overlap)
        const float nb = __shfl_down(n[i], off, kWave), mb = __shfl_down(mean[i], off, kWave), m2b = __shfl_down(m2[i], off, kWave);
        const float tot = n[i] + nb;
        const float delta = mb - mean[i], f = nb > 0.f ? nb * __builtin_amdgcn_rcpf(tot) : 0.f;   // (a weight, good to 1 ulp)
        mean[i] += delta * f;
        m2[i] += m2b + delta * delta * (n[i] * f);
        n[i] = tot;
      }
    }
#pragma unroll
    for (int i = 0; i < GB; ++i) {
      const int g = g0 + i * (256 / kWave);
      if (g < groups && tid % kWave == 0) {
        s_mean[g] = mean[i];
        s_rstd[g] = rsqrtf(m2[i] / n[i] + eps);
      }
    }
  }
  __syncthreads();
  constexpr int V = Elem<T>::kVec;                          // channels per lane and access: 16 bytes
  const int cg = channels / groups;
  const int64_t chunks = positions * (channels / V);
  float v[kGnApplyChunks][V];
  int64_t off[kGnApplyChunks];
  int ch0[kGnApplyChunks];
#pragma unroll
  for (int k = 0; k < kGnApplyChunks; ++k) {       // all loads of the thread first, so that they overlap
    int64_t c = ((int64_t)blockIdx.x * kGnApplyChunks + k) * 256 + tid;
    if (c >= chunks) c = chunks - 1;               // (a valid run; not stored below)
    ch0[k] = (int)(c % (channels / V)) * V;
    off[k] = (image * positions + c / (channels / V)) * channels + ch0[k];
    load_vec(x + off[k], v[k]);
  }
#pragma unroll
  for (int k = 0; k < kGnApplyChunks; ++k) {
    if (((int64_t)blockIdx.x * kGnApplyChunks + k) * 256 + tid >= chunks) break;
    float gg[V], sh[V];
    load_vec(gain + ch0[k], gg);
    load_vec(shift + ch0[k], sh);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const int g = (ch0[k] + i) / cg;
      const float t = (v[k][i] - s_mean[g]) * s_rstd[g] * gg[i] + sh[i];
      v[k][i] = act == AC_ACT_SILU ? t * sigmoidf(t) : t;
    }
    store_vec(y + off[k], v[k]);
  }
}

uint64_t group_norm_workspace_bytes(int64_t images, int groups) { return (uint64_t)images * groups * kGnParts * 3 * sizeof(float); }

hipError_t launch_group_norm(const void* x, const void* gain, const void* shift, void* y, void* partials, int64_t images,
                             int64_t positions, int channels, int groups, float eps, int act, int dtype, hipStream_t s) {
  if (images <= 0 || positions <= 0) return hipSuccess;
  if (channels <= 0 || groups <= 0 || groups > kGnMaxGroups || channels % groups != 0 || channels % 8 != 0 || !partials ||
      images > 65535 || (act != AC_ACT_NONE && act != AC_ACT_SILU))
    return hipErrorInvalidValue;
  const bool by_rows = channels / (dtype == AC_BF16 ? 8 : 4) <= 256;
  const dim3 g1 = by_rows ? dim3((unsigned)images, kGnParts) : dim3((unsigned)(images * groups), kGnParts);
  const int64_t chunks = positions * (channels / (dtype == AC_BF16 ? 8 : 4));
  const dim3 g2((unsigned)((chunks + 256 * kGnApplyChunks - 1) / (256 * kGnApplyChunks)), (unsigned)images);
  if (dtype == AC_BF16) {
    if (by_rows) hipLaunchKernelGGL((group_norm_partials_rows<bf16_t>), g1, dim3(256), 0, s, (const bf16_t*)x, (float*)partials, positions, channels, groups);
    else hipLaunchKernelGGL((group_norm_partials<bf16_t>), g1, dim3(256), 0, s, (const bf16_t*)x, (float*)partials, positions, channels, groups);
    hipLaunchKernelGGL((group_norm_apply<bf16_t>), g2, dim3(256), 0, s, (const bf16_t*)x, (const float*)partials, (const bf16_t*)gain,
                       (const bf16_t*)shift, (bf16_t*)y, positions, channels, groups, eps, act);
  } else {
    if (by_rows) hipLaunchKernelGGL((group_norm_partials_rows<float>), g1, dim3(256), 0, s, (const float*)x, (float*)partials, positions, channels, groups);
    else hipLaunchKernelGGL((group_norm_partials<float>), g1, dim3(256), 0, s, (const float*)x, (float*)partials, positions, channels, groups);
    hipLaunchKernelGGL((group_norm_apply<float>), g2, dim3(256), 0, s, (const float*)x, (const float*)partials, (const float*)gain,
                       (const float*)shift, (float*)y, positions, channels, groups, eps, act);
  }
  return hipGetLastError();
}

}  // namespace ac
