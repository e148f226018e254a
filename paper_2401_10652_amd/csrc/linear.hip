// Projection GEMMs of a chunked region: out = epilogue(a[m,k] . w[n,k]^T).
// (AutoChunk section 2.2: the QKV / output / feed-forward projections applied to one
// segment of rows; these are dense contractions and run on the bf16 matrix cores.)
//
// bf16 path: v_mfma_f32_32x32x16_bf16, 256 threads = 4 waves in a 2x2 arrangement, block
// tile BM x BN x 64 double-buffered in LDS (rows padded by 16 bytes so that the 128-bit
// fragment reads of 32 consecutive rows hit distinct banks).  The weight rows feed the
// MFMA "A" operand and the activation rows the "B" operand, so that every lane ends up
// with one output row m and groups of 4 consecutive output columns n: the bias, multiplier
// and residual are then 8-byte vector accesses and the result is stored 8 bytes at a time.
// The K loop order does not depend on the tile's position in m, so a row's result is
// bitwise the same for every chunk length.
//
// fp32 path and odd shapes: an LDS-tiled FMA kernel with full bounds checks.
#include "common.h"

namespace ac {

// ------------------------------------------------------------------------------------
// Epilogue for one element (generic kernel) — bias, activation, multiplier, residual,
// then the row-major or the strided ("transposed") store.
// ------------------------------------------------------------------------------------
// m = q * period + r for a row index m < 2^31 (the launchers refuse more rows): a 32-bit division,
// a fraction of the instructions and registers of the 64-bit one.  A period of 2^31 or more (the
// "no period" value) gives q = 0, r = m.
__device__ __forceinline__ void split_row(int64_t m, int64_t period, int64_t& q, int64_t& r) {
  if (period > 0x7fffffffLL) { q = 0; r = m; return; }
  const uint32_t qq = (uint32_t)m / (uint32_t)period;
  q = qq;
  r = (int64_t)((uint32_t)m - qq * (uint32_t)period);
}
// Offset of row m in the row-major part of the output.
__device__ __forceinline__ int64_t out_row(const LinearArgs& g, int64_t m) {
  if (g.o_period == INT64_MAX) return m * g.ldo;
  int64_t q, r;
  split_row(m, g.o_period, q, r);
  return q * g.o_s1 + r * g.o_s2;
}
// Offset of row m in the strided ("transposed") part of the output.
__device__ __forceinline__ int64_t out_t_row(const LinearArgs& g, int64_t m) {
  int64_t q, r;
  split_row(m, g.t_period, q, r);
  return q * g.t_s1 + r * g.t_s2;
}

template <typename T>
__device__ __forceinline__ void epilogue_store_one(const LinearArgs& g, int64_t m, int64_t n, float v) {
  if (g.bias) v += Elem<T>::ld((const T*)g.bias + n);
  v = apply_act_rt(v, g.act);
  if (g.mul) v *= Elem<T>::ld((const T*)g.mul + m * g.ldmul + n);
  if (g.resid) v += Elem<T>::ld((const T*)g.resid + m * g.ldr + n);
  if (n < g.n_split) {
    Elem<T>::st((T*)g.out + out_row(g, m) + n, v);
  } else {
    const int64_t off = out_t_row(g, m) + (n - g.n_split) * g.t_s3;
    Elem<T>::st((T*)g.out_t + off, v);
  }
}

template <typename T>
__global__ void __launch_bounds__(256) linear_fma(LinearArgs g) {
  __shared__ float sa[16][65];
  __shared__ float sw[16][65];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  const T* a = (const T*)g.a + (int64_t)blockIdx.z * g.sa_b;
  const T* w = (const T*)g.w + (int64_t)blockIdx.z * g.sw_b;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < g.k; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = threadIdx.x + 256 * i;
      const int row = idx / 16, kk = idx % 16;
      const bool kin = k0 + kk < g.k;
      sa[kk][row] = (kin && m0 + row < g.m) ? Elem<T>::ld(a + (m0 + row) * g.lda + k0 + kk) : 0.f;
      sw[kk][row] = (kin && n0 + row < g.n) ? Elem<T>::ld(w + (n0 + row) * g.ldw + k0 + kk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = sa[kk][ty * 4 + i]; wv[i] = sw[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < g.m && n < g.n) {
        if (g.batch > 1) Elem<T>::st((T*)g.out + (int64_t)blockIdx.z * g.so_b + m * g.ldo + n, acc[i][j]);
        else epilogue_store_one<T>(g, m, n, acc[i][j]);
      }
    }
}

// ------------------------------------------------------------------------------------
// bf16 MFMA kernel.
// ------------------------------------------------------------------------------------
constexpr int kBK = 64;            // k extent of one LDS stage
constexpr int kLdsRow = kBK + 8;   // padded row, in elements (144 bytes)
constexpr int kXcds = 8;

// Block id -> tile.  Consecutive block ids go round-robin to the 8 XCDs, each with its own
// L2; give every XCD a contiguous run of tiles, ordered in groups of 4 tile-rows so that
// tiles resident together share activation and weight panels.
__device__ __forceinline__ void tile_of_block(int64_t tiles_m, int64_t tiles_n, int64_t& tm, int64_t& tn) {
  const int64_t nb = gridDim.x, pid = blockIdx.x;
  const int64_t q = nb / kXcds, r = nb % kXcds;
  const int64_t x = pid % kXcds, idx = pid / kXcds;
  const int64_t t = x * q + (x < r ? x : r) + idx;
  constexpr int64_t GM = 4;
  const int64_t width = GM * tiles_n;
  const int64_t group = t / width;
  const int64_t first = group * GM;
  const int64_t gsz = tiles_m - first < GM ? tiles_m - first : GM;
  tm = first + (t % width) % gsz;
  tn = (t % width) / gsz;
}

// Block id -> position in a 1-D list of work items such that each XCD gets a contiguous run.
__device__ __forceinline__ int64_t xcd_run(int64_t pid, int64_t nb) {
  const int64_t q = nb / kXcds, r = nb % kXcds;
  const int64_t x = pid % kXcds, idx = pid / kXcds;
  return x * q + (x < r ? x : r) + idx;
}

// GELU (erf form) from a table in LDS.  gelu(x) = x/2 + |x| h(|x|) with h(a) = erf(a / sqrt 2) / 2,
// and h is read from 385 entries (value, step to the next) at a spacing of 1/64, interpolated
// linearly: |error of h| <= (1/64)^2 / 8 * max|h''| = 7.4e-6, and from |x| = 6 on h is 1/2 to
// fp32.  Nine instructions and one LDS read per element instead of a reciprocal, an exponential
// and a dozen more, which matters because the epilogue of an 8-wave tile overlaps with nothing.
constexpr int kGeluEntries = 385;
constexpr size_t kGeluTableBytes = (size_t)kGeluEntries * 2 * sizeof(float);
__device__ __forceinline__ void gelu_table_fill(float* tab, int tid, int nt) {
  for (int i = tid; i < kGeluEntries; i += nt) {
    const float h0 = 0.5f * erf_as((float)i * (0.70710678118654752f / 64.0f));
    const float h1 = i + 1 < kGeluEntries ? 0.5f * erf_as((float)(i + 1) * (0.70710678118654752f / 64.0f)) : h0;
    tab[2 * i] = h0;
    tab[2 * i + 1] = h1 - h0;
  }
}
__device__ __forceinline__ float gelu_table(float x, const float* tab) {
  const float a = fabsf(x);
  const float u = a * 64.0f;
  unsigned idx = (unsigned)u;                       // saturating conversion
  idx = idx < (unsigned)(kGeluEntries - 1) ? idx : (unsigned)(kGeluEntries - 1);
  const f32x2 e = *reinterpret_cast<const f32x2*>(tab + 2 * idx);
  const float h = fmaf(e[1], __builtin_amdgcn_fractf(u), e[0]);
  return fmaf(a, h, 0.5f * x);
}

// The epilogue of one block.  A tile that lies wholly in the row-major part of the output
// is rounded to bf16 into LDS (free after the k loop) and written out with 16-byte stores
// whose lanes walk along rows; other tiles (strided store, narrow or misaligned outputs)
// store 8 bytes per lane straight from the registers.
template <int ACT, int BM, int BN, int WAVES_M, int WAVES_N>
__device__ __forceinline__ void epilogue_tile(const LinearArgs& g, f32x16 (&acc)[BM / WAVES_M / 32][BN / WAVES_N / 32],
                                              bf16_t* lds, const float* gelu_tab, int64_t m0, int64_t n0,
                                              int wave_m, int wave_n, int l32, int half, int tid) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N, TM = WM / 32, TN = WN / 32;
  constexpr int CROW = BN + 8;   // padded row of the staged tile
  const bool staged = n0 + BN <= g.n_split && g.ldo % 8 == 0 && ((uintptr_t)g.out % 16) == 0 && g.n % 8 == 0 &&
                      (g.o_period == INT64_MAX || (g.o_s1 % 8 == 0 && g.o_s2 % 8 == 0));
  // a tile wholly in the strided part whose rows run contiguously (stride 1 along m, one
  // period) is staged TRANSPOSED, [n][m], and written with 16-byte stores along m
  constexpr int TROW = BM + 8;
  const bool tstaged = !staged && n0 >= g.n_split && g.t_s2 == 1 && g.m % 8 == 0 && g.t_s1 % 8 == 0 && g.t_s3 % 8 == 0 &&
                       ((uintptr_t)g.out_t % 16) == 0 && (g.t_period == INT64_MAX || (g.t_period % BM == 0));
  if (staged || tstaged) __syncthreads();   // every wave is done reading the k-loop buffers
  // Operand loads of the epilogue are issued in batches and from clamped, always valid
  // addresses, so that a lane waits for memory once per batch and not once per group of four
  // columns; only the stores are predicated.  A batch is a row of the wave's 32x32
  // accumulator tiles in the 8-wave shapes and a single tile in the 4-wave shapes, which
  // have no registers to spare.
  constexpr int JB = WAVES_M * WAVES_N == 8 ? TN : 1;
  const bf16x4 zero4 = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
  const int cl0 = wave_n * WN + 4 * half;      // this lane's first column of the tile
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int rl = wave_m * WM + i * 32 + l32;
    const int64_t m = m0 + rl;
    const bool row_ok = m < g.m;
    const int64_t mc = row_ok ? m : g.m - 1;
    // offset of row m in the strided ("transposed") output, if any
    const int64_t t_base = g.n_split < g.n ? out_t_row(g, mc) : 0;
    const int64_t bias_row = g.bias_period > 0 ? (int64_t)((uint32_t)mc / (uint32_t)g.bias_period) * g.n : 0;   // (m < 2^31)
#pragma unroll
    for (int jb = 0; jb < TN; jb += JB) {
      bf16x4 bias_v[JB][4], mul_v[JB][4], res_v[JB][4];
      int64_t nc[JB][4];
#pragma unroll
      for (int j = 0; j < JB; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t n = n0 + cl0 + (jb + j) * 32 + 8 * q;
          nc[j][q] = n < g.n ? n : g.n - 4;
          bias_v[j][q] = g.bias ? *reinterpret_cast<const bf16x4*>((const bf16_t*)g.bias + bias_row + nc[j][q]) : zero4;
        }
      if (g.mul) {
#pragma unroll
        for (int j = 0; j < JB; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            mul_v[j][q] = *reinterpret_cast<const bf16x4*>((const bf16_t*)g.mul + mc * g.ldmul + nc[j][q]);
      }
      if (g.resid) {
#pragma unroll
        for (int j = 0; j < JB; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            res_v[j][q] = *reinterpret_cast<const bf16x4*>((const bf16_t*)g.resid + mc * g.ldr + nc[j][q]);
      }
#pragma unroll
      for (int j = 0; j < JB; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int cl = cl0 + (jb + j) * 32 + 8 * q;
          const int64_t n = n0 + cl;
          float v[4] = {acc[i][jb + j][4 * q], acc[i][jb + j][4 * q + 1], acc[i][jb + j][4 * q + 2], acc[i][jb + j][4 * q + 3]};
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const float pre = v[jj] + bf2f(bias_v[j][q][jj]);
            v[jj] = ACT == AC_ACT_GELU_ERF ? gelu_table(pre, gelu_tab) : apply_act<ACT>(pre);
          }
          if (g.mul) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) v[jj] *= bf2f(mul_v[j][q][jj]);
          }
          if (g.resid) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) v[jj] += bf2f(res_v[j][q][jj]);
          }
          const bf16x4 o = {f2bf(v[0]), f2bf(v[1]), f2bf(v[2]), f2bf(v[3])};
          if (!row_ok || n >= g.n) continue;
          if (staged) {
            *reinterpret_cast<bf16x4*>(lds + rl * CROW + cl) = o;
          } else if (tstaged) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) lds[(cl + jj) * TROW + rl] = o[jj];
          } else if (n < g.n_split) {
            *reinterpret_cast<bf16x4*>((bf16_t*)g.out + out_row(g, m) + n) = o;
          } else {
            const int64_t base = t_base + (n - g.n_split) * g.t_s3;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) ((bf16_t*)g.out_t)[base + jj * g.t_s3] = o[jj];
          }
        }
      }
    }
  }
  if (tstaged) {
    __syncthreads();
    constexpr int CPT = BM / 8;   // 16-byte chunks per staged row (one output column n)
    int64_t tq, tr;
    split_row(m0, g.t_period, tq, tr);
    const int64_t t_tile = tq * g.t_s1 + tr;   // the tile's rows share a period (and t_s2 == 1 here)
#pragma unroll 4
    for (int c = tid; c < BN * CPT; c += NT) {
      const int nl = c / CPT, mm = (c % CPT) * 8;
      const int64_t n = n0 + nl;
      if (m0 + mm < g.m && n < g.n)
        *reinterpret_cast<bf16x8*>((bf16_t*)g.out_t + t_tile + mm + (n - g.n_split) * g.t_s3) =
            *reinterpret_cast<const bf16x8*>(lds + nl * TROW + mm);
    }
    return;
  }
  if (!staged) return;
  __syncthreads();
  constexpr int CPR = BN / 8;   // 16-byte chunks per tile row
  if (g.o_period == INT64_MAX) {   // (two loops: the common one carries no trace of the regrouping arithmetic)
#pragma unroll 4
    for (int c = tid; c < BM * CPR; c += NT) {
      const int rl = c / CPR, cc = (c % CPR) * 8;
      const int64_t m = m0 + rl, n = n0 + cc;
      if (m < g.m && n < g.n)
        *reinterpret_cast<bf16x8*>((bf16_t*)g.out + m * g.ldo + n) = *reinterpret_cast<const bf16x8*>(lds + rl * CROW + cc);
    }
  } else {
#pragma unroll 2
    for (int c = tid; c < BM * CPR; c += NT) {
      const int rl = c / CPR, cc = (c % CPR) * 8;
      const int64_t m = m0 + rl, n = n0 + cc;
      if (m < g.m && n < g.n)
        *reinterpret_cast<bf16x8*>((bf16_t*)g.out + out_row(g, m) + n) = *reinterpret_cast<const bf16x8*>(lds + rl * CROW + cc);
    }
  }
}

// CONV: the A operand is gathered from channels-last images as the 3x3 convolution needs it (implicit GEMM):
// a k tile of 64 lies inside one window position (conv_c is a multiple of 64), so it is the same 64 input
// channels of the pixel shifted by that position for every row of the tile, or zeros where the shifted pixel
// falls outside its image.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool CONV = false>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) linear_mfma_bf16(LinearArgs g) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;           // threads
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;            // 32x32 MFMA tiles per wave
  constexpr int A_CHUNKS = BM * 8 / NT, W_CHUNKS = BN * 8 / NT;   // 16-byte chunks per thread
  static_assert(A_CHUNKS >= 1 && W_CHUNKS >= 1 && TM >= 1 && TN >= 1, "tile / wave layout mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);                 // [2][BM][kLdsRow]
  bf16_t* sW = sA + 2 * BM * kLdsRow;                               // [2][BN][kLdsRow]
  float* gelu_tab = reinterpret_cast<float*>(sW + 2 * BN * kLdsRow);   // after the k-loop buffers
  if (g.act == AC_ACT_GELU_ERF) gelu_table_fill(gelu_tab, threadIdx.x, NT);   // read after many barriers

  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int l32 = lane % 32, half = lane / 32;
  const int64_t tiles_m = (g.m + BM - 1) / BM, tiles_n = (g.n + BN - 1) / BN;
  int64_t tm_, tn_;
  tile_of_block(tiles_m, tiles_n, tm_, tn_);
  const int64_t m0 = tm_ * BM, n0 = tn_ * BN;
  const int64_t product = g.batch_descending ? (int64_t)gridDim.y - 1 - blockIdx.y : (int64_t)blockIdx.y;
  const bf16_t* a = (const bf16_t*)g.a + product * g.sa_b;
  const bf16_t* w = (const bf16_t*)g.w + product * g.sw_b;
  g.out = (bf16_t*)g.out + product * g.so_b;

  // Global source of each 16-byte chunk this thread stages (rows clamped into range; the
  // results of clamped rows are never stored).
  const bf16_t* a_src[A_CHUNKS];
  const bf16_t* w_src[W_CHUNKS];
  int a_dst[A_CHUNKS], w_dst[W_CHUNKS];
  int a_taps[A_CHUNKS];   // CONV: bit t set = window position t of this row's pixel lies inside the image
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int c = tid + NT * i, row = c >> 3, ch = c & 7;
    int64_t gr = m0 + row; if (gr > g.m - 1) gr = g.m - 1;
    a_src[i] = a + gr * (CONV ? (int64_t)g.conv_c : g.lda) + ch * 8;
    a_dst[i] = row * kLdsRow + ch * 8;
    a_taps[i] = 0;
    if (CONV) {
      const int pix = (int)(gr % ((int64_t)g.conv_h * g.conv_w)), ph = pix / g.conv_w, pw = pix % g.conv_w;
      for (int t = 0; t < 9; ++t) {
        const int hh = ph + t / 3 - 1, ww = pw + t % 3 - 1;
        if (hh >= 0 && hh < g.conv_h && ww >= 0 && ww < g.conv_w) a_taps[i] |= 1 << t;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < W_CHUNKS; ++i) {
    const int c = tid + NT * i, row = c >> 3, ch = c & 7;
    int64_t gr = n0 + row; if (gr > g.n - 1) gr = g.n - 1;
    w_src[i] = w + gr * g.ldw + ch * 8;
    w_dst[i] = row * kLdsRow + ch * 8;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Software pipeline over k tiles with S register sets.  During step kt the wave
  //   - has the global loads of tiles kt+2 .. kt+S in flight into S-1 register sets,
  //   - multiplies tile kt out of LDS buffer kt & 1, and
  //   - between the MFMA groups of that multiply, writes tile kt+1 (loaded S-1 steps ago,
  //     so long since landed) from the remaining register set into the other LDS
  //     buffer.  LDS takes writes at about a third of its read rate, and all waves of the
  //     block reach the barrier together, so the writes must hide under the matrix work
  //     rather than sit between the multiply and the barrier.
  // Two sets are what the large tiles' accumulators leave room for.  The small tiles take four:
  // inside a model their operands were written by the kernel before (another XCD's L2, so they
  // come from memory), and a 512 x 768 x 3072 product on 32x64 tiles went from 15.6 to 12.3 us;
  // with operands that are already in L2 the depth makes no difference.
  const int64_t kt_count = g.k / kBK;
  constexpr int KSTEPS = kBK / 16;
  // register sets of the staging ring (registers allow four only in the small tiles)
  constexpr int S = TM * TN < 4 ? 4 : 2;
  auto load_regs = [&](bf16x8 (&ar)[A_CHUNKS], bf16x8 (&wr)[W_CHUNKS], int64_t kt) {
    const int64_t koff = kt * kBK;
    if (CONV) {
      const int tap = (int)(koff / g.conv_c), c0 = (int)(koff % g.conv_c);
      const int64_t shift = ((int64_t)(tap / 3 - 1) * g.conv_w + (tap % 3 - 1)) * g.conv_c + c0;
#pragma unroll
      for (int i = 0; i < A_CHUNKS; ++i) {
        const bool inside = (a_taps[i] >> tap) & 1;
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(a_src[i] + (inside ? shift : (int64_t)c0));   // always a valid address
        const bf16x8 zero = {};
        ar[i] = inside ? v : zero;
      }
    } else {
#pragma unroll
      for (int i = 0; i < A_CHUNKS; ++i) ar[i] = *reinterpret_cast<const bf16x8*>(a_src[i] + koff);
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) wr[i] = *reinterpret_cast<const bf16x8*>(w_src[i] + koff);
  };
  // chunk c of the A_CHUNKS + W_CHUNKS staged chunks -> LDS buffer `buf`
  auto store_chunk = [&](const bf16x8 (&ar)[A_CHUNKS], const bf16x8 (&wr)[W_CHUNKS], int buf, int c) {
    if (c < A_CHUNKS) *reinterpret_cast<bf16x8*>(sA + buf * BM * kLdsRow + a_dst[c]) = ar[c];
    else *reinterpret_cast<bf16x8*>(sW + buf * BN * kLdsRow + w_dst[c - A_CHUNKS]) = wr[c - A_CHUNKS];
  };
  constexpr int CHUNKS = A_CHUNKS + W_CHUNKS;
  auto step = [&](int64_t kt, bf16x8 (&hold_a)[A_CHUNKS], bf16x8 (&hold_w)[W_CHUNKS],
                  bf16x8 (&fill_a)[A_CHUNKS], bf16x8 (&fill_w)[W_CHUNKS]) {
    // No branches in the step: a conditional load would make the compiler lose count of the
    // loads in flight and wait for the newest ones before every LDS store.  Past the end the
    // last tile is simply loaded (and stored to the idle buffer) again.
    load_regs(fill_a, fill_w, kt + S < kt_count ? kt + S : kt_count - 1);
    const int buf = (int)(kt & 1);
    const bf16_t* cA = sA + buf * BM * kLdsRow + (wave_m * WM + l32) * kLdsRow + half * 8;
    const bf16_t* cW = sW + buf * BN * kLdsRow + (wave_n * WN + l32) * kLdsRow + half * 8;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      bf16x8 fa[TM], fw[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(cA + i * 32 * kLdsRow + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) fw[j] = *reinterpret_cast<const bf16x8*>(cW + j * 32 * kLdsRow + ks * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[j], fa[i], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int c = ks * CHUNKS / KSTEPS; c < (ks + 1) * CHUNKS / KSTEPS; ++c) store_chunk(hold_a, hold_w, buf ^ 1, c);
      __builtin_amdgcn_sched_barrier(0);   // keep each slice of the stores with its MFMA group
    }
    __syncthreads();
  };

  // One MFMA tile per wave (64x64 blocks: launches of a few hundred rows, one wave per SIMD): a k step is
  // then one matrix instruction behind two LDS reads, and with the reads issued just before it the loop
  // runs at the LDS latency, a third of the matrix rate.  Here the fragments of the WHOLE next tile are
  // read while this tile's (already in registers) are multiplied, so everything is staged one tile earlier:
  // during step kt the wave loads tile kt+S+1 from memory, reads the fragments of tile kt+1 out of LDS buffer
  // (kt+1) & 1, multiplies tile kt from registers and writes tile kt+2 into buffer kt & 1 (whose reads were
  // issued a step ago and have completed before the barrier).  Same instructions on the same operands in the
  // same order per output element as the loop above, so results do not depend on which loop ran.
  constexpr bool FRAGS_AHEAD = TM == 1 && TN == 1 && !CONV;
  if constexpr (FRAGS_AHEAD) {
    bf16x8 ra[S][A_CHUNKS], rw[S][W_CHUNKS];
    bf16x8 fa[2][KSTEPS], fw[2][KSTEPS];
    auto read_frags = [&](bf16x8 (&fa_)[KSTEPS], bf16x8 (&fw_)[KSTEPS], int buf) {
      const bf16_t* cA = sA + buf * BM * kLdsRow + (wave_m * WM + l32) * kLdsRow + half * 8;
      const bf16_t* cW = sW + buf * BN * kLdsRow + (wave_n * WN + l32) * kLdsRow + half * 8;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        fa_[ks] = *reinterpret_cast<const bf16x8*>(cA + ks * 16);
        fw_[ks] = *reinterpret_cast<const bf16x8*>(cW + ks * 16);
      }
    };
    auto clamp_kt = [&](int64_t t) { return t < kt_count ? t : kt_count - 1; };   // past the end: the last tile again
    // step kt: set `hold` carries tile kt+2, set `fill` (stored a step ago) takes tile kt+S+1
    auto ahead = [&](int64_t kt, bf16x8 (&hold_a)[A_CHUNKS], bf16x8 (&hold_w)[W_CHUNKS],
                     bf16x8 (&fill_a)[A_CHUNKS], bf16x8 (&fill_w)[W_CHUNKS],
                     const bf16x8 (&cur_a)[KSTEPS], const bf16x8 (&cur_w)[KSTEPS],
                     bf16x8 (&next_a)[KSTEPS], bf16x8 (&next_w)[KSTEPS]) {
      load_regs(fill_a, fill_w, clamp_kt(kt + S + 1));
      const int buf = (int)(kt & 1);
      read_frags(next_a, next_w, buf ^ 1);
      __builtin_amdgcn_sched_barrier(0);   // the reads go out before the first matrix instruction
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur_w[ks], cur_a[ks], acc[0][0], 0, 0, 0);
#pragma unroll
        for (int c = ks * CHUNKS / KSTEPS; c < (ks + 1) * CHUNKS / KSTEPS; ++c) store_chunk(hold_a, hold_w, buf, c);
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
    };
    load_regs(ra[0], rw[0], 0);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) store_chunk(ra[0], rw[0], 0, c);
    load_regs(ra[S - 1], rw[S - 1], clamp_kt(1));
#pragma unroll
    for (int u = 0; u + 1 < S; ++u) load_regs(ra[u], rw[u], clamp_kt(2 + u));
    __syncthreads();
    read_frags(fa[0], fw[0], 0);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) store_chunk(ra[S - 1], rw[S - 1], 1, c);
    __syncthreads();
    int64_t kt = 0;
    for (; kt + S <= kt_count; kt += S) {
#pragma unroll
      for (int u = 0; u < S; ++u)
        ahead(kt + u, ra[u], rw[u], ra[(u + S - 1) % S], rw[(u + S - 1) % S], fa[u & 1], fw[u & 1], fa[(u & 1) ^ 1], fw[(u & 1) ^ 1]);
    }
#pragma unroll
    for (int u = 0; u + 1 < S; ++u)
      if (kt + u < kt_count)
        ahead(kt + u, ra[u], rw[u], ra[(u + S - 1) % S], rw[(u + S - 1) % S], fa[u & 1], fw[u & 1], fa[(u & 1) ^ 1], fw[(u & 1) ^ 1]);
  } else {
    bf16x8 ra[S][A_CHUNKS], rw[S][W_CHUNKS];
    load_regs(ra[0], rw[0], 0);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) store_chunk(ra[0], rw[0], 0, c);
#pragma unroll
    for (int u = 0; u + 1 < S; ++u) load_regs(ra[u], rw[u], 1 + u < kt_count ? 1 + u : kt_count - 1);
    __syncthreads();
    int64_t kt = 0;
    for (; kt + S <= kt_count; kt += S) {
#pragma unroll
      for (int u = 0; u < S; ++u) step(kt + u, ra[u], rw[u], ra[(u + S - 1) % S], rw[(u + S - 1) % S]);
    }
#pragma unroll
    for (int u = 0; u + 1 < S; ++u)
      if (kt + u < kt_count) step(kt + u, ra[u], rw[u], ra[(u + S - 1) % S], rw[(u + S - 1) % S]);
  }

  // acc[i][j][r]: row m = .. + l32, column n = .. + 8*(r/4) + 4*half + (r%4).
  bf16_t* lds = reinterpret_cast<bf16_t*>(smem_raw);
  switch (g.act) {   // one branch per launch, so the activation is inlined without a per-element switch
    case AC_ACT_GELU_ERF: epilogue_tile<AC_ACT_GELU_ERF, BM, BN, WAVES_M, WAVES_N>(g, acc, lds, gelu_tab, m0, n0, wave_m, wave_n, l32, half, tid); break;
    case AC_ACT_GELU_TANH: epilogue_tile<AC_ACT_GELU_TANH, BM, BN, WAVES_M, WAVES_N>(g, acc, lds, gelu_tab, m0, n0, wave_m, wave_n, l32, half, tid); break;
    case AC_ACT_RELU: epilogue_tile<AC_ACT_RELU, BM, BN, WAVES_M, WAVES_N>(g, acc, lds, gelu_tab, m0, n0, wave_m, wave_n, l32, half, tid); break;
    case AC_ACT_SIGMOID: epilogue_tile<AC_ACT_SIGMOID, BM, BN, WAVES_M, WAVES_N>(g, acc, lds, gelu_tab, m0, n0, wave_m, wave_n, l32, half, tid); break;
    default: epilogue_tile<AC_ACT_NONE, BM, BN, WAVES_M, WAVES_N>(g, acc, lds, gelu_tab, m0, n0, wave_m, wave_n, l32, half, tid); break;
  }
}

template <int BM, int BN>
constexpr size_t mfma_lds_bytes() { return (size_t)2 * (BM + BN) * kLdsRow * sizeof(bf16_t) + kGeluTableBytes; }

template <int BM, int BN, int WAVES_M, int WAVES_N, bool CONV = false>
static hipError_t mfma_launch(const LinearArgs& g, hipStream_t s) {
  auto kern = linear_mfma_bf16<BM, BN, WAVES_M, WAVES_N, CONV>;
  constexpr size_t lds = mfma_lds_bytes<BM, BN>();
  // the attribute is per function; set once per process (the initialiser runs once, thread-safe)
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (attr_status != hipSuccess) return attr_status;
  const int64_t tiles = ((g.m + BM - 1) / BM) * ((g.n + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles, (unsigned)g.batch), dim3(64 * WAVES_M * WAVES_N), lds, s, g);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// LayerNorm + several projections of the same short rows in one kernel.
// The pair-stack modules project every LayerNorm output four or five times with K = c_z
// (gated a and b of the triangle update; q, k, v, gate and pair bias of the triangle attention;
// the transition's first layer).  Separate launches re-read the normalised rows each time and
// are bound by that traffic, not by the matrix cores.  Here a block normalises 64 rows once
// (the whole row is one k tile), keeps them in LDS as the matrix operand, and walks a list of
// 64-column weight tiles.  Tiles of 64 x 64 keep accumulators and LDS small enough for four blocks per
// CU, whose phases interleave: while one waits for its rows another multiplies and a third stores
// (measured against 64 x 128 tiles, two blocks per CU: the pair block at N = 1024 takes 9.7 instead of
// 10.4 ms in one segment per region, 11.7 instead of 12.5 ms in 64-row segments, where a launch's 1024
// blocks are then resident at once).  Each tile is prefetched into registers while the previous one is
// multiplied, and leaves through the same epilogue as the GEMM above (row-major, regrouped
// or strided store).  A gated pair keeps sigmoid(gate) in registers and multiplies the
// projection by it, so the gate never reaches memory.  Per-row arithmetic does not depend on
// the block a row falls in, so results are bitwise independent of the chunk length.
// ------------------------------------------------------------------------------------
struct LnProjKernelArgs {
  LnProjArgs a;
  int n_tiles;
  int tile_part[kMaxProjTiles];
  int tile_n0[kMaxProjTiles];
  int any_gelu;
};

constexpr int kLnProjRows = 64;   // rows per block
constexpr int kLnProjCols = 64;   // columns per weight tile

template <int K, int BN>
__global__ void __launch_bounds__(256, 2) ln_multi_proj_bf16(LnProjKernelArgs ka) {
  constexpr int BM = kLnProjRows, NT = 256;
  constexpr int TN = BN / 64;                 // 32-column MFMA tiles per wave (waves 2 x 2, 32 rows each)
  constexpr int AROW = K + 8;                 // padded LDS row (elements)
  constexpr int G = K / 8;                    // lanes per row in the LayerNorm pass (16-byte chunks per row)
  constexpr int RPP = NT / G;                 // rows per pass
  constexpr int PASSES = BM / RPP;
  constexpr int KSTEPS = K / 16;
  constexpr int W_CHUNKS = BN * G / NT;       // 16-byte chunks of a weight tile per thread
  constexpr int STAGE = BN * (BM + 8);        // elements the epilogue's staging tile needs (the transposed form is the larger)
  constexpr int WBUF = BN * AROW > STAGE ? BN * AROW : STAGE;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);     // [BM][AROW]: the normalised rows
  bf16_t* sW = sA + BM * AROW;                          // [BN][AROW]: weight tile; then the epilogue's staging tile
  float* gelu_tab = reinterpret_cast<float*>(sW + WBUF);
  const LnProjArgs& p = ka.a;
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wave_m = wave / 2, wave_n = wave % 2;
  const int l32 = lane % 32, half = lane / 32;
  // consecutive row tiles go to one XCD, so that neighbouring runs of a strided output meet in one L2
  const int64_t m0 = xcd_run(blockIdx.x, gridDim.x) * BM;
  if (ka.any_gelu) gelu_table_fill(gelu_tab, tid, NT);

  // ---- LayerNorm of the block's rows (G lanes per row, the row in registers, fp32 statistics)
  {
    const int lg = tid % G, rg = tid / G;
    const bf16_t* x = (const bf16_t*)p.x;
    float v[PASSES][8];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      int64_t r = m0 + ps * RPP + rg;
      if (r > p.rows - 1) r = p.rows - 1;     // rows past the end shadow the last row; never stored
      load_vec(x + r * p.ldx + lg * 8, v[ps]);
    }
    float gn[8], sh[8];
    load_vec((const bf16_t*)p.gain + lg * 8, gn);
    load_vec((const bf16_t*)p.shift + lg * 8, sh);
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += v[ps][j];
      const float mean = group_sum<G>(sum) * (1.0f / K);
      float sq = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) { const float d = v[ps][j] - mean; sq += d * d; }
      const float rstd = rsqrtf(group_sum<G>(sq) * (1.0f / K) + p.eps);
      float o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = (v[ps][j] - mean) * rstd * gn[j] + sh[j];
      store_vec(sA + (ps * RPP + rg) * AROW + lg * 8, o);
    }
  }

  bf16x8 wreg[W_CHUNKS];
  auto store_w = [&](int tid) {
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      const int c = tid + NT * i, row = c / G, ch = c % G;
      *reinterpret_cast<bf16x8*>(sW + row * AROW + ch * 8) = wreg[i];
    }
  };

  auto load_w = [&](const void* wbase, int64_t n_rows, int64_t n0, int tid) {
    const bf16_t* w = (const bf16_t*)wbase;
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      const int c = tid + NT * i, row = c / G, ch = c % G;
      int64_t gr = n0 + row; if (gr > n_rows - 1) gr = n_rows - 1;
      wreg[i] = *reinterpret_cast<const bf16x8*>(w + gr * K + ch * 8);
    }
  };
  // first weight tile of entry t: the gate's for a gated pair
  auto load_first = [&](int t, int tid) {
    const ProjPart& q = p.part[ka.tile_part[t]];
    load_w(q.gated ? q.w_gate : q.w, q.n, ka.tile_n0[t], tid);
  };
  f32x16 acc[1][TN];
  const bf16_t* cA = sA + (wave_m * 32 + l32) * AROW + half * 8;
  const bf16_t* cW = sW + (wave_n * (BN / 2) + l32) * AROW + half * 8;
  auto multiply = [&]() {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[0][j][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const bf16x8 fa = *reinterpret_cast<const bf16x8*>(cA + ks * 16);
      bf16x8 fw[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) fw[j] = *reinterpret_cast<const bf16x8*>(cW + j * 32 * AROW + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[j], fa, acc[0][j], 0, 0, 0);
    }
  };
  // this lane's 4 consecutive columns of group q in 32-column tile j: acc[i][j][4q .. 4q+3]
  auto lane_bias = [&](const void* bias, int64_t n_total, int64_t n0, int j, int q) {
    int64_t n = n0 + wave_n * (BN / 2) + j * 32 + 8 * q + 4 * half;
    if (n > n_total - 4) n = n_total - 4;
    bf16x4 bv = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
    if (bias) bv = *reinterpret_cast<const bf16x4*>((const bf16_t*)bias + n);
    return bv;
  };

  load_first(0, tid);
  for (int t = 0; t < ka.n_tiles; ++t) {
    const ProjPart& pp = p.part[ka.tile_part[t]];
    const int64_t n0 = ka.tile_n0[t];
    const bool gated = pp.gated != 0;
    // (opaque copy of the thread index: see the note at the epilogue below)
    int w_tid = tid;
    asm volatile("" : "+v"(w_tid));
    store_w(w_tid);
    __syncthreads();                         // the tile (and, the first time, the normalised rows) is in LDS
    // the next weight tile is in flight while this one is multiplied and stored
    if (gated) load_w(pp.w, pp.n, n0, w_tid);
    else if (t + 1 < ka.n_tiles) load_first(t + 1, w_tid);
    multiply();
    __syncthreads();                         // every wave is done reading the weight tile
    if (gated) {
      // sigmoid(gate) stays in registers; the projection tile of the pair follows at once
      f32x16 sg[1][TN];
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bf16x4 bv = lane_bias(pp.bias_gate, pp.n, n0, j, q);
#pragma unroll
          for (int i = 0; i < 1; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) sg[i][j][4 * q + jj] = sigmoidf(acc[i][j][4 * q + jj] + bf2f(bv[jj]));
        }
      store_w(w_tid);
      __syncthreads();
      if (t + 1 < ka.n_tiles) load_first(t + 1, w_tid);
      multiply();
      __syncthreads();
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bf16x4 bv = lane_bias(pp.bias, pp.n, n0, j, q);
#pragma unroll
          for (int i = 0; i < 1; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
              acc[i][j][4 * q + jj] = (acc[i][j][4 * q + jj] + bf2f(bv[jj])) * sg[i][j][4 * q + jj];
        }
    }
    if (!gated) {
      // bias and activation here, one uniform branch per tile, so that the epilogue below exists once
      const int act = pp.act;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bf16x4 bv = lane_bias(pp.bias, pp.n, n0, j, q);
#pragma unroll
          for (int i = 0; i < 1; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) acc[i][j][4 * q + jj] += bf2f(bv[jj]);
        }
      if (act == AC_ACT_GELU_ERF) {
#pragma unroll
        for (int i = 0; i < 1; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = gelu_table(acc[i][j][r], gelu_tab);
      } else if (act == AC_ACT_SIGMOID) {
#pragma unroll
        for (int i = 0; i < 1; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = sigmoidf(acc[i][j][r]);
      } else if (act == AC_ACT_RELU) {
#pragma unroll
        for (int i = 0; i < 1; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = fmaxf(acc[i][j][r], 0.f);
      } else if (act == AC_ACT_GELU_TANH) {
#pragma unroll
        for (int i = 0; i < 1; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = gelu_tanh(acc[i][j][r]);
      }
    }
    LinearArgs g{};
    g.out = pp.out; g.ldo = pp.ldo; g.o_period = pp.o_period; g.o_s1 = pp.o_s1; g.o_s2 = pp.o_s2;
    g.out_t = pp.out_t; g.n_split = pp.out_t ? 0 : pp.n;
    g.t_period = pp.t_period; g.t_s1 = pp.t_s1; g.t_s2 = pp.t_s2; g.t_s3 = pp.t_s3;
    g.m = p.rows; g.n = pp.n;
    // The epilogue's many per-lane addresses do not depend on the tile; hoisted out of this loop
    // they would occupy registers for the whole kernel (and spill).  Opaque copies of the lane
    // coordinates make them values of this iteration, recomputed per tile with a few ALU ops.
    int e_tid = tid, e_l32 = l32, e_half = half, e_wm = wave_m, e_wn = wave_n;
    asm volatile("" : "+v"(e_tid), "+v"(e_l32), "+v"(e_half), "+v"(e_wm), "+v"(e_wn));
    epilogue_tile<AC_ACT_NONE, BM, BN, 2, 2>(g, acc, sW, gelu_tab, m0, n0, e_wm, e_wn, e_l32, e_half, e_tid);
    __syncthreads();                         // the staging tile has been read out; sW is free for the next tile
  }
}

bool ln_proj_shapes_ok(int dtype, int64_t k, const int64_t* n, int n_parts) {
  if (dtype != AC_BF16 || (k != 64 && k != 128)) return false;
  if (n_parts < 1 || n_parts > kMaxProjParts) return false;
  int64_t tiles = 0;
  for (int i = 0; i < n_parts; ++i) {
    if (n[i] < 4 || n[i] % 4 != 0) return false;
    tiles += (n[i] + kLnProjCols - 1) / kLnProjCols;
  }
  return tiles <= kMaxProjTiles;
}

template <int K, int BN>
static hipError_t ln_proj_launch(const LnProjKernelArgs& ka, hipStream_t s) {
  auto kern = ln_multi_proj_bf16<K, BN>;
  constexpr int AROW = K + 8, STAGE = BN * (kLnProjRows + 8);
  constexpr int WBUF = BN * AROW > STAGE ? BN * AROW : STAGE;
  constexpr size_t lds_max = (size_t)(kLnProjRows * AROW + WBUF) * sizeof(bf16_t) + kGeluTableBytes;
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_max);
  if (attr_status != hipSuccess) return attr_status;
  // the GELU table is only there when a part needs it
  const size_t lds = lds_max - (ka.any_gelu ? 0 : kGeluTableBytes);
  const int64_t blocks = (ka.a.rows + kLnProjRows - 1) / kLnProjRows;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), lds, s, ka);
  return hipGetLastError();
}

hipError_t launch_ln_proj(const LnProjArgs& p_in, hipStream_t s) {
  if (p_in.rows <= 0) return hipSuccess;
  LnProjKernelArgs ka{};
  ka.a = p_in;
  LnProjArgs& p = ka.a;
  int64_t ns[kMaxProjParts];
  if (p.n_parts < 1 || p.n_parts > kMaxProjParts) return hipErrorInvalidValue;
  for (int i = 0; i < p.n_parts; ++i) ns[i] = p.part[i].n;
  if (!ln_proj_shapes_ok(AC_BF16, p.k, ns, p.n_parts)) return hipErrorNotSupported;
  if (p.ldx % 8 != 0 || ((uintptr_t)p.x % 16) != 0 || ((uintptr_t)p.gain % 16) != 0 || ((uintptr_t)p.shift % 16) != 0)
    return hipErrorNotSupported;
  if (p.rows > 0x7fffffffLL) return hipErrorInvalidValue;
  for (int i = 0; i < p.n_parts; ++i) {
    ProjPart& pp = p.part[i];
    if (!pp.w || ((uintptr_t)pp.w % 16) != 0 || ((uintptr_t)pp.w_gate % 16) != 0) return hipErrorNotSupported;
    if (pp.gated && !pp.w_gate) return hipErrorInvalidValue;
    if (((uintptr_t)pp.bias % 8) != 0 || ((uintptr_t)pp.bias_gate % 8) != 0) return hipErrorNotSupported;
    if (pp.out_t == nullptr && (pp.out == nullptr || pp.ldo % 4 != 0 || ((uintptr_t)pp.out % 8) != 0)) return hipErrorNotSupported;
    if (pp.t_period <= 0) pp.t_period = INT64_MAX;
    if (pp.o_period <= 0) pp.o_period = INT64_MAX;
    if (pp.o_period != INT64_MAX && (pp.o_s1 % 4 != 0 || pp.o_s2 % 4 != 0)) return hipErrorNotSupported;
    if (pp.act == AC_ACT_GELU_ERF && !pp.gated) ka.any_gelu = 1;
  }
  for (int i = 0; i < p.n_parts; ++i)
    for (int64_t n0 = 0; n0 < p.part[i].n; n0 += kLnProjCols) {   // a gated pair is one entry: two weight tiles, one output tile
      ka.tile_part[ka.n_tiles] = i;
      ka.tile_n0[ka.n_tiles++] = (int)n0;
    }
  return p.k == 128 ? ln_proj_launch<128, kLnProjCols>(ka, s) : ln_proj_launch<64, kLnProjCols>(ka, s);
}

static bool aligned_to(const void* p, uintptr_t a) { return p == nullptr || ((uintptr_t)p % a) == 0; }

static bool mfma_eligible(const LinearArgs& g) {
  if (g.dtype != AC_BF16) return false;
  if (g.k < kBK || g.k % kBK != 0) return false;
  if (g.n % 4 != 0 || g.n_split % 4 != 0) return false;
  if (g.lda % 8 != 0 || g.ldw % 8 != 0) return false;
  if (!aligned_to(g.a, 16) || !aligned_to(g.w, 16)) return false;
  if (g.n_split > 0 && (g.ldo % 4 != 0 || !aligned_to(g.out, 8))) return false;
  if (g.o_period != INT64_MAX && (g.o_s1 % 4 != 0 || g.o_s2 % 4 != 0)) return false;
  if (g.batch > 1 && (g.sa_b % 8 != 0 || g.sw_b % 8 != 0 || g.so_b % 4 != 0)) return false;
  if (g.bias && !aligned_to(g.bias, 8)) return false;
  if (g.mul && (g.ldmul % 4 != 0 || !aligned_to(g.mul, 8))) return false;
  if (g.resid && (g.ldr % 4 != 0 || !aligned_to(g.resid, 8))) return false;
  return true;
}

hipError_t launch_linear(const LinearArgs& g_in, hipStream_t s) {
  LinearArgs g = g_in;
  if (g.m <= 0 || g.n <= 0) return hipSuccess;
  if (g.k <= 0) return hipErrorInvalidValue;
  if (g.out_t == nullptr) g.n_split = g.n;
  if (g.n_split > g.n) g.n_split = g.n;
  if (g.t_period <= 0) g.t_period = INT64_MAX;
  if (g.o_period <= 0) g.o_period = INT64_MAX;
  if (g.batch < 1) g.batch = 1;
  if (g.batch > 1 && g.o_period != INT64_MAX) return hipErrorInvalidValue;
  if (g.batch > 1 && (g.bias || g.mul || g.resid || g.out_t || g.act != AC_ACT_NONE)) return hipErrorInvalidValue;
  if (g.batch > 65535 || g.m > 0x7fffffffLL) return hipErrorInvalidValue;
  if (g.conv_c > 0) {
    // 3x3 convolution as an implicit GEMM on 128x128 tiles; bf16 images with channels in multiples of 64 only
    if (g.dtype != AC_BF16 || g.conv_c % kBK != 0 || g.conv_h < 1 || g.conv_w < 1 || g.k != 9 * (int64_t)g.conv_c ||
        g.m % ((int64_t)g.conv_h * g.conv_w) != 0 || g.batch != 1)
      return hipErrorInvalidValue;
    g.lda = g.conv_c;
    if (!mfma_eligible(g)) return hipErrorInvalidValue;
    return mfma_launch<128, 128, 2, 2, true>(g, s);
  }
  if (mfma_eligible(g)) {
    // A CU takes in at most 64 bytes per clock from L2 while its matrix cores retire 4096
    // flops per clock, so a tile needs >= 64 flops per loaded byte just to break even: 128x128
    // tiles sit exactly there, 256x256 tiles have twice that.  Pick the tile with the least
    // estimated time: tiles per CU (rounded up) x padded tile area / measured efficiency of
    // that tile shape.  The k order is the same for all of them.
    // The small tiles are for launches of a few hundred rows.  Their k loop runs at the rate one CU
    // stages operands (measured: ~80 GB/s per CU, i.e. (BM + BN) x 128 bytes per k step), so with at
    // most one tile per CU the time goes with BM + BN, and a launch that needs a second tile on some
    // CUs takes twice as long: 512 x 768 is faster as 192 tiles of 32x64 than as 96 of 64x64 (and no
    // faster as 384 of 32x32).  64x128 tiles were measured too: 512 x 3072 x 768 takes 12.7 us as 192
    // of those against 11.0 us as 384 tiles of 64x64.
    struct Cand { int bm, bn; double eff; };
    static const Cand cands[6] = {{256, 256, 0.41}, {256, 128, 0.376}, {128, 128, 0.36}, {64, 256, 0.26},
                                  {64, 64, 0.253}, {32, 64, 0.169}};
    int best = 0;
    double best_t = 0;
    for (int c = 0; c < 6; ++c) {
      const int64_t tiles = ((g.m + cands[c].bm - 1) / cands[c].bm) * ((g.n + cands[c].bn - 1) / cands[c].bn) * g.batch;
      const double t = (double)((tiles + 255) / 256) * cands[c].bm * cands[c].bn / cands[c].eff;
      if (c == 0 || t < best_t) { best = c; best_t = t; }
    }
    switch (best) {
      case 0: return mfma_launch<256, 256, 2, 4>(g, s);
      case 1: return mfma_launch<256, 128, 4, 2>(g, s);
      case 2: return mfma_launch<128, 128, 2, 2>(g, s);
      case 3: return mfma_launch<64, 256, 1, 4>(g, s);
      case 4: return mfma_launch<64, 64, 2, 2>(g, s);
      default: return mfma_launch<32, 64, 1, 2>(g, s);
    }
  }
  dim3 grid((unsigned)((g.n + 63) / 64), (unsigned)((g.m + 63) / 64), (unsigned)g.batch);
  if (g.dtype == AC_BF16) hipLaunchKernelGGL((linear_fma<bf16_t>), grid, dim3(256), 0, s, g);
  else hipLaunchKernelGGL((linear_fma<float>), grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace ac
