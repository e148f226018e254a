// Query-chunked attention: ctx = softmax(q k^T / sqrt(d_h) [+ bias] [causal]) v [* gate]
// for the query rows of one segment against the WHOLE key/value set (the non-chunkable
// inputs of the attention region, AutoChunk section 3.1).  The scores never reach HBM:
// the intermediate activation that chunking divides by n (section 2.2, second activation
// equation) is here a 32x64 tile per wave that lives in registers, with a running
// maximum and sum per query row.
//
// bf16 MFMA kernel.  One wave owns 32 query rows; a block of 4 waves shares 64-key tiles
// of K (row-major, [key][d]) and of V^T ([d][key], as written by the projection's strided
// store) staged in double-buffered LDS.  The wave computes the TRANSPOSED score tile
// S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that a lane holds one query column and 16
// key rows per 32-key tile: the softmax max/sum over keys are in-lane reductions plus one
// exchange between the two half-waves, the rescale factor is a per-lane scalar, and the
// probabilities already sit in the register layout the next MFMA wants for its B operand
// (O^T = V^T P^T).  The k-slot order of that second MFMA is a fixed permutation of the keys
// of the tile, applied identically to P (registers) and V^T (two 8-byte LDS reads).
// Key tiles are visited in the same order for every query row regardless of which segment
// the row belongs to, so results do not depend on the chunk length.
//
// Generic kernel (fp32, odd head sizes, row-major v): one thread per query row.
#include "common.h"

#include <type_traits>

namespace ac {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kXcdCount = 8;

__device__ __forceinline__ int64_t xcd_contiguous(int64_t pid, int64_t nb) {
  const int64_t q = nb / kXcdCount, r = nb % kXcdCount;
  const int64_t x = pid % kXcdCount, idx = pid / kXcdCount;
  return x * q + (x < r ? x : r) + idx;
}

// ------------------------------------------------------------------------------------
// Generic kernel.
// ------------------------------------------------------------------------------------
template <typename T, int DH>
__global__ void __launch_bounds__(128) attention_rows(AttnArgs a) {
  constexpr int TK = 32;
  __shared__ float sK[TK][DH + 1];
  __shared__ float sV[TK][DH + 1];
  const int64_t b = blockIdx.z;
  const int h = blockIdx.y;
  const int64_t row = (int64_t)blockIdx.x * 128 + threadIdx.x;
  const bool live = row < a.sq;
  const int64_t r = live ? row : a.sq - 1;
  const T* q = (const T*)a.q + b * a.sq_b + r * a.ldq + h * DH;
  const T* kb = (const T*)a.k + b * a.sk_b + h * DH;
  const T* vb = (const T*)a.v + b * a.sv_b;
  const T* bias = a.bias ? (const T*)a.bias + h * a.s_bias_h + r * a.ld_bias : nullptr;
  const float scale = rsqrtf((float)DH);
  float qv[DH], o[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { qv[d] = Elem<T>::ld(q + d) * scale; o[d] = 0.f; }
  float m = -INFINITY, l = 0.f;
  const int64_t qpos = a.q_offset + r;
  // keys any row of this block can see
  int64_t kend = a.sk;
  if (a.causal) {
    const int64_t last = a.q_offset + ((int64_t)blockIdx.x * 128 + 127 < a.sq - 1 ? (int64_t)blockIdx.x * 128 + 127 : a.sq - 1);
    if (last + 1 < kend) kend = last + 1;
  }
  for (int64_t k0 = 0; k0 < kend; k0 += TK) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < TK * DH; idx += 128) {
      const int j = idx / DH, d = idx % DH;
      const int64_t key = k0 + j;
      float kv = 0.f, vv = 0.f;
      if (key < a.sk) {
        kv = Elem<T>::ld(kb + key * a.ldk + d);
        vv = a.v_transposed ? Elem<T>::ld(vb + (int64_t)(h * DH + d) * a.ldv + key)
                            : Elem<T>::ld(vb + key * a.ldv + h * DH + d);
      }
      sK[j][d] = kv;
      sV[j][d] = vv;
    }
    __syncthreads();
    float s[TK];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < TK; ++j) {
      float acc = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) acc = fmaf(qv[d], sK[j][d], acc);
      const int64_t key = k0 + j;
      if (bias && key < a.sk) acc += Elem<T>::ld(bias + key);
      if (key >= a.sk || (a.causal && key > qpos)) acc = -INFINITY;
      s[j] = acc;
      mx = fmaxf(mx, acc);
    }
    const float m_new = fmaxf(m, mx);
    if (m_new == -INFINITY) continue;          // nothing visible yet for this row
    const float alpha = __expf(m - m_new);     // m = -inf gives 0
    l *= alpha;
#pragma unroll
    for (int d = 0; d < DH; ++d) o[d] *= alpha;
#pragma unroll
    for (int j = 0; j < TK; ++j) {
      const float p = __expf(s[j] - m_new);
      l += p;
#pragma unroll
      for (int d = 0; d < DH; ++d) o[d] = fmaf(p, sV[j][d], o[d]);
    }
    m = m_new;
  }
  if (!live) return;
  const float inv = 1.0f / l;
  T* out = (T*)a.ctx + b * a.sc_b + row * a.ldc + h * DH;
  const T* gate = a.gate ? (const T*)a.gate + b * a.sg_b + row * a.ldg + h * DH : nullptr;
#pragma unroll
  for (int d = 0; d < DH; ++d) {
    float v = o[d] * inv;
    if (gate) v *= Elem<T>::ld(gate + d);
    Elem<T>::st(out + d, v);
  }
}

// ------------------------------------------------------------------------------------
// bf16 MFMA kernel.
// ------------------------------------------------------------------------------------
constexpr int kQB = 128;   // query rows per block of the 4-wave kernel (32 per wave)
constexpr int kKB = 64;    // keys per LDS tile

// Which instantiations run the software-pipelined loop with direct global-to-LDS staging: no bias tile to
// stage, whole key tiles only (a direct load cannot zero-fill), heads of 64 or 128.  The loop needs two
// score tiles in registers, which leaves two waves per SIMD where the plain loop has three at 64-wide
// heads; a causal launch at that width (many short blocks, three per CU co-resident) measured faster plain.
constexpr bool attention_pipelined(int dh, bool causal, bool bias, bool ragged) {
  return !bias && !ragged && (dh == 128 || (dh == 64 && !causal));
}
constexpr size_t attention_lds_bytes(int dh, bool causal, bool bias, bool ragged, int nw) {
  return attention_pipelined(dh, causal, bias, ragged)
             ? (size_t)2 * 1040 * (kKB * dh * 2 / 1024 + dh * kKB * 2 / 1024)
             : ((size_t)2 * (kKB * (dh + 8) + dh * (kKB + 8)) + (bias ? 32 * nw * (kKB + 4) : 0)) * sizeof(bf16_t);
}

// RAGGED: the key count is not a multiple of the tile (or of the 16-byte vector): loads are
// guarded and keys past the end are masked.  The other instantiation has no bounds work in
// its main loop.
template <int DH, bool CAUSAL, bool BIAS, bool RAGGED, int NW>
__global__ void __launch_bounds__(64 * NW, attention_pipelined(DH, CAUSAL, BIAS, RAGGED) ? 2 : 1) attention_mfma_bf16(AttnArgs a) {
  constexpr int NT = 64 * NW;         // threads
  constexpr int QB = 32 * NW;         // query rows per block
  constexpr int KROW = DH + 8;        // padded K row (elements): conflict-free 128-bit reads
  constexpr int VROW = kKB + 8;       // padded V^T row
  constexpr int KS = DH / 16;         // k-steps of the score MFMA
  constexpr int DT = DH / 32;         // 32-wide output tiles over d
  constexpr int K_CHUNKS = kKB * (DH / 8) / NT;   // 16-byte chunks per thread, K tile
  constexpr int V_CHUNKS = DH * (kKB / 8) / NT;   // and V^T tile
  static_assert(K_CHUNKS >= 1 && V_CHUNKS >= 1, "tile too small for the block");
  constexpr bool PIPE = attention_pipelined(DH, CAUSAL, BIAS, RAGGED);
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem_raw);     // [2][kKB][KROW]
  bf16_t* sV = sK + 2 * kKB * KROW;                      // [2][DH][VROW]
  // The bias tile [QB query rows][64 keys] of the block goes through LDS too: a lane needs 4
  // consecutive keys of ITS row, so direct loads touch 64 cache lines per instruction and the
  // kernel ends up bound by the L1's tag lookups; staged, a row's 128 bytes are one line read by
  // 8 lanes.
  constexpr int BROW = kKB + 4;                          // padded bias row (elements)
  constexpr int B_CHUNKS = BIAS ? QB * (kKB / 8) / NT : 1;
  bf16_t* sB = sV + 2 * DH * VROW;                       // [QB][BROW] (BIAS only), one buffer: the next tile waits in
                                                         // registers until every wave is done with this one

  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int l32 = lane % 32, half = lane / 32;
  const int sq = (int)a.sq, sk = (int)a.sk, q_offset = (int)a.q_offset;
  const int nqb = (sq + QB - 1) / QB;
  const int ns = a.n_splits > 1 ? a.n_splits : 1;
  const int64_t t = xcd_contiguous(blockIdx.x, gridDim.x);
  const int split = (int)(t % ns);
  const int64_t bq = t / ns;
  const int64_t bh = bq / nqb;
  int qb = (int)(bq % nqb);
  if (CAUSAL) {
    // Longest rows first, in a snake over runs of 32 (the CUs of an XCD, which take consecutive
    // blocks in turn): the first 32 blocks of a head are its longest in descending order, the next
    // 32 the following ones in ascending order, and so on, so that when all blocks of a launch are
    // resident at once (one sequence of a few thousand rows) every CU holds about the same number
    // of key tiles; with more blocks than places the order is still longest-first run by run.
    const int run = qb / 32, col = qb % 32;
    const int len = nqb - run * 32 < 32 ? nqb - run * 32 : 32;
    const int rank = run * 32 + ((run & 1) ? len - 1 - col : col);
    qb = nqb - 1 - rank;
  }
  // Problem-major order keeps the heads of one problem together (their q/k/v rows interleave in
  // memory).  Head-major order (set by the host when a bias shared by all problems is the
  // largest operand) gives each XCD a run of problems of ONE head, so that head's bias stays
  // in the XCD's L2 while keys and values stream through, instead of every problem fetching
  // every head's bias again.
  const int64_t b = a.head_major ? bh % a.batch : bh / a.heads;
  const int h = (int)(a.head_major ? bh / a.batch : bh % a.heads);
  const int q0 = qb * QB;

  const bf16_t* kbase = (const bf16_t*)a.k + b * a.sk_b + h * DH;
  const bf16_t* vbase = (const bf16_t*)a.v + b * a.sv_b + (int64_t)h * DH * a.ldv;

  // this lane's query row (clamped; clamped rows compute but never store)
  const int row = q0 + wave * 32 + l32;
  const int rowc = row < sq ? row : sq - 1;
  const int qpos = q_offset + rowc;
  bf16x8 qf[KS];
  {
    const bf16_t* qp = (const bf16_t*)a.q + b * a.sq_b + (int64_t)rowc * a.ldq + h * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }
  // bias chunk i of this thread: row b_row[i] of the block's query rows, keys b_col[i] .. +8 of the tile
  const bf16_t* b_src[B_CHUNKS];
  int b_dst[B_CHUNKS], b_col[B_CHUNKS];
  if (BIAS) {
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
      const int c = tid + NT * i, br = c / (kKB / 8);
      b_col[i] = (c % (kKB / 8)) * 8;
      int gr = q0 + br; if (gr > sq - 1) gr = sq - 1;
      b_src[i] = (const bf16_t*)a.bias + h * a.s_bias_h + (int64_t)gr * a.ld_bias + b_col[i];
      b_dst[i] = br * BROW + b_col[i];
    }
  }

  int kv_end = sk;
  if (CAUSAL) {
    int last = q0 + QB - 1; if (last > sq - 1) last = sq - 1;
    if (q_offset + last + 1 < kv_end) kv_end = q_offset + last + 1;
  }
  const int n_tiles_all = (kv_end + kKB - 1) / kKB;
  // this block's share of the key tiles: split s takes tiles [s * per, (s + 1) * per)
  const int per_split = (n_tiles_all + ns - 1) / ns;
  const int tile_lo = split * per_split;
  const int tile_hi = tile_lo + per_split < n_tiles_all ? tile_lo + per_split : n_tiles_all;
  // last key position any row of this wave may see, first row of the wave (wave-uniform)
  int wave_last = q0 + wave * 32 + 31; if (wave_last > sq - 1) wave_last = sq - 1;
  wave_last += q_offset;
  const int wave_first = q_offset + q0 + wave * 32;
  const bool wave_active = q0 + wave * 32 < sq;   // waves past the last query row only help staging

  // staging: which chunks of a K tile / V^T tile this thread moves.  A V^T chunk (8 keys of
  // one d row) is stored as two 8-byte halves, permuted inside its 16-key group to the slot
  // order [0-3, 8-11, 4-7, 12-15], so that the 8 keys one lane feeds to a PV MFMA are 16
  // contiguous bytes.
  int k_row[K_CHUNKS], k_col[K_CHUNKS], v_row[V_CHUNKS], v_col[V_CHUNKS];
  const bf16_t* k_src[K_CHUNKS];
  const bf16_t* v_src[V_CHUNKS];
  int k_dst[K_CHUNKS], v_dst[V_CHUNKS];
#pragma unroll
  for (int i = 0; i < K_CHUNKS; ++i) {
    const int c = tid + NT * i;
    k_row[i] = c / (DH / 8); k_col[i] = (c % (DH / 8)) * 8;
    k_src[i] = kbase + (int64_t)k_row[i] * a.ldk + k_col[i];
    k_dst[i] = k_row[i] * KROW + k_col[i];
  }
#pragma unroll
  for (int i = 0; i < V_CHUNKS; ++i) {
    const int c = tid + NT * i;
    v_row[i] = c / (kKB / 8);
    const int ch = c % (kKB / 8);
    v_col[i] = ch * 8;
    v_src[i] = vbase + (int64_t)v_row[i] * a.ldv + v_col[i];
    v_dst[i] = v_row[i] * VROW + (ch / 2) * 16 + (ch % 2) * 4;
  }
  bf16x8 k_reg[K_CHUNKS], v_reg[V_CHUNKS], b_reg[B_CHUNKS];

  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < K_CHUNKS; ++i) {
      if (RAGGED) {
        int key = k0 + k_row[i]; if (key > sk - 1) key = sk - 1;
        k_reg[i] = *reinterpret_cast<const bf16x8*>(kbase + (int64_t)key * a.ldk + k_col[i]);
      } else {
        k_reg[i] = *reinterpret_cast<const bf16x8*>(k_src[i] + (int64_t)k0 * a.ldk);
      }
    }
#pragma unroll
    for (int i = 0; i < V_CHUNKS; ++i) {
      const bf16_t* src = v_src[i] + k0;
      if (!RAGGED) {
        v_reg[i] = *reinterpret_cast<const bf16x8*>(src);
      } else {   // zero-fill past the end so that 0 * v stays 0
        const int key = k0 + v_col[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) v_reg[i][j] = key + j < sk ? src[j] : (bf16_t)0.0f;
      }
    }
    if (BIAS) {
#pragma unroll
      for (int i = 0; i < B_CHUNKS; ++i) {
        const bf16_t* src = b_src[i] + k0;
        if (!RAGGED) {
          b_reg[i] = *reinterpret_cast<const bf16x8*>(src);
        } else {   // keys past the end are masked later; stage zeros for them
          const int key = k0 + b_col[i];
#pragma unroll
          for (int j = 0; j < 8; ++j) b_reg[i][j] = key + j < sk ? src[j] : (bf16_t)0.0f;
        }
      }
    }
  };
  auto store_tile = [&](int buf) {
    bf16_t* dk = sK + buf * kKB * KROW;
    bf16_t* dv = sV + buf * DH * VROW;
#pragma unroll
    for (int i = 0; i < K_CHUNKS; ++i) *reinterpret_cast<bf16x8*>(dk + k_dst[i]) = k_reg[i];
#pragma unroll
    for (int i = 0; i < V_CHUNKS; ++i) {
      const bf16x4 lo = {v_reg[i][0], v_reg[i][1], v_reg[i][2], v_reg[i][3]};
      const bf16x4 hi = {v_reg[i][4], v_reg[i][5], v_reg[i][6], v_reg[i][7]};
      *reinterpret_cast<bf16x4*>(dv + v_dst[i]) = lo;
      *reinterpret_cast<bf16x4*>(dv + v_dst[i] + 8) = hi;
    }
    if (BIAS) {
      bf16_t* db = sB;
#pragma unroll
      for (int i = 0; i < B_CHUNKS; ++i) {
        const bf16x4 lo = {b_reg[i][0], b_reg[i][1], b_reg[i][2], b_reg[i][3]};
        const bf16x4 hi = {b_reg[i][4], b_reg[i][5], b_reg[i][6], b_reg[i][7]};
        *reinterpret_cast<bf16x4*>(db + b_dst[i]) = lo;       // (rows are 8-byte aligned, not 16)
        *reinterpret_cast<bf16x4*>(db + b_dst[i] + 4) = hi;
      }
    }
  };

  f32x16 acc_o[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[i][r] = 0.f;
  // running maximum (of scale2 * score [+ bias]) and sum, both in the log2 domain
  float m_run = -INFINITY, l_run = 0.f;
  const float scale2 = rsqrtf((float)DH) * kLog2e;

  if constexpr (!PIPE) {
    if (tile_lo < tile_hi) { load_tile(tile_lo * kKB); store_tile(tile_lo & 1); }
    __syncthreads();

    for (int kt = tile_lo; kt < tile_hi; ++kt) {
      const int buf = kt & 1;
      const int k0 = kt * kKB;
      const bool more = kt + 1 < tile_hi;
      if (more) load_tile(k0 + kKB);

      if (wave_active && (!CAUSAL || k0 <= wave_last)) {
        // ---- S^T = K Q^T for two 32-key tiles
        f32x16 acc_s[2];
        const bf16_t* ck = sK + buf * kKB * KROW + l32 * KROW + half * 8;
  #pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
  #pragma unroll
          for (int r = 0; r < 16; ++r) acc_s[tt][r] = 0.f;
  #pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ck + tt * 32 * KROW + ks * 16);
            acc_s[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[tt], 0, 0, 0);
          }
        }
        // ---- lane holds keys k0 + tt*32 + 8*(r/4) + 4*half + r%4.  Scores go to the log2 domain
        // only where needed: with a bias right away, otherwise folded into the exponent below.
        if (BIAS) {
          const bf16_t* cb = sB + (wave * 32 + l32) * BROW + 4 * half;
  #pragma unroll
          for (int tt = 0; tt < 2; ++tt)
  #pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
              const bf16x4 bb = *reinterpret_cast<const bf16x4*>(cb + tt * 32 + 8 * g4);
  #pragma unroll
              for (int j = 0; j < 4; ++j)
                acc_s[tt][4 * g4 + j] = fmaf(acc_s[tt][4 * g4 + j], scale2, bf2f(bb[j]) * kLog2e);
            }
        }
        const bool need_mask = (RAGGED && k0 + kKB > sk) || (CAUSAL && k0 + kKB - 1 > wave_first);
        if (need_mask) {
  #pragma unroll
          for (int tt = 0; tt < 2; ++tt)
  #pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int kj = k0 + tt * 32 + 8 * (r / 4) + 4 * half + (r % 4);
              if ((RAGGED && kj >= sk) || (CAUSAL && kj > qpos)) acc_s[tt][r] = -INFINITY;
            }
        }
        float mx = acc_s[0][0];
  #pragma unroll
        for (int tt = 0; tt < 2; ++tt)
  #pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[tt][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if (!BIAS) mx *= scale2;                       // scale2 > 0: max commutes with the scaling
        // rescale only when some row of the wave saw a new maximum
        if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {
          const float m_new = fmaxf(m_run, mx);
          const float alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
          m_run = m_new;
          l_run *= alpha;
  #pragma unroll
          for (int i = 0; i < DT; ++i)
  #pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
        }
        float psum = 0.f;
        bf16x8 pf[2][2];
  #pragma unroll
        for (int tt = 0; tt < 2; ++tt)
  #pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float e = BIAS ? acc_s[tt][r] - m_run : fmaf(acc_s[tt][r], scale2, -m_run);
            const float p = __builtin_amdgcn_exp2f(e);
            psum += p;
            pf[tt][r / 8][r % 8] = f2bf(p);
          }
        l_run += psum;
        // ---- O^T += V^T P^T
        const bf16_t* cv = sV + buf * DH * VROW + l32 * VROW + 8 * half;
  #pragma unroll
        for (int i = 0; i < DT; ++i)
  #pragma unroll
          for (int tt = 0; tt < 2; ++tt)
  #pragma unroll
            for (int u = 0; u < 2; ++u) {
              const bf16x8 vf = *reinterpret_cast<const bf16x8*>(cv + i * 32 * VROW + (tt * 2 + u) * 16);
              acc_o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[tt][u], acc_o[i], 0, 0, 0);
            }
      }
      if (BIAS && more) __syncthreads();   // the single bias buffer is overwritten next: every wave has read it
      if (more) store_tile(buf ^ 1);
      __syncthreads();
    }

  } else {
    // Software-pipelined loop.  The matrix instructions of the NEXT tile's scores are issued among
    // the exponentials of THIS tile, and this tile's probability-value products among the maximum of
    // the next: a SIMD overlaps the matrix and the vector instructions of one wave far better than
    // those of two different waves, and at 64- and 128-wide heads the two kinds of work are about
    // equal.  K is therefore staged one tile ahead of V: iteration kt reads K(kt+1) and V(kt) while
    // K(kt+2) and V(kt+1) arrive.
    //
    // Tiles come in by direct global-to-LDS loads (no staging registers, no LDS store instructions):
    // one wave instruction moves 64 x 16 bytes into 1 KB of consecutive LDS, i.e. RPI whole rows of
    // the tile.  Row r goes to group r % G at index r / G, and groups are 1 KB + 16 bytes apart, so
    // any 8 consecutive lanes of a fragment read (8 consecutive rows, same 16-byte column) fall into 8
    // different 16-byte slots modulo 128 bytes, which is what makes a 128-bit LDS read conflict free.
    constexpr int GB = 1040;                       // bytes from one group to the next
    constexpr int KRB = DH * 2;                    // bytes per K row
    constexpr int KG = kKB * KRB / 1024;           // groups (load instructions) per K tile: 16 or 8
    constexpr int VRB = kKB * 2;                   // bytes per V^T row
    constexpr int VG = DH * VRB / 1024;            // groups per V^T tile: 16 or 8
    static_assert((KG == 16 || (KG == 8 && KRB == 128)) && (VG == 16 || VG == 8), "row-to-group rule needs 8 or 16 groups");
    static_assert(KG % NW == 0 && VG % NW == 0, "groups are dealt to the waves in turn");
    constexpr int KBUF = KG * GB, VBUF = VG * GB;  // bytes per buffer
    unsigned char* const sKb = smem_raw;           // [2][KBUF]
    unsigned char* const sVb = smem_raw + 2 * KBUF;   // [2][VBUF]
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    // Global source of a load instruction: a wave-uniform base (scalar registers; advanced per tile and per
    // instruction) plus this lane's byte offset inside the wave's first group.
    // (K rows sit in LDS in the order the lanes of a score MFMA read them: LDS row x holds key swap23(x), see below)
    auto swap23 = [](int x) { return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1); };
    const uint32_t kg_off = (uint32_t)(swap23((lane / (KRB / 16)) * KG + wave) * (int)a.ldk + (lane % (KRB / 16)) * 8) * 2u;
    // (with 16 groups a V^T group holds 8 rows that are 16 apart; they sit in it in the order v_slot() gives, so
    // that rows l and l + 16, which the two quarter-waves of a fragment read fetch together, are 256 bytes apart
    // and the 32 lanes fall into 32 different 16-byte slots modulo 512 bytes)
    auto v_row_of_slot = [](int x) { return VG == 16 ? 2 * ((x & 1) + 2 * (x >> 2)) + ((x >> 1) & 1) : x; };
    const uint32_t vg_off = (uint32_t)((v_row_of_slot(lane / (VRB / 16)) * VG + wave) * (int)a.ldv + (lane % (VRB / 16)) * 8) * 2u;
    auto uniform = [](const void* ptr) {
      const uint64_t v = (uint64_t)ptr;
      const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
      return (const unsigned char*)(((uint64_t)hi << 32) | lo);
    };
    const unsigned char* const kg_base = uniform(kbase);
    const unsigned char* const vg_base = uniform(vbase);
    auto dma_k = [&](int kt, int buf) {
      const unsigned char* src = kg_base + (int64_t)kt * kKB * a.ldk * 2;
#pragma unroll
      for (int j = 0; j < KG / NW; ++j)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (int64_t)swap23(j * NW) * a.ldk * 2 + kg_off),
                                         (__attribute__((address_space(3))) void*)(sKb + buf * KBUF + (wave_u + NW * j) * GB), 16, 0, 0);
    };
    auto dma_v = [&](int kt, int buf) {
      const unsigned char* src = vg_base + (int64_t)kt * kKB * 2;
#pragma unroll
      for (int j = 0; j < VG / NW; ++j)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (int64_t)j * NW * a.ldv * 2 + vg_off),
                                         (__attribute__((address_space(3))) void*)(sVb + buf * VBUF + (wave_u + NW * j) * GB), 16, 0, 0);
    };
    auto arrived = [&]() {   // this wave's loads have landed, then every wave's
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
      __syncthreads();
    };

    // The score MFMA takes key pi(m) of a 32-key half as its row m, pi = m with bits 2 and 3 swapped:
    // a lane's accumulator registers 8u .. 8u+7 then hold the 8 CONSECUTIVE keys 16u + 8 half + (0..7),
    // so the probabilities go to the second MFMA as they are and its V^T fragment is one 16-byte read
    // of an unpermuted row.
    // K is laid out in LDS by MFMA row, not by key (LDS row x = key pi(x) of the tile), so that here too 8
    // consecutive lanes read 8 different 16-byte slots modulo 128 bytes.
    const unsigned char* const k_frag = sKb + (l32 % KG) * GB + (l32 / KG) * KRB + half * 16;
    const unsigned char* const v_frag = sVb + (l32 % VG) * GB + (VG == 16 ? 2 * (l32 / 16) : l32 / VG) * VRB + half * 16;

    int w_hi = tile_hi;                               // this wave computes tiles [tile_lo, w_hi)
    if (CAUSAL) { const int vis = wave_last / kKB + 1; if (vis < w_hi) w_hi = vis; }
    if (!wave_active) w_hi = tile_lo;
    float m_exp = 0.f;   // m_run, or 0 while the row has seen no key: exp2(-inf - m_exp) is then 0, not NaN

    // S^T = K Q^T of the tile in K buffer `buf`, one 32-key half after the other
    auto scores = [&](f32x16 (&s)[2], int buf) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[tt][r] = 0.f;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(k_frag + buf * KBUF + tt * (32 / KG) * KRB + ks * 32);
          s[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[tt], 0, 0, 0);
        }
    };
    auto needs_mask = [&](int kt) { return CAUSAL && kt * kKB + kKB - 1 > wave_first; };
    auto mask = [&](f32x16 (&s)[2], int kt) {
      const int k0 = kt * kKB;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kj = k0 + tt * 32 + 16 * (r / 8) + 8 * half + 4 * ((r / 4) % 2) + (r % 4);
          if (kj > qpos) s[tt][r] = -INFINITY;
        }
    };
    // the running maximum takes in a tile's largest score per lane; the accumulators are rescaled only when
    // some row of the wave saw a new maximum
    auto new_max = [&](float mx) {
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      mx *= scale2;                                  // scale2 > 0: max commutes with the scaling
      if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        m_exp = m_new == -INFINITY ? 0.f : m_new;
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
      }
    };
    auto take_max = [&](const f32x16 (&s)[2]) {
      float mx = s[0][0];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[tt][r]);
      new_max(mx);
    };
    // One tile of this wave: probabilities of `cur` (whose maximum m_run already holds), their products with the
    // V^T tile in V buffer `buf`, and meanwhile the scores of the next tile, in K buffer `buf ^ 1`, into `next`.
    // The order of issue is written out and pinned group by group (nothing crosses a scheduling barrier): one
    // matrix instruction, the read of the fragment PD instructions ahead, and a share of the vector work -
    // exponentials of this tile at a steady rate that has each quarter of the probabilities ready before the
    // products that consume it, then the maximum of the next tile's scores once those are complete.
    auto step = [&](auto has_next, auto mask_next, f32x16 (&cur)[2], f32x16 (&next)[2], int kt, int buf) {
      constexpr bool NEXT = decltype(has_next)::value, MASK = decltype(mask_next)::value;
      // (the three instantiations begin alike; an empty statement that differs keeps the compiler from
      // moving their common exponentials out in front of the branch, away from the matrix instructions)
      asm volatile("; tile step %c1" : "+v"(m_exp) : "n"(2 * (int)NEXT + (int)MASK));
      constexpr int NQK = NEXT ? 2 * KS : 0, NPV = 4 * DT, N = NQK + NPV, PD = DH >= 128 ? 4 : 2;
      constexpr int EXPD = NQK + 3 * DT - 1;   // the 32 exponentials are spread evenly over the groups before the last quarter's products
      constexpr int MAX0 = NQK + 2;                                   // first group that may read `next`
      constexpr int MAXS = (16 + N - MAX0 - 1) / (N - MAX0);          // pairs of scores per group for the maximum
      const unsigned char* const kf_base = k_frag + (buf ^ 1) * KBUF;
      const unsigned char* const vf_base = v_frag + buf * VBUF;
      auto frag = [&](int j) {
        if (j < NQK) return *reinterpret_cast<const bf16x8*>(kf_base + (j / KS) * (32 / KG) * KRB + (j % KS) * 32);
        const int pq = (j - NQK) / DT, i = (j - NQK) % DT;
        return *reinterpret_cast<const bf16x8*>(vf_base + (VG == 16 ? (i & 1) + 4 * (i >> 1) : i * (32 / VG)) * VRB + pq * 32);
      };
      if (NEXT) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int r = 0; r < 16; ++r) next[tt][r] = 0.f;
      }
      bf16x8 fr[PD];
#pragma unroll
      for (int j = 0; j < PD; ++j) fr[j] = frag(j);
      float psum = 0.f, mx = 0.f;
      bf16x8 pf[2][2];
      int e_done = 0, m_done = 0;
      auto exponential = [&](int e) {
        const int tt = e / 16, r = e % 16;
        const float p = __builtin_amdgcn_exp2f(fmaf(cur[tt][r], scale2, -m_exp));
        psum += p;
        pf[tt][r / 8][r % 8] = f2bf(p);
      };
      if (!NEXT) {   // the wave's last tile: nothing to hide the exponentials under
#pragma unroll
        for (int e = 0; e < 32; ++e) exponential(e);
        e_done = 32;
      }
#pragma unroll
      for (int j = 0; j < N; ++j) {
        if (j < NQK) {
          next[j / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % PD], qf[j % KS], next[j / KS], 0, 0, 0);
        } else {
          const int pq = (j - NQK) / DT, i = (j - NQK) % DT;
          acc_o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % PD], pf[pq / 2][pq % 2], acc_o[i], 0, 0, 0);
        }
        if (j + PD < N) fr[j % PD] = frag(j + PD);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (e_done < 32 && e_done < (j + 1) * 32 / EXPD) exponential(e_done++);
        }
        if (NEXT && !MASK && j >= MAX0) {
#pragma unroll
          for (int c = 0; c < MAXS; ++c) {
            if (m_done < 16) {
              const float s0 = next[m_done / 8][2 * (m_done % 8)], s1 = next[m_done / 8][2 * (m_done % 8) + 1];
              mx = m_done == 0 ? fmaxf(s0, s1) : fmaxf(fmaxf(mx, s0), s1);
              ++m_done;
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      l_run += psum;
      if constexpr (NEXT) {
        if constexpr (MASK) {
          mask(next, kt + 1);
          mx = next[0][0];
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, next[tt][r]);
        }
        new_max(mx);
      }
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    // buf = (kt - tile_lo) % 2: K(kt) and V(kt) are in buffers `buf`, K(kt+1) in `buf ^ 1`
    auto iteration = [&](f32x16 (&cur)[2], f32x16 (&next)[2], int kt, int buf) {
      if (kt + 2 < tile_hi) dma_k(kt + 2, buf);          // K(kt) was last read in the iteration before
      if (kt + 1 < tile_hi) dma_v(kt + 1, buf ^ 1);      // and so was V(kt-1)
      if (kt < w_hi) {
        if (kt + 1 >= w_hi) step(no{}, no{}, cur, next, kt, buf);
        else if (needs_mask(kt + 1)) step(yes{}, yes{}, cur, next, kt, buf);
        else step(yes{}, no{}, cur, next, kt, buf);
      }
      arrived();
    };

    f32x16 s_a[2], s_b[2];
    if (tile_lo < tile_hi) {
      dma_k(tile_lo, 0); dma_v(tile_lo, 0);
      if (tile_lo + 1 < tile_hi) dma_k(tile_lo + 1, 1);
    }
    arrived();
    if (tile_lo < w_hi) {
      scores(s_a, 0);
      if (needs_mask(tile_lo)) mask(s_a, tile_lo);
      take_max(s_a);
    }
    __syncthreads();   // K(tile_lo)'s buffer is written again from the first iteration on
    for (int kt = tile_lo; kt < tile_hi; kt += 2) {
      iteration(s_a, s_b, kt, 0);
      if (kt + 1 < tile_hi) iteration(s_b, s_a, kt + 1, 1);
    }
  }

  if (row >= sq) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (ns > 1) {
    // partial result of this key split: unnormalised O (fp32), running max and sum
    const int64_t prow = ((int64_t)split * a.batch + b) * sq + row;
    float* po = (float*)a.part_o + (prow * a.heads + h) * DH;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int d = i * 32 + 8 * g4 + 4 * half;
        const f32x4 o = {acc_o[i][4 * g4], acc_o[i][4 * g4 + 1], acc_o[i][4 * g4 + 2], acc_o[i][4 * g4 + 3]};
        *reinterpret_cast<f32x4*>(po + d) = o;
      }
    if (half == 0) {
      float* pml = (float*)a.part_ml + (prow * a.heads + h) * 2;
      pml[0] = m_run;
      pml[1] = l_tot;
    }
    return;
  }
  const float inv = 1.0f / l_tot;
  bf16_t* out = (bf16_t*)a.ctx + b * a.sc_b + (int64_t)row * a.ldc + h * DH;
  const bf16_t* gate = a.gate ? (const bf16_t*)a.gate + b * a.sg_b + (int64_t)row * a.ldg + h * DH : nullptr;
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int d = i * 32 + 8 * g4 + 4 * half;
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = acc_o[i][4 * g4 + j] * inv;
      if (gate) {
        const bf16x4 gg = *reinterpret_cast<const bf16x4*>(gate + d);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] *= bf2f(gg[j]);
      }
      const bf16x4 o = {f2bf(v[0]), f2bf(v[1]), f2bf(v[2]), f2bf(v[3])};
      *reinterpret_cast<bf16x4*>(out + d) = o;
    }
}

// Merge of the key splits: ctx = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M) [* gate].
// One thread per (problem, row, head, 4 consecutive d).
__global__ void __launch_bounds__(256) attention_merge_splits(AttnArgs a) {
  const int dh4 = a.head_dim / 4;
  const int64_t total = a.batch * a.sq * a.heads * dh4;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int d = (int)(i % dh4) * 4;
  const int64_t rh = i / dh4;                  // (b * sq + row) * heads + h
  const int h = (int)(rh % a.heads);
  const int64_t br = rh / a.heads;
  const int64_t row = br % a.sq, b = br / a.sq;
  const int64_t stride = a.batch * a.sq * a.heads;   // (row, head) pairs per split
  // all loads of a thread are issued before the first use (at most 16 splits), so their
  // latencies overlap instead of adding up
  constexpr int kMaxSplits = 16;
  const float* ml = (const float*)a.part_ml;
  const float* po = (const float*)a.part_o;
  f32x2 mls[kMaxSplits];
  f32x4 os[kMaxSplits];
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) {
    if (s < a.n_splits) {
      mls[s] = *reinterpret_cast<const f32x2*>(ml + (s * stride + rh) * 2);
      os[s] = *reinterpret_cast<const f32x4*>(po + (s * stride + rh) * a.head_dim + d);
    } else {
      mls[s] = f32x2{-INFINITY, 0.f};
      os[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) M = fmaxf(M, mls[s][0]);
  float L = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) {
    // a split that saw no key of this row reports m = -inf; its sum and context are not
    // meaningful (the kernel may have formed inf - inf there) and must not be touched
    if (mls[s][0] != -INFINITY) {
      const float w = __builtin_amdgcn_exp2f(mls[s][0] - M);
      L += mls[s][1] * w;
      acc += os[s] * w;
    }
  }
  const float inv = 1.0f / L;
  float v[4] = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
  if (a.gate) {
    const bf16x4 gg = *reinterpret_cast<const bf16x4*>((const bf16_t*)a.gate + b * a.sg_b + row * a.ldg + h * a.head_dim + d);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] *= bf2f(gg[j]);
  }
  const bf16x4 o = {f2bf(v[0]), f2bf(v[1]), f2bf(v[2]), f2bf(v[3])};
  *reinterpret_cast<bf16x4*>((bf16_t*)a.ctx + b * a.sc_b + row * a.ldc + h * a.head_dim + d) = o;
}

template <int DH, bool CAUSAL, bool BIAS, bool RAGGED, int NW>
static hipError_t mfma_attn_launch(const AttnArgs& a, hipStream_t s) {
  auto kern = attention_mfma_bf16<DH, CAUSAL, BIAS, RAGGED, NW>;
  constexpr size_t lds = attention_lds_bytes(DH, CAUSAL, BIAS, RAGGED, NW);
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (attr_status != hipSuccess) return attr_status;
  const int64_t nqb = (a.sq + 32 * NW - 1) / (32 * NW);
  const int ns = a.n_splits > 1 ? a.n_splits : 1;
  const int64_t blocks = nqb * a.heads * a.batch * ns;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * NW), lds, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || ns == 1) return e;
  const int64_t items = a.batch * a.sq * a.heads * (DH / 4);
  hipLaunchKernelGGL(attention_merge_splits, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

template <int DH, bool CAUSAL, bool BIAS>
static hipError_t mfma_attn_ragged(const AttnArgs& a, hipStream_t s) {
  // 64-row blocks (2 waves) when a problem has at most 64 query rows, so that no wave idles
  if (a.sq <= 64) {
    if (a.sk % kKB != 0) return mfma_attn_launch<DH, CAUSAL, BIAS, true, 2>(a, s);
    return mfma_attn_launch<DH, CAUSAL, BIAS, false, 2>(a, s);
  }
  if (a.sk % kKB != 0) return mfma_attn_launch<DH, CAUSAL, BIAS, true, 4>(a, s);
  // 256-row blocks (8 waves, one block per CU) when the launch has rounds of them to spare: a K / V^T tile
  // then serves twice the query rows, which halves the tile loads of the pipelined loop (measured +2.5 %)
  if constexpr (attention_pipelined(DH, CAUSAL, BIAS, false)) {
    if (a.n_splits <= 1 && ((a.sq + 255) / 256) * a.heads * a.batch >= 1024) return mfma_attn_launch<DH, CAUSAL, BIAS, false, 8>(a, s);
  }
  return mfma_attn_launch<DH, CAUSAL, BIAS, false, 4>(a, s);
}

template <int DH>
static hipError_t mfma_attn_dispatch(const AttnArgs& a, hipStream_t s) {
  if (a.causal) {
    if (a.bias) return mfma_attn_ragged<DH, true, true>(a, s);
    return mfma_attn_ragged<DH, true, false>(a, s);
  }
  if (a.bias) return mfma_attn_ragged<DH, false, true>(a, s);
  return mfma_attn_ragged<DH, false, false>(a, s);
}

static bool al(const void* p, uintptr_t n) { return p == nullptr || ((uintptr_t)p % n) == 0; }

static bool mfma_attn_eligible(const AttnArgs& a) {
  if (a.dtype != AC_BF16 || !a.v_transposed) return false;
  if (a.head_dim != 32 && a.head_dim != 64 && a.head_dim != 128) return false;
  if (a.ldq % 8 || a.ldk % 8 || a.ldv % 8 || a.sq_b % 8 || a.sk_b % 8 || a.sv_b % 8) return false;
  if (a.ldk >= (1 << 24) || a.ldv >= (1 << 24)) return false;   // a tile's rows are addressed with 32-bit byte offsets
  if (a.ldc % 4 || a.sc_b % 4) return false;
  if (!al(a.q, 16) || !al(a.k, 16) || !al(a.v, 16) || !al(a.ctx, 8)) return false;
  if (a.bias && (a.sk % 4 || a.ld_bias % 8 || a.s_bias_h % 8 || !al(a.bias, 16))) return false;   // 16-byte bias chunks
  if (a.gate && (a.ldg % 4 || a.sg_b % 4 || !al(a.gate, 8))) return false;
  return true;
}

template <typename T>
static hipError_t generic_attn_dispatch(const AttnArgs& a, hipStream_t s) {
  dim3 grid((unsigned)((a.sq + 127) / 128), (unsigned)a.heads, (unsigned)a.batch);
  switch (a.head_dim) {
    case 8: hipLaunchKernelGGL((attention_rows<T, 8>), grid, dim3(128), 0, s, a); break;
    case 16: hipLaunchKernelGGL((attention_rows<T, 16>), grid, dim3(128), 0, s, a); break;
    case 32: hipLaunchKernelGGL((attention_rows<T, 32>), grid, dim3(128), 0, s, a); break;
    case 64: hipLaunchKernelGGL((attention_rows<T, 64>), grid, dim3(128), 0, s, a); break;
    case 128: hipLaunchKernelGGL((attention_rows<T, 128>), grid, dim3(128), 0, s, a); break;
    default: return hipErrorNotSupported;
  }
  return hipGetLastError();
}

// Key splits for a launch that would leave most of the 256 CUs idle: as many as still give
// every block a place at once, which by register count is three blocks per CU, two with
// 128-wide heads (a launch that spills into a second round leaves those blocks to run alone
// at the end, at a fraction of the CU's rate), each split at least 512 keys long.  A pure
// function of the launch shape, so planning and execution agree.
int attention_key_splits(int64_t sq, int64_t sk, int heads, int64_t batch, int head_dim, int dtype, int v_transposed) {
  if (dtype != AC_BF16 || !v_transposed) return 1;
  if (head_dim != 32 && head_dim != 64 && head_dim != 128) return 1;
  const int64_t blocks = ((sq + kQB - 1) / kQB) * heads * batch;
  if (blocks <= 0 || blocks >= 512 || sk < 1024) return 1;
  int64_t want = (head_dim > 64 ? 512 : 768) / blocks;
  const int64_t by_len = sk / 512;
  if (want > by_len) want = by_len;
  if (want > 16) want = 16;
  return want < 1 ? 1 : (int)want;
}

uint64_t attention_split_workspace_bytes(int64_t sq, int heads, int64_t batch, int head_dim, int n_splits) {
  if (n_splits <= 1) return 0;
  const uint64_t rh = (uint64_t)n_splits * batch * sq * heads;
  return rh * head_dim * 4 + rh * 2 * 4;
}

hipError_t launch_attention(const AttnArgs& a_in, hipStream_t s) {
  AttnArgs a = a_in;
  // bytes of one head's bias against the keys and values of one (problem, head): whichever is
  // larger should be what consecutive blocks share
  a.head_major = a.bias != nullptr && a.batch > 1 && a.sq > 2 * (int64_t)a.head_dim;
  if (a.n_splits > 1 && (!a.part_o || !a.part_ml || !mfma_attn_eligible(a))) a.n_splits = 1;
  if (a.batch <= 0 || a.sq <= 0 || a.heads <= 0) return hipSuccess;
  if (a.sk <= 0 || a.sk > (1 << 30) || a.sq > (1 << 30) || a.q_offset > (1 << 30)) return hipErrorInvalidValue;
  if (mfma_attn_eligible(a)) {
    switch (a.head_dim) {
      case 32: return mfma_attn_dispatch<32>(a, s);
      case 64: return mfma_attn_dispatch<64>(a, s);
      default: return mfma_attn_dispatch<128>(a, s);
    }
  }
  if (a.dtype == AC_BF16) return generic_attn_dispatch<bf16_t>(a, s);
  return generic_attn_dispatch<float>(a, s);
}

}  // namespace ac
