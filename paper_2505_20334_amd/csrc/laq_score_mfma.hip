// bf16 scoring path on the matrix cores (gfx950, v_mfma_f32_32x32x16_bf16).
//
// For one KV head the logits of Eq. 4's observation window form a skinny product
// S = Q_g K^T with R = G*W rows (the group's query heads x the cached window queries)
// and L columns.  A workgroup of four waves holds CHUNK_ROWS key rows in LDS and walks
// them in 32-key tiles:
//
//   pass 1 (statistics):  D = K_tile * Q^T, so a lane owns one score row and 16 keys of
//           the tile; it keeps a running (max, sum-exp) for its row.  The two lanes that
//           share a row and the waves that share a row tile are merged through LDS and the
//           chunk's (m, z) per row is published.
//   pass 2 (normalise + sum): D = Q * K_tile^T, so a lane owns one key and 16 rows; with the
//           row constants c = M + log2 Z the probabilities exp2(s - c) are summed over the rows
//           in-lane, across the two lane halves with one cross-lane add and across row tiles
//           through LDS, and the raw score of every key of the chunk is written.
//
// The A and B operands of the 32x32x16 instruction have the same lane layout (lane l
// supplies row/column l%32 and the 8 consecutive reduction elements l/32), so the same
// registers serve both passes with the operands swapped.
//
// The fused kernel keeps a chunk's keys in LDS from pass 1 to pass 2, so K is read from HBM
// once; the chunks of a head exchange their statistics in between (see below).
#include "laq_internal.h"

namespace laq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float NEG_BIG = -1.0e30f;
constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int KTILES = CHUNK_ROWS / 32;

// LDS row stride: the key row plus 16 bytes, so that the 16 lanes of a 128-bit LDS read
// phase (rows r .. r+15, same column) fall on 16 distinct 4-bank groups.
template <int D> struct Tile {
  static constexpr int ROWB = D * 2 + 16;
  static constexpr int KSTEPS = D / 16;
  static constexpr int PIECES_PER_ROW = D / 8;                         // 16-byte pieces
  static constexpr int PIECES_PER_THREAD = CHUNK_ROWS * PIECES_PER_ROW / THREADS;
  static constexpr int K_BYTES = CHUNK_ROWS * ROWB;
};

template <int D, int NRT> struct Smem {
  static constexpr int OFF_STAT = Tile<D>::K_BYTES;                    // float2[THREADS]
  static constexpr int OFF_SLOT = OFF_STAT + THREADS * 8;              // float[NRT][CHUNK_ROWS]
  static constexpr int BYTES = OFF_SLOT + NRT * CHUNK_ROWS * 4;
};

#define LAQ_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Key rows j0 .. j0+CHUNK_ROWS-1 of one head into registers (128-bit coalesced loads), then
// into LDS.  Rows beyond L-1 repeat row L-1: they are masked out of the statistics and their
// scores are never written.
template <int D>
__device__ __forceinline__ void fetch_chunk(uint4 (&buf)[Tile<D>::PIECES_PER_THREAD],
                                            const uint16_t* __restrict__ khead, int j0, int L, int tid) {
  using T = Tile<D>;
#pragma unroll
  for (int it = 0; it < T::PIECES_PER_THREAD; ++it) {
    const int p = tid + THREADS * it;
    const int row = p / T::PIECES_PER_ROW, col = p % T::PIECES_PER_ROW;
    const int j = min(j0 + row, L - 1);
    buf[it] = *reinterpret_cast<const uint4*>(khead + (size_t)j * D + col * 8);
  }
}

template <int D>
__device__ __forceinline__ void commit_chunk(char* ldsK, const uint4 (&buf)[Tile<D>::PIECES_PER_THREAD], int tid) {
  using T = Tile<D>;
#pragma unroll
  for (int it = 0; it < T::PIECES_PER_THREAD; ++it) {
    const int p = tid + THREADS * it;
    const int row = p / T::PIECES_PER_ROW, col = p % T::PIECES_PER_ROW;
    *reinterpret_cast<uint4*>(ldsK + row * T::ROWB + col * 16) = buf[it];
  }
}

// Operand registers of one 32-row tile of Q_g (rows beyond R are zero).
template <int D>
__device__ __forceinline__ void load_q_tile(bf16x8 (&qreg)[Tile<D>::KSTEPS], const uint16_t* __restrict__ qg,
                                            int rt, int R, int lane) {
  const int r = rt * 32 + (lane & 31);
#pragma unroll
  for (int t = 0; t < Tile<D>::KSTEPS; ++t) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < R) v = *reinterpret_cast<const uint4*>(qg + (size_t)r * D + (2 * t + (lane >> 5)) * 8);
    qreg[t] = __builtin_bit_cast(bf16x8, v);
  }
}

__device__ __forceinline__ bf16x8 lds_operand(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }

// acc = (KEYS_AS_ROWS ? K_tile * Q^T : Q * K_tile^T) + init over the whole head size.
template <int D, bool KEYS_AS_ROWS>
__device__ __forceinline__ f32x16 tile_product(const char* ldsK, int kt, int lane,
                                               const bf16x8 (&qreg)[Tile<D>::KSTEPS], f32x16 init) {
  using T = Tile<D>;
  const char* p = ldsK + (kt * 32 + (lane & 31)) * T::ROWB + (lane >> 5) * 16;
  f32x16 acc = init;
#pragma unroll
  for (int t = 0; t < T::KSTEPS; ++t) {
    const bf16x8 kv = lds_operand(p + t * 32);
    if (KEYS_AS_ROWS)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qreg[t], acc, 0, 0, 0);
    else
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[t], kv, acc, 0, 0, 0);
  }
  return acc;
}

// Row index (0..31) of accumulator register i for a lane in half hf (32x32 output layout:
// groups of four consecutive rows alternate between the two lane halves).
__device__ __forceinline__ int acc_row(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

__device__ __forceinline__ void merge_stat(float& M, float& Z, float2 p) {
  const float Mn = fmaxf(M, p.x);
  Z = Z * __builtin_amdgcn_exp2f(M - Mn) + p.y * __builtin_amdgcn_exp2f(p.x - Mn);
  M = Mn;
}

// ---- software-pipelined passes for chunks without causally masked keys -----------------
// The MFMA chain of key tile i+1 is issued one instruction at a time, each followed by a
// slice of the VALU work of tile i, so that the matrix pipe and the vector ALU run
// concurrently inside one wave; LDS operands are fetched two MFMAs ahead.  The
// scheduling fences pin that interleaving.
template <int D, int NT>
__device__ __forceinline__ void pass1_pipe(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS], int kt0,
                                           float scale2, int lane, float& m_run, float& z_run) {
  using T = Tile<D>;
  constexpr int KS = T::KSTEPS, N = NT * KS;
  const char* base = ldsK + (kt0 * 32 + (lane & 31)) * T::ROWB + (lane >> 5) * 16;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 r0 = lds_operand(base), r1 = lds_operand(base + 32);
  f32x16 cur = zero, nxt = zero;
#pragma unroll
  for (int i = 0; i <= NT; ++i) {
    float m_new = m_run, s = 0.f;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      const int n = i * KS + t;
      if (i < NT) {
        bf16x8 r2 = r0;
        if (n + 2 < N) r2 = lds_operand(base + ((n + 2) / KS) * 32 * T::ROWB + ((n + 2) % KS) * 32);
        nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(r0, qreg[t], (t > 0) ? nxt : zero, 0, 0, 0);
        r0 = r1;
        r1 = r2;
      }
      if (i > 0) {
        if (t == 0) {
          float mx = fmaxf(fmaxf(cur[0], cur[1]), cur[2]);
#pragma unroll
          for (int e = 3; e < 15; e += 2) mx = fmaxf(fmaxf(mx, cur[e]), cur[e + 1]);
          mx = fmaxf(mx, cur[15]);
          m_new = fmaxf(m_run, mx * scale2);
        } else {
          constexpr int SL = KS - 1;
          const int lo = (t - 1) * 16 / SL, hi = t * 16 / SL;
          float x[16];
#pragma unroll
          for (int e = lo; e < hi; ++e) x[e] = fmaf(cur[e], scale2, -m_new);
#pragma unroll
          for (int e = lo; e < hi; ++e) x[e] = __builtin_amdgcn_exp2f(x[e]);
#pragma unroll
          for (int e = lo; e < hi; ++e) s += x[e];
        }
      }
      LAQ_SCHED_FENCE();
    }
    if (i > 0) {
      z_run = fmaf(z_run, __builtin_amdgcn_exp2f(m_run - m_new), s);
      m_run = m_new;
    }
    cur = nxt;
  }
}

template <int D, int NT>
__device__ __forceinline__ void pass2_pipe(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS], int kt0,
                                           const float (&c)[16], float scale2, int lane, float* slotbuf) {
  using T = Tile<D>;
  constexpr int KS = T::KSTEPS, N = NT * KS, PER = 16 / KS;
  const int hf = lane >> 5, n32 = lane & 31;
  const char* base = ldsK + (kt0 * 32 + n32) * T::ROWB + hf * 16;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 r0 = lds_operand(base), r1 = lds_operand(base + 32);
  f32x16 cur = zero, nxt = zero;
#pragma unroll
  for (int i = 0; i <= NT; ++i) {
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      const int n = i * KS + t;
      if (i < NT) {
        bf16x8 r2 = r0;
        if (n + 2 < N) r2 = lds_operand(base + ((n + 2) / KS) * 32 * T::ROWB + ((n + 2) % KS) * 32);
        nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[t], r0, (t > 0) ? nxt : zero, 0, 0, 0);
        r0 = r1;
        r1 = r2;
      }
      if (i > 0) {
        float x[16];
#pragma unroll
        for (int e = t * PER; e < (t + 1) * PER; ++e) x[e] = fmaf(cur[e], scale2, -c[e]);
#pragma unroll
        for (int e = t * PER; e < (t + 1) * PER; ++e) x[e] = __builtin_amdgcn_exp2f(x[e]);
#pragma unroll
        for (int e = t * PER; e < (t + 1) * PER; ++e) s += x[e];
      }
      LAQ_SCHED_FENCE();
    }
    if (i > 0) {
      s += __shfl_xor(s, 32);
      if (hf == 0) slotbuf[(kt0 + i - 1) * 32 + n32] += s;
    }
    cur = nxt;
  }
}

// ---- per-tile passes for chunks that touch the causal region (the last chunks of a head) ----
// A masked logit enters as -inf through the accumulator's initial value.
template <int D>
__device__ __forceinline__ void pass1_masked(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS],
                                             const ScoreGeom& g, int rt, int kt0, int kt1, int j0, int lane,
                                             float& m_run, float& z_run) {
  const int hf = lane >> 5;
  const int w = (rt * 32 + (lane & 31)) % g.W;
  const int t_hi = g.P + w - j0;          // last staged row this lane's score row may see
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kt = kt0; kt < kt1; ++kt) {
    const int t0 = kt * 32;
    f32x16 acc;
    if (j0 + t0 + 31 > g.P) {
      f32x16 bias;
#pragma unroll
      for (int i = 0; i < 16; ++i) bias[i] = (t0 + acc_row(i, hf) <= t_hi) ? 0.f : -INFINITY;
      acc = tile_product<D, true>(ldsK, kt, lane, qreg, bias);
    } else {
      acc = tile_product<D, true>(ldsK, kt, lane, qreg, zero);
    }
    float mx = acc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, acc[i]);
    const float m_new = fmaxf(m_run, mx * g.scale2);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += __builtin_amdgcn_exp2f(fmaf(acc[i], g.scale2, -m_new));
    z_run = fmaf(z_run, __builtin_amdgcn_exp2f(m_run - m_new), s);
    m_run = m_new;
  }
}

template <int D>
__device__ __forceinline__ void pass2_masked(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS],
                                             const ScoreGeom& g, const float (&c)[16], int rt, int kt0, int kt1,
                                             int j0, int lane, float* slotbuf) {
  const int hf = lane >> 5, n = lane & 31;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kt = kt0; kt < kt1; ++kt) {
    const int t0 = kt * 32;
    f32x16 acc;
    if (j0 + t0 + 31 > g.P) {
      f32x16 bias;
      const int j = j0 + t0 + n;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int w = (rt * 32 + acc_row(i, hf)) % g.W;
        bias[i] = (j <= g.P + w) ? 0.f : -INFINITY;
      }
      acc = tile_product<D, false>(ldsK, kt, lane, qreg, bias);
    } else {
      acc = tile_product<D, false>(ldsK, kt, lane, qreg, zero);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += __builtin_amdgcn_exp2f(fmaf(acc[i], g.scale2, -c[i]));
    s += __shfl_xor(s, 32);
    if (hf == 0) slotbuf[t0 + n] += s;
  }
}

// ---- words that workgroups hand to each other -------------------------------------------
// The fused kernel never relies on cache maintenance for them: agent-scope release/acquire
// fences write back and invalidate the whole L2 on this part and cost tens of microseconds
// each.  Instead each word is its own "ready" flag: it is written with one agent-scope atomic
// store and read with agent-scope atomic loads until its pattern says it is there.
//   reset kernel:        (NaN, NaN)   nothing yet
//   chunk's statistics:  (m, z)       both numbers
//   head's row constant: (c, NaN)     written by the head's last-arriving workgroup over
//                                     every chunk's copy of the row
// Nobody polls a word that many others poll: 128 workgroups reading one address in a loop make
// its memory channel a hot spot that stalls the whole key stream behind it.  A workgroup only
// polls its own chunk's words; the one shared word per head is an arrival counter that each
// workgroup bumps exactly once (returning add, not polled).
constexpr int SPIN_LIMIT = 1 << 20;   // probes; about a second, far beyond any legitimate wait

__device__ __forceinline__ void coherent_store(float2* p, float2 v) {
  const unsigned long long bits = ((unsigned long long)__float_as_uint(v.y) << 32) | __float_as_uint(v.x);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 coherent_load(const float2* p) {
  const unsigned long long b = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)b), __uint_as_float((unsigned)(b >> 32)));
}
__device__ __forceinline__ bool wait_failed(int probes, int* err) {
  // Every wait is bounded; once one has timed out, all later waits give up after a few probes,
  // so the kernel always drains.
  if (probes > SPIN_LIMIT ||
      ((probes & 63) == 63 && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
    __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
  }
  return false;
}
// (m, z) of a chunk, once both are numbers
__device__ __forceinline__ float2 await_stat(const float2* p, int* err) {
  for (int probes = 0;; ++probes) {
    const float2 v = coherent_load(p);
    if (v.y == v.y && v.x == v.x) return v;
    if (wait_failed(probes, err)) return make_float2(NEG_BIG, 0.f);
    __builtin_amdgcn_s_sleep(4);
  }
}
// the row constant that the head's last arriver writes over this chunk's copy of the row
__device__ __forceinline__ float await_const(const float2* p, int* err) {
  for (int probes = 0;; ++probes) {
    const float2 v = coherent_load(p);
    if (v.y != v.y && v.x == v.x) return v.x;
    if (wait_failed(probes, err)) return 1.0e30f;
    __builtin_amdgcn_s_sleep(16);
  }
}

// ---- one (head, chunk) unit ---------------------------------------------------------------
// Pass 1 over the staged chunk: (m, z) of every score row goes to out[0 .. Rpad).
// q0 holds this wave's Q tile of the first row group (loaded by the caller, reused by pass 2).
template <int D, int NRT, bool COHERENT>
__device__ __forceinline__ void unit_pass1(char* smem, const ScoreGeom& g, const uint16_t* __restrict__ qg,
                                           const bf16x8 (&q0)[Tile<D>::KSTEPS], int j0, int tid, int lane, int wave,
                                           float2* out) {
  using S = Smem<D, NRT>;
  constexpr int KSPLIT = WAVES / NRT, TPW = KTILES / KSPLIT;
  float2* stat = reinterpret_cast<float2*>(smem + S::OFF_STAT);
  const int slot = wave % NRT, ks = wave / NRT;
  const int ntile = g.Rpad / 32;
  const bool plain_chunk = (j0 + CHUNK_ROWS - 1 <= g.P);    // no key beyond the prefix: no causal mask
  for (int rg = 0; rg * NRT < ntile; ++rg) {
    const int rt = rg * NRT + slot;
    float m_run = NEG_BIG, z_run = 0.f;
    if (rt < ntile) {
      bf16x8 qreg[Tile<D>::KSTEPS];
      if (rg == 0) {
#pragma unroll
        for (int t = 0; t < Tile<D>::KSTEPS; ++t) qreg[t] = q0[t];
      } else {
        load_q_tile<D>(qreg, qg, rt, g.R, lane);
      }
      if (plain_chunk)
        pass1_pipe<D, TPW>(smem, qreg, ks * TPW, g.scale2, lane, m_run, z_run);
      else
        pass1_masked<D>(smem, qreg, g, rt, ks * TPW, ks * TPW + TPW, j0, lane, m_run, z_run);
    }
    stat[tid] = make_float2(m_run, z_run);
    __syncthreads();
    if (tid < NRT * 32) {
      const int s = tid >> 5, n = tid & 31;
      if (rg * NRT + s < ntile) {
        float M = NEG_BIG, Z = 0.f;
#pragma unroll
        for (int c = 0; c < KSPLIT; ++c) {
          const int wv = s + NRT * c;
          merge_stat(M, Z, stat[wv * 64 + n]);
          merge_stat(M, Z, stat[wv * 64 + 32 + n]);
        }
        if (COHERENT)
          coherent_store(out + (rg * NRT + s) * 32 + n, make_float2(M, Z));
        else
          out[(rg * NRT + s) * 32 + n] = make_float2(M, Z);
      }
    }
    __syncthreads();
  }
}

// Pass 2 over the staged chunk with the head's row constants c[0 .. Rpad): the raw score of
// every key of the chunk is written to raw_head.  If crow0_staged, the caller has already put
// the first row group's constants into the LDS slice.
template <int D, int NRT, bool COHERENT>
__device__ __forceinline__ void unit_pass2(char* smem, const ScoreGeom& g, const uint16_t* __restrict__ qg,
                                           const bf16x8 (&q0)[Tile<D>::KSTEPS], const float* c,
                                           const float2* own_words, bool crow0_staged, int* err, int j0, int tid,
                                           int lane, int wave, float* __restrict__ raw_head) {
  using S = Smem<D, NRT>;
  constexpr int KSPLIT = WAVES / NRT, TPW = KTILES / KSPLIT;
  float* crow = reinterpret_cast<float*>(smem + S::OFF_STAT);      // row constants of the current row group
  float* slots = reinterpret_cast<float*>(smem + S::OFF_SLOT);
#pragma unroll
  for (int s = 0; s < NRT; ++s) slots[s * CHUNK_ROWS + tid] = 0.f;
  const int slot = wave % NRT, ks = wave / NRT;
  const int ntile = g.Rpad / 32;
  for (int rg = 0; rg * NRT < ntile; ++rg) {
    if (rg > 0) __syncthreads();
    if (!(rg == 0 && crow0_staged) && tid < NRT * 32) {
      const int r = rg * NRT * 32 + tid;
      float v = 1.0e30f;                                            // padded rows: probability 0
      if (r < g.R) v = COHERENT ? await_const(own_words + r, err) : c[r];
      crow[tid] = v;
    }
    __syncthreads();
    const int rt = rg * NRT + slot;
    if (rt < ntile) {
      bf16x8 qreg[Tile<D>::KSTEPS];
      if (rg == 0) {
#pragma unroll
        for (int t = 0; t < Tile<D>::KSTEPS; ++t) qreg[t] = q0[t];
      } else {
        load_q_tile<D>(qreg, qg, rt, g.R, lane);
      }
      float cr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) cr[i] = crow[slot * 32 + acc_row(i, lane >> 5)];
      if (j0 + CHUNK_ROWS - 1 <= g.P)
        pass2_pipe<D, TPW>(smem, qreg, ks * TPW, cr, g.scale2, lane, slots + slot * CHUNK_ROWS);
      else
        pass2_masked<D>(smem, qreg, g, cr, rt, ks * TPW, ks * TPW + TPW, j0, lane, slots + slot * CHUNK_ROWS);
    }
  }
  __syncthreads();
  float v = slots[tid];
#pragma unroll
  for (int s = 1; s < NRT; ++s) v += slots[s * CHUNK_ROWS + tid];
  if (j0 + tid < g.L) raw_head[j0 + tid] = v;
}

// ---- two-kernel route (K read twice; for heads with more chunks than resident workgroups) ----
template <int D, int NRT>
__global__ __launch_bounds__(THREADS) void stats_mfma_kernel(ScoreGeom g, const uint16_t* __restrict__ q,
                                                             const uint16_t* __restrict__ k,
                                                             float2* __restrict__ part) {
  extern __shared__ __align__(16) char smem[];
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j0 = chunk * CHUNK_ROWS;
  const size_t hg = (size_t)inst * g.Hkv + head;
  const uint16_t* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * D;
  bf16x8 q0[Tile<D>::KSTEPS];
  load_q_tile<D>(q0, qg, wave % NRT, g.R, lane);
  uint4 buf[Tile<D>::PIECES_PER_THREAD];
  fetch_chunk<D>(buf, k + hg * g.L * D, j0, g.L, tid);
  commit_chunk<D>(smem, buf, tid);
  __syncthreads();
  unit_pass1<D, NRT, false>(smem, g, qg, q0, j0, tid, lane, wave, part + (hg * g.nchunk + chunk) * g.Rpad);
}

template <int D, int NRT>
__global__ __launch_bounds__(THREADS) void norm_mfma_kernel(ScoreGeom g, const uint16_t* __restrict__ q,
                                                            const uint16_t* __restrict__ k,
                                                            const float* __restrict__ rowc,
                                                            float* __restrict__ raw) {
  extern __shared__ __align__(16) char smem[];
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j0 = chunk * CHUNK_ROWS;
  const size_t hg = (size_t)inst * g.Hkv + head;
  const uint16_t* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * D;
  bf16x8 q0[Tile<D>::KSTEPS];
  load_q_tile<D>(q0, qg, wave % NRT, g.R, lane);
  uint4 buf[Tile<D>::PIECES_PER_THREAD];
  fetch_chunk<D>(buf, k + hg * g.L * D, j0, g.L, tid);
  commit_chunk<D>(smem, buf, tid);
  __syncthreads();
  unit_pass2<D, NRT, false>(smem, g, qg, q0, rowc + hg * g.Rpad, nullptr, false, nullptr, j0, tid, lane, wave,
                            raw + hg * g.L);
}

// ---- fused single-read kernel -----------------------------------------------------------
// Persistent workgroups walk the list of (KV head, chunk) units in order, unit u going to
// workgroup u mod gridDim.x.  A unit's key rows are read from HBM once: they stay in LDS from
// pass 1 to pass 2.  Between the passes the chunks of a head meet: each workgroup publishes its
// chunk's (m, z) per row and bumps the head's arrival counter; the one that arrives last
// combines all chunks' statistics (fixed order, so the result does not depend on who does it)
// and writes every row's constant over every chunk's copy of the row; the others wait for
// their own copy to change.
// All workgroups of the grid are resident at once (the grid is sized from the occupancy
// query) and no head has more chunks than the grid has workgroups, so a unit only ever waits
// for units that are in flight or earlier in their workgroups' lists: every wait ends.  The
// spins are bounded all the same and record a timeout in the error word.
// The next unit's key rows are requested as soon as the unit's own part of the exchange is
// done, so they travel from HBM to registers while the head is combined and pass 2 runs.

// All threads of the last-arriving workgroup: constants of rows [r0, r0 + rows) into crow_out
// (LDS) and over the rows' copies in every chunk.
__device__ __forceinline__ void combine_head(const ScoreGeom& g, float2* part_head, float2* stat, float* crow_all,
                                             int* err, int tid) {
  for (int r0 = 0; r0 < g.Rpad; r0 += THREADS) {
    const int rows = min(THREADS, g.Rpad - r0);
    const int tpr = (THREADS % rows == 0) ? THREADS / rows : 1;      // threads sharing a row
    const int r = tid % rows, sel = tid / rows;
    float M = NEG_BIG, Z = 0.f;
    if (sel < tpr && r0 + r < g.R) {
      // loads go out in batches (they are independent); only the merges are sequential
      constexpr int B = 32;
      const float2* p = part_head + r0 + r;
      for (int c0 = sel; c0 < g.nchunk; c0 += B * tpr) {
        float2 buf[B];
#pragma unroll
        for (int b = 0; b < B; ++b) buf[b] = coherent_load(p + (size_t)min(c0 + b * tpr, g.nchunk - 1) * g.Rpad);
#pragma unroll
        for (int b = 0; b < B; ++b) {
          if (c0 + b * tpr < g.nchunk) {
            if (!(buf[b].y == buf[b].y && buf[b].x == buf[b].x))     // arrival counted before the store landed
              buf[b] = await_stat(p + (size_t)(c0 + b * tpr) * g.Rpad, err);
            merge_stat(M, Z, buf[b]);
          }
        }
      }
    }
    stat[tid] = make_float2(M, Z);
    __syncthreads();
    if (tid < rows) {
      for (int s2 = 1; s2 < tpr; ++s2) merge_stat(M, Z, stat[s2 * rows + tid]);
      crow_all[r0 + tid] = (r0 + tid < g.R) ? M + __builtin_amdgcn_logf(Z) : 1.0e30f;
    }
    __syncthreads();
    // hand the constants to every chunk of the head; row 0, the one word each waiting workgroup
    // polls, goes last
    const bool mine = sel < tpr && r0 + r < g.R;
    const float cr = crow_all[min(r0 + r, g.Rpad - 1)];
    if (mine && r0 + r != 0)
      for (int c2 = sel; c2 < g.nchunk; c2 += tpr)
        coherent_store(part_head + (size_t)c2 * g.Rpad + r0 + r, make_float2(cr, __uint_as_float(0x7FC00000u)));
    __syncthreads();
    if (mine && r0 + r == 0)
      for (int c2 = sel; c2 < g.nchunk; c2 += tpr)
        coherent_store(part_head + (size_t)c2 * g.Rpad, make_float2(cr, __uint_as_float(0x7FC00000u)));
  }
}

template <int D, int NRT>
__global__ __launch_bounds__(THREADS, 2) void score_fused_kernel(ScoreGeom g, const uint16_t* __restrict__ q,
                                                                 const uint16_t* __restrict__ k, float2* part,
                                                                 int* sync, float* __restrict__ raw, int n_units) {
  extern __shared__ __align__(16) char smem[];
  using S = Smem<D, NRT>;
  __shared__ int sh_last;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float2* stat = reinterpret_cast<float2*>(smem + S::OFF_STAT);
  float* crow = reinterpret_cast<float*>(smem + S::OFF_STAT);
  float* crow_all = reinterpret_cast<float*>(smem + S::OFF_SLOT);    // free between the passes; Rpad <= NRT*256 checked by the host
  const int n_heads = g.n_inst * g.Hkv;
  int* arrived = sync;                    // per head: chunks whose statistics are published
  int* err = sync + n_heads;

  uint4 pre[Tile<D>::PIECES_PER_THREAD];
  int u = blockIdx.x;
  {
    const int hg = u / g.nchunk, c = u - hg * g.nchunk;
    fetch_chunk<D>(pre, k + (size_t)hg * g.L * D, c * CHUNK_ROWS, g.L, tid);
    commit_chunk<D>(smem, pre, tid);
  }
  __syncthreads();

  for (; u < n_units; u += gridDim.x) {
    const int hg = u / g.nchunk, c = u - hg * g.nchunk;
    const int inst = hg / g.Hkv, head = hg - inst * g.Hkv;
    const int j0 = c * CHUNK_ROWS;
    const uint16_t* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * D;
    float2* part_head = part + (size_t)hg * g.nchunk * g.Rpad;
    float2* own_words = part_head + (size_t)c * g.Rpad;
    bf16x8 q0[Tile<D>::KSTEPS];
    load_q_tile<D>(q0, qg, wave % NRT, g.R, lane);

    unit_pass1<D, NRT, true>(smem, g, qg, q0, j0, tid, lane, wave, own_words);
    if (tid == 0)
      sh_last = (__hip_atomic_fetch_add(&arrived[hg], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == g.nchunk - 1);
    __syncthreads();
    const bool last = sh_last != 0;

    // next unit's key rows (the last iteration fetches its own unit again: harmless).  Memory
    // operations retire in order, so the last arriver, whose reads everybody is waiting for,
    // starts its fetch only after them.
    const int un = (u + (int)gridDim.x < n_units) ? u + (int)gridDim.x : u;
    const int hn = un / g.nchunk, cn = un - hn * g.nchunk;
    if (last) {
      combine_head(g, part_head, stat, crow_all, err, tid);
      fetch_chunk<D>(pre, k + (size_t)hn * g.L * D, cn * CHUNK_ROWS, g.L, tid);
      __syncthreads();
      if (tid < NRT * 32) crow[tid] = (tid < g.Rpad) ? crow_all[tid] : 1.0e30f;
    } else {
      fetch_chunk<D>(pre, k + (size_t)hn * g.L * D, cn * CHUNK_ROWS, g.L, tid);
      // one thread polls one word (row 0 is written last); then each row's word is read, and
      // re-read in the rare case that it has not landed yet
      if (tid == 0) await_const(own_words, err);
      __syncthreads();
      if (tid < NRT * 32) crow[tid] = (tid < g.R) ? await_const(own_words + tid, err) : 1.0e30f;
    }

    unit_pass2<D, NRT, true>(smem, g, qg, q0, nullptr, own_words, true, err, j0, tid, lane, wave,
                             raw + (size_t)hg * g.L);
    __syncthreads();                      // every wave is done with this chunk's rows
    commit_chunk<D>(smem, pre, tid);
    __syncthreads();
  }
}

// NaN over the statistics words (their "nothing yet" mark), 0 in the counters and the error word
__global__ void reset_words_kernel(unsigned* words, size_t n, int* sync, int n_sync) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) words[i] = 0xFFFFFFFFu;
  if (i < (size_t)n_sync) sync[i] = 0;
}

template <int D, int NRT>
hipError_t launch_fused(const ScoreGeom& g, const uint16_t* q, const uint16_t* k, float* raw, const Workspace& ws,
                        hipStream_t st) {
  constexpr int bytes = Smem<D, NRT>::BYTES;
  static int resident = 0;                 // workgroups the device holds at once (queried once)
  const void* fn = reinterpret_cast<const void*>(&score_fused_kernel<D, NRT>);
  hipError_t e;
  if (resident == 0) {
    if ((e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&stats_mfma_kernel<D, NRT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&norm_mfma_kernel<D, NRT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0, per_cu = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, THREADS, bytes)) != hipSuccess) return e;
    if (cus < 1 || per_cu < 1) return hipErrorInvalidValue;
    resident = cus * per_cu;
  }
  const int n_heads = g.n_inst * g.Hkv;
  if (g.nchunk > resident || g.Rpad > NRT * CHUNK_ROWS) {
    // A head with more chunks than resident workgroups would make a workgroup wait for its own
    // later unit, and more than NRT*256 score rows do not fit the LDS slice that holds a head's
    // constants: such shapes take the two-kernel route, which reads K twice.
    dim3 grid2(g.nchunk, g.Hkv, g.n_inst), block2(THREADS);
    hipLaunchKernelGGL((stats_mfma_kernel<D, NRT>), grid2, block2, bytes, st, g, q, k, ws.part);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = launch_row_constants(g, ws, st)) != hipSuccess) return e;
    hipLaunchKernelGGL((norm_mfma_kernel<D, NRT>), grid2, block2, bytes, st, g, q, k, ws.rowc, raw);
    return hipGetLastError();
  }
  const long long n_units_ll = (long long)n_heads * g.nchunk;
  if (n_units_ll > 0x7fffffffLL) return hipErrorInvalidValue;
  const int n_units = (int)n_units_ll;
  const size_t n_words = (size_t)n_heads * g.nchunk * g.Rpad * 2;
  hipLaunchKernelGGL(reset_words_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<unsigned*>(ws.part), n_words, ws.sync, n_heads + 1);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int grid = n_units < resident ? n_units : resident;
  hipLaunchKernelGGL((score_fused_kernel<D, NRT>), dim3(grid), dim3(THREADS), bytes, st, g, q, k, ws.part,
                     ws.sync, raw, n_units);
  return hipGetLastError();
}

template <int D>
hipError_t launch_for_rows(const ScoreGeom& g, const uint16_t* q, const uint16_t* k, float* raw,
                           const Workspace& ws, hipStream_t st) {
  const int ntile = g.Rpad / 32;
  if (ntile == 1) return launch_fused<D, 1>(g, q, k, raw, ws, st);
  if (ntile == 2) return launch_fused<D, 2>(g, q, k, raw, ws, st);
  return launch_fused<D, 4>(g, q, k, raw, ws, st);
}

}  // namespace

bool score_mfma_supported(const ScoreGeom& g, int dtype) {
  return dtype == LAQ_BF16 && (g.d == 128 || g.d == 64) && g.R >= 16;
}

hipError_t launch_score_mfma(const ScoreGeom& g, const void* q, const void* k, float* raw, const Workspace& ws,
                             hipStream_t st) {
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  const uint16_t* kk = static_cast<const uint16_t*>(k);
  if (g.d == 128) return launch_for_rows<128>(g, qq, kk, raw, ws, st);
  return launch_for_rows<64>(g, qq, kk, raw, ws, st);
}

}  // namespace laq
