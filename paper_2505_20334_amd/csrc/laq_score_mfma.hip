// bf16 scoring path on the matrix cores (gfx950, v_mfma_f32_32x32x16_bf16).
//
// For one KV head the logits of Eq. 4's observation window form a skinny product
// S = Q_g K^T with R = G*W rows (the group's query heads x the cached window queries)
// and L columns.  A workgroup stages CHUNK_ROWS key rows in LDS (128-bit coalesced
// global loads, each key row read once per kernel) and walks them in 32-key tiles:
//
//   pass 1 (statistics):  D = K_tile * Q^T, so a lane owns one score row and 16 keys of
//           the tile; it keeps a running (max, sum-exp) for its row.  The two lanes that
//           share a row and the waves that share a row tile are merged through LDS and the
//           chunk's (m, z) per row goes to the workspace.
//   pass 2 (normalise + sum + pool): D = Q * K_tile^T, so a lane owns one key and 16 rows;
//           with the row constants c = M + log2 Z the probabilities exp2(s - c) are summed
//           over the rows in-lane, across the two lane halves with one cross-lane add and
//           across row tiles through LDS.  The chunk's raw scores (including a halo of
//           (pool-1)/2 keys on each side) are max-pooled in LDS and the owned keys written.
//
// The A and B operands of the 32x32x16 instruction have the same lane layout (lane l
// supplies row/column l%32 and the 8 consecutive reduction elements l/32), so the same
// registers serve both passes with the operands swapped.
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
  static constexpr int OFF_RAW = OFF_SLOT + NRT * CHUNK_ROWS * 4;      // float[CHUNK_ROWS]
  static constexpr int BYTES = OFF_RAW + CHUNK_ROWS * 4;
};

// Stage rows j0 .. j0+CHUNK_ROWS-1 of one KV head's key matrix; rows outside [0, L) are zero.
template <int D>
__device__ __forceinline__ void stage_chunk(char* ldsK, const uint16_t* __restrict__ khead, int j0, int L,
                                            int tid) {
  using T = Tile<D>;
  uint4 buf[T::PIECES_PER_THREAD];
#pragma unroll
  for (int it = 0; it < T::PIECES_PER_THREAD; ++it) {
    const int p = tid + THREADS * it;
    const int row = p / T::PIECES_PER_ROW, col = p % T::PIECES_PER_ROW;
    const int j = j0 + row;
    if (j >= 0 && j < L)
      buf[it] = *reinterpret_cast<const uint4*>(khead + (size_t)j * D + col * 8);
    else
      buf[it] = make_uint4(0, 0, 0, 0);
  }
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

// acc = (KEYS_AS_ROWS ? K_tile * Q^T : Q * K_tile^T) + init over the whole head size.
template <int D, bool KEYS_AS_ROWS>
__device__ __forceinline__ f32x16 tile_product(const char* ldsK, int kt, int lane,
                                               const bf16x8 (&qreg)[Tile<D>::KSTEPS], f32x16 init) {
  using T = Tile<D>;
  const char* p = ldsK + (kt * 32 + (lane & 31)) * T::ROWB + (lane >> 5) * 16;
  f32x16 acc = init;
#pragma unroll
  for (int t = 0; t < T::KSTEPS; ++t) {
    const bf16x8 kv = *reinterpret_cast<const bf16x8*>(p + t * 32);
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

// ---- pass 1 ---------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void pass1_wave(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS],
                                           const ScoreGeom& g, int rt, int kt0, int kt1, int j0, int lane,
                                           float& m_run, float& z_run) {
  const int hf = lane >> 5;
  const int w = (rt * 32 + (lane & 31)) % g.W;
  // staged rows this lane's score row may count: owned by the chunk and causally visible
  const int t_lo = g.half;
  const int t_hi = min(CHUNK_ROWS - g.half - 1, g.P + w - j0);
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kt = kt0; kt < kt1; ++kt) {
    const int t0 = kt * 32;
    const bool masked = (t0 < g.half) || (t0 + 31 > CHUNK_ROWS - g.half - 1) || (j0 + t0 + 31 > g.P);
    f32x16 acc;
    if (masked) {
      f32x16 bias;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int t = t0 + acc_row(i, hf);
        bias[i] = (t >= t_lo && t <= t_hi) ? 0.f : -INFINITY;
      }
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

template <int D, int NRT>
__global__ __launch_bounds__(THREADS) void stats_mfma_kernel(ScoreGeom g, const uint16_t* __restrict__ q,
                                                             const uint16_t* __restrict__ k,
                                                             float2* __restrict__ part) {
  extern __shared__ __align__(16) char smem[];
  using S = Smem<D, NRT>;
  constexpr int KSPLIT = WAVES / NRT, TPW = KTILES / KSPLIT;
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = chunk * g.own - g.half;
  const uint16_t* khead = k + ((size_t)inst * g.Hkv + head) * g.L * D;
  const uint16_t* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * D;
  float2* out = part + (((size_t)inst * g.Hkv + head) * g.nchunk + chunk) * g.Rpad;
  float2* stat = reinterpret_cast<float2*>(smem + S::OFF_STAT);

  stage_chunk<D>(smem, khead, j0, g.L, tid);
  __syncthreads();

  const int slot = wave % NRT, ks = wave / NRT;
  const int ntile = g.Rpad / 32;
  for (int rg = 0; rg * NRT < ntile; ++rg) {
    const int rt = rg * NRT + slot;
    float m_run = NEG_BIG, z_run = 0.f;
    if (rt < ntile) {
      bf16x8 qreg[Tile<D>::KSTEPS];
      load_q_tile<D>(qreg, qg, rt, g.R, lane);
      pass1_wave<D>(smem, qreg, g, rt, ks * TPW, ks * TPW + TPW, j0, lane, m_run, z_run);
    }
    stat[tid] = make_float2(m_run, z_run);
    __syncthreads();
    if (tid < NRT * 32) {
      const int s = tid >> 5, n = tid & 31;
      if (rg * NRT + s < ntile) {
        float M = NEG_BIG;
#pragma unroll
        for (int c = 0; c < KSPLIT; ++c) {
          const int wv = s + NRT * c;
          M = fmaxf(M, fmaxf(stat[wv * 64 + n].x, stat[wv * 64 + 32 + n].x));
        }
        float Z = 0.f;
#pragma unroll
        for (int c = 0; c < KSPLIT; ++c) {
          const int wv = s + NRT * c;
          const float2 a = stat[wv * 64 + n], b = stat[wv * 64 + 32 + n];
          Z += a.y * __builtin_amdgcn_exp2f(a.x - M);
          Z += b.y * __builtin_amdgcn_exp2f(b.x - M);
        }
        out[(rg * NRT + s) * 32 + n] = make_float2(M, Z);
      }
    }
    __syncthreads();
  }
}

// ---- pass 2 ---------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void pass2_wave(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS],
                                           const ScoreGeom& g, const float* __restrict__ rowc, int rt, int kt0,
                                           int kt1, int j0, int lane, float* slotbuf) {
  const int hf = lane >> 5, n = lane & 31;
  float c[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) c[i] = rowc[rt * 32 + acc_row(i, hf)];
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kt = kt0; kt < kt1; ++kt) {
    const int t0 = kt * 32;
    f32x16 acc;
    if (j0 + t0 + 31 > g.P) {           // some key of the tile lies in the causal region
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

template <int D, int NRT>
__global__ __launch_bounds__(THREADS) void norm_mfma_kernel(ScoreGeom g, const uint16_t* __restrict__ q,
                                                            const uint16_t* __restrict__ k,
                                                            const float* __restrict__ rowc,
                                                            float* __restrict__ scores) {
  extern __shared__ __align__(16) char smem[];
  using S = Smem<D, NRT>;
  constexpr int KSPLIT = WAVES / NRT, TPW = KTILES / KSPLIT;
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = chunk * g.own - g.half;
  const uint16_t* khead = k + ((size_t)inst * g.Hkv + head) * g.L * D;
  const uint16_t* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * D;
  const float* c = rowc + ((size_t)inst * g.Hkv + head) * g.Rpad;
  float* slots = reinterpret_cast<float*>(smem + S::OFF_SLOT);
  float* raw = reinterpret_cast<float*>(smem + S::OFF_RAW);

  stage_chunk<D>(smem, khead, j0, g.L, tid);
#pragma unroll
  for (int s = 0; s < NRT; ++s) slots[s * CHUNK_ROWS + tid] = 0.f;
  __syncthreads();

  const int slot = wave % NRT, ks = wave / NRT;
  const int ntile = g.Rpad / 32;
  for (int rg = 0; rg * NRT < ntile; ++rg) {
    const int rt = rg * NRT + slot;
    if (rt < ntile) {
      bf16x8 qreg[Tile<D>::KSTEPS];
      load_q_tile<D>(qreg, qg, rt, g.R, lane);
      pass2_wave<D>(smem, qreg, g, c, rt, ks * TPW, ks * TPW + TPW, j0, lane, slots + slot * CHUNK_ROWS);
    }
  }
  __syncthreads();
  float v = slots[tid];
#pragma unroll
  for (int s = 1; s < NRT; ++s) v += slots[s * CHUNK_ROWS + tid];
  raw[tid] = v;
  __syncthreads();

  const int j = j0 + tid;
  if (tid >= g.half && tid < CHUNK_ROWS - g.half && j < g.L) {
    if (j < g.P) {
      const int lo = max(j - g.half, 0) - j0, hi = min(j + g.half, g.P - 1) - j0;
      v = raw[lo];
      for (int i = lo + 1; i <= hi; ++i) v = fmaxf(v, raw[i]);
    }
    scores[((size_t)inst * g.Hkv + head) * g.L + j] = v;
  }
}

template <int D, int NRT>
hipError_t launch_pair(const ScoreGeom& g, const uint16_t* q, const uint16_t* k, float* scores,
                       const Workspace& ws, hipStream_t st) {
  constexpr int bytes = Smem<D, NRT>::BYTES;
  static bool attr_done = false;   // raising the dynamic-LDS limit is idempotent
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&stats_mfma_kernel<D, NRT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&norm_mfma_kernel<D, NRT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid(g.nchunk, g.Hkv, g.n_inst), block(THREADS);
  hipLaunchKernelGGL((stats_mfma_kernel<D, NRT>), grid, block, bytes, st, g, q, k, ws.part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_row_constants(g, ws, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((norm_mfma_kernel<D, NRT>), grid, block, bytes, st, g, q, k, ws.rowc, scores);
  return hipGetLastError();
}

template <int D>
hipError_t launch_for_rows(const ScoreGeom& g, const uint16_t* q, const uint16_t* k, float* scores,
                           const Workspace& ws, hipStream_t st) {
  const int ntile = g.Rpad / 32;
  if (ntile == 1) return launch_pair<D, 1>(g, q, k, scores, ws, st);
  if (ntile == 2) return launch_pair<D, 2>(g, q, k, scores, ws, st);
  return launch_pair<D, 4>(g, q, k, scores, ws, st);
}

}  // namespace

bool score_mfma_supported(const ScoreGeom& g, int dtype) {
  return dtype == LAQ_BF16 && (g.d == 128 || g.d == 64) && g.R >= 16;
}

hipError_t launch_score_mfma(const ScoreGeom& g, const void* q, const void* k, float* scores,
                             const Workspace& ws, hipStream_t st) {
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  const uint16_t* kk = static_cast<const uint16_t*>(k);
  if (g.d == 128) return launch_for_rows<128>(g, qq, kk, scores, ws, st);
  return launch_for_rows<64>(g, qq, kk, scores, ws, st);
}

}  // namespace laq
