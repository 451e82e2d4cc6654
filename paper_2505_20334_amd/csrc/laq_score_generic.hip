// Generic scoring path (plain fp32 FMA): any head size, any number of score rows,
// fp32 or bf16 storage.  Used for fp32 inputs and for shapes the MFMA path does not
// take (fewer than 16 score rows per KV head, unusual head sizes).
//
// Computes, per KV head, the window attention of Eq. 4's observation window in two
// passes over the keys: (1) per-row softmax statistics of each 256-key chunk,
// (2) after the statistics of all chunks are combined (row_constants_kernel), the
// normalised sum over rows.  Also here: the sequence max-pool over raw scores.
#include "laq_internal.h"

namespace laq {

namespace {

constexpr float NEG_BIG = -1.0e30f;   // finite "minus infinity" for running maxima

__device__ __forceinline__ float ld_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_elem(const uint16_t* p, size_t i) {
  return __uint_as_float((uint32_t)p[i] << 16);   // bf16 -> fp32 is exact
}

template <typename T>
__device__ __forceinline__ float dot_row(const T* __restrict__ qrow, const T* __restrict__ krow, int d) {
  float acc = 0.f;
  for (int c = 0; c < d; ++c) acc = fmaf(ld_elem(qrow, c), ld_elem(krow, c), acc);
  return acc;
}

__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One workgroup per (chunk, KV head, instance); thread t owns key chunk * 256 + t.
template <typename T>
__global__ __launch_bounds__(CHUNK_ROWS) void stats_generic_kernel(ScoreGeom g, QueryPos qp, KvLayout lay,
                                                                   const T* __restrict__ q,
                                                                   const T* __restrict__ k,
                                                                   float2* __restrict__ part) {
  __shared__ float red[4];
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int j = chunk * CHUNK_ROWS + t;
  const bool owned = j < g.L;
  const T* krow = k + (size_t)inst * lay.inst + (size_t)head * lay.head + (size_t)(owned ? j : 0) * lay.row;
  const T* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * g.d;
  float2* out = part + (((size_t)inst * g.Hkv + head) * g.nchunk + chunk) * g.Rpad;

  for (int r = 0; r < g.R; ++r) {
    const int w = r % g.W;
    const bool vis = owned && (j <= last_visible_key(g, qp, w));
    float s = vis ? g.scale2 * dot_row(qg + (size_t)r * g.d, krow, g.d) : NEG_BIG;
    float m = wave_max(s);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float e = vis ? exp2f(s - m) : 0.f;
    e = wave_sum(e);
    if (lane == 0) red[wave] = e;
    __syncthreads();
    if (t == 0) out[r] = make_float2(m, (red[0] + red[1]) + (red[2] + red[3]));
    __syncthreads();
  }
}

template <typename T>
__global__ __launch_bounds__(CHUNK_ROWS) void norm_generic_kernel(ScoreGeom g, QueryPos qp, KvLayout lay,
                                                                  const T* __restrict__ q,
                                                                  const T* __restrict__ k,
                                                                  const float* __restrict__ rowc,
                                                                  float* __restrict__ raw) {
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int j = chunk * CHUNK_ROWS + threadIdx.x;
  if (j >= g.L) return;
  const T* krow = k + (size_t)inst * lay.inst + (size_t)head * lay.head + (size_t)j * lay.row;
  const T* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * g.d;
  const float* c = rowc + ((size_t)inst * g.Hkv + head) * g.Rpad;
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int w = r % g.W;
    if (j <= last_visible_key(g, qp, w)) acc += exp2f(g.scale2 * dot_row(qg + (size_t)r * g.d, krow, g.d) - c[r]);
  }
  raw[((size_t)inst * g.Hkv + head) * g.L + j] = acc;
}

// pooled[j] = max (or mean) of raw[i], |i - j| <= half, 0 <= i < P, for prefix keys; the kept
// trailing columns are copied.  A workgroup stages POOL_TILE scores plus the window margins in
// LDS, with zeros for positions outside the prefix: the scores are sums of probabilities, never
// negative, so a zero leaves a maximum alone, and it leaves the ascending fp32 sum of the average
// bit-identical to pool_window()'s sum over the clipped window.  grid.x walks the (instance, KV
// head) pairs.
constexpr int POOL_TILE = 1024;
__global__ __launch_bounds__(256) void pool_kernel(int L, int P, int half, bool avg, const float* __restrict__ raw,
                                                   float* __restrict__ pooled) {
  __shared__ float tile[POOL_TILE + MAX_POOL - 1];
  const float* r = raw + (size_t)blockIdx.x * L;
  float* out = pooled + (size_t)blockIdx.x * L;
  const int j0 = blockIdx.y * POOL_TILE;
  for (int t = threadIdx.x; t < POOL_TILE + 2 * half; t += 256) {
    const int i = j0 - half + t;
    tile[t] = (i >= 0 && i < P) ? r[i] : 0.f;
  }
  __syncthreads();
  const float kernel_size = (float)(2 * half + 1);
  for (int t = threadIdx.x; t < POOL_TILE && j0 + t < L; t += 256) {
    const int j = j0 + t;
    float v;
    if (j >= P) {
      v = r[j];
    } else if (avg) {
      float acc = 0.f;
      for (int o = 0; o <= 2 * half; ++o) acc += tile[t + o];
      v = acc / kernel_size;
    } else {
      v = tile[t + half];
      for (int o = 0; o <= 2 * half; ++o) v = fmaxf(v, tile[t + o]);
    }
    out[j] = v;
  }
}

}  // namespace

// Combine the per-chunk (m, z) of every score row into c = M + log2(Z), so that the
// attention probability of a logit s (base-2 units) is exp2(s - c).  Rows beyond R
// (padding up to a multiple of 32) get a huge c, i.e. probability 0.
__global__ void row_constants_kernel(ScoreGeom g, const float2* __restrict__ part, float* __restrict__ rowc) {
  const int head = blockIdx.x, inst = blockIdx.y;
  const float2* p = part + ((size_t)inst * g.Hkv + head) * g.nchunk * g.Rpad;
  float* c = rowc + ((size_t)inst * g.Hkv + head) * g.Rpad;
  for (int r = threadIdx.x; r < g.Rpad; r += blockDim.x) {
    if (r >= g.R) { c[r] = 1.0e30f; continue; }
    float M = NEG_BIG;
    for (int ch = 0; ch < g.nchunk; ++ch) M = fmaxf(M, p[(size_t)ch * g.Rpad + r].x);
    float Z = 0.f;
    for (int ch = 0; ch < g.nchunk; ++ch) {
      float2 mz = p[(size_t)ch * g.Rpad + r];
      Z += mz.y * exp2f(mz.x - M);
    }
    c[r] = M + log2f(Z);
  }
}

hipError_t launch_row_constants(const ScoreGeom& g, const Workspace& ws, hipStream_t st) {
  dim3 grid(g.Hkv, g.n_inst);
  hipLaunchKernelGGL(row_constants_kernel, grid, dim3(128), 0, st, g, ws.part, ws.rowc);
  return hipGetLastError();
}

hipError_t launch_pool(const ScoreGeom& g, int pool, bool avg, const float* raw, float* pooled, hipStream_t st) {
  dim3 grid(g.n_inst * g.Hkv, (g.L + POOL_TILE - 1) / POOL_TILE);
  hipLaunchKernelGGL(pool_kernel, grid, dim3(256), 0, st, g.L, g.P, (pool - 1) / 2, avg, raw, pooled);
  return hipGetLastError();
}

hipError_t launch_score_generic(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int dtype, const void* q,
                                const void* k, float* raw, const Workspace& ws, hipStream_t st) {
  dim3 grid(g.nchunk, g.Hkv, g.n_inst), block(CHUNK_ROWS);
  if (dtype == LAQ_F32) {
    hipLaunchKernelGGL(stats_generic_kernel<float>, grid, block, 0, st, g, qp, lay, (const float*)q, (const float*)k,
                       ws.part);
  } else {
    hipLaunchKernelGGL(stats_generic_kernel<uint16_t>, grid, block, 0, st, g, qp, lay, (const uint16_t*)q,
                       (const uint16_t*)k, ws.part);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_row_constants(g, ws, st);
  if (e != hipSuccess) return e;
  if (dtype == LAQ_F32) {
    hipLaunchKernelGGL(norm_generic_kernel<float>, grid, block, 0, st, g, qp, lay, (const float*)q, (const float*)k,
                       ws.rowc, raw);
  } else {
    hipLaunchKernelGGL(norm_generic_kernel<uint16_t>, grid, block, 0, st, g, qp, lay, (const uint16_t*)q,
                       (const uint16_t*)k, ws.rowc, raw);
  }
  return hipGetLastError();
}

}  // namespace laq
