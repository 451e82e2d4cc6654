// Generic scoring path (vector ALU, no matrix cores): any head size up to 256, any number of
// score rows, fp32 or bf16 storage.  Used for fp32 inputs and for head sizes the MFMA path does
// not take.
//
// Computes, per KV head, the window attention of Eq. 4's observation window in two passes over
// the keys: (1) per-row softmax statistics of each 256-key chunk, (2) after the statistics of all
// chunks are combined (row_constants_kernel), the normalised sum over rows.  Also here: the
// sequence pooling over raw scores.
//
// Both passes give a key row to a group of PP adjacent lanes, 8 elements per lane, so that a
// wave's loads cover whole rows contiguously; the 256 / PP groups of a workgroup take the 256 keys
// of a chunk round-robin.  The score rows are walked in blocks of GEN_ROWS whose query pieces sit in
// registers; the chunk's key rows are re-read from cache once per block.
#include "laq_internal.h"
#include "laq_lanegroup.h"

namespace laq {

namespace {

constexpr float NEG_BIG = -1.0e30f;   // finite "minus infinity" for running maxima
constexpr int GEN_ROWS = 8;           // score rows per register block

// One workgroup per (chunk, KV head, instance).  part[chunk][r] = (m, z) of row r over the
// chunk's visible keys.
template <typename T, int PP>
__global__ __launch_bounds__(CHUNK_ROWS) void stats_generic_kernel(ScoreGeom g, QueryPos qp, KvLayout lay,
                                                                   const T* __restrict__ q,
                                                                   const T* __restrict__ k,
                                                                   float2* __restrict__ part) {
  using Piece = typename PieceOf<T>::type;
  constexpr int NG = CHUNK_ROWS / PP, KPG = CHUNK_ROWS / NG;     // lane groups; keys per group
  __shared__ float2 red[NG][GEN_ROWS];
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int tid = threadIdx.x, dc = tid % PP, ks = tid / PP;
  const bool active = dc * 8 < g.d;
  const int j0 = chunk * CHUNK_ROWS;
  // first row of the head (of a paged cache: where row 0 would lie if this chunk's block held the whole
  // head; a block holds whole chunks)
  int64_t head_off = (int64_t)inst * lay.inst;
  if (lay.table) {
    int r0;
    head_off = paged_block_offset(lay, inst, j0, &r0) - (int64_t)(j0 - r0) * lay.row;
  }
  const T* kbase = k + head_off + (int64_t)head * lay.head + dc * 8;
  const T* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * g.d + dc * 8;
  float2* out = part + (((size_t)inst * g.Hkv + head) * g.nchunk + chunk) * g.Rpad;

  for (int r0 = 0; r0 < g.R; r0 += GEN_ROWS) {
    Piece qv[GEN_ROWS];
    int last[GEN_ROWS];
    float m[GEN_ROWS], z[GEN_ROWS];
#pragma unroll
    for (int rb = 0; rb < GEN_ROWS; ++rb) {
      clear8(qv[rb]);
      m[rb] = NEG_BIG;
      z[rb] = 0.f;
      last[rb] = -1;                                   // rows beyond R see nothing
      if (r0 + rb < g.R) {
        last[rb] = last_visible_key(g, qp, (r0 + rb) % g.W);
        if (active) fetch8(qg + (size_t)(r0 + rb) * g.d, qv[rb]);
      }
    }
#pragma unroll 2
    for (int kk = 0; kk < KPG; ++kk) {
      const int j = j0 + ks + NG * kk;
      Piece kp;
      clear8(kp);
      if (active && j < g.L) fetch8(kbase + (size_t)j * lay.row, kp);
#pragma unroll
      for (int rb = 0; rb < GEN_ROWS; ++rb) {
        const float s = group_sum<PP>(dot8(qv[rb], kp)) * g.scale2;
        if (j < g.L && j <= last[rb]) {
          const float m_new = fmaxf(m[rb], s);
          z[rb] = fmaf(z[rb], exp2f(m[rb] - m_new), exp2f(s - m_new));
          m[rb] = m_new;
        }
      }
    }
    if (dc == 0) {
#pragma unroll
      for (int rb = 0; rb < GEN_ROWS; ++rb) red[ks][rb] = make_float2(m[rb], z[rb]);
    }
    __syncthreads();
    if (tid < GEN_ROWS && r0 + tid < g.R) {
      float M = NEG_BIG, Z = 0.f;
      for (int gidx = 0; gidx < NG; ++gidx) {           // fixed order
        const float2 mz = red[gidx][tid];
        const float Mn = fmaxf(M, mz.x);
        Z = Z * exp2f(M - Mn) + mz.y * exp2f(mz.x - Mn);
        M = Mn;
      }
      out[r0 + tid] = make_float2(M, Z);
    }
    __syncthreads();
  }
}

// raw[j] = sum over the score rows of exp2(s - c[r]) for the keys of the chunk.
template <typename T, int PP>
__global__ __launch_bounds__(CHUNK_ROWS) void norm_generic_kernel(ScoreGeom g, QueryPos qp, KvLayout lay,
                                                                  const T* __restrict__ q,
                                                                  const T* __restrict__ k,
                                                                  const float* __restrict__ rowc,
                                                                  float* __restrict__ raw) {
  using Piece = typename PieceOf<T>::type;
  constexpr int NG = CHUNK_ROWS / PP, KPG = CHUNK_ROWS / NG;
  const int chunk = blockIdx.x, head = blockIdx.y, inst = blockIdx.z;
  const int tid = threadIdx.x, dc = tid % PP, ks = tid / PP;
  const bool active = dc * 8 < g.d;
  const int j0 = chunk * CHUNK_ROWS;
  // first row of the head (of a paged cache: where row 0 would lie if this chunk's block held the whole
  // head; a block holds whole chunks)
  int64_t head_off = (int64_t)inst * lay.inst;
  if (lay.table) {
    int r0;
    head_off = paged_block_offset(lay, inst, j0, &r0) - (int64_t)(j0 - r0) * lay.row;
  }
  const T* kbase = k + head_off + (int64_t)head * lay.head + dc * 8;
  const T* qg = q + ((size_t)inst * g.Hq + (size_t)head * g.G) * g.W * g.d + dc * 8;
  const float* c = rowc + ((size_t)inst * g.Hkv + head) * g.Rpad;
  float acc[KPG];
#pragma unroll
  for (int kk = 0; kk < KPG; ++kk) acc[kk] = 0.f;

  for (int r0 = 0; r0 < g.R; r0 += GEN_ROWS) {
    Piece qv[GEN_ROWS];
    int last[GEN_ROWS];
    float cr[GEN_ROWS];
#pragma unroll
    for (int rb = 0; rb < GEN_ROWS; ++rb) {
      clear8(qv[rb]);
      last[rb] = -1;
      cr[rb] = 0.f;
      if (r0 + rb < g.R) {
        last[rb] = last_visible_key(g, qp, (r0 + rb) % g.W);
        cr[rb] = c[r0 + rb];
        if (active) fetch8(qg + (size_t)(r0 + rb) * g.d, qv[rb]);
      }
    }
#pragma unroll
    for (int kk = 0; kk < KPG; ++kk) {
      const int j = j0 + ks + NG * kk;
      Piece kp;
      clear8(kp);
      if (active && j < g.L) fetch8(kbase + (size_t)j * lay.row, kp);
#pragma unroll
      for (int rb = 0; rb < GEN_ROWS; ++rb) {
        const float s = group_sum<PP>(dot8(qv[rb], kp)) * g.scale2;
        if (j <= last[rb]) acc[kk] += exp2f(s - cr[rb]);
      }
    }
  }
  if (dc == 0) {
    float* rw = raw + ((size_t)inst * g.Hkv + head) * g.L;
#pragma unroll
    for (int kk = 0; kk < KPG; ++kk) {
      const int j = j0 + ks + NG * kk;
      if (j < g.L) rw[j] = acc[kk];
    }
  }
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
// (padding up to a multiple of 32) get a huge c, i.e. probability 0.  Also clears the workspace's
// status word (these kernels have no wait to give up).
__global__ void row_constants_kernel(ScoreGeom g, const float2* __restrict__ part, float* __restrict__ rowc,
                                     int* __restrict__ status) {
  const int head = blockIdx.x, inst = blockIdx.y;
  if (head == 0 && inst == 0 && threadIdx.x == 0) *status = 0;
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
  hipLaunchKernelGGL(row_constants_kernel, grid, dim3(128), 0, st, g, ws.part, ws.rowc, ws.status);
  return hipGetLastError();
}

hipError_t launch_pool(const ScoreGeom& g, int pool, bool avg, const float* raw, float* pooled, hipStream_t st) {
  dim3 grid(g.n_inst * g.Hkv, (g.L + POOL_TILE - 1) / POOL_TILE);
  hipLaunchKernelGGL(pool_kernel, grid, dim3(256), 0, st, g.L, g.P, (pool - 1) / 2, avg, raw, pooled);
  return hipGetLastError();
}

template <typename T, int PP>
static hipError_t launch_generic_pp(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, const T* q, const T* k,
                                    float* raw, const Workspace& ws, hipStream_t st) {
  dim3 grid(g.nchunk, g.Hkv, g.n_inst), block(CHUNK_ROWS);
  hipLaunchKernelGGL((stats_generic_kernel<T, PP>), grid, block, 0, st, g, qp, lay, q, k, ws.part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if ((e = launch_row_constants(g, ws, st)) != hipSuccess) return e;
  hipLaunchKernelGGL((norm_generic_kernel<T, PP>), grid, block, 0, st, g, qp, lay, q, k, ws.rowc, raw);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_generic_for(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, const void* q,
                                     const void* k, float* raw, const Workspace& ws, hipStream_t st) {
  const T* qq = static_cast<const T*>(q);
  const T* kk = static_cast<const T*>(k);
  const int pp = lanes_per_row(g.d);
  if (pp == 8) return launch_generic_pp<T, 8>(g, qp, lay, qq, kk, raw, ws, st);
  if (pp == 16) return launch_generic_pp<T, 16>(g, qp, lay, qq, kk, raw, ws, st);
  return launch_generic_pp<T, 32>(g, qp, lay, qq, kk, raw, ws, st);
}

hipError_t launch_score_generic(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int dtype, const void* q,
                                const void* k, float* raw, const Workspace& ws, hipStream_t st) {
  if (dtype == LAQ_F32) return launch_generic_for<float>(g, qp, lay, q, k, raw, ws, st);
  return launch_generic_for<uint16_t>(g, qp, lay, q, k, raw, ws, st);
}

}  // namespace laq
