// The steps around the re-eviction (Sec. 4.2 / 4.3): storing the queries of a lookahead step into
// the Q-cache, and the attention of one new token over the compacted cache that decoding
// continues on.
//
// Decode attention is bound by reading K' and V' once.  One workgroup serves up to four query
// heads that share a KV head (they share every key and value row it reads).  A row is read by a
// group of `pp` adjacent lanes, 8 elements each, so a wave's loads cover whole rows contiguously;
// the lane groups of the workgroup take the rows round-robin, several rows per turn; each group
// keeps its own running (max, sum, weighted value sum) per query head.  The groups of a wave are merged across lanes, the waves through
// LDS, in a fixed order (the results do not depend on timing).
#include "laq_internal.h"
#include "laq_lanegroup.h"

namespace laq {

namespace {

constexpr int DEC_MANY_WORKGROUPS = 1024;
constexpr float DEC_NEG_BIG = -1.0e30f;

// LDS layout: m[DEC_WAVES][GB], z[DEC_WAVES][GB], acc[DEC_WAVES][GB][d].  DEC_ROWS: rows per lane
// group and turn.  PREFETCH: the next turn's rows are requested before the current turn's
// arithmetic (more registers, fewer resident waves).  A workgroup works on one part of a cache
// (blockIdx.y): the whole cache writes `out`; one of several parts writes its unnormalised sums
// O[d], then M and Z, per query head, to partial[part][blockIdx.x][g][d + 2] for merge_parts_kernel.
template <int GB, typename T, int DEC_THREADS, int DEC_ROWS, bool PREFETCH, int PP, typename TAB>
__global__ __launch_bounds__(DEC_THREADS) void decode_kernel(int Hq, int Hkv, int d, float scale2,
                                                             TAB tab, const T* __restrict__ q,
                                                             const T* __restrict__ kc, const T* __restrict__ vc,
                                                             float* __restrict__ out, float* __restrict__ partial) {
  using Piece = typename PieceOf<T>::type;
  constexpr int DEC_WAVES = DEC_THREADS / 64;
  constexpr int pp = PP;                   // lanes per row
  extern __shared__ float sm[];
  const int G = Hq / Hkv, nbatch = (G + GB - 1) / GB;
  const int head = blockIdx.x / nbatch, g0 = (blockIdx.x % nbatch) * GB;
  const int li = blockIdx.y, inst = tab.inst_of(li);
  const int bk = tab.part_rows(li);        // rows of this part
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int dc = tid % pp, ks = tid / pp, nks = DEC_THREADS / pp;
  const bool active = dc * 8 < d;
  const int64_t first_row = tab.base_row(li) + (int64_t)head * tab.cache_rows(li) + tab.first_row(li);
  const T* K = kc + first_row * d + dc * 8;
  const T* V = vc + first_row * d + dc * 8;

  Piece qv[GB];                            // this lane's 8 elements of every query of the batch
  float acc[GB][8], m[GB], z[GB];
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    m[g] = DEC_NEG_BIG;
    z[g] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[g][c] = 0.f;
    clear8(qv[g]);
    if (active && g0 + g < G) fetch8(q + ((size_t)inst * Hq + (size_t)head * G + g0 + g) * d + dc * 8, qv[g]);
  }

  const int turns = ((bk + nks - 1) / nks + DEC_ROWS - 1) / DEC_ROWS;
  // rows ks + nks * (t * DEC_ROWS + u), u < DEC_ROWS, of turn t; rows beyond the cache read as zeros
  auto fetch_turn = [&](int t, Piece (&kp)[DEC_ROWS], Piece (&vp)[DEC_ROWS]) {
#pragma unroll
    for (int u = 0; u < DEC_ROWS; ++u) {
      const int j = ks + nks * (t * DEC_ROWS + u);
      clear8(kp[u]);
      clear8(vp[u]);
      if (active && j < bk) {
        fetch8(K + (size_t)j * d, kp[u]);
        fetch8(V + (size_t)j * d, vp[u]);
      }
    }
  };
  Piece kp[DEC_ROWS], vp[DEC_ROWS], kn[DEC_ROWS], vn[DEC_ROWS];
  if (PREFETCH) fetch_turn(0, kp, vp);
  for (int t = 0; t < turns; ++t) {
    if (!PREFETCH) fetch_turn(t, kp, vp);
    if (PREFETCH && t + 1 < turns) fetch_turn(t + 1, kn, vn);   // travels during this turn's arithmetic
    bool valid[DEC_ROWS];
#pragma unroll
    for (int u = 0; u < DEC_ROWS; ++u) valid[u] = ks + nks * (t * DEC_ROWS + u) < bk;
    float s[DEC_ROWS][GB];
#pragma unroll
    for (int u = 0; u < DEC_ROWS; ++u) {
#pragma unroll
      for (int g = 0; g < GB; ++g) s[u][g] = dot8(qv[g], kp[u]);
    }
    // every lane of a group gets the complete logits of the group's rows, in base-2 units
#pragma unroll
    for (int u = 0; u < DEC_ROWS; ++u)
#pragma unroll
      for (int g = 0; g < GB; ++g) s[u][g] = group_sum<PP>(s[u][g]) * scale2;
    float p[DEC_ROWS][GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      float m_new = m[g];
#pragma unroll
      for (int u = 0; u < DEC_ROWS; ++u)
        if (valid[u]) m_new = fmaxf(m_new, s[u][g]);
      const float a = __builtin_amdgcn_exp2f(m[g] - m_new);
      float zsum = 0.f;
#pragma unroll
      for (int u = 0; u < DEC_ROWS; ++u) {
        p[u][g] = valid[u] ? __builtin_amdgcn_exp2f(s[u][g] - m_new) : 0.f;
        zsum += p[u][g];
      }
      z[g] = fmaf(z[g], a, zsum);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[g][c] *= a;
      m[g] = m_new;
    }
#pragma unroll
    for (int u = 0; u < DEC_ROWS; ++u) {
      float vf[8];
      widen8(vp[u], vf);
#pragma unroll
      for (int g = 0; g < GB; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[g][c] = fmaf(p[u][g], vf[c], acc[g][c]);
    }
    if (PREFETCH) {
#pragma unroll
      for (int u = 0; u < DEC_ROWS; ++u) {
        kp[u] = kn[u];
        vp[u] = vn[u];
      }
    }
  }

  // merge the lane groups of a wave: after the last step the wave's first group holds the result
  for (int o = pp; o < 64; o <<= 1) {
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      const float m_o = __shfl_xor(m[g], o), z_o = __shfl_xor(z[g], o);
      const float M = fmaxf(m[g], m_o);
      const float a = __builtin_amdgcn_exp2f(m[g] - M), b = __builtin_amdgcn_exp2f(m_o - M);
      z[g] = fmaf(z[g], a, z_o * b);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[g][c] = fmaf(acc[g][c], a, __shfl_xor(acc[g][c], o) * b);
      m[g] = M;
    }
  }
  float* sm_m = sm;
  float* sm_z = sm + DEC_WAVES * GB;
  float* sm_acc = sm + 2 * DEC_WAVES * GB;
  if (lane < pp) {
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      if (lane == 0) {
        sm_m[wave * GB + g] = m[g];
        sm_z[wave * GB + g] = z[g];
      }
      if (active) {
#pragma unroll
        for (int c = 0; c < 8; ++c) sm_acc[((size_t)wave * GB + g) * d + dc * 8 + c] = acc[g][c];
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < GB * d; e += DEC_THREADS) {
    const int g = e / d, c = e - g * d;
    if (g0 + g >= G) continue;
    float M = DEC_NEG_BIG;
#pragma unroll
    for (int w = 0; w < DEC_WAVES; ++w) M = fmaxf(M, sm_m[w * GB + g]);
    float Z = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < DEC_WAVES; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(sm_m[w * GB + g] - M);
      Z = fmaf(sm_z[w * GB + g], wgt, Z);
      O = fmaf(sm_acc[((size_t)w * GB + g) * d + c], wgt, O);
    }
    if (tab.parts(li) == 1) {
      out[((size_t)inst * Hq + (size_t)head * G + g0 + g) * d + c] = O / Z;
    } else {
      float* rec = partial + (((size_t)li * gridDim.x + blockIdx.x) * GB + g) * (d + 2);
      rec[c] = O;
      if (c == 0) {
        rec[d] = M;
        rec[d + 1] = Z;
      }
    }
  }
}

// out[inst][h] from the parts of a cache that was split: the part records are merged in part
// order.  blockIdx.x = query head, blockIdx.y = part; the workgroup of a cache's first part does
// the work (the parts of a cache are consecutive entries of the table).
__global__ __launch_bounds__(128) void merge_parts_kernel(int Hq, int Hkv, int d, int gb, int blocks_x,
                                                          DecodeParts tab, const float* __restrict__ partial,
                                                          float* __restrict__ out) {
  const int li = blockIdx.y, h = blockIdx.x;
  const int S = tab.nsplit[li];
  if (S == 1 || tab.split[li] != 0) return;
  const int G = Hq / Hkv, nbatch = (G + gb - 1) / gb;
  const int head = h / G, gq = h - head * G;
  const int x = head * nbatch + gq / gb, g = gq % gb;
  const size_t rec_floats = (size_t)(d + 2), part_floats = (size_t)blocks_x * gb * rec_floats;
  const float* rec0 = partial + ((size_t)li * blocks_x + x) * gb * rec_floats + (size_t)g * rec_floats;
  float M = DEC_NEG_BIG;
  for (int s2 = 0; s2 < S; ++s2) M = fmaxf(M, rec0[s2 * part_floats + d]);
  float Z = 0.f;
  for (int s2 = 0; s2 < S; ++s2) Z = fmaf(rec0[s2 * part_floats + d + 1], __builtin_amdgcn_exp2f(rec0[s2 * part_floats + d] - M), Z);
  for (int c = threadIdx.x; c < d; c += 128) {
    float O = 0.f;
    for (int s2 = 0; s2 < S; ++s2)
      O = fmaf(rec0[s2 * part_floats + c], __builtin_amdgcn_exp2f(rec0[s2 * part_floats + d] - M), O);
    out[((size_t)tab.inst[li] * Hq + h) * d + c] = O / Z;
  }
}

// q_cache[inst][h][t][:] = q_step[inst][h][:], 16 bytes per thread
__global__ __launch_bounds__(256) void qcache_store_kernel(long long rows, int W, int t, int pieces,
                                                           const uint4* __restrict__ q_step,
                                                           uint4* __restrict__ q_cache) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * pieces) return;
  const long long row = i / pieces;
  const int piece = (int)(i - row * pieces);
  q_cache[(row * W + t) * pieces + piece] = q_step[i];
}

template <int GB, typename T, int THREADS, int ROWS, bool PREFETCH, int PP, typename TAB>
hipError_t launch_decode_pp(int n_parts, int Hq, int Hkv, int d, float scale2, const TAB& tab, const void* q,
                            const void* kc, const void* vc, float* out, float* partial, hipStream_t st) {
  const int G = Hq / Hkv, nbatch = (G + GB - 1) / GB;
  const size_t lds = (size_t)(THREADS / 64) * GB * (d + 2) * sizeof(float);
  hipLaunchKernelGGL((decode_kernel<GB, T, THREADS, ROWS, PREFETCH, PP, TAB>), dim3(Hkv * nbatch, n_parts), dim3(THREADS), lds,
                     st, Hq, Hkv, d, scale2, tab, static_cast<const T*>(q), static_cast<const T*>(kc),
                     static_cast<const T*>(vc), out, partial);
  return hipGetLastError();
}

// lanes per row: the power of two (at least 8) that covers the row's d / 8 pieces
template <int GB, typename T, int THREADS, int ROWS, bool PREFETCH, typename TAB>
hipError_t launch_decode_as(int n_parts, int Hq, int Hkv, int d, float scale2, const TAB& tab, const void* q,
                            const void* kc, const void* vc, float* out, float* partial, hipStream_t st) {
  if (d <= 64)
    return launch_decode_pp<GB, T, THREADS, ROWS, PREFETCH, 8>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
  if (d <= 128)
    return launch_decode_pp<GB, T, THREADS, ROWS, PREFETCH, 16>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
  return launch_decode_pp<GB, T, THREADS, ROWS, PREFETCH, 32>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
}

// Few workgroups (long caches, few heads): large workgroups that keep two turns of rows in flight.
// Many workgroups, or caches cut into parts (short row ranges, several parts per compute unit):
// small ones without the second set of row registers, so that more of them are resident at once.
template <int GB, typename T, typename TAB>
hipError_t launch_decode_for(int n_parts, int Hq, int Hkv, int d, float scale2, const TAB& tab, const void* q,
                             const void* kc, const void* vc, float* out, float* partial, hipStream_t st) {
  const int G = Hq / Hkv, nbatch = (G + GB - 1) / GB;
  if ((long long)Hkv * nbatch * n_parts >= DEC_MANY_WORKGROUPS || tab.parts(0) > 1 || tab.parts(n_parts - 1) > 1)
    return launch_decode_as<GB, T, 256, 4, false>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
  return launch_decode_as<GB, T, 512, (sizeof(T) == 2 ? 8 : 4), true>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
}

}  // namespace

int decode_head_batch(int Hq, int Hkv) {
  const int G = Hq / Hkv;
  return G == 1 ? 1 : (G == 2 ? 2 : 4);
}

hipError_t launch_merge_parts(int n_parts, int Hq, int Hkv, int d, const DecodeParts& tab, const float* partial,
                              float* out, hipStream_t st) {
  const int gb = decode_head_batch(Hq, Hkv), G = Hq / Hkv, nbatch = (G + gb - 1) / gb;
  hipLaunchKernelGGL(merge_parts_kernel, dim3(Hq, n_parts), dim3(128), 0, st, Hq, Hkv, d, gb, Hkv * nbatch, tab, partial,
                     out);
  return hipGetLastError();
}

template <typename TAB>
static hipError_t launch_decode_any(int n_parts, int Hq, int Hkv, int d, int dtype, float scale2, const TAB& tab,
                                    const void* q, const void* kc, const void* vc, float* out, float* partial,
                                    hipStream_t st) {
  const int G = Hq / Hkv;
  if (dtype == LAQ_BF16) {
    if (G == 1) return launch_decode_for<1, uint16_t>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
    if (G == 2) return launch_decode_for<2, uint16_t>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
    return launch_decode_for<4, uint16_t>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
  }
  if (G == 1) return launch_decode_for<1, float>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
  if (G == 2) return launch_decode_for<2, float>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
  return launch_decode_for<4, float>(n_parts, Hq, Hkv, d, scale2, tab, q, kc, vc, out, partial, st);
}

hipError_t launch_decode(int n_parts, int Hq, int Hkv, int d, int dtype, float scale2, const DecodeParts& tab,
                         const void* q, const void* kc, const void* vc, float* out, float* partial, hipStream_t st) {
  return launch_decode_any(n_parts, Hq, Hkv, d, dtype, scale2, tab, q, kc, vc, out, partial, st);
}

hipError_t launch_decode(int n_inst, int Hq, int Hkv, int d, int dtype, float scale2, const DecodeWhole& tab,
                         const void* q, const void* kc, const void* vc, float* out, hipStream_t st) {
  return launch_decode_any(n_inst, Hq, Hkv, d, dtype, scale2, tab, q, kc, vc, out, (float*)nullptr, st);
}

hipError_t launch_qcache_store(long long rows, int W, int t, int row_bytes, const void* q_step, void* q_cache,
                               hipStream_t st) {
  const int pieces = row_bytes / 16;
  const long long total = rows * pieces;
  hipLaunchKernelGGL(qcache_store_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, rows, W, t, pieces,
                     static_cast<const uint4*>(q_step), static_cast<uint4*>(q_cache));
  return hipGetLastError();
}

}  // namespace laq
