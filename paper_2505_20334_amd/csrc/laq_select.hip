// Per-KV-head selection: the "ArgSort(...)[:B]" of Eq. 4 done as a radix select (no sort).
//
// One workgroup of 16 waves ranks the prefix scores of one (instance, KV head).  Scores
// are mapped to order-preserving 32-bit keys; four most-significant-digit-first passes
// over 8-bit digits find the key T of the k-th largest score and how many keys equal to
// T still fit (ties go to the lower position).  A last sweep emits, in ascending
// position order, every key above T plus the first `want` keys equal to T, then the `keep`
// window positions.  Keys live in registers (each wave owns a contiguous segment of the
// prefix, 64 consecutive positions per register row -- or, where the scores need no pooling
// here and lie 16-byte aligned, 256 consecutive positions per four registers, a lane holding
// four neighbours that it fetched with one load) for prefixes up to 32768; longer prefixes
// re-read the scores from memory in every pass.
#include "laq_internal.h"

namespace laq {

namespace {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_MANY_WORKGROUPS = 768;   // from here on two workgroups per compute unit pay off

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);   // larger float <=> larger key
}

__device__ __forceinline__ int lanes_below(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// ITEMS > 0: keys of the wave's segment are held in ITEMS registers per lane.
// ITEMS == 0: keys are recomputed from memory on every sweep (any prefix length).
// WAVES_PER_SIMD = 4: one workgroup per compute unit, up to 128 registers per lane; 8: two workgroups
// per compute unit on 64 registers (the 32-key variant then spills a few of them, which costs
// 12 % when there is one workgroup per compute unit anyway and gains 30 % when there are many).
// QUADS: register 4q + c of a lane holds position seg0 + 256 q + 4 lane + c (one 16-byte load per q).
template <int ITEMS, int WAVES_PER_SIMD, bool QUADS>
__global__ __launch_bounds__(SEL_THREADS, WAVES_PER_SIMD) void select_kernel(int Hkv, int L, int keep, int pool, bool avg,
                                                             const float* __restrict__ scores, InstTable tab,
                                                             int inst0, int32_t* __restrict__ idx) {
  __shared__ int hist[256];
  __shared__ int sh_bin, sh_above;
  __shared__ int wtot_gt[SEL_WAVES], wtot_eq[SEL_WAVES];

  const int head = blockIdx.x, li = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int P = L - keep, half = (pool - 1) / 2;
  const int bk = tab.bk[li];
  const int ksel = bk - keep;
  const float* s = scores + ((size_t)(inst0 + li) * Hkv + head) * L;
  int32_t* out = idx + (tab.row0[li] + (int64_t)head * bk);

  for (int w = tid; w < keep; w += SEL_THREADS) out[ksel + w] = P + w;
  if (ksel <= 0) return;
  if (ksel >= P) {
    for (int j = tid; j < P; j += SEL_THREADS) out[j] = j;
    return;
  }

  constexpr int UNROLL = ITEMS > 0 ? ITEMS : 1;     // register-resident keys: full unrolling; memory path: none
  const int items = (ITEMS > 0) ? ITEMS : (P + SEL_THREADS - 1) / SEL_THREADS;
  const int seg0 = wave * items * 64;          // first position of this wave's segment

  static_assert(!QUADS || (ITEMS > 0 && ITEMS % 4 == 0), "four registers per load");
  uint32_t key[ITEMS > 0 ? ITEMS : 1];
  if constexpr (QUADS) {
#pragma unroll
    for (int q4 = 0; q4 < ITEMS / 4; ++q4) {
      const int pos = seg0 + q4 * 256 + lane * 4;
      if (pos + 3 < P) {
        const float4 v = *reinterpret_cast<const float4*>(s + pos);
        key[4 * q4] = order_key(v.x); key[4 * q4 + 1] = order_key(v.y);
        key[4 * q4 + 2] = order_key(v.z); key[4 * q4 + 3] = order_key(v.w);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) key[4 * q4 + c] = (pos + c < P) ? order_key(s[pos + c]) : 0u;
      }
    }
  } else if (ITEMS > 0) {
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int pos = seg0 + i * 64 + lane;
      key[i] = (pos < P) ? order_key(pool_window(s, pos, P, half, avg)) : 0u;
    }
  }
  auto key_of = [&](int i) -> uint32_t {
    if (ITEMS > 0) return key[i];
    const int pos = seg0 + i * 64 + lane;
    return (pos < P) ? order_key(pool_window(s, pos, P, half, avg)) : 0u;
  };

  // ---- radix passes: find the key of the ksel-th largest score ----
  uint32_t prefix = 0, mask = 0;
  int want = ksel;
#pragma unroll 1
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    int cur = -1, cnt = 0;            // run-length aggregation: one atomic per run of equal digits
#pragma unroll UNROLL
    for (int i = 0; i < items; ++i) {
      const uint32_t kv = key_of(i);
      if ((kv & mask) == prefix) {
        const int dg = (kv >> shift) & 255;
        if (dg == cur) {
          ++cnt;
        } else {
          if (cnt) atomicAdd(&hist[cur], cnt);
          cur = dg;
          cnt = 1;
        }
      }
    }
    if (cnt) atomicAdd(&hist[cur], cnt);
    __syncthreads();
    if (wave == 0) {
      // lane l covers bins 255-4l .. 252-4l (descending); scan from the top
      const int h0 = hist[255 - 4 * lane], h1 = hist[254 - 4 * lane];
      const int h2 = hist[253 - 4 * lane], h3 = hist[252 - 4 * lane];
      const int sum = h0 + h1 + h2 + h3;
      int incl = sum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      const int excl = incl - sum;
      if (excl < want && want <= incl) {
        int a = excl, bin = 255 - 4 * lane;
        if (a + h0 < want) { a += h0; --bin;
          if (a + h1 < want) { a += h1; --bin;
            if (a + h2 < want) { a += h2; --bin; } } }
        sh_bin = bin;
        sh_above = a;
      }
    }
    __syncthreads();
    want -= sh_above;
    prefix |= (uint32_t)sh_bin << shift;
    mask |= 0xFFu << shift;
  }
  const uint32_t T = prefix;      // key of the ksel-th largest; take `want` of the keys equal to T

  // ---- emission in ascending position order ----
  int wg = 0, we = 0;
#pragma unroll UNROLL
  for (int i = 0; i < items; ++i) {
    const uint32_t kv = key_of(i);
    wg += __popcll(__ballot(kv > T));
    we += __popcll(__ballot(kv == T));
  }
  if (lane == 0) { wtot_gt[wave] = wg; wtot_eq[wave] = we; }
  __syncthreads();
  int run_gt = 0, run_eq = 0;
  for (int v = 0; v < wave; ++v) { run_gt += wtot_gt[v]; run_eq += wtot_eq[v]; }
  if constexpr (QUADS) {
    // ascending positions = (q, lane, c): before a lane's four come those of the lower lanes
#pragma unroll
    for (int q4 = 0; q4 < ITEMS / 4; ++q4) {
      uint64_t mg[4], me[4];
      int g_before = run_gt, e_before = run_eq;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        mg[c] = __ballot(key[4 * q4 + c] > T);
        me[c] = __ballot(key[4 * q4 + c] == T);
        g_before += lanes_below(mg[c]);
        e_before += lanes_below(me[c]);
        run_gt += __popcll(mg[c]);
        run_eq += __popcll(me[c]);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t kv = key[4 * q4 + c];
        const bool gt = kv > T, eq = kv == T;
        if (gt || (eq && e_before < want)) out[g_before + min(e_before, want)] = seg0 + q4 * 256 + lane * 4 + c;
        g_before += gt;
        e_before += eq;
      }
    }
    return;
  }
#pragma unroll UNROLL
  for (int i = 0; i < items; ++i) {
    const uint32_t kv = key_of(i);
    const bool gt = kv > T, eq = kv == T;
    const uint64_t mg = __ballot(gt), me = __ballot(eq);
    const int g_before = run_gt + lanes_below(mg);
    const int e_before = run_eq + lanes_below(me);
    if (gt || (eq && e_before < want)) out[g_before + min(e_before, want)] = seg0 + i * 64 + lane;
    run_gt += __popcll(mg);
    run_eq += __popcll(me);
  }
}

template <int ITEMS>
hipError_t launch_one(int n_inst, int inst0, int Hkv, int L, int keep, int pool, bool avg, const float* scores,
                      const InstTable& tab, int32_t* idx, hipStream_t st) {
  // scores that are final (no pooling here) and whose rows start 16-byte aligned: four per load
  constexpr bool CAN_QUAD = ITEMS > 0 && ITEMS % 4 == 0;
  const bool quads = CAN_QUAD && pool == 1 && L % 4 == 0 && reinterpret_cast<uintptr_t>(scores) % 16 == 0;
  const bool many = (long long)Hkv * n_inst >= SEL_MANY_WORKGROUPS;
  const dim3 grid(Hkv, n_inst), block(SEL_THREADS);
  if constexpr (CAN_QUAD) {
    if (quads) {
      if (many) hipLaunchKernelGGL((select_kernel<ITEMS, 8, true>), grid, block, 0, st, Hkv, L, keep, pool, avg, scores, tab, inst0, idx);
      else hipLaunchKernelGGL((select_kernel<ITEMS, 4, true>), grid, block, 0, st, Hkv, L, keep, pool, avg, scores, tab, inst0, idx);
      return hipGetLastError();
    }
  }
  if (many) hipLaunchKernelGGL((select_kernel<ITEMS, 8, false>), grid, block, 0, st, Hkv, L, keep, pool, avg, scores, tab, inst0, idx);
  else hipLaunchKernelGGL((select_kernel<ITEMS, 4, false>), grid, block, 0, st, Hkv, L, keep, pool, avg, scores, tab, inst0, idx);
  return hipGetLastError();
}

// Score-free list (Sec. 2.1, StreamingLLM form): row = 0 .. s-1, then the Bk - s most recent
// positions, s = min(n_sink, Bk).  One workgroup per (KV head, instance).
__global__ __launch_bounds__(256) void sink_recent_kernel(int Hkv, int L, int n_sink, InstTable tab,
                                                          int32_t* __restrict__ idx) {
  const int head = blockIdx.x, li = blockIdx.y;
  const int bk = tab.bk[li];
  const int s = min(n_sink, bk);
  const int shift = L - bk;                 // recent entry at list slot t sits at position t + (L - Bk)
  int32_t* out = idx + (tab.row0[li] + (int64_t)head * bk);
  for (int t = threadIdx.x; t < bk; t += 256) out[t] = t < s ? t : t + shift;
}

}  // namespace

hipError_t launch_sink_recent(int n_inst, int Hkv, int L, int n_sink, const InstTable& tab, int32_t* idx,
                              hipStream_t st) {
  hipLaunchKernelGGL(sink_recent_kernel, dim3(Hkv, n_inst), dim3(256), 0, st, Hkv, L, n_sink, tab, idx);
  return hipGetLastError();
}

hipError_t launch_select(int n_inst, int inst0, int Hkv, int L, int keep, int pool, bool avg, const float* scores,
                         const InstTable& tab, int32_t* idx, hipStream_t st) {
  const int P = L - keep;
  if (P <= 2 * SEL_THREADS) return launch_one<2>(n_inst, inst0, Hkv, L, keep, pool, avg, scores, tab, idx, st);
  if (P <= 8 * SEL_THREADS) return launch_one<8>(n_inst, inst0, Hkv, L, keep, pool, avg, scores, tab, idx, st);
  if (P <= 32 * SEL_THREADS) return launch_one<32>(n_inst, inst0, Hkv, L, keep, pool, avg, scores, tab, idx, st);
  return launch_one<0>(n_inst, inst0, Hkv, L, keep, pool, avg, scores, tab, idx, st);
}

}  // namespace laq
