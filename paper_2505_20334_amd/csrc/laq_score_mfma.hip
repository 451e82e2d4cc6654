// bf16 scoring path on the matrix cores (gfx950, v_mfma_f32_32x32x16_bf16).
//
// For one KV head the logits of Eq. 4's observation window form a skinny product
// S = Q_g K^T with R = G*W rows (the group's query heads x the cached window queries)
// and L columns.  A workgroup of four waves holds MFMA_ROWS key rows in LDS and walks
// them in 32-key tiles:
//
//   pass 1 (statistics):  D = K_tile * Q^T, so a lane owns one score row and 16 keys of
//           the tile; it keeps a running (max, sum-exp) for its row.  The two lanes that
//           share a row and the waves that share a row tile are merged through LDS and the
//           chunk's (m, z) per row is published.
//   pass 2 (normalise + sum + pool): D = Q * K_tile^T, so a lane owns one key and 16 rows;
//           with the row constants c = M + log2 Z the probabilities exp2(s - c) are summed over
//           the rows in-lane, across the two lane halves with one cross-lane add and across row
//           tiles through LDS.  The sequence max-pool of every key whose window lies inside
//           the chunk is taken right there; the few keys next to a chunk boundary are pooled
//           by a small kernel afterwards, from raw scores that the chunks leave for it.
//
// The A and B operands of the 32x32x16 instruction have the same lane layout (lane l
// supplies row/column l%32 and the 8 consecutive reduction elements l/32), so the same
// registers serve both passes with the operands swapped.
//
// Each pass is one launch of persistent workgroups that stream runs of consecutive chunks:
// while a chunk is being worked on in LDS, the next chunk's key rows are already on their way
// into registers; Q and the row constants are loaded once per head.  Between the passes a
// small kernel combines the per-chunk statistics of every head.  K is therefore read twice.
// (A single-read variant has to keep a head's keys on chip while all its chunks meet between
// the passes; on this part that device-wide meeting costs more than the second read.)
#include <atomic>
#include <type_traits>

#include "laq_internal.h"

namespace laq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16 bytes of key data in flight between HBM and LDS.  A native vector (not HIP's uint4 class):
// arrays of it are promoted to registers reliably, copies of the class type become memcpy calls
// that can pin the whole array to stack memory.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float NEG_BIG = -1.0e30f;
constexpr int MAX_HALF = (MAX_POOL - 1) / 2;
constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int KTILES = MFMA_ROWS / 32;
#ifndef LAQ_MFMA_BLOCKS
#define LAQ_MFMA_BLOCKS 2
#endif
constexpr int MFMA_BLOCKS = LAQ_MFMA_BLOCKS;       // workgroups per compute unit the kernels are built for

#ifndef LAQ_LDS_AHEAD
#define LAQ_LDS_AHEAD 2
#endif
constexpr int LDS_AHEAD = LAQ_LDS_AHEAD;          // MFMA operands requested from LDS this many MFMAs ahead

// LDS row stride: the key row plus 16 bytes, so that the 16 lanes of a 128-bit LDS read
// phase (rows r .. r+15, same column) fall on 16 distinct 4-bank groups.
template <int D> struct Tile {
  static constexpr int ROWB = D * 2 + 16;
  static constexpr int KSTEPS = D / 16;
  static constexpr int PIECES_PER_ROW = D / 8;                         // 16-byte pieces
  static constexpr int PIECES_PER_THREAD = MFMA_ROWS * PIECES_PER_ROW / THREADS;
  static constexpr int K_BYTES = MFMA_ROWS * ROWB;
};

template <int D, int NRT> struct Smem {
  static constexpr int OFF_STAT = Tile<D>::K_BYTES;                    // float2[THREADS]: pass 1's per-thread statistics;
                                                                       // pass 2: the chunk's raw scores with a zero margin
  static constexpr int OFF_SLOT = OFF_STAT + THREADS * 8;              // float[NRT][MFMA_ROWS]
  static constexpr int OFF_CTL = OFF_SLOT + NRT * MFMA_ROWS * 4;      // int: the workgroup's next run of units
  static constexpr int BYTES = OFF_CTL + 16;
};

#define LAQ_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
// Forces `v` to be complete at this point of the instruction stream.  The scheduling fence
// alone does not hold arithmetic in its slot: instruction selection is free to sink pure
// computations down to their first use, across fences.
#define LAQ_PIN(v) asm volatile("" : "+v"(v))

// compile-time loop: f(std::integral_constant<int, I>) for I = FROM .. TO-1.  Used where an index
// must be a constant before the optimiser runs (register arrays that must never become stack).
template <int FROM, int TO, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FROM < TO) {
    f(std::integral_constant<int, FROM>{});
    static_for<FROM + 1, TO>(f);
  }
}

// Key rows j0 .. j0+MFMA_ROWS-1 (j0 >= 0) of one head travel HBM -> registers -> LDS in 16-byte
// pieces.  A thread owns one 16-byte column of PIECES_PER_THREAD consecutive rows, so its
// loads differ only in an immediate offset and the 16 (8) lanes that share a row read it
// contiguously.  The loads are buffer loads against a descriptor that spans exactly the head's
// L rows: the hardware range check returns zeros for rows beyond L-1 (they are causally
// masked), without address clamping.  The host guarantees (L + chunk) * D * 2 < 2^31.
struct KeyRows {
  __amdgpu_buffer_rsrc_t rsrc;
  int voff;                // byte offset of this thread's first piece within the head
};
// The same for a cache whose rows are not adjacent (e.g. token-major [L, Hkv, d]): the distance
// between rows is a run-time value, so the row offsets are added in registers instead of riding in
// the immediate field.  They are added to the vector offset, which the range check covers (a
// scalar offset operand would not be checked).  The descriptor ends with the head's last row.
struct KeyRowsStrided {
  __amdgpu_buffer_rsrc_t rsrc;
  int voff;
  int row_bytes;           // distance between consecutive key rows of the head
};

template <int D>
__device__ __forceinline__ KeyRows key_rows(const uint16_t* khead, int j0, int L, int tid) {
  using T = Tile<D>;
  KeyRows kr;
  kr.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(khead), 0, L * D * 2, 0x00020000);
  kr.voff = (j0 + (tid / T::PIECES_PER_ROW) * T::PIECES_PER_THREAD) * (D * 2) + (tid % T::PIECES_PER_ROW) * 16;
  return kr;
}

template <int D>
__device__ __forceinline__ KeyRowsStrided key_rows_strided(const uint16_t* khead, int j0, int L, int tid,
                                                           int row_bytes) {
  using T = Tile<D>;
  KeyRowsStrided kr;
  kr.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(khead), 0, (L - 1) * row_bytes + D * 2,
                                              0x00020000);
  kr.voff = (j0 + (tid / T::PIECES_PER_ROW) * T::PIECES_PER_THREAD) * row_bytes + (tid % T::PIECES_PER_ROW) * 16;
  kr.row_bytes = row_bytes;
  return kr;
}

template <int D>
__device__ __forceinline__ u32x4 load_piece(const KeyRows& kr, int voff, int it) {
  return __builtin_amdgcn_raw_buffer_load_b128(kr.rsrc, voff + it * (D * 2), 0, 0);
}
template <int D>
__device__ __forceinline__ u32x4 load_piece(const KeyRowsStrided& kr, int voff, int it) {
  return __builtin_amdgcn_raw_buffer_load_b128(kr.rsrc, voff + it * kr.row_bytes, 0, 0);
}

// The thread's byte offset, made opaque to the optimiser at the point of use: the row
// offsets added to it then stay next to their loads and fold into the instructions'
// immediate fields, instead of being precomputed into one live register per piece.
template <typename KR>
__device__ __forceinline__ int local_offset(const KR& kr) {
  int v = kr.voff;
  asm volatile("" : "+v"(v));
  return v;
}

template <int D, typename KR>
__device__ __forceinline__ void fetch_chunk(u32x4 (&buf)[Tile<D>::PIECES_PER_THREAD], const KR kr) {
  const int v = local_offset(kr);
#pragma unroll
  for (int it = 0; it < Tile<D>::PIECES_PER_THREAD; ++it) buf[it] = load_piece<D>(kr, v, it);
}

template <int D>
__device__ __forceinline__ void commit_chunk(char* ldsK, const u32x4 (&buf)[Tile<D>::PIECES_PER_THREAD], int tid) {
  using T = Tile<D>;
  char* dst = ldsK + (tid / T::PIECES_PER_ROW) * T::PIECES_PER_THREAD * T::ROWB + (tid % T::PIECES_PER_ROW) * 16;
#pragma unroll
  for (int it = 0; it < T::PIECES_PER_THREAD; ++it) *reinterpret_cast<u32x4*>(dst + it * T::ROWB) = buf[it];
}

// Row index (0..31) of accumulator register i for a lane in half hf (32x32 output layout:
// groups of four consecutive rows alternate between the two lane halves).
__device__ __forceinline__ int acc_row(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

// Operand registers of one 32-row tile of Q_g (rows beyond R are zero).
template <int D>
__device__ __forceinline__ void load_q_tile(bf16x8 (&qreg)[Tile<D>::KSTEPS], const uint16_t* __restrict__ qg,
                                            int rt, int R, int lane) {
  const int r = rt * 32 + (lane & 31);
#pragma unroll
  for (int t = 0; t < Tile<D>::KSTEPS; ++t) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < R) v = *reinterpret_cast<const u32x4*>(qg + (size_t)r * D + (2 * t + (lane >> 5)) * 8);
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

__device__ __forceinline__ void merge_stat(float& M, float& Z, float2 p) {
  const float Mn = fmaxf(M, p.x);
  Z = Z * __builtin_amdgcn_exp2f(M - Mn) + p.y * __builtin_amdgcn_exp2f(p.x - Mn);
  M = Mn;
}

// ---- software-pipelined passes for chunks without causally masked keys -----------------
// The MFMA chain of key tile i+1 is issued one instruction at a time, each followed by a
// slice of the VALU work of tile i, so that the matrix pipe and the vector ALU run
// concurrently inside one wave; LDS operands are fetched LDS_AHEAD MFMAs ahead (deeper did
// not measure faster: the loop is bound by VALU issue, about 89 issue slots per tile, not by
// LDS latency).  The scheduling fences and value pins hold that interleaving.
// With PREFETCH the wave also requests its share of the workgroup's next chunk, one 16-byte piece
// at a time, spread evenly over its MFMA slots: the requests then trickle out at the rate the
// texture path accepts them instead of blocking the wave in front of its arithmetic (all of them
// up front measured 2.5 % slower, all in the first quarter of the slots 0.7 % slower).
// (plain fmaxf, which the compiler fuses into three-input maxima: hand-written instructions on
// accumulator registers would bypass the wait states it inserts between an MFMA and the first
// read of its result)
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <int D, int NT, bool PREFETCH, typename KR>
__device__ __forceinline__ void pass1_pipe(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS], int kt0,
                                           float scale2, int lane, float& m_run, float& z_run,
                                           u32x4 (&pre)[Tile<D>::PIECES_PER_THREAD], const KR& nkr) {
  using T = Tile<D>;
  constexpr int KS = T::KSTEPS, N = NT * KS;
  static_assert(LDS_AHEAD <= N, "operand prefetch deeper than the wave's share of a chunk");
  static_assert(N % T::PIECES_PER_THREAD == 0, "the requests for the next chunk are spread evenly over the MFMA slots");
  constexpr int EVERY = N / T::PIECES_PER_THREAD;   // one request per EVERY slots
  const char* base = ldsK + (kt0 * 32 + (lane & 31)) * T::ROWB + (lane >> 5) * 16;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int voff = PREFETCH ? local_offset(nkr) : 0;
  bf16x8 ring[LDS_AHEAD];
#pragma unroll
  for (int n = 0; n < LDS_AHEAD; ++n) ring[n] = lds_operand(base + (n / KS) * 32 * T::ROWB + (n % KS) * 32);
  // running maximum of the raw dot products (the logit scale is positive, so the order is the
  // same); m_run enters as "nothing seen yet"
  float raw_max = -3.0e38f;
  f32x16 cur = zero, nxt = zero;
  static_for<0, NT + 1>([&](auto I) {
    constexpr int i = decltype(I)::value;
    float m_new = m_run, s = 0.f;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      const int n = i * KS + t;
      if (i < NT) {
        nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % LDS_AHEAD], qreg[t], (t > 0) ? nxt : zero, 0, 0, 0);
        const int f = n + LDS_AHEAD;
        if (f < N) ring[n % LDS_AHEAD] = lds_operand(base + (f / KS) * 32 * T::ROWB + (f % KS) * 32);
        if (PREFETCH && n % EVERY == 0) pre[n / EVERY] = load_piece<D>(nkr, voff, n / EVERY);
      }
      if (i > 0) {
        if (t == 0) {
          float mx = max3(raw_max, cur[0], cur[1]);
#pragma unroll
          for (int e = 2; e < 16; e += 2) mx = max3(mx, cur[e], cur[e + 1]);
          raw_max = mx;
          m_new = mx * scale2;
          LAQ_PIN(m_new);
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
          LAQ_PIN(s);
        }
      }
      LAQ_SCHED_FENCE();
    }
    if (i > 0) {
      z_run = fmaf(z_run, __builtin_amdgcn_exp2f(m_run - m_new), s);
      m_run = m_new;
    }
    cur = nxt;
  });
}

// `first`: this call's sums start the chunk's slot buffer (they are stored); otherwise they are added.
template <int D, int NT, bool PREFETCH, typename KR>
__device__ __forceinline__ void pass2_pipe(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS], int kt0,
                                           const float (&c)[16], float scale2, int lane, float* slotbuf, bool first,
                                           u32x4 (&pre)[Tile<D>::PIECES_PER_THREAD], const KR& nkr) {
  using T = Tile<D>;
  constexpr int KS = T::KSTEPS, N = NT * KS, PER = 16 / KS;
  static_assert(LDS_AHEAD <= N, "operand prefetch deeper than the wave's share of a chunk");
  static_assert(N % T::PIECES_PER_THREAD == 0, "the requests for the next chunk are spread evenly over the MFMA slots");
  constexpr int EVERY = N / T::PIECES_PER_THREAD;   // one request per EVERY slots
  const int hf = lane >> 5, n32 = lane & 31;
  const char* base = ldsK + (kt0 * 32 + n32) * T::ROWB + hf * 16;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int voff = PREFETCH ? local_offset(nkr) : 0;
  bf16x8 ring[LDS_AHEAD];
#pragma unroll
  for (int n = 0; n < LDS_AHEAD; ++n) ring[n] = lds_operand(base + (n / KS) * 32 * T::ROWB + (n % KS) * 32);
  f32x16 cur = zero, nxt = zero;
  static_for<0, NT + 1>([&](auto I) {
    constexpr int i = decltype(I)::value;
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      const int n = i * KS + t;
      if (i < NT) {
        nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[t], ring[n % LDS_AHEAD], (t > 0) ? nxt : zero, 0, 0, 0);
        const int f = n + LDS_AHEAD;
        if (f < N) ring[n % LDS_AHEAD] = lds_operand(base + (f / KS) * 32 * T::ROWB + (f % KS) * 32);
        if (PREFETCH && n % EVERY == 0) pre[n / EVERY] = load_piece<D>(nkr, voff, n / EVERY);
      }
      if (i > 0) {
        float x[16];
#pragma unroll
        for (int e = t * PER; e < (t + 1) * PER; ++e) x[e] = fmaf(cur[e], scale2, -c[e]);
#pragma unroll
        for (int e = t * PER; e < (t + 1) * PER; ++e) x[e] = __builtin_amdgcn_exp2f(x[e]);
#pragma unroll
        for (int e = t * PER; e < (t + 1) * PER; ++e) s += x[e];
        LAQ_PIN(s);
      }
      LAQ_SCHED_FENCE();
    }
    if (i > 0) {
      s += __shfl_xor(s, 32);
      if (hf == 0) {
        float* dst = slotbuf + (kt0 + i - 1) * 32 + n32;
        *dst = first ? s : *dst + s;
      }
    }
    cur = nxt;
  });
}

// ---- per-tile passes for chunks with keys that some window query does not see ----------------
// (with the trailing-window layout: the last chunks of a head).  Query w of the window sees keys
// j <= last_visible_key(w); a masked logit enters as -inf through the accumulator's initial value.
template <int D>
__device__ __forceinline__ void pass1_masked(const char* ldsK, const bf16x8 (&qreg)[Tile<D>::KSTEPS],
                                             const ScoreGeom& g, const QueryPos& qp, int rt, int kt0, int kt1,
                                             int j0, int lane, float& m_run, float& z_run) {
  const int hf = lane >> 5;
  const int w = (rt * 32 + (lane & 31)) % g.W;
  const int t_hi = qp.last[w] - j0;       // last staged row this lane's score row may see
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kt = kt0; kt < kt1; ++kt) {
    const int t0 = kt * 32;
    f32x16 acc;
    if (j0 + t0 + 31 > g.qmin) {
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
                                             const ScoreGeom& g, const QueryPos& qp, const float (&c)[16], int rt,
                                             int kt0, int kt1, int j0, int lane, float* slotbuf, bool first) {
  const int hf = lane >> 5, n = lane & 31;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kt = kt0; kt < kt1; ++kt) {
    const int t0 = kt * 32;
    f32x16 acc;
    if (j0 + t0 + 31 > g.qmin) {
      f32x16 bias;
      const int j = j0 + t0 + n;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int w = (rt * 32 + acc_row(i, hf)) % g.W;
        bias[i] = (j <= qp.last[w]) ? 0.f : -INFINITY;
      }
      acc = tile_product<D, false>(ldsK, kt, lane, qreg, bias);
    } else {
      acc = tile_product<D, false>(ldsK, kt, lane, qreg, zero);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += __builtin_amdgcn_exp2f(fmaf(acc[i], g.scale2, -c[i]));
    s += __shfl_xor(s, 32);
    if (hf == 0) slotbuf[t0 + n] = first ? s : slotbuf[t0 + n] + s;
  }
}

// ---- one chunk ----------------------------------------------------------------------------
// Both passes walk the score rows in groups of NRT 32-row tiles, one tile per wave slot.  The
// wave's Q operands (and, in pass 2, its row constants) live in registers owned by the caller:
// with a single row group they stay valid for as long as the workgroup stays on one head and
// are only loaded when `reload` is set; with several row groups every group loads its own.

// Both return with every wave's LDS reads of the key rows complete (their last barrier comes
// after them), so the caller may overwrite the rows at once.  The row group that runs first
// also requests the key rows of the workgroup's next chunk (nkr) into `pre`.

// Pass 1 over the staged chunk (keys j0 .. j0+MFMA_ROWS-1): (m, z) of every score row goes to
// out[0 .. Rpad).  The statistics of the last row group are handed back instead (returns true if
// this thread holds one, for out[idx_out]): the caller stores them after it has moved the next
// chunk's rows into LDS, so that the wait for those rows is not also a wait for the store.
template <int D, int NRT, typename KR>
__device__ __forceinline__ bool chunk_pass1(char* smem, const ScoreGeom& g, const QueryPos& qp,
                                            const uint16_t* __restrict__ qg,
                                            bf16x8 (&qreg)[Tile<D>::KSTEPS], bool reload, int j0, int tid, int lane,
                                            int wave, float2* __restrict__ out, int& idx_out, float2& mz_out,
                                            u32x4 (&pre)[Tile<D>::PIECES_PER_THREAD], const KR& nkr) {
  using S = Smem<D, NRT>;
  constexpr int KSPLIT = WAVES / NRT, TPW = KTILES / KSPLIT;
  bool pending = false;
  float2* stat = reinterpret_cast<float2*>(smem + S::OFF_STAT);
  const int slot = wave % NRT, ks = wave / NRT;
  const int ntile = g.Rpad / 32;
  const bool plain_chunk = (j0 + MFMA_ROWS - 1 <= g.qmin);  // every window query sees every key of the chunk
  for (int rg = 0; rg * NRT < ntile; ++rg) {
    const int rt = rg * NRT + slot;
    float m_run = NEG_BIG, z_run = 0.f;
    if (rg > 0) __syncthreads();                             // the previous group's statistics have been merged
    if (rt < ntile) {
      if (reload) load_q_tile<D>(qreg, qg, rt, g.R, lane);
      if (plain_chunk) {
        if (rg == 0)
          pass1_pipe<D, TPW, true>(smem, qreg, ks * TPW, g.scale2, lane, m_run, z_run, pre, nkr);
        else
          pass1_pipe<D, TPW, false>(smem, qreg, ks * TPW, g.scale2, lane, m_run, z_run, pre, nkr);
      } else {
        if (rg == 0) fetch_chunk<D>(pre, nkr);
        pass1_masked<D>(smem, qreg, g, qp, rt, ks * TPW, ks * TPW + TPW, j0, lane, m_run, z_run);
      }
    } else if (rg == 0) {
      fetch_chunk<D>(pre, nkr);                              // a wave without a row tile still fetches its share
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
        if ((rg + 1) * NRT < ntile) {
          out[(rg * NRT + s) * 32 + n] = make_float2(M, Z);
        } else {
          pending = true;
          idx_out = (rg * NRT + s) * 32 + n;
          mz_out = make_float2(M, Z);
        }
      }
    }
  }
  return pending;
}

// Pass 2 over the staged chunk (staged row t is key j0 + t, j0 a multiple of the chunk size): raw
// scores of its rows.  Returns whether this thread has a score to store (index j_out, raw value
// v_out); the caller stores it after it has moved the next chunk's rows into LDS, so that the wait
// for those rows is not also a wait for the store.  With pool_out set the stored value is the
// maximum over the key's pooling window instead, which pooled_score() takes from the copy of the
// raw scores left in LDS once the caller has passed a barrier.  A prefix key whose pooling window
// reaches into a neighbouring chunk is left out here: with `edges` set, the raw scores of the
// chunk's first and last 2*half rows are handed back as well (slot e_out of the chunk's edge
// record, value r_out, when the function sets edge_out) and pool_boundaries_kernel pools those
// keys from the records.  c points at the head's row constants.
template <int D, int NRT, typename KR>
__device__ __forceinline__ bool chunk_pass2(char* smem, const ScoreGeom& g, const QueryPos& qp, int half,
                                            bool edges,
                                            const uint16_t* __restrict__ qg, const float* __restrict__ c,
                                            bf16x8 (&qreg)[Tile<D>::KSTEPS], float (&cr)[16], bool reload, int j0,
                                            int tid, int lane, int wave, int& j_out, float& v_out,
                                            bool& pool_out, bool& edge_out, int& e_out, float& r_out,
                                            u32x4 (&pre)[Tile<D>::PIECES_PER_THREAD], const KR& nkr) {
  using S = Smem<D, NRT>;
  constexpr int KSPLIT = WAVES / NRT, TPW = KTILES / KSPLIT;
  float* slots = reinterpret_cast<float*>(smem + S::OFF_SLOT);
  const int slot = wave % NRT, ks = wave / NRT;
  const int ntile = g.Rpad / 32;
  const bool plain_chunk = (j0 + MFMA_ROWS - 1 <= g.qmin);
  // every (slot, key tile) cell of the slot buffer belongs to exactly one wave; a slot whose first
  // row tile does not exist (fewer tiles than slots) is cleared by its wave instead
  if (slot >= ntile) {
    for (int t = lane; t < TPW * 32; t += 64) slots[slot * MFMA_ROWS + ks * TPW * 32 + t] = 0.f;
    fetch_chunk<D>(pre, nkr);
  }
  for (int rg = 0; rg * NRT < ntile; ++rg) {
    const int rt = rg * NRT + slot;
    if (rt < ntile) {
      if (reload) {
        load_q_tile<D>(qreg, qg, rt, g.R, lane);
#pragma unroll
        for (int i = 0; i < 16; ++i) cr[i] = c[rt * 32 + acc_row(i, lane >> 5)];
      }
      float* myslot = slots + slot * MFMA_ROWS;
      if (plain_chunk) {
        if (rg == 0)
          pass2_pipe<D, TPW, true>(smem, qreg, ks * TPW, cr, g.scale2, lane, myslot, true, pre, nkr);
        else
          pass2_pipe<D, TPW, false>(smem, qreg, ks * TPW, cr, g.scale2, lane, myslot, false, pre, nkr);
      } else {
        if (rg == 0) fetch_chunk<D>(pre, nkr);
        pass2_masked<D>(smem, qreg, g, qp, cr, rt, ks * TPW, ks * TPW + TPW, j0, lane, myslot, rg == 0);
      }
    }
  }
  __syncthreads();                        // slots complete, key rows no longer read
  // raw score of staged row t = sum of the row-tile slots
  const int j = j0 + tid;
  j_out = j;
  v_out = 0.f;
  edge_out = false;
  e_out = 0;
  r_out = 0.f;
  bool owned = tid < MFMA_ROWS && j < g.L;
  float v = 0.f;
  if (tid < MFMA_ROWS) {
    v = slots[tid];
#pragma unroll
    for (int s = 1; s < NRT; ++s) v += slots[s * MFMA_ROWS + tid];
  }
  pool_out = false;
  if (half > 0) {
    // Pooling reads the raw scores through a copy with MAX_HALF zeros on either side (the zeros
    // were written when the kernel started), in which the keys outside the prefix are zero too:
    // scores are sums of probabilities, never negative, so a zero stands for "not in the window"
    // and every window position can be read without a bounds test.  The copy is complete at the
    // caller's next barrier; pooled_score() reads it then.
    float* rawbuf = reinterpret_cast<float*>(smem + S::OFF_STAT) + MAX_HALF;
    if (tid < MFMA_ROWS) rawbuf[tid] = j < g.P ? v : 0.f;
    if (owned) {
      if (edges) {
        r_out = v;
        if (tid < 2 * half) {
          edge_out = true;
          e_out = tid;
        } else if (tid >= MFMA_ROWS - 2 * half) {
          edge_out = true;
          e_out = tid - (MFMA_ROWS - 4 * half);
        }
      }
      if (j < g.P) {
        if ((j0 > 0 && tid < half) || min(j + half, g.P - 1) >= j0 + MFMA_ROWS)
          owned = false;                  // the window reaches into a neighbouring chunk
        else
          pool_out = true;
      }
    }
  }
  v_out = v;
  return owned;
}

// Maximum of the raw scores in the pooling window of staged row tid, from the zero-margined copy
// that chunk_pass2 left in LDS (call after a barrier that follows it).
template <int D, int NRT>
__device__ __forceinline__ float pooled_score(const char* smem, int half, int tid, float v) {
  const float* rawbuf = reinterpret_cast<const float*>(smem + Smem<D, NRT>::OFF_STAT) + MAX_HALF;
  if (half == 3) {
    float r[7];                           // the usual kernel of 7: all reads issued at once
#pragma unroll
    for (int o = 0; o < 7; ++o) r[o] = rawbuf[tid + o - 3];
#pragma unroll
    for (int o = 0; o < 7; ++o) v = fmaxf(v, r[o]);
  } else {
    for (int o = -half; o <= half; ++o) v = fmaxf(v, rawbuf[tid + o]);
  }
  return v;
}

// ---- the two streaming kernels ---------------------------------------------------------------
// PASS 1: units are (head, chunk of 256 keys); writes part[head][chunk][row].
// PASS 2: units are (head, chunk of 256 keys); reads rowc[head][row], writes scores and, through
//         `part`, the edge records float[head][chunk][4*half] of the pooling across chunk boundaries.
//
// A workgroup works through runs of consecutive units, i.e. it walks along one head, so Q and
// the row constants are loaded once per head and the only per-unit traffic is the key rows.  Its
// first run is a fixed share of `static_units` units; the units beyond static_units * gridDim.x
// are handed out in runs of RUN_UNITS through a counter, because the two workgroups that share
// a compute unit do not progress at the same speed (the older one wins instruction arbitration)
// and a purely static split leaves half the machine idle at the end.  The next run is claimed
// at the start of the current one, so the counter's round trip is never waited for.
// The next unit's key rows are requested during the current unit's arithmetic and stay in
// flight, in registers, for its whole duration.
constexpr int RUN_UNITS = 4;

struct StreamPlan {
  int units_per_head;      // units along one head
  int n_units;             // all units of the launch
  int static_units;        // units of every workgroup's first run
  int dynamic;             // 1: the units from static_units * gridDim.x on are claimed through ctr
};

template <int D, int NRT, int PASS, bool STRIDED>
__global__ __launch_bounds__(THREADS, MFMA_BLOCKS) void stream_kernel(ScoreGeom g, QueryPos qp, int half,
                                                                      StreamPlan plan, KvLayout lay,
                                                                      const uint16_t* __restrict__ q,
                                                            const uint16_t* __restrict__ k,
                                                            float2* __restrict__ part,
                                                            const float* __restrict__ rowc,
                                                            float* __restrict__ scores, int* __restrict__ ctr) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool one_group = (g.Rpad / 32 <= NRT);
  const int units_per_head = plan.units_per_head, n_units = plan.n_units;
  volatile int* ctl = reinterpret_cast<volatile int*>(smem + Smem<D, NRT>::OFF_CTL);
  const int dyn0 = min(plan.static_units * (int)gridDim.x, n_units);    // first dynamically assigned unit
  int run_u = blockIdx.x * plan.static_units;
  int run_end = min(run_u + plan.static_units, dyn0);
  if (run_u >= run_end) return;           // (host: never with a dynamic part, every workgroup has a first run)

  // key rows of chunk c_ of head hg_ (STRIDED: `lay` gives the element strides between instances and
  // heads and the byte distance between rows, or the block table of a paged cache, whose blocks hold
  // whole chunks; otherwise the cache is dense and `lay` is not read)
  auto rows_of = [&](int hg_, int c_) {
    if constexpr (STRIDED) {
      const int inst = hg_ / g.Hkv, head = hg_ - inst * g.Hkv;
      if (lay.table) {
        int r0;
        int64_t off = paged_block_offset(lay, inst, c_ * MFMA_ROWS, &r0);
        // (the same in every lane: the descriptor stays in scalar registers)
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)off);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)off >> 32));
        off = (int64_t)(((unsigned long long)hi << 32) | lo);
        return key_rows_strided<D>(k + off + (size_t)head * lay.head, r0, r0 + min(MFMA_ROWS, g.L - c_ * MFMA_ROWS), tid,
                                   lay.row_bytes);
      }
      return key_rows_strided<D>(k + (size_t)inst * lay.inst + (size_t)head * lay.head, c_ * MFMA_ROWS, g.L, tid,
                                 lay.row_bytes);
    } else {
      return key_rows<D>(k + (size_t)hg_ * g.L * D, c_ * MFMA_ROWS, g.L, tid);
    }
  };
  u32x4 pre[Tile<D>::PIECES_PER_THREAD];
  bf16x8 qreg[Tile<D>::KSTEPS];
  float cr[16];
  if (PASS == 2 && tid < 2 * MAX_HALF) {  // zero margins of the raw-score copy that pooling reads
    float* margin = reinterpret_cast<float*>(smem + Smem<D, NRT>::OFF_STAT);
    margin[tid < MAX_HALF ? tid : MFMA_ROWS + tid] = 0.f;
  }
  {
    const int hg = run_u / units_per_head, c = run_u - hg * units_per_head;
    fetch_chunk<D>(pre, rows_of(hg, c));
    commit_chunk<D>(smem, pre, tid);
  }
  __syncthreads();

  int hg_loaded = -1;
  // (head, chunk) of the current unit, kept incrementally: a division only where a run starts
  int hg = run_u / units_per_head, c = run_u - hg * units_per_head;
  for (;;) {
    int claimed = 0;                      // thread 0: the run claimed while this one is worked on
    for (int u = run_u; u < run_end; ++u) {
      const bool first = (u == run_u), single = (run_end - run_u == 1);
      if (plan.dynamic && first) {
        if (tid == 0) claimed = atomicAdd(ctr, 1);
        if (single) {                     // a one-unit run (tail only): its successor is needed at once
          __syncthreads();
          if (tid == 0) ctl[0] = claimed;
          __syncthreads();
        }
      }
      const int j0 = c * MFMA_ROWS;                // first staged key
      // the G query heads of KV head hg are consecutive: rows hg*R .. hg*R+R-1 of Q (R = G*W)
      const uint16_t* qg = q + (size_t)hg * g.R * D;
      const bool reload = !one_group || hg != hg_loaded;
      hg_loaded = hg;
      if (one_group && reload) {
        // operands of the new head first, so that they are not queued behind the key rows
        const int rt = wave % NRT;
        load_q_tile<D>(qreg, qg, rt, g.R, lane);
        if (PASS == 2) {
          const bool has_tile = rt * 32 < g.Rpad;     // (a slot beyond the head's row tiles reads nothing)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            cr[i] = has_tile ? rowc[(size_t)hg * g.Rpad + rt * 32 + acc_row(i, lane >> 5)] : 1.0e30f;
        }
      }
      // the unit after this one: the next of the run, else the first of the claimed run, else (nothing
      // left) this unit again, which is harmless and keeps the loads in flight the same everywhere
      int hn = hg, cn = c;
      if (u + 1 < run_end) {
        if (++cn == units_per_head) {
          cn = 0;
          ++hn;
        }
      } else if (plan.dynamic) {
        // (read from LDS, hence a per-lane value to the compiler: made wave-uniform by hand, or
        // every load through a descriptor derived from it is wrapped in a uniformity loop)
        const int s = dyn0 + __builtin_amdgcn_readfirstlane(ctl[0]) * RUN_UNITS;
        if (s < n_units) {
          hn = s / units_per_head;
          cn = s - hn * units_per_head;
        }
      }
      const auto nkr = rows_of(hn, cn);
      bool owned = false, edge_out = false, pool_out = false;
      int j_out = 0, e_out = 0;
      float v_out = 0.f, r_out = 0.f;
      float2 mz_out = make_float2(0.f, 0.f);
      float2* part_unit = part + ((size_t)hg * units_per_head + c) * g.Rpad;
      if (PASS == 1)
        owned = chunk_pass1<D, NRT>(smem, g, qp, qg, qreg, !one_group, j0, tid, lane, wave, part_unit, j_out, mz_out,
                                    pre, nkr);
      else
        owned = chunk_pass2<D, NRT>(smem, g, qp, half, half > 0 && units_per_head > 1, qg,
                                    rowc + (size_t)hg * g.Rpad, qreg, cr, !one_group, j0, tid, lane, wave, j_out,
                                    v_out, pool_out, edge_out, e_out, r_out, pre, nkr);
      // (every wave's reads of this chunk's rows are behind a barrier by now)
      if (plan.dynamic && first && !single && tid == 0) ctl[0] = claimed;
      commit_chunk<D>(smem, pre, tid);
      if (PASS == 1 && owned) part_unit[j_out] = mz_out;
      if (PASS == 2 && owned && !pool_out) scores[(size_t)hg * g.L + j_out] = v_out;
      if (PASS == 2 && edge_out)
        reinterpret_cast<float*>(part)[((size_t)hg * units_per_head + c) * (4 * half) + e_out] = r_out;
      __syncthreads();
      // (pooling comes after the barrier that completes the raw-score copy; the copy is next
      // written behind the next unit's first barrier, which every wave passes after these reads)
      if (PASS == 2 && pool_out) scores[(size_t)hg * g.L + j_out] = pooled_score<D, NRT>(smem, half, tid, v_out);
      hg = hn;                            // what was prefetched is what comes next
      c = cn;
    }
    if (!plan.dynamic) break;
    const int s = dyn0 + __builtin_amdgcn_readfirstlane(ctl[0]) * RUN_UNITS;
    if (s >= n_units) break;
    run_u = s;                            // (hg, c) already point at unit s
    run_end = min(s + RUN_UNITS, n_units);
  }
}

// Sets the work counters of the two streaming passes to zero (launched only when a pass claims units
// through them).
__global__ void reset_counters_kernel(int* ctr) {
  if (threadIdx.x < 2) ctr[threadIdx.x] = 0;
}

// Combine the (m, z) of all chunks of a head into c = M + log2 Z per score row.  One workgroup per
// (head, 32-row tile): 8 threads share a row and split the chunks; fixed merge order.  Also clears the
// workspace's status word (these kernels have no wait to give up).
__global__ __launch_bounds__(256) void row_constants_mfma_kernel(ScoreGeom g, const float2* __restrict__ part,
                                                                  float* __restrict__ rowc, int* __restrict__ status) {
  __shared__ float2 stat[256];
  const int hg = blockIdx.x, rt = blockIdx.y, tid = threadIdx.x;
  if (hg == 0 && rt == 0 && tid == 0) *status = 0;
  const int r = rt * 32 + (tid & 31), sel = tid >> 5;
  const float2* p = part + (size_t)hg * g.nchunk * g.Rpad + r;
  float M = NEG_BIG, Z = 0.f;
  constexpr int B = 16;
  for (int c0 = sel; c0 < g.nchunk; c0 += 8 * B) {
    float2 buf[B];
#pragma unroll
    for (int b = 0; b < B; ++b) buf[b] = p[(size_t)min(c0 + 8 * b, g.nchunk - 1) * g.Rpad];
#pragma unroll
    for (int b = 0; b < B; ++b)
      if (c0 + 8 * b < g.nchunk) merge_stat(M, Z, buf[b]);
  }
  stat[tid] = make_float2(M, Z);
  __syncthreads();
  if (tid < 32) {
    for (int s2 = 1; s2 < 8; ++s2) merge_stat(M, Z, stat[s2 * 32 + tid]);
    rowc[(size_t)hg * g.Rpad + r] = (r < g.R) ? M + __builtin_amdgcn_logf(Z) : 1.0e30f;
  }
}

// Pooled scores of the prefix keys whose pooling window crosses a boundary between two chunks of
// the scoring kernels, from the edge records (per chunk: raw scores of its first 2*half rows, then of its last
// 2*half rows).  The boundary before chunk c lies at key b = c * chunk_rows and the keys
// b-half .. b+half-1 are pooled here, one per thread; blockIdx.x is the head.
__global__ __launch_bounds__(256) void pool_boundaries_kernel(int L, int P, int half, int nchunk, int chunk_rows,
                                                               const float* __restrict__ edge,
                                                               float* __restrict__ scores) {
  const int hg = blockIdx.x;
  const int rec = 4 * half, per = 2 * half;
  const int it = blockIdx.y * 256 + threadIdx.x;
  if (it >= (nchunk - 1) * per) return;
  const int c = it / per + 1;
  const int b = c * chunk_rows;
  const int j = b - half + it % per;
  if (j >= P) return;
  // raw score of key i, b - 2*half <= i < b + 2*half, is e[i]: the tail of chunk c-1's record is
  // followed in memory by the head of chunk c's
  const float* e = edge + ((size_t)hg * nchunk + c - 1) * rec + per - (b - per);
  const int hi = min(j + half, P - 1);
  float v = 0.f;
  for (int i = j - half; i <= hi; ++i) v = fmaxf(v, e[i]);
  scores[(size_t)hg * L + j] = v;
}

// ---- per-device set-up ---------------------------------------------------------------------
// The streaming kernels need more dynamic LDS than the default limit (an attribute per kernel) and
// their grid is the number of workgroups the device holds at once (an occupancy query).  Both are
// looked up for every instantiation at once, per device, by score_mfma_init(): explicitly through
// laq_init(), else on the first scoring call on that device (host threads that race there compute
// the same values).  After it a scoring call makes no HIP call other than kernel launches.
constexpr int MAX_DEVICES = 64;
constexpr int N_VARIANTS = 12;             // 2 head sizes x 3 row-tile counts x dense / strided
template <int D, int NRT, bool STRIDED> constexpr int variant_id() {
  return ((D == 128 ? 0 : 1) * 3 + (NRT == 1 ? 0 : NRT == 2 ? 1 : 2)) * 2 + (STRIDED ? 1 : 0);
}
std::atomic<int> resident_of[MAX_DEVICES][N_VARIANTS];
std::atomic<int> device_ready[MAX_DEVICES];

template <int D, int NRT, bool STRIDED>
hipError_t init_variant(int dev, int cus) {
  constexpr int bytes = Smem<D, NRT>::BYTES;
  const void* f1 = reinterpret_cast<const void*>(&stream_kernel<D, NRT, 1, STRIDED>);
  const void* f2 = reinterpret_cast<const void*>(&stream_kernel<D, NRT, 2, STRIDED>);
  hipError_t e;
  if ((e = hipFuncSetAttribute(f1, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(f2, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  int n1 = 0, n2 = 0;
  if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n1, f1, THREADS, bytes)) != hipSuccess) return e;
  if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n2, f2, THREADS, bytes)) != hipSuccess) return e;
  if (n1 < 1 || n2 < 1) return hipErrorInvalidValue;
  resident_of[dev][variant_id<D, NRT, STRIDED>()].store(cus * (n1 < n2 ? n1 : n2), std::memory_order_release);
  return hipSuccess;
}

template <int D, int NRT, bool STRIDED>
hipError_t launch_stream(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const uint16_t* q,
                         const uint16_t* k, float* scores, const Workspace& ws, hipStream_t st) {
  constexpr int bytes = Smem<D, NRT>::BYTES;
  int dev = 0;
  hipError_t e;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = score_mfma_init(dev)) != hipSuccess) return e;
  const int resident = resident_of[dev][variant_id<D, NRT, STRIDED>()].load(std::memory_order_acquire);
  if (resident < 1) return hipErrorInvalidValue;
  const long long n_heads = (long long)g.n_inst * g.Hkv;
  const int half = (pool - 1) / 2;
  const int units1 = (g.L + MFMA_ROWS - 1) / MFMA_ROWS;
  const int units2 = units1;
  ScoreGeom gm = g;
  gm.nchunk = units1;                      // this path's chunking of the statistics
  const long long nu1 = n_heads * units1, nu2 = n_heads * units2;
  if (nu1 > 0x7fff0000LL || nu2 > 0x7fff0000LL) return hipErrorInvalidValue;
  // Few units per resident workgroup: one fixed run each, as few workgroups as keep every slot busy.
  // Many: 5/8 of the even share as the fixed first run, the rest claimed in short runs.
  auto make_plan = [&](long long nu, int units_per_head, int* grid) {
    StreamPlan p;
    p.units_per_head = units_per_head;
    p.n_units = (int)nu;
    const int share = (int)((nu + resident - 1) / resident);
    if (share < 4 * RUN_UNITS) {
      p.static_units = share;
      p.dynamic = 0;
      *grid = (int)((nu + share - 1) / share);
    } else {
      p.static_units = (int)(nu / resident) * 5 / 8;
      p.dynamic = 1;
      *grid = resident;
    }
    return p;
  };
  int grid1 = 0, grid2 = 0;
  const StreamPlan p1 = make_plan(nu1, units1, &grid1), p2 = make_plan(nu2, units2, &grid2);
  if (p1.dynamic || p2.dynamic) {
    hipLaunchKernelGGL(reset_counters_kernel, dim3(1), dim3(64), 0, st, ws.ctr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  hipLaunchKernelGGL((stream_kernel<D, NRT, 1, STRIDED>), dim3(grid1), dim3(THREADS), bytes, st, g, qp, 0, p1, lay, q, k,
                     ws.part,
                     (const float*)nullptr, (float*)nullptr, ws.ctr);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(row_constants_mfma_kernel, dim3((unsigned)n_heads, g.Rpad / 32), dim3(256), 0, st, gm, ws.part,
                     ws.rowc, ws.status);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // (the edge records, at most 124 floats per 256-key chunk and only written when a head has more
  // than one chunk, fit the workspace's raw-score area of L floats per head)
  hipLaunchKernelGGL((stream_kernel<D, NRT, 2, STRIDED>), dim3(grid2), dim3(THREADS), bytes, st, g, qp, half, p2, lay, q, k,
                     reinterpret_cast<float2*>(ws.raw), ws.rowc, scores, ws.ctr + 1);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (half > 0 && units2 > 1) return launch_pool_boundaries(g, half, units2, MFMA_ROWS, ws.raw, scores, st);
  return hipSuccess;
}

template <int D, bool STRIDED>
hipError_t launch_for_rows(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const uint16_t* q,
                           const uint16_t* k, float* scores, const Workspace& ws, hipStream_t st) {
  const int ntile = g.Rpad / 32;
  if (ntile == 1) return launch_stream<D, 1, STRIDED>(g, qp, lay, pool, q, k, scores, ws, st);
  if (ntile == 2) return launch_stream<D, 2, STRIDED>(g, qp, lay, pool, q, k, scores, ws, st);
  return launch_stream<D, 4, STRIDED>(g, qp, lay, pool, q, k, scores, ws, st);
}

}  // namespace

hipError_t launch_pool_boundaries(const ScoreGeom& g, int half, int nchunk, int chunk_rows, const float* edge,
                                  float* scores, hipStream_t st) {
  const long long n_heads = (long long)g.n_inst * g.Hkv;
  const int items = (nchunk - 1) * 2 * half;
  if (items <= 0) return hipSuccess;
  hipLaunchKernelGGL(pool_boundaries_kernel, dim3((unsigned)n_heads, (items + 255) / 256), dim3(256), 0, st, g.L, g.P,
                     half, nchunk, chunk_rows, edge, scores);
  return hipGetLastError();
}

hipError_t score_mfma_init(int dev) {
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (device_ready[dev].load(std::memory_order_acquire)) return hipSuccess;
  int cus = 0;
  hipError_t e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  if (cus < 1) return hipErrorInvalidValue;
#define LAQ_INIT_VARIANT(D, NRT) \
  if ((e = init_variant<D, NRT, false>(dev, cus)) != hipSuccess) return e; \
  if ((e = init_variant<D, NRT, true>(dev, cus)) != hipSuccess) return e;
  LAQ_INIT_VARIANT(128, 1) LAQ_INIT_VARIANT(128, 2) LAQ_INIT_VARIANT(128, 4)
  LAQ_INIT_VARIANT(64, 1) LAQ_INIT_VARIANT(64, 2) LAQ_INIT_VARIANT(64, 4)
#undef LAQ_INIT_VARIANT
  device_ready[dev].store(1, std::memory_order_release);
  return hipSuccess;
}

bool score_mfma_supported(const ScoreGeom& g, const KvLayout& lay, int dtype) {
  // the key loads address a head with 31-bit byte offsets (one chunk of slack past its end)
  return dtype == LAQ_BF16 && (g.d == 128 || g.d == 64) && g.W <= MAX_QPOS &&
         g.n_inst * (long long)g.Hkv <= 0x7fffffff &&
         ((long long)(lay.table ? lay.block_rows : g.L) + MFMA_ROWS) * lay.row_bytes < 0x7fffffffLL;
}

hipError_t launch_score_mfma(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const void* q,
                             const void* k, float* scores, const Workspace& ws, hipStream_t st) {
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  const uint16_t* kk = static_cast<const uint16_t*>(k);
  if (lay.dense) {
    if (g.d == 128) return launch_for_rows<128, false>(g, qp, lay, pool, qq, kk, scores, ws, st);
    return launch_for_rows<64, false>(g, qp, lay, pool, qq, kk, scores, ws, st);
  }
  if (g.d == 128) return launch_for_rows<128, true>(g, qp, lay, pool, qq, kk, scores, ws, st);
  return launch_for_rows<64, true>(g, qp, lay, pool, qq, kk, scores, ws, st);
}

}  // namespace laq
