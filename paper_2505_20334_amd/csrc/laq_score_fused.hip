// bf16 scoring on the matrix cores with K read ONCE and ONE exponential per (score row, key): the
// unnormalised probabilities of a head stay in registers until the softmax denominators are known.
//
// The softmax of Eq. 4's observation window needs every score row's denominator before a single
// probability can be summed over the rows (Sec. 4.3).  A kernel that streams K twice computes every
// exponential twice.  Here every wave computes the dot products of its keys once, keeps them -- 128
// accumulator registers: eight 32 x 32 tiles (32 keys x 32 rows) -- takes the row maxima m over
// the workgroup's keys, turns the dot products in place into e = exp2(s - m), and keeps these
// until the team of workgroups that shares the head has folded the rows' (m, Z = sum_keys e) into
// c = M + log2 Z.  The key's score is then sum_rows e * exp2(m - c): one multiply-add per stored
// number.  Key rows pass through registers once and are never needed again, so their loads do
// not depend on the exchange.  For KV heads with at most 128 score rows (32, 64 or 128: one
// instantiation each).
//
// A workgroup has four waves (one per SIMD; two workgroups share a compute unit, so that one of
// them computes while the other waits for its team); a wave holds 8 / (R / 32) key tiles, a
// workgroup four times that many keys, a team of ceil(L / keys per workgroup) workgroups one head.
// Per head, every workgroup of the team
//   B. D = Q * K_tile^T per (key tile, row tile): lane = key, accumulator registers = 16 rows; the
//      next key tiles are loaded while this one is worked on; the first two of the next head are
//      requested during the pass, one into registers, one into LDS (loads that write LDS directly),
//      and travel while the other steps run;
//   C. row maxima over its keys (registers, a transposition through LDS per wave, LDS across
//      waves), e = exp2(D * scale2 - m) in place, row sums the same way; publishes (m, Z) per row;
//   D. pools and stores the previous head's scores, stages the next head's Q;
//   E. reads the statistics of the whole team and folds them, in a fixed order, into c per row
//      (every member computes the same constants; nobody waits for a combiner), and from them one
//      weight per row, exp2(m - c);
//   F. score of a key = sum over rows of e * weight; the workgroup's raw scores meet in LDS,
//      where the sequence max-pool of every key whose window lies inside the workgroup's keys is
//      taken; the few keys next to a workgroup boundary are pooled by pool_boundaries_kernel from
//      raw scores left for it.
//
// The exchange in steps C and E uses no cache maintenance (agent-scope release/acquire fences write
// back and invalidate L2 on this part, tens of microseconds each), no read-modify-write and no
// separate flag: a statistic is one 8-byte word (m, Z) written with one device-coherent store
// (cache policy sc1) and read with device-coherent loads, and it validates itself -- Z is never
// negative, so its sign bit carries one bit of the head's number, which differs between two
// consecutive uses of the same word.  A reader loads the words it needs and re-loads those that
// are not there yet; one store-to-load hop in all.  The team alternates between two sets of
// words, so a word is only overwritten after every member has read it (a member that publishes
// head n+2 has been through the exchange of head n+1, for which every member had published,
// which it does after reading head n).  All waits are bounded, and end at once after one of
// them has timed out (status word of the workspace).  The kernel is started with a cooperative
// launch, which guarantees that the workgroups of a team are on the device together.
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "laq_internal.h"

namespace laq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr float NEG_BIG = -1.0e30f;
constexpr int D = 128;                       // head size this kernel is written for
constexpr int KS = D / 16;                   // MFMAs (reduction steps) per 32x32 tile
constexpr int TILE_BYTES = 32 * D * 2;       // a key tile: 32 rows
constexpr int F_WAVES = 4, F_THREADS = F_WAVES * 64;   // one wave per SIMD; two workgroups share a compute unit
// LDS row of Q: the d elements and 16 bytes that make 128-bit operand reads of 16 consecutive
// rows conflict-free
constexpr int QROWB = D * 2 + 16;
constexpr int ZT_STRIDE = 36;                // floats per row of a wave's transposition tile (conflict-free 128-bit reads)
constexpr int SPIN_LIMIT = 1 << 20;          // probes; about a second, far beyond any legitimate wait
constexpr int MAX_HALF = (MAX_POOL - 1) / 2;
constexpr int COHERENT = 16;                 // cache policy bit "sc1": coherent across the device

#define LAQ_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Issue priority of this wave against the waves of the other workgroup on the compute unit.  The
// steps between two heads are a chain of short, latency-bound pieces (reductions, the publication
// of the statistics, the reads of the team's) around two long pieces of bulk work (the matrix
// products with their loads, the sweep of exponentials).  Without priorities the older wave of a
// SIMD wins every arbitration, whatever it is doing; with them a wave in a short piece goes first
// and a wave in the sweep of exponentials yields (config 5: 4.15 -> 3.75 ms for the stage).
constexpr int PRIO_BULK = 0, PRIO_MATRIX = 1, PRIO_CHAIN = 3;

// Workgroup barrier for data that travels through LDS only: waits for this wave's LDS operations,
// not for its outstanding global loads (key rows are in flight most of the time, and the barrier of
// __syncthreads() would wait for all of them).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int FROM, int TO, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FROM < TO) {
    f(std::integral_constant<int, FROM>{});
    static_for<FROM + 1, TO>(f);
  }
}

// Sizes that follow from the number of 32-row tiles of a head's score rows.
template <int NRT> struct Cfg {
  static constexpr int ROWS = NRT * 32;
  static constexpr int PAIRS = 8;                                   // (key tile, row tile) pairs a wave keeps: 16 registers each
  static constexpr int KT = PAIRS / NRT;                            // key tiles per wave and head
  static constexpr bool ROTATE = NRT == 2;                          // see WaveCtx::rot (the other instantiations lose registers to it)
  static constexpr int KEYS_PER_WAVE = KT * 32, KEYS_PER_BLOCK = F_WAVES * KEYS_PER_WAVE;
  static constexpr int Q_BYTES = ROWS * QROWB;
  static constexpr int Q_PIECES = ROWS * (D / 8);                   // 16-byte pieces of one Q_g
  static constexpr int Q_PER_THREAD = (Q_PIECES + F_THREADS - 1) / F_THREADS;
  static constexpr int OFF_Q = 0;                                   // [ROWS][QROWB] bf16 rows of Q_g
  // float[F_WAVES][32][ZT_STRIDE]: transposition tiles.  They are used between the last read of a
  // head's Q and the arrival of the next head's, so where Q is large enough (128 score rows) they
  // lie inside it; a barrier then separates them from the last matrix product.
  static constexpr int ZT_BYTES = F_WAVES * 32 * ZT_STRIDE * 4;
  static constexpr bool ZT_IN_Q = Q_BYTES >= ZT_BYTES;
  static constexpr int OFF_ZT = ZT_IN_Q ? OFF_Q : OFF_Q + Q_BYTES;
  static constexpr int OFF_STAT = OFF_Q + Q_BYTES + (ZT_IN_Q ? 0 : ZT_BYTES);   // float[F_WAVES][ROWS]: the waves' maxima / sums
  static constexpr int OFF_REF = OFF_STAT + F_WAVES * ROWS * 4;     // float[ROWS]: the rows' maxima over the workgroup (log2 units)
  static constexpr int OFF_WTS = OFF_REF + ROWS * 4;                // float[ROWS]: the rows' weights exp2(m - c)
  static constexpr int RPAIRS = ROWS / 2, NSUB = F_THREADS / RPAIRS;   // the fold: threads per pair of rows
  static constexpr int OFF_FOLD = OFF_WTS + ROWS * 4;               // float2[NSUB][ROWS]: the team's statistics, per member subset
  static constexpr int OFF_LAST = OFF_FOLD + NSUB * ROWS * 8;       // int[ROWS]: last key every score row sees
  static constexpr int OFF_RAW = OFF_LAST + ROWS * 4;               // float[MAX_HALF + KEYS_PER_BLOCK + MAX_HALF]: the
                                                                    // workgroup's raw scores between zero margins
  static constexpr int OFF_FLAG = OFF_RAW + (KEYS_PER_BLOCK + 2 * MAX_HALF) * 4;   // int: "a wait has timed out"
  static constexpr int OFF_STAGE = (OFF_FLAG + 16 + 15) & ~15;      // char[F_WAVES][TILE_BYTES]: one key tile per wave, in flight
                                                                    // from memory across the steps that have no registers for it
  static constexpr int BYTES = OFF_STAGE + F_WAVES * TILE_BYTES;
};

// ---- words that workgroups hand to each other ------------------------------------------------
__device__ __forceinline__ void coherent_store(float2* p, float2 v) {
  const unsigned long long bits = ((unsigned long long)__float_as_uint(v.y) << 32) | __float_as_uint(v.x);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void merge_stat(float& M, float& Z, float2 p) {
  const float Mn = fmaxf(M, p.x);
  Z = Z * __builtin_amdgcn_exp2f(M - Mn) + p.y * __builtin_amdgcn_exp2f(p.x - Mn);
  M = Mn;
}

// Row index (0..31) of accumulator register i for a lane in half hf of the 32x32 output layout.
__device__ __forceinline__ int acc_row(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

__device__ __forceinline__ bf16x8 lds_operand(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }

// ---- key rows: global memory -> operand registers -------------------------------------------
// Lane l of a wave supplies key row l%32 of a tile and the 16-byte slice 2t + l/32 of that row
// for reduction step t.  Buffer loads against a descriptor that ends with the head's last row (of a
// paged cache: the block's last valid row): rows beyond it read as zeros (they are causally
// masked).  Consecutive rows lie row_bytes apart (256 in a dense cache, more in a token-major or
// padded one).
// Where a key tile lies: its first row is row `row0` of the `rows` rows that start at `base`.
struct TileRef {
  const uint16_t* base;
  int rows;
  int row0;
};
struct KeySource {
  __amdgpu_buffer_rsrc_t rsrc;
  int row0;
};
__device__ __forceinline__ KeySource key_source(const TileRef& r, int row_bytes) {
  // (the address is the same in every lane; saying so keeps the descriptor in scalar registers)
  const unsigned long long a = reinterpret_cast<unsigned long long>(r.base);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  KeySource s;
  s.rsrc = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((unsigned long long)hi << 32) | lo), 0,
                                             __builtin_amdgcn_readfirstlane(r.rows > 0 ? (r.rows - 1) * row_bytes + D * 2 : 0),
                                             0x00020000);
  s.row0 = r.row0;
  return s;
}
__device__ __forceinline__ bf16x8 load_operand(const KeySource& s, int voff_tile, int t) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(s.rsrc, voff_tile + t * 32, 0, 0));
}
// Byte offset from the descriptor's first row of (row l%32 of the tile, slice l/32).  Recomputed
// where it is needed (a register held across the whole kernel costs more than three instructions
// per tile), and opaque to the optimiser so that the step offsets fold into the instructions'
// immediate fields.
__device__ __forceinline__ int tile_offset(int row0, int lane, int row_bytes) {
  int l = lane;
  asm volatile("" : "+v"(l));
  return (row0 + (l & 31)) * row_bytes + (l >> 5) * 16;
}

// The same tile, memory -> LDS without passing through registers: eight 16-byte loads per lane
// whose data the memory pipeline writes to LDS itself, lane l's piece of reduction step t at
// stage + t * 1024 + l * 16 (rows beyond the descriptor's end arrive as zeros, as in registers).
// The loads count as vector memory loads of the wave (wait with stage_wait()); the compiler does
// not see them: its own waits for loads issued earlier can only become longer by that, never
// shorter, because loads complete in the order of their issue.  M0, which carries the LDS address, is put back.
__device__ __forceinline__ void stage_tile(const TileRef& r, int row_bytes, int lane, unsigned stage) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(r.base);
  u32x4 words;
  words[0] = __builtin_amdgcn_readfirstlane((unsigned)a);
  words[1] = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32)) & 0xffffu;
  words[2] = __builtin_amdgcn_readfirstlane(r.rows > 0 ? (r.rows - 1) * row_bytes + D * 2 : 0);
  words[3] = 0x00020000u;
  const int voff = tile_offset(r.row0, lane, row_bytes);
  const unsigned lds = __builtin_amdgcn_readfirstlane(stage);
#pragma unroll
  for (int t = 0; t < KS; ++t) {
    unsigned keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, %4 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep)
                 : "s"(lds + t * 1024), "v"(voff), "s"(words), "s"(t * 32)
                 : "memory");
  }
}
__device__ __forceinline__ void stage_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const char*)p;
}

struct WaveCtx {
  const char* q_lane;      // LDS: Q row (lane%32), slice (lane/32) of reduction step 0, row tile 0
  int lane, hf, n32;
  int key0;                // first key of this wave within the head
  int rot;                 // the wave's tile kt holds keys (kt + rot) % KT * 32 .. + 31 of its range
  int L;
  int row_bytes;           // distance between consecutive key rows
  int qmin;                // keys up to here are seen by every row: tiles below need no mask
  const int* last;         // LDS: last key every score row sees, for the causal mask
  const char* stage;       // LDS: this wave's staged key tile
};

// ---- step B: the wave's (key tile, row tile) pairs --------------------------------------------
// E[pair] = Q_rt * K_tile^T over the head size: lane = key, accumulator registers = 16 rows; -inf
// where a row does not see a key.  Key tile kt is in kring[kt % 4].  Tile 0 is there when the pass
// begins (loaded into registers during the previous head's pass) and tile 1 waits in the wave's LDS
// stage (requested at the end of the previous head's pass: it travels while the other steps run,
// which have no registers to receive it); the loads of the next two tiles are issued at once at
// the start -- the registers that will hold the later pairs' results are still free then -- and
// every slot is reloaded as soon as its tile has been through its last pair: with the tile four
// further on, or (slot 0, when `more`) with tile 0 of the next head.  Tile 1 of the next head is
// requested at the end.
constexpr int RING = 4;
// cur(kt) / next(kt): where key tile kt of this head / of the next head lies.
template <int NRT, typename CUR, typename NEXT, typename STAGE>
__device__ __forceinline__ void wave_main(const WaveCtx& w, f32x16 (&E)[Cfg<NRT>::PAIRS], bf16x8 (&kring)[RING][KS],
                                          CUR cur, NEXT next, STAGE stage_next, bool more) {
  constexpr int NP = Cfg<NRT>::PAIRS, KT = Cfg<NRT>::KT;
  constexpr int AHEAD = 2;                 // Q operands requested from LDS this many MFMAs ahead
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto q_addr = [&](int n) {               // operand of MFMA n = pair * KS + step
    const int rt = (n / KS) % NRT, t = n % KS;
    return w.q_lane + rt * 32 * QROWB + t * 32;
  };
  bf16x8 ring[AHEAD];
#pragma unroll
  for (int n = 0; n < AHEAD; ++n) ring[n] = lds_operand(q_addr(n));
  {
    static_assert(KT >= 2, "the staged tile is tile 1");
    stage_wait();
    int l = w.lane;
    asm volatile("" : "+v"(l));
#pragma unroll
    for (int t = 0; t < KS; ++t) kring[1][t] = lds_operand(w.stage + t * 1024 + l * 16);
  }
#pragma unroll
  for (int kt = 2; kt < RING && kt < KT; ++kt) {
    const KeySource src = cur(kt);
    const int v = tile_offset(src.row0, w.lane, w.row_bytes);
#pragma unroll
    for (int t = 0; t < KS; ++t) kring[kt][t] = load_operand(src, v, t);
  }

  static_for<0, NP>([&](auto I) {
    constexpr int i = decltype(I)::value;
    constexpr int kt = i / NRT, rt = i % NRT;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      const int n = i * KS + t;
      if (t == 0) {
        // The chain starts from zero; in tiles with a key that some row does not see (wave-uniform
        // test) from -inf where a key is not visible to a row.  The two cases are separate
        // instructions so that the common one needs no copy of its start value; the bound goes
        // through an opaque copy so that the start vectors of all pairs are not computed ahead and
        // kept alive.
        const int t0 = w.key0 + (Cfg<NRT>::ROTATE ? (kt + w.rot) % KT : kt) * 32;
        int qmin_here = __builtin_amdgcn_readfirstlane(w.qmin);
        asm volatile("" : "+s"(qmin_here));
        if (t0 + 31 > qmin_here) {
          int hf_here = w.hf, n32_here = w.n32;
          asm volatile("" : "+v"(hf_here), "+v"(n32_here));
          const int key = t0 + n32_here;                               // this lane's key
          f32x16 start = zero;
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {                             // rows 8*gq + 4*hf .. +3 of the tile
            const i32x4 lv = *reinterpret_cast<const i32x4*>(w.last + rt * 32 + 8 * gq + 4 * hf_here);
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (key > lv[j]) start[4 * gq + j] = -INFINITY;
          }
          E[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % AHEAD], kring[kt % RING][0], start, 0, 0, 0);
        } else {
          E[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % AHEAD], kring[kt % RING][0], zero, 0, 0, 0);
        }
      } else {
        E[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % AHEAD], kring[kt % RING][t], E[i], 0, 0, 0);
      }
      if (n + AHEAD < NP * KS) ring[n % AHEAD] = lds_operand(q_addr(n + AHEAD));
      LAQ_SCHED_FENCE();
    }
    if constexpr (rt == NRT - 1) {
      // the tile has been through its last pair: its slot takes the tile four further on, or the
      // first tile of the next head (slot 0, once no tile of this head needs it any more)
      constexpr int after = kt + RING;
      if constexpr (after < KT) {
        const KeySource src = cur(after);
        const int v = tile_offset(src.row0, w.lane, w.row_bytes);
#pragma unroll
        for (int t = 0; t < KS; ++t) kring[kt % RING][t] = load_operand(src, v, t);
      } else if constexpr (kt % RING == 0) {
        if (more) {
          const KeySource src = next(0);
          const int v = tile_offset(src.row0, w.lane, w.row_bytes);
#pragma unroll
          for (int t = 0; t < KS; ++t) kring[0][t] = load_operand(src, v, t);
        }
      }
    }
  });
  if (more) stage_next();
}

// ---- exchange buffers --------------------------------------------------------------------------
// Per team, two sets of statistics words [team size][rows]: (m, Z) with the validity bit in the
// sign of Z (see the head of the file).
struct FusedSync {
  float2* stats;           // [n_teams][2][T][rows]
  int* status;             // != 0: a wait has timed out (results are not valid)
};
struct FusedPlan {
  int T;                   // workgroups per team = ceil(L / keys per workgroup)
  int n_teams;
  int n_heads;             // team t takes heads t, t + n_teams, ...
  int half;                // (pool kernel - 1) / 2; 0: raw scores
};

template <int NRT, bool PAGED>
__global__ __launch_bounds__(F_THREADS, 2) void fused_kernel(ScoreGeom g, QueryPos qp, FusedPlan plan, KvLayout lay,
                                                             const uint16_t* __restrict__ q,
                                                             const uint16_t* __restrict__ k,
                                                             float* __restrict__ scores, float* __restrict__ edge,
                                                             FusedSync sy) {
  using S = Cfg<NRT>;
  constexpr int ROWS = S::ROWS, KT = S::KT, NP = S::PAIRS;
  constexpr int KEYS_PER_WAVE = S::KEYS_PER_WAVE, KEYS_PER_BLOCK = S::KEYS_PER_BLOCK;
  extern __shared__ __align__(16) char smem[];
  char* q_lds = smem + S::OFF_Q;
  float* stat_lds = reinterpret_cast<float*>(smem + S::OFF_STAT);
  float* ref_lds = reinterpret_cast<float*>(smem + S::OFF_REF);
  float* wts_lds = reinterpret_cast<float*>(smem + S::OFF_WTS);
  float2* fold_lds = reinterpret_cast<float2*>(smem + S::OFF_FOLD);
  int* last_lds = reinterpret_cast<int*>(smem + S::OFF_LAST);
  float* raw_lds = reinterpret_cast<float*>(smem + S::OFF_RAW) + MAX_HALF;       // key 0 of the workgroup
  volatile int* gave_up = reinterpret_cast<volatile int*>(smem + S::OFF_FLAG);

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = plan.T, half = plan.half;
  const int team = blockIdx.x / T, member = blockIdx.x - team * T;
  if (team >= plan.n_teams || team >= plan.n_heads) return;
  float* zt = reinterpret_cast<float*>(smem + S::OFF_ZT) + wave * 32 * ZT_STRIDE;

  WaveCtx w;
  w.lane = lane; w.hf = lane >> 5; w.n32 = lane & 31;
  w.q_lane = q_lds + w.n32 * QROWB + w.hf * 16;
  w.key0 = member * KEYS_PER_BLOCK + wave * KEYS_PER_WAVE;
  // (the members of a team start at different tiles of their ranges, so that the addresses the
  // device is asked for at the same time do not all lie the same distance into a 32 KiB piece: about
  // 2 % on the stage time of config 5, averaged over its modes)
  w.rot = S::ROTATE ? __builtin_amdgcn_readfirstlane(member % KT) : 0;
  w.L = g.L; w.qmin = g.qmin; w.row_bytes = lay.row_bytes;
  w.last = last_lds;
  w.stage = smem + S::OFF_STAGE + wave * TILE_BYTES;
  // rows beyond R (zero queries) see every key; their weight is zero
  for (int r = tid; r < ROWS; r += F_THREADS) last_lds[r] = r < g.R ? qp.last[r % g.W] : g.L - 1;
  if (tid < 2 * MAX_HALF) raw_lds[tid < MAX_HALF ? tid - MAX_HALF : KEYS_PER_BLOCK + tid - MAX_HALF] = 0.f;
  if (tid == 0) gave_up[0] = 0;

  f32x16 E[NP];
  bf16x8 kring[RING][KS];

  // (thread and lane numbers go through opaque copies in the steps outside the matrix loop: the
  // addresses derived from them are then computed where they are used, not ahead of the loop over
  // the heads and kept in -- or spilled from -- registers across it)
  auto opaque = [](int v) {
    asm volatile("" : "+v"(v));
    return v;
  };
  // Q_g of head `hq` (rows hq*R .. +R-1 of Q; rows beyond R are zero): global memory -> registers -> LDS
  auto fetch_q = [&](int hq, u32x4 (&qv)[S::Q_PER_THREAD]) {
    const int tid = opaque(threadIdx.x);
    const uint16_t* qg = q + (size_t)hq * g.R * D;
#pragma unroll
    for (int i = 0; i < S::Q_PER_THREAD; ++i) {
      const int p = tid + i * F_THREADS, row = p / (D / 8), col = p % (D / 8);
      qv[i] = u32x4{0u, 0u, 0u, 0u};
      if (p < S::Q_PIECES && row < g.R) qv[i] = *reinterpret_cast<const u32x4*>(qg + (size_t)row * D + col * 8);
    }
  };
  auto commit_q = [&](const u32x4 (&qv)[S::Q_PER_THREAD]) {
    const int tid = opaque(threadIdx.x);
#pragma unroll
    for (int i = 0; i < S::Q_PER_THREAD; ++i) {
      const int p = tid + i * F_THREADS, row = p / (D / 8), col = p % (D / 8);
      if (p < S::Q_PIECES) *reinterpret_cast<u32x4*>(q_lds + row * QROWB + col * 16) = qv[i];
    }
  };
  // The memory that holds this wave's keys of head hg_ (instance hg_ / Hkv, KV head hg_ % Hkv): the
  // head's first row, or in a paged cache the first row of the block with the wave's keys -- blocks
  // hold a multiple of 256 rows and a wave's keys are 128 or 256 aligned ones, so they share a block.
  // One look-up per head, made a step ahead of its first use.  (The table is not written while the
  // kernel runs: read as constant memory, an entry comes through the scalar cache; a vector load
  // would return behind every key load issued before it.)
  auto wave_base = [&](int hg_) -> const uint16_t* {
    const int inst = hg_ / g.Hkv, head = hg_ - inst * g.Hkv;
    if constexpr (PAGED) {
      if (w.key0 >= g.L) return k;
      typedef __attribute__((address_space(4))) const int32_t* ConstTable;
      const int32_t blk = ((ConstTable)(unsigned long long)lay.table)[(size_t)inst * lay.blocks_per_inst + w.key0 / lay.block_rows];
      return k + (int64_t)blk * lay.block + (size_t)head * lay.head;
    }
    return k + (size_t)inst * lay.inst + (size_t)head * lay.head;
  };
  // key tile kt of this wave; a tile beyond the head's end of a paged cache gets an empty range,
  // every row of it reads as zeros
  auto tile_at = [&](const uint16_t* base, int kt) {
    const int j0 = w.key0 + (S::ROTATE ? (kt + w.rot) % KT : kt) * 32;
    if constexpr (PAGED) {
      if (j0 >= g.L) return TileRef{k, 0, 0};
      const int first = w.key0 / lay.block_rows * lay.block_rows;      // the block's first key
      return TileRef{base, min(lay.block_rows, g.L - first), j0 - first};
    }
    return TileRef{base, g.L, j0};
  };
  // Scores of head hg_ from the raw scores that step F left in LDS (zero beyond the head's last key
  // and in the margins).  Keys behind the prefix and, without pooling, all keys are stored as they
  // are.  A prefix key whose pooling window lies inside the workgroup's keys gets the maximum over
  // the part of the window inside the prefix; the raw scores of the first and last 2*half keys go
  // to the edge record of this workgroup, from which pool_boundaries_kernel pools the keys next to
  // a boundary.
  auto pool_head = [&](int hg_) {
    const int tid = opaque(threadIdx.x);
    const int base = member * KEYS_PER_BLOCK;
    float* scores_head = scores + (size_t)hg_ * g.L;
    float* rec = edge + ((size_t)hg_ * T + member) * (4 * half);
#pragma unroll
    for (int rep = 0; rep < KEYS_PER_BLOCK / F_THREADS; ++rep) {
      const int i = tid + rep * F_THREADS, j = base + i;
      const float v = raw_lds[i];
      if (j >= g.L) continue;
      if (half == 0 || j >= g.P) {
        scores_head[j] = v;
        continue;
      }
      if (T > 1) {
        if (i < 2 * half) rec[i] = v;
        else if (i >= KEYS_PER_BLOCK - 2 * half) rec[i - (KEYS_PER_BLOCK - 4 * half)] = v;
      }
      if ((member > 0 && i < half) || min(j + half, g.P - 1) >= base + KEYS_PER_BLOCK) continue;
      const int room = g.P - 1 - j;          // window positions above the key that are still prefix
      float pv = v;
      if (half == 3) {
        float r[7];                          // the usual kernel of 7: all reads issued at once
#pragma unroll
        for (int o = 0; o < 7; ++o) r[o] = raw_lds[i + o - 3];
#pragma unroll
        for (int o = 0; o < 7; ++o) pv = fmaxf(pv, o - 3 <= room ? r[o] : 0.f);
      } else {
        for (int o = -half; o <= min(half, room); ++o) pv = fmaxf(pv, raw_lds[i + o]);
      }
      scores_head[j] = pv;
    }
  };

  // statistics words of the team's nth head, and the validity bit of that use of the words
  auto words_of = [&](int nth) { return sy.stats + ((size_t)(team * 2 + (nth & 1)) * T) * ROWS; };
  auto tag_of = [](int nth) { return (((unsigned)nth >> 1) & 1u) ^ 1u; };

  // A value per (row of tile rt, key of this wave) in v[16] -> per row, combined over the wave's 32
  // keys with `op`: written [row][key] to the wave's LDS tile, read back by rows (a wave's LDS
  // operations execute in order), two lanes per row.  Returns the row's value in lanes hf == 0.
  auto over_keys = [&](const f32x16& v, auto op, int n32, int hf) {
#pragma unroll
    for (int i = 0; i < 16; ++i) zt[acc_row(i, hf) * ZT_STRIDE + n32] = v[i];
    float r = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x4 x = *reinterpret_cast<const f32x4*>(zt + n32 * ZT_STRIDE + hf * 16 + 4 * j);
      const float part = op(op(x[0], x[1]), op(x[2], x[3]));
      r = j == 0 ? part : op(r, part);
    }
    return op(r, __shfl_xor(r, 32));
  };

  // Everybody folds the statistics of the team in the same fixed order; thread (sub, rp) folds the
  // row pair rp of the members sub, sub + NSUB, ...: up to B 16-byte device-coherent loads in
  // flight at a time; a word that is not there yet is loaded again.  Leaves the rows' weights.
  auto gather_fold = [&](int nth) {
    constexpr int RPAIRS = S::RPAIRS, NSUB = S::NSUB, B = NSUB >= 16 ? 2 : NSUB >= 8 ? 4 : 8;
    constexpr bool ALL_AT_ONCE = NSUB == 8;                   // (64 score rows; the other instantiations lose registers to it)
    const int tid = opaque(threadIdx.x);
    float2* team_stats = words_of(nth);
    const unsigned tag = tag_of(nth);
    const int rp = tid % RPAIRS, sub = tid / RPAIRS;
    float M = NEG_BIG, Z = 0.f, M1 = NEG_BIG, Z1 = 0.f;
    {
      const __amdgpu_buffer_rsrc_t words = __builtin_amdgcn_make_buffer_rsrc(team_stats, 0, T * ROWS * 8, 0x00020000);
      int probes = 0;
      for (int m0 = sub; m0 < T; m0 += NSUB * B) {
        u32x4 v[B];
#pragma unroll
        for (int b2 = 0; b2 < B; ++b2) {
          const int mb = m0 + b2 * NSUB;
          v[b2] = u32x4{0u, tag << 31, 0u, tag << 31};
          if (mb < T) v[b2] = __builtin_amdgcn_raw_buffer_load_b128(words, (mb * ROWS + 2 * rp) * 8, 0, COHERENT);
        }
        if constexpr (ALL_AT_ONCE) {
          // words that are not there yet are asked for again, all of them at once per round: one
          // round trip per round, however many members are late
          for (;;) {
            bool missing = false;
#pragma unroll
            for (int b2 = 0; b2 < B; ++b2) missing |= (v[b2][1] >> 31) != tag || (v[b2][3] >> 31) != tag;
            if (!missing) break;
            if (gave_up[0]) break;
            if (++probes > SPIN_LIMIT ||
                ((probes & 63) == 63 && __hip_atomic_load(sy.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
              __hip_atomic_store(sy.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              gave_up[0] = 1;
              break;
            }
            __builtin_amdgcn_s_sleep(1);
#pragma unroll
            for (int b2 = 0; b2 < B; ++b2) {
              const int mb = m0 + b2 * NSUB;
              if ((v[b2][1] >> 31) != tag || (v[b2][3] >> 31) != tag)
                v[b2] = __builtin_amdgcn_raw_buffer_load_b128(words, (mb * ROWS + 2 * rp) * 8, 0, COHERENT);
            }
          }
#pragma unroll
          for (int b2 = 0; b2 < B; ++b2) {
            const int mb = m0 + b2 * NSUB;
            if (mb < T) {
              merge_stat(M, Z, make_float2(__uint_as_float(v[b2][0]), __uint_as_float(v[b2][1] & 0x7fffffffu)));
              merge_stat(M1, Z1, make_float2(__uint_as_float(v[b2][2]), __uint_as_float(v[b2][3] & 0x7fffffffu)));
            }
          }
        } else {
          // one after the other
#pragma unroll
          for (int b2 = 0; b2 < B; ++b2) {
            const int mb = m0 + b2 * NSUB;
            if (mb < T) {
              while ((v[b2][1] >> 31) != tag || (v[b2][3] >> 31) != tag) {
                if (gave_up[0]) break;
                if (++probes > SPIN_LIMIT ||
                    ((probes & 63) == 63 && __hip_atomic_load(sy.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                  __hip_atomic_store(sy.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  gave_up[0] = 1;
                  break;
                }
                __builtin_amdgcn_s_sleep(1);
                v[b2] = __builtin_amdgcn_raw_buffer_load_b128(words, (mb * ROWS + 2 * rp) * 8, 0, COHERENT);
              }
              merge_stat(M, Z, make_float2(__uint_as_float(v[b2][0]), __uint_as_float(v[b2][1] & 0x7fffffffu)));
              merge_stat(M1, Z1, make_float2(__uint_as_float(v[b2][2]), __uint_as_float(v[b2][3] & 0x7fffffffu)));
            }
          }
        }
      }
      fold_lds[sub * ROWS + 2 * rp] = make_float2(M, Z);
      fold_lds[sub * ROWS + 2 * rp + 1] = make_float2(M1, Z1);
    }
    lds_barrier();
    if (tid < ROWS) {
      M = NEG_BIG; Z = 0.f;
#pragma unroll
      for (int s2 = 0; s2 < NSUB; ++s2) merge_stat(M, Z, fold_lds[s2 * ROWS + tid]);
      // rows beyond R: weight zero
      wts_lds[tid] = (tid < g.R) ? __builtin_amdgcn_exp2f(ref_lds[tid] - (M + __builtin_amdgcn_logf(Z))) : 0.f;
    }
    lds_barrier();
  };

  // ---- the team's heads -----------------------------------------------------------------------
  int hg = team;
  const uint16_t* base = wave_base(hg);
  {
    const KeySource src = key_source(tile_at(base, 0), lay.row_bytes);
    const int v = tile_offset(src.row0, lane, lay.row_bytes);
#pragma unroll
    for (int t = 0; t < KS; ++t) kring[0][t] = load_operand(src, v, t);
    stage_tile(tile_at(base, 1), lay.row_bytes, lane, lds_address(w.stage));
    u32x4 qv[S::Q_PER_THREAD];
    fetch_q(hg, qv);
    commit_q(qv);
  }
  lds_barrier();
  int hg_prev = -1;                        // the head whose raw scores wait in LDS
  for (int nth = 0;; ++nth) {
    hg = __builtin_amdgcn_readfirstlane(hg);                 // (leaving the loop depends on LDS: say that hg is uniform)
    const int hn = hg + plan.n_teams;
    const bool more = hn < plan.n_heads;
    // B
    __builtin_amdgcn_s_setprio(PRIO_MATRIX);
    const uint16_t* base_next = wave_base(more ? hn : hg);
    wave_main<NRT>(
        w, E, kring, [&](int kt) { return key_source(tile_at(base, kt), lay.row_bytes); },
        [&](int kt) { return key_source(tile_at(base_next, kt), lay.row_bytes); },
        [&]() { stage_tile(tile_at(base_next, 1), lay.row_bytes, opaque(threadIdx.x) & 63, lds_address(w.stage)); }, more);
    if constexpr (S::ZT_IN_Q) lds_barrier();                  // the transposition tiles lie inside Q: every wave is done with it
    // C: the rows' maxima over this workgroup's keys ...
    __builtin_amdgcn_s_setprio(PRIO_CHAIN);
    const int n32c = opaque(w.n32), hfc = opaque(w.hf);
    static_for<0, NRT>([&](auto RT) {
      constexpr int rt = decltype(RT)::value;
      f32x16 mx = E[rt];
#pragma unroll
      for (int kt = 1; kt < KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx[i] = fmaxf(mx[i], E[kt * NRT + rt][i]);
      const float m = over_keys(mx, [](float a, float b) { return fmaxf(a, b); }, n32c, hfc);
      if (hfc == 0) stat_lds[wave * ROWS + rt * 32 + n32c] = m;
    });
    lds_barrier();                         // every wave is done with this head's Q
    if (tid < ROWS) {
      float m = stat_lds[tid];
#pragma unroll
      for (int v = 1; v < F_WAVES; ++v) m = fmaxf(m, stat_lds[v * ROWS + tid]);
      // (a row that sees none of the workgroup's keys: a finite "nothing")
      ref_lds[tid] = (m > NEG_BIG ? m : NEG_BIG) * g.scale2;
    }
    lds_barrier();
    // ... e = exp2(s - m) in place, and the rows' sums
    __builtin_amdgcn_s_setprio(PRIO_BULK);
    static_for<0, NRT>([&](auto RT) {
      constexpr int rt = decltype(RT)::value;
      f32x4 mv[4];
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) mv[gq] = *reinterpret_cast<const f32x4*>(ref_lds + rt * 32 + 8 * gq + 4 * hfc);
      f32x16 zs;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {      // four rows at a time: few values live next to the stored tiles
          float x[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) x[i] = fmaf(E[kt * NRT + rt][4 * h + i], g.scale2, -mv[h][i]);
#pragma unroll
          for (int i = 0; i < 4; ++i) E[kt * NRT + rt][4 * h + i] = __builtin_amdgcn_exp2f(x[i]);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            zs[4 * h + i] = kt == 0 ? E[kt * NRT + rt][4 * h + i] : zs[4 * h + i] + E[kt * NRT + rt][4 * h + i];
        }
      }
      const float z = over_keys(zs, [](float a, float b) { return a + b; }, n32c, hfc);
      if (hfc == 0) stat_lds[wave * ROWS + rt * 32 + n32c] = z;
    });
    __builtin_amdgcn_s_setprio(PRIO_CHAIN);                  // (until step B of the next head)
    lds_barrier();
    if (tid < ROWS) {
      float Z = stat_lds[tid];
#pragma unroll
      for (int v = 1; v < F_WAVES; ++v) Z += stat_lds[v * ROWS + tid];
      // (Z is a sum of non-negative terms: its sign bit is free)
      coherent_store(words_of(nth) + (size_t)member * ROWS + tid,
                     make_float2(ref_lds[tid], __uint_as_float(__float_as_uint(Z) | (tag_of(nth) << 31))));
    }
    // D: while the statistics travel (every wave is past its last use of this head's Q)
    {
      u32x4 qv[S::Q_PER_THREAD];
      if (more) fetch_q(hn, qv);
      if (hg_prev >= 0) pool_head(hg_prev);
      if (more) commit_q(qv);
    }
    // E
    gather_fold(nth);
    // F: this wave's keys
    {
      const int n32f = opaque(w.n32), hff = opaque(w.hf);
      float part[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) part[kt] = 0.f;
      static_for<0, NRT>([&](auto RT) {
        constexpr int rt = decltype(RT)::value;
        f32x4 wv[4];
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) wv[gq] = *reinterpret_cast<const f32x4*>(wts_lds + rt * 32 + 8 * gq + 4 * hff);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) part[kt] = fmaf(E[kt * NRT + rt][i], wv[i >> 2][i & 3], part[kt]);
      });
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        const float tot = part[kt] + __shfl_xor(part[kt], 32);
        const int kp = S::ROTATE ? (kt + w.rot) % KT : kt;
        const int j = w.key0 + kp * 32 + n32f;
        if (hff == 0) raw_lds[wave * KEYS_PER_WAVE + kp * 32 + n32f] = j < g.L ? tot : 0.f;
      }
    }
    lds_barrier();                         // raw scores complete; weights and maxima free
    if (!more || __builtin_amdgcn_readfirstlane(gave_up[0])) {
      pool_head(hg);
      break;
    }
    // (the raw scores are pooled inside the next round; they are next overwritten by step F of
    // that round, behind its barriers)
    hg_prev = hg;
    hg = hn;
    base = base_next;
  }
  stage_wait();                            // (a tile requested before a wait timed out: nothing writes LDS after the end)
}

// zero in the statistics words (validity bit of "nothing yet") and the status word
__global__ void fused_reset_kernel(uint4* words, int n_words, int* status) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) words[i] = make_uint4(0u, 0u, 0u, 0u);
  if (i == 0) *status = 0;
}

// ---- per-device set-up (see score_fused_init) -------------------------------------------------
constexpr int MAX_DEVICES = 64;
std::atomic<int> fused_resident[MAX_DEVICES][3];    // per kernel (32, 64, 128 score rows): workgroups held at once; -1: unusable
constexpr int slot_of(int nrt) { return nrt == 4 ? 2 : nrt - 1; }
// row tiles of the kernel that takes Rpad score rows
int tiles_for(int Rpad) { return Rpad > 64 ? 4 : Rpad / 32; }
std::atomic<int> fused_ready[MAX_DEVICES];

template <int NRT>
hipError_t init_rows(int dev, int cus, int coop) {
  constexpr int bytes = Cfg<NRT>::BYTES;
  hipError_t e;
  int resident = 0x7fffffff;
  for (const void* fn : {reinterpret_cast<const void*>(&fused_kernel<NRT, false>),
                         reinterpret_cast<const void*>(&fused_kernel<NRT, true>)}) {
    int per_cu = 0;
    if ((e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
    if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, F_THREADS, bytes)) != hipSuccess) return e;
    resident = std::min(resident, cus * per_cu);
  }
  fused_resident[dev][slot_of(NRT)].store((coop && resident > 0) ? resident : -1, std::memory_order_release);
  return hipSuccess;
}

int keys_per_block(int nrt) {
  return nrt == 1 ? Cfg<1>::KEYS_PER_BLOCK : nrt == 2 ? Cfg<2>::KEYS_PER_BLOCK : Cfg<4>::KEYS_PER_BLOCK;
}

// The team layout of a call on this device; false: the device cannot hold a team of this length (or
// has no cooperative launch) and the caller takes the two-pass kernels.
bool make_plan(const ScoreGeom& g, int pool, int resident, FusedPlan* out) {
  const int nrt = tiles_for(g.Rpad);
  FusedPlan plan;
  plan.T = (g.L + keys_per_block(nrt) - 1) / keys_per_block(nrt);
  plan.half = (pool - 1) / 2;
  const long long n_heads = (long long)g.n_inst * g.Hkv;
  if (resident <= 0 || plan.T > resident || n_heads > 0x7fffffffLL) return false;
  plan.n_heads = (int)n_heads;
  plan.n_teams = resident / plan.T;
  if (plan.n_teams > plan.n_heads) plan.n_teams = plan.n_heads;
  // the exchange memory is sized for FUSED_MAX_RESIDENT workgroups
  if ((size_t)plan.n_teams * plan.T > (size_t)FUSED_MAX_RESIDENT) return false;
  *out = plan;
  return true;
}

template <int NRT>
hipError_t launch_fused_rows(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const uint16_t* q,
                             const uint16_t* k,
                             float* scores, const Workspace& ws, hipStream_t st, bool* done) {
  *done = false;
  int dev = 0;
  hipError_t e;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = score_fused_init(dev)) != hipSuccess) return e;
  constexpr int bytes = Cfg<NRT>::BYTES;
  constexpr int ROWS = NRT * 32;
  FusedPlan plan;
  if (!make_plan(g, pool, fused_resident[dev][slot_of(NRT)].load(std::memory_order_acquire), &plan)) return hipSuccess;
  const size_t slots = (size_t)plan.n_teams * 2 * plan.T;
  FusedSync sy;
  sy.stats = reinterpret_cast<float2*>(ws.fused);
  sy.status = ws.status;
  const int n16 = (int)(slots * ROWS / 2);         // 16-byte pieces of the statistics words
  hipLaunchKernelGGL(fused_reset_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<uint4*>(sy.stats), n16, sy.status);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  ScoreGeom gg = g;
  QueryPos qq = qp;
  KvLayout ll = lay;
  float* edge = ws.raw;
  const void* fn = lay.table ? reinterpret_cast<const void*>(&fused_kernel<NRT, true>)
                             : reinterpret_cast<const void*>(&fused_kernel<NRT, false>);
  void* args[] = {&gg, &qq, &plan, &ll, &q, &k, &scores, &edge, &sy};
  // LAQ_COOPERATIVE_LAUNCH=0 in the environment: an ordinary launch of the same grid, for tools that
  // cannot follow cooperative launches (a process profiled by rocprofv3 ends in a segmentation fault
  // after any cooperative launch, also of an empty kernel).  The grid still fits the device, but
  // nothing then keeps other work from taking its place; the kernel's bounded waits turn a team
  // that is not on the device together into LAQ_ERR_TIMEOUT.
  static const bool plain_launch = [] {
    const char* v = getenv("LAQ_COOPERATIVE_LAUNCH");
    return v != nullptr && v[0] == '0';
  }();
  if (plain_launch) e = hipLaunchKernel(fn, dim3(plan.n_teams * plan.T), dim3(F_THREADS), args, bytes, st);
  else e = hipLaunchCooperativeKernel(fn, dim3(plan.n_teams * plan.T), dim3(F_THREADS), args, bytes, st);
  if (e != hipSuccess) return e;
  if (plan.half > 0 && plan.T > 1) {
    if ((e = launch_pool_boundaries(g, plan.half, plan.T, Cfg<NRT>::KEYS_PER_BLOCK, edge, scores, st)) != hipSuccess) return e;
  }
  *done = true;
  return hipSuccess;
}

}  // namespace

hipError_t score_fused_init(int dev) {
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (fused_ready[dev].load(std::memory_order_acquire)) return hipSuccess;
  int coop = 0, cus = 0;
  hipError_t e;
  if ((e = hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  if ((e = init_rows<1>(dev, cus, coop)) != hipSuccess) return e;
  if ((e = init_rows<2>(dev, cus, coop)) != hipSuccess) return e;
  if ((e = init_rows<4>(dev, cus, coop)) != hipSuccess) return e;
  fused_ready[dev].store(1, std::memory_order_release);
  return hipSuccess;
}

// Bytes of exchange memory of the single-read kernel: two sets of statistics words for
// FUSED_MAX_RESIDENT workgroups.
size_t fused_sync_bytes(const ScoreGeom& g) {
  return 2 * (size_t)FUSED_MAX_RESIDENT * (size_t)(tiles_for(g.Rpad) * 32) * sizeof(float2);
}

bool score_fused_supported(const ScoreGeom& g, const KvLayout& lay, int dtype) {
  return dtype == LAQ_BF16 && g.d == D && g.Rpad <= 128 && g.W <= MAX_QPOS &&
         ((long long)(lay.table ? lay.block_rows : g.L) + keys_per_block(tiles_for(g.Rpad))) * lay.row_bytes < 0x7fffffffLL;
}

// Whether launch_score_fused would launch for this call on the current device.
hipError_t score_fused_applies(const ScoreGeom& g, const KvLayout& lay, int dtype, bool* yes) {
  *yes = false;
  if (!score_fused_supported(g, lay, dtype)) return hipSuccess;
  int dev = 0;
  hipError_t e;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = score_fused_init(dev)) != hipSuccess) return e;
  FusedPlan plan;
  *yes = make_plan(g, 1, fused_resident[dev][slot_of(tiles_for(g.Rpad))].load(std::memory_order_acquire), &plan);
  return hipSuccess;
}

// Scores of every head into `scores`: raw with pool == 1, else max-pooled over the prefix.  *done
// says whether the kernels were launched: when the device cannot hold a team (very long heads) or
// has no cooperative launch they are not, and the caller takes the two-pass path.
hipError_t launch_score_fused(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const void* q,
                              const void* k, float* scores, const Workspace& ws, hipStream_t st, bool* done) {
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  const uint16_t* kk = static_cast<const uint16_t*>(k);
  const int ntile = tiles_for(g.Rpad);
  if (ntile == 1) return launch_fused_rows<1>(g, qp, lay, pool, qq, kk, scores, ws, st, done);
  if (ntile == 2) return launch_fused_rows<2>(g, qp, lay, pool, qq, kk, scores, ws, st, done);
  return launch_fused_rows<4>(g, qp, lay, pool, qq, kk, scores, ws, st, done);
}

}  // namespace laq
