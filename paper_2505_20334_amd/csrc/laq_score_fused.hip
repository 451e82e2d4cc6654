// bf16 scoring on the matrix cores with K read ONCE: the keys of a head stay in registers
// between the two softmax passes.  For KV heads with at most 64 score rows (R = G * W): there the
// two streaming passes are bound by memory and a single read pays; with more rows both designs
// are bound by the exponentials, which either computes twice, and the streaming kernels are as fast.
//
// The softmax of Eq. 4's observation window needs every score row's global (max, sum-exp) before
// a single probability can be summed, so a head's keys are needed twice.  Here a *team* of
// workgroups holds one whole head on chip: every wave keeps 128 key rows (32 KiB, d = 128) in
// 128 vector registers, already in the operand layout of v_mfma_f32_32x32x16_bf16; a workgroup
// of four waves (one per SIMD) covers 512 keys, a team of ceil(L / 512) workgroups covers the
// head (64 workgroups = 8 MiB of registers for L = 32768), two workgroups share a compute unit
// (one computes while the other waits for its team), and the device works on as many heads at
// once as it has room for teams (8).
//
// Per head, every workgroup of the team
//   1. pass 1:  D = K_tile * Q^T per (key tile, row tile): running (max, sum-exp2) per score
//      row over its 512 keys; the Q operands come from LDS (one copy of the head's Q_g per
//      workgroup), the K operands from the registers;
//   2. publishes its 2*R statistics, reads those of the whole team and folds them, in a fixed
//      order, into c = M + log2 Z per row (every member computes the same constants; nobody
//      waits for a combiner).  While the statistics travel it pools and stores the previous
//      head's scores and stages the next head's Q;
//   3. pass 2:  D = Q * K_tile^T: sum over the rows of exp2(s - c) per key = the raw score.  A
//      key tile that has been through pass 2 is reloaded with the team's next head: its eight
//      loads are spread over the matrix instructions of the tile that follows (those of the last
//      tile over the start of the next head's pass 1), because loads in operand layout touch 32
//      cache lines each and a burst of them holds up the waves that issue it.  The workgroup's
//      512 raw scores meet in LDS, where the sequence max-pool of every key whose window lies
//      inside the 512 is taken; the few keys next to a workgroup boundary are pooled by
//      pool_boundaries_kernel from raw scores left for it.
// Loads return in the order of their issue, so a wait for a small load would also wait for every
// key load in front of it: the order above has no key load in flight when the statistics and Q
// are fetched (pass 1 has consumed them all).
//
// The exchange in step 2 uses no cache maintenance (agent-scope release/acquire fences write
// back and invalidate L2 on this part, tens of microseconds each), no read-modify-write and no
// separate flag: a statistic is one 8-byte word (m, z) written with one device-coherent store
// (cache policy sc1) and read with device-coherent loads, and it validates itself -- z is never
// negative, so its sign bit carries one bit of the head's number, which differs between two
// consecutive uses of the same word.  A reader simply loads the words it needs and re-loads those
// that are not there yet; one store-to-load hop in all.  The team alternates between two sets of
// words, so a word is only overwritten after every member has read it (a member that publishes
// head n+2 has been through the exchange of head n+1, for which every member had published,
// which it does after reading head n).  All waits are bounded, and give up at once after one of
// them has timed out (status word of the workspace).  The kernel is started with a cooperative
// launch, which guarantees that the workgroups of a team are on the device together.
#include <atomic>
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
constexpr int F_WAVES = 4, F_THREADS = F_WAVES * 64;   // one wave per SIMD; two workgroups share a compute unit
constexpr int KT = 4;                        // key tiles per wave: 4 * 32 keys * 256 B = 128 registers
constexpr int KEYS_PER_WAVE = KT * 32, KEYS_PER_BLOCK = F_WAVES * KEYS_PER_WAVE;
static_assert(KEYS_PER_BLOCK == FUSED_ROWS, "the boundary pooling is told this chunk size");
// LDS row of Q: the d elements, one more reduction step of 16 elements that pass 2 uses to add the
// row's softmax constant on the matrix cores, and 16 bytes that make 128-bit operand reads of 16
// consecutive rows conflict-free
constexpr int QROWB = D * 2 + 32 + 16;
constexpr int SPIN_LIMIT = 1 << 20;          // probes; about a second, far beyond any legitimate wait
constexpr int MAX_HALF = (MAX_POOL - 1) / 2;
constexpr int COHERENT = 16;                 // cache policy bit "sc1": coherent across the device

#define LAQ_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
// holds a value's computation in its slot of the instruction stream (the scheduling fence alone
// does not: instruction selection sinks pure arithmetic to its first use)
#define LAQ_PIN(v) asm volatile("" : "+v"(v))

// Workgroup barrier for data that travels through LDS only: waits for this wave's LDS operations,
// not for its outstanding global loads (the key rows of the next head are in flight most of the
// time, and the barrier of __syncthreads() would wait for all of them).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int FROM, int TO, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FROM < TO) {
    f(std::integral_constant<int, FROM>{});
    static_for<FROM + 1, TO>(f);
  }
}

template <int NRT> struct FSmem {
  static constexpr int ROWS = NRT * 32;
  static constexpr int Q_BYTES = ROWS * QROWB;
  static constexpr int Q_PIECES = ROWS * (D / 8);                   // 16-byte pieces of one Q_g
  static constexpr int Q_PER_THREAD = (Q_PIECES + F_THREADS - 1) / F_THREADS;
  static constexpr int Q_BUFS = 2;                                  // this head / next
  static constexpr int OFF_Q = 0;                                   // Q_BUFS x [ROWS][QROWB] bf16 rows of Q_g
  static constexpr int PAIRS = ROWS / 2, NSUB = F_THREADS / PAIRS;   // the fold: threads per row pair
  static constexpr int OFF_STAT = OFF_Q + Q_BUFS * Q_BYTES;               // float2[F_WAVES][ROWS]: the waves' statistics
  static constexpr int OFF_FOLD = OFF_STAT + F_WAVES * ROWS * 8;    // float2[NSUB][ROWS]: the team's, per member subset
  static constexpr int OFF_LAST = OFF_FOLD + NSUB * ROWS * 8;       // int[ROWS]: last key every score row sees
  static constexpr int OFF_RAW = OFF_LAST + ROWS * 4;               // float[MAX_HALF + KEYS_PER_BLOCK + MAX_HALF]: the
                                                                    // workgroup's raw scores between zero margins
  static constexpr int OFF_FLAG = OFF_RAW + (KEYS_PER_BLOCK + 2 * MAX_HALF) * 4;   // int: "a wait has timed out"
  static constexpr int BYTES = OFF_FLAG + 16;
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
// for reduction step t.  Buffer loads against a descriptor that ends with the head's last row: rows
// beyond L-1 read as zeros (they are causally masked).  Consecutive rows lie row_bytes apart (256
// in a dense cache, more in a token-major or padded one).
struct KeySource {
  __amdgpu_buffer_rsrc_t rsrc;
};
__device__ __forceinline__ KeySource key_source(const uint16_t* khead, int L, int row_bytes) {
  KeySource s;
  s.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(khead), 0, (L - 1) * row_bytes + D * 2, 0x00020000);
  return s;
}
__device__ __forceinline__ bf16x8 load_operand(const KeySource& s, int voff_tile, int t) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(s.rsrc, voff_tile + t * 32, 0, 0));
}
// Byte offset within the head of (key tile kt of the wave, row l%32, slice l/32).  Recomputed
// where it is needed (it is the same for every head, and a register held across the whole kernel
// costs more than three instructions per tile), and opaque to the optimiser so that the step
// offsets fold into the instructions' immediate fields.
__device__ __forceinline__ int tile_offset(int key0, int kt, int lane, int row_bytes) {
  int l = lane;
  asm volatile("" : "+v"(l));
  return (key0 + kt * 32 + (l & 31)) * row_bytes + (l >> 5) * 16;
}

// ---- one pass over the wave's KT x NRT (key tile, row tile) pairs ----------------------------
// Software pipeline over the pairs: the MFMA chain of pair i is issued one instruction per slot,
// each slot also carrying a slice of the VALU work of pair i-1 (the loop is bound by VALU issue,
// so the slices are what fills the time; the fences and pins hold the interleave).
//
// PASS 1: lane = score row, accumulator registers = 16 keys: running (max, sum-exp2) per row.
// PASS 2: lane = key, accumulator registers = 16 rows: sum over rows of exp2(s - c) per key;
//         after the last row tile of a key tile the key's raw score is handed over (see Pass2Out).
// Reloading the registers with the next head (`next`, when `prefetch`): a key tile is free once the
// matrix instructions of its last pair have been issued, i.e. from stage (tile + 1) * NRT on; its KS
// loads are spread over the NRT stages from there.  For the last tile that window reaches beyond
// pass 2: its first stage is pass 2's draining stage, the others are the first stages of the next
// head's pass 1, which is called with `prefetch` set and the same `next` for that purpose.
struct WaveCtx {
  const char* q_lane;      // LDS: Q row (lane%32), slice (lane/32) of reduction step 0, row tile 0
  int lane, hf, n32;
  int key0;                // first key of this wave within the head
  int L, P;
  int row_bytes;           // distance between consecutive key rows
  int qmin;                // keys up to here are seen by every row: tiles below need no mask
  const int* last;         // LDS: last key every score row sees, for the causal mask
  float scale2;
};
// Pass 2 leaves the raw score of every key in the workgroup's LDS copy (rawbuf: this wave's first
// key); nothing in a pass stores to global memory, so that no pointer has to stay live -- or be
// spilled and reloaded, which would wait for the key rows in flight -- across the loop.
struct Pass2Out {
  float* rawbuf;
};

// Pass 2 adds -c/scale2 of every row to its dot products with one more MFMA per (key tile, row
// tile): the Q rows in LDS carry a ninth reduction step whose first three elements are the bf16
// pieces hi + mid + lo of that number (24 significant bits), and the key side of the step is this
// constant operand: ones in those three places, zeros elsewhere.  The accumulator times scale2 is
// then s - c, with no per-row constant in registers.
__device__ __forceinline__ bf16x8 ones_operand(int hf) {
  const u32x4 v = {hf == 0 ? 0x3F803F80u : 0u, hf == 0 ? 0x00003F80u : 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, v);
}
// the three pieces of v as the first 8 bytes of a row's ninth step
__device__ __forceinline__ uint2 split_bf16x3(float v) {
  auto rne = [](float x) {                       // nearest bf16 (ties to even), as fp32 bits with a zero low half
    const unsigned b = __float_as_uint(x);
    return (b + 0x7fffu + ((b >> 16) & 1u)) & 0xffff0000u;
  };
  const unsigned hi = rne(v);
  const float r1 = v - __uint_as_float(hi);      // exact
  const unsigned mid = rne(r1);
  const float r2 = r1 - __uint_as_float(mid);    // exact
  const unsigned lo = rne(r2);
  return make_uint2((hi >> 16) | mid, lo >> 16);
}

template <int NRT, int PASS>
__device__ __forceinline__ void wave_pass(const WaveCtx& w, bf16x8 (&kreg)[KT][KS], float (&m_run)[NRT],
                                          float (&z_run)[NRT], const Pass2Out& out, bool prefetch,
                                          const KeySource& next) {
  constexpr int NP = KT * NRT;             // pairs, key tile outer, row tile inner
  constexpr int SLOTS = PASS == 2 ? KS + 1 : KS;   // MFMAs per pair = slots of a stage
  constexpr int AHEAD = 2;                 // Q operands requested from LDS this many MFMAs ahead
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto q_addr = [&](int n) {               // operand of MFMA n = pair * SLOTS + step (step KS: the constants)
    const int rt = (n / SLOTS) % NRT, t = n % SLOTS;
    return w.q_lane + rt * 32 * QROWB + t * 32;
  };
  const bf16x8 kones = ones_operand(w.hf);
  bf16x8 ring[AHEAD];
#pragma unroll
  for (int n = 0; n < AHEAD; ++n) ring[n] = lds_operand(q_addr(n));
  f32x16 cur = zero, nxt = zero;
  // pass 1: running maximum of the unscaled dot products (the logit scale is positive, so the
  // order is the same); "nothing seen yet" is the same number in both units, so that a tile in
  // which a row sees no key leaves its statistics untouched
  // (the product is made opaque: folded into a later difference as a fused multiply-add it would
  // leave that difference one rounding error away from zero, which exp2 turns into 0 or inf)
  float raw_max[NRT];
  float nothing_yet = NEG_BIG * w.scale2;
  LAQ_PIN(nothing_yet);
#pragma unroll
  for (int r = 0; r < NRT; ++r) {
    raw_max[r] = NEG_BIG;
    if (PASS == 1) { m_run[r] = nothing_yet; z_run[r] = 0.f; }
  }
  float tot = 0.f;                         // pass 2: this key's sum over the row tiles so far

  static_for<0, NP + 1>([&](auto I) {
    constexpr int i = decltype(I)::value;
    constexpr int kt = i / NRT, rt = i % NRT;                 // pair whose MFMAs are issued in this stage
    constexpr int pk = (i - 1) / NRT, pr = (i - 1) % NRT;     // pair whose VALU work is done in this stage
    float m_new = 0.f, s = 0.f;
    // the key tile whose reload window this stage lies in, and the window's stage
    constexpr int PF_STAGE = PASS == 2 ? i - NRT : i + (KT - 1) * NRT + 1;   // stages since tile 0 became free
    constexpr bool PF_HERE = PF_STAGE >= 0 && PF_STAGE / NRT < KT && (PASS == 2 || PF_STAGE / NRT == KT - 1);
    constexpr int PF_TILE = PF_HERE ? PF_STAGE / NRT : 0, PF_R = PF_HERE ? PF_STAGE % NRT : 0;
    constexpr int PF_LO = PF_R * KS / NRT, PF_HI = (PF_R + 1) * KS / NRT;    // its loads PF_LO .. PF_HI-1 are due here
    int voff_next = 0;
    if constexpr (PF_HERE && PF_HI > PF_LO) {
      if (prefetch) voff_next = tile_offset(w.key0, PF_TILE, w.lane, w.row_bytes);
    }
#pragma unroll
    for (int t = 0; t < SLOTS; ++t) {
      const int n = i * SLOTS + t;
      if constexpr (i < NP) {
        // The chain starts from zero; in tiles with a key that some row does not see (wave-uniform
        // test) from -inf where a key is not visible to a row.  The two cases are separate
        // instructions so that the common one needs no copy of its start value; the bound goes
        // through an opaque copy so that the start vectors of all stages are not computed ahead and
        // kept alive.
        bool masked = false;
        int qmin_here = 0;
        const int t0 = w.key0 + kt * 32;
        if (t == 0) {
          qmin_here = __builtin_amdgcn_readfirstlane(w.qmin);
          asm volatile("" : "+s"(qmin_here));
          masked = t0 + 31 > qmin_here;
        }
        f32x16 start = (t > 0) ? nxt : zero;
        if (t == 0 && masked) {
          // (the lane's position goes through an opaque copy: what is derived from it is then computed
          // here, in the rare masked tile, and not ahead of the loop and kept in -- or spilled from --
          // registers for all tiles)
          int hf_here = w.hf, n32_here = w.n32;
          asm volatile("" : "+v"(hf_here), "+v"(n32_here));
          if (PASS == 1) {
            const int last_visible = w.last[rt * 32 + n32_here];         // this lane's row
#pragma unroll
            for (int e = 0; e < 16; ++e)
              if (t0 + acc_row(e, hf_here) > last_visible) start[e] = -INFINITY;
          } else {
            const int key = t0 + n32_here;                               // this lane's key
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {                             // rows 8*gq + 4*hf .. +3 of the tile
              const i32x4 lv = *reinterpret_cast<const i32x4*>(w.last + rt * 32 + 8 * gq + 4 * hf_here);
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if (key > lv[j]) start[4 * gq + j] = -INFINITY;
            }
          }
        }
        if (PASS == 1)
          nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[kt][t < KS ? t : 0], ring[n % AHEAD], start, 0, 0, 0);
        else
          nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[n % AHEAD], t < KS ? kreg[kt][t < KS ? t : 0] : kones, start, 0,
                                                        0, 0);
        if (n + AHEAD < NP * SLOTS) ring[n % AHEAD] = lds_operand(q_addr(n + AHEAD));
      }
      if constexpr (i > 0) {
        if (PASS == 1) {
          if (t == 0) {
            float mx = fmaxf(fmaxf(raw_max[pr], cur[0]), cur[1]);
#pragma unroll
            for (int e = 2; e < 16; e += 2) mx = fmaxf(fmaxf(mx, cur[e]), cur[e + 1]);
            raw_max[pr] = mx;
            m_new = mx * w.scale2;
            LAQ_PIN(m_new);
          } else {
            constexpr int REST = KS - 1;
            const int lo = (t - 1) * 16 / REST, hi = t * 16 / REST;
            float x[16];
#pragma unroll
            for (int e = lo; e < hi; ++e) x[e] = fmaf(cur[e], w.scale2, -m_new);
#pragma unroll
            for (int e = lo; e < hi; ++e) x[e] = __builtin_amdgcn_exp2f(x[e]);
#pragma unroll
            for (int e = lo; e < hi; ++e) s += x[e];
            LAQ_PIN(s);
          }
        } else {
          const int lo = t * 16 / SLOTS, hi = (t + 1) * 16 / SLOTS;
          float x[16];
#pragma unroll
          for (int e = lo; e < hi; ++e) x[e] = cur[e] * w.scale2;
#pragma unroll
          for (int e = lo; e < hi; ++e) x[e] = __builtin_amdgcn_exp2f(x[e]);
#pragma unroll
          for (int e = lo; e < hi; ++e) s += x[e];
          LAQ_PIN(s);
        }
      }
      if constexpr (PF_HERE && PF_HI > PF_LO) {
        // load j of the window's share goes into slot (j - PF_LO) * SLOTS / (PF_HI - PF_LO)
        constexpr int N_HERE = PF_HI - PF_LO;
#pragma unroll
        for (int j = 0; j < N_HERE; ++j)
          if (t == j * SLOTS / N_HERE && prefetch) kreg[PF_TILE][PF_LO + j] = load_operand(next, voff_next, PF_LO + j);
      }
      LAQ_SCHED_FENCE();
    }
    if constexpr (i > 0) {
      if (PASS == 1) {
        z_run[pr] = fmaf(z_run[pr], __builtin_amdgcn_exp2f(fminf(m_run[pr] - m_new, 0.f)), s);
        m_run[pr] = m_new;
      } else {
        tot += s;
        if (pr == NRT - 1) {
          tot += __shfl_xor(tot, 32);
          const int j = w.key0 + pk * 32 + w.n32;
          if (w.hf == 0) out.rawbuf[pk * 32 + w.n32] = j < w.L ? tot : 0.f;
          tot = 0.f;
        }
      }
    }
    cur = nxt;
  });
}

// ---- exchange buffers --------------------------------------------------------------------------
// Per team, two sets of statistics words [team size][rows]: (m, z) with the validity bit in the
// sign of z (see the head of the file).
struct FusedSync {
  float2* stats;           // [n_teams][2][T][rows]
  int* status;             // != 0: a wait has timed out (results are not valid)
};
struct FusedPlan {
  int T;                   // workgroups per team = ceil(L / 512)
  int n_teams;
  int n_heads;             // team t takes heads t, t + n_teams, ...
  int half;                // (pool kernel - 1) / 2; 0: raw scores
  int stagger;             // team t starts t * stagger ticks (10 ns) late, so that the teams reload their
                           // registers at different times
};

template <int NRT>
__global__ __launch_bounds__(F_THREADS, 2) void fused_kernel(ScoreGeom g, QueryPos qp, FusedPlan plan, KvLayout lay,
                                                             const uint16_t* __restrict__ q,
                                                             const uint16_t* __restrict__ k,
                                                             float* __restrict__ scores, float* __restrict__ edge,
                                                             FusedSync sy) {
  using S = FSmem<NRT>;
  constexpr int ROWS = NRT * 32;
  extern __shared__ __align__(16) char smem[];
  float2* stat_lds = reinterpret_cast<float2*>(smem + S::OFF_STAT);
  float2* fold_lds = reinterpret_cast<float2*>(smem + S::OFF_FOLD);
  int* last_lds = reinterpret_cast<int*>(smem + S::OFF_LAST);
  float* raw_lds = reinterpret_cast<float*>(smem + S::OFF_RAW) + MAX_HALF;       // key 0 of the workgroup
  volatile int* gave_up = reinterpret_cast<volatile int*>(smem + S::OFF_FLAG);

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = plan.T, half = plan.half;
  const int team = blockIdx.x / T, member = blockIdx.x - team * T;
  if (team >= plan.n_teams || team >= plan.n_heads) return;

  WaveCtx w;
  w.lane = lane; w.hf = lane >> 5; w.n32 = lane & 31;
  w.q_lane = nullptr;
  w.key0 = member * KEYS_PER_BLOCK + wave * KEYS_PER_WAVE;
  w.L = g.L; w.P = g.P; w.qmin = g.qmin; w.scale2 = g.scale2; w.row_bytes = lay.row_bytes;
  w.last = last_lds;
  // rows beyond R (zero queries) see every key; their constant is huge, so they add nothing
  for (int r = tid; r < ROWS; r += F_THREADS) last_lds[r] = r < g.R ? qp.last[r % g.W] : g.L - 1;
  if (tid < 2 * MAX_HALF) raw_lds[tid < MAX_HALF ? tid - MAX_HALF : KEYS_PER_BLOCK + tid - MAX_HALF] = 0.f;
  if (tid == 0) gave_up[0] = 0;
  // the ninth reduction step of every Q row: zero except for the constant's pieces, written per head
  for (int r = tid; r < S::Q_BUFS * ROWS; r += F_THREADS) {
    char* ext = smem + S::OFF_Q + (r / ROWS) * S::Q_BYTES + (r % ROWS) * QROWB + D * 2;
    *reinterpret_cast<u32x4*>(ext) = u32x4{0u, 0u, 0u, 0u};
    *reinterpret_cast<u32x4*>(ext + 16) = u32x4{0u, 0u, 0u, 0u};
  }

  bf16x8 kreg[KT][KS];
  float m_run[NRT], z_run[NRT];

  // Q_g of head `hq` (rows hq*R .. +R-1 of Q; rows beyond R are zero): global memory -> registers,
  // and later registers -> LDS buffer `buf`
  auto fetch_q = [&](int hq, u32x4 (&qv)[S::Q_PER_THREAD]) {
    const uint16_t* qg = q + (size_t)hq * g.R * D;
#pragma unroll
    for (int i = 0; i < S::Q_PER_THREAD; ++i) {
      const int p = tid + i * F_THREADS, row = p / (D / 8), col = p % (D / 8);
      qv[i] = u32x4{0u, 0u, 0u, 0u};
      if (p < S::Q_PIECES && row < g.R) qv[i] = *reinterpret_cast<const u32x4*>(qg + (size_t)row * D + col * 8);
    }
  };
  auto commit_q = [&](char* dst, const u32x4 (&qv)[S::Q_PER_THREAD]) {
#pragma unroll
    for (int i = 0; i < S::Q_PER_THREAD; ++i) {
      const int p = tid + i * F_THREADS, row = p / (D / 8), col = p % (D / 8);
      if (p < S::Q_PIECES) *reinterpret_cast<u32x4*>(dst + row * QROWB + col * 16) = qv[i];
    }
  };
  // key rows of head hg_ (instance hg_ / Hkv, KV head hg_ % Hkv)
  auto keys_of = [&](int hg_) {
    const int inst = hg_ / g.Hkv, head = hg_ - inst * g.Hkv;
    return key_source(k + (size_t)inst * lay.inst + (size_t)head * lay.head, g.L, lay.row_bytes);
  };
  // Scores of head hg_ from the raw scores that its pass 2 left in LDS (zero beyond the head's last
  // key and in the margins).  Keys behind the prefix and, without pooling, all keys are stored as
  // they are.  A prefix key whose pooling window lies inside the workgroup's 512 keys gets the
  // maximum over the part of the window inside the prefix; the raw scores of the first and last
  // 2*half keys go to the edge record of this workgroup, from which pool_boundaries_kernel pools the
  // keys next to a boundary.
  auto pool_head = [&](int hg_) {
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
  auto q_buf_of = [&](int nth) { return smem + S::OFF_Q + (nth & 1) * S::Q_BYTES; };
  auto words_of = [&](int nth) { return sy.stats + ((size_t)(team * 2 + (nth & 1)) * T) * ROWS; };
  auto tag_of = [](int nth) { return (((unsigned)nth >> 1) & 1u) ^ 1u; };

  // Pass 1 of the team's nth head on the registers (its Q is in LDS buffer nth & 1); statistics
  // published.  `arriving`: the last key tile is still being reloaded, from `src` (see wave_pass).
  auto pass1_publish = [&](int nth, bool arriving, const KeySource& src) {
    w.q_lane = q_buf_of(nth) + w.n32 * QROWB + w.hf * 16;
    Pass2Out no_out;
    no_out.rawbuf = nullptr;
    wave_pass<NRT, 1>(w, kreg, m_run, z_run, no_out, arriving, src);
    // the two lanes that share a row, then the waves
#pragma unroll
    for (int r = 0; r < NRT; ++r) {
      float M = m_run[r], Z = z_run[r];
      const float Mo = __shfl_xor(M, 32), Zo = __shfl_xor(Z, 32);
      if (w.hf == 0) {
        merge_stat(M, Z, make_float2(Mo, Zo));
        stat_lds[wave * ROWS + r * 32 + w.n32] = make_float2(M, Z);
      }
    }
    lds_barrier();
    if (tid < ROWS) {
      float M = NEG_BIG, Z = 0.f;
#pragma unroll
      for (int v = 0; v < F_WAVES; ++v) merge_stat(M, Z, stat_lds[v * ROWS + tid]);
      // (Z is a sum of non-negative terms: its sign bit is free)
      coherent_store(words_of(nth) + (size_t)member * ROWS + tid,
                     make_float2(M, __uint_as_float(__float_as_uint(Z) | (tag_of(nth) << 31))));
    }
    // (the statistics buffer is next written after the next pass 1, several barriers on)
  };

  // Everybody folds the statistics of the team in the same fixed order; the row constants go into
  // the ninth reduction step of the head's Q rows.  Thread (sub, rp) folds the row pair rp of the
  // members sub, sub + NSUB, ...: up to B 16-byte device-coherent loads in flight at a time; a word
  // that is not there yet is loaded again.
  auto gather_fold = [&](int nth) {
    constexpr int PAIRS = S::PAIRS, NSUB = S::NSUB, B = NSUB >= 16 ? 4 : 8;
    float2* team_stats = words_of(nth);
    const unsigned tag = tag_of(nth);
    char* q_buf = q_buf_of(nth);
    const int rp = tid % PAIRS, sub = tid / PAIRS;
    float M = NEG_BIG, Z = 0.f, M1 = NEG_BIG, Z1 = 0.f;
    if (sub < NSUB) {
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
      fold_lds[sub * ROWS + 2 * rp] = make_float2(M, Z);
      fold_lds[sub * ROWS + 2 * rp + 1] = make_float2(M1, Z1);
    }
    lds_barrier();
    if (tid < ROWS) {
      M = NEG_BIG; Z = 0.f;
#pragma unroll
      for (int s2 = 0; s2 < NSUB; ++s2) merge_stat(M, Z, fold_lds[s2 * ROWS + tid]);
      const float c = (tid < g.R) ? M + __builtin_amdgcn_logf(Z) : 1.0e30f;
      *reinterpret_cast<uint2*>(q_buf + tid * QROWB + D * 2) = split_bf16x3(-c / g.scale2);
    }
    lds_barrier();
  };

  // ---- the team's heads -----------------------------------------------------------------------
  int hg = team;
  if (plan.stagger > 0) {
    const long long until = wall_clock64() + (long long)team * plan.stagger;
    while (wall_clock64() < until) __builtin_amdgcn_s_sleep(8);
  }
  {
    const KeySource src = keys_of(hg);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const int v = tile_offset(w.key0, kt, lane, lay.row_bytes);
#pragma unroll
      for (int t = 0; t < KS; ++t) kreg[kt][t] = load_operand(src, v, t);
    }
    u32x4 qv[S::Q_PER_THREAD];
    fetch_q(hg, qv);
    commit_q(q_buf_of(0), qv);
  }
  lds_barrier();
  int hg_prev = -1;                        // the head whose raw scores wait in LDS
  for (int nth = 0;; ++nth) {
    const int hn = hg + plan.n_teams;
    const bool more = hn < plan.n_heads;
    pass1_publish(nth, nth > 0, keys_of(hg));
    // while the statistics travel (no key load is in flight any more): the next head's Q is
    // requested, the previous head's scores are stored, Q is put into the other buffer
    {
      u32x4 qv[S::Q_PER_THREAD];
      if (more) fetch_q(hn, qv);
      if (hg_prev >= 0) pool_head(hg_prev);
      if (more) commit_q(q_buf_of(nth + 1), qv);
    }
    gather_fold(nth);
    Pass2Out out;
    out.rawbuf = raw_lds + wave * KEYS_PER_WAVE;
    wave_pass<NRT, 2>(w, kreg, m_run, z_run, out, more, keys_of(more ? hn : hg));
    lds_barrier();                         // every wave is done with this head's Q and constants; raw scores complete
    if (!more || gave_up[0]) {
      pool_head(hg);
      break;
    }
    // (the raw scores are pooled inside the next round; they are next overwritten by the pass 2 of
    // that round, behind its barriers)
    hg_prev = hg;
    hg = hn;
  }
}

// zero in the statistics words (validity bit of "nothing yet") and the status word
__global__ void fused_reset_kernel(uint4* words, int n_words, int* status) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) words[i] = make_uint4(0u, 0u, 0u, 0u);
  if (i == 0) *status = 0;
}

// ---- per-device set-up (see score_fused_init) -------------------------------------------------
constexpr int MAX_DEVICES = 64;
std::atomic<int> fused_resident[MAX_DEVICES][2];    // per row-tile count: workgroups held at once; -1: unusable
std::atomic<int> fused_ready[MAX_DEVICES];

template <int NRT>
hipError_t init_rows(int dev, int cus, int coop) {
  constexpr int bytes = FSmem<NRT>::BYTES;
  const void* fn = reinterpret_cast<const void*>(&fused_kernel<NRT>);
  hipError_t e;
  int per_cu = 0;
  if ((e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, F_THREADS, bytes)) != hipSuccess) return e;
  fused_resident[dev][NRT - 1].store((coop && per_cu > 0) ? cus * per_cu : -1, std::memory_order_release);
  return hipSuccess;
}

// The team layout of a call on this device; false: the device cannot hold a team of this length (or
// has no cooperative launch) and the caller takes the two-pass kernels.
bool make_plan(const ScoreGeom& g, int pool, int resident, FusedPlan* out) {
  const int nrt = g.Rpad / 32;
  FusedPlan plan;
  plan.T = (g.L + KEYS_PER_BLOCK - 1) / KEYS_PER_BLOCK;
  plan.half = (pool - 1) / 2;
  const long long n_heads = (long long)g.n_inst * g.Hkv;
  if (resident <= 0 || plan.T > resident || n_heads > 0x7fffffffLL) return false;
  plan.n_heads = (int)n_heads;
  plan.n_teams = resident / plan.T;
  if (plan.n_teams > plan.n_heads) plan.n_teams = plan.n_heads;
  // a head takes a team roughly 5 us per 32-row tile; with at least four heads per team the teams
  // are spread over that time
  plan.stagger = (plan.n_heads >= 4 * plan.n_teams && plan.n_teams > 1) ? 500 * nrt / plan.n_teams : 0;
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
  constexpr int bytes = FSmem<NRT>::BYTES;
  constexpr int ROWS = NRT * 32;
  FusedPlan plan;
  if (!make_plan(g, pool, fused_resident[dev][NRT - 1].load(std::memory_order_acquire), &plan)) return hipSuccess;
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
  const void* fn = reinterpret_cast<const void*>(&fused_kernel<NRT>);
  void* args[] = {&gg, &qq, &plan, &ll, &q, &k, &scores, &edge, &sy};
  e = hipLaunchCooperativeKernel(fn, dim3(plan.n_teams * plan.T), dim3(F_THREADS), args, bytes, st);
  if (e != hipSuccess) return e;
  if (plan.half > 0 && plan.T > 1) {
    if ((e = launch_pool_boundaries(g, plan.half, plan.T, KEYS_PER_BLOCK, edge, scores, st)) != hipSuccess) return e;
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
  fused_ready[dev].store(1, std::memory_order_release);
  return hipSuccess;
}

// Bytes of exchange memory of the single-read kernel: two sets of statistics words for
// FUSED_MAX_RESIDENT workgroups.
size_t fused_sync_bytes(const ScoreGeom& g) {
  return 2 * (size_t)FUSED_MAX_RESIDENT * (size_t)g.Rpad * sizeof(float2);
}

bool score_fused_supported(const ScoreGeom& g, const KvLayout& lay, int dtype) {
  return dtype == LAQ_BF16 && g.d == D && g.Rpad <= 64 && g.W <= MAX_QPOS && !lay.table &&
         ((long long)g.L + KEYS_PER_BLOCK) * lay.row_bytes < 0x7fffffffLL;
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
  *yes = make_plan(g, 1, fused_resident[dev][g.Rpad / 32 - 1].load(std::memory_order_acquire), &plan);
  return hipSuccess;
}

// Scores of every head into `scores`: raw with pool == 1, else max-pooled over the prefix.  *done
// says whether the kernels were launched: when the device cannot hold a team (very long heads) or
// has no cooperative launch they are not, and the caller takes the two-pass path.
hipError_t launch_score_fused(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const void* q,
                              const void* k, float* scores, const Workspace& ws, hipStream_t st, bool* done) {
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  const uint16_t* kk = static_cast<const uint16_t*>(k);
  const int ntile = g.Rpad / 32;
  if (ntile == 1) return launch_fused_rows<1>(g, qp, lay, pool, qq, kk, scores, ws, st, done);
  return launch_fused_rows<2>(g, qp, lay, pool, qq, kk, scores, ws, st, done);
}

}  // namespace laq
