// C ABI of the LAQ re-eviction library (declared in include/laq.h): argument checks,
// geometry, kernel dispatch.  No device memory is allocated here.
#include <math.h>
#include <string.h>

#include <atomic>

#include "laq_internal.h"

namespace laq {

static bool pool_ok(int pool) { return pool >= 1 && pool <= MAX_POOL && (pool % 2) == 1; }
static bool pool_avg(const laq_shape* s) { return s->pool_mode == LAQ_POOL_AVG; }

// Geometry of a call.  Returns LAQ_OK, LAQ_ERR_INVALID or LAQ_ERR_UNSUPPORTED; fills the query
// position table (qp may be null for calls that do not score) when positions are explicit.
static int make_geom(const laq_shape* s, ScoreGeom* g, QueryPos* qp = nullptr) {
  if (!s) return LAQ_ERR_INVALID;
  if (s->n_inst < 1 || s->Hq < 1 || s->Hkv < 1 || s->d < 8 || s->d > 256 || (s->d % 8) != 0) return LAQ_ERR_INVALID;
  if (s->L < 1 || s->W < 1 || (s->Hq % s->Hkv) != 0) return LAQ_ERR_INVALID;
  if ((!s->q_pos || s->keep < 0) && s->W > s->L) return LAQ_ERR_INVALID;   // trailing-window defaults need W <= L
  if (s->keep > s->L) return LAQ_ERR_INVALID;
  if (s->dtype != LAQ_F32 && s->dtype != LAQ_BF16) return LAQ_ERR_INVALID;
  if (s->pool_mode != LAQ_POOL_MAX && s->pool_mode != LAQ_POOL_AVG) return LAQ_ERR_INVALID;
  if (!(s->scale == s->scale) || isinf(s->scale)) return LAQ_ERR_INVALID;
  g->n_inst = s->n_inst; g->Hq = s->Hq; g->Hkv = s->Hkv; g->d = s->d; g->L = s->L; g->W = s->W;
  g->G = s->Hq / s->Hkv;
  g->R = g->G * s->W;
  g->keep = s->keep < 0 ? s->W : s->keep;
  g->P = s->L - g->keep;
  g->pos0 = s->L - s->W;
  g->explicit_pos = s->q_pos ? 1 : 0;
  g->qmin = g->pos0;
  if (s->q_pos) {
    if (s->W > MAX_QPOS) return LAQ_ERR_UNSUPPORTED;
    int qmin = s->L - 1;
    for (int w = 0; w < s->W; ++w) {
      if (s->q_pos[w] < 0) return LAQ_ERR_INVALID;
      const int last = s->q_pos[w] < s->L - 1 ? s->q_pos[w] : s->L - 1;
      if (qp) qp->last[w] = last;
      if (last < qmin) qmin = last;
    }
    g->qmin = qmin;
  } else if (qp && s->W <= MAX_QPOS) {
    for (int w = 0; w < s->W; ++w) qp->last[w] = g->pos0 + w;
  }
  g->Rpad = (g->R + 31) / 32 * 32;
  g->nchunk = (s->L + CHUNK_ROWS - 1) / CHUNK_ROWS;
  const float sc = s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->d);
  g->scale2 = sc * 1.44269504088896340736f;
  return LAQ_OK;
}

// Layout of k / v from the shape's strides (all zero: dense).  LAQ_ERR_INVALID on strides that are
// not 16-byte multiples, overlap a row, or mix zero and non-zero.
static int make_layout(const laq_shape* s, const ScoreGeom& g, KvLayout* lay) {
  const int eb = s->dtype == LAQ_F32 ? 4 : 2;
  const int64_t si = s->kv_stride_inst, sh = s->kv_stride_head, sr = s->kv_stride_row;
  lay->table = nullptr;
  lay->blocks_per_inst = 0;
  lay->block_rows = 0;
  lay->block = 0;
  if (s->block_table) {
    // a pool of blocks: strides inside a block, and between blocks
    const int64_t br = s->block_rows, sb = s->kv_stride_block;
    if (br < 256 || br % 256 || br > (1 << 24)) return LAQ_ERR_INVALID;
    if ((sh == 0) != (sr == 0)) return LAQ_ERR_INVALID;
    lay->row = sr ? sr : g.d;
    lay->head = sh ? sh : br * g.d;
    if (lay->row < g.d || lay->head < 1 || sb < 1 || (lay->row * eb) % 16 || (lay->head * eb) % 16 || (sb * eb) % 16)
      return LAQ_ERR_INVALID;
    if (lay->row * eb > 0x7fffffffLL) return LAQ_ERR_INVALID;
    lay->inst = 0;
    lay->dense = 0;
    lay->table = s->block_table;
    lay->blocks_per_inst = (int32_t)((g.L + br - 1) / br);
    lay->block_rows = (int32_t)br;
    lay->block = sb;
    lay->row_bytes = (int32_t)(lay->row * eb);
    return LAQ_OK;
  }
  if (s->block_rows != 0 || s->kv_stride_block != 0) return LAQ_ERR_INVALID;
  if (si == 0 && sh == 0 && sr == 0) {
    lay->row = g.d;
    lay->head = (int64_t)g.L * g.d;
    lay->inst = (int64_t)g.Hkv * g.L * g.d;
    lay->dense = 1;
  } else {
    if (sr < g.d || sh < 1 || si < 1 || (sr * eb) % 16 || (sh * eb) % 16 || (si * eb) % 16) return LAQ_ERR_INVALID;
    if (sr * eb > 0x7fffffffLL) return LAQ_ERR_INVALID;
    lay->row = sr;
    lay->head = sh;
    lay->inst = si;
    lay->dense = (sr == g.d && sh == (int64_t)g.L * g.d && si == (int64_t)g.Hkv * g.L * g.d) ? 1 : 0;
  }
  lay->row_bytes = (int32_t)(lay->row * eb);
  return LAQ_OK;
}

static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// chunks per head under the finest chunking any scoring path uses
static size_t max_chunks(const ScoreGeom& g) { return ((size_t)g.L + MIN_CHUNK_ROWS - 1) / MIN_CHUNK_ROWS; }

size_t workspace_bytes(const ScoreGeom& g) {
  const size_t heads = (size_t)g.n_inst * g.Hkv;
  return round256(heads * max_chunks(g) * g.Rpad * sizeof(float2)) + round256(heads * g.Rpad * sizeof(float)) +
         2 * round256(heads * g.L * sizeof(float)) + round256(fused_sync_bytes(g)) + 256;
}

Workspace carve_workspace(const ScoreGeom& g, void* ws) {
  const size_t heads = (size_t)g.n_inst * g.Hkv;
  char* base = static_cast<char*>(ws);
  Workspace w;
  w.part = reinterpret_cast<float2*>(base);
  base += round256(heads * max_chunks(g) * g.Rpad * sizeof(float2));
  w.rowc = reinterpret_cast<float*>(base);
  base += round256(heads * g.Rpad * sizeof(float));
  w.raw = reinterpret_cast<float*>(base);
  base += round256(heads * g.L * sizeof(float));
  w.pooled = reinterpret_cast<float*>(base);
  base += round256(heads * g.L * sizeof(float));
  w.fused = base;
  base += round256(fused_sync_bytes(g));
  w.ctr = reinterpret_cast<int*>(base);
  w.status = w.ctr + 8;
  return w;
}

// Fill the per-instance table for instances [i0, i0+n) and return the largest Bk among them.
static int fill_table(int Hkv, int L, const int32_t* budget, int i0, int n, int64_t row_base,
                      InstTable* tab, int64_t* rows_after) {
  int bk_max = 0;
  int64_t row = row_base;
  for (int i = 0; i < n; ++i) {
    const int bk = budget[i0 + i] < L ? budget[i0 + i] : L;
    tab->bk[i] = bk;
    tab->row0[i] = row;
    row += (int64_t)Hkv * bk;
    if (bk > bk_max) bk_max = bk;
  }
  *rows_after = row;
  return bk_max;
}

// The same for the gather, whose grid covers the rows of every instance exactly.
static void fill_compact_table(int Hkv, int L, int pieces_per_row, const int32_t* budget, int i0, int n,
                               int64_t row_base, CompactTable* tab, int64_t* rows_after) {
  int64_t row = row_base, blk = 0;
  for (int i = 0; i < n; ++i) {
    const int bk = budget[i0 + i] < L ? budget[i0 + i] : L;
    tab->bk[i] = bk;
    tab->row0[i] = row;
    tab->blk0[i] = (int32_t)blk;
    row += (int64_t)Hkv * bk;
    blk += ((int64_t)Hkv * bk * pieces_per_row + COMPACT_THREADS - 1) / COMPACT_THREADS;
  }
  tab->blk0[n] = (int32_t)blk;
  *rows_after = row;
}

static bool budgets_ok(const laq_shape* s, const ScoreGeom& g, const int32_t* budget) {
  if (!budget) return false;
  for (int i = 0; i < s->n_inst; ++i)
    if (budget[i] < g.keep || budget[i] < 1) return false;
  return true;
}

// ---- per-device set-up ---------------------------------------------------------------------
// Kernel attributes and residency of the scoring kernels on the current device, and the address of
// the library's own scratch array there.  `scratch` is the workspace of laq_evict_static: in host
// code its name is only a handle, and every device holds its own copy at its own address, which is
// looked up once per device (with that device current) and used from then on.
static __device__ __align__(256) unsigned char scratch[LAQ_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static std::atomic<void*> scratch_of[MAX_DEVICES];

static int init_current_device(int* dev_out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return LAQ_ERR_DEVICE;
  if (dev_out) *dev_out = dev;
  if (scratch_of[dev].load(std::memory_order_acquire)) return LAQ_OK;
  if (score_mfma_init(dev) != hipSuccess || score_fused_init(dev) != hipSuccess) return LAQ_ERR_DEVICE;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LAQ_ERR_DEVICE;
  scratch_of[dev].store(ptr, std::memory_order_release);
  return LAQ_OK;
}

// The single-read kernel's cooperative launch and its serial start cost about 15 us more than the
// launches of the two streaming passes; measured on an MI355X it is the faster one from 128 MiB of
// keys per call on (21-27 % at 1 GiB and more).
static bool single_read_wanted(const laq_shape* shape, const ScoreGeom& g) {
  if (shape->score_choice == LAQ_CHOOSE_SINGLE_READ) return true;
  if (shape->score_choice == LAQ_CHOOSE_TWO_PASS) return false;
  // by itself: where it is the faster one -- at most 64 score rows per KV head (with more, a
  // workgroup holds 256 keys and reads as many bytes of its team's statistics as of keys) and
  // enough keys to pay for the cooperative launch
  const long long key_bytes = (long long)g.n_inst * g.Hkv * g.L * g.d * (shape->dtype == LAQ_F32 ? 4 : 2);
  return g.Rpad <= 64 && key_bytes >= (128LL << 20);
}

static int score_impl(const laq_shape* shape, const void* q_win, const void* k, int pool, float* scores,
                      void* ws, size_t ws_bytes, hipStream_t st) {
  ScoreGeom g;
  QueryPos qp;
  memset(&qp, 0, sizeof qp);
  const int rc = make_geom(shape, &g, &qp);
  if (rc != LAQ_OK) return rc;
  KvLayout lay;
  if (make_layout(shape, g, &lay) != LAQ_OK) return LAQ_ERR_INVALID;
  if (!pool_ok(pool) || !q_win || !k || !scores) return LAQ_ERR_INVALID;
  if (!ws || ws_bytes < workspace_bytes(g)) return LAQ_ERR_WORKSPACE;
  if (g.Hkv > 65535 || g.n_inst > 65535 || (long long)g.Hkv * g.n_inst > 0x7fffffffLL) return LAQ_ERR_UNSUPPORTED;
  if ((g.L + 255) / 256 > 65535) return LAQ_ERR_UNSUPPORTED;      // grid limit of the pooling kernel
  const int rc_init = init_current_device(nullptr);
  if (rc_init != LAQ_OK) return rc_init;
  const Workspace w = carve_workspace(g, ws);
  hipError_t e;
  const bool avg = pool_avg(shape) && pool > 1;
  const bool mfma = score_mfma_supported(g, lay, shape->dtype);
  const bool fused = SINGLE_READ_ENABLED && score_fused_supported(g, lay, shape->dtype) && single_read_wanted(shape, g);
  // matrix cores: the single-read kernel where a team of workgroups can hold a head, else the two
  // streaming passes; both fuse the max pooling, the average goes through the raw-score plane
  auto score_on_matrix_cores = [&](int p, float* dst) -> hipError_t {
    bool done = false;
    if (fused) {
      const hipError_t ef = launch_score_fused(g, qp, lay, p, q_win, k, dst, w, st, &done);
      if (ef != hipSuccess || done) return ef;
    }
    return launch_score_mfma(g, qp, lay, p, q_win, k, dst, w, st);
  };
  if (mfma && !avg) {
    e = score_on_matrix_cores(pool, scores);
  } else {
    float* raw = pool > 1 ? w.raw : scores;
    e = mfma ? score_on_matrix_cores(1, raw) : launch_score_generic(g, qp, lay, shape->dtype, q_win, k, raw, w, st);
    if (e == hipSuccess && pool > 1) e = launch_pool(g, pool, avg, raw, scores, st);
  }
  return e == hipSuccess ? LAQ_OK : LAQ_ERR_DEVICE;
}

static int select_impl(const laq_shape* shape, const float* scores, const int32_t* budget, int pool,
                       int32_t* idx, hipStream_t st) {
  ScoreGeom g;
  const int rc = make_geom(shape, &g);
  if (rc != LAQ_OK) return rc;
  if (!pool_ok(pool) || !scores || !idx || !budgets_ok(shape, g, budget)) return LAQ_ERR_INVALID;
  if (g.Hkv > 65535) return LAQ_ERR_UNSUPPORTED;
  int64_t row = 0;
  for (int i0 = 0; i0 < shape->n_inst; i0 += MAX_INST_PER_LAUNCH) {
    const int n = shape->n_inst - i0 < MAX_INST_PER_LAUNCH ? shape->n_inst - i0 : MAX_INST_PER_LAUNCH;
    InstTable tab;
    memset(&tab, 0, sizeof tab);
    fill_table(g.Hkv, g.L, budget, i0, n, row, &tab, &row);
    if (launch_select(n, i0, g.Hkv, g.L, g.keep, pool, pool_avg(shape), scores, tab, idx, st) != hipSuccess) return LAQ_ERR_DEVICE;
  }
  return LAQ_OK;
}

static int compact_impl(const laq_shape* shape, const void* k, const void* v, const int32_t* idx,
                        const int32_t* budget, void* k_out, void* v_out, hipStream_t st) {
  ScoreGeom g;
  const int rc = make_geom(shape, &g);
  if (rc != LAQ_OK) return rc;
  if (!k || !k_out || !idx || !budgets_ok(shape, g, budget)) return LAQ_ERR_INVALID;
  if ((v == nullptr) != (v_out == nullptr)) return LAQ_ERR_INVALID;
  KvLayout lay;
  if (make_layout(shape, g, &lay) != LAQ_OK) return LAQ_ERR_INVALID;
  const int row_bytes = g.d * (shape->dtype == LAQ_F32 ? 4 : 2);
  int64_t row = 0;
  for (int i0 = 0; i0 < shape->n_inst; i0 += MAX_INST_PER_LAUNCH) {
    const int n = shape->n_inst - i0 < MAX_INST_PER_LAUNCH ? shape->n_inst - i0 : MAX_INST_PER_LAUNCH;
    CompactTable tab;
    memset(&tab, 0, sizeof tab);
    fill_compact_table(g.Hkv, g.L, row_bytes >> 4, budget, i0, n, row, &tab, &row);
    if (launch_compact(n, i0, g.Hkv, g.L, row_bytes, lay, k, v, idx, tab, k_out, v_out, st) != hipSuccess)
      return LAQ_ERR_DEVICE;
  }
  return LAQ_OK;
}

static int sink_recent_impl(int n_inst, int Hkv, int L, const int32_t* budget, int n_sink, int32_t* idx,
                            hipStream_t st) {
  if (n_inst < 1 || Hkv < 1 || L < 1 || n_sink < 0 || !budget || !idx) return LAQ_ERR_INVALID;
  for (int i = 0; i < n_inst; ++i)
    if (budget[i] < 1) return LAQ_ERR_INVALID;
  if (Hkv > 65535) return LAQ_ERR_UNSUPPORTED;
  int64_t row = 0;
  for (int i0 = 0; i0 < n_inst; i0 += MAX_INST_PER_LAUNCH) {
    const int n = n_inst - i0 < MAX_INST_PER_LAUNCH ? n_inst - i0 : MAX_INST_PER_LAUNCH;
    InstTable tab;
    memset(&tab, 0, sizeof tab);
    fill_table(Hkv, L, budget, i0, n, row, &tab, &row);
    if (launch_sink_recent(n, Hkv, L, n_sink, tab, idx, st) != hipSuccess) return LAQ_ERR_DEVICE;
  }
  return LAQ_OK;
}

// Decode attention splits long caches over several workgroups when the call has few of them: a
// cache of more than DECODE_SPLIT_ROWS rows becomes parts of at most that many rows, whose partial
// results go through the workspace.  Without a workspace every cache is one part.
constexpr int DECODE_SPLIT_ROWS = 512;
constexpr int DECODE_SPLIT_BELOW_WORKGROUPS = 1024;

static int decode_parts_of(int bk, bool split) {
  if (!split) return 1;
  const int s = (bk + DECODE_SPLIT_ROWS - 1) / DECODE_SPLIT_ROWS;
  return s < MAX_PARTS_PER_LAUNCH ? s : MAX_PARTS_PER_LAUNCH;
}

static bool decode_would_split(const laq_shape* shape, const ScoreGeom& g, const int32_t* budget) {
  const int gb = decode_head_batch(g.Hq, g.Hkv), nbatch = (g.G + gb - 1) / gb;
  if ((long long)g.Hkv * nbatch * g.n_inst >= DECODE_SPLIT_BELOW_WORKGROUPS) return false;
  for (int i = 0; i < shape->n_inst; ++i)
    if ((budget[i] < g.L ? budget[i] : g.L) > DECODE_SPLIT_ROWS) return true;
  return false;
}

// bytes of partial results: one record of d + 2 floats per part, workgroup column and query-head slot,
// for at most one launch's parts (launches reuse the area; they are ordered on the stream)
static size_t decode_ws_bytes(const laq_shape* shape, const ScoreGeom& g, const int32_t* budget) {
  if (!decode_would_split(shape, g, budget)) return 0;
  long long parts = 0;
  for (int i = 0; i < shape->n_inst; ++i) parts += decode_parts_of(budget[i] < g.L ? budget[i] : g.L, true);
  if (parts > MAX_PARTS_PER_LAUNCH) parts = MAX_PARTS_PER_LAUNCH;
  const int gb = decode_head_batch(g.Hq, g.Hkv), nbatch = (g.G + gb - 1) / gb;
  return round256((size_t)parts * g.Hkv * nbatch * gb * (g.d + 2) * sizeof(float));
}

static int decode_impl(const laq_shape* shape, const void* q, const void* kc, const void* vc,
                       const int32_t* budget, float* out, void* ws, size_t ws_bytes, hipStream_t st) {
  ScoreGeom g;
  const int rc = make_geom(shape, &g);
  if (rc != LAQ_OK) return rc;
  if (!q || !kc || !vc || !out || !budget) return LAQ_ERR_INVALID;
  for (int i = 0; i < shape->n_inst; ++i)
    if (budget[i] < 1) return LAQ_ERR_INVALID;
  if (g.Hkv > 65535) return LAQ_ERR_UNSUPPORTED;
  const bool split = ws != nullptr && decode_would_split(shape, g, budget);
  if (split && ws_bytes < decode_ws_bytes(shape, g, budget)) return LAQ_ERR_WORKSPACE;
  float* partial = static_cast<float*>(ws);
  if (!split) {                                      // every cache is one part: tables of whole instances
    int64_t row = 0;
    for (int i0 = 0; i0 < shape->n_inst; i0 += MAX_INST_PER_LAUNCH) {
      const int n = shape->n_inst - i0 < MAX_INST_PER_LAUNCH ? shape->n_inst - i0 : MAX_INST_PER_LAUNCH;
      DecodeWhole whole;
      whole.inst0 = i0;
      for (int i = 0; i < n; ++i) {
        whole.bk[i] = budget[i0 + i] < g.L ? budget[i0 + i] : g.L;
        whole.row0[i] = row;
        row += (int64_t)g.Hkv * whole.bk[i];
      }
      if (launch_decode(n, g.Hq, g.Hkv, g.d, shape->dtype, g.scale2, whole, q, kc, vc, out, st) != hipSuccess)
        return LAQ_ERR_DEVICE;
    }
    return LAQ_OK;
  }

  DecodeParts tab;
  int n_parts = 0;
  bool any_split = false;
  auto flush = [&]() -> bool {
    if (n_parts == 0) return true;
    if (launch_decode(n_parts, g.Hq, g.Hkv, g.d, shape->dtype, g.scale2, tab, q, kc, vc, out, partial, st) !=
        hipSuccess)
      return false;
    if (any_split && launch_merge_parts(n_parts, g.Hq, g.Hkv, g.d, tab, partial, out, st) != hipSuccess) return false;
    n_parts = 0;
    any_split = false;
    return true;
  };
  int64_t row = 0;
  for (int i = 0; i < shape->n_inst; ++i) {
    const int bk = budget[i] < g.L ? budget[i] : g.L;
    const int S = decode_parts_of(bk, split);
    if (n_parts + S > MAX_PARTS_PER_LAUNCH && !flush()) return LAQ_ERR_DEVICE;   // the parts of a cache stay together
    const int per = (bk + S - 1) / S;
    for (int p = 0; p < S; ++p) {
      const int start = p * per;
      tab.row0[n_parts] = row;
      tab.bk[n_parts] = bk;
      tab.start[n_parts] = start < bk ? start : bk;
      tab.rows[n_parts] = start < bk ? (bk - start < per ? bk - start : per) : 0;
      tab.inst[n_parts] = i;
      tab.split[n_parts] = (int16_t)p;
      tab.nsplit[n_parts] = (int16_t)S;
      ++n_parts;
    }
    any_split = any_split || S > 1;
    row += (int64_t)g.Hkv * bk;
  }
  return flush() ? LAQ_OK : LAQ_ERR_DEVICE;
}

static int qcache_store_impl(const laq_shape* shape, const void* q_step, int t, void* q_cache, hipStream_t st) {
  ScoreGeom g;
  const int rc = make_geom(shape, &g);
  if (rc != LAQ_OK) return rc;
  if (!q_step || !q_cache || t < 0 || t >= g.W) return LAQ_ERR_INVALID;
  const int row_bytes = g.d * (shape->dtype == LAQ_F32 ? 4 : 2);
  return launch_qcache_store((long long)g.n_inst * g.Hq, g.W, t, row_bytes, q_step, q_cache, st) == hipSuccess
             ? LAQ_OK
             : LAQ_ERR_DEVICE;
}

static int recall_impl(int n_inst, int Hkv, int L, const int32_t* idx_pred, const int32_t* budget_pred,
                       const int32_t* idx_gold, const int32_t* budget_gold, int32_t* overlap, float* recall,
                       hipStream_t st) {
  if (n_inst < 1 || Hkv < 1 || L < 1 || !idx_pred || !budget_pred || !idx_gold || !budget_gold || !overlap)
    return LAQ_ERR_INVALID;
  for (int i = 0; i < n_inst; ++i)
    if (budget_pred[i] < 1 || budget_gold[i] < 1) return LAQ_ERR_INVALID;
  if (Hkv > 65535) return LAQ_ERR_UNSUPPORTED;
  int64_t row_a = 0, row_b = 0;
  for (int i0 = 0; i0 < n_inst; i0 += MAX_PAIR_PER_LAUNCH) {
    const int n = n_inst - i0 < MAX_PAIR_PER_LAUNCH ? n_inst - i0 : MAX_PAIR_PER_LAUNCH;
    PairTable tab;
    memset(&tab, 0, sizeof tab);
    for (int i = 0; i < n; ++i) {
      tab.bk_a[i] = budget_pred[i0 + i] < L ? budget_pred[i0 + i] : L;
      tab.bk_b[i] = budget_gold[i0 + i] < L ? budget_gold[i0 + i] : L;
      tab.row_a[i] = row_a;
      tab.row_b[i] = row_b;
      row_a += (int64_t)Hkv * tab.bk_a[i];
      row_b += (int64_t)Hkv * tab.bk_b[i];
    }
    if (launch_recall(n, i0, Hkv, tab, idx_pred, idx_gold, overlap, recall, st) != hipSuccess) return LAQ_ERR_DEVICE;
  }
  return LAQ_OK;
}

}  // namespace laq

extern "C" {

size_t laq_workspace_bytes(const laq_shape* shape) {
  laq::ScoreGeom g;
  if (laq::make_geom(shape, &g) != LAQ_OK) return 0;
  return laq::workspace_bytes(g);
}

int laq_score(const laq_shape* shape, const void* q_win, const void* k, int pool_kernel, float* scores,
              void* ws, size_t ws_bytes, void* stream) {
  return laq::score_impl(shape, q_win, k, pool_kernel, scores, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int laq_select(const laq_shape* shape, const float* scores, const int32_t* budget, int pool_kernel,
               int32_t* idx, void* stream) {
  return laq::select_impl(shape, scores, budget, pool_kernel, idx, static_cast<hipStream_t>(stream));
}

int laq_select_sink_recent(int32_t n_inst, int32_t Hkv, int32_t L, const int32_t* budget, int32_t n_sink,
                           int32_t* idx, void* stream) {
  return laq::sink_recent_impl(n_inst, Hkv, L, budget, n_sink, idx, static_cast<hipStream_t>(stream));
}

size_t laq_decode_workspace_bytes(const laq_shape* shape, const int32_t* budget) {
  laq::ScoreGeom g;
  if (laq::make_geom(shape, &g) != LAQ_OK || !budget) return 0;
  for (int i = 0; i < shape->n_inst; ++i)
    if (budget[i] < 1) return 0;
  return laq::decode_ws_bytes(shape, g, budget);
}

int laq_decode_attention(const laq_shape* shape, const void* q, const void* k_c, const void* v_c,
                         const int32_t* budget, float* out, void* ws, size_t ws_bytes, void* stream) {
  return laq::decode_impl(shape, q, k_c, v_c, budget, out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int laq_qcache_store(const laq_shape* shape, const void* q_step, int32_t t, void* q_cache, void* stream) {
  return laq::qcache_store_impl(shape, q_step, t, q_cache, static_cast<hipStream_t>(stream));
}

int laq_recall(int32_t n_inst, int32_t Hkv, int32_t L, const int32_t* idx_pred, const int32_t* budget_pred,
               const int32_t* idx_gold, const int32_t* budget_gold, int32_t* overlap, float* recall, void* stream) {
  return laq::recall_impl(n_inst, Hkv, L, idx_pred, budget_pred, idx_gold, budget_gold, overlap, recall,
                          static_cast<hipStream_t>(stream));
}

int laq_compact(const laq_shape* shape, const void* k, const void* v, const int32_t* idx,
                const int32_t* budget, void* k_out, void* v_out, void* stream) {
  return laq::compact_impl(shape, k, v, idx, budget, k_out, v_out, static_cast<hipStream_t>(stream));
}

static int evict_impl(const laq_shape* shape, const void* q_win, const void* k, const void* v, const int32_t* budget,
                      int pool_kernel, float* scores, int32_t* idx, void* k_out, void* v_out, void* ws,
                      size_t ws_bytes, bool use_static_scratch, hipStream_t st) {
  // validate everything first so that a rejected call has enqueued nothing
  laq::ScoreGeom g;
  const int rc0 = laq::make_geom(shape, &g);
  if (rc0 != LAQ_OK) return rc0;
  if (!laq::pool_ok(pool_kernel) || !q_win || !k || !idx || !k_out ||
      !laq::budgets_ok(shape, g, budget) || ((v == nullptr) != (v_out == nullptr)))
    return LAQ_ERR_INVALID;
  laq::KvLayout lay;
  if (laq::make_layout(shape, g, &lay) != LAQ_OK) return LAQ_ERR_INVALID;
  if (use_static_scratch) {
    if (laq::workspace_bytes(g) > (size_t)LAQ_STATIC_SCRATCH_BYTES) return LAQ_ERR_WORKSPACE;
    int dev = 0;
    const int rc_init = laq::init_current_device(&dev);
    if (rc_init != LAQ_OK) return rc_init;
    ws = laq::scratch_of[dev].load(std::memory_order_acquire);
    ws_bytes = (size_t)LAQ_STATIC_SCRATCH_BYTES;
  }
  if (!ws || ws_bytes < laq::workspace_bytes(g)) return LAQ_ERR_WORKSPACE;
  if (!scores) scores = laq::carve_workspace(g, ws).pooled;      // the hand-over plane between the stages
  int rc = laq::score_impl(shape, q_win, k, pool_kernel, scores, ws, ws_bytes, st);
  if (rc != LAQ_OK) return rc;
  rc = laq::select_impl(shape, scores, budget, 1, idx, st);
  if (rc != LAQ_OK) return rc;
  return laq::compact_impl(shape, k, v, idx, budget, k_out, v_out, st);
}

int laq_evict(const laq_shape* shape, const void* q_win, const void* k, const void* v, const int32_t* budget,
              int pool_kernel, float* scores, int32_t* idx, void* k_out, void* v_out, void* ws,
              size_t ws_bytes, void* stream) {
  return evict_impl(shape, q_win, k, v, budget, pool_kernel, scores, idx, k_out, v_out, ws, ws_bytes, false,
                    static_cast<hipStream_t>(stream));
}

int laq_evict_static(const laq_shape* shape, const void* q_win, const void* k, const void* v, const int32_t* budget,
                     int pool_kernel, float* scores, int32_t* idx, void* k_out, void* v_out, void* stream) {
  return evict_impl(shape, q_win, k, v, budget, pool_kernel, scores, idx, k_out, v_out, nullptr, 0, true,
                    static_cast<hipStream_t>(stream));
}

int laq_init(void) { return laq::init_current_device(nullptr); }

int laq_score_kernel(const laq_shape* shape) {
  laq::ScoreGeom g;
  laq::QueryPos qp;
  memset(&qp, 0, sizeof qp);
  const int rc = laq::make_geom(shape, &g, &qp);
  if (rc != LAQ_OK) return rc;
  laq::KvLayout lay;
  if (laq::make_layout(shape, g, &lay) != LAQ_OK) return LAQ_ERR_INVALID;
  if (!laq::score_mfma_supported(g, lay, shape->dtype)) return LAQ_KERNEL_VECTOR;
  bool single = false;
  if (laq::SINGLE_READ_ENABLED && laq::single_read_wanted(shape, g) &&
      laq::score_fused_applies(g, lay, shape->dtype, &single) != hipSuccess)
    return LAQ_ERR_DEVICE;
  return single ? LAQ_KERNEL_SINGLE_READ : LAQ_KERNEL_TWO_PASS;
}

int laq_workspace_status(const laq_shape* shape, const void* ws, size_t ws_bytes, void* stream) {
  laq::ScoreGeom g;
  const int rc0 = laq::make_geom(shape, &g);
  if (rc0 != LAQ_OK) return rc0;
  if (!ws || ws_bytes < laq::workspace_bytes(g)) return LAQ_ERR_WORKSPACE;
  const laq::Workspace w = laq::carve_workspace(g, const_cast<void*>(ws));
  hipStream_t st = static_cast<hipStream_t>(stream);
  int word = 0;
  if (hipMemcpyAsync(&word, w.status, sizeof word, hipMemcpyDeviceToHost, st) != hipSuccess) return LAQ_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return LAQ_ERR_DEVICE;
  return word == 0 ? LAQ_OK : LAQ_ERR_TIMEOUT;
}

const char* laq_strerror(int code) {
  switch (code) {
    case LAQ_OK: return "ok";
    case LAQ_ERR_INVALID: return "invalid argument";
    case LAQ_ERR_UNSUPPORTED: return "unsupported shape";
    case LAQ_ERR_WORKSPACE: return "workspace missing or too small";
    case LAQ_ERR_DEVICE: return "HIP launch failed";
    case LAQ_ERR_TIMEOUT: return "a kernel gave up waiting for its peers; results are not valid";
    default: return "unknown error";
  }
}

}  // extern "C"
