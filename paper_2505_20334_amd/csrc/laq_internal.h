// Internal declarations shared by the HIP translation units of the LAQ library.
// Not part of the public boundary (that is include/laq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "laq.h"

namespace laq {

// Each scoring workgroup stages CHUNK_ROWS consecutive key rows of one KV head; a head is
// covered by nchunk = ceil(L / CHUNK_ROWS) chunks.
constexpr int CHUNK_ROWS = 256;
// The matrix-core path stages MFMA_ROWS key rows per workgroup (its own, finer chunking of the
// same per-chunk statistics); the workspace is sized for the finer of the two.
#ifndef LAQ_MFMA_ROWS
#define LAQ_MFMA_ROWS 256
#endif
constexpr int MFMA_ROWS = LAQ_MFMA_ROWS;
constexpr int MIN_CHUNK_ROWS = MFMA_ROWS < CHUNK_ROWS ? MFMA_ROWS : CHUNK_ROWS;
constexpr int MAX_POOL = 63;
constexpr int MAX_INST_PER_LAUNCH = 256;   // size of the per-instance tables passed as kernel arguments

constexpr int MAX_QPOS = 512;              // explicit query positions a call may carry
// The single-read scoring kernel: key rows per workgroup, and the number of its workgroups on the
// device at once that the exchange memory of a workspace is sized for.
constexpr int FUSED_ROWS = 512;
constexpr int FUSED_MAX_RESIDENT = 1024;
// Whether scoring takes the single-read kernel where it applies (it is slower than the two streaming
// passes on the shapes measured so far; the parity tests run with it switched on).
constexpr bool SINGLE_READ_ENABLED = true;

struct ScoreGeom {
  int n_inst, Hq, Hkv, d, L, W;
  int G, R;
  int keep;      // trailing keys always retained
  int P;         // L - keep: the prefix that is ranked and pooled
  int Rpad;      // R rounded up to a multiple of 32
  int nchunk;    // ceil(L / CHUNK_ROWS)
  int pos0;      // trailing-window layout: query w sees keys j <= pos0 + w (pos0 = L - W)
  int explicit_pos;   // 1: positions come from the QueryPos table instead
  int qmin;      // smallest last-visible key over the W queries: keys up to here need no mask
  float scale2;  // scale * log2(e): logits are kept in base-2 units
};

// Last key each window query sees (already clamped to L-1); passed by value to the kernels.
// Filled for every call with W <= MAX_QPOS (also with the trailing-window positions), so that the
// matrix-core kernels only ever look positions up; longer trailing windows take the generic path,
// which computes them.
struct QueryPos {
  int32_t last[MAX_QPOS];
};
__device__ __forceinline__ int last_visible_key(const ScoreGeom& g, const QueryPos& qp, int w) {
  return g.explicit_pos ? qp.last[w] : g.pos0 + w;
}

// Workspace carving: [partials | row constants | raw scores]
//   part:  float2 (m, z) per (instance, KV head, chunk, padded row): softmax statistics of a chunk
//   rowc:  float c = M + log2(Z) per (instance, KV head, padded row)
//   raw:   float per (instance, KV head, key): unpooled scores in front of a separate pooling
//          kernel (generic path, average pool); the MFMA path with the max pool keeps the edge
//          records of its chunk boundaries here instead
//   pooled: float per (instance, KV head, key): the hand-over plane between scoring and selection
//          when laq_evict is called without a scores buffer
//   ctr:   two work counters (one per streaming pass of the MFMA path), reset by every call
struct Workspace {
  float2* part;
  float* rowc;
  float* raw;
  float* pooled;
  void* fused;      // exchange memory of the single-read kernel (fused_sync_bytes)
  int* ctr;
  int* status;      // != 0 after a call whose single-read kernel gave up a wait (results invalid)
};

size_t workspace_bytes(const ScoreGeom& g);
Workspace carve_workspace(const ScoreGeom& g, void* ws);

// Per-instance output table for select / compact (passed by value as a kernel argument).
struct InstTable {
  int32_t bk[MAX_INST_PER_LAUNCH];      // rows kept per KV head
  int64_t row0[MAX_INST_PER_LAUNCH];    // first packed output row (sum of Hkv * Bk of earlier instances)
};
// The gather's own table: its grid covers exactly the rows of every instance, so a workgroup finds
// its instance by the first workgroup of each (blk0 ascending, blk0[n] = all workgroups).
struct CompactTable {
  int32_t bk[MAX_INST_PER_LAUNCH];
  int64_t row0[MAX_INST_PER_LAUNCH];
  int32_t blk0[MAX_INST_PER_LAUNCH + 1];
};

// Pooled score at prefix position pos, the one arithmetic every pooling site uses: the
// maximum over the part of the window inside [0, P), or (avg) the fp32 sum over it in
// ascending position divided by the kernel size 2*half+1 (zeros outside the prefix).
__device__ __forceinline__ float pool_window(const float* __restrict__ s, int pos, int P, int half, bool avg) {
  if (half == 0) return s[pos];
  const int lo = max(pos - half, 0), hi = min(pos + half, P - 1);
  if (avg) {
    float acc = 0.f;
    for (int i = lo; i <= hi; ++i) acc += s[i];
    return acc / (float)(2 * half + 1);
  }
  float v = s[pos];
  for (int i = lo; i <= hi; ++i) v = fmaxf(v, s[i]);
  return v;
}

// Where the rows of k and v lie: element strides between instances and KV heads, and between
// consecutive key rows (row_bytes is the latter in bytes).  dense = [n_inst, Hkv, L, d].
struct KvLayout {
  int64_t inst, head, row;
  int32_t row_bytes;
  int32_t dense;
  // paged cache (table != nullptr): key row j of instance i is row j % block_rows of block
  // table[i * blocks_per_inst + j / block_rows]; blocks lie `block` elements apart, head / row are
  // the strides inside a block, inst is not used
  const int32_t* table;
  int32_t blocks_per_inst;
  int32_t block_rows;
  int64_t block;
};

#ifdef __HIPCC__
// Paged caches: element offset, from the pool's start, of the block that holds key row j of an
// instance, and the row's number inside that block.
__device__ __forceinline__ int64_t paged_block_offset(const KvLayout& lay, int inst, int j, int* row_in_block) {
  const int b = j / lay.block_rows;
  *row_in_block = j - b * lay.block_rows;
  return (int64_t)lay.table[(size_t)inst * lay.blocks_per_inst + b] * lay.block;
}
#endif

// Two packed index lists side by side, for up to MAX_PAIR_PER_LAUNCH instances.
constexpr int MAX_PAIR_PER_LAUNCH = 128;
struct PairTable {
  int32_t bk_a[MAX_PAIR_PER_LAUNCH], bk_b[MAX_PAIR_PER_LAUNCH];       // row lengths
  int64_t row_a[MAX_PAIR_PER_LAUNCH], row_b[MAX_PAIR_PER_LAUNCH];     // first packed row of the instance
};

// Parts of compacted caches for decode attention, up to MAX_PARTS_PER_LAUNCH per launch: a cache
// is one part, or several consecutive ones that are merged afterwards.
constexpr int MAX_PARTS_PER_LAUNCH = 128;
struct DecodeParts {
  int64_t row0[MAX_PARTS_PER_LAUNCH];   // first packed row of the instance
  int32_t bk[MAX_PARTS_PER_LAUNCH];     // rows per KV head of the instance
  int32_t start[MAX_PARTS_PER_LAUNCH];  // first row of the part within a head's rows
  int32_t rows[MAX_PARTS_PER_LAUNCH];   // rows of the part
  int32_t inst[MAX_PARTS_PER_LAUNCH];   // instance
  int16_t split[MAX_PARTS_PER_LAUNCH];  // index of the part within its cache
  int16_t nsplit[MAX_PARTS_PER_LAUNCH]; // parts of its cache
  __host__ __device__ int inst_of(int i) const { return inst[i]; }
  __host__ __device__ int64_t base_row(int i) const { return row0[i]; }
  __host__ __device__ int cache_rows(int i) const { return bk[i]; }
  __host__ __device__ int first_row(int i) const { return start[i]; }
  __host__ __device__ int part_rows(int i) const { return rows[i]; }
  __host__ __device__ int parts(int i) const { return nsplit[i]; }
};
// The same view of a launch in which every cache is one part: instances inst0 .. of a call.
struct DecodeWhole {
  int64_t row0[MAX_INST_PER_LAUNCH];
  int32_t bk[MAX_INST_PER_LAUNCH];
  int32_t inst0;
  __host__ __device__ int inst_of(int i) const { return inst0 + i; }
  __host__ __device__ int64_t base_row(int i) const { return row0[i]; }
  __host__ __device__ int cache_rows(int i) const { return bk[i]; }
  __host__ __device__ int first_row(int) const { return 0; }
  __host__ __device__ int part_rows(int i) const { return bk[i]; }
  __host__ __device__ int parts(int) const { return 1; }
};

// launchers (each returns hipGetLastError() after its last launch); `raw` receives unpooled scores
hipError_t launch_score_generic(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int dtype, const void* q,
                                const void* k, float* raw, const Workspace& ws, hipStream_t st);
hipError_t launch_row_constants(const ScoreGeom& g, const Workspace& ws, hipStream_t st);
bool score_mfma_supported(const ScoreGeom& g, const KvLayout& lay, int dtype);
// kernel attributes and residency of every matrix-core scoring kernel on device `dev`, which must be
// the current device; idempotent
hipError_t score_mfma_init(int dev);
hipError_t score_fused_init(int dev);
size_t fused_sync_bytes(const ScoreGeom& g);
bool score_fused_supported(const ScoreGeom& g, const KvLayout& lay, int dtype);
hipError_t score_fused_applies(const ScoreGeom& g, const KvLayout& lay, int dtype, bool* yes);
// single-read scoring (K streamed once); *done = false: not launched, take the two-pass kernels
hipError_t launch_score_fused(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const void* q,
                              const void* k, float* scores, const Workspace& ws, hipStream_t st, bool* done);
// pooled scores of the prefix keys within `half` of a boundary between two chunks of chunk_rows keys,
// from the chunks' edge records
hipError_t launch_pool_boundaries(const ScoreGeom& g, int half, int nchunk, int chunk_rows, const float* edge,
                                  float* scores, hipStream_t st);
hipError_t launch_score_mfma(const ScoreGeom& g, const QueryPos& qp, const KvLayout& lay, int pool, const void* q,
                             const void* k, float* scores, const Workspace& ws, hipStream_t st);
hipError_t launch_pool(const ScoreGeom& g, int pool, bool avg, const float* raw, float* pooled, hipStream_t st);
hipError_t launch_select(int n_inst, int inst0, int Hkv, int L, int keep, int pool, bool avg, const float* scores,
                         const InstTable& tab, int32_t* idx, hipStream_t st);
hipError_t launch_sink_recent(int n_inst, int Hkv, int L, int n_sink, const InstTable& tab, int32_t* idx,
                              hipStream_t st);
hipError_t launch_recall(int n_inst, int inst0, int Hkv, const PairTable& tab, const int32_t* idx_pred,
                         const int32_t* idx_gold, int32_t* overlap, float* recall, hipStream_t st);
int decode_head_batch(int Hq, int Hkv);   // query heads of a KV head that one decode workgroup serves
hipError_t launch_decode(int n_parts, int Hq, int Hkv, int d, int dtype, float scale2, const DecodeParts& tab,
                         const void* q, const void* kc, const void* vc, float* out, float* partial, hipStream_t st);
hipError_t launch_decode(int n_inst, int Hq, int Hkv, int d, int dtype, float scale2, const DecodeWhole& tab,
                         const void* q, const void* kc, const void* vc, float* out, hipStream_t st);
hipError_t launch_merge_parts(int n_parts, int Hq, int Hkv, int d, const DecodeParts& tab, const float* partial,
                              float* out, hipStream_t st);
hipError_t launch_qcache_store(long long rows, int W, int t, int row_bytes, const void* q_step, void* q_cache,
                               hipStream_t st);
constexpr int COMPACT_THREADS = 256;      // one 16-byte piece of an output row per thread
hipError_t launch_compact(int n_inst, int inst0, int Hkv, int L, int row_bytes, const KvLayout& lay,
                          const void* k, const void* v, const int32_t* idx, const CompactTable& tab, void* k_out,
                          void* v_out, hipStream_t st);

}  // namespace laq
