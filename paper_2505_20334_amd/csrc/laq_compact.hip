// Cache compaction: gather the retained key / value rows into the compacted cache the
// decoder continues on (Sec. 4.3, the re-eviction that follows the ranking of Eq. 4).
// Pure data movement: each 16-byte piece of an output row is copied by one lane, so a
// 256-byte bf16 row (d = 128) is one coalesced 16-lane read and one coalesced write.  The source
// rows are addressed through byte strides (instance, head, row), or through the block table of a
// paged cache; the output is packed.
#include "laq_internal.h"

namespace laq {

namespace {

constexpr int CP_THREADS = COMPACT_THREADS;

__global__ __launch_bounds__(CP_THREADS) void compact_kernel(int n_inst, int Hkv, int L, int row_bytes, size_t inst_bytes,
                                                             size_t head_bytes, size_t src_row_bytes, KvLayout lay,
                                                             CompactTable tab,
                                                             int inst0, const char* __restrict__ k,
                                                             const char* __restrict__ v,
                                                             const int32_t* __restrict__ idx,
                                                             char* __restrict__ k_out, char* __restrict__ v_out) {
  // the instance of this workgroup: the last one whose first workgroup is not beyond it (uniform
  // bisection over the table in the kernel arguments)
  int lo = 0, hi = n_inst;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tab.blk0[mid] <= (int)blockIdx.x) lo = mid; else hi = mid;
  }
  const int li = lo;
  const int bk = tab.bk[li];
  const int ppr = row_bytes >> 4;                              // 16-byte pieces per row
  const int64_t piece = (int64_t)((int)blockIdx.x - tab.blk0[li]) * CP_THREADS + threadIdx.x;
  const int64_t row = piece / ppr;
  const int col = (int)(piece - row * ppr);
  if (row >= (int64_t)Hkv * bk) return;
  const int head = (int)(row / bk);
  const int64_t orow = tab.row0[li] + row;
  const int j = idx[orow];
  if (j < 0 || j >= L) return;
  const char* src = (blockIdx.y == 0) ? k : v;
  char* dst = (blockIdx.y == 0) ? k_out : v_out;
  size_t so = (size_t)(inst0 + li) * inst_bytes + (size_t)j * src_row_bytes;
  if (lay.table) {                       // paged cache: the row's block, and its row in there
    int r;
    const size_t eb = src_row_bytes / (size_t)lay.row;
    so = (size_t)paged_block_offset(lay, inst0 + li, j, &r) * eb;
    so += (size_t)r * src_row_bytes;
  }
  so += (size_t)head * head_bytes + (size_t)col * 16;
  const size_t dof = (size_t)orow * row_bytes + (size_t)col * 16;
  *reinterpret_cast<uint4*>(dst + dof) = *reinterpret_cast<const uint4*>(src + so);
}

}  // namespace

hipError_t launch_compact(int n_inst, int inst0, int Hkv, int L, int row_bytes, const KvLayout& lay,
                          const void* k, const void* v, const int32_t* idx, const CompactTable& tab, void* k_out,
                          void* v_out, hipStream_t st) {
  if (tab.blk0[n_inst] == 0) return hipSuccess;
  dim3 grid((unsigned)tab.blk0[n_inst], v ? 2 : 1);
  const size_t eb = (size_t)lay.row_bytes / (size_t)lay.row;        // element size of the source rows
  hipLaunchKernelGGL(compact_kernel, grid, dim3(CP_THREADS), 0, st, n_inst, Hkv, L, row_bytes, (size_t)lay.inst * eb,
                     (size_t)lay.head * eb, (size_t)lay.row_bytes, lay, tab, inst0,
                     static_cast<const char*>(k), static_cast<const char*>(v), idx, static_cast<char*>(k_out),
                     static_cast<char*>(v_out));
  return hipGetLastError();
}

}  // namespace laq
