// Cache compaction: gather the retained key / value rows into the compacted cache the
// decoder continues on (Sec. 4.3, the re-eviction that follows the ranking of Eq. 4).
// Pure data movement: each 16-byte piece of an output row is copied by one lane, so a
// 256-byte bf16 row (d = 128) is one coalesced 16-lane read and one coalesced write.  The source
// rows are addressed through byte strides (instance, head, row); the output is packed.
#include "laq_internal.h"

namespace laq {

namespace {

constexpr int CP_THREADS = 256;

__global__ __launch_bounds__(CP_THREADS) void compact_kernel(int Hkv, int L, int row_bytes, size_t inst_bytes,
                                                             size_t head_bytes, size_t src_row_bytes, InstTable tab,
                                                             int inst0, const char* __restrict__ k,
                                                             const char* __restrict__ v,
                                                             const int32_t* __restrict__ idx,
                                                             char* __restrict__ k_out, char* __restrict__ v_out) {
  const int li = blockIdx.y;
  const int bk = tab.bk[li];
  const int ppr = row_bytes >> 4;                              // 16-byte pieces per row
  const int64_t piece = (int64_t)blockIdx.x * CP_THREADS + threadIdx.x;
  const int64_t row = piece / ppr;
  const int col = (int)(piece - row * ppr);
  if (row >= (int64_t)Hkv * bk) return;
  const int head = (int)(row / bk);
  const int64_t orow = tab.row0[li] + row;
  const int j = idx[orow];
  if (j < 0 || j >= L) return;
  const char* src = (blockIdx.z == 0) ? k : v;
  char* dst = (blockIdx.z == 0) ? k_out : v_out;
  const size_t so = (size_t)(inst0 + li) * inst_bytes + (size_t)head * head_bytes + (size_t)j * src_row_bytes +
                    (size_t)col * 16;
  const size_t dof = (size_t)orow * row_bytes + (size_t)col * 16;
  *reinterpret_cast<uint4*>(dst + dof) = *reinterpret_cast<const uint4*>(src + so);
}

}  // namespace

hipError_t launch_compact(int n_inst, int inst0, int Hkv, int L, int row_bytes, const KvLayout& lay, int bk_max,
                          const void* k, const void* v, const int32_t* idx, const InstTable& tab, void* k_out,
                          void* v_out, hipStream_t st) {
  const int64_t pieces = (int64_t)Hkv * bk_max * (row_bytes >> 4);
  if (pieces == 0) return hipSuccess;
  dim3 grid((unsigned)((pieces + CP_THREADS - 1) / CP_THREADS), n_inst, v ? 2 : 1);
  const size_t eb = (size_t)lay.row_bytes / (size_t)lay.row;        // element size of the source rows
  hipLaunchKernelGGL(compact_kernel, grid, dim3(CP_THREADS), 0, st, Hkv, L, row_bytes, (size_t)lay.inst * eb,
                     (size_t)lay.head * eb, (size_t)lay.row_bytes, tab, inst0,
                     static_cast<const char*>(k), static_cast<const char*>(v), idx, static_cast<char*>(k_out),
                     static_cast<char*>(v_out));
  return hipGetLastError();
}

}  // namespace laq
