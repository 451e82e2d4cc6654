// Recall of one selection against another (Sec. 3, Eq. 1-3): per (instance, KV head) the size of
// the intersection of two ascending position lists, and its ratio to the reference list's length.
#include "laq_internal.h"

namespace laq {

namespace {

// One workgroup per (KV head, instance).  A thread takes every 256th entry of the first list and
// looks it up in the second by bisection; integer counts are reduced across lanes and waves.  A
// second list of up to RECALL_STAGED entries is copied to LDS first, so that the dependent reads
// of the bisection are LDS reads (a dozen round trips to memory otherwise).
constexpr int RECALL_STAGED = 8192;
__global__ __launch_bounds__(256) void recall_kernel(int Hkv, PairTable tab, int inst0,
                                                     const int32_t* __restrict__ idx_pred,
                                                     const int32_t* __restrict__ idx_gold,
                                                     int32_t* __restrict__ overlap, float* __restrict__ recall) {
  __shared__ int wave_count[4];
  __shared__ int32_t staged[RECALL_STAGED];
  const int head = blockIdx.x, li = blockIdx.y, tid = threadIdx.x;
  const int n_pred = tab.bk_a[li], n_gold = tab.bk_b[li];
  const int32_t* pred = idx_pred + (tab.row_a[li] + (int64_t)head * n_pred);
  const int32_t* gold = idx_gold + (tab.row_b[li] + (int64_t)head * n_gold);
  const bool in_lds = n_gold <= RECALL_STAGED;      // the same for every thread of the workgroup
  if (in_lds) {
    for (int t = tid; t < n_gold; t += 256) staged[t] = gold[t];
    __syncthreads();
  }
  auto gold_at = [&](int i) { return in_lds ? staged[i] : gold[i]; };
  int count = 0;
  for (int t = tid; t < n_pred; t += 256) {
    const int32_t want = pred[t];
    int lo = 0, hi = n_gold;              // first entry of gold that is >= want lies in [lo, hi]
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (gold_at(mid) < want) lo = mid + 1; else hi = mid;
    }
    count += (lo < n_gold && gold_at(lo) == want) ? 1 : 0;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) count += __shfl_xor(count, o);
  if ((tid & 63) == 0) wave_count[tid >> 6] = count;
  __syncthreads();
  if (tid == 0) {
    const int total = wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
    const size_t out = (size_t)(inst0 + li) * Hkv + head;
    overlap[out] = total;
    if (recall) recall[out] = (float)total / (float)n_gold;
  }
}

}  // namespace

hipError_t launch_recall(int n_inst, int inst0, int Hkv, const PairTable& tab, const int32_t* idx_pred,
                         const int32_t* idx_gold, int32_t* overlap, float* recall, hipStream_t st) {
  hipLaunchKernelGGL(recall_kernel, dim3(Hkv, n_inst), dim3(256), 0, st, Hkv, tab, inst0, idx_pred, idx_gold, overlap,
                     recall);
  return hipGetLastError();
}

}  // namespace laq
