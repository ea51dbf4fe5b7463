// Recall of an eviction decision (Sec. 3.3): Recall_W = |M_gold ∩ M_pred| / |M_gold|, per
// (layer, sequence, KV head), for two retained-index sets as dapq_topk writes them (ascending,
// distinct positions).
//
// One workgroup per head: every thread takes gold positions in turn and looks each up in the
// predicted list by binary search; the hits are summed over the workgroup.
#include "dapq_internal.h"

namespace dapq {
namespace {

constexpr int kRecallThreads = 256;

struct RecallParams {
  const int32_t* idx_gold;
  const int32_t* count_gold;
  const int32_t* idx_pred;
  const int32_t* count_pred;
  int32_t* common;
  float* recall;
  int32_t budget_gold, budget_pred;
};

__global__ __launch_bounds__(kRecallThreads) void recall_kernel(RecallParams p) {
  __shared__ int wave_hits[kRecallThreads / 64];
  const int64_t head = blockIdx.x;
  const int tid = threadIdx.x;
  int ng = p.count_gold[head], np = p.count_pred[head];
  ng = ng < 0 ? 0 : (ng > p.budget_gold ? p.budget_gold : ng);
  np = np < 0 ? 0 : (np > p.budget_pred ? p.budget_pred : np);
  const int32_t* gold = p.idx_gold + head * p.budget_gold;
  const int32_t* pred = p.idx_pred + head * p.budget_pred;
  int hits = 0;
  for (int i = tid; i < ng; i += kRecallThreads) {
    const int32_t v = gold[i];
    int lo = 0, hi = np;  // first position of pred with pred[pos] >= v
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (pred[mid] < v) lo = mid + 1; else hi = mid;
    }
    hits += (lo < np && pred[lo] == v) ? 1 : 0;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) hits += __shfl_xor(hits, d, 64);
  if ((tid & 63) == 0) wave_hits[tid >> 6] = hits;
  __syncthreads();
  if (tid == 0) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < kRecallThreads / 64; ++w) total += wave_hits[w];
    p.common[head] = total;
    if (p.recall != nullptr) p.recall[head] = ng > 0 ? (float)total / (float)ng : 0.0f;
  }
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_recall(const dapq_shape* shape, const int32_t* idx_gold, const int32_t* count_gold,
                                    int32_t budget_gold, const int32_t* idx_pred, const int32_t* count_pred,
                                    int32_t budget_pred, int32_t* common, float* recall, void* stream) {
  int rc = check_shape(shape, false, false, false);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(idx_gold != nullptr && count_gold != nullptr && idx_pred != nullptr && count_pred != nullptr &&
                   common != nullptr,
               DAPQ_ERR_INVALID_ARG, "idx_gold, count_gold, idx_pred, count_pred and common must not be NULL");
  DAPQ_REQUIRE(budget_gold >= 1 && budget_pred >= 1, DAPQ_ERR_INVALID_ARG, "budgets (%d, %d) must be >= 1",
               budget_gold, budget_pred);
  const int64_t heads = (int64_t)shape->n_layers * shape->batch * shape->n_kv_heads;
  DAPQ_REQUIRE(heads < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED, "too many heads");
  RecallParams p;
  p.idx_gold = idx_gold;
  p.count_gold = count_gold;
  p.idx_pred = idx_pred;
  p.count_pred = count_pred;
  p.common = common;
  p.recall = recall;
  p.budget_gold = budget_gold;
  p.budget_pred = budget_pred;
  hipLaunchKernelGGL(recall_kernel, dim3((unsigned)heads), dim3(kRecallThreads), 0, static_cast<hipStream_t>(stream), p);
  DAPQ_HIP_LAUNCH_CHECK("recall_kernel");
  return DAPQ_OK;
}
