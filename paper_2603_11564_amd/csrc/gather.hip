// Cache pruning (Sec. 4.2): only the key-value pairs in M_retain are kept; the pseudo segment is
// discarded.  Copies the retained K and V rows, bit for bit, into the compact cache
// [layer][sequence][KV head][slot][d].
//
// Pure copy: 16 lanes move one 256-byte row with one 16-byte load and store each, so every row is
// read and written in full cache lines; a workgroup of 256 threads moves 64 rows of K or of V, four
// per 16-lane group, with the four loads in flight together.
#include "dapq_internal.h"

namespace dapq {
namespace {

struct GatherParams {
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* idx;
  const int32_t* count;
  const int32_t* cu_seqlens;
  uint16_t* k_out;
  uint16_t* v_out;
  int64_t k_stride_layer, k_stride_seq, k_stride_head, k_stride_token;
  int64_t v_stride_layer, v_stride_seq, v_stride_head, v_stride_token;
  int64_t total_tokens;
  int32_t batch, n_kv_heads, budget;
};

constexpr int kGatherRowsPerGroup = 4;  // rows in flight per 16-lane group
constexpr int kGatherRowsPerBlock = 16 * kGatherRowsPerGroup;

__global__ __launch_bounds__(256) void gather_kernel(GatherParams p) {
  const int ch = threadIdx.x & 15;
  const int slot0 = blockIdx.x * kGatherRowsPerBlock + (threadIdx.x >> 4);  // this group's slots: slot0 + 16*r
  const int64_t head = blockIdx.y;  // (layer * batch + seq) * Hkv + kv
  const bool is_v = blockIdx.z == 1;
  const int n = p.count[head];
  if (slot0 >= n) return;
  const int kv = (int)(head % p.n_kv_heads);
  const int seq = (int)((head / p.n_kv_heads) % p.batch);
  const int layer = (int)(head / ((int64_t)p.n_kv_heads * p.batch));
  int64_t start;
  int L;
  if (p.cu_seqlens == nullptr) {
    L = (int)(p.total_tokens / p.batch);
    start = (int64_t)seq * L;
  } else {
    start = p.cu_seqlens[seq];
    L = p.cu_seqlens[seq + 1] - (int)start;
  }
  const uint16_t* base = is_v ? p.v + layer * p.v_stride_layer + seq * p.v_stride_seq + kv * p.v_stride_head
                              : p.k + layer * p.k_stride_layer + seq * p.k_stride_seq + kv * p.k_stride_head;
  const int64_t stride_token = is_v ? p.v_stride_token : p.k_stride_token;
  uint16_t* dst = (is_v ? p.v_out : p.k_out) + head * p.budget * kHeadDim;
  // all index loads first, then all row loads, then the stores: four rows in flight per group
  int j[kGatherRowsPerGroup];
#pragma unroll
  for (int r = 0; r < kGatherRowsPerGroup; ++r) {
    const int slot = slot0 + 16 * r;
    j[r] = slot < n ? p.idx[head * p.budget + slot] : -1;
  }
  uint4 row[kGatherRowsPerGroup];
#pragma unroll
  for (int r = 0; r < kGatherRowsPerGroup; ++r) {
    const bool ok = j[r] >= 0 && j[r] < L;  // never follow an index outside the sequence
    row[r] = ok ? reinterpret_cast<const uint4*>(base + (start + j[r]) * stride_token)[ch] : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int r = 0; r < kGatherRowsPerGroup; ++r) {
    const int slot = slot0 + 16 * r;
    if (j[r] >= 0 && j[r] < L) reinterpret_cast<uint4*>(dst + (int64_t)slot * kHeadDim)[ch] = row[r];
  }
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_gather(const dapq_shape* shape, const void* k, const void* v, const int32_t* idx,
                           const int32_t* count, int32_t budget, void* k_out, void* v_out, void* stream) {
  int rc = check_shape(shape, false, true, true);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(k != nullptr && v != nullptr && idx != nullptr && count != nullptr && k_out != nullptr &&
                   v_out != nullptr,
               DAPQ_ERR_INVALID_ARG, "k, v, idx, count, k_out and v_out must not be NULL");
  DAPQ_REQUIRE(budget >= 1, DAPQ_ERR_INVALID_ARG, "budget (%d) must be >= 1", budget);
  DAPQ_REQUIRE(((reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(k_out) |
                 reinterpret_cast<uintptr_t>(v_out)) & 15) == 0,
               DAPQ_ERR_UNSUPPORTED, "k, v, k_out and v_out must be 16-byte aligned");
  const int64_t heads = (int64_t)shape->n_layers * shape->batch * shape->n_kv_heads;
  DAPQ_REQUIRE(heads <= 65535, DAPQ_ERR_UNSUPPORTED, "n_layers * batch * n_kv_heads (%lld) exceeds 65535",
               (long long)heads);
  GatherParams p;
  p.k = static_cast<const uint16_t*>(k);
  p.v = static_cast<const uint16_t*>(v);
  p.idx = idx;
  p.count = count;
  p.cu_seqlens = shape->cu_seqlens;
  p.k_out = static_cast<uint16_t*>(k_out);
  p.v_out = static_cast<uint16_t*>(v_out);
  p.k_stride_layer = shape->k_stride_layer; p.k_stride_seq = shape->k_stride_seq;
  p.k_stride_head = shape->k_stride_head; p.k_stride_token = shape->k_stride_token;
  p.v_stride_layer = shape->v_stride_layer; p.v_stride_seq = shape->v_stride_seq;
  p.v_stride_head = shape->v_stride_head; p.v_stride_token = shape->v_stride_token;
  p.total_tokens = shape->total_tokens;
  p.batch = shape->batch;
  p.n_kv_heads = shape->n_kv_heads;
  p.budget = budget;
  hipLaunchKernelGGL(gather_kernel, dim3((unsigned)((budget + kGatherRowsPerBlock - 1) / kGatherRowsPerBlock), (unsigned)heads, 2), dim3(256), 0,
                     static_cast<hipStream_t>(stream), p);
  DAPQ_HIP_LAUNCH_CHECK("gather_kernel");
  return DAPQ_OK;
}
