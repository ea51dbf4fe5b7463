// M_retain = TopK_j S(j) (Sec. 4.2): per (layer, sequence, KV head) the budget positions with the
// largest pooled score, equal scores lowest position first, written in ascending position.
//
// One workgroup of 1024 threads per head.  The scores of the head are staged in LDS when they fit
// (up to 36864 keys = 144 KB of the 160 KB LDS), so HBM is read once; longer heads are re-read from
// L2.  Selection is an exact radix select on the order-preserving integer image of the fp32 score:
// four 8-bit digits from the top, each pass a 256-bin LDS histogram followed by a suffix scan that
// fixes one digit of the threshold T and the number of keys equal to T still needed.  The last step
// is an ordered compaction: key j is kept if score > T, or score == T and fewer than `need` equal
// keys precede it; one packed (greater, equal) prefix count per block of 1024 keys gives both the
// decision and the output slot, so the result is ascending and deterministic (no atomics decide
// an order).  Max-pooling makes runs of bit-equal scores, so the tie rule is on the main path.
#include "dapq_internal.h"

namespace dapq {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kTopkLdsKeys = 36864;

struct TopkParams {
  const float* pooled;
  const int32_t* cu_seqlens;
  const int32_t* budget_per_seq;
  int32_t* idx;
  int32_t* count;
  int64_t total_tokens;
  int32_t batch, n_kv_heads, budget;
};

// fp32 -> uint32 with the same order for all non-NaN values.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(TopkParams p) {
  extern __shared__ uint32_t smem[];
  uint32_t* hist = smem;             // [256]
  uint32_t* wave_tot = smem + 256;   // [16]
  uint32_t* bcast = smem + 256 + 16; // [4]: digit, need, running (greater, equal) base
  uint32_t* keys = smem + 320;       // [kTopkLdsKeys] staged order keys (if they fit)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kv = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
  int64_t start;
  int L;
  if (p.cu_seqlens == nullptr) {
    L = (int)(p.total_tokens / p.batch);
    start = (int64_t)b * L;
  } else {
    start = p.cu_seqlens[b];
    L = p.cu_seqlens[b + 1] - (int)start;
  }
  int want = p.budget_per_seq ? p.budget_per_seq[b] : p.budget;
  want = want < 0 ? 0 : (want > p.budget ? p.budget : want);
  const int keep = want < L ? want : L;
  const int64_t head = ((int64_t)layer * p.batch + b) * p.n_kv_heads + kv;
  int32_t* out = p.idx + head * p.budget;
  if (tid == 0) p.count[head] = keep;
  if (keep == 0) return;
  if (keep == L) {  // everything survives
    for (int j = tid; j < L; j += kTopkThreads) out[j] = j;
    return;
  }
  const float* src = p.pooled + ((int64_t)layer * p.n_kv_heads + kv) * p.total_tokens + start;
  const bool staged = L <= kTopkLdsKeys;
  if (staged) {
    for (int j = tid; j < L; j += kTopkThreads) keys[j] = order_key(src[j]);
  }
  __syncthreads();
  auto key_at = [&](int j) -> uint32_t { return staged ? keys[j] : order_key(src[j]); };

  // ---- radix select: threshold T = the keep-th largest key, need = how many keys == T to take
  uint32_t prefix = 0, mask = 0;
  int need = keep;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < L; j += kTopkThreads) {
      const uint32_t k = key_at(j);
      if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns digits 4l..4l+3; suffix sums over the lanes above, then inside the lane
      const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
      const uint32_t mine = h0 + h1 + h2 + h3;
      uint32_t incl = mine;  // inclusive suffix sum over lanes >= l
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_down(incl, d, 64);
        if (lane + d < 64) incl += o;
      }
      const uint32_t above = incl - mine;  // keys whose digit is > 4l+3
      const uint32_t g3 = above, g2 = g3 + h3, g1 = g2 + h2, g0 = g1 + h1;  // keys with a larger digit
      const uint32_t un = (uint32_t)need;
      // the digit d of T satisfies greater(d) < need <= greater(d) + hist[d]; exactly one digit does
      if (g3 < un && un <= g3 + h3) { bcast[0] = 4 * lane + 3; bcast[1] = un - g3; }
      if (g2 < un && un <= g2 + h2) { bcast[0] = 4 * lane + 2; bcast[1] = un - g2; }
      if (g1 < un && un <= g1 + h1) { bcast[0] = 4 * lane + 1; bcast[1] = un - g1; }
      if (g0 < un && un <= g0 + h0) { bcast[0] = 4 * lane + 0; bcast[1] = un - g0; }
    }
    __syncthreads();
    prefix |= bcast[0] << shift;
    mask |= 255u << shift;
    need = (int)bcast[1];
    __syncthreads();
  }
  const uint32_t T = prefix;

  // ---- ordered compaction
  uint32_t base_gt = 0, base_eq = 0;  // keys > T / == T before the current block (same in all threads)
  for (int j0 = 0; j0 < L; j0 += kTopkThreads) {
    const int j = j0 + tid;
    const uint32_t k = j < L ? key_at(j) : 0u;
    const bool gt = j < L && k > T;
    const bool eq = j < L && k == T;
    const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const uint32_t w_gt = __popcll(m_gt), w_eq = __popcll(m_eq);
    if (lane == 0) wave_tot[wave] = (w_gt << 16) | w_eq;
    __syncthreads();
    uint32_t pre_gt = base_gt, pre_eq = base_eq, blk_gt = 0, blk_eq = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
      const uint32_t t = wave_tot[w];
      if (w < wave) { pre_gt += t >> 16; pre_eq += t & 0xFFFFu; }
      blk_gt += t >> 16;
      blk_eq += t & 0xFFFFu;
    }
    pre_gt += __popcll(m_gt & below);
    pre_eq += __popcll(m_eq & below);
    const uint32_t un = (uint32_t)need;
    if (gt || (eq && pre_eq < un)) out[pre_gt + (pre_eq < un ? pre_eq : un)] = j;
    base_gt += blk_gt;
    base_eq += blk_eq;
    __syncthreads();
  }
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_topk(const dapq_shape* shape, const float* pooled, int32_t budget, const int32_t* budget_per_seq,
                         int32_t* idx, int32_t* count, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  int rc = check_shape(shape, false, false, false);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(pooled != nullptr && idx != nullptr && count != nullptr, DAPQ_ERR_INVALID_ARG,
               "pooled, idx and count must not be NULL");
  DAPQ_REQUIRE(budget >= 1, DAPQ_ERR_INVALID_ARG, "budget (%d) must be >= 1", budget);
  DAPQ_REQUIRE(shape->batch <= 65535 && shape->n_layers <= 65535, DAPQ_ERR_UNSUPPORTED,
               "batch and n_layers must be <= 65535");
  TopkParams p;
  p.pooled = pooled;
  p.cu_seqlens = shape->cu_seqlens;
  p.budget_per_seq = budget_per_seq;
  p.idx = idx;
  p.count = count;
  p.total_tokens = shape->total_tokens;
  p.batch = shape->batch;
  p.n_kv_heads = shape->n_kv_heads;
  p.budget = budget;
  const int lds_bytes = (320 + kTopkLdsKeys) * (int)sizeof(uint32_t);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(topk_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (e != hipSuccess) return fail(DAPQ_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
  hipLaunchKernelGGL(topk_kernel, dim3((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers),
                     dim3(kTopkThreads), lds_bytes, static_cast<hipStream_t>(stream), p);
  DAPQ_HIP_LAUNCH_CHECK("topk_kernel");
  return DAPQ_OK;
}
