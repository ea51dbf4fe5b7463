// Max-pooling of the accumulated scores along the key axis before selection (Sec. 1 / Sec. 5.1:
// the selection works on pooled accumulated attention scores): pooled(j) = max S(t), |t-j| <= r,
// t inside the sequence of j.
//
// Pure streaming work (4 B in, 4 B out per key).  Each lane loads one float4 (four consecutive
// keys); the neighbours' float4s arrive by wavefront shuffles, so for windows up to width 9 every
// score is read from memory once (plus two halo float4s per wave).  Wider windows take a plain
// loop over the window.
#include <math.h>

#include "dapq_internal.h"

namespace dapq {
namespace {

struct PoolParams {
  const float* scores;
  float* pooled;
  const int32_t* cu_seqlens;
  int64_t total_tokens;
  int32_t batch;
  int32_t radius;
};

// Sequence [start, end) that packed token t belongs to.
__device__ __forceinline__ void seq_of(const PoolParams& p, int64_t t, int64_t* start, int64_t* end) {
  if (p.cu_seqlens == nullptr) {
    const int64_t L = p.total_tokens / p.batch;
    const int64_t b = t / L;
    *start = b * L;
    *end = *start + L;
  } else {
    int lo = 0, hi = p.batch;  // largest b with cu[b] <= t; empty sequences are skipped by <=
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.cu_seqlens[mid] <= t) lo = mid; else hi = mid;
    }
    *start = p.cu_seqlens[lo];
    *end = p.cu_seqlens[lo + 1];
  }
}

__device__ __forceinline__ float4 load4(const float* row, int64_t t, int64_t total) {
  // tokens outside [0, total) read as -inf; the row base is 16-byte aligned only if total % 4 == 0
  float4 v;
  v.x = (t + 0 >= 0 && t + 0 < total) ? row[t + 0] : -INFINITY;
  v.y = (t + 1 >= 0 && t + 1 < total) ? row[t + 1] : -INFINITY;
  v.z = (t + 2 >= 0 && t + 2 < total) ? row[t + 2] : -INFINITY;
  v.w = (t + 3 >= 0 && t + 3 < total) ? row[t + 3] : -INFINITY;
  return v;
}

// radius <= 4: a wave covers 256 consecutive tokens of one (layer, head) row.
__global__ __launch_bounds__(256) void pool_shuffle_kernel(PoolParams p) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t t0 = wave * 256 + lane * 4;  // first token of this lane
  const float* row = p.scores + (int64_t)blockIdx.y * p.total_tokens;
  float* out = p.pooled + (int64_t)blockIdx.y * p.total_tokens;
  if (wave * 256 >= p.total_tokens) return;

  const bool vec = (p.total_tokens & 3) == 0 && t0 + 3 < p.total_tokens &&
                   ((reinterpret_cast<uintptr_t>(row) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  float4 mine = vec ? *reinterpret_cast<const float4*>(row + t0) : load4(row, t0, p.total_tokens);
  float4 left, right;
  left.x = __shfl_up(mine.x, 1, 64);  left.y = __shfl_up(mine.y, 1, 64);
  left.z = __shfl_up(mine.z, 1, 64);  left.w = __shfl_up(mine.w, 1, 64);
  right.x = __shfl_down(mine.x, 1, 64); right.y = __shfl_down(mine.y, 1, 64);
  right.z = __shfl_down(mine.z, 1, 64); right.w = __shfl_down(mine.w, 1, 64);
  if (lane == 0) left = load4(row, t0 - 4, p.total_tokens);
  if (lane == 63) right = load4(row, t0 + 4, p.total_tokens);
  const float win[12] = {left.x, left.y, left.z, left.w, mine.x, mine.y, mine.z, mine.w,
                         right.x, right.y, right.z, right.w};  // tokens t0-4 .. t0+7

  if (t0 >= p.total_tokens) return;
  int64_t s, e;
  seq_of(p, t0, &s, &e);
  float res[4];
#pragma unroll
  for (int o = 0; o < 4; ++o) {
    const int64_t t = t0 + o;
    if (t >= e && t < p.total_tokens) seq_of(p, t, &s, &e);  // crossed into the next sequence
    float m = -INFINITY;
#pragma unroll
    for (int d = -4; d <= 4; ++d) {
      const int64_t u = t + d;
      const bool in = d >= -p.radius && d <= p.radius && u >= s && u < e;
      m = in ? fmaxf(m, win[4 + o + d]) : m;
    }
    res[o] = m;
  }
  if (vec) {
    *reinterpret_cast<float4*>(out + t0) = make_float4(res[0], res[1], res[2], res[3]);
  } else {
#pragma unroll
    for (int o = 0; o < 4; ++o)
      if (t0 + o < p.total_tokens) out[t0 + o] = res[o];
  }
}

// Any radius: one thread per token.
__global__ __launch_bounds__(256) void pool_loop_kernel(PoolParams p) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= p.total_tokens) return;
  const float* row = p.scores + (int64_t)blockIdx.y * p.total_tokens;
  int64_t s, e;
  seq_of(p, t, &s, &e);
  const int64_t lo = t - p.radius > s ? t - p.radius : s;
  const int64_t hi = t + p.radius < e - 1 ? t + p.radius : e - 1;
  float m = -INFINITY;
  for (int64_t u = lo; u <= hi; ++u) m = fmaxf(m, row[u]);
  p.pooled[(int64_t)blockIdx.y * p.total_tokens + t] = m;
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_pool(const dapq_shape* shape, const float* scores, float* pooled, int32_t width, void* stream) {
  int rc = check_shape(shape, false, false, false);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(scores != nullptr && pooled != nullptr, DAPQ_ERR_INVALID_ARG, "scores and pooled must not be NULL");
  DAPQ_REQUIRE(scores != pooled, DAPQ_ERR_INVALID_ARG, "pooled must not alias scores");
  DAPQ_REQUIRE(width >= 1 && width <= 63 && (width & 1) == 1, DAPQ_ERR_INVALID_ARG,
               "pool width (%d) must be odd and in [1, 63]", width);
  if (shape->total_tokens == 0) return DAPQ_OK;
  PoolParams p;
  p.scores = scores;
  p.pooled = pooled;
  p.cu_seqlens = shape->cu_seqlens;
  p.total_tokens = shape->total_tokens;
  p.batch = shape->batch;
  p.radius = (width - 1) / 2;
  const unsigned rows = (unsigned)(shape->n_layers * shape->n_kv_heads);
  if (p.radius <= 4) {
    const int64_t blocks = (shape->total_tokens + 1023) / 1024;
    hipLaunchKernelGGL(pool_shuffle_kernel, dim3((unsigned)blocks, rows), dim3(256), 0,
                       static_cast<hipStream_t>(stream), p);
    DAPQ_HIP_LAUNCH_CHECK("pool_shuffle_kernel");
  } else {
    const int64_t blocks = (shape->total_tokens + 255) / 256;
    hipLaunchKernelGGL(pool_loop_kernel, dim3((unsigned)blocks, rows), dim3(256), 0,
                       static_cast<hipStream_t>(stream), p);
    DAPQ_HIP_LAUNCH_CHECK("pool_loop_kernel");
  }
  return DAPQ_OK;
}
