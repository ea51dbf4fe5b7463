// Position assignment (Sec. 4.1): rotary embedding of bf16 vectors at given absolute positions.
// The pseudo queries get positions L_p .. L_p+N-1, the positions of the first N decode steps.
//
// One thread owns one (row, channel pair) and a run of heads: it evaluates the angle
// pos * theta^(-2c/d) and its sine / cosine once in fp64 and then walks its heads, so the
// transcendental work (more than ten times the work of one rotation) is shared by the heads of a
// run; runs are 8 heads long, longer (up to 64) while the launch still has thousands of waves.
// fp64 keeps the angle exact enough at positions beyond 10^5 (an fp32 product pos * omega would be
// off by ~1e-2 rad there); the rotation is done in fp64 as well and rounded to bf16 once, which is
// what makes the result equal to a float64 evaluation bit for bit, and what the kernel's time goes
// into (fp64 multiplies and the two conversions per rotated pair).
#include <math.h>

#include "dapq_internal.h"

namespace dapq {
namespace {

__device__ __forceinline__ double bf16_to_f64(uint16_t b) { return (double)__uint_as_float((uint32_t)b << 16); }

// fp64 -> bf16, round to nearest even, as if in one step: the value is first brought to fp32 with rounding to odd
// (truncate toward zero, then set the last bit if anything was cut off: the cut-off part can then neither make nor
// break a tie 16 bits further up), and the 16 low bits are rounded by the hardware conversion.  The truncation is
// the ordinary (nearest) conversion stepped back by one unit when it went away from zero.
__device__ __forceinline__ uint16_t f64_to_bf16(double x) {
  const float f = (float)x;
  const double back = (double)f;
  uint32_t u = __float_as_uint(f);
  if (back != x) {  // inexact (also true for NaN, which stays NaN)
    if (fabs(back) > fabs(x)) u -= 1u;
    u |= 1u;
  }
  return __builtin_bit_cast(uint16_t, (__bf16)__uint_as_float(u));
}

__global__ void rope_kernel(const uint16_t* x_in, uint16_t* x_out, const int32_t* __restrict__ pos,
                            int64_t rows, int heads, int head_dim, int64_t stride_row, int64_t stride_head,
                            double neg_log2_theta_2_over_d, int pairing, int heads_per_thread) {
  const int half = head_dim >> 1;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= rows * half) return;
  const int64_t row = gid / half;
  const int c = (int)(gid - row * half);
  const double omega = exp2((double)c * neg_log2_theta_2_over_d);  // theta^(-2c/d)
  double sn, cs;
  sincos((double)pos[row] * omega, &sn, &cs);
  const int ia = pairing == 0 ? c : 2 * c;
  const int ib = pairing == 0 ? c + half : 2 * c + 1;
  const uint16_t* src = x_in + row * stride_row;
  uint16_t* dst = x_out + row * stride_row;
  const int hd0 = blockIdx.y * heads_per_thread;
  const int hd1 = hd0 + heads_per_thread < heads ? hd0 + heads_per_thread : heads;
  int hd = hd0;
  for (; hd + 4 <= hd1; hd += 4) {  // four heads per trip: eight loads in flight before the first rotation
    uint16_t ra[4], rb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ra[u] = src[(int64_t)(hd + u) * stride_head + ia];
      rb[u] = src[(int64_t)(hd + u) * stride_head + ib];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const double a = bf16_to_f64(ra[u]), b = bf16_to_f64(rb[u]);
      dst[(int64_t)(hd + u) * stride_head + ia] = f64_to_bf16(a * cs - b * sn);
      dst[(int64_t)(hd + u) * stride_head + ib] = f64_to_bf16(b * cs + a * sn);
    }
  }
  for (; hd < hd1; ++hd) {
    const double a = bf16_to_f64(src[(int64_t)hd * stride_head + ia]);
    const double b = bf16_to_f64(src[(int64_t)hd * stride_head + ib]);
    dst[(int64_t)hd * stride_head + ia] = f64_to_bf16(a * cs - b * sn);
    dst[(int64_t)hd * stride_head + ib] = f64_to_bf16(b * cs + a * sn);
  }
}

// Sec. 4.1 / Sec. 5.1: which prompt token each pseudo token copies (first m, last n) and the position
// it is given (L_p + i), for every sequence of a possibly ragged batch, without a host round trip
// for the sequence lengths.
__global__ void pseudo_tokens_kernel(const int32_t* cu_seqlens, int64_t total_tokens, int batch, int first_m, int last_n,
                                     int32_t* token_idx, int32_t* positions) {
  const int n = first_m + last_n;
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= batch * n) return;
  const int b = gid / n, i = gid - b * n;
  int64_t start;
  int L;
  if (cu_seqlens == nullptr) {
    L = (int)(total_tokens / batch);
    start = (int64_t)b * L;
  } else {
    start = cu_seqlens[b];
    L = cu_seqlens[b + 1] - (int)start;
  }
  int src;
  if (i < first_m) src = i < L - 1 ? i : L - 1;
  else src = L > 0 ? (L - last_n + (i - first_m) > 0 ? L - last_n + (i - first_m) : 0) : -1;
  token_idx[gid] = src >= 0 ? (int32_t)(start + src) : -1;
  positions[gid] = L + i;
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_pseudo_tokens(const dapq_shape* shape, int32_t first_m, int32_t last_n, int32_t* token_idx,
                                           int32_t* positions, void* stream) {
  int rc = check_shape(shape, false, false, false);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(token_idx != nullptr && positions != nullptr, DAPQ_ERR_INVALID_ARG, "token_idx and positions must not be NULL");
  DAPQ_REQUIRE(first_m >= 0 && last_n >= 0 && (int64_t)first_m + last_n == shape->n_pseudo, DAPQ_ERR_INVALID_ARG,
               "first_m (%d) + last_n (%d) must equal n_pseudo (%d)", first_m, last_n, shape->n_pseudo);
  const int64_t work = (int64_t)shape->batch * shape->n_pseudo;
  DAPQ_REQUIRE(work < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED, "batch * n_pseudo is too large");
  hipLaunchKernelGGL(pseudo_tokens_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), shape->cu_seqlens, shape->total_tokens, shape->batch, first_m, last_n,
                     token_idx, positions);
  DAPQ_HIP_LAUNCH_CHECK("pseudo_tokens_kernel");
  return DAPQ_OK;
}


extern "C" DAPQ_API int dapq_rope_apply(const void* x_in, void* x_out, const int32_t* pos, int64_t rows, int32_t heads,
                               int32_t head_dim, int64_t stride_row, int64_t stride_head, double theta,
                               int32_t pairing, void* stream) {
  DAPQ_REQUIRE(x_in != nullptr && x_out != nullptr && pos != nullptr, DAPQ_ERR_INVALID_ARG,
               "x_in, x_out and pos must not be NULL");
  DAPQ_REQUIRE(rows >= 0 && heads >= 1, DAPQ_ERR_INVALID_ARG, "rows (%lld) must be >= 0 and heads (%d) >= 1",
               (long long)rows, heads);
  DAPQ_REQUIRE(head_dim >= 2 && head_dim % 2 == 0, DAPQ_ERR_INVALID_ARG, "head_dim (%d) must be even and >= 2",
               head_dim);
  DAPQ_REQUIRE(pairing == 0 || pairing == 1, DAPQ_ERR_INVALID_ARG, "pairing must be 0 (half) or 1 (interleaved)");
  DAPQ_REQUIRE(theta > 0.0 && isfinite(theta), DAPQ_ERR_INVALID_ARG, "theta must be finite and > 0");
  DAPQ_REQUIRE(stride_head >= head_dim && stride_row >= 0, DAPQ_ERR_INVALID_ARG,
               "stride_head (%lld) must cover head_dim and stride_row (%lld) must be >= 0", (long long)stride_head,
               (long long)stride_row);
  const int64_t work = rows * (head_dim / 2);
  DAPQ_REQUIRE(work / 256 < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED, "too many rows");
  if (work == 0) return DAPQ_OK;
  int hpt = 8;
  while (hpt < 64 && hpt * 2 <= heads && (work / 64) * ((heads + 2 * hpt - 1) / (2 * hpt)) >= 4096) hpt *= 2;
  const int64_t head_runs = ((int64_t)heads + hpt - 1) / hpt;
  DAPQ_REQUIRE(head_runs <= 65535, DAPQ_ERR_UNSUPPORTED, "heads (%d) exceeds %d", heads, 65535 * hpt);
  const double e = -2.0 * log2(theta) / (double)head_dim;
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((work + 255) / 256), (unsigned)head_runs), dim3(256), 0,
                     static_cast<hipStream_t>(stream),
                     static_cast<const uint16_t*>(x_in), static_cast<uint16_t*>(x_out), pos, rows, heads, head_dim,
                     stride_row, stride_head, e, pairing, hpt);
  DAPQ_HIP_LAUNCH_CHECK("rope_kernel");
  return DAPQ_OK;
}
