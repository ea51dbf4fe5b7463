// Position assignment (Sec. 4.1): rotary embedding of bf16 vectors at given absolute positions.
// The pseudo queries get positions L_p .. L_p+N-1, the positions of the first N decode steps.
//
// One thread owns two neighbouring channel pairs of a row (one if the buffers are not 4-byte aligned)
// and a run of heads: it evaluates the angles pos * theta^(-2c/d) and their sines / cosines once in
// fp64 and then walks its heads, reading and writing two elements per access, so the transcendental
// work (more than ten times the work of one rotation) is shared by the heads of a run; runs are
// 8 heads long, longer (up to 64) while the launch still has thousands of waves.
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

// CPT = channel pairs per thread: 1, or 2 neighbouring ones, whose elements are then read and written two at a
// time (4-byte accesses; the launcher checks the alignment this needs).
template <int CPT>
__global__ void rope_kernel(const uint16_t* x_in, uint16_t* x_out, const int32_t* __restrict__ pos,
                            int64_t rows, int heads, int head_dim, int64_t stride_row, int64_t stride_head,
                            double neg_log2_theta_2_over_d, int pairing, int heads_per_thread) {
  const int half = head_dim >> 1;
  const int per_row = half / CPT;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= rows * per_row) return;
  const int64_t row = gid / per_row;
  const int c = (int)(gid - row * per_row) * CPT;
  double sn[CPT], cs[CPT];
#pragma unroll
  for (int t = 0; t < CPT; ++t) {
    const double omega = exp2((double)(c + t) * neg_log2_theta_2_over_d);  // theta^(-2c/d)
    sincos((double)pos[row] * omega, &sn[t], &cs[t]);
  }
  // element offsets of the thread's first accesses: the a and b of pair c (CPT = 1), or two words that hold the
  // a's and the b's of pairs c, c+1 (half pairing) / the (a, b) of pair c and of pair c+1 (interleaved pairing)
  const int i0 = pairing == 0 ? c : 2 * c;
  const int i1 = pairing == 0 ? c + half : 2 * c + (CPT == 1 ? 1 : 2);
  const uint16_t* src = x_in + row * stride_row;
  uint16_t* dst = x_out + row * stride_row;
  const int hd0 = blockIdx.y * heads_per_thread;
  const int hd1 = hd0 + heads_per_thread < heads ? hd0 + heads_per_thread : heads;
  auto rotate = [&](int hd, uint32_t r0, uint32_t r1) {
    if constexpr (CPT == 1) {
      const double a = bf16_to_f64((uint16_t)r0), b = bf16_to_f64((uint16_t)r1);
      dst[(int64_t)hd * stride_head + i0] = f64_to_bf16(a * cs[0] - b * sn[0]);
      dst[(int64_t)hd * stride_head + i1] = f64_to_bf16(b * cs[0] + a * sn[0]);
    } else {
      // half pairing: r0 = (a0, a1), r1 = (b0, b1); interleaved: r0 = (a0, b0), r1 = (a1, b1)
      const uint16_t a0 = (uint16_t)r0, a1 = pairing == 0 ? (uint16_t)(r0 >> 16) : (uint16_t)r1;
      const uint16_t b0 = pairing == 0 ? (uint16_t)r1 : (uint16_t)(r0 >> 16), b1 = (uint16_t)(r1 >> 16);
      const double fa0 = bf16_to_f64(a0), fb0 = bf16_to_f64(b0), fa1 = bf16_to_f64(a1), fb1 = bf16_to_f64(b1);
      const uint32_t oa0 = f64_to_bf16(fa0 * cs[0] - fb0 * sn[0]), ob0 = f64_to_bf16(fb0 * cs[0] + fa0 * sn[0]);
      const uint32_t oa1 = f64_to_bf16(fa1 * cs[1] - fb1 * sn[1]), ob1 = f64_to_bf16(fb1 * cs[1] + fa1 * sn[1]);
      uint32_t* d0 = reinterpret_cast<uint32_t*>(dst + (int64_t)hd * stride_head + i0);
      uint32_t* d1 = reinterpret_cast<uint32_t*>(dst + (int64_t)hd * stride_head + i1);
      *d0 = pairing == 0 ? (oa0 | (oa1 << 16)) : (oa0 | (ob0 << 16));
      *d1 = pairing == 0 ? (ob0 | (ob1 << 16)) : (oa1 | (ob1 << 16));
    }
  };
  auto fetch = [&](int hd, int i) -> uint32_t {
    const uint16_t* p = src + (int64_t)hd * stride_head + i;
    if constexpr (CPT == 1) return *p;
    else return *reinterpret_cast<const uint32_t*>(p);
  };
  int hd = hd0;
  for (; hd + 4 <= hd1; hd += 4) {  // four heads per trip: eight loads in flight before the first rotation
    uint32_t r0[4], r1[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      r0[u] = fetch(hd + u, i0);
      r1[u] = fetch(hd + u, i1);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) rotate(hd + u, r0[u], r1[u]);
  }
  for (; hd < hd1; ++hd) {
    const uint32_t r0 = fetch(hd, i0), r1 = fetch(hd, i1);
    rotate(hd, r0, r1);
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
  // two channel pairs per thread when every access of a thread is then a whole aligned 4-byte word
  const bool wide = (head_dim / 2) % 2 == 0 && stride_row % 2 == 0 && stride_head % 2 == 0 &&
                    (reinterpret_cast<uintptr_t>(x_in) | reinterpret_cast<uintptr_t>(x_out)) % 4 == 0;
  const int cpt = wide ? 2 : 1;
  // enough waves to keep every SIMD busy while the runs are as long as possible (measured on the pseudo queries of
  // the 8B shape: 64 rows x 1024 heads)
  const int64_t min_waves = wide ? 2048 : 4096;
  const int64_t work = rows * (head_dim / 2 / cpt);
  DAPQ_REQUIRE(work / 256 < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED, "too many rows");
  if (work == 0) return DAPQ_OK;
  int hpt = 8;
  while (hpt < 64 && hpt * 2 <= heads && (work / 64) * ((heads + 2 * hpt - 1) / (2 * hpt)) >= min_waves) hpt *= 2;
  const int64_t head_runs = ((int64_t)heads + hpt - 1) / hpt;
  DAPQ_REQUIRE(head_runs <= 65535, DAPQ_ERR_UNSUPPORTED, "heads (%d) exceeds %d", heads, 65535 * hpt);
  const double e = -2.0 * log2(theta) / (double)head_dim;
  const dim3 grid((unsigned)((work + 255) / 256), (unsigned)head_runs);
  if (cpt == 2)
    hipLaunchKernelGGL(rope_kernel<2>, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(x_in), static_cast<uint16_t*>(x_out), pos, rows, heads, head_dim,
                       stride_row, stride_head, e, pairing, hpt);
  else
    hipLaunchKernelGGL(rope_kernel<1>, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(x_in), static_cast<uint16_t*>(x_out), pos, rows, heads, head_dim,
                       stride_row, stride_head, e, pairing, hpt);
  DAPQ_HIP_LAUNCH_CHECK("rope_kernel");
  return DAPQ_OK;
}
