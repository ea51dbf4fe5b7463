// One decode step over the compact cache (Sec. 4.2, last paragraph: decoding starts at position L_p and
// uses only the compressed cache): out = softmax(q K_c^T / sqrt(d_k)) V_c per query head, over the first
// count rows of the KV head's compact cache as dapq_gather wrote it.
//
// One workgroup of 1024 threads per (layer, sequence, KV head); it serves the query heads of the group
// four at a time, so the cache rows are read once per four query heads.  The cache of a head is at
// most a few thousand rows: the step is a matrix-vector product bound by reading K_c and V_c, and with
// one workgroup per head what matters is how many rows a compute unit has in flight: sixteen waves, one
// row per thread in phase 1, eight rows per thread and trip in phase 3.
//   phase 1  a thread takes cache rows in turn: logits = q_h . k for the four heads (bf16 products, fp32
//            accumulation), kept in LDS
//   phase 2  weights 2^(c*logit - max) in LDS, their sums
//   phase 3  a thread owns two channels and a sixteenth of the rows: acc_h += weight_h * v, rows of V read
//            as contiguous 256-byte lines by each wave; the sixteen partial sums meet in LDS
#include <math.h>

#include <type_traits>

#include "dapq_internal.h"

namespace dapq {
namespace {

constexpr int kDecodeThreads = 1024;
constexpr int kDecodeWaves = kDecodeThreads / 64;
constexpr int kDecodeMaxRows = 8192;  // logits of four query heads in LDS (128 KB)
constexpr int kDecodeHeads = 4;       // query heads served per sweep over the cache
constexpr int kDecodeTrip = 8;        // value rows a wave has in flight in phase 3 (4: 7 % slower, 16: 2 %, 32: 15 %)

struct DecodeParams {
  const uint16_t* q;        // [layer][seq][Hq][d]
  const uint16_t* k_cache;  // [layer][seq][Hkv][budget][d]
  const uint16_t* v_cache;
  const int32_t* count;     // [layer][seq][Hkv]
  float* out;               // [layer][seq][Hq][d]
  int32_t n_q_heads, n_kv_heads, budget;
  float c;                  // scale * log2(e)
};

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// Maximum or sum over the workgroup of one value per head; red: [kDecodeWaves][kDecodeHeads].
template <bool IS_MAX>
__device__ __forceinline__ void block_reduce(float (&v)[kDecodeHeads], float* red) {
#pragma unroll
  for (int h = 0; h < kDecodeHeads; ++h) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const float o = __shfl_xor(v[h], d, 64);
      v[h] = IS_MAX ? fmaxf(v[h], o) : v[h] + o;
    }
  }
  const int wave = threadIdx.x >> 6;
  __syncthreads();  // red may still be read from the previous reduction
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int h = 0; h < kDecodeHeads; ++h) red[wave * kDecodeHeads + h] = v[h];
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < kDecodeHeads; ++h) {
    float r = red[h];
#pragma unroll
    for (int w = 1; w < kDecodeWaves; ++w) r = IS_MAX ? fmaxf(r, red[w * kDecodeHeads + h]) : r + red[w * kDecodeHeads + h];
    v[h] = r;
  }
}

__global__ __launch_bounds__(kDecodeThreads) void decode_attention_kernel(DecodeParams p) {
  extern __shared__ float lds[];
  float* qs = lds;                                  // [4][128] the queries in fp32
  float* red = qs + kDecodeHeads * kHeadDim;                   // [waves][4]
  float* w = red + kDecodeWaves * kDecodeHeads;                // [4][budget] logits, then weights
  float* part = w;                                             // [waves][4][128] partial outputs, once the weights are spent
  const int tid = threadIdx.x;
  const int kv = blockIdx.x, seq = blockIdx.y, layer = blockIdx.z;
  const int g = p.n_q_heads / p.n_kv_heads;
  const int64_t head = ((int64_t)layer * gridDim.y + seq) * p.n_kv_heads + kv;
  int n = p.count[head];
  n = n < 0 ? 0 : (n > p.budget ? p.budget : n);
  const uint16_t* kc = p.k_cache + head * p.budget * kHeadDim;
  const uint16_t* vc = p.v_cache + head * p.budget * kHeadDim;

  for (int h0 = 0; h0 < g; h0 += kDecodeHeads) {
    const int nh = g - h0 < kDecodeHeads ? g - h0 : kDecodeHeads;  // query heads of this sweep
    const int64_t qrow0 = ((int64_t)layer * gridDim.y + seq) * p.n_q_heads + (int64_t)kv * g + h0;
    if (n == 0) {  // an empty cache attends to nothing
      for (int e = tid; e < nh * kHeadDim; e += kDecodeThreads) p.out[qrow0 * kHeadDim + e] = 0.0f;
      continue;
    }
    __syncthreads();  // the previous sweep is done with qs, w and part
    for (int e = tid; e < kDecodeHeads * kHeadDim; e += kDecodeThreads)
      qs[e] = e < nh * kHeadDim ? __uint_as_float((uint32_t)p.q[qrow0 * kHeadDim + e] << 16) : 0.0f;
    __syncthreads();

    // phase 1: logits
    float mx[kDecodeHeads];
#pragma unroll
    for (int h = 0; h < kDecodeHeads; ++h) mx[h] = -INFINITY;
    for (int j = tid; j < n; j += kDecodeThreads) {
      const uint4* row = reinterpret_cast<const uint4*>(kc + (int64_t)j * kHeadDim);
      float acc[kDecodeHeads] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int ch = 0; ch < 16; ++ch) {
        const uint4 u = row[ch];
        const float kx[8] = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y),
                             bf16_lo(u.z), bf16_hi(u.z), bf16_lo(u.w), bf16_hi(u.w)};
#pragma unroll
        for (int h = 0; h < kDecodeHeads; ++h) {
          const float* qq = qs + h * kHeadDim + ch * 8;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[h] = fmaf(kx[e], qq[e], acc[h]);
        }
      }
#pragma unroll
      for (int h = 0; h < kDecodeHeads; ++h) {
        const float l = acc[h] * p.c;
        w[h * p.budget + j] = l;
        mx[h] = fmaxf(mx[h], l);
      }
    }
    block_reduce<true>(mx, red);

    // phase 2: weights and their sums
    float sum[kDecodeHeads] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int j = tid; j < n; j += kDecodeThreads) {
#pragma unroll
      for (int h = 0; h < kDecodeHeads; ++h) {
        const float e = exp2f(w[h * p.budget + j] - mx[h]);
        w[h * p.budget + j] = e;
        sum[h] += e;
      }
    }
    block_reduce<false>(sum, red);  // its barriers also publish the weights

    // phase 3: weighted sums of the value rows; a wave takes every kDecodeWaves-th row, kDecodeTrip rows per trip
    const int c2 = tid & 63, part_id = tid >> 6;
    float a0[kDecodeHeads] = {0.0f, 0.0f, 0.0f, 0.0f}, a1[kDecodeHeads] = {0.0f, 0.0f, 0.0f, 0.0f};
    const uint32_t* vcol = reinterpret_cast<const uint32_t*>(vc) + c2;
    int j = part_id;
    auto rows_per_trip = [&](auto trip) {  // `trip` value rows of this wave in flight at a time
      constexpr int kTrip = decltype(trip)::value;
      for (; j + (kTrip - 1) * kDecodeWaves < n; j += kTrip * kDecodeWaves) {
        uint32_t u[kTrip];
#pragma unroll
        for (int r = 0; r < kTrip; ++r) u[r] = vcol[(int64_t)(j + r * kDecodeWaves) * (kHeadDim / 2)];
#pragma unroll
        for (int r = 0; r < kTrip; ++r) {
          const float v0 = bf16_lo(u[r]), v1 = bf16_hi(u[r]);
#pragma unroll
          for (int h = 0; h < kDecodeHeads; ++h) {
            const float e = w[h * p.budget + j + r * kDecodeWaves];
            a0[h] = fmaf(e, v0, a0[h]);
            a1[h] = fmaf(e, v1, a1[h]);
          }
        }
      }
    };
    rows_per_trip(std::integral_constant<int, kDecodeTrip>{});
    rows_per_trip(std::integral_constant<int, 4>{});
    for (; j < n; j += kDecodeWaves) {
      const uint32_t u = vcol[(int64_t)j * (kHeadDim / 2)];
      const float v0 = bf16_lo(u), v1 = bf16_hi(u);
#pragma unroll
      for (int h = 0; h < kDecodeHeads; ++h) {
        const float e = w[h * p.budget + j];
        a0[h] = fmaf(e, v0, a0[h]);
        a1[h] = fmaf(e, v1, a1[h]);
      }
    }
    __syncthreads();  // every wave is done with the weights: their memory takes the partial sums
#pragma unroll
    for (int h = 0; h < kDecodeHeads; ++h) {
      part[(part_id * kDecodeHeads + h) * kHeadDim + 2 * c2] = a0[h];
      part[(part_id * kDecodeHeads + h) * kHeadDim + 2 * c2 + 1] = a1[h];
    }
    __syncthreads();
    for (int e = tid; e < nh * kHeadDim; e += kDecodeThreads) {
      const int h = e / kHeadDim;
      float o = 0.0f;
#pragma unroll
      for (int q = 0; q < kDecodeWaves; ++q) o += part[q * kDecodeHeads * kHeadDim + e];  // fixed order
      p.out[qrow0 * kHeadDim + e] = o / sum[h];
    }
  }
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_decode_attention(const dapq_shape* shape, const void* q_decode, const void* k_cache,
                                              const void* v_cache, const int32_t* count, int32_t budget, float* out,
                                              void* stream) {
  int rc = check_shape(shape, false, false, false);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(q_decode != nullptr && k_cache != nullptr && v_cache != nullptr && count != nullptr && out != nullptr,
               DAPQ_ERR_INVALID_ARG, "q_decode, k_cache, v_cache, count and out must not be NULL");
  DAPQ_REQUIRE(budget >= 1 && budget <= kDecodeMaxRows, DAPQ_ERR_UNSUPPORTED, "budget (%d) must be in [1, %d]", budget,
               kDecodeMaxRows);
  DAPQ_REQUIRE(isfinite(shape->scale) && shape->scale > 0.0f, DAPQ_ERR_INVALID_ARG, "scale must be finite and > 0");
  DAPQ_REQUIRE(((reinterpret_cast<uintptr_t>(k_cache) | reinterpret_cast<uintptr_t>(v_cache)) & 15) == 0,
               DAPQ_ERR_UNSUPPORTED, "k_cache and v_cache must be 16-byte aligned");
  DAPQ_REQUIRE(shape->batch <= 65535 && shape->n_layers <= 65535, DAPQ_ERR_UNSUPPORTED,
               "batch and n_layers must be <= 65535");
  DecodeParams p;
  p.q = static_cast<const uint16_t*>(q_decode);
  p.k_cache = static_cast<const uint16_t*>(k_cache);
  p.v_cache = static_cast<const uint16_t*>(v_cache);
  p.count = count;
  p.out = out;
  p.n_q_heads = shape->n_q_heads;
  p.n_kv_heads = shape->n_kv_heads;
  p.budget = budget;
  p.c = shape->scale * 1.4426950408889634f;
  auto lds_for = [](int b) {
    const int shared_floats = kDecodeHeads * b > kDecodeWaves * kDecodeHeads * kHeadDim
                                  ? kDecodeHeads * b
                                  : kDecodeWaves * kDecodeHeads * kHeadDim;  // weights, later the partial sums
    return (kDecodeHeads * kHeadDim + kDecodeWaves * kDecodeHeads + shared_floats) * (int)sizeof(float);
  };
  const int lds_bytes = lds_for(budget);
  // the limit is raised once, to what the largest supported budget needs
  const int rc_lds = set_max_dynamic_lds(reinterpret_cast<const void*>(decode_attention_kernel), lds_for(kDecodeMaxRows));
  if (rc_lds != DAPQ_OK) return rc_lds;
  hipLaunchKernelGGL(decode_attention_kernel, dim3((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers),
                     dim3(kDecodeThreads), lds_bytes, static_cast<hipStream_t>(stream), p);
  DAPQ_HIP_LAUNCH_CHECK("decode_attention_kernel");
  return DAPQ_OK;
}
