// M_retain = TopK_j S(j) (Sec. 4.2): per (layer, sequence, KV head) the budget positions with the
// largest pooled score, equal scores lowest position first, written in ascending position.
//
// One workgroup of 1024 threads per head.  Selection is an exact radix select on the
// order-preserving integer image of the fp32 score: four 8-bit digits from the top, each pass a
// 256-bin LDS histogram followed by a suffix scan that fixes one digit of the threshold T and the
// number of keys equal to T still needed.  The last step is an ordered compaction: key j is kept if
// score > T, or score == T and fewer than `need` equal keys precede it; prefix counts of (greater,
// equal) give both the decision and the output slot, so the result is ascending and deterministic
// (no atomic decides an order).  Max-pooling makes runs of bit-equal scores, so the tie rule is on
// the main path.
//
// Scores are positive and bunch into a few binades, so in the first pass nearly every key lands in
// the same bin: each wave therefore counts the keys that share the digit of its first candidate
// with a reduction and issues one atomic for them; only the others go to the histogram one by one.
//
// Heads of up to 65536 keys (topk_reg_kernel) are read from HBM once into registers, thread t
// owning the consecutive keys [t*KPT, (t+1)*KPT): every pass runs out of registers and the
// compaction needs a single workgroup scan.  Because a thread holds a run of consecutive scores, the
// same kernel can apply the max-pool that precedes selection (Sec. 1 / Sec. 5.1) on the way in
// (dapq_pool_topk): three halo scores per side for the window of 7, no pooled array in HBM.  Longer heads (topk_stream_kernel) stage what fits in
// LDS (36864 keys) or re-read the scores from L2 on every pass.
#include "dapq_internal.h"

namespace dapq {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kTopkLdsKeys = 36864;

struct TopkParams {
  const float* pooled;        // the scores selection runs on (the register variant can pool them itself)
  float* pooled_out;          // register variant with a pooling radius: where to write the pooled scores, or NULL
  const int32_t* cu_seqlens;
  const int32_t* budget_per_seq;
  int32_t* idx;
  int32_t* count;
  int64_t total_tokens;
  int32_t batch, n_kv_heads, budget;
  int32_t min_len, max_len;  // this launch handles the heads with min_len <= L <= max_len
};

// fp32 -> uint32 with the same order for all non-NaN values.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// What every variant needs to know about its head; heads of another launch (length outside
// [min_len, max_len]), keep == 0 and keep == L are finished here.
struct TopkHead {
  const float* src;
  int32_t* out;
  int L, keep;
  bool done;     // nothing left to select
  bool foreign;  // the head belongs to another launch
};

__device__ __forceinline__ TopkHead topk_head(const TopkParams& p) {
  TopkHead hd;
  const int tid = threadIdx.x;
  const int kv = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
  int64_t start;
  if (p.cu_seqlens == nullptr) {
    hd.L = (int)(p.total_tokens / p.batch);
    start = (int64_t)b * hd.L;
  } else {
    start = p.cu_seqlens[b];
    hd.L = p.cu_seqlens[b + 1] - (int)start;
  }
  hd.foreign = hd.L < p.min_len || hd.L > p.max_len;
  if (hd.foreign) {
    hd.done = true;
    hd.keep = 0;
    hd.out = nullptr;
    hd.src = nullptr;
    return hd;
  }
  int want = p.budget_per_seq ? p.budget_per_seq[b] : p.budget;
  want = want < 0 ? 0 : (want > p.budget ? p.budget : want);
  hd.keep = want < hd.L ? want : hd.L;
  const int64_t head = ((int64_t)layer * p.batch + b) * p.n_kv_heads + kv;
  hd.out = p.idx + head * p.budget;
  hd.src = p.pooled + ((int64_t)layer * p.n_kv_heads + kv) * p.total_tokens + start;
  if (tid == 0) p.count[head] = hd.keep;
  hd.done = hd.keep == 0;
  if (!hd.done && hd.keep == hd.L) {  // everything survives
    for (int j = tid; j < hd.L; j += (int)blockDim.x) hd.out[j] = j;
    hd.done = true;
  }
  return hd;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// After a histogram pass: wave 0 finds the digit d of T, the one with greater(d) < need <= greater(d)
// + hist[d], and publishes (d, need - greater(d)) in bcast.
__device__ __forceinline__ void topk_pick_digit(const uint32_t* hist, uint32_t* bcast, int need, int lane) {
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
  if (g3 < un && un <= g3 + h3) { bcast[0] = 4 * lane + 3; bcast[1] = un - g3; }
  if (g2 < un && un <= g2 + h2) { bcast[0] = 4 * lane + 2; bcast[1] = un - g2; }
  if (g1 < un && un <= g1 + h1) { bcast[0] = 4 * lane + 1; bcast[1] = un - g1; }
  if (g0 < un && un <= g0 + h0) { bcast[0] = 4 * lane + 0; bcast[1] = un - g0; }
}

// ---- heads that fit in registers.  R > 0: the input is the un-pooled score and the kernel applies
// the max-pool of radius R itself (window clipped at the ends of the sequence) before selecting.
template <int THREADS, int KPT, int R>
__global__ __launch_bounds__(THREADS) void topk_reg_kernel(TopkParams p) {
  constexpr int kWaves = THREADS / 64;
  __shared__ uint32_t hist[256];
  __shared__ uint32_t bcast[2];
  __shared__ uint32_t wave_gt[kWaves], wave_eq[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const TopkHead hd = topk_head(p);
  if (hd.foreign || (hd.done && p.pooled_out == nullptr)) return;  // a finished head may still owe its pooled scores
  const int L = hd.L;

  // thread t owns keys [t*KPT, t*KPT + KPT): registers i < nvalid hold a key.  (A layout with
  // contiguous rows per wave loads no faster here and makes the compaction twice as long.)
  const int j0 = tid * KPT;
  const int nvalid = L - j0 < 0 ? 0 : (L - j0 > KPT ? KPT : L - j0);
  float ext[KPT + 2 * R];  // scores j0-R .. j0+KPT+R-1; -inf outside the sequence
  if (nvalid == KPT && (reinterpret_cast<uintptr_t>(hd.src + j0) & 15) == 0) {
#pragma unroll
    for (int i = 0; i < KPT; i += 4) {
      const float4 v = *reinterpret_cast<const float4*>(hd.src + j0 + i);
      ext[R + i] = v.x;
      ext[R + i + 1] = v.y;
      ext[R + i + 2] = v.z;
      ext[R + i + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < KPT; ++i) ext[R + i] = i < nvalid ? hd.src[j0 + i] : -INFINITY;
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int jl = j0 - R + r, jr = j0 + KPT + r;
    ext[r] = (jl >= 0 && jl < L) ? hd.src[jl] : -INFINITY;
    ext[R + KPT + r] = jr < L ? hd.src[jr] : -INFINITY;
  }
  uint32_t key[KPT];
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    float m = ext[i];
#pragma unroll
    for (int t = 1; t <= 2 * R; ++t) m = fmaxf(m, ext[i + t]);
    if (p.pooled_out != nullptr && i < nvalid) p.pooled_out[(hd.src - p.pooled) + j0 + i] = m;
    key[i] = i < nvalid ? order_key(m) : 0u;
  }
  if (hd.done) return;

  // ---- radix select: threshold T = the keep-th largest key, need = how many keys == T to take
  uint32_t prefix = 0, mask = 0;
  int need = hd.keep;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int e = tid; e < 256; e += THREADS) hist[e] = 0;
    __syncthreads();
    // the digit most keys of this wave are likely to share: that of its first candidate
    int first = -1;
#pragma unroll
    for (int i = KPT - 1; i >= 0; --i)
      if (i < nvalid && (key[i] & mask) == prefix) first = (int)((key[i] >> shift) & 255u);
    const uint64_t have = __ballot(first >= 0);
    if (have != 0) {
      const uint32_t d0 = (uint32_t)__shfl(first, __ffsll((long long)have) - 1, 64);
      uint32_t same = 0;
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        if (i < nvalid && (key[i] & mask) == prefix) {
          const uint32_t d = (key[i] >> shift) & 255u;
          if (d == d0) ++same;
          else atomicAdd(&hist[d], 1u);
        }
      }
      same = wave_sum(same);
      if (lane == 0 && same != 0) atomicAdd(&hist[d0], same);
    }
    __syncthreads();
    if (wave == 0) topk_pick_digit(hist, bcast, need, lane);
    __syncthreads();
    prefix |= bcast[0] << shift;
    mask |= 255u << shift;
    need = (int)bcast[1];
    __syncthreads();
  }
  const uint32_t T = prefix;

  // ---- ordered compaction: one exclusive scan of the per-thread (greater, equal) counts
  uint32_t my_gt = 0, my_eq = 0;
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    my_gt += (i < nvalid && key[i] > T) ? 1u : 0u;
    my_eq += (i < nvalid && key[i] == T) ? 1u : 0u;
  }
  uint32_t inc_gt = my_gt, inc_eq = my_eq;  // inclusive scans inside the wave
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t a = __shfl_up(inc_gt, d, 64), c = __shfl_up(inc_eq, d, 64);
    if (lane >= d) {
      inc_gt += a;
      inc_eq += c;
    }
  }
  if (lane == 63) {
    wave_gt[wave] = inc_gt;
    wave_eq[wave] = inc_eq;
  }
  __syncthreads();
  uint32_t pre_gt = inc_gt - my_gt, pre_eq = inc_eq - my_eq;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) {
      pre_gt += wave_gt[w];
      pre_eq += wave_eq[w];
    }
  }
  const uint32_t un = (uint32_t)need;
  uint32_t pos = pre_gt + (pre_eq < un ? pre_eq : un);
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    if (i < nvalid) {
      if (key[i] > T) {
        hd.out[pos++] = j0 + i;
      } else if (key[i] == T) {
        if (pre_eq < un) hd.out[pos++] = j0 + i;
        ++pre_eq;
      }
    }
  }
}

// ---- longer heads
__global__ __launch_bounds__(kTopkThreads) void topk_stream_kernel(TopkParams p) {
  extern __shared__ uint32_t smem[];
  uint32_t* hist = smem;             // [256]
  uint32_t* wave_tot = smem + 256;   // [16]
  uint32_t* bcast = smem + 256 + 16; // [2]: digit, need
  uint32_t* keys = smem + 320;       // [kTopkLdsKeys] staged order keys (if they fit)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const TopkHead hd = topk_head(p);
  if (hd.done) return;
  const int L = hd.L;
  const float* src = hd.src;
  int32_t* out = hd.out;
  const bool staged = L <= kTopkLdsKeys;
  if (staged) {
    for (int j = tid; j < L; j += kTopkThreads) keys[j] = order_key(src[j]);
  }
  __syncthreads();
  // a thread takes four consecutive keys per trip (one 16-byte load when the head is 16-byte aligned): a trip is a
  // tile of 4096 keys, thread t owning keys [4t, 4t + 4) of it.  Keys past the end read as 0 and are never candidates.
  const bool aligned = (reinterpret_cast<uintptr_t>(src) & 15) == 0;
  auto keys_at = [&](int j, uint32_t (&k)[4]) {
    if (staged) {
      if (j + 3 < L) {
        const uint4 v = *reinterpret_cast<const uint4*>(keys + j);  // keys is 16-byte aligned, j a multiple of 4
        k[0] = v.x; k[1] = v.y; k[2] = v.z; k[3] = v.w;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) k[u] = j + u < L ? keys[j + u] : 0u;
      }
    } else if (aligned && j + 3 < L) {
      const float4 v = *reinterpret_cast<const float4*>(src + j);
      k[0] = order_key(v.x); k[1] = order_key(v.y); k[2] = order_key(v.z); k[3] = order_key(v.w);
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) k[u] = j + u < L ? order_key(src[j + u]) : 0u;
    }
  };
  constexpr int kTile = 4 * kTopkThreads;

  // ---- radix select: threshold T = the keep-th largest key, need = how many keys == T to take
  uint32_t prefix = 0, mask = 0;
  int need = hd.keep;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int jb = 0; jb < L; jb += kTile) {  // the trip count is the same for every thread
      const int j = jb + 4 * tid;
      uint32_t k[4];
      keys_at(j, k);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool cand = j + u < L && (k[u] & mask) == prefix;
        const uint32_t d = (k[u] >> shift) & 255u;
        const uint64_t have = __ballot(cand);
        if (have != 0) {
          const uint32_t d0 = (uint32_t)__shfl((int)d, __ffsll((long long)have) - 1, 64);
          const uint64_t same = __ballot(cand && d == d0);
          if (cand && d != d0) atomicAdd(&hist[d], 1u);
          if (lane == 0) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
        }
      }
    }
    __syncthreads();
    if (wave == 0) topk_pick_digit(hist, bcast, need, lane);
    __syncthreads();
    prefix |= bcast[0] << shift;
    mask |= 255u << shift;
    need = (int)bcast[1];
    __syncthreads();
  }
  const uint32_t T = prefix;

  // ---- ordered compaction, one tile of 4096 keys at a time: per-thread counts of (greater, equal), an inclusive
  // scan inside the wave, wave totals through LDS, then every thread writes its survivors in key order
  uint32_t base_gt = 0, base_eq = 0;  // keys > T / == T before the current tile (same in all threads)
  const uint32_t un = (uint32_t)need;
  for (int jb = 0; jb < L; jb += kTile) {
    const int j = jb + 4 * tid;
    uint32_t k[4];
    keys_at(j, k);
    uint32_t my = 0;  // (greater << 16) | equal over this thread's four keys
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (j + u < L) my += (k[u] > T ? 0x10000u : 0u) + (k[u] == T ? 1u : 0u);
    }
    uint32_t inc = my;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t o = __shfl_up(inc, d, 64);
      if (lane >= d) inc += o;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t pre = inc - my, blk = 0;  // packed counts before this thread inside the tile / of the whole tile
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
      const uint32_t t = wave_tot[w];
      if (w < wave) pre += t;
      blk += t;
    }
    uint32_t pre_gt = base_gt + (pre >> 16), pre_eq = base_eq + (pre & 0xFFFFu);
    if (my != 0) {
      uint32_t pos = pre_gt + (pre_eq < un ? pre_eq : un);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j + u < L) {
          if (k[u] > T) {
            out[pos++] = j + u;
          } else if (k[u] == T) {
            if (pre_eq < un) out[pos++] = j + u;
            ++pre_eq;
          }
        }
      }
    }
    base_gt += blk >> 16;
    base_eq += blk & 0xFFFFu;
    __syncthreads();
  }
}

}  // namespace
}  // namespace dapq

using namespace dapq;

namespace dapq {
namespace {

// Register-variant shapes: (threads, keys per thread).  Short heads use small workgroups so that
// several of them share a compute unit.
struct RegVariant {
  int threads, kpt;
  int64_t max_len() const { return (int64_t)threads * kpt; }
};

RegVariant reg_variant_for(int64_t len) {
  if (len <= 256 * 32) return {256, 32};
  if (len <= 256 * 64) return {256, 64};
  if (len <= 1024 * 32) return {1024, 32};
  return {1024, 64};
}

template <int R>
void launch_reg(RegVariant v, dim3 grid, hipStream_t st, const TopkParams& p) {
  if (v.threads == 256 && v.kpt == 32) hipLaunchKernelGGL((topk_reg_kernel<256, 32, R>), grid, dim3(256), 0, st, p);
  else if (v.threads == 256) hipLaunchKernelGGL((topk_reg_kernel<256, 64, R>), grid, dim3(256), 0, st, p);
  else if (v.kpt == 32) hipLaunchKernelGGL((topk_reg_kernel<1024, 32, R>), grid, dim3(1024), 0, st, p);
  else hipLaunchKernelGGL((topk_reg_kernel<1024, 64, R>), grid, dim3(1024), 0, st, p);
}

int topk_common_checks(const dapq_shape* shape, const float* in, int32_t budget, const int32_t* idx, const int32_t* count) {
  int rc = check_shape(shape, false, false, false);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(in != nullptr && idx != nullptr && count != nullptr, DAPQ_ERR_INVALID_ARG,
               "scores, idx and count must not be NULL");
  DAPQ_REQUIRE(budget >= 1, DAPQ_ERR_INVALID_ARG, "budget (%d) must be >= 1", budget);
  DAPQ_REQUIRE(shape->batch <= 65535 && shape->n_layers <= 65535, DAPQ_ERR_UNSUPPORTED,
               "batch and n_layers must be <= 65535");
  return DAPQ_OK;
}

}  // namespace
}  // namespace dapq

extern "C" DAPQ_API int dapq_topk(const dapq_shape* shape, const float* pooled, int32_t budget, const int32_t* budget_per_seq,
                         int32_t* idx, int32_t* count, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  int rc = topk_common_checks(shape, pooled, budget, idx, count);
  if (rc != DAPQ_OK) return rc;
  TopkParams p;
  p.pooled = pooled;
  p.pooled_out = nullptr;
  p.cu_seqlens = shape->cu_seqlens;
  p.budget_per_seq = budget_per_seq;
  p.idx = idx;
  p.count = count;
  p.total_tokens = shape->total_tokens;
  p.batch = shape->batch;
  p.n_kv_heads = shape->n_kv_heads;
  p.budget = budget;
  // Heads that fit the chosen register variant go there, longer ones to the streaming kernel.  A
  // dense batch knows its length; a ragged one launches both kernels, each skipping the heads of
  // the other.
  const dim3 grid((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t mean = shape->total_tokens / shape->batch;
  const int64_t longest = shape->cu_seqlens == nullptr ? mean : shape->total_tokens;
  // a ragged batch sizes the variant for 1.5 x its mean length (or everything, if that is less)
  const int64_t sized_for = shape->cu_seqlens == nullptr ? mean : (mean + mean / 2 < longest ? mean + mean / 2 : longest);
  const RegVariant variant = reg_variant_for(sized_for);
  const int64_t reg_max = variant.max_len();
  p.min_len = 0;
  p.max_len = (int32_t)reg_max;
  if (shape->cu_seqlens != nullptr || mean <= reg_max) {  // (a dense batch of longer heads has nothing for it)
    launch_reg<0>(variant, grid, st, p);
    DAPQ_HIP_LAUNCH_CHECK("topk_reg_kernel");
  }
  if (longest > reg_max) {
    p.min_len = (int32_t)reg_max + 1;
    p.max_len = INT32_MAX;
    // heads of up to kTopkLdsKeys keys are staged in LDS; if none of this launch can be that short the staging
    // area is left out
    const int lds_bytes = (320 + (p.min_len <= kTopkLdsKeys ? kTopkLdsKeys : 0)) * (int)sizeof(uint32_t);
    // the limit is raised once, to the size with the staging area
    const int rc_lds = set_max_dynamic_lds(reinterpret_cast<const void*>(topk_stream_kernel),
                                           (320 + kTopkLdsKeys) * (int)sizeof(uint32_t));
    if (rc_lds != DAPQ_OK) return rc_lds;
    hipLaunchKernelGGL(topk_stream_kernel, grid, dim3(kTopkThreads), lds_bytes, st, p);
    DAPQ_HIP_LAUNCH_CHECK("topk_stream_kernel");
  }
  return DAPQ_OK;
}

extern "C" DAPQ_API int dapq_pool_topk(const dapq_shape* shape, const float* scores, int32_t width, int32_t budget,
                                       const int32_t* budget_per_seq, int32_t* idx, int32_t* count, float* pooled,
                                       void* stream) {
  int rc = topk_common_checks(shape, scores, budget, idx, count);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(width >= 1 && width <= 63 && (width & 1) == 1, DAPQ_ERR_INVALID_ARG,
               "width (%d) must be odd and in [1, 63]", width);
  DAPQ_REQUIRE(pooled != scores, DAPQ_ERR_INVALID_ARG, "pooled must not alias scores");
  // one kernel if every head fits the register variant and the window is one of the compiled radii
  const int64_t longest = shape->cu_seqlens == nullptr ? shape->total_tokens / shape->batch : shape->total_tokens;
  const bool fused = width <= 9 && longest <= 64 * kTopkThreads;
  if (!fused) {
    DAPQ_REQUIRE(pooled != nullptr, DAPQ_ERR_UNSUPPORTED,
                 "width %d / head length %lld need the two-kernel path: pass a pooled buffer", width, (long long)longest);
    if ((rc = dapq_pool(shape, scores, pooled, width, stream)) != DAPQ_OK) return rc;
    return dapq_topk(shape, pooled, budget, budget_per_seq, idx, count, nullptr, 0, stream);
  }
  TopkParams p;
  p.pooled = scores;
  p.pooled_out = pooled;
  p.cu_seqlens = shape->cu_seqlens;
  p.budget_per_seq = budget_per_seq;
  p.idx = idx;
  p.count = count;
  p.total_tokens = shape->total_tokens;
  p.batch = shape->batch;
  p.n_kv_heads = shape->n_kv_heads;
  p.budget = budget;
  p.min_len = 0;
  p.max_len = INT32_MAX;
  const RegVariant variant = reg_variant_for(longest);
  const dim3 grid((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers);
  hipStream_t st = static_cast<hipStream_t>(stream);
  switch (width / 2) {
    case 0: launch_reg<0>(variant, grid, st, p); break;
    case 1: launch_reg<1>(variant, grid, st, p); break;
    case 2: launch_reg<2>(variant, grid, st, p); break;
    case 3: launch_reg<3>(variant, grid, st, p); break;
    default: launch_reg<4>(variant, grid, st, p); break;
  }
  DAPQ_HIP_LAUNCH_CHECK("topk_reg_kernel");
  return DAPQ_OK;
}
