// Importance scoring (Sec. 4.2, S(j) = sum_i Attention(q_i, k_j); Attention = softmax over the
// prompt keys, App. C.1) as two streaming passes over K for gfx950.
//
//   pass 1  (score_pass1_kernel + score_combine_kernel): lse2[row] = log2 sum_j 2^(c * q_row.k_j)
//   pass 2  (score_pass2_kernel):  S(j) = sum_rows 2^(c * q_row.k_j - lse2[row])
// with c = scale * log2(e).  "rows" are the R = g*N pseudo-query rows of the g query heads that
// share one KV head.  Nothing of size N x L_p is ever stored.
//
// Work split.  One workgroup = 4 waves walks a chunk of keys of one (layer, sequence, KV head).
// Keys stream through LDS in tiles of 128 rows (32 KB, double buffered, 16-byte chunks XOR-swizzled
// so that the MFMA operand reads are bank-conflict free); each wave keeps a 64-row slab of Q in
// registers for the whole chunk as MFMA operand fragments and runs v_mfma_f32_32x32x16_bf16 against
// every 32-key sub-block.  RW waves hold different slabs; the other 4/RW waves split the keys.
//   pass 1 uses D[key][query] (K as the A operand): a lane owns one query column, the reduction
//           over keys stays inside the lane;
//   pass 2 uses D[query][key] (Q as the A operand): a lane owns one key column, the reduction over
//           query rows stays inside the lane, and lse2 of the lane's 16 rows sits in registers.
// Pass 1 does not track a running maximum: it exponentiates against a per-row reference logit taken
// from the first sub-block (2^x has 127 binades of headroom above it) and only if a sum overflows
// redoes the chunk with a conventional online maximum.
#include <math.h>

#include "dapq_internal.h"

namespace dapq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct ScoreParams {
  const uint16_t* q;
  const uint16_t* k;
  const int32_t* cu_seqlens;  // NULL = dense
  int32_t* cu_chunks;         // [batch+1] prefix of per-sequence chunk counts (ragged only)
  float2* parts;              // [layer*Hkv][max_chunks][KW][rows_pad] (reference, sum) in the log2 domain
  float* lse2;                // [layer][batch][Hq][N]
  float* scores;              // [layer][Hkv][total_tokens]
  int64_t k_stride_layer, k_stride_seq, k_stride_head, k_stride_token;
  int64_t q_stride_layer, q_stride_seq, q_stride_head, q_stride_row;
  int64_t total_tokens;
  int32_t n_layers, batch, n_q_heads, n_kv_heads, group, n_pseudo;
  int32_t rows, rows_pad, n_super, chunk_keys, max_chunks;
  float c;  // scale * log2(e)
};

constexpr int kThreads = 256;
constexpr int kTileBytes = kTileKeys * kHeadDim * 2;  // 32 KB
constexpr int kLdsScore = 2 * kTileBytes;

// Which (sequence, chunk) a workgroup works on.
struct Work {
  int seq;
  int64_t tok0;  // packed token index of the first key of the chunk
  int key0;      // first key of the chunk inside the sequence
  int nkeys;     // keys in the chunk (<= chunk_keys), 0 = nothing to do
  int seq_len;
};

__device__ __forceinline__ Work locate(const ScoreParams& p, int gchunk) {
  Work w;
  w.nkeys = 0;
  if (p.cu_seqlens == nullptr) {
    const int L = (int)(p.total_tokens / p.batch);
    const int cps = (L + p.chunk_keys - 1) / p.chunk_keys;
    if (cps == 0) return w;
    w.seq = gchunk / cps;
    if (w.seq >= p.batch) return w;
    w.key0 = (gchunk - w.seq * cps) * p.chunk_keys;
    w.tok0 = (int64_t)w.seq * L + w.key0;
    w.seq_len = L;
  } else {
    if (gchunk >= p.cu_chunks[p.batch]) return w;
    int lo = 0, hi = p.batch;  // largest b with cu_chunks[b] <= gchunk
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.cu_chunks[mid] <= gchunk) lo = mid; else hi = mid;
    }
    w.seq = lo;
    const int start = p.cu_seqlens[lo];
    w.seq_len = p.cu_seqlens[lo + 1] - start;
    w.key0 = (gchunk - p.cu_chunks[lo]) * p.chunk_keys;
    w.tok0 = (int64_t)start + w.key0;
  }
  const int left = w.seq_len - w.key0;
  w.nkeys = left < p.chunk_keys ? left : p.chunk_keys;
  if (w.nkeys < 0) w.nkeys = 0;
  return w;
}

// Coalesced 16-byte loads of one 128-key tile: thread t takes chunk (t & 15) of keys (t >> 4) + 16*i.
__device__ __forceinline__ void tile_load(uint4 (&st)[8], const uint16_t* kbase, int64_t stride_token,
                                          int tile_key0, int nkeys, int tid) {
  const int ch = tid & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int key = (tid >> 4) + 16 * i;
    const int gk = tile_key0 + key;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (gk < nkeys) v = *reinterpret_cast<const uint4*>(kbase + (int64_t)gk * stride_token + ch * 8);
    st[i] = v;
  }
}

// LDS position of 16-byte chunk `ch` of tile row `key`: rows are 256 B apart, chunks XOR-swizzled by
// the row so that 16 consecutive rows reading the same logical chunk hit 16 different bank groups.
__device__ __forceinline__ int lds_chunk_index(int key, int ch) { return key * 16 + (ch ^ (key & 15)); }

__device__ __forceinline__ void tile_store(uint4* buf, const uint4 (&st)[8], int tid) {
  const int ch = tid & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int key = (tid >> 4) + 16 * i;
    buf[lds_chunk_index(key, ch)] = st[i];
  }
}

// MFMA operand fragments of one 32-row sub-block held in LDS: fragment s of lane (n, h) is the
// 8 channels [(2s+h)*8, +8) of row n.
__device__ __forceinline__ void frag_from_lds(bf16x8 (&f)[8], const uint4* buf, int sub, int n, int h) {
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const uint4 v = buf[lds_chunk_index(sub * 32 + n, 2 * s + h)];
    f[s] = __builtin_bit_cast(bf16x8, v);
  }
}

// The same fragments for a 32-row block of Q read straight from global memory; rows >= p.rows are zero.
__device__ __forceinline__ void frag_from_q(bf16x8 (&f)[8], const ScoreParams& p, const uint16_t* qbase, int row,
                                            int h) {
  uint4 v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) v[s] = make_uint4(0u, 0u, 0u, 0u);
  if (row < p.rows) {
    const int head = row / p.n_pseudo, i = row - head * p.n_pseudo;
    const uint16_t* src = qbase + (int64_t)head * p.q_stride_head + (int64_t)i * p.q_stride_row;
#pragma unroll
    for (int s = 0; s < 8; ++s) v[s] = *reinterpret_cast<const uint4*>(src + (2 * s + h) * 8);
  }
#pragma unroll
  for (int s = 0; s < 8; ++s) f[s] = __builtin_bit_cast(bf16x8, v[s]);
}

__device__ __forceinline__ float xhalf(float v) { return __shfl_xor(v, 32, 64); }

// Row of the 32x32 MFMA result held in accumulator register v of a lane in half h.
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// ---------------------------------------------------------------------------------------------
// Pass 1
// ---------------------------------------------------------------------------------------------
template <int RW, bool SAFE>
__device__ __forceinline__ bool pass1_chunk(const ScoreParams& p, const Work& w, const uint16_t* kbase,
                                            const bf16x8 (&qf)[2][8], uint4* lds, float (&ref)[2], float (&z)[2]) {
  constexpr int KW = 4 / RW;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
  const int kw = wave / RW;
  const float c = p.c;
  const int ntiles = (w.nkeys + kTileKeys - 1) / kTileKeys;
  bool first = !SAFE;
  ref[0] = ref[1] = -INFINITY;
  z[0] = z[1] = 0.0f;

  uint4 st[8];
  tile_load(st, kbase, p.k_stride_token, 0, w.nkeys, tid);
  for (int t = 0; t < ntiles; ++t) {
    uint4* buf = lds + (t & 1) * (kTileBytes / 16);
    tile_store(buf, st, tid);
    __syncthreads();
    if (t + 1 < ntiles) tile_load(st, kbase, p.k_stride_token, (t + 1) * kTileKeys, w.nkeys, tid);
    const int tile_key0 = t * kTileKeys;
    const bool full = tile_key0 + kTileKeys <= w.nkeys;
#pragma unroll 1
    for (int sub = kw; sub < 4; sub += KW) {
      const int sub_key0 = tile_key0 + sub * 32;
      if (sub_key0 >= w.nkeys) break;
      bf16x8 kf[8];
      frag_from_lds(kf, buf, sub, n, h);
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        f32x16 acc = {0};
#pragma unroll
        for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[rb][s], acc, 0, 0, 0);
        if (!full) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (sub_key0 + acc_row(v, h) >= w.nkeys) acc[v] = -INFINITY;
        }
        if (SAFE || first) {
          float m = acc[0];
#pragma unroll
          for (int v = 1; v < 16; ++v) m = fmaxf(m, acc[v]);
          m = fmaxf(m, xhalf(m)) * c;
          if (SAFE) {
            const float mnew = fmaxf(ref[rb], m);
            z[rb] *= __builtin_amdgcn_exp2f(ref[rb] - mnew);
            ref[rb] = mnew;
          } else {
            ref[rb] = m;
          }
        }
        const float nref = -ref[rb];
        float sum = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[v], c, nref));
        z[rb] += sum;
      }
      first = false;
    }
  }
  __syncthreads();  // every wave is done with the last tile before a caller reuses the buffers
  // a sum that is not finite means a logit sat more than ~127 binades above the reference
  const bool bad = !(z[0] < INFINITY) || !(z[1] < INFINITY);
  return bad;
}

template <int RW>
__global__ __launch_bounds__(kThreads, 2) void score_pass1_kernel(ScoreParams p) {
  extern __shared__ uint4 lds[];
  constexpr int KW = 4 / RW;
  const Work w = locate(p, blockIdx.x);
  if (w.nkeys == 0) return;
  const int layer = blockIdx.z / p.n_kv_heads, kv = blockIdx.z - layer * p.n_kv_heads;
  const int sg = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
  const int rw = wave % RW, kw = wave / RW;
  const int row0 = (sg * RW + rw) * 64;

  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)w.seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = p.k + (int64_t)layer * p.k_stride_layer + (int64_t)w.seq * p.k_stride_seq +
                          (int64_t)kv * p.k_stride_head + w.tok0 * p.k_stride_token;
  bf16x8 qf[2][8];
  frag_from_q(qf[0], p, qbase, row0 + n, h);
  frag_from_q(qf[1], p, qbase, row0 + 32 + n, h);

  float ref[2], z[2];
  bool bad = pass1_chunk<RW, false>(p, w, kbase, qf, lds, ref, z);
  if (__syncthreads_or(bad ? 1 : 0)) pass1_chunk<RW, true>(p, w, kbase, qf, lds, ref, z);

  // the two lane halves hold different keys of the same query
  const float z0 = z[0] + xhalf(z[0]);
  const float z1 = z[1] + xhalf(z[1]);
  if (h == 0) {
    float2* out = p.parts + (((int64_t)blockIdx.z * p.max_chunks + blockIdx.x) * KW + kw) * p.rows_pad + row0;
    out[n] = make_float2(ref[0], z0);
    out[32 + n] = make_float2(ref[1], z1);
  }
}

// Per-sequence prefix of chunk counts for ragged batches (tiny, one block).
__global__ void score_chunk_prefix_kernel(const int32_t* cu_seqlens, int32_t* cu_chunks, int batch, int chunk_keys) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int acc = 0;
    cu_chunks[0] = 0;
    for (int b = 0; b < batch; ++b) {
      const int L = cu_seqlens[b + 1] - cu_seqlens[b];
      acc += L > 0 ? (L + chunk_keys - 1) / chunk_keys : 0;
      cu_chunks[b + 1] = acc;
    }
  }
}

// Merge the per-chunk (reference, sum) pairs of a row: lse2 = log2 sum_c z_c 2^(ref_c).
__global__ void score_combine_kernel(ScoreParams p, int key_waves) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)p.n_layers * p.batch * p.n_q_heads * p.n_pseudo;
  if (gid >= total) return;
  const int i = (int)(gid % p.n_pseudo);
  const int hq = (int)((gid / p.n_pseudo) % p.n_q_heads);
  const int b = (int)((gid / ((int64_t)p.n_pseudo * p.n_q_heads)) % p.batch);
  const int layer = (int)(gid / ((int64_t)p.n_pseudo * p.n_q_heads * p.batch));
  const int kv = hq / p.group;
  const int row = (hq - kv * p.group) * p.n_pseudo + i;
  int c0, c1;
  if (p.cu_seqlens == nullptr) {
    const int L = (int)(p.total_tokens / p.batch);
    const int cps = (L + p.chunk_keys - 1) / p.chunk_keys;
    c0 = b * cps;
    c1 = c0 + cps;
  } else {
    c0 = p.cu_chunks[b];
    c1 = p.cu_chunks[b + 1];
  }
  const float2* src = p.parts + ((int64_t)(layer * p.n_kv_heads + kv) * p.max_chunks) * key_waves * p.rows_pad + row;
  float m = -INFINITY;
  for (int64_t e = (int64_t)c0 * key_waves; e < (int64_t)c1 * key_waves; ++e) {
    const float2 v = src[e * p.rows_pad];
    if (v.y > 0.0f) m = fmaxf(m, v.x + log2f(v.y));
  }
  float s = 0.0f;
  for (int64_t e = (int64_t)c0 * key_waves; e < (int64_t)c1 * key_waves; ++e) {
    const float2 v = src[e * p.rows_pad];
    if (v.y > 0.0f) s += exp2f(v.x + log2f(v.y) - m);
  }
  p.lse2[gid] = (s > 0.0f) ? m + log2f(s) : 0.0f;
}

// ---------------------------------------------------------------------------------------------
// Pass 2
// ---------------------------------------------------------------------------------------------
template <int RW>
__global__ __launch_bounds__(kThreads, 2) void score_pass2_kernel(ScoreParams p) {
  extern __shared__ uint4 lds[];
  constexpr int KW = 4 / RW;
  constexpr int NSUB = 4 / KW;  // sub-blocks of a tile per wave
  float* red = reinterpret_cast<float*>(lds + kLdsScore / 16);  // [RW][128] partial column sums
  const Work w = locate(p, blockIdx.x);
  if (w.nkeys == 0) return;
  const int layer = blockIdx.z / p.n_kv_heads, kv = blockIdx.z - layer * p.n_kv_heads;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
  const int rw = wave % RW, kw = wave / RW;
  const float c = p.c;

  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)w.seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = p.k + (int64_t)layer * p.k_stride_layer + (int64_t)w.seq * p.k_stride_seq +
                          (int64_t)kv * p.k_stride_head + w.tok0 * p.k_stride_token;
  const float* lse = p.lse2 + (((int64_t)layer * p.batch + w.seq) * p.n_q_heads + (int64_t)kv * p.group) * p.n_pseudo;
  float* out = p.scores + ((int64_t)layer * p.n_kv_heads + kv) * p.total_tokens + w.tok0;

  // Q slab and the normalisers of its rows; reloaded per super-group when R > RW*64.
  bf16x8 qf[2][8];
  float nb[2][16];  // -lse2 of the lane's accumulator rows; -inf for padding rows, which then add 0
  auto load_slab = [&](int sg) {
    const int row0 = (sg * RW + rw) * 64;
    frag_from_q(qf[0], p, qbase, row0 + n, h);
    frag_from_q(qf[1], p, qbase, row0 + 32 + n, h);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = row0 + rb * 32 + acc_row(v, h);
        nb[rb][v] = row < p.rows ? -lse[row] : -INFINITY;  // rows are laid out head-major: row = head*N + i
      }
  };
  if (p.n_super == 1) load_slab(0);

  const int ntiles = (w.nkeys + kTileKeys - 1) / kTileKeys;
  uint4 st[8];
  tile_load(st, kbase, p.k_stride_token, 0, w.nkeys, tid);
  for (int t = 0; t < ntiles; ++t) {
    uint4* buf = lds + (t & 1) * (kTileBytes / 16);
    tile_store(buf, st, tid);
    __syncthreads();
    if (t + 1 < ntiles) tile_load(st, kbase, p.k_stride_token, (t + 1) * kTileKeys, w.nkeys, tid);
    const int tile_key0 = t * kTileKeys;

    float col[NSUB];
#pragma unroll
    for (int j = 0; j < NSUB; ++j) col[j] = 0.0f;
    for (int sg = 0; sg < p.n_super; ++sg) {
      if (p.n_super > 1) load_slab(sg);
#pragma unroll
      for (int j = 0; j < NSUB; ++j) {
        const int sub = kw + j * KW;
        if (tile_key0 + sub * 32 >= w.nkeys) continue;
        bf16x8 kf[8];
        frag_from_lds(kf, buf, sub, n, h);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          f32x16 acc = {0};
#pragma unroll
          for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][s], kf[s], acc, 0, 0, 0);
          float sum = 0.0f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[v], c, nb[rb][v]));
          col[j] += sum;
        }
      }
    }
    // lane halves hold different query rows of the same key; then add the RW slabs through LDS
#pragma unroll
    for (int j = 0; j < NSUB; ++j) {
      const float v = col[j] + xhalf(col[j]);
      if (h == 0) red[rw * kTileKeys + (kw + j * KW) * 32 + n] = v;
    }
    __syncthreads();
    if (tid < kTileKeys && tile_key0 + tid < w.nkeys) {
      float s = red[tid];
#pragma unroll
      for (int r = 1; r < RW; ++r) s += red[r * kTileKeys + tid];
      out[tile_key0 + tid] = s;
    }
  }
}

template <typename F>
int set_lds(F kernel, int bytes) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return fail(DAPQ_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
  return DAPQ_OK;
}

int fill_params(const dapq_shape* s, const ScorePlan& plan, ScoreParams* p) {
  p->cu_seqlens = s->cu_seqlens;
  p->k_stride_layer = s->k_stride_layer; p->k_stride_seq = s->k_stride_seq;
  p->k_stride_head = s->k_stride_head; p->k_stride_token = s->k_stride_token;
  p->q_stride_layer = s->q_stride_layer; p->q_stride_seq = s->q_stride_seq;
  p->q_stride_head = s->q_stride_head; p->q_stride_row = s->q_stride_row;
  p->total_tokens = s->total_tokens;
  p->n_layers = s->n_layers; p->batch = s->batch; p->n_q_heads = s->n_q_heads; p->n_kv_heads = s->n_kv_heads;
  p->group = s->n_q_heads / s->n_kv_heads; p->n_pseudo = s->n_pseudo;
  p->rows = plan.rows; p->rows_pad = plan.rows_pad; p->n_super = plan.n_super;
  p->chunk_keys = plan.chunk_keys; p->max_chunks = (int32_t)plan.max_chunks;
  p->c = s->scale * 1.4426950408889634f;
  return DAPQ_OK;
}

int aligned16(const void* ptr, const char* name) {
  DAPQ_REQUIRE(ptr != nullptr, DAPQ_ERR_INVALID_ARG, "%s is NULL", name);
  DAPQ_REQUIRE((reinterpret_cast<uintptr_t>(ptr) & 15) == 0, DAPQ_ERR_UNSUPPORTED, "%s is not 16-byte aligned", name);
  return DAPQ_OK;
}

int launch_stats(const dapq_shape* s, const ScorePlan& plan, ScoreParams p, hipStream_t stream) {
  if (s->cu_seqlens != nullptr) {
    hipLaunchKernelGGL(score_chunk_prefix_kernel, dim3(1), dim3(64), 0, stream, s->cu_seqlens, p.cu_chunks, s->batch,
                       plan.chunk_keys);
    DAPQ_HIP_LAUNCH_CHECK("score_chunk_prefix_kernel");
  }
  const dim3 grid((unsigned)plan.max_chunks, (unsigned)plan.n_super, (unsigned)(s->n_layers * s->n_kv_heads));
  int rc = DAPQ_OK;
  switch (plan.row_waves) {
    case 1:
      if ((rc = set_lds(score_pass1_kernel<1>, kLdsScore)) != DAPQ_OK) return rc;
      hipLaunchKernelGGL(score_pass1_kernel<1>, grid, dim3(kThreads), kLdsScore, stream, p);
      break;
    case 2:
      if ((rc = set_lds(score_pass1_kernel<2>, kLdsScore)) != DAPQ_OK) return rc;
      hipLaunchKernelGGL(score_pass1_kernel<2>, grid, dim3(kThreads), kLdsScore, stream, p);
      break;
    default:
      if ((rc = set_lds(score_pass1_kernel<4>, kLdsScore)) != DAPQ_OK) return rc;
      hipLaunchKernelGGL(score_pass1_kernel<4>, grid, dim3(kThreads), kLdsScore, stream, p);
      break;
  }
  DAPQ_HIP_LAUNCH_CHECK("score_pass1_kernel");
  const int64_t rows_total = (int64_t)s->n_layers * s->batch * s->n_q_heads * s->n_pseudo;
  hipLaunchKernelGGL(score_combine_kernel, dim3((unsigned)((rows_total + 255) / 256)), dim3(256), 0, stream, p,
                     plan.key_waves);
  DAPQ_HIP_LAUNCH_CHECK("score_combine_kernel");
  return DAPQ_OK;
}

int launch_accumulate(const dapq_shape* s, const ScorePlan& plan, ScoreParams p, hipStream_t stream) {
  if (s->cu_seqlens != nullptr) {
    // pass 2 can be called on its own: rebuild the chunk prefix it walks
    hipLaunchKernelGGL(score_chunk_prefix_kernel, dim3(1), dim3(64), 0, stream, s->cu_seqlens, p.cu_chunks, s->batch,
                       plan.chunk_keys);
    DAPQ_HIP_LAUNCH_CHECK("score_chunk_prefix_kernel");
  }
  const dim3 grid((unsigned)plan.max_chunks, 1, (unsigned)(s->n_layers * s->n_kv_heads));
  const int lds_bytes = kLdsScore + 4 * kTileKeys * (int)sizeof(float);
  int rc = DAPQ_OK;
  switch (plan.row_waves) {
    case 1:
      if ((rc = set_lds(score_pass2_kernel<1>, lds_bytes)) != DAPQ_OK) return rc;
      hipLaunchKernelGGL(score_pass2_kernel<1>, grid, dim3(kThreads), lds_bytes, stream, p);
      break;
    case 2:
      if ((rc = set_lds(score_pass2_kernel<2>, lds_bytes)) != DAPQ_OK) return rc;
      hipLaunchKernelGGL(score_pass2_kernel<2>, grid, dim3(kThreads), lds_bytes, stream, p);
      break;
    default:
      if ((rc = set_lds(score_pass2_kernel<4>, lds_bytes)) != DAPQ_OK) return rc;
      hipLaunchKernelGGL(score_pass2_kernel<4>, grid, dim3(kThreads), lds_bytes, stream, p);
      break;
  }
  DAPQ_HIP_LAUNCH_CHECK("score_pass2_kernel");
  return DAPQ_OK;
}

}  // namespace
}  // namespace dapq

using namespace dapq;

static int check_workspace(void* workspace, size_t workspace_bytes, const ScorePlan& plan) {
  DAPQ_REQUIRE(workspace != nullptr, DAPQ_ERR_INVALID_ARG, "workspace is NULL");
  DAPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, DAPQ_ERR_UNSUPPORTED,
               "workspace is not 256-byte aligned");
  DAPQ_REQUIRE(workspace_bytes >= plan.total_bytes, DAPQ_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed",
               workspace_bytes, plan.total_bytes);
  return DAPQ_OK;
}

extern "C" DAPQ_API int dapq_score_stats(const dapq_shape* shape, const void* q, const void* k, float* lse2, void* workspace,
                                size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape, true, true, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  if ((rc = aligned16(q, "q")) != DAPQ_OK) return rc;
  if ((rc = aligned16(k, "k")) != DAPQ_OK) return rc;
  DAPQ_REQUIRE(lse2 != nullptr, DAPQ_ERR_INVALID_ARG, "lse2 is NULL");
  if ((rc = check_workspace(workspace, workspace_bytes, plan)) != DAPQ_OK) return rc;
  ScoreParams p;
  fill_params(shape, plan, &p);
  char* ws = static_cast<char*>(workspace);
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.cu_chunks = reinterpret_cast<int32_t*>(ws + plan.off_cu_chunks);
  p.parts = reinterpret_cast<float2*>(ws + plan.off_parts);
  p.lse2 = lse2;
  p.scores = nullptr;
  return launch_stats(shape, plan, p, static_cast<hipStream_t>(stream));
}

extern "C" DAPQ_API int dapq_score_accumulate(const dapq_shape* shape, const void* q, const void* k, const float* lse2,
                                     float* scores, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape, true, true, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  if ((rc = aligned16(q, "q")) != DAPQ_OK) return rc;
  if ((rc = aligned16(k, "k")) != DAPQ_OK) return rc;
  DAPQ_REQUIRE(lse2 != nullptr, DAPQ_ERR_INVALID_ARG, "lse2 is NULL");
  DAPQ_REQUIRE(scores != nullptr, DAPQ_ERR_INVALID_ARG, "scores is NULL");
  if ((rc = check_workspace(workspace, workspace_bytes, plan)) != DAPQ_OK) return rc;
  ScoreParams p;
  fill_params(shape, plan, &p);
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.cu_chunks = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + plan.off_cu_chunks);
  p.parts = nullptr;
  p.lse2 = const_cast<float*>(lse2);
  p.scores = scores;
  return launch_accumulate(shape, plan, p, static_cast<hipStream_t>(stream));
}

extern "C" DAPQ_API int dapq_score(const dapq_shape* shape, const void* q, const void* k, float* scores, void* workspace,
                          size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape, true, true, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  DAPQ_REQUIRE(scores != nullptr, DAPQ_ERR_INVALID_ARG, "scores is NULL");
  if ((rc = check_workspace(workspace, workspace_bytes, plan)) != DAPQ_OK) return rc;
  float* lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan.off_lse2);
  if ((rc = dapq_score_stats(shape, q, k, lse2, workspace, workspace_bytes, stream)) != DAPQ_OK) return rc;
  return dapq_score_accumulate(shape, q, k, lse2, scores, workspace, workspace_bytes, stream);
}
