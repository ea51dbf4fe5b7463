// Error reporting, shape validation and the launch plan of libdapq (host code only).
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "dapq_internal.h"

namespace dapq {

char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

int set_max_dynamic_lds(const void* kernel, int bytes) {
  struct Entry { const void* kernel; int device; };
  static std::mutex mu;
  static std::vector<Entry> done;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(DAPQ_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& it : done)
    if (it.kernel == kernel && it.device == dev) return DAPQ_OK;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return fail(DAPQ_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
  done.push_back({kernel, dev});
  return DAPQ_OK;
}

static bool stride_ok(int64_t s) { return s >= 0 && (s % 8) == 0; }

int check_shape(const dapq_shape* s, bool need_q, bool need_k, bool need_v) {
  DAPQ_REQUIRE(s != nullptr, DAPQ_ERR_INVALID_ARG, "shape is NULL");
  DAPQ_REQUIRE(s->n_layers >= 1 && s->batch >= 1, DAPQ_ERR_INVALID_ARG,
               "n_layers (%d) and batch (%d) must be >= 1", s->n_layers, s->batch);
  DAPQ_REQUIRE(s->n_kv_heads >= 1 && s->n_q_heads >= 1 && s->n_q_heads % s->n_kv_heads == 0,
               DAPQ_ERR_INVALID_ARG, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)",
               s->n_q_heads, s->n_kv_heads);
  DAPQ_REQUIRE(s->n_pseudo >= 1, DAPQ_ERR_INVALID_ARG, "n_pseudo (%d) must be >= 1", s->n_pseudo);
  DAPQ_REQUIRE(s->total_tokens >= 0, DAPQ_ERR_INVALID_ARG, "total_tokens is negative");
  DAPQ_REQUIRE(s->head_dim == kHeadDim, DAPQ_ERR_UNSUPPORTED, "head_dim %d is not supported (128 only)",
               s->head_dim);
  DAPQ_REQUIRE(s->total_tokens < (int64_t)1 << 31, DAPQ_ERR_UNSUPPORTED,
               "total_tokens %lld does not fit the int32 token offsets", (long long)s->total_tokens);
  DAPQ_REQUIRE((int64_t)s->n_layers * s->n_kv_heads <= 65535, DAPQ_ERR_UNSUPPORTED,
               "n_layers * n_kv_heads (%lld) exceeds the grid limit 65535",
               (long long)s->n_layers * s->n_kv_heads);
  if (s->cu_seqlens == nullptr) {
    DAPQ_REQUIRE(s->total_tokens % s->batch == 0, DAPQ_ERR_INVALID_ARG,
                 "dense batch: total_tokens (%lld) is not a multiple of batch (%d)",
                 (long long)s->total_tokens, s->batch);
  }
  if (need_q) {
    DAPQ_REQUIRE(stride_ok(s->q_stride_layer) && stride_ok(s->q_stride_seq) && stride_ok(s->q_stride_head) &&
                     stride_ok(s->q_stride_row) && s->q_stride_row >= kHeadDim,
                 DAPQ_ERR_UNSUPPORTED, "q strides must be non-negative multiples of 8 elements (row >= 128)");
    DAPQ_REQUIRE(isfinite(s->scale) && s->scale > 0.0f, DAPQ_ERR_INVALID_ARG, "scale must be finite and > 0");
  }
  if (need_k) {
    DAPQ_REQUIRE(stride_ok(s->k_stride_layer) && stride_ok(s->k_stride_seq) && stride_ok(s->k_stride_head) &&
                     stride_ok(s->k_stride_token) && s->k_stride_token >= kHeadDim,
                 DAPQ_ERR_UNSUPPORTED, "k strides must be non-negative multiples of 8 elements (token >= 128)");
    DAPQ_REQUIRE(s->k_stride_token < ((int64_t)1 << 26), DAPQ_ERR_UNSUPPORTED,
                 "k_stride_token (%lld) must be below 2^26 elements", (long long)s->k_stride_token);
  }
  if (need_v) {
    DAPQ_REQUIRE(stride_ok(s->v_stride_layer) && stride_ok(s->v_stride_seq) && stride_ok(s->v_stride_head) &&
                     stride_ok(s->v_stride_token) && s->v_stride_token >= kHeadDim,
                 DAPQ_ERR_UNSUPPORTED, "v strides must be non-negative multiples of 8 elements (token >= 128)");
  }
  return DAPQ_OK;
}

int make_score_plan(const dapq_shape* s, ScorePlan* p) {
  const int g = s->n_q_heads / s->n_kv_heads;
  const int64_t rows64 = (int64_t)g * s->n_pseudo;
  DAPQ_REQUIRE(rows64 <= (1 << 20), DAPQ_ERR_UNSUPPORTED, "group * n_pseudo = %lld rows per KV head is too large",
               (long long)rows64);
  p->rows = (int)rows64;
  const int64_t heads = (int64_t)s->n_layers * s->n_kv_heads;
  // one wave per (chunk, row group): a group is up to 256 rows, all in the wave's registers
  p->n_groups = (p->rows + 255) / 256;
  p->row_blocks = p->rows <= 64 ? 2 : (p->rows <= 128 ? 4 : 8);
  p->rows_pad = p->n_groups * p->row_blocks * 32;

  // Keys per wave.  The machine runs kWaveSlots waves at a time, each for as long as its chunk; a
  // wave pays a fixed start-up (Q fragments, ring fill) worth about kStartKeys keys.  Dense batches
  // run in whole rounds of equal chunks: pick the chunk with the shortest rounds x (chunk +
  // start-up).  Ragged batches (lengths unknown on the host) are handed out chunk by chunk to
  // persistent waves, so the cost is the work per slot plus half a chunk of tail imbalance on average.
  constexpr int64_t kWaveSlots = 1024, kStartKeys = 160;
  const int64_t units_per_chunk_row = heads * p->n_groups;
  int chunk = kMinChunkKeys;
  int64_t best = INT64_MAX;
  for (int c = kMaxChunkKeys; c >= kMinChunkKeys; c /= 2) {
    int64_t cost;
    if (s->cu_seqlens == nullptr) {
      const int64_t L = s->total_tokens / s->batch;
      const int64_t units = units_per_chunk_row * s->batch * ((L + c - 1) / c);
      const int64_t rounds = (units + kWaveSlots - 1) / kWaveSlots;
      cost = rounds * ((L < c ? L : c) + kStartKeys);
    } else {
      const int64_t chunks = (s->total_tokens + c - 1) / c + s->batch / 2;
      const int64_t units = units_per_chunk_row * chunks;
      cost = (units_per_chunk_row * s->total_tokens + units * kStartKeys) / kWaveSlots + c / 2;
    }
    if (cost < best) {
      best = cost;
      chunk = c;
    }
  }
  p->chunk_keys = chunk;
  if (s->cu_seqlens == nullptr) {
    const int64_t L = s->total_tokens / s->batch;
    p->max_chunks = (int64_t)s->batch * ((L + chunk - 1) / chunk);
  } else {
    p->max_chunks = (s->total_tokens + chunk - 1) / chunk + s->batch;
  }
  if (p->max_chunks < 1) p->max_chunks = 1;
  DAPQ_REQUIRE(p->max_chunks < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED, "too many key chunks");
  DAPQ_REQUIRE(p->n_groups <= 65535, DAPQ_ERR_UNSUPPORTED, "too many query rows per KV head");

  size_t off = 0;
  p->off_cu_chunks = off;
  off = align_up(off + sizeof(int32_t) * ((size_t)s->batch + 1), 256);
  p->off_work = off;  // ticket counter of a ragged batch's work list
  off += 256;
  p->off_parts = off;
  off = align_up(off + sizeof(float) * 2 * (size_t)heads * (size_t)p->max_chunks * p->rows_pad, 256);
  p->off_lse2 = off;
  off = align_up(off + sizeof(float) * (size_t)s->n_layers * s->batch * s->n_q_heads * s->n_pseudo, 256);
  p->off_partial = off;
  if (p->n_groups > 1) off = align_up(off + sizeof(float) * (size_t)(p->n_groups - 1) * (size_t)heads * (size_t)s->total_tokens, 256);
  p->total_bytes = off;
  return DAPQ_OK;
}

}  // namespace dapq

extern "C" DAPQ_API size_t dapq_workspace_bytes(const dapq_shape* shape) {
  if (dapq::check_shape(shape, false, false, false) != DAPQ_OK) return 0;
  dapq::ScorePlan plan;
  if (dapq::make_score_plan(shape, &plan) != DAPQ_OK) return 0;
  return plan.total_bytes;
}

extern "C" DAPQ_API const char* dapq_last_error(void) { return dapq::error_buffer(); }
