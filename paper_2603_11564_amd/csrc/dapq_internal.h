// Host-side helpers shared by the libdapq translation units: error reporting, argument checks and
// the launch plan (chunking of the key axis, workspace carving).  No device code here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "dapq.h"

namespace dapq {

// Thread-local message returned by dapq_last_error().
char* error_buffer();
int fail(int code, const char* fmt, ...);

#define DAPQ_REQUIRE(cond, code, ...)            \
  do {                                           \
    if (!(cond)) return ::dapq::fail((code), __VA_ARGS__); \
  } while (0)

#define DAPQ_HIP_LAUNCH_CHECK(what)                                                          \
  do {                                                                                       \
    hipError_t e__ = hipGetLastError();                                                      \
    if (e__ != hipSuccess) return ::dapq::fail(DAPQ_ERR_HIP, "%s: %s", (what), hipGetErrorString(e__)); \
  } while (0)

constexpr int kHeadDim = 128;
constexpr int kMinChunkKeys = 128;      // fewest keys one wave of a score pass walks over
constexpr int kMaxChunkKeys = 1 << 16;  // most

// How the score passes split the work; a pure function of the shape so that
// dapq_workspace_bytes() and the launchers agree.
struct ScorePlan {
  int rows;        // R = (H_q/H_kv) * N query rows scored against every key of a KV head
  int n_groups;    // row groups of row_blocks * 32 rows, one wave each per chunk
  int row_blocks;  // 32-row blocks per wave (2, 4 or 8)
  int rows_pad;    // n_groups * row_blocks * 32
  int chunk_keys;  // keys per wave (a power of two)
  int64_t max_chunks;  // grid size along the key axis: upper bound on sum_b ceil(L_b / chunk_keys)
  // workspace carving (byte offsets)
  size_t off_cu_chunks, off_work, off_parts, off_lse2, off_partial, total_bytes;
};

// Validates the fields every entry point relies on.  need_q / need_k / need_v say which stride
// groups must be usable.  Returns DAPQ_OK or sets the error and returns its code.
int check_shape(const dapq_shape* s, bool need_q, bool need_k, bool need_v);
int make_score_plan(const dapq_shape* s, ScorePlan* plan);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Raises a kernel's dynamic-LDS limit to `bytes` (the most that kernel is ever launched with), once per kernel
// and device.  The value never changes afterwards, so launches from several host threads cannot meet a smaller
// limit than they need.
int set_max_dynamic_lds(const void* kernel, int bytes);

}  // namespace dapq
