// Ceilings of this chip for the instruction mix of the score passes (Sec. 4.2 importance scores), measured
// rather than taken from the data sheet.  Benchmark support only: nothing of the eviction path calls this file,
// it is linked into a library of its own (libdapq_ceiling.so) and driven by `bench.py --ceilings`.
//
//   stream probes   how fast a 2 GiB array of key rows can be read with nothing else going on
//                   (a) plain 16-byte global loads, many waves per SIMD
//                   (b) the score kernels' own path: one wave per workgroup, buffer_load ... lds into a ring
//                       of 32-key sub-blocks, the MFMA operand fragments read back from LDS
//   issue probes    the score kernels' slice -- one v_mfma_f32_32x32x16_bf16 plus the vector work on two
//                   logits of the previous unit -- with no memory traffic at all, at one or two waves per SIMD,
//                   with the vector work varied (none / fma+exp+add / exp+add / plain fmas / extra
//                   instructions), which gives the cost of every ingredient in cycles per slice and SIMD
// Every probe reports the shader clock it ran at: the s_memtime ticks one wave counted from its first to its
// last instruction over the constant-rate (100 MHz) s_memrealtime ticks of the same interval.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#ifndef DAPQ_API
#define DAPQ_API
#endif

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct Ticks {
  unsigned long long shader, real;  // s_memtime / s_memrealtime ticks of block 0
};

__device__ __forceinline__ void tick_begin(unsigned long long& t0, unsigned long long& r0) {
  t0 = __builtin_readcyclecounter();
  r0 = __builtin_amdgcn_s_memrealtime();
}
__device__ __forceinline__ void tick_end(Ticks* out, unsigned long long t0, unsigned long long r0) {
  const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    out->shader = t1 - t0;
    out->real = r1 - r0;
  }
}

// ------------------------------------------------------------------------------------------ stream probes
__global__ __launch_bounds__(256) void read_plain_kernel(const u32x4* src, size_t n, unsigned* sink, Ticks* ticks) {
  unsigned long long t0, r0;
  tick_begin(t0, r0);
  unsigned acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n; i += 4 * stride) {  // four loads in flight per lane
    const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n; i += stride) {
    const u32x4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x12345678u) sink[0] = acc;  // keeps the loads alive, practically never taken
  tick_end(ticks, t0, r0);
}

// One wave per workgroup walks `rows_per_wave` 256-byte rows through a ring of NST 8 KB slots filled by
// buffer_load_dwordx4 ... lds (8 transfers of 1 KB per 32-row sub-block), and reads each sub-block back as eight
// 16-byte fragments per lane -- the data path of the score kernels with the arithmetic taken out.
template <int NST>
__global__ __launch_bounds__(64) void read_ring_kernel(const char* src, int rows_per_wave, unsigned* sink, Ticks* ticks) {
  extern __shared__ u32x4 ring[];
  unsigned long long t0, r0;
  tick_begin(t0, r0);
  const int lane = threadIdx.x;
  const char* base = src + (size_t)blockIdx.x * rows_per_wave * 256;
  const int nsubs = rows_per_wave / 32;
  const unsigned voff = (unsigned)(lane >> 4) * 256u + (unsigned)(lane & 15) * 16u;
  auto issue = [&](int sub) {
    const bool live = sub < nsubs;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(base) + (live ? (size_t)sub * 8192 : 0), 0, live ? 8192 : 0, 0x00020000);
    u32x4* slot = ring + (sub % NST) * 512;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(slot + i * 64), 16,
                                               (int)voff, i * 1024, 0, 0);
  };
  for (int i = 0; i < NST; ++i) issue(i);
  unsigned acc = 0;
  for (int sub = 0; sub < nsubs; ++sub) {
    // NST - 1 newer sub-blocks (8 operations each) may stay in flight
    if (NST == 5) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
    else if (NST == 4) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else if (NST == 3) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    const u32x4* slot = ring + (sub % NST) * 512;
    u32x4 f[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) f[s] = slot[s * 64 + lane];
#pragma unroll
    for (int s = 0; s < 8; ++s) acc ^= f[s].x ^ f[s].y ^ f[s].z ^ f[s].w;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    issue(sub + NST);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (acc == 0x12345678u) sink[0] = acc;
  tick_end(ticks, t0, r0);
}

// ------------------------------------------------------------------------------------------- issue probes
// What a slice holds: MFMAs (MF = 0: none, 1: one v_mfma_f32_32x32x16_bf16, 2: two v_mfma_f32_16x16x32_bf16, the same flops;
// 3, 4: as 1 with the MFMAs of eight units interleaved, see below), NE exponentials, NF fused multiply-adds, NA additions and NS scalar
// instructions.  CHAIN = true wires the vector work the way the score passes do (x = a*c + o, p = 2^x, sum += p, every
// result first read a slice later; needs NE = NF = NA = 2, any extra fmas run beside the chain); otherwise every
// instruction is independent of the others of its slice and reads results of the previous unit's MFMAs.
// NRB 32-row operand blocks stay in the accumulation registers like the kernels' Q fragments; a "unit" is 8 MFMAs
// that accumulate in place.
template <int NRB, int WAVES_PER_SIMD, int MF, int NE, int NF, int NA, int NS, bool CHAIN>
__global__ __launch_bounds__(64, WAVES_PER_SIMD) void slice_kernel(float* out, int iters, float c, Ticks* ticks) {
  static_assert(!CHAIN || (NE == 2 && NF >= 2 && NA == 2), "the chained mix is 2 fma + 2 exp2 + 2 add");
  extern __shared__ u32x4 pad[];  // only sized: keeps the number of resident waves per compute unit at 4 or 8
  unsigned long long t0, r0;
  tick_begin(t0, r0);
  bf16x8 q[NRB][8], kf[8];
#pragma unroll
  for (int r = 0; r < NRB; ++r)
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        unsigned hsh = (threadIdx.x * 2654435761u) ^ (i * 40503u) ^ (r * 69069u) ^ (s * 1234567u) ^ (blockIdx.x * 7919u);
        hsh ^= hsh >> 13; hsh *= 0x5bd1e995u; hsh ^= hsh >> 15;
        q[r][s][i] = (__bf16)(((hsh & 0xFFFF) / 65536.0f) * 4.0f - 2.0f);  // operands with all bits toggling
      }
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      unsigned hsh = (threadIdx.x * 2246822519u) ^ (i * 3266489917u) ^ (s * 668265263u);
      hsh ^= hsh >> 13; hsh *= 0x5bd1e995u; hsh ^= hsh >> 15;
      kf[s][i] = (__bf16)(((hsh & 0xFFFF) / 65536.0f) * 4.0f - 2.0f);
    }
#pragma unroll
  for (int r = 0; r < NRB; ++r)
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(q[r][s]));
  f32x16 prev;
#pragma unroll
  for (int v = 0; v < 16; ++v) prev[v] = -1.0f * v;
  float x0 = -1.0f, x1 = -2.0f, ea0 = 0, ea1 = 0, eb0 = 0, eb1 = 0, o = -3.0f;
  float acc[4] = {0, 0, 0, 0};
  int sc0 = iters, sc1 = 3;
  for (int it = 0; it < iters; ++it) {
    // opaque to the compiler: the products below are not loop invariants
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(kf[s]));
    if (MF >= 3) {
      // the same MFMAs in another order: one fragment of one operand serves NRB consecutive MFMAs (one per 32-row
      // block, NRB accumulators in flight) before the next fragment comes up, so that operand of the matrix pipe
      // stays put for NRB instructions instead of changing with every one (MF == 3: the second operand, 4: the first)
      f32x16 held[NRB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) held[rb] = f32x16{0};
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
          if (MF == 4) held[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], q[rb][s], held[rb], 0, 0, 0);
          else held[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[rb][s], kf[s], held[rb], 0, 0, 0);
        }
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) acc[rb & 3] += held[rb][rb];  // every product is "used"
      continue;
    }
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      f32x16 cur = {0};
      f32x4 tile[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};  // MF == 2: four 16x16 tiles of the unit
      if (!MF) asm volatile("" : "+v"(prev));  // no MFMA rewrites it: make it opaque so that the work is not hoisted
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        if (MF == 1) cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[rb][s], kf[s], cur, 0, 0, 0);
        if (MF == 2) {
          // the same flops as two 16x16x32 products: fragments s and s^1 stand in for the two 16-row halves
          tile[(2 * s) & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q[rb][s], kf[s], tile[(2 * s) & 3], 0, 0, 0);
          tile[(2 * s + 1) & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q[rb][s ^ 1], kf[s], tile[(2 * s + 1) & 3], 0, 0, 0);
        }
        if (CHAIN) {
          float& p0 = (s & 1) ? eb0 : ea0;
          float& p1 = (s & 1) ? eb1 : ea1;
          acc[0] += p0; acc[1] += p1;
          p0 = __builtin_amdgcn_exp2f(x0); p1 = __builtin_amdgcn_exp2f(x1);
          x0 = fmaf(prev[2 * s], c, o); x1 = fmaf(prev[2 * s + 1], c, o);
#pragma unroll
          for (int f = 2; f < NF; ++f) {
            const int n = s * (NF - 2) + f - 2;  // distinct operand pairs: no two of these are the same expression
            const float t = fmaf(prev[n & 15], c, prev[(2 * (n >> 4) + 1 + n) & 15]);
            asm volatile("" ::"v"(t));
          }
        } else {
#pragma unroll
          for (int e = 0; e < NE; ++e) {
            const int n = s * NE + e;  // 16 registers x 4 free input modifiers
            const float a = prev[n & 15];
            const float in = (n >> 4) == 0 ? a : ((n >> 4) == 1 ? -a : ((n >> 4) == 2 ? fabsf(a) : -fabsf(a)));
            const float t = __builtin_amdgcn_exp2f(in);
            asm volatile("" ::"v"(t));
          }
#pragma unroll
          for (int f = 0; f < NF; ++f) {
            const int n = s * NF + f;
            const float t = fmaf(prev[n & 15], c, prev[(2 * (n >> 4) + 1 + n) & 15]);
            asm volatile("" ::"v"(t));
          }
#pragma unroll
          for (int a = 0; a < NA; ++a) acc[a & 3] += prev[(2 * s + 5 + a) & 15];
        }
        if (NS > 0) {
#pragma unroll
          for (int k = 0; k < NS; k += 2)
            asm volatile("s_add_u32 %0, %0, 7\n\ts_xor_b32 %1, %1, %0" : "+s"(sc0), "+s"(sc1)::"scc");
        }
        // the order of the slice: the MFMA, then its vector (and scalar) companions
        if (MF) __builtin_amdgcn_sched_group_barrier(0x008, MF == 2 ? 2 : 1, 0);
        if (NE + NF + NA > 0) __builtin_amdgcn_sched_group_barrier(0x002, NE + NF + NA, 0);
        if (NS > 0) __builtin_amdgcn_sched_group_barrier(0x004, NS, 0);
      }
      if (MF) {
        asm volatile("" ::"v"(prev));  // every unit's products are "used", a full unit after they were made
        if (MF == 1) prev = cur;
        else {
#pragma unroll
          for (int v = 0; v < 16; ++v) prev[v] = tile[v >> 2][v & 3];
        }
      }
    }
  }
  float s = acc[0] + acc[1] + acc[2] + acc[3] + ea0 + ea1 + eb0 + eb1 + x0 + x1 + (float)(sc0 ^ sc1);
#pragma unroll
  for (int i = 0; i < 16; ++i) s += prev[i];
  out[blockIdx.x * 64 + threadIdx.x] = s;
  tick_end(ticks, t0, r0);
}

struct Scratch {
  float* out = nullptr;
  unsigned* sink = nullptr;
  Ticks* ticks = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
};

#define CEIL_CK(x)                                                                   \
  do {                                                                               \
    hipError_t e__ = (x);                                                            \
    if (e__ != hipSuccess) {                                                         \
      snprintf(g_error, sizeof g_error, "%s: %s", #x, hipGetErrorString(e__));       \
      return -1;                                                                     \
    }                                                                                \
  } while (0)

char g_error[256] = "";
Scratch g_s;

int ensure_scratch() {
  if (g_s.out != nullptr) return 0;
  CEIL_CK(hipMalloc(&g_s.out, 4096 * 64 * sizeof(float)));
  CEIL_CK(hipMalloc(&g_s.sink, 256));
  CEIL_CK(hipMalloc(&g_s.ticks, sizeof(Ticks)));
  CEIL_CK(hipEventCreate(&g_s.e0));
  CEIL_CK(hipEventCreate(&g_s.e1));
  return 0;
}

// Runs `launch` warm + reps times back to back on the null stream; result[0] = ms per launch, result[1] = shader
// clock in GHz seen by block 0 of the last launch, result[2] = its s_memtime ticks.
template <typename F>
int time_launches(F launch, int warm, int reps, double* result) {
  for (int i = 0; i < warm; ++i) launch();
  CEIL_CK(hipGetLastError());
  CEIL_CK(hipEventRecord(g_s.e0, 0));
  for (int i = 0; i < reps; ++i) launch();
  CEIL_CK(hipEventRecord(g_s.e1, 0));
  CEIL_CK(hipEventSynchronize(g_s.e1));
  CEIL_CK(hipGetLastError());
  float ms = 0;
  CEIL_CK(hipEventElapsedTime(&ms, g_s.e0, g_s.e1));
  Ticks t;
  CEIL_CK(hipMemcpy(&t, g_s.ticks, sizeof t, hipMemcpyDeviceToHost));
  result[0] = ms / reps;
  result[1] = t.real > 0 ? (double)t.shader / (double)t.real * 0.1 : 0.0;  // s_memrealtime runs at 100 MHz
  result[2] = (double)t.shader;
  return 0;
}

typedef void (*slice_fn)(float*, int, float, Ticks*);

struct SliceMix {
  const char* name;
  int mfma, n_exp, n_fma, n_add, n_salu;
  slice_fn one_wave, two_waves;  // 8 operand blocks at one wave per SIMD, 4 at two
};
#define CEIL_MIX(name, MF, NE, NF, NA, NS, CHAIN)                                                   \
  {name, MF, NE, NF, NA, NS, slice_kernel<8, 1, MF, NE, NF, NA, NS, CHAIN>, slice_kernel<4, 2, MF, NE, NF, NA, NS, CHAIN>}
const SliceMix kMixes[] = {
    CEIL_MIX("mfma", 1, 0, 0, 0, 0, false),
    CEIL_MIX("mfma + score chain (2 fma, 2 exp, 2 add)", 1, 2, 2, 2, 0, true),
    CEIL_MIX("two 16x16x32 mfma", 2, 0, 0, 0, 0, false),
    CEIL_MIX("two 16x16x32 mfma + score chain", 2, 2, 2, 2, 0, true),
    CEIL_MIX("mfma + score chain + 2 fma", 1, 2, 4, 2, 0, true),
    CEIL_MIX("mfma + score chain + 2 scalar", 1, 2, 2, 2, 2, true),
    CEIL_MIX("mfma + 2 fma 2 exp 2 add, independent", 1, 2, 2, 2, 0, false),
    CEIL_MIX("mfma + 2 exp 2 add", 1, 2, 0, 2, 0, false),
    CEIL_MIX("mfma + 1 exp", 1, 1, 0, 0, 0, false),
    CEIL_MIX("mfma + 2 exp", 1, 2, 0, 0, 0, false),
    CEIL_MIX("mfma + 4 exp", 1, 4, 0, 0, 0, false),
    CEIL_MIX("mfma + 2 fma", 1, 0, 2, 0, 0, false),
    CEIL_MIX("mfma + 4 fma", 1, 0, 4, 0, 0, false),
    CEIL_MIX("mfma + 6 fma", 1, 0, 6, 0, 0, false),
    CEIL_MIX("mfma + 8 fma", 1, 0, 8, 0, 0, false),
    CEIL_MIX("mfma + 12 fma", 1, 0, 12, 0, 0, false),
    CEIL_MIX("mfma, second operand held for 8 (4) in a row", 3, 0, 0, 0, 0, false),
    CEIL_MIX("mfma, first operand held for 8 (4) in a row", 4, 0, 0, 0, 0, false),
    CEIL_MIX("score chain alone (no mfma)", 0, 2, 2, 2, 0, true),
    CEIL_MIX("2 exp alone", 0, 2, 0, 0, 0, false),
    CEIL_MIX("6 fma alone", 0, 0, 6, 0, 0, false),
};
#undef CEIL_MIX
constexpr int kNumMixes = (int)(sizeof(kMixes) / sizeof(kMixes[0]));

int run_slice(const SliceMix& m, int wps, int iters, int warm, int reps, double* result) {
  slice_fn kern = wps == 1 ? m.one_wave : m.two_waves;
  const int lds = wps == 1 ? 40960 : 20480;  // 4 or 8 single-wave workgroups fit a compute unit
  CEIL_CK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  const int grid = 1024 * wps, nrb = wps == 1 ? 8 : 4;
  int rc = time_launches([&] { hipLaunchKernelGGL(kern, dim3(grid), dim3(64), lds, 0, g_s.out, iters, 0.1275f, g_s.ticks); },
                         warm, reps, result);
  if (rc != 0) return rc;
  // nanoseconds and cycles per slice and SIMD: a SIMD runs wps waves of iters * nrb * 8 slices each
  const double slices = (double)iters * nrb * 8 * wps;
  result[3] = result[0] * 1e6 / slices;
  result[4] = result[3] * result[1];
  return 0;
}

}  // namespace

extern "C" DAPQ_API const char* dapq_ceiling_last_error(void) { return g_error; }

// Reads `bytes` (a multiple of 1 MiB) of device memory at `src`.  path 0: plain loads, `param` workgroups of 256
// lanes (0 = 4096); path 1: the LDS ring, one wave per 8 MiB / `param`... see below.  result (host, 5 doubles):
// ms per launch, shader GHz, ticks, GB/s, 0.
//   path 1: `param` = ring slots (2..5); every wave walks bytes / (1024 * waves_per_simd) bytes, waves_per_simd =
//   `param2` (1, 2 or 4: 4, 8 or 16 single-wave workgroups per compute unit, bounded by the ring's LDS).
extern "C" DAPQ_API int dapq_ceiling_stream(const void* src, size_t bytes, int path, int param, int param2, int warm,
                                            int reps, double* result) {
  if (ensure_scratch() != 0) return -1;
  if (src == nullptr || bytes == 0 || bytes % (1u << 20) != 0 || result == nullptr) {
    snprintf(g_error, sizeof g_error, "dapq_ceiling_stream: bad arguments");
    return -1;
  }
  int rc;
  if (path == 0) {
    const int grid = param > 0 ? param : 4096;
    rc = time_launches([&] { hipLaunchKernelGGL(read_plain_kernel, dim3(grid), dim3(256), 0, 0, static_cast<const u32x4*>(src),
                                                bytes / 16, g_s.sink, g_s.ticks); }, warm, reps, result);
  } else {
    const int wps = param2;
    if ((wps != 1 && wps != 2 && wps != 4) || param < 2 || param > 5 || param * 8192 * wps * 4 > 160 * 1024) {
      snprintf(g_error, sizeof g_error, "dapq_ceiling_stream: ring of %d slots x %d waves per SIMD does not fit", param, wps);
      return -1;
    }
    const int waves = 1024 * wps;
    const size_t per_wave = bytes / waves;
    if (per_wave % 8192 != 0 || per_wave / 256 > 0x7fffffff) {
      snprintf(g_error, sizeof g_error, "dapq_ceiling_stream: %zu bytes per wave is not a whole number of sub-blocks", per_wave);
      return -1;
    }
    const int rows = (int)(per_wave / 256), lds = param * 8192;
#define CEIL_RING(NSTV)                                                                                               \
  do {                                                                                                                \
    CEIL_CK(hipFuncSetAttribute(reinterpret_cast<const void*>(read_ring_kernel<NSTV>),                                \
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds));                                    \
    rc = time_launches([&] { hipLaunchKernelGGL(read_ring_kernel<NSTV>, dim3(waves), dim3(64), lds, 0,                \
                                                static_cast<const char*>(src), rows, g_s.sink, g_s.ticks); },         \
                       warm, reps, result);                                                                           \
  } while (0)
    if (param == 2) CEIL_RING(2);
    else if (param == 3) CEIL_RING(3);
    else if (param == 4) CEIL_RING(4);
    else CEIL_RING(5);
#undef CEIL_RING
  }
  if (rc != 0) return rc;
  result[3] = (double)bytes / (result[0] * 1e-3) / 1e9;
  result[4] = 0.0;
  return 0;
}

// The score kernels' slice without memory traffic.  mix: index into the table of instruction mixes (name and counts via
// dapq_ceiling_slice_mix); waves_per_simd 1 (eight 32-row operand blocks per wave, the kernels' shape) or 2 (four
// blocks per wave).  result (host, 5 doubles): ms per launch, shader GHz, ticks, ns per slice and SIMD, cycles per
// slice and SIMD.
extern "C" DAPQ_API int dapq_ceiling_slice(int mix, int waves_per_simd, int iters, int warm, int reps, double* result) {
  if (ensure_scratch() != 0) return -1;
  if (result == nullptr || iters < 1 || (waves_per_simd != 1 && waves_per_simd != 2) || mix < 0 || mix >= kNumMixes) {
    snprintf(g_error, sizeof g_error, "dapq_ceiling_slice: bad arguments");
    return -1;
  }
  return run_slice(kMixes[mix], waves_per_simd, iters, warm, reps, result);
}

// Number of instruction mixes, and the name of mix `mix` (NULL if out of range); counts (host, 5 ints: mfma, exp,
// fma, add, scalar instructions per slice) may be NULL.
extern "C" DAPQ_API int dapq_ceiling_num_mixes(void) { return kNumMixes; }
extern "C" DAPQ_API const char* dapq_ceiling_slice_mix(int mix, int* counts) {
  if (mix < 0 || mix >= kNumMixes) return nullptr;
  if (counts != nullptr) {
    counts[0] = kMixes[mix].mfma > 0 ? 1 : 0; counts[1] = kMixes[mix].n_exp; counts[2] = kMixes[mix].n_fma;
    counts[3] = kMixes[mix].n_add; counts[4] = kMixes[mix].n_salu;
  }
  return kMixes[mix].name;
}
