// Importance scoring (Sec. 4.2, S(j) = sum_i Attention(q_i, k_j); Attention = softmax over the
// prompt keys, App. C.1) as two streaming passes over K for gfx950.
//
//   pass 1  (score_wave_pass1_kernel + score_combine_kernel): lse2[row] = log2 sum_j 2^(c * q_row.k_j)
//   pass 2  (score_wave_pass2_kernel [+ score_group_sum_kernel]): S(j) = sum_rows 2^(c * q_row.k_j - lse2[row])
// with c = scale * log2(e).  "rows" are the R = g*N pseudo-query rows of the g query heads that
// share one KV head.  Nothing of size N x L_p is ever stored.  Where a (layer, sequence, KV head) fits one
// workgroup -- one row group, at most 4 chunks per sequence of a dense batch -- dapq_score runs both passes in
// one launch (score_fused_kernel: the same two walks, the merge in between through LDS).
//
// Work split.  The unit of work is ONE wave (four independent ones are launched as a workgroup).  It keeps a group of up to 256 Q rows of one KV head in
// registers as MFMA operand fragments (eight 32-row blocks = 256 registers, pinned to the
// accumulation half of the register file; one wave per SIMD owns the whole 512-register file) and
// walks its own chunk of keys of one (layer, sequence, KV head).  Nothing is shared between waves:
// no barrier anywhere in the separate-pass kernels (the one-launch form has two, between its passes),
// no cross-wave reduction.  Heads with more than 256 rows are split into row
// groups (grid.y): pass 1 needs nothing more (its sums are per row), pass 2 writes one plane of
// column sums per group (group 0 into the result) and a small kernel adds the planes in group order.
// Keys arrive through a per-wave ring of 32-key sub-blocks in LDS (buffer_load_dwordx4 ... lds, five
// slots of 8 KB: four sub-blocks = 32 KB in flight per wave, 128 KB per compute unit; 16-byte
// chunks XOR-swizzled so that the MFMA operand reads are bank-conflict free), and every fragment is
// read from LDS exactly once per wave.  v_mfma_f32_32x32x16_bf16 runs on every (sub-block, row
// block) unit:
//   pass 1 uses D[key][query] (K as the A operand): a lane owns one query column, the reduction
//           over keys stays inside the lane;
//   pass 2 uses D[query][key] (Q as the A operand): a lane owns one key column, the reduction over
//           query rows stays inside the lane, and -lse2 of the lane's 16 rows per row block sits in
//           registers (128 of them).
// Pass 1 does not track a running maximum: it exponentiates against a per-row reference logit taken
// from the first sub-block (2^x has 127 binades of headroom above it) and only if a sum overflows
// redoes the chunk with a conventional online maximum.
//
// With one wave per SIMD every instruction costs issue time, so the kernels are built around the
// instruction count per MFMA ("slice"): one MFMA, and for two logits of the previous unit one FMA,
// one exponential and one add each; the rest (transfer issue, ring wait, fragment reads, loop
// control) is about one more instruction per slice.

#include <math.h>

#include <mutex>

#include "dapq_internal.h"

namespace dapq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // 16 bytes; native vector, stays in registers

constexpr int kLists = 8;  // work lists of a ragged batch, one per XCD (see ItemLists)

struct ScoreParams {
  const uint16_t* q;
  const uint16_t* k;
  const int32_t* cu_seqlens;  // NULL = dense
  int32_t* cu_chunks;         // [batch+1] prefix of per-sequence chunk counts (ragged only)
  unsigned* work;             // ragged only: [kLists] next ticket of every work list; zeroed with cu_chunks
  float2* parts;              // [layer*Hkv][max_chunks][rows_pad] (reference, sum) in the log2 domain
  float* lse2;                // [layer][batch][Hq][N]
  float* scores;              // [layer][Hkv][total_tokens]
  float* partial;             // [n_groups-1][layer][Hkv][total_tokens] column sums of row groups 1.. (n_groups > 1)
  int64_t k_stride_layer, k_stride_seq, k_stride_head, k_stride_token;
  int64_t q_stride_layer, q_stride_seq, q_stride_head, q_stride_row;
  int64_t total_tokens;
  int32_t n_layers, batch, n_q_heads, n_kv_heads, group, n_pseudo;
  int32_t rows, rows_pad, n_groups, chunk_keys, max_chunks;
  int32_t wg_groups;          // row groups that sit side by side in a workgroup (dense launches; 1, 2 or 4)
  float c;  // scale * log2(e)
};

constexpr int kSubBytes = 32 * kHeadDim * 2;          // one 32-key sub-block

// Which (sequence, chunk) a workgroup works on.
struct Work {
  int seq;
  int64_t tok0;  // packed token index of the first key of the chunk
  int key0;      // first key of the chunk inside the sequence
  int nkeys;     // keys in the chunk (<= chunk_keys), 0 = nothing to do
  int seq_len;
};

// The same for a wave-uniform chunk index, with the result pinned to scalar registers: everything
// derived from it (key base pointer, buffer descriptors, trip counts) then stays scalar too.
__device__ __forceinline__ int uniform_i32(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned uniform_u32(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* ptr) {
  const unsigned long long v = (unsigned long long)(uintptr_t)ptr;
  const unsigned lo = (unsigned)uniform_i32((int)(unsigned)(v & 0xFFFFFFFFull));
  const unsigned hi = (unsigned)uniform_i32((int)(unsigned)(v >> 32));
  return reinterpret_cast<const T*>((uintptr_t)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ Work locate(const ScoreParams& p, int gchunk);
__device__ __forceinline__ Work locate_uniform(const ScoreParams& p, int gchunk) {
  Work w = locate(p, gchunk);
  w.seq = uniform_i32(w.seq);
  w.key0 = uniform_i32(w.key0);
  w.nkeys = uniform_i32(w.nkeys);
  w.seq_len = uniform_i32(w.seq_len);
  const unsigned lo = (unsigned)uniform_i32((int)(unsigned)(w.tok0 & 0xFFFFFFFFll));
  const unsigned hi = (unsigned)uniform_i32((int)(unsigned)((unsigned long long)w.tok0 >> 32));
  w.tok0 = (int64_t)(((unsigned long long)hi << 32) | lo);
  return w;
}

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

// LDS position of 16-byte chunk `ch` of sub-block row `key`: rows are 256 B apart, chunks XOR-swizzled by
// the row so that 16 consecutive rows reading the same logical chunk hit 16 different bank groups.
__device__ __forceinline__ int lds_chunk_index(int key, int ch) { return key * 16 + (ch ^ (key & 15)); }

// Fragment s of lane (n, h) of an MFMA operand is the 8 channels [(2s+h)*8, +8) of row n: the same
// for a 32-row block of Q read straight from global memory.
__device__ __forceinline__ void frag_from_q(bf16x8 (&f)[8], const ScoreParams& p, const uint16_t* qbase, int row,
                                            int h) {
  const int rc = row < p.rows ? row : p.rows - 1;  // padding rows repeat the last row; their results are dropped
  const int head = rc / p.n_pseudo, i = rc - head * p.n_pseudo;
  const uint16_t* src = qbase + (int64_t)head * p.q_stride_head + (int64_t)i * p.q_stride_row;
#pragma unroll
  for (int s = 0; s < 8; ++s) f[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + (2 * s + h) * 8));
}

__device__ __forceinline__ float xhalf(float v) { return __shfl_xor(v, 32, 64); }

// v + (v of the lane 32 away), in every lane, on the vector ALU alone (v_permlane32_swap exchanges the upper half of
// its first operand with the lower half of its second): no trip through LDS, hence no wait on the LDS counter, which
// with a single wave per SIMD would be dead time.  The wait states around the swap are the ones the hazard rules
// of gfx950 ask for between a vector write and a lane swap of the same register, and between the swap and its use.
__device__ __forceinline__ float sum_halves(float v) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return a + b;  // a = (v.lo, v.lo), b = (v.hi, v.hi)
}

// Column sums of one sub-block go out through a buffer store whose range check drops what must not be written:
// lanes of the upper half carry an offset far past the end, and keys at or past nkeys fall outside num_records.
struct ColumnStore {
  __amdgpu_buffer_rsrc_t rsrc;
  unsigned lane_off;  // byte offset of this lane's key inside a sub-block; out of range for the upper half
};
__device__ __forceinline__ ColumnStore make_column_store(float* out, int nkeys, int n, int h) {
  ColumnStore cs;
  cs.rsrc = __builtin_amdgcn_make_buffer_rsrc(out, 0, nkeys * 4, 0x00020000);
  cs.lane_off = h == 0 ? (unsigned)n * 4u : 0xC0000000u;
  return cs;
}
__device__ __forceinline__ void store_columns(const ColumnStore& cs, int first_key, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), cs.rsrc,
                                            (int)(cs.lane_off + (unsigned)first_key * 4u), 0, 0);
}

// Row of the 32x32 MFMA result held in accumulator register v of a lane in half h.
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

typedef const u32x4 __attribute__((address_space(3))) * lds_vec_ptr;

// 16-byte LDS read at a per-lane byte address plus a compile-time offset (folds into the instruction).
__device__ __forceinline__ bf16x8 lds_read16(unsigned lane_addr, int const_off) {
  return __builtin_bit_cast(bf16x8, *(lds_vec_ptr)(uintptr_t)(lane_addr + const_off));
}

// Per-sequence prefix of chunk counts for ragged batches: one wave, 64 sequences per trip (a scan by shuffles
// inside the wave, the running total carried from trip to trip).
__global__ void score_chunk_prefix_kernel(const int32_t* cu_seqlens, int32_t* cu_chunks, unsigned* work,
                                         int batch, int chunk_keys) {
  const int lane = threadIdx.x;  // launched with exactly 64 threads
  if (lane == 0) cu_chunks[0] = 0;
  if (lane < kLists) work[lane] = 0u;  // the pass that follows hands its items out from here (one counter per work list)
  int carry = 0;
  for (int b0 = 0; b0 < batch; b0 += 64) {
    const int b = b0 + lane;
    int mine = 0;
    if (b < batch) {
      const int L = cu_seqlens[b + 1] - cu_seqlens[b];
      mine = L > 0 ? (L + chunk_keys - 1) / chunk_keys : 0;
    }
    int inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(inc, d, 64);
      if (lane >= d) inc += o;
    }
    if (b < batch) cu_chunks[b + 1] = carry + inc;
    carry += __shfl(inc, 63, 64);
  }
}

// Merge the per-chunk (reference, sum) pairs of a row: lse2 = log2 sum_c z_c 2^(ref_c).
__global__ void score_combine_kernel(ScoreParams p) {
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
  const float2* src = p.parts + ((int64_t)(layer * p.n_kv_heads + kv) * p.max_chunks) * p.rows_pad + row;
  float m = -INFINITY;
  for (int64_t e = c0; e < c1; ++e) {
    const float2 v = src[e * p.rows_pad];
    if (v.y > 0.0f) m = fmaxf(m, v.x + log2f(v.y));
  }
  float s = 0.0f;
  for (int64_t e = c0; e < c1; ++e) {
    const float2 v = src[e * p.rows_pad];
    if (v.y > 0.0f) s += exp2f(v.x + log2f(v.y) - m);
  }
  p.lse2[gid] = (s > 0.0f) ? m + log2f(s) : 0.0f;
}

// ---------------------------------------------------------------------------------------------
// The score kernels: one wave = a group of query rows x its own key stream.
// ---------------------------------------------------------------------------------------------
constexpr int kWaveStages = 5;            // ring slots (40 KB per wave, 160 KB per compute unit)
// Persistent workgroups of several waves (ragged batches with more than 256 query rows per KV head) need a few bytes
// of LDS to pass tickets around, which five slots per wave leave no room for; the ring depth makes no measurable
// difference between 3 and 5.
constexpr int kTeamStages = 4;
constexpr int kSubVec = kSubBytes / 16;   // 512 16-byte chunks per sub-block
// Dense launches start their waves up to four to a workgroup, one per SIMD of a compute unit, each with its own ring:
// they never meet at a barrier.  The waves of a workgroup are the row groups of a chunk side by side (a KV head with
// more than 256 query rows: they read the same keys at the same time, and the second reader finds them in the compute
// unit's L2 instead of fetching them through the fabric again: 6 % at 512 and 1024 rows) and then consecutive chunks
// (the dispatcher places fewer workgroups and the waves of a compute unit read one head's queries once: 2-3 % for the
// stream-bound shapes).  Every workgroup must be full -- waves of a half-empty one would idle their SIMDs for the whole
// launch -- so the number of consecutive chunks is the largest of 4, 2, 1 (divided by the row groups) that divides
// the chunk count.  (Ragged batches: see the DYN form of the kernels.)
constexpr int kWavesPerGroup = 4;
constexpr int wave_lds(int nst) { return nst * kSubBytes; }

// Per-lane byte offsets of the four distinct 16-byte chunks a lane fetches in sub_dma: transfer i
// moves key rows 4i..4i+3, lane (row0 = lane / 16, pos = lane % 16) fills LDS position pos of row
// 4i + row0 with the logical chunk pos ^ ((4i + row0) & 15) = (pos ^ row0) ^ (4 * (i & 3)).
__device__ __forceinline__ void sub_dma_lane_offsets(unsigned (&voff)[4], int64_t stride_token, int lane) {
  const unsigned row0 = (unsigned)lane >> 4, pos = (unsigned)lane & 15u;
#pragma unroll
  for (int j = 0; j < 4; ++j) voff[j] = row0 * (unsigned)stride_token * 2u + ((pos ^ row0) ^ (4u * j)) * 16u;
}

// One wave moves the 32-key sub-block that starts at key0 into an LDS slot: 8 transfers of 1 KB
// (buffer_load_dwordx4 ... lds).  The buffer descriptor spans from the first row of the sub-block to
// the end of the last key row of the chunk, so rows past the end of the chunk read as zeros; the
// uniform part of every address lives in scalar registers (descriptor base, scalar offset per
// transfer) and the lane part is one of the four precomputed offsets.  A sub-block that starts before
// the chunk or at or past its end gets an empty descriptor: the eight transfers still count as vector
// memory operations (the waits rely on a fixed number per sub-block) but fetch nothing and fill the
// slot with zeros.
__device__ __forceinline__ void sub_dma(u32x4* slot, const uint16_t* kbase, int64_t stride_token, int key0, int nkeys,
                                        const unsigned (&voff)[4]) {
  const int64_t stride_b = stride_token * 2;
  const bool live = key0 >= 0 && key0 < nkeys;
  const char* base = reinterpret_cast<const char*>(kbase) + (live ? (int64_t)key0 * stride_b : (int64_t)0);
  const int64_t span = (int64_t)(nkeys - key0 - 1) * stride_b + kHeadDim * 2;
  const unsigned records = !live ? 0u : (span > (int64_t)0xFFFFFFFFll ? 0xFFFFFFFFu : (unsigned)span);
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, (int)records, 0x00020000);
#pragma unroll
  for (int i = 0; i < 8; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(slot + i * 64), 16,
                                             (int)voff[i & 3], (int)((unsigned)(4 * i) * (unsigned)stride_b), 0, 0);
}

// Waits until at most `newer` sub-block transfers (8 operations each) of this wave are in flight.
__device__ __forceinline__ void wait_subblocks(int newer) {
  if (newer <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if (newer == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if (newer == 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else if (newer == 3) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
}

template <int NST>
__device__ __forceinline__ void wait_ring_full() {
  static_assert(NST >= 2 && NST <= 5, "ring sizes the kernels use");
  if (NST == 5) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
  else if (NST == 4) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
  else if (NST == 3) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
}

// The instruction order is pinned with empty asm statements that take values as read-write operands:
// what produces an operand must come before the statement, what uses it after.  One sits right
// after the MFMA of a slice (it "redefines" the K fragment the MFMA read and the two pending
// exponents, so the MFMA leads the slice and the vector work follows), one at the end of the slice.
// Neither names a transcendental's result or the accumulator in flight: both would cost wait states.
// (Naming the K fragment of the next MFMA at the slice end as well keeps that MFMA from starting
// early, but measures 1-2 % slower per pass over a few hundred back-to-back launches.)
#define DAPQ_WAVE_SLICE_MID(kfrag, x0, x1) asm volatile("" : "+v"(kfrag), "+v"(x0), "+v"(x1))
#define DAPQ_WAVE_SLICE_END(prev, x0, x1, t0, t1, addr) \
  asm volatile("" : "+v"(prev), "+v"(x0), "+v"(x1), "+v"(t0), "+v"(t1), "+v"(addr))

// One step of the four-stage vector pipeline over pairs of logits: the exponentials started two
// steps ago (p0, p1: two sets of registers take turns) are added to the sums they belong to (t0,
// t1), the exponents formed in the previous step are exponentiated into the registers just freed,
// and the exponents of a new pair are formed (x = a*c + o).  Every result is first read a full step
// after the instruction that produces it, whatever order the compiler picks inside a step.
#define DAPQ_VALU_STEP(a0, a1, o0, o1, t0, t1, p0, p1) \
  do {                                                 \
    t0 += p0;                                          \
    t1 += p1;                                          \
    p0 = __builtin_amdgcn_exp2f(x0);                   \
    p1 = __builtin_amdgcn_exp2f(x1);                   \
    x0 = fmaf((a0), c, (o0));                          \
    x1 = fmaf((a1), c, (o1));                          \
  } while (0)
// step k of a unit: even steps use the first set of pending exponentials, odd steps the second
#define DAPQ_VALU_STEP_K(k, a0, a1, o0, o1, t0, t1)                     \
  do {                                                                  \
    if ((k) % 2 == 0) DAPQ_VALU_STEP(a0, a1, o0, o1, t0, t1, ea0, ea1); \
    else DAPQ_VALU_STEP(a0, a1, o0, o1, t0, t1, eb0, eb1);              \
  } while (0)

// Pipelined walk of one wave over sub-blocks [sb0, sb1) of its chunk.
//   on entry  kf = fragments of sub-block sb0; the transfers of sub-blocks sb0+1 .. sb0+NST-1 are
//             under way (sub-block i lives in ring slot i % NST)
//   on exit   kf = fragments of sub-block sb1 (zeros if it does not exist)
// Every iteration issues the transfer of sub-block sub+NST into the slot of the current sub-block
// once its fragments are in registers, and waits for sub-block sub+1 before its last unit; as every
// sub-block is 8 operations, existing or not, that wait is a fixed count.
// A unit is one sub-block against one 32-row block of Q: 8 MFMAs, one per slice.  While the MFMAs
// of a unit issue, the 16 logits per lane of the unit before it enter the vector pipeline, one pair
// per slice (the MFMA leads its slice, so the last MFMA of a unit is a full slice old when its
// first result is read).  The sum a step adds to belongs to the pair three steps back: steps 0..2
// of a unit still feed the unit two back.
// PASS 1: off1[rb] = -(reference logit * c) of row block rb; acc[rb] receives the row sums.
// PASS 2: off2[rb][v] = -lse2 of the row that accumulator register v of this lane holds in row
//         block rb (-inf for padding rows, which then add 0).  S of every key goes to out.
// NST = slots of the sub-block ring.
template <int NRB, int PASS, int NST, bool REV = false>
__device__ __forceinline__ void wave_walk(u32x4* ring, const uint16_t* kbase, int64_t stride_token, int nkeys,
                                          int sb0, int sb1, bf16x8 (&kf)[8], const bf16x8 (&qf)[NRB][8], float c,
                                          const float (&off1)[NRB], const float (&off2)[PASS == 2 ? NRB : 1][16],
                                          float (&acc)[NRB], float* out, const unsigned (&voff)[4], int n, int h,
                                          int last_sub = 0) {
  // REV: step `sub` of the walk works on sub-block last_sub - sub of the chunk (the chunk is walked from
  // its end to its start); otherwise on sub-block sub
  auto first_key = [&](int sub) { return (REV ? last_sub - sub : sub) * 32; };
  const unsigned ring_base = (unsigned)(uintptr_t)(lds_vec_ptr)ring;
  unsigned fa[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) fa[s] = ring_base + (unsigned)(n * 16 + ((2 * s + h) ^ (n & 15))) * 16u;
  const ColumnStore cols = make_column_store(PASS == 2 ? out : nullptr, PASS == 2 ? nkeys : 0, n, h);
  f32x16 prev;
#pragma unroll
  for (int v = 0; v < 16; ++v) prev[v] = -INFINITY;  // 2^(-inf) = 0: the first steps add nothing
  float x0 = -INFINITY, x1 = -INFINITY, ea0 = 0.0f, ea1 = 0.0f, eb0 = 0.0f, eb1 = 0.0f, sa = 0.0f, sb = 0.0f;
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) acc[rb] = 0.0f;

  int issue_slot = sb0 % NST;          // ring slot of the current sub-block: the next transfer goes there
  int read_slot = (sb0 + 1) % NST;     // ring slot of the sub-block after the current one
  for (int sub = sb0; sub < sb1; ++sub) {
    const unsigned next_slot = (unsigned)read_slot * (unsigned)kSubBytes;
    read_slot = read_slot + 1 == NST ? 0 : read_slot + 1;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      constexpr int kLast = NRB - 1;
      const int rb1 = (rb + NRB - 1) % NRB;  // row block of the previous unit (prev)
      const int rb2 = (rb + NRB - 2) % NRB;  // row block of the unit before it
      if (rb == 1) {
        // the slot of this sub-block is free (its fragments are in registers and have been used)
        sub_dma(ring + issue_slot * kSubVec, kbase, stride_token, first_key(sub + NST), nkeys, voff);
        issue_slot = issue_slot + 1 == NST ? 0 : issue_slot + 1;
      }
      if (rb == kLast) wait_ring_full<NST>();  // sub-block sub+1 has landed: NST-1 newer ones are in flight
      f32x16 cur = {0};
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        if (PASS == 1) cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[rb][s], cur, 0, 0, 0);
        else cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][s], kf[s], cur, 0, 0, 0);
        DAPQ_WAVE_SLICE_MID(kf[s], x0, x1);
        if (rb == kLast) kf[s] = lds_read16(fa[s] + next_slot, 0);  // last use: fetch the next sub-block's
        if (PASS == 2) {
          DAPQ_VALU_STEP_K(s, prev[2 * s], prev[2 * s + 1], off2[PASS == 2 ? rb1 : 0][2 * s],
                           off2[PASS == 2 ? rb1 : 0][2 * s + 1], sa, sb);
          if (s == 2 && rb == 1) {
            // the adds above took in the last logits of the previous sub-block: its column sums are complete
            if (sub > sb0) store_columns(cols, first_key(sub - 1), sum_halves(sa + sb));
            sa = sb = 0.0f;
          }
          DAPQ_WAVE_SLICE_END(prev, x0, x1, sa, sb, fa[(s + 1) & 7]);
        } else {
          if (s < 3) DAPQ_VALU_STEP_K(s, prev[2 * s], prev[2 * s + 1], off1[rb1], off1[rb1], acc[rb2], acc[rb2]);
          else DAPQ_VALU_STEP_K(s, prev[2 * s], prev[2 * s + 1], off1[rb1], off1[rb1], acc[rb1], acc[rb1]);
          DAPQ_WAVE_SLICE_END(prev, x0, x1, acc[rb1], acc[rb2], fa[(s + 1) & 7]);
        }
      }
      prev = cur;
    }
  }

  // drain: prev = last unit (row block NRB-1); three more steps on -inf flush the pipeline
  {
    constexpr int rbl = NRB - 1, rbl1 = NRB - 2;
#pragma unroll
    for (int k = 0; k < 11; ++k) {
      const float a0 = k < 8 ? prev[(2 * k) & 15] : -INFINITY, a1 = k < 8 ? prev[(2 * k + 1) & 15] : -INFINITY;
      if (PASS == 1) {
        if (k < 3) DAPQ_VALU_STEP_K(k, a0, a1, off1[rbl], off1[rbl], acc[rbl1], acc[rbl1]);
        else DAPQ_VALU_STEP_K(k, a0, a1, off1[rbl], off1[rbl], acc[rbl], acc[rbl]);
      } else {
        DAPQ_VALU_STEP_K(k, a0, a1, off2[PASS == 2 ? rbl : 0][(2 * k) & 15], off2[PASS == 2 ? rbl : 0][(2 * k + 1) & 15], sa,
                         sb);
      }
    }
    if (PASS == 2 && sb1 > sb0) store_columns(cols, first_key(sb1 - 1), sum_halves(sa + sb));
  }
}

// One sub-block the plain way (pass 1): masks keys >= nkeys (or, CAUSAL, the keys after each query's
// own position), fixes the reference logits (FIRST) or tracks a running maximum (SAFE).
template <int NRB, bool SAFE, bool FIRST, bool CAUSAL = false>
__device__ __forceinline__ void wave_sub_simple(const bf16x8 (&kf)[8], const bf16x8 (&qf)[NRB][8], float c,
                                                float (&ref)[NRB], float (&z)[NRB], int key0, int nkeys, int h,
                                                const int* last_key = nullptr) {
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    f32x16 a = {0};
#pragma unroll
    for (int s = 0; s < 8; ++s) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[rb][s], a, 0, 0, 0);
    if (CAUSAL) {
      // last_key[rb]: the last key this lane's query of row block rb may see
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (key0 + acc_row(v, h) > last_key[rb]) a[v] = -INFINITY;
    } else if (key0 + 32 > nkeys) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (key0 + acc_row(v, h) >= nkeys) a[v] = -INFINITY;
    }
    if (SAFE || FIRST) {
      float m = a[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) m = fmaxf(m, a[v]);
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
    for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(a[v], c, nref));
    z[rb] += sum;
  }
}

// The Q fragments only ever feed MFMAs, which can read their A/B operands from the accumulation
// half of the register file: pin them there so that the vector half stays free for everything the
// vector ALU touches (accumulators, exponentials, offsets).
template <int NRB>
__device__ __forceinline__ void pin_q_in_agprs(bf16x8 (&qf)[NRB][8]) {
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qf[rb][s]));
}

template <int NRB>
__device__ __forceinline__ void wave_load_frags(bf16x8 (&kf)[8], const u32x4* slot, int n, int h) {
#pragma unroll
  for (int s = 0; s < 8; ++s) kf[s] = __builtin_bit_cast(bf16x8, slot[lds_chunk_index(n, 2 * s + h)]);
}

// The next item of a ragged batch's work list (see the kernels below): lane 0 takes a ticket, everybody gets it.
__device__ __forceinline__ unsigned take_item(unsigned* work, int lane) {
  unsigned v = 0;
  if (lane == 0) v = atomicAdd(work, 1u);
  return (unsigned)uniform_i32((int)v);
}

// The work lists of a ragged batch: one per XCD (kLists of them: each XCD has its own L2).  List x holds the chunks c of
// the packed key axis with c mod kLists == x, for every head and every block of row groups; ticket t of list x is item
// ((head * chunks_x + c') * blocks + block) with c = c' * kLists + x.  A block is the row groups that the waves of one
// workgroup (a team) take side by side: they read the same keys at the same time, so the second reader finds them in
// the compute unit's L2 and the keys go through the fabric once.  A team takes tickets from the list of the XCD it
// runs on (consecutive tickets are blocks of the same chunk: the same keys again, behind the same L2); when that list is
// empty it goes on to the others', so every list is drained whatever runs where.  (The host launches this form only
// if the item count fits 31 bits whatever the lengths are.)
struct Item {
  int head, block, chunk, seq, nkeys;
};
struct ItemLists {
  unsigned chunks, blocks, heads;
  __device__ __forceinline__ unsigned chunks_of(int x) const { return (chunks + (unsigned)(kLists - 1 - x)) / kLists; }
  __device__ __forceinline__ unsigned count(int x) const { return heads * chunks_of(x) * blocks; }
  // `reversed`: heads and chunks from the far end (pass 2)
  __device__ __forceinline__ Item at(const ScoreParams& p, int x, unsigned ticket, bool reversed) const {
    const unsigned cx = chunks_of(x);
    const unsigned u = uniform_u32(ticket / blocks), block = ticket - u * blocks;
    const unsigned head = uniform_u32(u / cx), c = u - head * cx;
    Item it;
    it.head = (int)(reversed ? heads - 1 - head : head);
    it.block = (int)block;
    it.chunk = (int)((reversed ? cx - 1 - c : c) * kLists + (unsigned)x);
    const Work w = locate_uniform(p, it.chunk);
    it.seq = w.seq;
    it.nkeys = w.nkeys;
    return it;
  }
};
__device__ __forceinline__ ItemLists item_lists(const ScoreParams& p) {
  ItemLists l;
  l.chunks = (unsigned)uniform_i32(p.cu_chunks[p.batch]);
  l.blocks = (unsigned)(p.n_groups / p.wg_groups);
  l.heads = (unsigned)(p.n_layers * p.n_kv_heads);
  return l;
}

// The tickets of a team.  A team of one wave keeps its ticket in a register; in a larger team wave 0 takes the ticket and
// leaves it in one of two LDS words (behind the rings), which the others read after the barrier that starts the item:
// the slots alternate, so a slot is rewritten only after two more barriers.
struct TeamTickets {
  unsigned* slots;  // LDS, two words (teams of more than one wave)
  unsigned mine;    // team of one: the ticket
  int parity;
  bool team, leader;
  __device__ __forceinline__ void post(unsigned ticket, int lane) {
    if (!team) mine = ticket;
    else if (leader && lane == 0) slots[parity] = ticket;
  }
  __device__ __forceinline__ unsigned next() {
    if (!team) return mine;
    __syncthreads();
    const unsigned t = uniform_u32(slots[parity]);
    parity ^= 1;
    return t;
  }
};
__device__ __forceinline__ TeamTickets team_tickets(u32x4* rings, int nst, int wave_id) {
  TeamTickets t;
  const int waves = (int)(blockDim.x >> 6);
  t.slots = reinterpret_cast<unsigned*>(rings + waves * (wave_lds(nst) / 16));
  t.mine = 0;
  t.parity = 0;
  t.team = waves > 1;
  t.leader = wave_id == 0;
  return t;
}
// The XCD this wave runs on (hardware register XCC_ID, bits 3:0).
__device__ __forceinline__ int home_list() {
  return (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & (unsigned)(kLists - 1));
}

// Pass 1 of one chunk: `head` = layer * n_kv_heads + KV head, `group` = row group, `chunk_id` = chunk along the packed
// key axis.  If `work` is not NULL the ticket for the wave's next item is taken from it while the chunk drains (so
// its round trip costs nothing) and returned.  The chunk must have keys.
// FUSED (score_fused_kernel): the chunk's (reference, sum) pairs go to the start of the wave's own ring, which is
// drained by then, instead of to global memory.
template <int NRB, int NST, bool FUSED = false>
__device__ __forceinline__ unsigned pass1_item(const ScoreParams& p, u32x4* ring, int chunk_id, int group, int head,
                                               bf16x8 (&qf)[NRB][8], const unsigned (&voff)[4], int lane,
                                               unsigned* work) {
  const Work w = locate_uniform(p, chunk_id);
  // (the division runs on the vector ALU: bring the quotient back to a scalar register)
  const int layer = uniform_i32(head / p.n_kv_heads), kv = head - layer * p.n_kv_heads;
  const int n = lane & 31, h = lane >> 5;
  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)w.seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = uniform_ptr(p.k + (int64_t)layer * p.k_stride_layer + (int64_t)w.seq * p.k_stride_seq +
                                      (int64_t)kv * p.k_stride_head + w.tok0 * p.k_stride_token);
  const int gbase = group * (NRB * 32);  // first row of this wave's row group
  const int nsubs = (w.nkeys + 31) / 32, nfull = w.nkeys / 32;
  // the ring is filled whether the sub-blocks exist or not (sub_dma): the waits count operations
#pragma unroll
  for (int i = 0; i < NST; ++i) sub_dma(ring + i * kSubVec, kbase, p.k_stride_token, i * 32, w.nkeys, voff);
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) frag_from_q(qf[rb], p, qbase, gbase + rb * 32 + n, h);
  if (NRB == 8) pin_q_in_agprs<NRB>(qf);

  float ref[NRB], z[NRB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    ref[rb] = -INFINITY;
    z[rb] = 0.0f;
  }
  bf16x8 kf[8];
  wait_subblocks(NST - 1);
  wave_load_frags<NRB>(kf, ring, n, h);
  // sub-block 0 the plain way: it fixes the reference logits
  wave_sub_simple<NRB, false, true>(kf, qf, p.c, ref, z, 0, w.nkeys, h);
  if (nsubs > 1) {
    wait_subblocks(NST - 2);
    wave_load_frags<NRB>(kf, ring + kSubVec, n, h);
    sub_dma(ring, kbase, p.k_stride_token, NST * 32, w.nkeys, voff);  // slot 0 is free
    if (nfull > 1) {
      float off[NRB], zs[NRB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) off[rb] = -ref[rb];
      const float no_off2[1][16] = {};
      wave_walk<NRB, 1, NST>(ring, kbase, p.k_stride_token, w.nkeys, 1, nfull, kf, qf, p.c, off, no_off2, zs,
                                      nullptr, voff, n, h);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) z[rb] += zs[rb];
    }
  }
  // (no counted wait follows: the ticket's round trip overlaps what is left of the chunk)
  const unsigned next = work != nullptr ? take_item(work, lane) : 0u;
  if (nsubs > 1 && nfull < nsubs && nfull >= 1)  // the partial last sub-block; its fragments are in kf
    wave_sub_simple<NRB, false, false>(kf, qf, p.c, ref, z, nfull * 32, w.nkeys, h);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // a sum that is not finite means a logit sat more than ~127 binades above the reference: redo
  // the chunk with a running maximum, one sub-block at a time
  bool bad = false;
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) bad = bad || !(z[rb] < INFINITY);
  if (__any(bad ? 1 : 0)) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      ref[rb] = -INFINITY;
      z[rb] = 0.0f;
    }
    for (int sub = 0; sub < nsubs; ++sub) {
      sub_dma(ring, kbase, p.k_stride_token, sub * 32, w.nkeys, voff);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      wave_load_frags<NRB>(kf, ring, n, h);
      wave_sub_simple<NRB, true, false>(kf, qf, p.c, ref, z, sub * 32, w.nkeys, h);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the fragments are out of the slot before it is refilled
    }
  }

  // the two lane halves hold different keys of the same query
  if constexpr (FUSED) {
    float2* outp = reinterpret_cast<float2*>(ring);
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const float zz = z[rb] + xhalf(z[rb]);
      if (h == 0) outp[rb * 32 + n] = make_float2(ref[rb], zz);
    }
  } else {
    float2* outp = p.parts + ((int64_t)head * p.max_chunks + chunk_id) * p.rows_pad + gbase;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const float zz = z[rb] + xhalf(z[rb]);
      if (h == 0) outp[rb * 32 + n] = make_float2(ref[rb], zz);
    }
  }
  return next;
}

// Which (chunk, row group) a wave of a dense launch works on.  The waves of a workgroup take p.wg_groups row groups of
// the same chunk side by side, then the next chunk: the row groups of a chunk read the same keys at the same time, and
// in one compute unit the second reader finds them in L2 instead of fetching them through the fabric again.
struct WaveSlot {
  int chunk, group;
};
__device__ __forceinline__ WaveSlot wave_slot(const ScoreParams& p, int wave_id) {
  const int waves = (int)(blockDim.x >> 6), gpw = p.wg_groups, cpw = waves / gpw;
  WaveSlot s;
  s.chunk = uniform_i32((int)blockIdx.x * cpw + wave_id / gpw);
  s.group = uniform_i32((int)blockIdx.y * gpw + wave_id % gpw);
  return s;
}

// DYN = false (dense batches): the grid names the items, one per wave: (chunk, row group, layer x KV head).
// DYN = true (ragged batches, whose lengths the host does not know): one persistent wave per SIMD takes items from
// work lists in device memory until they are empty (see ItemLists).  A short chunk costs a ticket and a ring refill
// instead of a workgroup launch; the hand-out also evens out the ragged tail.
template <int NRB, bool DYN, int NST>
__global__ __launch_bounds__(64 * kWavesPerGroup, 1) void score_wave_pass1_kernel(ScoreParams p) {
  extern __shared__ u32x4 rings[];
  const int wave_id = uniform_i32((int)(threadIdx.x >> 6));
  u32x4* ring = rings + wave_id * (wave_lds(NST) / 16);
  const int lane = threadIdx.x & 63;
  unsigned voff[4];
  sub_dma_lane_offsets(voff, p.k_stride_token, lane);
  bf16x8 qf[NRB][8];
  if (!DYN) {
    const WaveSlot slot = wave_slot(p, wave_id);
    if (locate_uniform(p, slot.chunk).nkeys == 0) return;
    pass1_item<NRB, NST>(p, ring, slot.chunk, slot.group, (int)blockIdx.z, qf, voff, lane, nullptr);
    return;
  }
  const ItemLists lists = item_lists(p);
  const int home = home_list();
  TeamTickets tickets = team_tickets(rings, NST, wave_id);
  for (int k = 0; k < kLists; ++k) {  // this XCD's list first, then the others: no list is left undrained
    const int x = (home + k) & (kLists - 1);
    unsigned* work = tickets.leader ? p.work + x : nullptr;  // (only the leader of a team takes tickets)
    const unsigned n_items = lists.count(x);
    tickets.post(work != nullptr ? take_item(work, lane) : 0u, lane);
    for (;;) {  // every team leaves: the tickets only grow
      const unsigned ticket = tickets.next();
      if (ticket >= n_items) break;
      const Item a = lists.at(p, x, ticket, false);
      if (a.nkeys == 0) {  // (no chunk of a list is empty; if one were, it would only cost its ticket)
        tickets.post(work != nullptr ? take_item(work, lane) : 0u, lane);
        continue;
      }
      tickets.post(pass1_item<NRB, NST>(p, ring, a.chunk, a.block * p.wg_groups + wave_id, a.head, qf, voff, lane, work),
                   lane);
    }
  }
}

// Pass 2 of one chunk (arguments as pass1_item).  FUSED (score_fused_kernel): the query fragments are still in
// registers from pass 1 and the caller has filled off2.
template <int NRB, int NST, bool FUSED = false>
__device__ __forceinline__ unsigned pass2_item(const ScoreParams& p, u32x4* ring, int chunk_id, int group, int head,
                                               bf16x8 (&qf)[NRB][8], float (&off2)[NRB][16],
                                               const unsigned (&voff)[4], int lane, unsigned* work) {
  const Work w = locate_uniform(p, chunk_id);
  // (the division runs on the vector ALU: bring the quotient back to a scalar register)
  const int layer = uniform_i32(head / p.n_kv_heads), kv = head - layer * p.n_kv_heads;
  const int n = lane & 31, h = lane >> 5;
  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)w.seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = uniform_ptr(p.k + (int64_t)layer * p.k_stride_layer + (int64_t)w.seq * p.k_stride_seq +
                                      (int64_t)kv * p.k_stride_head + w.tok0 * p.k_stride_token);
  const float* lse = p.lse2 + (((int64_t)layer * p.batch + w.seq) * p.n_q_heads + (int64_t)kv * p.group) * p.n_pseudo;
  const int gbase = group * (NRB * 32);  // first row of this wave's row group
  // with several row groups each writes its own plane of column sums (group 0 straight into the
  // result); a small kernel adds the others onto it
  float* plane = group == 0 ? p.scores : p.partial + (int64_t)(group - 1) * p.n_layers * p.n_kv_heads * p.total_tokens;
  float* out = const_cast<float*>(uniform_ptr(plane + ((int64_t)layer * p.n_kv_heads + kv) * p.total_tokens + w.tok0));
  const int nsubs = (w.nkeys + 31) / 32;
#pragma unroll
  for (int i = 0; i < NST; ++i)
    sub_dma(ring + i * kSubVec, kbase, p.k_stride_token, (nsubs - 1 - i) * 32, w.nkeys, voff);
  if constexpr (!FUSED) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) frag_from_q(qf[rb], p, qbase, gbase + rb * 32 + n, h);
    if (NRB == 8) pin_q_in_agprs<NRB>(qf);
    // -lse2 of the rows this lane's accumulator registers hold; -inf for padding rows, which then add 0
    if ((reinterpret_cast<uintptr_t>(lse) & 15) == 0 && (p.rows & 3) == 0) {
      // the four rows of an accumulator quad are consecutive: one 16-byte load each
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int row = gbase + rb * 32 + acc_row(4 * b, h);
          const float4 v = row < p.rows ? *reinterpret_cast<const float4*>(lse + row) : make_float4(INFINITY, INFINITY, INFINITY, INFINITY);
          off2[rb][4 * b] = -v.x;
          off2[rb][4 * b + 1] = -v.y;
          off2[rb][4 * b + 2] = -v.z;
          off2[rb][4 * b + 3] = -v.w;
        }
    } else {
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = gbase + rb * 32 + acc_row(v, h);
          off2[rb][v] = row < p.rows ? -lse[row] : -INFINITY;
        }
    }
  }
  bf16x8 kf[8];
  wait_subblocks(NST - 1);
  wave_load_frags<NRB>(kf, ring, n, h);
  float unused_off[NRB], unused_acc[NRB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) unused_off[rb] = 0.0f;
  wave_walk<NRB, 2, NST, true>(ring, kbase, p.k_stride_token, w.nkeys, 0, nsubs, kf, qf, p.c, unused_off, off2,
                                        unused_acc, out, voff, n, h, nsubs - 1);
  const unsigned next = work != nullptr ? take_item(work, lane) : 0u;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  return next;
}

// (DYN as in pass 1.)  Heads and, inside a chunk, the keys are walked in the opposite order to pass 1: what pass 1
// read last (the ends of the chunks in flight, the heads of the last round) is still in the 256 MB memory-side cache
// when pass 2 starts.
template <int NRB, bool DYN, int NST>
__global__ __launch_bounds__(64 * kWavesPerGroup, 1) void score_wave_pass2_kernel(ScoreParams p) {
  extern __shared__ u32x4 rings[];
  const int wave_id = uniform_i32((int)(threadIdx.x >> 6));
  u32x4* ring = rings + wave_id * (wave_lds(NST) / 16);
  const int lane = threadIdx.x & 63;
  unsigned voff[4];
  sub_dma_lane_offsets(voff, p.k_stride_token, lane);
  bf16x8 qf[NRB][8];
  float off2[NRB][16];
  if (!DYN) {
    const WaveSlot slot = wave_slot(p, wave_id);
    if (locate_uniform(p, slot.chunk).nkeys == 0) return;
    pass2_item<NRB, NST>(p, ring, slot.chunk, slot.group, (int)(gridDim.z - 1 - blockIdx.z), qf, off2, voff, lane, nullptr);
    return;
  }
  const ItemLists lists = item_lists(p);
  const int home = home_list();
  TeamTickets tickets = team_tickets(rings, NST, wave_id);
  for (int k = 0; k < kLists; ++k) {  // this XCD's list first, then the others: no list is left undrained
    const int x = (home + k) & (kLists - 1);
    unsigned* work = tickets.leader ? p.work + x : nullptr;  // (only the leader of a team takes tickets)
    const unsigned n_items = lists.count(x);
    tickets.post(work != nullptr ? take_item(work, lane) : 0u, lane);
    for (;;) {  // every team leaves: the tickets only grow
      const unsigned ticket = tickets.next();
      if (ticket >= n_items) break;
      const Item a = lists.at(p, x, ticket, true);
      if (a.nkeys == 0) {  // (no chunk of a list is empty; if one were, it would only cost its ticket)
        tickets.post(work != nullptr ? take_item(work, lane) : 0u, lane);
        continue;
      }
      tickets.post(pass2_item<NRB, NST>(p, ring, a.chunk, a.block * p.wg_groups + wave_id, a.head, qf, off2, voff, lane, work),
                   lane);
    }
  }
}

// Both passes in one launch, for dense batches whose (layer, sequence, KV head) problems are one workgroup each: at
// most 256 query rows (one row group) and as many chunks per sequence as the workgroup has waves (1 to 4).  A wave walks its
// chunk forward for pass 1, the waves of the workgroup exchange their (reference, sum) pairs through LDS (their rings
// are drained then) and each merges them -- the arithmetic of score_combine_kernel, chunk by chunk in the same order,
// so lse2 and with it the scores have the bits of the three-kernel path -- and walks its chunk backward for pass 2 with
// the query fragments still in registers.  What this saves is everything between the passes: a kernel boundary at
// which every wave of the chip waits for the slowest, the combine kernel, the second placement of the workgroups and
// the second read of the queries.  lse2 is not written anywhere.
template <int NRB, int NST>
__global__ __launch_bounds__(64 * kWavesPerGroup, 1) void score_fused_kernel(ScoreParams p) {
  extern __shared__ u32x4 rings[];
  const int wave_id = uniform_i32((int)(threadIdx.x >> 6)), waves = (int)(blockDim.x >> 6);
  u32x4* ring = rings + wave_id * (wave_lds(NST) / 16);
  const int lane = threadIdx.x & 63, h = lane >> 5;
  unsigned voff[4];
  sub_dma_lane_offsets(voff, p.k_stride_token, lane);
  bf16x8 qf[NRB][8];
  const int chunk = uniform_i32((int)blockIdx.x * waves + wave_id);  // blockIdx.x is the sequence
  const int head = (int)blockIdx.z;
  pass1_item<NRB, NST, true>(p, ring, chunk, 0, head, qf, voff, lane, nullptr);
  __syncthreads();
  // lse2 of rows lane, lane + 64, ...: every wave merges all chunks itself
  constexpr int kRowsPerLane = NRB * 32 / 64;
  float lse[kRowsPerLane];
#pragma unroll
  for (int r = 0; r < kRowsPerLane; ++r) {
    const int row = r * 64 + lane;
    float m = -INFINITY;
    for (int w = 0; w < waves; ++w) {
      const float2 v = reinterpret_cast<const float2*>(rings + w * (wave_lds(NST) / 16))[row];
      if (v.y > 0.0f) m = fmaxf(m, v.x + log2f(v.y));
    }
    float sum = 0.0f;
    for (int w = 0; w < waves; ++w) {
      const float2 v = reinterpret_cast<const float2*>(rings + w * (wave_lds(NST) / 16))[row];
      if (v.y > 0.0f) sum += exp2f(v.x + log2f(v.y) - m);
    }
    lse[r] = (sum > 0.0f) ? m + log2f(sum) : 0.0f;
  }
  __syncthreads();  // everybody has read everybody's pairs: the rings may be overwritten
  // -lse2 of the rows this lane's accumulator registers hold, through the wave's own ring (rows beyond the head's: -inf,
  // they then add 0)
  float* mine = reinterpret_cast<float*>(ring);
#pragma unroll
  for (int r = 0; r < kRowsPerLane; ++r) mine[r * 64 + lane] = (r * 64 + lane) < p.rows ? -lse[r] : -INFINITY;
  asm volatile("" ::: "memory");  // (the reads below are of another type than the writes above)
  float off2[NRB][16];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const float4 v = *reinterpret_cast<const float4*>(mine + rb * 32 + acc_row(4 * b, h));
      off2[rb][4 * b] = v.x;
      off2[rb][4 * b + 1] = v.y;
      off2[rb][4 * b + 2] = v.z;
      off2[rb][4 * b + 3] = v.w;
    }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // off2 is out of the ring before pass 2 refills it
  pass2_item<NRB, NST, true>(p, ring, chunk, 0, head, qf, off2, voff, lane, nullptr);
}

// The causal block of the pseudo tokens' own keys (Sec. 4.1: they are prefilled in-sequence): one wave
// per (sequence, row group, layer x KV head) scores its Q rows against the n_pseudo pseudo keys, row
// i = row % n_pseudo seeing keys 0..i, and folds the result into lse2 in place.  Every row sees key 0,
// so its running maximum is finite from the first sub-block on.
struct PseudoParams {
  const uint16_t* kp;
  int64_t stride_layer, stride_seq, stride_head, stride_row;
};

template <int NRB>
__global__ __launch_bounds__(64, 1) void score_wave_pseudo_kernel(ScoreParams p, PseudoParams pp) {
  extern __shared__ u32x4 ring[];
  const int seq = blockIdx.x;
  const int layer = uniform_i32(blockIdx.z / p.n_kv_heads), kv = blockIdx.z - layer * p.n_kv_heads;
  const int lane = threadIdx.x, n = lane & 31, h = lane >> 5;
  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = uniform_ptr(pp.kp + (int64_t)layer * pp.stride_layer + (int64_t)seq * pp.stride_seq +
                                      (int64_t)kv * pp.stride_head);
  float* lse = p.lse2 + (((int64_t)layer * p.batch + seq) * p.n_q_heads + (int64_t)kv * p.group) * p.n_pseudo;
  const int gbase = blockIdx.y * (NRB * 32);
  unsigned voff[4];
  sub_dma_lane_offsets(voff, pp.stride_row, lane);
  bf16x8 qf[NRB][8];
  int last_key[NRB];
  float ref[NRB], z[NRB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    frag_from_q(qf[rb], p, qbase, gbase + rb * 32 + n, h);
    const int row = gbase + rb * 32 + n;
    last_key[rb] = (row < p.rows ? row : p.rows - 1) % p.n_pseudo;
    ref[rb] = -INFINITY;
    z[rb] = 0.0f;
  }
  bf16x8 kf[8];
  const int nsubs = (p.n_pseudo + 31) / 32;
  for (int sub = 0; sub < nsubs; ++sub) {
    sub_dma(ring, kbase, pp.stride_row, sub * 32, p.n_pseudo, voff);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wave_load_frags<NRB>(kf, ring, n, h);
    wave_sub_simple<NRB, true, false, true>(kf, qf, p.c, ref, z, sub * 32, p.n_pseudo, h, last_key);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the fragments are out of the slot before it is refilled
  }
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    const float zz = z[rb] + xhalf(z[rb]);
    const int row = gbase + rb * 32 + n;
    if (h == 0 && row < p.rows) {
      const float block = ref[rb] + log2f(zz);  // log2 of the block's sum; zz >= 1
      const float old = lse[row];
      const float m = fmaxf(old, block);
      lse[row] = m + log2f(__builtin_amdgcn_exp2f(old - m) + __builtin_amdgcn_exp2f(block - m));
    }
  }
}

// S = sum over row groups of their planes of column sums, in group order; group 0's plane is the
// result array itself.
__global__ void score_group_sum_kernel(const float* partial, float* scores, int64_t count, int n_groups) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
    float s = scores[e];
    for (int g = 1; g < n_groups; ++g) s += partial[(int64_t)(g - 1) * count + e];
    scores[e] = s;
  }
}

template <typename F>
int set_lds(F kernel, int bytes) { return set_max_dynamic_lds(reinterpret_cast<const void*>(kernel), bytes); }

// SIMDs of the current device (4 per compute unit); 4 if the device cannot be asked.
int simd_count() {
  static std::mutex mu;
  static int simds[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 4;
  std::lock_guard<std::mutex> lock(mu);
  if (simds[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 1;
    simds[dev] = 4 * cus;
  }
  return simds[dev];
}

// How a dense launch packs its waves into workgroups: `waves` to a workgroup (kWavesPerGroup or 1), of which `groups`
// are the row groups of one chunk side by side (see wave_slot) and waves / groups consecutive chunks.
struct GroupShape {
  int waves, groups;
  dim3 grid(const ScorePlan& plan, const dapq_shape* s) const {
    const int cpw = waves / groups;
    return dim3((unsigned)((plan.max_chunks + cpw - 1) / cpw), (unsigned)(plan.n_groups / groups),
                (unsigned)(s->n_layers * s->n_kv_heads));
  }
};
GroupShape group_shape(const dapq_shape* s, const ScorePlan& plan) {
  if (s->cu_seqlens != nullptr) return {1, 1};
  const int groups = plan.n_groups % 4 == 0 ? 4 : (plan.n_groups % 2 == 0 ? 2 : 1);
  int chunks = kWavesPerGroup / groups;  // consecutive chunks in a workgroup: every workgroup must be full
  while (chunks > 1 && plan.max_chunks % chunks != 0) chunks /= 2;
  return {groups * chunks, groups};
}

// Waves of a persistent team of a ragged launch: the row groups of a chunk side by side (see ItemLists).
int team_size(const ScorePlan& plan) { return plan.n_groups % 4 == 0 ? 4 : (plan.n_groups % 2 == 0 ? 2 : 1); }

int fill_params(const dapq_shape* s, const ScorePlan& plan, ScoreParams* p) {
  p->cu_seqlens = s->cu_seqlens;
  p->k_stride_layer = s->k_stride_layer; p->k_stride_seq = s->k_stride_seq;
  p->k_stride_head = s->k_stride_head; p->k_stride_token = s->k_stride_token;
  p->q_stride_layer = s->q_stride_layer; p->q_stride_seq = s->q_stride_seq;
  p->q_stride_head = s->q_stride_head; p->q_stride_row = s->q_stride_row;
  p->total_tokens = s->total_tokens;
  p->n_layers = s->n_layers; p->batch = s->batch; p->n_q_heads = s->n_q_heads; p->n_kv_heads = s->n_kv_heads;
  p->group = s->n_q_heads / s->n_kv_heads; p->n_pseudo = s->n_pseudo;
  p->rows = plan.rows; p->rows_pad = plan.rows_pad; p->n_groups = plan.n_groups;
  p->chunk_keys = plan.chunk_keys; p->max_chunks = (int32_t)plan.max_chunks;
  p->wg_groups = 1;
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
    hipLaunchKernelGGL(score_chunk_prefix_kernel, dim3(1), dim3(64), 0, stream, s->cu_seqlens, p.cu_chunks, p.work,
                       s->batch, plan.chunk_keys);
    DAPQ_HIP_LAUNCH_CHECK("score_chunk_prefix_kernel");
  }
  int rc = DAPQ_OK;
  const int64_t waves = plan.max_chunks * plan.n_groups * s->n_layers * s->n_kv_heads;
  const GroupShape gs = group_shape(s, plan);
  const int wpg = gs.waves;
  // ragged: persistent teams (one wave per SIMD; a team = the row groups of a chunk side by side) take their chunks
  // from work lists (32-bit tickets)
  const bool dyn = s->cu_seqlens != nullptr && waves < ((int64_t)1 << 31);
  const int team = dyn ? team_size(plan) : 1;
  p.wg_groups = dyn ? team : gs.groups;
  const int64_t teams = waves / team, team_slots = simd_count() / team;
  const dim3 dyn_grid((unsigned)(teams < team_slots ? teams : team_slots));
  const dim3 grid = gs.grid(plan, s);
#define DAPQ_LAUNCH_W1(NRBV)                                                                                        \
  do {                                                                                                              \
    if (dyn && team > 1) { /* (more than 256 rows: eight row blocks per wave) */                                    \
      const int lds = team * wave_lds(kTeamStages) + 16;                                                            \
      if ((rc = set_lds(score_wave_pass1_kernel<8, true, kTeamStages>, kWavesPerGroup * wave_lds(kTeamStages) + 16)) != \
          DAPQ_OK)                                                                                                  \
        return rc;                                                                                                  \
      hipLaunchKernelGGL((score_wave_pass1_kernel<8, true, kTeamStages>), dyn_grid, dim3(64 * team), lds, stream, p);   \
    } else if (dyn) {                                                                                               \
      if ((rc = set_lds(score_wave_pass1_kernel<NRBV, true, kWaveStages>, wave_lds(kWaveStages))) != DAPQ_OK) return rc; \
      hipLaunchKernelGGL((score_wave_pass1_kernel<NRBV, true, kWaveStages>), dyn_grid, dim3(64), wave_lds(kWaveStages), \
                         stream, p);                                                                                \
    } else {                                                                                                        \
      if ((rc = set_lds(score_wave_pass1_kernel<NRBV, false, kWaveStages>, kWavesPerGroup * wave_lds(kWaveStages))) !=  \
          DAPQ_OK)                                                                                                  \
        return rc;                                                                                                  \
      hipLaunchKernelGGL((score_wave_pass1_kernel<NRBV, false, kWaveStages>), grid, dim3(64 * wpg),                     \
                         wpg * wave_lds(kWaveStages), stream, p);                                                   \
    }                                                                                                               \
  } while (0)
  if (plan.row_blocks == 2) DAPQ_LAUNCH_W1(2);
  else if (plan.row_blocks == 4) DAPQ_LAUNCH_W1(4);
  else DAPQ_LAUNCH_W1(8);
#undef DAPQ_LAUNCH_W1
  DAPQ_HIP_LAUNCH_CHECK("score_wave_pass1_kernel");
  const int64_t rows_total = (int64_t)s->n_layers * s->batch * s->n_q_heads * s->n_pseudo;
  hipLaunchKernelGGL(score_combine_kernel, dim3((unsigned)((rows_total + 255) / 256)), dim3(256), 0, stream, p);
  DAPQ_HIP_LAUNCH_CHECK("score_combine_kernel");
  return DAPQ_OK;
}

int launch_accumulate(const dapq_shape* s, const ScorePlan& plan, ScoreParams p, hipStream_t stream) {
  if (s->cu_seqlens != nullptr) {
    // pass 2 can be called on its own: rebuild the chunk prefix it walks
    hipLaunchKernelGGL(score_chunk_prefix_kernel, dim3(1), dim3(64), 0, stream, s->cu_seqlens, p.cu_chunks, p.work,
                       s->batch, plan.chunk_keys);
    DAPQ_HIP_LAUNCH_CHECK("score_chunk_prefix_kernel");
  }
  int rc = DAPQ_OK;
  const int64_t waves = plan.max_chunks * plan.n_groups * s->n_layers * s->n_kv_heads;
  const GroupShape gs = group_shape(s, plan);
  const int wpg = gs.waves;
  // ragged: persistent teams (one wave per SIMD; a team = the row groups of a chunk side by side) take their chunks
  // from work lists (32-bit tickets)
  const bool dyn = s->cu_seqlens != nullptr && waves < ((int64_t)1 << 31);
  const int team = dyn ? team_size(plan) : 1;
  p.wg_groups = dyn ? team : gs.groups;
  const int64_t teams = waves / team, team_slots = simd_count() / team;
  const dim3 dyn_grid((unsigned)(teams < team_slots ? teams : team_slots));
  const dim3 grid = gs.grid(plan, s);
#define DAPQ_LAUNCH_W2(NRBV)                                                                                        \
  do {                                                                                                              \
    if (dyn && team > 1) { /* (more than 256 rows: eight row blocks per wave) */                                    \
      const int lds = team * wave_lds(kTeamStages) + 16;                                                            \
      if ((rc = set_lds(score_wave_pass2_kernel<8, true, kTeamStages>, kWavesPerGroup * wave_lds(kTeamStages) + 16)) != \
          DAPQ_OK)                                                                                                  \
        return rc;                                                                                                  \
      hipLaunchKernelGGL((score_wave_pass2_kernel<8, true, kTeamStages>), dyn_grid, dim3(64 * team), lds, stream, p);   \
    } else if (dyn) {                                                                                               \
      if ((rc = set_lds(score_wave_pass2_kernel<NRBV, true, kWaveStages>, wave_lds(kWaveStages))) != DAPQ_OK) return rc; \
      hipLaunchKernelGGL((score_wave_pass2_kernel<NRBV, true, kWaveStages>), dyn_grid, dim3(64), wave_lds(kWaveStages), \
                         stream, p);                                                                                \
    } else {                                                                                                        \
      if ((rc = set_lds(score_wave_pass2_kernel<NRBV, false, kWaveStages>, kWavesPerGroup * wave_lds(kWaveStages))) !=  \
          DAPQ_OK)                                                                                                  \
        return rc;                                                                                                  \
      hipLaunchKernelGGL((score_wave_pass2_kernel<NRBV, false, kWaveStages>), grid, dim3(64 * wpg),                     \
                         wpg * wave_lds(kWaveStages), stream, p);                                                   \
    }                                                                                                               \
  } while (0)
  if (plan.row_blocks == 2) DAPQ_LAUNCH_W2(2);
  else if (plan.row_blocks == 4) DAPQ_LAUNCH_W2(4);
  else DAPQ_LAUNCH_W2(8);
#undef DAPQ_LAUNCH_W2
  DAPQ_HIP_LAUNCH_CHECK("score_wave_pass2_kernel");
  if (plan.n_groups > 1) {
    const int64_t count = (int64_t)s->n_layers * s->n_kv_heads * s->total_tokens;
    const int64_t want = (count + 255) / 256;
    const unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 16384 ? 16384 : want));
    hipLaunchKernelGGL(score_group_sum_kernel, dim3(blocks), dim3(256), 0, stream, p.partial, p.scores, count,
                       plan.n_groups);
    DAPQ_HIP_LAUNCH_CHECK("score_group_sum_kernel");
  }
  return DAPQ_OK;
}

// Whether one launch of score_fused_kernel can do both passes: a dense batch, one row group, and the chunks of a
// sequence exactly the waves of a workgroup.
// Returns the waves of such a workgroup (1 to 4), or 0 if the passes have to be separate launches.
int fused_waves(const dapq_shape* s, const ScorePlan& plan) {
  if (s->cu_seqlens != nullptr || plan.n_groups != 1 || s->total_tokens == 0) return 0;
  const int64_t chunks_per_seq = plan.max_chunks / s->batch;  // dense: max_chunks = batch * chunks per sequence
  if (chunks_per_seq * s->batch != plan.max_chunks) return 0;
  return chunks_per_seq >= 1 && chunks_per_seq <= kWavesPerGroup ? (int)chunks_per_seq : 0;
}
bool fused_applies(const dapq_shape* s, const ScorePlan& plan) { return fused_waves(s, plan) != 0; }

int launch_fused(const dapq_shape* s, const ScorePlan& plan, ScoreParams p, hipStream_t stream) {
  const GroupShape gs = {fused_waves(s, plan), 1};
  p.wg_groups = 1;
  const dim3 grid((unsigned)s->batch, 1u, (unsigned)(s->n_layers * s->n_kv_heads));
  int rc = DAPQ_OK;
#define DAPQ_LAUNCH_F(NRBV)                                                                                            \
  do {                                                                                                                 \
    if ((rc = set_lds(score_fused_kernel<NRBV, kWaveStages>, kWavesPerGroup * wave_lds(kWaveStages))) != DAPQ_OK)     \
      return rc;                                                                                                       \
    hipLaunchKernelGGL((score_fused_kernel<NRBV, kWaveStages>), grid, dim3(64 * gs.waves),                             \
                       gs.waves * wave_lds(kWaveStages), stream, p);                                                   \
  } while (0)
  if (plan.row_blocks == 2) DAPQ_LAUNCH_F(2);
  else if (plan.row_blocks == 4) DAPQ_LAUNCH_F(4);
  else DAPQ_LAUNCH_F(8);
#undef DAPQ_LAUNCH_F
  DAPQ_HIP_LAUNCH_CHECK("score_fused_kernel");
  return DAPQ_OK;
}

int check_workspace(void* workspace, size_t workspace_bytes, const ScorePlan& plan) {
  DAPQ_REQUIRE(workspace != nullptr, DAPQ_ERR_INVALID_ARG, "workspace is NULL");
  DAPQ_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255) == 0, DAPQ_ERR_UNSUPPORTED,
               "workspace is not 256-byte aligned");
  DAPQ_REQUIRE(workspace_bytes >= plan.total_bytes, DAPQ_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed",
               workspace_bytes, plan.total_bytes);
  return DAPQ_OK;
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API int dapq_score_stats(const dapq_shape* shape, const void* q, const void* k, float* lse2,
                                         void* workspace, size_t workspace_bytes, void* stream) {
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
  p.work = reinterpret_cast<unsigned*>(ws + plan.off_work);
  p.parts = reinterpret_cast<float2*>(ws + plan.off_parts);
  p.lse2 = lse2;
  p.scores = nullptr;
  p.partial = nullptr;
  return launch_stats(shape, plan, p, static_cast<hipStream_t>(stream));
}

extern "C" DAPQ_API int dapq_score_accumulate(const dapq_shape* shape, const void* q, const void* k,
                                              const float* lse2, float* scores, void* workspace,
                                              size_t workspace_bytes, void* stream) {
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
  p.work = reinterpret_cast<unsigned*>(static_cast<char*>(workspace) + plan.off_work);
  p.parts = nullptr;
  p.partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan.off_partial);
  p.lse2 = const_cast<float*>(lse2);
  p.scores = scores;
  return launch_accumulate(shape, plan, p, static_cast<hipStream_t>(stream));
}

extern "C" DAPQ_API int dapq_score_single_launch(const dapq_shape* shape) {
  int rc = check_shape(shape, true, true, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  return fused_applies(shape, plan) ? 1 : 0;
}

extern "C" DAPQ_API int dapq_score(const dapq_shape* shape, const void* q, const void* k, float* scores,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape, true, true, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  DAPQ_REQUIRE(scores != nullptr, DAPQ_ERR_INVALID_ARG, "scores is NULL");
  if ((rc = check_workspace(workspace, workspace_bytes, plan)) != DAPQ_OK) return rc;
  if (fused_applies(shape, plan)) {
    if ((rc = aligned16(q, "q")) != DAPQ_OK) return rc;
    if ((rc = aligned16(k, "k")) != DAPQ_OK) return rc;
    ScoreParams p;
    fill_params(shape, plan, &p);
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.cu_chunks = nullptr;
    p.work = nullptr;
    p.parts = nullptr;
    p.partial = nullptr;
    p.lse2 = nullptr;
    p.scores = scores;
    return launch_fused(shape, plan, p, static_cast<hipStream_t>(stream));
  }
  float* lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan.off_lse2);
  if ((rc = dapq_score_stats(shape, q, k, lse2, workspace, workspace_bytes, stream)) != DAPQ_OK) return rc;
  return dapq_score_accumulate(shape, q, k, lse2, scores, workspace, workspace_bytes, stream);
}


extern "C" DAPQ_API int dapq_score_stats_extend(const dapq_shape* shape, const void* q, const void* k_pseudo,
                                                int64_t kp_stride_layer, int64_t kp_stride_seq, int64_t kp_stride_head,
                                                int64_t kp_stride_row, float* lse2, void* stream) {
  int rc = check_shape(shape, true, false, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  if ((rc = aligned16(q, "q")) != DAPQ_OK) return rc;
  if ((rc = aligned16(k_pseudo, "k_pseudo")) != DAPQ_OK) return rc;
  DAPQ_REQUIRE(lse2 != nullptr, DAPQ_ERR_INVALID_ARG, "lse2 is NULL");
  DAPQ_REQUIRE(kp_stride_layer >= 0 && kp_stride_seq >= 0 && kp_stride_head >= 0, DAPQ_ERR_INVALID_ARG,
               "k_pseudo strides must be >= 0");
  DAPQ_REQUIRE(kp_stride_row >= shape->head_dim && kp_stride_row < ((int64_t)1 << 26), DAPQ_ERR_INVALID_ARG,
               "kp_stride_row (%lld) must be in [head_dim, 2^26)", (long long)kp_stride_row);
  DAPQ_REQUIRE(kp_stride_layer % 8 == 0 && kp_stride_seq % 8 == 0 && kp_stride_head % 8 == 0 && kp_stride_row % 8 == 0,
               DAPQ_ERR_UNSUPPORTED, "k_pseudo strides must be multiples of 8 elements (16-byte rows)");
  DAPQ_REQUIRE(shape->batch <= 65535, DAPQ_ERR_UNSUPPORTED, "batch must be <= 65535");
  ScoreParams p;
  fill_params(shape, plan, &p);
  p.q = static_cast<const uint16_t*>(q);
  p.k = nullptr;
  p.cu_chunks = nullptr;
  p.work = nullptr;
  p.parts = nullptr;
  p.partial = nullptr;
  p.scores = nullptr;
  p.lse2 = lse2;
  PseudoParams pp;
  pp.kp = static_cast<const uint16_t*>(k_pseudo);
  pp.stride_layer = kp_stride_layer; pp.stride_seq = kp_stride_seq;
  pp.stride_head = kp_stride_head; pp.stride_row = kp_stride_row;
  const dim3 grid((unsigned)shape->batch, (unsigned)plan.n_groups, (unsigned)(shape->n_layers * shape->n_kv_heads));
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (plan.row_blocks == 2) hipLaunchKernelGGL(score_wave_pseudo_kernel<2>, grid, dim3(64), kSubBytes, st, p, pp);
  else if (plan.row_blocks == 4) hipLaunchKernelGGL(score_wave_pseudo_kernel<4>, grid, dim3(64), kSubBytes, st, p, pp);
  else hipLaunchKernelGGL(score_wave_pseudo_kernel<8>, grid, dim3(64), kSubBytes, st, p, pp);
  DAPQ_HIP_LAUNCH_CHECK("score_wave_pseudo_kernel");
  return DAPQ_OK;
}

// ---------------------------------------------------------------------------------------------
// dapq_score for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops):
// the workspace of the two passes lives in a file-scope device array instead of a caller buffer.
// ---------------------------------------------------------------------------------------------
namespace {

constexpr size_t kStaticScratchBytes = DAPQ_STATIC_SCRATCH_BYTES;
// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress: the device address it stands for is looked up once per device and kept below.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(DAPQ_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  DAPQ_REQUIRE(dev >= 0 && dev < kMaxDevices, DAPQ_ERR_UNSUPPORTED, "device index %d is beyond the %d this library tracks",
               dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr)
      return fail(DAPQ_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DAPQ_OK;
}

}  // namespace

extern "C" DAPQ_API size_t dapq_score_static_capacity(void) { return kStaticScratchBytes; }

extern "C" DAPQ_API int dapq_score_static(const dapq_shape* shape, const void* q, const void* k, float* scores,
                                          void* stream) {
  int rc = check_shape(shape, true, true, false);
  if (rc != DAPQ_OK) return rc;
  ScorePlan plan;
  if ((rc = make_score_plan(shape, &plan)) != DAPQ_OK) return rc;
  DAPQ_REQUIRE(plan.total_bytes <= kStaticScratchBytes, DAPQ_ERR_WORKSPACE,
               "this shape needs %zu bytes of workspace, the built-in scratch array holds %zu: use dapq_score with a "
               "caller workspace", plan.total_bytes, kStaticScratchBytes);
  void* ptr = nullptr;
  if ((rc = scratch_of_current_device(&ptr)) != DAPQ_OK) return rc;
  // nothing in the workspace has to start at zero: pass 1 writes every partial that the combine step reads, and
  // the combine step writes every lse2 that pass 2 reads
  return dapq_score(shape, q, k, scores, ptr, kStaticScratchBytes, stream);
}
