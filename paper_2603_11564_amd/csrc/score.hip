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
//
// The vector ALU is the busiest unit of this kernel (one FMA, one exponential, one add per logit),
// the matrix pipe second, so the full tiles run software pipelined from a single wave: while the
// MFMAs of one (sub-block, row block) unit execute, the lane exponentiates the logits of the unit
// before it, across tile boundaries, with one barrier per tile.
#include <math.h>

#include "dapq_internal.h"

namespace dapq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // 16 bytes; native vector, stays in registers

struct ScoreParams {
  const uint16_t* q;
  const uint16_t* k;
  const int32_t* cu_seqlens;  // NULL = dense
  int32_t* cu_chunks;         // [batch+1] prefix of per-sequence chunk counts (ragged only)
  float2* parts;              // [layer*Hkv][max_chunks][KW][rows_pad] (reference, sum) in the log2 domain
  float* lse2;                // [layer][batch][Hq][N]
  float* scores;              // [layer][Hkv][total_tokens]
  float* partial;             // [n_groups][layer][Hkv][total_tokens] per-row-group column sums (n_groups > 1)
  int64_t k_stride_layer, k_stride_seq, k_stride_head, k_stride_token;
  int64_t q_stride_layer, q_stride_seq, q_stride_head, q_stride_row;
  int64_t total_tokens;
  int32_t n_layers, batch, n_q_heads, n_kv_heads, group, n_pseudo;
  int32_t rows, rows_pad, n_super, n_groups, chunk_keys, max_chunks;
  float c;  // scale * log2(e)
};

constexpr int kThreads = 256;
constexpr int kTileBytes = kTileKeys * kHeadDim * 2;  // 32 KB
constexpr int kTileVec = kTileBytes / 16;             // 16-byte chunks per tile
constexpr int kLdsScore = 2 * kTileBytes;
constexpr int kSubBytes = 32 * kHeadDim * 2;          // one 32-key sub-block

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
// Branch-free: nkeys >= 1 and out-of-range rows are clamped to the last key of the chunk.
__device__ __forceinline__ void tile_load(u32x4 (&st)[8], const uint16_t* kbase, int64_t stride_token,
                                          int tile_key0, int nkeys, int tid) {
  const int ch = tid & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int key = (tid >> 4) + 16 * i;
    int gk = tile_key0 + key;
    gk = gk < nkeys ? gk : nkeys - 1;  // rows past the end repeat the last key; callers mask or drop them
    st[i] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)gk * stride_token + ch * 8);
  }
}

// LDS position of 16-byte chunk `ch` of tile row `key`: rows are 256 B apart, chunks XOR-swizzled by
// the row so that 16 consecutive rows reading the same logical chunk hit 16 different bank groups.
__device__ __forceinline__ int lds_chunk_index(int key, int ch) { return key * 16 + (ch ^ (key & 15)); }

__device__ __forceinline__ void tile_store(u32x4* buf, const u32x4 (&st)[8], int tid) {
  const int ch = tid & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int key = (tid >> 4) + 16 * i;
    buf[lds_chunk_index(key, ch)] = st[i];
  }
}

// The same tile moved straight from global memory into LDS (global_load_lds_dwordx4): no staging
// registers, no LDS store instructions.  Each wave instruction fills 1 KB = 4 tile rows; the lane
// that owns LDS slot (row, pos) fetches the logical chunk pos ^ (row & 15), which is the swizzle of
// lds_chunk_index.  Nothing is issued for a tile that starts past the end of the chunk.  The data
// is in LDS once the issuing wave's vmcnt has drained (tile_dma_wait) and a barrier has passed.
__device__ __forceinline__ void tile_dma(u32x4* buf, const uint16_t* kbase, int64_t stride_token, int tile_key0,
                                         int nkeys, int tid) {
  if (tile_key0 >= nkeys) return;
  const int wave = tid >> 6, lane = tid & 63;
  const int row0 = wave * 4 + (lane >> 4);  // tile rows of this lane: row0 + 16*i
  const int ch = (lane & 15) ^ (row0 & 15);
  if (tile_key0 + kTileKeys <= nkeys) {
    // full tile: one per-lane byte offset for all eight transfers, the rest is a uniform base
    const unsigned lane_off = (unsigned)row0 * (unsigned)stride_token * 2u + (unsigned)ch * 16u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const char* base = reinterpret_cast<const char*>(kbase + (int64_t)(tile_key0 + 16 * i) * stride_token);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + lane_off),
                                       (__attribute__((address_space(3))) void*)(buf + (i * 4 + wave) * 64), 16, 0, 0);
    }
  } else {
    // partial tile: rows past the end repeat the last key; callers mask or drop them
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int gk = tile_key0 + row0 + 16 * i;
      gk = gk < nkeys ? gk : nkeys - 1;
      const uint16_t* src = kbase + (int64_t)gk * stride_token + ch * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(buf + (i * 4 + wave) * 64), 16, 0, 0);
    }
  }
}

// Waits until at most `pending` of this wave's vector memory operations are still in flight.
template <int pending>
__device__ __forceinline__ void tile_dma_wait() {
  static_assert(pending == 0 || pending == 8, "only the two counts the kernels use");
  if (pending == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
}

// MFMA operand fragments of one 32-row sub-block held in LDS: fragment s of lane (n, h) is the
// 8 channels [(2s+h)*8, +8) of row n.
__device__ __forceinline__ void frag_from_lds(bf16x8 (&f)[8], const u32x4* buf, int sub, int n, int h) {
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const u32x4 v = buf[lds_chunk_index(sub * 32 + n, 2 * s + h)];
    f[s] = __builtin_bit_cast(bf16x8, v);
  }
}

// The same fragments for a 32-row block of Q read straight from global memory.
__device__ __forceinline__ void frag_from_q(bf16x8 (&f)[8], const ScoreParams& p, const uint16_t* qbase, int row,
                                            int h) {
  const int rc = row < p.rows ? row : p.rows - 1;  // padding rows repeat the last row; their results are dropped
  const int head = rc / p.n_pseudo, i = rc - head * p.n_pseudo;
  const uint16_t* src = qbase + (int64_t)head * p.q_stride_head + (int64_t)i * p.q_stride_row;
#pragma unroll
  for (int s = 0; s < 8; ++s) f[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + (2 * s + h) * 8));
}

__device__ __forceinline__ float xhalf(float v) { return __shfl_xor(v, 32, 64); }

// Row of the 32x32 MFMA result held in accumulator register v of a lane in half h.
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// ---------------------------------------------------------------------------------------------
// Software-pipelined walk over the full tiles of a chunk (both passes).
//
// A unit is one 32-key sub-block against one 32-row block of Q: 8 MFMAs, 16 logits per lane.  A
// slice is one MFMA of the current unit plus the exponentials of two logits of the previous unit
// (2 FMAs, the 2 adds of the exponentials issued one slice earlier, 2 transcendentals) and, in the
// second row block of a sub-block, one LDS fragment read for the next sub-block.  The slice order
// is pinned with an empty asm statement after each slice that takes the slice's results and the
// next slice's inputs as read-write operands: what produces them must come before it, what
// consumes them after it.  It emits no instruction.
// ---------------------------------------------------------------------------------------------
#define DAPQ_SLICE_END(cur, prev, e0, e1, sa, sb, addr) \
  asm volatile("" : "+v"(cur), "+v"(prev), "+v"(e0), "+v"(e1), "+v"(sa), "+v"(sb), "+v"(addr))

typedef const u32x4 __attribute__((address_space(3))) * lds_vec_ptr;

// 16-byte LDS read at a per-lane byte address plus a compile-time offset (folds into the instruction).
__device__ __forceinline__ bf16x8 lds_read16(unsigned lane_addr, int const_off) {
  return __builtin_bit_cast(bf16x8, *(lds_vec_ptr)(uintptr_t)(lane_addr + const_off));
}

// Column sums of a tile -> S (pass 2): lane halves hold different query rows of the same key (one
// shuffle), the RW slabs of a workgroup are added through LDS by the first 128 threads after a barrier.
template <int RW>
__device__ __forceinline__ void publish_columns(float* red, const float* col, int kw, int rw, int n, int h) {
  constexpr int KW = 4 / RW, NSUB = 4 / KW;
#pragma unroll
  for (int j = 0; j < NSUB; ++j) {
    const float v = col[j] + xhalf(col[j]);
    if (h == 0) red[rw * kTileKeys + (kw + j * KW) * 32 + n] = v;
  }
}

template <int RW>
__device__ __forceinline__ void store_columns(const float* red, float* out, int tile_key0, int nkeys, int tid) {
  if (tid < kTileKeys && tile_key0 + tid < nkeys) {
    float s = red[tid];
#pragma unroll
    for (int r = 1; r < RW; ++r) s += red[r * kTileKeys + tid];
    out[tile_key0 + tid] = s;
  }
}

// Entry contract of walk_tiles: tile t0 is in buffer t0 & 1 (landed and fenced) and the transfer of
// tile t0+1 into the other buffer has been started.  On return every transfer has landed and tile t1
// (the partial last tile, if the chunk has one) is in buffer t1 & 1, fenced.
//
// State of the pipelined walk.  Plain locals of the one function that owns the loop (walk_tiles), so
// that all of it stays in registers; the macros below are that function's body, unit by unit.
//
//   kf[8]   fragments of the sub-block whose MFMAs run next
//   prev    logits of the unit whose exponentials are being taken (cur: the unit being multiplied)
//   e0,e1   exponentials issued in the previous slice, added in the next
//   sa,sb   running sums of the unit being added up
//   fa[8]   per-lane LDS byte address of fragment s of the wave's first sub-block (constant)
//   acc[]   pass 1: zsum[2] row sums; pass 2: colp[NSUB] / colc[NSUB] column sums of the previous /
//           current tile (the last two units of a tile finish during the next one)
template <int RW, int PASS>
__device__ __forceinline__ void walk_tiles(u32x4* lds, const uint16_t* kbase, int64_t stride_token, int nkeys,
                                           int t0, int t1, const bf16x8 (&qf)[2][8], float c,
                                           const float (&off)[2][16], float (&zsum)[2], float* red, float* out,
                                           int tid, int kw, int rw, int n, int h) {
  constexpr int KW = 4 / RW, NSUB = 4 / KW, NUNIT = 2 * NSUB;
  constexpr int kRed = RW * kTileKeys;
  constexpr int LAG = NUNIT == 2 ? 2 : 1;  // pass 2: tiles by which the store to S trails (see below)
  const unsigned lds_base = (unsigned)(uintptr_t)(lds_vec_ptr)lds;
  unsigned fa[8];
#pragma unroll
  for (int s = 0; s < 8; ++s)
    fa[s] = lds_base + (unsigned)(n * 16 + ((2 * s + h) ^ (n & 15))) * 16u + (unsigned)(kw * kSubBytes);
  bf16x8 kf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) kf[s] = lds_read16(fa[s] + (t0 & 1) * kTileBytes, 0);
  f32x16 prev;
#pragma unroll
  for (int v = 0; v < 16; ++v) prev[v] = -INFINITY;  // 2^(-inf) = 0: the first slices add nothing
  float e0 = 0.0f, e1 = 0.0f, sa = 0.0f, sb = 0.0f;
  float colp[NSUB], colc[NSUB];
#pragma unroll
  for (int j = 0; j < NSUB; ++j) colp[j] = colc[j] = 0.0f;
  zsum[0] = zsum[1] = 0.0f;

  for (int t = t0; t < t1; ++t) {
    // two copies of the tile body so that the buffer offsets are instruction immediates
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      if ((t & 1) != par) continue;
      const int cur_base = par * kTileBytes, nxt_base = (par ^ 1) * kTileBytes;
#pragma unroll
      for (int u = 0; u < NUNIT; ++u) {
        const int j = u >> 1, rb = u & 1, rbp = rb ^ 1;
        if (u == NUNIT - 1) {
          // before the last unit: its fragment reads reach into the next tile, whose transfer was
          // started a tile ago and must have landed; every wave is past its reads of this tile's
          // buffer, so the tile after next can start to overwrite it
          tile_dma_wait<0>();
          __syncthreads();  // also fences the column sums published since the previous barrier
          tile_dma(lds + (t & 1) * kTileVec, kbase, stride_token, (t + 2) * kTileKeys, nkeys, tid);
          if (PASS == 2 && t - t0 >= LAG)
            store_columns<RW>(red + ((t - LAG) & 1) * kRed, out, (t - LAG) * kTileKeys, nkeys, tid);
        }
        f32x16 cur = {0};
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          if (PASS == 1) cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[rb][s], cur, 0, 0, 0);
          else cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][s], kf[s], cur, 0, 0, 0);
          if (rb == 1) {  // last use of this fragment: fetch the next sub-block's into its place
            if (j + 1 < NSUB) kf[s] = lds_read16(fa[s], cur_base + (j + 1) * KW * kSubBytes);
            else kf[s] = lds_read16(fa[s], nxt_base);
          }
          const float x0 = fmaf(prev[2 * s], c, PASS == 1 ? off[rbp][0] : off[rbp][2 * s]);
          const float x1 = fmaf(prev[2 * s + 1], c, PASS == 1 ? off[rbp][0] : off[rbp][2 * s + 1]);
          sa += e0;
          sb += e1;
          if (s == 0) {  // those were the last two logits of unit u-2: bank its sum
            const float total = sa + sb;
            sa = sb = 0.0f;
            if (PASS == 1) zsum[rb] += total;                  // unit u-2 has the row block of u
            else if (u >= 2) colc[(u - 2) >> 1] += total;
            else colp[NSUB - 1] += total;                      // the last two units of the previous tile
          }
          e0 = __builtin_amdgcn_exp2f(x0);
          e1 = __builtin_amdgcn_exp2f(x1);
          DAPQ_SLICE_END(cur, prev, e0, e1, sa, sb, fa[(s + 1) & 7]);
          if (PASS == 2 && u == 1 && s == 0 && t > t0)  // the previous tile's column sums are complete
            publish_columns<RW>(red + ((t - 1) & 1) * kRed, colp, kw, rw, n, h);
        }
        prev = cur;
      }
      if (PASS == 2) {
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
          colp[j] = colc[j];
          colc[j] = 0.0f;
        }
      }
    }
  }

  // drain: the exponentials of the last unit, with no MFMAs to hide behind
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const float x0 = fmaf(prev[2 * s], c, PASS == 1 ? off[1][0] : off[1][2 * s]);
    const float x1 = fmaf(prev[2 * s + 1], c, PASS == 1 ? off[1][0] : off[1][2 * s + 1]);
    sa += e0;
    sb += e1;
    if (s == 0) {  // closes unit NUNIT-2 of the last tile (row block 0, last sub-block)
      if (PASS == 1) zsum[0] += sa + sb;
      else colp[NSUB - 1] += sa + sb;
      sa = sb = 0.0f;
    }
    e0 = __builtin_amdgcn_exp2f(x0);
    e1 = __builtin_amdgcn_exp2f(x1);
  }
  const float total = (sa + e0) + (sb + e1);
  tile_dma_wait<0>();  // the transfer started before the last unit (a tile nobody reads, if any)
  if (PASS == 1) {
    zsum[1] += total;
    __syncthreads();
  } else {
    // The column sums of tile t are published after slice 0 of unit 1 of tile t+1; the barrier that
    // follows is the one before the last unit, so the store trails by LAG tiles (2 when a tile has
    // only two units and that barrier comes first).  Flush what is left.
    colp[NSUB - 1] += total;
    publish_columns<RW>(red + ((t1 - 1) & 1) * kRed, colp, kw, rw, n, h);
    __syncthreads();
    if (LAG == 2 && t1 - t0 >= 2)
      store_columns<RW>(red + ((t1 - 2) & 1) * kRed, out, (t1 - 2) * kTileKeys, nkeys, tid);
    store_columns<RW>(red + ((t1 - 1) & 1) * kRed, out, (t1 - 1) * kTileKeys, nkeys, tid);
  }
}

// ---------------------------------------------------------------------------------------------
// Pass 1
// ---------------------------------------------------------------------------------------------
// One tile the plain way: handles partial tiles (keys >= nkeys are masked out), fixes the reference
// logit on the wave's first sub-block (first), or tracks a running maximum (SAFE).
template <int RW, bool SAFE>
__device__ __forceinline__ void pass1_tile_simple(const u32x4* buf, const bf16x8 (&qf)[2][8], float c,
                                                  float (&ref)[2], float (&z)[2], int tile_key0, int nkeys, bool& first,
                                                  int kw, int n, int h) {
  constexpr int KW = 4 / RW;
  const bool full = tile_key0 + kTileKeys <= nkeys;
#pragma unroll 1
  for (int sub = kw; sub < 4; sub += KW) {
    const int sub_key0 = tile_key0 + sub * 32;
    if (sub_key0 >= nkeys) break;
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
          if (sub_key0 + acc_row(v, h) >= nkeys) acc[v] = -INFINITY;
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

// The plain walk: every tile through pass1_tile_simple (the overflow redo, and chunks with fewer
// than two full tiles).
template <int RW, bool SAFE>
__device__ __forceinline__ void pass1_chunk_simple(const ScoreParams& p, const Work& w, const uint16_t* kbase,
                                                   const bf16x8 (&qf)[2][8], u32x4* lds, float (&ref)[2], float (&z)[2]) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
  const int kw = wave / RW;
  const int ntiles = (w.nkeys + kTileKeys - 1) / kTileKeys;
  bool first = !SAFE;
  ref[0] = ref[1] = -INFINITY;
  z[0] = z[1] = 0.0f;
  u32x4 st[8];
  tile_load(st, kbase, p.k_stride_token, 0, w.nkeys, tid);
  for (int t = 0; t < ntiles; ++t) {
    u32x4* buf = lds + (t & 1) * kTileVec;
    tile_store(buf, st, tid);
    __syncthreads();
    tile_load(st, kbase, p.k_stride_token, (t + 1) * kTileKeys, w.nkeys, tid);
    pass1_tile_simple<RW, SAFE>(buf, qf, p.c, ref, z, t * kTileKeys, w.nkeys, first, kw, n, h);
  }
  __syncthreads();  // every wave is done with the last tile before the buffers are reused
}

// The fast walk: tile 0 the plain way (it fixes the reference logits), full tiles 1.. pipelined,
// a partial last tile the plain way again.  Needs at least two full tiles.
template <int RW>
__device__ __forceinline__ void pass1_chunk_pipelined(const ScoreParams& p, const Work& w, const uint16_t* kbase,
                                                      const bf16x8 (&qf)[2][8], u32x4* lds, float (&ref)[2],
                                                      float (&z)[2]) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
  const int kw = wave / RW;
  const int nfull = w.nkeys / kTileKeys;
  const bool tail = (w.nkeys % kTileKeys) != 0;
  bool first = true;
  ref[0] = ref[1] = -INFINITY;
  z[0] = z[1] = 0.0f;

  tile_dma(lds, kbase, p.k_stride_token, 0, w.nkeys, tid);
  tile_dma(lds + kTileVec, kbase, p.k_stride_token, kTileKeys, w.nkeys, tid);
  tile_dma_wait<8>();  // tile 0 has landed, tile 1 may still be in flight
  __syncthreads();
  pass1_tile_simple<RW, false>(lds, qf, p.c, ref, z, 0, w.nkeys, first, kw, n, h);
  tile_dma_wait<0>();
  __syncthreads();  // tile 1 is in; every wave is done with tile 0's buffer
  tile_dma(lds, kbase, p.k_stride_token, 2 * kTileKeys, w.nkeys, tid);

  float off[2][16];
  off[0][0] = -ref[0];
  off[1][0] = -ref[1];
  float zsum[2];
  walk_tiles<RW, 1>(lds, kbase, p.k_stride_token, w.nkeys, 1, nfull, qf, p.c, off, zsum, nullptr, nullptr, tid, kw,
                    0, n, h);
  z[0] += zsum[0];
  z[1] += zsum[1];
  if (tail)  // already stored and fenced before the last unit of the last full tile
    pass1_tile_simple<RW, false>(lds + (nfull & 1) * kTileVec, qf, p.c, ref, z, nfull * kTileKeys, w.nkeys, first, kw,
                                 n, h);
  __syncthreads();
}

template <int RW>
__global__ __launch_bounds__(kThreads, 2) void score_pass1_kernel(ScoreParams p) {
  extern __shared__ u32x4 lds[];
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
  if (w.nkeys >= 2 * kTileKeys) pass1_chunk_pipelined<RW>(p, w, kbase, qf, lds, ref, z);
  else pass1_chunk_simple<RW, false>(p, w, kbase, qf, lds, ref, z);
  // a sum that is not finite means a logit sat more than ~127 binades above the reference
  const bool bad = !(z[0] < INFINITY) || !(z[1] < INFINITY);
  if (__syncthreads_or(bad ? 1 : 0)) pass1_chunk_simple<RW, true>(p, w, kbase, qf, lds, ref, z);

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
// The plain way, for partial tiles and when the Q slab changes per super-group.
template <int RW>
__device__ __forceinline__ void pass2_tile_simple(const u32x4* buf, const bf16x8 (&qf)[2][8], float c,
                                                  const float (&nb)[2][16], float (&col)[4], int tile_key0, int nkeys,
                                                  int kw, int n, int h) {
  constexpr int KW = 4 / RW, NSUB = 4 / KW;
#pragma unroll
  for (int j = 0; j < NSUB; ++j) {
    const int sub = kw + j * KW;
    if (tile_key0 + sub * 32 >= nkeys) continue;
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

template <int RW, bool MULTI>
__global__ __launch_bounds__(kThreads, 2) void score_pass2_kernel(ScoreParams p) {
  extern __shared__ u32x4 lds[];
  float* red = reinterpret_cast<float*>(lds + kLdsScore / 16);  // [2][RW][128] partial column sums
  constexpr int kRed = RW * kTileKeys;
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

  // Q slab and the normalisers of its rows; reloaded per super-group when R > RW*64 (MULTI).
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
        const int rc = row < p.rows ? row : p.rows - 1;
        const float l = lse[rc];  // rows are laid out head-major: row = head*N + i
        nb[rb][v] = row < p.rows ? -l : -INFINITY;
      }
  };
  if (!MULTI) load_slab(0);

  const int ntiles = (w.nkeys + kTileKeys - 1) / kTileKeys;
  const int nfull = w.nkeys / kTileKeys;

  if (!MULTI && nfull >= 1) {
    // ---- pipelined: all full tiles in one stream, the partial last tile (if any) the plain way
    tile_dma(lds, kbase, p.k_stride_token, 0, w.nkeys, tid);
    tile_dma(lds + kTileVec, kbase, p.k_stride_token, kTileKeys, w.nkeys, tid);
    if (kTileKeys < w.nkeys) tile_dma_wait<8>();  // tile 0 has landed, tile 1 may still be in flight
    else tile_dma_wait<0>();
    __syncthreads();
    float zsum[2];
    walk_tiles<RW, 2>(lds, kbase, p.k_stride_token, w.nkeys, 0, nfull, qf, c, nb, zsum, red, out, tid, kw, rw, n, h);
    if (nfull < ntiles) {  // the partial tile is in its buffer already (stored and fenced in the walk)
      float col[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      pass2_tile_simple<RW>(lds + (nfull & 1) * kTileVec, qf, c, nb, col, nfull * kTileKeys, w.nkeys, kw, n, h);
      __syncthreads();  // the stores above have read red before it is overwritten
      publish_columns<RW>(red + (nfull & 1) * kRed, col, kw, rw, n, h);
      __syncthreads();
      store_columns<RW>(red + (nfull & 1) * kRed, out, nfull * kTileKeys, w.nkeys, tid);
    }
    return;
  }

  // ---- plain: one tile at a time, staged through registers
  u32x4 st[8];
  tile_load(st, kbase, p.k_stride_token, 0, w.nkeys, tid);
  for (int t = 0; t < ntiles; ++t) {
    u32x4* buf = lds + (t & 1) * kTileVec;
    tile_store(buf, st, tid);
    __syncthreads();
    tile_load(st, kbase, p.k_stride_token, (t + 1) * kTileKeys, w.nkeys, tid);
    const int tile_key0 = t * kTileKeys;
    float col[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (MULTI) {
      for (int sg = 0; sg < p.n_super; ++sg) {
        load_slab(sg);
        pass2_tile_simple<RW>(buf, qf, c, nb, col, tile_key0, w.nkeys, kw, n, h);
      }
    } else {
      pass2_tile_simple<RW>(buf, qf, c, nb, col, tile_key0, w.nkeys, kw, n, h);
    }
    publish_columns<RW>(red + (t & 1) * kRed, col, kw, rw, n, h);
    __syncthreads();
    store_columns<RW>(red + (t & 1) * kRed, out, tile_key0, w.nkeys, tid);
  }
}

// ---------------------------------------------------------------------------------------------
// Wave-private kernels (R <= 256 rows per KV head): one wave = all query rows x its own key stream.
//
// A workgroup is a single wave that keeps ALL the Q rows of the KV head in registers (up to eight
// 32-row blocks = 256 registers of MFMA operands; the launch bound of one wave per SIMD gives it the
// whole 512-register file) and walks its own chunk of keys.  Nothing is shared between waves, so
// there is no barrier anywhere and no cross-wave reduction: in pass 2 the lane that owns a key
// column sees every query row.  Keys arrive through a per-wave ring of 32-key sub-blocks in LDS
// (global_load_lds_dwordx4, five slots of 8 KB in pass 1: four sub-blocks = 32 KB in flight per
// wave, 128 KB per compute unit), and each fragment is read from LDS exactly once per wave.
//
// The instruction stream is the software pipeline described above, per (sub-block, row block)
// unit, with the exponentials trailing the MFMAs by one unit plus one slice so that the first
// result of a unit is not touched until a slice after its last MFMA issued.
// ---------------------------------------------------------------------------------------------
constexpr int kWaveStages1 = 5;           // pass 1: ring slots (40 KB per wave, 160 KB per compute unit)
constexpr int kWaveStages2 = 4;           // pass 2: one slot less, a 1 KB table of row offsets instead
constexpr int kSubVec = kSubBytes / 16;   // 512 16-byte chunks per sub-block
constexpr int kWaveLds1 = kWaveStages1 * kSubBytes;
constexpr int kWaveLds2 = kWaveStages2 * kSubBytes + 256 * (int)sizeof(float);

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
// transfer) and the lane part is one of the four precomputed offsets.  A sub-block that starts at or
// past the end of the chunk gets an empty descriptor: the eight transfers still count as vector
// memory operations (the waits rely on a fixed number per sub-block) but fetch nothing and fill the
// slot with zeros.
__device__ __forceinline__ void sub_dma(u32x4* slot, const uint16_t* kbase, int64_t stride_token, int key0, int nkeys,
                                        const unsigned (&voff)[4]) {
  const int64_t stride_b = stride_token * 2;
  const bool live = key0 < nkeys;
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
// of a unit issue, the 16 logits per lane of the unit before it enter the vector pipeline in 8
// steps: none in slice 0 (the transfer issue, the ring wait and the loop bookkeeping sit there, and
// the first logits are then more than a slice old), one in each of slices 1..6, two in slice 7.
// The sum a step adds to belongs to the pair three steps back: steps 0..2 of a unit still feed the
// unit two back.
// PASS 1: off1[rb] = -(reference logit * c) of row block rb; acc[rb] receives the row sums.
// PASS 2: the LDS table at byte address nbt holds -lse2 of every row (-inf for padding rows); the
//         16 values a lane needs for a row block (its accumulator rows) are fetched one unit ahead.
//         S of every key goes to out.
// NST = slots of the sub-block ring.
template <int NRB, int PASS, int NST>
__device__ __forceinline__ void wave_walk(u32x4* ring, const uint16_t* kbase, int64_t stride_token, int nkeys,
                                          int sb0, int sb1, bf16x8 (&kf)[8], const bf16x8 (&qf)[NRB][8], float c,
                                          const float (&off1)[NRB], unsigned nbt, float (&acc)[NRB], float* out,
                                          const unsigned (&voff)[4], int n, int h) {
  const unsigned ring_base = (unsigned)(uintptr_t)(lds_vec_ptr)ring;
  unsigned fa[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) fa[s] = ring_base + (unsigned)(n * 16 + ((2 * s + h) ^ (n & 15))) * 16u;
  const unsigned nba = nbt + (unsigned)h * 16u;  // pass 2: this lane's first table entry (row 4h)
  f32x16 prev;
#pragma unroll
  for (int v = 0; v < 16; ++v) prev[v] = -INFINITY;  // 2^(-inf) = 0: the first steps add nothing
  float x0 = -INFINITY, x1 = -INFINITY, ea0 = 0.0f, ea1 = 0.0f, eb0 = 0.0f, eb1 = 0.0f, sa = 0.0f, sb = 0.0f;
  f32x4 oc[4], on[4];  // pass 2: offsets of prev's rows / of cur's rows
#pragma unroll
  for (int b = 0; b < 4; ++b) oc[b] = on[b] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
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
        sub_dma(ring + issue_slot * kSubVec, kbase, stride_token, (sub + NST) * 32, nkeys, voff);
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
          if (s >= 1 && s <= 4)  // offsets of this unit's rows, needed from the next unit on
            on[s - 1] = *(const f32x4 __attribute__((address_space(3)))*)(uintptr_t)(nba + (rb * 32 + 8 * (s - 1)) * 4);
          if (s == 7) {
            DAPQ_VALU_STEP_K(6, prev[12], prev[13], oc[3][0], oc[3][1], sa, sb);
            DAPQ_VALU_STEP_K(7, prev[14], prev[15], oc[3][2], oc[3][3], sa, sb);
          } else if (s >= 1) {
            DAPQ_VALU_STEP_K(s - 1, prev[2 * s - 2], prev[2 * s - 1], oc[(2 * s - 2) >> 2][(2 * s - 2) & 3],
                             oc[(2 * s - 1) >> 2][(2 * s - 1) & 3], sa, sb);
            if (s == 3 && rb == 1) {
              // the adds above took in the last logits of the previous sub-block: its column sums are complete
              if (sub > sb0) {
                const float total = sa + sb;
                const float both = total + xhalf(total);
                const int key = (sub - 1) * 32 + n;
                if (h == 0 && key < nkeys) out[key] = both;
              }
              sa = sb = 0.0f;
            }
          }
          DAPQ_WAVE_SLICE_END(prev, x0, x1, sa, sb, fa[(s + 1) & 7]);
        } else {
          if (s == 7) {
            DAPQ_VALU_STEP_K(6, prev[12], prev[13], off1[rb1], off1[rb1], acc[rb1], acc[rb1]);
            DAPQ_VALU_STEP_K(7, prev[14], prev[15], off1[rb1], off1[rb1], acc[rb1], acc[rb1]);
          } else if (s >= 1 && s <= 3) {
            DAPQ_VALU_STEP_K(s - 1, prev[2 * s - 2], prev[2 * s - 1], off1[rb1], off1[rb1], acc[rb2], acc[rb2]);
          } else if (s >= 4) {
            DAPQ_VALU_STEP_K(s - 1, prev[2 * s - 2], prev[2 * s - 1], off1[rb1], off1[rb1], acc[rb1], acc[rb1]);
          }
          DAPQ_WAVE_SLICE_END(prev, x0, x1, acc[rb1], acc[rb2], fa[(s + 1) & 7]);
        }
      }
      prev = cur;
      if (PASS == 2) {
#pragma unroll
        for (int b = 0; b < 4; ++b) oc[b] = on[b];
      }
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
        DAPQ_VALU_STEP_K(k, a0, a1, oc[((2 * k) & 15) >> 2][(2 * k) & 3], oc[((2 * k + 1) & 15) >> 2][(2 * k + 1) & 3], sa,
                         sb);
      }
    }
    if (PASS == 2 && sb1 > sb0) {
      const float total = sa + sb;
      const float both = total + xhalf(total);
      const int key = (sb1 - 1) * 32 + n;
      if (h == 0 && key < nkeys) out[key] = both;
    }
  }
}

// One sub-block the plain way (pass 1): masks keys >= nkeys, fixes the reference logits (FIRST) or
// tracks a running maximum (SAFE).
template <int NRB, bool SAFE, bool FIRST>
__device__ __forceinline__ void wave_sub_simple(const bf16x8 (&kf)[8], const bf16x8 (&qf)[NRB][8], float c,
                                                float (&ref)[NRB], float (&z)[NRB], int key0, int nkeys, int h) {
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    f32x16 a = {0};
#pragma unroll
    for (int s = 0; s < 8; ++s) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[rb][s], a, 0, 0, 0);
    if (key0 + 32 > nkeys) {
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

template <int NRB>
__global__ __launch_bounds__(64, 1) void score_wave_pass1_kernel(ScoreParams p) {
  extern __shared__ u32x4 ring[];
  const Work w = locate(p, blockIdx.x);
  if (w.nkeys == 0) return;
  const int layer = blockIdx.z / p.n_kv_heads, kv = blockIdx.z - layer * p.n_kv_heads;
  const int lane = threadIdx.x, n = lane & 31, h = lane >> 5;
  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)w.seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = p.k + (int64_t)layer * p.k_stride_layer + (int64_t)w.seq * p.k_stride_seq +
                          (int64_t)kv * p.k_stride_head + w.tok0 * p.k_stride_token;
  const int gbase = blockIdx.y * (NRB * 32);  // first row of this wave's row group
  const int nsubs = (w.nkeys + 31) / 32, nfull = w.nkeys / 32;
  unsigned voff[4];
  sub_dma_lane_offsets(voff, p.k_stride_token, lane);
  // the ring is filled whether the sub-blocks exist or not (sub_dma): the waits count operations
#pragma unroll
  for (int i = 0; i < kWaveStages1; ++i) sub_dma(ring + i * kSubVec, kbase, p.k_stride_token, i * 32, w.nkeys, voff);
  bf16x8 qf[NRB][8];
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
  wait_subblocks(kWaveStages1 - 1);
  wave_load_frags<NRB>(kf, ring, n, h);
  // sub-block 0 the plain way: it fixes the reference logits
  wave_sub_simple<NRB, false, true>(kf, qf, p.c, ref, z, 0, w.nkeys, h);
  if (nsubs > 1) {
    wait_subblocks(kWaveStages1 - 2);
    wave_load_frags<NRB>(kf, ring + kSubVec, n, h);
    sub_dma(ring, kbase, p.k_stride_token, kWaveStages1 * 32, w.nkeys, voff);  // slot 0 is free
    if (nfull > 1) {
      float off[NRB], zs[NRB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) off[rb] = -ref[rb];
      wave_walk<NRB, 1, kWaveStages1>(ring, kbase, p.k_stride_token, w.nkeys, 1, nfull, kf, qf, p.c, off, 0u, zs, nullptr,
                                      voff, n, h);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) z[rb] += zs[rb];
    }
    if (nfull < nsubs && nfull >= 1)  // the partial last sub-block; its fragments are in kf
      wave_sub_simple<NRB, false, false>(kf, qf, p.c, ref, z, nfull * 32, w.nkeys, h);
  }
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
    }
  }

  // the two lane halves hold different keys of the same query
  float2* outp = p.parts + ((int64_t)blockIdx.z * p.max_chunks + blockIdx.x) * p.rows_pad + gbase;
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    const float zz = z[rb] + xhalf(z[rb]);
    if (h == 0) outp[rb * 32 + n] = make_float2(ref[rb], zz);
  }
}

template <int NRB>
__global__ __launch_bounds__(64, 1) void score_wave_pass2_kernel(ScoreParams p) {
  extern __shared__ u32x4 ring[];
  const Work w = locate(p, blockIdx.x);
  if (w.nkeys == 0) return;
  const int layer = blockIdx.z / p.n_kv_heads, kv = blockIdx.z - layer * p.n_kv_heads;
  const int lane = threadIdx.x, n = lane & 31, h = lane >> 5;
  const uint16_t* qbase = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)w.seq * p.q_stride_seq +
                          (int64_t)kv * p.group * p.q_stride_head;
  const uint16_t* kbase = p.k + (int64_t)layer * p.k_stride_layer + (int64_t)w.seq * p.k_stride_seq +
                          (int64_t)kv * p.k_stride_head + w.tok0 * p.k_stride_token;
  const float* lse = p.lse2 + (((int64_t)layer * p.batch + w.seq) * p.n_q_heads + (int64_t)kv * p.group) * p.n_pseudo;
  const int gbase = blockIdx.y * (NRB * 32);  // first row of this wave's row group
  // with several row groups each writes its own plane of column sums; a small kernel adds them up
  float* plane = p.n_groups > 1 ? p.partial + (int64_t)blockIdx.y * p.n_layers * p.n_kv_heads * p.total_tokens : p.scores;
  float* out = plane + ((int64_t)layer * p.n_kv_heads + kv) * p.total_tokens + w.tok0;
  const int nsubs = (w.nkeys + 31) / 32;
  unsigned voff[4];
  sub_dma_lane_offsets(voff, p.k_stride_token, lane);
#pragma unroll
  for (int i = 0; i < kWaveStages2; ++i) sub_dma(ring + i * kSubVec, kbase, p.k_stride_token, i * 32, w.nkeys, voff);
  // table of -lse2 per row behind the ring; -inf for padding rows, which then add 0
  float* nbt = reinterpret_cast<float*>(ring + kWaveStages2 * kSubVec);
#pragma unroll
  for (int r = lane; r < NRB * 32; r += 64) nbt[r] = gbase + r < p.rows ? -lse[gbase + r] : -INFINITY;
  bf16x8 qf[NRB][8];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) frag_from_q(qf[rb], p, qbase, gbase + rb * 32 + n, h);
  if (NRB == 8) pin_q_in_agprs<NRB>(qf);
  __syncthreads();  // one wave: orders the table writes before the reads below
  bf16x8 kf[8];
  wait_subblocks(kWaveStages2 - 1);
  wave_load_frags<NRB>(kf, ring, n, h);
  float unused_off[NRB], unused_acc[NRB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) unused_off[rb] = 0.0f;
  wave_walk<NRB, 2, kWaveStages2>(ring, kbase, p.k_stride_token, w.nkeys, 0, nsubs, kf, qf, p.c,
                                  unused_off, (unsigned)(uintptr_t)(lds_vec_ptr)(ring + kWaveStages2 * kSubVec),
                                  unused_acc, out, voff, n, h);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// S = sum over row groups of their planes of column sums, in group order.
__global__ void score_group_sum_kernel(const float* partial, float* scores, int64_t count, int n_groups) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
    float s = partial[e];
    for (int g = 1; g < n_groups; ++g) s += partial[(int64_t)g * count + e];
    scores[e] = s;
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
  p->rows = plan.rows; p->rows_pad = plan.rows_pad; p->n_super = plan.n_super; p->n_groups = plan.n_groups;
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
  int rc = DAPQ_OK;
  if (plan.wave_path) {
    const dim3 grid((unsigned)plan.max_chunks, (unsigned)plan.n_groups, (unsigned)(s->n_layers * s->n_kv_heads));
#define DAPQ_LAUNCH_W1(NRBV)                                                                        \
  do {                                                                                              \
    if ((rc = set_lds(score_wave_pass1_kernel<NRBV>, kWaveLds1)) != DAPQ_OK) return rc;              \
    hipLaunchKernelGGL(score_wave_pass1_kernel<NRBV>, grid, dim3(64), kWaveLds1, stream, p);        \
  } while (0)
    if (plan.row_blocks == 2) DAPQ_LAUNCH_W1(2);
    else if (plan.row_blocks == 4) DAPQ_LAUNCH_W1(4);
    else DAPQ_LAUNCH_W1(8);
#undef DAPQ_LAUNCH_W1
  } else {
    const dim3 grid((unsigned)plan.max_chunks, (unsigned)plan.n_super, (unsigned)(s->n_layers * s->n_kv_heads));
    if ((rc = set_lds(score_pass1_kernel<4>, kLdsScore)) != DAPQ_OK) return rc;
    hipLaunchKernelGGL(score_pass1_kernel<4>, grid, dim3(kThreads), kLdsScore, stream, p);
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
  int rc = DAPQ_OK;
  if (plan.wave_path) {
    const dim3 wgrid((unsigned)plan.max_chunks, (unsigned)plan.n_groups, (unsigned)(s->n_layers * s->n_kv_heads));
#define DAPQ_LAUNCH_W2(NRBV)                                                                        \
  do {                                                                                              \
    if ((rc = set_lds(score_wave_pass2_kernel<NRBV>, kWaveLds2)) != DAPQ_OK) return rc;              \
    hipLaunchKernelGGL(score_wave_pass2_kernel<NRBV>, wgrid, dim3(64), kWaveLds2, stream, p);       \
  } while (0)
    if (plan.row_blocks == 2) DAPQ_LAUNCH_W2(2);
    else if (plan.row_blocks == 4) DAPQ_LAUNCH_W2(4);
    else DAPQ_LAUNCH_W2(8);
#undef DAPQ_LAUNCH_W2
    if (plan.n_groups > 1) {
      DAPQ_HIP_LAUNCH_CHECK("score_wave_pass2_kernel");
      const int64_t count = (int64_t)s->n_layers * s->n_kv_heads * s->total_tokens;
      const unsigned blocks = (unsigned)(count + 255) / 256 < 16384u ? (unsigned)((count + 255) / 256) : 16384u;
      hipLaunchKernelGGL(score_group_sum_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, stream, p.partial,
                         p.scores, count, plan.n_groups);
    }
  } else {
    // more than 256 rows: four row waves, the Q slab changes per super-group
    const int lds_bytes = kLdsScore + 2 * 4 * kTileKeys * (int)sizeof(float);
    if ((rc = set_lds(score_pass2_kernel<4, true>, lds_bytes)) != DAPQ_OK) return rc;
    hipLaunchKernelGGL((score_pass2_kernel<4, true>), grid, dim3(kThreads), lds_bytes, stream, p);
  }
  DAPQ_HIP_LAUNCH_CHECK("score_pass2_kernel");
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
  p.parts = nullptr;
  p.partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan.off_partial);
  p.lse2 = const_cast<float*>(lse2);
  p.scores = scores;
  return launch_accumulate(shape, plan, p, static_cast<hipStream_t>(stream));
}

extern "C" DAPQ_API int dapq_score(const dapq_shape* shape, const void* q, const void* k, float* scores,
                                   void* workspace, size_t workspace_bytes, void* stream) {
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
