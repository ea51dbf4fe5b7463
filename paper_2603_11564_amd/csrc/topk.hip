// M_retain = TopK_j S(j) (Sec. 4.2): per (layer, sequence, KV head) the budget positions with the
// largest pooled score, equal scores lowest position first, written in ascending position.
//
// One workgroup per head (256 threads for short heads, 1024 from 8193 keys on).  Selection is an exact radix
// select on the order-preserving integer image of the fp32 score: four 8-bit digits from the top, each pass a
// 256-bin LDS histogram followed by a suffix scan that fixes one digit of the threshold T and the
// number of keys equal to T still needed.  The last step is an ordered compaction: key j is kept if
// score > T, or score == T and fewer than `need` equal keys precede it; prefix counts of (greater,
// equal) give both the decision and the output slot, so the result is ascending and deterministic
// (no atomic decides an order).  Max-pooling makes runs of bit-equal scores, so the tie rule is on
// the main path.
//
// Scores are positive and bunch into a few binades, so in the first pass all keys land in a handful of
// neighbouring bins: there each thread counts its keys in packed byte fields and the wave issues eight atomics.
// In the later passes each wave counts the candidates that share the digit of its first candidate with a
// reduction and issues one atomic for them; only the others go to the histogram one by one.
//
// Heads of up to 65536 keys (topk_reg_kernel) are read from HBM once into registers, thread t
// owning the consecutive keys [t*KPT, (t+1)*KPT): every pass runs out of registers and the
// compaction needs a single workgroup scan.  Because a thread holds a run of consecutive scores, the
// same kernel can apply the max-pool that precedes selection (Sec. 1 / Sec. 5.1) on the way in
// (dapq_pool_topk): three halo scores per side for the window of 7, no pooled array in HBM.
// Longer heads go through the same kernel in pieces of 32768 keys, each leaving its survivors in candidate lists
// (caller's workspace), and topk_merge_kernel selects among the candidates of a head; without the workspace
// topk_stream_kernel stages what fits in LDS (36864 keys) or re-reads the scores on every pass.
#include "dapq_internal.h"

namespace dapq {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kTopkLdsKeys = 36864;
constexpr int kTopkTailCap = 2048;
constexpr int kStreamTiles = 4;                            // tiles of 4096 keys the streaming kernel has in flight
constexpr int kStreamLdsHead = 260 + kStreamTiles * 16 + 60;  // words of LDS in front of its staged keys (16-byte aligned)

// Orders the LDS accesses of one wave's lanes among themselves (the hardware runs a wave's LDS instructions in
// order; this keeps the compiler from moving them).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

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
  // Long heads in pieces (cand_idx != NULL): workgroup (kv * n_segs + seg) selects among keys [seg * seg_len,
  // (seg + 1) * seg_len) of its head and leaves its survivors (order keys and positions in the head, ascending) and
  // their number in the candidate lists; topk_merge_kernel then selects among the candidates of a head.
  int32_t n_segs, seg_len;
  uint32_t* cand_key;   // [head][n_segs][budget]
  int32_t* cand_idx;    // [head][n_segs][budget]
  int32_t* cand_count;  // [head][n_segs]
};

// fp32 -> uint32 with the same order for all non-NaN values.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// What every variant needs to know about its head; heads of another launch (length outside
// [min_len, max_len]), keep == 0 and keep == L are finished here.
struct TopkHead {
  const float* src;   // first score of the piece this workgroup selects from (the whole head, or a segment of it)
  int32_t* out;
  uint32_t* out_key;  // segments: where the survivors' keys go (else NULL)
  int L, keep;        // length of the piece, how many of it survive
  int base, head_len; // where the piece starts in its head, and the head's length (pooling windows cross pieces)
  bool done;          // nothing left to select
  bool foreign;       // the head belongs to another launch
};

__device__ __forceinline__ TopkHead topk_head(const TopkParams& p) {
  TopkHead hd;
  const int tid = threadIdx.x;
  const bool pieces = p.cand_idx != nullptr;
  const int nseg = pieces ? p.n_segs : 1;
  const int kv = (int)blockIdx.x / nseg, seg = (int)blockIdx.x - kv * nseg, b = blockIdx.y, layer = blockIdx.z;
  int64_t start;
  if (p.cu_seqlens == nullptr) {
    hd.head_len = (int)(p.total_tokens / p.batch);
    start = (int64_t)b * hd.head_len;
  } else {
    start = p.cu_seqlens[b];
    hd.head_len = p.cu_seqlens[b + 1] - (int)start;
  }
  hd.base = 0;
  hd.out_key = nullptr;
  hd.foreign = hd.head_len < p.min_len || hd.head_len > p.max_len;
  if (hd.foreign) {
    hd.done = true;
    hd.keep = 0;
    hd.L = 0;
    hd.out = nullptr;
    hd.src = nullptr;
    return hd;
  }
  int want = p.budget_per_seq ? p.budget_per_seq[b] : p.budget;
  want = want < 0 ? 0 : (want > p.budget ? p.budget : want);
  const int64_t head = ((int64_t)layer * p.batch + b) * p.n_kv_heads + kv;
  const float* head_src = p.pooled + ((int64_t)layer * p.n_kv_heads + kv) * p.total_tokens + start;
  if (pieces) {
    hd.base = seg * p.seg_len;
    const int left = hd.head_len - hd.base;
    hd.L = left < 0 ? 0 : (left > p.seg_len ? p.seg_len : left);
    hd.keep = want < hd.L ? want : hd.L;
    const int64_t slot = head * nseg + seg;
    hd.out = p.cand_idx + slot * p.budget;
    hd.out_key = p.cand_key + slot * p.budget;
    hd.src = head_src + hd.base;
    if (tid == 0) p.cand_count[slot] = hd.keep;
    hd.done = hd.keep == 0;  // (a piece that survives whole still goes through the selection: its keys are wanted)
    return hd;
  }
  hd.L = hd.head_len;
  hd.keep = want < hd.L ? want : hd.L;
  hd.out = p.idx + head * p.budget;
  hd.src = head_src;
  if (tid == 0) p.count[head] = hd.keep;
  hd.done = hd.keep == 0;
  if (!hd.done && hd.keep == hd.L) {  // everything survives
    for (int j = tid; j < hd.L; j += (int)blockDim.x) hd.out[j] = j;
    hd.done = true;
  }
  return hd;
}

// Scans and reductions over the 64 lanes of a wave with data-parallel-primitive moves (a register-to-register
// move between lanes costs a few clocks; a shuffle goes through the LDS crossbar and takes over a hundred, and a
// scan is six of them in a chain).  A wave is four rows of 16 lanes: shifts by 1, 2, 4, 8 scan inside the rows
// (lanes without a source take the identity), then lane 15 of a row is handed to the whole next row (rows 1 and 3),
// then lane 31 to rows 2 and 3.
enum : int {
  kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118,
  kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143
};
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_take(uint32_t identity, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xf, false);
}
struct OpAdd {
  static constexpr uint32_t identity = 0u;
  __device__ __forceinline__ static uint32_t apply(uint32_t a, uint32_t b) { return a + b; }
};
struct OpMin {
  static constexpr uint32_t identity = 0xFFFFFFFFu;
  __device__ __forceinline__ static uint32_t apply(uint32_t a, uint32_t b) { return a < b ? a : b; }
};
struct OpMax {
  static constexpr uint32_t identity = 0u;
  __device__ __forceinline__ static uint32_t apply(uint32_t a, uint32_t b) { return a > b ? a : b; }
};
// inclusive scan in lane order: lane l gets op(v[0], ..., v[l])
template <class Op>
__device__ __forceinline__ uint32_t wave_scan(uint32_t v) {
  v = Op::apply(v, dpp_take<kDppRowShr1, 0xf>(Op::identity, v));
  v = Op::apply(v, dpp_take<kDppRowShr2, 0xf>(Op::identity, v));
  v = Op::apply(v, dpp_take<kDppRowShr4, 0xf>(Op::identity, v));
  v = Op::apply(v, dpp_take<kDppRowShr8, 0xf>(Op::identity, v));
  v = Op::apply(v, dpp_take<kDppRowBcast15, 0xa>(Op::identity, v));
  v = Op::apply(v, dpp_take<kDppRowBcast31, 0xc>(Op::identity, v));
  return v;
}
// the reduction over all lanes, in every lane
template <class Op>
__device__ __forceinline__ uint32_t wave_reduce(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_scan<Op>(v), 63);
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { return wave_reduce<OpAdd>(v); }

// After a histogram pass: wave 0 finds the digit d of T, the one with greater(d) < need <= greater(d)
// + hist[d], and publishes (d, need - greater(d), hist[d]) in bcast.
__device__ __forceinline__ void topk_pick_digit(const uint32_t* hist, uint32_t* bcast, int need, int lane) {
  // lane l owns digits 4l..4l+3; suffix sums over the lanes above, then inside the lane
  const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
  const uint32_t mine = h0 + h1 + h2 + h3;
  const uint32_t upto = wave_scan<OpAdd>(mine);  // keys whose digit is <= 4l+3
  const uint32_t above = (uint32_t)__builtin_amdgcn_readlane((int)upto, 63) - upto;  // keys whose digit is > 4l+3
  const uint32_t g3 = above, g2 = g3 + h3, g1 = g2 + h2, g0 = g1 + h1;  // keys with a larger digit
  const uint32_t un = (uint32_t)need;
  if (g3 < un && un <= g3 + h3) { bcast[0] = 4 * lane + 3; bcast[1] = un - g3; bcast[2] = h3; }
  if (g2 < un && un <= g2 + h2) { bcast[0] = 4 * lane + 2; bcast[1] = un - g2; bcast[2] = h2; }
  if (g1 < un && un <= g1 + h1) { bcast[0] = 4 * lane + 1; bcast[1] = un - g1; bcast[2] = h1; }
  if (g0 < un && un <= g0 + h0) { bcast[0] = 4 * lane + 0; bcast[1] = un - g0; bcast[2] = h0; }
}

// Whether a register variant brings its head in through an LDS staging area of THREADS * (KPT + 4) words (launched
// as dynamic LDS): the variant for 8K..32K keys, which has a compute unit to itself anyway.  The short-head variants
// share a compute unit and would lose occupancy to the area; 64 keys per thread times 1024 threads do not fit.
constexpr bool reg_variant_is_staged(int threads, int kpt) { return threads == 1024 && kpt == 32; }
constexpr int reg_variant_stage_bytes(int threads, int kpt) {  // (two more rows: the halos of the first and last thread)
  return reg_variant_is_staged(threads, kpt) ? (threads + 2) * (kpt + 4) * (int)sizeof(float) : 0;
}

// ---- selection among the keys a workgroup holds in registers (KPT per thread, thread t's before thread t+1's):
// the `keep` largest, ties to the lowest position, handed to emit(i, slot) in ascending position order (register
// i of the calling thread is survivor number `slot`).  A register without a key holds 0 (a key is at least 1);
// n_empty = how many of this thread's registers are empty.  keep >= 1 and at most the number of keys.
template <int THREADS, int KPT, class Emit>
__device__ __forceinline__ void topk_select(const uint32_t (&key)[KPT], int n_empty, int keep, Emit emit) {
  constexpr int kWaves = THREADS / 64;
  static_assert(KPT <= 255, "the first pass counts a thread's keys in 8-bit fields");
  __shared__ uint32_t hists[2][256];  // passes alternate: the next one's is cleared while wave 0 reads this one's
  __shared__ uint32_t bcasts[5][3];   // one row per pass (no pass waits for the readers of the one before), one for the tail
  __shared__ uint32_t tail[kTopkTailCap];  // low halves of the candidates left after two passes
  __shared__ uint32_t tail_n;
  __shared__ uint32_t wave_gt[kWaves], wave_eq[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // ---- radix select: threshold T = the keep-th largest key, need = how many keys == T to take
  uint32_t prefix = 0, mask = 0;
  int need = keep;
  for (int e = tid; e < 256; e += THREADS) hists[0][e] = 0;
  if (tid == 0) tail_n = 0;
  __syncthreads();
  // What ends a pass: wave 0 finds the digit of T among the 256 counts while the others clear the next pass's
  // histogram (its last reader was wave 0, two barriers ago); returns how many candidates remain.
  auto settle = [&](int pass, int shift) -> uint32_t {
    __syncthreads();
    if (wave == 0) topk_pick_digit(hists[pass & 1], bcasts[pass], need, lane);
    else
      for (int e = tid - 64; e < 256; e += THREADS - 64) hists[(pass + 1) & 1][e] = 0;
    __syncthreads();
    prefix |= bcasts[pass][0] << shift;
    mask |= 255u << shift;
    need = (int)bcasts[pass][1];
    return bcasts[pass][2];
  };

  {
    // First pass: every key is a candidate and its digit is the sign and seven exponent bits.  Scores are sums of
    // probabilities: a wave's 64 * KPT digits fall into a handful of neighbouring bins, where one LDS atomic per
    // key would serialise on a few addresses.  If the wave's digits span at most 8 bins, each thread counts its
    // keys in eight 8-bit fields (KPT <= 255), the wave adds the fields up and eight lanes issue one atomic each.
    // (A register without a key holds 0: key - 1 wraps to the largest value and never is the minimum; for a key
    // whose low 24 bits are all 0 the minimum comes out one bin low, which only widens the span by one.)
    uint32_t* hist = hists[0];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      kmin = key[i] - 1u < kmin ? key[i] - 1u : kmin;
      kmax = key[i] > kmax ? key[i] : kmax;
    }
    const uint32_t dmin = wave_reduce<OpMin>(kmin) >> 24, dmax = wave_reduce<OpMax>(kmax) >> 24;
    if (dmax >= dmin && dmax - dmin < 8u) {  // (uniform over the wave; dmax < dmin: the wave holds no key)
      // the registers without a key are counted too, all in the field that digit 0 wraps to, and taken out after
      uint64_t fields = 0;
#pragma unroll
      for (int i = 0; i < KPT; ++i) fields += 1ull << ((((key[i] >> 24) - dmin) * 8u) & 63u);
      fields -= (uint64_t)n_empty << (((0u - dmin) * 8u) & 63u);
      // two bins per 32-bit word, 16 bits each: a wave's count is at most 64 * KPT < 65536
      uint32_t pair[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint32_t lo = (uint32_t)(fields >> (16 * b)) & 255u, hi = (uint32_t)(fields >> (16 * b + 8)) & 255u;
        pair[b] = wave_sum(lo | (hi << 16));
      }
      if (lane < 8) {
        const uint32_t w = lane < 2 ? pair[0] : (lane < 4 ? pair[1] : (lane < 6 ? pair[2] : pair[3]));
        const uint32_t c = (lane & 1) ? (w >> 16) : (w & 0xFFFFu);
        if (c != 0) atomicAdd(&hist[dmin + lane], c);
      }
    } else if (dmax >= dmin) {
#pragma unroll
      for (int i = 0; i < KPT; ++i)
        if (key[i] != 0u) atomicAdd(&hist[key[i] >> 24], 1u);
    }
    settle(0, 24);
  }

  // The other passes.  (From here on the registers without a key are not told apart: they hold 0, can only be
  // candidates while the prefix is 0, are then the least of all candidates, and there are always at least `need` real
  // ones above them.)
  for (int shift = 16; shift >= 0; shift -= 8) {
    const int pass = (24 - shift) >> 3;
    uint32_t* hist = hists[pass & 1];
    // the digit most candidates of this wave are likely to share: that of its first candidate
    int first = -1;
#pragma unroll
    for (int i = KPT - 1; i >= 0; --i)
      if ((key[i] & mask) == prefix) first = (int)((key[i] >> shift) & 255u);
    const uint64_t have = __ballot(first >= 0);
    if (have != 0) {
      const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane(first, __ffsll((long long)have) - 1);
      uint32_t same = 0;
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        const bool cand = (key[i] & mask) == prefix;
        const uint32_t d = (key[i] >> shift) & 255u;
        same += cand && d == d0 ? 1u : 0u;
        if (__ballot(cand && d != d0) != 0) {  // (skipped by the whole wave when nobody has one)
          if (cand && d != d0) atomicAdd(&hist[d], 1u);
        }
      }
      same = wave_sum(same);
      if (lane == 0 && same != 0) atomicAdd(&hist[d0], same);
    }
    const uint32_t left = settle(pass, shift);  // candidates that remain
    if (shift == 16 && left <= (uint32_t)kTopkTailCap) {
      // Few candidates remain (typically a few dozen): instead of two more rounds of the whole workgroup, with
      // their barriers, their low halves go to a list and one wave finishes the selection on its own.
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        const bool cand = (key[i] & mask) == prefix;
        if (__ballot(cand) != 0) {  // rare: most waves hold no candidate at all
          if (cand) tail[atomicAdd(&tail_n, 1u)] = key[i] & 0xFFFFu;
        }
      }
      __syncthreads();
      if (wave == 0) {
        uint32_t pre = 0, msk = 0;
        uint32_t* h = hists[0];
        uint32_t* bc = bcasts[4];
        for (int sh = 8; sh >= 0; sh -= 8) {
#pragma unroll
          for (int e = 0; e < 4; ++e) h[4 * lane + e] = 0;
          wave_lds_sync();
          for (uint32_t e = lane; e < left; e += 64) {
            const uint32_t v = tail[e];
            if ((v & msk) == pre) atomicAdd(&h[(v >> sh) & 255u], 1u);
          }
          wave_lds_sync();
          topk_pick_digit(h, bc, need, lane);
          wave_lds_sync();
          pre |= bc[0] << sh;
          msk |= 255u << sh;
          need = (int)bc[1];
          wave_lds_sync();
        }
        if (lane == 0) bc[0] = pre;  // bc[1] holds the final `need`
      }
      __syncthreads();
      prefix |= bcasts[4][0];
      need = (int)bcasts[4][1];
      break;
    }
  }
  const uint32_t T = prefix;

  // ---- ordered compaction: one exclusive scan of the per-thread (greater, equal) counts
  uint32_t my_gt = 0, my_eq = 0;
#pragma unroll
  for (int i = 0; i < KPT; ++i) {  // (T is a key, so T >= 1 and registers without a key count as neither)
    my_gt += key[i] > T ? 1u : 0u;
    my_eq += key[i] == T ? 1u : 0u;
  }
  const uint32_t inc_gt = wave_scan<OpAdd>(my_gt), inc_eq = wave_scan<OpAdd>(my_eq);  // inclusive, inside the wave
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
    const bool eq = key[i] == T;
    const bool take = key[i] > T || (eq && pre_eq < un);
    if (__ballot(take) != 0) {  // survivors are few: most of a wave's registers hold none
      if (take) emit(i, pos);
    }
    pos += take ? 1u : 0u;
    pre_eq += eq ? 1u : 0u;
  }
}

// ---- heads that fit in registers.  R > 0: the input is the un-pooled score and the kernel applies
// the max-pool of radius R itself (window clipped at the ends of the sequence) before selecting.
template <int THREADS, int KPT, int R>
__global__ __launch_bounds__(THREADS) void topk_reg_kernel(TopkParams p) {
  constexpr bool kStaged = reg_variant_is_staged(THREADS, KPT);
  const int tid = threadIdx.x;
  const TopkHead hd = topk_head(p);
  if (hd.foreign || (hd.done && p.pooled_out == nullptr)) return;  // a finished head may still owe its pooled scores
  const int L = hd.L;
  // position j of this piece is a position of its head (the pooling window does not stop at the end of a piece)
  auto in_head = [&](int j) { return (unsigned)(hd.base + j) < (unsigned)hd.head_len; };

  // thread t owns keys [t*KPT, t*KPT + KPT): registers i < nvalid hold a key.  (A layout with
  // contiguous rows per wave makes the compaction twice as long.)
  const int j0 = tid * KPT;
  const int nvalid = L - j0 < 0 ? 0 : (L - j0 > KPT ? KPT : L - j0);
  float ext[KPT + 2 * R];  // scores j0-R .. j0+KPT+R-1; -inf outside the sequence
  if (kStaged) {
    // The head comes in with coalesced 16-byte loads (a thread reading its own run straight from memory makes
    // every load instruction touch 64 cache lines, and the halo loads as many again) and is dealt out to its
    // owners through LDS.  Row t + 1 of the staging area is thread t's run; rows are KPT + 4 words apart, which keeps
    // them 16-byte aligned and spreads consecutive rows over the banks.  Row 0 ends with the four scores before the
    // piece and row THREADS + 1 starts with the four after it (neighbouring pieces of a long head), if the head has them.
    extern __shared__ float stage_area[];
    constexpr int kRow = KPT + 4;
    float* stage = stage_area + kRow;  // row 0 of `stage` is thread 0's
    static_assert(R <= 4, "the halo of a run is read as one 16-byte piece of each neighbouring row");
    if ((reinterpret_cast<uintptr_t>(hd.src) & 15) == 0) {
#pragma unroll
      for (int it = 0; it < KPT / 4; ++it) {
        const int g = (it * THREADS + tid) * 4;
        if (g + 4 <= L) {
          *reinterpret_cast<float4*>(&stage[(g / KPT) * kRow + (g % KPT)]) = *reinterpret_cast<const float4*>(hd.src + g);
        } else {
          for (int k = 0; k < 4 && g + k < L; ++k) stage[(g / KPT) * kRow + (g % KPT) + k] = hd.src[g + k];
        }
      }
    } else {
      for (int j = tid; j < L; j += THREADS) stage[(j / KPT) * kRow + (j % KPT)] = hd.src[j];
    }
    if (R > 0 && tid < 8) {
      const int j = tid < 4 ? tid - 4 : THREADS * KPT + (tid - 4);
      const float v = in_head(j) ? hd.src[j] : -INFINITY;
      if (tid < 4) stage[-kRow + KPT - 4 + tid] = v;
      else stage[THREADS * kRow + (tid - 4)] = v;
    }
    __syncthreads();
    // (words of the area that no key was written to are never selected below)
#pragma unroll
    for (int i = 0; i < KPT; i += 4) {
      const float4 v = *reinterpret_cast<const float4*>(&stage[tid * kRow + i]);
      ext[R + i] = i < nvalid ? v.x : -INFINITY;
      ext[R + i + 1] = i + 1 < nvalid ? v.y : -INFINITY;
      ext[R + i + 2] = i + 2 < nvalid ? v.z : -INFINITY;
      ext[R + i + 3] = i + 3 < nvalid ? v.w : -INFINITY;
    }
    if (R > 0) {
      const float4 lv = *reinterpret_cast<const float4*>(&stage[(tid - 1) * kRow + KPT - 4]);
      const float4 rv = *reinterpret_cast<const float4*>(&stage[(tid + 1) * kRow]);
      const float left[4] = {lv.x, lv.y, lv.z, lv.w}, right[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
      for (int r = 0; r < R; ++r) {  // (words of the area nobody wrote lie outside the head)
        ext[r] = in_head(j0 - R + r) ? left[4 - R + r] : -INFINITY;
        ext[R + KPT + r] = in_head(j0 + KPT + r) ? right[r] : -INFINITY;
      }
    }
  } else {
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
      ext[r] = in_head(jl) ? hd.src[jl] : -INFINITY;
      ext[R + KPT + r] = in_head(jr) ? hd.src[jr] : -INFINITY;
    }
  }
  uint32_t key[KPT];
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    float m = ext[i];
#pragma unroll
    for (int t = 1; t <= 2 * R; ++t) m = fmaxf(m, ext[i + t]);
    if (p.pooled_out != nullptr && i < nvalid) p.pooled_out[(hd.src - p.pooled) + j0 + i] = m;
    // registers past the end of the head hold 0, which no key is (a key is at least 1): everything below can then
    // tell them by value, and no per-register validity mask has to stay alive through the kernel
    const uint32_t k = order_key(m);
    key[i] = i < nvalid ? (k > 1u ? k : 1u) : 0u;
  }
  if (hd.done) return;


  topk_select<THREADS, KPT>(key, KPT - nvalid, hd.keep, [&](int i, uint32_t slot) {
    hd.out[slot] = hd.base + j0 + i;
    if (hd.out_key != nullptr) hd.out_key[slot] = key[i];
  });
}

// ---- a long head whose pieces have been through topk_reg_kernel: the `keep` largest of the candidates they left.
// A thread owns KPT consecutive slots of the head's [n_segs][budget] candidate lists; the slots a piece did not fill
// are empty.  Candidates are in ascending position inside a list and the lists in piece order, so ties still go to
// the lowest position and the result is ascending.
constexpr int kTopkMaxSegs = 64;
template <int THREADS, int KPT>
__global__ __launch_bounds__(THREADS) void topk_merge_kernel(TopkParams p) {
  __shared__ int32_t seg_count[kTopkMaxSegs];
  const int tid = threadIdx.x;
  const int kv = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
  int L;
  if (p.cu_seqlens == nullptr) L = (int)(p.total_tokens / p.batch);
  else L = p.cu_seqlens[b + 1] - p.cu_seqlens[b];
  if (L < p.min_len || L > p.max_len) return;
  int want = p.budget_per_seq ? p.budget_per_seq[b] : p.budget;
  want = want < 0 ? 0 : (want > p.budget ? p.budget : want);
  const int keep = want < L ? want : L;
  const int64_t head = ((int64_t)layer * p.batch + b) * p.n_kv_heads + kv;
  if (tid == 0) p.count[head] = keep;
  if (keep == 0) return;
  const int nseg = p.n_segs, slots = nseg * p.budget;
  if (tid < nseg) seg_count[tid] = p.cand_count[head * nseg + tid];
  __syncthreads();
  const uint32_t* ck = p.cand_key + head * slots;
  const int32_t* ci = p.cand_idx + head * slots;
  int32_t* out = p.idx + head * p.budget;
  const int s0 = tid * KPT;
  int seg = s0 / p.budget, r = s0 - seg * p.budget;
  uint32_t key[KPT];
  int n_empty = 0;
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const bool valid = s0 + i < slots && r < seg_count[seg < nseg ? seg : 0];
    key[i] = valid ? ck[s0 + i] : 0u;
    n_empty += valid ? 0 : 1;
    if (++r == p.budget) {
      r = 0;
      ++seg;
    }
  }
  topk_select<THREADS, KPT>(key, n_empty, keep, [&](int i, uint32_t slot) { out[slot] = ci[s0 + i]; });
}

// ---- longer heads
__global__ __launch_bounds__(kTopkThreads) void topk_stream_kernel(TopkParams p) {
  extern __shared__ uint32_t smem[];
  uint32_t* hist = smem;             // [256]
  uint32_t* bcast = smem + 256;      // [3]: digit, need, population of the digit
  uint32_t* wave_tot = smem + 260;   // [kStreamTiles][16]
  uint32_t* keys = smem + kStreamLdsHead;  // [kTopkLdsKeys] staged order keys (if they fit)

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
  // kStreamTiles tiles per trip, all their loads issued before the first key is looked at: with one workgroup per
  // head a pass is a chain of load latencies, and this is how many of them overlap

  // ---- radix select: threshold T = the keep-th largest key, need = how many keys == T to take
  uint32_t prefix = 0, mask = 0;
  int need = hd.keep;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int jb = 0; jb < L; jb += kStreamTiles * kTile) {  // the trip count is the same for every thread
      uint32_t k[kStreamTiles][4];
#pragma unroll
      for (int t = 0; t < kStreamTiles; ++t) keys_at(jb + t * kTile + 4 * tid, k[t]);
#pragma unroll
      for (int t = 0; t < kStreamTiles; ++t) {
        const int j = jb + t * kTile + 4 * tid;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool cand = j + u < L && (k[t][u] & mask) == prefix;
          const uint32_t d = (k[t][u] >> shift) & 255u;
          const uint64_t have = __ballot(cand);
          if (have != 0) {
            const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)d, __ffsll((long long)have) - 1);
            const uint64_t same = __ballot(cand && d == d0);
            if (cand && d != d0) atomicAdd(&hist[d], 1u);
            if (lane == 0) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
          }
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

  // ---- ordered compaction, kStreamTiles tiles of 4096 keys at a time: per-thread counts of (greater, equal) in
  // each tile, an inclusive scan inside the wave, wave totals through LDS, then every thread writes its survivors
  // in key order (all keys of a tile come before those of the next)
  uint32_t base_gt = 0, base_eq = 0;  // keys > T / == T before the current tile (same in all threads)
  const uint32_t un = (uint32_t)need;
  for (int jb = 0; jb < L; jb += kStreamTiles * kTile) {
    uint32_t k[kStreamTiles][4], my[kStreamTiles], inc[kStreamTiles];
#pragma unroll
    for (int t = 0; t < kStreamTiles; ++t) keys_at(jb + t * kTile + 4 * tid, k[t]);
#pragma unroll
    for (int t = 0; t < kStreamTiles; ++t) {
      const int j = jb + t * kTile + 4 * tid;
      my[t] = 0;  // (greater << 16) | equal over this thread's four keys of the tile
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j + u < L) my[t] += (k[t][u] > T ? 0x10000u : 0u) + (k[t][u] == T ? 1u : 0u);
      }
      inc[t] = wave_scan<OpAdd>(my[t]);
      if (lane == 63) wave_tot[t * kTopkWaves + wave] = inc[t];
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kStreamTiles; ++t) {
      const int j = jb + t * kTile + 4 * tid;
      uint32_t pre = inc[t] - my[t], blk = 0;  // packed counts before this thread inside the tile / of the whole tile
#pragma unroll
      for (int w = 0; w < kTopkWaves; ++w) {
        const uint32_t tot = wave_tot[t * kTopkWaves + w];
        if (w < wave) pre += tot;
        blk += tot;
      }
      uint32_t pre_gt = base_gt + (pre >> 16), pre_eq = base_eq + (pre & 0xFFFFu);
      if (my[t] != 0) {
        uint32_t pos = pre_gt + (pre_eq < un ? pre_eq : un);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (j + u < L) {
            if (k[t][u] > T) {
              out[pos++] = j + u;
            } else if (k[t][u] == T) {
              if (pre_eq < un) out[pos++] = j + u;
              ++pre_eq;
            }
          }
        }
      }
      base_gt += blk >> 16;
      base_eq += blk & 0xFFFFu;
    }
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
  if (len <= 512 * 32) return {512, 32};  // (32 keys per thread is the lean code: 64 per thread spills scalar registers)
  if (len <= 1024 * 32) return {1024, 32};
  return {1024, 64};
}

template <int R>
int launch_reg(RegVariant v, dim3 grid, hipStream_t st, const TopkParams& p) {
  if (v.threads == 256 && v.kpt == 32) hipLaunchKernelGGL((topk_reg_kernel<256, 32, R>), grid, dim3(256), 0, st, p);
  else if (v.threads == 512) hipLaunchKernelGGL((topk_reg_kernel<512, 32, R>), grid, dim3(512), 0, st, p);
  else if (v.kpt == 32) {
    constexpr int kBytes = reg_variant_stage_bytes(1024, 32);
    const int rc = set_max_dynamic_lds(reinterpret_cast<const void*>(topk_reg_kernel<1024, 32, R>), kBytes);
    if (rc != DAPQ_OK) return rc;
    hipLaunchKernelGGL((topk_reg_kernel<1024, 32, R>), grid, dim3(1024), kBytes, st, p);
  } else hipLaunchKernelGGL((topk_reg_kernel<1024, 64, R>), grid, dim3(1024), 0, st, p);
  return DAPQ_OK;
}

int launch_reg_radius(int radius, RegVariant v, dim3 grid, hipStream_t st, const TopkParams& p) {
  switch (radius) {
    case 0: return launch_reg<0>(v, grid, st, p);
    case 1: return launch_reg<1>(v, grid, st, p);
    case 2: return launch_reg<2>(v, grid, st, p);
    case 3: return launch_reg<3>(v, grid, st, p);
    default: return launch_reg<4>(v, grid, st, p);
  }
}

void launch_merge(RegVariant v, dim3 grid, hipStream_t st, const TopkParams& p) {
  if (v.threads == 256) hipLaunchKernelGGL((topk_merge_kernel<256, 32>), grid, dim3(256), 0, st, p);
  else if (v.kpt == 32) hipLaunchKernelGGL((topk_merge_kernel<1024, 32>), grid, dim3(1024), 0, st, p);
  else hipLaunchKernelGGL((topk_merge_kernel<1024, 64>), grid, dim3(1024), 0, st, p);
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

// Which kernels a batch goes to.  Heads that fit the chosen register variant go there; longer ones go in pieces of
// kTopkPieceLen keys through the variant for 32768 keys and a merge (if the caller brought the workspace for the
// candidate lists), else to the streaming kernel.  A dense batch knows its length; a ragged one launches both kinds,
// each skipping the heads of the other.
constexpr int kTopkPieceLen = 1024 * 32;
struct TopkRoute {
  RegVariant variant;
  int64_t reg_max;     // heads up to this length: the register variant
  bool any_short, any_long;
  // the long heads in pieces
  bool pieces_possible;
  int n_segs;
  size_t off_key, off_idx, off_count, pieces_bytes;
};

// with_pieces: the caller brought the workspace, so heads of more than one piece's length (32768 keys) need not go
// to the variant with 64 keys per thread (slower per key than two pieces and a merge) or to the streaming kernel.
TopkRoute topk_route(const dapq_shape* shape, int32_t budget, bool with_pieces) {
  TopkRoute r;
  const bool ragged = shape->cu_seqlens != nullptr;
  const int64_t mean = shape->total_tokens / shape->batch;
  const int64_t longest = ragged ? shape->total_tokens : mean;
  // a ragged batch sizes the variant for 1.5 x its mean length (or everything, if that is less)
  int64_t sized_for = !ragged ? mean : (mean + mean / 2 < longest ? mean + mean / 2 : longest);
  if (with_pieces && sized_for > kTopkPieceLen) sized_for = kTopkPieceLen;
  r.variant = reg_variant_for(sized_for);
  r.reg_max = r.variant.max_len();
  r.any_short = ragged || mean <= r.reg_max;  // (a dense batch of longer heads has nothing for the register variant)
  r.any_long = longest > r.reg_max;
  const int64_t n_segs = (longest + kTopkPieceLen - 1) / kTopkPieceLen;
  r.pieces_possible = r.any_long && n_segs <= kTopkMaxSegs && n_segs * budget <= 65536 &&
                      (int64_t)shape->n_kv_heads * n_segs <= 0x7FFFFFFF;
  r.n_segs = (int)n_segs;
  r.off_key = r.off_idx = r.off_count = r.pieces_bytes = 0;
  if (r.pieces_possible) {
    const size_t heads = (size_t)shape->n_layers * shape->batch * shape->n_kv_heads;
    const size_t list = align_up(heads * (size_t)n_segs * (size_t)budget * 4, 256);
    r.off_key = 0;
    r.off_idx = list;
    r.off_count = 2 * list;
    r.pieces_bytes = 2 * list + align_up(heads * (size_t)n_segs * 4, 256);
  }
  return r;
}

// The kernels for the long heads of a launch whose TopkParams are filled except for the long-head fields.
// radius > 0: the kernels of the pieces pool the scores themselves.
int launch_long_heads(const dapq_shape* shape, const TopkRoute& r, TopkParams p, int radius, void* workspace,
                      size_t workspace_bytes, hipStream_t st) {
  p.min_len = (int32_t)r.reg_max + 1;
  p.max_len = INT32_MAX;
  const dim3 grid((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers);
  if (r.pieces_possible && workspace != nullptr && workspace_bytes >= r.pieces_bytes) {
    char* ws = static_cast<char*>(workspace);
    p.n_segs = r.n_segs;
    p.seg_len = kTopkPieceLen;
    p.cand_key = reinterpret_cast<uint32_t*>(ws + r.off_key);
    p.cand_idx = reinterpret_cast<int32_t*>(ws + r.off_idx);
    p.cand_count = reinterpret_cast<int32_t*>(ws + r.off_count);
    const dim3 piece_grid((unsigned)(shape->n_kv_heads * r.n_segs), (unsigned)shape->batch, (unsigned)shape->n_layers);
    const int rc = launch_reg_radius(radius, RegVariant{1024, 32}, piece_grid, st, p);
    if (rc != DAPQ_OK) return rc;
    DAPQ_HIP_LAUNCH_CHECK("topk_reg_kernel (pieces)");
    // (one workgroup per long head: from 8193 candidate slots on, the large workgroup's sixteen waves)
    const int64_t slots = (int64_t)r.n_segs * p.budget;
    launch_merge(slots <= 256 * 32 ? RegVariant{256, 32} : (slots <= 1024 * 32 ? RegVariant{1024, 32} : RegVariant{1024, 64}),
                 grid, st, p);
    DAPQ_HIP_LAUNCH_CHECK("topk_merge_kernel");
    return DAPQ_OK;
  }
  DAPQ_REQUIRE(radius == 0, DAPQ_ERR_INVALID_ARG, "internal: the streaming kernel does not pool");
  // heads of up to kTopkLdsKeys keys are staged in LDS; if none of this launch can be that short the staging
  // area is left out
  const int lds_bytes = (kStreamLdsHead + (p.min_len <= kTopkLdsKeys ? kTopkLdsKeys : 0)) * (int)sizeof(uint32_t);
  // the limit is raised once, to the size with the staging area
  const int rc_lds = set_max_dynamic_lds(reinterpret_cast<const void*>(topk_stream_kernel),
                                         (kStreamLdsHead + kTopkLdsKeys) * (int)sizeof(uint32_t));
  if (rc_lds != DAPQ_OK) return rc_lds;
  hipLaunchKernelGGL(topk_stream_kernel, grid, dim3(kTopkThreads), lds_bytes, st, p);
  DAPQ_HIP_LAUNCH_CHECK("topk_stream_kernel");
  return DAPQ_OK;
}

TopkParams topk_params(const dapq_shape* shape, const float* in, float* pooled_out, int32_t budget,
                       const int32_t* budget_per_seq, int32_t* idx, int32_t* count) {
  TopkParams p;
  p.pooled = in;
  p.pooled_out = pooled_out;
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
  p.n_segs = 1;
  p.seg_len = 0;
  p.cand_key = nullptr;
  p.cand_idx = nullptr;
  p.cand_count = nullptr;
  return p;
}

}  // namespace
}  // namespace dapq

extern "C" DAPQ_API size_t dapq_topk_workspace_bytes(const dapq_shape* shape, int32_t budget) {
  if (check_shape(shape, false, false, false) != DAPQ_OK || budget < 1) return 0;
  return topk_route(shape, budget, true).pieces_bytes;
}

namespace dapq {
namespace {
// The route of a call: with the pieces if the caller's workspace holds their candidate lists.
TopkRoute topk_route_for(const dapq_shape* shape, int32_t budget, const void* workspace, size_t workspace_bytes) {
  const TopkRoute with = topk_route(shape, budget, true);
  if (with.pieces_possible && workspace != nullptr && workspace_bytes >= with.pieces_bytes) return with;
  return topk_route(shape, budget, false);
}
}  // namespace
}  // namespace dapq

extern "C" DAPQ_API int dapq_topk(const dapq_shape* shape, const float* pooled, int32_t budget, const int32_t* budget_per_seq,
                         int32_t* idx, int32_t* count, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = topk_common_checks(shape, pooled, budget, idx, count);
  if (rc != DAPQ_OK) return rc;
  TopkParams p = topk_params(shape, pooled, nullptr, budget, budget_per_seq, idx, count);
  const TopkRoute route = topk_route_for(shape, budget, workspace, workspace_bytes);
  const dim3 grid((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (route.any_short) {
    p.max_len = (int32_t)route.reg_max;
    if ((rc = launch_reg<0>(route.variant, grid, st, p)) != DAPQ_OK) return rc;
    DAPQ_HIP_LAUNCH_CHECK("topk_reg_kernel");
  }
  if (route.any_long) return launch_long_heads(shape, route, p, 0, workspace, workspace_bytes, st);
  return DAPQ_OK;
}

extern "C" DAPQ_API int dapq_pool_topk(const dapq_shape* shape, const float* scores, int32_t width, int32_t budget,
                                       const int32_t* budget_per_seq, int32_t* idx, int32_t* count, float* pooled,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  int rc = topk_common_checks(shape, scores, budget, idx, count);
  if (rc != DAPQ_OK) return rc;
  DAPQ_REQUIRE(width >= 1 && width <= 63 && (width & 1) == 1, DAPQ_ERR_INVALID_ARG,
               "width (%d) must be odd and in [1, 63]", width);
  DAPQ_REQUIRE(pooled != scores, DAPQ_ERR_INVALID_ARG, "pooled must not alias scores");
  const int64_t longest = shape->cu_seqlens == nullptr ? shape->total_tokens / shape->batch : shape->total_tokens;
  const dim3 grid((unsigned)shape->n_kv_heads, (unsigned)shape->batch, (unsigned)shape->n_layers);
  hipStream_t st = static_cast<hipStream_t>(stream);
  TopkParams p = topk_params(shape, scores, pooled, budget, budget_per_seq, idx, count);
  const TopkRoute route = topk_route_for(shape, budget, workspace, workspace_bytes);
  if (width <= 9 && route.any_long && route.pieces_possible && workspace != nullptr &&
      workspace_bytes >= route.pieces_bytes) {
    // heads of more than 32768 keys in pieces, whose kernels pool across the piece boundaries; the others in one
    // workgroup each
    if (route.any_short) {
      p.max_len = (int32_t)route.reg_max;
      if ((rc = launch_reg_radius(width / 2, route.variant, grid, st, p)) != DAPQ_OK) return rc;
      DAPQ_HIP_LAUNCH_CHECK("topk_reg_kernel");
    }
    return launch_long_heads(shape, route, p, width / 2, workspace, workspace_bytes, st);
  }
  if (width <= 9 && longest <= 64 * kTopkThreads) {
    // one kernel: every head fits a register variant, which pools on the way in
    if ((rc = launch_reg_radius(width / 2, reg_variant_for(longest), grid, st, p)) != DAPQ_OK) return rc;
    DAPQ_HIP_LAUNCH_CHECK("topk_reg_kernel");
    return DAPQ_OK;
  }
  DAPQ_REQUIRE(pooled != nullptr, DAPQ_ERR_UNSUPPORTED,
               "width %d / head length %lld need the two-kernel path: pass a pooled buffer (or, for width <= 9, a "
               "workspace of dapq_topk_workspace_bytes())", width, (long long)longest);
  if ((rc = dapq_pool(shape, scores, pooled, width, stream)) != DAPQ_OK) return rc;
  return dapq_topk(shape, pooled, budget, budget_per_seq, idx, count, workspace, workspace_bytes, stream);
}
