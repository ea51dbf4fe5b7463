// Queries of the pseudo tokens (Sec. 4.1): the model processes the pseudo tokens appended to the prompt
// only to obtain their queries.  For every layer the rows of the query projection's input that belong
// to the prompt tokens the pseudo tokens copy are gathered, multiplied with the layer's query weight
// (fp32 accumulation on v_mfma_f32_32x32x16_bf16), rounded to bf16 once, split into heads and written
// in the layout the score kernels read; the rotation to the positions L_p + i follows as the rope kernel.
//
//   q[layer][head][r][c] = bf16( sum_t x[layer][token_idx[r]][t] * w[layer][head*d + c][t] )
//
// The contraction is short in rows (batch * N pseudo tokens, 32 .. 128) and long in the weight
// (features x hidden, 32 MB per layer for a 4096-wide model), so the kernel is a stream over the
// weight: every weight element is read from HBM once and meets all rows of a sweep while it is in
// LDS.  A workgroup is ONE wave.  It owns FT tiles of 32 output features and MB blocks of 32 rows
// (FT * MB accumulator tiles, at most 128 registers) and walks the hidden axis in blocks of 64:
//   * the weight tile of a (hidden block, feature tile) "unit" is 32 rows x 128 B = 4 KB, four
//     buffer_load_dwordx4 ... lds transfers into a ring of four slots;
//   * the gathered x rows of a hidden block (MB * 4 KB) travel the same way, in FT parts that ride with
//     the units of the block before, so every unit issues the same number of transfers and the wait
//     before a unit is one constant s_waitcnt;
//   * rows are 128 B apart in LDS; 16-byte chunks are XOR-swizzled by bits 1..3 of the row so that
//     16 consecutive rows reading the same logical chunk hit 16 different bank groups.
// The weight is the A operand (D[feature][row]): a lane ends up with runs of four consecutive
// features of one row, stored as 8 bytes.  Nothing is shared between waves: no barrier anywhere.
// Work items are numbered sweep -> feature tile -> hidden split -> layer and dealt to the eight XCDs in
// contiguous ranges: the waves that read the same gathered rows share an L2, and the row sweeps of one
// feature tile run side by side, so the tile's weights leave HBM once.
// A call with too few tiles to fill the chip (a single layer) deals the hidden blocks of a tile to
// several waves; their fp32 sums go to a workspace and qproj_reduce_kernel adds them in a fixed order.
#include <math.h>

#include <type_traits>

#include "dapq_internal.h"

namespace dapq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct QprojParams {
  const uint16_t* x;
  const int32_t* token_idx;
  const uint16_t* w;
  uint16_t* q;
  int64_t x_stride_layer, x_stride_token;
  int64_t w_stride_layer, w_stride_row;
  int64_t q_stride_layer, q_stride_head, q_stride_row;
  int64_t total_tokens;
  int32_t n_layers, rows, hidden, n_features, head_dim;
  int32_t tiles_f, sweeps;
  int32_t k_splits, kb_per_split;  // hidden blocks are dealt to k_splits waves per tile; > 1 writes fp32 partial sums
  float* partial;                  // [k_splits][n_layers][sweeps * 32 MB rows][tiles_f * 32 FT features]
};

constexpr int kRing = 4;          // weight slots; a unit's transfers are issued four units ahead
constexpr int kBlockK = 64;       // hidden channels per block: 128-byte rows in LDS
constexpr int kTileBytes = 32 * kBlockK * 2;
constexpr int kTileVec = kTileBytes / 16;

__device__ __forceinline__ int qp_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t qp_rsrc(const void* base, int64_t bytes) {
  const unsigned records = bytes <= 0 ? 0u : (bytes > (int64_t)0xFFFFFFFFll ? 0xFFFFFFFFu : (unsigned)bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)records, 0x00020000);
}

// x buffers a kernel variant needs: the part of block b+1 that rides with the transfers of unit u + kRing
// must not land in a buffer whose block is still unread.
template <int FT>
struct XBuffers {
  static constexpr int value = (FT - 1 + kRing) / FT + 1;
};

template <int FT, int MB>
struct QprojLds {
  static constexpr int bytes = kRing * kTileBytes + XBuffers<FT>::value * MB * kTileBytes;
};

template <int N>
__device__ __forceinline__ void qp_wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int FT, int MB>
__global__ __launch_bounds__(64) void qproj_wave_kernel(QprojParams p) {
  constexpr int NXB = XBuffers<FT>::value;
  constexpr int XT = 4 * MB;       // 1 KB transfers per x block
  constexpr int XQ = XT / FT;      // of them riding with one unit
  constexpr int OPS = 4 + XQ;      // transfers per unit
  static_assert(XT % FT == 0 && (kRing % FT == 0) && (kRing - 1) * OPS <= 63, "unit bookkeeping");
  __shared__ u32x4 lds[QprojLds<FT, MB>::bytes / 16];
  u32x4* const wring = lds;
  u32x4* const xbuf = lds + kRing * kTileVec;

  const int lane = threadIdx.x, n = lane & 31, h = lane >> 5;
  // consecutive work items (all tiles of a layer, layer after layer) go to the same XCD when the grid
  // allows it: the waves that share a layer's x rows then share an L2
  int id = blockIdx.x;
  const int total = gridDim.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  id = qp_uniform(id);
  // the row sweeps of one feature tile are neighbours: they run at the same time and read the tile's weights
  // from HBM once
  const int sweep = qp_uniform(id % p.sweeps), rest = id / p.sweeps;
  const int tile = qp_uniform(rest % p.tiles_f), rest2 = rest / p.tiles_f;
  const int split = qp_uniform(rest2 % p.k_splits), layer = qp_uniform(rest2 / p.k_splits);
  const int f0 = tile * (32 * FT), m0 = sweep * (32 * MB);
  // this wave's hidden blocks [kb0, n_kb)
  const int kb0 = split * p.kb_per_split;
  const int n_kb = min(p.hidden / kBlockK, kb0 + p.kb_per_split);

  // ---- transfer addressing: lane (r0 = lane / 8, pos = lane % 8) fills LDS chunk `pos` of row 8i + r0 of a
  // tile with the logical chunk pos ^ (((8i + r0) >> 1) & 7) = pos ^ (r0 >> 1) ^ 4 (i & 1)
  const unsigned r0 = (unsigned)lane >> 3, pos = (unsigned)lane & 7u;
  const unsigned w_stride_b = (unsigned)(p.w_stride_row * 2);
  unsigned voff_w[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) voff_w[j] = r0 * w_stride_b + ((pos ^ (r0 >> 1) ^ (4u * j)) * 16u);
  unsigned voff_x[XT];
#pragma unroll
  for (int i = 0; i < XT; ++i) {
    const int row = m0 + 8 * i + (int)r0;
    const int tok = p.token_idx[row < p.rows ? row : p.rows - 1];  // padding rows repeat the last row; never stored
    // rows without a source read token 0; their results are replaced by zeros at the end
    voff_x[i] = (tok > 0 ? (unsigned)tok : 0u) * (unsigned)(p.x_stride_token * 2) + ((pos ^ (r0 >> 1) ^ (4u * (i & 1))) * 16u);
  }
  const __amdgpu_buffer_rsrc_t rsrc_none = qp_rsrc(p.x, 0);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      qp_rsrc(p.x + (int64_t)layer * p.x_stride_layer,
              p.total_tokens > 0 ? (p.total_tokens - 1) * p.x_stride_token * 2 + (int64_t)p.hidden * 2 : 0);
  __amdgpu_buffer_rsrc_t rsrc_w[FT];
#pragma unroll
  for (int t = 0; t < FT; ++t) {
    const int left = p.n_features - (f0 + 32 * t);  // feature rows from this tile to the end of the weight
    rsrc_w[t] = left > 0 ? qp_rsrc(p.w + (int64_t)layer * p.w_stride_layer + (int64_t)(f0 + 32 * t) * p.w_stride_row,
                                   (int64_t)(left - 1) * p.w_stride_row * 2 + (int64_t)p.hidden * 2)
                         : rsrc_none;
  }

  // transfers of the unit (hidden block kb, feature tile T): its weight tile into ring slot T-of-kb and part T
  // of the x rows of hidden block kb + 1.  Blocks past the end use the empty descriptor: the transfers
  // still count, fetch nothing and write zeros.
  auto issue = [&](int kb, auto tile_c) {
    constexpr int T = decltype(tile_c)::value;
    const bool live_w = kb < n_kb, live_x = kb + 1 < n_kb;
    const __amdgpu_buffer_rsrc_t rw = live_w ? rsrc_w[T] : rsrc_none;
    const __amdgpu_buffer_rsrc_t rx = live_x ? rsrc_x : rsrc_none;
    u32x4* const slot = wring + (((kb * FT) & (kRing - 1)) + T) * kTileVec;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void*)(slot + i * 64), 16,
                                               (int)voff_w[i & 1], (int)((unsigned)(8 * i) * w_stride_b + (unsigned)kb * 128u),
                                               0, 0);
    u32x4* const xb = xbuf + ((kb + 1) % NXB) * (MB * kTileVec);
#pragma unroll
    for (int i = T * XQ; i < (T + 1) * XQ; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(xb + i * 64), 16,
                                               (int)voff_x[i], (int)((unsigned)(kb + 1) * 128u), 0, 0);
  };

  // ---- prologue: x rows of the first block, then the first kRing units
  {
    u32x4* const xb = xbuf + (kb0 % NXB) * (MB * kTileVec);
#pragma unroll
    for (int i = 0; i < XT; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kb0 < n_kb ? rsrc_x : rsrc_none,
                                               (__attribute__((address_space(3))) void*)(xb + i * 64), 16, (int)voff_x[i],
                                               (int)((unsigned)kb0 * 128u), 0, 0);
    constexpr int kAhead = kRing / FT;  // hidden blocks the ring spans
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      issue(kb0 + a, std::integral_constant<int, 0>{});
      if constexpr (FT > 1) issue(kb0 + a, std::integral_constant<int, 1>{});
      if constexpr (FT > 2) {
        issue(kb0 + a, std::integral_constant<int, 2>{});
        issue(kb0 + a, std::integral_constant<int, 3>{});
      }
    }
  }

  f32x16 acc[FT][MB];
#pragma unroll
  for (int t = 0; t < FT; ++t)
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][rb][v] = 0.0f;

  // fragment s (16 hidden channels) of lane (n, h): the 8 channels [16 s + 8 h, +8) of row n = logical chunk 2s + h
  int frag_idx[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) frag_idx[s] = n * 8 + ((2 * s + h) ^ ((n >> 1) & 7));

  bf16x8 xf[MB][4];
  auto unit = [&](int kb, auto tile_c) {
    constexpr int T = decltype(tile_c)::value;
    qp_wait_vm<(kRing - 1) * OPS>();
    if constexpr (T == 0) {
      const u32x4* xb = xbuf + (kb % NXB) * (MB * kTileVec);
#pragma unroll
      for (int rb = 0; rb < MB; ++rb)
#pragma unroll
        for (int s = 0; s < 4; ++s) xf[rb][s] = __builtin_bit_cast(bf16x8, xb[rb * kTileVec + frag_idx[s]]);
    }
    const u32x4* slot = wring + (((kb * FT) & (kRing - 1)) + T) * kTileVec;
    bf16x8 wf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) wf[s] = __builtin_bit_cast(bf16x8, slot[frag_idx[s]]);
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int rb = 0; rb < MB; ++rb)
        acc[T][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s], xf[rb][s], acc[T][rb], 0, 0, 0);
    // the slot just read takes the tile of the unit kRing ahead (the MFMAs above have consumed the reads)
    issue(kb + kRing / FT, tile_c);
  };

  for (int kb = kb0; kb < n_kb; ++kb) {
    unit(kb, std::integral_constant<int, 0>{});
    if constexpr (FT > 1) unit(kb, std::integral_constant<int, 1>{});
    if constexpr (FT > 2) {
      unit(kb, std::integral_constant<int, 2>{});
      unit(kb, std::integral_constant<int, 3>{});
    }
  }
  qp_wait_vm<0>();

  // ---- epilogue: accumulator register v of lane (n, h) is feature 8 (v / 4) + 4 h + v % 4 of the tile, row n
  if (p.partial != nullptr) {
    // one of several waves of this tile: the fp32 sums go to this split's plane, padding included
    const int64_t rows_pad = (int64_t)p.sweeps * (32 * MB), feat_pad = (int64_t)p.tiles_f * (32 * FT);
    float* plane = p.partial + ((int64_t)split * p.n_layers + layer) * rows_pad * feat_pad;
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
      for (int t = 0; t < FT; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float4 o = make_float4(acc[t][rb][4 * g], acc[t][rb][4 * g + 1], acc[t][rb][4 * g + 2], acc[t][rb][4 * g + 3]);
          *reinterpret_cast<float4*>(plane + (int64_t)(m0 + 32 * rb + n) * feat_pad + f0 + 32 * t + 8 * g + 4 * h) = o;
        }
    return;
  }
#pragma unroll
  for (int rb = 0; rb < MB; ++rb) {
    const int row = m0 + 32 * rb + n;
    if (row >= p.rows) continue;
    const bool has_source = p.token_idx[row] >= 0;
    uint16_t* qrow = p.q + (int64_t)layer * p.q_stride_layer + (int64_t)row * p.q_stride_row;
#pragma unroll
    for (int t = 0; t < FT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int f = f0 + 32 * t + 8 * g + 4 * h;
        if (f >= p.n_features) continue;
        const int head = f / p.head_dim, c = f - head * p.head_dim;
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (__bf16)(has_source ? acc[t][rb][4 * g + e] : 0.0f);
        *reinterpret_cast<bf16x4*>(qrow + (int64_t)head * p.q_stride_head + c) = o;
      }
  }
}

// Adds the planes of the hidden splits in split order (the same order every run), rounds to bf16 once and
// writes the head layout.  One thread per run of four features of one row.
__global__ void qproj_reduce_kernel(QprojParams p, int rows_pad, int feat_pad) {
  const int quads = p.n_features / 4;  // head_dim is a multiple of 8
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_layer = (int64_t)p.rows * quads;
  if (gid >= per_layer * p.n_layers) return;
  const int layer = (int)(gid / per_layer);
  const int row = (int)((gid - layer * per_layer) / quads), f = (int)(gid % quads) * 4;
  const int64_t plane = (int64_t)p.n_layers * rows_pad * feat_pad;
  const float* src = p.partial + ((int64_t)layer * rows_pad + row) * feat_pad + f;
  float4 sum = *reinterpret_cast<const float4*>(src);
  for (int k = 1; k < p.k_splits; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(src + k * plane);
    sum.x += v.x;
    sum.y += v.y;
    sum.z += v.z;
    sum.w += v.w;
  }
  if (p.token_idx[row] < 0) sum = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  const int head = f / p.head_dim, c = f - head * p.head_dim;
  bf16x4 o;
  o[0] = (__bf16)sum.x;
  o[1] = (__bf16)sum.y;
  o[2] = (__bf16)sum.z;
  o[3] = (__bf16)sum.w;
  *reinterpret_cast<bf16x4*>(p.q + (int64_t)layer * p.q_stride_layer + (int64_t)head * p.q_stride_head +
                             (int64_t)row * p.q_stride_row + c) = o;
}

template <int FT, int MB>
void launch_qproj(const QprojParams& p, hipStream_t stream) {
  const int64_t grid = (int64_t)p.tiles_f * p.sweeps * p.k_splits * p.n_layers;
  hipLaunchKernelGGL((qproj_wave_kernel<FT, MB>), dim3((unsigned)grid), dim3(64), 0, stream, p);
}

// How a call is cut into waves; a pure function of the description so that the workspace query and the
// launcher agree.
struct QprojPlan {
  int ft, mb, tiles_f, sweeps, k_splits, kb_per_split;
  size_t workspace_bytes;
};

QprojPlan make_qproj_plan(const dapq_qproj& s) {
  QprojPlan pl;
  const int64_t features = (int64_t)s.n_q_heads * s.head_dim;
  // two row blocks per wave unless 32 rows are all there is
  pl.mb = s.rows > 32 ? 2 : 1;
  pl.sweeps = (int)(((int64_t)s.rows + 32 * pl.mb - 1) / (32 * pl.mb));
  // four feature tiles per wave while that still fills the chip (1024 SIMDs), two otherwise
  const int64_t waves4 = (features + 127) / 128 * pl.sweeps * s.n_layers;
  pl.ft = waves4 >= 768 ? 4 : 2;
  pl.tiles_f = (int)((features + 32 * pl.ft - 1) / (32 * pl.ft));
  // still too few waves: several waves per tile, each with a share of the hidden blocks (at least 8 per wave,
  // so that the ring's start-up is paid a few times at most), and one pass that adds their sums
  const int n_kb = s.hidden / kBlockK;
  const int64_t waves = (int64_t)pl.tiles_f * pl.sweeps * s.n_layers;
  pl.k_splits = 1;
  while (pl.k_splits < 16 && waves * pl.k_splits < 768 && n_kb / (pl.k_splits * 2) >= 8) pl.k_splits *= 2;
  pl.kb_per_split = (n_kb + pl.k_splits - 1) / pl.k_splits;
  pl.workspace_bytes = pl.k_splits == 1 ? 0
                                        : (size_t)pl.k_splits * s.n_layers * ((size_t)pl.sweeps * 32 * pl.mb) *
                                              ((size_t)pl.tiles_f * 32 * pl.ft) * sizeof(float);
  return pl;
}

int check_qproj(const dapq_qproj* desc) {
  DAPQ_REQUIRE(desc != nullptr, DAPQ_ERR_INVALID_ARG, "desc must not be NULL");
  const dapq_qproj& s = *desc;
  DAPQ_REQUIRE(s.n_layers >= 1 && s.rows >= 0 && s.hidden >= 1 && s.n_q_heads >= 1 && s.head_dim >= 1 &&
                   s.total_tokens >= 0,
               DAPQ_ERR_INVALID_ARG, "n_layers (%d), hidden (%d), n_q_heads (%d), head_dim (%d) must be >= 1, rows (%d) and total_tokens (%lld) >= 0",
               s.n_layers, s.hidden, s.n_q_heads, s.head_dim, s.rows, (long long)s.total_tokens);
  DAPQ_REQUIRE(s.hidden % kBlockK == 0, DAPQ_ERR_UNSUPPORTED, "hidden (%d) must be a multiple of %d", s.hidden, kBlockK);
  DAPQ_REQUIRE(s.head_dim % 8 == 0, DAPQ_ERR_UNSUPPORTED, "head_dim (%d) must be a multiple of 8", s.head_dim);
  DAPQ_REQUIRE((int64_t)s.n_q_heads * s.head_dim < ((int64_t)1 << 24), DAPQ_ERR_UNSUPPORTED,
               "n_q_heads * head_dim is too large");
  DAPQ_REQUIRE(s.x_stride_token >= s.hidden && s.w_stride_row >= s.hidden && s.x_stride_layer >= 0 && s.w_stride_layer >= 0,
               DAPQ_ERR_INVALID_ARG, "x_stride_token and w_stride_row must cover hidden, layer strides must be >= 0");
  DAPQ_REQUIRE(s.q_stride_row >= s.head_dim && s.q_stride_head >= s.head_dim && s.q_stride_layer >= 0, DAPQ_ERR_INVALID_ARG,
               "q_stride_row and q_stride_head must cover head_dim, q_stride_layer must be >= 0");
  DAPQ_REQUIRE(s.x_stride_token % 8 == 0 && s.w_stride_row % 8 == 0 && s.x_stride_layer % 8 == 0 &&
                   s.w_stride_layer % 8 == 0 && s.q_stride_row % 8 == 0 && s.q_stride_head % 8 == 0 &&
                   s.q_stride_layer % 8 == 0,
               DAPQ_ERR_UNSUPPORTED, "strides must be multiples of 8 elements");
  // lane offsets inside one layer of x and inside one 32-row weight tile are 32-bit byte offsets
  DAPQ_REQUIRE(s.total_tokens * s.x_stride_token * 2 < ((int64_t)1 << 32), DAPQ_ERR_UNSUPPORTED,
               "one layer of x (total_tokens * x_stride_token * 2 bytes) must be smaller than 4 GiB");
  DAPQ_REQUIRE(s.w_stride_row * 2 * 32 + (int64_t)s.hidden * 2 < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED,
               "w_stride_row is too large");
  return DAPQ_OK;
}

}  // namespace
}  // namespace dapq

using namespace dapq;

extern "C" DAPQ_API size_t dapq_pseudo_queries_workspace_bytes(const dapq_qproj* desc) {
  if (check_qproj(desc) != DAPQ_OK) return 0;
  return make_qproj_plan(*desc).workspace_bytes;
}

extern "C" DAPQ_API int dapq_pseudo_queries(const dapq_qproj* desc, const void* x, const int32_t* token_idx,
                                            const void* w_q, const int32_t* positions, double theta, int32_t pairing,
                                            void* q_out, void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_qproj(desc);
  if (rc != DAPQ_OK) return rc;
  const dapq_qproj& s = *desc;
  DAPQ_REQUIRE(x != nullptr && token_idx != nullptr && w_q != nullptr && q_out != nullptr, DAPQ_ERR_INVALID_ARG,
               "x, token_idx, w_q and q_out must not be NULL");
  DAPQ_REQUIRE(((uintptr_t)x | (uintptr_t)w_q | (uintptr_t)q_out) % 16 == 0, DAPQ_ERR_UNSUPPORTED,
               "x, w_q and q_out must be 16-byte aligned");
  if (positions != nullptr) {
    DAPQ_REQUIRE(s.head_dim % 2 == 0 && (pairing == 0 || pairing == 1) && theta > 0.0 && theta < INFINITY,
                 DAPQ_ERR_INVALID_ARG, "rotation needs an even head_dim, pairing 0 or 1 and a finite theta > 0");
  }
  const QprojPlan pl = make_qproj_plan(s);
  if (pl.workspace_bytes > 0) {
    DAPQ_REQUIRE(workspace != nullptr && workspace_bytes >= pl.workspace_bytes, DAPQ_ERR_WORKSPACE,
                 "workspace of %zu bytes needed (dapq_pseudo_queries_workspace_bytes), %zu given", pl.workspace_bytes,
                 workspace != nullptr ? workspace_bytes : (size_t)0);
    DAPQ_REQUIRE((uintptr_t)workspace % 16 == 0, DAPQ_ERR_UNSUPPORTED, "workspace must be 16-byte aligned");
  }
  if (s.rows == 0) return DAPQ_OK;

  QprojParams p;
  p.x = static_cast<const uint16_t*>(x);
  p.token_idx = token_idx;
  p.w = static_cast<const uint16_t*>(w_q);
  p.q = static_cast<uint16_t*>(q_out);
  p.x_stride_layer = s.x_stride_layer;
  p.x_stride_token = s.x_stride_token;
  p.w_stride_layer = s.w_stride_layer;
  p.w_stride_row = s.w_stride_row;
  p.q_stride_layer = s.q_stride_layer;
  p.q_stride_head = s.q_stride_head;
  p.q_stride_row = s.q_stride_row;
  p.total_tokens = s.total_tokens;
  p.n_layers = s.n_layers;
  p.rows = s.rows;
  p.hidden = s.hidden;
  p.n_features = s.n_q_heads * s.head_dim;
  p.head_dim = s.head_dim;
  p.tiles_f = pl.tiles_f;
  p.sweeps = pl.sweeps;
  p.k_splits = pl.k_splits;
  p.kb_per_split = pl.kb_per_split;
  p.partial = pl.k_splits > 1 ? static_cast<float*>(workspace) : nullptr;
  DAPQ_REQUIRE((int64_t)p.tiles_f * p.sweeps * p.k_splits * s.n_layers < ((int64_t)1 << 31), DAPQ_ERR_UNSUPPORTED,
               "too many tiles");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (pl.ft == 4 && pl.mb == 2) launch_qproj<4, 2>(p, st);
  else if (pl.ft == 4) launch_qproj<4, 1>(p, st);
  else if (pl.mb == 2) launch_qproj<2, 2>(p, st);
  else launch_qproj<2, 1>(p, st);
  DAPQ_HIP_LAUNCH_CHECK("qproj_wave_kernel");
  if (pl.k_splits > 1) {
    const int64_t work = (int64_t)s.n_layers * s.rows * (p.n_features / 4);
    hipLaunchKernelGGL(qproj_reduce_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st, p,
                       pl.sweeps * 32 * pl.mb, pl.tiles_f * 32 * pl.ft);
    DAPQ_HIP_LAUNCH_CHECK("qproj_reduce_kernel");
  }

  if (positions != nullptr) {
    // rotation in place, the same kernel dapq_rope_apply runs: one call if the layers nest as extra heads
    if (s.n_layers == 1 || s.q_stride_layer == (int64_t)s.n_q_heads * s.q_stride_head) {
      return dapq_rope_apply(q_out, q_out, positions, s.rows, s.n_layers * s.n_q_heads, s.head_dim, s.q_stride_row,
                             s.q_stride_head, theta, pairing, stream);
    }
    for (int l = 0; l < s.n_layers; ++l) {
      uint16_t* ql = p.q + (int64_t)l * s.q_stride_layer;
      const int rc2 = dapq_rope_apply(ql, ql, positions, s.rows, s.n_q_heads, s.head_dim, s.q_stride_row, s.q_stride_head,
                                      theta, pairing, stream);
      if (rc2 != DAPQ_OK) return rc2;
    }
  }
  return DAPQ_OK;
}
