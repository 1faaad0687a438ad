// ctc_draft_topk: LM head over vocabulary + blank, log-softmax and per-slot top-k in one pass over W.
//
// The head weights are read exactly once.  A workgroup owns 128 consecutive vocabulary rows; it
// leaves, per column (= draft slot of some sequence), the running max, the sum of exponentials and
// its k best (logit, id) pairs.  A second, tiny kernel merges the partials of all workgroups into
// lse / topk_id / topk_logp.  (Merging inside the first kernel behind an atomic ticket needs a
// device-scope release fence in every workgroup; on this GPU that is an L2 write-back per workgroup
// and costs far more than the launch of a second kernel.)
//
// Three producers of the 128 x columns logit block exist:
//   * lmhead_bf16_mfma_kernel  - bf16 operands, v_mfma_f32_16x16x32_bf16, HBM-streaming design: a wavefront
//                                streams 16 rows, the hidden states of all columns sit in LDS (up to 11
//                                columns at D = 4096)
//   * lmhead_bf16_tile_kernel  - bf16, more columns than that: the 128 x 64 tile loop of gemm_tile.h, both
//                                operands stepping through LDS
//   * lmhead_generic_kernel    - any dtype/shape within the limits, plain fp32 FMA
// All hand the block over in LDS to the same epilogue.
#include <mutex>
#include <type_traits>
#include <utility>

#include <hip/hip_ext.h>

#include "gemm_tile.h"
#include "topk_merge.h"

namespace ctcspec {

constexpr int kZStride = kRowsPerBlock + 4;  // floats per column in the LDS logit block
// bytes per staged W row: 256 bf16 + pad.  The LDS serves a 16-byte access 16 lanes at a time - lanes l .. l+7 with
// l+16 .. l+23 - so a fragment read (lane = row c, chunk g) is conflict-free when rows c .. c+7 at chunks g and g+1
// fall on 16 different groups of 4 banks: pitch = 32 mod 64 bytes (with 16 bytes of pad the conflict counter read
// 8200 cycles per workgroup)
constexpr int kWRowStride = 512 + 32;
constexpr int kWStageBytes = 16 * kWRowStride;  // per wave
constexpr int kMfmaWaves = 8;

struct LmHeadParams {
  const void* hidden;
  const void* w;
  const float* bias;
  int BT, D, Vp1, k;
  int KC;        // mfma kernel: hidden elements per column held in LDS (= D)
  int hs_bytes;  // mfma kernel: bytes of the LDS hidden-state region
  unsigned int hs_magic;  // mfma kernel: ceil(2^32 / (KC / 8)), for index / (KC / 8) by multiplication
  int n_blocks;
  const void* zeros;  // tile kernel: 256 bytes of zeros
  float* pmax;              // [kMaxCols][pstride]
  float* psum;              // [kMaxCols][pstride]
  unsigned long long* pkey; // [kMaxCols][kMaxTopk][pstride]
  int pstride;              // workgroups the partial arrays have room for
  int32_t* topk_id;
  float* topk_logp;
  float* lse;
  float* logits_out;
};

// Epilogue shared by both producers.  zbuf holds the block's logits column-major:
// zbuf[col * kZStride + r] = z of row (blockIdx.x*128 + r), -inf for rows >= Vp1.
// Whole wavefronts must call this (the reductions use every lane).
__device__ void lmhead_block_epilogue(const LmHeadParams& p, const float* zbuf) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  const int row_base = blockIdx.x * kRowsPerBlock;
  const int k = p.k;

  if (p.logits_out) {
    for (int idx = tid; idx < p.BT * kRowsPerBlock; idx += blockDim.x) {
      int m = idx / kRowsPerBlock, r = idx % kRowsPerBlock;
      if (row_base + r < p.Vp1) p.logits_out[(size_t)m * p.Vp1 + row_base + r] = zbuf[m * kZStride + r];
    }
  }

  // per column: max, sum of exponentials, k best keys of this block's 128 rows
  for (int m = wave; m < p.BT; m += nwaves) {
    float z0 = zbuf[m * kZStride + lane];
    float z1 = zbuf[m * kZStride + lane + 64];
    int id0 = row_base + lane, id1 = row_base + lane + 64;
    float mx = wave_max_f32(fmaxf(z0, z1));
    float e = 0.f;
    if (mx > -INFINITY) e = __expf(z0 - mx) + __expf(z1 - mx);
    float s = wave_sum_f32(e);
    unsigned long long a = id0 < p.Vp1 ? rank_key(z0, (unsigned)id0) : 0ull;
    unsigned long long b = id1 < p.Vp1 ? rank_key(z1, (unsigned)id1) : 0ull;
    if (b > a) { unsigned long long t = a; a = b; b = t; }
    const size_t slot = (size_t)m * p.pstride + blockIdx.x;
    for (int r = 0; r < k; ++r) {
      unsigned long long best = wave_max_u64(a);
      if (lane == 0) p.pkey[((size_t)m * kMaxTopk + r) * p.pstride + blockIdx.x] = best;
      if (a == best) { a = b; b = 0ull; }
    }
    if (lane == 0) { p.pmax[slot] = mx; p.psum[slot] = s; }
  }
}

// The same epilogue for many columns: a lane per column instead of a wavefront per column.  Wavefront w scans
// rows 16w .. 16w+15 of every column (lane = column, the 16 logits in registers, the k best keys kept sorted in
// registers), leaves its (max, sum, keys) per column in LDS, and wavefront 0 merges the eight partials of each
// column.  About 16 + 8 short steps per lane against eight columns in turn per wavefront, each with k 64-bit
// wavefront reductions.  `part` is LDS behind zbuf: 8 x kMaxCols x (2 floats + KMAX keys).
template <int KMAX>
__device__ void lmhead_block_epilogue_wide(const LmHeadParams& p, const float* zbuf, unsigned char* part) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row_base = blockIdx.x * kRowsPerBlock;
  static_assert(kMaxCols <= 64 && kRowsPerBlock == 16 * kMfmaWaves, "a lane per column, sixteen rows per wavefront");
  if (p.logits_out) {
    for (int idx = tid; idx < p.BT * kRowsPerBlock; idx += blockDim.x) {
      int m = idx / kRowsPerBlock, r = idx % kRowsPerBlock;
      if (row_base + r < p.Vp1) p.logits_out[(size_t)m * p.Vp1 + row_base + r] = zbuf[m * kZStride + r];
    }
  }
  float* pm = (float*)part;                                        // [8][kMaxCols]
  float* ps = pm + kMfmaWaves * kMaxCols;                          // [8][kMaxCols]
  unsigned long long* pk = (unsigned long long*)(ps + kMfmaWaves * kMaxCols);  // [8][kMaxCols][KMAX]
  const int m = lane;
  if (m < p.BT) {
    f32x4 z[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) z[q] = *(const f32x4*)(zbuf + m * kZStride + 16 * wave + 4 * q);
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < 4; ++q) mx = fmaxf(mx, fmaxf(fmaxf(z[q][0], z[q][1]), fmaxf(z[q][2], z[q][3])));
    float e = 0.f;
    KeyList<KMAX> list;
    list.clear();
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int id = row_base + 16 * wave + 4 * q + i;
        if (mx > -INFINITY) e += __expf(z[q][i] - mx);
        list.insert(id < p.Vp1 ? rank_key(z[q][i], (unsigned)id) : 0ull);
      }
    pm[wave * kMaxCols + m] = mx;
    ps[wave * kMaxCols + m] = e;
#pragma unroll
    for (int r = 0; r < KMAX; ++r) pk[(wave * kMaxCols + m) * KMAX + r] = list.v[r];
  }
  __syncthreads();
  if (wave == 0 && m < p.BT) {
    float m_run = -INFINITY, s_run = 0.f;
    KeyList<KMAX> list;
    list.clear();
#pragma unroll
    for (int w = 0; w < kMfmaWaves; ++w) {
      const float wm = pm[w * kMaxCols + m], wsum = ps[w * kMaxCols + m];
      if (wm > -INFINITY) {
        const float mn = fmaxf(m_run, wm);
        s_run = s_run * __expf(m_run - mn) + wsum * __expf(wm - mn);
        m_run = mn;
      }
#pragma unroll
      for (int r = 0; r < KMAX; ++r) list.insert(pk[(w * kMaxCols + m) * KMAX + r]);
    }
    const size_t slot = (size_t)m * p.pstride + blockIdx.x;
    p.pmax[slot] = m_run;
    p.psum[slot] = s_run;
    for (int r = 0; r < p.k; ++r)
      p.pkey[((size_t)m * kMaxTopk + r) * p.pstride + blockIdx.x] = r < KMAX ? list.v[r] : 0ull;
  }
}

// Merge of the per-workgroup partials: one wavefront per column (the merge itself: topk_merge.h).
template <int KMAX>
__global__ __launch_bounds__(64) void lmhead_merge_kernel(LmHeadParams p) {
  const int lane = threadIdx.x, k = p.k;
  const int col[1] = {(int)blockIdx.x};
  float lse[1];
  unsigned long long best[1][KMAX];
  merge_topk_columns<KMAX, 1>(p.pmax, p.psum, p.pkey, p.pstride, p.n_blocks, k, col, lse, best);
  if (lane == 0 && p.lse) p.lse[col[0]] = lse[0];
  if (lane < k) {
    unsigned long long key = 0ull;
#pragma unroll
    for (int r = 0; r < KMAX; ++r) key = lane == r ? best[0][r] : key;
    p.topk_id[col[0] * k + lane] = (int32_t)rank_key_index(key);
    p.topk_logp[col[0] * k + lane] = rank_key_value(key) - lse[0];
  }
}

// ---- generic producer ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void lmhead_generic_kernel(LmHeadParams p) {
  __shared__ float zbuf[kMaxCols * kZStride];
  const int tid = threadIdx.x;
  const int row_base = blockIdx.x * kRowsPerBlock;
  const T* hidden = (const T*)p.hidden;
  const T* w = (const T*)p.w;
  for (int idx = tid; idx < p.BT * kRowsPerBlock; idx += 256) {
    int m = idx / kRowsPerBlock, r = idx % kRowsPerBlock;
    int row = row_base + r;
    float z = -INFINITY;
    if (row < p.Vp1) {
      const T* hp = hidden + (size_t)m * p.D;
      const T* wp = w + (size_t)row * p.D;
      float acc = 0.f;
      for (int d = 0; d < p.D; ++d) acc = fmaf(load_as_float(hp + d), load_as_float(wp + d), acc);
      z = acc + (p.bias ? p.bias[row] : 0.f);
    }
    zbuf[m * kZStride + r] = z;
  }
  __syncthreads();
  lmhead_block_epilogue(p, zbuf);
}

// ---- bf16 MFMA streaming producer -----------------------------------------------------------------
// 8 waves; wave w owns the 16 rows [block*128 + 16w, +16) over the whole hidden dimension.
// Per step of 256 hidden elements a wave issues 8 coalesced 16-byte loads (each instruction covers
// two rows x 512 contiguous bytes), parks them in its private LDS strip and reads them back in the
// MFMA A-operand layout (lane = row, 8 consecutive k).  Loads run STAGES-1 steps ahead in registers.
// The hidden states (the B operand) sit in LDS for the whole workgroup.
//
// Every global load of the streaming path is issued unconditionally and in a fixed number per step
// (rows past the vocabulary re-read its last row, the tail of the k loop is peeled instead of
// guarded): the waits can then name the exact number of younger loads that may stay in flight, and
// the prefetch pipeline never drains.  A load under a condition makes every later wait a full drain.
template <int NT, int STAGES>
__global__ __launch_bounds__(64 * kMfmaWaves) void lmhead_bf16_mfma_kernel(LmHeadParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15, g = lane >> 4;
  // a load instruction covers two rows x 512 bytes; within a row the lanes take the 16-byte chunks in an order
  // that lets the 16 lanes the LDS serves together (l .. l+7, l+16 .. l+23) write 256 consecutive bytes
  const int lrow = lane >> 5, lch = (lane & 7) | ((lane & 16) >> 1) | ((lane & 8) << 1);
  unsigned char* hs = smem;
  const int HSS = p.KC * 2 + 32;
  unsigned char* wst = smem + p.hs_bytes + wave * kWStageBytes;
  const int row0 = blockIdx.x * kRowsPerBlock + wave * 16;

  const unsigned char* wp[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int row = row0 + 2 * j + lrow;
    row = row < p.Vp1 ? row : p.Vp1 - 1;  // the ragged last tile re-reads the last valid row
    wp[j] = (const unsigned char*)p.w + (size_t)row * p.D * 2 + lch * 16;
  }
  int bcol[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int col = nt * 16 + c;
    bcol[nt] = (col < p.BT ? col : p.BT - 1) * HSS + g * 16;
  }

  f32x4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int total_steps = p.D / 256;  // the host guarantees KC == D: the hidden states of all columns are in LDS

  // Hidden-state staging: every thread carries kHsPieces 16-byte pieces through registers (pieces past the
  // end repeat the last piece and are not written to LDS); they are requested before the first W loads.
  constexpr int kHsPieces = 12;
  const int per_row = p.KC / 8;  // 16-byte pieces per column
  const int hs_total = p.BT * per_row;
  u32x4 hreg[kHsPieces];
  int hs_dst[kHsPieces];  // LDS offset of piece u, -1: none
  size_t hs_src[kHsPieces];
#pragma unroll
  for (int u = 0; u < kHsPieces; ++u) {
    const int idx = tid + u * 64 * kMfmaWaves;
    const int cl = idx < hs_total ? idx : hs_total - 1;
    const int m = (int)__umulhi((unsigned)cl, p.hs_magic);  // cl / per_row
    const int q = cl - m * per_row;
    hs_dst[u] = idx < hs_total ? m * HSS + q * 16 : -1;
    hs_src[u] = (size_t)m * p.D * 2 + q * 16;
  }
  auto hs_request = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kHsPieces; ++u) hreg[u] = *(const u32x4*)((const unsigned char*)p.hidden + hs_src[u]);
  };
  auto hs_commit = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kHsPieces; ++u)
      if (hs_dst[u] >= 0) *(u32x4*)(hs + hs_dst[u]) = hreg[u];
  };

  u32x4 v[STAGES][8];
  auto w_request = [&](int step, auto stage_tag) __attribute__((always_inline)) {
    constexpr int ST = decltype(stage_tag)::value;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[ST][j] = __builtin_nontemporal_load((const u32x4*)(wp[j] + (size_t)step * 512));
    // keep the scheduler from mixing these loads with those of another step: the waits count loads in
    // issue order, and a stage whose loads are spread among younger ones can only be waited for late
    __builtin_amdgcn_sched_barrier(0);
  };
  // one step: W registers of stage ST -> LDS strip -> A fragments; i = step
  auto consume = [&](int i, auto stage_tag) __attribute__((always_inline)) {
    constexpr int ST = decltype(stage_tag)::value;
#pragma unroll
    for (int j = 0; j < 8; ++j) *(u32x4*)(wst + (2 * j + lrow) * kWRowStride + lch * 16) = v[ST][j];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)(wst + c * kWRowStride + kk * 64 + g * 16));
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        bf16x8 b = __builtin_bit_cast(bf16x8, *(const u32x4*)(hs + bcol[nt] + (i * 256 + kk * 32) * 2));
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[nt], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto for_each_stage = [&](auto&& fn) __attribute__((always_inline)) {
    [&]<int... I>(std::integer_sequence<int, I...>) { (fn(std::integral_constant<int, I>{}), ...); }
    (std::make_integer_sequence<int, STAGES>{});
  };

  hs_request();
  for_each_stage([&](auto st) __attribute__((always_inline)) {
    if constexpr (decltype(st)::value < STAGES - 1) w_request(decltype(st)::value, st);
  });

  {
    hs_commit();
    __syncthreads();
    // blocks of STAGES steps; step i refills, with step i + STAGES - 1, the stage that step i - 1 freed
    const int nblk = total_steps / STAGES;  // the host guarantees total_steps % STAGES == 0
    for (int blk = 0; blk + 1 < nblk; ++blk) {
      for_each_stage([&](auto st) __attribute__((always_inline)) {
        constexpr int SS = decltype(st)::value;
        const int i = blk * STAGES + SS;
        w_request(i + STAGES - 1, std::integral_constant<int, (SS + STAGES - 1) % STAGES>{});
        consume(i, st);
      });
    }
    // last block: only its first step still has something to prefetch
    for_each_stage([&](auto st) __attribute__((always_inline)) {
      constexpr int SS = decltype(st)::value;
      const int i = (nblk - 1) * STAGES + SS;
      if constexpr (SS == 0) w_request(i + STAGES - 1, std::integral_constant<int, STAGES - 1>{});
      consume(i, st);
    });
  }

  // hand the 128 x BT logit block to the epilogue (the W strips are no longer needed)
  __syncthreads();
  float* zbuf = (float*)(smem + p.hs_bytes);
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int col = nt * 16 + c;
    if (col < p.BT) {
      f32x4 z;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int row = row0 + g * 4 + i;
        z[i] = row < p.Vp1 ? acc[nt][i] + (p.bias ? p.bias[row] : 0.f) : -INFINITY;
      }
      *(f32x4*)(zbuf + col * kZStride + wave * 16 + g * 4) = z;
    }
  }
  __syncthreads();
  lmhead_block_epilogue(p, zbuf);
}

// ---- bf16 MFMA producer for many columns (more than fit in LDS over the whole hidden dimension) -----------------
// The 128 x 64 tile loop shared with the base-model head: both operands staged through LDS step by step, the
// weights still read exactly once.  Then the same block epilogue as the other producers.
constexpr int kLmTileDist = 4;
template <int CT>
__global__ __launch_bounds__(64 * kTileWaves) void lmhead_bf16_tile_kernel(LmHeadParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wr = wave >> 2, wc = wave & 3;
  const int c = lane & 15, g = lane >> 4;
  const int row_base = blockIdx.x * kRowsPerBlock;
  GemmTileArgs t;
  t.w = p.w; t.hidden = p.hidden; t.zeros = p.zeros; t.D = p.D; t.V = p.Vp1; t.cols = p.BT; t.row_base = row_base;
  f32x4 acc[4][CT];
  static_assert(CT == 1, "the 128 x 64 tile");
  gemm_tile<kLmTileDist, Tile128x64>(t, smem, acc);
  // (the loop's last barrier has every wavefront done with the LDS tiles)
  float* zbuf = (float*)smem;
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const int col = wc * 16 * CT + ct * 16 + c;
      if (col < p.BT) {
        f32x4 z;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = row_base + wr * 64 + rt * 16 + g * 4 + i;
          z[i] = row < p.Vp1 ? acc[rt][ct][i] + (p.bias ? p.bias[row] : 0.f) : -INFINITY;
        }
        *(f32x4*)(zbuf + col * kZStride + wr * 64 + rt * 16 + g * 4) = z;
      }
    }
  __syncthreads();
  unsigned char* part = smem + kMaxCols * kZStride * 4;
  if (p.BT <= 16) lmhead_block_epilogue(p, zbuf);  // a wavefront per column, at most two in turn
  else if (p.k <= 1) lmhead_block_epilogue_wide<1>(p, zbuf, part);
  else if (p.k <= 2) lmhead_block_epilogue_wide<2>(p, zbuf, part);
  else if (p.k <= 4) lmhead_block_epilogue_wide<4>(p, zbuf, part);
  else lmhead_block_epilogue_wide<8>(p, zbuf, part);
}
static_assert(kMaxCols <= 64 && kMaxCols * kZStride * 4 + kMfmaWaves * kMaxCols * (8 + 8 * kMaxTopk) <= Tile128x64::LDS_BYTES,
              "one 64-column tile holds every column and the epilogue's partials");

static void launch_merge(const LmHeadParams& p, hipStream_t stream) {
  if (p.k <= 1) hipLaunchKernelGGL(lmhead_merge_kernel<1>, dim3(p.BT), dim3(64), 0, stream, p);
  else if (p.k <= 2) hipLaunchKernelGGL(lmhead_merge_kernel<2>, dim3(p.BT), dim3(64), 0, stream, p);
  else if (p.k <= 4) hipLaunchKernelGGL(lmhead_merge_kernel<4>, dim3(p.BT), dim3(64), 0, stream, p);
  else hipLaunchKernelGGL(lmhead_merge_kernel<8>, dim3(p.BT), dim3(64), 0, stream, p);
}

int flush_deferred(ctcspec_ctx* ctx) {
  if (!ctx->lm_pending) return CTCSPEC_OK;
  ctx->lm_pending = 0;
  LmHeadParams p = {};
  p.BT = ctx->lm_owed.BT; p.k = ctx->lm_owed.k; p.n_blocks = ctx->lm_owed.n_blocks;
  p.pmax = ctx->lm_pmax; p.psum = ctx->lm_psum; p.pkey = ctx->lm_pkey; p.pstride = ctx->lm_max_blocks;
  p.topk_id = ctx->lm_owed.topk_id; p.topk_logp = ctx->lm_owed.topk_logp; p.lse = ctx->lm_owed.lse;
  launch_merge(p, ctx->stream);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}

static int pick_kc(int BT, int D, int stages, int budget) {
  const int unit = 256 * stages;
  if (D % unit != 0) return 0;
  for (int kc = D; kc >= unit; kc -= unit) {
    if (D % kc != 0) continue;
    if ((long long)BT * (2 * kc + 32) <= budget) return kc;
  }
  return 0;
}

// ev0/ev1, when given, are attached to the launch itself: they take the kernel's own begin and end timestamps (what a
// kernel trace reports), without the dispatch work that a pair of events recorded around the launch also spans.
template <int NT, int STAGES>
static hipError_t launch_mfma(const LmHeadParams& p, int lds_bytes, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1) {
  auto kern = lmhead_bf16_mfma_kernel<NT, STAGES>;
  if (ev0 && ev1)
    hipExtLaunchKernelGGL(kern, dim3(p.n_blocks), dim3(64 * kMfmaWaves), lds_bytes, stream, ev0, ev1, 0, p);
  else
    hipLaunchKernelGGL(kern, dim3(p.n_blocks), dim3(64 * kMfmaWaves), lds_bytes, stream, p);
  return hipGetLastError();
}

// the streaming kernel's LDS need depends on the call's shape; its budget (see ctc_draft_topk) is the limit set here
constexpr int kMfmaLdsLimit = 160 * 1024 - 64;

template <int NT, int STAGES>
static hipError_t allow_mfma_lds() {
  return hipFuncSetAttribute((const void*)lmhead_bf16_mfma_kernel<NT, STAGES>,
                             hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLdsLimit);
}

// dynamic LDS limits of this file's kernels, on the current device
static hipError_t allow_large_lds() {
  hipError_t e = allow_mfma_lds<1, 4>();
  if (e == hipSuccess) e = allow_mfma_lds<2, 4>();
  if (e == hipSuccess) e = allow_mfma_lds<3, 4>();
  if (e == hipSuccess) e = allow_mfma_lds<4, 4>();
  if (e == hipSuccess) e = allow_mfma_lds<1, 2>();
  if (e == hipSuccess) e = allow_mfma_lds<2, 2>();
  if (e == hipSuccess) e = allow_mfma_lds<3, 2>();
  if (e == hipSuccess) e = allow_mfma_lds<4, 2>();
  if (e == hipSuccess)
    e = hipFuncSetAttribute((const void*)lmhead_bf16_tile_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            Tile128x64::LDS_BYTES);
  return e;
}

// ---- scratch of the entry point that allocates nothing ------------------------------------------------------------
// The same partial results that ctc_draft_topk keeps in its context's workspace, in a device array of the library
// itself: [256 bytes of zeros][pmax][psum][pkey], the three laid out as in the context for kStaticMaxBlocks row blocks.  Every GPU the library
// runs on holds its own copy (2.4 MB) at its own address until the process ends.
constexpr int kStaticMaxBlocks = CTCSPEC_NOALLOC_MAX_VOCAB_ROWS / kRowsPerBlock;
constexpr size_t kScratchZeros = 0;
constexpr size_t kScratchPmax = 256;
constexpr size_t kScratchPsum = kScratchPmax + (size_t)kStaticMaxBlocks * kMaxCols * sizeof(float);
constexpr size_t kScratchPkey = kScratchPsum + (size_t)kStaticMaxBlocks * kMaxCols * sizeof(float);
constexpr size_t kScratchBytes = kScratchPkey + (size_t)kStaticMaxBlocks * kMaxCols * kMaxTopk * sizeof(unsigned long long);
static_assert(CTCSPEC_NOALLOC_MAX_VOCAB_ROWS % kRowsPerBlock == 0 && kScratchPkey % 256 == 0, "scratch layout");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle for the runtime, not a device address: the address on each device comes
// from hipGetSymbolAddress, once per device, and host code uses that pointer everywhere.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[kMaxDevices];

static hipError_t scratch_of_current_device(unsigned char** out, bool* first_use) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (first_use) *first_use = false;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = (unsigned char*)ptr;
    if (first_use) *first_use = true;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

hipError_t prepare_draft_topk() {
  // set-up of the allocation-free entry point on this device: address of its scratch, zeros block cleared (the
  // array starts out zeroed and no kernel writes that block; clearing it here costs nothing)
  unsigned char* sp = nullptr;
  hipError_t e = scratch_of_current_device(&sp, nullptr);
  if (e == hipSuccess) e = hipMemset(sp + kScratchZeros, 0, 256);
  if (e != hipSuccess) return e;
  return allow_large_lds();
}

}  // namespace ctcspec

using namespace ctcspec;

// Everything ctc_draft_topk does after its argument checks: producer kernel, then the merge kernel.  `err` receives
// error texts (NULL: the thread's context-less error slot); ev0/ev1 non-null: time the producer kernel; *timed is
// set when they were used.
struct LmScratch {
  float* pmax;
  float* psum;
  unsigned long long* pkey;
  int pstride;
  const void* zeros;
};

static int draft_topk_launch(ctcspec_ctx* err, hipStream_t stream, const LmScratch& sc, hipEvent_t ev0, hipEvent_t ev1,
                             int* timed, bool defer, ctcspec_dtype dt, const void* hidden, const void* w, const float* bias, int B,
                             int T, int D, int Vp1, int k, int32_t* topk_id, float* topk_logp, float* lse,
                             float* logits_out) {
  LmHeadParams p;
  p.hidden = hidden; p.w = w; p.bias = bias;
  p.BT = B * T; p.D = D; p.Vp1 = Vp1; p.k = k;
  p.KC = 0; p.hs_bytes = 0; p.hs_magic = 0; p.zeros = sc.zeros;
  p.n_blocks = (Vp1 + kRowsPerBlock - 1) / kRowsPerBlock;
  p.pmax = sc.pmax; p.psum = sc.psum; p.pkey = sc.pkey; p.pstride = sc.pstride;
  p.topk_id = topk_id; p.topk_logp = topk_logp; p.lse = lse; p.logits_out = logits_out;
  const bool timing = ev0 && ev1;
  // defer: leave the partials and record what is owed (err is the context then); the collapse/tree kernel or
  // flush_deferred does the merge
  auto finish = [&]() -> int {
    if (defer) {
      err->lm_owed.BT = p.BT; err->lm_owed.k = p.k; err->lm_owed.n_blocks = p.n_blocks;
      err->lm_owed.topk_id = topk_id; err->lm_owed.topk_logp = topk_logp; err->lm_owed.lse = lse;
      err->lm_pending = 1;
      return CTCSPEC_OK;
    }
    launch_merge(p, stream);
    CTCSPEC_HIP(err, hipGetLastError());
    return CTCSPEC_OK;
  };

  if (dt == CTCSPEC_BF16) {
    const int budget = kMfmaLdsLimit - kMfmaWaves * kWStageBytes;
    // the streaming kernel needs the hidden states of all columns in LDS over the whole hidden dimension
    // (4 register stages of prefetch; 2 when D is a multiple of 512 but not of 1024)
    int stages = 4;
    int kc = pick_kc(p.BT, D, stages, budget);
    if (kc != D) {
      stages = 2;
      kc = pick_kc(p.BT, D, stages, budget);
    }
    if (kc == D) {
      p.KC = kc;
      p.hs_bytes = p.BT * (2 * kc + 32);
      p.hs_magic = (unsigned int)((0x100000000ull + (unsigned)(kc / 8) - 1) / (unsigned)(kc / 8));
      int lds = p.hs_bytes + kMfmaWaves * kWStageBytes;
      int nt = (p.BT + 15) / 16;
      hipError_t e;
      if (stages == 4) {
        switch (nt) {
          case 1: e = launch_mfma<1, 4>(p, lds, stream, ev0, ev1); break;
          case 2: e = launch_mfma<2, 4>(p, lds, stream, ev0, ev1); break;
          case 3: e = launch_mfma<3, 4>(p, lds, stream, ev0, ev1); break;
          default: e = launch_mfma<4, 4>(p, lds, stream, ev0, ev1); break;
        }
      } else {
        switch (nt) {
          case 1: e = launch_mfma<1, 2>(p, lds, stream, ev0, ev1); break;
          case 2: e = launch_mfma<2, 2>(p, lds, stream, ev0, ev1); break;
          case 3: e = launch_mfma<3, 2>(p, lds, stream, ev0, ev1); break;
          default: e = launch_mfma<4, 2>(p, lds, stream, ev0, ev1); break;
        }
      }
      CTCSPEC_HIP(err, e);
      if (timing && timed) *timed = 1;
      return finish();
    }
    if (D % kTileStepK == 0 && p.BT <= 64 && (long long)Vp1 * D * 2 < (1LL << 32)) {
      // more columns than that: both operands step through LDS
      if (timing) CTCSPEC_HIP(err, hipEventRecord(ev0, stream));
      hipLaunchKernelGGL(lmhead_bf16_tile_kernel<1>, dim3(p.n_blocks), dim3(64 * kTileWaves), Tile128x64::LDS_BYTES,
                         stream, p);
      CTCSPEC_HIP(err, hipGetLastError());
      if (timing) {
        CTCSPEC_HIP(err, hipEventRecord(ev1, stream));
        if (timed) *timed = 1;
      }
      return finish();
    }
    hipLaunchKernelGGL(lmhead_generic_kernel<unsigned short>, dim3(p.n_blocks), dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(lmhead_generic_kernel<float>, dim3(p.n_blocks), dim3(256), 0, stream, p);
  }
  CTCSPEC_HIP(err, hipGetLastError());
  return finish();
}

// argument checks shared by the two entry points (`name` prefixes the messages)
static int draft_topk_check(ctcspec_ctx* err, const char* name, ctcspec_dtype dt, const void* hidden, const void* w,
                            int B, int T, int D, int Vp1, int k, const int32_t* topk_id, const float* topk_logp) {
  CTCSPEC_REQUIRE(err, hidden && w && topk_id && topk_logp, CTCSPEC_EINVAL, "%s: null pointer", name);
  CTCSPEC_REQUIRE(err, dt == CTCSPEC_F32 || dt == CTCSPEC_BF16, CTCSPEC_EINVAL, "%s: bad dtype", name);
  CTCSPEC_REQUIRE(err, B > 0 && T > 0 && D > 0 && Vp1 > 0 && k > 0, CTCSPEC_EINVAL, "%s: sizes must be positive", name);
  CTCSPEC_REQUIRE(err, aligned16(hidden) && aligned16(w), CTCSPEC_EINVAL, "%s: hidden and w must be 16-byte aligned",
                  name);
  CTCSPEC_REQUIRE(err, (long long)B * T <= kMaxCols, CTCSPEC_EUNSUPPORTED, "%s: B*T=%lld > %d", name, (long long)B * T,
                  kMaxCols);
  CTCSPEC_REQUIRE(err, k <= Vp1, CTCSPEC_EINVAL, "%s: k=%d > vocabulary rows %d", name, k, Vp1);
  return CTCSPEC_OK;
}

extern "C" int ctc_draft_topk(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* hidden, const void* w,
                              const float* bias, int B, int T, int D, int Vp1, int k, int32_t* topk_id,
                              float* topk_logp, float* lse, float* logits_out) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;  // the partials are about to be overwritten
  const int rc = draft_topk_check(ctx, "ctc_draft_topk", dt, hidden, w, B, T, D, Vp1, k, topk_id, topk_logp);
  if (rc != CTCSPEC_OK) return rc;
  CTCSPEC_REQUIRE(ctx, B <= ctx->lim.max_batch && T <= ctx->lim.max_slots && k <= ctx->lim.max_topk &&
                           Vp1 <= ctx->lim.max_vocab_rows,
                  CTCSPEC_EUNSUPPORTED, "ctc_draft_topk: shape exceeds the context's limits");
  const LmScratch sc = {ctx->lm_pmax, ctx->lm_psum, ctx->lm_pkey, ctx->lm_max_blocks, ctx->zeros};
  return draft_topk_launch(ctx, ctx->stream, sc, ctx->lm_profile ? ctx->lm_ev0 : nullptr,
                           ctx->lm_profile ? ctx->lm_ev1 : nullptr, &ctx->lm_profile_valid, ctx->lm_defer != 0, dt, hidden, w,
                           bias, B, T, D, Vp1, k, topk_id, topk_logp, lse, logits_out);
}

extern "C" int ctc_draft_topk_noalloc(void* hip_stream, ctcspec_dtype dt, const void* hidden, const void* w,
                                      const float* bias, int B, int T, int D, int Vp1, int k, int32_t* topk_id,
                                      float* topk_logp, float* lse, float* logits_out) {
  const char* name = "ctc_draft_topk_noalloc";
  const int rc = draft_topk_check(nullptr, name, dt, hidden, w, B, T, D, Vp1, k, topk_id, topk_logp);
  if (rc != CTCSPEC_OK) return rc;
  CTCSPEC_REQUIRE(nullptr, Vp1 <= CTCSPEC_NOALLOC_MAX_VOCAB_ROWS, CTCSPEC_EUNSUPPORTED,
                  "%s: %d vocabulary rows exceed the %d that the library's static scratch holds partial results for "
                  "(use ctc_draft_topk with a context)",
                  name, Vp1, CTCSPEC_NOALLOC_MAX_VOCAB_ROWS);
  CTCSPEC_REQUIRE(nullptr, k <= CTCSPEC_MAX_TOPK && T <= CTCSPEC_MAX_SLOTS, CTCSPEC_EUNSUPPORTED,
                  "%s: k <= %d and T <= %d required", name, CTCSPEC_MAX_TOPK, CTCSPEC_MAX_SLOTS);
  hipStream_t stream = (hipStream_t)hip_stream;
  unsigned char* sp = nullptr;
  bool first_use = false;
  CTCSPEC_HIP(nullptr, scratch_of_current_device(&sp, &first_use));
  if (first_use) {
    // No context was ever created on this device, so the dynamic LDS limits were never raised: do it now (host-side
    // attribute calls, no allocation).  The zeros block needs nothing: the array starts out zeroed and no kernel
    // writes that block.
    CTCSPEC_HIP(nullptr, allow_large_lds());
  }
  const LmScratch sc = {(float*)(sp + kScratchPmax), (float*)(sp + kScratchPsum),
                        (unsigned long long*)(sp + kScratchPkey), kStaticMaxBlocks, sp + kScratchZeros};
  return draft_topk_launch(nullptr, stream, sc, nullptr, nullptr, nullptr, false, dt, hidden, w, bias, B, T, D, Vp1, k, topk_id,
                           topk_logp, lse, logits_out);
}
