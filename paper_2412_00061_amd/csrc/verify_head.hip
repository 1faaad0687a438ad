// verify_head_argmax: the base model's LM head over the hidden states of the tree nodes, reduced to the
// greedy token per node.  kv_commit: append the accepted path's keys and values to the cached context.
//
// The head is the same stream over a [V, D] weight matrix as the draft head, but with up to 128 columns
// (one per tree node) instead of 8, and all that is kept of a column is its best (logit, id) key:
//   * verify_head_bf16_kernel    - bf16, D a multiple of 128: MFMA, 128 vocabulary rows x 128 columns
//                                  per workgroup, weights read once per block of 128 columns
//   * verify_head_generic_kernel - any dtype/shape: plain fp32 FMA, one atomic max per (row block, column)
//   * verify_head_merge_kernel   - best key over the row blocks -> token id, -1 for rows without a node
#include <type_traits>
#include <utility>

#include "common.h"

namespace ctcspec {

constexpr int kVhCols = kVerifyCols;            // columns (tree nodes) per pass over the weights
constexpr int kVhWaves = 8;
constexpr int kVhDist = 4;                      // prefetch distance in steps = register stages per operand
constexpr int kVhStepK = 128;                   // hidden elements per step
constexpr int kVhRowPitch = 2 * kVhStepK + 32;  // bytes per staged row: 128 bf16 + pad; fragment reads (16 rows x 4
                                                // chunks per instruction) measure conflict-free at this pitch
constexpr int kVhTileBytes = 128 * kVhRowPitch; // one operand of one step: 128 rows (or columns) x 128 k
constexpr int kVhLdsBytes = 4 * kVhTileBytes;   // W and hidden-state tile, double-buffered
constexpr int kVhZStride = kRowsPerBlock + 4;   // floats per column of the logit block
static_assert(kVhCols == 128 && kRowsPerBlock == 128, "tile shape");
static_assert(kVhCols * kVhZStride * 4 <= kVhLdsBytes, "logit block fits the staging area");

struct VerifyHeadParams {
  const void* hidden;   // [cols_total][D], this pass starts at column col0
  const void* w;        // [V][D]
  int col0, cols;       // columns of this pass (cols <= kVhCols)
  int D, V;
  int n_blocks;         // row blocks of 128
  unsigned long long* pkey;  // [n_blocks][kVhCols] best key per (row block, column of the pass)
  float* logits_out;    // [cols_total][V] or null
  const void* zeros;    // 256 bytes of zeros
  const int32_t* n_nodes;  // [B]
  int max_nodes;
  int32_t* target;      // [cols_total]
};

// ---- bf16 MFMA kernel -----------------------------------------------------------------------------------
// 128 vocabulary rows x 128 columns per workgroup, 8 wavefronts in a 2 x 4 grid: wavefront (wr, wc) owns
// rows [64 wr, +64) x columns [32 wc, +32) - 4 x 2 MFMA tiles.  Per step of 128 hidden elements both
// operands go through LDS: the W tile (128 rows x 256 B, nontemporal, the A operand) and the hidden states
// of the step (128 columns x 256 B, the B operand) are fetched by all threads together with coalesced
// 16-byte loads, DIST steps ahead, into rotating register stages, and written to one of two LDS buffers
// while the other one is computed from: one barrier per step.  A wavefront reads 4 A and 2 B fragments per
// 32 k for 8 MFMAs; the fragments of the next 32 k are read, and the tiles of the next step are written,
// between the MFMAs of the current 32 k (the instruction order is pinned with scheduling groups).
// What bounds it (measured, one CU): b128 fragment reads at 128 B per clock, b128 writes at 79 B per clock -
// per step 192 KB read + 64 KB written = 2300 clocks against 1024 clocks of MFMA and 1.35 us (3200 clocks)
// for the 32 KB of W at the HBM rate, so the LDS work fits under the stream only if nothing serialises.
// All loads are unconditional and counted (indices clamped), so the waits name the loads that stay in flight.
typedef __attribute__((address_space(1))) u32x4 GlobalU32x4;  // a pointer made from an integer is generic otherwise
template <int DIST>
__global__ __launch_bounds__(64 * kVhWaves) void verify_head_bf16_kernel(VerifyHeadParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NTHREADS = 64 * kVhWaves;
  constexpr int PIECES = 128 * (2 * kVhStepK / 16) / NTHREADS;  // 16-byte pieces per thread and tile: 4
  constexpr int ROWS_PER_PIECE = NTHREADS / 16;                 // 32
  constexpr int KK = kVhStepK / 32;                             // MFMA k-blocks per step
  constexpr int TRIP = DIST % 2 == 0 ? DIST : 2 * DIST;         // steps per loop trip: stage and buffer static
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 2, wc = wave & 3;
  const int c = lane & 15, g = lane >> 4;
  const int row_base = blockIdx.x * kRowsPerBlock;
  const int total_steps = p.D / kVhStepK;
  // LDS: buffer b holds the hidden-state tile at 2 b and the W tile at 2 b + 1 (in tiles)

  // piece u of a thread: tile row (tid >> 4) + 32 u, 16-byte chunk tid & 15; byte offsets in 32 bits (the host
  // checks that the matrices are smaller than 4 GB)
  const unsigned int lane_off = (tid & 15) * 16;
  const uintptr_t w_addr = (uintptr_t)p.w, h_addr = (uintptr_t)p.hidden + (size_t)p.col0 * p.D * 2;
  const uintptr_t z_addr = (uintptr_t)p.zeros;
  unsigned int woff[PIECES], hoff[PIECES];
  const int dst0 = (tid >> 4) * kVhRowPitch + (tid & 15) * 16;
#pragma unroll
  for (int u = 0; u < PIECES; ++u) {
    const int r = (tid >> 4) + ROWS_PER_PIECE * u;
    int row = row_base + r;
    row = row < p.V ? row : p.V - 1;            // the ragged last block re-reads the last row
    const int col = r < p.cols ? r : p.cols - 1;  // columns past the end repeat the last one (never read back)
    woff[u] = (unsigned int)row * (unsigned int)(p.D * 2);
    hoff[u] = (unsigned int)col * (unsigned int)(p.D * 2);
  }
  // A request past the last step still issues its loads, so that every wait counts the same loads: it reads
  // a 256-byte block of zeros (in L2, no HBM traffic) and nothing computes from the result.
  u32x4 wreg[DIST][PIECES], hreg[DIST][PIECES];
  auto request = [&](int step, auto stage) __attribute__((always_inline)) {
    constexpr int S = decltype(stage)::value;
    // address arithmetic in integers: a select between pointers would become a branch around each load
    const bool valid = step < total_steps;
    const unsigned int mask = valid ? ~0u : 0u;
    const unsigned int st = ((unsigned int)step * (unsigned int)(2 * kVhStepK)) & mask;
    const uintptr_t hb = (valid ? h_addr : z_addr) + st, wb = (valid ? w_addr : z_addr) + st;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < PIECES; ++u) hreg[S][u] = *(const GlobalU32x4*)(hb + ((hoff[u] & mask) + lane_off));
#pragma unroll
    for (int u = 0; u < PIECES; ++u)
      wreg[S][u] = __builtin_nontemporal_load((const GlobalU32x4*)(wb + ((woff[u] & mask) + lane_off)));
    __builtin_amdgcn_sched_barrier(0);
  };
  auto commit = [&](auto stage, auto buffer) __attribute__((always_inline)) {
    constexpr int S = decltype(stage)::value, BUF = decltype(buffer)::value;
    unsigned char* hs = smem + (2 * BUF) * kVhTileBytes;
    unsigned char* ws = smem + (2 * BUF + 1) * kVhTileBytes;
#pragma unroll
    for (int u = 0; u < PIECES; ++u) *(u32x4*)(hs + (dst0 + u * ROWS_PER_PIECE * kVhRowPitch)) = hreg[S][u];
#pragma unroll
    for (int u = 0; u < PIECES; ++u) *(u32x4*)(ws + (dst0 + u * ROWS_PER_PIECE * kVhRowPitch)) = wreg[S][u];
  };
  f32x4 acc[4][2];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int aoff = (wr * 64 + c) * kVhRowPitch + g * 16, boff = (wc * 32 + c) * kVhRowPitch + g * 16;
  // compute one step from LDS buffer BUF; with COMMIT, also write stage S of the registers to the other buffer.
  // Per 32 k: the next fragments' reads and two of the tile writes are issued, then the eight MFMAs of the
  // current fragments, under which those LDS operations run.
  auto compute = [&](auto buffer, auto with_commit, auto stage) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buffer)::value, S = decltype(stage)::value;
    constexpr bool COMMIT = decltype(with_commit)::value;
    const unsigned char* hs = smem + (2 * BUF) * kVhTileBytes;
    const unsigned char* ws = smem + (2 * BUF + 1) * kVhTileBytes;
    unsigned char* hs_next = smem + (2 * (1 - BUF)) * kVhTileBytes;
    unsigned char* ws_next = smem + (2 * (1 - BUF) + 1) * kVhTileBytes;
    bf16x8 a[2][4], b[2][2];
    auto read_fragments = [&](int kk, int slot) __attribute__((always_inline)) {
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
        a[slot][rt] = __builtin_bit_cast(bf16x8, *(const u32x4*)(ws + (aoff + rt * 16 * kVhRowPitch + kk * 64)));
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
        b[slot][ct] = __builtin_bit_cast(bf16x8, *(const u32x4*)(hs + (boff + ct * 16 * kVhRowPitch + kk * 64)));
    };
    static_assert(PIECES == KK, "one hidden-state and one W piece are written per 32 k");
    __builtin_amdgcn_sched_barrier(0);
    read_fragments(0, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_barrier(0);
      if (kk + 1 < KK) read_fragments(kk + 1, (kk + 1) & 1);
      if constexpr (COMMIT) {
        *(u32x4*)(hs_next + (dst0 + kk * ROWS_PER_PIECE * kVhRowPitch)) = hreg[S][kk];
        *(u32x4*)(ws_next + (dst0 + kk * ROWS_PER_PIECE * kVhRowPitch)) = wreg[S][kk];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
          acc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kk & 1][rt], b[kk & 1][ct], acc[rt][ct], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  using I0 = std::integral_constant<int, 0>;

  // The pipelined loop takes TRIP steps per trip with no exit in between (an exit inside the trip gives the
  // loop head a second, differently ordered set of loads in flight and the waits there fall back to draining
  // everything), so the total_steps % TRIP steps that do not fill a trip run first, unpipelined.
  const int lead = total_steps % TRIP;
  for (int i = 0; i < lead; ++i) {
    request(i, I0{});
    if (i > 0) lds_barrier();
    commit(I0{}, I0{});
    lds_barrier();
    compute(I0{}, std::false_type{}, I0{});
  }
  if (lead < total_steps) {
    // local step t = step - lead uses register stage t % DIST and LDS buffer t & 1
    [&]<int... U>(std::integer_sequence<int, U...>) __attribute__((always_inline)) {
      (request(lead + U, std::integral_constant<int, U>{}), ...);
    }(std::make_integer_sequence<int, DIST>{});
    if (lead > 0) lds_barrier();
    commit(I0{}, I0{});
    request(lead + DIST, I0{});
    lds_barrier();
    for (int t = lead; t < total_steps; t += TRIP) {
      [&]<int... U>(std::integer_sequence<int, U...>) __attribute__((always_inline)) {
        // step t + U: write step t + U + 1 (after the last step: zeros into the idle buffer), refill its stage
        ((compute(std::integral_constant<int, U & 1>{}, std::true_type{}, std::integral_constant<int, (U + 1) % DIST>{}),
          request(t + U + 1 + DIST, std::integral_constant<int, (U + 1) % DIST>{}), lds_barrier()),
         ...);
      }(std::make_integer_sequence<int, TRIP>{});
    }
  }

  // ---- best (logit, id) key per column ---------------------------------------------------------------------
  // (the loop's last barrier has every wavefront done with the LDS tiles)
  if (p.logits_out) {
    // the logit block goes through LDS so that it leaves in rows of the output
    float* zbuf = (float*)smem;
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
        *(f32x4*)(zbuf + (wc * 32 + ct * 16 + c) * kVhZStride + wr * 64 + rt * 16 + g * 4) = acc[rt][ct];
    __syncthreads();
    for (int idx = tid; idx < p.cols * kRowsPerBlock; idx += NTHREADS) {
      const int m = idx / kRowsPerBlock, r = idx % kRowsPerBlock;
      if (row_base + r < p.V) p.logits_out[(size_t)(p.col0 + m) * p.V + row_base + r] = zbuf[m * kVhZStride + r];
    }
    __syncthreads();
  }
  // a lane holds 16 rows of two columns: best of those, then over the 4 lane groups (64 rows), then over the
  // two wavefronts that share the columns
  unsigned long long* kbuf = (unsigned long long*)smem;  // [2][128]
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = row_base + wr * 64 + rt * 16 + g * 4 + i;
        const unsigned long long key = row < p.V ? rank_key(acc[rt][ct][i], (unsigned)row) : 0ull;
        best = key > best ? key : best;
      }
    unsigned long long o = __shfl_xor(best, 16);
    best = o > best ? o : best;
    o = __shfl_xor(best, 32);
    best = o > best ? o : best;
    if (g == 0) kbuf[wr * kVhCols + wc * 32 + ct * 16 + c] = best;
  }
  __syncthreads();
  if (tid < p.cols) {
    const unsigned long long k0 = kbuf[tid], k1 = kbuf[kVhCols + tid];
    p.pkey[(size_t)blockIdx.x * kVhCols + tid] = k0 > k1 ? k0 : k1;
  }
}

// ---- generic kernel: thread -> (row, column), the row block's best key per column by atomic max -----------
__global__ __launch_bounds__(256) void verify_head_clear_kernel(VerifyHeadParams p) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < p.n_blocks * kVhCols; i += gridDim.x * 256) p.pkey[i] = 0ull;
}
template <typename T>
__global__ __launch_bounds__(256) void verify_head_generic_kernel(VerifyHeadParams p) {
  const int row_base = blockIdx.x * kRowsPerBlock;
  const T* hidden = (const T*)p.hidden;
  const T* w = (const T*)p.w;
  for (int idx = threadIdx.x; idx < p.cols * kRowsPerBlock; idx += 256) {
    const int m = idx / kRowsPerBlock, row = row_base + idx % kRowsPerBlock;
    if (row >= p.V) continue;
    const T* hp = hidden + (size_t)(p.col0 + m) * p.D;
    const T* wr = w + (size_t)row * p.D;
    float z = 0.f;
    for (int d = 0; d < p.D; ++d) z = fmaf(load_as_float(hp + d), load_as_float(wr + d), z);
    if (p.logits_out) p.logits_out[(size_t)(p.col0 + m) * p.V + row] = z;
    atomicMax(&p.pkey[(size_t)blockIdx.x * kVhCols + m], rank_key(z, (unsigned)row));
  }
}

// best key over the row blocks: one wavefront per column; rows of the node table without a node get -1
__global__ __launch_bounds__(64) void verify_head_merge_kernel(VerifyHeadParams p) {
  const int m = blockIdx.x, lane = threadIdx.x;
  unsigned long long best = 0ull;
  for (int b0 = 0; b0 < p.n_blocks; b0 += 256) {
    unsigned long long x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int b = b0 + u * 64 + lane;
      x[u] = b < p.n_blocks ? p.pkey[(size_t)b * kVhCols + m] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) best = x[u] > best ? x[u] : best;
  }
  best = wave_max_u64(best);
  if (lane == 0) {
    const int col = p.col0 + m;
    const int b = col / p.max_nodes, i = col - b * p.max_nodes;
    int n = p.n_nodes[b];
    n = n < 0 ? 0 : (n > p.max_nodes ? p.max_nodes : n);
    p.target[col] = i < n ? (int32_t)rank_key_index(best) : -1;
  }
}

// ---- kv_commit ------------------------------------------------------------------------------------------------
struct KvCommitParams {
  const unsigned char* k_tree;
  const unsigned char* v_tree;
  const int32_t* accept_len;
  const int32_t* accept_nodes;
  const int64_t* kv_off;
  const int32_t* ctx_len;
  unsigned char* k_cache;
  unsigned char* v_cache;
  int32_t* ctx_len_out;
  int T, kv_cap, H, max_nodes;
  int row_bytes;  // dh * element size
  int elem_bytes;
};
// one workgroup per (head, sequence); the path has at most T + 1 rows of row_bytes each
__global__ __launch_bounds__(256) void kv_commit_kernel(KvCommitParams p) {
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  int len = p.accept_len[b];
  len = len < 0 ? 0 : (len > p.T ? p.T : len);
  int L = p.ctx_len[b];
  L = L < 0 ? 0 : (L > p.kv_cap ? p.kv_cap : L);
  const size_t cache_head = ((size_t)p.kv_off[b] * p.elem_bytes) + (size_t)h * p.kv_cap * p.row_bytes;
  const size_t tree_head = ((size_t)b * p.H + h) * p.max_nodes * (size_t)p.row_bytes;
  const bool vec = (p.row_bytes & 15) == 0 && (cache_head & 15) == 0;
  for (int j = 0; j <= len; ++j) {
    const int node = p.accept_nodes[(size_t)b * (p.T + 1) + j];
    const int pos = L + j;
    if (node < 0 || node >= p.max_nodes || pos >= p.kv_cap) continue;
    const size_t src = tree_head + (size_t)node * p.row_bytes, dst = cache_head + (size_t)pos * p.row_bytes;
    if (vec) {
      for (int q = tid; q < p.row_bytes / 16; q += 256) {
        *(u32x4*)(p.k_cache + dst + q * 16) = *(const u32x4*)(p.k_tree + src + q * 16);
        *(u32x4*)(p.v_cache + dst + q * 16) = *(const u32x4*)(p.v_tree + src + q * 16);
      }
    } else {
      for (int q = tid; q < p.row_bytes; q += 256) {
        p.k_cache[dst + q] = p.k_tree[src + q];
        p.v_cache[dst + q] = p.v_tree[src + q];
      }
    }
  }
  if (h == 0 && tid == 0 && p.ctx_len_out) {
    const int grown = L + len + 1;
    p.ctx_len_out[b] = grown > p.kv_cap ? p.kv_cap : grown;
  }
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int verify_head_argmax(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* node_hidden, const void* w_base,
                                  const int32_t* n_nodes, int B, int max_nodes, int D, int V,
                                  int32_t* target_argmax, float* logits_out) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx, node_hidden && w_base && n_nodes && target_argmax, CTCSPEC_EINVAL,
                  "verify_head_argmax: null pointer");
  CTCSPEC_REQUIRE(ctx, dt == CTCSPEC_F32 || dt == CTCSPEC_BF16, CTCSPEC_EINVAL, "verify_head_argmax: bad dtype");
  CTCSPEC_REQUIRE(ctx, B > 0 && max_nodes > 0 && D > 0 && V > 0, CTCSPEC_EINVAL,
                  "verify_head_argmax: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, aligned16(node_hidden) && aligned16(w_base), CTCSPEC_EINVAL,
                  "verify_head_argmax: node_hidden and w_base must be 16-byte aligned");
  CTCSPEC_REQUIRE(ctx, B <= ctx->lim.max_batch && max_nodes <= ctx->lim.max_nodes && V <= ctx->lim.max_vocab_rows,
                  CTCSPEC_EUNSUPPORTED, "verify_head_argmax: shape exceeds the context's limits");
  VerifyHeadParams p;
  p.hidden = node_hidden; p.w = w_base; p.D = D; p.V = V;
  p.n_blocks = (V + kRowsPerBlock - 1) / kRowsPerBlock;
  p.zeros = ctx->zeros; p.pkey = ctx->vh_pkey; p.logits_out = logits_out; p.n_nodes = n_nodes; p.max_nodes = max_nodes;
  p.target = target_argmax;
  const long long cols_total = (long long)B * max_nodes;
  const bool wide = dt == CTCSPEC_BF16 && D % kVhStepK == 0 && (long long)V * D * 2 < (1LL << 32) &&
                    cols_total * D * 2 < (1LL << 32);
  const int lds = kVhLdsBytes;
  if (wide) {
    static bool lds_allowed = false;  // raising the limit is needed once per process
    if (!lds_allowed) {
      CTCSPEC_HIP(ctx, hipFuncSetAttribute((const void*)verify_head_bf16_kernel<kVhDist>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds));
      lds_allowed = true;
    }
  }
  for (long long col0 = 0; col0 < cols_total; col0 += kVhCols) {
    p.col0 = (int)col0;
    p.cols = (int)(cols_total - col0 < kVhCols ? cols_total - col0 : kVhCols);
    if (wide) {
      hipLaunchKernelGGL(verify_head_bf16_kernel<kVhDist>, dim3(p.n_blocks), dim3(64 * kVhWaves), lds, ctx->stream, p);
    } else {
      hipLaunchKernelGGL(verify_head_clear_kernel, dim3(64), dim3(256), 0, ctx->stream, p);
      if (dt == CTCSPEC_BF16)
        hipLaunchKernelGGL(verify_head_generic_kernel<unsigned short>, dim3(p.n_blocks), dim3(256), 0, ctx->stream, p);
      else
        hipLaunchKernelGGL(verify_head_generic_kernel<float>, dim3(p.n_blocks), dim3(256), 0, ctx->stream, p);
    }
    CTCSPEC_HIP(ctx, hipGetLastError());
    hipLaunchKernelGGL(verify_head_merge_kernel, dim3(p.cols), dim3(64), 0, ctx->stream, p);
    CTCSPEC_HIP(ctx, hipGetLastError());
  }
  return CTCSPEC_OK;
}

extern "C" int kv_commit(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* k_tree, const void* v_tree,
                         const int32_t* accept_len, const int32_t* accept_nodes, int T, const int64_t* kv_off,
                         const int32_t* ctx_len, int kv_cap, int B, int H, int dh, int max_nodes, void* k_cache,
                         void* v_cache, int32_t* ctx_len_out) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx, k_tree && v_tree && accept_len && accept_nodes && kv_off && ctx_len && k_cache && v_cache,
                  CTCSPEC_EINVAL, "kv_commit: null pointer");
  CTCSPEC_REQUIRE(ctx, dt == CTCSPEC_F32 || dt == CTCSPEC_BF16, CTCSPEC_EINVAL, "kv_commit: bad dtype");
  CTCSPEC_REQUIRE(ctx, B > 0 && H > 0 && dh > 0 && max_nodes > 0 && T > 0 && kv_cap >= 0, CTCSPEC_EINVAL,
                  "kv_commit: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, ctx_len_out != ctx_len, CTCSPEC_EINVAL,
                  "kv_commit: ctx_len_out must not be ctx_len (every head's workgroup reads the old length)");
  CTCSPEC_REQUIRE(ctx, B <= 65535 && T <= CTCSPEC_MAX_SLOTS, CTCSPEC_EUNSUPPORTED,
                  "kv_commit: B <= 65535 and T <= %d required", CTCSPEC_MAX_SLOTS);
  KvCommitParams p;
  p.elem_bytes = dt == CTCSPEC_BF16 ? 2 : 4;
  p.k_tree = (const unsigned char*)k_tree; p.v_tree = (const unsigned char*)v_tree;
  p.accept_len = accept_len; p.accept_nodes = accept_nodes; p.kv_off = kv_off; p.ctx_len = ctx_len;
  p.k_cache = (unsigned char*)k_cache; p.v_cache = (unsigned char*)v_cache; p.ctx_len_out = ctx_len_out;
  p.T = T; p.kv_cap = kv_cap; p.H = H; p.max_nodes = max_nodes; p.row_bytes = dh * p.elem_bytes;
  hipLaunchKernelGGL(kv_commit_kernel, dim3(H, B), dim3(256), 0, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
