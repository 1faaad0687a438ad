// verify_head_argmax: the base model's LM head over the hidden states of the tree nodes, reduced to the
// greedy token per node.  kv_commit: append the accepted path's keys and values to the cached context.
//
// The head is the same stream over a [V, D] weight matrix as the draft head, but with up to 128 columns
// (one per tree node) instead of 8, and all that is kept of a column is its best (logit, id) key:
//   * verify_head_bf16_kernel    - bf16, D a multiple of 128: MFMA, 128 vocabulary rows x 128 columns per
//                                  workgroup (256 x 128 when there are several column blocks); all column blocks
//                                  in one launch, those of a row block side by side on one XCD (the weights come
//                                  from HBM once)
//   * verify_head_generic_kernel - any dtype/shape: plain fp32 FMA, one atomic max per (row block, column)
//   * verify_head_merge_kernel   - best key over the row blocks -> token id, -1 for rows without a node
#include "gemm_tile.h"

namespace ctcspec {

constexpr int kVhCols = kVerifyCols;            // columns (tree nodes) per pass over the weights
constexpr int kVhWaves = kTileWaves;
constexpr int kVhDist = 4;                      // prefetch distance in steps = register stages per operand
constexpr int kVhStepK = kTileStepK;
// dynamic LDS of a tile shape: the staging buffers, or the logit block (column-major, 4 floats of pad per column)
// when the caller asks for logits - whichever is larger
template <typename SH>
constexpr int vh_lds_bytes() {
  return SH::LDS_BYTES > kVhCols * (SH::ROWS + 4) * 4 ? SH::LDS_BYTES : kVhCols * (SH::ROWS + 4) * 4;
}
static_assert(kVhCols == 128 && Tile128x128::COLS == kVhCols && Tile256x128::COLS == kVhCols, "tile shape");
static_assert(vh_lds_bytes<Tile256x128>() <= 160 * 1024, "fits the compute unit's LDS");

struct VerifyHeadParams {
  const void* hidden;   // [cols_total][D]
  const void* w;        // [V][D]
  int col0, cols;       // generic kernels: columns of this launch (cols <= kVhCols), a whole column block
  int cols_total;       // all columns of the call; the bf16 kernel covers them in one launch, block by block
  int col_blocks;       // ceil(cols_total / kVhCols)
  int D, V;
  int n_blocks;         // row blocks (of the tile shape's rows: 128 or 256)
  unsigned long long* pkey;  // [col_blocks][n_blocks][kVhCols] best key per (column block, row block, column)
  float* logits_out;    // [cols_total][V] or null
  const void* zeros;    // 256 bytes of zeros
  const int32_t* n_nodes;  // [B]
  int max_nodes;
  int32_t* target;      // [cols_total]
};

// ---- bf16 MFMA kernel: the shared 128 x 128 tile loop, then the best (logit, id) key per column -----------------
template <int DIST, typename SH>
__global__ __launch_bounds__(64 * kVhWaves) void verify_head_bf16_kernel(VerifyHeadParams p) {
  constexpr int ROWS = SH::ROWS, CTW = SH::CTW, WR = SH::WR;
  constexpr int ZSTRIDE = ROWS + 4;  // floats per column of the logit block
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NTHREADS = 64 * kVhWaves;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave / SH::WC, wc = wave % SH::WC;
  const int c = lane & 15, g = lane >> 4;
  // Workgroup -> (row block, column block).  Workgroups are dealt to the 8 XCDs round robin, and each XCD has its
  // own L2: the column blocks of one row block get workgroup numbers that differ by multiples of 8 and are
  // neighbours in dispatch order, so they run on the same XCD at about the same time and the weight tile that the
  // first of them pulls from HBM serves the others from that L2 - one pass over the weights in HBM for any number
  // of columns.  (One column block: row block = workgroup number.)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int cb = slot % p.col_blocks, rb = (slot / p.col_blocks) * 8 + xcd;
  if (rb >= p.n_blocks) return;
  const int col0 = cb * kVhCols;
  const int cols = p.cols_total - col0 < kVhCols ? p.cols_total - col0 : kVhCols;
  const int row_base = rb * ROWS;
  GemmTileArgs t;
  t.w = p.w; t.hidden = (const unsigned char*)p.hidden + (size_t)col0 * p.D * 2; t.zeros = p.zeros;
  t.D = p.D; t.V = p.V; t.cols = cols; t.row_base = row_base;
  f32x4 acc[4][CTW];
  gemm_tile<DIST, SH>(t, smem, acc);

  // ---- best (logit, id) key per column ---------------------------------------------------------------------
  // (the loop's last barrier has every wavefront done with the LDS tiles)
  if (p.logits_out) {
    // the logit block goes through LDS so that it leaves in rows of the output
    float* zbuf = (float*)smem;
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
      for (int ct = 0; ct < CTW; ++ct)
        *(f32x4*)(zbuf + (wc * 16 * CTW + ct * 16 + c) * ZSTRIDE + wr * 64 + rt * 16 + g * 4) = acc[rt][ct];
    __syncthreads();
    for (int idx = tid; idx < cols * ROWS; idx += NTHREADS) {
      const int m = idx / ROWS, r = idx % ROWS;
      if (row_base + r < p.V) p.logits_out[(size_t)(col0 + m) * p.V + row_base + r] = zbuf[m * ZSTRIDE + r];
    }
    __syncthreads();
  }
  // a lane holds 16 rows of CTW columns: best of those, then over the 4 lane groups (64 rows), then over the
  // WR wavefronts that share the columns
  unsigned long long* kbuf = (unsigned long long*)smem;  // [WR][128]
#pragma unroll
  for (int ct = 0; ct < CTW; ++ct) {
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
    if (g == 0) kbuf[wr * kVhCols + wc * 16 * CTW + ct * 16 + c] = best;
  }
  __syncthreads();
  if (tid < cols) {
    unsigned long long best = kbuf[tid];
#pragma unroll
    for (int r = 1; r < WR; ++r) {
      const unsigned long long o = kbuf[r * kVhCols + tid];
      best = o > best ? o : best;
    }
    p.pkey[((size_t)cb * p.n_blocks + rb) * kVhCols + tid] = best;
  }
}

// ---- generic kernel: thread -> (row, column), the row block's best key per column by atomic max -----------
__global__ __launch_bounds__(256) void verify_head_clear_kernel(VerifyHeadParams p) {
  unsigned long long* pk = p.pkey + (size_t)(p.col0 / kVhCols) * p.n_blocks * kVhCols;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < p.n_blocks * kVhCols; i += gridDim.x * 256) pk[i] = 0ull;
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
    atomicMax(&p.pkey[((size_t)(p.col0 / kVhCols) * p.n_blocks + blockIdx.x) * kVhCols + m], rank_key(z, (unsigned)row));
  }
}

// best key over the row blocks: one wavefront per column; rows of the node table without a node get -1
__global__ __launch_bounds__(64) void verify_head_merge_kernel(VerifyHeadParams p) {
  const int col = p.col0 + blockIdx.x, lane = threadIdx.x;  // column of the call
  const int m = col % kVhCols;
  const unsigned long long* pk = p.pkey + (size_t)(col / kVhCols) * p.n_blocks * kVhCols;
  unsigned long long best = 0ull;
  for (int b0 = 0; b0 < p.n_blocks; b0 += 256) {
    unsigned long long x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int b = b0 + u * 64 + lane;
      x[u] = b < p.n_blocks ? pk[(size_t)b * kVhCols + m] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) best = x[u] > best ? x[u] : best;
  }
  best = wave_max_u64(best);
  if (lane == 0) {
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
  // 16-byte copies need every address a multiple of 16: the offsets and the four base pointers
  const bool vec = (p.row_bytes & 15) == 0 && (cache_head & 15) == 0 &&
                   ((((uintptr_t)p.k_cache | (uintptr_t)p.v_cache | (uintptr_t)p.k_tree | (uintptr_t)p.v_tree) & 15) == 0);
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

hipError_t prepare_verify_head() {
  hipError_t e = hipFuncSetAttribute((const void*)verify_head_bf16_kernel<kVhDist, Tile128x128>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, vh_lds_bytes<Tile128x128>());
  if (e == hipSuccess)
    e = hipFuncSetAttribute((const void*)verify_head_bf16_kernel<kVhDist, Tile256x128>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, vh_lds_bytes<Tile256x128>());
  return e;
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int verify_head_argmax(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* node_hidden, const void* w_base,
                                  const int32_t* n_nodes, int B, int max_nodes, int D, int V,
                                  int32_t* target_argmax, float* logits_out) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
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
  p.cols_total = (int)cols_total;
  p.col_blocks = (int)((cols_total + kVhCols - 1) / kVhCols);
  CTCSPEC_REQUIRE(ctx, p.col_blocks <= ctx->vh_col_blocks, CTCSPEC_EUNSUPPORTED,
                  "verify_head_argmax: %lld columns exceed the context's workspace", cols_total);
  if (wide) {
    // one launch for every column block (the kernel's workgroup numbering keeps a row block's column blocks on
    // one XCD), one merge launch over all columns.  One column block: 128-row tiles, one workgroup per compute
    // unit, the stream from HBM sets the pace.  Several: 256-row tiles - the workgroups of a row block share the
    // weight tile through L2 and the loop's own LDS traffic sets the pace, which the larger tile halves per flop.
    p.col0 = 0; p.cols = 0;
    const bool tall = p.col_blocks > 1;
    const int rows = tall ? Tile256x128::ROWS : Tile128x128::ROWS;
    p.n_blocks = (V + rows - 1) / rows;
    const long long grid = (long long)((p.n_blocks + 7) / 8) * 8 * p.col_blocks;
    CTCSPEC_REQUIRE(ctx, grid <= 0x7fffffffLL, CTCSPEC_EUNSUPPORTED, "verify_head_argmax: grid too large");
    if (tall)
      hipLaunchKernelGGL((verify_head_bf16_kernel<kVhDist, Tile256x128>), dim3((unsigned)grid), dim3(64 * kVhWaves),
                         vh_lds_bytes<Tile256x128>(), ctx->stream, p);
    else
      hipLaunchKernelGGL((verify_head_bf16_kernel<kVhDist, Tile128x128>), dim3((unsigned)grid), dim3(64 * kVhWaves),
                         vh_lds_bytes<Tile128x128>(), ctx->stream, p);
    CTCSPEC_HIP(ctx, hipGetLastError());
    hipLaunchKernelGGL(verify_head_merge_kernel, dim3((unsigned)cols_total), dim3(64), 0, ctx->stream, p);
    CTCSPEC_HIP(ctx, hipGetLastError());
    return CTCSPEC_OK;
  }
  for (long long col0 = 0; col0 < cols_total; col0 += kVhCols) {
    p.col0 = (int)col0;
    p.cols = (int)(cols_total - col0 < kVhCols ? cols_total - col0 : kVhCols);
    hipLaunchKernelGGL(verify_head_clear_kernel, dim3(64), dim3(256), 0, ctx->stream, p);
    if (dt == CTCSPEC_BF16)
      hipLaunchKernelGGL(verify_head_generic_kernel<unsigned short>, dim3(p.n_blocks), dim3(256), 0, ctx->stream, p);
    else
      hipLaunchKernelGGL(verify_head_generic_kernel<float>, dim3(p.n_blocks), dim3(256), 0, ctx->stream, p);
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
  if (const int owed = flush_deferred(ctx)) return owed;
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
