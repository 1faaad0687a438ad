// tree_verify_attn: tree-masked verification attention of the base model, one layer.
//
// Two kernels:
//   * tree_attn_bf16_kernel    - bf16 operands, head dimension 128: MFMA for Q.K^T and P.V, online
//                                softmax, every wavefront streams its own share of the keys
//   * tree_attn_generic_kernel - any dtype / head dimension within the limits: one workgroup per
//                                (node, head, sequence), keys in chunks with an online softmax
#include "common.h"

namespace ctcspec {

struct AttnParams {
  const void* q;
  const void* k_cache;
  const void* v_cache;
  const int64_t* kv_off;
  const int32_t* ctx_len;
  int kv_cap;
  const void* k_tree;
  const void* v_tree;
  const int32_t* n_nodes;
  const unsigned long long* anc_mask;
  int B, H, dh, max_nodes;
  float scale;
  float* out;
};

constexpr int kGenericThreads = 256;
constexpr int kGenericChunk = 1024;

template <typename T>
__global__ __launch_bounds__(kGenericThreads) void tree_attn_generic_kernel(AttnParams p) {
  __shared__ float qs[CTCSPEC_MAX_HEAD_DIM];
  __shared__ float sc[kGenericChunk];
  __shared__ float red[kGenericThreads / 64];
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n = p.n_nodes[b];
  n = n > p.max_nodes ? p.max_nodes : n;
  if (i >= n) return;
  const int dh = p.dh;
  int L = p.ctx_len[b];
  L = L < 0 ? 0 : (L > p.kv_cap ? p.kv_cap : L);
  const int W = (p.max_nodes + 63) / 64;
  const unsigned long long* mrow = p.anc_mask + ((size_t)b * p.max_nodes + i) * W;
  const size_t node_base = ((size_t)b * p.H + h) * p.max_nodes;
  const T* q = (const T*)p.q + (node_base + i) * dh;
  const T* kc = (const T*)p.k_cache + p.kv_off[b] + (size_t)h * p.kv_cap * dh;
  const T* vc = (const T*)p.v_cache + p.kv_off[b] + (size_t)h * p.kv_cap * dh;
  const T* kt = (const T*)p.k_tree + node_base * dh;
  const T* vt = (const T*)p.v_tree + node_base * dh;
  if (tid < dh) qs[tid] = load_as_float(q + tid);
  __syncthreads();

  const int total = L + n;  // key j < L: cache row j; else tree node j-L (subject to the mask)
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;  // acc: output component tid (tid < dh)
  for (int c0 = 0; c0 < total; c0 += kGenericChunk) {
    const int cn = total - c0 < kGenericChunk ? total - c0 : kGenericChunk;
    float mloc = -INFINITY;
    for (int jj = tid; jj < cn; jj += kGenericThreads) {
      const int j = c0 + jj;
      float s = -INFINITY;
      bool vis = true;
      const T* kr;
      if (j < L) kr = kc + (size_t)j * dh;
      else {
        int t = j - L;
        vis = (mrow[t >> 6] >> (t & 63)) & 1ull;
        kr = kt + (size_t)t * dh;
      }
      if (vis) {
        float d = 0.f;
        for (int e = 0; e < dh; ++e) d = fmaf(qs[e], load_as_float(kr + e), d);
        s = d * p.scale;
      }
      sc[jj] = s;
      mloc = fmaxf(mloc, s);
    }
    mloc = wave_max_f32(mloc);
    __syncthreads();
    if (lane == 0) red[wave] = mloc;
    __syncthreads();
    float m_new = m_run;
    for (int w = 0; w < kGenericThreads / 64; ++w) m_new = fmaxf(m_new, red[w]);
    // m_new is finite from the first chunk on: the first chunk holds a cache key or the root (tree
    // node 0, visible to every node)
    float lloc = 0.f;
    for (int jj = tid; jj < cn; jj += kGenericThreads) {
      float s = sc[jj];
      float pj = s > -INFINITY ? __expf(s - m_new) : 0.f;
      sc[jj] = pj;
      lloc += pj;
    }
    lloc = wave_sum_f32(lloc);
    __syncthreads();
    if (lane == 0) red[wave] = lloc;
    __syncthreads();
    float lsum = 0.f;
    for (int w = 0; w < kGenericThreads / 64; ++w) lsum += red[w];
    const float alpha = m_run > -INFINITY ? __expf(m_run - m_new) : 0.f;
    l_run = l_run * alpha + lsum;
    if (tid < dh) {
      float a = acc * alpha;
      for (int jj = 0; jj < cn; ++jj) {
        float pj = sc[jj];
        if (pj != 0.f) {
          const int j = c0 + jj;
          const T* vr = j < L ? vc + (size_t)j * dh : vt + (size_t)(j - L) * dh;
          a = fmaf(pj, load_as_float(vr + tid), a);
        }
      }
      acc = a;
    }
    m_run = m_new;
    __syncthreads();
  }
  if (tid < dh) p.out[(node_base + i) * dh + tid] = acc / l_run;
}


// ---- bf16, dh = 128 -------------------------------------------------------------------------------
// Workgroup = kAttnWaves wavefronts = one block of 16 query nodes of one (sequence, head).  The keys
// (cached context rows first, then the tree nodes) are cut into tiles of 32; wavefront w takes tiles
// w, w+kAttnWaves, ... and runs its own online softmax over them; the wavefronts' partial results are
// merged through LDS at the end, so there is no second kernel and no partial result in HBM.
//
// Per tile and wavefront:
//   S^T[key, q] = K.Q^T   : A = K rows (staged through a private LDS strip to get from coalesced
//                           256-byte row reads to the MFMA A layout), B = Q^T (resident in VGPRs)
//   P = exp2(S^T*c - m)   : in the MFMA C layout a lane holds 8 keys of ONE query column, so the
//                           running max/sum are per lane plus a 4-lane exchange
//   O^T[dh, q] += V^T.P   : P stays in registers as the B operand (hi + lo bf16 halves, so that P
//                           carries 16 mantissa bits); V is read straight from global memory, 16
//                           bytes (8 consecutive dh of one key) per lane and load, and an 8x8 16-bit
//                           transpose inside the lane turns that into A operands.  MFMA row r of
//                           output block db stands for dh = 8*r + db, which makes every V load a
//                           contiguous 16 bytes; the permutation is undone when O is written.
// Workgroups of the same (sequence, head) differ only in the query block and are given block
// indices congruent modulo 8, i.e. the same XCD, so K/V are fetched from HBM once and re-read from
// that XCD's L2.
constexpr int kAttnWaves = 4;
constexpr int kTileKeys = 32;
constexpr int kStripRow = 256 + 16;                    // bytes per staged K row
constexpr int kStripBytes = kTileKeys * kStripRow;     // per wavefront
constexpr int kMergeRow = 128 + 4;                     // floats per query row in the merge buffer
constexpr int kMergeBytes = 16 * kMergeRow * 4;        // per wavefront
constexpr int kAttnLdsPerWave = kStripBytes > kMergeBytes ? kStripBytes : kMergeBytes;

__global__ __launch_bounds__(64 * kAttnWaves) void tree_attn_bf16_kernel(AttnParams p, int QB) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float m_sh[kAttnWaves][16];
  __shared__ float l_sh[kAttnWaves][16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 15, g = lane >> 4;
  int bid = blockIdx.x;
  const int h = bid % p.H;
  bid /= p.H;
  const int qb = bid % QB;
  const int b = bid / QB;
  int n = p.n_nodes[b];
  n = n < 1 ? 1 : (n > p.max_nodes ? p.max_nodes : n);
  if (qb * 16 >= n) return;
  int L = p.ctx_len[b];
  L = L < 0 ? 0 : (L > p.kv_cap ? p.kv_cap : L);

  const size_t node_base = ((size_t)b * p.H + h) * p.max_nodes;
  const unsigned char* kc = (const unsigned char*)p.k_cache + ((size_t)p.kv_off[b] + (size_t)h * p.kv_cap * 128) * 2;
  const unsigned char* vc = (const unsigned char*)p.v_cache + ((size_t)p.kv_off[b] + (size_t)h * p.kv_cap * 128) * 2;
  const unsigned char* kt = (const unsigned char*)p.k_tree + node_base * 256;
  const unsigned char* vt = (const unsigned char*)p.v_tree + node_base * 256;

  // this lane's query column: Q fragments (B operand of K.Q^T) and mask words
  const int qi = qb * 16 + c;
  const int qrow = qi < p.max_nodes ? qi : p.max_nodes - 1;
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    qf[kk] = __builtin_bit_cast(
        bf16x8, *(const u32x4*)((const unsigned char*)p.q + (node_base + qrow) * 256 + kk * 64 + g * 16));
  const int W = (p.max_nodes + 63) >> 6;
  unsigned long long mw0 = 0ull, mw1 = 0ull;
  if (qi < n) {
    const unsigned long long* mrow = p.anc_mask + ((size_t)b * p.max_nodes + qi) * W;
    mw0 = mrow[0];
    if (W > 1) mw1 = mrow[1];
  }

  const int ctxT = (L + kTileKeys - 1) / kTileKeys, treeT = (n + kTileKeys - 1) / kTileKeys;
  const int NTL = ctxT + treeT;
  const float sl2 = p.scale * 1.4426950408889634f;
  unsigned char* strip = smem + wave * kAttnLdsPerWave;

  f32x4 o[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) o[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  u32x4 kr[8], vr[8];
  // tile t: rows [row0, row0+32) of `src`, rows >= limit do not exist (clamped for loads, masked later)
  auto issue_k = [&](int t) {
    const bool tree = t >= ctxT;
    const unsigned char* src = tree ? kt : kc;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys, limit = tree ? n : L;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int row = row0 + 4 * j + g;
      row = row < limit ? row : limit - 1;
      kr[j] = *(const u32x4*)(src + (size_t)row * 256 + c * 16);
    }
  };
  auto issue_v = [&](int t) {
    const bool tree = t >= ctxT;
    const unsigned char* src = tree ? vt : vc;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys, limit = tree ? n : L;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int row = row0 + (j >> 2) * 16 + 4 * g + (j & 3);  // key slot (g, j) of the P.V contraction
      row = row < limit ? row : limit - 1;
      vr[j] = *(const u32x4*)(src + (size_t)row * 256 + c * 16);
    }
  };

  int t = wave;
  if (t < NTL) {
    issue_k(t);
    issue_v(t);
  }
  for (; t < NTL; t += kAttnWaves) {
    const bool tree = t >= ctxT;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys;
    // K tile -> private strip (row = key, 272-byte pitch), then the next tile's K loads
#pragma unroll
    for (int j = 0; j < 8; ++j) *(u32x4*)(strip + (4 * j + g) * kStripRow + c * 16) = kr[j];
    const int tn = t + kAttnWaves;
    if (tn < NTL) issue_k(tn);
    // S^T = K.Q^T for the two blocks of 16 keys
    f32x4 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      s[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)(strip + (kb * 16 + c) * kStripRow + kk * 64 + g * 16));
        s[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[kk], s[kb], 0, 0, 0);
      }
    }
    // visibility, scaling, running max
    float sv[8];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = row0 + kb * 16 + 4 * g + i;
        bool vis;
        if (tree) vis = (((key < 64 ? mw0 : mw1) >> (key & 63)) & 1ull) != 0ull;
        else vis = key < L;
        const float x = vis ? s[kb][i] * sl2 : -INFINITY;
        sv[kb * 4 + i] = x;
        mx = fmaxf(mx, x);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_safe = m_new > -INFINITY ? m_new : 0.f;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
    float psum = 0.f;
    bf16x8 ph, pl;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float pj = __builtin_amdgcn_exp2f(sv[j] - m_safe);
      psum += pj;
      const __bf16 hi = (__bf16)pj;
      ph[j] = hi;
      pl[j] = (__bf16)(pj - (float)hi);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < 8; ++db) o[db] *= alpha;
    // O^T += V^T.P; the A operand of output block db is column db of this lane's 8x8 V block
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      u32x4 a4;
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) {
        const unsigned int x = vr[2 * jp][db >> 1], y = vr[2 * jp + 1][db >> 1];
        a4[jp] = __builtin_amdgcn_perm(y, x, (db & 1) ? 0x07060302u : 0x05040100u);
      }
      const bf16x8 a = __builtin_bit_cast(bf16x8, a4);
      o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ph, o[db], 0, 0, 0);
      o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pl, o[db], 0, 0, 0);
    }
    if (tn < NTL) issue_v(tn);
  }

  // ---- merge the wavefronts' partial results --------------------------------------------------
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (g == 0) {
    m_sh[wave][c] = m_run;
    l_sh[wave][c] = l_run;
  }
  __syncthreads();  // also: every wavefront is done with its strip, which the merge buffer reuses
  float* ob = (float*)(smem + wave * kAttnLdsPerWave);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // lane (c, g) holds O[q = c][dh = 32g + 8i + db], db = 0..7
    f32x4 lo4 = {o[0][i], o[1][i], o[2][i], o[3][i]};
    f32x4 hi4 = {o[4][i], o[5][i], o[6][i], o[7][i]};
    *(f32x4*)(ob + c * kMergeRow + 32 * g + 8 * i) = lo4;
    *(f32x4*)(ob + c * kMergeRow + 32 * g + 8 * i + 4) = hi4;
  }
  __syncthreads();
  constexpr int kRowsPerWave = 16 / kAttnWaves;
#pragma unroll
  for (int rr = 0; rr < kRowsPerWave; ++rr) {
    const int qr = wave * kRowsPerWave + rr;
    const int qg = qb * 16 + qr;
    if (qg >= n) continue;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, m_sh[w][qr]);
    float Lt = 0.f, a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      const float mw = m_sh[w][qr];
      const float f = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - M) : 0.f;
      const float* src = (const float*)(smem + w * kAttnLdsPerWave) + qr * kMergeRow;
      Lt += f * l_sh[w][qr];
      a0 += f * src[lane];
      a1 += f * src[lane + 64];
    }
    const float inv = 1.0f / Lt;
    float* dst = p.out + (node_base + qg) * 128;
    dst[lane] = a0 * inv;
    dst[lane + 64] = a1 * inv;
  }
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int tree_verify_attn(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* q, const void* k_cache,
                                const void* v_cache, const int64_t* kv_off, const int32_t* ctx_len, int kv_cap,
                                const void* k_tree, const void* v_tree, const int32_t* n_nodes,
                                const uint64_t* anc_mask, int B, int H, int dh, int max_nodes, float scale,
                                float* out) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx, q && k_cache && v_cache && kv_off && ctx_len && k_tree && v_tree && n_nodes && anc_mask && out,
                  CTCSPEC_EINVAL, "tree_verify_attn: null pointer");
  CTCSPEC_REQUIRE(ctx, dt == CTCSPEC_F32 || dt == CTCSPEC_BF16, CTCSPEC_EINVAL, "tree_verify_attn: bad dtype");
  CTCSPEC_REQUIRE(ctx, B > 0 && H > 0 && dh > 0 && max_nodes > 0 && kv_cap >= 0, CTCSPEC_EINVAL,
                  "tree_verify_attn: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, aligned16(q) && aligned16(k_cache) && aligned16(v_cache) && aligned16(k_tree) &&
                           aligned16(v_tree),
                  CTCSPEC_EINVAL, "tree_verify_attn: q/k/v pointers must be 16-byte aligned");
  CTCSPEC_REQUIRE(ctx, dh <= CTCSPEC_MAX_HEAD_DIM && dh % 8 == 0 && max_nodes <= CTCSPEC_MAX_NODES,
                  CTCSPEC_EUNSUPPORTED, "tree_verify_attn: dh<=%d, dh%%8==0, max_nodes<=%d required",
                  CTCSPEC_MAX_HEAD_DIM, CTCSPEC_MAX_NODES);
  CTCSPEC_REQUIRE(ctx, B <= ctx->lim.max_batch && H <= ctx->lim.max_heads && dh <= ctx->lim.max_head_dim &&
                           max_nodes <= ctx->lim.max_nodes,
                  CTCSPEC_EUNSUPPORTED, "tree_verify_attn: shape exceeds the context's limits");
  CTCSPEC_REQUIRE(ctx, B <= 65535 && H <= 65535, CTCSPEC_EUNSUPPORTED, "tree_verify_attn: grid too large");

  AttnParams p;
  p.q = q; p.k_cache = k_cache; p.v_cache = v_cache; p.kv_off = kv_off; p.ctx_len = ctx_len; p.kv_cap = kv_cap;
  p.k_tree = k_tree; p.v_tree = v_tree; p.n_nodes = n_nodes; p.anc_mask = (const unsigned long long*)anc_mask;
  p.B = B; p.H = H; p.dh = dh; p.max_nodes = max_nodes; p.scale = scale; p.out = out;
  if (dt == CTCSPEC_BF16 && dh == 128) {
    const int QB = (max_nodes + 15) / 16;
    const long long blocks = (long long)QB * H * B;
    CTCSPEC_REQUIRE(ctx, blocks <= 0x7fffffffLL, CTCSPEC_EUNSUPPORTED, "tree_verify_attn: grid too large");
    const int lds = kAttnWaves * kAttnLdsPerWave;
    static int lds_allowed = 0;
    if (lds > lds_allowed) {
      CTCSPEC_HIP(ctx, hipFuncSetAttribute((const void*)tree_attn_bf16_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds));
      lds_allowed = lds;
    }
    hipLaunchKernelGGL(tree_attn_bf16_kernel, dim3((unsigned)blocks), dim3(64 * kAttnWaves), lds, ctx->stream, p, QB);
    CTCSPEC_HIP(ctx, hipGetLastError());
    return CTCSPEC_OK;
  }
  dim3 grid(max_nodes, H, B);
  if (dt == CTCSPEC_BF16)
    hipLaunchKernelGGL(tree_attn_generic_kernel<unsigned short>, grid, dim3(kGenericThreads), 0, ctx->stream, p);
  else
    hipLaunchKernelGGL(tree_attn_generic_kernel<float>, grid, dim3(kGenericThreads), 0, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
