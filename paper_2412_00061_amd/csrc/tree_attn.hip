// tree_verify_attn: tree-masked verification attention of the base model, one layer.
//
// Two kernels:
//   * tree_attn_bf16_kernel    - bf16 operands, head dimension 128: MFMA for Q.K^T and P.V, online
//                                softmax, every wavefront streams its own share of the keys
//   * tree_attn_generic_kernel - any dtype / head dimension within the limits: one workgroup per
//                                (node, head, sequence), keys in chunks with an online softmax
#include <stdlib.h>

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
// Workgroup = kAttnWaves wavefronts = one block of 16*QT query nodes of one (sequence, head) and one
// of S splits of the keys.  The keys (cached context rows first, then the tree nodes) are cut into
// tiles of 32; the 4*S wavefronts that share a query block take the tiles round robin, each running
// its own online softmax; a workgroup's wavefronts are merged through LDS at the end.  With S == 1
// that is the result; otherwise the workgroup leaves an unnormalised partial (O, max, sum) in the
// context workspace and tree_attn_merge_kernel combines the S partials.
//
// Per tile and wavefront:
//   S^T[key, q] = K.Q^T   : A = K rows (staged through a private LDS strip to get from coalesced
//                           256-byte row reads to the MFMA A layout), B = Q^T (resident in VGPRs);
//                           every K fragment is used for all QT query tiles
//   P = exp2(S^T*c - m)   : in the MFMA C layout a lane holds 8 keys of ONE query column, so the
//                           running max/sum are per lane plus a 4-lane exchange
//   O^T[dh, q] += V^T.P   : P stays in registers as the B operand (hi + lo bf16 halves, so that P
//                           carries 16 mantissa bits); V is read straight from global memory, 16
//                           bytes (8 consecutive dh of one key) per lane and load, and an 8x8 16-bit
//                           transpose inside the lane turns that into A operands, shared by the QT
//                           query tiles.  MFMA row r of output block db stands for dh = 8*r + db,
//                           which makes every V load a contiguous 16 bytes; the permutation is
//                           undone when O is written.
// K/V are re-read once per query block; workgroups of the same (sequence, head) are given block
// indices congruent modulo 8, i.e. the same XCD, so those re-reads are served by that XCD's L2.
constexpr int kAttnWaves = 4;
constexpr int kTileKeys = 32;
constexpr int kStripRow = 256 + 16;                    // bytes per staged K row
constexpr int kStripBytes = kTileKeys * kStripRow;     // per wavefront
constexpr int kMergeRow = 128 + 4;                     // floats per query row in the merge buffer

template <int QT>
constexpr int attn_lds_per_wave() {
  return kStripBytes > QT * 16 * kMergeRow * 4 ? kStripBytes : QT * 16 * kMergeRow * 4;
}

struct AttnSplit {
  int QB;      // query blocks of 16*QT rows
  int S;       // key splits
  float* po;   // [unit][16*QT][128] partial O (unnormalised), unit = ((b*H + h)*QB + qb)*S + s
  float* pm;   // [unit][16*QT] running max (log2 domain)
  float* pl;   // [unit][16*QT] running sum
};

template <int QT>
__global__ __launch_bounds__(64 * kAttnWaves) void tree_attn_bf16_kernel(AttnParams p, AttnSplit sp) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float m_sh[kAttnWaves][16 * QT];
  __shared__ float l_sh[kAttnWaves][16 * QT];
  constexpr int kLdsPerWave = attn_lds_per_wave<QT>();
  constexpr int ROWS = 16 * QT;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 15, g = lane >> 4;
  int bid = blockIdx.x;
  const int h = bid % p.H;
  bid /= p.H;
  const int split = bid % sp.S;
  bid /= sp.S;
  const int qb = bid % sp.QB;
  const int b = bid / sp.QB;
  int n = p.n_nodes[b];
  n = n < 1 ? 1 : (n > p.max_nodes ? p.max_nodes : n);
  if (qb * ROWS >= n) return;
  int L = p.ctx_len[b];
  L = L < 0 ? 0 : (L > p.kv_cap ? p.kv_cap : L);

  const size_t node_base = ((size_t)b * p.H + h) * p.max_nodes;
  const unsigned char* kc = (const unsigned char*)p.k_cache + ((size_t)p.kv_off[b] + (size_t)h * p.kv_cap * 128) * 2;
  const unsigned char* vc = (const unsigned char*)p.v_cache + ((size_t)p.kv_off[b] + (size_t)h * p.kv_cap * 128) * 2;
  const unsigned char* kt = (const unsigned char*)p.k_tree + node_base * 256;
  const unsigned char* vt = (const unsigned char*)p.v_tree + node_base * 256;

  // this lane's query columns (one per query tile): Q fragments (B operand of K.Q^T) and mask words
  bf16x8 qf[QT][4];
  unsigned long long mw0[QT], mw1[QT];
  const int W = (p.max_nodes + 63) >> 6;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int qi = qb * ROWS + qt * 16 + c;
    const int qrow = qi < p.max_nodes ? qi : p.max_nodes - 1;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      qf[qt][kk] = __builtin_bit_cast(
          bf16x8, *(const u32x4*)((const unsigned char*)p.q + (node_base + qrow) * 256 + kk * 64 + g * 16));
    mw0[qt] = 0ull;
    mw1[qt] = 0ull;
    if (qi < n) {
      const unsigned long long* mrow = p.anc_mask + ((size_t)b * p.max_nodes + qi) * W;
      mw0[qt] = mrow[0];
      if (W > 1) mw1[qt] = mrow[1];
    }
  }

  const int ctxT = (L + kTileKeys - 1) / kTileKeys, treeT = (n + kTileKeys - 1) / kTileKeys;
  const int NTL = ctxT + treeT;
  const int tstep = kAttnWaves * sp.S;
  const float sl2 = p.scale * 1.4426950408889634f;
  unsigned char* strip = smem + wave * kLdsPerWave;

  f32x4 o[QT][8];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) o[qt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

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

  int t = split * kAttnWaves + wave;
  if (t < NTL) {
    issue_k(t);
    issue_v(t);
  }
  for (; t < NTL; t += tstep) {
    const bool tree = t >= ctxT;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys;
    // K tile -> private strip (row = key, 272-byte pitch), then the next tile's K loads
#pragma unroll
    for (int j = 0; j < 8; ++j) *(u32x4*)(strip + (4 * j + g) * kStripRow + c * 16) = kr[j];
    const int tn = t + tstep;
    if (tn < NTL) issue_k(tn);
    // S^T = K.Q^T for the two blocks of 16 keys, all query tiles
    f32x4 s[QT][2];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      s[qt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
      s[qt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 a =
            __builtin_bit_cast(bf16x8, *(const u32x4*)(strip + (kb * 16 + c) * kStripRow + kk * 64 + g * 16));
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          s[qt][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[qt][kk], s[qt][kb], 0, 0, 0);
      }
    // visibility, scaling, online softmax per query tile
    bf16x8 ph[QT], pl[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float sv[8];
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = row0 + kb * 16 + 4 * g + i;
          bool vis;
          if (tree) vis = (((key < 64 ? mw0[qt] : mw1[qt]) >> (key & 63)) & 1ull) != 0ull;
          else vis = key < L;
          const float x = vis ? s[qt][kb][i] * sl2 : -INFINITY;
          sv[kb * 4 + i] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[qt], mx);
      const float m_safe = m_new > -INFINITY ? m_new : 0.f;
      float psum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float pj = __builtin_amdgcn_exp2f(sv[j] - m_safe);
        psum += pj;
        const __bf16 hi = (__bf16)pj;
        ph[qt][j] = hi;
        pl[qt][j] = (__bf16)(pj - (float)hi);
      }
      if (m_new != m_run[qt]) {  // rescaling is needed only when the running max moved
        const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_safe);
        l_run[qt] *= alpha;
#pragma unroll
        for (int db = 0; db < 8; ++db) o[qt][db] *= alpha;
        m_run[qt] = m_new;
      }
      l_run[qt] += psum;
    }
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
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        o[qt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ph[qt], o[qt][db], 0, 0, 0);
        o[qt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pl[qt], o[qt][db], 0, 0, 0);
      }
    }
    if (tn < NTL) issue_v(tn);
  }

  // ---- merge the wavefronts' partial results --------------------------------------------------
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    l_run[qt] += __shfl_xor(l_run[qt], 16, 64);
    l_run[qt] += __shfl_xor(l_run[qt], 32, 64);
    if (g == 0) {
      m_sh[wave][qt * 16 + c] = m_run[qt];
      l_sh[wave][qt * 16 + c] = l_run[qt];
    }
  }
  __syncthreads();  // also: every wavefront is done with its strip, which the merge buffer reuses
  float* ob = (float*)(smem + wave * kLdsPerWave);
#pragma unroll
  for (int qt = 0; qt < QT; ++qt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // lane (c, g) holds O[q = 16*qt + c][dh = 32g + 8i + db], db = 0..7
      f32x4 lo4 = {o[qt][0][i], o[qt][1][i], o[qt][2][i], o[qt][3][i]};
      f32x4 hi4 = {o[qt][4][i], o[qt][5][i], o[qt][6][i], o[qt][7][i]};
      *(f32x4*)(ob + (qt * 16 + c) * kMergeRow + 32 * g + 8 * i) = lo4;
      *(f32x4*)(ob + (qt * 16 + c) * kMergeRow + 32 * g + 8 * i + 4) = hi4;
    }
  __syncthreads();
  constexpr int kRowsPerWave = ROWS / kAttnWaves;
  const size_t unit = (((size_t)b * p.H + h) * sp.QB + qb) * sp.S + split;
#pragma unroll
  for (int rr = 0; rr < kRowsPerWave; ++rr) {
    const int qr = wave * kRowsPerWave + rr;
    const int qg = qb * ROWS + qr;
    if (qg >= n) continue;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, m_sh[w][qr]);
    float Lt = 0.f, a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      const float mw = m_sh[w][qr];
      const float f = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - M) : 0.f;
      const float* src = (const float*)(smem + w * kLdsPerWave) + qr * kMergeRow;
      Lt += f * l_sh[w][qr];
      a0 += f * src[lane];
      a1 += f * src[lane + 64];
    }
    if (sp.S == 1) {
      const float inv = 1.0f / Lt;
      float* dst = p.out + (node_base + qg) * 128;
      dst[lane] = a0 * inv;
      dst[lane + 64] = a1 * inv;
    } else {
      float* dst = sp.po + (unit * ROWS + qr) * 128;
      dst[lane] = a0;
      dst[lane + 64] = a1;
      if (lane == 0) {
        sp.pm[unit * ROWS + qr] = M;
        sp.pl[unit * ROWS + qr] = Lt;
      }
    }
  }
}

// Combine the S key-split partials of every live query row: one wavefront per row.
__global__ __launch_bounds__(64) void tree_attn_merge_kernel(AttnParams p, AttnSplit sp, int rows_per_block) {
  const int lane = threadIdx.x;
  const int row = blockIdx.x % p.max_nodes;
  const int bh = blockIdx.x / p.max_nodes;
  const int b = bh / p.H;
  int n = p.n_nodes[b];
  n = n < 1 ? 1 : (n > p.max_nodes ? p.max_nodes : n);
  if (row >= n) return;
  const int qb = row / rows_per_block, qr = row % rows_per_block;
  const size_t unit0 = ((size_t)bh * sp.QB + qb) * sp.S;
  float M = -INFINITY;
  for (int s = 0; s < sp.S; ++s) M = fmaxf(M, sp.pm[(unit0 + s) * rows_per_block + qr]);
  float Lt = 0.f, a0 = 0.f, a1 = 0.f;
  for (int s = 0; s < sp.S; ++s) {
    const size_t r = (unit0 + s) * rows_per_block + qr;
    const float ms = sp.pm[r];
    const float f = ms > -INFINITY ? __builtin_amdgcn_exp2f(ms - M) : 0.f;
    Lt += f * sp.pl[r];
    a0 += f * sp.po[r * 128 + lane];
    a1 += f * sp.po[r * 128 + lane + 64];
  }
  const float inv = 1.0f / Lt;
  float* dst = p.out + ((size_t)bh * p.max_nodes + row) * 128;
  dst[lane] = a0 * inv;
  dst[lane + 64] = a1 * inv;
}

template <int QT>
static hipError_t launch_attn_bf16(const AttnParams& p, const AttnSplit& sp, hipStream_t stream) {
  auto kern = tree_attn_bf16_kernel<QT>;
  const int lds = kAttnWaves * attn_lds_per_wave<QT>();
  static bool lds_allowed = false;
  if (!lds_allowed) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    lds_allowed = true;
  }
  const long long blocks = (long long)sp.QB * sp.S * p.H * p.B;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * kAttnWaves), lds, stream, p, sp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.S == 1) return e;
  hipLaunchKernelGGL(tree_attn_merge_kernel, dim3((unsigned)((long long)p.B * p.H * p.max_nodes)), dim3(64), 0,
                     stream, p, sp, 16 * QT);
  return hipGetLastError();
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
    // Launch shape: QT query tiles of 16 rows per wavefront (K/V are re-read once per block of 16*QT
    // rows) and S key splits (each leaves a partial result).  Few (sequence, head) pairs: big query
    // blocks and more splits keep all compute units busy; many pairs: no split at all.
    const long long bh = (long long)B * H;
    int qt = 1;
    if (const char* e = getenv("CTCSPEC_ATTN_QT")) qt = atoi(e) == 1 ? 1 : (atoi(e) == 2 ? 2 : 4);
    AttnSplit sp;
    sp.QB = (max_nodes + 16 * qt - 1) / (16 * qt);
    const int key_tiles = (kv_cap + max_nodes + kTileKeys - 1) / kTileKeys;
    int S = 1;
    while (S < kMaxKvSplits && bh * sp.QB * S < 512 && key_tiles / (2 * S * kAttnWaves) >= 2) S *= 2;
    if (const char* e = getenv("CTCSPEC_ATTN_SPLITS")) S = atoi(e) < 1 ? 1 : (atoi(e) > kMaxKvSplits ? kMaxKvSplits : atoi(e));
    while (S > 1 && bh * S > ctx->attn_units) S /= 2;
    sp.S = S;
    sp.po = ctx->attn_po; sp.pm = ctx->attn_pm; sp.pl = ctx->attn_pl;
    CTCSPEC_REQUIRE(ctx, bh * sp.QB * S <= 0x7fffffffLL && bh * max_nodes <= 0x7fffffffLL, CTCSPEC_EUNSUPPORTED,
                    "tree_verify_attn: grid too large");
    hipError_t e = qt == 1 ? launch_attn_bf16<1>(p, sp, ctx->stream)
                           : (qt == 2 ? launch_attn_bf16<2>(p, sp, ctx->stream) : launch_attn_bf16<4>(p, sp, ctx->stream));
    CTCSPEC_HIP(ctx, e);
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
