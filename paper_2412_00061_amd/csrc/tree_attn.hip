// tree_verify_attn: tree-masked verification attention of the base model, one layer.
//
// Two kernels:
//   * tree_attn_bf16_kernel    - bf16 operands, head dimension 128: MFMA for Q.K^T and P.V, online
//                                softmax, every wavefront streams its own share of the keys
//   * tree_attn_generic_kernel - any dtype / head dimension within the limits: one workgroup per
//                                (node, head, sequence), keys in chunks with an online softmax
#include <stdlib.h>

#include <type_traits>
#include <utility>

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
// Workgroup = NW wavefronts = one block of 16*QT*NW query nodes of one (sequence, head) and one of S
// splits of the keys; wavefront w owns query rows [16*QT*w, 16*QT*(w+1)) of the block.  The keys
// (cached context rows first, then the tree nodes) are cut into tiles of 32; split s takes tiles s,
// s+S, ...  A tile (K and V, 16 KB) is fetched ONCE per workgroup by all threads together (one or two
// 16-byte loads of K and of V per thread, PF tiles ahead in registers), put into one of two LDS
// stages and used by every wavefront.  With S == 1 the workgroup writes the result; otherwise it
// leaves an unnormalised partial (O, max, sum) per row in the context workspace and
// tree_attn_merge_kernel combines the S partials.
//
// LDS tile layout: 32 rows (keys) of 256 bytes, 16-byte slot = chunk ^ (row & 15).  Both access
// patterns - 16 lanes reading the same chunk of 16 different rows (K as MFMA A operand) and 16 lanes
// reading the 16 chunks of one row (V) - then touch 16 different slots: conflict-free without padding.
//
// Per tile and wavefront:
//   S^T[key, q] = K.Q^T   : A = K rows from LDS, B = Q^T resident in VGPRs; every K fragment is used
//                           for all QT query tiles
//   P = exp2((S^T - m)*c) : in the MFMA C layout a lane holds 8 keys of ONE query column, so the
//                           running max/sum are per lane plus a 4-lane exchange
//   O^T[dh, q] += V^T.P   : P stays in registers as the B operand (hi + lo bf16 halves, so that P
//                           carries 16 mantissa bits); a lane reads 16 bytes (8 consecutive dh of one
//                           key) of V per key slot and an 8x8 16-bit transpose inside the lane turns
//                           that into A operands, shared by the QT query tiles.  MFMA row r of output
//                           block db stands for dh = 8*r + db; the permutation is undone when O is
//                           written.
constexpr int kTileKeys = 32;
constexpr int kTileBytes = kTileKeys * 256;        // K or V of one tile
constexpr int kStageBytes = 2 * kTileBytes;        // K then V
constexpr int kAttnLdsBytes = 2 * kStageBytes;     // two stages

struct AttnSplit {
  int QB;      // query blocks of 16*QT*NW rows
  int S;       // key splits
  float* po;   // [unit][rows][128] partial O (unnormalised), unit = ((b*H + h)*QB + qb)*S + s
  float* pm;   // [unit][rows] softmax reference, scaled to the log2 domain
  float* pl;   // [unit][rows] running sum
};

template <int QT, int NW, int PF>
__global__ __launch_bounds__(64 * NW) void tree_attn_bf16_kernel(AttnParams p, AttnSplit sp) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int ROWS = 16 * QT * NW;
  constexpr int kThreadsA = 64 * NW;
  constexpr int LU = 512 / kThreadsA;  // 16-byte pieces of K (and of V) per thread and tile
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

  const int ctxT = (L + kTileKeys - 1) / kTileKeys, treeT = (n + kTileKeys - 1) / kTileKeys;
  const int NTL = ctxT + treeT;
  const int nloc = split < NTL ? (NTL - split + sp.S - 1) / sp.S : 0;  // my tiles: split, split+S, ...

  // ---- tile loader: thread -> (row, chunk) of K and of V, twice ---------------------------------
  u32x4 ld[PF][2 * LU];
  auto issue = [&](int j, auto set_tag) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value;
    // past the last tile the loads are still issued (on the last tile again, an L2 hit): every wait on
    // an earlier tile can then count on exactly PF-1 younger tiles in flight
    const int t = split + (j < nloc ? j : nloc - 1) * sp.S;
    const bool tree = t >= ctxT;
    const unsigned char* ks = tree ? kt : kc;
    const unsigned char* vs = tree ? vt : vc;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys, limit = tree ? n : L;
#pragma unroll
    for (int u = 0; u < LU; ++u) {
      const int q = tid + kThreadsA * u;
      int row = row0 + (q >> 4);
      row = row < limit ? row : limit - 1;  // rows past the end re-read the last valid row (masked later)
      ld[SET][u] = *(const u32x4*)(ks + (size_t)row * 256 + (q & 15) * 16);
      ld[SET][LU + u] = *(const u32x4*)(vs + (size_t)row * 256 + (q & 15) * 16);
    }
  };
  auto commit = [&](auto set_tag, int stage) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value;
    unsigned char* base = smem + stage * kStageBytes;
#pragma unroll
    for (int u = 0; u < LU; ++u) {
      const int q = tid + kThreadsA * u;
      const int row = q >> 4, slot = (q & 15) ^ (row & 15);
      *(u32x4*)(base + row * 256 + slot * 16) = ld[SET][u];
      *(u32x4*)(base + kTileBytes + row * 256 + slot * 16) = ld[SET][LU + u];
    }
  };

  // ---- this wavefront's query columns: Q fragments (B operand of K.Q^T) and mask words -------------
  const int qbase = qb * ROWS + wave * 16 * QT;
  const bool live_wave = qbase < n;
  bf16x8 qf[QT][4];
  unsigned long long mw0[QT], mw1[QT];
  const int W = (p.max_nodes + 63) >> 6;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int qi = qbase + qt * 16 + c;
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
  const float sl2 = p.scale * 1.4426950408889634f;

  f32x4 o[QT][8];
  float m_run[QT], l_run[QT];  // m_run: softmax reference in raw (unscaled) score units
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) o[qt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  auto compute = [&](int j, int stage) __attribute__((always_inline)) {
    const int t = split + j * sp.S;
    const bool tree = t >= ctxT;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys;
    const bool full = !tree && row0 + kTileKeys <= L;  // every key of the tile is visible to every row
    const unsigned char* kbase = smem + stage * kStageBytes;
    const unsigned char* vbase = kbase + kTileBytes;
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
        // row kb*16 + c, chunk kk*4 + g; (row & 15) == c
        const bf16x8 a = __builtin_bit_cast(
            bf16x8, *(const u32x4*)(kbase + (kb * 16 + c) * 256 + (((kk * 4 + g) ^ c) * 16)));
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          s[qt][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[qt][kk], s[qt][kb], 0, 0, 0);
      }
    // V fragments of the tile: key slot (g, j) -> row (j>>2)*16 + 4g + (j&3), chunk c
    u32x4 vr[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int row = (jj >> 2) * 16 + 4 * g + (jj & 3);
      vr[jj] = *(const u32x4*)(vbase + row * 256 + ((c ^ (row & 15)) * 16));
    }
    // online softmax per query tile
    bf16x8 ph[QT], pl[QT];
    auto softmax = [&](auto full_tag) __attribute__((always_inline)) {
      constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        float sv[8];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float x = s[qt][kb][i];
            if (!FULL) {
              const int key = row0 + kb * 16 + 4 * g + i;
              const bool vis_tree = (((key < 64 ? mw0[qt] : mw1[qt]) >> (key & 63)) & 1ull) != 0ull;
              const bool vis = tree ? vis_tree : key < L;
              x = vis ? x : -INFINITY;
            }
            sv[kb * 4 + i] = x;
          }
        float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // The softmax reference m_run only has to be NEAR the running max: it is moved (and O, l
        // rescaled) when the tile's max exceeds it by more than 2^8 in the exponent domain, so P stays
        // below 256 and the rescaling of the accumulators - by far the most expensive part of the
        // step - happens about once per wavefront instead of once per tile.
        if ((mx - m_run[qt]) * sl2 > 8.0f) {
          const float alpha = __builtin_amdgcn_exp2f((m_run[qt] - mx) * sl2);  // 0 on first use
          l_run[qt] *= alpha;
#pragma unroll
          for (int db = 0; db < 8; ++db) o[qt][db] *= alpha;
          m_run[qt] = mx;
        }
        const float ms = (m_run[qt] > -INFINITY ? m_run[qt] : 0.f) * sl2;
        float psum = 0.f;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          const float pj = __builtin_amdgcn_exp2f(fmaf(sv[jj], sl2, -ms));
          psum += pj;
          const __bf16 hi = (__bf16)pj;
          ph[qt][jj] = hi;
          pl[qt][jj] = (__bf16)(pj - (float)hi);
        }
        l_run[qt] += psum;
      }
    };
    if (full) softmax(std::true_type{});
    else softmax(std::false_type{});
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
  };

  // ---- pipeline: loads PF tiles ahead in registers, LDS write one tile ahead -------------------------
  auto for_each_set = [&](auto&& fn) __attribute__((always_inline)) {
    [&]<int... I>(std::integer_sequence<int, I...>) { (fn(std::integral_constant<int, I>{}), ...); }
    (std::make_integer_sequence<int, PF>{});
  };
  if (nloc > 0) {
    for_each_set([&](auto jj_tag) __attribute__((always_inline)) { issue(decltype(jj_tag)::value, jj_tag); });
    commit(std::integral_constant<int, 0>{}, 0);
    lds_barrier();
    // the trip count is rounded up to a multiple of PF; the surplus iterations only move (already
    // cached) data - keeping loads, LDS writes and barriers free of conditions is what lets the
    // waits be exact
    const int nit = (nloc + PF - 1) / PF * PF;
    for (int j0 = 0; j0 < nit; j0 += PF) {
      for_each_set([&](auto jj_tag) __attribute__((always_inline)) {
        constexpr int JJ = decltype(jj_tag)::value;
        const int j = j0 + JJ;
        commit(std::integral_constant<int, (JJ + 1) % PF>{}, (JJ + 1) & 1);
        issue(j + PF, jj_tag);
        if (live_wave && j < nloc) compute(j, JJ & 1);
        lds_barrier();  // not __syncthreads(): the prefetched tiles must stay in flight
      });
    }
  }
  if (!live_wave) return;

  // ---- results ------------------------------------------------------------------------------------
  const size_t unit = (((size_t)b * p.H + h) * sp.QB + qb) * sp.S + split;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    float l = l_run[qt];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const int qr = wave * 16 * QT + qt * 16 + c;  // row inside the block
    const int qg = qb * ROWS + qr;
    if (qg >= n) continue;
    // lane (c, g) holds O[q = c][dh = 32g + 8i + db], db = 0..7
    if (sp.S == 1) {
      const float inv = 1.0f / l;
      float* dst = p.out + (node_base + qg) * 128 + 32 * g;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *(f32x4*)(dst + 8 * i) = f32x4{o[qt][0][i] * inv, o[qt][1][i] * inv, o[qt][2][i] * inv, o[qt][3][i] * inv};
        *(f32x4*)(dst + 8 * i + 4) = f32x4{o[qt][4][i] * inv, o[qt][5][i] * inv, o[qt][6][i] * inv, o[qt][7][i] * inv};
      }
    } else {
      float* dst = sp.po + (unit * ROWS + qr) * 128 + 32 * g;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *(f32x4*)(dst + 8 * i) = f32x4{o[qt][0][i], o[qt][1][i], o[qt][2][i], o[qt][3][i]};
        *(f32x4*)(dst + 8 * i + 4) = f32x4{o[qt][4][i], o[qt][5][i], o[qt][6][i], o[qt][7][i]};
      }
      if (g == 0) {
        sp.pm[unit * ROWS + qr] = m_run[qt] * sl2;  // -inf stays -inf (scale > 0)
        sp.pl[unit * ROWS + qr] = l;
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

template <int QT, int NW, int PF>
static hipError_t launch_attn_bf16(const AttnParams& p, const AttnSplit& sp, hipStream_t stream) {
  auto kern = tree_attn_bf16_kernel<QT, NW, PF>;
  const long long blocks = (long long)sp.QB * sp.S * p.H * p.B;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * NW), kAttnLdsBytes, stream, p, sp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.S == 1) return e;
  hipLaunchKernelGGL(tree_attn_merge_kernel, dim3((unsigned)((long long)p.B * p.H * p.max_nodes)), dim3(64), 0,
                     stream, p, sp, 16 * QT * NW);
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
    CTCSPEC_REQUIRE(ctx, scale > 0.f, CTCSPEC_EINVAL, "tree_verify_attn: scale must be positive");
    // Launch shape: blocks of 64 (max_nodes <= 64) or 128 query rows; S key splits chosen so that
    // about 256 workgroups exist and each still has a few tiles of 32 keys to stream.
    const long long bh = (long long)B * H;
    int rows = max_nodes > 64 ? 128 : 64;  // query rows per workgroup: 8 or 4 wavefronts of 16
    int pf = 4;
    if (const char* e = getenv("CTCSPEC_ATTN_ROWS")) rows = atoi(e) == 64 ? 64 : 128;
    if (const char* e = getenv("CTCSPEC_ATTN_PF")) pf = atoi(e);
    AttnSplit sp;
    sp.QB = (max_nodes + rows - 1) / rows;
    const int key_tiles = (kv_cap + max_nodes + kTileKeys - 1) / kTileKeys;
    long long S = 256 / (bh * sp.QB);
    if (S > key_tiles / 4) S = key_tiles / 4;
    if (S > kMaxKvSplits) S = kMaxKvSplits;
    if (const char* e = getenv("CTCSPEC_ATTN_SPLITS")) S = atoi(e);
    while (S > 1 && bh * sp.QB * S * rows > (long long)ctx->attn_units * ((ctx->lim.max_nodes + 63) / 64 * 64)) --S;
    if (S < 1) S = 1;
    sp.S = (int)S;
    sp.po = ctx->attn_po; sp.pm = ctx->attn_pm; sp.pl = ctx->attn_pl;
    CTCSPEC_REQUIRE(ctx, bh * sp.QB * S <= 0x7fffffffLL && bh * max_nodes <= 0x7fffffffLL, CTCSPEC_EUNSUPPORTED,
                    "tree_verify_attn: grid too large");
    hipError_t e;
    if (rows == 64) e = pf == 2 ? launch_attn_bf16<1, 4, 2>(p, sp, ctx->stream) : (pf == 3 ? launch_attn_bf16<1, 4, 3>(p, sp, ctx->stream) : launch_attn_bf16<1, 4, 4>(p, sp, ctx->stream));
    else e = pf == 2 ? launch_attn_bf16<1, 8, 2>(p, sp, ctx->stream) : (pf == 3 ? launch_attn_bf16<1, 8, 3>(p, sp, ctx->stream) : launch_attn_bf16<1, 8, 4>(p, sp, ctx->stream));
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
