// tree_verify_attn: tree-masked verification attention of the base model, one layer.
//
// Two kernels:
//   * tree_attn_bf16_kernel    - bf16 operands, head dimension 128: MFMA for Q.K^T and P.V, online
//                                softmax, K/V tiles shared by the wavefronts of a workgroup through LDS,
//                                optional key splits combined by tree_attn_merge_kernel
//   * tree_attn_generic_kernel - any dtype / head dimension within the limits: one workgroup per
//                                (node, head, sequence), keys in chunks with an online softmax
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
  // optional second form of the merged output (key splits only): rows [B*max_nodes][H*128], each value as two
  // bf16 numbers (high part in plane 0, low part in plane 1) - what the draft layer's next matrix product takes
  unsigned short* rows;
  long long rows_plane;  // elements per plane
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
// Workgroup = NW wavefronts = one block of 16*QT*CW query nodes of one (sequence, head) and one of S
// splits of the keys.  The wavefronts form CW row groups x KP = NW/CW key parts: wavefront w owns query
// rows [16*QT*rg, 16*QT*(rg+1)) of the block, rg = w % CW, and of every KP consecutive tiles of the
// workgroup the one numbered kp = w / CW (with 64-row blocks two wavefronts per SIMD compute, as with
// 128-row blocks; the two key parts of a row group are joined through LDS at the end).  The keys
// (cached context rows first, then the tree nodes) are cut into tiles of 32; split s takes tiles s,
// s+S, ...  A tile (K and V, 16 KB) is fetched ONCE per workgroup by all threads together (one
// 16-byte load of K and of V per thread and tile, PF iterations ahead in registers), put into one of
// two LDS stages of KP tiles.  With S == 1 the workgroup writes the result; otherwise it
// leaves an unnormalised partial (O, max, sum) per row in the context workspace and
// tree_attn_merge_kernel combines the S partials.
//
// LDS tile layout: 32 rows (keys) of 256 bytes in 16-byte slots.
//   K: slot = chunk ^ (row & 15).  16 lanes reading the same chunk of 16 different rows (the MFMA A
//      operand of K.Q^T: lane = key row, 8 consecutive dh) touch 16 different slots.
//   V: slot = chunk ^ ((row & 7) << 1).  V is read back with ds_read_b64_tr_b16: 16 lanes fetch 8 bytes
//      each from 4 rows x 32 bytes and the instruction hands every lane four CONSECUTIVE KEYS of one dh
//      column - the A operand of O^T += V^T.P - without any shuffling in registers.  With this swizzle
//      the 8 rows x 2 chunks a half wavefront reads lie in 32 different 8-byte bank pairs.
//
// Per tile and wavefront:
//   S^T[key, q] = K.Q^T   : A = K rows from LDS, B = Q^T resident in VGPRs; every K fragment is used
//                           for all QT query tiles
//   P = exp2((S^T - m)*c) : in the MFMA C layout a lane holds 8 keys of ONE query column, so the
//                           running max/sum are per lane plus an exchange between the 4 row groups (ds_bpermute)
//   O^T[dh, q] += V^T.P   : P stays in registers as the B operand, as hi + lo bf16 halves so that it
//                           carries 16 mantissa bits; MFMA row r of output block db is dh = 16*db + r
constexpr int kTileKeys = 32;
constexpr int kTileBytes = kTileKeys * 256;        // K or V of one tile
constexpr int kStageBytes = 2 * kTileBytes;        // K then V
// dynamic LDS of the kernel: two stages of KP tiles
constexpr int attn_lds_bytes(int kp) { return 2 * kp * kStageBytes; }

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// (Plain fmaxf on purpose.  As an inline-asm v_max3_f32 this read accumulators of the MFMAs issued right before it,
// and the compiler counts no wait states for inline asm: with the scores consumed straight out of the last product
// the maximum was taken over values that had not landed yet.)
__device__ __forceinline__ float max3_f32(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
// max / sum over the four lanes l, l^16, l^32, l^48 (the lanes that hold the same query column).
// (v_permlane16_swap / v_permlane32_swap would do this inside the vector ALU, and did in an earlier
// version - with results that changed from run to run in the last bits: the value read right after a
// swap was not always the swapped one.  The exchange goes through ds_bpermute instead.)
__device__ __forceinline__ float max_across_row_groups(float x) {
  x = fmaxf(x, __shfl_xor(x, 16, 64));
  return fmaxf(x, __shfl_xor(x, 32, 64));
}
__device__ __forceinline__ float sum_across_row_groups(float x) {
  x += __shfl_xor(x, 16, 64);
  return x + __shfl_xor(x, 32, 64);
}

struct AttnSplit {
  int QB;      // query blocks of 16*QT*CW rows
  int S;       // key splits
  float* po;   // [unit][rows][128] partial O (unnormalised), unit = ((b*H + h)*QB + qb)*S + s
  float* pm;   // [unit][rows] softmax reference, scaled to the log2 domain
  float* pl;   // [unit][rows] running sum
};

template <int QT, int NW, int CW, int PF>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void tree_attn_bf16_kernel(AttnParams p, AttnSplit sp) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int ROWS = 16 * QT * CW;
  constexpr int KP = NW / CW;  // key parts: tiles taken per iteration
  static_assert(NW == 8 && NW % CW == 0 && (KP == 1 || (KP == 2 && QT == 1)), "512 threads fetch a tile; the join of two key parts is written for one query tile");
  constexpr int kIterBytes = KP * kStageBytes;  // one LDS stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = wave % CW, kp = wave / CW;
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
  const int niter = (nloc + KP - 1) / KP;                              // iterations of KP tiles

  // ---- tile loader: thread -> (row, chunk) of K and of V in each of the iteration's KP tiles ----------
  u32x4 ld[PF][2 * KP];
  const int lrow = tid >> 4, lchunk = tid & 15;
  auto issue = [&](int j, auto set_tag) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value;
#pragma unroll
    for (int u = 0; u < KP; ++u) {
      // past the last tile the loads are still issued (on the last tile again, an L2 hit): every wait on
      // an earlier tile can then count on exactly PF-1 younger iterations in flight
      const int jl = KP * j + u;
      const int t = split + (jl < nloc ? jl : nloc - 1) * sp.S;
      const bool tree = t >= ctxT;
      const unsigned char* ks = tree ? kt : kc;
      const unsigned char* vs = tree ? vt : vc;
      const int row0 = (tree ? t - ctxT : t) * kTileKeys, limit = tree ? n : L;
      // tile start as a wavefront-uniform address (scalar arithmetic), the thread's place in the tile as a
      // 32-bit offset: two vector instructions per tile instead of 64-bit address arithmetic per thread
      const unsigned char* kt0 = ks + (size_t)row0 * 256;
      const unsigned char* vt0 = vs + (size_t)row0 * 256;
      const int last = limit - 1 - row0;  // >= 0: rows past the end re-read the last valid row (masked later)
      const unsigned int off = (unsigned int)((lrow < last ? lrow : last) * 256 + lchunk * 16);
      ld[SET][u] = *(const u32x4*)(kt0 + off);
      ld[SET][KP + u] = *(const u32x4*)(vt0 + off);
    }
  };
  const int coff_k = lrow * 256 + ((lchunk ^ (lrow & 15)) << 4);
  const int coff_v = kTileBytes + lrow * 256 + ((lchunk ^ ((lrow & 7) << 1)) << 4);
  auto commit = [&](auto set_tag, int stage) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value;
    unsigned char* base = smem + stage * kIterBytes;
#pragma unroll
    for (int u = 0; u < KP; ++u) {
      *(u32x4*)(base + u * kStageBytes + coff_k) = ld[SET][u];
      *(u32x4*)(base + u * kStageBytes + coff_v) = ld[SET][KP + u];
    }
  };

  // ---- LDS read addresses --------------------------------------------------------------------------
  // K fragment (kb, kk): row kb*16 + c, chunk kk*4 + g; (row & 15) == c
  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = c * 256 + (((kk * 4 + g) ^ c) << 4);
  // The read addresses are kept as complete LDS addresses that the compiler cannot take apart again: as
  // "start of the dynamic LDS block + offset" it recomputes all twelve inside the loop instead of keeping them
  // in registers.
  typedef __attribute__((address_space(3))) unsigned char lds_byte;
  const unsigned int lds0 = (unsigned int)(size_t)(lds_byte*)smem;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    koff[kk] += lds0 + kp * kStageBytes;  // this wavefront's tile of the stage
    asm volatile("" : "+v"(koff[kk]));
  }
  // V, transposing read: lane 16g + s fetches 8 bytes of row kb*16 + 4g + (s >> 2), dh 16db + 4(s & 3)..+3;
  // the 16 lanes of a row group then hold dh 16db + s, keys kb*16 + 4g .. + 3
  int toff[8];
  {
    const int s4 = c >> 2;
    const int x7 = ((4 * (g & 1) + s4) << 1) << 4;  // swizzle term of that row, in bytes
    const int rbase = kTileBytes + (4 * g + s4) * 256 + ((c & 2) ? 16 : 0) + ((c & 1) ? 8 : 0);
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      toff[db] = lds0 + kp * kStageBytes + rbase + ((db << 5) ^ x7);
      asm volatile("" : "+v"(toff[db]));
    }
  }

  // ---- this wavefront's query columns: Q fragments (B operand of K.Q^T) and mask words -------------
  const int qbase = qb * ROWS + rg * 16 * QT;
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

  f32x4 o[QT][8];              // lane (c, g): O[q = c][dh = 16db + 4g + i]
  float m_run[QT], l_run[QT];  // m_run: softmax reference in raw (unscaled) score units
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) o[qt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  auto compute = [&](int jl, auto stage_tag) __attribute__((always_inline)) {
    const int t = split + jl * sp.S;
    const bool tree = t >= ctxT;
    const int row0 = (tree ? t - ctxT : t) * kTileKeys;
    const bool full = !tree && row0 + kTileKeys <= L;  // every key of the tile is visible to every row
    constexpr int sbase = decltype(stage_tag)::value * kIterBytes;  // folds into the instructions' offset fields
    // S^T = K.Q^T for the two blocks of 16 keys, all query tiles
    f32x4 s[QT][2];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      s[qt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
      s[qt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = __builtin_bit_cast(
            bf16x8, *(const __attribute__((address_space(3))) u32x4*)(unsigned int)(koff[kk] + (sbase + kb * 4096)));
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          s[qt][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[qt][kk], s[qt][kb], 0, 0, 0);
      }
    // V^T fragments of the tile, one per output block of 16 dh
    s16x8 va[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(unsigned int)(toff[db] + sbase));
      const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(unsigned int)(toff[db] + (sbase + 4096)));
      va[db] = s16x8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
    }
    // online softmax per query tile
    bf16x8 ph[QT], pl[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float sv[8];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[kb * 4 + i] = s[qt][kb][i];
      if (!full) {
        // this lane's 8 keys are bits 4g..4g+3 and 16+4g..16+4g+3 of the tile's 32-bit visibility word
        const int left = (tree ? n : L) - row0;  // >= 1 keys of the tile exist
        unsigned int vis = left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
        if (tree) {
          const unsigned long long w = row0 < 64 ? mw0[qt] : mw1[qt];
          vis &= (unsigned int)(w >> (row0 & 63));
        }
        vis >>= 4 * g;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i) sv[kb * 4 + i] = ((vis >> (kb * 16 + i)) & 1u) ? sv[kb * 4 + i] : -INFINITY;
      }
      const float mx8 = max3_f32(max3_f32(sv[0], sv[1], sv[2]), max3_f32(sv[3], sv[4], sv[5]), fmaxf(sv[6], sv[7]));
      // The softmax reference m_run only has to be NEAR the running max: it is moved (and O, l
      // rescaled) when the tile's max exceeds it by more than 2^8 in the exponent domain, so P stays
      // below 256 and the rescaling of the accumulators - by far the most expensive part of the
      // step - happens about once per wavefront instead of once per tile.  A column's maximum is
      // spread over four lanes, but it exceeds the reference only if one of those lanes' own maxima
      // does: a vote over the wavefront decides whether anything moves, and the exchange between the
      // row groups (two LDS round trips in the middle of the tile's dependency chain) is only made then.
      if (__builtin_amdgcn_ballot_w64((mx8 - m_run[qt]) * sl2 > 8.0f) != 0ull) {
        const float mx = max_across_row_groups(mx8);
        if ((mx - m_run[qt]) * sl2 > 8.0f) {
          const float alpha = __builtin_amdgcn_exp2f((m_run[qt] - mx) * sl2);  // 0 on first use
          l_run[qt] *= alpha;
#pragma unroll
          for (int db = 0; db < 8; ++db) o[qt][db] *= alpha;
          m_run[qt] = mx;
        }
      }
      const float ms = (m_run[qt] > -INFINITY ? m_run[qt] : 0.f) * sl2;
      float psum = 0.f;
      u32x4 hi4, lo4;
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) {
        // P = hi + lo: hi is P cut to its upper 16 bits (a bf16 by construction), lo the rounded rest
        const float p0 = __builtin_amdgcn_exp2f(fmaf(sv[2 * jp], sl2, -ms));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(sv[2 * jp + 1], sl2, -ms));
        psum += p0 + p1;
        const unsigned int u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
        hi4[jp] = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
        const float r0 = p0 - __uint_as_float(u0 & 0xffff0000u);
        const float r1 = p1 - __uint_as_float(u1 & 0xffff0000u);
        const bf16x2 lo = bf16x2{(__bf16)r0, (__bf16)r1};
        lo4[jp] = __builtin_bit_cast(unsigned int, lo);
      }
      ph[qt] = __builtin_bit_cast(bf16x8, hi4);
      pl[qt] = __builtin_bit_cast(bf16x8, lo4);
      l_run[qt] += psum;
    }
    // O^T += V^T.P: the hi products of all dh blocks first, then the lo products, so that consecutive
    // MFMAs never wait for each other's accumulator
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
        o[qt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va[db]), ph[qt], o[qt][db], 0, 0, 0);
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
        o[qt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va[db]), pl[qt], o[qt][db], 0, 0, 0);
  };

  // ---- pipeline: loads PF iterations (of KP tiles) ahead in registers, LDS write one iteration ahead ----
  auto for_each_set = [&](auto&& fn) __attribute__((always_inline)) {
    [&]<int... I>(std::integer_sequence<int, I...>) { (fn(std::integral_constant<int, I>{}), ...); }
    (std::make_integer_sequence<int, PF>{});
  };
  if (nloc > 0) {
    for_each_set([&](auto jj_tag) __attribute__((always_inline)) { issue(decltype(jj_tag)::value, jj_tag); });
    commit(std::integral_constant<int, 0>{}, 0);
    lds_barrier();
    // loads, LDS writes and barriers are free of conditions inside an iteration (tile indices clamped), which is
    // what lets the waits be exact; the unrolled body is left after any of its PF steps
    bool more = true;
    for (int j0 = 0; more; j0 += PF) {
      for_each_set([&](auto jj_tag) __attribute__((always_inline)) {
        constexpr int JJ = decltype(jj_tag)::value;
        const int j = j0 + JJ;
        if (!more) return;
        commit(std::integral_constant<int, (JJ + 1) % PF>{}, (JJ + 1) & 1);
        issue(j + PF, jj_tag);
        if (live_wave && KP * j + kp < nloc) compute(KP * j + kp, std::integral_constant<int, (JJ & 1)>{});
        lds_barrier();  // not __syncthreads(): the prefetched tiles must stay in flight
        more = j + 1 < niter;
      });
    }
  }
  // ---- the two key parts of a row group joined: the upper wavefront hands (O, reference, sum) over in LDS ----
  if constexpr (KP == 2) {
    __syncthreads();  // every tile consumed: the stages are free
    f32x4* xo = (f32x4*)smem;                       // [8 dh blocks][CW * 64 lanes]
    float* xm = (float*)(smem + 8 * CW * 64 * 16);  // [CW * 64] reference, then [CW * 64] sum
    static_assert(8 * CW * 64 * 16 + 2 * CW * 64 * 4 <= attn_lds_bytes(KP), "the hand-over fits the stages");
    const int at = rg * 64 + lane;
    if (kp == 1 && live_wave) {
#pragma unroll
      for (int db = 0; db < 8; ++db) xo[db * (CW * 64) + at] = o[0][db];
      xm[at] = m_run[0];
      xm[CW * 64 + at] = l_run[0];
    }
    __syncthreads();
    if (kp == 1) return;
    if (live_wave) {
      const float m1 = xm[at], l1 = xm[CW * 64 + at];
      const float M = fmaxf(m_run[0], m1);
      // a part that saw no visible key has reference -inf and contributes nothing
      const float a0 = m_run[0] > -INFINITY ? __builtin_amdgcn_exp2f((m_run[0] - M) * sl2) : 0.f;
      const float a1 = m1 > -INFINITY ? __builtin_amdgcn_exp2f((m1 - M) * sl2) : 0.f;
#pragma unroll
      for (int db = 0; db < 8; ++db) o[0][db] = o[0][db] * a0 + xo[db * (CW * 64) + at] * a1;
      l_run[0] = l_run[0] * a0 + l1 * a1;
      m_run[0] = M;
    }
  }
  if (!live_wave) return;

  // ---- results ------------------------------------------------------------------------------------
  const size_t unit = (((size_t)b * p.H + h) * sp.QB + qb) * sp.S + split;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float l = sum_across_row_groups(l_run[qt]);
    const int qr = rg * 16 * QT + qt * 16 + c;  // row inside the block
    const int qg = qb * ROWS + qr;
    if (qg >= n) continue;
    if (sp.S == 1) {
      const float inv = 1.0f / l;
      float* dst = p.out + (node_base + qg) * 128 + 4 * g;
#pragma unroll
      for (int db = 0; db < 8; ++db) *(f32x4*)(dst + 16 * db) = o[qt][db] * inv;
    } else {
      // nontemporal: the partials are read once, by another kernel; written through, they do not wait in L2 for
      // the write-back at the kernel's end (0.6 us per launch)
      float* dst = sp.po + (unit * ROWS + qr) * 128 + 4 * g;
#pragma unroll
      for (int db = 0; db < 8; ++db) __builtin_nontemporal_store(o[qt][db], (f32x4*)(dst + 16 * db));
      if (g == 0) {
        sp.pm[unit * ROWS + qr] = m_run[qt] * sl2;  // -inf stays -inf (scale > 0)
        sp.pl[unit * ROWS + qr] = l;
      }
    }
  }
}

// Combine the S key-split partials of every live query row.  Thread -> (row, 4 consecutive dh), 32
// threads per row, 8 rows per workgroup; all of a thread's partials are requested before any is used,
// so the kernel costs about one memory round trip.  (Letting the split that finishes last do the
// merge inside the attention kernel was measured: one workgroup per query block then pulls all S
// partials through a single compute unit, which takes longer than this second launch.)
constexpr int kMergeThreads = 256;
__global__ __launch_bounds__(kMergeThreads) void tree_attn_merge_kernel(AttnParams p, AttnSplit sp, int rows_shift) {
  const int rows_per_block = 1 << rows_shift;  // 64 or 128 query rows per block
  // grid: (blocks of 8 rows, head of a sequence) - the indices come from the block numbers, not from divisions
  const int tid = threadIdx.x;
  const int row = blockIdx.x * (kMergeThreads / 32) + (tid >> 5);
  const long long bh = blockIdx.y;  // b * H + h
  if (row >= p.max_nodes) return;
  const int b = (int)blockIdx.y / p.H;
  int n = p.n_nodes[b];
  n = n < 1 ? 1 : (n > p.max_nodes ? p.max_nodes : n);
  if (row >= n) return;
  const int qb = row >> rows_shift, qr = row & (rows_per_block - 1);
  const size_t unit0 = ((size_t)bh * sp.QB + qb) * sp.S;
  const int d4 = (tid & 31) * 4;
  float pmv[kMaxKvSplits], plv[kMaxKvSplits];
  f32x4 pov[kMaxKvSplits];
#pragma unroll
  for (int s = 0; s < kMaxKvSplits; ++s) {
    const bool on = s < sp.S;
    const size_t r = (unit0 + (on ? s : 0)) * rows_per_block + qr;
    pmv[s] = on ? sp.pm[r] : -INFINITY;
    plv[s] = sp.pl[r];
    pov[s] = *(const f32x4*)(sp.po + r * 128 + d4);
  }
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < kMaxKvSplits; ++s) M = fmaxf(M, pmv[s]);
  float Lt = 0.f;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kMaxKvSplits; ++s) {
    const float f = pmv[s] > -INFINITY ? __builtin_amdgcn_exp2f(pmv[s] - M) : 0.f;
    Lt += f * plv[s];
    acc += pov[s] * f;
  }
  const f32x4 o = acc * (1.0f / Lt);
  if (p.rows) {
    const int h = (int)(bh - (long long)b * p.H);
    const size_t at = ((size_t)b * p.max_nodes + row) * ((size_t)p.H * 128) + (size_t)h * 128 + d4;
    unsigned short hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned int u = __float_as_uint(o[i]);
      hi[i] = (u & 0x7fffffffu) > 0x7f800000u ? 0x7fc0 : (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
      const unsigned int v = __float_as_uint(o[i] - __uint_as_float((unsigned int)hi[i] << 16));
      lo[i] = (v & 0x7fffffffu) > 0x7f800000u ? 0x7fc0 : (unsigned short)((v + 0x7fffu + ((v >> 16) & 1u)) >> 16);
    }
    *(u32x2*)(p.rows + at) = u32x2{(unsigned)hi[0] | ((unsigned)hi[1] << 16), (unsigned)hi[2] | ((unsigned)hi[3] << 16)};
    *(u32x2*)(p.rows + p.rows_plane + at) = u32x2{(unsigned)lo[0] | ((unsigned)lo[1] << 16), (unsigned)lo[2] | ((unsigned)lo[3] << 16)};
  } else {
    *(f32x4*)(p.out + ((size_t)bh * p.max_nodes + row) * 128 + d4) = o;
  }
}

template <int QT, int NW, int CW, int PF>
static hipError_t launch_attn_bf16(const AttnParams& p, const AttnSplit& sp, hipStream_t stream) {
  auto kern = tree_attn_bf16_kernel<QT, NW, CW, PF>;
  const long long blocks = (long long)sp.QB * sp.S * p.H * p.B;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * NW), attn_lds_bytes(NW / CW), stream, p, sp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.S == 1) return e;
  const unsigned mblocks = (unsigned)((p.max_nodes + kMergeThreads / 32 - 1) / (kMergeThreads / 32));
  constexpr int kRows = 16 * QT * CW;
  static_assert(kRows == 64 || kRows == 128, "the merge kernel takes the block size as a shift");
  hipLaunchKernelGGL(tree_attn_merge_kernel, dim3(mblocks, (unsigned)(p.B * p.H)), dim3(kMergeThreads), 0, stream, p, sp,
                     kRows == 64 ? 6 : 7);
  return hipGetLastError();
}

// code of this translation unit loaded onto the current device (context creation calls this: a stage call never
// triggers a load, so it can be the first thing a stream capture records)
hipError_t prepare_tree_attn() {
  hipFuncAttributes attr;
  hipError_t e = hipFuncGetAttributes(&attr, (const void*)tree_attn_merge_kernel);
  if (e != hipSuccess) return e;
  // the 64-row kernel's two stages of two tiles are 64 KB of dynamic LDS
  return hipFuncSetAttribute((const void*)tree_attn_bf16_kernel<1, 8, 4, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             attn_lds_bytes(2));
}

}  // namespace ctcspec

using namespace ctcspec;

int ctcspec::tree_verify_attn_rows(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* q, const void* k_cache,
                                   const void* v_cache, const int64_t* kv_off, const int32_t* ctx_len, int kv_cap,
                                   const void* k_tree, const void* v_tree, const int32_t* n_nodes,
                                   const uint64_t* anc_mask, int B, int H, int dh, int max_nodes, float scale,
                                   float* out, unsigned short* rows, long long rows_plane, int* rows_written) {
  if (rows_written) *rows_written = 0;
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
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
  p.rows = nullptr; p.rows_plane = 0;
  if (dt == CTCSPEC_BF16 && dh == 128) {
    CTCSPEC_REQUIRE(ctx, scale > 0.f, CTCSPEC_EINVAL, "tree_verify_attn: scale must be positive");
    // Launch shape.  A workgroup has 8 wavefronts that all fetch tiles and all compute: 8 row groups of 16
    // query rows (blocks of 128 rows per (sequence, head)), or 4 row groups x 2 key parts (blocks of 64
    // rows); S key splits, so that about 256 workgroups exist and each still has a few tiles of 32 keys
    // to stream.  Two 64-row blocks per head halve the partial results (fewer splits) at the price of a
    // second pass over K/V through L2; they are taken when they fill more compute units, or as many with
    // at least 4 splits (kernel and merge together then take the same time as one 128-row block with
    // twice the splits, with 20 MB less traffic at the 7B shape).  Trees of 17 to 64 nodes are one
    // 64-row block.
    const long long bh = (long long)B * H;
    const int key_tiles = (kv_cap + max_nodes + kTileKeys - 1) / kTileKeys;
    auto splits_for = [&](long long qblocks) {
      long long S = 256 / (bh * qblocks);
      if (S > key_tiles / 4) S = key_tiles / 4;
      if (S > kMaxKvSplits) S = kMaxKvSplits;
      while (S > 1 && bh * qblocks * S > (long long)ctx->attn_units) --S;  // partial slots of the workspace
      return S < 1 ? 1LL : S;
    };
    const long long s128 = splits_for(1), s64 = splits_for(2);
    const bool two_blocks = max_nodes > 64 && (2 * s64 > s128 || (2 * s64 == s128 && s64 >= 4));
    // (up to 16 rows, a single row group: the one-tile-per-iteration kernel, whose first tile is in LDS sooner -
    // 9.1 against 9.9 us for the draft layer's 8 rows)
    const bool rows64 = two_blocks || (max_nodes <= 64 && max_nodes > 16);
    AttnSplit sp;
    sp.QB = two_blocks ? 2 : 1;
    sp.S = (int)(two_blocks ? s64 : s128);
    sp.po = ctx->attn_po; sp.pm = ctx->attn_pm; sp.pl = ctx->attn_pl;
    CTCSPEC_REQUIRE(ctx, bh * sp.QB * sp.S <= 0x7fffffffLL && bh * max_nodes <= 0x7fffffffLL && bh <= 65535,
                    CTCSPEC_EUNSUPPORTED,
                    "tree_verify_attn: grid too large");
    if (rows && sp.S > 1) {  // the merge kernel writes the rows instead of `out`
      p.rows = rows; p.rows_plane = rows_plane;
      if (rows_written) *rows_written = 1;
    }
    const hipError_t e = rows64 ? launch_attn_bf16<1, 8, 4, 2>(p, sp, ctx->stream)
                                : launch_attn_bf16<1, 8, 8, 2>(p, sp, ctx->stream);
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

extern "C" int tree_verify_attn(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* q, const void* k_cache,
                                const void* v_cache, const int64_t* kv_off, const int32_t* ctx_len, int kv_cap,
                                const void* k_tree, const void* v_tree, const int32_t* n_nodes,
                                const uint64_t* anc_mask, int B, int H, int dh, int max_nodes, float scale,
                                float* out) {
  return ctcspec::tree_verify_attn_rows(ctx, dt, q, k_cache, v_cache, kv_off, ctx_len, kv_cap, k_tree, v_tree, n_nodes,
                                        anc_mask, B, H, dh, max_nodes, scale, out, nullptr, 0, nullptr);
}
