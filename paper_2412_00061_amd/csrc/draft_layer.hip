// draft_layer_forward: the transformer layer of the attention draft module (Sec. 3.1) - the base family's
// decoder layer (RMSNorm, rotary multi-head attention over the layer's own key/value cache, gated SiLU
// feed-forward, residuals) applied to the T draft positions of every sequence in parallel.
//
// At B*T of 8 to 16 columns the layer is four passes over its weight matrices (405 MB at the 7B shape) and
// one attention call; everything else is KB-sized.  The passes run in skinny_gemm_bf16_kernel:
//   * the unit of work is 16 weight rows x 256 hidden elements (8 KB).  The units of a matrix, row tile major,
//     are dealt to the wavefronts of the grid in equal contiguous ranges, so every compute unit streams the
//     same number of bytes whatever the matrix shape (12288, 4096 or 22016 rows; 4096 or 11008 columns);
//   * a wavefront streams its range through registers (STAGES - 1 units ahead) and a private LDS strip into
//     MFMA A fragments, as the draft head does; the activations (B operand) sit in LDS per workgroup.  A range
//     is at most twice as long as a row tile's units, so it touches at most three row tiles: three
//     accumulators, the A fragment zeroed for those that a unit does not belong to - no branch, no flush inside
//     the stream;
//   * matrices whose activation slice does not fit in LDS are split along k into groups of workgroups, each
//     with its slice of the activations;
//   * every wavefront leaves three 16 x 16 partial tiles; the kernel that follows (rotary embedding, residual +
//     norm, gate, residual) adds the partial tiles of a row tile in a fixed order - same bits on every run.
#include <type_traits>
#include <utility>

#include "common.h"

namespace ctcspec {

constexpr int kSgWaves = 8;
constexpr int kSgStages = 4;                    // register stages of the weight stream (prefetch distance + 1)
constexpr int kSgStripPitch = 512 + 32;         // bytes per strip row: 256 bf16 + pad (conflict-free fragment reads)
constexpr int kSgStripBytes = 16 * kSgStripPitch;
constexpr int kSgHsPieces = 12;                 // 16-byte activation pieces a thread carries to LDS
constexpr int kSgMaxGroups = 12;
constexpr int kSgMaxCols = 16;                  // columns per pass; each is two bf16 columns (high and low part)
constexpr int kSgAcc = 3;                       // row tiles a wavefront's range may touch
constexpr int kSgLdsBudget = 160 * 1024 - kSgWaves * kSgStripBytes - 256;  // for the activations

struct SkinnyPlan {
  int N, K, cols, tiles;                        // out features, in features, columns, row tiles of 16
  int nt;                                       // MFMA column tiles: ceil(2 * cols / 16)
  int groups;                                   // k groups
  int chunk_begin[kSgMaxGroups], chunks[kSgMaxGroups];  // in chunks of 256 hidden elements
  int wave_begin[kSgMaxGroups];                 // first wavefront (global index) that works on the group
  int per_wave[kSgMaxGroups];                   // units per wavefront (<= (kSgAcc - 1) * chunks of the group)
  // ceil(2^32 / d) for d = per_wave and d = chunks of the group: n / d = umulhi(n, magic) for the unit numbers that
  // occur (n * d < 2^32) - the kernels that add up the partial tiles divide per element, and a division by a
  // number the compiler does not know costs about forty instructions
  unsigned int magic_per_wave[kSgMaxGroups], magic_chunks[kSgMaxGroups];
  int total_waves;
  int hs_bytes;                                 // LDS bytes of the activation slice
};

struct SkinnyParams {
  const void* w;      // [N][K] bf16
  const void* x;      // [2][plane_cols][K] bf16: high parts, then low parts; this pass starts at column col0
  int plane_cols, col0;
  const void* zeros;  // 256 bytes
  float* part;        // [total_waves][kSgAcc][nt][16 columns][16 rows]
  // first pass of the layer (FIRST): x is the layer's input [plane_cols][K] bf16 as given, the kernel multiplies it
  // by gain [K] bf16 while staging it (the products are exact as two bf16 numbers) and the first workgroup of every
  // k group leaves the sums of x^2 over each 256 elements in ss_out [plane_cols][K / 256]
  const void* gain;
  float* ss_out;
  SkinnyPlan plan;
};

typedef __attribute__((address_space(1))) u32x4 GlobalVec4;  // a pointer made from an integer is generic otherwise

// The activations are fp32 values carried as two bf16 numbers (value = high + low, 16 bits of mantissa): column
// c of the pass is MFMA column c (high parts) and column cols + c (low parts), and the two products are added
// when the partial tiles are.  The weights are bf16 as stored, so the products lose nothing to a rounding of
// the activations.
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f);

template <int STAGES, int NT, bool FIRST>
__global__ __launch_bounds__(64 * kSgWaves) void skinny_gemm_bf16_kernel(SkinnyParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15, g = lane >> 4;
  // the chunks of a row in the lane order that lets the 16 lanes the LDS serves together (l .. l+7, l+16 .. l+23)
  // write 256 consecutive bytes of the strip
  const int lrow = lane >> 5, lch = (lane & 7) | ((lane & 16) >> 1) | ((lane & 8) << 1);
  const SkinnyPlan& pl = p.plan;
  // the k group of this workgroup (selected with compares: no indexed access to the kernel arguments)
  int Cg = pl.chunks[0], P = pl.per_wave[0], wave_begin = 0, chunk_begin = 0;
#pragma unroll
  for (int q = 1; q < kSgMaxGroups; ++q)
    if (q < pl.groups && (int)blockIdx.x * kSgWaves >= pl.wave_begin[q]) {
      Cg = pl.chunks[q]; P = pl.per_wave[q]; wave_begin = pl.wave_begin[q]; chunk_begin = pl.chunk_begin[q];
    }
  const int wave_global = blockIdx.x * kSgWaves + wave;
  const int u0 = (wave_global - wave_begin) * P;
  int n = pl.tiles * Cg - u0;  // units of this wavefront
  n = n > P ? P : (n < 0 ? 0 : n);
  const int tile0 = u0 / Cg, c0 = u0 - tile0 * Cg;
  const int HSS = Cg * 512 + 32;
  const int vcols = 2 * pl.cols;
  unsigned char* hs = smem;
  unsigned char* wst = smem + pl.hs_bytes + wave * kSgStripBytes;

  // ---- activation slice of the group -> LDS (loads unconditional, indices clamped) -----------------------
  // FIRST: a piece of the input and the matching piece of the gain per (column, 16 bytes); both planes of the
  // slice are made from them when the pieces are written to LDS.  Half as many (column, piece) pairs, the same
  // number of loads.
  const int per_row = Cg * 32;  // 16-byte pieces per column
  const int hs_total = (FIRST ? pl.cols : vcols) * per_row;
  constexpr int kLoads = FIRST ? kSgHsPieces / 2 : kSgHsPieces;
  u32x4 hreg[kSgHsPieces];
  int hs_dst[kLoads];
  int ss_dst[kLoads];  // FIRST: where the piece's 32-lane group leaves its sum of squares, -1: nowhere
#pragma unroll
  for (int u = 0; u < kLoads; ++u) {
    const int idx = tid + u * 64 * kSgWaves;
    const int cl = idx < hs_total ? idx : hs_total - 1;
    const int m = cl / per_row, q = cl - m * per_row;
    hs_dst[u] = idx < hs_total ? m * HSS + q * 16 : -1;
    if constexpr (FIRST) {
      hreg[2 * u] = *(const u32x4*)((const unsigned char*)p.x + (size_t)(p.col0 + m) * pl.K * 2 +
                                    (size_t)chunk_begin * 512 + q * 16);
      hreg[2 * u + 1] = *(const u32x4*)((const unsigned char*)p.gain + (size_t)chunk_begin * 512 + q * 16);
      ss_dst[u] = idx < hs_total ? (p.col0 + m) * (pl.K / 256) + chunk_begin + (q >> 5) : -1;
    } else {
      const int plane = m >= pl.cols ? 1 : 0, col = m - plane * pl.cols;
      hreg[u] = *(const u32x4*)((const unsigned char*)p.x +
                                ((size_t)plane * p.plane_cols + p.col0 + col) * pl.K * 2 + (size_t)chunk_begin * 512 + q * 16);
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- weight stream ---------------------------------------------------------------------------------------
  // row pointers of the first row tile of the range (N is a multiple of 16: every tile is whole)
  uintptr_t rowptr[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int r0 = tile0 * 16 + 2 * j + lrow;
    r0 = r0 < pl.N ? r0 : pl.N - 1;  // wavefronts without units
    rowptr[j] = (uintptr_t)p.w + (size_t)chunk_begin * 512 + lch * 16 + (size_t)r0 * pl.K * 2;
  }
  const size_t tile_stride = (size_t)16 * pl.K * 2;
  const uintptr_t zaddr = (uintptr_t)p.zeros + (lch & 15) * 16;
  u32x4 v[STAGES][8];
  // unit i of the range: chunk (c0 + i) % Cg of row tile tile0 + (c0 + i) / Cg.  A request past the range reads
  // zeros (from L2) so that every step issues the same number of loads and adds nothing.
  auto request = [&](int i, auto stage_tag) __attribute__((always_inline)) {
    constexpr int ST = decltype(stage_tag)::value;
    const bool valid = i < n;
    const int cc = c0 + i;
    const int which = (cc >= Cg ? 1 : 0) + (cc >= 2 * Cg ? 1 : 0);
    const size_t off = (size_t)which * tile_stride + (size_t)(cc - which * Cg) * 512;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uintptr_t a = valid ? rowptr[j] + off : zaddr;
      v[ST][j] = __builtin_nontemporal_load((const GlobalVec4*)a);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  int bcol[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int vc = nt * 16 + c;
    bcol[nt] = (vc < vcols ? vc : vcols - 1) * HSS + g * 16;
  }
  f32x4 acc[kSgAcc][NT];
#pragma unroll
  for (int a = 0; a < kSgAcc; ++a)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[a][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto consume = [&](int i, auto stage_tag) __attribute__((always_inline)) {
    constexpr int ST = decltype(stage_tag)::value;
    const bool valid = i < n;
    const int cc = c0 + i;
    const int which = (cc >= Cg ? 1 : 0) + (cc >= 2 * Cg ? 1 : 0);
    const int xoff = valid ? (cc - which * Cg) * 512 : 0;
    unsigned int mask[kSgAcc];
#pragma unroll
    for (int a = 0; a < kSgAcc; ++a) mask[a] = which == a ? ~0u : 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) *(u32x4*)(wst + (2 * j + lrow) * kSgStripPitch + lch * 16) = v[ST][j];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 a = *(const u32x4*)(wst + c * kSgStripPitch + kk * 64 + g * 16);
      bf16x8 b[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[nt] = __builtin_bit_cast(bf16x8, *(const u32x4*)(hs + bcol[nt] + xoff + kk * 64));
#pragma unroll
      for (int t = 0; t < kSgAcc; ++t) {
        const u32x4 am = {a[0] & mask[t], a[1] & mask[t], a[2] & mask[t], a[3] & mask[t]};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, am), b[nt], acc[t][nt], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto for_each_stage = [&](auto&& fn) __attribute__((always_inline)) {
    [&]<int... I>(std::integer_sequence<int, I...>) __attribute__((always_inline)) {
      (fn(std::integral_constant<int, I>{}), ...);
    }(std::make_integer_sequence<int, STAGES>{});
  };

  for_each_stage([&](auto st) __attribute__((always_inline)) {
    if constexpr (decltype(st)::value < STAGES - 1) request(decltype(st)::value, st);
  });
  if constexpr (FIRST) {
    const bool leaves_sums = (int)blockIdx.x * kSgWaves == wave_begin;  // the k group's first workgroup
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const u32x4 xv = hreg[2 * u], gv = hreg[2 * u + 1];
      u32x4 hi, lo;
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // two bf16 numbers per word: the low half is the earlier element
        const float x0 = __uint_as_float(xv[e] << 16), x1 = __uint_as_float(xv[e] & 0xffff0000u);
        const float v0 = x0 * __uint_as_float(gv[e] << 16), v1 = x1 * __uint_as_float(gv[e] & 0xffff0000u);
        const unsigned int h0 = float_to_bf16_bits(v0), h1 = float_to_bf16_bits(v1);
        const unsigned int l0 = float_to_bf16_bits(v0 - __uint_as_float(h0 << 16));
        const unsigned int l1 = float_to_bf16_bits(v1 - __uint_as_float(h1 << 16));
        hi[e] = h0 | (h1 << 16);
        lo[e] = l0 | (l1 << 16);
        ss = fmaf(x1, x1, fmaf(x0, x0, ss));
      }
      if (hs_dst[u] >= 0) {
        *(u32x4*)(hs + hs_dst[u]) = hi;
        *(u32x4*)(hs + hs_dst[u] + pl.cols * HSS) = lo;
      }
      if (leaves_sums) {
        // 256 elements are 32 consecutive pieces = the lanes of half a wavefront (a group is all live or all
        // clamped: the slice is a whole number of such groups); fixed order, the same bits on every run
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
        if ((lane & 31) == 0 && ss_dst[u] >= 0) p.ss_out[ss_dst[u]] = ss;
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < kLoads; ++u)
      if (hs_dst[u] >= 0) *(u32x4*)(hs + hs_dst[u]) = hreg[u];
  }
  lds_barrier();
  for (int i0 = 0; i0 < n; i0 += STAGES) {
    for_each_stage([&](auto st) __attribute__((always_inline)) {
      constexpr int SS = decltype(st)::value;
      request(i0 + SS + STAGES - 1, std::integral_constant<int, (SS + STAGES - 1) % STAGES>{});
      consume(i0 + SS, st);
    });
  }

  // ---- the partial tiles: [row tile of the range][column tile][column][row] ---------------------------------
  float* out = p.part + (size_t)wave_global * (kSgAcc * NT * 256) + c * 16 + g * 4;
#pragma unroll
  for (int a = 0; a < kSgAcc; ++a)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) *(f32x4*)(out + (a * NT + nt) * 256) = acc[a][nt];
}

// n / d with the plan's magic number for d (ceil(2^32 / d) does not fit 32 bits for d = 1)
__device__ __forceinline__ int sg_div(int n, int d, unsigned int magic) {
  return d == 1 ? n : (int)__umulhi((unsigned)n, magic);
}

// Entry (col, row) of the product: the partial tiles of row tile row/16 - high and low part of the column -
// added group by group and wavefront by wavefront in ascending order.
__device__ __forceinline__ float sg_result(const float* __restrict__ part, const SkinnyPlan& pl, int col, int row) {
  const int r = row >> 4, rr = row & 15;
  const int vhi = col, vlo = pl.cols + col;
  const int ohi = (vhi >> 4) * 256 + (vhi & 15) * 16 + rr, olo = (vlo >> 4) * 256 + (vlo & 15) * 16 + rr;
  float s = 0.f;
#pragma unroll 1
  for (int q = 0; q < pl.groups; ++q) {
    const int Cg = pl.chunks[q], P = pl.per_wave[q];
    const unsigned int mP = pl.magic_per_wave[q], mC = pl.magic_chunks[q];
    const int first = sg_div(r * Cg, P, mP), last = sg_div(r * Cg + Cg - 1, P, mP);
    for (int w = first; w <= last; ++w) {
      const int which = r - sg_div(w * P, Cg, mC);
      const float* t = part + ((size_t)(pl.wave_begin[q] + w) * kSgAcc + which) * (pl.nt * 256);
      s += t[ohi] + t[olo];
    }
  }
  return s;
}

__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;  // NaN
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// fp32 value -> two bf16 numbers whose sum carries 16 bits of its mantissa, at index i of a [2][plane] array
__device__ __forceinline__ void store_split(unsigned short* planes, size_t plane_elems, size_t i, float v) {
  const unsigned short hi = float_to_bf16_bits(v);
  planes[i] = hi;
  planes[plane_elems + i] = float_to_bf16_bits(v - bf16_bits_to_float(hi));
}

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum_f32(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

struct LayerParams {
  const unsigned short* x;     // [B*T][D] bf16 input hidden states
  const unsigned short* ln1;   // [D]
  const unsigned short* ln2;   // [D]
  const int32_t* pos0;         // [B]
  int B, T, D, H, dh, F;
  float eps, log2_theta;
  // workspace
  // activations that feed a matrix product are [2][B*T][K] bf16: high parts, then low parts
  unsigned short* q;           // [B][H][T][dh]
  float* attn;                 // [B][H][T][dh] attention output
  unsigned short* arows;       // [2][B*T][D] attention output, heads side by side
  float* h1;                   // [B*T][D] residual stream after attention
  unsigned short* xn2;         // [2][B*T][D]
  unsigned short* act;         // [2][B*T][F]
  int32_t* n_rows;             // [B] = T
  unsigned long long* causal;  // [B][T] bit j of row t set for j <= t
  float* ss1;                  // [B*T][D/256] partial sums of x^2
  float* ss2;                  // [B*T][D/256] partial sums of h1^2
  // outputs
  unsigned short* k_new;       // [B][H][T][dh]
  unsigned short* v_new;       // [B][H][T][dh]
  unsigned short* out;         // [B*T][D]
  float* out_f32;              // [B*T][D] or null
  const float* part;
  int col0, cols;              // columns of the current pass
};

// RMSNorm is a per-column scalar times an elementwise gain, and the scalar commutes with the matrix product
// that follows: the product is taken of x * gain, the kernel that consumes it multiplies by
// 1 / sqrt(mean(x^2) + eps).  The sum of squares is left as one partial sum per 256 elements, added up by the
// consumer in ascending order.
__device__ __forceinline__ float inv_rms(const float* __restrict__ ss, int col, int nseg, int D, float eps) {
  float t = 0.f;
  for (int i = 0; i < nseg; ++i) t += ss[col * nseg + i];
  return 1.0f / sqrtf(t / (float)D + eps);
}

// q, k, v of the pass's columns: sum of the partial tiles times the norm's scalar (the first pass took x * gain and
// left the sums of x^2), rotary embedding on q and k, bf16, head-major layout
__global__ __launch_bounds__(256) void dl_qkv_finish_kernel(LayerParams p, SkinnyPlan pl) {
  if (blockIdx.x == 0 && blockIdx.y == 0 && p.col0 == 0) {
    // the row counts and the causal mask that the attention call takes
    for (int i = threadIdx.x; i < p.B; i += 256) p.n_rows[i] = p.T;
    for (int i = threadIdx.x; i < p.B * p.T; i += 256) {
      const int t = i % p.T;
      p.causal[i] = t >= 63 ? ~0ull : ((2ull << t) - 1ull);
    }
  }
  // grid: (blocks over the column's 3 H dh / 2 pairs, column of the pass) - no division by a runtime number per
  // element except the one that finds the head
  const int half = p.dh / 2;
  const int per_col = 3 * p.H * half;
  const int cl = blockIdx.y, col = p.col0 + cl, b = col / p.T, t = col - b * p.T;
  const float inv = inv_rms(p.ss1, col, p.D / 256, p.D, p.eps);
  for (int rem = blockIdx.x * 256 + threadIdx.x; rem < per_col; rem += gridDim.x * 256) {
    const int hq = rem / half, i = rem - hq * half;  // hq: 0..H-1 q heads, H..2H-1 k heads, 2H..3H-1 v heads
    const int row = hq * p.dh + i;
    float a = inv * sg_result(p.part, pl, cl, row), c = inv * sg_result(p.part, pl, cl, row + half);
    const int kind = hq / p.H, h = hq - kind * p.H;
    if (kind < 2) {
      // pair (i, i + dh/2) turned by the angle pos * theta^(-2i/dh)
      const float ang = (float)(p.pos0[b] + t) * exp2f(-2.0f * (float)i / (float)p.dh * p.log2_theta);
      float sn, cs;
      sincosf(ang, &sn, &cs);
      const float ra = a * cs - c * sn, rc = c * cs + a * sn;
      a = ra;
      c = rc;
    }
    unsigned short* dst = (kind == 0 ? p.q : kind == 1 ? p.k_new : p.v_new) + (((size_t)b * p.H + h) * p.T + t) * p.dh;
    dst[i] = float_to_bf16_bits(a);
    dst[i + half] = float_to_bf16_bits(c);
  }
}

// attention output [B][H][T][dh] fp32 -> rows [B*T][H*dh] bf16
__global__ __launch_bounds__(256) void dl_attn_rows_kernel(LayerParams p) {
  const int total = p.B * p.T * p.D;
  for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
    const int col = idx / p.D, k = idx - col * p.D;
    const int b = col / p.T, t = col - b * p.T, h = k / p.dh, d = k - h * p.dh;
    store_split(p.arows, (size_t)total, (size_t)idx, p.attn[(((size_t)b * p.H + h) * p.T + t) * p.dh + d]);
  }
}

// h1 = x + attention projection; h1 * ln2 (as two bf16 numbers) and the partial sums of h1^2.
// One block per (column of the pass, 256 elements).
__global__ __launch_bounds__(256) void dl_oproj_finish_kernel(LayerParams p, SkinnyPlan pl) {
  __shared__ float red[4];
  const int nseg = p.D / 256;
  const int cl = blockIdx.x / nseg, seg = blockIdx.x - cl * nseg, tid = threadIdx.x;
  const int col = p.col0 + cl, d = seg * 256 + tid;
  const size_t o = (size_t)col * p.D + d;
  const float v = bf16_bits_to_float(p.x[o]) + sg_result(p.part, pl, cl, d);
  p.h1[o] = v;
  store_split(p.xn2, (size_t)p.B * p.T * p.D, o, v * bf16_bits_to_float(p.ln2[d]));
  const float ss = block_sum_256(v * v, red);
  if (tid == 0) p.ss2[col * nseg + seg] = ss;
}

// act = silu(gate) * up; rows [0, F) of the fused matrix are the gate, rows [F, 2F) the up projection
__global__ __launch_bounds__(256) void dl_gate_finish_kernel(LayerParams p, SkinnyPlan pl) {
  const int cl = blockIdx.y;  // grid: (blocks over F, column of the pass)
  const float inv = inv_rms(p.ss2, p.col0 + cl, p.D / 256, p.D, p.eps);
  for (int f = blockIdx.x * 256 + threadIdx.x; f < p.F; f += gridDim.x * 256) {
    const float gt = inv * sg_result(p.part, pl, cl, f), up = inv * sg_result(p.part, pl, cl, p.F + f);
    store_split(p.act, (size_t)p.B * p.T * p.F, (size_t)(p.col0 + cl) * p.F + f, gt / (1.0f + expf(-gt)) * up);
  }
}

// out = h1 + feed-forward output
__global__ __launch_bounds__(256) void dl_down_finish_kernel(LayerParams p, SkinnyPlan pl) {
  const int cl = blockIdx.y;  // grid: (blocks over D, column of the pass)
  for (int d = blockIdx.x * 256 + threadIdx.x; d < p.D; d += gridDim.x * 256) {
    const size_t o = (size_t)(p.col0 + cl) * p.D + d;
    const float v = p.h1[o] + sg_result(p.part, pl, cl, d);
    if (p.out_f32) p.out_f32[o] = v;
    p.out[o] = float_to_bf16_bits(v);
  }
}

// ---- host side ---------------------------------------------------------------------------------------------------
static int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

// how the units of an [N][K] matrix are dealt to wavefronts; false if the shape is not supported
static bool make_plan(SkinnyPlan& pl, int N, int K, int cols, int cus) {
  if (K % 256 != 0 || N < 16 || N % 16 != 0 || cols < 1 || cols > kSgMaxCols) return false;
  const int C = K / 256, vcols = 2 * cols;
  int cg_max = (kSgLdsBudget / vcols - 32) / 512;
  const int by_pieces = kSgHsPieces * 64 * kSgWaves / (vcols * 32);
  cg_max = cg_max < by_pieces ? cg_max : by_pieces;
  if (cg_max < 1) return false;
  const int G = (C + cg_max - 1) / cg_max;
  if (G > kSgMaxGroups) return false;
  pl.N = N; pl.K = K; pl.cols = cols; pl.tiles = N / 16; pl.groups = G; pl.nt = (vcols + 15) / 16;
  // a range may touch kSgAcc row tiles: it must not be longer than kSgAcc - 1 tiles' units
  const int min_waves = ((pl.tiles + kSgAcc - 2) / (kSgAcc - 1) + kSgWaves - 1) / kSgWaves * kSgWaves;
  const int target = cus * kSgWaves;
  int begin_chunk = 0, begin_wave = 0, max_chunks = 0;
  for (int q = 0; q < kSgMaxGroups; ++q) {
    pl.chunk_begin[q] = pl.chunks[q] = pl.wave_begin[q] = 0;
    pl.per_wave[q] = 1;
    pl.magic_per_wave[q] = pl.magic_chunks[q] = 0;
  }
  for (int q = 0; q < G; ++q) {
    const int cg = C / G + (q < C % G ? 1 : 0);
    int waves = (int)((long long)target * cg / C) / kSgWaves * kSgWaves;
    waves = waves < min_waves ? min_waves : waves;
    pl.chunk_begin[q] = begin_chunk; pl.chunks[q] = cg;
    pl.wave_begin[q] = begin_wave;
    pl.per_wave[q] = (int)(((long long)pl.tiles * cg + waves - 1) / waves);
    pl.magic_per_wave[q] = pl.per_wave[q] > 1 ? (unsigned int)(((1ull << 32) + pl.per_wave[q] - 1) / pl.per_wave[q]) : 0u;
    pl.magic_chunks[q] = cg > 1 ? (unsigned int)(((1ull << 32) + cg - 1) / cg) : 0u;
    // the magic numbers are exact while dividend * divisor < 2^32
    if ((long long)pl.tiles * cg * (pl.per_wave[q] > cg ? pl.per_wave[q] : cg) >= (1LL << 31)) return false;
    begin_chunk += cg; begin_wave += waves;
    max_chunks = cg > max_chunks ? cg : max_chunks;
  }
  pl.total_waves = begin_wave;
  pl.hs_bytes = vcols * (max_chunks * 512 + 32);
  return true;
}

struct LayerWorkspace {
  size_t q, attn, arows, h1, xn2, act, n_rows, causal, ss1, ss2, part, total;
};
static LayerWorkspace layer_workspace(int B, int T, int D, int H, int F, int cus) {
  LayerWorkspace w;
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t at = off; off = (off + bytes + 255) / 256 * 256; return at; };
  const size_t BT = (size_t)B * T;
  w.q = carve(BT * D * 2); w.attn = carve(BT * D * 4); w.arows = carve(BT * D * 4);
  w.h1 = carve(BT * D * 4); w.xn2 = carve(BT * D * 4); w.act = carve(BT * F * 4);
  w.n_rows = carve((size_t)B * 4); w.causal = carve(BT * 8);
  w.ss1 = carve(BT * (D / 256 + 1) * 4); w.ss2 = carve(BT * (D / 256 + 1) * 4);
  size_t max_floats = 0;
  const int shapes[4][2] = {{3 * D, D}, {D, D}, {2 * F, D}, {D, F}};
  for (auto& s : shapes) {
    SkinnyPlan pl;
    if (make_plan(pl, s[0], s[1], kSgMaxCols < (int)BT ? kSgMaxCols : (int)BT, cus)) {
      const size_t floats = (size_t)pl.total_waves * kSgAcc * pl.nt * 256;
      max_floats = floats > max_floats ? floats : max_floats;
    }
  }
  w.part = carve(max_floats * sizeof(float));
  w.total = off;
  return w;
}

template <int NT, bool FIRST>
static hipError_t launch_skinny_nt(const SkinnyParams& sp, hipStream_t stream) {
  const int lds = sp.plan.hs_bytes + kSgWaves * kSgStripBytes;
  hipLaunchKernelGGL((skinny_gemm_bf16_kernel<kSgStages, NT, FIRST>), dim3(sp.plan.total_waves / kSgWaves),
                     dim3(64 * kSgWaves), lds, stream, sp);
  return hipGetLastError();
}
// first: the layer's first pass (sp.gain and sp.ss_out set, sp.x the input as given)
static hipError_t launch_skinny(const SkinnyParams& sp, bool first, hipStream_t stream) {
  if (first) return sp.plan.nt == 1 ? launch_skinny_nt<1, true>(sp, stream) : launch_skinny_nt<2, true>(sp, stream);
  return sp.plan.nt == 1 ? launch_skinny_nt<1, false>(sp, stream) : launch_skinny_nt<2, false>(sp, stream);
}

hipError_t prepare_draft_layer() {
  const void* kernels[] = {(const void*)skinny_gemm_bf16_kernel<kSgStages, 1, false>,
                           (const void*)skinny_gemm_bf16_kernel<kSgStages, 2, false>,
                           (const void*)skinny_gemm_bf16_kernel<kSgStages, 1, true>,
                           (const void*)skinny_gemm_bf16_kernel<kSgStages, 2, true>};
  for (const void* k : kernels) {
    const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" size_t draft_layer_workspace_bytes(int B, int T, int D, int H, int F) {
  if (B < 1 || T < 1 || D < 1 || H < 1 || F < 1) return 0;
  return layer_workspace(B, T, D, H, F, device_cus()).total;
}

extern "C" int draft_layer_forward(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* x,
                                   const ctcspec_layer_weights* w, const int32_t* pos0, void* k_cache,
                                   void* v_cache, const int64_t* kv_off, const int32_t* ctx_len, int kv_cap, int B,
                                   int T, int D, int H, int F, float rms_eps, float rope_theta, void* workspace,
                                   size_t workspace_bytes, void* q_out, void* k_new, void* v_new, void* out, float* out_f32) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
  CTCSPEC_REQUIRE(ctx, x && w && pos0 && k_cache && v_cache && kv_off && ctx_len && workspace && k_new && v_new && out,
                  CTCSPEC_EINVAL, "draft_layer_forward: null pointer");
  CTCSPEC_REQUIRE(ctx, w->ln1 && w->wqkv && w->wo && w->ln2 && w->wgu && w->wd, CTCSPEC_EINVAL,
                  "draft_layer_forward: null weight pointer");
  CTCSPEC_REQUIRE(ctx, dt == CTCSPEC_BF16, CTCSPEC_EUNSUPPORTED, "draft_layer_forward: bf16 only");
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && D > 0 && H > 0 && F > 0 && kv_cap >= 0, CTCSPEC_EINVAL,
                  "draft_layer_forward: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, D % H == 0 && D % 256 == 0 && F % 256 == 0 && (D / H) % 8 == 0 && D / H <= CTCSPEC_MAX_HEAD_DIM,
                  CTCSPEC_EUNSUPPORTED,
                  "draft_layer_forward: D and F must be multiples of 256, D/H a multiple of 8 and <= %d",
                  CTCSPEC_MAX_HEAD_DIM);
  CTCSPEC_REQUIRE(ctx, T <= 64 && T <= ctx->lim.max_nodes && B <= ctx->lim.max_batch && H <= ctx->lim.max_heads &&
                           D / H <= ctx->lim.max_head_dim,
                  CTCSPEC_EUNSUPPORTED, "draft_layer_forward: shape exceeds the context's limits");
  CTCSPEC_REQUIRE(ctx, rms_eps >= 0.f && rope_theta > 1.f, CTCSPEC_EINVAL, "draft_layer_forward: bad eps or theta");
  const void* ptrs[] = {x, w->ln1, w->wqkv, w->wo, w->wgu, w->wd, workspace, q_out, k_new, v_new, out, k_cache, v_cache};
  for (const void* q : ptrs)
    CTCSPEC_REQUIRE(ctx, aligned16(q), CTCSPEC_EINVAL, "draft_layer_forward: pointers must be 16-byte aligned");
  const int cus = device_cus();
  const LayerWorkspace lw = layer_workspace(B, T, D, H, F, cus);
  CTCSPEC_REQUIRE(ctx, workspace_bytes >= lw.total, CTCSPEC_EINVAL,
                  "draft_layer_forward: workspace of %zu bytes needed, %zu given", lw.total, workspace_bytes);

  unsigned char* ws = (unsigned char*)workspace;
  LayerParams p;
  p.x = (const unsigned short*)x; p.ln1 = (const unsigned short*)w->ln1; p.ln2 = (const unsigned short*)w->ln2;
  p.pos0 = pos0; p.B = B; p.T = T; p.D = D; p.H = H; p.dh = D / H; p.F = F;
  p.eps = rms_eps; p.log2_theta = log2f(rope_theta);
  p.q = q_out ? (unsigned short*)q_out : (unsigned short*)(ws + lw.q); p.attn = (float*)(ws + lw.attn);
  p.arows = (unsigned short*)(ws + lw.arows); p.h1 = (float*)(ws + lw.h1); p.xn2 = (unsigned short*)(ws + lw.xn2);
  p.act = (unsigned short*)(ws + lw.act); p.n_rows = (int32_t*)(ws + lw.n_rows);
  p.causal = (unsigned long long*)(ws + lw.causal); p.ss1 = (float*)(ws + lw.ss1); p.ss2 = (float*)(ws + lw.ss2);
  p.k_new = (unsigned short*)k_new; p.v_new = (unsigned short*)v_new; p.out = (unsigned short*)out; p.out_f32 = out_f32;
  p.part = (const float*)(ws + lw.part); p.col0 = 0; p.cols = 0;
  const int BT = B * T;
  hipStream_t st = ctx->stream;

  // one pass over a weight matrix per block of 16 columns, each followed by the kernel that consumes the tiles
  auto gemm_passes = [&](const void* wmat, int N, int K, const unsigned short* xin, bool first, auto&& finish) -> int {
    for (int col0 = 0; col0 < BT; col0 += kSgMaxCols) {
      SkinnyParams sp;
      sp.gain = first ? (const void*)p.ln1 : nullptr;
      sp.ss_out = first ? p.ss1 : nullptr;
      const int cols = BT - col0 < kSgMaxCols ? BT - col0 : kSgMaxCols;
      CTCSPEC_REQUIRE(ctx, make_plan(sp.plan, N, K, cols, cus), CTCSPEC_EUNSUPPORTED,
                      "draft_layer_forward: a %d x %d matrix does not fit the streaming kernel", N, K);
      sp.w = wmat; sp.x = xin; sp.plane_cols = BT; sp.col0 = col0; sp.zeros = ctx->zeros; sp.part = (float*)(ws + lw.part);
      CTCSPEC_HIP(ctx, launch_skinny(sp, first, st));
      p.col0 = col0; p.cols = cols;
      finish(sp.plan);
      CTCSPEC_HIP(ctx, hipGetLastError());
    }
    return CTCSPEC_OK;
  };
  auto blocks_for = [](long long n) { long long b = (n + 255) / 256; return (unsigned)(b > 1024 ? 1024 : (b < 1 ? 1 : b)); };

  int rc = gemm_passes(w->wqkv, 3 * D, D, p.x, true, [&](const SkinnyPlan& pl) {
    hipLaunchKernelGGL(dl_qkv_finish_kernel, dim3(blocks_for((long long)3 * H * (p.dh / 2)), p.cols), dim3(256), 0, st, p, pl);
  });
  if (rc != CTCSPEC_OK) return rc;
  int rows_written = 0;  // with key splits the attention's merge kernel writes the rows itself
  rc = tree_verify_attn_rows(ctx, dt, p.q, k_cache, v_cache, kv_off, ctx_len, kv_cap, k_new, v_new, p.n_rows,
                             (const uint64_t*)p.causal, B, H, p.dh, T, 1.0f / sqrtf((float)p.dh), p.attn, p.arows,
                             (long long)BT * D, &rows_written);
  if (rc != CTCSPEC_OK) return rc;
  if (!rows_written) {
    hipLaunchKernelGGL(dl_attn_rows_kernel, dim3(blocks_for((long long)BT * D)), dim3(256), 0, st, p);
    CTCSPEC_HIP(ctx, hipGetLastError());
  }
  rc = gemm_passes(w->wo, D, D, p.arows, false, [&](const SkinnyPlan& pl) {
    hipLaunchKernelGGL(dl_oproj_finish_kernel, dim3(p.cols * (D / 256)), dim3(256), 0, st, p, pl);
  });
  if (rc != CTCSPEC_OK) return rc;
  rc = gemm_passes(w->wgu, 2 * F, D, p.xn2, false, [&](const SkinnyPlan& pl) {
    hipLaunchKernelGGL(dl_gate_finish_kernel, dim3(blocks_for((long long)F), p.cols), dim3(256), 0, st, p, pl);
  });
  if (rc != CTCSPEC_OK) return rc;
  rc = gemm_passes(w->wd, D, F, p.act, false, [&](const SkinnyPlan& pl) {
    hipLaunchKernelGGL(dl_down_finish_kernel, dim3(blocks_for((long long)D), p.cols), dim3(256), 0, st, p, pl);
  });
  return rc;
}
