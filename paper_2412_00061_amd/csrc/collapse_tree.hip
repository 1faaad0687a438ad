// ctc_collapse_tree: raw candidates -> CTC collapse -> dedupe -> best `beam` drafts -> prefix tree + mask.
//
// One workgroup of 256 threads per sequence; the k^T raw candidates are never all materialised.
//
// A raw candidate's score is a sum over slots, so the slots are split into a first and a second half
// with n1 and n2 rank combinations and partial sums X_a, Y_b (each the exact left-to-right float32
// partial sum).  With both lists sorted descending, X_(i) + Y_(j) is at least as large as every
// (i', j') with i' >= i and j' >= j; hence tau = max_i X_(i) + Y_(ceil(M/(i+1))-1) is passed by at
// least M raw candidates - a threshold without search.  The raw candidates passing it (about 2M)
// are expanded, given their exact float32 left-to-right score, sorted by (score desc, idx asc) and
// walked in that order: collapse, drop empties, keep first occurrences.  If fewer than `beam`
// distinct drafts turn up, M is quadrupled and the level redone; the last level takes every raw
// candidate.  The half-sum score fl(X+Y) used for thresholding differs from the exact score only by
// rounding; a margin delta on the threshold makes the walked prefix exactly the global order.
//
// Sorted candidates live in LDS while they fit (4096) and in the context's global workspace
// otherwise (mass ties, or nearly every raw candidate needed).
#include "common.h"

namespace ctcspec {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kHalfMax = 512;   // k^ceil(T/2) <= 8^3
constexpr int kLdsCap = 4096;   // sorted candidates kept in LDS
constexpr int kBlankCode = 127; // 7-bit local code of the blank / padding
constexpr unsigned int kEmptySlot = 0xffffffffu;

struct CollapseParams {
  const int32_t* topk_id;
  const float* topk_logp;
  const int32_t* root_token;
  int T, k, blank_id, beam, max_nodes;
  unsigned int magic;  // ceil(2^32 / k): division by k as a multiply-high
  int32_t* n_cand;
  int32_t* cand_tokens;
  int32_t* cand_len;
  float* cand_score;
  int32_t* cand_leaf;
  int32_t* n_nodes;
  int32_t* node_token;
  int32_t* node_parent;
  int32_t* node_depth;
  unsigned long long* anc_mask;
  unsigned char* ws;  // per-sequence global workspace base
};

struct CollapseShared {
  int ids[64];
  float logp[64];
  int code[64];
  float Xv[kHalfMax];  // sorted descending
  int Xi[kHalfMax];
  float Yv[kHalfMax];
  int Yi[kHalfMax];
  int prefix[kHalfMax + 1];
  int red[kWaves];
  float redf[kWaves];
  float delta;
  unsigned long long kept_ck[CTCSPEC_MAX_BEAM];
  unsigned long long kept_first[CTCSPEC_MAX_BEAM];  // per draft: first earlier draft sharing each prefix length
  int kept_len[CTCSPEC_MAX_BEAM];
  int kept_tok[CTCSPEC_MAX_BEAM][CTCSPEC_MAX_SLOTS];
  int kept_m[CTCSPEC_MAX_BEAM];
  int kept_base[CTCSPEC_MAX_BEAM];
  unsigned long long keys[kLdsCap];
  unsigned long long ckeys[kLdsCap];
  unsigned int table[2 * kLdsCap];
};

// inclusive prefix sum over the wavefront (DPP row shifts, then the row totals through readlane)
__device__ __forceinline__ int wave_inclusive_scan_i32(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
  const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
            t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row > 0 ? t0 : 0) + (row > 1 ? t1 : 0) + (row > 2 ? t2 : 0);
}

__device__ __forceinline__ int block_sum(int v, int* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_sum_i32(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) s += red[w];
  return s;
}

__device__ __forceinline__ float block_max(float v, float* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_max_f32(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) s = fmaxf(s, red[w]);
  return s;
}

// exclusive prefix of v over the workgroup's threads (thread order), total in *total
__device__ __forceinline__ int block_exclusive_scan(int v, int* red, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int incl = wave_inclusive_scan_i32(v);
  __syncthreads();
  if (lane == 63) red[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int x = red[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

// number of second-half combinations j (sorted descending) with fl(x + Yv[j]) >= tau
__device__ __forceinline__ int count_ge(float x, const float* Yv, int n2, float tau) {
  int lo = 0, hi = n2;  // invariant: entries < lo pass, entries >= hi fail
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (x + Yv[mid] >= tau) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ unsigned int hash_slot(unsigned long long ck, int log2_size) {
  return (unsigned int)((ck * 0x9E3779B97F4A7C15ull) >> (64 - log2_size));
}

#define CTCSPEC_CE(a, b, desc)                         \
  {                                                    \
    const unsigned long long x_ = a, y_ = b;           \
    const bool sw_ = (x_ < y_) == (desc);              \
    a = sw_ ? y_ : x_;                                 \
    b = sw_ ? x_ : y_;                                 \
  }

// descending bitonic sort of n (power of two, >= 4) keys by the whole workgroup; two compare-exchange
// stages are fused per pass (four keys per thread in registers) to halve the number of barriers
__device__ void block_bitonic_sort_desc(unsigned long long* keys, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    int stride = size >> 1;
    while (stride > 0) {
      if (stride >= 2) {
        const int s2 = stride >> 1;
        for (int t = threadIdx.x; t < (n >> 2); t += kThreads) {
          const int i = ((t & ~(s2 - 1)) << 2) | (t & (s2 - 1));
          const bool desc = (i & size) == 0;
          unsigned long long e0 = keys[i], e1 = keys[i + s2], e2 = keys[i + stride], e3 = keys[i + stride + s2];
          CTCSPEC_CE(e0, e2, desc)
          CTCSPEC_CE(e1, e3, desc)
          CTCSPEC_CE(e0, e1, desc)
          CTCSPEC_CE(e2, e3, desc)
          keys[i] = e0; keys[i + s2] = e1; keys[i + stride] = e2; keys[i + stride + s2] = e3;
        }
        stride >>= 2;
      } else {
        for (int t = threadIdx.x; t < (n >> 1); t += kThreads) {
          const int i = t << 1;
          const bool desc = (i & size) == 0;
          unsigned long long e0 = keys[i], e1 = keys[i + 1];
          CTCSPEC_CE(e0, e1, desc)
          keys[i] = e0; keys[i + 1] = e1;
        }
        stride = 0;
      }
      __syncthreads();
    }
  }
}
#undef CTCSPEC_CE


// ---- register-resident sorting -------------------------------------------------------------------
// value held by lane (l ^ D), D a power of two below 64
template <int D>
__device__ __forceinline__ unsigned int xor_fetch_u32(unsigned int v, bool ror4_is_up) {
  if constexpr (D == 1) return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);
  else if constexpr (D == 2) return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);
  else if constexpr (D == 4) {
    // a rotation by 4 inside the row of 16 reaches lane l^4 for half of the lanes, the rotation by 12
    // for the other half; which is which was probed once (ror4_is_up), not assumed
    const unsigned int a = dpp_row_ror<4>(v), b = dpp_row_ror<12>(v);
    return ror4_is_up ? a : b;
  } else if constexpr (D == 8) return dpp_row_ror<8>(v);
  else return (unsigned int)__shfl_xor((int)v, D, 64);
}
template <int D>
__device__ __forceinline__ unsigned long long xor_fetch_u64(unsigned long long v, bool ror4_is_up) {
  const unsigned int lo = xor_fetch_u32<D>((unsigned int)v, ror4_is_up);
  const unsigned int hi = xor_fetch_u32<D>((unsigned int)(v >> 32), ror4_is_up);
  return ((unsigned long long)hi << 32) | lo;
}

template <int E, int SIZE, int STRIDE>
__device__ __forceinline__ void bitonic_stage(unsigned long long (&v)[E], int lane, bool ror4_is_up) {
  if constexpr (STRIDE >= E) {
    constexpr int D = STRIDE / E;
    const bool lower = (lane & D) == 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const unsigned long long o = xor_fetch_u64<D>(v[e], ror4_is_up);
      const bool desc = ((lane * E + e) & SIZE) == 0;
      const bool keep_max = lower == desc;
      const bool o_larger = o > v[e];
      v[e] = (o_larger == keep_max) ? o : v[e];
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if ((e & STRIDE) == 0) {
        const bool desc = ((lane * E + e) & SIZE) == 0;
        const unsigned long long x = v[e], y = v[e + STRIDE];
        const bool sw = (x < y) == desc;
        v[e] = sw ? y : x;
        v[e + STRIDE] = sw ? x : y;
      }
    }
  }
}
template <int E, int SIZE, int STRIDE>
__device__ __forceinline__ void bitonic_merge(unsigned long long (&v)[E], int lane, bool ror4_is_up) {
  bitonic_stage<E, SIZE, STRIDE>(v, lane, ror4_is_up);
  if constexpr (STRIDE > 1) bitonic_merge<E, SIZE, STRIDE / 2>(v, lane, ror4_is_up);
}
template <int E, int SIZE>
__device__ __forceinline__ void bitonic_sort_upto(unsigned long long (&v)[E], int lane, bool ror4_is_up) {
  if constexpr (SIZE > 2) bitonic_sort_upto<E, SIZE / 2>(v, lane, ror4_is_up);
  bitonic_merge<E, SIZE, SIZE / 2>(v, lane, ror4_is_up);
}
// Sort the 64*E keys of one wavefront descending; key index inside the wavefront = lane*E + e.
template <int E>
__device__ __forceinline__ void wave_bitonic_sort_desc(unsigned long long (&v)[E], int lane, bool ror4_is_up) {
  bitonic_sort_upto<E, 64 * E>(v, lane, ror4_is_up);
}

// Sort kThreads*E keys descending: every wavefront sorts its 64*E keys in registers, the kWaves sorted
// runs are merged by rank (position in the own run + number of larger keys in every other run, found
// by binary search; equal keys are ordered by run).  v[e] is key number (tid*E + e) on entry.
// runs: LDS scratch of kThreads*E keys; out: kThreads*E keys, sorted on return (barrier included).
template <int E>
__device__ __forceinline__ void block_sort_desc_fast(unsigned long long (&v)[E], unsigned long long* runs,
                                                     unsigned long long* out, bool ror4_is_up) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int RUN = 64 * E;
  wave_bitonic_sort_desc<E>(v, lane, ror4_is_up);
#pragma unroll
  for (int e = 0; e < E; ++e) runs[wave * RUN + lane * E + e] = v[e];
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const unsigned long long key = v[e];
    int rank = lane * E + e;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if (w == wave) continue;
      const unsigned long long* r = runs + w * RUN;
      // number of keys of run w that come before `key`: strictly larger, or equal when w < wave
      int lo = 0, hi = RUN;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const unsigned long long x = r[mid];
        const bool before = (w < wave) ? (x >= key) : (x > key);
        if (before) lo = mid + 1; else hi = mid;
      }
      rank += lo;
    }
    out[rank] = key;
  }
  __syncthreads();
}

// a / k and a % k for 0 <= a < 65536, magic = ceil(2^32 / k)
__device__ __forceinline__ int div_small(int a, unsigned int magic) { return (int)__umulhi((unsigned)a, magic); }

// The four rank digits of a half-combination, most significant slot first.  a counts in base k with
// nt <= 4 digits; it is first shifted up to exactly four digits so that digit positions are static.
struct Digits4 {
  int r[4];  // r[t] = rank chosen for the half's slot t (valid for t < nt)
};
__device__ __forceinline__ Digits4 split_digits(int a, int pad, int k, unsigned int magic) {
  Digits4 d;
  int x = a * pad;  // pad = k^(4-nt)
#pragma unroll
  for (int u = 3; u >= 0; --u) {
    const int q = div_small(x, magic);
    d.r[u] = x - q * k;
    x = q;
  }
  return d;
}

// left-to-right float32 sum: acc, then the half's slots t0.. in order
__device__ __forceinline__ float add_slots(float acc, bool have_acc, const float* logp, const Digits4& d, int t0,
                                           int nt, int k) {
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    if (t < nt) {
      const float l = logp[(t0 + t) * k + d.r[t]];
      acc = (have_acc || t > 0) ? acc + l : l;
    }
  }
  return acc;
}

// Collapsed-sequence key of the raw candidate (a, b): 7-bit local token codes, position 0 in the low
// bits, unused positions = kBlankCode.  Optionally writes the collapsed token ids.
__device__ __forceinline__ unsigned long long collapse_key(const CollapseShared& s, const Digits4& da,
                                                           const Digits4& db, int T1, int T2, int k, int* len_out,
                                                           int* tok_out) {
  unsigned long long key = 0x00ffffffffffffffull;
  int len = 0, prev = -1;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const bool first_half = u < 4;
    const int t_in = first_half ? u : u - 4;
    const bool live = first_half ? (t_in < T1) : (t_in < T2);
    if (live) {
      const int slot = first_half ? t_in : T1 + t_in;
      const int r = first_half ? da.r[t_in] : db.r[t_in];
      const int cd = s.code[slot * k + r];
      if (cd != prev && cd != kBlankCode) {
        key &= ~(0x7full << (7 * len));
        key |= (unsigned long long)cd << (7 * len);
        if (tok_out) tok_out[len] = s.ids[slot * k + r];
        ++len;
      }
      prev = cd;
    }
  }
  *len_out = len;
  return key;
}

__global__ __launch_bounds__(kThreads) void collapse_tree_kernel(CollapseParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  CollapseShared& s = *reinterpret_cast<CollapseShared*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int T = p.T, k = p.k, TK = p.T * p.k;
  const int beam = p.beam, max_nodes = p.max_nodes;
  const unsigned int magic = p.magic;
  const bool ror4_is_up = dpp_row_ror<4>((unsigned)lane) == (unsigned)(lane ^ 4);

  // ---- inputs, local token codes, rounding margin (first wavefront, registers only) -------------
  if (wave == 0) {
    const int id = lane < TK ? p.topk_id[(size_t)b * TK + lane] : -1;
    const float lp = lane < TK ? p.topk_logp[(size_t)b * TK + lane] : 0.f;
    int cd = lane;  // code = position of the first entry with the same token id
    for (int j = 0; j < TK; ++j) {
      const int idj = __builtin_amdgcn_readlane(id, j);
      if (idj == id && j < cd) cd = j;
    }
    // delta bounds |fl(X+Y) - exact score|: both are sums of the same T terms, each addition off by
    // at most 2^-24 of a partial sum, partial sums bounded by A = sum_t max_j |logp[t,j]|.
    // 14 * 2^-24 * A would do; 16 * 2^-23 * A leaves room for rounding of the thresholds themselves.
    float A = 0.f;
    for (int t = 0; t < T; ++t) {
      float mx = 0.f;
      for (int j = 0; j < k; ++j)
        mx = fmaxf(mx, fabsf(__uint_as_float(readlane_u32(__float_as_uint(lp), t * k + j))));
      A += mx;
    }
    if (lane < TK) {
      s.ids[lane] = id;
      s.logp[lane] = lp;
      s.code[lane] = (id == p.blank_id) ? kBlankCode : cd;
    }
    if (lane == 0) s.delta = A * (16.0f / 8388608.0f);
  }
  const int T1 = (T + 1) >> 1, T2 = T - T1;
  int n1 = 1, n2 = 1, pad1 = 1, pad2 = 1;
  for (int t = 0; t < 4; ++t) {
    if (t < T1) n1 *= k; else pad1 *= k;
    if (t < T2) n2 *= k; else pad2 *= k;
  }
  const int total = n1 * n2;
  __syncthreads();
  const float delta = s.delta;

  // ---- half sums X (slots < T1) and Y (the rest), both sorted descending in one sort ------------
  // key = [is X : 1][ordered value : 32][~index : 31]: all X sort before all Y
  {
    const int nxy = n1 + n2;
    auto make_key = [&](int gi) -> unsigned long long {
      if (gi >= nxy) return 0ull;
      const bool is_x = gi < n1;
      const int a = is_x ? gi : gi - n1;
      const Digits4 d = split_digits(a, is_x ? pad1 : pad2, k, magic);
      const float v = add_slots(0.f, false, s.logp, d, is_x ? 0 : T1, is_x ? T1 : T2, k);
      return ((unsigned long long)(is_x ? 1 : 0) << 63) | ((unsigned long long)float_to_ordered(v) << 31) |
             (unsigned long long)(0x7fffffff - a);
    };
    if (nxy <= 2 * kThreads) {
      unsigned long long v[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) v[e] = make_key(tid * 2 + e);
      block_sort_desc_fast<2>(v, s.ckeys, s.keys, ror4_is_up);
    } else {
      unsigned long long v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = make_key(tid * 4 + e);
      block_sort_desc_fast<4>(v, s.ckeys, s.keys, ror4_is_up);
    }
    for (int i = tid; i < nxy; i += kThreads) {
      const unsigned long long key = s.keys[i];
      const float v = ordered_to_float((unsigned int)(key >> 31));
      const int a = 0x7fffffff - (int)(key & 0x7fffffffull);
      if (i < n1) { s.Xv[i] = v; s.Xi[i] = a; }
      else { s.Yv[i - n1] = v; s.Yi[i - n1] = a; }
    }
    __syncthreads();
  }

  unsigned long long* keys = s.keys;
  unsigned long long* ckeys = s.ckeys;
  unsigned int* table = s.table;
  bool in_lds = true;

  int M = beam;
  int n_v = 0, n_d = 0, log2_ts = 6;
  for (;;) {
    if (M > total) M = total;
    const bool final_level = (M >= total);
    float tau_valid = -INFINITY, tau_f = -INFINITY;
    if (!final_level) {
      // X_(i) + Y_(j) with (i+1)(j+1) >= M is passed by at least M raw candidates
      float best = -INFINITY;
      for (int i = tid; i < n1; i += kThreads) {
        const int j = (M + i) / (i + 1) - 1;
        if (j < n2) best = fmaxf(best, s.Xv[i] + s.Yv[j]);
      }
      const float tau = block_max(best, s.redf);
      tau_valid = tau - delta;
      tau_f = tau_valid - delta;
    }
    // survivors per (sorted) first-half combination, prefix sums
    int n_s = 0;
    {
      // kHalfMax <= 2 * kThreads: thread t owns entries 2t and 2t+1
      const int i0 = 2 * tid, i1 = 2 * tid + 1;
      const int c0 = i0 < n1 ? count_ge(s.Xv[i0], s.Yv, n2, tau_f) : 0;
      const int c1 = i1 < n1 ? count_ge(s.Xv[i1], s.Yv, n2, tau_f) : 0;
      const int excl = block_exclusive_scan(c0 + c1, s.red, &n_s);
      if (i0 < n1) s.prefix[i0] = excl;
      if (i1 < n1) s.prefix[i1] = excl + c0;
      if (tid == 0) s.prefix[n1] = n_s;
    }
    if (in_lds && n_s > kLdsCap) {
      in_lds = false;
      keys = reinterpret_cast<unsigned long long*>(p.ws + (size_t)b * kCollapseWsBytesPerSeq);
      ckeys = keys + kMaxAlign;
      table = reinterpret_cast<unsigned int*>(ckeys + kMaxAlign);
    }
    __syncthreads();
    // exact key of survivor number i (row = sorted X entry, column = sorted Y entry)
    auto survivor_key = [&](int i) -> unsigned long long {
      if (i >= n_s) return 0ull;
      int lo_a = 0, hi_a = n1;  // largest row with prefix[row] <= i
      while (hi_a - lo_a > 1) {
        const int mid = (lo_a + hi_a) >> 1;
        if (s.prefix[mid] <= i) lo_a = mid; else hi_a = mid;
      }
      const int ib = s.Yi[i - s.prefix[lo_a]];
      const Digits4 db = split_digits(ib, pad2, k, magic);
      // the first half's partial sum is exactly the left-to-right prefix of the score
      const float sc = add_slots(s.Xv[lo_a], true, s.logp, db, T1, T2, k);
      return rank_key(sc, (unsigned)(s.Xi[lo_a] * n2 + ib));
    };
    if (n_s <= 2 * kThreads) {
      unsigned long long v[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) v[e] = survivor_key(tid * 2 + e);
      block_sort_desc_fast<2>(v, s.ckeys, s.keys, ror4_is_up);
    } else if (n_s <= 8 * kThreads) {
      unsigned long long v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = survivor_key(tid * 8 + e);
      block_sort_desc_fast<8>(v, s.ckeys, s.keys, ror4_is_up);
    } else {
      int P2 = 64;
      while (P2 < n_s) P2 <<= 1;
      for (int i = tid; i < P2; i += kThreads) keys[i] = survivor_key(i);
      __syncthreads();
      block_bitonic_sort_desc(keys, P2);
    }

    // the prefix that is exactly the global (score desc, idx asc) order
    if (final_level) {
      n_v = n_s;
    } else {
      int c = 0;
      for (int i = tid; i < n_s; i += kThreads) c += (rank_key_value(keys[i]) >= tau_valid) ? 1 : 0;
      n_v = block_sum(c, s.red);
    }
    // collapse every walked candidate and find first occurrences through a hash table of positions
    log2_ts = 6;
    while ((1 << log2_ts) < 2 * n_v) ++log2_ts;
    const int TS = 1 << log2_ts;
    for (int i = tid; i < TS; i += kThreads) table[i] = kEmptySlot;
    for (int i = tid; i < n_v; i += kThreads) {
      const int idx = (int)rank_key_index(keys[i]);
      const int a = idx / n2, bb = idx - a * n2;
      int len;
      const unsigned long long ck = collapse_key(s, split_digits(a, pad1, k, magic), split_digits(bb, pad2, k, magic),
                                                 T1, T2, k, &len, nullptr);
      ckeys[i] = len ? ck : ~0ull;  // ~0 marks the empty draft (no real key has the top byte set)
    }
    __syncthreads();
    for (int i = tid; i < n_v; i += kThreads) {
      const unsigned long long ck = ckeys[i];
      if (ck == ~0ull) continue;
      unsigned int slot = hash_slot(ck, log2_ts);
      for (;;) {
        unsigned int cur = table[slot];
        if (cur == kEmptySlot) {
          cur = atomicCAS(&table[slot], kEmptySlot, (unsigned)i);
          if (cur == kEmptySlot) break;
        }
        if (ckeys[cur] == ck) { atomicMin(&table[slot], (unsigned)i); break; }
        slot = (slot + 1) & (TS - 1);
      }
    }
    __syncthreads();
    // count distinct non-empty drafts; thread t scans positions [t*per, (t+1)*per)
    const int per = (n_v + kThreads - 1) / kThreads;
    int first_cnt = 0;
    for (int i = tid * per; i < (tid + 1) * per && i < n_v; ++i) {
      const unsigned long long ck = ckeys[i];
      if (ck == ~0ull) continue;
      unsigned int slot = hash_slot(ck, log2_ts);
      while (ckeys[table[slot]] != ck) slot = (slot + 1) & (TS - 1);
      first_cnt += (table[slot] == (unsigned)i) ? 1 : 0;
    }
    const int rank0 = block_exclusive_scan(first_cnt, s.red, &n_d);
    if (n_d >= beam || final_level) {
      // write the kept drafts (rank < beam)
      int rank = rank0;
      for (int i = tid * per; i < (tid + 1) * per && i < n_v && rank < beam; ++i) {
        const unsigned long long ck = ckeys[i];
        if (ck == ~0ull) continue;
        unsigned int slot = hash_slot(ck, log2_ts);
        while (ckeys[table[slot]] != ck) slot = (slot + 1) & (TS - 1);
        if (table[slot] != (unsigned)i) continue;
        const int idx = (int)rank_key_index(keys[i]);
        const int a = idx / n2, bb = idx - a * n2;
        int len;
        collapse_key(s, split_digits(a, pad1, k, magic), split_digits(bb, pad2, k, magic), T1, T2, k, &len,
                     s.kept_tok[rank]);
        s.kept_ck[rank] = ck;
        s.kept_len[rank] = len;
        p.cand_score[(size_t)b * beam + rank] = rank_key_value(keys[i]);
        ++rank;
      }
      break;
    }
    M *= 4;
    __syncthreads();
  }
  __syncthreads();

  // ---- outputs: drafts --------------------------------------------------------------------------
  const int n_c = n_d < beam ? n_d : beam;
  for (int i = tid; i < beam * T; i += kThreads) {
    const int c = i / T, d = i - c * T;
    p.cand_tokens[(size_t)b * beam * T + i] = (c < n_c && d < s.kept_len[c]) ? s.kept_tok[c][d] : -1;
  }
  for (int c = tid; c < beam; c += kThreads) {
    p.cand_len[(size_t)b * beam + c] = c < n_c ? s.kept_len[c] : 0;
    if (c >= n_c) p.cand_score[(size_t)b * beam + c] = -INFINITY;
  }

  // ---- prefix tree --------------------------------------------------------------------------------
  // Draft c needs m = the longest prefix it shares with any earlier draft and, for every prefix length
  // d <= m, the FIRST earlier draft sharing it (that draft created the node).  Thread (c, half) walks
  // half of the earlier drafts; the halves are combined through LDS.  Tokens beyond m create nodes;
  // node ids are handed out in (draft, depth) order.
  {
    const int c = tid & 127, half = tid >> 7;  // beam <= 128, kThreads == 256
    int have = 0;
    unsigned long long first = 0ull;  // byte d-1 = first draft sharing the prefix of length d
    if (c < n_c) {
      const unsigned long long mine = s.kept_ck[c];
      const int lo2 = half * 64;
      const int hi2 = c < lo2 + 64 ? c : lo2 + 64;
      for (int c2 = lo2; c2 < hi2; ++c2) {
        const int lcp = (__builtin_ctzll(mine ^ s.kept_ck[c2]) * 37) >> 8;  // ctz / 7 for ctz < 64
        while (have < lcp) {
          first |= (unsigned long long)c2 << (8 * have);
          ++have;
        }
      }
    }
    if (half == 1) {
      s.kept_m[c] = have;       // scratch: second half's result
      s.kept_first[c] = first;
    }
    __syncthreads();
    int my_new = 0;
    if (half == 0 && c < n_c) {
      const int have1 = s.kept_m[c];
      const unsigned long long first1 = s.kept_first[c];
      // prefix lengths <= have come from the lower half (smaller draft numbers win); longer ones, if
      // any, from the upper half
      if (have1 > have) {
        const unsigned long long keep = have ? (~0ull >> (64 - 8 * have)) : 0ull;
        first = (first & keep) | (first1 & ~keep);
        have = have1;
      }
      my_new = s.kept_len[c] - have;
    }
    __syncthreads();
    if (half == 0 && c < n_c) {
      s.kept_m[c] = have;
      s.kept_first[c] = first;
    }
    int total_new;
    const int excl = block_exclusive_scan(my_new, s.red, &total_new);  // drafts are threads 0..127
    if (half == 0 && c < n_c) s.kept_base[c] = 1 + excl;
    __syncthreads();
    const int n_nodes = (1 + total_new) < max_nodes ? (1 + total_new) : max_nodes;
    const int W = (max_nodes + 63) / 64;
    int32_t* node_token = p.node_token + (size_t)b * max_nodes;
    int32_t* node_parent = p.node_parent + (size_t)b * max_nodes;
    int32_t* node_depth = p.node_depth + (size_t)b * max_nodes;
    unsigned long long* mask = p.anc_mask + (size_t)b * max_nodes * W;
    if (half == 0 && c < n_c) {
      const int len = s.kept_len[c], m = have, my_base = 1 + excl;
      int par = 0, leaf = -1;
      unsigned long long m0 = 1ull, m1 = 0ull;  // ancestors so far: the root
      for (int d = 0; d < len; ++d) {
        int node;
        if (d < m) {
          const int f = (int)((first >> (8 * d)) & 0xff);
          node = s.kept_base[f] + (d - s.kept_m[f]);
        } else {
          node = my_base + (d - m);
        }
        if (node >= max_nodes) { leaf = -1; break; }
        if (node < 64) m0 |= 1ull << node; else m1 |= 1ull << (node - 64);
        if (d >= m) {
          node_token[node] = s.kept_tok[c][d];
          node_parent[node] = par;
          node_depth[node] = d + 1;
          mask[(size_t)node * W] = m0;
          if (W > 1) mask[(size_t)node * W + 1] = m1;
        }
        par = node;
        leaf = node;
      }
      p.cand_leaf[(size_t)b * beam + c] = leaf;
    }
    for (int cc = tid; cc < beam; cc += kThreads)
      if (cc >= n_c) p.cand_leaf[(size_t)b * beam + cc] = -1;
    for (int i = tid; i < max_nodes; i += kThreads) {
      if (i == 0) {
        node_token[0] = p.root_token[b];
        node_parent[0] = -1;
        node_depth[0] = 0;
        mask[0] = 1ull;
        if (W > 1) mask[1] = 0ull;
      } else if (i >= n_nodes) {
        node_token[i] = -1;
        node_parent[i] = -1;
        node_depth[i] = -1;
        mask[(size_t)i * W] = 0ull;
        if (W > 1) mask[(size_t)i * W + 1] = 0ull;
      }
    }
    if (tid == 0) {
      p.n_cand[b] = n_c;
      p.n_nodes[b] = n_nodes;
    }
  }
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int ctc_collapse_tree(ctcspec_ctx* ctx, const int32_t* topk_id, const float* topk_logp,
                                 const int32_t* root_token, int B, int T, int k, int32_t blank_id, int beam,
                                 int max_nodes, int32_t* n_cand, int32_t* cand_tokens, int32_t* cand_len,
                                 float* cand_score, int32_t* cand_leaf, int32_t* n_nodes, int32_t* node_token,
                                 int32_t* node_parent, int32_t* node_depth, uint64_t* anc_mask) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx,
                  topk_id && topk_logp && root_token && n_cand && cand_tokens && cand_len && cand_score &&
                      cand_leaf && n_nodes && node_token && node_parent && node_depth && anc_mask,
                  CTCSPEC_EINVAL, "ctc_collapse_tree: null pointer");
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && k > 0 && beam > 0 && max_nodes > 0, CTCSPEC_EINVAL,
                  "ctc_collapse_tree: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, T <= CTCSPEC_MAX_SLOTS && k <= CTCSPEC_MAX_TOPK && beam <= CTCSPEC_MAX_BEAM &&
                           max_nodes <= CTCSPEC_MAX_NODES,
                  CTCSPEC_EUNSUPPORTED, "ctc_collapse_tree: T<=%d, k<=%d, beam<=%d, max_nodes<=%d required",
                  CTCSPEC_MAX_SLOTS, CTCSPEC_MAX_TOPK, CTCSPEC_MAX_BEAM, CTCSPEC_MAX_NODES);
  long long total = 1;
  for (int t = 0; t < T; ++t) total *= k;
  CTCSPEC_REQUIRE(ctx, total <= CTCSPEC_MAX_ALIGNMENTS, CTCSPEC_EUNSUPPORTED,
                  "ctc_collapse_tree: k^T=%lld exceeds %d", total, CTCSPEC_MAX_ALIGNMENTS);
  CTCSPEC_REQUIRE(ctx, B <= ctx->lim.max_batch, CTCSPEC_EUNSUPPORTED,
                  "ctc_collapse_tree: B=%d exceeds the context's max_batch=%d", B, ctx->lim.max_batch);

  CollapseParams p;
  p.topk_id = topk_id; p.topk_logp = topk_logp; p.root_token = root_token;
  p.T = T; p.k = k; p.blank_id = blank_id; p.beam = beam; p.max_nodes = max_nodes;
  p.magic = (unsigned int)((0x100000000ull + (unsigned)k - 1) / (unsigned)k);
  p.n_cand = n_cand; p.cand_tokens = cand_tokens; p.cand_len = cand_len; p.cand_score = cand_score;
  p.cand_leaf = cand_leaf; p.n_nodes = n_nodes; p.node_token = node_token; p.node_parent = node_parent;
  p.node_depth = node_depth; p.anc_mask = (unsigned long long*)anc_mask;
  p.ws = ctx->collapse_ws;
  static_assert(sizeof(CollapseShared) <= 160 * 1024, "collapse LDS footprint");
  static_assert(kHalfMax <= 2 * kThreads, "two sorted first-half entries per thread");
  static_assert(CTCSPEC_MAX_BEAM * 2 == kThreads, "tree build maps (draft, half) onto the threads");
  static_assert(CTCSPEC_MAX_SLOTS <= 8 && CTCSPEC_MAX_TOPK <= 8, "half combinations have at most four base-k digits");
  const int lds = (int)sizeof(CollapseShared);
  static bool lds_allowed = false;
  if (!lds_allowed) {
    CTCSPEC_HIP(ctx, hipFuncSetAttribute((const void*)collapse_tree_kernel,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    lds_allowed = true;
  }
  hipLaunchKernelGGL(collapse_tree_kernel, dim3(B), dim3(kThreads), lds, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
