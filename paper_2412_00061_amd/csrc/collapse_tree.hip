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
// The kernel runs on ONE compute unit, so what it costs is dependent LDS round trips and
// instruction count, not bandwidth.  Hence: sorting happens in registers (bitonic network over DPP
// lane exchanges per wavefront, then a rank merge of the wavefronts' runs), independent binary
// searches advance in lockstep, base-k digits come from multiply-high instead of division, and the
// prefix tree is built level by level by a single wavefront with LDS atomics while the other
// wavefronts write the draft arrays.
//
// Sorted candidates live in LDS while they fit (4096) and in the context's global workspace
// otherwise (mass ties, or nearly every raw candidate needed).
#include <type_traits>

#include "topk_merge.h"

namespace ctcspec {

constexpr int kThreads = 256;  // (512 was measured: 3 us slower - the phases are chains of barriers and LDS round trips)
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
  unsigned int magic_n2;  // ceil(2^32 / k^(T/2)): division of a candidate index by the number of second halves
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
  int32_t* node_removed;  // raw layout only
  unsigned char* ws;  // per-sequence global workspace base
  // deferred merge of the draft head (MK > 0): its per-workgroup partials in, the lists that ctc_draft_topk owes out
  const float* lm_pmax;
  const float* lm_psum;
  const unsigned long long* lm_pkey;
  int lm_blocks, lm_stride;
  int32_t* topk_id_out;
  float* topk_logp_out;
  float* lse_out;
};

struct CollapseShared {
  int ids[64];
  float logp[64];
  int code[64];
  float Xv[kHalfMax];  // first-half sums, sorted descending
  int Xi[kHalfMax];    // their rank combination
  float Yv[kHalfMax];
  int Yi[kHalfMax];
  int prefix[kHalfMax + 1];
  int red[kWaves];
  float delta;
  int n_nodes;
  int blank_code;  // raw layout: local code of the blank, -1 if no list holds it
  unsigned long long kept_ck[CTCSPEC_MAX_BEAM];
  int kept_len[CTCSPEC_MAX_BEAM];
  int kept_m[CTCSPEC_MAX_BEAM];
  int kept_base[CTCSPEC_MAX_BEAM];
  unsigned long long keys[kLdsCap];
  unsigned long long ckeys[kLdsCap];
  unsigned int table[2 * kLdsCap];
  unsigned int tree_table[128 * 64];  // (creator of the parent node, token code) -> (level, 127 - draft); zeroed at start
};

// ---- workgroup / wavefront primitives -------------------------------------------------------------
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

// number of binary-search steps that empty an interval of n entries
__device__ __forceinline__ int search_steps(int n) { return n > 0 ? 32 - __builtin_clz((unsigned)n) : 0; }

// Two independent searches in lockstep: number of leading entries i of [0, n) with pred(i), where pred
// is true exactly on a prefix.  Both probes of a step are issued before either result is used, so a
// step costs one LDS round trip.  (Cutting the interval to an eighth per step with seven probes was
// measured: the extra index arithmetic costs more than the saved round trips.)
template <typename P0, typename P1>
__device__ __forceinline__ void prefix_count2(int n, P0 pred0, P1 pred1, int& out0, int& out1) {
  int pos0 = 0, len0 = n, pos1 = 0, len1 = n;
  const int steps = search_steps(n);
  for (int it = 0; it < steps; ++it) {
    const int h0 = len0 >> 1, h1 = len1 >> 1;
    const int m0 = min(pos0 + h0, n - 1), m1 = min(pos1 + h1, n - 1);
    const bool t0 = pred0(m0), t1 = pred1(m1);
    const bool ok0 = len0 > 0 && t0, ok1 = len1 > 0 && t1;
    pos0 = ok0 ? m0 + 1 : pos0;
    len0 = ok0 ? len0 - h0 - 1 : h0;
    pos1 = ok1 ? m1 + 1 : pos1;
    len1 = ok1 ? len1 - h1 - 1 : h1;
  }
  out0 = pos0;
  out1 = pos1;
}

__device__ __forceinline__ unsigned int hash_slot(unsigned long long ck, int log2_size) {
  return (unsigned int)((ck * 0x9E3779B97F4A7C15ull) >> (64 - log2_size));
}

// ---- sorting in LDS / global memory (any size; the slow path) -------------------------------------
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

// ---- sorting in registers (the fast path) -----------------------------------------------------------
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

// Sort keys descending, kThreads*E of them (v[e] is key number tid*E + e on entry).  Every wavefront
// sorts its 64*E keys in registers; the sorted runs of each group of GROUP consecutive wavefronts are
// then merged by rank: position in the own run + number of keys in each other run of the group that
// come first (found by binary search, all searches of a thread in lockstep; equal keys are ordered by
// run).  Group g's result is out[g*GROUP*64*E ...].  runs: LDS scratch of kThreads*E keys.
// Barriers included; `out` is complete on return.
template <int E, int GROUP>
__device__ __forceinline__ void block_sort_desc_fast(unsigned long long (&v)[E], unsigned long long* runs,
                                                     unsigned long long* out, bool ror4_is_up) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int RUN = 64 * E;
  bitonic_sort_upto<E, RUN>(v, lane, ror4_is_up);
#pragma unroll
  for (int e = 0; e < E; ++e) runs[wave * RUN + lane * E + e] = v[e];
  __syncthreads();
  const int group0 = wave & ~(GROUP - 1);  // first wavefront of my group
  int pos[E][GROUP];
#pragma unroll
  for (int e = 0; e < E; ++e)
#pragma unroll
    for (int w = 0; w < GROUP; ++w) pos[e][w] = 0;
  // all keys of run w that come before mine form a prefix of the run; RUN is a power of two
#pragma unroll
  for (int h = RUN / 2; h >= 1; h >>= 1) {
    unsigned long long x[E][GROUP];
#pragma unroll
    for (int e = 0; e < E; ++e)
#pragma unroll
      for (int w = 0; w < GROUP; ++w) x[e][w] = runs[(group0 + w) * RUN + pos[e][w] + h - 1];
#pragma unroll
    for (int e = 0; e < E; ++e)
#pragma unroll
      for (int w = 0; w < GROUP; ++w) {
        const bool before = (group0 + w < wave) ? (x[e][w] >= v[e]) : (x[e][w] > v[e]);
        pos[e][w] += before ? h : 0;
      }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    int rank = lane * E + e;
#pragma unroll
    for (int w = 0; w < GROUP; ++w) {
      const unsigned long long x = runs[(group0 + w) * RUN + pos[e][w]];
      const bool before = (group0 + w < wave) ? (x >= v[e]) : (x > v[e]);
      rank += (group0 + w == wave) ? 0 : pos[e][w] + (before ? 1 : 0);
    }
    out[group0 * RUN + rank] = v[e];
  }
  __syncthreads();
}

// ---- raw candidates ---------------------------------------------------------------------------------
// a / k for 0 <= a < 65536, magic = ceil(2^32 / k)
__device__ __forceinline__ int div_small(int a, unsigned int magic) { return (int)__umulhi((unsigned)a, magic); }

// The rank digits of a half-combination, most significant slot first.  a counts in base k with
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

// left-to-right float32 sum: acc (if have_acc), then the half's slots t0.. in order
__device__ __forceinline__ float add_slots(float acc, bool have_acc, const float* logp, const Digits4& d, int t0,
                                           int nt, int k) {
  float l[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) l[t] = t < nt ? logp[(t0 + t) * k + d.r[t]] : 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
    if (t < nt) acc = (have_acc || t > 0) ? acc + l[t] : l[t];
  return acc;
}

// Collapsed-sequence key of the raw candidate (a, b): 7-bit local token codes, position 0 in the low
// bits, unused positions = kBlankCode.
// RAW: nothing is merged or dropped - the key holds the raw candidate itself (the literal layout of Sec. 3.1).
template <bool RAW>
__device__ __forceinline__ unsigned long long collapse_key(const CollapseShared& s, const Digits4& da,
                                                           const Digits4& db, int T1, int T2, int k, int* len_out) {
  int cd[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const bool first_half = u < 4;
    const int t_in = first_half ? u : u - 4;
    const bool live = first_half ? (t_in < T1) : (t_in < T2);
    const int slot = first_half ? t_in : T1 + t_in;
    const int r = first_half ? da.r[t_in] : db.r[t_in];
    cd[u] = live ? s.code[slot * k + r] : -2;  // -2: slot does not exist
  }
  unsigned long long key = 0x00ffffffffffffffull;
  int len = 0, prev = -1;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const bool emit = RAW ? cd[u] >= 0 : (cd[u] >= 0 && cd[u] != prev && cd[u] != kBlankCode);
    const int sh = 7 * len;
    key = emit ? ((key & ~(0x7full << sh)) | ((unsigned long long)cd[u] << sh)) : key;
    len += emit ? 1 : 0;
    prev = cd[u] >= 0 ? cd[u] : prev;
  }
  *len_out = len;
  return key;
}

// MK > 0: the top-k lists do not exist yet - the draft head left only its per-workgroup partials, and this kernel's
// wavefronts merge them first (two columns each, at most MK keys per list), write the lists out for the caller and
// go on from LDS: one dispatch and one trip through memory fewer than a merge kernel in between.
template <bool RAW, int MK>
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
  // the tree table is cleared by everybody while the first wavefront's loads are in flight
  int id = -1;
  float lp = 0.f;
  if constexpr (MK > 0) {
    static_assert(CTCSPEC_MAX_SLOTS <= 2 * kWaves, "two columns per wavefront cover every slot");
    const int col[2] = {wave < T ? b * T + wave : -1, wave + kWaves < T ? b * T + wave + kWaves : -1};
    float lse[2];
    unsigned long long best[2][MK];
    merge_topk_columns<MK, 2>(p.lm_pmax, p.lm_psum, p.lm_pkey, p.lm_stride, p.lm_blocks, k, col, lse, best);
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (col[c] < 0) continue;
      if (lane == 0 && p.lse_out) p.lse_out[col[c]] = lse[c];
      if (lane < k) {
        unsigned long long key = 0ull;
#pragma unroll
        for (int r = 0; r < MK; ++r) key = lane == r ? best[c][r] : key;
        const int tok = (int)rank_key_index(key);
        const float logp = rank_key_value(key) - lse[c];
        p.topk_id_out[(size_t)col[c] * k + lane] = tok;
        p.topk_logp_out[(size_t)col[c] * k + lane] = logp;
        const int t = col[c] - b * T;
        s.ids[t * k + lane] = tok;
        s.logp[t * k + lane] = logp;
      }
    }
  } else if (wave == 0 && lane < TK) {
    id = p.topk_id[(size_t)b * TK + lane];
    lp = p.topk_logp[(size_t)b * TK + lane];
  }
  for (int i = tid; i < 128 * 64 / 4; i += kThreads) reinterpret_cast<u32x4*>(s.tree_table)[i] = u32x4{0u, 0u, 0u, 0u};
  if constexpr (MK > 0) {
    __syncthreads();  // the merged lists are in LDS
  } else if (wave == 0) {
    if (lane < TK) {
      s.ids[lane] = id;
      s.logp[lane] = lp;
    }
    // the same wavefront reads the lists back below: its LDS operations execute in order, the compiler must not
    // reorder them either
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_wave_barrier();
  }
  if (wave == 0) {
    // local token code = position of the first entry with the same token id.  Every lane scans the lists in LDS
    // (all lanes read the same address: a broadcast), reads batched eight at a time - as a chain of readlane steps
    // this phase cost as much as the sort after it.
    if (MK > 0 && lane < TK) id = s.ids[lane];
    int cd = lane;
#pragma unroll 8
    for (int j = 0; j < TK; ++j) {
      const int idj = s.ids[j];
      cd = (idj == id && j < cd) ? j : cd;
    }
    // delta bounds |fl(X+Y) - exact score|: both are sums of the same T terms, each addition off by
    // at most 2^-24 of a partial sum, partial sums bounded by A = sum_t max_j |logp[t,j]|.
    // 14 * 2^-24 * A would do; 16 * 2^-23 * A leaves room for rounding of the thresholds themselves.
    float mx = 0.f;  // lane t < T: max_j |logp[t,j]|
    if (lane < T)
      for (int j = 0; j < k; ++j) mx = fmaxf(mx, fabsf(s.logp[lane * k + j]));
    float A = 0.f;
#pragma unroll
    for (int t = 0; t < CTCSPEC_MAX_SLOTS; ++t)
      if (t < T) A += __uint_as_float(readlane_u32(__float_as_uint(mx), t));
    if (lane < TK) s.code[lane] = (!RAW && id == p.blank_id) ? kBlankCode : cd;
    if (lane == 0) s.delta = A * (16.0f / 8388608.0f);
    if (RAW) {
      const unsigned long long has = __ballot(lane < TK && id == p.blank_id);
      const int bc = has ? __builtin_amdgcn_readlane(cd, __builtin_ctzll(has)) : -1;
      if (lane == 0) s.blank_code = bc;
    }
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

  // ---- half sums X (slots < T1) and Y (the rest), each sorted descending ---------------------------
  // the lower half of the wavefronts sorts X, the upper half Y: key slot gi belongs to X for gi < kHalfThreads*E
  {
    constexpr int kHalfThreads = kThreads / 2;
    auto sort_halves = [&](auto e_tag) {
      constexpr int E = decltype(e_tag)::value;
      unsigned long long v[E];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int gi = tid * E + e;
        const bool is_x = gi < kHalfThreads * E;
        const int a = is_x ? gi : gi - kHalfThreads * E;
        unsigned long long key = 0ull;
        if (a < (is_x ? n1 : n2)) {
          const Digits4 d = split_digits(a, is_x ? pad1 : pad2, k, magic);
          key = rank_key(add_slots(0.f, false, s.logp, d, is_x ? 0 : T1, is_x ? T1 : T2, k), (unsigned)a);
        }
        v[e] = key;
      }
      block_sort_desc_fast<E, kWaves / 2>(v, s.ckeys, s.keys, ror4_is_up);
      for (int i = tid; i < n1; i += kThreads) {
        s.Xv[i] = rank_key_value(s.keys[i]);
        s.Xi[i] = (int)rank_key_index(s.keys[i]);
      }
      for (int i = tid; i < n2; i += kThreads) {
        s.Yv[i] = rank_key_value(s.keys[kHalfThreads * E + i]);
        s.Yi[i] = (int)rank_key_index(s.keys[kHalfThreads * E + i]);
      }
    };
    const int nmax = n1 > n2 ? n1 : n2;
    static_assert(kHalfMax <= 4 * kHalfThreads, "four half sums per thread cover every half");
    if (nmax <= kHalfThreads) sort_halves(std::integral_constant<int, 1>{});
    else if (nmax <= 2 * kHalfThreads) sort_halves(std::integral_constant<int, 2>{});
    else sort_halves(std::integral_constant<int, 4>{});
    __syncthreads();
  }

  unsigned long long* keys = s.keys;
  unsigned long long* ckeys = s.ckeys;
  unsigned int* table = s.table;
  bool in_lds = true;

  int M = beam;
  int n_d = 0;
  for (;;) {
    if (M > total) M = total;
    const bool final_level = (M >= total);
    float tau_valid = -INFINITY, tau_f = -INFINITY;
    if (!final_level) {
      // X_(i) + Y_(j) with (i+1)(j+1) >= M is passed by at least M raw candidates; every wavefront
      // evaluates all i (j = ceil(M/(i+1)) - 1 = floor((M-1)/(i+1))), so no exchange is needed
      float best = -INFINITY;
      float xs[kHalfMax / 64], ys[kHalfMax / 64];
#pragma unroll
      for (int u = 0; u < kHalfMax / 64; ++u) {  // every probe is requested before the first is used
        const int i = lane + 64 * u;
        int j = (int)((float)(M - 1) / (float)(i + 1));
        j -= (j * (i + 1) > M - 1) ? 1 : 0;
        j += ((j + 1) * (i + 1) <= M - 1) ? 1 : 0;
        const bool on = i < n1 && j < n2;
        xs[u] = s.Xv[on ? i : 0];
        ys[u] = on ? s.Yv[j] : -INFINITY;
      }
#pragma unroll
      for (int u = 0; u < kHalfMax / 64; ++u) best = fmaxf(best, xs[u] + ys[u]);
      const float tau = wave_max_f32(best);
      tau_valid = tau - delta;
      tau_f = tau_valid - delta;
    }
    // survivors per (sorted) first-half combination, prefix sums
    int n_s = 0;
    {
      // kHalfMax <= 2 * kThreads: thread t owns entries 2t and 2t+1
      const int i0 = 2 * tid, i1 = 2 * tid + 1;
      const float x0 = s.Xv[i0 < n1 ? i0 : 0], x1 = s.Xv[i1 < n1 ? i1 : 0];
      int c0, c1;
      prefix_count2(
          n2, [&](int m) { return x0 + s.Yv[m] >= tau_f; }, [&](int m) { return x1 + s.Yv[m] >= tau_f; }, c0, c1);
      c0 = i0 < n1 ? c0 : 0;
      c1 = i1 < n1 ? c1 : 0;
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
    // exact key of a survivor at (row of sorted X, column of sorted Y): the first half's partial sum is
    // exactly the left-to-right prefix of the score
    auto key_at = [&](int row, int col, bool live) -> unsigned long long {
      const int ib = s.Yi[col];
      const Digits4 db = split_digits(ib, pad2, k, magic);
      const float sc = add_slots(s.Xv[row], true, s.logp, db, T1, T2, k);
      return live ? rank_key(sc, (unsigned)(s.Xi[row] * n2 + ib)) : 0ull;
    };
    // keys of survivors i0 and i0+1: their rows are (number of rows starting at or before them) - 1
    auto key_pair = [&](int i0, unsigned long long& k0, unsigned long long& k1) {
      const int i1 = i0 + 1;
      int r0, r1;
      prefix_count2(
          n1, [&](int m) { return s.prefix[m] <= i0; }, [&](int m) { return s.prefix[m] <= i1; }, r0, r1);
      const bool l0 = i0 < n_s, l1 = i1 < n_s;
      r0 = l0 ? r0 - 1 : 0;
      r1 = l1 ? r1 - 1 : 0;
      k0 = key_at(r0, l0 ? i0 - s.prefix[r0] : 0, l0);
      k1 = key_at(r1, l1 ? i1 - s.prefix[r1] : 0, l1);
    };
    auto sort_survivors_fast = [&](auto e_tag) {
      constexpr int E = decltype(e_tag)::value;
      unsigned long long v[E];
#pragma unroll
      for (int e = 0; e < E; e += 2) key_pair(tid * E + e, v[e], v[e + 1]);
      block_sort_desc_fast<E, kWaves>(v, s.ckeys, s.keys, ror4_is_up);
    };
    if (n_s <= 2 * kThreads) {
      sort_survivors_fast(std::integral_constant<int, 2>{});
    } else if (n_s <= 8 * kThreads) {
      sort_survivors_fast(std::integral_constant<int, 8>{});
    } else {
      int P2 = 64;
      while (P2 < n_s) P2 <<= 1;
      for (int i0 = 2 * tid; i0 < P2; i0 += 2 * kThreads) {
        unsigned long long k0, k1;
        key_pair(i0, k0, k1);
        keys[i0] = k0;
        keys[i0 + 1] = k1;
      }
      __syncthreads();
      block_bitonic_sort_desc(keys, P2);
    }

    // The walk is instantiated twice, once on the LDS lists and once on the lists in the global workspace: with
    // one set of pointers that may be either, every access would be a flat instruction.
    auto walk = [&](unsigned long long* keys, unsigned long long* ckeys, unsigned int* table) -> bool {
      // Walk the sorted survivors.  Down to score tau_valid the list is exactly the global order (every
      // raw candidate that good is a survivor); those positions are collapsed and first occurrences are
      // found through a hash table of positions.
      int log2_ts = 6;
      while ((1 << log2_ts) < 2 * n_s) ++log2_ts;
      const int TS = 1 << log2_ts;
      for (int i = tid; i < TS; i += kThreads) table[i] = kEmptySlot;
      for (int i = tid; i < n_s; i += kThreads) {
        const unsigned long long key = keys[i];
        unsigned long long ck = ~0ull;  // ~0: not walked (below tau_valid) or the empty draft
        if (final_level || rank_key_value(key) >= tau_valid) {
          const int idx = (int)rank_key_index(key);
          const int a = n2 == 1 ? idx : (int)__umulhi((unsigned)idx, p.magic_n2), bb = idx - a * n2;  // idx / n2
          int len;
          const unsigned long long c =
              collapse_key<RAW>(s, split_digits(a, pad1, k, magic), split_digits(bb, pad2, k, magic), T1, T2, k, &len);
          ck = len ? c : ~0ull;
        }
        ckeys[i] = ck;
      }
      __syncthreads();
      for (int i = tid; i < n_s; i += kThreads) {
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
      // distinct non-empty drafts in walk order; thread t owns positions [t*per, (t+1)*per)
      const int per = (n_s + kThreads - 1) / kThreads;
      const int i_begin = tid * per, i_end = min(n_s, (tid + 1) * per);
      int first_cnt = 0;
      unsigned int first_bits = 0u;  // flags of my first 32 positions, so that they are not looked up twice
      for (int i = i_begin; i < i_end; ++i) {
        const unsigned long long ck = ckeys[i];
        if (ck == ~0ull) continue;
        unsigned int slot = hash_slot(ck, log2_ts);
        while (ckeys[table[slot]] != ck) slot = (slot + 1) & (TS - 1);
        const bool is_first = table[slot] == (unsigned)i;
        first_cnt += is_first ? 1 : 0;
        if (is_first && i - i_begin < 32) first_bits |= 1u << (i - i_begin);
      }
      const int rank0 = block_exclusive_scan(first_cnt, s.red, &n_d);
      if (n_d >= beam || final_level) {
        int rank = rank0;
        for (int i = i_begin; i < i_end && rank < beam; ++i) {
          const unsigned long long ck = ckeys[i];
          bool is_first;
          if (i - i_begin < 32) {
            is_first = (first_bits >> (i - i_begin)) & 1u;
          } else {
            if (ck == ~0ull) continue;
            unsigned int slot = hash_slot(ck, log2_ts);
            while (ckeys[table[slot]] != ck) slot = (slot + 1) & (TS - 1);
            is_first = table[slot] == (unsigned)i;
          }
          if (!is_first) continue;
          int len = 0;
  #pragma unroll
          for (int d = 0; d < 8; ++d) len += (((ck >> (7 * d)) & 0x7f) != kBlankCode) ? 1 : 0;
          s.kept_ck[rank] = ck;
          s.kept_len[rank] = len;
          p.cand_score[(size_t)b * beam + rank] = rank_key_value(keys[i]);
          ++rank;
        }
        return true;
      }
      return false;
    };
    const bool done = in_lds ? walk(s.keys, s.ckeys, s.table) : walk(keys, ckeys, table);
    if (done) break;
    M *= 4;
    __syncthreads();
  }
  __syncthreads();  // the kept list is complete

  const int n_c = n_d < beam ? n_d : beam;
  const int W = (max_nodes + 63) / 64;
  int32_t* node_token = p.node_token + (size_t)b * max_nodes;
  int32_t* node_parent = p.node_parent + (size_t)b * max_nodes;
  int32_t* node_depth = p.node_depth + (size_t)b * max_nodes;
  unsigned long long* mask = p.anc_mask + (size_t)b * max_nodes * W;

  // The nodes a draft creates are scattered over the node arrays: they are collected in LDS (the hash table of the
  // walk is dead by now) and leave in one coalesced sweep at the end - as scattered global stores of one wavefront,
  // up to 64 separate words per instruction, they took half of the tree phase.
  int* st_tok = reinterpret_cast<int*>(s.table);
  int* st_par = st_tok + CTCSPEC_MAX_NODES;
  int* st_dep = st_par + CTCSPEC_MAX_NODES;
  int* st_rem = st_dep + CTCSPEC_MAX_NODES;
  unsigned long long* st_mask = reinterpret_cast<unsigned long long*>(st_rem + CTCSPEC_MAX_NODES);  // [nodes][2]
  static_assert(CTCSPEC_MAX_NODES * (4 * 4 + 2 * 8) <= sizeof(CollapseShared::table) && CTCSPEC_MAX_NODES % 2 == 0,
                "node staging fits the hash table's LDS");
  if (wave == 0) {
    // ---- prefix tree, by one wavefront; lane l owns drafts l and l+64 --------------------------
    // A node is a distinct draft prefix; it is created by the first (best-ranked) draft that has it.
    // Level by level, drafts announce (creator of their parent node, token code) in a direct-address
    // table with an atomic max of (level, 127 - draft): per entry the current level's smallest draft
    // number wins and is read back as the creator of the draft's node on that level.  LDS operations
    // of one wavefront execute in order, so no barrier is needed between the levels.
    unsigned long long ck[2], creators[2] = {0ull, 0ull};  // byte d-1: creator of my node at depth d
    int len[2], fprev[2] = {0, 0};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + 64 * u;
      ck[u] = c < n_c ? s.kept_ck[c] : 0ull;
      len[u] = c < n_c ? s.kept_len[c] : 0;
    }
    for (int d = 1; d <= T; ++d) {
      unsigned int key[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        key[u] = ((unsigned)fprev[u] << 6) | (unsigned)((ck[u] >> (7 * (d - 1))) & 0x3f);
        if (d <= len[u]) atomicMax(&s.tree_table[key[u]], ((unsigned)d << 8) | (unsigned)(127 - (lane + 64 * u)));
      }
      // every lane's announcements must be issued before any lane reads a winner back: keep the
      // compiler from moving the reads up (the hardware executes a wavefront's LDS operations in order)
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      __builtin_amdgcn_wave_barrier();
      // both winners are read back in one round trip (the keys always lie inside the table, so the reads need no
      // condition; a draft that has ended ignores what it reads)
      unsigned int won[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
        won[u] = __hip_atomic_load(&s.tree_table[key[u]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bool on = d <= len[u];
        fprev[u] = on ? 127 - (int)(won[u] & 0xffu) : fprev[u];
        creators[u] |= on ? (unsigned long long)fprev[u] << (8 * (d - 1)) : 0ull;
      }
    }
    // m = number of leading levels whose node another draft created; my tokens beyond m create nodes,
    // node ids are handed out in (draft, depth) order
    int m[2], excl[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + 64 * u;
      int mm = 0;
#pragma unroll
      for (int d = 0; d < 8; ++d) mm += (d < len[u] && (int)((creators[u] >> (8 * d)) & 0xff) != c) ? 1 : 0;
      m[u] = mm;
    }
    const int inc0 = wave_inclusive_scan_i32(len[0] - m[0]);
    const int tot0 = __builtin_amdgcn_readlane(inc0, 63);
    const int inc1 = wave_inclusive_scan_i32(len[1] - m[1]);
    const int total_new = tot0 + __builtin_amdgcn_readlane(inc1, 63);
    excl[0] = inc0 - (len[0] - m[0]);
    excl[1] = tot0 + inc1 - (len[1] - m[1]);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + 64 * u;
      if (c < n_c) {
        s.kept_m[c] = m[u];
        s.kept_base[c] = 1 + excl[u];
      }
    }
    const int n_nodes = (1 + total_new) < max_nodes ? (1 + total_new) : max_nodes;
    if (lane == 0) {
      s.n_nodes = n_nodes;
      p.n_cand[b] = n_c;
      p.n_nodes[b] = n_nodes;
    }
    // Every draft walks its path once: node id, token, ancestors of each level.  All LDS lookups of both drafts are
    // requested up front and the walk is free of branches (node ids grow along a path, so "this level's node
    // exists" already implies it for the levels above): as a loop with an early exit per level it waited for one
    // LDS round trip per level.
    int path_node[2][8], path_tok[2][8];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        const int f = d < len[u] ? (int)((creators[u] >> (8 * d)) & 0xff) : 0;
        path_node[u][d] = s.kept_base[f] + (d - s.kept_m[f]);
        path_tok[u][d] = s.ids[(int)((ck[u] >> (7 * d)) & 0x7f) & 63];
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + 64 * u;
      int par = 0, leaf = 0;
      bool whole = true;  // every level of the draft has its node (none cut by the node cap)
      unsigned long long m0 = 1ull, m1 = 0ull;  // ancestors so far: the root
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        const int f = (int)((creators[u] >> (8 * d)) & 0xff);
        const int node = path_node[u][d];
        const bool level = c < n_c && d < len[u];
        const bool exists = level && node < max_nodes;
        whole = whole && (!level || exists);
        // raw layout: a blank, or a token equal to the raw token right before it, is removed by the CTC transform -
        // it sees its own prefix but nothing below it sees it
        const int code = (int)((ck[u] >> (7 * d)) & 0x7f);
        const bool removed = RAW && (code == s.blank_code || (d > 0 && code == (int)((ck[u] >> (7 * (d - 1))) & 0x7f)));
        const unsigned long long b0 = node < 64 ? 1ull << (node & 63) : 0ull, b1 = node < 64 ? 0ull : 1ull << (node & 63);
        if (exists && f == c) {
          st_tok[node] = path_tok[u][d];
          st_par[node] = par;
          st_dep[node] = d + 1;
          st_mask[2 * node] = m0 | b0;
          st_mask[2 * node + 1] = m1 | b1;
          if (RAW) st_rem[node] = removed ? 1 : 0;
        }
        if (exists && !removed) { m0 |= b0; m1 |= b1; }
        par = exists ? node : par;
        leaf = exists ? node : leaf;
      }
      if (c < n_c) p.cand_leaf[(size_t)b * beam + c] = (whole && len[u] > 0) ? leaf : -1;
    }
  } else {
    // ---- draft arrays, by the other wavefronts ----------------------------------------------------
    for (int i = tid - 64; i < beam * 8; i += kThreads - 64) {
      const int c = i >> 3, d = i & 7;
      if (d < T) {
        int tok = -1;
        if (c < n_c && d < s.kept_len[c]) tok = s.ids[(int)((s.kept_ck[c] >> (7 * d)) & 0x7f)];
        p.cand_tokens[((size_t)b * beam + c) * T + d] = tok;
      }
    }
    for (int c = tid - 64; c < beam; c += kThreads - 64) {
      p.cand_len[(size_t)b * beam + c] = c < n_c ? s.kept_len[c] : 0;
      if (c >= n_c) {
        p.cand_score[(size_t)b * beam + c] = -INFINITY;
        p.cand_leaf[(size_t)b * beam + c] = -1;
      }
    }
  }
  __syncthreads();
  const int n_nodes = s.n_nodes;
  for (int i = tid; i < max_nodes; i += kThreads) {
    if (i == 0) {
      node_token[0] = p.root_token[b];
      node_parent[0] = -1;
      node_depth[0] = 0;
      mask[0] = 1ull;
      if (W > 1) mask[1] = 0ull;
      if (RAW) p.node_removed[(size_t)b * max_nodes] = 0;
    } else if (i < n_nodes) {
      node_token[i] = st_tok[i];
      node_parent[i] = st_par[i];
      node_depth[i] = st_dep[i];
      mask[(size_t)i * W] = st_mask[2 * i];
      if (W > 1) mask[(size_t)i * W + 1] = st_mask[2 * i + 1];
      if (RAW) p.node_removed[(size_t)b * max_nodes + i] = st_rem[i];
    } else {
      if (RAW) p.node_removed[(size_t)b * max_nodes + i] = -1;
      node_token[i] = -1;
      node_parent[i] = -1;
      node_depth[i] = -1;
      mask[(size_t)i * W] = 0ull;
      if (W > 1) mask[(size_t)i * W + 1] = 0ull;
    }
  }
}

// the deferred merge is built into the kernel for lists of up to this many keys (the workloads' k = 4)
constexpr int kFusedMergeK = 4;

hipError_t prepare_collapse_tree() {
  const int lds = (int)sizeof(CollapseShared);
  hipError_t e = hipFuncSetAttribute((const void*)collapse_tree_kernel<false, 0>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess)
    e = hipFuncSetAttribute((const void*)collapse_tree_kernel<true, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess)
    e = hipFuncSetAttribute((const void*)collapse_tree_kernel<false, kFusedMergeK>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  return e;
}

}  // namespace ctcspec

using namespace ctcspec;

static int collapse_tree_call(ctcspec_ctx* ctx, const char* name, bool raw, const int32_t* topk_id, const float* topk_logp,
                              const int32_t* root_token, int B, int T, int k, int32_t blank_id, int beam,
                              int max_nodes, int32_t* n_cand, int32_t* cand_tokens, int32_t* cand_len,
                              float* cand_score, int32_t* cand_leaf, int32_t* n_nodes, int32_t* node_token,
                              int32_t* node_parent, int32_t* node_depth, uint64_t* anc_mask, int32_t* node_removed) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx,
                  topk_id && topk_logp && root_token && n_cand && cand_tokens && cand_len && cand_score &&
                      cand_leaf && n_nodes && node_token && node_parent && node_depth && anc_mask &&
                      (!raw || node_removed),
                  CTCSPEC_EINVAL, "%s: null pointer", name);
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && k > 0 && beam > 0 && max_nodes > 0, CTCSPEC_EINVAL,
                  "%s: sizes must be positive", name);
  CTCSPEC_REQUIRE(ctx, T <= CTCSPEC_MAX_SLOTS && k <= CTCSPEC_MAX_TOPK && beam <= CTCSPEC_MAX_BEAM &&
                           max_nodes <= CTCSPEC_MAX_NODES,
                  CTCSPEC_EUNSUPPORTED, "%s: T<=%d, k<=%d, beam<=%d, max_nodes<=%d required", name,
                  CTCSPEC_MAX_SLOTS, CTCSPEC_MAX_TOPK, CTCSPEC_MAX_BEAM, CTCSPEC_MAX_NODES);
  long long total = 1;
  for (int t = 0; t < T; ++t) total *= k;
  CTCSPEC_REQUIRE(ctx, total <= CTCSPEC_MAX_ALIGNMENTS, CTCSPEC_EUNSUPPORTED,
                  "%s: k^T=%lld exceeds %d", name, total, CTCSPEC_MAX_ALIGNMENTS);
  CTCSPEC_REQUIRE(ctx, B <= ctx->lim.max_batch, CTCSPEC_EUNSUPPORTED,
                  "%s: B=%d exceeds the context's max_batch=%d", name, B, ctx->lim.max_batch);

  CollapseParams p;
  p.topk_id = topk_id; p.topk_logp = topk_logp; p.root_token = root_token;
  p.T = T; p.k = k; p.blank_id = blank_id; p.beam = beam; p.max_nodes = max_nodes;
  p.magic = (unsigned int)((0x100000000ull + (unsigned)k - 1) / (unsigned)k);
  {
    unsigned long long n2 = 1;
    for (int t = 0; t < T / 2; ++t) n2 *= (unsigned)k;  // T2 = T - ceil(T/2) = floor(T/2)
    p.magic_n2 = n2 == 1 ? 0u : (unsigned int)((0x100000000ull + n2 - 1) / n2);  // n2 == 1: not used
  }
  p.n_cand = n_cand; p.cand_tokens = cand_tokens; p.cand_len = cand_len; p.cand_score = cand_score;
  p.cand_leaf = cand_leaf; p.n_nodes = n_nodes; p.node_token = node_token; p.node_parent = node_parent;
  p.node_depth = node_depth; p.anc_mask = (unsigned long long*)anc_mask; p.node_removed = node_removed;
  p.ws = ctx->collapse_ws;
  static_assert(sizeof(CollapseShared) <= 160 * 1024, "collapse LDS footprint");
  static_assert(kHalfMax <= 2 * kThreads, "two sorted first-half entries per thread");
  static_assert(CTCSPEC_MAX_BEAM <= 128, "the tree build keeps two drafts per lane of one wavefront");
  static_assert(CTCSPEC_MAX_SLOTS <= 8 && CTCSPEC_MAX_TOPK <= 8, "half combinations have at most four base-k digits");
  static_assert(CTCSPEC_MAX_SLOTS * CTCSPEC_MAX_TOPK <= 64, "token codes fit 6 bits; the top-k lists fit one wavefront");
  static_assert(CTCSPEC_MAX_BEAM <= 128 && CTCSPEC_MAX_SLOTS * CTCSPEC_MAX_TOPK <= 64, "direct-address table of (creator, code) pairs");
  const int lds = (int)sizeof(CollapseShared);
  // A deferred ctc_draft_topk call may still owe its lists.  If they are the very lists given here, this launch
  // settles the debt itself (the kernel merges the draft head's partials first and writes the lists out);
  // otherwise the merge kernel runs now.
  bool fused = false;
  if (ctx->lm_pending) {
    if (!raw && ctx->lm_owed.topk_id == topk_id && ctx->lm_owed.topk_logp == topk_logp && ctx->lm_owed.BT == B * T &&
        ctx->lm_owed.k == k && k <= kFusedMergeK) {
      fused = true;
      ctx->lm_pending = 0;
    } else if (const int owed = flush_deferred(ctx)) {
      return owed;
    }
  }
  p.lm_pmax = nullptr; p.lm_psum = nullptr; p.lm_pkey = nullptr; p.lm_blocks = 0; p.lm_stride = 0;
  p.topk_id_out = nullptr; p.topk_logp_out = nullptr; p.lse_out = nullptr;
  if (fused) {
    p.lm_pmax = ctx->lm_pmax; p.lm_psum = ctx->lm_psum; p.lm_pkey = ctx->lm_pkey; p.lm_blocks = ctx->lm_owed.n_blocks;
    p.lm_stride = ctx->lm_max_blocks;
    p.topk_id_out = ctx->lm_owed.topk_id; p.topk_logp_out = ctx->lm_owed.topk_logp; p.lse_out = ctx->lm_owed.lse;
    hipLaunchKernelGGL((collapse_tree_kernel<false, kFusedMergeK>), dim3(B), dim3(kThreads), lds, ctx->stream, p);
  } else if (raw) {
    hipLaunchKernelGGL((collapse_tree_kernel<true, 0>), dim3(B), dim3(kThreads), lds, ctx->stream, p);
  } else {
    hipLaunchKernelGGL((collapse_tree_kernel<false, 0>), dim3(B), dim3(kThreads), lds, ctx->stream, p);
  }
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}

extern "C" int ctc_collapse_tree(ctcspec_ctx* ctx, const int32_t* topk_id, const float* topk_logp,
                                 const int32_t* root_token, int B, int T, int k, int32_t blank_id, int beam,
                                 int max_nodes, int32_t* n_cand, int32_t* cand_tokens, int32_t* cand_len,
                                 float* cand_score, int32_t* cand_leaf, int32_t* n_nodes, int32_t* node_token,
                                 int32_t* node_parent, int32_t* node_depth, uint64_t* anc_mask) {
  return collapse_tree_call(ctx, "ctc_collapse_tree", false, topk_id, topk_logp, root_token, B, T, k, blank_id, beam,
                            max_nodes, n_cand, cand_tokens, cand_len, cand_score, cand_leaf, n_nodes, node_token,
                            node_parent, node_depth, anc_mask, nullptr);
}

extern "C" int ctc_raw_tree(ctcspec_ctx* ctx, const int32_t* topk_id, const float* topk_logp,
                            const int32_t* root_token, int B, int T, int k, int32_t blank_id, int beam, int max_nodes,
                            int32_t* n_cand, int32_t* cand_tokens, int32_t* cand_len, float* cand_score,
                            int32_t* cand_leaf, int32_t* n_nodes, int32_t* node_token, int32_t* node_parent,
                            int32_t* node_depth, uint64_t* anc_mask, int32_t* node_removed) {
  return collapse_tree_call(ctx, "ctc_raw_tree", true, topk_id, topk_logp, root_token, B, T, k, blank_id, beam,
                            max_nodes, n_cand, cand_tokens, cand_len, cand_score, cand_leaf, n_nodes, node_token,
                            node_parent, node_depth, anc_mask, node_removed);
}
