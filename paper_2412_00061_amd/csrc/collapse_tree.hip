// ctc_collapse_tree: raw candidates -> CTC collapse -> dedupe -> best `beam` drafts -> prefix tree + mask.
//
// One workgroup of 1024 threads per sequence.  The k^T raw candidates are never all materialised.
// Raw-candidate scores are sums over slots, so the slots are split in two halves with n1 and n2
// combinations; with the second half's partial sums sorted, "how many raw candidates score at least
// tau" is n1 binary searches.  A bisection on tau finds a threshold that at least M raw candidates
// pass; those (a few hundred) are expanded, given their exact float32 left-to-right score, sorted by
// (score desc, idx asc) and walked in that order: collapse, drop empties, keep first occurrences.
// If fewer than `beam` distinct drafts turn up, M is quadrupled and the level is redone; the last
// level takes every raw candidate.  The half-sum score used for thresholding differs from the exact
// left-to-right sum only by rounding; a margin delta on the threshold makes the walked prefix exactly
// the global order (see `delta` below).
//
// Buffers for the sorted candidates live in LDS while they fit (4096 entries) and in the context's
// global workspace otherwise (mass ties / nearly everything needed).
#include "common.h"

namespace ctcspec {

constexpr int kThreads = 1024;
constexpr int kHalfMax = 512;   // k^ceil(T/2) <= 8^3
constexpr int kLdsCap = 4096;   // sorted candidates kept in LDS
constexpr int kBlankCode = 127; // 7-bit local code of the blank / padding
constexpr unsigned int kEmptySlot = 0xffffffffu;

struct CollapseParams {
  const int32_t* topk_id;
  const float* topk_logp;
  const int32_t* root_token;
  int T, k, blank_id, beam, max_nodes;
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
  int pow_k[CTCSPEC_MAX_SLOTS + 1];
  float X[kHalfMax];
  float Ys[kHalfMax];
  int Yi[kHalfMax];
  int prefix[kHalfMax + 1];
  int red[32];
  int bcast[4];
  unsigned long long kept_ck[CTCSPEC_MAX_BEAM];
  int kept_len[CTCSPEC_MAX_BEAM];
  int kept_tok[CTCSPEC_MAX_BEAM][CTCSPEC_MAX_SLOTS];
  int kept_m[CTCSPEC_MAX_BEAM];
  int kept_base[CTCSPEC_MAX_BEAM];
  int nodeid[CTCSPEC_MAX_BEAM][CTCSPEC_MAX_SLOTS];
  int parent[CTCSPEC_MAX_NODES];
  unsigned long long keys[kLdsCap];
  unsigned long long ckeys[kLdsCap];
  unsigned int table[2 * kLdsCap];
};

__device__ __forceinline__ int block_sum(int v, int* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_sum_i32(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) s += red[w];
  return s;
}

// exclusive prefix of v over the workgroup's threads (thread order), total in *total
__device__ __forceinline__ int block_exclusive_scan(int v, int* red, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  __syncthreads();
  if (lane == 63) red[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    int x = red[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

// number of second-half combinations j (sorted descending) with fl(x + Ys[j]) >= tau
__device__ __forceinline__ int count_ge(float x, const float* Ys, int n2, float tau) {
  int lo = 0, hi = n2;  // invariant: entries < lo pass, entries >= hi fail
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (x + Ys[mid] >= tau) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// exact score of raw candidate idx: float32 sum over slots, left to right
__device__ __forceinline__ float exact_score(const CollapseShared& s, int idx, int T, int k) {
  float acc = 0.f;
  for (int t = 0; t < T; ++t) {
    int r = (idx / s.pow_k[T - 1 - t]) % k;
    float l = s.logp[t * k + r];
    acc = (t == 0) ? l : acc + l;
  }
  return acc;
}

// collapsed-sequence key of raw candidate idx: 7-bit local token codes, position 0 in the low bits,
// unused positions = kBlankCode.  Optionally writes the collapsed token ids.
__device__ __forceinline__ unsigned long long collapse_key(const CollapseShared& s, int idx, int T, int k,
                                                           int* len_out, int* tok_out) {
  unsigned long long key = 0x00ffffffffffffffull;
  int len = 0, prev = -1;
  for (int t = 0; t < T; ++t) {
    int r = (idx / s.pow_k[T - 1 - t]) % k;
    int cd = s.code[t * k + r];
    if (cd != prev && cd != kBlankCode) {
      key &= ~(0x7full << (7 * len));
      key |= (unsigned long long)cd << (7 * len);
      if (tok_out) tok_out[len] = s.ids[t * k + r];
      ++len;
    }
    prev = cd;
  }
  *len_out = len;
  return key;
}

__device__ __forceinline__ unsigned int hash_slot(unsigned long long ck, int log2_size) {
  return (unsigned int)((ck * 0x9E3779B97F4A7C15ull) >> (64 - log2_size));
}

// descending bitonic sort of n (power of two) keys by the whole workgroup
__device__ void block_bitonic_sort_desc(unsigned long long* keys, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = threadIdx.x; t < (n >> 1); t += kThreads) {
        int i = ((t / stride) * stride << 1) + (t % stride);
        int j = i + stride;
        bool desc = (i & size) == 0;
        unsigned long long a = keys[i], b = keys[j];
        if ((a < b) == desc) { keys[i] = b; keys[j] = a; }
      }
      __syncthreads();
    }
  }
}

__global__ __launch_bounds__(kThreads) void collapse_tree_kernel(CollapseParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  CollapseShared& s = *reinterpret_cast<CollapseShared*>(smem_raw);
  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const int T = p.T, k = p.k, TK = p.T * p.k;
  const int beam = p.beam, max_nodes = p.max_nodes;

  if (tid < TK) {
    s.ids[tid] = p.topk_id[(size_t)b * TK + tid];
    s.logp[tid] = p.topk_logp[(size_t)b * TK + tid];
  }
  if (tid == 0) {
    int pw = 1;
    for (int t = 0; t <= T; ++t) { s.pow_k[t] = pw; pw *= k; }
  }
  __syncthreads();
  if (tid < TK) {
    int cd = tid;
    for (int j = 0; j < tid; ++j)
      if (s.ids[j] == s.ids[tid]) { cd = j; break; }
    s.code[tid] = (s.ids[tid] == p.blank_id) ? kBlankCode : cd;
  }
  const int T1 = (T + 1) >> 1, T2 = T - T1;
  const int n1 = s.pow_k[T1], n2 = s.pow_k[T2];
  const int total = s.pow_k[T];

  // delta bounds |half-sum score - exact score|: both are sums of the same T terms, each addition
  // off by at most 2^-24 of a partial sum, partial sums bounded by A = sum_t max_j |logp[t,j]|.
  // 14 * 2^-24 * A would do; 16 * 2^-23 * A leaves room for rounding of the thresholds themselves.
  float A = 0.f;
  for (int t = 0; t < T; ++t) {
    float mx = 0.f;
    for (int j = 0; j < k; ++j) mx = fmaxf(mx, fabsf(s.logp[t * k + j]));
    A += mx;
  }
  const float delta = A * (16.0f / 8388608.0f);

  // half sums
  if (tid < n1) {
    float acc = 0.f;
    for (int t = 0; t < T1; ++t) {
      int r = (tid / s.pow_k[T1 - 1 - t]) % k;
      float l = s.logp[t * k + r];
      acc = (t == 0) ? l : acc + l;
    }
    s.X[tid] = acc;
  }
  {
    // second-half sums sorted descending (ties: smaller index first) through the key buffer
    int n2p = 64;
    while (n2p < n2) n2p <<= 1;
    for (int i = tid; i < n2p; i += kThreads) {
      unsigned long long key = 0ull;
      if (i < n2) {
        float acc = 0.f;
        for (int t = 0; t < T2; ++t) {
          int r = (i / s.pow_k[T2 - 1 - t]) % k;
          float l = s.logp[(T1 + t) * k + r];
          acc = (t == 0) ? l : acc + l;
        }
        key = rank_key(acc, (unsigned)i);
      }
      s.keys[i] = key;
    }
    __syncthreads();
    block_bitonic_sort_desc(s.keys, n2p);
    if (tid < n2) {
      s.Ys[tid] = rank_key_value(s.keys[tid]);
      s.Yi[tid] = (int)rank_key_index(s.keys[tid]);
    }
    __syncthreads();
  }

  unsigned long long* keys = s.keys;
  unsigned long long* ckeys = s.ckeys;
  unsigned int* table = s.table;
  bool in_lds = true;

  int M = 2 * beam < 64 ? 64 : 2 * beam;
  int n_v = 0, n_d = 0, log2_ts = 6;
  for (;;) {
    if (M > total) M = total;
    const bool final_level = (M >= total);
    float tau_valid = -INFINITY, tau_f = -INFINITY;
    if (!final_level) {
      // extremes of the half sums
      float xmax = -INFINITY, xmin = INFINITY;
      for (int a = 0; a < n1; ++a) { xmax = fmaxf(xmax, s.X[a]); xmin = fminf(xmin, s.X[a]); }
      unsigned int lo = float_to_ordered(xmin + s.Ys[n2 - 1]);
      unsigned int hi = float_to_ordered(xmax + s.Ys[0]) + 1u;
      int c_lo = total;
      while (hi - lo > 1u && c_lo > 2 * M) {
        unsigned int mid = lo + ((hi - lo) >> 1);
        float tau = ordered_to_float(mid);
        int c = block_sum(tid < n1 ? count_ge(s.X[tid], s.Ys, n2, tau) : 0, s.red);
        if (c >= M) { lo = mid; c_lo = c; } else hi = mid;
      }
      float tau = ordered_to_float(lo);
      tau_valid = tau - delta;
      tau_f = tau_valid - delta;
    }
    // survivors per first-half combination, prefix sums
    int cnt = tid < n1 ? count_ge(s.X[tid], s.Ys, n2, tau_f) : 0;
    int n_s;
    int excl = block_exclusive_scan(cnt, s.red, &n_s);
    if (tid < n1) s.prefix[tid] = excl;
    if (tid == 0) s.prefix[n1] = n_s;
    if (in_lds && n_s > kLdsCap) {
      in_lds = false;
      keys = reinterpret_cast<unsigned long long*>(p.ws + (size_t)b * kCollapseWsBytesPerSeq);
      ckeys = keys + kMaxAlign;
      table = reinterpret_cast<unsigned int*>(ckeys + kMaxAlign);
    }
    __syncthreads();
    int P2 = 64;
    while (P2 < n_s) P2 <<= 1;
    for (int i = tid; i < P2; i += kThreads) {
      unsigned long long key = 0ull;
      if (i < n_s) {
        int lo_a = 0, hi_a = n1;  // largest a with prefix[a] <= i
        while (hi_a - lo_a > 1) {
          int mid = (lo_a + hi_a) >> 1;
          if (s.prefix[mid] <= i) lo_a = mid; else hi_a = mid;
        }
        int idx = lo_a * n2 + s.Yi[i - s.prefix[lo_a]];
        key = rank_key(exact_score(s, idx, T, k), (unsigned)idx);
      }
      keys[i] = key;
    }
    __syncthreads();
    block_bitonic_sort_desc(keys, P2);

    // the prefix that is exactly the global (score desc, idx asc) order
    {
      int c = 0;
      for (int i = tid; i < n_s; i += kThreads) c += (rank_key_value(keys[i]) >= tau_valid) ? 1 : 0;
      n_v = final_level ? n_s : block_sum(c, s.red);
    }
    // collapse every walked candidate and find first occurrences through a hash table of positions
    log2_ts = 6;
    while ((1 << log2_ts) < 2 * n_v) ++log2_ts;
    const int TS = 1 << log2_ts;
    for (int i = tid; i < TS; i += kThreads) table[i] = kEmptySlot;
    for (int i = tid; i < n_v; i += kThreads) {
      int len;
      unsigned long long ck = collapse_key(s, (int)rank_key_index(keys[i]), T, k, &len, nullptr);
      ckeys[i] = len ? ck : ~0ull;  // ~0 marks the empty draft (no real key has the top byte set)
    }
    __syncthreads();
    for (int i = tid; i < n_v; i += kThreads) {
      unsigned long long ck = ckeys[i];
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
      unsigned long long ck = ckeys[i];
      if (ck == ~0ull) continue;
      unsigned int slot = hash_slot(ck, log2_ts);
      while (ckeys[table[slot]] != ck) slot = (slot + 1) & (TS - 1);
      first_cnt += (table[slot] == (unsigned)i) ? 1 : 0;
    }
    int rank0 = block_exclusive_scan(first_cnt, s.red, &n_d);
    if (n_d >= beam || final_level) {
      // write the kept drafts (rank < beam)
      int rank = rank0;
      for (int i = tid * per; i < (tid + 1) * per && i < n_v && rank < beam; ++i) {
        unsigned long long ck = ckeys[i];
        if (ck == ~0ull) continue;
        unsigned int slot = hash_slot(ck, log2_ts);
        while (ckeys[table[slot]] != ck) slot = (slot + 1) & (TS - 1);
        if (table[slot] != (unsigned)i) continue;
        int len;
        int idx = (int)rank_key_index(keys[i]);
        collapse_key(s, idx, T, k, &len, s.kept_tok[rank]);
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
    int c = i / T, d = i % T;
    p.cand_tokens[(size_t)b * beam * T + i] = (c < n_c && d < s.kept_len[c]) ? s.kept_tok[c][d] : -1;
  }
  for (int c = tid; c < beam; c += kThreads) {
    p.cand_len[(size_t)b * beam + c] = c < n_c ? s.kept_len[c] : 0;
    if (c >= n_c) p.cand_score[(size_t)b * beam + c] = -INFINITY;
    s.kept_m[c] = 0;
  }
  __syncthreads();

  // ---- prefix tree --------------------------------------------------------------------------------
  // m[c] = longest prefix draft c shares with an earlier draft; its tokens beyond m[c] create nodes.
  for (int i = tid; i < n_c * n_c; i += kThreads) {
    int c = i / n_c, c2 = i % n_c;
    if (c2 < c) {
      int lcp = __builtin_ctzll(s.kept_ck[c] ^ s.kept_ck[c2]) / 7;
      atomicMax(&s.kept_m[c], lcp);
    }
  }
  __syncthreads();
  if (tid < n_c) {
    int base = 1;
    for (int c = 0; c < tid; ++c) base += s.kept_len[c] - s.kept_m[c];
    s.kept_base[tid] = base;
  }
  __syncthreads();
  int total_nodes = 1;
  if (n_c > 0) total_nodes = s.kept_base[n_c - 1] + s.kept_len[n_c - 1] - s.kept_m[n_c - 1];
  const int n_nodes = total_nodes < max_nodes ? total_nodes : max_nodes;
  // node of draft c's prefix of length d+1: created by the first draft f <= c sharing that prefix
  for (int i = tid; i < n_c * T; i += kThreads) {
    int c = i / T, d = i % T;
    int node = -1;
    if (d < s.kept_len[c]) {
      int f = c;
      for (int c2 = 0; c2 < c; ++c2) {
        int lcp = __builtin_ctzll(s.kept_ck[c] ^ s.kept_ck[c2]) / 7;
        if (lcp >= d + 1) { f = c2; break; }
      }
      node = s.kept_base[f] + (d - s.kept_m[f]);
      if (node >= max_nodes) node = -1;
    }
    s.nodeid[c][d] = node;
  }
  for (int i = tid; i < max_nodes; i += kThreads) s.parent[i] = -1;
  __syncthreads();
  int32_t* node_token = p.node_token + (size_t)b * max_nodes;
  int32_t* node_parent = p.node_parent + (size_t)b * max_nodes;
  int32_t* node_depth = p.node_depth + (size_t)b * max_nodes;
  for (int i = tid; i < n_c * T; i += kThreads) {
    int c = i / T, d = i % T;
    if (d < s.kept_len[c] && d >= s.kept_m[c]) {  // this draft created the node
      int node = s.nodeid[c][d];
      if (node >= 0) {
        int par = d == 0 ? 0 : s.nodeid[c][d - 1];
        node_token[node] = s.kept_tok[c][d];
        node_parent[node] = par;
        node_depth[node] = d + 1;
        s.parent[node] = par;
      }
    }
  }
  for (int i = tid; i < max_nodes; i += kThreads) {
    if (i == 0) {
      node_token[0] = p.root_token[b];
      node_parent[0] = -1;
      node_depth[0] = 0;
    } else if (i >= n_nodes) {
      node_token[i] = -1;
      node_parent[i] = -1;
      node_depth[i] = -1;
    }
  }
  for (int c = tid; c < beam; c += kThreads)
    p.cand_leaf[(size_t)b * beam + c] = c < n_c ? s.nodeid[c][s.kept_len[c] - 1] : -1;
  if (tid == 0) {
    p.n_cand[b] = n_c;
    p.n_nodes[b] = n_nodes;
  }
  __syncthreads();
  // ancestor mask
  const int W = (max_nodes + 63) / 64;
  for (int i = tid; i < max_nodes; i += kThreads) {
    unsigned long long m0 = 0ull, m1 = 0ull;
    if (i < n_nodes) {
      int j = i;
      while (j >= 0) {
        if (j < 64) m0 |= 1ull << j; else m1 |= 1ull << (j - 64);
        j = s.parent[j];
      }
    }
    unsigned long long* row = p.anc_mask + ((size_t)b * max_nodes + i) * W;
    row[0] = m0;
    if (W > 1) row[1] = m1;
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
  p.n_cand = n_cand; p.cand_tokens = cand_tokens; p.cand_len = cand_len; p.cand_score = cand_score;
  p.cand_leaf = cand_leaf; p.n_nodes = n_nodes; p.node_token = node_token; p.node_parent = node_parent;
  p.node_depth = node_depth; p.anc_mask = (unsigned long long*)anc_mask;
  p.ws = ctx->collapse_ws;
  static_assert(sizeof(CollapseShared) <= 160 * 1024, "collapse LDS footprint");
  const int lds = (int)sizeof(CollapseShared);
  CTCSPEC_HIP(ctx, hipFuncSetAttribute((const void*)collapse_tree_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  hipLaunchKernelGGL(collapse_tree_kernel, dim3(B), dim3(kThreads), lds, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
