// Merge of the draft head's per-workgroup partial results into lse / top-k of a column (Sec. 3.2: log-softmax over
// the vocabulary plus the blank; Sec. 3.3: the k most probable symbols of every slot).  Used by the small merge kernel
// of ctc_draft_topk and, when the merge is deferred, by the prologue of the collapse/tree kernel - one piece of
// code, so both produce the same bits.
#pragma once

#include "common.h"

namespace ctcspec {

// Sorted (descending) register list of the best keys seen by one lane.
template <int KMAX>
struct KeyList {
  unsigned long long v[KMAX];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int i = 0; i < KMAX; ++i) v[i] = 0ull;
  }
  __device__ __forceinline__ void insert(unsigned long long key) {
#pragma unroll
    for (int i = 0; i < KMAX; ++i) {
      unsigned long long hi = key > v[i] ? key : v[i];
      unsigned long long lo = key > v[i] ? v[i] : key;
      v[i] = hi;
      key = lo;
    }
  }
  __device__ __forceinline__ void pop() {
#pragma unroll
    for (int i = 0; i + 1 < KMAX; ++i) v[i] = v[i + 1];
    v[KMAX - 1] = 0ull;
  }
};

// Key-wise maximum / compare-exchange on 64-bit keys.
__device__ __forceinline__ unsigned long long key_max(unsigned long long a, unsigned long long b) { return a > b ? a : b; }
__device__ __forceinline__ void key_sort2(unsigned long long& a, unsigned long long& b) {  // a >= b afterwards
  const unsigned long long hi = a > b ? a : b, lo = a > b ? b : a;
  a = hi;
  b = lo;
}

// The KMAX best of two descending lists of KMAX keys each, descending, into a.  The i-th best of a against the
// i-th worst of b leaves the KMAX largest of the union as a bitonic sequence; a merge network sorts it.
template <int KMAX>
__device__ __forceinline__ void merge_sorted_lists(unsigned long long (&a)[KMAX], const unsigned long long (&b)[KMAX]) {
#pragma unroll
  for (int i = 0; i < KMAX; ++i) a[i] = key_max(a[i], b[KMAX - 1 - i]);
#pragma unroll
  for (int stride = KMAX / 2; stride >= 1; stride >>= 1)
#pragma unroll
    for (int i = 0; i < KMAX; ++i)
      if ((i & stride) == 0) key_sort2(a[i], a[i + stride]);
}

// One wavefront merges NC columns at once (col[c] < 0: none).  The partials are [column][workgroup] arrays of pstride
// workgroups per column, every workgroup's keys in descending order.  Lane l owns workgroups l, l+64, ...; all of a
// lane's partials, of all NC columns, are requested before any is used, so the merge costs about one memory round
// trip.  A lane merges its workgroups' lists list by list (they are sorted: a merge network, not insertions); the
// wavefront's k best then come off the heads of the lanes' lists, one wavefront-wide maximum per key.
// On return every lane holds lse[c] and, best key first, the k best (logit, id) keys of column col[c] in best[c][0..k).
template <int KMAX, int NC>
__device__ __forceinline__ void merge_topk_columns(const float* pmax, const float* psum, const unsigned long long* pkey,
                                                   int pstride, int nb, int k, const int (&col)[NC], float (&lse)[NC],
                                                   unsigned long long (&best)[NC][KMAX]) {
  static_assert((KMAX & (KMAX - 1)) == 0, "the merge network takes a power of two");
  const int lane = threadIdx.x & 63;
  float m_run[NC], s_run[NC];
  unsigned long long list[NC][KMAX];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    m_run[c] = -INFINITY;
    s_run[c] = 0.f;
#pragma unroll
    for (int r = 0; r < KMAX; ++r) list[c][r] = 0ull;
  }
  for (int b0 = 0; b0 < nb; b0 += 256) {
    float pm[NC][4], ps[NC][4];
    unsigned long long pk[NC][4][KMAX];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        // column-major partials [column][workgroup]: the lanes of a load read consecutive addresses.  Every load is
        // issued, on a clamped index (what it fetches is dropped below): loads under a condition would be waited
        // for group by group instead of all being in flight together
        const int b = b0 + u * 64 + lane;
        const size_t cm = col[c] >= 0 ? col[c] : 0, bb = b < nb ? b : nb - 1;
        pm[c][u] = pmax[cm * pstride + bb];
        ps[c][u] = psum[cm * pstride + bb];
#pragma unroll
        for (int r = 0; r < KMAX; ++r) pk[c][u][r] = pkey[(cm * kMaxTopk + (r < k ? r : 0)) * pstride + bb];
      }
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool ok = b0 + u * 64 + lane < nb && col[c] >= 0;
        pm[c][u] = ok ? pm[c][u] : -INFINITY;
        ps[c][u] = ok ? ps[c][u] : 0.f;
#pragma unroll
        for (int r = 0; r < KMAX; ++r) pk[c][u][r] = (ok && r < k) ? pk[c][u][r] : 0ull;
      }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (pm[c][u] > -INFINITY) {
          const float mn = fmaxf(m_run[c], pm[c][u]);
          s_run[c] = s_run[c] * __expf(m_run[c] - mn) + ps[c][u] * __expf(pm[c][u] - mn);
          m_run[c] = mn;
        }
      }
      merge_sorted_lists<KMAX>(pk[c][0], pk[c][1]);
      merge_sorted_lists<KMAX>(pk[c][2], pk[c][3]);
      merge_sorted_lists<KMAX>(pk[c][0], pk[c][2]);
      merge_sorted_lists<KMAX>(list[c], pk[c][0]);
    }
  }
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const float mx = wave_max_f32(m_run[c]);
    const float s = wave_sum_f32(m_run[c] > -INFINITY ? s_run[c] * __expf(m_run[c] - mx) : 0.f);
    lse[c] = mx + __logf(s);
#pragma unroll
    for (int r = 0; r < KMAX; ++r) {
      if (r < k) {
        const unsigned long long b = wave_max_u64(list[c][0]);
        if (list[c][0] == b) {  // keys are distinct (they carry the row id): one lane pops
#pragma unroll
          for (int i = 0; i + 1 < KMAX; ++i) list[c][i] = list[c][i + 1];
          list[c][KMAX - 1] = 0ull;
        }
        best[c][r] = b;
      }
    }
  }
}

}  // namespace ctcspec
