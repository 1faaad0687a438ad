// ctc_sum_score: the value of every candidate draft under Eq. 5 - the probability of the collapsed sequence
// summed over ALL raw sequences (whole vocabulary plus blank in every slot) that collapse to it - and the rank
// order of the candidates by that value.  ctc_collapse_tree values a draft by its best single alignment
// (Eq. 6); this call gives the alternative the paper trains with.
//
// Forward recursion of the CTC paper cited in Sec. 3.2 over the extended sequence blank, y1, blank, ..., blank
// (at most 2T+1 = 17 states): one wavefront per candidate (all candidates side by side), lane s holds log alpha(s), the
// neighbours come by lane shifts, T steps; a second small kernel ranks the values.  Only the log-probabilities of the draft's own tokens and of the blank are needed:
// log p_t(v) = logits[t][v] - lse[t] from ctc_draft_topk.  KB-sized and latency-bound.
#include "common.h"

namespace ctcspec {

struct SumScoreParams {
  const float* logits;         // [B][T][Vp1]
  const float* lse;            // [B][T]
  const int32_t* cand_tokens;  // [B][beam][T]
  const int32_t* cand_len;     // [B][beam]
  const int32_t* n_cand;       // [B]
  int B, T, Vp1, blank, beam;
  float* sum;                  // [B][beam]
  int32_t* rank;               // [B][beam]
};

__device__ __forceinline__ float log_add(float a, float b) {
  const float hi = fmaxf(a, b), lo = fminf(a, b);
  if (hi == -INFINITY) return -INFINITY;
  return hi + log1pf(expf(lo - hi));
}

// one wavefront per (sequence, candidate)
__global__ __launch_bounds__(64) void sum_score_kernel(SumScoreParams p) {
  const int i = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  int n = p.n_cand[b];
  n = n < 0 ? 0 : (n > p.beam ? p.beam : n);
  float total = -INFINITY;
  if (i < n) {
    int len = p.cand_len[b * p.beam + i];
    len = len < 0 ? 0 : (len > p.T ? p.T : len);
    const int S = 2 * len + 1;
    // symbol of state s: blank for even s, token (s-1)/2 for odd s
    int sym = p.blank, sym2 = -1;  // sym2: symbol two states back (odd s >= 3)
    if ((lane & 1) && lane < S) {
      sym = p.cand_tokens[((size_t)b * p.beam + i) * p.T + (lane >> 1)];
      if (lane >= 3) sym2 = p.cand_tokens[((size_t)b * p.beam + i) * p.T + (lane >> 1) - 1];
    }
    sym = sym < 0 ? 0 : (sym >= p.Vp1 ? p.Vp1 - 1 : sym);  // ids come from the caller
    const bool skip_ok = (lane & 1) && lane >= 3 && sym != sym2;
    const float* z = p.logits + (size_t)b * p.T * p.Vp1;
    // the T log-probabilities of this state's symbol, requested together
    float lp[CTCSPEC_MAX_SLOTS];
#pragma unroll
    for (int t = 0; t < CTCSPEC_MAX_SLOTS; ++t) {
      const int tt = t < p.T ? t : p.T - 1;
      lp[t] = lane < S ? z[(size_t)tt * p.Vp1 + sym] - p.lse[b * p.T + tt] : -INFINITY;
    }
    float alpha = lane < 2 ? lp[0] : -INFINITY;
#pragma unroll
    for (int t = 1; t < CTCSPEC_MAX_SLOTS; ++t) {
      if (t < p.T) {
        float a1 = __shfl_up(alpha, 1, 64), a2 = __shfl_up(alpha, 2, 64);
        a1 = lane >= 1 ? a1 : -INFINITY;
        a2 = skip_ok ? a2 : -INFINITY;
        alpha = lane < S ? log_add(log_add(alpha, a1), a2) + lp[t] : -INFINITY;
      }
    }
    const float last = __shfl(alpha, S - 1, 64), prev = S > 1 ? __shfl(alpha, S - 2, 64) : -INFINITY;
    total = log_add(last, prev);
  }
  if (lane == 0) p.sum[b * p.beam + i] = total;
}

// rank in the order (value descending, index ascending); one block per sequence
__global__ __launch_bounds__(128) void sum_rank_kernel(SumScoreParams p) {
  __shared__ float s_sum[CTCSPEC_MAX_BEAM];
  const int b = blockIdx.x, tid = threadIdx.x;
  int n = p.n_cand[b];
  n = n < 0 ? 0 : (n > p.beam ? p.beam : n);
  for (int i = tid; i < p.beam; i += 128) s_sum[i] = p.sum[b * p.beam + i];
  __syncthreads();
  for (int i = tid; i < p.beam; i += 128) {
    int r = -1;
    if (i < n) {
      r = 0;
      const float v = s_sum[i];
      for (int j = 0; j < n; ++j) {
        const float u = s_sum[j];
        r += (u > v || (u == v && j < i)) ? 1 : 0;
      }
    }
    p.rank[b * p.beam + i] = r;
  }
}

// code of this translation unit loaded onto the current device (context creation calls this: a stage call never
// triggers a load, so it can be the first thing a stream capture records)
hipError_t prepare_sum_score() {
  hipFuncAttributes attr;
  return hipFuncGetAttributes(&attr, (const void*)sum_score_kernel);
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int ctc_sum_score(ctcspec_ctx* ctx, const float* logits, const float* lse, const int32_t* cand_tokens,
                             const int32_t* cand_len, const int32_t* n_cand, int B, int T, int Vp1, int32_t blank_id,
                             int beam, float* cand_logp_sum, int32_t* cand_rank_sum) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
  CTCSPEC_REQUIRE(ctx, logits && lse && cand_tokens && cand_len && n_cand && cand_logp_sum && cand_rank_sum,
                  CTCSPEC_EINVAL, "ctc_sum_score: null pointer");
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && Vp1 > 0 && beam > 0, CTCSPEC_EINVAL, "ctc_sum_score: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, T <= CTCSPEC_MAX_SLOTS && beam <= CTCSPEC_MAX_BEAM && B <= ctx->lim.max_batch && B <= 65535,
                  CTCSPEC_EUNSUPPORTED, "ctc_sum_score: T <= %d, beam <= %d and B within the context's limits required",
                  CTCSPEC_MAX_SLOTS, CTCSPEC_MAX_BEAM);
  CTCSPEC_REQUIRE(ctx, blank_id >= 0 && blank_id < Vp1, CTCSPEC_EINVAL, "ctc_sum_score: blank_id out of range");
  SumScoreParams p;
  p.logits = logits; p.lse = lse; p.cand_tokens = cand_tokens; p.cand_len = cand_len; p.n_cand = n_cand;
  p.B = B; p.T = T; p.Vp1 = Vp1; p.blank = blank_id; p.beam = beam; p.sum = cand_logp_sum; p.rank = cand_rank_sum;
  hipLaunchKernelGGL(sum_score_kernel, dim3(beam, B), dim3(64), 0, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  hipLaunchKernelGGL(sum_rank_kernel, dim3(B), dim3(128), 0, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
