// accept_longest: greedy acceptance walk over the token tree, one wavefront per sequence.
#include "common.h"

namespace ctcspec {

// Lane l looks at nodes l and l+64.  At each step the lanes whose node is a child of the current
// node carrying the target token raise a ballot; sibling tokens are distinct, so at most one does.
// Everything the walk reads is fetched up front in one round of loads (the node count included, so
// nothing waits for it): the walk itself then runs on registers, lane to lane.
__global__ __launch_bounds__(64) void accept_longest_kernel(const int32_t* n_nodes, const int32_t* node_token,
                                                            const int32_t* node_parent,
                                                            const int32_t* target, int T, int max_nodes,
                                                            int32_t* accept_len, int32_t* accept_nodes,
                                                            int32_t* accept_tokens, int32_t* next_token) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int32_t* tok = node_token + (size_t)b * max_nodes;
  const int32_t* par = node_parent + (size_t)b * max_nodes;
  const int32_t* tgt = target + (size_t)b * max_nodes;
  const int j0 = lane, j1 = lane + 64;
  const int c0 = j0 < max_nodes ? j0 : max_nodes - 1, c1 = j1 < max_nodes ? j1 : max_nodes - 1;
  int n = n_nodes[b];
  int t0 = tok[c0], p0 = par[c0], g0 = tgt[c0];
  int t1 = tok[c1], p1 = par[c1], g1 = tgt[c1];
  n = n < 1 ? 1 : (n > max_nodes ? max_nodes : n);
  if (j0 >= n) { t0 = -1; p0 = -2; }
  if (j1 >= n) { t1 = -1; p1 = -2; }
  const int root_token = __builtin_amdgcn_readfirstlane(t0);
  int cur = 0, len = 0;
  int want = __builtin_amdgcn_readfirstlane(g0);  // target at the root
  int my_node = lane == 0 ? 0 : -1, my_token = lane == 0 ? root_token : -1;  // lane i: entry i of the outputs
  while (len < T) {
    const unsigned long long hit0 = __ballot(j0 > 0 && p0 == cur && t0 == want);
    const unsigned long long hit1 = __ballot(p1 == cur && t1 == want);
    int nxt = -1;
    if (hit0) nxt = __builtin_ctzll(hit0);
    else if (hit1) nxt = 64 + __builtin_ctzll(hit1);
    if (nxt < 0) break;
    cur = nxt;
    ++len;
    if (lane == len) { my_node = cur; my_token = want; }
    want = __builtin_amdgcn_readlane(cur < 64 ? g0 : g1, cur & 63);
  }
  if (lane <= T) {
    accept_nodes[(size_t)b * (T + 1) + lane] = my_node;
    accept_tokens[(size_t)b * (T + 1) + lane] = my_token;
  }
  if (lane == 0) {
    accept_len[b] = len;
    next_token[b] = want;
  }
}

// code of this translation unit loaded onto the current device (context creation calls this: a stage call never
// triggers a load, so it can be the first thing a stream capture records)
hipError_t prepare_accept() {
  hipFuncAttributes attr;
  return hipFuncGetAttributes(&attr, (const void*)accept_longest_kernel);
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int accept_longest(ctcspec_ctx* ctx, const int32_t* n_nodes, const int32_t* node_token,
                              const int32_t* node_parent, const int32_t* node_depth,
                              const int32_t* target_argmax, int B, int T, int max_nodes, int32_t* accept_len,
                              int32_t* accept_nodes, int32_t* accept_tokens, int32_t* next_token) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
  (void)node_depth;  // the walk needs parents and tokens only; depth is accepted for symmetry with stage 3
  CTCSPEC_REQUIRE(ctx,
                  n_nodes && node_token && node_parent && target_argmax && accept_len && accept_nodes &&
                      accept_tokens && next_token,
                  CTCSPEC_EINVAL, "accept_longest: null pointer");
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && max_nodes > 0, CTCSPEC_EINVAL, "accept_longest: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, max_nodes <= CTCSPEC_MAX_NODES && T <= CTCSPEC_MAX_SLOTS, CTCSPEC_EUNSUPPORTED,
                  "accept_longest: max_nodes<=%d and T<=%d required", CTCSPEC_MAX_NODES, CTCSPEC_MAX_SLOTS);
  hipLaunchKernelGGL(accept_longest_kernel, dim3(B), dim3(64), 0, ctx->stream, n_nodes, node_token,
                     node_parent, target_argmax, T, max_nodes, accept_len, accept_nodes, accept_tokens,
                     next_token);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
