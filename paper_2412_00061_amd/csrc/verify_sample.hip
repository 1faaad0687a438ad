// verify_sample_tokens: the target model's sampled token after every tree node - sampling-based acceptance
// (Sec. 2.1: accept / re-sample rule of speculative sampling; Sec. 3.3: the longest sequence that satisfies the
// criterion).  The tree is built deterministically, so the draft distribution behind a node's token is a point
// mass; the rule of Sec. 2.1 then emits tokens with the target model's own distribution, and one uniform number
// per node realises it: draw the target's token at the node, move to the child that carries it, stop when none
// does.  This file is the draw; the walk is accept_longest, given these tokens in place of the greedy ones.
//
// The draw inverts the cumulative distribution of softmax(logits / temperature) in vocabulary order: the first
// token whose cumulative probability exceeds u.  One workgroup per node holds the row (128 KB at V = 32000) in
// registers, 16 bytes per lane and load, all loads in flight at once.  The cumulative sum is taken in three
// levels with a fixed order - wavefront totals per 4096-element chunk, lanes of the wavefront that holds the
// crossing, the four elements of that lane - so the same inputs give the same token on every run.
#include "common.h"

namespace ctcspec {

constexpr int kSampleThreads = 1024;
constexpr int kSampleWaves = kSampleThreads / 64;
constexpr int kSampleMaxNV = 16;  // 16-byte groups per thread: rows up to 65533 elements at any alignment

struct SampleParams {
  const float* logits;    // [B][N][V]
  const int32_t* n_nodes; // [B]
  const float* uniforms;  // [B][N]
  float inv_temp;
  int B, N, V;
  int32_t* target;        // [B][N]
};

// inclusive prefix sum over the lanes of a wavefront, lane order
__device__ __forceinline__ float wave_scan_incl(float v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const float o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

template <int NV>
__global__ __launch_bounds__(kSampleThreads) void verify_sample_kernel(SampleParams p) {
  __shared__ float red[kSampleWaves];
  __shared__ float wtot[NV * kSampleWaves];  // chunk-major: entry k * 16 + w
  __shared__ int pick_entry;
  __shared__ float pick_rest;
  const int i = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int32_t* out = p.target + (size_t)b * p.N + i;
  if (i >= p.n_nodes[b]) {
    if (tid == 0) *out = -1;
    return;
  }
  // The row starts `lead` elements past a 16-byte boundary; group g holds the row's elements 4g - lead .. 4g - lead + 3.
  const size_t row0 = ((size_t)b * p.N + i) * p.V;
  const int lead = (int)(row0 & 3);
  const float* base = p.logits + (row0 - lead);
  const int ngroups = (lead + p.V + 3) >> 2;
  f32x4 x[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int g = k * kSampleThreads + tid;
    const int e0 = 4 * g - lead;
    if (g < ngroups && e0 >= 0 && e0 + 3 < p.V) {
      x[k] = *(const f32x4*)(base + 4 * (size_t)g);
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int e = e0 + c;
        x[k][c] = (g < ngroups && e >= 0 && e < p.V) ? base[4 * (size_t)g + c] : -INFINITY;
      }
    }
  }
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    x[k] = x[k] * p.inv_temp;
    mx = fmaxf(fmaxf(fmaxf(mx, x[k][0]), fmaxf(x[k][1], x[k][2])), x[k][3]);
  }
  mx = wave_max_f32(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < kSampleWaves; ++w) mx = fmaxf(mx, red[w]);
  // unnormalised probabilities; a lane's group total is taken in element order, as the last level of the search is
  float s[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
#pragma unroll
    for (int c = 0; c < 4; ++c) x[k][c] = expf(x[k][c] - mx);
    s[k] = ((x[k][0] + x[k][1]) + x[k][2]) + x[k][3];
    const float wt = wave_sum_f32(s[k]);
    if (lane == 0) wtot[k * kSampleWaves + wave] = wt;
  }
  __syncthreads();
  // level 1 (wavefront 0): cumulative sum over the NV * 16 wavefront totals in vocabulary order
  constexpr int kEntries = NV * kSampleWaves;
  constexpr int kPer = (kEntries + 63) / 64;
  if (wave == 0) {
    float local = 0.f;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const int j = lane * kPer + q;
      local += j < kEntries ? wtot[j] : 0.f;
    }
    const float incl = wave_scan_incl(local, lane);
    const float total = __shfl(incl, 63, 64);
    const float want = p.uniforms[(size_t)b * p.N + i] * total;
    float run = incl - local;  // what lies before this lane's entries
    int found = -1, last_nonzero = -1;
    float rest = 0.f;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const int j = lane * kPer + q;
      const float v = j < kEntries ? wtot[j] : 0.f;
      if (found < 0 && run + v > want) {
        found = j;
        rest = want - run;
      }
      if (v > 0.f) last_nonzero = j;
      run += v;
    }
    const unsigned long long hit = __ballot(found >= 0);
    if (hit) {
      const int src = __ffsll((long long)hit) - 1;
      found = __shfl(found, src, 64);
      rest = __shfl(rest, src, 64);
    } else {  // u * total rounded up to the total: the last entry that holds any probability, all of it before u
      const unsigned long long any = __ballot(last_nonzero >= 0);
      const int src = any ? 63 - __clzll((long long)any) : 0;
      found = __shfl(last_nonzero, src, 64);
      found = found < 0 ? 0 : found;
      rest = INFINITY;
    }
    if (lane == 0) {
      pick_entry = found;
      pick_rest = rest;
    }
  }
  __syncthreads();
  // level 2: the lanes of the wavefront that holds the crossing; level 3: the four elements of that lane
  const int kstar = pick_entry / kSampleWaves, wstar = pick_entry % kSampleWaves;
  if (wave != wstar) return;
  float sv = 0.f;
  f32x4 ev = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < NV; ++k)
    if (k == kstar) {
      sv = s[k];
      ev = x[k];
    }
  const float rest = pick_rest;
  const float incl = wave_scan_incl(sv, lane);
  const unsigned long long cross = __ballot(incl > rest);
  const unsigned long long some = __ballot(sv > 0.f);
  int src;
  if (cross) src = __ffsll((long long)cross) - 1;
  else src = some ? 63 - __clzll((long long)some) : 0;
  if (lane != src) return;
  const float r3 = cross ? rest - (incl - sv) : INFINITY;
  int c_pick = -1, c_last = 0;
  float run = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    run += ev[c];
    if (c_pick < 0 && run > r3) c_pick = c;
    if (ev[c] > 0.f) c_last = c;
  }
  if (c_pick < 0) c_pick = c_last;
  int token = 4 * (kstar * kSampleThreads + tid) - lead + c_pick;
  token = token < 0 ? 0 : (token >= p.V ? p.V - 1 : token);
  *out = token;
}

// code of this translation unit loaded onto the current device (context creation calls this: a stage call never
// triggers a load, so it can be the first thing a stream capture records)
hipError_t prepare_verify_sample() {
  hipFuncAttributes attr;
  return hipFuncGetAttributes(&attr, (const void*)verify_sample_kernel<1>);
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int verify_sample_tokens(ctcspec_ctx* ctx, const float* logits, const int32_t* n_nodes, const float* uniforms,
                                    float temperature, int B, int max_nodes, int V, int32_t* target_sampled) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
  CTCSPEC_REQUIRE(ctx, logits && n_nodes && uniforms && target_sampled, CTCSPEC_EINVAL, "verify_sample_tokens: null pointer");
  CTCSPEC_REQUIRE(ctx, B > 0 && max_nodes > 0 && V > 0, CTCSPEC_EINVAL, "verify_sample_tokens: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, temperature > 0.f && temperature < INFINITY, CTCSPEC_EINVAL,
                  "verify_sample_tokens: temperature must be positive and finite");
  CTCSPEC_REQUIRE(ctx, aligned16(logits), CTCSPEC_EINVAL, "verify_sample_tokens: logits must be 16-byte aligned");
  const int nv = ((V + 6) / 4 + kSampleThreads - 1) / kSampleThreads;  // groups of a row that starts 3 past a boundary
  CTCSPEC_REQUIRE(ctx, nv <= kSampleMaxNV && B <= 65535, CTCSPEC_EUNSUPPORTED,
                  "verify_sample_tokens: V <= %d (a row is held in one workgroup's registers), B <= 65535",
                  kSampleMaxNV * kSampleThreads * 4 - 3);
  SampleParams p;
  p.logits = logits; p.n_nodes = n_nodes; p.uniforms = uniforms; p.inv_temp = 1.f / temperature;
  p.B = B; p.N = max_nodes; p.V = V; p.target = target_sampled;
  const dim3 grid(max_nodes, B), block(kSampleThreads);
  hipStream_t st = ctx->stream;
  if (nv <= 1) hipLaunchKernelGGL(verify_sample_kernel<1>, grid, block, 0, st, p);
  else if (nv <= 2) hipLaunchKernelGGL(verify_sample_kernel<2>, grid, block, 0, st, p);
  else if (nv <= 4) hipLaunchKernelGGL(verify_sample_kernel<4>, grid, block, 0, st, p);
  else if (nv <= 8) hipLaunchKernelGGL(verify_sample_kernel<8>, grid, block, 0, st, p);
  else hipLaunchKernelGGL(verify_sample_kernel<16>, grid, block, 0, st, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
