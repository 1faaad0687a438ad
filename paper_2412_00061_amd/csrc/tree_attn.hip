// tree_verify_attn: tree-masked verification attention of the base model, one layer.
//
// Generic path (any dtype / head dimension within the limits): one workgroup per (node, head,
// sequence); keys are processed in chunks with an online softmax.
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
  dim3 grid(max_nodes, H, B);
  if (dt == CTCSPEC_BF16)
    hipLaunchKernelGGL(tree_attn_generic_kernel<unsigned short>, grid, dim3(kGenericThreads), 0, ctx->stream, p);
  else
    hipLaunchKernelGGL(tree_attn_generic_kernel<float>, grid, dim3(kGenericThreads), 0, ctx->stream, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}
