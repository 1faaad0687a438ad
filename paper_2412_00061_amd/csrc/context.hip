// Context of libctcspec: stream binding, limits, the one device workspace, error reporting.
#include <stdarg.h>
#include <stdlib.h>

#include <new>

#include "common.h"

namespace ctcspec {

static thread_local char g_create_err[256] = "";

int fail(ctcspec_ctx* ctx, int code, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_create_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 256, fmt, ap);
  va_end(ap);
  return code;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace ctcspec

namespace ctcspec {

// Read-only streaming probe: every wavefront reads contiguous 128 KB pieces (sixteen 8 KB rows of a 7B-shaped head)
// with coalesced, non-temporal 16-byte loads, eight of them in flight, and folds the words together - the rate at
// which this GPU delivers a matrix that is read once and used for nothing.  The draft head's roofline figure is also
// quoted against this measured rate.
constexpr int kProbePiece = 128 * 1024;
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4* __restrict__ src, long long pieces,
                                                           unsigned int* __restrict__ out) {
  const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (wave >= pieces) return;
  const u32x4* p = src + wave * (kProbePiece / 16) + lane;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int i = 0; i < kProbePiece / 1024; i += 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + (size_t)(i + u) * 64);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  const unsigned int r = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (r == 0x12345678u) out[0] = r;  // keeps the loads alive; practically never taken
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" int ctcspec_stream_probe(ctcspec_ctx* ctx, const void* src, size_t bytes, uint32_t* sink) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
  CTCSPEC_REQUIRE(ctx, src && sink && aligned16(src), CTCSPEC_EINVAL, "ctcspec_stream_probe: null or misaligned pointer");
  const long long pieces = (long long)(bytes / kProbePiece);
  CTCSPEC_REQUIRE(ctx, pieces >= 1 && pieces <= 0x7fffffffLL, CTCSPEC_EINVAL,
                  "ctcspec_stream_probe: at least %d bytes required", kProbePiece);
  hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)((pieces + 3) / 4)), dim3(256), 0, ctx->stream,
                     (const u32x4*)src, pieces, sink);
  CTCSPEC_HIP(ctx, hipGetLastError());
  return CTCSPEC_OK;
}

extern "C" int ctcspec_create(ctcspec_ctx** out, void* hip_stream, const ctcspec_limits* lim) {
  if (out) *out = nullptr;
  CTCSPEC_REQUIRE(nullptr, out && lim, CTCSPEC_EINVAL, "ctcspec_create: null argument");
  CTCSPEC_REQUIRE(nullptr,
                  lim->max_batch > 0 && lim->max_slots > 0 && lim->max_topk > 0 &&
                      lim->max_vocab_rows > 0 && lim->max_nodes > 0 && lim->max_heads > 0 &&
                      lim->max_head_dim > 0,
                  CTCSPEC_EINVAL, "ctcspec_create: every limit must be positive");
  CTCSPEC_REQUIRE(nullptr,
                  lim->max_slots <= CTCSPEC_MAX_SLOTS && lim->max_topk <= CTCSPEC_MAX_TOPK &&
                      lim->max_nodes <= CTCSPEC_MAX_NODES &&
                      lim->max_head_dim <= CTCSPEC_MAX_HEAD_DIM &&
                      (long long)lim->max_batch * lim->max_slots <= CTCSPEC_MAX_COLUMNS,
                  CTCSPEC_EUNSUPPORTED,
                  "ctcspec_create: limits exceed the compiled maxima (T<=%d, k<=%d, nodes<=%d, "
                  "dh<=%d, B*T<=%d)",
                  CTCSPEC_MAX_SLOTS, CTCSPEC_MAX_TOPK, CTCSPEC_MAX_NODES, CTCSPEC_MAX_HEAD_DIM,
                  CTCSPEC_MAX_COLUMNS);
  ctcspec_ctx* ctx = new (std::nothrow) ctcspec_ctx();
  CTCSPEC_REQUIRE(nullptr, ctx, CTCSPEC_EINVAL, "ctcspec_create: out of host memory");
  memset(ctx, 0, sizeof(*ctx));
  ctx->stream = (hipStream_t)hip_stream;
  ctx->lim = *lim;
  hipError_t e = hipGetDevice(&ctx->device);
  if (e != hipSuccess) {
    delete ctx;
    return fail(nullptr, CTCSPEC_EHIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  }

  // dynamic LDS limits of the large kernels, for this device (no stage call touches function attributes)
  e = prepare_draft_topk();
  if (e == hipSuccess) e = prepare_collapse_tree();
  if (e == hipSuccess) e = prepare_verify_head();
  if (e == hipSuccess) e = prepare_draft_layer();
  if (e == hipSuccess) e = prepare_tree_attn();
  if (e == hipSuccess) e = prepare_accept();
  if (e == hipSuccess) e = prepare_sum_score();
  if (e == hipSuccess) e = prepare_ctc_loss();
  if (e == hipSuccess) e = prepare_verify_sample();
  if (e != hipSuccess) {
    delete ctx;
    return fail(nullptr, CTCSPEC_EHIP, "preparing the kernels failed: %s", hipGetErrorString(e));
  }

  ctx->lm_max_blocks = (lim->max_vocab_rows + kRowsPerBlock - 1) / kRowsPerBlock;
  long long bh = (long long)lim->max_batch * lim->max_heads;
  ctx->attn_units = (int)(bh > 256 ? bh : 256);

  size_t off = 0;
  auto carve = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  size_t o_pmax = carve((size_t)ctx->lm_max_blocks * kMaxCols * sizeof(float));
  size_t o_psum = carve((size_t)ctx->lm_max_blocks * kMaxCols * sizeof(float));
  size_t o_pkey = carve((size_t)ctx->lm_max_blocks * kMaxCols * kMaxTopk * sizeof(unsigned long long));
  ctx->vh_col_blocks = (int)(((long long)lim->max_batch * lim->max_nodes + kVerifyCols - 1) / kVerifyCols);
  size_t o_vh = carve((size_t)ctx->vh_col_blocks * ctx->lm_max_blocks * kVerifyCols * sizeof(unsigned long long));
  size_t o_zero = carve(256);
  size_t o_coll = carve((size_t)lim->max_batch * kCollapseWsBytesPerSeq);
  // attention partials: one slot of 128 query rows per (sequence, head, key split)
  const size_t attn_rows = (size_t)ctx->attn_units * 128;
  size_t o_po = carve(attn_rows * lim->max_head_dim * sizeof(float));
  size_t o_pm = carve(attn_rows * sizeof(float));
  size_t o_pl = carve(attn_rows * sizeof(float));
  ctx->ws_bytes = off;
  e = hipMalloc(&ctx->ws, ctx->ws_bytes);
  if (e != hipSuccess) {
    delete ctx;
    return fail(nullptr, CTCSPEC_EHIP, "hipMalloc of %zu workspace bytes failed: %s", off,
                hipGetErrorString(e));
  }
  unsigned char* base = (unsigned char*)ctx->ws;
  e = hipMemset(base + o_zero, 0, 256);  // read by loads that must fetch something harmless
  if (e != hipSuccess) {
    (void)hipFree(ctx->ws);
    delete ctx;
    return fail(nullptr, CTCSPEC_EHIP, "hipMemset failed: %s", hipGetErrorString(e));
  }
  ctx->lm_pmax = (float*)(base + o_pmax);
  ctx->lm_psum = (float*)(base + o_psum);
  ctx->lm_pkey = (unsigned long long*)(base + o_pkey);
  ctx->vh_pkey = (unsigned long long*)(base + o_vh);
  ctx->zeros = base + o_zero;
  ctx->collapse_ws = base + o_coll;
  ctx->attn_po = (float*)(base + o_po);
  ctx->attn_pm = (float*)(base + o_pm);
  ctx->attn_pl = (float*)(base + o_pl);
  g_create_err[0] = 0;
  *out = ctx;
  return CTCSPEC_OK;
}

extern "C" int ctcspec_profile_draft_head(ctcspec_ctx* ctx, int enable) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (enable && !ctx->lm_ev0) {
    CTCSPEC_HIP(ctx, hipEventCreate(&ctx->lm_ev0));
    CTCSPEC_HIP(ctx, hipEventCreate(&ctx->lm_ev1));
  }
  ctx->lm_profile = enable ? 1 : 0;
  ctx->lm_profile_valid = 0;
  return CTCSPEC_OK;
}

extern "C" int ctcspec_draft_head_kernel_ms(ctcspec_ctx* ctx, float* ms) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx, ms, CTCSPEC_EINVAL, "ctcspec_draft_head_kernel_ms: null pointer");
  CTCSPEC_REQUIRE(ctx, ctx->lm_profile && ctx->lm_profile_valid, CTCSPEC_EINVAL,
                  "ctcspec_draft_head_kernel_ms: profiling is off or no call was recorded");
  CTCSPEC_HIP(ctx, hipEventSynchronize(ctx->lm_ev1));
  CTCSPEC_HIP(ctx, hipEventElapsedTime(ms, ctx->lm_ev0, ctx->lm_ev1));
  return CTCSPEC_OK;
}

extern "C" void ctcspec_destroy(ctcspec_ctx* ctx) {
  if (!ctx) return;
  if (ctx->lm_ev0) (void)hipEventDestroy(ctx->lm_ev0);
  if (ctx->lm_ev1) (void)hipEventDestroy(ctx->lm_ev1);
  if (ctx->ws) (void)hipFree(ctx->ws);
  delete ctx;
}

extern "C" int ctcspec_defer_topk_merge(ctcspec_ctx* ctx, int enable) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;
  ctx->lm_defer = enable ? 1 : 0;
  return CTCSPEC_OK;
}

extern "C" int ctcspec_flush(ctcspec_ctx* ctx) {
  if (!ctx) return CTCSPEC_EINVAL;
  return flush_deferred(ctx);
}

extern "C" int ctcspec_set_stream(ctcspec_ctx* ctx, void* hip_stream) {
  if (!ctx) return CTCSPEC_EINVAL;
  if (const int owed = flush_deferred(ctx)) return owed;  // on the stream the partials were produced on
  ctx->stream = (hipStream_t)hip_stream;
  return CTCSPEC_OK;
}

extern "C" const char* ctcspec_last_error(const ctcspec_ctx* ctx) {
  return ctx ? ctx->err : g_create_err;
}

extern "C" size_t ctcspec_workspace_bytes(const ctcspec_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }
