// Internal definitions shared by the translation units of libctcspec (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "ctcspec.h"

namespace ctcspec {

constexpr int kWave = 64;

// ---- draft head workspace geometry -------------------------------------------------------------
// A workgroup of the draft-head kernels owns kRowsPerBlock consecutive vocabulary rows and leaves one
// partial result per column: running max, sum of exponentials and its k best (logit, id) keys.
constexpr int kRowsPerBlock = 128;
constexpr int kMaxCols = CTCSPEC_MAX_COLUMNS;
constexpr int kMaxTopk = CTCSPEC_MAX_TOPK;

// ---- collapse/tree workspace geometry ----------------------------------------------------------
constexpr int kMaxAlign = CTCSPEC_MAX_ALIGNMENTS;
// Per sequence, for the rare case that more raw candidates than fit in LDS must be ordered:
// sort keys, collapsed-sequence keys (8 B each) and a hash table of 2*kMaxAlign 4-byte slots.
constexpr size_t kCollapseWsBytesPerSeq = (size_t)kMaxAlign * 8 * 2 + (size_t)kMaxAlign * 2 * 4;

// ---- verifier head workspace geometry ---------------------------------------------------------
constexpr int kVerifyCols = 128;  // columns (tree nodes) per pass over the base model's head weights

// ---- attention workspace geometry --------------------------------------------------------------
constexpr int kMaxKvSplits = 8;

}  // namespace ctcspec

struct ctcspec_ctx {
  hipStream_t stream;
  int device;
  ctcspec_limits lim;
  char err[256];
  // one device allocation, carved up below
  void* ws;
  size_t ws_bytes;
  // draft head
  int lm_max_blocks;
  // column-major, so that the merge reads each column's partials as contiguous runs over the workgroups
  float* lm_pmax;               // [kMaxCols][lm_max_blocks]
  float* lm_psum;               // [kMaxCols][lm_max_blocks]
  unsigned long long* lm_pkey;  // [kMaxCols][kMaxTopk][lm_max_blocks]
  // deferred merge (ctcspec_defer_topk_merge): a ctc_draft_topk call has left its per-workgroup partials in the
  // workspace and owes the caller these outputs; the next call on the context settles the debt first
  int lm_defer;
  int lm_pending;
  struct {
    int BT, k, n_blocks;
    int32_t* topk_id;
    float* topk_logp;
    float* lse;
  } lm_owed;
  // optional timing of the draft-head kernel
  int lm_profile;               // events are recorded around the main kernel when non-zero
  int lm_profile_valid;
  hipEvent_t lm_ev0, lm_ev1;
  // verifier head
  const void* zeros;            // 256 bytes of zeros
  int vh_col_blocks;            // column blocks of kVerifyCols the limits allow: ceil(max_batch * max_nodes / 128)
  unsigned long long* vh_pkey;  // [vh_col_blocks][lm_max_blocks][kVerifyCols] best (logit, id) key per row block and column
  // collapse / tree
  unsigned char* collapse_ws;   // [max_batch][kCollapseWsBytesPerSeq]
  // attention
  int attn_units;               // number of (sequence, head, split) partial slots
  float* attn_po;               // [attn_units][128][max_head_dim]
  float* attn_pm;               // [attn_units][128]
  float* attn_pl;               // [attn_units][128]
};

namespace ctcspec {

int fail(ctcspec_ctx* ctx, int code, const char* fmt, ...);

// Launches the merge kernel that a deferred ctc_draft_topk call still owes, if any.  Every entry point other than
// ctc_collapse_tree calls this first; ctc_collapse_tree does so unless the owed lists are the very ones it is given.
int flush_deferred(ctcspec_ctx* ctx);

// tree_verify_attn with an optional second output form for callers inside the library: when `rows` is given and
// the launch uses key splits, the merged result is written as rows [B*max_nodes][H*128] of two-bf16 values
// (planes of rows_plane elements) instead of `out`, and *rows_written is set to 1.
int tree_verify_attn_rows(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* q, const void* k_cache,
                          const void* v_cache, const int64_t* kv_off, const int32_t* ctx_len, int kv_cap,
                          const void* k_tree, const void* v_tree, const int32_t* n_nodes, const uint64_t* anc_mask,
                          int B, int H, int dh, int max_nodes, float scale, float* out, unsigned short* rows,
                          long long rows_plane, int* rows_written);

// Kernels that need more dynamic LDS than the default limit have the limit raised here, once per context creation
// (with the context's device current), never inside a stage call: a stage call then only enqueues launches and can
// be the first thing a stream capture records.  One function per translation unit that owns such kernels.
hipError_t prepare_draft_topk();
hipError_t prepare_collapse_tree();
hipError_t prepare_verify_head();
hipError_t prepare_draft_layer();
// the other translation units only have their code loaded onto the device
hipError_t prepare_tree_attn();
hipError_t prepare_accept();
hipError_t prepare_sum_score();
hipError_t prepare_ctc_loss();
hipError_t prepare_verify_sample();

#define CTCSPEC_REQUIRE(ctx, cond, code, ...) \
  do {                                        \
    if (!(cond)) return ::ctcspec::fail((ctx), (code), __VA_ARGS__); \
  } while (0)

#define CTCSPEC_HIP(ctx, expr)                                                              \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return ::ctcspec::fail((ctx), CTCSPEC_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device helpers ----------------------------------------------------------------------------
#if defined(__HIPCC__)

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Monotone map float -> uint32 (a < b  <=>  ord(a) < ord(b)); -0 is first turned into +0.
__device__ __forceinline__ unsigned int float_to_ordered(float f) {
  f = f + 0.0f;
  unsigned int u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(unsigned int o) {
  unsigned int u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
  return __uint_as_float(u);
}

// Ranking key of a (value, index) pair: larger value first, then smaller index first.
__device__ __forceinline__ unsigned long long rank_key(float v, unsigned int idx) {
  return ((unsigned long long)float_to_ordered(v) << 32) | (unsigned long long)(0xffffffffu - idx);
}
__device__ __forceinline__ float rank_key_value(unsigned long long key) {
  return ordered_to_float((unsigned int)(key >> 32));
}
__device__ __forceinline__ unsigned int rank_key_index(unsigned long long key) {
  return 0xffffffffu - (unsigned int)(key & 0xffffffffu);
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits for every
// outstanding global load (vmcnt(0)), which would drain a register prefetch pipeline at each barrier;
// this one waits for the wavefront's own LDS operations and then joins the barrier.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// ---- wavefront reductions ------------------------------------------------------------------------
// Inside each row of 16 lanes the partial results travel by DPP row rotations (no LDS round trip);
// the four row results are then combined through v_readlane.  Every lane returns the full result.
template <int ROT>
__device__ __forceinline__ unsigned int dpp_row_ror(unsigned int v) {
  return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x120 + ROT, 0xf, 0xf, false);
}
__device__ __forceinline__ unsigned int readlane_u32(unsigned int v, int lane) {
  return (unsigned int)__builtin_amdgcn_readlane((int)v, lane);
}

#define CTCSPEC_ROW_STEP_U64(ROT)                                                   \
  {                                                                                 \
    unsigned int olo = dpp_row_ror<ROT>(lo), ohi = dpp_row_ror<ROT>(hi);            \
    bool take = ohi > hi || (ohi == hi && olo > lo);                                \
    lo = take ? olo : lo;                                                           \
    hi = take ? ohi : hi;                                                           \
  }
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
  unsigned int lo = (unsigned int)v, hi = (unsigned int)(v >> 32);
  CTCSPEC_ROW_STEP_U64(1)
  CTCSPEC_ROW_STEP_U64(2)
  CTCSPEC_ROW_STEP_U64(4)
  CTCSPEC_ROW_STEP_U64(8)
  unsigned long long best = 0ull;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    unsigned long long x = ((unsigned long long)readlane_u32(hi, 16 * r) << 32) | readlane_u32(lo, 16 * r);
    best = x > best ? x : best;
  }
  return best;
}
#undef CTCSPEC_ROW_STEP_U64

__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, __uint_as_float(dpp_row_ror<1>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_row_ror<2>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_row_ror<4>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_row_ror<8>(__float_as_uint(v))));
  float a = __uint_as_float(readlane_u32(__float_as_uint(v), 0));
  float b = __uint_as_float(readlane_u32(__float_as_uint(v), 16));
  float c = __uint_as_float(readlane_u32(__float_as_uint(v), 32));
  float d = __uint_as_float(readlane_u32(__float_as_uint(v), 48));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}
__device__ __forceinline__ float wave_sum_f32(float v) {
  v += __uint_as_float(dpp_row_ror<1>(__float_as_uint(v)));
  v += __uint_as_float(dpp_row_ror<2>(__float_as_uint(v)));
  v += __uint_as_float(dpp_row_ror<4>(__float_as_uint(v)));
  v += __uint_as_float(dpp_row_ror<8>(__float_as_uint(v)));
  float a = __uint_as_float(readlane_u32(__float_as_uint(v), 0));
  float b = __uint_as_float(readlane_u32(__float_as_uint(v), 16));
  float c = __uint_as_float(readlane_u32(__float_as_uint(v), 32));
  float d = __uint_as_float(readlane_u32(__float_as_uint(v), 48));
  return (a + b) + (c + d);
}
__device__ __forceinline__ int wave_sum_i32(int v) {
  v += (int)dpp_row_ror<1>((unsigned)v);
  v += (int)dpp_row_ror<2>((unsigned)v);
  v += (int)dpp_row_ror<4>((unsigned)v);
  v += (int)dpp_row_ror<8>((unsigned)v);
  return (int)(readlane_u32((unsigned)v, 0) + readlane_u32((unsigned)v, 16) + readlane_u32((unsigned)v, 32) +
               readlane_u32((unsigned)v, 48));
}

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
  return __uint_as_float(((unsigned int)b) << 16);
}

template <typename T>
__device__ __forceinline__ float load_as_float(const T* p);
template <>
__device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_as_float<unsigned short>(const unsigned short* p) {
  return bf16_bits_to_float(*p);
}

#endif  // __HIPCC__

}  // namespace ctcspec
