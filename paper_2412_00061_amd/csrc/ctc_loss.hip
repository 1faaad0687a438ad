// ctc_loss: the training objective of Sec. 3.2 - the negative log of Eq. 5 for a label sequence - and its gradient
// with respect to the logits, by the forward-backward recursions of the CTC paper the section cites.
//
// Two kinds of work, kept apart:
//   * the rows of logits ([V+1] floats per frame, 128 KB at V = 32000) are what costs HBM time.  They are read
//     twice and written once, each time a whole row through LDS by one workgroup: ctc_row_kernel takes the
//     log-sum-exp of a row and picks out the few log-probabilities the recursions need (the label's tokens and
//     the blank); ctc_grad_kernel turns the row into its softmax, subtracts the occupancies of those few
//     symbols and writes the gradient row.
//   * the recursions themselves are KB-sized and sequential in the frames: ctc_dp_kernel, one workgroup per
//     sequence, a thread per state of the extended sequence (blank, y1, blank, ..., blank), the neighbours'
//     values through LDS, one barrier per frame.  Forward stores log alpha per frame; backward turns it in place
//     into the occupancy gamma_t(s) = alpha_t(s) beta_t(s) / (p_t(z_s) P).
// A token that occurs several times in a label has several states; their occupancies are added in label order
// by the thread of the first occurrence (links built once per sequence), so no atomic is needed and the result
// has the same bits on every run.
#include "common.h"

namespace ctcspec {

constexpr int kCtcMaxLabels = 2047;  // 2L + 1 states <= 4 per thread of a 1024-thread workgroup
constexpr int kCtcRowThreads = 512;

struct CtcParams {
  const float* logits;      // [B][T][Vp1]
  const int32_t* labels;    // [B][Lmax]
  const int32_t* label_len; // [B]
  const int32_t* frame_len; // [B]
  int B, T, Vp1, Lmax, blank;
  // workspace
  float* lse;     // [B][T]
  float* lpc;     // [B][T][Lmax + 1]: log p_t(y_j) for j < L, log p_t(blank) at Lmax
  float* ag;      // [B][T][2 Lmax + 1]: log alpha minus the frame's offset, then gamma
  double* coff;   // [B][T]: offset of the frame's log alpha values
  int32_t* next;  // [B][Lmax]: next label position with the same token, -1: none
  int32_t* first; // [B][Lmax]: 1 when no earlier position holds the same token
  // outputs
  float* loss;    // [B]
  float* grad;    // [B][T][Vp1] or null
};

__device__ __forceinline__ float ctc_log_add(float a, float b) {
  const float hi = fmaxf(a, b), lo = fminf(a, b);
  if (hi == -INFINITY) return -INFINITY;
  return hi + log1pf(expf(lo - hi));
}
// largest of the wavefronts' maxima of one frame; 0 when every state is impossible, so that offsets stay finite
__device__ __forceinline__ float frame_max(const float* w, int n) {
  float m = w[0];
  for (int i = 1; i < n; ++i) m = fmaxf(m, w[i]);
  return m > -INFINITY ? m : 0.f;
}
__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// per sequence: links between the label positions that hold the same token
__global__ __launch_bounds__(256) void ctc_links_kernel(CtcParams p) {
  const int b = blockIdx.x;
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  const int32_t* y = p.labels + (size_t)b * p.Lmax;
  for (int j = threadIdx.x; j < p.Lmax; j += 256) {
    int nx = -1, fst = 1;
    if (j < L) {
      const int tok = y[j];
      for (int i = j + 1; i < L; ++i)
        if (y[i] == tok) { nx = i; break; }
      for (int i = 0; i < j; ++i)
        if (y[i] == tok) { fst = 0; break; }
    } else {
      fst = 0;
    }
    p.next[(size_t)b * p.Lmax + j] = nx;
    p.first[(size_t)b * p.Lmax + j] = fst;
  }
}

// one workgroup per frame row: row -> LDS, log-sum-exp, the log-probabilities of the label's tokens and the blank
__global__ __launch_bounds__(kCtcRowThreads) void ctc_row_kernel(CtcParams p) {
  extern __shared__ __attribute__((aligned(16))) float row[];
  __shared__ float red[kCtcRowThreads / 64];
  const int t = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int Tb = clampi(p.frame_len[b], 0, p.T);
  if (t >= Tb) return;
  const float* z = p.logits + ((size_t)b * p.T + t) * p.Vp1;
  float mx = -INFINITY;
  for (int v = tid; v < p.Vp1; v += kCtcRowThreads) {
    const float x = z[v];
    row[v] = x;
    mx = fmaxf(mx, x);
  }
  mx = wave_max_f32(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < kCtcRowThreads / 64; ++w) mx = fmaxf(mx, red[w]);
  float sum = 0.f;
  for (int v = tid; v < p.Vp1; v += kCtcRowThreads) sum += expf(row[v] - mx);
  sum = wave_sum_f32(sum);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = sum;
  __syncthreads();
  sum = 0.f;
#pragma unroll
  for (int w = 0; w < kCtcRowThreads / 64; ++w) sum += red[w];
  const float lse = mx + logf(sum);
  if (tid == 0) p.lse[(size_t)b * p.T + t] = lse;
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  float* out = p.lpc + ((size_t)b * p.T + t) * (p.Lmax + 1);
  for (int j = tid; j < L; j += kCtcRowThreads) out[j] = row[clampi(p.labels[(size_t)b * p.Lmax + j], 0, p.Vp1 - 1)] - lse;
  if (tid == 0) out[p.Lmax] = row[p.blank] - lse;
}

// one workgroup per sequence: forward and backward recursion over the frames
template <int NS>  // states per thread
__global__ __launch_bounds__(1024) void ctc_dp_kernel(CtcParams p) {
  extern __shared__ float lds[];  // two rows of Smax + 4 values (two -inf entries in front and behind)
  const int b = blockIdx.x, tid = threadIdx.x, nthreads = blockDim.x;
  const int Smax = 2 * p.Lmax + 1;
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  const int S = 2 * L + 1;
  const int Tb = clampi(p.frame_len[b], 0, p.T);
  const int pitch = Smax + 4;
  float* rowbuf[2] = {lds + 2, lds + pitch + 2};
  __shared__ float wmax[2][16];  // per frame parity: the wavefronts' largest value
  const int nwaves = nthreads >> 6;
  const int32_t* y = p.labels + (size_t)b * p.Lmax;
  const float* lpc = p.lpc + (size_t)b * p.T * (p.Lmax + 1);
  float* ag = p.ag + (size_t)b * p.T * Smax;
  double* coff = p.coff + (size_t)b * p.T;
  if (Tb == 0) {
    if (tid == 0) p.loss[b] = L == 0 ? 0.f : INFINITY;
    return;
  }
  // per state of this thread: index of its log-probability in a frame's compact row, and whether the transition
  // that skips the blank before it exists (into s from s - 2) / after it (from s into s + 2)
  int col[NS];
  bool skip_in[NS], skip_out[NS];
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    const int s = tid + u * nthreads;
    const int j = s >> 1;
    col[u] = (s & 1) ? j : p.Lmax;
    skip_in[u] = (s & 1) && s >= 3 && s < S && y[j] != y[j - 1];
    skip_out[u] = (s & 1) && s + 2 < S && y[j] != y[j + 1];
  }
  for (int i = tid; i < 2 * pitch; i += nthreads) lds[i] = -INFINITY;
  __syncthreads();

  // ---- forward ------------------------------------------------------------------------------------------------
  double c_alpha = 0.0;  // the stored values of the frame are log alpha - c_alpha
  for (int t = 0; t < Tb; ++t) {
    float* cur = rowbuf[t & 1];
    const float* prev = rowbuf[(t & 1) ^ 1];
    const float* lp = lpc + (size_t)t * (p.Lmax + 1);
    float shift = 0.f;
    if (t > 0) {
      shift = frame_max(wmax[(t & 1) ^ 1], nwaves);
      c_alpha += (double)shift;
    }
    float mine = -INFINITY;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int s = tid + u * nthreads;
      if (s < S) {
        float a;
        if (t == 0) {
          a = s < 2 ? 0.f : -INFINITY;
        } else {
          a = ctc_log_add(prev[s], prev[s - 1]);
          if (skip_in[u]) a = ctc_log_add(a, prev[s - 2]);
        }
        a += lp[col[u]] - shift;
        cur[s] = a;
        ag[(size_t)t * Smax + s] = a;
        mine = fmaxf(mine, a);
      }
    }
    mine = wave_max_f32(mine);
    if ((tid & 63) == 0) wmax[t & 1][tid >> 6] = mine;
    if (tid == 0) coff[t] = c_alpha;
    __syncthreads();
  }
  const float* last = rowbuf[(Tb - 1) & 1];
  const float tail = S > 1 ? ctc_log_add(last[S - 1], last[S - 2]) : last[S - 1];
  const double logP = c_alpha + (double)tail;  // -inf when the label cannot be reached
  if (tid == 0) p.loss[b] = (float)-logP;
  __syncthreads();
  for (int i = tid; i < 2 * pitch; i += nthreads) lds[i] = -INFINITY;
  __syncthreads();
  if (!p.grad) return;

  // ---- backward; log alpha in the workspace becomes gamma -------------------------------------------------------
  const bool reachable = tail > -INFINITY;
  double c_beta = 0.0;  // the values of the frame in LDS are log beta - c_beta
  for (int t = Tb - 1; t >= 0; --t) {
    float* cur = rowbuf[t & 1];
    const float* nxt = rowbuf[(t & 1) ^ 1];
    const float* lp = lpc + (size_t)t * (p.Lmax + 1);
    float shift = 0.f;
    if (t < Tb - 1) {
      shift = frame_max(wmax[(t & 1) ^ 1], nwaves);
      c_beta += (double)shift;
    }
    // log of P over the two offsets of this frame: what alpha-hat + beta-hat - log p has to be measured against
    const float z = reachable ? (float)(logP - coff[t] - c_beta) : 0.f;
    float mine = -INFINITY;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int s = tid + u * nthreads;
      if (s < S) {
        float bt;
        if (t == Tb - 1) {
          bt = s >= S - 2 ? 0.f : -INFINITY;
        } else {
          bt = ctc_log_add(nxt[s], nxt[s + 1]);
          if (skip_out[u]) bt = ctc_log_add(bt, nxt[s + 2]);
        }
        const float l = lp[col[u]];
        bt += l - shift;
        cur[s] = bt;
        mine = fmaxf(mine, bt);
        const float al = ag[(size_t)t * Smax + s];
        const float e = al + bt - l - z;
        ag[(size_t)t * Smax + s] = (reachable && al > -INFINITY && bt > -INFINITY) ? expf(e) : 0.f;
      }
    }
    mine = wave_max_f32(mine);
    if ((tid & 63) == 0) wmax[t & 1][tid >> 6] = mine;
    __syncthreads();
  }
}

// one workgroup per frame row: softmax of the row minus the occupancies of the label's tokens and of the blank
__global__ __launch_bounds__(kCtcRowThreads) void ctc_grad_kernel(CtcParams p) {
  extern __shared__ __attribute__((aligned(16))) float row[];
  __shared__ float red[kCtcRowThreads / 64];
  const int t = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int Tb = clampi(p.frame_len[b], 0, p.T);
  float* g = p.grad + ((size_t)b * p.T + t) * p.Vp1;
  const float loss = p.loss[b];
  if (t >= Tb || !(loss < INFINITY)) {  // frames past the sequence, or a label that cannot be reached: no gradient
    for (int v = tid; v < p.Vp1; v += kCtcRowThreads) g[v] = 0.f;
    return;
  }
  const float* z = p.logits + ((size_t)b * p.T + t) * p.Vp1;
  const float lse = p.lse[(size_t)b * p.T + t];
  for (int v = tid; v < p.Vp1; v += kCtcRowThreads) row[v] = expf(z[v] - lse);
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  const int Smax = 2 * p.Lmax + 1;
  const float* gamma = p.ag + ((size_t)b * p.T + t) * Smax;
  // the blank: all even states, added in a fixed order
  float gb = 0.f;
  for (int s = 2 * tid; s < 2 * L + 1; s += 2 * kCtcRowThreads) gb += gamma[s];
  gb = wave_sum_f32(gb);
  if ((tid & 63) == 0) red[tid >> 6] = gb;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kCtcRowThreads / 64; ++w) tot += red[w];
    row[p.blank] -= tot;
  }
  // the label's tokens: the thread of a token's first position adds the occupancies of all its positions
  const int32_t* y = p.labels + (size_t)b * p.Lmax;
  const int32_t* nx = p.next + (size_t)b * p.Lmax;
  const int32_t* fs = p.first + (size_t)b * p.Lmax;
  for (int j = tid; j < L; j += kCtcRowThreads) {
    if (!fs[j]) continue;
    float tot = 0.f;
    for (int i = j; i >= 0; i = nx[i]) tot += gamma[2 * i + 1];
    const int tok = clampi(y[j], 0, p.Vp1 - 1);
    if (tok != p.blank) row[tok] -= tot;  // a label never holds the blank; ids come from the caller
  }
  __syncthreads();
  for (int v = tid; v < p.Vp1; v += kCtcRowThreads) g[v] = row[v];
}

struct CtcWorkspace {
  size_t lse, lpc, ag, coff, next, first, total;
};
static CtcWorkspace ctc_workspace(int B, int T, int Lmax) {
  CtcWorkspace w;
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t at = off; off = (off + bytes + 255) / 256 * 256; return at; };
  w.lse = carve((size_t)B * T * 4);
  w.lpc = carve((size_t)B * T * (Lmax + 1) * 4);
  w.ag = carve((size_t)B * T * (2 * (size_t)Lmax + 1) * 4);
  w.coff = carve((size_t)B * T * 8);
  w.next = carve((size_t)B * Lmax * 4);
  w.first = carve((size_t)B * Lmax * 4);
  w.total = off;
  return w;
}

}  // namespace ctcspec

using namespace ctcspec;

extern "C" size_t ctc_loss_workspace_bytes(int B, int T, int Lmax) {
  if (B < 1 || T < 1 || Lmax < 1) return 0;
  return ctc_workspace(B, T, Lmax).total;
}

extern "C" int ctc_loss(ctcspec_ctx* ctx, const float* logits, const int32_t* labels, const int32_t* label_len,
                        const int32_t* frame_len, int B, int T, int Vp1, int Lmax, int32_t blank_id, void* workspace,
                        size_t workspace_bytes, float* loss, float* grad) {
  if (!ctx) return CTCSPEC_EINVAL;
  CTCSPEC_REQUIRE(ctx, logits && labels && label_len && frame_len && workspace && loss, CTCSPEC_EINVAL,
                  "ctc_loss: null pointer");
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && Vp1 > 0 && Lmax > 0, CTCSPEC_EINVAL, "ctc_loss: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, blank_id >= 0 && blank_id < Vp1, CTCSPEC_EINVAL, "ctc_loss: blank_id out of range");
  CTCSPEC_REQUIRE(ctx, Lmax <= kCtcMaxLabels && (long long)Vp1 * 4 <= 150 * 1024 && B <= 65535 && T <= 65535 * 32,
                  CTCSPEC_EUNSUPPORTED, "ctc_loss: Lmax <= %d, (V+1) * 4 bytes <= 150 KB (a row goes through LDS), B <= 65535",
                  kCtcMaxLabels);
  CTCSPEC_REQUIRE(ctx, aligned16(workspace), CTCSPEC_EINVAL, "ctc_loss: workspace must be 16-byte aligned");
  const CtcWorkspace w = ctc_workspace(B, T, Lmax);
  CTCSPEC_REQUIRE(ctx, workspace_bytes >= w.total, CTCSPEC_EINVAL, "ctc_loss: workspace of %zu bytes needed, %zu given",
                  w.total, workspace_bytes);
  unsigned char* ws = (unsigned char*)workspace;
  CtcParams p;
  p.logits = logits; p.labels = labels; p.label_len = label_len; p.frame_len = frame_len;
  p.B = B; p.T = T; p.Vp1 = Vp1; p.Lmax = Lmax; p.blank = blank_id;
  p.lse = (float*)(ws + w.lse); p.lpc = (float*)(ws + w.lpc); p.ag = (float*)(ws + w.ag);
  p.coff = (double*)(ws + w.coff);
  p.next = (int32_t*)(ws + w.next); p.first = (int32_t*)(ws + w.first);
  p.loss = loss; p.grad = grad;
  hipStream_t st = ctx->stream;
  const int row_lds = Vp1 * 4;
  static bool lds_allowed = false;  // raising the limit is needed once per process
  if (!lds_allowed) {
    CTCSPEC_HIP(ctx, hipFuncSetAttribute((const void*)ctc_row_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    CTCSPEC_HIP(ctx, hipFuncSetAttribute((const void*)ctc_grad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    lds_allowed = true;
  }
  hipLaunchKernelGGL(ctc_links_kernel, dim3(B), dim3(256), 0, st, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  hipLaunchKernelGGL(ctc_row_kernel, dim3(T, B), dim3(kCtcRowThreads), row_lds, st, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  const int S = 2 * Lmax + 1;
  int threads = (S + 63) / 64 * 64;
  threads = threads > 1024 ? 1024 : threads;
  const int ns = (S + threads - 1) / threads;
  const int dp_lds = 2 * (S + 4) * 4;
  switch (ns) {
    case 1: hipLaunchKernelGGL(ctc_dp_kernel<1>, dim3(B), dim3(threads), dp_lds, st, p); break;
    case 2: hipLaunchKernelGGL(ctc_dp_kernel<2>, dim3(B), dim3(threads), dp_lds, st, p); break;
    case 3: hipLaunchKernelGGL(ctc_dp_kernel<3>, dim3(B), dim3(threads), dp_lds, st, p); break;
    default: hipLaunchKernelGGL(ctc_dp_kernel<4>, dim3(B), dim3(threads), dp_lds, st, p); break;
  }
  CTCSPEC_HIP(ctx, hipGetLastError());
  if (grad) {
    hipLaunchKernelGGL(ctc_grad_kernel, dim3(T, B), dim3(kCtcRowThreads), row_lds, st, p);
    CTCSPEC_HIP(ctx, hipGetLastError());
  }
  return CTCSPEC_OK;
}
