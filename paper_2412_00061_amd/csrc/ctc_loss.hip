// ctc_loss: the training objective of Sec. 3.2 - the negative log of Eq. 5 for a label sequence - and its gradient
// with respect to the logits, by the forward-backward recursions of the CTC paper the section cites.
//
// Two kinds of work, kept apart:
//   * the rows of logits ([V+1] floats per frame, 128 KB at V = 32000) are what costs HBM time.  Each is read
//     once and its gradient row written once, by one workgroup that holds the row in registers: ctc_row_kernel takes
//     the log-sum-exp, picks out the few log-probabilities the recursions need (the label's tokens and the
//     blank) and writes the row's softmax as the gradient; after the recursions ctc_fix_kernel subtracts the
//     occupancies from those few entries.
//   * the recursions themselves are KB-sized and sequential in the frames: ctc_dp_kernel, one workgroup per
//     sequence and direction, a thread per state of the extended sequence (blank, y1, blank, ..., blank), the neighbours'
//     values through LDS, one barrier per frame.  The forward and the backward recursion of a sequence run at
//     the same time in two workgroups; the occupancy gamma_t(s) = alpha_t(s) beta_t(s) / (p_t(z_s) P) is formed
//     where it is used.
// A token that occurs several times in a label has several states; their occupancies are added in label order
// by the thread of the first occurrence (links built once per sequence), so no atomic is needed and the result
// has the same bits on every run.
#include "common.h"

namespace ctcspec {

typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kCtcMaxLabels = 2047;  // L + 1 pairs of states <= 2 per thread of a 1024-thread workgroup
constexpr int kCtcRowThreads = 1024;  // with two label positions per thread: kCtcMaxLabels + 1 <= 2 * kCtcRowThreads
constexpr int kCtcMaxRow = 16 * kCtcRowThreads * 4;  // 65536 symbols: 16 16-byte loads per thread
constexpr int kCtcFixThreads = 256;
constexpr int kCtcAhead = 8;  // frames between a load and its use in the recursions

static_assert(kCtcMaxLabels + 1 <= 2 * kCtcRowThreads, "ctc_row_kernel fetches two label positions per thread");

struct CtcParams {
  const float* logits;      // [B][T][Vp1]
  const int32_t* labels;    // [B][Lmax]
  const int32_t* label_len; // [B]
  const int32_t* frame_len; // [B]
  int B, T, Vp1, Lmax, blank;
  // workspace
  float* lpc;     // [B][T][Lmax + 1]: log2 p_t(y_j) for j < L, log2 p_t(blank) at Lmax
  float* ag;      // [B][T][2 Lmax + 2]: log2 alpha minus the frame's offset (state s at s; the last entry unused)
  float* bg;      // [B][T][2 Lmax + 2]: log2 beta minus the frame's offset
  double* coff_a; // [B][T]: offset of the frame's log alpha values
  double* coff_b; // [B][T]: offset of the frame's log beta values
  double* logp;   // [B]: log2 P(Y | X)
  int32_t* next;  // [B][Lmax]: next label position with the same token, -1: none
  int32_t* first; // [B][Lmax]: 1 when no earlier position holds the same token
  // outputs
  float* loss;    // [B]
  float* grad;    // [B][T][Vp1] or null
};

// The recursions run on base-2 logarithms (ctc_row_kernel hands out log2 p, the loss is turned back at the end):
// the exp2 and log2 instructions then need no scaling of their argument or result.
// log2(2^a + 2^b + 2^c) without a branch; -inf stands for an impossible state and any of the three may be -inf.
// The bare instructions carry an absolute error near 1e-7 here (the arguments of exp2 are <= 0, the argument of
// log2 is in [1, 3]; a term below 2^-126 of the largest is dropped), far below what the occupancies need.
__device__ __forceinline__ float ctc_log_add3(float a, float b, float c) {
  const float m = fmaxf(fmaxf(a, b), c);
  const float ms = m > -INFINITY ? m : 0.f;
  const float sum = __builtin_amdgcn_exp2f(a - ms) + __builtin_amdgcn_exp2f(b - ms) + __builtin_amdgcn_exp2f(c - ms);
  return ms + __builtin_amdgcn_logf(sum);  // the bare log2 instruction; sum = 0 gives -inf
}
// the reference value a frame's results are stored against: the largest value of the frame before, 0 when every
// state is impossible, so that offsets stay finite
__device__ __forceinline__ float frame_shift(float frame_max) { return frame_max > -INFINITY ? frame_max : 0.f; }
__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }
// floats per frame in the alpha and beta arrays: the 2 Lmax + 1 states and one more, so that pairs of states sit
// on 8-byte boundaries
__host__ __device__ __forceinline__ int ctc_state_pitch(int Lmax) { return 2 * Lmax + 2; }

// per sequence: links between the label positions that hold the same token.  The label is staged in LDS; one
// wavefront per position looks for the nearest later position with the same token and for any earlier one, 256
// candidates per round trip to LDS.  The positions of a sequence are dealt to gridDim.y workgroups; every entry
// of next and first is written by the wavefront that owns the position, so the workgroups share nothing.
__global__ __launch_bounds__(1024) void ctc_links_kernel(CtcParams p) {
  extern __shared__ int32_t ytok[];  // [Lmax]
  const int b = blockIdx.x, tid = threadIdx.x, n = blockDim.x;
  const int lane = tid & 63, nwaves = n >> 6;
  const int wave = (tid >> 6) + nwaves * blockIdx.y, stride = nwaves * gridDim.y;
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  int32_t* next = p.next + (size_t)b * p.Lmax;
  int32_t* first = p.first + (size_t)b * p.Lmax;
  for (int j = tid; j < L; j += n) ytok[j] = p.labels[(size_t)b * p.Lmax + j];
  __syncthreads();
  for (int j = wave; j < p.Lmax; j += stride) {
    int found = -1;
    bool earlier = false;
    if (j < L) {
      const int tok = ytok[j];
      for (int i0 = j + 1; i0 < L && found < 0; i0 += 256) {
        unsigned long long hits[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i = i0 + 64 * r + lane;
          hits[r] = __ballot(i < L && ytok[i] == tok);
        }
#pragma unroll
        for (int r = 3; r >= 0; --r)
          if (hits[r]) found = i0 + 64 * r + __ffsll((long long)hits[r]) - 1;  // the lowest group with a hit wins
      }
      for (int i0 = 0; i0 < j && !earlier; i0 += 256) {
        unsigned long long any = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i = i0 + 64 * r + lane;
          any |= __ballot(i < j && ytok[i] == tok);
        }
        earlier = any != 0;
      }
    }
    if (lane == 0) {
      next[j] = found;
      first[j] = (j < L && !earlier) ? 1 : 0;
    }
  }
}

// One workgroup per frame row, the row held in registers: every load of the row is in flight before the first
// is used, then log-sum-exp, the few log-probabilities the recursions need (the label's tokens and the blank),
// and the row's softmax written as the gradient.  Rows start at any multiple of 4 bytes (V + 1 is odd at
// V = 32000), so the up to three elements in front of the first 16-byte boundary and behind the last go through
// single lanes and the body through 16-byte loads and stores.
template <int NV, int THREADS>  // 16-byte loads per thread: NV * THREADS * 4 >= V + 1
__global__ __launch_bounds__(THREADS) void ctc_row_kernel(CtcParams p) {
  __shared__ float red[THREADS / 64];
  const int t = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int Tb = clampi(p.frame_len[b], 0, p.T);
  const size_t row0 = ((size_t)b * p.T + t) * p.Vp1;
  int head = (int)((4 - (row0 & 3)) & 3);
  head = head < p.Vp1 ? head : p.Vp1;
  const int nvec = (p.Vp1 - head) >> 2;
  const int tail0 = head + 4 * nvec;
  // the lane of an edge element: lanes 0..2 take the head, lanes 64..66 the tail
  int edge = -1;
  if (tid < head) edge = tid;
  else if (tid >= 64 && tid - 64 < p.Vp1 - tail0) edge = tail0 + tid - 64;
  float* g = p.grad ? p.grad + row0 : nullptr;
  if (t >= Tb) {  // frames past the sequence: no gradient
    if (g) {
      f32x4* gv = (f32x4*)(g + head);
      for (int i = tid; i < nvec; i += THREADS) gv[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (edge >= 0) g[edge] = 0.f;
    }
    return;
  }
  const float* z = p.logits + row0;
  const f32x4* zv = (const f32x4*)(z + head);
  // the label's token ids first (kCtcMaxLabels < 2 * THREADS: two per thread), then the row, then the label's
  // logits while the row's cache lines are still on their way - asked for later they come from HBM a second time
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  int yid[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int j = tid + r * THREADS;
    yid[r] = j < L ? clampi(p.labels[(size_t)b * p.Lmax + j], 0, p.Vp1 - 1) : p.blank;
  }
  f32x4 x[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = tid + k * THREADS;
    x[k] = i < nvec ? zv[i] : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  }
  float xe = edge >= 0 ? z[edge] : -INFINITY;
  const float zy[2] = {z[yid[0]], z[yid[1]]};
  float mx = xe;
#pragma unroll
  for (int k = 0; k < NV; ++k) mx = fmaxf(fmaxf(fmaxf(mx, x[k][0]), fmaxf(x[k][1], x[k][2])), x[k][3]);
  mx = wave_max_f32(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < THREADS / 64; ++w) mx = fmaxf(mx, red[w]);
  // e = exp(x - max) stays in the registers: the softmax is e / sum
  xe = expf(xe - mx);
  float sum = xe;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x[k][c] = expf(x[k][c] - mx);
      sum += x[k][c];
    }
  }
  sum = wave_sum_f32(sum);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = sum;
  __syncthreads();
  sum = 0.f;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) sum += red[w];
  const float lse = mx + logf(sum);
  float* out = p.lpc + ((size_t)b * p.T + t) * (p.Lmax + 1);
  constexpr float kLog2e = 1.4426950408889634f;  // the recursions take base-2 logarithms
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int j = tid + r * THREADS;
    if (j < L) out[j] = (zy[r] - lse) * kLog2e;
    else if (j == L) out[p.Lmax] = (zy[r] - lse) * kLog2e;  // this thread's spare slot fetched the blank
  }
  if (g) {
    const float inv = 1.f / sum;
    f32x4* gv = (f32x4*)(g + head);
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = tid + k * THREADS;
      if (i < nvec) gv[i] = x[k] * inv;
    }
    if (edge >= 0) g[edge] = xe * inv;
  }
}

// log2(2^a + 2^b) without a branch (see ctc_log_add3)
__device__ __forceinline__ float ctc_log_add2(float a, float b) {
  const float m = fmaxf(a, b);
  const float ms = m > -INFINITY ? m : 0.f;
  const float sum = __builtin_amdgcn_exp2f(a - ms) + __builtin_amdgcn_exp2f(b - ms);
  return ms + __builtin_amdgcn_logf(sum);
}

// Two workgroups per sequence, on different compute units at the same time: blockIdx.y = 0 runs the forward
// recursion (log alpha, the loss), blockIdx.y = 1 the backward one (log beta).  Neither needs the other's values;
// the occupancies that need both are formed afterwards, in ctc_fix_kernel.
//
// A thread owns pairs of states: pair q is the blank in front of label position q (state 2q) and that label's own
// state (2q + 1); pair L is the final blank alone.  The two states of a pair share their neighbours' values (three
// LDS reads forward, four backward, instead of three per state), the blank needs a two-way log-add and only the
// label a three-way one, and no lane has to find out which kind of state it holds.
template <int NP>  // pairs per thread
__global__ __launch_bounds__(1024) void ctc_dp_kernel(CtcParams p) {
  extern __shared__ __attribute__((aligned(16))) float lds[];  // two rows of 2 Lmax + 6 values, -inf around the states
  const int b = blockIdx.x, tid = threadIdx.x, nthreads = blockDim.x;
  const bool backward = blockIdx.y != 0;
  const int SP = ctc_state_pitch(p.Lmax);
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  const int S = 2 * L + 1;
  const int Tb = clampi(p.frame_len[b], 0, p.T);
  const int pitch = 2 * p.Lmax + 6;  // even: state 2q of either row sits on an 8-byte boundary
  // The largest value of a frame: every wavefront's maximum goes into one LDS word with an atomic max.  Three
  // words in turn: frame t collects into word t % 3, reads word (t - 1) % 3 and resets word (t + 1) % 3, which
  // was last read before the barrier of frame t - 1 and is next written after the barrier of frame t.
  __shared__ float fmax3[3];
  const int32_t* y = p.labels + (size_t)b * p.Lmax;
  const float* lpc = p.lpc + (size_t)b * p.T * (p.Lmax + 1);
  if (Tb == 0) {
    if (tid == 0 && !backward) {
      p.loss[b] = L == 0 ? 0.f : INFINITY;
      p.logp[b] = L == 0 ? 0.0 : -(double)INFINITY;
    }
    return;
  }
  // per pair of this thread: whether the pair (its blank) and its label state exist, the label's entry in a
  // frame's compact row, and whether the transition that skips the blank exists into the label state (from
  // state 2q - 1) / out of it (to state 2q + 3)
  int col[NP];
  bool has_pair[NP], has_label[NP], skip_in[NP], skip_out[NP];
#pragma unroll
  for (int u = 0; u < NP; ++u) {
    const int q = tid + u * nthreads;
    has_pair[u] = q <= L;
    has_label[u] = q < L;
    col[u] = q < L ? q : p.Lmax;  // pairs without a label read the blank's entry and drop it
    skip_in[u] = q >= 1 && q < L && y[q] != y[q - 1];
    skip_out[u] = q + 1 < L && y[q] != y[q + 1];
  }
  for (int i = tid; i < 2 * pitch; i += nthreads) lds[i] = -INFINITY;
  if (tid < 3) fmax3[tid] = -INFINITY;
  __syncthreads();

  // A frame's log-probabilities are loaded several frames before the frame's turn, into a ring of registers: the
  // chain from frame to frame then runs through LDS and arithmetic only.  The barrier of a frame orders LDS
  // alone, so these loads and the stores of the frame's results stay in flight across it.
  constexpr int AHEAD = kCtcAhead;
  const int lp_pitch = p.Lmax + 1;
  float lpr[AHEAD][NP], lpb[AHEAD];

  if (!backward) {
    float* ag = p.ag + (size_t)b * p.T * SP;
    double* coff = p.coff_a + (size_t)b * p.T;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) {
      const int tt = i < Tb ? i : Tb - 1;
      lpb[i] = lpc[(size_t)tt * lp_pitch + p.Lmax];
#pragma unroll
      for (int u = 0; u < NP; ++u) lpr[i][u] = lpc[(size_t)tt * lp_pitch + col[u]];
    }
    double c_alpha = 0.0;  // the stored values of the frame are log alpha - c_alpha
    int slot_prev = 2, slot = 0, slot_next = 1;
    for (int t0 = 0; t0 < Tb; t0 += AHEAD) {
#pragma unroll
      for (int i = 0; i < AHEAD; ++i) {
        const int t = t0 + i;
        if (t < Tb) {
          float* cur = lds + 2 + (t & 1) * pitch;  // offsets, not a table of pointers: keeps these LDS accesses
          const float* prev = lds + 2 + ((t & 1) ^ 1) * pitch;
          float shift = 0.f;
          if (t > 0) {
            shift = frame_shift(fmax3[slot_prev]);
            c_alpha += (double)shift;
          }
          float mine = -INFINITY;
#pragma unroll
          for (int u = 0; u < NP; ++u) {
            const int q = tid + u * nthreads;
            if (has_pair[u]) {
              float a_blank, a_label;
              if (t == 0) {
                a_blank = q == 0 ? 0.f : -INFINITY;
                a_label = q == 0 ? 0.f : -INFINITY;
              } else {
                const float before = prev[2 * q - 1];
                const f32x2 own = *(const f32x2*)(prev + 2 * q);
                a_blank = ctc_log_add2(own[0], before);
                a_label = ctc_log_add3(own[1], own[0], skip_in[u] ? before : -INFINITY);
              }
              a_blank += lpb[i] - shift;
              a_label = has_label[u] ? a_label + (lpr[i][u] - shift) : -INFINITY;
              const f32x2 both = {a_blank, a_label};
              *(f32x2*)(cur + 2 * q) = both;
              *(f32x2*)(ag + (size_t)t * SP + 2 * q) = both;
              mine = fmaxf(mine, fmaxf(a_blank, a_label));
            }
          }
          mine = wave_max_f32(mine);
          if ((tid & 63) == 0) __hip_atomic_fetch_max(&fmax3[slot], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          if (tid == 0) {
            fmax3[slot_next] = -INFINITY;
            coff[t] = c_alpha;
          }
          slot_prev = slot; slot = slot_next; slot_next = slot_next == 2 ? 0 : slot_next + 1;
          const int tn = t + AHEAD < Tb ? t + AHEAD : Tb - 1;
          lpb[i] = lpc[(size_t)tn * lp_pitch + p.Lmax];
#pragma unroll
          for (int u = 0; u < NP; ++u) lpr[i][u] = lpc[(size_t)tn * lp_pitch + col[u]];
          lds_barrier();
        }
      }
    }
    const float* last = lds + 2 + ((Tb - 1) & 1) * pitch;
    const float tail = ctc_log_add2(last[S - 1], S > 1 ? last[S - 2] : -INFINITY);
    const double logP = c_alpha + (double)tail;  // base 2; -inf when the label cannot be reached
    if (tid == 0) {
      p.loss[b] = (float)(-logP * 0.6931471805599453);
      p.logp[b] = logP;
    }
  } else {
    float* bg = p.bg + (size_t)b * p.T * SP;
    double* coff = p.coff_b + (size_t)b * p.T;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) {
      const int tt = Tb - 1 - i >= 0 ? Tb - 1 - i : 0;
      lpb[i] = lpc[(size_t)tt * lp_pitch + p.Lmax];
#pragma unroll
      for (int u = 0; u < NP; ++u) lpr[i][u] = lpc[(size_t)tt * lp_pitch + col[u]];
    }
    double c_beta = 0.0;  // the stored values of the frame are log beta - c_beta
    int slot_prev = 2, slot = 0, slot_next = 1;
    for (int t0 = Tb - 1; t0 >= 0; t0 -= AHEAD) {
#pragma unroll
      for (int i = 0; i < AHEAD; ++i) {
        const int t = t0 - i;
        if (t >= 0) {
          float* cur = lds + 2 + (t & 1) * pitch;
          const float* nxt = lds + 2 + ((t & 1) ^ 1) * pitch;
          float shift = 0.f;
          if (t < Tb - 1) {
            shift = frame_shift(fmax3[slot_prev]);
            c_beta += (double)shift;
          }
          float mine = -INFINITY;
#pragma unroll
          for (int u = 0; u < NP; ++u) {
            const int q = tid + u * nthreads;
            if (has_pair[u]) {
              float b_blank, b_label;
              if (t == Tb - 1) {
                b_blank = q == L ? 0.f : -INFINITY;
                b_label = q == L - 1 ? 0.f : -INFINITY;
              } else {
                const f32x2 own = *(const f32x2*)(nxt + 2 * q);        // states 2q, 2q + 1
                const f32x2 after = *(const f32x2*)(nxt + 2 * q + 2);  // states 2q + 2, 2q + 3
                b_blank = ctc_log_add2(own[0], own[1]);
                b_label = ctc_log_add3(own[1], after[0], skip_out[u] ? after[1] : -INFINITY);
              }
              b_blank += lpb[i] - shift;  // beta_t(s) includes p_t(z_s)
              b_label = has_label[u] ? b_label + (lpr[i][u] - shift) : -INFINITY;
              const f32x2 both = {b_blank, b_label};
              *(f32x2*)(cur + 2 * q) = both;
              *(f32x2*)(bg + (size_t)t * SP + 2 * q) = both;
              mine = fmaxf(mine, fmaxf(b_blank, b_label));
            }
          }
          mine = wave_max_f32(mine);
          if ((tid & 63) == 0) __hip_atomic_fetch_max(&fmax3[slot], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          if (tid == 0) {
            fmax3[slot_next] = -INFINITY;
            coff[t] = c_beta;
          }
          slot_prev = slot; slot = slot_next; slot_next = slot_next == 2 ? 0 : slot_next + 1;
          const int tn = t - AHEAD >= 0 ? t - AHEAD : 0;
          lpb[i] = lpc[(size_t)tn * lp_pitch + p.Lmax];
#pragma unroll
          for (int u = 0; u < NP; ++u) lpr[i][u] = lpc[(size_t)tn * lp_pitch + col[u]];
          lds_barrier();
        }
      }
    }
  }
}

// One wavefront per frame: the occupancies gamma_t(s) = alpha_t(s) beta_t(s) / (p_t(z_s) P) of the label's tokens
// and of the blank come off the softmax in the gradient row.  Only these few entries of the row are touched.
__global__ __launch_bounds__(kCtcFixThreads) void ctc_fix_kernel(CtcParams p) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (kCtcFixThreads / 64) + (threadIdx.x >> 6), b = blockIdx.y;
  const int Tb = clampi(p.frame_len[b], 0, p.T);
  if (t >= Tb) return;  // rows past the sequence were written as zeros
  float* __restrict__ g = p.grad + ((size_t)b * p.T + t) * p.Vp1;
  const double logP = p.logp[b];
  if (!(logP > -(double)INFINITY)) {  // a label that cannot be reached has no gradient
    for (int v = lane; v < p.Vp1; v += 64) g[v] = 0.f;
    return;
  }
  const int L = clampi(p.label_len[b], 0, p.Lmax);
  const int SP = ctc_state_pitch(p.Lmax);
  const size_t frame = (size_t)b * p.T + t;
  const float* __restrict__ al = p.ag + frame * SP;
  const float* __restrict__ be = p.bg + frame * SP;
  const float* __restrict__ lp = p.lpc + frame * (p.Lmax + 1);
  // log of P over the two offsets of this frame: what the stored alpha + beta - log p is measured against
  const float z = (float)(logP - p.coff_a[frame] - p.coff_b[frame]);
  auto gamma = [&](int s, float l) {
    const float a = al[s], bt = be[s];
    return (a > -INFINITY && bt > -INFINITY) ? exp2f(a + bt - l - z) : 0.f;  // base-2 logarithms throughout
  };
  // The occupancies of a frame sum to one (every alignment is in exactly one state at frame t).  What is left
  // of the recursions' rounding after thousands of frames is mostly common to all states of a frame - it sits in
  // z - so dividing by the computed sum removes it.  First pass: the sums, in a fixed order.
  const float lblank = lp[p.Lmax];
  float gb = 0.f, go = 0.f;
#pragma unroll 4
  for (int s = 2 * lane; s < 2 * L + 1; s += 128) gb += gamma(s, lblank);
#pragma unroll 4
  for (int j = lane; j < L; j += 64) go += gamma(2 * j + 1, lp[j]);
  gb = wave_sum_f32(gb);
  go = wave_sum_f32(go);
  const float total = gb + go;
  const float inv = total > 0.f ? 1.f / total : 1.f;
  // the blank: all even states
  // The entries are written, not updated: the softmax value that ctc_row_kernel left there is formed again from
  // the log-probability at hand, which saves fetching a cache line per entry.
  if (lane == 0) g[p.blank] = exp2f(lblank) - gb * inv;
  // the label's tokens: the lane of a token's first position adds the occupancies of all its positions (nearly
  // always just the one, so every lane forms its own position's occupancy first and the loads of several
  // positions are in flight together)
  const int32_t* __restrict__ y = p.labels + (size_t)b * p.Lmax;
  const int32_t* __restrict__ nx = p.next + (size_t)b * p.Lmax;
  const int32_t* __restrict__ fs = p.first + (size_t)b * p.Lmax;
#pragma unroll 4
  for (int j = lane; j < L; j += 64) {
    const int is_first = fs[j];
    const int tok = clampi(y[j], 0, p.Vp1 - 1);
    const float l = lp[j];
    float tot = gamma(2 * j + 1, l);
    if (is_first) {
      for (int i = nx[j]; i >= 0; i = nx[i]) tot += gamma(2 * i + 1, lp[i]);
      if (tok != p.blank) g[tok] = exp2f(l) - tot * inv;  // a label never holds the blank; ids come from the caller
    }
  }
}

struct CtcWorkspace {
  size_t lpc, ag, bg, coff_a, coff_b, logp, next, first, total;
};
static CtcWorkspace ctc_workspace(int B, int T, int Lmax) {
  CtcWorkspace w;
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t at = off; off = (off + bytes + 255) / 256 * 256; return at; };
  w.lpc = carve((size_t)B * T * (Lmax + 1) * 4);
  w.ag = carve((size_t)B * T * ctc_state_pitch(Lmax) * 4);
  w.bg = carve((size_t)B * T * ctc_state_pitch(Lmax) * 4);
  w.coff_a = carve((size_t)B * T * 8);
  w.coff_b = carve((size_t)B * T * 8);
  w.logp = carve((size_t)B * 8);
  w.next = carve((size_t)B * Lmax * 4);
  w.first = carve((size_t)B * Lmax * 4);
  w.total = off;
  return w;
}

// code of this translation unit loaded onto the current device (context creation calls this: a stage call never
// triggers a load, so it can be the first thing a stream capture records)
hipError_t prepare_ctc_loss() {
  hipFuncAttributes attr;
  return hipFuncGetAttributes(&attr, (const void*)ctc_links_kernel);
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
  if (const int owed = flush_deferred(ctx)) return owed;
  CTCSPEC_REQUIRE(ctx, logits && labels && label_len && frame_len && workspace && loss, CTCSPEC_EINVAL,
                  "ctc_loss: null pointer");
  CTCSPEC_REQUIRE(ctx, B > 0 && T > 0 && Vp1 > 0 && Lmax > 0, CTCSPEC_EINVAL, "ctc_loss: sizes must be positive");
  CTCSPEC_REQUIRE(ctx, blank_id >= 0 && blank_id < Vp1, CTCSPEC_EINVAL, "ctc_loss: blank_id out of range");
  CTCSPEC_REQUIRE(ctx, Lmax <= kCtcMaxLabels && Vp1 <= kCtcMaxRow && B <= 65535 && T <= 65535 * 32,
                  CTCSPEC_EUNSUPPORTED, "ctc_loss: Lmax <= %d, V+1 <= %d (a row is held in one workgroup's registers), B <= 65535",
                  kCtcMaxLabels, kCtcMaxRow);
  CTCSPEC_REQUIRE(ctx, aligned16(workspace) && aligned16(logits) && (!grad || aligned16(grad)), CTCSPEC_EINVAL,
                  "ctc_loss: logits, grad and workspace must be 16-byte aligned");
  const CtcWorkspace w = ctc_workspace(B, T, Lmax);
  CTCSPEC_REQUIRE(ctx, workspace_bytes >= w.total, CTCSPEC_EINVAL, "ctc_loss: workspace of %zu bytes needed, %zu given",
                  w.total, workspace_bytes);
  unsigned char* ws = (unsigned char*)workspace;
  CtcParams p;
  p.logits = logits; p.labels = labels; p.label_len = label_len; p.frame_len = frame_len;
  p.B = B; p.T = T; p.Vp1 = Vp1; p.Lmax = Lmax; p.blank = blank_id;
  p.lpc = (float*)(ws + w.lpc); p.ag = (float*)(ws + w.ag);
  p.bg = (float*)(ws + w.bg);
  p.coff_a = (double*)(ws + w.coff_a); p.coff_b = (double*)(ws + w.coff_b); p.logp = (double*)(ws + w.logp);
  p.next = (int32_t*)(ws + w.next); p.first = (int32_t*)(ws + w.first);
  p.loss = loss; p.grad = grad;
  hipStream_t st = ctx->stream;
  const int link_blocks = Lmax > 256 ? (Lmax + 127) / 128 : 1;  // eight positions per wavefront at the most
  hipLaunchKernelGGL(ctc_links_kernel, dim3(B, link_blocks), dim3(Lmax > 256 ? 1024 : 256), Lmax * 4, st, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  const int nv = (Vp1 / 4 + kCtcRowThreads - 1) / kCtcRowThreads;  // 16-byte loads per thread
  const dim3 rows(T, B), row_threads(kCtcRowThreads);
  if (nv <= 1) hipLaunchKernelGGL((ctc_row_kernel<1, kCtcRowThreads>), rows, row_threads, 0, st, p);
  else if (nv <= 2) hipLaunchKernelGGL((ctc_row_kernel<2, kCtcRowThreads>), rows, row_threads, 0, st, p);
  else if (nv <= 4) hipLaunchKernelGGL((ctc_row_kernel<4, kCtcRowThreads>), rows, row_threads, 0, st, p);
  else if (nv <= 8) hipLaunchKernelGGL((ctc_row_kernel<8, kCtcRowThreads>), rows, row_threads, 0, st, p);
  else hipLaunchKernelGGL((ctc_row_kernel<16, kCtcRowThreads>), rows, row_threads, 0, st, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  const int pairs = Lmax + 1;  // a blank and a label state each; the last one is the final blank alone
  int threads = (pairs + 63) / 64 * 64;
  threads = threads > 1024 ? 1024 : threads;
  const int np = (pairs + threads - 1) / threads;
  const int dp_lds = 2 * (2 * Lmax + 6) * 4;
  const dim3 dp_grid(B, grad ? 2 : 1);  // without a gradient only the forward recursion runs
  if (np <= 1) hipLaunchKernelGGL(ctc_dp_kernel<1>, dp_grid, dim3(threads), dp_lds, st, p);
  else hipLaunchKernelGGL(ctc_dp_kernel<2>, dp_grid, dim3(threads), dp_lds, st, p);
  CTCSPEC_HIP(ctx, hipGetLastError());
  if (grad) {
    const int per = kCtcFixThreads / 64;
    hipLaunchKernelGGL(ctc_fix_kernel, dim3((T + per - 1) / per, B), dim3(kCtcFixThreads), 0, st, p);
    CTCSPEC_HIP(ctx, hipGetLastError());
  }
  return CTCSPEC_OK;
}
