// 128 weight rows x 64 or 128 columns of a [V, D] x [cols, D]^T product, bf16 operands, fp32 accumulators:
// the main loop shared by the base-model head (verify_head_argmax) and the draft head with many columns.
//
// 8 wavefronts in a 2 x 4 grid: wavefront (wr, wc) owns rows [64 wr, +64) x columns [16 CT wc, +16 CT) -
// 4 x CT MFMA tiles.  Per step of 128 hidden elements both operands go through LDS: the W tile (128 rows x
// 256 B, nontemporal, the A operand) and the hidden states of the step (64 CT columns x 256 B, the B operand)
// are fetched by all threads together with coalesced 16-byte loads, DIST steps ahead, into rotating register
// stages (the VGPR file, 512 KB per compute unit, is the deep staging buffer), and written to one of two LDS
// buffers while the other one is computed from: one barrier per step.  Within a step the fragment reads of
// the next 32 k and the tile writes are issued in front of the MFMAs of the current 32 k and run under them.
// What bounds it (measured, one compute unit): b128 fragment reads at 128 B per clock, b128 writes at 79 B per
// clock - with CT = 2, per step 192 KB read + 64 KB written = 2300 clocks against 1024 clocks of MFMA and 1.35 us
// (3200 clocks) for the 32 KB of W at the HBM rate, so the LDS work fits under the stream only if nothing
// serialises.  All loads are unconditional and counted (indices clamped; a request past the last step reads a
// block of zeros), so the waits name the loads that stay in flight.
#pragma once

#include <type_traits>
#include <utility>

#include "common.h"

namespace ctcspec {

constexpr int kTileWaves = 8;
constexpr int kTileStepK = 128;                     // hidden elements per step
constexpr int kTileRowPitch = 2 * kTileStepK + 32;  // bytes per staged row: 128 bf16 + pad; fragment reads (16 rows
                                                    // x 4 chunks per instruction) measure conflict-free at this pitch
template <int CT>
constexpr int tile_lds_bytes() { return 2 * (64 * CT + 128) * kTileRowPitch; }

struct GemmTileArgs {
  const void* w;       // [V][D] bf16
  const void* hidden;  // [cols][D] bf16, first column of the tile
  const void* zeros;   // 256 bytes of zeros
  int D, V;            // D a multiple of kTileStepK; both matrices smaller than 4 GB (32-bit byte offsets)
  int cols;            // live columns, 1 .. 64 CT
  int row_base;        // first weight row of the tile
};

typedef __attribute__((address_space(1))) u32x4 GlobalU32x4;  // a pointer made from an integer is generic otherwise

// acc[rt][ct][i]: row row_base + 64 wr + 16 rt + 4 (lane >> 4) + i, column 16 CT wc + 16 ct + (lane & 15).
// Every wavefront of the workgroup (8) must call it; it ends with a barrier after the last read of LDS.
template <int DIST, int CT>
__device__ __forceinline__ void gemm_tile_128(const GemmTileArgs& t, unsigned char* smem, f32x4 (&acc)[4][CT]) {
  constexpr int NTHREADS = 64 * kTileWaves;
  constexpr int PIECES = 128 * (2 * kTileStepK / 16) / NTHREADS;  // 16-byte pieces per thread and tile: 4
  constexpr int ROWS_PER_PIECE = NTHREADS / 16;                 // 32
  constexpr int KK = kTileStepK / 32;                             // MFMA k-blocks per step
  constexpr int TRIP = DIST % 2 == 0 ? DIST : 2 * DIST;         // steps per loop trip: stage and buffer static
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 2, wc = wave & 3;
  const int c = lane & 15, g = lane >> 4;
  const int row_base = t.row_base;
  const int total_steps = t.D / kTileStepK;
  // LDS: buffer b = hidden-state tile (COLS rows) then W tile (128 rows)
  constexpr int COLS = 64 * CT, HP = COLS * 16 / NTHREADS;  // columns of the tile; hidden-state pieces per thread
  constexpr int HS_BYTES = COLS * kTileRowPitch, BUF_BYTES = (COLS + 128) * kTileRowPitch;

  // piece u of a thread: tile row (tid >> 4) + 32 u, 16-byte chunk tid & 15; byte offsets in 32 bits (the host
  // checks that the matrices are smaller than 4 GB)
  const unsigned int lane_off = (tid & 15) * 16;
  const uintptr_t w_addr = (uintptr_t)t.w, h_addr = (uintptr_t)t.hidden;
  const uintptr_t z_addr = (uintptr_t)t.zeros;
  unsigned int woff[PIECES], hoff[HP];
  const int dst0 = (tid >> 4) * kTileRowPitch + (tid & 15) * 16;
#pragma unroll
  for (int u = 0; u < PIECES; ++u) {
    const int r = (tid >> 4) + ROWS_PER_PIECE * u;
    int row = row_base + r;
    row = row < t.V ? row : t.V - 1;            // the ragged last block re-reads the last row
    woff[u] = (unsigned int)row * (unsigned int)(t.D * 2);
    if (u < HP) {
      const int col = r < t.cols ? r : t.cols - 1;  // columns past the end repeat the last one (never read back)
      hoff[u] = (unsigned int)col * (unsigned int)(t.D * 2);
    }
  }
  // A request past the last step still issues its loads, so that every wait counts the same loads: it reads
  // a 256-byte block of zeros (in L2, no HBM traffic) and nothing computes from the result.
  u32x4 wreg[DIST][PIECES], hreg[DIST][HP];
  auto request = [&](int step, auto stage) __attribute__((always_inline)) {
    constexpr int S = decltype(stage)::value;
    // address arithmetic in integers: a select between pointers would become a branch around each load
    const bool valid = step < total_steps;
    const unsigned int mask = valid ? ~0u : 0u;
    const unsigned int st = ((unsigned int)step * (unsigned int)(2 * kTileStepK)) & mask;
    const uintptr_t hb = (valid ? h_addr : z_addr) + st, wb = (valid ? w_addr : z_addr) + st;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < HP; ++u) hreg[S][u] = *(const GlobalU32x4*)(hb + ((hoff[u] & mask) + lane_off));
#pragma unroll
    for (int u = 0; u < PIECES; ++u)
      wreg[S][u] = __builtin_nontemporal_load((const GlobalU32x4*)(wb + ((woff[u] & mask) + lane_off)));
    __builtin_amdgcn_sched_barrier(0);
  };
  auto commit = [&](auto stage, auto buffer) __attribute__((always_inline)) {
    constexpr int S = decltype(stage)::value, BUF = decltype(buffer)::value;
    unsigned char* hs = smem + BUF * BUF_BYTES;
    unsigned char* ws = hs + HS_BYTES;
#pragma unroll
    for (int u = 0; u < HP; ++u) *(u32x4*)(hs + (dst0 + u * ROWS_PER_PIECE * kTileRowPitch)) = hreg[S][u];
#pragma unroll
    for (int u = 0; u < PIECES; ++u) *(u32x4*)(ws + (dst0 + u * ROWS_PER_PIECE * kTileRowPitch)) = wreg[S][u];
  };
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int aoff = (wr * 64 + c) * kTileRowPitch + g * 16, boff = (wc * 16 * CT + c) * kTileRowPitch + g * 16;
  // compute one step from LDS buffer BUF; with COMMIT, also write stage S of the registers to the other buffer.
  // Per 32 k: the next fragments' reads and two of the tile writes are issued, then the eight MFMAs of the
  // current fragments, under which those LDS operations run.
  auto compute = [&](auto buffer, auto with_commit, auto stage) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buffer)::value, S = decltype(stage)::value;
    constexpr bool COMMIT = decltype(with_commit)::value;
    const unsigned char* hs = smem + BUF * BUF_BYTES;
    const unsigned char* ws = hs + HS_BYTES;
    unsigned char* hs_next = smem + (1 - BUF) * BUF_BYTES;
    unsigned char* ws_next = hs_next + HS_BYTES;
    bf16x8 a[2][4], b[2][CT];
    auto read_fragments = [&](int kk, int slot) __attribute__((always_inline)) {
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
        a[slot][rt] = __builtin_bit_cast(bf16x8, *(const u32x4*)(ws + (aoff + rt * 16 * kTileRowPitch + kk * 64)));
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
        b[slot][ct] = __builtin_bit_cast(bf16x8, *(const u32x4*)(hs + (boff + ct * 16 * kTileRowPitch + kk * 64)));
    };
    static_assert(PIECES == KK && HP <= KK, "per 32 k one W piece and at most one hidden-state piece are written");
    __builtin_amdgcn_sched_barrier(0);
    read_fragments(0, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_barrier(0);
      if (kk + 1 < KK) read_fragments(kk + 1, (kk + 1) & 1);
      if constexpr (COMMIT) {
        if (kk < HP) *(u32x4*)(hs_next + (dst0 + kk * ROWS_PER_PIECE * kTileRowPitch)) = hreg[S][kk < HP ? kk : 0];
        *(u32x4*)(ws_next + (dst0 + kk * ROWS_PER_PIECE * kTileRowPitch)) = wreg[S][kk];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
          acc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kk & 1][rt], b[kk & 1][ct], acc[rt][ct], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  using I0 = std::integral_constant<int, 0>;

  // The pipelined loop takes TRIP steps per trip with no exit in between (an exit inside the trip gives the
  // loop head a second, differently ordered set of loads in flight and the waits there fall back to draining
  // everything), so the total_steps % TRIP steps that do not fill a trip run first, unpipelined.
  const int lead = total_steps % TRIP;
  for (int i = 0; i < lead; ++i) {
    request(i, I0{});
    if (i > 0) lds_barrier();
    commit(I0{}, I0{});
    lds_barrier();
    compute(I0{}, std::false_type{}, I0{});
  }
  if (lead < total_steps) {
    // local step t = step - lead uses register stage t % DIST and LDS buffer t & 1
    [&]<int... U>(std::integer_sequence<int, U...>) __attribute__((always_inline)) {
      (request(lead + U, std::integral_constant<int, U>{}), ...);
    }(std::make_integer_sequence<int, DIST>{});
    if (lead > 0) lds_barrier();
    commit(I0{}, I0{});
    request(lead + DIST, I0{});
    lds_barrier();
    for (int t = lead; t < total_steps; t += TRIP) {
      [&]<int... U>(std::integer_sequence<int, U...>) __attribute__((always_inline)) {
        // step t + U: write step t + U + 1 (after the last step: zeros into the idle buffer), refill its stage
        ((compute(std::integral_constant<int, U & 1>{}, std::true_type{}, std::integral_constant<int, (U + 1) % DIST>{}),
          request(t + U + 1 + DIST, std::integral_constant<int, (U + 1) % DIST>{}), lds_barrier()),
         ...);
      }(std::make_integer_sequence<int, TRIP>{});
    }
  }

}

}  // namespace ctcspec
