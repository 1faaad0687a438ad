// A tile of a [V, D] x [cols, D]^T product, bf16 operands, fp32 accumulators: the main loop shared by the
// base-model head (verify_head_argmax) and the draft head with many columns.
//
// 8 wavefronts in a WR x WC grid (WR * WC = 8): wavefront (wr, wc) owns weight rows [64 wr, +64) x columns
// [16 CTW wc, +16 CTW) - 4 x CTW MFMA tiles.  Shapes in use (rows x columns, step): 128 x 64 and 128 x 128 with steps
// of 128 hidden elements (2 x 4 wavefronts, 64 x 16 or 64 x 32 per wavefront), and 256 x 128 with steps of 64
// (4 x 2 wavefronts, 64 x 64 per wavefront) for products with several column blocks: per flop it reads two thirds
// of the fragments from LDS and fetches half of the hidden-state tiles from L2.
// Per step both operands go through LDS: the W tile (nontemporal, the A operand) and the hidden states of the step
// (the B operand) are fetched by all threads together with coalesced 16-byte loads, DIST steps ahead, into
// rotating register stages (the VGPR file, 512 KB per compute unit, is the deep staging buffer), and written to
// one of two LDS buffers while the other one is computed from: one barrier per step.  Within a step the fragment
// reads of the next 32 k and the tile writes are issued in front of the MFMAs of the current 32 k and run under them.
// What bounds it (measured, one compute unit): b128 fragment reads at 128 B per clock, b128 writes at 79 B per
// clock - at 128 x 128, per step 192 KB read + 64 KB written = 2300 clocks against 1024 clocks of MFMA and 1.35 us
// (3200 clocks) for the 32 KB of W at the HBM rate, so the LDS work fits under the stream only if nothing
// serialises.  All loads are unconditional and counted (indices clamped; a request past the last step reads a
// block of zeros), so the waits name the loads that stay in flight.
#pragma once

#include <type_traits>
#include <utility>

#include "common.h"

namespace ctcspec {

constexpr int kTileWaves = 8;
constexpr int kTileStepK = 128;  // hidden elements per step of the 128-row shapes

template <int WR_, int CTW_, int STEPK_>
struct TileShape {
  static constexpr int WR = WR_, WC = kTileWaves / WR_;  // wavefront grid
  static constexpr int CTW = CTW_;                       // 16-column MFMA tiles per wavefront
  static constexpr int STEPK = STEPK_;                   // hidden elements per step
  static constexpr int ROWS = 64 * WR, COLS = 16 * CTW * WC;
  static constexpr int CPR = STEPK * 2 / 16;             // 16-byte chunks per staged row
  // bytes per staged row: the step's elements + 32.  A 16-byte LDS access of a wavefront is served 16 lanes per
  // clock, lanes {l .. l+7} together with {l+16 .. l+23} (what the conflict counter shows: a fragment read - lane =
  // row c, chunk g - is conflict-free when rows c .. c+7 at chunks g and g+1 fall on 16 different groups of 4
  // banks, i.e. when the pitch is 32 mod 64 bytes; at 128 + 16 bytes every read took one extra clock in four)
  static constexpr int PITCH = STEPK * 2 + 32;
  static constexpr int RPP = 64 * kTileWaves / CPR;      // rows that one 16-byte piece per thread covers
  static constexpr int WP = ROWS / RPP, HP = COLS / RPP;  // pieces per thread: W tile, hidden-state tile
  static constexpr int KK = STEPK / 32;                  // MFMA k-blocks per step
  static constexpr int HS_BYTES = COLS * PITCH, BUF_BYTES = (COLS + ROWS) * PITCH;
  static constexpr int LDS_BYTES = 2 * BUF_BYTES;
  static_assert(WR * WC == kTileWaves && ROWS % RPP == 0 && COLS % RPP == 0 && WP % KK == 0, "tile shape");
};
using Tile128x64 = TileShape<2, 1, 128>;
using Tile128x128 = TileShape<2, 2, 128>;
using Tile256x128 = TileShape<4, 4, 64>;

struct GemmTileArgs {
  const void* w;       // [V][D] bf16
  const void* hidden;  // [cols][D] bf16, first column of the tile
  const void* zeros;   // 256 bytes of zeros
  int D, V;            // D a multiple of the shape's step; both matrices smaller than 4 GB (32-bit byte offsets)
  int cols;            // live columns, 1 .. COLS
  int row_base;        // first weight row of the tile
};

typedef __attribute__((address_space(1))) u32x4 GlobalU32x4;  // a pointer made from an integer is generic otherwise

// acc[rt][ct][i]: row row_base + 64 wr + 16 rt + 4 (lane >> 4) + i, column 16 CTW wc + 16 ct + (lane & 15),
// wr = wave / WC, wc = wave % WC.
// Every wavefront of the workgroup (8) must call it; it ends with a barrier after the last read of LDS.
template <int DIST, typename SH>
__device__ __forceinline__ void gemm_tile(const GemmTileArgs& t, unsigned char* smem, f32x4 (&acc)[4][SH::CTW]) {
  constexpr int CTW = SH::CTW, STEPK = SH::STEPK, PITCH = SH::PITCH, CPR = SH::CPR, RPP = SH::RPP;
  constexpr int WP = SH::WP, HP = SH::HP, KK = SH::KK;
  constexpr int WPK = WP / KK, HPK = (HP + KK - 1) / KK;  // pieces written to LDS per 32 k of the step before
  constexpr int HS_BYTES = SH::HS_BYTES, BUF_BYTES = SH::BUF_BYTES;
  constexpr int TRIP = DIST % 2 == 0 ? DIST : 2 * DIST;    // steps per loop trip: stage and buffer static
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave / SH::WC, wc = wave % SH::WC;
  const int c = lane & 15, g = lane >> 4;
  const int row_base = t.row_base;
  const int total_steps = t.D / STEPK;
  // LDS: buffer b = hidden-state tile (COLS rows) then W tile (ROWS rows)

  // piece u of a thread: tile row prow + RPP u, 16-byte chunk pchunk; byte offsets in 32 bits (the host checks
  // that the matrices are smaller than 4 GB).  A wavefront covers whole rows (4 of 256 bytes or 8 of 128), and
  // the lanes are dealt so that the 16 lanes the LDS serves together write 256 bytes that cover every bank once:
  // both halves of one 256-byte row, or two 128-byte rows 4 apart (4 x 160 bytes = 32 banks further on).
  int prow, pchunk;
  if constexpr (CPR == 16) {
    prow = (tid >> 6) * 4 + ((lane >> 3) & 1) + 2 * (lane >> 5);
    pchunk = (lane & 7) + 8 * ((lane >> 4) & 1);
  } else {
    static_assert(CPR == 8, "rows of 128 or 256 bytes");
    const int j = (lane >> 3) & 7;
    prow = (tid >> 6) * 8 + ((j & 1) | ((j & 2) << 1) | ((j & 4) >> 1));
    pchunk = lane & 7;
  }
  const unsigned int lane_off = pchunk * 16;
  const uintptr_t w_addr = (uintptr_t)t.w, h_addr = (uintptr_t)t.hidden;
  const uintptr_t z_addr = (uintptr_t)t.zeros;
  unsigned int woff[WP], hoff[HP];
  const int dst0 = prow * PITCH + pchunk * 16;
#pragma unroll
  for (int u = 0; u < WP; ++u) {
    int row = row_base + prow + RPP * u;
    row = row < t.V ? row : t.V - 1;            // the ragged last block re-reads the last row
    woff[u] = (unsigned int)row * (unsigned int)(t.D * 2);
  }
#pragma unroll
  for (int u = 0; u < HP; ++u) {
    const int r = prow + RPP * u;
    const int col = r < t.cols ? r : t.cols - 1;  // columns past the end repeat the last one (never read back)
    hoff[u] = (unsigned int)col * (unsigned int)(t.D * 2);
  }
  // A request past the last step still issues its loads, so that every wait counts the same loads: it reads
  // a 256-byte block of zeros (in L2, no HBM traffic) and nothing computes from the result.
  u32x4 wreg[DIST][WP], hreg[DIST][HP];
  auto request = [&](int step, auto stage) __attribute__((always_inline)) {
    constexpr int S = decltype(stage)::value;
    // address arithmetic in integers: a select between pointers would become a branch around each load
    const bool valid = step < total_steps;
    const unsigned int mask = valid ? ~0u : 0u;
    const unsigned int st = ((unsigned int)step * (unsigned int)(2 * STEPK)) & mask;
    const uintptr_t hb = (valid ? h_addr : z_addr) + st, wb = (valid ? w_addr : z_addr) + st;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < HP; ++u) hreg[S][u] = *(const GlobalU32x4*)(hb + ((hoff[u] & mask) + lane_off));
#pragma unroll
    for (int u = 0; u < WP; ++u)
      wreg[S][u] = __builtin_nontemporal_load((const GlobalU32x4*)(wb + ((woff[u] & mask) + lane_off)));
    __builtin_amdgcn_sched_barrier(0);
  };
  auto commit = [&](auto stage, auto buffer) __attribute__((always_inline)) {
    constexpr int S = decltype(stage)::value, BUF = decltype(buffer)::value;
    unsigned char* hs = smem + BUF * BUF_BYTES;
    unsigned char* ws = hs + HS_BYTES;
#pragma unroll
    for (int u = 0; u < HP; ++u) *(u32x4*)(hs + (dst0 + u * RPP * PITCH)) = hreg[S][u];
#pragma unroll
    for (int u = 0; u < WP; ++u) *(u32x4*)(ws + (dst0 + u * RPP * PITCH)) = wreg[S][u];
  };
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int ct = 0; ct < CTW; ++ct) acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int aoff = (wr * 64 + c) * PITCH + g * 16, boff = (wc * 16 * CTW + c) * PITCH + g * 16;
  // compute one step from LDS buffer BUF; with COMMIT, also write stage S of the registers to the other buffer.
  // Per 32 k: the next fragments' reads and that k-block's share of the tile writes are issued, then the MFMAs of
  // the current fragments, under which those LDS operations run.
  auto compute = [&](auto buffer, auto with_commit, auto stage) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buffer)::value, S = decltype(stage)::value;
    constexpr bool COMMIT = decltype(with_commit)::value;
    const unsigned char* hs = smem + BUF * BUF_BYTES;
    const unsigned char* ws = hs + HS_BYTES;
    unsigned char* hs_next = smem + (1 - BUF) * BUF_BYTES;
    unsigned char* ws_next = hs_next + HS_BYTES;
    bf16x8 a[2][4], b[2][CTW];
    auto read_fragments = [&](int kk, int slot) __attribute__((always_inline)) {
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
        a[slot][rt] = __builtin_bit_cast(bf16x8, *(const u32x4*)(ws + (aoff + rt * 16 * PITCH + kk * 64)));
#pragma unroll
      for (int ct = 0; ct < CTW; ++ct)
        b[slot][ct] = __builtin_bit_cast(bf16x8, *(const u32x4*)(hs + (boff + ct * 16 * PITCH + kk * 64)));
    };
    __builtin_amdgcn_sched_barrier(0);
    read_fragments(0, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_barrier(0);
      if (kk + 1 < KK) read_fragments(kk + 1, (kk + 1) & 1);
      if constexpr (COMMIT) {
#pragma unroll
        for (int j = 0; j < HPK; ++j) {
          const int u = kk * HPK + j;
          if (u < HP) *(u32x4*)(hs_next + (dst0 + u * RPP * PITCH)) = hreg[S][u < HP ? u : 0];
        }
#pragma unroll
        for (int j = 0; j < WPK; ++j) {
          const int u = kk * WPK + j;
          *(u32x4*)(ws_next + (dst0 + u * RPP * PITCH)) = wreg[S][u];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct)
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
