// Variable-K grouped GEMM of training for gfx950 (MI355X): the weight gradient of the expert layer whose forward
// pass is the grouped GEMM of gemm_kernel.h (paper Sec. 2.1), computed without padding any group (the capability
// of Sec. 2.2 carried over to the contraction dimension).  The paper's title names training and its Sec. 4 the
// kernels around the grouped GEMM, but it defines no layouts or scale granularity for this operation; the
// definition below is this library's own reading.
//
//   dW[g][n][k] = sum over token blocks j, ascending, of
//                 SDY[j][n] * SX[j][k] * sum_{tokens r in block j and in group g} dec(DYT[n][r]) * dec(XT[k][r])
//
// XT [K, M_total] and DYT [N, M_total] are e4m3 bytes with the token index contiguous (both operands of the
// contraction are then "row x 128 bytes" slabs, as in the forward kernel), SX [ceil(M_total/128), K] and
// SDY [ceil(M_total/128), N] hold one fp32 scale per block of 128 tokens and row (block-major: the 256 + 128 scales
// a tile needs for one block are 12 cache lines; row-major they would be 384, as many requests as the operand
// tiles themselves), the blocks being [128 j, 128 j + 128) of the concatenated token axis whatever the groups
// are, and dW [G, N, K] is fp32 (or bfloat16).
// Group boundaries may fall anywhere: the first and the last block of a group are fetched whole (16-byte aligned,
// like every other block) and the bytes of tokens outside the group are cleared in registers, in BOTH operands, so
// that a neighbouring group's bytes (NaN codes included) never reach a product.  A group without tokens gives zeros.
//
// Structure: persistent workgroups (8 waves, 4 along k x 2 along n) walk the output tiles of 256 features x 128
// rows of dY^T; per token block the two operand tiles and their scales go global -> LDS by DMA into a ring of 3
// buffers, swizzled like the forward kernels' tiles, and the fetch stream runs three blocks ahead of the arithmetic
// across tile boundaries (a group of 1000 tokens is 8 blocks: without that, every tile would start with an empty
// pipeline and end with an idle one).  A wave holds the 4 + 4 operand fragments and the scales of the block it
// multiplies in registers and refills them from the next block's buffer while it multiplies, and 64 x 64 fp32
// accumulators; one v_mfma_f32_16x16x128_f8f6f4 from zero per scale block (dY^T fragment first, and the features
// permuted on their way into LDS: an output row's 16 lanes then hold 32 consecutive features, two each), then
// acc += p * (sdy * sx) with sdy one of the lane's four dY^T rows and sx the lane's feature: 8 vector instructions
// per matrix instruction (the factor differs per output element, not per lane as in the forward pass).
#pragma once
#include "gemm_kernel.h"

namespace gg {

struct WgradArgs {
  const uint8_t* XT;    // [K, M_total]
  const float* SX;      // [MB, K]
  const uint8_t* DYT;   // [N, M_total]
  const float* SDY;     // [MB, N]
  const int32_t* off;   // [G + 1]
  float* dW;            // [G, N, K] fp32, or bfloat16 in the OUT16 instantiation
  int G, M_total, N, K, MB;
  int n_tiles, k_tiles;   // N / 128, K / 256
  int tiles;              // G * n_tiles * k_tiles
  int slots;              // workgroups per XCD when the grid is a multiple of 8, else 0 (plain round-robin)
  int blocked;            // 1: a group's tiles are listed in blocks of 4 k tiles x 8 n tiles (k_tiles % 4 == 0, n_tiles % 8 == 0)
};

// cache policy bits of a buffer store: sc0 | nt | sc1
constexpr int kStoreStreaming = 1 | 2 | 16;

struct WgradCfg {
  static constexpr int TK = 256, TN = 128, NW = 8, NT = 512, S = 3;
  static constexpr int X_BYTES = TK * 128, Y_BYTES = TN * 128, SX_BYTES = TK * 4, SY_BYTES = TN * 4, DUMP_BYTES = 256;
  static constexpr int STAGE_BYTES = X_BYTES + Y_BYTES + SX_BYTES + SY_BYTES + DUMP_BYTES;
  static constexpr int LDS_BYTES = S * STAGE_BYTES;
  static constexpr int X_ITERS = TK / 8 / NW, Y_ITERS = TN / 8 / NW;   // 8-row slabs per wave
  static constexpr int NDMA = X_ITERS + Y_ITERS + 1;                   // per wave and token block, scale fetch included
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// The 32 operand bytes of a lane are bytes [32 q, 32 q + 32) of a 128-token block; dword d of the fragment holds
// tokens 32 q + 4 d .. + 3.  x4 = 4 * (bound - first token of the dword): the number of the dword's bytes below the
// bound, times 4, is clamp(x4, 0, 16), and a shift by 32 bits is taken as two shifts by 16.
__device__ __forceinline__ int bytes_from(int x4) {        // keeps the bytes at and above the bound
  const int h = clampi(x4, 0, 16);
  return (int)((0xFFFFFFFFu << h) << h);
}
__device__ __forceinline__ int bytes_below(int x4) {       // keeps the bytes below the bound
  return ~bytes_from(x4);
}

// TIMING (measurement builds of the probe library only; the GEMM library instantiates 0): parts of a block's work
// left out to time the rest.  Only accesses, waits and the masks are removed: every access that remains is one the
// full kernel makes.  The outputs of such builds are meaningless.
enum : int { kWgNoFetch = 1, kWgNoStore = 2, kWgNoBarrier = 4, kWgNoMask = 8, kWgNoLdsReads = 16 };

// OUT16: dW is bfloat16 (round to nearest even), half the output bytes.
template <int TIMING, bool OUT16 = false>
__global__ void __launch_bounds__(WgradCfg::NT) gg_wgrad_kernel(const WgradArgs a) {
  using Cfg = WgradCfg;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l = tid & 63;
  const int r = l & 15, q = l >> 4;
  const int wk = w >> 1, wn = w & 1;
  const int M = a.M_total;

  // ---- persistent walk over the tile list (group by group; inside a group blocks of 4 x 8 tiles, or k tile by k
  // tile).  Workgroup b runs on XCD b % 8; every XCD takes contiguous runs of `slots` tiles, which share operand
  // rows in that XCD's L2.
  struct Tile {
    bool valid;
    int g, k0, n0, lo, hi, j0, steps;
  };
  const GG_CONST_I32* offc = (const GG_CONST_I32*)a.off;
  const int per_group = a.n_tiles * a.k_tiles;
  auto tile_at = [&](int it) __attribute__((always_inline)) -> Tile {
    Tile t = {false, 0, 0, 0, 0, 0, 0, 0};
    int T;
    if (a.slots > 0) T = (it * 8 + (int)(blockIdx.x & 7)) * a.slots + (int)(blockIdx.x >> 3);
    else T = it * (int)gridDim.x + (int)blockIdx.x;
    if (T >= a.tiles) return t;
    t.valid = true;
    t.g = T / per_group;
    const int local = T - t.g * per_group;
    int kt, nt;
    if (a.blocked) {
      // 32 consecutive tiles (the tiles an XCD's workgroups work on at the same time, when it has 32) are 4 k tiles
      // x 8 n tiles: they fetch 1024 + 1024 operand rows per token block between them, where a run of 32 n tiles
      // fetches 256 + 4096, and what several workgroups fetch at about the same time comes out of the XCD's L2 once
      const int sb = local >> 5, in = local & 31, per_row = a.n_tiles >> 3;
      const int sbk = sb / per_row;
      kt = sbk * 4 + (in >> 3);
      nt = (sb - sbk * per_row) * 8 + (in & 7);
    } else {
      kt = local / a.n_tiles;
      nt = local - kt * a.n_tiles;
    }
    t.k0 = kt * Cfg::TK;
    t.n0 = nt * Cfg::TN;
    t.lo = clampi(offc[t.g], 0, M);
    t.hi = clampi(offc[t.g + 1], t.lo, M);
    t.j0 = t.lo >> 7;
    t.steps = t.hi > t.lo ? ((t.hi + 127) >> 7) - t.j0 : 0;     // token blocks [j0, j0 + steps)
    return t;
  };

  // ---- fetches: whole-tensor views (an offset past the end reads zeros), 16 bytes per lane, lane l of a slab lands
  // at LDS byte 16 l (row l / 8, chunk l % 8); LDS chunk c of a row holds global chunk c ^ key(row).  The tile and
  // the token block travel in the scalar offset, so the lane offsets are the same for every fetch.
  const __amdgpu_buffer_rsrc_t dX = __builtin_amdgcn_make_buffer_rsrc((void*)a.XT, 0, a.K * M, GG_RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t dY = __builtin_amdgcn_make_buffer_rsrc((void*)a.DYT, 0, a.N * M, GG_RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t dSX = __builtin_amdgcn_make_buffer_rsrc((void*)a.SX, 0, a.K * a.MB * 4, GG_RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t dSY = __builtin_amdgcn_make_buffer_rsrc((void*)a.SDY, 0, a.N * a.MB * 4, GG_RSRC_FLAGS);
  const int lrow = l >> 3, pch = l & 7;
  const int slab_row = w * 8 + lrow;                               // + 64 i
  const int vRow = slab_row * M + ((pch ^ swz_key_a(slab_row)) << 4);   // key(row + 64 i) == key(row)
  // Features change places on the way into LDS: slot 16 f + r of a wave's 64 features (fragment f, row r) holds
  // feature 32 (f / 2) + 2 r + f % 2, so that the lane of row r has two neighbouring features in the accumulators of
  // a fragment pair and the 16 lanes of an output row write 128 consecutive bytes.
  auto feature_of_slot = [](int s) { return 32 * (s >> 5) + 2 * (s & 15) + ((s >> 4) & 1); };
  const int vRowX = feature_of_slot(slab_row) * M + ((pch ^ swz_key_a(slab_row)) << 4);
  // scale fetch, one per wave: waves 0..3 the scales of 64 features each, waves 4, 5 those of 64 dY^T rows each,
  // waves 6, 7 an out-of-range offset into a dump area (every wave issues the same number of fetches)
  const bool sx_wave = w < 4, sy_wave = w == 4 || w == 5;
  const int vS = sx_wave ? (w * 64 + feature_of_slot(l)) * 4 : sy_wave ? ((w - 4) * 64 + l) * 4 : GG_OOB_OFFSET;
  const int s_pitch = sx_wave ? a.K * 4 : a.N * 4;                 // bytes from one token block's scales to the next
  const int ldsS = Cfg::X_BYTES + Cfg::Y_BYTES + (sx_wave ? w * 256 : sy_wave ? Cfg::SX_BYTES + (w - 4) * 256 : Cfg::SX_BYTES + Cfg::SY_BYTES);

  // The fetch stream runs three token blocks ahead of the arithmetic and on from tile to tile: F is the tile whose
  // block sF comes next (tiles without tokens have nothing to fetch and are passed over), so the first blocks of a
  // workgroup's next tile are in flight while the current one is finished and stored.
  Tile F = tile_at(0);
  int itF = 0, sF = 0;
  // A block's fetches are prepared at the top of a step (the cursor moves on, the scalar offsets are formed) and
  // issued one at a time between the matrix instructions of the step: issued together, the eight waves' 56 fetches
  // wait for the address unit one behind the other, and a wave that waits there issues no matrix instruction.
  int f_x_off = 0, f_y_off = 0, f_s_off = 0;     // scalar offsets of the prepared block: XT, DYT, scales
  int vXsel = GG_OOB_OFFSET, vYsel = GG_OOB_OFFSET, vSsel = GG_OOB_OFFSET;   // lane offsets, out of range when no tile is left
  auto fetch_prepare = [&]() __attribute__((always_inline)) {
    while (F.valid && sF >= F.steps) {
      ++itF;
      F = tile_at(itF);
      sF = 0;
    }
    const bool in = F.valid;
    const int j = F.j0 + sF;
    f_x_off = __builtin_amdgcn_readfirstlane(j * 128 + F.k0 * M);
    f_y_off = __builtin_amdgcn_readfirstlane(j * 128 + F.n0 * M);
    f_s_off = __builtin_amdgcn_readfirstlane(j * s_pitch + (sx_wave ? F.k0 : F.n0) * 4);
    vXsel = in ? vRowX : GG_OOB_OFFSET;
    vYsel = in ? vRow : GG_OOB_OFFSET;
    vSsel = in ? vS : GG_OOB_OFFSET;
    ++sF;
  };
  // piece 0: the wave's scales; 1 .. X_ITERS: its slabs of the X tile; the rest: its slabs of the dY^T tile
  auto fetch_piece = [&](auto ic, uint8_t* st) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value;
    if constexpr (I == 0) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(sx_wave ? dSX : dSY, GG_LDS_PTR(st + ldsS), 4, vSsel, f_s_off, 0, 0);
    } else if constexpr (I <= Cfg::X_ITERS) {
      constexpr int i = I - 1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dX, GG_LDS_PTR(st + (w + i * 8) * 1024), 16, vXsel, f_x_off + i * 64 * M, 0, 0);
    } else {
      constexpr int i = I - 1 - Cfg::X_ITERS;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dY, GG_LDS_PTR(st + Cfg::X_BYTES + (w + i * 8) * 1024), 16, vYsel, f_y_off + i * 64 * M, 0, 0);
    }
  };
  auto fetch_next = [&](int stage) __attribute__((always_inline)) {     // all of a block at once (the prologue)
    fetch_prepare();
    uint8_t* st = lds + stage * Cfg::STAGE_BYTES;
    static_for<0, Cfg::NDMA>([&](auto ic) __attribute__((always_inline)) { fetch_piece(ic, st); });
  };

  // ---- operand reads: fragment row r, chunks 2q and 2q+1
  const int keyR = swz_key_a(r);
  const int rd0 = r * 128 + (((2 * q) ^ keyR) << 4), rd1 = r * 128 + (((2 * q + 1) ^ keyR) << 4);
  const int xBase = (wk * 64) * 128, yBase = Cfg::X_BYTES + (wn * 64) * 128;
  // a matrix instruction's output has dY^T rows 4 q .. 4 q + 3 of its fragment in the lane's four registers and
  // feature r of its fragment in the lane, so that the 16 lanes of a row hold 64 consecutive bytes of dW
  const int sxRd = Cfg::X_BYTES + Cfg::Y_BYTES + (wk * 64 + r) * 4;                     // + 64 kf
  const int syRd = Cfg::X_BYTES + Cfg::Y_BYTES + Cfg::SX_BYTES + (wn * 64 + 4 * q) * 4;     // + 64 nf: four consecutive rows
  auto read_frag = [&](const uint8_t* p) __attribute__((always_inline)) -> v8i {
    const v4i x = *(const v4i*)(p + rd0);
    const v4i y = *(const v4i*)(p + rd1);
    return (v8i){x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
  };

  // The operand fragments and scales of the block that is multiplied next live in registers: they are read out of
  // LDS one block ahead, each into the registers of its predecessor as soon as that has been used for the last time.
  v8i xf[4], yf[4];
  float sx[4];
  v4f sy[4];

  // One token block out of the registers, while they are refilled from `nx` (the LDS buffer of the following block).
  // Where the block holds tokens before the group's first or from the group's end on (it is the group's first or
  // last block), their bytes are cleared in both operands first.
  auto block = [&](int first, int lo, int hi, const uint8_t* nx, uint8_t* fst, v2f (&acc)[2][4][4]) __attribute__((always_inline)) {   // first: the block's first token; fst: the buffer the prepared fetches go to
    const bool cut_lo = !(TIMING & kWgNoMask) && lo > first, cut_hi = !(TIMING & kWgNoMask) && hi < first + 128;
    if (cut_lo || cut_hi) {
      const int lo4 = 4 * (lo - first - 32 * q), hi4 = 4 * (hi - first - 32 * q);    // valid tokens of the block: [lo - first, hi - first)
      v8i m;
      if (cut_lo) {
#pragma unroll
        for (int d = 0; d < 8; ++d) m[d] = bytes_from(lo4 - 16 * d);
        if (cut_hi) {
#pragma unroll
          for (int d = 0; d < 8; ++d) m[d] &= bytes_below(hi4 - 16 * d);
        }
      } else {
#pragma unroll
        for (int d = 0; d < 8; ++d) m[d] = bytes_below(hi4 - 16 * d);
      }
#pragma unroll
      for (int f = 0; f < 4; ++f) {
        xf[f] &= m;
        yf[f] &= m;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // Software pipeline in 18 slots: slot t issues matrix instruction t (dY^T fragment t / 4 x feature fragment
    // t % 4), the 8 vector instructions that consume matrix instruction t - 2 (the factor product and the FMA of each
    // of its four outputs), and the LDS reads that refill what was used for the last time in the slot before.
    v4f p[16];
    static_for<0, 16 + 2>([&](auto tc) __attribute__((always_inline)) {
      constexpr int t = decltype(tc)::value;
      if constexpr (t < 16)
        p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(yf[t / 4], xf[t % 4], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
      if constexpr (t >= 2) {
        constexpr int u = t - 2, nf = u / 4, kf = u % 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[kf >> 1][nf][i][kf & 1] += p[u][i] * (sy[nf][i] * sx[kf]);
      }
      if constexpr (!(TIMING & kWgNoFetch) && t % 2 == 1 && t / 2 < Cfg::NDMA) fetch_piece(std::integral_constant<int, t / 2>{}, fst);
      if constexpr (!(TIMING & kWgNoLdsReads)) {
        if constexpr (t == 4 || t == 8 || t == 12 || t == 16) yf[t / 4 - 1] = read_frag(nx + yBase + (t / 4 - 1) * 2048);
        if constexpr (t >= 13 && t <= 16) xf[t - 13] = read_frag(nx + xBase + (t - 13) * 2048);
        if constexpr (t == 6 || t == 10 || t == 14) sy[(t - 6) / 4] = *(const v4f*)(nx + syRd + ((t - 6) / 4) * 64);
        if constexpr (t == 17) {
          sy[3] = *(const v4f*)(nx + syRd + 3 * 64);
#pragma unroll
          for (int f = 0; f < 4; ++f) sx[f] = *(const float*)(nx + sxRd + f * 64);
        }
      } else if constexpr (t == 17) {
        // the registers keep what the prologue read; they are made opaque, so that the block is not hoisted out of the loop
#pragma unroll
        for (int f = 0; f < 4; ++f) asm volatile("" : "+v"(xf[f]), "+v"(yf[f]), "+v"(sx[f]), "+v"(sy[f]));
      }
    });
    static_for<0, 16 + 2>([&](auto tc) __attribute__((always_inline)) {
      constexpr int t = decltype(tc)::value;
      if constexpr (t < 16) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if constexpr (t >= 2) __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
      if constexpr (!(TIMING & kWgNoFetch) && t % 2 == 1 && t / 2 < Cfg::NDMA) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      constexpr int reads = (t == 4 || t == 8 || t == 12 ? 2 : 0) + (t >= 13 && t <= 15 ? 2 : 0) + (t == 16 ? 4 : 0) +
                            (t == 6 || t == 10 || t == 14 ? 1 : 0) + (t == 17 ? 5 : 0);
      if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);
    });
    __builtin_amdgcn_sched_barrier(0);
    // the accumulators are "used" here, so that every update above lands in the accumulator's own register
#pragma unroll
    for (int pr = 0; pr < 2; ++pr)
#pragma unroll
      for (int nf = 0; nf < 4; ++nf)
#pragma unroll
        for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(acc[pr][nf][i]));
  };

  // ---- ring of 3 LDS buffers + the registers: while block b is multiplied out of the registers, block b + 1 has
  // landed and is being read into them, blocks b + 2 and b + 3 are in flight (b + 3 into the buffer block b came from)
  fetch_next(0);
  fetch_next(1);
  fetch_next(2);
  wait_vmcnt<2 * Cfg::NDMA>();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    xf[f] = read_frag(lds + xBase + f * 2048);
    yf[f] = read_frag(lds + yBase + f * 2048);
    sx[f] = *(const float*)(lds + sxRd + f * 64);
    sy[f] = *(const v4f*)(lds + syRd + f * 64);
  }
  int stage = 0;            // the buffer the block in the registers came from
  int st_prev = 0, st_prev2 = 0;   // batches of 32 stores issued since the last top of a step / between the two before
  // The top of a step.  This wave has read all of the block it multiplies next, and its part of the following block
  // has landed: those fetches were issued two steps ago; newer are the fetches of the last step and the stores of
  // the tiles finished since, which may all stay in flight (vector memory operations of a wave complete in the order
  // they were issued; the counter holds 63 and never gets there: no batch of stores begins with more than 31
  // outstanding and no step's fetches with more than 56, and with two batches and a fetch behind it the awaited fetch
  // cannot be among 56 outstanding operations).
  auto top = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const int batches = st_prev + st_prev2;
    if (batches == 0) wait_vmcnt<Cfg::NDMA>();
    else if (batches == 1) wait_vmcnt<Cfg::NDMA + 32>();
    else wait_vmcnt<63 - Cfg::NDMA>();          // room for this step's fetches
    st_prev2 = st_prev;
    st_prev = 0;
    if constexpr (!(TIMING & kWgNoBarrier)) __builtin_amdgcn_s_barrier();       // ... and everybody's; nobody reads the buffer of the coming block any more
    asm volatile("" ::: "memory");
    if constexpr (!(TIMING & kWgNoFetch)) fetch_prepare();                    // three steps ahead, into that buffer
  };
  for (int it = 0;; ++it) {
    const Tile cur = tile_at(it);
    if (!cur.valid) break;
    v2f acc[2][4][4];             // [pair of feature fragments][dY^T fragment][row 4 q + i]: two neighbouring features
#pragma unroll
    for (int pr = 0; pr < 2; ++pr)
#pragma unroll
      for (int nf = 0; nf < 4; ++nf)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[pr][nf][i] = (v2f){0.f, 0.f};
    for (int s = 0; s < cur.steps; ++s) {
      top();
      const int next_stage = stage == 2 ? 0 : stage + 1;
      block((cur.j0 + s) * 128, cur.lo, cur.hi, lds + next_stage * Cfg::STAGE_BYTES, lds + stage * Cfg::STAGE_BYTES, acc);
      stage = next_stage;
    }
    // ---- epilogue: fp32 through a view of the tile, 8 bytes per lane: the 16 lanes of a dY^T row write 128
    // consecutive bytes (with the features in a lane's registers and 16 bytes per lane, neighbouring lanes would write
    // to different rows and every lane's piece would be a request of its own: a quarter of the store rate).  Written
    // once and never read here, so the stores carry the streaming cache policy (sc0 sc1 nt): the gradients do not
    // push the operand tiles out of the L2 and the fetches beside them keep their latency.
    constexpr int ES = OUT16 ? 2 : 4;      // bytes per element of dW
    const __amdgpu_buffer_rsrc_t dOut = __builtin_amdgcn_make_buffer_rsrc((void*)((uint8_t*)a.dW + (((int64_t)cur.g * a.N + cur.n0) * a.K + cur.k0) * ES), 0, ((Cfg::TN - 1) * a.K + Cfg::TK) * ES, GG_RSRC_FLAGS);
    const int vOut = (4 * q * a.K + 2 * r) * ES;
    wait_vmcnt<31>();
#pragma unroll
    for (int nf = 0; nf < 4; ++nf)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          const v2f v = acc[pr][nf][i];
          if constexpr (TIMING & kWgNoStore) asm volatile("" : : "v"(v));
          else if constexpr (OUT16)      // the lane's two neighbouring features in one dword: a row's 16 lanes write 64 bytes
            __builtin_amdgcn_raw_buffer_store_b32(pack2_rne(v.x, v.y, false), dOut, vOut + 64 * pr, ((wn * 64 + 16 * nf + i) * a.K + wk * 64) * 2, kStoreStreaming);
          else
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(v2i, v), dOut, vOut + 128 * pr, ((wn * 64 + 16 * nf + i) * a.K + wk * 64) * 4, kStoreStreaming);
        }
    ++st_prev;
  }
  wait_vmcnt<0>();     // the fetches past the last block still write zeros into this workgroup's LDS: let them land
}

}  // namespace gg
