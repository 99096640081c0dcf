// Second kernel of the padding-free block-scaled FP8 grouped GEMM (same operation as gemm_kernel.h: paper
// Sec. 2.1, Table 1, with the padding-free capability of Sec. 2.2 through bounded buffer descriptors).
//
// The first kernel keeps [A | B] of a K block in one LDS buffer and all waves meet at a barrier per K block
// before anyone reads either operand.  At the largest tile the accumulators allow (256 x 256) only two such
// buffers fit in 160 KB: one K block of look-ahead, a DMA stream that drains at every block boundary and a
// matrix pipe that waits for the first LDS reads after every barrier.  This kernel splits the two operands:
//
//  * 8 waves side by side along N: wave w owns columns [32w, 32w+32) of the 256-wide tile and all BM rows, so no
//    two waves need the same weight row.  Each wave fetches ITS 32 weight rows of a K block (two fragments of
//    16 rows x 128 B) by DMA into three private 2 KB LDS slots, copies a fragment into registers half a K block
//    or more before it is needed (two register sets, one per K-block parity) and refills the slot at once.  No
//    other wave touches these slots: the weight path needs no barrier at all.
//  * The shared A tile (BM x 128 B per K block, plus scales) lives in a ring of 3 LDS buffers.  The one barrier
//    per K block, at the top of block kb, publishes block kb+1 (not kb): the first activation fragments of the
//    next block are read before the block boundary, so the matrix pipe never waits for LDS after a barrier.
//  * Every wave issues the same number of fetches per K block (blocks past the end of K and waves without a
//    scale to fetch use an out-of-range offset: zeros, no traffic), so all s_waitcnt counts are compile-time
//    constants.  Order inside block kb: scale and A DMAs of block kb+2 first, then the refills of the two
//    weight slots; the wait at the top of block kb+1 lets exactly the refills stay in flight.
//  * The K loop is carried from one tile of a workgroup into its next: the fetches of a K step run two to three
//    K blocks ahead, and past a tile's last K block they fetch the next tile's first blocks (the descriptors are
//    re-pointed when a fetch stream reaches the end of the tile), so only a workgroup's first tile has a
//    prologue.  The register sets alternate by K-block parity: the number of K blocks must be even and >= 4.
//
//  * SKIP (variants "-rbs"): every K step leaves out the 16-row activation blocks past the tile's last valid row
//    (operand reads, MFMAs, FMAs: paper Sec. 2.2, no work on rows that do not exist).  Measured, it does not pay:
//    a partly filled tile is bound by its weight fetches and the fixed cost of a K step, not by its MFMAs, and the
//    scalar test per block costs 1-3 % on full tiles; the variants are kept selectable, the automatic choice
//    does not take them.
//
// Arithmetic per output element is the same as in the first kernel (one C=0 MFMA per 128-wide scale block,
// 4 fp32 FMAs with the per-lane scale, the K blocks in the same order), so results are bit-identical to it unless KP is set.
// KP: a lane's 32 operand bytes of a 128-byte row are [16q, 16q+16) and [64+16q, 64+16q+16) (q = lane/16)
// instead of [32q, 32q+32): a permutation of k inside the K block applied to both operands alike; every dot
// product has the same terms, the matrix instruction adds them in another order.
#pragma once
#include "gemm_kernel.h"
#include "quant_kernel.h"

namespace gg {

// FUSE: the tile's 256 weight rows are 128 rows of the gate projection and the 128 matching rows of the up
// projection of an expert MLP's first GEMM, and the epilogue turns the two 128-column halves into
// silu(gate) * up, quantised to e4m3 with one scale per row (see the epilogue).
// SKIP: every K step leaves out the 16-row activation blocks past the tile's last valid row (a scalar test per
// block: 1-3 % slower on full tiles, and a tile's cost follows its height).  Without it every tile costs a full one.
// RAGGED: N need not be a multiple of 256 nor K of 128 (the ceilings in Table 1 of the paper; N % 8 == 0 and
// K % 16 == 0 remain): lane masks on the last K block's fetches, weight rows, scale blocks and output columns bounded
// by N.  A few selects per fetch and store, hence an instantiation of its own.
// ODDK: the number of K blocks may be odd (one more, empty K step per tile; see KBe in the kernel).  One more value
// that lives in a scalar register through the whole kernel, which the largest tiles have no room for: the
// instantiations for whole blocks keep to an even number.
// TIMING (measurement builds of the probe library only; 0 in every kernel the GEMM library launches): a bit mask of
// parts of a K step that are LEFT OUT, to time what each costs.  1: the fetches of the K steps (the prologue of a
// workgroup's first tile still fetches); 2: every fetch goes to the out-of-range offset (issued, no traffic, zeros);
// 4: the barrier of the K step; 8: the LDS reads of activation fragments and scales (the registers keep what the
// prologue read); 16: the K step's waits for its fetches (operands are read whether they have arrived or not).
// Accesses and waits are only ever removed, so everything that remains stays in bounds and every wait ends; the
// results are meaningless.
// 64: every fetch of the K steps goes to four registers that nobody reads instead of to LDS (the same requests to
// memory; the operands in LDS stay what the prologue fetched).
enum : int { kTimingNoFetch = 1, kTimingFetchNowhere = 2, kTimingNoBarrier = 4, kTimingNoLdsReads = 8, kTimingNoFetchWaits = 16,
             kTimingFetchToRegs = 64 };
template <int BM_, int AFR_ = 4, bool KP_ = false, bool FUSE_ = false, bool SKIP_ = false, bool RAGGED_ = false, bool ODDK_ = RAGGED_, int TIMING_ = 0>
struct RbCfg {
  static constexpr bool KP = KP_, FUSE = FUSE_, SKIP = SKIP_, RAGGED = RAGGED_, ODDK = ODDK_;
  static constexpr int TIMING = TIMING_;
  static_assert(TIMING_ == 0 || !(FUSE_ || SKIP_ || RAGGED_ || ODDK_), "measurement builds exist for the plain tile only");
  static_assert(!(FUSE_ && SKIP_), "the activation epilogue runs full K steps only");
  static_assert(!(FUSE_ && RAGGED_), "the activation epilogue takes whole blocks only");
  static constexpr int BM = BM_, BN = 256, S = 3;
  static constexpr int NW = 8, NT = 512;
  static constexpr int TM = BM / 16, TN = 2;
  static constexpr int A_ITERS = (BM + 63) / 64;   // 8-row slabs per wave per K block
  // BM need not be a multiple of 64: the last band of 64 rows is then partly outside the tile, its rows fail the
  // bounds check like any row past the group's end (zeros into LDS rows nobody reads, no traffic)
  static constexpr int A_BYTES = A_ITERS * 64 * 128;
  static constexpr int SA_WAVES = (BM + 63) / 64;
  // Activation scales are read one band (four activation blocks, 64 rows) at a time into one of two registers of
  // four: band b of a K step at block 4b - 3, band 0 of the next K step at block R_NEXT (three blocks before the
  // end where the register's previous band has had its last use by then, else right after that use).
  static constexpr int NBAND = SA_WAVES;
  static constexpr int R_NEXT = BM / 16 - 3 > 4 * NBAND - 5 ? BM / 16 - 3 : 4 * NBAND - 5;
  static constexpr int SA_BYTES = SA_WAVES * 256;
  static constexpr int SB_BYTES = 256;
  static constexpr int DUMP_BYTES = 256;           // target of the scale DMA of waves that have no scales to fetch
  static constexpr int STAGE_BYTES = A_BYTES + SA_BYTES + SB_BYTES + DUMP_BYTES;
  static constexpr int B_SLOTS = 3, B_SLOT_BYTES = 2048;        // per wave: fragments of 16 rows x 128 B
  static constexpr int B_BASE = S * STAGE_BYTES;
  static constexpr int RED_BASE = B_BASE + NW * B_SLOTS * B_SLOT_BYTES;   // FUSE: per row, the 8 waves' partial maxima
  static constexpr int LDS_BYTES = RED_BASE + (FUSE ? BM * NW * 4 : 0);
  static constexpr int SB_WAVE = NW - 1;
  static constexpr int MFMAS = TM * TN;
  // MFMAs in flight before their FMAs are issued: the two of one activation block (at 256 rows 1 % faster than 3,
  // at 192 and 224 rows no difference), so that the FMAs of a block sit in the block after it and a K step that
  // stops early needs one block to drain
  static constexpr int PIPE = 2;
  static constexpr int AFR = AFR_;                 // ring of activation fragments (prefetch distance AFR-1 blocks)
  // fetches per wave per K block, in issue order: 1 scale DMA, A_ITERS A slabs, 2 + 2 weight-slot refills
  static constexpr int N_A = 1 + A_ITERS;
  // SPREAD: the fetches of a K step are dealt out over its matrix instructions one at a time (an A slab after every
  // third, the two halves of a refill two apart) instead of in groups of three and two: the eight waves of a
  // workgroup run in step, so a group in the source is a burst of 16 to 24 KB-sized requests at the fetch path.
  // 2 - 3.5 % faster at 192 to 256 rows (gate_up, interleaved A/B); the shorter tiles have no room for it.
  static constexpr bool SPREAD = BM_ >= 192 && !SKIP_;
  static constexpr int A_STEP = SPREAD ? 3 : 1;    // MFMAs from one A DMA to the next
  static constexpr int R_STEP = SPREAD ? 2 : 0;    // MFMAs between the two DMAs of a refill (0: back to back)
  static constexpr int T_A0 = 0;                   // A DMAs after MFMAs T_A0, T_A0 + A_STEP, ...
  static constexpr int T_R0 = SPREAD ? A_STEP * (A_ITERS - 1) + 2 : A_ITERS + 2;         // refill of the slot read at the top of the block
  static constexpr int T_MID = MFMAS / 2 + 2;      // wait for and read of the second fragment of the next block
  static constexpr int T_R1 = T_MID + 6 <= MFMAS ? T_MID + 4 : MFMAS - 2;   // refill of that slot
  // in flight across the top of a block: the 4 refill DMAs of the previous block
  static constexpr int W_TOP = 4;
  // in flight across the mid-block wait: the later refill of the previous block (2), this block's scale and A
  // DMAs (N_A) and its first refill (2)
  static constexpr int W_MID = 2 + N_A + 2;
  static_assert(BM % 16 == 0 && BM <= 256 && AFR_ >= 2 && TM % AFR_ == 0, "BM a multiple of 16, fragment ring a divisor of BM/16");
  static_assert(PIPE == TN, "the FMAs of an activation block are issued with the MFMAs of the next one");
  static_assert(SA_WAVES <= SB_WAVE, "scale fetchers must be distinct waves");
  static_assert(T_R0 + R_STEP + 2 <= T_MID && T_R1 >= T_MID + 2 && T_R1 + R_STEP + 2 <= MFMAS && T_MID % TN == 0, "issue slots must fit the MFMA stream");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// swizzle key for an A tile whose lanes read chunks q and 4+q of row base+r: see swz_key_a for the lane groups
// that ds_read_b128 serves together; here the chunk index advances by ONE (not two) for r in 4..11
__device__ __forceinline__ int swz_key_a1(int row) {
  const int u = (row >> 1) & 7;
  return u ^ (((u >> 1) ^ (u >> 2)) & 1);
}

// Buffer descriptor from wave-uniform values.  readfirstlane states the uniformity for the compiler, which
// otherwise may keep a descriptor in vector registers and loop over its values at every use.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t uniform_rsrc(const void* ptr, int bytes) {
  const uint64_t p = (uint64_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, __builtin_amdgcn_readfirstlane(bytes), GG_RSRC_FLAGS);
}

// kTimingFetchToRegs: the fetch as an ordinary load into registers that stay allocated to the end of the kernel
// (the compiler does not know that the asm is a load; "+v" keeps it from giving the registers to anything else)
__device__ __forceinline__ void timing_fetch16(v4i& sink, int voffset, __amdgpu_buffer_rsrc_t rsrc, int soffset) {
  asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "+v"(sink) : "v"(voffset), "s"(rsrc), "s"(soffset));
}
__device__ __forceinline__ void timing_fetch4(v4i& sink, int voffset, __amdgpu_buffer_rsrc_t rsrc, int soffset) {
  asm volatile("buffer_load_dword %0, %1, %2, %3 offen" : "+v"(sink.x) : "v"(voffset), "s"(rsrc), "s"(soffset));
}

template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gg_gemm_rb_kernel(const GemmArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, NW = Cfg::NW, S = Cfg::S;
  constexpr int TM = Cfg::TM, TN = Cfg::TN, MF = Cfg::MFMAS, PIPE = Cfg::PIPE, AFR = Cfg::AFR;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l = tid & 63;
  const int r = l & 15, q = l >> 4;
  const int K = a.K, KB = a.KB, N = a.N;
  // K steps per tile: the two register sets alternate by step parity and the loop runs on from tile to tile, so an
  // odd number of K blocks (ODDK) gets one more step, whose fetches (block KB of the tile: past its end) all use the
  // out-of-range offset: zero operands and zero scales, which add exact zeros
  const int KBe = Cfg::ODDK ? (KB + 1) & ~1 : KB;

  // ---- per-lane constants ---------------------------------------------------------------------------
  // DMA: lane l of a wave-wide 16 B DMA lands at LDS byte 16*l of its 1 KB slab (row l/8, chunk l%8); the
  // swizzle is applied on the global side: LDS chunk c of a row holds global chunk c ^ key(row)
  const int a_row = w * 8 + (l >> 3);                                  // + i * 64
  const int vA = a_row * K + (((l & 7) ^ (Cfg::KP ? swz_key_a1(a_row) : swz_key_a(a_row))) << 4);
  // weight fragment j, fragment row rr (= MFMA row) is tile column 32w + 8*(rr/4) + 4j + rr%4: the 8 outputs
  // a lane ends up with (MFMA rows 4q..4q+3 of both fragments) are then 8 consecutive columns
  // FUSE: fragment 0 is rows [16w, 16w+16) of the tile's gate rows, fragment 1 the same rows of its up rows, so a
  // lane ends up with gate and up of the same 4 activation columns 16w + 4q .. + 3
  const int f_row = l >> 3;                                            // slab 0; slab 1 is fragment row f_row + 8
  const int vBrow = (Cfg::FUSE ? w * 16 + f_row : w * 32 + 8 * (f_row >> 2) + (f_row & 3)) * K;
  const int vB0 = vBrow + (((l & 7) ^ (Cfg::KP ? swz_key_a1(f_row) : swz_key_a(f_row))) << 4);
  const int vB1 = vBrow + (Cfg::FUSE ? 8 : 16) * K + (((l & 7) ^ (Cfg::KP ? swz_key_a1(f_row + 8) : swz_key_a(f_row + 8))) << 4);
  // RAGGED, K % 128 != 0: in the last K block a lane whose 16-byte chunk starts at or past byte k_rem of the block
  // would fetch the start of the next row; it fetches from the out-of-range offset instead (zeros).  Kept as a
  // second lane offset per stream (vector registers; the scalar registers are all taken).
  const int vA_last = Cfg::RAGGED && (((l & 7) ^ (Cfg::KP ? swz_key_a1(a_row) : swz_key_a(a_row))) << 4) >= a.k_rem ? GG_OOB_OFFSET : vA;
  const int vB0_last = Cfg::RAGGED && (((l & 7) ^ (Cfg::KP ? swz_key_a1(f_row) : swz_key_a(f_row))) << 4) >= a.k_rem ? GG_OOB_OFFSET : vB0;
  const int vB1_last = Cfg::RAGGED && (((l & 7) ^ (Cfg::KP ? swz_key_a1(f_row + 8) : swz_key_a(f_row + 8))) << 4) >= a.k_rem ? GG_OOB_OFFSET : vB1;
  const int nb_all = Cfg::RAGGED ? (N + 127) >> 7 : N >> 7;             // 128-column scale blocks of a group's weights
  const int inter = N >> 1;                                            // FUSE: activation columns (N = gate + up rows)
  const int frag1_off = Cfg::FUSE ? inter * K : 4 * K;                 // from fragment 0's weight rows to fragment 1's
  // Every wave issues exactly one scale DMA per K block: waves [0, SA_WAVES) fetch 64 activation scales each,
  // wave SB_WAVE the two weight scales, the others an out-of-range offset into a dump area.
  const bool sa_wave = w < Cfg::SA_WAVES, sb_wave = w == Cfg::SB_WAVE;
  const int s_kb_stride = sa_wave ? a.sa_kb_stride : 4;             // bytes from one K block's scale to the next
  // activation scales: lane l fetches the scale of row 64w + 16*(l%4) + l/4 of the tile, so that LDS word 4r + i of
  // the wave's 256 bytes holds row 16i + r and a lane reads the scales of its row r in four consecutive activation
  // blocks with ONE 16-byte read (a 4-byte read per block costs the LDS pipe as much as a quarter of the operand reads)
  const int vS = sa_wave ? (w * 64 + 16 * (l & 3) + (l >> 2)) * a.sa_row_stride : sb_wave ? (l < BN / 128 ? l : BN / 128 - 1) * (Cfg::FUSE ? inter >> 7 : 1) * KB * 4 : GG_OOB_OFFSET;
  const int ldsS = Cfg::A_BYTES + (sa_wave ? w * 256 : sb_wave ? Cfg::SA_BYTES : Cfg::SA_BYTES + Cfg::SB_BYTES);
  // operand reads: row r, chunks (2q, 2q+1), or (q, 4+q) with KP
  const int keyR = Cfg::KP ? swz_key_a1(r) : swz_key_a(r);
  const int rd0 = r * 128 + (((Cfg::KP ? q : 2 * q) ^ keyR) << 4);
  const int rd1 = r * 128 + (((Cfg::KP ? 4 + q : 2 * q + 1) ^ keyR) << 4);
  const int saRd = Cfg::A_BYTES + r * 16;                               // + 256 * band: scales of blocks 4*band .. 4*band+3
  const int sbRd = Cfg::A_BYTES + Cfg::SA_BYTES + (Cfg::FUSE ? 0 : ((w * 32) >> 7) * 4);   // FUSE: gate block, up block at + 4
  uint8_t* const bslots = lds + Cfg::B_BASE + w * (Cfg::B_SLOTS * Cfg::B_SLOT_BYTES);   // this wave's weight slots

  // ---- persistent walk over the tile list; a workgroup looks one tile ahead (see "carry" below) -------------
  struct Tile {
    bool valid;
    int g, n0, rows_valid;
    int64_t grow;
  };
  int g = 0, base = 0;
  const int nwg = gridDim.x;
  const GG_CONST_I32* offc = (const GG_CONST_I32*)a.off;
  auto find_tile = [&](int it) __attribute__((always_inline)) -> Tile {
    Tile t = {false, 0, 0, 0, 0};
    int T;
    if (a.slots > 0) T = (it * 8 + (int)(blockIdx.x & 7)) * a.slots + (int)(blockIdx.x >> 3);
    else T = it * nwg + blockIdx.x;
    int row0 = 0, Mg = 0, mtiles = 0;
    for (;;) {
      if (g >= a.G) return t;
      row0 = clampi(offc[g], 0, a.M_total);
      const int row1 = clampi(offc[g + 1], row0, a.M_total);
      Mg = row1 - row0;
      mtiles = (Mg + BM - 1) / BM;
      const int cnt = mtiles * a.n_tiles;
      if (T < base + cnt) break;
      base += cnt;
      ++g;
    }
    const int local = T - base;
    const int per_chunk = mtiles * a.n_chunk;
    const int nc = local / per_chunk;
    const int rem = local - nc * per_chunk;
    int csz = a.n_tiles - nc * a.n_chunk;
    csz = csz < a.n_chunk ? csz : a.n_chunk;
    const int mtile = rem / csz;
    const int ntile = nc * a.n_chunk + (rem - mtile * csz);
    const int m0 = mtile * BM;
    t.g = g;
    t.n0 = ntile * (Cfg::FUSE ? 128 : BN);     // FUSE: first of the tile's 128 activation columns
    t.rows_valid = Mg - m0 < BM ? Mg - m0 : BM;
    t.grow = (int64_t)row0 + m0;
    t.valid = true;
    return t;
  };
  // Bounded descriptors: rows past the group's end read as zero and are never written (paper Sec. 2.2:
  // no padding, no out-of-group access).  on = false: views of length zero (every fetch through them is dropped).
  // One descriptor per 64-row band of the A tile: a lane's offset inside its band is then the same for every
  // slab it fetches (one register instead of one per slab).
  auto band = [&](const Tile& t, int i, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    int rows_i = t.rows_valid - 64 * i;
    rows_i = rows_i < 0 ? 0 : (rows_i > 64 ? 64 : rows_i);
    return uniform_rsrc(a.A + (t.grow + 64 * i) * K, on ? rows_i * K : 0);
  };
  // RAGGED: the weight rows, scale blocks and output columns at or past N do not exist; the views end before them
  // (the range check adds the lane and the scalar part of an offset before it compares with the view's length)
  auto desc_b = [&](const Tile& t, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    const int n_rem = N - t.n0;
    return uniform_rsrc(a.B + ((int64_t)t.g * N + t.n0) * K, on ? (Cfg::FUSE ? inter + 128 : Cfg::RAGGED && n_rem < BN ? n_rem : BN) * K : 0);
  };
  // this wave's scale source: the activation scales of the tile's rows, or the weight scales of its two column blocks
  auto desc_s = [&](const Tile& t, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    return sa_wave ? uniform_rsrc((const uint8_t*)a.SA + t.grow * a.sa_row_stride, on ? sa_view_bytes(a, t.grow, t.rows_valid) : 0)
                   : uniform_rsrc(a.SB + ((int64_t)t.g * nb_all + (t.n0 >> 7)) * KB,
                                  on ? (Cfg::FUSE ? (inter >> 7) + 1
                                                  : Cfg::RAGGED && nb_all - (t.n0 >> 7) < BN / 128 ? nb_all - (t.n0 >> 7) : BN / 128) * KB * 4 : 0);
  };

  // Carry: the fetches a K step issues run two to three K blocks ahead; at the end of a tile those blocks are the
  // first blocks of the workgroup's next tile.  With an even number of K blocks (the two register sets alternate
  // by K-block parity) the descriptors are re-pointed to the next tile as its first fetches come up, the K loop
  // runs on into it, and the state at the end of the last K block IS the state the prologue would have built.
  // The host only launches this kernel with KB >= 3, and with an even KB unless ODDK is set.
  Tile cur = find_tile(0);
  if (!cur.valid) return;
  __amdgpu_buffer_rsrc_t dA0 = band(cur, 0, true), dA1 = band(cur, 1 % Cfg::A_ITERS, true), dA2 = band(cur, 2 % Cfg::A_ITERS, true),
                         dA3 = band(cur, 3 % Cfg::A_ITERS, true);
  __amdgpu_buffer_rsrc_t dB = desc_b(cur, true), dB0 = dB;     // dB0: the stream of fragments j = 0, one K block further ahead
  __amdgpu_buffer_rsrc_t dS = desc_s(cur, true);
  int rot = k_rotation(a, cur.n0), rot0 = rot;
  int kbase = 0, kbase0 = 0;      // K-block index at which the tile behind dA.., dB, dS (resp. dB0) starts
  bool primed = false;
  v4i sink = {0, 0, 0, 0};        // kTimingFetchToRegs: where the fetches land (kept alive to the end of the kernel)
  v8i bfr[2][TN];                 // weight fragments of K block kb in set kb % 2
  v8i afr[AFR];
  v4f sa4[2];                     // activation scales of two bands of four activation blocks (see band_reg)
  float sb_next = 0.f, sb_next_up = 0.f;     // FUSE: the weight scales of the gate block and of the up block
  int stage = 0;                  // LDS buffer of block kb
  int bslot = 2;                  // slot of fragment 2*kb + 2
  for (int it = 0;; ++it) {
    const int n0 = cur.n0, rows_valid = cur.rows_valid;
    const int64_t grow = cur.grow;
    // SKIP: activation blocks a K step of this tile runs: those with a valid row, and one more that carries the
    // FMAs of the last of them
    const int tm_act = rows_valid > BM - 16 ? TM : (rows_valid + 15) / 16 + 1;

    // K blocks are taken in the order rot, rot+1, ..., KB-1, 0, ..., rot-1 (see k_rotation).
    // A fetch stream reaches K block KB of the tile its descriptor points to only in the empty step that ODDK adds
    // (every stream is re-pointed to the next tile right after its fetch of block KB-1, and with no next tile the
    // descriptors have length zero).  That block is "fetched" from an out-of-range offset: same instruction count,
    // no traffic.  Without ODDK the test would never fire and is left out.
    auto dma_a = [&](auto ic, int kb_t, int stage) __attribute__((always_inline)) {   // one 8-row slab of block kb's A tile
      constexpr int i = decltype(ic)::value;
      const int kb = kb_t - kbase;
      const int kp = k_wrapped(kb + rot, KB);
      const int vo = (Cfg::TIMING & kTimingFetchNowhere) ? GG_OOB_OFFSET
                     : !Cfg::ODDK || kb < KB ? (Cfg::RAGGED && kp == KB - 1 ? vA_last : vA) : GG_OOB_OFFSET;
      if constexpr (Cfg::TIMING & kTimingFetchToRegs)
        timing_fetch16(sink, vo, i == 0 ? dA0 : i == 1 ? dA1 : i == 2 ? dA2 : dA3, __builtin_amdgcn_readfirstlane(kp * 128));
      else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(i == 0 ? dA0 : i == 1 ? dA1 : i == 2 ? dA2 : dA3, GG_LDS_PTR(lds + stage * Cfg::STAGE_BYTES + (w + i * NW) * 1024), 16, vo,
                                               __builtin_amdgcn_readfirstlane(kp * 128), 0, 0);
    };
    auto dma_scales = [&](int kb_t, int stage) __attribute__((always_inline)) {     // exactly one DMA in every wave
      const int kb = kb_t - kbase;
      const int vo = (Cfg::TIMING & kTimingFetchNowhere) ? GG_OOB_OFFSET : !Cfg::ODDK || kb < KB ? vS : GG_OOB_OFFSET;
      if constexpr (Cfg::TIMING & kTimingFetchToRegs)
        timing_fetch4(sink, vo, dS, __builtin_amdgcn_readfirstlane(k_wrapped(kb + rot, KB) * s_kb_stride));
      else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dS, GG_LDS_PTR(lds + stage * Cfg::STAGE_BYTES + ldsS), 4, vo,
                                               __builtin_amdgcn_readfirstlane(k_wrapped(kb + rot, KB) * s_kb_stride), 0, 0);
    };
    // weight fragment j of block kb into slot `slot` of this wave: two slabs of 8 fragment rows
    auto dma_b = [&](int kb_t, auto jc, int slot, int halves = 3) __attribute__((always_inline)) {   // halves: bit 0 slab 0, bit 1 slab 1
      constexpr int j = decltype(jc)::value;
      const int kb = kb_t - (j == 0 ? kbase0 : kbase);
      const bool in = !(Cfg::TIMING & kTimingFetchNowhere) && (!Cfg::ODDK || kb < KB);
      uint8_t* dst = bslots + slot * Cfg::B_SLOT_BYTES;
      // all 256 weight rows of the tile exist: only the lane part of the offset needs the bounds check
      const int kp = k_wrapped(kb + (j == 0 ? rot0 : rot), KB);
      const bool last = Cfg::RAGGED && kp == KB - 1;
      const int so = __builtin_amdgcn_readfirstlane(kp * 128 + j * frag1_off);
      if constexpr (Cfg::TIMING & kTimingFetchToRegs) {
        if (halves & 1) timing_fetch16(sink, vB0, j == 0 ? dB0 : dB, so);
        if (halves & 2) timing_fetch16(sink, vB1, j == 0 ? dB0 : dB, so);
        return;
      }
      if (halves & 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(j == 0 ? dB0 : dB, GG_LDS_PTR(dst), 16, in ? (last ? vB0_last : vB0) : GG_OOB_OFFSET, so, 0, 0);
      if (halves & 2) __builtin_amdgcn_raw_ptr_buffer_load_lds(j == 0 ? dB0 : dB, GG_LDS_PTR(dst + 1024), 16, in ? (last ? vB1_last : vB1) : GG_OOB_OFFSET, so, 0, 0);
    };
    constexpr std::integral_constant<int, 0> J0{};
    constexpr std::integral_constant<int, 1> J1{};
    auto read_frag = [&](const uint8_t* p) __attribute__((always_inline)) -> v8i {   // 16 rows x 128 B at p -> MFMA operand
      const v4i lo = *(const v4i*)(p + rd0);
      const v4i hi = *(const v4i*)(p + rd1);
      return (v8i){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };

    // The next tile is looked up here, not where it is first needed: the four K steps at the end of the tile stay
    // one basic block.
    const Tile nxt = find_tile(it + 1);
    const bool has_next = nxt.valid;
    // (One copy of the tile's code per kernel: with a copy for full and a copy for partly filled tiles behind a
    // branch, the state carried from tile to tile ends up in different registers in the two and the kernel spills.)
    constexpr std::bool_constant<Cfg::SKIP> pred_c{};
    v4f acc[TM][TN];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[mt][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    // ---- prologue ---------------------------------------------------------------------------------------
    // Weight fragments are numbered F = 2*kb + j and go through slot F % 3.  Fetch A(0), fragments 0..2 and
    // A(1); once A(0) and fragments 0, 1 have landed, copy those to registers and refill their slots with
    // fragments 3 and 4.  That is the state every K block starts from: A(kb+1) and fragment 2kb+2 older than
    // the last 4 fetches, which are the refills with fragments 2kb+3 and 2kb+4.
    if (!primed) {
      dma_scales(0, 0);
      static_for<0, Cfg::A_ITERS>([&](auto ic) __attribute__((always_inline)) { dma_a(ic, 0, 0); });
      dma_b(0, J0, 0);
      dma_b(0, J1, 1);
      dma_b(1, J0, 2);
      dma_scales(1, 1);
      static_for<0, Cfg::A_ITERS>([&](auto ic) __attribute__((always_inline)) { dma_a(ic, 1, 1); });
      wait_vmcnt<2 + Cfg::N_A>();
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");

      bfr[0][0] = read_frag(bslots);
      bfr[0][1] = read_frag(bslots + Cfg::B_SLOT_BYTES);
#pragma unroll
      for (int i = 0; i < AFR - 1; ++i) afr[i] = read_frag(lds + i * 2048);
      sa4[0] = *(const v4f*)(lds + saRd);
      // the slot reads must be done before their slots are refilled
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      dma_b(1, J1, 0);
      dma_b(2, J0, 1);

      sb_next = *(const float*)(lds + sbRd);                   // weight scale of block 0
      if constexpr (Cfg::FUSE) sb_next_up = *(const float*)(lds + sbRd + 4);
      stage = 0;
      bslot = 2;
    }
    // One K block; BS = kb % 2 is the register set that holds its weights.  PRED: the step of a partly filled tile,
    // which runs the activation blocks [0, tm_act) only; the fetches, the copies of the weight fragments and the
    // reads of the next K block's first activation fragments are those of a full step.
    auto kstep = [&](int kb, auto bs_c, auto pred_c) __attribute__((always_inline)) {
      constexpr int BS = decltype(bs_c)::value;
      constexpr bool PRED = decltype(pred_c)::value;
      static_assert(!(PRED && Cfg::FUSE), "the activation epilogue runs full steps only");
      // opaque to the compiler, which otherwise hoists the tests on it out of the K loop and keeps one copy of the
      // loop per tile height
      int tm_run = tm_act;
      if constexpr (PRED) asm volatile("" : "+s"(tm_run));
      const int stage1 = stage + 1 == S ? 0 : stage + 1;       // buffer of block kb+1
      const int stageN = stage == 0 ? S - 1 : stage - 1;       // buffer of block kb+2 (= of block kb-1)
      const int bslot1 = bslot + 1 == Cfg::B_SLOTS ? 0 : bslot + 1;   // slot of fragment 2*kb + 3
      const uint8_t* st = lds + stage * Cfg::STAGE_BYTES;
      const uint8_t* st1 = lds + stage1 * Cfg::STAGE_BYTES;
      // A(kb+1), its scales and weight fragment 2kb+2 are older than the 4 refill DMAs of block kb-1.  (Stores
      // of the previous tile are older still: they can only make this wait longer, never shorter.)
      if constexpr (!(Cfg::TIMING & kTimingNoFetchWaits)) wait_vmcnt<Cfg::W_TOP>();
      // every wave has its part of block kb+1 in LDS and is done reading block kb-1
      if constexpr (!(Cfg::TIMING & kTimingNoBarrier)) __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      const float sb = sb_next, sb_up = sb_next_up;            // read a block ago: no LDS wait ahead of the first MFMA
      bfr[BS ^ 1][0] = read_frag(bslots + bslot * Cfg::B_SLOT_BYTES);
      if constexpr (!(Cfg::TIMING & kTimingNoFetch)) dma_scales(kb + 2, stageN);
      __builtin_amdgcn_sched_barrier(0);

      v4f p[MF];
      float s[TM], s_up[Cfg::FUSE ? TM : 1];
      // register of band b of this K step: bands are numbered through the K steps (an odd number of bands per step
      // flips the assignment from step to step; a tile has an even number of steps and starts with register 0)
      auto band_reg = [](int b) constexpr { return (BS * (Cfg::NBAND & 1) + b) & 1; };
      // the scale reads of activation block mt (after the block's own scale product: in-order issue keeps the
      // register's previous band intact for it)
      auto read_scales = [&](auto mc) __attribute__((always_inline)) {
        constexpr int mt = decltype(mc)::value;
        if constexpr (Cfg::TIMING & kTimingNoLdsReads) {
          // the empty asm makes the register's old contents a new value for the compiler, as a read would
          if constexpr (mt % 4 == 1 && mt / 4 + 1 < Cfg::NBAND) asm volatile("" : "+v"(sa4[band_reg(mt / 4 + 1)]));
          if constexpr (mt == Cfg::R_NEXT) asm volatile("" : "+v"(sa4[band_reg(Cfg::NBAND)]));
        } else {
          if constexpr (mt % 4 == 1 && mt / 4 + 1 < Cfg::NBAND) sa4[band_reg(mt / 4 + 1)] = *(const v4f*)(st + saRd + (mt / 4 + 1) * 256);
          if constexpr (mt == Cfg::R_NEXT) sa4[band_reg(Cfg::NBAND)] = *(const v4f*)(st1 + saRd);
        }
      };
      auto body = [&](auto tc) __attribute__((always_inline)) {
        constexpr int t = decltype(tc)::value;
        if constexpr (t < MF) {
          constexpr int mt = t / TN, j = t % TN;
          if constexpr (j == 0) {
            s[mt] = sa4[band_reg(mt / 4)][mt % 4] * sb;
            if constexpr (Cfg::FUSE) s_up[mt] = sa4[band_reg(mt / 4)][mt % 4] * sb_up;
            // fragment of activation block mt + AFR - 1 into the slot block mt - 1 has left; past the end of
            // this K block that is the next K block's, published by the barrier above
            constexpr int nb = mt + AFR - 1;
            if constexpr (Cfg::TIMING & kTimingNoLdsReads) {
              asm volatile("" : "+v"(afr[nb % AFR]));
            } else if constexpr (nb < TM) {
              afr[nb % AFR] = read_frag(st + nb * 2048);
            } else {
              afr[nb % AFR] = read_frag(st1 + (nb - TM) * 2048);
              if constexpr (nb == TM) {                                         // next block's weight scale(s)
                sb_next = *(const float*)(st1 + sbRd);
                if constexpr (Cfg::FUSE) sb_next_up = *(const float*)(st1 + sbRd + 4);
              }
            }
            read_scales(std::integral_constant<int, mt>{});
          }
          p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[BS][j], afr[mt % AFR], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
          if constexpr (!(Cfg::TIMING & kTimingNoFetch)) {
            if constexpr (t >= Cfg::T_A0 && t < Cfg::T_A0 + Cfg::A_STEP * Cfg::A_ITERS && (t - Cfg::T_A0) % Cfg::A_STEP == 0)
              dma_a(std::integral_constant<int, (t - Cfg::T_A0) / Cfg::A_STEP>{}, kb + 2, stageN);
            // refills: fragment F+3 into the slot fragment F was copied from, some MFMAs (and the LDS reads they
            // waited for, which return in order) after that copy
            if constexpr (Cfg::R_STEP == 0) {
              if constexpr (t == Cfg::T_R0) dma_b(kb + 2, J1, bslot);       // 2kb+2 -> 2kb+5
              if constexpr (t == Cfg::T_R1) dma_b(kb + 3, J0, bslot1);      // 2kb+3 -> 2kb+6
            } else {
              if constexpr (t == Cfg::T_R0) dma_b(kb + 2, J1, bslot, 1);
              if constexpr (t == Cfg::T_R0 + Cfg::R_STEP) dma_b(kb + 2, J1, bslot, 2);
              if constexpr (t == Cfg::T_R1) dma_b(kb + 3, J0, bslot1, 1);
              if constexpr (t == Cfg::T_R1 + Cfg::R_STEP) dma_b(kb + 3, J0, bslot1, 2);
            }
          }
        }
        if constexpr (t >= PIPE) {
          constexpr int u = t - PIPE;
          if constexpr (Cfg::FUSE && u % TN == 1) acc[u / TN][1] += p[u] * s_up[u / TN];
          else acc[u / TN][u % TN] += p[u] * s[u / TN];
        }
      };
      auto order = [&](auto tc) __attribute__((always_inline)) {               // issue order of what body creates
        constexpr int t = decltype(tc)::value;
        if constexpr (t < MF) {
          constexpr int j = t % TN;
          if constexpr (j == 0) {
            __builtin_amdgcn_sched_group_barrier(0x002, Cfg::FUSE ? 2 : 1, 0);                   // scale product(s)
            constexpr int mt = t / TN;                                                           // DS reads: 2 of a fragment,
            if constexpr (!(Cfg::TIMING & kTimingNoLdsReads))
              __builtin_amdgcn_sched_group_barrier(0x100, 2 + (mt + AFR - 1 == TM ? (Cfg::FUSE ? 2 : 1) : 0)   // weight scale(s),
                                                              + (mt % 4 == 1 && mt / 4 + 1 < Cfg::NBAND ? 1 : 0) + (mt == Cfg::R_NEXT ? 1 : 0), 0);   // a band of scales
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                     // 1 MFMA
          if constexpr (t >= Cfg::T_A0 && t < Cfg::T_A0 + Cfg::A_STEP * Cfg::A_ITERS && (t - Cfg::T_A0) % Cfg::A_STEP == 0) {
            __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);                                   // offset select
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          }
          if constexpr (Cfg::R_STEP == 0) {
            if constexpr (t == Cfg::T_R0 || t == Cfg::T_R1) {
              __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
              __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
            }
          } else if constexpr (t == Cfg::T_R0 || t == Cfg::T_R1 || t == Cfg::T_R0 + Cfg::R_STEP || t == Cfg::T_R1 + Cfg::R_STEP) {
            __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          }
        }
        if constexpr (t >= PIPE) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);              // 4 FMAs
      };
      // One scheduling region per activation block (2 MFMAs, the 8 FMAs of earlier MFMAs, 3 LDS reads, at most
      // two fetches): the software pipeline is written out in the source, the regions keep the compiler from
      // rearranging it across blocks.
      static_for<0, TM>([&](auto mc) __attribute__((always_inline)) {
        constexpr int mt = decltype(mc)::value;
        if constexpr (mt * TN == Cfg::T_MID) {
          // weight fragment 2kb+3, fetched a K block ago, is older than the W_MID newest fetches
          if constexpr (!(Cfg::TIMING & kTimingNoFetchWaits)) wait_vmcnt<Cfg::W_MID>();
          bfr[BS ^ 1][1] = read_frag(bslots + bslot1 * Cfg::B_SLOT_BYTES);
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (!PRED) {
          static_for<mt * TN, mt * TN + TN>(body);
          static_for<mt * TN, mt * TN + TN>(order);
        } else {
          constexpr int nb = mt + AFR - 1;
          s[mt] = sa4[band_reg(mt / 4)][mt % 4] * sb;     // before the band reads below, which may refill that register
          if constexpr (nb >= TM) {              // the next K block's first fragments and scales: always
            afr[nb % AFR] = read_frag(st1 + (nb - TM) * 2048);
            if constexpr (nb == TM) sb_next = *(const float*)(st1 + sbRd);
          }
          read_scales(std::integral_constant<int, mt>{});
          if (mt < tm_run) {
            if constexpr (nb < TM) afr[nb % AFR] = read_frag(st + nb * 2048);
            p[mt * TN] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[BS][0], afr[mt % AFR], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
            p[mt * TN + 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[BS][1], afr[mt % AFR], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
            if constexpr (mt >= 1) {             // the FMAs of the block before this one
              acc[mt - 1][0] += p[(mt - 1) * TN] * s[mt - 1];
              acc[mt - 1][1] += p[(mt - 1) * TN + 1] * s[mt - 1];
            }
            if constexpr (nb < TM) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if constexpr (mt >= 1) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if constexpr (mt >= 1) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          }
          static_for<mt * TN, mt * TN + TN>([&](auto tc) __attribute__((always_inline)) {
            constexpr int t = decltype(tc)::value;
            if constexpr (t >= Cfg::T_A0 && t < Cfg::T_A0 + Cfg::A_ITERS)
              dma_a(std::integral_constant<int, t - Cfg::T_A0>{}, kb + 2, stageN);
            if constexpr (t == Cfg::T_R0) dma_b(kb + 2, J1, bslot);
            if constexpr (t == Cfg::T_R1) dma_b(kb + 3, J0, bslot1);
          });
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      if constexpr (!PRED) {
        static_for<MF, MF + PIPE>(body);
        static_for<MF, MF + PIPE>(order);
        __builtin_amdgcn_sched_barrier(0);
      } else {
        if (tm_run >= TM) {                      // a full tile: the FMAs of its last block
          acc[TM - 1][0] += p[(TM - 1) * TN] * s[TM - 1];
          acc[TM - 1][1] += p[(TM - 1) * TN + 1] * s[TM - 1];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      stage = stage1;
      bslot = bslot1 + 1 == Cfg::B_SLOTS ? 0 : bslot1 + 1;
      // The accumulators are "used" here: outside a loop the compiler otherwise sinks a step's accumulator updates
      // down to their next use in a later basic block, and every product of the step stays alive until there.
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(acc[mt][j]));
    };

    // The copies of the block for the two register sets follow each other in a straight line (no if/else over
    // copies: their identical accumulator updates would be merged behind the branches, and all products of a
    // block would be live at once).
    constexpr std::integral_constant<int, 0> SET0{};
    constexpr std::integral_constant<int, 1> SET1{};
    {
      for (int kb = 0; kb < KBe - 4; kb += 2) {
        kstep(kb, SET0, pred_c);
        kstep(kb + 1, SET1, pred_c);
      }
      // step KB-4 issues the last fetch of this tile's j = 0 fragments (block KB-1); step KB-3 the last fetches of
      // its activations, scales and j = 1 fragments.  After each, that stream moves on to the next tile.
      kstep(KBe - 4, SET0, pred_c);
      dB0 = desc_b(nxt, has_next);
      rot0 = k_rotation(a, nxt.n0);
      kbase0 = KBe;
      kstep(KBe - 3, SET1, pred_c);
      dA0 = band(nxt, 0, has_next); dA1 = band(nxt, 1 % Cfg::A_ITERS, has_next);
      dA2 = band(nxt, 2 % Cfg::A_ITERS, has_next); dA3 = band(nxt, 3 % Cfg::A_ITERS, has_next);
      dB = dB0;
      dS = desc_s(nxt, has_next);
      rot = rot0;
      kbase = KBe;
      kstep(KBe - 2, SET0, pred_c);
      kstep(KBe - 1, SET1, pred_c);
      kbase = kbase0 = 0;
    }

    if constexpr (Cfg::FUSE) {
      // ---- fused epilogue: act = bf16(silu(bf16(gate)) * bf16(up)), then the 1x128 block quantiser on act ------
      // The two projections are rounded to bfloat16 first, as if the GEMM had stored them, and everything after
      // that is the arithmetic of the separate activation kernel, so the bytes, scales and activations equal
      // that kernel's on this GEMM's output bit for bit.  A row's 128 activation columns are spread over the 8
      // waves (16 columns each: 4 lane groups x 4 values): the block maximum goes through LDS.
      uint8_t* red = lds + Cfg::RED_BASE;
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        const v4f x = acc[mt][0], y = acc[mt][1];
        const int a01 = swiglu2(pack2_rne(x[0], x[1], false), pack2_rne(y[0], y[1], false));
        const int a23 = swiglu2(pack2_rne(x[2], x[3], false), pack2_rne(y[2], y[3], false));
        const float v[4] = {__builtin_bit_cast(float, a01 << 16), __builtin_bit_cast(float, a01 & (int)0xFFFF0000),
                            __builtin_bit_cast(float, a23 << 16), __builtin_bit_cast(float, a23 & (int)0xFFFF0000)};
        unsigned top = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned t = amax_bits_of(v[i]);
          top = top > t ? top : t;
        }
        unsigned o = (unsigned)__shfl_xor((int)top, 16);
        top = top > o ? top : o;
        o = (unsigned)__shfl_xor((int)top, 32);
        top = top > o ? top : o;
        if (q == 0) *(unsigned*)(red + ((mt * 16 + r) * NW + w) * 4) = top;
        acc[mt][0] = (v4f){v[0], v[1], v[2], v[3]};                  // keep the activations, drop the projections
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      const int ntile = n0 >> 7;
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        const v4i m0 = *(const v4i*)(red + (mt * 16 + r) * NW * 4);
        const v4i m1 = *(const v4i*)(red + (mt * 16 + r) * NW * 4 + 16);
        unsigned top = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          top = top > (unsigned)m0[i] ? top : (unsigned)m0[i];
          top = top > (unsigned)m1[i] ? top : (unsigned)m1[i];
        }
        const float amax = block_amax(top);
        const float scale = amax / 448.0f;
        const float inv = 448.0f / amax;
        const float v[4] = {acc[mt][0][0], acc[mt][0][1], acc[mt][0][2], acc[mt][0][3]};
        const int bytes = e4m3x4_of(v, inv);
        int rows_mt = rows_valid - 16 * mt;
        rows_mt = rows_mt < 0 ? 0 : rows_mt;
        // bounded views of 16 rows, as for C below; a lane's 4 columns are 16w + 4q .. + 3 of the tile's 128
        __amdgpu_buffer_rsrc_t dQ = uniform_rsrc(a.A2 + (grow + 16 * mt) * inter + n0, rows_mt > 0 ? rows_mt * inter - n0 : 0);
        __builtin_amdgcn_raw_buffer_store_b32(bytes, dQ, r * inter + w * 16 + 4 * q, 0, 0);
        if (a.act_out) {
          __amdgpu_buffer_rsrc_t dAct = uniform_rsrc(a.act_out + (grow + 16 * mt) * inter + n0, rows_mt > 0 ? (rows_mt * inter - n0) * 2 : 0);
          // the activations are bfloat16 values held as floats: their upper halves are the bits to store
          const v2i pk = {(int)((__builtin_bit_cast(unsigned, v[0]) >> 16) | (__builtin_bit_cast(unsigned, v[1]) & 0xFFFF0000u)),
                          (int)((__builtin_bit_cast(unsigned, v[2]) >> 16) | (__builtin_bit_cast(unsigned, v[3]) & 0xFFFF0000u))};
          __builtin_amdgcn_raw_buffer_store_b64(pk, dAct, (r * inter + w * 16 + 4 * q) * 2, 0, 0);
        }
        if (w == 0 && q == 0 && r < rows_mt) a.SA2[(grow + 16 * mt + r) * a.sa2_row_stride + (int64_t)ntile * a.sa2_kb_stride] = scale;
      }
    } else {
    // ---- epilogue: bf16 (or binary16) RNE, one bounded 16-byte store per activation block ---------------------------------
    const int cSrc = (16 * (l & 3) + (l >> 2)) * 4;      // byte address of the lane whose 16 bytes lane l stores
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const v4f x = acc[mt][0], y = acc[mt][1];
      const bool f16 = a.out_f16 != 0;
      v4i out;
      out.x = pack2_rne(x[0], x[1], f16);
      out.y = pack2_rne(x[2], x[3], f16);
      out.z = pack2_rne(y[0], y[1], f16);
      out.w = pack2_rne(y[2], y[3], f16);
      // one descriptor per 16-row block (scalar work): the lane offset is then the same for every block, and
      // rows past the group's end still fail its bounds check
      int rows_mt = rows_valid - 16 * mt;
      rows_mt = rows_mt < 0 ? 0 : rows_mt;
      __amdgpu_buffer_rsrc_t dC = uniform_rsrc(a.C + (grow + 16 * mt) * N + n0, rows_mt > 0 ? rows_mt * N * 2 - n0 * 2 : 0);
      // The lane (q, r) holds 16 bytes of row r; stored from there, neighbouring lanes would write to different
      // rows and every lane's piece would be a request of its own.  Lane 4 r + q takes them instead (a transpose of
      // the lane grid through the LDS crossbar), so that four neighbouring lanes write the wave's 64 bytes of a row.
      out.x = __builtin_amdgcn_ds_bpermute(cSrc, out.x);
      out.y = __builtin_amdgcn_ds_bpermute(cSrc, out.y);
      out.z = __builtin_amdgcn_ds_bpermute(cSrc, out.z);
      out.w = __builtin_amdgcn_ds_bpermute(cSrc, out.w);
      // RAGGED: N is a multiple of 8, so a lane's 8 columns exist together or not at all
      const bool col_ok = !Cfg::RAGGED || n0 + w * 32 + 8 * (l & 3) < N;
      __builtin_amdgcn_raw_buffer_store_b128(out, dC, col_ok ? (l >> 2) * N * 2 + (w * 32 + 8 * (l & 3)) * 2 : GG_OOB_OFFSET, 0, 0);
    }
    }
    if (!has_next) {
      // the dropped fetches of the last K blocks still write zeros into this workgroup's LDS: let them land
      wait_vmcnt<0>();
      if constexpr (Cfg::TIMING & kTimingFetchToRegs) asm volatile("" : : "v"(sink));
      return;
    }
    cur = nxt;
    primed = true;
  }
}

}  // namespace gg
