// Padding-free block-scaled FP8 grouped GEMM kernel for gfx950 (MI355X).
//
// Computes, for every group g, row r of the group and column n (paper Sec. 2.1, Table 1):
//   C[r][n] = bf16( sum_kb SA[r][kb] * SB[g][n/128][kb] * sum_{k in block kb} A[r][k] * B[g][n][k] )
// with arbitrary rows per group and no padded copy (the capability of Sec. 2.2).  What the paper
// obtains on Hopper with a pool of store descriptors and two overlapping stores is obtained here
// with buffer descriptors whose num_records ends at the last valid row of the tile: loads past it
// return zero, stores past it are dropped by the hardware.
//
// Structure
//  * persistent workgroups walk the list of (group, m-tile, n-tile) derived on the device from
//    group_offsets; workgroup b serves XCD b % 8, and every XCD takes contiguous runs of the tile
//    list so that tiles running together on one XCD share A row panels and B column panels in
//    that XCD's L2;
//  * per K block of 128 the A tile [BM x 128 B], the B tile [BN x 128 B] and BM scales of A are
//    DMA'd global -> LDS (buffer_load ... lds, 16 B per lane) into a ring of STAGES buffers, with an
//    XOR swizzle on 16-byte chunks applied on the global-address side so that the later
//    ds_read_b128 operand reads are bank-conflict free;
//  * one v_mfma_f32_16x16x128_f8f6f4 with a zero C operand produces the partial sums of one scale
//    block; the weights sit on the MFMA row side and the activations on the column side, so a lane
//    holds ONE activation row per MFMA and the dequantisation is 4 fp32 FMAs with a per-lane
//    scalar  s = SA[row][kb] * SB[g][n/128][kb]  into the fp32 accumulators (the scale fusion);
//  * the epilogue rounds to bf16 (RNE) and issues bounded 16-byte stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace gg {

// compile-time loop: f(std::integral_constant<int, I>{}) for I in [B, E)
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}


typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

// two fp32 -> one dword of two 2-byte floats, round to nearest even: bfloat16, or IEEE binary16 when f16 is set
// (the two readings of the paper's "half-precision" output; f16 is uniform over the launch)
__device__ __forceinline__ int pack2_rne(float a, float b, bool f16) {
  if (f16) return __builtin_bit_cast(int, __builtin_convertvector((v2f){a, b}, v2h));
  return __builtin_bit_cast(int, __builtin_convertvector((v2f){a, b}, v2bf));
}

#define GG_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
// The group offsets are read through the constant address space: nothing writes them while a kernel of this library
// runs, and the compiler then fetches them with scalar loads wherever the index is uniform.  (As plain global loads
// they become vector loads once the kernel has stored anything, each followed by a wait for every fetch in flight.)
#define GG_CONST_I32 __attribute__((address_space(4))) int32_t
// dword 3 of a raw buffer descriptor on gfx9-family parts: 32-bit data format, no swizzle
#define GG_RSRC_FLAGS 0x00020000
// a lane offset that fails the bounds check of every descriptor used here: the access returns zeros / is dropped
#define GG_OOB_OFFSET 0x7fffff00

struct GemmArgs {
  const uint8_t* A;
  const float* SA;
  const uint8_t* B;
  const float* SB;
  const int32_t* off;
  uint16_t* C;
  int G;
  int M_total;   // rows of A / C (clamp for untrusted offsets)
  int N, K, KB;  // KB = ceil(K / 128)
  int n_tiles;   // N / BN
  int n_chunk;   // n-tiles that are walked together before moving to the next m-tile
  int slots;     // workgroups per XCD when the grid is a multiple of 8, else 0 (plain round-robin)
  int k_rem;     // bytes of a row that fall into the last K block: K - 128 * (KB - 1), in (0, 128]
  int out_f16;   // 0: C is bfloat16, 1: C is IEEE binary16
  int rot_mul;   // K blocks by which neighbouring 256-column blocks shift the start of their K loop (0: none)
  // Storage order of SA, in bytes: the scale of (row, K block kb) is at row * sa_row_stride + kb * sa_kb_stride.
  // Row-major [M_total, KB]: (4 * KB, 4); K-block-major [KB, M_total]: (4, 4 * M_total), where the scales one
  // K block of a tile needs are contiguous (a few cache lines instead of one per row).
  int sa_row_stride, sa_kb_stride;
  int sa_kmajor;   // 1 for the second order
  // fused activation epilogue of the second kernel (N = 2 * I weight rows: gate rows [0, I), up rows [I, 2I)):
  // A2 [M_total, I] e4m3, SA2 one scale per (row, 128 activation columns) at row * sa2_row_stride + block *
  // sa2_kb_stride (elements), act_out [M_total, I] bf16 or null
  uint8_t* A2;
  float* SA2;
  uint16_t* act_out;
  int64_t sa2_row_stride, sa2_kb_stride;
  // split-K instantiation: partial sums [2][M_total][N] fp32 (K blocks [0, KB/2) and [KB/2, KB) of every valid row)
  float* P;
};

// Length in bytes of the view of SA that starts at the scale of (first row of a tile, K block 0).  The K-block part
// of a scale's address travels in the scalar offset of the fetch, which the range check adds to the lane offset
// before it compares with the length.  Row-major: rows_valid scale rows, so rows past the group's end read as
// zero.  K-block-major: everything up to the end of the tensor; a row past the group's end then reads some other
// row's scale, which only ever meets that row's all-zero activations in an accumulator that is never stored.
__device__ __forceinline__ int sa_view_bytes(const GemmArgs& a, int64_t grow, int rows_valid) {
  return a.sa_kmajor ? (int)(((int64_t)a.KB * a.M_total - grow) * 4) : rows_valid * a.sa_row_stride;
}

template <int BM_, int BN_, int WM_, int WN_, int STAGES_, bool XPF_ = false, int GAP_ = 0, int PIPE_ = 3>
struct GemmCfg {
  static constexpr int GAP = GAP_;            // MFMAs between two in-stream DMAs (0 = spread over the whole stream)
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, STAGES = STAGES_;
  static constexpr int NW = WM * WN;          // waves per workgroup
  static constexpr int NT = 64 * NW;          // threads per workgroup
  static constexpr int WTM = BM / WM;         // rows of A per wave
  static constexpr int WTN = BN / WN;         // columns per wave
  static constexpr int TM = WTM / 16;         // MFMA column blocks (activation rows) per wave
  static constexpr int TN = WTN / 16;         // MFMA row blocks (weight rows) per wave
  static constexpr int A_BYTES = BM * 128;
  static constexpr int B_BYTES = BN * 128;
  static constexpr int SA_WAVES = (BM + 63) / 64;   // one 64-lane dword DMA fetches the scales of 64 rows
  static constexpr int SA_ROWS = SA_WAVES * 64;
  static constexpr int SA_BYTES = SA_ROWS * 4;
  static constexpr int SB_BYTES = 256;         // BN/128 scales of B per K block, replicated over one wave-wide DMA
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES + SA_BYTES + SB_BYTES;
  static constexpr int SB_WAVE = NW - 1;      // the wave that fetches them
  static constexpr int MFMAS = (BM / WM / 16) * (BN / WN / 16);   // MFMAs per wave per K block
  static constexpr int PIPE = MFMAS < PIPE_ ? MFMAS : PIPE_;               // MFMAs in flight before their FMAs are issued
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
  // cross-block operand prefetch with a mid-stream barrier (see the kernel): needs a ring of 3 and an even TM
  static constexpr bool XPF = XPF_;
  static_assert(!XPF_ || (STAGES_ >= 3 && (BM_ / WM_ / 16) % 2 == 0), "XPF needs a ring of 3 buffers and an even TM");
  static constexpr int A_SLABS = BM / 8;      // one slab = 8 rows x 128 B = one wave-wide DMA
  static constexpr int B_SLABS = BN / 8;
  static constexpr int A_ITERS = (A_SLABS + NW - 1) / NW;
  static constexpr int B_ITERS = (B_SLABS + NW - 1) / NW;
  static_assert(BM % (16 * WM) == 0 && BN % (32 * WN) == 0, "wave tile must be 16 x 32 granular");
  static_assert(WTN <= 128 && 128 % WTN == 0, "a wave must stay inside one 128-wide scale block of B");
  static_assert(BM % 8 == 0 && BN % 8 == 0 && NW % 4 == 0, "slab mapping");
  static_assert(TN % 2 == 0, "n sub-tiles are paired for 16-byte stores");
};

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// s_waitcnt vmcnt(N): at most N of this wave's vector-memory operations may still be in flight
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Waits until all but the newest `younger` groups of PER operations have completed (younger <= MAXY).
template <int PER, int MAXY>
__device__ __forceinline__ void wait_all_but_n(int younger) {
  if constexpr (MAXY <= 0) {
    wait_vmcnt<0>();
  } else {
    if (younger >= MAXY) wait_vmcnt<MAXY * PER>();
    else wait_all_but_n<PER, MAXY - 1>(younger);
  }
}
// The same with PER = BASE + extra, extra in [0, 3] known only at run time (wave-uniform).
template <int BASE, int MAXY>
__device__ __forceinline__ void wait_all_but(int younger, int extra) {
  if constexpr (MAXY <= 0) {
    wait_vmcnt<0>();
  } else {
    if (extra == 0) wait_all_but_n<BASE, MAXY>(younger);
    else if (extra == 1) wait_all_but_n<BASE + 1, MAXY>(younger);
    else if (extra == 2) wait_all_but_n<BASE + 2, MAXY>(younger);
    else wait_all_but_n<BASE + 3, MAXY>(younger);
  }
}

// Start of a tile's K loop.  When the row pitch K is 4096 bytes, the 128-byte pieces that a K block takes from the
// rows of a tile all sit at the same offset inside a 4 KB frame, and the workgroups of an XCD walk K nearly in
// step: a pure fetch stream of this shape reaches 4.8 TB/s instead of the 5.9 TB/s of other pitches, and the
// weight-streaming shapes (few rows per group) lose 3-11 % (measured).  Letting the tiles of neighbouring
// 256-column blocks start 4 K blocks (512 B) apart and wrap around gives that back; compute-bound shapes do not
// notice.  The start depends on the column block alone, never on the row tile, the workgroup or the tile shape,
// so that an output element is accumulated in the same order by every variant and in the padded and the
// padding-free path (their bitwise equality, paper Sec. 3.1, is kept).  The host sets rot_mul = 4 for pitches
// that are odd multiples of 4096 and 0 otherwise (at K = 8192 the shift costs 1-8 %, measured).
__device__ __forceinline__ int k_rotation(const GemmArgs& a, int n0) { return ((n0 >> 8) & 7) * a.rot_mul; }
__device__ __forceinline__ int k_wrapped(int k, int KB) { return k >= KB ? k - KB : k; }

// XOR keys of the LDS swizzle: 16-byte chunk c of tile row `row` is stored at chunk position c ^ key(row).
// ds_read_b128 serves 16 lanes per cycle, and on gfx950 those are not 16 consecutive lanes: of every 32
// lanes, the quads {0,3,5,6} go together and the quads {1,2,4,7} go together (measured with two-lane
// probes and SQ_LDS_BANK_CONFLICT).  With MFMA operand lanes (r = lane % 16, q = lane / 16) reading chunks
// 2q and 2q+1 of row f(r), a cycle therefore sees every r once, with q advanced by one for r in 4..11.
// The keys below make the 16 lanes of each such cycle hit 16 different 16-byte bank groups.
__device__ __forceinline__ int swz_key_a(int row) {   // rows read: base + r
  const int u = (row >> 1) & 7;
  return u ^ ((((u >> 1) ^ (u >> 2)) & 1) << 1);
}
__device__ __forceinline__ int swz_key_b(int row) {   // rows read: base + 8*(r/4) + r%4
  const int b1 = (row >> 1) & 1, b4 = (row >> 4) & 1;
  return b1 | (b4 << 1) | (b4 << 2);
}

// RAGGED: N need not be a multiple of the tile width nor K of 128 (the ceilings in Table 1 of the paper); costs a
// few lane selects per fetch, so shapes made of whole blocks use the instantiation without it.
// SPLITK: the work list holds two units per tile, one per half of the K loop (K blocks [0, KB/2) and [KB/2, KB)),
// and a unit stores its fp32 partial sums instead of C; gg_splitk_combine_kernel adds the two halves in that order
// and rounds (paper Sec. 3.2: where few rows meet many weights, a launch has too few tiles to fill the chip; the K
// loop is the one dimension left to split).  KB must be even; whole tiles and whole K blocks only.
// BSTREAM: the weight fetches carry the streaming cache policy (nt sc1).  For groups of at most one row tile every
// weight byte is fetched once; left to the default policy the 7.5 GB of a 256-expert layer push the activation tiles
// (which the 16 column tiles of a group share) out of the L2.  Where several row tiles share a group's weights the
// policy costs 17 - 35 %, so the host asks for it only when M_total <= G * BM.
template <class Cfg, bool RAGGED = false, bool SPLITK = false, bool BSTREAM = false>
__global__ void __launch_bounds__(Cfg::NT) gg_gemm_kernel(const GemmArgs a) {
  constexpr int kBAux = BSTREAM ? (2 | 16) : 0;
  static_assert(!(SPLITK && (RAGGED || Cfg::XPF)), "split-K: whole tiles, the ring-of-buffers path");
  constexpr int BM = Cfg::BM, BN = Cfg::BN, WN = Cfg::WN, NW = Cfg::NW;
  constexpr int TM = Cfg::TM, TN = Cfg::TN, WTM = Cfg::WTM, WTN = Cfg::WTN, STAGES = Cfg::STAGES;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l = tid & 63;
  const int r = l & 15, q = l >> 4;
  const int wm = w / WN, wn = w % WN;
  const int K = a.K, KB = a.KB, N = a.N;
  const int KBu = SPLITK ? KB >> 1 : KB;      // K blocks per work unit

  // ---- per-lane constants of the global -> LDS DMA -------------------------------------------
  // lane l of a wave-wide 16 B DMA lands at LDS byte 16*l of the slab: row l/8, physical chunk l%8.
  // The logical chunk it must fetch is physical ^ key(row).
  const int lrow = l >> 3, pch = l & 7;
  const int a_row = w * 8 + lrow;                                   // + i*NW*8
  const int keyA_ld = swz_key_a(a_row);
  const int b_row = w * 8 + lrow;
  const int keyB_ld = swz_key_b(b_row);
  const int vA = a_row * K + ((pch ^ keyA_ld) << 4);
  const int vB = b_row * K + ((pch ^ keyB_ld) << 4);
  // K not a multiple of 128 (ceilings in Table 1 of the paper): in the last K block the 16-byte chunks at or past
  // byte k_rem of the block belong to the next row; those lanes fetch from an out-of-range offset, i.e. zeros
  const bool a_tail = RAGGED && ((pch ^ keyA_ld) << 4) >= a.k_rem;
  const bool b_tail = RAGGED && ((pch ^ keyB_ld) << 4) >= a.k_rem;
  const int vSA = (w * 64 + l) * a.sa_row_stride;
  const int vSB = (l < BN / 128 ? l : BN / 128 - 1) * KB * 4;        // lane -> which 128-wide N block of the tile

  // DMAs this wave issues per K block = A_SLABS/NW + B_SLABS/NW + dma_extra (slab remainders, scale fetches)
  static_assert(Cfg::SA_WAVES <= Cfg::SB_WAVE, "scale fetchers must be distinct waves");
  static_assert((Cfg::A_SLABS % NW != 0) + (Cfg::B_SLABS % NW != 0) + 1 <= 3, "extra DMA count out of range");
  const int dma_extra = (w < Cfg::A_SLABS % NW) + (w < Cfg::B_SLABS % NW) + ((w < Cfg::SA_WAVES) || (w == Cfg::SB_WAVE));

  // ---- per-lane constants of the LDS operand reads --------------------------------------------
  const int keyA_rd = swz_key_a(r);
  const int rowB_rd = 8 * (r >> 2) + (r & 3);
  const int keyB_rd = swz_key_b(rowB_rd);
  const int aRd0 = (wm * WTM + r) * 128 + (((2 * q) ^ keyA_rd) << 4);
  const int aRd1 = (wm * WTM + r) * 128 + (((2 * q + 1) ^ keyA_rd) << 4);
  const int bRd0 = Cfg::A_BYTES + (wn * WTN + rowB_rd) * 128 + (((2 * q) ^ keyB_rd) << 4);
  const int bRd1 = Cfg::A_BYTES + (wn * WTN + rowB_rd) * 128 + (((2 * q + 1) ^ keyB_rd) << 4);
  const int saRd = Cfg::A_BYTES + Cfg::B_BYTES + (wm * WTM + r) * 4;
  const int sbRd = Cfg::A_BYTES + Cfg::B_BYTES + Cfg::SA_BYTES + ((wn * WTN) >> 7) * 4;

  // ---- persistent walk over the tile list ---------------------------------------------------------
  // A workgroup knows its next tile while it works on the current one: in the ring-of-buffers path without the
  // mid-stream barrier the last STAGES-1 K blocks of a tile, which have nothing left to fetch for it, fetch the
  // first STAGES-1 K blocks of the next tile instead, so the ring does not run dry across the epilogue.
  struct Tile {
    bool valid;
    int g, n0, rows_valid;
    int64_t grow;
    int ks;          // SPLITK: which half of the K loop
  };
  int g = 0, base = 0;
  const int nwg = gridDim.x;
  const GG_CONST_I32* offc = (const GG_CONST_I32*)a.off;
  auto find_tile = [&](int it) __attribute__((always_inline)) -> Tile {
    Tile t = {false, 0, 0, 0, 0, 0};
    int T;
    if (a.slots > 0) T = (it * 8 + (int)(blockIdx.x & 7)) * a.slots + (int)(blockIdx.x >> 3);
    else T = it * nwg + blockIdx.x;
    if constexpr (SPLITK) {          // the two halves of a tile are neighbours in the list
      t.ks = T & 1;
      T >>= 1;
    }

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
    // order inside a group: chunks of n_chunk n-tiles; inside a chunk m-tile major, n-tile minor
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
    t.n0 = ntile * BN;
    t.rows_valid = Mg - m0 < BM ? Mg - m0 : BM;
    t.grow = (int64_t)row0 + m0;
    t.valid = true;
    return t;
  };
  // bounded views: nothing past the last valid row of a tile is loaded or stored.
  // N not a multiple of the tile width: the weight rows, scale blocks and output columns past N do not exist
  // (the range check compares lane offset + scalar offset + access size with the view's length, so a view that
  // ends after the last existing row refuses exactly the fetches past it)
  const int nb_all = RAGGED ? (N + 127) >> 7 : N >> 7;
  // on = false: a view of length zero, through which every fetch is dropped (same instruction count, no traffic)
  auto desc_a = [&](const Tile& t, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    return __builtin_amdgcn_make_buffer_rsrc((void*)(a.A + t.grow * K), 0, on ? t.rows_valid * K : 0, GG_RSRC_FLAGS);
  };
  auto desc_sa = [&](const Tile& t, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    return __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)a.SA + t.grow * a.sa_row_stride), 0, on ? sa_view_bytes(a, t.grow, t.rows_valid) : 0, GG_RSRC_FLAGS);
  };
  auto desc_b = [&](const Tile& t, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    const int n_rem = N - t.n0;
    return __builtin_amdgcn_make_buffer_rsrc((void*)(a.B + ((int64_t)t.g * N + t.n0) * K), 0, on ? (RAGGED && n_rem < BN ? n_rem : BN) * K : 0, GG_RSRC_FLAGS);
  };
  auto desc_sb = [&](const Tile& t, bool on) __attribute__((always_inline)) -> __amdgpu_buffer_rsrc_t {
    int nb_valid = nb_all - (t.n0 >> 7);
    nb_valid = RAGGED && nb_valid < BN / 128 ? nb_valid : BN / 128;
    return __builtin_amdgcn_make_buffer_rsrc((void*)(a.SB + ((int64_t)t.g * nb_all + (t.n0 >> 7)) * KB), 0, on ? nb_valid * KB * 4 : 0, GG_RSRC_FLAGS);
  };

  // cross-tile prefetch needs a full ring's worth of K blocks per tile, and the path that has it
  const bool xt = !Cfg::XPF && KBu >= STAGES - 1;
  Tile cur = find_tile(0);
  if (!cur.valid) return;
  __amdgpu_buffer_rsrc_t dA = desc_a(cur, true), dSA = desc_sa(cur, true), dB = desc_b(cur, true), dSB = desc_sb(cur, true);
  // first K block of a work unit: the rotation of its column block, or the start of its half of the K loop
  auto k_start = [&](const Tile& t) __attribute__((always_inline)) -> int { return SPLITK ? t.ks * KBu : k_rotation(a, t.n0); };
  int rot = k_start(cur);
  bool primed = false;      // the first STAGES-1 K blocks of `cur` were already fetched by the previous tile
  int stage = 0;            // LDS buffer of the current K block; runs on across tiles
  for (int it = 0;; ++it) {
    const int n0 = cur.n0, rows_valid = cur.rows_valid;
    const int n_rem = N - n0;
    __amdgpu_buffer_rsrc_t dC = __builtin_amdgcn_make_buffer_rsrc((void*)(a.C + cur.grow * N + n0), 0, rows_valid * N * 2 - n0 * 2, GG_RSRC_FLAGS);
    Tile nxt = {false, 0, 0, 0, 0, 0};
    bool has_next = false, prefetch = false;   // known once this tile's own fetches are all issued

    // ---- global -> LDS DMA of one K block, split so that it can be fed into the MFMA stream --------
    // A wave that issues its 8-9 DMAs back to back sits in the issue stage until the CU's vector-memory
    // front end has taken them all (about a thousand cycles when all 8 waves do it at once), so the
    // tile DMAs that every wave issues are spread over the MFMA stream, one per few MFMAs; the ones
    // only some waves issue (slab remainders, scales) would need a branch and go before the stream.
    constexpr int A_FULL = Cfg::A_SLABS / NW, B_FULL = Cfg::B_SLABS / NW;
    constexpr int NDMA_ALL = A_FULL + B_FULL;                                  // issued by every wave
    constexpr int NDMA_STREAM = NDMA_ALL < Cfg::MFMAS ? NDMA_ALL : Cfg::MFMAS;  // of those, inside the stream
    constexpr int DMA_GAP = Cfg::GAP > 0 ? Cfg::GAP : Cfg::MFMAS / (NDMA_STREAM > 0 ? NDMA_STREAM : 1);
    // K blocks are taken in the order rot, rot+1, ..., KB-1, 0, ..., rot-1 (see k_rotation).  dA, dSA, dB, dSB and
    // rot are those of the current tile until its last fetch has been issued, and those of the next tile from then on.
    auto dma_tile = [&](auto idx_c, int kb_l, int stg) {
      constexpr int idx = decltype(idx_c)::value;
      const int kb = k_wrapped(kb_l + rot, KB);
      const bool last = kb == KB - 1;
      uint8_t* st = lds + stg * Cfg::STAGE_BYTES;
      if constexpr (idx < A_FULL) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(dA, GG_LDS_PTR(st + (w + idx * NW) * 1024), 16, (RAGGED && last && a_tail) ? GG_OOB_OFFSET : vA + idx * (NW * 8) * K, kb * 128, 0, 0);
      } else {
        constexpr int i = idx - A_FULL;
        if constexpr (RAGGED)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(dB, GG_LDS_PTR(st + Cfg::A_BYTES + (w + i * NW) * 1024), 16, (last && b_tail) ? GG_OOB_OFFSET : vB + i * (NW * 8) * K, kb * 128, 0, kBAux);
        else
          __builtin_amdgcn_raw_ptr_buffer_load_lds(dB, GG_LDS_PTR(st + Cfg::A_BYTES + (w + i * NW) * 1024), 16, vB, i * (NW * 8) * K + kb * 128, 0, kBAux);
      }
    };
    auto dma_head = [&](int kb_l, int stg) {   // everything that is not issued inside the stream
      const int kb = k_wrapped(kb_l + rot, KB);
      const bool last = kb == KB - 1;
      uint8_t* st = lds + stg * Cfg::STAGE_BYTES;
      if (w < Cfg::SA_WAVES)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(dSA, GG_LDS_PTR(st + Cfg::A_BYTES + Cfg::B_BYTES + w * 256), 4, vSA, kb * a.sa_kb_stride, 0, 0);
      if (w == Cfg::SB_WAVE)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(dSB, GG_LDS_PTR(st + Cfg::A_BYTES + Cfg::B_BYTES + Cfg::SA_BYTES), 4, vSB, kb * 4, 0, 0);
      if constexpr (Cfg::A_SLABS % NW != 0) {
        if (w < Cfg::A_SLABS % NW)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(dA, GG_LDS_PTR(st + (w + A_FULL * NW) * 1024), 16, (RAGGED && last && a_tail) ? GG_OOB_OFFSET : vA + A_FULL * (NW * 8) * K, kb * 128, 0, 0);
      }
      if constexpr (Cfg::B_SLABS % NW != 0) {
        if (w < Cfg::B_SLABS % NW)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(dB, GG_LDS_PTR(st + Cfg::A_BYTES + (w + B_FULL * NW) * 1024), 16,
                                                   RAGGED ? ((last && b_tail) ? GG_OOB_OFFSET : vB + B_FULL * (NW * 8) * K) : vB,
                                                   (RAGGED ? 0 : B_FULL * (NW * 8) * K) + kb * 128, 0, kBAux);
      }
    };
    auto dma_all = [&](int kb, int stg) {
      dma_head(kb, stg);
      static_for<0, NDMA_ALL>([&](auto ic) { dma_tile(ic, kb, stg); });
    };

    v4f acc[TM][TN];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[mt][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    auto read_b = [&](int j, const uint8_t* st) -> v8i {
      const int o = (32 * (j >> 1) + 4 * (j & 1)) * 128;
      const v4i lo = *(const v4i*)(st + bRd0 + o);
      const v4i hi = *(const v4i*)(st + bRd1 + o);
      return (v8i){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };
    auto read_a = [&](int mt, const uint8_t* st) -> v8i {
      const v4i lo = *(const v4i*)(st + aRd0 + mt * 2048);
      const v4i hi = *(const v4i*)(st + aRd1 + mt * 2048);
      return (v8i){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };

    if constexpr (Cfg::XPF) {
      // ======== ring of >= 3 buffers: no barrier at the K-block boundary ==================================
      // The barrier that publishes block kb+1 sits in the MIDDLE of the MFMA stream of block kb, and the
      // operand registers of block kb+1 are refilled during the last activation block of block kb, each
      // right after its last use.  A wave that waits at the barrier has its MFMAs in flight and the other
      // wave of its SIMD keeps issuing, so the matrix pipe does not drain at block boundaries.
      //   WAR: the DMA of block kb+STAGES-1 is issued after the mid barrier of block kb, when every wave has
      //        finished its reads of block kb-1, whose buffer it refills.
      //   RAW: block kb+1 was DMA'd at least one block earlier; every wave waits for its own DMAs before the
      //        mid barrier of block kb, and block kb+1 is first read after it.
      constexpr int HALF = TN;                                           // MFMAs before the mid barrier
      constexpr int NDMA_X = NDMA_ALL < Cfg::MFMAS - HALF ? NDMA_ALL : Cfg::MFMAS - HALF;   // DMAs inside the stream
      constexpr int GAP_X = (Cfg::MFMAS - HALF) / (NDMA_X > 0 ? NDMA_X : 1);
      static_assert(TM % 2 == 0 && TM >= 2, "operand double buffer needs an even number of activation blocks");

#pragma unroll
      for (int s = 0; s < STAGES - 1; ++s)
        if (s < KB) dma_all(s, s);
      wait_vmcnt<0>();                 // first block landed (and the previous tile's stores are done)
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      v8i bfr[TN], afr[2];
      float sa_c, sb_c;
      {
        const uint8_t* st = lds;
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[j] = read_b(j, st);
        afr[0] = read_a(0, st);
        sa_c = *(const float*)(st + saRd);
        sb_c = *(const float*)(st + sbRd);
      }

      stage = 0;
      auto kstep_x = [&](int kb, auto issue_c, auto last_c) {
        constexpr bool ISSUE = decltype(issue_c)::value, LAST = decltype(last_c)::value;
        const int stage1 = stage + 1 == STAGES ? 0 : stage + 1;                   // buffer of block kb+1
        const int stageN = stage == 0 ? STAGES - 1 : stage - 1;                   // buffer of block kb+STAGES-1
        const uint8_t* st = lds + stage * Cfg::STAGE_BYTES;
        const uint8_t* st1 = lds + stage1 * Cfg::STAGE_BYTES;
        float s[TM];
        s[0] = sa_c * sb_c;
        float sa_n = 0.f, sb_n = 0.f;
        v4f p[Cfg::MFMAS];

        auto body = [&](auto tc) {
          constexpr int t = decltype(tc)::value;
          if constexpr (t < Cfg::MFMAS) {
            constexpr int mt = t / TN, j = t % TN;
            if constexpr (j == 0 && mt + 1 < TM) {
              afr[(mt + 1) & 1] = read_a(mt + 1, st);
              s[mt + 1] = *(const float*)(st + saRd + (mt + 1) * 64) * sb_c;
            }
            if constexpr (j == 0 && mt + 1 == TM && !LAST) {
              afr[0] = read_a(0, st1);                      // TM is even: slot 0 is free during the last block
              sa_n = *(const float*)(st1 + saRd);
              sb_n = *(const float*)(st1 + sbRd);
            }
            p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[j], afr[mt & 1], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
            if constexpr (mt + 1 == TM && !LAST) bfr[j] = read_b(j, st1);   // last use of bfr[j] was the MFMA above
            if constexpr (ISSUE && t >= HALF && NDMA_X > 0 && (t - HALF + 1) % GAP_X == 0 && (t - HALF + 1) / GAP_X <= NDMA_X)
              dma_tile(std::integral_constant<int, (t - HALF + 1) / GAP_X - 1>{}, kb + STAGES - 1, stageN);
          }
          if constexpr (t >= Cfg::PIPE) {
            constexpr int u = t - Cfg::PIPE;
            acc[u / TN][u % TN] += p[u] * s[u / TN];
          }
        };
        auto order = [&](auto tc) {      // the issue order of the instructions `body` creates for step t
          constexpr int t = decltype(tc)::value;
          if constexpr (t < Cfg::MFMAS) {
            constexpr int mt = t / TN, j = t % TN;
            if constexpr (j == 0 && mt + 1 < TM) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
            if constexpr (j == 0 && mt + 1 == TM && !LAST) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if constexpr (mt + 1 == TM && !LAST) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            if constexpr (ISSUE && t >= HALF && NDMA_X > 0 && (t - HALF + 1) % GAP_X == 0 && (t - HALF + 1) / GAP_X <= NDMA_X)
              __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            if constexpr (j == 1 || (TN == 1)) __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);   // the scale product of the next block
          }
          if constexpr (t >= Cfg::PIPE) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        };

        static_for<0, HALF>(body);
        static_for<0, HALF>(order);
        // ---- mid barrier: block kb+1 becomes readable, the buffer of block kb-1 becomes writable ----------
        {
          int younger = KB - 2 - kb;
          younger = younger < STAGES - 3 ? younger : STAGES - 3;
          if (younger < 0) younger = 0;
          wait_all_but<NDMA_ALL, STAGES - 3>(younger, dma_extra);
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if constexpr (ISSUE) {
          dma_head(kb + STAGES - 1, stageN);
          static_for<NDMA_X, NDMA_ALL>([&](auto ic) { dma_tile(ic, kb + STAGES - 1, stageN); });
        }
        __builtin_amdgcn_sched_barrier(0);
        static_for<HALF, Cfg::MFMAS + Cfg::PIPE>(body);
        static_for<HALF, Cfg::MFMAS + Cfg::PIPE>(order);
        __builtin_amdgcn_sched_barrier(0);
        sa_c = sa_n;
        sb_c = sb_n;
        stage = stage1;
      };

      const int kb_issue_end = KB - (STAGES - 1) > 0 ? KB - (STAGES - 1) : 0;
      int kb = 0;
      for (; kb < kb_issue_end; ++kb) kstep_x(kb, std::true_type{}, std::false_type{});
      for (; kb < KB - 1; ++kb) kstep_x(kb, std::false_type{}, std::false_type{});
      kstep_x(kb, std::false_type{}, std::true_type{});
      nxt = find_tile(it + 1);
      has_next = nxt.valid;
    } else {
      // ======== ring of 2 buffers (or odd TM): one barrier per K block, at the block boundary ============
      if (!primed) {
        int sp = stage;
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s) {
          if (s < KBu) dma_all(s, sp);
          sp = sp + 1 == STAGES ? 0 : sp + 1;
        }
      }

      // FMAs of the last PIPE MFMAs of a K block are carried into the next block's stream (their
      // accumulators are fixed at compile time), so the matrix pipe does not wait for a VALU tail
      // before the barrier.  Flushed after the last block.
      constexpr int PIPE = Cfg::PIPE, MF = Cfg::MFMAS;
      v4f pend[PIPE];
      float s_pend[PIPE];
#pragma unroll
      for (int i = 0; i < PIPE; ++i) { pend[i] = (v4f){0.f, 0.f, 0.f, 0.f}; s_pend[i] = 0.f; }

      // One K block.  MODE 1: the DMA of block kb + STAGES - 1 is issued during this block; MODE 2: this tile has
      // no such block any more and the DMA of block kb + STAGES - 1 - KB of the next tile is issued instead (through
      // views of length zero when there is no next tile to fetch for: every K block issues the same fetches).
      auto kstep = [&](int kb, auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;
        constexpr bool ISSUE = true;
        int kb_new = MODE == 2 ? kb + STAGES - 1 - KBu : kb + STAGES - 1;
        if (MODE == 2 && kb_new >= KBu) kb_new = KBu - 1;      // fewer K blocks than ring buffers: dropped anyway
        const int nstage = stage == 0 ? STAGES - 1 : stage - 1;
        // The DMA of this K block (issued STAGES-1 blocks ago by every wave) must have landed; the newer
        // blocks (of this tile, then of the next) may stay in flight.  Loads complete in order, but stores do not
        // order with loads, so the first block of a tile drains everything (the previous tile's epilogue stores too).
        {
          // every K block issues one group of fetches, so STAGES-2 groups are younger than block kb (KB-1 if the
          // tile has fewer K blocks than the ring has buffers)
          int younger = KBu - 1 < STAGES - 2 ? KBu - 1 : STAGES - 2;
          if (kb == 0) younger = 0;
          wait_all_but<NDMA_ALL, STAGES - 2>(younger, dma_extra);
        }
        // ... in every wave, and every wave must be done with the buffer that is refilled next.  A bare
        // s_barrier: __syncthreads() would add a fence that drains every DMA in flight (vmcnt(0)) and
        // with it the whole point of the ring.  Visibility is by construction: each wave has waited for
        // its own DMAs above, and its LDS reads of the previous block were consumed by MFMAs already.
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");   // no LDS access may be moved above the barrier by the compiler

        // Operand reads in the order the MFMAs need them; nothing here waits, so the first MFMA can go
        // as soon as its two operands are back while the rest is still in flight.
        const uint8_t* st = lds + stage * Cfg::STAGE_BYTES;
        v8i bfr[TN], afr[2];
        bfr[0] = read_b(0, st);
        afr[0] = read_a(0, st);
        const float sb = *(const float*)(st + sbRd);
        float sa[TM];
        sa[0] = *(const float*)(st + saRd);
#pragma unroll
        for (int j = 1; j < TN; ++j) bfr[j] = read_b(j, st);
#pragma unroll
        for (int mt = 1; mt < TM; ++mt) sa[mt] = *(const float*)(st + saRd + mt * 64);
        if constexpr (ISSUE) {
          dma_head(kb_new, nstage);
          static_for<NDMA_STREAM, NDMA_ALL>([&](auto ic) { dma_tile(ic, kb_new, nstage); });
        }
        __builtin_amdgcn_sched_barrier(0);   // the reads above keep their order; the stream below is ordered by hand

        // software pipeline: MFMA t is issued PIPE steps before the 4 FMAs that consume it, the operand
        // reads of the next activation block are issued one block ahead, one DMA every DMA_GAP MFMAs
        v4f p[MF];
        float s[TM];
        static_for<0, MF>([&](auto tc) {
          constexpr int t = decltype(tc)::value;
          constexpr int mt = t / TN, j = t % TN;
          if constexpr (j == 0) s[mt] = sa[mt] * sb;
          if constexpr (j == 0 && mt + 1 < TM) afr[(mt + 1) & 1] = read_a(mt + 1, st);
          p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[j], afr[mt & 1], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
          if constexpr (ISSUE && NDMA_STREAM > 0 && (t + 1) % DMA_GAP == 0 && (t + 1) / DMA_GAP <= NDMA_STREAM)
            dma_tile(std::integral_constant<int, (t + 1) / DMA_GAP - 1>{}, kb_new, nstage);
          if constexpr (t < PIPE) {
            constexpr int u = MF - PIPE + t;                 // carried over from the previous K block
            acc[u / TN][u % TN] += pend[t] * s_pend[t];
          } else {
            constexpr int u = t - PIPE;
            acc[u / TN][u % TN] += p[u] * s[u / TN];
          }
        });
        static_for<0, MF>([&](auto tc) {
          constexpr int t = decltype(tc)::value;
          if constexpr (t % TN == 0) __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);                       // scale product
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                 // 1 MFMA
          if constexpr (t % TN == 0 && t / TN + 1 < TM) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // 2 DS reads
          if constexpr (ISSUE && NDMA_STREAM > 0 && (t + 1) % DMA_GAP == 0 && (t + 1) / DMA_GAP <= NDMA_STREAM)
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                               // 1 DMA
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                                 // 4 FMAs
        });
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < PIPE; ++i) { pend[i] = p[MF - PIPE + i]; s_pend[i] = s[(MF - PIPE + i) / TN]; }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
      };

      const int kb_issue_end = KBu - (STAGES - 1) > 0 ? KBu - (STAGES - 1) : 0;
      int kb = 0;
      for (; kb < kb_issue_end; ++kb) kstep(kb, std::integral_constant<int, 1>{});
      // this tile has issued its last fetch: from here on the descriptors are the next tile's
      nxt = find_tile(it + 1);
      has_next = nxt.valid;
      prefetch = has_next && xt;
      dA = desc_a(nxt, prefetch); dSA = desc_sa(nxt, prefetch); dB = desc_b(nxt, prefetch); dSB = desc_sb(nxt, prefetch);
      rot = k_start(nxt);
      for (; kb < KBu; ++kb) kstep(kb, std::integral_constant<int, 2>{});
      static_for<0, PIPE>([&](auto ic) {
        constexpr int u = MF - PIPE + decltype(ic)::value;
        acc[u / TN][u % TN] += pend[decltype(ic)::value] * s_pend[decltype(ic)::value];
      });
    }
    // every wave is done reading LDS before the next tile's prologue overwrites it; with the next tile's first
    // blocks already in flight there is no prologue, and the barrier of its first K block does the same job
    if (!prefetch) __syncthreads();

    if constexpr (SPLITK) {
      // ---- epilogue of a K half: the fp32 sums as they are, through a view bounded like the one of C -----------
      __amdgpu_buffer_rsrc_t dP = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(a.P + ((int64_t)cur.ks * a.M_total + cur.grow) * N + n0), 0, (rows_valid * N - n0) * 4, GG_RSRC_FLAGS);
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        const int row = wm * WTM + 16 * mt + r;
#pragma unroll
        for (int pr = 0; pr < TN / 2; ++pr) {
          const int col = wn * WTN + 32 * pr + 8 * q;
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, acc[mt][2 * pr]), dP, (row * N + col) * 4, 0, 0);
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, acc[mt][2 * pr + 1]), dP, (row * N + col + 4) * 4, 0, 0);
        }
      }
    } else {
    // ---- epilogue: bf16 (or binary16) RNE, 16-byte bounded stores ---------------------------------------------
    // Lane (q, r) holds 16 bytes of row r; stored from there, neighbouring lanes would write to different rows and
    // every lane's piece would be a request of its own.  Lane 4 r + q takes them instead (a transpose of the lane
    // grid through the LDS crossbar), so that four neighbouring lanes write 64 consecutive bytes of a row.
    const int cSrc = (16 * (l & 3) + (l >> 2)) * 4;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const int row = wm * WTM + 16 * mt + (l >> 2);
#pragma unroll
      for (int pr = 0; pr < TN / 2; ++pr) {
        const v4f x = acc[mt][2 * pr], y = acc[mt][2 * pr + 1];
        const bool f16 = a.out_f16 != 0;
        v4i out;
        out.x = pack2_rne(x[0], x[1], f16);
        out.y = pack2_rne(x[2], x[3], f16);
        out.z = pack2_rne(y[0], y[1], f16);
        out.w = pack2_rne(y[2], y[3], f16);
        out.x = __builtin_amdgcn_ds_bpermute(cSrc, out.x);
        out.y = __builtin_amdgcn_ds_bpermute(cSrc, out.y);
        out.z = __builtin_amdgcn_ds_bpermute(cSrc, out.z);
        out.w = __builtin_amdgcn_ds_bpermute(cSrc, out.w);
        const int col = wn * WTN + 32 * pr + 8 * (l & 3);     // 8 columns; N is a multiple of 8, so they exist together or not at all
        // streaming cache policy (nt sc1): C is written once and not read here; left to the default policy it takes
        // room in the L2 from the weights that the row tiles of a group share (2.6 % on 256 groups of ~128 rows)
        __builtin_amdgcn_raw_buffer_store_b128(out, dC, (!RAGGED || col < n_rem) ? row * N * 2 + col * 2 : GG_OOB_OFFSET, 0, 2 | 16);
      }
    }
    }
    if (!has_next) {
      wait_vmcnt<0>();     // the dropped fetches of the last K blocks still write zeros into this workgroup's LDS
      return;
    }
    if (!prefetch) {
      dA = desc_a(nxt, true); dSA = desc_sa(nxt, true); dB = desc_b(nxt, true); dSB = desc_sb(nxt, true);
      rot = k_start(nxt);
    }
    cur = nxt;
    primed = prefetch;
  }
}

// Second pass of the split-K path: C[r][n] = round(P[0][r][n] + P[1][r][n]) for the rows of the groups, i.e. rows
// [off[0], off[G]) clamped to [0, M_total).  One thread per 8 columns; the sum of the two halves in a fixed order,
// so the result does not depend on how the first pass was scheduled.
__global__ void __launch_bounds__(256) gg_splitk_combine_kernel(const float* __restrict__ P, const int32_t* __restrict__ off,
                                                                 uint16_t* __restrict__ C, int G, int M_total, int N, int out_f16) {
  const int row_lo = clampi(off[0], 0, M_total), row_hi = clampi(off[G], row_lo, M_total);
  const int64_t groups8 = (int64_t)(row_hi - row_lo) * (N >> 3);
  const int64_t half = (int64_t)M_total * N;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < groups8; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t e = (int64_t)row_lo * N + i * 8;
    const v4f a0 = *(const v4f*)(P + e), a1 = *(const v4f*)(P + e + 4);
    const v4f b0 = *(const v4f*)(P + half + e), b1 = *(const v4f*)(P + half + e + 4);
    const v4f x = a0 + b0, y = a1 + b1;
    v4i out;
    out.x = pack2_rne(x[0], x[1], out_f16 != 0);
    out.y = pack2_rne(x[2], x[3], out_f16 != 0);
    out.z = pack2_rne(y[0], y[1], out_f16 != 0);
    out.w = pack2_rne(y[2], y[3], out_f16 != 0);
    *(v4i*)(C + e) = out;
  }
}

}  // namespace gg
