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
//    scalar  s = SA[row][kb] * SB[g][n/128][kb]  into the fp32 accumulators (a5 of the hot path);
//  * the epilogue rounds to bf16 (RNE) and issues bounded 16-byte stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gg {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

#define GG_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
// dword 3 of a raw buffer descriptor on gfx9-family parts: 32-bit data format, no swizzle
#define GG_RSRC_FLAGS 0x00020000

struct GemmArgs {
  const uint8_t* A;
  const float* SA;
  const uint8_t* B;
  const float* SB;
  const int32_t* off;
  uint16_t* C;
  int G;
  int M_total;   // rows of A / C (clamp for untrusted offsets)
  int N, K, KB;  // KB = K / 128
  int n_tiles;   // N / BN
  int n_chunk;   // n-tiles that are walked together before moving to the next m-tile
  int slots;     // workgroups per XCD when the grid is a multiple of 8, else 0 (plain round-robin)
};

template <int BM_, int BN_, int WM_, int WN_, int STAGES_>
struct GemmCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, STAGES = STAGES_;
  static constexpr int NW = WM * WN;          // waves per workgroup
  static constexpr int NT = 64 * NW;          // threads per workgroup
  static constexpr int WTM = BM / WM;         // rows of A per wave
  static constexpr int WTN = BN / WN;         // columns per wave
  static constexpr int TM = WTM / 16;         // MFMA column blocks (activation rows) per wave
  static constexpr int TN = WTN / 16;         // MFMA row blocks (weight rows) per wave
  static constexpr int A_BYTES = BM * 128;
  static constexpr int B_BYTES = BN * 128;
  static constexpr int SA_ROWS = BM < 64 ? 64 : BM;
  static constexpr int SA_BYTES = SA_ROWS * 4;
  static constexpr int SB_BYTES = 256;         // BN/128 scales of B per K block, replicated over one wave-wide DMA
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES + SA_BYTES + SB_BYTES;
  static constexpr int SB_WAVE = NW - 1;      // the wave that fetches them
  static constexpr int MFMAS = (BM / WM / 16) * (BN / WN / 16);   // MFMAs per wave per K block
  static constexpr int PIPE = MFMAS < 3 ? MFMAS : 3;               // MFMAs in flight before their FMAs are issued
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
  static constexpr int A_SLABS = BM / 8;      // one slab = 8 rows x 128 B = one wave-wide DMA
  static constexpr int B_SLABS = BN / 8;
  static constexpr int A_ITERS = (A_SLABS + NW - 1) / NW;
  static constexpr int B_ITERS = (B_SLABS + NW - 1) / NW;
  static constexpr int SA_WAVES = SA_ROWS / 64;
  static_assert(BM % (16 * WM) == 0 && BN % (32 * WN) == 0, "wave tile must be 16 x 32 granular");
  static_assert(WTN <= 128 && 128 % WTN == 0, "a wave must stay inside one 128-wide scale block of B");
  static_assert(BM % 8 == 0 && BN % 8 == 0 && NW % 4 == 0, "slab mapping");
  static_assert(TN % 2 == 0, "n sub-tiles are paired for 16-byte stores");
};

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gg_gemm_kernel(const GemmArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, WN = Cfg::WN, NW = Cfg::NW;
  constexpr int TM = Cfg::TM, TN = Cfg::TN, WTM = Cfg::WTM, WTN = Cfg::WTN, STAGES = Cfg::STAGES;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l = tid & 63;
  const int r = l & 15, q = l >> 4;
  const int wm = w / WN, wn = w % WN;
  const int K = a.K, KB = a.KB, N = a.N;

  // ---- per-lane constants of the global -> LDS DMA -------------------------------------------
  // lane l of a wave-wide 16 B DMA lands at LDS byte 16*l of the slab: row l/8, physical chunk l%8.
  // The logical chunk it must fetch is physical ^ key(row).
  const int lrow = l >> 3, pch = l & 7;
  const int a_row = w * 8 + lrow;                                   // + i*NW*8
  const int keyA_ld = ((a_row >> 1) & 7);
  const int b_row = w * 8 + lrow;
  const int keyB_ld = ((b_row >> 1) & 1) | (((b_row >> 3) & 3) << 1);
  const int vA = a_row * K + ((pch ^ keyA_ld) << 4);
  const int vB = b_row * K + ((pch ^ keyB_ld) << 4);
  const int vSA = (w * 64 + l) * KB * 4;
  const int vSB = (l < BN / 128 ? l : BN / 128 - 1) * KB * 4;        // lane -> which 128-wide N block of the tile

  // ---- per-lane constants of the LDS operand reads --------------------------------------------
  const int keyA_rd = (r >> 1) & 7;
  const int rowB_rd = 8 * (r >> 2) + (r & 3);
  const int keyB_rd = ((r >> 1) & 1) | ((r >> 2) << 1);
  const int aRd0 = (wm * WTM + r) * 128 + (((2 * q) ^ keyA_rd) << 4);
  const int aRd1 = (wm * WTM + r) * 128 + (((2 * q + 1) ^ keyA_rd) << 4);
  const int bRd0 = Cfg::A_BYTES + (wn * WTN + rowB_rd) * 128 + (((2 * q) ^ keyB_rd) << 4);
  const int bRd1 = Cfg::A_BYTES + (wn * WTN + rowB_rd) * 128 + (((2 * q + 1) ^ keyB_rd) << 4);
  const int saRd = Cfg::A_BYTES + Cfg::B_BYTES + (wm * WTM + r) * 4;
  const int sbRd = Cfg::A_BYTES + Cfg::B_BYTES + Cfg::SA_BYTES + ((wn * WTN) >> 7) * 4;

  // ---- persistent walk over the tile list ---------------------------------------------------------
  int g = 0, base = 0;
  const int nwg = gridDim.x;
  for (int it = 0;; ++it) {
    int T;
    if (a.slots > 0) T = (it * 8 + (int)(blockIdx.x & 7)) * a.slots + (int)(blockIdx.x >> 3);
    else T = it * nwg + blockIdx.x;

    int row0 = 0, Mg = 0, mtiles = 0;
    for (;;) {
      if (g >= a.G) return;
      row0 = clampi(a.off[g], 0, a.M_total);
      const int row1 = clampi(a.off[g + 1], row0, a.M_total);
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
    const int n0 = ntile * BN;
    int rows_valid = Mg - m0;
    rows_valid = rows_valid < BM ? rows_valid : BM;
    const int64_t grow = (int64_t)row0 + m0;

    // bounded views: nothing past the last valid row of this tile is loaded or stored
    __amdgpu_buffer_rsrc_t dA = __builtin_amdgcn_make_buffer_rsrc((void*)(a.A + grow * K), 0, rows_valid * K, GG_RSRC_FLAGS);
    __amdgpu_buffer_rsrc_t dSA = __builtin_amdgcn_make_buffer_rsrc((void*)(a.SA + grow * KB), 0, rows_valid * KB * 4, GG_RSRC_FLAGS);
    __amdgpu_buffer_rsrc_t dB = __builtin_amdgcn_make_buffer_rsrc((void*)(a.B + ((int64_t)g * N + n0) * K), 0, BN * K, GG_RSRC_FLAGS);
    __amdgpu_buffer_rsrc_t dC = __builtin_amdgcn_make_buffer_rsrc((void*)(a.C + grow * N + n0), 0, rows_valid * N * 2 - n0 * 2, GG_RSRC_FLAGS);
    __amdgpu_buffer_rsrc_t dSB = __builtin_amdgcn_make_buffer_rsrc((void*)(a.SB + ((int64_t)g * (N >> 7) + (n0 >> 7)) * KB), 0, (BN / 128) * KB * 4, GG_RSRC_FLAGS);

    auto issue_loads = [&](int kb, int stage) {
      uint8_t* st = lds + stage * Cfg::STAGE_BYTES;
#pragma unroll
      for (int i = 0; i < Cfg::A_ITERS; ++i) {
        const int sl = w + i * NW;
        if (Cfg::A_SLABS % NW == 0 || sl < Cfg::A_SLABS)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(dA, GG_LDS_PTR(st + sl * 1024), 16, vA + i * (NW * 8) * K, kb * 128, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < Cfg::B_ITERS; ++i) {
        const int sl = w + i * NW;
        if (Cfg::B_SLABS % NW == 0 || sl < Cfg::B_SLABS)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(dB, GG_LDS_PTR(st + Cfg::A_BYTES + sl * 1024), 16, vB, i * (NW * 8) * K + kb * 128, 0, 0);
      }
      if (w < Cfg::SA_WAVES)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(dSA, GG_LDS_PTR(st + Cfg::A_BYTES + Cfg::B_BYTES + w * 256), 4, vSA, kb * 4, 0, 0);
      if (w == Cfg::SB_WAVE)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(dSB, GG_LDS_PTR(st + Cfg::A_BYTES + Cfg::B_BYTES + Cfg::SA_BYTES), 4, vSB, kb * 4, 0, 0);
    };

    v4f acc[TM][TN];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[mt][j] = (v4f){0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
      if (s < KB) issue_loads(s, s);
    for (int kb = 0; kb < KB; ++kb) {
      const int stage = kb % STAGES;
      // the DMA of this K block (issued STAGES-1 iterations ago by every wave) must have landed ...
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      // ... in every wave, and every wave must be done with the buffer that is refilled next
      __syncthreads();
      if (kb + STAGES - 1 < KB) issue_loads(kb + STAGES - 1, (kb + STAGES - 1) % STAGES);

      const uint8_t* st = lds + stage * Cfg::STAGE_BYTES;
      const float sb = *(const float*)(st + sbRd);
      v8i bfr[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int o = (32 * (j >> 1) + 4 * (j & 1)) * 128;
        const v4i lo = *(const v4i*)(st + bRd0 + o);
        const v4i hi = *(const v4i*)(st + bRd1 + o);
        bfr[j] = (v8i){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      }
      float s[TM];
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) s[mt] = *(const float*)(st + saRd + mt * 64) * sb;

      // software pipeline: MFMA t is issued PIPE steps before the 4 FMAs that consume it, and the
      // operand reads of the next activation block are issued one block ahead
      v8i afr[2];
      {
        const v4i lo = *(const v4i*)(st + aRd0);
        const v4i hi = *(const v4i*)(st + aRd1);
        afr[0] = (v8i){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      }
      v4f p[Cfg::MFMAS];
#pragma unroll
      for (int t = 0; t < Cfg::MFMAS + Cfg::PIPE; ++t) {
        if (t < Cfg::MFMAS) {
          const int mt = t / TN, j = t % TN;
          if (j == 0 && mt + 1 < TM) {
            const v4i lo = *(const v4i*)(st + aRd0 + (mt + 1) * 2048);
            const v4i hi = *(const v4i*)(st + aRd1 + (mt + 1) * 2048);
            afr[(mt + 1) & 1] = (v8i){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          }
          p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[j], afr[mt & 1], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
        }
        if (t >= Cfg::PIPE) {
          const int u = t - Cfg::PIPE;
          acc[u / TN][u % TN] += p[u] * s[u / TN];
        }
      }
#pragma unroll
      for (int t = 0; t < Cfg::MFMAS + Cfg::PIPE; ++t) {
        if (t < Cfg::MFMAS) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // 1 MFMA
          if (t % TN == 0 && t / TN + 1 < TM) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // 2 DS reads
        }
        if (t >= Cfg::PIPE) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);    // 4 VALU
      }
    }
    __syncthreads();  // every wave is done reading LDS before the next tile's prologue overwrites it

    // ---- epilogue: bf16 RNE, 16-byte bounded stores ---------------------------------------------
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const int row = wm * WTM + 16 * mt + r;
#pragma unroll
      for (int pr = 0; pr < TN / 2; ++pr) {
        const v4f x = acc[mt][2 * pr], y = acc[mt][2 * pr + 1];
        const v2bf c0 = __builtin_convertvector((v2f){x[0], x[1]}, v2bf);
        const v2bf c1 = __builtin_convertvector((v2f){x[2], x[3]}, v2bf);
        const v2bf c2 = __builtin_convertvector((v2f){y[0], y[1]}, v2bf);
        const v2bf c3 = __builtin_convertvector((v2f){y[2], y[3]}, v2bf);
        v4i out;
        out.x = __builtin_bit_cast(int, c0);
        out.y = __builtin_bit_cast(int, c1);
        out.z = __builtin_bit_cast(int, c2);
        out.w = __builtin_bit_cast(int, c3);
        const int col = wn * WTN + 32 * pr + 8 * q;
        __builtin_amdgcn_raw_buffer_store_b128(out, dC, row * N * 2 + col * 2, 0, 0);
      }
    }
  }
}

}  // namespace gg
