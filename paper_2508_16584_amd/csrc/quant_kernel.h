// The step in front of the grouped GEMM: bf16 rows -> e4m3 bytes + one fp32 scale per 1x128 block (the scaling
// of A stated below Table 1 of the paper), gathered straight into group-contiguous order.  With the
// padding-free GEMM this kernel runs on the valid rows only; nothing is padded and nothing is copied again.
//
// Per output row r and K block kb, in fp32:
//     amax  = max( max |x| over the 128 values with NaNs skipped, 2^-100 )
//     scale = amax / 448                                       (a dequantisation multiplier)
//     byte  = e4m3( clamp(x * (448 / amax), -448, 448) )       round to nearest even; NaN -> 0x7F
// The two divisions per block, the product and the conversion are the hardware's correctly rounded ones, so the
// bytes and scales are reproducible bit for bit on the host.
//
// Mapping: 16 lanes (one DPP row) own one block: a lane loads 8 bf16 (16 B), the row reduces amax with four
// row rotations, a lane stores 8 bytes.  A workgroup of 256 threads takes 32 blocks of one row per pass, both
// loads of a lane issued before any arithmetic; rows are strided over the grid.  HBM-bound: 2K bytes in,
// K + K/32 out per row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gg {

constexpr int Q_THREADS = 256;

typedef int q_v4i __attribute__((ext_vector_type(4)));
typedef int q_v2i __attribute__((ext_vector_type(2)));

// max over the 16 lanes of a DPP row, result in every lane
__device__ __forceinline__ unsigned row16_max(unsigned v) {
#define GG_ROR(x, n) ((unsigned)__builtin_amdgcn_update_dpp(0, (int)(x), 0x120 + (n), 0xF, 0xF, false))
  unsigned t;
  t = GG_ROR(v, 8); v = v > t ? v : t;
  t = GG_ROR(v, 4); v = v > t ? v : t;
  t = GG_ROR(v, 2); v = v > t ? v : t;
  t = GG_ROR(v, 1); v = v > t ? v : t;
#undef GG_ROR
  return v;
}

__device__ __forceinline__ void quantize_block(const q_v4i raw, uint8_t* dst, float* dst_scale, int sub) {
  float v[8];
  unsigned u[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __builtin_bit_cast(float, raw[i] << 16);
    v[2 * i + 1] = __builtin_bit_cast(float, raw[i] & (int)0xFFFF0000);
  }
  // |x| of non-NaN floats orders like its bit pattern
  unsigned top = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    u[i] = __builtin_bit_cast(unsigned, v[i]) & 0x7FFFFFFFu;
    top = top > u[i] ? top : u[i];
  }
  // NaNs and infinities are rare: one wave-uniform branch keeps their handling out of the common path
  const bool special = __builtin_amdgcn_ballot_w64(top >= 0x7F800000u) != 0;
  if (special) {
    top = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const unsigned t = u[i] > 0x7F800000u ? 0u : u[i];     // a NaN (quiet or signalling) counts as zero
      top = top > t ? top : t;
    }
  }
  top = row16_max(top);
  top = top > 0x0D800000u ? top : 0x0D800000u;               // floor 2^-100: 448 / amax stays finite
  const float amax = __builtin_bit_cast(float, top);
  const float scale = amax / 448.0f;
  const float inv = 448.0f / amax;
  int lo = 0, hi = 0;
  if (!special) {
    float y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] = __builtin_amdgcn_fmed3f(v[i] * inv, -448.0f, 448.0f);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
  } else {
    float y[8];
    unsigned nan_lo = 0, nan_hi = 0;                         // 0x7F in the byte of every NaN, whatever its sign or payload
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float t = v[i] * inv;
      const bool is_nan = t != t;
      y[i] = is_nan ? 0.f : __builtin_fminf(__builtin_fmaxf(t, -448.0f), 448.0f);
      if (i < 4) nan_lo |= is_nan ? (0x7Fu << (8 * i)) : 0u;
      else nan_hi |= is_nan ? (0x7Fu << (8 * (i - 4))) : 0u;
    }
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
    lo |= (int)nan_lo;
    hi |= (int)nan_hi;
  }
  *(q_v2i*)dst = (q_v2i){lo, hi};
  if (sub == 0) *dst_scale = scale;
}

// A workgroup works on two adjacent rows at a time.  Pair t of workgroup b (t = 0, 1, ...):
//   by_xcd = 0: pair number b + t * grid (pairs dealt out round-robin);
//   by_xcd = 1 (grid a multiple of 8): the eight rows of a "sector" (8 adjacent rows: with K-block-major scales their
//     eight 4-byte scale stores of one K block make up one 32-byte piece of memory) go to four workgroups in
//     neighbouring slots of ONE XCD (workgroup b runs on XCD b % 8), which run at the same time, so the pieces leave
//     that XCD's L2 as whole writes.  Dealt out round-robin they come from four XCDs, and each L2 writes a masked
//     32-byte piece for its 8 bytes.
// pair_of() returns the pair number, -1 when the workgroup is done, -2 for a pair to skip.  The 2 * KB blocks of a
// pair are numbered through and
// taken 32 per pass, so that short rows (KB <= 16) still fill both load slots of every lane.
__device__ __forceinline__ int64_t pair_of(int64_t t, int64_t npairs, int by_xcd) {
  const int64_t b = blockIdx.x, grid = gridDim.x;
  if (!by_xcd) {
    const int64_t p = b + t * grid;
    return p < npairs ? p : -1;
  }
  const int64_t u = b / 8 + t * (grid / 8);          // position in this XCD's list of pairs: 4 per sector
  const int64_t sector = (u / 4) * 8 + b % 8;
  const int64_t p = sector * 4 + u % 4;
  if (sector * 4 >= npairs) return -1;               // sectors only grow with t
  return p < npairs ? p : -2;                        // a pair past the end inside the last sector
}

struct RowPairSlot {
  bool valid;     // this 16-lane group has a block in this pass
  int row, blk;
};
__device__ __forceinline__ RowPairSlot row_pair_slot(int v, int KB, int r, int r2, int M_total) {
  const bool second = v >= KB;
  RowPairSlot s;
  s.row = second ? r2 : r;
  s.blk = v - (second ? KB : 0);
  s.valid = v < 2 * KB && s.row < M_total;
  return s;
}

__global__ void __launch_bounds__(Q_THREADS) gg_quantize_rows_kernel(const uint16_t* __restrict__ X,
                                                                     const int32_t* __restrict__ row_src,
                                                                     uint8_t* __restrict__ A, float* __restrict__ SA,
                                                                     int64_t T, int M_total, int K, int KB,
                                                                     int64_t sa_rs, int64_t sa_ks,     // SA[row * sa_rs + blk * sa_ks]
                                                                     int by_xcd) {
  const int grp = threadIdx.x >> 4, sub = threadIdx.x & 15;
  const int64_t npairs = ((int64_t)M_total + 1) / 2;
  for (int64_t t = 0;; ++t) {
    const int64_t pr = pair_of(t, npairs, by_xcd);
    if (pr == -1) break;
    if (pr < 0) continue;
    const int64_t r64 = 2 * pr;
    const int r = (int)r64;
    const int r2 = r64 + 1 < M_total ? (int)(r64 + 1) : M_total;     // M_total = no second row
    const int64_t s1 = row_src ? (int64_t)row_src[r] : (int64_t)r;
    const int64_t s2 = r2 < M_total ? (row_src ? (int64_t)row_src[r2] : (int64_t)r2) : -1;
    for (int v0 = 0; v0 < 2 * KB; v0 += 32) {
      const RowPairSlot a = row_pair_slot(v0 + grp, KB, r, r2, M_total);            // uniform over the 16 lanes of a row
      const RowPairSlot b = row_pair_slot(v0 + 16 + grp, KB, r, r2, M_total);
      const int64_t sa = a.row == r ? s1 : s2, sb = b.row == r ? s1 : s2;
      // a source outside [0, T) stands for a row of zeros
      q_v4i rawA = {0, 0, 0, 0}, rawB = {0, 0, 0, 0};
      if (a.valid && sa >= 0 && sa < T) rawA = *(const q_v4i*)(X + sa * K + a.blk * 128 + sub * 8);
      if (b.valid && sb >= 0 && sb < T) rawB = *(const q_v4i*)(X + sb * K + b.blk * 128 + sub * 8);
      if (a.valid) quantize_block(rawA, A + (int64_t)a.row * K + a.blk * 128 + sub * 8, SA + a.row * sa_rs + a.blk * sa_ks, sub);
      if (b.valid) quantize_block(rawB, A + (int64_t)b.row * K + b.blk * 128 + sub * 8, SA + b.row * sa_rs + b.blk * sa_ks, sub);
    }
  }
}

// The activation between the two grouped GEMMs of an expert MLP, fused with the quantiser above: H [M, 2I] bf16
// (columns [0, I): gate projection, [I, 2I): up projection) ->
//     act = bf16_rne( silu(gate) * up ),  silu(g) = g / (1 + exp(-g))   in fp32
// and then exactly quantize_block on the bf16 bits of act.  act is also written out when act_out is not null.
// Same mapping: 16 lanes own one block of 128 activation columns, a lane loads 8 gate and 8 up values.
// two (gate, up) pairs, each a dword of two bf16 -> one dword of two bf16 activations
__device__ __forceinline__ int swiglu2(const int g_raw, const int u_raw) {
  float g[2] = {__builtin_bit_cast(float, g_raw << 16), __builtin_bit_cast(float, g_raw & (int)0xFFFF0000)};
  float u[2] = {__builtin_bit_cast(float, u_raw << 16), __builtin_bit_cast(float, u_raw & (int)0xFFFF0000)};
  float a[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    // sigmoid through t = exp(-|g|) in [0, 1]: no overflow for any g; the hardware exponential (a few fp32
    // ulps, denormal results flushed: t = 0 below g = -87.3) and the hardware reciprocal (1 ulp; 1 + t lies in
    // [1, 2]) are far inside the bf16 rounding.  A division here compiles to the 10-instruction correctly
    // rounded sequence, which made this kernel bound by vector arithmetic.
    const float t = __expf(-__builtin_fabsf(g[h]));
    const float sig = (g[h] >= 0.f ? 1.0f : t) * __builtin_amdgcn_rcpf(1.0f + t);
    a[h] = g[h] * sig * u[h];
  }
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  const bf2 r = __builtin_convertvector((f2){a[0], a[1]}, bf2);     // round to nearest even
  return __builtin_bit_cast(int, r);
}

__device__ __forceinline__ q_v4i swiglu8(const q_v4i g_raw, const q_v4i u_raw) {
  q_v4i out;
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = swiglu2(g_raw[i], u_raw[i]);
  return out;
}

// The block quantiser's arithmetic for callers that hold a block's values spread over lanes in another way than
// quantize_block's 16 x 8: amax_bits_of() of every value, reduced by the caller with an integer max, then
// block_scale() and e4m3_of().  Same results as quantize_block, bit for bit (its fast path and its NaN/inf path
// agree on ordinary values; this is the general path throughout).
__device__ __forceinline__ unsigned amax_bits_of(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v) & 0x7FFFFFFFu;
  return u > 0x7F800000u ? 0u : u;                             // a NaN counts as zero
}
__device__ __forceinline__ float block_amax(unsigned top) {
  top = top > 0x0D800000u ? top : 0x0D800000u;                 // floor 2^-100
  return __builtin_bit_cast(float, top);
}
// four values -> four e4m3 bytes in a dword (value 0 in the low byte)
__device__ __forceinline__ int e4m3x4_of(const float* v, float inv) {
  float y[4];
  unsigned nan = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float t = v[i] * inv;
    const bool is_nan = t != t;
    y[i] = is_nan ? 0.f : __builtin_fminf(__builtin_fmaxf(t, -448.0f), 448.0f);
    nan |= is_nan ? (0x7Fu << (8 * i)) : 0u;
  }
  int w = 0;
  w = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], w, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], w, true);
  return w | (int)nan;
}

// The producer of the weight-gradient GEMM's operands: the same block quantiser ALONG THE TOKENS, with the transpose
// that GEMM wants.  X [T, K] bf16 (token-major) -> XT [K, M_total] e4m3 (token index contiguous) and SX [MB, K]:
// output token r is input row row_src[r]; feature k's block j holds tokens [128 j, 128 j + 128) of the output order,
// the last block those that exist.  (The paper defines neither this operation nor its layouts.)
// A workgroup takes tiles of one token block x 64 features: 128 rows of 128 bytes go through LDS (every group of 16
// rows shifted by 32 bytes, so that the eight lanes of a feature pair read from different banks); lane 8 f + p then
// owns tokens 16 p .. 16 p + 15 of features 2 f and 2 f + 1 (one 4-byte LDS read per token): amax over its 16 values
// per feature and over the eight lanes, 16 bytes out per feature - the eight lanes of a feature write one 128-byte
// line of XT.
constexpr int QC_FEATS = 64;
constexpr int QC_LDS_BYTES = 128 * 128 + 7 * 32;

__global__ void __launch_bounds__(Q_THREADS) gg_quantize_cols_kernel(const uint16_t* __restrict__ X,
                                                                     const int32_t* __restrict__ row_src,
                                                                     uint8_t* __restrict__ XT, float* __restrict__ SX,
                                                                     int64_t T, int M_total, int K, int MB) {
  __shared__ __attribute__((aligned(16))) uint8_t tile[QC_LDS_BYTES];
  const int t = threadIdx.x;
  const int kt = K / QC_FEATS;
  const int64_t tiles = (int64_t)MB * kt;
  const int fp = t >> 3, part = t & 7;
  // piece t + 256 i of a tile: token (t + 256 i) / 8 of the block, features 8 (t % 8) .. + 7
  q_v4i raw[4];
  auto load_tile = [&](int64_t id) __attribute__((always_inline)) {
    const int j = (int)(id / kt), k0 = (int)(id - (int64_t)j * kt) * QC_FEATS;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 128 * j + ((t + 256 * i) >> 3);
      raw[i] = (q_v4i){0, 0, 0, 0};                        // a token past the end or a source outside [0, T): zeros
      if (r < M_total) {
        const int64_t src = row_src ? (int64_t)row_src[r] : (int64_t)r;
        if (src >= 0 && src < T) raw[i] = *(const q_v4i*)(X + src * K + k0 + 8 * (t & 7));
      }
    }
  };
  if ((int64_t)blockIdx.x < tiles) load_tile(blockIdx.x);
  for (int64_t id = blockIdx.x; id < tiles; id += gridDim.x) {
    const int j = (int)(id / kt), k0 = (int)(id - (int64_t)j * kt) * QC_FEATS;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tok = (t + 256 * i) >> 3;
      *(q_v4i*)(tile + tok * 128 + (tok >> 4) * 32 + 16 * (t & 7)) = raw[i];
    }
    __syncthreads();
    if (id + gridDim.x < tiles) load_tile(id + gridDim.x);      // the next tile's rows are on their way during this one's arithmetic
    float v[2][16];
    unsigned top[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const unsigned two = *(const unsigned*)(tile + (16 * part + i) * 128 + part * 32 + 4 * fp);
      v[0][i] = __builtin_bit_cast(float, two << 16);
      v[1][i] = __builtin_bit_cast(float, two & 0xFFFF0000u);
      const unsigned a0 = two & 0x7FFFu, a1 = (two >> 16) & 0x7FFFu;      // |x| of non-NaN values orders like its bit pattern
      top[0] = top[0] > a0 ? top[0] : a0;
      top[1] = top[1] > a1 ? top[1] : a1;
    }
    // NaNs and infinities are rare: one wave-uniform branch keeps their handling out of the common path
    const bool special = __builtin_amdgcn_ballot_w64((top[0] > top[1] ? top[0] : top[1]) >= 0x7F80u) != 0;
    q_v4i out[2];
    float scale[2];
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      unsigned m = top[f];
      if (special) {
        m = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const unsigned a = amax_bits_of(v[f][i]) >> 16;               // a NaN counts as zero
          m = m > a ? m : a;
        }
      }
      unsigned o;
      o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xF, 0xF, false);       // quad_perm [1, 0, 3, 2]
      m = m > o ? m : o;
      o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xF, 0xF, false);       // quad_perm [2, 3, 0, 1]
      m = m > o ? m : o;
      o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0x141, 0xF, 0xF, false);      // row_half_mirror: the other quad of the eight
      m = m > o ? m : o;
      const float amax = block_amax(m << 16);
      scale[f] = amax / 448.0f;
      const float inv = 448.0f / amax;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if (!special) {
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = __builtin_amdgcn_fmed3f(v[f][4 * d + e] * inv, -448.0f, 448.0f);
          int wd = 0;
          wd = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], wd, false);
          wd = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], wd, true);
          out[f][d] = wd;
        } else {
          out[f][d] = e4m3x4_of(v[f] + 4 * d, inv);
        }
      }
    }
    // M_total is a multiple of 16: a 16-byte piece of a row of XT exists whole or not at all
    const int tok0 = 128 * j + 16 * part;
    if (tok0 < M_total) {
      uint8_t* dst = XT + (int64_t)(k0 + 2 * fp) * M_total + tok0;
      *(q_v4i*)dst = out[0];
      *(q_v4i*)(dst + M_total) = out[1];
    }
    if (part == 0) *(q_v2i*)(SX + (int64_t)j * K + k0 + 2 * fp) = (q_v2i){__builtin_bit_cast(int, scale[0]), __builtin_bit_cast(int, scale[1])};
    __syncthreads();                                        // before the next tile's rows overwrite these
  }
}

__global__ void __launch_bounds__(Q_THREADS) gg_swiglu_quantize_rows_kernel(const uint16_t* __restrict__ H,
                                                                            uint8_t* __restrict__ A, float* __restrict__ SA,
                                                                            uint16_t* __restrict__ act_out,
                                                                            int M_total, int I, int IB,
                                                                            int64_t sa_rs, int64_t sa_ks,     // SA[row * sa_rs + blk * sa_ks]
                                                                            int by_xcd) {
  const int grp = threadIdx.x >> 4, sub = threadIdx.x & 15;
  const int64_t npairs = ((int64_t)M_total + 1) / 2;
  for (int64_t t = 0;; ++t) {
    const int64_t pr = pair_of(t, npairs, by_xcd);
    if (pr == -1) break;
    if (pr < 0) continue;
    const int64_t r64 = 2 * pr;
    const int r = (int)r64;
    const int r2 = r64 + 1 < M_total ? (int)(r64 + 1) : M_total;
    for (int v0 = 0; v0 < 2 * IB; v0 += 32) {
      const RowPairSlot a = row_pair_slot(v0 + grp, IB, r, r2, M_total);
      const RowPairSlot b = row_pair_slot(v0 + 16 + grp, IB, r, r2, M_total);
      q_v4i gA = {0, 0, 0, 0}, uA = {0, 0, 0, 0}, gB = {0, 0, 0, 0}, uB = {0, 0, 0, 0};
      if (a.valid) {
        const uint16_t* src = H + (int64_t)a.row * 2 * I + a.blk * 128 + sub * 8;
        gA = *(const q_v4i*)src;
        uA = *(const q_v4i*)(src + I);
      }
      if (b.valid) {
        const uint16_t* src = H + (int64_t)b.row * 2 * I + b.blk * 128 + sub * 8;
        gB = *(const q_v4i*)src;
        uB = *(const q_v4i*)(src + I);
      }
      if (a.valid) {
        const q_v4i act = swiglu8(gA, uA);
        const int64_t o = (int64_t)a.row * I + a.blk * 128 + sub * 8;
        if (act_out) *(q_v4i*)(act_out + o) = act;
        quantize_block(act, A + o, SA + a.row * sa_rs + a.blk * sa_ks, sub);
      }
      if (b.valid) {
        const q_v4i act = swiglu8(gB, uB);
        const int64_t o = (int64_t)b.row * I + b.blk * 128 + sub * 8;
        if (act_out) *(q_v4i*)(act_out + o) = act;
        quantize_block(act, A + o, SA + b.row * sa_rs + b.blk * sa_ks, sub);
      }
    }
  }
}

}  // namespace gg
