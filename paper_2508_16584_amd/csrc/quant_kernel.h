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

__global__ void __launch_bounds__(Q_THREADS) gg_quantize_rows_kernel(const uint16_t* __restrict__ X,
                                                                     const int32_t* __restrict__ row_src,
                                                                     uint8_t* __restrict__ A, float* __restrict__ SA,
                                                                     int64_t T, int M_total, int K, int KB) {
  const int grp = threadIdx.x >> 4, sub = threadIdx.x & 15;
  for (int r = blockIdx.x; r < M_total; r += gridDim.x) {
    const int64_t s = row_src ? (int64_t)row_src[r] : (int64_t)r;
    const bool ok = s >= 0 && s < T;                       // a source outside [0, T) stands for a row of zeros
    const uint16_t* src = X + (ok ? s : 0) * K;
    uint8_t* dstA = A + (int64_t)r * K;
    float* dstS = SA + (int64_t)r * KB;
    for (int kb0 = 0; kb0 < KB; kb0 += 32) {
      const int kbA = kb0 + grp, kbB = kb0 + 16 + grp;   // uniform over the 16 lanes of a row
      q_v4i rawA = {0, 0, 0, 0}, rawB = {0, 0, 0, 0};
      if (ok && kbA < KB) rawA = *(const q_v4i*)(src + kbA * 128 + sub * 8);
      if (ok && kbB < KB) rawB = *(const q_v4i*)(src + kbB * 128 + sub * 8);
      if (kbA < KB) quantize_block(rawA, dstA + kbA * 128 + sub * 8, dstS + kbA, sub);
      if (kbB < KB) quantize_block(rawB, dstA + kbB * 128 + sub * 8, dstS + kbB, sub);
    }
  }
}

}  // namespace gg
