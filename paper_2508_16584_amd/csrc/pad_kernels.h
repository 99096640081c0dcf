// The pad / unpad kernels of the pad-then-GEMM comparison path (the baseline of paper Sec. 3:
// A and S_A of every group are copied to offsets that are multiples of 128 rows, pad rows are
// zero; after the GEMM the valid rows of the padded output are gathered back).  Pure HBM-bound
// copies: 16 bytes per lane, four loads in flight per lane, 16-row (pad) and 8-row (unpad) blocks per
// workgroup so that a problem of a few thousand rows still puts several workgroups on every compute unit,
// group lookup once per block.  Rows of the padded buffers past the last group (between padded_offsets[G]
// and the capacity the caller allocated) belong to no group: nothing reads them and nothing writes them.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gg {

typedef int pv4i __attribute__((ext_vector_type(4)));

constexpr int PAD_ALIGN = 128;       // row alignment of a padded group
constexpr int PAD_BLOCK_ROWS = 16;   // rows one workgroup moves per step (divides PAD_ALIGN)
constexpr int UNPAD_BLOCK_ROWS = 8;  // output rows per workgroup and step: two per wave, moved together
constexpr int PAD_THREADS = 256;

__device__ __forceinline__ int pad_clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// padded_offsets[0] = 0, padded_offsets[g+1] = padded_offsets[g] + 128 * ceil(M^g / 128).  One workgroup.
__global__ void __launch_bounds__(PAD_THREADS) gg_pad_offsets_kernel(const int32_t* __restrict__ off,
                                                                       int32_t* __restrict__ poff, int G, int M_total) {
  __shared__ int part[PAD_THREADS];
  const int t = threadIdx.x;
  const int per = (G + PAD_THREADS - 1) / PAD_THREADS;
  const int g0 = t * per, g1 = (g0 + per < G) ? g0 + per : G;
  int sum = 0;
  for (int g = g0; g < g1; ++g) {
    const int lo = pad_clampi(off[g], 0, M_total);
    const int hi = pad_clampi(off[g + 1], lo, M_total);
    sum += (hi - lo + PAD_ALIGN - 1) / PAD_ALIGN * PAD_ALIGN;
  }
  part[t] = sum;
  __syncthreads();
  // exclusive scan over the 256 partial sums (Hillis-Steele)
  for (int d = 1; d < PAD_THREADS; d <<= 1) {
    const int v = (t >= d) ? part[t - d] : 0;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  int run = part[t] - sum;
  if (t == 0) poff[0] = 0;
  for (int g = g0; g < g1; ++g) {
    const int lo = pad_clampi(off[g], 0, M_total);
    const int hi = pad_clampi(off[g + 1], lo, M_total);
    run += (hi - lo + PAD_ALIGN - 1) / PAD_ALIGN * PAD_ALIGN;
    poff[g + 1] = run;
  }
}

// group whose padded range holds padded row p, or G if p is past the last group
__device__ __forceinline__ int pad_find_group(const int32_t* __restrict__ poff, int G, int p) {
  int lo = 0, hi = G;  // invariant: poff[lo] <= p (poff[0] = 0), answer in [lo, hi]
  if (p >= poff[G]) return G;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (poff[mid] <= p) lo = mid; else hi = mid;
  }
  return lo;  // poff[lo] <= p < poff[lo + 1]: empty groups are never returned
}

// One workgroup per 16-row block of the padded matrices (grid-stride).  The block lies inside one
// group's padded range, so the group is looked up once; blocks past the last group are left alone.
__global__ void __launch_bounds__(PAD_THREADS) gg_pad_rows_kernel(const uint8_t* __restrict__ A, const float* __restrict__ SA,
                                                                    const int32_t* __restrict__ off, const int32_t* __restrict__ poff,
                                                                    uint8_t* __restrict__ A_pad, float* __restrict__ SA_pad,
                                                                    int G, int M_total, int M_pad_cap, int K, int KB, int sa_kmajor) {
  const int nblocks = (M_pad_cap + PAD_BLOCK_ROWS - 1) / PAD_BLOCK_ROWS;
  const int chunks = K >> 4;  // 16-byte chunks per row of A
  for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const int p0 = blk * PAD_BLOCK_ROWS;
    const int g = pad_find_group(poff, G, p0);
    if (g >= G) break;            // past the last group, and so is every later block of this workgroup
    int src0 = 0, valid = 0;
    {
      const int lo = pad_clampi(off[g], 0, M_total);
      const int hi = pad_clampi(off[g + 1], lo, M_total);
      const int within = p0 - poff[g];
      src0 = lo + within;
      valid = pad_clampi(hi - src0, 0, PAD_BLOCK_ROWS);
    }
    int rows = M_pad_cap - p0;
    rows = rows < PAD_BLOCK_ROWS ? rows : PAD_BLOCK_ROWS;
    const pv4i* __restrict__ src = (const pv4i*)(A + (int64_t)src0 * K);
    pv4i* __restrict__ dst = (pv4i*)(A_pad + (int64_t)p0 * K);
    const int total = rows * chunks, nvalid = valid * chunks;   // rows are contiguous: flat copy
    for (int i = threadIdx.x; i < total; i += PAD_THREADS * 4) {
      pv4i v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = i + u * PAD_THREADS;
        v[u] = (pv4i){0, 0, 0, 0};
        if (j < nvalid) v[u] = __builtin_nontemporal_load(src + j);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = i + u * PAD_THREADS;
        if (j < total) __builtin_nontemporal_store(v[u], dst + j);
      }
    }
    if (sa_kmajor) {
      // SA [KB, M_total] -> SA_pad [KB, M_pad_cap]: per K block, the block's 16 rows are contiguous
      for (int i = threadIdx.x; i < PAD_BLOCK_ROWS * KB; i += PAD_THREADS) {
        const int kb = i / PAD_BLOCK_ROWS, j = i % PAD_BLOCK_ROWS;
        if (j < rows) SA_pad[(int64_t)kb * M_pad_cap + p0 + j] = j < valid ? SA[(int64_t)kb * M_total + src0 + j] : 0.f;
      }
    } else {
      const float* __restrict__ ssrc = SA + (int64_t)src0 * KB;
      float* __restrict__ sdst = SA_pad + (int64_t)p0 * KB;
      for (int i = threadIdx.x; i < rows * KB; i += PAD_THREADS) sdst[i] = (i < valid * KB) ? ssrc[i] : 0.f;
    }
  }
}

// C[off[g] + i][:] = C_pad[poff[g] + i][:].  One workgroup per 8 output rows (grid-stride); wave w moves rows w and
// w + 4 of the block together, two 16-byte loads of each in flight per lane.  Rows of C outside [off[0], off[G])
// are not touched.
__global__ void __launch_bounds__(PAD_THREADS) gg_unpad_rows_kernel(const uint16_t* __restrict__ C_pad, const int32_t* __restrict__ off,
                                                                      const int32_t* __restrict__ poff, uint16_t* __restrict__ C,
                                                                      int G, int M_total, int N) {
  const int nblocks = (M_total + UNPAD_BLOCK_ROWS - 1) / UNPAD_BLOCK_ROWS;
  const int chunks = N >> 3;  // 16-byte chunks per bf16 row
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const int r0 = blk * UNPAD_BLOCK_ROWS;
    // first group that ends after r0
    int lo = 0, hi = G;  // answer in [lo, hi]; hi == G means none
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (pad_clampi(off[mid + 1], 0, M_total) > r0) hi = mid; else lo = mid + 1;
    }
    int g = lo;
    // source row of output row `row`, or -1 if the row belongs to no group (g only ever moves forward)
    auto source_of = [&](int row) -> int64_t {
      if (row >= M_total) return -1;
      while (g < G && pad_clampi(off[g + 1], 0, M_total) <= row) ++g;
      if (g >= G) return -1;
      const int start = pad_clampi(off[g], 0, M_total);
      return row < start ? -1 : (int64_t)poff[g] + (row - start);
    };
    const int row_a = r0 + wave, row_b = r0 + wave + PAD_THREADS / 64;
    const int64_t sa = source_of(row_a), sb = source_of(row_b);
    const pv4i* __restrict__ src_a = (const pv4i*)(C_pad + (sa < 0 ? 0 : sa) * N);
    const pv4i* __restrict__ src_b = (const pv4i*)(C_pad + (sb < 0 ? 0 : sb) * N);
    pv4i* __restrict__ dst_a = (pv4i*)(C + (int64_t)row_a * N);
    pv4i* __restrict__ dst_b = (pv4i*)(C + (int64_t)row_b * N);
    for (int c = lane; c < chunks; c += 128) {
      const bool second = c + 64 < chunks;
      pv4i v[4];
      if (sa >= 0) {
        v[0] = __builtin_nontemporal_load(src_a + c);
        if (second) v[1] = __builtin_nontemporal_load(src_a + c + 64);
      }
      if (sb >= 0) {
        v[2] = __builtin_nontemporal_load(src_b + c);
        if (second) v[3] = __builtin_nontemporal_load(src_b + c + 64);
      }
      if (sa >= 0) {
        __builtin_nontemporal_store(v[0], dst_a + c);
        if (second) __builtin_nontemporal_store(v[1], dst_a + c + 64);
      }
      if (sb >= 0) {
        __builtin_nontemporal_store(v[2], dst_b + c);
        if (second) __builtin_nontemporal_store(v[3], dst_b + c + 64);
      }
    }
  }
}

}  // namespace gg
