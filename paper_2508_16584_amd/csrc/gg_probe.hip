// libgg_probe: the ceilings the grouped GEMM kernels run into, measured with the kernels' own instructions and access
// shapes and nothing around them (see include/gg_probe.h).  Not part of the hot path.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <vector>

#include "gg_probe.h"
#include "gemm_kernel.h"   // operand vector types, buffer descriptor flags, wait_vmcnt
#include "gemm_kernel_rb.h"   // the second GEMM kernel, for its measurement builds (RbCfg<..., TIMING>)
#include "wgrad_kernel.h"     // the weight-gradient kernel, for its measurement builds (gg_wgrad_kernel<TIMING>)

namespace {

using gg::v4f;
using gg::v4i;
using gg::v8i;
typedef float v16f __attribute__((ext_vector_type(16)));

#define PROBE_TRY(x)                 \
  do {                               \
    hipError_t e_ = (x);             \
    if (e_ != hipSuccess) {          \
      cleanup();                     \
      return (int)e_;                \
    }                                \
  } while (0)

int cus() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  return n;
}

// ---------------------------------------------------------------------------------------------- matrix pipe
// Every wave holds 4 + 4 operand fragments (64 rows x 128 B of each side) and 64 x 64 fp32 accumulators, as a wave
// of the GEMM kernels does, and multiplies them over and over.  The empty asm per trip keeps the compiler from
// hoisting the products out of the loop.
template <int MODE>
__global__ void __launch_bounds__(512) mfma_loop_kernel(const v8i* __restrict__ src, const float* __restrict__ scales, float* out, int iters) {
  v8i a[4], b[4];
  for (int j = 0; j < 4; ++j) {
    a[j] = src[j * 512 + threadIdx.x];
    b[j] = src[(4 + j) * 512 + threadIdx.x];
  }
  float s[4];
  for (int j = 0; j < 4; ++j) s[j] = scales[j * 64 + threadIdx.x % 64];
  float total = 0.f;
  if constexpr (MODE < 2) {
    v4f acc[4][4];
    for (int j = 0; j < 4; ++j)
      for (int n = 0; n < 4; ++n) acc[j][n] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
      asm volatile("" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
      v4f p[16];
      // the FMAs of a product are issued three matrix instructions after it, as in the kernels
#pragma unroll
      for (int t = 0; t < 16 + 3; ++t) {
        if (t < 16) {
          if (MODE == 1) p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[t % 4], a[t / 4], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
          else acc[t / 4][t % 4] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[t % 4], a[t / 4], acc[t / 4][t % 4], 0, 0, 0, 0, 0, 0);
        }
        if (MODE == 1 && t >= 3) {
          const int u = t - 3;
          acc[u / 4][u % 4] += p[u] * s[u / 4];
        }
      }
      if (MODE == 1) {
#pragma unroll
        for (int t = 0; t < 16 + 3; ++t) {
          if (t < 16) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (t >= 3) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
      }
    }
    for (int j = 0; j < 4; ++j)
      for (int n = 0; n < 4; ++n) total += acc[j][n][0] + acc[j][n][1] + acc[j][n][2] + acc[j][n][3];
  } else {
    // 2 x 2 blocks of 32 x 32 outputs; operands a[2 * block + half], b[2 * block + half] for the two 64-wide halves
    // of a 128-wide scale block
    v16f acc[2][2];
    for (int j = 0; j < 2; ++j)
      for (int n = 0; n < 2; ++n)
        for (int i = 0; i < 16; ++i) acc[j][n][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
      asm volatile("" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
      if constexpr (MODE == 2) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          acc[u / 2][u % 2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[2 * (u % 2)], a[2 * (u / 2)], acc[u / 2][u % 2], 0, 0, 0, 0, 0, 0);
          acc[u / 2][u % 2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[2 * (u % 2) + 1], a[2 * (u / 2) + 1], acc[u / 2][u % 2], 0, 0, 0, 0, 0, 0);
        }
      } else {
        v16f p[4];
        v16f zero;
        for (int i = 0; i < 16; ++i) zero[i] = 0.f;
#pragma unroll
        for (int u = 0; u < 4 + 1; ++u) {
          if (u < 4) {
            p[u] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[2 * (u % 2)], a[2 * (u / 2)], zero, 0, 0, 0, 0, 0, 0);
            p[u] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[2 * (u % 2) + 1], a[2 * (u / 2) + 1], p[u], 0, 0, 0, 0, 0, 0);
          }
          if (u >= 1) {
            const int v = u - 1;
            acc[v / 2][v % 2] += p[v] * s[v / 2];
          }
        }
#pragma unroll
        for (int u = 0; u < 4 + 1; ++u) {
          if (u < 4) __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
          if (u >= 1) __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
        }
      }
    }
    for (int j = 0; j < 2; ++j)
      for (int n = 0; n < 2; ++n)
        for (int i = 0; i < 16; ++i) total += acc[j][n][i];
  }
  out[blockIdx.x * 512 + threadIdx.x] = total;
}

// The matrix loop of mode 1 with NS scalar, NV vector and NL LDS-read instructions more per matrix instruction: what
// each instruction beside the matrix instruction and its 4 FMAs costs in matrix-pipe time.  The extra instructions do
// nothing useful (counters, reads of a conflict-free 16 KB whose results are only waited for once per trip).
template <int NS, int NV, int NL>
__global__ void __launch_bounds__(512) issue_mix_kernel(const v8i* __restrict__ src, const float* __restrict__ scales, float* out, int iters) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[16384];
  for (int i = threadIdx.x; i < 4096; i += 512) ((int*)lds)[i] = i;
  __syncthreads();
  v8i a[4], b[4];
  for (int j = 0; j < 4; ++j) {
    a[j] = src[j * 512 + threadIdx.x];
    b[j] = src[(4 + j) * 512 + threadIdx.x];
  }
  float s[4];
  for (int j = 0; j < 4; ++j) s[j] = scales[j * 64 + threadIdx.x % 64];
  v4f acc[4][4];
  for (int j = 0; j < 4; ++j)
    for (int n = 0; n < 4; ++n) acc[j][n] = (v4f){0.f, 0.f, 0.f, 0.f};
  int sx = iters, vx = threadIdx.x;
  // every lane reads its own 16 bytes of its wave's 1 KB: no bank conflicts
  const unsigned rd = (unsigned)(size_t)GG_LDS_PTR(lds) + (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 2048;
  for (int it = 0; it < iters; ++it) {
    asm volatile("" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
    v4f p[16];
#pragma unroll
    for (int t = 0; t < 16 + 3; ++t) {
      if (t < 16) {
        p[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[t % 4], a[t / 4], (v4f){0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NS; ++q) asm volatile("s_add_u32 %0, %0, 3" : "+s"(sx) : : "scc");
#pragma unroll
        for (int q = 0; q < NV; ++q) asm volatile("v_add_u32 %0, %0, 3" : "+v"(vx));
#pragma unroll
        for (int q = 0; q < NL; ++q) {
          v4i r;
          asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(rd));
          asm volatile("" : : "v"(r));
        }
      }
      if (t >= 3) {
        const int u = t - 3;
        acc[u / 4][u % 4] += p[u] * s[u / 4];
      }
    }
    if (NL) asm volatile("s_waitcnt lgkmcnt(0)");
  }
  float total = (float)(sx + vx);
  for (int j = 0; j < 4; ++j)
    for (int n = 0; n < 4; ++n) total += acc[j][n][0] + acc[j][n][1] + acc[j][n][2] + acc[j][n][3];
  out[blockIdx.x * 512 + threadIdx.x] = total;
}

// e4m3 code of a float, round to nearest (ties away: operand statistics are all that matters here)
uint8_t e4m3_of(float v) {
  const float av = std::fabs(v);
  if (av < 0.0009765625f) return 0;
  int e = 0;
  const float m = std::frexp(av, &e);   // av = m * 2^e, m in [0.5, 1)
  int E = e - 1 + 7;
  int mant = (int)std::lround((m * 2.f - 1.f) * 8.f);
  if (mant == 8) {
    mant = 0;
    ++E;
  }
  if (E < 1) {
    E = 0;
    mant = (int)std::lround(av * 512.f);
    if (mant > 7) {
      E = 1;
      mant = 0;
    }
  }
  if (E > 15 || (E == 15 && mant > 6)) {
    E = 15;
    mant = 6;
  }
  return (uint8_t)((v < 0 ? 0x80 : 0) | (E << 3) | mant);
}

// ---------------------------------------------------------------------------------------------- HBM streams
__global__ void __launch_bounds__(256) hbm_read_kernel(const v4i* __restrict__ src, size_t n16, int* out) {
  int acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
    const v4i v = __builtin_nontemporal_load(src + i);
    acc += v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x5EEDBEEF) out[0] = acc;   // practically never: keeps the loads alive
}
__global__ void __launch_bounds__(256) hbm_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------- L2 -> LDS fetch stream
// One step = 8 fetch instructions per wave (4 slabs of 8 rows x 128 B of "A", 4 of "B"): 64 KB per workgroup.  All
// steps land in the same 64 KB of LDS (nobody reads it); how many steps are in flight is set by the wait alone.
constexpr int kFetchK = 7168, kFetchKB = kFetchK / 128;
constexpr size_t kFetchABytes = (size_t)8 * 4 * 256 * kFetchK;   // per die: 4 tiles of 256 rows
constexpr size_t kFetchBBytes = (size_t)8 * 8 * 256 * kFetchK;   // per die: 8 tiles of 256 rows

template <int DEPTH>
__global__ void __launch_bounds__(512) lds_fetch_kernel(const uint8_t* A, const uint8_t* B, int pattern, int steps) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
  const int b = blockIdx.x;
  const int xcd = b & 7, slot = (b >> 3) & 31;
  const __amdgpu_buffer_rsrc_t dA = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, (int)kFetchABytes, GG_RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t dB = __builtin_amdgcn_make_buffer_rsrc((void*)B, 0, (int)kFetchBBytes, GG_RSRC_FLAGS);
  int vA, vB, pitch_rows;     // lane offsets of slab 0; a slab further down is pitch_rows bytes on
  const int row = w * 8 + (l >> 3), chunk = (l & 7) << 4;
  if (pattern == 0) {
    // contiguous: "rows" of 128 B one after the other, 32 KB from each buffer
    vA = b * 32768 + row * 128 + chunk;
    vB = vA;
    pitch_rows = 64 * 128;
  } else if (pattern == 1) {
    vA = (b & 31) * 256 * kFetchK + (b % kFetchKB) * 128 + row * kFetchK + chunk;
    vB = (b & 63) * 256 * kFetchK + (b % kFetchKB) * 128 + row * kFetchK + chunk;
    pitch_rows = 64 * kFetchK;
  } else {
    vA = (xcd * 4 + (slot >> 3)) * 256 * kFetchK + row * kFetchK + chunk;
    vB = (xcd * 8 + (slot & 7)) * 256 * kFetchK + row * kFetchK + chunk;
    pitch_rows = 64 * kFetchK;
  }
  int kb = 0;
  for (int s = 0; s < steps; ++s) {
    const int so = pattern == 2 ? kb * 128 : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dA, GG_LDS_PTR(lds + (w + i * 8) * 1024), 16, vA + i * pitch_rows, so, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dB, GG_LDS_PTR(lds + 32768 + (w + i * 8) * 1024), 16, vB + i * pitch_rows, so, 0, 0);
    gg::wait_vmcnt<(DEPTH - 1) * 8>();
    __builtin_amdgcn_s_barrier();     // the kernels synchronise once per K block
    kb = kb + 1 == kFetchKB ? 0 : kb + 1;
  }
  gg::wait_vmcnt<0>();
}

template <int DEPTH>
hipError_t launch_fetch(const uint8_t* A, const uint8_t* B, int pattern, int steps, int grid) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lds_fetch_kernel<DEPTH>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(lds_fetch_kernel<DEPTH>, dim3(grid), dim3(512), 65536, 0, A, B, pattern, steps);
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------- K step of the GEMM
// Operand bytes like e4m3-quantised normal samples (sum of four uniforms, 3 sigma at the format's largest value),
// made on the device with the hardware conversion; scales: positive values around 2^-7.
__global__ void __launch_bounds__(256) fill_e4m3_kernel(uint8_t* p, size_t n, unsigned seed) {
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += stride) {
    float v[4];
    for (int j = 0; j < 4; ++j) {
      unsigned x = (unsigned)(i + j) * 2654435761u + seed;
      float g = 0.f;
      for (int u = 0; u < 4; ++u) {
        x = x * 1664525u + 1013904223u;
        g += (float)(x >> 8) * (1.0f / 16777216.0f) - 0.5f;
      }
      v[j] = g * 1.7320508f * (448.0f / 3.0f);
    }
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], w, true);
    *(int*)(p + i) = w;
  }
}
__global__ void __launch_bounds__(256) fill_scale_kernel(float* p, size_t n, unsigned seed) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const unsigned x = ((unsigned)i * 2654435761u + seed) * 1664525u + 1013904223u;
    p[i] = 0.0078125f * (1.0f + (float)(x >> 8) * (1.0f / 16777216.0f));
  }
}

template <class Cfg>
hipError_t launch_rb(const gg::GemmArgs& args, int grid) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gg::gg_gemm_rb_kernel<Cfg>), hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gg::gg_gemm_rb_kernel<Cfg>, dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, 0, args);
  return hipGetLastError();
}
template <int TIMING>
hipError_t launch_rb_rows(int tile_rows, const gg::GemmArgs& args, int grid) {
  if (tile_rows == 192) return launch_rb<gg::RbCfg<192, 4, false, false, false, false, false, TIMING>>(args, grid);
  return launch_rb<gg::RbCfg<256, 2, false, false, false, false, false, TIMING>>(args, grid);
}

template <int TIMING>
hipError_t launch_wgrad(const gg::WgradArgs& args, int grid) {
  static bool prepared = false;
  if (!prepared) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gg::gg_wgrad_kernel<TIMING>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, gg::WgradCfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    prepared = true;
  }
  hipLaunchKernelGGL(gg::gg_wgrad_kernel<TIMING>, dim3((unsigned)grid), dim3(gg::WgradCfg::NT), gg::WgradCfg::LDS_BYTES, 0, args);
  return hipGetLastError();
}

}  // namespace

extern "C" {

int gg_probe_mfma(int mode, int data_kind, int iters, double* tflops_out) {
  if (mode < 0 || mode > 3 || data_kind < 0 || data_kind > 2 || iters <= 0 || !tflops_out) return (int)hipErrorInvalidValue;
  v8i* src = nullptr;
  float *scales = nullptr, *out = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&] {
    if (src) (void)hipFree(src);
    if (scales) (void)hipFree(scales);
    if (out) (void)hipFree(out);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  const int blocks = cus();
  std::vector<uint8_t> h((size_t)8 * 512 * 32);
  unsigned x = 777u;
  for (uint8_t& byte : h) {
    x = x * 1664525u + 1013904223u;
    if (data_kind == 0) {
      byte = 0x38;
    } else if (data_kind == 2) {
      byte = (uint8_t)(x >> 24);
      if ((byte & 0x7F) == 0x7F) byte = 0x40;
    } else {
      // sum of 4 uniforms: close enough to a normal sample; 3 sigma at the format's largest value
      unsigned y = x;
      float g = 0.f;
      for (int i = 0; i < 4; ++i) {
        y = y * 1664525u + 1013904223u;
        g += (y >> 8) / 16777216.0f - 0.5f;
      }
      byte = e4m3_of(g * 1.7320508f * (448.0f / 3.0f));
    }
  }
  std::vector<float> ones(256, 1.0f);
  PROBE_TRY(hipMalloc(&src, h.size()));
  PROBE_TRY(hipMalloc(&scales, ones.size() * 4));
  PROBE_TRY(hipMalloc(&out, (size_t)blocks * 512 * 4));
  PROBE_TRY(hipMemcpy(src, h.data(), h.size(), hipMemcpyHostToDevice));
  PROBE_TRY(hipMemcpy(scales, ones.data(), ones.size() * 4, hipMemcpyHostToDevice));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {   // the first launch warms up
    PROBE_TRY(hipEventRecord(e0, 0));
    if (mode == 0) hipLaunchKernelGGL(mfma_loop_kernel<0>, dim3(blocks), dim3(512), 0, 0, src, scales, out, iters);
    else if (mode == 1) hipLaunchKernelGGL(mfma_loop_kernel<1>, dim3(blocks), dim3(512), 0, 0, src, scales, out, iters);
    else if (mode == 2) hipLaunchKernelGGL(mfma_loop_kernel<2>, dim3(blocks), dim3(512), 0, 0, src, scales, out, iters);
    else hipLaunchKernelGGL(mfma_loop_kernel<3>, dim3(blocks), dim3(512), 0, 0, src, scales, out, iters);
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
  }
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  const double flop = 2.0 * 64 * 64 * 128 * (double)iters * blocks * 8.0;
  *tflops_out = flop / ((double)ms * 1e-3) * 1e-12;
  cleanup();
  return 0;
}

int gg_probe_issue_mix(int extra_salu, int extra_valu, int extra_lds_reads, int iters, double* tflops_out) {
  if (iters <= 0 || !tflops_out) return (int)hipErrorInvalidValue;
  // the combinations that are built
  const int key = extra_salu * 100 + extra_valu * 10 + extra_lds_reads;
  v8i* src = nullptr;
  float *scales = nullptr, *out = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&] {
    if (src) (void)hipFree(src);
    if (scales) (void)hipFree(scales);
    if (out) (void)hipFree(out);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  switch (key) {
    case 0: case 200: case 400: case 800: case 10: case 20: case 1: case 2: case 211: case 212: break;
    default: return (int)hipErrorInvalidValue;
  }
  const int blocks = cus();
  std::vector<float> ones(256, 1.0f);
  PROBE_TRY(hipMalloc(&src, (size_t)8 * 512 * 32));
  PROBE_TRY(hipMalloc(&scales, ones.size() * 4));
  PROBE_TRY(hipMalloc(&out, (size_t)blocks * 512 * 4));
  PROBE_TRY(hipMemset(src, 0x38, (size_t)8 * 512 * 32));   // every operand byte 1.0: the clock stays up, so times compare as cycles
  PROBE_TRY(hipMemcpy(scales, ones.data(), ones.size() * 4, hipMemcpyHostToDevice));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {   // the first launch warms up
    PROBE_TRY(hipEventRecord(e0, 0));
#define GG_MIX(S, V, L) hipLaunchKernelGGL((issue_mix_kernel<S, V, L>), dim3(blocks), dim3(512), 0, 0, src, scales, out, iters)
    switch (key) {
      case 0: GG_MIX(0, 0, 0); break;
      case 200: GG_MIX(2, 0, 0); break;
      case 400: GG_MIX(4, 0, 0); break;
      case 800: GG_MIX(8, 0, 0); break;
      case 10: GG_MIX(0, 1, 0); break;
      case 20: GG_MIX(0, 2, 0); break;
      case 1: GG_MIX(0, 0, 1); break;
      case 2: GG_MIX(0, 0, 2); break;
      case 211: GG_MIX(2, 1, 1); break;
      default: GG_MIX(2, 1, 2); break;
    }
#undef GG_MIX
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
  }
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  *tflops_out = 2.0 * 64 * 64 * 128 * (double)iters * blocks * 8.0 / ((double)ms * 1e-3) * 1e-12;
  cleanup();
  return 0;
}

int gg_probe_hbm(int kind, size_t bytes, int reps, double* gbytes_per_s_out) {
  if (kind < 0 || kind > 1 || bytes == 0 || bytes % 4096 != 0 || reps < 1 || !gbytes_per_s_out) return (int)hipErrorInvalidValue;
  v4i *src = nullptr, *dst = nullptr;
  int* flag = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&] {
    if (src) (void)hipFree(src);
    if (dst) (void)hipFree(dst);
    if (flag) (void)hipFree(flag);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  PROBE_TRY(hipMalloc(&src, bytes));
  if (kind == 1) PROBE_TRY(hipMalloc(&dst, bytes));
  PROBE_TRY(hipMalloc(&flag, 4));
  PROBE_TRY(hipMemset(src, 1, bytes));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  const int grid = cus() * 8;
  float best = 0.f;
  for (int rep = 0; rep < reps + 1; ++rep) {   // the first launch warms up
    PROBE_TRY(hipEventRecord(e0, 0));
    if (kind == 0) hipLaunchKernelGGL(hbm_read_kernel, dim3(grid), dim3(256), 0, 0, src, bytes / 16, flag);
    else hipLaunchKernelGGL(hbm_copy_kernel, dim3(grid), dim3(256), 0, 0, src, dst, bytes / 16);
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    if (rep > 0 && (best == 0.f || ms < best)) best = ms;
  }
  *gbytes_per_s_out = (double)bytes * (kind == 1 ? 2.0 : 1.0) / ((double)best * 1e-3) * 1e-9;
  cleanup();
  return 0;
}

int gg_probe_lds_fetch(int pattern, int depth, int reps, double* gbytes_per_s_out, double* bytes_per_clk_cu_out) {
  if (pattern < 0 || pattern > 2 || depth < 1 || depth > 7 || reps < 1 || !gbytes_per_s_out || !bytes_per_clk_cu_out) return (int)hipErrorInvalidValue;
  uint8_t *A = nullptr, *B = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&] {
    if (A) (void)hipFree(A);
    if (B) (void)hipFree(B);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  // one workgroup per compute unit, at most the 256 the patterns are laid out for (every offset stays inside the
  // two buffers for any such grid: pattern 0 reaches 256 * 32 KB, the others tile (8 * 4 or 8 * 8) * 256 rows)
  int grid = cus();
  if (grid > 256) grid = 256;
  grid -= grid % 8;
  if (grid < 8) return (int)hipErrorInvalidValue;
  PROBE_TRY(hipMalloc(&A, kFetchABytes));
  PROBE_TRY(hipMalloc(&B, kFetchBBytes));
  PROBE_TRY(hipMemset(A, 0x38, kFetchABytes));
  PROBE_TRY(hipMemset(B, 0x38, kFetchBBytes));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  const int steps = reps * kFetchKB;
  for (int rep = 0; rep < 2; ++rep) {   // the first launch warms up
    PROBE_TRY(hipEventRecord(e0, 0));
    hipError_t e = hipSuccess;
    switch (depth) {
      case 1: e = launch_fetch<1>(A, B, pattern, steps, grid); break;
      case 2: e = launch_fetch<2>(A, B, pattern, steps, grid); break;
      case 3: e = launch_fetch<3>(A, B, pattern, steps, grid); break;
      case 4: e = launch_fetch<4>(A, B, pattern, steps, grid); break;
      case 5: e = launch_fetch<5>(A, B, pattern, steps, grid); break;
      case 6: e = launch_fetch<6>(A, B, pattern, steps, grid); break;
      default: e = launch_fetch<7>(A, B, pattern, steps, grid); break;
    }
    PROBE_TRY(e);
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
  }
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  int dev = 0, khz = 0;
  PROBE_TRY(hipGetDevice(&dev));
  PROBE_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev));
  const double bytes = 65536.0 * steps * grid, sec = (double)ms * 1e-3;
  *gbytes_per_s_out = bytes / sec * 1e-9;
  *bytes_per_clk_cu_out = khz > 0 ? bytes / sec / ((double)khz * 1e3) / grid : 0.0;
  cleanup();
  return 0;
}

int gg_probe_gemm_kstep(int tile_rows, int left_out, int groups, int rows_per_group, int n, int k, int reps, double* us_out) {
  if ((tile_rows != 192 && tile_rows != 256) || groups < 1 || groups > 4096 || rows_per_group < 1 || n < 256 || n % 256 != 0 ||
      k < 512 || k % 256 != 0 || reps < 1 || !us_out)
    return (int)hipErrorInvalidValue;
  const int64_t m_total = (int64_t)groups * rows_per_group;
  if (m_total * k > 0x7FFFFFFFLL || (int64_t)n * k > 0x7FFFFFFFLL || m_total * n > 0x3FFFFFFFLL) return (int)hipErrorInvalidValue;
  switch (left_out) {
    case 0: case 1: case 2: case 4: case 8: case 5: case 13: case 16: case 20: case 28: case 32: case 92: break;
    default: return (int)hipErrorInvalidValue;
  }
  const int kb = k / 128, nb = n / 128;
  uint8_t *A = nullptr, *B = nullptr;
  float *SA = nullptr, *SB = nullptr;
  int32_t* off = nullptr;
  uint16_t* C = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&] {
    if (A) (void)hipFree(A);
    if (B) (void)hipFree(B);
    if (SA) (void)hipFree(SA);
    if (SB) (void)hipFree(SB);
    if (off) (void)hipFree(off);
    if (C) (void)hipFree(C);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  const size_t a_bytes = (size_t)m_total * k, b_bytes = (size_t)groups * n * k;
  PROBE_TRY(hipMalloc(&A, a_bytes));
  PROBE_TRY(hipMalloc(&B, b_bytes));
  PROBE_TRY(hipMalloc(&SA, (size_t)m_total * kb * 4));
  PROBE_TRY(hipMalloc(&SB, (size_t)groups * nb * kb * 4));
  PROBE_TRY(hipMalloc(&off, (size_t)(groups + 1) * 4));
  PROBE_TRY(hipMalloc(&C, (size_t)m_total * n * 2));
  std::vector<int32_t> h_off(groups + 1);
  for (int g = 0; g <= groups; ++g) h_off[g] = g * rows_per_group;
  PROBE_TRY(hipMemcpy(off, h_off.data(), h_off.size() * 4, hipMemcpyHostToDevice));
  const int fgrid = cus() * 8;
  if (left_out == 32) {   // the kernel as launched, on operands that are all zero bytes
    PROBE_TRY(hipMemset(A, 0, a_bytes));
    PROBE_TRY(hipMemset(B, 0, b_bytes));
  } else {
    hipLaunchKernelGGL(fill_e4m3_kernel, dim3(fgrid), dim3(256), 0, 0, A, a_bytes, 1u);
    hipLaunchKernelGGL(fill_e4m3_kernel, dim3(fgrid), dim3(256), 0, 0, B, b_bytes, 2u);
  }
  hipLaunchKernelGGL(fill_scale_kernel, dim3(fgrid), dim3(256), 0, 0, SA, (size_t)m_total * kb, 3u);
  hipLaunchKernelGGL(fill_scale_kernel, dim3(fgrid), dim3(256), 0, 0, SB, (size_t)groups * nb * kb, 4u);
  PROBE_TRY(hipGetLastError());
  PROBE_TRY(hipMemset(C, 0, (size_t)m_total * n * 2));

  // the launch arguments as the GEMM library fills them for whole tiles and blocks, row-major activation scales
  gg::GemmArgs args{};
  args.A = A;
  args.SA = SA;
  args.B = B;
  args.SB = SB;
  args.off = off;
  args.C = C;
  args.G = groups;
  args.M_total = (int)m_total;
  args.N = n;
  args.K = k;
  args.KB = kb;
  args.k_rem = 128;
  args.n_tiles = n / 256;
  args.n_chunk = args.n_tiles < 8 ? args.n_tiles : 8;
  args.sa_row_stride = 4 * kb;
  args.sa_kb_stride = 4;
  args.rot_mul = (k % 8192 == 4096) ? 4 : 0;
  const int64_t max_tiles = (int64_t)groups * ((rows_per_group + tile_rows - 1) / tile_rows) * args.n_tiles;
  int64_t grid = cus();
  if (grid > max_tiles) grid = max_tiles;
  if (grid >= 8) {
    grid -= grid % 8;
    args.slots = (int)(grid / 8);
  }
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  auto launch = [&]() -> hipError_t {
    switch (left_out) {
      case 0: case 32: return launch_rb_rows<0>(tile_rows, args, (int)grid);
      case 1: return launch_rb_rows<1>(tile_rows, args, (int)grid);
      case 2: return launch_rb_rows<2>(tile_rows, args, (int)grid);
      case 4: return launch_rb_rows<4>(tile_rows, args, (int)grid);
      case 8: return launch_rb_rows<8>(tile_rows, args, (int)grid);
      case 5: return launch_rb_rows<5>(tile_rows, args, (int)grid);
      case 16: return launch_rb_rows<16>(tile_rows, args, (int)grid);
      case 20: return launch_rb_rows<20>(tile_rows, args, (int)grid);
      case 28: return launch_rb_rows<28>(tile_rows, args, (int)grid);
      case 92: return launch_rb_rows<92>(tile_rows, args, (int)grid);
      default: return launch_rb_rows<13>(tile_rows, args, (int)grid);
    }
  };
  // warm-up: launches of the same build for about 150 ms, so that the timed ones run at the sustained clock (after
  // an idle period the clock takes about a hundred launches of this size to settle)
  for (float warm_ms = 0.f; warm_ms < 150.f;) {
    PROBE_TRY(hipEventRecord(e0, 0));
    for (int i = 0; i < 10; ++i) PROBE_TRY(launch());
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
    float t = 0.f;
    PROBE_TRY(hipEventElapsedTime(&t, e0, e1));
    warm_ms += t > 0.01f ? t : 0.01f;
  }
  PROBE_TRY(hipEventRecord(e0, 0));
  for (int i = 0; i < reps; ++i) PROBE_TRY(launch());
  PROBE_TRY(hipEventRecord(e1, 0));
  PROBE_TRY(hipEventSynchronize(e1));
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  *us_out = (double)ms * 1e3 / reps;
  cleanup();
  return 0;
}

int gg_probe_wgrad_parts(int left_out, int groups, int tokens_per_group, int n, int k, int reps, double* us_out) {
  if (groups < 1 || groups > 4096 || tokens_per_group < 1 || n < 128 || n % 128 != 0 || k < 256 || k % 256 != 0 || reps < 1 || !us_out)
    return (int)hipErrorInvalidValue;
  switch (left_out) {
    case 0: case 1: case 2: case 3: case 7: case 11: case 19: case 31: break;
    default: return (int)hipErrorInvalidValue;
  }
  // the token axis is padded to a multiple of 16 behind the last group, as the library asks
  const int64_t m_total = ((int64_t)groups * tokens_per_group + 15) / 16 * 16;
  const int64_t mb = (m_total + 127) / 128;
  if ((int64_t)k * m_total > 0x7FFFFFFFLL || (int64_t)n * m_total > 0x7FFFFFFFLL || (int64_t)groups * n * k > 0x3FFFFFFFLL)
    return (int)hipErrorInvalidValue;
  uint8_t *XT = nullptr, *DYT = nullptr;
  float *SX = nullptr, *SDY = nullptr, *dW = nullptr;
  int32_t* off = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&] {
    if (XT) (void)hipFree(XT);
    if (DYT) (void)hipFree(DYT);
    if (SX) (void)hipFree(SX);
    if (SDY) (void)hipFree(SDY);
    if (dW) (void)hipFree(dW);
    if (off) (void)hipFree(off);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  const size_t x_bytes = (size_t)k * m_total, y_bytes = (size_t)n * m_total, w_bytes = (size_t)groups * n * k * 4;
  PROBE_TRY(hipMalloc(&XT, x_bytes));
  PROBE_TRY(hipMalloc(&DYT, y_bytes));
  PROBE_TRY(hipMalloc(&SX, (size_t)mb * k * 4));
  PROBE_TRY(hipMalloc(&SDY, (size_t)mb * n * 4));
  PROBE_TRY(hipMalloc(&dW, w_bytes));
  PROBE_TRY(hipMalloc(&off, (size_t)(groups + 1) * 4));
  std::vector<int32_t> h_off(groups + 1);
  for (int g = 0; g <= groups; ++g) h_off[g] = g * tokens_per_group;
  PROBE_TRY(hipMemcpy(off, h_off.data(), h_off.size() * 4, hipMemcpyHostToDevice));
  const int fgrid = cus() * 8;
  hipLaunchKernelGGL(fill_e4m3_kernel, dim3(fgrid), dim3(256), 0, 0, XT, x_bytes, 5u);
  hipLaunchKernelGGL(fill_e4m3_kernel, dim3(fgrid), dim3(256), 0, 0, DYT, y_bytes, 6u);
  hipLaunchKernelGGL(fill_scale_kernel, dim3(fgrid), dim3(256), 0, 0, SX, (size_t)mb * k, 7u);
  hipLaunchKernelGGL(fill_scale_kernel, dim3(fgrid), dim3(256), 0, 0, SDY, (size_t)mb * n, 8u);
  PROBE_TRY(hipGetLastError());
  PROBE_TRY(hipMemset(dW, 0, w_bytes));

  // the launch arguments as the GEMM library fills them
  gg::WgradArgs args{};
  args.XT = XT;
  args.SX = SX;
  args.DYT = DYT;
  args.SDY = SDY;
  args.off = off;
  args.dW = dW;
  args.G = groups;
  args.M_total = (int)m_total;
  args.N = n;
  args.K = k;
  args.MB = (int)mb;
  args.n_tiles = n / gg::WgradCfg::TN;
  args.k_tiles = k / gg::WgradCfg::TK;
  args.tiles = groups * args.n_tiles * args.k_tiles;
  args.blocked = args.k_tiles % 4 == 0 && args.n_tiles % 8 == 0;
  int64_t grid = cus();
  if (grid > args.tiles) grid = args.tiles;
  if (grid >= 8) {
    grid -= grid % 8;
    args.slots = (int)(grid / 8);
  }
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  auto launch = [&]() -> hipError_t {
    switch (left_out) {
      case 0: return launch_wgrad<0>(args, (int)grid);
      case 1: return launch_wgrad<1>(args, (int)grid);
      case 2: return launch_wgrad<2>(args, (int)grid);
      case 3: return launch_wgrad<3>(args, (int)grid);
      case 7: return launch_wgrad<7>(args, (int)grid);
      case 11: return launch_wgrad<11>(args, (int)grid);
      case 19: return launch_wgrad<19>(args, (int)grid);
      default: return launch_wgrad<31>(args, (int)grid);
    }
  };
  for (float warm_ms = 0.f; warm_ms < 150.f;) {     // the sustained clock, as in gg_probe_gemm_kstep
    PROBE_TRY(hipEventRecord(e0, 0));
    for (int i = 0; i < 10; ++i) PROBE_TRY(launch());
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
    float t = 0.f;
    PROBE_TRY(hipEventElapsedTime(&t, e0, e1));
    warm_ms += t > 0.01f ? t : 0.01f;
  }
  PROBE_TRY(hipEventRecord(e0, 0));
  for (int i = 0; i < reps; ++i) PROBE_TRY(launch());
  PROBE_TRY(hipEventRecord(e1, 0));
  PROBE_TRY(hipEventSynchronize(e1));
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  *us_out = (double)ms * 1e3 / reps;
  cleanup();
  return 0;
}

}  // extern "C"
