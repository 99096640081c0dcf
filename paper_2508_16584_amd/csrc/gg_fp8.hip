// libgg_fp8: C-ABI entry points, argument validation and kernel dispatch.
// The operation and every convention are documented in include/gg_fp8.h.
#include "../../include/gg_fp8.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <vector>

#include "gemm_kernel.h"
#include "gemm_kernel_rb.h"
#include "pad_kernels.h"
#include "quant_kernel.h"
#include "wgrad_kernel.h"

// Scratch of gg_fp8_grouped_gemm_splitk_noalloc: the partial sums of a split-K call, [2][M_total][N] fp32, for
// problems of up to kScratchBytes / 8 output elements.  One copy per GPU the library runs on, held until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address the kernels
// get is the one that call returns (scratch_ptr below).
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kVersion = 200;  // 0.2.0: the weight-gradient GEMM and the column quantiser
constexpr int kXcds = 8;       // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// Number of compute units of the current device (queried once per device, cached).
int device_cus() {
  static std::atomic<int> cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int v = cache[dev].load(std::memory_order_relaxed);
  if (v > 0) return v;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
  cache[dev].store(cus, std::memory_order_relaxed);
  return cus;
}

struct Variant {
  const char* name;
  int BM, BN;
  int lds_bytes;
  int wg_per_cu;
  hipError_t (*launch)(const gg::GemmArgs&, int grid, hipStream_t);
  // the same tile for N % BN != 0 or K % 128 != 0 (partial tiles, short last K block); null: whole blocks only
  hipError_t (*launch_ragged)(const gg::GemmArgs&, int grid, hipStream_t) = nullptr;
  bool min_kb3 = false;        // the second kernel: its prologue fetches three K blocks (K > 256)
  bool splitk = false;         // two work units per tile (halves of the K loop) and a combine pass; needs a workspace
  // the same tile with the streaming cache policy on the weight fetches, for groups of at most one row tile; null: none
  hipError_t (*launch_bstream)(const gg::GemmArgs&, int grid, hipStream_t) = nullptr;
};

template <class Cfg, bool RAGGED = false, bool SPLITK = false, bool BSTREAM = false>
hipError_t launch_gemm(const gg::GemmArgs& args, int grid, hipStream_t stream) {
  static std::atomic<int> prepared[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && !prepared[dev].load(std::memory_order_acquire)) {
    // more than 64 KB of LDS per workgroup has to be requested explicitly
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gg::gg_gemm_kernel<Cfg, RAGGED, SPLITK, BSTREAM>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    prepared[dev].store(1, std::memory_order_release);
  }
  hipLaunchKernelGGL((gg::gg_gemm_kernel<Cfg, RAGGED, SPLITK, BSTREAM>), dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, stream, args);
  return hipGetLastError();
}

// name = "BMxBN/WMxWNw/STAGESs[x]": tile, wave grid, LDS ring depth; x = barrier in the middle of the MFMA
// stream with operand prefetch across K blocks.  GAP = MFMAs between two DMAs fed into the MFMA stream.
template <class Cfg>
hipError_t launch_gemm_rb(const gg::GemmArgs& args, int grid, hipStream_t stream) {
  static std::atomic<int> prepared[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && !prepared[dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gg::gg_gemm_rb_kernel<Cfg>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    prepared[dev].store(1, std::memory_order_release);
  }
  hipLaunchKernelGGL(gg::gg_gemm_rb_kernel<Cfg>, dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, stream, args);
  return hipGetLastError();
}

#define GG_VARIANT(BM, BN, WM, WN, ST, XPF, GAP, WGPC)                                                        \
  {#BM "x" #BN "/" #WM "x" #WN "w/" #ST "s" XPF_SUFFIX_##XPF, BM, BN, gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>::LDS_BYTES, \
   WGPC, &launch_gemm<gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>>, nullptr}
#define GG_VARIANT_R(BM, BN, WM, WN, ST, XPF, GAP, WGPC)   /* with the instantiation for ragged N and K */         \
  {#BM "x" #BN "/" #WM "x" #WN "w/" #ST "s" XPF_SUFFIX_##XPF, BM, BN, gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>::LDS_BYTES, \
   WGPC, &launch_gemm<gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>>, &launch_gemm<gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>, true>}
#define GG_VARIANT_RS(BM, BN, WM, WN, ST, XPF, GAP, WGPC)   /* ... and the one with streamed weight fetches */     \
  {#BM "x" #BN "/" #WM "x" #WN "w/" #ST "s" XPF_SUFFIX_##XPF, BM, BN, gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>::LDS_BYTES, \
   WGPC, &launch_gemm<gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>>, &launch_gemm<gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>, true>, \
   false, false, &launch_gemm<gg::GemmCfg<BM, BN, WM, WN, ST, XPF, GAP>, false, false, true>}
#define XPF_SUFFIX_false ""
#define XPF_SUFFIX_true "x"

const Variant kVariants[] = {
    GG_VARIANT_RS(160, 256, 2, 4, 3, false, 2, 1),   // 0: the largest tile that leaves room for a ring of 3 in 160 KB of LDS
    GG_VARIANT(256, 256, 2, 4, 2, false, 2, 1),   // 1: the largest tile the accumulators allow; ring of 2 only
    GG_VARIANT_R(128, 128, 2, 4, 4, false, 0, 1),   // 2: for N % 256 != 0
    GG_VARIANT_RS(128, 256, 2, 4, 3, false, 0, 1),   // 3
    GG_VARIANT(64, 256, 1, 8, 3, false, 0, 1),    // 4
    GG_VARIANT_R(32, 256, 1, 8, 4, false, 0, 1),    // 5
    GG_VARIANT(16, 256, 1, 8, 2, false, 0, 2),    // 6
    GG_VARIANT(256, 128, 4, 2, 3, false, 0, 1),   // 7
    GG_VARIANT(128, 256, 2, 4, 3, true, 0, 1),    // 8
    GG_VARIANT(128, 128, 2, 4, 4, true, 0, 1),    // 9
    GG_VARIANT(32, 256, 1, 8, 4, true, 0, 1),     // 10
    GG_VARIANT(128, 128, 2, 4, 2, false, 0, 2),   // 11
    {"256x256/1x8w/3s-rb", 256, 256, gg::RbCfg<256, 2, false>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<256, 2, false>>, &launch_gemm_rb<gg::RbCfg<256, 2, false, false, false, true>>, true},   // 12
    {"256x256/1x8w/3s-rbk", 256, 256, gg::RbCfg<256, 2, true>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<256, 2, true>>, nullptr, true},    // 13
    // ring of 4 activation fragments at 192 rows: 1 % faster than 2 there, no gain (and 249 VGPRs) at 256 rows
    {"192x256/1x8w/3s-rb", 192, 256, gg::RbCfg<192, 4, false>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<192, 4, false>>, &launch_gemm_rb<gg::RbCfg<192, 4, false, false, false, true>>, true},   // 14
    {"224x256/1x8w/3s-rb", 224, 256, gg::RbCfg<224, 2, false>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<224, 2, false>>, &launch_gemm_rb<gg::RbCfg<224, 2, false, false, false, true>>, true},   // 15
    {"128x256/1x8w/3s-rb", 128, 256, gg::RbCfg<128, 4, false>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<128, 4, false>>, &launch_gemm_rb<gg::RbCfg<128, 4, false, false, false, true>>, true},   // 16
    {"160x256/1x8w/3s-rb", 160, 256, gg::RbCfg<160, 2, false>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<160, 2, false>>, nullptr, true},   // 17
    {"96x256/1x8w/3s-rb", 96, 256, gg::RbCfg<96, 2, false>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<96, 2, false>>, nullptr, true},   // 18
    // "-rbs": the second kernel with K steps that leave out the activation blocks past a tile's last valid row
    {"256x256/1x8w/3s-rbs", 256, 256, gg::RbCfg<256, 2, false, false, true>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<256, 2, false, false, true>>, nullptr, true},   // 19
    {"192x256/1x8w/3s-rbs", 192, 256, gg::RbCfg<192, 4, false, false, true>::LDS_BYTES, 1, &launch_gemm_rb<gg::RbCfg<192, 4, false, false, true>>, nullptr, true},   // 20
    // "-k2": split-K, two halves of the K loop per tile and a combine pass (needs K % 256 == 0 and a workspace)
    {"128x256/2x4w/3s-k2", 128, 256, gg::GemmCfg<128, 256, 2, 4, 3, false, 0>::LDS_BYTES, 1,
     &launch_gemm<gg::GemmCfg<128, 256, 2, 4, 3, false, 0>, false, true>, nullptr, false, true},
    {"64x256/1x8w/3s-k2", 64, 256, gg::GemmCfg<64, 256, 1, 8, 3, false, 0>::LDS_BYTES, 1,
     &launch_gemm<gg::GemmCfg<64, 256, 1, 8, 3, false, 0>, false, true>, nullptr, false, true},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));
constexpr int kDefaultSplitK = kNumVariants - 2;   // 128 x 256 tile

// The second kernel with the activation epilogue (gg_fp8_grouped_gemm_swiglu): same tiles as variants 14, 15, 12.
struct FusedVariant {
  int variant;   // the plain variant it is the twin of
  int BM;
  hipError_t (*launch)(const gg::GemmArgs&, int, hipStream_t);
  // the instantiation for an odd number of K blocks (one more value in a scalar register: only the 192-row tile
  // has room for it); null: even numbers only
  hipError_t (*launch_odd)(const gg::GemmArgs&, int, hipStream_t);
};
const FusedVariant kFused[] = {
    {14, 192, &launch_gemm_rb<gg::RbCfg<192, 2, false, true>>, &launch_gemm_rb<gg::RbCfg<192, 2, false, true, false, false, true>>},
    {15, 224, &launch_gemm_rb<gg::RbCfg<224, 2, false, true>>, nullptr},
    {12, 256, &launch_gemm_rb<gg::RbCfg<256, 2, false, true>>, nullptr},
};

// Automatic choice.  The host sees only sizes (the offsets stay on the device), so the choice works with the
// expected tile count: a group ends in a partial tile half of the time on average, which adds G/2 tiles per
// column of tiles.  Candidates and their measured character on MI355X:
//   160x256, ring 3 (variant 0): the safe default; best when groups are short;
//   256x256, ring 2 (variant 1): fewest bytes per flop, one K block of look-ahead: was the best on the problems of
//       24576 rows or more with K >= 4096 in the paper's grid and was forced there; since the second kernel deals its
//       fetches out over the K step it is within -3 ... +1 % of that kernel's 256-row tile on such problems (five
//       measured) and competes through the estimate like the others;
//   second kernel at 192, 224 and 256 rows (variants 14, 15, 12): weights through registers, better overlap, K loop
//       carried from tile to tile: best on the smaller problems and on every problem with a short K loop (K = 1024
//       to 2560: the 256-row one is within 2 % of the per-point best everywhere on the paper's size generator, while
//       with strongly skewed group sizes the heights differ by under 3 %); needs an even number of K blocks.
//       Three heights, because on a few hundred tiles the number of rounds over the 256 workgroups matters more
//       than anything else (8192 rows in 8 groups, N = 4096: 2.9 rounds at 192 rows, 2.25 at 256, 3.45 at 160);
//   128x256 (variant 3): very short groups (weight streaming).
// Between the candidates allowed for a shape, the estimated time is rounds x tile height / efficiency, where a
// partly filled last round costs 0.3 + 0.7 x its fill (measured: the workgroups that do run get more of the L2
// bandwidth) and the efficiency per row is 1 : 1.06 : 1.07 : 1.10 for 160 : 192 : 224 : 256 rows of the kernels
// named above and, for the 256x256 ring-2 tile, 1.02 from K = 4096 on and 0.94 below.  The constants are a fit to the
// five candidates on the paper's grid (Sec. 3.1) extended to K = 1024 ... 8192 (960 points) with caches flushed
// before every launch: mean loss against the per-point best of the five 0.8 % (224 rows at 1.08 fitted the grid
// equally well; 1.07 also takes the 192-row tile on the strongly skewed sizes of the down workload, where it is 0 - 4 %
// the faster of the two).
int pick_variant(int G, int64_t M_total, int N, int K) {
  const double avg = G > 0 ? (double)M_total / G : 0.0;
  const int n_tiles = (N + 255) / 256;
  const bool ragged = N % 256 != 0 || K % 128 != 0;
  // A ragged N on 256-wide tiles: the columns past N of the last tile are computed for nothing.  Up to 1/8 of
  // waste the choice below stands; beyond that the 128-wide tile of the first kernel wastes least.
  if (N % 256 != 0 && (N % 128 != 0 || N < 256) && (double)n_tiles * 256 > 1.125 * N) return 2;
  if (avg < 64) return 3;
  if (avg < 192) return 0;
  const double cus = (double)device_cus();   // the constants below are a fit on 256 CUs; the round count follows the chip
  auto cost = [&](int BM, double eff) {
    const double rounds = ((double)M_total / BM + 0.5 * G) * n_tiles / cus;
    const double whole = std::floor(rounds), frac = rounds - whole;
    return (whole + (frac > 1e-9 ? 0.3 + 0.7 * frac : 0.0)) * BM / eff;
  };
  const bool second_kernel = K > 256;   // its prologue fetches three K blocks
  int best = 0;
  double c_best = cost(160, 1.0);
  auto consider = [&](int variant, double c) {
    if (c < c_best) { c_best = c; best = variant; }
  };
  if (second_kernel) consider(14, cost(192, 1.06));
  if (second_kernel) consider(15, cost(224, 1.07));
  if (second_kernel) consider(12, cost(256, 1.10));
  if (!ragged) consider(1, cost(256, K >= 4096 ? 1.02 : 0.94));   // the 256 x 256 ring-2 tile takes whole blocks only
  return best;
}

// The padded problem (Sec. 3: every group a multiple of 128 rows; M_pad_cap = 128 * (ceil(M_total / 128) + G) is a
// capacity, the groups hold about M_pad_cap - 64 * G rows).  Short groups (one or two 128-row blocks on average):
// the 128-row tile, which wastes nothing on them; otherwise the choice of the plain path on the estimated row
// count.  Measured on the padded full-size workloads (hot caches, K-block-major scales): many_small 1763 us with the
// 128-row tile against 1955 us with the 256 x 256 tile that the capacity alone used to select, decode 339 against
// 343 us; gate_up 266 us (224-row tile of the second kernel, the best of seven candidates), down 320 us (224 rows;
// best of seven: 300 us at 256 rows).
int pick_variant_padded(int G, int64_t M_pad_cap, int N, int K) {
  int64_t rows = M_pad_cap - 64 * (int64_t)G;
  if (rows < 128) rows = M_pad_cap;
  if (N % 256 == 0 && K % 128 == 0 && G > 0 && rows / G < 320) return 3;
  return pick_variant(G, rows, N, K);
}

// Grid of the row kernels (a workgroup takes rows in pairs).  With K-block-major scales and at least 8 workgroups the
// pairs are dealt out by XCD (see pair_of in quant_kernel.h), which needs a grid that is a multiple of 8.
int64_t row_kernel_grid(int64_t M_total, bool kmajor, int* by_xcd) {
  int64_t grid = (int64_t)device_cus() * 8;
  const int64_t npairs = (M_total + 1) / 2;
  if (grid > npairs) grid = npairs;
  *by_xcd = 0;
  if (kmajor && grid >= kXcds) {
    grid -= grid % kXcds;
    *by_xcd = 1;
  }
  return grid < 1 ? 1 : grid;
}

// Device scratch a GEMM call with this variant uses: the split-K variants keep the fp32 partial sums of the two
// halves of the K loop, [2][M_total][N]; the others nothing.
size_t workspace_need(int variant, int64_t M_total, int N) {
  if (variant < 0 || variant >= kNumVariants || !kVariants[variant].splitk) return 0;
  return (size_t)2 * (size_t)M_total * (size_t)N * sizeof(float);
}

// A caller's workspace: at least `need` bytes, 16-byte aligned (NULL is fine when nothing is needed).
bool workspace_ok(const void* workspace, size_t bytes, size_t need) {
  if (need == 0) return true;
  return workspace && ((uintptr_t)workspace & 15) == 0 && bytes >= need;
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
void* scratch_ptr() {
  static std::atomic<void*> cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  void* p = cache[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  cache[dev].store(p, std::memory_order_release);
  return p;
}

int validate_gemm(const void* A, const float* SA, const void* B, const float* SB, const int32_t* off, void* C,
                  int G, int64_t M_total, int N, int K) {
  if (G < 0 || M_total < 0 || N <= 0 || K <= 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || N > (1 << 21) || K > (1 << 22)) return GG_ERR_SHAPE;
  if (N % 8 != 0 || K % 16 != 0) return GG_ERR_UNSUPPORTED;    // 16-byte stores of C, 16-byte fetches of A and B
  if (G == 0 || M_total == 0) return GG_OK;
  if (!A || !SA || !B || !SB || !off || !C) return GG_ERR_NULL;
  return GG_OK;
}

int run_gemm(const void* A, const float* SA, const void* B, const float* SB, const int32_t* off, void* C,
             int G, int64_t M_total, int N, int K, void* workspace, size_t workspace_bytes, void* stream, int variant,
             unsigned flags = 0) {
  if (flags & ~(unsigned)(GG_OUT_F16 | GG_SA_KMAJOR | GG_PADDED_GROUPS)) return GG_ERR_UNSUPPORTED;
  int st = validate_gemm(A, SA, B, SB, off, C, G, M_total, N, K);
  if (st != GG_OK) return st;
  if (G == 0 || M_total == 0) return GG_OK;
  if (variant >= kNumVariants) return GG_ERR_UNSUPPORTED;
  if (variant < 0) variant = (flags & GG_PADDED_GROUPS) ? pick_variant_padded(G, M_total, N, K) : pick_variant(G, M_total, N, K);
  const Variant& v = kVariants[variant];
  // split-K: an even number of K blocks, whole tiles, offsets of the partial sums within 32 bits
  if (v.splitk && (K % 256 != 0 || N % v.BN != 0 || N > (1 << 20))) return GG_ERR_UNSUPPORTED;
  if (!workspace_ok(workspace, workspace_bytes, workspace_need(variant, M_total, N))) return GG_ERR_WORKSPACE;
  // the instantiation for partial tiles and a short last K block; in the second kernel it is also the one that takes
  // an odd number of K blocks
  const bool ragged = N % v.BN != 0 || K % 128 != 0 || (v.min_kb3 && (((K + 127) / 128) & 1));
  if (ragged && !v.launch_ragged) return GG_ERR_UNSUPPORTED;   // this variant takes whole tiles and whole K blocks only
  // the second kernel's prologue fetches three K blocks (an odd number of K blocks is fine: it adds one empty step)
  if (v.min_kb3 && K <= 256) return GG_ERR_UNSUPPORTED;

  gg::GemmArgs args;
  args.A = static_cast<const uint8_t*>(A);
  args.SA = SA;
  args.B = static_cast<const uint8_t*>(B);
  args.SB = SB;
  args.off = off;
  args.C = static_cast<uint16_t*>(C);
  args.G = G;
  args.M_total = (int)M_total;
  args.N = N;
  args.K = K;
  args.KB = (K + 127) / 128;
  args.k_rem = K - 128 * (args.KB - 1);
  args.n_tiles = (N + v.BN - 1) / v.BN;
  args.n_chunk = args.n_tiles < 8 ? args.n_tiles : 8;
  args.A2 = nullptr;
  args.SA2 = nullptr;
  args.act_out = nullptr;
  args.sa2_row_stride = args.sa2_kb_stride = 0;
  args.out_f16 = (flags & GG_OUT_F16) ? 1 : 0;
  if (flags & GG_SA_KMAJOR) {
    // the K-block part of a scale's address travels in a 32-bit scalar offset
    if (M_total * 4 * (int64_t)args.KB > 0x7FFFFFFFLL) return GG_ERR_SHAPE;
    args.sa_row_stride = 4;
    args.sa_kb_stride = (int)(M_total * 4);
    args.sa_kmajor = 1;
  } else {
    args.sa_kmajor = 0;
    args.sa_row_stride = 4 * args.KB;
    args.sa_kb_stride = 4;
  }
  args.rot_mul = (K % 8192 == 4096) ? 4 : 0;   // 7 * 4 < K / 128; a function of K alone (see k_rotation)

  // upper bound on the number of tiles for any offsets: every group adds at most one partial m-tile
  const int64_t max_tiles = (M_total / v.BM + G) * (int64_t)args.n_tiles * (v.splitk ? 2 : 1);   // split-K: two units per tile
  if (max_tiles > 0x7FFFFFFFLL) return GG_ERR_SHAPE;   // the kernels count tiles in 32 bits
  args.P = v.splitk ? static_cast<float*>(workspace) : nullptr;
  int64_t grid = (int64_t)device_cus() * v.wg_per_cu;
  if (grid > max_tiles) grid = max_tiles;
  if (grid < 1) grid = 1;
  if (grid >= kXcds) {
    grid -= grid % kXcds;
    args.slots = (int)(grid / kXcds);
  } else {
    args.slots = 0;
  }
  // groups of at most one row tile on average: every weight byte is fetched once, and streamed past the L2
  const bool bstream = !ragged && v.launch_bstream && M_total <= (int64_t)G * v.BM;
  hipError_t e = (ragged ? v.launch_ragged : bstream ? v.launch_bstream : v.launch)(args, (int)grid, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return GG_ERR_HIP;
  if (v.splitk) {
    const int64_t groups8 = M_total * (int64_t)(N / 8);
    int64_t cgrid = (groups8 + 255) / 256;
    if (cgrid > (int64_t)device_cus() * 8) cgrid = (int64_t)device_cus() * 8;
    hipLaunchKernelGGL(gg::gg_splitk_combine_kernel, dim3((unsigned)cgrid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       args.P, off, args.C, G, (int)M_total, N, args.out_f16);
    if (hipGetLastError() != hipSuccess) return GG_ERR_HIP;
  }
  return GG_OK;
}

}  // namespace

extern "C" {

int gg_fp8_version(void) { return kVersion; }

const char* gg_fp8_status_str(int status) {
  switch (status) {
    case GG_OK: return "ok";
    case GG_ERR_NULL: return "a required pointer is NULL";
    case GG_ERR_SHAPE: return "invalid or overflowing size argument";
    case GG_ERR_UNSUPPORTED: return "unsupported shape (N must be a multiple of 8 and K of 16; some variants and the row kernels need multiples of 128) or variant";
    case GG_ERR_WORKSPACE: return "workspace too small";
    case GG_ERR_HIP: return "HIP runtime error";
    case GG_ERR_OFFSETS: return "group offsets are not non-decreasing within [0, M_total]";
    default: return "unknown status";
  }
}

size_t gg_fp8_workspace_bytes(int G, int64_t M_total, int N, int K) {
  return gg_fp8_workspace_bytes_variant(G, M_total, N, K, -1);
}

size_t gg_fp8_workspace_bytes_variant(int G, int64_t M_total, int N, int K, int variant) {
  if (G <= 0 || M_total <= 0 || N <= 0 || K <= 0 || M_total > 0x7FFFFFFFLL || N % 8 != 0 || K % 16 != 0) return 0;
  if (variant < 0) variant = pick_variant(G, M_total, N, K);
  return workspace_need(variant, M_total, N);
}

int gg_fp8_num_variants(void) { return kNumVariants; }

const char* gg_fp8_variant_name(int variant) {
  return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

int gg_fp8_auto_variant(int G, int64_t M_total, int N, int K) {
  if (G < 0 || M_total < 0 || N <= 0 || K <= 0) return -GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || N > (1 << 21) || K > (1 << 22)) return -GG_ERR_SHAPE;
  if (N % 8 != 0 || K % 16 != 0) return -GG_ERR_UNSUPPORTED;
  return pick_variant(G, M_total, N, K);
}

int gg_fp8_auto_variant_padded(int G, int64_t M_pad_cap, int N, int K) {
  if (G < 0 || M_pad_cap < 0 || N <= 0 || K <= 0) return -GG_ERR_SHAPE;
  if (M_pad_cap > 0x7FFFFFFFLL || N > (1 << 21) || K > (1 << 22)) return -GG_ERR_SHAPE;
  if (N % 8 != 0 || K % 16 != 0) return -GG_ERR_UNSUPPORTED;
  return pick_variant_padded(G, M_pad_cap, N, K);
}

int gg_fp8_grouped_gemm_variant(const void* A, const float* SA, const void* B, const float* SB,
                                const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                                void* workspace, size_t workspace_bytes, void* stream, int variant) {
  return run_gemm(A, SA, B, SB, group_offsets, C, G, M_total, N, K, workspace, workspace_bytes, stream, variant);
}

int gg_fp8_grouped_gemm(const void* A, const float* SA, const void* B, const float* SB,
                        const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                        void* workspace, size_t workspace_bytes, void* stream) {
  return gg_fp8_grouped_gemm_variant(A, SA, B, SB, group_offsets, C, G, M_total, N, K, workspace, workspace_bytes,
                                     stream, -1);
}

int gg_fp8_grouped_gemm_f16(const void* A, const float* SA, const void* B, const float* SB,
                            const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                            void* workspace, size_t workspace_bytes, void* stream, int variant) {
  return run_gemm(A, SA, B, SB, group_offsets, C, G, M_total, N, K, workspace, workspace_bytes, stream, variant, GG_OUT_F16);
}

int gg_fp8_grouped_gemm_ex(const void* A, const float* SA, const void* B, const float* SB,
                           const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                           void* workspace, size_t workspace_bytes, void* stream, int variant, unsigned flags) {
  return run_gemm(A, SA, B, SB, group_offsets, C, G, M_total, N, K, workspace, workspace_bytes, stream, variant, flags);
}

int gg_fp8_grouped_gemm_splitk_noalloc(const void* A, const float* SA, const void* B, const float* SB,
                                       const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                                       void* stream, int variant, unsigned flags) {
  if (variant < 0) variant = kDefaultSplitK;
  if (variant >= kNumVariants || !kVariants[variant].splitk) return GG_ERR_UNSUPPORTED;
  if (flags & GG_PADDED_GROUPS) return GG_ERR_UNSUPPORTED;
  int st = validate_gemm(A, SA, B, SB, group_offsets, C, G, M_total, N, K);
  if (st != GG_OK) return st;
  if (G == 0 || M_total == 0) return GG_OK;
  if (workspace_need(variant, M_total, N) > kScratchBytes) return GG_ERR_WORKSPACE;   // beyond the built-in scratch
  void* ptr = scratch_ptr();
  if (!ptr) return GG_ERR_HIP;
  return run_gemm(A, SA, B, SB, group_offsets, C, G, M_total, N, K, ptr, kScratchBytes, stream, variant, flags);
}

size_t gg_fp8_noalloc_max_elements(void) { return kScratchBytes / (2 * sizeof(float)); }

int gg_fp8_grouped_gemm_wgrad_ex(const void* XT, const float* SX, const void* DYT, const float* SDY,
                                 const int32_t* group_offsets, void* dW, int G, int64_t M_total, int N, int K, void* stream,
                                 unsigned flags) {
  if (flags & ~(unsigned)GG_OUT_BF16) return GG_ERR_UNSUPPORTED;
  const bool out16 = (flags & GG_OUT_BF16) != 0;
  if (G < 0 || M_total < 0 || N <= 0 || K <= 0) return GG_ERR_SHAPE;
  // whole output tiles of 256 features x 128 rows of dY^T; a row pitch that keeps every 128-token block 16-byte aligned
  if (M_total % 16 != 0 || N % gg::WgradCfg::TN != 0 || K % gg::WgradCfg::TK != 0) return GG_ERR_UNSUPPORTED;
  // the operands are addressed with 32-bit offsets from the start of each tensor, an output tile with 32-bit
  // offsets from its first element
  if (K > (1 << 20) || (int64_t)K * M_total > 0x7FFFFFFFLL || (int64_t)N * M_total > 0x7FFFFFFFLL) return GG_ERR_SHAPE;
  if (G == 0) return GG_OK;
  if (!group_offsets || !dW) return GG_ERR_NULL;
  if (M_total > 0 && (!XT || !SX || !DYT || !SDY)) return GG_ERR_NULL;
  const int64_t tiles = (int64_t)G * (N / gg::WgradCfg::TN) * (K / gg::WgradCfg::TK);
  if (tiles > 0x7FFFFFFFLL) return GG_ERR_SHAPE;
  gg::WgradArgs args;
  args.XT = static_cast<const uint8_t*>(XT);
  args.SX = SX;
  args.DYT = static_cast<const uint8_t*>(DYT);
  args.SDY = SDY;
  args.off = group_offsets;
  args.dW = static_cast<float*>(dW);
  args.G = G;
  args.M_total = (int)M_total;
  args.N = N;
  args.K = K;
  args.MB = (int)((M_total + 127) / 128);
  args.n_tiles = N / gg::WgradCfg::TN;
  args.k_tiles = K / gg::WgradCfg::TK;
  args.tiles = (int)tiles;
  args.blocked = args.k_tiles % 4 == 0 && args.n_tiles % 8 == 0;
  int64_t grid = device_cus();
  if (grid > tiles) grid = tiles;
  if (grid >= kXcds) {
    grid -= grid % kXcds;
    args.slots = (int)(grid / kXcds);
  } else {
    args.slots = 0;
  }
  static std::atomic<int> prepared[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return GG_ERR_HIP;
  if (dev >= 0 && dev < 64 && !prepared[dev].load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gg::gg_wgrad_kernel<0, false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            gg::WgradCfg::LDS_BYTES) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(&gg::gg_wgrad_kernel<0, true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            gg::WgradCfg::LDS_BYTES) != hipSuccess)
      return GG_ERR_HIP;
    prepared[dev].store(1, std::memory_order_release);
  }
  if (out16)
    hipLaunchKernelGGL((gg::gg_wgrad_kernel<0, true>), dim3((unsigned)grid), dim3(gg::WgradCfg::NT), gg::WgradCfg::LDS_BYTES,
                       static_cast<hipStream_t>(stream), args);
  else
    hipLaunchKernelGGL((gg::gg_wgrad_kernel<0, false>), dim3((unsigned)grid), dim3(gg::WgradCfg::NT), gg::WgradCfg::LDS_BYTES,
                       static_cast<hipStream_t>(stream), args);
  return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int gg_fp8_grouped_gemm_wgrad(const void* XT, const float* SX, const void* DYT, const float* SDY,
                              const int32_t* group_offsets, float* dW, int G, int64_t M_total, int N, int K, void* stream) {
  return gg_fp8_grouped_gemm_wgrad_ex(XT, SX, DYT, SDY, group_offsets, dW, G, M_total, N, K, stream, 0);
}

int gg_fp8_grouped_gemm_swiglu(const void* A, const float* SA, const void* B, const float* SB,
                               const int32_t* group_offsets, void* A2, float* SA2, void* act_out,
                               int G, int64_t M_total, int I, int K, void* stream, int variant, unsigned flags) {
  if (flags & ~(unsigned)GG_SA_KMAJOR) return GG_ERR_UNSUPPORTED;
  if (G < 0 || M_total < 0 || I <= 0 || K <= 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || I > (1 << 20) || K > (1 << 22)) return GG_ERR_SHAPE;
  // whole 128-column blocks of activations and whole K blocks; the second kernel's prologue fetches three K blocks
  if (I % 128 != 0 || K % 128 != 0 || K <= 256) return GG_ERR_UNSUPPORTED;
  if ((int64_t)2 * I * K > 0x7FFFFFFFLL) return GG_ERR_SHAPE;       // an expert's weights are addressed with 32-bit offsets
  if (G == 0 || M_total == 0) return GG_OK;
  if (!A || !SA || !B || !SB || !group_offsets || !A2 || !SA2) return GG_ERR_NULL;
  const int N = 2 * I;
  const FusedVariant* fv = nullptr;
  const bool odd_kb = ((K / 128) & 1) != 0;
  if (variant < 0 && odd_kb) {
    fv = &kFused[0];
  } else if (variant < 0) {
    // the cheapest of the three tile heights under the cost model of the automatic choice
    double c_best = 0;
    const double eff[3] = {1.06, 1.08, 1.10};
    for (int i = 0; i < 3; ++i) {
      const double rounds = ((double)M_total / kFused[i].BM + 0.5 * G) * (I / 128) / 256.0;
      const double whole = std::floor(rounds), frac = rounds - whole;
      const double c = (whole + (frac > 1e-9 ? 0.3 + 0.7 * frac : 0.0)) * kFused[i].BM / eff[i];
      if (!fv || c < c_best) { c_best = c; fv = &kFused[i]; }
    }
  } else {
    for (const FusedVariant& f : kFused)
      if (f.variant == variant) fv = &f;
    if (!fv || (odd_kb && !fv->launch_odd)) return GG_ERR_UNSUPPORTED;
  }
  gg::GemmArgs args;
  args.A = static_cast<const uint8_t*>(A);
  args.SA = SA;
  args.B = static_cast<const uint8_t*>(B);
  args.SB = SB;
  args.off = group_offsets;
  args.C = nullptr;
  args.G = G;
  args.M_total = (int)M_total;
  args.N = N;
  args.K = K;
  args.KB = K / 128;
  args.k_rem = 128;
  args.n_tiles = I / 128;
  args.n_chunk = args.n_tiles < 8 ? args.n_tiles : 8;
  args.out_f16 = 0;
  args.rot_mul = 0;      // a tile holds columns of two far-apart column blocks: every K loop starts at block 0
  const bool km = (flags & GG_SA_KMAJOR) != 0;
  if (km && M_total * 4 * (int64_t)args.KB > 0x7FFFFFFFLL) return GG_ERR_SHAPE;
  args.sa_row_stride = km ? 4 : 4 * args.KB;
  args.sa_kb_stride = km ? (int)(M_total * 4) : 4;
  args.sa_kmajor = km ? 1 : 0;
  args.P = nullptr;
  args.A2 = static_cast<uint8_t*>(A2);
  args.SA2 = SA2;
  args.act_out = static_cast<uint16_t*>(act_out);
  args.sa2_row_stride = km ? 1 : I / 128;
  args.sa2_kb_stride = km ? M_total : 1;
  const int64_t max_tiles = (M_total / fv->BM + G) * (int64_t)args.n_tiles;
  if (max_tiles > 0x7FFFFFFFLL) return GG_ERR_SHAPE;
  int64_t grid = device_cus();
  if (grid > max_tiles) grid = max_tiles;
  if (grid < 1) grid = 1;
  if (grid >= kXcds) {
    grid -= grid % kXcds;
    args.slots = (int)(grid / kXcds);
  } else {
    args.slots = 0;
  }
  return (odd_kb ? fv->launch_odd : fv->launch)(args, (int)grid, static_cast<hipStream_t>(stream)) == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int64_t gg_fp8_padded_rows_cap(int G, int64_t M_total) {
  if (G < 0 || M_total < 0) return 0;
  return 128 * ((M_total + 127) / 128 + (int64_t)G);
}

int gg_fp8_pad_ex(const void* A, const float* SA, const int32_t* group_offsets, void* A_pad, float* SA_pad,
                  int32_t* padded_offsets, int G, int64_t M_total, int64_t M_pad_cap, int K, void* stream, unsigned flags) {
  if (flags & ~(unsigned)GG_SA_KMAJOR) return GG_ERR_UNSUPPORTED;
  if (G < 0 || M_total < 0 || K <= 0 || M_pad_cap < 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || M_pad_cap > 0x7FFFFFFFLL || K > (1 << 22)) return GG_ERR_SHAPE;
  if (M_pad_cap < gg_fp8_padded_rows_cap(G, M_total)) return GG_ERR_SHAPE;
  if (K % 16 != 0) return GG_ERR_UNSUPPORTED;
  if (!padded_offsets || !group_offsets) return GG_ERR_NULL;
  if (M_pad_cap > 0 && (!A_pad || !SA_pad)) return GG_ERR_NULL;
  if (M_total > 0 && (!A || !SA)) return GG_ERR_NULL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(gg::gg_pad_offsets_kernel, dim3(1), dim3(gg::PAD_THREADS), 0, s, group_offsets, padded_offsets, G,
                     (int)M_total);
  if (hipGetLastError() != hipSuccess) return GG_ERR_HIP;
  if (M_pad_cap == 0) return GG_OK;
  const int64_t nblocks = (M_pad_cap + gg::PAD_BLOCK_ROWS - 1) / gg::PAD_BLOCK_ROWS;
  int64_t grid = (int64_t)device_cus() * 8;
  if (grid > nblocks) grid = nblocks;
  hipLaunchKernelGGL(gg::gg_pad_rows_kernel, dim3((unsigned)grid), dim3(gg::PAD_THREADS), 0, s,
                     static_cast<const uint8_t*>(A), SA, group_offsets, padded_offsets, static_cast<uint8_t*>(A_pad),
                     SA_pad, G, (int)M_total, (int)M_pad_cap, K, (K + 127) / 128, (flags & GG_SA_KMAJOR) ? 1 : 0);
  return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int gg_fp8_pad(const void* A, const float* SA, const int32_t* group_offsets, void* A_pad, float* SA_pad,
               int32_t* padded_offsets, int G, int64_t M_total, int64_t M_pad_cap, int K, void* stream) {
  return gg_fp8_pad_ex(A, SA, group_offsets, A_pad, SA_pad, padded_offsets, G, M_total, M_pad_cap, K, stream, 0);
}

int gg_fp8_grouped_gemm_padded(const void* A_pad, const float* SA_pad, const void* B, const float* SB,
                               const int32_t* padded_offsets, void* C_pad, int G, int64_t M_pad_cap, int N, int K,
                               void* workspace, size_t workspace_bytes, void* stream) {
  return run_gemm(A_pad, SA_pad, B, SB, padded_offsets, C_pad, G, M_pad_cap, N, K, workspace, workspace_bytes, stream, -1,
                  GG_PADDED_GROUPS);
}

int gg_fp8_unpad(const void* C_pad, const int32_t* group_offsets, const int32_t* padded_offsets, void* C, int G,
                 int64_t M_total, int N, void* stream) {
  if (G < 0 || M_total < 0 || N <= 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || N > (1 << 21)) return GG_ERR_SHAPE;
  if (N % 8 != 0) return GG_ERR_UNSUPPORTED;
  if (G == 0 || M_total == 0) return GG_OK;
  if (!C_pad || !group_offsets || !padded_offsets || !C) return GG_ERR_NULL;
  const int64_t nblocks = (M_total + gg::UNPAD_BLOCK_ROWS - 1) / gg::UNPAD_BLOCK_ROWS;
  int64_t grid = (int64_t)device_cus() * 8;
  if (grid > nblocks) grid = nblocks;
  hipLaunchKernelGGL(gg::gg_unpad_rows_kernel, dim3((unsigned)grid), dim3(gg::PAD_THREADS), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(C_pad), group_offsets, padded_offsets,
                     static_cast<uint16_t*>(C), G, (int)M_total, N);
  return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int gg_fp8_quantize_rows_ex(const void* X, const int32_t* row_src, void* A, float* SA, int64_t T, int64_t M_total, int K,
                            void* stream, unsigned flags) {
  if (flags & ~(unsigned)GG_SA_KMAJOR) return GG_ERR_UNSUPPORTED;
  if (T < 0 || M_total < 0 || K <= 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || T > 0x7FFFFFFFLL || K > (1 << 22)) return GG_ERR_SHAPE;
  if (K % 128 != 0) return GG_ERR_UNSUPPORTED;
  if (M_total == 0) return GG_OK;
  if (!A || !SA || (!X && T > 0)) return GG_ERR_NULL;
  int by_xcd = 0;
  const int64_t grid = row_kernel_grid(M_total, (flags & GG_SA_KMAJOR) != 0, &by_xcd);
  hipLaunchKernelGGL(gg::gg_quantize_rows_kernel, dim3((unsigned)grid), dim3(gg::Q_THREADS), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(X), row_src,
                     static_cast<uint8_t*>(A), SA, T, (int)M_total, K, K / 128,
                     (flags & GG_SA_KMAJOR) ? (int64_t)1 : (int64_t)(K / 128), (flags & GG_SA_KMAJOR) ? M_total : (int64_t)1,
                     by_xcd);
  return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int gg_fp8_quantize_rows(const void* X, const int32_t* row_src, void* A, float* SA, int64_t T, int64_t M_total, int K,
                         void* stream) {
  return gg_fp8_quantize_rows_ex(X, row_src, A, SA, T, M_total, K, stream, 0);
}

int gg_fp8_swiglu_quantize_rows_ex(const void* H, void* A, float* SA, void* act_out, int64_t M_total, int I, void* stream,
                                   unsigned flags) {
  if (flags & ~(unsigned)GG_SA_KMAJOR) return GG_ERR_UNSUPPORTED;
  if (M_total < 0 || I <= 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || I > (1 << 21)) return GG_ERR_SHAPE;
  if (I % 128 != 0) return GG_ERR_UNSUPPORTED;
  if (M_total == 0) return GG_OK;
  if (!H || !A || !SA) return GG_ERR_NULL;
  int by_xcd = 0;
  const int64_t grid = row_kernel_grid(M_total, (flags & GG_SA_KMAJOR) != 0, &by_xcd);
  hipLaunchKernelGGL(gg::gg_swiglu_quantize_rows_kernel, dim3((unsigned)grid), dim3(gg::Q_THREADS), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(H), static_cast<uint8_t*>(A), SA,
                     static_cast<uint16_t*>(act_out), (int)M_total, I, I / 128,
                     (flags & GG_SA_KMAJOR) ? (int64_t)1 : (int64_t)(I / 128), (flags & GG_SA_KMAJOR) ? M_total : (int64_t)1,
                     by_xcd);
  return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int gg_fp8_swiglu_quantize_rows(const void* H, void* A, float* SA, void* act_out, int64_t M_total, int I, void* stream) {
  return gg_fp8_swiglu_quantize_rows_ex(H, A, SA, act_out, M_total, I, stream, 0);
}

int gg_fp8_quantize_cols(const void* X, const int32_t* row_src, void* XT, float* SX, int64_t T, int64_t M_total, int K,
                         void* stream) {
  if (T < 0 || M_total < 0 || K <= 0) return GG_ERR_SHAPE;
  if (M_total > 0x7FFFFFFFLL || T > 0x7FFFFFFFLL || K > (1 << 22)) return GG_ERR_SHAPE;
  // tiles of 64 features; a row pitch of XT that keeps every 16-byte piece aligned (what the weight-gradient GEMM asks too)
  if (K % gg::QC_FEATS != 0 || M_total % 16 != 0) return GG_ERR_UNSUPPORTED;
  if (M_total == 0) return GG_OK;
  if (!XT || !SX || (!X && T > 0)) return GG_ERR_NULL;
  const int64_t mb = (M_total + 127) / 128;
  const int64_t tiles = mb * (K / gg::QC_FEATS);
  int64_t grid = (int64_t)device_cus() * 5;      // five workgroups fit a compute unit (registers); each walks its tiles with the next one's rows in flight
  if (grid > tiles) grid = tiles;
  hipLaunchKernelGGL(gg::gg_quantize_cols_kernel, dim3((unsigned)grid), dim3(gg::Q_THREADS), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(X), row_src,
                     static_cast<uint8_t*>(XT), SX, T, (int)M_total, K, (int)mb);
  return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP;
}

int gg_fp8_check_offsets(const int32_t* group_offsets, int G, int64_t M_total, void* stream) {
  if (G < 0 || M_total < 0) return GG_ERR_SHAPE;
  if (!group_offsets) return GG_ERR_NULL;
  std::vector<int32_t> host((size_t)G + 1);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(host.data(), group_offsets, host.size() * sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess)
    return GG_ERR_HIP;
  if (hipStreamSynchronize(s) != hipSuccess) return GG_ERR_HIP;
  if (host[0] < 0 || (int64_t)host[G] > M_total) return GG_ERR_OFFSETS;
  for (int g = 0; g < G; ++g)
    if (host[g + 1] < host[g]) return GG_ERR_OFFSETS;
  return GG_OK;
}

}  // extern "C"
