// C ABI and host-side dispatch of the per-layer DP weight-gradient library (see include/flashdp.h).
// Host code only validates, sizes the workspace, picks kernels and enqueues them; every step of
// Algorithm 1 runs in the kernels.
#include "../../include/flashdp.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <map>
#include <mutex>
#include <vector>

#include "elementwise.hip.h"
#include "gemm_mfma.hip.h"
#include "gemm_mfma_dma.hip.h"
#include "gemm_mfma_dma_shaped.hip.h"
#include "gemm_mfma_dma16.hip.h"
#include "gemm_mfma_f32.hip.h"
#include "gemm_mfma_streamk.hip.h"
#include "fused_dp.hip.h"
#include "gemm_simple.hip.h"
#include "gram_norm.hip.h"
#include "mfma_probe.hip.h"

using namespace flashdp;

// Working memory of flashdp_linear_dp_grad_static: the per-layer workspace of the scratch schedule (clip
// factors, per-workgroup norm partials, the parked per-sample tiles) in device memory that comes with the
// code object, so that the entry point never allocates.  Every device the library is loaded on holds its own
// copy at its own address until the process ends.  In host code the name below only stands for the symbol:
// the address kernels are given comes from hipGetSymbolAddress, once per device (static_scratch_ptr).
#define FLASHDP_STATIC_SCRATCH_BYTES (size_t(64) << 20)
static __device__ __align__(256) unsigned char scratch[FLASHDP_STATIC_SCRATCH_BYTES];

namespace {

struct Context {
  hipStream_t stream = nullptr;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  int dtype = FLASHDP_BF16;
  uint32_t layer = 0;
  int schedule = FLASHDP_SCHEDULE_AUTO;
  int stages = FLASHDP_STAGE_ALL;
  const char* last_schedule = "none";
  const char* last_kernel = "none";
  int64_t last_chunk = 0;
};
thread_local Context g_ctx;

struct OwnedWs { void* ptr = nullptr; size_t bytes = 0; };
std::mutex g_ws_mutex;
std::map<int, OwnedWs> g_owned;   // device -> library-owned workspace

// Per-device second stream and events of the overlapped schedule (default priority, created on first use).
struct SideStream {
  hipStream_t stream = nullptr;
  std::vector<hipEvent_t> ready, done;   // per layer slot: contraction done / aggregation done
};
std::map<int, SideStream> g_side;
std::mutex g_side_mutex;

std::mutex g_static_mutex;
std::map<int, void*> g_static_ptr;   // device -> address of that device's copy of `scratch`

// Device address of the current device's copy of the static scratch (looked up once per device).
int static_scratch_ptr(int dev, char** ptr) {
  std::lock_guard<std::mutex> lock(g_static_mutex);
  auto it = g_static_ptr.find(dev);
  if (it == g_static_ptr.end()) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) { (void)hipGetLastError(); return FLASHDP_HIP_ERROR; }
    it = g_static_ptr.emplace(dev, p).first;
  }
  *ptr = static_cast<char*>(it->second);
  return FLASHDP_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool valid_dtype(int d) { return d == FLASHDP_BF16 || d == FLASHDP_F32 || d == FLASHDP_F16; }
inline bool valid_schedule(int s) { return s >= FLASHDP_SCHEDULE_AUTO && s <= FLASHDP_SCHEDULE_FUSED; }
inline size_t elt_bytes(int dtype) { return dtype == FLASHDP_F32 ? 4 : 2; }

// ---- kernel plans --------------------------------------------------------------------------------

using Cfg256x8 = TileCfg<256, 256, 64, 2, 4>;   // 8 waves, 128x64 per wave
using Cfg128x4 = TileCfg<128, 128, 64, 2, 2>;   // 4 waves, 64x64 per wave
using Cfg256x8k32 = TileCfg<256, 256, 32, 2, 4>; // 8 waves, 32-deep k-tiles (half the LDS)

using CfgDma = DmaCfg<4>;                        // 8 waves, 32-deep k-tiles loaded straight into 4 LDS stages
using CfgDma384x192 = ShapedCfg<384, 192, 4, 2, 4>;   // the same pipeline, 8 waves of 96x96
using CfgDma192x384 = ShapedCfg<192, 384, 2, 4, 4>;

enum Path { PATH_SIMPLE = 0, PATH_256x8 = 2, PATH_128x4 = 3, PATH_256x8k32 = 4, PATH_F32 = 5, PATH_DMA = 6,
            PATH_DMA_384x192 = 7, PATH_DMA_192x384 = 8, PATH_DMA16 = 9 };

struct Plan {
  Path path;         // per-sample passes (norm, spill)
  Path accum_path;   // batch-accumulating pass (second pass of the two-pass schedule, plain gradient)
  int bm, bn;
  int tiles_m, tiles_n;
  int accum_tiles_m, accum_tiles_n;   // the accumulating pass has one workgroup per tile (not per sample and tile)
};

// Environment overrides (measurement aids).  Read once per process, at the first call that needs them; with
// FLASHDP_DEBUG_ENV=1 in the environment at that moment they are read again at every call instead (the test
// suite switches kernels and schedules between calls this way).
struct EnvOverrides { int tile = 0; int overlap_grid = 0; int schedule = -1; };

int parse_schedule_name(const char* s) {
  if (!s || !*s) return -1;
  if (!std::strcmp(s, "twopass")) return FLASHDP_SCHEDULE_TWOPASS;
  if (!std::strcmp(s, "scratch")) return FLASHDP_SCHEDULE_SCRATCH;
  if (!std::strcmp(s, "explicit")) return FLASHDP_SCHEDULE_EXPLICIT;
  if (!std::strcmp(s, "overlap")) return FLASHDP_SCHEDULE_OVERLAP;
  if (!std::strcmp(s, "ghost")) return FLASHDP_SCHEDULE_GHOST;
  if (!std::strcmp(s, "fused")) return FLASHDP_SCHEDULE_FUSED;
  return -1;
}

EnvOverrides read_env() {
  EnvOverrides e;
  const char* s = std::getenv("FLASHDP_TILE");
  if (s && *s) e.tile = std::atoi(s);
  s = std::getenv("FLASHDP_OVERLAP_GRID");
  if (s && *s) e.overlap_grid = std::atoi(s);
  e.schedule = parse_schedule_name(std::getenv("FLASHDP_SCHEDULE"));
  return e;
}

EnvOverrides env() {
  static std::once_flag once;
  static EnvOverrides cached;
  static bool live = false;
  std::call_once(once, [] {
    const char* d = std::getenv("FLASHDP_DEBUG_ENV");
    live = d && d[0] == '1';
    cached = read_env();
  });
  return live ? read_env() : cached;
}

// Number of compute units of the current device (looked up once per device).
int device_cus() {
  static std::mutex m;
  static std::map<int, int> cus;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  std::lock_guard<std::mutex> lock(m);
  auto it = cus.find(dev);
  if (it == cus.end()) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    it = cus.emplace(dev, n).first;
  }
  return it->second;
}

Plan make_plan(int64_t B, int64_t T, int64_t P, int64_t D, int dtype) {
  Plan p;
  const bool mfma_ok = dtype != FLASHDP_F32 && P % 8 == 0 && D % 8 == 0 &&
                       (T + 320) * (P > D ? P : D) * 2 < (int64_t(1) << 31);   // incl. the parked prefetches past the end
  // fp32 inputs: fp32 matrix-core kernel when rows are 16-byte multiples and the problem spans a few tiles
  const bool f32_ok = dtype == FLASHDP_F32 && P % 4 == 0 && D % 4 == 0 && P * D >= 128 * 128 &&
                      (T + 48) * (P > D ? P : D) * 4 < (int64_t(1) << 31) && env().tile != -1;
  if (f32_ok) {
    p.path = p.accum_path = PATH_F32; p.bm = p.bn = 256;
  } else if (!mfma_ok) {
    p.path = p.accum_path = PATH_SIMPLE; p.bm = 64; p.bn = 64;
  } else {
    int choice = env().tile;
    if (choice != PATH_DMA && choice != PATH_DMA16 && choice != PATH_DMA_384x192 && choice != PATH_DMA_192x384 && (choice < PATH_256x8 || choice > PATH_256x8k32))
      choice = 0;   // (-1 only switches the fp32 matrix-core kernel off)
    if (choice == 0) {
      // The 256x256 direct-to-LDS kernel unless the problem has too few such work items to occupy the chip:
      // measured on MI355X (scratch schedule, T = 1024..2048, features 768..13824, B = 1..8) it beats the
      // 128x128 register-staged kernel by 20-35 % from about 140 work items up (half the CUs busy), ties around
      // 70-130, and loses below (36 items: 160 vs 206 TFLOP/s).
      // Llama-13B block, B = 8, spill pass, N(0,1) data: 8 waves of 128x64 with 32-deep
      // k-tiles loaded straight into LDS 1.22 PFLOP/s; the same tiling with the tiles staged through
      // registers 1.07 (32-deep) resp. 1.0 (64-deep); 4 waves of 128x128 (one wave per SIMD) reached 0.96 and
      // spilled registers, and is no longer built.  The same pipeline on the 16x16x32 matrix-core instruction
      // (gemm_mfma_dma16_kernel, the default) 1.26-1.33 against 1.18-1.28 for the 32x32x16 form on the same boxes:
      // the part clocks higher on it.  The other kernels stay selectable (FLASHDP_TILE).
      const int64_t items = ((D + 255) / 256) * ((P + 255) / 256) * B;
      choice = items >= 128 ? PATH_DMA16 : PATH_128x4;
      if (choice == PATH_DMA16) {
        // Work items are equally long, so a per-sample pass takes ceil(items / CUs) rounds of one item each: where
        // 384x192 or 192x384 tiles (9/8 the work of a 256x256 one) need enough fewer rounds, they are taken
        // (3072 x 768 at B = 8: 288 items = 2 rounds, against 256 = 1 round of 1.125).  A clear margin is asked for:
        // the 256x256 kernel is the one tuned and measured on the large layers.
        const int64_t cus = device_cus() > 0 ? device_cus() : 256;   // sizing calls may come before a device is there
        auto rounds = [&](int64_t bm, int64_t bn) { return (((D + bm - 1) / bm) * ((P + bn - 1) / bn) * B + cus - 1) / cus; };
        const double c256 = (double)rounds(256, 256), ca = 1.125 * rounds(384, 192), cb = 1.125 * rounds(192, 384);
        if (std::min(ca, cb) <= 0.9 * c256) choice = ca <= cb ? PATH_DMA_384x192 : PATH_DMA_192x384;
      }
    }
    p.path = (Path)choice;
    p.accum_path = p.path;
    const bool shaped = p.path == PATH_DMA_384x192 || p.path == PATH_DMA_192x384;
    // the batch-accumulating pass has one workgroup per tile: it needs about the same number of 256x256 tiles by
    // itself before the large tile pays (and the shaped kernels have no such pass)
    if (shaped) p.accum_path = ((D + 255) / 256) * ((P + 255) / 256) < 128 ? PATH_128x4 : PATH_DMA16;
    if (env().tile == 0 && p.path == PATH_DMA16 && ((D + 255) / 256) * ((P + 255) / 256) < 128) p.accum_path = PATH_128x4;
    p.bm = p.bn = (p.path == PATH_128x4) ? 128 : 256;
    if (p.path == PATH_DMA_384x192) { p.bm = 384; p.bn = 192; }
    if (p.path == PATH_DMA_192x384) { p.bm = 192; p.bn = 384; }
  }
  p.tiles_m = (int)((D + p.bm - 1) / p.bm);
  p.tiles_n = (int)((P + p.bn - 1) / p.bn);
  const int abm = (p.accum_path == p.path) ? p.bm : p.accum_path == PATH_128x4 ? 128 : 256;
  const int abn = (p.accum_path == p.path) ? p.bn : p.accum_path == PATH_128x4 ? 128 : 256;
  p.accum_tiles_m = (int)((D + abm - 1) / abm);
  p.accum_tiles_n = (int)((P + abn - 1) / abn);
  return p;
}

const char* path_kernel_name(Path p) {
  switch (p) {
    case PATH_DMA: return "gemm_mfma_dma_kernel";
    case PATH_DMA16: return "gemm_mfma_dma16_kernel";
    case PATH_DMA_384x192: case PATH_DMA_192x384: return "gemm_mfma_dma_shaped_kernel";
    case PATH_F32: return "gemm_mfma_f32_kernel";
    case PATH_SIMPLE: return "gemm_simple_kernel";
    default: return "gemm_mfma_kernel";
  }
}

struct WsLayout { size_t factors, partials, scratch, total; };

// Number of squared-norm partials per sample the explicit schedule's norm kernel writes.
int explicit_chunks(int64_t P, int64_t D) {
  const int64_t c = ((int64_t)P * D + 16383) / 16384;
  return (int)(c < 1 ? 1 : (c > 2048 ? 2048 : c));
}

// Ghost-norm schedule: matrix-core Gram kernel (128-row blocks) or the generic one (64-row blocks).
bool gram_mfma_ok(int64_t T, int64_t P, int64_t D, int dtype) {
  return dtype != FLASHDP_F32 && P % 8 == 0 && D % 8 == 0 && (T + 128) * (P > D ? P : D) * 2 < (int64_t(1) << 31);
}
int64_t gram_blocks(int64_t T, int64_t P, int64_t D, int dtype) {
  const int64_t bt = gram_mfma_ok(T, P, D, dtype) ? GramCfg::BT : 64;
  return (T + bt - 1) / bt;
}

// mode: FLASHDP_SCHEDULE_TWOPASS / _GHOST (no scratch), _SCRATCH (input-width scratch), _EXPLICIT (fp32 scratch)
WsLayout ws_layout(const Plan& p, int64_t B, int64_t T, int64_t P, int64_t D, int dtype, int mode) {
  WsLayout w;
  w.factors = 0;
  w.partials = align_up((size_t)B * 4, 256);
  size_t n_part = (size_t)p.tiles_m * p.tiles_n;
  if (mode == FLASHDP_SCHEDULE_EXPLICIT) n_part = std::max(n_part, (size_t)explicit_chunks(P, D));
  if (mode == FLASHDP_SCHEDULE_GHOST) {
    const size_t nb = (size_t)gram_blocks(T, P, D, dtype);
    n_part = std::max(n_part, nb * (nb + 1) / 2);
  }
  w.scratch = w.partials + align_up((size_t)B * n_part * 4, 256);
  size_t sc = 0;
  if (mode == FLASHDP_SCHEDULE_SCRATCH) sc = (size_t)B * D * P * elt_bytes(dtype);
  if (mode == FLASHDP_SCHEDULE_EXPLICIT) sc = (size_t)B * D * P * 4;
  w.total = w.scratch + align_up(sc, 256);
  return w;
}

// Raises a kernel's dynamic-LDS limit, once per device and kernel (under a lock: any thread, any device).
hipError_t ensure_lds_limit(const void* kern, int bytes) {
  static std::mutex m;
  static std::map<std::pair<int, const void*>, bool> attr_set;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(m);
  bool& done = attr_set[std::make_pair(dev, kern)];
  if (!done) {
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done = true;
  }
  return hipSuccess;
}

// Launches one of the tiled matrix-core kernels: grid = tiles (x samples for the per-sample modes).
template <typename Cfg>
hipError_t launch_tiled(void (*kern)(GemmArgs), int mode, const GemmArgs& a, hipStream_t st, bool lockstep = false) {
  {
    hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(kern), Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
  }
  const int tiles = a.tiles_m * a.tiles_n;
  // lockstep: the per-sample grid in blocks of 32 tiles dealt to the XCDs in turn (see shared_block_item)
  const int64_t grid = (mode == MODE_ACCUM) ? tiles : lockstep ? shared_block_grid(tiles, a.B) : (int64_t)tiles * a.B;
  if (grid >= (int64_t(1) << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Cfg::NT), Cfg::LDS_BYTES, st, a);
  return hipGetLastError();
}

template <typename Cfg, int MODE, int DT>
hipError_t launch_mfma(const GemmArgs& a, hipStream_t st) {
  return launch_tiled<Cfg>(gemm_mfma_kernel<Cfg, MODE, DT>, MODE, a, st);
}

template <int MODE, int DT>
hipError_t launch_gemm_dt(const Plan& p, const GemmArgs& args, hipStream_t st) {
  GemmArgs a = args;
  if (MODE == MODE_ACCUM) { a.tiles_m = p.accum_tiles_m; a.tiles_n = p.accum_tiles_n; }
  if constexpr (DT != DT_F32) {
    switch (MODE == MODE_ACCUM ? p.accum_path : p.path) {
      case PATH_256x8: return launch_mfma<Cfg256x8, MODE, DT>(a, st);
      case PATH_128x4: return launch_mfma<Cfg128x4, MODE, DT>(a, st);
      case PATH_256x8k32: return launch_mfma<Cfg256x8k32, MODE, DT>(a, st);
      case PATH_DMA: return launch_tiled<CfgDma>(gemm_mfma_dma_kernel<CfgDma, MODE, DT>, MODE, a, st, /*lockstep=*/true);
      case PATH_DMA16: return launch_tiled<CfgDma>(gemm_mfma_dma16_kernel<CfgDma, MODE, DT>, MODE, a, st, /*lockstep=*/true);
      case PATH_DMA_384x192:
        if constexpr (MODE != MODE_ACCUM)
          return launch_tiled<CfgDma384x192>(gemm_mfma_dma_shaped_kernel<CfgDma384x192, MODE, DT>, MODE, a, st, /*lockstep=*/true);
        return hipErrorInvalidValue;
      case PATH_DMA_192x384:
        if constexpr (MODE != MODE_ACCUM)
          return launch_tiled<CfgDma192x384>(gemm_mfma_dma_shaped_kernel<CfgDma192x384, MODE, DT>, MODE, a, st, /*lockstep=*/true);
        return hipErrorInvalidValue;
      default: break;
    }
  }
  const int tiles = a.tiles_m * a.tiles_n;
  const int grid = (MODE == MODE_ACCUM) ? tiles : tiles * a.B;
  if constexpr (DT == DT_F32) {
    if (p.path == PATH_F32) return launch_tiled<F32Cfg>(gemm_mfma_f32_kernel<MODE>, MODE, a, st, /*lockstep=*/true);
  }
  hipLaunchKernelGGL((gemm_simple_kernel<MODE, DT>), dim3(grid), dim3(256), 0, st, a);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_gemm(const Plan& p, int dtype, const GemmArgs& a, hipStream_t st) {
  switch (dtype) {
    case FLASHDP_BF16: return launch_gemm_dt<MODE, DT_BF16>(p, a, st);
    case FLASHDP_F16: return launch_gemm_dt<MODE, DT_F16>(p, a, st);
    default: return launch_gemm_dt<MODE, DT_F32>(p, a, st);
  }
}

hipError_t launch_aggregate(int dtype, const void* scratch, const float* factors, int B, size_t S, float noise_scale,
                            uint64_t seed, uint32_t layer, float* out, int accumulate, hipStream_t st, int persistent_grid = 0) {
  if (persistent_grid > 0 && dtype != FLASHDP_F32 && S % 8 == 0) {
    const size_t n8 = S / 8;
    hipLaunchKernelGGL((aggregate16_persistent_kernel<DT_BF16>), dim3(persistent_grid), dim3(256), 0, st, scratch, factors, B, S, n8, noise_scale, seed, layer, out, accumulate);
    return hipGetLastError();
  }
  if (dtype != FLASHDP_F32 && S % 8 == 0) {
    const size_t n8 = S / 8;
    const unsigned grid = (unsigned)((n8 + 255) / 256);
    hipLaunchKernelGGL((aggregate16_kernel<DT_BF16>), dim3(grid), dim3(256), 0, st, scratch, factors, B, S, n8, noise_scale, seed, layer, out, accumulate);
  } else {
    const size_t groups = (S + 3) / 4;
    const unsigned grid = (unsigned)((groups + 255) / 256);
    if (dtype != FLASHDP_F32)   // the scratch of both 16-bit input types is bfloat16
      hipLaunchKernelGGL((aggregate_generic_kernel<DT_BF16>), dim3(grid), dim3(256), 0, st, scratch, factors, B, S, noise_scale, seed, layer, out, accumulate);
    else
      hipLaunchKernelGGL(aggregate32_kernel, dim3(grid), dim3(256), 0, st, (const float*)scratch, factors, B, S, noise_scale, seed, layer, out, accumulate);
  }
  return hipGetLastError();
}

hipError_t launch_gram(int dtype, bool mfma, const GramArgs& g, hipStream_t st) {
  const unsigned grid = (unsigned)((int64_t)g.B * g.n_tri);
  if (mfma) {
    auto kern = dtype == FLASHDP_BF16 ? gram_norm_mfma_kernel<DT_BF16> : gram_norm_mfma_kernel<DT_F16>;
    hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(kern), GramCfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(GramCfg::NT), GramCfg::LDS_BYTES, st, g);
  } else if (dtype == FLASHDP_BF16) {
    hipLaunchKernelGGL((gram_norm_simple_kernel<DT_BF16>), dim3(grid), dim3(256), 0, st, g);
  } else if (dtype == FLASHDP_F16) {
    hipLaunchKernelGGL((gram_norm_simple_kernel<DT_F16>), dim3(grid), dim3(256), 0, st, g);
  } else {
    hipLaunchKernelGGL((gram_norm_simple_kernel<DT_F32>), dim3(grid), dim3(256), 0, st, g);
  }
  return hipGetLastError();
}

// ---- validation ----------------------------------------------------------------------------------

int check_dims(int64_t B, int64_t T, int64_t P, int64_t D) {
  if (B <= 0 || T <= 0 || P <= 0 || D <= 0) return FLASHDP_INVALID_ARGUMENT;
  const int64_t lim = int64_t(1) << 31;
  if (B >= (1 << 20) || T >= lim || P >= lim || D >= lim) return FLASHDP_UNSUPPORTED_SHAPE;
  if (T * P >= lim || T * D >= lim) return FLASHDP_UNSUPPORTED_SHAPE;   // per-sample tensors are indexed with 32 bits
  const int64_t tiles = ((D + 63) / 64) * ((P + 63) / 64);
  if (tiles * B >= lim) return FLASHDP_UNSUPPORTED_SHAPE;              // grid size
  return FLASHDP_OK;
}

int check_layer(const flashdp_layer_t& L, int64_t B, int64_t T) {
  if (!L.X || !L.dY || !L.out_grad) return FLASHDP_INVALID_ARGUMENT;
  if (!(L.C > 0.0f) || !std::isfinite(L.C)) return FLASHDP_INVALID_ARGUMENT;
  if (!(L.sigma >= 0.0f) || !std::isfinite(L.sigma)) return FLASHDP_INVALID_ARGUMENT;
  int st = check_dims(B, T, L.d_in, L.d_out);
  if (st != FLASHDP_OK) return st;
  if (!aligned16(L.X) || !aligned16(L.dY) || !aligned16(L.out_grad) || (L.out_norms && (reinterpret_cast<uintptr_t>(L.out_norms) & 3u)))
    return FLASHDP_MISALIGNED;
  return FLASHDP_OK;
}

int device_or_error(int* dev) {
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) { (void)hipGetLastError(); return FLASHDP_NO_DEVICE; }
  if (hipGetDevice(dev) != hipSuccess) { (void)hipGetLastError(); return FLASHDP_NO_DEVICE; }
  return FLASHDP_OK;
}

int owned_workspace(size_t need, void** ptr, size_t* bytes) {
  int dev = 0;
  int st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  OwnedWs& w = g_owned[dev];
  if (w.bytes < need) {
    // Growing costs a device-wide synchronisation (earlier calls may still use the old block), a free and an
    // allocation, inside what may be a training step: grow by at least half, so that a sequence of slowly growing
    // requests (layers met in increasing size) reallocates a few times, not every time.  A caller that must not
    // stall passes its own workspace.
    const size_t want = std::max(need, w.bytes + w.bytes / 2);
    if (w.ptr) {
      if (hipDeviceSynchronize() != hipSuccess) return FLASHDP_HIP_ERROR;
      (void)hipFree(w.ptr);
      w.ptr = nullptr; w.bytes = 0;
    }
    void* p = nullptr;
    size_t got = want;
    if (hipMalloc(&p, want) != hipSuccess) {
      (void)hipGetLastError();
      got = need;
      if (hipMalloc(&p, need) != hipSuccess) { (void)hipGetLastError(); return FLASHDP_HIP_ERROR; }
    }
    w.ptr = p; w.bytes = got;
  }
  *ptr = w.ptr; *bytes = w.bytes;
  return FLASHDP_OK;
}

int resolve_schedule(int schedule) {
  const int forced = env().schedule;
  return forced >= 0 ? forced : schedule;
}

// The single-launch form needs a workgroup per 256 x 256 tile resident at the same time (one per CU: its ring takes
// most of a CU's LDS), 16-bit inputs on the matrix-core path, and clip factors for all samples in LDS.
bool fused_ok(int64_t B, int64_t T, int64_t P, int64_t D, int dtype, int cus) {
  const int64_t tiles = ((D + 255) / 256) * ((P + 255) / 256);
  return dtype != FLASHDP_F32 && P % 8 == 0 && D % 8 == 0 && B <= 16 && tiles <= cus &&
         (T + 320) * (P > D ? P : D) * 2 < (int64_t(1) << 31);
}

struct FusedWs { size_t sync, partials, scratch, total; };
FusedWs fused_ws(int64_t B, int64_t P, int64_t D) {
  const size_t tiles = (size_t)((D + 255) / 256) * ((P + 255) / 256);
  FusedWs w;
  w.sync = 0;
  w.partials = 256;
  w.scratch = w.partials + align_up((size_t)B * tiles * 8 * 4, 256);
  w.total = w.scratch + align_up((size_t)(B > 1 ? B - 1 : 0) * D * P * 2, 256);
  return w;
}

size_t layer_ws_bytes(const flashdp_layer_t& L, int64_t B, int64_t T, int dtype, int mode) {
  if (mode == FLASHDP_SCHEDULE_FUSED) {
    // a layer the single-launch form does not apply to takes the scratch schedule; without a device, assume 256 CUs
    const int cus = device_cus();
    if (fused_ok(B, T, L.d_in, L.d_out, dtype, cus > 0 ? cus : 256)) return fused_ws(B, L.d_in, L.d_out).total;
    mode = FLASHDP_SCHEDULE_SCRATCH;
  }
  const Plan p = make_plan(B, T, L.d_in, L.d_out, dtype);
  return ws_layout(p, B, T, L.d_in, L.d_out, dtype, mode).total;
}

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return FLASHDP_HIP_ERROR; } } while (0)

// Enqueues Algorithm 1 for one layer.
// `parts` restricts what is enqueued (a subset of the stage mask); persistent_grid > 0 selects the bounded
// aggregation grid of the overlapped schedule.
// Samples [s0, s0 + B) of the layer's batch are processed (B is the number of samples of THIS call: the whole
// batch, or one chunk of it when the workspace holds fewer parked samples than the batch has).
int run_layer(const flashdp_layer_t& L0, int64_t B, int64_t T, int dtype, int mode, char* ws, hipStream_t st,
              bool accumulate, bool add_noise, int parts = FLASHDP_STAGE_ALL, int persistent_grid = 0, int64_t s0 = 0) {
  flashdp_layer_t L = L0;
  L.X = static_cast<const char*>(L0.X) + (size_t)s0 * T * L0.d_in * elt_bytes(dtype);
  L.dY = static_cast<const char*>(L0.dY) + (size_t)s0 * T * L0.d_out * elt_bytes(dtype);
  if (L0.out_norms) L.out_norms = L0.out_norms + s0;
  if (mode == FLASHDP_SCHEDULE_FUSED) {
    if (g_ctx.stages == FLASHDP_STAGE_ALL && parts == FLASHDP_STAGE_ALL && fused_ok(B, T, L.d_in, L.d_out, dtype, device_cus())) {
      const FusedWs fw = fused_ws(B, L.d_in, L.d_out);
      FusedArgs f;
      f.X = L.X; f.dY = L.dY; f.B = (int)B; f.T = (int)T; f.P = (int)L.d_in; f.D = (int)L.d_out;
      f.tiles_m = (int)((L.d_out + 255) / 256); f.tiles_n = (int)((L.d_in + 255) / 256);
      f.C = L.C; f.noise_scale = add_noise ? L.sigma * L.C : 0.0f; f.seed = L.seed; f.layer = L.layer;
      f.accumulate = accumulate ? 1 : 0;
      f.sync = reinterpret_cast<unsigned int*>(ws + fw.sync);
      f.partials = reinterpret_cast<float*>(ws + fw.partials);
      f.scratch = ws + fw.scratch;
      f.out = L.out_grad; f.out_norms = L.out_norms;
      f.spin_limit = 1u << 21;   // about two seconds of 1 us naps
      auto kern = dtype == FLASHDP_BF16 ? fused_dp_kernel<DT_BF16> : fused_dp_kernel<DT_F16>;
      HIP_TRY(ensure_lds_limit(reinterpret_cast<const void*>(kern), FusedCfg::LDS_BYTES));
      hipLaunchKernelGGL(fused_sync_reset_kernel, dim3(1), dim3(64), 0, st, f.sync);
      HIP_TRY(hipGetLastError());
      hipLaunchKernelGGL(kern, dim3((unsigned)(f.tiles_m * f.tiles_n)), dim3(FusedCfg::NT), FusedCfg::LDS_BYTES, st, f);
      HIP_TRY(hipGetLastError());
      g_ctx.last_kernel = "fused_dp_kernel";
      return FLASHDP_OK;
    }
    mode = FLASHDP_SCHEDULE_SCRATCH;
  }
  const bool use_scratch = mode == FLASHDP_SCHEDULE_SCRATCH;
  const int stages = g_ctx.stages & parts;
  const int64_t P = L.d_in, D = L.d_out;
  const Plan plan = make_plan(B, T, P, D, dtype);
  const WsLayout wl = ws_layout(plan, B, T, P, D, dtype, mode);
  GemmArgs a;
  a.X = L.X; a.dY = L.dY;
  a.B = (int)B; a.T = (int)T; a.P = (int)P; a.D = (int)D;
  a.tiles_m = plan.tiles_m; a.tiles_n = plan.tiles_n;
  a.partials = reinterpret_cast<float*>(ws + wl.partials);
  a.scratch = (mode == FLASHDP_SCHEDULE_SCRATCH || mode == FLASHDP_SCHEDULE_EXPLICIT) ? (void*)(ws + wl.scratch) : nullptr;
  float* factors = reinterpret_cast<float*>(ws + wl.factors);
  a.factors = factors;
  a.out = L.out_grad;
  a.accumulate = accumulate ? 1 : 0;
  a.trace = nullptr;
  const int tiles = plan.tiles_m * plan.tiles_n;
  const size_t S = (size_t)D * P;
  const float noise_scale = add_noise ? L.sigma * L.C : 0.0f;
  g_ctx.last_kernel = path_kernel_name(plan.path);

  if (mode == FLASHDP_SCHEDULE_EXPLICIT) {
    // The explicit four-stage flow of Appendix B.2, every stage a kernel of its own with the fp32
    // per-sample gradients going through HBM in between: the comparison the fused schedules are measured against.
    float* G = reinterpret_cast<float*>(a.scratch);
    const int chunks = explicit_chunks(P, D);
    if (stages & FLASHDP_STAGE_CONTRACT) HIP_TRY(launch_gemm<MODE_MATERIALIZE>(plan, dtype, a, st));      // stage 1
    if (stages & FLASHDP_STAGE_CLIP) {
      hipLaunchKernelGGL(explicit_norm_kernel, dim3((unsigned)chunks, (unsigned)B), dim3(256), 0, st, G, S, chunks, a.partials);   // stage 2
      HIP_TRY(hipGetLastError());
      hipLaunchKernelGGL(clip_factors_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, st, a.partials, chunks, L.C, (int)B, factors, L.out_norms);
      HIP_TRY(hipGetLastError());
      hipLaunchKernelGGL(explicit_clip_kernel, dim3((unsigned)((S / 4 + 256) / 256), (unsigned)B), dim3(256), 0, st, G, S, factors);  // stage 3
      HIP_TRY(hipGetLastError());
    }
    if (stages & FLASHDP_STAGE_AGGREGATE) {
      hipLaunchKernelGGL(aggregate32_kernel, dim3((unsigned)(((S + 3) / 4 + 255) / 256)), dim3(256), 0, st, G, (const float*)nullptr, (int)B, S,
                         noise_scale, L.seed, L.layer, L.out_grad, accumulate ? 1 : 0);                                                             // stage 4
      HIP_TRY(hipGetLastError());
    }
  } else if (use_scratch) {
    if (stages & FLASHDP_STAGE_CONTRACT) HIP_TRY(launch_gemm<MODE_SPILL>(plan, dtype, a, st));
    // 16-bit scratch in whole 16-byte groups: the inter-block reduce and the clip factors are done by the streaming
    // kernel itself (one launch less per layer) when that is cheap: every workgroup reads all B * tiles partials, so
    // with the ordinary grid (one workgroup per 2048 elements) this is only done while those redundant reads stay
    // below 64 MB (a 4096 x 4096 layer: 32 MB; the Llama-13B layers would re-read 0.16-1.2 GB, and a grid bounded
    // to avoid that streams measurably slower: 191 vs 153 + 7 us per layer); the bounded grid of the overlapped
    // schedule always qualifies.
    const size_t n8_all = S / 8, full_grid = (n8_all + 255) / 256;
    const size_t agg_grid = persistent_grid > 0 ? std::min((size_t)persistent_grid, full_grid) : full_grid;
    const bool fold_clip = dtype != FLASHDP_F32 && S % 8 == 0 && B <= MAX_FUSED_CLIP_B &&
                           agg_grid * (size_t)B * tiles * 4 <= (size_t(64) << 20) &&
                           (stages & (FLASHDP_STAGE_CLIP | FLASHDP_STAGE_AGGREGATE)) == (FLASHDP_STAGE_CLIP | FLASHDP_STAGE_AGGREGATE);
    if (fold_clip) {
      auto kern = persistent_grid > 0 ? clip_aggregate16_kernel<DT_BF16, false> : clip_aggregate16_kernel<DT_BF16, true>;
      hipLaunchKernelGGL(kern, dim3((unsigned)agg_grid), dim3(256), 0, st, a.scratch, a.partials, tiles,
                         L.C, L.out_norms, (int)B, S, n8_all, noise_scale, L.seed, L.layer, L.out_grad, accumulate ? 1 : 0);
      HIP_TRY(hipGetLastError());
    } else {
      if (stages & FLASHDP_STAGE_CLIP) {
        hipLaunchKernelGGL(clip_factors_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, st, a.partials, tiles, L.C, (int)B, factors, L.out_norms);
        HIP_TRY(hipGetLastError());
      }
      if (stages & FLASHDP_STAGE_AGGREGATE)
        HIP_TRY(launch_aggregate(dtype, a.scratch, factors, (int)B, S, noise_scale, L.seed, L.layer, L.out_grad, accumulate ? 1 : 0, st, persistent_grid));
    }
  } else {
    int n_partials = tiles;
    if (mode == FLASHDP_SCHEDULE_GHOST) {
      // norms from the Gram matrices (never stored): partials[B][blocks on or above the diagonal]
      GramArgs g;
      g.X = L.X; g.dY = L.dY; g.B = (int)B; g.T = (int)T; g.P = (int)P; g.D = (int)D;
      g.nb = (int)gram_blocks(T, P, D, dtype);
      g.n_tri = g.nb * (g.nb + 1) / 2;
      g.partials = a.partials;
      n_partials = g.n_tri;
      if (stages & FLASHDP_STAGE_CONTRACT) HIP_TRY(launch_gram(dtype, gram_mfma_ok(T, P, D, dtype), g, st));
    } else if (stages & FLASHDP_STAGE_CONTRACT) {
      HIP_TRY(launch_gemm<MODE_NORM>(plan, dtype, a, st));
    }
    if (stages & FLASHDP_STAGE_CLIP) {
      hipLaunchKernelGGL(clip_factors_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, st, a.partials, n_partials, L.C, (int)B, factors, L.out_norms);
      HIP_TRY(hipGetLastError());
    }
    if (stages & FLASHDP_STAGE_AGGREGATE) HIP_TRY(launch_gemm<MODE_ACCUM>(plan, dtype, a, st));
    if ((stages & FLASHDP_STAGE_AGGREGATE) && noise_scale != 0.0f) {
      const size_t groups = (S + 3) / 4;
      hipLaunchKernelGGL((noise_kernel<true>), dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, L.out_grad, S, noise_scale, L.seed, L.layer);
      HIP_TRY(hipGetLastError());
    }
  }
  return FLASHDP_OK;
}

}  // namespace

extern "C" {

int flashdp_block_dp_grad_micro(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                                int schedule, void* workspace, size_t workspace_bytes, void* stream,
                                int accumulate, int add_noise) {
  if (!layers || n_layers <= 0 || !valid_dtype(dtype) || !valid_schedule(schedule)) return FLASHDP_INVALID_ARGUMENT;
  for (int l = 0; l < n_layers; ++l) {
    int st = check_layer(layers[l], B, T);
    if (st != FLASHDP_OK) return st;
  }
  if (workspace && !aligned16(workspace)) return FLASHDP_MISALIGNED;
  schedule = resolve_schedule(schedule);
  size_t need_scratch = 0, need_small = 0, need_explicit = 0, need_ghost = 0, need_fused = 0;
  for (int l = 0; l < n_layers; ++l) {
    need_fused = std::max(need_fused, layer_ws_bytes(layers[l], B, T, dtype, FLASHDP_SCHEDULE_FUSED));
    need_scratch = std::max(need_scratch, layer_ws_bytes(layers[l], B, T, dtype, FLASHDP_SCHEDULE_SCRATCH));
    need_small = std::max(need_small, layer_ws_bytes(layers[l], B, T, dtype, FLASHDP_SCHEDULE_TWOPASS));
    need_explicit = std::max(need_explicit, layer_ws_bytes(layers[l], B, T, dtype, FLASHDP_SCHEDULE_EXPLICIT));
    need_ghost = std::max(need_ghost, layer_ws_bytes(layers[l], B, T, dtype, FLASHDP_SCHEDULE_GHOST));
    if (schedule == FLASHDP_SCHEDULE_GHOST) {   // grid of the Gram kernel
      const int64_t nb = gram_blocks(T, layers[l].d_in, layers[l].d_out, dtype);
      if (nb > 32768 || nb * (nb + 1) / 2 * B >= (int64_t(1) << 31)) return FLASHDP_UNSUPPORTED_SHAPE;   // 32-bit block arithmetic
    }
  }
  int dev = 0;
  int st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  // The overlapped schedule needs two work items or more (layers, or sample chunks of a layer), 16-bit inputs on
  // the large-tile matrix-core path (where the aggregation is worth hiding) and the full stage mask; otherwise it is
  // the scratch schedule.
  auto overlap_fits = [&](int64_t b) {
    bool ok = dtype != FLASHDP_F32 && g_ctx.stages == FLASHDP_STAGE_ALL;
    for (int l = 0; l < n_layers && ok; ++l) {
      const Plan p = make_plan(b, T, layers[l].d_in, layers[l].d_out, dtype);
      // (not the 384x192 / 192x384 kernels: their 248 registers leave no room for an aggregation wave beside two
      // contraction waves per SIMD, and a bounded aggregation workgroup that takes a CU would keep the next
      // contraction workgroup out of it until its whole share is done)
      ok = (p.path == PATH_256x8k32 || p.path == PATH_256x8 || p.path == PATH_DMA || p.path == PATH_DMA16) && ((size_t)layers[l].d_in * layers[l].d_out) % 8 == 0;
    }
    return ok;
  };
  // workspace of the scratch schedule when b samples are parked at a time (the largest layer decides)
  auto scratch_need = [&](int64_t b) {
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) need = std::max(need, layer_ws_bytes(layers[l], b, T, dtype, FLASHDP_SCHEDULE_SCRATCH));
    return align_up(need, 256);
  };
  const bool overlap_ok = n_layers >= 2 && overlap_fits(B);
  const size_t need_overlap = 2 * scratch_need(B);
  char* ws = static_cast<char*>(workspace);
  int mode;
  int64_t chunk = B;   // samples parked at a time
  if (workspace) {
    if (schedule == FLASHDP_SCHEDULE_AUTO) {
      mode = (overlap_ok && workspace_bytes >= need_overlap) ? FLASHDP_SCHEDULE_OVERLAP
             : workspace_bytes >= need_scratch ? FLASHDP_SCHEDULE_SCRATCH : FLASHDP_SCHEDULE_TWOPASS;
      if (mode == FLASHDP_SCHEDULE_TWOPASS && B > 1 && g_ctx.stages == FLASHDP_STAGE_ALL) {
        // The workspace does not hold the whole batch: park as many samples as fit and go through the batch in
        // chunks, each chunk's clipped sum added to out_grad (what the micro-batch form does), rather than compute
        // every G_i twice.  Two slots of a smaller chunk (overlapped schedule) are taken when that chunk still has two
        // samples or more: every chunk re-reads and re-writes out_grad, so single-sample chunks cost more in traffic
        // and in small grids than hiding their aggregation saves (up_proj 13B, B = 8, memory for two samples: 1.27x
        // the full-scratch time as 1 + 1 overlapped, 1.11x as one slot of 2).
        int64_t b1 = 0, b2 = 0;
        for (int64_t b = B - 1; b >= 1 && (b1 == 0 || b2 == 0); --b) {
          const size_t n = scratch_need(b);
          if (b1 == 0 && n <= workspace_bytes) b1 = b;
          if (b2 == 0 && 2 * n <= workspace_bytes && overlap_fits(b)) b2 = b;
        }
        if (b2 >= 2) { mode = FLASHDP_SCHEDULE_OVERLAP; chunk = b2; }
        else if (b1 >= 1) { mode = FLASHDP_SCHEDULE_SCRATCH; chunk = b1; }
      }
    } else {
      mode = schedule;
    }
    if (chunk == B) {
      if (mode == FLASHDP_SCHEDULE_OVERLAP && !overlap_ok) mode = FLASHDP_SCHEDULE_SCRATCH;
      const size_t need = mode == FLASHDP_SCHEDULE_OVERLAP ? need_overlap : mode == FLASHDP_SCHEDULE_SCRATCH ? need_scratch
                          : mode == FLASHDP_SCHEDULE_EXPLICIT ? need_explicit : mode == FLASHDP_SCHEDULE_GHOST ? need_ghost
                          : mode == FLASHDP_SCHEDULE_FUSED ? need_fused : need_small;
      if (workspace_bytes < need) return FLASHDP_WORKSPACE_TOO_SMALL;
    }
  } else {
    mode = schedule == FLASHDP_SCHEDULE_AUTO ? (overlap_ok ? FLASHDP_SCHEDULE_OVERLAP : FLASHDP_SCHEDULE_SCRATCH) : schedule;
    if (mode == FLASHDP_SCHEDULE_OVERLAP && !overlap_ok) mode = FLASHDP_SCHEDULE_SCRATCH;
    const size_t need = mode == FLASHDP_SCHEDULE_OVERLAP ? need_overlap : mode == FLASHDP_SCHEDULE_SCRATCH ? need_scratch
                        : mode == FLASHDP_SCHEDULE_EXPLICIT ? need_explicit : mode == FLASHDP_SCHEDULE_GHOST ? need_ghost
                        : mode == FLASHDP_SCHEDULE_FUSED ? need_fused : need_small;
    void* p = nullptr; size_t got = 0;
    st = owned_workspace(need, &p, &got);
    if (st != FLASHDP_OK) return st;
    ws = static_cast<char*>(p);
  }
  g_ctx.last_chunk = chunk;
  hipStream_t main_st = static_cast<hipStream_t>(stream);

  // Work items: (layer, chunk of samples).  The first chunk of a layer overwrites out_grad unless the caller
  // accumulates, the later ones add to it; the noise goes in with the last chunk.
  struct Item { int layer; int64_t s0, b; bool acc, noise; };
  std::vector<Item> items;
  {
    std::vector<int> order(n_layers);
    for (int l = 0; l < n_layers; ++l) order[l] = l;
    if (mode == FLASHDP_SCHEDULE_OVERLAP) {
      // Layers are independent, so they are taken largest first: the one aggregation that has nothing to hide
      // behind (the last) is then the smallest.
      std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
        return layers[x].d_in * layers[x].d_out > layers[y].d_in * layers[y].d_out;
      });
    }
    for (int l : order)
      for (int64_t s0 = 0; s0 < B; s0 += chunk) {
        const int64_t b = std::min(chunk, B - s0);
        items.push_back(Item{l, s0, b, accumulate != 0 || s0 > 0, add_noise != 0 && s0 + b == B});
      }
  }
  const int n_items = (int)items.size();

  if (mode == FLASHDP_SCHEDULE_OVERLAP) {
    // Item k: contraction on the caller's stream into scratch slot k % 2; its clip factors and aggregation
    // on the side stream, beside the contraction of item k+1 (which then follows item k's back to back).  Events order the two streams; the caller's
    // stream waits for the last aggregations before the call's work counts as complete.  The aggregations of the
    // chunks of one layer add to the same out_grad one after the other: they share the side stream, which is in order.
    // The side stream and its events are shared by every thread using this device: the whole enqueue
    // sequence below is done under the lock, so that one call's record/wait pairs are never interleaved
    // with another's (an event wait refers to the latest record at the time of the wait).
    std::lock_guard<std::mutex> lock(g_side_mutex);
    SideStream* side = &g_side[dev];
    if (!side->stream) HIP_TRY(hipStreamCreateWithFlags(&side->stream, hipStreamNonBlocking));
    while ((int)side->ready.size() < n_items) {
      hipEvent_t e1 = nullptr, e2 = nullptr;
      HIP_TRY(hipEventCreateWithFlags(&e1, hipEventDisableTiming));
      HIP_TRY(hipEventCreateWithFlags(&e2, hipEventDisableTiming));
      side->ready.push_back(e1);
      side->done.push_back(e2);
    }
    // One aggregation workgroup (4 waves, one load in flight each) per compute unit.  Measured on the Llama-13B
    // block, ms per step: 9.07-9.16 with 256 workgroups on 256 CUs, 9.22-9.24 with 192-224, 9.29-9.51 with 288-2048
    // (a CU with two of them falls behind the others that share its operand panels), 9.18-9.19 with 256 workgroups
    // of 8 waves, 9.23 with four loads in flight per thread (more registers: one wave per SIMD fits beside the
    // contraction's two, as before, but nothing is gained).
    const int grid = env().overlap_grid > 0 ? env().overlap_grid : std::max(device_cus(), 1);
    const size_t slot = scratch_need(chunk);
    for (int k = 0; k < n_items; ++k) {
      const Item& it = items[k];
      const flashdp_layer_t& Lr = layers[it.layer];
      char* wsl = ws + (size_t)(k & 1) * slot;
      if (k >= 2) HIP_TRY(hipStreamWaitEvent(main_st, side->done[k - 2], 0));   // slot free again
      st = run_layer(Lr, it.b, T, dtype, FLASHDP_SCHEDULE_SCRATCH, wsl, main_st, it.acc, it.noise, FLASHDP_STAGE_CONTRACT, 0, it.s0);
      if (st != FLASHDP_OK) return st;
      HIP_TRY(hipEventRecord(side->ready[k], main_st));
      HIP_TRY(hipStreamWaitEvent(side->stream, side->ready[k], 0));
      // the last item has nothing to hide behind: ordinary grid
      st = run_layer(Lr, it.b, T, dtype, FLASHDP_SCHEDULE_SCRATCH, wsl, side->stream, it.acc, it.noise,
                     FLASHDP_STAGE_CLIP | FLASHDP_STAGE_AGGREGATE, k + 1 < n_items ? grid : 0, it.s0);
      if (st != FLASHDP_OK) return st;
      HIP_TRY(hipEventRecord(side->done[k], side->stream));
    }
    HIP_TRY(hipStreamWaitEvent(main_st, side->done[n_items - 1], 0));
    if (n_items >= 2) HIP_TRY(hipStreamWaitEvent(main_st, side->done[n_items - 2], 0));
    g_ctx.last_schedule = "overlap";
    return FLASHDP_OK;
  }
  for (const Item& it : items) {
    st = run_layer(layers[it.layer], it.b, T, dtype, mode, ws, main_st, it.acc, it.noise, FLASHDP_STAGE_ALL, 0, it.s0);
    if (st != FLASHDP_OK) return st;
  }
  g_ctx.last_schedule = mode == FLASHDP_SCHEDULE_SCRATCH ? "scratch" : mode == FLASHDP_SCHEDULE_EXPLICIT ? "explicit"
                        : mode == FLASHDP_SCHEDULE_GHOST ? "ghost" : mode == FLASHDP_SCHEDULE_FUSED ? "fused" : "twopass";
  return FLASHDP_OK;
}

int flashdp_block_dp_grad(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                          int schedule, void* workspace, size_t workspace_bytes, void* stream) {
  return flashdp_block_dp_grad_micro(layers, n_layers, B, T, dtype, schedule, workspace, workspace_bytes, stream, 0, 1);
}

int flashdp_linear_dp_grad(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                           float C, float sigma, uint64_t seed, float* out_grad, float* out_norms) {
  flashdp_layer_t L;
  L.X = X; L.dY = dY; L.d_in = d_in; L.d_out = d_out; L.C = C; L.sigma = sigma; L.seed = seed;
  L.layer = g_ctx.layer; L.out_grad = out_grad; L.out_norms = out_norms;
  return flashdp_block_dp_grad(&L, 1, B, T, g_ctx.dtype, g_ctx.schedule, g_ctx.ws, g_ctx.ws_bytes, g_ctx.stream);
}

size_t flashdp_static_scratch_bytes(void) { return FLASHDP_STATIC_SCRATCH_BYTES; }

int flashdp_linear_dp_grad_static(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                  int dtype, float C, float sigma, uint64_t seed, uint32_t layer, float* out_grad,
                                  float* out_norms, void* stream) {
  if (!valid_dtype(dtype)) return FLASHDP_INVALID_ARGUMENT;
  flashdp_layer_t L;
  L.X = X; L.dY = dY; L.d_in = d_in; L.d_out = d_out; L.C = C; L.sigma = sigma; L.seed = seed;
  L.layer = layer; L.out_grad = out_grad; L.out_norms = out_norms;
  int st = check_layer(L, B, T);
  if (st != FLASHDP_OK) return st;
  if (layer_ws_bytes(L, B, T, dtype, FLASHDP_SCHEDULE_SCRATCH) > FLASHDP_STATIC_SCRATCH_BYTES) return FLASHDP_WORKSPACE_TOO_SMALL;
  int dev = 0;
  st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  char* ws = nullptr;
  st = static_scratch_ptr(dev, &ws);
  if (st != FLASHDP_OK) return st;
  // Every part of the workspace a call reads it has written itself first (partials by the contraction, factors
  // by the clip kernel, the parked tiles by the spill), so nothing has to be cleared between calls.
  st = run_layer(L, B, T, dtype, FLASHDP_SCHEDULE_SCRATCH, ws, static_cast<hipStream_t>(stream), false, true);
  if (st == FLASHDP_OK) g_ctx.last_schedule = "scratch";
  return st;
}

size_t flashdp_workspace_bytes(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype, int schedule) {
  if (!layers || n_layers <= 0 || !valid_dtype(dtype) || !valid_schedule(schedule)) return 0;
  size_t need = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (check_dims(B, T, layers[l].d_in, layers[l].d_out) != FLASHDP_OK) return 0;
    const int m = (schedule == FLASHDP_SCHEDULE_AUTO || schedule == FLASHDP_SCHEDULE_OVERLAP) ? FLASHDP_SCHEDULE_SCRATCH : schedule;
    need = std::max(need, layer_ws_bytes(layers[l], B, T, dtype, m));
  }
  if (schedule == FLASHDP_SCHEDULE_OVERLAP) need = 2 * align_up(need, 256);
  return need;
}

size_t flashdp_workspace_bytes_chunked(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                                       int64_t chunk_samples, int slots) {
  if (!layers || n_layers <= 0 || !valid_dtype(dtype) || chunk_samples <= 0 || chunk_samples > B || slots < 1 || slots > 2) return 0;
  size_t need = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (check_dims(B, T, layers[l].d_in, layers[l].d_out) != FLASHDP_OK) return 0;
    need = std::max(need, layer_ws_bytes(layers[l], chunk_samples, T, dtype, FLASHDP_SCHEDULE_SCRATCH));
  }
  return (size_t)slots * align_up(need, 256);
}

int flashdp_plain_grad(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                       int dtype, float* out_grad, void* stream) {
  if (!X || !dY || !out_grad || !valid_dtype(dtype)) return FLASHDP_INVALID_ARGUMENT;
  int st = check_dims(B, T, d_in, d_out);
  if (st != FLASHDP_OK) return st;
  if (!aligned16(X) || !aligned16(dY) || !aligned16(out_grad)) return FLASHDP_MISALIGNED;
  int dev = 0;
  st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  const Plan plan = make_plan(B, T, d_in, d_out, dtype);
  GemmArgs a;
  a.X = X; a.dY = dY; a.B = (int)B; a.T = (int)T; a.P = (int)d_in; a.D = (int)d_out;
  a.tiles_m = plan.tiles_m; a.tiles_n = plan.tiles_n;
  a.partials = nullptr; a.scratch = nullptr; a.factors = nullptr; a.out = out_grad; a.accumulate = 0; a.trace = nullptr;
  HIP_TRY(launch_gemm<MODE_ACCUM>(plan, dtype, a, static_cast<hipStream_t>(stream)));
  return FLASHDP_OK;
}

size_t flashdp_plain_grad_balanced_workspace_bytes(void) {
  return (size_t)STREAMK_SLOTS * STREAMK_WG_PER_XCD * 256 * 256 * sizeof(float);
}

int flashdp_plain_grad_balanced(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                int dtype, float* out_grad, void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !dY || !out_grad || !valid_dtype(dtype)) return FLASHDP_INVALID_ARGUMENT;
  int st = check_dims(B, T, d_in, d_out);
  if (st != FLASHDP_OK) return st;
  if (!aligned16(X) || !aligned16(dY) || !aligned16(out_grad) || (workspace && !aligned16(workspace))) return FLASHDP_MISALIGNED;
  // the balanced form exists for the large-tile 16-bit kernel; other problems take the ordinary plain gradient
  const bool eligible = dtype != FLASHDP_F32 && d_in % 8 == 0 && d_out % 8 == 0 &&
                        (T + 320) * (d_in > d_out ? d_in : d_out) * 2 < (int64_t(1) << 31);
  if (!eligible) return flashdp_plain_grad(X, dY, B, T, d_in, d_out, dtype, out_grad, stream);
  const size_t need = flashdp_plain_grad_balanced_workspace_bytes();
  if (workspace && workspace_bytes < need) return FLASHDP_WORKSPACE_TOO_SMALL;
  int dev = 0;
  st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  if (!workspace) {
    size_t got = 0;
    st = owned_workspace(need, &workspace, &got);
    if (st != FLASHDP_OK) return st;
  }
  StreamKArgs a;
  a.X = X; a.dY = dY; a.B = (int)B; a.T = (int)T; a.P = (int)d_in; a.D = (int)d_out;
  a.tiles_m = (int)((d_out + 255) / 256); a.tiles_n = (int)((d_in + 255) / 256);
  const int tiles = a.tiles_m * a.tiles_n;
  long n_blocks = 0, nk_pad = 0, per = 0;
  streamk_sizes((long)B, (long)T, (long)tiles, CfgDma::BK, CfgDma::STAGES, &n_blocks, &nk_pad, &per);
  a.n_blocks = (int)n_blocks;
  if (nk_pad >= (int64_t(1) << 30) || per >= (int64_t(1) << 30)) return FLASHDP_UNSUPPORTED_SHAPE;
  a.nk_pad = (int)nk_pad;
  a.units_per_xcd = (int)per;
  a.out = out_grad;
  a.partial = static_cast<float*>(workspace);
  // which pieces make up each cut block: the same walk as the kernel's, range by range (= in reduction order)
  StreamKCuts cuts;
  cuts.n = 0;
  for (int x = 0; x < STREAMK_XCDS; ++x) {
    streamk_walk(x, a.n_blocks, a.nk_pad, a.units_per_xcd, [&](const StreamKPiece& pc) {
      if (pc.slot < 0) return;
      int c = 0;
      while (c < cuts.n && cuts.block[c] != pc.block) ++c;
      if (c == cuts.n) { cuts.block[c] = pc.block; cuts.count[c] = 0; ++cuts.n; }
      cuts.slot[c][cuts.count[c]++] = pc.slot;
    });
  }
  hipStream_t hs = static_cast<hipStream_t>(stream);
  auto kern = dtype == FLASHDP_BF16 ? gemm_mfma_streamk_kernel<CfgDma, DT_BF16> : gemm_mfma_streamk_kernel<CfgDma, DT_F16>;
  HIP_TRY(ensure_lds_limit(reinterpret_cast<const void*>(kern), CfgDma::LDS_BYTES));
  hipLaunchKernelGGL(kern, dim3(STREAMK_XCDS * STREAMK_WG_PER_XCD), dim3(CfgDma::NT), CfgDma::LDS_BYTES, hs, a);
  HIP_TRY(hipGetLastError());
  if (cuts.n > 0) {
    hipLaunchKernelGGL(streamk_fixup_kernel, dim3((unsigned)(cuts.n * STREAMK_WG_PER_XCD)), dim3(256), 0, hs, a, cuts);
    HIP_TRY(hipGetLastError());
  }
  return FLASHDP_OK;
}

int flashdp_noise_field(uint64_t seed, uint32_t layer, int64_t n, float* z, void* stream) {
  if (!z || n <= 0) return FLASHDP_INVALID_ARGUMENT;
  if (reinterpret_cast<uintptr_t>(z) & 3u) return FLASHDP_MISALIGNED;
  int dev = 0;
  int st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  const size_t groups = ((size_t)n + 3) / 4;
  if (groups / 256 >= (size_t(1) << 31)) return FLASHDP_UNSUPPORTED_SHAPE;
  hipLaunchKernelGGL((noise_kernel<false>), dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream), z, (size_t)n, 1.0f, seed, layer);
  HIP_TRY(hipGetLastError());
  return FLASHDP_OK;
}

int flashdp_box_muller(const uint32_t* words, int64_t n_groups, float* z, void* stream) {
  if (!words || !z || n_groups <= 0) return FLASHDP_INVALID_ARGUMENT;
  int dev = 0;
  int st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  hipLaunchKernelGGL(box_muller_kernel, dim3((unsigned)((n_groups + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream), words, (size_t)n_groups, z);
  HIP_TRY(hipGetLastError());
  return FLASHDP_OK;
}

int flashdp_mfma_probe(int pattern, int iters, int workgroups, float* sink, void* stream) {
  if (pattern < 0 || pattern > 12 || iters <= 0 || iters > (1 << 24) || workgroups <= 0 || workgroups > (1 << 20) || !sink)
    return FLASHDP_INVALID_ARGUMENT;
  int dev = 0;
  int st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  if (pattern == 2 || pattern == 3 || pattern == 8 || pattern == 12) {   // the operand fragments re-read from LDS every k-step
    const dim3 g((unsigned)workgroups), b(512);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t lds_bytes = lds_plan::STAGE_ELEMS * 2;
    if (pattern == 2) hipLaunchKernelGGL((mfma_lds_probe_kernel<false, 0>), g, b, lds_bytes, s, iters, sink);
    else if (pattern == 3) hipLaunchKernelGGL((mfma_lds_probe_kernel<true, 0>), g, b, lds_bytes, s, iters, sink);
    else if (pattern == 8) hipLaunchKernelGGL((mfma_lds_probe_kernel<true, 1>), g, b, lds_bytes, s, iters, sink);
    else hipLaunchKernelGGL((mfma_lds_probe_kernel<true, 2>), g, b, lds_bytes, s, iters, sink);
  } else {
    const dim3 g((unsigned)workgroups), b(512);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (pattern) {
      case 0: hipLaunchKernelGGL(mfma_probe_kernel<0>, g, b, 0, s, iters, sink); break;
      case 1: hipLaunchKernelGGL(mfma_probe_kernel<1>, g, b, 0, s, iters, sink); break;
      case 4: hipLaunchKernelGGL(mfma_probe_kernel<4>, g, b, 0, s, iters, sink); break;
      case 5: hipLaunchKernelGGL(mfma_probe_kernel<5>, g, b, 0, s, iters, sink); break;
      case 6: hipLaunchKernelGGL(mfma_probe_kernel<6>, g, b, 0, s, iters, sink); break;
      case 7: hipLaunchKernelGGL(mfma_probe_kernel<7>, g, b, 0, s, iters, sink); break;
      case 9: hipLaunchKernelGGL(mfma_probe_kernel<9>, g, b, 0, s, iters, sink); break;
      case 10: hipLaunchKernelGGL(mfma_probe_kernel<10>, g, b, 0, s, iters, sink); break;
      default: hipLaunchKernelGGL(mfma_probe_kernel<11>, g, b, 0, s, iters, sink); break;
    }
  }
  HIP_TRY(hipGetLastError());
  return FLASHDP_OK;
}

int64_t flashdp_contraction_timeline(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                     int park, void* workspace, size_t workspace_bytes, uint64_t* trace, int64_t trace_entries,
                                     void* stream) {
  if (!X || !dY || !workspace || !trace) return FLASHDP_INVALID_ARGUMENT;
  int st = check_dims(B, T, d_in, d_out);
  if (st != FLASHDP_OK) return st;
  if (!aligned16(X) || !aligned16(dY) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(trace) & 7u)) return FLASHDP_MISALIGNED;
  if (d_in % 8 != 0 || d_out % 8 != 0 || (T + 320) * (d_in > d_out ? d_in : d_out) * 2 >= (int64_t(1) << 31)) return FLASHDP_UNSUPPORTED_SHAPE;
  int dev = 0;
  st = device_or_error(&dev);
  if (st != FLASHDP_OK) return st;
  Plan plan = make_plan(B, T, d_in, d_out, FLASHDP_BF16);
  plan.path = plan.accum_path = PATH_DMA16; plan.bm = plan.bn = 256;
  plan.tiles_m = (int)((d_out + 255) / 256); plan.tiles_n = (int)((d_in + 255) / 256);
  const WsLayout wl = ws_layout(plan, B, T, d_in, d_out, FLASHDP_BF16, park ? FLASHDP_SCHEDULE_SCRATCH : FLASHDP_SCHEDULE_TWOPASS);
  if (workspace_bytes < wl.total) return FLASHDP_WORKSPACE_TOO_SMALL;
  GemmArgs a;
  a.X = X; a.dY = dY; a.B = (int)B; a.T = (int)T; a.P = (int)d_in; a.D = (int)d_out;
  a.tiles_m = plan.tiles_m; a.tiles_n = plan.tiles_n;
  char* ws = static_cast<char*>(workspace);
  a.partials = reinterpret_cast<float*>(ws + wl.partials);
  a.scratch = park ? (void*)(ws + wl.scratch) : nullptr;
  a.factors = nullptr; a.out = nullptr; a.accumulate = 0;
  a.trace = reinterpret_cast<unsigned long long*>(trace);
  const int64_t grid = shared_block_grid(plan.tiles_m * plan.tiles_n, (int)B);
  if (trace_entries < grid) return FLASHDP_WORKSPACE_TOO_SMALL;
  const bool small_blocks = env().tile != PATH_DMA;   // the kernel the library takes by default
  if (small_blocks) {
    if (park) HIP_TRY(launch_tiled<CfgDma>(gemm_mfma_dma16_kernel<CfgDma, MODE_SPILL, DT_BF16, true>, MODE_SPILL, a, static_cast<hipStream_t>(stream), true));
    else HIP_TRY(launch_tiled<CfgDma>(gemm_mfma_dma16_kernel<CfgDma, MODE_NORM, DT_BF16, true>, MODE_NORM, a, static_cast<hipStream_t>(stream), true));
  } else {
    if (park) HIP_TRY(launch_tiled<CfgDma>(gemm_mfma_dma_kernel<CfgDma, MODE_SPILL, DT_BF16, true>, MODE_SPILL, a, static_cast<hipStream_t>(stream), true));
    else HIP_TRY(launch_tiled<CfgDma>(gemm_mfma_dma_kernel<CfgDma, MODE_NORM, DT_BF16, true>, MODE_NORM, a, static_cast<hipStream_t>(stream), true));
  }
  return grid;
}

int flashdp_set_stream(void* hip_stream) { g_ctx.stream = static_cast<hipStream_t>(hip_stream); return FLASHDP_OK; }

int flashdp_set_workspace(void* device_ptr, size_t bytes) {
  if ((device_ptr == nullptr) != (bytes == 0)) return FLASHDP_INVALID_ARGUMENT;
  if (device_ptr && !aligned16(device_ptr)) return FLASHDP_MISALIGNED;
  g_ctx.ws = device_ptr; g_ctx.ws_bytes = bytes;
  return FLASHDP_OK;
}

int flashdp_set_dtype(int dtype) {
  if (!valid_dtype(dtype)) return FLASHDP_INVALID_ARGUMENT;
  g_ctx.dtype = dtype;
  return FLASHDP_OK;
}

int flashdp_set_layer(uint32_t layer) { g_ctx.layer = layer; return FLASHDP_OK; }

int flashdp_set_schedule(int schedule) {
  if (!valid_schedule(schedule)) return FLASHDP_INVALID_ARGUMENT;
  g_ctx.schedule = schedule;
  return FLASHDP_OK;
}

int flashdp_set_stages(int mask) {
  if (mask <= 0 || mask > FLASHDP_STAGE_ALL) return FLASHDP_INVALID_ARGUMENT;
  g_ctx.stages = mask;
  return FLASHDP_OK;
}

int flashdp_release(void) {
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  int cur = 0;
  const bool have_cur = hipGetDevice(&cur) == hipSuccess;
  for (auto& kv : g_owned) {
    if (!kv.second.ptr) continue;
    if (hipSetDevice(kv.first) != hipSuccess) continue;
    (void)hipDeviceSynchronize();
    (void)hipFree(kv.second.ptr);
    kv.second = OwnedWs();
  }
  std::lock_guard<std::mutex> side_lock(g_side_mutex);
  for (auto& kv : g_side) {
    if (hipSetDevice(kv.first) != hipSuccess) continue;
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : kv.second.ready) (void)hipEventDestroy(e);
    for (hipEvent_t e : kv.second.done) (void)hipEventDestroy(e);
    if (kv.second.stream) (void)hipStreamDestroy(kv.second.stream);
    kv.second = SideStream();
  }
  if (have_cur) (void)hipSetDevice(cur);
  (void)hipGetLastError();
  return FLASHDP_OK;
}

const char* flashdp_last_schedule(void) { return g_ctx.last_schedule; }

const char* flashdp_last_kernel(void) { return g_ctx.last_kernel; }

int64_t flashdp_last_chunk(void) { return g_ctx.last_chunk; }

const char* flashdp_status_string(int status) {
  switch (status) {
    case FLASHDP_OK: return "ok";
    case FLASHDP_INVALID_ARGUMENT: return "invalid argument";
    case FLASHDP_MISALIGNED: return "pointer not 16-byte aligned";
    case FLASHDP_UNSUPPORTED_SHAPE: return "unsupported shape";
    case FLASHDP_WORKSPACE_TOO_SMALL: return "workspace too small";
    case FLASHDP_NO_DEVICE: return "no HIP device";
    case FLASHDP_HIP_ERROR: return "HIP runtime error";
    default: return "unknown status";
  }
}

int flashdp_version(void) { return 100; }

}  // extern "C"
