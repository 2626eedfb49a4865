// Shared host/device helpers of libard: index maps, bf16 conversion, error plumbing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/ard.h"

namespace ard {

// ---- error plumbing -------------------------------------------------------
void set_error(const char* fmt, ...);
int32_t fail(int32_t code, const char* fmt, ...);

// ---- launches -------------------------------------------------------------
// Every kernel launch of the library goes through ARD_LAUNCH.  In dry-run mode (ard_debug_set_dry_run)
// nothing is enqueued and no HIP call is made: the entry points run their argument checks, their
// dispatch and the host-side bounds proof of the LDS-direct loaders, and count the launches they
// would have issued.  The mode exists so that host logic can be tested on a machine without a GPU.
bool dry_run();
void note_dry_launch(const char* kernel);
hipError_t launch_status();  // hipGetLastError(), or hipSuccess in dry-run mode
hipError_t raise_lds_limit(const void* kernel, int bytes);  // hipFuncSetAttribute(max dynamic LDS); no-op in dry-run mode
#define ARD_LAUNCH_NAMED(name, kernel, ...)                      \
  do {                                                           \
    if (ard::dry_run()) ard::note_dry_launch(name);              \
    else hipLaunchKernelGGL(kernel, __VA_ARGS__);                \
  } while (0)
#define ARD_LAUNCH(kernel, ...) ARD_LAUNCH_NAMED(#kernel, kernel, __VA_ARGS__)
#define ARD_HIP_CHECK(expr)                                                        \
  do {                                                                             \
    hipError_t e__ = (expr);                                                       \
    if (e__ != hipSuccess)                                                         \
      return ard::fail(ARD_EHIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
  } while (0)
#define ARD_LAUNCH_CHECK(name)                                                     \
  do {                                                                             \
    hipError_t e__ = ard::launch_status();                                           \
    if (e__ != hipSuccess)                                                         \
      return ard::fail(ARD_EHIP, "launch of %s failed: %s", name, hipGetErrorString(e__)); \
  } while (0)

// byte ranges [lo, hi) the loaders of one LDS-direct launch touch behind A and B (host-side proof)
struct DirectBounds {
  long a_lo, a_hi, b_lo, b_hi;
};
void note_direct_bounds(const DirectBounds& b, long a_bytes, long b_bytes);
long extent_slack();  // elements the proofs pretend each operand is shorter by (ard_debug_set_extent_slack; 0 in normal use)

// ---- grouped launches -------------------------------------------------------
// Between ard_batch_begin() and ard_batch_launch() (per thread) the launches of the kernels that have a
// GK_* kind are recorded instead of issued; ard_batch_launch() then runs all recorded launches of a
// stage as ONE grid of a kernel that holds every such body (gemm.hip).  Stage 0: launches that depend on
// nothing recorded in the batch; stage 1: passes that finish a stage-0 product of the same call.
bool batch_open();
// A call may open a batch of its own for kernels of its that do not depend on each other (then launches it
// itself): only when the caller has none, open or suspended.  false: launch one by one.
bool batch_self_begin();
int32_t batch_self_end(bool ok, hipStream_t stream);
// While one lives, this thread's launches are issued at once even inside an open batch: for kernels
// whose consumer in the same call is recorded too, or issued at once, and must find their result.
struct BatchSuspend {
  bool was_open;
  BatchSuspend();
  ~BatchSuspend();
};

// ---- index maps -------------------------------------------------------------
// A logical (compact) index j in [0, n) maps to a physical index in [0, nphys):
//   AFFINE  off + j*step          (row pattern: off = b-1, step = dp; identity: 0, 1)
//   LIST    list[j]               (explicit kept-unit list)
//   BLOCK   list[j / bs]*bs + j%bs (kept tiles: list of block ids, block size bs)
//   BAFF    (off + (j / bs)*step)*bs + j%bs   (every step-th block starting at block off)
enum { AX_AFFINE = 0, AX_LIST = 1, AX_BLOCK = 2, AX_BAFF = 3 };

struct Axis {
  const int* list;
  int kind;
  int off, step;
  int bs;
  int n;      // logical length
  int nphys;  // physical extent
};

__host__ __device__ static inline Axis axis_identity(int n) { return Axis{nullptr, AX_AFFINE, 0, 1, 1, n, n}; }
static inline Axis axis_affine(int off, int step, int n, int nphys) {
  return Axis{nullptr, AX_AFFINE, off, step, 1, n, nphys};
}
static inline Axis axis_list(const int* l, int n, int nphys) { return Axis{l, AX_LIST, 0, 1, 1, n, nphys}; }
static inline Axis axis_block(const int* l, int bs, int nblocks, int nphys) {
  return Axis{l, AX_BLOCK, 0, 1, bs, nblocks * bs, nphys};
}
__host__ __device__ static inline Axis axis_baff(int off, int step, int bs, int nblocks, int nphys) {
  return Axis{nullptr, AX_BAFF, off, step, bs, nblocks * bs, nphys};
}
// A run of `ce` logical elements starting at a multiple of `ce` is physically
// contiguous and starts at a multiple of `ce`.
static inline bool axis_chunk_contiguous(const Axis& a, int ce) {
  if (a.kind == AX_AFFINE) return a.step == 1 && (a.off % ce) == 0;
  if (a.kind == AX_BLOCK || a.kind == AX_BAFF) return (a.bs % ce) == 0;
  return false;
}

__host__ __device__ static inline int imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ static inline int imax(int a, int b) { return a > b ? a : b; }

// (host callers: every kind except LIST, whose entries live in device memory)
__host__ __device__ __forceinline__ int ax_phys(const Axis& a, int j) {
  if (a.kind == AX_AFFINE) return a.off + j * a.step;
  if (a.kind == AX_LIST) return a.list[j];
  int q = j / a.bs;
  if (a.kind == AX_BAFF) return (a.off + q * a.step) * a.bs + (j - q * a.bs);
  return a.list[q] * a.bs + (j - q * a.bs);
}

// ---- bf16 -------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);                      // round to nearest even
  return (uint16_t)(u >> 16);
}

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
  static constexpr int CE = 4;  // elements per 16-byte chunk
  __device__ static __forceinline__ float to_f32(float v) { return v; }
  __device__ static __forceinline__ float from_f32(float v) { return v; }
};
template <> struct ElemTraits<uint16_t> {
  static constexpr int CE = 8;
  __device__ static __forceinline__ float to_f32(uint16_t v) { return bf16_bits_to_f32(v); }
  __device__ static __forceinline__ uint16_t from_f32(float v) { return f32_to_bf16_bits(v); }
};

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
// column count of a compact matrix: kept count rounded up to a whole 16-byte chunk of bf16
// Development switches, read once from the environment: ARD_NO_FAST=1 sends every product
// through the general engine, ARD_NO_SCATTER=1 disables the scattering epilogue (partial sums +
// finishing pass instead), ARD_FORCE_TILE=64|128 pins the general engine's workgroup tile,
// ARD_CLASS_TILE=1..5 pins the tile of the tile-pattern products (position in their tile list).
// ARD_PROVE_BOUNDS=1 runs the exhaustive host-side bounds proof of the LDS-direct loaders before
// every launch (the cheap envelope check always runs).
struct DevKnobs {
  bool no_fast, no_scatter;
  int force_tile, class_tile;
  bool prove_bounds;
};
const DevKnobs& dev_knobs();

__host__ __device__ static inline int pad8(int n) { return (n + 7) & ~7; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- pattern helpers (host) ---------------------------------------------------
int32_t check_pattern(const ard_pattern* p, int units, const char* what);
// number of kept units of a ROW pattern (or NONE/LIST) over `units`
int kept_count(const ard_pattern* p, int units);
// logical->physical map of a ROW / LIST / NONE pattern over `units`
Axis axis_of_pattern(const ard_pattern* p, int units);

// Exact unsigned division by a divisor known on the host (multiply-high and shifts instead of the 30-odd
// instructions of a division by a run-time value).
struct FastDiv {
  uint32_t mul;
  int shift;  // -1: divisor 1
};
static FastDiv fast_div(uint32_t d) {
  if (d <= 1) return FastDiv{0u, -1};
  int l = 0;
  while ((1ull << l) < d) ++l;  // ceil(log2 d) >= 1
  const uint64_t m = ((1ull << 32) * ((1ull << l) - d)) / d + 1;
  return FastDiv{(uint32_t)m, l - 1};
}
static __device__ __forceinline__ uint32_t fdiv(uint32_t a, const FastDiv& f) {
  if (f.shift < 0) return a;
  const uint32_t t = __umulhi(a, f.mul);
  return (t + ((a - t) >> 1)) >> f.shift;
}

}  // namespace ard
