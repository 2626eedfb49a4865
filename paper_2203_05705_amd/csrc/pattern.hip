// Dropout patterns: host-side distribution search and sampling (Sections 3.3, 3.4)
// and device-side mask + kept-list generation (Sections 3.1, 3.2, 6).
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "pattern.hpp"

namespace ard {

const DevKnobs& dev_knobs() {
  static const DevKnobs k = {getenv("ARD_NO_FAST") != nullptr, getenv("ARD_NO_SCATTER") != nullptr,
                             getenv("ARD_FORCE_TILE") ? atoi(getenv("ARD_FORCE_TILE")) : 0,
                             getenv("ARD_CLASS_TILE") ? atoi(getenv("ARD_CLASS_TILE")) : 0,
                             getenv("ARD_PROVE_BOUNDS") != nullptr};
  return k;
}


static thread_local char g_err[512] = "";

// ---- dry-run mode (see common.hpp) ----------------------------------------
static int g_dry_run = 0;                       // process-wide switch
static thread_local int g_dry_count = 0;        // launches skipped on this thread since the last reset
static thread_local char g_dry_log[2048] = "";  // their kernel names, comma separated (truncated when full)
bool dry_run() { return g_dry_run != 0; }
void note_dry_launch(const char* kernel) {
  ++g_dry_count;
  // keep the template name without its argument list
  size_t len = strlen(g_dry_log), n = 0;
  while (*kernel == '(') ++kernel;
  while (kernel[n] && kernel[n] != '<' && kernel[n] != '(' && kernel[n] != ')') ++n;
  if (len + n + 2 < sizeof(g_dry_log)) {
    if (len) g_dry_log[len++] = ',';
    memcpy(g_dry_log + len, kernel, n);
    g_dry_log[len + n] = 0;
  }
}
// [a_lo, a_hi, a_bytes, b_lo, b_hi, b_bytes] of this thread's most recent exhaustive bounds proof, and
// the number of proofs since the last query
static thread_local long g_last_bounds[6] = {0, 0, 0, 0, 0, 0};
static thread_local int g_n_proofs = 0;
void note_direct_bounds(const DirectBounds& b, long a_bytes, long b_bytes) {
  g_last_bounds[0] = b.a_lo, g_last_bounds[1] = b.a_hi, g_last_bounds[2] = a_bytes;
  g_last_bounds[3] = b.b_lo, g_last_bounds[4] = b.b_hi, g_last_bounds[5] = b_bytes;
  ++g_n_proofs;
}
static long g_extent_slack = 0;
long extent_slack() { return g_extent_slack; }
hipError_t launch_status() { return g_dry_run ? hipSuccess : hipGetLastError(); }
hipError_t raise_lds_limit(const void* kernel, int bytes) {
  if (g_dry_run) return hipSuccess;
  return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int32_t check_pattern(const ard_pattern* p, int units, const char* what) {
  if (!p || p->kind == ARD_PAT_NONE) return ARD_OK;
  if (p->kind == ARD_PAT_ROW || p->kind == ARD_PAT_TILE) {
    // dp ranges over 1..number of units (dp_max of Sections 3.1 / 3.2), b over 1..dp
    if (p->dp < 1 || p->dp > (units > 1 ? units : 1))
      return fail(ARD_EINVAL, "%s: dp=%d outside 1..%d", what, p->dp, units);
    if (p->b < 1 || p->b > p->dp) return fail(ARD_EINVAL, "%s: b=%d outside 1..dp=%d", what, p->b, p->dp);
    return ARD_OK;
  }
  if (p->kind == ARD_PAT_LIST) {
    if (p->count < 0 || p->count > units) return fail(ARD_EINVAL, "%s: list count %d outside 0..%d", what, p->count, units);
    if (p->count > 0 && !p->d_keep) return fail(ARD_EINVAL, "%s: list pattern without d_keep", what);
    return ARD_OK;
  }
  return fail(ARD_EINVAL, "%s: unknown pattern kind %d", what, p->kind);
}

int kept_count(const ard_pattern* p, int units) {
  if (!p || p->kind == ARD_PAT_NONE) return units;
  if (p->kind == ARD_PAT_LIST) return p->count;
  int o = p->b - 1;
  return units > o ? (units - o + p->dp - 1) / p->dp : 0;
}

Axis axis_of_pattern(const ard_pattern* p, int units) {
  if (!p || p->kind == ARD_PAT_NONE) return axis_identity(units);
  if (p->kind == ARD_PAT_LIST) return axis_list(p->d_keep, p->count, units);
  return axis_affine(p->b - 1, p->dp, kept_count(p, units), units);
}

// One workgroup walks the units in enumeration order e = 0..n-1 and compacts the
// kept ones: per wavefront a ballot of the keep predicate, mbcnt for the lane's
// rank inside the ballot, wave totals combined through LDS.
// colmajor = 0: unit id = e (row-major over the TR x TC grid), value stored = e.
// colmajor = 1: e = tc*TR + tr, unit id = tr*TC + tc, value stored = tr.
// ptr[g] = number of kept units enumerated before group g (group size gsize).
__global__ __launch_bounds__(1024) void pattern_compact_kernel(int n, int dp, int o, int TR, int TC, int colmajor,
                                                              int gsize, uint8_t* mask, int* keep, int* count,
                                                              int* ptr) {
  __shared__ int wave_tot[16];
  __shared__ int running_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) running_s = 0;
  __syncthreads();
  for (int base = 0; base < n; base += 1024) {
    const int e = base + tid;
    bool kept = false;
    int unit = 0, value = 0;
    if (e < n) {
      if (colmajor) {
        int tc = e / TR, tr = e - tc * TR;
        unit = tr * TC + tc;
        value = tr;
      } else {
        unit = e;
        value = e;
      }
      kept = ((unit + dp - o) % dp) == 0;  // Eq. (1) with the 0-based offset o = b-1 < dp
    }
    const unsigned long long bal = __ballot(kept);
    const int rank = __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int before = running_s, total = 0;
    for (int w = 0; w < 16; ++w) {
      int t = wave_tot[w];
      if (w < wave) before += t;
      total += t;
    }
    const int pos = before + rank;
    if (e < n) {
      if (mask && !colmajor) mask[e] = kept ? 1 : 0;
      if (kept && keep) keep[pos] = value;
      if (ptr && (e % gsize) == 0) ptr[e / gsize] = pos;
    }
    __syncthreads();
    if (tid == 0) running_s += total;
    __syncthreads();
  }
  if (tid == 0) {
    if (count) *count = running_s;
    if (ptr) ptr[(n + gsize - 1) / gsize] = running_s;
  }
}

int32_t pattern_gen_launch(const ard_pattern* pat, int32_t rows, int32_t cols, uint8_t* d_mask, int32_t* d_keep,
                           int32_t* d_count, int32_t* d_rowptr, int32_t* d_colptr, int32_t* d_csc_rows,
                           hipStream_t stream) {
  const int o = pat->b - 1, dp = pat->dp;
  if (pat->kind == ARD_PAT_ROW) {
    ARD_LAUNCH(pattern_compact_kernel, dim3(1), dim3(1024), 0, stream, rows, dp, o, 1, rows, 0, rows, d_mask,
                       d_keep, d_count, (int*)nullptr);
    ARD_LAUNCH_CHECK("pattern_compact_kernel");
    return ARD_OK;
  }
  const int TR = ceil_div(rows, pat->tile_r), TC = ceil_div(cols, pat->tile_c);
  if (d_mask || d_keep || d_count || d_rowptr) {
    ARD_LAUNCH(pattern_compact_kernel, dim3(1), dim3(1024), 0, stream, TR * TC, dp, o, TR, TC, 0, TC, d_mask,
                       d_keep, d_count, d_rowptr);
    ARD_LAUNCH_CHECK("pattern_compact_kernel");
  }
  if (d_colptr || d_csc_rows) {
    ARD_LAUNCH(pattern_compact_kernel, dim3(1), dim3(1024), 0, stream, TR * TC, dp, o, TR, TC, 1, TR,
                       (uint8_t*)nullptr, d_csc_rows, (int*)nullptr, d_colptr);
    ARD_LAUNCH_CHECK("pattern_compact_kernel");
  }
  return ARD_OK;
}

// SplitMix64 finaliser (Steele, Lea, Flood 2014; public domain constants).
static inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}
static const uint64_t kGolden = 0x9E3779B97F4A7C15ULL;

}  // namespace ard

using namespace ard;

extern "C" const char* ard_last_error(void) { return g_err; }
extern "C" int32_t ard_version(void) { return 200; }

extern "C" void ard_debug_set_dry_run(int32_t on) {
  g_dry_run = on ? 1 : 0;
  g_dry_count = 0;
  g_dry_log[0] = 0;
}
extern "C" int32_t ard_debug_dry_launches(char* names, size_t cap) {
  if (names && cap) {
    strncpy(names, g_dry_log, cap - 1);
    names[cap - 1] = 0;
  }
  const int n = g_dry_count;
  g_dry_count = 0;
  g_dry_log[0] = 0;
  return n;
}

extern "C" void ard_debug_set_extent_slack(int64_t elems) { g_extent_slack = elems; }

extern "C" int32_t ard_debug_last_bounds(int64_t* six) {
  if (six)
    for (int i = 0; i < 6; ++i) six[i] = g_last_bounds[i];
  const int n = g_n_proofs;
  g_n_proofs = 0;
  return n;
}

extern "C" int32_t ard_kept_count(const ard_pattern* pat, int32_t units) {
  if (units < 0) return fail(ARD_ESHAPE, "negative unit count");
  if (pat && pat->kind == ARD_PAT_TILE) return fail(ARD_EINVAL, "ard_kept_count takes ROW, LIST or NONE patterns");
  int32_t st = check_pattern(pat, units, "pattern");
  if (st) return st;
  return kept_count(pat, units);
}
extern "C" int32_t ard_compact_dim(const ard_pattern* pat, int32_t units) {
  const int32_t n = ard_kept_count(pat, units);
  return n < 0 ? n : pad8(n);
}
extern "C" int32_t ard_tile_grid(const ard_pattern* pat, int32_t rows, int32_t cols, int32_t* tile_rows,
                                 int32_t* tile_cols) {
  if (!pat || pat->kind != ARD_PAT_TILE) return fail(ARD_EINVAL, "ard_tile_grid needs a TILE pattern");
  if (pat->tile_r <= 0 || pat->tile_c <= 0) return fail(ARD_EINVAL, "tile size must be positive");
  if (rows <= 0 || cols <= 0) return fail(ARD_ESHAPE, "rows and cols must be positive (got %d, %d)", rows, cols);
  if (!tile_rows || !tile_cols) return fail(ARD_EINVAL, "null output pointer");
  *tile_rows = ceil_div(rows, pat->tile_r);
  *tile_cols = ceil_div(cols, pat->tile_c);
  return ARD_OK;
}

extern "C" int32_t ard_pattern_gen(const ard_pattern* pat, int32_t rows, int32_t cols, uint8_t* d_mask,
                                   int32_t* d_keep, int32_t* d_count, int32_t* d_rowptr, int32_t* d_colptr,
                                   int32_t* d_csc_rows, void* stream) {
  if (!pat) return fail(ARD_EINVAL, "null pattern");
  if (pat->kind == ARD_PAT_ROW) {
    if (rows <= 0) return fail(ARD_ESHAPE, "rows must be positive (got %d)", rows);
    int32_t st = check_pattern(pat, rows, "pattern");
    if (st) return st;
    if (d_rowptr || d_colptr || d_csc_rows) return fail(ARD_EINVAL, "row patterns have no tile offsets");
  } else if (pat->kind == ARD_PAT_TILE) {
    if (rows <= 0 || cols <= 0) return fail(ARD_ESHAPE, "rows and cols must be positive (got %d, %d)", rows, cols);
    if (pat->tile_r <= 0 || pat->tile_c <= 0) return fail(ARD_EINVAL, "tile size must be positive");
    long units = (long)ceil_div(rows, pat->tile_r) * ceil_div(cols, pat->tile_c);
    if (units > 0x7fffffffL) return fail(ARD_ESHAPE, "tile grid too large");
    int32_t st = check_pattern(pat, (int)units, "pattern");
    if (st) return st;
    if (d_csc_rows && !d_colptr) return fail(ARD_EINVAL, "d_csc_rows needs d_colptr");
  } else {
    return fail(ARD_EINVAL, "pattern_gen needs a ROW or TILE pattern (kind %d)", pat->kind);
  }
  return pattern_gen_launch(pat, rows, cols, d_mask, d_keep, d_count, d_rowptr, d_colptr, d_csc_rows,
                            (hipStream_t)stream);
}

extern "C" int32_t ard_pattern_sample(const uint64_t* cdf, int32_t n, uint64_t seed, uint64_t iter, uint32_t stream_id,
                                      int32_t* dp_out, int32_t* b_out) {
  if (!cdf || !dp_out || !b_out) return fail(ARD_EINVAL, "null pointer");
  if (n < 1) return fail(ARD_ESHAPE, "n must be positive");
  uint64_t h = mix64(seed + kGolden);
  h = mix64((h ^ iter) + kGolden);
  h = mix64((h ^ (uint64_t)stream_id) + kGolden);
  const uint64_t r1 = h >> 32, r2 = h & 0xFFFFFFFFULL;
  int dp = n;
  for (int i = 0; i < n; ++i)
    if (r1 < cdf[i]) {
      dp = i + 1;
      break;
    }
  *dp_out = dp;
  *b_out = 1 + (int32_t)((r2 * (uint64_t)dp) >> 32);
  return ARD_OK;
}

extern "C" int32_t ard_search_k(double p, int32_t n, uint64_t seed, double* k_out, uint64_t* cdf_out) {
  if (!(p >= 0.0 && p < 1.0)) return fail(ARD_EINVAL, "target rate must be in [0,1) (got %g)", p);
  if (n < 1 || n > 4096) return fail(ARD_ESHAPE, "n must be in 1..4096 (got %d)", n);
  if (!k_out || !cdf_out) return fail(ARD_EINVAL, "null output pointer");
  const double lam_p = 1.0, lam_e = 1e-3;
  std::vector<double> v(n, 0.0), d(n), g(n), gv(n), vt(n), dt(n), pu(n);
  for (int i = 0; i < n; ++i) pu[i] = (double)i / (double)(i + 1);  // (i-1)/i for the 1-based period
  if (seed != 0)
    for (int i = 0; i < n; ++i) v[i] = ((double)(mix64(seed + kGolden * (uint64_t)(i + 1)) >> 11) * 0x1.0p-53 - 0.5);
  auto eval = [&](const std::vector<double>& vv, std::vector<double>& dd) {
    double mx = vv[0];
    for (int i = 1; i < n; ++i) mx = vv[i] > mx ? vv[i] : mx;
    double s = 0;
    for (int i = 0; i < n; ++i) {
      dd[i] = exp(vv[i] - mx);
      s += dd[i];
    }
    double rate = 0, ent = 0;
    for (int i = 0; i < n; ++i) {
      dd[i] /= s;
      rate += dd[i] * pu[i];
      ent += dd[i] * log(dd[i] > 1e-300 ? dd[i] : 1e-300);
    }
    return lam_p * (rate - p) * (rate - p) + lam_e * ent;
  };
  double cur = eval(v, d), lr = 1.0;
  for (int step = 0; step < 200000; ++step) {
    double rate = 0;
    for (int i = 0; i < n; ++i) rate += d[i] * pu[i];
    double dg = 0;
    for (int i = 0; i < n; ++i) {
      g[i] = 2.0 * lam_p * (rate - p) * pu[i] + lam_e * (log(d[i] > 1e-300 ? d[i] : 1e-300) + 1.0);
      dg += d[i] * g[i];
    }
    double gmax = 0;
    for (int i = 0; i < n; ++i) {
      gv[i] = d[i] * (g[i] - dg);  // through the softmax Jacobian
      gmax = fabs(gv[i]) > gmax ? fabs(gv[i]) : gmax;
    }
    double nxt;
    for (;;) {
      for (int i = 0; i < n; ++i) vt[i] = v[i] - lr * gv[i];
      nxt = eval(vt, dt);
      if (nxt <= cur || lr < 1e-12) break;
      lr *= 0.5;
    }
    v = vt;
    d = dt;
    double delta = cur - nxt;
    cur = nxt;
    lr = lr * 2.0 < 1e6 ? lr * 2.0 : 1e6;
    if (delta < 1e-15 && gmax < 1e-10) break;
  }
  double c = 0;
  uint64_t prev = 0;
  for (int i = 0; i < n; ++i) {
    k_out[i] = d[i];
    c += d[i];
    double q = floor(c * 4294967296.0 + 0.5);
    if (q < 0) q = 0;
    if (q > 4294967296.0) q = 4294967296.0;
    uint64_t u = (uint64_t)q;
    if (u < prev) u = prev;
    cdf_out[i] = u;
    prev = u;
  }
  cdf_out[n - 1] = 4294967296ULL;
  return ARD_OK;
}
