// Fully connected layer under a dropout pattern: forward, backward-data and
// backward-weight entry points (Sections 3.1, 3.2), all mapped onto the gathered
// MFMA engine.
#include <stdlib.h>

#include <mutex>

#include <string.h>

#include <vector>

#include "engine.hpp"
#include "fast.hpp"
#include "pattern.hpp"
#include "skinny.hpp"

namespace ard {

// Launch with dynamic LDS; kernels above the 64 KiB default get their limit raised once.
template <typename K>
static int32_t launch_one(K kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, const GemmParams& P) {
  if (lds_bytes > 65536) {
    static thread_local const void* raised[64];
    static thread_local int n_raised = 0;
    bool seen = false;
    for (int i = 0; i < n_raised; ++i) seen = seen || raised[i] == (const void*)kernel;
    if (!seen) {
      ARD_HIP_CHECK(ard::raise_lds_limit((const void*)kernel, (int)lds_bytes));
      if (n_raised < 64 && !dry_run()) raised[n_raised++] = (const void*)kernel;
    }
  }
  ARD_LAUNCH_NAMED("gemm_kernel", kernel, grid, block, lds_bytes, stream, P);
  ARD_LAUNCH_CHECK("gemm_kernel");
  return ARD_OK;
}

template <typename T, int BM, int BN, int WGM, int WGN>
static int32_t launch_cfg(bool a_kc, bool b_kc, GemmParams& P, hipStream_t stream) {
  P.tiles_m = ceil_div(P.M, BM);
  P.tiles_n = ceil_div(P.N, BN);
  long blocks = (long)P.tiles_m * P.tiles_n;
  if (blocks <= 0) return ARD_OK;
  if (blocks > 0x7fffffffL) return fail(ARD_ESHAPE, "too many workgroups");
  dim3 grid((unsigned)blocks, (unsigned)(P.part ? P.splits : 1)), block(64 * WGM * WGN);
  constexpr size_t lds_bytes = (size_t)2 * (BM + BN) * LDS_ROW_U4 * sizeof(uint4);
  if (a_kc && b_kc)
    return launch_one(gemm_kernel<T, BM, BN, WGM, WGN, true, true>, grid, block, lds_bytes, stream, P);
  if (a_kc && !b_kc)
    return launch_one(gemm_kernel<T, BM, BN, WGM, WGN, true, false>, grid, block, lds_bytes, stream, P);
  if (!a_kc && !b_kc)
    return launch_one(gemm_kernel<T, BM, BN, WGM, WGN, false, false>, grid, block, lds_bytes, stream, P);
  return fail(ARD_EUNSUPPORTED, "operand layout combination not built");
}

template <typename T>
static int32_t run_gemm_t(bool a_kc, bool b_kc, GemmParams& P, int max_bn, hipStream_t stream) {
  if (const int v = dev_knobs().force_tile) {
    if (v == 256) return launch_cfg<T, 128, 128, 2, 2>(a_kc, b_kc, P, stream);
    if (v == 128) return launch_cfg<T, 128, 128, 2, 2>(a_kc, b_kc, P, stream);
    if (v == 64) return launch_cfg<T, 64, 64, 2, 2>(a_kc, b_kc, P, stream);
  }
  if (max_bn == 32) return launch_cfg<T, 128, 32, 4, 1>(a_kc, b_kc, P, stream);
  if (max_bn == 64) return launch_cfg<T, 128, 64, 2, 2>(a_kc, b_kc, P, stream);
  long t128 = (long)ceil_div(P.M, 128) * ceil_div(P.N, 128);
  if (t128 >= 192) return launch_cfg<T, 128, 128, 2, 2>(a_kc, b_kc, P, stream);
  return launch_cfg<T, 64, 64, 2, 2>(a_kc, b_kc, P, stream);
}

static bool try_direct(int32_t dtype, bool a_kc, bool b_kc, const GemmParams& P, void* ws, size_t ws_bytes,
                       hipStream_t stream, int32_t& st, int* raw_splits = nullptr);

// The product as fp32 partial sums part[split][M][N] (compact, alpha not applied) for a caller
// whose next kernel sums them itself; *splits receives their number.  Returns false (nothing
// launched) when the product does not qualify for the LDS-direct kernels or the room is too small.
bool run_gemm_partials(int32_t dtype, bool a_kc, bool b_kc, const GemmParams& P, hipStream_t stream, void* part,
                       size_t part_bytes, int* splits, int32_t* status) {
  *status = ARD_OK;
  return try_direct(dtype, a_kc, b_kc, P, part, part_bytes, stream, *status, splits);
}

int32_t run_gemm(int32_t dtype, bool a_kc, bool b_kc, GemmParams P, int max_bn, int /*max_bm*/, hipStream_t stream,
                 void* ws, size_t ws_bytes) {
  int32_t st_fast = ARD_OK;
  if (try_direct(dtype, a_kc, b_kc, P, ws, ws_bytes, stream, st_fast)) return st_fast;
  if (dtype != ARD_BF16 && dtype != ARD_F32) return fail(ARD_EDTYPE, "unknown dtype %d", dtype);
  // A product with too few tiles for the chip splits its contraction over blockIdx.y into fp32
  // partial sums (fixed split: deterministic) that the finishing pass reduces and stores.
  auto inv_ok = [](const Axis& a) { return a.kind == AX_AFFINE || a.kind == AX_LIST; };
  const long tiles = (long)ceil_div(P.M, 64) * ceil_div(P.N, 64);
  const int steps = ceil_div(P.k.n, dtype == ARD_BF16 ? 64 : 32);
  if (ws && !P.kb_ptr && !P.tmask && !P.C.plane && inv_ok(P.C.rm) && inv_ok(P.C.cn) && tiles > 0 && tiles < 128 &&
      steps >= 4 && (long)P.M * P.N < (1L << 31)) {
    int splits = (int)(256 / tiles);
    if (splits > steps / 2) splits = steps / 2;
    if (splits > 8) splits = 8;
    if (splits > 1 && (size_t)splits * P.M * P.N * 4 <= ws_bytes) {
      P.part = (float*)ws;
      P.splits = splits;
    }
  }
  int32_t st = dtype == ARD_BF16 ? run_gemm_t<uint16_t>(a_kc, b_kc, P, max_bn, stream)
                                 : run_gemm_t<float>(a_kc, b_kc, P, max_bn, stream);
  if (st || !P.part) return st;
  const OutMat& C = P.C;
  const long total = C.fill ? (long)C.rm.nphys * C.cn.nphys : (long)P.M * P.N;
  long blocks = (total + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  if (dtype == ARD_BF16)
    ARD_LAUNCH(gemm_finish_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)ws,
                       P.splits, P.M, P.N, C);
  else
    ARD_LAUNCH(gemm_finish_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)ws, P.splits,
                       P.M, P.N, C);
  ARD_LAUNCH_CHECK("gemm_finish_kernel");
  return ARD_OK;
}

// ---- large-tile path -------------------------------------------------------------------

static int gcd_int(int a, int b) {
  while (b) {
    int t = a % b;
    a = b;
    b = t;
  }
  return a;
}

template <int BM, int BN, int NW>
static int32_t launch_direct_cfg(bool a_kc, bool b_kc, FastParams& F, int grid_x, hipStream_t stream) {
  if (a_kc && b_kc) return launch_direct_kernel<true, true, BM, BN, NW, 0>(F, grid_x, stream);
  if (a_kc && !b_kc) return launch_direct_kernel<true, false, BM, BN, NW, 0>(F, grid_x, stream);
  if (!a_kc && !b_kc) return launch_direct_kernel<false, false, BM, BN, NW, 0>(F, grid_x, stream);
  return fail(ARD_EUNSUPPORTED, "operand layout combination not built");
}

// Grid of the large-tile kernel: every XCD takes the share [x*n/8, (x+1)*n/8) of each class.
static int fast_grid(const FastParams& F) {
  int worst = 0;
  for (int x = 0; x < 8; ++x) {
    int sum = 0;
    if (F.tab.ncls == 0) {
      sum = (int)((long)(x + 1) * F.total_tiles / 8) - (int)((long)x * F.total_tiles / 8);
    } else {
      for (int c = 0; c < F.tab.ncls; ++c)
        sum += (int)((long)(x + 1) * F.tab.nblk[c] / 8) - (int)((long)x * F.tab.nblk[c] / 8);
    }
    worst = sum > worst ? sum : worst;
  }
  return worst * 8;
}

struct TileCfg {
  int bm, bn;
};
static const TileCfg kTileCfgs[] = {{256, 256}, {256, 128}, {128, 128}, {128, 64}, {64, 64}};

static int32_t launch_direct(bool a_kc, bool b_kc, FastParams& F, int bm, int bn, hipStream_t stream) {
  if (F.total_tiles <= 0) return ARD_OK;
  if (F.splits < 1) F.splits = 1;
  // an XCD's share should be about square in tiles: bands of group_m tile rows
  const int per_xcd = ceil_div(F.total_tiles, 8);
  int gm = 1;
  while (gm * gm * 2 <= per_xcd && gm < 8) gm *= 2;
  F.group_m = gm;
  const int grid = fast_grid(F);
  if (bm == 256 && bn == 256) return launch_direct_cfg<256, 256, 8>(a_kc, b_kc, F, grid, stream);
  if (bm == 256 && bn == 128) return launch_direct_cfg<256, 128, 8>(a_kc, b_kc, F, grid, stream);
  if (bm == 128 && bn == 128) return launch_direct_cfg<128, 128, 4>(a_kc, b_kc, F, grid, stream);
  if (bm == 128 && bn == 64) return launch_direct_cfg<128, 64, 4>(a_kc, b_kc, F, grid, stream);
  if (bm == 64 && bn == 64) return launch_direct_cfg<64, 64, 4>(a_kc, b_kc, F, grid, stream);
  return fail(ARD_EUNSUPPORTED, "tile configuration not built");
}

static bool fast_ptr_ok(const void* p, long ld) { return ((uintptr_t)p & 15) == 0 && (ld % 8) == 0 && ld < (1L << 24); }

// bf16 products whose operands can be fetched with 16-byte loads go through the LDS-direct
// kernels; results that the kernel cannot store itself (split contraction, element-level
// scatter with zero fill) pass through fp32 partials in the workspace and a finishing kernel.
static bool try_direct(int32_t dtype, bool a_kc, bool b_kc, const GemmParams& P, void* ws, size_t ws_bytes,
                       hipStream_t stream, int32_t& st, int* raw_splits) {
  if (dtype != ARD_BF16 || dev_knobs().no_fast) return false;
  if (!P.A.vec || !P.B.vec || P.kb_ptr || P.tmask) return false;
  Axis k = P.k;
  auto ident = [](const Axis& a) { return a.kind == AX_AFFINE && a.off == 0 && a.step == 1; };
  if (P.A.kdense && P.B.kdense) k = axis_identity(P.k.n);
  else if ((P.A.kdense || P.B.kdense) && !ident(P.k)) return false;
  if (k.kind != AX_AFFINE || k.step != 1 || (k.off % 8)) return false;
  if ((k.n % 8) && (a_kc || b_kc)) {
    // (an operand whose rows run along the contraction ends at any row: only contraction-contiguous ones
    // are fetched in pieces of 8.)  Both operands carry zero padding along the contraction: run it to the
    // padded length
    if (!P.A.kpad || !P.B.kpad || !ident(k)) return false;
    k = axis_identity(pad8(k.n));
  }
  Axis ax_m = P.A.r, ax_n = P.B.r;
  if (!a_kc && (ax_m.n % 8)) {
    if (!P.A.rpad || !ident(ax_m)) return false;
    ax_m = axis_identity(pad8(ax_m.n));
  }
  if (!b_kc && (ax_n.n % 8)) {
    if (!P.B.rpad || !ident(ax_n)) return false;
    ax_n = axis_identity(pad8(ax_n.n));
  }
  const OutMat& C = P.C;
  if (C.plane) return false;
  if (!fast_ptr_ok(P.A.p, P.A.ld) || !fast_ptr_ok(P.B.p, P.B.ld)) return false;
  if ((long)P.A.r.nphys * P.A.ld >= (1L << 31) || (long)P.B.r.nphys * P.B.ld >= (1L << 31)) return false;
  if ((long)P.M * P.N >= (1L << 31)) return false;
  // rows of A beyond its extent would be stored (only columns beyond B's are zeroed by the kernel)
  if (ax_m.n < P.M || ax_m.n < 1 || ax_n.n < 1 || (!b_kc && ax_n.n < P.N)) return false;
  const bool direct_out = ident(C.rm) && ident(C.cn);
  if (!direct_out) {
    auto inv_ok = [](const Axis& a) { return a.kind == AX_AFFINE || a.kind == AX_LIST; };
    if (!inv_ok(C.rm) || !inv_ok(C.cn)) return false;
  }
  // workgroup tile: the largest one that still fills the chip; then split the contraction of
  // products with too few tiles
  const int steps = ceil_div(k.n, 64);
  int bm = 64, bn = 64;
  long tiles = 0;
  const bool plain_out = !raw_splits && direct_out && !C.out_f32 && C.beta == 0.0f && !C.relu_src;
  for (const TileCfg& c : kTileCfgs) {
    if (c.bm == 256 && c.bn == 256 && !plain_out) continue;  // that tile only stores plain bf16
    tiles = (long)ceil_div(P.M, c.bm) * ceil_div(P.N, c.bn);
    bm = c.bm, bn = c.bn;
    // An 8-wavefront tile wants a workgroup per CU; a 4-wavefront tile runs one wavefront per SIMD
    // and wants two workgroups per CU to overlap its waits (measured at batch 1024: 256 tiles of
    // 128 x 64 take 23.5 us where 512 tiles of 64 x 64 take 15.8 us).
    if (tiles >= (c.bm * c.bn >= 256 * 128 ? 220 : 440)) break;
  }
  if (tiles >= (1L << 24)) return false;
  // A scattered bf16 output with zero fill through affine maps is stored by the product's own
  // epilogue (no partial sums, no finishing pass) unless the product is so small that it has to
  // be split to occupy the chip at all.
  auto owns_groups = [](const Axis& a) { return a.kind == AX_AFFINE && a.step >= 1 && a.off < a.step; };
  bool scatter = !raw_splits && !direct_out && C.fill && !C.out_f32 && C.beta == 0.0f && owns_groups(C.rm) && owns_groups(C.cn) &&
                 (long)C.rm.nphys * C.ld < (1L << 31) && !dev_knobs().no_scatter;
  if (scatter) {
    // tile: as large as still gives every CU a workgroup; at least 64 workgroups or no scatter
    bm = bn = 64;
    for (const TileCfg& c : kTileCfgs) {
      if (c.bm == 256 && c.bn == 256) continue;
      const long t = (long)ceil_div(P.M, c.bm) * ceil_div(P.N, c.bn);
      if (t >= 220) {
        bm = c.bm, bn = c.bn;
        break;
      }
    }
    tiles = (long)ceil_div(P.M, bm) * ceil_div(P.N, bn);
    const long region = (long)bm * C.rm.step * bn * C.cn.step;
    // Measured on the weight gradients of the MLP chain, every (row step, column step) in 1..8:
    // what the epilogue costs grows with the column step (rows of the owned region get long and
    // ragged).  With identity columns it always beats the finishing pass; with column step 2 up
    // to row step 4; beyond that only while the region is small or the tiles many, and never for
    // column groups wider than 4 (25 us against 15 us through the pass).
    // What made wide groups slow was the volume of zeros a tile had to write for the dropped ROWS of its
    // region (step^2 times its own size, by 16 to 64 workgroups): those rows are now zeroed by a pass of
    // their own that runs beside the product (zero_rows_kernel), the tile writes its kept rows in full.
    const int cs = C.cn.step;
    (void)region;
    scatter = cs == 1 ? tiles >= 4 : tiles >= 64;
  }
  // Splitting the contraction s ways shortens a workgroup's loop by steps * (1 - 1/s) steps of about
  // 0.19 us (a step takes that long however few tiles there are), and costs about 2.6 us per
  // additional split in the pass that sums the partial sums (they come back from memory, written
  // by other XCDs), plus the pass itself (about 6 us) for a product that could have stored its own
  // result.  Measured on 256 x 784 x 1024: 8.4 + 6.2 us unsplit against 6.6 + 19.8 us in 6 splits.
  // A caller that sums the partials in a kernel it runs anyway (LSTM cell) keeps the old rule.
  int splits = 1;
  if (!scatter && tiles < 160 && steps >= 4) {
    int cap = (int)(320 / tiles);
    if (cap > steps / 2) cap = steps / 2;
    if (cap > 8) cap = 8;
    if (cap < 1) cap = 1;
    if (raw_splits) {
      splits = cap;
    } else {
      const bool own_store = direct_out;  // no pass needed without a split
      float best = 0.0f;
      for (int sp = 2; sp <= cap; ++sp) {
        const float gain = steps * 0.19f * (1.0f - 1.0f / sp) - 2.6f * (sp - 1) - (own_store ? 6.0f : 0.0f);
        if (gain > best) best = gain, splits = sp;
      }
    }
  }
  if (bm == 256 && bn == 256) splits = 1;
  size_t need = (splits > 1 || raw_splits || (!direct_out && !scatter)) ? (size_t)splits * P.M * P.N * 4 : 0;
  if (raw_splits && (need > ws_bytes || !ws)) return false;
  if (need > ws_bytes || (need && !ws)) {
    if (!direct_out) return false;  // no room for the partials: the general kernel scatters itself
    splits = 1;
    need = 0;
  }
  bool self_batch = false;
  ZeroRowsArgs zero_args{};
  long zero_gx = 0;
  FastParams F{};
  F.A = (const uint16_t*)P.A.p;
  F.B = (const uint16_t*)P.B.p;
  F.C = (uint16_t*)C.p;
  F.lda = (int)P.A.ld;
  F.ldb = (int)P.B.ld;
  F.ldc = (int)C.ld;
  // what the caller's matrices hold: physical rows x leading dimension (a contraction-strided operand
  // has one stored row per contraction index)
  F.a_elems = (long)(a_kc ? P.A.r.nphys : k.nphys) * P.A.ld;
  F.b_elems = (long)(b_kc ? P.B.r.nphys : k.nphys) * P.B.ld;
  F.am = ax_m;
  F.bn = ax_n;
  F.k = k;
  F.alpha = C.alpha;
  F.beta = C.beta;
  F.relu = C.relu;
  F.out_f32 = C.out_f32;
  F.relu_src = (const uint16_t*)C.relu_src;
  F.part = need ? (float*)ws : nullptr;
  F.splits = splits;
  F.M = P.M;
  F.N = P.N;
  F.tiles_m = ceil_div(P.M, bm);
  F.tiles_n = ceil_div(P.N, bn);
  F.total_tiles = (int)tiles;
  if (scatter && !need) {
    F.scatter = 1;
    F.srm = C.rm;
    F.scn = C.cn;
    F.scatter_vec = (C.cn.nphys % 8) == 0 && (C.ld % 8) == 0 && ((uintptr_t)C.p & 15) == 0 &&
                    (!C.relu_src || ((uintptr_t)C.relu_src & 15) == 0) && C.cn.nphys < (1 << 23);
    const int dropped_rows = C.rm.nphys - C.rm.n;
    if (C.rm.step > 1 && dropped_rows > 0) {
      // dropped rows: their own pass over all CUs (recorded with the product in a grouped launch; a call that
      // is not part of a caller's batch makes one of its own for the two)
      F.scatter_rows_only = 1;
      self_batch = batch_self_begin();
      zero_args = ZeroRowsArgs{(uint16_t*)C.p, (int)C.ld, C.rm.nphys, C.cn.nphys, C.rm.off, C.rm.step, C.rm.n, F.scatter_vec};
      const long pieces = (long)dropped_rows * (F.scatter_vec ? C.cn.nphys / 8 : C.cn.nphys);
      zero_gx = (pieces + 1023) / 1024;  // four stores per thread
      zero_gx = zero_gx < 1 ? 1 : (zero_gx > 2048 ? 2048 : zero_gx);
      // (recorded behind the product: the product's workgroups have the longer way to go and start first)
    }
  }
  const long total = C.fill ? (long)C.rm.nphys * C.cn.nphys : (long)P.M * P.N;
  const int out_cols = C.fill ? C.cn.nphys : P.N;
  const bool vec_out = !C.out_f32 && C.beta == 0.0f && (out_cols % 8) == 0 && (C.ld % 8) == 0 &&
                       ((uintptr_t)C.p & 15) == 0 && (!C.relu_src || ((uintptr_t)C.relu_src & 15) == 0) &&
                       (C.fill || ident(C.cn)) && out_cols < (1 << 23);
  if (raw_splits || (need && !vec_out)) {
    // whoever sums these partial sums is not a recordable kernel: the product runs at once
    BatchSuspend now;
    st = launch_direct(a_kc, b_kc, F, bm, bn, stream);
  } else {
    st = launch_direct(a_kc, b_kc, F, bm, bn, stream);
  }
  if (zero_gx && st == ARD_OK) {
    if (!batch_push_zero_rows(zero_args, (int)zero_gx)) ARD_LAUNCH(zero_rows_kernel, dim3((unsigned)zero_gx), dim3(256), 0, stream, zero_args);
    const hipError_t e = ard::launch_status();
    if (e != hipSuccess) st = fail(ARD_EHIP, "launch of zero_rows_kernel failed: %s", hipGetErrorString(e));
  }
  if (self_batch) {
    const int32_t bst = batch_self_end(st == ARD_OK, stream);
    if (!st) st = bst;
  }
  if (raw_splits) {
    *raw_splits = splits;
    return true;
  }
  if (st || !need) return true;
  long blocks = (total + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  if (vec_out) {
    const int out_rows = C.fill ? C.rm.nphys : P.M;
    const int grid_rows = ceil_div(out_rows, 8) * 8;  // the pass deals rows to the XCDs in eighths
    dim3 grid((unsigned)ceil_div(out_cols / 8, 256), (unsigned)(grid_rows < 32768 ? grid_rows : 32768));
    const FinishArgs fa{(const float*)ws, splits, P.M, P.N, C};
    if (!batch_push_finish(fa, (int)grid.x, (int)grid.y)) ARD_LAUNCH(gemm_finish_vec_kernel, grid, dim3(256), 0, stream, fa);
  }
  else
    ARD_LAUNCH(gemm_finish_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)ws,
                       splits, P.M, P.N, C);
  hipError_t e = ard::launch_status();
  if (e != hipSuccess) st = fail(ARD_EHIP, "launch of gemm_finish_kernel failed: %s", hipGetErrorString(e));
  return true;
}

static int elem_size(int32_t dtype) { return dtype == ARD_BF16 ? 2 : 4; }
static int chunk_elems(int32_t dtype) { return 16 / elem_size(dtype); }
static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

int32_t fill_matrix(int32_t dtype, void* p, long n, float beta, hipStream_t stream) {
  if (n <= 0 || beta == 1.0f) return ARD_OK;
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == ARD_BF16)
    ARD_LAUNCH(scale_fill_kernel<uint16_t>, grid, block, 0, stream, (uint16_t*)p, n, beta);
  else
    ARD_LAUNCH(scale_fill_kernel<float>, grid, block, 0, stream, (float*)p, n, beta);
  ARD_LAUNCH_CHECK("scale_fill_kernel");
  return ARD_OK;
}

struct LayerArgs {
  int32_t dtype, B, I, O;
  const ard_pattern *po, *pi;
  bool tile;
  int TR, TC;
};

static int32_t check_layer(LayerArgs& a, const void* p0, const void* p1, const void* p2) {
  if (a.dtype != ARD_F32 && a.dtype != ARD_BF16) return fail(ARD_EDTYPE, "unknown dtype %d", a.dtype);
  if (a.B <= 0 || a.I <= 0 || a.O <= 0) return fail(ARD_ESHAPE, "B, I, O must be positive (got %d, %d, %d)", a.B, a.I, a.O);
  if (!p0 || !p1 || !p2) return fail(ARD_EINVAL, "null tensor pointer");
  a.tile = a.po && a.po->kind == ARD_PAT_TILE;
  if (a.pi && a.pi->kind == ARD_PAT_TILE) return fail(ARD_EINVAL, "a tile pattern goes in pat_out");
  if (a.tile) {
    if (a.pi && a.pi->kind != ARD_PAT_NONE) return fail(ARD_EINVAL, "tile pattern cannot be combined with pat_in");
    if (a.po->tile_r <= 0 || a.po->tile_c <= 0) return fail(ARD_EINVAL, "tile size must be positive");
    a.TR = ceil_div(a.O, a.po->tile_r);
    a.TC = ceil_div(a.I, a.po->tile_c);
    int32_t st = check_pattern(a.po, a.TR * a.TC, "pat_out");
    if (st) return st;
    if (a.po->tile_r % 32 || a.po->tile_c % 32)
      return fail(ARD_EUNSUPPORTED, "tile sizes must be multiples of 32 (got %d x %d)", a.po->tile_r, a.po->tile_c);
  } else {
    int32_t st = check_pattern(a.po, a.O, "pat_out");
    if (st) return st;
    st = check_pattern(a.pi, a.I, "pat_in");
    if (st) return st;
  }
  return ARD_OK;
}

// Workspace layout for a tile pattern: mask | keep | count | rowptr | colptr | csc_rows
struct TileLists {
  const uint8_t* mask;
  const int32_t *keep, *rowptr, *colptr, *csc_rows;
};

static size_t tile_ws_bytes(int TR, int TC) {
  size_t n = (size_t)TR * TC;
  return align_up(n, 256) + align_up(n * 4, 256) + 256 + align_up((size_t)(TR + 1) * 4, 256) +
         align_up((size_t)(TC + 1) * 4, 256) + align_up(n * 4, 256);
}

static int32_t tile_lists(const LayerArgs& a, void* ws, size_t ws_bytes, hipStream_t stream, TileLists& L) {
  const ard_pattern* p = a.po;
  if (p->d_keep && p->d_mask && p->d_rowptr && p->d_colptr && p->d_csc_rows) {
    L = TileLists{p->d_mask, p->d_keep, p->d_rowptr, p->d_colptr, p->d_csc_rows};
    return ARD_OK;
  }
  size_t need = tile_ws_bytes(a.TR, a.TC);
  if (!ws || ws_bytes < need) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", need, ws_bytes);
  size_t n = (size_t)a.TR * a.TC;
  char* w = (char*)ws;
  uint8_t* mask = (uint8_t*)w;
  w += align_up(n, 256);
  int32_t* keep = (int32_t*)w;
  w += align_up(n * 4, 256);
  int32_t* count = (int32_t*)w;
  w += 256;
  int32_t* rowptr = (int32_t*)w;
  w += align_up((size_t)(a.TR + 1) * 4, 256);
  int32_t* colptr = (int32_t*)w;
  w += align_up((size_t)(a.TC + 1) * 4, 256);
  int32_t* csc = (int32_t*)w;
  int32_t st = pattern_gen_launch(p, a.O, a.I, mask, keep, count, rowptr, colptr, csc, stream);
  if (st) return st;
  L = TileLists{mask, keep, rowptr, colptr, csc};
  return ARD_OK;
}

// Tile pattern on the large-tile path: classes of tile rows / columns (see fast.hpp).
// op 0: Y = X . W^T   1: dX = dY . W   2: dW = dY^T . X
static bool try_fast_tile(int op, const LayerArgs& a, const void* Ap, const void* Bp, void* Cp, float alpha, int relu,
                          hipStream_t stream, int32_t& st, const void* relu_src = nullptr) {
  if (a.dtype != ARD_BF16 || dev_knobs().no_fast) return false;
  const int x = a.po->tile_r, y = a.po->tile_c, dp = a.po->dp, o = a.po->b - 1, TR = a.TR, TC = a.TC;
  const int B = a.B, I = a.I, O = a.O;
  if ((I % 8) || (O % 8) || (long)B * O >= (1L << 31) || (long)B * I >= (1L << 31) || (long)O * I >= (1L << 31)) return false;
  if (((uintptr_t)Ap & 15) || ((uintptr_t)Bp & 15)) return false;
  const int g = gcd_int(TC, dp), Pp = dp / g;
  FastParams F{};
  ClassTab& t = F.tab;
  auto cnt = [](int total, int first, int step) { return first < total ? (total - first + step - 1) / step : 0; };
  if (op == 0) {
    // contraction blocks: whole 64-deep steps, or the 32-wide tiles of Section 3.2 taken two per step
    if ((256 % x) || ((y % 64) && y != 32) || Pp > F_MAXCLS) return false;
    t.ncls = Pp;
    t.n_step = Pp, t.n_bs = x, t.n_phys = O;
    t.k_step = dp, t.k_bs = y, t.k_phys = I;
    for (int c = 0; c < Pp; ++c) {
      t.n_off[c] = c;
      t.n_cnt[c] = cnt(TR, c, Pp);
      const int t0 = (int)((((long)o - (long)c * TC) % dp + dp) % dp);
      t.k_off[c] = t0;
      t.k_cnt[c] = cnt(TC, t0, dp);
      t.mblk[c] = 1;
    }
    F.A = (const uint16_t*)Ap, F.lda = I, F.am = axis_identity(B);
    F.B = (const uint16_t*)Bp, F.ldb = I;
    F.a_elems = (long)B * I, F.b_elems = (long)O * I;
    F.C = (uint16_t*)Cp, F.ldc = O;
    F.c_cols_mapped = 1;
    F.M = B, F.N = O;
  } else if (op == 1) {
    if ((256 % y) || ((x % 64) && x != 32) || dp > F_MAXCLS) return false;
    t.ncls = dp;
    t.n_step = dp, t.n_bs = y, t.n_phys = I;
    t.k_step = Pp, t.k_bs = x, t.k_phys = O;
    for (int c = 0; c < dp; ++c) {
      t.n_off[c] = c;
      t.n_cnt[c] = cnt(TC, c, dp);
      int J0 = -1;
      for (int J = 0; J < Pp; ++J)
        if ((((long)J * TC + c - o) % dp + dp) % dp == 0) {
          J0 = J;
          break;
        }
      t.k_off[c] = J0 < 0 ? 0 : J0;
      t.k_cnt[c] = J0 < 0 ? 0 : cnt(TR, J0, Pp);
      t.mblk[c] = 1;
    }
    F.A = (const uint16_t*)Ap, F.lda = O, F.am = axis_identity(B);
    F.B = (const uint16_t*)Bp, F.ldb = I;
    F.a_elems = (long)B * O, F.b_elems = (long)O * I;
    F.C = (uint16_t*)Cp, F.ldc = I;
    F.c_cols_mapped = 1;
    F.M = B, F.N = I;
  } else {
    if ((256 % x) || (256 % y) || (x % 8) || (y % 8) || Pp > F_MAXCLS) return false;
    t.ncls = Pp;
    t.m_step = Pp, t.m_bs = x, t.m_phys = O;
    t.n_step = dp, t.n_bs = y, t.n_phys = I;
    t.k_bs = 0;
    for (int c = 0; c < Pp; ++c) {
      t.m_off[c] = c;
      t.m_cnt[c] = cnt(TR, c, Pp);
      const int t0 = (int)((((long)o - (long)c * TC) % dp + dp) % dp);
      t.n_off[c] = t0;
      t.n_cnt[c] = cnt(TC, t0, dp);
      t.mblk[c] = ceil_div(t.m_cnt[c], 256 / x);
    }
    F.A = (const uint16_t*)Ap, F.lda = O;
    F.B = (const uint16_t*)Bp, F.ldb = I;
    F.a_elems = (long)B * O, F.b_elems = (long)B * I;
    F.k = axis_identity(B);
    F.C = (uint16_t*)Cp, F.ldc = I;
    F.c_rows_mapped = F.c_cols_mapped = 1;
    F.M = O, F.N = I;
  }
  // workgroups per class for a BM x BN tile; "heavy" ones have something to contract
  auto count = [&](int bm, int bn, int& heavy) {
    int total = 0;
    heavy = 0;
    for (int c = 0; c < t.ncls; ++c) {
      const int mb = op == 2 ? ceil_div(t.m_cnt[c], bm / x) : ceil_div(B, bm);
      const int nb = ceil_div(t.n_cnt[c], bn / t.n_bs);
      t.mblk[c] = mb > 0 ? mb : 1;
      t.nblk[c] = (t.n_cnt[c] > 0 && mb > 0) ? mb * nb : 0;
      total += t.nblk[c];
      if (op == 2 || t.k_cnt[c] > 0) heavy += t.nblk[c];
    }
    return total;
  };
  // Tile choice by estimated time: rounds of workgroups over the chip x contraction steps x the time one
  // round of one step takes with that tile.  A period that does not divide the tile grid leaves classes of
  // 21 or 13 tile rows: wide tiles then end in a mostly empty block and the workgroup count lands just above
  // a multiple of the CU count (288 for dp = 3), which smaller tiles avoid.  Round times (us) measured on
  // the dense 4096^3 product per tile and operand layout; an 8-wavefront tile has one slot per CU, a
  // 4-wavefront tile two.
  static const float kRoundUs[3][5] = {{2.21f, 1.33f, 1.32f, 0.79f, 0.464f},   // forward (both operands contraction-contiguous)
                                       {2.04f, 1.19f, 1.17f, 0.70f, 0.43f},    // data gradient
                                       {1.98f, 1.14f, 1.16f, 0.66f, 0.44f}};   // weight gradient
  int steps = op == 2 ? ceil_div(B, 64) : 0;
  if (op != 2)
    for (int c = 0; c < t.ncls; ++c) steps = imax(steps, ceil_div(t.k_cnt[c] * t.k_bs, 64));
  int heavy = 0, bm = 0, bn = 0, total = 0;
  float best = 0.0f;
  for (int ci = 0; ci < 5; ++ci) {
    const TileCfg& c = kTileCfgs[ci];
    if ((c.bn % t.n_bs) || (op == 2 && (c.bm % x))) continue;
    if (dev_knobs().class_tile && ci != dev_knobs().class_tile - 1) continue;
    if (relu_src && c.bm == 256 && c.bn == 256) continue;  // (that tile only stores plain results)
    int h = 0;
    const int tot = count(c.bm, c.bn, h);
    if (tot == 0) continue;
    const int slots = c.bm * c.bn >= 256 * 128 ? 256 : 512;
    const float est = (float)ceil_div(h > 0 ? h : 1, slots) * (float)steps * kRoundUs[op][ci];
    if (bm == 0 || est < best) best = est, bm = c.bm, bn = c.bn;
  }
  if (bm == 0) return false;
  total = count(bm, bn, heavy);
  if (total == 0) return false;
  // (however few tiles there are, this path wins: the general engine's block-list products take 2-3x as
  // long even on a batch of 128 rows)
  F.alpha = alpha;
  F.relu = relu;
  F.relu_src = (const uint16_t*)relu_src;
  F.total_tiles = total;
  if (op == 2) {
    ARD_LAUNCH(zero_dropped_tiles_kernel, dim3((unsigned)(TR * TC)), dim3(256), 0, stream, (uint16_t*)Cp, I, O, I,
                       x, y, TC, dp, o);
    hipError_t e = ard::launch_status();
    if (e != hipSuccess) {
      st = fail(ARD_EHIP, "launch of zero_dropped_tiles_kernel failed: %s", hipGetErrorString(e));
      return true;
    }
  }
  F.splits = 1;
  st = launch_direct(op != 2, op == 0, F, bm, bn, stream);
  return true;
}

static int pick_bn(int t) { return t % 128 == 0 ? 128 : (t % 64 == 0 ? 64 : 32); }

}  // namespace ard

using namespace ard;

namespace ard {

// Wc[r][c] = W[out(r)][in(c)]; rows and columns up to the next multiple of 8 are zero
struct CompactWArgs {
  const void* W;
  void* Wc;
  long ld;
  Axis ao, ai;
};
// a workgroup gathers kCwRows rows x 256 columns: a thread's loads of its rows are independent and in
// flight together
constexpr int kCwRows = 16;
template <typename T>
__device__ __forceinline__ void compact_weight_body(const CompactWArgs& a, const int bx, const int by) {
  const int c = bx * 256 + threadIdx.x;
  const int cols = pad8(a.ai.n), rows = pad8(a.ao.n);
  if (c >= cols) return;
  const T* W = reinterpret_cast<const T*>(a.W);
  T* Wc = reinterpret_cast<T*>(a.Wc);
  const bool c_ok = c < a.ai.n;
  const long pc = c_ok ? ax_phys(a.ai, c) : 0;
  T v[kCwRows];
#pragma unroll
  for (int i = 0; i < kCwRows; ++i) {
    const int r = by * kCwRows + i;
    const bool ok = c_ok && r < a.ao.n;
    const T t = W[(long)(ok ? ax_phys(a.ao, r) : 0) * a.ld + pc];  // unconditional (clamped) load
    v[i] = ok ? t : (T)0;
  }
#pragma unroll
  for (int i = 0; i < kCwRows; ++i) {
    const int r = by * kCwRows + i;
    if (r < rows) Wc[(long)r * cols + c] = v[i];
  }
}
template <typename T>
__global__ __launch_bounds__(256) void compact_weight_kernel(const CompactWArgs a) {
  compact_weight_body<T>(a, (int)blockIdx.x, (int)blockIdx.y);
}
static bool batch_push_compact_w(const CompactWArgs& a, int gx, int gy);

// out[r][c] = c < cols ? in[r*cols + c] : 0 for c < pad8(cols): aligned copy of a narrow activation
template <typename T>
__global__ void pad_cols_kernel(const T* in, int rows, int cols, T* out) {
  const int pc = pad8(cols);
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)rows * pc) return;
  const int r = (int)(idx / pc), c = (int)(idx - (long)r * pc);
  out[idx] = c < cols ? in[(long)r * cols + c] : (T)0;
}

static int32_t compact_weight(int32_t dtype, int I, const void* W, void* Wc, const Axis& ao, const Axis& ai,
                              hipStream_t stream) {
  if (ao.n <= 0 || ai.n <= 0) return ARD_OK;
  if (ceil_div(pad8(ao.n), kCwRows) > 65535) return fail(ARD_ESHAPE, "too many kept output neurons for one launch");
  dim3 grid(ceil_div(pad8(ai.n), 256), ceil_div(pad8(ao.n), kCwRows)), block(256);
  const CompactWArgs ca{W, Wc, (long)I, ao, ai};
  if (dtype == ARD_BF16) {
    if (!batch_push_compact_w(ca, (int)grid.x, (int)grid.y)) ARD_LAUNCH(compact_weight_kernel<uint16_t>, grid, block, 0, stream, ca);
  } else {
    ARD_LAUNCH(compact_weight_kernel<float>, grid, block, 0, stream, ca);
  }
  ARD_LAUNCH_CHECK("compact_weight_kernel");
  return ARD_OK;
}

// A [rows x cols] activation whose rows are not 16-byte aligned (cols % 8 != 0, bf16) is
// copied once into the workspace with zero-padded rows, so the product can use 16-byte loads.
// Returns the pointer to use and its leading dimension; advances ws_off.
static int32_t aligned_activation(int32_t dtype, const void* p, int rows, int cols, void* ws, size_t ws_bytes,
                                  size_t& ws_off, hipStream_t stream, const void*& out, int& ld) {
  out = p;
  ld = cols;
  if (dtype != ARD_BF16 || (cols % 8) == 0 || cols > 256) return ARD_OK;
  const size_t need = align_up((size_t)rows * pad8(cols) * 2, 256);
  if (!ws || ws_off + need > ws_bytes) return ARD_OK;  // no room: the general kernel copes with the original
  uint16_t* dst = (uint16_t*)((char*)ws + ws_off);
  const long total = (long)rows * pad8(cols);
  ARD_LAUNCH(pad_cols_kernel<uint16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     (const uint16_t*)p, rows, cols, dst);
  ARD_LAUNCH_CHECK("pad_cols_kernel");
  ws_off += need;
  out = dst;
  ld = pad8(cols);
  return ARD_OK;
}

constexpr int32_t kLayoutFlags = ARD_IN_COMPACT | ARD_OUT_COMPACT | ARD_W_COMPACT | ARD_DW_COMPACT;
static bool is_identity(const Axis& a) { return a.kind == AX_AFFINE && a.off == 0 && a.step == 1; }

// Row / list pattern layer: resolves the layout flags into operand descriptions.
struct RowLayer {
  Axis ao, ai;      // kept output / input neurons
  bool in_c, out_c; // activations compact on the input / output side
  const void* Wp;   // weight operand actually multiplied
  long w_ld;
  Axis w_rows, w_cols;  // maps into Wp (identity when Wp is compact)
  bool w_compact;
  size_t ws_used;  // bytes of the workspace taken by the gathered weight
};

static int32_t resolve_row_layer(const LayerArgs& a, int32_t flags, const void* W, bool need_w, void* ws, size_t ws_bytes,
                                 hipStream_t stream, RowLayer& L) {
  if (flags & ~(ARD_IN_COMPACT | ARD_OUT_COMPACT | ARD_W_COMPACT | ARD_DW_COMPACT))
    return fail(ARD_EINVAL, "unknown flag bits 0x%x", flags);
  L.ao = axis_of_pattern(a.po, a.O);
  L.ai = axis_of_pattern(a.pi, a.I);
  L.in_c = (flags & ARD_IN_COMPACT) != 0;
  L.out_c = (flags & ARD_OUT_COMPACT) != 0;
  L.Wp = W;
  L.w_ld = a.I;
  L.w_rows = L.ao;
  L.w_cols = L.ai;
  L.w_compact = false;
  L.ws_used = 0;
  if (!need_w) return ARD_OK;
  const int es = a.dtype == ARD_BF16 ? 2 : 4;
  if (flags & ARD_W_COMPACT) {
    L.w_compact = true;
  } else if (!is_identity(L.ai) && L.ai.n > 0 && L.ao.n > 0) {
    // the kept input neurons are strided along the contiguous axis of W: gather the kept block once
    const size_t need = (size_t)pad8(L.ao.n) * pad8(L.ai.n) * es;
    if (!ws || ws_bytes < need) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", need, ws_bytes);
    int32_t st;
    {
      BatchSuspend now;  // the product of this very call reads the gathered block
      st = compact_weight(a.dtype, a.I, W, ws, L.ao, L.ai, stream);
    }
    if (st) return st;
    L.Wp = ws;
    L.w_compact = true;
    L.ws_used = align_up(need, 256);
  }
  if (L.w_compact) {
    L.w_ld = pad8(L.ai.n);
    L.w_rows = axis_identity(pad8(L.ao.n));
    L.w_cols = axis_identity(pad8(L.ai.n));
  }
  return ARD_OK;
}

}  // namespace ard


// ---- grouped launches ----------------------------------------------------------------------------
//
// A training iteration of a small layer chain is a handful of products of a few microseconds each,
// so what it costs is mostly the fixed part of every launch.  Calls that do not depend on each other
// (the weight compaction and the first forward product; the three products of the classifier layer;
// the weight and data gradients of a hidden layer) can be recorded and then issued as one grid of
// group_kernel, which holds the bodies of every kernel such a chain uses (all run 256 threads per
// workgroup); each workgroup looks up the segment of the grid it belongs to and runs that body.
namespace ard {

constexpr int kGroupMaxSeg = 6;
constexpr int kGroupArgBytes = 3584;
struct GroupSeg {
  int kind;      // GK_*
  int first;     // first workgroup of the segment (a multiple of 8: workgroup ids go round-robin over the XCDs)
  int nblocks;   // gx * gy
  int gx, gy;
  int arg_off;   // byte offset of the body's argument struct in GroupTable::args
};
struct GroupTable {
  int nseg;
  GroupSeg seg[kGroupMaxSeg];
  alignas(16) char args[kGroupArgBytes];
};
static_assert(sizeof(GroupTable) <= 4096, "kernel arguments are limited to 4 KiB");

// (The table is read through the kernel-argument segment itself: indexing the by-value parameter with a
// run-time segment number would make the compiler copy all of it into every lane's private memory.)
__global__ __launch_bounds__(256) void group_kernel(const GroupTable table_in_kernarg) {
  extern __shared__ uint4 group_lds[];
  const GroupTable& T = *(const GroupTable*)__builtin_amdgcn_kernarg_segment_ptr();
  int s = 0;
  while (s + 1 < T.nseg && (int)blockIdx.x >= T.seg[s + 1].first) ++s;
  const GroupSeg sg = T.seg[s];
  const int local = (int)blockIdx.x - sg.first;
  if (local >= sg.nblocks) return;
  const char* arg = T.args + sg.arg_off;
  switch (sg.kind) {
    case GK_DIRECT_KK_64:
      direct_body<true, true, 64, 64, 4, 0>(*reinterpret_cast<const FastParams*>(arg), local, group_lds);
      break;
    case GK_DIRECT_KM_64:
      direct_body<true, false, 64, 64, 4, 0>(*reinterpret_cast<const FastParams*>(arg), local, group_lds);
      break;
    case GK_DIRECT_MM_64:
      direct_body<false, false, 64, 64, 4, 0>(*reinterpret_cast<const FastParams*>(arg), local, group_lds);
      break;
    case GK_DIRECT_MM_128x64:
      direct_body<false, false, 128, 64, 4, 0>(*reinterpret_cast<const FastParams*>(arg), local, group_lds);
      break;
    case GK_SKINNY_FWD:
      skinny_fwd_body(*reinterpret_cast<const SkinnyArgs*>(arg), local, group_lds);
      break;
    case GK_SKINNY_BWD_DATA:
      skinny_bwd_data_body(*reinterpret_cast<const SkinnyArgs*>(arg), local % sg.gx, local / sg.gx, group_lds);
      break;
    case GK_SKINNY_BWD_WEIGHT:
      skinny_bwd_weight_body(*reinterpret_cast<const SkinnyArgs*>(arg), local, group_lds);
      break;
    case GK_COMPACT_W:
      compact_weight_body<uint16_t>(*reinterpret_cast<const CompactWArgs*>(arg), local % sg.gx, local / sg.gx);
      break;
    case GK_FINISH_VEC:
      finish_vec_body(*reinterpret_cast<const FinishArgs*>(arg), local % sg.gx, local / sg.gx, sg.gy);
      break;
    case GK_ZERO_ROWS:
      zero_rows_body(*reinterpret_cast<const ZeroRowsArgs*>(arg), local, sg.nblocks);
      break;
    default:
      break;
  }
}

struct BatchItem {
  int kind, stage, gx, gy;
  size_t lds, arg_bytes;
  alignas(16) char args[1024];
};
struct Batch {
  bool open = false;
  int suspended = 0;  // live BatchSuspend objects
  std::vector<BatchItem> items;
};
static thread_local Batch g_batch;

bool batch_open() { return g_batch.open; }
BatchSuspend::BatchSuspend() : was_open(g_batch.open) {
  g_batch.open = false;
  ++g_batch.suspended;
}
BatchSuspend::~BatchSuspend() {
  g_batch.open = was_open;
  --g_batch.suspended;
}
bool batch_self_begin() {
  if (g_batch.open || g_batch.suspended > 0 || !g_batch.items.empty()) return false;
  g_batch.open = true;
  return true;
}
int32_t batch_self_end(bool ok, hipStream_t stream) {
  if (!ok) {
    g_batch.open = false;
    g_batch.items.clear();
    return ARD_OK;
  }
  return ard_batch_launch(stream);
}

static bool batch_push(int kind, int stage, const void* args, size_t arg_bytes, int gx, int gy, size_t lds) {
  if (!g_batch.open) return false;
  if (arg_bytes > sizeof(BatchItem::args) || gx < 1 || gy < 1 || (long)gx * gy >= (1L << 30)) return false;
  BatchItem it{};
  it.kind = kind, it.stage = stage, it.gx = gx, it.gy = gy, it.lds = lds, it.arg_bytes = arg_bytes;
  memcpy(it.args, args, arg_bytes);
  g_batch.items.push_back(it);
  return true;
}
bool batch_push_direct(int kind, const FastParams& F, int grid_x, size_t lds_bytes) {
  return batch_push(kind, 0, &F, sizeof(F), grid_x, 1, lds_bytes);
}
bool batch_push_finish(const FinishArgs& a, int gx, int gy) { return batch_push(GK_FINISH_VEC, 1, &a, sizeof(a), gx, gy, 0); }
bool batch_push_zero_rows(const ZeroRowsArgs& a, int gx) { return batch_push(GK_ZERO_ROWS, 0, &a, sizeof(a), gx, 1, 0); }
static bool batch_push_skinny(int kind, const SkinnyArgs& a, int gx, int gy, size_t lds) {
  return batch_push(kind, 0, &a, sizeof(a), gx, gy, lds);
}
static bool batch_push_compact_w(const CompactWArgs& a, int gx, int gy) { return batch_push(GK_COMPACT_W, 0, &a, sizeof(a), gx, gy, 0); }

// one recorded launch by itself, exactly as it would have been issued without a batch
static int32_t launch_item_alone(const BatchItem& it, hipStream_t stream) {
  const dim3 grid((unsigned)it.gx, (unsigned)it.gy), block(256);
  switch (it.kind) {
    case GK_DIRECT_KK_64:
      ARD_LAUNCH_NAMED("gemm_direct_kernel", (gemm_direct_kernel<true, true, 64, 64, 4, 0>), grid, block, it.lds, stream,
                       *reinterpret_cast<const FastParams*>(it.args));
      break;
    case GK_DIRECT_KM_64:
      ARD_LAUNCH_NAMED("gemm_direct_kernel", (gemm_direct_kernel<true, false, 64, 64, 4, 0>), grid, block, it.lds, stream,
                       *reinterpret_cast<const FastParams*>(it.args));
      break;
    case GK_DIRECT_MM_64:
      ARD_LAUNCH_NAMED("gemm_direct_kernel", (gemm_direct_kernel<false, false, 64, 64, 4, 0>), grid, block, it.lds, stream,
                       *reinterpret_cast<const FastParams*>(it.args));
      break;
    case GK_DIRECT_MM_128x64:
      ARD_LAUNCH_NAMED("gemm_direct_kernel", (gemm_direct_kernel<false, false, 128, 64, 4, 0>), grid, block, it.lds, stream,
                       *reinterpret_cast<const FastParams*>(it.args));
      break;
    case GK_SKINNY_FWD:
      ARD_LAUNCH(skinny_fwd_kernel, grid, block, it.lds, stream, *reinterpret_cast<const SkinnyArgs*>(it.args));
      break;
    case GK_SKINNY_BWD_DATA:
      ARD_LAUNCH(skinny_bwd_data_kernel, grid, block, it.lds, stream, *reinterpret_cast<const SkinnyArgs*>(it.args));
      break;
    case GK_SKINNY_BWD_WEIGHT:
      ARD_LAUNCH(skinny_bwd_weight_kernel, grid, block, it.lds, stream, *reinterpret_cast<const SkinnyArgs*>(it.args));
      break;
    case GK_COMPACT_W:
      ARD_LAUNCH(compact_weight_kernel<uint16_t>, grid, block, 0, stream, *reinterpret_cast<const CompactWArgs*>(it.args));
      break;
    case GK_FINISH_VEC:
      ARD_LAUNCH(gemm_finish_vec_kernel, grid, block, 0, stream, *reinterpret_cast<const FinishArgs*>(it.args));
      break;
    case GK_ZERO_ROWS:
      ARD_LAUNCH(zero_rows_kernel, grid, block, 0, stream, *reinterpret_cast<const ZeroRowsArgs*>(it.args));
      break;
    default:
      return fail(ARD_EINVAL, "unknown recorded kernel kind %d", it.kind);
  }
  ARD_LAUNCH_CHECK("recorded kernel");
  return ARD_OK;
}

static int32_t launch_stage(const std::vector<const BatchItem*>& items, hipStream_t stream) {
  size_t i = 0;
  while (i < items.size()) {
    // as many consecutive items as fit into one table
    GroupTable T{};
    size_t lds = 0, arg_used = 0;
    int blocks = 0;
    size_t j = i;
    for (; j < items.size() && T.nseg < kGroupMaxSeg; ++j) {
      const BatchItem& it = *items[j];
      const size_t a16 = align_up(it.arg_bytes, 16);
      if (arg_used + a16 > (size_t)kGroupArgBytes) break;
      GroupSeg& sg = T.seg[T.nseg++];
      sg.kind = it.kind, sg.first = blocks, sg.gx = it.gx, sg.gy = it.gy, sg.nblocks = it.gx * it.gy;
      sg.arg_off = (int)arg_used;
      memcpy(T.args + arg_used, it.args, it.arg_bytes);
      arg_used += a16;
      blocks += (sg.nblocks + 7) & ~7;
      lds = it.lds > lds ? it.lds : lds;
    }
    if (j - i == 1) {
      if (int32_t st = launch_item_alone(*items[i], stream)) return st;
    } else {
      static thread_local bool raised = false;
      if (!raised) {
        ARD_HIP_CHECK(raise_lds_limit((const void*)group_kernel, 4096 + 16 * (SK_MAX_COLS + 16) * 2 + 256));
        raised = !dry_run();
      }
      ARD_LAUNCH(group_kernel, dim3((unsigned)blocks), dim3(256), lds, stream, T);
      ARD_LAUNCH_CHECK("group_kernel");
    }
    i = j;
  }
  return ARD_OK;
}

}  // namespace ard

extern "C" int32_t ard_batch_begin(void) {
  if (g_batch.open) return fail(ARD_EINVAL, "ard_batch_begin: a batch is already open on this thread");
  g_batch.open = true;
  g_batch.items.clear();
  return ARD_OK;
}

extern "C" int32_t ard_batch_launch(void* stream_) {
  if (!g_batch.open) return fail(ARD_EINVAL, "ard_batch_launch without ard_batch_begin");
  g_batch.open = false;
  int32_t st = ARD_OK;
  for (int stage = 0; stage < 2 && !st; ++stage) {
    std::vector<const BatchItem*> sel;
    for (const BatchItem& it : g_batch.items)
      if (it.stage == stage) sel.push_back(&it);
    if (!sel.empty()) st = launch_stage(sel, (hipStream_t)stream_);
  }
  g_batch.items.clear();
  return st;
}

extern "C" void ard_batch_abort(void) {
  g_batch.open = false;
  g_batch.items.clear();
}

extern "C" size_t ard_gemm_workspace_bytes(int32_t dtype, int32_t B, int32_t I, int32_t O, const ard_pattern* pat_out,
                                           const ard_pattern* pat_in) {
  (void)B;
  if (I <= 0 || O <= 0) return 0;
  if (pat_out && pat_out->kind == ARD_PAT_TILE && pat_out->tile_r > 0 && pat_out->tile_c > 0)
    return tile_ws_bytes(ceil_div(O, pat_out->tile_r), ceil_div(I, pat_out->tile_c));
  // gathered kept block of W, then room for fp32 partial results of up to 8 contraction splits
  const size_t Ok = (size_t)kept_count(pat_out, O), Ik = (size_t)kept_count(pat_in, I), Bn = B > 0 ? (size_t)B : 0;
  size_t bytes = 0;
  const size_t es = dtype == ARD_BF16 ? 2 : 4;
  if (pat_in && pat_in->kind != ARD_PAT_NONE) bytes += align_up((size_t)pad8((int)Ok) * pad8((int)Ik) * es, 256);
  if (O % 8) bytes += align_up(Bn * pad8(O) * es, 256);
  if (I % 8) bytes += align_up(Bn * pad8(I) * es, 256);
  const size_t Okp = pad8((int)Ok), Ikp = pad8((int)Ik);
  size_t big = Bn * Okp;
  if (Bn * Ikp > big) big = Bn * Ikp;
  if (Okp * Ikp > big) big = Okp * Ikp;
  size_t part = big * 4 * 8;
  if (part > ((size_t)256 << 20)) part = (size_t)256 << 20;
  return bytes + part;
}

extern "C" int32_t ard_compact_weight(int32_t dtype, int32_t I, int32_t O, const void* W, void* Wc,
                                      const ard_pattern* pat_out, const ard_pattern* pat_in, void* stream) {
  LayerArgs a{dtype, 1, I, O, pat_out, pat_in, false, 0, 0};
  int32_t st = check_layer(a, W, Wc, W);
  if (st) return st;
  if (a.tile) return fail(ARD_EINVAL, "ard_compact_weight takes row or list patterns");
  return compact_weight(dtype, I, W, Wc, axis_of_pattern(pat_out, O), axis_of_pattern(pat_in, I), (hipStream_t)stream);
}

extern "C" int32_t ard_drop_gemm_fwd(int32_t dtype, int32_t B, int32_t I, int32_t O, const void* X, const void* W,
                                     void* Y, const ard_pattern* pat_out, const ard_pattern* pat_in, float alpha,
                                     int32_t fuse_relu, int32_t flags, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  LayerArgs a{dtype, B, I, O, pat_out, pat_in, false, 0, 0};
  int32_t st = check_layer(a, X, W, Y);
  if (st) return st;
  const int ce = chunk_elems(dtype);
  GemmParams P{};
  int max_bn = 0;
  size_t ws_used = 0;
  if (a.tile) {
    if (flags) return fail(ARD_EINVAL, "tile patterns take no layout flags");
    if (try_fast_tile(0, a, X, W, Y, alpha, fuse_relu != 0, stream, st)) return st;
    TileLists L;
    st = tile_lists(a, ws, ws_bytes, stream, L);
    if (st) return st;
    P.A = Operand{X, I, axis_identity(B), 0, 0};
    P.B = Operand{W, I, axis_identity(O), 0, 0};
    P.k = axis_block(L.keep, pat_out->tile_c, 0, I);
    P.kb_ptr = L.rowptr;
    P.kb_ncols = pat_out->tile_r;
    P.kb_bias = -a.TC;
    P.C.cn = axis_identity(O);
    P.C.ld = O;
    P.C.fill = 1;
    max_bn = pick_bn(pat_out->tile_r);
  } else {
    if (flags & ARD_DW_COMPACT) return fail(ARD_EINVAL, "ARD_DW_COMPACT belongs to the weight gradient");
    if (!(flags & ~kLayoutFlags) && try_skinny(0, dtype, B, I, O, X, W, Y, axis_of_pattern(pat_out, O), axis_of_pattern(pat_in, I),
                                               flags, alpha, 0.0f, fuse_relu != 0, nullptr, stream, &st))
      return st;
    RowLayer L;
    st = resolve_row_layer(a, flags, W, true, ws, ws_bytes, stream, L);
    if (st) return st;
    // contraction over the kept input neurons; an operand that is already compact ignores the map.
    // Compact matrices have pad8(count) columns, a compact W also pad8(count) rows, zero filled.
    ws_used = L.ws_used;
    P.k = L.ai;
    P.A = Operand{X, L.in_c ? pad8(L.ai.n) : I, axis_identity(B), 0, L.in_c, L.in_c, 0};
    P.B = Operand{L.Wp, L.w_ld, L.w_rows, 0, L.w_compact, L.w_compact, 0};
    if (L.out_c) {
      // the padding columns are written too (as zeros: W has no rows there)
      P.N = pad8(L.ao.n);
      P.C.cn = axis_identity(P.N);
      P.C.ld = P.N;
      P.C.fill = 0;
    } else {
      P.N = L.ao.n;
      P.C.cn = L.ao;
      P.C.ld = O;
      P.C.fill = 1;
    }
  }
  P.A.vec = operand_vec_ok(P.A, true, P.k, ce);
  P.B.vec = operand_vec_ok(P.B, true, P.k, ce);
  P.C.p = Y;
  P.C.rm = axis_identity(B);
  P.C.relu = fuse_relu != 0;
  P.C.alpha = alpha;
  P.C.beta = 0.0f;
  P.M = B;
  if (a.tile) P.N = O;
  if (P.N == 0) return (flags & ARD_OUT_COMPACT) ? ARD_OK : fill_matrix(dtype, Y, (long)B * O, 0.0f, stream);
  return run_gemm(dtype, true, true, P, max_bn, 0, stream, a.tile ? nullptr : (char*)ws + ws_used,
                  a.tile || ws_bytes < ws_used ? 0 : ws_bytes - ws_used);
}

extern "C" int32_t ard_drop_gemm_bwd_data(int32_t dtype, int32_t B, int32_t I, int32_t O, const void* dY, const void* W,
                                          void* dX, const ard_pattern* pat_out, const ard_pattern* pat_in, float alpha,
                                          const void* relu_src, int32_t flags, void* ws, size_t ws_bytes,
                                          void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  LayerArgs a{dtype, B, I, O, pat_out, pat_in, false, 0, 0};
  int32_t st = check_layer(a, dY, W, dX);
  if (st) return st;
  const int ce = chunk_elems(dtype);
  GemmParams P{};
  int max_bn = 0;
  size_t ws_used = 0;
  if (a.tile) {
    if (flags) return fail(ARD_EINVAL, "tile patterns take no layout flags");
    if ((!relu_src || ((uintptr_t)relu_src & 3) == 0) && try_fast_tile(1, a, dY, W, dX, alpha, 0, stream, st, relu_src)) return st;
    TileLists L;
    st = tile_lists(a, ws, ws_bytes, stream, L);
    if (st) return st;
    P.A = Operand{dY, O, axis_identity(B), 0, 0};
    P.B = Operand{W, I, axis_identity(I), 0, 0};  // element (n = input neuron, k = output neuron) at W[k*I + n]
    P.k = axis_block(L.csc_rows, pat_out->tile_r, 0, O);
    P.kb_ptr = L.colptr;
    P.kb_ncols = pat_out->tile_c;
    P.kb_bias = 0;
    P.C.cn = axis_identity(I);
    P.C.ld = I;
    P.C.fill = 1;
    max_bn = pick_bn(pat_out->tile_c);
  } else {
    if (flags & ARD_DW_COMPACT) return fail(ARD_EINVAL, "ARD_DW_COMPACT belongs to the weight gradient");
    if (!(flags & ~kLayoutFlags) && try_skinny(1, dtype, B, I, O, dY, W, dX, axis_of_pattern(pat_out, O), axis_of_pattern(pat_in, I),
                                               flags, alpha, 0.0f, 0, relu_src, stream, &st))
      return st;
    RowLayer L;
    st = resolve_row_layer(a, flags, W, true, ws, ws_bytes, stream, L);
    if (st) return st;
    // contraction over the kept output neurons
    ws_used = L.ws_used;
    P.k = L.ao;
    P.A = Operand{dY, L.out_c ? pad8(L.ao.n) : O, axis_identity(B), 0, L.out_c, L.out_c, 0};
    P.B = Operand{L.Wp, L.w_ld, L.w_cols, 0, L.w_compact, L.w_compact, L.w_compact};
    if (!L.out_c && L.w_compact && is_identity(L.ao)) {
      // narrow dY (last layer): a zero-padded copy lets the contraction run over whole chunks
      const void* dYp;
      int dy_ld;
      st = aligned_activation(dtype, dY, B, O, ws, ws_bytes, ws_used, stream, dYp, dy_ld);
      if (st) return st;
      if (dYp != dY) P.A = Operand{dYp, dy_ld, axis_identity(B), 0, 0, 1, 0};
    }
    if (L.in_c) {
      P.N = pad8(L.ai.n);
      P.C.cn = axis_identity(P.N);
      P.C.ld = P.N;
      P.C.fill = 0;
    } else {
      P.N = L.ai.n;
      P.C.cn = L.ai;
      P.C.ld = I;
      P.C.fill = 1;
    }
  }
  P.A.vec = operand_vec_ok(P.A, true, P.k, ce);
  P.B.vec = operand_vec_ok(P.B, false, P.k, ce);
  P.C.p = dX;
  P.C.relu_src = relu_src;
  P.C.rm = axis_identity(B);
  P.C.alpha = alpha;
  P.M = B;
  if (a.tile) P.N = I;
  if (P.N == 0) return (flags & ARD_IN_COMPACT) ? ARD_OK : fill_matrix(dtype, dX, (long)B * I, 0.0f, stream);
  return run_gemm(dtype, true, false, P, max_bn, 0, stream, a.tile ? nullptr : (char*)ws + ws_used,
                  a.tile || ws_bytes < ws_used ? 0 : ws_bytes - ws_used);
}

extern "C" int32_t ard_drop_gemm_bwd_weight(int32_t dtype, int32_t B, int32_t I, int32_t O, const void* dY,
                                            const void* X, void* dW, const ard_pattern* pat_out,
                                            const ard_pattern* pat_in, float alpha, float beta, int32_t flags,
                                            void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  LayerArgs a{dtype, B, I, O, pat_out, pat_in, false, 0, 0};
  int32_t st = check_layer(a, dY, X, dW);
  if (st) return st;
  const int ce = chunk_elems(dtype);
  GemmParams P{};
  P.k = axis_identity(B);
  size_t ws_used = 0;
  bool dw_compact = false;
  if (a.tile) {
    if (flags) return fail(ARD_EINVAL, "tile patterns take no layout flags");
    if (beta == 0.0f && try_fast_tile(2, a, dY, X, dW, alpha, 0, stream, st)) return st;
    TileLists L;
    st = tile_lists(a, ws, ws_bytes, stream, L);
    if (st) return st;
    P.A = Operand{dY, O, axis_identity(O), 0, 0};  // element (m = output neuron, k = batch row) at dY[k*O + m]
    P.B = Operand{X, I, axis_identity(I), 0, 0};   // element (n = input neuron, k = batch row) at X[k*I + n]
    P.C.rm = axis_identity(O);
    P.C.cn = axis_identity(I);
    P.tmask = L.mask;
    P.tm_r = pat_out->tile_r;
    P.tm_c = pat_out->tile_c;
    P.tm_tc = a.TC;
  } else {
    if (flags & ARD_W_COMPACT) return fail(ARD_EINVAL, "ARD_W_COMPACT has no meaning for the weight gradient");
    RowLayer L;
    st = resolve_row_layer(a, flags, nullptr, false, ws, ws_bytes, stream, L);
    if (st) return st;
    P.A = Operand{dY, L.out_c ? pad8(L.ao.n) : O, L.out_c ? axis_identity(L.ao.n) : L.ao, 0, 0, 0, L.out_c};
    P.B = Operand{X, L.in_c ? pad8(L.ai.n) : I, L.in_c ? axis_identity(L.ai.n) : L.ai, 0, 0, 0, L.in_c};
    if (!L.out_c && is_identity(L.ao)) {
      const void* q;
      int q_ld;
      st = aligned_activation(dtype, dY, B, O, ws, ws_bytes, ws_used, stream, q, q_ld);
      if (st) return st;
      if (q != dY) P.A = Operand{q, q_ld, L.ao, 0, 0, 0, 1};
    }
    if (!L.in_c && is_identity(L.ai)) {
      const void* q;
      int q_ld;
      st = aligned_activation(dtype, X, B, I, ws, ws_bytes, ws_used, stream, q, q_ld);
      if (st) return st;
      if (q != X) P.B = Operand{q, q_ld, L.ai, 0, 0, 0, 1};
    }
    P.C.rm = L.ao;
    P.C.cn = L.ai;
    if (flags & ARD_DW_COMPACT) {
      // dW of the kept synapses only, [pad8(O') x pad8(I')] like a compact weight: both activations
      // come compact, so the padding rows and columns are products of zeros
      if (!L.out_c || !L.in_c) return fail(ARD_EINVAL, "ARD_DW_COMPACT needs ARD_IN_COMPACT and ARD_OUT_COMPACT");
      const int Mp = pad8(L.ao.n), Np = pad8(L.ai.n);
      P.A.r = axis_identity(Mp);
      P.B.r = axis_identity(Np);
      P.C.rm = axis_identity(Mp);
      P.C.cn = axis_identity(Np);
      dw_compact = true;
    }
  }
  if (!a.tile && try_skinny(2, dtype, B, I, O, dY, X, dW, axis_of_pattern(pat_out, O), axis_of_pattern(pat_in, I), flags, alpha,
                            beta, 0, nullptr, stream, &st))
    return st;
  P.A.vec = operand_vec_ok(P.A, false, P.k, ce);
  P.B.vec = operand_vec_ok(P.B, false, P.k, ce);
  P.C.p = dW;
  P.C.ld = dw_compact ? P.C.cn.n : I;
  P.C.fill = dw_compact ? 0 : 1;
  P.C.alpha = alpha;
  P.C.beta = beta;
  P.M = P.A.r.n;
  P.N = P.B.r.n;
  if (P.M == 0 || P.N == 0) return dw_compact ? ARD_OK : fill_matrix(dtype, dW, (long)O * I, beta, stream);
  return run_gemm(dtype, false, false, P, 0, 0, stream, a.tile ? nullptr : (char*)ws + ws_used,
                  a.tile || ws_bytes < ws_used ? 0 : ws_bytes - ws_used);
}

// ---- weight gradient for callers that cannot allocate ------------------------------------------
//
// The library's own scratch: one array per GPU, part of the loaded code object, alive until the
// process ends.  Host code never uses the array's name as an address: the device address is looked
// up once per device (with that device current) and kept.
namespace ard {
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static int32_t static_scratch(void** out) {
  constexpr int kMaxDev = 64;
  static void* ptr_of_device[kMaxDev] = {};
  static std::mutex mu;
  if (dry_run()) {
    *out = (void*)(uintptr_t)0x7E0000000000ULL;  // never dereferenced
    return ARD_OK;
  }
  int dev = -1;
  ARD_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDev) return fail(ARD_EHIP, "device ordinal %d outside 0..%d", dev, kMaxDev - 1);
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    ARD_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255)) return fail(ARD_EHIP, "scratch symbol resolved to %p", p);
    ptr_of_device[dev] = p;
  }
  *out = ptr_of_device[dev];
  return ARD_OK;
}
}  // namespace ard

extern "C" size_t ard_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int32_t ard_drop_gemm_bwd_weight_static(int32_t dtype, int32_t B, int32_t I, int32_t O, const void* dY,
                                                   const void* X, void* dW, const ard_pattern* pat_out,
                                                   const ard_pattern* pat_in, float alpha, float beta, int32_t flags,
                                                   void* stream) {
  // same argument checks as the workspace variant, before the size test (clear errors first)
  LayerArgs a{dtype, B, I, O, pat_out, pat_in, false, 0, 0};
  int32_t st = check_layer(a, dY, X, dW);
  if (st) return st;
  const size_t need = ard_gemm_workspace_bytes(dtype, B, I, O, pat_out, pat_in);
  if (need > kStaticScratchBytes)
    return fail(ARD_EWORKSPACE,
                "ard_drop_gemm_bwd_weight_static: this layer asks for %zu bytes of scratch (ard_gemm_workspace_bytes), the "
                "library's static scratch holds %zu; use ard_drop_gemm_bwd_weight with a workspace",
                need, kStaticScratchBytes);
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st) return st;
  return ard_drop_gemm_bwd_weight(dtype, B, I, O, dY, X, dW, pat_out, pat_in, alpha, beta, flags, ws, kStaticScratchBytes,
                                  stream);
}

namespace ard {
template <typename T>
__global__ void relu_bwd_kernel(const T* dY, const T* Y, T* dX, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dX[i] = ElemTraits<T>::to_f32(Y[i]) > 0.0f ? dY[i] : ElemTraits<T>::from_f32(0.0f);
}
}  // namespace ard

extern "C" int32_t ard_relu_bwd(int32_t dtype, int64_t n, const void* dY, const void* Y, void* dX, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (n < 0) return fail(ARD_ESHAPE, "negative length");
  if (n == 0) return ARD_OK;
  if (!dY || !Y || !dX) return fail(ARD_EINVAL, "null tensor pointer");
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == ARD_BF16)
    ARD_LAUNCH(relu_bwd_kernel<uint16_t>, grid, block, 0, stream, (const uint16_t*)dY, (const uint16_t*)Y,
                       (uint16_t*)dX, (long)n);
  else if (dtype == ARD_F32)
    ARD_LAUNCH(relu_bwd_kernel<float>, grid, block, 0, stream, (const float*)dY, (const float*)Y, (float*)dX,
                       (long)n);
  else
    return fail(ARD_EDTYPE, "unknown dtype %d", dtype);
  ARD_LAUNCH_CHECK("relu_bwd_kernel");
  return ARD_OK;
}
