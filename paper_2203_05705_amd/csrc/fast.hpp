// LDS-direct bf16 path of the gathered GEMM for gfx950.
//
// Workgroup tiles BM x BN x 64 of 32x32x16 bf16 MFMA tiles: 256x256, 256x128, 128x256 with 8
// wavefronts (two per SIMD), 128x128, 128x64 and 64x64 with 4 wavefronts for products too small
// to fill 256 CUs with large tiles; optional split of the contraction over blockIdx.y with
// fp32 partial sums that a finishing kernel reduces (fixed split: deterministic).
//
// Operand staging uses LDS-direct loads (global_load_lds_dwordx4): a wavefront instruction
// moves 64 x 16 bytes from per-lane global addresses into 1 KiB of consecutive LDS with no
// register in between, so a whole stage stays in flight behind the MFMAs of the previous one.
// The LDS layout is therefore fixed by lane order, and each lane picks WHICH chunk it fetches
// so that the layout comes out swizzled (bank-conflict free for the fragment reads):
//   KC operand (contraction-contiguous in memory): LDS tile [rows][8 chunks of 16 B]; an
//     instruction fills 8 rows; lane = (row, slot) fetches logical chunk slot ^ xr(row).
//     Fragments: ds_read_b128.
//   MC operand (contraction-strided in memory): LDS tile [64 k][rows] exactly as in memory; lane
//     = (k, pos) fetches chunk pos ^ 4*(k & 3).  Fragments: two ds_read_b64_tr_b16 (the
//     transposing LDS read of gfx950) per MFMA operand, no register transpose anywhere.
// LDS: [A stages | B stages] (2 stages, 3 for the 64x64 tile); the stage is an immediate offset
// of the fragment reads, so every read address is a loop invariant.
//
// Tile patterns (Section 3.2) are period patterns over the linear tile index, so the tile
// rows (or columns) fall into a few CLASSES that share one kept-column (kept-row) set:
// class members, and the kept set of a class, are both arithmetic progressions.  A
// workgroup takes consecutive members of ONE class as its rows or columns and walks that
// class's kept set along the contraction, so dropped tiles cost nothing and the macro
// tile stays wide.  ClassTab carries the progressions.
//
// The same kernel runs the convolutions on a channels-last grid of the kept feature maps
// (MODE 1: rows of B are output pixels, contraction = (tap, channel); MODE 2: weight gradient,
// contraction over the grid's pixels).
//
// Restrictions checked on the host (anything else goes through gemm_kernel): bf16, 16-byte
// aligned operands, every extent along a 16-byte run a multiple of 8 (or zero-padded storage),
// contraction map = identity or a block progression with block size a multiple of 64.
#pragma once
#include <type_traits>

#include "engine.hpp"

namespace ard {

constexpr int F_MAXCLS = 16;

struct ClassTab {
  int ncls;                       // 0: plain tiles_m x tiles_n grid over P.am / P.bn / P.k
  int nblk[F_MAXCLS];             // workgroups of class c
  int mblk[F_MAXCLS];             // workgroup rows of class c
  // row side (M): block progression off + i*step, `cnt` blocks of size bs (bs == 0: identity rows)
  int m_off[F_MAXCLS], m_cnt[F_MAXCLS], m_step, m_bs, m_phys;
  // column side (N)
  int n_off[F_MAXCLS], n_cnt[F_MAXCLS], n_step, n_bs, n_phys;
  // contraction side (K) (bs == 0: identity contraction P.k)
  int k_off[F_MAXCLS], k_cnt[F_MAXCLS], k_step, k_bs, k_phys;
};

// Implicit-GEMM convolution on a channels-last, zero-bordered copy of the activations
// T[(n*Hg + h)*Wg + w][Cp] (Cp channels per pixel, a multiple of 64): the patch of output pixel
// (n, ho, wo) and tap (r, s) is the Cp-run that starts at pixel (n*Hg + ho + r)*Wg + wo + s, so
// along the contraction k = (tap, c) every row of the im2col matrix is its base pixel plus an
// offset that depends on k only.
struct ConvMap {
  int HoWo, Wo;     // output pixels per image / per row
  int HgWg, Wg;     // pixels per image / per row of the bordered grid
  int Cp, kw;       // channels per pixel of the grid, taps per filter row
  int npix;         // output pixels over the batch (rows of the im2col matrix)
  int out_chan;     // channels per image of the output tensor (NCHW)
  const int* chan;  // optional: output channel of compact row i (kept-channel list), else i
  int n_rows;       // valid compact output rows (channels)
  // optional list of kept output pixels (row-based sensitivity-aware pattern, Section 5.2.1): compact
  // column j of the product is pixel pix[j] of the pix_total pixels; npix then counts the kept ones.
  // pix_fixed >= 0 (host-side bounds proof only): every column reads that pixel instead of the list.
  const int* pix;
  int pix_total, pix_fixed;
  int pix_pairs;  // list entries 2i, 2i+1 are pixels 2m, 2m+1 of one image (or both padding): stored as one word
};

struct FastParams {
  const uint16_t* A;
  const uint16_t* B;
  uint16_t* C;
  int lda, ldb, ldc;
  long a_elems, b_elems;  // elements the caller owns behind A / B: what the loaders may touch (host-side proof)
  Axis am, bn, k;  // plain mode: compact -> physical rows of A (M), rows of B (N), contraction
  ClassTab tab;
  int c_rows_mapped, c_cols_mapped;  // output rows / columns go through the M / N map (else identity)
  float alpha, beta;
  int relu, out_f32;
  const uint16_t* relu_src;  // optional, same layout as C
  float* part;               // != NULL: write fp32 partial sums part[split][M][N] instead of C
  int splits;
  int M, N, tiles_m, tiles_n, group_m, total_tiles;
  ConvMap cv;  // MODE 1 / 2 of the kernel only
  // MODE 1, optional (block-based sensitivity-aware pattern, Section 5.2.2): the column tile t of the
  // product contracts over the kb_cnt[t] 64-wide blocks kb_list[t * kb_stride ...] of the contraction only
  // (at most 128 of them); entries of cv.pix may then be -1 (padding of a tile: nothing is stored).
  const int* kb_list;
  const int* kb_cnt;
  int kb_stride;
  // Scattering epilogue (row patterns without compact outputs): the tile's results go through
  // LDS and are written, with the dropped positions it owns as +0.0, through these affine maps.
  int scatter, scatter_vec;
  int scatter_rows_only;  // the tile writes its kept rows only (a separate pass zeroes the dropped rows)
  Axis srm, scn;
};

// Two fp32 values to packed bf16 (low half = first) with the conversion instruction of gfx950
// (round to nearest even, the same rounding as f32_to_bf16_bits for finite values).
typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_hw_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw_t));
}

#define ARD_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))
#define ARD_GLB_PTR(p) ((const void __attribute__((address_space(1)))*)(p))

// 64 zero bytes: source of the chunks that lie beyond the end of the contraction
static __device__ uint4 g_zero_chunk[4];

// physical start of the 64-wide contraction slab that begins at compact index ks (uniform)
__host__ __device__ __forceinline__ int fast_kslab(const Axis& k, int ks) {
  if (k.kind == AX_AFFINE) return k.off + ks;
  const int q = ks / k.bs;
  if (k.kind == AX_BAFF) return (k.off + q * k.step) * k.bs + (ks - q * k.bs);
  return (k.list[q] + k.off) * k.bs + (ks - q * k.bs);
}

// A contraction axis made of 32-wide blocks in arithmetic progression (the paper's 32 x 32 tiles): a
// 64-deep step holds two kept blocks, `step` blocks apart in memory.  The slab of a step starts at its
// first block; the lanes that fetch the step's upper half add this constant (in contraction elements) to
// their offset once, at set-up, so the loop itself does not change.
__host__ __device__ __forceinline__ int direct_kbump(const Axis& k) {
  return (k.kind == AX_BAFF && k.bs == 32) ? (k.step - 1) * 32 : 0;
}

template <bool KC, int ROWS, int NW> struct DirectLoader;

// Both loaders keep, per lane and instruction, a loop-invariant 32-bit BYTE offset from a base that
// is uniform over the workgroup; a contraction step only moves the uniform base, so a load costs
// no vector ALU work.  A lane whose tile row lies beyond the operand reads some valid row instead
// (clamped at set-up): such rows only feed outputs that are never stored, or that the epilogue
// overwrites with zeros.  Only the last, partial step of a contraction redirects lanes to a zero chunk.
template <int ROWS, int NW> struct DirectLoader<true, ROWS, NW> {
  static constexpr int NI = ROWS / 8 / NW;  // instructions per wavefront and stage (8 rows each)
  static_assert(NI >= 1, "tile too small for the workgroup");
  const char* base;
  uint32_t voff[NI];
  __host__ __device__ static __forceinline__ int chunk_k(int lane, int wave, int j) {
    const int row = (wave * NI + j) * 8 + (lane >> 3);
    return ((lane & 7) ^ (row & 7) ^ ((row >> 3) & 7)) * 8;
  }
  // (host-callable: the host-side bounds proof runs this very arithmetic for every lane)
  __host__ __device__ __forceinline__ void init(const uint16_t* p, int ld, const Axis& r, int row0, int lane, int wave,
                                                int kbump = 0) {
    base = reinterpret_cast<const char*>(p);
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int row = imin(row0 + (wave * NI + j) * 8 + (lane >> 3), r.n - 1);
      // (a block axis counts its last block in full even when the operand ends inside it)
      int prow = ax_phys(r, row);
      if (r.kind == AX_BLOCK || r.kind == AX_BAFF) prow = imin(prow, r.nphys - 1);
      const int ck = chunk_k(lane, wave, j);
      voff[j] = (uint32_t)(prow * ld + ck + (ck >= 32 ? kbump : 0)) * 2u;
    }
  }
  // rows = output pixels of a convolution: base pixel of the patch in the bordered grid
  __host__ __device__ __forceinline__ void init_pixels(const uint16_t* p, const ConvMap& cv, int row0, int lane, int wave) {
    base = reinterpret_cast<const char*>(p);
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      int row = imin(row0 + (wave * NI + j) * 8 + (lane >> 3), cv.npix - 1);
      if (cv.pix_fixed >= 0) row = cv.pix_fixed;
      else if (cv.pix) row = imax(cv.pix[row], 0);  // (-1: padding entry, reads pixel 0, stores nothing)
      const int n = row / cv.HoWo, rem = row - n * cv.HoWo;
      const int ho = rem / cv.Wo, wo = rem - ho * cv.Wo;
      voff[j] = (uint32_t)((n * cv.HgWg + ho * cv.Wg + wo) * cv.Cp + chunk_k(lane, wave, j)) * 2u;
    }
  }
  // full step: nothing but the loads
  __device__ __forceinline__ void issue(uint4* op_tile, int kslab, int wave) const {
    const char* sb = base + (long)kslab * 2;  // uniform
#pragma unroll
    for (int j = 0; j < NI; ++j)
      __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(sb + voff[j]), ARD_LDS_PTR(op_tile + (wave * NI + j) * 64), 16, 0, 0);
  }
  // one of the NI loads of a full step (for callers that spread them between other instructions)
  __device__ __forceinline__ void issue_one(uint4* op_tile, int kslab, int wave, int j) const {
    const char* sb = base + (long)kslab * 2;
    __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(sb + voff[j]), ARD_LDS_PTR(op_tile + (wave * NI + j) * 64), 16, 0, 0);
  }
  // last, partial step of a contraction: chunks beyond its end come from the zero chunk
  __host__ __device__ static __forceinline__ bool tail_live(int lane, int wave, int j, int kslab, int krem, int kphys_end,
                                                            int kbump = 0) {
    const int k = chunk_k(lane, wave, j);
    return k < krem && kslab + k + (k >= 32 ? kbump : 0) + 8 <= kphys_end;
  }
  // byte offset from the operand's base of instruction j's chunk in the step whose slab starts at kslab
  __host__ __device__ __forceinline__ long byte_offset(int j, int kslab) const { return (long)kslab * 2 + voff[j]; }
  __device__ __forceinline__ void issue_tail(uint4* op_tile, int kslab, int krem, int kphys_end, int lane, int wave,
                                             int kbump = 0) const {
    asm volatile("; partial contraction step" ::: "memory");  // keeps this path out of the full step's code
    const char* sb = base + (long)kslab * 2;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const char* src = sb + voff[j];
      if (!tail_live(lane, wave, j, kslab, krem, kphys_end, kbump)) src = reinterpret_cast<const char*>(g_zero_chunk);
      __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(src), ARD_LDS_PTR(op_tile + (wave * NI + j) * 64), 16, 0, 0);
    }
  }
};

// swizzle of an MC tile: chunk c of contraction row k sits at position c ^ mc_swz(k).  Rows are
// ROWS*2 bytes apart; the XOR makes the four rows a transposing read touches land in different
// banks (rows of 256+ bytes all start at the same bank, rows of 128 bytes alternate).
template <int ROWS>
__host__ __device__ __forceinline__ int mc_swz(int k) {
  return ROWS >= 128 ? 4 * (k & 3) : 4 * ((k >> 1) & 1);
}

template <int ROWS, int NW> struct DirectLoader<false, ROWS, NW> {
  static constexpr int CPR = ROWS / 8;         // 16-byte chunks per contraction row
  static constexpr int KPI = 64 / CPR;         // contraction rows per instruction
  static constexpr int NI = 64 / KPI / NW;     // instructions per wavefront and stage
  static_assert(NI >= 1, "tile too small for the workgroup");
  const char* base;
  int ld;
  uint32_t voff[NI];  // (contraction row within the step) * ld + column of this lane's chunk, in bytes
  __host__ __device__ __forceinline__ int lane_chunk(int lane, int wave, int j) const {
    const int kloc = KPI * (wave * NI + j) + lane / CPR;
    return (lane % CPR) ^ mc_swz<ROWS>(kloc);
  }
  __host__ __device__ __forceinline__ void init(const uint16_t* p, int ld_, const Axis& r, int row0, int lane, int wave,
                                                int kbump = 0) {
    base = reinterpret_cast<const char*>(p);
    ld = ld_;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int kl = KPI * (wave * NI + j) + lane / CPR;
      const int kloc = kl + (kl >= 32 ? kbump : 0);
      const int col = imin(row0 + lane_chunk(lane, wave, j) * 8, r.n - 8);  // runs beyond the axis: clamped
      // (a block axis counts its last block in full even when the operand ends inside it)
      int pcol = ax_phys(r, col);
      if (r.kind == AX_BLOCK || r.kind == AX_BAFF) pcol = imax(imin(pcol, (r.nphys - 8) & ~7), 0);
      voff[j] = (uint32_t)(kloc * ld + pcol) * 2u;
    }
  }
  // columns = (tap, channel) of the weight gradient: pixel offset of the tap plus the channel
  __host__ __device__ __forceinline__ void init_tap_columns(const uint16_t* p, const ConvMap& cv, int ncols, int row0,
                                                            int lane, int wave) {
    base = reinterpret_cast<const char*>(p);
    ld = cv.Cp;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int kloc = KPI * (wave * NI + j) + lane / CPR;
      const int col = imin(row0 + lane_chunk(lane, wave, j) * 8, ncols - 8);
      const int t = col / cv.Cp;
      voff[j] = (uint32_t)(kloc * ld + ((t / cv.kw) * cv.Wg + t % cv.kw) * cv.Cp + (col - t * cv.Cp)) * 2u;
    }
  }
  __device__ __forceinline__ void issue(uint4* op_tile, int kslab, int wave) const {
    const char* sb = base + (long)kslab * ld * 2;  // uniform
#pragma unroll
    for (int j = 0; j < NI; ++j)
      __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(sb + voff[j]), ARD_LDS_PTR(op_tile + (wave * NI + j) * 64), 16, 0, 0);
  }
  __device__ __forceinline__ void issue_one(uint4* op_tile, int kslab, int wave, int j) const {
    const char* sb = base + (long)kslab * ld * 2;
    __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(sb + voff[j]), ARD_LDS_PTR(op_tile + (wave * NI + j) * 64), 16, 0, 0);
  }
  __host__ __device__ static __forceinline__ bool tail_live(int lane, int wave, int j, int kslab, int krem, int kphys_end,
                                                            int kbump = 0) {
    const int kloc = KPI * (wave * NI + j) + lane / CPR;
    return kloc < krem && kslab + kloc + (kloc >= 32 ? kbump : 0) < kphys_end;
  }
  __host__ __device__ __forceinline__ long byte_offset(int j, int kslab) const { return (long)kslab * ld * 2 + voff[j]; }
  __device__ __forceinline__ void issue_tail(uint4* op_tile, int kslab, int krem, int kphys_end, int lane, int wave,
                                             int kbump = 0) const {
    asm volatile("; partial contraction step" ::: "memory");
    const char* sb = base + (long)kslab * ld * 2;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const char* src = sb + voff[j];
      if (!tail_live(lane, wave, j, kslab, krem, kphys_end, kbump)) src = reinterpret_cast<const char*>(g_zero_chunk);
      __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(src), ARD_LDS_PTR(op_tile + (wave * NI + j) * 64), 16, 0, 0);
    }
  }
};

// Byte offset, inside an MC operand tile of `ROWS` rows, of this lane's source position for the
// transposing reads of the 32-wide MFMA tile that starts at tile row `tile_col0`.  The reads
// of slice q, half h add the immediate (q*16 + h*4) * ROWS*2.
// ds_read_b64_tr_b16 works on groups of 16 lanes: result lane i, element e comes from source
// lane 4e + i/4, element i%4.  With source lane s at (k = s/4, column 4*(s%4)) of a 4 x 16
// block, result lane i holds column i for k = 0..3: the MFMA operand order.
template <int ROWS>
__device__ __forceinline__ int mc_frag_base(int tile_col0, int lane) {
  const int s = lane & 15, G = lane >> 4;
  const int g = G >> 1, jhalf = G & 1;
  const int c = (tile_col0 >> 3) + 2 * jhalf + ((s & 3) >> 1);
  const int pc = c ^ mc_swz<ROWS>(s >> 2);
  return (g * 8 + (s >> 2)) * (ROWS * 2) + pc * 16 + 8 * (s & 1);
}

// LDS fragment reads are issued as volatile asm with ONE explicit wait per 16-wide slice: the
// compiler cannot sink a read next to its consumer, so a slice's reads are in flight while
// the previous slice's MFMAs run (left to itself the scheduler waits right after each read).
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
struct Frag {  // one MFMA operand: a full 16-byte read (KC) or two transposing 8-byte reads (MC)
  u32x4_t v;
  u32x2_t lo, hi;
};
template <int OFF>
__device__ __forceinline__ void lds_read_b128(u32x4_t& dst, unsigned byte_addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(byte_addr), "n"(OFF));
}
template <int OFF>
__device__ __forceinline__ void lds_read_tr16_b64(u32x2_t& dst, unsigned byte_addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(byte_addr), "n"(OFF));
}
template <bool KC>
__device__ __forceinline__ void frag_wait(Frag& f) {
  // tie the destination registers to the wait so no consumer can be scheduled before it
  if (KC) asm volatile("" : "+v"(f.v));
  else asm volatile("" : "+v"(f.lo), "+v"(f.hi));
}
template <bool KC>
__device__ __forceinline__ bf16x8_t frag_value(const Frag& f) {
  if (KC) return __builtin_bit_cast(bf16x8_t, f.v);
  u32x4_t t = {f.lo[0], f.lo[1], f.hi[0], f.hi[1]};
  return __builtin_bit_cast(bf16x8_t, t);
}

// LDS stages of a tile configuration: the loads of NST - 1 contraction steps are in flight
// while one step is multiplied.  A 4-wavefront workgroup wants a second workgroup on its CU
// (8 wavefronts hide the LDS and MFMA latencies), so its stages must fit twice into the 160 KiB
// LDS; only the smallest tile has room for a third stage.
#ifndef ARD_NST_SMALL
#define ARD_NST_SMALL 3
#endif
constexpr int direct_stages(int bm, int bn) { return bm + bn <= 128 ? ARD_NST_SMALL : 2; }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Plain barrier.  The LDS stages are filled by LDS-direct loads (each wave waits for its own
// with wait_vmcnt before the barrier) and read by volatile asm, so no fence is wanted: a fence
// would also wait for the younger stages still in flight.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Scattering store of one workgroup tile.  `tile` holds the final bf16 values of compact rows
// [m0, m1) x columns [n0, n1) ([.][ldt] in LDS).  Output maps are affine with off < step: compact
// index i owns the physical group [i*step, (i+1)*step) that contains its kept position, the last
// index also the tail up to nphys; everything in the owned region that is not a kept position is
// written as +0.0.  VEC: 16-byte pieces (host checks extents, leading dimension and alignment).
template <bool VEC>
__device__ __forceinline__ void direct_scatter_tile(const uint16_t* tile, int ldt, const FastParams& P, int m0, int m1,
                                                    int n0, int n1, int tid, int nthreads) {
  const Axis& rm = P.srm;
  const Axis& cn = P.scn;
  const int sr = rm.step, sc = cn.step;
  const int c_lo = n0 * sc, c_hi = n1 == P.N ? cn.nphys : n1 * sc;
  constexpr int W = VEC ? 8 : 1;
  const int CW = (c_hi - c_lo + W - 1) / W;
  // threads = (row slot, piece slot): a power-of-two number of lanes walks the pieces of a row
  int sh = 0;
  while ((1 << sh) < CW && sh < 6) ++sh;
  const int LPR = 1 << sh, RPP = nthreads >> sh;
  const int rsub = tid >> sh, cl = tid & (LPR - 1);
  auto write_row = [&](int r, int li) {
    uint16_t* rowp = P.C + (long)r * P.ldc;
    if (li < 0) {
      for (int cq = cl; cq < CW; cq += LPR) {
        if (VEC) *reinterpret_cast<uint4*>(rowp + c_lo + cq * W) = make_uint4(0, 0, 0, 0);
        else rowp[c_lo + cq] = 0;
      }
      return;
    }
    const uint16_t* trow = tile + li * ldt - n0;
    for (int cq = cl; cq < CW; cq += LPR) {
      const int c0 = c_lo + cq * W;
      int j = 0;
      const int d = c0 - cn.off + sc - 1;
      if (d >= sc) {
        j = (int)((float)d / (float)sc);
        j += ((j + 1) * sc <= d) - (j * sc > d);
      }
      uint4 gate = make_uint4(0, 0, 0, 0);
      if (P.relu_src) {
        const uint16_t* g = P.relu_src + (long)r * P.ldc + c0;
        if (VEC) gate = *reinterpret_cast<const uint4*>(g);
        else gate.x = *g;
      }
      const uint32_t* gw = reinterpret_cast<const uint32_t*>(&gate);
      uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int t = 0; t < W; ++t) {
        if (!(j < n1 && cn.off + j * sc == c0 + t)) continue;
        uint32_t v = trow[j];
        ++j;
        if (P.relu_src) {
          const uint32_t g = (gw[t >> 1] >> (16 * (t & 1))) & 0xffffu;
          if (!(bf16_bits_to_f32((uint16_t)g) > 0.0f)) v = 0;
        }
        w[t >> 1] |= v << (16 * (t & 1));
      }
      if (VEC) *reinterpret_cast<uint4*>(rowp + c0) = make_uint4(w[0], w[1], w[2], w[3]);
      else rowp[c0] = (uint16_t)w[0];
    }
  };
  if (P.scatter_rows_only) {
    // kept rows only, whole rows (kept columns and the zeros between them)
    for (int i = m0 + rsub; i < m1; i += RPP) write_row(i * sr + rm.off, i - m0);
    return;
  }
  // the groups of this tile's compact rows: one kept row and step - 1 dropped ones each
  for (int i = m0 + rsub; i < m1; i += RPP)
    for (int g = 0; g < sr; ++g) {
      const int r = i * sr + g;
      if (r >= rm.nphys) break;
      write_row(r, g == rm.off ? i - m0 : -1);
    }
  // the last tile also owns the rows behind the last group
  if (m1 == P.M)
    for (int r = P.M * sr + rsub; r < rm.nphys; r += RPP) write_row(r, -1);
}

// What one workgroup computes: its row / column / contraction maps (class-based launches build them
// from the class tables), the first compact row and column of its tile and its share of the
// contraction.  Shared by the kernel and by the host-side bounds proof.
struct DirectWork {
  Axis am, bn, kax;
  int m0, n0, split;
};
template <int F_BM, int BN>
__host__ __device__ __forceinline__ bool direct_assign(const FastParams& P, int block_id, DirectWork& w) {
  // Workgroup ids go round-robin over the 8 XCDs.  XCD x = id % 8 takes, of every class, the
  // contiguous share [x*n/8, (x+1)*n/8) of its n workgroups: the shares are compact rectangles
  // (operand panels stay in that XCD's L2) and heavy and light classes are spread evenly.
  const int xcd = block_id & 7;
  int local = block_id >> 3;
  Axis am = P.am, bn = P.bn, kax = P.k;
  int m0 = 0, n0 = 0;
  int split = 0;  // share of the contraction this workgroup takes
  if (P.tab.ncls == 0) {
    // work items = (split, tile), split-major: an XCD's contiguous share holds whole splits (or long
    // runs of one), so the workgroups in flight on it read the same slab of the contraction
    const int total = P.total_tiles * P.splits;
    const int lo = (int)((long)xcd * total / 8), hi = (int)((long)(xcd + 1) * total / 8);
    if (local >= hi - lo) return false;
    int L = lo + local;
    split = L / P.total_tiles;
    L -= split * P.total_tiles;
    // bands of group_m tile rows, walked column by column
    const int band_sz = P.group_m * P.tiles_n;
    const int band = L / band_sz, inb = L - band * band_sz;
    const int rows_in_band = imin(P.group_m, P.tiles_m - band * P.group_m);
    m0 = (band * P.group_m + inb % rows_in_band) * F_BM;
    n0 = (inb / rows_in_band) * BN;
    // per-tile contraction lists: the length comes from the tile's count, the blocks are looked up step
    // by step (the host-side proof clears kb_cnt and walks the whole contraction, which bounds every list)
    if (P.kb_cnt) kax.n = imin(imax(P.kb_cnt[n0 / BN], 0), imin(kax.nphys / 64, 128)) * 64;
  } else {
    const ClassTab& t = P.tab;
    int c = 0, l = -1;
    for (; c < t.ncls; ++c) {
      const int lo = (int)((long)xcd * t.nblk[c] / 8), hi = (int)((long)(xcd + 1) * t.nblk[c] / 8);
      if (local < hi - lo) {
        l = lo + local;
        break;
      }
      local -= hi - lo;
    }
    if (l < 0) return false;
    // bands of group_m row blocks, walked column by column (as in the plain case): an XCD's share
    // of a class is about square, so its operand panels are reused out of that XCD's L2
    const int nbc = t.nblk[c] / t.mblk[c];
    const int band_sz = P.group_m * nbc;
    const int band = l / band_sz, inb = l - band * band_sz;
    const int rows_in_band = imin(P.group_m, t.mblk[c] - band * P.group_m);
    const int mi = band * P.group_m + inb % rows_in_band, ni = inb / rows_in_band;
    if (t.m_bs) {
      const int g = F_BM / t.m_bs;
      const int left = t.m_cnt[c] - mi * g;
      am = axis_baff(t.m_off[c] + mi * g * t.m_step, t.m_step, t.m_bs, left < g ? left : g, t.m_phys);
    } else {
      m0 = mi * F_BM;
    }
    {
      const int g = BN / t.n_bs;
      const int left = t.n_cnt[c] - ni * g;
      bn = axis_baff(t.n_off[c] + ni * g * t.n_step, t.n_step, t.n_bs, left < g ? left : g, t.n_phys);
    }
    if (t.k_bs) kax = axis_baff(t.k_off[c], t.k_step, t.k_bs, t.k_cnt[c], t.k_phys);
  }
  w.am = am, w.bn = bn, w.kax = kax;
  w.m0 = m0, w.n0 = n0, w.split = split;
  return true;
}

// Physical start of the contraction slab of absolute step s: `ks` along the A operand, `ksb` along B
// (MODE 1: slab (tap, c0) of the im2col row = offset of the tap's pixel plus the channel).
template <int MODE>
__host__ __device__ __forceinline__ void direct_slab(const FastParams& P, const Axis& kax, int s, int& ks, int& ksb) {
  if constexpr (MODE == 1) {
    // The steps run channel group by channel group, all taps of a group in a row: consecutive steps then read
    // the same 128 bytes of pixels that lie a few positions apart, nearly all of them lines the step before
    // left in L2 (tap by tap, a whole pass over the tile's channels lies between two reads of a line).
    const int taps = kax.nphys / P.cv.Cp, cg = s / taps, t = s - cg * taps;
    ks = t * P.cv.Cp + cg * 64;
    ksb = ((t / P.cv.kw) * P.cv.Wg + t % P.cv.kw) * P.cv.Cp + cg * 64;
    return;
  }
  ks = fast_kslab(kax, s * 64);
  ksb = ks;
}

// MODE 0: plain product.  MODE 1: convolution, B rows are output pixels gathered from the
// bordered channels-last grid (contraction = (tap, channel)), output NCHW.  MODE 2: weight
// gradient of the convolution, contraction over the grid's pixels, B columns = (tap, channel).
// (body of the kernel as a device function: the grouped kernel of gemm.hip runs it on a range of
// its workgroups; block_id is the workgroup's index within the product, lds its dynamic LDS)
template <bool A_KC, bool B_KC, int F_BM, int BN, int NW, int MODE = 0>
__device__ __forceinline__ void direct_body(const FastParams& P, const int block_id, uint4* const lds) {
  constexpr int NST = direct_stages(F_BM, BN);
  constexpr int WGN = (NW == 8 && BN == 256) ? 4 : 2, WGM = NW / WGN;
  constexpr int WTM = F_BM / WGM, WTN = BN / WGN;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must hold whole MFMA tiles");
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int OPA = F_BM * LDS_ROW_U4, OPB = BN * LDS_ROW_U4;  // u4 entries of one operand stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  DirectWork wk;
  if (!direct_assign<F_BM, BN>(P, block_id, wk)) return;
  const Axis am = wk.am, bn = wk.bn, kax = wk.kax;
  const int m0 = wk.m0, n0 = wk.n0, split = wk.split;
  const int Kn = kax.n;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int im = 0; im < TM; ++im)
#pragma unroll
    for (int in = 0; in < TN; ++in)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[im][in][v] = 0.0f;

  // per-tile contraction list (MODE 1): lane l keeps the tile's l-th and (64+l)-th block, a step reads its
  // block out of the lane that holds it, so the loop touches no memory for the list
  int kbl0 = 0, kbl1 = 0;
  bool kb_mode = false;
  if constexpr (MODE == 1) {
    if (P.kb_cnt) {
      kb_mode = true;
      const int* lst = P.kb_list + (long)(n0 / BN) * P.kb_stride;
      const int cnt = Kn >> 6, last = kax.nphys / 64 - 1;
      // (read whatever the count says, from inside the tile's own row of the list: the loads do not wait for it)
      const int e0 = lst[imin(lane, P.kb_stride - 1)], e1 = lst[imin(64 + lane, P.kb_stride - 1)];
      kbl0 = lane < cnt ? imin(imax(e0, 0), last) : 0;
      kbl1 = 64 + lane < cnt ? imin(imax(e1, 0), last) : 0;
    }
  }
  // the pixels this lane's columns are stored to, looked up before the contraction instead of after it
  int out_pix[TN];
  if constexpr (MODE == 1) {
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      const int jc = n0 + wn * WTN + in * 32 + (lane & 31);
      out_pix[in] = jc < P.cv.npix ? (P.cv.pix ? P.cv.pix[jc] : jc) : -1;
    }
  }
  auto slab = [&](int s, int& ks, int& ksb) {
    if constexpr (MODE == 1) {
      if (kb_mode) {
        ks = (s < 64 ? __builtin_amdgcn_readlane(kbl0, s) : __builtin_amdgcn_readlane(kbl1, s - 64)) * 64;
        const int t = ks / P.cv.Cp;
        ksb = ((t / P.cv.kw) * P.cv.Wg + t % P.cv.kw) * P.cv.Cp + (ks - t * P.cv.Cp);
        return;
      }
    }
    direct_slab<MODE>(P, kax, s, ks, ksb);
  };

  if (Kn > 0) {
    DirectLoader<A_KC, F_BM, NW> la;
    DirectLoader<B_KC, BN, NW> lb;
    const int kbump = MODE == 0 ? direct_kbump(kax) : 0;
    la.init(P.A, P.lda, am, m0, lane, wave, kbump);
    if constexpr (MODE == 1) lb.init_pixels(P.B, P.cv, n0, lane, wave);
    else if constexpr (MODE == 2) lb.init_tap_columns(P.B, P.cv, P.N, n0, lane, wave);
    else lb.init(P.B, P.ldb, bn, n0, lane, wave, kbump);
    const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)lds);
    unsigned aaddr[TM][A_KC ? 4 : 1], baddr[TN][B_KC ? 4 : 1];
#pragma unroll
    for (int im = 0; im < TM; ++im) {
      if (A_KC) {
        const int row = wm * WTM + im * 32 + (lane & 31);
        const int xr = (row & 7) ^ ((row >> 3) & 7);
#pragma unroll
        for (int q = 0; q < 4; ++q) aaddr[im][q] = lds_base + (unsigned)(row * 8 + ((2 * q + (lane >> 5)) ^ xr)) * 16u;
      } else {
        aaddr[im][0] = lds_base + (unsigned)mc_frag_base<F_BM>(wm * WTM + im * 32, lane);
      }
    }
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      if (B_KC) {
        const int row = wn * WTN + in * 32 + (lane & 31);
        const int xr = (row & 7) ^ ((row >> 3) & 7);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          baddr[in][q] = lds_base + (unsigned)(NST * OPA + row * 8 + ((2 * q + (lane >> 5)) ^ xr)) * 16u;
      } else {
        baddr[in][0] = lds_base + (unsigned)(NST * OPA) * 16u + (unsigned)mc_frag_base<BN>(wn * WTN + in * 32, lane);
      }
    }
    // contraction steps of this workgroup (a share of them when the contraction is split)
    const int S_all = (Kn + 63) >> 6;
    const int s_lo = (int)((long)split * S_all / P.splits), s_hi = (int)((long)(split + 1) * S_all / P.splits);
    const int S = s_hi - s_lo;
    auto load_stage = [&](int it, int buf) {
      const int krem = Kn - (s_lo + it) * 64;
      int ks, ksb;
      slab(s_lo + it, ks, ksb);
      const bool tail = krem < 64 || ks + 64 + kbump > kax.nphys;
      if (__builtin_expect(tail, 0)) {
        la.issue_tail(lds + buf * OPA, ks, krem, kax.nphys, lane, wave, kbump);
        lb.issue_tail(lds + NST * OPA + buf * OPB, ksb, krem, MODE == 1 ? 0x7fffffff : kax.nphys, lane, wave, kbump);
      } else {
        la.issue(lds + buf * OPA, ks, wave);
        lb.issue(lds + NST * OPA + buf * OPB, ksb, wave);
      }
    };
    constexpr int QA = 16 * F_BM * 2, QB = 16 * BN * 2;  // bytes per 16-wide slice of an MC tile
    Frag fa[2][TM], fb[2][TN];
    // issue the fragment reads of slice Q of stage BUF (both compile-time: immediates) into `set`
    auto issue = [&](auto bufc, auto qc, int set) {
      constexpr int BUF = decltype(bufc)::value, Q = decltype(qc)::value;
      constexpr int SA = BUF * OPA * 16, SB = BUF * OPB * 16;  // byte offsets of the stage
#pragma unroll
      for (int im = 0; im < TM; ++im) {
        if (A_KC) {
          lds_read_b128<SA>(fa[set][im].v, aaddr[im][A_KC ? Q : 0]);
        } else {
          lds_read_tr16_b64<SA + Q * QA>(fa[set][im].lo, aaddr[im][0]);
          lds_read_tr16_b64<SA + Q * QA + QA / 4>(fa[set][im].hi, aaddr[im][0]);
        }
      }
#pragma unroll
      for (int in = 0; in < TN; ++in) {
        if (B_KC) {
          lds_read_b128<SB>(fb[set][in].v, baddr[in][B_KC ? Q : 0]);
        } else {
          lds_read_tr16_b64<SB + Q * QB>(fb[set][in].lo, baddr[in][0]);
          lds_read_tr16_b64<SB + Q * QB + QB / 4>(fb[set][in].hi, baddr[in][0]);
        }
      }
    };
    auto wait = [&](int set) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int im = 0; im < TM; ++im) frag_wait<A_KC>(fa[set][im]);
#pragma unroll
      for (int in = 0; in < TN; ++in) frag_wait<B_KC>(fb[set][in]);
    };
    auto mma = [&](int set) {
#pragma unroll
      for (int im = 0; im < TM; ++im)
#pragma unroll
        for (int in = 0; in < TN; ++in)
          acc[im][in] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_value<A_KC>(fa[set][im]),
                                                                frag_value<B_KC>(fb[set][in]), acc[im][in], 0, 0, 0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    // One contraction step from stage BUF.  Slice q+1's reads are in flight behind slice q's
    // MFMAs; the stage hand-over (wait for the next stage's loads, barrier, start the loads of
    // stage it+NST into the buffer just released, read the next stage's first slice) sits in
    // front of the LAST slice's MFMAs, so neither the barrier nor the first LDS latency of a
    // stage leaves the matrix cores idle.  Loads complete in order: with NST - 2 younger
    // stages allowed in flight, stage it+1 has landed.
    constexpr int LPS = decltype(la)::NI + decltype(lb)::NI;  // loads of one thread per stage
    auto step = [&](auto bufc, int it) {
      constexpr int BUF = decltype(bufc)::value;
      using B = std::integral_constant<int, BUF>;
      using NB = std::integral_constant<int, (BUF + 1) % NST>;
      wait(0);
      issue(B{}, I1{}, 1);
      mma(0);
      wait(1);
      issue(B{}, I2{}, 0);
      mma(1);
      wait(0);
      issue(B{}, I3{}, 1);
      mma(0);
      wait(1);
      if (it + 1 < S) {
        if (it + NST - 1 < S) wait_vmcnt<(NST - 2) * LPS>();
        else wait_vmcnt<0>();
        wg_barrier();  // stage it+1 is complete and visible; nobody reads stage it any more
        issue(NB{}, I0{}, 0);
      }
      mma(1);
      // the loads of stage it+NST go into the buffer just released; issued behind the MFMAs so
      // that nothing but the barrier and one fragment read sits between two slices' MFMAs
      if (it + NST < S) load_stage(it + NST, BUF);
    };
    // The same step where every question is settled: a successor stage exists, the stage to load
    // exists and is a full one (the axis is affine, or made of whole blocks that hold whole steps:
    // then only the last stage can be partial).  No tail handling, no branches.
    auto steady_step = [&](auto bufc, int it) {
      constexpr int BUF = decltype(bufc)::value;
      using B = std::integral_constant<int, BUF>;
      using NB = std::integral_constant<int, (BUF + 1) % NST>;
      wait(0);
      issue(B{}, I1{}, 1);
      mma(0);
      wait(1);
      issue(B{}, I2{}, 0);
      mma(1);
      wait(0);
      issue(B{}, I3{}, 1);
      mma(0);
      wait(1);
      wait_vmcnt<(NST - 2) * LPS>();
      wg_barrier();
      issue(NB{}, I0{}, 0);
      int ks, ksb;
      slab(s_lo + it + NST, ks, ksb);
      // the loads of stage it+NST spread between the last slice's MFMAs (a burst of LPS load instructions
      // keeps this wavefront from issuing MFMAs for as long as it takes to issue them)
      {
        constexpr int NA = decltype(la)::NI, MM = TM * TN;
        int li = 0, mi = 0;
#pragma unroll
        for (int im = 0; im < TM; ++im)
#pragma unroll
          for (int in = 0; in < TN; ++in) {
            acc[im][in] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_value<A_KC>(fa[1][im]), frag_value<B_KC>(fb[1][in]),
                                                                  acc[im][in], 0, 0, 0);
            ++mi;
#pragma unroll
            for (int r = 0; r < (LPS + MM - 1) / MM; ++r)
              if (li < LPS && li * MM < mi * LPS) {
                if (li < NA) la.issue_one(lds + BUF * OPA, ks, wave, li);
                else lb.issue_one(lds + NST * OPA + BUF * OPB, ksb, wave, li - NA);
                ++li;
              }
            __builtin_amdgcn_sched_barrier(0);
          }
      }
    };
    if (S > 0) {
#pragma unroll
      for (int st = 0; st < NST; ++st)
        if (st < S) load_stage(st, st);
      if (S >= NST) wait_vmcnt<(NST - 1) * LPS>();
      else wait_vmcnt<0>();
      wg_barrier();
      issue(I0{}, I0{}, 0);
      int it0 = 0;
      if (kax.kind == AX_AFFINE || (kax.kind == AX_BAFF && (kax.bs % 64 == 0 || kax.bs == 32) && kax.nphys % kax.bs == 0)) {
        // steps whose stage it+NST is not the last one (only the last can be partial)
        for (; it0 + 2 * NST < S; it0 += NST) {
          steady_step(I0{}, it0);
          steady_step(I1{}, it0 + 1);
          if (NST > 2) steady_step(std::integral_constant<int, 2 % NST>{}, it0 + 2);
          if (NST > 3) steady_step(std::integral_constant<int, 3 % NST>{}, it0 + 3);
        }
      }
      for (int it = it0; it < S; it += NST) {
        step(I0{}, it);
        if (NST > 1 && it + 1 < S) step(std::integral_constant<int, 1 % NST>{}, it + 1);
        if (NST > 2 && it + 2 < S) step(std::integral_constant<int, 2 % NST>{}, it + 2);
        if (NST > 3 && it + 3 < S) step(std::integral_constant<int, 3 % NST>{}, it + 3);
        static_assert(NST >= 2 && NST <= 4, "pipeline depth");
      }
    }
  }

  // epilogue: lane holds column (lane & 31) of each 32x32 tile, rows 8*(v/4) + 4*(lane>>5) + v%4.
  // Mapped rows / columns come in blocks that are multiples of 32, so one index lookup per
  // 32x32 tile places all of its rows (columns).
  const int nlim = P.c_cols_mapped ? bn.n : P.N, mlim = P.c_rows_mapped ? am.n : P.M;
  const int nphys = P.c_cols_mapped ? bn.nphys : P.N, mphys = P.c_rows_mapped ? am.nphys : P.M;
  // Columns at or beyond the B operand's extent (padding of a compact output) are stored as zeros:
  // the loaders fed them clamped, i.e. arbitrary, rows.
  const int n_valid = (MODE == 0 && P.tab.ncls == 0) ? bn.n : 0x7fffffff;
  // (the 256 x 256 tile has no registers to spare: it only stores plain bf16 results)
  constexpr bool GENERAL_OUT = !(F_BM == 256 && BN == 256);
  if (GENERAL_OUT && P.part) {
    // fp32 partial sums of this share of the contraction, compact [M x N]
    float* part = P.part + (long)split * P.M * P.N;
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      const int j = n0 + wn * WTN + in * 32 + (lane & 31);
      if (j >= P.N) continue;
#pragma unroll
      for (int im = 0; im < TM; ++im) {
        const int i0 = m0 + wm * WTM + im * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = i0 + 8 * (v >> 2) + (v & 3);
          if (i < P.M) part[(long)i * P.N + j] = j < n_valid ? acc[im][in][v] : 0.0f;
        }
      }
    }
    return;
  }
  if constexpr (MODE == 1) {
    // NCHW output: compact row i -> channel (through the kept-channel list when there is one),
    // column j -> pixel (n, hw) at n*out_chan*HW + hw.  Pairs of adjacent pixels are packed
    // into 32-bit stores as below when the plane size is even.
    const ConvMap& cv = P.cv;
    const int HW = cv.HoWo;
    const bool odd = lane & 1;
    // (listed pixels are not adjacent unless the list says so)
    const bool pair_ok = ((HW & 1) == 0) && (((uintptr_t)P.C & 3) == 0) && (!cv.pix || cv.pix_pairs);
    // Consecutive pixels in planes of whole 16-byte pieces: the tile goes through LDS (the operand stages are
    // dead by now) as bf16 [row][BN pixels] and leaves as 16-byte stores, a row of the tile one contiguous run
    // of 2 BN bytes of its channel's plane (straight from the registers a store instruction writes runs of 64).
    // Rows lie 2 BN bytes apart; the 16-byte pieces of a row are exchanged by two bits of its number, so the
    // four rows one store instruction of a wave touches land on different banks.
    if (!cv.pix && (HW & 7) == 0 && (((uintptr_t)P.C & 15) == 0)) {
      constexpr int CH = BN / 8;                               // 16-byte pieces per row
      constexpr int NT = 64 * NW;
      static_assert(NT % CH == 0, "whole rows per pass");
      static_assert(F_BM * BN * 2 <= NST * (F_BM + BN) * LDS_ROW_U4 * 16, "the staged tile fits the operand stages");
      char* const tile = reinterpret_cast<char*>(lds);
      auto piece_of = [](int row, int piece) { return piece ^ ((((row & 1) << 2) | (((row >> 2) & 1) << 3)) & (CH - 1)); };
      __syncthreads();
#pragma unroll
      for (int in = 0; in < TN; ++in) {
        const int lj = wn * WTN + in * 32 + (lane & 31);
#pragma unroll
        for (int im = 0; im < TM; ++im) {
          const int li0 = wm * WTM + im * 32 + 4 * (lane >> 5);
#pragma unroll
          for (int v = 0; v < 16; v += 2) {
            float x0 = P.alpha * acc[im][in][v], x1 = P.alpha * acc[im][in][v + 1];
            if (P.relu) {
              x0 = fmaxf(x0, 0.0f);
              x1 = fmaxf(x1, 0.0f);
            }
            const uint32_t b01 = pack_bf16x2(x0, x1);
            const uint32_t b0 = b01 & 0xffffu, b1 = b01 >> 16;
            // the even lane keeps row v of its own and its neighbour's pixel, the odd lane row v + 1
            const uint32_t send = odd ? b0 : b1;
            const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0xB1, 0xF, 0xF, true);
            const uint32_t word = odd ? (got | (b1 << 16)) : (b0 | (got << 16));
            const int row = li0 + 8 * (v >> 2) + (v & 3) + (odd ? 1 : 0);
            const int w = lj >> 1;  // word of the row: pixels 2w, 2w + 1
            *reinterpret_cast<uint32_t*>(tile + row * (BN * 2) + piece_of(row, w >> 2) * 16 + (w & 3) * 4) = word;
          }
        }
      }
      __syncthreads();
      const int piece = tid % CH;
      const int jc = n0 + piece * 8;
      if (jc >= cv.npix) return;  // (npix is a multiple of 8 here: a piece is in or out as a whole)
      const int n = jc / HW;
      uint16_t* const col = P.C + (long)n * cv.out_chan * HW + (jc - n * HW);
      for (int r = tid / CH; r < F_BM; r += NT / CH) {
        const int i = m0 + r;
        if (i >= cv.n_rows) break;
        const int ch = cv.chan ? cv.chan[i] : i;
        *reinterpret_cast<uint4*>(col + (long)ch * HW) = *reinterpret_cast<const uint4*>(tile + r * (BN * 2) + piece_of(r, piece) * 16);
      }
      return;
    }
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      const int j = out_pix[in];  // (columns beyond npix hold -1; npix is even whenever pair_ok: a pair is in or out together)
      if (j < 0) continue;        // padding entry of a tile
      const int n = j / HW;
      uint16_t* col = P.C + (long)n * cv.out_chan * HW + (j - n * HW);
#pragma unroll
      for (int im = 0; im < TM; ++im) {
        const int i0 = m0 + wm * WTM + im * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
          const int ia = i0 + 8 * (v >> 2) + (v & 3);  // row of v; v+1 is the next row
          float x0 = P.alpha * acc[im][in][v], x1 = P.alpha * acc[im][in][v + 1];
          if (P.relu) {
            x0 = fmaxf(x0, 0.0f);
            x1 = fmaxf(x1, 0.0f);
          }
          const uint32_t b01 = pack_bf16x2(x0, x1);
          const uint32_t b0 = b01 & 0xffffu, b1 = b01 >> 16;
          if (pair_ok) {
            const uint32_t send = odd ? b0 : b1;
            const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0xB1, 0xF, 0xF, true);
            const uint32_t word = odd ? (got | (b1 << 16)) : (b0 | (got << 16));
            const int i = odd ? ia + 1 : ia;
            if (i < cv.n_rows) {
              const int ch = cv.chan ? cv.chan[i] : i;
              *reinterpret_cast<uint32_t*>(col - (odd ? 1 : 0) + (long)ch * HW) = word;
            }
          } else {
            if (ia < cv.n_rows) col[(long)(cv.chan ? cv.chan[ia] : ia) * HW] = (uint16_t)b0;
            if (ia + 1 < cv.n_rows) col[(long)(cv.chan ? cv.chan[ia + 1] : ia + 1) * HW] = (uint16_t)b1;
          }
        }
      }
    }
    return;
  }
  if (GENERAL_OUT && MODE == 0 && P.scatter) {
    // final bf16 values -> LDS (the operand stages are dead once every wave is past its last read)
    constexpr int LDT = BN + 2;
    uint16_t* tile = reinterpret_cast<uint16_t*>(lds);
    __syncthreads();
#pragma unroll
    for (int im = 0; im < TM; ++im)
#pragma unroll
      for (int in = 0; in < TN; ++in) {
        const int lj = wn * WTN + in * 32 + (lane & 31);
        const int li0 = wm * WTM + im * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float x = n0 + lj < n_valid ? P.alpha * acc[im][in][v] : 0.0f;
          if (P.relu) x = fmaxf(x, 0.0f);
          tile[(li0 + 8 * (v >> 2) + (v & 3)) * LDT + lj] = f32_to_bf16_bits(x);
        }
      }
    __syncthreads();
    const int m1 = min(m0 + F_BM, P.M), n1 = min(n0 + BN, P.N);
    if (P.scatter_vec) direct_scatter_tile<true>(tile, LDT, P, m0, m1, n0, n1, tid, 64 * NW);
    else direct_scatter_tile<false>(tile, LDT, P, m0, m1, n0, n1, tid, 64 * NW);
    return;
  }
  int prow[TM];
#pragma unroll
  for (int im = 0; im < TM; ++im) {
    const int i0 = m0 + wm * WTM + im * 32;
    prow[im] = i0 < mlim ? (P.c_rows_mapped ? ax_phys(am, i0) : i0) : mphys;
  }
  const bool plain_bf16 = !GENERAL_OUT || (!P.out_f32 && P.beta == 0.0f);
#pragma unroll
  for (int in = 0; in < TN; ++in) {
    const int j0 = n0 + wn * WTN + in * 32;
    if (j0 >= nlim) continue;
    const int pc = (P.c_cols_mapped ? ax_phys(bn, j0) : j0) + (lane & 31);
    if (pc >= nphys) continue;
#pragma unroll
    for (int im = 0; im < TM; ++im) {
      const int rbase = prow[im] + 4 * (lane >> 5);
      if (!plain_bf16) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = rbase + 8 * (v >> 2) + (v & 3);
          if (r >= mphys) continue;
          const long idx = (long)r * P.ldc + pc;
          float x = (j0 + (lane & 31)) < n_valid ? P.alpha * acc[im][in][v] : 0.0f;
          if (P.beta != 0.0f) x += P.beta * (P.out_f32 ? reinterpret_cast<const float*>(P.C)[idx] : bf16_bits_to_f32(P.C[idx]));
          if (P.relu) x = fmaxf(x, 0.0f);
          if (P.relu_src) x = bf16_bits_to_f32(P.relu_src[idx]) > 0.0f ? x : 0.0f;
          if (P.out_f32) reinterpret_cast<float*>(P.C)[idx] = x;
          else P.C[idx] = f32_to_bf16_bits(x);
        }
        continue;
      }
      // Adjacent lanes hold adjacent columns of the same row.  Rows come in pairs (v, v+1):
      // the even lane takes the odd lane's value of row v, the odd lane the even lane's value
      // of row v+1 (one DPP swap), and each stores one packed 32-bit word.
      const bool odd = lane & 1;
      uint16_t* dst = P.C + (long)rbase * P.ldc + (pc & ~1);
      const bool pair_ok = ((pc | 1) < nphys) && ((P.ldc & 1) == 0) && ((nphys & 1) == 0) && (((uintptr_t)P.C & 3) == 0) &&
                           (((uintptr_t)P.relu_src & 3) == 0);
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        float x0 = P.alpha * acc[im][in][v], x1 = P.alpha * acc[im][in][v + 1];
        if (P.relu) {
          x0 = fmaxf(x0, 0.0f);
          x1 = fmaxf(x1, 0.0f);
        }
        if ((j0 + (lane & 31)) >= n_valid) x0 = x1 = 0.0f;
        const uint32_t b01 = pack_bf16x2(x0, x1);
        const uint32_t b0 = b01 & 0xffffu, b1 = b01 >> 16;
        const int dr0 = 8 * (v >> 2) + (v & 3);  // row of v; v+1 is the next row
        if (pair_ok) {
          const uint32_t send = odd ? b0 : b1;
          const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0xB1, 0xF, 0xF, true);  // swap with lane^1
          const uint32_t word = odd ? (got | (b1 << 16)) : (b0 | (got << 16));
          const int dr = odd ? dr0 + 1 : dr0;
          if (rbase + dr < mphys) {
            uint32_t out = word;
            if (GENERAL_OUT && P.relu_src) {
              // ReLU mask of the same two positions (same layout as the output)
              const uint32_t g = *reinterpret_cast<const uint32_t*>(P.relu_src + (long)(rbase + dr) * P.ldc + (pc & ~1));
              if (!(bf16_bits_to_f32((uint16_t)(g & 0xffffu)) > 0.0f)) out &= 0xffff0000u;
              if (!(bf16_bits_to_f32((uint16_t)(g >> 16)) > 0.0f)) out &= 0x0000ffffu;
            }
            *reinterpret_cast<uint32_t*>(dst + (long)dr * P.ldc) = out;
          }
        } else {
          uint16_t* d1 = P.C + (long)rbase * P.ldc + pc;
          const uint16_t* g1 = P.relu_src + (long)rbase * P.ldc + pc;
          uint16_t o0 = (uint16_t)b0, o1 = (uint16_t)b1;
          if (GENERAL_OUT && P.relu_src) {
            if (rbase + dr0 < mphys && !(bf16_bits_to_f32(g1[(long)dr0 * P.ldc]) > 0.0f)) o0 = 0;
            if (rbase + dr0 + 1 < mphys && !(bf16_bits_to_f32(g1[(long)(dr0 + 1) * P.ldc]) > 0.0f)) o1 = 0;
          }
          if (rbase + dr0 < mphys) d1[(long)dr0 * P.ldc] = o0;
          if (rbase + dr0 + 1 < mphys) d1[(long)(dr0 + 1) * P.ldc] = o1;
        }
      }
    }
  }
}

template <bool A_KC, bool B_KC, int F_BM, int BN, int NW, int MODE = 0>
__global__ __launch_bounds__(64 * NW) void gemm_direct_kernel(const FastParams P) {
  extern __shared__ uint4 direct_lds[];
  direct_body<A_KC, B_KC, F_BM, BN, NW, MODE>(P, (int)blockIdx.x, direct_lds);
}

// Finishing pass of a product whose result could not be stored by the GEMM itself (split
// contraction, or an output scattered at element granularity with dropped positions to zero):
// sums the fp32 partials part[split][M][N] and writes the output through its maps, walking the
// PHYSICAL output when dropped positions have to be written.
__device__ __forceinline__ int ax_inverse(const Axis& a, int p) {
  // compact index of physical index p, or -1
  if (a.kind == AX_AFFINE) {
    const int d = p - a.off;
    if (d < 0 || d % a.step) return -1;
    const int j = d / a.step;
    return j < a.n ? j : -1;
  }
  if (a.kind == AX_LIST) {
    int lo = 0, hi = a.n - 1;
    while (lo <= hi) {
      const int mid = (lo + hi) >> 1, v = a.list[mid];
      if (v == p) return mid;
      if (v < p) lo = mid + 1;
      else hi = mid - 1;
    }
    return -1;
  }
  return -1;
}

template <typename T>
__global__ __launch_bounds__(256) void gemm_finish_kernel(const float* part, int splits, int M, int N, OutMat C) {
  const int rows = C.fill ? C.rm.nphys : M, cols = C.fill ? C.cn.nphys : N;
  const long total = (long)rows * cols;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
    const int r = (int)(e / cols), c = (int)(e - (long)r * cols);
    int i, j, pr, pc;
    if (C.fill) {
      pr = r, pc = c;
      i = ax_inverse(C.rm, r);
      j = ax_inverse(C.cn, c);
    } else {
      i = r, j = c;
      pr = ax_phys(C.rm, r);
      pc = ax_phys(C.cn, c);
    }
    float x = 0.0f;
    if (i >= 0 && j >= 0) {
      const float* p = part + (long)i * N + j;
      for (int s = 0; s < splits; ++s) x += p[(long)s * M * N];
      x *= C.alpha;
    }
    store_out<T>(C, (long)pr * C.ld + pc, x, true);
  }
}

// The same pass for bf16 outputs whose rows can be written in 16-byte pieces (host checks:
// bf16 result, beta == 0, 16-byte aligned rows, column count a multiple of 8; without zero
// fill the column map is the identity).  A thread produces 8 adjacent physical columns.
struct FinishArgs {
  const float* part;
  int splits, M, N;
  OutMat C;
};
static __device__ __forceinline__ void finish_vec_body(const FinishArgs& a, const int bx, const int by, const int gy) {
  const float* part = a.part;
  const int splits = a.splits, M = a.M, N = a.N;
  const OutMat& C = a.C;
  // grid: x over the 8-column pieces of a row, y over rows (uniform per workgroup, so the row
  // lookup is scalar work)
  const int rows = C.fill ? C.rm.nphys : M, cols8 = (C.fill ? C.cn.nphys : N) >> 3;
  const long MN = (long)M * N;
  const int piece = bx * 256 + threadIdx.x;
  if (piece >= cols8) return;
  const int c0 = piece * 8;
  // Workgroup ids go round-robin over the 8 XCDs: XCD x takes the contiguous rows
  // [x * chunk, (x + 1) * chunk).  (Row r on XCD r % 8 would put every kept row of a step-8
  // pattern, i.e. all the work, on one XCD.)
  const int chunk = (rows + 7) >> 3;
  for (int y = by; y < chunk * 8; y += gy) {
    const int r = (y & 7) * chunk + (y >> 3);
    if (r >= rows) continue;
    const int i = C.fill ? ax_inverse(C.rm, r) : r;
    const int pr = C.fill ? r : ax_phys(C.rm, r);
    const long idx = (long)pr * C.ld + c0;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (i >= 0) {
      uint4 gate = make_uint4(0, 0, 0, 0);
      if (C.relu_src) gate = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(C.relu_src) + idx);
      const uint32_t* gw = reinterpret_cast<const uint32_t*>(&gate);
      int j = C.fill ? -1 : c0;
      if (C.fill && C.cn.kind == AX_AFFINE) {
        // first kept column at or after c0 (exact for the 24-bit operands of this division)
        const int d = c0 - C.cn.off + C.cn.step - 1;
        j = 0;
        if (d >= C.cn.step) {
          j = (int)((float)d / (float)C.cn.step);
          j += ((j + 1) * C.cn.step <= d) - (j * C.cn.step > d);
        }
      }
      int jj[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        if (!C.fill) jj[t] = j + t;
        else if (C.cn.kind == AX_AFFINE) jj[t] = (j < C.cn.n && C.cn.off + j * C.cn.step == c0 + t) ? j++ : -1;
        else jj[t] = ax_inverse(C.cn, c0 + t);
      }
      // the 8 loads of one split are independent; splits are summed in order
      float x[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
      const float* prow = part + (long)i * N;
      for (int sp = 0; sp < splits; ++sp) {
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = jj[t] >= 0 ? prow[sp * MN + jj[t]] : 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t) x[t] += v[t];
      }
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        if (jj[t] < 0) continue;
        float v = x[t] * C.alpha;
        if (C.relu) v = fmaxf(v, 0.0f);
        if (C.relu_src) {
          const uint32_t g = (gw[t >> 1] >> (16 * (t & 1))) & 0xffffu;
          v = bf16_bits_to_f32((uint16_t)g) > 0.0f ? v : 0.0f;
        }
        w[t >> 1] |= (uint32_t)f32_to_bf16_bits(v) << (16 * (t & 1));
      }
    }
    *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(C.p) + idx) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

static __global__ __launch_bounds__(256) void gemm_finish_vec_kernel(const FinishArgs a) {
  finish_vec_body(a, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y);
}

// Rows of a bf16 matrix that an affine row map (off + i * step, i < n_kept) does NOT reach, set to +0.0:
// the dropped output neurons of a weight gradient.  Independent of the product that writes the kept rows.
struct ZeroRowsArgs {
  uint16_t* C;
  int ld, rows, cols, off, step, n_kept, vec;
};
static __device__ __forceinline__ void zero_rows_body(const ZeroRowsArgs& a, const int bx, const int nblocks) {
  const int dropped = a.rows - a.n_kept;
  const int per_row = a.vec ? a.cols >> 3 : a.cols;
  const long total = (long)dropped * per_row;
  for (long e = (long)bx * 256 + threadIdx.x; e < total; e += (long)nblocks * 256) {
    // (a 64-bit division costs several times a 32-bit one, and nearly every matrix stays below 2^32 pieces)
    const int d = total < (1L << 32) ? (int)((uint32_t)e / (uint32_t)per_row) : (int)(e / per_row);
    const int c = (int)(e - (long)d * per_row);
    // d-th dropped row: rows before `off` come first, then step - 1 per group, then the tail
    int r;
    if (d < a.off) {
      r = d;
    } else {
      const int q = (d - a.off) / (a.step - 1), t = (d - a.off) - q * (a.step - 1);
      r = q < a.n_kept ? a.off + q * a.step + 1 + t : a.off + a.n_kept * a.step + (d - a.off - a.n_kept * (a.step - 1)) - (a.step - 1);
    }
    if (a.vec) *reinterpret_cast<uint4*>(a.C + (long)r * a.ld + c * 8) = make_uint4(0, 0, 0, 0);
    else a.C[(long)r * a.ld + c] = 0;
  }
}
static __global__ __launch_bounds__(256) void zero_rows_kernel(const ZeroRowsArgs a) {
  zero_rows_body(a, (int)blockIdx.x, (int)gridDim.x);
}

// Zero the dropped tiles of a tile-masked matrix (weight gradient): one workgroup per tile.
static __global__ __launch_bounds__(256) void zero_dropped_tiles_kernel(uint16_t* C, int ld, int rows, int cols, int tr, int tc,
                                                                 int TC, int dp, int o) {
  const int t = blockIdx.x;
  if (((t + dp - o) % dp) == 0) return;  // kept tile: written by the GEMM
  const int r0 = (t / TC) * tr, c0 = (t % TC) * tc;
  const int h = min(tr, rows - r0), w = min(tc, cols - c0);
  if (((w | c0 | ld) & 7) == 0) {
    const int w8 = w >> 3;
    for (int i = threadIdx.x; i < h * w8; i += 256) {
      const int r = i / w8, c = (i - r * w8) * 8;
      *reinterpret_cast<uint4*>(C + (long)(r0 + r) * ld + c0 + c) = make_uint4(0, 0, 0, 0);
    }
  } else {
    for (int i = threadIdx.x; i < h * w; i += 256) {
      const int r = i / w, c = i - r * w;
      C[(long)(r0 + r) * ld + c0 + c] = 0;
    }
  }
}

// Grid of a plain (class-free) launch: every XCD takes the share [x*n/8, (x+1)*n/8) of the tiles.
static inline int direct_plain_grid(int total_tiles) {
  int worst = 0;
  for (int x = 0; x < 8; ++x) {
    const int sum = (int)((long)(x + 1) * total_tiles / 8) - (int)((long)x * total_tiles / 8);
    worst = sum > worst ? sum : worst;
  }
  return worst * 8;
}

// ---- host-side bounds proof of the LDS-direct loaders -------------------------------------------
// A lane of these kernels forms its global address as base + uniform slab offset + per-lane offset
// with no bounds test in the loop, so the host shows before every launch that no lane of any
// workgroup can leave the operand (a_elems / b_elems elements behind A / B, stated by the caller).
//  * direct_envelope (always, O(classes)): the extreme physical rows, columns and contraction
//    indices the clamps in DirectLoader::init* and the tail rules allow, as inequalities.
//  * direct_prove (dry-run mode and ARD_PROVE_BOUNDS=1, every workgroup x wave x lane x step): runs
//    the kernel's own assignment and address arithmetic (direct_assign, DirectLoader::init*,
//    direct_slab, tail_live are host-callable) and records the smallest and largest byte touched.
static inline bool axis_rows_ok(const Axis& r, bool has_list) {
  // rows of a KC operand after the clamp of init(): min(row, n-1), block axes also clamped to nphys-1
  if (r.n < 1 || r.nphys < 1) return false;
  if (r.kind == AX_AFFINE) return r.off >= 0 && r.step >= 0 && (long)r.off + (long)(r.n - 1) * r.step < r.nphys;
  if (r.kind == AX_BAFF) return r.off >= 0 && r.step >= 0 && r.bs >= 1;
  if (r.kind == AX_LIST) return has_list && r.n <= r.nphys;  // entries are the caller's contract
  return false;
}
static inline bool axis_cols_ok(const Axis& r, int ld) {
  // 8-column runs of an MC operand after the clamp of init(): min(col, n-8), block axes to nphys-8
  if (r.n < 8 || r.nphys < 8 || r.nphys > ld) return false;
  if (r.kind == AX_AFFINE) return r.step == 1 && r.off >= 0 && r.off + r.n <= r.nphys;
  if (r.kind == AX_BAFF) return r.off >= 0 && r.step >= 0 && r.bs >= 8 && (r.bs % 8) == 0;
  return false;
}

template <bool A_KC, bool B_KC, int BM, int BN, int MODE>
static int32_t direct_envelope(const FastParams& F) {
  if (F.a_elems <= 0 || F.b_elems <= 0) return fail(ARD_EINVAL, "bounds proof: operand extents not stated");
  if (F.a_elems >= (1L << 31) || F.b_elems >= (1L << 31)) return fail(ARD_ESHAPE, "bounds proof: operand beyond 32-bit offsets");
  if (F.lda < 8 || F.ldb < 8) return fail(ARD_ESHAPE, "bounds proof: leading dimension below one 16-byte run");
  const ClassTab& t = F.tab;
  const int ncls = t.ncls ? t.ncls : 1;
  for (int c = 0; c < ncls; ++c) {
    if (t.ncls && t.nblk[c] == 0) continue;
    // the maps a workgroup of this class can get (direct_assign): whole progression of the class
    Axis am = F.am, bn = F.bn, k = F.k;
    if (t.ncls) {
      if (t.m_bs) am = axis_baff(t.m_off[c], t.m_step, t.m_bs, t.m_cnt[c], t.m_phys);
      bn = axis_baff(t.n_off[c], t.n_step, t.n_bs, t.n_cnt[c], t.n_phys);
      if (t.k_bs) k = axis_baff(t.k_off[c], t.k_step, t.k_bs, t.k_cnt[c], t.k_phys);
    }
    if (k.n <= 0) continue;  // nothing is loaded
    if (k.kind != AX_AFFINE && k.kind != AX_BAFF) return fail(ARD_EINVAL, "bounds proof: contraction map kind %d", k.kind);
    if (k.kind == AX_AFFINE && (k.step != 1 || k.off < 0 || k.off + k.n > k.nphys))
      return fail(ARD_ESHAPE, "bounds proof: contraction [%d, %d) outside its extent %d", k.off, k.off + k.n, k.nphys);
    if (k.kind == AX_BAFF && (k.off < 0 || k.step < 0 || k.bs < 32 || (k.bs % 64 && k.bs != 32)))
      return fail(ARD_ESHAPE, "bounds proof: contraction blocks of %d", k.bs);
    // 32-wide blocks: the upper half of a step lies `step` blocks further; the last kept block must
    // start inside the extent (a step that reaches beyond it takes the tail rule, chunk by chunk)
    if (k.kind == AX_BAFF && k.bs == 32 &&
        ((k.nphys % 8) || (k.n % 32) || ((long)k.off + (long)(k.n / 32 - 1) * k.step) * 32 >= k.nphys))
      return fail(ARD_ESHAPE, "bounds proof: 32-wide contraction blocks (%d of them from %d every %d) leave the extent %d", k.n / 32,
                  k.off, k.step, k.nphys);
    // every contraction index a live lane touches is < k.nphys (full steps need ks + 64 <= nphys, the
    // lanes of a partial step test their own chunk against nphys)
    const long kphys = k.nphys;
    // A
    if (A_KC) {
      if (!axis_rows_ok(am, F.A != nullptr) || kphys > F.lda || (long)am.nphys * F.lda > F.a_elems)
        return fail(ARD_ESHAPE, "bounds proof: A rows (kind %d, n %d, extent %d, ld %d, k %ld) leave %ld elements", am.kind, am.n,
                    am.nphys, F.lda, kphys, F.a_elems);
    } else {
      if (!axis_cols_ok(am, F.lda) || kphys * F.lda > F.a_elems)
        return fail(ARD_ESHAPE, "bounds proof: A columns (kind %d, n %d, extent %d, ld %d, k %ld) leave %ld elements", am.kind,
                    am.n, am.nphys, F.lda, kphys, F.a_elems);
    }
    // B
    if (MODE == 1) {
      const ConvMap& cv = F.cv;
      if (cv.npix < 1 || cv.Cp < 64 || (cv.Cp % 64) || cv.kw < 1 || kphys % cv.Cp) return fail(ARD_ESHAPE, "bounds proof: bad grid");
      // (a list with per-tile contraction lists is padded tile by tile and may be longer than the pixels)
      if (cv.pix && (cv.pix_total < 1 || (cv.npix > cv.pix_total && !F.kb_cnt)))
        return fail(ARD_ESHAPE, "bounds proof: pixel list longer than the pixels");
      if (F.kb_cnt && (!cv.pix || !F.kb_list || F.kb_stride < 1 || F.splits > 1 || k.kind != AX_AFFINE || (kphys % 64)))
        return fail(ARD_EINVAL, "bounds proof: per-tile contraction lists need a pixel list, whole 64-wide blocks and no split");
      const int row = (cv.pix ? cv.pix_total : cv.npix) - 1, n = row / cv.HoWo, rem = row - n * cv.HoWo;
      const long base = (long)n * cv.HgWg + (long)(rem / cv.Wo) * cv.Wg + rem % cv.Wo;
      const int tl = (int)(kphys / cv.Cp) - 1;  // last tap
      const long last = base + (long)(tl / cv.kw) * cv.Wg + tl % cv.kw;
      if ((last + 1) * cv.Cp > F.b_elems) return fail(ARD_ESHAPE, "bounds proof: patch rows leave the grid");
    } else if (MODE == 2) {
      const ConvMap& cv = F.cv;
      if (F.N < 8 || cv.Cp < 64 || (cv.Cp % 64) || cv.kw < 1) return fail(ARD_ESHAPE, "bounds proof: bad grid");
      const int tl = (F.N - 8) / cv.Cp;
      const long shift = (long)(tl / cv.kw) * cv.Wg + tl % cv.kw;
      if ((kphys - 1 + shift + 1) * cv.Cp > F.b_elems) return fail(ARD_ESHAPE, "bounds proof: shifted grid rows leave the grid");
    } else if (B_KC) {
      if (!axis_rows_ok(bn, F.B != nullptr) || kphys > F.ldb || (long)bn.nphys * F.ldb > F.b_elems)
        return fail(ARD_ESHAPE, "bounds proof: B rows (kind %d, n %d, extent %d, ld %d, k %ld) leave %ld elements", bn.kind, bn.n,
                    bn.nphys, F.ldb, kphys, F.b_elems);
    } else {
      if (!axis_cols_ok(bn, F.ldb) || kphys * F.ldb > F.b_elems)
        return fail(ARD_ESHAPE, "bounds proof: B columns (kind %d, n %d, extent %d, ld %d, k %ld) leave %ld elements", bn.kind,
                    bn.n, bn.nphys, F.ldb, kphys, F.b_elems);
    }
  }
  return ARD_OK;
}

// A LIST axis cannot be read on the host: its two extreme readings (every row first / last) bound it.
static inline Axis axis_list_surrogate(const Axis& r, bool last) {
  return r.kind == AX_LIST ? Axis{nullptr, AX_AFFINE, last ? r.nphys - 1 : 0, 0, 1, r.n, r.nphys} : r;
}

template <bool A_KC, bool B_KC, int BM, int BN, int NW, int MODE>
static int32_t direct_prove(const FastParams& P_in, int grid_x, DirectBounds& out) {
  constexpr long NONE_LO = 0x7fffffffffffffffL;
  out = DirectBounds{NONE_LO, -1, NONE_LO, -1};
  using LA = DirectLoader<A_KC, BM, NW>;
  using LB = DirectLoader<B_KC, BN, NW>;
  FastParams P = P_in;
  P.kb_cnt = nullptr;  // device memory: every list of whole blocks stays inside the full contraction walked here
  P.kb_list = nullptr;
  for (int bid = 0; bid < grid_x; ++bid) {
    DirectWork wk;
    if (!direct_assign<BM, BN>(P, bid, wk)) continue;
    const int Kn = wk.kax.n;
    if (Kn <= 0) continue;
    const int S_all = (Kn + 63) >> 6;
    const int s_lo = (int)((long)wk.split * S_all / P.splits), s_hi = (int)((long)(wk.split + 1) * S_all / P.splits);
    for (int pass = 0; pass < 2; ++pass) {  // (second pass only differs for LIST axes and pixel lists)
      if (pass == 1 && wk.am.kind != AX_LIST && wk.bn.kind != AX_LIST && !P.cv.pix) break;
      const Axis am = axis_list_surrogate(wk.am, pass == 1), bn = axis_list_surrogate(wk.bn, pass == 1);
      ConvMap cvp = P.cv;  // a pixel list lives in device memory: its two extreme readings bound it
      if (cvp.pix) cvp.pix = nullptr, cvp.pix_fixed = pass == 1 ? cvp.pix_total - 1 : 0;
      for (int wave = 0; wave < NW; ++wave)
        for (int lane = 0; lane < 64; ++lane) {
          LA la;
          LB lb;
          const int kbump = MODE == 0 ? direct_kbump(wk.kax) : 0;
          la.init(P.A, P.lda, am, wk.m0, lane, wave, kbump);
          if constexpr (MODE == 1) lb.init_pixels(P.B, cvp, wk.n0, lane, wave);
          else if constexpr (MODE == 2) lb.init_tap_columns(P.B, P.cv, P.N, wk.n0, lane, wave);
          else lb.init(P.B, P.ldb, bn, wk.n0, lane, wave, kbump);
          for (int s = s_lo; s < s_hi; ++s) {
            const int krem = Kn - s * 64;
            int ks, ksb;
            direct_slab<MODE>(P, wk.kax, s, ks, ksb);
            const bool tail = krem < 64 || ks + 64 + kbump > wk.kax.nphys;
            const int kend_b = MODE == 1 ? 0x7fffffff : wk.kax.nphys;
            for (int j = 0; j < LA::NI; ++j) {
              if (tail && !LA::tail_live(lane, wave, j, ks, krem, wk.kax.nphys, kbump)) continue;
              const long o = la.byte_offset(j, ks);
              out.a_lo = o < out.a_lo ? o : out.a_lo;
              out.a_hi = o + 16 > out.a_hi ? o + 16 : out.a_hi;
            }
            for (int j = 0; j < LB::NI; ++j) {
              if (tail && !LB::tail_live(lane, wave, j, ksb, krem, kend_b, kbump)) continue;
              const long o = lb.byte_offset(j, ksb);
              out.b_lo = o < out.b_lo ? o : out.b_lo;
              out.b_hi = o + 16 > out.b_hi ? o + 16 : out.b_hi;
            }
          }
        }
    }
  }
  const long a_bytes = (P.a_elems - extent_slack()) * 2, b_bytes = (P.b_elems - extent_slack()) * 2;
  if (out.a_hi >= 0 && (out.a_lo < 0 || out.a_hi > a_bytes))
    return fail(ARD_ESHAPE, "bounds proof: A bytes [%ld, %ld) outside [0, %ld)", out.a_lo, out.a_hi, a_bytes);
  if (out.b_hi >= 0 && (out.b_lo < 0 || out.b_hi > b_bytes))
    return fail(ARD_ESHAPE, "bounds proof: B bytes [%ld, %ld) outside [0, %ld)", out.b_lo, out.b_hi, b_bytes);
  return ARD_OK;
}

// Kinds of LDS-direct products the grouped kernel holds (the 4-wavefront tiles a batch-1024 layer chain
// uses); -1: this instantiation is always launched by itself.
enum { GK_DIRECT_KK_64 = 0, GK_DIRECT_KM_64 = 1, GK_DIRECT_MM_64 = 2, GK_DIRECT_MM_128x64 = 3, GK_COMPACT_W = 10, GK_FINISH_VEC = 11,
       GK_ZERO_ROWS = 12 };
template <bool A_KC, bool B_KC, int BM, int BN, int NW, int MODE>
constexpr int direct_group_kind() {
  if (MODE != 0 || NW != 4) return -1;
  if (BM == 64 && BN == 64) return A_KC ? (B_KC ? GK_DIRECT_KK_64 : GK_DIRECT_KM_64) : (B_KC ? -1 : GK_DIRECT_MM_64);
  if (BM == 128 && BN == 64 && !A_KC && !B_KC) return GK_DIRECT_MM_128x64;
  return -1;
}
// records the launch in this thread's open batch; false: no batch is open (gemm.hip)
bool batch_push_direct(int kind, const FastParams& F, int grid_x, size_t lds_bytes);
bool batch_push_finish(const FinishArgs& a, int gx, int gy);
bool batch_push_zero_rows(const ZeroRowsArgs& a, int gx);

// Host side: launch one instantiation with its dynamic LDS (stages x (BM + BN) rows of 128 bytes);
// kernels above the 64 KiB default get their limit raised once.
template <bool A_KC, bool B_KC, int BM, int BN, int NW, int MODE>
static int32_t launch_direct_kernel(const FastParams& F_in, int grid_x, hipStream_t stream) {
  FastParams F = F_in;
  if (F.splits < 1) F.splits = 1;
  auto kernel = gemm_direct_kernel<A_KC, B_KC, BM, BN, NW, MODE>;
  const size_t lds_bytes = (size_t)direct_stages(BM, BN) * (BM + BN) * LDS_ROW_U4 * sizeof(uint4);
  static thread_local bool raised = false;
  if (!raised && lds_bytes >= 65536) {
    ARD_HIP_CHECK(ard::raise_lds_limit((const void*)kernel, (int)lds_bytes));
    raised = !dry_run();
  }
  // class-free launches: the (split, tile) items are dealt to the XCDs inside the kernel
  if (F.tab.ncls == 0) grid_x = direct_plain_grid(F.total_tiles * (F.splits < 1 ? 1 : F.splits));
  // no lane may leave its operand: cheap envelope always, the exhaustive walk on request
  if (int32_t st = direct_envelope<A_KC, B_KC, BM, BN, MODE>(F)) return st;
  if (dry_run() || dev_knobs().prove_bounds) {
    DirectBounds b;
    if (int32_t st = direct_prove<A_KC, B_KC, BM, BN, NW, MODE>(F, grid_x, b)) return st;
    note_direct_bounds(b, F.a_elems * 2, F.b_elems * 2);
  }
  constexpr int gk = direct_group_kind<A_KC, B_KC, BM, BN, NW, MODE>();
  if (gk >= 0 && batch_open() && batch_push_direct(gk, F, grid_x, lds_bytes)) return ARD_OK;
  ARD_LAUNCH_NAMED("gemm_direct_kernel", kernel, dim3((unsigned)grid_x), dim3(64 * NW), lds_bytes, stream, F);
  ARD_LAUNCH_CHECK("gemm_direct_kernel");
  return ARD_OK;
}

// an XCD's share should be about square in tiles: bands of group_m tile rows
static inline int direct_group_m(int total_tiles) {
  const int per_xcd = ceil_div(total_tiles, 8);
  int gm = 1;
  while (gm * gm * 2 <= per_xcd && gm < 8) gm *= 2;
  return gm;
}

}  // namespace ard
