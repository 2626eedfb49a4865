// Large-tile bf16 path of the gathered GEMM: 256 x 256 x 64 workgroup tiles, 8 wavefronts
// (2 x 4, each 128 x 64 = 4 x 2 MFMA 32x32x16 tiles), two wavefronts per SIMD so one
// wavefront's LDS/global waits hide behind the other's MFMAs, double-buffered swizzled LDS
// (128 KiB of the 160 KiB per CU), XCD-aware tile order.
//
// Tile patterns (Section 3.2) are period patterns over the linear tile index, so the tile
// rows (or columns) fall into a few CLASSES that share one kept-column (kept-row) set:
// class members, and the kept set of a class, are both arithmetic progressions.  A
// workgroup takes 256/tile consecutive members of ONE class as its rows or columns and
// walks that class's kept set along the contraction, so dropped tiles cost nothing and
// the macro tile stays 256 wide.  ClassTab carries the progressions.
//
// Restrictions checked on the host (anything else goes through gemm_kernel):
//   bf16 operands fetched with 16-byte loads only; contraction map identity or block
//   progression with block size a multiple of 64; every extent along a 16-byte run is a
//   multiple of 8.
#pragma once
#include <type_traits>

#include "engine.hpp"

namespace ard {

constexpr int F_MAXCLS = 16;

struct ClassTab {
  int ncls;                       // 0: plain tiles_m x tiles_n grid over P.am / P.bn / P.k
  int prefix[F_MAXCLS + 1];       // workgroups before class c
  int mblk[F_MAXCLS];             // workgroup rows of class c
  // row side (M): block progression off + i*step, `cnt` blocks of size bs (bs == 0: identity rows)
  int m_off[F_MAXCLS], m_cnt[F_MAXCLS], m_step, m_bs, m_phys;
  // column side (N)
  int n_off[F_MAXCLS], n_cnt[F_MAXCLS], n_step, n_bs, n_phys;
  // contraction side (K) (bs == 0: identity contraction P.k)
  int k_off[F_MAXCLS], k_cnt[F_MAXCLS], k_step, k_bs, k_phys;
};

struct FastParams {
  const uint16_t* A;
  const uint16_t* B;
  uint16_t* C;
  int lda, ldb, ldc;
  Axis am, bn, k;  // plain mode: compact -> physical rows of A (M), rows of B (N), contraction
  ClassTab tab;
  int c_rows_mapped, c_cols_mapped;  // output rows / columns go through the M / N map (else identity)
  float alpha;
  int relu;
  int M, N, tiles_m, tiles_n, group_m, tiles_per_xcd, total_tiles;
};

constexpr int F_BM = 256, F_BN = 256, F_NT = 512;

typedef short v4i16_t __attribute__((ext_vector_type(4)));
#define ARD_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))
#define ARD_GLB_PTR(p) ((const void __attribute__((address_space(1)))*)(p))

// 64 zero bytes: source of the chunks that lie beyond the end of the contraction
__device__ uint4 g_zero_chunk[4];

// physical start of the 64-wide contraction slab that begins at compact index ks (uniform)
__device__ __forceinline__ int fast_kslab(const Axis& k, int ks) {
  if (k.kind == AX_AFFINE) return k.off + ks;
  const int q = ks / k.bs;
  if (k.kind == AX_BAFF) return (k.off + q * k.step) * k.bs + (ks - q * k.bs);
  return (k.list[q] + k.off) * k.bs + (ks - q * k.bs);
}

// Operand staging with LDS-direct loads (global_load_lds_dwordx4): a wavefront instruction
// moves 64 x 16 bytes from per-lane global addresses into 1 KiB of consecutive LDS, with no
// register in between, so a whole 64 KiB stage stays in flight behind the MFMAs.  The LDS
// layout is therefore fixed by lane order, and each lane picks WHICH chunk it fetches so
// that the layout comes out swizzled:
//   KC operand (contraction-contiguous): LDS tile [256 rows][8 chunks]; an instruction fills
//     8 rows; lane = (row, slot) fetches logical chunk slot ^ xr(row).  Fragments: ds_read_b128.
//   MC operand (contraction-strided): LDS tile [64 k][32 chunks of 8 rows] exactly as in
//     memory; an instruction fills 2 k-rows; lane = (k, pos) fetches chunk pos ^ 4*(k & 3).
//     Fragments: two ds_read_b64_tr_b16 (transposing reads) per MFMA operand.
template <bool KC> struct DirectLoader;

template <> struct DirectLoader<true> {
  const uint16_t* base;
  int goff[4];   // element offset of this lane's chunk for instruction j, without the slab start
  int kc;        // first contraction element of the chunk inside the slab
  __device__ __forceinline__ void init(const uint16_t* p, int ld, const Axis& r, int row0, int lane, int wave) {
    base = p;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = (wave * 4 + j) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ (row & 7) ^ ((row >> 3) & 7);
      int ph = row0 + row < r.n ? ax_phys(r, row0 + row) : 0;
      ph = ph < r.nphys ? ph : 0;  // rows outside the matrix: fetch row 0, the result is never stored
      goff[j] = ph * ld + c * 8;
      if (j == 0) kc = c * 8;      // (row & 7) and ((row >> 3) & 7) differ per j: kc is per j below
    }
  }
  // chunk index of instruction j (recomputed: cheaper than four more registers)
  __device__ __forceinline__ int chunk_k(int lane, int wave, int j) const {
    const int row = (wave * 4 + j) * 8 + (lane >> 3);
    return ((lane & 7) ^ (row & 7) ^ ((row >> 3) & 7)) * 8;
  }
  __device__ __forceinline__ void issue(uint4* op_tile, int kslab, int krem, int kphys_end, bool tail, int lane,
                                        int wave) const {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint16_t* src = base + (long)goff[j] + kslab;
      if (tail) {
        const int k = chunk_k(lane, wave, j);
        if (!(k < krem && kslab + k + 8 <= kphys_end)) src = reinterpret_cast<const uint16_t*>(g_zero_chunk);
      }
      __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(src), ARD_LDS_PTR(op_tile + (wave * 4 + j) * 64), 16, 0, 0);
    }
  }
};

template <> struct DirectLoader<false> {
  const uint16_t* base;
  int ld;
  int coff[2];  // physical column of this lane's chunk for even / odd instructions
  __device__ __forceinline__ void init(const uint16_t* p, int ld_, const Axis& r, int row0, int lane, int wave) {
    base = p;
    ld = ld_;
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int kloc = 2 * par + (lane >> 5);               // k & 3 of the row this lane fills
      const int c = (lane & 31) ^ (4 * (kloc & 3));
      const int j = row0 + c * 8;
      int ph = j + 8 <= r.n ? ax_phys(r, j) : 0;
      coff[par] = ph + 8 <= r.nphys ? ph : 0;
    }
  }
  __device__ __forceinline__ void issue(uint4* op_tile, int kslab, int krem, int kphys_end, bool tail, int lane,
                                        int wave) const {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kloc = 2 * (wave * 4 + j) + (lane >> 5);
      const uint16_t* src = base + (long)(kslab + kloc) * ld + coff[j & 1];
      if (tail && !(kloc < krem && kslab + kloc < kphys_end)) src = reinterpret_cast<const uint16_t*>(g_zero_chunk);
      __builtin_amdgcn_global_load_lds(ARD_GLB_PTR(src), ARD_LDS_PTR(op_tile + (wave * 4 + j) * 64), 16, 0, 0);
    }
  }
};

// Fragment addressing.  KC: u4 index of (row, chunk 2q+g).  MC: byte address of the lane's
// source position for the transposing read of MFMA tile `t` (k offset q*16 + h*4 added as
// an immediate by the caller).
__device__ __forceinline__ int mc_frag_base(int tile_col0, int lane) {
  const int s = lane & 15, G = lane >> 4;
  const int g = G >> 1, jhalf = G & 1;
  const int c = (tile_col0 >> 3) + 2 * jhalf + ((s & 3) >> 1);
  const int pc = c ^ (4 * ((s >> 2) & 3));
  return (g * 8 + (s >> 2)) * 512 + pc * 16 + 8 * (s & 1);
}

__device__ __forceinline__ uint4 mc_frag_read(const char* op_bytes, int base, int q) {
  typedef v4i16_t __attribute__((address_space(3))) * lds_v4;
  const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(op_bytes + base + q * 8192));
  const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(op_bytes + base + q * 8192 + 2048));
  uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
  return make_uint4(l.x, l.y, h.x, h.y);
}

// LDS fragment reads are issued as volatile asm: the compiler then cannot move a read next to
// its consumer, and the single wait below (tied to the fragment registers) is the only place
// where a slice's MFMAs meet their operands.  One slice ahead is always in flight.
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

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(F_NT) void gemm256_kernel(const FastParams P) {
  constexpr int TM = 4, TN = 2, WTM = 128, WTN = 64;
  constexpr int STAGE = (F_BM + F_BN) * LDS_ROW_U4;  // 64 KiB
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  // XCD-aware order: workgroup ids go round-robin over the 8 XCDs, so XCD x = id % 8 gets the
  // contiguous range [x * tiles_per_xcd, ...) of the logical order.
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int L = xcd * P.tiles_per_xcd + local;
  if (local >= P.tiles_per_xcd || L >= P.total_tiles) return;

  Axis am = P.am, bn = P.bn, kax = P.k;
  int m0 = 0, n0 = 0;
  if (P.tab.ncls == 0) {
    // bands of group_m tile rows, walked column by column: an XCD's share is a compact rectangle
    const int band_sz = P.group_m * P.tiles_n;
    const int band = L / band_sz, inb = L - band * band_sz;
    const int rows_in_band = min(P.group_m, P.tiles_m - band * P.group_m);
    m0 = (band * P.group_m + inb % rows_in_band) * F_BM;
    n0 = (inb / rows_in_band) * F_BN;
  } else {
    const ClassTab& t = P.tab;
    int c = 0;
    while (c + 1 < t.ncls && L >= t.prefix[c + 1]) ++c;
    const int l = L - t.prefix[c];
    const int mi = l % t.mblk[c], ni = l / t.mblk[c];
    if (t.m_bs) {
      const int g = F_BM / t.m_bs;
      const int left = t.m_cnt[c] - mi * g;
      am = axis_baff(t.m_off[c] + mi * g * t.m_step, t.m_step, t.m_bs, left < g ? left : g, t.m_phys);
    } else {
      m0 = mi * F_BM;
    }
    {
      const int g = F_BN / t.n_bs;
      const int left = t.n_cnt[c] - ni * g;
      bn = axis_baff(t.n_off[c] + ni * g * t.n_step, t.n_step, t.n_bs, left < g ? left : g, t.n_phys);
    }
    if (t.k_bs) kax = axis_baff(t.k_off[c], t.k_step, t.k_bs, t.k_cnt[c], t.k_phys);
  }
  const int Kn = kax.n;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int im = 0; im < TM; ++im)
#pragma unroll
    for (int in = 0; in < TN; ++in)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[im][in][v] = 0.0f;

  if (Kn > 0) {
    DirectLoader<A_KC> la;
    DirectLoader<B_KC> lb;
    la.init(P.A, P.lda, am, m0, lane, wave);
    lb.init(P.B, P.ldb, bn, n0, lane, wave);
    // LDS: [A stage 0 | A stage 1 | B stage 0 | B stage 1], 32 KiB each, so the stage is an
    // immediate offset of the fragment reads and every read address is a loop invariant.
    constexpr int OPT = F_BM * LDS_ROW_U4;  // u4 entries of one operand tile
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
        aaddr[im][0] = lds_base + (unsigned)mc_frag_base(wm * WTM + im * 32, lane);
      }
    }
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      if (B_KC) {
        const int row = wn * WTN + in * 32 + (lane & 31);
        const int xr = (row & 7) ^ ((row >> 3) & 7);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          baddr[in][q] = lds_base + (unsigned)(2 * OPT + row * 8 + ((2 * q + (lane >> 5)) ^ xr)) * 16u;
      } else {
        baddr[in][0] = lds_base + (unsigned)(2 * OPT) * 16u + (unsigned)mc_frag_base(wn * WTN + in * 32, lane);
      }
    }
    const int S = (Kn + 63) >> 6;
    auto load_stage = [&](int it, int buf) {
      const int krem = Kn - it * 64;
      const int ks = fast_kslab(kax, it * 64);
      const bool tail = krem < 64 || ks + 64 > kax.nphys;
      la.issue(lds + buf * OPT, ks, krem, kax.nphys, tail, lane, wave);
      lb.issue(lds + (2 + buf) * OPT, ks, krem, kax.nphys, tail, lane, wave);
    };
    // One contraction step from stage BUF (compile-time, so its offset is an immediate).
    // LDS fragment reads are volatile asm with one explicit wait per 16-wide slice: a slice's
    // reads are issued while the previous slice's MFMAs run and meet their consumers only at
    // that wait.
    auto step = [&](auto bufc) {
      constexpr int BUF = decltype(bufc)::value;
      constexpr int SOFF = BUF * OPT * 16;  // byte offset of the stage inside its operand pair
      Frag fa[2][TM], fb[2][TN];
      auto issue = [&](auto qc, int set) {
        constexpr int Q = decltype(qc)::value;
#pragma unroll
        for (int im = 0; im < TM; ++im) {
          if (A_KC) {
            lds_read_b128<SOFF>(fa[set][im].v, aaddr[im][A_KC ? Q : 0]);
          } else {
            lds_read_tr16_b64<SOFF + Q * 8192>(fa[set][im].lo, aaddr[im][0]);
            lds_read_tr16_b64<SOFF + Q * 8192 + 2048>(fa[set][im].hi, aaddr[im][0]);
          }
        }
#pragma unroll
        for (int in = 0; in < TN; ++in) {
          if (B_KC) {
            lds_read_b128<SOFF>(fb[set][in].v, baddr[in][B_KC ? Q : 0]);
          } else {
            lds_read_tr16_b64<SOFF + Q * 8192>(fb[set][in].lo, baddr[in][0]);
            lds_read_tr16_b64<SOFF + Q * 8192 + 2048>(fb[set][in].hi, baddr[in][0]);
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
      issue(std::integral_constant<int, 0>{}, 0);
      wait(0);
      issue(std::integral_constant<int, 1>{}, 1);
      mma(0);
      wait(1);
      issue(std::integral_constant<int, 2>{}, 0);
      mma(1);
      wait(0);
      issue(std::integral_constant<int, 3>{}, 1);
      mma(0);
      wait(1);
      mma(1);
    };
    load_stage(0, 0);
    for (int it = 0; it < S; it += 2) {
      // stage `it` has landed once every wavefront's loads are done; the barrier also tells us
      // that everybody finished reading the other buffer, which the next loads overwrite
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (it + 1 < S) load_stage(it + 1, 1);
      step(std::integral_constant<int, 0>{});
      if (it + 1 < S) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (it + 2 < S) load_stage(it + 2, 0);
        step(std::integral_constant<int, 1>{});
      }
    }
  }

  // epilogue: lane holds column (lane & 31) of each 32x32 tile, rows 8*(v/4) + 4*(lane>>5) + v%4.
  // Mapped rows / columns come in blocks that are multiples of 32, so one index lookup per
  // 32x32 tile places all of its rows (columns).
  const int nlim = P.c_cols_mapped ? bn.n : P.N, mlim = P.c_rows_mapped ? am.n : P.M;
  const int nphys = P.c_cols_mapped ? bn.nphys : P.N, mphys = P.c_rows_mapped ? am.nphys : P.M;
  int prow[TM];
#pragma unroll
  for (int im = 0; im < TM; ++im) {
    const int i0 = m0 + wm * WTM + im * 32;
    prow[im] = i0 < mlim ? (P.c_rows_mapped ? ax_phys(am, i0) : i0) : mphys;
  }
#pragma unroll
  for (int in = 0; in < TN; ++in) {
    const int j0 = n0 + wn * WTN + in * 32;
    if (j0 >= nlim) continue;
    const int pc = (P.c_cols_mapped ? ax_phys(bn, j0) : j0) + (lane & 31);
    if (pc >= nphys) continue;
#pragma unroll
    for (int im = 0; im < TM; ++im) {
      uint16_t* dst = P.C + (long)(prow[im] + 4 * (lane >> 5)) * P.ldc + pc;
      const int rbase = prow[im] + 4 * (lane >> 5);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int dr = 8 * (v >> 2) + (v & 3);
        if (rbase + dr >= mphys) continue;
        float x = P.alpha * acc[im][in][v];
        if (P.relu) x = fmaxf(x, 0.0f);
        dst[(long)dr * P.ldc] = f32_to_bf16_bits(x);
      }
    }
  }
}

// Zero the dropped tiles of a tile-masked matrix (weight gradient): one workgroup per tile.
__global__ __launch_bounds__(256) void zero_dropped_tiles_kernel(uint16_t* C, int ld, int rows, int cols, int tr, int tc,
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

}  // namespace ard
