// Gathered MFMA GEMM engine for gfx950.
//
//   C[cm(i), cn(j)] = alpha * sum_k A(am(i), ak(k)) * B(bn(j), ak(k))  (+ beta * C_old)
//
// i, j, k are COMPACT indices: only kept rows / columns / contraction indices
// exist in the iteration space, and every operand access goes through an index
// map (common.hpp) to the physical row or column.  Dropped rows, columns and
// tiles are therefore never loaded or multiplied (Sections 3.1, 3.2); the
// epilogue scatters results to their physical positions and writes zeros into
// the dropped positions it owns.
//
// One workgroup = 256 threads = 4 wavefronts computes a BM x BN tile with
// 32x32 MFMA tiles (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32),
// operands staged through LDS in rows of 128 bytes (+16 bytes of padding, which
// makes the 16-byte fragment reads bank-conflict free).
#pragma once
#include "common.hpp"

namespace ard {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

struct Operand {
  const void* p;
  long ld;   // elements between consecutive physical rows of the stored matrix
  Axis r;    // map of the non-contracted axis (M for A, N for B)
  int vec;   // 16-byte chunk loads are legal (contiguity and alignment checked on the host)
  int kdense;  // this operand is already compact along the contraction: it ignores the K map
};

struct OutMat {
  void* p;
  const void* relu_src;  // optional: zero the result where relu_src <= 0 (same layout/dtype as the output)
  long ld;
  Axis rm, cn;           // compact -> physical row / column of the output
  // optional batched-plane addressing (NCHW tensors): physical column c = (image, position)
  // with `plane` positions per image; element (r, c) lives at
  // (c / plane) * img_stride + r * plane + c % plane.  plane == 0: plain r * ld + c.
  int plane;
  long img_stride;
  int out_f32;           // output is fp32 regardless of the input dtype
  int fill;              // write zeros (or beta*old) into dropped rows/columns
  int relu;
  float alpha, beta;
};

struct GemmParams {
  Operand A, B;
  Axis k;
  // optional per-column-group contraction lists (tile pattern): group g = n0 / kb_ncols
  // contracts over blocks k.list[kb_ptr[g] .. kb_ptr[g+1]) + g * kb_bias
  const int* kb_ptr;
  int kb_ncols, kb_bias;
  // optional mask over tm_r x tm_c output tiles (tile pattern, weight gradient)
  const uint8_t* tmask;
  int tm_r, tm_c, tm_tc;
  OutMat C;
  int M, N;
  int tiles_m, tiles_n;
};

template <typename T> struct Mma;
template <> struct Mma<uint16_t> {
  __device__ static __forceinline__ void run(const uint4& a, const uint4& b, f32x16_t& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                0, 0, 0);
  }
};
template <> struct Mma<float> {
  __device__ static __forceinline__ void run(const uint4& a, const uint4& b, f32x16_t& c) {
    f32x4_t af = __builtin_bit_cast(f32x4_t, a), bf = __builtin_bit_cast(f32x4_t, b);
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[e], bf[e], c, 0, 0, 0);
  }
};

constexpr int LDS_ROW_U4 = 9;  // 128 data bytes + 16 pad bytes, in uint4 units

__device__ __forceinline__ int ax_phys_k(const Axis& a, int j) {
  // contraction axis: BLOCK lists carry a bias in `off`
  if (a.kind == AX_AFFINE) return a.off + j * a.step;
  if (a.kind == AX_LIST) return a.list[j];
  int q = j / a.bs;
  return (a.list[q] + a.off) * a.bs + (j - q * a.bs);
}

// Global -> register -> LDS staging of a ROWS x 128-byte operand tile.
// KC: the stored matrix is contraction-contiguous (element (row, k) at p[row*ld + k]).
// otherwise the contraction index selects the stored row (element at p[k*ld + row]).
template <typename T, int ROWS, bool KC>
struct TileLoader {
  static constexpr int CE = ElemTraits<T>::CE;
  static constexpr int PASSES = ROWS / 32;
  const T* base;
  long ld;
  int vec;
  Axis kax;
  long roff[PASSES];
  bool rvalid[PASSES];
  int lr[PASSES], lc[PASSES];

  __device__ __forceinline__ void init(const Operand& op, const Axis& k, int row0, int tid) {
    base = (const T*)op.p;
    ld = op.ld;
    vec = op.vec;
    kax = op.kdense ? axis_identity(k.n) : k;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      int r, c;
      if (KC) {
        c = tid & 7;
        r = (tid >> 3) + 32 * p;
      } else if (ROWS >= 64) {
        constexpr int RP = ROWS >= 64 ? ROWS / 64 : 1;
        r = (tid & 63) + 64 * (p % RP);
        c = (tid >> 6) + 4 * (p / RP);
      } else {
        r = tid & 31;
        c = tid >> 5;
      }
      lr[p] = r;
      lc[p] = c;
      int j = row0 + r;
      rvalid[p] = j < op.r.n;
      int ph = rvalid[p] ? ax_phys(op.r, j) : 0;
      roff[p] = KC ? (long)ph * ld : (long)ph;
    }
  }

  __device__ __forceinline__ void load(int k0, uint4 (&regs)[PASSES]) const {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int kc = k0 + lc[p] * CE;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (rvalid[p] && kc < kax.n) {
        bool done = false;
        if (KC && vec && kc + CE <= kax.n) {
          int kp = ax_phys_k(kax, kc);
          if (kp + CE <= kax.nphys) {
            v = *reinterpret_cast<const uint4*>(base + roff[p] + kp);
            done = true;
          }
        }
        if (!done) {
          T tmp[CE];
#pragma unroll
          for (int e = 0; e < CE; ++e) {
            int k = kc + e;
            T x = 0;
            if (k < kax.n) {
              int kp = ax_phys_k(kax, k);
              if (kp < kax.nphys) x = KC ? base[roff[p] + kp] : base[(long)kp * ld + roff[p]];
            }
            tmp[e] = x;
          }
          v = *reinterpret_cast<const uint4*>(tmp);
        }
      }
      regs[p] = v;
    }
  }

  __device__ __forceinline__ void store(uint4* tile, const uint4 (&regs)[PASSES]) const {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) tile[lr[p] * LDS_ROW_U4 + lc[p]] = regs[p];
  }
};

__device__ __forceinline__ void own_range(const Axis& a, int j, int fill, int& lo, int& hi, int& p) {
  p = ax_phys(a, j);
  if (!fill) {
    lo = p;
    hi = p + 1;
    return;
  }
  lo = (j == 0) ? 0 : p;
  hi = (j == a.n - 1) ? a.nphys : ax_phys(a, j + 1);
}

template <typename T>
__device__ __forceinline__ void store_out(const OutMat& C, long idx, float x, bool kept) {
  float v = kept ? x : 0.0f;
  if (C.beta != 0.0f) {
    float old = C.out_f32 ? ((const float*)C.p)[idx] : ElemTraits<T>::to_f32(((const T*)C.p)[idx]);
    v += C.beta * old;
  }
  if (C.relu) v = fmaxf(v, 0.0f);
  if (C.relu_src) {
    float g = ElemTraits<T>::to_f32(((const T*)C.relu_src)[idx]);
    v = g > 0.0f ? v : 0.0f;
  }
  if (C.out_f32)
    ((float*)C.p)[idx] = v;
  else
    ((T*)C.p)[idx] = ElemTraits<T>::from_f32(v);
}

// Contraction loop of one workgroup tile.  LA / LB stage the A (BM rows) and B (BN rows)
// operand tiles: load(k0, regs) fetches the 128-byte-per-row slab starting at compact
// contraction index k0 into registers, store(tile, regs) writes it to LDS.
template <typename T, int BM, int BN, int WGM, int WGN, class LA, class LB>
__device__ __forceinline__ void gemm_mainloop(const LA& la, const LB& lb, int k_begin, int k_end, uint4* lds,
                                              f32x16_t (&acc)[BM / WGM / 32][BN / WGN / 32],
                                              const bool (&act)[BM / WGM / 32][BN / WGN / 32]) {
  constexpr int CE = ElemTraits<T>::CE;
  constexpr int BK = 8 * CE;  // contraction elements per step (128 bytes per row)
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int PA = BM / 32, PB = BN / 32;
  uint4* As = lds;
  uint4* Bs = lds + BM * LDS_ROW_U4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  uint4 ra[PA], rb[PB];
  la.load(k_begin, ra);
  lb.load(k_begin, rb);
  const uint4* Arow = As + (wm * WTM + (lane & 31)) * LDS_ROW_U4 + (lane >> 5);
  const uint4* Brow = Bs + (wn * WTN + (lane & 31)) * LDS_ROW_U4 + (lane >> 5);
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    la.store(As, ra);
    lb.store(Bs, rb);
    __syncthreads();
    if (k0 + BK < k_end) {
      la.load(k0 + BK, ra);
      lb.load(k0 + BK, rb);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint4 a[TM], b[TN];
#pragma unroll
      for (int im = 0; im < TM; ++im) a[im] = Arow[im * 32 * LDS_ROW_U4 + 2 * q];
#pragma unroll
      for (int in = 0; in < TN; ++in) b[in] = Brow[in * 32 * LDS_ROW_U4 + 2 * q];
#pragma unroll
      for (int im = 0; im < TM; ++im)
#pragma unroll
        for (int in = 0; in < TN; ++in)
          if (act[im][in]) Mma<T>::run(a[im], b[in], acc[im][in]);
    }
    __syncthreads();
  }
}

// Scatter of the accumulators: lane holds column (lane & 31) of each 32x32 tile, rows
// 8*(v/4) + 4*(lane>>5) + v%4.  Each compact row / column also owns the dropped physical
// rows / columns that follow it (the first one also those before it) and writes their zeros.
template <typename T, int BM, int BN, int WGM, int WGN>
__device__ __forceinline__ void gemm_epilogue(const OutMat& C, const f32x16_t (&acc)[BM / WGM / 32][BN / WGN / 32],
                                              int m0, int n0, int M, int N) {
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
#pragma unroll
  for (int in = 0; in < TN; ++in) {
    const int j = n0 + wn * WTN + in * 32 + (lane & 31);
    if (j >= N) continue;
    int clo, chi, cp;
    own_range(C.cn, j, C.fill, clo, chi, cp);
#pragma unroll
    for (int im = 0; im < TM; ++im) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = m0 + wm * WTM + im * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (i >= M) continue;
        int rlo, rhi, rp;
        own_range(C.rm, i, C.fill, rlo, rhi, rp);
        const float x = C.alpha * acc[im][in][v];
        for (int c = clo; c < chi; ++c) {
          long cbase = c, rmul = C.ld;
          if (C.plane) {
            int img = c / C.plane;
            cbase = (long)img * C.img_stride + (c - img * C.plane);
            rmul = C.plane;
          }
          for (int r = rlo; r < rhi; ++r) store_out<T>(C, (long)r * rmul + cbase, x, r == rp && c == cp);
        }
      }
    }
  }
}

template <typename T, int BM, int BN, int WGM, int WGN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmParams P) {
  static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");

  __shared__ uint4 lds[(BM + BN) * LDS_ROW_U4];

  const int tid = threadIdx.x, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int mb = blockIdx.x / P.tiles_n, nb = blockIdx.x % P.tiles_n;
  const int m0 = mb * BM, n0 = nb * BN;

  Axis kax = P.k;
  if (P.kb_ptr) {
    const int g = n0 / P.kb_ncols;
    const int s = P.kb_ptr[g], e = P.kb_ptr[g + 1];
    kax.list = P.k.list + s;
    kax.n = (e - s) * kax.bs;
    kax.off = g * P.kb_bias;
  }

  // output-tile mask: which 32x32 MFMA tiles of this wave are kept, and whether
  // anything in the workgroup is
  bool act[TM][TN];
  bool any = true;
  if (P.tmask) {
    any = false;
    for (int i = 0; i < BM; i += 32)
      for (int j = 0; j < BN; j += 32) {
        int pi = m0 + i, pj = n0 + j;
        if (pi < P.M && pj < P.N && P.tmask[(pi / P.tm_r) * P.tm_tc + pj / P.tm_c]) any = true;
      }
#pragma unroll
    for (int im = 0; im < TM; ++im)
#pragma unroll
      for (int in = 0; in < TN; ++in) {
        int pi = m0 + wm * WTM + im * 32, pj = n0 + wn * WTN + in * 32;
        act[im][in] = pi < P.M && pj < P.N && P.tmask[(pi / P.tm_r) * P.tm_tc + pj / P.tm_c] != 0;
      }
  } else {
#pragma unroll
    for (int im = 0; im < TM; ++im)
#pragma unroll
      for (int in = 0; in < TN; ++in) act[im][in] = true;
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int im = 0; im < TM; ++im)
#pragma unroll
    for (int in = 0; in < TN; ++in)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[im][in][v] = 0.0f;

  if (any && kax.n > 0) {
    TileLoader<T, BM, A_KC> la;
    TileLoader<T, BN, B_KC> lb;
    la.init(P.A, kax, m0, tid);
    lb.init(P.B, kax, n0, tid);
    gemm_mainloop<T, BM, BN, WGM, WGN>(la, lb, 0, kax.n, lds, acc, act);
  }
  gemm_epilogue<T, BM, BN, WGM, WGN>(P.C, acc, m0, n0, P.M, P.N);
}

// Fill a dense matrix region with zeros (or scale by beta): used when a pattern keeps nothing.
template <typename T>
__global__ void scale_fill_kernel(T* p, long n, float beta) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = beta == 0.0f ? ElemTraits<T>::from_f32(0.0f) : ElemTraits<T>::from_f32(beta * ElemTraits<T>::to_f32(p[i]));
}

// Host-side dispatch: picks the workgroup tile for the problem and launches.
// max_bn: the widest column tile the contraction lists allow (tile pattern), or 0.
int32_t run_gemm(int32_t dtype, bool a_kc, bool b_kc, GemmParams P, int max_bn, int max_bm, hipStream_t stream);

}  // namespace ard
