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
// One workgroup of 4 or 8 wavefronts computes a BM x BN tile with
// 32x32 MFMA tiles (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32),
// operands staged through double-buffered LDS in XOR-swizzled rows of 128 bytes.
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
  int kpad;    // storage along the contraction is zero padded up to the next multiple of 8
  int rpad;    // storage along the non-contracted axis is readable up to the next multiple of 8
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
  // contraction split over blockIdx.y: fp32 partial sums part[split][M][N] (compact, alpha not
  // applied) that a finishing pass reduces; NULL: the kernel stores the result itself
  float* part;
  int splits;
};

// Host: may this operand be fetched with 16-byte loads?  KC operands need contiguous,
// aligned runs along the contraction axis; MC operands along their row axis.
static inline bool operand_vec_ok(const Operand& op, bool kc, const Axis& k, int ce) {
  if (((uintptr_t)op.p & 15) != 0 || (op.ld % ce) != 0) return false;
  if (kc) return op.kdense ? true : axis_chunk_contiguous(k, ce);
  return axis_chunk_contiguous(op.r, ce);
}

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

// LDS operand tiles: rows of 128 bytes = 8 chunks of 16 bytes, no padding.  Chunk c of
// row r sits at slot c ^ (r & 7) ^ ((r >> 3) & 7): the 16-byte fragment reads of 8 (and 16)
// consecutive rows, the row-major chunk writes and the transposed 8-byte writes below all
// spread over every bank.
constexpr int LDS_ROW_U4 = 8;
__device__ __forceinline__ int swz(int row, int c) { return row * 8 + (c ^ (row & 7) ^ ((row >> 3) & 7)); }

__device__ __forceinline__ int ax_phys_k(const Axis& a, int j) {
  // contraction axis: BLOCK lists carry a bias in `off`
  if (a.kind == AX_AFFINE) return a.off + j * a.step;
  if (a.kind == AX_LIST) return a.list[j];
  int q = j / a.bs;
  if (a.kind == AX_BAFF) return (a.off + q * a.step) * a.bs + (j - q * a.bs);
  return (a.list[q] + a.off) * a.bs + (j - q * a.bs);
}

// Global -> register -> LDS staging of a ROWS x 128-byte operand tile by NT threads.
// KC: the stored matrix is contraction-contiguous (element (row, k) at p[row*ld + k]); each
// thread moves 16-byte chunks (one global_load_dwordx4 when the chunk is contiguous and
// aligned, element loads through the index map otherwise).
template <typename T, int ROWS, int NT>
struct LoaderKC {
  static constexpr int CE = ElemTraits<T>::CE;
  static constexpr int PASSES = ROWS * 8 / NT;
  static constexpr int NREG = PASSES;
  static_assert(PASSES >= 1, "tile too small for the workgroup");
  const T* base;
  int vec, lc, lr0;
  Axis kax;
  long roff[PASSES];
  bool rvalid[PASSES];

  __device__ __forceinline__ void init(const Operand& op, const Axis& k, int row0, int tid) {
    base = (const T*)op.p;
    vec = op.vec;
    kax = op.kdense ? axis_identity(k.n) : k;
    lc = tid & 7;
    lr0 = tid >> 3;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      int j = row0 + lr0 + (NT / 8) * p;
      rvalid[p] = j < op.r.n;
      int ph = rvalid[p] ? ax_phys(op.r, j) : 0;
      roff[p] = (long)ph * op.ld;
    }
  }

  __device__ __forceinline__ void load(int k0, uint4 (&regs)[NREG]) const {
    const int kc = k0 + lc * CE;
    const bool kin = kc < kax.n;
    int kp = 0;
    bool kvec = false;
    if (kin && vec && kc + CE <= kax.n) {
      kp = ax_phys_k(kax, kc);
      kvec = kp + CE <= kax.nphys;
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (rvalid[p] && kin) {
        if (kvec) {
          v = *reinterpret_cast<const uint4*>(base + roff[p] + kp);
        } else {
          T tmp[CE];
#pragma unroll
          for (int e = 0; e < CE; ++e) {
            int k = kc + e;
            T x = 0;
            if (k < kax.n) {
              int kq = ax_phys_k(kax, k);
              if (kq < kax.nphys) x = base[roff[p] + kq];
            }
            tmp[e] = x;
          }
          v = *reinterpret_cast<const uint4*>(tmp);
        }
      }
      regs[p] = v;
    }
  }

  __device__ __forceinline__ void store(uint4* tile, const uint4 (&regs)[NREG]) const {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) tile[swz(lr0 + (NT / 8) * p, lc)] = regs[p];
  }
};

// MC: the contraction index selects the stored row (element (row, k) at p[k*ld + row]).
// A thread fetches a unit of 4 contraction rows x one 16-byte run along the tile rows,
// transposes it in registers and writes, per tile row, the 4 contraction values (8 bytes
// for bf16, one full chunk for fp32).  Lanes of a wavefront cover 8 adjacent runs (one
// 128-byte line) x 8 contraction quads.
template <typename T, int ROWS, int NT>
struct LoaderMC {
  static constexpr int CE = ElemTraits<T>::CE;
  static constexpr int KU = 4;
  static constexpr int KQ = 8 * CE / KU;          // contraction quads per step
  static constexpr int NBT = ROWS / CE;           // 16-byte runs per tile
  static constexpr int UNITS = KQ * NBT;
  static constexpr int PASSES = (UNITS + NT - 1) / NT;
  static constexpr int NREG = PASSES * KU;
  static constexpr int NB_L = NBT < 8 ? NBT : 8;
  static constexpr int KQ_L = 64 / NB_L;
  static constexpr int NBG = NBT / NB_L;
  const T* base;
  long ld;
  int vec;
  Axis kax, rax;
  int nb[PASSES], kq[PASSES], jrow[PASSES];
  long roff[PASSES];
  bool uvalid[PASSES], rfull[PASSES];

  __device__ __forceinline__ void init(const Operand& op, const Axis& k, int row0, int tid) {
    base = (const T*)op.p;
    ld = op.ld;
    vec = op.vec;
    kax = op.kdense ? axis_identity(k.n) : k;
    rax = op.r;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int u = tid + NT * p;
      const int ul = u & 63, g = u >> 6;
      nb[p] = (g % NBG) * NB_L + (ul % NB_L);
      kq[p] = (g / NBG) * KQ_L + (ul / NB_L);
      uvalid[p] = u < UNITS;
      jrow[p] = row0 + nb[p] * CE;
      rfull[p] = jrow[p] + CE <= rax.n;
      roff[p] = (uvalid[p] && jrow[p] < rax.n) ? (long)ax_phys(rax, jrow[p]) : 0;
    }
  }

  __device__ __forceinline__ void load(int k0, uint4 (&regs)[NREG]) const {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
#pragma unroll
      for (int e = 0; e < KU; ++e) {
        uint4 v = make_uint4(0, 0, 0, 0);
        const int k = k0 + kq[p] * KU + e;
        if (uvalid[p] && k < kax.n && jrow[p] < rax.n) {
          const int kp = ax_phys_k(kax, k);
          if (kp < kax.nphys) {
            const T* rowp = base + (long)kp * ld;
            if (vec && rfull[p]) {
              v = *reinterpret_cast<const uint4*>(rowp + roff[p]);
            } else {
              T tmp[CE];
#pragma unroll
              for (int i = 0; i < CE; ++i) {
                int j = jrow[p] + i;
                tmp[i] = j < rax.n ? rowp[ax_phys(rax, j)] : (T)0;
              }
              v = *reinterpret_cast<const uint4*>(tmp);
            }
          }
        }
        regs[p * KU + e] = v;
      }
    }
  }

  __device__ __forceinline__ void store(uint4* tile, const uint4 (&regs)[NREG]) const {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      if (!uvalid[p]) continue;
      const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&regs[p * KU + 0]);
      const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&regs[p * KU + 1]);
      const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&regs[p * KU + 2]);
      const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&regs[p * KU + 3]);
      if (sizeof(T) == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int d = i >> 1;
          uint2 o;
          if (i & 1) {
            o.x = (w0[d] >> 16) | (w1[d] & 0xffff0000u);
            o.y = (w2[d] >> 16) | (w3[d] & 0xffff0000u);
          } else {
            o.x = (w0[d] & 0xffffu) | (w1[d] << 16);
            o.y = (w2[d] & 0xffffu) | (w3[d] << 16);
          }
          const int row = nb[p] * 8 + i;
          uint2* dst = reinterpret_cast<uint2*>(tile + swz(row, kq[p] >> 1)) + (kq[p] & 1);
          *dst = o;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = nb[p] * 4 + i;
          tile[swz(row, kq[p])] = make_uint4(w0[i], w1[i], w2[i], w3[i]);
        }
      }
    }
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
// operand tiles: load(k0, regs) fetches the 128-byte-per-row slab that starts at compact
// contraction index k0 into registers, store(tile, regs) writes it to LDS.  Two LDS
// buffers: the slab of step s+1 is fetched before and written after the MFMAs of step s,
// one barrier per step.
template <typename T, int BM, int BN, int WGM, int WGN, class LA, class LB>
__device__ __forceinline__ void gemm_mainloop(const LA& la, const LB& lb, int k_begin, int k_end, uint4* lds,
                                              f32x16_t (&acc)[BM / WGM / 32][BN / WGN / 32],
                                              const bool (&act)[BM / WGM / 32][BN / WGN / 32]) {
  constexpr int CE = ElemTraits<T>::CE;
  constexpr int BK = 8 * CE;  // contraction elements per step (128 bytes per row)
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * LDS_ROW_U4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  uint4 ra[LA::NREG], rb[LB::NREG];
  int aidx[TM], axr[TM], bidx[TN], bxr[TN];
#pragma unroll
  for (int im = 0; im < TM; ++im) {
    const int row = wm * WTM + im * 32 + (lane & 31);
    aidx[im] = row * 8;
    axr[im] = (row & 7) ^ ((row >> 3) & 7);
  }
#pragma unroll
  for (int in = 0; in < TN; ++in) {
    const int row = wn * WTN + in * 32 + (lane & 31);
    bidx[in] = BM * LDS_ROW_U4 + row * 8;
    bxr[in] = (row & 7) ^ ((row >> 3) & 7);
  }
  la.load(k_begin, ra);
  lb.load(k_begin, rb);
  la.store(lds, ra);
  lb.store(lds + BM * LDS_ROW_U4, rb);
  __syncthreads();
  int buf = 0;
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    const bool more = k0 + BK < k_end;
    if (more) {
      la.load(k0 + BK, ra);
      lb.load(k0 + BK, rb);
    }
    const uint4* cur = lds + buf * STAGE;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = 2 * q + (lane >> 5);
      uint4 a[TM], b[TN];
#pragma unroll
      for (int im = 0; im < TM; ++im) a[im] = cur[aidx[im] + (c ^ axr[im])];
#pragma unroll
      for (int in = 0; in < TN; ++in) b[in] = cur[bidx[in] + (c ^ bxr[in])];
#pragma unroll
      for (int im = 0; im < TM; ++im)
#pragma unroll
        for (int in = 0; in < TN; ++in)
          if (act[im][in]) Mma<T>::run(a[im], b[in], acc[im][in]);
    }
    if (more) {
      uint4* nxt = lds + (buf ^ 1) * STAGE;
      la.store(nxt, ra);
      lb.store(nxt + BM * LDS_ROW_U4, rb);
    }
    __syncthreads();
    buf ^= 1;
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

template <bool KC, typename T, int ROWS, int NT> struct PickLoader { typedef LoaderKC<T, ROWS, NT> type; };
template <typename T, int ROWS, int NT> struct PickLoader<false, T, ROWS, NT> { typedef LoaderMC<T, ROWS, NT> type; };

template <typename T, int BM, int BN, int WGM, int WGN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(const GemmParams P) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");

  extern __shared__ uint4 lds[];  // 2 * (BM + BN) * LDS_ROW_U4 entries, sized at launch

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
    typename PickLoader<A_KC, T, BM, NT>::type la;
    typename PickLoader<B_KC, T, BN, NT>::type lb;
    la.init(P.A, kax, m0, tid);
    lb.init(P.B, kax, n0, tid);
    int k_begin = 0, k_end = kax.n;
    if (P.part) {
      // whole 128-byte steps per split
      constexpr int BK = 8 * ElemTraits<T>::CE;
      const int steps = (kax.n + BK - 1) / BK;
      k_begin = (int)((long)blockIdx.y * steps / P.splits) * BK;
      k_end = min(kax.n, (int)((long)(blockIdx.y + 1) * steps / P.splits) * BK);
    }
    if (k_begin < k_end) gemm_mainloop<T, BM, BN, WGM, WGN>(la, lb, k_begin, k_end, lds, acc, act);
  }
  if (P.part) {
    float* part = P.part + (long)blockIdx.y * P.M * P.N;
    const int lane = tid & 63;
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
          if (i < P.M) part[(long)i * P.N + j] = acc[im][in][v];
        }
      }
    }
    return;
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
int32_t run_gemm(int32_t dtype, bool a_kc, bool b_kc, GemmParams P, int max_bn, int max_bm, hipStream_t stream,
                 void* ws = nullptr, size_t ws_bytes = 0);
bool run_gemm_partials(int32_t dtype, bool a_kc, bool b_kc, const GemmParams& P, hipStream_t stream, void* part,
                       size_t part_bytes, int* splits, int32_t* status);

}  // namespace ard
