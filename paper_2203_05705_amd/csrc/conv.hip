// Convolution with dropped input feature maps (Sections 5, 6), channel-level reading:
// one sensitivity score per input feature map, the lowest-scoring maps are dropped and
// their activations, weights and gradients are never loaded.
//
// All three passes are implicit GEMMs on the matrix cores:
//   FWD        Y[co, (n,oh,ow)]  = sum_{tap, c kept}  Wp[co, (tap,c)]  * A[n, c, oh*s+kh-p, ow*s+kw-p]
//   BWD_DATA   dA[c kept, (n,y,x)] = sum_{tap, co}    Wq[c, (tap,co)]  * dY[n, co, y-kh+p, x-kw+p]
//   BWD_WEIGHT dW[co, (c kept,tap)] = sum_{(n,oh,ow)} dY[n, co, oh, ow] * A[n, c, oh*s+kh-p, ow*s+kw-p]
// Wp / Wq are compact repacked copies of the kept-channel weights (tiny, built per call).
//
// Two paths.  bf16 with stride 1: the kept maps are copied once into a zero-bordered
// channels-last grid and the products run on the LDS-direct kernel of fast.hpp (second half of
// this file).  Everything else (fp32, strides): the general engine with loaders that compute
// the patch addresses on the fly, im2col never materialised (first half).
#include <stdlib.h>

#include "engine.hpp"
#include "fast.hpp"
#include "pattern.hpp"

namespace ard {

// ---- sensitivity score and selection -------------------------------------------------------

// part[y * C + c] = sum over workgroup (c, y)'s share of (n, h, w) of floor(min(|a|, 2^15) * 2^24): exact
// integers, so the result does not depend on the order of summation.  Every workgroup writes its own
// partial (no atomics, nothing to clear beforehand); the selection kernel adds the few partials of a map.
constexpr int kScoreParts = 64;  // at most this many workgroups share a feature map
constexpr int kScorePlanes = 4;  // planes a wavefront reads at a time (x 2 pieces per lane = 8 loads in flight)
template <typename T>
__global__ __launch_bounds__(256) void channel_score_kernel(const T* A, int N, int C, int HW, int n_per_block, int vec,
                                                           unsigned long long* part) {
  constexpr int CE = ElemTraits<T>::CE;
  __shared__ unsigned long long wave_acc[4];
  const int c = blockIdx.x;
  const int n_begin = blockIdx.y * n_per_block;
  const int n_end = min(N, n_begin + n_per_block);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // floor(x * 2^24) for x in [0, 2^15] needs 40 bits; a float-to-64-bit conversion per element made this
  // pass ALU-bound.  Split exactly instead: hi = trunc(x * 2^8) < 2^24, lo = trunc(x * 2^24 - hi * 2^16)
  // < 2^16 (both products and the difference are exact in fp32), floor(x * 2^24) = hi * 2^16 + lo.
  // hi and lo are summed in 32 bits and folded into the 64-bit sum every `flush` (at most 128 elements).
  unsigned long long acc = 0;
  uint32_t acc_hi = 0, acc_lo = 0;
  auto add = [&](T v) {
    const float x = fminf(fabsf(ElemTraits<T>::to_f32(v)), 32768.0f);
    const uint32_t hi = (uint32_t)(x * 256.0f);
    const float lo_f = fmaf(-65536.0f, (float)hi, x * 16777216.0f);
    acc_hi += hi;
    acc_lo += (uint32_t)lo_f;
  };
  auto flush = [&]() {
    acc += ((unsigned long long)acc_hi << 16) + acc_lo;
    acc_hi = acc_lo = 0;
  };
  if (vec) {
    // planes are whole numbers of 16-byte pieces.  A wavefront takes kScorePlanes planes at a time and its
    // lanes two pieces of each: 8 loads, all unconditional (clamped index, contribution zeroed afterwards)
    // so that they are in flight together -- a load behind a branch is waited for before the next is issued.
    const int chunks = HW / CE;
    const int planes = n_end - n_begin;
    const T* const a0 = A + ((long)n_begin * C + c) * HW;
    for (int pb = wave * kScorePlanes; pb < planes; pb += 4 * kScorePlanes)
      for (int cb = lane; cb < chunks; cb += 128) {
        uint4 q[kScorePlanes][2];
#pragma unroll
        for (int u = 0; u < kScorePlanes; ++u) {
          const uint4* pl = reinterpret_cast<const uint4*>(a0 + (long)min(pb + u, planes - 1) * C * HW);
#pragma unroll
          for (int v = 0; v < 2; ++v) q[u][v] = pl[min(cb + 64 * v, chunks - 1)];
        }
#pragma unroll
        for (int u = 0; u < kScorePlanes; ++u)
#pragma unroll
          for (int v = 0; v < 2; ++v) {
            const bool live = pb + u < planes && cb + 64 * v < chunks;
            const uint4 z = live ? q[u][v] : uint4{0u, 0u, 0u, 0u};
            const T* e = reinterpret_cast<const T*>(&z);
#pragma unroll
            for (int t = 0; t < CE; ++t) add(e[t]);   // (a zero piece adds nothing)
          }
        flush();
      }
  } else {
    for (int n = n_begin; n < n_end; ++n) {
      const T* p = A + ((long)n * C + c) * HW;
      for (int i = threadIdx.x; i < HW; i += 256) {
        add(p[i]);
        flush();
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
  if (lane == 0) wave_acc[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) part[(long)blockIdx.y * C + c] = wave_acc[0] + wave_acc[1] + wave_acc[2] + wave_acc[3];
}

// Adds the `parts` partial scores of every map (score_out gets the totals), then drops the n_drop maps that
// come first in ascending (score, index) order; writes the mask (1 = kept) and the ascending kept list
// (ballot + mbcnt compaction, one workgroup).  The rank of a map is counted by four threads, a quarter
// of the other maps each.  IN_LDS: the scores fit the staging array (else they are re-read from memory).
// The code is kept short on purpose: a single workgroup that runs once pays every instruction-cache line it
// touches with a fetch from memory (3 KB of straight-line code took 10 us for 256 maps).
template <bool IN_LDS>
__global__ __launch_bounds__(1024) void channel_select_kernel(const unsigned long long* part, int parts,
                                                             unsigned long long* score_out, int C, int n_drop, uint8_t* mask,
                                                             int* keep, int* count) {
  constexpr int STAGED = 4096;
  __shared__ unsigned long long staged[IN_LDS ? STAGED : 1];
  __shared__ int wave_tot[16];
  __shared__ int running_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) running_s = 0;
  for (int i = tid; i < C; i += 1024) {
    unsigned long long t = 0;
#pragma unroll 1
    for (int y0 = 0; y0 < parts; y0 += 8) {
      unsigned long long v[8];  // eight unconditional loads in flight (clamped index, contribution zeroed)
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = part[(long)min(y0 + u, parts - 1) * C + i];
#pragma unroll
      for (int u = 0; u < 8; ++u) t += y0 + u < parts ? v[u] : 0ull;
    }
    score_out[i] = t;
    if (IN_LDS) staged[i] = t;
  }
  if (!IN_LDS) __threadfence_block();
  __syncthreads();
  for (int base = 0; base < C; base += 256) {
    const int c = base + (tid >> 2), part_id = tid & 3;
    int rank = 0;
    if (c < C) {
      const int o_lo = (int)((long)C * part_id / 4), o_hi = (int)((long)C * (part_id + 1) / 4);
      const unsigned long long s = IN_LDS ? staged[c] : score_out[c];
#pragma unroll 4
      for (int o = o_lo; o < o_hi; ++o) {
        const unsigned long long so = IN_LDS ? staged[o] : score_out[o];
        rank += (so < s || (so == s && o < c)) ? 1 : 0;
      }
    }
    rank += __shfl_xor(rank, 1, 64);
    rank += __shfl_xor(rank, 2, 64);
    const bool kept = c < C && part_id == 0 && rank >= n_drop;
    if (c < C && part_id == 0) mask[c] = kept ? 1 : 0;
    const unsigned long long bal = __ballot(kept);
    const int r = __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int before = running_s, total = 0;
#pragma unroll 1
    for (int w = 0; w < 16; ++w) {
      int t = wave_tot[w];
      if (w < wave) before += t;
      total += t;
    }
    if (kept) keep[before + r] = c;
    __syncthreads();
    if (tid == 0) running_s += total;
    __syncthreads();
  }
  if (tid == 0 && count) *count = running_s;
}

// ---- weight repacking ------------------------------------------------------------------------

// flip == 0: out[r = co][tap][q = kept c] = Wt[co][keep[q]][tap]            (rows = Cout, inner = Ck)
// flip == 1: out[r = kept c][tap][q = co] = Wt[co][keep[r]][taps-1-tap]    (rows = Ck, inner = Cout)
template <typename T>
__global__ void pack_weights_kernel(const T* Wt, const int* keep, int C, int taps, int rows, int inner, int flip,
                                    T* out) {
  const long total = (long)rows * taps * inner;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int q = (int)(idx % inner);
  const int tap = (int)((idx / inner) % taps);
  const int r = (int)(idx / ((long)inner * taps));
  long src = flip ? ((long)q * C + (keep ? keep[r] : r)) * taps + (taps - 1 - tap) : ((long)r * C + (keep ? keep[q] : q)) * taps + tap;
  out[idx] = Wt[src];
}

// ---- implicit-GEMM operand loaders ---------------------------------------------------------------

struct ConvGeom {
  int N, Cin, Hin, Win;      // tensor the patches are cut from
  int Hout, Wout;            // position grid (one GEMM column per (n, oh, ow))
  int KH, KW, stride, pad_h, pad_w;
  int Ck;                    // gathered channels per tap
  const int* chan;           // channel list (NULL = identity)
  // block-based sensitivity-aware pattern (Section 5.2.2): entry (p, q) of an image's input matrix,
  // q = (channel * KH + kh) * KW + kw, is absent when blk[(n * RB + p / bx) * CB + q / by] == 0
  const uint8_t* blk;
  int bx, by, RB, CB;
};

// B operand of FWD / BWD_DATA: row = position (n, oh, ow), contraction index k = tap*Ck + cc.
template <typename T, int ROWS>
struct PatchLoader {
  static constexpr int CE = ElemTraits<T>::CE;
  static constexpr int PASSES = ROWS / 32;
  static constexpr int NREG = PASSES;
  const T* src;
  ConvGeom g;
  int K;
  long ibase[PASSES];
  int bband[PASSES];  // (n * RB + row band) * CB of this thread's position (block pattern only)
  int ih0[PASSES], iw0[PASSES];
  bool rvalid[PASSES];
  int lr[PASSES], lc[PASSES];

  __device__ __forceinline__ void init(const void* p, const ConvGeom& geom, int row0, int tid) {
    src = (const T*)p;
    g = geom;
    K = g.KH * g.KW * g.Ck;
    const int hw = g.Hout * g.Wout;
    const long ntot = (long)g.N * hw;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      int r, c;
      if (ROWS >= 64) {
        constexpr int RP = ROWS >= 64 ? ROWS / 64 : 1;
        r = (tid & 63) + 64 * (ps % RP);
        c = (tid >> 6) + 4 * (ps / RP);
      } else {
        r = tid & 31;
        c = tid >> 5;
      }
      lr[ps] = r;
      lc[ps] = c;
      const long j = (long)row0 + r;
      rvalid[ps] = j < ntot;
      const int n = rvalid[ps] ? (int)(j / hw) : 0;
      const int rem = rvalid[ps] ? (int)(j - (long)n * hw) : 0;
      const int oh = rem / g.Wout, ow = rem - oh * g.Wout;
      ibase[ps] = (long)n * g.Cin * g.Hin * g.Win;
      ih0[ps] = oh * g.stride - g.pad_h;
      iw0[ps] = ow * g.stride - g.pad_w;
      bband[ps] = g.blk ? (n * g.RB + rem / g.bx) * g.CB : 0;
    }
  }

  __device__ __forceinline__ void load(int k0, uint4 (&regs)[PASSES]) const {
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      const int kc = k0 + lc[ps] * CE;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (rvalid[ps] && kc < K) {
        T tmp[CE];
        int tap = kc / g.Ck, cc = kc - tap * g.Ck;
#pragma unroll
        for (int e = 0; e < CE; ++e) {
          while (cc >= g.Ck) {
            cc -= g.Ck;
            ++tap;
          }
          T x = 0;
          if (kc + e < K) {
            const int kh = tap / g.KW, kw = tap - kh * g.KW;
            const int ih = ih0[ps] + kh, iw = iw0[ps] + kw;
            if (ih >= 0 && ih < g.Hin && iw >= 0 && iw < g.Win) {
              const int ch = g.chan ? g.chan[cc] : cc;
              if (!g.blk || g.blk[bband[ps] + (ch * g.KH * g.KW + tap) / g.by])
                x = src[ibase[ps] + ((long)ch * g.Hin + ih) * g.Win + iw];
            }
          }
          tmp[e] = x;
          ++cc;
        }
        v = *reinterpret_cast<const uint4*>(tmp);
      }
      regs[ps] = v;
    }
  }

  __device__ __forceinline__ void store(uint4* tile, const uint4 (&regs)[PASSES]) const {
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) tile[swz(lr[ps], lc[ps])] = regs[ps];
  }
};

struct ConvGemmParams {
  Operand Wp;       // packed weights [M x K], contraction-contiguous
  const void* src;  // activations (FWD) or output gradient (BWD_DATA)
  ConvGeom g;
  OutMat C;
  int M, K;
  long Ncols;
  int tiles_n;
};

template <typename T, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void conv_gemm_kernel(const ConvGemmParams P) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  __shared__ uint4 lds[2 * (BM + BN) * LDS_ROW_U4];
  const int tid = threadIdx.x;
  const int mb = blockIdx.x / P.tiles_n, nb = blockIdx.x % P.tiles_n;
  const int m0 = mb * BM, n0 = nb * BN;
  bool act[TM][TN];
  f32x16_t acc[TM][TN];
#pragma unroll
  for (int im = 0; im < TM; ++im)
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      act[im][in] = true;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[im][in][v] = 0.0f;
    }
  if (P.K > 0) {
    LoaderKC<T, BM, 256> la;
    PatchLoader<T, BN> lb;
    la.init(P.Wp, axis_identity(P.K), m0, tid);
    lb.init(P.src, P.g, n0, tid);
    gemm_mainloop<T, BM, BN, WGM, WGN>(la, lb, 0, P.K, lds, acc, act);
  }
  gemm_epilogue<T, BM, BN, WGM, WGN>(P.C, acc, m0, n0, P.M, (int)P.Ncols);
}

// Data gradient under the block pattern (Section 5.2.2).  An entry (p, q) of a dropped block of the input
// matrix receives no gradient, so the term of (input channel c, output position p, filter tap) counts or
// not as a whole: whether it does depends on the output row (c), the output column (the input pixel, which
// with the tap fixes p) and the tap, on no operand alone.  The contraction therefore runs tap by tap into
// a second accumulator that is added where the mask keeps the entry.  P.g is the geometry of the ordinary
// data gradient (positions = input pixels, source = dY, taps flipped, stride 1) and carries the mask with
// RB, CB of the forward input matrices; Cin_fwd = P.M channels, all kept.
template <typename T, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void conv_bwd_data_blocks_kernel(const ConvGemmParams P) {
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  __shared__ uint4 lds[2 * (BM + BN) * LDS_ROW_U4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int mb = blockIdx.x / P.tiles_n, nb = blockIdx.x % P.tiles_n;
  const int m0 = mb * BM, n0 = nb * BN;
  const ConvGeom& g = P.g;
  bool act[TM][TN];
  f32x16_t acc[TM][TN], tacc[TM][TN];
#pragma unroll
  for (int im = 0; im < TM; ++im)
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      act[im][in] = true;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[im][in][v] = 0.0f;
    }
  // this lane's output columns: image and input pixel
  int img[TN], ph[TN], pw[TN];
  bool cvalid[TN];
  const int hw = g.Hout * g.Wout;
#pragma unroll
  for (int in = 0; in < TN; ++in) {
    const long j = (long)n0 + wn * WTN + in * 32 + (lane & 31);
    cvalid[in] = j < P.Ncols;
    img[in] = cvalid[in] ? (int)(j / hw) : 0;
    const int rem = cvalid[in] ? (int)(j - (long)img[in] * hw) : 0;
    ph[in] = rem / g.Wout;
    pw[in] = rem - ph[in] * g.Wout;
  }
  LoaderKC<T, BM, 256> la;
  PatchLoader<T, BN> lb;
  la.init(P.Wp, axis_identity(P.K), m0, tid);
  ConvGeom plain = g;
  plain.blk = nullptr;
  lb.init(P.src, plain, n0, tid);
  const int taps = g.KH * g.KW;
  for (int tap = 0; tap < taps; ++tap) {
#pragma unroll
    for (int im = 0; im < TM; ++im)
#pragma unroll
      for (int in = 0; in < TN; ++in)
#pragma unroll
        for (int v = 0; v < 16; ++v) tacc[im][in][v] = 0.0f;
    lb.K = (tap + 1) * g.Ck;  // the patch loader returns zeros beyond this tap's output channels
    gemm_mainloop<T, BM, BN, WGM, WGN>(la, lb, tap * g.Ck, (tap + 1) * g.Ck, lds, tacc, act);
    const int fh = tap / g.KW, fw = tap - fh * g.KW;        // flipped tap the loader walked
    const int kh = g.KH - 1 - fh, kw = g.KW - 1 - fw;        // the filter tap it stands for
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      const int oh = ph[in] - g.pad_h + fh, ow = pw[in] - g.pad_w + fw;   // output position of this term
      if (!cvalid[in] || oh < 0 || oh >= g.Hin || ow < 0 || ow >= g.Win) continue;
      const uint8_t* band = g.blk + (long)(img[in] * g.RB + (oh * g.Win + ow) / g.bx) * g.CB;
#pragma unroll
      for (int im = 0; im < TM; ++im)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int c = m0 + wm * WTM + im * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (c < P.M && band[((c * g.KH + kh) * g.KW + kw) / g.by]) acc[im][in][v] += tacc[im][in][v];
        }
    }
  }
  gemm_epilogue<T, BM, BN, WGM, WGN>(P.C, acc, m0, n0, P.M, (int)P.Ncols);
}

// A operand of BWD_WEIGHT: row = co, contraction index k = (n, oh, ow) over dY[N, Cout, Ho, Wo].
template <typename T, int ROWS>
struct GradRowLoader {
  static constexpr int CE = ElemTraits<T>::CE;
  static constexpr int PASSES = ROWS / 32;
  static constexpr int NREG = PASSES;
  const T* src;
  int Cout, HW, vec;
  long K;
  int row[PASSES];
  bool rvalid[PASSES];
  int lr[PASSES], lc;

  __device__ __forceinline__ void init(const void* p, int cout, int hw, long k, int v, int row0, int tid) {
    src = (const T*)p;
    Cout = cout;
    HW = hw;
    K = k;
    vec = v;
    lc = tid & 7;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      lr[ps] = (tid >> 3) + 32 * ps;
      row[ps] = row0 + lr[ps];
      rvalid[ps] = row[ps] < Cout;
    }
  }
  __device__ __forceinline__ void load(int k0, uint4 (&regs)[PASSES]) const {
    const long kc = (long)k0 + lc * CE;
    const int n = (int)(kc / HW);
    const int p = (int)(kc - (long)n * HW);
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (rvalid[ps] && kc < K) {
        const T* base = src + ((long)n * Cout + row[ps]) * HW;
        if (vec && p + CE <= HW) {
          v = *reinterpret_cast<const uint4*>(base + p);
        } else {
          T tmp[CE];
          int nn = 0, pp = p;
#pragma unroll
          for (int e = 0; e < CE; ++e) {
            if (pp >= HW) {
              pp -= HW;
              ++nn;
            }
            tmp[e] = (kc + e < K) ? base[(long)nn * Cout * HW + pp] : (T)0;
            ++pp;
          }
          v = *reinterpret_cast<const uint4*>(tmp);
        }
      }
      regs[ps] = v;
    }
  }
  __device__ __forceinline__ void store(uint4* tile, const uint4 (&regs)[PASSES]) const {
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) tile[swz(lr[ps], lc)] = regs[ps];
  }
};

// B operand of BWD_WEIGHT: row j = (kept channel, tap), contraction index k = (n, oh, ow).
template <typename T, int ROWS>
struct PatchColLoader {
  static constexpr int CE = ElemTraits<T>::CE;
  static constexpr int PASSES = ROWS / 32;
  static constexpr int NREG = PASSES;
  const T* src;
  ConvGeom g;
  long K;
  long rbase[PASSES];
  int kh[PASSES], kw[PASSES];
  int cblk[PASSES];  // column block of this row's (channel, tap) (block pattern only)
  bool rvalid[PASSES];
  int lr[PASSES], lc;

  __device__ __forceinline__ void init(const void* p, const ConvGeom& geom, int row0, int tid) {
    src = (const T*)p;
    g = geom;
    const int taps = g.KH * g.KW;
    K = (long)g.N * g.Hout * g.Wout;
    lc = tid & 7;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      lr[ps] = (tid >> 3) + 32 * ps;
      const int j = row0 + lr[ps];
      rvalid[ps] = j < g.Ck * taps;
      const int cc = rvalid[ps] ? j / taps : 0;
      const int tap = rvalid[ps] ? j - cc * taps : 0;
      const int ch = g.chan ? g.chan[cc] : cc;
      rbase[ps] = (long)ch * g.Hin * g.Win;
      kh[ps] = tap / g.KW;
      kw[ps] = tap - kh[ps] * g.KW;
      cblk[ps] = g.blk ? (ch * taps + tap) / g.by : 0;
    }
  }
  __device__ __forceinline__ void load(int k0, uint4 (&regs)[PASSES]) const {
    const long kc = (long)k0 + lc * CE;
    const int hw = g.Hout * g.Wout;
    const int n0 = (int)(kc / hw);
    const int p0 = (int)(kc - (long)n0 * hw);
    const int oh0 = p0 / g.Wout, ow0 = p0 - oh0 * g.Wout;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (rvalid[ps] && kc < K) {
        T tmp[CE];
        int n = n0, oh = oh0, ow = ow0;
#pragma unroll
        for (int e = 0; e < CE; ++e) {
          if (ow >= g.Wout) {
            ow = 0;
            if (++oh >= g.Hout) {
              oh = 0;
              ++n;
            }
          }
          T x = 0;
          if (kc + e < K) {
            const int ih = oh * g.stride - g.pad_h + kh[ps], iw = ow * g.stride - g.pad_w + kw[ps];
            if (ih >= 0 && ih < g.Hin && iw >= 0 && iw < g.Win &&
                (!g.blk || g.blk[(n * g.RB + (oh * g.Wout + ow) / g.bx) * g.CB + cblk[ps]]))
              x = src[(long)n * g.Cin * g.Hin * g.Win + rbase[ps] + (long)ih * g.Win + iw];
          }
          tmp[e] = x;
          ++ow;
        }
        v = *reinterpret_cast<const uint4*>(tmp);
      }
      regs[ps] = v;
    }
  }
  __device__ __forceinline__ void store(uint4* tile, const uint4 (&regs)[PASSES]) const {
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) tile[swz(lr[ps], lc)] = regs[ps];
  }
};

struct ConvWgradParams {
  const void* dY;
  const void* A;
  ConvGeom g;
  float* part;   // [splits][Cout][Nn] fp32 partial sums
  int Cout, Nn, dy_vec;
  long K;
  int k_per_split;
  int tiles_n;
};

template <typename T, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void conv_wgrad_kernel(const ConvWgradParams P) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  __shared__ uint4 lds[2 * (BM + BN) * LDS_ROW_U4];
  const int tid = threadIdx.x;
  const int mb = blockIdx.x / P.tiles_n, nb = blockIdx.x % P.tiles_n;
  const int m0 = mb * BM, n0 = nb * BN;
  const int split = blockIdx.y;
  const long kb = (long)split * P.k_per_split;
  const long ke = kb + P.k_per_split < P.K ? kb + P.k_per_split : P.K;
  bool act[TM][TN];
  f32x16_t acc[TM][TN];
#pragma unroll
  for (int im = 0; im < TM; ++im)
#pragma unroll
    for (int in = 0; in < TN; ++in) {
      act[im][in] = true;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[im][in][v] = 0.0f;
    }
  if (kb < ke) {
    GradRowLoader<T, BM> la;
    PatchColLoader<T, BN> lb;
    la.init(P.dY, P.Cout, P.g.Hout * P.g.Wout, P.K, P.dy_vec, m0, tid);
    lb.init(P.A, P.g, n0, tid);
    gemm_mainloop<T, BM, BN, WGM, WGN>(la, lb, (int)kb, (int)ke, lds, acc, act);
  }
  OutMat C{};
  C.p = P.part + (long)split * P.Cout * P.Nn;
  C.ld = P.Nn;
  C.rm = axis_identity(P.Cout);
  C.cn = axis_identity(P.Nn);
  C.out_f32 = 1;
  C.alpha = 1.0f;
  gemm_epilogue<T, BM, BN, WGM, WGN>(C, acc, m0, n0, P.Cout, P.Nn);
}

// dWt[co][c][tap] = rank[c] >= 0 ? sum over splits of part[s][co][rank[c]*taps + tap] : 0
template <typename T>
__global__ void conv_wgrad_reduce_kernel(const float* part, const int* rank, int splits, int Cout, int C, int taps,
                                         int Nn, int kept_only, T* dWt) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long total = (long)Cout * C * taps;
  if (idx >= total) return;
  const int tap = (int)(idx % taps);
  const int c = (int)((idx / taps) % C);
  const int co = (int)(idx / ((long)taps * C));
  float s = 0.0f;
  const int r = rank[c];
  if (r < 0 && kept_only) return;
  if (r >= 0)
    for (int sp = 0; sp < splits; ++sp) s += part[((long)sp * Cout + co) * Nn + (long)r * taps + tap];
  dWt[idx] = ElemTraits<T>::from_f32(s);
}

__global__ void rank_from_keep_kernel(const int* keep, int n_keep, int C, int* rank) {
  for (int c = threadIdx.x; c < C; c += blockDim.x) rank[c] = -1;
  __syncthreads();
  for (int j = threadIdx.x; j < n_keep; j += blockDim.x) rank[keep[j]] = j;
}


// ---- bf16, stride 1: channels-last grid + LDS-direct implicit GEMM ----------------------------------
//
// The kept feature maps are copied once into a zero-bordered channels-last grid
// T[(n*Hg + h + oh)*Wg + w + ow][Cp] (compaction of the kept maps and layout change in one pass;
// Cp = kept channels rounded up to 64, extra channels zero).  On that grid the patch of an
// output pixel is, per filter tap, one contiguous Cp-run at a pixel offset that depends on the
// tap only, so the im2col operand streams through 16-byte LDS-direct loads like a plain matrix.

__host__ __device__ static inline int pad64(int n) { return (n + 63) & ~63; }

// Optional mask of the copy (gradients under a block pattern, Section 5.2.2): source pixel p of image n is
// copied iff blk[(n * RB + p / x) * CB + cb] != 0, else it becomes zeros.  blk == NULL: everything is copied.
struct BandMask {
  const uint8_t* blk;
  int RB, CB, cb, x;
};
__device__ __forceinline__ bool band_kept(const BandMask& m, int n, int p) {
  return !m.blk || m.blk[((long)n * m.RB + p / m.x) * m.CB + m.cb] != 0;
}

// position of channel c in the ascending kept list, or -1 (uniform per workgroup where c is)
__device__ __forceinline__ int kept_rank(const int* keep, int n_keep, int c) {
  int lo = 0, hi = n_keep - 1;
  while (lo <= hi) {
    const int mid = (lo + hi) >> 1, v = keep[mid];
    if (v == c) return mid;
    if (v < c) lo = mid + 1;
    else hi = mid - 1;
  }
  return -1;
}

// planes of dropped channels of an NCHW tensor to +0.0 (the GEMM writes the kept ones); a workgroup
// takes one channel of ZP_IMGS images, 16-byte stores where the planes allow them
constexpr int ZP_IMGS = 8;
struct ZeroPlanesJob {
  uint16_t* dst;
  const int* keep;
  int n_keep, N, C, HW, vec;
  int blocks;  // C * ceil(N / ZP_IMGS) workgroups of 256 threads (0: no job)
};
__device__ __forceinline__ void zero_dropped_planes_body(const ZeroPlanesJob& z, int block) {
  const int c = block % z.C;
  if (kept_rank(z.keep, z.n_keep, c) >= 0) return;
  const int n0 = (block / z.C) * ZP_IMGS, n1 = min(n0 + ZP_IMGS, z.N);
  if (z.vec) {
    const int chunks = z.HW >> 3;
    for (int i = threadIdx.x; i < (n1 - n0) * chunks; i += 256) {
      const int n = n0 + i / chunks, q = i % chunks;
      *reinterpret_cast<uint4*>(z.dst + ((long)n * z.C + c) * z.HW + q * 8) = make_uint4(0, 0, 0, 0);
    }
  } else {
    for (int i = threadIdx.x; i < (n1 - n0) * z.HW; i += 256) z.dst[((long)(n0 + i / z.HW) * z.C + c) * z.HW + i % z.HW] = 0;
  }
}
__global__ __launch_bounds__(256) void zero_dropped_planes_kernel(ZeroPlanesJob z) { zero_dropped_planes_body(z, (int)blockIdx.x); }

// output positions of dropped rows of the input matrix to +0.0 (row-based sensitivity-aware pattern,
// Section 5.2.1: the results of the kept rows fill the same rows of the output, the others are zero);
// one workgroup per (channel, image) plane, eight positions per thread and step
constexpr int ZPX = 8;  // planes (channels of one image) per workgroup
struct ZeroPixelsJob {
  uint16_t* Y;
  const uint8_t* row_mask;
  int Cout, HW;
  int blocks;  // N * ceil(Cout / ZPX) workgroups of 256 threads (0: no job)
  int all;     // 1: zero every position (a plain stream of 16-byte stores; the product that follows writes the kept ones)
};
__device__ __forceinline__ void zero_dropped_pixels_body(const ZeroPixelsJob& z, int block) {
  const int cgs = (z.Cout + ZPX - 1) / ZPX;
  const int co0 = (block % cgs) * ZPX, n = block / cgs;
  const int nco = min(ZPX, z.Cout - co0);
  uint16_t* p = z.Y + ((long)n * z.Cout + co0) * z.HW;
  const uint8_t* m = z.row_mask + (long)n * z.HW;
  const bool vec = (z.HW % 8) == 0 && (((uintptr_t)z.Y | (uintptr_t)z.row_mask) & 15) == 0;
  if (z.all) {  // (host: only with HW % 8 == 0 and Y on a 16-byte boundary)
    uint4* dst = reinterpret_cast<uint4*>(p);
    for (int i = threadIdx.x; i < nco * (z.HW >> 3); i += 256) dst[i] = make_uint4(0, 0, 0, 0);
  } else if (vec) {
    const int chunks = z.HW >> 3;
    for (int i = threadIdx.x; i < nco * chunks; i += 256) {
      const int c = i / chunks, q = (i - c * chunks) * 8;
      const uint2 mk = *reinterpret_cast<const uint2*>(m + q);
      uint16_t* dst = p + (long)c * z.HW + q;
      if ((mk.x | mk.y) == 0) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(0, 0, 0, 0);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (!(((e < 4 ? mk.x : mk.y) >> ((e & 3) * 8)) & 0xff)) dst[e] = 0;
      }
    }
  } else {
    for (int i = threadIdx.x; i < nco * z.HW; i += 256)
      if (!m[i % z.HW]) p[i] = 0;
  }
}

__global__ __launch_bounds__(256) void zero_dropped_pixels_grid_kernel(ZeroPixelsJob z) { zero_dropped_pixels_body(z, (int)blockIdx.x); }

// Block-based pattern on the LDS-direct path (Section 5.2.2).  When a block of the input matrix spans
// whole 64-channel groups over all filter taps (y a multiple of 64 * taps), a kept block is a set of whole
// 64-deep contraction steps of the grid's (tap, channel) order, and a row band of x output positions can be
// laid out as column tiles of its own (padded with entries that store nothing): every tile then contracts
// over the kept blocks of ONE band, and dropped blocks are neither loaded nor multiplied.
// Tile T = ((image * RB + band) * tpb + part) holds positions band*x + part*BN ... of its image.
struct BlockPlan {
  int N, HoWo, x, RB, CB, tpb, BN, taps, CG, cg_per_blk, KB;
};
// kept 64-channel groups of tile T's band (0 for a tile that holds no position)
__device__ __forceinline__ int block_tile_groups(const uint8_t* blk, const BlockPlan& p, int T) {
  const int part = T % p.tpb, band = (T / p.tpb) % p.RB, n = T / (p.tpb * p.RB);
  if (part * p.BN >= p.x || band * p.x + part * p.BN >= p.HoWo) return 0;
  const uint8_t* row = blk + (long)(n * p.RB + band) * p.CB;
  int g = 0;
  for (int cg = 0; cg < p.CG; ++cg) g += row[cg / p.cg_per_blk] ? 1 : 0;
  return g;
}

// One workgroup (256 threads) lays out tile T: its padded pixel list, the list of its kept contraction steps
// and their number.  Where the tile goes in the launch: longest contraction first on every XCD (workgroups
// start in order, so the long ones do not end up alone at the end).  Every workgroup finds the rank of its own
// tile by counting the tiles that come before it (more kept groups, or as many and a lower index): no pass of
// its own, no hand-over.  order = 0: tile T stays at T.
constexpr int kBlockOrderMaxTiles = 1 << 11;  // (each of n workgroups reads n keys)
struct BlockPlanJob {
  const uint8_t* blk;
  BlockPlan p;
  int tiles, order;
  int *pix, *kb_list, *kb_cnt;
  int blocks;  // = tiles (0: no job)
};
__device__ __forceinline__ void block_plan_body(const BlockPlanJob& j, int T, int* red4) {
  const BlockPlan& p = j.p;
  const int tid = threadIdx.x;
  int at = T;
  if (j.order) {
    const int mine = block_tile_groups(j.blk, p, T);
    int before = 0;
    for (int U = tid; U < j.tiles; U += 256) {
      const int k = block_tile_groups(j.blk, p, U);
      before += (k > mine || (k == mine && U < T)) ? 1 : 0;
    }
    for (int o = 32; o > 0; o >>= 1) before += __shfl_down(before, o, 64);
    if ((tid & 63) == 0) red4[tid >> 6] = before;
    __syncthreads();
    const int r = red4[0] + red4[1] + red4[2] + red4[3];
    // The kernel deals its work items to the 8 XCDs in contiguous shares [x*n/8, (x+1)*n/8) and a share's
    // workgroups start in order: rank r goes to XCD r % 8, place r / 8 of its share; the last n % 8 ranks
    // fill the shares that are one longer than the others.
    const int even = j.tiles / 8;
    int x = r & 7;
    at = r >> 3;
    if (r >= 8 * even) {
      int q = r - 8 * even;
      at = even;
      for (x = 0; x < 8; ++x) {
        const int size = (int)((long)(x + 1) * j.tiles / 8) - (int)((long)x * j.tiles / 8);
        if (size > even && q-- == 0) break;
      }
    }
    at += (int)((long)x * j.tiles / 8);
  }
  const int part = T % p.tpb, band = (T / p.tpb) % p.RB, n = T / (p.tpb * p.RB);
  for (int i = tid; i < p.BN; i += 256) {
    const int in_band = part * p.BN + i, pos = band * p.x + in_band;
    j.pix[(long)at * p.BN + i] = (in_band < p.x && pos < p.HoWo) ? n * p.HoWo + pos : -1;
  }
  if (tid == 0) {
    int cnt = 0;
    const bool any = part * p.BN < p.x && band * p.x + part * p.BN < p.HoWo;
    const uint8_t* row = j.blk + (long)(n * p.RB + band) * p.CB;
    if (any)
      for (int cg = 0; cg < p.CG; ++cg)  // (all taps of a channel group in a row: they share their lines in L2)
        if (row[cg / p.cg_per_blk])
          for (int tap = 0; tap < p.taps; ++tap) j.kb_list[(long)at * p.KB + cnt++] = tap * p.CG + cg;
    j.kb_cnt[at] = cnt;
  }
}
__global__ __launch_bounds__(256) void block_plan_kernel(BlockPlanJob j) {
  __shared__ int red4[4];
  block_plan_body(j, (int)blockIdx.x, red4);
}

// Wp[row][tap*Cp + q]: forward (flip = 0): row = output channel, q = kept input channel;
// data gradient (flip = 1): row = kept input channel, q = output channel, taps reversed.
struct PackJob {
  const uint16_t* Wt;
  const int* keep;
  int C, taps, rows, inner, Cp, flip;
  uint16_t* out;
  int blocks;  // workgroups of 256 threads that cover rows * taps * Cp entries (0: no job)
};
__device__ __forceinline__ void pack_weights_body(const PackJob& j, long idx) {
  const long total = (long)j.rows * j.taps * j.Cp;
  if (idx >= total) return;
  int q, tap, r;
  if (total < (1L << 31)) {  // (32-bit divisions: a fraction of the instructions of 64-bit ones)
    const uint32_t i32 = (uint32_t)idx, a = i32 / (uint32_t)j.Cp;
    q = (int)(i32 - a * (uint32_t)j.Cp);
    r = (int)(a / (uint32_t)j.taps);
    tap = (int)(a - (uint32_t)r * (uint32_t)j.taps);
  } else {
    q = (int)(idx % j.Cp);
    tap = (int)((idx / j.Cp) % j.taps);
    r = (int)(idx / ((long)j.Cp * j.taps));
  }
  uint16_t v = 0;
  if (q < j.inner)
    v = j.flip ? j.Wt[((long)q * j.C + (j.keep ? j.keep[r] : r)) * j.taps + (j.taps - 1 - tap)]
               : j.Wt[((long)r * j.C + (j.keep ? j.keep[q] : q)) * j.taps + tap];
  j.out[idx] = v;
}
__global__ void pack_weights_grid_kernel(PackJob j) { pack_weights_body(j, (long)blockIdx.x * blockDim.x + threadIdx.x); }
static PackJob pack_job(const void* Wt, const int* keep, int C, int taps, int rows, int inner, int Cp, int flip, uint16_t* out) {
  return PackJob{(const uint16_t*)Wt, keep, C, taps, rows, inner, Cp, flip, out, (int)(((long)rows * taps * Cp + 255) / 256)};
}

// 8 neighbouring pixels of one channel plane, of which the first `valid` exist: one 16-byte load where the
// address allows it, two 8-byte loads or element by element elsewhere (planes of 14 x 14 or 7 x 7 positions
// do not start on 16-byte boundaries)
__device__ __forceinline__ uint4 load_pixels8(const uint16_t* p, int valid) {
  if (valid >= 8 && (((uintptr_t)p) & 15) == 0) return *reinterpret_cast<const uint4*>(p);
  if (valid >= 8 && (((uintptr_t)p) & 7) == 0) {
    const uint2 a = *reinterpret_cast<const uint2*>(p), b = *reinterpret_cast<const uint2*>(p + 4);
    return make_uint4(a.x, a.y, b.x, b.y);
  }
  uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < 8; ++e)
    if (e < valid) w[e >> 1] |= (uint32_t)p[e] << ((e & 1) * 16);
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// The copy, driven from the source side:
// a workgroup reads 64 channels x 64 source pixels with 16-byte loads (a thread takes 8 pixels of two
// neighbouring channels), pairs the channels in registers, transposes the pairs through LDS and writes each
// pixel's 64 channels as 128 contiguous bytes.  The border pixels of an image are dealt to the image's
// workgroups and the margin behind the last image to all of them: every pixel of the grid is written once.
// LDS holds [pixel row][32 channel pairs] without padding: pixel 8q + e sits in row 8e + q and its 16-byte
// groups are exchanged by q's upper bits, which spreads both the 4-byte stores of a wave and its 16-byte
// loads over all banks.
__global__ __launch_bounds__(256) void to_grid_src_kernel(const uint16_t* src, const int* chan, int n_chan, int Cs, int Hs,
                                                          int Ws, FastDiv div_ws, int Hg, int Wg, int oh, int ow, int Cp,
                                                          int N,
                                                          long n_pix_total, BandMask bm, uint16_t* dst, PackJob pj,
                                                          ZeroPlanesJob zj, ZeroPixelsJob zp, BlockPlanJob bj, int main_x) {
  __shared__ uint32_t tile[64 * 32];
  __shared__ int red4[4];
  // (workgroups beyond the copy's own pack the weights of the product that follows and zero the planes it will
  // not write: independent small jobs that would otherwise be launches of their own)
  // (they come first in the launch: started last they would be a tail of their own behind the copy)
  const int extra_x = (int)gridDim.x - main_x;
  if ((int)blockIdx.x < extra_x) {
    const int b = (int)blockIdx.x * (int)gridDim.y + (int)blockIdx.y;
    if (b < pj.blocks) pack_weights_body(pj, (long)b * 256 + threadIdx.x);
    else if (b < pj.blocks + zj.blocks) zero_dropped_planes_body(zj, b - pj.blocks);
    else if (b < pj.blocks + zj.blocks + zp.blocks) zero_dropped_pixels_body(zp, b - pj.blocks - zj.blocks);
    else if (b < pj.blocks + zj.blocks + zp.blocks + bj.blocks) block_plan_body(bj, b - pj.blocks - zj.blocks - zp.blocks, red4);
    return;
  }
  const int HW = Hs * Ws;
  const int px_tiles = (HW + 63) / 64;
  // Channel rows start at any multiple of 2 * HW bytes, so a tile's 128-byte runs straddle cache lines that the
  // neighbouring pixel tile reads too.  Workgroups are dealt to the 8 XCDs in turn: XCD x takes the x-th eighth
  // of the tiles in order, so the second read of a line finds it in that XCD's L2 (half the fetched bytes).
  const int even = main_x / 8, bx = (int)blockIdx.x - extra_x;
  const int m = bx < 8 * even ? (bx & 7) * even + (bx >> 3) : bx;
  const int n = m / px_tiles, tile_j = m - n * px_tiles, p0 = tile_j * 64;
  const int c0 = blockIdx.y * 64;
  const int t = threadIdx.x;
  // masked copy: which of the tile's 64 pixels count is the same for all of its channels, looked up once
  __shared__ uint8_t piece_keep[8];
  if (bm.blk) {
    if (t < 8) {
      unsigned bits = 0;
      for (int e = 0; e < 8; ++e) {
        const int p = p0 + t * 8 + e;
        if (p < HW && band_kept(bm, n, p)) bits |= 1u << e;
      }
      piece_keep[t] = (uint8_t)bits;
    }
    __syncthreads();
  }
  {
    const int cp = t >> 3, q = t & 7;  // channel pair, piece of 8 pixels
    const int c = c0 + 2 * cp, p = p0 + q * 8;
    uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
    if (p < HW) {
      if (c < n_chan) v0 = load_pixels8(src + ((long)n * Cs + (chan ? chan[c] : c)) * HW + p, HW - p);
      if (c + 1 < n_chan) v1 = load_pixels8(src + ((long)n * Cs + (chan ? chan[c + 1] : c + 1)) * HW + p, HW - p);
    }
    uint32_t lo[4] = {v0.x, v0.y, v0.z, v0.w}, hi[4] = {v1.x, v1.y, v1.z, v1.w};
    if (bm.blk) {
      const unsigned bits = piece_keep[q];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (!((bits >> e) & 1)) {
          lo[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
          hi[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
        }
    }
    const int col = (((cp >> 2) ^ (q & 6)) << 2) | (cp & 3);
#pragma unroll
    for (int e = 0; e < 8; ++e)  // pixel e of the piece: channel c in the low half, c + 1 in the high half
      tile[(e * 8 + q) * 32 + col] = __builtin_amdgcn_perm(hi[e >> 1], lo[e >> 1], (e & 1) ? 0x07060302u : 0x05040100u);
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = (t >> 3) + 32 * i, c8 = t & 7;  // LDS row, group of 8 channels
    const int q = r & 7, p = p0 + 8 * q + (r >> 3);
    if (p >= HW) continue;
    const int h = (int)fdiv((uint32_t)p, div_ws), w = p - h * Ws;
    const long g = ((long)n * Hg + h + oh) * Wg + w + ow;
    *reinterpret_cast<uint4*>(dst + g * Cp + c0 + c8 * 8) = *reinterpret_cast<const uint4*>(&tile[r * 32 + ((c8 ^ (q & 6)) << 2)]);
  }
  // zero pass, for this workgroup's 64 channels.  The border of image n: `top` whole rows above, `bot` below,
  // then per image row ow pixels on the left and the rest of `side` on the right; border index b of the image
  // belongs to workgroup b * px_tiles / B of the image's px_tiles.
  const uint4 zero = make_uint4(0, 0, 0, 0);
  const int top = oh * Wg, bot = (Hg - oh - Hs) * Wg, side = Wg - Ws, B = top + bot + Hs * side;
  const int b0 = (int)((long)tile_j * B / px_tiles), b1 = (int)((long)(tile_j + 1) * B / px_tiles);
  for (int b = b0 + (t >> 3); b < b1; b += 32) {
    int pos;
    if (b < top) pos = b;
    else if (b < top + bot) pos = (oh + Hs) * Wg + (b - top);
    else {
      const int s = b - top - bot, row = s / (side > 0 ? side : 1), k = s - row * side;
      pos = (oh + row) * Wg + (k < ow ? k : k + Ws);
    }
    *reinterpret_cast<uint4*>(dst + ((long)n * Hg * Wg + pos) * Cp + c0 + (t & 7) * 8) = zero;
  }
  // the margin behind the last image, 32 pixels per workgroup
  for (long g = (long)N * Hg * Wg + (long)bx * 32 + (t >> 3); g < n_pix_total; g += (long)main_x * 32)
    *reinterpret_cast<uint4*>(dst + g * Cp + c0 + (t & 7) * 8) = zero;
}


// output positions of dropped rows of the input matrix to +0.0 (row-based sensitivity-aware pattern,
// Section 5.2.1: the results of the kept rows fill the same rows of the output, the others are zero);
// one workgroup per (channel, image) plane
template <typename T>
__global__ __launch_bounds__(256) void zero_dropped_pixels_kernel(T* Y, const uint8_t* row_mask, int Cout, int HW) {
  const int co = blockIdx.x, n = blockIdx.y;
  T* p = Y + ((long)n * Cout + co) * HW;
  const uint8_t* m = row_mask + (long)n * HW;
  for (int i = threadIdx.x; i < HW; i += 256)
    if (!m[i]) p[i] = (T)0;
}

// out = Y with the positions of dropped rows of the input matrix as +0.0 (the gradient of a row pattern's
// forward pass only arrives on kept positions); one workgroup per (channel, image) plane
template <typename T>
__global__ __launch_bounds__(256) void mask_pixels_kernel(const T* Y, const uint8_t* row_mask, int Cout, int HW, T* out) {
  const int co = blockIdx.x, n = blockIdx.y;
  const long base = ((long)n * Cout + co) * HW;
  const uint8_t* m = row_mask + (long)n * HW;
  for (int i = threadIdx.x; i < HW; i += 256) out[base + i] = m[i] ? Y[base + i] : (T)0;
}
// the same with the mask of one column block of a block pattern: position p of image n is kept iff
// blk[(n * RB + p / x) * CB + cb] != 0
template <typename T>
__global__ __launch_bounds__(256) void mask_bands_kernel(const T* Y, const uint8_t* blk, int RB, int CB, int cb, int x, int Cout,
                                                         int HW, T* out) {
  const int co = blockIdx.x, n = blockIdx.y;
  const long base = ((long)n * Cout + co) * HW;
  const uint8_t* m = blk + (long)n * RB * CB + cb;
  for (int i = threadIdx.x; i < HW; i += 256) out[base + i] = m[(long)(i / x) * CB] ? Y[base + i] : (T)0;
}
__global__ void iota_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}

// dW[co][c][tap] = sum over splits of part[sp][co][tap*Cp + rank(c)] (dropped channels: +0.0).
// A thread owns one kept synapse (co, tap, r): consecutive threads read consecutive r (coalesced), the
// loads of the splits are independent and summed in split order.  The same launch writes the zeros of
// the dropped channels (its first gridDim.x - zero_blocks workgroups sum, the rest zero).
__global__ __launch_bounds__(256) void wgrad_grid_reduce_kernel(const float* part, const int* keep, int n_keep, int splits,
                                                                int Cout, int C, int taps, int Cp, int sum_blocks,
                                                                uint16_t* dWt) {
  const int Nn = taps * Cp;
  if ((int)blockIdx.x < sum_blocks) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)Cout * taps * n_keep) return;
    // (the host refuses 2^31 kept synapses or more: 32-bit divisions, a fraction of the instructions of 64-bit ones)
    const uint32_t i32 = (uint32_t)idx, q1 = i32 / (uint32_t)n_keep;
    const int r = (int)(i32 - q1 * (uint32_t)n_keep);
    const int co = (int)(q1 / (uint32_t)taps), tap = (int)(q1 - (uint32_t)co * (uint32_t)taps);
    const float* p = part + (long)co * Nn + tap * Cp + r;
    const long stride = (long)Cout * Nn;
    float s = 0.0f;
    int sp = 0;
    for (; sp + 4 <= splits; sp += 4) {
      const float v0 = p[(sp + 0) * stride], v1 = p[(sp + 1) * stride], v2 = p[(sp + 2) * stride], v3 = p[(sp + 3) * stride];
      s += v0;
      s += v1;
      s += v2;
      s += v3;
    }
    for (; sp < splits; ++sp) s += p[sp * stride];
    dWt[((long)co * C + keep[r]) * taps + tap] = f32_to_bf16_bits(s);
    return;
  }
  // zeros of the dropped channels: one thread per (co, c)
  const long idx = (long)(blockIdx.x - sum_blocks) * 256 + threadIdx.x;
  if (idx >= (long)Cout * C) return;
  const int c = (int)(idx % C);
  if (kept_rank(keep, n_keep, c) >= 0) return;
  uint16_t* o = dWt + idx * taps;
  for (int t = 0; t < taps; ++t) o[t] = 0;
}

struct ConvArgs {
  int32_t mode, dtype, N, C, H, W, Cout, kh, kw, stride, pad, n_keep, Ho, Wo, es;
  int32_t reuse;  // ARD_CONV_REUSE_* bits of the mode argument
  // block-based pattern of the forward pass (ard_conv_fwd_blocks): x-by-y blocks of the input matrices
  const uint8_t* blk;
  int32_t bx, by;
  int32_t kept_only;  // gradients: write the kept channels' part of the output only (the caller covers the rest)
  BandMask dy_mask;   // gradients on the channels-last grids: positions of dY that count (blk == NULL: all)
};

struct ConvWs {
  unsigned long long* score;
  unsigned long long* score_part;  // [kScoreParts x C] partial scores of the workgroups
  int* rank;
  int* all_chan;   // 0 .. C-1: the kept list of the passes that drop no channel
  char* dy_rows;   // [N, Cout, Ho, Wo] dtype: dY with the dropped rows of a row pattern zeroed
  char* wp;
  float* part;
  uint16_t *grid_a, *grid_y;  // channels-last grids of the fast path (NULL when it does not apply)
  uint16_t* gwp;              // its packed weights
  float* gpart;               // its weight-gradient partial sums
  int *blk_pix, *blk_kb, *blk_cnt;  // block pattern on the fast path: padded pixel list, per-tile block lists and counts
  size_t blk_ints;                  // ints reserved for blk_pix and for blk_kb
  size_t total;
  int splits;
  int gsplits;  // contraction splits of the fast weight-gradient product
};

// The LDS-direct path: bf16, stride 1, padding no larger than the filter allows for the data
// gradient, and grids small enough for 32-bit element offsets.
static bool conv_fast_ok(const ConvArgs& a);
static long conv_grid_pixels(const ConvArgs& a, int* hg, int* wg);
static int conv_grid_splits(const ConvArgs& a);

static int wgrad_splits(const ConvArgs& a) {
  long tiles = (long)ceil_div(a.Cout, 128) * ceil_div(a.C * a.kh * a.kw, 128);
  long K = (long)a.N * a.Ho * a.Wo;
  long want = (1024 + tiles - 1) / tiles;
  long maxs = (K + 255) / 256;
  long s = want < maxs ? want : maxs;
  return (int)(s < 1 ? 1 : (s > 64 ? 64 : s));
}

static ConvWs conv_ws_layout(char* base, const ConvArgs& a) {
  ConvWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes ? bytes : 1, 256);
    return p;
  };
  const size_t taps = (size_t)a.kh * a.kw;
  w.splits = wgrad_splits(a);
  w.score = (unsigned long long*)take((size_t)a.C * 8);
  w.score_part = (unsigned long long*)take((size_t)a.C * 8 * kScoreParts);
  w.rank = (int*)take((size_t)a.C * 4);
  w.all_chan = (int*)take((size_t)a.C * 4);
  w.dy_rows = take((size_t)a.N * a.Cout * a.Ho * a.Wo * a.es);
  w.wp = take((size_t)a.Cout * a.C * taps * a.es);
  w.part = (float*)take((size_t)w.splits * a.Cout * a.C * taps * 4);
  w.grid_a = w.grid_y = w.gwp = nullptr;
  w.gpart = nullptr;
  w.blk_pix = w.blk_kb = w.blk_cnt = nullptr;
  w.blk_ints = 0;
  w.gsplits = 1;
  if (conv_fast_ok(a)) {
    int hg, wg;
    const long pix = conv_grid_pixels(a, &hg, &wg);
    w.gsplits = conv_grid_splits(a);
    const size_t cpa = pad64(a.C), cpy = pad64(a.Cout);
    w.grid_a = (uint16_t*)take((size_t)pix * cpa * 2);
    w.grid_y = (uint16_t*)take((size_t)pix * cpy * 2);
    w.gwp = (uint16_t*)take((size_t)(a.Cout > a.C ? a.Cout : a.C) * taps * (cpa > cpy ? cpa : cpy) * 2);
    w.gpart = (float*)take((size_t)w.gsplits * a.Cout * taps * cpa * 4);
    // tiles padded to at most twice the output positions; at most 128 blocks per tile of at least 128 positions
    w.blk_ints = 2 * (size_t)a.N * a.Ho * a.Wo + 512;
    w.blk_pix = (int*)take(w.blk_ints * 4);
    w.blk_kb = (int*)take(w.blk_ints * 4);
    w.blk_cnt = (int*)take((w.blk_ints / 128 + 1) * 4 * 2);  // counts, then the tiles' places in the launch
  }
  w.total = off;
  return w;
}


static bool conv_fast_ok(const ConvArgs& a) {
  if (a.dtype != ARD_BF16 || a.stride != 1) return false;
  if (a.pad > a.kh - 1 || a.pad > a.kw - 1) return false;
  int hg, wg;
  const long pix = conv_grid_pixels(a, &hg, &wg);
  const long cmax = pad64(a.C > a.Cout ? a.C : a.Cout);
  return pix * cmax < (1L << 31) && (long)a.kh * a.kw * cmax < (1L << 24);
}

// Pixels of the largest grid any mode builds (input grid with its border, or the output grid
// bordered for the data gradient), plus the margin the shifted reads of the weight gradient
// and the 64-pixel tiles of the copy kernel may touch.
static long conv_grid_pixels(const ConvArgs& a, int* hg, int* wg) {
  const int ho = a.H + 2 * a.pad - a.kh + 1, wo = a.W + 2 * a.pad - a.kw + 1;
  const int h1 = a.H + 2 * a.pad, w1 = a.W + 2 * a.pad;
  const int h2 = ho + 2 * (a.kh - 1 - a.pad), w2 = wo + 2 * (a.kw - 1 - a.pad);
  *hg = h1 > h2 ? h1 : h2;
  *wg = w1 > w2 ? w1 : w2;
  const long margin = (long)a.kh * *wg + a.kw + 128;
  return (long)a.N * *hg * *wg + margin;
}

static int conv_grid_splits(const ConvArgs& a) {
  const long tiles = (long)ceil_div(a.Cout, 128) * ceil_div(a.kh * a.kw * pad64(a.C), 128);
  long s = 512 / tiles;  // about two 128 x 128 workgroups per CU
  return (int)(s < 1 ? 1 : (s > 64 ? 64 : s));
}

static bool al16c(const void* p) { return ((uintptr_t)p & 15) == 0; }

static int32_t to_grid(const void* src, const int* chan, int n_chan, int Cs, int Hs, int Ws, int N, int Hg, int Wg, int oh,
                       int ow, int Cp, long margin, uint16_t* dst, hipStream_t stream, BandMask bm = BandMask{},
                       PackJob pj = PackJob{}, ZeroPlanesJob zj = ZeroPlanesJob{}, ZeroPixelsJob zp = ZeroPixelsJob{},
                       BlockPlanJob bj = BlockPlanJob{}) {
  const long total = (long)N * Hg * Wg + margin;
  if (oh < 0 || ow < 0 || Hg < oh + Hs || Wg < ow + Ws) return fail(ARD_EINVAL, "grid copy: the image does not fit the grid");
  const int main_x = N * ceil_div(Hs * Ws, 64);
  const int gy = Cp / 64;
  dim3 grid((unsigned)(main_x + ceil_div(pj.blocks + zj.blocks + zp.blocks + bj.blocks, gy)), (unsigned)gy);
  ARD_LAUNCH(to_grid_src_kernel, grid, dim3(256), 0, stream, (const uint16_t*)src, chan, n_chan, Cs, Hs, Ws,
             fast_div((uint32_t)Ws), Hg, Wg, oh, ow, Cp, N, total, bm, dst, pj, zj, zp, bj, main_x);
  ARD_LAUNCH_CHECK("to_grid_src_kernel");
  return ARD_OK;
}

// Y[row][pixel] = sum_k Wp[row][k] * im2col[pixel][k] on the grid; NCHW output
// force_bn / kb_*: the block-based pattern's launch (column tile fixed by its plan, per-tile contraction lists)
static int32_t conv_grid_gemm(const uint16_t* Wp, int rows, int K, const uint16_t* grid_t, long grid_pixels,
                              const ConvMap& cv, void* out, hipStream_t stream, int force_bn = 0,
                              const int* kb_list = nullptr, const int* kb_cnt = nullptr, int kb_stride = 0) {
  FastParams F{};
  F.A = Wp;
  F.B = grid_t;
  F.a_elems = (long)rows * K;
  F.b_elems = grid_pixels * cv.Cp;
  F.C = (uint16_t*)out;
  F.lda = K;
  F.ldb = cv.Cp;
  F.am = axis_identity(rows);
  F.bn = axis_identity(cv.npix);
  F.k = axis_identity(K);
  F.alpha = 1.0f;
  F.splits = 1;
  F.M = rows;
  F.N = cv.npix;
  F.cv = cv;
  F.kb_list = kb_list, F.kb_cnt = kb_cnt, F.kb_stride = kb_stride;
  int bm, bn;
  if (force_bn) {
    bm = force_bn == 128 || rows > 128 ? 256 : 128;
    bn = force_bn;
  } else {
    // A launch runs in rounds: one workgroup of a large shape fills a CU (256 at a time), three of the 64 x 64
    // shape share one (768 at a time).  Measured on the 3x3 layers, a round of 256 x 128 or 128 x 256 tiles
    // takes 0.68 and a round of 64 x 64 tiles 0.34 of a round of 256 x 256 tiles: fewest rounds x cost wins
    // (so a layer with few output positions goes to small tiles on many CUs instead of large ones on a few).
    const auto rounds = [&](int tm, int tn, long slots) { return ((long)ceil_div(rows, tm) * ceil_div(cv.npix, tn) + slots - 1) / slots; };
    long best = rounds(64, 64, 768) * 34;
    bm = bn = 64;
    if (rows > 64) {
      const long c = rounds(128, 256, 256) * 68;
      if (c <= best) best = c, bm = 128, bn = 256;
    }
    if (rows > 128) {
      const long c1 = rounds(256, 128, 256) * 68, c2 = rounds(256, 256, 256) * 100;
      if (c1 <= best) best = c1, bm = 256, bn = 128;
      if (c2 <= best) best = c2, bm = 256, bn = 256;
    }
  }
  F.tiles_m = ceil_div(rows, bm);
  F.tiles_n = ceil_div(cv.npix, bn);
  const long tiles = (long)F.tiles_m * F.tiles_n;
  if (tiles >= (1L << 24)) return fail(ARD_ESHAPE, "convolution too large for one launch");
  F.total_tiles = (int)tiles;
  F.group_m = direct_group_m(F.total_tiles);
  const int grid = direct_plain_grid(F.total_tiles);
  if (bm == 256 && bn == 256) return launch_direct_kernel<true, true, 256, 256, 8, 1>(F, grid, stream);
  if (bm == 256) return launch_direct_kernel<true, true, 256, 128, 8, 1>(F, grid, stream);
  if (bm == 128) return launch_direct_kernel<true, true, 128, 256, 8, 1>(F, grid, stream);
  return launch_direct_kernel<true, true, 64, 64, 4, 1>(F, grid, stream);
}

// The column tile (128 or 256 positions) that wastes the least padding, or 0 when this path does not apply.
static int block_fast_tile(const ConvArgs& a, const ConvWs& w) {
  const int taps = a.kh * a.kw;
  if (!w.grid_a || !w.blk_pix || dev_knobs().no_fast || a.Cout <= 64) return 0;
  if (a.by % (64 * taps)) return 0;
  const int CG = pad64(a.C) / 64;
  if (taps * CG > 128) return 0;
  const long hw = (long)a.Ho * a.Wo, RB = ceil_div(a.Ho * a.Wo, a.bx);
  int best = 0;
  long best_len = 0;
  for (int bn : {256, 128}) {
    if (bn == 128 && a.Cout <= 128) continue;  // (the 128-row tile comes with 256 columns only)
    const long len = RB * ceil_div(a.bx, bn) * bn;  // padded positions per image
    if (len > 2 * hw) continue;
    if (!best || len < best_len) best = bn, best_len = len;
  }
  if (!best) return 0;
  const long tiles = (long)a.N * best_len / best;
  if ((size_t)(a.N * best_len) > w.blk_ints || (size_t)(tiles * taps * CG) > w.blk_ints || tiles >= (1L << 22)) return 0;
  return best;
}

static int32_t conv_run_grid(const ConvArgs& a, const void* A, const void* Wt, const void* dYin, void* out,
                             const int32_t* d_keep, const uint8_t* row_mask, const ConvWs& w, hipStream_t stream) {
  const int taps = a.kh * a.kw, Ck = a.n_keep;
  int hgm, wgm;
  const long pix_cap = conv_grid_pixels(a, &hgm, &wgm);
  (void)pix_cap;
  // Both grids are laid out the same way whichever pass builds them, so a later pass of the same layer
  // can take the grid an earlier one left in the workspace (ARD_CONV_REUSE_A / ARD_CONV_REUSE_DY):
  // A: zero border of `pad` pixels; dY: zero border of k-1-pad pixels (what the data gradient convolves).
  // The weight gradient wants dY on the grid of A without a border: for a size-preserving filter
  // (k - 1 = 2 pad) that is the bordered dY grid read from (k-1-pad) rows and columns further on.
  const long margin = (long)a.kh * wgm + a.kw + 128;
  const bool same = a.kh - 1 == 2 * a.pad && a.kw - 1 == 2 * a.pad;
  if (a.mode == ARD_CONV_FWD_ROWS) {
    // every channel, only the kept output positions: the product's columns are the listed pixels
    const int Cp = pad64(a.C), Hg = a.H + 2 * a.pad, Wg = a.W + 2 * a.pad, K = taps * Cp;
    // (the zeros of the dropped positions and the packed weights ride in the copy's launch)
    // (with few rows kept, zeros everywhere as one stream cost less than the masked stores of the dropped ones)
    const int fill_all = ((a.Ho * a.Wo) % 8) == 0 && al16c(out) && (long)Ck * 10 <= (long)a.N * a.Ho * a.Wo * 7;
    const ZeroPixelsJob zp{(uint16_t*)out, row_mask, a.Cout, a.Ho * a.Wo, a.N * ceil_div(a.Cout, ZPX), fill_all};
    int32_t st = to_grid(A, nullptr, a.C, a.C, a.H, a.W, a.N, Hg, Wg, a.pad, a.pad, Cp, margin, w.grid_a, stream, BandMask{},
                         pack_job(Wt, nullptr, a.C, taps, a.Cout, a.C, Cp, 0, w.gwp), ZeroPlanesJob{}, zp);
    if (st) return st;
    if (Ck == 0) return ARD_OK;
    ConvMap cv{a.Ho * a.Wo, a.Wo, Hg * Wg, Wg, Cp, a.kw, Ck, a.Cout, nullptr, a.Cout, (const int*)d_keep, a.N * a.Ho * a.Wo, -1};
    return conv_grid_gemm(w.gwp, a.Cout, K, w.grid_a, (long)a.N * Hg * Wg + margin, cv, out, stream);
  }
  if (a.mode == ARD_CONV_FWD) {
    const int Cp = pad64(Ck), Hg = a.H + 2 * a.pad, Wg = a.W + 2 * a.pad, K = taps * Cp;
    int32_t st = ARD_OK;
    const PackJob pj = pack_job(Wt, (const int*)d_keep, a.C, taps, a.Cout, Ck, Cp, 0, w.gwp);
    BlockPlanJob bj{};
    int bn = 0;
    if (a.blk) {
      bn = block_fast_tile(a, w);
      if (!bn) return fail(ARD_EUNSUPPORTED, "block pattern outside the fast path");  // (callers test block_fast_tile first)
      bj.p = BlockPlan{a.N, a.Ho * a.Wo, a.bx, ceil_div(a.Ho * a.Wo, a.bx), ceil_div(a.C * taps, a.by), ceil_div(a.bx, bn), bn, taps,
                       Cp / 64, a.by / (64 * taps), taps * (Cp / 64)};
      bj.blk = a.blk;
      bj.tiles = bj.blocks = a.N * bj.p.RB * bj.p.tpb;
      bj.order = bj.tiles > 256 && bj.tiles <= kBlockOrderMaxTiles;  // (up to one tile per CU there is nothing to order)
      bj.pix = w.blk_pix, bj.kb_list = w.blk_kb, bj.kb_cnt = w.blk_cnt;
    }
    if (!(a.reuse & ARD_CONV_REUSE_A)) {
      // (the packed weights and the tile plan of a block pattern ride in the copy's launch)
      st = to_grid(A, d_keep, Ck, a.C, a.H, a.W, a.N, Hg, Wg, a.pad, a.pad, Cp, margin, w.grid_a, stream, BandMask{}, pj,
                   ZeroPlanesJob{}, ZeroPixelsJob{}, bj);
    } else {
      ARD_LAUNCH(pack_weights_grid_kernel, dim3((unsigned)pj.blocks), dim3(256), 0, stream, pj);
      ARD_LAUNCH_CHECK("pack_weights_grid_kernel");
      if (bj.blocks) {
        ARD_LAUNCH(block_plan_kernel, dim3((unsigned)bj.blocks), dim3(256), 0, stream, bj);
        ARD_LAUNCH_CHECK("block_plan_kernel");
      }
    }
    if (st) return st;
    if (a.blk) {
      const BlockPlan& bp = bj.p;
      const int tiles = bj.tiles;
      // bands of an even number of positions in planes of an even size: the tiles hold whole pairs of neighbours
      const int pairs = (a.bx % 2 == 0) && ((a.Ho * a.Wo) % 2 == 0);
      ConvMap cv{a.Ho * a.Wo, a.Wo, Hg * Wg, Wg, Cp, a.kw, tiles * bn, a.Cout, nullptr, a.Cout, w.blk_pix, a.N * a.Ho * a.Wo, -1, pairs};
      return conv_grid_gemm(w.gwp, a.Cout, K, w.grid_a, (long)a.N * Hg * Wg + margin, cv, out, stream, bn, w.blk_kb, w.blk_cnt,
                            bp.KB);
    }
    ConvMap cv{a.Ho * a.Wo, a.Wo, Hg * Wg, Wg, Cp, a.kw, a.N * a.Ho * a.Wo, a.Cout, nullptr, a.Cout, nullptr, 0, -1};
    return conv_grid_gemm(w.gwp, a.Cout, K, w.grid_a, (long)a.N * Hg * Wg + margin, cv, out, stream);
  }
  if (a.mode == ARD_CONV_BWD_DATA) {
    // dA = dY (bordered by k-1-pad) convolved with the reversed filter, contraction over (tap, co)
    const int ph = a.kh - 1 - a.pad, pw = a.kw - 1 - a.pad;
    const int Cp = pad64(a.Cout), Hg = a.Ho + 2 * ph, Wg = a.Wo + 2 * pw, K = taps * Cp;
    int32_t st = ARD_OK;
    const PackJob pj = pack_job(Wt, (const int*)d_keep, a.C, taps, Ck, a.Cout, Cp, 1, w.gwp);
    ZeroPlanesJob zj{};
    if (Ck < a.C && !a.kept_only) {
      const int hw = a.H * a.W;
      zj = ZeroPlanesJob{(uint16_t*)out, (const int*)d_keep, Ck, a.N, a.C, hw, (int)((hw % 8) == 0 && al16c(out)),
                         a.C * ceil_div(a.N, ZP_IMGS)};
    }
    if (!(a.reuse & ARD_CONV_REUSE_DY)) {
      st = to_grid(dYin, nullptr, a.Cout, a.Cout, a.Ho, a.Wo, a.N, Hg, Wg, ph, pw, Cp, margin, w.grid_y, stream, a.dy_mask, pj, zj);
    } else {
      ARD_LAUNCH(pack_weights_grid_kernel, dim3((unsigned)pj.blocks), dim3(256), 0, stream, pj);
      ARD_LAUNCH_CHECK("pack_weights_grid_kernel");
      if (zj.blocks) {
        ARD_LAUNCH(zero_dropped_planes_kernel, dim3((unsigned)zj.blocks), dim3(256), 0, stream, zj);
        ARD_LAUNCH_CHECK("zero_dropped_planes_kernel");
      }
    }
    if (st) return st;
    ConvMap cv{a.H * a.W, a.W, Hg * Wg, Wg, Cp, a.kw, a.N * a.H * a.W, a.C, (const int*)d_keep, Ck, nullptr, 0, -1};
    return conv_grid_gemm(w.gwp, Ck, K, w.grid_y, (long)a.N * Hg * Wg + margin, cv, out, stream);
  }
  // BWD_WEIGHT: contraction over the pixels of the input grid; dY sits on the same grid (top-left
  // aligned, zero elsewhere), the tap shifts the activation grid by (r*Wg + s) pixels.
  const int Cpa = pad64(Ck), Cpy = pad64(a.Cout), Hg = a.H + 2 * a.pad, Wg = a.W + 2 * a.pad;
  int32_t st = ARD_OK;
  if (!(a.reuse & ARD_CONV_REUSE_A))
    st = to_grid(A, d_keep, Ck, a.C, a.H, a.W, a.N, Hg, Wg, a.pad, a.pad, Cpa, margin, w.grid_a, stream);
  if (st) return st;
  // dY: bordered like the data gradient's grid when the filter preserves the size (then shared with it)
  const int ph = same ? a.kh - 1 - a.pad : 0, pw = same ? a.kw - 1 - a.pad : 0;
  const long y_shift = (long)ph * Wg + pw;  // pixels between the bordered grid's origin and dY(., 0, 0)
  if (!(a.reuse & ARD_CONV_REUSE_DY))
    st = to_grid(dYin, nullptr, a.Cout, a.Cout, a.Ho, a.Wo, a.N, Hg, Wg, ph, pw, Cpy, margin, w.grid_y, stream, a.dy_mask);
  if (st) return st;
  const int Kq = a.N * Hg * Wg, Nn = taps * Cpa;
  FastParams F{};
  F.A = w.grid_y + y_shift * Cpy;
  F.B = w.grid_a;
  F.lda = Cpy;
  F.ldb = Cpa;
  F.a_elems = ((long)a.N * Hg * Wg + margin - y_shift) * Cpy;
  F.b_elems = ((long)a.N * Hg * Wg + margin) * Cpa;
  F.am = axis_identity(Cpy);
  F.bn = axis_identity(Nn);
  F.k = axis_identity(Kq);
  F.alpha = 1.0f;
  F.part = w.gpart;
  // tile 256 x 128 (8 wavefronts) when there are enough output channels, else 128 x 128; the
  // contraction is split until every CU has a workgroup (two of the small ones), within the
  // room the workspace has for partial sums
  const bool big = a.Cout > 128;
  const int bm = big ? 256 : 128;
  const long cap = (long)w.gsplits * taps * pad64(a.C) / Nn;
  F.tiles_m = ceil_div(a.Cout, bm);
  F.tiles_n = ceil_div(Nn, 128);
  F.total_tiles = F.tiles_m * F.tiles_n;
  int splits = (big ? 256 : 512) / F.total_tiles;
  if (splits > cap) splits = (int)cap;
  const int steps = ceil_div(Kq, 64);
  if (splits > steps) splits = steps;
  if (splits < 1) splits = 1;
  F.splits = splits;
  F.M = a.Cout;
  F.N = Nn;
  F.cv = ConvMap{0, 0, Hg * Wg, Wg, Cpa, a.kw, 0, 0, nullptr, 0, nullptr, 0, -1};
  F.group_m = direct_group_m(F.total_tiles);
  st = big ? launch_direct_kernel<false, false, 256, 128, 8, 2>(F, direct_plain_grid(F.total_tiles), stream)
           : launch_direct_kernel<false, false, 128, 128, 4, 2>(F, direct_plain_grid(F.total_tiles), stream);
  if (st) return st;
  if ((long)a.Cout * taps * Ck >= (1L << 31)) return fail(ARD_ESHAPE, "weight gradient beyond 2^31 kept synapses");
  const int sum_blocks = (int)(((long)a.Cout * taps * Ck + 255) / 256);
  const int zero_blocks = Ck < a.C && !a.kept_only ? (int)(((long)a.Cout * a.C + 255) / 256) : 0;
  ARD_LAUNCH(wgrad_grid_reduce_kernel, dim3((unsigned)(sum_blocks + zero_blocks)), dim3(256), 0, stream, (const float*)w.gpart,
             (const int*)d_keep, Ck, splits, a.Cout, a.C, taps, Cpa, sum_blocks, (uint16_t*)out);
  ARD_LAUNCH_CHECK("wgrad_grid_reduce_kernel");
  return ARD_OK;
}

static int32_t conv_check(ConvArgs& a) {
  if (a.dtype != ARD_F32 && a.dtype != ARD_BF16) return fail(ARD_EDTYPE, "unknown dtype %d", a.dtype);
  if (a.N <= 0 || a.C <= 0 || a.H <= 0 || a.W <= 0 || a.Cout <= 0 || a.kh <= 0 || a.kw <= 0 || a.stride <= 0 || a.pad < 0)
    return fail(ARD_ESHAPE, "non-positive convolution size");
  if (a.H + 2 * a.pad < a.kh || a.W + 2 * a.pad < a.kw) return fail(ARD_ESHAPE, "kernel larger than the padded input");
  a.Ho = (a.H + 2 * a.pad - a.kh) / a.stride + 1;
  a.Wo = (a.W + 2 * a.pad - a.kw) / a.stride + 1;
  a.es = a.dtype == ARD_BF16 ? 2 : 4;
  if ((long)a.N * a.H * a.W > 0x7fffff00L || (long)a.N * a.Ho * a.Wo > 0x7fffff00L || (long)a.C * a.kh * a.kw > 0x7fffff00L)
    return fail(ARD_ESHAPE, "tensor too large for 32-bit position indices");
  return ARD_OK;
}


template <typename T>
static int32_t conv_run(const ConvArgs& a, double rate, const void* A, const void* Wt, const void* dYin, void* out,
                        uint8_t* d_mask, int32_t* d_keep, int32_t* d_count, int64_t* d_score, const ConvWs& w,
                        hipStream_t stream) {
  const int taps = a.kh * a.kw, ce = 16 / a.es;
  if (a.mode == ARD_CONV_SELECT) {
    if (!(rate >= 0.0 && rate <= 1.0)) return fail(ARD_EINVAL, "rate must be in [0,1] (got %g)", rate);
    if (!A || !d_mask || !d_keep) return fail(ARD_EINVAL, "SELECT needs A, d_mask and d_keep");
    if ((long)a.N * a.H * a.W > (1L << 24)) return fail(ARD_ESHAPE, "SELECT needs N*H*W <= 2^24");
    unsigned long long* score = d_score ? (unsigned long long*)d_score : w.score;
    int ysplit = ceil_div(2048, a.C);
    if (ysplit > a.N) ysplit = a.N;
    if (ysplit > kScoreParts) ysplit = kScoreParts;
    if (ysplit < 1) ysplit = 1;
    const int n_per_block = ceil_div(a.N, ysplit);
    const int parts = ceil_div(a.N, n_per_block);
    const int vec = ((a.H * a.W) % ce) == 0 && al16c(A);
    ARD_LAUNCH(channel_score_kernel<T>, dim3(a.C, parts), dim3(256), 0, stream, (const T*)A, a.N, a.C, a.H * a.W,
                       n_per_block, vec, w.score_part);
    ARD_LAUNCH_CHECK("channel_score_kernel");
    const int n_drop = (int)floor(rate * (double)a.C);
    if (a.C <= 4096)
      ARD_LAUNCH(channel_select_kernel<true>, dim3(1), dim3(1024), 0, stream, (const unsigned long long*)w.score_part, parts,
                         score, a.C, n_drop, d_mask, d_keep, d_count);
    else
      ARD_LAUNCH(channel_select_kernel<false>, dim3(1), dim3(1024), 0, stream, (const unsigned long long*)w.score_part, parts,
                         score, a.C, n_drop, d_mask, d_keep, d_count);
    ARD_LAUNCH_CHECK("channel_select_kernel");
    return ARD_OK;
  }
  if (a.mode == ARD_CONV_FWD_ROWS) {
    // d_keep lists the kept rows (output positions) of the input matrices, n * Ho*Wo + p, ascending;
    // d_mask is the same set as a 0/1 mask
    const long n_rows = (long)a.N * a.Ho * a.Wo;
    if (a.n_keep < 0 || a.n_keep > n_rows) return fail(ARD_EINVAL, "n_keep=%d outside 0..%ld", a.n_keep, n_rows);
    if (!A || !Wt || !out || !d_mask || (a.n_keep > 0 && !d_keep)) return fail(ARD_EINVAL, "FWD_ROWS needs A, Wt, out, d_mask and d_keep");
    if (a.reuse) return fail(ARD_EUNSUPPORTED, "FWD_ROWS builds its own grid");
    if (w.grid_a && !dev_knobs().no_fast) return conv_run_grid(a, A, Wt, nullptr, out, d_keep, d_mask, w, stream);
    // general path (fp32, strides): every position is computed, the dropped ones are zeroed afterwards
    ConvArgs full = a;
    full.mode = ARD_CONV_FWD;
    full.n_keep = a.C;
    int32_t st = conv_run<T>(full, 0.0, A, Wt, nullptr, out, nullptr, nullptr, nullptr, nullptr, w, stream);
    if (st) return st;
    ARD_LAUNCH(zero_dropped_pixels_kernel<T>, dim3(a.Cout, a.N), dim3(256), 0, stream, (T*)out, (const uint8_t*)d_mask, a.Cout,
               a.Ho * a.Wo);
    ARD_LAUNCH_CHECK("zero_dropped_pixels_kernel");
    return ARD_OK;
  }
  if (a.mode == ARD_CONV_BWD_DATA_ROWS || a.mode == ARD_CONV_BWD_WEIGHT_ROWS) {
    // gradients of FWD_ROWS: positions of dropped rows carry no gradient.  dY is copied once with those
    // positions zeroed, then the ordinary passes run over every position with every channel kept.
    if (!dYin || !d_mask || !out) return fail(ARD_EINVAL, "the row-pattern gradients need dYin, d_mask and out");
    // (the reuse flags mean what they mean for the ordinary gradients: the grid of A that FWD_ROWS left, the
    // masked grid of dY that BWD_DATA_ROWS left -- same mask, same layout)
    ARD_LAUNCH(iota_kernel, dim3(ceil_div(a.C, 256)), dim3(256), 0, stream, w.all_chan, a.C);
    ARD_LAUNCH_CHECK("iota_kernel");
    ConvArgs full = a;
    full.mode = a.mode == ARD_CONV_BWD_DATA_ROWS ? ARD_CONV_BWD_DATA : ARD_CONV_BWD_WEIGHT;
    full.n_keep = a.C;
    const void* dy_use = w.dy_rows;
    if (w.grid_a && !dev_knobs().no_fast) {
      // the pass copies dY into a channels-last grid anyway: that copy drops the positions (bands of one row)
      full.dy_mask = BandMask{(const uint8_t*)d_mask, a.Ho * a.Wo, 1, 0, 1};
      dy_use = dYin;
    } else {
      ARD_LAUNCH(mask_pixels_kernel<T>, dim3(a.Cout, a.N), dim3(256), 0, stream, (const T*)dYin, (const uint8_t*)d_mask, a.Cout,
                 a.Ho * a.Wo, (T*)w.dy_rows);
      ARD_LAUNCH_CHECK("mask_pixels_kernel");
    }
    return conv_run<T>(full, 0.0, A, Wt, dy_use, out, nullptr, w.all_chan, nullptr, nullptr, w, stream);
  }
  if (a.n_keep < 0 || a.n_keep > a.C) return fail(ARD_EINVAL, "n_keep=%d outside 0..%d", a.n_keep, a.C);
  if (a.n_keep > 0 && a.n_keep < a.C && !d_keep) return fail(ARD_EINVAL, "d_keep is required");
  if (!out) return fail(ARD_EINVAL, "null output pointer");
  const int Ck = a.n_keep;
  if (a.reuse) {
    const bool grid_path = Ck > 0 && w.grid_a;
    if (!grid_path) return fail(ARD_EUNSUPPORTED, "grid reuse needs the bf16 stride-1 path and at least one kept channel");
    if ((a.reuse & ARD_CONV_REUSE_A) && a.mode == ARD_CONV_BWD_DATA) return fail(ARD_EINVAL, "BWD_DATA has no grid of A to reuse");
    if ((a.reuse & ARD_CONV_REUSE_DY) && a.mode == ARD_CONV_FWD) return fail(ARD_EINVAL, "FWD has no grid of dY to reuse");
    if ((a.reuse & ARD_CONV_REUSE_DY) && a.mode == ARD_CONV_BWD_WEIGHT && !(a.kh - 1 == 2 * a.pad && a.kw - 1 == 2 * a.pad))
      return fail(ARD_EUNSUPPORTED, "the weight gradient shares dY's grid with the data gradient only for k - 1 = 2 pad");
    if (dev_knobs().no_fast) {
      // (development switch: every pass runs on the general engine, which builds no grid; nothing to share)
      ConvArgs plain = a;
      plain.reuse = 0;
      return conv_run<T>(plain, rate, A, Wt, dYin, out, d_mask, d_keep, d_count, d_score, w, stream);
    }
  }
  if (Ck > 0 && w.grid_a && a.mode >= ARD_CONV_FWD && a.mode <= ARD_CONV_BWD_WEIGHT && !dev_knobs().no_fast &&
      (!a.blk || (a.mode == ARD_CONV_FWD && block_fast_tile(a, w)))) {
    if (a.mode == ARD_CONV_FWD && (!A || !Wt)) return fail(ARD_EINVAL, "FWD needs A and Wt");
    if (a.mode == ARD_CONV_BWD_DATA && (!dYin || !Wt)) return fail(ARD_EINVAL, "BWD_DATA needs dYin and Wt");
    if (a.mode == ARD_CONV_BWD_WEIGHT && (!dYin || !A)) return fail(ARD_EINVAL, "BWD_WEIGHT needs dYin and A");
    return conv_run_grid(a, A, Wt, dYin, out, d_keep, nullptr, w, stream);
  }

  if (a.mode == ARD_CONV_FWD) {
    if (!A || !Wt) return fail(ARD_EINVAL, "FWD needs A and Wt");
    if (Ck == 0) return fill_matrix(a.dtype, out, (long)a.N * a.Cout * a.Ho * a.Wo, 0.0f, stream);
    const long total = (long)a.Cout * taps * Ck;
    ARD_LAUNCH(pack_weights_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const T*)Wt, (const int*)d_keep, a.C, taps, a.Cout, Ck, 0, (T*)w.wp);
    ARD_LAUNCH_CHECK("pack_weights_kernel");
    ConvGemmParams P{};
    P.K = taps * Ck;
    P.Wp = Operand{w.wp, P.K, axis_identity(a.Cout), (P.K % ce) == 0};
    P.src = A;
    P.g = ConvGeom{a.N, a.C, a.H, a.W, a.Ho, a.Wo, a.kh, a.kw, a.stride, a.pad, a.pad, Ck, d_keep};
    if (a.blk) {
      P.g.blk = a.blk;
      P.g.bx = a.bx, P.g.by = a.by;
      P.g.RB = ceil_div(a.Ho * a.Wo, a.bx), P.g.CB = ceil_div(a.C * taps, a.by);
    }
    P.M = a.Cout;
    P.Ncols = (long)a.N * a.Ho * a.Wo;
    P.C.p = out;
    P.C.rm = axis_identity(a.Cout);
    P.C.cn = axis_identity((int)P.Ncols);
    P.C.plane = a.Ho * a.Wo;
    P.C.img_stride = (long)a.Cout * a.Ho * a.Wo;
    P.C.alpha = 1.0f;
    P.tiles_n = ceil_div((int)P.Ncols, 128);
    long blocks = (long)ceil_div(P.M, 128) * P.tiles_n;
    ARD_LAUNCH((conv_gemm_kernel<T, 128, 128, 2, 2>), dim3((unsigned)blocks), dim3(256), 0, stream, P);
    ARD_LAUNCH_CHECK("conv_gemm_kernel");
    return ARD_OK;
  }

  if (a.mode == ARD_CONV_BWD_DATA) {
    if (!dYin || !Wt) return fail(ARD_EINVAL, "BWD_DATA needs dYin and Wt");
    if (a.stride != 1) return fail(ARD_EUNSUPPORTED, "BWD_DATA is built for stride 1 only (got %d)", a.stride);
    if (a.kh - 1 - a.pad < 0 || a.kw - 1 - a.pad < 0) return fail(ARD_EUNSUPPORTED, "BWD_DATA needs pad <= k-1");
    if (Ck == 0) return fill_matrix(a.dtype, out, (long)a.N * a.C * a.H * a.W, 0.0f, stream);
    const long total = (long)Ck * taps * a.Cout;
    ARD_LAUNCH(pack_weights_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const T*)Wt, (const int*)d_keep, a.C, taps, Ck, a.Cout, 1, (T*)w.wp);
    ARD_LAUNCH_CHECK("pack_weights_kernel");
    ConvGemmParams P{};
    P.K = taps * a.Cout;
    P.Wp = Operand{w.wp, P.K, axis_identity(Ck), (P.K % ce) == 0};
    P.src = dYin;
    P.g = ConvGeom{a.N, a.Cout, a.Ho, a.Wo, a.H, a.W, a.kh, a.kw, 1, a.kh - 1 - a.pad, a.kw - 1 - a.pad, a.Cout, nullptr};
    if (a.blk) {
      P.Wp.vec = (a.Cout % ce) == 0;  // the contraction is walked tap by tap: every tap must start on a chunk
      P.g.blk = a.blk;
      P.g.bx = a.bx, P.g.by = a.by;
      P.g.RB = ceil_div(a.Ho * a.Wo, a.bx), P.g.CB = ceil_div(a.C * taps, a.by);
    }
    P.M = Ck;
    P.Ncols = (long)a.N * a.H * a.W;
    P.C.p = out;
    P.C.rm = axis_list(d_keep, Ck, a.C);
    P.C.cn = axis_identity((int)P.Ncols);
    P.C.plane = a.H * a.W;
    P.C.img_stride = (long)a.C * a.H * a.W;
    P.C.fill = a.kept_only ? 0 : 1;
    P.C.alpha = 1.0f;
    P.tiles_n = ceil_div((int)P.Ncols, 128);
    long blocks = (long)ceil_div(P.M, 128) * P.tiles_n;
    if (a.blk) {
      ARD_LAUNCH((conv_bwd_data_blocks_kernel<T, 128, 128, 2, 2>), dim3((unsigned)blocks), dim3(256), 0, stream, P);
      ARD_LAUNCH_CHECK("conv_bwd_data_blocks_kernel");
      return ARD_OK;
    }
    ARD_LAUNCH((conv_gemm_kernel<T, 128, 128, 2, 2>), dim3((unsigned)blocks), dim3(256), 0, stream, P);
    ARD_LAUNCH_CHECK("conv_gemm_kernel");
    return ARD_OK;
  }

  if (a.mode == ARD_CONV_BWD_WEIGHT) {
    if (!dYin || !A) return fail(ARD_EINVAL, "BWD_WEIGHT needs dYin and A");
    if (Ck == 0) return fill_matrix(a.dtype, out, (long)a.Cout * a.C * taps, 0.0f, stream);
    ARD_LAUNCH(rank_from_keep_kernel, dim3(1), dim3(1024), 0, stream, (const int*)d_keep, Ck, a.C, w.rank);
    ARD_LAUNCH_CHECK("rank_from_keep_kernel");
    ConvWgradParams P{};
    P.dY = dYin;
    P.A = A;
    P.g = ConvGeom{a.N, a.C, a.H, a.W, a.Ho, a.Wo, a.kh, a.kw, a.stride, a.pad, a.pad, Ck, d_keep};
    if (a.blk) {
      P.g.blk = a.blk;
      P.g.bx = a.bx, P.g.by = a.by;
      P.g.RB = ceil_div(a.Ho * a.Wo, a.bx), P.g.CB = ceil_div(a.C * taps, a.by);
    }
    P.part = w.part;
    P.Cout = a.Cout;
    P.Nn = Ck * taps;
    P.K = (long)a.N * a.Ho * a.Wo;
    const int hw = a.Ho * a.Wo;
    P.dy_vec = (hw % ce) == 0 && al16c(dYin);
    const int bk = 8 * ce;
    int splits = w.splits;
    long per = (P.K + splits - 1) / splits;
    per = (per + bk - 1) / bk * bk;
    splits = (int)((P.K + per - 1) / per);
    P.k_per_split = (int)per;
    P.tiles_n = ceil_div(P.Nn, 128);
    dim3 grid((unsigned)(ceil_div(P.Cout, 128) * P.tiles_n), (unsigned)splits);
    ARD_LAUNCH((conv_wgrad_kernel<T, 128, 128, 2, 2>), grid, dim3(256), 0, stream, P);
    ARD_LAUNCH_CHECK("conv_wgrad_kernel");
    const long total = (long)a.Cout * a.C * taps;
    ARD_LAUNCH(conv_wgrad_reduce_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const float*)w.part, (const int*)w.rank, splits, a.Cout, a.C, taps, P.Nn, a.kept_only, (T*)out);
    ARD_LAUNCH_CHECK("conv_wgrad_reduce_kernel");
    return ARD_OK;
  }
  return fail(ARD_EINVAL, "unknown conv mode %d", a.mode);
}

}  // namespace ard

using namespace ard;

extern "C" int32_t ard_conv_out_size(int32_t in, int32_t k, int32_t stride, int32_t pad) {
  if (in <= 0 || k <= 0 || stride <= 0 || pad < 0) return fail(ARD_ESHAPE, "non-positive convolution size");
  if (in + 2 * pad < k) return fail(ARD_ESHAPE, "kernel larger than the padded input");
  return (in + 2 * pad - k) / stride + 1;
}

extern "C" size_t ard_conv_workspace_bytes(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t Cout,
                                           int32_t kh, int32_t kw, int32_t stride, int32_t pad) {
  ConvArgs a{0, dtype, N, C, H, Wd, Cout, kh, kw, stride, pad, 0, 0, 0, 0, 0};
  if (conv_check(a)) return 0;
  return conv_ws_layout(nullptr, a).total;
}

extern "C" int32_t ard_conv_fwd_blocks(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t Cout, int32_t kh,
                                       int32_t kw, int32_t stride, int32_t pad, int32_t x, int32_t y, const void* A,
                                       const void* Wt, const uint8_t* d_block_keep, void* out, void* ws, size_t ws_bytes,
                                       void* stream) {
  BatchSuspend not_recorded;
  ConvArgs a{ARD_CONV_FWD, dtype, N, C, H, Wd, Cout, kh, kw, stride, pad, C, 0, 0, 0, 0, d_block_keep, x, y};
  int32_t st = conv_check(a);
  if (st) return st;
  if (x < 1 || y < 0) return fail(ARD_EINVAL, "block size must be positive (y = 0: the whole width)");
  if (y == 0) a.by = C * kh * kw;
  if (!A || !Wt || !d_block_keep || !out) return fail(ARD_EINVAL, "null pointer");
  ConvWs w = conv_ws_layout((char*)ws, a);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16)
    return conv_run<uint16_t>(a, 0.0, A, Wt, nullptr, out, nullptr, nullptr, nullptr, nullptr, w, (hipStream_t)stream);
  return conv_run<float>(a, 0.0, A, Wt, nullptr, out, nullptr, nullptr, nullptr, nullptr, w, (hipStream_t)stream);
}

extern "C" int32_t ard_conv_bwd_blocks(int32_t mode, int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t Cout,
                                       int32_t kh, int32_t kw, int32_t stride, int32_t pad, int32_t x, int32_t y,
                                       const void* A, const void* Wt, const void* dYin, const uint8_t* d_block_keep, void* out,
                                       void* ws, size_t ws_bytes, void* stream) {
  BatchSuspend not_recorded;
  if (mode != ARD_CONV_BWD_DATA && mode != ARD_CONV_BWD_WEIGHT)
    return fail(ARD_EINVAL, "mode must be ARD_CONV_BWD_DATA or ARD_CONV_BWD_WEIGHT (got %d)", mode);
  ConvArgs a{mode, dtype, N, C, H, Wd, Cout, kh, kw, stride, pad, C, 0, 0, 0, 0, d_block_keep, x, y};
  int32_t st = conv_check(a);
  if (st) return st;
  if (x < 1 || y < 0) return fail(ARD_EINVAL, "block size must be positive (y = 0: the whole width)");
  if (y == 0) a.by = C * kh * kw;
  if (!dYin || !d_block_keep || !out) return fail(ARD_EINVAL, "null pointer");
  if (mode == ARD_CONV_BWD_WEIGHT && !A) return fail(ARD_EINVAL, "BWD_WEIGHT needs A");
  if (mode == ARD_CONV_BWD_DATA) {
    if (!Wt) return fail(ARD_EINVAL, "BWD_DATA needs Wt");
    if (stride != 1) return fail(ARD_EUNSUPPORTED, "BWD_DATA is built for stride 1 only (got %d)", stride);
    if (kh - 1 - pad < 0 || kw - 1 - pad < 0) return fail(ARD_EUNSUPPORTED, "BWD_DATA needs pad <= k-1");
  }
  ConvWs w = conv_ws_layout((char*)ws, a);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  hipStream_t s = (hipStream_t)stream;
  // every channel is kept: the passes take the identity list
  ARD_LAUNCH(iota_kernel, dim3(ceil_div(C, 256)), dim3(256), 0, s, w.all_chan, C);
  ARD_LAUNCH_CHECK("iota_kernel");
  // Blocks of whole channels (y a multiple of kh*kw), not too many of them: column block cb is the channel
  // range [cb*cpb, (cb+1)*cpb) over all taps, and whether a term of those channels counts depends on the band
  // of the output position alone.  Per column block: dY copied with the positions of its dropped bands zeroed,
  // then the ordinary gradient pass (whichever engine takes the shape) with that channel range as the kept
  // list, writing its channels' part of the output only.  Work is not skipped, but the passes are the fast ones.
  const int taps = kh * kw;
  const int CB = ceil_div(C * taps, a.by), RB = ceil_div(a.Ho * a.Wo, a.bx);
  if (a.by % taps == 0 && CB <= 16 && !(mode == ARD_CONV_BWD_DATA && stride != 1)) {
    const int cpb = a.by / taps;
    for (int cb = 0; cb < CB; ++cb) {
      ConvArgs g = a;
      g.blk = nullptr;
      g.kept_only = 1;
      g.n_keep = (cb + 1) * cpb <= C ? cpb : C - cb * cpb;
      const void* dy_use = w.dy_rows;
      if (w.grid_a && !dev_knobs().no_fast) {
        // the pass copies dY into a channels-last grid anyway: that copy applies the mask
        g.dy_mask = BandMask{d_block_keep, RB, CB, cb, a.bx};
        dy_use = dYin;
      } else {
        if (dtype == ARD_BF16)
          ARD_LAUNCH(mask_bands_kernel<uint16_t>, dim3(Cout, N), dim3(256), 0, s, (const uint16_t*)dYin, d_block_keep, RB, CB, cb,
                     a.bx, Cout, a.Ho * a.Wo, (uint16_t*)w.dy_rows);
        else
          ARD_LAUNCH(mask_bands_kernel<float>, dim3(Cout, N), dim3(256), 0, s, (const float*)dYin, d_block_keep, RB, CB, cb, a.bx,
                     Cout, a.Ho * a.Wo, (float*)w.dy_rows);
        ARD_LAUNCH_CHECK("mask_bands_kernel");
      }
      st = dtype == ARD_BF16 ? conv_run<uint16_t>(g, 0.0, A, Wt, dy_use, out, nullptr, w.all_chan + cb * cpb, nullptr, nullptr, w, s)
                             : conv_run<float>(g, 0.0, A, Wt, dy_use, out, nullptr, w.all_chan + cb * cpb, nullptr, nullptr, w, s);
      if (st) return st;
    }
    return ARD_OK;
  }
  if (dtype == ARD_BF16)
    return conv_run<uint16_t>(a, 0.0, A, Wt, dYin, out, nullptr, w.all_chan, nullptr, nullptr, w, s);
  return conv_run<float>(a, 0.0, A, Wt, dYin, out, nullptr, w.all_chan, nullptr, nullptr, w, s);
}

extern "C" int32_t ard_fmap_drop_conv(int32_t mode, int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd,
                                      int32_t Cout, int32_t kh, int32_t kw, int32_t stride, int32_t pad, double rate,
                                      int32_t n_keep, const void* A, const void* Wt, const void* dYin, void* out,
                                      uint8_t* d_mask, int32_t* d_keep, int32_t* d_count, int64_t* d_score, void* ws,
                                      size_t ws_bytes, void* stream) {
  BatchSuspend not_recorded;  // this entry point's kernels depend on each other: never part of a grouped launch
  if (mode < 0 || (mode & ~(0xff | ARD_CONV_REUSE_A | ARD_CONV_REUSE_DY))) return fail(ARD_EINVAL, "unknown conv mode bits 0x%x", mode);
  ConvArgs a{mode & 0xff, dtype, N, C, H, Wd, Cout, kh, kw, stride, pad, n_keep, 0, 0, 0, mode & (ARD_CONV_REUSE_A | ARD_CONV_REUSE_DY)};
  if (a.reuse && a.mode == ARD_CONV_SELECT) return fail(ARD_EINVAL, "SELECT builds no grid");
  int32_t st = conv_check(a);
  if (st) return st;
  ConvWs w = conv_ws_layout((char*)ws, a);
  if (!ws || ws_bytes < w.total)
    return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16)
    return conv_run<uint16_t>(a, rate, A, Wt, dYin, out, d_mask, d_keep, d_count, d_score, w, (hipStream_t)stream);
  return conv_run<float>(a, rate, A, Wt, dYin, out, d_mask, d_keep, d_count, d_score, w, (hipStream_t)stream);
}
