// Region-level sensitivity prediction and the sensitivity-aware dropout patterns of the CNN variant
// (Sections 5.1, 5.2.1, 5.2.2): which rows (output positions) or blocks of a layer's input matrix are
// dropped in this iteration.
//
// The input matrix of an image has one row per output position p = oh * Wo + ow and one column per
// (c, kh, kw), q = (c * KH + kh) * KW + kw, entry = zero-padded A[c, oh*s + kh - pad, ow*s + kw - pad];
// it is never built: the kernels address the activations directly.  It is cut into x-by-y regions
// (row band rb = p / x, column block cb = q / y, edge regions clipped).
//
// Every random draw is a 32-bit word of the SplitMix64 finaliser chained over
// (seed, iteration, stream, index) -- stateless and integer only, so the masks are reproducible bit for
// bit on any number of devices (the host folds the first three links, the kernels add the index).
#include <math.h>

#include "common.hpp"

namespace ard {

static __host__ __device__ inline uint64_t sens_mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}
constexpr uint64_t kSensGolden = 0x9E3779B97F4A7C15ULL;
enum { SENS_STREAM_SAMPLE = 0x5E01, SENS_STREAM_ROWS = 0x5E02, SENS_STREAM_BLOCKS = 0x5E03 };

static uint64_t sens_prefix(uint64_t seed, uint64_t iter, uint32_t stream) {
  uint64_t h = sens_mix64(seed + kSensGolden);
  h = sens_mix64((h ^ iter) + kSensGolden);
  return sens_mix64((h ^ (uint64_t)stream) + kSensGolden);
}
static __device__ __forceinline__ uint32_t sens_draw(uint64_t prefix, uint64_t index) {
  return (uint32_t)(sens_mix64((prefix ^ index) + kSensGolden) >> 32);
}
static uint64_t sens_threshold(double p) {
  double q = floor(p * 4294967296.0);
  if (q < 0) q = 0;
  if (q > 4294967296.0) q = 4294967296.0;
  return (uint64_t)q;
}

struct SensGeom {
  int N, C, H, W, KH, KW, stride, pad, Ho, Wo;
  int rows, cols;  // of the input matrix of one image
  int x, y, RB, CB;
};

// One workgroup per (image, region): s = max(1, k * size / 1000) draws with replacement, count of the
// drawn entries above the threshold (Section 5.1, steps 2 and 3).
template <typename T>
__global__ __launch_bounds__(256) void sens_predict_kernel(const T* A, SensGeom g, int k_permille, int t_permille, float thr,
                                                           uint64_t prefix, int* count, int* samples, uint8_t* sens) {
  __shared__ int wave_cnt[4];
  const int region = blockIdx.x;  // (image * RB + rb) * CB + cb
  const int cb = region % g.CB, rb = (region / g.CB) % g.RB, n = region / (g.CB * g.RB);
  const int r0 = rb * g.x, q0 = cb * g.y;
  const int h = min(g.x, g.rows - r0), w = min(g.y, g.cols - q0);
  const int size = h * w;
  int s = (int)(((long)k_permille * size) / 1000);
  if (s < 1) s = 1;
  const T* img = A + (long)n * g.C * g.H * g.W;
  const int taps = g.KH * g.KW;
  int c = 0;
  for (int j = threadIdx.x; j < s; j += 256) {
    const uint32_t u = sens_draw(prefix, (uint64_t)region * 65536u + (uint64_t)j);
    const int e = (int)(((uint64_t)u * (uint64_t)size) >> 32);
    const int p = r0 + e / w, q = q0 + e % w;
    const int oh = p / g.Wo, ow = p - oh * g.Wo;
    const int ch = q / taps, tap = q - ch * taps;
    const int kh = tap / g.KW, kw = tap - kh * g.KW;
    const int ih = oh * g.stride + kh - g.pad, iw = ow * g.stride + kw - g.pad;
    float v = 0.0f;  // the zero border of the input matrix
    if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) v = ElemTraits<T>::to_f32(img[((long)ch * g.H + ih) * g.W + iw]);
    c += v > thr ? 1 : 0;
  }
  for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off, 64);
  if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int tot = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    count[region] = tot;
    samples[region] = s;
    sens[region] = (1000L * tot >= (long)t_permille * s) ? 1 : 0;
  }
}

// The same prediction with the region's geometry tabulated in LDS once per workgroup: per column of the
// region its channel's offset in the image and its tap (kh, kw), per row of the band its top-left input
// position.  A draw is then the mixer, one division by the region's width, two LDS reads and the gather.
// Same draws, same elements, same counts as sens_predict_kernel (bit for bit); used when the table fits
// (region width <= kSensLutCols, channel offsets below 2^24, taps below 16).
constexpr int kSensLutCols = 8192, kSensLutRows = 1024;
template <typename T>
__global__ __launch_bounds__(256) void sens_predict_lut_kernel(const T* A, SensGeom g, int k_permille, int t_permille, float thr,
                                                               uint64_t prefix, FastDiv div_w, int* count, int* samples,
                                                               uint8_t* sens) {
  extern __shared__ int sens_lut[];  // [w] columns, then [h] rows
  __shared__ int wave_cnt[4];
  const int region = blockIdx.x;  // (image * RB + rb) * CB + cb
  const int cb = region % g.CB, rb = (region / g.CB) % g.RB, n = region / (g.CB * g.RB);
  const int r0 = rb * g.x, q0 = cb * g.y;
  const int h = min(g.x, g.rows - r0), w = min(g.y, g.cols - q0);
  const int size = h * w;
  int s = (int)(((long)k_permille * size) / 1000);
  if (s < 1) s = 1;
  const int taps = g.KH * g.KW;
  int* col_lut = sens_lut;
  int* row_lut = sens_lut + w;
  for (int i = threadIdx.x; i < w; i += 256) {
    const int q = q0 + i;
    const int ch = q / taps, tap = q - ch * taps;
    const int kh = tap / g.KW, kw = tap - kh * g.KW;
    col_lut[i] = (ch * g.H * g.W) | (kh << 24) | (kw << 28);
  }
  for (int i = threadIdx.x; i < h; i += 256) {
    const int p = r0 + i;
    const int oh = p / g.Wo, ow = p - oh * g.Wo;
    // input position of tap (0, 0), biased by the padding so that both halves are non-negative
    row_lut[i] = (oh * g.stride) | ((ow * g.stride) << 16);
  }
  __syncthreads();
  const T* img = A + (long)n * g.C * g.H * g.W;
  int c = 0;
  for (int j = threadIdx.x; j < s; j += 256) {
    const uint32_t u = sens_draw(prefix, (uint64_t)region * 65536u + (uint64_t)j);
    const uint32_t e = (uint32_t)(((uint64_t)u * (uint64_t)size) >> 32);
    const uint32_t r = fdiv(e, div_w), q = e - r * (uint32_t)w;
    const int ci = col_lut[q], ri = row_lut[r];
    const int ih = (ri & 0xffff) + ((ci >> 24) & 15) - g.pad, iw = (ri >> 16) + ((ci >> 28) & 15) - g.pad;
    float v = 0.0f;  // the zero border of the input matrix
    if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) v = ElemTraits<T>::to_f32(img[(ci & 0xffffff) + ih * g.W + iw]);
    c += v > thr ? 1 : 0;
  }
  for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off, 64);
  if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int tot = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    count[region] = tot;
    samples[region] = s;
    sens[region] = (1000L * tot >= (long)t_permille * s) ? 1 : 0;
  }
}

// The prediction once more, with the footprint of the workgroup's regions in the activations brought into LDS
// first: the draws of a region fall on a few input rows of its channels (config 5, a band of 8 positions:
// 4 rows x 28 x 256 channels for 5529 draws), and a gather from memory costs a whole cache-line transaction per
// draw (69 M of them made the pass take 460 us) where the copy is a few coalesced 16-byte loads per thread.
// Same draws, same elements, same counts.  Needs planes that are whole numbers of 16-byte pieces (then every
// channel's run starts at the same offset within a piece); the host checks it.
struct SensStage {
  int nrow_max, chp;  // input rows a workgroup's bands can touch; elements reserved per channel (a multiple of the piece)
  FastDiv div_taps, div_kw, div_wo;
  int G, RBG;         // consecutive row bands (of one image and column block) per workgroup; groups per image
};
template <typename T>
__global__ __launch_bounds__(256) void sens_predict_staged_kernel(const T* A, SensGeom g, SensStage sg, int k_permille,
                                                                  int t_permille, float thr, uint64_t prefix, FastDiv div_w,
                                                                  int* count, int* samples, uint8_t* sens) {
  constexpr int CE = ElemTraits<T>::CE;  // elements per 16-byte piece
  extern __shared__ uint4 sens_stage_lds[];
  __shared__ int wave_cnt[4];
  // workgroup = (image, group of G row bands, column block)
  const int cb = blockIdx.x % g.CB, rbg = (blockIdx.x / g.CB) % sg.RBG, n = blockIdx.x / (g.CB * sg.RBG);
  const int rb_first = rbg * sg.G, nb = min(sg.G, g.RB - rb_first);
  const int r0 = rb_first * g.x, q0 = cb * g.y;
  const int h = min(nb * g.x, g.rows - r0), w = min(g.y, g.cols - q0);  // rows of the group, columns of the block
  const int taps = g.KH * g.KW;
  // footprint: channels [ch_lo, ch_hi], input rows [ih_lo, ih_hi] (clipped to the image), all columns
  const int ch_lo = q0 / taps, ch_hi = (q0 + w - 1) / taps;
  const int oh_lo = r0 / g.Wo, oh_hi = (r0 + h - 1) / g.Wo;
  const int ih_lo = max(0, oh_lo * g.stride - g.pad), ih_hi = min(g.H - 1, oh_hi * g.stride - g.pad + g.KH - 1);
  const int nch = ch_hi - ch_lo + 1;
  const int run0 = ih_lo * g.W, run = max(0, ih_hi - ih_lo + 1) * g.W;  // elements of a channel's plane that are staged
  const int off = run0 % CE;                                           // the run's offset within its first piece
  const int pieces = run > 0 ? (off + run + CE - 1) / CE : 0;           // 16-byte pieces per channel
  // What a draw needs of an element is one bit (above the threshold or not): the copy keeps one byte per
  // 16-byte piece, bit e = element e of the piece.  The footprint shrinks 16 (bf16) or 32 (fp32) times, so
  // the CU holds as many workgroups as its wavefront slots allow and many bands can share one copy.
  uint8_t* stage = reinterpret_cast<uint8_t*>(sens_stage_lds);
  const int chpb = sg.chp / CE;                               // bytes per channel (chp is a multiple of the piece)
  const int nch_max = min(g.C, (g.y + taps - 2) / taps + 1);  // channels a column block can touch
  int* col_lut = reinterpret_cast<int*>(stage + (((size_t)chpb * nch_max + 3) & ~(size_t)3));
  int* row_lut = col_lut + w;
  const T* img = A + (long)n * g.C * g.H * g.W;
  // consecutive threads take consecutive pieces, running on from one channel into the next
  for (int i = threadIdx.x; i < nch * pieces; i += 256) {
    const int c = i / pieces, pc = i - c * pieces;
    const T* src = img + (long)(ch_lo + c) * g.H * g.W + (run0 - off) + pc * CE;
    const uint4 v = *reinterpret_cast<const uint4*>(src);
    T el[CE];
    *reinterpret_cast<uint4*>(el) = v;
    unsigned bits = 0;
#pragma unroll
    for (int e = 0; e < CE; ++e) bits |= (ElemTraits<T>::to_f32(el[e]) > thr ? 1u : 0u) << e;
    stage[(size_t)c * chpb + pc] = (uint8_t)bits;
  }
  const int border_above = 0.0f > thr ? 1 : 0;  // the zero border of the input matrix
  for (int i = threadIdx.x; i < w; i += 256) {
    const int q = q0 + i;
    const int ch = (int)fdiv((uint32_t)q, sg.div_taps), tap = q - ch * taps;
    const int kh = (int)fdiv((uint32_t)tap, sg.div_kw), kw = tap - kh * g.KW;
    col_lut[i] = ((ch - ch_lo) * sg.chp) | (kh << 24) | (kw << 28);
  }
  for (int i = threadIdx.x; i < h; i += 256) {
    const int p = r0 + i;
    const int oh = (int)fdiv((uint32_t)p, sg.div_wo), ow = p - oh * g.Wo;
    row_lut[i] = (oh * g.stride) | ((ow * g.stride) << 16);
  }
  __syncthreads();
  for (int gi = 0; gi < nb; ++gi) {
    const int region = ((n * g.RB) + rb_first + gi) * g.CB + cb;
    const int rr0 = gi * g.x;                   // first row of this band within the group
    const int hb = min(g.x, h - rr0);
    const int size = hb * w;
    int s = (int)(((long)k_permille * size) / 1000);
    if (s < 1) s = 1;
    int c = 0;
    // (four draws in flight per thread: their table and LDS reads overlap)
#pragma unroll 4
    for (int j = threadIdx.x; j < s; j += 256) {
      const uint32_t u = sens_draw(prefix, (uint64_t)region * 65536u + (uint64_t)j);
      const uint32_t e = (uint32_t)(((uint64_t)u * (uint64_t)size) >> 32);
      const uint32_t r = fdiv(e, div_w), q = e - r * (uint32_t)w;
      const int ci = col_lut[q], ri = row_lut[rr0 + r];
      const int ih = (ri & 0xffff) + ((ci >> 24) & 15) - g.pad, iw = (ri >> 16) + ((ci >> 28) & 15) - g.pad;
      int above = border_above;
      if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
        const int idx = (ci & 0xffffff) + off + (ih - ih_lo) * g.W + iw;  // element within the staged channels
        above = (stage[idx / CE] >> (idx % CE)) & 1;
      }
      c += above;
    }
    for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o, 64);
    if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
      const int tot = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
      count[region] = tot;
      samples[region] = s;
      sens[region] = (1000L * tot >= (long)t_permille * s) ? 1 : 0;
    }
    __syncthreads();  // (wave_cnt is reused by the next band)
  }
}

// Row-based pattern (Section 5.2.1): global row g = image * rows + p is dropped iff its draw is below the
// possibility of its band (m if sensitive, n otherwise); mask (1 = kept) and ascending kept list by
// ballot + mbcnt compaction.  A workgroup takes `chunk` consecutive rows.  Where its part of the kept list
// starts is the number of kept rows before its chunk.  No scratch memory and no hand-over between
// workgroups: with a mask, a first launch (phase 0) writes it and the second (phase 1) counts its ones
// before the chunk with 16-byte loads; without one (phase 2, a single launch) the workgroup recounts the
// rows before its chunk -- a draw is a pure function of the row.
__global__ __launch_bounds__(1024) void sens_row_pattern_kernel(const uint8_t* sens, int n_rows_total, int rows, int x, int RB,
                                                               int CB, uint64_t tm, uint64_t tn, uint64_t prefix, int chunk,
                                                               int phase, uint8_t* mask, int* keep, int* count) {
  __shared__ int wave_tot[16];
  __shared__ int running_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int start = blockIdx.x * chunk, end = min(n_rows_total, start + chunk);
  auto row_kept = [&](int gr) {
    const int n = gr / rows, p = gr - n * rows;
    const bool sv = sens[((long)n * RB + p / x) * CB] != 0;  // (regions span the width: CB = 1)
    return !((uint64_t)sens_draw(prefix, (uint64_t)gr) < (sv ? tm : tn));
  };
  if (phase == 0) {
    for (int gr = start + tid; gr < end; gr += 1024) mask[gr] = row_kept(gr) ? 1 : 0;
    return;
  }
  int before = 0;
  if (phase == 1) {
    // ones of mask[0, start): start is a multiple of 1024, the mask 16-byte aligned (host checks)
    const uint4* m16 = reinterpret_cast<const uint4*>(mask);
    for (int i = tid; i < start / 16; i += 1024) {
      const uint4 v = m16[i];
      before += __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
    }
  } else {
    for (int gr = tid; gr < start; gr += 1024) before += row_kept(gr) ? 1 : 0;
  }
  for (int off = 32; off > 0; off >>= 1) before += __shfl_down(before, off, 64);
  if (lane == 0) wave_tot[wave] = before;
  __syncthreads();
  if (tid == 0) {
    int t = 0;
    for (int w = 0; w < 16; ++w) t += wave_tot[w];
    running_s = t;
  }
  __syncthreads();
  for (int base = start; base < end; base += 1024) {
    const int gr = base + tid;
    bool kept = false;
    if (gr < end) kept = phase == 1 ? mask[gr] != 0 : row_kept(gr);
    const unsigned long long bal = __ballot(kept);
    const int r = __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int before_me = running_s, total = 0;
    for (int w = 0; w < 16; ++w) {
      const int t = wave_tot[w];
      if (w < wave) before_me += t;
      total += t;
    }
    if (kept && keep) keep[before_me + r] = gr;
    __syncthreads();
    if (tid == 0) running_s += total;
    __syncthreads();
  }
  if (tid == 0 && count && end == n_rows_total) *count = running_s;
}

// Block-based pattern (Section 5.2.2): one workgroup per (image, row band).  Balancing: S = mean number
// of sensitive blocks per band of this image, rounded half up; the S blocks of the band with the
// largest share count / samples (compared exactly by cross-multiplication, ties to the lower block)
// are the sensitive ones.  Then every block is dropped iff its draw is below m (sensitive) or n.
__global__ __launch_bounds__(256) void sens_block_pattern_kernel(const int* count, const int* samples, const uint8_t* sens,
                                                                 int RB, int CB, int balance, uint64_t tm, uint64_t tn,
                                                                 uint64_t prefix, uint8_t* sens_out, uint8_t* block_keep) {
  __shared__ int wave_sum[4];
  __shared__ int S_s;
  const int band = blockIdx.x;  // image * RB + rb
  const int n = band / RB;
  int tot = 0;
  for (int i = threadIdx.x; i < RB * CB; i += 256) tot += sens[(long)n * RB * CB + i];
  for (int off = 32; off > 0; off >>= 1) tot += __shfl_down(tot, off, 64);
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = tot;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
    int S = (2 * total + RB) / (2 * RB);
    S_s = S < CB ? S : CB;
  }
  __syncthreads();
  const int S = S_s;
  const int* cnt = count + (long)band * CB;
  const int* smp = samples + (long)band * CB;
  for (int cb = threadIdx.x; cb < CB; cb += 256) {
    uint8_t sv = sens[(long)band * CB + cb];
    if (balance) {
      // rank = number of blocks of the band that come before this one
      const long ca = cnt[cb], sa = smp[cb];
      int rank = 0;
      for (int o = 0; o < CB; ++o) {
        const long lhs = (long)cnt[o] * sa, rhs = ca * (long)smp[o];  // o before cb iff cnt_o/smp_o > cnt_cb/smp_cb
        rank += (lhs > rhs || (lhs == rhs && o < cb)) ? 1 : 0;
      }
      sv = rank < S ? 1 : 0;
    }
    if (sens_out) sens_out[(long)band * CB + cb] = sv;
    const uint32_t u = sens_draw(prefix, (uint64_t)band * (uint64_t)CB + (uint64_t)cb);
    block_keep[(long)band * CB + cb] = ((uint64_t)u < (sv ? tm : tn)) ? 0 : 1;
  }
}

static int32_t sens_geom(SensGeom& g, int32_t dtype, int N, int C, int H, int W, int kh, int kw, int stride, int pad, int x,
                         int y) {
  if (dtype != ARD_F32 && dtype != ARD_BF16) return fail(ARD_EDTYPE, "unknown dtype %d", dtype);
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
    return fail(ARD_ESHAPE, "non-positive convolution size");
  if (H + 2 * pad < kh || W + 2 * pad < kw) return fail(ARD_ESHAPE, "kernel larger than the padded input");
  g = SensGeom{N, C, H, W, kh, kw, stride, pad, (H + 2 * pad - kh) / stride + 1, (W + 2 * pad - kw) / stride + 1, 0, 0, 0, 0, 0, 0};
  g.rows = g.Ho * g.Wo;
  if ((long)C * kh * kw > 0x7fffff00L || (long)N * g.rows > 0x7fffff00L) return fail(ARD_ESHAPE, "input matrix too large");
  g.cols = C * kh * kw;
  if (x < 1 || y < 0) return fail(ARD_EINVAL, "region size must be positive (y = 0: the whole width)");
  g.x = x;
  g.y = y == 0 ? g.cols : y;
  g.RB = ceil_div(g.rows, g.x);
  g.CB = ceil_div(g.cols, g.y);
  if ((long)N * g.RB * g.CB > 0x7fffff00L) return fail(ARD_ESHAPE, "too many regions");
  return ARD_OK;
}

}  // namespace ard

using namespace ard;

extern "C" int32_t ard_sens_regions(int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t kh, int32_t kw, int32_t stride,
                                    int32_t pad, int32_t x, int32_t y, int32_t* rows, int32_t* row_bands,
                                    int32_t* col_blocks) {
  SensGeom g;
  if (int32_t st = sens_geom(g, ARD_BF16, N, C, H, Wd, kh, kw, stride, pad, x, y)) return st;
  if (rows) *rows = g.rows;
  if (row_bands) *row_bands = g.RB;
  if (col_blocks) *col_blocks = g.CB;
  return ARD_OK;
}

extern "C" int32_t ard_sens_predict(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t kh, int32_t kw,
                                    int32_t stride, int32_t pad, int32_t x, int32_t y, int32_t k_permille,
                                    int32_t t_permille, float threshold, uint64_t seed, uint64_t iteration, const void* A,
                                    int32_t* d_count, int32_t* d_samples, uint8_t* d_sens, void* stream) {
  BatchSuspend not_recorded;
  SensGeom g;
  if (int32_t st = sens_geom(g, dtype, N, C, H, Wd, kh, kw, stride, pad, x, y)) return st;
  if (k_permille < 1 || k_permille > 1000 || t_permille < 0 || t_permille > 1000)
    return fail(ARD_EINVAL, "k and t are per-mille values (k in 1..1000, t in 0..1000)");
  if ((long)g.x * g.y > (1L << 31) - 1 || ((long)k_permille * g.x * g.y) / 1000 > 65536)
    return fail(ARD_ESHAPE, "a region may hold at most 65536 samples (x * y * k / 1000)");
  if (!A || !d_count || !d_samples || !d_sens) return fail(ARD_EINVAL, "null pointer");
  const uint64_t prefix = sens_prefix(seed, iteration, SENS_STREAM_SAMPLE);
  const unsigned regions = (unsigned)((long)N * g.RB * g.CB);
  // tabulated geometry when it fits: the width of every region is g.y except the clipped last column block,
  // which only exists when the width does not divide the matrix -- then each region would need its own divisor
  const bool lut_ok = g.y <= kSensLutCols && g.x <= kSensLutRows && (long)C * H * Wd < (1L << 24) && kh < 16 && kw < 16 &&
                      (long)(g.Ho - 1) * stride < 65536 && (long)(g.Wo - 1) * stride < 32768 && g.cols % g.y == 0;
  if (lut_ok) {
    const FastDiv dw = fast_div((uint32_t)g.y);
    // footprint of a region in LDS when it fits: rows a band can touch x whole width x channels of a block
    const int ce = dtype == ARD_BF16 ? 8 : 4, taps = kh * kw;
    const int nch_max = imin(C, (g.y + taps - 2) / taps + 1);
    // Bands per workgroup.  Consecutive bands touch nearly the same input rows when they are shorter than an
    // output row (98 bands of 8 positions would copy a 28 x 28 image 14 times over), and a band with few draws
    // does not pay for its copy: a workgroup takes up to 16 bands, as many as bring it to about 40 k draws,
    // provided their common footprint is well below the sum of theirs (else grouping only costs workgroups) and
    // the launch keeps two workgroups per CU.  Config-5 layer, 30 % sampled, one band -> chosen number:
    // rows of 8 positions 185 -> 138 us (7 bands: two whole rows), of 4 positions 248 -> 139 us (14), of 16
    // positions 149 -> 147 us (3), 8 x 64 blocks 951 -> 285 us (16); regions of 112 x 576 stay alone (113 us,
    // two per workgroup 131 us).
    int G = 1, nrow_max = 0, chp = 0, rows1 = 0;
    size_t stage_bytes = 0;
    const long draws = imax(1, (int)(((long)k_permille * g.x * g.y) / 1000));
    const int g_cap = (int)imin(16, imax(1, (int)(40000 / draws)));
    for (int cand = 1; cand <= g_cap && cand <= imax(1, g.RB); ++cand) {
      // output rows a group can span: groups of whole rows start on a row, any other may start anywhere in one
      const int oh_span = (cand * g.x) % g.Wo == 0 ? cand * g.x / g.Wo : (cand * g.x + g.Wo - 2) / g.Wo + 1;
      const int nr = imin(H, (oh_span - 1) * stride + kh);
      const int cp = (int)align_up((size_t)(ce - 1 + nr * Wd), (size_t)ce);
      const size_t bytes = align_up((size_t)(cp / ce) * nch_max, (size_t)4) + (size_t)(g.y + cand * g.x) * sizeof(int);
      if (cand == 1) rows1 = nr;
      if (cand == 1 || (4 * nr <= 3 * cand * rows1 && bytes <= 64 * 1024 && (long)N * ceil_div(g.RB, cand) * g.CB >= 512))
        G = cand, nrow_max = nr, chp = cp, stage_bytes = bytes;
    }
    // (pad < filter size: every window then starts inside the image, which the copy's bounds rely on)
    if (((H * Wd) % ce) == 0 && (((uintptr_t)A) & 15) == 0 && stage_bytes <= 150 * 1024 && (long)chp * nch_max < (1L << 24) &&
        pad < kh && pad < kw) {
      const int RBG = ceil_div(g.RB, G);
      const SensStage sg{nrow_max, chp, fast_div((uint32_t)taps), fast_div((uint32_t)kw), fast_div((uint32_t)g.Wo), G, RBG};
      const unsigned groups = (unsigned)((long)N * RBG * g.CB);
      hipError_t e = hipSuccess;
      if (dtype == ARD_BF16) {
        if (stage_bytes > 65536) e = raise_lds_limit((const void*)sens_predict_staged_kernel<uint16_t>, (int)stage_bytes);
        if (e == hipSuccess)
          ARD_LAUNCH(sens_predict_staged_kernel<uint16_t>, dim3(groups), dim3(256), stage_bytes, (hipStream_t)stream,
                     (const uint16_t*)A, g, sg, k_permille, t_permille, threshold, prefix, dw, d_count, d_samples, d_sens);
      } else {
        if (stage_bytes > 65536) e = raise_lds_limit((const void*)sens_predict_staged_kernel<float>, (int)stage_bytes);
        if (e == hipSuccess)
          ARD_LAUNCH(sens_predict_staged_kernel<float>, dim3(groups), dim3(256), stage_bytes, (hipStream_t)stream, (const float*)A, g,
                     sg, k_permille, t_permille, threshold, prefix, dw, d_count, d_samples, d_sens);
      }
      if (e != hipSuccess) return fail(ARD_EHIP, "raising the LDS limit failed: %s", hipGetErrorString(e));
      ARD_LAUNCH_CHECK("sens_predict_staged_kernel");
      return ARD_OK;
    }
    const size_t lds = (size_t)(g.y + g.x) * sizeof(int);
    if (dtype == ARD_BF16)
      ARD_LAUNCH(sens_predict_lut_kernel<uint16_t>, dim3(regions), dim3(256), lds, (hipStream_t)stream, (const uint16_t*)A, g, k_permille,
                 t_permille, threshold, prefix, dw, d_count, d_samples, d_sens);
    else
      ARD_LAUNCH(sens_predict_lut_kernel<float>, dim3(regions), dim3(256), lds, (hipStream_t)stream, (const float*)A, g, k_permille,
                 t_permille, threshold, prefix, dw, d_count, d_samples, d_sens);
    ARD_LAUNCH_CHECK("sens_predict_lut_kernel");
    return ARD_OK;
  }
  if (dtype == ARD_BF16)
    ARD_LAUNCH(sens_predict_kernel<uint16_t>, dim3(regions), dim3(256), 0, (hipStream_t)stream, (const uint16_t*)A, g, k_permille,
               t_permille, threshold, prefix, d_count, d_samples, d_sens);
  else
    ARD_LAUNCH(sens_predict_kernel<float>, dim3(regions), dim3(256), 0, (hipStream_t)stream, (const float*)A, g, k_permille,
               t_permille, threshold, prefix, d_count, d_samples, d_sens);
  ARD_LAUNCH_CHECK("sens_predict_kernel");
  return ARD_OK;
}

extern "C" int32_t ard_sens_row_pattern(int32_t N, int32_t rows, int32_t x, const uint8_t* d_sens, double m, double n,
                                        uint64_t seed, uint64_t iteration, uint8_t* d_mask, int32_t* d_keep, int32_t* d_count,
                                        void* stream) {
  BatchSuspend not_recorded;
  if (N <= 0 || rows <= 0 || x <= 0) return fail(ARD_ESHAPE, "N, rows and x must be positive");
  if ((long)N * rows > 0x7fffff00L) return fail(ARD_ESHAPE, "too many rows");
  if (!(m >= 0.0 && m <= 1.0) || !(n >= 0.0 && n <= 1.0)) return fail(ARD_EINVAL, "possibilities must lie in [0, 1]");
  if (!d_sens || (!d_mask && !d_keep && !d_count)) return fail(ARD_EINVAL, "null pointer");
  const int total = N * rows;
  const int chunk = (int)align_up((size_t)ceil_div(total, 128), 1024);  // at most 128 workgroups of whole 1024-row rounds
  const dim3 grid((unsigned)ceil_div(total, chunk));
  const uint64_t tm = sens_threshold(m), tn = sens_threshold(n), pre = sens_prefix(seed, iteration, SENS_STREAM_ROWS);
  const int RB = ceil_div(rows, x);
  const bool via_mask = d_mask && (((uintptr_t)d_mask & 15) == 0);
  if (d_mask) {
    ARD_LAUNCH(sens_row_pattern_kernel, grid, dim3(1024), 0, (hipStream_t)stream, d_sens, total, rows, x, RB, 1, tm, tn, pre, chunk, 0,
               d_mask, d_keep, d_count);
    ARD_LAUNCH_CHECK("sens_row_pattern_kernel");
    if (!d_keep && !d_count) return ARD_OK;
  }
  ARD_LAUNCH(sens_row_pattern_kernel, grid, dim3(1024), 0, (hipStream_t)stream, d_sens, total, rows, x, RB, 1, tm, tn, pre, chunk,
             via_mask ? 1 : 2, d_mask, d_keep, d_count);
  ARD_LAUNCH_CHECK("sens_row_pattern_kernel");
  return ARD_OK;
}

extern "C" int32_t ard_sens_block_pattern(int32_t N, int32_t row_bands, int32_t col_blocks, const int32_t* d_count,
                                          const int32_t* d_samples, const uint8_t* d_sens, int32_t balance, double m, double n,
                                          uint64_t seed, uint64_t iteration, uint8_t* d_sens_out, uint8_t* d_block_keep,
                                          void* stream) {
  BatchSuspend not_recorded;
  if (N <= 0 || row_bands <= 0 || col_blocks <= 0) return fail(ARD_ESHAPE, "N, row_bands and col_blocks must be positive");
  if ((long)N * row_bands * col_blocks > 0x7fffff00L) return fail(ARD_ESHAPE, "too many blocks");
  if (!(m >= 0.0 && m <= 1.0) || !(n >= 0.0 && n <= 1.0)) return fail(ARD_EINVAL, "possibilities must lie in [0, 1]");
  if (!d_sens || !d_block_keep || (balance && (!d_count || !d_samples))) return fail(ARD_EINVAL, "null pointer");
  ARD_LAUNCH(sens_block_pattern_kernel, dim3((unsigned)(N * row_bands)), dim3(256), 0, (hipStream_t)stream, d_count, d_samples,
             d_sens, row_bands, col_blocks, balance, sens_threshold(m), sens_threshold(n),
             sens_prefix(seed, iteration, SENS_STREAM_BLOCKS), d_sens_out, d_block_keep);
  ARD_LAUNCH_CHECK("sens_block_pattern_kernel");
  return ARD_OK;
}
