// LSTM layer under a row pattern on its hidden units (Section 7.2.3: the LSTM runs as
// matrix multiplications, so the same patterns apply).
//
// Fused weight W[4H x (I+H)], gate blocks i, f, g, o of H rows, columns [x | h].
// A dropped unit has no gate rows and no recurrent column in any product.  Everything between
// the products lives in a COMPACT layout: Hk kept units stored with stride Hp = Hk rounded up
// to 8 (padding entries are zeros), gate g of kept unit j at index g*Hp + j.  All compact
// extents are then multiples of 8 and every product is a plain matrix product with 16-byte
// rows:
//   - the kept rows of the input and recurrent weights are gathered once per call
//     (Wx'[4Hp x I], Wh'[4Hp x Hp], zero rows / columns at the padding),
//   - the input projection of all T steps is one product, each step multiplies the compact
//     hidden state by Wh',
//   - the pointwise cell kernels run over physical units and write zeros for dropped ones,
//   - the weight gradient is computed compact and scattered into dW (zeros elsewhere) by one pass.
#include <stdlib.h>

#include <type_traits>

#include "engine.hpp"
#include "pattern.hpp"

namespace ard {

// rank[u] = compact index of unit u or -1
__global__ __launch_bounds__(1024) void lstm_setup_kernel(Axis ax, int H, int* rank) {
  for (int u = threadIdx.x; u < H; u += 1024) rank[u] = -1;
  __syncthreads();
  for (int j = threadIdx.x; j < ax.n; j += 1024) rank[ax_phys(ax, j)] = j;
}

// Tile pattern over the fused weight W[4H x (I+H)] (Section 3.2): the synapse at (row, col) lies in tile
// (row / tr, col / tc), tiles are numbered row-major over a grid of `tcols` tile columns, and tile number
// t (0-based) is kept iff (t - o) mod dp == 0 (o = b - 1).  dp == 0: no tile pattern.
struct LstmTiles {
  int dp, o, tr, tc, tcols;
};
__device__ __forceinline__ bool lstm_synapse_kept(const LstmTiles& tp, int row, int col) {
  if (tp.dp <= 1) return true;
  const long t = (long)(row / tp.tr) * tp.tcols + col / tp.tc - tp.o;
  return t % tp.dp == 0;  // (sign of t is irrelevant for == 0)
}

// out[g*Hp + j][q] = W[(g*H + unit(j)) * ldw + col(q)] for kept j, 0 at the padding and for synapses of
// dropped tiles.
// cols == 0: the input columns, q < ncol identity; cols == 1: the recurrent columns,
// q < Hp -> I + unit(q) (0 at the padding); out has `ldo` columns.
template <typename T>
__global__ void lstm_gather_w_kernel(const T* W, long ldw, Axis ax, int H, int I, int Hp, int recurrent, int ldo,
                                     LstmTiles tp, T* out) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  const int r = blockIdx.y;  // compact gate row
  if (q >= ldo) return;
  const int g = r / Hp, j = r - g * Hp;
  T v = (T)0;
  if (j < ax.n) {
    const int prow = g * H + ax_phys(ax, j);
    const long row = (long)prow * ldw;
    int col = -1;
    if (!recurrent) col = q < I ? q : -1;
    else if (q < ax.n) col = I + ax_phys(ax, q);
    if (col >= 0 && lstm_synapse_kept(tp, prow, col)) v = W[row + col];
  }
  out[(long)r * ldo + q] = v;
}

// out[r][j] = j < Hk ? src[r*H + unit(j)] : 0 (compact copy of stored hidden states)
template <typename T>
__global__ void lstm_gather_h_kernel(const T* src, int H, Axis ax, int Hp, T* out) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const long r = blockIdx.y;
  if (j < Hp) out[r * Hp + j] = j < ax.n ? src[r * H + ax_phys(ax, j)] : (T)0;
}

__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

// One time step, forward.  G: compact pre-activations [B x 4Hp] (fp32).  Writes the
// activated gates [B x 4H], c [B x H] (fp32), h [B x H] (dtype) with zeros for dropped
// units, and the compact h [B x Hp] (zeros at the padding) that feeds the next step's product.
// Threads u >= H take the padding entries.
// `part` (optional): `splits` fp32 partial sums [B x 4Hp] of this step's recurrent product, `pstride`
// floats apart, added to G here (the product then needs no finishing pass).
template <typename T>
__global__ void lstm_cell_fwd_kernel(const float* G, const float* part, int splits, long pstride, const int* rank,
                                     const float* c_prev, int B, int H, int Hk, int Hp, float* gates, float* c, T* h,
                                     T* hc) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (u >= H) {
    const int j = Hk + (u - H);
    if (j < Hp) hc[(long)b * Hp + j] = (T)0;
    return;
  }
  const int j = rank[u];
  float gi = 0, gf = 0, gg = 0, go = 0, cv = 0, hv = 0;
  if (j >= 0) {
    const float* g = G + (long)b * 4 * Hp;
    float zi = g[j], zf = g[Hp + j], zg = g[2 * Hp + j], zo = g[3 * Hp + j];
    for (int s = 0; s < splits; ++s) {
      const float* q = part + s * pstride + (long)b * 4 * Hp;
      zi += q[j], zf += q[Hp + j], zg += q[2 * Hp + j], zo += q[3 * Hp + j];
    }
    gi = sigmoidf_(zi);
    gf = sigmoidf_(zf);
    gg = tanhf(zg);
    go = sigmoidf_(zo);
    const float cp = c_prev ? c_prev[(long)b * H + u] : 0.0f;
    cv = gf * cp + gi * gg;
    hv = go * tanhf(cv);
    hc[(long)b * Hp + j] = ElemTraits<T>::from_f32(hv);
  }
  float* ga = gates + (long)b * 4 * H;
  ga[u] = gi;
  ga[H + u] = gf;
  ga[2 * H + u] = gg;
  ga[3 * H + u] = go;
  c[(long)b * H + u] = cv;
  h[(long)b * H + u] = ElemTraits<T>::from_f32(hv);
}

// One time step, backward.  dh_next: compact [B x Hp] fp32 (NULL at the last step);
// dc_next: [B x H] fp32, read unless `first`, then overwritten.  Writes the compact gate
// gradient dG [B x 4Hp] in the storage dtype (zeros at the padding).
// dh_next may come as `splits` partial sums `pstride` floats apart (summed here).
template <typename T>
__global__ void lstm_cell_bwd_kernel(const float* gates, const float* c, const float* c_prev, const T* dh_ext,
                                     const float* dh_next, int splits, long pstride, float* dc_next, const int* rank, int B,
                                     int H, int Hk, int Hp, int first, T* dG) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  T* d = dG + (long)b * 4 * Hp;
  if (u >= H) {
    const int j = Hk + (u - H);
    if (j < Hp) d[j] = d[Hp + j] = d[2 * Hp + j] = d[3 * Hp + j] = (T)0;
    return;
  }
  const int j = rank[u];
  if (j < 0) return;
  const float* ga = gates + (long)b * 4 * H;
  const float gi = ga[u], gf = ga[H + u], gg = ga[2 * H + u], go = ga[3 * H + u];
  const float tc = tanhf(c[(long)b * H + u]);
  const float cp = c_prev ? c_prev[(long)b * H + u] : 0.0f;
  float dh = ElemTraits<T>::to_f32(dh_ext[(long)b * H + u]);
  if (dh_next)
    for (int s = 0; s < splits; ++s) dh += dh_next[s * pstride + (long)b * Hp + j];
  float dc = dh * go * (1.0f - tc * tc);
  if (!first) dc += dc_next[(long)b * H + u];
  d[j] = ElemTraits<T>::from_f32(dc * gg * gi * (1.0f - gi));
  d[Hp + j] = ElemTraits<T>::from_f32(dc * cp * gf * (1.0f - gf));
  d[2 * Hp + j] = ElemTraits<T>::from_f32(dc * gi * (1.0f - gg * gg));
  d[3 * Hp + j] = ElemTraits<T>::from_f32(dh * tc * go * (1.0f - go));
  dc_next[(long)b * H + u] = dc * gf;
}

// dst[r][0..cols) = src[r][0..cols) for rows of different lengths (ld_src, ld_dst): strips the padding of dx
template <typename T>
__global__ void lstm_copy_rows_kernel(const T* src, long ld_src, int cols, long ld_dst, T* dst) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const long r = blockIdx.y;
  if (j < cols) dst[r * ld_dst + j] = src[r * ld_src + j];
}

// dW[(g*H + u)][q] from the compact gradients dwx[4Hp x Ip] and dwh[4Hp x Hp]; +0.0 for every
// row of a dropped unit, every recurrent column of a dropped unit and every synapse of a dropped tile.
template <typename T>
__global__ void lstm_scatter_dw_kernel(const T* dwx, const T* dwh, const int* rank, int H, int I, int Ip, int Hp, LstmTiles tp,
                                       T* dW) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  const int p = blockIdx.y;  // physical gate row
  if (q >= I + H) return;
  const int g = p / H, u = p - g * H;
  const int j = rank[u];
  T v = (T)0;
  if (j >= 0 && lstm_synapse_kept(tp, p, q)) {
    const long r = (long)g * Hp + j;
    if (q < I) {
      v = dwx[r * Ip + q];
    } else {
      const int jv = rank[q - I];
      if (jv >= 0) v = dwh[r * Hp + jv];
    }
  }
  dW[(long)p * (I + H) + q] = v;
}

static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// ---- the recurrence in one launch (Section 7.2.3) -----------------------------------------------
//
// The per-step products of a batch-128 LSTM are a few hundred MFLOP each: issued as launches, a step
// costs two dependent launches however few units are kept.  This kernel walks all T steps itself.
// Workgroup (s, bb) owns 8 kept units (their 4 x 8 = 32 gate rows of Wh', staged ONCE in LDS for the whole
// sequence) and the MB = 32 * TMB batch rows of block bb: per step it multiplies h_{t-1}[rows, :] by its 32
// gate rows (32x32x16 MFMAs, the contraction dealt over the 4 wavefronts and summed through LDS), adds
// the input projection, runs the cell for its (row, unit) pairs (c stays in a register) and writes h_t.
// Steps are separated by one flag per workgroup: after its h_t is written a workgroup posts t + 1; a
// workgroup starts step t when the S workgroups of its batch block have all posted t.  h_t travels between workgroups on
// different XCDs through device-scope (write-through) stores and device-scope loads; a workgroup waits for
// its own stores before it signals.  All workgroups must be resident together (the host launches this
// kernel only with at most one workgroup per CU); the wait is bounded all the same: a workgroup that gives
// up sets *err and leaves, and every workgroup that sees *err leaves too.
struct LstmPersist {
  const float* Gx;     // [T][B][4Hp] input projection
  const uint16_t* Wh;  // [4Hp][Hp] compact recurrent weight
  uint16_t* hc;        // [T][B][Hp] compact hidden states (written here, read by the next step)
  uint16_t* h;         // [T][B][H]
  float* c;            // [T][B][H]
  float* gates;        // [T][B][4H]
  int* counters;       // flags[batch block][unit slice] = steps posted by that workgroup, zero at launch
  int* err;            // zero at launch; 1: the recurrence gave up
  int T, B, H, Hk, Hp, S;
  int off, step;       // kept unit j is physical unit off + j * step
  long spin_limit;
};

// VIA_L2: h_{t-1} is read through the XCD's L2 after an agent-scope acquire (else with device-scope loads)
template <int TMB, bool VIA_L2>
__global__ __launch_bounds__(256) void lstm_persist_fwd_kernel(const LstmPersist P) {
  constexpr int MB = 32 * TMB;
  extern __shared__ uint4 lp_lds[];
  __shared__ int go_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = blockIdx.x % P.S, bb = blockIdx.x / P.S;
  const int Hp = P.Hp, B = P.B, H = P.H;
  const int pitch = Hp * 2 + 16;  // bytes between the staged weight rows (rows start 16 bytes apart in the banks)
  char* wl = reinterpret_cast<char*>(lp_lds);
  float* red = reinterpret_cast<float*>(wl + 32 * pitch);  // [4][MB][33]
  // this workgroup's 32 gate rows, r = gate * 8 + local unit, staged once
  const int chunks = Hp >> 3;
  for (int i = tid; i < 32 * chunks; i += 256) {
    const int r = i / chunks, ch = i - r * chunks;
    const long row = (long)(r >> 3) * Hp + s * 8 + (r & 7);
    *reinterpret_cast<uint4*>(wl + r * pitch + ch * 16) = *reinterpret_cast<const uint4*>(P.Wh + row * Hp + ch * 8);
  }
  __syncthreads();
  const int nslice = (Hp + 15) >> 4;
  // cell: thread = (row rb of each 32-row tile, local unit ul)
  const int rb = tid >> 3, ul = tid & 7;
  const int j = s * 8 + ul;  // compact unit
  const bool kept = j < P.Hk;
  const int u = P.off + j * P.step;  // physical unit
  // zeros of the dropped units this thread owns: the rest of its group [j*step, (j+1)*step), the last kept
  // unit also the tail up to H
  const int z_lo = j * P.step, z_hi = !kept ? z_lo : (j == P.Hk - 1 ? H : z_lo + P.step);
  float c_reg[TMB];
#pragma unroll
  for (int rt = 0; rt < TMB; ++rt) c_reg[rt] = 0.0f;
  for (int t = 0; t < P.T; ++t) {
    f32x16_t acc[TMB];
#pragma unroll
    for (int rt = 0; rt < TMB; ++rt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rt][v] = 0.0f;
    // this step's input projections do not depend on h_{t-1}: fetched before the wait, so that their
    // trip to memory overlaps it
    float zx[TMB][4];
    {
      const float* Gt = P.Gx + (long)t * B * 4 * Hp;
#pragma unroll
      for (int rt = 0; rt < TMB; ++rt) {
        const int row = bb * MB + rt * 32 + rb;
#pragma unroll
        for (int g = 0; g < 4; ++g) zx[rt][g] = (row < B && kept) ? Gt[(long)row * 4 * Hp + g * Hp + j] : 0.0f;
      }
    }
    if (t > 0) {
      if (wave == 0) {
        // every workgroup of this batch block has posted step t - 1: one flag per workgroup (no contended
        // counter), the 64 lanes read 64 flags per poll
        const int* flags = P.counters + (long)bb * P.S;
        long spins = 0;
        int ok = 1;
        for (;;) {
          bool ready = true;
          for (int i = lane; i < P.S; i += 64) ready = ready && __hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= t;
          // (a negative bound is the host's way to force the give-up path: the first wait fails whatever it saw --
          // with a bound of zero a poll that finds everything posted, which is the common case, would still pass)
          if (__all(ready) && P.spin_limit >= 0) break;
          if (++spins > P.spin_limit || __hip_atomic_load(P.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
            __hip_atomic_store(P.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = 0;
            break;
          }
        }
        if (lane == 0) go_s = ok;
        // (h_{t-1} is complete in memory: drop what this CU's L1 and this XCD's L2 may hold of it)
        if (VIA_L2) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
      __syncthreads();
      if (!go_s) return;  // uniform: every thread of the workgroup leaves
      // recurrent product: this wavefront's 16-wide slices of the contraction
      const unsigned long long* hp = reinterpret_cast<const unsigned long long*>(P.hc + (long)(t - 1) * B * Hp);
      const int khalf = lane >> 5;
      // the device-scope loads of h_{t-1} travel a long way: a wavefront issues those of CH slices
      // together and multiplies afterwards (one round trip per CH slices instead of one per slice)
      constexpr int CH = TMB == 4 ? 4 : 8;
      for (int q0 = wave; q0 < nslice; q0 += 4 * CH) {
        unsigned long long lo[CH][TMB], hi[CH][TMB];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const int q = q0 + 4 * i;
          const int kk = q * 16 + khalf * 8;
          const int kc = (q < nslice && kk < Hp) ? kk : 0;  // (clamped: the value is discarded below)
#pragma unroll
          for (int rt = 0; rt < TMB; ++rt) {
            int row = bb * MB + rt * 32 + (lane & 31);
            row = row < B ? row : B - 1;  // rows beyond the batch are never stored
            const unsigned long long* src = hp + (((long)row * Hp + kc) >> 2);
            if (VIA_L2) {
              const ulonglong2 v = *reinterpret_cast<const ulonglong2*>(src);
              lo[i][rt] = v.x, hi[i][rt] = v.y;
            } else {
              lo[i][rt] = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              hi[i][rt] = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
          }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const int q = q0 + 4 * i;
          if (q >= nslice) break;
          const int kk = q * 16 + khalf * 8;
          const bool k_ok = kk < Hp;
          const uint4 bw = *reinterpret_cast<const uint4*>(wl + (lane & 31) * pitch + (k_ok ? kk : 0) * 2);
          const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, k_ok ? bw : make_uint4(0, 0, 0, 0));
#pragma unroll
          for (int rt = 0; rt < TMB; ++rt) {
            const uint4 aw = make_uint4((unsigned)lo[i][rt], (unsigned)(lo[i][rt] >> 32), (unsigned)hi[i][rt], (unsigned)(hi[i][rt] >> 32));
            acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, aw), bfrag, acc[rt], 0, 0, 0);
          }
        }
      }
    }
    // partial tiles of the four wavefronts -> LDS: lane holds column (lane & 31), rows 8*(v/4) + 4*(lane>>5) + v%4
#pragma unroll
    for (int rt = 0; rt < TMB; ++rt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        red[(wave * MB + rt * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * 33 + (lane & 31)] = acc[rt][v];
    __syncthreads();
    // cell.  What the other workgroups wait for is h_t alone: it is stored first (device scope), the
    // workgroup signals as soon as those stores have completed, and only then writes gates, c and h to
    // the caller's tensors (their trip to memory is off the critical path of the recurrence).
    float gi[TMB], gf[TMB], gg[TMB], go[TMB], hv[TMB];
#pragma unroll
    for (int rt = 0; rt < TMB; ++rt) {
      const int rl = rt * 32 + rb, row = bb * MB + rl;
      hv[rt] = gi[rt] = gf[rt] = gg[rt] = go[rt] = 0.0f;
      if (row < B && kept) {
        float z[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int col = g * 8 + ul;
          z[g] = zx[rt][g] + ((red[(0 * MB + rl) * 33 + col] + red[(1 * MB + rl) * 33 + col]) +
                              (red[(2 * MB + rl) * 33 + col] + red[(3 * MB + rl) * 33 + col]));
        }
        gi[rt] = sigmoidf_(z[0]), gf[rt] = sigmoidf_(z[1]), gg[rt] = tanhf(z[2]), go[rt] = sigmoidf_(z[3]);
        const float cv = gf[rt] * c_reg[rt] + gi[rt] * gg[rt];
        c_reg[rt] = cv;
        hv[rt] = go[rt] * tanhf(cv);
      }
      if (row < B) {
        // compact h_t for the next step: device-scope store (the padding units store their zero)
        const unsigned bits = f32_to_bf16_bits(hv[rt]);
        const unsigned other = (unsigned)__shfl_xor((int)bits, 1, 64);
        if (!(ul & 1))
          __hip_atomic_store(reinterpret_cast<unsigned*>(P.hc + ((long)t * B + row) * Hp + j), bits | (other << 16), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // every thread's h_t stores have completed before the workgroup signals
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0 && t + 1 < P.T)
      __hip_atomic_store(&P.counters[(long)bb * P.S + s], t + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int rt = 0; rt < TMB; ++rt) {
      const int row = bb * MB + rt * 32 + rb;
      if (row >= B) continue;
      float* ga = P.gates + ((long)t * B + row) * 4 * H;
      if (kept) {
        ga[u] = gi[rt];
        ga[H + u] = gf[rt];
        ga[2 * H + u] = gg[rt];
        ga[3 * H + u] = go[rt];
        P.c[((long)t * B + row) * H + u] = c_reg[rt];
        P.h[((long)t * B + row) * H + u] = f32_to_bf16_bits(hv[rt]);
      }
      // zeros of the dropped units of this thread's group
      for (int uz = z_lo; uz < z_hi; ++uz) {
        if (uz == u) continue;
        ga[uz] = ga[H + uz] = ga[2 * H + uz] = ga[3 * H + uz] = 0.0f;
        P.c[((long)t * B + row) * H + uz] = 0.0f;
        P.h[((long)t * B + row) * H + uz] = 0;
      }
    }
  }
}

// ---- the backward recurrence in one launch ------------------------------------------------------
//
// Back-propagation through time has the same shape of problem: step t needs dG_{t+1} . Wh', the gradient
// that reaches h_t through the recurrence -- a contraction over all 4Hp gate rows (four times the forward
// one) for Hp outputs.  Workgroup (s, bb) owns UW kept units (16 or 32: their columns of Wh' are staged
// once in LDS, transposed) and MB = 16 * TM16 batch rows.  Per step it multiplies dG_{t+1}[rows, :] by its
// columns (16x16x32 MFMAs, the contraction dealt over the four wavefronts and summed through LDS), adds the
// gradient arriving at the output, runs the cell's backward for its (row, unit) pairs (the cell-state
// gradient stays in registers) and writes its 4 x UW columns of dG_t, which is the result and also what
// the other workgroups of the batch block wait for.  What a workgroup reads per step is MB x 4Hp values
// whatever UW is, so few rows per workgroup (and many workgroups) keep the step short.  Flags, scopes and
// the bounded wait are those of the forward kernel.
struct LstmPersistBwd {
  const float* gates;   // [T][B][4H]
  const float* c;       // [T][B][H]
  const uint16_t* dh;   // [T][B][H] gradient arriving at the outputs
  const uint16_t* Wh;   // [4Hp][Hp] compact recurrent weight
  uint16_t* dG;         // [T][B][4Hp] compact gate gradients
  int* counters;        // flags[batch block][unit slice] = steps posted by that workgroup, zero at launch
  int* err;             // zero at launch; 1: the recurrence gave up
  int T, B, H, Hk, Hp, S, UW;
  int off, step;        // kept unit j is physical unit off + j * step
  long spin_limit;
};

template <int TM16, bool VIA_L2>
__global__ __launch_bounds__(256) void lstm_persist_bwd_kernel(const LstmPersistBwd P) {
  constexpr int MB = 16 * TM16;
  constexpr int NPMAX = 2 * TM16;  // (row, unit) pairs of a thread when UW = 32
  extern __shared__ uint4 lp_lds[];
  __shared__ int go_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = blockIdx.x % P.S, bb = blockIdx.x / P.S;
  const int Hp = P.Hp, B = P.B, H = P.H, UW = P.UW, K = 4 * Hp;
  const int pitch = K * 2 + 64;  // bytes between the staged columns (64 bytes apart in the banks)
  const int RW = UW + 1;
  char* wl = reinterpret_cast<char*>(lp_lds);
  float* red = reinterpret_cast<float*>(wl + UW * pitch);  // [4][MB][RW]
  // this workgroup's UW columns of Wh', wl[local unit][gate row], staged once
  // (a row of Wh' is read in 16-byte pieces of 8 units: Hp and UW are multiples of 8)
  const int cpr = UW >> 3;
  for (int i = tid; i < K * cpr; i += 256) {
    const int k = i / cpr, x0 = (i - k * cpr) * 8;
    const int jj = s * UW + x0;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (jj < Hp) v = *reinterpret_cast<const uint4*>(P.Wh + (long)k * Hp + jj);
    const unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e)
      *reinterpret_cast<uint16_t*>(wl + (x0 + e) * pitch + k * 2) = (uint16_t)(w4[e >> 1] >> ((e & 1) * 16));
  }
  __syncthreads();
  const int nslice = K >> 5;  // 32-deep slices (4Hp is a multiple of 32: no partial slice)
  const int nct = UW >> 4;    // 16-unit column tiles
  // cell: thread = (local unit ul, rows r0, r0 + rstep, ...)
  const int ul = tid % UW, r0 = tid / UW, rstep = 256 / UW, np = MB / rstep;
  const int j = s * UW + ul;  // compact unit
  const bool kept = j < P.Hk, in_store = j < Hp;
  const int u = kept ? P.off + j * P.step : 0;  // physical unit
  float dc_next[NPMAX];
#pragma unroll
  for (int i = 0; i < NPMAX; ++i) dc_next[i] = 0.0f;
  for (int tt = 0; tt < P.T; ++tt) {
    const int t = P.T - 1 - tt;
    // what the cell needs of the forward pass does not depend on the other workgroups: fetched before the wait
    float gi[NPMAX], gf[NPMAX], gg[NPMAX], go[NPMAX], ct[NPMAX], cp[NPMAX], dhe[NPMAX];
#pragma unroll
    for (int i = 0; i < NPMAX; ++i) {
      gi[i] = gf[i] = gg[i] = go[i] = ct[i] = cp[i] = dhe[i] = 0.0f;
      const int row = bb * MB + r0 + i * rstep;
      if (i < np && row < B && kept) {
        const float* ga = P.gates + ((long)t * B + row) * 4 * H;
        gi[i] = ga[u], gf[i] = ga[H + u], gg[i] = ga[2 * H + u], go[i] = ga[3 * H + u];
        ct[i] = P.c[((long)t * B + row) * H + u];
        if (t > 0) cp[i] = P.c[((long)(t - 1) * B + row) * H + u];
        dhe[i] = bf16_bits_to_f32(P.dh[((long)t * B + row) * H + u]);
      }
    }
    f32x4_t acc[TM16][2];
#pragma unroll
    for (int rt = 0; rt < TM16; ++rt)
#pragma unroll
      for (int cti = 0; cti < 2; ++cti)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[rt][cti][v] = 0.0f;
    if (tt > 0) {
      if (wave == 0) {
        // every workgroup of this batch block has posted dG_{t+1}
        const int* flags = P.counters + (long)bb * P.S;
        long spins = 0;
        int ok = 1;
        for (;;) {
          bool ready = true;
          for (int i = lane; i < P.S; i += 64) ready = ready && __hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= tt;
          if (__all(ready) && P.spin_limit >= 0) break;  // (a negative bound forces the give-up path)
          if (++spins > P.spin_limit || __hip_atomic_load(P.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
            __hip_atomic_store(P.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = 0;
            break;
          }
        }
        if (lane == 0) go_s = ok;
        if (VIA_L2) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
      __syncthreads();
      if (!go_s) return;  // uniform: every thread of the workgroup leaves
      const uint16_t* gsrc = P.dG + (long)(t + 1) * B * K;
      const int kgrp = lane >> 4, n = lane & 15;
      constexpr int CH = 16 / TM16;  // slices whose loads a wavefront issues together
      for (int q0 = wave; q0 < nslice; q0 += 4 * CH) {
        uint4 av[CH][TM16];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const int q = q0 + 4 * i;
          const int kc = q < nslice ? q * 32 + kgrp * 8 : 0;  // (clamped: the value is discarded below)
#pragma unroll
          for (int rt = 0; rt < TM16; ++rt) {
            int row = bb * MB + rt * 16 + n;
            row = row < B ? row : B - 1;  // rows beyond the batch are never stored
            const uint16_t* src = gsrc + (long)row * K + kc;
            if (VIA_L2) {
              av[i][rt] = *reinterpret_cast<const uint4*>(src);
            } else {
              const unsigned long long* s8 = reinterpret_cast<const unsigned long long*>(src);
              const unsigned long long lo = __hip_atomic_load(s8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              const unsigned long long hi = __hip_atomic_load(s8 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              av[i][rt] = make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
            }
          }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const int q = q0 + 4 * i;
          if (q >= nslice) break;
          const int kk = q * 32 + kgrp * 8;
#pragma unroll
          for (int cti = 0; cti < 2; ++cti) {
            if (cti >= nct) break;  // (uniform)
            const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(wl + (cti * 16 + n) * pitch + kk * 2));
#pragma unroll
            for (int rt = 0; rt < TM16; ++rt)
              acc[rt][cti] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[i][rt]), bfrag, acc[rt][cti], 0, 0, 0);
          }
        }
      }
    }
    // partial tiles of the four wavefronts -> LDS: lane holds column (lane & 15) of a tile, rows 4*(lane>>4) + v
#pragma unroll
    for (int rt = 0; rt < TM16; ++rt)
#pragma unroll
      for (int cti = 0; cti < 2; ++cti) {
        if (cti >= nct) break;
#pragma unroll
        for (int v = 0; v < 4; ++v)
          red[(wave * MB + rt * 16 + 4 * (lane >> 4) + v) * RW + cti * 16 + (lane & 15)] = acc[rt][cti][v];
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NPMAX; ++i) {
      if (i >= np) break;  // (uniform)
      const int rl = r0 + i * rstep, row = bb * MB + rl;
      float d[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (row < B && kept) {
        const float dh = dhe[i] + ((red[(0 * MB + rl) * RW + ul] + red[(1 * MB + rl) * RW + ul]) +
                                   (red[(2 * MB + rl) * RW + ul] + red[(3 * MB + rl) * RW + ul]));
        const float tc = tanhf(ct[i]);
        const float dc = dh * go[i] * (1.0f - tc * tc) + dc_next[i];
        d[0] = dc * gg[i] * gi[i] * (1.0f - gi[i]);
        d[1] = dc * cp[i] * gf[i] * (1.0f - gf[i]);
        d[2] = dc * gi[i] * (1.0f - gg[i] * gg[i]);
        d[3] = dh * tc * go[i] * (1.0f - go[i]);
        dc_next[i] = dc * gf[i];
      }
      // dG_t: pairs of adjacent units as one word, device-scope stores (the padding units store their zeros)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const unsigned bits = f32_to_bf16_bits(d[g]);
        const unsigned other = (unsigned)__shfl_xor((int)bits, 1, 64);
        if (!(ul & 1) && row < B && in_store)
          __hip_atomic_store(reinterpret_cast<unsigned*>(P.dG + ((long)t * B + row) * K + g * Hp + j), bits | (other << 16),
                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // every thread's stores have completed before the workgroup signals
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0 && tt + 1 < P.T)
      __hip_atomic_store(&P.counters[(long)bb * P.S + s], tt + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__global__ void lstm_zero_ints_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

static int lstm_cu_count() {
  static int cus = -1;
  if (cus < 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    cus = (!dry_run() && hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) ? prop.multiProcessorCount : 256;
  }
  return cus;
}

struct LstmWs {
  int* rank;
  char* wxc;     // [4Hp x Ip] dtype (Ip = I rounded up to 8: every row a whole number of 16-byte pieces)
  char* xp;      // [T*B x Ip] dtype, only when Ip != I: x with padded rows (forward, weight gradient)
  char* dxp;     // [T*B x Ip] dtype, only when Ip != I: dx before its padding is stripped
  char* whc;     // [4Hp x Hp] dtype
  char* hc;      // [T*B x Hp] dtype
  char* big;     // fwd: Gx [T*B x 4Hp] fp32; bwd: dG [T*B x 4Hp] dtype
  float* dh_next;  // [B x Hp]
  float* dc_next;  // [B x H]
  char* dwx;     // [4Hp x Ip] dtype
  char* dwh;     // [4Hp x Hp] dtype
  char* part;    // fp32 partial sums of split products
  size_t part_bytes;
  int* sync;     // step counters (one per batch block of 32 rows) and the give-up flag of the one-launch recurrence
  size_t total;
};

static LstmWs lstm_ws_layout(char* base, int es, int T, int B, int I, int H, int Hk) {
  LstmWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes ? bytes : 1, 256);
    return p;
  };
  const size_t Hp = pad8(Hk);
  w.rank = (int*)take((size_t)H * 4);
  const size_t Ip = pad8(I);
  w.wxc = take(4 * Hp * Ip * es);
  w.xp = (int)Ip != I ? take((size_t)T * B * Ip * es) : nullptr;
  w.dxp = (int)Ip != I ? take((size_t)T * B * Ip * es) : nullptr;
  w.whc = take(4 * Hp * Hp * es);
  w.hc = take((size_t)T * B * Hp * es);
  w.big = take((size_t)T * B * 4 * Hp * 4);
  w.dh_next = (float*)take((size_t)B * Hp * 4);
  w.dc_next = (float*)take((size_t)B * H * 4);
  w.dwx = take(4 * Hp * Ip * es);
  w.dwh = take(4 * Hp * Hp * es);
  // room for the partial sums of any product here split 8 ways, capped at 256 MiB
  size_t big = 4 * Hp * (size_t)(Ip > Hp ? Ip : Hp);
  if ((size_t)B * 4 * Hp > big) big = (size_t)B * 4 * Hp;
  w.part_bytes = big * 4 * 8;
  if (w.part_bytes > ((size_t)256 << 20)) w.part_bytes = (size_t)256 << 20;
  w.part = take(w.part_bytes);
  w.sync = (int*)take(((size_t)pad8(Hk) / 8 * ((size_t)B / 32 + 1) + 8) * 4);
  w.total = off;
  return w;
}

struct LstmArgs {
  int32_t dtype, T, B, I, H, Hk, es;
  Axis ax;
  LstmTiles tiles;
};

static int32_t lstm_check(LstmArgs& a, const ard_pattern* pat) {
  if (a.dtype != ARD_F32 && a.dtype != ARD_BF16) return fail(ARD_EDTYPE, "unknown dtype %d", a.dtype);
  if (a.T <= 0 || a.B <= 0 || a.I <= 0 || a.H <= 0)
    return fail(ARD_ESHAPE, "T, B, I, H must be positive (got %d, %d, %d, %d)", a.T, a.B, a.I, a.H);
  if (4L * a.H > 65535) return fail(ARD_ESHAPE, "more than 16383 hidden units");
  a.tiles = LstmTiles{0, 0, 1, 1, 1};
  int32_t st;
  if (pat && pat->kind == ARD_PAT_TILE) {
    // synapses are dropped, every unit stays
    if (pat->tile_r <= 0 || pat->tile_c <= 0) return fail(ARD_EINVAL, "tile size must be positive");
    const int TR = ceil_div(4 * a.H, pat->tile_r), TC = ceil_div(a.I + a.H, pat->tile_c);
    st = check_pattern(pat, TR * TC, "pat");
    if (st) return st;
    a.tiles = LstmTiles{pat->dp, pat->b - 1, pat->tile_r, pat->tile_c, TC};
    a.ax = axis_identity(a.H);
  } else {
    st = check_pattern(pat, a.H, "pat");
    if (st) return st;
    a.ax = axis_of_pattern(pat, a.H);
  }
  a.Hk = a.ax.n;
  a.es = a.dtype == ARD_BF16 ? 2 : 4;
  if ((long)a.T * a.B > 0x7fffffffL / 4 || (long)a.B > 65535 || (long)a.T * a.B > 65535 * 64L)
    return fail(ARD_ESHAPE, "T*B or B too large");
  return ARD_OK;
}

// plain product C[M x N] (+)= A . B with identity maps on every side
static GemmParams plain_gemm(const void* A, long lda, const void* B, long ldb, void* C, long ldc, int M, int N, int K,
                             bool a_kc, bool b_kc, int ce, bool out_f32, float beta) {
  GemmParams P{};
  P.k = axis_identity(K);
  P.A = Operand{A, lda, axis_identity(M), 0, 0, 0, 0};
  P.B = Operand{B, ldb, axis_identity(N), 0, 0, 0, 0};
  P.A.vec = operand_vec_ok(P.A, a_kc, P.k, ce);
  P.B.vec = operand_vec_ok(P.B, b_kc, P.k, ce);
  P.C.p = C;
  P.C.ld = ldc;
  P.C.rm = axis_identity(M);
  P.C.cn = axis_identity(N);
  P.C.out_f32 = out_f32 ? 1 : 0;
  P.C.alpha = 1.0f;
  P.C.beta = beta;
  P.M = M;
  P.N = N;
  return P;
}

template <typename T>
static int32_t lstm_prepare(const LstmArgs& a, const void* W, const LstmWs& w, hipStream_t stream) {
  ARD_LAUNCH(lstm_setup_kernel, dim3(1), dim3(1024), 0, stream, a.ax, a.H, w.rank);
  ARD_LAUNCH_CHECK("lstm_setup_kernel");
  const int Hp = pad8(a.Hk);
  if (a.Hk > 0) {
    ARD_LAUNCH(lstm_gather_w_kernel<T>, dim3(ceil_div(pad8(a.I), 256), 4 * Hp), dim3(256), 0, stream, (const T*)W,
                       (long)(a.I + a.H), a.ax, a.H, a.I, Hp, 0, pad8(a.I), a.tiles, (T*)w.wxc);
    ARD_LAUNCH_CHECK("lstm_gather_w_kernel");
    ARD_LAUNCH(lstm_gather_w_kernel<T>, dim3(ceil_div(Hp, 256), 4 * Hp), dim3(256), 0, stream, (const T*)W,
                       (long)(a.I + a.H), a.ax, a.H, a.I, Hp, 1, Hp, a.tiles, (T*)w.whc);
    ARD_LAUNCH_CHECK("lstm_gather_w_kernel");
  }
  return ARD_OK;
}

// x with rows padded to a multiple of 8 elements (zeros), so that the products over it can use 16-byte
// loads whatever the input width; returns x itself when no padding is needed
template <typename T>
static int32_t lstm_padded_x(const LstmArgs& a, const void* x, const LstmWs& w, hipStream_t stream, const void** xo) {
  const int Ip = pad8(a.I);
  *xo = x;
  if (Ip == a.I) return ARD_OK;
  const long rows_total = (long)a.T * a.B;
  for (long r0 = 0; r0 < rows_total; r0 += 65535) {
    const long rows = rows_total - r0 < 65535 ? rows_total - r0 : 65535;
    ARD_LAUNCH(lstm_gather_h_kernel<T>, dim3(ceil_div(Ip, 256), (unsigned)rows), dim3(256), 0, stream,
                       (const T*)x + r0 * a.I, a.I, axis_identity(a.I), Ip, (T*)w.xp + r0 * Ip);
    ARD_LAUNCH_CHECK("lstm_gather_h_kernel");
  }
  *xo = w.xp;
  return ARD_OK;
}

// Does the forward pass of this layer run its recurrence in one launch, and how?  (bf16, affine pattern,
// at most one workgroup per CU, bounded exchange traffic)
struct PersistPlan {
  int tmb, S, nbb;
  int via_l2;  // read h_{t-1} through L2 (large states) instead of with device-scope loads
  size_t lds;
};
static bool lstm_persist_plan(const LstmArgs& a, PersistPlan& p) {
  const int Hp = pad8(a.Hk);
  if (a.dtype != ARD_BF16 || a.Hk <= 0 || a.T <= 1 || a.ax.kind != AX_AFFINE || getenv("ARD_NO_PERSIST")) return false;
  p.S = Hp / 8;
  p.tmb = 0;
  const int cus = lstm_cu_count();
  for (int cand = 1; cand <= 4 && !p.tmb; cand *= 2)
    if ((long)p.S * ceil_div(a.B, 32 * cand) <= cus) p.tmb = cand;
  if (!p.tmb) return false;
  p.nbb = ceil_div(a.B, 32 * p.tmb);
  p.lds = (size_t)32 * (Hp * 2 + 16) + (size_t)4 * 32 * p.tmb * 33 * 4;
  // Every unit slice reads the whole h_{t-1} of its batch rows: S * B * Hp * 2 bytes per step over the chip.
  // Device-scope loads fetch each copy from the memory side: best while that volume is small (B = 128,
  // 512 kept units: 8 MB, 6.5 us per step against 12.6 for two launches per step), 15 us per step at 33 MB
  // (1024 units).  Larger states are read through the XCD's L2 after an agent-scope acquire, so the slices
  // of one XCD share one fetch: 12.8 us per step at 33 MB against 14.6 for launches, but 7.1 against 6.5 at
  // 8 MB (every workgroup's acquire drops what its neighbours just fetched).  Beyond 40 MB nothing was
  // measured: launch per step.
  const long traffic = (long)p.S * a.B * Hp * 2;
  p.via_l2 = traffic > (12L << 20);
  const bool traffic_ok = traffic <= (40L << 20);
  return traffic_ok && p.lds <= 160 * 1024 - 1024;
}

struct PersistBwdPlan {
  int tm16, S, nbb, UW, via_l2;
  size_t lds;
};
// The backward recurrence in one launch.  Every unit slice reads the whole dG_{t+1} of its batch rows:
// S * B * 4Hp * 2 bytes per step over the chip, MB * 4Hp * 2 per workgroup.
static bool lstm_persist_bwd_plan(const LstmArgs& a, PersistBwdPlan& p) {
  const int Hp = pad8(a.Hk);
  if (a.dtype != ARD_BF16 || a.Hk <= 0 || a.T <= 1 || a.ax.kind != AX_AFFINE || getenv("ARD_NO_PERSIST")) return false;
  const int cus = lstm_cu_count();
  // Few rows and narrow slices first (most workgroups): at B = 128 with 512 kept units, per step of the whole
  // backward pass, 16 rows x 16 units (256 workgroups) 8.9 us, 16 x 32 10.4, 32 x 16 11.2, 32 x 32 13.6;
  // a launch per step 15.5.
  for (int tm = 1; tm <= 4; tm *= 2)
    for (int uw = 16; uw <= 32; uw *= 2) {
      const size_t lds = (size_t)uw * (8 * Hp + 64) + (size_t)4 * 16 * tm * (uw + 1) * 4;
      const int S = ceil_div(Hp, uw), nbb = ceil_div(a.B, 16 * tm);
      if (lds > 160 * 1024 - 1024 || (long)S * nbb > cus) continue;
      const long traffic = (long)S * a.B * 4 * Hp * 2;
      if (traffic > (40L << 20)) continue;
      // device-scope loads up to the volume they were measured best at (16 MB: 8.9 against 9.5 us through L2)
      p = PersistBwdPlan{tm, S, nbb, uw, traffic > (20L << 20), lds};
      return true;
    }
  return false;
}

template <typename T>
static int32_t lstm_fwd_t(const LstmArgs& a, const void* x, const void* W, void* h, float* c, float* gates,
                          const LstmWs& w, hipStream_t stream) {
  const int T_ = a.T, B = a.B, I = a.I, H = a.H, Hk = a.Hk, Hp = pad8(Hk), ce = 16 / a.es;
  int32_t st = lstm_prepare<T>(a, W, w, stream);
  if (st) return st;
  float* Gx = (float*)w.big;
  const int Ip = pad8(I);
  if (Hk > 0) {
    // input projection of every step: Gx[T*B x 4Hp] = x . Wx'^T
    const void* xs;
    st = lstm_padded_x<T>(a, x, w, stream, &xs);
    if (st) return st;
    GemmParams P = plain_gemm(xs, Ip, w.wxc, Ip, Gx, 4 * Hp, T_ * B, 4 * Hp, Ip, true, true, ce, true, 0.0f);
    st = run_gemm(a.dtype, true, true, P, 0, 0, stream, w.part, w.part_bytes);
    if (st) return st;
  }
  // the whole recurrence in one launch when all of its workgroups fit on the chip together
  PersistPlan pp;
  if (std::is_same<T, uint16_t>::value && lstm_persist_plan(a, pp)) {
    const int S = pp.S, nbb = pp.nbb, tmb = pp.tmb;
    const size_t lds = pp.lds;
    // (ARD_LSTM_SPIN_LIMIT: test hook for the give-up path, negative = the first wait fails; a workgroup that
    // gives up leaves normally)
    const long spin_limit = getenv("ARD_LSTM_SPIN_LIMIT") ? atol(getenv("ARD_LSTM_SPIN_LIMIT")) : 4000000L;
    LstmPersist P{Gx, (const uint16_t*)w.whc, (uint16_t*)w.hc, (uint16_t*)h, c, gates, w.sync + 1, w.sync, T_, B, H, Hk, Hp, S,
                  a.ax.off, a.ax.step, spin_limit};
    ARD_LAUNCH(lstm_zero_ints_kernel, dim3(ceil_div(S * nbb + 1, 256)), dim3(256), 0, stream, w.sync, S * nbb + 1);
    ARD_LAUNCH_CHECK("lstm_zero_ints_kernel");
    const dim3 grid((unsigned)(S * nbb));
    auto launch = [&](auto kernel) -> int32_t {
      if (lds > 65536) ARD_HIP_CHECK(raise_lds_limit((const void*)kernel, (int)lds));
      ARD_LAUNCH_NAMED("lstm_persist_fwd_kernel", kernel, grid, dim3(256), lds, stream, P);
      return ARD_OK;
    };
    if (pp.via_l2) st = tmb == 1 ? launch(lstm_persist_fwd_kernel<1, true>) : tmb == 2 ? launch(lstm_persist_fwd_kernel<2, true>)
                                                                                          : launch(lstm_persist_fwd_kernel<4, true>);
    else st = tmb == 1 ? launch(lstm_persist_fwd_kernel<1, false>) : tmb == 2 ? launch(lstm_persist_fwd_kernel<2, false>)
                                                                               : launch(lstm_persist_fwd_kernel<4, false>);
    if (st) return st;
    ARD_LAUNCH_CHECK("lstm_persist_fwd_kernel");
    return ARD_OK;
  }
  dim3 cgrid(ceil_div(H + (Hp - Hk), 256), B);
  for (int t = 0; t < T_; ++t) {
    float* Gt = Gx + (long)t * B * 4 * Hp;
    T* hc_t = (T*)w.hc + (long)t * B * Hp;
    int splits = 0;
    if (t > 0 && Hk > 0) {
      // recurrent part: G_t += h_{t-1}[kept] . Wh'^T, left as partial sums for the cell kernel when
      // the product runs on the LDS-direct kernels
      const T* hc_prev = (const T*)w.hc + (long)(t - 1) * B * Hp;
      GemmParams P = plain_gemm(hc_prev, Hp, w.whc, Hp, Gt, 4 * Hp, B, 4 * Hp, Hp, true, true, ce, true, 1.0f);
      if (run_gemm_partials(a.dtype, true, true, P, stream, w.part, w.part_bytes, &splits, &st)) {
        if (st) return st;
      } else {
        splits = 0;
        st = run_gemm(a.dtype, true, true, P, 0, 0, stream, w.part, w.part_bytes);
        if (st) return st;
      }
    }
    ARD_LAUNCH(lstm_cell_fwd_kernel<T>, cgrid, dim3(256), 0, stream, (const float*)Gt, (const float*)w.part, splits,
                       (long)B * 4 * Hp, (const int*)w.rank,
                       t > 0 ? (const float*)(c + (long)(t - 1) * B * H) : (const float*)nullptr, B, H, Hk, Hp,
                       gates + (long)t * B * 4 * H, c + (long)t * B * H, (T*)h + (long)t * B * H, hc_t);
    ARD_LAUNCH_CHECK("lstm_cell_fwd_kernel");
  }
  return ARD_OK;
}

template <typename T>
static int32_t lstm_bwd_t(const LstmArgs& a, const void* x, const void* W, const void* h, const float* c,
                          const float* gates, const void* dh, void* dx, void* dW, const LstmWs& w,
                          hipStream_t stream) {
  const int T_ = a.T, B = a.B, I = a.I, H = a.H, Hk = a.Hk, Hp = pad8(Hk), ce = 16 / a.es;
  const int Ip = pad8(I);
  int32_t st = lstm_prepare<T>(a, W, w, stream);
  if (st) return st;
  if (Hk == 0) {
    st = fill_matrix(a.dtype, dx, (long)T_ * B * I, 0.0f, stream);
    if (st) return st;
    return fill_matrix(a.dtype, dW, (long)4 * H * (I + H), 0.0f, stream);
  }
  // compact copy of the stored hidden states: hc[T*B x Hp] = h[:, kept]
  for (long r0 = 0; r0 < (long)T_ * B; r0 += 65535) {
    const long rows = (long)T_ * B - r0 < 65535 ? (long)T_ * B - r0 : 65535;
    ARD_LAUNCH(lstm_gather_h_kernel<T>, dim3(ceil_div(Hp, 256), (unsigned)rows), dim3(256), 0, stream,
                       (const T*)h + r0 * H, H, a.ax, Hp, (T*)w.hc + r0 * Hp);
    ARD_LAUNCH_CHECK("lstm_gather_h_kernel");
  }
  T* dG = (T*)w.big;
  dim3 cgrid(ceil_div(H + (Hp - Hk), 256), B);
  const float* dh_src = nullptr;  // dh_t[kept] from the product of step t+1: partial sums or w.dh_next
  int dh_splits = 0;
  PersistBwdPlan bp;
  const bool one_launch = std::is_same<T, uint16_t>::value && lstm_persist_bwd_plan(a, bp);
  if (one_launch) {
    const long spin_limit = getenv("ARD_LSTM_SPIN_LIMIT") ? atol(getenv("ARD_LSTM_SPIN_LIMIT")) : 4000000L;
    LstmPersistBwd P{gates, c, (const uint16_t*)dh, (const uint16_t*)w.whc, (uint16_t*)dG, w.sync + 1, w.sync, T_, B, H, Hk, Hp,
                     bp.S, bp.UW, a.ax.off, a.ax.step, spin_limit};
    ARD_LAUNCH(lstm_zero_ints_kernel, dim3(ceil_div(bp.S * bp.nbb + 1, 256)), dim3(256), 0, stream, w.sync, bp.S * bp.nbb + 1);
    ARD_LAUNCH_CHECK("lstm_zero_ints_kernel");
    const dim3 grid((unsigned)(bp.S * bp.nbb));
    const size_t lds = bp.lds;
    auto launch = [&](auto kernel) -> int32_t {
      if (lds > 65536) ARD_HIP_CHECK(raise_lds_limit((const void*)kernel, (int)lds));
      ARD_LAUNCH_NAMED("lstm_persist_bwd_kernel", kernel, grid, dim3(256), lds, stream, P);
      return ARD_OK;
    };
    if (bp.via_l2) st = bp.tm16 == 1 ? launch(lstm_persist_bwd_kernel<1, true>) : bp.tm16 == 2 ? launch(lstm_persist_bwd_kernel<2, true>)
                                                                                              : launch(lstm_persist_bwd_kernel<4, true>);
    else st = bp.tm16 == 1 ? launch(lstm_persist_bwd_kernel<1, false>) : bp.tm16 == 2 ? launch(lstm_persist_bwd_kernel<2, false>)
                                                                                    : launch(lstm_persist_bwd_kernel<4, false>);
    if (st) return st;
    ARD_LAUNCH_CHECK("lstm_persist_bwd_kernel");
  }
  for (int t = one_launch ? -1 : T_ - 1; t >= 0; --t) {
    T* dGt = dG + (long)t * B * 4 * Hp;
    ARD_LAUNCH(lstm_cell_bwd_kernel<T>, cgrid, dim3(256), 0, stream, gates + (long)t * B * 4 * H,
                       c + (long)t * B * H, t > 0 ? c + (long)(t - 1) * B * H : (const float*)nullptr,
                       (const T*)dh + (long)t * B * H, dh_src, dh_splits, (long)B * Hp, w.dc_next, (const int*)w.rank, B, H,
                       Hk, Hp, t == T_ - 1 ? 1 : 0, dGt);
    ARD_LAUNCH_CHECK("lstm_cell_bwd_kernel");
    if (t > 0) {
      // dh_{t-1}[kept] = dG_t . Wh'
      GemmParams P = plain_gemm(dGt, 4 * Hp, w.whc, Hp, w.dh_next, Hp, B, Hp, 4 * Hp, true, false, ce, true, 0.0f);
      if (run_gemm_partials(a.dtype, true, false, P, stream, w.part, w.part_bytes, &dh_splits, &st)) {
        if (st) return st;
        dh_src = (const float*)w.part;
      } else {
        st = run_gemm(a.dtype, true, false, P, 0, 0, stream, w.part, w.part_bytes);
        if (st) return st;
        dh_src = w.dh_next;
        dh_splits = 1;
      }
    }
  }
  {
    // dx[T*B x I] = dG . Wx'
    void* dxo = Ip != I ? (void*)w.dxp : dx;
    GemmParams P = plain_gemm(dG, 4 * Hp, w.wxc, Ip, dxo, Ip, T_ * B, Ip, 4 * Hp, true, false, ce, false, 0.0f);
    st = run_gemm(a.dtype, true, false, P, 0, 0, stream, w.part, w.part_bytes);
    if (st) return st;
    if (Ip != I) {
      const long rows_total = (long)T_ * B;
      for (long r0 = 0; r0 < rows_total; r0 += 65535) {
        const long rows = rows_total - r0 < 65535 ? rows_total - r0 : 65535;
        ARD_LAUNCH(lstm_copy_rows_kernel<T>, dim3(ceil_div(I, 256), (unsigned)rows), dim3(256), 0, stream,
                           (const T*)w.dxp + r0 * Ip, (long)Ip, I, (long)I, (T*)dx + r0 * I);
        ARD_LAUNCH_CHECK("lstm_copy_rows_kernel");
      }
    }
  }
  {
    // compact weight gradients: dwx[4Hp x I] = dG^T . x, dwh[4Hp x Hp] = dG[1:]^T . h[kept][:-1]
    const void* xs;
    st = lstm_padded_x<T>(a, x, w, stream, &xs);
    if (st) return st;
    GemmParams P = plain_gemm(dG, 4 * Hp, xs, Ip, w.dwx, Ip, 4 * Hp, Ip, T_ * B, false, false, ce, false, 0.0f);
    st = run_gemm(a.dtype, false, false, P, 0, 0, stream, w.part, w.part_bytes);
    if (st) return st;
    if (T_ > 1) {
      P = plain_gemm(dG + (long)B * 4 * Hp, 4 * Hp, w.hc, Hp, w.dwh, Hp, 4 * Hp, Hp, (T_ - 1) * B, false, false, ce, false,
                     0.0f);
      st = run_gemm(a.dtype, false, false, P, 0, 0, stream, w.part, w.part_bytes);
    } else {
      st = fill_matrix(a.dtype, w.dwh, (long)4 * Hp * Hp, 0.0f, stream);
    }
    if (st) return st;
  }
  ARD_LAUNCH(lstm_scatter_dw_kernel<T>, dim3(ceil_div(I + H, 256), 4 * H), dim3(256), 0, stream, (const T*)w.dwx,
                     (const T*)w.dwh, (const int*)w.rank, H, I, Ip, Hp, a.tiles, (T*)dW);
  ARD_LAUNCH_CHECK("lstm_scatter_dw_kernel");
  return ARD_OK;
}

}  // namespace ard

using namespace ard;

extern "C" size_t ard_lstm_workspace_bytes(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H,
                                           const ard_pattern* pat) {
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}, LstmTiles{}};
  if (lstm_check(a, pat)) return 0;
  return lstm_ws_layout(nullptr, a.es, T, B, I, H, a.Hk).total;
}

extern "C" size_t ard_lstm_status_offset(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const ard_pattern* pat) {
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}, LstmTiles{}};
  PersistPlan pp;
  if (lstm_check(a, pat) || !lstm_persist_plan(a, pp)) return (size_t)-1;
  const LstmWs w = lstm_ws_layout((char*)nullptr + 256, a.es, T, B, I, H, a.Hk);
  return (size_t)((char*)w.sync - ((char*)nullptr + 256));
}

extern "C" int32_t ard_lstm_fwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const void* x,
                                const void* W, const ard_pattern* pat, void* h, float* c, float* gates, void* ws,
                                size_t ws_bytes, void* stream) {
  BatchSuspend not_recorded;  // this entry point's kernels depend on each other: never part of a grouped launch
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}, LstmTiles{}};
  int32_t st = lstm_check(a, pat);
  if (st) return st;
  if (!x || !W || !h || !c || !gates) return fail(ARD_EINVAL, "null tensor pointer");
  LstmWs w = lstm_ws_layout((char*)ws, a.es, T, B, I, H, a.Hk);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16) return lstm_fwd_t<uint16_t>(a, x, W, h, c, gates, w, (hipStream_t)stream);
  return lstm_fwd_t<float>(a, x, W, h, c, gates, w, (hipStream_t)stream);
}

extern "C" int32_t ard_lstm_bwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const void* x,
                                const void* W, const ard_pattern* pat, const void* h, const float* c,
                                const float* gates, const void* dh, void* dx, void* dW, void* ws, size_t ws_bytes,
                                void* stream) {
  BatchSuspend not_recorded;  // this entry point's kernels depend on each other: never part of a grouped launch
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}, LstmTiles{}};
  int32_t st = lstm_check(a, pat);
  if (st) return st;
  if (!x || !W || !h || !c || !gates || !dh || !dx || !dW) return fail(ARD_EINVAL, "null tensor pointer");
  LstmWs w = lstm_ws_layout((char*)ws, a.es, T, B, I, H, a.Hk);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16) return lstm_bwd_t<uint16_t>(a, x, W, h, c, gates, dh, dx, dW, w, (hipStream_t)stream);
  return lstm_bwd_t<float>(a, x, W, h, c, gates, dh, dx, dW, w, (hipStream_t)stream);
}
