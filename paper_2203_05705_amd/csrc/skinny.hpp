// Layers with at most 16 output neurons (the classifier at the end of the MLP; Section 3.1 applies
// the row pattern to its INPUT neurons only, since output units are never dropped): bf16 kernels
// without the tile machinery that take the kept-input map themselves (a dense W is copied into LDS
// with 16-byte loads and read through the map there), so neither a gathered copy of W in memory
// nor a split contraction with a finishing pass is needed.
//
//   forward          Y[B x O]   = alpha * Xc[B x K'] . W[O x kept]^T        (16x16x32 MFMA, K' split over 4 waves)
//   backward, data   dXc[B x K'] = alpha * dY[B x O] . W[O x kept]           (vector FMAs, a thread's 16 x 8 weights in registers)
//   backward, weight dW[O x kept] = alpha * dY^T . Xc                         (16x16x32 MFMA, batch split over 4 waves)
//
// Xc / dXc are activations in the compact layout (pad8(K') columns, zero padded) or, without a
// pattern on the inputs, the dense ones.  W is the dense [O x I] matrix or its compact form.
#pragma once
#include "common.hpp"
#include "engine.hpp"

namespace ard {

typedef __bf16 sk_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float sk_f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned short sk_u16x8_t __attribute__((ext_vector_type(8)));

struct SkinnyArgs {
  const uint16_t* act;   // Xc (forward, weight gradient) / unused (data gradient)
  const uint16_t* dy;    // dY (both gradients)
  const uint16_t* w;     // W (forward, data gradient)
  uint16_t* out;
  const uint16_t* relu_src;
  int B, O, Kk;          // batch rows, output neurons, kept input neurons
  int ld_act, ld_dy, ld_w, ld_out;
  int w_compact;         // W is [pad8(O) x pad8(Kk)]; else dense with columns through `ki`
  int w_rows;            // rows of W that exist (O, or pad8(O) when compact)
  int out_cols;          // forward: columns of Y that are stored (O, or pad8(O) when compact)
  int dw_compact, I;     // weight gradient: compact output / physical inputs of the dense one
  Axis ki;               // kept input neuron j -> physical input neuron (affine)
  float alpha;
  int relu;
};

__device__ __forceinline__ sk_bf16x8_t sk_zero8() {
  const sk_u16x8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
  return __builtin_bit_cast(sk_bf16x8_t, z);
}
__device__ __forceinline__ sk_bf16x8_t sk_load8(const uint16_t* p) {
  return __builtin_bit_cast(sk_bf16x8_t, *reinterpret_cast<const uint4*>(p));
}

// Columns [p0, p0 + span) of a dense W for one workgroup, copied into LDS with 16-byte loads:
// wl[m][c] = W[m][p0 + c] for m < O (p0 and span multiples of 8).  Kept input j is then read from
// column ki(j) - p0 of the copy.
constexpr int SK_MAX_COLS = 4096;  // physical inputs a workgroup can hold (up to 16 rows of bf16 in LDS: 129 KiB of the 160)
__device__ __forceinline__ int sk_pitch(int span) { return span + 8; }  // in elements: rows start 16 bytes apart in the banks
__device__ __forceinline__ void sk_stage_w(uint16_t* wl, const SkinnyArgs& a, int p0, int span) {
  const int pitch = sk_pitch(span), chunks = span >> 3, total = a.O * chunks;
#pragma unroll 4
  for (int i = threadIdx.x; i < total; i += 256) {
    const int m = i / chunks, c = i - m * chunks;
    *reinterpret_cast<uint4*>(wl + m * pitch + c * 8) = *reinterpret_cast<const uint4*>(a.w + (long)m * a.ld_w + p0 + c * 8);
  }
  __syncthreads();
}

// Forward.  One workgroup = 16 batch rows; wave w multiplies the 32-wide slabs w, w+4, ... of
// the contraction; the four partial 16x16 tiles are summed through LDS.
// MFMA 16x16x32: lane l supplies row (l % 16), contraction chunk (l / 16) * 8 .. +8 of each
// operand and receives column (l % 16), rows 4 * (l / 16) + v of the product.
// A dense W is first gathered into LDS (sk_stage_w); a compact one is read from global memory.
__device__ __forceinline__ void skinny_fwd_body(const SkinnyArgs& a, const int bx, uint4* const sk_lds) {
  float(*part)[256] = reinterpret_cast<float(*)[256]>(sk_lds);  // [4][256]
  uint16_t* wl = reinterpret_cast<uint16_t*>(sk_lds + 256);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kc = (lane >> 4) * 8;
  const int row = bx * 16 + r;
  const bool row_ok = row < a.B, w_ok = r < a.w_rows;
  const int kpad = pad8(a.Kk);
  // a dense W: all columns up to the last kept one
  const int span = a.w_compact ? 0 : pad8(a.ki.off + (a.Kk - 1) * a.ki.step + 1);
  if (!a.w_compact) sk_stage_w(wl, a, 0, span);
  const uint16_t* xrow = a.act + (long)(row_ok ? row : 0) * a.ld_act;
  const uint16_t* wrow = a.w_compact ? a.w + (long)(w_ok ? r : 0) * a.ld_w : wl + (w_ok ? r : 0) * sk_pitch(span) + a.ki.off;
  sk_f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int k0 = wave * 32; k0 < kpad; k0 += 128) {
    const int k = k0 + kc;
    // every load is unconditional (clamped index, result discarded where it does not count), so
    // the loads of the unrolled slabs are all in flight together; rows beyond the batch read
    // row 0 and are never stored
    const bool k_ok = k < kpad;
    const int kk = k_ok ? k : kpad - 8;
    sk_bf16x8_t xa = sk_load8(xrow + kk), wb;
    if (a.w_compact) {
      wb = sk_load8(wrow + kk);
    } else {
      sk_u16x8_t g;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t t = wrow[min(kk + e, a.Kk - 1) * a.ki.step];
        g[e] = (kk + e < a.Kk) ? t : (uint16_t)0;
      }
      wb = __builtin_bit_cast(sk_bf16x8_t, g);
    }
    if (!k_ok) xa = sk_zero8();
    if (!k_ok || !w_ok) wb = sk_zero8();
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wb, acc, 0, 0, 0);
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) part[wave][lane * 4 + v] = acc[v];
  __syncthreads();
  // thread e -> batch row e / 16, output neuron e % 16
  const int m = threadIdx.x >> 4, n = threadIdx.x & 15;
  const int src = ((m >> 2) * 16 + n) * 4 + (m & 3);
  float v = a.alpha * (part[0][src] + part[1][src] + part[2][src] + part[3][src]);
  if (a.relu) v = fmaxf(v, 0.0f);
  const int orow = bx * 16 + m;
  if (orow < a.B && n < a.out_cols) a.out[(long)orow * a.ld_out + n] = n < a.O ? f32_to_bf16_bits(v) : (uint16_t)0;
}
__global__ __launch_bounds__(256) void skinny_fwd_kernel(const SkinnyArgs a) {
  extern __shared__ uint4 sk_lds_fwd[];
  skinny_fwd_body(a, (int)blockIdx.x, sk_lds_fwd);
}

// Data gradient.  One workgroup = 1024 kept inputs x SK_BD_ROWS batch rows: thread t owns the 8
// kept inputs of group t % 128 (one 16-byte store per row) for the rows of half t / 128, and keeps
// their 16 x 8 weights in registers.  The rows of dY go through LDS, the masks of a thread's rows
// are fetched before its first store: nothing in the row loop waits for memory.
constexpr int SK_BD_ROWS = 4, SK_BD_COLS = 1024;
__device__ __forceinline__ void skinny_bwd_data_body(const SkinnyArgs& a, const int bx, const int by, uint4* const sk_lds) {
  float(*dys)[16] = reinterpret_cast<float(*)[16]>(sk_lds);  // [SK_BD_ROWS][16]
  uint16_t* wl = reinterpret_cast<uint16_t*>(sk_lds + SK_BD_ROWS * 4);
  const int kpad = pad8(a.Kk);
  const int jb = bx * SK_BD_COLS;
  const int cols = min(SK_BD_COLS, kpad - jb);
  const int g = threadIdx.x & 127, half = threadIdx.x >> 7;
  const int j0 = jb + g * 8;
  const int r0 = by * SK_BD_ROWS;
  constexpr int RPT = SK_BD_ROWS / 2;  // rows per thread
  if (threadIdx.x < SK_BD_ROWS * 16) {
    const int i = threadIdx.x >> 4, m = threadIdx.x & 15;
    dys[i][m] = (r0 + i < a.B && m < a.O) ? bf16_bits_to_f32(a.dy[(long)min(r0 + i, a.B - 1) * a.ld_dy + min(m, a.O - 1)]) : 0.0f;
  }
  const bool active = g * 8 < cols;
  uint4 src[RPT];
  if (active && a.relu_src) {
#pragma unroll
    for (int i = 0; i < RPT; ++i)
      src[i] = *reinterpret_cast<const uint4*>(a.relu_src + (long)min(r0 + half * RPT + i, a.B - 1) * a.ld_out + j0);
  }
  // a dense W: the columns from this workgroup's first kept input to its last
  const int valid = min(cols, a.Kk - jb);
  const int p0 = (a.ki.off + jb * a.ki.step) & ~7;
  const int span = a.w_compact ? 0 : pad8(a.ki.off + (jb + valid - 1) * a.ki.step + 1) - p0;
  if (!a.w_compact) sk_stage_w(wl, a, p0, span);
  else __syncthreads();
  if (!active) return;
  float w[16][8];
#pragma unroll
  for (int m = 0; m < 16; ++m) {
    if (a.w_compact) {
      uint4 q = make_uint4(0, 0, 0, 0);
      if (m < a.O) q = *reinterpret_cast<const uint4*>(a.w + (long)m * a.ld_w + j0);
      const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) w[m][e] = bf16_bits_to_f32((uint16_t)(u[e >> 1] >> ((e & 1) * 16)));
    } else {
      const uint16_t* wr = wl + min(m, a.O - 1) * sk_pitch(span) + (a.ki.off - p0);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t t = wr[min(j0 + e, a.Kk - 1) * a.ki.step];
        w[m][e] = (m < a.O && j0 + e < a.Kk) ? bf16_bits_to_f32(t) : 0.0f;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int ri = half * RPT + i, row = r0 + ri;
    if (row >= a.B) break;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const float gy = dys[ri][m];  // zero beyond the layer's outputs
#pragma unroll
      for (int e = 0; e < 8; ++e) s[e] = fmaf(gy, w[m][e], s[e]);
    }
    uint32_t mask[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
    if (a.relu_src) {
      const uint32_t u[4] = {src[i].x, src[i].y, src[i].z, src[i].w};
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const float lo = bf16_bits_to_f32((uint16_t)u[h]), hi = bf16_bits_to_f32((uint16_t)(u[h] >> 16));
        mask[h] = (lo > 0.0f ? 0xffffu : 0u) | (hi > 0.0f ? 0xffff0000u : 0u);
      }
    }
    uint32_t bits[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bits[e] = (j0 + e < a.Kk) ? f32_to_bf16_bits(a.alpha * s[e]) : 0u;  // padding stays +0.0
    uint4 o;
    o.x = (bits[0] | (bits[1] << 16)) & mask[0];
    o.y = (bits[2] | (bits[3] << 16)) & mask[1];
    o.z = (bits[4] | (bits[5] << 16)) & mask[2];
    o.w = (bits[6] | (bits[7] << 16)) & mask[3];
    *reinterpret_cast<uint4*>(a.out + (long)row * a.ld_out + j0) = o;
  }
}
__global__ __launch_bounds__(256) void skinny_bwd_data_kernel(const SkinnyArgs a) {
  extern __shared__ uint4 sk_lds_bd[];
  skinny_bwd_data_body(a, (int)blockIdx.x, (int)blockIdx.y, sk_lds_bd);
}

// Weight gradient.  One workgroup = 16 kept inputs; wave w contracts the 32-row slabs w, w+4, ...
// of the batch.  Operand rows run along the batch here, so a lane gathers its 8 values of dY
// (output neuron l % 16) and of Xc (kept input l % 16) with 2-byte loads; the 16 lanes of a group
// read 32 contiguous bytes of each row.  The workgroup also writes the zeros of the dropped
// inputs between its first kept input and the next workgroup's.
__device__ __forceinline__ void skinny_bwd_weight_body(const SkinnyArgs& a, const int bx, uint4* const sk_lds) {
  float(*part)[256] = reinterpret_cast<float(*)[256]>(sk_lds);  // [4][256]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, rc = (lane >> 4) * 8;
  const int j = bx * 16 + c;  // kept input of this lane (B operand); output neuron c (A operand)
  const int xcols = pad8(a.Kk);
  const bool j_ok = j < a.Kk, m_ok = c < a.O;
  sk_f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int r0 = wave * 32; r0 < a.B; r0 += 128) {
    sk_u16x8_t ga, gb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int row = r0 + rc + e;
      const bool ok = row < a.B;
      const long rr = ok ? row : a.B - 1;  // unconditional loads: all sixteen are in flight together
      const uint16_t ta = a.dy[rr * a.ld_dy + (m_ok ? c : 0)];
      const uint16_t tb = a.act[rr * a.ld_act + (j_ok ? j : 0)];
      ga[e] = (ok && m_ok) ? ta : (uint16_t)0;
      gb[e] = (ok && j_ok) ? tb : (uint16_t)0;
    }
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(sk_bf16x8_t, ga), __builtin_bit_cast(sk_bf16x8_t, gb),
                                                  acc, 0, 0, 0);
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) part[wave][lane * 4 + v] = acc[v];
  __syncthreads();
  // thread e -> output neuron e / 16, kept input bx * 16 + e % 16
  const int m = threadIdx.x >> 4, n = threadIdx.x & 15;
  const int src = ((m >> 2) * 16 + n) * 4 + (m & 3);
  const float v = a.alpha * (part[0][src] + part[1][src] + part[2][src] + part[3][src]);
  const int jj = bx * 16 + n;
  if (a.dw_compact) {
    if (m < pad8(a.O) && jj < xcols) a.out[(long)m * a.ld_out + jj] = (m < a.O && jj < a.Kk) ? f32_to_bf16_bits(v) : (uint16_t)0;
    return;
  }
  if (m >= a.O) return;
  // physical columns owned by this workgroup: from its first kept input (from 0 for the first
  // workgroup) up to the next workgroup's first kept input (up to I for the last)
  const int jb = bx * 16, je = min(jb + 16, a.Kk);
  const int p_lo = bx == 0 ? 0 : a.ki.off + jb * a.ki.step;
  const int p_hi = je >= a.Kk ? a.I : a.ki.off + je * a.ki.step;
  uint16_t* orow = a.out + (long)m * a.ld_out;
  if (a.ki.step != 1 || a.ki.off != 0) {
    for (int p = p_lo + n; p < p_hi; p += 16) {
      const int d = p - a.ki.off;
      const bool kept = d >= 0 && d % a.ki.step == 0 && d / a.ki.step < a.Kk;
      if (!kept) orow[p] = 0;
    }
  }
  if (jj < a.Kk) orow[a.ki.off + jj * a.ki.step] = f32_to_bf16_bits(v);
}
__global__ __launch_bounds__(256) void skinny_bwd_weight_kernel(const SkinnyArgs a) {
  extern __shared__ uint4 sk_lds_bw[];
  skinny_bwd_weight_body(a, (int)blockIdx.x, sk_lds_bw);
}

enum { GK_SKINNY_FWD = 100, GK_SKINNY_BWD_DATA = 101, GK_SKINNY_BWD_WEIGHT = 102 };
// records the launch in the open batch of this thread (gemm.hip); false: no batch is open, launch now
static bool batch_push_skinny(int kind, const SkinnyArgs& a, int gx, int gy, size_t lds);

static bool sk_aligned(const void* p, long ld) { return ((uintptr_t)p & 15) == 0 && (ld % 8) == 0; }

// op 0: forward (p0 = X, p1 = W, out = Y); op 1: data gradient (p0 = dY, p1 = W, out = dX);
// op 2: weight gradient (p0 = dY, p1 = X, out = dW).  Returns false when the layer is not one of
// the shapes above (nothing launched); otherwise *status holds the launch result.
static bool try_skinny(int op, int32_t dtype, int B, int I, int O, const void* p0, const void* p1, void* out, const Axis& ao,
                const Axis& ai, int32_t flags, float alpha, float beta, int relu, const void* relu_src, hipStream_t stream,
                int32_t* status) {
  *status = ARD_OK;
  if (dtype != ARD_BF16 || dev_knobs().no_fast) return false;
  if (O > 16 || O < 1 || B < 1) return false;
  if (!(ao.kind == AX_AFFINE && ao.off == 0 && ao.step == 1 && ao.n == O)) return false;  // outputs are never dropped here
  if (ai.kind != AX_AFFINE || ai.n < 1 || ai.step < 1) return false;
  if (beta != 0.0f) return false;
  const bool ident_in = ai.off == 0 && ai.step == 1;
  const bool in_c = (flags & ARD_IN_COMPACT) != 0, out_c = (flags & ARD_OUT_COMPACT) != 0;
  const bool w_c = (flags & ARD_W_COMPACT) != 0;
  // the activation on the input side must hold the kept inputs side by side
  if (!in_c && !ident_in) return false;
  const int ld_in = in_c ? pad8(ai.n) : I;   // Xc / dXc
  const int ld_o = out_c ? pad8(O) : O;      // Y / dY
  SkinnyArgs a{};
  a.B = B;
  a.O = O;
  a.Kk = ai.n;
  a.I = I;
  a.ki = ai;
  a.alpha = alpha;
  a.relu = relu;
  a.out = (uint16_t*)out;
  if (op == 0 || op == 1) {
    a.w = (const uint16_t*)p1;
    a.w_compact = w_c;
    a.ld_w = w_c ? pad8(ai.n) : I;
    a.w_rows = w_c ? pad8(O) : O;
    if (w_c && !sk_aligned(p1, a.ld_w)) return false;
  }
  if (op == 0) {
    if (!sk_aligned(p0, ld_in)) return false;
    a.act = (const uint16_t*)p0;
    a.ld_act = ld_in;
    a.ld_out = ld_o;
    a.out_cols = ld_o;
    if (!w_c && (I > SK_MAX_COLS || (I % 8) || ((uintptr_t)p1 & 15))) return false;
    const size_t lds = 4096 + (w_c ? 0 : (size_t)O * (pad8(ai.off + (ai.n - 1) * ai.step + 1) + 8) * 2);
    static thread_local bool raised = false;
    if (!raised && lds > 65536) {
      hipError_t e = ard::raise_lds_limit((const void*)skinny_fwd_kernel, 4096 + 16 * (SK_MAX_COLS + 8) * 2);  // the most any qualifying layer asks for
      if (e != hipSuccess) return false;
      raised = !dry_run();
    }
    if (!batch_push_skinny(GK_SKINNY_FWD, a, ceil_div(B, 16), 1, lds))
      ARD_LAUNCH(skinny_fwd_kernel, dim3((unsigned)ceil_div(B, 16)), dim3(256), lds, stream, a);
  } else if (op == 1) {
    if (!sk_aligned(out, ld_in) || (relu_src && !sk_aligned(relu_src, ld_in))) return false;
    if (!in_c && (I % 8)) return false;
    a.dy = (const uint16_t*)p0;
    a.ld_dy = ld_o;
    a.ld_out = ld_in;
    a.relu_src = (const uint16_t*)relu_src;
    if (ceil_div(B, SK_BD_ROWS) > 65535) return false;
    if (!w_c && (I > SK_MAX_COLS || (I % 8) || ((uintptr_t)p1 & 15))) return false;
    const size_t lds = SK_BD_ROWS * 64 + (w_c ? 0 : (size_t)O * (pad8(I) + 16) * 2);
    static thread_local bool raised_bd = false;
    if (!raised_bd && lds > 65536) {
      hipError_t e = ard::raise_lds_limit((const void*)skinny_bwd_data_kernel, SK_BD_ROWS * 64 + 16 * (SK_MAX_COLS + 16) * 2);
      if (e != hipSuccess) return false;
      raised_bd = !dry_run();
    }
    if (!batch_push_skinny(GK_SKINNY_BWD_DATA, a, ceil_div(pad8(ai.n), SK_BD_COLS), ceil_div(B, SK_BD_ROWS), lds))
      ARD_LAUNCH(skinny_bwd_data_kernel, dim3((unsigned)ceil_div(pad8(ai.n), SK_BD_COLS), (unsigned)ceil_div(B, SK_BD_ROWS)),
                 dim3(256), lds, stream, a);
  } else {
    a.dy = (const uint16_t*)p0;
    a.ld_dy = ld_o;
    a.act = (const uint16_t*)p1;
    a.ld_act = ld_in;
    a.dw_compact = (flags & ARD_DW_COMPACT) != 0;
    a.ld_out = a.dw_compact ? pad8(ai.n) : I;
    if (!batch_push_skinny(GK_SKINNY_BWD_WEIGHT, a, ceil_div(pad8(ai.n), 16), 1, 4096))
      ARD_LAUNCH(skinny_bwd_weight_kernel, dim3((unsigned)ceil_div(pad8(ai.n), 16)), dim3(256), 4096, stream, a);
  }
  hipError_t e = ard::launch_status();
  if (e != hipSuccess) *status = fail(ARD_EHIP, "launch of a skinny-layer kernel failed: %s", hipGetErrorString(e));
  return true;
}

}  // namespace ard
