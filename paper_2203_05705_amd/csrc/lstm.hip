// LSTM layer under a row pattern on its hidden units (Section 7.2.3: the LSTM runs as
// matrix multiplications, so the same patterns apply).
//
// Fused weight W[4H x (I+H)], gate blocks i, f, g, o of H rows, columns [x | h].
// A dropped unit has no gate rows and no recurrent column in any product:
//   - the input projection of all T steps is one gathered GEMM over the kept gate rows,
//   - the recurrent weight of the kept units is compacted once per sequence
//     (W_h'[4H' x H']), and each step multiplies the compact hidden state by it,
//   - the pointwise cell kernels run over physical units and write zeros for dropped ones.
#include "engine.hpp"
#include "pattern.hpp"

namespace ard {

// rank[u] = compact index of unit u or -1; grows[g*Hk + j] = g*H + unit(j)
__global__ __launch_bounds__(1024) void lstm_setup_kernel(Axis ax, int H, int* rank, int* grows) {
  for (int u = threadIdx.x; u < H; u += 1024) rank[u] = -1;
  __syncthreads();
  const int Hk = ax.n;
  for (int j = threadIdx.x; j < Hk; j += 1024) {
    int u = ax_phys(ax, j);
    rank[u] = j;
#pragma unroll
    for (int g = 0; g < 4; ++g) grows[g * Hk + j] = g * H + u;
  }
}

// out[r][j] = src[rowlist ? rowlist[r] : r][col0 + unit(j)]
template <typename T>
__global__ void gather_cols_kernel(const T* src, long ld, const int* rowlist, int col0, Axis ax, T* out, int rows) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int r = blockIdx.y;
  if (j < ax.n && r < rows) {
    long pr = rowlist ? rowlist[r] : r;
    out[(long)r * ax.n + j] = src[pr * ld + col0 + ax_phys(ax, j)];
  }
}

__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

// One time step, forward.  G: compact pre-activations [B x 4Hk] (fp32).  Writes the
// activated gates [B x 4H], c [B x H] (fp32), h [B x H] (dtype) with zeros for dropped
// units, and the compact h [B x Hk] that feeds the next step's product.
template <typename T>
__global__ void lstm_cell_fwd_kernel(const float* G, const int* rank, const float* c_prev, int B, int H, int Hk,
                                     float* gates, float* c, T* h, T* hc) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (u >= H) return;
  const int j = rank[u];
  float gi = 0, gf = 0, gg = 0, go = 0, cv = 0, hv = 0;
  if (j >= 0) {
    const float* g = G + (long)b * 4 * Hk;
    gi = sigmoidf_(g[j]);
    gf = sigmoidf_(g[Hk + j]);
    gg = tanhf(g[2 * Hk + j]);
    go = sigmoidf_(g[3 * Hk + j]);
    const float cp = c_prev ? c_prev[(long)b * H + u] : 0.0f;
    cv = gf * cp + gi * gg;
    hv = go * tanhf(cv);
    hc[(long)b * Hk + j] = ElemTraits<T>::from_f32(hv);
  }
  float* ga = gates + (long)b * 4 * H;
  ga[u] = gi;
  ga[H + u] = gf;
  ga[2 * H + u] = gg;
  ga[3 * H + u] = go;
  c[(long)b * H + u] = cv;
  h[(long)b * H + u] = ElemTraits<T>::from_f32(hv);
}

// One time step, backward.  dh_next: compact [B x Hk] fp32 (NULL at the last step);
// dc_next: [B x H] fp32, read unless `first`, then overwritten.  Writes the compact gate
// gradient dG [B x 4Hk] in the storage dtype.
template <typename T>
__global__ void lstm_cell_bwd_kernel(const float* gates, const float* c, const float* c_prev, const T* dh_ext,
                                     const float* dh_next, float* dc_next, const int* rank, int B, int H, int Hk,
                                     int first, T* dG) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (u >= H) return;
  const int j = rank[u];
  if (j < 0) return;
  const float* ga = gates + (long)b * 4 * H;
  const float gi = ga[u], gf = ga[H + u], gg = ga[2 * H + u], go = ga[3 * H + u];
  const float tc = tanhf(c[(long)b * H + u]);
  const float cp = c_prev ? c_prev[(long)b * H + u] : 0.0f;
  float dh = ElemTraits<T>::to_f32(dh_ext[(long)b * H + u]);
  if (dh_next) dh += dh_next[(long)b * Hk + j];
  float dc = dh * go * (1.0f - tc * tc);
  if (!first) dc += dc_next[(long)b * H + u];
  T* d = dG + (long)b * 4 * Hk;
  d[j] = ElemTraits<T>::from_f32(dc * gg * gi * (1.0f - gi));
  d[Hk + j] = ElemTraits<T>::from_f32(dc * cp * gf * (1.0f - gf));
  d[2 * Hk + j] = ElemTraits<T>::from_f32(dc * gi * (1.0f - gg * gg));
  d[3 * Hk + j] = ElemTraits<T>::from_f32(dh * tc * go * (1.0f - go));
  dc_next[(long)b * H + u] = dc * gf;
}

static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

struct LstmWs {
  int* rank;
  int* grows;
  char* whc;     // [4Hk x Hk] dtype
  char* hc;      // [T*B x Hk] dtype
  char* big;     // fwd: Gx [T*B x 4Hk] fp32; bwd: dG [T*B x 4Hk] dtype
  float* dh_next;  // [B x Hk]
  float* dc_next;  // [B x H]
  size_t total;
};

static LstmWs lstm_ws_layout(char* base, int es, int T, int B, int H, int Hk) {
  LstmWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes ? bytes : 1, 256);
    return p;
  };
  w.rank = (int*)take((size_t)H * 4);
  w.grows = (int*)take((size_t)4 * Hk * 4);
  w.whc = take((size_t)4 * Hk * Hk * es);
  w.hc = take((size_t)T * B * Hk * es);
  w.big = take((size_t)T * B * 4 * Hk * 4);
  w.dh_next = (float*)take((size_t)B * Hk * 4);
  w.dc_next = (float*)take((size_t)B * H * 4);
  w.total = off;
  return w;
}

struct LstmArgs {
  int32_t dtype, T, B, I, H, Hk, es;
  Axis ax;
};

static int32_t lstm_check(LstmArgs& a, const ard_pattern* pat) {
  if (a.dtype != ARD_F32 && a.dtype != ARD_BF16) return fail(ARD_EDTYPE, "unknown dtype %d", a.dtype);
  if (a.T <= 0 || a.B <= 0 || a.I <= 0 || a.H <= 0)
    return fail(ARD_ESHAPE, "T, B, I, H must be positive (got %d, %d, %d, %d)", a.T, a.B, a.I, a.H);
  if (pat && pat->kind == ARD_PAT_TILE) return fail(ARD_EINVAL, "the LSTM takes a ROW, LIST or NONE pattern");
  int32_t st = check_pattern(pat, a.H, "pat");
  if (st) return st;
  a.ax = axis_of_pattern(pat, a.H);
  a.Hk = a.ax.n;
  a.es = a.dtype == ARD_BF16 ? 2 : 4;
  if ((long)a.T * a.B > 0x7fffffffL / 4 || (long)a.B > 65535) return fail(ARD_ESHAPE, "T*B or B too large");
  return ARD_OK;
}

template <typename T>
static int32_t lstm_prepare(const LstmArgs& a, const void* W, const LstmWs& w, hipStream_t stream) {
  hipLaunchKernelGGL(lstm_setup_kernel, dim3(1), dim3(1024), 0, stream, a.ax, a.H, w.rank, w.grows);
  ARD_LAUNCH_CHECK("lstm_setup_kernel");
  if (a.Hk > 0) {
    dim3 grid(ceil_div(a.Hk, 256), 4 * a.Hk);
    hipLaunchKernelGGL(gather_cols_kernel<T>, grid, dim3(256), 0, stream, (const T*)W, (long)(a.I + a.H),
                       (const int*)w.grows, a.I, a.ax, (T*)w.whc, 4 * a.Hk);
    ARD_LAUNCH_CHECK("gather_cols_kernel");
  }
  return ARD_OK;
}

template <typename T>
static int32_t lstm_fwd_t(const LstmArgs& a, const void* x, const void* W, void* h, float* c, float* gates,
                          const LstmWs& w, hipStream_t stream) {
  const int T_ = a.T, B = a.B, I = a.I, H = a.H, Hk = a.Hk, ce = 16 / a.es;
  int32_t st = lstm_prepare<T>(a, W, w, stream);
  if (st) return st;
  float* Gx = (float*)w.big;
  if (Hk > 0) {
    // input projection of every step: Gx[T*B x 4Hk] = x . W[kept gate rows, 0:I]^T
    GemmParams P{};
    P.A = Operand{x, I, axis_identity(T_ * B), (I % ce) == 0 && al16(x)};
    P.B = Operand{W, I + H, axis_list(w.grows, 4 * Hk, 4 * H), (I % ce) == 0 && ((I + H) % ce) == 0 && al16(W)};
    P.k = axis_identity(I);
    P.C.p = Gx;
    P.C.ld = 4 * Hk;
    P.C.rm = axis_identity(T_ * B);
    P.C.cn = axis_identity(4 * Hk);
    P.C.out_f32 = 1;
    P.C.alpha = 1.0f;
    P.M = T_ * B;
    P.N = 4 * Hk;
    st = run_gemm(a.dtype, true, true, P, 0, 0, stream);
    if (st) return st;
  }
  dim3 cgrid(ceil_div(H, 256), B);
  for (int t = 0; t < T_; ++t) {
    float* Gt = Gx + (long)t * B * 4 * Hk;
    T* hc_t = (T*)w.hc + (long)t * B * Hk;
    if (t > 0 && Hk > 0) {
      // recurrent part: G_t += h_{t-1}[kept] . W_h'^T
      const T* hc_prev = (const T*)w.hc + (long)(t - 1) * B * Hk;
      GemmParams P{};
      P.A = Operand{hc_prev, Hk, axis_identity(B), (Hk % ce) == 0 && al16(hc_prev)};
      P.B = Operand{w.whc, Hk, axis_identity(4 * Hk), (Hk % ce) == 0};
      P.k = axis_identity(Hk);
      P.C.p = Gt;
      P.C.ld = 4 * Hk;
      P.C.rm = axis_identity(B);
      P.C.cn = axis_identity(4 * Hk);
      P.C.out_f32 = 1;
      P.C.alpha = 1.0f;
      P.C.beta = 1.0f;
      P.M = B;
      P.N = 4 * Hk;
      st = run_gemm(a.dtype, true, true, P, 0, 0, stream);
      if (st) return st;
    }
    hipLaunchKernelGGL(lstm_cell_fwd_kernel<T>, cgrid, dim3(256), 0, stream, (const float*)Gt, (const int*)w.rank,
                       t > 0 ? (const float*)(c + (long)(t - 1) * B * H) : (const float*)nullptr, B, H, Hk,
                       gates + (long)t * B * 4 * H, c + (long)t * B * H, (T*)h + (long)t * B * H, hc_t);
    ARD_LAUNCH_CHECK("lstm_cell_fwd_kernel");
  }
  return ARD_OK;
}

template <typename T>
static int32_t lstm_bwd_t(const LstmArgs& a, const void* x, const void* W, const void* h, const float* c,
                          const float* gates, const void* dh, void* dx, void* dW, const LstmWs& w,
                          hipStream_t stream) {
  const int T_ = a.T, B = a.B, I = a.I, H = a.H, Hk = a.Hk, ce = 16 / a.es;
  int32_t st = lstm_prepare<T>(a, W, w, stream);
  if (st) return st;
  if (Hk == 0) {
    st = fill_matrix(a.dtype, dx, (long)T_ * B * I, 0.0f, stream);
    if (st) return st;
    return fill_matrix(a.dtype, dW, (long)4 * H * (I + H), 0.0f, stream);
  }
  // compact copy of the stored hidden states: hc[T*B x Hk] = h[:, kept]
  {
    dim3 grid(ceil_div(Hk, 256), T_ * B);
    if ((long)T_ * B > 65535) return fail(ARD_ESHAPE, "T*B above 65535 is not supported by the LSTM backward");
    hipLaunchKernelGGL(gather_cols_kernel<T>, grid, dim3(256), 0, stream, (const T*)h, (long)H, (const int*)nullptr, 0,
                       a.ax, (T*)w.hc, T_ * B);
    ARD_LAUNCH_CHECK("gather_cols_kernel");
  }
  T* dG = (T*)w.big;
  dim3 cgrid(ceil_div(H, 256), B);
  for (int t = T_ - 1; t >= 0; --t) {
    T* dGt = dG + (long)t * B * 4 * Hk;
    hipLaunchKernelGGL(lstm_cell_bwd_kernel<T>, cgrid, dim3(256), 0, stream, gates + (long)t * B * 4 * H,
                       c + (long)t * B * H, t > 0 ? c + (long)(t - 1) * B * H : (const float*)nullptr,
                       (const T*)dh + (long)t * B * H, t < T_ - 1 ? (const float*)w.dh_next : (const float*)nullptr,
                       w.dc_next, (const int*)w.rank, B, H, Hk, t == T_ - 1 ? 1 : 0, dGt);
    ARD_LAUNCH_CHECK("lstm_cell_bwd_kernel");
    if (t > 0) {
      // dh_{t-1}[kept] = dG_t . W_h'
      GemmParams P{};
      P.A = Operand{dGt, 4 * Hk, axis_identity(B), ((4 * Hk) % ce) == 0 && al16(dGt)};
      P.B = Operand{w.whc, Hk, axis_identity(Hk), 0};
      P.k = axis_identity(4 * Hk);
      P.C.p = w.dh_next;
      P.C.ld = Hk;
      P.C.rm = axis_identity(B);
      P.C.cn = axis_identity(Hk);
      P.C.out_f32 = 1;
      P.C.alpha = 1.0f;
      P.M = B;
      P.N = Hk;
      P.B.vec = operand_vec_ok(P.B, false, P.k, ce);
      st = run_gemm(a.dtype, true, false, P, 0, 0, stream);
      if (st) return st;
    }
  }
  // dx[T*B x I] = dG . W[kept gate rows, 0:I]
  {
    GemmParams P{};
    P.A = Operand{dG, 4 * Hk, axis_identity(T_ * B), ((4 * Hk) % ce) == 0 && al16(dG), 1};
    P.B = Operand{W, I + H, axis_identity(I), 0};
    P.k = axis_list(w.grows, 4 * Hk, 4 * H);
    P.C.p = dx;
    P.C.ld = I;
    P.C.rm = axis_identity(T_ * B);
    P.C.cn = axis_identity(I);
    P.C.alpha = 1.0f;
    P.M = T_ * B;
    P.N = I;
    P.B.vec = operand_vec_ok(P.B, false, P.k, ce);
    st = run_gemm(a.dtype, true, false, P, 0, 0, stream);
    if (st) return st;
  }
  // dW[kept gate rows, 0:I] = dG^T . x ; the other rows of these columns get zeros
  {
    GemmParams P{};
    P.A = Operand{dG, 4 * Hk, axis_identity(4 * Hk), 0};
    P.B = Operand{x, I, axis_identity(I), 0};
    P.k = axis_identity(T_ * B);
    P.C.p = dW;
    P.C.ld = I + H;
    P.C.rm = axis_list(w.grows, 4 * Hk, 4 * H);
    P.C.cn = axis_identity(I);
    P.C.fill = 1;
    P.C.alpha = 1.0f;
    P.M = 4 * Hk;
    P.N = I;
    P.A.vec = operand_vec_ok(P.A, false, P.k, ce);
    P.B.vec = operand_vec_ok(P.B, false, P.k, ce);
    st = run_gemm(a.dtype, false, false, P, 0, 0, stream);
    if (st) return st;
  }
  // dW[kept gate rows, I + kept units] = dG[1:]^T . h[kept][:-1] ; zeros elsewhere in columns I..I+H
  {
    GemmParams P{};
    P.A = Operand{dG + (long)B * 4 * Hk, 4 * Hk, axis_identity(4 * Hk), 0};
    P.B = Operand{w.hc, Hk, axis_identity(Hk), 0};
    P.k = axis_identity((T_ - 1) * B);
    P.C.p = (T*)dW + I;
    P.C.ld = I + H;
    P.C.rm = axis_list(w.grows, 4 * Hk, 4 * H);
    P.C.cn = a.ax;
    P.C.fill = 1;
    P.C.alpha = 1.0f;
    P.M = 4 * Hk;
    P.N = Hk;
    P.A.vec = operand_vec_ok(P.A, false, P.k, ce);
    P.B.vec = operand_vec_ok(P.B, false, P.k, ce);
    st = run_gemm(a.dtype, false, false, P, 0, 0, stream);
    if (st) return st;
  }
  return ARD_OK;
}

}  // namespace ard

using namespace ard;

extern "C" size_t ard_lstm_workspace_bytes(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H,
                                           const ard_pattern* pat) {
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}};
  if (lstm_check(a, pat)) return 0;
  return lstm_ws_layout(nullptr, a.es, T, B, H, a.Hk).total;
}

extern "C" int32_t ard_lstm_fwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const void* x,
                                const void* W, const ard_pattern* pat, void* h, float* c, float* gates, void* ws,
                                size_t ws_bytes, void* stream) {
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}};
  int32_t st = lstm_check(a, pat);
  if (st) return st;
  if (!x || !W || !h || !c || !gates) return fail(ARD_EINVAL, "null tensor pointer");
  LstmWs w = lstm_ws_layout((char*)ws, a.es, T, B, H, a.Hk);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16) return lstm_fwd_t<uint16_t>(a, x, W, h, c, gates, w, (hipStream_t)stream);
  return lstm_fwd_t<float>(a, x, W, h, c, gates, w, (hipStream_t)stream);
}

extern "C" int32_t ard_lstm_bwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const void* x,
                                const void* W, const ard_pattern* pat, const void* h, const float* c,
                                const float* gates, const void* dh, void* dx, void* dW, void* ws, size_t ws_bytes,
                                void* stream) {
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}};
  int32_t st = lstm_check(a, pat);
  if (st) return st;
  if (!x || !W || !h || !c || !gates || !dh || !dx || !dW) return fail(ARD_EINVAL, "null tensor pointer");
  LstmWs w = lstm_ws_layout((char*)ws, a.es, T, B, H, a.Hk);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16) return lstm_bwd_t<uint16_t>(a, x, W, h, c, gates, dh, dx, dW, w, (hipStream_t)stream);
  return lstm_bwd_t<float>(a, x, W, h, c, gates, dh, dx, dW, w, (hipStream_t)stream);
}
