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
#include "engine.hpp"
#include "pattern.hpp"

namespace ard {

// rank[u] = compact index of unit u or -1
__global__ __launch_bounds__(1024) void lstm_setup_kernel(Axis ax, int H, int* rank) {
  for (int u = threadIdx.x; u < H; u += 1024) rank[u] = -1;
  __syncthreads();
  for (int j = threadIdx.x; j < ax.n; j += 1024) rank[ax_phys(ax, j)] = j;
}

// out[g*Hp + j][q] = W[(g*H + unit(j)) * ldw + col(q)] for kept j, 0 at the padding.
// cols == 0: the input columns, q < ncol identity; cols == 1: the recurrent columns,
// q < Hp -> I + unit(q) (0 at the padding); out has `ldo` columns.
template <typename T>
__global__ void lstm_gather_w_kernel(const T* W, long ldw, Axis ax, int H, int I, int Hp, int recurrent, int ldo, T* out) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  const int r = blockIdx.y;  // compact gate row
  if (q >= ldo) return;
  const int g = r / Hp, j = r - g * Hp;
  T v = (T)0;
  if (j < ax.n) {
    const long row = (long)(g * H + ax_phys(ax, j)) * ldw;
    if (!recurrent) v = W[row + q];
    else if (q < ax.n) v = W[row + I + ax_phys(ax, q)];
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

// dW[(g*H + u)][q] from the compact gradients dwx[4Hp x I] and dwh[4Hp x Hp]; +0.0 for every
// row of a dropped unit and every recurrent column of a dropped unit.
template <typename T>
__global__ void lstm_scatter_dw_kernel(const T* dwx, const T* dwh, const int* rank, int H, int I, int Hp, T* dW) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  const int p = blockIdx.y;  // physical gate row
  if (q >= I + H) return;
  const int g = p / H, u = p - g * H;
  const int j = rank[u];
  T v = (T)0;
  if (j >= 0) {
    const long r = (long)g * Hp + j;
    if (q < I) {
      v = dwx[r * I + q];
    } else {
      const int jv = rank[q - I];
      if (jv >= 0) v = dwh[r * Hp + jv];
    }
  }
  dW[(long)p * (I + H) + q] = v;
}

static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

struct LstmWs {
  int* rank;
  char* wxc;     // [4Hp x I] dtype
  char* whc;     // [4Hp x Hp] dtype
  char* hc;      // [T*B x Hp] dtype
  char* big;     // fwd: Gx [T*B x 4Hp] fp32; bwd: dG [T*B x 4Hp] dtype
  float* dh_next;  // [B x Hp]
  float* dc_next;  // [B x H]
  char* dwx;     // [4Hp x I] dtype
  char* dwh;     // [4Hp x Hp] dtype
  char* part;    // fp32 partial sums of split products
  size_t part_bytes;
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
  w.wxc = take(4 * Hp * I * es);
  w.whc = take(4 * Hp * Hp * es);
  w.hc = take((size_t)T * B * Hp * es);
  w.big = take((size_t)T * B * 4 * Hp * 4);
  w.dh_next = (float*)take((size_t)B * Hp * 4);
  w.dc_next = (float*)take((size_t)B * H * 4);
  w.dwx = take(4 * Hp * I * es);
  w.dwh = take(4 * Hp * Hp * es);
  // room for the partial sums of any product here split 8 ways, capped at 256 MiB
  size_t big = 4 * Hp * (size_t)(I > (int)Hp ? I : (int)Hp);
  if ((size_t)B * 4 * Hp > big) big = (size_t)B * 4 * Hp;
  w.part_bytes = big * 4 * 8;
  if (w.part_bytes > ((size_t)256 << 20)) w.part_bytes = (size_t)256 << 20;
  w.part = take(w.part_bytes);
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
  if ((long)a.T * a.B > 0x7fffffffL / 4 || (long)a.B > 65535 || (long)a.T * a.B > 65535 * 64L)
    return fail(ARD_ESHAPE, "T*B or B too large");
  if (4L * a.H > 65535) return fail(ARD_ESHAPE, "more than 16383 hidden units");
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
    ARD_LAUNCH(lstm_gather_w_kernel<T>, dim3(ceil_div(a.I, 256), 4 * Hp), dim3(256), 0, stream, (const T*)W,
                       (long)(a.I + a.H), a.ax, a.H, a.I, Hp, 0, a.I, (T*)w.wxc);
    ARD_LAUNCH_CHECK("lstm_gather_w_kernel");
    ARD_LAUNCH(lstm_gather_w_kernel<T>, dim3(ceil_div(Hp, 256), 4 * Hp), dim3(256), 0, stream, (const T*)W,
                       (long)(a.I + a.H), a.ax, a.H, a.I, Hp, 1, Hp, (T*)w.whc);
    ARD_LAUNCH_CHECK("lstm_gather_w_kernel");
  }
  return ARD_OK;
}

template <typename T>
static int32_t lstm_fwd_t(const LstmArgs& a, const void* x, const void* W, void* h, float* c, float* gates,
                          const LstmWs& w, hipStream_t stream) {
  const int T_ = a.T, B = a.B, I = a.I, H = a.H, Hk = a.Hk, Hp = pad8(Hk), ce = 16 / a.es;
  int32_t st = lstm_prepare<T>(a, W, w, stream);
  if (st) return st;
  float* Gx = (float*)w.big;
  if (Hk > 0) {
    // input projection of every step: Gx[T*B x 4Hp] = x . Wx'^T
    GemmParams P = plain_gemm(x, I, w.wxc, I, Gx, 4 * Hp, T_ * B, 4 * Hp, I, true, true, ce, true, 0.0f);
    st = run_gemm(a.dtype, true, true, P, 0, 0, stream, w.part, w.part_bytes);
    if (st) return st;
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
  for (int t = T_ - 1; t >= 0; --t) {
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
    GemmParams P = plain_gemm(dG, 4 * Hp, w.wxc, I, dx, I, T_ * B, I, 4 * Hp, true, false, ce, false, 0.0f);
    st = run_gemm(a.dtype, true, false, P, 0, 0, stream, w.part, w.part_bytes);
    if (st) return st;
  }
  {
    // compact weight gradients: dwx[4Hp x I] = dG^T . x, dwh[4Hp x Hp] = dG[1:]^T . h[kept][:-1]
    GemmParams P = plain_gemm(dG, 4 * Hp, x, I, w.dwx, I, 4 * Hp, I, T_ * B, false, false, ce, false, 0.0f);
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
                     (const T*)w.dwh, (const int*)w.rank, H, I, Hp, (T*)dW);
  ARD_LAUNCH_CHECK("lstm_scatter_dw_kernel");
  return ARD_OK;
}

}  // namespace ard

using namespace ard;

extern "C" size_t ard_lstm_workspace_bytes(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H,
                                           const ard_pattern* pat) {
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}};
  if (lstm_check(a, pat)) return 0;
  return lstm_ws_layout(nullptr, a.es, T, B, I, H, a.Hk).total;
}

extern "C" int32_t ard_lstm_fwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const void* x,
                                const void* W, const ard_pattern* pat, void* h, float* c, float* gates, void* ws,
                                size_t ws_bytes, void* stream) {
  BatchSuspend not_recorded;  // this entry point's kernels depend on each other: never part of a grouped launch
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}};
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
  LstmArgs a{dtype, T, B, I, H, 0, 0, Axis{}};
  int32_t st = lstm_check(a, pat);
  if (st) return st;
  if (!x || !W || !h || !c || !gates || !dh || !dx || !dW) return fail(ARD_EINVAL, "null tensor pointer");
  LstmWs w = lstm_ws_layout((char*)ws, a.es, T, B, I, H, a.Hk);
  if (!ws || ws_bytes < w.total) return fail(ARD_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", w.total, ws_bytes);
  if (dtype == ARD_BF16) return lstm_bwd_t<uint16_t>(a, x, W, h, c, gates, dh, dx, dW, w, (hipStream_t)stream);
  return lstm_bwd_t<float>(a, x, W, h, c, gates, dh, dx, dW, w, (hipStream_t)stream);
}
