/*
 * libard -- training matrix multiplications under Approximate Random Dropout,
 * hand-written HIP for AMD MI355X (gfx950), behind a plain C ABI.
 *
 * Conventions shared by every entry point
 *  - Pointers named d_* and every tensor argument (X, W, Y, dY, ...) are DEVICE
 *    pointers owned by the caller; the library never frees or keeps them.
 *    Pointers without that prefix (pattern structs, host tables, out scalars) are
 *    HOST pointers read or written before the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *    entry points only enqueue work on it and return; they never synchronise.
 *  - `ws` is a caller-provided device workspace of `ws_bytes` bytes, at least what
 *    the matching *_workspace_bytes() call returns (may be NULL when that is 0).
 *    The library allocates no device memory.
 *  - Matrices are row-major and dense (leading dimension = number of columns).
 *    X[B x I] activations, W[O x I] weights (row o = output neuron o of the layer),
 *    Y[B x O] = X . W^T.  dtype ARD_F32 = float, ARD_BF16 = bfloat16 bit patterns;
 *    products always accumulate in fp32; outputs have the input dtype unless stated.
 *  - Every element of an output tensor is written: kept positions get the value,
 *    dropped positions get exactly +0.0 (or beta * old value where beta is given).
 *  - Return value: ARD_OK or a negative ard_status.  All argument checks happen on
 *    the host before anything is enqueued; ard_last_error() gives the message.
 *    Nothing throws or aborts across this boundary.
 *  - Same inputs give bit-identical outputs (no floating-point atomics).
 */
#ifndef ARD_H
#define ARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ARD_OK = 0,
  ARD_EINVAL = -1,       /* bad pattern parameters, null pointer, bad flag        */
  ARD_ESHAPE = -2,       /* non-positive or inconsistent sizes                    */
  ARD_EDTYPE = -3,       /* unknown dtype                                         */
  ARD_EWORKSPACE = -4,   /* workspace missing or too small                        */
  ARD_EHIP = -5,         /* the HIP runtime reported an error on launch           */
  ARD_EUNSUPPORTED = -6  /* valid request this build does not implement           */
} ard_status;

typedef enum { ARD_F32 = 0, ARD_BF16 = 1 } ard_dtype;

typedef enum {
  ARD_PAT_NONE = 0,  /* nothing dropped                                              */
  ARD_PAT_ROW = 1,   /* row-based pattern (Section 3.1, Eq. 1): parameters dp, b     */
  ARD_PAT_TILE = 2,  /* tile-based pattern (Section 3.2): dp, b, tile_r x tile_c     */
  ARD_PAT_LIST = 3   /* explicit ascending device list of kept units (d_keep, count) */
} ard_pat_kind;

/*
 * A dropout pattern.  dp is the period and b the bias in the paper's 1-based
 * convention, b in {1..dp}: the unit with 1-based index i is dropped iff
 * (i - b) mod dp != 0, so dp=3, b=1 keeps units 1, 4, 7, ... (Section 3.1).
 * ROW: units are the neurons of one layer (rows of W for an output pattern,
 * columns of W for an input pattern); dp <= number of units.
 * TILE: units are the tile_r x tile_c tiles of W[O x I] numbered row-major over
 * the tile grid ceil(O/tile_r) x ceil(I/tile_c), edge tiles clipped (Section 3.2);
 * dp <= number of tiles.
 * LIST: d_keep holds `count` strictly ascending unit indices (device memory).
 * The d_* fields below d_keep are optional for TILE: the outputs of a previous
 * ard_pattern_gen() call for the same pattern; when NULL the GEMM entry points
 * regenerate them in their workspace.
 */
typedef struct {
  int32_t kind;            /* ard_pat_kind                                   */
  int32_t dp, b;           /* ROW, TILE                                      */
  int32_t tile_r, tile_c;  /* TILE                                           */
  int32_t count;           /* LIST: number of kept units                     */
  const int32_t* d_keep;   /* LIST: kept units; TILE (optional): kept tiles  */
  const uint8_t* d_mask;   /* TILE (optional): tile mask, 1 = kept           */
  const int32_t* d_rowptr; /* TILE (optional): CSR offsets into d_keep       */
  const int32_t* d_colptr; /* TILE (optional): CSC offsets into d_csc_rows   */
  const int32_t* d_csc_rows; /* TILE (optional): kept tile rows per column   */
} ard_pattern;

/* ---- pattern distribution and sampling (host only) ---------------------- */

/*
 * Search for the pattern distribution K (Section 3.3): v in R^n, d = softmax(v),
 * loss = (d . p_u - p)^2 + 1e-3 * sum d ln d with p_u[i] = (i-1)/i, descent on v
 * from v = 0 (perturbed deterministically when seed != 0) until the loss stops
 * moving.  Writes k_out[n] (doubles summing to 1) and cdf_out[n], the 2^32
 * fixed-point cumulative table round(2^32 * sum_{j<=i} k_j) with cdf_out[n-1] = 2^32.
 * Both are host arrays.  Needs 0 <= p < 1, 1 <= n <= 4096.
 */
int32_t ard_search_k(double p, int32_t n, uint64_t seed, double* k_out, uint64_t* cdf_out);

/*
 * Pattern of one iteration (Section 3.4): dp drawn from K, then b uniform in
 * {1..dp}.  Stateless and integer-only: two 32-bit words r1, r2 come from the
 * SplitMix64 finaliser chained over (seed, iter, stream_id);
 * dp = 1 + min{i : r1 < cdf[i]}, b = 1 + ((r2 * dp) >> 32).  cdf is the host table
 * from ard_search_k.  Writes the two host ints.
 */
int32_t ard_pattern_sample(const uint64_t* cdf, int32_t n, uint64_t seed, uint64_t iter,
                           uint32_t stream_id, int32_t* dp_out, int32_t* b_out);

/* ---- pattern generation on the device (Sections 3.1, 3.2, 6) ------------ */

/*
 * Binary mask (uint8, 1 = kept, Section 6) and compacted ascending list of the
 * kept units of a ROW or TILE pattern.
 * ROW : units = `rows` neurons (`cols` ignored).  d_mask[rows], d_keep[>= kept],
 *       d_count[1].  d_rowptr, d_colptr, d_csc_rows must be NULL.
 * TILE: W is rows x cols (= O x I); TR = ceil(rows/tile_r), TC = ceil(cols/tile_c).
 *       d_mask[TR*TC] row-major, d_keep[>= kept] linear tile ids (ascending, which
 *       is also CSR order: tile column = id - tile_row*TC), d_count[1],
 *       d_rowptr[TR+1], d_colptr[TC+1], d_csc_rows[>= kept] (tile rows, grouped by
 *       tile column, ascending inside each column).  Any output pointer may be NULL
 *       to skip it, except that d_csc_rows needs d_colptr.
 * Kept count is ceil((units - (b-1)) / dp) (0 if b-1 >= units).
 */
int32_t ard_pattern_gen(const ard_pattern* pat, int32_t rows, int32_t cols,
                        uint8_t* d_mask, int32_t* d_keep, int32_t* d_count,
                        int32_t* d_rowptr, int32_t* d_colptr, int32_t* d_csc_rows,
                        void* stream);

/* ---- fully connected layer under a pattern (Sections 3.1, 3.2) ---------- */

/*
 * Layout flags of the three layer calls below (OR them into `flags`).  The method multiplies
 * compacted operands and scatters the result (Section 3.1); these flags let a chain of
 * layers keep its activations compact between calls instead of scattering and re-gathering:
 *   ARD_IN_COMPACT   the input-side activation (X, dX, relu_src) is [B x pad8(I')] and holds only
 *                    the kept input neurons of pat_in, in ascending order;
 *   ARD_OUT_COMPACT  the output-side activation (Y, dY) is [B x pad8(O')] and holds only the kept
 *                    output neurons of pat_out (nothing is zero-filled then);
 *   ARD_W_COMPACT    W is the compact matrix written by ard_compact_weight();
 *   ARD_DW_COMPACT   (weight gradient only, together with the two flags above) dW is the gradient
 *                    of the kept synapses only, [pad8(O') x pad8(I')] in the layout of a compact
 *                    weight; the gradient of every dropped synapse is zero and is not stored.
 * pad8(n) = n rounded up to a multiple of 8.  Every compact matrix stores its kept-unit axes
 * padded to pad8 with ZEROS (rows of 16-byte pieces whatever the kept count is): compact inputs
 * must carry zero padding, compact outputs are written with it.  With a NONE pattern a compact
 * activation is simply the dense one with its rows padded to pad8 columns (useful for narrow
 * matrices such as a 10-column loss gradient).
 * Without ARD_DW_COMPACT dW is the full [O x I] matrix.  Without ARD_W_COMPACT, a forward or backward-data
 * call whose pat_in is not NONE first gathers W[kept o, kept i] into its workspace.
 * Tile patterns take no flags.
 */
enum { ARD_IN_COMPACT = 1, ARD_OUT_COMPACT = 2, ARD_W_COMPACT = 4, ARD_DW_COMPACT = 8 };

/* Wc[pad8(O') x pad8(I')]: W[kept o, kept i] in the top-left corner, zeros in the padding
 * (ROW/LIST/NONE patterns). One gather kernel, no workspace. */
int32_t ard_compact_weight(int32_t dtype, int32_t I, int32_t O, const void* W, void* Wc,
                           const ard_pattern* pat_out, const ard_pattern* pat_in, void* stream);

/*
 * pat_out / pat_in select what is dropped (either may be NULL = NONE):
 *   pat_out ROW/LIST over the O output neurons, pat_in ROW/LIST over the I input
 *   neurons (the previous layer's pattern): synapse (o,i) survives iff both do.
 *   pat_out TILE: tile pattern on W; pat_in must then be NULL/NONE.
 * Workspace for any of the three calls below with the same arguments.
 */
size_t ard_gemm_workspace_bytes(int32_t dtype, int32_t B, int32_t I, int32_t O,
                                const ard_pattern* pat_out, const ard_pattern* pat_in);

/*
 * Forward: Y[:, kept o] = alpha * X[:, kept i] . W[kept o, kept i]^T, optional
 * ReLU (fuse_relu != 0); Y[:, dropped o] = 0 (Section 3.1: only the kept rows of
 * W and the kept part of the input are fetched and multiplied, the rest of the
 * output is zero).  TILE: Y[:, block J] = alpha * sum over kept tiles (J,k) of
 * X[:, block k] . W[J,k]^T (Section 3.2).
 */
int32_t ard_drop_gemm_fwd(int32_t dtype, int32_t B, int32_t I, int32_t O,
                          const void* X, const void* W, void* Y,
                          const ard_pattern* pat_out, const ard_pattern* pat_in,
                          float alpha, int32_t fuse_relu, int32_t flags,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * Backward w.r.t. the input: dX[:, kept i] = alpha * dY[:, kept o] . W[kept o, kept i];
 * dX[:, dropped i] = 0.  If relu_src != NULL (same shape and dtype as dX: the
 * stored activation this layer consumed), dX is additionally zeroed wherever
 * relu_src <= 0 (ReLU backward fused).  The paper does not write the backward
 * pass; this is the derivative of the masked forward above.
 */
int32_t ard_drop_gemm_bwd_data(int32_t dtype, int32_t B, int32_t I, int32_t O,
                               const void* dY, const void* W, void* dX,
                               const ard_pattern* pat_out, const ard_pattern* pat_in,
                               float alpha, const void* relu_src, int32_t flags,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * Backward w.r.t. the weight: dW[kept o, kept i] = alpha * dY[:, kept o]^T . X[:, kept i]
 * + beta * dW_old; every dropped synapse gets beta * dW_old (exactly 0 for beta = 0).
 */
int32_t ard_drop_gemm_bwd_weight(int32_t dtype, int32_t B, int32_t I, int32_t O,
                                 const void* dY, const void* X, void* dW,
                                 const ard_pattern* pat_out, const ard_pattern* pat_in,
                                 float alpha, float beta, int32_t flags,
                                 void* ws, size_t ws_bytes, void* stream);

/*
 * The weight gradient for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.
 * Same arguments, results and errors as ard_drop_gemm_bwd_weight without `ws`: the partial sums
 * of split contractions, padded operand copies and tile lists live in a scratch array that is part
 * of the library (ard_static_scratch_bytes() bytes, 64 MiB, one copy per GPU, held until the
 * process ends).  The call makes no allocation of any kind; the first call on a device looks the
 * array's address up.  A layer for which ard_gemm_workspace_bytes() exceeds the array is refused
 * with ARD_EWORKSPACE before anything is enqueued.  Nothing in the scratch has to start at zero
 * (every partial sum is written before it is read), so nothing is cleared.  All calls on one GPU
 * share that GPU's array: two calls that overlap in time on the same GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.
 */
size_t ard_static_scratch_bytes(void);
int32_t ard_drop_gemm_bwd_weight_static(int32_t dtype, int32_t B, int32_t I, int32_t O,
                                        const void* dY, const void* X, void* dW,
                                        const ard_pattern* pat_out, const ard_pattern* pat_in,
                                        float alpha, float beta, int32_t flags, void* stream);

/*
 * Grouped launches.  A training iteration of a small layer chain (Section 3.2, last paragraph: FC ->
 * activation with the dropout layer skipped) is a handful of products of a few microseconds each, so
 * most of its time is the fixed cost of launches.  Calls that do not depend on each other can be
 * issued as ONE launch:
 *     ard_batch_begin();
 *     ard_drop_gemm_bwd_weight(...);  ard_drop_gemm_bwd_data(...);   // recorded, nothing is enqueued
 *     ard_batch_launch(stream);                                      // one grid runs all of them
 * Between begin and launch (per host thread) ard_compact_weight and the three layer calls record
 * their kernels when these are of the kinds a batch-sized layer chain uses (bf16 LDS-direct products
 * on 4-wavefront tiles, the narrow-layer kernels, the 16-byte finishing pass); everything else
 * (fp32, tile patterns on large tiles, LSTM, convolution) is enqueued at once as usual on the stream
 * given to that call.  ard_batch_launch enqueues, on ITS stream, one launch with every recorded
 * kernel that depends on nothing else in the batch, then (if any) one with the finishing passes.
 * The caller promises that no call of a batch reads what another call of the same batch writes, and
 * gives every call of a batch its own workspace.  Results are bit-identical to the same calls issued
 * one by one.  ard_batch_abort() drops what was recorded.  Errors: ARD_EINVAL for begin inside an
 * open batch or launch without one.
 */
int32_t ard_batch_begin(void);
int32_t ard_batch_launch(void* stream);
void ard_batch_abort(void);

/* Standalone ReLU backward: dX = dY where Y > 0 else 0; n elements of `dtype`. */
int32_t ard_relu_bwd(int32_t dtype, int64_t n, const void* dY, const void* Y, void* dX, void* stream);

/* ---- LSTM layer under a row pattern on its hidden units (Section 7.2.3) -- */

/*
 * Fused weight W[4H x (I+H)], gate blocks of H rows in the order i, f, g, o,
 * columns [x | h]; no bias; zero initial state.  `pat` (ROW/LIST/NONE over the H
 * hidden units) holds for the whole sequence: a dropped unit has h = c = 0 at
 * every step, its four gate rows and its recurrent column are never loaded.
 * A TILE pattern (Section 3.2 applied to this layer, the "TILE" variant of Section 7.2.3) lies over the
 * fused weight itself: tile grid ceil(4H/tile_r) x ceil((I+H)/tile_c), any positive tile size; the synapses
 * of dropped tiles are absent for the whole sequence, every unit stays alive, and dW is zero on them.
 * x[T,B,I] dtype; outputs h[T,B,H] dtype, c[T,B,H] fp32, gates[T,B,4H] fp32
 * (activated i,f,g,o; entries of dropped units are 0), all fully written.
 */
size_t ard_lstm_workspace_bytes(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H,
                                const ard_pattern* pat);
int32_t ard_lstm_fwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H,
                     const void* x, const void* W, const ard_pattern* pat,
                     void* h, float* c, float* gates,
                     void* ws, size_t ws_bytes, void* stream);
/*
 * bf16 layers whose kept state is small enough run the whole recurrence of ard_lstm_fwd in ONE launch
 * whose workgroups exchange h_t through memory and wait for each other step by step.  The wait is
 * bounded: should the workgroups not all be resident together (another kernel holding CUs), they give
 * up, leave normally and set an int32 in the workspace to 1; the outputs are then incomplete.
 * ard_lstm_status_offset returns that word's byte offset in the workspace ((size_t)-1 when this layer
 * takes the launch-per-step path, which has no such state); it is 0 after a completed call.
 */
size_t ard_lstm_status_offset(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H, const ard_pattern* pat);
/*
 * Back-propagation through time with the same pattern.  dh[T,B,H] (dtype) is the
 * gradient arriving on every h_t; h, c, gates are ard_lstm_fwd's outputs.
 * Writes dx[T,B,I] (dtype) and dW[4H x (I+H)] (dtype; zero outside kept gate rows
 * x ([x] + kept recurrent columns)).  bf16 layers whose backward exchange (the gate gradient
 * of a step, read by every unit slice) is small enough run this recurrence in one launch as
 * well, with the same bounded wait and the same status word as ard_lstm_fwd (a layer may take
 * the one-launch form forward and the launch-per-step form backward; the word then stays 0).
 */
int32_t ard_lstm_bwd(int32_t dtype, int32_t T, int32_t B, int32_t I, int32_t H,
                     const void* x, const void* W, const ard_pattern* pat,
                     const void* h, const float* c, const float* gates, const void* dh,
                     void* dx, void* dW,
                     void* ws, size_t ws_bytes, void* stream);

/* ---- convolution with dropped input feature maps (Sections 5, 6) -------- */

typedef enum {
  ARD_CONV_SELECT = 0,    /* sensitivity score + selection -> d_mask, d_keep, d_count, d_score */
  ARD_CONV_FWD = 1,       /* out = Y[N,Cout,Ho,Wo]                                        */
  ARD_CONV_BWD_DATA = 2,  /* out = dA[N,C,H,W], dropped channels exactly 0               */
  ARD_CONV_BWD_WEIGHT = 3,/* out = dWt[Cout,C,KH,KW], dropped channels exactly 0         */
  ARD_CONV_FWD_ROWS = 4,  /* out = Y under a row-based sensitivity-aware pattern (below)  */
  ARD_CONV_BWD_DATA_ROWS = 5,   /* out = dA, gradient of FWD_ROWS                         */
  ARD_CONV_BWD_WEIGHT_ROWS = 6  /* out = dWt, gradient of FWD_ROWS                        */
} ard_conv_mode;
/*
 * bf16, stride 1: every pass first copies what it convolves into a channels-last, zero-bordered grid
 * in the workspace (the kept maps of A for FWD and BWD_WEIGHT, dY for BWD_DATA and BWD_WEIGHT).  The
 * passes of one layer can share those copies: OR a flag into `mode` and the pass takes the grid an
 * earlier call left in the SAME workspace instead of building it again.  The caller vouches that the
 * earlier call had the same shape arguments, the same tensor (A or dYin), the same kept list, and that
 * nothing else wrote the workspace in between (the other passes of the layer do not disturb it).
 *   ARD_CONV_REUSE_A   FWD, BWD_WEIGHT: the grid of A built by an earlier FWD or BWD_WEIGHT (of the *_ROWS modes:
 *                      by FWD_ROWS or BWD_WEIGHT_ROWS)
 *   ARD_CONV_REUSE_DY  BWD_DATA, BWD_WEIGHT: the grid of dY built by an earlier BWD_DATA or BWD_WEIGHT;
 *                      across the two passes only for size-preserving filters (k - 1 = 2 pad), else
 *                      ARD_EUNSUPPORTED
 * Any other use of the flags (fp32, stride > 1, n_keep = 0, SELECT) is refused.
 */
enum { ARD_CONV_REUSE_A = 0x100, ARD_CONV_REUSE_DY = 0x200 };

size_t ard_conv_workspace_bytes(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd,
                                int32_t Cout, int32_t kh, int32_t kw, int32_t stride, int32_t pad);

/*
 * NCHW activations A[N,C,H,Wd], OIHW weights Wt[Cout,C,kh,kw], output spatial
 * size Ho = (H + 2 pad - kh)/stride + 1 (same for Wo).
 * SELECT (channel-level reading of the sensitivity-aware drop of Section 5):
 *   score[c] = sum over (n,h,w) of floor(min(|A|, 2^15) * 2^24) as an exact int64
 *   (order-independent; mean |A| = score / 2^24 / (N*H*Wd)); the floor(rate*C)
 *   channels that come first in ascending (score, channel) order are dropped.
 *   Writes d_mask[C] (1 = kept), d_keep[C - floor(rate*C)] ascending, d_count[1]
 *   and, if non-NULL, d_score[C] (int64).  Needs N*H*Wd <= 2^24.
 * FWD_ROWS (row-based sensitivity-aware pattern, Section 5.2.1): every channel takes part, but only the
 *   kept rows of the input matrix (= output positions) are gathered and multiplied; d_keep lists them
 *   as n * Ho*Wo + p, ascending, n_keep entries (0 .. N*Ho*Wo), d_mask[N*Ho*Wo] is the same set as a
 *   0/1 mask (both as written by ard_sens_row_pattern).  out = Y[N,Cout,Ho,Wo], dropped positions +0.0.
 *   Needs A, Wt.  fp32 and strided layers compute every position and zero the dropped ones.
 * BWD_DATA_ROWS / BWD_WEIGHT_ROWS: the gradients of FWD_ROWS with respect to A and Wt.  Only kept rows took
 *   part in the product, so gradient arriving on a dropped position counts as zero: d_mask[N*Ho*Wo] is the
 *   row mask; BWD_DATA / BWD_WEIGHT run with every channel kept on a dY whose dropped positions are zero
 *   (zeroed while dY is copied into its grid; a masked copy for fp32 and strided layers).  No time is saved
 *   over an undropped layer; n_keep, d_keep are ignored.  Needs dYin, d_mask and Wt (data) or A (weight).
 *   The reuse flags apply as for BWD_DATA / BWD_WEIGHT: ARD_CONV_REUSE_A takes the grid FWD_ROWS left,
 *   ARD_CONV_REUSE_DY the masked grid an earlier *_ROWS gradient of the same mask left.
 * FWD / BWD_DATA / BWD_WEIGHT read the kept channels from d_keep (n_keep entries,
 *   n_keep given on the host) and never load a dropped channel:
 *   FWD        Y  = conv(A restricted to kept channels, Wt)       needs A, Wt
 *   BWD_DATA   dA[:, kept] = conv^T(dY, Wt), others 0              needs dYin, Wt
 *   BWD_WEIGHT dWt[:, kept] = corr(dY, A), others 0                needs dYin, A
 */
int32_t ard_fmap_drop_conv(int32_t mode, int32_t dtype,
                           int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t Cout,
                           int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                           double rate, int32_t n_keep,
                           const void* A, const void* Wt, const void* dYin, void* out,
                           uint8_t* d_mask, int32_t* d_keep, int32_t* d_count, int64_t* d_score,
                           void* ws, size_t ws_bytes, void* stream);

/* ---- sensitivity prediction and sensitivity-aware patterns (Sections 5.1, 5.2) ---- */

/*
 * The input matrix of one image (Section 5.1) has one row per output position p = oh*Wo + ow and one
 * column per (c, kh, kw), q = (c*kh_size + kh)*kw_size + kw; its entries are the zero-padded
 * activations.  It is cut into x-by-y regions (y = 0: regions span the whole width), edge regions
 * clipped: row band rb = p / x, column block cb = q / y, region id (image*RB + rb)*CB + cb.
 * ard_sens_regions returns rows = Ho*Wo, RB and CB for buffer sizing (host only).
 *
 * Random draws: the 32-bit word u(seed, iteration, stream, index) = upper half of the SplitMix64
 * finaliser chained over the four values (as ard_pattern_sample chains three), streams 0x5E01
 * (samples), 0x5E02 (rows), 0x5E03 (blocks).  A possibility p becomes the threshold floor(p * 2^32)
 * and a unit is dropped iff u < threshold.
 *
 * ard_sens_predict (steps 2, 3): per region, s = max(1, k_permille * size / 1000) draws with
 *   replacement (at most 65536), draw j (index region*65536 + j) picks element (u * size) >> 32 of the
 *   region in row-major order; d_count = how many drawn entries exceed `threshold`, d_samples = s,
 *   d_sens = 1 iff 1000 * count >= t_permille * s.  All three are device arrays of N*RB*CB entries.
 * ard_sens_row_pattern (Section 5.2.1; regions span the width, d_sens[N*RB]): row g = image*rows + p is
 *   dropped with possibility m if its band is sensitive, n otherwise (index g).  Writes d_mask[N*rows]
 *   (1 = kept, Section 6), the ascending kept list d_keep[>= kept] and d_count[1]; any may be NULL.
 * ard_sens_block_pattern (Section 5.2.2): the blocks of one row band form a group.  balance != 0:
 *   S = mean number of sensitive blocks per group of the image, rounded half up; in every group the
 *   S blocks with the largest share count/samples (exact comparison, ties to the lower block) become
 *   the sensitive ones (d_sens_out, may be NULL), so all groups hold the same number.  Then block
 *   (image*RB + rb)*CB + cb (= its index) is dropped with possibility m (sensitive) or n:
 *   d_block_keep[N*RB*CB], 1 = kept.
 * The paper fixes none of these procedures beyond k, t, the threshold and m < n; see the oracle's notes.
 */
int32_t ard_sens_regions(int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                         int32_t x, int32_t y, int32_t* rows, int32_t* row_bands, int32_t* col_blocks);
int32_t ard_sens_predict(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t kh, int32_t kw,
                         int32_t stride, int32_t pad, int32_t x, int32_t y, int32_t k_permille, int32_t t_permille,
                         float threshold, uint64_t seed, uint64_t iteration, const void* A,
                         int32_t* d_count, int32_t* d_samples, uint8_t* d_sens, void* stream);
int32_t ard_sens_row_pattern(int32_t N, int32_t rows, int32_t x, const uint8_t* d_sens, double m, double n,
                             uint64_t seed, uint64_t iteration, uint8_t* d_mask, int32_t* d_keep, int32_t* d_count,
                             void* stream);
int32_t ard_sens_block_pattern(int32_t N, int32_t row_bands, int32_t col_blocks, const int32_t* d_count,
                               const int32_t* d_samples, const uint8_t* d_sens, int32_t balance, double m, double n,
                               uint64_t seed, uint64_t iteration, uint8_t* d_sens_out, uint8_t* d_block_keep,
                               void* stream);

/*
 * Forward convolution under a block-based sensitivity-aware pattern (Section 5.2.2): entry (p, q) of an
 * image's input matrix takes part iff d_block_keep[(image*RB + p/x)*CB + q/y] != 0 (the array
 * ard_sens_block_pattern writes; y = 0: blocks span the width).  out = Y[N,Cout,Ho,Wo], every element
 * written.  Arguments and workspace as for ard_fmap_drop_conv(ARD_CONV_FWD) with every channel kept.
 * Dropped blocks are skipped (neither loaded nor multiplied) when the blocks are whole 64-channel groups
 * over all filter taps and the bands fill at least half a tile: bf16, stride 1, Cout > 64,
 * y % (64*kh*kw) == 0, kh*kw*ceil(C/64) <= 128, and x such that the bands of an image, each padded to
 * whole tiles of 128 or 256 positions, take at most twice the image's positions.  Any other shape runs on
 * the general convolution engine, which applies the mask while it gathers the patches: correct in both
 * dtypes and for any stride, no time saved.
 */
int32_t ard_conv_fwd_blocks(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t Cout,
                            int32_t kh, int32_t kw, int32_t stride, int32_t pad, int32_t x, int32_t y,
                            const void* A, const void* Wt, const uint8_t* d_block_keep, void* out,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * Gradients of ard_conv_fwd_blocks (Section 5.2.2): an entry of a dropped block takes no part in the
 * product, so it contributes nothing to the weight gradient and receives no gradient itself.
 *   mode = ARD_CONV_BWD_WEIGHT: out = dWt[Cout,C,kh,kw], dWt[co,q] = sum over images and positions p with
 *          block (p/x, q/y) kept of dY[n,co,p] * X_n[p,q]; needs A and dYin (Wt unused, may be NULL).
 *   mode = ARD_CONV_BWD_DATA:   out = dA[N,C,H,W], the sum over the kept entries (p, q) that were cut from a
 *          pixel of sum_co dY[n,co,p] * Wt[co,q]; needs Wt and dYin (A unused, may be NULL); stride 1 and
 *          pad <= k-1 only, as for ARD_CONV_BWD_DATA of ard_fmap_drop_conv (else ARD_EUNSUPPORTED).
 * Every element of out is written.  d_block_keep, x, y, workspace and dtypes as for ard_conv_fwd_blocks.
 * No work is skipped.  Blocks of whole channels (y % (kh*kw) == 0, at most 16 column blocks): per column
 * block, dY is copied with the positions of that block's dropped bands zeroed and the ordinary gradient
 * pass runs on the copy with the block's channels as the kept list (the fast path where the shape allows).
 * Other block shapes run on the general convolution engine: the weight gradient masks the patches it
 * gathers, the data gradient contracts tap by tap and adds a tap's partial product where the mask keeps
 * the entry.  Both dtypes.
 */
int32_t ard_conv_bwd_blocks(int32_t mode, int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t Wd, int32_t Cout,
                            int32_t kh, int32_t kw, int32_t stride, int32_t pad, int32_t x, int32_t y,
                            const void* A, const void* Wt, const void* dYin, const uint8_t* d_block_keep,
                            void* out, void* ws, size_t ws_bytes, void* stream);

/* ---- dynamic dropout-ratio tuning (Section 5.3, host only) ---------------- */

/*
 * The prune possibility over the training epochs follows the skew-normal curve of Eq. (4),
 * f(y) = (2/sigma) phi((y-mu)/sigma) Phi(lambda (y-mu)/sigma).
 * ard_skew_normal_params solves Eq. (5) and (6) for mu and sigma given the mean E(Y), the variance
 * D(Y) > 0 and the skew lambda; ard_skew_normal_pdf evaluates Eq. (4).
 * ard_prune_schedule fills p_out[n_epochs] (host doubles): epoch e sits at the normalised time
 * (e + 1/2) / n_epochs, its possibility is proportional to the curve there, scaled so that the
 * average over the run equals `total`, then clipped to [0, p_max] (how the curve becomes a per-epoch
 * value is not spelled out in the paper; this is the reading taken).  mean and var are in normalised time.
 */
int32_t ard_skew_normal_params(double mean, double var, double lambda, double* mu, double* sigma);
double ard_skew_normal_pdf(double y, double mu, double sigma, double lambda);
int32_t ard_prune_schedule(int32_t n_epochs, double total, double mean, double var, double lambda,
                           double p_max, double* p_out);

/* ---- sizes of compact buffers and grids (host only, nothing is launched) --- */

/* Number of kept units of a ROW / LIST / NONE pattern over `units` units: ceil((units - (b-1)) / dp)
 * for ROW (Section 3.1; the "(dp-1)/dp dropped" of the text is exact only when dp divides units),
 * `count` for LIST, `units` for NONE or NULL.  Negative ard_status on a bad pattern. */
int32_t ard_kept_count(const ard_pattern* pat, int32_t units);
/* Stored extent of that axis in a compact matrix: the kept count rounded up to a multiple of 8. */
int32_t ard_compact_dim(const ard_pattern* pat, int32_t units);
/* Tile grid of a TILE pattern over W[rows x cols]: ceil(rows/tile_r) x ceil(cols/tile_c) (Section 3.2). */
int32_t ard_tile_grid(const ard_pattern* pat, int32_t rows, int32_t cols, int32_t* tile_rows, int32_t* tile_cols);
/* Output extent of a convolution along one axis: (in + 2 pad - k) / stride + 1, or a negative status. */
int32_t ard_conv_out_size(int32_t in, int32_t k, int32_t stride, int32_t pad);

/* ---- debugging aids (host logic without a GPU) ----------------------------- */

/*
 * Dry-run mode, process-wide.  While on, every entry point runs its argument checks, its dispatch
 * and the host-side bounds proof of its loaders (every workgroup, wavefront, lane and contraction
 * step of every launch that fetches operands with unchecked per-lane addresses), but enqueues nothing
 * and makes no HIP call; device pointers are never dereferenced, so any non-NULL, 16-byte aligned
 * value will do.  Turning the mode on or off resets the counters below.
 */
void ard_debug_set_dry_run(int32_t on);
/* Launches skipped on this thread since the last call (or mode switch); if names != NULL their kernel
 * names, comma separated and truncated to cap-1 characters, are copied there. */
int32_t ard_debug_dry_launches(char* names, size_t cap);
/* Bounds proofs run on this thread since the last call; six[0..5] = first byte, end byte and size of
 * operand A, then of operand B, of the most recent one (offsets relative to the operand's pointer). */
int32_t ard_debug_last_bounds(int64_t* six);
/* The proofs treat every operand as `elems` elements shorter than stated (0 = normal).  Lets a test
 * show that a proof rejects a launch whose loads would end past a (pretended) operand end. */
void ard_debug_set_extent_slack(int64_t elems);

/* ---- misc ---------------------------------------------------------------- */

/* Message of the last failing call on this thread (static storage, never NULL). */
const char* ard_last_error(void);
/* Library version as major*10000 + minor*100 + patch. */
int32_t ard_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ARD_H */
