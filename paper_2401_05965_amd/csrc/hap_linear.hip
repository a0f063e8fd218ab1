/*
 * Sharded fully-connected layer and sufficient-factor rebuild: argument validation and the mapping
 * of each sharding rule (Fig. "semantics") onto the GEMM engine.  No arithmetic happens here.
 *
 *   forward   Y  = X W            A = X (K-contiguous),   B = W (N-contiguous)
 *   bwd-data  dX = dP W^T         A = dP (K-contiguous),  B = W read as [n=in][k=out] (K-contiguous)
 *   bwd-wgt   dW = X^T dP         A = X read as [m=in][k=token] (M-contiguous), B = dP (N-contiguous)
 *   SFB       dW = sum_i X_i^T dY_i   the bwd-wgt form with the contracted axis split in m segments
 */
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "hap_gemm.h"

namespace {

inline int esize(int dtype) { return dtype == HAP_BF16 ? 2 : 4; }
inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

/* Row pitch (elements) of the dP = dY * act'(preact) copy the backward keeps in the workspace.  A multiple of 128 bytes: dP is
 * the K-contiguous operand of the bwd-data product, whose tiles fetch 64 or 128 consecutive bytes of every row - rows that do
 * not start on such a boundary make every fetch straddle two cache sectors (measured: 10-20 % of the product's time).  The 8
 * spare elements let the copy take the 16-byte phase of W's slice. */
inline int64_t dp_pitch(int64_t out_n, int es) { return round_up(out_n + 8, 128 / es); }

struct View {
  int64_t tok_lo, tok_n;   // rows of X / Y owned
  int64_t in_lo, in_n;     // columns of X / rows of W owned
  int64_t out_lo, out_n;   // columns of W / Y owned
};

int resolve(const hap_linear_desc* d, int j, View* v) {
  if (!d) return hap_fail(HAP_EINVAL, "descriptor is NULL");
  if (d->tokens < 0 || d->in_features < 1 || d->out_features < 1) return hap_fail(HAP_EINVAL, "bad layer sizes");
  if (d->io_dtype != HAP_F32 && d->io_dtype != HAP_BF16) return hap_fail(HAP_EINVAL, "bad io_dtype %d", d->io_dtype);
  if (d->act != HAP_ACT_NONE && d->act != HAP_ACT_GELU_ERF) return hap_fail(HAP_EINVAL, "bad act %d", d->act);
  v->tok_lo = 0; v->tok_n = d->tokens;
  v->in_lo = 0; v->in_n = d->in_features;
  v->out_lo = 0; v->out_n = d->out_features;
  int64_t lo = 0, hi = 0;
  int rc;
  switch (d->mode) {
    case HAP_SHARD_BATCH:
      if ((rc = hap_shard_range(d->m, d->offsets, d->tokens, j, &lo, &hi))) return rc;
      v->tok_lo = lo; v->tok_n = hi - lo;
      break;
    case HAP_SHARD_FEATURE:
      if ((rc = hap_shard_range(d->m, d->offsets, d->out_features, j, &lo, &hi))) return rc;
      v->out_lo = lo; v->out_n = hi - lo;
      break;
    case HAP_SHARD_REDUCTION:
      if ((rc = hap_shard_range(d->m, d->offsets, d->in_features, j, &lo, &hi))) return rc;
      v->in_lo = lo; v->in_n = hi - lo;
      if (d->has_bias) return hap_fail(HAP_EINVAL, "bias belongs after the all-reduce: has_bias must be 0 in reduction mode");
      if (d->act != HAP_ACT_NONE) return hap_fail(HAP_EINVAL, "no activation on a partial sum (reduction mode)");
      break;
    case HAP_REPLICATED:
      if (d->m < 1) return hap_fail(HAP_EINVAL, "m = %d < 1", d->m);
      if (j < 0 || j >= d->m) return hap_fail(HAP_EINVAL, "shard_index %d outside [0, %d)", j, d->m);
      break;
    default:
      return hap_fail(HAP_EINVAL, "bad shard mode %d", d->mode);
  }
  // leading dimensions must cover the widths of the buffers actually passed
  const bool full = d->operands_are_full != 0;
  const int64_t xw = (d->mode == HAP_SHARD_REDUCTION && !full) ? v->in_n : d->in_features;
  const int64_t ww = (d->mode == HAP_SHARD_FEATURE && !full) ? v->out_n : d->out_features;
  const int64_t yw = ww;
  if (d->ldx < xw || d->ldw < ww || d->ldy < yw)
    return hap_fail(HAP_ESHAPE, "leading dimension too small (ldx %lld < %lld or ldw %lld < %lld or ldy %lld < %lld)",
                    (long long)d->ldx, (long long)xw, (long long)d->ldw, (long long)ww, (long long)d->ldy, (long long)yw);
  return HAP_OK;
}

/* Element offsets of the device's slice inside the buffers passed for X-like, W-like, Y-like, bias-like tensors. */
struct Offs { int64_t x, w, y, b; };

Offs offsets_of(const hap_linear_desc* d, const View& v) {
  Offs o = {0, 0, 0, 0};
  if (!d->operands_are_full) return o;
  switch (d->mode) {
    case HAP_SHARD_BATCH: o.x = v.tok_lo * d->ldx; o.y = v.tok_lo * d->ldy; break;
    case HAP_SHARD_FEATURE: o.w = v.out_lo; o.y = v.out_lo; o.b = v.out_lo; break;
    case HAP_SHARD_REDUCTION: o.x = v.in_lo; o.w = v.in_lo * d->ldw; break;
    default: break;
  }
  return o;
}

inline const char* at(const void* p, int64_t elems, int es) { return static_cast<const char*>(p) + elems * es; }
inline char* at(void* p, int64_t elems, int es) { return static_cast<char*>(p) + elems * es; }

}  // namespace

extern "C" {

size_t hap_linear_fwd_workspace(const hap_linear_desc*, int) { return HAP_GEMM_WS_BYTES; }   // optional: split-K partial tiles

static size_t required_bwd_bytes(const hap_linear_desc* d, int shard_index) {
  View v;
  if (resolve(d, shard_index, &v) != HAP_OK) return 0;
  size_t need = 0;
  if (d->act != HAP_ACT_NONE) need += (size_t)(v.tok_n * dp_pitch(v.out_n, esize(d->io_dtype))) * esize(d->io_dtype);
  need = (size_t)round_up((int64_t)need, 256);
  need += (size_t)round_up((int64_t)hap_colsum_workspace(v.tok_n, v.out_n), 256);
  return need;
}

/* required_bwd_bytes(): the part that must be there (dP and column-sum scratch); the rest of what
 * hap_linear_bwd_workspace() reports is optional split-K scratch for the GEMM engine. */
size_t hap_linear_bwd_workspace(const hap_linear_desc* d, int shard_index) {
  return required_bwd_bytes(d, shard_index) + HAP_GEMM_WS_BYTES;
}

int hap_sharded_linear_fwd(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                           const void* bias, void* Y, void* preact, void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  View v;
  int rc = resolve(d, shard_index, &v);
  if (rc) return rc;
  if (v.tok_n == 0 || v.out_n == 0) return HAP_OK;   // the device owns no part of the output
  if (!Y || ((!X || !W) && v.in_n > 0)) return hap_fail(HAP_EINVAL, "X, W or Y is NULL");
  if ((d->has_bias != 0) != (bias != NULL)) return hap_fail(HAP_EINVAL, "bias pointer and has_bias disagree");
  const int es = esize(d->io_dtype);
  const Offs o = offsets_of(d, v);
  hap_gemm_problem p = {};
  p.M = v.tok_n; p.N = v.out_n;
  p.nseg = 1; p.k[0] = v.in_n;
  p.a[0] = at(X, o.x, es); p.lda = d->ldx; p.a_kcontig = 1;
  p.b[0] = at(W, o.w, es); p.ldb = d->ldw; p.b_kcontig = 0;
  p.in_dtype = d->io_dtype;
  p.c = at(Y, o.y, es); p.ldc = d->ldy; p.c_dtype = d->io_dtype;
  p.bias = bias ? at(bias, o.b, es) : NULL;
  p.preact = preact ? at(preact, o.y, es) : NULL; p.ldp = d->ldy;
  p.act = d->act;
  p.ws = ws; p.ws_bytes = ws ? ws_bytes : 0;
  return hap_gemm_run(&p, stream);
}

static int linear_bwd_impl(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                           const void* preact, const void* dY, void* dX, void* dW, int dW_dtype,
                           float* dbias, const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream);

int hap_sharded_linear_bwd(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                           const void* preact, const void* dY, void* dX, void* dW, int dW_dtype,
                           float* dbias, void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  return linear_bwd_impl(d, shard_index, X, W, preact, dY, dX, dW, dW_dtype, dbias, NULL, HAP_ACT_NONE, ws, ws_bytes, stream);
}

int hap_sharded_linear_bwd_dact(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                                const void* preact, const void* dY, void* dX, void* dW, int dW_dtype,
                                float* dbias, const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  if (x_act != HAP_ACT_NONE && x_act != HAP_ACT_GELU_ERF) return hap_fail(HAP_EINVAL, "bad x_act %d", x_act);
  if (x_act != HAP_ACT_NONE) {
    if (!d) return hap_fail(HAP_EINVAL, "descriptor is NULL");
    // act' is applied to a complete dX only: the feature rule yields a partial sum that is all-reduced first
    if (d->mode == HAP_SHARD_FEATURE) return hap_fail(HAP_EINVAL, "dX of a feature-sharded layer is a partial sum: the producer's activation backward comes after its All-Reduce");
  }
  return linear_bwd_impl(d, shard_index, X, W, preact, dY, dX, dW, dW_dtype, dbias, x_preact, x_act, ws, ws_bytes, stream);
}

static int linear_bwd_impl(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                           const void* preact, const void* dY, void* dX, void* dW, int dW_dtype,
                           float* dbias, const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream) {
  View v;
  int rc = resolve(d, shard_index, &v);
  if (rc) return rc;
  // pointers to slices the device owns nothing of may be NULL (a compact slice of size 0)
  const bool has_dp = v.tok_n > 0 && v.out_n > 0;
  if (x_act != HAP_ACT_NONE && v.tok_n > 0 && v.in_n > 0 && (!dX || !x_preact)) return hap_fail(HAP_EINVAL, "x_act given but dX or x_preact is NULL");
  if (x_act == HAP_ACT_NONE) x_preact = NULL;
  if (!dY && has_dp) return hap_fail(HAP_EINVAL, "dY is NULL");
  if (dX && !W && has_dp && v.in_n > 0) return hap_fail(HAP_EINVAL, "dX requested but W is NULL");
  if (dW && !X && has_dp && v.in_n > 0) return hap_fail(HAP_EINVAL, "dW requested but X is NULL");
  if (dW && dW_dtype != HAP_F32 && dW_dtype != HAP_BF16) return hap_fail(HAP_EINVAL, "bad dW_dtype %d", dW_dtype);
  if (dW && d->io_dtype == HAP_F32 && dW_dtype != HAP_F32) return hap_fail(HAP_EINVAL, "fp32 layer needs fp32 dW");
  if (dbias && d->mode == HAP_SHARD_REDUCTION) return hap_fail(HAP_EINVAL, "dbias is not defined for a reduction-sharded partial");
  if (d->act != HAP_ACT_NONE && !preact && has_dp) return hap_fail(HAP_EINVAL, "activation backward needs the saved pre-activation");
  const size_t need = required_bwd_bytes(d, shard_index);
  if (need && (d->act != HAP_ACT_NONE || dbias) && (!ws || ws_bytes < need))
    return hap_fail(HAP_EWORKSPACE, "linear_bwd needs %zu workspace bytes", need);
  // Empty shards need no special case: a product with an empty output is skipped by the engine and
  // one with an empty contraction (a partial of a device that owns nothing) is written as zeros.
  const int es = esize(d->io_dtype);
  const Offs o = offsets_of(d, v);

  // dP = dY * act'(preact), or dY itself
  const void* dP = at(dY, o.y, es);
  int64_t lddp = d->ldy;
  char* wsp = static_cast<char*>(ws);
  if (d->act != HAP_ACT_NONE) {
    // dP goes to the workspace with the same 16-byte phase as W's slice so that both K-contiguous
    // operands of the bwd-data product can be fetched with aligned chunks.
    lddp = dp_pitch(v.out_n, es);
    const int64_t phase = W ? (int64_t)(((uintptr_t)at(W, o.w, es) % 16) / es) : 0;
    char* dst = wsp + phase * es;
    rc = hap_gelu_bwd(v.tok_n, v.out_n, d->io_dtype, at(preact, o.y, es), d->ldy, dP, d->ldy, dst, lddp, stream);
    if (rc) return rc;
    dP = dst;
    wsp += round_up((int64_t)((size_t)(v.tok_n * lddp) * es), 256);
  }
  // [dP][column-sum scratch][optional split-K scratch for the GEMM engine]
  char* colsum_ws = wsp;
  char* gemm_ws = colsum_ws + round_up((int64_t)hap_colsum_workspace(v.tok_n, v.out_n), 256);
  const size_t used = ws ? (size_t)(gemm_ws - static_cast<char*>(ws)) : 0;
  const size_t gemm_ws_bytes = (ws && ws_bytes > used) ? ws_bytes - used : 0;
  if (dX) {
    hap_gemm_problem p = {};
    p.M = v.tok_n; p.N = v.in_n;
    p.nseg = 1; p.k[0] = v.out_n;
    p.a[0] = dP; p.lda = lddp; p.a_kcontig = 1;
    p.b[0] = at(W, o.w, es); p.ldb = d->ldw; p.b_kcontig = 1;   // B(k = out, n = in) = W[n*ldw + k]
    p.in_dtype = d->io_dtype;
    p.c = at(dX, o.x, es); p.ldc = d->ldx; p.c_dtype = d->io_dtype;
    if (x_preact) { p.dact_preact = at(x_preact, o.x, es); p.ldd = d->ldx; p.dact = x_act; }
    p.ws = gemm_ws_bytes ? gemm_ws : NULL; p.ws_bytes = gemm_ws_bytes;
    rc = hap_gemm_run(&p, stream);
    if (rc) return rc;
  }
  if (dW) {
    const int wes = esize(dW_dtype);
    hap_gemm_problem p = {};
    p.M = v.in_n; p.N = v.out_n;
    p.nseg = 1; p.k[0] = v.tok_n;
    p.a[0] = at(X, o.x, es); p.lda = d->ldx; p.a_kcontig = 0;   // A(m = in, k = token) = X[k*ldx + m]
    p.b[0] = dP; p.ldb = lddp; p.b_kcontig = 0;
    p.in_dtype = d->io_dtype;
    p.c = at(dW, o.w, wes); p.ldc = d->ldw; p.c_dtype = dW_dtype;
    p.ws = gemm_ws_bytes ? gemm_ws : NULL; p.ws_bytes = gemm_ws_bytes;
    rc = hap_gemm_run(&p, stream);
    if (rc) return rc;
  }
  if (dbias) {
    rc = hap_colsum(v.tok_n, v.out_n, d->io_dtype, dP, lddp, dbias + o.b, colsum_ws, hap_colsum_workspace(v.tok_n, v.out_n), stream);
    if (rc) return rc;
  }
  return HAP_OK;
}

size_t hap_sfb_workspace(int, const int64_t*, int64_t, int64_t) { return HAP_GEMM_WS_BYTES; }   // optional: split-K partial tiles

static int sfb_grad_impl(int m, const void* const* X, const void* const* dY, const int64_t* rows,
                         int64_t in_features, int64_t out_features, int64_t ldx, int64_t ldy, int in_dtype,
                         float* dW, int64_t lddw, int accumulate, void* ws, size_t ws_bytes, void* stream);

int hap_sfb_grad(int m, const void* const* X, const void* const* dY, const int64_t* rows,
                 int64_t in_features, int64_t out_features, int64_t ldx, int64_t ldy, int in_dtype,
                 float* dW, int64_t lddw, int accumulate, void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  return sfb_grad_impl(m, X, dY, rows, in_features, out_features, ldx, ldy, in_dtype, dW, lddw, accumulate, ws, ws_bytes, stream);
}

/* Split-K partial tiles of hap_sfb_grad_static: one array per GPU, held until the process ends.  In host code the
 * array's name is only a handle for hipGetSymbolAddress; kernels get the device address resolved below. */
static __device__ __align__(256) unsigned char scratch[HAP_SFB_STATIC_SCRATCH_BYTES];

int hap_sfb_grad_static(int m, const void* const* X, const void* const* dY, const int64_t* rows,
                        int64_t in_features, int64_t out_features, int64_t ldx, int64_t ldy, int in_dtype,
                        float* dW, int64_t lddw, int accumulate, void* stream) {
  hap_clear_error();
  if (in_features < 1 || out_features < 1) return hap_fail(HAP_EINVAL, "bad feature sizes");
  if (in_features > HAP_SFB_STATIC_MAX_ELEMS / out_features)
    return hap_fail(HAP_EUNSUPPORTED, "hap_sfb_grad_static: dW of %lld x %lld exceeds the %lld elements its fixed scratch is sized for; "
                    "use hap_sfb_grad with a caller workspace", (long long)in_features, (long long)out_features, (long long)HAP_SFB_STATIC_MAX_ELEMS);
  // each GPU holds its own copy of the array at its own address: resolve it once per device, with that device current
  static void* resolved[64] = {};
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return hap_fail(HAP_EDEVICE, "cannot identify the current device");
  void* ptr = __atomic_load_n(&resolved[device], __ATOMIC_ACQUIRE);
  if (!ptr) {
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return hap_fail(HAP_EDEVICE, "cannot resolve the static scratch array: %s", hipGetErrorString(e));
    __atomic_store_n(&resolved[device], ptr, __ATOMIC_RELEASE);     // every thread resolves the same address
  }
  // The partial tiles are written in full before the reduction reads them, so nothing has to be cleared between calls.
  return sfb_grad_impl(m, X, dY, rows, in_features, out_features, ldx, ldy, in_dtype, dW, lddw, accumulate, ptr,
                       (size_t)HAP_SFB_STATIC_SCRATCH_BYTES, stream);
}

static int sfb_grad_impl(int m, const void* const* X, const void* const* dY, const int64_t* rows,
                         int64_t in_features, int64_t out_features, int64_t ldx, int64_t ldy, int in_dtype,
                         float* dW, int64_t lddw, int accumulate, void* ws, size_t ws_bytes, void* stream) {
  if (m < 1 || m > HAP_SFB_MAX_DEVICES) return hap_fail(HAP_EINVAL, "m = %d outside [1, %d]", m, HAP_SFB_MAX_DEVICES);
  if (!X || !dY || !rows || !dW) return hap_fail(HAP_EINVAL, "NULL argument");
  if (in_features < 1 || out_features < 1) return hap_fail(HAP_EINVAL, "bad feature sizes");
  if (in_dtype != HAP_F32 && in_dtype != HAP_BF16) return hap_fail(HAP_EINVAL, "bad in_dtype %d", in_dtype);
  if (ldx < in_features || ldy < out_features || lddw < out_features) return hap_fail(HAP_ESHAPE, "leading dimension too small");
  hap_gemm_problem p = {};
  p.M = in_features; p.N = out_features;
  p.nseg = m;
  for (int i = 0; i < m; ++i) {
    if (rows[i] < 0) return hap_fail(HAP_EINVAL, "rows[%d] < 0", i);
    if (rows[i] > 0 && (!X[i] || !dY[i])) return hap_fail(HAP_EINVAL, "factor %d is NULL", i);
    p.k[i] = rows[i]; p.a[i] = X[i]; p.b[i] = dY[i];
  }
  p.lda = ldx; p.a_kcontig = 0;
  p.ldb = ldy; p.b_kcontig = 0;
  p.in_dtype = in_dtype;
  p.c = dW; p.ldc = lddw; p.c_dtype = HAP_F32;
  p.accumulate = accumulate ? 1 : 0;
  p.ws = ws; p.ws_bytes = ws ? ws_bytes : 0;
  return hap_gemm_run(&p, stream);
}

}  // extern "C"
