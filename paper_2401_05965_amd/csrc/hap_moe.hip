/*
 * Expert-sharded Mixture-of-Experts layer (Sec. 7.6, "Uneven Placement of Experts"): argument
 * validation and the mapping of a device's experts onto ONE grouped launch of the GEMM engine per
 * product.  No arithmetic happens here.
 *
 *   forward   Y_e  = X_e W_e          group e: A = X_e (K-contiguous), B = W_e (N-contiguous); rows[e] bounds M
 *   bwd-data  dX_e = dP_e W_e^T       A = dP_e (K-contiguous), B = W_e read as [n=in][k=out];  rows[e] bounds M
 *   bwd-wgt   dW_e = X_e^T dP_e       A = X_e read as [m=in][k=token], B = dP_e;               rows[e] bounds K
 *   bias-grad db_e = column sums of the first rows[e] rows of dP_e
 */
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "hap_gemm.h"

namespace {

inline int esize(int dtype) { return dtype == HAP_BF16 ? 2 : 4; }
inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline const char* at(const void* p, int64_t elems, int es) { return static_cast<const char*>(p) + elems * es; }
inline char* at(void* p, int64_t elems, int es) { return static_cast<char*>(p) + elems * es; }

int resolve(const hap_moe_desc* d, int j, int64_t* lo, int64_t* n) {
  if (!d) return hap_fail(HAP_EINVAL, "descriptor is NULL");
  if (d->experts < 1 || d->capacity < 0 || d->in_features < 1 || d->out_features < 1) return hap_fail(HAP_EINVAL, "bad layer sizes");
  if (d->io_dtype != HAP_F32 && d->io_dtype != HAP_BF16) return hap_fail(HAP_EINVAL, "bad io_dtype %d", d->io_dtype);
  if (d->act != HAP_ACT_NONE && d->act != HAP_ACT_GELU_ERF) return hap_fail(HAP_EINVAL, "bad act %d", d->act);
  int64_t hi = 0;
  const int rc = hap_shard_range(d->m, d->offsets, d->experts, j, lo, &hi);
  if (rc) return rc;
  *n = hi - *lo;
  if (d->ldx < d->in_features || d->ldw < d->out_features || d->ldy < d->out_features)
    return hap_fail(HAP_ESHAPE, "leading dimension too small (ldx %lld < %lld or ldw %lld < %lld or ldy %lld < %lld)", (long long)d->ldx,
                    (long long)d->in_features, (long long)d->ldw, (long long)d->out_features, (long long)d->ldy, (long long)d->out_features);
  if (*n > 65535) return hap_fail(HAP_EUNSUPPORTED, "more than 65535 experts on one device");
  if (d->capacity > 0x7fffffff) return hap_fail(HAP_EUNSUPPORTED, "capacity beyond 2^31");
  return HAP_OK;
}

/* Row pitch of the dP copy: a multiple of 128 bytes (it is the K-contiguous operand of the bwd-data products, whose row fetches
 * should not straddle cache sectors), with 8 spare elements for the 16-byte phase of W's slice. */
inline int64_t lddp_of(const hap_moe_desc* d) { return round_up(d->out_features + 8, 128 / esize(d->io_dtype)); }

size_t dp_bytes(const hap_moe_desc* d, int64_t n) {
  return d->act == HAP_ACT_NONE ? 0 : (size_t)round_up((n * d->capacity * lddp_of(d) + 8) * esize(d->io_dtype), 256);
}

/* The fields every product of the layer shares. */
hap_gemm_problem grouped(const hap_moe_desc* d, int64_t n, const int32_t* rows, int ragged) {
  hap_gemm_problem p = {};
  p.nseg = 1;
  p.in_dtype = d->io_dtype;
  p.groups = (int)n;
  p.group_len = rows;
  p.group_ragged = rows ? ragged : 0;
  return p;
}

}  // namespace

extern "C" {

static size_t required_bwd_bytes(const hap_moe_desc* d, int64_t n, bool with_dbias) {
  return dp_bytes(d, n) + (with_dbias ? (size_t)round_up((int64_t)hap_colsum_grouped_workspace((int)n, d->capacity, d->out_features), 256) : 0);
}

size_t hap_moe_linear_fwd_workspace(const hap_moe_desc* d, int shard_index) {
  int64_t lo, n;
  if (resolve(d, shard_index, &lo, &n) != HAP_OK || n == 0 || d->capacity == 0) return 0;
  return HAP_GEMM_WS_BYTES;                                   // optional: split-K partial tiles
}

size_t hap_moe_linear_bwd_workspace(const hap_moe_desc* d, int shard_index) {
  int64_t lo, n;
  if (resolve(d, shard_index, &lo, &n) != HAP_OK || n == 0 || d->capacity == 0) return 0;
  return required_bwd_bytes(d, n, true) + HAP_GEMM_WS_BYTES;  // the last part is optional split-K scratch
}

int hap_moe_linear_fwd(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* bias,
                       const int32_t* rows, void* Y, void* preact, void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  int64_t lo, n;
  const int rc = resolve(d, shard_index, &lo, &n);
  if (rc) return rc;
  if (n == 0 || d->capacity == 0) return HAP_OK;        // the device owns no expert
  if (!X || !W || !Y) return hap_fail(HAP_EINVAL, "X, W or Y is NULL");
  if ((d->has_bias != 0) != (bias != NULL)) return hap_fail(HAP_EINVAL, "bias pointer and has_bias disagree");
  const int es = esize(d->io_dtype);
  const int64_t first = d->operands_are_full ? lo : 0;
  const int64_t gx = d->capacity * d->ldx, gw = d->in_features * d->ldw, gy = d->capacity * d->ldy;
  hap_gemm_problem p = grouped(d, n, rows ? rows + first : NULL, 1);
  p.M = d->capacity; p.N = d->out_features; p.k[0] = d->in_features;
  p.a[0] = at(X, first * gx, es); p.lda = d->ldx; p.a_kcontig = 1; p.ga = gx;
  p.b[0] = at(W, first * gw, es); p.ldb = d->ldw; p.b_kcontig = 0; p.gb = gw;
  p.c = at(Y, first * gy, es); p.ldc = d->ldy; p.c_dtype = d->io_dtype; p.gc = gy;
  if (bias) { p.bias = at(bias, first * d->out_features, es); p.gbias = d->out_features; }
  if (preact) { p.preact = at(preact, first * gy, es); p.ldp = d->ldy; p.gp = gy; }
  p.act = d->act;
  p.ws = ws; p.ws_bytes = ws ? ws_bytes : 0;
  return hap_gemm_run(&p, stream);
}

static int moe_linear_bwd_impl(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* preact,
                               const void* dY, const int32_t* rows, void* dX, void* dW, int dW_dtype, float* dbias,
                               const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream);

int hap_moe_linear_bwd(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* preact,
                       const void* dY, const int32_t* rows, void* dX, void* dW, int dW_dtype, float* dbias,
                       void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  return moe_linear_bwd_impl(d, shard_index, X, W, preact, dY, rows, dX, dW, dW_dtype, dbias, NULL, HAP_ACT_NONE, ws, ws_bytes, stream);
}

int hap_moe_linear_bwd_dact(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* preact,
                            const void* dY, const int32_t* rows, void* dX, void* dW, int dW_dtype, float* dbias,
                            const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  if (x_act != HAP_ACT_NONE && x_act != HAP_ACT_GELU_ERF) return hap_fail(HAP_EINVAL, "bad x_act %d", x_act);
  return moe_linear_bwd_impl(d, shard_index, X, W, preact, dY, rows, dX, dW, dW_dtype, dbias, x_act != HAP_ACT_NONE ? x_preact : NULL, x_act,
                             ws, ws_bytes, stream);
}

static int moe_linear_bwd_impl(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* preact,
                               const void* dY, const int32_t* rows, void* dX, void* dW, int dW_dtype, float* dbias,
                               const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream) {
  int64_t lo, n;
  int rc = resolve(d, shard_index, &lo, &n);
  if (rc) return rc;
  if (n == 0) return HAP_OK;
  if (dW && dW_dtype != HAP_F32 && dW_dtype != HAP_BF16) return hap_fail(HAP_EINVAL, "bad dW_dtype %d", dW_dtype);
  if (dW && d->io_dtype == HAP_F32 && dW_dtype != HAP_F32) return hap_fail(HAP_EINVAL, "fp32 layer needs fp32 dW");
  const bool live = d->capacity > 0;
  if (live && !dY) return hap_fail(HAP_EINVAL, "dY is NULL");
  if (live && dX && !W) return hap_fail(HAP_EINVAL, "dX requested but W is NULL");
  if (live && dW && !X) return hap_fail(HAP_EINVAL, "dW requested but X is NULL");
  if (live && d->act != HAP_ACT_NONE && !preact) return hap_fail(HAP_EINVAL, "activation backward needs the saved pre-activation");
  if (live && x_act != HAP_ACT_NONE && (!dX || !x_preact)) return hap_fail(HAP_EINVAL, "x_act given but dX or x_preact is NULL");
  const size_t need = required_bwd_bytes(d, n, dbias != NULL);
  if (live && need && (!ws || ws_bytes < need)) return hap_fail(HAP_EWORKSPACE, "moe_linear_bwd needs %zu workspace bytes", need);
  // [dP][column-sum scratch][optional split-K scratch for the GEMM engine]
  char* gemm_ws = ws ? static_cast<char*>(ws) + need : NULL;
  const size_t gemm_ws_bytes = (ws && ws_bytes > need) ? ws_bytes - need : 0;
  const int es = esize(d->io_dtype);
  const int64_t first = d->operands_are_full ? lo : 0;
  const int64_t gx = d->capacity * d->ldx, gw = d->in_features * d->ldw, gy = d->capacity * d->ldy;
  const int32_t* rows_j = rows ? rows + first : NULL;

  // dP = dY * act'(preact) over the token rows of the device's experts, or dY itself
  const void* dP = dY ? at(dY, first * gy, es) : NULL;
  int64_t lddp = d->ldy, gdp = gy;
  char* wsp = static_cast<char*>(ws);
  if (live && d->act != HAP_ACT_NONE) {
    // same 16-byte phase as the experts' W so that both K-contiguous operands of the bwd-data product take aligned chunks
    lddp = lddp_of(d); gdp = d->capacity * lddp;
    const int64_t phase = W ? (int64_t)(((uintptr_t)at(W, first * gw, es) % 16) / es) : 0;
    char* dst = wsp + phase * es;
    rc = hap_gelu_bwd_grouped((int)n, d->capacity, d->out_features, d->io_dtype, at(preact, first * gy, es), d->ldy, dP, d->ldy, dst, lddp,
                              rows_j, stream);
    if (rc) return rc;
    dP = dst;
    wsp += dp_bytes(d, n);
  }
  if (dX && live) {
    hap_gemm_problem p = grouped(d, n, rows_j, 1);
    p.M = d->capacity; p.N = d->in_features; p.k[0] = d->out_features;
    p.a[0] = dP; p.lda = lddp; p.a_kcontig = 1; p.ga = gdp;
    p.b[0] = at(W, first * gw, es); p.ldb = d->ldw; p.b_kcontig = 1; p.gb = gw;     // B(k = out, n = in) = W_e[n*ldw + k]
    p.c = at(dX, first * gx, es); p.ldc = d->ldx; p.c_dtype = d->io_dtype; p.gc = gx;
    if (x_preact) { p.dact_preact = at(x_preact, first * gx, es); p.ldd = d->ldx; p.gd = gx; p.dact = x_act; }
    p.ws = gemm_ws_bytes ? gemm_ws : NULL; p.ws_bytes = gemm_ws_bytes;
    if ((rc = hap_gemm_run(&p, stream))) return rc;
  }
  if (dW) {
    const int wes = esize(dW_dtype);
    hap_gemm_problem p = grouped(d, n, rows_j, 2);
    p.M = d->in_features; p.N = d->out_features; p.k[0] = d->capacity;
    p.a[0] = live ? at(X, first * gx, es) : NULL; p.lda = d->ldx; p.a_kcontig = 0; p.ga = gx;   // A(m = in, k = token) = X_e[k*ldx + m]
    p.b[0] = dP; p.ldb = lddp; p.b_kcontig = 0; p.gb = gdp;
    p.c = at(dW, first * gw, wes); p.ldc = d->ldw; p.c_dtype = dW_dtype; p.gc = gw;
    p.ws = gemm_ws_bytes ? gemm_ws : NULL; p.ws_bytes = gemm_ws_bytes;
    if ((rc = hap_gemm_run(&p, stream))) return rc;
  }
  if (dbias) {
    rc = hap_colsum_grouped((int)n, d->capacity, d->out_features, d->io_dtype, dP, lddp, gdp, rows_j, dbias + first * d->out_features,
                            d->out_features, wsp, hap_colsum_grouped_workspace((int)n, d->capacity, d->out_features), stream);
    if (rc) return rc;
  }
  return HAP_OK;
}

}  // extern "C"
