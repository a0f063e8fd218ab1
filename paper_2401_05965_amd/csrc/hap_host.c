/*
 * Host side of libhap: sharding-ratio LP (Sec. 5.1, Eq. (opt_B)), the cost model it minimises
 * (Sec. 3.2), integer rounding of shard sizes (Sec. 5.1) and ownership ranges (Sec. 6).
 * Plain C, no GPU calls.
 */
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hap_internal.h"

static _Thread_local char g_err[512];

int hap_fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}

void hap_clear_error(void) { g_err[0] = 0; }

const char* hap_last_error(void) { return g_err; }

const char* hap_version(void) { return "libhap 0.1 (gfx950)"; }

const char* hap_strerror(int status) {
  switch (status) {
    case HAP_OK: return "ok";
    case HAP_EINVAL: return "invalid argument";
    case HAP_ESHAPE: return "inconsistent shape, offsets or leading dimension";
    case HAP_EINFEASIBLE: return "linear program infeasible";
    case HAP_EUNBOUNDED: return "linear program unbounded";
    case HAP_EWORKSPACE: return "workspace missing or too small";
    case HAP_EDEVICE: return "HIP launch failed";
    case HAP_EUNSUPPORTED: return "not supported by this build";
    default: return "unknown status";
  }
}

int hap_shard_range(int m, const int64_t* offsets, int64_t dim_len, int j, int64_t* lo, int64_t* hi) {
  if (m < 1) return hap_fail(HAP_EINVAL, "m = %d < 1", m);
  if (!offsets) return hap_fail(HAP_EINVAL, "offsets is NULL");
  if (j < 0 || j >= m) return hap_fail(HAP_EINVAL, "shard_index %d outside [0, %d)", j, m);
  if (offsets[0] != 0) return hap_fail(HAP_ESHAPE, "offsets[0] = %lld, expected 0", (long long)offsets[0]);
  for (int x = 0; x < m; ++x)
    if (offsets[x + 1] < offsets[x])
      return hap_fail(HAP_ESHAPE, "offsets not monotone at %d", x);
  if (offsets[m] != dim_len)
    return hap_fail(HAP_ESHAPE, "offsets[m] = %lld, expected the dimension length %lld",
                    (long long)offsets[m], (long long)dim_len);
  *lo = offsets[j];
  *hi = offsets[j + 1];
  return HAP_OK;
}

/* ---------------------------------------------------------------- cost model (Sec. 3.2) --- */

static int check_lp_inputs(int m, const double* speed, int n_stages, const hap_stage* st) {
  if (m < 1 || m > 256) return hap_fail(HAP_EINVAL, "m = %d outside [1, 256]", m);
  if (n_stages < 1 || n_stages > 256) return hap_fail(HAP_EINVAL, "n_stages = %d outside [1, 256]", n_stages);
  if (!speed || !st) return hap_fail(HAP_EINVAL, "speed or stages is NULL");
  for (int j = 0; j < m; ++j)
    if (!(speed[j] > 0.0) || !isfinite(speed[j])) return hap_fail(HAP_EINVAL, "speed[%d] must be positive and finite", j);
  for (int i = 0; i < n_stages; ++i) {
    const double v[4] = {st[i].flops_sharded, st[i].flops_fixed, st[i].comm_latency, st[i].comm_per_ratio};
    for (int q = 0; q < 4; ++q)
      if (!(v[q] >= 0.0) || !isfinite(v[q])) return hap_fail(HAP_EINVAL, "stage %d has a negative or non-finite field", i);
  }
  return HAP_OK;
}

int hap_iteration_time(int m, const double* speed, int n_stages, const hap_stage* st,
                       const double* ratios, double* seconds) {
  hap_clear_error();
  int rc = check_lp_inputs(m, speed, n_stages, st);
  if (rc) return rc;
  if (!ratios || !seconds) return hap_fail(HAP_EINVAL, "ratios or seconds is NULL");
  double bmax = ratios[0];
  for (int j = 1; j < m; ++j) if (ratios[j] > bmax) bmax = ratios[j];
  double total = 0.0;
  for (int i = 0; i < n_stages; ++i) {
    double comp = 0.0;
    for (int j = 0; j < m; ++j) {
      double c = (st[i].flops_sharded * ratios[j] + st[i].flops_fixed) / speed[j];
      if (j == 0 || c > comp) comp = c;
    }
    total += st[i].comm_latency + st[i].comm_per_ratio * bmax + comp;
  }
  *seconds = total;
  return HAP_OK;
}

/* ---------------------------------------------------------------- simplex --- */

/* Dense tableau, rows 0..R-1 constraints (all equalities with rhs >= 0), row R the reduced costs.
 * Column C is the right-hand side.  basis[r] = index of the basic variable of row r. */
typedef struct { int R, C; double* a; int* basis; } tableau;

#define T(t, r, c) ((t)->a[(size_t)(r) * ((t)->C + 1) + (c)])

static void pivot(tableau* t, int pr, int pc) {
  const int W = t->C + 1;
  double* prow = &t->a[(size_t)pr * W];
  const double inv = 1.0 / prow[pc];
  for (int c = 0; c < W; ++c) prow[c] *= inv;
  prow[pc] = 1.0;
  for (int r = 0; r <= t->R; ++r) {
    if (r == pr) continue;
    double* row = &t->a[(size_t)r * W];
    const double f = row[pc];
    if (f == 0.0) continue;
    for (int c = 0; c < W; ++c) row[c] -= f * prow[c];
    row[pc] = 0.0;
  }
  t->basis[pr] = pc;
}

/* Minimises the objective held in row R over the first `ncols` columns (Bland's rule: lowest-index
 * entering column, lowest-index leaving basic variable among ties).  0 ok, 1 unbounded. */
static int simplex_run(tableau* t, int ncols, double eps) {
  for (long it = 0; it < 200000L + 50L * t->R * t->C; ++it) {
    int pc = -1;
    for (int c = 0; c < ncols; ++c)
      if (T(t, t->R, c) < -eps) { pc = c; break; }
    if (pc < 0) return 0;
    int pr = -1; double best = 0.0;
    for (int r = 0; r < t->R; ++r) {
      const double a = T(t, r, pc);
      if (a > eps) {
        const double q = T(t, r, t->C) / a;
        if (pr < 0 || q < best - 1e-15 * fabs(best) ||
            (q <= best + 1e-15 * fabs(best) && t->basis[r] < t->basis[pr])) { pr = r; best = q; }
      }
    }
    if (pr < 0) return 1;
    pivot(t, pr, pc);
  }
  return 2;
}

int hap_shard_ratios(int m, const double* speed, int n_stages, const hap_stage* st,
                     double* ratios, double* objective) {
  hap_clear_error();
  int rc = check_lp_inputs(m, speed, n_stages, st);
  if (rc) return rc;
  if (!ratios) return hap_fail(HAP_EINVAL, "ratios is NULL");

  /* Presolve: stages whose compute term has the same fixed/sharded proportion share one epigraph
   * variable, since max_j (F B_j + G)/s_j = F max_j (B_j + G/F)/s_j.  Stages without sharded flops
   * contribute the constant G / min_j s_j. */
  double smin = speed[0];
  for (int j = 1; j < m; ++j) if (speed[j] < smin) smin = speed[j];
  double* clsF = (double*)calloc((size_t)n_stages, sizeof(double));
  double* clsRho = (double*)calloc((size_t)n_stages, sizeof(double));
  if (!clsF || !clsRho) { free(clsF); free(clsRho); return hap_fail(HAP_EINVAL, "out of host memory"); }
  int S = 0;
  double constant = 0.0, ccoef = 0.0;
  for (int i = 0; i < n_stages; ++i) {
    constant += st[i].comm_latency;
    ccoef += st[i].comm_per_ratio;
    if (st[i].flops_sharded == 0.0) { constant += st[i].flops_fixed / smin; continue; }
    const double rho = st[i].flops_fixed / st[i].flops_sharded;
    int k = 0;
    for (; k < S; ++k) if (clsRho[k] == rho) break;
    if (k == S) { clsRho[S] = rho; clsF[S] = 0.0; ++S; }
    clsF[k] += st[i].flops_sharded;
  }

  /* Scale times so the largest coefficient is O(1). */
  double scale = ccoef;
  for (int k = 0; k < S; ++k) { const double v = clsF[k] * (1.0 + clsRho[k]) / smin; if (v > scale) scale = v; }
  if (scale <= 0.0) scale = 1.0;

  /* Columns: B_0..B_{m-1} | u | tau_0..tau_{S-1} | slack of (B_j <= u) | slack of epigraph rows | artificial.
   * tau_k = t_k - gmax_k with gmax_k = F_k rho_k / smin >= 0 keeps every right-hand side non-negative. */
  const int cB = 0, cU = m, cT = m + 1, cS1 = m + 1 + S, cS2 = cS1 + m, cArt = cS2 + m * S;
  tableau t;
  t.R = 1 + m + m * S;
  t.C = cArt + 1;
  if ((double)(t.R + 1) * (double)(t.C + 1) > 6.4e7) {
    free(clsF); free(clsRho);
    return hap_fail(HAP_EUNSUPPORTED, "LP too large for the dense solver (%d rows x %d columns)", t.R, t.C);
  }
  t.a = (double*)calloc((size_t)(t.R + 1) * (size_t)(t.C + 1), sizeof(double));
  t.basis = (int*)calloc((size_t)t.R, sizeof(int));
  if (!t.a || !t.basis) { free(t.a); free(t.basis); free(clsF); free(clsRho); return hap_fail(HAP_EINVAL, "out of host memory"); }

  for (int j = 0; j < m; ++j) T(&t, 0, cB + j) = 1.0;        /* sum B = 1 */
  T(&t, 0, cArt) = 1.0; T(&t, 0, t.C) = 1.0; t.basis[0] = cArt;
  for (int j = 0; j < m; ++j) {                              /* B_j - u + s = 0 */
    const int r = 1 + j;
    T(&t, r, cB + j) = 1.0; T(&t, r, cU) = -1.0; T(&t, r, cS1 + j) = 1.0; t.basis[r] = cS1 + j;
  }
  for (int k = 0; k < S; ++k) {
    const double gmax = clsF[k] * clsRho[k] / smin;
    for (int j = 0; j < m; ++j) {                            /* F/s_j B_j - tau_k + s = gmax - G/s_j */
      const int r = 1 + m + k * m + j;
      T(&t, r, cB + j) = clsF[k] / speed[j] / scale;
      T(&t, r, cT + k) = -1.0;
      T(&t, r, cS2 + k * m + j) = 1.0;
      T(&t, r, t.C) = (gmax - clsF[k] * clsRho[k] / speed[j]) / scale;
      t.basis[r] = cS2 + k * m + j;
    }
  }
  const double eps = 1e-11;
  int status = HAP_OK;
  /* Phase 1: minimise the artificial.  Reduced-cost row = -(row 0), artificial column priced out. */
  for (int c = 0; c <= t.C; ++c) T(&t, t.R, c) = -T(&t, 0, c);
  T(&t, t.R, cArt) = 0.0;
  int sr = simplex_run(&t, cArt, eps);
  if (sr != 0 || fabs(T(&t, t.R, t.C)) > 1e-9) status = hap_fail(HAP_EINFEASIBLE, "phase 1 did not reach a feasible point");
  if (status == HAP_OK) {
    for (int r = 0; r < t.R; ++r)
      if (t.basis[r] == cArt) {                              /* degenerate: drive the artificial out */
        for (int c = 0; c < cArt; ++c) if (fabs(T(&t, r, c)) > eps) { pivot(&t, r, c); break; }
      }
    /* Phase 2 objective: ccoef*u + sum_k tau_k (scaled), priced out against the basis. */
    for (int c = 0; c <= t.C; ++c) T(&t, t.R, c) = 0.0;
    T(&t, t.R, cU) = ccoef / scale;
    for (int k = 0; k < S; ++k) T(&t, t.R, cT + k) = 1.0;
    for (int r = 0; r < t.R; ++r) {
      const int b = t.basis[r];
      const double f = T(&t, t.R, b);
      if (b < cArt && f != 0.0)
        for (int c = 0; c <= t.C; ++c) T(&t, t.R, c) -= f * T(&t, r, c);
    }
    sr = simplex_run(&t, cArt, eps);
    if (sr == 1) status = hap_fail(HAP_EUNBOUNDED, "phase 2 unbounded");
    else if (sr == 2) status = hap_fail(HAP_EINFEASIBLE, "simplex iteration limit reached");
  }
  if (status == HAP_OK) {
    double sum = 0.0;
    for (int j = 0; j < m; ++j) ratios[j] = 0.0;
    for (int r = 0; r < t.R; ++r)
      if (t.basis[r] >= cB && t.basis[r] < cB + m) {
        double v = T(&t, r, t.C);
        ratios[t.basis[r] - cB] = v > 0.0 ? v : 0.0;
      }
    for (int j = 0; j < m; ++j) sum += ratios[j];
    for (int j = 0; j < m; ++j) ratios[j] /= sum;
    if (objective) {
      double sec;
      hap_iteration_time(m, speed, n_stages, st, ratios, &sec);
      *objective = sec;
    }
  }
  free(t.a); free(t.basis); free(clsF); free(clsRho);
  return status;
}

/* ---------------------------------------------------------------- per-segment ratios (Sec. 5.2) --- */

static int check_segments(int n_stages, int g, const int* seg_offsets) {
  if (g < 1) return hap_fail(HAP_EINVAL, "g = %d < 1", g);
  if (!seg_offsets) return hap_fail(HAP_EINVAL, "seg_offsets is NULL");
  if (seg_offsets[0] != 0 || seg_offsets[g] != n_stages) return hap_fail(HAP_ESHAPE, "segments must cover stages [0, %d)", n_stages);
  for (int k = 0; k < g; ++k)
    if (seg_offsets[k + 1] <= seg_offsets[k]) return hap_fail(HAP_ESHAPE, "segment %d holds no stage", k);
  return HAP_OK;
}

int hap_shard_ratios_segments(int m, const double* speed, int n_stages, const hap_stage* st, int g, const int* seg_offsets,
                              double* ratios, double* objective) {
  hap_clear_error();
  int rc = check_lp_inputs(m, speed, n_stages, st);
  if (rc) return rc;
  if ((rc = check_segments(n_stages, g, seg_offsets))) return rc;
  if (!ratios) return hap_fail(HAP_EINVAL, "ratios is NULL");
  double total = 0.0;
  for (int k = 0; k < g; ++k) {   /* a synchronisation point at every boundary: the segments are independent problems */
    double sec = 0.0;
    rc = hap_shard_ratios(m, speed, seg_offsets[k + 1] - seg_offsets[k], st + seg_offsets[k], ratios + (size_t)k * m, &sec);
    if (rc) return rc;
    total += sec;
  }
  if (objective) *objective = total;
  return HAP_OK;
}

int hap_iteration_time_segments(int m, const double* speed, int n_stages, const hap_stage* st, int g, const int* seg_offsets,
                                const double* ratios, double* seconds) {
  hap_clear_error();
  int rc = check_lp_inputs(m, speed, n_stages, st);
  if (rc) return rc;
  if ((rc = check_segments(n_stages, g, seg_offsets))) return rc;
  if (!ratios || !seconds) return hap_fail(HAP_EINVAL, "ratios or seconds is NULL");
  double total = 0.0;
  for (int k = 0; k < g; ++k) {
    double sec = 0.0;
    rc = hap_iteration_time(m, speed, seg_offsets[k + 1] - seg_offsets[k], st + seg_offsets[k], ratios + (size_t)k * m, &sec);
    if (rc) return rc;
    total += sec;
  }
  *seconds = total;
  return HAP_OK;
}

/* ---------------------------------------------------------------- rounding (Sec. 5.1) --- */

int hap_round_shards(int m, const double* ratios, int64_t dim_len, int64_t granule,
                     int64_t* sizes, int64_t* offsets) {
  hap_clear_error();
  if (m < 1) return hap_fail(HAP_EINVAL, "m = %d < 1", m);
  if (!ratios || !sizes || !offsets) return hap_fail(HAP_EINVAL, "NULL argument");
  if (dim_len < 0) return hap_fail(HAP_EINVAL, "dim_len < 0");
  if (granule < 1 || dim_len % granule) return hap_fail(HAP_ESHAPE, "granule %lld must be >= 1 and divide dim_len %lld",
                                                       (long long)granule, (long long)dim_len);
  double rs = 0.0;
  for (int j = 0; j < m; ++j) {
    if (!(ratios[j] >= 0.0) || !isfinite(ratios[j])) return hap_fail(HAP_EINVAL, "ratios[%d] negative or non-finite", j);
    rs += ratios[j];
  }
  if (fabs(rs - 1.0) > 1e-6) return hap_fail(HAP_EINVAL, "ratios sum to %.9g, expected 1", rs);
  const int64_t units = dim_len / granule;
  double* x = (double*)malloc((size_t)m * sizeof(double));
  if (!x) return hap_fail(HAP_EINVAL, "out of host memory");
  int64_t total = 0;
  for (int j = 0; j < m; ++j) {
    x[j] = ratios[j] * (double)units;
    sizes[j] = (int64_t)floor(x[j] + 0.5);
    total += sizes[j];
  }
  while (total > units) {
    int best = -1; double be = 0.0;
    for (int j = 0; j < m; ++j) {
      if (sizes[j] <= 0) continue;
      const double e = fabs((double)(sizes[j] - 1) - x[j]);
      if (best < 0 || e < be) { best = j; be = e; }
    }
    sizes[best] -= 1; total -= 1;
  }
  while (total < units) {
    int best = -1; double be = 0.0;
    for (int j = 0; j < m; ++j) {
      const double e = fabs((double)(sizes[j] + 1) - x[j]);
      if (best < 0 || e < be) { best = j; be = e; }
    }
    sizes[best] += 1; total += 1;
  }
  free(x);
  offsets[0] = 0;
  for (int j = 0; j < m; ++j) { sizes[j] *= granule; offsets[j + 1] = offsets[j] + sizes[j]; }
  return HAP_OK;
}
