/*
 * Internal GEMM engine of libhap.  One problem description covers every matrix product of the
 * hot path: the three sharded-MatMul rules and their backward products (Fig. "semantics") and the
 * sufficient-factor rebuild, whose contracted axis is a list of ragged segments (Fig. "sfb"(c)).
 *
 *   C[M x N] (+)= sum over segments s, k < k_s of  A_s(m, k) * B_s(k, n)      then bias / activation
 *
 * Operand element (m, k) of A lives at a[m*lda + k] (K-contiguous, a_kcontig = 1) or a[k*lda + m]
 * (M-contiguous, a_kcontig = 0); likewise B with (n, k).  No alignment is required of the caller:
 * the launcher derives aligned views or falls back to a scalar kernel.
 */
#ifndef HAP_GEMM_H
#define HAP_GEMM_H

#include <stddef.h>
#include <stdint.h>

#include "hap_internal.h"

#define HAP_GEMM_MAX_SEG HAP_SFB_MAX_DEVICES

struct hap_gemm_problem {
  int64_t M, N;
  int nseg;
  int64_t k[HAP_GEMM_MAX_SEG];         /* contracted length of each segment (>= 0)               */
  const void* a[HAP_GEMM_MAX_SEG];     /* per segment operand bases                              */
  const void* b[HAP_GEMM_MAX_SEG];
  int64_t lda, ldb;
  int a_kcontig, b_kcontig;
  int in_dtype;                        /* hap_dtype of A and B                                   */
  void* c; int64_t ldc; int c_dtype;   /* output; fp32 accumulate inside                          */
  int accumulate;                      /* C += result (c_dtype fp32 only)                         */
  const void* bias;                    /* [N] in in_dtype or NULL, added before the activation    */
  void* preact; int64_t ldp;           /* optional copy of (product + bias) in c_dtype            */
  int act;                             /* hap_act                                                 */
  int force_generic;                   /* testing aid: take the scalar fallback kernel            */
  void* ws; size_t ws_bytes;           /* optional device scratch for split-K partial tiles (NULL: never split K)   */
  int tile;                            /* 0: engine chooses (and may split the problem); 128 / 256: fixed output tile */
};

/* Validates nothing beyond what the kernels need (callers validate user input); returns hap_status. */
int hap_gemm_run(const hap_gemm_problem* p, void* stream);

/* Name of the kernel variant the launcher would choose, for reports. */
const char* hap_gemm_variant(const hap_gemm_problem* p);

/* Scratch that lets every problem split K as far as the engine would like to (an upper bound). */
#define HAP_GEMM_WS_BYTES ((size_t)64 << 20)

#endif
