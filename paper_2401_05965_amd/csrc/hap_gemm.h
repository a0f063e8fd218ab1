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
  const void* dact_preact; int64_t ldd; /* optional, in c_dtype: the result is multiplied by act'(dact_preact[m][n]) before it is
                                           stored (the activation backward of the layer that produced the output's tensor,
                                           folded into this product's epilogue); dact = the hap_act in question            */
  int dact;
  int force_generic;                   /* testing aid: take the scalar fallback kernel            */
  void* ws; size_t ws_bytes;           /* optional device scratch for split-K partial tiles (NULL: never split K)   */
  int tile;                            /* 0: engine chooses (and may split the problem); 128 / 256: fixed output tile */
  /* Grouped launch: `groups` independent products of the same shape in one launch, group g's operands
   * g strides further on (the experts of an MoE layer, Sec. 7.6).  Needs nseg == 1; neither strip
   * splitting nor split-K apply.  group_len (a DEVICE array, one int per group, or NULL) holds the valid
   * length of the ragged axis per group, clamped to [0, the problem's extent]: group_ragged = 1 bounds M
   * (rows of A and C beyond it are neither read nor written), 2 bounds the contraction k[0]. */
  int groups;                          /* 0 or 1: a single product                               */
  int64_t ga, gb, gbias;               /* strides between groups, in in_dtype elements           */
  int64_t gc, gp, gd;                  /* ... of C, preact and dact_preact, in c_dtype elements  */
  const int32_t* group_len;
  int group_ragged;
};

/* Validates nothing beyond what the kernels need (callers validate user input); returns hap_status. */
int hap_gemm_run(const hap_gemm_problem* p, void* stream);

/* Name of the kernel variant the launcher would choose, for reports. */
const char* hap_gemm_variant(const hap_gemm_problem* p);

/* Scratch that lets every problem split K as far as the engine would like to (an upper bound). */
#define HAP_GEMM_WS_BYTES ((size_t)64 << 20)

#endif
