/* Internal helpers shared by the host C file and the HIP translation units of libhap. */
#ifndef HAP_INTERNAL_H
#define HAP_INTERNAL_H

#include "libhap.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Records a printf-style detail message for hap_last_error() and returns `status`. */
int hap_fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void hap_clear_error(void);

/* Validates a shard descriptor's offsets array over an axis of length dim_len and returns the
 * half-open range of device j in lo and hi.  Returns HAP_OK or an error already recorded. */
int hap_shard_range(int m, const int64_t* offsets, int64_t dim_len, int j, int64_t* lo, int64_t* hi);

/* Column sums of `groups` matrices [rows x cols] (ld = lda) that lie group_stride elements apart; group g sums only
 * its first group_len[g] rows (group_len: DEVICE array clamped to [0, rows], or NULL = all rows) into out[g*ldo + c].
 * Does not clear the error state (hap_colsum is the public entry). */
size_t hap_colsum_grouped_workspace(int groups, int64_t rows, int64_t cols);
int hap_colsum_grouped(int groups, int64_t rows, int64_t cols, int io_dtype, const void* a, int64_t lda, int64_t group_stride,
                       const int32_t* group_len, float* out, int64_t ldo, void* ws, size_t ws_bytes, void* stream);

/* hap_gelu_bwd over `groups` row groups of `rows` rows each, stacked in the same buffers (group g starts at row g * rows);
 * group_len: DEVICE array clamped to [0, rows] (NULL = all rows): rows at or beyond it are neither read nor written.
 * Does not clear the error state. */
int hap_gelu_bwd_grouped(int groups, int64_t rows, int64_t cols, int io_dtype, const void* preact, int64_t ldp, const void* dy,
                         int64_t lddy, void* out, int64_t ldo, const int32_t* group_len, void* stream);

/* Test hook, not part of the public interface.  The tiled GEMM kernels address an operand with 32-bit offsets, so the
 * engine cuts a product whose operand view reaches 2 GiB into row blocks (K-contiguous operand: separate launches) or
 * contraction segments (M- / N-contiguous operand: one launch).  This lowers that threshold so that the cutting can be
 * exercised on small inputs; bytes <= 0 (or above the hardware reach) restores the default.  Returns how many products
 * the engine has run in pieces so far in this process.  Process-wide, not thread-safe. */
int64_t hap_debug_set_gemm_view_limit(int64_t bytes);

#ifdef __cplusplus
}
#endif
#endif
