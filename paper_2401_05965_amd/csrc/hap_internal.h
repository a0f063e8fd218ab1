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

#ifdef __cplusplus
}
#endif
#endif
