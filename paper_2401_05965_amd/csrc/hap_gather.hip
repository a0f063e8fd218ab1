/*
 * Data movement of an All-Gather over unevenly sharded tensors, as one device performs it
 * (Sec. 2.2; Sec. 2.3.1 and Fig. "comm_opt": padded All-Gather vs grouped Broadcast).
 *
 * Both layouts end with the same step: piece j (a padded slot, or the shard at its own size) is
 * copied to its range of the sharded axis of the full tensor.  All m pieces move in ONE launch:
 * blockIdx.y is the piece, the blocks of a piece stride over its rows x 16-byte chunks.  Shard sizes
 * are arbitrary integers, so nothing is assumed about alignment (see the kernel).
 * "Pad" (shard -> front of the device's send slot) is the same copy with a single piece.
 * A Reduce-Scatter over uneven shards needs equal pieces as well (Sec. 2.3.1): there the device cuts
 * its full partial tensor into m capacity-sized slots, shard range first, zeros behind.
 */
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "hap_internal.h"

namespace {

constexpr int kMaxPieces = HAP_SFB_MAX_DEVICES;

struct PieceArgs {
  int m;
  char* out;
  long long ld_out;                  // bytes
  const char* src[kMaxPieces];
  long long ld_src[kMaxPieces];      // bytes
  long long dst_off[kMaxPieces];     // bytes from out to the piece's first element
  long long rows[kMaxPieces];
  long long width[kMaxPieces];       // valid bytes per row
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

/* One thread per 16-byte chunk of a destination row, the chunks aligned in the DESTINATION's address space: whole
 * chunks are written with one aligned 16-byte store and read from wherever the source happens to lie (global
 * loads need no alignment on this target); the chunks that straddle the row's ends are copied bytewise.  A row has
 * at most (width + 30) / 16 chunks; rows whose start is aligned use fewer and leave the last index empty. */
__global__ __launch_bounds__(256) void copy_pieces_kernel(const PieceArgs a) {
  const int j = blockIdx.y;
  const long long width = a.width[j], nch = (width + 30) / 16, total = a.rows[j] * nch;
  const char* src = a.src[j];
  char* dst = a.out + a.dst_off[j];
  const long long lds = a.ld_src[j], ldd = a.ld_out;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long r = i / nch, k = i - r * nch;
    char* drow = dst + r * ldd;
    const char* srow = src + r * lds;
    const long long lo = 16 * k - (long long)(reinterpret_cast<uintptr_t>(drow) & 15), hi = lo + 16;   // byte range within the row
    if (lo >= 0 && hi <= width) {
      u32x4 v;
      __builtin_memcpy(&v, srow + lo, 16);
      *reinterpret_cast<u32x4*>(drow + lo) = v;
    } else {
      const long long b0 = lo < 0 ? 0 : lo, b1 = hi < width ? hi : width;
      for (long long b = b0; b < b1; ++b) drow[b] = srow[b];
    }
  }
}

int launch_pieces(const PieceArgs& a, hipStream_t s) {
  long long most = 0;
  for (int j = 0; j < a.m; ++j) {
    const long long chunks = a.rows[j] * ((a.width[j] + 30) / 16);
    if (a.rows[j] > 0 && a.width[j] > 0 && chunks > most) most = chunks;
  }
  if (most == 0) return HAP_OK;
  long long gx = (most + 255) / 256;
  if (gx > 256 * 32) gx = 256 * 32;        // grid-stride beyond 32 blocks per CU and piece
  hipLaunchKernelGGL(copy_pieces_kernel, dim3((unsigned)gx, (unsigned)a.m), dim3(256), 0, s, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "piece copy launch: %s", hipGetErrorString(e));
  return HAP_OK;
}

struct SplitArgs {
  const char* src;
  long long ld_src;                  // bytes
  long long srows, swidth;           // extent of every slot: rows, bytes per row
  char* dst[kMaxPieces];
  long long ld_dst[kMaxPieces];      // bytes
  long long src_off[kMaxPieces];     // bytes from src to the shard's first element
  long long vrows[kMaxPieces];       // the shard's part of the slot: rows, bytes per row; the rest is zero-filled
  long long vwidth[kMaxPieces];
};

/* The reverse movement: slot j (blockIdx.y) receives shard j's range of the full tensor and zeros up to the slot's
 * extent.  Same chunking as above: 16-byte chunks aligned in the destination, the source read wherever it lies,
 * chunks that straddle the row's ends or the shard's edge byte by byte. */
__global__ __launch_bounds__(256) void split_pieces_kernel(const SplitArgs a) {
  const int j = blockIdx.y;
  const long long swidth = a.swidth, vwidth = a.vwidth[j], vrows = a.vrows[j];
  const long long nch = (swidth + 30) / 16, total = a.srows * nch;
  const char* src = a.src + a.src_off[j];
  char* dst = a.dst[j];
  const long long lds = a.ld_src, ldd = a.ld_dst[j];
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long r = i / nch, k = i - r * nch;
    char* drow = dst + r * ldd;
    const char* srow = src + r * lds;                       // dereferenced for rows of the shard only
    const bool row_ok = r < vrows;
    const long long lo = 16 * k - (long long)(reinterpret_cast<uintptr_t>(drow) & 15), hi = lo + 16;
    if (lo >= 0 && hi <= swidth && row_ok && hi <= vwidth) {
      u32x4 v;
      __builtin_memcpy(&v, srow + lo, 16);
      *reinterpret_cast<u32x4*>(drow + lo) = v;
    } else if (lo >= 0 && hi <= swidth && (!row_ok || lo >= vwidth)) {
      const u32x4 z = {0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4*>(drow + lo) = z;
    } else {
      const long long b0 = lo < 0 ? 0 : lo, b1 = hi < swidth ? hi : swidth;
      for (long long b = b0; b < b1; ++b) drow[b] = (row_ok && b < vwidth) ? srow[b] : (char)0;
    }
  }
}

int check_desc(const hap_gather_desc* d) {
  if (!d) return hap_fail(HAP_EINVAL, "descriptor is NULL");
  if (d->rows < 0 || d->cols < 0) return hap_fail(HAP_EINVAL, "negative tensor size");
  if (d->dim != 0 && d->dim != 1) return hap_fail(HAP_EINVAL, "dim must be 0 or 1");
  if (d->elem_bytes != 1 && d->elem_bytes != 2 && d->elem_bytes != 4 && d->elem_bytes != 8) return hap_fail(HAP_EINVAL, "elem_bytes must be 1, 2, 4 or 8");
  if (d->m < 1 || d->m > kMaxPieces) return hap_fail(HAP_EINVAL, "m = %d outside [1, %d]", d->m, kMaxPieces);
  return HAP_OK;
}

}  // namespace

extern "C" {

int64_t hap_allgather_capacity(const hap_gather_desc* d) {
  hap_clear_error();
  if (check_desc(d)) return -1;
  int64_t cap = 0;
  for (int j = 0; j < d->m; ++j) {
    int64_t lo, hi;
    if (hap_shard_range(d->m, d->offsets, d->dim == 0 ? d->rows : d->cols, j, &lo, &hi)) return -1;
    if (hi - lo > cap) cap = hi - lo;
  }
  return cap;
}

int hap_allgather_pad(const hap_gather_desc* d, int shard_index, const void* shard, int64_t ld_shard, void* slot, int64_t ld_slot, void* stream) {
  hap_clear_error();
  int rc = check_desc(d);
  if (rc) return rc;
  int64_t lo, hi;
  if ((rc = hap_shard_range(d->m, d->offsets, d->dim == 0 ? d->rows : d->cols, shard_index, &lo, &hi))) return rc;
  const int64_t r = d->dim == 0 ? hi - lo : d->rows, c = d->dim == 0 ? d->cols : hi - lo;
  if (r == 0 || c == 0) return HAP_OK;
  if (!shard || !slot) return hap_fail(HAP_EINVAL, "NULL pointer");
  if (ld_shard < c || ld_slot < c) return hap_fail(HAP_ESHAPE, "leading dimension below the shard's width %lld", (long long)c);
  PieceArgs a = {};
  a.m = 1; a.out = static_cast<char*>(slot); a.ld_out = ld_slot * d->elem_bytes;
  a.src[0] = static_cast<const char*>(shard); a.ld_src[0] = ld_shard * d->elem_bytes;
  a.rows[0] = r; a.width[0] = c * d->elem_bytes;
  return launch_pieces(a, static_cast<hipStream_t>(stream));
}

int hap_allgather_assemble(const hap_gather_desc* d, const void* const* pieces, const int64_t* ld_pieces, void* out, int64_t ld_out, void* stream) {
  hap_clear_error();
  int rc = check_desc(d);
  if (rc) return rc;
  if (!pieces || !ld_pieces) return hap_fail(HAP_EINVAL, "NULL piece table");
  if (ld_out < d->cols) return hap_fail(HAP_ESHAPE, "ld_out below cols");
  PieceArgs a = {};
  a.m = d->m; a.out = static_cast<char*>(out); a.ld_out = ld_out * d->elem_bytes;
  for (int j = 0; j < d->m; ++j) {
    int64_t lo, hi;
    if ((rc = hap_shard_range(d->m, d->offsets, d->dim == 0 ? d->rows : d->cols, j, &lo, &hi))) return rc;
    const int64_t r = d->dim == 0 ? hi - lo : d->rows, c = d->dim == 0 ? d->cols : hi - lo;
    if (r == 0 || c == 0) continue;                      // an empty shard contributes nothing
    if (!pieces[j] || !out) return hap_fail(HAP_EINVAL, "piece %d or out is NULL", j);
    if (ld_pieces[j] < c) return hap_fail(HAP_ESHAPE, "piece %d: leading dimension %lld below its width %lld", j, (long long)ld_pieces[j], (long long)c);
    a.src[j] = static_cast<const char*>(pieces[j]); a.ld_src[j] = ld_pieces[j] * d->elem_bytes;
    a.dst_off[j] = (d->dim == 0 ? lo * ld_out : lo) * d->elem_bytes;
    a.rows[j] = r; a.width[j] = c * d->elem_bytes;
  }
  return launch_pieces(a, static_cast<hipStream_t>(stream));
}

int hap_reducescatter_split(const hap_gather_desc* d, const void* full, int64_t ld_full, void* const* slots, const int64_t* ld_slots, void* stream) {
  hap_clear_error();
  int rc = check_desc(d);
  if (rc) return rc;
  if (!slots || !ld_slots) return hap_fail(HAP_EINVAL, "NULL slot table");
  const int64_t cap = hap_allgather_capacity(d);
  if (cap < 0) return HAP_ESHAPE;
  const int64_t srows = d->dim == 0 ? cap : d->rows, scols = d->dim == 0 ? d->cols : cap;
  if (srows == 0 || scols == 0) return HAP_OK;
  if (!full) return hap_fail(HAP_EINVAL, "full is NULL");
  if (ld_full < d->cols) return hap_fail(HAP_ESHAPE, "ld_full below cols");
  SplitArgs a = {};
  a.src = static_cast<const char*>(full); a.ld_src = ld_full * d->elem_bytes;
  a.srows = srows; a.swidth = scols * d->elem_bytes;
  for (int j = 0; j < d->m; ++j) {
    int64_t lo, hi;
    if ((rc = hap_shard_range(d->m, d->offsets, d->dim == 0 ? d->rows : d->cols, j, &lo, &hi))) return rc;
    if (!slots[j]) return hap_fail(HAP_EINVAL, "slot %d is NULL", j);
    if (ld_slots[j] < scols) return hap_fail(HAP_ESHAPE, "slot %d: leading dimension %lld below the slot's width %lld", j, (long long)ld_slots[j], (long long)scols);
    a.dst[j] = static_cast<char*>(slots[j]); a.ld_dst[j] = ld_slots[j] * d->elem_bytes;
    a.src_off[j] = (d->dim == 0 ? lo * ld_full : lo) * d->elem_bytes;
    a.vrows[j] = d->dim == 0 ? hi - lo : d->rows;
    a.vwidth[j] = (d->dim == 0 ? d->cols : hi - lo) * d->elem_bytes;
  }
  long long gx = (srows * ((a.swidth + 30) / 16) + 255) / 256;
  if (gx > 256 * 32) gx = 256 * 32;
  hipLaunchKernelGGL(split_pieces_kernel, dim3((unsigned)gx, (unsigned)d->m), dim3(256), 0, static_cast<hipStream_t>(stream), a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "slot split launch: %s", hipGetErrorString(e));
  return HAP_OK;
}

}  // extern "C"
