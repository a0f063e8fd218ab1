/*
 * Softmax attention restricted to a device's head or batch slice, forward and backward, bf16 with
 * fp32 softmax and accumulation, for gfx950.  Heads and batch entries are independent, so a
 * slice is simply a sub-grid of (batch, head) pairs of the whole [batch, seq, heads, head_dim] tensors.
 *
 * All three kernels work on TRANSPOSED score tiles so that the probabilities never leave registers:
 * an MFMA 32x32 accumulator holds, per lane, 16 rows of ONE column.  With scores laid out as
 * [key][query] (forward, dQ) a lane owns one query, so the running max / sum of the online softmax
 * are per-lane scalars (one cross-half shuffle finishes a row reduction) and the bf16-converted
 * accumulator is directly the B operand of the next MFMA (O^T = V^T P^T).  The matching A operand is
 * fetched from LDS with the transposing read, in the same permuted key order the accumulator has.
 *
 *   forward      per 32-query wave:  S^T = K Q^T,  online softmax,  O^T += V^T P^T
 *   backward dQ  per 32-query wave:  S^T, dP^T = V dO^T, dS^T = P^T (dP^T - D),  dQ^T += K^T dS^T
 *   backward dKV per 32-key wave:    S = Q K^T, dP = dO V^T, dS,  dV^T += dO^T P,  dK^T += Q^T dS
 * D[q] = sum_d dO[q,d] O[q,d] comes from a small pre-pass.  No atomics, deterministic.
 */
#include <hip/hip_runtime.h>

#include <type_traits>

#include <stdint.h>

#include "hap_internal.h"

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kTile = 64;     // rows of a K/V (or Q/dO) tile staged in LDS
constexpr int kWaves = 4;     // waves per workgroup, 32 rows of the outer axis each

struct AttnArgs {
  const __bf16 *q, *k, *v, *o, *dout;
  __bf16 *out, *dq, *dk, *dv;
  float* lse;        // [batch][heads][seq] whole-tensor indexing
  float* dsum;       // same indexing as lse, workspace
  float* lse2;       // lse * log2(e), workspace
  long long stride_b, stride_s, stride_h;      // Q, K, V and their gradients
  long long ostride_b, ostride_s, ostride_h;   // O and dO
  int seq, heads;    // whole-tensor head count (for lse indexing)
  int b0, h0;        // first batch entry / head of the slice
  float scale;
};

/* 16-byte chunk c of LDS row `row` (a row is D bf16) sits at chunk position c ^ f(row).  LDS serves 64
 * four-byte banks per clock: a 128-bit row read is served 16 lanes (16 consecutive rows, one chunk) at
 * a time, a transposing 64-bit read 32 lanes (4 consecutive rows x 4 consecutive chunks) at a time; f
 * spreads both over all 64 banks. */
template <int D>
__device__ __forceinline__ int swz(int row, int c) {
  if constexpr (D == 128) return c ^ (((row & 3) << 2) | ((row >> 2) & 3));
  else return c ^ ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

/* MFMA operand fetches from an LDS tile.
 *   rows (A operand, K-contiguous): rows of the tile are the MFMA M index, head_dim the contraction; one 128-bit read.
 *   cols (A operand, transposed): M index = head_dim column (32 starting at dt*32), contraction = tile rows in the
 *     accumulator's order (k-slot j of lane half h is row row_base + (j/4)*8 + h*4 + j%4); two transposing 64-bit reads.
 * The address arithmetic is folded: because the swizzle is an XOR, the byte address of every fragment of a tile is
 * ((lane constant + tile address) ^ small constant) + multiple of the row size, so a wave keeps two lane constants
 * instead of one address per fragment.
 *   rows:  row = row_base + lane%32, chunk ks*2 + lane/32:   (rows + tile) ^ (ks << 5)            + row_base * row bytes
 *   cols:  rows r0, r0 + 8 with r0 = row_base + (lane/32)*4 + (lane%16)/4, columns dt*32 + ((lane/16)%2)*16 + (lane%4)*4 ..:
 *          (cols + tile) ^ (dt << 6) [^ 32] + (row_base [+ 8]) * row bytes
 * (row_base a multiple of 16, tile address a multiple of 256; f(r + 8) = f(r) ^ 2 and f(r + 16) = f(r)). */
template <int D>
struct FragAddr {
  static constexpr int ROWB = D * 2;
  unsigned rows, cols;
  __device__ __forceinline__ void init(int lane) {
    const int r = lane & 31, h = lane >> 5;
    rows = (unsigned)(r * ROWB + ((h ^ swz<D>(r, 0)) << 4));
    const int g = lane >> 4, i = lane & 15;
    const int r0 = (g >> 1) * 4 + (i >> 2), cl = (g & 1) * 2 + ((i & 3) >> 1);
    cols = (unsigned)(r0 * ROWB + ((cl ^ swz<D>(r0, 0)) << 4) + (i & 1) * 8);
  }
};

__device__ __forceinline__ unsigned lds_addr(const void* p) { return (unsigned)(unsigned long)LDS_PTR(const char, p); }

/* `at` = FragAddr::rows + lds_addr(tile) */
template <int D>
__device__ __forceinline__ bf16x8_t frag_rows_at(unsigned at, int row_base, int ks) {
  const unsigned addr = (at ^ (unsigned)(ks << 5)) + (unsigned)(row_base * D * 2);
  return __builtin_bit_cast(bf16x8_t, *(LDS_PTR(const i32x4_t, (unsigned long)addr)));
}

/* `at` = FragAddr::cols + lds_addr(tile) */
template <int D>
__device__ __forceinline__ bf16x8_t frag_cols_at(unsigned at, int row_base, int dt) {
  const unsigned lo_addr = (at ^ (unsigned)(dt << 6)) + (unsigned)(row_base * D * 2);
  const unsigned hi_addr = (at ^ (unsigned)((dt << 6) ^ 32)) + (unsigned)((row_base + 8) * D * 2);
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, (unsigned long)lo_addr));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, (unsigned long)hi_addr));
  return __builtin_bit_cast(bf16x8_t, (s16x8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

/* B operand kept in registers: row `row` of a [seq][D] matrix, lane = row, 8 contiguous d per k-step. */
template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8_t (&f)[D / 16], const __bf16* base, long long stride_s, int row, int seq, int lane) {
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    i32x4_t v = {0, 0, 0, 0};
    if (row < seq) v = *reinterpret_cast<const i32x4_t*>(base + (long long)row * stride_s + ks * 16 + (lane >> 5) * 8);
    f[ks] = __builtin_bit_cast(bf16x8_t, v);
  }
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& a, int s) {
  bf16x8_t r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (__bf16)a[8 * s + j];
  return r;
}

__device__ __forceinline__ f32x16_t zero16() {
  f32x16_t z;
#pragma unroll
  for (int e = 0; e < 16; ++e) z[e] = 0.0f;
  return z;
}

__device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

/* accumulator element e of lane l: row (e/4)*8 + (l/32)*4 + e%4 */
__device__ __forceinline__ int acc_row(int e, int lane) { return (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3); }

/* Stores a transposed accumulator set acc[D/32] (rows = d, column = this lane's sequence row) to out[row][d]. */
template <int D>
__device__ __forceinline__ void store_rows(__bf16* base, long long stride_s, int row, int seq, const f32x16_t (&acc)[D / 32], float mul, int lane) {
  if (row >= seq) return;
  __bf16* p = base + (long long)row * stride_s;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4_t v;
#pragma unroll
      for (int x = 0; x < 4; ++x) v[x] = (__bf16)(acc[dt][g * 4 + x] * mul);
      *reinterpret_cast<bf16x4_t*>(p + dt * 32 + g * 8 + (lane >> 5) * 4) = v;
    }
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

/* Buffer descriptor over `bytes` bytes at `base` (wave-uniform): loads past the end return zero. */
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  const uintptr_t u = (uintptr_t)base;
  const uintptr_t v = ((uintptr_t)(unsigned)uni((int)(u >> 32)) << 32) | (unsigned)uni((int)(u & 0xffffffffu));
  return __builtin_amdgcn_make_buffer_rsrc((void*)v, 0, uni((int)bytes), 0x00020000);
}

/* One wave-wide direct load to LDS: lane l's 16 (4) bytes at byte offset voff + soff of the buffer land
 * at lds + 16*l (4*l).  `lds` must be wave-uniform.  The host pass of hipcc lacks the builtin. */
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, char* lds, unsigned voff, unsigned soff) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(void, lds), 16, voff, soff, 0, 0);
#else
  (void)rsrc; (void)lds; (void)voff; (void)soff;
#endif
}
__device__ __forceinline__ void dma4(__amdgpu_buffer_rsrc_t rsrc, char* lds, unsigned voff, unsigned soff) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(void, lds), 4, voff, soff, 0, 0);
#else
  (void)rsrc; (void)lds; (void)voff; (void)soff;
#endif
}

/* Rows [row0, row0 + ROWS) of a [seq x D] matrix (row stride in bytes given at init) go straight from
 * global memory to the swizzled LDS tile, no registers in between; the descriptor ends with row
 * seq - 1, so rows past the end arrive as zeros.  The loads are asynchronous: the caller waits for
 * vmcnt(0) and a barrier before any wave reads the tile. */
template <int D, int ROWS = kTile, int NT = 64 * kWaves>
struct TileDma {
  static constexpr int CPR = D / 8;
  static constexpr int CPT = ROWS * CPR / NT;     // NT: threads of the workgroup
  unsigned voff[CPT];
  unsigned stride_bytes;
  __device__ __forceinline__ void init(long long stride_s, int tid) {
    stride_bytes = (unsigned)stride_s * 2u;
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int id = tid + i * NT;                // 16-byte slot of the LDS tile this lane fills
      const int row = id / CPR, pos = id % CPR;
      voff[i] = (unsigned)row * stride_bytes + (unsigned)swz<D>(row, pos) * 16u;   // the chunk that belongs there
    }
  }
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, char* lds_tile, int row0, int tid) const {
    const int wave_first = uni(tid & ~63);
    const unsigned soff = (unsigned)uni(row0) * (unsigned)uni((int)stride_bytes);
#pragma unroll
    for (int i = 0; i < CPT; ++i) dma16(rsrc, lds_tile + (wave_first + i * NT) * 16, voff[i], soff);
  }
};

template <int D>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const __bf16* base, int seq, long long stride_s) {
  return make_rsrc(base, (unsigned)(((long long)(seq - 1) * stride_s + D) * 2));
}

__device__ __forceinline__ void wait_tiles_and_sync() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

/* Workgroups go to the 8 XCDs round-robin by linear id.  This renumbers them so that the workgroups of
 * one (batch entry, head) pair, which stream the same K/V (or Q/dO) rows, run on one XCD and share its
 * L2.  Returns the logical (x, y, z) of this workgroup. */
__device__ __forceinline__ void block_coords_of(unsigned id, unsigned gx, unsigned gy, unsigned gz, int& x, int& y, int& z) {
  const unsigned total = gx * gy * gz;
  if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
  x = (int)(id % gx); y = (int)((id / gx) % gy); z = (int)(id / (gx * gy));
}
__device__ __forceinline__ void block_coords(int& x, int& y, int& z) {
  block_coords_of(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), gridDim.x, gridDim.y, gridDim.z, x, y, z);
}

/* Largest growth of a row's running maximum (log2 units) that is absorbed without rescaling the
 * accumulators: probabilities are then at most 2^kLazy times larger than with the exact maximum, far
 * inside fp32 / bf16 range, and the final division by the row sum is unaffected. */
constexpr float kLazy = 8.0f;

template <int D>
__global__ __launch_bounds__(64 * kWaves, 2) void attn_fwd_kernel(const AttnArgs a) {
  constexpr int kTileBytes = kTile * D * 2;
  __shared__ __attribute__((aligned(256))) char lds[2][2][kTileBytes];   // [buffer][K, V]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  FragAddr<D> fa;
  fa.init(lane);
  int bx, by, bz;
  block_coords(bx, by, bz);
  const int b = a.b0 + bz, h = a.h0 + by;
  const long long head_off = (long long)b * a.stride_b + (long long)h * a.stride_h;
  const int q = bx * (32 * kWaves) + wave * 32 + (lane & 31);
  const __bf16* kbase = a.k + head_off;
  const __bf16* vbase = a.v + head_off;
  bf16x8_t qf[D / 16];
  load_row_frags<D>(qf, a.q + head_off, a.stride_s, q, a.seq, lane);
  f32x16_t o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) o[dt] = zero16();
  float m_ref = -INFINITY, l_i = 0.0f;    // m_ref: reference maximum of the exponent (scaled, log2 units)
  const float c = a.scale * kLog2e;
  const int ntiles = (a.seq + kTile - 1) / kTile;
  const __amdgpu_buffer_rsrc_t rk = tile_rsrc<D>(kbase, a.seq, a.stride_s), rv = tile_rsrc<D>(vbase, a.seq, a.stride_s);
  TileDma<D> td;
  td.init(a.stride_s, tid);
  td.issue(rk, lds[0][0], 0, tid);
  td.issue(rv, lds[0][1], 0, tid);
  wait_tiles_and_sync();
  // One tile of 64 keys; HALF: the last tile when its second 32 keys all lie past the end of the sequence (a 197-long
  // sequence: 3 tiles and 5 keys), which then costs half the matrix and exponential work.
  auto tile_body = [&](int t, auto half_tag) __attribute__((always_inline)) {
    constexpr int NSUB = decltype(half_tag)::value ? 1 : 2;
    const int kv0 = t * kTile;
    const char* lds_k = lds[t & 1][0];
    const char* lds_v = lds[t & 1][1];
    if (t + 1 < ntiles) {     // the other buffer was last read in iteration t-1, before the barrier
      td.issue(rk, lds[(t + 1) & 1][0], kv0 + kTile, tid);
      td.issue(rv, lds[(t + 1) & 1][1], kv0 + kTile, tid);
    }
    f32x16_t s[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
      s[sub] = zero16();
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) s[sub] = mfma(frag_rows_at<D>(fa.rows + lds_addr(lds_k), sub * 32, ks), qf[ks], s[sub]);
    }
    if (kv0 + kTile > a.seq) {   // ragged last tile: keys past the end drop out
#pragma unroll
      for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (kv0 + sub * 32 + acc_row(e, lane) >= a.seq) s[sub][e] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[sub][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c;   // finite: every tile holds at least one valid key
    if (__any(mx > m_ref + kLazy)) {
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
      l_i *= alpha;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
      m_ref = m_new;
    }
    float rs = 0.0f;
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s[sub][e] = __builtin_amdgcn_exp2f(fmaf(s[sub][e], c, -m_ref));
        rs += s[sub][e];
      }
    l_i += rs;      // this lane's half of the row; the halves meet after the loop
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
      for (int ss = 0; ss < 2; ++ss) {
        const bf16x8_t p = pack8(s[sub], ss);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) o[dt] = mfma(frag_cols_at<D>(fa.cols + lds_addr(lds_v), sub * 32 + ss * 16, dt), p, o[dt]);
      }
    wait_tiles_and_sync();
  };
  const bool last_half = (ntiles - 1) * kTile + 32 >= a.seq;
  const int nwhole = last_half ? ntiles - 1 : ntiles;
  for (int t = 0; t < nwhole; ++t) tile_body(t, std::false_type());
  if (last_half) tile_body(ntiles - 1, std::true_type());
  l_i += __shfl_xor(l_i, 32, 64);
  const long long ohead_off = (long long)b * a.ostride_b + (long long)h * a.ostride_h;
  store_rows<D>(a.out + ohead_off, a.ostride_s, q, a.seq, o, 1.0f / l_i, lane);
  if (q < a.seq && lane < 32) a.lse[((long long)b * a.heads + h) * a.seq + q] = (m_ref + log2f(l_i)) * kLn2;
}

/* D[q] = sum_d dO[q,d] * O[q,d] and lse[q] * log2(e); D/8 adjacent lanes share a (b, h, q) row, 16 bytes
 * of it each. */
template <int D>
__global__ __launch_bounds__(256) void attn_dsum_kernel(const AttnArgs a) {
  constexpr int LPR = D / 8;                       // lanes per row
  const int q = blockIdx.x * (256 / LPR) + threadIdx.x / LPR, c = threadIdx.x % LPR;
  const int b = a.b0 + blockIdx.z, h = a.h0 + blockIdx.y;
  float acc = 0.0f;
  if (q < a.seq) {
    const long long off = (long long)b * a.ostride_b + (long long)h * a.ostride_h + (long long)q * a.ostride_s + c * 8;
    const bf16x8_t x = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const i32x4_t*>(a.dout + off));
    const bf16x8_t y = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const i32x4_t*>(a.o + off));
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)x[e] * (float)y[e];
  }
#pragma unroll
  for (int sh = LPR / 2; sh >= 1; sh >>= 1) acc += __shfl_xor(acc, sh, 64);
  if (q < a.seq && c == 0) {
    const long long at = ((long long)b * a.heads + h) * a.seq + q;
    a.dsum[at] = acc;
    a.lse2[at] = a.lse[at] * kLog2e;
  }
}

/* dQ of 32 queries per wave (recomputes S and dP against every K/V tile).  smem: kDqSmem<D> bytes, 256-byte aligned. */
template <int D> constexpr int kDqSmem = 2 * 2 * kTile * D * 2;

template <int D>
__device__ __forceinline__ void attn_bwd_dq_body(const AttnArgs& a, char* smem, int bx, int by, int bz) {
  constexpr int kTileBytes = kTile * D * 2;
  char (*lds)[2][kTileBytes] = reinterpret_cast<char (*)[2][kTileBytes]>(smem);   // [buffer][K, V]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  FragAddr<D> fa;
  fa.init(lane);
  const int b = a.b0 + bz, h = a.h0 + by;
  const long long head_off = (long long)b * a.stride_b + (long long)h * a.stride_h;
  const long long stat_off = ((long long)b * a.heads + h) * a.seq;
  const int q = bx * (32 * kWaves) + wave * 32 + (lane & 31);
  const __bf16* kbase = a.k + head_off;
  const __bf16* vbase = a.v + head_off;
  bf16x8_t qf[D / 16], dof[D / 16];
  load_row_frags<D>(qf, a.q + head_off, a.stride_s, q, a.seq, lane);
  const long long ohead_off = (long long)b * a.ostride_b + (long long)h * a.ostride_h;
  load_row_frags<D>(dof, a.dout + ohead_off, a.ostride_s, q, a.seq, lane);
  const float lse2 = q < a.seq ? a.lse2[stat_off + q] : 0.0f;
  const float dsum = q < a.seq ? a.dsum[stat_off + q] : 0.0f;
  const float c = a.scale * kLog2e;
  f32x16_t dq[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) dq[dt] = zero16();
  const int ntiles = (a.seq + kTile - 1) / kTile;
  const __amdgpu_buffer_rsrc_t rk = tile_rsrc<D>(kbase, a.seq, a.stride_s), rv = tile_rsrc<D>(vbase, a.seq, a.stride_s);
  TileDma<D> td;
  td.init(a.stride_s, tid);
  td.issue(rk, lds[0][0], 0, tid);
  td.issue(rv, lds[0][1], 0, tid);
  wait_tiles_and_sync();
  // HALF: the last tile when its second 32 keys all lie past the end (their K rows are zero: nothing to add to dQ)
  auto tile_body = [&](int t, auto half_tag) __attribute__((always_inline)) {
    constexpr int NSUB = decltype(half_tag)::value ? 1 : 2;
    const int kv0 = t * kTile;
    const char* lds_k = lds[t & 1][0];
    const char* lds_v = lds[t & 1][1];
    if (t + 1 < ntiles) {     // the other buffer was last read in iteration t-1, before the barrier
      td.issue(rk, lds[(t + 1) & 1][0], kv0 + kTile, tid);
      td.issue(rv, lds[(t + 1) & 1][1], kv0 + kTile, tid);
    }
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
      f32x16_t s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        s = mfma(frag_rows_at<D>(fa.rows + lds_addr(lds_k), sub * 32, ks), qf[ks], s);
        dp = mfma(frag_rows_at<D>(fa.rows + lds_addr(lds_v), sub * 32, ks), dof[ks], dp);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[e], c, -lse2));
        s[e] = p * (dp[e] - dsum);          // dS^T
      }
      // keys past the end: their K rows are zero in LDS, so whatever dS holds there adds nothing to dQ
#pragma unroll
      for (int ss = 0; ss < 2; ++ss) {
        const bf16x8_t ds = pack8(s, ss);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) dq[dt] = mfma(frag_cols_at<D>(fa.cols + lds_addr(lds_k), sub * 32 + ss * 16, dt), ds, dq[dt]);
      }
    }
    wait_tiles_and_sync();
  };
  const bool last_half = (ntiles - 1) * kTile + 32 >= a.seq;
  const int nwhole = last_half ? ntiles - 1 : ntiles;
  for (int t = 0; t < nwhole; ++t) tile_body(t, std::false_type());
  if (last_half) tile_body(ntiles - 1, std::true_type());
  store_rows<D>(a.dq + head_off, a.stride_s, q, a.seq, dq, a.scale, lane);
}

/* dK, dV of 32 keys per wave.  K stays in registers; the block's 128 rows of V stay in LDS for the
 * whole kernel (each wave re-reads its own 32 rows as the second operand of dP = dO V^T), which keeps
 * the wave under 256 registers so that two blocks share a compute unit.  Q, dO and the row statistics
 * stream through LDS in 32-query tiles, double buffered. */
constexpr int kQTile = 32;
template <int D> constexpr int kDkvSmem = 2 * 2 * kQTile * D * 2 + 32 * kWaves * D * 2 + 2 * 2 * 64 * 4;

template <int D>
__device__ __forceinline__ void attn_bwd_dkv_body(const AttnArgs& a, char* smem, int bx, int by, int bz) {
  constexpr int kTileBytes = kQTile * D * 2;
  char (*lds)[2][kTileBytes] = reinterpret_cast<char (*)[2][kTileBytes]>(smem);                     // [buffer][Q, dO]
  char* lds_vres = smem + 4 * kTileBytes;                                                            // the block's 128 rows of V
  float (*lds_stat)[2][64] = reinterpret_cast<float (*)[2][64]>(smem + 4 * kTileBytes + 32 * kWaves * D * 2);   // [buffer][lse * log2(e), D]; 32 used
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  FragAddr<D> fa;
  fa.init(lane);
  const int b = a.b0 + bz, h = a.h0 + by;
  const long long head_off = (long long)b * a.stride_b + (long long)h * a.stride_h;
  const long long stat_off = ((long long)b * a.heads + h) * a.seq;
  const long long ohead_off = (long long)b * a.ostride_b + (long long)h * a.ostride_h;
  const int key0 = bx * (32 * kWaves);
  const int key = key0 + wave * 32 + (lane & 31);
  const __bf16* qbase = a.q + head_off;
  const __bf16* dobase = a.dout + ohead_off;
  // rows of keys past the end read as zero; whatever they accumulate is never stored
  bf16x8_t kf[D / 16];
  load_row_frags<D>(kf, a.k + head_off, a.stride_s, key, a.seq, lane);
  const float c = a.scale * kLog2e;
  f32x16_t dk[D / 32], dv[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) { dk[dt] = zero16(); dv[dt] = zero16(); }
  const int ntiles = (a.seq + kQTile - 1) / kQTile;
  const __amdgpu_buffer_rsrc_t rq = tile_rsrc<D>(qbase, a.seq, a.stride_s), rdo = tile_rsrc<D>(dobase, a.seq, a.ostride_s);
  const __amdgpu_buffer_rsrc_t rl = make_rsrc(a.lse2 + stat_off, (unsigned)a.seq * 4u), rd = make_rsrc(a.dsum + stat_off, (unsigned)a.seq * 4u);
  {
    const __amdgpu_buffer_rsrc_t rv = tile_rsrc<D>(a.v + head_off, a.seq, a.stride_s);
    TileDma<D, 32 * kWaves> tv;
    tv.init(a.stride_s, tid);
    tv.issue(rv, lds_vres, key0, tid);
  }
  TileDma<D, kQTile> tq, tdo;
  tq.init(a.stride_s, tid);
  tdo.init(a.ostride_s, tid);
  // Queries past the end arrive as zeros everywhere (Q, dO, lse, D): P = 1 there but dO = 0 and dS = 0,
  // so they add nothing to dV or dK.
  auto issue_tile = [&](int buf, int q0) {
    tq.issue(rq, lds[buf][0], q0, tid);
    tdo.issue(rdo, lds[buf][1], q0, tid);
    if (wave == 0) {
      dma4(rl, reinterpret_cast<char*>(lds_stat[buf][0]), (unsigned)lane * 4u, (unsigned)uni(q0) * 4u);
      dma4(rd, reinterpret_cast<char*>(lds_stat[buf][1]), (unsigned)lane * 4u, (unsigned)uni(q0) * 4u);
    }
  };
  issue_tile(0, 0);
  wait_tiles_and_sync();
  for (int t = 0; t < ntiles; ++t) {
    const char* lds_q = lds[t & 1][0];
    const char* lds_do = lds[t & 1][1];
    const float* lds_lse = lds_stat[t & 1][0];
    const float* lds_dsum = lds_stat[t & 1][1];
    if (t + 1 < ntiles) issue_tile((t + 1) & 1, (t + 1) * kQTile);   // that buffer was last read in iteration t-1, before the barrier
    f32x16_t s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      s = mfma(frag_rows_at<D>(fa.rows + lds_addr(lds_q), 0, ks), kf[ks], s);
      dp = mfma(frag_rows_at<D>(fa.rows + lds_addr(lds_do), 0, ks), frag_rows_at<D>(fa.rows + lds_addr(lds_vres), wave * 32, ks), dp);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int ql = g * 8 + (lane >> 5) * 4;
      const f32x4_t l4 = *reinterpret_cast<const f32x4_t*>(lds_lse + ql);
      const f32x4_t d4 = *reinterpret_cast<const f32x4_t*>(lds_dsum + ql);
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int e = g * 4 + x;
        const float p = __builtin_amdgcn_exp2f(fmaf(s[e], c, -l4[x]));
        dp[e] = p * (dp[e] - d4[x]);   // dS
        s[e] = p;                       // P
      }
    }
#pragma unroll
    for (int ss = 0; ss < 2; ++ss) {
      const bf16x8_t pf = pack8(s, ss), dsf = pack8(dp, ss);
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
        dv[dt] = mfma(frag_cols_at<D>(fa.cols + lds_addr(lds_do), ss * 16, dt), pf, dv[dt]);
        dk[dt] = mfma(frag_cols_at<D>(fa.cols + lds_addr(lds_q), ss * 16, dt), dsf, dk[dt]);
      }
    }
    wait_tiles_and_sync();
  }
  store_rows<D>(a.dv + head_off, a.stride_s, key, a.seq, dv, 1.0f, lane);
  store_rows<D>(a.dk + head_off, a.stride_s, key, a.seq, dk, a.scale, lane);
}

/* Both halves of the backward in ONE launch of 2 x (blocks per half) workgroups: z < gridDim.z / 2 computes dK / dV,
 * the rest dQ.  The two are independent, so the dQ workgroups start as soon as slots free up behind the (longer) dK / dV
 * ones instead of waiting for that kernel's last, partly filled round: 640 + 640 workgroups on 512 slots are 2.5 rounds
 * rather than 2 + 2.  Both bodies carve the same LDS buffer, which keeps two workgroups per compute unit. */
template <int D>
__global__ __launch_bounds__(64 * kWaves, 2) void attn_bwd_kernel(const AttnArgs a) {
  constexpr int kSmem = kDkvSmem<D> > kDqSmem<D> ? kDkvSmem<D> : kDqSmem<D>;
  __shared__ __attribute__((aligned(256))) char smem[kSmem];
  const unsigned gz = gridDim.z / 2;
  const bool dq_role = blockIdx.z >= gz;
  int bx, by, bz;
  block_coords_of(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * (blockIdx.z - (dq_role ? gz : 0u))), gridDim.x, gridDim.y, gz, bx, by, bz);
  if (dq_role) attn_bwd_dq_body<D>(a, smem, bx, by, bz);
  else attn_bwd_dkv_body<D>(a, smem, bx, by, bz);
}

int resolve(const hap_attn_desc* d, int j, int* b0, int* nb, int* h0, int* nh) {
  if (!d) return hap_fail(HAP_EINVAL, "descriptor is NULL");
  if (d->batch < 1 || d->heads < 1 || d->seq < 1) return hap_fail(HAP_EINVAL, "bad attention sizes");
  if (d->head_dim != 64 && d->head_dim != 128) return hap_fail(HAP_EUNSUPPORTED, "head_dim %lld (supported: 64, 128)", (long long)d->head_dim);
  if (d->io_dtype != HAP_BF16) return hap_fail(HAP_EUNSUPPORTED, "attention supports bf16 only");
  if (d->seq > 0x7fffffff / 2 || d->heads > 65535 || d->batch > 65535) return hap_fail(HAP_EUNSUPPORTED, "attention extent too large");
  if (d->stride_s < d->head_dim || d->stride_h < d->head_dim) return hap_fail(HAP_ESHAPE, "strides overlap head_dim");
  if (d->stride_s % 8 || d->stride_h % 8 || d->stride_b % 8) return hap_fail(HAP_EUNSUPPORTED, "strides must be multiples of 8 elements");
  if (d->o_stride_s || d->o_stride_h || d->o_stride_b) {
    if (d->o_stride_s < d->head_dim || d->o_stride_h < d->head_dim) return hap_fail(HAP_ESHAPE, "O strides overlap head_dim");
    if (d->o_stride_s % 8 || d->o_stride_h % 8 || d->o_stride_b % 8) return hap_fail(HAP_EUNSUPPORTED, "strides must be multiples of 8 elements");
  }
  // tiles are fetched through 32-bit buffer offsets within one (batch entry, head) matrix
  const int64_t widest = d->o_stride_s > d->stride_s ? d->o_stride_s : d->stride_s;
  if ((d->seq + kTile) * widest * 2 >= ((int64_t)1 << 31)) return hap_fail(HAP_EUNSUPPORTED, "seq * stride_s beyond 2^30 elements");
  int64_t lo, hi;
  const int rc = hap_shard_range(d->m, d->offsets, d->shard_over_heads ? d->heads : d->batch, j, &lo, &hi);
  if (rc) return rc;
  *b0 = 0; *nb = (int)d->batch; *h0 = 0; *nh = (int)d->heads;
  if (d->shard_over_heads) { *h0 = (int)lo; *nh = (int)(hi - lo); }
  else { *b0 = (int)lo; *nb = (int)(hi - lo); }
  return HAP_OK;
}

int check_ptr(const void* p, const char* name) {
  if (!p) return hap_fail(HAP_EINVAL, "%s is NULL", name);
  if ((uintptr_t)p % 16) return hap_fail(HAP_EUNSUPPORTED, "%s must be 16-byte aligned", name);
  return HAP_OK;
}

int launched(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "%s launch: %s", what, hipGetErrorString(e));
  return HAP_OK;
}

}  // namespace

extern "C" {

int hap_sharded_attn_fwd(const hap_attn_desc* d, int shard_index, const void* Q, const void* K, const void* V,
                         void* O, float* lse, void*, size_t, void* stream) {
  hap_clear_error();
  int b0, nb, h0, nh;
  int rc = resolve(d, shard_index, &b0, &nb, &h0, &nh);
  if (rc) return rc;
  if (nb == 0 || nh == 0) return HAP_OK;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(V, "V")) || (rc = check_ptr(O, "O"))) return rc;
  if (!lse) return hap_fail(HAP_EINVAL, "lse is NULL");
  AttnArgs a = {};
  a.q = (const __bf16*)Q; a.k = (const __bf16*)K; a.v = (const __bf16*)V; a.out = (__bf16*)O; a.lse = lse;
  a.stride_b = d->stride_b; a.stride_s = d->stride_s; a.stride_h = d->stride_h;
  const bool own_o = d->o_stride_s || d->o_stride_h || d->o_stride_b;
  a.ostride_b = own_o ? d->o_stride_b : d->stride_b; a.ostride_s = own_o ? d->o_stride_s : d->stride_s; a.ostride_h = own_o ? d->o_stride_h : d->stride_h;
  a.seq = (int)d->seq; a.heads = (int)d->heads; a.b0 = b0; a.h0 = h0;
  a.scale = 1.0f / sqrtf((float)d->head_dim);
  const dim3 grid((unsigned)((d->seq + 32 * kWaves - 1) / (32 * kWaves)), (unsigned)nh, (unsigned)nb);
  hipStream_t s = (hipStream_t)stream;
  if (d->head_dim == 128) hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(64 * kWaves), 0, s, a);
  else hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(64 * kWaves), 0, s, a);
  return launched("attn_fwd");
}

size_t hap_attn_bwd_workspace(const hap_attn_desc* d, int) {
  if (!d || d->batch < 1 || d->heads < 1 || d->seq < 1) return 0;
  return (size_t)(d->batch * d->heads * d->seq) * 2 * sizeof(float);   // D and lse * log2(e)
}

int hap_sharded_attn_bwd(const hap_attn_desc* d, int shard_index, const void* Q, const void* K, const void* V,
                         const void* O, const float* lse, const void* dO, void* dQ, void* dK, void* dV,
                         void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  int b0, nb, h0, nh;
  int rc = resolve(d, shard_index, &b0, &nb, &h0, &nh);
  if (rc) return rc;
  if (nb == 0 || nh == 0) return HAP_OK;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(V, "V")) || (rc = check_ptr(O, "O")) ||
      (rc = check_ptr(dO, "dO")) || (rc = check_ptr(dQ, "dQ")) || (rc = check_ptr(dK, "dK")) || (rc = check_ptr(dV, "dV"))) return rc;
  if (!lse) return hap_fail(HAP_EINVAL, "lse is NULL");
  const size_t need = hap_attn_bwd_workspace(d, shard_index);
  if (!ws || ws_bytes < need) return hap_fail(HAP_EWORKSPACE, "attn_bwd needs %zu workspace bytes", need);
  AttnArgs a = {};
  a.q = (const __bf16*)Q; a.k = (const __bf16*)K; a.v = (const __bf16*)V; a.o = (const __bf16*)O; a.dout = (const __bf16*)dO;
  a.dq = (__bf16*)dQ; a.dk = (__bf16*)dK; a.dv = (__bf16*)dV;
  a.lse = const_cast<float*>(lse); a.dsum = (float*)ws; a.lse2 = a.dsum + d->batch * d->heads * d->seq;
  a.stride_b = d->stride_b; a.stride_s = d->stride_s; a.stride_h = d->stride_h;
  const bool own_o = d->o_stride_s || d->o_stride_h || d->o_stride_b;
  a.ostride_b = own_o ? d->o_stride_b : d->stride_b; a.ostride_s = own_o ? d->o_stride_s : d->stride_s; a.ostride_h = own_o ? d->o_stride_h : d->stride_h;
  a.seq = (int)d->seq; a.heads = (int)d->heads; a.b0 = b0; a.h0 = h0;
  a.scale = 1.0f / sqrtf((float)d->head_dim);
  hipStream_t s = (hipStream_t)stream;
  const dim3 grid((unsigned)((d->seq + 32 * kWaves - 1) / (32 * kWaves)), (unsigned)nh, (unsigned)nb);
  const int rows_per_block = 256 / (int)(d->head_dim / 8);
  const dim3 grid_d((unsigned)((d->seq + rows_per_block - 1) / rows_per_block), (unsigned)nh, (unsigned)nb);
  if (2 * (int64_t)nb > 65535) return hap_fail(HAP_EUNSUPPORTED, "more than 32767 batch entries in one call");
  const dim3 grid2(grid.x, grid.y, 2 * grid.z);     // dK / dV workgroups first, dQ workgroups behind them
  if (d->head_dim == 128) {
    hipLaunchKernelGGL(attn_dsum_kernel<128>, grid_d, dim3(256), 0, s, a);
    if ((rc = launched("attn_dsum"))) return rc;
    hipLaunchKernelGGL(attn_bwd_kernel<128>, grid2, dim3(64 * kWaves), 0, s, a);
  } else {
    hipLaunchKernelGGL(attn_dsum_kernel<64>, grid_d, dim3(256), 0, s, a);
    if ((rc = launched("attn_dsum"))) return rc;
    hipLaunchKernelGGL(attn_bwd_kernel<64>, grid2, dim3(64 * kWaves), 0, s, a);
  }
  return launched("attn_bwd");
}

}  // extern "C"
