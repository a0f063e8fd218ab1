/*
 * Memory-bound row / element kernels of libhap: GeLU backward, residual / bias add, column sums
 * (bias gradients), LayerNorm forward / backward.  The paper treats these as stock single-device
 * operators; here they are the HBM-bound epilogues around the sharded GEMMs.  All arithmetic is
 * fp32, I/O in the tensor dtype; reductions across a wavefront use 64-lane shuffles.
 */
#include <hip/hip_runtime.h>

#include <stdint.h>

#include <type_traits>

#include "hap_internal.h"

namespace {

constexpr float kLnEps = 1e-5f;

template <typename T> __device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<__bf16>(const __bf16* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void st(T* p, float v);
template <> __device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<__bf16>(__bf16* p, float v) { *p = (__bf16)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float gelu_grad(float x) {
  const float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
  const float pdf = 0.3989422804014327f * __expf(-0.5f * x * x);
  return cdf + x * pdf;
}

/* Vector of V elements of T moved as one access when V > 1. */
template <typename T, int V> struct Pack { T v[V]; } __attribute__((aligned(sizeof(T) * V)));

/* out[r,c] = dy[r,c] * gelu'(pre[r,c]); V elements per thread along the row (V = 1 handles any alignment).  With V > 1 the
 * leading dimensions are multiples of V, so the last chunk of a ragged row (cols % V != 0) is still read whole - the
 * bytes lie inside the row's pitch, and an aligned chunk that starts inside an allocation cannot leave its page - and only
 * its valid elements are stored. */
/* blockIdx.y: one of several row groups of `rows` rows each, stacked in the same buffers; with group_len only the first
 * group_len[g] rows of group g are processed (the experts of an MoE layer and their token counts). */
/* skew (RAGGED only): the three views start `skew` elements past a 16-byte boundary (a column range of whole tensors, e.g.
 * columns 8402.. of a bf16 matrix); the pointers passed are the views' bases moved down to that boundary, chunks are
 * aligned in the buffers' own address space and the first chunk of a row is ragged as well. */
template <typename T, int V, bool RAGGED>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(int64_t rows, int64_t cols, const T* pre, int64_t ldp,
                                                       const T* dy, int64_t lddy, T* out, int64_t ldo, const int* group_len, int skew) {
  cols += skew;      // physical columns counted from the aligned base; logical column = physical - skew
  const int64_t cv = (cols + V - 1) / V;
  pre += (int64_t)blockIdx.y * rows * ldp; dy += (int64_t)blockIdx.y * rows * lddy; out += (int64_t)blockIdx.y * rows * ldo;
  if (group_len) {
    const int64_t len = group_len[blockIdx.y];
    rows = len < 0 ? 0 : (len < rows ? len : rows);
  }
  const int64_t total = rows * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cv, c = (i % cv) * V;
    Pack<T, V> p = *reinterpret_cast<const Pack<T, V>*>(pre + r * ldp + c);
    Pack<T, V> g = *reinterpret_cast<const Pack<T, V>*>(dy + r * lddy + c);
    Pack<T, V> o;
#pragma unroll
    for (int e = 0; e < V; ++e) o.v[e] = (T)((float)g.v[e] * gelu_grad((float)p.v[e]));
    if (!RAGGED || (c + V <= cols && c >= skew)) {
      *reinterpret_cast<Pack<T, V>*>(out + r * ldo + c) = o;
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (c + e < cols && c + e >= skew) out[r * ldo + c + e] = o.v[e];
    }
  }
}

/* out = a + b (+ bias per column).  BV: the bias can be fetched as one V-element chunk (its base is aligned like the rows). */
template <typename T, int V, bool BV>
__global__ __launch_bounds__(256) void add_kernel(int64_t rows, int64_t cols, const T* a, int64_t lda, const T* b,
                                                  int64_t ldb, const T* bias, T* out, int64_t ldo) {
  const int64_t cv = (cols + V - 1) / V;
  const int64_t total = rows * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cv, c = (i % cv) * V;
    Pack<T, V> x = *reinterpret_cast<const Pack<T, V>*>(a + r * lda + c);
    Pack<T, V> y = *reinterpret_cast<const Pack<T, V>*>(b + r * ldb + c);
    Pack<T, V> o, bb;
    if (BV && bias) bb = *reinterpret_cast<const Pack<T, V>*>(bias + c);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      float v = (float)x.v[e] + (float)y.v[e];
      if (bias) v += BV ? (float)bb.v[e] : (float)bias[c + e];
      o.v[e] = (T)v;
    }
    *reinterpret_cast<Pack<T, V>*>(out + r * ldo + c) = o;
  }
}

/* Column sums, stage 1: block (bx, by) sums rows [by*rpb, (by+1)*rpb) of the 64*V columns starting at
 * bx*64*V - skew.  `a` is the caller's pointer moved down by `skew` elements to a multiple of V
 * elements, so each lane reads one aligned V-element chunk per row (a chunk is read only when it
 * holds at least one wanted column).  The 4 waves stride over the rows, eight rows in flight each, and
 * their partials meet in LDS.  partial[by][col] is fp32. */
template <typename T, int V>
__global__ __launch_bounds__(256) void colsum_partial_kernel(int64_t rows, int64_t cols, const T* a, int64_t lda, int skew,
                                                             int64_t rpb, float* partial, int64_t group_stride, const int* group_len) {
  __shared__ float red[4][64 * V];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // blockIdx.z: one of several matrices group_stride elements apart, each with its own count of valid rows
  a += blockIdx.z * group_stride;
  partial += (int64_t)blockIdx.z * gridDim.y * cols;
  if (group_len) {
    const int64_t len = group_len[blockIdx.z];
    rows = len < 0 ? 0 : (len < rows ? len : rows);
  }
  const int64_t c0 = ((int64_t)blockIdx.x * 64 + lane) * V - skew;
  const int64_t r0 = (int64_t)blockIdx.y * rpb;
  const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
  float s[V];
#pragma unroll
  for (int e = 0; e < V; ++e) s[e] = 0.0f;
  if (c0 + V > 0 && c0 < cols) {
    const T* p = a + c0 + skew;
    int64_t r = r0 + wave;
    for (; r + 28 < r1; r += 32) {
      Pack<T, V> q[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) q[u] = *reinterpret_cast<const Pack<T, V>*>(p + (r + 4 * u) * lda);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < V; ++e) s[e] += (float)q[u].v[e];
    }
    for (; r < r1; r += 4) {
      const Pack<T, V> q = *reinterpret_cast<const Pack<T, V>*>(p + r * lda);
#pragma unroll
      for (int e = 0; e < V; ++e) s[e] += (float)q.v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < V; ++e) red[wave][lane * V + e] = s[e];
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * V; i += 256) {
    const int64_t c = (int64_t)blockIdx.x * 64 * V + i - skew;
    if (c >= 0 && c < cols) partial[(int64_t)blockIdx.y * cols + c] = red[0][i] + red[1][i] + red[2][i] + red[3][i];
  }
}

/* Stage 2: out[c] = sum over nparts of partial[p][c].  A block owns 16 columns; its 16 thread groups
 * walk the partial rows 16 apart and meet in LDS. */
__global__ __launch_bounds__(256) void colsum_final_kernel(int64_t cols, int nparts, const float* partial, float* out, int64_t ldo) {
  __shared__ float red[16][17];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  partial += (int64_t)blockIdx.y * nparts * cols;     // blockIdx.y: group
  out += blockIdx.y * ldo;
  const int64_t c = (int64_t)blockIdx.x * 16 + tx;
  float a = 0.0f;
  if (c < cols) {    // four independent partial sums keep four loads in flight per thread
    float a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    int p = ty;
    for (; p + 48 < nparts; p += 64) {
      a += partial[(int64_t)p * cols + c];
      a1 += partial[(int64_t)(p + 16) * cols + c];
      a2 += partial[(int64_t)(p + 32) * cols + c];
      a3 += partial[(int64_t)(p + 48) * cols + c];
    }
    for (; p < nparts; p += 16) a += partial[(int64_t)p * cols + c];
    a = (a + a1) + (a2 + a3);
  }
  red[ty][tx] = a;
  __syncthreads();
  if (ty == 0 && c < cols) {
    float t = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) t += red[r][tx];
    out[c] = t;
  }
}

/* LayerNorm kernels: one wavefront per row, the row held in registers as NCH chunks of V elements per
 * lane (chunk index i*64 + lane, so a wave reads 64*V contiguous elements per access: 16-byte accesses
 * when V = 16 / sizeof(T)).  Row length n <= 64 * V * NCH; n % V == 0 when V > 1. */
template <typename T, int V, int NCH>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(int64_t rows, int n, const T* x, const T* gamma, const T* beta,
                                                            T* y, float* mean, float* rstd) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + row * n;
  float v[NCH][V];
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * 64 + lane) * V;
    Pack<T, V> p;
    if (c < n) p = *reinterpret_cast<const Pack<T, V>*>(xr + c);
#pragma unroll
    for (int e = 0; e < V; ++e) { v[i][e] = c < n ? (float)p.v[e] : 0.0f; s += v[i][e]; }
  }
  const float mu = wave_sum(s) / (float)n;
  float q = 0.0f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * 64 + lane) * V;
#pragma unroll
    for (int e = 0; e < V; ++e) { const float d = c < n ? v[i][e] - mu : 0.0f; q += d * d; }
  }
  const float rs = rsqrtf(wave_sum(q) / (float)n + kLnEps);
  T* yr = y + row * n;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * 64 + lane) * V;
    if (c < n) {
      const Pack<T, V> g = *reinterpret_cast<const Pack<T, V>*>(gamma + c);
      const Pack<T, V> b = *reinterpret_cast<const Pack<T, V>*>(beta + c);
      Pack<T, V> o;
#pragma unroll
      for (int e = 0; e < V; ++e) o.v[e] = (T)((v[i][e] - mu) * rs * (float)g.v[e] + (float)b.v[e]);
      *reinterpret_cast<Pack<T, V>*>(yr + c) = o;
    }
  }
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}

/* LayerNorm backward.  Block = 4 waves, each wave walks rows (stride 4*gridDim.x); per row it forms dx
 * (plus the row of dres when given: the gradient that bypasses the normalisation on the residual path) and adds the row's contribution to its lanes' dgamma / dbeta accumulators; the four waves' sums meet
 * in LDS and go to part[block][2][n]; layernorm_bwd_final_kernel folds the blocks. */
template <typename T, int V, int NCH>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(int64_t rows, int n, const T* x, const T* gamma, const float* mean,
                                                            const float* rstd, const T* dy, const T* dres, T* dx, float* part) {
  __shared__ float red[4][64 * V * NCH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float dg[NCH][V], db[NCH][V];
  Pack<T, V> gm[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * 64 + lane) * V;
    if (c < n) gm[i] = *reinterpret_cast<const Pack<T, V>*>(gamma + c);
#pragma unroll
    for (int e = 0; e < V; ++e) { dg[i][e] = 0.0f; db[i][e] = 0.0f; if (c >= n) gm[i].v[e] = (T)0.0f; }
  }
  for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < rows; row += (int64_t)gridDim.x * 4) {
    const float mu = mean[row], rs = rstd[row];
    float xh[NCH][V], g[NCH][V];
    // Rows of up to 1024 elements fetch the residual path's gradient together with x and dy (one round trip to memory per
    // row instead of two: -12 %); wider rows would pay for the extra registers with occupancy (+25 % measured) and fetch it late.
    constexpr bool kEarly = NCH <= 2;
    Pack<T, V> res[kEarly ? NCH : 1];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = (i * 64 + lane) * V;
      Pack<T, V> px, pd;
      if (c < n) {
        px = *reinterpret_cast<const Pack<T, V>*>(x + row * n + c); pd = *reinterpret_cast<const Pack<T, V>*>(dy + row * n + c);
        if constexpr (kEarly) { if (dres) res[i] = *reinterpret_cast<const Pack<T, V>*>(dres + row * n + c); }
      }
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const float dv = c < n ? (float)pd.v[e] : 0.0f;
        xh[i][e] = c < n ? ((float)px.v[e] - mu) * rs : 0.0f;
        g[i][e] = dv * (float)gm[i].v[e];
        s1 += g[i][e];
        s2 += g[i][e] * xh[i][e];
        dg[i][e] += dv * xh[i][e];
        db[i][e] += dv;
      }
    }
    s1 = wave_sum(s1) / (float)n;
    s2 = wave_sum(s2) / (float)n;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = (i * 64 + lane) * V;
      if (c < n) {
        Pack<T, V> o, r;
        if constexpr (kEarly) r = res[i];
        else if (dres) r = *reinterpret_cast<const Pack<T, V>*>(dres + row * n + c);
#pragma unroll
        for (int e = 0; e < V; ++e) o.v[e] = (T)(rs * (g[i][e] - s1 - xh[i][e] * s2) + (dres ? (float)r.v[e] : 0.0f));
        *reinterpret_cast<Pack<T, V>*>(dx + row * n + c) = o;
      }
    }
  }
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
      for (int e = 0; e < V; ++e) red[wave][(i * 64 + lane) * V + e] = pass == 0 ? dg[i][e] : db[i][e];
    __syncthreads();
    for (int c = threadIdx.x; c < n; c += 256)
      part[((int64_t)blockIdx.x * 2 + pass) * n + c] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
  }
}

/* Folds layernorm_bwd partials: part[block][2][n] -> dgamma[n] (blockIdx.y = 0), dbeta[n] (1).  A block
 * owns 16 columns; its 16 thread groups walk the partial rows 16 apart and meet in LDS. */
__global__ __launch_bounds__(256) void layernorm_bwd_final_kernel(int n, int nblocks, const float* part, float* dgamma, float* dbeta) {
  __shared__ float red[16][17];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + tx;
  float a = 0.0f;
  if (c < n) {       // four independent partial sums keep four loads in flight per thread
    float a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    int p = ty;
    for (; p + 48 < nblocks; p += 64) {
      a += part[((int64_t)p * 2 + blockIdx.y) * n + c];
      a1 += part[((int64_t)(p + 16) * 2 + blockIdx.y) * n + c];
      a2 += part[((int64_t)(p + 32) * 2 + blockIdx.y) * n + c];
      a3 += part[((int64_t)(p + 48) * 2 + blockIdx.y) * n + c];
    }
    for (; p < nblocks; p += 16) a += part[((int64_t)p * 2 + blockIdx.y) * n + c];
    a = (a + a1) + (a2 + a3);
  }
  red[ty][tx] = a;
  __syncthreads();
  if (ty == 0 && c < n) {
    float t = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) t += red[r][tx];
    (blockIdx.y == 0 ? dgamma : dbeta)[c] = t;
  }
}

/* Register-resident MFMA loop: 8 independent 32x32x16 bf16 accumulators per wave, 8 waves per block,
 * one block per CU.  With `random` the operands are pseudo-random in [-1, 1) (switching activity of a
 * real GEMM, which lowers the sustained clock), else constants. */
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(512) void mfma_probe_kernel(float* out, int random, int iters) {
  probe_bf16x8 a[4], b[2];
  unsigned s = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
  for (int q = 0; q < 6; ++q)
    for (int i = 0; i < 8; ++i) {
      s = s * 1664525u + 1013904223u;
      const float v = random ? (float)((int)((s >> 8) % 2001u) - 1000) * 0.001f : 0.5f;
      if (q < 4) a[q][i] = (__bf16)v; else b[q - 4][i] = (__bf16)v;
    }
  probe_f32x16 c[8];
  for (int j = 0; j < 8; ++j)
    for (int e = 0; e < 16; ++e) c[j][e] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j / 2], b[j % 2], c[j], 0, 0, 0);
  }
  float t = 0.0f;
  for (int j = 0; j < 8; ++j)
    for (int e = 0; e < 16; ++e) t += c[j][e];
  out[blockIdx.x * 512 + threadIdx.x] = t;
}

inline int check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "%s launch: %s", what, hipGetErrorString(e));
  return HAP_OK;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p % 16) == 0; }

inline int grid_for(int64_t work_items) {
  int64_t g = (work_items + 255) / 256;
  if (g > 256 * 32) g = 256 * 32;   // grid-stride beyond 32 blocks per CU
  return g < 1 ? 1 : (int)g;
}

constexpr int kLnBlocks = 512;    // layernorm backward: blocks (= partial rows of dgamma/dbeta)
constexpr int kColsumRowsPerBlock = 128;

template <typename T>
int gelu_bwd_t(int groups, int64_t rows, int64_t cols, const void* pre, int64_t ldp, const void* dy, int64_t lddy, void* out, int64_t ldo,
               const int* group_len, hipStream_t s) {
  constexpr int V = 16 / sizeof(T);
  // 16-byte accesses need pitches of whole chunks and views that share one phase inside their chunks (any phase: a skewed view is
  // read and written through chunks aligned in the buffers' own address space)
  const uintptr_t ph = (uintptr_t)pre % 16;
  const bool vec = ldp % V == 0 && lddy % V == 0 && ldo % V == 0 && ph % sizeof(T) == 0 && (uintptr_t)dy % 16 == ph && (uintptr_t)out % 16 == ph &&
                   (groups == 1 || ph == 0 || (rows * ldp) % V == 0);
  const int skew = vec ? (int)(ph / sizeof(T)) : 0;
  const T* pre_a = (const T*)pre - skew; const T* dy_a = (const T*)dy - skew; T* out_a = (T*)out - skew;
  const unsigned gy = (unsigned)groups;
  if (vec && skew == 0 && cols % V == 0) hipLaunchKernelGGL((gelu_bwd_kernel<T, V, false>), dim3(grid_for(rows * (cols / V)), gy), dim3(256), 0, s, rows, cols, pre_a, ldp, dy_a, lddy, out_a, ldo, group_len, 0);
  else if (vec) hipLaunchKernelGGL((gelu_bwd_kernel<T, V, true>), dim3(grid_for(rows * ((cols + skew + V - 1) / V)), gy), dim3(256), 0, s, rows, cols, pre_a, ldp, dy_a, lddy, out_a, ldo, group_len, skew);
  else hipLaunchKernelGGL((gelu_bwd_kernel<T, 1, false>), dim3(grid_for(rows * cols), gy), dim3(256), 0, s, rows, cols, (const T*)pre, ldp, (const T*)dy, lddy, (T*)out, ldo, group_len, 0);
  return check_launch("gelu_bwd");
}

template <typename T>
int add_t(int64_t rows, int64_t cols, const void* a, int64_t lda, const void* b, int64_t ldb, const void* bias, void* out, int64_t ldo, hipStream_t s) {
  constexpr int V = 16 / sizeof(T);
  const bool vec = cols % V == 0 && lda % V == 0 && ldb % V == 0 && ldo % V == 0 && aligned16(a) && aligned16(b) && aligned16(out);
  if (vec && aligned16(bias)) hipLaunchKernelGGL((add_kernel<T, V, true>), dim3(grid_for(rows * (cols / V))), dim3(256), 0, s, rows, cols, (const T*)a, lda, (const T*)b, ldb, (const T*)bias, (T*)out, ldo);
  else if (vec) hipLaunchKernelGGL((add_kernel<T, V, false>), dim3(grid_for(rows * (cols / V))), dim3(256), 0, s, rows, cols, (const T*)a, lda, (const T*)b, ldb, (const T*)bias, (T*)out, ldo);
  else hipLaunchKernelGGL((add_kernel<T, 1, false>), dim3(grid_for(rows * cols)), dim3(256), 0, s, rows, cols, (const T*)a, lda, (const T*)b, ldb, (const T*)bias, (T*)out, ldo);
  return check_launch("add");
}

/* Picks the access width and chunk count: 16-byte chunks when the row length and the pointers allow. */
template <typename T, typename F>
bool ln_dispatch(int n, bool vec_ok, F&& launch) {
  constexpr int VV = 16 / sizeof(T);
  if (vec_ok && n % VV == 0) {
    const int chunks = (n / VV + 63) / 64;
    if (chunks <= 1) { launch(std::integral_constant<int, VV>(), std::integral_constant<int, 1>()); return true; }
    if (chunks <= 2) { launch(std::integral_constant<int, VV>(), std::integral_constant<int, 2>()); return true; }
    if (chunks <= 4) { launch(std::integral_constant<int, VV>(), std::integral_constant<int, 4>()); return true; }
    if (chunks <= 8) { launch(std::integral_constant<int, VV>(), std::integral_constant<int, 8>()); return true; }
  }
  const int chunks = (n + 63) / 64;
  if (chunks <= 4) { launch(std::integral_constant<int, 1>(), std::integral_constant<int, 4>()); return true; }
  if (chunks <= 16) { launch(std::integral_constant<int, 1>(), std::integral_constant<int, 16>()); return true; }
  if (chunks <= 32) { launch(std::integral_constant<int, 1>(), std::integral_constant<int, 32>()); return true; }
  return false;
}

template <typename T>
int layernorm_fwd_t(int64_t rows, int n, const void* x, const void* g, const void* b, void* y, float* mean, float* rstd, hipStream_t s) {
  const dim3 grid((unsigned)((rows + 3) / 4));
  const bool vec_ok = aligned16(x) && aligned16(y) && aligned16(g) && aligned16(b);
  const bool ok = ln_dispatch<T>(n, vec_ok, [&](auto v, auto nch) {
    hipLaunchKernelGGL((layernorm_fwd_kernel<T, decltype(v)::value, decltype(nch)::value>), grid, dim3(256), 0, s, rows, n, (const T*)x, (const T*)g,
                       (const T*)b, (T*)y, mean, rstd);
  });
  if (!ok) return hap_fail(HAP_EUNSUPPORTED, "layernorm row of %d elements is too long for this layout", n);
  return check_launch("layernorm_fwd");
}

template <typename T>
int layernorm_bwd_t(int64_t rows, int n, const void* x, const void* g, const float* mean, const float* rstd, const void* dy,
                    const void* dres, void* dx, float* dgamma, float* dbeta, float* part, hipStream_t s) {
  const int nblocks = (int)((rows + 3) / 4 < kLnBlocks ? (rows + 3) / 4 : kLnBlocks);
  const bool vec_ok = aligned16(x) && aligned16(dy) && aligned16(dx) && aligned16(g) && aligned16(dres);
  const bool ok = ln_dispatch<T>(n, vec_ok, [&](auto v, auto nch) {
    hipLaunchKernelGGL((layernorm_bwd_kernel<T, decltype(v)::value, decltype(nch)::value>), dim3(nblocks), dim3(256), 0, s, rows, n, (const T*)x,
                       (const T*)g, mean, rstd, (const T*)dy, (const T*)dres, (T*)dx, part);
  });
  if (!ok) return hap_fail(HAP_EUNSUPPORTED, "layernorm row of %d elements is too long for this layout", n);
  int rc = check_launch("layernorm_bwd");
  if (rc) return rc;
  hipLaunchKernelGGL(layernorm_bwd_final_kernel, dim3((n + 15) / 16, 2), dim3(256), 0, s, n, nblocks, part, dgamma, dbeta);
  return check_launch("layernorm_bwd_final");
}

}  // namespace

extern "C" {

int hap_probe_mfma_bf16(int random_operands, int iters, float* scratch, double* flops, void* stream) {
  hap_clear_error();
  if (!scratch || iters < 1) return hap_fail(HAP_EINVAL, "scratch is NULL or iters < 1");
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(256), dim3(512), 0, (hipStream_t)stream, scratch, random_operands, iters);
  if (flops) *flops = 2.0 * 32 * 32 * 16 * 8.0 * (double)iters * 8.0 * 256.0;
  return check_launch("mfma_probe");
}

int hap_device_info(int* compute_units, int* clock_khz) {
  hap_clear_error();
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hap_fail(HAP_EDEVICE, "cannot query the device");
  if (compute_units) *compute_units = prop.multiProcessorCount;
  if (clock_khz) *clock_khz = prop.clockRate;
  return HAP_OK;
}

int hap_gelu_bwd(int64_t rows, int64_t cols, int io_dtype, const void* preact, int64_t ldp, const void* dy,
                 int64_t lddy, void* out, int64_t ldo, void* stream) {
  hap_clear_error();
  return hap_gelu_bwd_grouped(1, rows, cols, io_dtype, preact, ldp, dy, lddy, out, ldo, NULL, stream);
}

int hap_gelu_bwd_grouped(int groups, int64_t rows, int64_t cols, int io_dtype, const void* preact, int64_t ldp, const void* dy,
                         int64_t lddy, void* out, int64_t ldo, const int32_t* group_len, void* stream) {
  if (rows < 0 || cols < 0 || groups < 0) return hap_fail(HAP_EINVAL, "negative size");
  if (groups > 65535) return hap_fail(HAP_EUNSUPPORTED, "more than 65535 groups");
  if (rows == 0 || cols == 0 || groups == 0) return HAP_OK;
  if (!preact || !dy || !out) return hap_fail(HAP_EINVAL, "NULL pointer");
  if (ldp < cols || lddy < cols || ldo < cols) return hap_fail(HAP_ESHAPE, "leading dimension below cols");
  hipStream_t s = (hipStream_t)stream;
  if (io_dtype == HAP_BF16) return gelu_bwd_t<__bf16>(groups, rows, cols, preact, ldp, dy, lddy, out, ldo, group_len, s);
  if (io_dtype == HAP_F32) return gelu_bwd_t<float>(groups, rows, cols, preact, ldp, dy, lddy, out, ldo, group_len, s);
  return hap_fail(HAP_EINVAL, "bad dtype %d", io_dtype);
}

int hap_add(int64_t rows, int64_t cols, int io_dtype, const void* a, int64_t lda, const void* b, int64_t ldb,
            const void* bias, void* out, int64_t ldo, void* stream) {
  hap_clear_error();
  if (rows < 0 || cols < 0) return hap_fail(HAP_EINVAL, "negative size");
  if (rows == 0 || cols == 0) return HAP_OK;
  if (!a || !b || !out) return hap_fail(HAP_EINVAL, "NULL pointer");
  if (lda < cols || ldb < cols || ldo < cols) return hap_fail(HAP_ESHAPE, "leading dimension below cols");
  hipStream_t s = (hipStream_t)stream;
  if (io_dtype == HAP_BF16) return add_t<__bf16>(rows, cols, a, lda, b, ldb, bias, out, ldo, s);
  if (io_dtype == HAP_F32) return add_t<float>(rows, cols, a, lda, b, ldb, bias, out, ldo, s);
  return hap_fail(HAP_EINVAL, "bad dtype %d", io_dtype);
}

size_t hap_colsum_workspace(int64_t rows, int64_t cols) {
  if (rows <= 0 || cols <= 0) return 0;
  const int64_t parts = (rows + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock;
  return (size_t)(parts * cols) * sizeof(float);
}

int hap_colsum(int64_t rows, int64_t cols, int io_dtype, const void* a, int64_t lda, float* out,
               void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  return hap_colsum_grouped(1, rows, cols, io_dtype, a, lda, 0, NULL, out, cols, ws, ws_bytes, stream);
}

size_t hap_colsum_grouped_workspace(int groups, int64_t rows, int64_t cols) {
  return (size_t)(groups > 1 ? groups : 1) * hap_colsum_workspace(rows, cols);
}

int hap_colsum_grouped(int groups, int64_t rows, int64_t cols, int io_dtype, const void* a, int64_t lda, int64_t group_stride,
                       const int32_t* group_len, float* out, int64_t ldo, void* ws, size_t ws_bytes, void* stream) {
  if (rows < 0 || cols < 0 || groups < 0) return hap_fail(HAP_EINVAL, "negative size");
  if (cols == 0 || groups == 0) return HAP_OK;
  if (groups > 65535) return hap_fail(HAP_EUNSUPPORTED, "more than 65535 groups");
  if (!out) return hap_fail(HAP_EINVAL, "NULL output");
  if (ldo < cols) return hap_fail(HAP_ESHAPE, "output stride below cols");
  hipStream_t s = (hipStream_t)stream;
  const dim3 fgrid((unsigned)((cols + 15) / 16), (unsigned)groups);
  if (rows == 0) {   // empty sums
    hipLaunchKernelGGL(colsum_final_kernel, fgrid, dim3(256), 0, s, cols, 0, (const float*)out, out, ldo);
    return check_launch("colsum");
  }
  if (!a) return hap_fail(HAP_EINVAL, "NULL input");
  if (lda < cols) return hap_fail(HAP_ESHAPE, "leading dimension below cols");
  if (io_dtype != HAP_BF16 && io_dtype != HAP_F32) return hap_fail(HAP_EINVAL, "bad dtype %d", io_dtype);
  const size_t need = hap_colsum_grouped_workspace(groups, rows, cols);
  if (!ws || ws_bytes < need) return hap_fail(HAP_EWORKSPACE, "colsum needs %zu workspace bytes", need);
  const int64_t parts = (rows + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock;
  if (parts > 65535) return hap_fail(HAP_EUNSUPPORTED, "colsum over more than 65535 * 128 rows");
  const int esz = io_dtype == HAP_BF16 ? 2 : 4, V = 16 / esz;
  const bool vec = (uintptr_t)a % esz == 0 && lda % V == 0 && (groups == 1 || group_stride % V == 0);
  const int skew = vec ? (int)(((uintptr_t)a % 16) / esz) : 0;
  const char* base = static_cast<const char*>(a) - (size_t)skew * esz;
  const int64_t per_block = vec ? 64 * V : 64;
  const dim3 grid((unsigned)((cols + skew + per_block - 1) / per_block), (unsigned)parts, (unsigned)groups);
  const int64_t rpb = kColsumRowsPerBlock;
  const int* gl = group_len;
  if (io_dtype == HAP_BF16) {
    if (vec) hipLaunchKernelGGL((colsum_partial_kernel<__bf16, 8>), grid, dim3(256), 0, s, rows, cols, (const __bf16*)base, lda, skew, rpb, (float*)ws, group_stride, gl);
    else hipLaunchKernelGGL((colsum_partial_kernel<__bf16, 1>), grid, dim3(256), 0, s, rows, cols, (const __bf16*)a, lda, 0, rpb, (float*)ws, group_stride, gl);
  } else {
    if (vec) hipLaunchKernelGGL((colsum_partial_kernel<float, 4>), grid, dim3(256), 0, s, rows, cols, (const float*)base, lda, skew, rpb, (float*)ws, group_stride, gl);
    else hipLaunchKernelGGL((colsum_partial_kernel<float, 1>), grid, dim3(256), 0, s, rows, cols, (const float*)a, lda, 0, rpb, (float*)ws, group_stride, gl);
  }
  int rc = check_launch("colsum_partial");
  if (rc) return rc;
  hipLaunchKernelGGL(colsum_final_kernel, fgrid, dim3(256), 0, s, cols, (int)parts, (const float*)ws, out, ldo);
  return check_launch("colsum_final");
}

int hap_layernorm_fwd(int64_t rows, int64_t n, int io_dtype, const void* x, const void* gamma, const void* beta,
                      void* y, float* mean, float* rstd, void* stream) {
  hap_clear_error();
  if (rows < 0 || n < 1) return hap_fail(HAP_EINVAL, "bad size");
  if (rows == 0) return HAP_OK;
  if (!x || !gamma || !beta || !y || !mean || !rstd) return hap_fail(HAP_EINVAL, "NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  if (io_dtype == HAP_BF16) return layernorm_fwd_t<__bf16>(rows, (int)n, x, gamma, beta, y, mean, rstd, s);
  if (io_dtype == HAP_F32) return layernorm_fwd_t<float>(rows, (int)n, x, gamma, beta, y, mean, rstd, s);
  return hap_fail(HAP_EINVAL, "bad dtype %d", io_dtype);
}

size_t hap_layernorm_bwd_workspace(int64_t rows, int64_t n) {
  if (rows <= 0 || n <= 0) return 0;
  const int64_t nblocks = (rows + 3) / 4 < kLnBlocks ? (rows + 3) / 4 : kLnBlocks;
  return (size_t)(nblocks * 2 * n) * sizeof(float);
}

int hap_layernorm_bwd(int64_t rows, int64_t n, int io_dtype, const void* x, const void* gamma, const float* mean,
                      const float* rstd, const void* dy, const void* dresidual, void* dx, float* dgamma, float* dbeta,
                      void* ws, size_t ws_bytes, void* stream) {
  hap_clear_error();
  if (rows < 0 || n < 1) return hap_fail(HAP_EINVAL, "bad size");
  if (rows == 0) {
    // A device whose batch shard is empty (B_j = 0 is feasible in Eq. (opt_B)) still contributes its partial parameter
    // gradients to the all-reduce: they are empty sums, written as zeros (the column-sum fold over zero partial rows).
    if (!dgamma || !dbeta) return hap_fail(HAP_EINVAL, "NULL pointer");
    const dim3 fgrid((unsigned)((n + 15) / 16), 1);
    hipLaunchKernelGGL(colsum_final_kernel, fgrid, dim3(256), 0, (hipStream_t)stream, n, 0, (const float*)dgamma, dgamma, n);
    hipLaunchKernelGGL(colsum_final_kernel, fgrid, dim3(256), 0, (hipStream_t)stream, n, 0, (const float*)dbeta, dbeta, n);
    return check_launch("layernorm_bwd (empty)");
  }
  if (!x || !gamma || !mean || !rstd || !dy || !dx || !dgamma || !dbeta) return hap_fail(HAP_EINVAL, "NULL pointer");
  const size_t need = hap_layernorm_bwd_workspace(rows, n);
  if (!ws || ws_bytes < need) return hap_fail(HAP_EWORKSPACE, "layernorm_bwd needs %zu workspace bytes", need);
  hipStream_t s = (hipStream_t)stream;
  if (io_dtype == HAP_BF16) return layernorm_bwd_t<__bf16>(rows, (int)n, x, gamma, mean, rstd, dy, dresidual, dx, dgamma, dbeta, (float*)ws, s);
  if (io_dtype == HAP_F32) return layernorm_bwd_t<float>(rows, (int)n, x, gamma, mean, rstd, dy, dresidual, dx, dgamma, dbeta, (float*)ws, s);
  return hap_fail(HAP_EINVAL, "bad dtype %d", io_dtype);
}

}  // extern "C"
