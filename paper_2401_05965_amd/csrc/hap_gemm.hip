/*
 * GEMM engine of libhap for gfx950 (CDNA4): bf16 / fp32 MFMA, LDS-tiled, ragged edges handled by
 * predication instead of padding the problem.
 *
 * Data movement.  A tile of each operand is fetched as 16-byte chunks with raw buffer loads
 * (an out-of-range chunk costs no memory access and reads as zero) and stored in LDS in the
 * operand's own contiguous direction:
 *   K-contiguous operand  -> LDS rows are m (or n), chunks run along k; MFMA fragments come from
 *                            one 128-bit LDS read per lane;
 *   M/N-contiguous operand-> LDS rows are k, chunks run along m (or n); fragments come from the
 *                            transposing LDS read of gfx950 (ds_read_b64_tr_b16), which hands each
 *                            lane 4 consecutive k of one column.
 * 16-byte chunks are XOR-swizzled inside a row so both kinds of fragment read are bank-conflict free.
 *
 * Raggedness.  Shard ranges start at arbitrary elements (e.g. column 13443 of a bf16 matrix), so the
 * launcher aligns every operand base DOWN to 16 bytes and passes the number of leading elements
 * (skew) that do not belong to the shard.  Leading / trailing elements along k are zeroed in
 * registers before they reach LDS; leading / trailing rows and columns of C are simply not stored.
 *
 * Kernels.  gemm_pp_kernel: bf16, 256 x 256 tiles, two wave groups that alternate a memory phase and a matrix phase over a
 * 4-stage ring of direct-to-LDS K tiles (all layouts but "both operands K-contiguous").  gemm_dma_kernel: bf16, two-stage ring,
 * 256 x 256 (both operands K-contiguous) and 128 x 128 (small outputs, remainder strips).  gemm_kernel: register-staged, fp32
 * and what the direct kernels cannot address.  gemm_skinny_f32_kernel: fp32 products of at most 64 rows, contraction split over
 * the waves of a workgroup.  gemm_generic_kernel: scalar fallback.  Epilogues: bias, GeLU, pre-activation copy, fp32
 * accumulation, or the product times gelu'(saved pre-activation) - the activation backward of the layer that produced the
 * output's tensor.
 */
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "hap_gemm.h"

namespace hap_gemm_detail {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

#if defined(HAP_GEMM_EXPERIMENT)
// (development harness only) wall-clock stamps of every workgroup: 0 start, 1 main loop start, 2 main loop end, 3 end, 4..7 after each
// 32-row block of the epilogue
__device__ unsigned long long hap_exp_stamps[8 * 2048];
#define HAP_EXP_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 2048) hap_exp_stamps[blockIdx.x * 8 + (i)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define HAP_EXP_STAMP(i) do { } while (0)
#endif


constexpr unsigned kOobOffset = 0x80000000u;  // beyond any num_records we pass: reads as zero
constexpr int64_t kViewLimitBytes = 2147483000;  // reach of the tiled kernels' 32-bit buffer offsets: operand views stay below it
constexpr int kRsrcFlags = 0x00020000;        // raw buffer, 32-bit data format

struct SegArg {
  const void* a;   // aligned-down base of this segment's A view
  const void* b;
  int k;           // logical contracted length of the segment
  unsigned a_bytes, b_bytes;  // valid extent from the aligned bases
  int pad;
};

struct GemmArgs {
  int M, N;            // logical extent of C
  int skewM, skewN;    // physical columns preceding logical 0 in an M-/N-contiguous operand; for a K-contiguous B, skewN rows of the
                       // tile grid precede its first row (the grid then sits on C's 16-byte chunks)
  int skewK;           // physical k preceding logical 0 in a K-contiguous operand
  int nseg;
  int tiles_m, tiles_n;
  int vec_store;       // C (and preact) rows are 16-byte addressable: whole-chunk stores allowed
  int cdelta;          // columns by which tile columns are shifted in the store patch so that its 16-byte chunks coincide with
                       // 16-byte chunks of C's address space (0 when C has the B operand's phase; see epilogue_transposed)
  int ksplit;          // >1: each output tile is computed by ksplit workgroups over disjoint K-tile ranges, fp32 partials go to `partial`
  float* partial;      // [group][tile][ksplit][BM][BN] fp32 workspace when ksplit > 1
  int ntiles;          // K tiles (of 64) over all segments
  long long lda, ldb, ldc, ldp;
  void* c;
  void* preact;
  const void* bias;
  int act, accumulate;
  const void* dact_preact;   // optional [M x N] in C's dtype, leading dimension ldd: C = (product + bias) * act'(dact_preact)
  long long ldd;
  // Grouped launch (gridDim.y groups): a workgroup works on one of `groups` independent products that differ only in their base
  // addresses (byte strides below) and, when group_len is given, in the valid length of one axis.
  int ragged;              // 0: every group is M x N x k;  1: group_len bounds M;  2: group_len bounds the contraction (nseg == 1)
  const int* group_len;    // device array [groups], or nullptr
  long long ga, gb, gc, gp, gbias, gd;
  SegArg seg[HAP_GEMM_MAX_SEG];
};

/* What the workgroup's group changes: valid rows, contracted length of the single segment (-1: as in
 * the segment table), byte offsets of the operands and outputs. */
struct GroupView {
  int M, k;
  long long oa, ob;
};

__device__ __forceinline__ GroupView group_view(const GemmArgs& args, int grp) {
  GroupView g;
  g.M = args.M; g.k = -1;
  g.oa = grp * args.ga; g.ob = grp * args.gb;
  if (args.ragged) {
    int len = __builtin_amdgcn_readfirstlane(args.group_len[grp]);
    len = len < 0 ? 0 : len;
    if (args.ragged == 1) g.M = len < args.M ? len : args.M;
    else g.k = len < args.seg[0].k ? len : args.seg[0].k;
  }
  return g;
}

/* The arguments as the epilogue of this workgroup's group sees them. */
__device__ __forceinline__ GemmArgs group_outputs(const GemmArgs& args, const GroupView& g, int grp) {
  GemmArgs e = args;
  e.M = g.M;
  e.c = static_cast<char*>(args.c) + grp * args.gc;
  if (args.preact) e.preact = static_cast<char*>(args.preact) + grp * args.gp;
  if (args.bias) e.bias = static_cast<const char*>(args.bias) + grp * args.gbias;
  if (args.dact_preact) e.dact_preact = static_cast<const char*>(args.dact_preact) + grp * args.gd;
  return e;
}

/* Compile-time loop: f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N-1>). */
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>());
    static_for<N, I + 1>(f);
  }
}

/* Values that are the same in every lane but that the compiler cannot prove uniform (they depend on
 * a table entry picked by a loop-carried index) are pinned to scalar registers; otherwise every
 * buffer instruction using them is wrapped in a per-lane "waterfall" loop. */
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const void* uni(const void* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const void*>(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(uni(base)), 0, uni((int)bytes), kRsrcFlags);
}

/* One wave-wide direct load: lane l's 16 bytes at (voff + soff) of the buffer land at lds + 16*l.
 * `lds` must be wave-uniform.  The host pass of hipcc has no such builtin, hence the guard. */
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, char* lds, unsigned voff, unsigned soff) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(void, lds), 16, voff, soff, 0, 0);
#else
  (void)rsrc; (void)lds; (void)voff; (void)soff;
#endif
}

/* erf by the rational-times-Gaussian form of Abramowitz & Stegun 7.1.26 (absolute error <= 1.5e-7, far
 * inside the fp32 and bf16 output tolerances): one reciprocal, one exponential and five multiply-adds
 * instead of the branchy library routine, because the epilogue evaluates it for every output element. */
__device__ __forceinline__ float erf_fast(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(ax * ax * -1.4426950408889634f);
  return copysignf(1.0f - p * t * e, x);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erf_fast(x * 0.70710678118654752f)); }
/* d gelu / dx = Phi(x) + x phi(x); exp(-x^2/2) serves both the erf approximation (its argument is x/sqrt 2) and phi */
__device__ __forceinline__ float gelu_erf_grad(float x) {
  const float ax = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(x * x * -0.7213475204444817f);
  const float half_erf = copysignf(fmaf(p * t, -0.5f * e, 0.5f), x);      // erf(x / sqrt 2) / 2
  return fmaf(x, 0.3989422804014327f * e, 0.5f + half_erf);
}

template <typename T> struct Elem;
template <> struct Elem<__bf16> {
  static constexpr int kStep = 16;  // k per MFMA (v_mfma_f32_32x32x16_bf16)
};
template <> struct Elem<float> {
  static constexpr int kStep = 2;   // v_mfma_f32_32x32x2_f32
};

/* Swizzled position of 16-byte chunk c in LDS row `row`.  The LDS of gfx950 serves 256 bytes per clock
 * (64 banks x 4 bytes): a 128-bit read is conflict free when every 16 consecutive lanes cover 16
 * different chunk positions modulo 256 bytes, a transposing 64-bit read when every 32 lanes do.
 *   K-contiguous tile: 16 lanes read the same logical chunk of 16 consecutive rows -> XOR the chunk
 *     index with the row's index inside its 256-byte group.
 *   M/N-contiguous tile (rows are 512 bytes or more): 32 lanes read 64 contiguous bytes of each of 4
 *     consecutive rows -> XOR bits 2..3 of the chunk index with row & 3.                              */
template <bool KC, int CPR>
__device__ __forceinline__ int swz(int row, int c) {
  if constexpr (KC) {
    constexpr int RPS = CPR >= 16 ? 1 : 16 / CPR;    // rows per 256-byte bank sweep
    constexpr int MASK = (CPR >= 16 ? 16 : CPR) - 1;
    return c ^ ((row / RPS) & MASK);
  } else {
    static_assert(CPR >= 8, "M/N-contiguous tiles need rows of at least 128 bytes");
    if constexpr (CPR >= 16) return c ^ ((row & 3) << 2);
    else return c ^ ((row & 3) << 1);
  }
}

template <typename T> __device__ __forceinline__ void store_c(T* p, float v);
template <> __device__ __forceinline__ void store_c<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_c<__bf16>(__bf16* p, float v) { *p = (__bf16)v; }
template <typename T> __device__ __forceinline__ float load_s(const T* p);
template <> __device__ __forceinline__ float load_s<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_s<__bf16>(const __bf16* p) { return (float)*p; }

/* Loads one operand tile's chunks owned by this thread into registers.
 * KC:  rows = ROWS (m or n), chunk c covers k in [c*EPC, (c+1)*EPC)
 * !KC: rows = BK (k), chunk c covers m (or n) in [c*EPC, ...)                                   */
template <typename T, bool KC, int ROWS, int BK, int NT>
struct TileLoader {
  static constexpr int ES = sizeof(T);
  static constexpr int EPC = 16 / ES;
  static constexpr int LROWS = KC ? ROWS : BK;
  static constexpr int CPR = (KC ? BK : ROWS) / EPC;
  static constexpr int CPT = LROWS * CPR / NT;
  static_assert(LROWS * CPR % NT == 0, "tile chunks must divide evenly over threads");

  i32x4_t regs[CPT];

  /* mn0: first physical row (KC) or column (!KC) of the tile in the MN direction.
   * mn_lim: physical MN extent.  k0: first physical k of the tile; kskew/kend: logical k range in
   * physical coordinates [kskew, kend).  ld in elements.                                        */
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, int tid, int mn0, int mn_lim, long long ld,
                                       int k0, int kskew, int kend) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int id = tid + i * NT;
      const int row = id / CPR, c = id % CPR;
      unsigned off;
      if constexpr (KC) {
        const int mn = mn0 + row, kp = k0 + c * EPC;
        const bool ok = mn < mn_lim && kp < kend && kp + EPC > kskew;
        off = ok ? (unsigned)(((long long)mn * ld + kp) * ES) : kOobOffset;
      } else {
        const int kl = k0 + row, mn = mn0 + c * EPC;
        const bool ok = kl >= kskew && kl < kend && mn < mn_lim;
        off = ok ? (unsigned)(((long long)(kl - kskew) * ld + mn) * ES) : kOobOffset;
      }
      regs[i] = __builtin_bit_cast(i32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
    }
  }

  /* Zeroes elements outside [kskew, kend) of K-contiguous chunks (needed on a segment's first and
   * last tile only; callers skip it elsewhere). */
  __device__ __forceinline__ void mask_k(int tid, int k0, int kskew, int kend) {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < CPT; ++i) {
        const int id = tid + i * NT;
        const int c = id % CPR;
        const int kp = k0 + c * EPC;
        if (kp < kskew || kp + EPC > kend) {
          T v[EPC];
          __builtin_memcpy(v, &regs[i], 16);
#pragma unroll
          for (int e = 0; e < EPC; ++e)
            if (kp + e < kskew || kp + e >= kend) v[e] = (T)0.0f;
          __builtin_memcpy(&regs[i], v, 16);
        }
      }
    }
  }

  __device__ __forceinline__ void store(char* lds, int tid) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int id = tid + i * NT;
      const int row = id / CPR, c = id % CPR;
      *reinterpret_cast<i32x4_t*>(lds + row * (CPR * 16) + swz<KC, CPR>(row, c) * 16) = regs[i];
    }
  }
};

/* MFMA operand fragment for a 32-row block starting at LDS row/column `mn` (multiple of 32) and
 * k-step kk of the tile. */
template <typename T, bool KC, int ROWS, int BK>
struct Frag;

template <bool KC, int ROWS, int BK>
struct Frag<__bf16, KC, ROWS, BK> {
  typedef bf16x8_t type;
  static constexpr int CPR = (KC ? BK : ROWS) / 8;
  static __device__ __forceinline__ type read(const char* lds, int mn, int kk, int lane) {
    if constexpr (KC) {
      const int row = mn + (lane & 31);
      const int c = kk * 2 + (lane >> 5);
      return __builtin_bit_cast(type, *reinterpret_cast<const i32x4_t*>(lds + row * (CPR * 16) + swz<true, CPR>(row, c) * 16));
    } else {
      const int g = lane >> 4, i = lane & 15;
      const int col = mn + (g & 1) * 16 + (i & 3) * 4;
      const int krow = kk * 16 + (g >> 1) * 8 + (i >> 2);
      const int c = col >> 3, sub = (col & 7) * 2;
      const char* p0 = lds + krow * (CPR * 16) + swz<false, CPR>(krow, c) * 16 + sub;
      const char* p1 = lds + (krow + 4) * (CPR * 16) + swz<false, CPR>(krow + 4, c) * 16 + sub;
      s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, p0));
      s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, p1));
      typedef short s16x8_t __attribute__((ext_vector_type(8)));
      s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(type, v);
    }
  }
};

/* The same two fragment fetches as FragReader::read, written as instructions of their own.  The compiler treats every
 * LDS read it knows about as possibly aliasing the direct-to-LDS loads in flight and waits for ALL of them (vmcnt 0)
 * in front of it, which would drain a ring of several tiles on every tile.  These reads are ordered by hand instead:
 * the kernel waits for the awaited tile's loads (vmcnt) and a barrier before it reads a slot, and for the LDS counter
 * before it uses the values.  `off` is a compile-time byte offset (below 65536). */
template <int OFF>
__device__ __forceinline__ bf16x8_t lds_read_b128_at(unsigned addr) {
  i32x4_t v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return __builtin_bit_cast(bf16x8_t, v);
}
template <int OFF_LO, int OFF_HI>
__device__ __forceinline__ bf16x8_t lds_read_tr_pair_at(unsigned addr) {
  typedef int i32x2_t __attribute__((ext_vector_type(2)));
  i32x2_t lo, hi;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(OFF_LO));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(OFF_HI));
  i32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8_t, v);
}

/* The same bf16 fragment fetch with the address arithmetic folded.  The swizzles are XORs, so the byte
 * address of the fragment of 32-row block i (rows wave_mn + 32 i ..) at k-step kk of a tile is
 *   K-contiguous:    ((lane constant + tile address) ^ (kk << 5)) + i * 32 rows
 *   M/N-contiguous:  (lane constant ^ (block index << 6)) + tile address + kk * 16 rows (+ 4 rows, second half)
 * and a wave keeps one register (K-contiguous) or one per block (M/N-contiguous) instead of an address
 * per fragment.  Tile addresses are multiples of 512 bytes. */
template <bool KC, int ROWS, int BK, int NBLK>
struct FragReader {
  static constexpr int CPR = (KC ? BK : ROWS) / 8;
  static constexpr int ROWB = CPR * 16;
  unsigned at[KC ? 1 : NBLK];
  __device__ __forceinline__ void init(int lane, int wave_mn) {
    if constexpr (KC) {
      const int r = lane & 31, h = lane >> 5;
      at[0] = (unsigned)((wave_mn + r) * ROWB + ((h ^ swz<true, CPR>(r, 0)) << 4));
    } else {
      static_assert(CPR >= 16, "M/N-contiguous fragment addressing assumes rows of 256 bytes or more");
      const int g = lane >> 4, i = lane & 15;
      const int x = i >> 2, cl = (g & 1) * 2 + ((i & 3) >> 1);
      const unsigned lc = (unsigned)(((g >> 1) * 8 + x) * ROWB + (x << 6) + (cl << 4) + (i & 1) * 8);
#pragma unroll
      for (int b = 0; b < NBLK; ++b) at[b] = lc ^ (unsigned)(((wave_mn >> 5) + b) << 6);
    }
  }
  /* read() with the hand-ordered LDS instructions (see lds_read_b128_at); BLK and KKI fold into the offset field. */
  template <int BLK, int KKI>
  __device__ __forceinline__ bf16x8_t read_unordered(unsigned tile) const {
    if constexpr (KC) return lds_read_b128_at<BLK * 32 * ROWB>((at[0] + tile) ^ (unsigned)(KKI << 5));
    else return lds_read_tr_pair_at<KKI * 16 * ROWB, KKI * 16 * ROWB + 4 * ROWB>(at[BLK] + tile);
  }
  __device__ __forceinline__ bf16x8_t read(unsigned tile, int blk, int kk) const {
    if constexpr (KC) {
      const unsigned addr = ((at[0] + tile) ^ (unsigned)(kk << 5)) + (unsigned)(blk * 32 * ROWB);
      return __builtin_bit_cast(bf16x8_t, *(LDS_PTR(const i32x4_t, (unsigned long)addr)));
    } else {
      const unsigned addr = at[blk] + tile + (unsigned)(kk * 16 * ROWB);
      s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, (unsigned long)addr));
      s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, (unsigned long)(addr + 4 * ROWB)));
      typedef short s16x8_t __attribute__((ext_vector_type(8)));
      s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, v);
    }
  }
};

__device__ __forceinline__ unsigned lds_addr(const void* p) { return (unsigned)(unsigned long)LDS_PTR(const char, p); }

template <bool KC, int ROWS, int BK>
struct Frag<float, KC, ROWS, BK> {
  typedef float type;
  static constexpr int CPR = (KC ? BK : ROWS) / 4;
  static __device__ __forceinline__ type read(const char* lds, int mn, int kk, int lane) {
    if constexpr (KC) {
      const int row = mn + (lane & 31);
      const int k = kk * 2 + (lane >> 5);
      return *reinterpret_cast<const float*>(lds + row * (CPR * 16) + swz<true, CPR>(row, k >> 2) * 16 + (k & 3) * 4);
    } else {
      const int krow = kk * 2 + (lane >> 5);
      const int col = mn + (lane & 31);
      return *reinterpret_cast<const float*>(lds + krow * (CPR * 16) + swz<false, CPR>(krow, col >> 2) * 16 + (col & 3) * 4);
    }
  }
};

__device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16_t mfma(float a, float b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

/* Workgroup id -> tile, keeping the workgroups that share an XCD (ids congruent mod 8 are
 * dispatched to the same die and L2) on a compact block of the tile grid. */
__device__ __forceinline__ int xcd_logical(int bid, int nblocks) {
  constexpr int XCDS = 8;
  const int xcd = bid % XCDS, local = bid / XCDS;
  const int q = nblocks / XCDS, r = nblocks % XCDS;
  return xcd * q + (xcd < r ? xcd : r) + local;
}

__device__ __forceinline__ void tile_of_logical(int logical, int tiles_m, int tiles_n, int* tm, int* tn) {
  constexpr int GM = 4;
  const int per_group = GM * tiles_n;
  const int group = logical / per_group, in_group = logical % per_group;
  const int first_m = group * GM;
  const int gsize = tiles_m - first_m < GM ? tiles_m - first_m : GM;
  *tm = first_m + in_group % gsize;
  *tn = in_group / gsize;
}

__device__ __forceinline__ void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n, int* tm, int* tn) {
  tile_of_logical(xcd_logical(bid, nblocks), tiles_m, tiles_n, tm, tn);
}

/* Which group, output tile and K split a workgroup of the tiled kernels works on.  A single product keeps
 * the map above.  In a grouped launch (gridDim.y groups of gridDim.x workgroups, dispatched x-fastest)
 * the XCD-contiguous renumbering runs over ALL workgroups, so an XCD works through whole groups one
 * after the other (a group's tiles share its operands in that XCD's L2) and every XCD gets the same
 * number of workgroups whatever the group count. */
struct BlockPos { int grp, out_tile, split, tm, tn; };
__device__ __forceinline__ BlockPos block_pos(const GemmArgs& args) {
  BlockPos b;
  const int ksplit = args.ksplit;
  if (gridDim.y == 1) {
    b.grp = 0;
    b.out_tile = blockIdx.x / ksplit; b.split = blockIdx.x - b.out_tile * ksplit;
    tile_of_block(b.out_tile, gridDim.x / ksplit, args.tiles_m, args.tiles_n, &b.tm, &b.tn);
  } else {
    const int logical = xcd_logical(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
    b.grp = logical / (int)gridDim.x;
    const int in_group = logical - b.grp * (int)gridDim.x;
    b.out_tile = in_group / ksplit; b.split = in_group - b.out_tile * ksplit;
    tile_of_logical(b.out_tile, args.tiles_m, args.tiles_n, &b.tm, &b.tn);
  }
  return b;
}

/* Writes a wave's TM x TN accumulator tiles.  Accumulator element e of lane l is row
 * (e/4)*8 + (l/32)*4 + e%4, column l%32 of its 32x32 tile.  (row0, col0): physical origin of the
 * wave tile; rows / columns outside the logical extent are dropped. */
template <typename T, typename TC, int TM, int TN>
__device__ __forceinline__ void epilogue(const GemmArgs& args, f32x16_t (&acc)[TM][TN], int row0, int col0, int lane) {
  TC* C = static_cast<TC*>(args.c);
  TC* P = static_cast<TC*>(args.preact);
  const T* bias = static_cast<const T*>(args.bias);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = col0 + j * 32 + (lane & 31) - args.skewN;
    const bool n_ok = n >= 0 && n < args.N;
    const float bv = (bias && n_ok) ? load_s<T>(bias + n) : 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = row0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3) - args.skewM;
        if (n_ok && m >= 0 && m < args.M) {
          float v = acc[i][j][e] + bv;
          if (P) store_c<TC>(P + (long long)m * args.ldp + n, v);
          if (args.act == HAP_ACT_GELU_ERF) v = gelu_erf((float)(TC)v);     // the activation sees the value as stored
          if (args.dact_preact) v *= gelu_erf_grad(load_s<TC>(static_cast<const TC*>(args.dact_preact) + (long long)m * args.ldd + n));
          TC* dst = C + (long long)m * args.ldc + n;
          if (args.accumulate) v += load_s<TC>(dst);
          store_c<TC>(dst, v);
        }
      }
    }
  }
}

template <typename T, typename TC, bool AKC, bool BKC, int BM, int BN, int BK, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(const GemmArgs args) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int ES = sizeof(T);
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int KSTEP = Elem<T>::kStep;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % KSTEP == 0, "tile shape");

  __shared__ __attribute__((aligned(16))) char lds_a[BM * BK * ES];
  __shared__ __attribute__((aligned(16))) char lds_b[BN * BK * ES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WGN) * WTM, wn0 = (wave % WGN) * WTN;
  // With split-K, ksplit consecutive workgroups share an output tile and take consecutive K-tile ranges.
  const BlockPos bp = block_pos(args);
  const int ksplit = args.ksplit, out_tile = bp.out_tile, split = bp.split, tm = bp.tm, tn = bp.tn;
  const int m0 = tm * BM, n0 = tn * BN;                 // physical tile origin
  const GroupView gv = group_view(args, bp.grp);
  const int m_lim = args.skewM + gv.M, n_lim = args.skewN + args.N;
  if (args.ragged == 1 && (gv.M == 0 || m0 >= m_lim)) return;   // the group's rows end before this tile
  const int all_tiles = gv.k >= 0 ? (args.skewK + gv.k + BK - 1 >= BK ? (args.skewK + gv.k + BK - 1) / BK : 1) : args.ntiles;

  TileLoader<T, AKC, BM, BK, NT> la;
  TileLoader<T, BKC, BN, BK, NT> lb;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // this workgroup's range [first, first + ntiles) of the K tiles of all segments laid end to end
  const int first = (int)((long long)all_tiles * split / ksplit);
  int ntiles = (int)((long long)all_tiles * (split + 1) / ksplit) - first;
  int seg = 0, skip = first;
  while (seg + 1 < args.nseg) {
    const int in_seg = (args.skewK + args.seg[seg].k + BK - 1) / BK;
    if (skip < in_seg) break;
    skip -= in_seg;
    seg = uni(seg + 1);
  }
  // loader state runs one tile ahead of the compute
  int k0 = skip * BK;
  int kend = uni(args.skewK + (gv.k >= 0 ? gv.k : args.seg[seg].k));
  __amdgpu_buffer_rsrc_t ra = make_rsrc(static_cast<const char*>(args.seg[seg].a) + gv.oa, args.seg[seg].a_bytes);
  __amdgpu_buffer_rsrc_t rb = make_rsrc(static_cast<const char*>(args.seg[seg].b) + gv.ob, args.seg[seg].b_bytes);

  auto fetch = [&]() {
    la.load(ra, tid, m0, m_lim, args.lda, k0, args.skewK, kend);
    lb.load(rb, tid, n0, n_lim, args.ldb, k0, args.skewK, kend);
  };
  auto commit = [&](int ck0, int ckend) {
    if (ck0 < args.skewK || ck0 + BK > ckend) {
      la.mask_k(tid, ck0, args.skewK, ckend);
      lb.mask_k(tid, ck0, args.skewK, ckend);
    }
    la.store(lds_a, tid);
    lb.store(lds_b, tid);
  };

  if (ntiles > 0) fetch();
  while (ntiles > 0) {     // (a split's share of a contraction shortened on the device side can be empty)
    const int ck0 = k0, ckend = kend;
    // advance the loader to the next tile
    k0 += BK;
    bool more = --ntiles > 0;
    if (more && k0 >= kend) {
      ++seg;
      if (seg < args.nseg) {
        k0 = 0;
        seg = uni(seg);
        kend = uni(args.skewK + args.seg[seg].k);
        ra = make_rsrc(static_cast<const char*>(args.seg[seg].a) + gv.oa, args.seg[seg].a_bytes);
        rb = make_rsrc(static_cast<const char*>(args.seg[seg].b) + gv.ob, args.seg[seg].b_bytes);
      } else {
        more = false;
      }
    }
    commit(ck0, ckend);
    __syncthreads();
    if (more) fetch();
#pragma unroll
    for (int kk = 0; kk < BK / KSTEP; ++kk) {
      typename Frag<T, AKC, BM, BK>::type fa[TM];
      typename Frag<T, BKC, BN, BK>::type fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = Frag<T, AKC, BM, BK>::read(lds_a, wm0 + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = Frag<T, BKC, BN, BK>::read(lds_b, wn0 + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma(fa[i], fb[j], acc[i][j]);
    }
    if (!more) break;
    __syncthreads();
  }

  if (ksplit > 1) {
    // raw fp32 partial tile [BM][BN]; bias, activation and the real store happen in the reduction kernel
    GemmArgs pa = args;
    pa.c = args.partial + (((long long)bp.grp * (gridDim.x / ksplit) + out_tile) * ksplit + split) * (BM * BN);
    pa.ldc = BN; pa.M = BM; pa.N = BN; pa.skewM = 0; pa.skewN = 0;
    pa.preact = nullptr; pa.bias = nullptr; pa.act = HAP_ACT_NONE; pa.accumulate = 0; pa.vec_store = 1; pa.cdelta = 0; pa.dact_preact = nullptr;
    epilogue<T, float, TM, TN>(pa, acc, wm0, wn0, lane);
    return;
  }
  epilogue<T, TC, TM, TN>(group_outputs(args, gv, bp.grp), acc, m0 + wm0, n0 + wn0, lane);
}

/* Epilogue of the direct-to-LDS kernels.  Their accumulators are TRANSPOSED tiles (the MFMA is fed
 * B-fragment first), so element e of lane l belongs to output row l%32 and columns
 * (e/4)*8 + (l/32)*4 + e%4: four consecutive columns per register quad.  Each wave passes one
 * 32-row block at a time through a private LDS patch and writes it out as whole 16-byte chunks,
 * eight (bf16) or four (fp32) lanes per 128-byte line, instead of 2-byte scattered stores.
 * Bias, activation, the optional pre-activation copy and fp32 accumulation are applied on the way.
 * Falls back to element stores where the destination is not 16-byte addressable or at ragged ends. */
template <typename TC> struct Vec16;
template <> struct Vec16<__bf16> { typedef __bf16 type __attribute__((ext_vector_type(8))); };
template <> struct Vec16<float> { typedef float type __attribute__((ext_vector_type(4))); };

/* MODE 0: bias, optional pre-activation copy (a pass of its own), optional accumulation; no activation.
 * MODE 1 (DACT): the product times act'(dact_preact); no bias, activation, copy or accumulation (the host sees to that).
 * MODE 2 (ACTP): activation, with the optional pre-activation copy in the SAME pass through the patch: the pre-activation chunk is
 *         stored as it comes out of the patch and the activation is applied to those same, already rounded values,
 *         H = act(round(P)) - what a framework computes that stores P and then applies the activation to the stored tensor, and
 *         the point at which the backward evaluates act'.  Every epilogue of the engine rounds before the activation, with or
 *         without a copy, so a layer's output does not depend on whether its pre-activation is kept. */
template <typename T, typename TC, int TM, int TN, bool SHIFTED, int MODE>
__device__ __forceinline__ void epilogue_transposed_impl(const GemmArgs& args, f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, char* patch) {
  constexpr bool DACT = MODE == 1, ACTP = MODE == 2;
  constexpr int ES = sizeof(TC);
  constexpr int EPC = 16 / ES;
  constexpr int COLS = TN * 32;
  constexpr int ROWB = COLS * ES + 16;            // padded row of the LDS patch
  constexpr int CH = COLS * ES / 16;              // 16-byte chunks per row
  typedef typename Vec16<TC>::type vec_t;
  TC* C = static_cast<TC*>(args.c);
  TC* P = static_cast<TC*>(args.preact);
  const T* bias = static_cast<const T*>(args.bias);
  const int h = lane >> 5, ml = lane & 31;
  const bool vec_ok = args.vec_store != 0;
  // A shard's columns start anywhere (column 8402 of a bf16 matrix is byte 16804), so C's 16-byte chunks need not coincide with the
  // tile's: the tile is written into the patch `delta` columns to the right (the row padding takes the overflow), which makes patch
  // chunk c the destination chunk that starts at tile column c * EPC - delta; only row ends are then stored element by element.
  const int delta = SHIFTED ? args.cdelta : 0;
  constexpr int nchunks = SHIFTED ? CH + 1 : CH;
  // this lane's bias values: the same 4 consecutive columns of every 8-column group, for all row blocks and passes
  // (DACT: the host admits no bias either, which frees these registers for the pre-activation chunks below)
  float bv[DACT ? 1 : TN][4][4];
  if constexpr (!DACT) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const int n = col0 + j * 32 + g * 8 + h * 4 + x - args.skewN;
          bv[j][g][x] = (bias && n >= 0 && n < args.N) ? load_s<T>(bias + n) : 0.0f;
        }
  }
  constexpr int ITS = (32 * nchunks + 63) / 64;          // 16-byte chunks of one 32-row block per lane
  // (row, column, valid part) of the chunk this lane stores in iteration `it` of row block i
  auto chunk_at = [&](int i, int it, int* m, int* n, int* t_lo, int* t_hi) -> bool {
    const int idx = it * 64 + lane;
    const int r = idx / nchunks, c = idx % nchunks;
    *m = row0 + i * 32 + r - args.skewM;
    *n = col0 + c * EPC - delta - args.skewN;
    // (a patch chunk also ends where the tile's columns end: what lies beyond was not written in this pass)
    *t_lo = c * EPC - delta < 0 ? delta - c * EPC : 0;
    *t_hi = c * EPC - delta + EPC > COLS ? COLS - (c * EPC - delta) : EPC;
    return (!SHIFTED || idx < 32 * nchunks) && *m >= 0 && *m < args.M && *n + *t_lo < args.N && *n + *t_hi > 0;
  };
  // DACT: all pre-activation chunks of the wave's tile are requested now, in one burst, so that the stores below wait for one
  // memory round trip instead of one per chunk
  // (an fp32 tile has twice the chunks: there the requests go out one row block at a time, ahead of that block's patch traffic)
  constexpr int BURST = !DACT ? 0 : ES == 2 ? TM : 1;
  vec_t pvs[DACT ? BURST : 1][DACT ? ITS : 1];
  auto request_preact = [&](int i, int slot) {
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      int m, n, t_lo, t_hi;
      // (a chunk that this wave stores only part of - its other columns belong to the neighbouring wave's tile - is still read whole)
      if (chunk_at(i, it, &m, &n, &t_lo, &t_hi) && vec_ok && n >= 0 && n + EPC <= args.N)
        pvs[slot][it] = *reinterpret_cast<const vec_t*>(static_cast<const TC*>(args.dact_preact) + (long long)m * args.ldd + n);
    }
  };
  if constexpr (BURST == TM) {
#pragma unroll
    for (int i = 0; i < TM; ++i) request_preact(i, i);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if (pass == 0 && (DACT || ACTP || !P)) continue;
      if constexpr (BURST == 1) request_preact(i, 0);
      TC* dst_base = pass == 0 ? P : C;
      const long long ldd = pass == 0 ? args.ldp : args.ldc;
      // registers -> LDS patch [32 rows][COLS]
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int cl = j * 32 + g * 8 + h * 4;            // first of 4 consecutive columns
          TC v[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            float f = acc[i][j][g * 4 + x];
            if constexpr (!DACT) f += bv[j][g][x];
            v[x] = (TC)f;
          }
          if constexpr (!SHIFTED) {
            __builtin_memcpy(patch + ml * ROWB + cl * ES, v, 4 * ES);
          } else {
            TC* q = reinterpret_cast<TC*>(patch + ml * ROWB) + cl + delta;
#pragma unroll
            for (int x = 0; x < 4; ++x) q[x] = v[x];
          }
        }
      // Order the patch accesses of this wave only: LDS operations of a wave execute in order, so a
      // wait on the LDS counter is enough (a fence would also drain the global stores in flight).
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_wave_barrier();
      // LDS patch -> global, 16 bytes per lane.  (An fp32 tile has eight iterations per block; all of them in flight at once, each
      // with its chunk, its address and - when accumulating - the old chunk, overflowed the registers the accumulators leave.)
      constexpr int kStoreUnroll = (ES == 4 && !DACT) ? 2 : ITS;
#pragma unroll kStoreUnroll
      for (int it = 0; it < ITS; ++it) {
        int m, n, t_lo, t_hi;
        if (!chunk_at(i, it, &m, &n, &t_lo, &t_hi)) continue;
        const int idx = it * 64 + lane;
        const int r = idx / nchunks, c = idx % nchunks;
        vec_t val = *reinterpret_cast<const vec_t*>(patch + r * ROWB + c * 16);
        TC* dst = dst_base + (long long)m * ldd + n;
        const TC* dpre = DACT ? static_cast<const TC*>(args.dact_preact) + (long long)m * args.ldd + n : nullptr;
        // (vec_ok implies that dact_preact shares C's 16-byte phase and pitch rule.)  The multiplication is done once, for whole
        // chunks, before the lanes part into chunk stores and element stores; elements of a partly stored chunk that lie outside
        // this wave's columns hold patch leftovers and are dropped below.
        const bool pv_ok = DACT && vec_ok && n >= 0 && n + EPC <= args.N;
        if constexpr (DACT) {
          if (pv_ok) {
            const vec_t pv = pvs[BURST == TM ? i : 0][it];
#pragma unroll
            for (int x = 0; x < EPC; ++x) val[x] = (TC)((float)val[x] * gelu_erf_grad((float)pv[x]));
          }
        }
        // ACTP: keep the pre-activation chunk, apply the activation to the whole chunk once (leftover elements are dropped below)
        vec_t pre = val;
        TC* pdst = ACTP ? P + (long long)m * args.ldp + n : nullptr;
        if constexpr (ACTP) {
#pragma unroll
          for (int x = 0; x < EPC; ++x) val[x] = (TC)gelu_erf((float)val[x]);
        }
        if (vec_ok && n >= 0 && n + EPC <= args.N && t_lo == 0 && t_hi == EPC) {
          if constexpr (ACTP) { if (P) *reinterpret_cast<vec_t*>(pdst) = pre; }
          if (!DACT && pass == 1 && args.accumulate) {
            const vec_t old = *reinterpret_cast<const vec_t*>(dst);
#pragma unroll
            for (int x = 0; x < EPC; ++x) val[x] = (TC)((float)val[x] + (float)old[x]);
          }
          *reinterpret_cast<vec_t*>(dst) = val;
        } else {
          // Rare (a chunk cut by a row end or by the wave's strip, or a destination that is not 16-byte addressable): element by
          // element, straight from the patch, as a real loop - unrolled eight-fold into every iteration above it made the epilogue
          // several times the size of the instruction cache, and the waves waited for code, not for data.
          // (read through an LDS-space pointer: a generic one makes the load a flat instruction, which counts on the memory
          // counter as well and makes every later wait for patch data a wait for the global stores in flight)
          const unsigned pe = lds_addr(patch + r * ROWB + c * 16);
#pragma unroll 1
          for (int x = t_lo; x < t_hi; ++x) {
            if (n + x < 0 || n + x >= args.N) continue;
            float f = (float)*LDS_PTR(const TC, (unsigned long)(pe + x * ES));
            if constexpr (ACTP) { if (P) store_c<TC>(pdst + x, f); f = gelu_erf(f); }
            if constexpr (DACT) f = (float)(TC)f * gelu_erf_grad(load_s<TC>(dpre + x));
            if (!DACT && pass == 1 && args.accumulate) f += load_s<TC>(dst + x);
            store_c<TC>(dst + x, f);
          }
        }
      }
      // Order the patch accesses of this wave only: LDS operations of a wave execute in order, so a
      // wait on the LDS counter is enough (a fence would also drain the global stores in flight).
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_wave_barrier();
    }
    HAP_EXP_STAMP(4 + (i & 3));
  }
}

template <typename T, typename TC, int TM, int TN>
__device__ __forceinline__ void epilogue_transposed(const GemmArgs& args, f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, char* patch) {
  if (args.dact_preact) {
    if (args.cdelta) epilogue_transposed_impl<T, TC, TM, TN, true, 1>(args, acc, row0, col0, lane, patch);
    else epilogue_transposed_impl<T, TC, TM, TN, false, 1>(args, acc, row0, col0, lane, patch);
  } else if (args.act == HAP_ACT_GELU_ERF) {
    if (args.cdelta) epilogue_transposed_impl<T, TC, TM, TN, true, 2>(args, acc, row0, col0, lane, patch);
    else epilogue_transposed_impl<T, TC, TM, TN, false, 2>(args, acc, row0, col0, lane, patch);
  } else if (args.cdelta) epilogue_transposed_impl<T, TC, TM, TN, true, 0>(args, acc, row0, col0, lane, patch);
  else epilogue_transposed_impl<T, TC, TM, TN, false, 0>(args, acc, row0, col0, lane, patch);
}

/* ---------------------------------------------------------------------------------------------
 * bf16 main kernel: global -> LDS by buffer loads that write LDS directly (no register staging),
 * STAGES-deep ring of tiles, one barrier per tile.
 *
 * A wave-wide direct load writes 64 lanes x 16 bytes to CONSECUTIVE LDS bytes, so the XOR swizzle is
 * applied on the global side: the lane that fills LDS chunk position p of a row fetches the chunk
 * whose swizzled position is p.  Interior tiles use precomputed per-lane offsets plus one scalar
 * offset per tile; the first / last tile of a segment recompute validity per chunk and, for
 * K-contiguous operands, zero the elements outside the logical k range in LDS once the data landed.
 * ------------------------------------------------------------------------------------------- */
template <bool KC, int ROWS, int BK, int NT>
struct DmaLoader {
  static constexpr int EPC = 8;
  static constexpr int LROWS = KC ? ROWS : BK;
  static constexpr int CPR = (KC ? BK : ROWS) / EPC;
  static constexpr int CPT = LROWS * CPR / NT;
  static constexpr int TILE_BYTES = ROWS * BK * 2;
  static_assert(LROWS * CPR % NT == 0, "tile chunks must divide evenly over threads");

  unsigned base[CPT];   // byte offset of this lane's chunk for k0 = 0, or the out-of-range marker

  /* LDS position id -> (row, logical chunk) */
  static __device__ __forceinline__ void where(int id, int* row, int* c) {
    *row = id / CPR;
    *c = swz<KC, CPR>(*row, id % CPR);
  }

  /* mn0: the tile's first physical row / column; [mn_lo, mn_lim): the physical range that holds the operand's logical rows /
   * columns.  A K-contiguous operand's rows may be placed mn_lo rows into the tile grid (so that the OUTPUT's columns fall on
   * its 16-byte chunks): grid rows below mn_lo do not exist and read as zero.  mn_lo is 0 for an M-/N-contiguous operand,
   * whose skew is part of its aligned-down base address. */
  __device__ __forceinline__ void init(int tid, int mn0, int mn_lo, int mn_lim, long long ld) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      int row, c;
      where(tid + i * NT, &row, &c);
      if constexpr (KC) {
        const int mn = mn0 + row;
        base[i] = (mn >= mn_lo && mn < mn_lim) ? (unsigned)(((long long)(mn - mn_lo) * ld + c * EPC) * 2) : kOobOffset;
      } else {
        const int mn = mn0 + c * EPC;
        base[i] = mn < mn_lim ? (unsigned)(((long long)row * ld + mn) * 2) : kOobOffset;
      }
    }
  }

  /* Byte offset of a tile starting at physical k0: k0 elements along a row (KC) or (k0 - kskew) rows. */
  static __device__ __forceinline__ unsigned tile_offset(int k0, int kskew, long long ld) {
    if constexpr (KC) return (unsigned)k0 * 2u;
    else return (unsigned)((long long)(k0 - kskew) * ld * 2);
  }

  /* Interior tile: every k of the tile is inside the logical range; soff = tile_offset() >= 0 goes in
   * the instruction's scalar offset. */
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, char* lds, int tid, unsigned soff) const {
    const int wave_first = uni(tid & ~63);      // pinned to a scalar register: it feeds M0, the LDS address of the direct load
#pragma unroll
    for (int i = 0; i < CPT; ++i) dma16(rsrc, lds + (wave_first + i * NT) * 16, base[i], soff);
  }

  /* The loads i of an interior tile with i % nparts == part.  A tile's loads are spread between the
   * MFMA groups of the previous tile: issued back to back they fill the memory queue and the wave
   * blocks on it instead of feeding the matrix unit.  `part` and `nparts` fold at compile time. */
  __device__ __forceinline__ void issue_part(__amdgpu_buffer_rsrc_t rsrc, char* lds, int tid, unsigned soff, int part, int nparts) const {
    const int wave_first = (tid & ~63);
#pragma unroll
    for (int i = 0; i < CPT; ++i)
      if (i % nparts == part) dma16(rsrc, lds + (wave_first + i * NT) * 16, base[i], soff);
  }

  /* Edge tile: validity along k decided per chunk; the tile offset (which may be "negative" for the
   * rows a skewed first tile does not use) is added per lane so valid chunks get an exact offset. */
  __device__ __forceinline__ void issue_edge(__amdgpu_buffer_rsrc_t rsrc, char* lds, int tid, unsigned toff, int k0, int kskew, int kend) const {
    const int wave_first = (tid & ~63);
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      int row, c;
      where(tid + i * NT, &row, &c);
      bool ok;
      if constexpr (KC) { const int kp = k0 + c * EPC; ok = kp < kend && kp + EPC > kskew; }
      else { const int kl = k0 + row; ok = kl >= kskew && kl < kend; }
      ok = ok && base[i] != kOobOffset;
      dma16(rsrc, lds + (wave_first + i * NT) * 16, ok ? base[i] + toff : kOobOffset, 0);
    }
  }

  /* After the edge tile landed: zero elements outside [kskew, kend) in this thread's own chunks. */
  __device__ __forceinline__ void fixup(char* lds, int tid, int k0, int kskew, int kend) const {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < CPT; ++i) {
        int row, c;
        where(tid + i * NT, &row, &c);
        const int kp = k0 + c * EPC;
        if (kp < kend && kp + EPC > kskew && (kp < kskew || kp + EPC > kend)) {
          i32x4_t* q = reinterpret_cast<i32x4_t*>(lds + (tid + i * NT) * 16);
          bf16x8_t v = __builtin_bit_cast(bf16x8_t, *q);
#pragma unroll
          for (int e = 0; e < EPC; ++e)
            if (kp + e < kskew || kp + e >= kend) v[e] = (__bf16)0.0f;
          *q = __builtin_bit_cast(i32x4_t, v);
        }
      }
    }
  }
};

template <typename TC, bool AKC, bool BKC, int BM, int BN, int BK, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN <= 4 ? 2 : 1))   /* the 4-wave kernel is built to share a compute unit with a second workgroup: two waves per SIMD */ void gemm_dma_kernel(const GemmArgs args) {
  typedef __bf16 T;
  constexpr int NT = 64 * WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  typedef DmaLoader<AKC, BM, BK, NT> LA;
  typedef DmaLoader<BKC, BN, BK, NT> LB;
  constexpr int LOADS_PER_TILE = LA::CPT + LB::CPT;

  extern __shared__ __attribute__((aligned(1024))) char smem[];   // FragReader needs tile addresses that are multiples of 512

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WGN) * WTM, wn0 = (wave % WGN) * WTN;
  // With split-K, ksplit consecutive workgroups share an output tile and take consecutive K-tile ranges.
  const BlockPos bp = block_pos(args);
  const int ksplit = args.ksplit, out_tile = bp.out_tile, split = bp.split, tm = bp.tm, tn = bp.tn;
  const int m0 = tm * BM, n0 = tn * BN;
  const GroupView gv = group_view(args, bp.grp);
  const int m_lim = args.skewM + gv.M, n_lim = args.skewN + args.N;
  if (args.ragged == 1 && (gv.M == 0 || m0 >= m_lim)) return;   // the group's rows end before this tile
  const int all_tiles = gv.k >= 0 ? (args.skewK + gv.k + BK - 1 >= BK ? (args.skewK + gv.k + BK - 1) / BK : 1) : args.ntiles;

  LA la; LB lb;
  la.init(tid, m0, AKC ? args.skewM : 0, m_lim, args.lda);
  lb.init(tid, n0, BKC ? args.skewN : 0, n_lim, args.ldb);
  FragReader<AKC, BM, BK, TM> fra;
  FragReader<BKC, BN, BK, TN> frb;
  fra.init(lane, wm0);
  frb.init(lane, wn0);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // this workgroup's range [first, first + ntiles) of the K tiles of all segments laid end to end
  const int first = (int)((long long)all_tiles * split / ksplit);
  const int ntiles = (int)((long long)all_tiles * (split + 1) / ksplit) - first;
  int seg0 = 0, skip = first;
  while (seg0 + 1 < args.nseg) {
    const int in_seg = (args.skewK + args.seg[seg0].k + BK - 1) / BK;
    if (skip < in_seg) break;
    skip -= in_seg;
    seg0 = uni(seg0 + 1);
  }
  // producer state (runs STAGES-1 tiles ahead of the consumer)
  int pseg = seg0, pk0 = skip * BK, pkend = uni(args.skewK + (gv.k >= 0 ? gv.k : args.seg[seg0].k)), pslot = 0;
  __amdgpu_buffer_rsrc_t ra = make_rsrc(static_cast<const char*>(args.seg[seg0].a) + gv.oa, args.seg[seg0].a_bytes);
  __amdgpu_buffer_rsrc_t rb = make_rsrc(static_cast<const char*>(args.seg[seg0].b) + gv.ob, args.seg[seg0].b_bytes);
  // consumer state: k range of the tile being consumed (for the edge fix-up)
  int cseg = seg0, ck0 = pk0, ckend = pkend, cslot = 0;
  constexpr int KK = BK / 16;
  constexpr int MF = TM * TN;                       // MFMAs per k-step

  auto advance_producer = [&]() {
    pslot = pslot + 1 == STAGES ? 0 : pslot + 1;
    pk0 += BK;
    if (pk0 >= pkend && pseg + 1 < args.nseg) {
      pseg = uni(pseg + 1);
      pk0 = 0;
      pkend = uni(args.skewK + args.seg[pseg].k);
      ra = make_rsrc(static_cast<const char*>(args.seg[pseg].a) + gv.oa, args.seg[pseg].a_bytes);
      rb = make_rsrc(static_cast<const char*>(args.seg[pseg].b) + gv.ob, args.seg[pseg].b_bytes);
    }
  };

  // prologue: request the first STAGES-1 tiles
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < ntiles) {
      char* pa = smem + pslot * STAGE_BYTES;
      la.issue_edge(ra, pa, tid, LA::tile_offset(pk0, args.skewK, args.lda), pk0, args.skewK, pkend);
      lb.issue_edge(rb, pa + A_BYTES, tid, LB::tile_offset(pk0, args.skewK, args.ldb), pk0, args.skewK, pkend);
      advance_producer();
    }

  // One K tile.  FAST: the tile consumed and the tile requested are both interior tiles of their segments (all k
  // valid) and a request is due: no per-chunk validity, no fix-up, no data-dependent branch between the MFMAs, so
  // the whole tile is one scheduling region.  Otherwise the general form.
  auto tile = [&](int t, auto fast_tag) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value;
    char* sa = smem + cslot * STAGE_BYTES;
    char* sb = sa + A_BYTES;
    // tile t must have landed; up to STAGES-2 newer tiles may stay in flight
    if (STAGES > 2 && t + STAGES - 2 < ntiles) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((STAGES - 2) * LOADS_PER_TILE) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (!FAST && (ck0 < args.skewK || ck0 + BK > ckend)) {
      la.fixup(sa, tid, ck0, args.skewK, ckend);
      lb.fixup(sb, tid, ck0, args.skewK, ckend);
    }
    ck0 += BK;
    if (!FAST && ck0 >= ckend && cseg + 1 < args.nseg) { cseg = uni(cseg + 1); ck0 = 0; ckend = uni(args.skewK + args.seg[cseg].k); }
    __syncthreads();          // tile visible to all waves; every wave is done with the slot refilled below

    // the next request goes out in pieces between the MFMA groups of this tile (interior tiles), or
    // at once (first / last tile of a segment, where validity is decided per chunk)
    const bool produce = FAST || t + STAGES - 1 < ntiles;
    const bool edge = !FAST && (pk0 < args.skewK || pk0 + BK > pkend);
    char* pa = smem + pslot * STAGE_BYTES;
    char* pb = pa + A_BYTES;
    const unsigned soa = LA::tile_offset(pk0, args.skewK, args.lda);
    const unsigned sob = LB::tile_offset(pk0, args.skewK, args.ldb);
    if (!FAST && produce && edge) {
      la.issue_edge(ra, pa, tid, soa, pk0, args.skewK, pkend);
      lb.issue_edge(rb, pb, tid, sob, pk0, args.skewK, pkend);
    }
    const bool spread = !FAST && produce && !edge;
    constexpr bool kAtOnce = AKC && BKC;   // measured: with two 128-bit-read operands the whole request right after the barrier is faster, otherwise spread

    // fragments run kFragAhead k-steps ahead of the MFMAs that use them: a wave that has its SIMD to itself
    // (its partner waits at the barrier) must not stall on LDS latency between k-steps
    constexpr int kFragAhead = KK > 3 ? 3 : (KK > 2 ? 2 : 1), NB = kFragAhead + 1;
    bf16x8_t fa[NB][TM], fb[NB][TN];
    const unsigned ta = lds_addr(sa), tb = lds_addr(sb);
#pragma unroll
    for (int k0 = 0; k0 < kFragAhead; ++k0) {
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[k0][i] = fra.read(ta, i, k0);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[k0][j] = frb.read(tb, j, k0);
    }
    // The scheduling fences keep this order: without them the compiler moves each fragment read down to just before
    // the MFMA that uses it (fewer live registers), and the wave then waits on LDS in front of every MFMA.
    if (FAST) __builtin_amdgcn_sched_barrier(0);
    if (FAST && kAtOnce) { la.issue(ra, pa, tid, soa); lb.issue(rb, pb, tid, sob); __builtin_amdgcn_sched_barrier(0); }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int cur = kk % NB, nxt = (kk + kFragAhead) % NB;
      if (kk + kFragAhead < KK) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[nxt][i] = fra.read(ta, i, kk + kFragAhead);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[nxt][j] = frb.read(tb, j, kk + kFragAhead);
        if (FAST) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int x = 0; x < MF / 2; ++x) acc[x / TN][x % TN] = mfma(fb[cur][x % TN], fa[cur][x / TN], acc[x / TN][x % TN]);
      if ((FAST && !kAtOnce) || spread) la.issue_part(ra, pa, tid, soa, kk, KK);
      if (FAST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int x = MF / 2; x < MF; ++x) acc[x / TN][x % TN] = mfma(fb[cur][x % TN], fa[cur][x / TN], acc[x / TN][x % TN]);
      if ((FAST && !kAtOnce) || spread) lb.issue_part(rb, pb, tid, sob, kk, KK);
      if (FAST) __builtin_amdgcn_sched_barrier(0);
    }
    if (FAST) {      // the producer stays inside its segment
      pslot = pslot + 1 == STAGES ? 0 : pslot + 1;
      pk0 += BK;
    } else if (produce) {
      advance_producer();
    }
    cslot = cslot + 1 == STAGES ? 0 : cslot + 1;
  };
  // interior for the consumer: all of [ck0, ck0+BK) valid and not the segment's last tile; for the producer likewise,
  // and its next position stays inside the segment
  auto fast = [&](int t) {
    return t + STAGES - 1 < ntiles && ck0 >= args.skewK && ck0 + 2 * BK <= ckend && pk0 >= args.skewK && pk0 + 2 * BK <= pkend;
  };
  for (int t = 0; t < ntiles;) {
    for (; t < ntiles && !fast(t); ++t) tile(t, std::false_type());
    for (; t < ntiles && fast(t); ++t) tile(t, std::true_type());
  }

  __syncthreads();   // every wave is done reading the ring: reuse it as per-wave store patches
  if (ksplit > 1) {
    // raw fp32 partial tile [BM][BN]; bias, activation and the real store happen in the reduction kernel
    GemmArgs pa = args;
    pa.c = args.partial + (((long long)bp.grp * (gridDim.x / ksplit) + out_tile) * ksplit + split) * (BM * BN);
    pa.ldc = BN; pa.M = BM; pa.N = BN; pa.skewM = 0; pa.skewN = 0;
    pa.preact = nullptr; pa.bias = nullptr; pa.act = HAP_ACT_NONE; pa.accumulate = 0; pa.vec_store = 1; pa.cdelta = 0; pa.dact_preact = nullptr;
    epilogue_transposed<T, float, TM, TN>(pa, acc, wm0, wn0, lane, smem + wave * (32 * (TN * 32 * 4 + 16)));
    return;
  }
  epilogue_transposed<T, TC, TM, TN>(group_outputs(args, gv, bp.grp), acc, m0 + wm0, n0 + wn0, lane, smem + wave * (32 * (TN * 32 * (int)sizeof(TC) + 16)));
}

/* ---------------------------------------------------------------------------------------------
 * bf16 main kernel for 256 x 256 output tiles: the same direct-to-LDS loads, swizzles and fragment
 * addressing as gemm_dma_kernel, with the eight waves run as two groups that alternate between a
 * memory phase and a matrix phase, half a K tile apart ("ping-pong").
 *
 * A SIMD hosts one wave of each group (waves w and w + 4).  For K tile u a wave first runs
 *   Mem(u): fetch ALL of its fragments of tile u from LDS into registers, request the tile STAGES-1
 *           ahead from global memory, wait for its own chunks of tile u+1 (zeroing ragged k ends),
 * then, after a barrier,
 *   Cmp(u): nothing but the tile's MFMAs, at raised priority,
 * and another barrier.  Group 1 enters the loop one barrier later than group 0, so whenever one wave
 * of a SIMD is in Cmp the other is in Mem: the matrix unit always has a wave that issues nothing but
 * MFMAs, and the LDS reads and load issue of the other wave hide behind them instead of delaying
 * every wave's first MFMA after a common barrier.
 *
 * Ring discipline (phase p = interval between consecutive barriers; group 0 runs Mem(u) in phase 2u,
 * group 1 in phase 2u+1):
 *   - tile v is first read in phase 2v; every wave has waited for its own chunks of tile v in its
 *     Mem(v-1), i.e. by the barrier that ends phase 2v-1 (tile 0: before the first barrier);
 *   - the request issued in Mem(u) overwrites the slot of tile u-1, which both groups finished
 *     reading (LDS counter waited) by the barrier that ends phase 2u-1.
 * ------------------------------------------------------------------------------------------- */
#if !defined(HAP_PP_PRIO)
#define HAP_PP_PRIO 1
#endif
constexpr bool kPingPongPrio = HAP_PP_PRIO != 0;    // raise the wave's priority for its matrix phase
#if !defined(HAP_PP_DEFER)
#define HAP_PP_DEFER 1
#endif
constexpr bool kPingPongDefer = HAP_PP_DEFER != 0;  // group 0 awaits the next tile behind its MFMAs instead of in its memory phase
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

/* Fragment addressing of the ping-pong kernel: every address is (a register computed once before the K loop) +
 * (a compile-time offset in the instruction), so fetching a tile's fragments costs no vector ALU work at all - the
 * other wave of the SIMD owns the vector ALU port with its MFMAs meanwhile.  The ring lies at byte `ring` of LDS and
 * is wider than the 16-bit offset field reaches, hence one base register per 64 KiB of it. */
template <bool KC, int ROWS, int BK, int NBLK, int NH>
struct PinnedFrag {
  static constexpr int KK = BK / 16;
  static constexpr int CPR = (KC ? BK : ROWS) / 8;
  static constexpr int ROWB = CPR * 16;
  static constexpr int NB = KC ? KK : NBLK;      // K-contiguous: one base per k-step (the swizzle XOR); M/N-contiguous: one per 32-column block
  unsigned base[NB][NH];
  __device__ __forceinline__ void init(int lane, int wave_mn, unsigned ring) {
    FragReader<KC, ROWS, BK, NBLK> fr;
    fr.init(lane, wave_mn);
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int h = 0; h < NH; ++h) base[b][h] = (KC ? (fr.at[0] ^ (unsigned)(b << 5)) : fr.at[b]) + ring + (unsigned)h * 65536u;
  }
  /* Fragment of 32-row block BLK at k-step KKI of the tile that starts OFF bytes into the ring. */
  template <int OFF, int BLK, int KKI>
  __device__ __forceinline__ bf16x8_t read() const {
    constexpr int H = OFF >> 16, LO = OFF & 0xffff;
    if constexpr (KC) {
      static_assert(LO + BLK * 32 * ROWB < 65536, "offset field");
      return lds_read_b128_at<LO + BLK * 32 * ROWB>(base[KKI][H]);
    } else {
      static_assert(LO + KKI * 16 * ROWB + 4 * ROWB < 65536, "offset field");
      return lds_read_tr_pair_at<LO + KKI * 16 * ROWB, LO + KKI * 16 * ROWB + 4 * ROWB>(base[BLK][H]);
    }
  }
};

template <typename TC, bool AKC, bool BKC, int BM, int BN, int BK, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_pp_kernel(const GemmArgs args) {
  typedef __bf16 T;
  constexpr int NT = 64 * WGM * WGN;
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int NH = (STAGES * STAGE_BYTES + 65535) / 65536;
  typedef DmaLoader<AKC, BM, BK, NT> LA;
  typedef DmaLoader<BKC, BN, BK, NT> LB;
  constexpr int LPT = LA::CPT + LB::CPT;            // loads per thread and tile
  constexpr int KK = BK / 16;
  static_assert(STAGES >= 2 && STAGES <= 5 && (STAGES - 1) * LPT < 64, "ring depth");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  HAP_EXP_STAMP(0);

  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int wm0 = (wave / WGN) * WTM, wn0 = (wave % WGN) * WTN;
  const bool late_group = wave >= NW / 2;            // waves w and w + NW/2 share a SIMD
  const BlockPos bp = block_pos(args);
  const int ksplit = args.ksplit, out_tile = bp.out_tile, split = bp.split, tm = bp.tm, tn = bp.tn;
  const int m0 = tm * BM, n0 = tn * BN;
  const GroupView gv = group_view(args, bp.grp);
  const int m_lim = args.skewM + gv.M, n_lim = args.skewN + args.N;
  if (args.ragged == 1 && (gv.M == 0 || m0 >= m_lim)) return;
  const int all_tiles = gv.k >= 0 ? (args.skewK + gv.k + BK - 1 >= BK ? (args.skewK + gv.k + BK - 1) / BK : 1) : args.ntiles;

  LA la; LB lb;
  la.init(tid, m0, AKC ? args.skewM : 0, m_lim, args.lda);
  lb.init(tid, n0, BKC ? args.skewN : 0, n_lim, args.ldb);
  PinnedFrag<AKC, BM, BK, TM, NH> fra;
  PinnedFrag<BKC, BN, BK, TN, NH> frb;
  fra.init(lane, wm0, lds_addr(smem));
  frb.init(lane, wn0, lds_addr(smem));

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int first = (int)((long long)all_tiles * split / ksplit);
  const int ntiles = (int)((long long)all_tiles * (split + 1) / ksplit) - first;
  int seg0 = 0, skip = first;
  while (seg0 + 1 < args.nseg) {
    const int in_seg = (args.skewK + args.seg[seg0].k + BK - 1) / BK;
    if (skip < in_seg) break;
    skip -= in_seg;
    seg0 = uni(seg0 + 1);
  }
  // request cursor (runs STAGES-1 tiles ahead) and landing cursor (the next tile whose arrival is awaited); tile v lives in slot v % STAGES
  int pseg = seg0, pk0 = skip * BK, pkend = uni(args.skewK + (gv.k >= 0 ? gv.k : args.seg[seg0].k)), issued = 0;
  __amdgpu_buffer_rsrc_t ra = make_rsrc(static_cast<const char*>(args.seg[seg0].a) + gv.oa, args.seg[seg0].a_bytes);
  __amdgpu_buffer_rsrc_t rb = make_rsrc(static_cast<const char*>(args.seg[seg0].b) + gv.ob, args.seg[seg0].b_bytes);
  int lseg = seg0, lk0 = pk0, lkend = pkend;

  auto request = [&](auto slot_tag) {
    constexpr int SLOT = decltype(slot_tag)::value;
    char* pa = smem + SLOT * STAGE_BYTES;
    char* pb = pa + A_BYTES;
    const unsigned soa = LA::tile_offset(pk0, args.skewK, args.lda), sob = LB::tile_offset(pk0, args.skewK, args.ldb);
    if (pk0 < args.skewK || pk0 + BK > pkend) {      // first / last tile of a segment: validity per chunk
      la.issue_edge(ra, pa, tid, soa, pk0, args.skewK, pkend);
      lb.issue_edge(rb, pb, tid, sob, pk0, args.skewK, pkend);
    } else {
      la.issue(ra, pa, wave << 6, soa);          // (issue() needs only the wave's first thread id, here already a scalar)
      lb.issue(rb, pb, wave << 6, sob);
    }
    pk0 += BK;
    ++issued;
    if (pk0 >= pkend && pseg + 1 < args.nseg) {
      pseg = uni(pseg + 1);
      pk0 = 0;
      pkend = uni(args.skewK + args.seg[pseg].k);
      ra = make_rsrc(static_cast<const char*>(args.seg[pseg].a) + gv.oa, args.seg[pseg].a_bytes);
      rb = make_rsrc(static_cast<const char*>(args.seg[pseg].b) + gv.ob, args.seg[pseg].b_bytes);
    }
  };
  // Waits until at most `newer` tiles requested after the awaited one are still in flight, then zeroes the awaited
  // tile's k elements outside the logical range (own chunks only) and moves the landing cursor on.
  auto land = [&](auto slot_tag, int newer) {
    constexpr int SLOT = decltype(slot_tag)::value;
    if (newer >= STAGES - 2) wait_vmcnt<(STAGES - 2) * LPT>();          // the steady state
    else if (STAGES > 3 && newer == 2) wait_vmcnt<(STAGES > 3 ? 2 : 0) * LPT>();
    else if (STAGES > 2 && newer == 1) wait_vmcnt<(STAGES > 2 ? 1 : 0) * LPT>();
    else wait_vmcnt<0>();
    if (lk0 < args.skewK || lk0 + BK > lkend) {
      char* sa = smem + SLOT * STAGE_BYTES;
      la.fixup(sa, tid, lk0, args.skewK, lkend);
      lb.fixup(sa + A_BYTES, tid, lk0, args.skewK, lkend);
    }
    lk0 += BK;
    if (lk0 >= lkend && lseg + 1 < args.nseg) { lseg = uni(lseg + 1); lk0 = 0; lkend = uni(args.skewK + args.seg[lseg].k); }
  };

  static_for<STAGES - 1>([&](auto s) { if (s < ntiles) request(s); });
  if (ntiles > 0) land(std::integral_constant<int, 0>(), issued - 1);
  __builtin_amdgcn_s_barrier();                      // tile 0 is in LDS for everybody
  HAP_EXP_STAMP(1);
  if (late_group) __builtin_amdgcn_s_barrier();      // group 1 runs one phase behind group 0

  // one K tile whose ring slot is known at compile time
  // FAST: the tile requested and the tile awaited are interior tiles of their segments and both cursors stay inside their
  // segments, a request is due and a tile follows - no per-chunk validity, no fix-up, no data-dependent branch at all.
  // (The two forms share ONE copy of the matrix phase: two copies of the tile body made the compiler shuffle the 128
  // accumulator registers between them through scratch memory.)
  auto tile = [&](auto slot_tag, const bool fast, int u) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    constexpr int PREV = (SLOT + STAGES - 1) % STAGES, NEXT = (SLOT + 1) % STAGES;
    // ---- Mem(u): all fragments of the tile, the request STAGES-1 tiles ahead (into the slot of tile u-1), arrival of tile u+1
    bf16x8_t fa[KK][TM], fb[KK][TN];
    static_for<KK>([&](auto kk) {
      static_for<TN>([&](auto j) { fb[kk][j] = frb.template read<SLOT * STAGE_BYTES + A_BYTES, j, kk>(); });
      static_for<TM>([&](auto i) { fa[kk][i] = fra.template read<SLOT * STAGE_BYTES, i, kk>(); });
    });
    if (fast) {
      char* pa = smem + PREV * STAGE_BYTES;
      la.issue(ra, pa, wave << 6, LA::tile_offset(pk0, args.skewK, args.lda));
      lb.issue(rb, pa + A_BYTES, wave << 6, LB::tile_offset(pk0, args.skewK, args.ldb));
      pk0 += BK;
      ++issued;
    } else {
      if (issued < ntiles) request(std::integral_constant<int, PREV>());
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // this wave's reads of tile u are done (its slot is refilled two phases on)
    if (fast) {
      // Tile u+1 is first read by group 0, in its memory phase behind the NEXT barrier but one (group 0's matrix phase lies
      // between).  Group 1 is one phase behind: the barrier that ends this memory phase is already the last one before that read,
      // so it waits here; group 0 has its whole matrix phase to go and waits behind its MFMAs.
      if (late_group || !kPingPongDefer) wait_vmcnt<(STAGES - 2) * LPT>();
      lk0 += BK;
    } else {
      if (u + 1 < ntiles) land(std::integral_constant<int, NEXT>(), issued - (u + 2));
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // ---- Cmp(u)
    if (kPingPongPrio) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
      for (int x = 0; x < TM * TN; ++x) acc[x / TN][x % TN] = mfma(fb[kk][x % TN], fa[kk][x / TN], acc[x / TN][x % TN]);
    if (kPingPongPrio) __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    // group 0 awaits its share of tile u+1 here: one more phase for the loads to arrive, and the wait is out of the memory phase
    // that group 1's MFMAs run against
    if (kPingPongDefer && fast && !late_group) wait_vmcnt<(STAGES - 2) * LPT>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  for (int u0 = 0; u0 < ntiles; u0 += STAGES) {
    const bool fast = issued + STAGES <= ntiles && pk0 >= args.skewK && pk0 + STAGES * BK < pkend &&
                      lk0 >= args.skewK && lk0 + STAGES * BK < lkend;
    static_for<STAGES>([&](auto s) { if (fast || u0 + s < ntiles) tile(s, fast, u0 + s); });
  }
  if (!late_group) __builtin_amdgcn_s_barrier();     // group 1's last matrix phase: after it nobody reads the ring any more
  HAP_EXP_STAMP(2);

  if (ksplit > 1) {
    GemmArgs pa = args;
    pa.c = args.partial + (((long long)bp.grp * (gridDim.x / ksplit) + out_tile) * ksplit + split) * (BM * BN);
    pa.ldc = BN; pa.M = BM; pa.N = BN; pa.skewM = 0; pa.skewN = 0;
    pa.preact = nullptr; pa.bias = nullptr; pa.act = HAP_ACT_NONE; pa.accumulate = 0; pa.vec_store = 1; pa.cdelta = 0; pa.dact_preact = nullptr;
    epilogue_transposed<T, float, TM, TN>(pa, acc, wm0, wn0, lane, smem + wave * (32 * (TN * 32 * 4 + 16)));
    return;
  }
  epilogue_transposed<T, TC, TM, TN>(group_outputs(args, gv, bp.grp), acc, m0 + wm0, n0 + wn0, lane, smem + wave * (32 * (TN * 32 * (int)sizeof(TC) + 16)));
  HAP_EXP_STAMP(3);
}

/* Split-K reduction: sums the ksplit fp32 partial tiles of every output tile and applies what the
 * one-pass epilogue would have (bias, pre-activation copy, activation, accumulation, conversion),
 * storing only the logical rows / columns.  One thread per 4 consecutive columns. */
template <typename T, typename TC, int BM, int BN>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs args_in, int out_tiles) {
  const GemmArgs args = group_outputs(args_in, group_view(args_in, blockIdx.y), blockIdx.y);   // blockIdx.y: group
  constexpr int QPT = BM * BN / 4;                 // column quads per tile
  const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
  const int tile = (int)(gid / QPT), q = (int)(gid % QPT);
  if (tile >= out_tiles) return;
  int tm, tn;
  if (gridDim.y == 1) tile_of_block(tile, out_tiles, args.tiles_m, args.tiles_n, &tm, &tn);   // the maps of block_pos()
  else tile_of_logical(tile, args.tiles_m, args.tiles_n, &tm, &tn);
  const int r = q / (BN / 4), c4 = (q % (BN / 4)) * 4;
  const int m = tm * BM + r - args.skewM, n = tn * BN + c4 - args.skewN;
  if (m < 0 || m >= args.M || n >= args.N || n + 4 <= 0) return;
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  f32x4_t sum = {0.0f, 0.0f, 0.0f, 0.0f};
  const float* p = args.partial + ((long long)blockIdx.y * out_tiles + tile) * args.ksplit * (BM * BN) + r * BN + c4;
  for (int s = 0; s < args.ksplit; ++s) sum += *reinterpret_cast<const f32x4_t*>(p + (long long)s * (BM * BN));
  TC* C = static_cast<TC*>(args.c);
  TC* P = static_cast<TC*>(args.preact);
  const T* bias = static_cast<const T*>(args.bias);
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int nn = n + x;
    if (nn < 0 || nn >= args.N) continue;
    float v = sum[x];
    if (bias) v += load_s<T>(bias + nn);
    if (P) store_c<TC>(P + (long long)m * args.ldp + nn, v);
    if (args.act == HAP_ACT_GELU_ERF) v = gelu_erf((float)(TC)v);     // the activation sees the value as stored
    if (args.dact_preact) v *= gelu_erf_grad(load_s<TC>(static_cast<const TC*>(args.dact_preact) + (long long)m * args.ldd + nn));
    TC* dst = C + (long long)m * args.ldc + nn;
    if (args.accumulate) v += load_s<TC>(dst);
    store_c<TC>(dst, v);
  }
}

/* ---------------------------------------------------------------------------------------------
 * fp32 products with at most 64 output rows (a layer whose batch shard is a few dozen samples: the single fully-connected layer
 * of the smallest workload, 38 / 26 rows of 64).  Such a product has far too few output tiles for the chip, and splitting its
 * contraction over workgroups costs a second, dependent launch for the reduction - on this machine about as long as the product
 * itself.  Here the split happens INSIDE a workgroup: one workgroup owns all (<= 64) rows of 16 output columns, its 16 waves each
 * contract 1/16 of K with v_mfma_f32_16x16x4_f32, and their partial tiles are summed through LDS in a fixed order (deterministic).
 *   A (K-contiguous): lane (row r = lane % 16, k-quad q = lane / 16) fetches the 4 consecutive k values 16c + 4q .. + 3 of a
 *   16-wide chunk c as one 16-byte load and feeds element s to step s; B's lane (k-quad q, column) supplies the same k, so the
 *   order in which a chunk's k values are consumed is a permutation that both operands share.
 * ------------------------------------------------------------------------------------------- */
struct SkinnyArgs {
  int M, N, K;
  long long lda, ldb, ldc, ldp;
  const float* a; const float* b; float* c; float* preact; const float* bias;
  int act, accumulate;
};

typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <bool BKC>
__global__ __launch_bounds__(1024) void gemm_skinny_f32_kernel(const SkinnyArgs g) {
  __shared__ float red[16][64][16];                  // one partial [rows][columns] tile per wave: 64 KB
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, kq = lane >> 4;
  const int n0 = blockIdx.x * 16, col = n0 + r;
  const int rb = (g.M + 15) >> 4;                    // 16-row blocks in use
  const int kslice = ((g.K + 255) >> 8) << 4;        // k values per wave, a multiple of 16
  const int kb0 = wave * kslice;
  const int kb1 = kb0 + kslice < g.K ? kb0 + kslice : g.K;      // (K is a multiple of 4: a lane's quad is inside or outside as a whole)
  f32x4_t acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int kb = kb0; kb < kb1; kb += 64) {
    f32x4_t av[4][4], bv[4];
    // all loads of four chunks first, then their MFMAs
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int kk = kb + 16 * c + 4 * kq;
      const bool kin = kk < kb1;
      bv[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (kin && col < g.N) {
        if constexpr (BKC) bv[c] = *reinterpret_cast<const f32x4_t*>(g.b + (long long)col * g.ldb + kk);
        else {
#pragma unroll
          for (int x = 0; x < 4; ++x) bv[c][x] = g.b[(long long)(kk + x) * g.ldb + col];
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = i * 16 + r;
        av[c][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (i < rb && kin && row < g.M) av[c][i] = *reinterpret_cast<const f32x4_t*>(g.a + (long long)row * g.lda + kk);
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (i < rb) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[c][i][x], bv[c][x], acc[i], 0, 0, 0);
  }
  // accumulator element v of lane l is output (row 4 * (l / 16) + v, column l % 16) of its 16-row block
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][i * 16 + 4 * kq + v][r] = acc[i][v];
  __syncthreads();
  const int row = tid >> 4, c = tid & 15, n = n0 + c;
  if (row >= g.M || n >= g.N) return;
  float v = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) v += red[w][row][c];
  if (g.bias) v += g.bias[n];
  if (g.preact) g.preact[(long long)row * g.ldp + n] = v;
  if (g.act == HAP_ACT_GELU_ERF) v = gelu_erf(v);
  float* dst = g.c + (long long)row * g.ldc + n;
  if (g.accumulate) v += *dst;
  *dst = v;
}

/* Whether hap_gemm_run hands the product to gemm_skinny_f32_kernel (see there). */
static bool skinny_f32_applies(const hap_gemm_problem* p) {
  if (p->in_dtype != HAP_F32 || p->c_dtype != HAP_F32 || p->M > 64 || !p->a_kcontig || p->nseg != 1) return false;
  if (p->groups > 1 || p->group_len || p->force_generic || p->tile || p->dact) return false;
  const int64_t K = p->k[0];
  if (K < 256 || K % 4 || K > 0x7fffffff || (p->N + 63) / 64 >= 128) return false;      // enough 64-wide tiles: the tiled kernel fills the chip by itself
  if (p->lda % 4 || (uintptr_t)p->a[0] % 16) return false;
  if (p->b_kcontig && (p->ldb % 4 || (uintptr_t)p->b[0] % 16)) return false;
  return true;
}

/* Scalar fallback for operand views the tiled kernel cannot address with aligned 16-byte chunks
 * (leading dimension not a multiple of 16 bytes, or differently skewed K-contiguous operands). */
struct GenericArgs {
  int M, N, nseg;
  long long lda, ldb, ldc, ldp;
  int a_kcontig, b_kcontig;
  void* c; void* preact; const void* bias;
  int act, accumulate;
  const void* dact_preact; long long ldd;
  int ragged;                        // as in GemmArgs; blockIdx.z is the group
  const int* group_len;
  long long ga, gb, gc, gp, gbias, gd;   // byte strides between groups
  const void* a[HAP_GEMM_MAX_SEG];
  const void* b[HAP_GEMM_MAX_SEG];
  int k[HAP_GEMM_MAX_SEG];
};

template <typename T, typename TC>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const GenericArgs g) {
  const int n = blockIdx.x * 16 + (threadIdx.x & 15);
  const int m = blockIdx.y * 16 + (threadIdx.x >> 4);
  const int grp = blockIdx.z;
  int len = g.ragged ? g.group_len[grp] : 0;
  len = len < 0 ? 0 : len;
  const int M = g.ragged == 1 && len < g.M ? len : g.M;
  if (m >= M || n >= g.N) return;
  float acc = 0.0f;
  for (int s = 0; s < g.nseg; ++s) {
    const T* A = reinterpret_cast<const T*>(static_cast<const char*>(g.a[s]) + grp * g.ga);
    const T* B = reinterpret_cast<const T*>(static_cast<const char*>(g.b[s]) + grp * g.gb);
    const int ks = g.ragged == 2 && len < g.k[s] ? len : g.k[s];
    for (int k = 0; k < ks; ++k) {
      const float av = load_s<T>(g.a_kcontig ? A + (long long)m * g.lda + k : A + (long long)k * g.lda + m);
      const float bv = load_s<T>(g.b_kcontig ? B + (long long)n * g.ldb + k : B + (long long)k * g.ldb + n);
      acc = fmaf(av, bv, acc);
    }
  }
  if (g.bias) acc += load_s<T>(reinterpret_cast<const T*>(static_cast<const char*>(g.bias) + grp * g.gbias) + n);
  if (g.preact) store_c<TC>(reinterpret_cast<TC*>(static_cast<char*>(g.preact) + grp * g.gp) + (long long)m * g.ldp + n, acc);
  if (g.act == HAP_ACT_GELU_ERF) acc = gelu_erf((float)(TC)acc);     // the activation sees the value as stored
  if (g.dact_preact) acc *= gelu_erf_grad(load_s<TC>(reinterpret_cast<const TC*>(static_cast<const char*>(g.dact_preact) + grp * g.gd) + (long long)m * g.ldd + n));
  TC* dst = reinterpret_cast<TC*>(static_cast<char*>(g.c) + grp * g.gc) + (long long)m * g.ldc + n;
  if (g.accumulate) acc += load_s<TC>(dst);
  store_c<TC>(dst, acc);
}

/* Compute units of the current device (256 on MI355X), asked once per device; the planner's round arithmetic uses it. */
int cu_count() {
  static int cached[64] = {};
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return 256;
  if (cached[device] == 0) {     // benign race: every thread stores the same value
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n < 8) n = 256;
    cached[device] = n;
  }
  return cached[device];
}

#if defined(HAP_GEMM_EXPERIMENT)
int hap_exp_variant = 0;          // experiment builds only: 0 = ping-pong BK 32 x 4 stages, 1 = BK 32 x 5, 2 = BK 64 x 2, 3 = the two-stage kernel
#define kPingPongBK (hap_exp_variant == 2 || hap_exp_variant == 3 ? 64 : 32)
#define kPingPongSkipsKK false
#else
constexpr int kPingPongBK = 32;   // K step and ring depth of the 256 x 256 kernel: 4 stages of 32 KiB
constexpr bool kPingPongSkipsKK = true;
#endif
constexpr int kPingPongStages = 4;

struct Plan {
  bool tiled;
  int skewM, skewN, skewK;
  int bm, bn;       // tile
  int bk;           // K step of the kernel that will run (the K-tile counts handed to it are in this unit)
  const char* name;
  int dma;          // 1: bf16, direct-to-LDS kernel; 0: fp32, register-staged kernel
  bool pingpong;    // 256 x 256 tiles run by gemm_pp_kernel
};

inline int esize(int dtype) { return dtype == HAP_BF16 ? 2 : 4; }

/* Decides whether the aligned-chunk kernel can address the operands and with which skews. */
Plan make_plan(const hap_gemm_problem* p) {
  Plan pl = {false, 0, 0, 0, 0, 0, 64, "generic", 0, false};
  if (p->force_generic) return pl;
  const int es = esize(p->in_dtype);
  if ((p->lda * es) % 16 || (p->ldb * es) % 16) return pl;
  if (p->groups > 1 && ((p->ga * es) % 16 || (p->gb * es) % 16)) return pl;   // every group needs the first one's 16-byte phase
  int sa = -1, sb = -1;
  for (int s = 0; s < p->nseg; ++s) {
    if (p->k[s] == 0) continue;
    const int xa = (int)(((uintptr_t)p->a[s] % 16) / es), xb = (int)(((uintptr_t)p->b[s] % 16) / es);
    if (((uintptr_t)p->a[s] % es) || ((uintptr_t)p->b[s] % es)) return pl;
    if (sa < 0) { sa = xa; sb = xb; }
    else if (sa != xa || sb != xb) return pl;
  }
  if (sa < 0) { sa = sb = 0; }
  if (p->a_kcontig && p->b_kcontig && sa != sb) return pl;
  // K-contiguous operands: a K tile fetches 64 or 128 consecutive bytes of every row, so the K-tile grid is laid on 128-byte
  // (else 64-byte) boundaries of the operand's own address space where the pitch allows it - the view's first k then sits up
  // to 63 elements into its first tile, which is masked like any skew.  Fetches that straddle cache sectors cost 10-20 %.
  if (p->in_dtype == HAP_BF16 && !(p->groups > 1) && (p->a_kcontig || p->b_kcontig)) {
    for (int gran = 128; gran >= 32; gran /= 2) {
      if ((p->a_kcontig && (p->lda * es) % gran) || (p->b_kcontig && (p->ldb * es) % gran)) continue;
      int ka = -1, kb = -1;
      bool ok = true;
      for (int s = 0; s < p->nseg && ok; ++s) {
        if (p->k[s] == 0) continue;
        const int xa = (int)(((uintptr_t)p->a[s] % gran) / es), xb = (int)(((uintptr_t)p->b[s] % gran) / es);
        if (ka < 0) { ka = xa; kb = xb; }
        else ok = (!p->a_kcontig || ka == xa) && (!p->b_kcontig || kb == xb);
      }
      if (!ok || ka < 0 || (p->a_kcontig && p->b_kcontig && ka != kb)) continue;
      if (p->a_kcontig) sa = ka;
      if (p->b_kcontig) sb = kb;
      break;
    }
  }
  pl.skewK = p->a_kcontig ? sa : (p->b_kcontig ? sb : 0);
  pl.skewM = p->a_kcontig ? 0 : sa;
  pl.skewN = p->b_kcontig ? 0 : sb;
  // A K-contiguous B has no preferred column origin of its own (its rows are the output's columns), so the tile grid is laid on
  // the 16-byte chunks of the OUTPUT instead: the reduction rule's dX[:, k_j] of a whole tensor starts at an arbitrary column, and
  // with the grid on its chunks the epilogue stores whole chunks everywhere but at the matrix's two ends.
  if (p->b_kcontig && p->in_dtype == HAP_BF16 && !(p->groups > 1) && !p->group_len) {
    const int ces = esize(p->c_dtype), cepc = 16 / ces;
    if ((uintptr_t)p->c % ces == 0 && p->ldc % cepc == 0) pl.skewN = (int)(((uintptr_t)p->c % 16) / ces);
  }
  // operand views must stay below 2 GiB so 32-bit buffer offsets and the out-of-range marker work
  for (int s = 0; s < p->nseg; ++s) {
    const double ea = p->a_kcontig ? ((double)(p->M - 1) * p->lda + pl.skewK + p->k[s]) : ((double)(p->k[s] - 1) * p->lda + pl.skewM + p->M);
    const double eb = p->b_kcontig ? ((double)(p->N - 1) * p->ldb + pl.skewK + p->k[s]) : ((double)(p->k[s] - 1) * p->ldb + pl.skewN + p->N);
    if (ea * es >= (double)kViewLimitBytes || eb * es >= (double)kViewLimitBytes) return pl;
  }
  pl.tiled = true;
  if (p->in_dtype == HAP_F32) { pl.bm = pl.bn = 64; pl.name = "f32_64x64x16"; }
  else {
    bool big = p->tile ? p->tile == 256 : (p->M + pl.skewM > 128 && p->N + pl.skewN > 128);
    if (big && !p->tile && (p->groups > 1 || p->group_len)) {
      const int kCUs = cu_count();
      // A grouped launch is not cut into strips: compare whole rounds of big tiles (one per CU, time 1 each) with rounds
      // of small ones (two per CU, a quarter of the work each at lower efficiency: 0.6 per round, 0.3 when half empty).
      const long long g = p->groups > 1 ? p->groups : 1;
      const long long nb = g * ((p->M + pl.skewM + 255) / 256) * ((p->N + pl.skewN + 255) / 256);
      const long long ns = g * ((p->M + pl.skewM + 127) / 128) * ((p->N + pl.skewN + 127) / 128);
      // few big tiles: split-K can spread them over the chip at about a third of a round for the partial-tile traffic
      const double tb = nb * 2 <= kCUs ? 0.35 + 1.0 / (double)(kCUs / nb) : (double)((nb + kCUs - 1) / kCUs);
      const double ts = ns <= kCUs ? 0.3 : 0.6 * (double)((ns + 2 * kCUs - 1) / (2 * kCUs));
      big = tb <= ts;
    }
    pl.bm = pl.bn = big ? 256 : 128;
    pl.dma = 1;
    // 256-tiles: the ping-pong kernel, except when both operands are K-contiguous (bwd-data), where the two-stage kernel
    // with 128-byte rows per K tile is the faster one
    // ... and except short contractions: below about 20 K tiles of 64 the four-stage ring's fill does not pay off (measured at
    // K = 512 / 768 / 1024: the two-stage kernel is 7 / 4 / 1 % faster, from K = 1536 on the ping-pong kernel wins)
    long long nk64 = 0;
    for (int s = 0; s < p->nseg; ++s) nk64 += p->k[s] > 0 ? (pl.skewK + p->k[s] + 63) / 64 : 0;
    const bool short_k = kPingPongSkipsKK && nk64 < 20 && !(!p->a_kcontig && p->b_kcontig);
    pl.pingpong = big && !(p->a_kcontig && p->b_kcontig && kPingPongSkipsKK) && !short_k;
    pl.bk = pl.pingpong ? kPingPongBK : 64;
    pl.name = pl.pingpong ? "bf16_256x256x32_pingpong4" : (big ? "bf16_256x256x64_dma2" : "bf16_128x128x64_dma2");
  }
  return pl;
}

template <typename T, typename TC, bool AKC, bool BKC, int BM, int BN, int BK, int WGM, int WGN>
int launch_tiled(const GemmArgs& a, int groups, hipStream_t st) {
  const int out_tiles = a.tiles_m * a.tiles_n;
  hipLaunchKernelGGL((gemm_kernel<T, TC, AKC, BKC, BM, BN, BK, WGM, WGN>), dim3(out_tiles * a.ksplit, groups), dim3(64 * WGM * WGN), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "gemm launch: %s", hipGetErrorString(e));
  if (a.ksplit > 1) {
    const long long threads = (long long)out_tiles * (BM * BN / 4);
    hipLaunchKernelGGL((splitk_reduce_kernel<T, TC, BM, BN>), dim3((unsigned)((threads + 255) / 256), groups), dim3(256), 0, st, a, out_tiles);
    e = hipGetLastError();
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "split-K reduce launch: %s", hipGetErrorString(e));
  }
  return HAP_OK;
}

template <typename TC, bool AKC, bool BKC, int BM, int BN, int BK, int STAGES, int WGM, int WGN>
int launch_dma(const GemmArgs& a, int groups, hipStream_t st) {
  constexpr size_t smem = (size_t)STAGES * (BM + BN) * BK * 2;
  void (*kernel)(const GemmArgs) = &gemm_dma_kernel<TC, AKC, BKC, BM, BN, BK, WGM, WGN, STAGES>;
  // the attribute belongs to the kernel's copy on the current device (benign race: the call is idempotent)
  static bool configured[64] = {};
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) device = -1;
  if (device < 0 || !configured[device]) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "cannot reserve %zu bytes of LDS: %s", smem, hipGetErrorString(e));
    if (device >= 0) configured[device] = true;
  }
  const int out_tiles = a.tiles_m * a.tiles_n;
  hipLaunchKernelGGL(kernel, dim3(out_tiles * a.ksplit, groups), dim3(64 * WGM * WGN), smem, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "gemm launch: %s", hipGetErrorString(e));
  if (a.ksplit > 1) {
    const long long threads = (long long)out_tiles * (BM * BN / 4);
    hipLaunchKernelGGL((splitk_reduce_kernel<__bf16, TC, BM, BN>), dim3((unsigned)((threads + 255) / 256), groups), dim3(256), 0, st, a, out_tiles);
    e = hipGetLastError();
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "split-K reduce launch: %s", hipGetErrorString(e));
  }
  return HAP_OK;
}

template <typename TC, int BM, int BN, int BK, int STAGES, int WGM, int WGN>
int dispatch_dma(const hap_gemm_problem* p, const GemmArgs& a, int groups, hipStream_t st) {
  if (p->a_kcontig && p->b_kcontig) return launch_dma<TC, true, true, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
  if (p->a_kcontig && !p->b_kcontig) return launch_dma<TC, true, false, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
  if (!p->a_kcontig && !p->b_kcontig) return launch_dma<TC, false, false, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
  return launch_dma<TC, false, true, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
}

template <typename TC, bool AKC, bool BKC, int BM, int BN, int BK, int STAGES, int WGM, int WGN>
int launch_pp(const GemmArgs& a, int groups, hipStream_t st) {
  constexpr size_t smem = (size_t)STAGES * (BM + BN) * BK * 2;
  void (*kernel)(const GemmArgs) = &gemm_pp_kernel<TC, AKC, BKC, BM, BN, BK, WGM, WGN, STAGES>;
  // the attribute belongs to the kernel's copy on the current device (benign race: the call is idempotent)
  static bool configured[64] = {};
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) device = -1;
  if (device < 0 || !configured[device]) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "cannot reserve %zu bytes of LDS: %s", smem, hipGetErrorString(e));
    if (device >= 0) configured[device] = true;
  }
  const int out_tiles = a.tiles_m * a.tiles_n;
  hipLaunchKernelGGL(kernel, dim3(out_tiles * a.ksplit, groups), dim3(64 * WGM * WGN), smem, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "gemm launch: %s", hipGetErrorString(e));
  if (a.ksplit > 1) {
    const long long threads = (long long)out_tiles * (BM * BN / 4);
    hipLaunchKernelGGL((splitk_reduce_kernel<__bf16, TC, BM, BN>), dim3((unsigned)((threads + 255) / 256), groups), dim3(256), 0, st, a, out_tiles);
    e = hipGetLastError();
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "split-K reduce launch: %s", hipGetErrorString(e));
  }
  return HAP_OK;
}

template <typename TC, int BM, int BN, int BK, int STAGES, int WGM, int WGN>
int dispatch_pp(const hap_gemm_problem* p, const GemmArgs& a, int groups, hipStream_t st) {
  if (p->a_kcontig && p->b_kcontig) return launch_pp<TC, true, true, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
  if (p->a_kcontig && !p->b_kcontig) return launch_pp<TC, true, false, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
  if (!p->a_kcontig && !p->b_kcontig) return launch_pp<TC, false, false, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
  return launch_pp<TC, false, true, BM, BN, BK, STAGES, WGM, WGN>(a, groups, st);
}

template <typename T, typename TC, int BM, int BN, int BK, int WGM, int WGN>
int dispatch_layout(const hap_gemm_problem* p, const GemmArgs& a, int groups, hipStream_t st) {
  if (p->a_kcontig && p->b_kcontig) return launch_tiled<T, TC, true, true, BM, BN, BK, WGM, WGN>(a, groups, st);
  if (p->a_kcontig && !p->b_kcontig) return launch_tiled<T, TC, true, false, BM, BN, BK, WGM, WGN>(a, groups, st);
  if (!p->a_kcontig && !p->b_kcontig) return launch_tiled<T, TC, false, false, BM, BN, BK, WGM, WGN>(a, groups, st);
  return launch_tiled<T, TC, false, true, BM, BN, BK, WGM, WGN>(a, groups, st);
}

template <typename T, typename TC>
int dispatch_tile(const hap_gemm_problem* p, const Plan& pl, const GemmArgs& a, int groups, hipStream_t st) {
  if constexpr (sizeof(T) == 4) {
    return dispatch_layout<T, TC, 64, 64, 64, 2, 2>(p, a, groups, st);
  } else {
#if defined(HAP_GEMM_EXPERIMENT)
#if defined(HAP_GEMM_EXPERIMENT_ALL)
    if (pl.bm == 256 && hap_exp_variant == 1) return dispatch_pp<TC, 256, 256, 32, 5, 2, 4>(p, a, groups, st);
    if (pl.bm == 256 && hap_exp_variant == 2) return dispatch_pp<TC, 256, 256, 64, 2, 2, 4>(p, a, groups, st);
#endif
    if (pl.bm == 256 && hap_exp_variant == 3) return dispatch_dma<TC, 256, 256, 64, 2, 2, 4>(p, a, groups, st);
#endif
    if (pl.pingpong) return dispatch_pp<TC, 256, 256, 32, kPingPongStages, 2, 4>(p, a, groups, st);
#if defined(HAP_GEMM_EXPERIMENT)
    if (pl.bm == 256) return dispatch_dma<TC, 256, 256, 64, 2, 2, 4>(p, a, groups, st);
#else
    // 256-tiles outside the ping-pong kernel: both operands K-contiguous, or a short contraction (A M-contiguous with B
    // K-contiguous always takes the ping-pong kernel, so that layout of the two-stage kernel is not built at this size)
    if (pl.bm == 256) {
      if (p->a_kcontig && p->b_kcontig) return launch_dma<TC, true, true, 256, 256, 64, 2, 2, 4>(a, groups, st);
      if (p->a_kcontig) return launch_dma<TC, true, false, 256, 256, 64, 2, 2, 4>(a, groups, st);
      if (!p->b_kcontig) return launch_dma<TC, false, false, 256, 256, 64, 2, 2, 4>(a, groups, st);
      return hap_fail(HAP_EDEVICE, "internal: no 256-tile two-stage kernel for this layout");
    }
#endif
    return dispatch_dma<TC, 128, 128, 64, 2, 2, 2>(p, a, groups, st);
  }
}

}  // namespace hap_gemm_detail

using namespace hap_gemm_detail;

const char* hap_gemm_variant(const hap_gemm_problem* p) { return make_plan(p).name; }

namespace {

/* Relative time of n output tiles of 128x128 (one 256x256 tile on one CU = 1): a small tile does a
 * quarter of the work at lower efficiency, and two of them share a CU. */
double small_tiles_time(long long n) {
  if (n <= 0) return 0.0;
  const int kCUs = cu_count();
  // measured: a round of 512 small tiles takes 0.58 of a round of 256 big ones; a last round that leaves every CU at
  // most one small tile 0.36 (the tile has the CU to itself)
  const long long full = n / (2 * kCUs), rest = n % (2 * kCUs);
  return 0.58 * (double)full + (rest == 0 ? 0.0 : (rest <= kCUs ? 0.36 : 0.58));
}

inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }

/* The sub-problem of p over logical rows [m_lo, m_hi) and columns [n_lo, n_hi). */
hap_gemm_problem sub_problem(const hap_gemm_problem* p, int64_t m_lo, int64_t m_hi, int64_t n_lo, int64_t n_hi, int tile) {
  hap_gemm_problem q = *p;
  const int es = esize(p->in_dtype), ces = esize(p->c_dtype);
  q.M = m_hi - m_lo; q.N = n_hi - n_lo; q.tile = tile;
  for (int s = 0; s < p->nseg; ++s) {
    q.a[s] = static_cast<const char*>(p->a[s]) + (p->a_kcontig ? m_lo * p->lda : m_lo) * es;
    q.b[s] = static_cast<const char*>(p->b[s]) + (p->b_kcontig ? n_lo * p->ldb : n_lo) * es;
  }
  q.c = static_cast<char*>(p->c) + (m_lo * p->ldc + n_lo) * ces;
  if (p->preact) q.preact = static_cast<char*>(p->preact) + (m_lo * p->ldp + n_lo) * ces;
  if (p->dact_preact) q.dact_preact = static_cast<const char*>(p->dact_preact) + (m_lo * p->ldd + n_lo) * ces;
  if (p->bias) q.bias = static_cast<const char*>(p->bias) + n_lo * es;
  return q;
}

}  // namespace

static int64_t g_view_limit = kViewLimitBytes;
static int64_t g_cut_products = 0;      // products run in pieces so far (testing aid, not synchronised)

/* Test hook (declared in hap_internal.h, not part of the public interface): lowers the reach at which operand views are
 * cut so the cutting can be exercised on small inputs; returns how many products have run in pieces so far. */
extern "C" int64_t hap_debug_set_gemm_view_limit(int64_t bytes) {
  g_view_limit = bytes > 0 && bytes < kViewLimitBytes ? bytes : kViewLimitBytes;
  return g_cut_products;
}

/* Operand views of 2 GiB and more.  The product is cut on the host so that every piece stays inside that reach:
 * a K-contiguous operand by rows (row or column blocks of C, one launch each), an M- / N-contiguous operand, whose
 * rows are k, along the contraction (more segments of the same launch; cuts at multiples of 64 keep every piece's
 * 16-byte phase).  Returns true if it ran the product (status in *rc), false if nothing needs cutting or a cut is
 * not possible (more than HAP_GEMM_MAX_SEG pieces, unaligned leading dimensions): the caller goes on as before. */
static bool run_large(const hap_gemm_problem* p, void* stream, int* rc) {
  const int es = esize(p->in_dtype);
  if ((p->lda * es) % 16 || (p->ldb * es) % 16) return false;
  const double limit = (double)g_view_limit / es;       // elements
  const int64_t slack = 16;                              // skew and chunk rounding
  int64_t kmax = 0;
  for (int s = 0; s < p->nseg; ++s) kmax = p->k[s] > kmax ? p->k[s] : kmax;
  // rows r of pitch ld and width w with ((r - 1) * ld + w + slack) elements inside the reach
  auto rows_fit = [&](int64_t ld, int64_t w, int64_t granule) -> int64_t {
    const double r = (limit - (double)(w + slack)) / (double)ld;
    return r < (double)granule ? 0 : (int64_t)(r / granule) * granule;
  };
  auto too_big = [&](int64_t rows, int64_t ld, int64_t w) { return (double)(rows - 1) * ld + w + slack >= limit; };
  if (p->a_kcontig && too_big(p->M, p->lda, kmax)) {
    const int64_t r = rows_fit(p->lda, kmax, 256);
    if (r == 0) return false;
    ++g_cut_products;
    for (int64_t lo = 0; lo < p->M; lo += r) {
      const hap_gemm_problem q = sub_problem(p, lo, lo + r < p->M ? lo + r : p->M, 0, p->N, p->tile);
      if ((*rc = hap_gemm_run(&q, stream))) return true;
    }
    *rc = HAP_OK;
    return true;
  }
  if (p->b_kcontig && too_big(p->N, p->ldb, kmax)) {
    const int64_t r = rows_fit(p->ldb, kmax, 256);
    if (r == 0) return false;
    ++g_cut_products;
    for (int64_t lo = 0; lo < p->N; lo += r) {
      const hap_gemm_problem q = sub_problem(p, 0, p->M, lo, lo + r < p->N ? lo + r : p->N, p->tile);
      if ((*rc = hap_gemm_run(&q, stream))) return true;
    }
    *rc = HAP_OK;
    return true;
  }
  bool cut = false;
  for (int s = 0; s < p->nseg; ++s)
    cut = cut || (!p->a_kcontig && too_big(p->k[s], p->lda, p->M)) || (!p->b_kcontig && too_big(p->k[s], p->ldb, p->N));
  if (!cut) return false;
  int64_t piece = INT64_MAX;
  if (!p->a_kcontig) piece = rows_fit(p->lda, p->M, 64);
  if (!p->b_kcontig) { const int64_t r = rows_fit(p->ldb, p->N, 64); piece = r < piece ? r : piece; }
  if (piece == 0) return false;
  hap_gemm_problem q = *p;
  q.nseg = 0;
  for (int s = 0; s < p->nseg; ++s)
    for (int64_t k0 = 0; k0 < p->k[s]; k0 += piece) {
      if (q.nseg == HAP_GEMM_MAX_SEG) return false;
      q.a[q.nseg] = static_cast<const char*>(p->a[s]) + (p->a_kcontig ? k0 : k0 * p->lda) * es;
      q.b[q.nseg] = static_cast<const char*>(p->b[s]) + (p->b_kcontig ? k0 : k0 * p->ldb) * es;
      q.k[q.nseg] = p->k[s] - k0 < piece ? p->k[s] - k0 : piece;
      ++q.nseg;
    }
  if (q.nseg == 0) return false;
  ++g_cut_products;
  *rc = hap_gemm_run(&q, stream);
  return true;
}

/* 256x256 tiles on 256 CUs quantise badly: 33 tile columns of 32 rows are 4.1 rounds of work that take
 * 5.  The engine therefore cuts the output into a part whose big tiles fill whole rounds and a
 * remainder strip computed with 128x128 tiles, when its cost model says that is faster. */
static int run_auto_tiled(const hap_gemm_problem* p, const Plan& pl, void* stream) {
  const int kCUs = cu_count();
  const long long Mp = p->M + pl.skewM, Np = p->N + pl.skewN;
  const long long tm = cdiv(Mp, 256), tn = cdiv(Np, 256);
  const long long sm = cdiv(Mp, 128), sn = cdiv(Np, 128);
  // A remainder strip of r big tiles can also stay on big tiles with its K range split over the idle CUs
  // (needs workspace); that costs about a third of a round for the partial-tile traffic plus 1/g rounds.
  const bool can_split_k = p->ws && p->ws_bytes >= (size_t)8 << 20;
  long long nk = 0;                 // K tiles of the contraction
  for (int s = 0; s < p->nseg; ++s) nk += p->k[s] > 0 ? cdiv(pl.skewK + p->k[s], 64) : 0;
  // A part whose big tiles cannot fill the chip: 128-tiles (two per CU) or 256-tiles, either with the K range split over
  // the idle slots as the launcher will do it.  Measured on this chip (microseconds): a workgroup spends 2.0 per K tile
  // on a 256-tile and 1.05 on a 128-tile that shares its CU, plus 7 / 5 for prologue and epilogue; a split costs 3 for
  // the reduction launch and 0.025 / 0.00625 per partial tile written and read back.  Returned in rounds of big tiles.
  auto few_tiles_us = [&](long long tiles, long long slots, double per_ktile, double fixed, double per_partial) {
    long long g = can_split_k ? slots / tiles : 1;
    if (g > nk / 4) g = nk / 4;
    if (g > 16) g = 16;
    if (g < 1) g = 1;
    const double rounds = (double)cdiv(tiles * g, slots);
    return rounds * ((double)nk / (double)g * per_ktile + fixed) + (g > 1 ? 3.0 + (double)(tiles * g) * per_partial : 0.0);
  };
  auto strip_time = [&](long long big_tiles, long long small_tiles, int* tile) {
    if (big_tiles < kCUs && nk > 0) {
      const double round_us = (double)nk * 2.0 + 7.0;
      const double tb = few_tiles_us(big_tiles, kCUs, 2.0, 7.0, 0.025), ts = few_tiles_us(small_tiles, 2 * kCUs, 1.05, 5.0, 0.00625);
      *tile = tb <= ts ? 256 : 128;
      return (tb <= ts ? tb : ts) / round_us;
    }
    *tile = 128;
    return small_tiles_time(small_tiles);
  };
  double best = (double)cdiv(tm * tn, kCUs);
  int choice = 0;                 // 0: all big, 1: all small, 2: split columns, 3: split rows
  int strip_tile = 128;
  long long cut = 0;
  if (tm * tn < kCUs) {           // cannot fill the chip: small tiles, or big tiles with split-K (chosen at launch)
    int tl;
    const double t = strip_time(tm * tn, sm * sn, &tl);
    if (t < best - 1e-9) { best = t; choice = tl == 128 ? 1 : 0; }
  } else {
    const double all_small = small_tiles_time(sm * sn);
    if (all_small < best - 1e-9) { best = all_small; choice = 1; }
  }
  // a plan of two launches pays for the second one: the strip starts when the last big tile has finished (~10 us)
  const double second_launch = nk > 0 ? 10.0 / ((double)nk * 2.0 + 7.0) : 0.0;
  for (long long c = tn - 1; c >= 1; --c)
    if ((tm * c) % kCUs == 0) {
      int tl;
      const double t = (double)(tm * c / kCUs) + strip_time(tm * (tn - c), sm * cdiv(Np - c * 256, 128), &tl) + second_launch;
      if (t < best - 1e-9) { best = t; choice = 2; cut = c; strip_tile = tl; }
      break;
    }
  for (long long r = tm - 1; r >= 1; --r)
    if ((tn * r) % kCUs == 0) {
      int tl;
      const double t = (double)(tn * r / kCUs) + strip_time(tn * (tm - r), sn * cdiv(Mp - r * 256, 128), &tl) + second_launch;
      if (t < best - 1e-9) { best = t; choice = 3; cut = r; strip_tile = tl; }
      break;
    }
  hap_gemm_problem q;
  int rc;
  switch (choice) {
    case 1:
      q = sub_problem(p, 0, p->M, 0, p->N, 128);
      return hap_gemm_run(&q, stream);
    case 2: {
      const int64_t n_cut = cut * 256 - pl.skewN;
      q = sub_problem(p, 0, p->M, 0, n_cut, 256);
      if ((rc = hap_gemm_run(&q, stream))) return rc;
      q = sub_problem(p, 0, p->M, n_cut, p->N, strip_tile);
      return hap_gemm_run(&q, stream);
    }
    case 3: {
      const int64_t m_cut = cut * 256 - pl.skewM;
      q = sub_problem(p, 0, m_cut, 0, p->N, 256);
      if ((rc = hap_gemm_run(&q, stream))) return rc;
      q = sub_problem(p, m_cut, p->M, 0, p->N, strip_tile);
      return hap_gemm_run(&q, stream);
    }
    default:
      q = sub_problem(p, 0, p->M, 0, p->N, 256);
      return hap_gemm_run(&q, stream);
  }
}

int hap_gemm_run(const hap_gemm_problem* p, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (p->M <= 0 || p->N <= 0) return HAP_OK;
  if (p->M > 0x7fffffff || p->N > 0x7fffffff) return hap_fail(HAP_EUNSUPPORTED, "GEMM extent exceeds 2^31");
  if (p->accumulate && p->c_dtype != HAP_F32) return hap_fail(HAP_EINVAL, "accumulate needs an fp32 output");
  if (p->in_dtype == HAP_F32 && p->c_dtype != HAP_F32) return hap_fail(HAP_EUNSUPPORTED, "fp32 inputs need fp32 output");
  if (p->dact != HAP_ACT_NONE) {
    if (p->dact != HAP_ACT_GELU_ERF || !p->dact_preact) return hap_fail(HAP_EINVAL, "bad activation backward in the epilogue (dact %d)", p->dact);
    if (p->act != HAP_ACT_NONE || p->accumulate || p->preact || p->bias)
      return hap_fail(HAP_EINVAL, "an epilogue with an activation backward has no bias, activation, pre-activation copy or accumulation");
  }
  const int es = esize(p->in_dtype), ces_out = esize(p->c_dtype);
  const int groups = p->groups > 1 ? p->groups : 1;
  const bool grouped = groups > 1 || p->group_len;
  if (grouped) {
    if (p->nseg != 1) return hap_fail(HAP_EINVAL, "a grouped product has one contracted segment");
    if (groups > 65535) return hap_fail(HAP_EUNSUPPORTED, "more than 65535 groups");
    if (p->group_len && p->group_ragged != 1 && p->group_ragged != 2) return hap_fail(HAP_EINVAL, "group_len needs group_ragged 1 or 2");
    if (p->k[0] > 0x7fffffff) return hap_fail(HAP_EUNSUPPORTED, "segment longer than 2^31");
  }
  const int ragged = p->group_len ? p->group_ragged : 0;
  if (!grouped && !p->force_generic) {
    int rc;
    if (run_large(p, stream, &rc)) return rc;
  }
  if (skinny_f32_applies(p)) {
    SkinnyArgs g;
    g.M = (int)p->M; g.N = (int)p->N; g.K = (int)p->k[0];
    g.lda = p->lda; g.ldb = p->ldb; g.ldc = p->ldc; g.ldp = p->ldp;
    g.a = static_cast<const float*>(p->a[0]); g.b = static_cast<const float*>(p->b[0]);
    g.c = static_cast<float*>(p->c); g.preact = static_cast<float*>(p->preact); g.bias = static_cast<const float*>(p->bias);
    g.act = p->act; g.accumulate = p->accumulate;
    const dim3 grid((unsigned)((p->N + 15) / 16));
    if (p->b_kcontig) hipLaunchKernelGGL(gemm_skinny_f32_kernel<true>, grid, dim3(1024), 0, st, g);
    else hipLaunchKernelGGL(gemm_skinny_f32_kernel<false>, grid, dim3(1024), 0, st, g);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "skinny fp32 gemm launch: %s", hipGetErrorString(e));
    return HAP_OK;
  }
  const Plan pl = make_plan(p);
  if (pl.tiled && pl.dma && p->tile == 0 && pl.bm == 256 && !grouped) return run_auto_tiled(p, pl, stream);

  if (!pl.tiled) {
    GenericArgs g;
    g.M = (int)p->M; g.N = (int)p->N; g.nseg = 0;
    g.lda = p->lda; g.ldb = p->ldb; g.ldc = p->ldc; g.ldp = p->ldp;
    g.a_kcontig = p->a_kcontig; g.b_kcontig = p->b_kcontig;
    g.c = p->c; g.preact = p->preact; g.bias = p->bias; g.act = p->act; g.accumulate = p->accumulate;
    g.dact_preact = p->dact ? p->dact_preact : nullptr; g.ldd = p->ldd;
    g.ragged = ragged; g.group_len = p->group_len;
    g.ga = p->ga * es; g.gb = p->gb * es; g.gc = p->gc * ces_out; g.gp = p->gp * ces_out; g.gbias = p->gbias * es; g.gd = p->gd * ces_out;
    for (int s = 0; s < p->nseg; ++s) {
      if (p->k[s] <= 0) continue;
      if (p->k[s] > 0x7fffffff) return hap_fail(HAP_EUNSUPPORTED, "segment longer than 2^31");
      g.a[g.nseg] = p->a[s]; g.b[g.nseg] = p->b[s]; g.k[g.nseg] = (int)p->k[s]; ++g.nseg;
    }
    dim3 grid((unsigned)((p->N + 15) / 16), (unsigned)((p->M + 15) / 16), (unsigned)groups);
    if (grid.y > 65535u) return hap_fail(HAP_EUNSUPPORTED, "generic GEMM fallback: too many rows");
    if (p->in_dtype == HAP_BF16 && p->c_dtype == HAP_BF16) hipLaunchKernelGGL((gemm_generic_kernel<__bf16, __bf16>), grid, dim3(256), 0, st, g);
    else if (p->in_dtype == HAP_BF16) hipLaunchKernelGGL((gemm_generic_kernel<__bf16, float>), grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL((gemm_generic_kernel<float, float>), grid, dim3(256), 0, st, g);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hap_fail(HAP_EDEVICE, "generic gemm launch: %s", hipGetErrorString(e));
    return HAP_OK;
  }

  GemmArgs a;
  a.M = (int)p->M; a.N = (int)p->N;
  a.skewM = pl.skewM; a.skewN = pl.skewN; a.skewK = pl.skewK;
  a.lda = p->lda; a.ldb = p->ldb; a.ldc = p->ldc; a.ldp = p->ldp;
  a.c = p->c; a.preact = p->preact; a.bias = p->bias; a.act = p->act; a.accumulate = p->accumulate;
  a.dact_preact = p->dact ? p->dact_preact : nullptr; a.ldd = p->ldd;
  a.ragged = ragged; a.group_len = p->group_len;
  a.ga = p->ga * es; a.gb = p->gb * es; a.gc = p->gc * ces_out; a.gp = p->gp * ces_out; a.gbias = p->gbias * es; a.gd = p->gd * ces_out;
  a.tiles_m = (int)((p->M + pl.skewM + pl.bm - 1) / pl.bm);
  a.tiles_n = (int)((p->N + pl.skewN + pl.bn - 1) / pl.bn);
  a.nseg = 0;
  for (int s = 0; s < p->nseg; ++s) {
    if (p->k[s] <= 0) continue;
    SegArg& sg = a.seg[a.nseg++];
    const int skew_a = p->a_kcontig ? pl.skewK : pl.skewM, skew_b = p->b_kcontig ? pl.skewK : pl.skewN;
    sg.a = static_cast<const char*>(p->a[s]) - (size_t)skew_a * es;
    sg.b = static_cast<const char*>(p->b[s]) - (size_t)skew_b * es;
    sg.k = (int)p->k[s];
    const long long ea = p->a_kcontig ? ((p->M - 1) * p->lda + pl.skewK + p->k[s]) : ((p->k[s] - 1) * p->lda + pl.skewM + p->M);
    const long long eb = p->b_kcontig ? ((p->N - 1) * p->ldb + pl.skewK + p->k[s]) : ((p->k[s] - 1) * p->ldb + pl.skewN + p->N);
    // Extents are rounded up to whole 16-byte chunks: the hardware range check works per dword, and
    // a chunk that starts inside the view must come back whole (its tail is discarded by the kernel).
    // An aligned chunk never crosses a page, so the bytes past the view are still mapped memory.
    sg.a_bytes = (unsigned)((ea * es + 15) / 16 * 16);
    sg.b_bytes = (unsigned)((eb * es + 15) / 16 * 16);
    sg.pad = 0;
  }
  if (a.nseg == 0) {   // empty contraction: the product is zero; run one empty segment so the epilogue still applies
    a.nseg = 1;
    a.seg[0].a = p->c; a.seg[0].b = p->c; a.seg[0].k = 0; a.seg[0].a_bytes = 0; a.seg[0].b_bytes = 0; a.seg[0].pad = 0;
  }
  {
    // Whole-chunk stores need rows of C (and of the pre-activation copy, with C's phase) that start on the same 16-byte phase;
    // the phase itself is arbitrary: cdelta shifts the tile inside the store patch onto C's chunk grid.
    const int ces = esize(p->c_dtype), cepc = 16 / ces;
    a.vec_store = ((uintptr_t)p->c % ces) == 0 && p->ldc % cepc == 0 &&
                  (!p->preact || (((uintptr_t)p->preact % 16) == ((uintptr_t)p->c % 16) && p->ldp % cepc == 0)) &&
                  (groups == 1 || (p->gc % cepc == 0 && (!p->preact || p->gp % cepc == 0))) &&
                  (!(p->dact && p->dact_preact) || (((uintptr_t)p->dact_preact % 16) == ((uintptr_t)p->c % 16) && p->ldd % cepc == 0 &&
                                                    (groups == 1 || p->gd % cepc == 0)));
    const int skew_c = (int)(((uintptr_t)p->c % 16) / ces);       // columns of C's 16-byte chunk that precede logical column 0
    a.cdelta = a.vec_store ? ((skew_c - pl.skewN) % cepc + cepc) % cepc : 0;
  }
  a.ntiles = 0;
  a.ksplit = 1;
  a.partial = nullptr;
  {
    const int bk = pl.bk;                // the chosen kernel's K step
    for (int s = 0; s < a.nseg; ++s) a.ntiles += (pl.skewK + a.seg[s].k + bk - 1) / bk;
    if (a.ntiles == 0) a.ntiles = 1;     // empty contraction still runs one (all-zero) tile
  }
  if (pl.dma || p->in_dtype == HAP_F32) {
    // Split-K when the output tiles cannot occupy the chip: spread each tile's K range over the idle CUs,
    // keeping at least 4 K tiles per workgroup (2 for the small fp32 tiles, whose loop is bound by one load
    // latency per tile), as far as the caller's workspace allows.
    const long long out_tiles = (long long)a.tiles_m * a.tiles_n * groups;
    const int kCUs = cu_count();
    const long long slots = pl.bm == 256 ? kCUs : (pl.bm == 128 ? 2 * kCUs : 4 * kCUs);
    const int min_tiles = pl.bm == 64 ? 2 : 4 * (64 / pl.bk);      // in K steps of the chosen kernel
    long long g = slots / out_tiles;
    if (g > a.ntiles / min_tiles) g = a.ntiles / min_tiles;
    if (g > 16) g = 16;
    const size_t per_split = (size_t)out_tiles * pl.bm * pl.bn * sizeof(float);
    if (g >= 2 && p->ws && per_split * 2 <= p->ws_bytes) {
      if (per_split * (size_t)g > p->ws_bytes) g = (long long)(p->ws_bytes / per_split);
      a.ksplit = (int)g;
      a.partial = static_cast<float*>(p->ws);
    }
  }
  if (p->in_dtype == HAP_BF16 && p->c_dtype == HAP_BF16) return dispatch_tile<__bf16, __bf16>(p, pl, a, groups, st);
  if (p->in_dtype == HAP_BF16) return dispatch_tile<__bf16, float>(p, pl, a, groups, st);
  return dispatch_tile<float, float>(p, pl, a, groups, st);
}
