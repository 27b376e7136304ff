// Shared declarations of the MuLoCo HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/muloco.h"

namespace mlc {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(((unsigned int)v) << 16);
}
// fp32 -> bf16, round to nearest, ties to even (v_cvt_pk_bf16_f32 on gfx950).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
  f32x2_t v;
  v.x = lo;
  v.y = hi;
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu);
}
__device__ __forceinline__ float bf16lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(unsigned int w) { return __uint_as_float(w & 0xffff0000u); }

// 8 adjacent elements of a float or bf16 array <-> 8 floats (16-byte accesses: one for bf16,
// two for float; p is 16-byte aligned).
template <typename T> struct Vec8;
template <> struct Vec8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    f32x4 a, b;
    a.x = v[0]; a.y = v[1]; a.z = v[2]; a.w = v[3]; b.x = v[4]; b.y = v[5]; b.z = v[6]; b.w = v[7];
    *reinterpret_cast<f32x4*>(p) = a;
    *reinterpret_cast<f32x4*>(p + 4) = b;
  }
  // non-temporal variants (measured faster for the parameter update, slower for the
  // momentum pass and the outer step)
  static __device__ __forceinline__ void load_nt(const float* p, float (&v)[8]) {
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)),
                b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p + 4));
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store_nt(float* p, const float (&v)[8]) {
    f32x4 a, b;
    a.x = v[0]; a.y = v[1]; a.z = v[2]; a.w = v[3]; b.x = v[4]; b.y = v[5]; b.z = v[6]; b.w = v[7];
    __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(p));
    __builtin_nontemporal_store(b, reinterpret_cast<f32x4*>(p + 4));
  }
  static __device__ __forceinline__ float load1(const float* p) { return *p; }
  static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
  static __device__ __forceinline__ float round(float v) { return v; }   // value as stored
  // 8 values as they sit in memory (held back while earlier values are worked on)
  struct raw_t { f32x4 a, b; };
  static __device__ __forceinline__ raw_t load_raw(const float* p) {
    raw_t r;
    r.a = *reinterpret_cast<const f32x4*>(p);
    r.b = *reinterpret_cast<const f32x4*>(p + 4);
    return r;
  }
  static __device__ __forceinline__ void unpack(const raw_t& r, float (&v)[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
  }
};
template <> struct Vec8<bf16_t> {
  typedef u32x4 raw_t;
  static __device__ __forceinline__ void unpack(const u32x4& w, float (&v)[8]) {
    v[0] = bf16lo(w.x); v[1] = bf16hi(w.x); v[2] = bf16lo(w.y); v[3] = bf16hi(w.y);
    v[4] = bf16lo(w.z); v[5] = bf16hi(w.z); v[6] = bf16lo(w.w); v[7] = bf16hi(w.w);
  }
  static __device__ __forceinline__ u32x4 pack(const float (&v)[8]) {
    u32x4 w;
    w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
    w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
    return w;
  }
  static __device__ __forceinline__ raw_t load_raw(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) { unpack(load_raw(p), v); }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    *reinterpret_cast<u32x4*>(p) = pack(v);
  }
  static __device__ __forceinline__ void load_nt(const bf16_t* p, float (&v)[8]) {
    unpack(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)), v);
  }
  static __device__ __forceinline__ void store_nt(bf16_t* p, const float (&v)[8]) {
    __builtin_nontemporal_store(pack(v), reinterpret_cast<u32x4*>(p));
  }
  static __device__ __forceinline__ float load1(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store1(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off, 64));
  return v;
}

static inline int64_t round_up(int64_t x, int64_t to) { return (x + to - 1) / to * to; }

// Per-device host-side caches (kernel attributes, unit counts) are arrays of this many slots.
constexpr int MAX_DEVICES = 64;
// Index of the current device in such a cache, or -1 when it has no slot.
static inline int device_slot() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return -1;
  return dev;
}

// ---- timing recorder -------------------------------------------------------------
struct LaunchScope {
  LaunchScope(int family, hipStream_t stream, double flops, double bytes);
  ~LaunchScope();
  int slot;
  hipStream_t stream;
};

// ---- batched bf16 GEMM of Newton-Schulz (ns_gemm.hip) ------------------------------
// D[b] = alpha_b * op(A[b]) * op(B[b])^T + beta * C[b] + gamma * I, all bf16, fp32 accum.
// Operand A is M x K, operand B is N x K.  An operand is either K-contiguous (element
// (i,k) at ptr[i*ld + k]) or K-strided (element (i,k) at ptr[k*ld + i]).
// M, N and K must be multiples of 128; all leading dimensions and batch
// strides multiples of 8 elements.
struct GemmDesc {
  const bf16_t* A; int64_t lda, strideA; int a_kstrided;
  const bf16_t* B; int64_t ldb, strideB; int b_kstrided;
  bf16_t* D; int64_t ldd, strideD;
  const bf16_t* C; int64_t ldc, strideC;   // may be null (beta ignored)
  int M, N, K, batch;
  float alpha, beta, gamma;
  const float* bscale;   // optional per-batch factor
  int bscale_pow;        // alpha_b = alpha * bscale[b]^bscale_pow (pow in {1,2})
  int symmetric;         // the result is symmetric (M == N): compute the lower triangle of
                         // tiles and store each off-diagonal tile twice
};
int launch_ns_gemm(const GemmDesc& d, hipStream_t stream);
// n independent products (n <= 64).  Those of equal depth K that use the large tile and the
// same kind of epilogue share launches, up to three at a time; each result is what
// launch_ns_gemm gives for that product, bit for bit.
int launch_ns_gemm_set(const GemmDesc* d, int n, hipStream_t stream);

// ---- whole Newton-Schulz chain of a small matrix in one workgroup (ns_chain_small.hip) ----
// Fits when the padded short side is 128 and the padded long side at most 512.
bool ns_chain_small_fits(int64_t mp, int64_t np);
// in/out: [count] padded mp x np bf16 matrices, row pitch ld, batch stride `stride`
// (elements); partials: per matrix nblk partial sums of squares of the input, from which the
// kernel forms 1 / (norm + eps); iters >= 1.  in == out is allowed.
int launch_ns_chain_small(const bf16_t* in, bf16_t* out, int64_t ld, int64_t stride, int64_t mp,
                          int64_t np, const float* partials, int nblk, float eps, int64_t count,
                          int iters, float a, float b, float c, hipStream_t stream);

// ---- elementwise kernels of the inner step (inner_elementwise.hip) ----------------
int launch_momentum(const void* grad, int grad_dtype, float* mom, bf16_t* U, float* partials,
                    int nblk, int64_t count, int64_t m, int64_t n, int64_t mp, int64_t np,
                    int64_t ldx, float beta, int nesterov, hipStream_t stream);
int launch_ns_load(const void* in, int dtype, bf16_t* U, float* partials, int nblk,
                   int64_t count, int64_t m, int64_t n, int64_t mp, int64_t np, int64_t ldx,
                   hipStream_t stream);
int launch_norm_finalize(const float* partials, int nblk, float* scale, int64_t count,
                         float eps, hipStream_t stream);
int launch_param_update(void* W, int dtype, const bf16_t* O, const float* oscale,
                        int64_t count, int64_t m, int64_t n, int64_t mp, int64_t ldx,
                        float decay_factor, float step, hipStream_t stream);
int launch_ns_store(const bf16_t* X, const float* oscale, void* out, int dtype, int64_t count,
                    int64_t m, int64_t n, int64_t mp, int64_t ldx, hipStream_t stream);

int launch_adamw(void* theta, int param_dtype, const void* grad, int grad_dtype, float* m, float* v,
                 int64_t n, float lr, float b1, float b2, float eps, float decay, float c1, float c2,
                 hipStream_t stream);

// ---- outer step kernels (outer.hip) ----------------------------------------------
struct WorkerPtrs { void* p[MLC_MAX_WORKERS]; };
struct CodePtrs { uint8_t* p[MLC_MAX_WORKERS]; };
struct ScalePtrs { float* p[MLC_MAX_WORKERS]; };
int launch_outer_fused(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                       float* u, int64_t n_elems, int K, float eta_out, float mu, int nesterov,
                       int write_back, hipStream_t stream);
// residual (error-feedback) accumulators per worker; all null = no error feedback
struct ResidualPtrs { float* p[MLC_MAX_WORKERS]; };
// Several groups in one launch: at most this many groups and workers (their table travels
// in the kernel arguments).
constexpr int OUTER_MAX_SEG = 4;
constexpr int OUTER_MAX_SEG_K = 8;
struct OuterGroupArgs {
  WorkerPtrs w; CodePtrs codes; ScalePtrs scales; ScalePtrs offsets; ResidualPtrs ef;
  void* theta_g; float* u; int64_t rows, n;
};
// >= 0 when the one-pass quantiser covers rows of length n; rows up to 8192 columns
// (configurations 0 .. QUANT_MULTI_MAX_CFG) can share a launch with other groups, longer ones
// need so many registers per thread that they would halve the occupancy of the whole launch.
int quant_reg_cfg(int64_t n);
constexpr int QUANT_MULTI_MAX_CFG = 4;
struct QuantForm;
int launch_outer_fused_multi(const OuterGroupArgs* gs, int ng, int worker_dtype, int global_dtype, int K,
                             float eta_out, float mu, int nesterov, int write_back, hipStream_t stream);
int launch_quantize_outer_multi(const OuterGroupArgs* gs, int ng, int worker_dtype, int global_dtype, int K,
                                const QuantForm& form, float eta_out, float mu, int nesterov, int write_back,
                                hipStream_t stream);
// Radix-select state of one (worker, matrix) pair of the top-k sparsifier.
constexpr int TOPK_BINS = 2048;     // widest digit of the radix select: 11 bits
struct TopkState { unsigned int hist[TOPK_BINS]; unsigned int prefix, mask, rank, pad; };
size_t topk_workspace_bytes(int64_t count, int K);
// thresholds: per worker [count] floats (may be null): the k-th largest magnitude found.
int launch_topk_outer(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype, float* u,
                      const ResidualPtrs& ef, const ScalePtrs& thresholds, int64_t count, int64_t m,
                      int64_t n, int K, unsigned int kcount, float ef_beta, float eta_out, float mu,
                      int nesterov, int write_back, void* workspace, hipStream_t stream);
// Form of the linear quantiser (see muloco.h).
struct QuantForm {
  int bits;              // 2, 4 or 8
  int offset;            // 0: range [-amax, amax]; 1: range [min, max], stored with an offset
  int rows_per_range;    // 0: one range per row; m: one range per matrix of m rows
  float levels;          // 2^(bits-1) - 1 without offset, 2^bits - 1 with
  int code_bias;         // stored code = level + code_bias: 2^(bits-1) without offset, 0 with
  float ef_beta;         // decay of the error-feedback residual
};
QuantForm make_quant_form(int bits, int offset, int64_t rows_per_range, float ef_beta);
// per-worker lower ends of the ranges (offset form); all null otherwise
typedef ScalePtrs OffsetPtrs;
// Ranges per matrix, written to scales (and offsets) ahead of the quantiser proper.
int launch_matrix_ranges(const WorkerPtrs& w, int worker_dtype, const void* theta_g, int global_dtype,
                         const ScalePtrs& scales, const OffsetPtrs& offsets, const ResidualPtrs& ef,
                         int64_t count, int64_t m, int64_t n, int K, const QuantForm& form,
                         hipStream_t stream);
int launch_quantize(const WorkerPtrs& w, int worker_dtype, const void* theta_g, int global_dtype,
                    const CodePtrs& codes, const ScalePtrs& scales, const OffsetPtrs& offsets,
                    const ResidualPtrs& ef, int64_t rows, int64_t n, int K, const QuantForm& form,
                    hipStream_t stream);
// mean_*: outputs of the second quantisation (requant != 0), each may be null.
int launch_quantize_outer_fused(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                                float* u, const CodePtrs& codes, const ScalePtrs& scales,
                                const OffsetPtrs& offsets, const ResidualPtrs& ef, int64_t rows,
                                int64_t n, int K, const QuantForm& form, float eta_out, float mu,
                                int nesterov, int write_back, int requant, uint8_t* mean_codes,
                                float* mean_scales, float* mean_offsets, hipStream_t stream);
int launch_dequant_outer(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                         float* u, const CodePtrs& codes, const ScalePtrs& scales,
                         const OffsetPtrs& offsets, int64_t rows, int64_t n, int K,
                         const QuantForm& form, float eta_out, float mu, int nesterov,
                         int write_back, hipStream_t stream);

}  // namespace mlc
