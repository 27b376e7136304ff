// HBM-bound kernels of the DiLoCo outer step (paper Sec. 4.1 eqs. 2-3, Algorithm 1 lines
// after the inner loop, Algorithm 2 "compress parameter delta"):
//   * fused pseudogradient / K-way average / outer Nesterov / write-back,
//   * row-wise 4-bit linear quantiser of theta_g - theta_k (IEEE fp32, ties to even),
//   * dequantise + K-way average + outer update + write-back.
// The K worker replicas live on this GPU, so the average is a loop over K pointers
// in a fixed order: ((d_1 + d_2) + ...) * (1/K).
#include "common.h"

namespace mlc {
namespace {

constexpr int OT_THREADS = 256;

template <typename T> struct Ld;
template <> struct Ld<float> {
  static __device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    f32x4 a, b;
    a.x = v[0]; a.y = v[1]; a.z = v[2]; a.w = v[3]; b.x = v[4]; b.y = v[5]; b.z = v[6]; b.w = v[7];
    *reinterpret_cast<f32x4*>(p) = a;
    *reinterpret_cast<f32x4*>(p + 4) = b;
  }
  static __device__ __forceinline__ float load1(const float* p) { return *p; }
  static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
  static __device__ __forceinline__ float round(float v) { return v; }   // value as stored
};
template <> struct Ld<bf16_t> {
  static __device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(p);
    v[0] = bf16lo(w.x); v[1] = bf16hi(w.x); v[2] = bf16lo(w.y); v[3] = bf16hi(w.y);
    v[4] = bf16lo(w.z); v[5] = bf16hi(w.z); v[6] = bf16lo(w.w); v[7] = bf16hi(w.w);
  }
  static __device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
    u32x4 w;
    w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
    w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<u32x4*>(p) = w;
  }
  static __device__ __forceinline__ float load1(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store1(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

// eq. 3; theta comes back as the value the global buffer will hold after the store, so the
// write-back hands every worker exactly the new theta_g.
template <typename GT>
__device__ __forceinline__ void outer_update(float& theta, float& u, float psi, float eta, float mu,
                                             int nesterov) {
  const float step = eta * psi;
  u = mu * u + step;
  theta = Ld<GT>::round(nesterov ? theta - mu * u - step : theta - u);
}

// ---- unquantised fused outer step ---------------------------------------------------
template <typename WT, typename GT>
__global__ __launch_bounds__(OT_THREADS) void outer_fused_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, long n_elems, int K, float eta,
    float mu, float inv_k, int nesterov, int write_back) {
  const long n_vec = n_elems / 8;
  for (long i = (long)blockIdx.x * OT_THREADS + threadIdx.x; i < n_vec;
       i += (long)gridDim.x * OT_THREADS) {
    const long off = i * 8;
    float tg[8], uv[8], acc[8];
    Ld<GT>::load8(theta_g + off, tg);
    Ld<float>::load8(u + off, uv);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      float tk[8];
      Ld<WT>::load8(reinterpret_cast<const WT*>(w.p[k]) + off, tk);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += tg[j] - tk[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) outer_update<GT>(tg[j], uv[j], acc[j] * inv_k, eta, mu, nesterov);
    Ld<GT>::store8(theta_g + off, tg);
    Ld<float>::store8(u + off, uv);
    if (write_back)
      for (int k = 0; k < K; ++k) Ld<WT>::store8(reinterpret_cast<WT*>(w.p[k]) + off, tg);
  }
  // ragged tail (fewer than 8 elements), one thread each
  const long tail0 = n_vec * 8;
  const long t = tail0 + (long)blockIdx.x * OT_THREADS + threadIdx.x;
  if (t < n_elems) {
    float tg = Ld<GT>::load1(theta_g + t), uv = u[t], acc = 0.f;
    for (int k = 0; k < K; ++k) acc += tg - Ld<WT>::load1(reinterpret_cast<const WT*>(w.p[k]) + t);
    outer_update<GT>(tg, uv, acc * inv_k, eta, mu, nesterov);
    Ld<GT>::store1(theta_g + t, tg);
    u[t] = uv;
    if (write_back)
      for (int k = 0; k < K; ++k) Ld<WT>::store1(reinterpret_cast<WT*>(w.p[k]) + t, tg);
  }
}

// ---- row-wise 4-bit quantiser: one wavefront per row, all K workers ------------------
// Two passes over the row (absmax, then codes); the second pass re-reads data the first
// pass just pulled through L2.
__device__ __forceinline__ int quant_level(float delta, float scale) {
  float q = rintf(delta / scale);           // IEEE division, round half to even
  q = fminf(fmaxf(q, -7.f), 7.f);
  return (int)q;
}

template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void quantize_rows_kernel(
    WorkerPtrs w, const GT* __restrict__ theta_g, CodePtrs codes, ScalePtrs scales, long rows, int n,
    int K) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (OT_THREADS / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const GT* tg = theta_g + row * n;
  constexpr int W = VEC ? 8 : 2;            // elements per lane per step
  for (int k = 0; k < K; ++k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + row * n;
    float amax = 0.f;
    for (int c = lane * W; c < n; c += 64 * W) {
      float a[8], b[8];
      if (VEC) { Ld<GT>::load8(tg + c, a); Ld<WT>::load8(tk + c, b); }
      else { a[0] = Ld<GT>::load1(tg + c); a[1] = Ld<GT>::load1(tg + c + 1);
             b[0] = Ld<WT>::load1(tk + c); b[1] = Ld<WT>::load1(tk + c + 1); }
#pragma unroll
      for (int j = 0; j < W; ++j) amax = fmaxf(amax, fabsf(a[j] - b[j]));
    }
    amax = wave_max(amax);
    const float scale = amax / 7.0f;
    if (lane == 0) scales.p[k][row] = scale;
    uint8_t* crow = codes.p[k] + row * (long)(n / 2);
    for (int c = lane * W; c < n; c += 64 * W) {
      float a[8], b[8];
      if (VEC) { Ld<GT>::load8(tg + c, a); Ld<WT>::load8(tk + c, b); }
      else { a[0] = Ld<GT>::load1(tg + c); a[1] = Ld<GT>::load1(tg + c + 1);
             b[0] = Ld<WT>::load1(tk + c); b[1] = Ld<WT>::load1(tk + c + 1); }
      unsigned int packed = 0;
#pragma unroll
      for (int j = 0; j < W; ++j) {
        const int q = (amax > 0.f) ? quant_level(a[j] - b[j], scale) : 0;
        packed |= (unsigned int)(q + 8) << (4 * j);
      }
      if (VEC) *reinterpret_cast<unsigned int*>(crow + c / 2) = packed;
      else crow[c / 2] = (uint8_t)packed;
    }
  }
}

// Single-pass variant: a group of G threads (a wavefront or the whole workgroup) owns a row
// and keeps it in registers (NV vectors of 8 elements per thread), so theta_g is read once
// for all K workers and every theta_k exactly once.  Same arithmetic as above.
template <typename WT, typename GT, int NV, int G>
__global__ __launch_bounds__(OT_THREADS) void quantize_rows_reg_kernel(
    WorkerPtrs w, const GT* __restrict__ theta_g, CodePtrs codes, ScalePtrs scales, long rows, int n,
    int K) {
  constexpr int ROWS_PER_BLOCK = OT_THREADS / G;
  __shared__ float red[2][OT_THREADS / 64];
  const int t = threadIdx.x % G;
  const long row = (long)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / G;
  const bool live = row < rows;            // whole groups are live or not; no early return
  const long rbase = live ? row * n : 0;   // (the workgroup-wide barrier below needs everyone)
  float tg[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (t + i * G) * 8;
    if (live && c < n) Ld<GT>::load8(theta_g + rbase + c, tg[i]);
    else
#pragma unroll
      for (int j = 0; j < 8; ++j) tg[i][j] = 0.f;
  }
  for (int k = 0; k < K; ++k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + rbase;
    float d[NV][8];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        float b[8];
        Ld<WT>::load8(tk + c, b);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          d[i][j] = tg[i][j] - b[j];
          amax = fmaxf(amax, fabsf(d[i][j]));
        }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) d[i][j] = 0.f;
      }
    }
    amax = wave_max(amax);
    if constexpr (G > 64) {
      if ((threadIdx.x & 63) == 0) red[k & 1][threadIdx.x >> 6] = amax;
      __syncthreads();
      amax = fmaxf(fmaxf(red[k & 1][0], red[k & 1][1]), fmaxf(red[k & 1][2], red[k & 1][3]));
    }
    const float scale = amax / 7.0f;
    if (live && t == 0) scales.p[k][row] = scale;
    uint8_t* crow = codes.p[k] + row * (long)(n / 2);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        unsigned int packed = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int q = (amax > 0.f) ? quant_level(d[i][j], scale) : 0;
          packed |= (unsigned int)(q + 8) << (4 * j);
        }
        *reinterpret_cast<unsigned int*>(crow + c / 2) = packed;
      }
    }
  }
}

// Quantiser and outer update in one pass over a row held in registers: codes and scales are
// written as the stand-alone quantiser writes them, and the dequantised deltas go straight
// into the mean and eq. 3 without re-reading theta_g or the codes.
template <typename WT, typename GT, int NV, int G>
__global__ __launch_bounds__(OT_THREADS) void quantize_outer_rows_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, CodePtrs codes, ScalePtrs scales,
    long rows, int n, int K, float eta, float mu, float inv_k, int nesterov, int write_back) {
  constexpr int ROWS_PER_BLOCK = OT_THREADS / G;
  __shared__ float red[2][OT_THREADS / 64];
  const int t = threadIdx.x % G;
  const long row = (long)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / G;
  const bool live = row < rows;
  const long rbase = live ? row * n : 0;
  float tg[NV][8], acc[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (t + i * G) * 8;
    if (live && c < n) Ld<GT>::load8(theta_g + rbase + c, tg[i]);
    else
#pragma unroll
      for (int j = 0; j < 8; ++j) tg[i][j] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  }
  for (int k = 0; k < K; ++k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + rbase;
    float d[NV][8];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        float b[8];
        Ld<WT>::load8(tk + c, b);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          d[i][j] = tg[i][j] - b[j];
          amax = fmaxf(amax, fabsf(d[i][j]));
        }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) d[i][j] = 0.f;
      }
    }
    amax = wave_max(amax);
    if constexpr (G > 64) {
      if ((threadIdx.x & 63) == 0) red[k & 1][threadIdx.x >> 6] = amax;
      __syncthreads();
      amax = fmaxf(fmaxf(red[k & 1][0], red[k & 1][1]), fmaxf(red[k & 1][2], red[k & 1][3]));
    }
    const float scale = amax / 7.0f;
    if (live && t == 0) scales.p[k][row] = scale;
    uint8_t* crow = codes.p[k] + row * (long)(n / 2);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        unsigned int packed = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int q = (amax > 0.f) ? quant_level(d[i][j], scale) : 0;
          packed |= (unsigned int)(q + 8) << (4 * j);
          acc[i][j] += __fmul_rn((float)q, scale);
        }
        *reinterpret_cast<unsigned int*>(crow + c / 2) = packed;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (t + i * G) * 8;
    if (live && c < n) {
      float uv[8];
      Ld<float>::load8(u + rbase + c, uv);
#pragma unroll
      for (int j = 0; j < 8; ++j) outer_update<GT>(tg[i][j], uv[j], acc[i][j] * inv_k, eta, mu, nesterov);
      Ld<GT>::store8(theta_g + rbase + c, tg[i]);
      Ld<float>::store8(u + rbase + c, uv);
      if (write_back)
        for (int k = 0; k < K; ++k) Ld<WT>::store8(reinterpret_cast<WT*>(w.p[k]) + rbase + c, tg[i]);
    }
  }
}

// ---- dequantise + average + outer update --------------------------------------------
template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void dequant_outer_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, CodePtrs codes, ScalePtrs scales,
    long rows, int n, int K, float eta, float mu, float inv_k, int nesterov, int write_back) {
  constexpr int W = VEC ? 8 : 2;
  const int per_row = n / W;
  const long items = rows * per_row;
  for (long i = (long)blockIdx.x * OT_THREADS + threadIdx.x; i < items;
       i += (long)gridDim.x * OT_THREADS) {
    const long row = i / per_row;
    const int c = (int)(i - row * per_row) * W;
    const long off = row * n + c;
    float tg[8], uv[8], acc[8];
    if (VEC) { Ld<GT>::load8(theta_g + off, tg); Ld<float>::load8(u + off, uv); }
    else { tg[0] = Ld<GT>::load1(theta_g + off); tg[1] = Ld<GT>::load1(theta_g + off + 1);
           uv[0] = u[off]; uv[1] = u[off + 1]; }
#pragma unroll
    for (int j = 0; j < W; ++j) acc[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      const float sc = scales.p[k][row];
      const uint8_t* cp = codes.p[k] + row * (long)(n / 2) + c / 2;
      const unsigned int packed = VEC ? *reinterpret_cast<const unsigned int*>(cp) : (unsigned int)*cp;
#pragma unroll
      for (int j = 0; j < W; ++j) {
        const int q = (int)((packed >> (4 * j)) & 0xfu) - 8;
        acc[j] += __fmul_rn((float)q, sc);
      }
    }
#pragma unroll
    for (int j = 0; j < W; ++j) outer_update<GT>(tg[j], uv[j], acc[j] * inv_k, eta, mu, nesterov);
    if (VEC) {
      Ld<GT>::store8(theta_g + off, tg);
      Ld<float>::store8(u + off, uv);
      if (write_back)
        for (int k = 0; k < K; ++k) Ld<WT>::store8(reinterpret_cast<WT*>(w.p[k]) + off, tg);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        Ld<GT>::store1(theta_g + off + j, tg[j]);
        u[off + j] = uv[j];
        if (write_back)
          for (int k = 0; k < K; ++k) Ld<WT>::store1(reinterpret_cast<WT*>(w.p[k]) + off + j, tg[j]);
      }
    }
  }
}

int check_launch() { return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH; }

int cap_blocks(long blocks, long cap) {
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

double esize(int dtype) { return dtype == MLC_F32 ? 4.0 : 2.0; }

}  // namespace

#define MLC_DISPATCH2(WD, GD, CALL)                                  \
  do {                                                               \
    if ((WD) == MLC_F32 && (GD) == MLC_F32) { CALL(float, float); }  \
    else if ((WD) == MLC_BF16 && (GD) == MLC_F32) { CALL(bf16_t, float); } \
    else if ((WD) == MLC_BF16 && (GD) == MLC_BF16) { CALL(bf16_t, bf16_t); } \
    else { CALL(float, bf16_t); }                                    \
  } while (0)

int launch_outer_fused(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                       float* u, int64_t n_elems, int K, float eta_out, float mu, int nesterov,
                       int write_back, hipStream_t stream) {
  const long n_vec = n_elems / 8;
  const int blocks = cap_blocks((n_vec + OT_THREADS - 1) / OT_THREADS, 256 * 16);
  const double bytes = (double)n_elems * (K * esize(worker_dtype) * (write_back ? 2 : 1) +
                                          2 * esize(global_dtype) + 8);
  LaunchScope scope(MLC_KERNEL_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_CALL(WT, GT)                                                                          \
  hipLaunchKernelGGL((outer_fused_kernel<WT, GT>), dim3(blocks), dim3(OT_THREADS), 0, stream, w,  \
                     (GT*)theta_g, u, (long)n_elems, K, eta_out, mu, inv_k, nesterov, write_back)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

int launch_quantize(const WorkerPtrs& w, int worker_dtype, const void* theta_g, int global_dtype,
                    const CodePtrs& codes, const ScalePtrs& scales, int64_t rows, int64_t n, int K,
                    hipStream_t stream) {
  const long blocks = (rows + OT_THREADS / 64 - 1) / (OT_THREADS / 64);
  if (blocks > 0x7fffffffL) return MLC_ERR_SHAPE;
  const double bytes = (double)rows * n * (K * esize(worker_dtype) + esize(global_dtype) + 0.5 * K) +
                       (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_QUANTIZE, stream, 0.0, bytes);
  const bool vec = n % 8 == 0;
  // single-pass register kernel: a wavefront per row up to 2048 columns, a workgroup per row
  // up to 24576; otherwise (or for odd row lengths) the two-pass kernel
  if (vec && n <= 24576 && !(worker_dtype == MLC_F32 && global_dtype == MLC_BF16)) {
    const int g = n <= 2048 ? 64 : OT_THREADS;
    const int need = (int)((n + g * 8 - 1) / (g * 8));
    const int nv = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : need <= 8 ? 8 : 12;
    const long rpb = OT_THREADS / g;
    const long nblk = (rows + rpb - 1) / rpb;
#define MLC_QR(WT, GT, NV, G)                                                                     \
  hipLaunchKernelGGL((quantize_rows_reg_kernel<WT, GT, NV, G>), dim3((unsigned)nblk),              \
                     dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, codes, scales, (long)rows, \
                     (int)n, K)
#define MLC_QR_NV(WT, GT)                                                                         \
  do {                                                                                            \
    if (g == 64) { if (nv == 1) MLC_QR(WT, GT, 1, 64); else if (nv == 2) MLC_QR(WT, GT, 2, 64);   \
                   else MLC_QR(WT, GT, 4, 64); }                                                  \
    else { if (nv <= 2) MLC_QR(WT, GT, 2, 256); else if (nv == 4) MLC_QR(WT, GT, 4, 256);         \
           else if (nv == 8) MLC_QR(WT, GT, 8, 256); else MLC_QR(WT, GT, 12, 256); }              \
  } while (0)
    if (worker_dtype == MLC_BF16 && global_dtype == MLC_F32) MLC_QR_NV(bf16_t, float);
    else if (worker_dtype == MLC_BF16) MLC_QR_NV(bf16_t, bf16_t);
    else MLC_QR_NV(float, float);
#undef MLC_QR_NV
#undef MLC_QR
    return check_launch();
  }
#define MLC_CALL(WT, GT)                                                                          \
  do {                                                                                            \
    if (vec)                                                                                      \
      hipLaunchKernelGGL((quantize_rows_kernel<WT, GT, true>), dim3((unsigned)blocks),            \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, codes, scales,       \
                         (long)rows, (int)n, K);                                                  \
    else                                                                                          \
      hipLaunchKernelGGL((quantize_rows_kernel<WT, GT, false>), dim3((unsigned)blocks),           \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, codes, scales,       \
                         (long)rows, (int)n, K);                                                  \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

int launch_dequant_outer(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                         float* u, const CodePtrs& codes, const ScalePtrs& scales, int64_t rows,
                         int64_t n, int K, float eta_out, float mu, int nesterov, int write_back,
                         hipStream_t stream) {
  const bool vec = n % 8 == 0;
  const long items = rows * (n / (vec ? 8 : 2));
  const int blocks = cap_blocks((items + OT_THREADS - 1) / OT_THREADS, 256 * 16);
  const double bytes = (double)rows * n * (0.5 * K + 2 * esize(global_dtype) + 8 +
                                           (write_back ? K * esize(worker_dtype) : 0)) +
                       (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_DEQUANT_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_CALL(WT, GT)                                                                          \
  do {                                                                                            \
    if (vec)                                                                                      \
      hipLaunchKernelGGL((dequant_outer_kernel<WT, GT, true>), dim3(blocks), dim3(OT_THREADS), 0, \
                         stream, w, (GT*)theta_g, u, codes, scales, (long)rows, (int)n, K,        \
                         eta_out, mu, inv_k, nesterov, write_back);                               \
    else                                                                                          \
      hipLaunchKernelGGL((dequant_outer_kernel<WT, GT, false>), dim3(blocks), dim3(OT_THREADS), 0,\
                         stream, w, (GT*)theta_g, u, codes, scales, (long)rows, (int)n, K,        \
                         eta_out, mu, inv_k, nesterov, write_back);                               \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

// Returns MLC_ERR_UNSUPPORTED when the one-pass kernel does not cover the request (the
// caller then runs the quantiser and the dequantising update as two launches).
int launch_quantize_outer_fused(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                                float* u, const CodePtrs& codes, const ScalePtrs& scales, int64_t rows,
                                int64_t n, int K, float eta_out, float mu, int nesterov, int write_back,
                                hipStream_t stream) {
  if (n % 8 || n > 16384 || (worker_dtype == MLC_F32 && global_dtype == MLC_BF16))
    return MLC_ERR_UNSUPPORTED;
  const int g = n <= 2048 ? 64 : OT_THREADS;
  const int need = (int)((n + g * 8 - 1) / (g * 8));
  const int nv = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
  const long rpb = OT_THREADS / g;
  const long nblk = (rows + rpb - 1) / rpb;
  if (nblk > 0x7fffffffL) return MLC_ERR_SHAPE;
  const double bytes = (double)rows * n * (K * esize(worker_dtype) * (write_back ? 2 : 1) + 0.5 * K +
                                           2 * esize(global_dtype) + 8) + (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_DEQUANT_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_QO(WT, GT, NV, G)                                                                     \
  hipLaunchKernelGGL((quantize_outer_rows_kernel<WT, GT, NV, G>), dim3((unsigned)nblk),            \
                     dim3(OT_THREADS), 0, stream, w, (GT*)theta_g, u, codes, scales, (long)rows,   \
                     (int)n, K, eta_out, mu, inv_k, nesterov, write_back)
#define MLC_QO_NV(WT, GT)                                                                         \
  do {                                                                                            \
    if (g == 64) { if (nv == 1) MLC_QO(WT, GT, 1, 64); else if (nv == 2) MLC_QO(WT, GT, 2, 64);   \
                   else MLC_QO(WT, GT, 4, 64); }                                                  \
    else { if (nv <= 2) MLC_QO(WT, GT, 2, 256); else if (nv == 4) MLC_QO(WT, GT, 4, 256);         \
           else MLC_QO(WT, GT, 8, 256); }                                                         \
  } while (0)
  if (worker_dtype == MLC_BF16 && global_dtype == MLC_F32) MLC_QO_NV(bf16_t, float);
  else if (worker_dtype == MLC_BF16) MLC_QO_NV(bf16_t, bf16_t);
  else MLC_QO_NV(float, float);
#undef MLC_QO_NV
#undef MLC_QO
  return check_launch();
}

}  // namespace mlc
