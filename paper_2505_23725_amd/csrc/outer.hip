// HBM-bound kernels of the DiLoCo outer step (paper Sec. 4.1 eqs. 2-3, Algorithm 1 lines
// after the inner loop, Algorithm 2 "compress parameter delta"):
//   * fused pseudogradient / K-way average / outer Nesterov / write-back,
//   * row-wise 2/4/8-bit linear quantiser of theta_g - theta_k (IEEE fp32, ties to even),
//     optionally with error feedback (Algorithm 2, EF branch),
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

// ---- row-wise linear quantiser (Sec. 2 "Compressed Communication"; Algorithm 2) --------
// bits = 2, 4 or 8: levels -qmax..qmax with qmax = 2^(bits-1) - 1, code = level + 2^(bits-1),
// 8 / bits codes per byte with the lowest column in the lowest bits.  With error feedback
// the value quantised is e = fl32(fl32(beta * E) + delta) and the residual becomes
// E <- fl32(e - level * scale); both are fixed in fp32 (no fused multiply-add) so that codes
// and residuals are reproducible bit for bit.
__device__ __forceinline__ int quant_level(float v, float scale, float qmax) {
  float q = rintf(v / scale);               // IEEE division, round half to even
  q = fminf(fmaxf(q, -qmax), qmax);
  return (int)q;
}

__device__ __forceinline__ float ef_input(float delta, float residual, float beta) {
  return __fadd_rn(__fmul_rn(beta, residual), delta);
}

// 8 adjacent levels of a row, first column c (a multiple of 8) <-> bits bytes of its codes
__device__ __forceinline__ void store_codes8(uint8_t* crow, int c, const int (&q)[8], int bits) {
  if (bits == 4) {
    unsigned int p = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) p |= (unsigned int)(q[j] + 8) << (4 * j);
    *reinterpret_cast<unsigned int*>(crow + c / 2) = p;
  } else if (bits == 8) {
    u32x2 p = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p.x |= (unsigned int)(q[j] + 128) << (8 * j);
      p.y |= (unsigned int)(q[j + 4] + 128) << (8 * j);
    }
    *reinterpret_cast<u32x2*>(crow + c) = p;
  } else {
    unsigned int p = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) p |= (unsigned int)(q[j] + 2) << (2 * j);
    *reinterpret_cast<unsigned short*>(crow + c / 4) = (unsigned short)p;
  }
}

__device__ __forceinline__ void load_levels8(const uint8_t* crow, int c, int (&q)[8], int bits) {
  if (bits == 4) {
    const unsigned int p = *reinterpret_cast<const unsigned int*>(crow + c / 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (int)((p >> (4 * j)) & 0xfu) - 8;
  } else if (bits == 8) {
    const u32x2 p = *reinterpret_cast<const u32x2*>(crow + c);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      q[j] = (int)((p.x >> (8 * j)) & 0xffu) - 128;
      q[j + 4] = (int)((p.y >> (8 * j)) & 0xffu) - 128;
    }
  } else {
    const unsigned int p = *reinterpret_cast<const unsigned short*>(crow + c / 4);
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (int)((p >> (2 * j)) & 0x3u) - 2;
  }
}

// Two passes over the row (absmax, then codes), one wavefront per row, all K workers; the
// second pass re-reads data the first pass just pulled through L2.  Rows whose length is
// not a multiple of 8 go one code byte (8 / bits columns) per lane and step.
template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void quantize_rows_kernel(
    WorkerPtrs w, const GT* __restrict__ theta_g, CodePtrs codes, ScalePtrs scales, ResidualPtrs ef,
    long rows, int n, int K, int bits, float qmax, float ef_beta) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (OT_THREADS / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const GT* tg = theta_g + row * n;
  const int W = VEC ? 8 : 8 / bits;         // elements per lane per step
  const long row_bytes = (long)n * bits / 8;
  for (int k = 0; k < K; ++k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + row * n;
    float* res = ef.p[k] ? ef.p[k] + row * n : nullptr;
    float amax = 0.f;
    for (int c = lane * W; c < n; c += 64 * W) {
      float a[8], b[8], e[8];
      if (VEC) {
        Ld<GT>::load8(tg + c, a); Ld<WT>::load8(tk + c, b);
        if (res) Ld<float>::load8(res + c, e);
      } else {
        for (int j = 0; j < W; ++j) {
          a[j] = Ld<GT>::load1(tg + c + j); b[j] = Ld<WT>::load1(tk + c + j);
          if (res) e[j] = res[c + j];
        }
      }
      for (int j = 0; j < W; ++j) {
        const float d = a[j] - b[j];
        amax = fmaxf(amax, fabsf(res ? ef_input(d, e[j], ef_beta) : d));
      }
    }
    amax = wave_max(amax);
    const float scale = amax / qmax;
    if (lane == 0) scales.p[k][row] = scale;
    uint8_t* crow = codes.p[k] + row * row_bytes;
    for (int c = lane * W; c < n; c += 64 * W) {
      float a[8], b[8], e[8];
      if (VEC) {
        Ld<GT>::load8(tg + c, a); Ld<WT>::load8(tk + c, b);
        if (res) Ld<float>::load8(res + c, e);
      } else {
        for (int j = 0; j < W; ++j) {
          a[j] = Ld<GT>::load1(tg + c + j); b[j] = Ld<WT>::load1(tk + c + j);
          if (res) e[j] = res[c + j];
        }
      }
      int q[8];
      for (int j = 0; j < W; ++j) {
        const float d = a[j] - b[j];
        const float v = res ? ef_input(d, e[j], ef_beta) : d;
        q[j] = (amax > 0.f) ? quant_level(v, scale, qmax) : 0;
        e[j] = __fsub_rn(v, __fmul_rn((float)q[j], scale));
      }
      if (VEC) {
        store_codes8(crow, c, q, bits);
        if (res) Ld<float>::store8(res + c, e);
      } else {
        unsigned int p = 0;
        for (int j = 0; j < W; ++j) p |= (unsigned int)(q[j] + (1 << (bits - 1))) << (bits * j);
        crow[c / W] = (uint8_t)p;
        if (res)
          for (int j = 0; j < W; ++j) res[c + j] = e[j];
      }
    }
  }
}

// Single-pass variant: a group of G threads (a wavefront or the whole workgroup) owns a row
// and keeps it in registers (NV vectors of 8 elements per thread), so theta_g is read once
// for all K workers and every theta_k exactly once.  Same arithmetic as above.  With
// OUTER the dequantised values go straight into the mean and eq. 3 without re-reading
// theta_g or the codes; codes and scales are written either way.
template <typename WT, typename GT, int NV, int G, bool OUTER>
__global__ __launch_bounds__(OT_THREADS) void quantize_rows_reg_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, CodePtrs codes, ScalePtrs scales,
    ResidualPtrs ef, long rows, int n, int K, int bits, float qmax, float ef_beta, float eta,
    float mu, float inv_k, int nesterov, int write_back, int requant, uint8_t* mean_codes,
    float* mean_scales) {
  constexpr int ROWS_PER_BLOCK = OT_THREADS / G;
  __shared__ float red[2][OT_THREADS / 64];
  __shared__ float red2[OT_THREADS / 64];
  const int t = threadIdx.x % G;
  const long row = (long)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / G;
  const bool live = row < rows;            // whole groups are live or not; no early return
  const long rbase = live ? row * n : 0;   // (the workgroup-wide barrier below needs everyone)
  const long row_bytes = (long)n * bits / 8;
  float tg[NV][8], acc[OUTER ? NV : 1][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (t + i * G) * 8;
    if (live && c < n) Ld<GT>::load8(theta_g + rbase + c, tg[i]);
    else
#pragma unroll
      for (int j = 0; j < 8; ++j) tg[i][j] = 0.f;
    if constexpr (OUTER)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  }
  for (int k = 0; k < K; ++k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + rbase;
    float* res = ef.p[k] ? ef.p[k] + rbase : nullptr;
    float d[NV][8];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        float b[8];
        Ld<WT>::load8(tk + c, b);
#pragma unroll
        for (int j = 0; j < 8; ++j) d[i][j] = tg[i][j] - b[j];
        if (res) {
          float e[8];
          Ld<float>::load8(res + c, e);
#pragma unroll
          for (int j = 0; j < 8; ++j) d[i][j] = ef_input(d[i][j], e[j], ef_beta);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(d[i][j]));
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
    const float scale = amax / qmax;
    if (live && t == 0) scales.p[k][row] = scale;
    uint8_t* crow = codes.p[k] + row * row_bytes;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        int q[8];
        float e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          q[j] = (amax > 0.f) ? quant_level(d[i][j], scale, qmax) : 0;
          const float sent = __fmul_rn((float)q[j], scale);
          e[j] = __fsub_rn(d[i][j], sent);
          if constexpr (OUTER) acc[i][j] += sent;
        }
        store_codes8(crow, c, q, bits);
        if (res) Ld<float>::store8(res + c, e);
      }
    }
  }
  if constexpr (OUTER) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = __fmul_rn(acc[i][j], inv_k);     // Psi
    if (requant) {
      // Second quantisation (the dequantise-reduce-quantise step between the two modelled
      // collectives): Psi is quantised row-wise again and its dequantised value is used.
      float amax = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(acc[i][j]));    // dead lanes hold 0
      amax = wave_max(amax);
      if constexpr (G > 64) {
        if ((threadIdx.x & 63) == 0) red2[threadIdx.x >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(red2[0], red2[1]), fmaxf(red2[2], red2[3]));
      }
      const float scale = amax / qmax;
      if (mean_scales && live && t == 0) mean_scales[row] = scale;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (t + i * G) * 8;
        if (live && c < n) {
          int q[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            q[j] = (amax > 0.f) ? quant_level(acc[i][j], scale, qmax) : 0;
            acc[i][j] = __fmul_rn((float)q[j], scale);
          }
          if (mean_codes) store_codes8(mean_codes + row * row_bytes, c, q, bits);
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
        for (int j = 0; j < 8; ++j) outer_update<GT>(tg[i][j], uv[j], acc[i][j], eta, mu, nesterov);
        Ld<GT>::store8(theta_g + rbase + c, tg[i]);
        Ld<float>::store8(u + rbase + c, uv);
        if (write_back)
          for (int k = 0; k < K; ++k) Ld<WT>::store8(reinterpret_cast<WT*>(w.p[k]) + rbase + c, tg[i]);
      }
    }
  }
}

// ---- dequantise + average + outer update --------------------------------------------
template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void dequant_outer_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, CodePtrs codes, ScalePtrs scales,
    long rows, int n, int K, int bits, float eta, float mu, float inv_k, int nesterov, int write_back) {
  const int W = VEC ? 8 : 8 / bits;
  const int per_row = n / W;
  const long items = rows * per_row;
  const long row_bytes = (long)n * bits / 8;
  for (long i = (long)blockIdx.x * OT_THREADS + threadIdx.x; i < items;
       i += (long)gridDim.x * OT_THREADS) {
    const long row = i / per_row;
    const int c = (int)(i - row * per_row) * W;
    const long off = row * n + c;
    float tg[8], uv[8], acc[8];
    if (VEC) { Ld<GT>::load8(theta_g + off, tg); Ld<float>::load8(u + off, uv); }
    else
      for (int j = 0; j < W; ++j) { tg[j] = Ld<GT>::load1(theta_g + off + j); uv[j] = u[off + j]; }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      const float sc = scales.p[k][row];
      const uint8_t* crow = codes.p[k] + row * row_bytes;
      int q[8];
      if (VEC) {
        load_levels8(crow, c, q, bits);
      } else {
        const unsigned int p = crow[c / W];
        for (int j = 0; j < W; ++j) q[j] = (int)((p >> (bits * j)) & ((1u << bits) - 1u)) - (1 << (bits - 1));
      }
      for (int j = 0; j < W; ++j) acc[j] += __fmul_rn((float)q[j], sc);
    }
    for (int j = 0; j < W; ++j) outer_update<GT>(tg[j], uv[j], acc[j] * inv_k, eta, mu, nesterov);
    if (VEC) {
      Ld<GT>::store8(theta_g + off, tg);
      Ld<float>::store8(u + off, uv);
      if (write_back)
        for (int k = 0; k < K; ++k) Ld<WT>::store8(reinterpret_cast<WT*>(w.p[k]) + off, tg);
    } else {
      for (int j = 0; j < W; ++j) {
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

namespace {
float quant_qmax(int bits) { return (float)((1 << (bits - 1)) - 1); }
bool has_residuals(const ResidualPtrs& ef) { return ef.p[0] != nullptr; }
}  // namespace

int launch_quantize(const WorkerPtrs& w, int worker_dtype, const void* theta_g, int global_dtype,
                    const CodePtrs& codes, const ScalePtrs& scales, const ResidualPtrs& ef,
                    int64_t rows, int64_t n, int K, int bits, float ef_beta, hipStream_t stream) {
  const long blocks = (rows + OT_THREADS / 64 - 1) / (OT_THREADS / 64);
  if (blocks > 0x7fffffffL) return MLC_ERR_SHAPE;
  const double bytes = (double)rows * n * (K * esize(worker_dtype) + esize(global_dtype) + bits / 8.0 * K +
                                           (has_residuals(ef) ? 8.0 * K : 0.0)) +
                       (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_QUANTIZE, stream, 0.0, bytes);
  const bool vec = n % 8 == 0;
  const float qmax = quant_qmax(bits);
  // single-pass register kernel: a wavefront per row up to 2048 columns, a workgroup per row
  // up to 24576; otherwise (or for odd row lengths) the two-pass kernel
  if (vec && n <= 24576 && !(worker_dtype == MLC_F32 && global_dtype == MLC_BF16)) {
    const int g = n <= 2048 ? 64 : OT_THREADS;
    const int need = (int)((n + g * 8 - 1) / (g * 8));
    const int nv = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : need <= 8 ? 8 : 12;
    const long rpb = OT_THREADS / g;
    const long nblk = (rows + rpb - 1) / rpb;
#define MLC_QR(WT, GT, NV, G)                                                                     \
  hipLaunchKernelGGL((quantize_rows_reg_kernel<WT, GT, NV, G, false>), dim3((unsigned)nblk),       \
                     dim3(OT_THREADS), 0, stream, w, (GT*)const_cast<void*>(theta_g), (float*)nullptr, \
                     codes, scales, ef, (long)rows, (int)n, K, bits, qmax, ef_beta, 0.f, 0.f, 0.f, 0, 0, 0, \
                     (uint8_t*)nullptr, (float*)nullptr)
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
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, codes, scales, ef,   \
                         (long)rows, (int)n, K, bits, qmax, ef_beta);                             \
    else                                                                                          \
      hipLaunchKernelGGL((quantize_rows_kernel<WT, GT, false>), dim3((unsigned)blocks),           \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, codes, scales, ef,   \
                         (long)rows, (int)n, K, bits, qmax, ef_beta);                             \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

int launch_dequant_outer(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                         float* u, const CodePtrs& codes, const ScalePtrs& scales, int64_t rows,
                         int64_t n, int K, int bits, float eta_out, float mu, int nesterov,
                         int write_back, hipStream_t stream) {
  const bool vec = n % 8 == 0;
  const long items = rows * (n / (vec ? 8 : 8 / bits));
  const int blocks = cap_blocks((items + OT_THREADS - 1) / OT_THREADS, 256 * 16);
  const double bytes = (double)rows * n * (bits / 8.0 * K + 2 * esize(global_dtype) + 8 +
                                           (write_back ? K * esize(worker_dtype) : 0)) +
                       (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_DEQUANT_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_CALL(WT, GT)                                                                          \
  do {                                                                                            \
    if (vec)                                                                                      \
      hipLaunchKernelGGL((dequant_outer_kernel<WT, GT, true>), dim3(blocks), dim3(OT_THREADS), 0, \
                         stream, w, (GT*)theta_g, u, codes, scales, (long)rows, (int)n, K, bits,  \
                         eta_out, mu, inv_k, nesterov, write_back);                               \
    else                                                                                          \
      hipLaunchKernelGGL((dequant_outer_kernel<WT, GT, false>), dim3(blocks), dim3(OT_THREADS), 0,\
                         stream, w, (GT*)theta_g, u, codes, scales, (long)rows, (int)n, K, bits,  \
                         eta_out, mu, inv_k, nesterov, write_back);                               \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

// Returns MLC_ERR_UNSUPPORTED when the one-pass kernel does not cover the request (the
// caller then runs the quantiser and the dequantising update as two launches).
int launch_quantize_outer_fused(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                                float* u, const CodePtrs& codes, const ScalePtrs& scales,
                                const ResidualPtrs& ef, int64_t rows, int64_t n, int K, int bits,
                                float ef_beta, float eta_out, float mu, int nesterov, int write_back,
                                int requant, uint8_t* mean_codes, float* mean_scales,
                                hipStream_t stream) {
  if (n % 8 || n > 16384 || (worker_dtype == MLC_F32 && global_dtype == MLC_BF16))
    return MLC_ERR_UNSUPPORTED;
  const int g = n <= 2048 ? 64 : OT_THREADS;
  const int need = (int)((n + g * 8 - 1) / (g * 8));
  const int nv = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
  const long rpb = OT_THREADS / g;
  const long nblk = (rows + rpb - 1) / rpb;
  if (nblk > 0x7fffffffL) return MLC_ERR_SHAPE;
  const double bytes = (double)rows * n * (K * esize(worker_dtype) * (write_back ? 2 : 1) + bits / 8.0 * K +
                                           (has_residuals(ef) ? 8.0 * K : 0.0) +
                                           (mean_codes ? bits / 8.0 : 0.0) +
                                           2 * esize(global_dtype) + 8) + (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_DEQUANT_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
  const float qmax = quant_qmax(bits);
#define MLC_QO(WT, GT, NV, G)                                                                     \
  hipLaunchKernelGGL((quantize_rows_reg_kernel<WT, GT, NV, G, true>), dim3((unsigned)nblk),        \
                     dim3(OT_THREADS), 0, stream, w, (GT*)theta_g, u, codes, scales, ef, (long)rows, \
                     (int)n, K, bits, qmax, ef_beta, eta_out, mu, inv_k, nesterov, write_back, requant, \
                     mean_codes, mean_scales)
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
