// HBM-bound kernels of the Muon inner step (paper Sec. 2 "Muon", Sec. 5 "MuLoCo"):
//   momentum + look-ahead + sum of squares in one pass, the per-matrix norm, the parameter
//   update, and the layout conversions around the stand-alone newton_schulz call.
//
// The matrix handed to the Newton-Schulz GEMMs lives in a work-space layout padded to
// multiples of 128 in both dimensions ([count][mp][np], bf16, pad = 0), so the GEMM
// kernels need no bounds checks; zero padding does not change the iteration on the real
// block.  Each thread handles 8 adjacent columns (16 bytes of bf16).
#include "common.h"

namespace mlc {
namespace {

constexpr int EW_THREADS = 256;

// Sum over the workgroup in a fixed order: wavefront shuffles, then an LDS tree of 4.
__device__ __forceinline__ float block_sum(float v) {
  __shared__ float part[EW_THREADS / 64];
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
  if (threadIdx.x == 0) s = (part[0] + part[1]) + (part[2] + part[3]);
  return s;   // valid in thread 0
}

// m <- beta m + g ; U = g + beta m (or m) -> padded bf16 ; per-workgroup sum of U^2.
// WITH_MOM = false: U = in (stand-alone Newton-Schulz entry).
template <typename GT, bool WITH_MOM, bool VEC>
__global__ __launch_bounds__(EW_THREADS) void muon_momentum_kernel(
    const GT* __restrict__ grad, float* __restrict__ mom, bf16_t* __restrict__ U,
    float* __restrict__ partials, int m, int n, int mp, int np, int ldx, float beta, int nesterov) {
  const int b = blockIdx.y;
  const long mat = (long)b * m * n;
  const GT* g = grad + mat;
  float* mo = WITH_MOM ? mom + mat : nullptr;
  bf16_t* u = U + (long)b * mp * ldx;
  const int vec_per_row = np / 8;
  const long items = (long)mp * vec_per_row;
  float ss = 0.f;
  for (long it = (long)blockIdx.x * EW_THREADS + threadIdx.x; it < items;
       it += (long)gridDim.x * EW_THREADS) {
    const int row = (int)(it / vec_per_row);
    const int col = (int)(it - (long)row * vec_per_row) * 8;
    float uv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) uv[j] = 0.f;
    if (row < m && col < n) {
      const long off = (long)row * n + col;
      float gv[8], mv[8];
      if (VEC) {
        Vec8<GT>::load(g + off, gv);
        if (WITH_MOM) Vec8<float>::load(mo + off, mv);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool in = col + j < n;
          gv[j] = in ? Vec8<GT>::load1(g + off + j) : 0.f;
          mv[j] = (WITH_MOM && in) ? mo[off + j] : 0.f;
        }
      }
      if (WITH_MOM) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          mv[j] = beta * mv[j] + gv[j];
          uv[j] = nesterov ? gv[j] + beta * mv[j] : mv[j];
        }
        if (VEC) {
          Vec8<float>::store(mo + off, mv);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (col + j < n) mo[off + j] = mv[j];
        }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) uv[j] = gv[j];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) ss += uv[j] * uv[j];
    }
    Vec8<bf16_t>::store(u + (long)row * ldx + col, uv);
  }
  const float tot = block_sum(ss);
  if (threadIdx.x == 0) partials[(long)b * gridDim.x + blockIdx.x] = tot;
}

// scale[b] = 1 / (sqrt(sum_b) + eps); an all-zero matrix gets 0, also when eps = 0
__global__ __launch_bounds__(EW_THREADS) void muon_norm_kernel(const float* __restrict__ partials,
                                                               int nblk, float* __restrict__ scale,
                                                               float eps) {
  const int b = blockIdx.x;
  float s = 0.f;
  for (int i = threadIdx.x; i < nblk; i += EW_THREADS) s += partials[(long)b * nblk + i];
  const float tot = block_sum(s);
  if (threadIdx.x == 0) scale[b] = tot > 0.f ? 1.0f / (sqrtf(tot) + eps) : 0.f;
}

// W <- decay_factor * W - step * oscale_b * O     (decay_factor = 1 - eta*lambda,
//                                                  step = eta * lr_scale)
template <typename WT, bool VEC>
__global__ __launch_bounds__(EW_THREADS) void muon_update_kernel(
    WT* __restrict__ W, const bf16_t* __restrict__ O, const float* __restrict__ oscale, int m, int n,
    int mp, int ldx, float decay_factor, float step) {
  const int b = blockIdx.y;
  WT* w = W + (long)b * m * n;
  const bf16_t* o = O + (long)b * mp * ldx;
  const float st = oscale ? step * oscale[b] : step;
  const int vec_per_row = (n + 7) / 8;
  const long items = (long)m * vec_per_row;
  const long per_blk = (items + gridDim.x - 1) / gridDim.x;
  const long it_end = min(items, (long)(blockIdx.x + 1) * per_blk);
#pragma unroll 2
  for (long it = (long)blockIdx.x * per_blk + threadIdx.x; it < it_end; it += EW_THREADS) {
    const int row = (int)(it / vec_per_row);
    const int col = (int)(it - (long)row * vec_per_row) * 8;
    const long off = (long)row * n + col;
    float ov[8], wv[8];
    Vec8<bf16_t>::load_nt(o + (long)row * ldx + col, ov);   // padded layout: always in bounds
    if (VEC) {
      Vec8<WT>::load_nt(w + off, wv);
#pragma unroll
      for (int j = 0; j < 8; ++j) wv[j] = decay_factor * wv[j] - st * ov[j];
      Vec8<WT>::store_nt(w + off, wv);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (col + j < n)
          Vec8<WT>::store1(w + off + j, decay_factor * Vec8<WT>::load1(w + off + j) - st * ov[j]);
    }
  }
}

// out = oscale_b * X (padded bf16 -> caller's layout and dtype)
template <typename OT, bool VEC>
__global__ __launch_bounds__(EW_THREADS) void ns_store_kernel(
    const bf16_t* __restrict__ X, const float* __restrict__ oscale, OT* __restrict__ out, int m,
    int n, int mp, int ldx) {
  const int b = blockIdx.y;
  OT* o = out + (long)b * m * n;
  const bf16_t* x = X + (long)b * mp * ldx;
  const float sc = oscale ? oscale[b] : 1.0f;
  const int vec_per_row = (n + 7) / 8;
  const long items = (long)m * vec_per_row;
  for (long it = (long)blockIdx.x * EW_THREADS + threadIdx.x; it < items;
       it += (long)gridDim.x * EW_THREADS) {
    const int row = (int)(it / vec_per_row);
    const int col = (int)(it - (long)row * vec_per_row) * 8;
    const long off = (long)row * n + col;
    float xv[8];
    Vec8<bf16_t>::load(x + (long)row * ldx + col, xv);
#pragma unroll
    for (int j = 0; j < 8; ++j) xv[j] *= sc;
    if (VEC) {
      Vec8<OT>::store(o + off, xv);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (col + j < n) Vec8<OT>::store1(o + off + j, xv[j]);
    }
  }
}

// AdamW for the parameters Muon does not cover (paper Sec. 4, "AdamW inner updates"):
//   m <- b1 m + (1 - b1) g ; v <- b2 v + (1 - b2) g^2
//   theta <- theta - lr * (m * c1) / (sqrt(v) * c2 + eps) - lr * lambda * theta
// c1 = 1 / (1 - b1^t), c2 = 1 / sqrt(1 - b2^t) with bias correction, else 1.
// (Plain loads and stores: non-temporal ones measured 6 % slower here.)
template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(EW_THREADS) void adamw_kernel(
    WT* __restrict__ theta, const GT* __restrict__ grad, float* __restrict__ m, float* __restrict__ v,
    long n, float lr, float b1, float b2, float eps, float decay, float c1, float c2) {
  constexpr int W = VEC ? 8 : 1;
  const long items = (n + W - 1) / W;
  const long per_blk = (items + gridDim.x - 1) / gridDim.x;
  const long it_end = min(items, (long)(blockIdx.x + 1) * per_blk);
  for (long it = (long)blockIdx.x * per_blk + threadIdx.x; it < it_end; it += EW_THREADS) {
    const long off = it * W;
    float th[8], g[8], mv[8], vv[8];
    if (VEC) {
      Vec8<WT>::load(theta + off, th); Vec8<GT>::load(grad + off, g);
      Vec8<float>::load(m + off, mv); Vec8<float>::load(v + off, vv);
    } else {
      th[0] = Vec8<WT>::load1(theta + off); g[0] = Vec8<GT>::load1(grad + off);
      mv[0] = m[off]; vv[0] = v[off];
    }
#pragma unroll
    for (int j = 0; j < W; ++j) {
      mv[j] = b1 * mv[j] + (1.0f - b1) * g[j];
      vv[j] = b2 * vv[j] + (1.0f - b2) * g[j] * g[j];
      const float step = (mv[j] * c1) / (sqrtf(vv[j]) * c2 + eps);
      th[j] = th[j] - lr * step - decay * th[j];
    }
    if (VEC) {
      Vec8<WT>::store(theta + off, th);
      Vec8<float>::store(m + off, mv); Vec8<float>::store(v + off, vv);
    } else {
      Vec8<WT>::store1(theta + off, th[0]);
      m[off] = mv[0]; v[off] = vv[0];
    }
  }
}

int check_launch() { return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH; }

int grid_blocks(long items, int cap) {
  long blocks = (items + EW_THREADS - 1) / EW_THREADS;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

template <typename GT, bool WITH_MOM>
int launch_momentum_t(const GT* grad, float* mom, bf16_t* U, float* partials, int nblk,
                      int64_t count, int64_t m, int64_t n, int64_t mp, int64_t np, int64_t ldx,
                      float beta, int nesterov, hipStream_t stream, int family) {
  const dim3 grid(nblk, (unsigned)count), block(EW_THREADS);
  const double elems = (double)count * m * n;
  const double bytes = elems * (sizeof(GT) + (WITH_MOM ? 8 : 0)) + (double)count * mp * np * 2;
  LaunchScope scope(family, stream, 0.0, bytes);
  if (n % 8 == 0)
    hipLaunchKernelGGL((muon_momentum_kernel<GT, WITH_MOM, true>), grid, block, 0, stream, grad, mom,
                       U, partials, (int)m, (int)n, (int)mp, (int)np, (int)ldx, beta, nesterov);
  else
    hipLaunchKernelGGL((muon_momentum_kernel<GT, WITH_MOM, false>), grid, block, 0, stream, grad, mom,
                       U, partials, (int)m, (int)n, (int)mp, (int)np, (int)ldx, beta, nesterov);
  return check_launch();
}

}  // namespace

int launch_momentum(const void* grad, int grad_dtype, float* mom, bf16_t* U, float* partials,
                    int nblk, int64_t count, int64_t m, int64_t n, int64_t mp, int64_t np,
                    int64_t ldx, float beta, int nesterov, hipStream_t stream) {
  if (grad_dtype == MLC_F32)
    return launch_momentum_t<float, true>((const float*)grad, mom, U, partials, nblk, count, m, n,
                                          mp, np, ldx, beta, nesterov, stream, MLC_KERNEL_MOMENTUM);
  return launch_momentum_t<bf16_t, true>((const bf16_t*)grad, mom, U, partials, nblk, count, m, n,
                                         mp, np, ldx, beta, nesterov, stream, MLC_KERNEL_MOMENTUM);
}

int launch_ns_load(const void* in, int dtype, bf16_t* U, float* partials, int nblk, int64_t count,
                   int64_t m, int64_t n, int64_t mp, int64_t np, int64_t ldx, hipStream_t stream) {
  if (dtype == MLC_F32)
    return launch_momentum_t<float, false>((const float*)in, nullptr, U, partials, nblk, count, m,
                                           n, mp, np, ldx, 0.f, 0, stream, MLC_KERNEL_CONVERT);
  return launch_momentum_t<bf16_t, false>((const bf16_t*)in, nullptr, U, partials, nblk, count, m,
                                          n, mp, np, ldx, 0.f, 0, stream, MLC_KERNEL_CONVERT);
}

int launch_norm_finalize(const float* partials, int nblk, float* scale, int64_t count, float eps,
                         hipStream_t stream) {
  LaunchScope scope(MLC_KERNEL_NORM, stream, 0.0, (double)count * nblk * 4);
  hipLaunchKernelGGL(muon_norm_kernel, dim3((unsigned)count), dim3(EW_THREADS), 0, stream, partials,
                     nblk, scale, eps);
  return check_launch();
}

int launch_param_update(void* W, int dtype, const bf16_t* O, const float* oscale, int64_t count,
                        int64_t m, int64_t n, int64_t mp, int64_t ldx, float decay_factor, float step,
                        hipStream_t stream) {
  const long items = m * ((n + 7) / 8);
  const dim3 grid(grid_blocks(items, 2048), (unsigned)count), block(EW_THREADS);
  const double elems = (double)count * m * n;
  const double bytes = elems * (2 + 2 * (dtype == MLC_F32 ? 4 : 2));
  LaunchScope scope(MLC_KERNEL_UPDATE, stream, 0.0, bytes);
  const bool vec = n % 8 == 0;
#define MLC_UPD(WT, V)                                                                          \
  hipLaunchKernelGGL((muon_update_kernel<WT, V>), grid, block, 0, stream, (WT*)W, O, oscale, (int)m, \
                     (int)n, (int)mp, (int)ldx, decay_factor, step)
  if (dtype == MLC_F32) { if (vec) MLC_UPD(float, true); else MLC_UPD(float, false); }
  else { if (vec) MLC_UPD(bf16_t, true); else MLC_UPD(bf16_t, false); }
#undef MLC_UPD
  return check_launch();
}

int launch_ns_store(const bf16_t* X, const float* oscale, void* out, int dtype, int64_t count,
                    int64_t m, int64_t n, int64_t mp, int64_t ldx, hipStream_t stream) {
  const long items = m * ((n + 7) / 8);
  const dim3 grid(grid_blocks(items, 2048), (unsigned)count), block(EW_THREADS);
  const double elems = (double)count * m * n;
  LaunchScope scope(MLC_KERNEL_CONVERT, stream, 0.0, elems * (2 + (dtype == MLC_F32 ? 4 : 2)));
  const bool vec = n % 8 == 0;
#define MLC_ST(OT, V)                                                                             \
  hipLaunchKernelGGL((ns_store_kernel<OT, V>), grid, block, 0, stream, X, oscale, (OT*)out, (int)m, \
                     (int)n, (int)mp, (int)ldx)
  if (dtype == MLC_F32) { if (vec) MLC_ST(float, true); else MLC_ST(float, false); }
  else { if (vec) MLC_ST(bf16_t, true); else MLC_ST(bf16_t, false); }
#undef MLC_ST
  return check_launch();
}

int launch_adamw(void* theta, int param_dtype, const void* grad, int grad_dtype, float* m, float* v,
                 int64_t n, float lr, float b1, float b2, float eps, float decay, float c1, float c2,
                 hipStream_t stream) {
  const bool vec = n % 8 == 0;
  const long items = vec ? n / 8 : n;
  const dim3 grid(grid_blocks(items, 256 * 16)), block(EW_THREADS);
  const double bytes = (double)n * (2 * (param_dtype == MLC_F32 ? 4 : 2) + (grad_dtype == MLC_F32 ? 4 : 2) + 16);
  LaunchScope scope(MLC_KERNEL_ADAMW, stream, 0.0, bytes);
#define MLC_AW(WT, GT, V)                                                                         \
  hipLaunchKernelGGL((adamw_kernel<WT, GT, V>), grid, block, 0, stream, (WT*)theta, (const GT*)grad, m, v, \
                     (long)n, lr, b1, b2, eps, decay, c1, c2)
#define MLC_AW_V(WT, GT) do { if (vec) MLC_AW(WT, GT, true); else MLC_AW(WT, GT, false); } while (0)
  if (param_dtype == MLC_F32 && grad_dtype == MLC_F32) MLC_AW_V(float, float);
  else if (param_dtype == MLC_F32) MLC_AW_V(float, bf16_t);
  else if (grad_dtype == MLC_F32) MLC_AW_V(bf16_t, float);
  else MLC_AW_V(bf16_t, bf16_t);
#undef MLC_AW_V
#undef MLC_AW
  return check_launch();
}

}  // namespace mlc
