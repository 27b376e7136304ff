// HBM-bound kernels of the DiLoCo outer step (paper Sec. 4.1 eqs. 2-3, Algorithm 1 lines
// after the inner loop, Algorithm 2 "compress parameter delta"):
//   * fused pseudogradient / K-way average / outer Nesterov / write-back,
//   * 2/4/8-bit linear quantiser of theta_g - theta_k (IEEE fp32, ties to even), range per row
//     or per matrix, with or without an offset, optionally with error feedback (Algorithm 2,
//     EF branch) and a second quantisation of the mean,
//   * dequantise + K-way average + outer update + write-back.
// The K worker replicas live on this GPU, so the average is a loop over K pointers
// in a fixed order: ((d_1 + d_2) + ...) * (1/K).
#include "common.h"

namespace mlc {
namespace {

constexpr int OT_THREADS = 256;

// eq. 3; theta comes back as the value the global buffer will hold after the store, so the
// write-back hands every worker exactly the new theta_g.
template <typename GT>
__device__ __forceinline__ void outer_update(float& theta, float& u, float psi, float eta, float mu,
                                             int nesterov) {
  const float step = eta * psi;
  u = mu * u + step;
  theta = Vec8<GT>::round(nesterov ? theta - mu * u - step : theta - u);
}

// ---- unquantised fused outer step ---------------------------------------------------
// Workgroup blk of nblk walks over its share of the n_elems elements.
template <typename WT, typename GT, typename PW>
__device__ __forceinline__ void outer_fused_body(
    const PW& w, GT* __restrict__ theta_g, float* __restrict__ u, long n_elems, int K, float eta,
    float mu, float inv_k, int nesterov, int write_back, long blk, long nblk) {
  const long n_vec = n_elems / 8;
  for (long i = blk * OT_THREADS + threadIdx.x; i < n_vec; i += nblk * OT_THREADS) {
    const long off = i * 8;
    float tg[8], uv[8], acc[8];
    Vec8<GT>::load(theta_g + off, tg);
    Vec8<float>::load(u + off, uv);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      float tk[8];
      Vec8<WT>::load(reinterpret_cast<const WT*>(w.p[k]) + off, tk);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += tg[j] - tk[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) outer_update<GT>(tg[j], uv[j], acc[j] * inv_k, eta, mu, nesterov);
    Vec8<GT>::store(theta_g + off, tg);
    Vec8<float>::store(u + off, uv);
    if (write_back)
      for (int k = 0; k < K; ++k) Vec8<WT>::store(reinterpret_cast<WT*>(w.p[k]) + off, tg);
  }
  // ragged tail (fewer than 8 elements), one thread each
  const long tail0 = n_vec * 8;
  const long t = tail0 + blk * OT_THREADS + threadIdx.x;
  if (t < n_elems) {
    float tg = Vec8<GT>::load1(theta_g + t), uv = u[t], acc = 0.f;
    for (int k = 0; k < K; ++k) acc += tg - Vec8<WT>::load1(reinterpret_cast<const WT*>(w.p[k]) + t);
    outer_update<GT>(tg, uv, acc * inv_k, eta, mu, nesterov);
    Vec8<GT>::store1(theta_g + t, tg);
    u[t] = uv;
    if (write_back)
      for (int k = 0; k < K; ++k) Vec8<WT>::store1(reinterpret_cast<WT*>(w.p[k]) + t, tg);
  }
}

template <typename WT, typename GT>
__global__ __launch_bounds__(OT_THREADS) void outer_fused_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, long n_elems, int K, float eta,
    float mu, float inv_k, int nesterov, int write_back) {
  outer_fused_body<WT, GT>(w, theta_g, u, n_elems, K, eta, mu, inv_k, nesterov, write_back,
                           (long)blockIdx.x, (long)gridDim.x);
}

// ---- linear quantiser (Sec. 2 "Compressed Communication"; Algorithm 2) -----------------
// bits = 2, 4 or 8.  Without offset: levels -L..L, L = 2^(bits-1) - 1, over [-amax, amax],
// stored code = level + 2^(bits-1).  With offset: levels 0..L, L = 2^bits - 1, over
// [min, max], stored as they are, dequantised value = level * scale + min.  8 / bits codes
// per byte, the lowest column in the lowest bits.  The range is taken per row, or per matrix
// (then it has been computed beforehand and is read from the scale / offset arrays).  With
// error feedback the value quantised is e = fl32(fl32(beta * E) + delta) and the residual
// becomes E <- fl32(e - dequantised value).  Every operation is a single fp32 operation
// (no fused multiply-add) so that codes and residuals are reproducible bit for bit.
struct Range { float scale, lo; };

__device__ __forceinline__ Range make_range(float mn, float mx, const QuantForm& f) {
  Range r;
  if (f.offset) { r.lo = mn; r.scale = __fsub_rn(mx, mn) / f.levels; }
  else { r.lo = 0.f; r.scale = fmaxf(mx, -mn) / f.levels; }
  return r;
}

__device__ __forceinline__ int quant_level(float v, const Range& r, const QuantForm& f) {
  if (!(r.scale > 0.f)) return 0;
  const float x = f.offset ? __fsub_rn(v, r.lo) : v;
  float q = rintf(x / r.scale);             // IEEE division, round half to even
  q = fminf(fmaxf(q, f.offset ? 0.f : -f.levels), f.levels);
  return (int)q;
}

__device__ __forceinline__ float dequant_level(int q, const Range& r, const QuantForm& f) {
  const float s = __fmul_rn((float)q, r.scale);
  return f.offset ? __fadd_rn(s, r.lo) : s;
}

__device__ __forceinline__ float ef_input(float delta, float residual, float beta) {
  return __fadd_rn(__fmul_rn(beta, residual), delta);
}

// 8 adjacent levels of a row, first column c (a multiple of 8) <-> bits bytes of its codes
__device__ __forceinline__ void store_codes8(uint8_t* crow, int c, const int (&q)[8], int bits, int bias) {
  if (bits == 4) {
    unsigned int p = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) p |= (unsigned int)(q[j] + bias) << (4 * j);
    *reinterpret_cast<unsigned int*>(crow + c / 2) = p;
  } else if (bits == 8) {
    u32x2 p = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p.x |= (unsigned int)(q[j] + bias) << (8 * j);
      p.y |= (unsigned int)(q[j + 4] + bias) << (8 * j);
    }
    *reinterpret_cast<u32x2*>(crow + c) = p;
  } else {
    unsigned int p = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) p |= (unsigned int)(q[j] + bias) << (2 * j);
    *reinterpret_cast<unsigned short*>(crow + c / 4) = (unsigned short)p;
  }
}

__device__ __forceinline__ void load_levels8(const uint8_t* crow, int c, int (&q)[8], int bits, int bias) {
  if (bits == 4) {
    const unsigned int p = *reinterpret_cast<const unsigned int*>(crow + c / 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (int)((p >> (4 * j)) & 0xfu) - bias;
  } else if (bits == 8) {
    const u32x2 p = *reinterpret_cast<const u32x2*>(crow + c);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      q[j] = (int)((p.x >> (8 * j)) & 0xffu) - bias;
      q[j + 4] = (int)((p.y >> (8 * j)) & 0xffu) - bias;
    }
  } else {
    const unsigned int p = *reinterpret_cast<const unsigned short*>(crow + c / 4);
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (int)((p >> (2 * j)) & 0x3u) - bias;
  }
}

// Range of worker k's row (or of the matrix the row belongs to) as stored by an earlier pass.
template <typename PS, typename PO>
__device__ __forceinline__ Range stored_range(const PS& scales, const PO& offsets, int k,
                                              long grp, const QuantForm& f) {
  Range r;
  r.scale = scales.p[k][grp];
  r.lo = f.offset ? offsets.p[k][grp] : 0.f;
  return r;
}

// ---- ranges per matrix (the "global" scope): init, reduce with atomics, finalise --------
// Floats are ordered through an order-preserving map to unsigned keys, so that the
// reduction is exact and independent of the order in which workgroups arrive.
__device__ __forceinline__ unsigned int float_key(float v) {
  const unsigned int b = __float_as_uint(v);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(unsigned int k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void matrix_range_init_kernel(ScalePtrs scales, OffsetPtrs offsets, long count, int offset) {
  const long b = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const int k = blockIdx.y;
  if (b >= count) return;
  reinterpret_cast<unsigned int*>(scales.p[k])[b] = 0u;                    // below every key
  if (offset) reinterpret_cast<unsigned int*>(offsets.p[k])[b] = 0xffffffffu;   // above every key
}

template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void matrix_range_kernel(
    WorkerPtrs w, const GT* __restrict__ theta_g, ScalePtrs scales, OffsetPtrs offsets, ResidualPtrs ef,
    long elems, QuantForm form) {
  __shared__ float red[2][OT_THREADS / 64];
  const long b = blockIdx.y;
  const int k = blockIdx.z;
  const GT* tg = theta_g + b * elems;
  const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + b * elems;
  const float* res = ef.p[k] ? ef.p[k] + b * elems : nullptr;
  constexpr int W = VEC ? 8 : 1;
  float mn = INFINITY, mx = -INFINITY;
  for (long i = ((long)blockIdx.x * OT_THREADS + threadIdx.x) * W; i < elems;
       i += (long)gridDim.x * OT_THREADS * W) {
    float a[8], c[8], e[8];
    if (VEC) {
      Vec8<GT>::load(tg + i, a); Vec8<WT>::load(tk + i, c);
      if (res) Vec8<float>::load(res + i, e);
    } else {
      a[0] = Vec8<GT>::load1(tg + i); c[0] = Vec8<WT>::load1(tk + i);
      if (res) e[0] = res[i];
    }
#pragma unroll
    for (int j = 0; j < W; ++j) {
      const float d = a[j] - c[j];
      const float v = res ? ef_input(d, e[j], form.ef_beta) : d;
      mn = fminf(mn, v); mx = fmaxf(mx, v);
    }
  }
  mn = wave_min(mn); mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = mn; red[1][threadIdx.x >> 6] = mx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    mn = fminf(fminf(red[0][0], red[0][1]), fminf(red[0][2], red[0][3]));
    mx = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
    if (mn <= mx) {          // this workgroup saw at least one element
      if (form.offset) {
        atomicMax(reinterpret_cast<unsigned int*>(scales.p[k]) + b, float_key(mx));
        atomicMin(reinterpret_cast<unsigned int*>(offsets.p[k]) + b, float_key(mn));
      } else {               // amax >= 0: its bit pattern is ordered like an unsigned
        atomicMax(reinterpret_cast<unsigned int*>(scales.p[k]) + b, __float_as_uint(fmaxf(mx, -mn)));
      }
    }
  }
}

__global__ void matrix_range_finish_kernel(ScalePtrs scales, OffsetPtrs offsets, long count, QuantForm form) {
  const long b = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const int k = blockIdx.y;
  if (b >= count) return;
  if (form.offset) {
    const float mx = key_float(reinterpret_cast<unsigned int*>(scales.p[k])[b]);
    const float mn = key_float(reinterpret_cast<unsigned int*>(offsets.p[k])[b]);
    const Range r = make_range(mn, mx, form);
    scales.p[k][b] = r.scale;
    offsets.p[k][b] = r.lo;
  } else {
    scales.p[k][b] = scales.p[k][b] / form.levels;     // the array holds amax
  }
}

// Two passes over the row (range, then codes), one wavefront per row, all K workers; the
// second pass re-reads data the first pass just pulled through L2.  Rows whose length is
// not a multiple of 8 go one code byte (8 / bits columns) per lane and step.
template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void quantize_rows_kernel(
    WorkerPtrs w, const GT* __restrict__ theta_g, CodePtrs codes, ScalePtrs scales, OffsetPtrs offsets,
    ResidualPtrs ef, long rows, int n, int K, QuantForm form) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (OT_THREADS / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const GT* tg = theta_g + row * n;
  const int bits = form.bits;
  const int W = VEC ? 8 : 8 / bits;         // elements per lane per step
  const long row_bytes = (long)n * bits / 8;
  for (int k = 0; k < K; ++k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + row * n;
    float* res = ef.p[k] ? ef.p[k] + row * n : nullptr;
    Range rg;
    if (form.rows_per_range) {
      rg = stored_range(scales, offsets, k, row / form.rows_per_range, form);
    } else {
      float mn = INFINITY, mx = -INFINITY;
      for (int c = lane * W; c < n; c += 64 * W) {
        float a[8], b[8], e[8];
        if (VEC) {
          Vec8<GT>::load(tg + c, a); Vec8<WT>::load(tk + c, b);
          if (res) Vec8<float>::load(res + c, e);
        } else {
          for (int j = 0; j < W; ++j) {
            a[j] = Vec8<GT>::load1(tg + c + j); b[j] = Vec8<WT>::load1(tk + c + j);
            if (res) e[j] = res[c + j];
          }
        }
        for (int j = 0; j < W; ++j) {
          const float d = a[j] - b[j];
          const float v = res ? ef_input(d, e[j], form.ef_beta) : d;
          mn = fminf(mn, v); mx = fmaxf(mx, v);
        }
      }
      rg = make_range(wave_min(mn), wave_max(mx), form);
      if (lane == 0) {
        scales.p[k][row] = rg.scale;
        if (form.offset) offsets.p[k][row] = rg.lo;
      }
    }
    uint8_t* crow = codes.p[k] + row * row_bytes;
    for (int c = lane * W; c < n; c += 64 * W) {
      float a[8], b[8], e[8];
      if (VEC) {
        Vec8<GT>::load(tg + c, a); Vec8<WT>::load(tk + c, b);
        if (res) Vec8<float>::load(res + c, e);
      } else {
        for (int j = 0; j < W; ++j) {
          a[j] = Vec8<GT>::load1(tg + c + j); b[j] = Vec8<WT>::load1(tk + c + j);
          if (res) e[j] = res[c + j];
        }
      }
      int q[8];
      for (int j = 0; j < W; ++j) {
        const float d = a[j] - b[j];
        const float v = res ? ef_input(d, e[j], form.ef_beta) : d;
        q[j] = quant_level(v, rg, form);
        e[j] = __fsub_rn(v, dequant_level(q[j], rg, form));
      }
      if (VEC) {
        store_codes8(crow, c, q, bits, form.code_bias);
        if (res) Vec8<float>::store(res + c, e);
      } else {
        unsigned int p = 0;
        for (int j = 0; j < W; ++j) p |= (unsigned int)(q[j] + form.code_bias) << (bits * j);
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
// theta_g or the codes; codes, scales and offsets are written either way.
// `blk` is the index of the workgroup among those that share these arguments; the pointer sets
// may be the 32-wide ones of a single-group launch or the narrow ones of a launch that covers
// several groups.
template <typename WT, typename GT, int NV, int G, bool OUTER, typename PW, typename PC, typename PS,
          typename PO, typename PE>
__device__ __forceinline__ void quantize_rows_reg_body(
    const PW& w, GT* __restrict__ theta_g, float* __restrict__ u, const PC& codes, const PS& scales,
    const PO& offsets, const PE& ef, long rows, int n, int K, const QuantForm& form, float eta, float mu,
    float inv_k, int nesterov, int write_back, int requant, uint8_t* mean_codes, float* mean_scales,
    float* mean_offsets, long blk) {
  constexpr int ROWS_PER_BLOCK = OT_THREADS / G;
  constexpr int NW = OT_THREADS / 64;
  __shared__ float red[2][2][NW];          // [parity of k][min, max][wavefront]
  __shared__ float red2[2][NW];
  const int t = threadIdx.x % G;
  const long row = blk * ROWS_PER_BLOCK + threadIdx.x / G;
  const bool live = row < rows;            // whole groups are live or not; no early return
  const long rbase = live ? row * n : 0;   // (the workgroup-wide barrier below needs everyone)
  const int bits = form.bits;
  const long row_bytes = (long)n * bits / 8;
  const long grp = form.rows_per_range ? (live ? row / form.rows_per_range : 0) : (live ? row : 0);
  float tg[NV][8], acc[OUTER ? NV : 1][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (t + i * G) * 8;
    if (live && c < n) Vec8<GT>::load(theta_g + rbase + c, tg[i]);
    else
#pragma unroll
      for (int j = 0; j < 8; ++j) tg[i][j] = 0.f;
    if constexpr (OUTER)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  }
  // The next worker's row is requested before this worker's row is reduced and quantised, so
  // that with several workers only the first request waits for memory with nothing to do.
  typedef typename Vec8<WT>::raw_t RawT;
  RawT ahead[NV];
  auto request = [&](int k) {
    const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + rbase;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) ahead[i] = Vec8<WT>::load_raw(tk + c);
    }
  };
  request(0);
  for (int k = 0; k < K; ++k) {
    float* res = ef.p[k] ? ef.p[k] + rbase : nullptr;
    float d[NV][8];
    float mn = INFINITY, mx = -INFINITY;
    RawT cur[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) cur[i] = ahead[i];
    if (k + 1 < K) request(k + 1);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        float b[8];
        Vec8<WT>::unpack(cur[i], b);
#pragma unroll
        for (int j = 0; j < 8; ++j) d[i][j] = tg[i][j] - b[j];
        if (res) {
          float e[8];
          Vec8<float>::load(res + c, e);
#pragma unroll
          for (int j = 0; j < 8; ++j) d[i][j] = ef_input(d[i][j], e[j], form.ef_beta);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) { mn = fminf(mn, d[i][j]); mx = fmaxf(mx, d[i][j]); }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) d[i][j] = 0.f;
      }
    }
    Range rg;
    if (form.rows_per_range) {
      rg = stored_range(scales, offsets, k, grp, form);
    } else {
      mn = wave_min(mn); mx = wave_max(mx);
      if constexpr (G > 64) {
        if ((threadIdx.x & 63) == 0) { red[k & 1][0][threadIdx.x >> 6] = mn; red[k & 1][1][threadIdx.x >> 6] = mx; }
        __syncthreads();
        mn = fminf(fminf(red[k & 1][0][0], red[k & 1][0][1]), fminf(red[k & 1][0][2], red[k & 1][0][3]));
        mx = fmaxf(fmaxf(red[k & 1][1][0], red[k & 1][1][1]), fmaxf(red[k & 1][1][2], red[k & 1][1][3]));
      }
      rg = make_range(mn, mx, form);
      if (live && t == 0) {
        scales.p[k][row] = rg.scale;
        if (form.offset) offsets.p[k][row] = rg.lo;
      }
    }
    uint8_t* crow = codes.p[k] + row * row_bytes;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        int q[8];
        float e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          q[j] = quant_level(d[i][j], rg, form);
          const float sent = dequant_level(q[j], rg, form);
          e[j] = __fsub_rn(d[i][j], sent);
          if constexpr (OUTER) acc[i][j] += sent;
        }
        store_codes8(crow, c, q, bits, form.code_bias);
        if (res) Vec8<float>::store(res + c, e);
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
      float mn = INFINITY, mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (t + i * G) * 8;
        if (live && c < n)
#pragma unroll
          for (int j = 0; j < 8; ++j) { mn = fminf(mn, acc[i][j]); mx = fmaxf(mx, acc[i][j]); }
      }
      mn = wave_min(mn); mx = wave_max(mx);
      if constexpr (G > 64) {
        if ((threadIdx.x & 63) == 0) { red2[0][threadIdx.x >> 6] = mn; red2[1][threadIdx.x >> 6] = mx; }
        __syncthreads();
        mn = fminf(fminf(red2[0][0], red2[0][1]), fminf(red2[0][2], red2[0][3]));
        mx = fmaxf(fmaxf(red2[1][0], red2[1][1]), fmaxf(red2[1][2], red2[1][3]));
      }
      const Range rg = make_range(mn, mx, form);
      if (live && t == 0) {
        if (mean_scales) mean_scales[row] = rg.scale;
        if (mean_offsets && form.offset) mean_offsets[row] = rg.lo;
      }
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (t + i * G) * 8;
        if (live && c < n) {
          int q[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            q[j] = quant_level(acc[i][j], rg, form);
            acc[i][j] = dequant_level(q[j], rg, form);
          }
          if (mean_codes) store_codes8(mean_codes + row * row_bytes, c, q, bits, form.code_bias);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (t + i * G) * 8;
      if (live && c < n) {
        float uv[8];
        Vec8<float>::load(u + rbase + c, uv);
#pragma unroll
        for (int j = 0; j < 8; ++j) outer_update<GT>(tg[i][j], uv[j], acc[i][j], eta, mu, nesterov);
        Vec8<GT>::store(theta_g + rbase + c, tg[i]);
        Vec8<float>::store(u + rbase + c, uv);
        if (write_back)
          for (int k = 0; k < K; ++k) Vec8<WT>::store(reinterpret_cast<WT*>(w.p[k]) + rbase + c, tg[i]);
      }
    }
  }
}

// Wavefronts per SIMD the register allocation is held to: one more than the compiler reaches on
// its own where that is a few registers away (these kernels wait on memory with little else to
// do, so a resident wavefront more is worth more than the registers).
constexpr int quant_min_waves(int nv, bool outer) {
  return outer ? (nv <= 1 ? 6 : nv <= 2 ? 4 : nv <= 4 ? 3 : 1) : (nv <= 1 ? 7 : nv <= 2 ? 5 : nv <= 4 ? 3 : 1);
}

template <typename WT, typename GT, int NV, int G, bool OUTER>
__global__ __launch_bounds__(OT_THREADS, quant_min_waves(NV, OUTER)) void quantize_rows_reg_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, CodePtrs codes, ScalePtrs scales,
    OffsetPtrs offsets, ResidualPtrs ef, long rows, int n, int K, QuantForm form, float eta, float mu,
    float inv_k, int nesterov, int write_back, int requant, uint8_t* mean_codes, float* mean_scales,
    float* mean_offsets) {
  quantize_rows_reg_body<WT, GT, NV, G, OUTER>(w, theta_g, u, codes, scales, offsets, ef, rows, n, K, form,
                                               eta, mu, inv_k, nesterov, write_back, requant, mean_codes,
                                               mean_scales, mean_offsets, (long)blockIdx.x);
}

// ---- one launch over several groups ----------------------------------------------------
// A streaming fragment (one transformer layer: three shape groups) is small enough that
// three launches of 70-80 us each spend a good part of their time filling and draining the
// chip; here the workgroups of one launch are dealt to the groups of a table that travels in
// the kernel arguments (up to OUTER_MAX_SEG groups, OUTER_MAX_SEG_K workers).
template <typename T> struct SegPtrs { T p[OUTER_MAX_SEG_K]; };
struct QuantSeg {
  SegPtrs<void*> w;
  SegPtrs<uint8_t*> codes;
  SegPtrs<float*> scales, offsets, ef;
  void* theta_g;
  float* u;
  long rows;
  int n;
  int cfg;                  // index into the (vectors per thread, threads per row) table below
  unsigned int blk0;        // first workgroup of this group
};
struct QuantSegTable { QuantSeg s[OUTER_MAX_SEG]; int nseg; };

// (NV, G) of a row length, as launch_quantize_outer_fused picks them; -1: not covered
struct RegCfg { int nv, g; };
__host__ __device__ constexpr RegCfg reg_cfg(int idx) {
  return idx == 0 ? RegCfg{1, 64} : idx == 1 ? RegCfg{2, 64} : idx == 2 ? RegCfg{4, 64}
       : idx == 3 ? RegCfg{2, 256} : idx == 4 ? RegCfg{4, 256} : idx == 5 ? RegCfg{6, 256}
       : idx == 6 ? RegCfg{8, 256} : RegCfg{12, 256};
}

template <typename WT, typename GT>
__global__ __launch_bounds__(OT_THREADS, 3) void quantize_outer_multi_kernel(
    QuantSegTable tab, int K, QuantForm form, float eta, float mu, float inv_k, int nesterov, int write_back) {
  int si = 0;
#pragma unroll
  for (int i = 1; i < OUTER_MAX_SEG; ++i)
    if (i < tab.nseg && blockIdx.x >= tab.s[i].blk0) si = i;
  const QuantSeg& sg = tab.s[si];
  const long blk = (long)(blockIdx.x - sg.blk0);
#define MLC_SEG_BODY(IDX)                                                                              \
  quantize_rows_reg_body<WT, GT, reg_cfg(IDX).nv, reg_cfg(IDX).g, true>(                               \
      sg.w, (GT*)sg.theta_g, sg.u, sg.codes, sg.scales, sg.offsets, sg.ef, sg.rows, sg.n, K, form, eta, \
      mu, inv_k, nesterov, write_back, 0, nullptr, nullptr, nullptr, blk)
  switch (sg.cfg) {      // uniform over the workgroup
    case 0: MLC_SEG_BODY(0); break;
    case 1: MLC_SEG_BODY(1); break;
    case 2: MLC_SEG_BODY(2); break;
    case 3: MLC_SEG_BODY(3); break;
    default: MLC_SEG_BODY(4); break;      // rows that need more vectors per thread (and with
  }                                        // them more registers) are not taken: see the launcher
#undef MLC_SEG_BODY
}

struct OuterSeg {
  SegPtrs<void*> w;
  void* theta_g;
  float* u;
  long n_elems;
  unsigned int blk0, nblk;
};
struct OuterSegTable { OuterSeg s[OUTER_MAX_SEG]; int nseg; };

template <typename WT, typename GT>
__global__ __launch_bounds__(OT_THREADS) void outer_fused_multi_kernel(
    OuterSegTable tab, int K, float eta, float mu, float inv_k, int nesterov, int write_back) {
  int si = 0;
#pragma unroll
  for (int i = 1; i < OUTER_MAX_SEG; ++i)
    if (i < tab.nseg && blockIdx.x >= tab.s[i].blk0) si = i;
  const OuterSeg& sg = tab.s[si];
  outer_fused_body<WT, GT>(sg.w, (GT*)sg.theta_g, sg.u, sg.n_elems, K, eta, mu, inv_k, nesterov, write_back,
                           (long)(blockIdx.x - sg.blk0), (long)sg.nblk);
}

// ---- dequantise + average + outer update --------------------------------------------
template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void dequant_outer_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, CodePtrs codes, ScalePtrs scales,
    OffsetPtrs offsets, long rows, int n, int K, QuantForm form, float eta, float mu, float inv_k,
    int nesterov, int write_back) {
  const int bits = form.bits;
  const int W = VEC ? 8 : 8 / bits;
  const int per_row = n / W;
  const long items = rows * per_row;
  const long row_bytes = (long)n * bits / 8;
  for (long i = (long)blockIdx.x * OT_THREADS + threadIdx.x; i < items;
       i += (long)gridDim.x * OT_THREADS) {
    const long row = i / per_row;
    const int c = (int)(i - row * per_row) * W;
    const long off = row * n + c;
    const long grp = form.rows_per_range ? row / form.rows_per_range : row;
    float tg[8], uv[8], acc[8];
    if (VEC) { Vec8<GT>::load(theta_g + off, tg); Vec8<float>::load(u + off, uv); }
    else
      for (int j = 0; j < W; ++j) { tg[j] = Vec8<GT>::load1(theta_g + off + j); uv[j] = u[off + j]; }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      const Range rg = stored_range(scales, offsets, k, grp, form);
      const uint8_t* crow = codes.p[k] + row * row_bytes;
      int q[8];
      if (VEC) {
        load_levels8(crow, c, q, bits, form.code_bias);
      } else {
        const unsigned int p = crow[c / W];
        for (int j = 0; j < W; ++j) q[j] = (int)((p >> (bits * j)) & ((1u << bits) - 1u)) - form.code_bias;
      }
      for (int j = 0; j < W; ++j) acc[j] += dequant_level(q[j], rg, form);
    }
    for (int j = 0; j < W; ++j) outer_update<GT>(tg[j], uv[j], __fmul_rn(acc[j], inv_k), eta, mu, nesterov);
    if (VEC) {
      Vec8<GT>::store(theta_g + off, tg);
      Vec8<float>::store(u + off, uv);
      if (write_back)
        for (int k = 0; k < K; ++k) Vec8<WT>::store(reinterpret_cast<WT*>(w.p[k]) + off, tg);
    } else {
      for (int j = 0; j < W; ++j) {
        Vec8<GT>::store1(theta_g + off + j, tg[j]);
        u[off + j] = uv[j];
        if (write_back)
          for (int k = 0; k < K; ++k) Vec8<WT>::store1(reinterpret_cast<WT*>(w.p[k]) + off + j, tg[j]);
      }
    }
  }
}

// ---- top-k sparsification (Sec. 2 "Compressed Communication") --------------------------
// Of each matrix of each worker the k entries of largest magnitude are kept (all entries
// that tie with the k-th one included).  The k-th largest magnitude is found exactly by a
// radix select over the bit pattern of |v| (ordered like an unsigned for non-negative
// floats; bit 31 is always clear): three passes with digits of 11, 10 and 10 bits, each a
// histogram of the entries that match the digits found so far, then the digit in which the
// k-th entry falls.
__global__ void topk_init_kernel(TopkState* st, unsigned int kcount) {
  TopkState& s = st[blockIdx.x];
  for (int i = threadIdx.x; i < TOPK_BINS; i += blockDim.x) s.hist[i] = 0u;
  if (threadIdx.x == 0) { s.prefix = 0u; s.mask = 0u; s.rank = kcount; s.pad = 0u; }
}

template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void topk_hist_kernel(
    WorkerPtrs w, const GT* __restrict__ theta_g, ResidualPtrs ef, TopkState* st, long elems, int count,
    int shift, int nbins, float ef_beta) {
  __shared__ unsigned int lh[OT_THREADS / 64][TOPK_BINS];     // one histogram per wavefront
  const long b = blockIdx.y;
  const int k = blockIdx.z;
  TopkState& s = st[(long)k * count + b];
  const unsigned int prefix = s.prefix, mask = s.mask;
  const unsigned int digit_mask = (unsigned int)nbins - 1u;
  for (int wv = 0; wv < OT_THREADS / 64; ++wv)
    for (int i = threadIdx.x; i < nbins; i += OT_THREADS) lh[wv][i] = 0u;
  __syncthreads();
  unsigned int* mine = lh[threadIdx.x >> 6];
  const GT* tg = theta_g + b * elems;
  const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + b * elems;
  const float* res = ef.p[k] ? ef.p[k] + b * elems : nullptr;
  constexpr int W = VEC ? 8 : 1;
  unsigned int cur = 0xffffffffu, run = 0u;       // run-length of the current digit
  for (long i = ((long)blockIdx.x * OT_THREADS + threadIdx.x) * W; i < elems;
       i += (long)gridDim.x * OT_THREADS * W) {
    float a[8], c[8], e[8];
    if (VEC) {
      Vec8<GT>::load(tg + i, a); Vec8<WT>::load(tk + i, c);
      if (res) Vec8<float>::load(res + i, e);
    } else {
      a[0] = Vec8<GT>::load1(tg + i); c[0] = Vec8<WT>::load1(tk + i);
      if (res) e[0] = res[i];
    }
#pragma unroll
    for (int j = 0; j < W; ++j) {
      const float d = a[j] - c[j];
      const float v = res ? ef_input(d, e[j], ef_beta) : d;
      const unsigned int key = __float_as_uint(fabsf(v));
      if ((key & mask) == prefix) {
        const unsigned int bin = (key >> shift) & digit_mask;
        if (bin == cur) {
          ++run;
        } else {
          if (run) atomicAdd(&mine[cur], run);
          cur = bin; run = 1u;
        }
      }
    }
  }
  if (run) atomicAdd(&mine[cur], run);
  __syncthreads();
  for (int i = threadIdx.x; i < nbins; i += OT_THREADS) {
    unsigned int tot = 0u;
#pragma unroll
    for (int wv = 0; wv < OT_THREADS / 64; ++wv) tot += lh[wv][i];
    if (tot) atomicAdd(&s.hist[i], tot);
  }
}

// The digit that holds the k-th largest entry: the highest bin b for which the bins b and
// above hold at least `rank` entries (bin 0 if none does).  Thread t owns the PER = nbins / 256
// adjacent bins [PER t, PER (t + 1)); a suffix scan over the per-thread sums finds the owner.
__global__ __launch_bounds__(256) void topk_pick_kernel(TopkState* st, int shift, int nbins) {
  TopkState& s = st[blockIdx.x];
  __shared__ unsigned int suffix[256];       // entries in the bins of threads t .. 255
  const int t = threadIdx.x;
  const int per = nbins / 256;               // 8 or 4
  constexpr int MAX_PER = TOPK_BINS / 256;
  unsigned int h[MAX_PER];
  unsigned int mine = 0u;
#pragma unroll
  for (int i = 0; i < MAX_PER; ++i) {
    h[i] = i < per ? s.hist[t * per + i] : 0u;
    mine += h[i];
  }
  suffix[t] = mine;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    const unsigned int add = t + off < 256 ? suffix[t + off] : 0u;
    __syncthreads();
    suffix[t] += add;
    __syncthreads();
  }
  const unsigned int rank = s.rank;
  const unsigned int above = suffix[t] - mine;          // entries in the bins of threads t+1 .. 255
  const unsigned int total = suffix[0];
  __syncthreads();                                       // everyone has read the old rank
#pragma unroll
  for (int i = 0; i < MAX_PER; ++i)
    if (i < per) s.hist[t * per + i] = 0u;               // ready for the next pass
  const bool owner = (above < rank && above + mine >= rank) || (t == 0 && total < rank);
  if (owner) {
    // from the thread's top bin down (bins at and beyond `per` are empty); with
    // total < rank (more entries asked for than matched) this ends in bin 0 of thread 0
    unsigned int ab = above;
    int pick = 0;
    bool found = false;
#pragma unroll
    for (int i = MAX_PER - 1; i > 0; --i) {
      if (!found) {
        if (ab + h[i] >= rank) { pick = i; found = true; }
        else ab += h[i];
      }
    }
    const unsigned int bin = (unsigned int)(t * per + pick);
    s.prefix |= bin << shift;
    s.mask |= ((unsigned int)nbins - 1u) << shift;
    s.rank = rank - ab;
  }
}

template <typename WT, typename GT, bool VEC>
__global__ __launch_bounds__(OT_THREADS) void topk_outer_kernel(
    WorkerPtrs w, GT* __restrict__ theta_g, float* __restrict__ u, ResidualPtrs ef, ScalePtrs thresholds,
    const TopkState* st, long elems, int count, int K, float ef_beta, float eta, float mu, float inv_k,
    int nesterov, int write_back) {
  __shared__ unsigned int tau[MLC_MAX_WORKERS];
  const long b = blockIdx.y;
  if (threadIdx.x < K) {
    tau[threadIdx.x] = st[(long)threadIdx.x * count + b].prefix;
    if (blockIdx.x == 0 && thresholds.p[threadIdx.x])
      thresholds.p[threadIdx.x][b] = __uint_as_float(tau[threadIdx.x]);
  }
  __syncthreads();
  GT* tg = theta_g + b * elems;
  float* ub = u + b * elems;
  constexpr int W = VEC ? 8 : 1;
  for (long i = ((long)blockIdx.x * OT_THREADS + threadIdx.x) * W; i < elems;
       i += (long)gridDim.x * OT_THREADS * W) {
    float a[8], uv[8], acc[8];
    if (VEC) { Vec8<GT>::load(tg + i, a); Vec8<float>::load(ub + i, uv); }
    else { a[0] = Vec8<GT>::load1(tg + i); uv[0] = ub[i]; }
#pragma unroll
    for (int j = 0; j < W; ++j) acc[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      const WT* tk = reinterpret_cast<const WT*>(w.p[k]) + b * elems;
      float* res = ef.p[k] ? ef.p[k] + b * elems : nullptr;
      float c[8], e[8];
      if (VEC) {
        Vec8<WT>::load(tk + i, c);
        if (res) Vec8<float>::load(res + i, e);
      } else {
        c[0] = Vec8<WT>::load1(tk + i);
        if (res) e[0] = res[i];
      }
#pragma unroll
      for (int j = 0; j < W; ++j) {
        const float d = a[j] - c[j];
        const float v = res ? ef_input(d, e[j], ef_beta) : d;
        const bool keep = __float_as_uint(fabsf(v)) >= tau[k];
        acc[j] += keep ? v : 0.f;
        e[j] = keep ? 0.f : v;           // what was not sent
      }
      if (res) {
        if (VEC) Vec8<float>::store(res + i, e);
        else res[i] = e[0];
      }
    }
#pragma unroll
    for (int j = 0; j < W; ++j) outer_update<GT>(a[j], uv[j], __fmul_rn(acc[j], inv_k), eta, mu, nesterov);
    if (VEC) {
      Vec8<GT>::store(tg + i, a);
      Vec8<float>::store(ub + i, uv);
      if (write_back)
        for (int k = 0; k < K; ++k) Vec8<WT>::store(reinterpret_cast<WT*>(w.p[k]) + b * elems + i, a);
    } else {
      Vec8<GT>::store1(tg + i, a[0]);
      ub[i] = uv[0];
      if (write_back)
        for (int k = 0; k < K; ++k) Vec8<WT>::store1(reinterpret_cast<WT*>(w.p[k]) + b * elems + i, a[0]);
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
bool has_residuals(const ResidualPtrs& ef) { return ef.p[0] != nullptr; }
}  // namespace

QuantForm make_quant_form(int bits, int offset, int64_t rows_per_range, float ef_beta) {
  QuantForm f;
  f.bits = bits;
  f.offset = offset ? 1 : 0;
  f.rows_per_range = (int)rows_per_range;
  f.levels = offset ? (float)((1 << bits) - 1) : (float)((1 << (bits - 1)) - 1);
  f.code_bias = offset ? 0 : (1 << (bits - 1));
  f.ef_beta = ef_beta;
  return f;
}

int launch_matrix_ranges(const WorkerPtrs& w, int worker_dtype, const void* theta_g, int global_dtype,
                         const ScalePtrs& scales, const OffsetPtrs& offsets, const ResidualPtrs& ef,
                         int64_t count, int64_t m, int64_t n, int K, const QuantForm& form,
                         hipStream_t stream) {
  if (count > 65535 || K > 65535) return MLC_ERR_SHAPE;
  const long elems = m * n;
  const bool vec = elems % 8 == 0;
  const int nblk = cap_blocks((elems / (vec ? 8 : 1) + OT_THREADS - 1) / OT_THREADS, 512);
  const double bytes = (double)count * elems * (K * esize(worker_dtype) + K * esize(global_dtype) +
                                                (has_residuals(ef) ? 4.0 * K : 0.0));
  LaunchScope scope(MLC_KERNEL_QUANTIZE, stream, 0.0, bytes);
  const dim3 small((unsigned)((count + 255) / 256), (unsigned)K);
  hipLaunchKernelGGL(matrix_range_init_kernel, small, dim3(256), 0, stream, scales, offsets, (long)count,
                     form.offset);
#define MLC_CALL(WT, GT)                                                                          \
  do {                                                                                            \
    if (vec)                                                                                      \
      hipLaunchKernelGGL((matrix_range_kernel<WT, GT, true>), dim3(nblk, (unsigned)count, K),      \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, scales, offsets, ef,  \
                         elems, form);                                                            \
    else                                                                                          \
      hipLaunchKernelGGL((matrix_range_kernel<WT, GT, false>), dim3(nblk, (unsigned)count, K),     \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, scales, offsets, ef,  \
                         elems, form);                                                            \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  hipLaunchKernelGGL(matrix_range_finish_kernel, small, dim3(256), 0, stream, scales, offsets, (long)count,
                     form);
  return check_launch();
}

int launch_quantize(const WorkerPtrs& w, int worker_dtype, const void* theta_g, int global_dtype,
                    const CodePtrs& codes, const ScalePtrs& scales, const OffsetPtrs& offsets,
                    const ResidualPtrs& ef, int64_t rows, int64_t n, int K, const QuantForm& form,
                    hipStream_t stream) {
  const long blocks = (rows + OT_THREADS / 64 - 1) / (OT_THREADS / 64);
  if (blocks > 0x7fffffffL) return MLC_ERR_SHAPE;
  const int bits = form.bits;
  const double bytes = (double)rows * n * (K * esize(worker_dtype) + esize(global_dtype) + bits / 8.0 * K +
                                           (has_residuals(ef) ? 8.0 * K : 0.0)) +
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
  hipLaunchKernelGGL((quantize_rows_reg_kernel<WT, GT, NV, G, false>), dim3((unsigned)nblk),       \
                     dim3(OT_THREADS), 0, stream, w, (GT*)const_cast<void*>(theta_g), (float*)nullptr, \
                     codes, scales, offsets, ef, (long)rows, (int)n, K, form, 0.f, 0.f, 0.f, 0, 0, 0, \
                     (uint8_t*)nullptr, (float*)nullptr, (float*)nullptr)
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
                         offsets, ef, (long)rows, (int)n, K, form);                               \
    else                                                                                          \
      hipLaunchKernelGGL((quantize_rows_kernel<WT, GT, false>), dim3((unsigned)blocks),           \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, codes, scales,       \
                         offsets, ef, (long)rows, (int)n, K, form);                               \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

int launch_dequant_outer(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                         float* u, const CodePtrs& codes, const ScalePtrs& scales,
                         const OffsetPtrs& offsets, int64_t rows, int64_t n, int K,
                         const QuantForm& form, float eta_out, float mu, int nesterov,
                         int write_back, hipStream_t stream) {
  const bool vec = n % 8 == 0;
  const int bits = form.bits;
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
                         stream, w, (GT*)theta_g, u, codes, scales, offsets, (long)rows, (int)n,  \
                         K, form, eta_out, mu, inv_k, nesterov, write_back);                      \
    else                                                                                          \
      hipLaunchKernelGGL((dequant_outer_kernel<WT, GT, false>), dim3(blocks), dim3(OT_THREADS), 0,\
                         stream, w, (GT*)theta_g, u, codes, scales, offsets, (long)rows, (int)n,  \
                         K, form, eta_out, mu, inv_k, nesterov, write_back);                      \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

// Returns MLC_ERR_UNSUPPORTED when the one-pass kernel does not cover the request (the
// caller then runs the quantiser and the dequantising update as two launches).
int launch_quantize_outer_fused(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype,
                                float* u, const CodePtrs& codes, const ScalePtrs& scales,
                                const OffsetPtrs& offsets, const ResidualPtrs& ef, int64_t rows,
                                int64_t n, int K, const QuantForm& form, float eta_out, float mu,
                                int nesterov, int write_back, int requant, uint8_t* mean_codes,
                                float* mean_scales, float* mean_offsets, hipStream_t stream) {
  if (n % 8 || n > 24576 || (worker_dtype == MLC_F32 && global_dtype == MLC_BF16))
    return MLC_ERR_UNSUPPORTED;
  const int g = n <= 2048 ? 64 : OT_THREADS;
  const int need = (int)((n + g * 8 - 1) / (g * 8));
  // Vectors per thread.  The row, its running mean and the current worker's delta all live in
  // registers (24 floats per vector), so the steps are fine where it buys occupancy: 6 instead
  // of 8 vectors lets two workgroups share a CU (10240 columns: 3.3 -> 4.x TB/s with K = 4).
  const int nv = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : 12;
  const long rpb = OT_THREADS / g;
  const long nblk = (rows + rpb - 1) / rpb;
  if (nblk > 0x7fffffffL) return MLC_ERR_SHAPE;
  const int bits = form.bits;
  const double bytes = (double)rows * n * (K * esize(worker_dtype) * (write_back ? 2 : 1) + bits / 8.0 * K +
                                           (has_residuals(ef) ? 8.0 * K : 0.0) +
                                           (mean_codes ? bits / 8.0 : 0.0) +
                                           2 * esize(global_dtype) + 8) + (double)rows * 4 * K;
  LaunchScope scope(MLC_KERNEL_DEQUANT_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_QO(WT, GT, NV, G)                                                                     \
  hipLaunchKernelGGL((quantize_rows_reg_kernel<WT, GT, NV, G, true>), dim3((unsigned)nblk),        \
                     dim3(OT_THREADS), 0, stream, w, (GT*)theta_g, u, codes, scales, offsets, ef,  \
                     (long)rows, (int)n, K, form, eta_out, mu, inv_k, nesterov, write_back, requant, \
                     mean_codes, mean_scales, mean_offsets)
#define MLC_QO_NV(WT, GT)                                                                         \
  do {                                                                                            \
    if (g == 64) { if (nv == 1) MLC_QO(WT, GT, 1, 64); else if (nv == 2) MLC_QO(WT, GT, 2, 64);   \
                   else MLC_QO(WT, GT, 4, 64); }                                                  \
    else { if (nv <= 2) MLC_QO(WT, GT, 2, 256); else if (nv == 4) MLC_QO(WT, GT, 4, 256);         \
           else if (nv == 6) MLC_QO(WT, GT, 6, 256);                                              \
           else if (nv == 8) MLC_QO(WT, GT, 8, 256); else MLC_QO(WT, GT, 12, 256); }              \
  } while (0)
  if (worker_dtype == MLC_BF16 && global_dtype == MLC_F32) MLC_QO_NV(bf16_t, float);
  else if (worker_dtype == MLC_BF16) MLC_QO_NV(bf16_t, bf16_t);
  else MLC_QO_NV(float, float);
#undef MLC_QO_NV
#undef MLC_QO
  return check_launch();
}

// One launch for the fused un-quantised outer step of up to OUTER_MAX_SEG groups.
int launch_outer_fused_multi(const OuterGroupArgs* gs, int ng, int worker_dtype, int global_dtype, int K,
                             float eta_out, float mu, int nesterov, int write_back, hipStream_t stream) {
  if (ng < 1 || ng > OUTER_MAX_SEG || K > OUTER_MAX_SEG_K) return MLC_ERR_UNSUPPORTED;
  OuterSegTable tab;
  tab.nseg = ng;
  double total = 0.0;
  for (int i = 0; i < ng; ++i) total += (double)gs[i].rows * (double)gs[i].n;
  // about 16 workgroups per compute unit in all, dealt in proportion to the groups' sizes
  const double budget = 256.0 * 16.0;
  unsigned int blk = 0;
  double bytes = 0.0;
  for (int i = 0; i < OUTER_MAX_SEG; ++i) {
    OuterSeg& sg = tab.s[i];
    if (i >= ng) { sg = tab.s[0]; sg.blk0 = 0xffffffffu; sg.nblk = 0; continue; }
    const long n_elems = gs[i].rows * gs[i].n;
    for (int k = 0; k < OUTER_MAX_SEG_K; ++k) sg.w.p[k] = k < K ? gs[i].w.p[k] : nullptr;
    sg.theta_g = gs[i].theta_g;
    sg.u = gs[i].u;
    sg.n_elems = n_elems;
    const long want = (n_elems / 8 + OT_THREADS - 1) / OT_THREADS;
    long nb = (long)(budget * (double)n_elems / total + 0.5);
    if (nb > want) nb = want;
    if (nb < 1) nb = 1;
    sg.blk0 = blk;
    sg.nblk = (unsigned int)nb;
    blk += (unsigned int)nb;
    bytes += (double)n_elems * (K * esize(worker_dtype) * (write_back ? 2 : 1) + 2 * esize(global_dtype) + 8);
  }
  LaunchScope scope(MLC_KERNEL_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_CALL(WT, GT)                                                                              \
  hipLaunchKernelGGL((outer_fused_multi_kernel<WT, GT>), dim3(blk), dim3(OT_THREADS), 0, stream, tab, K, \
                     eta_out, mu, inv_k, nesterov, write_back)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

// Index of the (vectors per thread, threads per row) pair of the one-pass kernel for rows of
// length n, or -1 when the one-pass kernel does not cover them.
int quant_reg_cfg(int64_t n) {
  if (n % 8 || n > 24576) return -1;
  const int g = n <= 2048 ? 64 : OT_THREADS;
  const int need = (int)((n + g * 8 - 1) / (g * 8));
  if (g == 64) return need <= 1 ? 0 : need <= 2 ? 1 : 2;
  return need <= 2 ? 3 : need <= 4 ? 4 : need <= 6 ? 5 : need <= 8 ? 6 : 7;
}

// One launch for the quantised outer step (quantise + dequantise + mean + eq. 3 + write-back)
// of up to OUTER_MAX_SEG groups; ranges per row, no second quantisation.
int launch_quantize_outer_multi(const OuterGroupArgs* gs, int ng, int worker_dtype, int global_dtype, int K,
                                const QuantForm& form, float eta_out, float mu, int nesterov, int write_back,
                                hipStream_t stream) {
  if (ng < 1 || ng > OUTER_MAX_SEG || K > OUTER_MAX_SEG_K || form.rows_per_range != 0) return MLC_ERR_UNSUPPORTED;
  if (worker_dtype == MLC_F32 && global_dtype == MLC_BF16) return MLC_ERR_UNSUPPORTED;
  QuantSegTable tab;
  tab.nseg = ng;
  unsigned long blk = 0;
  double bytes = 0.0;
  bool ef_any = false;
  for (int i = 0; i < OUTER_MAX_SEG; ++i) {
    QuantSeg& sg = tab.s[i];
    if (i >= ng) { sg = tab.s[0]; sg.blk0 = 0xffffffffu; continue; }
    const int cfg = quant_reg_cfg(gs[i].n);
    if (cfg < 0 || cfg > QUANT_MULTI_MAX_CFG) return MLC_ERR_UNSUPPORTED;
    for (int k = 0; k < OUTER_MAX_SEG_K; ++k) {
      sg.w.p[k] = k < K ? gs[i].w.p[k] : nullptr;
      sg.codes.p[k] = k < K ? gs[i].codes.p[k] : nullptr;
      sg.scales.p[k] = k < K ? gs[i].scales.p[k] : nullptr;
      sg.offsets.p[k] = k < K ? gs[i].offsets.p[k] : nullptr;
      sg.ef.p[k] = k < K ? gs[i].ef.p[k] : nullptr;
    }
    ef_any = gs[i].ef.p[0] != nullptr;
    sg.theta_g = gs[i].theta_g;
    sg.u = gs[i].u;
    sg.rows = gs[i].rows;
    sg.n = (int)gs[i].n;
    sg.cfg = cfg;
    const long rpb = OT_THREADS / reg_cfg(cfg).g;
    sg.blk0 = (unsigned int)blk;
    blk += (unsigned long)((gs[i].rows + rpb - 1) / rpb);
    if (blk > 0x7fffffffUL) return MLC_ERR_SHAPE;
    bytes += (double)gs[i].rows * gs[i].n * (K * esize(worker_dtype) * (write_back ? 2 : 1) + form.bits / 8.0 * K +
                                             (ef_any ? 8.0 * K : 0.0) + 2 * esize(global_dtype) + 8) +
             (double)gs[i].rows * 4 * K;
  }
  LaunchScope scope(MLC_KERNEL_DEQUANT_OUTER, stream, 0.0, bytes);
  const float inv_k = 1.0f / (float)K;
#define MLC_QM(WT, GT)                                                                             \
  hipLaunchKernelGGL((quantize_outer_multi_kernel<WT, GT>), dim3((unsigned)blk), dim3(OT_THREADS), 0, \
                     stream, tab, K, form, eta_out, mu, inv_k, nesterov, write_back)
  if (worker_dtype == MLC_BF16 && global_dtype == MLC_F32) MLC_QM(bf16_t, float);
  else if (worker_dtype == MLC_BF16) MLC_QM(bf16_t, bf16_t);
  else MLC_QM(float, float);
#undef MLC_QM
  return check_launch();
}

size_t topk_workspace_bytes(int64_t count, int K) { return (size_t)count * K * sizeof(TopkState); }

int launch_topk_outer(const WorkerPtrs& w, int worker_dtype, void* theta_g, int global_dtype, float* u,
                      const ResidualPtrs& ef, const ScalePtrs& thresholds, int64_t count, int64_t m,
                      int64_t n, int K, unsigned int kcount, float ef_beta, float eta_out, float mu,
                      int nesterov, int write_back, void* workspace, hipStream_t stream) {
  if (count > 65535) return MLC_ERR_SHAPE;
  TopkState* st = (TopkState*)workspace;
  const long elems = m * n;
  const bool vec = elems % 8 == 0;
  const int nblk = cap_blocks((elems / (vec ? 8 : 1) + OT_THREADS - 1) / OT_THREADS, 256);
  const int n_states = (int)(count * K);
  const double pass_bytes = (double)count * elems * (K * esize(worker_dtype) + K * esize(global_dtype) +
                                                     (has_residuals(ef) ? 4.0 * K : 0.0));
  const double last_bytes = (double)count * elems * (K * esize(worker_dtype) * (write_back ? 2 : 1) +
                                                     (has_residuals(ef) ? 8.0 * K : 0.0) +
                                                     2 * esize(global_dtype) + 8);
  LaunchScope scope(MLC_KERNEL_TOPK, stream, 0.0, 3 * pass_bytes + last_bytes);
  hipLaunchKernelGGL(topk_init_kernel, dim3(n_states), dim3(256), 0, stream, st, kcount);
  // digits of 11, 10 and 10 bits cover bits 30 .. 0 of |v|
  const int shifts[3] = {20, 10, 0}, bins[3] = {2048, 1024, 1024};
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = shifts[pass], nbins = bins[pass];
#define MLC_CALL(WT, GT)                                                                          \
  do {                                                                                            \
    if (vec)                                                                                      \
      hipLaunchKernelGGL((topk_hist_kernel<WT, GT, true>), dim3(nblk, (unsigned)count, K),         \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, ef, st, elems,       \
                         (int)count, shift, nbins, ef_beta);                                      \
    else                                                                                          \
      hipLaunchKernelGGL((topk_hist_kernel<WT, GT, false>), dim3(nblk, (unsigned)count, K),        \
                         dim3(OT_THREADS), 0, stream, w, (const GT*)theta_g, ef, st, elems,       \
                         (int)count, shift, nbins, ef_beta);                                      \
  } while (0)
    MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
    hipLaunchKernelGGL(topk_pick_kernel, dim3(n_states), dim3(256), 0, stream, st, shift, nbins);
  }
  const float inv_k = 1.0f / (float)K;
#define MLC_CALL(WT, GT)                                                                          \
  do {                                                                                            \
    if (vec)                                                                                      \
      hipLaunchKernelGGL((topk_outer_kernel<WT, GT, true>), dim3(nblk, (unsigned)count),           \
                         dim3(OT_THREADS), 0, stream, w, (GT*)theta_g, u, ef, thresholds, st, elems, \
                         (int)count, K, ef_beta, eta_out, mu, inv_k, nesterov, write_back);       \
    else                                                                                          \
      hipLaunchKernelGGL((topk_outer_kernel<WT, GT, false>), dim3(nblk, (unsigned)count),          \
                         dim3(OT_THREADS), 0, stream, w, (GT*)theta_g, u, ef, thresholds, st, elems, \
                         (int)count, K, ef_beta, eta_out, mu, inv_k, nesterov, write_back);       \
  } while (0)
  MLC_DISPATCH2(worker_dtype, global_dtype, MLC_CALL);
#undef MLC_CALL
  return check_launch();
}

}  // namespace mlc
