// Whole Newton-Schulz chain of a small matrix inside one workgroup (paper Sec. 2 "Muon":
// the quintic iteration X <- a X + b (X X^T) X + c (X X^T)^2 X, run `iters` times).
//
// For matrices whose short side pads to 128 and whose long side pads to at most 512 the
// fifteen products of the five iterations are far too small to fill the chip one launch at
// a time: their cost is launch latency and the round trips of X, A and B' through memory.
// Here one workgroup (256 threads, 4 wavefronts) owns one matrix of the batch and keeps
// X (128 x L, bf16) and the 128 x 128 matrix A = X X^T, later B' = a I + b A + c A^2, in LDS
// from the first iteration to the last; HBM is touched once to read X and once to write it.
// The arithmetic and its rounding points are those of the batched path: A, B' and X are
// rounded to bf16 where that path stores them, products accumulate in fp32 on
// v_mfma_f32_32x32x16_bf16, the normalisation s = 1/(|U| + eps) enters as a factor s^2 of the
// first Gram matrix and s of the first product with X.  The kernel forms s itself from the
// partial sums of squares that the pass which wrote U left per matrix.
//
// A tall matrix (more rows than columns) is held transposed, so that the resident X is
// always 128 x L with L >= 128: the iteration commutes with transposition.
//
// LDS layout: X is [128][LP] bf16 (LP = 128, 256 or 512), A is [128][128] bf16 behind it;
// with LP = 512 that is all 160 KiB of a CU.  The 16-byte chunk c of row r sits at position
// c ^ (r % 16) of its aligned group of 16 chunks, so that the 32 rows an MFMA operand
// fragment touches (same k chunk) spread over all banks.
#include <atomic>

#include "common.h"

namespace mlc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int S = 128;                 // padded short side
constexpr int A_PITCH = S * 2;         // bytes per row of A

struct ChainArgs {
  const bf16_t* in;        // [batch] matrices, row pitch ld, batch stride `stride` (elements)
  bf16_t* out;             // same layout
  long ld, stride;
  int tall;                // 0: matrix is 128 x L in memory ; 1: L x 128
  int L;                   // padded long side, a multiple of 128, <= LP
  const float* partials;   // per matrix nblk partial sums of squares of the input
  int nblk;
  float eps;               // scale = 1 / (sqrt(sum) + eps)
  int iters;               // >= 1
  float a, b, c;
};

// the low (high) 16-bit halves of x and y, x in the low half
__device__ __forceinline__ unsigned int halves_lo(unsigned int x, unsigned int y) {
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ unsigned int halves_hi(unsigned int x, unsigned int y) {
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

// byte offset of element (r, c) in a swizzled matrix of `pitch` bytes per row
__device__ __forceinline__ int swz_pos(int r, int c, int pitch) {
  return r * pitch + ((((c >> 3) ^ (r & 15))) << 4) + ((c & 7) << 1);
}

__device__ __forceinline__ f32x16 mfma(const u32x4& a, const u32x4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int TT>
__global__ __launch_bounds__(256) void ns_chain_small_kernel(ChainArgs g) {
  constexpr int LP = 128 * TT;
  constexpr int X_PITCH = LP * 2;
  constexpr int X_BYTES = S * X_PITCH;
  constexpr int CPR = LP / 8;              // 16-byte chunks per row of X
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* xs = smem;
  unsigned char* as = smem + X_BYTES;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;
  const bf16_t* in = g.in + (long)blockIdx.x * g.stride;
  bf16_t* out = g.out + (long)blockIdx.x * g.stride;
  const int L = g.L;
  // 1 / (|U| + eps) from the partial sums the pass that wrote U left behind (every wavefront
  // adds them up for itself, in the same order)
  float tot = 0.f;
  for (int i = lane; i < g.nblk; i += 64) tot += g.partials[(long)blockIdx.x * g.nblk + i];
  const float sumsq = wave_sum(tot);
  const float s = sumsq > 0.f ? 1.0f / (sqrtf(sumsq) + g.eps) : 0.f;   // all-zero matrix: 0, also when eps = 0

  // ---- X from memory into LDS (columns L .. LP-1 are zero) -----------------------------
  if (!g.tall) {
#pragma unroll 4
    for (int q = tid; q < S * CPR; q += 256) {
      const int r = q / CPR, ch = q % CPR;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ch * 8 < L) v = *reinterpret_cast<const u32x4*>(in + (long)r * g.ld + ch * 8);
      *reinterpret_cast<u32x4*>(xs + r * X_PITCH + ((ch ^ (r & 15)) << 4)) = v;
    }
  } else {
    // memory row rg = resident column; consecutive lanes take consecutive rg, so that the
    // 2-byte LDS stores of a wavefront fall side by side
#pragma unroll 2
    for (int q = tid; q < LP * (S / 8); q += 256) {
      const int cg = q / LP, rg = q % LP;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (rg < L) v = *reinterpret_cast<const u32x4*>(in + (long)rg * g.ld + cg * 8);
      const unsigned int w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const unsigned short h = (unsigned short)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
        *reinterpret_cast<unsigned short*>(xs + swz_pos(cg * 8 + e, rg, X_PITCH)) = h;
      }
    }
  }
  __syncthreads();

  const int wm = wave >> 1, wn = wave & 1;     // 2 x 2 wavefronts over the 128 x 128 products
  const int ra = wm * 64 + l32, rb = wn * 64 + l32;
  const int swz = l32 & 15;                    // (row % 16) of every row this lane reads as an operand
  const int cb = wave * 32 * TT;               // first column of the wavefront's block of X

  for (int it = 0; it < g.iters; ++it) {
    const float alpha_a = it == 0 ? s * s : 1.f;
    const float alpha_x = it == 0 ? s : 1.f;

    // ---- A = alpha_a X X^T : each wavefront one 64 x 64 block -------------------------
    {
      f32x16 acc[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      // four 16-deep steps per trip, so that the LDS reads of one step overlap the MFMAs of
      // another (L is a multiple of 128)
      for (int k64 = 0; k64 < L / 64; ++k64) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int chunk = (((k64 * 4 + u) * 2 + lg) ^ swz) << 4;
          u32x4 fa[2], fb[2];
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            fa[i] = *reinterpret_cast<const u32x4*>(xs + (ra + 32 * i) * X_PITCH + chunk);
            fb[i] = *reinterpret_cast<const u32x4*>(xs + (rb + 32 * i) * X_PITCH + chunk);
          }
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma(fa[i], fb[j], acc[i][j]);
        }
      }
      // The lane holds, for a fixed column, groups of 4 consecutive rows.  A is symmetric bit
      // for bit (the same products are summed in the same order for (i, j) and (j, i)), so
      // element (row, col) is stored at [col][row]: four adjacent values, one 8-byte store.
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int row0 = wm * 64 + i * 32 + q4 * 8 + lg * 4;
            const int col = wn * 64 + j * 32 + l32;
            u32x2 w;
            w.x = pack_bf16x2(alpha_a * acc[i][j][4 * q4], alpha_a * acc[i][j][4 * q4 + 1]);
            w.y = pack_bf16x2(alpha_a * acc[i][j][4 * q4 + 2], alpha_a * acc[i][j][4 * q4 + 3]);
            *reinterpret_cast<u32x2*>(as + swz_pos(col, row0, A_PITCH)) = w;
          }
    }
    __syncthreads();

    // ---- B' = c A A + b A + a I, in place over A ---------------------------------------
    {
      f32x16 acc[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll 4
      for (int k16 = 0; k16 < S / 16; ++k16) {
        const int chunk = ((k16 * 2 + lg) ^ swz) << 4;
        u32x4 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          fa[i] = *reinterpret_cast<const u32x4*>(as + (ra + 32 * i) * A_PITCH + chunk);
          fb[i] = *reinterpret_cast<const u32x4*>(as + (rb + 32 * i) * A_PITCH + chunk);   // column of A = its row
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = mfma(fa[i], fb[j], acc[i][j]);
      }
      u32x2 res[2][2][4];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int row0 = wm * 64 + i * 32 + q4 * 8 + lg * 4;
            const int col = wn * 64 + j * 32 + l32;
            const u32x2 av = *reinterpret_cast<const u32x2*>(as + swz_pos(col, row0, A_PITCH));
            float v[4];
            v[0] = g.c * acc[i][j][4 * q4] + g.b * bf16lo(av.x);
            v[1] = g.c * acc[i][j][4 * q4 + 1] + g.b * bf16hi(av.x);
            v[2] = g.c * acc[i][j][4 * q4 + 2] + g.b * bf16lo(av.y);
            v[3] = g.c * acc[i][j][4 * q4 + 3] + g.b * bf16hi(av.y);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (row0 + e == col) v[e] += g.a;
            res[i][j][q4].x = pack_bf16x2(v[0], v[1]);
            res[i][j][q4].y = pack_bf16x2(v[2], v[3]);
          }
      __syncthreads();            // every wavefront is done reading A
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int row0 = wm * 64 + i * 32 + q4 * 8 + lg * 4;
            const int col = wn * 64 + j * 32 + l32;
            *reinterpret_cast<u32x2*>(as + swz_pos(col, row0, A_PITCH)) = res[i][j][q4];
          }
    }
    __syncthreads();

    // ---- X <- alpha_x B' X, in place: each wavefront all 128 rows of 32 TT columns --------
    // Lane l of column tile t owns column cb + TT l + t: the TT values it needs from a row
    // of X are adjacent, and so are the TT results it stores.
    {
      f32x16 acc[4][TT];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.f;
      const int c0 = cb + TT * l32;
      auto step = [&](int k16) {
        const int chunk = ((k16 * 2 + lg) ^ swz) << 4;
        u32x4 fa[4], fb[TT];
#pragma unroll
        for (int i = 0; i < 4; ++i)
          fa[i] = *reinterpret_cast<const u32x4*>(as + (32 * i + l32) * A_PITCH + chunk);
        const int k0 = k16 * 16 + lg * 8;
        if constexpr (TT == 1) {
          unsigned int raw[8];
#pragma unroll
          for (int e = 0; e < 8; ++e)
            raw[e] = *reinterpret_cast<const unsigned short*>(xs + swz_pos(k0 + e, c0, X_PITCH));
#pragma unroll
          for (int q = 0; q < 4; ++q) fb[0][q] = raw[2 * q] | (raw[2 * q + 1] << 16);
        } else if constexpr (TT == 2) {
          unsigned int raw[8];
#pragma unroll
          for (int e = 0; e < 8; ++e)
            raw[e] = *reinterpret_cast<const unsigned int*>(xs + swz_pos(k0 + e, c0, X_PITCH));
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            fb[0][q] = halves_lo(raw[2 * q], raw[2 * q + 1]);
            fb[1][q] = halves_hi(raw[2 * q], raw[2 * q + 1]);
          }
        } else {
          static_assert(TT == 1 || TT == 2 || TT == 4, "L pads to 128, 256 or 512");
          u32x2 raw[8];
#pragma unroll
          for (int e = 0; e < 8; ++e)
            raw[e] = *reinterpret_cast<const u32x2*>(xs + swz_pos(k0 + e, c0, X_PITCH));
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            fb[0][q] = halves_lo(raw[2 * q].x, raw[2 * q + 1].x);
            fb[1][q] = halves_hi(raw[2 * q].x, raw[2 * q + 1].x);
            fb[2 % TT][q] = halves_lo(raw[2 * q].y, raw[2 * q + 1].y);
            fb[3 % TT][q] = halves_hi(raw[2 * q].y, raw[2 * q + 1].y);
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int t = 0; t < TT; ++t) acc[i][t] = mfma(fa[i], fb[t], acc[i][t]);
      };
      if constexpr (TT == 4) {    // 256 accumulators: a second set of fragments in flight would spill
        for (int k16 = 0; k16 < S / 16; ++k16) step(k16);
      } else {
#pragma unroll 2
        for (int k16 = 0; k16 < S / 16; ++k16) step(k16);
      }
      __syncthreads();            // every wavefront is done reading X and B'
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 32 * i + (r >> 2) * 8 + lg * 4 + (r & 3);
          unsigned char* p = xs + swz_pos(row, c0, X_PITCH);
          if constexpr (TT == 1) {
            *reinterpret_cast<unsigned short*>(p) =
                (unsigned short)(pack_bf16x2(alpha_x * acc[i][0][r], 0.f) & 0xffffu);
          } else if constexpr (TT == 2) {
            *reinterpret_cast<unsigned int*>(p) = pack_bf16x2(alpha_x * acc[i][0][r], alpha_x * acc[i][1][r]);
          } else {
            u32x2 w;
            w.x = pack_bf16x2(alpha_x * acc[i][0][r], alpha_x * acc[i][1 % TT][r]);
            w.y = pack_bf16x2(alpha_x * acc[i][2 % TT][r], alpha_x * acc[i][3 % TT][r]);
            *reinterpret_cast<u32x2*>(p) = w;
          }
        }
    }
    __syncthreads();
  }

  // ---- X back to memory (the padded columns L .. LP-1 are not stored) --------------------
  if (!g.tall) {
#pragma unroll 4
    for (int q = tid; q < S * CPR; q += 256) {
      const int r = q / CPR, ch = q % CPR;
      if (ch * 8 < L)
        *reinterpret_cast<u32x4*>(out + (long)r * g.ld + ch * 8) =
            *reinterpret_cast<const u32x4*>(xs + r * X_PITCH + ((ch ^ (r & 15)) << 4));
    }
  } else {
#pragma unroll 2
    for (int q = tid; q < LP * (S / 8); q += 256) {
      const int cg = q / LP, rg = q % LP;
      if (rg < L) {
        unsigned int h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
          h[e] = *reinterpret_cast<const unsigned short*>(xs + swz_pos(cg * 8 + e, rg, X_PITCH));
        u32x4 v;
        v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16);
        v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
        *reinterpret_cast<u32x4*>(out + (long)rg * g.ld + cg * 8) = v;
      }
    }
  }
}

template <int TT>
int launch_tt(const ChainArgs& g, int64_t count, hipStream_t stream) {
  constexpr size_t lds = (size_t)S * 128 * TT * 2 + (size_t)S * A_PITCH;
  auto kern = ns_chain_small_kernel<TT>;
  // raised once per instantiation and device; the call is idempotent
  static std::atomic<bool> attr_set[MAX_DEVICES];
  const int slot = device_slot();
  if (slot < 0 || !attr_set[slot].load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return MLC_ERR_LAUNCH;
    if (slot >= 0) attr_set[slot].store(true, std::memory_order_release);
  }
  // executed: the full Gram matrix and square (no triangle saving), all LP columns of X
  const double per_iter = 2.0 * S * S * (double)g.L + 2.0 * S * S * S + 2.0 * S * S * (128.0 * TT);
  LaunchScope scope(MLC_KERNEL_NS_GEMM, stream, per_iter * g.iters * (double)count, 0.0);
  hipLaunchKernelGGL(kern, dim3((unsigned int)count), dim3(256), lds, stream, g);
  return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH;
}

}  // namespace

bool ns_chain_small_fits(int64_t mp, int64_t np) {
  const int64_t sp = mp < np ? mp : np, lp = mp < np ? np : mp;
  return sp == S && lp <= 512;
}

int launch_ns_chain_small(const bf16_t* in, bf16_t* out, int64_t ld, int64_t stride, int64_t mp,
                          int64_t np, const float* partials, int nblk, float eps, int64_t count,
                          int iters, float a, float b, float c, hipStream_t stream) {
  if (!ns_chain_small_fits(mp, np) || mp % 128 || np % 128) return MLC_ERR_SHAPE;
  if (!in || !out || !partials) return MLC_ERR_NULL;
  if (iters < 1 || count < 1 || count > 0x7fffffff || nblk < 1) return MLC_ERR_ARG;
  const bool tall = mp > np;
  // every 16-byte access stays inside a row of the padded matrix
  if (ld % 8 || stride % 8 || ld < np || stride < mp * ld) return MLC_ERR_SHAPE;
  ChainArgs g;
  g.in = in; g.out = out; g.ld = ld; g.stride = stride;
  g.tall = tall ? 1 : 0;
  g.L = (int)(tall ? mp : np);
  g.partials = partials; g.nblk = nblk; g.eps = eps;
  g.iters = iters; g.a = a; g.b = b; g.c = c;
  if (g.L <= 128) return launch_tt<1>(g, count, stream);
  if (g.L <= 256) return launch_tt<2>(g, count, stream);
  return launch_tt<4>(g, count, stream);
}

}  // namespace mlc
