// Batched bf16 matrix-core GEMM for the three products of a Newton-Schulz iteration
// (paper Sec. 2 "Muon": Gram matrix X X^T, polynomial b A + c A^2, product with X).
//
// One workgroup = 256 threads = 4 wavefronts in a 2 x 2 arrangement; each wavefront owns a
// (BM/2) x (BN/2) block of the output tile as TM x TN accumulators of v_mfma_f32_32x32x16_bf16.
// Tiles of both operands are staged through LDS (double buffered, one barrier per 64-deep
// K step) from registers that were filled by the previous step's global loads.
//
// An operand whose K index is the slow one in memory ("K-strided": X in B'X for wide
// matrices, both operands of X^T X for tall ones) is never transposed in HBM.  Its tile is
// stored in LDS as it is in memory ([k][row]) and each lane reads, for 8 consecutive k,
// the TT adjacent rows it owns, then regroups 16-bit halves in registers.  This works
// because a lane of the 32-wide MFMA may own any row, as long as the epilogue knows which:
// lane l of accumulator tile t owns row  TT*(l%32) + t  of the wavefront's block, so the TT
// values a lane needs are adjacent in memory.  K-contiguous operands use the same
// interleaved ownership so that a lane's TN output columns are adjacent and are stored
// as one 4- or 8-byte word.
#include "common.h"

namespace mlc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BK = 64;           // K depth of one LDS stage
constexpr int NTHREADS = 256;
constexpr int NUM_XCD = 8;

struct GemmArgs {
  const bf16_t* A; long lda, strideA;
  const bf16_t* B; long ldb, strideB;
  bf16_t* D; long ldd, strideD;
  const bf16_t* C; long ldc, strideC;
  int K, batch;
  int tiles_m, tiles_n, total_tiles, tiles_per_xcd;
  float alpha, beta, gamma;
  const float* bscale; int bscale_pow;
};

// ---- global -> register staging of one operand tile (R rows x 64 k) -----------------
template <int R, bool KS>
struct TileLoader {
  static constexpr int NCH = R / 32;            // 16-byte chunks per thread
  static constexpr int CPR = R / 8;             // chunks per k-row when K-strided
  const bf16_t* ptr;                            // this thread's first chunk at k-step 0
  long it_stride;                               // elements between a thread's chunks
  long k_stride;                                // elements per K step
  int lds_off;                                  // byte offset of the first chunk in the stage
  static constexpr int LDS_IT = 4096;           // bytes between a thread's chunks in LDS

  template <int TT>
  __device__ __forceinline__ void init(const bf16_t* base, long ld, int row0, int tid) {
    if constexpr (!KS) {
      const int row = tid >> 3, ch = tid & 7;
      ptr = base + (long)(row0 + row) * ld + ch * 8;
      it_stride = 32 * ld;
      k_stride = BK;
      lds_off = row * 128 + ((ch ^ ((row / TT) & 7)) << 4);
    } else {
      const int krow = tid / CPR, ch = tid % CPR;
      ptr = base + (long)krow * ld + row0 + ch * 8;
      it_stride = (long)(NTHREADS / CPR) * ld;
      k_stride = (long)BK * ld;
      lds_off = krow * (R * 2) + ch * 16;
    }
  }
  __device__ __forceinline__ void load(u32x4 (&regs)[NCH], int kt) const {
    const bf16_t* p = ptr + (long)kt * k_stride;
#pragma unroll
    for (int it = 0; it < NCH; ++it)
      regs[it] = *reinterpret_cast<const u32x4*>(p + it * it_stride);
  }
  __device__ __forceinline__ void store(const u32x4 (&regs)[NCH], unsigned char* stage) const {
#pragma unroll
    for (int it = 0; it < NCH; ++it)
      *reinterpret_cast<u32x4*>(stage + lds_off + it * LDS_IT) = regs[it];
  }
};

// ---- LDS -> MFMA fragments ------------------------------------------------------------
// K-contiguous stage: [R][64] bf16, 16-byte chunks XOR-swizzled by (row / TT) & 7.
template <int TT>
__device__ __forceinline__ void read_frags_kc(const unsigned char* stage, int wbase, int l32,
                                              int lg, int kk, u32x4 (&frag)[TT]) {
  const int chunk = kk * 2 + lg;
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int row = wbase + TT * l32 + t;
    frag[t] = *reinterpret_cast<const u32x4*>(stage + row * 128 + ((chunk ^ (l32 & 7)) << 4));
  }
}

// K-strided stage: [64][R] bf16.  Lane reads TT adjacent rows for each of its 8 k values.
template <int R, int TT>
__device__ __forceinline__ void read_frags_ks(const unsigned char* stage, int wbase, int l32,
                                              int lg, int kk, u32x4 (&frag)[TT]) {
  const unsigned char* p = stage + (kk * 16 + lg * 8) * (R * 2) + (wbase + TT * l32) * 2;
  if constexpr (TT == 2) {
    unsigned int raw[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) raw[t] = *reinterpret_cast<const unsigned int*>(p + t * (R * 2));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      frag[0][q] = (raw[2 * q] & 0xffffu) | (raw[2 * q + 1] << 16);
      frag[1][q] = (raw[2 * q] >> 16) | (raw[2 * q + 1] & 0xffff0000u);
    }
  } else {
    static_assert(TT == 4, "tile interleave is 2 or 4");
    u32x2 raw[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) raw[t] = *reinterpret_cast<const u32x2*>(p + t * (R * 2));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      frag[0][q] = (raw[2 * q].x & 0xffffu) | (raw[2 * q + 1].x << 16);
      frag[1][q] = (raw[2 * q].x >> 16) | (raw[2 * q + 1].x & 0xffff0000u);
      frag[2][q] = (raw[2 * q].y & 0xffffu) | (raw[2 * q + 1].y << 16);
      frag[3][q] = (raw[2 * q].y >> 16) | (raw[2 * q + 1].y & 0xffff0000u);
    }
  }
}

template <int BM, int BN, bool AKS, bool BKS>
__global__ __launch_bounds__(NTHREADS) void ns_gemm_bf16_kernel(GemmArgs g) {
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto sA = [&](int buf) { return smem + buf * A_BYTES; };
  auto sB = [&](int buf) { return smem + 2 * A_BYTES + buf * B_BYTES; };

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
  // tiles so that the tiles sharing operand panels also share that XCD's L2.
  const int bid = blockIdx.x;
  const int logical = (bid % NUM_XCD) * g.tiles_per_xcd + bid / NUM_XCD;
  if (logical >= g.total_tiles) return;
  const int per_mat = g.tiles_m * g.tiles_n;
  const int b = logical / per_mat;
  const int rem = logical - b * per_mat;
  const int tile_m = rem / g.tiles_n, tile_n = rem - tile_m * g.tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int wbase_m = wm * (BM / 2), wbase_n = wn * (BN / 2);

  TileLoader<BM, AKS> ldA;
  TileLoader<BN, BKS> ldB;
  ldA.template init<TM>(g.A + (long)b * g.strideA, g.lda, m0, tid);
  ldB.template init<TN>(g.B + (long)b * g.strideB, g.ldb, n0, tid);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[TileLoader<BM, AKS>::NCH], rb[TileLoader<BN, BKS>::NCH];
  const int KT = g.K / BK;
  ldA.load(ra, 0);
  ldB.load(rb, 0);
  ldA.store(ra, sA(0));
  ldB.store(rb, sB(0));
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) {
      ldA.load(ra, kt + 1);
      ldB.load(rb, kt + 1);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      u32x4 fa[TM], fb[TN];
      if constexpr (AKS) read_frags_ks<BM, TM>(sA(cur), wbase_m, l32, lg, kk, fa);
      else read_frags_kc<TM>(sA(cur), wbase_m, l32, lg, kk, fa);
      if constexpr (BKS) read_frags_ks<BN, TN>(sB(cur), wbase_n, l32, lg, kk, fb);
      else read_frags_kc<TN>(sB(cur), wbase_n, l32, lg, kk, fb);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, fa[i]), __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
    }
    if (more) {
      ldA.store(ra, sA(cur ^ 1));
      ldB.store(rb, sB(cur ^ 1));
    }
    __syncthreads();
  }

  // ---- epilogue: D = alpha_b * acc + beta * C + gamma * I ---------------------------
  float alpha = g.alpha;
  if (g.bscale) {
    const float s = g.bscale[b];
    alpha *= (g.bscale_pow == 2) ? s * s : s;
  }
  bf16_t* Dp = g.D + (long)b * g.strideD;
  const bf16_t* Cp = g.C ? g.C + (long)b * g.strideC : nullptr;
  const int col0 = n0 + wbase_n + TN * l32;      // this lane's TN adjacent columns
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rho = 8 * (r >> 2) + 4 * lg + (r & 3);   // row of the 32 x 32 accumulator
      const int row = m0 + wbase_m + TM * rho + i;
      float v[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) v[j] = alpha * acc[i][j][r];
      if (Cp) {
        const bf16_t* c = Cp + (long)row * g.ldc + col0;
        if constexpr (TN == 2) {
          const unsigned int w = *reinterpret_cast<const unsigned int*>(c);
          v[0] += g.beta * bf16lo(w);
          v[1] += g.beta * bf16hi(w);
        } else {
          const u32x2 w = *reinterpret_cast<const u32x2*>(c);
          v[0] += g.beta * bf16lo(w.x);
          v[1] += g.beta * bf16hi(w.x);
          v[2] += g.beta * bf16lo(w.y);
          v[3] += g.beta * bf16hi(w.y);
        }
      }
      if (g.gamma != 0.f) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          if (row == col0 + j) v[j] += g.gamma;
      }
      bf16_t* d = Dp + (long)row * g.ldd + col0;
      if constexpr (TN == 2) {
        *reinterpret_cast<unsigned int*>(d) = pack_bf16x2(v[0], v[1]);
      } else {
        u32x2 w;
        w.x = pack_bf16x2(v[0], v[1]);
        w.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<u32x2*>(d) = w;
      }
    }
  }
}

template <int BM, int BN, bool AKS, bool BKS>
int launch_cfg(const GemmDesc& d, hipStream_t stream) {
  GemmArgs g;
  g.A = d.A; g.lda = d.lda; g.strideA = d.strideA;
  g.B = d.B; g.ldb = d.ldb; g.strideB = d.strideB;
  g.D = d.D; g.ldd = d.ldd; g.strideD = d.strideD;
  g.C = d.C; g.ldc = d.ldc; g.strideC = d.strideC;
  g.K = d.K; g.batch = d.batch;
  g.tiles_m = d.M / BM; g.tiles_n = d.N / BN;
  const long total = (long)g.tiles_m * g.tiles_n * d.batch;
  if (total <= 0 || total > (1L << 30)) return MLC_ERR_SHAPE;
  g.total_tiles = (int)total;
  g.tiles_per_xcd = (int)((total + NUM_XCD - 1) / NUM_XCD);
  g.alpha = d.alpha; g.beta = d.beta; g.gamma = d.gamma;
  g.bscale = d.bscale; g.bscale_pow = d.bscale_pow;
  const size_t lds = 2 * (size_t)(BM + BN) * BK * 2;
  auto kern = ns_gemm_bf16_kernel<BM, BN, AKS, BKS>;
  static bool attr_set = false;   // per instantiation; raising the LDS limit is idempotent
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return MLC_ERR_LAUNCH;
    attr_set = true;
  }
  const double flops = 2.0 * d.M * d.N * (double)d.K * d.batch;
  LaunchScope scope(MLC_KERNEL_NS_GEMM, stream, flops, 0.0);
  hipLaunchKernelGGL(kern, dim3(g.tiles_per_xcd * NUM_XCD), dim3(NTHREADS), lds, stream, g);
  return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH;
}

template <int BM, int BN>
int launch_layout(const GemmDesc& d, hipStream_t stream) {
  if (!d.a_kstrided && !d.b_kstrided) return launch_cfg<BM, BN, false, false>(d, stream);
  if (!d.a_kstrided && d.b_kstrided) return launch_cfg<BM, BN, false, true>(d, stream);
  if (d.a_kstrided && d.b_kstrided) return launch_cfg<BM, BN, true, true>(d, stream);
  return MLC_ERR_UNSUPPORTED;
}

}  // namespace

int launch_ns_gemm(const GemmDesc& d, hipStream_t stream) {
  if (d.M % 128 || d.N % 128 || d.K % BK || d.M <= 0 || d.N <= 0 || d.K <= 0 || d.batch <= 0)
    return MLC_ERR_SHAPE;
  if ((d.lda | d.ldb | d.ldd | d.strideA | d.strideB | d.strideD) % 8) return MLC_ERR_SHAPE;
  if (d.C && ((d.ldc | d.strideC) % 8)) return MLC_ERR_SHAPE;
  const long tiles256 = (long)(d.M / 256) * (d.N / 256) * d.batch;
  if (d.M % 256 == 0 && d.N % 256 == 0 && tiles256 >= 256) return launch_layout<256, 256>(d, stream);
  return launch_layout<128, 128>(d, stream);
}

}  // namespace mlc
