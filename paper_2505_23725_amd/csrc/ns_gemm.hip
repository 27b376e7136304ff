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
#include <type_traits>

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
  int tiles_m, tiles_n, tiles_per_mat, total_tiles, tiles_per_xcd, wg_per_xcd;
  int symmetric;
  float alpha, beta, gamma;
  const float* bscale; int bscale_pow;
};

// K-contiguous stage layout: [R row slots][8 chunks of 16 B].  The LDS has 64 four-byte
// banks and serves a 128-bit read 16 lanes at a time, so the 16 chunks read by lanes
// 0-15 (same k chunk, rows TT apart) must land on 16 different 16-byte columns of the
// 256-byte bank line.  Row r therefore lives in slot kc_slot(r) = r with bit 0 and bit
// log2(TT) exchanged (rows TT apart alternate between the two 128-byte halves), and chunk c
// of row r sits at position c ^ ((r / (2 TT)) & 7) inside the slot.
template <int TT>
__device__ __forceinline__ int kc_slot(int row) {
  constexpr int HB = TT == 4 ? 2 : 1;             // log2(TT)
  const int b0 = row & 1, bh = (row >> HB) & 1;
  return (row & ~(1 | (1 << HB))) | (b0 << HB) | bh;
}

// ---- global -> register staging of one operand tile (R rows x 64 k) -----------------
// Loads go through a raw buffer resource on the matrix (base in SGPRs, one 32-bit lane
// offset in a VGPR, everything that changes per chunk or per K step in a scalar offset),
// so the loader costs one address VGPR instead of a 64-bit pointer per chunk.
template <int R, bool KS>
struct TileLoader {
  static constexpr int NCH = R / 32;            // 16-byte chunks per thread
  static constexpr int CPR = R / 8;             // chunks per k-row when K-strided
  __amdgpu_buffer_rsrc_t rsrc;                  // the matrix (at most 4 GiB)
  unsigned int voff;                            // lane's byte offset of its first chunk, k = 0
  unsigned int voff_odd;                        // same for odd chunk indices (K-contiguous, TT = 4)
  unsigned int it_stride;                       // bytes between a thread's chunks
  unsigned int k_stride;                        // bytes per K step
  int lds_off;                                  // byte offset of the first chunk in the stage
  static constexpr int LDS_IT = 4096;           // bytes between a thread's chunks in LDS

  template <int TT>
  __device__ __forceinline__ void init(const bf16_t* base, long ld, int row0, int tid) {
    rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(base), 0, 0xffffffff, 0x00020000);
    if constexpr (!KS) {
      // LDS is written linearly (slot = tid); the thread picks the global chunk that
      // belongs in its slot under the K-contiguous stage layout (see kc_slot below).
      const int slot = tid >> 3, pos = tid & 7;
      const int row = kc_slot<TT>(slot);             // the bit swap is its own inverse
      const int ch = pos ^ ((row / (2 * TT)) & 7);
      voff = (unsigned int)(((long)(row0 + row) * ld + ch * 8) * 2);
      // chunk `it` of a thread is 32 rows further down; with TT = 4 that flips bit 2 of the
      // row's swizzle on odd `it`
      voff_odd = TT == 4 ? (unsigned int)(((long)(row0 + row) * ld + (ch ^ 4) * 8) * 2) : voff;
      it_stride = (unsigned int)(32 * ld * 2);
      k_stride = BK * 2;
      lds_off = tid * 16;
    } else {
      const int krow = tid / CPR, ch = tid % CPR;
      voff = (unsigned int)(((long)krow * ld + row0 + ch * 8) * 2);
      voff_odd = voff;
      it_stride = (unsigned int)((NTHREADS / CPR) * ld * 2);
      k_stride = (unsigned int)(BK * ld * 2);
      lds_off = krow * (R * 2) + ch * 16;
    }
  }
  __device__ __forceinline__ u32x4 load_chunk(int it, int kt) const {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (it & 1) ? voff_odd : voff,
                                                 kt * k_stride + it * it_stride, 0);
  }
  __device__ __forceinline__ void load(u32x4 (&regs)[NCH], int kt) const {
#pragma unroll
    for (int it = 0; it < NCH; ++it) regs[it] = load_chunk(it, kt);
  }
  __device__ __forceinline__ void store(const u32x4 (&regs)[NCH], unsigned char* stage) const {
#pragma unroll
    for (int it = 0; it < NCH; ++it)
      *reinterpret_cast<u32x4*>(stage + lds_off + it * LDS_IT) = regs[it];
  }
  // chunks [PART * NCH / 3, (PART + 1) * NCH / 3): a third of the tile per call
  template <int PART>
  __device__ __forceinline__ void store_part(const u32x4 (&regs)[NCH], unsigned char* stage) const {
#ifdef MLC_PROBE_SKIP_LDS_STORE
    if (regs[0].x != 0x7fc12345u) return;
#endif
#pragma unroll
    for (int it = PART * NCH / 3; it < (PART + 1) * NCH / 3; ++it)
      *reinterpret_cast<u32x4*>(stage + lds_off + it * LDS_IT) = regs[it];
  }
  template <int PART>
  static constexpr int part_count() { return (PART + 1) * NCH / 3 - PART * NCH / 3; }
  template <int PART>
  __device__ __forceinline__ void load_part(u32x4 (&regs)[NCH], int kt) const {
#pragma unroll
    for (int it = PART * NCH / 3; it < (PART + 1) * NCH / 3; ++it) regs[it] = load_chunk(it, kt);
  }
};

// ---- LDS -> MFMA fragments ------------------------------------------------------------
// Reading one operand's fragments for one 16-deep k slice is split in two so that the LDS
// reads can be issued one slice ahead of the MFMAs that consume them:
//   issue()  : LDS loads into raw registers
//   finish() : raw registers -> TT fragments of 8 bf16 (a no-op for K-contiguous tiles,
//              sixteen-bit regrouping for K-strided ones)
// K-contiguous stage: [R][64] bf16 in the bank-conflict-free slot order of kc_slot.
// K-strided stage:    [64][R] bf16; a lane reads its TT adjacent rows for each of its 8 k.
// One v_perm_b32 each: the low (high) 16-bit halves of x and y, x in the low half.
__device__ __forceinline__ unsigned int pair_lo(unsigned int x, unsigned int y) {
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ unsigned int pair_hi(unsigned int x, unsigned int y) {
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

template <int R, int TT, bool KS>
struct FragReader {
  static constexpr int NRAW = KS ? (TT == 2 ? 8 : 16) : 4 * TT;   // raw dwords
  static constexpr int NLOADS = KS ? 8 : TT;                      // LDS read instructions
  static constexpr int NPERM = KS ? 4 * TT : 0;                   // regrouping instructions
  unsigned int raw[NRAW];
  int off;     // lane's byte offset inside a stage for k slice 0

  __device__ __forceinline__ void init(int wbase, int l32, int lg) {
    if constexpr (KS) off = lg * 8 * (R * 2) + (wbase + TT * l32) * 2;
    else off = (wbase + 2 * TT * (l32 >> 1) + (l32 & 1)) * 128;   // slot of row TT * l32
    lane_swz = (l32 >> 1) & 7;
    lane_lg = lg;
  }
  int lane_swz, lane_lg;

  __device__ __forceinline__ void issue(const unsigned char* stage, int kk) {
    if constexpr (KS) {
      const unsigned char* p = stage + off + kk * 16 * (R * 2);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        if constexpr (TT == 2) {
          raw[t] = *reinterpret_cast<const unsigned int*>(p + t * (R * 2));
        } else {
          const u32x2 v = *reinterpret_cast<const u32x2*>(p + t * (R * 2));
          raw[2 * t] = v.x;
          raw[2 * t + 1] = v.y;
        }
      }
    } else {
      const int chunk = ((kk * 2 + lane_lg) ^ lane_swz) << 4;
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        // row TT * l32 + t: bit 0 of t moves up to bit log2(TT) of the slot, bit 1 stays
        constexpr int SLOT_T[4] = {0, TT, 2, TT + 2};
        const u32x4 v = *reinterpret_cast<const u32x4*>(stage + off + SLOT_T[t] * 128 + chunk);
        raw[4 * t] = v.x; raw[4 * t + 1] = v.y; raw[4 * t + 2] = v.z; raw[4 * t + 3] = v.w;
      }
    }
  }
  __device__ __forceinline__ void finish(u32x4 (&frag)[TT]) const {
    if constexpr (!KS) {
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        frag[t].x = raw[4 * t]; frag[t].y = raw[4 * t + 1]; frag[t].z = raw[4 * t + 2]; frag[t].w = raw[4 * t + 3];
      }
    } else if constexpr (TT == 2) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        frag[0][q] = pair_lo(raw[2 * q], raw[2 * q + 1]);
        frag[1][q] = pair_hi(raw[2 * q], raw[2 * q + 1]);
      }
    } else {
      static_assert(!KS || TT == 2 || TT == 4, "tile interleave is 2 or 4");
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        // raw[2t], raw[2t+1] = the 4 adjacent rows at k = t; pair k = 2q with k = 2q+1
        frag[0][q] = pair_lo(raw[4 * q], raw[4 * q + 2]);
        frag[1][q] = pair_hi(raw[4 * q], raw[4 * q + 2]);
        frag[2][q] = pair_lo(raw[4 * q + 1], raw[4 * q + 3]);
        frag[3][q] = pair_hi(raw[4 * q + 1], raw[4 * q + 3]);
      }
    }
  }
};

// Scheduling hint for one k slice (sched_group_barrier masks): the memory instructions
// (LDS reads and writes, global loads) go between the first MFMAs of the slice, the VALU
// regrouping of the fragments just read goes between the last ones, by which time the LDS
// reads it depends on have returned.
template <int NMFMA, int DSR, int DSW, int VMEM, int VALU>
__device__ __forceinline__ void interleave_hint() {
  constexpr int NMEM = VALU > 0 ? NMFMA / 2 : NMFMA;      // MFMAs that carry memory instructions
  constexpr int NVAL = NMFMA - NMEM;
  constexpr int r = (DSR + NMEM - 1) / NMEM, w = (DSW + NMEM - 1) / NMEM, v = (VMEM + NMEM - 1) / NMEM;
  constexpr int a = NVAL > 0 ? (VALU + NVAL - 1) / NVAL : 0;
#pragma unroll
  for (int i = 0; i < NMFMA; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (i < NMEM) {
      if (r > 0 && i * r < DSR) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
      if (w > 0 && i * w < DSW) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);
      if (v > 0 && i * v < VMEM) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
    } else {
      if (a > 0 && (i - NMEM) * a < VALU) __builtin_amdgcn_sched_group_barrier(0x002, a, 0);
    }
  }
}

// Position of an output tile.
struct TileCoord { int b, m0, n0; bool mirror; };

// Epilogue of one tile: D = alpha_b * acc + beta * C + gamma * I, stored as bf16.  With
// tc.mirror the transposed tile is stored as well (symmetric outputs compute only the lower
// triangle of tiles).  HAS_C is compile-time so that the C loads can be issued back to back.
template <int TM, int TN, bool HAS_C>
__device__ __forceinline__ void store_tile(const GemmArgs& g, const f32x16 (&acc)[TM][TN],
                                           const TileCoord& tc, float alpha, bool on_diag,
                                           int wbase_m, int wbase_n, int l32, int lg) {
  // Lane owns TN adjacent columns; accumulator register r of tile i is row
  // TM * (8 * (r / 4) + 4 * lg + r % 4) + i of the wavefront's block: for a fixed r / 4 that
  // is 4 * TM consecutive rows.  All accesses go through buffer resources on the batch's
  // matrix: one lane offset in a VGPR, the row offset in a scalar register.
  const int col0 = tc.n0 + wbase_n + TN * l32;
  const int row_lane = tc.m0 + wbase_m + TM * 4 * lg;
  const __amdgpu_buffer_rsrc_t rd =
      __builtin_amdgcn_make_buffer_rsrc(g.D + (long)tc.b * g.strideD, 0, 0xffffffff, 0x00020000);
  const unsigned int ldd2 = (unsigned int)(g.ldd * 2), ldc2 = (unsigned int)(g.ldc * 2);
  const unsigned int voff_d = (unsigned int)(((long)row_lane * g.ldd + col0) * 2);
  const unsigned int voff_m = (unsigned int)(((long)col0 * g.ldd + row_lane) * 2);   // transposed
  const unsigned int voff_c = HAS_C ? (unsigned int)(((long)row_lane * g.ldc + col0) * 2) : 0u;
  __amdgpu_buffer_rsrc_t rc = rd;
  if constexpr (HAS_C)
    rc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(g.C) + (long)tc.b * g.strideC, 0,
                                           0xffffffff, 0x00020000);
  const int diag = col0 - row_lane;     // row offset (within the lane's rows) that meets column col0
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    unsigned int packed[4][TM][TN / 2];                   // [r % 4][i][column pair]
    u32x2 cval[4][TM];
    if constexpr (HAS_C) {
#pragma unroll
      for (int rl = 0; rl < 4; ++rl)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const unsigned int soff = (unsigned int)(TM * (8 * q + rl) + i) * ldc2;
          if constexpr (TN == 2) cval[rl][i].x = __builtin_amdgcn_raw_buffer_load_b32(rc, voff_c, soff, 0);
          else cval[rl][i] = __builtin_amdgcn_raw_buffer_load_b64(rc, voff_c, soff, 0);
        }
    }
#pragma unroll
    for (int rl = 0; rl < 4; ++rl) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = 4 * q + rl;
        const int roff = TM * (8 * q + rl) + i;           // compile-time row offset
        float v[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) v[j] = alpha * acc[i][j][r];
        if constexpr (HAS_C) {
          v[0] += g.beta * bf16lo(cval[rl][i].x);
          v[1] += g.beta * bf16hi(cval[rl][i].x);
          if constexpr (TN == 4) {
            v[2] += g.beta * bf16lo(cval[rl][i].y);
            v[3] += g.beta * bf16hi(cval[rl][i].y);
          }
        }
        if (on_diag) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
            if (roff == diag + j) v[j] += g.gamma;
        }
        packed[rl][i][0] = pack_bf16x2(v[0], v[1]);
        if constexpr (TN == 4) packed[rl][i][1] = pack_bf16x2(v[2], v[3]);
        const unsigned int soff = (unsigned int)roff * ldd2;
        if constexpr (TN == 2) {
          __builtin_amdgcn_raw_buffer_store_b32(packed[rl][i][0], rd, voff_d, soff, 0);
        } else {
          u32x2 w;
          w.x = packed[rl][i][0];
          w.y = packed[rl][i][1];
          __builtin_amdgcn_raw_buffer_store_b64(w, rd, voff_d, soff, 0);
        }
      }
    }
    if (tc.mirror) {
      // Column col0 + j of this tile becomes a row of the mirrored tile; the lane's 4 * TM
      // consecutive rows (order: r % 4 major, i minor) become 4 * TM adjacent elements.
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        unsigned int w[2 * TM];
#pragma unroll
        for (int e = 0; e < 4 * TM; e += 2) {
          // elements e and e + 1: (rl, i) = (e / TM, e % TM) and the next i
          const unsigned int lo = packed[e / TM][e % TM][j / 2];
          const unsigned int hi = packed[(e + 1) / TM][(e + 1) % TM][j / 2];
          w[e / 2] = (j & 1) ? pair_hi(lo, hi) : pair_lo(lo, hi);
        }
        const unsigned int soff = (unsigned int)j * ldd2 + (unsigned int)(TM * 8 * q) * 2;
#pragma unroll
        for (int x = 0; x < 2 * TM; x += 4) {
          u32x4 ww;
          ww.x = w[x]; ww.y = w[x + 1]; ww.z = w[x + 2]; ww.w = w[x + 3];
          __builtin_amdgcn_raw_buffer_store_b128(ww, rd, voff_m, soff + x * 4, 0);
        }
      }
    }
  }
}

// Persistent kernel: one workgroup per CU slot walks over its share of the output tiles.
// Workgroups are dealt round-robin to the 8 XCDs, so XCD x owns the contiguous range of
// tiles [x * tiles_per_xcd, (x + 1) * tiles_per_xcd) and its workgroups take them in
// order: tiles that share operand panels run at the same time behind the same L2.  The
// first global loads of the next tile are issued before the epilogue of the current one.
template <int BM, int BN, bool AKS, bool BKS>
__global__ __launch_bounds__(NTHREADS) void ns_gemm_bf16_kernel(GemmArgs g) {
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto sA = [&](int buf) { return smem + buf * A_BYTES; };
  auto sB = [&](int buf) { return smem + 2 * A_BYTES + buf * B_BYTES; };

  const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD;
  const int range_end = min((xcd + 1) * g.tiles_per_xcd, g.total_tiles);
  int logical = xcd * g.tiles_per_xcd + slot;
  if (logical >= range_end) return;

  auto decode = [&](int t) {
    TileCoord tc;
    tc.b = t / g.tiles_per_mat;
    const int rem = t - tc.b * g.tiles_per_mat;
    int tm, tn;
    if (g.symmetric) {          // lower triangle, row-major: rem = tm (tm + 1) / 2 + tn
      tm = (int)((sqrtf(8.f * (float)rem + 1.f) - 1.f) * 0.5f);
      while ((tm + 1) * (tm + 2) / 2 <= rem) ++tm;
      while (tm * (tm + 1) / 2 > rem) --tm;
      tn = rem - tm * (tm + 1) / 2;
    } else {
      tm = rem / g.tiles_n;
      tn = rem - tm * g.tiles_n;
    }
    tc.m0 = tm * BM;
    tc.n0 = tn * BN;
    tc.mirror = g.symmetric && tm != tn;
    return tc;
  };

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int wbase_m = wm * (BM / 2), wbase_n = wn * (BN / 2);

  using LoaderA = TileLoader<BM, AKS>;
  using LoaderB = TileLoader<BN, BKS>;
  using ReaderA = FragReader<BM, TM, AKS>;
  using ReaderB = FragReader<BN, TN, BKS>;
  LoaderA ldA;
  LoaderB ldB;
  // Two sets of staging registers: while one set's tile is being written to LDS, the
  // other set's global loads (two tiles ahead) are still in flight.
  u32x4 ra[2][LoaderA::NCH], rb[2][LoaderB::NCH];
  ReaderA rdA;
  ReaderB rdB;
  rdA.init(wbase_m, l32, lg);
  rdB.init(wbase_n, l32, lg);
  u32x4 fa[2][TM], fb[2][TN];
  f32x16 acc[TM][TN];
  const int KT = g.K / BK;      // even: K is a multiple of 128

  auto start_tile = [&](const TileCoord& tc) {   // loader state + the first K tile
    ldA.template init<TM>(g.A + (long)tc.b * g.strideA, g.lda, tc.m0, tid);
    ldB.template init<TN>(g.B + (long)tc.b * g.strideB, g.ldb, tc.n0, tid);
    ldA.load(ra[0], 0);
    ldB.load(rb[0], 0);
  };

  auto mfma_slice = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, fa[buf][i]), __builtin_bit_cast(bf16x8, fb[buf][j]), acc[i][j],
            0, 0, 0);
  };
  constexpr int NM = TM * TN;
  constexpr int NDSR = ReaderA::NLOADS + ReaderB::NLOADS;
  constexpr int NPERM = ReaderA::NPERM + ReaderB::NPERM;

  // One 64-deep step on stage kt & 1, software-pipelined over its four 16-deep k slices.
  // While the MFMAs of slice kk run, the LDS reads of slice kk+1 are in flight; slices 0-2
  // also move a third of tile kt+1 from its staging set to the other LDS stage, and slices
  // 1-3 issue the global loads of tile kt+3 into the registers just freed (spread out so
  // that the 64 B/clk vector-memory path never has to absorb a whole tile at once).  One
  // barrier per step, after slice 2.
  // SET: staging set that holds tile kt+1 (= (kt+1) & 1).  STORE: tile kt+1 exists and goes
  // to the other stage.  LOAD: tile kt+3 exists.
  auto kstep = [&](int kt, auto set_tag, auto store_tag, auto load_tag) {
    constexpr int SET = decltype(set_tag)::value;
    constexpr bool STORE = decltype(store_tag)::value, LOAD = decltype(load_tag)::value;
    const int cur = kt & 1;
    unsigned char* a_cur = sA(cur); unsigned char* b_cur = sB(cur);
    unsigned char* a_nxt = sA(cur ^ 1); unsigned char* b_nxt = sB(cur ^ 1);
    constexpr int P0 = LoaderA::template part_count<0>() + LoaderB::template part_count<0>();
    constexpr int P1 = LoaderA::template part_count<1>() + LoaderB::template part_count<1>();
    constexpr int P2 = LoaderA::template part_count<2>() + LoaderB::template part_count<2>();
    // slice 0
    rdA.issue(a_cur, 1); rdB.issue(b_cur, 1);
    if constexpr (STORE) { ldA.template store_part<0>(ra[SET], a_nxt); ldB.template store_part<0>(rb[SET], b_nxt); }
    mfma_slice(0);
    rdA.finish(fa[1]); rdB.finish(fb[1]);
    interleave_hint<NM, NDSR, STORE ? P0 : 0, 0, NPERM>();
    // slice 1
    rdA.issue(a_cur, 2); rdB.issue(b_cur, 2);
    if constexpr (STORE) { ldA.template store_part<1>(ra[SET], a_nxt); ldB.template store_part<1>(rb[SET], b_nxt); }
    if constexpr (LOAD) { ldA.template load_part<0>(ra[SET], kt + 3); ldB.template load_part<0>(rb[SET], kt + 3); }
    mfma_slice(1);
    rdA.finish(fa[0]); rdB.finish(fb[0]);
    interleave_hint<NM, NDSR, STORE ? P1 : 0, LOAD ? P0 : 0, NPERM>();
    // slice 2
    rdA.issue(a_cur, 3); rdB.issue(b_cur, 3);
    if constexpr (STORE) { ldA.template store_part<2>(ra[SET], a_nxt); ldB.template store_part<2>(rb[SET], b_nxt); }
    if constexpr (LOAD) { ldA.template load_part<1>(ra[SET], kt + 3); ldB.template load_part<1>(rb[SET], kt + 3); }
    mfma_slice(0);
    rdA.finish(fa[1]); rdB.finish(fb[1]);
    interleave_hint<NM, NDSR, STORE ? P2 : 0, LOAD ? P1 : 0, NPERM>();
    if constexpr (STORE) __syncthreads();
    // slice 3
    if constexpr (STORE) { rdA.issue(a_nxt, 0); rdB.issue(b_nxt, 0); }
    if constexpr (LOAD) { ldA.template load_part<2>(ra[SET], kt + 3); ldB.template load_part<2>(rb[SET], kt + 3); }
    mfma_slice(1);
    if constexpr (STORE) { rdA.finish(fa[0]); rdB.finish(fb[0]); }
    interleave_hint<NM, STORE ? NDSR : 0, 0, LOAD ? P2 : 0, STORE ? NPERM : 0>();
  };
  using T = std::true_type;
  using F = std::false_type;
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  TileCoord tc = decode(logical);
  start_tile(tc);
  while (true) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // K tile 1 -> set 1; K tile 0 -> LDS stage 0 (every wave has left the previous tile's
    // step KT-2, the last one that read stage 0, through that step's barrier); K tile 2 ->
    // set 0.
    ldA.load(ra[1], 1);
    ldB.load(rb[1], 1);
    ldA.store(ra[0], sA(0));
    ldB.store(rb[0], sB(0));
    if (KT > 2) {
      ldA.load(ra[0], 2);
      ldB.load(rb[0], 2);
    }
    __syncthreads();
    rdA.issue(sA(0), 0);
    rdB.issue(sB(0), 0);
    rdA.finish(fa[0]);
    rdB.finish(fb[0]);

    int kt = 0;
    for (; kt + 4 < KT; kt += 2) {
      kstep(kt, S1{}, T{}, T{});
      kstep(kt + 1, S0{}, T{}, T{});
    }
    if (kt + 4 == KT) {            // four steps left: only the first still has a tile to fetch
      kstep(kt, S1{}, T{}, T{});
      kstep(kt + 1, S0{}, T{}, F{});
      kt += 2;
    }
    kstep(kt, S1{}, T{}, F{});     // two steps left
    kstep(kt + 1, S0{}, F{}, F{});

    const int next = logical + g.wg_per_xcd;
    const bool more = next < range_end;
    float alpha = g.alpha;
    if (g.bscale) {
      const float sc = g.bscale[tc.b];
      alpha *= (g.bscale_pow == 2) ? sc * sc : sc;
    }
    // the diagonal crosses this tile only if its row and column ranges overlap
    const bool on_diag = g.gamma != 0.f && tc.m0 < tc.n0 + BN && tc.n0 < tc.m0 + BM;
#ifdef MLC_PROBE_SKIP_EPILOGUE
    if (alpha == 12345.f)
#endif
    {
      if (g.C) store_tile<TM, TN, true>(g, acc, tc, alpha, on_diag, wbase_m, wbase_n, l32, lg);
      else store_tile<TM, TN, false>(g, acc, tc, alpha, on_diag, wbase_m, wbase_n, l32, lg);
    }
    if (!more) break;
    logical = next;
    tc = decode(logical);
    start_tile(tc);
  }
}

int cus_per_xcd() {
  static int cached = 0;
  if (cached == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0) != hipSuccess || cus < NUM_XCD)
      cus = 256;
    cached = cus / NUM_XCD;
  }
  return cached;
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
  g.symmetric = d.symmetric ? 1 : 0;
  if (g.symmetric && (BM != BN || d.M != d.N)) return MLC_ERR_SHAPE;
  g.tiles_per_mat = g.symmetric ? g.tiles_m * (g.tiles_m + 1) / 2 : g.tiles_m * g.tiles_n;
  const long total = (long)g.tiles_per_mat * d.batch;
  if (total <= 0 || total > (1L << 30)) return MLC_ERR_SHAPE;
  g.total_tiles = (int)total;
  g.tiles_per_xcd = (int)((total + NUM_XCD - 1) / NUM_XCD);
  // one workgroup per CU for the 256 x 256 tile (128 KiB of LDS each), two for 128 x 128
  const int per_cu = (BM == 256) ? 1 : 2;
#ifdef MLC_PROBE_NONPERSISTENT
  g.wg_per_xcd = g.tiles_per_xcd; (void)per_cu;
#else
  g.wg_per_xcd = cus_per_xcd() * per_cu;
#endif
  if (g.wg_per_xcd > g.tiles_per_xcd) g.wg_per_xcd = g.tiles_per_xcd;
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
  const double flops = 2.0 * BM * BN * (double)d.K * (double)total;   // executed, not nominal
  LaunchScope scope(MLC_KERNEL_NS_GEMM, stream, flops, 0.0);
  hipLaunchKernelGGL(kern, dim3(g.wg_per_xcd * NUM_XCD), dim3(NTHREADS), lds, stream, g);
  return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH;
}

template <int BM, int BN>
int launch_layout(const GemmDesc& d, hipStream_t stream) {
  // Newton-Schulz needs only these two: a symmetric operand can be read either way, so the
  // mixed cases never arise.
  if (!d.a_kstrided && !d.b_kstrided) return launch_cfg<BM, BN, false, false>(d, stream);
  if (d.a_kstrided && d.b_kstrided) return launch_cfg<BM, BN, true, true>(d, stream);
  return MLC_ERR_UNSUPPORTED;
}

}  // namespace

int launch_ns_gemm(const GemmDesc& d, hipStream_t stream) {
  if (d.M % 128 || d.N % 128 || d.K % (2 * BK) || d.M <= 0 || d.N <= 0 || d.K <= 0 || d.batch <= 0)
    return MLC_ERR_SHAPE;
  if ((d.lda | d.ldb | d.ldd | d.strideA | d.strideB | d.strideD) % 8) return MLC_ERR_SHAPE;
  if (d.C && ((d.ldc | d.strideC) % 8)) return MLC_ERR_SHAPE;
  const long tiles256 = (long)(d.M / 256) * (d.N / 256) * d.batch;
  if (d.M % 256 == 0 && d.N % 256 == 0 && tiles256 >= 256) return launch_layout<256, 256>(d, stream);
  return launch_layout<128, 128>(d, stream);
}

}  // namespace mlc
