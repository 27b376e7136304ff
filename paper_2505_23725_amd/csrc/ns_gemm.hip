// Batched bf16 matrix-core GEMM for the three products of a Newton-Schulz iteration
// (paper Sec. 2 "Muon": Gram matrix X X^T, polynomial b A + c A^2, product with X).
//
// One workgroup = 256 threads = 4 wavefronts in a 2 x 2 arrangement; each wavefront owns a
// (BM/2) x (BN/2) block of the output tile as TM x TN accumulators of v_mfma_f32_32x32x16_bf16.
//
// Operand tiles travel HBM -> LDS directly (buffer_load ... lds): no staging registers, no
// LDS store instructions.  The LDS holds a ring of five 32-deep stages (all 160 KiB of a CU
// for the 256 x 256 tile).  K tiles are requested in pairs (2i, 2i+1), row by row with the
// two requests of a row back to back: a K-contiguous operand row contributes 64 bytes per
// K tile, half a 128-byte cache line, and the vector L1 merges the second half into the
// line fill the first one started, which halves the requests the L2 has to serve.  A pair
// is requested as soon as both of its stages are free, two to three K tiles ahead of its
// use; with five stages that is as far ahead as a four-stage ring of single tiles.  The
// ring does not drain between output tiles: the last two steps of a tile request the first
// four K tiles of the workgroup's next tile, which are on chip when the epilogue starts, and
// the next tile's first MFMAs start from zero instead of clearing the accumulators.  The
// compiler does not model these transfers, so their completion is awaited
// explicitly (s_waitcnt vmcnt(n): a wavefront's vector-memory loads complete in issue
// order) before the barrier that publishes a stage.
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
#include <atomic>
#include <type_traits>

#include "common.h"

namespace mlc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

template <int V> using I = std::integral_constant<int, V>;

namespace {

constexpr int BK = 32;           // K depth of one LDS stage
constexpr int NSTAGE = 5;        // stages in the LDS ring
constexpr int NPRE = 4;          // K tiles of an output tile that are requested ahead of its first step
constexpr int NTHREADS = 256;
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;        // most tile rows per group of the tile order
constexpr long MIN_TILES_256 = 160;   // fewest 256 x 256 tiles of a product for which that tile is used

struct GemmArgs {
  const bf16_t* A; long lda, strideA;
  const bf16_t* B; long ldb, strideB;
  bf16_t* D; long ldd, strideD;
  const bf16_t* C; long ldc, strideC;
  int K, batch;
  int tiles_m, tiles_n, tiles_per_mat, total_tiles, tiles_per_xcd, wg_per_xcd;
  int group_m;                    // tile rows per group of the tile order
  int symmetric;
  float alpha, beta, gamma;
  const float* bscale; int bscale_pow;
};

// ---- K-contiguous stage layout ------------------------------------------------------
// [R row slots][4 chunks of 16 B].  The LDS has 64 four-byte banks and serves a 128-bit read
// 16 lanes at a time, so the 16 chunks read by lanes 0-15 (same k chunk, rows TT apart) must
// land on 16 different 16-byte columns of the 256-byte bank line, i.e. on 4 different slots
// mod 4 times 4 different chunk positions.  Row TT*l + t (l = lane % 32) lives in slot
// 4*TT*(l/4) + 4*t + l%4, and chunk c of that row sits at position c ^ ((l/4) & 3).
template <int TT>
__device__ __forceinline__ int kc_slot_to_row(int slot) {     // inverse of the map above
  const int l_lo = slot & 3, t = (slot >> 2) & (TT - 1), hi = slot / (4 * TT);
  return TT * (4 * hi + l_lo) + t;
}
template <int TT>
__device__ __forceinline__ int kc_swizzle(int row) { return (row / (4 * TT)) & 3; }

// Raw buffer resource (base, no stride, unbounded, dword data format) for a matrix.
__device__ __forceinline__ i32x4 make_rsrc(const void* p) {
  const unsigned long a = (unsigned long)p;
  i32x4 r;
  r.x = __builtin_amdgcn_readfirstlane((int)(a & 0xffffffffu));
  r.y = __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu));
  r.z = -1;
  r.w = 0x00020000;
  return r;
}

// 16 bytes per lane from rsrc[voff + soff] straight into LDS at lds_off + 16 * lane
// (lds_off is wavefront-uniform and relative to the workgroup's LDS allocation).
// The statement writes m0; it is on the clobber list so that the compiler keeps nothing live
// in it across a transfer (clang notes that m0 is a reserved register: that note is expected).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\t"
               "s_nop 0\n\t"
               "buffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_off), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// ---- HBM -> LDS transfer of one operand's stage (R rows x 32 k) -----------------------
// Chunk c = it * 256 + tid of a stage lands at LDS byte c * 16, so a wavefront's 64 lanes
// fill 1 KiB contiguously; which global chunk a lane fetches follows from the stage layout.
template <int R, int TT, bool KS>
struct StageLoader {
  static constexpr int NCH = R / 64;            // transfers per thread per stage
  static constexpr int CPR = R / 8;             // chunks per k-row when K-strided
  i32x4 rsrc;
  unsigned int voff;                            // lane's byte offset of its first chunk, k = 0
  unsigned int it_stride;                       // bytes between a thread's chunks
  unsigned int k_stride;                        // bytes per stage
  unsigned int wave_lds;                        // wave * 1024

  __device__ __forceinline__ void init(const bf16_t* base, long ld, int row0, int tid) {
    rsrc = make_rsrc(base);
    wave_lds = (unsigned int)__builtin_amdgcn_readfirstlane((tid >> 6) * 1024);
    if constexpr (!KS) {
      const int slot = tid >> 2, pos = tid & 3;
      const int row = kc_slot_to_row<TT>(slot);
      const int ch = pos ^ kc_swizzle<TT>(row);
      voff = (unsigned int)(((long)(row0 + row) * ld + ch * 8) * 2);
      it_stride = (unsigned int)(64 * ld * 2);      // 64 slots = 64 rows further down
      k_stride = BK * 2;
    } else {
      const int krow = tid / CPR, ch = tid % CPR;
      voff = (unsigned int)(((long)krow * ld + row0 + ch * 8) * 2);
      it_stride = (unsigned int)((NTHREADS / CPR) * ld * 2);
      k_stride = (unsigned int)(BK * ld * 2);
    }
  }
  // transfer `it` (of NCH) of K tile kt into the stage at LDS byte offset `stage`
  __device__ __forceinline__ void issue_one(int kt, unsigned int stage, int it) const {
    dma16(rsrc, voff, kt * k_stride + it * it_stride, stage + it * 4096 + wave_lds);
  }
};

// ---- LDS -> MFMA fragments ------------------------------------------------------------
// Reading one operand's fragments for one 16-deep k slice is split in two so that the LDS
// reads can be issued one slice ahead of the MFMAs that consume them:
//   issue_part() : LDS loads into raw registers
//   finish()     : raw registers -> TT fragments of 8 bf16 (a no-op for K-contiguous tiles,
//              sixteen-bit regrouping for K-strided ones)
// K-strided stage: [32][R] bf16; a lane reads its TT adjacent rows for each of its 8 k.
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
  int lane_swz, lane_lg;

  __device__ __forceinline__ void init(int wbase, int l32, int lg) {
    if constexpr (KS) off = lg * 8 * (R * 2) + (wbase + TT * l32) * 2;
    else off = (wbase + 4 * TT * (l32 >> 2) + (l32 & 3)) * 64;     // slot of row TT * l32
    lane_swz = (l32 >> 2) & 3;
    lane_lg = lg;
  }
  // Part PART of NPARTS of the LDS reads of k slice kk (the parts are issued between the
  // transfers of a refill so that neither kind of request arrives in a burst).
  template <int PART, int NPARTS>
  __device__ __forceinline__ void issue_part(const unsigned char* stage, int kk) {
    if constexpr (KS) {
      const unsigned char* p = stage + off + kk * 16 * (R * 2);
#pragma unroll
      for (int t = PART * 8 / NPARTS; t < (PART + 1) * 8 / NPARTS; ++t) {
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
      for (int t = PART * TT / NPARTS; t < (PART + 1) * TT / NPARTS; ++t) {   // row TT * l32 + t: 256 B per t
        const u32x4 v = *reinterpret_cast<const u32x4*>(stage + off + t * 256 + chunk);
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

// Scheduling hint for one k slice (sched_group_barrier masks): LDS reads go between the
// first MFMAs of the slice, the VALU regrouping of the fragments just read goes between the
// last ones, by which time the LDS reads it depends on have returned.
template <int NMFMA, int DSR, int VALU>
__device__ __forceinline__ void interleave_hint() {
  constexpr int NMEM = VALU > 0 ? NMFMA / 2 : NMFMA;
  constexpr int NVAL = NMFMA - NMEM;
  constexpr int r = (DSR + NMEM - 1) / NMEM;
  constexpr int a = NVAL > 0 ? (VALU + NVAL - 1) / NVAL : 0;
#pragma unroll
  for (int i = 0; i < NMFMA; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (i < NMEM) {
      if (r > 0 && i * r < DSR) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
    } else {
      if (a > 0 && (i - NMEM) * a < VALU) __builtin_amdgcn_sched_group_barrier(0x002, a, 0);
    }
  }
}

// One accumulator element, read where it is needed: the statement keeps the accumulators in
// their accumulation registers until then (left to itself the compiler copies all of them to
// ordinary registers first, and from there to scratch memory).
__device__ __forceinline__ float acc_read(float a) {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(a));
  return x;
}
// The wait states between the last MFMA and the first acc_read of its result (the compiler
// does not see into either statement); the operands tie the statement to every accumulator.
template <int TM, int TN>
__device__ __forceinline__ void acc_settle(const f32x16 (&acc)[TM][TN]) {
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (TM == 4)
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7"
                 :: "a"(acc[0][0][15]), "a"(acc[0][1][15]), "a"(acc[0][2][15]), "a"(acc[0][3][15]),
                    "a"(acc[1][0][15]), "a"(acc[1][1][15]), "a"(acc[1][2][15]), "a"(acc[1][3][15]),
                    "a"(acc[2][0][15]), "a"(acc[2][1][15]), "a"(acc[2][2][15]), "a"(acc[2][3][15]),
                    "a"(acc[3][0][15]), "a"(acc[3][1][15]), "a"(acc[3][2][15]), "a"(acc[3][3][15]));
  else
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7"
                 :: "a"(acc[0][0][15]), "a"(acc[0][1][15]), "a"(acc[1][0][15]), "a"(acc[1][1][15]));
  __builtin_amdgcn_sched_barrier(0);
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
  // C is fetched one quarter ahead: the loads of quarter q + 1 are in flight while quarter q
  // is converted and stored, so only the first quarter waits for memory.
  u32x2 cnext[4][TM];
  auto load_c = [&](int q) {
#pragma unroll
    for (int rl = 0; rl < 4; ++rl)
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const unsigned int soff = (unsigned int)(TM * (8 * q + rl) + i) * ldc2;
        if constexpr (TN == 2) cnext[rl][i].x = __builtin_amdgcn_raw_buffer_load_b32(rc, voff_c, soff, 0);
        else cnext[rl][i] = __builtin_amdgcn_raw_buffer_load_b64(rc, voff_c, soff, 0);
      }
  };
  if constexpr (HAS_C) load_c(0);
  acc_settle(acc);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    // keep the scheduler from pulling the next quarter's accumulator reads up here: all 256
    // accumulators in VGPRs at once do not fit
    __builtin_amdgcn_sched_barrier(0);
    unsigned int packed[4][TM][TN / 2];                   // [r % 4][i][column pair]
    u32x2 cval[4][TM];
    if constexpr (HAS_C) {
#pragma unroll
      for (int rl = 0; rl < 4; ++rl)
#pragma unroll
        for (int i = 0; i < TM; ++i) cval[rl][i] = cnext[rl][i];
      if (q < 3) load_c(q + 1);
    }
#pragma unroll
    for (int rl = 0; rl < 4; ++rl) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = 4 * q + rl;
        const int roff = TM * (8 * q + rl) + i;           // compile-time row offset
        float v[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) v[j] = alpha * acc_read(acc[i][j][r]);
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
// order: tiles that share operand panels run at the same time behind the same L2.
// The tiles logical, logical + g.wg_per_xcd, ... below range_end of one product, by one workgroup.
template <int BM, int BN, bool AKS, bool BKS>
__device__ __forceinline__ void run_tiles(const GemmArgs& g, int logical, const int range_end) {
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const unsigned int lds0 =
      (unsigned int)(unsigned long)(__attribute__((address_space(3))) unsigned char*)smem;
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
      // Groups of group_m tile rows, column by column inside a group: the tiles an XCD works
      // on at one time (consecutive indices) then form a block about as tall as it is wide
      // and share few operand panels, which its L2 can hold.
      const int per_group = g.group_m * g.tiles_n;
      const int grp = rem / per_group, r = rem - grp * per_group;
      const int first_m = grp * g.group_m;
      const int rows = min(g.tiles_m - first_m, g.group_m);
      tn = r / rows;
      tm = first_m + (r - tn * rows);
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

  using LoaderA = StageLoader<BM, TM, AKS>;
  using LoaderB = StageLoader<BN, TN, BKS>;
  using ReaderA = FragReader<BM, TM, AKS>;
  using ReaderB = FragReader<BN, TN, BKS>;
  constexpr int NDMA = LoaderA::NCH + LoaderB::NCH;     // transfers per thread per K tile
  LoaderA ldA;
  LoaderB ldB;
  ReaderA rdA;
  ReaderB rdB;
  rdA.init(wbase_m, l32, lg);
  rdB.init(wbase_n, l32, lg);
  u32x4 fa[2][TM], fb[2][TN];
  f32x16 acc[TM][TN];
  const int KT = g.K / BK;      // a multiple of 4: K is a multiple of 128

  // Request the first NPRE K tiles of the first output tile into stages 0 .. NPRE-1, as pairs.
  auto start_tile = [&]() {
#pragma unroll
    for (int st = 0; st < NPRE; st += 2) {
#pragma unroll
      for (int it = 0; it < LoaderA::NCH; ++it) {
        ldA.issue_one(st, lds0 + st * STAGE_BYTES, it);
        ldA.issue_one(st + 1, lds0 + (st + 1) * STAGE_BYTES, it);
      }
#pragma unroll
      for (int it = 0; it < LoaderB::NCH; ++it) {
        ldB.issue_one(st, lds0 + st * STAGE_BYTES + A_BYTES, it);
        ldB.issue_one(st + 1, lds0 + (st + 1) * STAGE_BYTES + A_BYTES, it);
      }
    }
  };

  auto mfma_slice = [&](int buf, auto zero_tag) {
    constexpr bool ZERO = decltype(zero_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        f32x16 c = acc[i][j];
        if constexpr (ZERO) {
#pragma unroll
          for (int r = 0; r < 16; ++r) c[r] = 0.f;
        }
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, fa[buf][i]), __builtin_bit_cast(bf16x8, fb[buf][j]), c, 0, 0, 0);
      }
  };
  constexpr int NM = TM * TN;
  constexpr int NDSR = ReaderA::NLOADS + ReaderB::NLOADS;
  constexpr int NPERM = ReaderA::NPERM + ReaderB::NPERM;
  static_assert(TM == TN && LoaderA::NCH == TM && LoaderB::NCH == TN, "square tiles: one transfer per part");

  // LDS reads of k slice kk of the stage at byte offset `st`, in TM parts; part P is
  // followed by the two transfers extra(P) issues (or none).
  auto reads = [&](unsigned int st, int kk, auto&& extra) {
    auto part = [&](auto p_tag) {
      constexpr int P = decltype(p_tag)::value;
      rdA.template issue_part<P, TM>(smem + st, kk);
      rdB.template issue_part<P, TN>(smem + st + A_BYTES, kk);
      extra(P);
    };
    part(I<0>{}); part(I<1>{});
    if constexpr (TM == 4) { part(I<2>{}); part(I<3>{}); }
  };
  auto nothing = [](int) {};
  // Workgroup barrier that waits for this wavefront's LDS reads only (a fence would also wait
  // for every store of the previous tile's epilogue that is still on its way).
  auto block_sync = []() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  // The ring never drains between output tiles: a body is two 32-deep steps on K tiles t
  // (stage r0) and t+1 (stage r1); r2 holds K tile t+2 and r4 is free.  Each step is two
  // 16-deep slices:
  //   slice 0: MFMAs on fragments 0 | LDS reads of the stage's second slice
  //   wait until the next K tile has landed, barrier: publishes it and retires this stage
  //   slice 1: MFMAs on fragments 1 | LDS reads of the next stage's first slice
  // Every body requests two K tiles, k4 and k4 + 1 of loader (la, lb), into r4 and r0 (r0 is
  // free after the first barrier): K tiles t+4 and t+5 of this output tile or, in its last
  // two bodies, K tiles 0..3 of the workgroup's next output tile, so that tile's first
  // operands are on chip before this tile's epilogue starts.  With a K-contiguous operand the
  // two go as a pair, operand A during slice 1 of the first step and operand B during slice 0
  // of the second; when both operands are K-strided (whole cache lines anyway) they are
  // spread over the four slices instead: A(k4), B(k4), A(k4+1), B(k4+1).
  // W1 / W2: vector-memory operations that may still be in flight at the first / second
  // barrier, i.e. all those issued after the K tile the barrier publishes (they complete in
  // the order they were issued).  ZERO: the body's first MFMAs start from zero accumulators.
  constexpr bool SPREAD = AKS && BKS;
  auto body = [&](const LoaderA& la, const LoaderB& lb, int k4, unsigned int r0, unsigned int r1,
                  unsigned int r2, unsigned int r4, auto w1_tag, auto w2_tag, auto zero_tag) {
    constexpr int W1 = decltype(w1_tag)::value, W2 = decltype(w2_tag)::value;
    // ---- first step, slice 0
    reads(r0, 1, [&](int p) {
      if constexpr (SPREAD) la.issue_one(k4, lds0 + r4, p);
    });
    mfma_slice(0, zero_tag);
    rdA.finish(fa[1]); rdB.finish(fb[1]);
    interleave_hint<NM, NDSR, NPERM>();
    // keep slice 0's MFMAs above the barrier: they cover the wait for its LDS reads
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<W1>();
    block_sync();
    // ---- first step, slice 1
    reads(r1, 0, [&](int p) {
      if constexpr (SPREAD) lb.issue_one(k4, lds0 + r4 + A_BYTES, p);
      else {
        la.issue_one(k4, lds0 + r4, p);
        la.issue_one(k4 + 1, lds0 + r0, p);
      }
    });
    mfma_slice(1, std::false_type{});
    rdA.finish(fa[0]); rdB.finish(fb[0]);
    interleave_hint<NM, NDSR, NPERM>();
    // ---- second step, slice 0
    reads(r1, 1, [&](int p) {
      if constexpr (SPREAD) la.issue_one(k4 + 1, lds0 + r0, p);
      else {
        lb.issue_one(k4, lds0 + r4 + A_BYTES, p);
        lb.issue_one(k4 + 1, lds0 + r0 + A_BYTES, p);
      }
    });
    mfma_slice(0, std::false_type{});
    rdA.finish(fa[1]); rdB.finish(fb[1]);
    interleave_hint<NM, NDSR, NPERM>();
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<W2>();
    block_sync();
    reads(r2, 0, [&](int p) {
      if constexpr (SPREAD) lb.issue_one(k4 + 1, lds0 + r0 + A_BYTES, p);
    });
    // ---- second step, slice 1
    mfma_slice(1, std::false_type{});
    rdA.finish(fa[0]); rdB.finish(fb[0]);
    interleave_hint<NM, NDSR, NPERM>();
  };
  using T = std::true_type;
  using F = std::false_type;
  // Operations in flight at a barrier when every body since the K tile it publishes has
  // requested its two K tiles.  The first three barriers of an output tile publish K tiles
  // that had landed before the previous tile's epilogue (or before the first tile started):
  // they wait for nothing (63 is the counter's largest value).
  constexpr int STEADY = SPREAD ? 2 * NDMA + LoaderA::NCH : 2 * NDMA;
  constexpr int LANDED = 63;

  TileCoord tc = decode(logical);
  ldA.init(g.A + (long)tc.b * g.strideA, g.lda, tc.m0, tid);
  ldB.init(g.B + (long)tc.b * g.strideB, g.ldb, tc.n0, tid);
  start_tile();
  // All four K tiles land before the first body, as they do for every later tile.  Through
  // the builtin, so that the compiler's own bookkeeping sees every earlier vector-memory
  // operation as complete.
  __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt(0), other counters unconstrained
  block_sync();
  reads(0u, 0, nothing);
  rdA.finish(fa[0]);
  rdB.finish(fb[0]);
  // The ring rotates by two stages per body: r[x] = byte offset of the stage that holds
  // (or will hold) K tile t + x.
  unsigned int r0 = 0, r1 = STAGE_BYTES, r2 = 2 * STAGE_BYTES, r3 = 3 * STAGE_BYTES, r4 = 4 * STAGE_BYTES;
  auto rotate = [&]() {
    const unsigned int a0 = r0, a1 = r1;
    r0 = r2; r1 = r3; r2 = r4; r3 = a0; r4 = a1;
  };
  while (true) {
    // The next output tile of this workgroup; after the last one the same requests go to this
    // tile's own first K tiles again (in bounds, never read).
    const int next = logical + g.wg_per_xcd;
    const bool more = next < range_end;
    const TileCoord tn = more ? decode(next) : tc;
    LoaderA nxA;
    LoaderB nxB;
    nxA.init(g.A + (long)tn.b * g.strideA, g.lda, tn.m0, tid);
    nxB.init(g.B + (long)tn.b * g.strideB, g.ldb, tn.n0, tid);
    auto run = [&](int t, auto w1_tag, auto w2_tag, auto zero_tag) {
      const bool tail = t + 4 >= KT;
      LoaderA la = ldA;
      LoaderB lb = ldB;
      if (tail) { la = nxA; lb = nxB; }
      body(la, lb, tail ? t + 4 - KT : t + 4, r0, r1, r2, r4, w1_tag, w2_tag, zero_tag);
      rotate();
    };
    run(0, I<LANDED>{}, I<LANDED>{}, T{});
    run(2, I<LANDED>{}, I<STEADY>{}, F{});
#pragma unroll 1
    for (int t = 4; t < KT; t += 2) run(t, I<STEADY>{}, I<STEADY>{}, F{});

    // Everything requested so far (the next tile's first four K tiles) lands before the
    // first store is issued: the waits of the next two bodies then never depend on how
    // loads and stores complete relative to each other.
    wait_vmcnt<0>();
    float alpha = g.alpha;
    if (g.bscale) {
      const float sc = g.bscale[tc.b];
      alpha *= (g.bscale_pow == 2) ? sc * sc : sc;
    }
    // the diagonal crosses this tile only if its row and column ranges overlap
    const bool on_diag = g.gamma != 0.f && tc.m0 < tc.n0 + BN && tc.n0 < tc.m0 + BM;
    if (g.C) store_tile<TM, TN, true>(g, acc, tc, alpha, on_diag, wbase_m, wbase_n, l32, lg);
    else store_tile<TM, TN, false>(g, acc, tc, alpha, on_diag, wbase_m, wbase_n, l32, lg);
    if (!more) break;
    logical = next;
    tc = tn;
    ldA = nxA;
    ldB = nxB;
  }
  // nothing may land in the ring after this workgroup has left it
  __builtin_amdgcn_s_waitcnt(0x0f70);
  block_sync();
}

template <int BM, int BN, bool AKS, bool BKS>
__global__ __launch_bounds__(NTHREADS) void ns_gemm_bf16_kernel(GemmArgs g) {
  const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD;
  const int range_end = min((xcd + 1) * g.tiles_per_xcd, g.total_tiles);
  run_tiles<BM, BN, AKS, BKS>(g, xcd * g.tiles_per_xcd + slot, range_end);
}

// Several products of equal depth K in one launch (the same product of a Newton-Schulz
// iteration for several shape groups).  A launch whose tile count is not a multiple of the
// number of compute units pays for a partly empty last round; sharing a launch leaves one
// such round instead of one per group.  XCD x still owns a contiguous range of every
// product's tile order; inside it the workgroups take the products one after the other, each
// starting with the workgroup after the one that took the previous product's last tile, so
// that no workgroup ends up with more than one tile over the average.  LAYOUTS: bit 0 =
// both operands K-contiguous, bit 1 = both K-strided, bit 2 = A K-contiguous and B
// K-strided; only the listed tile loops are compiled in.
constexpr int MAX_MULTI = 3;
enum { LAYOUT_KC_KC = 0, LAYOUT_KS_KS = 1, LAYOUT_KC_KS = 2 };
struct MultiArgs { GemmArgs seg[MAX_MULTI]; int layout[MAX_MULTI]; int nseg; };

template <int BM, int BN, int LAYOUTS>
__global__ __launch_bounds__(NTHREADS) void ns_gemm_multi_kernel(MultiArgs m) {
  const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD;
  const int W = (int)(gridDim.x / NUM_XCD);
  int off = 0;         // workgroups of this XCD that already received a tile more than the others
#pragma unroll 1
  for (int j = 0; j < m.nseg; ++j) {
    const GemmArgs& g = m.seg[j];
    const int lo = min(xcd * g.tiles_per_xcd, g.total_tiles);
    const int hi = min((xcd + 1) * g.tiles_per_xcd, g.total_tiles);
    int pos = slot - off;
    if (pos < 0) pos += W;
    const int first = lo + pos;
    const int lay = m.layout[j];
    if (first < hi) {
      if ((LAYOUTS & 1) && lay == LAYOUT_KC_KC) run_tiles<BM, BN, false, false>(g, first, hi);
      if ((LAYOUTS & 2) && lay == LAYOUT_KS_KS) run_tiles<BM, BN, true, true>(g, first, hi);
      if ((LAYOUTS & 4) && lay == LAYOUT_KC_KS) run_tiles<BM, BN, false, true>(g, first, hi);
    }
    off = (off + (hi - lo)) % W;
    // the next product's first transfers overwrite the ring: every wavefront must have left it
    __syncthreads();
  }
}

// Compute units behind one L2 (one XCD) of the current device.
int cus_per_xcd(int slot) {
  static std::atomic<int> cached[MAX_DEVICES];
  if (slot >= 0) {
    const int c = cached[slot].load(std::memory_order_relaxed);
    if (c > 0) return c;
  }
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < NUM_XCD)
    cus = 256;
  if (slot >= 0) cached[slot].store(cus / NUM_XCD, std::memory_order_relaxed);
  return cus / NUM_XCD;
}

// Dynamic LDS a kernel asks for: its ring, and at least 96 KiB so that no second workgroup
// fits beside it on a CU.
template <int BM, int BN>
constexpr size_t exclusive_lds_bytes() {
  return (size_t)NSTAGE * (BM + BN) * BK * 2 > 96 * 1024 ? (size_t)NSTAGE * (BM + BN) * BK * 2 : (size_t)96 * 1024;
}

// Kernel arguments of one product with BM x BN tiles; wg_per_xcd is left to the caller.
template <int BM, int BN>
int make_args(const GemmDesc& d, GemmArgs& g) {
  g.A = d.A; g.lda = d.lda; g.strideA = d.strideA;
  g.B = d.B; g.ldb = d.ldb; g.strideB = d.strideB;
  g.D = d.D; g.ldd = d.ldd; g.strideD = d.strideD;
  g.C = d.C; g.ldc = d.ldc; g.strideC = d.strideC;
  g.K = d.K; g.batch = d.batch;
  g.tiles_m = d.M / BM; g.tiles_n = d.N / BN;
  g.symmetric = d.symmetric ? 1 : 0;
  {   // equal groups of at most GROUP_M tile rows (10 rows -> 5 + 5, not 8 + 2)
    const int ngroups = (g.tiles_m + GROUP_M - 1) / GROUP_M;
    g.group_m = (g.tiles_m + ngroups - 1) / ngroups;
  }
  if (g.symmetric && (BM != BN || d.M != d.N)) return MLC_ERR_SHAPE;
  g.tiles_per_mat = g.symmetric ? g.tiles_m * (g.tiles_m + 1) / 2 : g.tiles_m * g.tiles_n;
  const long total = (long)g.tiles_per_mat * d.batch;
  if (total <= 0 || total > (1L << 30)) return MLC_ERR_SHAPE;
  g.total_tiles = (int)total;
  g.tiles_per_xcd = (int)((total + NUM_XCD - 1) / NUM_XCD);
  g.wg_per_xcd = 0;
  g.alpha = d.alpha; g.beta = d.beta; g.gamma = d.gamma;
  g.bscale = d.bscale; g.bscale_pow = d.bscale_pow;
  return MLC_OK;
}

// The LDS limit of a kernel is raised once per instantiation and device (the call is
// idempotent, so a race between two host threads only repeats it).
template <typename Kern>
int raise_lds_limit(Kern kern, std::atomic<bool>* done, int slot, size_t lds) {
  if (slot < 0 || !done[slot].load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return MLC_ERR_LAUNCH;
    if (slot >= 0) done[slot].store(true, std::memory_order_release);
  }
  return MLC_OK;
}

template <int BM, int BN, bool AKS, bool BKS>
int launch_cfg(const GemmDesc& d, hipStream_t stream) {
  GemmArgs g;
  int rc = make_args<BM, BN>(d, g);
  if (rc != MLC_OK) return rc;
  // One workgroup per CU.  The ring of the 256 x 256 tile fills the 160 KiB of LDS anyway; the
  // 128 x 128 tile's ring is 80 KiB and two such workgroups would fit, but with two of them
  // on one CU the tiles of the second one came out wrong (garbage, from run to run on
  // different tiles), so the kernel asks for more than half of the LDS and a CU never holds
  // two.  (Suspected, not established: the LDS address of `buffer_load ... lds`, taken from
  // m0, when the workgroup's LDS allocation does not start at 0.)
  const int slot = device_slot();
  g.wg_per_xcd = cus_per_xcd(slot);
  if (g.wg_per_xcd > g.tiles_per_xcd) g.wg_per_xcd = g.tiles_per_xcd;
  const size_t lds = exclusive_lds_bytes<BM, BN>();
  auto kern = ns_gemm_bf16_kernel<BM, BN, AKS, BKS>;
  static std::atomic<bool> attr_set[MAX_DEVICES];
  rc = raise_lds_limit(kern, attr_set, slot, lds);
  if (rc != MLC_OK) return rc;
  const double flops = 2.0 * BM * BN * (double)d.K * (double)g.total_tiles;   // executed, not nominal
  LaunchScope scope(MLC_KERNEL_NS_GEMM, stream, flops, 0.0);
  hipLaunchKernelGGL(kern, dim3(g.wg_per_xcd * NUM_XCD), dim3(NTHREADS), lds, stream, g);
  return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH;
}

int layout_of(const GemmDesc& d) {
  if (!d.a_kstrided && !d.b_kstrided) return LAYOUT_KC_KC;
  if (d.a_kstrided && d.b_kstrided) return LAYOUT_KS_KS;
  if (!d.a_kstrided && d.b_kstrided) return LAYOUT_KC_KS;
  return -1;
}

bool valid_desc(const GemmDesc& d) {
  if (d.M % 128 || d.N % 128 || d.K % 128 || d.M <= 0 || d.N <= 0 || d.K <= 0 || d.batch <= 0) return false;
  if ((d.lda | d.ldb | d.ldd | d.strideA | d.strideB | d.strideD) % 8) return false;
  if (d.C && ((d.ldc | d.strideC) % 8)) return false;
  return true;
}

// n (2 or 3) products of one depth K with 256 x 256 tiles in one launch.
template <int LAYOUTS>
int launch_multi(const GemmDesc* const* d, int n, hipStream_t stream) {
  MultiArgs m;
  m.nseg = n;
  const int slot = device_slot();
  const int W = cus_per_xcd(slot);
  double flops = 0.0;
  for (int j = 0; j < MAX_MULTI; ++j) {
    const GemmDesc& dj = *d[j < n ? j : 0];
    const int rc = make_args<256, 256>(dj, m.seg[j]);
    if (rc != MLC_OK) return rc;
    m.seg[j].wg_per_xcd = W;
    m.layout[j] = layout_of(dj);
    if (j < n) flops += 2.0 * 256 * 256 * (double)dj.K * (double)m.seg[j].total_tiles;
  }
  const size_t lds = exclusive_lds_bytes<256, 256>();
  auto kern = ns_gemm_multi_kernel<256, 256, LAYOUTS>;
  static std::atomic<bool> attr_set[MAX_DEVICES];
  const int rc = raise_lds_limit(kern, attr_set, slot, lds);
  if (rc != MLC_OK) return rc;
  LaunchScope scope(MLC_KERNEL_NS_GEMM, stream, flops, 0.0);
  hipLaunchKernelGGL(kern, dim3(W * NUM_XCD), dim3(NTHREADS), lds, stream, m);
  return hipGetLastError() == hipSuccess ? MLC_OK : MLC_ERR_LAUNCH;
}

template <int BM, int BN>
int launch_layout(const GemmDesc& d, hipStream_t stream) {
  // Newton-Schulz needs only these two: a symmetric operand can be read either way, so the
  // mixed cases never arise.
  if (!d.a_kstrided && !d.b_kstrided) return launch_cfg<BM, BN, false, false>(d, stream);
  if (d.a_kstrided && d.b_kstrided) return launch_cfg<BM, BN, true, true>(d, stream);
  if (!d.a_kstrided && d.b_kstrided) return launch_cfg<BM, BN, false, true>(d, stream);
  return MLC_ERR_UNSUPPORTED;
}

}  // namespace

int launch_ns_gemm(const GemmDesc& d, hipStream_t stream) {
  if (!valid_desc(d)) return MLC_ERR_SHAPE;
  // The large tile as soon as it occupies most of the chip for one round: the small tile moves
  // twice the operand bytes per FLOP and needs four times the tiles.
  const long tiles256 = (long)(d.M / 256) * (d.N / 256) * d.batch;
  if (d.M % 256 == 0 && d.N % 256 == 0 && tiles256 >= MIN_TILES_256) return launch_layout<256, 256>(d, stream);
  return launch_layout<128, 128>(d, stream);
}

int launch_ns_gemm_set(const GemmDesc* d, int n, hipStream_t stream) {
  if (n < 0 || n > 64) return MLC_ERR_ARG;
  bool done[64] = {};
  for (int i = 0; i < n; ++i) {
    if (done[i]) continue;
    if (!valid_desc(d[i])) return MLC_ERR_SHAPE;
    // products that can share a launch with product i: same depth (a tile then takes the same
    // time in each, so dealing tiles out evenly balances the time), 256 x 256 tiles, the same
    // kind of epilogue, and a combination of operand layouts one of the kernels holds
    const GemmDesc* pick[MAX_MULTI] = {&d[i], nullptr, nullptr};
    int idx[MAX_MULTI] = {i, -1, -1};
    int np = 1, layouts = 1 << (layout_of(d[i]) < 0 ? 0 : layout_of(d[i]));
    const bool tile256 = d[i].M % 256 == 0 && d[i].N % 256 == 0 && layout_of(d[i]) >= 0;
    long tiles = tile256 ? (long)(d[i].M / 256) * (d[i].N / 256) * d[i].batch : 0;
    for (int j = i + 1; tile256 && j < n && np < MAX_MULTI; ++j) {
      if (done[j] || !valid_desc(d[j]) || layout_of(d[j]) < 0) continue;
      if (d[j].K != d[i].K || d[j].M % 256 || d[j].N % 256 || (d[j].symmetric != 0) != (d[i].symmetric != 0) ||
          (d[j].C != nullptr) != (d[i].C != nullptr))
        continue;
      const int both = layouts | (1 << layout_of(d[j]));
      if (both != 1 && both != 3 && both != 4 && both != 5) continue;      // the combinations that are built
      layouts = both;
      pick[np] = &d[j];
      idx[np] = j;
      tiles += (long)(d[j].M / 256) * (d[j].N / 256) * d[j].batch;
      ++np;
    }
    int rc;
    if (np >= 2 && tiles >= MIN_TILES_256) {
      if (layouts == 1) rc = launch_multi<1>(pick, np, stream);
      else if (layouts == 3) rc = launch_multi<3>(pick, np, stream);
      else rc = launch_multi<5>(pick, np, stream);      // also serves two products with layout bit 2 alone
      if (rc != MLC_OK) return rc;
      for (int k = 0; k < np; ++k) done[idx[k]] = true;
      continue;
    }
    rc = launch_ns_gemm(d[i], stream);
    if (rc != MLC_OK) return rc;
    done[i] = true;
  }
  return MLC_OK;
}

}  // namespace mlc
