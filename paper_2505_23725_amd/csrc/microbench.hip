// Achievable-peak microbenchmarks for one MI355X (not part of the method): the sustained
// v_mfma_f32_32x32x16_bf16 rate of a register-resident loop with constant operands, with
// random bit patterns (the most switching activity the datapath can see) and with operands
// drawn like the workload's (bf16 roundings of 1e-3 * N(0, 1); accumulators stay finite):
// the chip is power-limited, so the sustained rate depends on the data.  Also the HBM
// bandwidth of a plain 16-byte copy, of a pure read (plain and non-temporal), of a pure write
// and of an in-place read-modify-write stream.  Prints one JSON line.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(2); } } while (0)

__global__ __launch_bounds__(256) void mfma_loop(const u32x4* in, float* out, int iters) {
  f32x16 acc[16];
  for (int i = 0; i < 16; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  u32x4 a[4], b[4];
  for (int i = 0; i < 4; ++i) { a[i] = in[threadIdx.x * 8 + i]; b[i] = in[threadIdx.x * 8 + 4 + i]; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]), acc[i * 4 + j], 0, 0, 0);
  }
  float s = 0;
  for (int i = 0; i < 16; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 12345.f) out[0] = s;
}

// each workgroup owns a contiguous chunk; non-temporal accesses, four vectors in flight
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, long n) {
  const long per_blk = (n + gridDim.x - 1) / gridDim.x;
  const long b0 = (long)blockIdx.x * per_blk, b1 = (b0 + per_blk < n) ? b0 + per_blk : n;
  long i = b0 + threadIdx.x;
  for (; i + 3 * 256 < b1; i += 4 * 256) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(in + i + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], out + i + u * 256);
  }
  for (; i < b1; i += 256) out[i] = in[i];
}
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, long n) {
  const long stride = (long)gridDim.x * 256;
  u32x4 acc = {0, 0, 0, 0};
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i + 3 * stride < n; i += 4 * stride) {
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= in[i + u * stride];
  }
  if (acc.x == 0x12345) out[0] = acc;
}

// In-place read-modify-write of one stream (what an optimizer update does), and a pure write.
__global__ __launch_bounds__(256) void rmw_kernel(u32x4* __restrict__ a, long n) {
  const long per_blk = (n + gridDim.x - 1) / gridDim.x;
  const long b0 = (long)blockIdx.x * per_blk, b1 = (b0 + per_blk < n) ? b0 + per_blk : n;
  for (long i = b0 + threadIdx.x; i < b1; i += 4 * 256) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (i + u * 256 < b1) v[u] = a[i + u * 256];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (i + u * 256 < b1) { v[u].x += 1; a[i + u * 256] = v[u]; }
  }
}
__global__ __launch_bounds__(256) void write_kernel(u32x4* __restrict__ a, long n) {
  const long per_blk = (n + gridDim.x - 1) / gridDim.x;
  const long b0 = (long)blockIdx.x * per_blk, b1 = (b0 + per_blk < n) ? b0 + per_blk : n;
  for (long i = b0 + threadIdx.x; i < b1; i += 256) a[i] = u32x4{1u, 2u, 3u, (unsigned)i};
}
__global__ __launch_bounds__(256) void read_nt_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, long n) {
  const long per_blk = (n + gridDim.x - 1) / gridDim.x;
  const long b0 = (long)blockIdx.x * per_blk, b1 = (b0 + per_blk < n) ? b0 + per_blk : n;
  u32x4 acc = {0, 0, 0, 0};
  for (long i = b0 + threadIdx.x; i + 3 * 256 < b1; i += 4 * 256) {
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= __builtin_nontemporal_load(in + i + u * 256);
  }
  if (acc.x == 0x12345) out[0] = acc;
}

int main() {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0.f;
  float* d; CK(hipMalloc(&d, 4096));
  u32x4* in; CK(hipMalloc(&in, 256 * 8 * 16));
  auto gauss_bf16 = []() -> unsigned {      // bf16 bits of 1e-3 * N(0, 1), Box-Muller on rand()
    const double u1 = (rand() + 1.0) / (RAND_MAX + 2.0), u2 = (rand() + 1.0) / (RAND_MAX + 2.0);
    const float f = (float)(1e-3 * std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586 * u2));
    unsigned u; std::memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);         // round to nearest even
    return u >> 16;
  };
  double tf[3];
  for (int mode = 0; mode < 3; ++mode) {
    std::vector<unsigned> h(256 * 8 * 4);
    srand(1);
    for (auto& v : h) {
      if (mode == 0) v = 0x3c3c3c3cu;                                  // every operand 0.0115
      else if (mode == 1) { v = ((unsigned)rand() << 16) ^ (unsigned)rand(); v &= 0xbfffbfffu; }   // random finite bf16 pairs
      else v = gauss_bf16() | (gauss_bf16() << 16);
    }
    CK(hipMemcpy(in, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    const int iters = 6000, blocks = 512;
    hipLaunchKernelGGL(mfma_loop, dim3(blocks), dim3(256), 0, 0, in, d, 100);
    CK(hipEventRecord(e0, 0));
    hipLaunchKernelGGL(mfma_loop, dim3(blocks), dim3(256), 0, 0, in, d, iters);
    CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    tf[mode] = 2.0 * 32 * 32 * 16 * 16.0 * iters * 4 * blocks / ms * 1e-9;
  }
  const size_t bytes = (size_t)2 << 30;
  u32x4 *a, *b; CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, bytes));
  CK(hipMemset(a, 1, bytes)); CK(hipMemset(b, 2, bytes));
  const long n = bytes / 16;
  double copy_gbs, read_gbs;
  hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, 0, a, b, n);
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, 0, a, b, n);
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  copy_gbs = 2.0 * bytes / (ms / 5 * 1e-3) * 1e-9;
  hipLaunchKernelGGL(read_kernel, dim3(16384), dim3(256), 0, 0, a, b, n);
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(read_kernel, dim3(16384), dim3(256), 0, 0, a, b, n);
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  read_gbs = 1.0 * bytes / (ms / 5 * 1e-3) * 1e-9;
  double read_nt_gbs, write_gbs, rmw_gbs;
  hipLaunchKernelGGL(read_nt_kernel, dim3(8192), dim3(256), 0, 0, a, b, n);
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(read_nt_kernel, dim3(8192), dim3(256), 0, 0, a, b, n);
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  read_nt_gbs = 1.0 * bytes / (ms / 5 * 1e-3) * 1e-9;
  hipLaunchKernelGGL(write_kernel, dim3(8192), dim3(256), 0, 0, b, n);
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(write_kernel, dim3(8192), dim3(256), 0, 0, b, n);
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  write_gbs = 1.0 * bytes / (ms / 5 * 1e-3) * 1e-9;
  hipLaunchKernelGGL(rmw_kernel, dim3(8192), dim3(256), 0, 0, a, n);
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(rmw_kernel, dim3(8192), dim3(256), 0, 0, a, n);
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  rmw_gbs = 2.0 * bytes / (ms / 5 * 1e-3) * 1e-9;
  printf("{\"mfma_bf16_tflops_constant_operands\": %.1f, \"mfma_bf16_tflops_random_operands\": %.1f, "
         "\"mfma_bf16_tflops_gaussian_operands\": %.1f, \"hbm_copy_GBps\": %.0f, \"hbm_read_GBps\": %.0f, "
         "\"hbm_read_nontemporal_GBps\": %.0f, \"hbm_write_GBps\": %.0f, \"hbm_rmw_in_place_GBps\": %.0f}\n",
         tf[0], tf[1], tf[2], copy_gbs, read_gbs, read_nt_gbs, write_gbs, rmw_gbs);
  return 0;
}
