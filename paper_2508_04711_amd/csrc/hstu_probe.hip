// Measurement kernels behind hstu_debug_mfma_loop and hstu_debug_dq_atomic_rate: what the chip
// sustains on nothing but matrix instructions (the ceiling the attention kernels' rates are read
// against), and how fast fp32 atomic adds go in the access pattern a dk/dv pass that also produced
// dq would need (the measurement behind keeping dq a pass of its own).
#include "hstu_common.h"

namespace hstu {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Four independent accumulators per wave, two waves per SIMD: the matrix pipe always has an
// instruction whose operands are ready.  Operands: the same value in every lane (random == 0) or
// values from a per-lane generator; they stay fixed over the loop (what matters for the power the
// loop draws is how many bits differ between the lanes' operands, not that they change).
__global__ void __launch_bounds__(256, 2) mfma_loop_kernel(int iters, int random, float* sink) {
  const int tid = blockIdx.x * 256 + threadIdx.x;
  bf16x8 a[4], b[4];
  uint32_t x = 0x9E3779B9u * (uint32_t)(tid + 1);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      x = x * 1664525u + 1013904223u;
      const float va = random ? ((int)(x >> 8) - (1 << 23)) * (1.0f / (1 << 23)) : 0.5f;
      x = x * 1664525u + 1013904223u;
      const float vb = random ? ((int)(x >> 8) - (1 << 23)) * (1.0f / (1 << 23)) : 0.25f;
      a[i][e] = (__bf16)va;
      b[i][e] = (__bf16)vb;
    }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 12345.678f) sink[tid & 63] = s;  // keeps the loop; practically never true
}

// One workgroup per CU (through its LDS request) sweeps 32-row blocks of a [rows][heads][128] fp32
// array for one head; per block each of its four waves issues 16 no-return atomic adds, every
// instruction covering two rows x 128 contiguous bytes: the 16 KB a 128-key tile would add to dq
// for one block of 32 queries.  local != 0: workgroup i works on head i % heads (with 8 heads every
// XCD, which takes every eighth workgroup, has a head of its own); else heads are mixed over XCDs.
__global__ void __launch_bounds__(256, 1) dq_atomic_kernel(float* buf, int rows, int heads, int nblk, int local) {
  __shared__ char pad[100 * 1024];
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5, w = tid >> 6;
  const int wg = blockIdx.x;
  const int h = local ? wg % heads : (wg / 8) % heads;
  const int64_t rs = (int64_t)heads * 128;
  int row0 = (int)(((int64_t)(wg / 8) * 128) % (rows - 32));
  for (int b = 0; b < nblk; ++b) {
    int r0 = row0 + b * 32;
    if (r0 + 32 > rows) r0 %= (rows - 32);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int q = 8 * (r >> 2) + 4 * hh + (r & 3), d = 32 * w + n;
      __builtin_amdgcn_global_atomic_fadd_f32(buf + (int64_t)(r0 + q) * rs + h * 128 + d, 1.0f);
    }
  }
  if (pad[tid] == 77 && nblk < 0) buf[0] = 1.f;  // keeps the LDS request
}

}  // namespace

hipError_t launch_mfma_loop(int iters, int random, float* sink, double* flops, hipStream_t stream) {
  const int grid = 256 * 2;  // two workgroups of four waves per CU
  *flops = (double)grid * 4 * iters * 4 * 32768.0;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(grid), dim3(256), 0, stream, iters, random, sink);
  return hipGetLastError();
}

hipError_t launch_dq_atomic(float* buf, int64_t rows, int heads, int nblk, int local, double* bytes,
                            hipStream_t stream) {
  const int grid = 256;
  *bytes = (double)grid * nblk * 32 * 128 * 4;
  hipLaunchKernelGGL(dq_atomic_kernel, dim3(grid), dim3(256), 0, stream, buf, (int)rows, heads, nblk, local);
  return hipGetLastError();
}

}  // namespace hstu
