// Measured ceilings of the machine the library runs on, as kernels of the library's own so that
// the benchmark can quote its fractions against them next to the published peaks:
//   * the matrix cores fed from registers only (no LDS, no memory): back-to-back
//     v_mfma_f32_32x32x16_bf16 on four independent accumulator sets per wave, one wave per SIMD
//     (the GEMM's occupancy), operands either all zero or pseudo-random bf16 bit patterns --
//     the chip holds a different clock for the two, and the GEMMs see data like the second;
//   * a plain copy, 16 bytes per lane, grid-stride: what HBM delivers to a kernel that does
//     nothing else.
#include "fax_internal.h"

namespace fax {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, unsigned seed, float* __restrict__ sink) {
  // operands: zero, or per-lane bit patterns of finite bf16 values of moderate exponent
  // (four different first and four different second operands, so that consecutive instructions
  // see different bits, as they do in a GEMM)
  uint4 ua[4], ub[4];
#pragma unroll
  for (int k = 0; k < 4; k++) ua[k] = ub[k] = make_uint4(0, 0, 0, 0);
  if (seed) {
    unsigned x = seed * 2654435761u + (blockIdx.x * 256u + threadIdx.x) * 40503u + 1u;
    auto next = [&]() {
      x ^= x << 13; x ^= x >> 17; x ^= x << 5;
      // two bf16 per word: sign and 7 mantissa bits random, exponent in [120, 127]: |v| in [2^-7, 2)
      const unsigned lo = (x & 0x807fu) | ((120u + ((x >> 8) & 7u)) << 7);
      const unsigned hi = ((x >> 16) & 0x807fu) | ((120u + ((x >> 28) & 7u)) << 7);
      return lo | (hi << 16);
    };
#pragma unroll
    for (int k = 0; k < 4; k++) {
      ua[k] = make_uint4(next(), next(), next(), next());
      ub[k] = make_uint4(next(), next(), next(), next());
    }
  }
  bf16x8 a[4], b[4];
#pragma unroll
  for (int k = 0; k < 4; k++) {
    a[k] = __builtin_bit_cast(bf16x8, ua[k]);
    b[k] = __builtin_bit_cast(bf16x8, ub[k]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; k++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[k][v] = 0.f;
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int k = 0; k < 4; k++) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r], b[k], acc[k], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; k++)
#pragma unroll
    for (int v = 0; v < 16; v++) s += acc[k][v];
  if (s == 123.456f) sink[0] = s;  // keeps the loop alive; never true for these operands in practice, harmless if it is
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  // four independent 16-byte loads in flight per lane, then their stores
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

// flops of one launch: workgroups x 4 waves x iters x 16 MFMAs x 2 * 32 * 32 * 16
int probe_mfma(int workgroups, int iters, unsigned seed, float* sink, hipStream_t s) {
  Timed t_(seed ? "probe_mfma_random" : "probe_mfma_zero", WORK_FLOP, (double)workgroups * 4.0 * iters * 16.0 * 32768.0, s);
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, s, iters, seed, sink);
  FAX_LAUNCH_CHECK("probe_mfma");
  return FAX_OK;
}

int probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  Timed t_("probe_copy", WORK_BYTE, 2.0 * (double)bytes, s);
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, bytes / 16);
  FAX_LAUNCH_CHECK("probe_copy");
  return FAX_OK;
}

}  // namespace fax
