// Device probe: the bf16 MFMA rate this chip sustains on register-resident operands, with all-zero or with
// random (sign, exponent, mantissa) operand values. The clock the chip holds depends on the switching power of
// the data, so the second figure, not the nominal peak, is what a kernel working on N(0,1) inputs can approach.
// Built into its own small library (libzeppelin_bench.so): a measurement aid, not part of the engine.
#include "zp_common.h"

namespace {
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;

__device__ __forceinline__ unsigned probe_hash(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(256) void mfma_probe_kernel(float *out, int iters, int random_operands) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    u16x8 ua, ub;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const unsigned h = probe_hash((blockIdx.x * 256 + threadIdx.x) * 64 + j * 8 + i);
      // random sign, magnitude in [2^-2, 2^2), random mantissa
      ua[i] = random_operands ? (unsigned short)(((h & 1) << 15) | ((125 + ((h >> 1) & 3)) << 7) | ((h >> 8) & 0x7F)) : 0;
      ub[i] = random_operands ? (unsigned short)((((h >> 3) & 1) << 15) | ((125 + ((h >> 4) & 3)) << 7) | ((h >> 16) & 0x7F)) : 0;
    }
    a[j] = __builtin_bit_cast(bf16x8, ua);
    b[j] = __builtin_bit_cast(bf16x8, ub);
  }
  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; c++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[c][r] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int u = 0; u < 8; u++)
#pragma unroll
      for (int c = 0; c < 4; c++)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + c) & 3], b[u & 3], acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < 4; c++)
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc[c][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace

// 256 workgroups of 4 waves; each wave issues iters * 32 MFMAs of 32x32x16 (32768 flop each).
extern "C" int zp_mfma_probe(float *out, int32_t iters, int32_t random_operands, void *stream) {
  if (!out || ((uintptr_t)out & 15) || iters < 1 || iters > (1 << 22)) return -1;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(256), dim3(256), 0, (hipStream_t)stream, out, iters, random_operands ? 1 : 0);
  return (int)hipGetLastError();
}
