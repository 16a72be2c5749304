// Measurement aid, not part of libvs: what this chip sustains for the INSTRUCTION MIX of the
// attention step when nothing else is in the way -- no global memory traffic, no barriers, no
// tile walk, no dependence of the vector arithmetic on the matrix results.  Two workgroups of
// four waves per compute unit (the occupancy of k_attention); per v_mfma_f32_32x32x16_bf16 one
// operand fragment read from LDS (ds_read_b128), NV independent v_fma_f32 and NX v_exp_f32.
// The attention step issues, per MFMA, one fragment read, one exponential and about three other
// vector instructions (section 5.2: one exponential per score is what softmax attention costs).
// With RANDOM the operands are pseudo-random bf16 values in (-2, 2), as Q/K/V and the
// probabilities of the workloads are; without, small integers -- the chip is power-limited and
// the clock it sustains depends on how many bits toggle.
//
//   vsc_launch(variant, blocks, iters, out, stream): out = device buffer of blocks * 256 floats
//   (a checksum per thread, so that nothing is optimised away); returns 0, or -1 for a bad
//   variant.  FLOPs of a launch = blocks * 4 waves * iters * 16 MFMAs * 32768.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int NV, int NX, int RANDOM>
__global__ __launch_bounds__(256, 2) void k_mix(float* out, int iters, float seed) {
  __shared__ __attribute__((aligned(16))) __bf16 lds[16384];
  auto value = [&](uint32_t x) -> float {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return RANDOM ? ((int)(x & 0xffff) - 32768) * (1.0f / 16384.f) : seed + (x & 15);
  };
  for (int i = threadIdx.x; i < 16384; i += 256) lds[i] = (__bf16)value(i * 7919u + blockIdx.x);
  __syncthreads();
  const int lane = threadIdx.x & 63;
  bf16x8 b;
  for (int i = 0; i < 8; ++i) b[i] = (__bf16)value(threadIdx.x * 131u + i + 77u);
  f32x16 acc;
  float v[8];
  for (int i = 0; i < 8; ++i) v[i] = seed + i + threadIdx.x;
  // conflict-free fragment addresses (16-byte chunks XOR-swizzled by row, as the attention kernel lays K out)
  const int base = (lane & 31) * 128 + (((lane >> 5) ^ (lane & 15)) * 8);
  auto load = [&](int m) -> bf16x8 { return *(const bf16x8*)&lds[(base + m * 16) & 16383 & ~7]; };
  constexpr int PF = 3;   // fragments in flight, as in the attention kernel
  float sum = 0.f;
  for (int it = 0; it < iters; ++it) {
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    bf16x8 f[PF + 1];
#pragma unroll
    for (int j = 0; j < PF; ++j) f[j] = load(j);
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      if (m + PF < 16) f[(m + PF) % (PF + 1)] = load(m + PF);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[m % (PF + 1)], b, acc, 0, 0, 0);
#pragma unroll
      for (int x = 0; x < NV; ++x) v[x % 8] = __builtin_fmaf(v[x % 8], 1.0001f, seed);
#pragma unroll
      for (int x = 0; x < NX; ++x) v[(x + 4) % 8] = __builtin_amdgcn_exp2f(v[(x + 4) % 8]);
      __builtin_amdgcn_sched_barrier(0);
    }
    sum += acc[it & 15];
  }
  for (int i = 0; i < 8; ++i) sum += v[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}
}  // namespace

extern "C" int vsc_launch(int variant, int blocks, int iters, float* out, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  if (blocks < 1 || iters < 1 || !out) return -1;
  switch (variant) {
    case 0: hipLaunchKernelGGL((k_mix<0, 0, 0>), dim3(blocks), dim3(256), 0, st, out, iters, 0.5f); break;
    case 1: hipLaunchKernelGGL((k_mix<0, 0, 1>), dim3(blocks), dim3(256), 0, st, out, iters, 0.5f); break;
    case 2: hipLaunchKernelGGL((k_mix<3, 1, 0>), dim3(blocks), dim3(256), 0, st, out, iters, 0.5f); break;
    case 3: hipLaunchKernelGGL((k_mix<3, 1, 1>), dim3(blocks), dim3(256), 0, st, out, iters, 0.5f); break;
    case 4: hipLaunchKernelGGL((k_mix<2, 1, 1>), dim3(blocks), dim3(256), 0, st, out, iters, 0.5f); break;
    case 5: hipLaunchKernelGGL((k_mix<4, 1, 1>), dim3(blocks), dim3(256), 0, st, out, iters, 0.5f); break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
