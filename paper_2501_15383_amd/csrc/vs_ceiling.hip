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

// ---- the fused step of k_attention on its own --------------------------------------------------
// The arithmetic stream of one steady-state step (head_dim 128, one wave = 32 query rows, four waves
// and two workgroups per compute unit, as in the kernel): K Q^T of a 64-key tile, the exponentials
// of its scores, and V^T P^T of the tile before it, with the same operand layouts in LDS, the same
// interleaving and the same dependences -- but no tile walk, no masks, no pace keeping, and LDS tiles
// that either keep their first contents (COPY 0) or are refilled every step by the same global -> LDS
// copies as in the kernel (COPY 1: K and V, 32 KiB per step; COPY 2: K only) from a small buffer that
// stays in the L2.  What the kernel itself reaches on a dense list belongs next to the COPY 1 figure.
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

__device__ __forceinline__ void copy16x4(uint32_t lds_addr, const void* sbase, uint32_t o0, uint32_t o1,
                                         uint32_t o2, uint32_t o3, uint32_t step) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  step = __builtin_amdgcn_readfirstlane(step);
  const uint64_t b = (uint64_t)sbase;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  sbase = (const void*)(((uint64_t)hi << 32) | lo);
  asm volatile(
      "s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %5\n\t"
      "s_add_u32 m0, m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %5\n\t"
      "s_add_u32 m0, m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %5\n\t"
      "s_add_u32 m0, m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %5"
      :: "s"(lds_addr), "v"(o0), "v"(o1), "v"(o2), "v"(o3), "s"(sbase), "s"(step) : "memory", "scc");
}

constexpr int kStepSrcSlots = 32;                       // source tiles the copies cycle through
constexpr size_t kStepSrcBytes = (kStepSrcSlots + 1) * 65536;

template <int COPY>
__global__ __launch_bounds__(256, 2) void k_step(float* out, int iters, float c, const char* src) {
  constexpr int D = 128, DCH = 16, DSTEPS = 8, DB = 4, TILE = 64 * D, NM = 8, PF = 3, NB = PF + 1, NBQ = NM / 2;
  extern __shared__ __attribute__((aligned(16))) __bf16 tiles[];   // K buffers 0, 1, V buffers 0, 1
  __bf16* Ks = tiles;
  __bf16* Vs = tiles + 2 * TILE;
  auto value = [&](uint32_t x) -> float {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return ((int)(x & 0xffff) - 32768) * (1.0f / 65536.f);
  };
  for (int i = threadIdx.x; i < 4 * TILE; i += 256) tiles[i] = (__bf16)value(i * 7919u + blockIdx.x);
  __syncthreads();
  const int lane = threadIdx.x & 63, hh = lane >> 5, wv = threadIdx.x >> 6;
  uint32_t koff[4];   // a lane's 16 bytes in copy e of a tile: 64 rows of 256 bytes, 1 KiB apart (a [n][4][128] cache)
  for (int e = 0; e < 4; ++e) koff[e] = (uint32_t)((e * 16 + wv * 4 + (lane >> 4)) * 1024 + (lane & 15) * 16);
  const uint32_t ks_addr = (uint32_t)(size_t)(const __attribute__((address_space(3))) char*)Ks;
  const uint32_t vs_addr = (uint32_t)(size_t)(const __attribute__((address_space(3))) char*)Vs;
  bf16x8 qreg[DSTEPS];
  for (int s = 0; s < DSTEPS; ++s)
    for (int i = 0; i < 8; ++i) qreg[s][i] = (__bf16)value(threadIdx.x * 131u + s * 8 + i + 77u);
  int k_ofs[DSTEPS], v_ofs[DB];
  {
    const int y = hh ^ ((lane & 31) % DCH);
    for (int st = 0; st < DSTEPS; ++st) k_ofs[st] = (lane & 31) * D + ((2 * st) ^ y) * 8;
    const int rl = ((lane & 15) >> 2) + 4 * hh;
    const int gl = ((rl & 3) << 2) & (DCH - 1);
    const int ul = 2 * ((lane >> 4) & 1) + ((lane >> 1) & 1);
    for (int db = 0; db < DB; ++db) v_ofs[db] = rl * D + (((4 * db + ul) ^ gl) * 8) + 4 * (lane & 1);
  }
  auto k_load = [&](const __bf16* kb, int jb, int st) -> bf16x8 { return *(const bf16x8*)&kb[k_ofs[st] + 32 * jb * D]; };
  auto v_frag = [&](const __bf16* vb, int u) -> bf16x8 {
    typedef bf16x4 __attribute__((address_space(3))) * lds_b4;
    const __bf16* p0 = &vb[v_ofs[u % DB] + (32 * (u / NM) + 16 * ((u % NM) / DB)) * D];
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b4)(p0));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b4)(p0 + 8 * D));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  auto exp_pair = [&](const f32x16& sv, int x, float ref, bf16x8& P0, bf16x8& P1, float& ps) {
    f32x2 pf;
    pf[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x], c, -ref));
    pf[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x + 1], c, -ref));
    const bf16x2 pk = __builtin_convertvector(pf, bf16x2);
    ps += pf[0] + pf[1];
    bf16x8& P = x < 8 ? P0 : P1;
    P[x & 7] = pk[0];
    P[(x & 7) + 1] = pk[1];
  };
  f32x16 oacc[DB];
  for (int db = 0; db < DB; ++db) for (int x = 0; x < 16; ++x) oacc[db][x] = 0.f;
  bf16x8 pp[4];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 8; ++j) pp[i][j] = (__bf16)value(threadIdx.x * 17u + i * 8 + j);
  float l_run = 0.f;
  const float m_o = 1.0f;
  // MFMA n of the step: which operand it takes from LDS (K for the scores, V for the tile before)
  auto is_k = [&](int n) -> bool { return n < NM || (n < NM + 3 * NBQ && (n - NM) % 3 != 2); };
  auto k_index = [&](int n) -> int { return n < NM ? n : NM + 2 * ((n - NM) / 3) + (n - NM) % 3; };
  auto v_index = [&](int n) -> int { return n < NM + 3 * NBQ ? (n - NM) / 3 : n - NM - 2 * NBQ; };
  for (int it = 0; it < iters; ++it) {
    const int buf = it & 1;
    const __bf16* kb = Ks + buf * TILE;
    const __bf16* vbp = Vs + (buf ^ 1) * TILE;
    auto frag = [&](int n) -> bf16x8 {
      if (is_k(n)) return k_load(kb, k_index(n) / NM, k_index(n) % NM);
      return v_frag(vbp, v_index(n));
    };
    bf16x8 fq[NB];
    f32x16 sa, sn;
#pragma unroll
    for (int x = 0; x < 16; ++x) { sa[x] = 0.f; sn[x] = 0.f; }
#pragma unroll
    for (int j = 0; j < PF; ++j) fq[j] = frag(j);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (COPY != 0) {
      const char* kt = src + (size_t)(it % kStepSrcSlots) * 65536;
      copy16x4(ks_addr + (uint32_t)((buf ^ 1) * TILE * 2 + wv * 1024), kt, koff[0], koff[1], koff[2], koff[3], 4096);
      if (COPY == 1) copy16x4(vs_addr + (uint32_t)(buf * TILE * 2 + wv * 1024), kt + 256, koff[0], koff[1], koff[2], koff[3], 4096);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(2);
    bf16x8 q0, q1;
    float ps = 0.f;
    int xa = 0, xb = 0;
#pragma unroll
    for (int n = 0; n < 4 * NM; ++n) {
      if (n + PF < 4 * NM) fq[(n + PF) % NB] = frag(n + PF);
      if (is_k(n)) {
        const int ki = k_index(n);
        if (ki < NM) sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % NB], qreg[ki], sa, 0, 0, 0);
        else sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % NB], qreg[ki - NM], sn, 0, 0, 0);
      } else {
        const int u = v_index(n);
        oacc[u % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % NB], pp[u / DB], oacc[u % DB], 0, 0, 0);
      }
      if (n >= NM && n < NM + 3 * NBQ) {
        const int hi = 16 * (n - NM + 1) / (3 * NBQ);
        for (; xa + 2 <= hi; xa += 2) exp_pair(sa, xa, m_o, q0, q1, ps);
      } else if (n >= NM + 3 * NBQ) {
        const int hi = 16 * (n - NM - 3 * NBQ + 1) / (3 * NBQ);
        for (; xb + 2 <= hi; xb += 2) exp_pair(sn, xb, m_o, pp[0], pp[1], ps);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(0);
    l_run += ps;
    pp[2] = pp[0]; pp[3] = pp[1]; pp[0] = q0; pp[1] = q1;
    if (COPY != 0) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the copies of this step have landed
    __syncthreads();
  }
  float sum = l_run;
  for (int db = 0; db < DB; ++db) for (int x = 0; x < 16; ++x) sum += oacc[db][x];
  out[blockIdx.x * 256 + threadIdx.x] = sum;
}
}  // namespace

// Bytes of the source buffer vsc_launch_step reads (any contents; random bf16 values are what the
// workloads hold -- constant data lets the chip clock higher).
extern "C" size_t vsc_step_src_bytes(void) { return kStepSrcBytes; }

// variant 0: the step alone; 1: with the K and V copies of the kernel; 2: with the K copy only.
// src: device buffer of vsc_step_src_bytes() bytes.  FLOPs = blocks * 4 waves * iters * 32 MFMAs * 32768.
extern "C" int vsc_launch_step(int variant, int blocks, int iters, float* out, const void* src, size_t src_bytes,
                               void* stream) {
  hipStream_t st = (hipStream_t)stream;
  if (blocks < 1 || iters < 1 || !out || !src || src_bytes < kStepSrcBytes) return -1;
  const void* fn = variant == 0 ? (const void*)k_step<0> : variant == 1 ? (const void*)k_step<1> : variant == 2 ? (const void*)k_step<2> : nullptr;
  if (!fn) return -1;
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess) return -2;
  const float c = 0.05f;
  const char* s = (const char*)src;
  switch (variant) {
    case 0: hipLaunchKernelGGL(k_step<0>, dim3(blocks), dim3(256), 65536, st, out, iters, c, s); break;
    case 1: hipLaunchKernelGGL(k_step<1>, dim3(blocks), dim3(256), 65536, st, out, iters, c, s); break;
    default: hipLaunchKernelGGL(k_step<2>, dim3(blocks), dim3(256), 65536, st, out, iters, c, s); break;
  }
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

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
