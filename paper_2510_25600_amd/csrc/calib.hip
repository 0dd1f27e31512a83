// Board calibration, not a step of the method: a register-resident loop of the matrix instruction the prefill
// kernel is built on (v_mfma_f32_32x32x16_bf16), alone or with the per-MFMA companions of an attention tile, on the
// same grid as the prefill kernel (one workgroup of eight wavefronts per CU, two wavefronts per SIMD).  It answers
// "what does this board sustain for this instruction mix and this kind of data", which is what the prefill kernel's
// rate has to be read against: the shader clock settles where the board's power limit puts it, and the power an
// MFMA draws depends on how many operand bits change from one instruction to the next.
#include "common.h"

namespace purekv {
namespace {

constexpr int CALIB_MFMAS = 16;   // MFMAs per wavefront and outer iteration

// MIX 0: MFMA only.  MIX 1: every MFMA takes its A operand from a fresh 1 KB LDS fragment read (the score product's
// K fragments).  MIX 2: MIX 1 plus the vector work of one exponential slot (2 multiply-adds, 2 v_exp_f32, 1 convert
// to packed bf16) per MFMA.
template <int MIX>
__global__ __launch_bounds__(512, 1) void calib_mfma_kernel(float* sink, unsigned long long* ticks, int iters,
                                                            int random_operands) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[2 * 64 * 128];
  const int lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 2 * 64 * 128; i += blockDim.x) {
    // bf16 bits of a value in (-1, 1) from a multiplicative hash, or a constant pattern
    const float r = ((int)((((uint32_t)i + 1u) * 2654435761u) >> 16 & 0xFFFFu) - 32768) * (1.0f / 32768.f);
    tile[i] = random_operands ? (uint16_t)(__float_as_uint(r) >> 16) : (uint16_t)0x3c00;
  }
  bf16x8 b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t hsh = ((uint32_t)(lane * 8 + i) + blockIdx.x * 977u + threadIdx.x * 131u) * 2654435761u;
    const float r = ((int)(hsh >> 16 & 0xFFFFu) - 32768) * (1.0f / 32768.f) * 0.02f;
    b[i] = random_operands ? (__bf16)r : (__bf16)0.5f;
  }
  floatx16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = 0.001f * (float)(lane + i);
  const float c1 = -6.0f, c2 = 0.0001f;   // x -> 2^(c1 x + c2) stays in (0, 1] and keeps oscillating
  uint32_t pk = 0;
  // same swizzled fragment addresses as the score product's K reads
  const int kq0 = kswz<128>(lane & 31, lane >> 5);
  bf16x8 f[3];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) f[i] = *reinterpret_cast<const bf16x8*>(tile + (kq0 ^ (16 * i)));
  const unsigned long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < CALIB_MFMAS; ++i) {
      if (MIX >= 1)
        f[(i + 2) % 3] = *reinterpret_cast<const bf16x8*>(tile + (it & 1) * 8192 + (kq0 ^ (16 * ((i + 2) & 7))));
      acc[i % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(MIX >= 1 ? f[i % 3] : b, b, acc[i % 4], 0, 0, 0);
      if (MIX >= 2) {
        float y0 = x[(2 * i) % 8], y1 = x[(2 * i + 1) % 8];
        asm volatile("v_fma_f32 %0, %0, %2, %3\n\tv_fma_f32 %1, %1, %2, %3" : "+v"(y0), "+v"(y1) : "v"(c1), "v"(c2));
        asm volatile("v_exp_f32 %0, %0\n\tv_exp_f32 %1, %1" : "+v"(y0), "+v"(y1));
        asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(y0), "v"(y1));
        x[(2 * i) % 8] = y0;
        x[(2 * i + 1) % 8] = y1;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = (float)pk;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    ticks[0] = t1 - t0;   // shader cycles of wavefront 0
    ticks[1] = r1 - r0;   // the same span on the constant 100 MHz counter
  }
}

}  // namespace

double calib_mfma_flops(const purekv_plan& p, int32_t iters) {
  return 2.0 * 32 * 32 * 16 * CALIB_MFMAS * (double)iters * PUREKV_WAVES * (double)p.n_queues;
}

int launch_calib_mfma(const purekv_plan& p, int mix, int random_operands, int32_t iters, float* sink, uint64_t* ticks,
                      hipStream_t st) {
  const dim3 grid((unsigned)p.n_queues), block(512);
  auto* tk = reinterpret_cast<unsigned long long*>(ticks);
  switch (mix) {
    case 0: hipLaunchKernelGGL(calib_mfma_kernel<0>, grid, block, 0, st, sink, tk, iters, random_operands); break;
    case 1: hipLaunchKernelGGL(calib_mfma_kernel<1>, grid, block, 0, st, sink, tk, iters, random_operands); break;
    default: hipLaunchKernelGGL(calib_mfma_kernel<2>, grid, block, 0, st, sink, tk, iters, random_operands); break;
  }
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
