// Recent-window column sums C (Eq. 2), summed over the query heads of each KV group.
//
// A workgroup owns 128 non-recent keys of one KV head (32 per wavefront, held in registers as the
// MFMA A operand for the whole kernel) and walks every window row of every query head of the group in
// blocks of 32 rows.  Scores are formed transposed (keys x queries) so a lane owns one query row of the
// block: it needs one log-sum-exp value and turns its 16 scores into probabilities exp(s - lse) in
// fp32.  Every lane keeps 16 running sums (one per key it sees); only at the very end are the 32 lanes
// that saw the same keys added together, in a fixed butterfly order.  No atomics: results are
// reproducible bit for bit.
#include "common.h"

namespace purekv {
namespace {

struct ImportanceArgs {
  const uint16_t* q;
  const uint16_t* k;
  const float* lse;
  float* c_out;
  int32_t N, Nv, P, Hq, G, w;
  uint32_t pattern;
  float scale_log2;
};

template <int D>
__global__ __launch_bounds__(256) void importance_kernel(const ImportanceArgs a) {
  constexpr int KSTEPS = D / 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int kvh = blockIdx.y;
  const int n_keys = a.N - a.w;           // non-recent keys
  const int jw = blockIdx.x * 128 + wave * 32;  // first key of this wavefront
  const int row0 = a.N - a.w;             // first window row

  bf16x8 kf[KSTEPS];
  {
    const int j = min(jw + n, a.N - 1);
    const uint16_t* kr = a.k + ((size_t)kvh * a.N + j) * D;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) kf[s] = *reinterpret_cast<const bf16x8*>(kr + 16 * s + 8 * h);
  }

  // Window rows that are text (or any row under the dense pattern) see every non-recent key: no mask.
  const bool need_mask = a.pattern != 0u && row0 < a.Nv;

  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  const int n_qblocks = (a.w + 31) / 32;
  for (int g = 0; g < a.G; ++g) {
    const int hq = kvh * a.G + g;
    for (int qb = 0; qb < n_qblocks; ++qb) {
      const int row = row0 + qb * 32 + n;
      const bool row_ok = row < a.N;
      const int rowc = min(row, a.N - 1);
      const uint16_t* qr = a.q + ((size_t)hq * a.N + rowc) * D;
      floatx16 sacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qr + 16 * s + 8 * h);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf, sacc, 0, 0, 0);
      }
      const float lse2 = a.lse[(size_t)hq * a.N + rowc] * kLog2e;
      if (!need_mask) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f(sacc[i] * a.scale_log2 - lse2);
          acc[i] += row_ok ? p : 0.f;
        }
      } else {
        const bool video = rowc < a.Nv;
        const int frame = video ? rowc / a.P : 0;
        const int own0 = frame * a.P;
        const int prev = (frame >= 1) ? rowc - a.P : -1;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = jw + 8 * (i >> 2) + 4 * h + (i & 3);
          bool ok = row_ok && j <= rowc;
          if (video) {
            bool allowed = j < a.P;
            if (a.pattern & 1u) allowed |= (j >= own0);
            if (a.pattern & 2u) allowed |= (j == prev) | (j == rowc);
            ok &= allowed && j < a.Nv;
          }
          const float p = __builtin_amdgcn_exp2f(sacc[i] * a.scale_log2 - lse2);
          acc[i] += ok ? p : 0.f;
        }
      }
    }
  }

  // Sum over the 32 query slots (lanes with equal h hold the same keys).
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float x = acc[i];
    x += __shfl_xor(x, 1, 64);
    x += __shfl_xor(x, 2, 64);
    x += __shfl_xor(x, 4, 64);
    x += __shfl_xor(x, 8, 64);
    x += __shfl_xor(x, 16, 64);
    acc[i] = x;
  }
  if (n == 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = jw + 8 * (i >> 2) + 4 * h + (i & 3);
      if (j < n_keys) a.c_out[(size_t)kvh * n_keys + j] = acc[i];
    }
  }
}

}  // namespace

int launch_importance(const purekv_plan& p, const void* q, const void* k, const float* lse, int32_t w,
                      float* c_out, hipStream_t st) {
  const int n_keys = p.g.N - w;
  if (n_keys <= 0) return PUREKV_OK;  // w == N: there is no non-recent segment
  ImportanceArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.lse = lse;
  a.c_out = c_out;
  a.N = p.g.N;
  a.Nv = p.g.Nv;
  a.P = p.g.P;
  a.Hq = p.g.Hq;
  a.G = p.g.G;
  a.w = w;
  a.pattern = p.g.pattern;
  a.scale_log2 = p.g.scale * kLog2e;
  const dim3 grid((unsigned)((n_keys + 127) / 128), (unsigned)p.g.Hkv), block(256);
  if (p.g.d == 128)
    hipLaunchKernelGGL(importance_kernel<128>, grid, block, 0, st, a);
  else
    hipLaunchKernelGGL(importance_kernel<64>, grid, block, 0, st, a);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
