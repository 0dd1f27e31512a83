// Decode attention of one new token against the compact cache (the decode stage of the paper's
// inference-speed table).  HBM/latency bound: the kept keys are cut into chunks, one workgroup per (chunk,
// KV head); every K/V row is read once and used for all query heads of the group.  A 16-lane group
// (8 lanes for head_dim 64) owns a key row: 16-byte loads, fp32 dot products on the vector ALU, online
// softmax per head; groups, wavefronts and finally chunks are merged with the usual (max, sum, output)
// rule in a fixed order.
#include "common.h"

namespace purekv {
namespace {

constexpr int DEC_CHUNK = 64;   // keys per workgroup
constexpr int GT = 8;           // query heads handled together (register tile)

inline int decode_splits(int n) { return n <= 0 ? 1 : (n + DEC_CHUNK - 1) / DEC_CHUNK; }

struct DecodeArgs {
  const uint16_t* q;
  const uint16_t* kc;
  const uint16_t* vc;
  uint16_t* out;
  float* ws_o;   // [n_splits, Hq, D] unnormalised partial outputs
  float* ws_ml;  // [n_splits, Hq, 2] running maximum (log2 domain) and sum
  int32_t Hq, G, n_cached, cap, n_splits;
  float scale_log2;
};

__device__ __forceinline__ void merge_state(float& m, float& l, float (&o)[8], float m2, float l2, const float (&o2)[8]) {
  const float mn = fmaxf(m, m2);
  const float mu = (mn == -INFINITY) ? 0.f : mn;
  const float a1 = __builtin_amdgcn_exp2f(m - mu), a2 = __builtin_amdgcn_exp2f(m2 - mu);
  l = l * a1 + l2 * a2;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = o[e] * a1 + o2[e] * a2;
  m = mn;
}

template <int D>
__global__ __launch_bounds__(256) void decode_kernel(const DecodeArgs a) {
  constexpr int LPR = D / 8;        // lanes per key row
  constexpr int GPW = 64 / LPR;     // row groups per wavefront
  constexpr int GPB = 4 * GPW;      // row groups per workgroup
  __shared__ float lds_o[4][GT][D];
  __shared__ float lds_ml[4][GT][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = wave * GPW + lane / LPR;
  const int split = blockIdx.x, kvh = blockIdx.y, g0 = blockIdx.z * GT;
  const int ng = min(GT, a.G - g0);
  const int c0 = split * DEC_CHUNK, c1 = min(c0 + DEC_CHUNK, a.n_cached);

  float qv[GT][8];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const int hq = kvh * a.G + g0 + min(g, ng - 1);
    const u32x4 x = *reinterpret_cast<const u32x4*>(a.q + (size_t)hq * D + sub * 8);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      qv[g][2 * w] = bf16_lo(x[w]) * a.scale_log2;
      qv[g][2 * w + 1] = bf16_hi(x[w]) * a.scale_log2;
    }
  }
  float m[GT], l[GT], o[GT][8];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
  }

  const uint16_t* kb = a.kc + (size_t)kvh * a.cap * D;
  const uint16_t* vb = a.vc + (size_t)kvh * a.cap * D;
  // all rows of this group are requested before the first is used (a chunk is at most RPG rows per group)
  constexpr int RPG = DEC_CHUNK / GPB;
  u32x4 kxs[RPG], vxs[RPG];
#pragma unroll
  for (int r = 0; r < RPG; ++r) {
    const int j = min(c0 + grp + r * GPB, a.n_cached - 1);
    kxs[r] = *reinterpret_cast<const u32x4*>(kb + (size_t)j * D + sub * 8);
    vxs[r] = *reinterpret_cast<const u32x4*>(vb + (size_t)j * D + sub * 8);
  }
#pragma unroll
  for (int r = 0; r < RPG; ++r) {
    if (c0 + grp + r * GPB >= c1) break;
    const u32x4 kx = kxs[r], vx = vxs[r];
    float kf[8], vf[8];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      kf[2 * w] = bf16_lo(kx[w]);
      kf[2 * w + 1] = bf16_hi(kx[w]);
      vf[2 * w] = bf16_lo(vx[w]);
      vf[2 * w + 1] = bf16_hi(vx[w]);
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s += qv[g][e] * kf[e];
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) s += __shfl_xor(s, off, 64);
      const float mn = fmaxf(m[g], s);
      const float al = __builtin_amdgcn_exp2f(m[g] - mn), p = __builtin_amdgcn_exp2f(s - mn);
      l[g] = l[g] * al + p;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[g][e] = o[g][e] * al + p * vf[e];
      m[g] = mn;
    }
  }

  // merge the row groups of a wavefront (butterfly: afterwards every group holds the wavefront's state)
#pragma unroll
  for (int g = 0; g < GT; ++g) {
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
      const float m2 = __shfl_xor(m[g], off, 64), l2 = __shfl_xor(l[g], off, 64);
      float o2[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o2[e] = __shfl_xor(o[g][e], off, 64);
      merge_state(m[g], l[g], o[g], m2, l2, o2);
    }
    if (lane < LPR) {
#pragma unroll
      for (int e = 0; e < 8; ++e) lds_o[wave][g][sub * 8 + e] = o[g][e];
      if (sub == 0) {
        lds_ml[wave][g][0] = m[g];
        lds_ml[wave][g][1] = l[g];
      }
    }
  }
  __syncthreads();
  // merge the four wavefronts; thread t -> (head t / D, element t % D)
  for (int t = tid; t < ng * D; t += 256) {
    const int g = t / D, dd = t % D;
    float mn = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) mn = fmaxf(mn, lds_ml[wv][g][0]);
    const float mu = (mn == -INFINITY) ? 0.f : mn;
    float acc = 0.f, ls = 0.f;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      const float sc = __builtin_amdgcn_exp2f(lds_ml[wv][g][0] - mu);
      acc += lds_o[wv][g][dd] * sc;
      ls += lds_ml[wv][g][1] * sc;
    }
    const int hq = kvh * a.G + g0 + g;
    a.ws_o[((size_t)split * a.Hq + hq) * D + dd] = acc;
    if (dd == 0) {
      a.ws_ml[((size_t)split * a.Hq + hq) * 2] = mn;
      a.ws_ml[((size_t)split * a.Hq + hq) * 2 + 1] = ls;
    }
  }
}

// One workgroup per query head; thread -> (output element, one of MERGE_PARTS interleaved subsets of the chunks).
// A thread requests all its chunks' values before it combines them; the subsets are combined through LDS in a
// fixed order.
constexpr int MERGE_PARTS = 4;
template <int D>
__global__ __launch_bounds__(D * MERGE_PARTS) void decode_merge_kernel(const DecodeArgs a) {
  __shared__ float sm[MERGE_PARTS][D], sl[MERGE_PARTS], smax[MERGE_PARTS];
  const int hq = blockIdx.x, dd = threadIdx.x % D, part = threadIdx.x / D;
  constexpr int U = 8;
  float mn = -INFINITY;
  for (int s0 = part; s0 < a.n_splits; s0 += MERGE_PARTS * U) {
    float mv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = s0 + u * MERGE_PARTS;
      mv[u] = s < a.n_splits ? a.ws_ml[((size_t)s * a.Hq + hq) * 2] : -INFINITY;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) mn = fmaxf(mn, mv[u]);
  }
  if (dd == 0) smax[part] = mn;
  __syncthreads();
  mn = smax[0];
#pragma unroll
  for (int p2 = 1; p2 < MERGE_PARTS; ++p2) mn = fmaxf(mn, smax[p2]);
  float acc = 0.f, ls = 0.f;
  for (int s0 = part; s0 < a.n_splits; s0 += MERGE_PARTS * U) {
    float mv[U], ov[U], lv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = min(s0 + u * MERGE_PARTS, a.n_splits - 1);
      mv[u] = a.ws_ml[((size_t)s * a.Hq + hq) * 2];
      lv[u] = a.ws_ml[((size_t)s * a.Hq + hq) * 2 + 1];
      ov[u] = a.ws_o[((size_t)s * a.Hq + hq) * D + dd];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (s0 + u * MERGE_PARTS < a.n_splits) {
        const float sc = __builtin_amdgcn_exp2f(mv[u] - mn);
        acc += ov[u] * sc;
        ls += lv[u] * sc;
      }
    }
  }
  sm[part][dd] = acc;
  if (dd == 0) sl[part] = ls;
  __syncthreads();
  if (part == 0) {
#pragma unroll
    for (int p2 = 1; p2 < MERGE_PARTS; ++p2) {
      acc += sm[p2][dd];
      ls += sl[p2];
    }
    a.out[(size_t)hq * D + dd] = (uint16_t)f32_to_bf16(acc / ls);
  }
}

}  // namespace

size_t decode_ws_bytes(const purekv_plan& p, int32_t cap) {
  return (size_t)decode_splits(cap) * p.g.Hq * (p.g.d + 2) * sizeof(float);
}

int launch_decode(const purekv_plan& p, const void* q_new, const void* kc, const void* vc, int32_t n_cached,
                  int32_t cap, void* out, void* ws, hipStream_t st) {
  DecodeArgs a;
  a.q = static_cast<const uint16_t*>(q_new);
  a.kc = static_cast<const uint16_t*>(kc);
  a.vc = static_cast<const uint16_t*>(vc);
  a.out = static_cast<uint16_t*>(out);
  a.n_splits = decode_splits(n_cached);
  a.ws_o = static_cast<float*>(ws);
  a.ws_ml = a.ws_o + (size_t)decode_splits(cap) * p.g.Hq * p.g.d;
  a.Hq = p.g.Hq;
  a.G = p.g.G;
  a.n_cached = n_cached;
  a.cap = cap;
  a.scale_log2 = p.g.scale * kLog2e;
  const dim3 grid((unsigned)a.n_splits, (unsigned)p.g.Hkv, (unsigned)((p.g.G + GT - 1) / GT));
  if (p.g.d == 128) {
    hipLaunchKernelGGL(decode_kernel<128>, grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(decode_merge_kernel<128>, dim3((unsigned)p.g.Hq), dim3(128 * MERGE_PARTS), 0, st, a);
  } else {
    hipLaunchKernelGGL(decode_kernel<64>, grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(decode_merge_kernel<64>, dim3((unsigned)p.g.Hq), dim3(64 * MERGE_PARTS), 0, st, a);
  }
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
