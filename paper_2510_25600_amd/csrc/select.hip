// V-norm weighting (Eq. 3 / Eq. 4) and per-KV-head selection "top h of the non-recent segment plus
// the recent window" (Sec. 3.1), batched over layers that share one C.
//
//   score kernel : S[l, kv, j] = C[kv, j] * ||V[l, kv, j, :]||_2.  Pure HBM stream over V: one 16-lane
//                  group per row, 16-byte loads, fp32 sum of squares, fixed-order lane reduction.
//   select kernel: one workgroup per (layer, KV head).  MSB-first radix select over the order-preserving
//                  integer image of the fp32 scores finds the h-th largest value exactly; an ordered
//                  pass then emits, ascending, every index above it plus the lowest-index ties.
//                  Integer work only: the result is the one a stable full sort would give.
#include "common.h"

namespace purekv {
namespace {

constexpr int SEL_THREADS = 1024;

// Order-preserving map from fp32 to uint32 (-0.0 first folded onto +0.0).
__device__ __forceinline__ uint32_t sort_key(float s) {
  const uint32_t u = __float_as_uint(s + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int D>
__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ c, const uint16_t* __restrict__ v,
                                                    int64_t v_layer_stride, float* __restrict__ s_out, int32_t N,
                                                    int32_t n_keys, int32_t Hkv, int64_t total_rows) {
  constexpr int LPR = D / 8;         // lanes per row
  constexpr int RPB = 256 / LPR;     // rows per block pass
  constexpr int UNROLL = 4;
  const int sub = threadIdx.x % LPR, rslot = threadIdx.x / LPR;
  for (int64_t base = (int64_t)blockIdx.x * RPB * UNROLL; base < total_rows;
       base += (int64_t)gridDim.x * RPB * UNROLL) {
    u32x4 x[UNROLL];
    int64_t rid[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      rid[u] = base + u * RPB + rslot;
      const int64_t r = rid[u] < total_rows ? rid[u] : total_rows - 1;
      const int64_t lk = r / n_keys;  // layer * Hkv + kv
      const int32_t j = (int32_t)(r - lk * n_keys);
      const int64_t layer = lk / Hkv, kvh = lk - layer * Hkv;
      x[u] = *reinterpret_cast<const u32x4*>(v + layer * v_layer_stride + (kvh * N + j) * D + sub * 8);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      float ss = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float lo = bf16_lo(x[u][w]), hi = bf16_hi(x[u][w]);
        ss += lo * lo + hi * hi;
      }
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o, 64);
      if (sub == 0 && rid[u] < total_rows) {
        const int64_t lk = rid[u] / n_keys;
        const int64_t kvh = lk % Hkv;
        const int32_t j = (int32_t)(rid[u] - lk * n_keys);
        s_out[rid[u]] = c[kvh * n_keys + j] * __builtin_sqrtf(ss);
      }
    }
  }
}

// Block-wide exclusive scan of two counters (1024 threads = 16 wavefronts).
__device__ __forceinline__ void block_scan2(uint32_t& a, uint32_t& b, uint32_t* lds /* 34 words */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t ia = a, ib = b;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t ta = __shfl_up(ia, o, 64), tb = __shfl_up(ib, o, 64);
    if (lane >= o) {
      ia += ta;
      ib += tb;
    }
  }
  if (lane == 63) {
    lds[wave] = ia;
    lds[16 + wave] = ib;
  }
  __syncthreads();
  uint32_t oa = 0, ob = 0;
  for (int wv = 0; wv < wave; ++wv) {
    oa += lds[wv];
    ob += lds[16 + wv];
  }
  a = oa + ia - a;
  b = ob + ib - b;
  __syncthreads();
}

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(const float* __restrict__ s, int32_t* __restrict__ idx_out,
                                                             int32_t N, int32_t w, int32_t h) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t scan_lds[34];
  __shared__ uint32_t sel[2];  // chosen digit, remaining count
  const int tid = threadIdx.x, lane = tid & 63;
  const int n_keys = N - w;
  const float* sv = s + (size_t)blockIdx.x * n_keys;
  int32_t* out = idx_out + (size_t)blockIdx.x * (h + w);

  for (int t = tid; t < w; t += SEL_THREADS) out[h + t] = N - w + t;
  if (h == 0) return;

  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)h;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int j0 = 0; j0 < n_keys; j0 += SEL_THREADS) {
      const int j = j0 + tid;
      const bool in = j < n_keys;
      const uint32_t u = in ? sort_key(sv[j]) : 0u;
      const bool cand = in && ((u & mask) == prefix);
      const uint32_t dgt = (u >> shift) & 255u;
      // wave-uniform digits (the common case for the exponent byte) cost one atomic per wavefront
      const uint64_t votes = __ballot(cand);
      if (votes != 0) {
        const int leader = __ffsll((unsigned long long)votes) - 1;
        const uint32_t d0 = __shfl(dgt, leader, 64);
        const bool uniform = __all(!cand || dgt == d0);
        if (uniform) {
          if (lane == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(votes));
        } else if (cand) {
          atomicAdd(&hist[dgt], 1u);
        }
      }
    }
    __syncthreads();
    if (tid < 64) {
      // lane t owns digits 255-4t .. 252-4t (descending); find where the count from the top reaches `remaining`
      uint32_t cnt[4], tot = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        cnt[r] = hist[255 - 4 * tid - r];
        tot += cnt[r];
      }
      uint32_t inc = tot;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t tv = __shfl_up(inc, o, 64);
        if (tid >= o) inc += tv;
      }
      const uint32_t before = inc - tot;  // elements with larger digits than this lane's
      if (before < remaining && remaining <= inc) {
        uint32_t run = before;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (run < remaining && remaining <= run + cnt[r]) {
            sel[0] = 255 - 4 * tid - r;
            sel[1] = remaining - run;
          }
          run += cnt[r];
        }
      }
    }
    __syncthreads();
    prefix |= sel[0] << shift;
    mask |= 255u << shift;
    remaining = sel[1];
    __syncthreads();
  }
  // prefix = key of the h-th largest score; `remaining` of the keys equal to it are kept (lowest indices)
  const uint32_t tau = prefix, need = remaining;
  const int chunk = (n_keys + SEL_THREADS - 1) / SEL_THREADS;
  const int jb = tid * chunk, je = min(jb + chunk, n_keys);
  uint32_t gt = 0, eq = 0;
  for (int j = jb; j < je; ++j) {
    const uint32_t u = sort_key(sv[j]);
    gt += u > tau;
    eq += u == tau;
  }
  block_scan2(gt, eq, scan_lds);
  for (int j = jb; j < je; ++j) {
    const uint32_t u = sort_key(sv[j]);
    if (u > tau) {
      out[gt + min(eq, need)] = j;
      ++gt;
    } else if (u == tau) {
      if (eq < need) out[gt + eq] = j;
      ++eq;
    }
  }
}

}  // namespace

size_t topk_ws_bytes(const purekv_plan& p, int32_t n_layers, int32_t w) {
  // scores, when the caller does not ask for them
  const int64_t n_keys = (int64_t)p.g.N - w;
  return n_keys > 0 ? (size_t)n_layers * p.g.Hkv * n_keys * sizeof(float) : 0;
}

int launch_topk(const purekv_plan& p, const float* c, const void* v, int64_t v_layer_stride, int32_t n_layers,
                int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws, hipStream_t st) {
  const int32_t n_keys = p.g.N - w;
  const float* scores = c;
  if (v != nullptr && n_keys > 0) {
    float* sbuf = s_out ? s_out : static_cast<float*>(ws);
    const int64_t total = (int64_t)n_layers * p.g.Hkv * n_keys;
    const int lpr = p.g.d / 8, rows_per_block = (256 / lpr) * 4;
    const int64_t want = (total + rows_per_block - 1) / rows_per_block;
    const unsigned grid = (unsigned)(want < 65536 ? want : 65536);
    if (p.g.d == 128)
      hipLaunchKernelGGL(score_kernel<128>, dim3(grid), dim3(256), 0, st, c, static_cast<const uint16_t*>(v),
                         v_layer_stride, sbuf, p.g.N, n_keys, p.g.Hkv, total);
    else
      hipLaunchKernelGGL(score_kernel<64>, dim3(grid), dim3(256), 0, st, c, static_cast<const uint16_t*>(v),
                         v_layer_stride, sbuf, p.g.N, n_keys, p.g.Hkv, total);
    scores = sbuf;
  } else if (s_out != nullptr && n_keys > 0) {
    PUREKV_HIP_TRY(hipMemcpyAsync(s_out, c, (size_t)p.g.Hkv * n_keys * sizeof(float), hipMemcpyDeviceToDevice, st));
  }
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)(n_layers * p.g.Hkv)), dim3(SEL_THREADS), 0, st, scores, idx_out,
                     p.g.N, w, h);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
