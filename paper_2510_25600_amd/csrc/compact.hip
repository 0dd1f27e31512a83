// KV-cache compaction: gather of the kept rows (selection rule of Sec. 3.1) into a compact cache, and the
// append of one decoded token.  Pure byte movement: one 16-lane group (8 for head_dim 64) moves one
// row of K and one of V with 16-byte loads and stores; indices ascend, so reads walk HBM forwards.
#include "common.h"

namespace purekv {
namespace {

template <int D>
__global__ __launch_bounds__(256) void compact_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                      int64_t layer_stride, int64_t head_stride, int64_t tok_stride,
                                                      const int32_t* __restrict__ idx,
                                                      uint16_t* __restrict__ kc, uint16_t* __restrict__ vc, int32_t N,
                                                      int32_t Hkv, int32_t n_keep, int32_t cap, int64_t total_rows) {
  constexpr int LPR = D / 8, RPB = 256 / LPR, UNROLL = 4;
  const int sub = threadIdx.x % LPR, rslot = threadIdx.x / LPR;
  for (int64_t base = (int64_t)blockIdx.x * RPB * UNROLL; base < total_rows;
       base += (int64_t)gridDim.x * RPB * UNROLL) {
    u32x4 xk[UNROLL], xv[UNROLL];
    int64_t dst[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t rid = base + u * RPB + rslot;
      const int64_t r = rid < total_rows ? rid : total_rows - 1;
      const int64_t lk = r / n_keep;  // layer * Hkv + kv
      const int32_t pos = (int32_t)(r - lk * n_keep);
      const int64_t layer = lk / Hkv, kvh = lk - layer * Hkv;
      int32_t j = idx[r];
      j = j < 0 ? 0 : (j >= N ? N - 1 : j);
      const int64_t src = layer * layer_stride + kvh * head_stride + j * tok_stride + sub * 8;
      xk[u] = *reinterpret_cast<const u32x4*>(k + src);
      xv[u] = *reinterpret_cast<const u32x4*>(v + src);
      dst[u] = rid < total_rows ? (lk * cap + pos) * D + sub * 8 : -1;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (dst[u] >= 0) {
        // (non-temporal: the compact cache is written once here and read by a later launch: 28.0 against 29.0 us
        // for the 26-layer batch of the 32-frame shape; the same hint on the gathered loads costs 8 %)
        __builtin_nontemporal_store(xk[u], reinterpret_cast<u32x4*>(kc + dst[u]));
        __builtin_nontemporal_store(xv[u], reinterpret_cast<u32x4*>(vc + dst[u]));
      }
  }
}

__global__ void append_kernel(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                              uint16_t* __restrict__ kc, uint16_t* __restrict__ vc, int32_t Hkv, int32_t d,
                              int32_t n_cached, int32_t cap) {
  const int chunks = d / 8;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= Hkv * chunks) return;
  const int kvh = t / chunks, c = t % chunks;
  const size_t dst = ((size_t)kvh * cap + n_cached) * d + c * 8, src = (size_t)kvh * d + c * 8;
  *reinterpret_cast<u32x4*>(kc + dst) = *reinterpret_cast<const u32x4*>(k_new + src);
  *reinterpret_cast<u32x4*>(vc + dst) = *reinterpret_cast<const u32x4*>(v_new + src);
}

}  // namespace

int launch_compact(const purekv_plan& p, const void* k, const void* v, int64_t kv_layer_stride, int32_t n_layers,
                   const int32_t* idx, int32_t n_keep, void* kc, void* vc, int32_t cap, hipStream_t st) {
  const int64_t total = (int64_t)n_layers * p.g.Hkv * n_keep;
  if (total == 0) return PUREKV_OK;
  const int lpr = p.g.d / 8, rows_per_block = (256 / lpr) * 4;
  const int64_t want = (total + rows_per_block - 1) / rows_per_block;
  const unsigned grid = (unsigned)(want < 65536 ? want : 65536);
  if (p.g.d == 128)
    hipLaunchKernelGGL(compact_kernel<128>, dim3(grid), dim3(256), 0, st, static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), kv_layer_stride, p.g.kv_sh, p.g.kv_st, idx, static_cast<uint16_t*>(kc),
                       static_cast<uint16_t*>(vc), p.g.N, p.g.Hkv, n_keep, cap, total);
  else
    hipLaunchKernelGGL(compact_kernel<64>, dim3(grid), dim3(256), 0, st, static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), kv_layer_stride, p.g.kv_sh, p.g.kv_st, idx, static_cast<uint16_t*>(kc),
                       static_cast<uint16_t*>(vc), p.g.N, p.g.Hkv, n_keep, cap, total);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

int launch_append(const purekv_plan& p, const void* k_new, const void* v_new, void* kc, void* vc, int32_t n_cached,
                  int32_t cap, hipStream_t st) {
  const int total = p.g.Hkv * (p.g.d / 8);
  hipLaunchKernelGGL(append_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                     static_cast<uint16_t*>(kc), static_cast<uint16_t*>(vc), p.g.Hkv, p.g.d, n_cached, cap);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
