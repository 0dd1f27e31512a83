// V-norm weighting (Eq. 3 / Eq. 4) and per-KV-head selection "top h of the non-recent segment plus
// the recent window" (Sec. 3.1), batched over layers that share one C.
//
//   score kernel : S[l, kv, j] = C[kv, j] * ||V[l, kv, j, :]||_2.  Pure HBM stream over V: one 16-lane
//                  group per row, 16-byte loads (8 rows in flight per group), fp32 sum of squares,
//                  fixed-order lane reduction.
//   select kernel: one workgroup per (layer, KV head).  The h-th largest value is found exactly on the
//                  order-preserving integer image of the fp32 scores by an MSB-first radix select (rows of up to
//                  32768 scores stay in registers and are read from memory once; longer rows re-read L2 in
//                  every pass); an ordered pass then emits, ascending, every
//                  index above it plus the lowest-index ties.  Integer work only: the result is the one a
//                  stable full sort would give.
#include <mutex>

#include "common.h"

namespace purekv {
namespace {

constexpr int SEL_THREADS = 1024;

// Order-preserving map from fp32 to uint32 (-0.0 first folded onto +0.0).
__device__ __forceinline__ uint32_t sort_key(float s) {
  const uint32_t u = __float_as_uint(s + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// grid = (row blocks, layers * Hkv): a workgroup streams SCORE_ROWS consecutive rows of one (layer, KV head).
constexpr int SCORE_UNROLL = 8;
// Cross-lane primitives on the DPP path of the vector ALU (a few cycles each; the generic shuffles go through
// the LDS crossbar, ~100 cycles a step with 16 wavefronts on the CU).
// row_shr:n = 0x110 + n moves a value n lanes up within a row of 16 lanes; row_bcast:15 (0x142) hands lane 15 of
// each row to the next row, row_bcast:31 (0x143) lane 31 to rows 2 and 3.  Lanes without a source receive `ident`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_move(uint32_t ident, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)ident, (int)v, CTRL, ROW_MASK, 0xf, false);
}
// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t v) {
  v += dpp_move<0x111, 0xf>(0u, v);
  v += dpp_move<0x112, 0xf>(0u, v);
  v += dpp_move<0x114, 0xf>(0u, v);
  v += dpp_move<0x118, 0xf>(0u, v);
  v += dpp_move<0x142, 0xa>(0u, v);
  v += dpp_move<0x143, 0xc>(0u, v);
  return v;
}
// Minimum / maximum over the wavefront, valid in lane 63 (the scans run upwards).
__device__ __forceinline__ uint32_t wave_scan_min(uint32_t v) {
  v = min(v, dpp_move<0x111, 0xf>(0xffffffffu, v));
  v = min(v, dpp_move<0x112, 0xf>(0xffffffffu, v));
  v = min(v, dpp_move<0x114, 0xf>(0xffffffffu, v));
  v = min(v, dpp_move<0x118, 0xf>(0xffffffffu, v));
  v = min(v, dpp_move<0x142, 0xa>(0xffffffffu, v));
  v = min(v, dpp_move<0x143, 0xc>(0xffffffffu, v));
  return v;
}
__device__ __forceinline__ uint32_t wave_scan_max(uint32_t v) {
  v = max(v, dpp_move<0x111, 0xf>(0u, v));
  v = max(v, dpp_move<0x112, 0xf>(0u, v));
  v = max(v, dpp_move<0x114, 0xf>(0u, v));
  v = max(v, dpp_move<0x118, 0xf>(0u, v));
  v = max(v, dpp_move<0x142, 0xa>(0u, v));
  v = max(v, dpp_move<0x143, 0xc>(0u, v));
  return v;
}

template <int D>
__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ c, const uint16_t* __restrict__ v,
                                                    int64_t v_layer_stride, int64_t v_head_stride,
                                                    int64_t v_tok_stride, float* __restrict__ s_out,
                                                    int32_t n_keys, int32_t Hkv) {
  constexpr int LPR = D / 8;         // lanes per row
  constexpr int RPB = 256 / LPR;     // rows per pass of the workgroup
  const int sub = threadIdx.x % LPR, rslot = threadIdx.x / LPR;
  const int lk = blockIdx.y, layer = lk / Hkv, kvh = lk - layer * Hkv;
  const uint16_t* vh = v + (int64_t)layer * v_layer_stride + (int64_t)kvh * v_head_stride;
  const int j0 = blockIdx.x * (RPB * SCORE_UNROLL) + rslot;
  u32x4 x[SCORE_UNROLL];
#pragma unroll
  for (int u = 0; u < SCORE_UNROLL; ++u) {
    const int j = min(j0 + u * RPB, n_keys - 1);
    x[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vh + (int64_t)j * v_tok_stride + sub * 8));
  }
#pragma unroll
  for (int u = 0; u < SCORE_UNROLL; ++u) {
    float ss = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float lo = bf16_lo(x[u][w]), hi = bf16_hi(x[u][w]);
      ss += lo * lo + hi * hi;
    }
#pragma unroll
    for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o, 64);
    const int j = j0 + u * RPB;
    if (sub == 0 && j < n_keys) s_out[(int64_t)lk * n_keys + j] = c[(int64_t)kvh * n_keys + j] * __builtin_sqrtf(ss);
  }
}

// Squared norms of all V rows of one layer, as a pass of its own (same access pattern as the score kernel).
template <int D>
__global__ __launch_bounds__(256) void vnorm2_kernel(const uint16_t* __restrict__ v, int64_t v_head_stride,
                                                     int64_t v_tok_stride, float* __restrict__ n2_out, int32_t N,
                                                     int32_t kvh0) {
  constexpr int LPR = D / 8, RPB = 256 / LPR;
  const int sub = threadIdx.x % LPR, rslot = threadIdx.x / LPR;
  const int kvh = kvh0 + blockIdx.y;
  const uint16_t* vh = v + (int64_t)kvh * v_head_stride;
  const int j0 = blockIdx.x * (RPB * SCORE_UNROLL) + rslot;
  u32x4 x[SCORE_UNROLL];
#pragma unroll
  for (int u = 0; u < SCORE_UNROLL; ++u) {
    const int j = min(j0 + u * RPB, N - 1);
    x[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vh + (int64_t)j * v_tok_stride + sub * 8));
  }
#pragma unroll
  for (int u = 0; u < SCORE_UNROLL; ++u) {
    float ss = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float lo = bf16_lo(x[u][w]), hi = bf16_hi(x[u][w]);
      ss += lo * lo + hi * hi;
    }
#pragma unroll
    for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o, 64);
    const int j = j0 + u * RPB;
    if (sub == 0 && j < N) n2_out[(int64_t)kvh * N + j] = ss;
  }
}

// The same scores from squared norms that already exist (the prefill kernel emits them while the V tiles are in
// LDS): S[l, kv, j] = C[kv, j] * sqrt(n2[l, kv, j]).  4 bytes per key instead of a V row.
__global__ __launch_bounds__(256) void score_from_norms_kernel(const float* __restrict__ c, const float* __restrict__ n2,
                                                               int64_t n2_layer_stride, float* __restrict__ s_out,
                                                               int32_t N, int32_t n_keys, int32_t Hkv) {
  const int lk = blockIdx.y, layer = lk / Hkv, kvh = lk - layer * Hkv;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n_keys) return;
  const float x = n2[(int64_t)layer * n2_layer_stride + (int64_t)kvh * N + j];
  s_out[(int64_t)lk * n_keys + j] = c[(int64_t)kvh * n_keys + j] * __builtin_sqrtf(x);
}

// Block-wide exclusive scan of two counters (1024 threads = 16 wavefronts).
__device__ __forceinline__ void block_scan2(uint32_t& a, uint32_t& b, uint32_t* lds /* 34 words */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t ia = wave_scan_add(a), ib = wave_scan_add(b);
  if (lane == 63) {
    lds[wave] = ia;
    lds[16 + wave] = ib;
  }
  __syncthreads();
  // lanes 0..15 scan the 16 wavefront totals of a, lanes 16..31 those of b (one row of 16 lanes each)
  uint32_t tot = lane < 32 ? lds[lane] : 0u, inc = tot;
  inc += dpp_move<0x111, 0xf>(0u, inc);
  inc += dpp_move<0x112, 0xf>(0u, inc);
  inc += dpp_move<0x114, 0xf>(0u, inc);
  inc += dpp_move<0x118, 0xf>(0u, inc);
  const uint32_t excl = inc - tot;
  const uint32_t oa = __builtin_amdgcn_readlane(excl, wave), ob = __builtin_amdgcn_readlane(excl, 16 + wave);
  a = oa + ia - a;
  b = ob + ib - b;
  __syncthreads();
}

// EPT = scores per thread: thread t owns the contiguous scores [t * chunk, (t + 1) * chunk), chunk <= EPT, and keeps
// their integer images in registers, so the scores are read from memory once.
//
// MSB-first radix select, 8 bits a pass, LDS histogram.  The passes start at the highest bit in which the keys
// differ at all (floats of similar size share sign and most of the exponent: starting at bit 31 would send every
// key to one or two bins, and LDS atomics to one address are serialised); below that bit the digits spread.
template <int EPT>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(const float* __restrict__ s, int32_t* __restrict__ idx_out,
                                                             int32_t N, int32_t w, int32_t h) {
  constexpr int HCOPIES = 16, HSTRIDE = 257;
  __shared__ uint32_t hist[HCOPIES * HSTRIDE];
  __shared__ uint32_t total[256];
  __shared__ uint32_t scan_lds[34];
  __shared__ uint32_t sel[2];        // chosen digit, remaining count
  __shared__ uint32_t ext[2][16];    // per-wavefront minimum and maximum key
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_keys = N - w;
  const float* sv = s + (size_t)blockIdx.x * n_keys;
  int32_t* out = idx_out + (size_t)blockIdx.x * (h + w);

  for (int t = tid; t < w; t += SEL_THREADS) out[h + t] = N - w + t;
  if (h == 0) return;

  const int chunk = (n_keys + SEL_THREADS - 1) / SEL_THREADS;   // <= EPT (checked by the launcher)
  const int jb = tid * chunk;
  const int live = max(0, min(chunk, n_keys - jb));             // valid entries of key[]
  uint32_t key[EPT];
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int i = tid; i < HCOPIES * HSTRIDE; i += SEL_THREADS) hist[i] = 0;   // every pass leaves it cleared again
  // The row comes in with lane-contiguous loads (whole cache lines per instruction) and is handed over through
  // LDS to the thread that owns each contiguous chunk.
  extern __shared__ float stage[];   // EPT * SEL_THREADS floats
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = e * SEL_THREADS + tid;
    stage[j] = sv[min(j, n_keys - 1)];
  }
  __syncthreads();
  float raw[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) raw[e] = stage[min(jb + e, EPT * SEL_THREADS - 1)];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    key[e] = e < live ? sort_key(raw[e]) : 0u;
    kmin = e < live ? min(kmin, key[e]) : kmin;
    kmax = e < live ? max(kmax, key[e]) : kmax;
  }
  kmin = wave_scan_min(kmin);
  kmax = wave_scan_max(kmax);
  if (lane == 63) {
    ext[0][wave] = kmin;
    ext[1][wave] = kmax;
  }
  __syncthreads();
  {  // lanes 0..15 hold the wavefronts' minima, lanes 16..31 their maxima: one row of 16 lanes each
    const uint32_t e0 = lane < 16 ? ext[0][lane] : 0xffffffffu, e1 = (lane >= 16 && lane < 32) ? ext[1][lane - 16] : 0u;
    uint32_t mn = e0, mx = e1;
    mn = min(mn, dpp_move<0x111, 0xf>(0xffffffffu, mn));
    mn = min(mn, dpp_move<0x112, 0xf>(0xffffffffu, mn));
    mn = min(mn, dpp_move<0x114, 0xf>(0xffffffffu, mn));
    mn = min(mn, dpp_move<0x118, 0xf>(0xffffffffu, mn));
    mx = max(mx, dpp_move<0x111, 0xf>(0u, mx));
    mx = max(mx, dpp_move<0x112, 0xf>(0u, mx));
    mx = max(mx, dpp_move<0x114, 0xf>(0u, mx));
    mx = max(mx, dpp_move<0x118, 0xf>(0u, mx));
    kmin = __builtin_amdgcn_readlane(mn, 15);
    kmax = __builtin_amdgcn_readlane(mx, 31);
  }
  // bits above `top` are common to all keys
  int top = 31 - __clz((int)(kmin ^ kmax));   // -1 when all keys are equal
  uint32_t prefix = top >= 31 ? 0u : (top < 0 ? kmax : (kmax >> (top + 1)) << (top + 1));
  uint32_t remaining = (uint32_t)h;
  while (top >= 0) {
    const int shift = max(top - 7, 0);
    const uint32_t dmask = (2u << (top - shift)) - 1u;           // digit = bits top .. shift
    const uint32_t cmask = top >= 31 ? 0u : ~((2u << top) - 1u); // bits above the digit decide candidacy
    // LDS atomics to one address are serialised, and digits made of exponent bits are shared by many lanes: lane
    // l counts in copy l % 16 of the histogram (copies 257 words apart, so one bin's copies sit in 16 banks).
    uint32_t* const my_hist = hist + (lane & (HCOPIES - 1)) * HSTRIDE;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const uint32_t u = key[e];
      if (e < live && (u & cmask) == prefix) atomicAdd(&my_hist[(u >> shift) & dmask], 1u);
    }
    __syncthreads();
    if (tid < 256) {   // add up the copies of one bin and clear them for the next pass
      uint32_t t = 0;
#pragma unroll
      for (int cp = 0; cp < HCOPIES; ++cp) {
        t += hist[cp * HSTRIDE + tid];
        hist[cp * HSTRIDE + tid] = 0;
      }
      total[tid] = t;
    }
    __syncthreads();
    if (tid < 64) {
      // lane t owns digits 255-4t .. 252-4t (descending); find where the count from the top reaches `remaining`
      uint32_t cnt[4], tot = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        cnt[r] = total[255 - 4 * tid - r];
        tot += cnt[r];
      }
      const uint32_t inc = wave_scan_add(tot);
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
    remaining = sel[1];
    top = shift - 1;
  }
  // prefix = key of the h-th largest score; `remaining` of the keys equal to it are kept (lowest indices)
  const uint32_t tau = prefix, need = remaining;
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    gt += (e < live) & (key[e] > tau);
    eq += (e < live) & (key[e] == tau);
  }
  block_scan2(gt, eq, scan_lds);
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (e < live) {
      const uint32_t u = key[e];
      if (u > tau) {
        out[gt + min(eq, need)] = jb + e;
        ++gt;
      } else if (u == tau) {
        if (eq < need) out[gt + eq] = jb + e;
        ++eq;
      }
    }
  }
}

// Any length: the scores are re-read from memory (L2) in every pass.
__global__ __launch_bounds__(SEL_THREADS) void select_kernel_stream(const float* __restrict__ s,
                                                                    int32_t* __restrict__ idx_out, int32_t N,
                                                                    int32_t w, int32_t h) {
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

// Score buffer of purekv_topk_select_static: device memory that exists from the moment the library is loaded
// on a GPU until the process ends, so that the call needs no workspace from its caller and no allocation.  Host
// code never uses the array's name as an address (in host code the name is only a handle for the symbol look-up):
// static_score_buffer() asks the runtime once per device for the array's device address and hands that out.
constexpr size_t kStaticScoreFloats = (size_t)1 << 20;   // 4 MiB
static __device__ __align__(256) float scratch[kStaticScoreFloats];

}  // namespace

size_t topk_static_capacity_floats() { return kStaticScoreFloats; }

int static_score_buffer(int device, float** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static float* ptrs[kMaxDevices] = {};
  if (device < 0 || device >= kMaxDevices) return PUREKV_EINVAL;
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[device] == nullptr) {
    int cur = -1;
    PUREKV_HIP_TRY(hipGetDevice(&cur));
    if (cur != device) return PUREKV_EINVAL;   // every GPU has its own copy of the array: look it up on its own device
    void* p = nullptr;
    PUREKV_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return PUREKV_EHIP;
    ptrs[device] = static_cast<float*>(p);
  }
  *out = ptrs[device];
  return PUREKV_OK;
}

size_t topk_ws_bytes(const purekv_plan& p, int32_t n_layers, int32_t w) {
  // scores, when the caller does not ask for them
  const int64_t n_keys = (int64_t)p.g.N - w;
  return n_keys > 0 ? (size_t)n_layers * p.g.Hkv * n_keys * sizeof(float) : 0;
}

static int launch_select(const purekv_plan& p, const float* scores, int32_t n_layers, int32_t w, int32_t h,
                         int32_t* idx_out, hipStream_t st);

int launch_vnorm2(const purekv_plan& p, const void* v, float* vnorm2, hipStream_t st) {
  const int rows_per_block = (256 / (p.g.d / 8)) * SCORE_UNROLL;
  const unsigned gx = (unsigned)((p.g.N + rows_per_block - 1) / rows_per_block);
  auto launch = [&](int kvh0, int count) {
    const dim3 grid(gx, (unsigned)count);
    if (p.g.d == 128)
      hipLaunchKernelGGL(vnorm2_kernel<128>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(v), p.g.kv_sh,
                         p.g.kv_st, vnorm2, p.g.N, kvh0);
    else
      hipLaunchKernelGGL(vnorm2_kernel<64>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(v), p.g.kv_sh,
                         p.g.kv_st, vnorm2, p.g.N, kvh0);
  };
  if (p.head_sel.empty()) {
    launch(0, p.g.Hkv);
  } else {   // a plan over a head subset: only the KV heads it reads
    for (int kvh = 0; kvh < p.g.Hkv; ++kvh) {
      bool any = false;
      for (int gq = 0; gq < p.g.G; ++gq) any |= p.head_sel[(size_t)kvh * p.g.G + gq] != 0;
      if (any) launch(kvh, 1);
    }
  }
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

int launch_topk_norms(const purekv_plan& p, const float* c, const float* vnorm2, int64_t vn_layer_stride,
                      int32_t n_layers, int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws, hipStream_t st) {
  const int32_t n_keys = p.g.N - w;
  const float* scores = c;
  if (n_keys > 0) {
    float* sbuf = s_out ? s_out : static_cast<float*>(ws);
    const dim3 grid((unsigned)((n_keys + 255) / 256), (unsigned)(n_layers * p.g.Hkv));
    hipLaunchKernelGGL(score_from_norms_kernel, grid, dim3(256), 0, st, c, vnorm2, vn_layer_stride, sbuf, p.g.N, n_keys,
                       p.g.Hkv);
    scores = sbuf;
  }
  return launch_select(p, scores, n_layers, w, h, idx_out, st);
}

int launch_topk(const purekv_plan& p, const float* c, const void* v, int64_t v_layer_stride, int32_t n_layers,
                int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws, hipStream_t st) {
  const int32_t n_keys = p.g.N - w;
  const float* scores = c;
  if (v != nullptr && n_keys > 0) {
    float* sbuf = s_out ? s_out : static_cast<float*>(ws);
    const int rows_per_block = (256 / (p.g.d / 8)) * SCORE_UNROLL;
    const dim3 grid((unsigned)((n_keys + rows_per_block - 1) / rows_per_block), (unsigned)(n_layers * p.g.Hkv));
    if (p.g.d == 128)
      hipLaunchKernelGGL(score_kernel<128>, grid, dim3(256), 0, st, c, static_cast<const uint16_t*>(v),
                         v_layer_stride, p.g.kv_sh, p.g.kv_st, sbuf, n_keys, p.g.Hkv);
    else
      hipLaunchKernelGGL(score_kernel<64>, grid, dim3(256), 0, st, c, static_cast<const uint16_t*>(v),
                         v_layer_stride, p.g.kv_sh, p.g.kv_st, sbuf, n_keys, p.g.Hkv);
    scores = sbuf;
  } else if (s_out != nullptr && n_keys > 0) {
    PUREKV_HIP_TRY(hipMemcpyAsync(s_out, c, (size_t)p.g.Hkv * n_keys * sizeof(float), hipMemcpyDeviceToDevice, st));
  }
  return launch_select(p, scores, n_layers, w, h, idx_out, st);
}

static int launch_select(const purekv_plan& p, const float* scores, int32_t n_layers, int32_t w, int32_t h,
                         int32_t* idx_out, hipStream_t st) {
  const int32_t n_keys = p.g.N - w;
  const dim3 sgrid((unsigned)(n_layers * p.g.Hkv)), sblock(SEL_THREADS);
  const int chunk = (n_keys + SEL_THREADS - 1) / SEL_THREADS;
  if (chunk <= 8) {
    hipLaunchKernelGGL(select_kernel<8>, sgrid, sblock, 8 * SEL_THREADS * sizeof(float), st, scores, idx_out, p.g.N, w,
                       h);
  } else if (chunk <= 16) {
    hipLaunchKernelGGL(select_kernel<16>, sgrid, sblock, 16 * SEL_THREADS * sizeof(float), st, scores, idx_out, p.g.N,
                       w, h);
  } else if (chunk <= 32) {
    constexpr int lds_bytes = 32 * SEL_THREADS * sizeof(float);   // 128 KB: above the default limit
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<32>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    PUREKV_HIP_TRY(attr);
    hipLaunchKernelGGL(select_kernel<32>, sgrid, sblock, lds_bytes, st, scores, idx_out, p.g.N, w, h);
  } else
    hipLaunchKernelGGL(select_kernel_stream, sgrid, sblock, 0, st, scores, idx_out, p.g.N, w, h);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
