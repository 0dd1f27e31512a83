// Decode attention of one new token against the compact cache (the decode stage of the paper's
// inference-speed table), optionally fused with the append of that token's key and value.  Latency bound: a few MB of
// cache, one query row per head.  ONE launch does everything:
//   * the kept keys are cut into chunks of 256, one workgroup (8 wavefronts x 32 keys) per (chunk, KV head, block of
//     16 query heads of the group); every K/V row is read once and used for all heads of the block;
//   * scores S^T = K Q^T on the matrix pipe (v_mfma_f32_16x16x32_bf16: 16 keys x 16 heads per instruction; the K rows
//     and the query rows are the operands as they lie in memory, 16 bytes per lane), softmax over the keys in fp32
//     (a lane holds 4 keys of one head: in-lane reduction plus two cross-lane steps), probabilities rounded to bf16 and
//     O = P V with v_mfma_f32_16x16x16_bf16, whose A operand is the probabilities exactly as the score product left
//     them; V rows pass through LDS once and come back through the transposing read ds_read_b64_tr_b16;
//   * every load of a wavefront (query, 32 K rows, 32 V rows) is issued before the first is used;
//   * the wavefronts are merged through LDS, the chunks through a workspace in global memory: each workgroup
//     writes its (max, sum, unnormalised output), and the workgroup that arrives last at a per-(KV head, head block)
//     counter merges all chunks in a fixed order and writes the result.  Nobody waits for anybody: a workgroup that is
//     not the last simply ends.  The counters lead the caller's workspace and are zero between calls (the last
//     workgroup resets its counter): calls on different workspaces are independent of each other.
// With k_new/v_new given, row n_cached - 1 of the cache is taken from them instead of the cache and the workgroup
// that owns that key also stores it there (append and attention in one pass over the cache).
#include "common.h"

namespace purekv {
namespace {

constexpr int DEC_WAVES = 8;     // wavefronts per workgroup
constexpr int DEC_NT = 64 * DEC_WAVES;
constexpr int DEC_WAVE = 32;     // keys per wavefront (two 16-key tiles)
constexpr int DEC_CHUNK = DEC_WAVES * DEC_WAVE;   // keys per workgroup
constexpr int DEC_HB = 16;       // query heads per workgroup

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) shortx4* LdsShortx4;

inline int decode_splits(int n) { return n <= 0 ? 1 : (n + DEC_CHUNK - 1) / DEC_CHUNK; }

struct DecodeArgs {
  const uint16_t* q;
  const uint16_t* k_new;   // [Hkv, D] or null
  const uint16_t* v_new;
  uint16_t* kc;
  uint16_t* vc;
  uint16_t* out;
  float* ws_o;        // [n_splits, Hq, D] unnormalised partial outputs
  float* ws_ml;       // [n_splits, Hq, 2] running maximum (log2 domain) and sum
  int32_t* counters;  // [Hkv * n_head_blocks], zero on entry and on exit
  int32_t Hq, G, n_cached, cap, n_splits;
  float scale_log2;
};

// Device-scope (agent) relaxed accesses: coherent across the XCDs' L2s without any cache maintenance.
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(float* p, float x) {
  __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
__global__ __launch_bounds__(DEC_NT) void decode_kernel(const DecodeArgs a) {
  constexpr int KS = D / 32;            // k-steps of the score product
  constexpr int NC = D / 16;            // 16-column blocks of the output
  constexpr int CPR = D / 8;            // 16-byte pieces per row
  constexpr int NV = DEC_WAVE * CPR / 64;   // V pieces per lane
  constexpr int VROW = D * 2 + 32;      // bytes per V row in LDS (padded: consecutive rows start 8 banks apart)
  static_assert(DEC_WAVE * VROW >= DEC_HB * D * 4, "a wavefront's output block reuses its V rows' LDS");
  __shared__ __attribute__((aligned(16))) uint8_t smem[DEC_WAVES][DEC_WAVE * VROW];
  __shared__ float lds_ml[DEC_WAVES][DEC_HB][2];
  __shared__ float lds_red[DEC_NT / 16][DEC_HB];
  __shared__ float lds_pass[2][DEC_HB];
  __shared__ int lds_last;
  constexpr int EPT = DEC_HB * D / DEC_NT;   // output elements per thread in the merges

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, kg = lane >> 4;
  const int split = blockIdx.x, kvh = blockIdx.y, g0 = blockIdx.z * DEC_HB;
  const int ng = min(DEC_HB, a.G - g0);
  const int key0 = split * DEC_CHUNK + wave * DEC_WAVE;
  const int last = a.n_cached - 1;
  const int j_new = a.k_new != nullptr ? last : -1;   // the key that comes from k_new / v_new

  // ---- every load of this wavefront, before any use ----
  bf16x8 qf[KS], kf[2][KS];
  {
    const uint16_t* qr = a.q + (size_t)(kvh * a.G + g0 + min(n, ng - 1)) * D + 8 * kg;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qr + 32 * s);
  }
  const size_t head_base = (size_t)kvh * a.cap * D;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = min(key0 + 16 * t + n, last);   // rows past the end repeat the last key (masked below)
    const uint16_t* kr = (j == j_new ? a.k_new + (size_t)kvh * D : a.kc + head_base + (size_t)j * D) + 8 * kg;
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[t][s] = *reinterpret_cast<const bf16x8*>(kr + 32 * s);
  }
  u32x4 vreg[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int p = i * 64 + lane, r = p / CPR, c = p % CPR;
    const int j = min(key0 + r, last);
    const uint16_t* vr = j == j_new ? a.v_new + (size_t)kvh * D : a.vc + head_base + (size_t)j * D;
    vreg[i] = *reinterpret_cast<const u32x4*>(vr + c * 8);
  }

  // ---- append: the wavefront that owns key j_new stores it (head block 0 only) ----
  if (j_new >= 0 && blockIdx.z == 0 && j_new >= key0 && j_new < key0 + DEC_WAVE) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      if (key0 + 16 * t + n == j_new) {
        uint16_t* kw = a.kc + head_base + (size_t)j_new * D + 8 * kg;
#pragma unroll
        for (int s = 0; s < KS; ++s) *reinterpret_cast<bf16x8*>(kw + 32 * s) = kf[t][s];
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int p = i * 64 + lane, r = p / CPR, c = p % CPR;
      if (key0 + r == j_new) *reinterpret_cast<u32x4*>(a.vc + head_base + (size_t)j_new * D + c * 8) = vreg[i];
    }
  }

  // ---- V rows to LDS ----
  uint8_t* vs = smem[wave];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int p = i * 64 + lane, r = p / CPR, c = p % CPR;
    *reinterpret_cast<u32x4*>(vs + r * VROW + c * 16) = vreg[i];
  }

  // ---- scores: lane (n, kg) holds keys 16 t + 4 kg + i of head n ----
  const int n_valid = a.n_cached - key0;   // keys of this wavefront that exist (may be <= 0 or > 32)
  float sc[2][4];
  float m = -INFINITY;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    floatx4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][s], qf[s], sacc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sc[t][i] = (16 * t + 4 * kg + i < n_valid) ? sacc[i] * a.scale_log2 : -INFINITY;
      m = fmaxf(m, sc[t][i]);
    }
  }
  m = fmaxf(m, __shfl_xor(m, 16, 64));
  m = fmaxf(m, __shfl_xor(m, 32, 64));
  const float mu = (m == -INFINITY) ? 0.f : m;
  float l = 0.f;
  shortx4 pa[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint32_t w0 = pack_bf16(__builtin_amdgcn_exp2f(sc[t][0] - mu), __builtin_amdgcn_exp2f(sc[t][1] - mu));
    const uint32_t w1 = pack_bf16(__builtin_amdgcn_exp2f(sc[t][2] - mu), __builtin_amdgcn_exp2f(sc[t][3] - mu));
    l += (bf16_lo(w0) + bf16_hi(w0)) + (bf16_lo(w1) + bf16_hi(w1));   // the sum of what is multiplied with V
    pa[t] = __builtin_bit_cast(shortx4, u32x2{w0, w1});
  }
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);

  __syncthreads();   // V rows are in LDS

  // ---- O = P V: lane (n, kg) receives heads 4 kg + i, column 16 c + n ----
  // transposing read: in a 16-lane group lane s gives the address of row s / 4, columns 4 (s % 4) .. + 3 and lane j
  // receives column j of those four rows: the B operand (keys 4 kg .. + 3 of column n) of the 16x16x16 product.
  floatx4 o[NC];
  {
    const uint8_t* vb = vs + (4 * kg + (n >> 2)) * VROW + 8 * (n & 3);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      o[c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const shortx4 vfrag = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsShortx4)(vb + 16 * t * VROW + 32 * c));
        o[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa[t], vfrag, o[c], 0, 0, 0);
      }
    }
  }
  // ---- the wavefront's block [16 heads][D] fp32 replaces its V rows in LDS ----
  float* ow = reinterpret_cast<float*>(vs);
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int i = 0; i < 4; ++i) ow[(4 * kg + i) * D + 16 * c + n] = o[c][i];
  if (kg == 0) {
    lds_ml[wave][n][0] = m;
    lds_ml[wave][n][1] = l;
  }
  __syncthreads();

  // ---- merge the wavefronts; thread -> elements e = tid + DEC_NT k: head e / D, column e % D ----
  const bool single = a.n_splits == 1;
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int e = tid + DEC_NT * k;
    if (e >= ng * D) break;
    const int g = e / D, dd = e % D;
    float mn = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < DEC_WAVES; ++wv) mn = fmaxf(mn, lds_ml[wv][g][0]);
    const float mref = (mn == -INFINITY) ? 0.f : mn;
    float acc = 0.f, ls = 0.f;
#pragma unroll
    for (int wv = 0; wv < DEC_WAVES; ++wv) {
      const float f = __builtin_amdgcn_exp2f(lds_ml[wv][g][0] - mref);
      acc += reinterpret_cast<const float*>(smem[wv])[g * D + dd] * f;
      ls += lds_ml[wv][g][1] * f;
    }
    const int hq = kvh * a.G + g0 + g;
    if (single) {
      a.out[(size_t)hq * D + dd] = (uint16_t)f32_to_bf16(acc / ls);
    } else {
      st_agent(a.ws_o + ((size_t)split * a.Hq + hq) * D + dd, acc);
      if (dd == 0) {
        st_agent(a.ws_ml + ((size_t)split * a.Hq + hq) * 2, mn);
        st_agent(a.ws_ml + ((size_t)split * a.Hq + hq) * 2 + 1, ls);
      }
    }
  }
  if (single) return;

  // ---- the workgroup that arrives last merges the chunks ----
  // Partial results travel through device-scope stores and loads only (they pass through the L2 of the XCD that
  // issues them, so the eight L2s need no write-back or invalidation); the arrival is counted once every store of
  // the workgroup has completed.
  int32_t* counter = a.counters + kvh * gridDim.z + blockIdx.z;
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this thread's stores have completed
  __syncthreads();
  if (tid == 0) lds_last = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.n_splits - 1;
  __syncthreads();
  if (!lds_last) return;

  // Chunks are merged in passes of up to SB; within a pass: (max, sum) of all chunks -> LDS, maximum and weights
  // 2^(m_s - max) per head, then the weighted sum of the partial outputs, U chunks in flight per thread and element.
  constexpr int SB = 128, U = 16;
  float* pm = reinterpret_cast<float*>(&smem[0][0]);   // [SB][16] maxima, then weights
  float* pl = pm + SB * DEC_HB;                        // [SB][16] sums
  static_assert(2 * SB * DEC_HB * 4 <= DEC_WAVES * DEC_WAVE * VROW, "merge tables fit the V area");
  constexpr int RP = DEC_NT / 16;
  const int rg = tid & 15, rpart = tid >> 4;           // reductions: head rg, every RP-th chunk from rpart
  int eg[EPT];
  bool ev[EPT];
  const float* eo[EPT];
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int e = min(tid + DEC_NT * k, ng * D - 1);   // elements past the end repeat the last one (not written)
    ev[k] = tid + DEC_NT * k < ng * D;
    eg[k] = e / D;
    eo[k] = a.ws_o + (size_t)(kvh * a.G + g0 + eg[k]) * D + e % D;
  }
  const size_t chunk_stride = (size_t)a.Hq * D;
  float run_m[EPT], run_l[EPT], acc[EPT];
#pragma unroll
  for (int k = 0; k < EPT; ++k) run_m[k] = -INFINITY, run_l[k] = 0.f, acc[k] = 0.f;

  for (int s0 = 0; s0 < a.n_splits; s0 += SB) {
    const int nsb = min(SB, a.n_splits - s0);
    float ov[U][EPT];
    auto load_batch = [&](int b0) {   // only what exists is requested
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < EPT; ++k)
          ov[u][k] = (b0 + u < nsb && ev[k]) ? ld_agent(eo[k] + (size_t)(s0 + b0 + u) * chunk_stride) : 0.f;
    };
    load_batch(0);
    constexpr int PPT = SB * DEC_HB / DEC_NT;   // (chunk, head) pairs per thread
    float mreg[PPT], lreg[PPT];
#pragma unroll
    for (int r = 0; r < PPT; ++r) {
      const int i = tid + DEC_NT * r, sl = min(i >> 4, nsb - 1), g = i & 15;
      const size_t row = (size_t)(s0 + sl) * a.Hq + kvh * a.G + g0 + min(g, ng - 1);
      const bool need = i < nsb * DEC_HB;
      mreg[r] = need ? ld_agent(a.ws_ml + row * 2) : 0.f;
      lreg[r] = need ? ld_agent(a.ws_ml + row * 2 + 1) : 0.f;
    }
    __syncthreads();   // the tables of the previous pass (or the wavefronts' blocks) are no longer read
#pragma unroll
    for (int r = 0; r < PPT; ++r) {
      const int i = tid + DEC_NT * r;
      if (i < nsb * DEC_HB) pm[i] = mreg[r], pl[i] = lreg[r];
    }
    __syncthreads();
    {
      float mx = -INFINITY;
      for (int sl = rpart; sl < nsb; sl += RP) mx = fmaxf(mx, pm[sl * DEC_HB + rg]);
      lds_red[rpart][rg] = mx;
    }
    __syncthreads();
    float pmax = -INFINITY;   // this pass' maximum of head rg (every chunk holds at least one key: finite)
#pragma unroll
    for (int p = 0; p < RP; ++p) pmax = fmaxf(pmax, lds_red[p][rg]);
    __syncthreads();
    {
      float sum = 0.f;
      for (int sl = rpart; sl < nsb; sl += RP) {
        const float f = __builtin_amdgcn_exp2f(pm[sl * DEC_HB + rg] - pmax);
        pm[sl * DEC_HB + rg] = f;
        sum += pl[sl * DEC_HB + rg] * f;
      }
      lds_red[rpart][rg] = sum;
      if (rpart == 0) lds_pass[0][rg] = pmax;
    }
    __syncthreads();
    if (rpart == 0) {
      float sum = 0.f;
#pragma unroll
      for (int p = 0; p < RP; ++p) sum += lds_red[p][rg];
      lds_pass[1][rg] = sum;
    }
    __syncthreads();
    // fold the pass into the running state: its outputs are relative to its own maximum
    float wpass[EPT];
#pragma unroll
    for (int k = 0; k < EPT; ++k) {
      const float pmk = lds_pass[0][eg[k]], plk = lds_pass[1][eg[k]];
      const float mnew = fmaxf(run_m[k], pmk);
      const float fo = __builtin_amdgcn_exp2f(run_m[k] - mnew);   // first pass: 2^(-inf) = 0
      wpass[k] = __builtin_amdgcn_exp2f(pmk - mnew);
      acc[k] *= fo;
      run_l[k] = run_l[k] * fo + plk * wpass[k];
      run_m[k] = mnew;
    }
    for (int b0 = 0; b0 < nsb; b0 += U) {
      if (b0 > 0) load_batch(b0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (b0 + u < nsb) {
#pragma unroll
          for (int k = 0; k < EPT; ++k) acc[k] += ov[u][k] * (pm[(b0 + u) * DEC_HB + eg[k]] * wpass[k]);
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int e = tid + DEC_NT * k;
    if (e < ng * D) a.out[(size_t)(kvh * a.G + g0) * D + e] = (uint16_t)f32_to_bf16(acc[k] / run_l[k]);
  }
  if (tid == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
}

}  // namespace

// Workspace: [arrival counters, padded to 256 bytes][partial outputs][their (max, sum)].
static int decode_counter_count(const purekv_plan& p) { return p.g.Hkv * ((p.g.G + DEC_HB - 1) / DEC_HB); }
static size_t decode_counter_bytes(const purekv_plan& p) {
  return ((size_t)decode_counter_count(p) * sizeof(int32_t) + 255) / 256 * 256;
}

size_t decode_ws_bytes(const purekv_plan& p, int32_t cap) {
  return decode_counter_bytes(p) + (size_t)decode_splits(cap) * p.g.Hq * (p.g.d + 2) * sizeof(float);
}

namespace {
__global__ void clear_decode_counters_kernel(int32_t* c, int n) {   // a kernel, not a memset: callers may be capturing
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) c[i] = 0;
}
}  // namespace

int launch_decode_ws_init(const purekv_plan& p, void* ws, hipStream_t st) {
  const int n = decode_counter_count(p);
  hipLaunchKernelGGL(clear_decode_counters_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     static_cast<int32_t*>(ws), n);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

int launch_decode(const purekv_plan& p, const void* q_new, const void* k_new, const void* v_new, void* kc, void* vc,
                  int32_t n_cached, int32_t cap, void* out, void* ws, hipStream_t st) {
  DecodeArgs a;
  a.q = static_cast<const uint16_t*>(q_new);
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.kc = static_cast<uint16_t*>(kc);
  a.vc = static_cast<uint16_t*>(vc);
  a.out = static_cast<uint16_t*>(out);
  a.n_splits = decode_splits(n_cached);
  a.counters = static_cast<int32_t*>(ws);
  a.ws_o = reinterpret_cast<float*>(static_cast<char*>(ws) + decode_counter_bytes(p));
  a.ws_ml = a.ws_o + (size_t)decode_splits(cap) * p.g.Hq * p.g.d;
  a.Hq = p.g.Hq;
  a.G = p.g.G;
  a.n_cached = n_cached;
  a.cap = cap;
  a.scale_log2 = p.g.scale * kLog2e;
  const dim3 grid((unsigned)a.n_splits, (unsigned)p.g.Hkv, (unsigned)((p.g.G + DEC_HB - 1) / DEC_HB));
  if (p.g.d == 128)
    hipLaunchKernelGGL(decode_kernel<128>, grid, dim3(DEC_NT), 0, st, a);
  else
    hipLaunchKernelGGL(decode_kernel<64>, grid, dim3(DEC_NT), 0, st, a);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
