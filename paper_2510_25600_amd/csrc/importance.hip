// Recent-window column sums C (Eq. 2), summed over the query heads of each KV group.
//
// A workgroup owns 128 non-recent keys of one KV head (32 per wavefront, held in registers as the
// MFMA A operand for the whole kernel) and walks every window row of every query head of the group in
// blocks of 32 rows.  The workgroup has two such sets of four wavefronts: set 0 takes the even blocks, set 1 the
// odd ones (two wavefronts per SIMD hide each other's LDS and MFMA latencies), and their sums are added at the
// end in a fixed order.  The four wavefronts of a set need the same query rows: a block of 32 rows is fetched
// once per set with whole-row loads (16 lanes x 16 bytes), parked in LDS (double-buffered, one barrier per
// block; the block after the next is in flight in registers) and read from there as the MFMA B operand.
// Scores are formed transposed (keys x queries) so a lane owns one query row of the
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
__global__ __launch_bounds__(512) void importance_kernel(const ImportanceArgs a) {
  constexpr int KSTEPS = D / 16;
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int NLD = 32 * CPR / 256;   // 16-byte loads per thread and block of 32 query rows
  __shared__ __attribute__((aligned(16))) uint16_t Qs_all[2][2][32 * D];   // [set][buffer]
  __shared__ float part[4][16][64];                                        // set 1's sums, per wavefront
  const int set = threadIdx.x >> 8;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;      // within the set
  uint16_t (*Qs)[32 * D] = Qs_all[set];
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
  const int n_blocks = a.G * n_qblocks;   // block b: query head b / n_qblocks of the group, rows 32 (b % n_qblocks) ..
  const int n_iter = (n_blocks + 1) / 2;  // set s handles blocks 2 it + s

  // staging map: thread -> NLD 16-byte pieces of a block (position p of the swizzled tile holds row r, slot u)
  int st_row[NLD], st_col[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) kunswz<D>(i * 256 + tid, st_row[i], st_col[i]);
  u32x4 qreg[NLD];
  float lse_reg = 0.f;   // this lane's row of the block in flight
  auto load_block = [&](int b) {
    const int bc = min(b, n_blocks - 1);   // past the end: re-read the last block (never used)
    const int g = bc / n_qblocks, qb = bc - g * n_qblocks;
    const size_t hrow = (size_t)(kvh * a.G + g) * a.N;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int r = min(row0 + qb * 32 + st_row[i], a.N - 1);
      qreg[i] = *reinterpret_cast<const u32x4*>(a.q + (hrow + r) * D + st_col[i] * 8);
    }
    lse_reg = a.lse[hrow + min(row0 + qb * 32 + n, a.N - 1)];
  };
  auto store_block = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) *reinterpret_cast<u32x4*>(&Qs[buf][(i * 256 + tid) * 8]) = qreg[i];
  };

  load_block(set);
  store_block(0);
  float lse_cur = lse_reg;
  load_block(2 + set);
  for (int it = 0; it < n_iter; ++it) {
    const int b = 2 * it + set;
    __syncthreads();   // block b is in Qs[it & 1]; nobody reads Qs[(it + 1) & 1] any more
    store_block((it + 1) & 1);
    const float lse_next = lse_reg;
    load_block(b + 4);

    const int bc = min(b, n_blocks - 1);
    const int g = bc / n_qblocks, qb = bc - g * n_qblocks;
    const int row = row0 + qb * 32 + n;
    const bool row_ok = row < a.N && b < n_blocks;   // an odd block count leaves set 1 one idle round
    const int rowc = min(row, a.N - 1);
    const uint16_t* Qb = Qs[it & 1];
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(Qb + kswz<D>(n, 2 * s + h));
    floatx16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], sacc, 0, 0, 0);
    const float lse2 = lse_cur * kLog2e;
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
    lse_cur = lse_next;
  }

  // set 0 adds set 1's sums (same wavefront index, same lane: same keys and query slots), then
  // sum over the 32 query slots (lanes with equal h hold the same keys).
  if (set == 1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) part[wave][i][lane] = acc[i];
  }
  __syncthreads();
  if (set == 1) return;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] += part[wave][i][lane];
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
  const dim3 grid((unsigned)((n_keys + 127) / 128), (unsigned)p.g.Hkv), block(512);
  if (p.g.d == 128)
    hipLaunchKernelGGL(importance_kernel<128>, grid, block, 0, st, a);
  else
    hipLaunchKernelGGL(importance_kernel<64>, grid, block, 0, st, a);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
