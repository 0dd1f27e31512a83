// Spearman's rank correlation between two score arrays (Sec. 3.3, Eq. 5-7): the statistical check that the scores
// estimated from a low layer's column sums (Eq. 4) rank the keys like the scores of the layer's own attention (Eq. 6).
//
// rank(S): position of a score in its row's descending order, equal scores in index order (the tie rule of the top-h
// selection), so the ranks of a row are a permutation of 0 .. n-1 and a rank is a COUNT: r_j = #{k : s_k > s_j} +
// #{k < j : s_k = s_j}.  A thread owns one key j and counts over all k for both arrays at once; the scores it compares
// with are the same for every thread, so they come through the scalar cache and cost the vector ALU nothing: two
// vector instructions per comparison (compare, add with carry).  Keys before the workgroup's own 256 count with >=,
// keys after them with >, only the 256 in between need the index.  O(n^2) comparisons -- a diagnostic that runs once
// per model, exact in integers (a row of 32 768 scores: about a millisecond) -- and no workspace.
// The squared rank differences are added up as 64-bit integers (atomic adds of integers: any order gives the same
// bits); rho = 1 - 6 sum / (n (n^2 - 1)) is formed in fp64 from integers that fp64 holds exactly (n <= 2^17).
#include "common.h"

namespace purekv {
namespace {

typedef const float __attribute__((address_space(4))) * ConstFloats;

__global__ void rank_clear_kernel(unsigned long long* sum_d2, int n_rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_rows) sum_d2[i] = 0ull;
}

__global__ __launch_bounds__(256) void rank_diff_kernel(const float* __restrict__ s_hat, const float* __restrict__ s,
                                                        int n, unsigned long long* __restrict__ sum_d2) {
  const int row = blockIdx.y;
  const ConstFloats ch = (ConstFloats)(uintptr_t)(s_hat + (size_t)row * n);
  const ConstFloats cs = (ConstFloats)(uintptr_t)(s + (size_t)row * n);
  const int j0 = blockIdx.x * 256, j = j0 + threadIdx.x, jc = min(j, n - 1);
  const float vh = s_hat[(size_t)row * n + jc], vs = s[(size_t)row * n + jc];
  int rh = 0, rs = 0;   // ranks of key j in the two arrays
  const int k_own0 = j0, k_own1 = min(j0 + 256, n);
#pragma unroll 8
  for (int k = 0; k < k_own0; ++k) {        // keys with a lower index: they rank first on a tie
    rh += ch[k] >= vh;
    rs += cs[k] >= vs;
  }
  for (int k = k_own0; k < k_own1; ++k) {   // the workgroup's own keys: the index decides a tie
    const float xh = ch[k], xs = cs[k];
    rh += (xh > vh) | ((xh == vh) & (k < j));
    rs += (xs > vs) | ((xs == vs) & (k < j));
  }
#pragma unroll 8
  for (int k = k_own1; k < n; ++k) {        // keys with a higher index: they rank later on a tie
    rh += ch[k] > vh;
    rs += cs[k] > vs;
  }
  const long long d = j < n ? (long long)(rh - rs) : 0ll;
  unsigned long long d2 = (unsigned long long)(d * d);
  // sum over the wavefront, then one atomic per wavefront
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const unsigned lo = __shfl_xor((unsigned)(d2 & 0xFFFFFFFFull), o, 64), hi = __shfl_xor((unsigned)(d2 >> 32), o, 64);
    d2 += ((unsigned long long)hi << 32) | lo;
  }
  if ((threadIdx.x & 63) == 0 && d2 != 0ull)
    (void)__hip_atomic_fetch_add(sum_d2 + row, d2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void rank_rho_kernel(const unsigned long long* __restrict__ sum_d2, double* __restrict__ rho, int n_rows,
                                int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows) return;
  // n <= 2^17: n (n^2 - 1) < 2^51 and 6 sum <= 2 n^3 <= 2^52 are exact in fp64, so is their difference, and the
  // quotient is the correctly rounded value of the exact rational number
  const double denom = (double)n * ((double)n * (double)n - 1.0);
  rho[i] = (denom - 6.0 * (double)sum_d2[i]) / denom;
}

}  // namespace

int launch_spearman(const float* s_hat, const float* s, int32_t n_rows, int32_t n_keys, uint64_t* sum_d2, double* rho,
                    hipStream_t st) {
  auto* acc = reinterpret_cast<unsigned long long*>(sum_d2);
  const unsigned rb = (unsigned)((n_rows + 255) / 256);
  hipLaunchKernelGGL(rank_clear_kernel, dim3(rb), dim3(256), 0, st, acc, n_rows);
  hipLaunchKernelGGL(rank_diff_kernel, dim3((unsigned)((n_keys + 255) / 256), (unsigned)n_rows), dim3(256), 0, st, s_hat, s,
                     n_keys, acc);
  if (rho != nullptr) hipLaunchKernelGGL(rank_rho_kernel, dim3(rb), dim3(256), 0, st, acc, rho, n_rows, n_keys);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
