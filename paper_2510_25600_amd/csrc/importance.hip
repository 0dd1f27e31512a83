// Recent-window column sums C (Eq. 2), summed over the query heads of each KV group.
//
// A workgroup owns 128 non-recent keys of one KV head (32 per wavefront, held in registers as the
// MFMA A operand for the whole kernel) and walks every window row of every query head of the group in
// blocks of 32 rows.  The workgroup has two such sets of four wavefronts: set 0 takes the even blocks, set 1 the
// odd ones (two wavefronts per SIMD hide each other's LDS and MFMA latencies), and their sums are added at the
// end in a fixed order.  The four wavefronts of a set need the same query rows: a block of 32 rows (and its 32
// log-sum-exp values) goes from global memory straight into a ring of six LDS slots per set
// (global_load_lds: no staging registers), five blocks ahead of its use -- an iteration is a few hundred
// nanoseconds, an L2 hit about as long, so a shallow prefetch leaves every iteration waiting for its rows --
// with one barrier per block, and is read from LDS as the MFMA B operand.
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
  int64_t q_sh, kv_sh;    // element strides of the head axes of Q and K
  uint32_t q_st, kv_st;   // and of their token axes
  uint32_t pattern;
  float scale_log2;
};

// MASK = false: every window row sees every non-recent key (text rows, or the dense pattern).
template <int D, bool MASK>
__global__ __launch_bounds__(512) void importance_kernel(const ImportanceArgs a) {
  constexpr int KSTEPS = D / 16;
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int NLD = 32 * CPR / 256;   // 16-byte loads per thread and block of 32 query rows
  constexpr int NB = 6;                 // ring of query blocks per set: NB - 1 blocks are in flight or in use
  constexpr int LPB = NLD + 1;          // loads per thread and block (query pieces + one log-sum-exp word)
  constexpr int WAIT_BLOCK = ((NB - 2) * LPB & 15) | (((NB - 2) * LPB >> 4) << 14) | 0x0F70;   // vmcnt((NB-2) LPB)
  static_assert((NB - 2) * LPB < 64, "vmcnt has six bits");
  __shared__ __attribute__((aligned(16))) uint16_t Qs_all[2][NB][32 * D];   // [set][slot]
  __shared__ float lse_all[2][NB][4][64];                                   // [set][slot][wavefront]: own copy each
  __shared__ float part[4][16][64];                                         // set 1's sums, per wavefront
  const int set = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
  const int tid = threadIdx.x & 255, lane = tid & 63;                       // within the set
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint16_t (*Qs)[32 * D] = Qs_all[set];
  const int n = lane & 31, h = lane >> 5;
  const int kvh = blockIdx.y;
  const int n_keys = a.N - a.w;           // non-recent keys
  const int jw = blockIdx.x * 128 + wave * 32;  // first key of this wavefront
  const int row0 = a.N - a.w;             // first window row

  bf16x8 kf[KSTEPS];
  {
    const int j = min(jw + n, a.N - 1);
    const uint16_t* kr = a.k + (int64_t)kvh * a.kv_sh + (int64_t)j * a.kv_st;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) kf[s] = *reinterpret_cast<const bf16x8*>(kr + 16 * s + 8 * h);
  }

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
  // Starts the loads of the next block of this set into ring slot `slot`: LPB loads per thread, always (past the
  // end the last block is repeated and never used), so that the count of loads in flight is the same in every
  // iteration.  The set's blocks advance by two: (head, row block) are kept as counters.
  int is_g = 0, is_qb = set;   // block the next call loads
  auto normalise = [&](int& g, int& qb) {
    while (qb >= n_qblocks) qb -= n_qblocks, ++g;
    if (g >= a.G) g = a.G - 1, qb = n_qblocks - 1;
  };
  normalise(is_g, is_qb);
  auto issue_next = [&](int slot) {
    const size_t hrow = (size_t)(kvh * a.G + is_g) * a.N;
    const uint16_t* qhead = a.q + (int64_t)(kvh * a.G + is_g) * a.q_sh;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int r = min(row0 + is_qb * 32 + st_row[i], a.N - 1);
      load_to_lds_16(qhead, ((uint32_t)r * a.q_st + (uint32_t)st_col[i] * 8u) * 2u, &Qs[slot][(i * 256 + wave * 64) * 8]);
    }
    load_to_lds_4(a.lse + hrow, (uint32_t)min(row0 + is_qb * 32 + n, a.N - 1) * 4u, &lse_all[set][slot][wave][0]);
    is_qb += 2;
    normalise(is_g, is_qb);
  };

#pragma unroll 1
  for (int s = 0; s < NB - 1; ++s) issue_next(s);

  // Software pipeline inside the wavefront, one stage per block: the eight MFMAs of block `it`, whose query
  // fragments were read from LDS during the previous stage, with, between them, the exponentials of block it - 1
  // (two scores per MFMA), the LDS reads of block it + 1's fragments and the start of the loads of block
  // it + NB - 1.  The matrix pipe, the vector ALU and LDS overlap although the one barrier per stage keeps all
  // eight wavefronts in step.
  struct Pending {   // what the exponentials of a block need besides its scores
    float neg_lse2;  // minus the log-sum-exp of the lane's row in log2 units; -inf when the row does not exist
    int rowc;        // the lane's row (clamped) and what the mask needs of it
    int own0, prev;
    bool ok, video;
  };
  struct Block {     // a block ready for its MFMAs
    bf16x8 qf[KSTEPS];
    Pending pd;
  };
  const float scale_v = a.scale_log2;
  auto exp_step = [&](const floatx16& S, const Pending& pd, int i) {
    // Assembly, volatile: the three instructions of a score stay between the MFMAs where they are written (plain
    // arithmetic is collected ahead of or behind the products by the compiler, and the wavefronts of a SIMD then
    // take turns instead of overlapping).  The s_nop is the wait state a vector instruction needs before it reads
    // the result of a transcendental one.
    float p;
    if constexpr (!MASK) {
      asm volatile("v_fma_f32 %0, %2, %3, %4\n\tv_exp_f32 %0, %0\n\ts_nop 0\n\tv_add_f32 %1, %1, %0"
                   : "=&v"(p), "+v"(acc[i])
                   : "v"(S[i]), "v"(scale_v), "v"(pd.neg_lse2));
    } else {
      asm volatile("v_fma_f32 %0, %1, %2, %3\n\tv_exp_f32 %0, %0\n\ts_nop 0"
                   : "=v"(p)
                   : "v"(S[i]), "v"(scale_v), "v"(pd.neg_lse2));
    }
    if constexpr (MASK) {
      const int j = jw + 8 * (i >> 2) + 4 * h + (i & 3);
      bool ok = pd.ok && j <= pd.rowc;
      bool allowed = j < a.P;
      if (a.pattern & 1u) allowed |= (j >= pd.own0);
      if (a.pattern & 2u) allowed |= (j == pd.prev) | (j == pd.rowc);
      ok &= !pd.video || (allowed && j < a.Nv);
      acc[i] += ok ? p : 0.f;
    }
  };
  // Scores i and i + 1 together (the unmasked variant): the second score's instructions fill the latency of the
  // first one's exponential.
  auto exp_pair = [&](const floatx16& S, const Pending& pd, int i) {
    if constexpr (!MASK) {
      float p0, p1;
      asm volatile("v_fma_f32 %0, %4, %6, %7\n\tv_fma_f32 %1, %5, %6, %7\n\tv_exp_f32 %0, %0\n\tv_exp_f32 %1, %1\n\t"
                   "s_nop 0\n\tv_add_f32 %2, %2, %0\n\tv_add_f32 %3, %3, %1"
                   : "=&v"(p0), "=&v"(p1), "+v"(acc[i]), "+v"(acc[i + 1])
                   : "v"(S[i]), "v"(S[i + 1]), "v"(scale_v), "v"(pd.neg_lse2));
    } else {
      exp_step(S, pd, i);
      exp_step(S, pd, i + 1);
    }
  };
  int rd_slot = 0, rd_g = 0, rd_qb = set, rd_b = set;   // block the next read_pending / read_frag calls fetch
  normalise(rd_g, rd_qb);
  auto read_pending = [&](Pending& pd) {
    const int row = row0 + rd_qb * 32 + n;
    pd.ok = row < a.N && rd_b < n_blocks;   // an odd block count leaves set 1 one idle round
    pd.rowc = min(row, a.N - 1);
    const float lse_row = lse_all[set][rd_slot][wave][lane];   // read unconditionally: no branch, no early wait
    pd.neg_lse2 = pd.ok ? lse_row * -kLog2e : -INFINITY;
    if constexpr (MASK) {
      pd.video = pd.rowc < a.Nv;
      const int frame = pd.video ? pd.rowc / a.P : 0;
      pd.own0 = frame * a.P;
      pd.prev = frame >= 1 ? pd.rowc - a.P : -1;
    }
  };
  auto read_frag = [&](Block& blk, int s) {
    blk.qf[s] = *reinterpret_cast<const bf16x8*>(Qs[rd_slot] + kswz<D>(n, 2 * s + h));
  };
  auto advance_read = [&]() {
    rd_slot = rd_slot == NB - 1 ? 0 : rd_slot + 1;
    rd_b += 2;
    rd_qb += 2;
    normalise(rd_g, rd_qb);
  };
  // One stage: cur's MFMAs into Sn; Sp's exponentials; nxt <- fragments of the following block.
  constexpr int WAIT_NEXT = ((NB - 3) * LPB & 15) | (((NB - 3) * LPB >> 4) << 14) | 0x0F70;   // vmcnt((NB-3) LPB)
  // nxt still holds the pending data of the block before cur (the one Sp belongs to) on entry.
  auto stage = [&](const Block& cur, Block& nxt, floatx16& Sn, const floatx16& Sp, bool have_prev) {
    const Pending pp = nxt.pd;
    __builtin_amdgcn_s_waitcnt(WAIT_NEXT);   // this thread's pieces of the following block have landed
    __syncthreads();   // everybody's have; the slot of the previous block (read a stage ago) is free
#pragma unroll
    for (int i = 0; i < 16; ++i) Sn[i] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], cur.qf[s], Sn, 0, 0, 0);
      read_frag(nxt, s);
      if (s == 0) read_pending(nxt.pd);
      if (s == 1) issue_next(rd_slot < 2 ? rd_slot + NB - 2 : rd_slot - 2);   // the slot read a stage ago
      if (have_prev) {
#pragma unroll
        for (int i = s * (16 / KSTEPS); i < (s + 1) * (16 / KSTEPS); i += 2) exp_pair(Sp, pp, i);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    advance_read();
  };
  Block A, B;
  floatx16 S0, S1;
#pragma unroll
  for (int i = 0; i < 16; ++i) S1[i] = 0.f;   // passed to the first stage, which reads nothing of it
  // block 0 of this set: wait for it alone, read it
  __builtin_amdgcn_s_waitcnt(WAIT_BLOCK);
  __syncthreads();
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) read_frag(A, s);
  read_pending(A.pd);
  advance_read();
  stage(A, B, S0, S1, false);
  int it = 1;
  for (; it + 1 < n_iter; it += 2) {
    stage(B, A, S1, S0, true);
    stage(A, B, S0, S1, true);
  }
  if (it < n_iter) {
    stage(B, A, S1, S0, true);
#pragma unroll
    for (int i = 0; i < 16; i += 2) exp_pair(S1, B.pd, i);
  } else {
#pragma unroll
    for (int i = 0; i < 16; i += 2) exp_pair(S0, A.pd, i);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // the loads started past the end have landed before LDS is reused or freed

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
  a.q_sh = p.g.q_sh;
  a.kv_sh = p.g.kv_sh;
  a.q_st = (uint32_t)p.g.q_st;
  a.kv_st = (uint32_t)p.g.kv_st;
  a.w = w;
  a.pattern = p.g.pattern;
  a.scale_log2 = p.g.scale * kLog2e;
  const dim3 grid((unsigned)((n_keys + 127) / 128), (unsigned)p.g.Hkv), block(512);
  const bool mask = p.g.pattern != 0u && p.g.N - w < p.g.Nv;   // some window row is a video row under a sparse pattern
  if (p.g.d == 128) {
    if (mask) hipLaunchKernelGGL((importance_kernel<128, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((importance_kernel<128, false>), grid, block, 0, st, a);
  } else {
    if (mask) hipLaunchKernelGGL((importance_kernel<64, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((importance_kernel<64, false>), grid, block, 0, st, a);
  }
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
