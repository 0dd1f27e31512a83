// ST-SpAttn / dense causal prefill attention for gfx950 (Sec. 3.2; Eq. 1 for the dense pattern).
//
// A persistent workgroup of 8 wavefronts walks a host-planned stream of 64-key tiles.  Each wavefront owns 32
// query rows of one head.  Scores are formed transposed, S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that a
// lane holds 16 keys of ONE query: the softmax row maximum is an in-lane reduction plus one exchange between
// the two halves of the wavefront, and the probabilities leave the accumulator already in the register layout
// that the second product O^T = V^T P^T takes as its B operand.  K tiles sit in LDS row-major, V tiles
// transposed (the contraction index of the second product is the key), both XOR-swizzled in 16-byte units so
// the 128-bit operand reads are conflict-free.  The attention matrix never exists.
//
// The softmax denominator is the sum of the bf16-ROUNDED probabilities, i.e. exactly the weights the second
// product applies, so each output row is a true convex combination of V rows.  It comes from the matrix pipe
// as well: one more MFMA per 16 keys multiplies the probabilities by an all-ones operand.
//
// Two-phase schedule.  Wavefronts w and w+4 share a SIMD.  A step of a wavefront is a matrix phase (second
// product of the previous tile, score product of this tile) and a vector phase (mask, maximum, exponentials,
// K/V staging), separated by workgroup barriers.  Wavefronts 4-7 run one phase behind wavefronts 0-3, so on
// every SIMD one wavefront is in its matrix phase while the other is in its vector phase and the two pipes
// overlap without relying on instruction scheduling inside a wavefront.
//
// K/V tiles travel HBM -> registers (bounds-checked buffer loads: rows past the end read as zero, a tile index
// past the list reads nothing) -> LDS, through rings of three K and three V buffers: while tile t is multiplied,
// wavefronts 0-3 write their share of tile t+1 and wavefronts 4-7 (one phase later) theirs of tile t+2.
#include "common.h"

namespace purekv {
namespace {

constexpr int BQ = PUREKV_BQ;
constexpr int BK = PUREKV_BK;
constexpr float kRescaleGap = 8.0f;

struct PrefillArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* out;
  float* lse;
  float* ws_o;    // [n_slots, Hq, BQ, D] normalised partial outputs
  float* ws_lse;  // [n_slots, Hq, BQ, 2] log2-domain log-sum-exp of the partial: {merge weight, exact}
  const StreamEntry* stream;
  const Unit* units;
  const int32_t* queue_begin;
  const MergeItem* merges;
  int32_t N, Nv, P, Hq, Hkv;
  uint32_t pattern;
  float scale_log2;  // softmax scale * log2(e)
#ifdef PUREKV_PHASE_TRACE
  unsigned long long* trace;  // [grid, 2, 64, 8] cycle stamps of wavefronts 0 and 4, development builds only
#endif
};

#ifdef PUREKV_PHASE_TRACE
#define PHASE_MARK(i)                                                                                  \
  if ((threadIdx.x & 255) == 0 && t - t_begin < 64)                                                    \
  a.trace[(((size_t)blockIdx.x * 2 + (threadIdx.x >> 8)) * 64 + (t - t_begin)) * 8 + (i)] = __builtin_readcyclecounter()
#else
#define PHASE_MARK(i)
#endif

// Element offset of 16-byte slot `u` of row `r` in a row-major bf16 LDS tile with ROW elements per row.
// The slot index is XOR-ed with the row so that the 16 lanes the LDS serves together (rows that differ
// in their low four bits) fall into 16 different 16-byte slots of a 256-byte bank period.
template <int ROW>
__device__ __forceinline__ int swz(int r, int u) {
  if constexpr (ROW == 128) {
    return r * 128 + ((u ^ (r & 15)) * 8);
  } else {  // 64 elements = 128 bytes: two rows share one 256-byte period
    return (r >> 1) * 128 + ((((r & 1) * 8 + u) ^ ((r >> 1) & 15)) * 8);
  }
}

// Raw buffer descriptor over `bytes` bytes at `p`: loads past the end return zero instead of faulting.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buffer_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0));
}

// ST  = false: dense causal pattern only (no frame arithmetic); true: any pattern.
// LSE = true : also keeps the exact fp32 row sum for the log-sum-exp output.
//
// Persistent kernel: workgroup q walks stream[queue_begin[q] .. queue_begin[q+1]).  Every stream entry is one
// key tile: all wavefronts stage it, the wavefronts whose `need` bit is set multiply it.  Units (query tile
// slice x head) follow each other in the stream without draining the K/V pipeline.
template <int D, bool ST, bool LSE>
__global__ __launch_bounds__(512, 1) void prefill_kernel(const PrefillArgs a) {
  constexpr int KSTEPS = D / 16;        // MFMA k-steps of the score product
  constexpr int DBLK = D / 32;          // 32-row blocks of O^T
  constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
  constexpr int KCH = BK * CPR / 512;   // K chunks staged per thread
  constexpr int NBUF = 3;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* const Ks_base = smem;                     // NBUF x [BK][D]
  uint16_t* const Vt_base = smem + NBUF * BK * D;     // NBUF x [D][BK]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;            // 0: leading wavefronts, 1: the ones that run one phase behind
  const int n = lane & 31, h = lane >> 5;
  const int t_begin = a.queue_begin[blockIdx.x], t_end = a.queue_begin[blockIdx.x + 1];
  if (t_begin >= t_end) return;

  const uint32_t kv_bytes = (uint32_t)a.Hkv * (uint32_t)a.N * D * 2u;
  const __amdgpu_buffer_rsrc_t krs = make_rsrc(a.k, kv_bytes), vrs = make_rsrc(a.v, kv_bytes);

  // ---- staging maps (per-thread constants) ----
  // K: chunk id = tid + 512 r -> (row id / CPR, 16-byte chunk id % CPR): a row is read by CPR neighbouring lanes.
  // V: the first 16*CPR threads (all in wavefronts 0-3) own 4 consecutive keys (quad vg) x 8 consecutive d
  //    (chunk vc) each; 4 neighbouring lanes read 64 contiguous bytes of one row.  Quad vg holds keys
  //    16*grp + 8*aa + 4*hh + 0..3; the MFMA k-order wants, per 16 keys, [hh=0: aa=0, aa=1 | hh=1: aa=0, aa=1],
  //    i.e. 16-byte unit 2*grp + hh, 8-byte half aa.
  const int vcl = tid & 3, vg = (tid >> 2) & 15, vc = (tid >> 6) * 4 + vcl;
  const bool v_active = vc < CPR;
  const int v_unit = 2 * (vg >> 2) + (vg & 1), v_half = (vg >> 1) & 1;
  uint32_t k_goff[KCH], v_goff[4];
  int k_loff[KCH];
#pragma unroll
  for (int r = 0; r < KCH; ++r) {
    const int id = tid + 512 * r, rk = id / CPR, cc = id % CPR;
    k_goff[r] = (uint32_t)(rk * D + cc * 8) * 2u;
    k_loff[r] = swz<D>(rk, cc);
  }
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
    v_goff[jj] = v_active ? (uint32_t)((4 * vg + jj) * D + vc * 8) * 2u : kv_bytes;  // idle threads read nothing
  u32x4 kreg[KCH], vreg[4];

  // An offset at or past the end of the tensor reads zeros and touches no memory.
  auto load_tile = [&](uint32_t base) {
#pragma unroll
    for (int r = 0; r < KCH; ++r) kreg[r] = buffer_load16(krs, base + k_goff[r]);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) vreg[jj] = buffer_load16(vrs, base + v_goff[jj]);
  };
  auto store_tile = [&](int buf) {
    uint16_t* Ks = Ks_base + buf * (BK * D);
    uint16_t* Vt = Vt_base + buf * (D * BK);
#pragma unroll
    for (int r = 0; r < KCH; ++r) *reinterpret_cast<u32x4*>(Ks + k_loff[r]) = kreg[r];
    if (v_active) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int dd = 8 * vc + e;
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;  // high / low halves of two dwords
        u32x2 w;
        w[0] = __builtin_amdgcn_perm(vreg[1][e >> 1], vreg[0][e >> 1], sel);
        w[1] = __builtin_amdgcn_perm(vreg[3][e >> 1], vreg[2][e >> 1], sel);
        *reinterpret_cast<u32x2*>(Vt + swz<BK>(dd, v_unit) + v_half * 4) = w;
      }
    }
  };
  // Stream entries are wave-uniform and read-only: fetch them through the scalar cache (constant address space),
  // one step before they are used, so that no phase waits for a global load.
  static_assert(sizeof(StreamEntry) == 16, "a stream entry is read as four dwords");
  typedef const u32x4 __attribute__((address_space(4))) * ConstStream;
  const ConstStream stream_c = (ConstStream)(uintptr_t)a.stream;
  auto stream_entry = [&](int t) {
    const u32x4 w = stream_c[t];
    StreamEntry e;
    e.kv_off = w[0];
    e.masks = w[1];
    e.unit = (int32_t)w[2];
    e.last = (int32_t)w[3];
    return e;
  };
  auto tile_off = [&](int t) {
    const uint32_t off = stream_c[min(t, t_end - 1)][0];
    return t < t_end ? off : kv_bytes;
  };
  auto next_buf = [](int b) { return b == NBUF - 1 ? 0 : b + 1; };
  // Barrier between phases; the scheduling fences keep the matrix work of a phase on its side.
  auto phase_barrier = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- per-unit state ----
  int hq = 0, row = 0, rowc = 0, a_i = 0, lo_i = 0, prev_j = -1, self_j = -1;
  int u_nsplits = 1, u_slot = -1;
  bf16x8 qf[KSTEPS];
  // m: reference maximum (log2 units); lacc: every element holds the sum of the bf16-rounded probabilities of
  // query n (accumulated by the matrix pipe against an all-ones operand); lx: exact fp32 sum (LSE only).
  float m = -INFINITY, lx = 0.f;
  floatx16 oacc[DBLK], lacc;
  bf16x8 ones8;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones8[i] = (__bf16)1.0f;

  auto begin_unit = [&](int uid) {
    const Unit u = a.units[uid];
    hq = u.head;
    u_nsplits = u.n_splits;
    u_slot = u.slot;
    row = u.qtile * BQ + wave * 32 + n;
    rowc = min(row, a.N - 1);
    // allowed keys of this lane's row: j <= rowc and (j <= a_i or j >= lo_i or j == prev_j or j == self_j)
    const bool sparse_row = ST && a.pattern != 0u && rowc < a.Nv;
    const int frame = sparse_row ? rowc / a.P : 0;
    a_i = sparse_row ? min(rowc, a.P - 1) : rowc;
    lo_i = sparse_row ? ((a.pattern & 1u) ? frame * a.P : rowc + 1) : 0;
    prev_j = (sparse_row && (a.pattern & 2u) && frame >= 1) ? rowc - a.P : -1;
    self_j = (sparse_row && (a.pattern & 2u)) ? rowc : -1;
    const uint16_t* qrow = a.q + ((size_t)hq * a.N + rowc) * D;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qrow + 16 * s + 8 * h);
    m = -INFINITY;
    lx = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) lacc[i] = 0.f;
#pragma unroll
    for (int b = 0; b < DBLK; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[b][i] = 0.f;
  };

  // Normalise and write this wavefront's 32 rows of the unit that just finished.
  auto finish_unit = [&]() {
    const float l_tot = lacc[0];
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse2 = m + __builtin_amdgcn_logf(l_tot);  // log2 domain; -inf when the slice saw no key
    const float lse2x = LSE ? m + __builtin_amdgcn_logf(lx + other_half(lx)) : lse2;
    if (u_nsplits == 1) {
      if (row < a.N) {
        uint16_t* orow = a.out + ((size_t)hq * a.N + row) * D;
#pragma unroll
        for (int b = 0; b < DBLK; ++b)
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            u32x2 w;
            w[0] = pack_bf16(oacc[b][4 * g4 + 0] * inv, oacc[b][4 * g4 + 1] * inv);
            w[1] = pack_bf16(oacc[b][4 * g4 + 2] * inv, oacc[b][4 * g4 + 3] * inv);
            *reinterpret_cast<u32x2*>(orow + 32 * b + 8 * g4 + 4 * h) = w;
          }
        if (LSE && h == 0) a.lse[(size_t)hq * a.N + row] = lse2x * kLn2;
      }
    } else {
      const size_t prow = ((size_t)u_slot * a.Hq + hq) * BQ + wave * 32 + n;
      float* orow = a.ws_o + prow * D;
#pragma unroll
      for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          floatx4 w;
#pragma unroll
          for (int r = 0; r < 4; ++r) w[r] = oacc[b][4 * g4 + r] * inv;
          *reinterpret_cast<floatx4*>(orow + 32 * b + 8 * g4 + 4 * h) = w;
        }
      if (h == 0) {
        a.ws_lse[2 * prow] = lse2;
        a.ws_lse[2 * prow + 1] = lse2x;
      }
    }
  };

  // Operand fragments are read from LDS two MFMAs ahead of their use (ring of three registers); the scheduling
  // fences keep that order, so each wait covers only the oldest read.
  // S^T = K Q^T: two 32-key blocks x 32 queries
  auto qk_tile = [&](int buf, floatx16 (&sacc)[2]) {
    const uint16_t* Ks = Ks_base + buf * (BK * D);
    constexpr int NF = 2 * KSTEPS;
    auto rd = [&](int i) {   // fragment i: k-step i/2 of key block i%2
      return *reinterpret_cast<const bf16x8*>(Ks + swz<D>(32 * (i & 1) + n, 2 * (i >> 1) + h));
    };
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
    bf16x8 f[3];
    f[0] = rd(0);
    f[1] = rd(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      if (i + 2 < NF) f[(i + 2) % 3] = rd(i + 2);
      sacc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % 3], qf[i >> 1], sacc[i & 1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // O^T += V^T P^T, row sums += 1 P^T
  auto pv_tile = [&](int buf, const bf16x8 (&pf)[4]) {
    const uint16_t* Vt = Vt_base + buf * (D * BK);
    constexpr int NF = 4 * DBLK;
    auto rd = [&](int i) {   // fragment i: 16-key step i%4 of output block i/4
      return *reinterpret_cast<const bf16x8*>(Vt + swz<BK>(32 * (i >> 2) + n, 2 * (i & 3) + h));
    };
    bf16x8 f[3];
    f[0] = rd(0);
    f[1] = rd(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) lacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones8, pf[ks], lacc, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      if (i + 2 < NF) f[(i + 2) % 3] = rd(i + 2);
      oacc[i >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % 3], pf[i & 3], oacc[i >> 2], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Mask, running maximum, exponentials: scores of one tile -> bf16 B-operand fragments; pf[ks] covers keys
  // 16*ks .. 16*ks+15 of the tile.
  auto softmax_tile = [&](floatx16 (&sacc)[2], bf16x8 (&pf)[4], int k0, bool full) {
    // element mask (tiles not flagged full for this wavefront: one uniform branch, selects inside)
    if (!full) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = k0 + 32 * kb + 8 * (i >> 2) + 4 * h + (i & 3);
          const bool ok = ST ? ((j <= rowc) & ((j <= a_i) | (j >= lo_i) | (j == prev_j) | (j == self_j)))
                             : (j <= rowc);
          sacc[kb][i] = ok ? sacc[kb][i] : -INFINITY;
        }
    }
    float mt = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, sacc[kb][i]);
    mt = fmaxf(mt, other_half(mt)) * a.scale_log2;
    // The reference maximum m only moves when a tile exceeds it by more than kRescaleGap (log2 units):
    // probabilities then stay below 2^kRescaleGap, exact in fp32/bf16 range, and the accumulators are
    // rescaled rarely.  The final normalisation divides the same factor out again.
    if (__any(mt > m + kRescaleGap)) {
      const float m_new = (mt > m + kRescaleGap) ? mt : m;
      const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m - m_ref);
      lacc[0] *= alpha;   // only element 0 is read back
      if (LSE) lx *= alpha;
#pragma unroll
      for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
      m = m_new;
    }
    const float neg_m = (m == -INFINITY) ? 0.f : -m;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        u32x4 pk;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][8 * half + 2 * w], a.scale_log2, neg_m));
          const float p1 =
              __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][8 * half + 2 * w + 1], a.scale_log2, neg_m));
          if (LSE) lx += p0 + p1;
          pk[w] = pack_bf16(p0, p1);
        }
        pf[2 * kb + half] = __builtin_bit_cast(bf16x8, pk);
      }
  };

  // ---- pipeline fill: tile 0 complete in LDS, the lagging wavefronts' share of tile 1 too ----
  load_tile(tile_off(t_begin));
  store_tile(0);
  load_tile(tile_off(t_begin + 1));
  if (grp == 1) {
    store_tile(1);
    load_tile(tile_off(t_begin + 2));
  }
  __syncthreads();
  if (grp == 1) phase_barrier();   // run one phase behind wavefronts 0-3

  int buf = 0;                     // LDS buffer of tile t
  int pv_buf = 0;
  bool pv_pending = false, fin_pending = false;
  bf16x8 pf[4];
  floatx16 sacc[2];

  StreamEntry ent = stream_entry(t_begin);
  uint32_t off_stage = tile_off(t_begin + 2 + grp);   // tile whose loads start in this step's vector phase
  for (int t = t_begin; t < t_end; ++t) {
    const StreamEntry ent_next = stream_entry(min(t + 1, t_end - 1));
    const uint32_t off_stage_next = tile_off(t + 3 + grp);
    const bool need = (ent.masks >> wave) & 1u;
    const bool full = (ent.masks >> (8 + wave)) & 1u;

    // ---- matrix phase: second product of the previous tile, unit switch, score product of this tile ----
    PHASE_MARK(0);
    if (pv_pending) pv_tile(pv_buf, pf);
    PHASE_MARK(4);
    if (fin_pending) finish_unit();
    if (ent.unit >= 0) begin_unit(ent.unit);
    if (need) qk_tile(buf, sacc);
    PHASE_MARK(1);
    phase_barrier();
    PHASE_MARK(2);

    // ---- vector phase: stage this wavefront's share of tile t+1+grp, start loading t+2+grp; softmax ----
    const int b1 = next_buf(buf);
    store_tile(grp ? next_buf(b1) : b1);
    load_tile(off_stage);
    PHASE_MARK(5);
    if (need) {
      const int k0 = (int)((ent.kv_off / (D * 2u)) % (uint32_t)a.N);  // first key of the tile within its head
      softmax_tile(sacc, pf, k0, full);
    }
    pv_pending = need;
    pv_buf = buf;
    fin_pending = ent.last != 0;
    buf = b1;
    ent = ent_next;
    off_stage = off_stage_next;
    PHASE_MARK(3);
    phase_barrier();
  }
  if (pv_pending) pv_tile(pv_buf, pf);
  if (fin_pending) finish_unit();
  if (grp == 0) phase_barrier();   // matches the extra barrier the lagging wavefronts took at the start
}

// Combines the partial results of a query tile whose key list was cut into slices.  One workgroup
// handles 16 rows of one (query tile, head): thread -> (row, 4 consecutive output elements).
constexpr int MERGE_ROWS = 16;
template <int D>
__global__ __launch_bounds__(256) void merge_kernel(const PrefillArgs a) {
  constexpr int C4 = D / 4, RB = BQ / MERGE_ROWS;
  const int rb = blockIdx.x % RB, hq = (blockIdx.x / RB) % a.Hq, mid = blockIdx.x / (RB * a.Hq);
  const MergeItem mi = a.merges[mid];
  const int r = rb * MERGE_ROWS + threadIdx.x / 16;
  const int row = mi.qtile * BQ + r;
  if (row >= a.N) return;
  float mx = -INFINITY, mxx = -INFINITY;
  for (int s = 0; s < mi.n_splits; ++s) {
    const size_t prow = ((size_t)(mi.slot0 + s) * a.Hq + hq) * BQ + r;
    mx = fmaxf(mx, a.ws_lse[2 * prow]);
    mxx = fmaxf(mxx, a.ws_lse[2 * prow + 1]);
  }
  float wsum = 0.f, xsum = 0.f;
  floatx4 acc[C4 / 16];
#pragma unroll
  for (int c = 0; c < C4 / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < mi.n_splits; ++s) {
    const size_t prow = ((size_t)(mi.slot0 + s) * a.Hq + hq) * BQ + r;
    const float w = __builtin_amdgcn_exp2f(a.ws_lse[2 * prow] - mx);
    wsum += w;
    xsum += __builtin_amdgcn_exp2f(a.ws_lse[2 * prow + 1] - mxx);
#pragma unroll
    for (int c = 0; c < C4 / 16; ++c) {
      const int c4 = (threadIdx.x % 16) + 16 * c;
      acc[c] += *reinterpret_cast<const floatx4*>(a.ws_o + prow * D + 4 * c4) * w;
    }
  }
  const float inv = 1.f / wsum;
#pragma unroll
  for (int c = 0; c < C4 / 16; ++c) {
    const int c4 = (threadIdx.x % 16) + 16 * c;
    u32x2 w2;
    w2[0] = pack_bf16(acc[c][0] * inv, acc[c][1] * inv);
    w2[1] = pack_bf16(acc[c][2] * inv, acc[c][3] * inv);
    *reinterpret_cast<u32x2*>(a.out + ((size_t)hq * a.N + row) * D + 4 * c4) = w2;
  }
  if (a.lse != nullptr && (threadIdx.x % 16) == 0)
    a.lse[(size_t)hq * a.N + row] = (mxx + __builtin_amdgcn_logf(xsum)) * kLn2;
}

template <int D, bool ST, bool LSE>
hipError_t launch_one(const PrefillArgs& a, dim3 grid, hipStream_t st) {
  constexpr unsigned lds_bytes = 6u * BK * D * sizeof(uint16_t);   // 3 K buffers + 3 V buffers
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kernel<D, ST, LSE>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((prefill_kernel<D, ST, LSE>), grid, dim3(512), lds_bytes, st, a);
  return hipSuccess;
}

template <int D, bool ST>
hipError_t launch_variant(const PrefillArgs& a, dim3 grid, hipStream_t st) {
  return a.lse != nullptr ? launch_one<D, ST, true>(a, grid, st) : launch_one<D, ST, false>(a, grid, st);
}

}  // namespace

size_t prefill_ws_bytes(const purekv_plan& p) {
  return (size_t)p.n_slots * p.g.Hq * BQ * (p.g.d + 2) * sizeof(float);
}

int launch_prefill(const purekv_plan& p, const void* q, const void* k, const void* v, void* out, float* lse,
                   void* ws, hipStream_t st) {
  PrefillArgs a{};
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.out = static_cast<uint16_t*>(out);
  a.lse = lse;
  a.ws_o = static_cast<float*>(ws);
  a.ws_lse = a.ws_o ? a.ws_o + (size_t)p.n_slots * p.g.Hq * BQ * p.g.d : nullptr;
  a.stream = p.d_stream;
  a.units = p.d_units;
  a.queue_begin = p.d_queue_begin;
  a.merges = p.d_merges;
  a.N = p.g.N;
  a.Nv = p.g.Nv;
  a.P = p.g.P;
  a.Hq = p.g.Hq;
  a.Hkv = p.g.Hkv;
  a.pattern = p.g.pattern;
  a.scale_log2 = p.g.scale * kLog2e;
  const dim3 grid((unsigned)p.n_queues), block(256);
  const dim3 mgrid((unsigned)(p.merges.size() * p.g.Hq * (BQ / MERGE_ROWS)));
  const bool sparse = p.g.pattern != PUREKV_PATTERN_DENSE;
  if (p.g.d == 128) {
    if (sparse)
      PUREKV_HIP_TRY((launch_variant<128, true>(a, grid, st)));
    else
      PUREKV_HIP_TRY((launch_variant<128, false>(a, grid, st)));
    if (!p.merges.empty()) hipLaunchKernelGGL(merge_kernel<128>, mgrid, block, 0, st, a);
  } else {
    if (sparse)
      PUREKV_HIP_TRY((launch_variant<64, true>(a, grid, st)));
    else
      PUREKV_HIP_TRY((launch_variant<64, false>(a, grid, st)));
    if (!p.merges.empty()) hipLaunchKernelGGL(merge_kernel<64>, mgrid, block, 0, st, a);
  }
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

}  // namespace purekv
