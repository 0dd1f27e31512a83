// ST-SpAttn / dense causal prefill attention for gfx950 (Sec. 3.2; Eq. 1 for the dense pattern).
//
// A persistent workgroup of 8 wavefronts walks a host-planned stream of 64-key tiles.  Each wavefront owns 32
// query rows of one head; the workgroup stacks Gs heads of one KV group x R row blocks (the mask depends on
// the row only, so stacked heads need the same tiles and nobody idles at the tile barriers).  Scores are
// formed transposed, S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that a lane holds 16 keys of ONE query: the
// softmax row maximum is an in-lane reduction plus one exchange between the two halves of the wavefront, and
// the probabilities leave the accumulator already in the register layout that the second product
// O^T = V^T P^T takes as its B operand.  The attention matrix never exists.
//
// K and V tiles sit in LDS row-major, XOR-swizzled in 16-byte units, and get there straight from global memory
// (16-byte loads whose destination is LDS: no staging registers, no vector ALU work, no LDS write instructions).
// K fragments are 128-bit LDS reads.  The second product contracts over the key, which runs ACROSS the rows of
// a row-major V tile: its fragments come from the LDS transpose read (ds_read_b64_tr_b16), which hands each
// lane 4 consecutive keys of one column.
//
// The softmax denominator is the sum of the bf16-ROUNDED probabilities, i.e. exactly the weights the second
// product applies, so each output row is a true convex combination of V rows.  It comes from the matrix pipe
// as well: one more MFMA per 16 keys multiplies the probabilities by an all-ones operand.
//
// Software pipeline inside every wavefront.  One iteration handles the score product of tile j and the second
// product of tile j-1: the exponentials of tile j-1 sit between the MFMAs of the score product, the running
// maximum of tile j and the address arithmetic of the next K/V loads between the MFMAs of the second product
// (scheduling fences pin every MFMA and the vector work behind it).  A wavefront thus keeps the matrix pipe and
// the vector ALU busy at the same time, the two wavefronts of a SIMD fill each other's gaps, and the workgroup
// meets at one barrier per tile, where the K/V buffers change hands.  The reference maximum of the online
// softmax moves lazily; when it does, the accumulators are rescaled at the top of the next iteration, after the
// second product that was still running in the old units.
//
// K and V each rotate through three LDS buffers: iteration j reads K(j) and V(j-1) and starts the loads of K(j+2)
// and V(j+1), whose buffers were last read in iteration j-1.  Every wavefront waits for its own loads at the top
// of an iteration, before the barrier; the loads are written as assembly so that these are the only waits (the
// compiler cannot tell which buffer a load of the builtin form fills and waits for all of them before LDS reads).
//
// Query tiles whose key list is long (the text rows, which see every key) are cut into slices run by different
// workgroups; every slice leaves a normalised fp32 partial result and its log-sum-exp in the workspace, and the
// slices are combined INSIDE the launch: wavefront by wavefront they count themselves in at a counter in the
// workspace, and at the end of its queue a workgroup adds up every list it took part in that is complete and not
// yet combined (compare-and-swap on the counter: exactly once, nobody waits).  One launch per call.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace purekv {
namespace {

constexpr int BK = PUREKV_BK;
constexpr int WG_ROWS = PUREKV_WAVES * PUREKV_BLOCK;   // rows of one workgroup's partial result
constexpr float kRescaleGap = 8.0f;
constexpr int kXTile = 4096;   // bf16 elements of a wavefront's private LDS tile (8 KB)
// Operand fragments are read from LDS this many MFMAs ahead of their use.
#ifndef PUREKV_QK_AHEAD
#define PUREKV_QK_AHEAD 2
#endif
#ifndef PUREKV_PV_AHEAD
#define PUREKV_PV_AHEAD 2
#endif
constexpr int kQkAhead = PUREKV_QK_AHEAD, kPvAhead = PUREKV_PV_AHEAD;

struct PrefillArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* out;
  float* lse;
  float* vnorm2;  // [Hkv, N] squared L2 norms of the V rows (VN variants), or null
  float* ws_o;    // [n_slots, n_groups, WG_ROWS, D] normalised partial outputs
  float* ws_lse;  // [n_slots, n_groups, WG_ROWS, 2] log2-domain log-sum-exp of the partial: {merge weight, exact}
  int32_t* counters;   // [n_slots, n_groups, PUREKV_WAVES] slices arrived per (split query tile, head group, wavefront);
                       // zero on entry, zero again on exit
  const StreamEntry* stream;
  const Unit* units;
  const int32_t* queue_begin;   // [n_queues + 1] offsets into stream
  const int32_t* queue_unit0;   // [n_queues + 1] first unit of each queue (units are numbered in stream order)
  int32_t N, Nv, P, Hq, Hkv, G;
  // byte strides of the (head, token) axes: Q, O per head and row, K/V per row (the head is in the stream entries)
  int64_t q_head_bytes, o_head_bytes;
  uint32_t q_row_bytes, kv_row_bytes, o_row_bytes;
  int32_t Gs, R, n_groups;   // workgroup shape: wavefront w -> row block w / Gs, head w % Gs
  uint32_t pattern;
  float scale_log2;  // softmax scale * log2(e)
  // Window plans: the log-sum-exp is written for rows >= lse_row0 only, and only the workgroups from lse_queue0 on
  // run units with such rows (the window kernel: only they keep the exact row sum).  Else 0 and 0.
  int32_t lse_row0, lse_queue0;
};

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) shortx4* LdsShortx4;

// Device-scope ("agent") accesses for data that crosses workgroups inside one launch: buffer instructions with the
// sc1 bit, which go through to memory instead of staying in (or being served from) the issuing XCD's L2.  The
// compiler keeps track of their completion like of any other load or store.
typedef __amdgpu_buffer_rsrc_t BufferRsrc;
constexpr int kDeviceScope = 16;   // cache-policy operand of the buffer builtins: bit 4 = sc1
__device__ __forceinline__ BufferRsrc make_rsrc(const void* base) {   // base must be wave-uniform
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ void store_device_16(BufferRsrc r, uint32_t off, floatx4 x) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x), r, (int)off, 0, kDeviceScope);
}
__device__ __forceinline__ void store_device_8(BufferRsrc r, uint32_t off, floatx2 x) {
  __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, x), r, (int)off, 0, kDeviceScope);
}
__device__ __forceinline__ floatx4 load_device_16(BufferRsrc r, uint32_t off) {
  return __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, kDeviceScope));
}
__device__ __forceinline__ floatx2 load_device_8(BufferRsrc r, uint32_t off) {
  return __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, kDeviceScope));
}

// V tile [BK][D] bf16 in LDS, row-major; the transpose read of a 16-lane group touches 4 consecutive rows x 32
// bytes, two such groups run side by side: XOR-ing the 32-byte pair index with the row's low bits keeps them on
// distinct banks.
template <int D>
__device__ __forceinline__ int vswz(int r, int u) {
  return r * D + ((u ^ ((r & (D / 32 - 1)) << 2)) * 8);
}
template <int D>
__device__ __forceinline__ void vunswz(int p, int& r, int& u) {
  constexpr int CPR = D / 8;
  r = p / CPR;
  u = (p % CPR) ^ ((r & (D / 32 - 1)) << 2);
}

// Wave-uniform, read-only tables are fetched through the scalar cache (constant address space).
typedef const u32x4 __attribute__((address_space(4))) * ConstQuads;

// Stream entry as the kernel uses it.
struct Step {
  uint32_t kv_off;   // byte offset of the tile in K and V
  uint32_t need;     // need bits | last << 16 | first << 17 | (valid rows - 1) << 18
  uint32_t kinds;
  int32_t k0;        // first key of the tile
};

// Combination, at the end of the workgroup's queue (the pipeline's registers are free then): for every slice this
// wavefront ran, a counter that stands at n_splits means "all slices in memory, nobody has combined them yet";
// whoever moves it to n_splits + 1 (compare-and-swap: exactly one wavefront can) adds the partial results up in a
// fixed order (slice 0, 1, ...: reproducible bit for bit), writes the output rows and leaves the counter at zero
// for the next launch.  The wavefront whose slice arrived last always finds n_splits or a combination already
// claimed when it gets here, so every split tile is combined exactly once before the launch ends, and nobody ever
// waits for anybody.  The planner runs the closing slice of a list last in its queue and the other slices first
// in theirs: the workgroup it charged for the combination is then normally the one that does it.  Partial results
// and counters travel as device-scope accesses (they bypass the L2 of the issuing XCD), ordered by "stores
// acknowledged -> counter increment ... counter read -> loads".
// Kept out of line (and called after the tile loop only): inlined, its registers and branches changed the
// allocation of the loop itself and cost the dense kernel, which never combines anything, 3.5 %.
typedef __attribute__((address_space(3))) float LdsFloat;
typedef __attribute__((address_space(3))) floatx2 LdsFloatx2;
struct CombineCall {
  int32_t* counters;
  const float* ws_o;
  const float* ws_lse;
  uint16_t* out;
  float* lse;
  LdsFloat* xs;   // this wavefront's private 8 KB of LDS (an LDS pointer: the table below is read with LDS instructions)
  int64_t o_head_bytes;
  uint32_t o_row_bytes;
  int32_t N, n_groups, wave, hl, rb, lse_row0;
};
template <int D, bool LSE>
__device__ __noinline__ void combine_slices(const CombineCall c, const u32x4 un, const u32x4 mu) {
  const int ns = (int)un[2];
  int32_t* const counter = c.counters + (int)mu[1] * PUREKV_WAVES + c.wave;
  int claimed = 0;
  if ((threadIdx.x & 63) == 0) {
    int expected = ns;
    claimed = __hip_atomic_compare_exchange_strong(counter, &expected, ns + 1, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!__builtin_amdgcn_readfirstlane(claimed)) return;
  asm volatile("" ::: "memory");
  const int hq = (int)un[1] + c.hl, row0 = (int)un[0] + c.rb * 32;
  int ln = threadIdx.x & 63;
  asm volatile("" : "+v"(ln));
  const uint32_t slice_rows = (uint32_t)c.n_groups * WG_ROWS;   // rows between consecutive slices' blocks
  const float* const po = c.ws_o + ((size_t)mu[0] + c.wave * 32) * D;      // this wavefront's block in slice 0
  const float* const pl = c.ws_lse + 2 * ((size_t)mu[0] + c.wave * 32);
  LdsFloat* const Wt = c.xs;   // [32 rows][ns]{merge weight, exact log-sum-exp}: <= 8 KB
  // (row, slice) pairs over the lanes: one round trip fetches every slice's two log-sum-exp values of every row
  for (int pb = 0; pb < 32 * ns; pb += 64) {
    const int pr = min(pb + ln, 32 * ns - 1), r = pr & 31, sl = pr >> 5;
    const floatx2 l2 = load_device_8(make_rsrc(pl), ((uint32_t)sl * slice_rows + (uint32_t)r) * 8u);
    *(LdsFloatx2*)(Wt + 2 * (r * ns + sl)) = l2;
  }
  {  // lane (n, h): row n (both halves compute the same): maxima, weights normalised to sum 1, exact log-sum-exp
    const int n = ln & 31;
    float mx = -INFINITY, mxx = -INFINITY;
    for (int sl = 0; sl < ns; ++sl) {
      const floatx2 l2 = *(const LdsFloatx2*)(Wt + 2 * (n * ns + sl));
      mx = fmaxf(mx, l2[0]);
      mxx = fmaxf(mxx, l2[1]);
    }
    float wsum = 0.f, xsum = 0.f;
    for (int sl = 0; sl < ns; ++sl) {
      const floatx2 l2 = *(const LdsFloatx2*)(Wt + 2 * (n * ns + sl));
      wsum += __builtin_amdgcn_exp2f(l2[0] - mx);
      xsum += __builtin_amdgcn_exp2f(l2[1] - mxx);
    }
    const float inv = 1.f / wsum;
    for (int sl = 0; sl < ns; ++sl) {
      const float wgt = __builtin_amdgcn_exp2f(Wt[2 * (n * ns + sl)] - mx) * inv;
      if ((ln >> 5) == 0) Wt[2 * (n * ns + sl)] = wgt;
    }
    if (LSE && (ln >> 5) == 0 && row0 + n < c.N && row0 + n >= c.lse_row0)
      c.lse[(size_t)hq * c.N + row0 + n] = (mxx + __builtin_amdgcn_logf(xsum)) * kLn2;
  }
  // Weighted sum, PB 16-byte pieces (4 columns of one row each) per lane at a time, the pieces of up to four
  // slices in flight together (the pipeline's registers are free here): what this costs is round trips to memory.
  constexpr int CH = D / 4, NI = 32 * CH / 64, PB = 8;   // pieces per row; pieces per lane; pieces per batch
  static_assert(NI % PB == 0, "batches cover the block");
  char* const otile = reinterpret_cast<char*>(c.out) + (int64_t)hq * c.o_head_bytes + (int64_t)row0 * c.o_row_bytes;
  const int rows_left = c.N - row0;
#pragma unroll 1
  for (int i0 = 0; i0 < NI; i0 += PB) {
    floatx4 acc[PB];
#pragma unroll
    for (int i = 0; i < PB; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int s0 = 0; s0 < ns; s0 += 4) {
      floatx4 x[4][PB];
#pragma unroll
      for (int ss = 0; ss < 4; ++ss) {
        const int sl = min(s0 + ss, ns - 1);   // slices past the end repeat the last one (weight 0 below)
        const BufferRsrc pbuf = make_rsrc(po + (size_t)sl * slice_rows * D);
#pragma unroll
        for (int i = 0; i < PB; ++i) x[ss][i] = load_device_16(pbuf, (uint32_t)((i0 + i) * 64 + ln) * 16u);
      }
#pragma unroll
      for (int ss = 0; ss < 4; ++ss)
#pragma unroll
        for (int i = 0; i < PB; ++i) {
          const int r = ((i0 + i) * 64 + ln) / CH;
          const float wgt = s0 + ss < ns ? Wt[2 * (r * ns + min(s0 + ss, ns - 1))] : 0.f;
          acc[i] += x[ss][i] * wgt;
        }
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int r = ((i0 + i) * 64 + ln) / CH, c4 = ((i0 + i) * 64 + ln) % CH;
      u32x2 w2;
      w2[0] = pack_bf16(acc[i][0], acc[i][1]);
      w2[1] = pack_bf16(acc[i][2], acc[i][3]);
      if (r < rows_left) __builtin_nontemporal_store(w2, reinterpret_cast<u32x2*>(otile + (uint32_t)r * c.o_row_bytes + 8 * c4));
    }
  }
  if ((threadIdx.x & 63) == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
}

// ST  = false: dense causal pattern only (block kinds full and causal); true: any pattern.
// LSE = true : also keeps the exact fp32 row sum for the log-sum-exp output.
//
// Persistent kernel: workgroup q walks stream[queue_begin[q] .. queue_begin[q+1]).  Every stream entry is one
// key tile: all wavefronts load it, the wavefronts whose row block needs it multiply the 32-key halves they
// need.  Units (query tile slice x head group) follow each other in the stream without draining the K/V
// pipeline; the query rows of the next unit are fetched while the last tile of the current one is finished.
// VN  = true : for plans that leave the last wavefront without rows (seven stacked heads): that wavefront emits the
//              squared norms of the V rows of every tile this step owns (Eq. 3 / Eq. 4 need ||V||: the tile is in
//              LDS anyway).  Plans that keep all eight wavefronts busy get the norms from a pass of their own.
template <int D, bool ST, bool LSE, bool VN>
__device__ __forceinline__ void prefill_body(const PrefillArgs& a) {
  constexpr int KSTEPS = D / 16;        // MFMA k-steps of the score product
  constexpr int DBLK = D / 32;          // 32-row blocks of O^T
  constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
  constexpr int NLD = BK * CPR / 512;   // 16-byte loads per thread and tile, for K and for V
  constexpr int NBUF = 3;
  static_assert(sizeof(StreamEntry) == 16 && sizeof(Unit) == 32, "tables are read as 16-byte quads");
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* const Ks_base = smem;                     // NBUF x [BK][D]
  uint16_t* const Vs_base = smem + NBUF * BK * D;     // NBUF x [BK][D]
  // One private 8 KB tile per wavefront (32 rows x 256 bytes) through which query rows come in and output rows
  // go out: global memory sees whole rows (16 lanes x 16 bytes each), the MFMA register layouts see LDS.
  uint16_t* const Xs_base = smem + 2 * NBUF * BK * D; // PUREKV_WAVES x kXTile

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int rb = wave / a.Gs, hl = wave - rb * a.Gs;   // row block and stacked head of this wavefront
  const bool active = wave < a.Gs * a.R;
  const int t_begin = a.queue_begin[blockIdx.x], t_end = a.queue_begin[blockIdx.x + 1];
  if (t_begin >= t_end) return;

  // ---- load maps (per-thread constants) ----
  // Load i of this wavefront fills 16-byte positions (NLD*wave + i)*64 + lane of a tile: 1 KB of LDS, contiguous
  // (the hardware writes lane l's 16 bytes at base + 16 l); which (row, slot) of the global tile a lane fetches
  // follows from the swizzle of that position.  Rows past the end of the sequence re-read the last valid row
  // (their scores are masked, their probabilities zero).
  int k_row[NLD], v_row[NLD];
  uint32_t k_col[NLD], v_col[NLD];   // byte offset within the row
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int p = (NLD * wave + i) * 64 + lane;
    int r, u;
    kunswz<D>(p, r, u);
    k_row[i] = r;
    k_col[i] = (uint32_t)u * 16u;
    vunswz<D>(p, r, u);
    v_row[i] = r;
    v_col[i] = (uint32_t)u * 16u;
  }
  const uint32_t kv_rb = a.kv_row_bytes;   // below 2^24: one 24-bit multiply-add per load address
  const char* const k_bytes = reinterpret_cast<const char*>(a.k);
  const char* const v_bytes = reinterpret_cast<const char*>(a.v);
  auto issue_k = [&](const Step& s, int buf) {
    const int rv = (int)((s.need >> 18) & 63u);
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const uint32_t off = __umul24((uint32_t)min(k_row[i], rv), kv_rb) + (s.kv_off + k_col[i]);
      load_to_lds_16(k_bytes, off, Ks_base + buf * (BK * D) + (NLD * wave + i) * 512);
    }
  };
  auto issue_v = [&](const Step& s, int buf) {
    const int rv = (int)((s.need >> 18) & 63u);
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const uint32_t off = __umul24((uint32_t)min(v_row[i], rv), kv_rb) + (s.kv_off + v_col[i]);
      load_to_lds_16(v_bytes, off, Vs_base + buf * (BK * D) + (NLD * wave + i) * 512);
    }
  };
  // All loads of this wavefront have written LDS (vmcnt == 0; the other counters are left alone).
  auto wait_loads = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };

  // Stream entries and unit records: fetched before they are needed, so that no phase waits for a global load.
  const ConstQuads stream_c = (ConstQuads)(uintptr_t)a.stream;
  const ConstQuads units_c = (ConstQuads)(uintptr_t)a.units;
  auto fetch_step = [&](int t) {   // entries past the end repeat the last one; their loads are skipped
    const u32x4 w = stream_c[min(t, t_end - 1)];
    Step s;
    s.kv_off = w[0];
    s.need = w[1];
    s.kinds = w[2];
    s.k0 = (int32_t)w[3];
    return s;
  };
  auto next_buf = [](int b) { return b == NBUF - 1 ? 0 : b + 1; };
  // ---- per-unit state ----
  int hq = 0, row0 = 0, rowc = 0, a_i = 0, lo_i = 0, prev_j = -1, self_j = -1;
  int u_nsplits = 1, u_ws_row0 = -1, u_unit = 0;
  int unit_id = a.queue_unit0[blockIdx.x];   // unit of the tile on the score side (units are numbered in stream order)
  bf16x8 qf[KSTEPS];
  // m: reference maximum (log2 units); lacc: every element holds the sum of the bf16-rounded probabilities of
  // query n, accumulated by the matrix pipe: an output row is an exact convex combination of V rows (normalising
  // with the exact sum instead saves the LSE variant its row-sum MFMAs, 3.6 % of the dense kernel, but a row
  // dominated by one key then carries that key's probability rounding, 2^-9 |v|, on top of the output rounding:
  // 0.023 was seen against the 0.02 bound); lx: exact fp32 sum of the lane's probabilities (LSE variant only).
  // The row sum uses the 16x16x32 MFMA (4 accumulator registers, half the pipe time of a 32x32x16).  Its B operand
  // takes lane l as (column l % 16, k-group l / 16); a probability fragment has lane l = (query l % 32, keys
  // 8 (l / 32) ..), so k-groups 0 and 2 of column j are the 16 keys of query j and k-groups 1 and 3 those of query
  // j + 16.  The A operand (lane l = row l % 16, k-group l / 16) is 1 where the row's output lanes 16 (row / 4) ..
  // want that k-group and 0 elsewhere: output lane l (column l % 16, rows 4 (l / 16) ..) then holds the sum of
  // query l % 32 in all four registers.
  float m = -INFINITY, lx = 0.f;
  floatx16 oacc[DBLK];
  floatx4 lacc;
  const uint32_t ones_word = ((((lane >> 4) ^ (lane >> 2)) & 1) == 0) ? 0x3F803F80u : 0u;   // two bf16 ones or zeros

  uint16_t* const Xs = Xs_base + wave * kXTile;
  constexpr int XQ = 32 * CPR / 64;   // 1 KB pieces of a 32-row bf16 tile
  // Unit record {row0, head0, n_splits, ws_row0}: start fetching this wavefront's 32 query rows into its private
  // LDS tile (same swizzled layout as a K tile; rows past the end repeat the last row).
  auto prefetch_q = [&](const u32x4 un) {
    if (active) {
      int ln = lane;   // opaque copy: keeps the address arithmetic inside the unit switch
      asm volatile("" : "+v"(ln));
      const int r0 = (int)un[0] + rb * 32;
      // uniform base of the head + 32-bit lane offsets (a tensor spans at most 2^31 bytes); the row is clamped to
      // the last row of the sequence, also when the whole block lies past it (ragged last query tile)
      const char* const qhead = reinterpret_cast<const char*>(a.q) + (int64_t)((int)un[1] + hl) * a.q_head_bytes;
      if constexpr (D == 128) {
        // piece i of this lane: row 4 i + ln / 16, slot (ln % 16) ^ (row % 16) = (ln % 16) ^ (ln / 16) ^ (4 i % 16):
        // one lane constant, then per piece a row (add, clamp, multiply) and one xor-add
        const int row_l = r0 + (ln >> 4);
        const uint32_t slot_l = (uint32_t)(((ln & 15) ^ (ln >> 4)) * 16);
#pragma unroll
        for (int i = 0; i < XQ; ++i) {
          const uint32_t off = (uint32_t)min(row_l + 4 * i, a.N - 1) * a.q_row_bytes + (slot_l ^ (uint32_t)(((4 * i) & 15) * 16));
          load_to_lds_16(qhead, off, Xs + i * 512);
        }
      } else {
#pragma unroll
        for (int i = 0; i < XQ; ++i) {
          int r, u;
          kunswz<D>(i * 64 + ln, r, u);
          const uint32_t off = (uint32_t)min(r0 + r, a.N - 1) * a.q_row_bytes + (uint32_t)u * 16u;
          load_to_lds_16(qhead, off, Xs + i * 512);
        }
      }
    }
  };
  // Query fragments of the unit that starts: B operand of k-step s = columns 16 s + 8 h .. of row n.
  auto load_q_frags = [&]() {
    wait_loads();
    int ln = lane;   // opaque copy: the eight addresses are formed here, not kept in registers across the loop
    asm volatile("" : "+v"(ln));
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
      qf[s] = *reinterpret_cast<const bf16x8*>(Xs + kswz<D>(ln & 31, 2 * s + (ln >> 5)));
  };
  // Normalise and write this wavefront's 32 rows of the unit that just finished.  The accumulators hold, per
  // lane, 4 consecutive columns of ONE row at a time; the rows are assembled in the private LDS tile and leave
  // as whole 256-byte pieces (a version that stored 8-byte pieces per lane straight from the accumulator layout
  // produced 1024 partial-line writes per wavefront and cost several thousand cycles per unit).
  float fin_inv = 0.f, fin_lse = 0.f;   // 1 / row sum and log-sum-exp (natural log) of the unit being finished
  float m_fin = -INFINITY;              // its reference maximum
  constexpr int NPIECE = 4 * DBLK;      // (output block, group of 4 accumulator registers): 8 bytes per lane
  auto finish_sums = [&]() {
    const float l_tot = lacc[0];
    fin_inv = l_tot > 0.f ? __builtin_amdgcn_rcpf(l_tot) : 0.f;
    if (LSE) fin_lse = (m_fin + __builtin_amdgcn_logf(lx + other_half(lx))) * kLn2;
  };
  // `ln` is an opaque copy of the lane id: addresses derived from it are recomputed where they are used instead
  // of being hoisted out of the tile loop, where they would occupy registers all the time.
  auto stage_piece = [&](int j, int ln) {
    const int b = j >> 2, g4 = j & 3;
    u32x2 w;
    w[0] = pack_bf16(oacc[b][4 * g4 + 0] * fin_inv, oacc[b][4 * g4 + 1] * fin_inv);
    w[1] = pack_bf16(oacc[b][4 * g4 + 2] * fin_inv, oacc[b][4 * g4 + 3] * fin_inv);
    *reinterpret_cast<u32x2*>(Xs + kswz<D>(ln & 31, 4 * b + g4) + 4 * (ln >> 5)) = w;   // columns 32 b + 8 g4 + 4 h ..
  };
  auto flush_rows = [&]() {
    if (!active) return;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    // uniform base of the tile's first row + 32-bit lane offsets
    char* const otile = reinterpret_cast<char*>(a.out) + (int64_t)hq * a.o_head_bytes + (int64_t)row0 * a.o_row_bytes;
    const int rows_left = a.N - row0;   // rows of the tile that exist
    // read the pieces back in batches of four before storing any: the LDS latencies overlap
#pragma unroll
    for (int i0 = 0; i0 < XQ; i0 += 4) {
      u32x4 w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = *reinterpret_cast<const u32x4*>(Xs + ((i0 + i) * 64 + ln) * 8);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int r, u;
        kunswz<D>((i0 + i) * 64 + ln, r, u);
        const uint32_t off = (uint32_t)r * a.o_row_bytes + (uint32_t)u * 16u;
        // (non-temporal: the output rows are not read again by this launch and should not push the K/V tiles of the
        // KV head this XCD serves out of its L2 -- measured on the 32-frame ST shape: 1.5-2 us of 103)
        if (rows_left >= 32 || r < rows_left) __builtin_nontemporal_store(w[i], reinterpret_cast<u32x4*>(otile + off));
      }
    }
    if (LSE && (ln >> 5) == 0 && (ln & 31) < rows_left && row0 + (ln & 31) >= a.lse_row0)
      a.lse[(size_t)hq * a.N + row0 + (ln & 31)] = fin_lse;
  };
  // fp32 partial result of a slice: 64 columns (256 bytes a row) per round through the same tile
  auto finish_slice = [&]() {
    if (!active) return;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int n = ln & 31, h = ln >> 5;
    const float l_tot = lacc[0];
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse2 = m_fin + __builtin_amdgcn_logf(l_tot);  // log2 domain; -inf when the slice saw no key
    const float lse2x = LSE ? m_fin + __builtin_amdgcn_logf(lx + other_half(lx)) : lse2;
    float* const Xf = reinterpret_cast<float*>(Xs);
    // The partial result is read by another workgroup (possibly on another XCD, behind another L2) later in this
    // launch: device-scope stores, which go through to memory.
    const BufferRsrc wbuf = make_rsrc(a.ws_o + ((size_t)u_ws_row0 + wave * 32) * D);
#pragma unroll
    for (int rnd = 0; rnd < D / 64; ++rnd) {
#pragma unroll
      for (int bb = 0; bb < 2; ++bb)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          floatx4 w;
#pragma unroll
          for (int r = 0; r < 4; ++r) w[r] = oacc[2 * rnd + bb][4 * g4 + r] * inv;
          // columns 32 bb + 8 g4 + 4 h .. of the round: 16-byte slot 8 bb + 2 g4 + h of a 256-byte row
          *reinterpret_cast<floatx4*>(Xf + kswz<128>(n, 8 * bb + 2 * g4 + h) / 2) = w;
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
      for (int i0 = 0; i0 < 8; i0 += 4) {
        floatx4 w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = *reinterpret_cast<const floatx4*>(Xf + ((i0 + i) * 64 + ln) * 4);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int r, u;
          kunswz<128>((i0 + i) * 64 + ln, r, u);
          store_device_16(wbuf, (uint32_t)(r * D + 64 * rnd + 4 * u) * 4u, w[i]);
        }
      }
    }
    if (h == 0) store_device_8(make_rsrc(a.ws_lse + 2 * ((size_t)u_ws_row0 + wave * 32)), (uint32_t)n * 8u, floatx2{lse2, lse2x});
  };
  // Hand-off of a finished slice, wavefront by wavefront (wavefront w of every slice of a query tile holds the same
  // 32 rows of the same head).  Arrival: once this wavefront's stores are acknowledged (device scope: they are in
  // memory) it adds one to the counter of its (query tile, head group, wavefront index) -- nothing more inside the
  // tile loop, whose registers are all taken.
  auto slice_arrive = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const u32x4 mu = units_c[2 * u_unit + 1];   // {first workspace row of slice 0, counter, -, -}
    if (lane == 0)
      (void)__hip_atomic_fetch_add(a.counters + (int)mu[1] * PUREKV_WAVES + wave, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  // Finish of a unit that holds a whole key list: normalise, round, stage, store.
  auto finish_unit = [&]() {
    if (active) {
      int ln = lane;
      asm volatile("" : "+v"(ln));
      finish_sums();
#pragma unroll
      for (int j = 0; j < NPIECE; ++j) stage_piece(j, ln);
    }
    flush_rows();
  };

  // Operand fragments are read from LDS a few MFMAs ahead of their use (register ring); the scheduling fences
  // keep that order, so each wait covers only the oldest read.
  // Scores of one 32-key half: S^T[32 keys, 32 queries] = K Q^T; Kh = first row of the half in its LDS tile.
  // `between(i)` runs after MFMA i is issued (independent vector work that hides under the matrix pipe).
  const int kq0 = kswz<D>(n, h);
  auto qk_half = [&](const uint16_t* Kh, floatx16& s, auto between) {
    // fragment i sits at kswz(n, 2 i + h) = kswz(n, h) ^ 16 i: one XOR per read from a single per-lane base (an
    // opaque copy, or the eight offsets would be hoisted out of the tile loop into registers of their own)
    int kq = kq0;
    auto rd = [&](int i) { return *reinterpret_cast<const bf16x8*>(Kh + (kq ^ (16 * i))); };
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    constexpr int A = kQkAhead < KSTEPS ? kQkAhead : KSTEPS;
    bf16x8 f[A + 1];
#pragma unroll
    for (int i = 0; i < A; ++i) f[i] = rd(i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < KSTEPS; ++i) {
      if (i + A < KSTEPS) f[(i + A) % (A + 1)] = rd(i + A);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % (A + 1)], qf[i], s, 0, 0, 0);
      between(i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // O^T += V^T P^T and row sums += 1 P^T over the four 16-key steps of a tile (a half the row block does not
  // need carries zero probabilities).
  // A operand of step ks, output block b: lane (d = 32 b + n, key group h) needs keys 16 ks + 4 h + {0..3} and
  // 16 ks + 8 + 4 h + {0..3} of column d, in that order (the order the probabilities have in the B operand).
  // One transpose read gives the lanes of a 16-lane group 4 consecutive rows of 16 consecutive columns: lane s
  // of the group supplies the address of row (s / 4), columns 4 (s % 4) .. +3, and lane j receives column j.
  const int tr_row = 4 * h + ((lane & 15) >> 2);                 // row within a 16-key step, first read
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);    // column within a 32-column block
  const int v_off0 = vswz<D>(tr_row, tr_col >> 3) + (tr_col & 7);   // output block b: v_off0 ^ 32 b
  auto pv_tile = [&](int buf, const bf16x8 (&pf)[4], auto between) {
    const uint16_t* Vs = Vs_base + buf * (BK * D);
    constexpr int NF = 4 * DBLK;
    int vo = v_off0;   // opaque copy, as for the K fragments
    asm volatile("" : "+v"(vo));
    auto rd = [&](int i) {   // fragment i: 16-key step i % 4 of output block i / 4
      const uint16_t* p = Vs + (vo ^ (32 * (i >> 2))) + 16 * (i & 3) * D;   // rows 16 ks + .. : the swizzle ignores them
      const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsShortx4)p);
      const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsShortx4)(p + 8 * D));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    uint32_t ow = ones_word;   // opaque: the four-register operand exists only here
    asm volatile("" : "+v"(ow));
    const bf16x8 ones8 = __builtin_bit_cast(bf16x8, u32x4{ow, ow, ow, ow});
    constexpr int A = kPvAhead;
    bf16x8 f[A + 1];
#pragma unroll
    for (int i = 0; i < A; ++i) f[i] = rd(i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones8, pf[ks], lacc, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      if (i + A < NF) f[(i + A) % (A + 1)] = rd(i + A);
      oacc[i >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % (A + 1)], pf[i & 3], oacc[i >> 2], 0, 0, 0);
      between(i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Element mask of one 32-key block whose first key is `kbase`; element i of the accumulator is key
  // kbase + 4h + 8 (i / 4) + i % 4 of this lane's query.  One uniform branch per block, selects inside.
  auto mask_block = [&](floatx16& s, uint32_t kind, int kbase) {
    if (kind == kKindFull) return;
    const int jb = kbase + 4 * h;
    if (!ST || kind == kKindCausal) {
      const int thr = rowc - jb;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = (8 * (i >> 2) + (i & 3) <= thr) ? s[i] : -INFINITY;
    } else if (kind == kKindPrev) {
      const int eq = prev_j - jb;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = (8 * (i >> 2) + (i & 3) == eq) ? s[i] : -INFINITY;
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int j = jb + 8 * (i >> 2) + (i & 3);
        const bool ok = (j <= rowc) & ((j <= a_i) | (j >= lo_i) | (j == prev_j) | (j == self_j));
        s[i] = ok ? s[i] : -INFINITY;
      }
    }
  };
  // ---- software pipeline inside every wavefront ----
  // Iteration j: the score product of tile j with the exponentials of tile j-1 between its MFMAs, then the second
  // product of tile j-1 with the running maximum of tile j between its MFMAs.  A wavefront keeps its own matrix
  // pipe and vector ALU busy at the same time, and the two wavefronts of a SIMD fill each other's gaps; the
  // workgroup meets once per tile, where the K/V buffers change hands.
  // K tile x and V tile x live in ring buffer (x - t_begin) % 3.  Iteration j reads K(j) and V(j-1) and starts the
  // loads of K(j+2) and V(j+1): their buffers were last read in iteration j-1, which every wavefront has left when
  // it passes the barrier at the top of iteration j.
  floatx16 S[2][2];   // scores of two consecutive tiles, two 32-key halves each
  bf16x8 pf[4];       // probabilities of the tile whose second product comes next
  float alpha = 1.f;  // pending rescale of the accumulators (the reference maximum moved)
  bool resc = false;
  int q_hq = 0, q_row0 = 0, q_nsplits = 1, q_ws_row0 = -1, q_unit = 0;   // unit of the tile on the score side
  auto begin_qk_unit = [&](const u32x4 un) {
    q_hq = (int)un[1] + hl;
    q_nsplits = (int)un[2];
    q_ws_row0 = (int)un[3];
    q_unit = unit_id;
    q_row0 = (int)un[0] + rb * 32;
    rowc = min(q_row0 + n, a.N - 1);
    const bool sparse_row = ST && a.pattern != 0u && rowc < a.Nv;
    const int frame = sparse_row ? rowc / a.P : 0;
    a_i = sparse_row ? min(rowc, a.P - 1) : rowc;
    lo_i = sparse_row ? ((a.pattern & 1u) ? frame * a.P : rowc + 1) : 0;
    prev_j = (sparse_row && (a.pattern & 2u) && frame >= 1) ? rowc - a.P : -1;
    self_j = (sparse_row && (a.pattern & 2u)) ? rowc : -1;
  };
  auto adopt_unit = [&]() {   // the second-product side moves on to the unit of the score side
    hq = q_hq;
    row0 = q_row0;
    u_nsplits = q_nsplits;
    u_ws_row0 = q_ws_row0;
    u_unit = q_unit;
    lx = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) lacc[i] = 0.f;
#pragma unroll
    for (int b = 0; b < DBLK; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[b][i] = 0.f;
  };
  auto fill_ninf = [&](floatx16& x) {
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = -INFINITY;
  };
  // Slice i of 16: probabilities of elements 2 w, 2 w + 1 (w = i % 8) of half i / 8 -> one word of pf.
  auto exp_slice = [&](const floatx16 (&Sp)[2], float neg_m, int i) {
    const int hf = i >> 3, w = i & 7;
    // The multiply-adds are volatile: the whole slice stays where it is called (between two MFMAs) instead of
    // being collected ahead of the product.
    float y0, y1;
    asm volatile("v_fma_f32 %0, %2, %3, %4\n\tv_fma_f32 %1, %5, %3, %4"
                 : "=&v"(y0), "=&v"(y1)
                 : "v"(Sp[hf][2 * w]), "s"(a.scale_log2), "v"(neg_m), "v"(Sp[hf][2 * w + 1]));
    const float e0 = __builtin_amdgcn_exp2f(y0);
    const float e1 = __builtin_amdgcn_exp2f(y1);
    if (LSE) lx += e0 + e1;
    u32x4 pk = __builtin_bit_cast(u32x4, pf[2 * hf + (w >> 2)]);
    pk[w & 3] = pack_bf16(e0, e1);
    pf[2 * hf + (w >> 2)] = __builtin_bit_cast(bf16x8, pk);
  };
  auto max_slice = [&](const floatx16 (&Sn)[2], float& mt, int i) {
    const int hf = i >> 3, w = i & 7;
    mt = fmaxf(fmaxf(mt, Sn[hf][2 * w]), Sn[hf][2 * w + 1]);
  };
  // New reference maximum after a tile whose (masked) maximum is mt; `first`: the tile starts a unit.
  auto update_reference = [&](float mt, bool first) {
    mt = fmaxf(mt, other_half(mt)) * a.scale_log2;
    m_fin = m;
    if (first) m = -INFINITY;
    // The reference only moves when a tile exceeds it by more than kRescaleGap (log2 units): probabilities stay
    // below 2^kRescaleGap and the accumulators are rescaled rarely (before the next second product).
    if (__any(mt > m + kRescaleGap)) {
      const float m_new = (mt > m + kRescaleGap) ? mt : m;
      const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
      alpha = __builtin_amdgcn_exp2f(m - m_ref);
      resc = !first;   // a unit that starts has nothing accumulated yet
      m = m_new;
    }
  };

  Step e_prev = fetch_step(t_begin), e_cur = fetch_step(t_begin + 1), e_n1 = fetch_step(t_begin + 2),
       e_n2 = fetch_step(t_begin + 3);
  u32x4 un_next = units_c[2 * unit_id];   // the first entry of a queue always starts a unit
  bool q_pref = false;
  // Query rows of the next unit: requested one tile before the current unit's last one when it has that many
  // (x: index of the tile on the score side, ex / ex1: its entry and the next one), and never before the rows of
  // a unit finished in the same iteration have left the private tile.
  auto maybe_prefetch_q = [&](int x, const Step& ex, const Step& ex1, const u32x4 un_rec) {
    if (q_pref || x >= t_end) return;
    const bool lastc = (ex.need >> 16) & 1u;
    const bool lastn = x + 1 < t_end && ((ex1.need >> 16) & 1u);
    const int s_next = lastc ? x + 1 : x + 2;   // first entry of the next unit
    if ((lastc || lastn) && s_next < t_end) {
      un_next = un_rec;
      __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): every read of the private tile has returned
      prefetch_q(un_next);
      q_pref = true;
    }
  };
  prefetch_q(un_next);
  issue_k(e_prev, 0);
  issue_v(e_prev, 0);
  if (t_begin + 1 < t_end) {
    issue_k(e_cur, 1);
    issue_v(e_cur, 1);
  }
  if (t_begin + 2 < t_end) issue_k(e_n1, 2);
  load_q_frags();
  begin_qk_unit(un_next);
  adopt_unit();
  maybe_prefetch_q(t_begin, e_prev, e_cur, units_c[2 * (unit_id + 1)]);
  __syncthreads();
  // scores and reference maximum of the first tile
  if (active) {
    const uint32_t nb = (e_prev.need >> (2 * rb)) & 3u, kinds = (e_prev.kinds >> (4 * rb)) & 15u;
    if (nb & 1u) {
      qk_half(Ks_base, S[0][0], [](int) {});
      mask_block(S[0][0], kinds & 3u, e_prev.k0);
    } else {
      fill_ninf(S[0][0]);
    }
    if (nb & 2u) {
      qk_half(Ks_base + 32 * D, S[0][1], [](int) {});
      mask_block(S[0][1], (kinds >> 2) & 3u, e_prev.k0 + 32);
    } else {
      fill_ninf(S[0][1]);
    }
    float mt = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) max_slice(S[0], mt, i);
    update_reference(mt, true);
  }

  // Squared norms of the V rows of an owned tile (V ring buffer `buf`, stream entry e, unit `unit`): LPR lanes per
  // row, 16 bytes each (the swizzle permutes a row's pieces, the sum does not care), RPP rows per pass.
  auto vnorm_tile = [&](const Step& e, int buf, int unit) {
    constexpr int LPR = D / 8, RPP = 64 / LPR, NP = BK / RPP;
    const u32x4 un = units_c[2 * unit];
    const int kvh = (int)un[1] / a.G, rv = (int)((e.need >> 18) & 63u);
    const uint16_t* Vs = Vs_base + buf * (BK * D);
    float* const dst = a.vnorm2 + (size_t)kvh * a.N + e.k0;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    // sum over the LPR lanes of a row on the DPP path of the vector ALU (lane ^ 1, lane ^ 2, mirror of 8, mirror of
    // 16): the wavefront must be back at the tile barrier long before the others, a chain of LDS shuffles is not
    auto dpp_add = [](float x, auto ctrl) {
      return x + __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), decltype(ctrl)::value,
                                                                          0xf, 0xf, false));
    };
#pragma unroll 4
    for (int pass = 0; pass < NP; ++pass) {
      const int r = pass * RPP + ln / LPR;
      const u32x4 x = *reinterpret_cast<const u32x4*>(Vs + r * D + (ln % LPR) * 8);
      float ss = 0.f;
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const uint32_t word = x[wd];   // (a bit_cast applied directly to a vector element picks element 0 with this compiler)
        const bf16x2 pr = __builtin_bit_cast(bf16x2, word);
        ss = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ss, false);
      }
      ss = dpp_add(ss, std::integral_constant<int, 0xB1>{});    // quad_perm [1, 0, 3, 2]
      ss = dpp_add(ss, std::integral_constant<int, 0x4E>{});    // quad_perm [2, 3, 0, 1]
      ss = dpp_add(ss, std::integral_constant<int, 0x141>{});   // row_half_mirror: lane i <-> 7 - i of each 8
      if (LPR == 16) ss = dpp_add(ss, std::integral_constant<int, 0x140>{});   // row_mirror: lane i <-> 15 - i
      if ((ln % LPR) == 0 && r <= rv) dst[r] = ss;
    }
  };

  int bj = 1;   // ring buffer of tile j
  // One iteration; Sn receives the scores of tile j, Sp holds those of tile j-1.
  auto iteration = [&](int j, floatx16 (&Sn)[2], floatx16 (&Sp)[2]) {
    const bool have = j < t_end;
    const uint32_t nb = (have && active) ? (e_cur.need >> (2 * rb)) & 3u : 0u;
    const uint32_t kinds = (e_cur.kinds >> (4 * rb)) & 15u;
    const bool first = have && ((e_cur.need >> 17) & 1u);
    const bool lastp = (e_prev.need >> 16) & 1u;   // the unit of tile j-1 ends with it
    const int b_next = next_buf(bj), b_prev = next_buf(b_next);
    if (resc) {
      lacc[0] *= alpha;   // only element 0 is read back
      if (LSE) lx *= alpha;
#pragma unroll
      for (int b = 0; b < DBLK; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
      resc = false;
    }
    const float neg_m = (m == -INFINITY) ? 0.f : -m;   // m: reference after tile j-1, until this tile's maximum is in
    const int unit_prev = unit_id;   // unit of tile j-1
    if (first) {
      load_q_frags();   // frees the private tile, which the finished unit's rows leave through
      ++unit_id;
      q_pref = false;
      begin_qk_unit(un_next);
    }
    // Table entries for later tiles are requested before the barrier, which then also covers their latency:
    // scalar loads and LDS reads share a counter that cannot tell them apart, so a scalar load still pending
    // during a product would turn every wait for an operand fragment into a wait for everything.
    const Step e_f = fetch_step(j + 3);
    const u32x4 un_fetch = units_c[2 * (unit_id + 1)];   // the unit table ends with a spare record
    wait_loads();
    __syncthreads();
    // The loads of K(j+2) and V(j+1) are started between the MFMAs of the second product below (their address
    // arithmetic hides there); a wavefront without rows of its own starts them here.
    if (!active) {
      if (j + 2 < t_end) issue_k(e_n2, b_prev);
      if (j + 1 < t_end) issue_v(e_n1, b_next);
      // (only here: the same few lines inside the computing wavefronts' path cost them half their speed)
      if (VN) {
        if (((e_prev.need >> 24) & 1u) && wave == PUREKV_WAVES - 1) vnorm_tile(e_prev, b_prev, unit_prev);
      }
    }
    if (active) {
      // ---- score product of tile j, exponentials of tile j-1 ----
      constexpr int SPM = 8 / KSTEPS;   // slices per MFMA
      const uint16_t* Ks = Ks_base + bj * (BK * D);
      if (nb & 1u) {
        qk_half(Ks, Sn[0], [&](int i) {
#pragma unroll
          for (int q = 0; q < SPM; ++q) exp_slice(Sp, neg_m, SPM * i + q);
        });
      } else {
        fill_ninf(Sn[0]);
#pragma unroll
        for (int i = 0; i < 8; ++i) exp_slice(Sp, neg_m, i);
      }
      if (nb & 2u) {
        qk_half(Ks + 32 * D, Sn[1], [&](int i) {
#pragma unroll
          for (int q = 0; q < SPM; ++q) exp_slice(Sp, neg_m, 8 + SPM * i + q);
        });
      } else {
        fill_ninf(Sn[1]);
#pragma unroll
        for (int i = 0; i < 8; ++i) exp_slice(Sp, neg_m, 8 + i);
      }
      // ---- second product of tile j-1, running maximum of tile j ----
      if (nb & 1u) mask_block(Sn[0], kinds & 3u, e_cur.k0);
      if (nb & 2u) mask_block(Sn[1], (kinds >> 2) & 3u, e_cur.k0 + 32);
      float mt = -INFINITY;
      constexpr int MPM = 16 / (4 * DBLK);   // maximum slices per MFMA
      pv_tile(b_prev, pf, [&](int i) {
#pragma unroll
        for (int q = 0; q < MPM; ++q) max_slice(Sn, mt, MPM * i + q);
        if (i == 1 && j + 2 < t_end) issue_k(e_n2, b_prev);
        if (i == 3 && j + 1 < t_end) issue_v(e_n1, b_next);
      });
      update_reference(mt, first);
      if (lastp) {
        if (u_nsplits == 1) {
          finish_unit();
        } else {
          finish_slice();
          slice_arrive();
        }
        adopt_unit();
      }
    }
    maybe_prefetch_q(j, e_cur, e_n1, un_fetch);
    bj = b_next;
    e_prev = e_cur;
    e_cur = e_n1;
    e_n1 = e_n2;
    e_n2 = e_f;
  };
  for (int j = t_begin + 1;; j += 2) {
    iteration(j, S[1], S[0]);
    if (j == t_end) break;
    iteration(j + 1, S[0], S[1]);
    if (j + 1 == t_end) break;
  }
  // split lists whose slices this workgroup ran: combine those that are complete and still uncombined
  if (active) {
    const int u_end = a.queue_unit0[blockIdx.x + 1];
    for (int u = a.queue_unit0[blockIdx.x]; u < u_end; ++u) {
      const u32x4 un = units_c[2 * u];
      if ((int)un[2] > 1) {
        CombineCall cc;
        cc.counters = a.counters;
        cc.ws_o = a.ws_o;
        cc.ws_lse = a.ws_lse;
        cc.out = a.out;
        cc.lse = a.lse;
        cc.xs = (LdsFloat*)reinterpret_cast<float*>(Xs);
        cc.o_head_bytes = a.o_head_bytes;
        cc.o_row_bytes = a.o_row_bytes;
        cc.N = a.N;
        cc.n_groups = a.n_groups;
        cc.wave = wave;
        cc.hl = hl;
        cc.rb = rb;
        cc.lse_row0 = a.lse_row0;
        combine_slices<D, LSE>(cc, un, units_c[2 * u + 1]);
      }
    }
  }
}

template <int D, bool ST, bool LSE, bool VN>
__global__ __launch_bounds__(512, 1) void prefill_kernel(const PrefillArgs a) {
  prefill_body<D, ST, LSE, VN>(a);
}

// Window plans with the log-sum-exp asked for: the workgroups before lse_queue0 run no unit that wants it and take
// the loop without the exact row sum (7-10 % faster), the others the loop with it.  Two copies of the loop in one
// kernel; written with the early return, the first copy comes out of the compiler as it does alone (with a plain
// if / else it ran 2.5 % slower).
template <int D, bool ST>
__global__ __launch_bounds__(512, 1) void prefill_window_kernel(const PrefillArgs a) {
  if (__builtin_expect((int)blockIdx.x < a.lse_queue0, 1)) {
    prefill_body<D, ST, false, false>(a);
    return;
  }
  prefill_body<D, ST, true, false>(a);
}

// Clears the arrival counters of a prefill workspace (a kernel, not a memset: callers may be capturing a graph).
__global__ void clear_counters_kernel(int32_t* c, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) c[i] = 0;
}

template <int D, bool ST, bool LSE, bool VN>
hipError_t launch_one(const PrefillArgs& a, dim3 grid, hipStream_t st) {
  // 3 K buffers + 3 V buffers + one private tile per wavefront
  constexpr unsigned lds_bytes = (6u * BK * D + PUREKV_WAVES * kXTile) * sizeof(uint16_t);
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kernel<D, ST, LSE, VN>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((prefill_kernel<D, ST, LSE, VN>), grid, dim3(512), lds_bytes, st, a);
  return hipSuccess;
}

template <int D, bool ST>
hipError_t launch_window(const PrefillArgs& a, dim3 grid, hipStream_t st) {
  constexpr unsigned lds_bytes = (6u * BK * D + PUREKV_WAVES * kXTile) * sizeof(uint16_t);
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_window_kernel<D, ST>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((prefill_window_kernel<D, ST>), grid, dim3(512), lds_bytes, st, a);
  return hipSuccess;
}

template <int D, bool ST>
hipError_t launch_variant(const PrefillArgs& a, dim3 grid, hipStream_t st) {
  // a window plan whose log-sum-exp is wanted: the divided kernel (the V norms, if wanted too, come from their own pass)
  if (a.lse != nullptr && a.lse_queue0 > 0) return launch_window<D, ST>(a, grid, st);
  if (a.vnorm2 != nullptr && a.Gs * a.R < PUREKV_WAVES)
    return a.lse != nullptr ? launch_one<D, ST, true, true>(a, grid, st) : launch_one<D, ST, false, true>(a, grid, st);
  return a.lse != nullptr ? launch_one<D, ST, true, false>(a, grid, st) : launch_one<D, ST, false, false>(a, grid, st);
}

}  // namespace

// Workspace of a plan with split lists: [arrival counters, padded to 256 bytes][partial outputs][their log-sum-exps].
static size_t prefill_counter_count(const purekv_plan& p) { return (size_t)p.n_slots * p.g.n_groups * PUREKV_WAVES; }
static size_t prefill_counter_bytes(const purekv_plan& p) {
  return (prefill_counter_count(p) * sizeof(int32_t) + 255) / 256 * 256;
}
size_t prefill_counter_region_bytes(const purekv_plan& p) { return prefill_counter_bytes(p); }

size_t prefill_ws_bytes(const purekv_plan& p) {
  if (p.n_slots == 0) return 0;
  return prefill_counter_bytes(p) + (size_t)p.n_slots * p.g.n_groups * WG_ROWS * (p.g.d + 2) * sizeof(float);
}

int launch_prefill_ws_init(const purekv_plan& p, void* ws, hipStream_t st) {
  const int n = (int)prefill_counter_count(p);
  if (n == 0) return PUREKV_OK;
  hipLaunchKernelGGL(clear_counters_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, static_cast<int32_t*>(ws), n);
  PUREKV_HIP_TRY(hipGetLastError());
  return PUREKV_OK;
}

int launch_prefill(const purekv_plan& p, const void* q, const void* k, const void* v, void* out, float* lse,
                   float* vnorm2, void* ws, hipStream_t st) {
  PrefillArgs a{};
  a.vnorm2 = vnorm2;
  a.G = p.g.G;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.out = static_cast<uint16_t*>(out);
  a.lse = lse;
  a.counters = static_cast<int32_t*>(ws);
  a.ws_o = ws ? reinterpret_cast<float*>(static_cast<char*>(ws) + prefill_counter_bytes(p)) : nullptr;
  a.ws_lse = a.ws_o ? a.ws_o + (size_t)p.n_slots * p.g.n_groups * WG_ROWS * p.g.d : nullptr;
  a.stream = p.d_stream;
  a.units = p.d_units;
  a.queue_begin = p.d_queue_begin;
  a.queue_unit0 = p.d_queue_unit0;
  a.N = p.g.N;
  a.Nv = p.g.Nv;
  a.P = p.g.P;
  a.Hq = p.g.Hq;
  a.Hkv = p.g.Hkv;
  a.q_head_bytes = p.g.q_sh * 2;
  a.o_head_bytes = p.g.o_sh * 2;
  a.q_row_bytes = (uint32_t)(p.g.q_st * 2);
  a.kv_row_bytes = (uint32_t)(p.g.kv_st * 2);
  a.o_row_bytes = (uint32_t)(p.g.o_st * 2);
  a.Gs = p.g.Gs;
  a.R = p.g.R;
  a.n_groups = p.g.n_groups;
  a.pattern = p.g.pattern;
  a.scale_log2 = p.g.scale * kLog2e;
  a.lse_row0 = p.lse_rows > 0 ? std::max(0, p.g.N - p.lse_rows) : 0;
  a.lse_queue0 = p.lse_queue0;
  const bool window_launch = lse != nullptr && p.lse_queue0 > 0;
  if (window_launch) a.vnorm2 = nullptr;
  const dim3 grid((unsigned)p.n_queues);
  const bool sparse = p.g.pattern != PUREKV_PATTERN_DENSE;
  if (p.g.d == 128) {
    if (sparse)
      PUREKV_HIP_TRY((launch_variant<128, true>(a, grid, st)));
    else
      PUREKV_HIP_TRY((launch_variant<128, false>(a, grid, st)));
  } else {
    if (sparse)
      PUREKV_HIP_TRY((launch_variant<64, true>(a, grid, st)));
    else
      PUREKV_HIP_TRY((launch_variant<64, false>(a, grid, st)));
  }
  PUREKV_HIP_TRY(hipGetLastError());
  // every wavefront of this plan's workgroups has rows: the norms come from a stream over V of their own
  if (vnorm2 != nullptr && (p.g.Gs * p.g.R >= PUREKV_WAVES || window_launch)) return launch_vnorm2(p, v, vnorm2, st);
  return PUREKV_OK;
}

}  // namespace purekv
