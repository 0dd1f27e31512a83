// Internal helpers shared by the HIP translation units (device-side types, error plumbing).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan.h"

namespace purekv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (inputs are finite here).
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));  // v_cvt_pk_bf16_f32, nearest even
}

// Value held by the lane 32 positions away (the other half of the wavefront).
// v_permlane32_swap exchanges the two halves in the vector ALU (no LDS traffic, unlike ds_bpermute).
__device__ __forceinline__ float other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  // r[0]: lanes 0-31 keep their own value and lanes 32-63 receive lanes 0-31's; r[1] the converse
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// Row-major bf16 tile of D columns in LDS (K tiles, query tiles): element offset of 16-byte slot `u` of row `r`.  The slot index is XOR-ed with the
// row so that the 16 lanes the LDS serves together (rows that differ in their low four bits) fall into 16
// different 16-byte slots of a 256-byte bank period.
template <int D>
__device__ __forceinline__ int kswz(int r, int u) {
  if constexpr (D == 128) {
    return r * 128 + ((u ^ (r & 15)) * 8);
  } else {  // 64 elements = 128 bytes: two rows share one 256-byte period
    return (r >> 1) * 128 + ((((r & 1) * 8 + u) ^ ((r >> 1) & 15)) * 8);
  }
}
// Inverse: 16-byte position p of the tile -> (row, slot) stored there.
template <int D>
__device__ __forceinline__ void kunswz(int p, int& r, int& u) {
  if constexpr (D == 128) {
    r = p >> 4;
    u = (p & 15) ^ (r & 15);
  } else {
    const int rr = p >> 4, y = (p & 15) ^ (rr & 15);
    r = 2 * rr + (y >> 3);
    u = y & 7;
  }
}
// Global memory straight into LDS, 16 or 4 bytes per lane: lane l's piece lands at lds_ptr + 16 l (4 l), its source
// is base + off (a 32-bit byte offset per lane).  Written as assembly so that every wait for these loads is the
// kernel's own: the compiler does not know which LDS buffer a load of the builtin form fills and would wait for ALL
// outstanding ones, the loads just issued for later tiles included, before any LDS read.  base and lds_ptr must be
// wave-uniform.  The LDS address travels in m0, which the statement overwrites (declared, so that the compiler
// keeps nothing live in it across the load).
typedef __attribute__((address_space(3))) void* LdsPtr;
__device__ __forceinline__ void load_to_lds_16(const void* base, uint32_t off, const void* lds_ptr) {
  const uint32_t lds_base = (uint32_t)(size_t)(LdsPtr)lds_ptr;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(off), "s"(base)
               : "memory", "m0");
}
__device__ __forceinline__ void load_to_lds_4(const void* base, uint32_t off, const void* lds_ptr) {
  const uint32_t lds_base = (uint32_t)(size_t)(LdsPtr)lds_ptr;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_base), "v"(off), "s"(base)
               : "memory", "m0");
}

// Records a failed HIP call for purekv_strerror and maps it to PUREKV_EHIP.
int note_hip_error(hipError_t e);

#define PUREKV_HIP_TRY(expr)                                \
  do {                                                      \
    hipError_t e__ = (expr);                                \
    if (e__ != hipSuccess) return purekv::note_hip_error(e__); \
  } while (0)

// Kernel launchers (one per translation unit); all arguments validated by the caller.
int launch_prefill(const purekv_plan& p, const void* q, const void* k, const void* v, void* out, float* lse,
                   float* vnorm2, void* ws, hipStream_t st);
int launch_importance(const purekv_plan& p, const void* q, const void* k, const float* lse, int32_t w,
                      float* c_out, hipStream_t st);
int launch_topk(const purekv_plan& p, const float* c, const void* v, int64_t v_layer_stride, int32_t n_layers,
                int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws, hipStream_t st);
// vnorm2[kv, j] = sum_c v[kv, j, c]^2 for all N keys, as a pass of its own over V
int launch_vnorm2(const purekv_plan& p, const void* v, float* vnorm2, hipStream_t st);
// the same with the squared norms of the V rows ([n_layers][Hkv, N] fp32, as the prefill emits them) instead of V
int launch_topk_norms(const purekv_plan& p, const float* c, const float* vnorm2, int64_t vn_layer_stride,
                      int32_t n_layers, int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws, hipStream_t st);
// Library-owned score buffer of the current device (looked up once per device) and its capacity in floats.
int static_score_buffer(int device, float** out);
size_t topk_static_capacity_floats();
int launch_compact(const purekv_plan& p, const void* k, const void* v, int64_t kv_layer_stride, int32_t n_layers,
                   const int32_t* idx, int32_t n_keep, void* kc, void* vc, int32_t cap, hipStream_t st);
int launch_append(const purekv_plan& p, const void* k_new, const void* v_new, void* kc, void* vc, int32_t n_cached,
                  int32_t cap, hipStream_t st);
// k_new, v_new null: attention only; else row n_cached - 1 comes from them and is stored into kc, vc
int launch_decode(const purekv_plan& p, const void* q_new, const void* k_new, const void* v_new, void* kc, void* vc,
                  int32_t n_cached, int32_t cap, void* out, void* ws, hipStream_t st);

int launch_calib_mfma(const purekv_plan& p, int mix, int random_operands, int32_t iters, float* sink, uint64_t* ticks,
                      hipStream_t st);
double calib_mfma_flops(const purekv_plan& p, int32_t iters);
int launch_calib_step(const purekv_plan& p, int rows_per_wavefront, int32_t iters, const void* src, float* sink,
                      uint64_t* ticks, hipStream_t st);
double calib_step_flops(const purekv_plan& p, int32_t iters);

size_t prefill_ws_bytes(const purekv_plan& p);
// Arrival counters lead the prefill and decode workspaces: zero whenever no call is running on the workspace.
size_t prefill_counter_region_bytes(const purekv_plan& p);
int launch_spearman(const float* s_hat, const float* s, int32_t n_rows, int32_t n_keys, uint64_t* sum_d2, double* rho,
                    hipStream_t st);
int launch_prefill_ws_init(const purekv_plan& p, void* ws, hipStream_t st);
int launch_decode_ws_init(const purekv_plan& p, void* ws, hipStream_t st);
size_t topk_ws_bytes(const purekv_plan& p, int32_t n_layers, int32_t w);
size_t decode_ws_bytes(const purekv_plan& p, int32_t cap);

}  // namespace purekv
