// Shared device helpers and host-side plumbing of librtp (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>

#include "../../include/rtp.h"

namespace rtp {

constexpr int kHeadDim = RTP_HEAD_DIM;    // 128
constexpr int kIndexDim = RTP_INDEX_DIM;  // 16
constexpr int kWave = 64;                 // CDNA wavefront

// ---- host side -----------------------------------------------------------------------------
// Records a printf-style message for rtp_last_error() and returns `code`.
int32_t fail(int32_t code, const char* fmt, ...);
void clear_error();
// Checks a layer descriptor; fills group size and per-head role table (1 = retrieval).
int32_t check_layer(const rtp_layer_desc* L, const char* who);
// hipGetLastError() after launches -> RTP_ERR_HIP with the HIP text, or RTP_OK.
int32_t check_launch(const char* who);
inline float softmax_scale_of(const rtp_layer_desc* L) {
  return L->softmax_scale != 0.f ? L->softmax_scale : 0.08838834764831845f;  // 1/sqrt(128)
}
inline float index_scale_of(const rtp_layer_desc* L) { return L->index_scale != 0.f ? L->index_scale : 1.f; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Per-launch timing (rtp_profile_start / rtp_profile_stop): while it is on, every kernel launch of the library
// carries a start and a stop event that the runtime stamps with the dispatch's own begin and end times (the
// clocks a profiler reads), so the figures are kernel durations, not enqueue-to-enqueue gaps.  Off (the default) a
// launch costs one load of a flag more.
bool profile_slot(const char* kernel, hipEvent_t* start, hipEvent_t* stop);
#define RTP_LAUNCH(kernel, grid, block, shmem, stream, ...)                                                  \
  do {                                                                                                       \
    hipEvent_t rtp_e0_ = nullptr, rtp_e1_ = nullptr;                                                         \
    if (rtp::profile_slot(#kernel, &rtp_e0_, &rtp_e1_))                                                      \
      hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, rtp_e0_, rtp_e1_, 0, __VA_ARGS__);          \
    else                                                                                                     \
      hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                   \
  } while (0)

// Head-role tables passed to kernels by value (n_q_heads <= 128).
struct HeadTable {
  int32_t n_ret;
  int32_t ret_heads[64];     // retrieval query-head ids, ascending
  uint8_t is_ret[128];       // per query head
};
int32_t fill_head_table(const rtp_layer_desc* L, HeadTable* t, const char* who);

// ---- device side ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// The attention tensors come in one of two 16-bit formats (F16 = IEEE binary16, else bf16): the halves of a
// 32-bit word as floats, and fp32 rounded to the format (nearest even).
template <bool F16> __device__ __forceinline__ float lo16(uint32_t u) {
  if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu));
  else return bf16_lo(u);
}
template <bool F16> __device__ __forceinline__ float hi16(uint32_t u) {
  if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16));
  else return bf16_hi(u);
}

// fp32 -> bf16 round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint16_t f32_to_f16_rne(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }
// by a run-time flag (merge launches: one conversion per output element)
__device__ __forceinline__ uint16_t f32_to_16(float x, bool f16) { return f16 ? f32_to_f16_rne(x) : f32_to_bf16_rne(x); }

// fp64 -> bf16 round-to-nearest-even in ONE rounding step (normal range; tiny values flush to 0,
// huge ones saturate to the largest finite bf16).
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
  uint64_t u = (uint64_t)__double_as_longlong(x);
  uint32_t sign = (uint32_t)(u >> 48) & 0x8000u;
  int32_t e = (int32_t)((u >> 52) & 0x7ff) - 1023 + 127;
  if (e <= 0) return (uint16_t)sign;
  if (e >= 255) return (uint16_t)(sign | 0x7f7fu);
  uint64_t man = u & 0xfffffffffffffull;           // 52 bits
  uint32_t keep = (uint32_t)(man >> 45);           // top 7 bits
  uint64_t rest = man & ((1ull << 45) - 1);
  uint32_t r = ((uint32_t)e << 7) | keep;          // exponent|mantissa; a carry ripples into e
  const uint64_t half = 1ull << 44;
  if (rest > half || (rest == half && (keep & 1u))) r += 1;
  if (r >= (255u << 7)) r = 0x7f7fu;
  return (uint16_t)(sign | r);
}

// Order-preserving map fp32 -> uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t float_key(float s) {
  uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, true));  // row_half_mirror
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, true));  // row_mirror
  return x;
}
// Sum of a lane and its xor-1 neighbour.
__device__ __forceinline__ float pair_sum(float x) {
  return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- wave-wide inclusive prefix sums on the DPP data path ------------------------------------------
// Four shifts inside the 16-lane rows, then lane 15 of rows 0 and 2 into rows 1 and 3 (row_bcast:15) and
// lane 31 into the upper half (row_bcast:31): six dependent vector-ALU steps, where a shuffle-based scan
// makes six round trips through the LDS crossbar.  A lane without a source (and a row the mask leaves
// out) receives 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_or_zero(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, false); }

#define RTP_WAVE_SCAN_STEPS(STEP) \
  STEP(0x111, 0xf) STEP(0x112, 0xf) STEP(0x114, 0xf) STEP(0x118, 0xf) STEP(0x142, 0xa) STEP(0x143, 0xc)

__device__ __forceinline__ int wave_incl_scan(int x) {
#define RTP_STEP(CTRL, MASK) x += dpp_or_zero<CTRL, MASK>(x);
  RTP_WAVE_SCAN_STEPS(RTP_STEP)
#undef RTP_STEP
  return x;
}
__device__ __forceinline__ uint64_t wave_incl_scan(uint64_t x) {
#define RTP_STEP(CTRL, MASK)                                                                   \
  x += ((uint64_t)(uint32_t)dpp_or_zero<CTRL, MASK>((int)(uint32_t)(x >> 32)) << 32) |        \
       (uint64_t)(uint32_t)dpp_or_zero<CTRL, MASK>((int)(uint32_t)x);
  RTP_WAVE_SCAN_STEPS(RTP_STEP)
#undef RTP_STEP
  return x;
}
__device__ __forceinline__ double wave_incl_scan(double x) {
#define RTP_STEP(CTRL, MASK)                                                                   \
  {                                                                                            \
    const uint64_t b = (uint64_t)__double_as_longlong(x);                                      \
    const uint64_t t = ((uint64_t)(uint32_t)dpp_or_zero<CTRL, MASK>((int)(uint32_t)(b >> 32)) << 32) | \
                       (uint64_t)(uint32_t)dpp_or_zero<CTRL, MASK>((int)(uint32_t)b);          \
    x += __longlong_as_double((long long)t);                                                   \
  }
  RTP_WAVE_SCAN_STEPS(RTP_STEP)
#undef RTP_STEP
  return x;
}
// The value of lane 63 in every lane (a scalar register): the wave total after an inclusive scan.
__device__ __forceinline__ int wave_last(int x) { return __builtin_amdgcn_readlane(x, 63); }
// Wave-wide sum / maximum of non-negative-or-(-1) ints, in every lane.
__device__ __forceinline__ int wave_sum(int x) { return wave_last(wave_incl_scan(x)); }
// max(a, b) of two values that are never NaN, as ONE vector instruction (the median of a, b and +inf).  fmaxf()
// has to quiet signalling NaNs, which costs a canonicalising instruction for every operand the compiler cannot
// prove quiet -- matrix-core results, cross-lane moves -- i.e. three instructions per maximum in such places.
// (+inf comes out of an assembly statement: given the constant, the compiler turns the median back into a maximum.)
__device__ __forceinline__ float max_nn(float a, float b) {
  float pinf;
  asm("s_mov_b32 %0, 0x7f800000" : "=s"(pinf));
  return __builtin_amdgcn_fmed3f(a, b, pinf);
}

// Wave-wide maximum of floats, in every lane (same six steps; a lane without a source takes -inf).
__device__ __forceinline__ float wave_max_f32(float x) {
  const int ninf_bits = 0xff800000;
#define RTP_STEP(CTRL, MASK) x = max_nn(x, __int_as_float(__builtin_amdgcn_update_dpp(ninf_bits, __float_as_int(x), CTRL, MASK, 0xf, false)));
  RTP_WAVE_SCAN_STEPS(RTP_STEP)
#undef RTP_STEP
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ int wave_max_ge_m1(int x) {      // x >= -1 in every lane
#define RTP_STEP(CTRL, MASK) x = max(x, __builtin_amdgcn_update_dpp(-1, x, CTRL, MASK, 0xf, false));
  RTP_WAVE_SCAN_STEPS(RTP_STEP)
#undef RTP_STEP
  return wave_last(x);
}

}  // namespace rtp
