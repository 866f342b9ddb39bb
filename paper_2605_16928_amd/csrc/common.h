// Shared device helpers and host-side plumbing of librtp (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

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

// fp32 -> bf16 round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

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

}  // namespace rtp
