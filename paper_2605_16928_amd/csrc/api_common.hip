// Host-side plumbing shared by every entry point: error text, descriptor checks.
#include "common.h"

#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>

namespace rtp {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = 0; }

int32_t check_layer(const rtp_layer_desc* L, const char* who) {
  if (!L) return fail(RTP_ERR_INVALID_ARG, "%s: layer descriptor is NULL", who);
  if (L->head_dim != kHeadDim)
    return fail(RTP_ERR_UNSUPPORTED, "%s: head_dim %d unsupported (must be 128)", who, L->head_dim);
  if (L->index_dim != kIndexDim)
    return fail(RTP_ERR_UNSUPPORTED, "%s: index_dim %d unsupported (must be 16)", who, L->index_dim);
  if (L->n_q_heads <= 0 || L->n_kv_heads <= 0 || L->n_q_heads > 128)
    return fail(RTP_ERR_INVALID_ARG, "%s: head counts %d/%d out of range", who, L->n_q_heads, L->n_kv_heads);
  if (L->n_q_heads % L->n_kv_heads != 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, L->n_q_heads,
                L->n_kv_heads);
  int g = L->n_q_heads / L->n_kv_heads;
  if (g != 1 && g != 2 && g != 4 && g != 8)
    return fail(RTP_ERR_UNSUPPORTED, "%s: GQA group size %d unsupported (1, 2, 4 or 8)", who, g);
  if (L->n_ret < 0 || L->n_ret > 64 || L->n_ret > L->n_q_heads)
    return fail(RTP_ERR_INVALID_ARG, "%s: n_ret %d out of range", who, L->n_ret);
  if (L->n_ret > 0 && !L->ret_heads) return fail(RTP_ERR_INVALID_ARG, "%s: ret_heads is NULL", who);
  for (int j = 0; j < L->n_ret; ++j) {
    int h = L->ret_heads[j];
    if (h < 0 || h >= L->n_q_heads)
      return fail(RTP_ERR_INVALID_ARG, "%s: ret_heads[%d] = %d out of range", who, j, h);
    if (j > 0 && h <= L->ret_heads[j - 1])
      return fail(RTP_ERR_INVALID_ARG, "%s: ret_heads must be strictly ascending", who);
  }
  if (L->sink < 0 || L->window < 0 || (int64_t)L->sink + L->window <= 0)
    return fail(RTP_ERR_INVALID_ARG, "%s: sink %d / window %d invalid", who, L->sink, L->window);
  if (L->kv_dtype != RTP_DTYPE_BF16 && L->kv_dtype != RTP_DTYPE_FP16)
    return fail(RTP_ERR_UNSUPPORTED, "%s: kv_dtype %d unsupported (RTP_DTYPE_BF16 or RTP_DTYPE_FP16)", who, L->kv_dtype);
  if (!(L->softmax_scale >= 0.f) || !(L->index_scale >= 0.f))
    return fail(RTP_ERR_INVALID_ARG, "%s: scales must be >= 0 (0 selects the default)", who);
  return RTP_OK;
}

int32_t fill_head_table(const rtp_layer_desc* L, HeadTable* t, const char* who) {
  int32_t rc = check_layer(L, who);
  if (rc != RTP_OK) return rc;
  memset(t, 0, sizeof(*t));
  t->n_ret = L->n_ret;
  for (int j = 0; j < L->n_ret; ++j) {
    t->ret_heads[j] = L->ret_heads[j];
    t->is_ret[L->ret_heads[j]] = 1;
  }
  return RTP_OK;
}

int32_t check_launch(const char* who) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(RTP_ERR_HIP, "%s: launch failed: %s", who, hipGetErrorString(e));
  return RTP_OK;
}

// ---- per-launch timing ---------------------------------------------------------------------------------
namespace {
struct ProfileState {
  std::mutex mu;
  std::atomic<bool> on{false};
  int cap = 0, n = 0, dropped = 0;
  hipEvent_t* ev = nullptr;          // 2 * cap events: start, stop of launch i
  const char** name = nullptr;
} g_prof;
}  // namespace

bool profile_slot(const char* kernel, hipEvent_t* start, hipEvent_t* stop) {
  if (!g_prof.on.load(std::memory_order_relaxed)) return false;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (!g_prof.on.load()) return false;
  if (g_prof.n >= g_prof.cap) { ++g_prof.dropped; return false; }
  const int slot = g_prof.n++;
  g_prof.name[slot] = kernel;
  *start = g_prof.ev[2 * slot];
  *stop = g_prof.ev[2 * slot + 1];
  return true;
}

}  // namespace rtp

extern "C" int32_t rtp_profile_start(int32_t max_launches) {
  using namespace rtp;
  if (max_launches <= 0 || max_launches > (1 << 20))
    return fail(RTP_ERR_INVALID_ARG, "rtp_profile_start: max_launches must be in [1, 2^20]");
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (g_prof.on.load()) return fail(RTP_ERR_INVALID_ARG, "rtp_profile_start: already recording");
  g_prof.ev = (hipEvent_t*)calloc((size_t)2 * max_launches, sizeof(hipEvent_t));
  g_prof.name = (const char**)calloc((size_t)max_launches, sizeof(const char*));
  if (!g_prof.ev || !g_prof.name) return fail(RTP_ERR_INVALID_ARG, "rtp_profile_start: out of host memory");
  for (int i = 0; i < 2 * max_launches; ++i) {
    const hipError_t e = hipEventCreate(&g_prof.ev[i]);
    if (e != hipSuccess) return fail(RTP_ERR_HIP, "rtp_profile_start: hipEventCreate failed: %s", hipGetErrorString(e));
  }
  g_prof.cap = max_launches;
  g_prof.n = 0;
  g_prof.dropped = 0;
  clear_error();
  g_prof.on.store(true);
  return RTP_OK;
}

extern "C" int32_t rtp_profile_stop(rtp_launch_time* out, int32_t out_cap, int32_t* n_out) {
  using namespace rtp;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (!g_prof.on.load()) return fail(RTP_ERR_INVALID_ARG, "rtp_profile_stop: not recording");
  g_prof.on.store(false);
  int n = 0;
  int32_t rc = RTP_OK;
  for (int i = 0; i < g_prof.n; ++i) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(g_prof.ev[2 * i + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
    if (e != hipSuccess) { rc = fail(RTP_ERR_HIP, "rtp_profile_stop: %s", hipGetErrorString(e)); break; }
    if (out && n < out_cap) { out[n].kernel = g_prof.name[i]; out[n].us = ms * 1e3f; ++n; }
  }
  for (int i = 0; i < 2 * g_prof.cap; ++i) (void)hipEventDestroy(g_prof.ev[i]);
  free(g_prof.ev);
  free(g_prof.name);
  g_prof.ev = nullptr;
  g_prof.name = nullptr;
  if (n_out) *n_out = rc == RTP_OK ? n : 0;
  if (rc == RTP_OK) clear_error();
  return rc;
}

extern "C" const char* rtp_last_error(void) { return rtp::g_err; }
extern "C" const char* rtp_version(void) { return "rtp-gfx950 0.1"; }
