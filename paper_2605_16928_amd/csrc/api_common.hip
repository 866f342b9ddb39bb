// Host-side plumbing shared by every entry point: error text, descriptor checks.
#include "common.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

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

}  // namespace rtp

extern "C" const char* rtp_last_error(void) { return rtp::g_err; }
extern "C" const char* rtp_version(void) { return "rtp-gfx950 0.1"; }
