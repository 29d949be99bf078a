// Entry points of the gated FFN's first step (gate and up projection as one GEMM).
#include <algorithm>
#include <cstdint>

#include "internal.h"

using namespace spd;

static int ffn_shape_check(int32_t hidden, int32_t inter) {
  // slices of 32 hidden entries; tiles of 128 outputs (256 joint columns)
  if (hidden <= 0 || inter <= 0 || hidden % 32 || inter % 128) return SPD_EINVAL;
  if ((int64_t)hidden * 2 * 255 > INT32_MAX) return SPD_EINVAL;   // per-lane row offsets are 32-bit
  return SPD_OK;
}

extern "C" int spd_ffn_pack_gate_up(spd_ctx* ctx, int phase, const void* w_gate, const void* w_up, void* w_gu, int32_t hidden,
                                    int32_t inter) {
  if (!ctx || (phase != SPD_PHASE_PREFILL && phase != SPD_PHASE_DECODE)) return SPD_EINVAL;
  int rc = ffn_shape_check(hidden, inter);
  if (rc != SPD_OK) return rc;
  if (!w_gate || !w_up || !w_gu || (((uintptr_t)w_gate | (uintptr_t)w_up | (uintptr_t)w_gu) & 15)) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  hipStream_t stream;
  if ((rc = phase_enter(ctx, phase, &stream)) != SPD_OK) return rc;
  SPD_HIP(launch_ffn_pack(w_gate, w_up, w_gu, hidden, inter, stream));
  return SPD_OK;
}

extern "C" int spd_ffn_gate_up(spd_ctx* ctx, int phase, const void* x, const void* w_gu, void* out, int32_t n_tokens,
                               int32_t hidden, int32_t inter) {
  if (!ctx || (phase != SPD_PHASE_PREFILL && phase != SPD_PHASE_DECODE)) return SPD_EINVAL;
  int rc = ffn_shape_check(hidden, inter);
  if (rc != SPD_OK) return rc;
  if (n_tokens < 0) return SPD_EINVAL;
  if (n_tokens > 0 && (!x || !w_gu || !out || (((uintptr_t)x | (uintptr_t)w_gu) & 15) || ((uintptr_t)out & 1))) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  if (n_tokens == 0) return SPD_OK;
  hipStream_t stream;
  if ((rc = phase_enter(ctx, phase, &stream)) != SPD_OK) return rc;
  if ((rc = kernel_timing_mark(ctx, phase, 0, stream)) != SPD_OK) return rc;
  SPD_HIP(launch_ffn_gate_up(x, w_gu, out, n_tokens, hidden, inter, ctx->xcds, std::max(1, ctx->phase[phase].active_cus), stream));
  return kernel_timing_mark(ctx, phase, 1, stream);
}
