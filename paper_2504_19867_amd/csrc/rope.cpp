// Host side of the rotary-embedding step: argument checks, the frequency table, staging, launch.
//
// Paper, Evaluation, "Implementation based on DistServe": a RoPE kernel modified for Llama-3.1 runs
// before the attention step.  The frequency table is the published definition: w_i = theta^(-2i/R),
// and with factor != 1 the Llama-3.1 rule on the wavelength 2 pi / w_i (unchanged below
// original_max_pos / high_freq_factor, divided by factor above original_max_pos / low_freq_factor,
// a linear blend of the two in between).
#include <cmath>
#include <cstring>

#include "internal.h"

using namespace spd;

namespace spd {
int rope_config_check(const spd_rope_config* c) {
  if (!c) return SPD_EINVAL;
  if (!(c->theta > 0.0) || !std::isfinite(c->theta) || !(c->factor >= 1.0) || !std::isfinite(c->factor)) return SPD_EINVAL;
  if (c->rotary_dim <= 0 || c->rotary_dim % 2 || c->rotary_offset < 0) return SPD_EINVAL;
  if (c->factor != 1.0) {
    if (!(c->low_freq_factor > 0.0) || !(c->high_freq_factor > c->low_freq_factor) || c->original_max_pos <= 0) return SPD_EINVAL;
  }
  return SPD_OK;
}

void rope_frequencies(const spd_rope_config* c, double* out) {
  const double two_pi = 6.283185307179586476925286766559;
  for (int i = 0; i < c->rotary_dim / 2; ++i) {
    double w = std::pow(c->theta, -2.0 * i / c->rotary_dim);
    if (c->factor != 1.0) {
      const double wavelen = two_pi / w;
      if (wavelen < c->original_max_pos / c->high_freq_factor) {
        // high frequency: as it is
      } else if (wavelen > c->original_max_pos / c->low_freq_factor) {
        w = w / c->factor;
      } else {
        const double s = (c->original_max_pos / wavelen - c->low_freq_factor) / (c->high_freq_factor - c->low_freq_factor);
        w = (1.0 - s) * w / c->factor + s * w;
      }
    }
    out[i] = w;
  }
}
}  // namespace spd

extern "C" int spd_rope_inv_freq(const spd_rope_config* cfg, double* out, int32_t cap) {
  const int rc = rope_config_check(cfg);
  if (rc != SPD_OK) return rc;
  if (!out || cap < cfg->rotary_dim / 2) return SPD_EINVAL;
  rope_frequencies(cfg, out);
  return SPD_OK;
}

extern "C" int spd_rope_qk(spd_ctx* ctx, int phase, const spd_rope_config* cfg, const int32_t* positions, int32_t n_tokens,
                           void* q, int32_t n_q_heads, void* k, int32_t n_kv_heads, int32_t dim) {
  if (!ctx || (phase != SPD_PHASE_PREFILL && phase != SPD_PHASE_DECODE)) return SPD_EINVAL;
  const int rc = rope_config_check(cfg);
  if (rc != SPD_OK) return rc;
  if (n_tokens < 0 || (n_tokens > 0 && !positions)) return SPD_EINVAL;
  if (!q && !k) return SPD_EINVAL;
  if ((q && n_q_heads <= 0) || (k && n_kv_heads <= 0) || dim <= 0) return SPD_EINVAL;
  // the kernel moves 16-byte pieces of 8 entries: rows, the rotating range and its halves start on such pieces
  if (dim % 8 || cfg->rotary_dim % 16 || cfg->rotary_offset % 8 || cfg->rotary_offset + cfg->rotary_dim > dim) return SPD_EINVAL;
  if (((uintptr_t)q | (uintptr_t)k) & 15) return SPD_EINVAL;
  for (int32_t t = 0; t < n_tokens; ++t)
    if (positions[t] < 0) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  if (n_tokens == 0) return SPD_OK;

  hipStream_t stream;
  int st_rc = phase_enter(ctx, phase, &stream);
  if (st_rc != SPD_OK) return st_rc;
  const int half = cfg->rotary_dim / 2;
  const size_t w_bytes = (size_t)half * sizeof(double), p_bytes = (size_t)n_tokens * sizeof(int32_t);
  spd_stage* st = nullptr;
  st_rc = stage_acquire(ctx, phase, w_bytes + p_bytes, &st);
  if (st_rc != SPD_OK) return st_rc;
  rope_frequencies(cfg, (double*)st->host);
  std::memcpy(st->host + w_bytes, positions, p_bytes);
  void* host_dev = nullptr;
  st_rc = stage_host_as_device(st, &host_dev);
  if (st_rc != SPD_OK) return st_rc;
  // the kernel reads the table and the positions straight out of the pinned buffer
  const void* qq = q ? q : k;
  const int hq = q ? n_q_heads : n_kv_heads;
  st_rc = kernel_timing_mark(ctx, phase, 0, stream);
  if (st_rc != SPD_OK) return st_rc;
  SPD_HIP(launch_rope((void*)qq, hq, q ? k : nullptr, n_kv_heads, dim, cfg->rotary_dim, cfg->rotary_offset, cfg->interleaved != 0,
                      n_tokens, (const int32_t*)((const char*)host_dev + w_bytes), (const double*)host_dev, stream));
  st_rc = kernel_timing_mark(ctx, phase, 1, stream);
  if (st_rc != SPD_OK) return st_rc;
  return stage_commit(ctx, phase, st, w_bytes + p_bytes, stream, false);
}
