// Decode attention: launch planning and dispatch.
#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

hipError_t launch_decode_attn_ref(const Shape& s, const lq_cache& c, const void* q, float scale,
                                  void* out, void* ws, int splits, hipStream_t st);

void plan_decode(const Shape& s, int n_fp, int n_q, lq_plan* plan) {
  const int T = n_fp + n_q;
  int splits = (T + 255) / 256;
  if (splits > max_splits(s)) splits = max_splits(s);
  if (splits < 1) splits = 1;
  plan->splits = splits;
  plan->waves_per_block = 4;
  plan->blocks = splits * s.B * s.Hkv;
  plan->fp_waves = 0;
  plan->bytes_read = cache_bytes_read(s, n_fp, n_q);
}

hipError_t launch_decode_attn(const Shape& s, const lq_cache& c, const void* q, float scale,
                              void* out, void* ws, const lq_plan& plan, hipStream_t st) {
  return launch_decode_attn_ref(s, c, q, scale, out, ws, plan.splits, st);
}

}  // namespace lq
