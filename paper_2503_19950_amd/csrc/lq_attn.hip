// Decode attention: launch planning and dispatch.
#include <math.h>
#include <stdlib.h>

#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

hipError_t launch_decode_attn_ref(const Shape& s, const lq_cache& c, const void* q, float scale,
                                  void* out, void* ws, int splits, hipStream_t st);
hipError_t launch_decode_attn_mfma(const Shape& s, const lq_cache& c, const void* q, float scale,
                                   void* out, void* ws, const lq_plan& plan, hipStream_t st);

constexpr int WPB = 8;   // wavefronts per workgroup of the attention kernel

static int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return v && *v ? atoi(v) : dflt;
}

// Context splits and the share of wavefronts that walks the fp rows.  Work is
// counted in bytes: a 64-slot quantized tile against a 32-row fp unit.
void plan_decode(const Shape& s, int n_fp, int n_q, lq_plan* plan) {
  const int TQ = (n_q + 63) / 64, TF = (n_fp + 31) / 32;
  const double q_tile_bytes = 64.0 * (s.d / 2 + 4 * s.ngc + 4.0 * s.d / s.G);
  const double fp_unit_bytes = 32.0 * 4 * s.d;
  const double r = fp_unit_bytes / q_tile_bytes;
  const double units = TQ + r * TF;
  const int hb = s.gh % 4 == 0 ? 4 : (s.gh % 2 == 0 ? 2 : 1);
  const int groups = s.B * s.Hkv * (s.gh / hb);
  static const int target_blocks = env_int("LOGQUANT_ATTN_BLOCKS", 256);
  static const int min_tiles = env_int("LOGQUANT_ATTN_MIN_TILES", 2);
  int splits = (target_blocks + groups - 1) / groups;
  const int by_work = (int)ceil(units / (WPB * (double)min_tiles));
  if (splits > by_work) splits = by_work;
  if (splits > max_splits(s)) splits = max_splits(s);
  if (splits < 1) splits = 1;
  const int NW = WPB * splits;
  int nwf = (int)lround(NW * (r * TF) / units);
  if (TF > 0) {
    if (nwf < 1) nwf = 1;
    if (nwf > TF) nwf = TF;
  } else {
    nwf = 0;
  }
  if (TQ > 0 && nwf > NW - 1) nwf = NW - 1;
  if (TQ == 0) nwf = NW;
  plan->splits = splits;
  plan->waves_per_block = WPB;
  plan->blocks = splits * groups;
  plan->fp_waves = nwf;
  plan->bytes_read = cache_bytes_read(s, n_fp, n_q);
}

hipError_t launch_decode_attn(const Shape& s, const lq_cache& c, const void* q, float scale,
                              void* out, void* ws, const lq_plan& plan, hipStream_t st) {
  // LOGQUANT_ATTN_PLAIN=1 selects the plain one-token-at-a-time kernel (cross-check).
  static const int plain = env_int("LOGQUANT_ATTN_PLAIN", 0);
  if (plain) return launch_decode_attn_ref(s, c, q, scale, out, ws, plan.splits, st);
  return launch_decode_attn_mfma(s, c, q, scale, out, ws, plan, st);
}

}  // namespace lq
