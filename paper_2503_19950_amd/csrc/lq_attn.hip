// Decode attention: launch planning and dispatch.
#include <math.h>
#include <stdlib.h>

#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

hipError_t launch_decode_attn_mfma(const Shape& s, const lq_cache& c, const void* q, float scale,
                                   void* out, const Workspace& ws, const lq_plan& plan, hipStream_t st,
                                   const void* k_new, const void* v_new, const SeqArg* seq);

static int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return v && *v ? atoi(v) : dflt;
}

// Launch shape: wavefronts per workgroup (12, 8 or 4), context splits per (b, kv head,
// head group), and the share of wavefronts that walks the fp rows.  Work is counted
// in units of one 64-slot quantized tile; a 32-row fp unit weighs its bytes relative
// to that.  A compute unit holds eight wavefronts of this kernel, i.e. one
// workgroup of 8 or two of 4; the candidate shapes are ranked by
//     rounds * (units per wavefront + fixed) + merge cost per split,
// rounds = how many times the chip has to be refilled, fixed = start-up and merge
// tail of a workgroup expressed in tiles.
static double fp_unit_weight(const Shape& s) {
  const double q_tile_bytes = 64.0 * (s.d * s.bits / 4 + 4 * s.ngc + 4.0 * s.d / s.G);
  const double fp_unit_bytes = 32.0 * 4 * s.d;
  return fp_unit_bytes / q_tile_bytes;
}

// Wavefronts for the fp rows: units of 32 rows are dealt out statically (a wavefront
// takes every nwf-th unit), the quantized tiles are shared by the others.  Pick the
// count that minimises the longer of the two sides, whole units per fp wavefront
// counted (with 16 units, 9 wavefronts are no better than 8: some still take two).
int fp_wave_share(const Shape& s, int NW, int n_fp, int n_q) {
  const int TQ = (n_q + 63) / 64, TF = (n_fp + 31) / 32;
  if (TF == 0) return 0;
  if (TQ == 0) return NW;
  const double r = fp_unit_weight(s);   // (measured: halving or doubling this weight changes nothing on the five workloads)
  int best = 1;
  double best_t = 1e300;
  const int hi = TF < NW - 1 ? TF : NW - 1;
  for (int n = 1; n <= hi; ++n) {
    const double t_fp = (double)((TF + n - 1) / n) * r, t_q = (double)TQ / (NW - n);
    const double t = t_fp > t_q ? t_fp : t_q;
    if (t < best_t - 1e-9) { best_t = t; best = n; }
  }
  return best;
}

void plan_decode(const Shape& s, int n_fp, int n_q, lq_plan* plan, bool per_sequence) {
  const int TQ = (n_q + 63) / 64, TF = (n_fp + 31) / 32;
  const double r = fp_unit_weight(s);
  const double units = TQ + r * TF;
  const int hb = s.gh % 4 == 0 ? 4 : (s.gh % 2 == 0 ? 2 : 1);
  const int groups = s.B * s.Hkv * (s.gh / hb);
  static const int cus = env_int("LOGQUANT_ATTN_CUS", 256);
  static const int force_wpb = env_int("LOGQUANT_ATTN_WPB", 0);
  static const int force_splits = env_int("LOGQUANT_ATTN_SPLITS", 0);
  const double fixed = 2.5, per_split = 0.02, merge_tail = 1.5;
  int best_wpb = 8, best_splits = 1;
  double best = 1e300;
  // padding slots in the quantized region, per-sequence counts: 8-wavefront kernel only
  const bool ragged = s.Wq != s.W || per_sequence;
  for (int wpb = 8; wpb >= 4; wpb -= 4) {
    if (ragged && wpb != 8) continue;   // (12 is derived from 8 below)
    if (!ragged && force_wpb && force_wpb != 12 && wpb != force_wpb) continue;
    const int slots = cus * (8 / wpb);
    int smax = (int)ceil(units / wpb);            // at least one unit per wavefront
    if (smax > max_splits(s)) smax = max_splits(s);
    if (smax < 1) smax = 1;
    for (int sp = 1; sp <= smax; ++sp) {
      if (force_splits && sp != force_splits && force_splits <= smax) continue;
      const int rounds = (sp * groups + slots - 1) / slots;
      // more than one split adds the cross-workgroup merge: a chain of memory round trips
      // (store, ticket, fetch) worth about a tile and a half (measured on the smallest
      // workload: 8.4 us with three splits, 6.8 us with one)
      const double t = rounds * (units / ((double)sp * wpb) + fixed) + per_split * sp + (sp > 1 ? merge_tail : 0.0);
      if (t < best - 1e-9) { best = t; best_wpb = wpb; best_splits = sp; }
    }
  }
  // Twelve wavefronts per workgroup (three per SIMD) pay off for long contexts on few
  // groups: measured on 131072 tokens x 8 kv heads 25.7 against 27.3 us, but slower
  // than 8 with fewer than ~6 tiles per wavefront and slower than 4 when every
  // compute unit holds two workgroups anyway.  Only built for 2-bit codes (with 4-bit
  // codes it was measured to make no difference: 37.3 against 37.2 us).
  // (and only when the launch fits the chip in one round: with more workgroups than
  // compute units, as in a batch of 64 rows with per-row counts, 8 is faster: 49 against 54 us)
  if (s.bits == 2 && (force_wpb == 12 || (!force_wpb && best_wpb == 8 && units / (best_splits * 8.0) >= 6.0 &&
                                          (int64_t)best_splits * groups <= cus)))
    best_wpb = 12;
  const int splits = best_splits, WPB = best_wpb;
  const int NW = WPB * splits;
  const int nwf = fp_wave_share(s, NW, n_fp, n_q);
  plan->splits = splits;
  plan->waves_per_block = WPB;
  plan->blocks = splits * groups;
  plan->fp_waves = nwf;
  plan->bytes_read = cache_bytes_read(s, n_fp, n_q);
}

hipError_t launch_decode_attn(const Shape& s, const lq_cache& c, const void* q, float scale,
                              void* out, const Workspace& ws, const lq_plan& plan, hipStream_t st, const SeqArg* seq) {
  return launch_decode_attn_mfma(s, c, q, scale, out, ws, plan, st, nullptr, nullptr, seq);
}

// `c` already counts the new row (n_fp includes it); the row itself is still only in
// k_new / v_new.
hipError_t launch_decode_step(const Shape& s, const lq_cache& c, const void* k_new, const void* v_new,
                              const void* q, float scale, void* out, const Workspace& ws, const lq_plan& plan,
                              hipStream_t st, const SeqArg* seq) {
  return launch_decode_attn_mfma(s, c, q, scale, out, ws, plan, st, k_new, v_new, seq);
}

}  // namespace lq
