// Host-side internals: validated shape bundle and kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/logquant.h"

namespace lq {

struct Shape {
  int B, Hq, Hkv, d, W, G, cap, qcap, gh;  // gh = Hq/Hkv; cap = fp rows allocated per slice (3W rounded up to 32)
  int full;                                // 3W: list length at which the filtering step runs
  int Wq;                                  // quantized slots per filtering event: ceil(W/G) * G (W when G divides W)
  int nkc, nnt, ngc;                       // d/32, d/16, ceil(d/G)
  int bits;                                // 2 or 4
  bool bf16;
};

// Per-sequence lengths: one entry per batch row in device memory, written by the
// library at the start of every call of the per-sequence entry points and read by
// that call's kernels (a way to hand B sets of counts to a launch, not state).
struct SeqState {
  int n_fp, n_q;      // rows in the fp region, slots in the quantized region
  int cur;            // which fp buffer is live
  int nwf;            // attention: wavefronts of a head group that walk the fp rows
  int n_tok_q;        // tokens held in the n_q slots
  int item;           // compress: the i-th entry names the i-th sequence that is compressed
  int flag;           // append: 1 if the sequence takes a token; prefill: prompt length
  int order;          // attention: the i-th entry names the row with the i-th most tokens
};

constexpr int SEQ_CHUNK = 64;   // entries that fit a launch's own arguments (2 KB)
hipError_t launch_seq_upload(SeqState* dst, const SeqState* host, int n, hipStream_t st);

// How a launch gets the per-sequence state: batches of up to SEQ_CHUNK rows carry it in
// their own kernel arguments (`host`), larger ones read the device array (`dev`), which
// the caller of the launcher has filled with launch_seq_upload on the same stream.
struct SeqArg {
  const SeqState* dev;
  const SeqState* host;
  int n;
  bool in_args() const { return n <= SEQ_CHUNK; }
};
struct SeqInline { SeqState e[SEQ_CHUNK]; };
inline void fill_inline(SeqInline* S, const SeqArg* a) {
  if (a && a->in_args())
    for (int i = 0; i < a->n; ++i) S->e[i] = a->host[i];
}
// Kernel side: the state array inside the launch's own argument block.  It is read through
// the argument segment's address (scalar loads at a run-time index); indexing the by-value
// parameter itself makes the compiler copy all of it into private memory first.
// `offset` = where the array parameter starts in the argument block.
typedef const SeqState __attribute__((address_space(4))) * SeqArgsPtr;
__device__ __forceinline__ SeqArgsPtr seq_in_args(size_t offset) {
  typedef const char __attribute__((address_space(4))) * BytePtr;
  return (SeqArgsPtr)((BytePtr)__builtin_amdgcn_kernarg_segment_ptr() + offset);
}
__device__ __forceinline__ SeqState seq_load(SeqArgsPtr p, int i) {
  SeqState r;
  r.n_fp = p[i].n_fp; r.n_q = p[i].n_q; r.cur = p[i].cur; r.nwf = p[i].nwf;
  r.n_tok_q = p[i].n_tok_q; r.item = p[i].item; r.flag = p[i].flag; r.order = p[i].order;
  return r;
}
constexpr size_t args_offset_after(size_t bytes_before) { return (bytes_before + 3) / 4 * 4; }   // SeqState is 4-byte aligned
// kernel-side selector: 0 = no per-sequence state, 1 = in the kernel arguments, 2 = device array
inline int seq_mode(const SeqArg* a) { return !a ? 0 : a->in_args() ? 1 : 2; }

// Fills `s`; returns LQ_OK or the config error.  Pure host arithmetic.
lq_status make_shape(const lq_config* cfg, Shape* s);

// Upper bound on context splits per (b, kv head) that decode_attn may use.
int max_splits(const Shape& s);

// The workspace starts with the counters of the attention kernel: per (b, kv head,
// head group) CTR_LINES cache lines of CTR_LINE ints, each holding one counter in
// its first int: line 0 the ticket counter, lines 1..NSUB the tile pool counters.
// The splits' partial results follow.
constexpr int CTR_LINE = 32, NSUB = 8, CTR_LINES = 1 + NSUB;
inline size_t counter_bytes(const Shape& s) {
  return (size_t)s.B * s.Hkv * s.gh * CTR_LINES * CTR_LINE * sizeof(int);
}
hipError_t launch_workspace_init(const Shape& s, void* ws, hipStream_t st);
// The two parts of a workspace as the attention launchers take them.
struct Workspace {
  int* counters;
  float* partials;
};
inline Workspace split_workspace(const Shape& s, void* ws) {
  return Workspace{(int*)ws, (float*)((char*)ws + counter_bytes(s))};
}
// `n` ints at `p` set to zero by a small kernel (safe to record into a HIP graph).
hipError_t launch_zero_ints(int* p, int n, hipStream_t st);

// Bytes one decode step reads from the cache (live slots only).
int64_t cache_bytes_read(const Shape& s, int n_fp, int n_q);
// Tokens held in n_q quantized slots (n_q is a multiple of Wq; W of every Wq slots are live).
inline int quantized_tokens(const Shape& s, int n_q) { return n_q / s.Wq * s.W; }

// hipGetLastError() also reports failures of earlier, unrelated runtime calls made
// by other code in the process (an expected hipErrorNotReady, say).  Launchers
// clear that state first and report only what their own launch produced.
inline void clear_stale_error() { (void)hipGetLastError(); }
hipError_t launch_status(const char* what);

// --- launchers (enqueue only) -------------------------------------------------
hipError_t launch_append(const Shape& s, const lq_cache& c, const void* k_new, const void* v_new,
                         int n_new, hipStream_t st);
hipError_t launch_append_seq(const Shape& s, const lq_cache& c, const void* k_new, const void* v_new,
                             const SeqArg* seq, hipStream_t st);
// seq == nullptr: every sequence is compressed, from the counts of `c`.  Otherwise the
// n_items sequences named by seq[0..n_items).item, each from its own counts.
hipError_t launch_compress(const Shape& s, const lq_cache& c, hipStream_t st, const SeqArg* seq = nullptr,
                           int n_items = 0);
// seq == nullptr: one prompt length L for all.  Otherwise seq[b].flag is the prompt length of
// sequence b (n_fp / n_q what it leads to), L the row stride of the prompt tensors and
// E / n_fp the largest values over the batch (they size the grid).
hipError_t launch_prefill(const Shape& s, const lq_cache& c, const void* k, const void* v, int L, int E,
                          int n_fp, hipStream_t st, const SeqArg* seq = nullptr);
hipError_t launch_decode_attn(const Shape& s, const lq_cache& c, const void* q, float scale,
                              void* out, const Workspace& ws, const lq_plan& plan, hipStream_t st,
                              const SeqArg* seq = nullptr);
hipError_t launch_decode_step(const Shape& s, const lq_cache& c, const void* k_new, const void* v_new,
                              const void* q, float scale, void* out, const Workspace& ws, const lq_plan& plan,
                              hipStream_t st, const SeqArg* seq = nullptr);
void plan_decode(const Shape& s, int n_fp, int n_q, lq_plan* plan, bool per_sequence = false);
// Wavefronts (of the NW a head group has under `plan`) that walk n_fp fp rows when the
// quantized region holds n_q slots.
int fp_wave_share(const Shape& s, int NW, int n_fp, int n_q);

}  // namespace lq
