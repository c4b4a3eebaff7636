// C ABI of the library: argument checks on the host, then kernel launches.
// Every check happens before the first HIP call, so bad arguments are reported
// on machines without a GPU as well.
#include <stdio.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

lq_status make_shape(const lq_config* cfg, Shape* s) {
  if (!cfg || !s) return LQ_ERR_NULL;
  if (cfg->B <= 0 || cfg->Hq <= 0 || cfg->Hkv <= 0 || cfg->d <= 0 || cfg->fp_budget <= 0 ||
      cfg->group <= 0 || cfg->q_capacity <= 0)
    return LQ_ERR_SHAPE;
  if (cfg->Hq % cfg->Hkv) return LQ_ERR_SHAPE;
  if (cfg->fp_budget % 2) return LQ_ERR_SHAPE;
  if (cfg->dtype != LQ_F16 && cfg->dtype != LQ_BF16) return LQ_ERR_SHAPE;
  if (cfg->bits != 2 && cfg->bits != 4) return LQ_ERR_UNSUPPORTED;
  if (cfg->d != 64 && cfg->d != 96 && cfg->d != 128) return LQ_ERR_UNSUPPORTED;
  if (cfg->group != 32 && cfg->group != 64 && cfg->group != 128) return LQ_ERR_UNSUPPORTED;
  const int W = cfg->fp_budget / 2;
  const int Wq = (W + cfg->group - 1) / cfg->group * cfg->group;
  if (cfg->q_capacity % Wq || cfg->q_capacity % 64) return LQ_ERR_SHAPE;
  if ((int64_t)cfg->B * cfg->Hkv * (int64_t)cfg->q_capacity * cfg->d > ((int64_t)1 << 40))
    return LQ_ERR_SHAPE;
  // one grid row per (batch row, kv head, head group): the y extent of a launch is 16 bits
  if ((int64_t)cfg->B * cfg->Hq > 65535) return LQ_ERR_UNSUPPORTED;
  s->B = cfg->B; s->Hq = cfg->Hq; s->Hkv = cfg->Hkv; s->d = cfg->d;
  s->W = W; s->G = cfg->group; s->full = 3 * W; s->cap = (3 * W + 31) / 32 * 32; s->Wq = Wq;
  s->qcap = cfg->q_capacity;
  s->gh = cfg->Hq / cfg->Hkv;
  s->nkc = cfg->d / 32; s->nnt = cfg->d / 16; s->ngc = (cfg->d + cfg->group - 1) / cfg->group;
  s->bf16 = cfg->dtype == LQ_BF16;
  s->bits = cfg->bits;
  return LQ_OK;
}

int max_splits(const Shape& s) {
  const int bh = s.B * s.Hkv;
  int m = (1024 + bh - 1) / bh;
  if (m < 1) m = 1;
  if (m > 256) m = 256;
  return m;
}

int64_t cache_bytes_read(const Shape& s, int n_fp, int n_q) {
  // per quantized token: K codes and V codes d*bits/8 bytes each, value scale+zero 4
  // bytes per channel group; key scale+zero 4d bytes per key group (G slots).
  const int64_t q_bytes = (int64_t)quantized_tokens(s, n_q) * (s.d * s.bits / 4 + 4 * s.ngc) +
                          (int64_t)(n_q / s.G) * 4 * s.d;
  const int64_t fp_bytes = (int64_t)n_fp * 4 * s.d;
  return (int64_t)s.B * s.Hkv * (q_bytes + fp_bytes);
}

hipError_t launch_status(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) fprintf(stderr, "logquant: %s: %s\n", what, hipGetErrorString(e));
  return e;
}

static bool cache_ptrs_ok(const lq_cache* c) {
  return c && c->k_fp[0] && c->k_fp[1] && c->v_fp[0] && c->v_fp[1] && c->pos_fp[0] &&
         c->pos_fp[1] && c->k_codes && c->v_codes && c->k_scale && c->k_zero && c->v_scale &&
         c->v_zero && c->pos_q;
}

static lq_status cache_state_ok(const Shape& s, const lq_cache* c) {
  if (c->cur != 0 && c->cur != 1) return LQ_ERR_STATE;
  if (c->n_fp < 0 || c->n_fp > s.full) return LQ_ERR_STATE;
  if (c->n_q < 0 || c->n_q > s.qcap || c->n_q % s.Wq) return LQ_ERR_STATE;
  return LQ_OK;
}

}  // namespace lq

using namespace lq;

extern "C" {

lq_status logquant_sizes(const lq_config* cfg, lq_sizes* out) {
  if (!cfg || !out) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  const size_t bh = (size_t)s.B * s.Hkv;
  out->k_fp = bh * s.cap * s.d * 2;
  out->v_fp = out->k_fp;
  out->pos_fp = (size_t)s.B * s.cap * 4;
  out->k_codes = bh * s.qcap * s.d * s.bits / 8;
  out->v_codes = out->k_codes;
  out->k_meta = bh * (s.qcap / s.G) * s.d * 2;
  out->v_meta = bh * s.qcap * s.ngc * 2;
  out->pos_q = (size_t)s.B * s.qcap * 4;
  out->workspace = logquant_workspace_bytes(cfg);
  return LQ_OK;
}

size_t logquant_workspace_bytes(const lq_config* cfg) {
  Shape s;
  if (make_shape(cfg, &s) != LQ_OK) return 0;
  // ticket counters, then per (b, kv head, split): gh * (d + 4) floats (o, m, l, padding to 16 bytes)
  return counter_bytes(s) + (size_t)s.B * s.Hkv * max_splits(s) * s.gh * (s.d + 4) * sizeof(float);
}

lq_status logquant_workspace_init(const lq_config* cfg, void* workspace, void* stream) {
  if (!cfg || !workspace) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  clear_stale_error();
  if (launch_workspace_init(s, workspace, (hipStream_t)stream) != hipSuccess) return LQ_ERR_HIP;
  return LQ_OK;
}

lq_status logquant_append(const lq_config* cfg, lq_cache* cache, const void* k_new,
                          const void* v_new, int32_t n_new, void* stream) {
  if (!cfg || !cache || !k_new || !v_new) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (!cache_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = cache_state_ok(s, cache)) != LQ_OK) return st;
  if (n_new <= 0) return LQ_ERR_SHAPE;
  if (cache->n_fp + n_new > s.full) return LQ_ERR_CAPACITY;
  clear_stale_error();
  if (launch_append(s, *cache, k_new, v_new, n_new, (hipStream_t)stream) != hipSuccess)
    return LQ_ERR_HIP;
  cache->n_fp += n_new;
  return LQ_OK;
}

lq_status logquant_compress(const lq_config* cfg, lq_cache* cache, void* workspace, void* stream) {
  (void)workspace;
  if (!cfg || !cache) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (!cache_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = cache_state_ok(s, cache)) != LQ_OK) return st;
  if (cache->n_fp != s.full) return LQ_ERR_STATE;
  if (cache->n_q + s.Wq > s.qcap) return LQ_ERR_CAPACITY;
  clear_stale_error();
  if (launch_compress(s, *cache, (hipStream_t)stream) != hipSuccess) return LQ_ERR_HIP;
  cache->cur ^= 1;
  cache->n_fp = 2 * s.W;
  cache->n_q += s.Wq;
  return LQ_OK;
}

// number of filtering events after L appends (filtering as soon as the list holds 3W)
static int events_after(int L, int W) { return L < 3 * W ? 0 : (L - 3 * W) / W + 1; }

lq_status logquant_prefill(const lq_config* cfg, lq_cache* cache, const void* k, const void* v,
                           int32_t L, void* stream) {
  if (!cfg || !cache || !k || !v) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (!cache_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = cache_state_ok(s, cache)) != LQ_OK) return st;
  if (L < 1) return LQ_ERR_SHAPE;
  if (cache->n_fp != 0 || cache->n_q != 0) return LQ_ERR_STATE;
  const int E = events_after(L, s.W);
  if ((int64_t)E * s.Wq > s.qcap) return LQ_ERR_CAPACITY;
  const int n_fp = L - E * s.W;
  clear_stale_error();
  if (launch_prefill(s, *cache, k, v, L, E, n_fp, (hipStream_t)stream) != hipSuccess) return LQ_ERR_HIP;
  cache->n_fp = n_fp;
  cache->n_q = E * s.Wq;
  return LQ_OK;
}

lq_status logquant_prefill_positions(int32_t W, int32_t L, int32_t* pos_fp, int32_t* n_fp,
                                     int32_t* pos_q, int32_t* n_q) {
  if (W < 1 || L < 0) return LQ_ERR_SHAPE;
  const int E = events_after(L, W);
  const int nf = L - E * W, nq = E * W;
  if (n_fp) *n_fp = nf;
  if (n_q) *n_q = nq;
  if (pos_fp)
    for (int i = 0; i < nf; ++i) pos_fp[i] = fp_position(E, i, W);
  if (pos_q)
    for (int e = 1; e <= E; ++e)
      for (int i = 0; i < W; ++i) pos_q[(e - 1) * W + i] = evicted_position(e, i, W);
  return LQ_OK;
}

lq_status logquant_decode_plan(const lq_config* cfg, int32_t n_fp, int32_t n_q, lq_plan* out) {
  if (!cfg || !out) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (n_fp < 0 || n_fp > s.full || n_q < 0 || n_q > s.qcap || n_q % s.Wq || n_fp + n_q < 1)
    return LQ_ERR_STATE;
  plan_decode(s, n_fp, n_q, out);
  return LQ_OK;
}

lq_status logquant_decode_attn(const lq_config* cfg, const lq_cache* cache, const void* q,
                               float softmax_scale, void* out, void* workspace, void* stream) {
  if (!cfg || !cache || !q || !out || !workspace) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (!cache_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = cache_state_ok(s, cache)) != LQ_OK) return st;
  if (cache->n_fp + cache->n_q < 1) return LQ_ERR_STATE;
  lq_plan plan;
  plan_decode(s, cache->n_fp, cache->n_q, &plan);
  if (!(softmax_scale > 0.f)) softmax_scale = 1.0f / sqrtf((float)s.d);
  clear_stale_error();
  if (launch_decode_attn(s, *cache, q, softmax_scale, out, split_workspace(s, workspace), plan, (hipStream_t)stream) !=
      hipSuccess)
    return LQ_ERR_HIP;
  return LQ_OK;
}

// ---- decode attention for callers that cannot allocate -------------------------------
// The scratch that logquant_decode_attn takes as `workspace` (ticket and tile-pool counters,
// partial softmax states of the context splits) lives in a device array of the library
// itself: a counter area of fixed size at its start, the partials behind it.  The counter
// area never holds anything but counters, whatever configuration a call has, and every call
// leaves its counters at zero, so it is cleared once per device, by the first call there.
namespace {
constexpr size_t STATIC_COUNTER_BYTES = (size_t)4 << 20;
constexpr size_t STATIC_PARTIAL_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_COUNTER_BYTES + STATIC_PARTIAL_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_ptr[STATIC_MAX_DEVICES];        // per device: the device address of `scratch` there
bool scratch_cleared[STATIC_MAX_DEVICES];
}  // namespace

lq_status logquant_decode_attn_static(const lq_config* cfg, const lq_cache* cache, const void* q,
                                      float softmax_scale, void* out, void* stream) {
  if (!cfg || !cache || !q || !out) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (!cache_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = cache_state_ok(s, cache)) != LQ_OK) return st;
  if (cache->n_fp + cache->n_q < 1) return LQ_ERR_STATE;
  const size_t partial_bytes = logquant_workspace_bytes(cfg) - counter_bytes(s);
  if (counter_bytes(s) > STATIC_COUNTER_BYTES || partial_bytes > STATIC_PARTIAL_BYTES) return LQ_ERR_CAPACITY;
  lq_plan plan;
  plan_decode(s, cache->n_fp, cache->n_q, &plan);
  if (!(softmax_scale > 0.f)) softmax_scale = 1.0f / sqrtf((float)s.d);
  clear_stale_error();
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return LQ_ERR_HIP;
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
      // the array's name is a host-side handle: its address on the current device comes from the runtime
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LQ_ERR_HIP;
      scratch_ptr[dev] = p;
    }
    base = scratch_ptr[dev];
    if (!scratch_cleared[dev]) {
      if (launch_zero_ints((int*)base, (int)(STATIC_COUNTER_BYTES / sizeof(int)), (hipStream_t)stream) != hipSuccess)
        return LQ_ERR_HIP;
      scratch_cleared[dev] = true;
    }
  }
  const Workspace ws{(int*)base, (float*)((char*)base + STATIC_COUNTER_BYTES)};
  if (launch_decode_attn(s, *cache, q, softmax_scale, out, ws, plan, (hipStream_t)stream) != hipSuccess)
    return LQ_ERR_HIP;
  return LQ_OK;
}

lq_status logquant_decode_step(const lq_config* cfg, lq_cache* cache, const void* k_new,
                               const void* v_new, const void* q, float softmax_scale, void* out,
                               void* workspace, void* stream) {
  if (!cfg || !cache || !k_new || !v_new || !q || !out || !workspace) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (!cache_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = cache_state_ok(s, cache)) != LQ_OK) return st;
  if (cache->n_fp + 1 >= s.full) return LQ_ERR_STATE;   // the window would be full: append, compress, attend
  lq_cache after = *cache;
  after.n_fp += 1;
  lq_plan plan;
  plan_decode(s, after.n_fp, after.n_q, &plan);
  if (!(softmax_scale > 0.f)) softmax_scale = 1.0f / sqrtf((float)s.d);
  clear_stale_error();
  if (launch_decode_step(s, after, k_new, v_new, q, softmax_scale, out, split_workspace(s, workspace), plan,
                         (hipStream_t)stream) != hipSuccess)
    return LQ_ERR_HIP;
  cache->n_fp = after.n_fp;
  return LQ_OK;
}

// ---- per-sequence lengths ---------------------------------------------------------
// The same kernels; every call writes the B sets of counts its kernels need into
// cache->seq_state first (same stream, so the order is kept) and then updates the
// host arrays.

static bool seq_ptrs_ok(const lq_cache_seq* c) {
  return c && c->k_fp[0] && c->k_fp[1] && c->v_fp[0] && c->v_fp[1] && c->pos_fp[0] && c->pos_fp[1] &&
         c->k_codes && c->v_codes && c->k_scale && c->k_zero && c->v_scale && c->v_zero && c->pos_q &&
         c->cur && c->n_fp && c->n_q && c->seq_state;
}

static lq_status seq_state_ok(const Shape& s, const lq_cache_seq* c) {
  for (int b = 0; b < s.B; ++b) {
    if (c->cur[b] != 0 && c->cur[b] != 1) return LQ_ERR_STATE;
    if (c->n_fp[b] < 0 || c->n_fp[b] > s.full) return LQ_ERR_STATE;
    if (c->n_q[b] < 0 || c->n_q[b] > s.qcap || c->n_q[b] % s.Wq) return LQ_ERR_STATE;
  }
  return LQ_OK;
}

// the buffers as the launchers take them; counts = the largest over the batch
static lq_cache seq_view(const Shape& s, const lq_cache_seq* c, const int* n_fp, const int* n_q) {
  lq_cache v;
  for (int i = 0; i < 2; ++i) { v.k_fp[i] = c->k_fp[i]; v.v_fp[i] = c->v_fp[i]; v.pos_fp[i] = c->pos_fp[i]; }
  v.k_codes = c->k_codes; v.v_codes = c->v_codes;
  v.k_scale = c->k_scale; v.k_zero = c->k_zero; v.v_scale = c->v_scale; v.v_zero = c->v_zero;
  v.pos_q = c->pos_q;
  v.cur = 0; v.n_fp = 0; v.n_q = 0;
  for (int b = 0; b < s.B; ++b) {
    if (n_fp[b] > v.n_fp) v.n_fp = n_fp[b];
    if (n_q[b] > v.n_q) v.n_q = n_q[b];
  }
  return v;
}

static SeqState seq_entry(const Shape& s, int n_fp, int n_q, int cur) {
  SeqState e{};
  e.n_fp = n_fp; e.n_q = n_q; e.cur = cur; e.n_tok_q = quantized_tokens(s, n_q);
  return e;
}

// Plan for the longest sequence; bytes and the fp share of the wavefronts per sequence.
static void plan_seq(const Shape& s, const int* n_fp, const int* n_q, lq_plan* plan, SeqState* st) {
  int mf = 0, mq = 0;
  for (int b = 0; b < s.B; ++b) { if (n_fp[b] > mf) mf = n_fp[b]; if (n_q[b] > mq) mq = n_q[b]; }
  plan_decode(s, mf, mq, plan, true);
  const int NW = plan->splits * plan->waves_per_block;
  int64_t bytes = 0;
  Shape one = s;
  one.B = 1;
  for (int b = 0; b < s.B; ++b) {
    bytes += cache_bytes_read(one, n_fp[b], n_q[b]);
    if (st) st[b].nwf = fp_wave_share(s, NW, n_fp[b], n_q[b]);
  }
  plan->bytes_read = bytes;
  if (st) {   // rows by decreasing work (stable: equal rows keep their order)
    std::vector<int> idx(s.B);
    for (int b = 0; b < s.B; ++b) idx[b] = b;
    std::stable_sort(idx.begin(), idx.end(), [&](int x, int y) {
      return cache_bytes_read(one, n_fp[x], n_q[x]) > cache_bytes_read(one, n_fp[y], n_q[y]);
    });
    for (int b = 0; b < s.B; ++b) st[b].order = idx[b];
  }
}

size_t logquant_seq_state_bytes(const lq_config* cfg) {
  Shape s;
  if (make_shape(cfg, &s) != LQ_OK) return 0;
  return (size_t)s.B * sizeof(SeqState);
}

// Common start of the per-sequence calls: shape, pointers, per-row counts; sizes the host
// copy of the state array.
// Makes the state reachable for the launch: in its arguments (small batches) or through
// the device array, which is then filled first on the same stream.
static hipError_t seq_hand_over(const lq_cache_seq* cache, const std::vector<SeqState>& host, hipStream_t st, SeqArg* arg) {
  arg->dev = (const SeqState*)cache->seq_state;
  arg->host = host.data();
  arg->n = (int)host.size();
  if (arg->in_args()) return hipSuccess;
  return launch_seq_upload((SeqState*)cache->seq_state, host.data(), arg->n, st);
}

static lq_status seq_begin(const lq_config* cfg, const lq_cache_seq* cache, Shape* s, std::vector<SeqState>* host) {
  lq_status st = make_shape(cfg, s);
  if (st != LQ_OK) return st;
  if (!seq_ptrs_ok(cache)) return LQ_ERR_NULL;
  if ((st = seq_state_ok(*s, cache)) != LQ_OK) return st;
  host->assign(s->B, SeqState{});
  return LQ_OK;
}

lq_status logquant_prefill_seq(const lq_config* cfg, lq_cache_seq* cache, const void* k, const void* v,
                               const int32_t* L, int32_t L_stride, void* stream) {
  if (!cfg || !cache || !k || !v || !L) return LQ_ERR_NULL;
  Shape s;
  std::vector<SeqState> host;
  const lq_status st0 = seq_begin(cfg, cache, &s, &host);
  if (st0 != LQ_OK) return st0;
  if (L_stride < 1) return LQ_ERR_SHAPE;
  std::vector<int> nf(s.B), nq(s.B);
  int Emax = 0, fmax = 0;
  for (int b = 0; b < s.B; ++b) {
    if (L[b] < 0 || L[b] > L_stride) return LQ_ERR_SHAPE;
    if (cache->n_fp[b] != 0 || cache->n_q[b] != 0) return LQ_ERR_STATE;
    const int E = events_after(L[b], s.W);
    if ((int64_t)E * s.Wq > s.qcap) return LQ_ERR_CAPACITY;
    nf[b] = L[b] - E * s.W; nq[b] = E * s.Wq;
    host[b] = seq_entry(s, nf[b], nq[b], cache->cur[b]);
    host[b].flag = L[b];
    if (E > Emax) Emax = E;
    if (nf[b] > fmax) fmax = nf[b];
  }
  if (Emax == 0 && fmax == 0) return LQ_OK;   // every prompt is empty
  clear_stale_error();
  SeqArg arg;
  if (seq_hand_over(cache, host, (hipStream_t)stream, &arg) != hipSuccess) return LQ_ERR_HIP;
  const lq_cache view = seq_view(s, cache, nf.data(), nq.data());
  if (launch_prefill(s, view, k, v, L_stride, Emax, fmax, (hipStream_t)stream, &arg) != hipSuccess) return LQ_ERR_HIP;
  for (int b = 0; b < s.B; ++b) { cache->n_fp[b] = nf[b]; cache->n_q[b] = nq[b]; }
  return LQ_OK;
}

lq_status logquant_append_seq(const lq_config* cfg, lq_cache_seq* cache, const void* k_new,
                              const void* v_new, const int32_t* active, void* stream) {
  if (!cfg || !cache || !k_new || !v_new) return LQ_ERR_NULL;
  Shape s;
  std::vector<SeqState> host;
  const lq_status st0 = seq_begin(cfg, cache, &s, &host);
  if (st0 != LQ_OK) return st0;
  int n_active = 0;
  for (int b = 0; b < s.B; ++b) {
    const int a = active ? (active[b] != 0) : 1;
    if (a && cache->n_fp[b] + 1 > s.full) return LQ_ERR_CAPACITY;
    host[b] = seq_entry(s, cache->n_fp[b] + a, cache->n_q[b], cache->cur[b]);   // counts after the append
    host[b].flag = a;
    n_active += a;
  }
  if (!n_active) return LQ_OK;
  clear_stale_error();
  SeqArg arg;
  if (seq_hand_over(cache, host, (hipStream_t)stream, &arg) != hipSuccess) return LQ_ERR_HIP;
  const lq_cache view = seq_view(s, cache, cache->n_fp, cache->n_q);
  if (launch_append_seq(s, view, k_new, v_new, &arg, (hipStream_t)stream) != hipSuccess) return LQ_ERR_HIP;
  for (int b = 0; b < s.B; ++b) cache->n_fp[b] = host[b].n_fp;
  return LQ_OK;
}

lq_status logquant_compress_seq(const lq_config* cfg, lq_cache_seq* cache, void* stream) {
  if (!cfg || !cache) return LQ_ERR_NULL;
  Shape s;
  std::vector<SeqState> host;
  const lq_status st0 = seq_begin(cfg, cache, &s, &host);
  if (st0 != LQ_OK) return st0;
  int n_items = 0;
  for (int b = 0; b < s.B; ++b) {
    host[b] = seq_entry(s, cache->n_fp[b], cache->n_q[b], cache->cur[b]);      // counts before the event
    if (cache->n_fp[b] == s.full) {
      if (cache->n_q[b] + s.Wq > s.qcap) return LQ_ERR_CAPACITY;
      host[n_items++].item = b;
    }
  }
  if (!n_items) return LQ_OK;
  clear_stale_error();
  SeqArg arg;
  if (seq_hand_over(cache, host, (hipStream_t)stream, &arg) != hipSuccess) return LQ_ERR_HIP;
  const lq_cache view = seq_view(s, cache, cache->n_fp, cache->n_q);
  if (launch_compress(s, view, (hipStream_t)stream, &arg, n_items) != hipSuccess) return LQ_ERR_HIP;
  for (int i = 0; i < n_items; ++i) {
    const int b = host[i].item;
    cache->cur[b] ^= 1;
    cache->n_fp[b] = 2 * s.W;
    cache->n_q[b] += s.Wq;
  }
  return LQ_OK;
}

lq_status logquant_decode_plan_seq(const lq_config* cfg, const int32_t* n_fp, const int32_t* n_q, lq_plan* out) {
  if (!cfg || !n_fp || !n_q || !out) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  for (int b = 0; b < s.B; ++b)
    if (n_fp[b] < 0 || n_fp[b] > s.full || n_q[b] < 0 || n_q[b] > s.qcap || n_q[b] % s.Wq || n_fp[b] + n_q[b] < 1)
      return LQ_ERR_STATE;
  plan_seq(s, n_fp, n_q, out, nullptr);
  return LQ_OK;
}

lq_status logquant_decode_attn_seq(const lq_config* cfg, const lq_cache_seq* cache, const void* q,
                                   float softmax_scale, void* out, void* workspace, void* stream) {
  if (!cfg || !cache || !q || !out || !workspace) return LQ_ERR_NULL;
  Shape s;
  std::vector<SeqState> host;
  const lq_status st0 = seq_begin(cfg, cache, &s, &host);
  if (st0 != LQ_OK) return st0;
  for (int b = 0; b < s.B; ++b) {
    if (cache->n_fp[b] + cache->n_q[b] < 1) return LQ_ERR_STATE;
    host[b] = seq_entry(s, cache->n_fp[b], cache->n_q[b], cache->cur[b]);
  }
  lq_plan plan;
  plan_seq(s, cache->n_fp, cache->n_q, &plan, host.data());
  if (!(softmax_scale > 0.f)) softmax_scale = 1.0f / sqrtf((float)s.d);
  clear_stale_error();
  SeqArg arg;
  if (seq_hand_over(cache, host, (hipStream_t)stream, &arg) != hipSuccess) return LQ_ERR_HIP;
  const lq_cache view = seq_view(s, cache, cache->n_fp, cache->n_q);
  if (launch_decode_attn(s, view, q, softmax_scale, out, split_workspace(s, workspace), plan, (hipStream_t)stream, &arg) != hipSuccess)
    return LQ_ERR_HIP;
  return LQ_OK;
}

lq_status logquant_decode_step_seq(const lq_config* cfg, lq_cache_seq* cache, const void* k_new,
                                   const void* v_new, const void* q, float softmax_scale, void* out,
                                   void* workspace, void* stream) {
  if (!cfg || !cache || !k_new || !v_new || !q || !out || !workspace) return LQ_ERR_NULL;
  Shape s;
  std::vector<SeqState> host;
  const lq_status st0 = seq_begin(cfg, cache, &s, &host);
  if (st0 != LQ_OK) return st0;
  std::vector<int> nf(s.B);
  for (int b = 0; b < s.B; ++b) {
    if (cache->n_fp[b] + 1 >= s.full) return LQ_ERR_STATE;   // some window would be full: separate calls
    nf[b] = cache->n_fp[b] + 1;
    host[b] = seq_entry(s, nf[b], cache->n_q[b], cache->cur[b]);
    host[b].flag = 1;
  }
  lq_plan plan;
  plan_seq(s, nf.data(), cache->n_q, &plan, host.data());
  if (!(softmax_scale > 0.f)) softmax_scale = 1.0f / sqrtf((float)s.d);
  clear_stale_error();
  SeqArg arg;
  if (seq_hand_over(cache, host, (hipStream_t)stream, &arg) != hipSuccess) return LQ_ERR_HIP;
  const lq_cache view = seq_view(s, cache, nf.data(), cache->n_q);
  if (launch_decode_step(s, view, k_new, v_new, q, softmax_scale, out, split_workspace(s, workspace), plan, (hipStream_t)stream, &arg) !=
      hipSuccess)
    return LQ_ERR_HIP;
  for (int b = 0; b < s.B; ++b) cache->n_fp[b] = nf[b];
  return LQ_OK;
}

const char* logquant_status_string(lq_status s) {
  switch (s) {
    case LQ_OK: return "ok";
    case LQ_ERR_NULL: return "null pointer";
    case LQ_ERR_SHAPE: return "inconsistent shape";
    case LQ_ERR_UNSUPPORTED: return "unsupported configuration";
    case LQ_ERR_CAPACITY: return "capacity exceeded";
    case LQ_ERR_STATE: return "call not allowed in this cache state";
    case LQ_ERR_HIP: return "HIP launch error";
  }
  return "unknown status";
}

}  // extern "C"
