// Append branch of Algorithm 1 (Sec. 2.5): new tokens go to the end of the
// original-precision list.  The rows arrive row-major and are scattered into the
// operand-ordered fp buffers (keys: 16-byte octets of channels; values: one
// 2-byte element per channel into the token-interleaved tiles).
#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

// grid (n_new, B*Hkv), block d/8 * 8 = d threads.
__global__ void append_kernel(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                              uint16_t* __restrict__ k_fp, uint16_t* __restrict__ v_fp,
                              int32_t* __restrict__ pos_fp, int n_new, int n_fp, int pos0, int d,
                              int cap, int Hkv) {
  const int j = blockIdx.x;        // which new token
  const int bh = blockIdx.y;
  const int c = threadIdx.x;       // channel
  const int t = n_fp + j;          // destination slot
  const int64_t src = ((int64_t)bh * n_new + j) * d + c;
  const int64_t slice = (int64_t)bh * cap * d;
  k_fp[slice + k_fp_index(t, c, d >> 5)] = k_new[src];
  v_fp[slice + v_fp_index(t, c, d >> 4)] = v_new[src];
  if (c == 0 && bh % Hkv == 0) pos_fp[(bh / Hkv) * cap + t] = pos0 + j;
}

// Per-sequence lengths: sequence b appends (flag set) or sits the call out.  The entry
// already counts the new row: it becomes fp slot n_fp - 1 of the sequence's live buffer.
// grid (1, B*Hkv), block d.
__global__ void append_seq_kernel(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                                  uint16_t* k_fp0, uint16_t* v_fp0, int32_t* pos_fp0, uint16_t* k_fp1,
                                  uint16_t* v_fp1, int32_t* pos_fp1, const SeqState* __restrict__ seq,
                                  int mode, int d, int cap, int Hkv, const SeqInline S) {
  const int bh = blockIdx.y, c = threadIdx.x;
  // argument block: nine pointers, four ints, then S
  const SeqState sq = mode == 1 ? seq_load(seq_in_args(args_offset_after(9 * 8 + 4 * 4)), bh / Hkv) : seq[bh / Hkv];
  (void)S;
  if (!sq.flag) return;
  uint16_t* k_fp = sq.cur ? k_fp1 : k_fp0;
  uint16_t* v_fp = sq.cur ? v_fp1 : v_fp0;
  int32_t* pos_fp = sq.cur ? pos_fp1 : pos_fp0;
  const int t = sq.n_fp - 1;
  const int64_t src = (int64_t)bh * d + c;
  const int64_t slice = (int64_t)bh * cap * d;
  k_fp[slice + k_fp_index(t, c, d >> 5)] = k_new[src];
  v_fp[slice + v_fp_index(t, c, d >> 4)] = v_new[src];
  if (c == 0 && bh % Hkv == 0) pos_fp[(bh / Hkv) * cap + t] = t + sq.n_tok_q;
}

// Hands up to SEQ_CHUNK entries of per-sequence state to the device by value (kernel
// arguments), so that no host buffer has to outlive the call.
struct SeqChunk { int base, n; SeqState e[SEQ_CHUNK]; };
__global__ void seq_upload_kernel(SeqState* dst, const SeqChunk ch) {
  const int i = threadIdx.x;
  if (i < ch.n) dst[ch.base + i] = ch.e[i];
}

hipError_t launch_seq_upload(SeqState* dst, const SeqState* host, int n, hipStream_t st) {
  for (int base = 0; base < n; base += SEQ_CHUNK) {
    SeqChunk ch;
    ch.base = base;
    ch.n = n - base < SEQ_CHUNK ? n - base : SEQ_CHUNK;
    for (int i = 0; i < ch.n; ++i) ch.e[i] = host[base + i];
    for (int i = ch.n; i < SEQ_CHUNK; ++i) ch.e[i] = SeqState{};
    hipLaunchKernelGGL(seq_upload_kernel, dim3(1), dim3(SEQ_CHUNK), 0, st, dst, ch);
  }
  return launch_status(__func__);
}

hipError_t launch_append_seq(const Shape& s, const lq_cache& c, const void* k_new, const void* v_new,
                             const SeqArg* seq, hipStream_t st) {
  SeqInline S;
  fill_inline(&S, seq);
  hipLaunchKernelGGL(append_seq_kernel, dim3(1, s.B * s.Hkv), dim3(s.d), 0, st, (const uint16_t*)k_new,
                     (const uint16_t*)v_new, (uint16_t*)c.k_fp[0], (uint16_t*)c.v_fp[0], c.pos_fp[0],
                     (uint16_t*)c.k_fp[1], (uint16_t*)c.v_fp[1], c.pos_fp[1], seq->dev, seq_mode(seq), s.d,
                     s.cap, s.Hkv, S);
  return launch_status(__func__);
}

// Zero the ticket counters at the head of the workspace (a fill kernel rather than
// a memset node, so the call can be recorded into a HIP graph).
__global__ void zero_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

hipError_t launch_zero_ints(int* p, int n, hipStream_t st) {
  hipLaunchKernelGGL(zero_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
  return launch_status(__func__);
}

hipError_t launch_workspace_init(const Shape& s, void* ws, hipStream_t st) {
  return launch_zero_ints((int*)ws, (int)(counter_bytes(s) / sizeof(int)), st);
}

hipError_t launch_append(const Shape& s, const lq_cache& c, const void* k_new, const void* v_new,
                         int n_new, hipStream_t st) {
  dim3 grid(n_new, s.B * s.Hkv);
  hipLaunchKernelGGL(append_kernel, grid, dim3(s.d), 0, st, (const uint16_t*)k_new,
                     (const uint16_t*)v_new, (uint16_t*)c.k_fp[c.cur], (uint16_t*)c.v_fp[c.cur],
                     c.pos_fp[c.cur], n_new, c.n_fp, c.n_fp + quantized_tokens(s, c.n_q), s.d, s.cap, s.Hkv);
  return launch_status(__func__);
}

}  // namespace lq
