// Decode attention, plain formulation (Eq. 2 with Eq. 6's 1/sqrt(d); Sec. 2.4: one
// softmax over the original-precision rows and the dequantized rows).  One
// wavefront walks tokens one at a time, lanes own channels, the running
// (max, sum, output) triple is merged across wavefronts and context splits.
// Slow and simple: it reads every element through the layout index functions.
// Kept as the cross-check of the matrix-instruction kernel.
#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}

// grid (splits, B*Hkv*(gh/HB)), block 256 (4 wavefronts).
template <bool BF16, int HB>
__global__ void __launch_bounds__(256)
attn_ref_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_fp0,
                const uint16_t* __restrict__ v_fp0, const uint16_t* __restrict__ k_fp1,
                const uint16_t* __restrict__ v_fp1, const SeqState* __restrict__ seq,
                const uint32_t* __restrict__ k_codes,
                const uint32_t* __restrict__ v_codes, const uint16_t* __restrict__ k_scale,
                const uint16_t* __restrict__ k_zero, const uint16_t* __restrict__ v_scale,
                const uint16_t* __restrict__ v_zero, float* __restrict__ ws, int d, int G, int cap,
                int qcap, int n_fp, int n_q, int gh, int splits, float scale_log2e, int bits, int W,
                int Wq, int Hkv) {
  __shared__ float sm_o[4][HB][128];
  __shared__ float sm_ml[4][HB][2];
  const int split = blockIdx.x;
  const int hsub = blockIdx.y % (gh / HB), bh = blockIdx.y / (gh / HB);
  const uint16_t* k_fp = k_fp0;
  const uint16_t* v_fp = v_fp0;
  if (seq) {   // per-sequence lengths and live buffers
    const SeqState sq = seq[bh / Hkv];
    n_fp = sq.n_fp; n_q = sq.n_q;
    if (sq.cur) { k_fp = k_fp1; v_fp = v_fp1; }
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nkc = d >> 5, nnt = d >> 4, ngc = (d + G - 1) / G;
  const int T = n_fp + n_q;
  const int chunk = (T + splits - 1) / splits;
  const int t0 = split * chunk, t1 = min(T, t0 + chunk);
  const int c0 = lane, c1 = lane + 64;
  const bool has1 = c1 < d, has0 = c0 < d;

  float qv[HB][2];
#pragma unroll
  for (int g = 0; g < HB; ++g) {
    const int64_t qi = ((int64_t)bh * gh + hsub * HB + g) * d;
    qv[g][0] = has0 ? t2f<BF16>(q[qi + c0]) * scale_log2e : 0.f;
    qv[g][1] = has1 ? t2f<BF16>(q[qi + c1]) * scale_log2e : 0.f;
  }
  float m[HB], l[HB], o[HB][2];
#pragma unroll
  for (int g = 0; g < HB; ++g) { m[g] = -INFINITY; l[g] = 0.f; o[g][0] = o[g][1] = 0.f; }

  const int64_t fp_slice = (int64_t)bh * cap * d;
  const int64_t code_slice = (int64_t)bh * (qcap >> 5) * 64 * nkc * (bits >> 1);
  const uint32_t cmask = (1u << bits) - 1u;
  const int64_t kmeta_slice = (int64_t)bh * (qcap / G) * d;
  const int64_t vmeta_slice = (int64_t)bh * (qcap >> 5) * ngc * 32;

  for (int t = t0 + wave; t < t1; t += 4) {
    if (t >= n_fp && (t - n_fp) % Wq >= W) continue;   // padding slot behind a short key group
    float kx[2] = {0.f, 0.f}, vx[2] = {0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int c = e ? c1 : c0;
      if (c >= d) continue;
      if (t < n_fp) {
        kx[e] = t2f<BF16>(k_fp[fp_slice + k_fp_index(t, c, nkc)]);
        vx[e] = t2f<BF16>(v_fp[fp_slice + v_fp_index(t, c, nnt)]);
      } else {
        const int s = t - n_fp;
        {  // key code, scale, zero
          const int o_ = ((s & 31) >> 4) * nkc + (c >> 5);
          const int64_t ln = ((int64_t)(s >> 5)) * 64 + 16 * ((c & 31) >> 3) + (s & 15);
          const int64_t w = bits == 2 ? ln * nkc + (o_ >> 1) : ln * 2 * nkc + o_;
          const int bit = bits == 2 ? 8 * (o_ & 1) + 2 * ((c & 7) >> 1) + 16 * (c & 1)
                                    : 4 * ((c & 7) >> 1) + 16 * (c & 1);
          const float code = (float)((k_codes[code_slice + w] >> bit) & cmask);
          const int64_t mi = kmeta_slice + (int64_t)(s / G) * d + c;
          kx[e] = fmaf(code, t2f<false>(k_scale[mi]), t2f<false>(k_zero[mi]));   // parameters are stored as fp16
        }
        {  // value code, scale, zero
          const int k = kperm(s & 31);
          const int64_t ln = ((int64_t)(s >> 5)) * 64 + 16 * (k >> 3) + (c & 15);
          const int64_t w = bits == 2 ? ln * nkc + ((c >> 4) >> 1) : ln * 2 * nkc + (c >> 4);
          const int bit = bits == 2 ? 8 * ((c >> 4) & 1) + 2 * ((k & 7) >> 1) + 16 * (k & 1)
                                    : 4 * ((k & 7) >> 1) + 16 * (k & 1);
          const float code = (float)((v_codes[code_slice + w] >> bit) & cmask);
          const int64_t mi = vmeta_slice + v_meta_index(s, c / G, ngc);
          vx[e] = fmaf(code, t2f<false>(v_scale[mi]), t2f<false>(v_zero[mi]));
        }
      }
    }
#pragma unroll
    for (int g = 0; g < HB; ++g) {
      const float s = wave_sum(qv[g][0] * kx[0] + qv[g][1] * kx[1]);   // log2-domain logit
      const float mn = fmaxf(m[g], s);
      const float a = exp2f(m[g] - mn), p = exp2f(s - mn);
      l[g] = l[g] * a + p;
      o[g][0] = o[g][0] * a + p * vx[0];
      o[g][1] = o[g][1] * a + p * vx[1];
      m[g] = mn;
    }
  }
#pragma unroll
  for (int g = 0; g < HB; ++g) {
    sm_o[wave][g][c0] = o[g][0];
    sm_o[wave][g][c1] = o[g][1];
    if (lane == 0) { sm_ml[wave][g][0] = m[g]; sm_ml[wave][g][1] = l[g]; }
  }
  __syncthreads();
  // merge the four wavefronts, write the split's partial: per head d floats of o, then m, l
  for (int idx = threadIdx.x; idx < HB * d; idx += 256) {
    const int g = idx / d, c = idx % d;
    float M = -INFINITY;
    for (int w = 0; w < 4; ++w) M = fmaxf(M, sm_ml[w][g][0]);
    float acc = 0.f, L = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float a = sm_ml[w][g][0] == -INFINITY ? 0.f : exp2f(sm_ml[w][g][0] - M);
      acc += a * sm_o[w][g][c];
      L += a * sm_ml[w][g][1];
    }
    const int64_t base = (((int64_t)bh * splits + split) * gh + hsub * HB + g) * (d + 4);
    ws[base + c] = acc;
    if (c == 0) { ws[base + d] = M; ws[base + d + 1] = L; }
  }
}

hipError_t launch_combine(const Shape& s, const float* ws, void* out, int splits, hipStream_t st);

template <bool BF16, int HB>
static hipError_t launch_ref_t(const Shape& s, const lq_cache& c, const void* q, float scale,
                               void* ws, int splits, hipStream_t st, const SeqState* seq) {
  dim3 grid(splits, s.B * s.Hkv * (s.gh / HB));
  const int first = seq ? 0 : c.cur;
  hipLaunchKernelGGL((attn_ref_kernel<BF16, HB>), grid, dim3(256), 0, st, (const uint16_t*)q,
                     (const uint16_t*)c.k_fp[first], (const uint16_t*)c.v_fp[first],
                     (const uint16_t*)c.k_fp[first ^ 1], (const uint16_t*)c.v_fp[first ^ 1], seq, c.k_codes,
                     c.v_codes, (const uint16_t*)c.k_scale, (const uint16_t*)c.k_zero,
                     (const uint16_t*)c.v_scale, (const uint16_t*)c.v_zero, (float*)ws, s.d, s.G,
                     s.cap, s.qcap, c.n_fp, c.n_q, s.gh, splits, scale * 1.4426950408889634f, s.bits,
                     s.W, s.Wq, s.Hkv);
  return launch_status(__func__);
}

hipError_t launch_decode_attn_ref(const Shape& s, const lq_cache& c, const void* q, float scale,
                                  void* out, const Workspace& ws_all, int splits, hipStream_t st, const SeqArg* arg) {
  // this kernel reads per-sequence state from the device array only: fill it here when
  // the batch is small enough that the caller left it to the launch's arguments
  const SeqState* seq = arg ? arg->dev : nullptr;
  if (arg && arg->in_args() &&
      launch_seq_upload(const_cast<SeqState*>(arg->dev), arg->host, arg->n, st) != hipSuccess)
    return hipErrorLaunchFailure;
  void* ws = ws_all.partials;
  const int hb = s.gh % 4 == 0 ? 4 : (s.gh % 2 == 0 ? 2 : 1);
  hipError_t e;
  if (s.bf16) {
    e = hb == 4 ? launch_ref_t<true, 4>(s, c, q, scale, ws, splits, st, seq)
        : hb == 2 ? launch_ref_t<true, 2>(s, c, q, scale, ws, splits, st, seq)
                  : launch_ref_t<true, 1>(s, c, q, scale, ws, splits, st, seq);
  } else {
    e = hb == 4 ? launch_ref_t<false, 4>(s, c, q, scale, ws, splits, st, seq)
        : hb == 2 ? launch_ref_t<false, 2>(s, c, q, scale, ws, splits, st, seq)
                  : launch_ref_t<false, 1>(s, c, q, scale, ws, splits, st, seq);
  }
  if (e != hipSuccess) return e;
  return launch_combine(s, (const float*)ws, out, splits, st);
}

}  // namespace lq
