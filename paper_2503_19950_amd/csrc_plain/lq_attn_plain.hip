// Decode attention, plain formulation (Eq. 2 with Eq. 6's 1/sqrt(d); Sec. 2.4: one
// softmax over the original-precision rows and the dequantized rows) on the vector unit.
// One wavefront walks tokens one at a time, lanes own channels, the running
// (max, sum, output) triple is merged across wavefronts and context splits by a second
// launch.  Slow and simple: it reads every element through the layout index functions.
//
// NOT part of the product library: this file is built into liblogquant_plain.so, which
// only the tests (cross-check of the matrix-instruction kernel) and the benchmark's
// --plain-valu measurement (matrix unit against vector unit) load.  It takes shapes,
// plans and the workspace layout from liblogquant.so.
#include <math.h>

#include "../csrc/lq_device.h"
#include "../csrc/lq_internal.h"

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

// Log-sum-exp merge of the splits' partials (softmax normalisation of Eq. 2).
// One workgroup per (batch row, query head); threads = channels x PARTS, each part
// takes every PARTS-th split.
template <bool BF16>
__global__ void __launch_bounds__(512)
combine_kernel(const float* __restrict__ ws, uint16_t* __restrict__ out, int d, int gh, int splits) {
  __shared__ float w_s[256];        // weight of each split (splits <= 256)
  __shared__ float red[512];
  __shared__ float stat[2];
  const int bhq = blockIdx.x, tid = threadIdx.x;
  const int bh = bhq / gh, g = bhq % gh;
  const int64_t stride = (int64_t)gh * (d + 4);
  const float* base = ws + ((int64_t)bh * splits * gh + g) * (d + 4);
  // weights: w_s = 2^(m_s - M); L = sum_s w_s l_s
  float m = -INFINITY, l = 0.f;
  if (tid < splits) { m = base[tid * stride + d]; l = base[tid * stride + d + 1]; }
  red[tid] = m;
  __syncthreads();
  for (int k = 256; k >= 1; k >>= 1) {
    if (tid < k) red[tid] = fmaxf(red[tid], red[tid + k]);
    __syncthreads();
  }
  const float M = red[0];
  __syncthreads();
  const float w = (tid < splits && m != -INFINITY) ? exp2f(m - M) : 0.f;
  if (tid < 256) w_s[tid] = w;
  red[tid] = w * l;
  __syncthreads();
  for (int k = 256; k >= 1; k >>= 1) {
    if (tid < k) red[tid] += red[tid + k];
    __syncthreads();
  }
  if (tid == 0) stat[0] = red[0];
  __syncthreads();
  const float L = stat[0];
  __syncthreads();
  const int parts = 512 / d;
  const int c = tid % d, part = tid / d;
  float acc = 0.f;
  if (part < parts) {
#pragma unroll 8
    for (int s = part; s < splits; s += parts) acc = fmaf(w_s[s], base[s * stride + c], acc);
  }
  red[tid] = acc;
  __syncthreads();
  if (tid < d) {
    float o = 0.f;
    for (int pth = 0; pth < parts; ++pth) o += red[pth * d + tid];
    out[(int64_t)bhq * d + tid] = f2t<BF16>(o / L);
  }
}

static hipError_t launch_combine(const Shape& s, const float* ws, void* out, int splits, hipStream_t st) {
  auto kern = s.bf16 ? combine_kernel<true> : combine_kernel<false>;
  hipLaunchKernelGGL(kern, dim3(s.B * s.Hq), dim3(512), 0, st, ws, (uint16_t*)out, s.d, s.gh, splits);
  return launch_status(__func__);
}

template <bool BF16, int HB>
static hipError_t launch_plain_t(const Shape& s, const lq_cache& c, const void* q, float scale,
                                 void* ws, int splits, hipStream_t st) {
  dim3 grid(splits, s.B * s.Hkv * (s.gh / HB));
  hipLaunchKernelGGL((attn_ref_kernel<BF16, HB>), grid, dim3(256), 0, st, (const uint16_t*)q,
                     (const uint16_t*)c.k_fp[c.cur], (const uint16_t*)c.v_fp[c.cur],
                     (const uint16_t*)c.k_fp[c.cur ^ 1], (const uint16_t*)c.v_fp[c.cur ^ 1], (const SeqState*)nullptr,
                     c.k_codes, c.v_codes, (const uint16_t*)c.k_scale, (const uint16_t*)c.k_zero,
                     (const uint16_t*)c.v_scale, (const uint16_t*)c.v_zero, (float*)ws, s.d, s.G,
                     s.cap, s.qcap, c.n_fp, c.n_q, s.gh, splits, scale * 1.4426950408889634f, s.bits,
                     s.W, s.Wq, s.Hkv);
  return launch_status(__func__);
}

}  // namespace lq

using namespace lq;

// Same arguments, requirements and results as logquant_decode_attn (lock-step batch); the
// context is cut into the number of splits the product's planner picks.
extern "C" lq_status logquant_plain_decode_attn(const lq_config* cfg, const lq_cache* cache, const void* q,
                                                float softmax_scale, void* out, void* workspace, void* stream) {
  if (!cfg || !cache || !q || !out || !workspace) return LQ_ERR_NULL;
  Shape s;
  lq_status st = make_shape(cfg, &s);
  if (st != LQ_OK) return st;
  if (cache->n_fp + cache->n_q < 1) return LQ_ERR_STATE;
  lq_plan plan;
  plan_decode(s, cache->n_fp, cache->n_q, &plan);
  if (!(softmax_scale > 0.f)) softmax_scale = 1.0f / sqrtf((float)s.d);
  clear_stale_error();
  void* ws = split_workspace(s, workspace).partials;
  const int hb = s.gh % 4 == 0 ? 4 : (s.gh % 2 == 0 ? 2 : 1);
  hipStream_t hs = (hipStream_t)stream;
  hipError_t e;
  if (s.bf16) {
    e = hb == 4 ? launch_plain_t<true, 4>(s, *cache, q, softmax_scale, ws, plan.splits, hs)
        : hb == 2 ? launch_plain_t<true, 2>(s, *cache, q, softmax_scale, ws, plan.splits, hs)
                  : launch_plain_t<true, 1>(s, *cache, q, softmax_scale, ws, plan.splits, hs);
  } else {
    e = hb == 4 ? launch_plain_t<false, 4>(s, *cache, q, softmax_scale, ws, plan.splits, hs)
        : hb == 2 ? launch_plain_t<false, 2>(s, *cache, q, softmax_scale, ws, plan.splits, hs)
                  : launch_plain_t<false, 1>(s, *cache, q, softmax_scale, ws, plan.splits, hs);
  }
  if (e != hipSuccess) return LQ_ERR_HIP;
  return launch_combine(s, (const float*)ws, out, plan.splits, hs) == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
