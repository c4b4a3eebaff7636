// Filtering branch of Algorithm 1 (Sec. 2.5) plus quantization of what it removes
// (Fig. 6 caption, Sec. 2.3): logical fp rows 1,3,..,2W-1 are quantized to 2 bits
// (keys per channel over G evicted tokens, values per token over G channels) and
// appended to the quantized region; rows 0,2,..,2W-2 and 2W..3W-1 are moved to
// the front of the other fp buffer.
#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

// One group of values: zero z = min, scale s = T((max - min) / 3) with the
// difference and the quotient correctly rounded to fp32 (the fp64 quotient
// rounded once more to fp32 equals the IEEE fp32 quotient, 53 >= 2*24 + 2).
template <bool BF16>
__device__ __forceinline__ void group_params(float mn, float mx, float* z, float* s, uint16_t* zt,
                                             uint16_t* st) {
  if (mn == 0.f) mn = 0.f;  // -0 -> +0 (min/max do not order signed zeros)
  if (mx == 0.f) mx = 0.f;
  const float diff = mx - mn;
  const float quo = (float)((double)diff / 3.0);
  *st = f2t<BF16>(quo);
  *s = t2f<BF16>(*st);
  *zt = f2t<BF16>(mn);  // exact: mn is an element of T
  *z = mn;
}

// round-half-up of (x - z)/s clamped to 0..3, by threshold compares on the exact
// (fp64) difference.
__device__ __forceinline__ uint32_t code_of(float x, float z, float s) {
  const double dl = (double)x - (double)z;
  const double sd = (double)s;
  const uint32_t c = (uint32_t)(dl >= 0.5 * sd) + (uint32_t)(dl >= 1.5 * sd) + (uint32_t)(dl >= 2.5 * sd);
  return s == 0.f ? 0u : c;
}

// grid (W/G, B*Hkv), block 256.  Dynamic LDS: G * (d + 2) uint16.
template <bool BF16>
__global__ void __launch_bounds__(256)
quantize_kernel(const uint16_t* __restrict__ k_fp, const uint16_t* __restrict__ v_fp,
                const int32_t* __restrict__ pos_fp, uint32_t* __restrict__ k_codes,
                uint32_t* __restrict__ v_codes, uint16_t* __restrict__ k_scale,
                uint16_t* __restrict__ k_zero, uint16_t* __restrict__ v_scale,
                uint16_t* __restrict__ v_zero, int32_t* __restrict__ pos_q, int d, int G, int cap,
                int qcap, int n_q, int Hkv) {
  extern __shared__ uint16_t sm[];  // [G][d + 2]; values first, then their codes in place
  const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  const int nkc = d >> 5, nnt = d >> 4, ngc = (d + G - 1) / G, ld = d + 2;
  const int64_t fp_slice = (int64_t)bh * cap * d;
  const int q0 = n_q + j * G;  // first quantized slot written by this block
  const int64_t code_base = ((int64_t)bh * (qcap >> 5) + (q0 >> 5)) * 64 * nkc;

  // ---------------- keys ----------------
  for (int idx = tid; idx < G * nkc * 4; idx += 256) {
    const int oct = idx % (nkc * 4), e = idx / (nkc * 4);
    const int ts = 2 * (j * G + e) + 1;
    const uint4 v = *reinterpret_cast<const uint4*>(k_fp + fp_slice + k_fp_index(ts, oct * 8, nkc));
    uint32_t* dst = reinterpret_cast<uint32_t*>(sm + e * ld + oct * 8);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  __syncthreads();
  if (tid < d) {
    const int c = tid;
    float mn = INFINITY, mx = -INFINITY;
    for (int e = 0; e < G; ++e) {
      const float x = t2f<BF16>(sm[e * ld + c]);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    float z, s;
    uint16_t zt, st;
    group_params<BF16>(mn, mx, &z, &s, &zt, &st);
    const int64_t mi = ((int64_t)bh * (qcap / G) + q0 / G) * d + c;
    k_scale[mi] = st;
    k_zero[mi] = zt;
    for (int e = 0; e < G; ++e) sm[e * ld + c] = (uint16_t)code_of(t2f<BF16>(sm[e * ld + c]), z, s);
  }
  __syncthreads();
  for (int idx = tid; idx < (G >> 5) * 64 * nkc; idx += 256) {
    const int m = idx % nkc, lane = (idx / nkc) & 63, blk = idx / (nkc * 64);
    const int r = lane & 15, qq = lane >> 4;
    uint32_t w = 0;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int o = 2 * m + (jj >> 2);
      const int uu = o / nkc, kc = o % nkc;
      const int e = blk * 32 + 16 * uu + r;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int c = 32 * kc + 8 * qq + 2 * (jj & 3) + half;
        w |= (uint32_t)sm[e * ld + c] << (2 * jj + 16 * half);
      }
    }
    k_codes[code_base + idx] = w;
  }
  __syncthreads();

  // ---------------- values ----------------
  // source rows of this block: logical slots 2jG .. 2jG + 2G - 1 (whole 32-slot tiles)
  for (int idx = tid; idx < (2 * G >> 5) * nnt * 64; idx += 256) {
    const int lane = idx & 63, nt = (idx >> 6) % nnt, sb = idx / (64 * nnt);
    const int qq = lane >> 4, n = lane & 15;
    const int64_t src = fp_slice + ((((int64_t)((2 * j * G) >> 5) + sb) * nnt + nt) * 64 + lane) * 8;
    const uint4 v = *reinterpret_cast<const uint4*>(v_fp + src);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 1; i < 8; i += 2) {  // odd element <=> odd logical slot <=> evicted
      const int x = kperm_inv(8 * qq + i);
      const int e = (sb * 32 + x - 1) >> 1;
      sm[e * ld + 16 * nt + n] = (uint16_t)(w[i >> 1] >> 16);
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * ngc; idx += 256) {
    const int e = idx % G, gc = idx / G;
    const int lo = gc * G, hi = min(lo + G, d);
    float mn = INFINITY, mx = -INFINITY;
    for (int c = lo; c < hi; ++c) {
      const float x = t2f<BF16>(sm[e * ld + c]);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    float z, s;
    uint16_t zt, st;
    group_params<BF16>(mn, mx, &z, &s, &zt, &st);
    const int64_t mi = (int64_t)bh * (qcap >> 5) * ngc * 32 + v_meta_index(q0 + e, gc, ngc);
    v_scale[mi] = st;
    v_zero[mi] = zt;
    for (int c = lo; c < hi; ++c) sm[e * ld + c] = (uint16_t)code_of(t2f<BF16>(sm[e * ld + c]), z, s);
  }
  __syncthreads();
  for (int idx = tid; idx < (G >> 5) * 64 * nkc; idx += 256) {
    const int m = idx % nkc, lane = (idx / nkc) & 63, blk = idx / (nkc * 64);
    const int n = lane & 15, qq = lane >> 4;
    uint32_t w = 0;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int nt = 2 * m + (jj >> 2);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int k = 8 * qq + 2 * (jj & 3) + half;
        const int e = blk * 32 + kperm_inv(k);
        w |= (uint32_t)sm[e * ld + 16 * nt + n] << (2 * jj + 16 * half);
      }
    }
    v_codes[code_base + idx] = w;
  }
  // positions of the evicted tokens, once per batch row
  if (bh % Hkv == 0) {
    const int b = bh / Hkv;
    for (int e = tid; e < G; e += 256)
      pos_q[(int64_t)b * qcap + q0 + e] = pos_fp[b * cap + 2 * (j * G + e) + 1];
  }
}

// Kept rows -> rows 0..2W-1 of the other fp buffer.  grid (2W/32, B*Hkv), block 256.
__global__ void __launch_bounds__(256)
compact_kernel(const uint16_t* __restrict__ k_old, const uint16_t* __restrict__ v_old,
               const int32_t* __restrict__ pos_old, uint16_t* __restrict__ k_new,
               uint16_t* __restrict__ v_new, int32_t* __restrict__ pos_new, int d, int W, int cap,
               int Hkv) {
  const int nb = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  const int nkc = d >> 5, nnt = d >> 4;
  const int64_t slice = (int64_t)bh * cap * d;
  for (int idx = tid; idx < 32 * nkc * 4; idx += 256) {
    const int x = idx & 31, oct = idx >> 5;
    const int tn = nb * 32 + x;
    const int ts = tn < W ? 2 * tn : tn + W;
    *reinterpret_cast<uint4*>(k_new + slice + k_fp_index(tn, oct * 8, nkc)) =
        *reinterpret_cast<const uint4*>(k_old + slice + k_fp_index(ts, oct * 8, nkc));
  }
  for (int idx = tid; idx < nnt * 64; idx += 256) {
    const int lane = idx & 63, nt = idx >> 6;
    const int qq = lane >> 4, n = lane & 15;
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tn = nb * 32 + kperm_inv(8 * qq + i);
      const int ts = tn < W ? 2 * tn : tn + W;
      const uint32_t e = v_old[slice + v_fp_index(ts, 16 * nt + n, nnt)];
      w[i >> 1] |= e << (16 * (i & 1));
    }
    *reinterpret_cast<uint4*>(v_new + slice + (((int64_t)nb * nnt + nt) * 64 + lane) * 8) =
        make_uint4(w[0], w[1], w[2], w[3]);
  }
  if (bh % Hkv == 0 && tid < 32) {
    const int b = bh / Hkv, tn = nb * 32 + tid;
    const int ts = tn < W ? 2 * tn : tn + W;
    pos_new[b * cap + tn] = pos_old[b * cap + ts];
  }
}

hipError_t launch_compress(const Shape& s, const lq_cache& c, hipStream_t st) {
  const int cur = c.cur, alt = cur ^ 1;
  const size_t lds = (size_t)s.G * (s.d + 2) * sizeof(uint16_t);
  dim3 grid(s.W / s.G, s.B * s.Hkv);
  auto kern = s.bf16 ? quantize_kernel<true> : quantize_kernel<false>;
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const uint16_t*)c.k_fp[cur],
                     (const uint16_t*)c.v_fp[cur], c.pos_fp[cur], c.k_codes, c.v_codes,
                     (uint16_t*)c.k_scale, (uint16_t*)c.k_zero, (uint16_t*)c.v_scale,
                     (uint16_t*)c.v_zero, c.pos_q, s.d, s.G, s.cap, s.qcap, c.n_q, s.Hkv);
  hipError_t e = launch_status(__func__);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(compact_kernel, dim3(2 * s.W / 32, s.B * s.Hkv), dim3(256), 0, st,
                     (const uint16_t*)c.k_fp[cur], (const uint16_t*)c.v_fp[cur], c.pos_fp[cur],
                     (uint16_t*)c.k_fp[alt], (uint16_t*)c.v_fp[alt], c.pos_fp[alt], s.d, s.W, s.cap,
                     s.Hkv);
  return launch_status(__func__);
}

}  // namespace lq
