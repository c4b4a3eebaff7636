// Fused decode attention for gfx950 (Eq. 2 with Eq. 6's 1/sqrt(d), one softmax over
// the original-precision rows and the 2-bit rows, Sec. 2.4).  The 2-bit rows are
// never dequantized in memory:
//
//   logits   q.k_hat_t = sum_c q_c z_c + sum_c (q_c s_c) code_tc
//            -> per key group (G tokens) the products q_c s_c are formed once, split
//               into an fp16 head and an fp16 tail (together exact for 11-bit or
//               8-bit factors) and become the B operands of two 16x16x32 matrix
//               instructions whose A operand is the code tile; sum_c q_c z_c is a
//               per-group bias.  (A single fp16 rounding of q_c s_c is not enough:
//               with outlier channels its error alone moves the logits by ~1e-2.)
//   output   sum_t p_t v_hat_tc = sum_t p_t vz_t + sum_t (p_t vs_t) code_tc
//            -> p_t vs_t (one per token and channel group) is the A operand, the
//               code tile the B operand; sum_t p_t vz_t is kept per channel group.
//
// A 2-bit code sits in the low mantissa bits of an fp16 lane of the operand, i.e.
// it is the subnormal number code * 2^-24; gfx950's matrix cores take subnormal
// operands exactly, so unpacking is a shift and a mask for two codes at a time and
// needs no integer-to-float conversion.
//
// The up to four query heads that share a kv head occupy four of the 16 columns of
// the logits tile; the other twelve columns repeat them for three more 16-token
// tiles, so one accumulator quad per lane ends up holding logits of 64 tokens x 4
// heads with every lane busy in the softmax.
//
// Work split: a workgroup has four independent wavefronts; the wavefronts of all
// workgroups of one (batch row, kv head) are numbered 0..NW-1, the first `nwf` walk
// the fp rows in units of 32, the others walk the quantized rows in tiles of 64,
// each taking every NWQ-th tile so that all wavefronts sweep memory side by side.
// Partial (max, sum, output) triples are merged in LDS per workgroup and written
// to the workspace; a second small kernel merges the splits.
#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

struct AttnParams {
  const uint16_t* q;
  const uint16_t* k_fp;
  const uint16_t* v_fp;
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const uint16_t* k_scale;
  const uint16_t* k_zero;
  const uint16_t* v_scale;
  const uint16_t* v_zero;
  float* ws;
  int cap, qcap, n_fp, n_q, gh, hb, splits, nwf;
  float c;  // softmax scale * log2(e)
};

__device__ __forceinline__ floatx4 mfma_f16(uint4 a, uint4 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a),
                                                __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ floatx4 mfma_bf16(uint4 a, uint4 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                 __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
template <bool BF16>
__device__ __forceinline__ floatx4 mfma_T(uint4 a, uint4 b, floatx4 c) {
  if constexpr (BF16) return mfma_bf16(a, b, c); else return mfma_f16(a, b, c);
}

// Eight codes of one operand: register v gets the codes at bits 2(j0+v) and
// 2(j0+v)+16 of `w` in the low two bits of its two fp16 lanes (value code * 2^-24).
__device__ __forceinline__ uint4 unpack4(uint32_t w, int j0) {
  uint4 r;
  r.x = (w >> (2 * j0)) & 0x00030003u;
  r.y = (w >> (2 * j0 + 2)) & 0x00030003u;
  r.z = (w >> (2 * j0 + 4)) & 0x00030003u;
  r.w = (w >> (2 * j0 + 6)) & 0x00030003u;
  return r;
}

__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
  half2_t h = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, h);
}
template <bool BF16>
__device__ __forceinline__ uint32_t pack_T(float a, float b) {
  if constexpr (BF16) return (uint32_t)f2t<true>(a) | ((uint32_t)f2t<true>(b) << 16);
  else return pack_f16(a, b);
}
template <bool BF16>
__device__ __forceinline__ float lo_T(uint32_t w) {
  if constexpr (BF16) return __uint_as_float(w << 16);
  else return (float)__builtin_bit_cast(half2_t, w)[0];
}
template <bool BF16>
__device__ __forceinline__ float hi_T(uint32_t w) {
  if constexpr (BF16) return __uint_as_float(w & 0xFFFF0000u);
  else return (float)__builtin_bit_cast(half2_t, w)[1];
}
template <bool BF16>
__device__ __forceinline__ void unpack8_T(uint4 v, float* f) {
  f[0] = lo_T<BF16>(v.x); f[1] = hi_T<BF16>(v.x); f[2] = lo_T<BF16>(v.y); f[3] = hi_T<BF16>(v.y);
  f[4] = lo_T<BF16>(v.z); f[5] = hi_T<BF16>(v.z); f[6] = lo_T<BF16>(v.w); f[7] = hi_T<BF16>(v.w);
}

// all-reduce over the 16 lanes that share lane & 3 (one query head)
__device__ __forceinline__ float head_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 4));
  v = fmaxf(v, __shfl_xor(v, 8));
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ __forceinline__ float head_sum(float v) {
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 8);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

// LDS-visible ordering inside one wavefront (no workgroup barrier needed: DS
// instructions of a wavefront execute in order).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int N>
struct Words { uint32_t w[N]; };

// Running softmax state of one wavefront.  m, l, zacc belong to head (lane & 3);
// acc[nt][j] is output row 4*(lane>>4)+j, column lane&15 of channel tile nt.
template <int NNT>
struct State {
  floatx4 acc[NNT];
  float m, l, zacc;
};

// s[0..3]: log2-domain logits of this lane's four tokens -> p[0..3]; updates state.
template <int NNT>
__device__ __forceinline__ void online_softmax(State<NNT>& st, const float* s, float* p) {
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  mx = head_max(mx);
  const float m_new = fmaxf(st.m, mx);
  if (__any(m_new > st.m)) {
    const float alpha = exp2f(st.m - m_new);   // 0 on the first tile (m = -inf)
    st.l *= alpha;
    st.zacc *= alpha;
    float a4[4];
#pragma unroll
    for (int gg = 0; gg < 4; ++gg) a4[gg] = __shfl(alpha, (threadIdx.x & 60) | gg);
#pragma unroll
    for (int nt = 0; nt < NNT; ++nt) {
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) st.acc[nt][gg] *= a4[gg];
    }
    st.m = m_new;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) p[j] = exp2f(s[j] - st.m);
  st.l += (p[0] + p[1]) + (p[2] + p[3]);
}

template <bool BF16, int D, int G>
__global__ void __launch_bounds__(256)
attn_mfma_kernel(const AttnParams P) {
  constexpr int NKC = D / 32, NNT = D / 16, NGC = (D + G - 1) / G;
  constexpr int NGRP = G < 64 ? 64 / G : 1;     // key groups per 64-token tile
  __shared__ __attribute__((aligned(16))) uint16_t qs_lds[4][NGRP][2][4][D];   // fp16 head/tail of q*s per wave
  __shared__ float o_lds[4][4][D];
  __shared__ float ml_lds[4][4][2];
  __shared__ float zs_lds[4][4][4];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nhg = P.gh / P.hb;
  const int split = blockIdx.x, hsub = blockIdx.y % nhg, bh = blockIdx.y / nhg;
  const int q4 = lane >> 4, n16 = lane & 15, up = n16 >> 2, g = lane & 3;
  const bool head_ok = g < P.hb;
  const int64_t qrow = ((int64_t)bh * P.gh + hsub * P.hb + (head_ok ? g : 0)) * D;

  const int NW = P.splits * 4, NWF = P.nwf, NWQ = NW - NWF;
  const int gw = split * 4 + wave;
  const int TQ = (P.n_q + 63) >> 6, TF = (P.n_fp + 31) >> 5;

  State<NNT> st;
#pragma unroll
  for (int nt = 0; nt < NNT; ++nt) st.acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY; st.l = 0.f; st.zacc = 0.f;

  if (gw >= NWF) {
    // ------------------------- quantized rows -------------------------
    const int wq = gw - NWF;
    const int64_t code_slice = (int64_t)bh * (P.qcap >> 5) * 64 * NKC;
    const uint32_t* kcb = P.k_codes + code_slice + lane * NKC;
    const uint32_t* vcb = P.v_codes + code_slice + lane * NKC;
    const uint16_t* ksb = P.k_scale + (int64_t)bh * (P.qcap / G) * D;
    const uint16_t* kzb = P.k_zero + (int64_t)bh * (P.qcap / G) * D;
    const int64_t vm_slice = (int64_t)bh * (P.qcap >> 5) * NGC * 32;
    const int upc = up < NGC ? up : 0;
    const uint16_t* vsb = P.v_scale + vm_slice + upc * 32 + 8 * q4;
    const uint16_t* vzb = P.v_zero + vm_slice + upc * 32 + 8 * q4;
    const int c8 = lane >> 2;                 // channel octet this lane prepares q*s for
    const bool prep = 8 * c8 < D;
    const int c8c = prep ? c8 : 0;

    float qv[8];
    {
      const uint4 raw = *reinterpret_cast<const uint4*>(P.q + qrow + 8 * c8c);
      unpack8_T<BF16>(raw, qv);
      if (!prep || !head_ok) {
#pragma unroll
        for (int i = 0; i < 8; ++i) qv[i] = 0.f;
      }
    }
    const float c24 = P.c * 16777216.f;       // codes enter as code * 2^-24

    struct Tile {
      Words<NKC> kc[2], vc[2];
      uint4 vs[2], vz[2];
      uint4 ks8[NGRP], kz8[NGRP];
    };
    auto load_tile = [&](int t) {
      Tile T;
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        T.kc[b2] = *reinterpret_cast<const Words<NKC>*>(kcb + (int64_t)(2 * t + b2) * 64 * NKC);
        T.vc[b2] = *reinterpret_cast<const Words<NKC>*>(vcb + (int64_t)(2 * t + b2) * 64 * NKC);
        T.vs[b2] = *reinterpret_cast<const uint4*>(vsb + (int64_t)(2 * t + b2) * NGC * 32);
        T.vz[b2] = *reinterpret_cast<const uint4*>(vzb + (int64_t)(2 * t + b2) * NGC * 32);
      }
#pragma unroll
      for (int e = 0; e < NGRP; ++e) {
        const int grp = G <= 64 ? t * NGRP + e : t / (G / 64);
        T.ks8[e] = *reinterpret_cast<const uint4*>(ksb + (int64_t)grp * D + 8 * c8c);
        T.kz8[e] = *reinterpret_cast<const uint4*>(kzb + (int64_t)grp * D + 8 * c8c);
      }
      return T;
    };

    if (wq < TQ) {
      Tile cur = load_tile(wq);
      for (int t = wq; t < TQ; t += NWQ) {
        const int tn = t + NWQ < TQ ? t + NWQ : t;
        Tile nxt = load_tile(tn);

        // ---- q*s (fp16) and bias = sum_c q_c z_c for each key group of the tile
        float bias[NGRP];
#pragma unroll
        for (int e = 0; e < NGRP; ++e) {
          float s8[8], z8[8];
          unpack8_T<BF16>(cur.ks8[e], s8);
          unpack8_T<BF16>(cur.kz8[e], z8);
          float bp = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) bp = fmaf(qv[i], z8[i], bp);
          if (prep) {
            float x[8], r[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              x[i] = qv[i] * s8[i];
              r[i] = x[i] - (float)(_Float16)x[i];
            }
            uint4 h, l;
            h.x = pack_f16(x[0], x[1]); h.y = pack_f16(x[2], x[3]);
            h.z = pack_f16(x[4], x[5]); h.w = pack_f16(x[6], x[7]);
            l.x = pack_f16(r[0], r[1]); l.y = pack_f16(r[2], r[3]);
            l.z = pack_f16(r[4], r[5]); l.w = pack_f16(r[6], r[7]);
            *reinterpret_cast<uint4*>(&qs_lds[wave][e][0][g][8 * c8]) = h;
            *reinterpret_cast<uint4*>(&qs_lds[wave][e][1][g][8 * c8]) = l;
          }
          bias[e] = head_sum(bp) * P.c;
        }
        wave_lds_sync();

        // ---- logits: four 16-token tiles x NKC channel chunks
        floatx4 Du[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) Du[u] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < NGRP; ++e) {
#pragma unroll
          for (int kc = 0; kc < NKC; ++kc) {
            const uint4 bh_ = *reinterpret_cast<const uint4*>(&qs_lds[wave][e][0][g][32 * kc + 8 * q4]);
            const uint4 bl_ = *reinterpret_cast<const uint4*>(&qs_lds[wave][e][1][g][32 * kc + 8 * q4]);
#pragma unroll
            for (int u = e * (4 / NGRP); u < (e + 1) * (4 / NGRP); ++u) {
              const int o = (u & 1) * NKC + kc;
              const uint4 a = unpack4(cur.kc[u >> 1].w[o >> 1], 4 * (o & 1));
              Du[u] = mfma_f16(a, bh_, Du[u]);
              Du[u] = mfma_f16(a, bl_, Du[u]);
            }
          }
        }
        wave_lds_sync();   // qs_lds is rewritten by the next tile

        float s[4], p[4];
        {
          const floatx4 d = up == 0 ? Du[0] : up == 1 ? Du[1] : up == 2 ? Du[2] : Du[3];
          const float b = bias[NGRP == 1 ? 0 : (up * NGRP) >> 2];
          const int tok0 = 64 * t + 16 * up + 4 * q4;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            s[j] = fmaf(d[j], c24, b);
            if (tok0 + j >= P.n_q) s[j] = -INFINITY;
          }
        }
        online_softmax<NNT>(st, s, p);

        // ---- output: two 32-token steps x NNT channel tiles
        const bool partial = 64 * t + 64 > P.n_q;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          float pv[8], vs8[8], vz8[8];
          const int src0 = (lane & 0x33) | ((2 * ks) << 2), src1 = (lane & 0x33) | ((2 * ks + 1) << 2);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            pv[j] = __shfl(p[j], src0);
            pv[4 + j] = __shfl(p[j], src1);
          }
          unpack8_T<BF16>(cur.vs[ks], vs8);
          unpack8_T<BF16>(cur.vz[ks], vz8);
          if (partial) {   // slots beyond n_q hold unspecified bits: keep them out of the sums
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const int x = 16 * ((i >> 2) & 1) + 4 * q4 + (i & 3);   // slot of k = 8*q4 + i in its 32-block
              if (64 * t + 32 * ks + x >= P.n_q) { vs8[i] = 0.f; vz8[i] = 0.f; }
            }
          }
          float ps[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            ps[i] = up < NGC ? pv[i] * vs8[i] * 256.f : 0.f;
            st.zacc = up < NGC ? fmaf(pv[i], vz8[i], st.zacc) : st.zacc;
          }
          uint4 a;
          a.x = pack_f16(ps[0], ps[1]); a.y = pack_f16(ps[2], ps[3]);
          a.z = pack_f16(ps[4], ps[5]); a.w = pack_f16(ps[6], ps[7]);
#pragma unroll
          for (int nt = 0; nt < NNT; ++nt) {
            const uint4 b = unpack4(cur.vc[ks].w[nt >> 1], 4 * (nt & 1));
            st.acc[nt] = mfma_f16(a, b, st.acc[nt]);
          }
        }
        cur = nxt;
      }
    }
    // canonical partial of this wavefront: o[g][c], m[g], l[g]
    const float l_tot = head_sum(st.l);
    float zs = st.zacc;
    zs += __shfl_xor(zs, 16);
    zs += __shfl_xor(zs, 32);
    if (q4 == 0) zs_lds[wave][up][g] = zs;
    if (lane < 4) { ml_lds[wave][g][0] = st.m; ml_lds[wave][g][1] = l_tot; }
    wave_lds_sync();
#pragma unroll
    for (int nt = 0; nt < NNT; ++nt) {
      const int gc = (16 * nt) / G;
      if (q4 == gc) {
#pragma unroll
        for (int gg = 0; gg < 4; ++gg)
          o_lds[wave][gg][16 * nt + n16] = st.acc[nt][gg] * 65536.f + zs_lds[wave][gc][gg];
      }
    }
  } else {
    // ------------------------- original-precision rows -------------------------
    const int wf = gw;
    const int64_t fp_slice = (int64_t)bh * P.cap * D;
    const uint16_t* kb = P.k_fp + fp_slice + lane * 8;
    const uint16_t* vb = P.v_fp + fp_slice + lane * 8;
    uint4 qreg[NKC];
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
      qreg[kc] = *reinterpret_cast<const uint4*>(P.q + qrow + 32 * kc + 8 * q4);
      if (!head_ok) qreg[kc] = make_uint4(0, 0, 0, 0);
    }
    for (int unit = wf; unit < TF; unit += NWF) {
      uint4 ka[2][NKC], va[NNT];
#pragma unroll
      for (int uu = 0; uu < 2; ++uu)
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc)
          ka[uu][kc] = *reinterpret_cast<const uint4*>(kb + ((int64_t)(2 * unit + uu) * NKC + kc) * 512);
#pragma unroll
      for (int nt = 0; nt < NNT; ++nt)
        va[nt] = *reinterpret_cast<const uint4*>(vb + ((int64_t)unit * NNT + nt) * 512);

      floatx4 Du[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int kc = 0; kc < NKC; ++kc) {
        Du[0] = mfma_T<BF16>(ka[0][kc], qreg[kc], Du[0]);
        Du[1] = mfma_T<BF16>(ka[1][kc], qreg[kc], Du[1]);
      }
      float s[4], p[4];
      {
        const floatx4 d = up == 0 ? Du[0] : Du[1];
        const int tok0 = 32 * unit + 16 * up + 4 * q4;
#pragma unroll
        for (int j = 0; j < 4; ++j) s[j] = (up < 2 && tok0 + j < P.n_fp) ? d[j] * P.c : -INFINITY;
      }
      online_softmax<NNT>(st, s, p);

      float pv[8];
      const int src0 = (lane & 0x33), src1 = (lane & 0x33) | 4;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        pv[j] = __shfl(p[j], src0);
        pv[4 + j] = __shfl(p[j], src1);
      }
      // rows 0..3: p rounded to T; rows 4..7: the rounding residual, again in T
      float av[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float hi = t2f<BF16>(f2t<BF16>(pv[i]));
        av[i] = up == 0 ? hi : up == 1 ? pv[i] - hi : 0.f;
      }
      uint4 a;
      a.x = pack_T<BF16>(av[0], av[1]); a.y = pack_T<BF16>(av[2], av[3]);
      a.z = pack_T<BF16>(av[4], av[5]); a.w = pack_T<BF16>(av[6], av[7]);
      if (32 * unit + 32 > P.n_fp) {   // slots beyond n_fp hold unspecified bits
        uint32_t keep[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i0 = 2 * r, i1 = 2 * r + 1;
          const int x0 = 16 * ((i0 >> 2) & 1) + 4 * q4 + (i0 & 3), x1 = 16 * ((i1 >> 2) & 1) + 4 * q4 + (i1 & 3);
          keep[r] = (32 * unit + x0 < P.n_fp ? 0x0000FFFFu : 0u) | (32 * unit + x1 < P.n_fp ? 0xFFFF0000u : 0u);
        }
#pragma unroll
        for (int nt = 0; nt < NNT; ++nt) {
          va[nt].x &= keep[0]; va[nt].y &= keep[1]; va[nt].z &= keep[2]; va[nt].w &= keep[3];
        }
      }
#pragma unroll
      for (int nt = 0; nt < NNT; ++nt) st.acc[nt] = mfma_T<BF16>(a, va[nt], st.acc[nt]);
    }
    const float l_tot = head_sum(st.l);
    if (lane < 4) { ml_lds[wave][g][0] = st.m; ml_lds[wave][g][1] = l_tot; }
#pragma unroll
    for (int nt = 0; nt < NNT; ++nt) {
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) {
        const float v = st.acc[nt][gg] + __shfl_xor(st.acc[nt][gg], 16);
        if (q4 == 0) o_lds[wave][gg][16 * nt + n16] = v;
      }
    }
  }
  __syncthreads();
  // merge the four wavefronts; write this split's partial: per head D floats, then m, l
  for (int idx = threadIdx.x; idx < P.hb * D; idx += 256) {
    const int gg = idx / D, c = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, ml_lds[w][gg][0]);
    float acc = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = ml_lds[w][gg][0];
      const float a = mw == -INFINITY ? 0.f : exp2f(mw - M);
      acc += a * o_lds[w][gg][c];
      L += a * ml_lds[w][gg][1];
    }
    const int64_t base = (((int64_t)bh * P.splits + split) * P.gh + hsub * P.hb + gg) * (D + 2);
    P.ws[base + c] = acc;
    if (c == 0) { P.ws[base + D] = M; P.ws[base + D + 1] = L; }
  }
}

hipError_t launch_combine(const Shape& s, const float* ws, void* out, int splits, hipStream_t st);

template <bool BF16, int D>
static hipError_t launch_mfma_dg(const Shape& s, const AttnParams& P, dim3 grid, hipStream_t st) {
  switch (s.G) {
    case 32: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 32>), grid, dim3(256), 0, st, P); break;
    case 64: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 64>), grid, dim3(256), 0, st, P); break;
    default: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 128>), grid, dim3(256), 0, st, P); break;
  }
  return launch_status(__func__);
}

template <bool BF16>
static hipError_t launch_mfma_d(const Shape& s, const AttnParams& P, dim3 grid, hipStream_t st) {
  switch (s.d) {
    case 64: return launch_mfma_dg<BF16, 64>(s, P, grid, st);
    case 96: return launch_mfma_dg<BF16, 96>(s, P, grid, st);
    default: return launch_mfma_dg<BF16, 128>(s, P, grid, st);
  }
}

hipError_t launch_decode_attn_mfma(const Shape& s, const lq_cache& c, const void* q, float scale,
                                   void* out, void* ws, const lq_plan& plan, hipStream_t st) {
  AttnParams P;
  P.q = (const uint16_t*)q;
  P.k_fp = (const uint16_t*)c.k_fp[c.cur];
  P.v_fp = (const uint16_t*)c.v_fp[c.cur];
  P.k_codes = c.k_codes; P.v_codes = c.v_codes;
  P.k_scale = (const uint16_t*)c.k_scale; P.k_zero = (const uint16_t*)c.k_zero;
  P.v_scale = (const uint16_t*)c.v_scale; P.v_zero = (const uint16_t*)c.v_zero;
  P.ws = (float*)ws;
  P.cap = s.cap; P.qcap = s.qcap; P.n_fp = c.n_fp; P.n_q = c.n_q; P.gh = s.gh;
  P.hb = s.gh % 4 == 0 ? 4 : (s.gh % 2 == 0 ? 2 : 1);
  P.splits = plan.splits; P.nwf = plan.fp_waves;
  P.c = scale * 1.4426950408889634f;
  dim3 grid(plan.splits, s.B * s.Hkv * (s.gh / P.hb));
  hipError_t e = s.bf16 ? launch_mfma_d<true>(s, P, grid, st) : launch_mfma_d<false>(s, P, grid, st);
  if (e != hipSuccess) return e;
  return launch_combine(s, (const float*)ws, out, plan.splits, st);
}

}  // namespace lq
