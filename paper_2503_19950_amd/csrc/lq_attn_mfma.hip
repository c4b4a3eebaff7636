// Fused decode attention for gfx950 (Eq. 2 with Eq. 6's 1/sqrt(d), one softmax over
// the original-precision rows and the quantized rows, Sec. 2.4).  The quantized rows
// (2-bit codes, or 4-bit: Sec. 3.2.1) are never dequantized in memory:
//
//   logits   q.k_hat_t = sum_c q_c z_c + sum_c (q_c s_c) code_tc
//            -> per key group (G tokens) the products q_c s_c are formed once, split
//               into three fp16 pieces (the top six bits of the rounded product, its
//               other five bits, the rounding residual: together exact for 11-bit or
//               8-bit factors) and become three rows of the A operand of a 16x16x32
//               matrix instruction: row 4*head + piece (piece 3 is zero).
//               The code tile is the B operand, 16 tokens per instruction.  Lane
//               (row group q4, column n16) of the result then holds, for head q4 and
//               token n16, the pieces in three registers: two adds give the logit.
//               sum_c q_c z_c is a per-group bias.  (A single fp16 rounding of
//               q_c s_c is not enough: with outlier channels its error alone moves
//               the logits by ~1e-2.)
//   output   sum_t p_t v_hat_tc = sum_t p_t vz_t + sum_t (p_t vs_t) code_tc
//            -> p_t vs_t (row 4*channel group + head) is the A operand, the code
//               tile the B operand; sum_t p_t vz_t is kept per channel group.  The
//               probabilities go from the softmax lanes (head x token) to the lanes
//               of the output step (token octets) through LDS as fp16.
//
// Codes as operands.  An fp16 lane whose only set bits are mantissa bits 2v, 2v+1 is
// the subnormal number code * 2^(2v-24); gfx950's matrix cores take subnormal
// operands exactly.  The packed layout puts the eight 2-bit codes a lane feeds to
// one matrix instruction into one byte of the low and one byte of the high half of
// a 32-bit word, so four ANDs (plus one shift by 8 for the odd operand of a word)
// produce the four operand registers: 9 VALU instructions per 16 codes, no
// integer-to-float conversion.  The factor 2^(2v) that depends on the position v
// of a code inside its byte is cancelled in the other operand: q is pre-multiplied
// by 2^(3-2v) per channel, and the probabilities by the same factor per token slot
// (folded into the exponent of exp2, so it costs nothing).  4-bit codes work the
// same way with two nibble positions (see codes4).
//
// Work split: a workgroup has eight (or four) independent wavefronts; the
// wavefronts of all workgroups of one (batch row, kv head) are numbered 0..NW-1,
// the first `nwf` walk the fp rows in units of 32, the others walk the quantized
// rows in tiles of 64 (schedule: see "Tile schedule" below).
// Partial (max, sum, output) triples are merged in LDS per workgroup and written
// to the workspace.  Every workgroup then takes a ticket from a counter of its
// (batch row, kv head, head group); the one that draws the last ticket merges all
// splits of that group and writes the output, so no second launch is needed and
// the merge of one group overlaps the tail of the others.  Nobody waits on anybody.
// The partials and the counter are accessed with device-scope relaxed atomics
// (write-through stores, cache-bypassing loads): a device-scope fence would write
// back and invalidate a whole L2 per workgroup, which costs more than the kernel.
#include <stdlib.h>

#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

struct AttnParams {
  const uint16_t* q;
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const uint16_t* k_scale;
  const uint16_t* k_zero;
  const uint16_t* v_scale;
  const uint16_t* v_zero;
  float* ws;          // partials
  int* counters;      // CTR_LINES lines per group (ticket, tile pools), zero between launches
  uint16_t* out;
  // fused append (null k_new: none): the new row of every (b, kv head), [B][Hkv][d],
  // becomes fp slot n_fp - 1 (n_fp already counts it)
  const uint16_t* k_new;
  const uint16_t* v_new;
  uint16_t* k_fp[2];      // [0]: the live fp buffer (the same for every sequence), or, with
  uint16_t* v_fp[2];      // per-sequence state, the two buffers, chosen by the sequence's `cur`
  int32_t* pos_fp[2];
  const SeqState* seq;    // device array of per-sequence state (seq_mode 2)
  int seq_mode;           // 0: counts below hold for every sequence; 1: state in the kernel arguments
  int Hkv;
  int cap, qcap, n_fp, n_q, gh, hb, splits, nwf;
  int W, Wq;          // of every Wq quantized slots (one filtering event) the first W hold tokens
  int n_tok_q;        // tokens in the n_q quantized slots
  int dynamic;        // 0: static tile schedule only
  float c;  // softmax scale * log2(e)
};

constexpr int PSHIFT = 5;   // probabilities are kept relative to 2^(max - PSHIFT)
constexpr float MAX_SLACK = 4.f;
constexpr float DEAD_LOGIT = -1e30f;   // logit of a padding slot; exp2(DEAD_LOGIT - anything finite) == 0

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

// The eight codes of one operand live in byte 0 and byte 2 of `w` (even operand of
// the word) or in byte 1 and byte 3 (odd operand).  Register v keeps the code at
// bits 2v, 2v+1 of each fp16 lane: value code * 2^(2v-24).
__device__ __forceinline__ uint4 codes_even(uint32_t w) {
  return make_uint4(w & 0x00030003u, w & 0x000C000Cu, w & 0x00300030u, w & 0x00C000C0u);
}
__device__ __forceinline__ uint4 codes_odd(uint32_t w) { return codes_even(w >> 8); }
__device__ __forceinline__ uint4 codes_of(uint32_t w, int odd) {
  return odd ? codes_odd(w) : codes_even(w);
}
// 4-bit codes: a word holds the eight codes of one operand, element i = 2v + h in
// nibble v of half h.  Registers 0 and 2 keep their codes at mantissa bits 0..3
// (code * 2^-24), registers 1 and 3 at bits 4..7 (code * 2^-20); two of the four
// nibbles of a half would reach into the exponent and are shifted down first.
__device__ __forceinline__ uint4 codes4(uint32_t w) {
  const uint32_t h = w >> 8;
  return make_uint4(w & 0x000F000Fu, w & 0x00F000F0u, h & 0x000F000Fu, h & 0x00F000F0u);
}
// Operand o (of the 2 * NKC a lane holds for one 32-slot block) of a code tile, and
// the power of two by which the other operand's register v has to be scaled so that
// every product carries the common factor 2^-CODE_SHIFT.
template <int BITS, int N>
__device__ __forceinline__ uint4 operand_codes(const uint32_t (&w)[N], int o) {
  if constexpr (BITS == 2) return codes_of(w[o >> 1], o & 1);
  else return codes4(w[o]);
}
template <int BITS>
__device__ __forceinline__ constexpr int pos_exp(int v) {   // log2 of the scale of register v's partner
  return BITS == 2 ? 3 - 2 * v : 2 - 4 * (v & 1);
}
template <int BITS>
constexpr float CODE_SCALE = BITS == 2 ? 2097152.f : 4194304.f;   // 2^21, 2^22

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
// a pair of T values -> a pair of fp16 values (exact for normal-range bf16 inputs)
template <bool BF16>
__device__ __forceinline__ half2_t pair_to_f16(uint32_t w) {
  if constexpr (BF16) return half2_t{(_Float16)lo_T<true>(w), (_Float16)hi_T<true>(w)};
  else return __builtin_bit_cast(half2_t, w);
}
// Scales and zero-points are stored as fp16 whatever the cache type (for a bf16 cache
// converting them here cost a sixth of the tile loop's instructions): a stored pair is
// an operand as it is.
__device__ __forceinline__ half2_t meta_pair(uint32_t w) { return __builtin_bit_cast(half2_t, w); }
// fp32 accumulate of a two-element dot product of fp16 pairs (exact products)
__device__ __forceinline__ float dot2_h(half2_t a, half2_t b, float c) {
  return __builtin_amdgcn_fdot2(a, b, c, false);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
// lane i <-> lane i^16 and lane i <-> lane i^32 exchanges without the LDS crossbar:
// the swap instructions trade rows (halves) between two registers, so swapping a
// register with a copy of itself leaves one holding the even rows (low half) twice
// and the other the odd rows (high half) twice.
__device__ __forceinline__ void xor16_pair(float v, float* a, float* b) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  *a = __uint_as_float(r[0]); *b = __uint_as_float(r[1]);
}
__device__ __forceinline__ void xor32_pair(float v, float* a, float* b) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  *a = __uint_as_float(r[0]); *b = __uint_as_float(r[1]);
}
// all-reduce over the 16 lanes that share lane & 3 (one query head): two rotations
// inside the row of 16 lanes, two exchanges across rows
__device__ __forceinline__ float head_max(float v) {
  float a, b;
  v = fmaxf(v, dpp_f<0x124>(v));   // row_ror:4
  v = fmaxf(v, dpp_f<0x128>(v));   // row_ror:8
  xor16_pair(v, &a, &b); v = fmaxf(a, b);
  xor32_pair(v, &a, &b); v = fmaxf(a, b);
  return v;
}
__device__ __forceinline__ float head_sum(float v) {
  float a, b;
  v += dpp_f<0x124>(v);
  v += dpp_f<0x128>(v);
  xor16_pair(v, &a, &b); v = a + b;
  xor32_pair(v, &a, &b); v = a + b;
  return v;
}
// all-reduce over the 16 lanes of a lane row (lanes that share lane >> 4)
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_f<0x128>(v);   // row_ror:8
  v += dpp_f<0x124>(v);
  v += dpp_f<0x122>(v);
  v += dpp_f<0x121>(v);
  return v;
}
__device__ __forceinline__ float row_max(float v) {
  v = fmaxf(v, dpp_f<0x128>(v));
  v = fmaxf(v, dpp_f<0x124>(v));
  v = fmaxf(v, dpp_f<0x122>(v));
  v = fmaxf(v, dpp_f<0x121>(v));
  return v;
}
// sum over the four lanes that differ in lane >> 4
__device__ __forceinline__ float rows_sum(float v) {
  float a, b;
  xor16_pair(v, &a, &b); v = a + b;
  xor32_pair(v, &a, &b); v = a + b;
  return v;
}

// LDS-visible ordering inside one wavefront (no workgroup barrier needed: DS
// instructions of a wavefront execute in order).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// device-coherent accesses to the partial results (see the ticket merge below)
__device__ __forceinline__ void st_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int N>
struct Words { uint32_t w[N]; };

// Running softmax state of one wavefront.  m and l belong to head (lane & 3);
// acc[nt][j] is output row 4*(lane>>4)+j, column lane&15 of channel tile nt.
// Everything is relative to 2^(m - PSHIFT); l[j] additionally carries the factor
// 2^offs[j] of its token slot.
template <int NNT>
struct State {
  floatx4 acc[NNT];
  float m;
  float l[4];
  float zacc[4];   // per code position v (token slots 2v, 2v+1 of a lane)
};

// s[0..3]: log2-domain logits (slot offsets included) of this lane's four tokens
// -> p[0..3] = 2^(s - m + PSHIFT); updates the state.
template <int NNT, bool ZACC>
__device__ __forceinline__ void online_softmax(State<NNT>& st, const float* s, float* p) {
  // the running maximum only has to bound every logit seen so far: the cross-lane
  // reduction runs only when some lane's tile maximum exceeds it
  // (a logit may exceed the reference by up to MAX_SLACK before that happens:
  // probabilities then reach 2^(PSHIFT + MAX_SLACK), still far inside fp16 range)
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  if (__any(mx > st.m + MAX_SLACK)) {
    mx = head_max(mx);
    const float m_new = fmaxf(st.m, mx);
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // 0 on the first tile (m = -inf)
#pragma unroll
    for (int j = 0; j < 4; ++j) st.l[j] *= alpha;
    if constexpr (ZACC) {
#pragma unroll
      for (int i = 0; i < 4; ++i) st.zacc[i] *= alpha;
    }
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
  const float mref = st.m - (float)PSHIFT;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    p[j] = __builtin_amdgcn_exp2f(s[j] - mref);
    st.l[j] += p[j];
  }
}

// Quantized-row variant: lane row q4 = lane >> 4 is a query head, the 16 lanes of a
// row hold different tokens; s[u], u = 0..3, are this lane's tokens.  The output
// accumulators and zacc are laid out by the output step: acc[nt][j] belongs to head
// j, zacc to head g = lane & 3.
// ROUND_P: the probabilities come back already rounded to fp16, the form in which the
// output step uses them, and the denominator sums these rounded values.  Numerator and
// denominator then describe the same (slightly perturbed) weights, so that the rounding
// cancels where one token dominates instead of scaling the whole output.
template <int NNT, bool ROUND_P>
__device__ __forceinline__ void online_softmax_rows(State<NNT>& st, const float* s, float* p, int g) {
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  if (__any(mx > st.m + MAX_SLACK)) {
    mx = row_max(mx);
    const float m_new = fmaxf(st.m, mx);
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // 0 on the first tile (m = -inf)
#pragma unroll
    for (int u = 0; u < 4; ++u) st.l[u] *= alpha;
    float a4[4];
#pragma unroll
    for (int gg = 0; gg < 4; ++gg)
      a4[gg] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(alpha), 16 * gg));
    const float ag = g == 0 ? a4[0] : g == 1 ? a4[1] : g == 2 ? a4[2] : a4[3];
#pragma unroll
    for (int i = 0; i < 4; ++i) st.zacc[i] *= ag;
#pragma unroll
    for (int nt = 0; nt < NNT; ++nt) {
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) st.acc[nt][gg] *= a4[gg];
    }
    st.m = m_new;
  }
  const float mref = st.m - (float)PSHIFT;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    p[u] = __builtin_amdgcn_exp2f(s[u] - mref);
    if constexpr (ROUND_P) p[u] = (float)(_Float16)p[u];
    st.l[u] += p[u];
  }
}

// NWB: wavefronts per workgroup: 8; 4 when there are enough (b, kv head) groups to put
// two workgroups on every compute unit; 12 (three wavefronts per SIMD, at most 168
// registers) for long contexts, where the extra wavefront hides more than the tighter
// register budget costs.
// GENERAL: the variant that also handles padding slots in the quantized region (group
// size not dividing the window) and per-sequence counts; built for 8 and 12 wavefronts
// per workgroup.  The other instantiations carry neither check.
// per-sequence state in the kernel arguments: only the general instantiation has any
template <bool GENERAL> struct SeqArgs {};
template <> struct SeqArgs<true> { SeqState e[SEQ_CHUNK]; };

template <bool BF16, int D, int G, int NWB, int BITS, bool GENERAL = false>
__global__ void __launch_bounds__(64 * NWB, NWB == 12 ? 3 : 2)
attn_mfma_kernel(const AttnParams P, const SeqArgs<GENERAL> S) {
  constexpr int NKC = D / 32, NNT = D / 16, NGC = (D + G - 1) / G;
  constexpr int WPL = NKC * (BITS / 2);           // code words per lane and 32-slot block
  constexpr int NGRP = G < 64 ? 64 / G : 1;     // key groups per 64-token tile
  // fp16 pieces of q*s per wave, one row per (piece, head).  The 16 lanes of a
  // lane row read 16 bytes each from thirteen different rows at the same column; a row
  // pitch that is an odd number of 16-byte units puts those on different banks.
  constexpr int QS_ROW = D + 8;
  static_assert((QS_ROW * 2 / 16) % 2 == 1, "q*s row pitch");
  constexpr int QS_ROWS = 13;
  __shared__ __attribute__((aligned(16))) uint16_t qs_lds[NWB][NGRP][QS_ROWS][QS_ROW];   // rows 4*piece+head (three pieces), row 12 = zeros
  __shared__ __attribute__((aligned(16))) uint16_t p_lds[NWB][2][9][32];            // [wave][32-token step][row][token]: rows 0-3 p of head, 4 zeros, 5-8 p's fp16 rounding residual
  __shared__ float o_lds[NWB][4][D];
  __shared__ float ml_lds[NWB][4][2];
  __shared__ float zs_lds[NWB][4][4];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nhg = P.gh / P.hb;
  // Workgroups are handed to the eight XCDs in turn (linear index mod 8).  When the
  // number of groups allows it, all splits of one group are placed on one XCD, so
  // that the partials they exchange at the end meet in that XCD's L2.
  int split = blockIdx.x, group = blockIdx.y;
  if (gridDim.y % 8 == 0) {
    const int L = blockIdx.y * gridDim.x + blockIdx.x;
    const int r = L >> 3;
    group = (L & 7) + 8 * (r / (int)gridDim.x);
    split = r % (int)gridDim.x;
  }
  const int hsub = group % nhg;
  int bh = group / nhg;
  if constexpr (GENERAL) {
    // per-sequence lengths: workgroups are dispatched in index order, so the rows are
    // taken longest first (seq[i].order = the row with the i-th most tokens)
    if (P.seq_mode) {
      const int i = bh / P.Hkv;
      bh = (P.seq_mode == 1 ? seq_in_args(args_offset_after(sizeof(AttnParams)))[i].order : P.seq[i].order) * P.Hkv +
           bh % P.Hkv;   // (the argument block is P, then S)
    }
  }
  const int q4 = lane >> 4, n16 = lane & 15, up = n16 >> 2, g = lane & 3;
  const bool head_ok = g < P.hb;
  const int64_t qrow = ((int64_t)bh * P.gh + hsub * P.hb + (head_ok ? g : 0)) * D;

  // counts and live fp buffer: the same for every sequence, or (per-sequence lengths)
  // read from the sequence's entry of the state array
  int n_fp = P.n_fp, n_q = P.n_q, nwf = P.nwf, n_tok_q = P.n_tok_q, cur = 0;
  if constexpr (GENERAL) {
    if (P.seq_mode) {
      const SeqState sq = P.seq_mode == 1 ? seq_load(seq_in_args(args_offset_after(sizeof(AttnParams))), bh / P.Hkv)
                                          : P.seq[bh / P.Hkv];
      n_fp = sq.n_fp; n_q = sq.n_q; nwf = sq.nwf; n_tok_q = sq.n_tok_q; cur = sq.cur;
    }
  }
  // (a select between two kernel arguments, not a load that depends on `cur`)
  uint16_t* k_fp_w = cur ? P.k_fp[1] : P.k_fp[0];
  uint16_t* v_fp_w = cur ? P.v_fp[1] : P.v_fp[0];
  int32_t* pos_fp = cur ? P.pos_fp[1] : P.pos_fp[0];
  const uint16_t* k_fp = k_fp_w;
  const uint16_t* v_fp = v_fp_w;
  const int NW = P.splits * NWB, NWF = nwf, NWQ = NW - NWF;
  const int gw = split * NWB + wave;
  const int TQ = (n_q + 63) >> 6, TF = (n_fp + 31) >> 5;
  const int64_t part_base = (((int64_t)bh * P.splits + split) * P.gh + hsub * P.hb) * (D + 4);
  State<NNT> st;
#pragma unroll
  for (int nt = 0; nt < NNT; ++nt) st.acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j) st.l[j] = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) st.zacc[i] = 0.f;

  if (gw >= NWF) {
    // ------------------------- quantized rows -------------------------
    const int wq = gw - NWF;
    const char* kcb = (const char*)(P.k_codes + (int64_t)bh * (P.qcap >> 5) * 64 * WPL);
    const char* vcb = (const char*)(P.v_codes + (int64_t)bh * (P.qcap >> 5) * 64 * WPL);
    const char* ksb = (const char*)(P.k_scale + (int64_t)bh * (P.qcap / G) * D);
    const char* kzb = (const char*)(P.k_zero + (int64_t)bh * (P.qcap / G) * D);
    const char* vsb = (const char*)(P.v_scale + (int64_t)bh * (P.qcap >> 5) * NGC * 32);
    const char* vzb = (const char*)(P.v_zero + (int64_t)bh * (P.qcap >> 5) * NGC * 32);
    // Rows of the probability operand of the output step: row 4*up + g.  With at most
    // two channel groups there are rows to spare, and the probabilities enter in two
    // pieces: a head piece (p rounded to fp16; for bf16 caches cut to three significant
    // bits, see where it is written) and what that leaves out (rows up = piece * NGC +
    // channel group), so that only the rounding of the product p * vs remains.
    // With three or four groups there is one piece (up = channel group); the softmax
    // denominator then sums the rounded probabilities, so that the rounding does not
    // bias the normalised weights.
    constexpr int VPIECES = NGC <= 2 ? 2 : 1;
    // The operand p * vs is rounded to fp16.  Where the cache type is fp16 (whose output
    // tolerance that rounding alone can use up when one token carries most of the weight
    // and its code is large) the part the rounding drops is carried as well: in the
    // residual rows when there are two pieces, in a second product otherwise.
    constexpr bool PROD_LO = !BF16;
    const bool row_live = up < VPIECES * NGC;
    const int upc = row_live ? up % NGC : 0;          // channel group of this lane's row
    const bool tail_row = VPIECES == 2 && up >= NGC;  // this lane feeds the residual piece
    const uint32_t code_off = lane * WPL * 4;                 // byte offsets of this lane
    const uint32_t vm_off = (upc * 32 + 8 * q4) * 2;
    // Lane roles.  Logits and softmax: lane row q4 is query head q4, lane column n16
    // is a token of each of the four 16-token tiles.  q*s preparation: head q4,
    // channel octet n16.  Output step: row n16 = (channel group up, head g) of the
    // probability operand, token octet q4.
    const int c8 = n16;
    const bool prep = 8 * c8 < D;
    const uint32_t km_off = (prep ? 8 * c8 : 0) * 2;
    const bool headq_ok = q4 < P.hb;

    struct Tile {
      Words<WPL> kc[2], vc[2];
      uint4 vs[2], vz[2];
      uint4 ks8[NGRP], kz8[NGRP];
    };
    // A tile's registers are refilled piecewise with the next tile's data as soon as
    // their content has been consumed (key scales right after the q*s preparation,
    // key codes after the logits, value codes and scales after each output step), so
    // only one tile's worth of registers is live and every piece still has most of a
    // tile's processing time to arrive.
    // The tile loads are buffer loads: one descriptor per array over this slice, the
    // lane's offset in a register, the tile's offset in a scalar register, so that the
    // per-tile address arithmetic runs on the scalar unit (and a load past the slice
    // would return zeros instead of faulting).
    const uint32_t code_bytes = (uint32_t)(P.qcap >> 5) * 64 * WPL * 4;
    const auto rs_kc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kcb), 0, code_bytes, 0x00020000);
    const auto rs_vc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vcb), 0, code_bytes, 0x00020000);
    const uint32_t kmeta_bytes = (uint32_t)(P.qcap / G) * D * 2, vmeta_bytes = (uint32_t)(P.qcap >> 5) * NGC * 32 * 2;
    const auto rs_ks = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(ksb), 0, kmeta_bytes, 0x00020000);
    const auto rs_kz = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kzb), 0, kmeta_bytes, 0x00020000);
    const auto rs_vs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vsb), 0, vmeta_bytes, 0x00020000);
    const auto rs_vz = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vzb), 0, vmeta_bytes, 0x00020000);
    auto load16 = [&](__amdgpu_buffer_rsrc_t rs, uint32_t voff, uint32_t soff) {
      const auto v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, (int)soff, 0);
      return make_uint4(v[0], v[1], v[2], v[3]);
    };
    auto load_words = [&](__amdgpu_buffer_rsrc_t rs, uint32_t voff, uint32_t soff) {
      Words<WPL> r;
#pragma unroll
      for (int i = 0; i + 4 <= WPL; i += 4) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff + 4 * i, (int)soff, 0);
        r.w[i] = v[0]; r.w[i + 1] = v[1]; r.w[i + 2] = v[2]; r.w[i + 3] = v[3];
      }
      if constexpr (WPL % 4 == 3) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b96(rs, (int)voff + 4 * (WPL - 3), (int)soff, 0);
        r.w[WPL - 3] = v[0]; r.w[WPL - 2] = v[1]; r.w[WPL - 1] = v[2];
      } else if constexpr (WPL % 4 == 2) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)voff + 4 * (WPL - 2), (int)soff, 0);
        r.w[WPL - 2] = v[0]; r.w[WPL - 1] = v[1];
      }
      return r;
    };
    auto load_kmeta = [&](Tile& T, int t) {
#pragma unroll
      for (int e = 0; e < NGRP; ++e) {
        const int grp = G <= 64 ? t * NGRP + e : t / (G / 64);
        T.ks8[e] = load16(rs_ks, km_off, (uint32_t)grp * (D * 2));
        T.kz8[e] = load16(rs_kz, km_off, (uint32_t)grp * (D * 2));
      }
    };
    auto load_kcodes = [&](Tile& T, int t) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
        T.kc[b2] = load_words(rs_kc, code_off, (uint32_t)t * (2 * 64 * WPL * 4) + b2 * (64 * WPL * 4));
    };
    auto load_v = [&](Tile& T, int t, int b2) {
      T.vc[b2] = load_words(rs_vc, code_off, (uint32_t)t * (2 * 64 * WPL * 4) + b2 * (64 * WPL * 4));
      T.vs[b2] = load16(rs_vs, vm_off, (uint32_t)t * (2 * NGC * 32 * 2) + b2 * (NGC * 32 * 2));
      T.vz[b2] = load16(rs_vz, vm_off, (uint32_t)t * (2 * NGC * 32 * 2) + b2 * (NGC * 32 * 2));
    };

    // Tile schedule.  The first two tiles of a wavefront are fixed (wq, wq + NWQ) and
    // the loads of the first go out before anything else touches memory.  The later
    // tiles are dealt out dynamically, so that wavefronts that start late or see
    // slower memory take fewer of them: tile 2 * NWQ + v * NSUB + j belongs to
    // pool j (NSUB pools), and the wavefronts with wq % NSUB == j, spread over the
    // whole chip, draw v from that pool's counter.  Several pools because atomics on
    // one address are serialised at a rate that a single counter could not sustain.
    // A draw is issued a whole tile ahead of its use and before that tile's loads: loads
    // and atomics return in issue order, so waiting for the drawn index does not wait
    // for the loads behind it.  The draw is a buffer atomic over a 4-byte buffer: only
    // lane 0 is in range, the other lanes are dropped by the bounds check, and no
    // branch is needed (the join of a branch would make the compiler wait for every
    // outstanding load).
    // With few tiles per wavefront, or no more wavefronts than pools, there is nothing
    // to balance: the schedule is then static (tile wq + v * NWQ) and the atomic is
    // aimed out of range.
    // A single split has no last workgroup that could re-arm the pool counters for the
    // next launch (it returns before the ticket): static as well.
    const bool dyn = P.dynamic && P.splits > 1 && NWQ > NSUB && TQ >= 5 * NWQ;
    const int nsub = dyn ? NSUB : NWQ;
    const int sub = wq % nsub;
    int v_static = 0;
    const __amdgpu_buffer_rsrc_t pool = __builtin_amdgcn_make_buffer_rsrc(
        P.counters + (group * CTR_LINES + 1 + sub) * CTR_LINE, 0, 4, 0x00020000);
    auto draw = [&]() {   // raw counter value in lane 0
      return __builtin_amdgcn_raw_ptr_buffer_atomic_add_i32(1, pool, dyn ? lane * 4 : 4, 0, 0);
    };
    auto drawn_tile = [&](int k) {
      const int v = dyn ? __builtin_amdgcn_readfirstlane(k) : v_static++;
      return 2 * NWQ + v * nsub + sub;
    };
    int ta = wq, tb = wq + NWQ;
    Tile A;
    if (ta < TQ) {
      load_kmeta(A, ta);
      load_kcodes(A, ta);
      load_v(A, ta, 0);
      load_v(A, ta, 1);
    }

    // q of (head q4, channels 8*c8..+7): fp16 pairs for the bias dot products, and
    // fp16 pairs pre-multiplied by 2^(3-2v) (v = pair index) for the q*s operands
    uint32_t qraw[4];
    half2_t qz[4], qh[4];
    {
      const int64_t qrow_q = ((int64_t)bh * P.gh + hsub * P.hb + (headq_ok ? q4 : 0)) * D;
      uint4 raw = *reinterpret_cast<const uint4*>(P.q + qrow_q + (prep ? 8 * c8 : 0));
      if (!prep || !headq_ok) raw = make_uint4(0, 0, 0, 0);
      qraw[0] = raw.x; qraw[1] = raw.y; qraw[2] = raw.z; qraw[3] = raw.w;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float f = __builtin_ldexpf(1.f, pos_exp<BITS>(v));
        qh[v] = half2_t{(_Float16)(lo_T<BF16>(qraw[v]) * f), (_Float16)(hi_T<BF16>(qraw[v]) * f)};
        qz[v] = pair_to_f16<BF16>(qraw[v]);
      }
    }
    const float c21 = P.c * CODE_SCALE<BITS>;   // codes and the pre-scaled q*s together carry 1 / CODE_SCALE
    // slot offsets: this lane's token of tile u is token x = 16*(u&1) + n16 of its
    // 32-token output step, element i = 4*(x/16) + x%4 of its lane group there, whose
    // codes sit at position v = i >> 1
    float offs[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int v = 2 * (u & 1) + ((n16 & 3) >> 1);
      offs[u] = (float)(BITS == 2 ? 3 - 2 * v : 2 - 4 * (v & 1));
    }

    // rows of the q*s operand: matrix row n16 = 4*head + piece, piece 3 is zero
    const uint16_t* qs_rd = &qs_lds[wave][0][(n16 & 3) < 3 ? 4 * (n16 & 3) + (n16 >> 2) : 12][8 * q4];
    uint16_t* qs_wr = &qs_lds[wave][0][q4][8 * c8];
    // probabilities: written per (head q4, token), read per (head g, token octet q4);
    // lanes of absent channel groups read the zero row
    const uint16_t* p_rd = &p_lds[wave][0][!row_live ? 4 : tail_row ? 5 + g : g][4 * q4];
    const uint16_t* p_hd = &p_lds[wave][0][!row_live ? 4 : g][4 * q4];
    uint16_t* p_wr = &p_lds[wave][0][q4][n16];
    {
      for (int e = 0; e < NGRP; ++e)
        for (int c = lane; c < QS_ROW; c += 64) qs_lds[wave][e][12][c] = 0;
      if (lane < 32) { p_lds[wave][0][4][lane] = 0; p_lds[wave][1][4][lane] = 0; }
    }

    auto process = [&](Tile& cur, int t, int tn) {   // tn: the tile to refill the registers with
      // ---- q*s (fp16 head and tail) and bias = sum_c q_c z_c for each key group
      float bo[4];
      {
        float bias[NGRP];
#pragma unroll
        for (int e = 0; e < NGRP; ++e) {
          const uint32_t sw[4] = {cur.ks8[e].x, cur.ks8[e].y, cur.ks8[e].z, cur.ks8[e].w};
          const uint32_t zw[4] = {cur.kz8[e].x, cur.kz8[e].y, cur.kz8[e].z, cur.kz8[e].w};
          float bp = 0.f;
          // q*s in three pieces whose sum is the exact product: the top six significant
          // bits of the rounded product, its other five bits, and what the rounding dropped.
          // The code operands are fp16 subnormals; the matrix unit aligns the addends of a
          // dot product by the exponent fields of their operands and keeps about 24 bits
          // below the largest, while a code's bits lie up to 9 bits below its nominal
          // exponent: measured, an 11-bit operand loses its low bits as soon as another
          // channel of the block has a q*s a few times larger.  A six-bit piece has 5 bits
          // of room more, and the two small pieces lose nothing that matters (they may be
          // subnormal themselves: single products of two subnormals were measured exact).
          uint32_t h[4], r[4], l[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
#pragma clang fp contract(off)   // hi - top must subtract from the ROUNDED product: fused into fma(q, s, -top) it would hold lo as well
            bp = dot2_h(qz[v], meta_pair(zw[v]), bp);
            const half2_t sh = meta_pair(sw[v]);
            const half2_t hi = qh[v] * sh;
            const half2_t lo = __builtin_elementwise_fma(qh[v], sh, -hi);
            h[v] = __builtin_bit_cast(uint32_t, hi) & 0xFFE0FFE0u;
            r[v] = __builtin_bit_cast(uint32_t, hi - __builtin_bit_cast(half2_t, h[v]));
            l[v] = __builtin_bit_cast(uint32_t, lo);
          }
          if (prep) {
            *reinterpret_cast<uint4*>(qs_wr + e * (QS_ROWS * QS_ROW)) = make_uint4(h[0], h[1], h[2], h[3]);
            *reinterpret_cast<uint4*>(qs_wr + e * (QS_ROWS * QS_ROW) + 4 * QS_ROW) = make_uint4(r[0], r[1], r[2], r[3]);
            *reinterpret_cast<uint4*>(qs_wr + e * (QS_ROWS * QS_ROW) + 8 * QS_ROW) = make_uint4(l[0], l[1], l[2], l[3]);
          }
          bias[e] = row_sum(bp) * P.c;
        }
        load_kmeta(cur, tn);
#pragma unroll
        for (int u = 0; u < 4; ++u) bo[u] = bias[(u * NGRP) >> 2] + offs[u];
      }
      wave_lds_sync();

      // ---- logits: rows (head, piece) x four 16-token tiles, NKC channel chunks each
      floatx4 Du[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) Du[u] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int e = 0; e < NGRP; ++e) {
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc) {
          const uint4 qa = *reinterpret_cast<const uint4*>(qs_rd + e * (QS_ROWS * QS_ROW) + 32 * kc);
#pragma unroll
          for (int u = e * (4 / NGRP); u < (e + 1) * (4 / NGRP); ++u) {
            const int o = (u & 1) * NKC + kc;
            const uint4 b = operand_codes<BITS>(cur.kc[u >> 1].w, o);
            Du[u] = mfma_f16(qa, b, Du[u]);
          }
        }
      }

      load_kcodes(cur, tn);

      // this lane: head q4, token 16*u + n16 of the tile; the three pieces are rows j = 0, 1, 2
      float s[4], p[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) s[u] = fmaf(Du[u][0] + (Du[u][1] + Du[u][2]), c21, bo[u]);
      const bool partial = 64 * t + 64 > n_q;
      if (partial) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (64 * t + 16 * u + n16 >= n_q) s[u] = -INFINITY;
      }
      if (GENERAL && P.Wq != P.W) {
        // padding slots behind a short key group (zero codes, zero value scales and
        // zero-points): a finite sentinel, so that a tile made of padding only leaves
        // a state whose weight in every later merge is exactly 0
        const int r0 = (64 * t) % P.Wq;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          int r = r0 + 16 * u + n16;
          r = r >= P.Wq ? r - P.Wq : r;
          if (r >= P.W) s[u] = DEAD_LOGIT;
        }
      }
      online_softmax_rows<NNT, VPIECES == 1>(st, s, p, g);

      // ---- hand the probabilities (fp16) to the lanes that feed the output step
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        _Float16 ph16 = (_Float16)p[u];
        // Two pieces and no carried product residual (bf16 caches): the head piece keeps only the three
        // leading significant bits of p, so that its product with a value scale - a bf16 number, 8
        // significant bits - is exact in fp16; the rounding of the product then hits the second piece
        // only, which is at most a quarter of p.
        if constexpr (VPIECES == 2 && !PROD_LO)
          ph16 = __builtin_bit_cast(_Float16, (uint16_t)(__builtin_bit_cast(uint16_t, ph16) & 0xFF00u));
        p_wr[(u >> 1) * (9 * 32) + 16 * (u & 1)] = __builtin_bit_cast(uint16_t, ph16);
        if constexpr (VPIECES == 2)   // what the head piece leaves out, for the residual rows
          p_wr[(u >> 1) * (9 * 32) + 16 * (u & 1) + 5 * 32] = __builtin_bit_cast(uint16_t, (_Float16)(p[u] - (float)ph16));
      }
      wave_lds_sync();

      // ---- output: two 32-token steps x NNT channel tiles
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const uint2 pa = *reinterpret_cast<const uint2*>(p_rd + ks * (9 * 32));        // tokens 4*q4 .. +3
        const uint2 pb = *reinterpret_cast<const uint2*>(p_rd + ks * (9 * 32) + 16);   // tokens 16 + 4*q4 .. +3
        const uint32_t ph[4] = {pa.x, pa.y, pb.x, pb.y};      // slots (0,1) (2,3) (4,5) (6,7)
        uint32_t hd[4] = {pa.x, pa.y, pb.x, pb.y};            // the head piece of the same slots
        if constexpr (PROD_LO && VPIECES == 2) {
          const uint2 ha = *reinterpret_cast<const uint2*>(p_hd + ks * (9 * 32));
          const uint2 hb = *reinterpret_cast<const uint2*>(p_hd + ks * (9 * 32) + 16);
          hd[0] = ha.x; hd[1] = ha.y; hd[2] = hb.x; hd[3] = hb.y;
        }
        uint4 vsr = cur.vs[ks], vzr = cur.vz[ks];
        if (partial) {   // slots beyond n_q hold unspecified bits: keep them out of the sums
          uint32_t keep[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i0 = 2 * r, i1 = 2 * r + 1;
            const int x0 = 16 * ((i0 >> 2) & 1) + 4 * q4 + (i0 & 3), x1 = 16 * ((i1 >> 2) & 1) + 4 * q4 + (i1 & 3);
            keep[r] = (64 * t + 32 * ks + x0 < n_q ? 0x0000FFFFu : 0u) |
                      (64 * t + 32 * ks + x1 < n_q ? 0xFFFF0000u : 0u);
          }
          vsr.x &= keep[0]; vsr.y &= keep[1]; vsr.z &= keep[2]; vsr.w &= keep[3];
          vzr.x &= keep[0]; vzr.y &= keep[1]; vzr.z &= keep[2]; vzr.w &= keep[3];
        }
        const uint32_t vsw[4] = {vsr.x, vsr.y, vsr.z, vsr.w}, vzw[4] = {vzr.x, vzr.y, vzr.z, vzr.w};
        uint32_t aw[4], al[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const half2_t pp = __builtin_bit_cast(half2_t, ph[v]);
          const half2_t sv = meta_pair(vsw[v]);
          if constexpr (!PROD_LO) {
            aw[v] = __builtin_bit_cast(uint32_t, pp * sv);
          } else if constexpr (VPIECES == 2) {
            // head rows: p_hi * vs rounded; residual rows: what that rounding dropped plus p_lo * vs
            const half2_t hh = __builtin_bit_cast(half2_t, hd[v]);
            const half2_t hi = hh * sv;
            const half2_t lo = __builtin_elementwise_fma(pp, sv, __builtin_elementwise_fma(hh, sv, -hi));
            aw[v] = __builtin_bit_cast(uint32_t, tail_row ? lo : hi);
          } else {
            const half2_t hi = pp * sv;
            aw[v] = __builtin_bit_cast(uint32_t, hi);
            al[v] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(pp, sv, -hi));
          }
          st.zacc[v] = __builtin_amdgcn_fdot2(pp, meta_pair(vzw[v]), st.zacc[v], false);
        }
        const uint4 a = make_uint4(aw[0], aw[1], aw[2], aw[3]);
#pragma unroll
        for (int nt = 0; nt < NNT; ++nt) {
          const uint4 b = operand_codes<BITS>(cur.vc[ks].w, nt);
          st.acc[nt] = mfma_f16(a, b, st.acc[nt]);
          if constexpr (PROD_LO && VPIECES == 1)   // no spare rows: the dropped part takes a product of its own
            st.acc[nt] = mfma_f16(make_uint4(al[0], al[1], al[2], al[3]), b, st.acc[nt]);
        }
        load_v(cur, tn, ks);
      }
      wave_lds_sync();   // p_lds and qs_lds are rewritten by the next tile
    };

    if (ta < TQ) {
      while (true) {
        const bool more = tb < TQ;
        const int kd = draw();                 // for the tile after tb
        process(A, ta, more ? tb : ta);
        if (!more) break;
        ta = tb;
        tb = drawn_tile(kd);
      }
    }
    // canonical partial of this wavefront: o[g][c], m[g], l[g]
    float lsum = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) lsum += st.l[u] * __builtin_amdgcn_exp2f(-offs[u]);
    const float l_tot = row_sum(lsum);
    float zs = 0.f;
    {
#pragma unroll
      for (int v = 0; v < 4; ++v) zs += st.zacc[v] * __builtin_ldexpf(1.f, -pos_exp<BITS>(v));
    }
    zs = rows_sum(zs);
    if (q4 == 0) zs_lds[wave][up][g] = zs;       // the residual rows hold the residual's share of sum_t p_t vz_t
    if (n16 == 0) { ml_lds[wave][q4][0] = st.m; ml_lds[wave][q4][1] = l_tot; }
    wave_lds_sync();
    // the accumulators of lane group q4 are the rows of channel group q4 (and of its
    // residual piece, q4 + NGC): sum_t p_t vz_t of that group, both pieces, per head
    if constexpr (VPIECES == 2 && NGC == 2) {
      // Two channel groups, two pieces: lane groups 0 and 2 hold the two pieces of
      // channel group 0, lane groups 1 and 3 those of channel group 1.  One swap of
      // the 32-lane halves of two registers sums the pieces of FOUR channel tiles at
      // once - lane group 0 ends up with the total of tile a, 2 with that of tile b
      // (both of channel group 0), 1 and 3 with tiles c and d of channel group 1 - and
      // every lane group writes its own.
      constexpr int T0 = G / 16;                 // channel tiles of group 0 (group 1: the rest, at most as many)
      const int grp = q4 & 1;
      float zsv[4];
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) zsv[gg] = zs_lds[wave][grp][gg] + zs_lds[wave][grp + NGC][gg];
#pragma unroll
      for (int k = 0; k < (T0 + 1) / 2; ++k) {
        constexpr int NONE = -1;
        const int ta = 2 * k, tb = 2 * k + 1 < T0 ? 2 * k + 1 : NONE;
        const int tc = T0 + 2 * k < NNT ? T0 + 2 * k : NONE, td = T0 + 2 * k + 1 < NNT ? T0 + 2 * k + 1 : NONE;
        const int mine = grp ? (q4 >> 1 ? td : tc) : (q4 >> 1 ? tb : ta);
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          const float xa = st.acc[ta][gg], xb = st.acc[tb == NONE ? ta : tb][gg];
          const float xc = st.acc[tc == NONE ? ta : tc][gg], xd = st.acc[td == NONE ? ta : td][gg];
          const unsigned X = __float_as_uint(grp ? xc : xa), Y = __float_as_uint(grp ? xd : xb);
          const auto r = __builtin_amdgcn_permlane32_swap(X, Y, false, false);
          const float tot = __uint_as_float(r[0]) + __uint_as_float(r[1]);
          if (mine != NONE) o_lds[wave][gg][16 * mine + n16] = tot * CODE_SCALE<BITS> + zsv[gg];
        }
      }
    } else {
      const int gq = q4 < NGC ? q4 : 0;
      float zsv[4];
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) {
        zsv[gg] = zs_lds[wave][gq][gg];
        if constexpr (VPIECES == 2) zsv[gg] += zs_lds[wave][gq + NGC][gg];
      }
#pragma unroll
      for (int nt = 0; nt < NNT; ++nt) {
        const int gc = (16 * nt) / G;
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          float a = st.acc[nt][gg];
          if constexpr (VPIECES == 2) {   // add the residual piece's row: lane group q4 + NGC
            float x, y;
            if constexpr (NGC == 2) xor32_pair(a, &x, &y); else xor16_pair(a, &x, &y);
            a = x + y;
          }
          if (q4 == gc) o_lds[wave][gg][16 * nt + n16] = a * CODE_SCALE<BITS> + zsv[gg];
        }
      }
    }
  } else {
    // ------------------------- original-precision rows -------------------------
    const int wf = gw;
    const int64_t fp_slice = (int64_t)bh * P.cap * D;
    const uint16_t* kb = k_fp + fp_slice + lane * 8;
    const uint16_t* vb = v_fp + fp_slice + lane * 8;
    uint4 qreg[NKC];
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
      qreg[kc] = *reinterpret_cast<const uint4*>(P.q + qrow + 32 * kc + 8 * q4);
      if (!head_ok) qreg[kc] = make_uint4(0, 0, 0, 0);
    }
    // Fused append: the wavefront that owns the unit receiving the new row fetches the row
    // right away, so that it has arrived by the time that unit is processed.
    const int new_unit = (n_fp - 1) >> 5, new_sx = (n_fp - 1) & 31, new_kx = kperm(new_sx);
    const bool owner = P.k_new && new_unit >= wf && (new_unit - wf) % NWF == 0;
    uint4 kn_r[NKC];
    uint32_t vn_r[NNT];
    if (owner) {
      const uint16_t* kn = P.k_new + (int64_t)bh * D;
      const uint16_t* vn = P.v_new + (int64_t)bh * D;
#pragma unroll
      for (int kc = 0; kc < NKC; ++kc) kn_r[kc] = *reinterpret_cast<const uint4*>(kn + 32 * kc + 8 * q4);
#pragma unroll
      for (int nt = 0; nt < NNT; ++nt) vn_r[nt] = vn[16 * nt + n16];
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

      if (owner && unit == new_unit) {
        // Fused append.  This wavefront is the only reader of the unit that receives
        // the new row: it takes the row from the caller's buffers instead of the cache
        // (whatever the loads above found in that slot is replaced) and stores it into
        // the cache for the steps to come (once per (b, kv head): head group 0).
        const int sx = new_sx, uu_ = sx >> 4;
        if (n16 == (sx & 15)) {
#pragma unroll
          for (int kc = 0; kc < NKC; ++kc) {
            const uint4 x = kn_r[kc];
            if (uu_ == 0) ka[0][kc] = x; else ka[1][kc] = x;
            if (hsub == 0)
              *reinterpret_cast<uint4*>(k_fp_w + fp_slice + lane * 8 + ((int64_t)(2 * unit + uu_) * NKC + kc) * 512) = x;
          }
        }
        const int kx = new_kx;         // element kx & 7 of the lanes of token octet kx >> 3
        if (q4 == (kx >> 3)) {
          const int sh = 16 * (kx & 1), wi = (kx & 7) >> 1;
#pragma unroll
          for (int nt = 0; nt < NNT; ++nt) {
            const uint32_t e = vn_r[nt];
            uint32_t w[4] = {va[nt].x, va[nt].y, va[nt].z, va[nt].w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (i == wi) w[i] = (w[i] & ~(0xFFFFu << sh)) | (e << sh);
            va[nt] = make_uint4(w[0], w[1], w[2], w[3]);
            if (hsub == 0)
              v_fp_w[fp_slice + (((int64_t)unit * NNT + nt) * 64 + lane) * 8 + (kx & 7)] = (uint16_t)e;
          }
        }
        if (hsub == 0 && bh % P.Hkv == 0 && lane == 0)
          pos_fp[(bh / P.Hkv) * P.cap + n_fp - 1] = n_fp - 1 + n_tok_q;
      }

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
        for (int j = 0; j < 4; ++j) s[j] = (up < 2 && tok0 + j < n_fp) ? d[j] * P.c : -INFINITY;
      }
      online_softmax<NNT, false>(st, s, p);

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
      if (32 * unit + 32 > n_fp) {   // slots beyond n_fp hold unspecified bits
        uint32_t keep[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i0 = 2 * r, i1 = 2 * r + 1;
          const int x0 = 16 * ((i0 >> 2) & 1) + 4 * q4 + (i0 & 3), x1 = 16 * ((i1 >> 2) & 1) + 4 * q4 + (i1 & 3);
          keep[r] = (32 * unit + x0 < n_fp ? 0x0000FFFFu : 0u) | (32 * unit + x1 < n_fp ? 0xFFFF0000u : 0u);
        }
#pragma unroll
        for (int nt = 0; nt < NNT; ++nt) {
          va[nt].x &= keep[0]; va[nt].y &= keep[1]; va[nt].z &= keep[2]; va[nt].w &= keep[3];
        }
      }
#pragma unroll
      for (int nt = 0; nt < NNT; ++nt) st.acc[nt] = mfma_T<BF16>(a, va[nt], st.acc[nt]);
    }
    const float l_tot = head_sum((st.l[0] + st.l[1]) + (st.l[2] + st.l[3]));
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
  // merge the wavefronts; write this split's partial: per head D floats, then m, l
  for (int idx = threadIdx.x; idx < P.hb * D; idx += 64 * NWB) {
    const int gg = idx / D, c = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NWB; ++w) M = fmaxf(M, ml_lds[w][gg][0]);
    float acc = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < NWB; ++w) {
      const float mw = ml_lds[w][gg][0];
      const float a = mw == -INFINITY ? 0.f : exp2f(mw - M);
      acc += a * o_lds[w][gg][c];
      L += a * ml_lds[w][gg][1];
    }
    if (P.splits == 1) {   // nothing to merge across workgroups: this is the result
      P.out[((int64_t)bh * P.gh + hsub * P.hb + gg) * D + c] = f2t<BF16>(acc / L);
      continue;
    }
    const int64_t base = part_base + gg * (D + 4);
    st_dev(P.ws + base + c, acc);
    if (c == 0) { st_dev(P.ws + base + D, M); st_dev(P.ws + base + D + 1, L); }
  }
  if (P.splits == 1) return;

  // ---- ticket: the last workgroup of this (b, kv head, head group) merges the splits.
  // The barrier waits for this workgroup's stores to be acknowledged before thread 0
  // draws; a workgroup that draws the last ticket therefore finds every partial.
  __shared__ int is_last;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0): the write-through stores above have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    int* ctr = P.counters + group * (CTR_LINES * CTR_LINE);
    const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    is_last = old == P.splits - 1;
    if (is_last) {   // every other workgroup is past its tile loop and its ticket: re-arm for the next launch
#pragma unroll
      for (int i = 0; i < CTR_LINES; ++i)
        __hip_atomic_store(ctr + i * CTR_LINE, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
  if (!is_last) return;
  static_assert(NWB * 4 * D >= 4 * 256, "o_lds too small for the merge weights");
  static_assert(NWB >= 4, "one wavefront per head merges the splits");
  float* w_lds = &o_lds[0][0][0];              // [4][256] weights, o_lds is free again
  // Wavefront w merges head w.  The partials are read past the caches (device-
  // coherent loads), 16 bytes per lane so that the address unit sees few, wide
  // instructions, and all of them are issued before anything is consumed: the merge
  // then costs about one memory round trip.
  if (wave < P.hb) {
    constexpr int PR = D + 4;                    // floats per partial row
    constexpr int C4 = D / 4;                    // 16-byte chunks per row
    constexpr int RPI = 64 / C4;                 // rows covered by one wave-level load
    constexpr int PASS = 32;                     // splits per pass
    constexpr int NI = PASS / RPI;               // loads per pass
    const int rows = P.splits;
    const int64_t gstride = (int64_t)P.gh * PR;  // floats between consecutive splits
    const float* gbase = P.ws + ((int64_t)bh * P.splits * P.gh + hsub * P.hb + wave) * PR;
    // buffer descriptor over this head's rows of all splits: out-of-range lanes read 0
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(gbase), 0, (int)(((int64_t)(rows - 1) * gstride + PR) * 4), 0x00020000);
    const int r = lane / C4, c4 = lane % C4;
    const int oob = 0x7FFFFFF0;
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    u32x2 ml[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int sidx = lane + 64 * k;
      ml[k] = __builtin_amdgcn_raw_buffer_load_b64(rs, sidx < rows ? (int)((sidx * gstride + D) * 4) : oob, 0, 16);
    }
    u32x4 ov[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int sidx = i * RPI + r;
      ov[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (r < RPI && sidx < rows) ? (int)((sidx * gstride + 4 * c4) * 4) : oob, 0, 16);
    }
    float m[4], l[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool live = lane + 64 * k < rows;
      m[k] = live ? __uint_as_float(ml[k][0]) : -INFINITY;
      l[k] = live ? __uint_as_float(ml[k][1]) : 0.f;
    }
    float mx = fmaxf(fmaxf(m[0], m[1]), fmaxf(m[2], m[3]));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float ls = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float w = m[k] == -INFINITY ? 0.f : exp2f(m[k] - mx);
      w_lds[wave * 256 + lane + 64 * k] = w;
      ls += w * l[k];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) ls += __shfl_xor(ls, o);
    wave_lds_sync();
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0;;) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int sidx = s0 + i * RPI + r;
        const float w = (r < RPI && sidx < rows) ? w_lds[wave * 256 + sidx] : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaf(w, __uint_as_float(ov[i][e]), acc[e]);
      }
      s0 += PASS;
      if (s0 >= rows) break;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int sidx = s0 + i * RPI + r;
        ov[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (r < RPI && sidx < rows) ? (int)((sidx * gstride + 4 * c4) * 4) : oob, 0, 16);
      }
    }
    // add the RPI row classes: lanes c4, c4 + C4, ...
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t = acc[e];
#pragma unroll
      for (int k = 1; k < RPI; ++k) t += __shfl(acc[e], (lane + k * C4) & 63);
      acc[e] = t;
    }
    if (lane < C4) {
      const float inv = 1.0f / ls;
      uint16_t* o = P.out + ((int64_t)bh * P.gh + hsub * P.hb + wave) * D + 4 * c4;
      const uint32_t lo = (uint32_t)f2t<BF16>(acc[0] * inv) | ((uint32_t)f2t<BF16>(acc[1] * inv) << 16);
      const uint32_t hi = (uint32_t)f2t<BF16>(acc[2] * inv) | ((uint32_t)f2t<BF16>(acc[3] * inv) << 16);
      *reinterpret_cast<uint2*>(o) = make_uint2(lo, hi);
    }
  }
}

template <bool BF16, int D, int NWB, int BITS>
static hipError_t launch_mfma_dg(const Shape& s, const AttnParams& P, const SeqArg* seq, dim3 grid, hipStream_t st) {
  if constexpr (NWB == 8 || NWB == 12) {
    if (s.Wq != s.W || seq) {
      SeqArgs<true> S;
      if (seq && seq->in_args())
        for (int i = 0; i < seq->n; ++i) S.e[i] = seq->host[i];
      switch (s.G) {
        case 32: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 32, NWB, BITS, true>), grid, dim3(64 * NWB), 0, st, P, S); break;
        case 64: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 64, NWB, BITS, true>), grid, dim3(64 * NWB), 0, st, P, S); break;
        default: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 128, NWB, BITS, true>), grid, dim3(64 * NWB), 0, st, P, S); break;
      }
      return launch_status(__func__);
    }
  }
  const SeqArgs<false> S;
  switch (s.G) {
    case 32: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 32, NWB, BITS>), grid, dim3(64 * NWB), 0, st, P, S); break;
    case 64: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 64, NWB, BITS>), grid, dim3(64 * NWB), 0, st, P, S); break;
    default: hipLaunchKernelGGL((attn_mfma_kernel<BF16, D, 128, NWB, BITS>), grid, dim3(64 * NWB), 0, st, P, S); break;
  }
  return launch_status(__func__);
}

template <bool BF16, int NWB, int BITS>
static hipError_t launch_mfma_d(const Shape& s, const AttnParams& P, const SeqArg* seq, dim3 grid, hipStream_t st) {
  switch (s.d) {
    case 64: return launch_mfma_dg<BF16, 64, NWB, BITS>(s, P, seq, grid, st);
    case 96: return launch_mfma_dg<BF16, 96, NWB, BITS>(s, P, seq, grid, st);
    default: return launch_mfma_dg<BF16, 128, NWB, BITS>(s, P, seq, grid, st);
  }
}

template <int NWB, int BITS>
static hipError_t launch_mfma_t(const Shape& s, const AttnParams& P, const SeqArg* seq, dim3 grid, hipStream_t st) {
  return s.bf16 ? launch_mfma_d<true, NWB, BITS>(s, P, seq, grid, st)
                : launch_mfma_d<false, NWB, BITS>(s, P, seq, grid, st);
}

// seq == nullptr: every sequence has the counts of `c` and the live buffer c.cur;
// otherwise the kernel reads counts, live buffer and fp-wavefront share per sequence
// from the state array (in its own arguments for small batches, else on the device;
// c.n_fp / c.n_q are then the largest counts, which `plan` was made for).
hipError_t launch_decode_attn_mfma(const Shape& s, const lq_cache& c, const void* q, float scale,
                                   void* out, const Workspace& ws, const lq_plan& plan, hipStream_t st,
                                   const void* k_new, const void* v_new, const SeqArg* seq) {
  AttnParams P;
  P.k_new = (const uint16_t*)k_new; P.v_new = (const uint16_t*)v_new;
  const int first = seq ? 0 : c.cur;
  P.k_fp[0] = (uint16_t*)c.k_fp[first]; P.k_fp[1] = (uint16_t*)c.k_fp[first ^ 1];
  P.v_fp[0] = (uint16_t*)c.v_fp[first]; P.v_fp[1] = (uint16_t*)c.v_fp[first ^ 1];
  P.pos_fp[0] = c.pos_fp[first]; P.pos_fp[1] = c.pos_fp[first ^ 1];
  P.seq = seq ? seq->dev : nullptr; P.seq_mode = seq_mode(seq);
  P.Hkv = s.Hkv;
  P.q = (const uint16_t*)q;
  P.k_codes = c.k_codes; P.v_codes = c.v_codes;
  P.k_scale = (const uint16_t*)c.k_scale; P.k_zero = (const uint16_t*)c.k_zero;
  P.v_scale = (const uint16_t*)c.v_scale; P.v_zero = (const uint16_t*)c.v_zero;
  P.counters = ws.counters;
  P.ws = ws.partials;
  P.out = (uint16_t*)out;
  P.cap = s.cap; P.qcap = s.qcap; P.n_fp = c.n_fp; P.n_q = c.n_q; P.gh = s.gh;
  P.W = s.W; P.Wq = s.Wq; P.n_tok_q = quantized_tokens(s, c.n_q);
  P.hb = s.gh % 4 == 0 ? 4 : (s.gh % 2 == 0 ? 2 : 1);
  P.splits = plan.splits; P.nwf = plan.fp_waves;
  P.c = scale * 1.4426950408889634f;
  static const int dynamic = [] { const char* v = getenv("LOGQUANT_ATTN_DYNAMIC"); return v && *v ? atoi(v) : 1; }();
  P.dynamic = dynamic;
  dim3 grid(plan.splits, s.B * s.Hkv * (s.gh / P.hb));
  if (s.Wq != s.W || seq) {   // padding slots, per-sequence counts: that kernel variant exists for 8 and 12 wavefronts
    if (plan.waves_per_block == 12 && s.bits == 2) return launch_mfma_t<12, 2>(s, P, seq, grid, st);
    if (plan.waves_per_block != 8) return hipErrorInvalidConfiguration;
    return s.bits == 4 ? launch_mfma_t<8, 4>(s, P, seq, grid, st) : launch_mfma_t<8, 2>(s, P, seq, grid, st);
  }
  if (plan.waves_per_block == 12 && s.bits == 2) return launch_mfma_t<12, 2>(s, P, seq, grid, st);
  if (plan.waves_per_block == 4)
    return s.bits == 4 ? launch_mfma_t<4, 4>(s, P, seq, grid, st) : launch_mfma_t<4, 2>(s, P, seq, grid, st);
  return s.bits == 4 ? launch_mfma_t<8, 4>(s, P, seq, grid, st) : launch_mfma_t<8, 2>(s, P, seq, grid, st);
}

}  // namespace lq
