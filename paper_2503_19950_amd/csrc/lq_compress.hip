// Filtering branch of Algorithm 1 (Sec. 2.5) plus quantization of what it removes
// (Fig. 6 caption, Sec. 2.3): logical fp rows 1,3,..,2W-1 are quantized to 2 bits
// (keys per channel over G evicted tokens, values per token over G channels) and
// appended to the quantized region; rows 0,2,..,2W-2 and 2W..3W-1 are moved to
// the front of the other fp buffer.
#include "lq_device.h"
#include "lq_internal.h"

namespace lq {

// One group of values: zero z = min, scale s = T((max - min) / STEPS) with the
// difference and the quotient correctly rounded to fp32.  The quotient takes three
// operations: with y = fp32(1/STEPS), q0 = fp32(a y), the remainder r = a - STEPS q0 (exact
// in one fused multiply-add), and fp32(q0 + r y) is the correctly rounded a / STEPS; for
// STEPS = 3 and 15 this was checked against the fp64 quotient rounded to fp32 (which equals
// the IEEE fp32 quotient, 53 >= 2*24 + 2) for every finite non-negative fp32 a.
// z and s (values of T) are what the codes are formed with; zt and st are what is
// stored: the same two values as fp16 (bit-identical for an fp16 cache; for a bf16
// cache exact whenever the value is in fp16's normal range).
template <bool BF16, int BITS>
__device__ __forceinline__ void group_params(float mn, float mx, float* z, float* s, uint16_t* zt,
                                             uint16_t* st) {
  if (mn == 0.f) mn = 0.f;  // -0 -> +0 (min/max do not order signed zeros)
  if (mx == 0.f) mx = 0.f;
  constexpr float STEPS = (float)((1 << BITS) - 1), y = 1.0f / STEPS;
  const float diff = mx - mn;
  const float q0 = diff * y;
  float quo = __fmaf_rn(__fmaf_rn(-STEPS, q0, diff), y, q0);
  asm("" : "+v"(quo));      // the fp32 quotient is rounded before the conversion to T: keeps the compiler from
                            // merging the last operation and the conversion into one that rounds once, to fp16
  *s = t2f<BF16>(f2t<BF16>(quo));
  *z = mn;                  // an element of T
  *st = f2t<false>(*s);
  *zt = f2t<false>(mn);
}

// Encoder of one group: round-half-up of (x - z)/s clamped to 0..2^BITS-1, by
// threshold compares on the exact (fp64) difference; (k + 0.5) * s is exact in fp64.
// The thresholds grow with k, so with 4 bits the number of them that x - z reaches is found
// by bisection (BITS compares instead of 2^BITS - 1).
template <int BITS>
struct Encoder {
  double z, sd;
  bool flat;
  __device__ __forceinline__ Encoder(float zf, float s) {
    z = (double)zf; sd = (double)s; flat = s == 0.f;
  }
  __device__ __forceinline__ uint32_t operator()(float x) const {
    const double dl = (double)x - z;
    uint32_t c = 0;
#pragma unroll
    for (int step = 1 << (BITS - 1); step >= 1; step >>= 1)
      if (dl >= ((double)(c + step) - 0.5) * sd) c += step;
    return flat ? 0u : c;
  }
};
// ---- 2-bit groups: statistics and codes on order-preserving 16-bit keys, two values per
// instruction.  The bits of a T value (sign, then magnitude) map to an unsigned key that
// orders like the value: negative values have every bit flipped, the others the sign bit
// set (-0 -> 0x7FFF sits just below +0 -> 0x8000).  Minima and maxima are then unsigned
// packed min/max.  For the codes, x - z >= (k + 1/2) s  <=>  x >= z + (k + 1/2) s, that sum
// is exact in fp64 (s comes from a group that holds z, so it is at least a third of the
// spacing of T at |z|: the two addends lie within 13 binary places of each other, with at
// most 11 and 14 significant bits), and since x is a value of T it reaches the sum exactly
// when it reaches the smallest value of T at or above it.  The three thresholds are turned
// into keys once per group - each by one of the lanes that share the group, handed round by
// lane shuffles - and per pair of values the code is then two threshold tests (a packed
// saturating subtraction and a packed minimum each) and two packed multiply-adds.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u16x2 keys_of(uint32_t w) {   // two T values -> two keys
  const i16x2 x = __builtin_bit_cast(i16x2, w);
  const i16x2 flip = (x >> 15) | (i16x2)((short)0x8000);   // 0xFFFF for a negative value, 0x8000 otherwise
  return __builtin_bit_cast(u16x2, x ^ flip);
}
__device__ __forceinline__ uint32_t key_of(uint16_t bits) { return (bits & 0x8000u) ? (~(uint32_t)bits & 0xFFFFu) : (bits | 0x8000u); }
__device__ __forceinline__ uint16_t bits_of_key(uint32_t key) { return (uint16_t)((key & 0x8000u) ? (key ^ 0x8000u) : (~key & 0xFFFFu)); }

// key(smallest value of T that is >= t) - 1: a key above it belongs to a value that reaches t.
// f = fp32(t) and "up" = [f < t] locate t between neighbouring fp32 numbers; h = T(f) is a
// neighbour of f in T.  The smallest value of T at or above t is h, or the next one upwards
// (the next key: keys step with the values whatever the sign) when h < f, or when h == f
// and t lies above f.  A threshold of zero (either sign) is taken as -0, which both zeros
// reach.  In a flat group (s == 0) every code is 0: 0xFFFF, which no key exceeds.
template <bool BF16>
__device__ __forceinline__ uint32_t threshold_key(float zf, float s, float k_plus_half) {
  const double t = (double)zf + (double)k_plus_half * (double)s;   // exact
  const float f = (float)t;
  const bool up = (double)f < t;
  const uint16_t h = f2t<BF16>(f);
  const float hb = t2f<BF16>(h);
  uint32_t key = key_of(h) + ((hb < f || (hb == f && up)) ? 1u : 0u);
  if (key == 0x8000u) key = 0x7FFFu;
  return s == 0.f ? 0xFFFFu : key - 1u;
}

// codes of two keys; tk[k]: the two values' k-th thresholds (low half: first value).  [key > t] per half is
// min(key -sat t, 1).  Two such tests: the middle threshold gives the high bit b1, the lower or the upper one -
// t0 + b1 (t2 - t0), a packed multiply-add - the low bit.  Written as instructions because the compiler turns
// the expression into 16-bit compares and selects, one value at a time.
__device__ __forceinline__ u16x2 codes_of(u16x2 key, const u16x2* tk, u16x2 t20) {   // t20 = tk[2] - tk[0]
  uint32_t c, b;
  asm("v_pk_sub_u16 %1, %2, %4 clamp\n\t"
      "v_pk_min_u16 %1, %1, %6\n\t"          // b1
      "v_pk_mad_u16 %0, %1, %5, %3\n\t"      // the threshold that decides the low bit
      "v_pk_sub_u16 %0, %2, %0 clamp\n\t"
      "v_pk_min_u16 %0, %0, %6\n\t"          // b0
      "v_pk_mad_u16 %0, %1, %7, %0"            // 2 b1 + b0
      : "=&v"(c), "=&v"(b)
      : "v"(__builtin_bit_cast(uint32_t, key)), "v"(__builtin_bit_cast(uint32_t, tk[0])),
        "v"(__builtin_bit_cast(uint32_t, tk[1])), "v"(__builtin_bit_cast(uint32_t, t20)), "v"(0x00010001u), "v"(0x00020002u));
  return __builtin_bit_cast(u16x2, c);
}

// Minimum and maximum over the lanes that differ in the bits CPW .. 32 of the lane index
// (CPW = 8 or 16), by wavefront shuffles: a rotation by 8 inside the row of 16 lanes, then the
// swap instructions, which trade rows (halves) between two registers - swapping a register
// with a copy of itself leaves one holding the even rows (lower half) twice and the other the
// odd rows (upper half) twice, so the minimum of the two is the minimum over both.
template <int CPW>
__device__ __forceinline__ void reduce_over_parts(float* mn, float* mx) {
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    if constexpr (CPW <= 8) {
      mn[k] = fminf(mn[k], __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mn[k]), 0x128, 0xF, 0xF, false)));   // row_ror:8
      mx[k] = fmaxf(mx[k], __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx[k]), 0x128, 0xF, 0xF, false)));
    }
    {
      const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(mn[k]), __float_as_uint(mn[k]), false, false);
      const auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(mx[k]), __float_as_uint(mx[k]), false, false);
      mn[k] = fminf(__uint_as_float(a[0]), __uint_as_float(a[1]));
      mx[k] = fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
    }
    {
      const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(mn[k]), __float_as_uint(mn[k]), false, false);
      const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx[k]), __float_as_uint(mx[k]), false, false);
      mn[k] = fminf(__uint_as_float(a[0]), __uint_as_float(a[1]));
      mx[k] = fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
    }
  }
}

// The same reduction for packed keys (two channels per register).
template <int CPW>
__device__ __forceinline__ void reduce_keys_over_parts(u16x2& mn, u16x2& mx) {
  uint32_t a = __builtin_bit_cast(uint32_t, mn), b = __builtin_bit_cast(uint32_t, mx);
  auto lo = [](uint32_t x, uint32_t y) { return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, x), __builtin_bit_cast(u16x2, y))); };
  auto hi = [](uint32_t x, uint32_t y) { return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, x), __builtin_bit_cast(u16x2, y))); };
  if constexpr (CPW <= 8) {
    a = lo(a, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x128, 0xF, 0xF, false));   // row_ror:8
    b = hi(b, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)b, 0x128, 0xF, 0xF, false));
  }
  {
    const auto p = __builtin_amdgcn_permlane16_swap(a, a, false, false);
    const auto q = __builtin_amdgcn_permlane16_swap(b, b, false, false);
    a = lo(p[0], p[1]); b = hi(q[0], q[1]);
  }
  {
    const auto p = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const auto q = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    a = lo(p[0], p[1]); b = hi(q[0], q[1]);
  }
  mn = __builtin_bit_cast(u16x2, a); mx = __builtin_bit_cast(u16x2, b);
}

// Eight codes (one byte each, in x: elements 0..3, y: elements 4..7) -> the operand
// order of the packed layouts: element i at bit BITS*(i>>1) + 16*(i&1).
template <int BITS>
__device__ __forceinline__ uint32_t pack8(uint32_t x, uint32_t y) {
  constexpr uint32_t M = (1u << BITS) - 1u;
  uint32_t w = (x & M) | (((x >> 8) & M) << 16) | (((x >> 16) & M) << BITS) | (((x >> 24) & M) << (16 + BITS));
  w |= ((y & M) << (2 * BITS)) | (((y >> 8) & M) << (16 + 2 * BITS)) | (((y >> 16) & M) << (3 * BITS)) |
       (((y >> 24) & M) << (16 + 3 * BITS));
  return w;
}

// The same for two operands of 2-bit codes at once (the two byte positions h = 0, 1 of a word), the bytes
// holding nothing but a code (0..3): t = x | y << 4 has elements j and 4 + j in byte j; t | t >> 14 then has
// bytes 0 and 2 (elements 0, 2, 4, 6: the low half's byte) interleaved in its byte 0 and bytes 1 and 3 (the
// high half's) in its byte 1; one byte permute puts the four bytes of the two operands in place.
__device__ __forceinline__ uint32_t pack16_2bit(uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1) {
  const uint32_t t0 = x0 | (y0 << 4), t1 = x1 | (y1 << 4);
  const uint32_t u0 = t0 | (t0 >> 14), u1 = t1 | (t1 >> 14);
  return __builtin_amdgcn_perm(u1, u0, 0x05010400u);   // bytes: u0.0, u1.0, u0.1, u1.1
}

// Where the G rows of one key group come from.
// (a) the filtering step on a full list: odd logical slots of the live fp buffer
template <int d, int G>
struct FpSource {
  static constexpr int nkc = d >> 5, nnt = d >> 4;
  const uint16_t* k_fp;   // slice base
  const uint16_t* v_fp;
  const int32_t* pos_fp;  // row of this batch entry
  int j;
  int ng;                 // rows of this group (G, fewer in the last group of an event when G does not divide W)
  int cap;                // rows allocated per slice (multiple of 32)
  // Not null: this workgroup also moves the rows that stay - the even logical slots 2jG .. 2jG + 2G - 2 of
  // the lines it reads anyway - to slots jG .. jG + G - 1 of the other buffer (slice bases).  Only for
  // whole groups with d a multiple of 64.
  uint16_t* k_keep;
  uint16_t* v_keep;
  // FULL: the group has all G rows (compile-time trip counts, no row checks)
  template <bool FULL>
  __device__ __forceinline__ void stage_keys(uint16_t* sm, int ld) const {
    for (int idx = threadIdx.x; idx < G * nkc * 4; idx += 256) {
      const int oct = idx % (nkc * 4), e = idx / (nkc * 4);
      const int ts = 2 * (j * G + e) + 1;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (FULL || e < ng) v = *reinterpret_cast<const uint4*>(k_fp + k_fp_index(ts, oct * 8, nkc));
      uint32_t* dst = reinterpret_cast<uint32_t*>(sm + e * ld + oct * 8);
      dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
      if (FULL && k_keep)   // the row before it (same 32 bytes) stays: 16 bytes to its new slot
        *reinterpret_cast<uint4*>(k_keep + k_fp_index(j * G + e, oct * 8, nkc)) =
            *reinterpret_cast<const uint4*>(k_fp + k_fp_index(ts - 1, oct * 8, nkc));
    }
  }
  // The value rows are fetched into registers while the keys are being processed (the
  // loads are issued before the key phase and first used after it) and written to LDS
  // afterwards.  Source rows: logical slots 2jG .. 2jG + 2G - 1 (whole 32-slot tiles).
  static constexpr int VLOADS = ((2 * G >> 5) * nnt * 64 + 255) / 256;
  struct ValueRegs { uint4 v[VLOADS]; };
  template <bool FULL>
  __device__ __forceinline__ ValueRegs load_values() const {
    ValueRegs r;
#pragma unroll
    for (int it = 0; it < VLOADS; ++it) {
      const int idx = threadIdx.x + 256 * it;
      const int lane = idx & 63, nt = (idx >> 6) % nnt, sb = idx / (64 * nnt);
      const int tile = ((2 * j * G) >> 5) + sb;
      const int64_t src = (((int64_t)tile * nnt + nt) * 64 + lane) * 8;
      r.v[it] = make_uint4(0u, 0u, 0u, 0u);
      if (idx < (2 * G >> 5) * nnt * 64 && (FULL || (32 * tile < cap && 16 * sb < ng)))
        r.v[it] = *reinterpret_cast<const uint4*>(v_fp + src);
    }
    return r;
  }
  template <bool FULL>
  __device__ __forceinline__ void store_values(const ValueRegs& r, uint16_t* sm, int ld) const {
    if constexpr (FULL && nnt % 4 == 0) {
      if (v_keep) {
        // The rows that stay are the even elements (low halves) of the registers just loaded.  Lane (qq, n)
        // of old tile sb holds old slots 4qq, 4qq+2, 16+4qq, 16+4qq+2 -> new slots 16 (sb & 1) + 2qq, +1 and
        // 16 (sb & 1) + 8 + 2qq, +1 of new tile sb >> 1: word 2 (sb & 1) + (qq & 1) of new lane (qq >> 1, n)
        // and of new lane (2 + (qq >> 1), n).  A thread holds both old tiles of a new one (registers k and
        // PER_SB + k of the pair); the row swap gives both rows of a pair (qq, qq ^ 1) each other's words,
        // and then the even row stores the 16 bytes of new lane qq >> 1, the odd row those of 2 + (qq >> 1).
        constexpr int PER_SB = nnt / 4;   // registers per thread and old tile
        const int lane = threadIdx.x & 63, qq = lane >> 4, n = lane & 15;
        const int to = ((qq & 1) ? 2 + (qq >> 1) : (qq >> 1)) * 16 + n;
#pragma unroll
        for (int t2 = 0; t2 < G / 32; ++t2)
#pragma unroll
          for (int k = 0; k < PER_SB; ++k) {
            const uint4 a = r.v[(2 * t2) * PER_SB + k], b = r.v[(2 * t2 + 1) * PER_SB + k];
            const int nt = (threadIdx.x >> 6) + 4 * k;
            const uint32_t a0 = (a.x & 0xFFFFu) | (a.y << 16), b0 = (a.z & 0xFFFFu) | (a.w << 16);
            const uint32_t a1 = (b.x & 0xFFFFu) | (b.y << 16), b1 = (b.z & 0xFFFFu) | (b.w << 16);
            const auto sa0 = __builtin_amdgcn_permlane16_swap(a0, a0, false, false);   // [0]: the even row's word, [1]: the odd row's
            const auto sb0 = __builtin_amdgcn_permlane16_swap(b0, b0, false, false);
            const auto sa1 = __builtin_amdgcn_permlane16_swap(a1, a1, false, false);
            const auto sb1 = __builtin_amdgcn_permlane16_swap(b1, b1, false, false);
            const uint4 out = (qq & 1) ? make_uint4(sb0[0], sb0[1], sb1[0], sb1[1]) : make_uint4(sa0[0], sa0[1], sa1[0], sa1[1]);
            *reinterpret_cast<uint4*>(v_keep + (((int64_t)((j * G >> 5) + t2) * nnt + nt) * 64 + to) * 8) = out;
          }
      }
    }
#pragma unroll
    for (int it = 0; it < VLOADS; ++it) {
      const int idx = threadIdx.x + 256 * it;
      if (idx >= (2 * G >> 5) * nnt * 64) break;
      const int lane = idx & 63, nt = (idx >> 6) % nnt, sb = idx / (64 * nnt);
      const int qq = lane >> 4, n = lane & 15;
      const uint32_t w[4] = {r.v[it].x, r.v[it].y, r.v[it].z, r.v[it].w};
#pragma unroll
      for (int i = 1; i < 8; i += 2) {  // odd element <=> odd logical slot <=> evicted
        const int x = kperm_inv(8 * qq + i);
        const int e = (sb * 32 + x - 1) >> 1;
        sm[e * ld + 16 * nt + n] = (FULL || e < ng) ? (uint16_t)(w[i >> 1] >> 16) : (uint16_t)0;
      }
    }
  }
  __device__ __forceinline__ int position(int e) const { return e < ng ? pos_fp[2 * (j * G + e) + 1] : -1; }
};
// (b) bulk prefill: rows of a row-major prompt tensor, at the positions Algorithm 1
// evicts at event `ev`
template <int d, int G>
struct PromptSource {
  const uint16_t* k;      // slice base, [L][d]
  const uint16_t* v;
  const int* posl;        // LDS: positions of the G rows
  template <bool FULL>
  __device__ __forceinline__ void stage_keys(uint16_t* sm, int ld) const { stage<FULL>(k, sm, ld); }
  // value rows: into registers before the key phase, to LDS after it
  static constexpr int VLOADS = (G * (d >> 3) + 255) / 256;
  struct ValueRegs { uint4 v[VLOADS]; };
  template <bool FULL>
  __device__ __forceinline__ ValueRegs load_values() const {
    constexpr int octs = d >> 3;
    ValueRegs r;
#pragma unroll
    for (int it = 0; it < VLOADS; ++it) {
      const int idx = threadIdx.x + 256 * it;
      const int oct = idx % octs, e = idx / octs;
      r.v[it] = make_uint4(0u, 0u, 0u, 0u);   // rows past a short group: zeros
      if (idx < G * octs && (FULL || posl[e] >= 0))
        r.v[it] = *reinterpret_cast<const uint4*>(v + (int64_t)posl[e] * d + oct * 8);
    }
    return r;
  }
  template <bool FULL>
  __device__ __forceinline__ void store_values(const ValueRegs& r, uint16_t* sm, int ld) const {
    constexpr int octs = d >> 3;
#pragma unroll
    for (int it = 0; it < VLOADS; ++it) {
      const int idx = threadIdx.x + 256 * it;
      if (idx >= G * octs) break;
      const int oct = idx % octs, e = idx / octs;
      uint32_t* dst = reinterpret_cast<uint32_t*>(sm + e * ld + oct * 8);
      dst[0] = r.v[it].x; dst[1] = r.v[it].y; dst[2] = r.v[it].z; dst[3] = r.v[it].w;
    }
  }
  template <bool FULL>
  __device__ __forceinline__ void stage(const uint16_t* x, uint16_t* sm, int ld) const {
    constexpr int octs = d >> 3;
    for (int idx = threadIdx.x; idx < G * octs; idx += 256) {
      const int oct = idx % octs, e = idx / octs;
      uint4 val = make_uint4(0u, 0u, 0u, 0u);   // rows past a short group: zeros
      if (FULL || posl[e] >= 0) val = *reinterpret_cast<const uint4*>(x + (int64_t)posl[e] * d + oct * 8);
      uint32_t* dst = reinterpret_cast<uint32_t*>(sm + e * ld + oct * 8);
      dst[0] = val.x; dst[1] = val.y; dst[2] = val.z; dst[3] = val.w;
    }
  }
  __device__ __forceinline__ int position(int e) const { return posl[e]; }
};

// Quantize one key group (ng <= G rows) of slice bh into quantized slots q0 .. q0+G-1.
// Slots past a short group (the last group of an event when G does not divide W) get
// zero codes, zero value scales and zero-points and position -1; the key statistics
// run over the ng rows only.  The staged rows past ng are zeros.
// 256 threads.  LDS: sm = staged_bytes(d, G) (the staged rows), cb = QG_CODE_BYTES
// bytes (the codes, one byte each: keys [token][d + 4], values transposed
// [channel][G + 4], so that the eight codes of a packed operand are two aligned
// 32-bit reads).
// Row pitch (in elements) of the staged KEY rows: the key statistics read one 32-bit word per
// lane with lane = part * CPW + pair and part's rows per * pitch / 2 words apart; the pitch is
// the one of d + 4, d + 6, .. that spreads a wavefront's 64 reads most evenly over the 32 LDS banks.
constexpr int key_pitch(int d, int G) {
  const int parts = d == 96 ? 4 : 512 / d, per = G / parts, cpw = 64 / parts;
  int best = d + 4, best_worst = 1 << 30;
  for (int pitch = d + 4; pitch <= d + 36; pitch += 2) {
    int hits[32] = {};
    for (int part = 0; part < parts; ++part)
      for (int cl = 0; cl < cpw; ++cl) ++hits[(part * per * (pitch / 2) + cl) % 32];
    int worst = 0;
    for (int b = 0; b < 32; ++b) worst = hits[b] > worst ? hits[b] : worst;
    if (worst < best_worst) { best_worst = worst; best = pitch; }
  }
  return best;
}
// LDS bytes of the staged rows: key pitch or value pitch (d + 4), whichever is larger
constexpr int staged_bytes(int d, int G) { return G * (key_pitch(d, G) > d + 4 ? key_pitch(d, G) : d + 4) * 2; }

template <int d, int G>
constexpr int QG_CODE_BYTES = (G * (d + 4) > d * (G + 4) ? G * (d + 4) : d * (G + 4));

template <bool BF16, int d, int G, int BITS, bool FULL, class Src>
__device__ __forceinline__ void quantize_group_t(
    uint16_t* sm, uint8_t* cb, const Src& src, int ng_in, int bh, int q0, uint32_t* __restrict__ k_codes,
    uint32_t* __restrict__ v_codes, uint16_t* __restrict__ k_scale, uint16_t* __restrict__ k_zero,
    uint16_t* __restrict__ v_scale, uint16_t* __restrict__ v_zero, int32_t* __restrict__ pos_q,
    int qcap, int Hkv) {
  const int tid = threadIdx.x;
  const int ng = FULL ? G : ng_in;        // a compile-time constant for whole groups
  constexpr int nkc = d >> 5, ngc = (d + G - 1) / G, ld = d + 4, ldk = key_pitch(d, G);
  constexpr int WPL = nkc * (BITS / 2);   // code words per lane and 32-slot block
  constexpr int KP = d + 4, VP = G + 4;   // byte pitches of the code arrays
  const int64_t code_base = ((int64_t)bh * (qcap >> 5) + (q0 >> 5)) * 64 * WPL;
  const uint32_t* cw = reinterpret_cast<const uint32_t*>(cb);

  // ---------------- keys ----------------
  src.template stage_keys<FULL>(sm, ldk);
  const typename Src::ValueRegs vregs = src.template load_values<FULL>();   // in flight during the key phase
  __syncthreads();
  // Per pair of neighbouring channels, `parts` lanes of ONE wavefront each scan a share of the
  // G tokens (one 32-bit LDS read per token, kept in registers), combine their minima and
  // maxima by wavefront shuffles and then encode their own share.  A wavefront owns CPW
  // channel pairs; lane = part * CPW + pair.  The workgroup is bound by the number of LDS
  // instructions, hence pairs, one pass over LDS, and two code bytes per write.
  {
    constexpr int PAIRS = d / 2;
    constexpr int parts = d == 96 ? 4 : 512 / d;      // lanes per channel pair (d = 96: three wavefronts work); divides G
    constexpr int per = G / parts;                    // tokens per lane
    constexpr int CPW = 64 / parts;                   // channel pairs per wavefront
    static_assert(G % parts == 0 && (PAIRS + CPW - 1) / CPW <= 4 && (CPW == 8 || CPW == 16), "key statistics split");
    const int lane = tid & 63;
    const int cp = (tid >> 6) * CPW + lane % CPW, part = lane / CPW;
    const int e0 = part * per;
    if (cp < PAIRS) {   // (whole wavefronts)
      if constexpr (BITS == 2) {
        u16x2 kv[per];
        u16x2 mn = (u16x2)((unsigned short)0xFFFF), mx = (u16x2)((unsigned short)0);
#pragma unroll
        for (int i = 0; i < per; ++i) {
          kv[i] = keys_of(*reinterpret_cast<const uint32_t*>(sm + (e0 + i) * ldk + 2 * cp));
          if (FULL || e0 + i < ng) {
            mn = __builtin_elementwise_min(mn, kv[i]);
            mx = __builtin_elementwise_max(mx, kv[i]);
          }
        }
        reduce_keys_over_parts<CPW>(mn, mx);
        float z0, s0, z1, s1;
        uint16_t zt0, st0, zt1, st1;
        group_params<BF16, BITS>(t2f<BF16>(bits_of_key(mn.x)), t2f<BF16>(bits_of_key(mx.x)), &z0, &s0, &zt0, &st0);
        group_params<BF16, BITS>(t2f<BF16>(bits_of_key(mn.y)), t2f<BF16>(bits_of_key(mx.y)), &z1, &s1, &zt1, &st1);
        if (part == 0) {
          const int64_t mi = ((int64_t)bh * (qcap / G) + q0 / G) * d + 2 * cp;
          *reinterpret_cast<uint32_t*>(k_scale + mi) = (uint32_t)st0 | ((uint32_t)st1 << 16);
          *reinterpret_cast<uint32_t*>(k_zero + mi) = (uint32_t)zt0 | ((uint32_t)zt1 << 16);
        }
        // threshold k of both channels by the lanes of row k (16 lanes: parts 16k/CPW ..), then
        // every row's word to all four rows by the swap instructions
        u16x2 tk[3];
        {
          const float kh = (float)(lane >> 4) + 0.5f;
          const uint32_t x = threshold_key<BF16>(z0, s0, kh) | (threshold_key<BF16>(z1, s1, kh) << 16);
          const auto eo = __builtin_amdgcn_permlane16_swap(x, x, false, false);       // rows 0 0 2 2 | 1 1 3 3
          const auto e = __builtin_amdgcn_permlane32_swap(eo[0], eo[0], false, false);  // rows 0 0 0 0 | 2 2 2 2
          const auto o = __builtin_amdgcn_permlane32_swap(eo[1], eo[1], false, false);  // rows 1 1 1 1 | 3 3 3 3
          tk[0] = __builtin_bit_cast(u16x2, (uint32_t)e[0]);
          tk[1] = __builtin_bit_cast(u16x2, (uint32_t)o[0]);
          tk[2] = __builtin_bit_cast(u16x2, (uint32_t)e[1]);
        }
        const u16x2 t20 = tk[2] - tk[0];
#pragma unroll
        for (int i = 0; i < per; ++i) {
          const uint32_t c = __builtin_bit_cast(uint32_t, codes_of(kv[i], tk, t20));
          *reinterpret_cast<uint16_t*>(cb + (e0 + i) * KP + 2 * cp) =
              (FULL || e0 + i < ng) ? (uint16_t)(c | (c >> 8)) : (uint16_t)0;
        }
      } else {
      uint32_t xv[per];
      float mn[2] = {INFINITY, INFINITY}, mx[2] = {-INFINITY, -INFINITY};
#pragma unroll
      for (int i = 0; i < per; ++i) {
        xv[i] = *reinterpret_cast<const uint32_t*>(sm + (e0 + i) * ldk + 2 * cp);
        if (FULL || e0 + i < ng) {
          const float x0 = t2f<BF16>((uint16_t)xv[i]), x1 = t2f<BF16>((uint16_t)(xv[i] >> 16));
          mn[0] = fminf(mn[0], x0); mx[0] = fmaxf(mx[0], x0);
          mn[1] = fminf(mn[1], x1); mx[1] = fmaxf(mx[1], x1);
        }
      }
      reduce_over_parts<CPW>(mn, mx);
      float z0, s0, z1, s1;
      uint16_t zt0, st0, zt1, st1;
      group_params<BF16, BITS>(mn[0], mx[0], &z0, &s0, &zt0, &st0);
      group_params<BF16, BITS>(mn[1], mx[1], &z1, &s1, &zt1, &st1);
      if (part == 0) {
        const int64_t mi = ((int64_t)bh * (qcap / G) + q0 / G) * d + 2 * cp;
        *reinterpret_cast<uint32_t*>(k_scale + mi) = (uint32_t)st0 | ((uint32_t)st1 << 16);
        *reinterpret_cast<uint32_t*>(k_zero + mi) = (uint32_t)zt0 | ((uint32_t)zt1 << 16);
      }
      const Encoder<BITS> enc0(z0, s0), enc1(z1, s1);
#pragma unroll
      for (int i = 0; i < per; ++i) {
        const uint32_t c0 = enc0(t2f<BF16>((uint16_t)xv[i])), c1 = enc1(t2f<BF16>((uint16_t)(xv[i] >> 16)));
        *reinterpret_cast<uint16_t*>(cb + (e0 + i) * KP + 2 * cp) =
            (FULL || e0 + i < ng) ? (uint16_t)(c0 | (c1 << 8)) : (uint16_t)0;
      }
      }
    }
  }
  __syncthreads();
  // one word per (32-slot block, lane (qq, r), m): the operand(s) of token 16*uu + r,
  // channels 32*kc + 8*qq .. +7
  for (int idx = tid; idx < (G >> 5) * 64 * WPL; idx += 256) {
    const int m = idx % WPL, lane = (idx / WPL) & 63, blk = idx / (WPL * 64);
    const int r = lane & 15, qq = lane >> 4;
    uint32_t w;
    if constexpr (BITS == 2) {
      int at[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int o = 2 * m + h, uu = o / nkc, kc = o % nkc;
        at[h] = ((blk * 32 + 16 * uu + r) * KP + 32 * kc + 8 * qq) >> 2;
      }
      w = pack16_2bit(cw[at[0]], cw[at[0] + 1], cw[at[1]], cw[at[1] + 1]);
    } else {
      const int uu = m / nkc, kc = m % nkc;
      const int at = ((blk * 32 + 16 * uu + r) * KP + 32 * kc + 8 * qq) >> 2;
      w = pack8<4>(cw[at], cw[at + 1]);
    }
    k_codes[code_base + idx] = w;
  }
  __syncthreads();

  // ---------------- values ----------------
  src.template store_values<FULL>(vregs, sm, ld);
  __syncthreads();
  // per (token, channel group): VP threads each scan a share of the channels; the
  // shares of one group sit in neighbouring lanes and are combined by lane shuffles
  {
    constexpr int vp = 2 * G * ngc > 256 ? 1 : 4 * G * ngc > 256 ? 2 : 8 * G * ngc > 256 ? 4 : 8;
    constexpr int PER = ((G < d ? G : d) + vp - 1) / vp;    // channels per thread in a full group
    static_assert(PER % 4 == 0, "a thread's channels are read four at a time");
    for (int idx = tid; idx < G * ngc * vp; idx += 256) {   // a multiple of vp; all lanes of a group take the same trips
      const int part = idx % vp, e = (idx / vp) % G, gc = idx / (vp * G);
      const int lo = gc * G, hi = min(lo + G, d);
      const int per = (hi - lo + vp - 1) / vp;              // fewer in the ragged last group (still a multiple of 4)
      const int c0 = lo + part * per, n = min(per, hi - c0);
      const uint16_t* row = sm + e * ld + c0;               // 8-byte aligned: ld and c0 are multiples of 4
      uint8_t* col = cb + c0 * VP + e;
      // one pass over LDS, four channels per read; the values stay in registers for the encode
      if constexpr (BITS == 2) {
        u16x2 ka[PER / 4], kb[PER / 4];
        u16x2 mn2 = (u16x2)((unsigned short)0xFFFF), mx2 = (u16x2)((unsigned short)0);
#pragma unroll
        for (int k = 0; k < PER / 4; ++k) {
          const uint2 x = *reinterpret_cast<const uint2*>(row + (4 * k < n ? 4 * k : 0));
          ka[k] = keys_of(x.x); kb[k] = keys_of(x.y);
          if (4 * k < n) {
            mn2 = __builtin_elementwise_min(mn2, __builtin_elementwise_min(ka[k], kb[k]));
            mx2 = __builtin_elementwise_max(mx2, __builtin_elementwise_max(ka[k], kb[k]));
          }
        }
        uint32_t mn = min((uint32_t)mn2.x, (uint32_t)mn2.y), mx = max((uint32_t)mx2.x, (uint32_t)mx2.y);
        for (int o = 1; o < vp; o <<= 1) {
          mn = min(mn, (uint32_t)__shfl_xor((int)mn, o));
          mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
        }
        float z, sc;
        uint16_t zt, st;
        group_params<BF16, BITS>(t2f<BF16>(bits_of_key(mn)), t2f<BF16>(bits_of_key(mx)), &z, &sc, &zt, &st);
        if (part == 0) {
          const int64_t mi = (int64_t)bh * (qcap >> 5) * ngc * 32 + v_meta_index(q0 + e, gc, ngc);
          v_scale[mi] = st;
          v_zero[mi] = zt;
        }
        // the lanes of a group share out the thresholds and hand them round inside their quad
        u16x2 tk[3];
        if constexpr (vp >= 4) {
          const uint32_t x = threshold_key<BF16>(z, sc, (float)min(part & 3, 2) + 0.5f) * 0x10001u;
          tk[0] = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x00, 0xF, 0xF, false));   // quad_perm:[0,0,0,0]
          tk[1] = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x55, 0xF, 0xF, false));   // quad_perm:[1,1,1,1]
          tk[2] = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xAA, 0xF, 0xF, false));   // quad_perm:[2,2,2,2]
        } else if constexpr (vp == 2) {
          const uint32_t x = threshold_key<BF16>(z, sc, (float)part + 0.5f) * 0x10001u;
          tk[0] = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xA0, 0xF, 0xF, false));   // quad_perm:[0,0,2,2]
          tk[1] = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xF5, 0xF, 0xF, false));   // quad_perm:[1,1,3,3]
          tk[2] = __builtin_bit_cast(u16x2, threshold_key<BF16>(z, sc, 2.5f) * 0x10001u);
        } else {
#pragma unroll
          for (int k = 0; k < 3; ++k) tk[k] = __builtin_bit_cast(u16x2, threshold_key<BF16>(z, sc, (float)k + 0.5f) * 0x10001u);
        }
        const u16x2 t20 = tk[2] - tk[0];
#pragma unroll
        for (int k = 0; k < PER / 4; ++k)
          if (4 * k < n) {
            const u16x2 ca = codes_of(ka[k], tk, t20), cc = codes_of(kb[k], tk, t20);
            col[(4 * k + 0) * VP] = (uint8_t)ca.x;
            col[(4 * k + 1) * VP] = (uint8_t)ca.y;
            col[(4 * k + 2) * VP] = (uint8_t)cc.x;
            col[(4 * k + 3) * VP] = (uint8_t)cc.y;
          }
      } else {
      uint2 xv[PER / 4];
      float mn = INFINITY, mx = -INFINITY;
#pragma unroll
      for (int k = 0; k < PER / 4; ++k) {
        xv[k] = *reinterpret_cast<const uint2*>(row + (4 * k < n ? 4 * k : 0));
        if (4 * k < n) {
          const float a = t2f<BF16>((uint16_t)xv[k].x), b = t2f<BF16>((uint16_t)(xv[k].x >> 16));
          const float c = t2f<BF16>((uint16_t)xv[k].y), e4 = t2f<BF16>((uint16_t)(xv[k].y >> 16));
          mn = fminf(fminf(mn, fminf(a, b)), fminf(c, e4));
          mx = fmaxf(fmaxf(mx, fmaxf(a, b)), fmaxf(c, e4));
        }
      }
      for (int o = 1; o < vp; o <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
      }
      float z, sc;
      uint16_t zt, st;
      group_params<BF16, BITS>(mn, mx, &z, &sc, &zt, &st);
      if (part == 0) {
        const int64_t mi = (int64_t)bh * (qcap >> 5) * ngc * 32 + v_meta_index(q0 + e, gc, ngc);
        v_scale[mi] = st;
        v_zero[mi] = zt;
      }
      const Encoder<BITS> enc(z, sc);
#pragma unroll
      for (int k = 0; k < PER / 4; ++k)
        if (4 * k < n) {
          col[(4 * k + 0) * VP] = (uint8_t)enc(t2f<BF16>((uint16_t)xv[k].x));
          col[(4 * k + 1) * VP] = (uint8_t)enc(t2f<BF16>((uint16_t)(xv[k].x >> 16)));
          col[(4 * k + 2) * VP] = (uint8_t)enc(t2f<BF16>((uint16_t)xv[k].y));
          col[(4 * k + 3) * VP] = (uint8_t)enc(t2f<BF16>((uint16_t)(xv[k].y >> 16)));
        }
      }
    }
  }
  __syncthreads();
  // one word per (32-slot block, lane (qq, n), m): the operand(s) of channel 16*nt + n,
  // tokens kperm_inv(8*qq + i), i = 0..7: local slots 4*qq .. +3 and 16 + 4*qq .. +3
  for (int idx = tid; idx < (G >> 5) * 64 * WPL; idx += 256) {
    const int m = idx % WPL, lane = (idx / WPL) & 63, blk = idx / (WPL * 64);
    const int n = lane & 15, qq = lane >> 4;
    uint32_t w;
    if constexpr (BITS == 2) {
      const int a0 = ((16 * (2 * m) + n) * VP + blk * 32 + 4 * qq) >> 2, a1 = ((16 * (2 * m + 1) + n) * VP + blk * 32 + 4 * qq) >> 2;
      w = pack16_2bit(cw[a0], cw[a0 + 4], cw[a1], cw[a1 + 4]);
    } else {
      const int at = ((16 * m + n) * VP + blk * 32 + 4 * qq) >> 2;
      w = pack8<4>(cw[at], cw[at + 4]);
    }
    v_codes[code_base + idx] = w;
  }
  // positions of the evicted tokens, once per batch row
  if (bh % Hkv == 0) {
    const int b = bh / Hkv;
    for (int e = tid; e < G; e += 256) pos_q[(int64_t)b * qcap + q0 + e] = src.position(e);   // -1 past a short group
  }
}

template <bool BF16, int d, int G, int BITS, class Src>
__device__ __forceinline__ void quantize_group(
    uint16_t* sm, uint8_t* cb, const Src& src, int ng, int bh, int q0, uint32_t* __restrict__ k_codes,
    uint32_t* __restrict__ v_codes, uint16_t* __restrict__ k_scale, uint16_t* __restrict__ k_zero,
    uint16_t* __restrict__ v_scale, uint16_t* __restrict__ v_zero, int32_t* __restrict__ pos_q,
    int qcap, int Hkv) {
  if (ng == G)
    quantize_group_t<BF16, d, G, BITS, true>(sm, cb, src, ng, bh, q0, k_codes, v_codes, k_scale, k_zero, v_scale,
                                             v_zero, pos_q, qcap, Hkv);
  else
    quantize_group_t<BF16, d, G, BITS, false>(sm, cb, src, ng, bh, q0, k_codes, v_codes, k_scale, k_zero, v_scale,
                                              v_zero, pos_q, qcap, Hkv);
}

// Kept rows -> rows 32*nb .. 32*nb+31 of the other fp buffer of slice bh.  256 threads.
__device__ __forceinline__ void compact_rows(
    int nb, int bh, const uint16_t* __restrict__ k_old, const uint16_t* __restrict__ v_old,
    const int32_t* __restrict__ pos_old, uint16_t* __restrict__ k_new, uint16_t* __restrict__ v_new,
    int32_t* __restrict__ pos_new, int d, int W, int cap, int Hkv) {
  const int tid = threadIdx.x;
  const int nkc = d >> 5, nnt = d >> 4;
  const int64_t slice = (int64_t)bh * cap * d;
  for (int idx = tid; idx < 32 * nkc * 4; idx += 256) {
    const int x = idx & 31, oct = idx >> 5;
    const int tn = nb * 32 + x;
    const int ts = tn < W ? 2 * tn : tn + W;
    if (tn < 2 * W)   // the last block is short when 32 does not divide 2W
      *reinterpret_cast<uint4*>(k_new + slice + k_fp_index(tn, oct * 8, nkc)) =
          *reinterpret_cast<const uint4*>(k_old + slice + k_fp_index(ts, oct * 8, nkc));
  }
  // Values: a lane of the value layout holds, of one channel, the 8 slots 4qq .. +3 and 16 + 4qq .. +3 of
  // its 32-slot tile.
  if (32 * (nb + 1) <= W) {
    // A tile of thinned rows: new slot x <- old slot 2x of the tile pair 2nb, 2nb + 1.  New element
    // i = 4 hi + 2 jh + jl of lane (qq, n) is element 4 (qq >> 1) + 2 jl of lane (2 (qq & 1) + jh, n) of old tile
    // 2nb + hi: four 8-byte reads per lane, elements 0 and 2 of each kept.
    for (int idx = tid; idx < nnt * 64; idx += 256) {
      const int lane = idx & 63, nt = idx >> 6;
      const int qq = lane >> 4, n = lane & 15;
      uint32_t w[4];
#pragma unroll
      for (int hi = 0; hi < 2; ++hi)
#pragma unroll
        for (int jh = 0; jh < 2; ++jh) {
          const int from = 16 * (2 * (qq & 1) + jh) + n;
          const uint2 u = *reinterpret_cast<const uint2*>(
              v_old + slice + (((int64_t)(2 * nb + hi) * nnt + nt) * 64 + from) * 8 + 4 * (qq >> 1));
          w[2 * hi + jh] = (u.x & 0xFFFFu) | (u.y << 16);
        }
      *reinterpret_cast<uint4*>(v_new + slice + (((int64_t)nb * nnt + nt) * 64 + lane) * 8) =
          make_uint4(w[0], w[1], w[2], w[3]);
    }
  } else if (32 * nb >= W && (W & 31) == 0 && 32 * (nb + 1) <= 2 * W) {
    // A tile of the recent window, moved by a whole number of tiles: the same lanes, 16 bytes each.
    for (int idx = tid; idx < nnt * 64; idx += 256)
      *reinterpret_cast<uint4*>(v_new + slice + ((int64_t)nb * nnt * 64 + idx) * 8) =
          *reinterpret_cast<const uint4*>(v_old + slice + ((int64_t)(nb + (W >> 5)) * nnt * 64 + idx) * 8);
  } else {
    // A tile that straddles the two kinds, or a window that is no multiple of 32: slot by slot.
    for (int idx = tid; idx < nnt * 64; idx += 256) {
      const int lane = idx & 63, nt = idx >> 6;
      const int qq = lane >> 4, n = lane & 15;
      uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tn = nb * 32 + kperm_inv(8 * qq + i);
        const int ts = tn < W ? 2 * tn : tn + W;
        const uint32_t e = tn < 2 * W ? v_old[slice + v_fp_index(ts, 16 * nt + n, nnt)] : 0u;
        w[i >> 1] |= e << (16 * (i & 1));
      }
      *reinterpret_cast<uint4*>(v_new + slice + (((int64_t)nb * nnt + nt) * 64 + lane) * 8) =
          make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
  if (bh % Hkv == 0 && tid < 32) {
    const int b = bh / Hkv, tn = nb * 32 + tid;
    const int ts = tn < W ? 2 * tn : tn + W;
    if (tn < 2 * W) pos_new[b * cap + tn] = pos_old[b * cap + ts];
  }
}

struct CompressParams {
  uint16_t *k_buf[2], *v_buf[2];   // the two fp buffers: `cur` is read, the other written
  int32_t* pos_buf[2];
  const SeqState* seq;             // device array of per-sequence state (seq_mode 2)
  int seq_mode;                    // 0: every sequence, with the counts below; 1: state in the kernel arguments
  int cur;
  uint32_t *k_codes, *v_codes;
  uint16_t *k_scale, *k_zero, *v_scale, *v_zero;
  int32_t* pos_q;
  int d, G, W, cap, qcap, n_q, Hkv;
  int nb0;                         // first 32-row tile left to the moving workgroups (W/32 when the quantizing ones move the thinned rows, else 0)
};

// One launch does both halves of the filtering branch; they read the same buffer and
// write disjoint ones.  grid (ceil(W/G) + ceil(2W/32), B*Hkv), block 256: workgroups
// x < ceil(W/G) quantize one key group each, the others move 32 kept rows each.
// Dynamic LDS: staged_bytes(d, G).
template <bool BF16, int D, int G, int BITS>
__global__ void __launch_bounds__(256) compress_kernel(const CompressParams P, const SeqInline S) {
  extern __shared__ __attribute__((aligned(16))) uint16_t sm[];  // [G][d + 4]: the staged rows
  __shared__ __attribute__((aligned(16))) uint8_t cb[QG_CODE_BYTES<D, G>];
  const int nq = (P.W + G - 1) / G;
  // (quantizing and moving workgroups alternate in launch order: started that way they overlap arithmetic
  // with memory traffic; all the quantizing ones first measured 8% slower)
  const int bx = blockIdx.x, by = blockIdx.y;
  int bh = by, cur = P.cur, n_q = P.n_q;
  if (P.seq_mode) {   // per-sequence lengths: grid row -> (i-th sequence to compress, kv head); counts before the event
    const int i = by / P.Hkv;
    const SeqArgsPtr in_args = seq_in_args(args_offset_after(sizeof(CompressParams)));   // = S
    const int b = P.seq_mode == 1 ? in_args[i].item : P.seq[i].item;
    const SeqState sq = P.seq_mode == 1 ? seq_load(in_args, b) : P.seq[b];
    (void)S;
    bh = b * P.Hkv + by % P.Hkv;
    cur = sq.cur;
    n_q = sq.n_q;
  }
  // (selects between kernel arguments, not loads that depend on `cur`)
  const uint16_t* k_old = cur ? P.k_buf[1] : P.k_buf[0];
  const uint16_t* v_old = cur ? P.v_buf[1] : P.v_buf[0];
  const int32_t* pos_old = cur ? P.pos_buf[1] : P.pos_buf[0];
  if (bx < nq) {
    const int j = bx;
    const int ng = min(G, P.W - j * G);
    const int64_t fp_slice = (int64_t)bh * P.cap * D;
    const bool keep = P.nb0 > 0;
    uint16_t* k_new = cur ? P.k_buf[0] : P.k_buf[1];
    uint16_t* v_new = cur ? P.v_buf[0] : P.v_buf[1];
    const FpSource<D, G> src{k_old + fp_slice, v_old + fp_slice, pos_old + (bh / P.Hkv) * P.cap, j, ng, P.cap,
                             keep ? k_new + fp_slice : nullptr, keep ? v_new + fp_slice : nullptr};
    if (keep && bh % P.Hkv == 0 && (int)threadIdx.x < G) {
      int32_t* pos_new = cur ? P.pos_buf[0] : P.pos_buf[1];
      const int b = bh / P.Hkv, tn = j * G + threadIdx.x;
      pos_new[b * P.cap + tn] = pos_old[b * P.cap + 2 * tn];
    }
    quantize_group<BF16, D, G, BITS>(sm, cb, src, ng, bh, n_q + j * G, P.k_codes, P.v_codes, P.k_scale, P.k_zero,
                               P.v_scale, P.v_zero, P.pos_q, P.qcap, P.Hkv);
  } else {
    compact_rows(bx - nq + P.nb0, bh, k_old, v_old, pos_old, cur ? P.k_buf[0] : P.k_buf[1],
                 cur ? P.v_buf[0] : P.v_buf[1], cur ? P.pos_buf[0] : P.pos_buf[1], P.d, P.W, P.cap, P.Hkv);
  }
}

// ---- bulk prefill ---------------------------------------------------------------
// The state Algorithm 1 (filtering as soon as the list is full) reaches after L
// appends, computed from the whole prompt in one launch.  Which position ends up in
// which slot is known in closed form (list_entry / evicted_position), so every key
// group of every event is independent: grid (E * KG + ceil(n_fp/32), B*Hkv), KG =
// ceil(W/G), block 256; workgroups x < E*KG quantize key group x % KG of event x / KG + 1
// exactly as the filtering step would have, the others place 32 fp rows each.
struct PrefillParams {
  const uint16_t *k, *v;          // [B*Hkv][L][d]
  uint16_t *k_buf[2], *v_buf[2];  // [0]: the buffer to fill (the same for every sequence), or, with
  int32_t* pos_buf[2];            // per-sequence state, the two buffers, chosen by the sequence's `cur`
  const SeqState* seq;            // device array of per-sequence state (seq_mode 2)
  int seq_mode;                   // 0: E and n_fp below hold for every sequence; 1: state in the kernel arguments
  uint32_t *k_codes, *v_codes;
  uint16_t *k_scale, *k_zero, *v_scale, *v_zero;
  int32_t* pos_q;
  int d, G, W, cap, qcap, Hkv, L, E, n_fp;
};

template <bool BF16, int D, int G, int BITS>
__global__ void __launch_bounds__(256) prefill_kernel(const PrefillParams P, const SeqInline S) {
  extern __shared__ __attribute__((aligned(16))) uint16_t sm[];
  __shared__ __attribute__((aligned(16))) uint8_t cb[QG_CODE_BYTES<D, G>];
  __shared__ int posl[128];
  const int tid = threadIdx.x, bh = blockIdx.y;
  const int per_event = (P.W + G - 1) / G;
  int E = P.E, n_fp = P.n_fp, cur = 0;
  if (P.seq_mode) {   // per-sequence prompt lengths: the grid is sized for the longest
    const SeqState sq = P.seq_mode == 1 ? seq_load(seq_in_args(args_offset_after(sizeof(PrefillParams))), bh / P.Hkv)   // = S
                                        : P.seq[bh / P.Hkv];
    (void)S;
    E = sq.n_q / (per_event * G); n_fp = sq.n_fp; cur = sq.cur;
  }
  const int nqb = E * per_event;
  const int64_t prompt = (int64_t)bh * P.L * D;   // P.L: rows per slice of the prompt tensors
  if ((int)blockIdx.x < nqb) {
    const int ev = blockIdx.x / per_event + 1, j = blockIdx.x % per_event;
    const int ng = min(G, P.W - j * G);
    if (tid < G) posl[tid] = tid < ng ? evicted_position(ev, j * G + tid, P.W) : -1;
    __syncthreads();
    const PromptSource<D, G> src{P.k + prompt, P.v + prompt, posl};
    quantize_group<BF16, D, G, BITS>(sm, cb, src, ng, bh, (ev - 1) * per_event * G + j * G, P.k_codes, P.v_codes, P.k_scale,
                               P.k_zero, P.v_scale, P.v_zero, P.pos_q, P.qcap, P.Hkv);
    return;
  }
  const int nb = blockIdx.x - nqb;
  if (32 * nb >= n_fp) return;
  uint16_t* k_fp = cur ? P.k_buf[1] : P.k_buf[0];
  uint16_t* v_fp = cur ? P.v_buf[1] : P.v_buf[0];
  int32_t* pos_fp = cur ? P.pos_buf[1] : P.pos_buf[0];
  const int nkc = P.d >> 5, nnt = P.d >> 4;
  const int64_t slice = (int64_t)bh * P.cap * P.d;
  if (tid < 32) {
    const int tn = nb * 32 + tid;
    posl[tid] = tn < n_fp ? fp_position(E, tn, P.W) : -1;
  }
  __syncthreads();
  for (int idx = tid; idx < 32 * nkc * 4; idx += 256) {
    const int x = idx & 31, oct = idx >> 5;
    const int p = posl[x];
    if (p >= 0)
      *reinterpret_cast<uint4*>(k_fp + slice + k_fp_index(nb * 32 + x, oct * 8, nkc)) =
          *reinterpret_cast<const uint4*>(P.k + prompt + (int64_t)p * P.d + oct * 8);
  }
  for (int idx = tid; idx < nnt * 64; idx += 256) {
    const int lane = idx & 63, nt = idx >> 6;
    const int qq = lane >> 4, n = lane & 15;
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p = posl[kperm_inv(8 * qq + i)];
      const uint32_t e = p >= 0 ? P.v[prompt + (int64_t)p * P.d + 16 * nt + n] : 0u;
      w[i >> 1] |= e << (16 * (i & 1));
    }
    *reinterpret_cast<uint4*>(v_fp + slice + (((int64_t)nb * nnt + nt) * 64 + lane) * 8) =
        make_uint4(w[0], w[1], w[2], w[3]);
  }
  if (bh % P.Hkv == 0 && tid < 32 && posl[tid] >= 0)
    pos_fp[(bh / P.Hkv) * P.cap + nb * 32 + tid] = posl[tid];
}

// compile-time head dimension, group size and bit width: the index arithmetic of the staging,
// encoding and packing loops is then shifts and masks
struct CompressLaunch {
  template <bool BF16, int D, int G, int BITS>
  static void go(dim3 grid, size_t lds, hipStream_t st, const CompressParams& P, const SeqInline& S) {
    hipLaunchKernelGGL((compress_kernel<BF16, D, G, BITS>), grid, dim3(256), lds, st, P, S);
  }
};
struct PrefillLaunch {
  template <bool BF16, int D, int G, int BITS>
  static void go(dim3 grid, size_t lds, hipStream_t st, const PrefillParams& P, const SeqInline& S) {
    hipLaunchKernelGGL((prefill_kernel<BF16, D, G, BITS>), grid, dim3(256), lds, st, P, S);
  }
};
template <class L, bool BF16, int D, class Params>
static void dispatch_g(const Shape& s, dim3 grid, size_t lds, hipStream_t st, const Params& P, const SeqInline& S) {
  const int key = s.G * 8 + s.bits;
  switch (key) {
    case 32 * 8 + 2: L::template go<BF16, D, 32, 2>(grid, lds, st, P, S); break;
    case 64 * 8 + 2: L::template go<BF16, D, 64, 2>(grid, lds, st, P, S); break;
    case 128 * 8 + 2: L::template go<BF16, D, 128, 2>(grid, lds, st, P, S); break;
    case 32 * 8 + 4: L::template go<BF16, D, 32, 4>(grid, lds, st, P, S); break;
    case 64 * 8 + 4: L::template go<BF16, D, 64, 4>(grid, lds, st, P, S); break;
    default: L::template go<BF16, D, 128, 4>(grid, lds, st, P, S); break;
  }
}
template <class L, bool BF16, class Params>
static void dispatch_d(const Shape& s, dim3 grid, size_t lds, hipStream_t st, const Params& P, const SeqInline& S) {
  switch (s.d) {
    case 64: dispatch_g<L, BF16, 64>(s, grid, lds, st, P, S); break;
    case 96: dispatch_g<L, BF16, 96>(s, grid, lds, st, P, S); break;
    default: dispatch_g<L, BF16, 128>(s, grid, lds, st, P, S); break;
  }
}
template <class L, class Params>
static void dispatch_dg(const Shape& s, dim3 grid, size_t lds, hipStream_t st, const Params& P, const SeqInline& S) {
  if (s.bf16) dispatch_d<L, true>(s, grid, lds, st, P, S);
  else dispatch_d<L, false>(s, grid, lds, st, P, S);
}

hipError_t launch_compress(const Shape& s, const lq_cache& c, hipStream_t st, const SeqArg* seq, int n_items) {
  CompressParams P;
  SeqInline S;
  fill_inline(&S, seq);
  for (int i = 0; i < 2; ++i) {
    P.k_buf[i] = (uint16_t*)c.k_fp[i]; P.v_buf[i] = (uint16_t*)c.v_fp[i]; P.pos_buf[i] = c.pos_fp[i];
  }
  P.seq = seq ? seq->dev : nullptr; P.seq_mode = seq_mode(seq); P.cur = c.cur;
  P.k_codes = c.k_codes; P.v_codes = c.v_codes;
  P.k_scale = (uint16_t*)c.k_scale; P.k_zero = (uint16_t*)c.k_zero;
  P.v_scale = (uint16_t*)c.v_scale; P.v_zero = (uint16_t*)c.v_zero;
  P.pos_q = c.pos_q;
  P.d = s.d; P.G = s.G; P.W = s.W; P.cap = s.cap; P.qcap = s.qcap; P.n_q = c.n_q; P.Hkv = s.Hkv;
  const size_t lds = (size_t)staged_bytes(s.d, s.G);
  // With whole key groups (G | W; then 32 | W too) and d a multiple of 64 the quantizing workgroups can also move the
  // thinned rows - they read those lines anyway - and the moving ones start at the recent window.
  // That pays when the launch is bound by memory traffic (every line fetched once instead of twice: 41.8 -> 36.3 us
  // at 512 slices); a launch of a few hundred workgroups is bound by the time one quantizing workgroup takes, which
  // the extra stores lengthen (64 slices: 9.9 -> 10.4 .. 11.5 us), so small launches keep the separate workgroups.
  const int slices = (seq ? n_items : s.B) * s.Hkv;
  const int tiles = (2 * s.W + 31) / 32;
  const bool fuse = s.W % s.G == 0 && s.d % 64 == 0 && (int64_t)slices * (s.Wq / s.G + tiles) >= 2048;
  P.nb0 = fuse ? s.W / 32 : 0;
  dim3 grid(s.Wq / s.G + tiles - P.nb0, slices);
  dispatch_dg<CompressLaunch>(s, grid, lds, st, P, S);
  return launch_status(__func__);
}

hipError_t launch_prefill(const Shape& s, const lq_cache& c, const void* k, const void* v, int L, int E,
                          int n_fp, hipStream_t st, const SeqArg* seq) {
  PrefillParams P;
  SeqInline S;
  fill_inline(&S, seq);
  P.k = (const uint16_t*)k; P.v = (const uint16_t*)v;
  const int first = seq ? 0 : c.cur;
  for (int i = 0; i < 2; ++i) {
    P.k_buf[i] = (uint16_t*)c.k_fp[first ^ i]; P.v_buf[i] = (uint16_t*)c.v_fp[first ^ i];
    P.pos_buf[i] = c.pos_fp[first ^ i];
  }
  P.seq = seq ? seq->dev : nullptr; P.seq_mode = seq_mode(seq);
  P.k_codes = c.k_codes; P.v_codes = c.v_codes;
  P.k_scale = (uint16_t*)c.k_scale; P.k_zero = (uint16_t*)c.k_zero;
  P.v_scale = (uint16_t*)c.v_scale; P.v_zero = (uint16_t*)c.v_zero;
  P.pos_q = c.pos_q;
  P.d = s.d; P.G = s.G; P.W = s.W; P.cap = s.cap; P.qcap = s.qcap; P.Hkv = s.Hkv;
  P.L = L; P.E = E; P.n_fp = n_fp;
  const size_t lds = (size_t)staged_bytes(s.d, s.G);
  dim3 grid(E * (s.Wq / s.G) + (n_fp + 31) / 32, s.B * s.Hkv);
  dispatch_dg<PrefillLaunch>(s, grid, lds, st, P, S);
  return launch_status(__func__);
}

}  // namespace lq
