// Device-side helpers shared by the gfx950 kernels: element type conversion and
// the physical index functions documented in include/logquant.h.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace lq {

// ---- cache element type T, handled as raw 16-bit patterns --------------------
template <bool BF16>
__device__ __forceinline__ float t2f(uint16_t u) {
  if constexpr (BF16) {
    return __uint_as_float(static_cast<uint32_t>(u) << 16);
  } else {
    return __half2float(__ushort_as_half(u));
  }
}

// fp32 -> T, round to nearest even (finite inputs).
template <bool BF16>
__device__ __forceinline__ uint16_t f2t(float x) {
  if constexpr (BF16) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
  } else {
    return __half_as_ushort(__float2half_rn(x));
  }
}

// ---- layouts (one (b,h) slice; offsets relative to the slice) ----------------
__host__ __device__ __forceinline__ int kperm(int x) {
  return 8 * ((x & 15) >> 2) + 4 * (x >> 4) + (x & 3);
}
__host__ __device__ __forceinline__ int kperm_inv(int k) {   // k = 8a + 4b + c -> 16b + 4a + c
  return 16 * ((k >> 2) & 1) + 4 * (k >> 3) + (k & 3);
}
// element index of fp key (slot t, channel c); NKC = d/32
__host__ __device__ __forceinline__ int64_t k_fp_index(int t, int c, int nkc) {
  return ((((int64_t)(t >> 4) * nkc + (c >> 5)) * 64 + 16 * ((c & 31) >> 3) + (t & 15)) << 3) + (c & 7);
}
// element index of fp value (slot t, channel c); NNT = d/16
__host__ __device__ __forceinline__ int64_t v_fp_index(int t, int c, int nnt) {
  const int k = kperm(t & 31);
  return ((((int64_t)(t >> 5) * nnt + (c >> 4)) * 64 + 16 * (k >> 3) + (c & 15)) << 3) + (k & 7);
}
// index of the v_scale / v_zero entry of (slot t, channel group gc)
__host__ __device__ __forceinline__ int64_t v_meta_index(int t, int gc, int ngc) {
  return ((int64_t)(t >> 5) * ngc + gc) * 32 + kperm(t & 31);
}

// ---- Algorithm 1 in closed form ------------------------------------------------
// Filtering events are numbered e = 1, 2, ..; event e happens when (e + 2) * W tokens
// have arrived.  Right after event e the list holds 2W entries: the newest window
// [(e+1)W, (e+2)W) in its upper half, and in its lower half entry i is what entry 2i
// was after event e - 1 (the even logical indices survive).  With the convention
// that "after event 0" entry i is position i:
//   entry(e, i) = e*W + i                 for W <= i < 2W, e >= 1
//               = entry(e - 1, 2i)        for i < W, e >= 1
//               = i                       for e = 0
__host__ __device__ __forceinline__ int list_entry(int e, int i, int W) {
  if (i == 0) return 0;   // position 0 never leaves
  while (e >= 1 && i < W) { i <<= 1; --e; }
  return e == 0 ? i : e * W + i;
}
// position of the i-th row (0 <= i < W) that leaves the list at event e >= 1: odd
// logical index 2i + 1 of the list as it stood after event e - 1
__host__ __device__ __forceinline__ int evicted_position(int e, int i, int W) {
  return list_entry(e - 1, 2 * i + 1, W);
}
// position held by logical fp slot i after L tokens (E events happened)
__host__ __device__ __forceinline__ int fp_position(int E, int i, int W) {
  if (E == 0) return i;
  return i < 2 * W ? list_entry(E, i, W) : E * W + i;
}

}  // namespace lq
