/* Host check of an arithmetic identity the quantizing kernels rely on: for STEPS = 3 and 15,
 * with y = fp32(1/STEPS), q0 = fp32(a*y), r = a - STEPS*q0 (one fused multiply-add, exact) the
 * value fp32(q0 + r*y) is the correctly rounded quotient a / STEPS for finite a >= 0.  The
 * reference is the fp64 quotient rounded to fp32 (53 >= 2*24 + 2: no double rounding).
 * usage: div_three_ops <stride>   (1: every non-negative finite fp32 value) */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float quotient(float a, float steps, float y) {
  const float q0 = a * y;
  const float r = fmaf(-steps, q0, a);
  return fmaf(r, y, q0);
}

int main(int argc, char** argv) {
  const uint32_t stride = argc > 1 ? (uint32_t)strtoul(argv[1], 0, 10) : 1u;
  const float steps[2] = {3.f, 15.f};
  long checked = 0, bad = 0;
  for (int s = 0; s < 2; ++s) {
    const float y = 1.0f / steps[s];
    for (uint64_t u = 0; u < 0x7F800000u; u += stride) {
      const uint32_t bits = (uint32_t)u;
      float a;
      memcpy(&a, &bits, 4);
      const float want = (float)((double)a / (double)steps[s]);
      const float got = quotient(a, steps[s], y);
      ++checked;
      if (memcmp(&want, &got, 4)) {
        if (bad < 5) printf("steps %g a %a want %a got %a\n", steps[s], a, want, got);
        ++bad;
      }
    }
  }
  printf("checked %ld mismatches %ld\n", checked, bad);
  return bad != 0;
}
