/* Checks on the CPU that q1 = fma(fma(-d, x*c, x), c, x*c) with c = RN(1/d) is the correctly rounded x/d for d = 2^b - 1,
 * b in {2,3,4,6,8} (the quantizer's scale factor, App. B "Preliminaries"), over non-negative finite binary32 x.
 * usage: division_check STRIDE   -- every STRIDE-th bit pattern (1 = all of them, about two minutes on 8 cores).
 * Prints the number of mismatches per divisor; exit status 1 if any. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
int main(int argc, char** argv) {
  const uint32_t stride = argc > 1 ? (uint32_t)strtoul(argv[1], NULL, 10) : 64u;
  const float ds[] = {3.f, 7.f, 15.f, 63.f, 255.f};
  int fail = 0;
  for (int k = 0; k < 5; ++k) {
    const float d = ds[k], c = 1.0f / d;
    unsigned long long bad = 0;
    for (uint32_t u = 0; u < 0x7F800000u; u += stride) {
      float x;
      memcpy(&x, &u, 4);
      const float q0 = x * c;
      const float r = fmaf(-d, q0, x);
      const float q1 = fmaf(r, c, q0);
      if (q1 != x / d) ++bad;
    }
    printf("d=%g mismatches=%llu\n", d, bad);
    if (bad) fail = 1;
  }
  return fail;
}
