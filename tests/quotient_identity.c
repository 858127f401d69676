/* Exhaustive CPU check of the arithmetic identity that the GPU quantizer relies on to produce
 * bit-exact codes without a division per element (it is a statement about IEEE binary32, not about
 * any implementation):
 *
 *   scale = fl(amax / QMAX), amax any bf16 value with scale in [2^-60, 2^60], QMAX in {7, 127};
 *   (1) scale == fma(fma(-QMAX, q, amax), c, q) with c = fl(1/QMAX), q = fl(amax * c);
 *   (2) for a reciprocal estimate y0 within one ulp of fl(1/scale), fma(fma(-scale, y0, 1), y0, y0)
 *       equals fl(1/scale);
 *   (3) with inv = fl(1/scale): q0 = fl(x*inv), r = fma(-scale, q0, x), y = fma(r, inv, q0) gives
 *       rint(y) == rint(fl(x / scale)) for every bf16 x with |x| <= amax, either sign.
 * Prints "pairs bad1 bad2 bad3" per QMAX; exit status 0 iff nothing is bad. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

static float bf16(uint32_t bits) { uint32_t u = bits << 16; float f; memcpy(&f, &u, 4); return f; }
static float step(float x, int dir) { uint32_t u; memcpy(&u, &x, 4); u += (uint32_t)dir; float f; memcpy(&f, &u, 4); return f; }

int main(void) {
  const int qmaxs[2] = {7, 127};
  long total_bad = 0;
  for (int qi = 0; qi < 2; ++qi) {
    const float Q = (float)qmaxs[qi], c = 1.0f / Q;
    long bad1 = 0, bad2 = 0, bad3 = 0, pairs = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : bad1, bad2, bad3, pairs)
    for (uint32_t ab = 1; ab < 0x7F80; ++ab) {
      const float amax = bf16(ab);
      const float scale = amax / Q;
      const float q = amax * c;
      if (fmaf(fmaf(-Q, q, amax), c, q) != scale) bad1++;
      if (!(scale >= 0x1p-60f && scale <= 0x1p60f)) continue;
      const float inv = 1.0f / scale;
      for (int dir = -1; dir <= 1; ++dir) {
        const float y0 = step(inv, dir);
        if (fmaf(fmaf(-scale, y0, 1.0f), y0, y0) != inv) bad2++;
      }
      for (uint32_t xb = 0; xb <= ab; ++xb)
        for (int sign = 0; sign < 2; ++sign) {
          const float x = sign ? -bf16(xb) : bf16(xb);
          const float q0 = x * inv;
          const float r = fmaf(-scale, q0, x);
          const float y = fmaf(r, inv, q0);
          pairs++;
          if (rintf(y) != rintf(x / scale)) bad3++;
        }
    }
    printf("%d %ld %ld %ld %ld\n", qmaxs[qi], pairs, bad1, bad2, bad3);
    total_bad += bad1 + bad2 + bad3;
  }
  return total_bad ? 1 : 0;
}
