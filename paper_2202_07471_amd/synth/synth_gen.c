/* Seeded synthetic weight generator (host side).
 *
 * Input plumbing only: it holds none of the quantization method's arithmetic
 * and is the one module both the GPU tests/benchmark and the CPU reference
 * checker draw their inputs from.  Every element is a pure function of
 * (seed, stream, element index), so tensors are reproducible element by
 * element and generation parallelises freely.
 *
 * Random bits: Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11), counter = (index lo, index hi, stream,
 * draw), key = (seed lo, seed hi).  Uniforms are (r + 0.5) / 2^32 in (0, 1);
 * normals by Box-Muller in double precision; the value is rounded to float once.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC synth_gen.c -lm
 */
#include <math.h>
#include <stdint.h>

static void philox4x32_10(uint32_t c[4], uint32_t k0, uint32_t k1) {
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

static void draw4(uint64_t seed, uint32_t stream, uint64_t idx, uint32_t draw, uint32_t out[4]) {
  out[0] = (uint32_t)idx; out[1] = (uint32_t)(idx >> 32); out[2] = stream; out[3] = draw;
  philox4x32_10(out, (uint32_t)seed, (uint32_t)(seed >> 32));
}

static double unit(uint32_t r) { return ((double)r + 0.5) * (1.0 / 4294967296.0); }

/* Two independent standard normals from two words. */
static void box_muller(uint32_t a, uint32_t b, double* z0, double* z1) {
  const double rad = sqrt(-2.0 * log(unit(a)));
  const double ang = 6.283185307179586476925286766559 * unit(b);
  *z0 = rad * cos(ang);
  *z1 = rad * sin(ang);
}

/* out[i] ~ N(0, sigma^2) */
void synth_fill_normal(float* out, int64_t n, uint64_t seed, uint32_t stream, double sigma) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t r[4]; double z0, z1;
    draw4(seed, stream, (uint64_t)i, 0u, r);
    box_muller(r[0], r[1], &z0, &z1);
    out[i] = (float)(sigma * z0);
  }
}

/* out[i] ~ sigma * Student-t(nu = 3) = sigma * Z / sqrt((Y1^2 + Y2^2 + Y3^2) / 3) */
void synth_fill_student_t3(float* out, int64_t n, uint64_t seed, uint32_t stream, double sigma) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t r[4]; double z, y1, y2, y3;
    draw4(seed, stream, (uint64_t)i, 0u, r);
    box_muller(r[0], r[1], &z, &y1);
    box_muller(r[2], r[3], &y2, &y3);
    out[i] = (float)(sigma * z / sqrt((y1 * y1 + y2 * y2 + y3 * y3) / 3.0));
  }
}

/* out[i] ~ N(0, sigma^2), except with probability `prob` Laplace(0, b) (inverse CDF). */
void synth_fill_normal_laplace(float* out, int64_t n, uint64_t seed, uint32_t stream,
                               double sigma, double prob, double b) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t r[4]; double z0, z1;
    draw4(seed, stream, (uint64_t)i, 0u, r);
    box_muller(r[0], r[1], &z0, &z1);
    double v = sigma * z0;
    if (unit(r[2]) < prob) {
      const double u = unit(r[3]) - 0.5;
      v = (u < 0 ? b : -b) * log(1.0 - 2.0 * fabs(u));
    }
    out[i] = (float)v;
  }
}

/* One fair coin per (seed, stream): 0 or 1. */
int32_t synth_coin(uint64_t seed, uint32_t stream) {
  uint32_t r[4];
  draw4(seed, stream, 0xFFFFFFFFFFFFFFFFull, 1u, r);
  return (int32_t)(r[0] >> 31);
}
