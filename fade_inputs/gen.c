/*
 * gen.c — seeded synthetic byte-stream generators shared by the tests, the bench and the oracle timing.
 * Input data only: nothing of the compression method lives here.
 *
 * PRNG: xoshiro256** seeded through splitmix64. Every generator is a pure function of (seed, n).
 * The four sources stand in for the kinds of data the paper evaluates on (text, genome, floating-point
 * scientific data, heterogeneous mix); none of those datasets is reproduced.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint64_t s[4]; } rng_t;

static uint64_t splitmix64(uint64_t *x) {
  uint64_t z = (*x += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}
static void rng_seed(rng_t *r, uint64_t seed) {
  for (int i = 0; i < 4; ++i) r->s[i] = splitmix64(&seed);
}
static inline uint64_t rotl(uint64_t x, int k) { return (x << k) | (x >> (64 - k)); }
static uint64_t rng_next(rng_t *r) {
  uint64_t *s = r->s;
  const uint64_t result = rotl(s[1] * 5, 7) * 9, t = s[1] << 17;
  s[2] ^= s[0]; s[3] ^= s[1]; s[1] ^= s[2]; s[0] ^= s[3]; s[2] ^= t; s[3] = rotl(s[3], 45);
  return result;
}
static double rng_unit(rng_t *r) { return (double)(rng_next(r) >> 11) * (1.0 / 9007199254740992.0); } /* [0,1) */
static double rng_unit_open(rng_t *r) { return ((double)(rng_next(r) >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
static double rng_normal(rng_t *r) { /* Box-Muller, one value per call */
  const double u1 = rng_unit_open(r), u2 = rng_unit(r);
  return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}
/* Gamma(shape, 1): Marsaglia-Tsang for shape >= 1, boosted by U^(1/shape) below 1. */
static double rng_gamma(rng_t *r, double shape) {
  if (shape < 1.0) return rng_gamma(r, shape + 1.0) * pow(rng_unit_open(r), 1.0 / shape);
  const double d = shape - 1.0 / 3.0, c = 1.0 / sqrt(9.0 * d);
  for (;;) {
    double x, v;
    do { x = rng_normal(r); v = 1.0 + c * x; } while (v <= 0.0);
    v = v * v * v;
    const double u = rng_unit_open(r);
    if (log(u) < 0.5 * x * x + d - d * v + d * log(v)) return d * v;
  }
}
/* One Dirichlet(alpha,...,alpha) row as a 32-bit cumulative table: cum[i] = floor(2^32 * P(X <= i)). */
static void dirichlet_cum(rng_t *r, double alpha, int k, uint32_t *cum) {
  double g[256], s = 0.0;
  for (int i = 0; i < k; ++i) { g[i] = rng_gamma(r, alpha) + 1e-300; s += g[i]; }
  double acc = 0.0;
  for (int i = 0; i < k; ++i) {
    acc += g[i] / s;
    double v = acc * 4294967296.0;
    cum[i] = v >= 4294967295.0 ? 0xffffffffu : (uint32_t)v;
  }
  cum[k - 1] = 0xffffffffu;
}
static int sample_cum(const uint32_t *cum, int k, uint32_t u) {
  int lo = 0, hi = k - 1;
  while (lo < hi) { int mid = (lo + hi) >> 1; if (u <= cum[mid]) hi = mid; else lo = mid + 1; }
  return lo;
}

/* Source 1: order-2 Markov chain over 256 symbols, each of the 65,536 transition rows ~ Dirichlet(0.1). */
int fade_gen_markov2(uint64_t seed, size_t n, uint8_t *out) {
  rng_t r; rng_seed(&r, seed);
  uint32_t *rows = (uint32_t *)malloc((size_t)65536 * 256 * sizeof(uint32_t));
  if (!rows) return -1;
  for (int c = 0; c < 65536; ++c) dirichlet_cum(&r, 0.1, 256, rows + (size_t)c * 256);
  uint32_t a = (uint32_t)(rng_next(&r) >> 56), b = (uint32_t)(rng_next(&r) >> 56);
  for (size_t i = 0; i < n; ++i) {
    if (i == 0) { out[i] = (uint8_t)a; continue; }
    if (i == 1) { out[i] = (uint8_t)b; continue; }
    const int s = sample_cum(rows + ((size_t)(a << 8 | b)) * 256, 256, (uint32_t)(rng_next(&r) >> 32));
    out[i] = (uint8_t)s; a = b; b = (uint32_t)s;
  }
  free(rows);
  return 0;
}

/* Source 2: text-like order-3 source whose marginal is Zipf(s = 1.1) over a seeded permutation of the
 * byte values. The 2^24 contexts are procedural: a context hashes to four candidate successors (each a
 * Zipf draw); the next symbol is candidate j with probability 1/2, 1/4, 1/8, 1/16, else a fresh Zipf draw. */
int fade_gen_text(uint64_t seed, size_t n, uint8_t *out) {
  rng_t r; rng_seed(&r, seed);
  uint32_t zipf[256]; double w[256], s = 0.0, acc = 0.0;
  for (int i = 0; i < 256; ++i) { w[i] = pow((double)(i + 1), -1.1); s += w[i]; }
  for (int i = 0; i < 256; ++i) { acc += w[i] / s; double v = acc * 4294967296.0; zipf[i] = v >= 4294967295.0 ? 0xffffffffu : (uint32_t)v; }
  zipf[255] = 0xffffffffu;
  uint8_t perm[256];
  for (int i = 0; i < 256; ++i) perm[i] = (uint8_t)i;
  for (int i = 255; i > 0; --i) { int j = (int)(rng_next(&r) % (uint64_t)(i + 1)); uint8_t t = perm[i]; perm[i] = perm[j]; perm[j] = t; }
  uint32_t ctx = 0;
  for (size_t i = 0; i < n; ++i) {
    uint64_t h = seed ^ (0x51ed270b7a1f3c95ull * (uint64_t)(ctx + 1));
    uint8_t cand[4];
    for (int j = 0; j < 4; ++j) cand[j] = perm[sample_cum(zipf, 256, (uint32_t)(splitmix64(&h) >> 32))];
    const uint32_t u = (uint32_t)(rng_next(&r) >> 60); /* 0..15 */
    uint8_t x;
    if (u < 8) x = cand[0]; else if (u < 12) x = cand[1]; else if (u < 14) x = cand[2]; else if (u < 15) x = cand[3];
    else x = perm[sample_cum(zipf, 256, (uint32_t)(rng_next(&r) >> 32))];
    out[i] = x;
    ctx = ((ctx << 8) | x) & 0xffffffu;
  }
  return 0;
}

/* Source 3: genome-like: order-8 chain on {A,C,G,T} (65,536 rows ~ Dirichlet(0.5)); at every output
 * position 'N' with probability 0.01 and newline with probability 0.001 are inserted instead. */
int fade_gen_genome(uint64_t seed, size_t n, uint8_t *out) {
  static const uint8_t sym[4] = {'A', 'C', 'G', 'T'};
  rng_t r; rng_seed(&r, seed);
  uint32_t *rows = (uint32_t *)malloc((size_t)65536 * 4 * sizeof(uint32_t));
  if (!rows) return -1;
  for (int c = 0; c < 65536; ++c) dirichlet_cum(&r, 0.5, 4, rows + (size_t)c * 4);
  uint32_t ctx = (uint32_t)(rng_next(&r) >> 48);
  for (size_t i = 0; i < n; ++i) {
    const double u = rng_unit(&r);
    if (u < 0.01) { out[i] = 'N'; continue; }
    if (u < 0.011) { out[i] = '\n'; continue; }
    const int s = sample_cum(rows + (size_t)ctx * 4, 4, (uint32_t)(rng_next(&r) >> 32));
    out[i] = sym[s];
    ctx = ((ctx << 2) | (uint32_t)s) & 0xffffu;
  }
  free(rows);
  return 0;
}

/* Source 4: float32 AR(1) series x_t = 0.99 x_{t-1} + N(0,1), serialised little-endian; n is rounded
 * down to a multiple of 4 and the tail (if any) is zero. */
int fade_gen_float_ar1(uint64_t seed, size_t n, uint8_t *out) {
  rng_t r; rng_seed(&r, seed);
  float x = 0.0f;
  size_t i = 0;
  for (; i + 4 <= n; i += 4) {
    x = 0.99f * x + (float)rng_normal(&r);
    uint32_t u; memcpy(&u, &x, 4);
    out[i] = (uint8_t)u; out[i + 1] = (uint8_t)(u >> 8); out[i + 2] = (uint8_t)(u >> 16); out[i + 3] = (uint8_t)(u >> 24);
  }
  for (; i < n; ++i) out[i] = 0;
  return 0;
}

/* Gaussian fill for weight blobs: out[i] = mean + std * N(0,1), in fp32. */
int fade_gen_normal_f32(uint64_t seed, size_t n, float mean, float std, float *out) {
  rng_t r; rng_seed(&r, seed);
  for (size_t i = 0; i < n; ++i) out[i] = mean + std * (float)rng_normal(&r);
  return 0;
}
