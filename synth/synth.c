/*
 * Seeded synthetic input generator (weights, activations, token ids).
 *
 * Holds none of the decoder's arithmetic: it only draws random numbers and
 * stores them.  Both the CPU oracle's tests and the GPU path's tests/bench take
 * their inputs from here, so the two sides see identical bytes.
 *
 * Counter based and order free: element i of tensor t under seed s is a pure
 * function of (s, t, i), so threads may fill any range in any order.
 *
 *   key    = s XOR (t * 2^40 + i)
 *   h      = splitmix64 finaliser of key        (Steele/Lea/Flood mixing constants)
 *   u1, u2 = ((high 32 bits of h) + 0.5) / 2^32, ((low 32 bits of h) + 0.5) / 2^32
 *   normal = sqrt(-2 ln u1) * cos(2 pi u2)      (Box-Muller, fp64)
 *
 * The workload these stand in for is the Qwen3 checkpoints and prompts of the
 * paper's evaluation (Section 4, experimental setup), which are not available
 * here; shapes follow the public Qwen3 sizes.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint64_t draw(uint64_t seed, uint64_t tensor, uint64_t i) {
  return mix64(seed ^ ((tensor << 40) + i));
}

static inline double std_normal(uint64_t h) {
  const double u1 = ((double)(uint32_t)(h >> 32) + 0.5) * (1.0 / 4294967296.0);
  const double u2 = ((double)(uint32_t)(h & 0xffffffffu) + 0.5) * (1.0 / 4294967296.0);
  return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
}

/* fp32 -> bf16 storage format, round to nearest, ties to even. Inputs here are
 * finite normals, so no NaN handling is needed. */
static inline uint16_t store_bf16(float f) {
  uint32_t b;
  memcpy(&b, &f, 4);
  b += 0x7fffu + ((b >> 16) & 1u);
  return (uint16_t)(b >> 16);
}

/* fp32 -> IEEE binary16 storage format, round to nearest, ties to even, for finite
 * inputs below the binary16 overflow threshold (weights are ~N(0, 0.02^2)). */
static inline uint16_t store_f16(float f) {
  uint32_t b;
  memcpy(&b, &f, 4);
  const uint16_t sgn = (uint16_t)((b >> 16) & 0x8000u);
  const uint32_t a = b & 0x7fffffffu;
  if (a >= 0x477ff000u) return sgn | 0x7c00u;          /* >= 65520: rounds to infinity */
  if (a < 0x38800000u) {                               /* below 2^-14: multiples of 2^-24 */
    float av;
    memcpy(&av, &a, 4);
    return sgn | (uint16_t)lrintf(av * 16777216.0f);   /* exact scaling, nearest-even rounding */
  }
  uint32_t r = a + 0xfffu + ((a >> 13) & 1u);           /* drop 13 fraction bits, nearest even */
  return sgn | (uint16_t)((r - 0x38000000u) >> 13);
}

void synth_normal_f32(uint64_t seed, uint64_t tensor, uint64_t first, uint64_t n,
                      double scale, float *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = (float)(scale * std_normal(draw(seed, tensor, first + (uint64_t)i)));
}

void synth_normal_bf16(uint64_t seed, uint64_t tensor, uint64_t first, uint64_t n,
                       double scale, uint16_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = store_bf16((float)(scale * std_normal(draw(seed, tensor, first + (uint64_t)i))));
}

void synth_normal_f16(uint64_t seed, uint64_t tensor, uint64_t first, uint64_t n,
                      double scale, uint16_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = store_f16((float)(scale * std_normal(draw(seed, tensor, first + (uint64_t)i))));
}

/* Weight-only 8-bit storage of a [rows, cols] matrix drawn as N(0, scale^2): per output row one
 * scale s (a bf16-representable fp32: the row's largest magnitude / 127 rounded up to 8 significant
 * bits, 1.0 for an all-zero row) and cols signed bytes q = nearest integer of w / s (ties to even),
 * so that the stored weight is exactly s * q with |q| <= 127.  A storage format of the inputs, like
 * the 16-bit ones above; the forward pass that uses s * q is not here. */
void synth_normal_w8(uint64_t seed, uint64_t tensor, uint64_t rows, uint64_t cols, double scale,
                     int8_t *q, float *row_scale) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < (int64_t)rows; ++r) {
    double amax = 0.0;
    for (uint64_t c = 0; c < cols; ++c) {
      const double w = scale * std_normal(draw(seed, tensor, (uint64_t)r * cols + c));
      if (fabs(w) > amax) amax = fabs(w);
    }
    float s = 1.0f;
    if (amax > 0.0) {
      uint32_t b;
      s = (float)(amax / 127.0);
      memcpy(&b, &s, 4);
      b = (b + 0xffffu) & 0xffff0000u;   /* up to the next bf16-representable value */
      memcpy(&s, &b, 4);
    }
    row_scale[r] = s;
    for (uint64_t c = 0; c < cols; ++c) {
      const double w = scale * std_normal(draw(seed, tensor, (uint64_t)r * cols + c));
      double v = nearbyint(w / (double)s);
      if (v > 127.0) v = 127.0;
      if (v < -127.0) v = -127.0;
      q[(uint64_t)r * cols + c] = (int8_t)v;
    }
  }
}

/* Uniform integers in [0, bound): floor(u * bound) with u the high 32 bits / 2^32. */
void synth_uniform_i32(uint64_t seed, uint64_t tensor, uint64_t first, uint64_t n,
                       uint32_t bound, int32_t *out) {
  for (uint64_t i = 0; i < n; ++i) {
    const uint64_t hi = draw(seed, tensor, first + i) >> 32;
    out[i] = (int32_t)((hi * (uint64_t)bound) >> 32);
  }
}

uint64_t synth_raw(uint64_t seed, uint64_t tensor, uint64_t i) { return draw(seed, tensor, i); }
