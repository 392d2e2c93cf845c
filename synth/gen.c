/*
 * Seeded synthetic-input generator (weights, prompts) shared by the CPU oracle's
 * tests and the HIP path's tests/bench.  It holds NONE of the method's arithmetic:
 * it only turns (seed, tensor id, element index) into a number.
 *
 * Element rule (integer-exact, so every caller gets identical bits):
 *   h   = mix64(mix64(seed ^ (tid+1)*0x9E3779B97F4A7C15) + index)
 *   z   = qtable[h >> 48]            qtable[j] = Phi^-1((j+0.5)/65536), supplied by the caller
 *   val = (float)(z * std + mean)    (one fp64 multiply-add, one rounding to fp32)
 * bf16 outputs round that fp32 value to nearest-even.
 *
 * Build: gcc -O3 -fopenmp -shared -fPIC gen.c -o libsynth.so
 */
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

static inline uint64_t tensor_base(uint64_t seed, uint64_t tid) {
  return mix64(seed ^ ((tid + 1) * 0x9E3779B97F4A7C15ull));
}

static inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static inline float gen_one(const double *qtable, uint64_t base, uint64_t idx, double std, double mean) {
  uint64_t h = mix64(base + idx);
  return (float)(qtable[h >> 48] * std + mean);
}

/* out[i] = element (start+i) of tensor tid, as fp32 */
void synth_normal_f32(const double *qtable, uint64_t seed, uint64_t tid, uint64_t start, uint64_t count,
                      double std, double mean, float *out) {
  uint64_t base = tensor_base(seed, tid);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i) out[i] = gen_one(qtable, base, start + (uint64_t)i, std, mean);
}

/* same element, rounded to bf16 (raw 16-bit pattern) */
void synth_normal_bf16(const double *qtable, uint64_t seed, uint64_t tid, uint64_t start, uint64_t count,
                       double std, double mean, uint16_t *out) {
  uint64_t base = tensor_base(seed, tid);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i)
    out[i] = f32_to_bf16_rne(gen_one(qtable, base, start + (uint64_t)i, std, mean));
}

/* same element, rounded to bf16 and widened back to fp32 (what a bf16 weight *means*) */
void synth_normal_bf16_as_f32(const double *qtable, uint64_t seed, uint64_t tid, uint64_t start,
                              uint64_t count, double std, double mean, float *out) {
  uint64_t base = tensor_base(seed, tid);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i) {
    uint32_t u = (uint32_t)f32_to_bf16_rne(gen_one(qtable, base, start + (uint64_t)i, std, mean)) << 16;
    float f;
    memcpy(&f, &u, 4);
    out[i] = f;
  }
}

/* token ids uniform on [0, vocab) */
void synth_tokens(uint64_t seed, uint64_t tid, uint64_t start, uint64_t count, uint32_t vocab, int32_t *out) {
  uint64_t base = tensor_base(seed, tid);
  for (uint64_t i = 0; i < count; ++i) out[i] = (int32_t)((mix64(base + start + i) >> 16) % vocab);
}
