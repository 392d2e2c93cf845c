// Shared device/host helpers for libeagle (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;   // raw bfloat16 bits
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define EAGLE_MAX_NODES 64
#define EAGLE_MAX_DEPTH 15
#define EAGLE_MAX_CHILD 8
#define EAGLE_PREFILL_CHUNK 128

// Per-work-group time stamps (100 MHz wall clock) exist only in a library built with -DEAGLE_TRACE (a profiling build);
// in the product build the macros expand to nothing and no kernel carries a trace store.
#ifdef EAGLE_TRACE
#define TRACE_PTR(expr) (expr)
#define TRACE_STAMP(tr, i) do { if (tr) (tr)[i] = wall_clock64(); } while (0)
#define TRACE_STAMP_AFTER(tr, i, value_used) do { if (tr) (tr)[i] = wall_clock64() + ((value_used) == 123.456f ? 1 : 0); } while (0)
#else
#define TRACE_PTR(expr) nullptr
#define TRACE_STAMP(tr, i) do { (void)(tr); } while (0)
#define TRACE_STAMP_AFTER(tr, i, value_used) do { (void)(tr); } while (0)
#endif

// ---------------------------------------------------------------- bf16
__host__ __device__ inline bf16_t f32_to_bf16(float f) {   // round to nearest even
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__host__ __device__ inline float bf16_to_f32(bf16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }

// x == p0 + p1 (+ p2) with every piece a bf16: the planes the MFMA GEMM multiplies.
__device__ inline void split_bf16(float x, bf16_t* p, int nplanes) {
  float r = x;
  for (int i = 0; i < nplanes; ++i) {
    bf16_t b = f32_to_bf16(r);
    p[i] = b;
    r -= bf16_to_f32(b);
  }
}

// ---------------------------------------------------------------- layouts
// Packed weight matrix: 32-row x 16-k tiles of 1 KiB, tile (rb, ks) at ((rb*KS + ks) * 512) elements; inside a
// tile lane l (0..63) owns 8 consecutive elements: row rb*32 + l%32, k = ks*16 + (l/32)*8 + t.  One wave reads
// a tile with a single fully coalesced 16-byte-per-lane load and gets the MFMA 32x32x16 A operand directly.
__host__ __device__ inline size_t wpack_index(int n, int k, int KS) {
  return ((size_t)(n >> 5) * KS + (k >> 4)) * 512 + (size_t)((n & 31) + 32 * ((k & 15) >> 3)) * 8 + (k & 7);
}
// Activation matrix in "fragment" layout (XF): same tiling for X[m][k], tile (plane, mt, ks) at
// (((plane*MT + mt)*KS + ks) * 512); it is the MFMA B operand as it sits in memory.
__host__ __device__ inline size_t xf_index(int m, int k, int plane, int MT, int KS) {
  return (((size_t)plane * MT + (m >> 5)) * KS + (k >> 4)) * 512 + (size_t)((m & 31) + 32 * ((k & 15) >> 3)) * 8 + (k & 7);
}
// Split-K partial sums of the general path: PT[s][m][n], n fastest (Mpad = 32*MT rows of Npad floats per split).

// ---------------------------------------------------------------- counter-based uniforms (24-bit)
#define EAGLE_GOLDEN 0x9E3779B97F4A7C15ull
enum { PURPOSE_ACCEPT = 1, PURPOSE_FINAL = 2, PURPOSE_GUMBEL = 3, PURPOSE_HINT = 4, PURPOSE_NOISE = 5 };
__host__ __device__ inline uint64_t mix64(uint64_t x) {
  x += EAGLE_GOLDEN;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
__host__ __device__ inline uint64_t rng_prefix(uint64_t seed, uint32_t purpose, uint64_t step) {
  return mix64(mix64(seed ^ ((uint64_t)purpose * EAGLE_GOLDEN)) + step);
}
__host__ __device__ inline uint32_t rng_u24(uint64_t prefix, uint32_t seq, uint32_t node, uint32_t idx) {
  return (uint32_t)(mix64(prefix ^ (((uint64_t)seq << 48) | ((uint64_t)node << 32) | (uint64_t)idx)) >> 40);
}
