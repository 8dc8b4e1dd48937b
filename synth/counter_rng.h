/* Seeded synthetic-input generator: integer-only counter hash.
 *
 * This header holds no arithmetic of the eviction / attention method.  It maps
 * (stream key, logical element index) to a 16-bit table index with integer
 * operations only, so a host build (gcc) and a device build (hipcc) produce the
 * same bits.  The table itself (an inverse-normal-CDF lookup, 65,536 entries,
 * already rounded to the tensor's element type) is built by the Python side and
 * handed to both fills as plain data.
 *
 * The mixing function is the public splitmix64 output stage (Steele, Lea,
 * Flood 2014: "Fast splittable pseudorandom number generators").
 */
#ifndef SAGEKV_SYNTH_COUNTER_RNG_H
#define SAGEKV_SYNTH_COUNTER_RNG_H

#include <stdint.h>

#ifdef __HIPCC__
#define SYNTH_FN __host__ __device__ static inline
#else
#define SYNTH_FN static inline
#endif

#define SYNTH_GOLDEN 0x9E3779B97F4A7C15ull

SYNTH_FN uint64_t synth_mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* One independent stream per (seed, tensor id). */
SYNTH_FN uint64_t synth_stream_key(uint64_t seed, uint64_t tensor_id) {
  return synth_mix64(synth_mix64(seed + SYNTH_GOLDEN) + tensor_id * SYNTH_GOLDEN);
}

/* 64 random bits for counter value `ctr` of a stream. */
SYNTH_FN uint64_t synth_bits64(uint64_t key, uint64_t ctr) {
  return synth_mix64(key + (ctr + 1) * SYNTH_GOLDEN);
}

/* Table index of logical element `elem`: four elements share one 64-bit draw. */
SYNTH_FN uint32_t synth_u16(uint64_t key, uint64_t elem) {
  uint64_t h = synth_bits64(key, elem >> 2);
  return (uint32_t)(h >> (16u * (uint32_t)(elem & 3u))) & 0xFFFFu;
}

#endif
