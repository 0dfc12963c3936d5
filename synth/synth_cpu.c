/*
 * Seeded synthetic-input generator, host side.
 *
 * This module only produces INPUT DATA (weights, KV rows, token ids).  It holds none of the
 * decoder's arithmetic and none of the task-graph method; the CPU oracle and the GPU test
 * harness both draw their inputs from it so that the two sides see bit-identical tensors.
 *
 * Element i of tensor `tid` under `seed` is   table[ mix64(seed, tid, i) >> 48 ]
 * where `table` has 65,536 bf16 bit patterns (quantiles of the wanted distribution, built in
 * synth/gen.py) and mix64 is the splitmix64 output function applied to an affine combination
 * of (seed, tid, i).  Integer-only, so a device implementation reproduces it exactly.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint64_t synth_mix64(uint64_t seed, uint64_t tid, uint64_t i) {
  uint64_t z = seed * 0x9E3779B97F4A7C15ull + tid * 0xD1B54A32D192ED03ull + i;
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

uint64_t synth_hash(uint64_t seed, uint64_t tid, uint64_t i) { return synth_mix64(seed, tid, i); }

/* out[k] = table[hash(seed, tid, i0 + k) >> 48] for k in [0, n). */
void synth_fill_bf16(uint16_t *out, uint64_t seed, uint64_t tid, uint64_t i0, uint64_t n,
                     const uint16_t *table) {
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < (int64_t)n; ++k)
    out[k] = table[synth_mix64(seed, tid, i0 + (uint64_t)k) >> 48];
}
