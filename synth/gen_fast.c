/* Fast path of the seeded weight generator documented in synth/model.py (same integer recipe, same
 * single fp32 multiply / add, same bf16 rounding): fills `count` consecutive elements e0.. of one
 * tensor stream.  Input generation only; none of the method's arithmetic lives here.
 * Built by __graft_entry__.build() with gcc -O3 -fopenmp; synth/model.py falls back to its numpy
 * version when this library is absent, and tests/test_synth.py compares the two bit for bit. */
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* key: stream key of (seed, tensor, layer); scale: fp32 factor; gain != 0: value = 1 + n; bf16 != 0: round
 * to bf16 (nearest even) and widen again.  out: float32[count], or float64[count] holding the same values when
 * wide != 0. */
void synth_fill(uint64_t key, uint64_t e0, uint64_t count, float scale, int gain, int bf16, int wide, void* out) {
  const uint64_t GOLD = 0x9E3779B97F4A7C15ull;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i) {
    const uint64_t e = e0 + (uint64_t)i;
    const uint64_t base = key + (3ull * e + 1ull) * GOLD;
    uint64_t s = 0;
    for (int j = 0; j < 3; ++j) {
      const uint64_t w = mix64(base + (uint64_t)j * GOLD);
      s += (w & 0xFFFFull) + ((w >> 16) & 0xFFFFull) + ((w >> 32) & 0xFFFFull) + (w >> 48);
    }
    float v = (float)((int32_t)s - 393210) * scale;
    if (gain) v = 1.0f + v;
    if (bf16) {
      uint32_t u;
      memcpy(&u, &v, 4);
      u = ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16) << 16;
      memcpy(&v, &u, 4);
    }
    if (wide) ((double*)out)[i] = (double)v;
    else ((float*)out)[i] = v;
  }
}
