/* CPU fast path of the counter-based weight generator (same recipe as generator.py,
 * bit for bit): used where the torch integer code is too slow on the host, i.e. when a
 * full-size model has to be regenerated tensor by tensor.  Holds no arithmetic of the
 * decoding method, only the input generator.
 *
 *   z_j   = mix(key + (3e + j + 1) * GOLDEN), j = 0, 1, 2      (mix = splitmix64 finaliser)
 *   s     = sum of the twelve 16-bit fields of z_0, z_1, z_2
 *   value = fp32((s - 393210) / 65536) * fp32(std) [+ 1 for norm gains], RNE to bf16 on request
 *
 * Build: gcc -O3 -fopenmp -shared -fPIC fastgen.c -o libfastgen.so
 */
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint32_t fields16(uint64_t z) {
    return (uint32_t)(z & 0xFFFF) + (uint32_t)((z >> 16) & 0xFFFF) +
           (uint32_t)((z >> 32) & 0xFFFF) + (uint32_t)(z >> 48);
}

static inline float normal_at(uint64_t key, uint64_t e) {
    uint64_t base = e * 3ull;
    uint32_t s = 0;
    for (int j = 1; j <= 3; ++j) s += fields16(mix64((base + (uint64_t)j) * 0x9E3779B97F4A7C15ull + key));
    return (float)((int32_t)s - 393210) * (1.0f / 65536.0f);
}

static inline uint16_t bf16_rne(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);   /* inf / nan: not produced here */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* out_kind: 0 = fp32, 1 = bf16 (uint16 bit patterns).  add_one: norm gains are 1 + std * n. */
void synth_fill(uint64_t key, int64_t start, int64_t count, float std, int add_one, int out_kind, void* out) {
    float* of = (float*)out;
    uint16_t* ob = (uint16_t*)out;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        float x = normal_at(key, (uint64_t)(start + i)) * std;
        if (add_one) x = x + 1.0f;
        if (out_kind == 1) ob[i] = bf16_rne(x);
        else of[i] = x;
    }
}
