/*
 * Seeded synthetic tensor data: a counter-based generator keyed on
 * (seed, tensor id, logical element index).  It holds no contraction
 * arithmetic; both the CPU oracle's tests and the GPU path's tests and bench
 * take their inputs from here so that they see identical values.
 *
 * Each 64-bit draw is the splitmix64 output function applied to
 * key + (counter + 1) * golden, with key = seed ^ (tid * golden2).
 */
#include <math.h>
#include <stdint.h>

static inline uint64_t mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

static inline uint64_t draw(uint64_t key, uint64_t counter)
{
    return mix64(key + (counter + 1ULL) * 0x9E3779B97F4A7C15ULL);
}

static inline uint64_t make_key(uint64_t seed, uint64_t tid)
{
    return seed ^ (tid * 0xD1B54A32D192ED03ULL);
}

/* kind: 0 = uniform[-1,1), 1 = normal(0,1) (Box-Muller on two draws),
 *       2 = integers in [-4,4].  Elements first..first+count-1 go to out[0..count-1]. */
int wl_fill(double *out, int64_t first, int64_t count, uint64_t seed, uint64_t tid, int kind)
{
    const uint64_t key = make_key(seed, tid);
    const double two53 = 1.0 / 9007199254740992.0;
    if (kind < 0 || kind > 2)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < count; ++e) {
        uint64_t c = (uint64_t)(first + e);
        if (kind == 0) {
            uint64_t x = draw(key, c);
            out[e] = 2.0 * ((double)(x >> 11) * two53) - 1.0;
        } else if (kind == 1) {
            uint64_t x1 = draw(key, 2 * c), x2 = draw(key, 2 * c + 1);
            double u1 = ((double)(x1 >> 11) + 1.0) * two53; /* (0,1] */
            double u2 = (double)(x2 >> 11) * two53;         /* [0,1) */
            out[e] = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
        } else {
            uint64_t x = draw(key, c);
            out[e] = (double)((int64_t)((x >> 11) % 9ULL) - 4);
        }
    }
    return 0;
}
