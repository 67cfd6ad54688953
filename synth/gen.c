/*
 * Seeded synthetic-input generator shared by the tests, the benchmark and the
 * CPU oracle's callers.  It holds none of the method's arithmetic: it only
 * turns (key, element index) into reproducible pseudo-random tensors, so that
 * the oracle and the GPU library are fed the very same bytes and any slice of
 * any tensor can be regenerated alone.
 *
 * Generator: counter based.  Word j of stream `key` is splitmix64's output
 * function applied to key + j (Steele, Lea & Flood's finaliser).  Normal
 * variates come in Box-Muller pairs: pair p of a stream uses words 2p and
 * 2p+1, element 2p takes the cosine branch and 2p+1 the sine branch, all in
 * double.  Outlier decisions use a second stream so that turning them on does
 * not change the underlying normal values.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t sm64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t fqs_hash64(uint64_t z) { return sm64(z); }

/* float -> IEEE binary16 bits, round to nearest even, overflow to infinity. */
static inline uint16_t f32_to_f16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x7F800000u) /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((a > 0x7F800000u) ? 0x200u : 0u));
    if (a >= 0x477FF000u) /* rounds to >= 65520 -> inf */
        return (uint16_t)(sign | 0x7C00u);
    if (a < 0x38800000u) { /* below the smallest normal half: subnormal or zero */
        if (a < 0x33000000u) /* < 2^-25 */
            return (uint16_t)sign;
        uint32_t e = a >> 23;                          /* 102..112 */
        uint32_t m = (a & 0x7FFFFFu) | 0x800000u;      /* 24-bit significand */
        uint32_t shift = 126u - e;                     /* 14..24 */
        uint32_t q = m >> shift;
        uint32_t rem = m & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1u);
        if (rem > half || (rem == half && (q & 1u)))
            q++;
        return (uint16_t)(sign | q);
    }
    uint32_t q = (a - 0x38000000u) >> 13; /* rebias 127 -> 15, keep 10 bits */
    uint32_t rem = a & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (q & 1u)))
        q++;
    return (uint16_t)(sign | q);
}

uint16_t fqs_f32_to_f16(float f) { return f32_to_f16_bits(f); }

static inline void normal_pair(uint64_t key, uint64_t p, double *c, double *s)
{
    const double two_pi = 6.283185307179586476925286766559;
    uint64_t a = sm64(key + 2u * p), b = sm64(key + 2u * p + 1u);
    double u1 = (double)((a >> 11) + 1u) * (1.0 / 9007199254740992.0); /* (0,1] */
    double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);        /* [0,1) */
    double r = sqrt(-2.0 * log(u1));
    *c = r * cos(two_pi * u2);
    *s = r * sin(two_pi * u2);
}

static inline double outlier_gain(uint64_t okey, uint64_t i, double p, double mul)
{
    if (p <= 0.0)
        return 1.0;
    double u = (double)(sm64(okey + i) >> 11) * (1.0 / 9007199254740992.0);
    return u < p ? mul : 1.0;
}

/*
 * Elements [first, first+count) of the stream: mean + std * n_i, multiplied by
 * `mul` with probability `p` (decided by stream `okey`), rounded double ->
 * float -> half (both to nearest even).  Output: binary16 bit patterns.
 */
void fqs_normal_f16(uint64_t key, uint64_t okey, uint64_t first, uint64_t count,
                    double mean, double std, double p, double mul, uint16_t *out)
{
    if (count == 0)
        return;
    uint64_t p0 = first >> 1, p1 = (first + count - 1u) >> 1;
    long long np = (long long)(p1 - p0 + 1u);
#pragma omp parallel for schedule(static)
    for (long long t = 0; t < np; t++) {
        uint64_t pr = p0 + (uint64_t)t;
        double c, s;
        normal_pair(key, pr, &c, &s);
        uint64_t i0 = 2u * pr, i1 = i0 + 1u;
        if (i0 >= first && i0 < first + count)
            out[i0 - first] = f32_to_f16_bits((float)((mean + std * c) * outlier_gain(okey, i0, p, mul)));
        if (i1 >= first && i1 < first + count)
            out[i1 - first] = f32_to_f16_bits((float)((mean + std * s) * outlier_gain(okey, i1, p, mul)));
    }
}

/* Same stream, rounded to float.  out[i] = base[i] + value when base != NULL. */
void fqs_normal_f32(uint64_t key, uint64_t first, uint64_t count, double mean, double std,
                    const float *base, float *out)
{
    if (count == 0)
        return;
    uint64_t p0 = first >> 1, p1 = (first + count - 1u) >> 1;
    long long np = (long long)(p1 - p0 + 1u);
#pragma omp parallel for schedule(static)
    for (long long t = 0; t < np; t++) {
        uint64_t pr = p0 + (uint64_t)t;
        double c, s;
        normal_pair(key, pr, &c, &s);
        uint64_t i0 = 2u * pr, i1 = i0 + 1u;
        if (i0 >= first && i0 < first + count) {
            uint64_t j = i0 - first;
            out[j] = (float)((base ? (double)base[j] : 0.0) + mean + std * c);
        }
        if (i1 >= first && i1 < first + count) {
            uint64_t j = i1 - first;
            out[j] = (float)((base ? (double)base[j] : 0.0) + mean + std * s);
        }
    }
}

/* out[i] = choices[ word_i mod n_choices ] for elements [first, first+count). */
void fqs_choice_i32(uint64_t key, uint64_t first, uint64_t count, const int32_t *choices,
                    int32_t n_choices, int32_t *out)
{
    for (uint64_t i = 0; i < count; i++)
        out[i] = choices[(sm64(key + first + i) >> 16) % (uint64_t)n_choices];
}
