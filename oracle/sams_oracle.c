/*
 * CPU oracle for the SketchedAMSGrad (gradient averaging) step -- TEST INFRASTRUCTURE ONLY.
 * Not part of the product: nothing in the HIP library or its Python binding may call it.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC sams_oracle.c -o libsams_oracle.so -lm
 * (no contraction, no reassociation: every + and * below is one IEEE operation in REAL).
 *
 * The arithmetic lives in sams_oracle_impl.h, instantiated for float (_f32: the
 * precision the kernels compute in, used wherever a floating value decides an
 * integer such as the top-k set) and for double (_f64: the reference for value
 * tolerances and for the Lemma 3 invariant).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* Hash family (Sec. II-C speaks of bucket and sign hashes without fixing a family; this is the
 * seeded 2-universal family y = (a*l + b) mod p with the Mersenne prime p = 2^31 - 1,
 * l the 0-based coordinate).  a*l + b < 2^62 + 2^31 fits in 64 bits, so plain % is exact. */
uint32_t orc_hash_y(uint32_t a, uint32_t b, uint32_t l)
{
    return (uint32_t)(((uint64_t)a * (uint64_t)l + (uint64_t)b) % 2147483647ULL);
}

/* bucket hash h_j(l) = y mod c */
int64_t orc_bucket(uint32_t a, uint32_t b, uint32_t l, int64_t c)
{
    return (int64_t)((uint64_t)orc_hash_y(a, b, l) % (uint64_t)c);
}

/* sign hash s_j(l) = +1 if y is even, -1 if odd */
int orc_sign(uint32_t a, uint32_t b, uint32_t l)
{
    return (orc_hash_y(a, b, l) & 1u) ? -1 : 1;
}

/* Dump h_j(l) and s_j(l) for every row and coordinate (for the bit-exact hash comparison). */
void orc_hash_dump(const uint32_t *hash, int32_t r, int64_t c, int64_t d,
                   int32_t *bucket /* [r][d] */, int8_t *sign /* [r][d] */)
{
    for (int32_t j = 0; j < r; ++j)
        for (int64_t l = 0; l < d; ++l) {
            bucket[(int64_t)j * d + l] = (int32_t)orc_bucket(hash[4 * j], hash[4 * j + 1], (uint32_t)l, c);
            sign[(int64_t)j * d + l] = (int8_t)orc_sign(hash[4 * j + 2], hash[4 * j + 3], (uint32_t)l);
        }
}

static int orc_cmp_i32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

static float orc_sqrt_f32(float v) { return sqrtf(v); }
static double orc_sqrt_f64(double v) { return sqrt(v); }

#define REAL float
#define SUFFIX _f32
#include "sams_oracle_impl.h"
#undef REAL
#undef SUFFIX

#define REAL double
#define SUFFIX _f64
#include "sams_oracle_impl.h"
#undef REAL
#undef SUFFIX
