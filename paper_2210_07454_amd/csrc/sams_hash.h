// Device-side hash family of the Count Sketch (Sec. II-C of arXiv 2210.07454 names the bucket and
// sign hashes; the family itself is y = (a*l + b) mod p, p = 2^31 - 1, as declared in sams.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sams {

constexpr uint32_t kP31 = 2147483647u;

// (a*l + b) mod (2^31 - 1) for a, b, l < 2^31.  The 62-bit product is folded twice with the
// Mersenne identity 2^31 = 1 (mod p); after two folds the value is at most p + 1.
__device__ __forceinline__ uint32_t hash_y(uint32_t a, uint32_t b, uint32_t l)
{
    uint64_t x = (uint64_t)a * (uint64_t)l + (uint64_t)b;          // < 2^62 + 2^31
    uint64_t f = (x & kP31) + (x >> 31);                            // < 2^32
    uint32_t g = ((uint32_t)f & kP31) + (uint32_t)(f >> 31);        // <= p + 1
    return g >= kP31 ? g - kP31 : g;
}

// y mod c without a hardware divide: m = floor(2^64 / c) + 1, fastmod(y) = mulhi64(m * y, c).
// Exact for all 32-bit y and c (Lemire, Kaser, Kurz 2019).  c a power of two uses a mask.
struct ModC {
    uint64_t magic;
    uint32_t c;
    uint32_t mask;   // c - 1 if c is a power of two, else 0xffffffff with pow2 == 0
    uint32_t pow2;
};

__host__ inline ModC make_modc(uint32_t c)
{
    ModC m;
    m.c = c;
    m.pow2 = (c & (c - 1)) == 0 ? 1u : 0u;
    m.mask = c - 1;
    m.magic = c > 1 ? (~(uint64_t)0) / c + 1 : 0;
    return m;
}

__device__ __forceinline__ uint32_t mod_c(const ModC &m, uint32_t y)
{
    if (m.pow2) return y & m.mask;
    uint64_t low = m.magic * (uint64_t)y;
    return (uint32_t)__umul64hi(low, (uint64_t)m.c);
}

struct RowHash {
    uint32_t ah, bh, as, bs;
};

struct HashParams {
    RowHash row[16];
    ModC modc;
    int32_t r;
};

__device__ __forceinline__ uint32_t bucket_of(const HashParams &hp, int j, uint32_t l)
{
    return mod_c(hp.modc, hash_y(hp.row[j].ah, hp.row[j].bh, l));
}

// true = negative sign (hash value odd)
__device__ __forceinline__ bool sign_neg(const HashParams &hp, int j, uint32_t l)
{
    return (hash_y(hp.row[j].as, hp.row[j].bs, l) & 1u) != 0;
}

}  // namespace sams
