/*
 * Philox4x32-10 counter-based generator, written from the published definition
 * (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11):
 * ten rounds of two 32x32->64 multiplies whose high halves are xored with the other
 * counter words and the round key, with a Weyl key schedule.
 *
 * Part of the CPU oracle (test infrastructure; shares nothing with the GPU library).
 * The paper under study leaves the random source unspecified (JAX keys); using a
 * counter-based generator keyed by (seed, env, step, draw) is this build's reading.
 */
#include "craftax_oracle.h"

#define PHILOX_M0 0xD2511F53u
#define PHILOX_M1 0xCD9E8D57u
#define PHILOX_W0 0x9E3779B9u
#define PHILOX_W1 0xBB67AE85u

void orc_philox_round(uint32_t c[4], const uint32_t k[2])
{
    uint64_t p0 = (uint64_t)PHILOX_M0 * c[0];
    uint64_t p1 = (uint64_t)PHILOX_M1 * c[2];
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k[0];
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k[1];
    uint32_t n3 = (uint32_t)p0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

/* Multiplicative inverse of an odd 32-bit number modulo 2^32 (Newton iteration). */
static uint32_t inv32(uint32_t a)
{
    uint32_t x = a;               /* correct to 3 bits */
    for (int i = 0; i < 5; i++) x *= 2u - a * x;
    return x;
}

/* Inverts orc_philox_round: the low product words give back c0 and c2 because the
 * multipliers are odd; the high words are then recomputed and xored away. */
void orc_philox_round_inv(uint32_t c[4], const uint32_t k[2])
{
    uint32_t c0 = c[3] * inv32(PHILOX_M0);
    uint32_t c2 = c[1] * inv32(PHILOX_M1);
    uint32_t hi0 = (uint32_t)(((uint64_t)PHILOX_M0 * c0) >> 32);
    uint32_t hi1 = (uint32_t)(((uint64_t)PHILOX_M1 * c2) >> 32);
    uint32_t c1 = c[0] ^ hi1 ^ k[0];
    uint32_t c3 = c[2] ^ hi0 ^ k[1];
    c[0] = c0; c[1] = c1; c[2] = c2; c[3] = c3;
}

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    uint32_t k[2] = { key[0], key[1] };
    for (int r = 0; r < 10; r++) {
        if (r > 0) { k[0] += PHILOX_W0; k[1] += PHILOX_W1; }
        orc_philox_round(c, k);
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* n independent evaluations: ctrs[4n], keys[2n] -> out[4n]. */
void orc_philox_batch(const uint32_t *ctrs, const uint32_t *keys, uint32_t *out, int n)
{
    for (int i = 0; i < n; i++) orc_philox4x32_10(ctrs + 4 * i, keys + 2 * i, out + 4 * i);
}
