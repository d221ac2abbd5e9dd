/*
 * TEST INFRASTRUCTURE, NOT THE PRODUCT.  Counter-based random numbers for sampling-mode decoding:
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC 2011),
 * written from the published algorithm; it shares no code with the HIP library's generator, which
 * the tests compare it with word for word.
 *
 * The state is four 32-bit counter words c0..c3 and two key words k0, k1.  One round computes the
 * two 64-bit products  p0 = 0xD2511F53 * c0  and  p1 = 0xCD9E8D57 * c2  and sets
 *     (c0, c1, c2, c3) <- (hi(p1) ^ c1 ^ k0,  lo(p1),  hi(p0) ^ c3 ^ k1,  lo(p0));
 * ten rounds are applied, and before every round but the first the key is advanced by the Weyl
 * constants  k0 += 0x9E3779B9,  k1 += 0xBB67AE85  (mod 2^32).
 *
 * How the decoder uses it (a reading of this build; the paper only asks that the sampling
 * distribution be preserved, abstract and Section 3): the uniform number of (absolute token position,
 * purpose) is  u = (w >> 8) * 2^-24  in [0, 1), w = the first output word for counter
 * (position, purpose, 0, 0) and key (seed mod 2^32, seed >> 32); purpose 0 draws a draft token,
 * 1 tests its acceptance, 2 draws a resampled / bonus / first token.  Indexing by position keeps
 * the numbers independent of the control flow.
 *
 * Parity unpinned against an external implementation: no known-answer vectors of the published
 * generator are at hand here.  What pins this file: the HIP library's independently written
 * generator agrees with it word for word, the round function is checked against its definition
 * with Python integers, and the uniforms pass a chi-square test.
 */
#include <stdint.h>

void ko_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; round++) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* first output words for counters (pos0 + i, purpose, 0, 0), i = 0..n-1 */
void ko_philox_words(uint64_t seed, uint32_t pos0, uint32_t purpose, int n, uint32_t *out)
{
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int i = 0; i < n; i++) {
        uint32_t ctr[4] = {pos0 + (uint32_t)i, purpose, 0u, 0u}, w[4];
        ko_philox4x32_10(ctr, key, w);
        out[i] = w[0];
    }
}

/* u[pos][purpose], pos = 0..n_positions-1, purpose = 0..2: the table a sampling-mode decoder reads */
void ko_philox_uniforms(uint64_t seed, int n_positions, float *u)
{
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int pos = 0; pos < n_positions; pos++)
        for (uint32_t purpose = 0; purpose < 3; purpose++) {
            uint32_t ctr[4] = {(uint32_t)pos, purpose, 0u, 0u}, w[4];
            ko_philox4x32_10(ctr, key, w);
            u[(long)pos * 3 + purpose] = (float)(w[0] >> 8) * (1.0f / 16777216.0f);
        }
}
