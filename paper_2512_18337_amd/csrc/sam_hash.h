// The 64-bit hash of a (state, token) key, shared by the host automaton (its transition table and the
// overlay table it exports) and by the device lookup that probes the overlay.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define AGENTSAM_HD __host__ __device__
#else
#define AGENTSAM_HD
#endif

#define AGENTSAM_HASH_EMPTY (~0ull)
#define AGENTSAM_WIDE_DEGREE 64          /* states with more transitions than this are also in the wide table */

AGENTSAM_HD inline uint64_t agentsam_hash64(uint64_t k) {
    k ^= k >> 33; k *= 0xff51afd7ed558ccdull; k ^= k >> 33; k *= 0xc4ceb9fe1a85ec53ull; k ^= k >> 33;
    return k;
}
