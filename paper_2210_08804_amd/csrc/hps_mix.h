// The one 64-bit mixing function of the library: the finaliser of the splitmix64 generator (three
// xor-shifts around two odd multipliers; a bijection on 64-bit words with full avalanche).  The
// cache takes the set index from its upper half (Alg. 2, "slabset hasher"), the dedup operator and
// the host map take their slots and partitions from other bit ranges of the same word.
#ifndef HPS_MIX_H
#define HPS_MIX_H

#include <cstdint>

#if defined(__HIP__)
#define HPS_HOST_DEVICE __attribute__((host)) __attribute__((device)) inline __attribute__((always_inline))
#else
#define HPS_HOST_DEVICE inline
#endif

HPS_HOST_DEVICE uint64_t mix64(uint64_t x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

#endif  // HPS_MIX_H
