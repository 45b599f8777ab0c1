/*
 * libtagc -- exports for tests and tools only; not part of the hot path's
 * interface (that is tagc.h).
 */
#ifndef TAGC_TEST_H
#define TAGC_TEST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Hash function j (0..2) of c-index i under partition salt `salt`, for a
 * sub-table of m_sub cells, exactly as the device code computes it (the three
 * hash functions with +-1 signs of the Count Sketch, section 2.2): slot in
 * [0, m_sub), sign +1 or -1.  Host memory only; never touches the device.
 */
void tagc_hash_host(uint32_t i, uint64_t seed, uint32_t j, uint32_t salt, uint32_t m_sub,
                    uint32_t *slot, int32_t *sign);

#ifdef __cplusplus
}
#endif
#endif /* TAGC_TEST_H */
