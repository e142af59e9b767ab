/*
 * CPU oracle for the key of a transaction -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Sec. 4.1 of the paper (Dragon, arXiv 1707.08265) binds a function -- the graph pruned for one choice of
 * fetches and feeds -- to a hashing key generated from that choice, so that running a session again with an
 * existing transaction builds no second graph.  The paper names no hash function.  The reading taken here:
 * the key of (graph, target sets) is the graph's identity plus a 128-bit digest of the target sets as the prune
 * receives them, i.e. of the word sequence
 *
 *     w = [ num_sets, n, rowptr[0], ..., rowptr[n], idx[0], ..., idx[m-1] ]        (n row pointers + 1, m targets)
 *
 * digest_k = sum over positions i of  mix( (i + 1) * G  +  w_i * C_k  +  S_k )   mod 2^64,   k = 0, 1
 *
 * where mix is the output function of SplitMix64 (Steele, Lea, Flood: "Fast splittable pseudorandom number
 * generators", OOPSLA 2014; the constants of its public-domain reference code), G = 0x9E3779B97F4A7C15 its
 * increment, w_i is taken as an unsigned 32-bit number, and C_k, S_k are odd constants that differ between the
 * two halves.  A sum of position-keyed terms: changing, moving, adding or dropping a word changes it, and the
 * terms can be added up in any order -- which is what a parallel implementation needs.
 *
 * Plain, sequential C; shares no source with the GPU library.  Parity status: mix pinned to the published
 * SplitMix64 outputs, the digest to properties (see tests/test_oracle_transaction_pins.py).
 */
#include <stdint.h>

#define ORC_G  0x9E3779B97F4A7C15ull
#define ORC_C0 0xC2B2AE3D27D4EB4Full
#define ORC_S0 0x165667B19E3779F9ull
#define ORC_C1 0xD6E8FEB86659FD93ull
#define ORC_S1 0x27D4EB2F165667C5ull

uint64_t orc_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static void add_word(uint64_t pos, int32_t word, uint64_t digest[2])
{
    const uint64_t w = (uint64_t)(uint32_t)word;
    digest[0] += orc_mix64((pos + 1) * ORC_G + w * ORC_C0 + ORC_S0);
    digest[1] += orc_mix64((pos + 1) * ORC_G + w * ORC_C1 + ORC_S1);
}

/* n = number of target sets in all (num_sets per graph times the number of graphs): tgt_rowptr has n + 1 entries. */
void orc_target_digest(int32_t num_sets, int64_t n, const int32_t *tgt_rowptr, int64_t num_targets,
                       const int32_t *tgt_idx, uint64_t digest[2])
{
    uint64_t pos = 0;
    digest[0] = digest[1] = 0;
    add_word(pos++, num_sets, digest);
    add_word(pos++, (int32_t)n, digest);
    for (int64_t s = 0; s <= n; ++s) add_word(pos++, tgt_rowptr[s], digest);
    for (int64_t j = 0; j < num_targets; ++j) add_word(pos++, tgt_idx[j], digest);
}
