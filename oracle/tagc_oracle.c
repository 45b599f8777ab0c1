/*
 * TAGC oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, sequential, single-threaded C implementation of what one TAGC
 * communication-hook call computes for a gradient bucket (paper Algorithm 1,
 * the accumulate / sparsify / create_index / compress / peeling_decompress
 * steps, with the
 * two collectives replaced by an element-wise OR and an element-wise sum over
 * N simulated ranks).  It exists so that the HIP library can be checked
 * against something that can be read side by side with the paper.  It shares
 * no code, header, table or constant generator with the HIP path; only tests,
 * the smoke check and the bench's cpu_baseline leg may call it.
 *
 * Arithmetic type: the paper states that the inherited LHC implementation is
 * float32-only (section 5), so sketch cells and decoded values are float32
 * and every add/subtract below is a single float32 operation in a fixed,
 * stated order.  Integer work (keys, counts, hashes, bit maps, degrees) is
 * exact.
 *
 * Where the paper only names a structure (Index, Count Sketch, peeling;
 * section 2.2) the concrete encoding used here is the one this repository
 * fixes for both sides; each function says which passage it follows and what
 * it had to decide on its own.
 *
 * Pinning: every function is pinned by a CPU test against something other
 * than itself (brute force, closed forms, library routines, invariants, the
 * numbers the paper prints); the single exception is the absolute value of a
 * sketch cell for random float inputs, which depends on summation order by
 * design ("parity unpinned" beyond tolerance for that one quantity).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define TAGCO_F32 0
#define TAGCO_BF16 1

#define TAGCO_SIZE_LOAD_FACTOR 0
#define TAGCO_SIZE_FIXED_RATIO 1

/* ------------------------------------------------------------------ keys */

/* Raw bits of element `pos` widened to a float32 bit pattern.  bf16 is the
 * upper half of a float32, so widening is exact. */
static uint32_t f32_bits_at(const void *g, int dtype, uint64_t pos)
{
    if (dtype == TAGCO_F32) {
        uint32_t b;
        memcpy(&b, (const char *)g + 4 * pos, 4);
        return b;
    }
    uint16_t h;
    memcpy(&h, (const char *)g + 2 * pos, 2);
    return (uint32_t)h << 16;
}

/* Magnitude key: the float32 bit pattern with the sign bit cleared.  For
 * finite values unsigned order of keys equals order of |g|; +0 and -0 map to
 * key 0.  (Sparsification by magnitude: section 3.2, "Gradient
 * Sparsification".) */
uint32_t tagco_key(uint32_t f32_bits) { return f32_bits & 0x7FFFFFFFu; }

/* k = floor(n * keep_ppm / 10^6): the number of entries that may survive so
 * that at least theta = 1 - keep_ppm/10^6 of the fragment becomes zero
 * (section 3.2: "at least theta% of the values become zero"). */
uint64_t tagco_keep_count(uint64_t n, uint32_t keep_ppm)
{
    return (uint64_t)(((unsigned __int128)n * keep_ppm) / 1000000u);
}

typedef struct {
    uint32_t key;
    uint32_t pos;
} key_pos;

static int cmp_key_desc_pos_asc(const void *a, const void *b)
{
    const key_pos *x = (const key_pos *)a, *y = (const key_pos *)b;
    if (x->key != y->key)
        return x->key > y->key ? -1 : 1;
    if (x->pos != y->pos)
        return x->pos < y->pos ? -1 : 1;
    return 0;
}

static int cmp_u32_asc(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return x < y ? -1 : (x > y);
}

/*
 * sparsify + create_index for one gradient fragment (Algorithm 1, the
 * sparsify and create_index steps; threshold rule of section 3.2).
 *
 * Definition written out: order the n positions by (magnitude descending,
 * position ascending); the first k survive, except that exact zeros never
 * survive.  Survivors are reported as (c-index, float32 value) in ascending
 * c-index, c-index = c_off + position, and their bits are set in `bitmap`
 * (bit j of the Index lives in word j>>5, bit j&31; 1 bit per parameter as
 * in section 3.1 / Figure 1).
 *
 * Returns the number of non-finite inputs seen (the method is undefined for
 * them; callers treat >0 as an error), or -1 on allocation failure.
 */
int64_t tagco_sparsify_segment(const void *g, int dtype, uint64_t offset,
                               uint64_t n, uint64_t k, uint32_t c_off,
                               uint32_t *idx_out, float *val_out,
                               uint32_t *bitmap, uint64_t *cnt_out)
{
    int64_t nonfinite = 0;
    *cnt_out = 0;
    if (n == 0)
        return 0;
    key_pos *kp = (key_pos *)malloc(n * sizeof(key_pos));
    if (!kp)
        return -1;
    for (uint64_t p = 0; p < n; ++p) {
        uint32_t key = tagco_key(f32_bits_at(g, dtype, offset + p));
        if (key >= 0x7F800000u)
            ++nonfinite;
        kp[p].key = key;
        kp[p].pos = (uint32_t)p;
    }
    qsort(kp, n, sizeof(key_pos), cmp_key_desc_pos_asc);
    uint64_t take = k < n ? k : n;
    while (take > 0 && kp[take - 1].key == 0)
        --take; /* zeros sort last; they never survive */
    uint32_t *pos = (uint32_t *)malloc((take ? take : 1) * sizeof(uint32_t));
    if (!pos) {
        free(kp);
        return -1;
    }
    for (uint64_t t = 0; t < take; ++t)
        pos[t] = kp[t].pos;
    free(kp);
    qsort(pos, take, sizeof(uint32_t), cmp_u32_asc);
    for (uint64_t t = 0; t < take; ++t) {
        uint32_t bits = f32_bits_at(g, dtype, offset + pos[t]);
        uint32_t ci = c_off + pos[t];
        float v;
        memcpy(&v, &bits, 4);
        idx_out[t] = ci;
        val_out[t] = v;
        bitmap[ci >> 5] |= 1u << (ci & 31);
    }
    free(pos);
    *cnt_out = take;
    return nonfinite;
}

/* --------------------------------------------------- error feedback */

/* Algorithm 1, first line: g_shard <- g_shard + acc, the local gradient
 * accumulation of section 3.2 ("Gradient Sparsification": the values that
 * were zeroed are kept locally and added to the gradient of the next
 * iteration).  The paper does not say in which precision; this repository
 * reads it as the in-place add of the hook, i.e. in the gradient's own type:
 * one float32 add of the two widened operands, rounded to nearest-even back
 * to bf16 for bf16 gradients.  Elements [offset, offset + n) of `g` and
 * `acc` (raw buffers of `dtype`) are read, the sums written to `out` (same
 * layout; may alias either input). */
void tagco_accumulate(const void *g, const void *acc, int dtype,
                      uint64_t offset, uint64_t n, void *out)
{
    for (uint64_t p = offset; p < offset + n; ++p) {
        uint32_t ga = f32_bits_at(g, dtype, p), aa = f32_bits_at(acc, dtype, p);
        float gf, af, sum;
        memcpy(&gf, &ga, 4);
        memcpy(&af, &aa, 4);
        sum = gf + af;
        uint32_t sb;
        memcpy(&sb, &sum, 4);
        if (dtype == TAGCO_F32) {
            memcpy((char *)out + 4 * p, &sb, 4);
        } else {
            /* round to nearest, ties to even, on the 16 discarded bits
             * (NaN keeps a set mantissa bit) */
            uint16_t h;
            if ((sb & 0x7F800000u) == 0x7F800000u && (sb & 0x007FFFFFu))
                h = (uint16_t)((sb >> 16) | 0x0040u);
            else
                h = (uint16_t)((sb + 0x7FFFu + ((sb >> 16) & 1u)) >> 16);
            memcpy((char *)out + 2 * p, &h, 2);
        }
    }
}

/* Algorithm 1, second line, second result: acc_next keeps what sparsify
 * removed.  `summed` holds g + acc for segment elements [offset, offset+n);
 * `sel_pos` the `cnt` selected positions (relative to the segment,
 * ascending).  acc_next = summed at every other position and zero (+0) at
 * the selected ones, so that summed = sent + acc_next element by element.
 * `acc_next` may alias `summed`. */
void tagco_residual(const void *summed, int dtype, uint64_t offset, uint64_t n,
                    const uint32_t *sel_pos, uint64_t cnt, void *acc_next)
{
    const uint64_t eb = dtype == TAGCO_F32 ? 4 : 2;
    if (acc_next != summed)
        memcpy((char *)acc_next + eb * offset, (const char *)summed + eb * offset, eb * n);
    for (uint64_t t = 0; t < cnt; ++t)
        memset((char *)acc_next + eb * (offset + sel_pos[t]), 0, eb);
}

/* --------------------------------------------------------- index merging */

/* index <- All-Reduce(local_index) with the operation the paper says is the
 * intended one, bitwise OR (section 2.2, last paragraph); returns the number
 * of set bits U of the merged Index. */
uint64_t tagco_index_or(const uint32_t *const *maps, uint32_t n_ranks,
                        uint64_t words, uint32_t *out)
{
    uint64_t u = 0;
    for (uint64_t w = 0; w < words; ++w) {
        uint32_t x = 0;
        for (uint32_t r = 0; r < n_ranks; ++r)
            x |= maps[r][w];
        out[w] = x;
        u += (uint64_t)__builtin_popcount(x);
    }
    return u;
}

/* ---------------------------------------------------------- sketch layout */

/*
 * The Index as the paper's implementation has to move it: NCCL has no bitwise
 * OR, so the OR is simulated by addition (section 2.2), either on the 1-bit
 * Index ("faster, but with a higher amount of collisions") or on a 4-bit one
 * ("stable, but 4 times bigger").  The paper gives no layout; this
 * repository's reading:
 *
 *   wire words are unsigned 32-bit integers and the All-Reduce adds them as
 *   such (wrapping), so a carry runs into the next parameter's field and the
 *   carry out of a word is lost;
 *   1 bit:  the wire Index is the local Index itself (parameter j = bit j&31
 *           of word j>>5);
 *   4 bit:  one counter per parameter, 0 or 1 locally, parameter j in bits
 *           4*(j&7) .. 4*(j&7)+3 of wire word j>>3;
 *   the merged Index has parameter j set iff its field of the sum is not 0.
 *
 * With 4 bits and at most 15 ranks no field can overflow and the result is
 * the OR.  With 1 bit every position that an even number of ranks kept
 * disappears and its carries set or clear higher positions of the word: the
 * "collisions".
 */

/* local 1-bit Index -> 4-bit wire Index (4 * words words) */
void tagco_index_widen4(const uint32_t *map, uint64_t words, uint32_t *wire)
{
    for (uint64_t w = 0; w < words; ++w)
        for (uint32_t q = 0; q < 4; ++q) {
            uint32_t x = 0;
            for (uint32_t p = 0; p < 8; ++p)
                x |= ((map[w] >> (8 * q + p)) & 1u) << (4 * p);
            wire[4 * w + q] = x;
        }
}

/* All-Reduce by addition of the ranks' wire Indexes; `maps` are the local
 * 1-bit Indexes, `bits` is 1 or 4; writes the merged 1-bit Index and returns
 * its number of set bits. */
uint64_t tagco_index_add(const uint32_t *const *maps, uint32_t n_ranks,
                         uint64_t words, uint32_t bits, uint32_t *out)
{
    uint64_t U = 0;
    for (uint64_t w = 0; w < words; ++w) {
        uint32_t merged = 0;
        if (bits == 1) {
            for (uint32_t r = 0; r < n_ranks; ++r)
                merged += maps[r][w];
        } else {
            for (uint32_t q = 0; q < 4; ++q) {
                uint32_t sum = 0;
                for (uint32_t r = 0; r < n_ranks; ++r) {
                    uint32_t wire[4];
                    tagco_index_widen4(&maps[r][w], 1, wire);
                    sum += wire[q];
                }
                for (uint32_t p = 0; p < 8; ++p)
                    if ((sum >> (4 * p)) & 0xFu)
                        merged |= 1u << (8 * q + p);
            }
        }
        out[w] = merged;
        for (uint32_t b = 0; b < 32; ++b)
            U += (merged >> b) & 1u;
    }
    return U;
}

static uint64_t ceil_div_u64(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

/*
 * Size and partitioning of the Count Sketch.
 *
 * The paper fixes only the total: n/c cells of 32 bit for "c-x compression"
 * (Figure 1 caption, Table 1), or -- in this repository's workloads -- a
 * multiple lf of the number U of non-zeros of the merged Index.  Everything
 * else is this repository's format:
 *
 *   target cells  M = ceil(lf_milli*U/1000)           (load-factor mode)
 *                 M = ceil(n_real*1000/ratio_milli)   (fixed-ratio mode)
 *   partitions    A = max(1, ceil(U/P_cap), ceil(M/(3q))),  q = T_cap/3
 *                 (A = 0 when U = 0)
 *   sub-table     m_sub = max(1, ceil(M/(3A)))  resp.  max(1, floor(M/(3A)))
 *   total         m = 3*A*m_sub
 *
 * The U non-zeros, in ascending index order, are dealt to the A partitions
 * in contiguous runs: partition a holds ranks [floor(a*U/A), floor((a+1)*U/A)).
 * A partition owns the 3*m_sub consecutive cells starting at a*3*m_sub; hash
 * function j of an index addresses sub-table j of its partition.
 */
void tagco_layout(uint64_t U, uint32_t mode, uint32_t milli, uint64_t n_real,
                  uint32_t P_cap, uint32_t T_cap, uint64_t *A_out,
                  uint64_t *m_sub_out, uint64_t *m_out)
{
    if (U == 0) {
        *A_out = 0;
        *m_sub_out = 0;
        *m_out = 0;
        return;
    }
    uint64_t M = (mode == TAGCO_SIZE_LOAD_FACTOR)
                     ? ceil_div_u64((uint64_t)milli * U, 1000)
                     : ceil_div_u64(n_real * 1000, milli);
    uint64_t q = T_cap / 3;
    uint64_t A = ceil_div_u64(U, P_cap);
    uint64_t A2 = ceil_div_u64(M, 3 * q);
    if (A2 > A)
        A = A2;
    if (A < 1)
        A = 1;
    uint64_t m_sub = (mode == TAGCO_SIZE_LOAD_FACTOR) ? ceil_div_u64(M, 3 * A)
                                                      : M / (3 * A);
    if (m_sub < 1)
        m_sub = 1;
    *A_out = A;
    *m_sub_out = m_sub;
    *m_out = 3 * A * m_sub;
}

/* First rank of partition a: floor(a*U/A). */
uint64_t tagco_part_start(uint64_t a, uint64_t U, uint64_t A)
{
    return (uint64_t)(((unsigned __int128)a * U) / A);
}

/*
 * bnd[a] = c-index of the non-zero whose rank is the first of partition a
 * (n_c if the partition and all later ones are empty), bnd[A] = n_c.  An
 * index i belongs to partition a iff bnd[a] <= i < bnd[a+1] and i is set.
 */
void tagco_bounds(const uint32_t *bitmap, uint64_t n_c, uint64_t U, uint64_t A,
                  uint32_t *bnd)
{
    uint64_t a = 0, rank = 0;
    for (uint64_t i = 0; i < n_c && a < A; ++i) {
        if (!((bitmap[i >> 5] >> (i & 31)) & 1u))
            continue;
        while (a < A && tagco_part_start(a, U, A) == rank)
            bnd[a++] = (uint32_t)i;
        ++rank;
    }
    while (a <= A)
        bnd[a++] = (uint32_t)n_c;
}

/* ------------------------------------------------------------------ hash */

/* 32-bit finaliser: xor-shift / odd-multiply, twice, closing xor-shift.  The
 * two multipliers are the leading fractional bits of sqrt(2) and sqrt(3). */
uint32_t tagco_mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

/* Seed word of hash function j, from the 64-bit configuration seed. */
uint32_t tagco_seed_word(uint64_t seed, uint32_t j)
{
    uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    return tagco_mix32(lo ^ tagco_mix32(hi + 0x9E3779B9u * (j + 1)));
}

/*
 * Hash function j of c-index i (a Count Sketch has, per hash function, a
 * bucket hash and a +-1 sign hash; the paper cites the structure by name
 * only, section 2.2), under the salt of i's partition (tagco_salts below;
 * salt 0 for nearly every partition):
 *   h    = mix32(i xor seed_word(j + 3*salt))
 *   slot = floor(h * m_sub / 2^32)   within sub-table j of i's partition
 *   sign = -1 if h is odd else +1
 */
void tagco_hash(uint32_t i, uint64_t seed, uint32_t j, uint32_t salt,
                uint32_t m_sub, uint32_t *slot, int32_t *sign)
{
    uint32_t h = tagco_mix32(i ^ tagco_seed_word(seed, j + 3 * salt));
    *slot = (uint32_t)(((uint64_t)h * m_sub) >> 32);
    *sign = (h & 1u) ? -1 : 1;
}

static uint64_t cell_of(uint32_t i, uint64_t a, uint32_t j, uint64_t m_sub,
                        uint64_t seed, uint32_t salt, int plus_only,
                        float *sgn)
{
    uint32_t slot;
    int32_t s;
    tagco_hash(i, seed, j, salt, (uint32_t)m_sub, &slot, &s);
    *sgn = plus_only ? 1.0f : (float)s;
    return a * 3 * m_sub + (uint64_t)j * m_sub + slot;
}

/* ------------------------------------------------------------------ salts */

static int cmp_u64_asc(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return x < y ? -1 : (x > y);
}

/*
 * The paper calls the compression lossless (section 2.2, Table 1).  Peeling
 * can never separate two non-zeros that fall into the same three cells, and
 * with the three cells confined to one partition of m_sub cells per hash
 * function that happens to some pair of a partition's P non-zeros with
 * probability about P^2 / (2 m_sub^3): a few pairs per 10^8 non-zeros at this
 * format's partition sizes, each costing two entries of the gradient.
 *
 * This repository's remedy uses what Algorithm 1 already provides: the merged
 * Index reaches every rank before compress(g_shard, index) runs, so encoder
 * and decoder can both derive, from the Index alone, a per-partition salt for
 * the hash functions:
 *
 *   salt[a] = the smallest s in [0, TAGCO_SALT_LIMIT) under which no two
 *             non-zeros of partition a have the same (slot_0, slot_1, slot_2);
 *             TAGCO_SALT_LIMIT - 1 if there is none (then peeling reports the
 *             entries it cannot recover, as always).
 *
 * Written out as the definition: for each s in turn, the triples of the
 * partition's non-zeros are sorted and neighbours compared.  Nothing travels:
 * the salts are a function of the merged Index and the seed.
 */
#define TAGCO_SALT_LIMIT 16

int tagco_salts(const uint32_t *bitmap, uint64_t n_c, uint64_t U, uint64_t A,
                uint64_t m_sub, uint64_t seed, uint32_t *salt_out)
{
    if (U == 0 || A == 0)
        return 0;
    uint32_t *idx = (uint32_t *)malloc(U * sizeof(uint32_t));
    uint64_t *key = (uint64_t *)malloc(U * sizeof(uint64_t));
    if (!idx || !key) {
        free(idx);
        free(key);
        return -1;
    }
    uint64_t t = 0;
    for (uint64_t i = 0; i < n_c; ++i)
        if ((bitmap[i >> 5] >> (i & 31)) & 1u)
            idx[t++] = (uint32_t)i;
    for (uint64_t a = 0; a < A; ++a) {
        uint64_t r0 = tagco_part_start(a, U, A), r1 = tagco_part_start(a + 1, U, A);
        uint64_t n = r1 - r0;
        salt_out[a] = TAGCO_SALT_LIMIT - 1;
        for (uint32_t s = 0; s < TAGCO_SALT_LIMIT; ++s) {
            for (uint64_t u = 0; u < n; ++u) {
                uint64_t k = 0;
                for (uint32_t j = 0; j < 3; ++j) {
                    uint32_t slot;
                    int32_t sign;
                    tagco_hash(idx[r0 + u], seed, j, s, (uint32_t)m_sub, &slot, &sign);
                    k = (k << 21) | slot; /* m_sub < 2^21 */
                }
                key[u] = k;
            }
            qsort(key, n, sizeof(uint64_t), cmp_u64_asc);
            int dup = 0;
            for (uint64_t u = 1; u < n; ++u)
                if (key[u] == key[u - 1])
                    dup = 1;
            if (!dup) {
                salt_out[a] = s;
                break;
            }
        }
    }
    free(idx);
    free(key);
    return 0;
}

/* ---------------------------------------------------------------- encode */

/*
 * local_count_sketch <- compress(g_shard, index)  (Algorithm 1).  The merged
 * Index enters only through the layout (A, m_sub), the partition bounds and
 * the partitions' salts (`salt`, A entries).
 * Pairs are taken in ascending c-index, hash functions j = 0,1,2 in order,
 * each update one float32 add.  `plus_only` replaces every sign by +1 (used
 * by a test that shows signs do not matter to peeling).
 *
 * `mask` (NULL, or the merged Index): a pair whose position is not set in it
 * is left out.  With a true OR every pair is in the merged Index; after an
 * addition-simulated OR (tagco_index_add) some are not, and this repository
 * reads compress(g_shard, index) as encoding the entries the Index names and
 * no others, so that the decoder's unknowns are exactly what the cells hold.
 */
void tagco_encode(const uint32_t *idx, const float *val, uint64_t cnt,
                  const uint32_t *bnd, uint64_t A, uint64_t m_sub,
                  uint64_t seed, const uint32_t *salt, int plus_only,
                  const uint32_t *mask, float *sketch)
{
    uint64_t m = 3 * A * m_sub;
    for (uint64_t c = 0; c < m; ++c)
        sketch[c] = 0.0f;
    uint64_t a = 0;
    for (uint64_t t = 0; t < cnt; ++t) {
        uint32_t i = idx[t];
        if (mask && !((mask[i >> 5] >> (i & 31)) & 1u))
            continue;
        while (a + 1 < A && i >= bnd[a + 1])
            ++a;
        for (uint32_t j = 0; j < 3; ++j) {
            float s;
            uint64_t c = cell_of(i, a, j, m_sub, seed, salt[a], plus_only, &s);
            sketch[c] = sketch[c] + s * val[t];
        }
    }
}

/*
 * Quantised communication of the sketch (section 5: the inherited
 * implementation is float32-only; combining the compression with
 * quantisation of what is communicated, e.g. to bfloat16, is named as the
 * next step).  This repository's reading: a rank builds its Count Sketch in
 * float32 exactly as before and rounds every cell to the nearest bfloat16,
 * ties to even, when it puts the sketch on the wire (16 bits per cell); the
 * Reduce widens the cells back and adds them in float32 in rank order, and
 * decoding is unchanged.  The cells are rounded in place and stay float32
 * values (low 16 bits zero).  Non-finite cells are not expected.
 */
void tagco_quantize_cells_bf16(float *sketch, uint64_t m)
{
    for (uint64_t c = 0; c < m; ++c) {
        uint32_t b;
        memcpy(&b, &sketch[c], 4);
        b = (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
        memcpy(&sketch[c], &b, 4);
    }
}

/* Reduce(local_count_sketch, d): element-wise float32 sum in rank order,
 * ((C_0 + C_1) + C_2) + ...  (Algorithm 1; section 3.1). */
void tagco_sum(const float *const *sketches, uint32_t n_ranks, uint64_t m,
               float *out)
{
    for (uint64_t c = 0; c < m; ++c) {
        float acc = sketches[0][c];
        for (uint32_t r = 1; r < n_ranks; ++r)
            acc = acc + sketches[r][c];
        out[c] = acc;
    }
}

/* ------------------------------------------------------------------ peel */

/*
 * g <- peeling_decompress(index, count_sketch)  (Algorithm 1; section 2.2).
 *
 * The unknowns are the set bits of the merged Index, ascending: S.  Each
 * unknown touches three cells.  deg[c] counts the unresolved unknowns that
 * touch cell c.  Rounds are synchronous:
 *   1. every unresolved unknown that touches a cell of degree 1 is selected;
 *      its value is sign_j * C[cell_j] for the smallest such j, read from the
 *      sketch as it stood when the round began;
 *   2. then, in ascending index order and j = 0,1,2, each selected unknown
 *      subtracts sign_j * x from its three cells and lowers their degrees.
 * Peeling stops at the first round that selects nothing.  Unknowns left over
 * get value 0 and are counted.  Every unknown is reported, including those
 * whose summed value is 0.
 *
 * `sketch` is modified in place.  round_out[t] = round (1-based) in which
 * unknown t was resolved, 0 if never.  `salt`: the partitions' salts (A
 * entries), the same the encoders used.
 */
int tagco_peel(const uint32_t *bitmap, uint64_t n_c, uint64_t U, uint64_t A,
               uint64_t m_sub, uint64_t seed, const uint32_t *salt,
               int plus_only, float *sketch,
               uint32_t *idx_out, float *val_out, uint32_t *round_out,
               uint32_t *rounds, uint64_t *n_unresolved)
{
    uint64_t m = 3 * A * m_sub;
    *rounds = 0;
    *n_unresolved = 0;
    if (U == 0)
        return 0;
    uint32_t *deg = (uint32_t *)calloc(m ? m : 1, sizeof(uint32_t));
    uint64_t *part = (uint64_t *)malloc(U * sizeof(uint64_t));
    uint8_t *picked = (uint8_t *)malloc(U);
    if (!deg || !part || !picked) {
        free(deg);
        free(part);
        free(picked);
        return -1;
    }
    uint64_t t = 0;
    for (uint64_t i = 0; i < n_c; ++i)
        if ((bitmap[i >> 5] >> (i & 31)) & 1u)
            idx_out[t++] = (uint32_t)i;
    /* partition of each unknown, from its rank */
    {
        uint64_t a = 0;
        for (t = 0; t < U; ++t) {
            while (a + 1 < A && tagco_part_start(a + 1, U, A) <= t)
                ++a;
            part[t] = a;
        }
    }
    for (t = 0; t < U; ++t) {
        val_out[t] = 0.0f;
        round_out[t] = 0;
        for (uint32_t j = 0; j < 3; ++j) {
            float s;
            deg[cell_of(idx_out[t], part[t], j, m_sub, seed, salt[part[t]],
                        plus_only, &s)]++;
        }
    }
    uint64_t resolved = 0;
    for (uint32_t round = 1;; ++round) {
        uint64_t n_picked = 0;
        for (t = 0; t < U; ++t) {
            picked[t] = 0;
            if (round_out[t])
                continue;
            for (uint32_t j = 0; j < 3; ++j) {
                float s;
                uint64_t c = cell_of(idx_out[t], part[t], j, m_sub, seed,
                                     salt[part[t]], plus_only, &s);
                if (deg[c] == 1) {
                    val_out[t] = s * sketch[c]; /* snapshot: no write yet */
                    picked[t] = 1;
                    ++n_picked;
                    break;
                }
            }
        }
        if (n_picked == 0)
            break;
        for (t = 0; t < U; ++t) {
            if (!picked[t])
                continue;
            for (uint32_t j = 0; j < 3; ++j) {
                float s;
                uint64_t c = cell_of(idx_out[t], part[t], j, m_sub, seed,
                                     salt[part[t]], plus_only, &s);
                sketch[c] = sketch[c] - s * val_out[t];
                deg[c]--;
            }
            round_out[t] = round;
        }
        resolved += n_picked;
        *rounds = round;
    }
    *n_unresolved = U - resolved;
    free(deg);
    free(part);
    free(picked);
    return 0;
}

/*
 * Estimation, the second of the two decompression algorithms named in
 * section 2.2 (it works at any density but is noisy; TAGC sparsifies so that
 * peeling suffices, section 3.2).  The paper gives no formula; this is the
 * textbook Count Sketch point query: an unknown with index i is estimated as
 * the median of its three readings sign_j(i) * C[cell_j(i)].
 *
 * It is applied to the unknowns with round_in[t] == 0 (all of them when
 * round_in is NULL), on `sketch` as it is handed in: the raw summed sketch
 * for estimation-only decoding, or what tagco_peel left behind (every
 * resolved unknown already subtracted) for the residue of a stalled peeling.
 * Estimates do not interact: nothing is subtracted between them.  val_out[t]
 * of the other unknowns is left alone.  The median of three is the middle one
 * in numeric order.  Returns the number of unknowns estimated.
 */
uint64_t tagco_estimate(const uint32_t *idx, const uint32_t *round_in,
                        uint64_t U, uint64_t A, uint64_t m_sub, uint64_t seed,
                        const uint32_t *salt, const float *sketch,
                        float *val_out)
{
    uint64_t a = 0, n_est = 0;
    for (uint64_t t = 0; t < U; ++t) {
        while (a + 1 < A && tagco_part_start(a + 1, U, A) <= t)
            ++a;
        if (round_in && round_in[t])
            continue;
        float r[3];
        for (uint32_t j = 0; j < 3; ++j) {
            float s;
            uint64_t c = cell_of(idx[t], a, j, m_sub, seed, salt[a], 0, &s);
            r[j] = s * sketch[c];
        }
        /* sort the three readings ascending, take the middle one */
        if (r[0] > r[1]) { float x = r[0]; r[0] = r[1]; r[1] = x; }
        if (r[1] > r[2]) { float x = r[1]; r[1] = r[2]; r[2] = x; }
        if (r[0] > r[1]) { float x = r[0]; r[0] = r[1]; r[1] = x; }
        val_out[t] = r[1];
        ++n_est;
    }
    return n_est;
}

/* --------------------------------------------------- communication volume */

/*
 * Bits per parameter per rank on the wire (Figures 1 and 2): an All-Reduce
 * moves its payload twice, a Reduce once.  TAGC: Index by All-Reduce, Count
 * Sketch by Reduce; LHC: both by All-Reduce.  The sketch costs 32/c bits per
 * parameter at c-x compression.
 */
double tagco_wire_bits_per_param(double index_bits, double ratio, int lhc)
{
    double sketch = 32.0 / ratio;
    return 2.0 * index_bits + (lhc ? 2.0 : 1.0) * sketch;
}
