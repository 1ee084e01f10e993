/*
 * NUQSGD compression path -- plain CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Slow, sequential, fp64, one coordinate at a time, written from the paper.
 * It is the reference the HIP kernels are checked against; it shares no code
 * with them and must never be called from the product path.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What each function follows:
 *   nuqo_bucket_norms      Def. 1 (Sec. 3.1): r_i = |v_i| / ||v||, Euclidean norm,
 *                          one norm per bucket (Sec. 5 "bucket size").
 *   nuqo_quantize_coord    Def. 1 with the level set of Sec. 3.1
 *                          (0, 2^-s, ..., 1/2, 1); App. B eqs. (h_case1), (h_case2)
 *                          for the two-point law and its probabilities.
 *   nuqo_erc_*             App. A, Alg. 2 (Elias recursive coding).
 *   nuqo_encode            App. A, ENCODE: rounds of ERC(gap), sign bit,
 *                          ERC(log2(2^{s+1} h)); App. C parts R and E.
 *   nuqo_decode_average    App. A, DECODE, then the aggregate of Alg. 1:
 *                          (1/K) * sum_k decoded gradient.
 *   nuqo_*_table,          the same quantizer for an arbitrary level sequence
 *   nuqo_bucket_norms_linf l_0 = 0 < l_1 < ... < l_{s+1} = 1 (Sec. 3.1 before the special
 *                          case; Sec. 4.1 "Generally spaced levels", eqs. (genh_case1),
 *                          (genh_case2); the exponential family (0, p^s, ..., p, 1) of
 *                          Sec. 4.1; uniform levels = QSGD, with the maximum norm = QSGDinf,
 *                          Sec. 1 and Sec. 2).
 *
 *   nuqo_pack_fixed,       Sec. 5: the fixed-width variants ("4-bit", "8-bit" NUQSGD; 3 bits in
 *   nuqo_unpack_fixed      Table 1): every coordinate sends its sign and level index in b bits.
 *                          The paper gives no layout; the one used is in the design notes.
 *
 *   nuqo_huffman_*         Sec. 5, "Efficient Encoding": a Huffman code for the level indices,
 *                          built once from a sample's histogram ("encoded NUQSGD").  The
 *                          paper says no more; construction and layout are in the design notes.
 *
 * Points the paper leaves open (random number source, bit order, how the end
 * of a bucket's records is known, padding) are fixed by the wire-format
 * description in the project's design notes; this file implements that text.
 *
 * Pinned by tests/test_oracle_*.py: level sets, rounding probabilities by
 * exhaustive enumeration of the 2^24 uniform draws, unbiasedness, the exact
 * variance formula and Theorem 1's bound, Lemma 4's sparsity bound, hand-worked
 * ERC codewords, decode(encode(x)) == x, a hand-worked ENCODE bit string.
 * The exact random bits of a particular (seed, bucket, index) are fixed by
 * the format text, not by the paper: "parity unpinned" by the paper for those.
 * The fixed-width functions are pinned by tests/test_oracle_fixed.py: a hand-packed
 * example, the size formula, unpack(pack(q)) == q, bit positions of single codes.
 * The Huffman functions are pinned by tests/test_oracle_huffman.py: textbook code lengths
 * (dyadic and Fibonacci weights), Kraft equality, optimality against brute force over all
 * length assignments, hand-built canonical codes, a hand-coded bit string, the round trip.
 * The level-table functions are pinned by tests/test_oracle_levels.py: equality
 * with the functions above on the table (0, 2^-s, ..., 1/2, 1), exhaustive
 * enumeration of the draws against p(r) as an exact fraction, unbiasedness and
 * the variance formula on uniform and exponential tables, the ordering of the
 * three schemes' variances on Gaussian vectors.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NUQO_OK 0
#define NUQO_EINVAL (-1)
#define NUQO_ECAPACITY (-2)
#define NUQO_EMALFORMED (-5)

/* ------------------------------------------------------------------ norms */

/* Def. 1: ||v|| of every bucket, fp64, plain left-to-right sum. */
void nuqo_bucket_norms(const float *v, uint64_t d, uint32_t bucket, double *norms)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    for (uint64_t b = 0; b < nb; b++) {
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        double acc = 0.0;
        for (uint64_t i = lo; i < hi; i++)
            acc += (double)v[i] * (double)v[i];
        norms[b] = sqrt(acc);
    }
}

/* -------------------------------------------------------------------- rng */

/*
 * Counter-based uniform draw u in [0, 2^24) for coordinate `idx` of bucket
 * `bucket_index` under `seed`.  The paper only asks for independent draws;
 * the generator is this project's choice:
 *   per bucket : z = seed + (bucket_index + 1) * 0x9E3779B97F4A7C15, then the
 *                SplitMix64 output function; k0 = low word, k1 = high word.
 *   per index  : x = (k0 + idx) * 0x9E3779B1;  x ^= (x >> 15) ^ k1;
 *                x *= 0x85EBCA6B;  x ^= x >> 16;  u = x >> 8.
 */
void nuqo_rng_key(uint64_t seed, uint64_t bucket_index, uint32_t *k0, uint32_t *k1)
{
    uint64_t z = seed + (bucket_index + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z = z ^ (z >> 31);
    *k0 = (uint32_t)z;
    *k1 = (uint32_t)(z >> 32);
}

uint32_t nuqo_rng_u24(uint32_t k0, uint32_t k1, uint32_t idx)
{
    uint32_t x = (k0 + idx) * 0x9E3779B1u;
    x = x ^ (x >> 15) ^ k1;
    x = x * 0x85EBCA6Bu;
    x = x ^ (x >> 16);
    return x >> 8;
}

/* Fill u[i] for every coordinate of a d-vector cut into buckets. */
void nuqo_rng_fill(uint64_t seed, uint64_t d, uint32_t bucket, uint32_t *u)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    for (uint64_t b = 0; b < nb; b++) {
        uint32_t k0, k1;
        nuqo_rng_key(seed, b, &k0, &k1);
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        for (uint64_t i = lo; i < hi; i++)
            u[i] = nuqo_rng_u24(k0, k1, (uint32_t)(i - lo));
    }
}

/* --------------------------------------------------------------- quantizer */

/*
 * Level index j in {0..s+1} of h_i for one coordinate (l_0 = 0, l_j = 2^(j-1-s)).
 *
 * Def. 1: r = |v_i| / ||v||; level(r) is the bin with l_j <= r <= l_{j+1};
 * p(r) = (r - l_j) / (l_{j+1} - l_j); h = l_{j+1} with probability p(r), else l_j.
 * The draw is "up" iff u/2^24 < p(r), u a 24-bit uniform integer.
 *
 * Everything is done on r*||v|| instead of r so that no division is needed:
 * l_j*||v|| is exact in fp64, |v_i| - l_j*||v|| is exact (the two are within
 * a factor of two), u * (tau*||v||) is a 24-bit by 24-bit product, exact.
 * So the comparison below is the real-number statement, with no rounding.
 *
 * r >= 1 can only come from a norm that was rounded down; it maps to the top
 * level.  A zero norm or a zero coordinate gives level 0 (Q_s(0) = 0).
 */
int nuqo_quantize_coord(float vi, float norm, int s, uint32_t u24)
{
    double n = (double)norm;
    double a = fabs((double)vi);
    if (!(n > 0.0) || a == 0.0)
        return 0;
    int j = 0; /* largest j with l_j * n <= a */
    for (int t = 1; t <= s + 1; t++)
        if (ldexp(n, t - 1 - s) <= a)
            j = t;
    if (j == s + 1)
        return s + 1;
    double lo_n = (j == 0) ? 0.0 : ldexp(n, j - 1 - s); /* l_j * n      */
    double hi_n = ldexp(n, j - s);                      /* l_{j+1} * n  */
    double tau_n = hi_n - lo_n;
    int up = ((double)u24 * tau_n) < ((a - lo_n) * 16777216.0);
    return up ? j + 1 : j;
}

/* Same, vectorised over an array of draws for one fixed (vi, norm, s). */
void nuqo_quantize_coord_many(float vi, float norm, int s, const uint32_t *u24,
                              uint64_t count, uint8_t *levels)
{
    for (uint64_t i = 0; i < count; i++)
        levels[i] = (uint8_t)nuqo_quantize_coord(vi, norm, s, u24[i]);
}

/* hist[j] += number of draws u in [u_begin, u_end) that give level index j. */
void nuqo_level_histogram(float vi, float norm, int s, uint32_t u_begin, uint32_t u_end,
                          uint64_t *hist)
{
    for (uint32_t u = u_begin; u < u_end; u++)
        hist[nuqo_quantize_coord(vi, norm, s, u)]++;
}

/*
 * q[i] = level index (bits 0..6) | sign (bit 7, 1 = negative, only when the
 * level is nonzero).  `u24` holds one draw per coordinate.
 */
void nuqo_quantize_given_u(const float *v, uint64_t d, uint32_t bucket, int s,
                           const float *norms, const uint32_t *u24, uint8_t *q)
{
    for (uint64_t i = 0; i < d; i++) {
        int j = nuqo_quantize_coord(v[i], norms[i / bucket], s, u24[i]);
        uint8_t sign = (j > 0 && signbit(v[i])) ? 0x80 : 0;
        q[i] = (uint8_t)j | sign;
    }
}

/* Same with the counter generator above.  v, norms and q describe buckets
 * first_bucket, first_bucket+1, ... of a longer vector (first_bucket = 0 for a
 * whole vector); only the generator's bucket index depends on it. */
void nuqo_quantize(const float *v, uint64_t d, uint32_t bucket, int s, uint64_t seed,
                   const float *norms, uint64_t first_bucket, uint8_t *q)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    for (uint64_t b = 0; b < nb; b++) {
        uint32_t k0, k1;
        nuqo_rng_key(seed, first_bucket + b, &k0, &k1);
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        for (uint64_t i = lo; i < hi; i++) {
            uint32_t u = nuqo_rng_u24(k0, k1, (uint32_t)(i - lo));
            int j = nuqo_quantize_coord(v[i], norms[b], s, u);
            uint8_t sign = (j > 0 && signbit(v[i])) ? 0x80 : 0;
            q[i] = (uint8_t)j | sign;
        }
    }
}

/* ---------------------------------------------------- general level sets */

/* Maximum norm of every bucket (the normalization of QSGDinf): max_i |v_i|, exact. */
void nuqo_bucket_norms_linf(const float *v, uint64_t d, uint32_t bucket, double *norms)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    for (uint64_t b = 0; b < nb; b++) {
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        double m = 0.0;
        for (uint64_t i = lo; i < hi; i++) {
            double a = fabs((double)v[i]);
            if (a > m || a != a)
                m = a;
        }
        norms[b] = m;
    }
}

/*
 * Exact sign of a sum of doubles, for the decision below.  two_sum and two_prod
 * are the classical error-free transformations (Knuth; Dekker, with fma): the
 * pair they return adds up to the real-number sum or product exactly.  Adding a
 * term to a list of nonoverlapping parts with a chain of two_sum keeps the list
 * exact and nonoverlapping, smallest part first (Shewchuk's "grow expansion"),
 * so the sign of the whole is the sign of its last nonzero part.  Valid while
 * nothing overflows or underflows: the terms here lie between 2^-400 and 2^160.
 */
static void two_sum(double x, double y, double *sum, double *err)
{
    double t = x + y;
    double yy = t - x;
    *err = (x - (t - yy)) + (y - yy);
    *sum = t;
}

static void two_prod(double x, double y, double *prod, double *err)
{
    *prod = x * y;
    *err = fma(x, y, -*prod);
}

static int sign_of_sum(const double *term, int count)
{
    double part[16];
    int parts = 0;
    for (int i = 0; i < count; i++) {
        double carry = term[i];
        for (int k = 0; k < parts; k++)
            two_sum(carry, part[k], &carry, &part[k]);
        part[parts++] = carry;
    }
    for (int k = parts - 1; k >= 0; k--)
        if (part[k] != 0.0)
            return part[k] > 0.0 ? 1 : -1;
    return 0;
}

/*
 * Level index of one coordinate for an arbitrary level sequence lev[0..s+1]
 * (fp32 values, lev[0] = 0 < lev[1] < ... < lev[s+1] = 1).  Def. 1 with the
 * two cases of Sec. 4.1: r in [l_j, l_{j+1}] goes up to l_{j+1} with probability
 * p = (r - l_j) / tau_j, tau_j = l_{j+1} - l_j, i.e. for the draw u of 24 bits
 * iff u / 2^24 < p.
 *
 * As above everything is multiplied through by ||v||: the test is
 *     u * (l_{j+1} ||v|| - l_j ||v||)  <  (|v_i| - l_j ||v||) * 2^24
 * over the real numbers.  The products l ||v|| of two 24-bit significands are
 * exact in fp64; for levels that are not powers of two the differences and the
 * product with u need more than 53 bits, so the two sides are not rounded but
 * compared exactly: the sign of
 *     |v_i| 2^24 - l_j ||v|| 2^24 - u l_{j+1} ||v|| + u l_j ||v||,
 * each product with u split into an exact pair.
 */
int nuqo_quantize_coord_table(float vi, float norm, int s, const float *lev, uint32_t u24)
{
    double n = (double)norm;
    double a = fabs((double)vi);
    if (!(n > 0.0) || a == 0.0)
        return 0;
    /* not finite (the exact comparison below needs finite terms): a NaN coordinate has no level, an
     * infinite one exceeds every level, and under an infinite norm every finite coordinate is at zero */
    if (a != a)
        return 0;
    if (isinf(a))
        return s + 1;
    if (isinf(n))
        return 0;
    int j = 0; /* largest j with l_j * n <= a */
    for (int t = 1; t <= s + 1; t++)
        if ((double)lev[t] * n <= a)
            j = t;
    if (j == s + 1)
        return s + 1;
    double lo_n = (double)lev[j] * n;
    double hi_n = (double)lev[j + 1] * n;
    double term[6];
    term[0] = a * 16777216.0;
    term[1] = -lo_n * 16777216.0;
    two_prod(-(double)u24, hi_n, &term[2], &term[3]);
    two_prod((double)u24, lo_n, &term[4], &term[5]);
    return sign_of_sum(term, 6) > 0 ? j + 1 : j;
}

/* hist[j] += number of draws u in [u_begin, u_end) that give level index j. */
void nuqo_level_histogram_table(float vi, float norm, int s, const float *lev, uint32_t u_begin,
                                uint32_t u_end, uint64_t *hist)
{
    for (uint32_t u = u_begin; u < u_end; u++)
        hist[nuqo_quantize_coord_table(vi, norm, s, lev, u)]++;
}

/* q bytes of a whole vector with the counter generator, as nuqo_quantize. */
void nuqo_quantize_table(const float *v, uint64_t d, uint32_t bucket, int s, const float *lev,
                         uint64_t seed, const float *norms, uint64_t first_bucket, uint8_t *q)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    for (uint64_t b = 0; b < nb; b++) {
        uint32_t k0, k1;
        nuqo_rng_key(seed, first_bucket + b, &k0, &k1);
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        for (uint64_t i = lo; i < hi; i++) {
            uint32_t u = nuqo_rng_u24(k0, k1, (uint32_t)(i - lo));
            int j = nuqo_quantize_coord_table(v[i], norms[b], s, lev, u);
            uint8_t sign = (j > 0 && signbit(v[i])) ? 0x80 : 0;
            q[i] = (uint8_t)j | sign;
        }
    }
}

/* --------------------------------------------------------------------- ERC */

/*
 * Alg. 2, encoder.  The code of N is: the binary expansions of N, of
 * (bits(N) - 1), of (bits of that - 1), ... down to (but excluding) 1, written
 * last-computed first, then a single 0.  Writes '0'/'1' characters into `out`
 * (at least 64 bytes), returns the length.
 */
static int bit_width(uint64_t x)
{
    int w = 0;
    while (x) {
        w++;
        x >>= 1;
    }
    return w;
}

int nuqo_erc_encode(uint64_t N, char *out)
{
    if (N < 1)
        return NUQO_EINVAL;
    uint64_t groups[8];
    int ng = 0;
    while (N != 1) { /* App. A, Alg. 2: the group binary(N) is preceded by the code groups of its own length - 1 */
        groups[ng++] = N;
        N = (uint64_t)bit_width(N) - 1;
    }
    int len = 0;
    for (int g = ng - 1; g >= 0; g--) { /* the last group computed is the first written */
        int w = bit_width(groups[g]);
        for (int k = w - 1; k >= 0; k--)
            out[len++] = ((groups[g] >> k) & 1) ? '1' : '0';
    }
    out[len++] = '0'; /* App. A, Alg. 2: a single 0 closes the codeword (every group starts with a 1) */
    return len;
}

int nuqo_erc_length(uint64_t N)
{
    char tmp[96];
    return nuqo_erc_encode(N, tmp);
}

/* A bit string held MSB-first in 32-bit words: stream bit t is bit 31-(t&31)
 * of words[t>>5]. */
static inline int get_bit(const uint32_t *words, uint64_t t)
{
    return (int)((words[t >> 5] >> (31 - (t & 31))) & 1u);
}

static inline void put_bit(uint32_t *words, uint64_t t, int bit)
{
    if (bit)
        words[t >> 5] |= 1u << (31 - (t & 31));
}

/*
 * App. A, Alg. 2, decoder, reading from bit `*pos` and never at or beyond `end`.
 * The value so far (1 at first) is the number of bits that follow a group's
 * leading 1; a 0 where a group would start ends the codeword and the value so far
 * is the result.  Returns 0 on success, NUQO_EMALFORMED
 * if the code runs past `end` or N leaves the 32-bit range.
 */
int nuqo_erc_decode(const uint32_t *words, uint64_t *pos, uint64_t end, uint64_t *N_out)
{
    uint64_t N = 1, t = *pos;
    for (;;) {
        if (t >= end)
            return NUQO_EMALFORMED;
        if (get_bit(words, t) == 0) {
            *pos = t + 1;
            *N_out = N;
            return NUQO_OK;
        }
        if (N + 1 > 33 || t + N + 1 > end)
            return NUQO_EMALFORMED;
        uint64_t val = 0;
        for (uint64_t k = 0; k < N + 1; k++)
            val = (val << 1) | (uint64_t)get_bit(words, t + k);
        t += N + 1;
        N = val;
    }
}

/* ------------------------------------------------------------------ ENCODE */

/*
 * Decoder index (this project's addition to the message; the bit strings do not
 * depend on it).  A bucket is cut into blocks of NUQO_SYNC_BLOCK = 2048
 * coordinates and the records of every block into P pieces of equal count, so
 * that a parallel decoder can hand the pieces of a block to threads that all get
 * the same number of records.  P = the smallest power of two that is at least
 * min(bucket, 2048) / sync_stride: sync_stride is the mean number of coordinates
 * per piece.  A bucket has nblk * P entries, nblk = ceil(bucket / 2048).
 */
#define NUQO_SYNC_BLOCK 2048u

static uint32_t sync_pieces(uint32_t bucket, uint32_t sync_stride)
{
    uint32_t span = bucket < NUQO_SYNC_BLOCK ? bucket : NUQO_SYNC_BLOCK;
    uint32_t need = (span + sync_stride - 1) / sync_stride, P = 1;
    while (P < need)
        P *= 2;
    return P;
}

uint64_t nuqo_num_sync(uint32_t bucket, uint32_t sync_stride)
{
    if (sync_stride == 0 || bucket == 0)
        return 0;
    return (uint64_t)((bucket + NUQO_SYNC_BLOCK - 1) / NUQO_SYNC_BLOCK) * sync_pieces(bucket, sync_stride);
}

/* Index entries per bucket of the Huffman-coded message: one per multiple of the stride inside the bucket. */
static uint64_t num_sync_coords(uint32_t bucket, uint32_t sync_stride)
{
    if (sync_stride == 0)
        return 0;
    return (bucket + sync_stride - 1) / sync_stride - 1;
}

/*
 * ENCODE (App. A) of every bucket of q into one word array.
 *
 * Per bucket (the bucket is the paper's vector v; its 32-bit norm travels in the
 * norms array next to the bit string): scan coordinates in index order; for
 * every nonzero h emit ERC(gap) where gap = index - previous nonzero index
 * (indices 1-based with t_0 = 0, so the first gap is the 1-based position),
 * then one sign bit (1 = negative), then ERC(log2(2^(s+1) h)) = ERC(j), j the
 * level index.  Nothing is emitted after the last nonzero.
 *
 * Layout: bit_off[0] = 0.  Bucket b's records start at the first 32-bit
 * boundary at or after bit_off[b] and end (exclusive) at bit_off[b+1]; pad bits
 * are zero.  words must hold words_cap zero-initialised entries on entry.
 *
 * sync (may be NULL when sync_stride == 0), nsync = nuqo_num_sync entries per
 * bucket: number the bucket's records 0 .. N-1 in index order; block t holds
 * the n_t records whose index is in [2048 t, 2048 (t+1)), the first of them
 * being record f_t (f_t = number of records before the block).  Entry (t, g),
 * g = 0 .. P-1, stored at sync[b*nsync + t*P + g], describes record
 * r = f_t + floor(g * n_t / P): bits 0..20 = bit offset of record r from the
 * bucket's first bit (the bucket's bit length if r = N); bits 21..31 = index of
 * record r minus 2048 t if n_t > 0, else 0.  Piece (t, g) is the records from
 * entry (t, g)'s up to, not including, the next entry's (entry (t, g+1), or
 * (t+1, 0), or the bucket's end): floor((g+1) n_t / P) - floor(g n_t / P) of them.
 *
 * Returns 0, or NUQO_ECAPACITY if words_cap is too small, NUQO_EINVAL on bad
 * arguments or a level index above s+1.
 */
int nuqo_encode(const uint8_t *q, uint64_t d, uint32_t bucket, int s, uint32_t sync_stride,
                uint64_t *bit_off, uint32_t *words, uint64_t words_cap, uint32_t *sync)
{
    if (d == 0 || bucket == 0 || s < 1)
        return NUQO_EINVAL;
    if (sync_stride != 0 && (sync_stride > 1024 || (sync_stride & (sync_stride - 1))))
        return NUQO_EINVAL;
    uint64_t nb = (d + bucket - 1) / bucket;
    uint64_t nsync = nuqo_num_sync(bucket, sync_stride);
    uint32_t P = nsync ? sync_pieces(bucket, sync_stride) : 0;
    uint64_t *rec_idx = NULL, *rec_off = NULL; /* index and bit offset of the bucket's records, for the entries */
    if (nsync) {
        rec_idx = (uint64_t *)malloc(sizeof(uint64_t) * bucket);
        rec_off = (uint64_t *)malloc(sizeof(uint64_t) * bucket);
        if (!rec_idx || !rec_off) {
            free(rec_idx);
            free(rec_off);
            return NUQO_EINVAL;
        }
    }
    int rc = NUQO_OK;
    uint64_t end_prev = 0;
    bit_off[0] = 0;
    char code[96];
    for (uint64_t b = 0; b < nb && rc == NUQO_OK; b++) {
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        uint64_t start = (end_prev + 31) / 32 * 32;
        uint64_t t = start;
        int64_t prev = -1; /* 0-based index of the previous nonzero; t_0 = 0 in 1-based terms */
        uint64_t N = 0;    /* records so far */
        for (uint64_t i = lo; i < hi; i++) {
            int j = q[i] & 0x7f;
            if (j == 0)
                continue;
            if (j > s + 1) {
                rc = NUQO_EINVAL;
                break;
            }
            int64_t idx = (int64_t)(i - lo);
            uint64_t gap = (uint64_t)(idx - prev);
            int glen = nuqo_erc_encode(gap, code);
            int jlen = nuqo_erc_encode((uint64_t)j, code + glen + 1);
            code[glen] = (q[i] & 0x80) ? '1' : '0';
            int len = glen + 1 + jlen;
            if ((t + len + 31) / 32 > words_cap) {
                rc = NUQO_ECAPACITY;
                break;
            }
            if (nsync) {
                rec_idx[N] = (uint64_t)idx;
                rec_off[N] = t - start;
            }
            N++;
            for (int k = 0; k < len; k++)
                put_bit(words, t + k, code[k] == '1');
            t += len;
            prev = idx;
        }
        if (rc != NUQO_OK)
            break;
        uint64_t next = 0; /* first record not yet assigned to a block (records are in index order) */
        for (uint64_t blk = 0; nsync && blk < nsync / P; blk++) {
            uint64_t f = next; /* records before the block */
            while (next < N && rec_idx[next] < (blk + 1) * NUQO_SYNC_BLOCK)
                next++;
            uint64_t n = next - f; /* records inside it */
            for (uint64_t g = 0; g < P; g++) {
                uint64_t r = f + g * n / P;
                uint64_t off = r < N ? rec_off[r] : t - start;
                uint64_t rel = n > 0 ? rec_idx[r] - blk * NUQO_SYNC_BLOCK : 0;
                sync[b * nsync + blk * P + g] = (uint32_t)(off | (rel << 21));
            }
        }
        bit_off[b + 1] = t;
        end_prev = t;
    }
    free(rec_idx);
    free(rec_off);
    return rc;
}

/* ------------------------------------------------------------------ DECODE */

/*
 * DECODE (App. A) of one worker's bit strings into q (level | sign<<7 per
 * coordinate): per bucket read ERC^-1 -> gap, one sign bit, ERC^-1 -> level
 * index, until the bucket's bits are used up.  Returns NUQO_EMALFORMED if a
 * record crosses the bucket's end, an index leaves the bucket, or a level
 * index is outside 1..s+1.
 */
int nuqo_decode_levels(const uint64_t *bit_off, const uint32_t *words, uint64_t d,
                       uint32_t bucket, int s, uint8_t *q)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    memset(q, 0, d);
    for (uint64_t b = 0; b < nb; b++) {
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        uint64_t t = (bit_off[b] + 31) / 32 * 32, end = bit_off[b + 1];
        if (end < t)
            return NUQO_EMALFORMED;
        int64_t prev = -1;
        while (t < end) {
            uint64_t gap, j;
            int rc = nuqo_erc_decode(words, &t, end, &gap);
            if (rc)
                return rc;
            if (t >= end)
                return NUQO_EMALFORMED;
            int neg = get_bit(words, t++);
            rc = nuqo_erc_decode(words, &t, end, &j);
            if (rc)
                return rc;
            int64_t idx = prev + (int64_t)gap;
            if (idx >= (int64_t)(hi - lo) || j < 1 || j > (uint64_t)s + 1)
                return NUQO_EMALFORMED;
            q[lo + idx] = (uint8_t)j | (neg ? 0x80 : 0);
            prev = idx;
        }
    }
    return NUQO_OK;
}

/*
 * DECODE each of K workers, rebuild Q_s(v) = ||v|| * sign * l_j (Def. 1), and
 * aggregate as in Alg. 1: out = [out +] scale * sum_k Q_k, fp64, workers in
 * order.  out64 has d entries; if accumulate is zero it is overwritten.
 */
static int decode_average_any(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                              const uint32_t *const *words, uint64_t d, uint32_t bucket, int s,
                              const float *lev, double scale, int accumulate, double *out64)
{
    uint8_t *q = (uint8_t *)malloc(d);
    double *sum = (double *)calloc(d, sizeof(double));
    if (!q || !sum) {
        free(q);
        free(sum);
        return NUQO_EINVAL;
    }
    for (uint32_t k = 0; k < K; k++) {
        int rc = nuqo_decode_levels(bit_off[k], words[k], d, bucket, s, q);
        if (rc) {
            free(q);
            free(sum);
            return rc;
        }
        for (uint64_t i = 0; i < d; i++) {
            int j = q[i] & 0x7f;
            if (j == 0)
                continue;
            double h = lev ? (double)lev[j] : ldexp(1.0, j - 1 - s); /* l_j */
            double val = (double)norms[k][i / bucket] * h;
            sum[i] += (q[i] & 0x80) ? -val : val;
        }
    }
    for (uint64_t i = 0; i < d; i++)
        out64[i] = (accumulate ? out64[i] : 0.0) + scale * sum[i];
    free(q);
    free(sum);
    return NUQO_OK;
}

int nuqo_decode_average(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                        const uint32_t *const *words, uint64_t d, uint32_t bucket, int s,
                        double scale, int accumulate, double *out64)
{
    return decode_average_any(K, norms, bit_off, words, d, bucket, s, NULL, scale, accumulate, out64);
}

/* The same with Q(v_i) = ||v|| * sign * lev[j] for an arbitrary level sequence lev[0..s+1]. */
int nuqo_decode_average_table(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                              const uint32_t *const *words, uint64_t d, uint32_t bucket, int s,
                              const float *lev, double scale, int accumulate, double *out64)
{
    return decode_average_any(K, norms, bit_off, words, d, bucket, s, lev, scale, accumulate, out64);
}

/* ------------------------------------------------------- fixed-width coding */

/*
 * Fixed-width message (Sec. 5, "4-bit"/"8-bit" variants): coordinate i of a
 * bucket is the b-bit code  sign << (b-1) | level index  (level index < 2^(b-1),
 * so s + 2 <= 2^(b-1); a zero level carries sign 0), at bits [i*b, i*b + b) of the
 * bucket's field, most significant bit first, in 32-bit words as in ENCODE.
 * Every bucket's field is wpb = ceil(bucket * b / 32) words (the last, short
 * bucket too; unused bits are 0), so bucket k starts at word k * wpb.
 */
uint64_t nuqo_fixed_words(uint64_t d, uint32_t bucket, uint32_t b)
{
    uint64_t nb = (d + bucket - 1) / bucket;
    return nb * (((uint64_t)bucket * b + 31) / 32);
}

int nuqo_pack_fixed(const uint8_t *q, uint64_t d, uint32_t bucket, int s, uint32_t b, uint32_t *packed)
{
    if (b < 2 || b > 8 || (uint32_t)(s + 2) > (1u << (b - 1)))
        return NUQO_EINVAL;
    uint64_t nb = (d + bucket - 1) / bucket, wpb = ((uint64_t)bucket * b + 31) / 32;
    memset(packed, 0, nb * wpb * sizeof(uint32_t));
    for (uint64_t k = 0; k < nb; k++) {
        uint64_t lo = k * bucket, hi = lo + bucket < d ? lo + bucket : d;
        for (uint64_t i = lo; i < hi; i++) {
            uint32_t level = q[i] & 0x7f, neg = q[i] >> 7;
            if (level > (uint32_t)s + 1 || (level == 0 && neg))
                return NUQO_EINVAL;
            uint32_t code = (neg << (b - 1)) | level;
            for (uint32_t t = 0; t < b; t++) /* most significant bit of the code first */
                put_bit(packed + k * wpb, (i - lo) * b + t, (code >> (b - 1 - t)) & 1);
        }
    }
    return NUQO_OK;
}

int nuqo_unpack_fixed(const uint32_t *packed, uint64_t d, uint32_t bucket, int s, uint32_t b, uint8_t *q)
{
    if (b < 2 || b > 8 || (uint32_t)(s + 2) > (1u << (b - 1)))
        return NUQO_EINVAL;
    uint64_t nb = (d + bucket - 1) / bucket, wpb = ((uint64_t)bucket * b + 31) / 32;
    for (uint64_t k = 0; k < nb; k++) {
        uint64_t lo = k * bucket, hi = lo + bucket < d ? lo + bucket : d;
        for (uint64_t i = lo; i < hi; i++) {
            uint32_t code = 0;
            for (uint32_t t = 0; t < b; t++)
                code = (code << 1) | (uint32_t)get_bit(packed + k * wpb, (i - lo) * b + t);
            uint32_t level = code & ((1u << (b - 1)) - 1u), neg = code >> (b - 1);
            if (level > (uint32_t)s + 1 || (level == 0 && neg))
                return NUQO_EMALFORMED;
            q[i] = (uint8_t)(level | (neg << 7));
        }
    }
    return NUQO_OK;
}

/* ----------------------------------------------------- Huffman-coded levels */

/*
 * Code lengths for the level indices 0..s+1 from a histogram (Sec. 5: the code is built from
 * an initial sample and then kept).  Huffman's algorithm on the weights hist[j] + 1 (so that a
 * level the sample never showed still has a code): repeatedly merge the two smallest nodes,
 * nodes ordered by (weight, id), a leaf's id being its symbol, the k-th merged node's id being
 * nsym + k.  The length of a symbol is its depth.  nsym = s + 2 <= 16, so lengths are <= 15.
 */
int nuqo_huffman_lengths(const uint64_t *hist, int s, uint8_t *lengths)
{
    int nsym = s + 2;
    if (s < 1 || nsym > 16)
        return NUQO_EINVAL;
    uint64_t weight[32];
    int parent[32], alive[32];
    for (int j = 0; j < nsym; j++) {
        weight[j] = hist[j] + 1;
        parent[j] = -1;
        alive[j] = 1;
    }
    int nodes = nsym;
    for (int step = 0; step < nsym - 1; step++) {
        int a = -1, b = -1; /* smallest and second smallest by (weight, id): ids ascend with the index */
        for (int i = 0; i < nodes; i++) {
            if (!alive[i])
                continue;
            if (a < 0 || weight[i] < weight[a]) {
                b = a;
                a = i;
            } else if (b < 0 || weight[i] < weight[b]) {
                b = i;
            }
        }
        weight[nodes] = weight[a] + weight[b];
        parent[nodes] = -1;
        alive[nodes] = 1;
        alive[a] = alive[b] = 0;
        parent[a] = parent[b] = nodes;
        nodes++;
    }
    for (int j = 0; j < nsym; j++) {
        int depth = 0;
        for (int i = j; parent[i] >= 0; i = parent[i])
            depth++;
        lengths[j] = (uint8_t)depth;
    }
    return NUQO_OK;
}

/*
 * Canonical code for given lengths: symbols in order of (length, symbol); the first gets
 * code 0, each next one (previous code + 1) shifted left by the increase in length.
 */
int nuqo_huffman_codes(const uint8_t *lengths, int s, uint32_t *codes)
{
    int nsym = s + 2;
    uint32_t code = 0;
    int prev_len = 0, first = 1;
    for (int len = 1; len <= 15; len++)
        for (int j = 0; j < nsym; j++) {
            if (lengths[j] != len)
                continue;
            if (!first)
                code = (code + 1) << (len - prev_len);
            first = 0;
            prev_len = len;
            codes[j] = code;
        }
    /* a complete code: the last codeword is all ones */
    return (!first && code == (1u << prev_len) - 1u) ? NUQO_OK : NUQO_EINVAL;
}

/*
 * Message of the level|sign bytes q: per bucket, for every coordinate in order, the codeword of
 * its level index (most significant bit first) followed, when the level is not zero, by its sign
 * bit.  bit_off, words and alignment as in nuqo_encode.  sync entry (b, g), g = 1..nsync: the
 * bit offset, from the bucket's start, of coordinate g * sync_stride.
 */
int nuqo_encode_huffman(const uint8_t *q, uint64_t d, uint32_t bucket, int s, uint32_t sync_stride,
                        const uint8_t *lengths, uint64_t *bit_off, uint32_t *words, uint64_t words_cap,
                        uint32_t *sync)
{
    uint32_t codes[16];
    if (nuqo_huffman_codes(lengths, s, codes))
        return NUQO_EINVAL;
    uint64_t nb = (d + bucket - 1) / bucket, nsync = num_sync_coords(bucket, sync_stride);
    uint64_t t = 0;
    memset(words, 0, words_cap * sizeof(uint32_t));
    bit_off[0] = 0;
    for (uint64_t b = 0; b < nb; b++) {
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        t = (t + 31) / 32 * 32;
        uint64_t start = t;
        for (uint64_t g = 1; g <= nsync; g++)
            sync[b * nsync + g - 1] = 0;
        for (uint64_t i = lo; i < hi; i++) {
            uint32_t level = q[i] & 0x7f, neg = q[i] >> 7;
            if (level > (uint32_t)s + 1 || (level == 0 && neg))
                return NUQO_EINVAL;
            if (sync_stride && (i - lo) % sync_stride == 0 && i > lo)
                sync[b * nsync + (i - lo) / sync_stride - 1] = (uint32_t)(t - start);
            uint32_t need = lengths[level] + (level ? 1u : 0u);
            if ((t + need + 31) / 32 > words_cap)
                return NUQO_ECAPACITY;
            for (int k = lengths[level] - 1; k >= 0; k--)
                put_bit(words, t++, (codes[level] >> k) & 1);
            if (level)
                put_bit(words, t++, (int)neg);
        }
        for (uint64_t g = 1; g <= nsync; g++) /* boundaries at or beyond a short last bucket's end: its end */
            if (g * sync_stride >= hi - lo)
                sync[b * nsync + g - 1] = (uint32_t)(t - start);
        bit_off[b + 1] = t;
    }
    return NUQO_OK;
}

/* Back to level|sign bytes, bit by bit: walk the canonical code one length at a time. */
int nuqo_decode_huffman(const uint64_t *bit_off, const uint32_t *words, uint64_t d, uint32_t bucket, int s,
                        const uint8_t *lengths, uint8_t *q)
{
    uint32_t codes[16];
    if (nuqo_huffman_codes(lengths, s, codes))
        return NUQO_EINVAL;
    int nsym = s + 2;
    uint64_t nb = (d + bucket - 1) / bucket;
    for (uint64_t b = 0; b < nb; b++) {
        uint64_t lo = b * bucket, hi = lo + bucket < d ? lo + bucket : d;
        uint64_t t = (bit_off[b] + 31) / 32 * 32, end = bit_off[b + 1];
        for (uint64_t i = lo; i < hi; i++) {
            uint32_t prefix = 0;
            int len = 0, level = -1;
            while (level < 0) {
                if (t >= end || len == 15)
                    return NUQO_EMALFORMED;
                prefix = (prefix << 1) | (uint32_t)get_bit(words, t++);
                len++;
                for (int j = 0; j < nsym; j++)
                    if (lengths[j] == len && codes[j] == prefix)
                        level = j;
            }
            int neg = 0;
            if (level) {
                if (t >= end)
                    return NUQO_EMALFORMED;
                neg = get_bit(words, t++);
            }
            q[i] = (uint8_t)(level | (neg << 7));
        }
        if (t != end)
            return NUQO_EMALFORMED;
    }
    return NUQO_OK;
}
