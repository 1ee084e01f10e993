/*
 * nuq.h -- C ABI of the NUQSGD gradient-compression hot path for AMD MI355X (gfx950).
 *
 * The path (arXiv 1908.06077): per-bucket Euclidean norms -> nonuniform stochastic
 * quantization of |v_i|/||v|| onto the levels (0, 2^-s, ..., 1/2, 1) with sign
 * (Sec. 3.1, Def. 1) -> ENCODE into Elias-recursive-coded bit strings (App. A,
 * Alg. 2) -> DECODE, dequantize and average K workers' gradients (App. A; the
 * aggregate line of Alg. 1).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless the
 *     comment says "host".  The library never frees or keeps them.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work and
 *     return without synchronising, except nuq_last_error_flags.
 *   - Return value: NUQ_OK or a negative NUQ_E* code.  Argument errors are detected
 *     on the host before anything is enqueued.  Conditions only visible on the device
 *     (capacity overflow, non-finite norm, malformed stream) set sticky device flags
 *     read back with nuq_last_error_flags.
 *   - d = number of coordinates (>= 1), bucket = bucket size n (1..NUQ_MAX_BUCKET),
 *     B = ceil(d / bucket) buckets, bucket b covers [b*n, min((b+1)*n, d)),
 *     s = number of internal levels (1..NUQ_MAX_S), level index j in 0..s+1 with
 *     l_0 = 0 and l_j = 2^(j-1-s).
 *
 * Message layout produced by nuq_encode / nuq_quantize_encode (one per worker):
 *   norms[B]      fp32 bucket norms (the 32-bit ||v|| of App. A, kept beside the bits).
 *   bit_off[B+1]  u64.  bit_off[0] = 0.  Bucket b's records are stream bits
 *                 [start_b, bit_off[b+1]) with start_b = bit_off[b] rounded up to a
 *                 multiple of 32.
 *   words[W]      u32, W = ceil(bit_off[B] / 32).  Stream bit t is bit 31-(t%32) of
 *                 words[t/32].  Pad bits are zero.
 *   sync[B*nsync] u32 decoder index (this library's addition to the paper's message; the bit
 *                 strings do not depend on it), nsync = nuq_num_sync(bucket, sync_stride).  A bucket
 *                 is cut into blocks of NUQ_SYNC_BLOCK = 2048 coordinates and the records of every
 *                 block into P pieces of equal record count, P = the smallest power of two that is
 *                 at least min(bucket, 2048) / sync_stride (sync_stride = mean coordinates per
 *                 piece); nsync = ceil(bucket / 2048) * P.  With the bucket's records numbered in
 *                 index order, block t holding n_t of them from record f_t on, entry (t, g),
 *                 g = 0..P-1, stored at sync[b*nsync + t*P + g], describes record
 *                 f_t + floor(g * n_t / P): bits 0..20 = its bit offset from start_b (the bucket's
 *                 bit length if the bucket has no such record), bits 21..31 = its in-bucket index
 *                 minus 2048 t (0 if n_t = 0).  Piece (t, g) = the records from its entry's up to
 *                 the next entry's (or the bucket's end): a decoder parses every piece on its own,
 *                 taking the first record's index from the entry instead of from its gap code.
 *   A record, for a nonzero at in-bucket index i whose previous nonzero is at i_prev
 *   (-1 if none): ERC(i - i_prev), one sign bit (1 = negative), ERC(j).
 */
#ifndef NUQ_H
#define NUQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *nuq_stream_t; /* hipStream_t */

enum {
    NUQ_OK = 0,
    NUQ_EINVAL = -1,     /* bad argument (size, range, NULL, misaligned)            */
    NUQ_ECAPACITY = -2,  /* a caller-provided buffer is too small (host-detectable) */
    NUQ_ENONFINITE = -3, /* reserved for host-side checks                           */
    NUQ_EHIP = -4        /* a HIP runtime call failed                               */
};

/* Sticky device flags (nuq_last_error_flags). */
enum {
    NUQ_FLAG_CAPACITY = 1,  /* encoded words did not fit words_cap; words is incomplete */
    NUQ_FLAG_NONFINITE = 2, /* a bucket norm was Inf/NaN; that bucket was encoded empty */
    NUQ_FLAG_MALFORMED = 4  /* a decoded stream broke the format; output is incomplete  */
};

/* A bucket's coordinates stay in the registers of one workgroup between the norm and the quantizer, so
 * that v is read from memory once: the largest workgroup (1024 threads) x 8 float4 = 32768 coordinates.
 * (The paper's bucket sizes are 8192 and 16384: Sec. 5, App. K.) */
#define NUQ_MAX_BUCKET 32768u
#define NUQ_MAX_S 14u
#define NUQ_MAX_WORKERS 32u /* K per nuq_decode_accumulate call */
#define NUQ_SYNC_BLOCK 2048u /* coordinates per block of the decoder index */

/* ---- sizes (pure host arithmetic, no device work) -------------------------------- */

/* B = ceil(d / bucket); 0 if bucket == 0. */
uint64_t nuq_num_buckets(uint64_t d, uint32_t bucket);

/* Decoder index entries per bucket of an ERC message: 0 if sync_stride == 0 (or not a power of two in
 * 64..1024), else ceil(bucket / 2048) * P with P as above. */
uint32_t nuq_num_sync(uint32_t bucket, uint32_t sync_stride);

/* The same for a Huffman-coded message (an entry per multiple of sync_stride inside the bucket):
 * 0 if sync_stride == 0, else ceil(bucket / sync_stride) - 1. */
uint32_t nuq_huffman_num_sync(uint32_t bucket, uint32_t sync_stride);

/* Upper bound on W for any input: every coordinate nonzero at the longest level code,
 * i.e. d * (2 + |ERC(s+1)|) bits, plus one word of padding per bucket. */
uint64_t nuq_max_words(uint64_t d, uint32_t bucket, uint32_t s);

/* Bytes of scratch the encoders need for K workers of these sizes (K = 1 for nuq_encode and
 * nuq_quantize_encode); 0 on invalid sizes. */
uint64_t nuq_encode_workspace_bytes(uint32_t K, uint64_t d, uint32_t bucket, uint32_t s);

/* Bytes of scratch that suffice for every entry point of this header at these sizes, whatever s:
 * nuq_encode_workspace_bytes(K, d, bucket, NUQ_MAX_S) (the decoders need none); 0 on invalid sizes. */
uint64_t nuq_workspace_bytes(uint64_t d, uint32_t bucket, uint32_t K);

/* ---- step 1: bucket norms (Def. 1: r_i = |v_i| / ||v||) --------------------------- */

/* norms[b] = sqrt(sum of v_i^2 over bucket b), rounded to fp32.
 * v: d floats, 4-byte aligned (16-byte alignment with bucket % 4 == 0 takes the
 * vector-load path).  norms: B floats. */
int nuq_bucket_norms(const float *v, uint64_t d, uint32_t bucket, float *norms,
                     nuq_stream_t stream);

/* ---- step 2: quantizer (Def. 1; App. B eqs. h_case1, h_case2) --------------------- */

/* q[i] = level index j (bits 0..6) | sign (bit 7, 1 = negative, only if j > 0).
 * With r = |v_i| / norms[b] in bin [l_j, l_{j+1}) the result is j+1 with probability
 * p = (r - l_j) / (l_{j+1} - l_j), else j; the draw is the counter hash of
 * (seed, b, index in bucket) (24 uniform bits, "up" iff u / 2^24 < p, evaluated
 * exactly).  r >= 1 gives s+1; a zero norm or coordinate gives 0.
 * norms: B floats, normally the output of nuq_bucket_norms.  q: d bytes. */
int nuq_quantize(const float *v, uint64_t d, uint32_t bucket, uint32_t s, uint64_t seed,
                 const float *norms, uint8_t *q, nuq_stream_t stream);

/* ---- step 3: ENCODE (App. A; Alg. 2) ------------------------------------------------ */

/* Encodes the level/sign bytes q[d] into bit_off[B+1], words[<= words_cap] and, when
 * sync_stride != 0, sync[B*nsync] (sync may be NULL when sync_stride == 0).
 * sync_stride: 0, or a power of two in 64..1024.
 * workspace: at least nuq_encode_workspace_bytes(1, d, bucket, s) bytes, 16-byte aligned;
 * contents are scratch.  If the encoded size exceeds words_cap the device flag
 * NUQ_FLAG_CAPACITY is raised, bit_off is still complete and words holds the buckets
 * that fit.  A level index above s+1 in q is a caller error (undefined bits). */
int nuq_encode(const uint8_t *q, uint64_t d, uint32_t bucket, uint32_t s, uint32_t sync_stride,
               uint64_t *bit_off, uint32_t *words, uint64_t words_cap, uint32_t *sync,
               void *workspace, uint64_t workspace_bytes, nuq_stream_t stream);

/* Steps 1-3 fused: v is read from memory once.  Outputs norms[B] as nuq_bucket_norms
 * would, and bit_off / words / sync exactly as nuq_encode(nuq_quantize(v, norms)) would.
 * A bucket whose norm is not finite is encoded as empty and raises NUQ_FLAG_NONFINITE. */
int nuq_quantize_encode(const float *v, uint64_t d, uint32_t bucket, uint32_t s, uint64_t seed,
                        uint32_t sync_stride, float *norms, uint64_t *bit_off, uint32_t *words,
                        uint64_t words_cap, uint32_t *sync, void *workspace,
                        uint64_t workspace_bytes, nuq_stream_t stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): nuq_quantize_encode with the workspace in a device array that is part of
 * the library itself, NUQ_STATIC_WORKSPACE_BYTES per GPU, held from the library's load to the end of
 * the process.  Same arguments otherwise, same kernels, same outputs bit for bit.  The call allocates
 * and frees nothing; its first call on a device looks the array's address up (make that call outside a
 * capture).  Sizes with nuq_encode_workspace_bytes(1, d, bucket, s) > NUQ_STATIC_WORKSPACE_BYTES are
 * rejected with NUQ_ECAPACITY before anything is enqueued (bucket 8192, s <= 5: up to 33.5 M
 * coordinates).  All calls on one GPU share the one array: calls that overlap in time (different
 * streams, or threads) race; calls on one stream do not.  Nothing in it has to be cleared between
 * calls: every word a call reads was written by that call. */
#define NUQ_STATIC_WORKSPACE_BYTES (32u << 20)
int nuq_quantize_encode_static(const float *v, uint64_t d, uint32_t bucket, uint32_t s, uint64_t seed,
                               uint32_t sync_stride, float *norms, uint64_t *bit_off, uint32_t *words,
                               uint64_t words_cap, uint32_t *sync, nuq_stream_t stream);

/* The same for K workers' gradients in one launch (the K simulated workers of Alg. 1 on one
 * device).  v, norms, bit_off, words, sync: HOST arrays of K device pointers; seeds, words_cap:
 * HOST arrays of K values.  Worker k's message equals what
 * nuq_quantize_encode(v[k], ..., seeds[k], ...) produces.  1 <= K <= NUQ_MAX_WORKERS.
 * workspace: at least nuq_encode_workspace_bytes(K, d, bucket, s) bytes. */
int nuq_quantize_encode_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                              uint32_t bucket, uint32_t s, uint32_t sync_stride, float *const *norms,
                              uint64_t *const *bit_off, uint32_t *const *words,
                              const uint64_t *words_cap, uint32_t *const *sync, void *workspace,
                              uint64_t workspace_bytes, nuq_stream_t stream);

/* ---- step 4: DECODE + dequantize + aggregate (App. A DECODE; Alg. 1 aggregate) ------ */

/* out[i] = (accumulate ? out[i] : 0) + scale * sum_k norms_k[b] * sign * l_j, where
 * (sign, j) of coordinate i is decoded from worker k's bit string (0 if absent).
 * norms, bit_off, words, sync: HOST arrays of K device pointers (one message per
 * worker, all encoded with the same d, bucket, s, sync_stride); sync may be NULL or hold
 * NULLs when sync_stride == 0.  words_len: HOST array of K counts, the u32 words that
 * words[k] holds (as received).  1 <= K <= NUQ_MAX_WORKERS; average with scale = 1/K.
 * The sum over workers is taken in fp64 (in no fixed order, which cannot change it unless the
 * terms' exponents span more than 2^29), scaled in fp64 and rounded to fp32 once; with accumulate the
 * old out[i] is then added in fp32.  out: d floats.
 * A record that leaves its bucket's bit range or index range, a level index outside 1..s+1, or a
 * sync entry that contradicts the bit offsets raises NUQ_FLAG_MALFORMED and ends that part's
 * decoding.  So does a bucket whose offsets run backwards (bit_off[b+1] < bit_off[b]), end beyond
 * the words received (bit_off[b+1] > 32 * words_len[k]) or span 2^21 bits or more: such a bucket
 * contributes nothing and no word of it is read, so a cut-off or corrupted message cannot make the
 * kernels read outside words[k].  (norms, bit_off and sync are sized by d, bucket and sync_stride,
 * which the caller vouches for.) */
int nuq_decode_accumulate(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                          const uint32_t *const *words, const uint64_t *words_len,
                          const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                          uint32_t sync_stride, float scale, int accumulate, float *out,
                          nuq_stream_t stream);

/* ---- other level sequences and the maximum norm (Sec. 3.1 before the special case; Sec. 4.1,
 *      "Generally spaced levels": exponential levels (0, p^s, ..., p, 1); uniform levels = QSGD,
 *      with the maximum norm = QSGDinf, Sec. 1 and Sec. 2) ------------------------------------ */

#define NUQ_NORM_L2 0u   /* Euclidean norm of the bucket */
#define NUQ_NORM_LINF 1u /* maximum norm of the bucket   */

/* A level table is s + 2 floats in HOST memory, 0 = levels[0] < levels[1] < ... < levels[s+1] = 1
 * (anything else: NUQ_EINVAL).  It is read during the call. */

/* norms[b] = max_i |v_i| over bucket b (exact; NaN if the bucket holds a NaN).  Arguments as
 * nuq_bucket_norms. */
int nuq_bucket_norms_linf(const float *v, uint64_t d, uint32_t bucket, float *norms,
                          nuq_stream_t stream);

/* nuq_quantize for the level sequence `levels`: with e_t = levels[t] * norms[b] and a = |v_i|,
 * j = largest t with e_t <= a (j = s+1: the top level), else j+1 iff
 * u * (e_{j+1} - e_j) < (a - e_j) * 2^24, evaluated as exactly that sequence of IEEE fp64 operations
 * (the products e_t are exact; the two differences and the product with u round to nearest), u the
 * 24-bit draw of nuq_quantize.  For levels[t] = 2^(t-1-s) nothing rounds and q equals nuq_quantize's.
 * norms may come from nuq_bucket_norms or nuq_bucket_norms_linf; a zero or non-finite norm gives an
 * all-zero bucket.  q feeds nuq_encode unchanged (a level index is coded the same way whatever its
 * value). */
int nuq_quantize_table(const float *v, uint64_t d, uint32_t bucket, uint32_t s, const float *levels,
                       uint64_t seed, const float *norms, uint8_t *q, nuq_stream_t stream);

/* nuq_quantize_encode_batch for the level sequence `levels` and the norm `norm_kind` (NUQ_NORM_L2:
 * as nuq_bucket_norms; NUQ_NORM_LINF: as nuq_bucket_norms_linf): v is read once; worker k's norms are
 * what the norm entry point gives and its message is what
 * nuq_encode(nuq_quantize_table(v[k], ..., levels, seeds[k], norms[k])) gives.  Other arguments as
 * nuq_quantize_encode_batch. */
int nuq_quantize_encode_table_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                    uint32_t bucket, uint32_t s, const float *levels, uint32_t norm_kind,
                                    uint32_t sync_stride, float *const *norms, uint64_t *const *bit_off,
                                    uint32_t *const *words, const uint64_t *words_cap,
                                    uint32_t *const *sync, void *workspace, uint64_t workspace_bytes,
                                    nuq_stream_t stream);

/* nuq_decode_accumulate with l_j = levels[j]: out[i] = (accumulate ? out[i] : 0) +
 * scale * sum_k norms_k[b] * sign * levels[j].  Everything else as nuq_decode_accumulate. */
int nuq_decode_accumulate_table(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                                const uint32_t *const *words, const uint64_t *words_len,
                                const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                                uint32_t sync_stride, const float *levels, float scale, int accumulate,
                                float *out, nuq_stream_t stream);

/* ---- fixed-width coding (Sec. 5: the "4-bit" and "8-bit" variants; 3 bits in Table 1) ------------ */

/* Every coordinate sends sign and level index in b bits, 3 <= b <= 8 with s + 2 <= 2^(b-1) (else
 * NUQ_EINVAL).  Message of one worker = norms[B] and packed[nuq_fixed_words(d, bucket, b)] u32:
 * coordinate i of a bucket is the code  sign << (b-1) | level index  at bits [i*b, i*b + b) of the
 * bucket's field, most significant bit first (bit t of a field = bit 31 - t%32 of its word t/32);
 * each bucket's field is ceil(bucket * b / 32) words (the short last bucket's too; unused bits 0). */
uint64_t nuq_fixed_words(uint64_t d, uint32_t bucket, uint32_t b);

/* packed <- the level|sign bytes q[d] (as nuq_quantize writes them). */
int nuq_pack_fixed(const uint8_t *q, uint64_t d, uint32_t bucket, uint32_t s, uint32_t b,
                   uint32_t *packed, nuq_stream_t stream);

/* Norms, quantizer and packing of K workers' gradients in one launch, v read once: norms[k] as
 * nuq_bucket_norms(v[k]) and packed[k] as nuq_pack_fixed(nuq_quantize(v[k], ..., seeds[k], norms[k])).
 * v, norms, packed: HOST arrays of K device pointers; seeds: HOST array.  1 <= K <= NUQ_MAX_WORKERS. */
int nuq_quantize_pack_fixed_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                  uint32_t bucket, uint32_t s, uint32_t b, float *const *norms,
                                  uint32_t *const *packed, nuq_stream_t stream);

/* out[i] = (accumulate ? out[i] : 0) + scale * sum_k norms_k[b] * sign * l_j from K fixed-width
 * messages (HOST arrays of K device pointers): fp64 sum in worker order, rounded to fp32 once.
 * A code with a level index above s+1, or a signed zero, raises NUQ_FLAG_MALFORMED. */
int nuq_unpack_accumulate_fixed(uint32_t K, const float *const *norms, const uint32_t *const *packed,
                                uint64_t d, uint32_t bucket, uint32_t s, uint32_t b, float scale,
                                int accumulate, float *out, nuq_stream_t stream);

/* The two fused calls above for a level sequence `levels` (s + 2 floats in HOST memory, as for
 * nuq_quantize_table) and the norm `norm_kind` (NUQ_NORM_L2 / NUQ_NORM_LINF): the fixed-width coding
 * of QSGD and QSGDinf (Sec. 1, Sec. 2; Sec. 5 compares the schemes at equal bit widths).  norms[k] is
 * what the norm entry point gives, packed[k] = nuq_pack_fixed(nuq_quantize_table(v[k], ..., levels,
 * seeds[k], norms[k])); the receiver sums norms_k[b] * sign * levels[j].  Other arguments, rounding
 * and flags as in the two calls above. */
int nuq_quantize_pack_fixed_table_batch(uint32_t K, const float *const *v, const uint64_t *seeds,
                                        uint64_t d, uint32_t bucket, uint32_t s, const float *levels,
                                        uint32_t norm_kind, uint32_t b, float *const *norms,
                                        uint32_t *const *packed, nuq_stream_t stream);
int nuq_unpack_accumulate_fixed_table(uint32_t K, const float *const *norms,
                                      const uint32_t *const *packed, uint64_t d, uint32_t bucket,
                                      uint32_t s, const float *levels, uint32_t b, float scale,
                                      int accumulate, float *out, nuq_stream_t stream);

/* ---- Huffman-coded levels (Sec. 5, "Efficient Encoding": a Huffman code for the level indices, built
 *      from a sample and then kept) ------------------------------------------------------------------ */

/* hist[0..15] (DEVICE, overwritten) <- how often each level index occurs in the level|sign bytes q[d]. */
int nuq_level_histogram(const uint8_t *q, uint64_t d, uint64_t *hist, nuq_stream_t stream);

/* Host arithmetic.  lengths[0..s+1] <- code lengths from the histogram hist[0..s+1] (both HOST):
 * Huffman's algorithm on hist[j] + 1 (a level the sample never showed still gets a code), merging
 * the two smallest nodes by (weight, id), a leaf's id being its symbol, the k-th merged node's id
 * s + 2 + k.  Lengths are 1..s+1.  The codewords are the canonical ones: symbols by (length, symbol),
 * the first is 0, each next one (previous + 1) shifted left by the increase in length. */
int nuq_huffman_lengths(const uint64_t *hist, uint32_t s, uint8_t *lengths);

/* Capacity that always suffices for nuq_encode_huffman's words, and its workspace size. */
uint64_t nuq_huffman_max_words(uint64_t d, uint32_t bucket);
uint64_t nuq_encode_huffman_workspace_bytes(uint64_t d, uint32_t bucket);

/* Message of the bytes q[d] under the code `lengths` (HOST, s + 2 values; NUQ_EINVAL unless they give a
 * complete prefix code): per bucket, for every coordinate in order, the codeword of its level index
 * (most significant bit first), then its sign bit when the level is not zero.  bit_off[B+1], words,
 * word alignment, capacity flag and workspace alignment as for nuq_encode.  sync[B * nsync],
 * nsync = nuq_huffman_num_sync(bucket, sync_stride): entry (b, g), g = 1..nsync, at sync[b*nsync + g-1]
 * = bit offset, from the bucket's start, of coordinate g * sync_stride (the bucket's bit length where
 * the bucket ends before it). */
int nuq_encode_huffman(const uint8_t *q, uint64_t d, uint32_t bucket, uint32_t s, uint32_t sync_stride,
                       const uint8_t *lengths, uint64_t *bit_off, uint32_t *words, uint64_t words_cap,
                       uint32_t *sync, void *workspace, uint64_t workspace_bytes, nuq_stream_t stream);

/* Norms, quantizer and Huffman coding of K workers' gradients in one launch, v read once: norms[k] as
 * nuq_bucket_norms(v[k]) and the message as nuq_encode_huffman(nuq_quantize(v[k], ..., seeds[k],
 * norms[k])).  Array arguments as nuq_quantize_encode_batch; workspace of at least
 * nuq_encode_huffman_batch_workspace_bytes(K, d, bucket, s) bytes, 16-byte aligned. */
uint64_t nuq_encode_huffman_batch_workspace_bytes(uint32_t K, uint64_t d, uint32_t bucket, uint32_t s);
int nuq_quantize_encode_huffman_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                      uint32_t bucket, uint32_t s, uint32_t sync_stride,
                                      const uint8_t *lengths, float *const *norms, uint64_t *const *bit_off,
                                      uint32_t *const *words, const uint64_t *words_cap,
                                      uint32_t *const *sync, void *workspace, uint64_t workspace_bytes,
                                      nuq_stream_t stream);

/* q[d] <- the level|sign bytes of such a message.  A segment that does not end where the next one
 * starts, a prefix that is no codeword, or a sync entry out of order raises NUQ_FLAG_MALFORMED. */
int nuq_decode_huffman(const uint64_t *bit_off, const uint32_t *words, const uint32_t *sync, uint64_t d,
                       uint32_t bucket, uint32_t s, uint32_t sync_stride, const uint8_t *lengths,
                       uint8_t *q, nuq_stream_t stream);

/* The same for K messages in one launch (bit_off, words, sync, q: HOST arrays of K device pointers;
 * one code for all).  1 <= K <= NUQ_MAX_WORKERS. */
int nuq_decode_huffman_batch(uint32_t K, const uint64_t *const *bit_off, const uint32_t *const *words,
                             const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                             uint32_t sync_stride, const uint8_t *lengths, uint8_t *const *q,
                             nuq_stream_t stream);

/* nuq_decode_accumulate for K Huffman-coded messages (Sec. 5, "Efficient Encoding"; App. A DECODE;
 * Alg. 1 aggregate) in one launch: out[i] = (accumulate ? out[i] : 0) + scale * sum_k norms_k[b] *
 * sign * 2^(j-1-s), (sign, j) decoded from worker k's string; the level|sign bytes are never written.
 * Arguments, summation, rounding and NUQ_FLAG_MALFORMED as nuq_decode_accumulate (words_len included),
 * lengths as nuq_encode_huffman.  Geometry: bucket > sync_stride (the messages carry an index), and
 * the pieces of the K messages of a 2048-coordinate tile must fit the tile's 64 parsing lanes with a
 * power-of-two group of lanes per message: for bucket > 2048, K' * 2048 / sync_stride <= 64 with K' =
 * K rounded up to a power of two (K <= 8 at stride 256); else NUQ_EINVAL, and the caller uses
 * nuq_decode_huffman_batch + nuq_average_levels. */
int nuq_decode_accumulate_huffman(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                                  const uint32_t *const *words, const uint64_t *words_len,
                                  const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                                  uint32_t sync_stride, const uint8_t *lengths, float scale, int accumulate,
                                  float *out, nuq_stream_t stream);

/* out[i] = (accumulate ? out[i] : 0) + scale * sum_k norms_k[b] * sign * l_j from K arrays of
 * level|sign bytes (norms, q: HOST arrays of K device pointers): the aggregate of Alg. 1 for messages
 * already decoded to bytes.  fp64 sum in worker order, rounded to fp32 once. */
int nuq_average_levels(uint32_t K, const float *const *norms, const uint8_t *const *q, uint64_t d,
                       uint32_t bucket, uint32_t s, float scale, int accumulate, float *out,
                       nuq_stream_t stream);

/* ---- parameter update and variance diagnostic (Alg. 1 aggregate; Sec. 4.2; App. J) --------------- */

/* The plain aggregate step of Alg. 1 with Omega = R^d,  w <- w - (alpha/K) sum_k Q_k,  is
 * nuq_decode_accumulate (or its table / fixed-width / byte variants) with out = w, accumulate = 1 and
 * scale = -alpha/K: no separate pass over w.
 *
 * Momentum rule of Sec. 4.2 on d fp32 values in DEVICE memory, g the averaged gradient:
 *   y = w - alpha g;  y^l = w - l alpha g;  w <- y + mu (y^l - yl);  yl <- y^l.
 * l = 0 is heavy ball, l = 1 Nesterov's method.  The caller sets yl = w before the first step and owns
 * all three arrays; w and yl are updated in place.  Evaluated in fp64 in this order from the fp32
 * inputs, one rounding per stored value.  NUQ_EINVAL for a null pointer with d > 0, a non-finite
 * alpha, mu or l, or mu outside [0, 1). */
int nuq_momentum_step(float *w, float *yl, const float *g, uint64_t d, float alpha, float mu, float l,
                      nuq_stream_t stream);

/* nuq_decode_accumulate and nuq_momentum_step in one launch: (w, yl) <- momentum rule with
 * g[i] = the fp32 value nuq_decode_accumulate(..., scale, accumulate = 0, ...) would store at i (scale =
 * 1/K for Alg. 1's average).  Same bits in w and yl as the two calls give; the average itself is not
 * stored, which saves its write and read (8 of the update's 24 bytes per coordinate).  Message
 * arguments as nuq_decode_accumulate; alpha, mu, l, w, yl as nuq_momentum_step. */
int nuq_decode_momentum_step(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                             const uint32_t *const *words, const uint64_t *words_len,
                             const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                             uint32_t sync_stride, float scale, float alpha, float mu, float l, float *w,
                             float *yl, nuq_stream_t stream);

/* First and second moments of a gradient estimate across draws (App. J): sum[i] += g[i],
 * sumsq[i] += g[i]^2 in fp64; g, sum, sumsq: DEVICE arrays of d values, sum and sumsq zeroed by the
 * caller before the first draw. */
int nuq_moments_accumulate(const float *g, double *sum, double *sumsq, uint64_t d, nuq_stream_t stream);

/* Mean normalized variance of App. J after M >= 1 draws: out2[0] = sum_i (sumsq_i/M - (sum_i/M)^2),
 * out2[1] = sum_i sumsq_i/M (DEVICE doubles); the diagnostic is out2[0] / out2[1] (the two means over
 * coordinates share the factor 1/d).  Variance = mean squared deviation from the mean of the M draws.
 * workspace: DEVICE memory of at least NUQ_VARIANCE_WORKSPACE_BYTES bytes, 8-byte aligned, overwritten.
 * The summation order is fixed: equal inputs give equal bits. */
#define NUQ_VARIANCE_WORKSPACE_BYTES 16384u
int nuq_normalized_variance(const double *sum, const double *sumsq, uint64_t d, uint64_t M, void *workspace,
                            uint64_t workspace_bytes, double *out2, nuq_stream_t stream);

/* ---- errors ---------------------------------------------------------------------- */

/* Waits for `stream`, copies the sticky device flags of the current device to
 * *host_flags (host pointer) and clears them. */
int nuq_last_error_flags(uint32_t *host_flags, nuq_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* NUQ_H */
