// Norms, quantizer and ENCODE kernels (Def. 1, App. A) -- one team of threads per bucket.
//
// Element layout inside a team: thread t, row i holds the four consecutive coordinates
// 4*(i*TEAM + t) .. +3 of its bucket, so every row is one fully coalesced 16-byte load per
// lane.  Level/sign bytes are exchanged through LDS so that in the coding phase thread t
// owns the contiguous coordinates [t*C, (t+1)*C), C = 4*ceil(n / (4*TEAM)) <= 64.
#pragma once
#include "nuq_device.hpp"

namespace nuq {

constexpr uint32_t kFlagCapacity = 1u, kFlagNonfinite = 2u, kFlagMalformed = 4u;

// Decoder index of an ERC message: a bucket is cut into blocks of 2^kSyncBlockShift coordinates and the records of a
// block into 2^pieces_shift pieces of equal count.  An entry = bit offset of the piece's first record (bits 0..20) |
// that record's index inside its block (bits 21..31).
constexpr uint32_t kSyncBlockShift = 11;
constexpr uint32_t kSyncOffMask = 0x1FFFFFu;

constexpr uint32_t kMaxBatch = 32;   // workers per launch

// Per-worker pointers of a batched launch (blockIdx.y selects the worker).
struct EncodeWorker {
    const float *v;        // fused / quantize / norms input
    const uint8_t *q_in;   // encode-from-bytes input
    uint8_t *q_out;        // quantize output
    const float *norms_in; // quantize input
    float *norms_out;      // norms / fused output
    uint32_t *sync;        // [nb * nsync]
    uint64_t *bit_off;     // [nb + 1]
    uint32_t *words;
    uint64_t words_cap;
    uint64_t seed;
};

struct EncodeBatch {
    EncodeWorker w[kMaxBatch];
};

struct EncodeParams {
    uint64_t d;
    uint64_t nb;
    uint32_t bucket;
    uint32_t s;
    uint32_t sync_shift;   // Huffman-coded messages: log2(sync stride), 0 = no index
    uint32_t nsync;        // index entries per bucket (0 = no index)
    uint32_t pieces_shift; // ERC messages: log2(pieces per block)
    uint32_t nblk;         // ERC messages: blocks per bucket = ceil(bucket / 2048)
    uint32_t slot_words;   // staging words per bucket
    uint32_t rows;         // ceil(bucket / (4*TEAM))
    uint32_t lds_words;    // LDS words per team
    uint32_t rec_cap;      // nonzeros of a bucket whose indices fit the team's LDS list
    uint32_t out_cap;      // words of a bucket's bit string that fit the team's LDS buffer
    uint64_t nb_stride;    // nb rounded up to a multiple of 4: stride between workers in lens
    uint32_t *lens;        // [K * nb_stride] payload bits per bucket, worker-major
    uint32_t *staging;     // [K * nb * slot_words]
    uint32_t *flags;
    uint32_t norm_linf;    // level-table mode: 0 = Euclidean norm, 1 = maximum norm
};

template <int TEAM>
struct TeamGeom {
    static constexpr int kWG = TEAM < 256 ? 256 : TEAM;
    static constexpr int kTeamsPerWG = kWG / TEAM;
};

// A 16-byte load of data that is read once (gradients): non-temporal, so that the stream does not push the
// staged bit strings, lengths and messages, which the next kernel reads, out of the caches.  Used by teams of a
// wave or more (measured: 172 -> 164 us on 8192-coordinate buckets, 3 % on 16384); quarter-wave teams, whose loads
// are 256-byte pieces, lose 5 % with it and keep plain loads.
__device__ __forceinline__ float4 load_once4(const float4 *p)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 r = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return float4{r.x, r.y, r.z, r.w};
}

// The same for 16 bytes of a result that this kernel does not read again (the averaged gradient): measured on the
// decoder, 3 % on 8192-coordinate buckets of eight workers and 15 % on 16384-coordinate buckets of four.
__device__ __forceinline__ void store_once4(float4 *p, float4 v)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4 *>(p));
}

// Load the four coordinates of vector `vi` of a bucket of `nbk` coordinates starting at `vb`.
__device__ __forceinline__ float4 load_vec4(const float *vb, uint32_t vi, uint32_t nbk, bool aligned)
{
    const uint32_t e0 = 4u * vi;
    if (aligned && e0 + 3u < nbk)
        return reinterpret_cast<const float4 *>(vb)[vi];
    float4 r;
    r.x = e0 + 0u < nbk ? vb[e0 + 0u] : 0.0f;
    r.y = e0 + 1u < nbk ? vb[e0 + 1u] : 0.0f;
    r.z = e0 + 2u < nbk ? vb[e0 + 2u] : 0.0f;
    r.w = e0 + 3u < nbk ? vb[e0 + 3u] : 0.0f;
    return r;
}

// Bucket norm from a per-row accessor.  fp32 partial sums (four accumulators per thread),
// fp64 across the team; if the fp32 result could have lost range (tiny or huge sums) the
// whole sum is redone in fp64.  Every thread of the team returns the same value.
template <int TEAM, int VPT, class Row>
__device__ __forceinline__ float team_norm(Row row, double *scratch)
{
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const float4 x = row(i);
        a0 = __builtin_fmaf(x.x, x.x, a0);
        a1 = __builtin_fmaf(x.y, x.y, a1);
        a2 = __builtin_fmaf(x.z, x.z, a2);
        a3 = __builtin_fmaf(x.w, x.w, a3);
    }
    double tot = team_sum_f64<TEAM>((double)((a0 + a1) + (a2 + a3)), scratch);
    if (!(tot >= 0x1p-80 && tot <= 0x1p100)) {   // also catches NaN
        double p = 0.0;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const float4 x = row(i);
            p += (double)x.x * (double)x.x;
            p += (double)x.y * (double)x.y;
            p += (double)x.z * (double)x.z;
            p += (double)x.w * (double)x.w;
        }
        tot = team_sum_f64<TEAM>(p, scratch);
    }
    return (float)sqrt(tot);
}

// ------------------------------------------------------------------ norms kernel
template <int TEAM, int VPT>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_bucket_norms(EncodeParams P, EncodeBatch Wk)
{
    __shared__ double scratch[16];
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t tid = threadIdx.x % TEAM;
    const uint64_t b = (uint64_t)blockIdx.x * TeamGeom<TEAM>::kTeamsPerWG + threadIdx.x / TEAM;
    const bool active = b < P.nb;
    const uint64_t base = active ? b * P.bucket : 0;
    const uint32_t nbk = active ? (uint32_t)min((uint64_t)P.bucket, P.d - base) : 0u;
    const float *vb = W.v + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(vb) & 15u) == 0;
    auto row = [&](int i) { return load_vec4(vb, (uint32_t)i * TEAM + tid, nbk, aligned); };
    const float nrm = team_norm<TEAM, VPT>(row, scratch);
    if (active && tid == 0)
        W.norms_out[b] = nrm;
}

// Quantize the four coordinates of one vector; returns the four level|sign<<7 bytes.
// x0 = (k0 + index of first coordinate) * C1.  The caller has applied B.prescale to x.
//
// Three routes, chosen per wave from the largest |v_i| of the vector over all lanes:
//   below the first level (the usual case: |v_i| < 2^-s ||v||): the level is 0 or 1, "up" is the sign bit of
//     t = fma(u, c, -|v|), and the bytes are assembled from the top bytes of v (sign) and t (up) with byte permutes;
//   below twice the first level (s >= 1): bins [0, ns) and [ns, 2 ns) have the same width, so only the bin's lower end
//     differs per coordinate;
//   anything else: no branches; |v| is scaled into [ns, 2 ns) by replacing its exponent (its distance to the lower
//     end of its bin, divided by the bin's width in units of c, is then a - ns for every bin), bin index from the
//     difference of the bit patterns.
__device__ __forceinline__ uint32_t quantize_vec4(const float4 &x, uint32_t x0, uint32_t k1,
                                                  const BucketScale &B)
{
    const float xs[4] = {x.x, x.y, x.z, x.w};   // already multiplied by B.prescale
    const float big = fmaxf(fmaxf(fabsf(xs[0]), fabsf(xs[1])), fmaxf(fabsf(xs[2]), fabsf(xs[3])));
    uint32_t u[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
        u[c] = draw24(x0 + (uint32_t)c * kRngC1, k1);
    if (__all(big < B.ns)) {
        uint32_t tb[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            tb[c] = f2u(__builtin_fmaf((float)u[c], B.c, -fabsf(xs[c])));
        // top bytes of t0..t3 and of v0..v3, one per result byte
        const uint32_t t01 = __builtin_amdgcn_perm(tb[1], tb[0], 0x0c0c0703u);
        const uint32_t t23 = __builtin_amdgcn_perm(tb[3], tb[2], 0x0c0c0703u);
        const uint32_t v01 = __builtin_amdgcn_perm(f2u(xs[1]), f2u(xs[0]), 0x0c0c0703u);
        const uint32_t v23 = __builtin_amdgcn_perm(f2u(xs[3]), f2u(xs[2]), 0x0c0c0703u);
        const uint32_t up7 = __builtin_amdgcn_perm(t23, t01, 0x05040100u) & 0x80808080u;   // bit 7 of byte c = up_c
        const uint32_t sg = __builtin_amdgcn_perm(v23, v01, 0x05040100u);
        return (sg & up7) | (up7 >> 7);
    }
    uint32_t levels = 0;
    if (B.s >= 1 && __all(big < B.ns2)) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float a = fabsf(xs[c]);
            const float over = a - B.ns;                       // exact when it is used (ns <= a < 2 ns)
            const bool low = over < 0.0f;
            const float t = __builtin_fmaf((float)u[c], B.c, -(low ? a : over));
            levels |= ((low ? 0u : 1u) + (t < 0.0f ? 1u : 0u)) << (8 * c);
        }
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int diff = (int)((f2u(xs[c]) & 0x7fffffffu) - B.ns_bits);
            const int m = diff >> 23;                          // bin: floor(log2(a / ns)), negative below the first level
            const float a2 = u2f(B.ns_bits + ((uint32_t)diff & 0x007fffffu));
            const float t = __builtin_fmaf((float)u[c], B.c, -(m < 0 ? fabsf(xs[c]) : a2 - B.ns));
            const int j = min(max(m, -1) + 1 + (t < 0.0f ? 1 : 0), B.s + 1);   // m >= s: the top level, no draw
            levels |= (uint32_t)j << (8 * c);
        }
    }
    // sign bytes of the four coordinates, kept where the level is not zero (a level is below 128)
    const uint32_t v01 = __builtin_amdgcn_perm(f2u(xs[1]), f2u(xs[0]), 0x0c0c0703u);
    const uint32_t v23 = __builtin_amdgcn_perm(f2u(xs[3]), f2u(xs[2]), 0x0c0c0703u);
    const uint32_t sg = __builtin_amdgcn_perm(v23, v01, 0x05040100u);
    const uint32_t nz7 = (levels + 0x7f7f7f7fu) & 0x80808080u;
    return (sg & nz7) | levels;
}

// --------------------------------------------------------------- quantize kernel
template <int TEAM, int VPT>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_quantize(EncodeParams P, EncodeBatch Wk)
{
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t tid = threadIdx.x % TEAM;
    const uint64_t b = (uint64_t)blockIdx.x * TeamGeom<TEAM>::kTeamsPerWG + team_uniform_u32<TEAM>(threadIdx.x / TEAM);
    if (b >= P.nb)
        return;
    const uint64_t base = b * P.bucket;
    const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - base);
    const float *vb = W.v + base;
    uint8_t *qb = W.q_out + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(vb) & 15u) == 0;
    const bool qaligned = (reinterpret_cast<uintptr_t>(qb) & 3u) == 0;
    const BucketScale B = make_scale(team_uniform_f32<TEAM>(W.norms_in[b]), (int)P.s);
    const BucketKey key = bucket_key(W.seed, b);
#pragma unroll 1
    for (uint32_t i = 0; i < P.rows; ++i) {
        const uint32_t vi = i * TEAM + tid;
        const uint32_t e0 = 4u * vi;
        if (e0 >= nbk)
            break;
        float4 x = load_vec4(vb, vi, nbk, aligned);
        if (B.prescale != 1.0f) {
            x.x *= B.prescale;
            x.y *= B.prescale;
            x.z *= B.prescale;
            x.w *= B.prescale;
        }
        const uint32_t packed = B.dead ? 0u : quantize_vec4(x, (key.k0 + e0) * kRngC1, key.k1, B);
        if (qaligned && e0 + 3u < nbk) {
            reinterpret_cast<uint32_t *>(qb)[vi] = packed;
        } else {
            for (uint32_t c = 0; c < 4u && e0 + c < nbk; ++c)
                qb[e0 + c] = (uint8_t)(packed >> (8 * c));
        }
    }
}

// ----------------------------------------------------------------- coding phase
//
// On entry the team's level/sign bytes are in LDS (qb32, bytes at or beyond the bucket's
// length are zero) and a barrier has been passed.  Produces the bucket's bit string in
// LDS `out`, copies it to the bucket's staging slot, writes its bit length and its sync
// entries.  Every thread of the workgroup must call it (it contains barriers).
//
// Steps: (1) every thread finds the nonzeros of its contiguous chunk and the team compacts
// their indices into `rec` (a prefix sum gives the ranks); (2) the records are dealt out evenly,
// a thread takes a contiguous run of them, looks up gap and level codes in a 256-entry table
// and sums their lengths; a second prefix sum gives every run its bit offset; (3) the same
// runs are walked again to OR the record bits into `out`.

// Code table for N < 256, built at compile time: code (right-aligned) | length << 16; entry 0 repeats entry 1.
// A workgroup copies it to LDS once instead of computing it.
struct ErcTable {
    uint32_t v[256];
};
constexpr uint32_t bit_width_c(uint32_t x)
{
    uint32_t w = 0;
    while (x) {
        ++w;
        x >>= 1;
    }
    return w;
}
constexpr ErcTable make_erc_table()
{
    ErcTable t{};
    for (uint32_t i = 0; i < 256u; ++i) {
        const uint32_t N = i ? i : 1u;
        // Alg. 2: groups binary(N), binary(bits(N) - 1), ... while the value is at least 2, last computed first, one 0
        uint32_t code = 0, len = 0;
        for (uint32_t g = N; g >= 2u; g = bit_width_c(g) - 1u) {
            code |= g << len;
            len += bit_width_c(g);
        }
        t.v[i] = (code << 1) | ((len + 1u) << 16);
    }
    return t;
}
__device__ const ErcTable kErcTable = make_erc_table();

// Table for the tail of a record, indexed by the level|sign byte (level in bits 0..6, 1..15; sign in bit 7): the
// sign bit followed by the level's code, right-aligned, | their length << 16.
constexpr ErcTable make_tail_table()
{
    const ErcTable erc = make_erc_table();
    ErcTable t{};
    for (uint32_t i = 0; i < 256u; ++i) {
        const uint32_t e = erc.v[i & 15u], code = e & 0xffffu, len = e >> 16;
        t.v[i] = ((i >> 7) << len) | code | ((len + 1u) << 16);
    }
    return t;
}
__device__ const ErcTable kTailTable = make_tail_table();

// erc_lut[N] for N < 256: code (right-aligned) | length << 16.
__device__ __forceinline__ uint32_t erc_lookup(const uint32_t *erc_lut, uint32_t N, uint32_t &len)
{
    if (N < 256u) {
        const uint32_t e = erc_lut[N];
        len = e >> 16;
        return e & 0xffffu;
    }
    return erc_code(N, len);
}

// Orders a team's LDS traffic between the phases of the coding pass.  A team of one wave needs no hardware barrier
// (its lanes run in lockstep and its LDS operations complete in order), only the wait and a fence for the
// compiler; the teams of a workgroup are independent of each other.
template <int TEAM>
__device__ __forceinline__ void team_barrier()
{
    if constexpr (TEAM > kWave) {
        __syncthreads();
    } else {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        __builtin_amdgcn_wave_barrier();
    }
}

// LDS is what bounds the number of buckets in flight on a CU, and a bucket's worst case (every coordinate
// nonzero at the longest level code) is four to ten times what gradients produce.  So the team's index list and
// bit-string buffer hold `rec_cap` nonzeros and `out_cap` words, sized for the usual case, and a bucket that
// exceeds one of them takes a slower way around it:
//   nonzeros fit, bits fit  : compacted index list, balanced record runs, bit string assembled in LDS
//   nonzeros fit, bits don't: the same, but records are OR-ed into the (zeroed) staging slot in global memory
//   nonzeros don't fit      : every thread codes the records of its own chunk; the bit string is assembled in LDS
//                             over the list's and the buffer's words together if it fits there, else in the slot
template <int TEAM, int VPT>
__device__ __forceinline__ void encode_from_lds(const EncodeParams &P, const EncodeWorker &W, bool active, uint64_t b,
                                                const uint32_t *qb32, uint32_t *out, uint16_t *rec,
                                                const uint32_t *erc_lut, const uint32_t *tail_lut, uint32_t *sync_l,
                                                uint32_t *blk, uint32_t *run_off, uint32_t *scratch)
{
    const uint32_t tid = threadIdx.x % TEAM;
    const uint32_t rows = P.rows;
    const uint32_t base = tid * rows * 4u;
    const uint8_t *qbytes = reinterpret_cast<const uint8_t *>(qb32);

    // (1) nonzero mask of this thread's chunk (rows <= VPT <= 16 words: two 32-bit halves), ranks, compaction
    static_assert(VPT <= 16, "the chunk's mask is 64 bits");
    uint32_t nz_lo = 0, nz_hi = 0;
#pragma unroll
    for (int w = 0; w < VPT; ++w) {
        if ((uint32_t)w < rows) {
            const uint32_t word = qb32[tid * rows + (uint32_t)w];
            // bit 0 of every byte whose low seven bits (the level) are not all zero, then the four bits side by side
            const uint32_t t = (((word & 0x7f7f7f7fu) + 0x7f7f7f7fu) >> 7) & 0x01010101u;
            const uint32_t nib = __builtin_amdgcn_udot4(t, 0x08040201u, 0u, false);
            if (w < 8)
                nz_lo |= nib << (4 * w);
            else
                nz_hi |= nib << (4 * (w - 8));
        }
    }
    const uint64_t nz = ((uint64_t)nz_hi << 32) | nz_lo;
    uint32_t nnz;
    uint32_t rank = team_exclusive_sum<TEAM>((uint32_t)(__popc(nz_lo) + __popc(nz_hi)), scratch, nnz);
    const uint32_t rank0 = rank;                   // records before this thread's chunk
    const bool listed = nnz <= P.rec_cap;          // uniform over the team
    if (P.nsync) {
        // blk[t] = records before block t of the decoder index: the thread whose chunk holds the block's first
        // coordinate counts its own nonzeros below it (every block starts inside exactly one chunk)
        constexpr uint32_t kBlock = 1u << kSyncBlockShift;
        const uint32_t c = (base + kBlock - 1u) & ~(kBlock - 1u);
        const uint32_t t = c >> kSyncBlockShift;
        if (c < base + rows * 4u && t < P.nblk) {
            const uint32_t sh = c - base;                                    // < 64
            const uint64_t below = sh ? nz & (~0ull >> (64u - sh)) : 0ull;
            blk[t] = rank0 + (uint32_t)__popcll((unsigned long long)below);
        }
        if (tid == 0)
            blk[P.nblk] = nnz;
    }
    int before_chunk = -1;                         // last nonzero before this thread's chunk (unlisted buckets)
    if (listed) {
        auto list = [&](uint32_t m, uint32_t at) {
            while (m) {
                const uint32_t k = (uint32_t)__builtin_ctz(m);
                m &= m - 1u;
                rec[rank++] = (uint16_t)(at + k);
            }
        };
        list(nz_lo, base);
        if constexpr (VPT > 8)
            list(nz_hi, base + 32u);
    } else {
        const int last = nz ? (int)base + 63 - __clzll((long long)nz) : -1;
        before_chunk = team_exclusive_max<TEAM>(last, -1, reinterpret_cast<int *>(scratch + 16));
    }
    team_barrier<TEAM>();

    // The records this thread codes, in index order: f(index, previous nonzero's index, level|sign byte).
    const uint32_t per = (nnz + TEAM - 1u) / TEAM;
    const uint32_t r0 = min(tid * per, nnz), r1 = min(r0 + per, nnz);
    auto for_my_records = [&](auto &&f) {
        if (listed) {
            int p = r0 ? (int)rec[r0 - 1u] : -1;
            for (uint32_t r = r0; r < r1; ++r) {
                const int e = (int)rec[r];
                f(e, p, (uint32_t)qbytes[e]);
                p = e;
            }
        } else {
            int p = before_chunk;
            uint64_t m = nz;
            while (m) {
                const int e = (int)base + __ffsll((unsigned long long)m) - 1;
                m &= m - 1;
                f(e, p, (uint32_t)qbytes[e]);
                p = e;
            }
        }
    };

    // A record's bits (right-aligned) and length: ERC(gap), then sign and ERC(level) from the tail table.
    auto make_record = [&](int e, int p, uint32_t byte, uint32_t &len) {
        uint32_t lg;
        const uint32_t cg = erc_lookup(erc_lut, (uint32_t)(e - p), lg);
        const uint32_t tl = tail_lut[byte];
        len = lg + (tl >> 16);
        return (cg << (tl >> 16)) | (tl & 0xffffu);
    };

    // (2) lengths of this thread's records.  The first kKept records of a run from the list stay in registers
    // for the third pass (a run is nnz / TEAM records: two or three for gradients in large buckets, eight where
    // a quarter of a 512-coordinate bucket is nonzero).
    constexpr uint32_t kKept = TEAM <= 64 ? 8 : 4;
    uint32_t kept_bits[kKept], kept_len[kKept];
    int kept_e[kKept];
    uint32_t bits = 0;
    if (listed) {
        int p = r0 ? (int)rec[r0 - 1u] : -1;
#pragma unroll
        for (uint32_t i = 0; i < kKept; ++i) {
            kept_len[i] = 0;
            kept_bits[i] = 0;
            kept_e[i] = p;
            if (r0 + i < r1) {
                const int e = (int)rec[r0 + i];
                kept_bits[i] = make_record(e, p, (uint32_t)qbytes[e], kept_len[i]);
                kept_e[i] = e;
                bits += kept_len[i];
                p = e;
            }
        }
        for (uint32_t r = r0 + kKept; r < r1; ++r) {
            const int e = (int)rec[r];
            uint32_t len;
            make_record(e, p, (uint32_t)qbytes[e], len);
            bits += len;
            p = e;
        }
    } else {
        for_my_records([&](int e, int p, uint32_t byte) {
            uint32_t len;
            make_record(e, p, byte, len);
            bits += len;
        });
    }
    uint32_t total;
    const uint32_t off0 = team_exclusive_sum<TEAM>(bits, scratch + 32, total);
    const uint32_t nwords = (total + 31u) >> 5;
    // An unlisted bucket does not use the index list, so its bit string may spread over the list's LDS as well
    // (the two regions are adjacent): three quarters of the worst case for large buckets.
    uint32_t *const obuf = listed ? out : reinterpret_cast<uint32_t *>(rec);
    const uint32_t ocap = listed ? P.out_cap : (P.rec_cap + 1u) / 2u + P.out_cap;
    const bool in_lds = nwords <= ocap;                          // uniform over the team
    const uint64_t gb = (uint64_t)blockIdx.y * P.nb + b;         // bucket index over the whole batch
    uint32_t *slot = P.staging + (active ? gb : 0) * P.slot_words;
    if (in_lds) {
        for (uint32_t i = tid; i < nwords; i += TEAM)
            obuf[i] = 0u;
    } else if (active) {
        for (uint32_t i = tid; i < nwords; i += TEAM)
            slot[i] = 0u;
        __threadfence();       // the zeros are in place before any record is OR-ed over them
    }
    // Decoder index: entry i = (block t, piece g) describes record blk[t] + floor(g n_t / pieces) of the bucket.
    uint32_t *const sg = W.sync + (active ? b : 0) * P.nsync;
    const uint32_t pmask = (1u << P.pieces_shift) - 1u;
    // Small teams (a wave or less: short runs, few entries) let the thread that owns a listed record write its entry
    // from the lengths it holds in registers; large teams look the record up from the entry's side.
    constexpr bool kOwnerWrites = TEAM <= (int)kWave;
    const bool targets_to_lds = !listed || kOwnerWrites;
    if (listed && !kOwnerWrites)
        run_off[tid] = off0;              // where this thread's run of records starts in the bit string
    if (targets_to_lds) {
        // the entries' record numbers go to LDS (bit 31: a block without records); an entry past the last record is
        // the bucket's length.  Unlisted records: whoever emits such a record writes the entry (below)
        for (uint32_t i = tid; i < P.nsync; i += TEAM) {
            const uint32_t f = blk[i >> P.pieces_shift], n = blk[(i >> P.pieces_shift) + 1u] - f;
            const uint32_t r = f + (((i & pmask) * n) >> P.pieces_shift);
            if (r >= nnz && active)
                sg[i] = total;
            sync_l[i] = r | (n ? 0u : 0x80000000u);
        }
    }
    team_barrier<TEAM>();
    if (listed && kOwnerWrites) {
        // this thread's run is records [r0, r1), the first at bit off0: the entries that point into it (their record
        // numbers are sorted) are found by bisection, a record's offset is the sum of the lengths before it in the run
        if (r0 < r1 && P.nsync) {
            uint32_t lo = 0, hi = P.nsync;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if ((sync_l[mid] & 0x7fffffffu) < r0)
                    lo = mid + 1u;
                else
                    hi = mid;
            }
            for (uint32_t cur = lo; cur < P.nsync; ++cur) {
                const uint32_t tg = sync_l[cur], r = tg & 0x7fffffffu;
                if (r >= r1)
                    break;
                uint32_t pos = off0;
#pragma unroll
                for (uint32_t i = 0; i < kKept; ++i)
                    pos += r0 + i < r ? kept_len[i] : 0u;
                for (uint32_t q = r0 + kKept; q < r; ++q) {      // (a run longer than the records kept in registers)
                    const int e = (int)rec[q];
                    uint32_t len;
                    make_record(e, (int)rec[q - 1u], (uint32_t)qbytes[e], len);
                    pos += len;
                }
                const uint32_t rel = (tg >> 31) ? 0u : (uint32_t)rec[r] - ((cur >> P.pieces_shift) << kSyncBlockShift);
                if (active)
                    sg[cur] = pos | (rel << 21);
            }
        }
    } else if (listed) {
        // the run that holds the record starts at run_off[owner]; the lengths of the records before it in that run
        // are looked up again (a run is nnz / TEAM records)
        for (uint32_t i = tid; i < P.nsync; i += TEAM) {
            const uint32_t t = i >> P.pieces_shift;
            const uint32_t f = blk[t], n = blk[t + 1u] - f;
            const uint32_t r = f + (((i & pmask) * n) >> P.pieces_shift);
            uint32_t entry = total;
            if (r < nnz) {
                const uint32_t owner = r / per;
                uint32_t q0 = owner * per;
                uint32_t pos = run_off[owner];
                int p = q0 ? (int)rec[q0 - 1u] : -1;
                for (; q0 < r; ++q0) {
                    const int e = (int)rec[q0];
                    uint32_t len;
                    make_record(e, p, (uint32_t)qbytes[e], len);
                    pos += len;
                    p = e;
                }
                entry = pos | ((n ? (uint32_t)rec[r] - (t << kSyncBlockShift) : 0u) << 21);
            }
            if (active)
                sg[i] = entry;
        }
    }

    // (3) emit.  A thread's records are consecutive in the bit string: they are shifted into a 64-bit register and
    // leave it 32 bits at a time (a record is at most 31 bits, so at most 31 + 31 bits are pending), OR-ed into the
    // zeroed words because a thread's first and last word are shared with its neighbours.
    {
        uint32_t t = off0, wi = off0 >> 5, fill = off0 & 31u;
        uint64_t acc = 0;
        // unlisted records: the index entries that point at this thread's records (their numbers are sorted)
        uint32_t cur = P.nsync, rno = rank0;
        if (!listed && P.nsync) {
            uint32_t lo = 0, hi = P.nsync;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if ((sync_l[mid] & 0x7fffffffu) < rank0)
                    lo = mid + 1u;
                else
                    hi = mid;
            }
            cur = lo;
        }
        auto emit = [&](uint32_t *dst, int e, int p, uint32_t bitsrec, uint32_t len) {
            (void)p;
            if (!listed) {
                while (cur < P.nsync) {
                    const uint32_t tg = sync_l[cur];
                    if ((tg & 0x7fffffffu) != rno)
                        break;
                    const uint32_t rel = (tg >> 31) ? 0u : (uint32_t)e - ((cur >> P.pieces_shift) << kSyncBlockShift);
                    if (active)
                        sg[cur] = t | (rel << 21);
                    ++cur;
                }
                ++rno;
            }
            acc = (acc << len) | bitsrec;
            fill += len;
            t += len;
            if (fill >= 32u) {
                fill -= 32u;
                atomicOr(&dst[wi++], (uint32_t)(acc >> fill));
                acc &= (1ull << fill) - 1ull;
            }
        };
        auto flush = [&](uint32_t *dst) {
            if (fill && t != off0)
                atomicOr(&dst[wi], (uint32_t)(acc << (32u - fill)));
        };
        auto emit_all = [&](uint32_t *dst) {
            if (listed) {
                int p = r0 ? (int)rec[r0 - 1u] : -1;
#pragma unroll
                for (uint32_t i = 0; i < kKept; ++i) {
                    if (kept_len[i])
                        emit(dst, kept_e[i], p, kept_bits[i], kept_len[i]);
                    p = kept_e[i];
                }
                for (uint32_t r = r0 + kKept; r < r1; ++r) {
                    const int e = (int)rec[r];
                    uint32_t len;
                    const uint32_t bitsrec = make_record(e, p, (uint32_t)qbytes[e], len);
                    emit(dst, e, p, bitsrec, len);
                    p = e;
                }
            } else {
                for_my_records([&](int e, int p, uint32_t byte) {
                    uint32_t len;
                    const uint32_t bitsrec = make_record(e, p, byte, len);
                    emit(dst, e, p, bitsrec, len);
                });
            }
        };
        if (in_lds) {
            emit_all(obuf);
            flush(obuf);
        } else if (active) {
            emit_all(slot);
            flush(slot);
        }
    }
    team_barrier<TEAM>();
    if (active) {
        if (in_lds)
            for (uint32_t i = tid; i < nwords; i += TEAM)
                slot[i] = obuf[i];
        if (tid == 0)
            P.lens[(uint64_t)blockIdx.y * P.nb_stride + b] = total;
    }
}

// What a team's LDS holds of a bucket's nonzero list and bit string: everything for small buckets, a quarter
// of the worst case for large ones (about four times what a Gaussian gradient produces).
__host__ __device__ inline uint32_t team_rec_cap(uint32_t bucket)
{
    const uint32_t quarter = bucket / 4u;
    return bucket <= 1024u ? bucket : (quarter > 1024u ? quarter : 1024u);
}
__host__ __device__ inline uint32_t team_out_cap(uint32_t slot_words)
{
    const uint32_t quarter = slot_words / 4u;
    return slot_words <= 256u ? slot_words : (quarter > 256u ? quarter : 256u);
}

// LDS carve-up per team (in 32-bit words): [qb32: rows*TEAM][rec: rec_cap/2 (u16 per listed nonzero)]
// [out: out_cap + 1][sync: nsync][blk: nblk + 1][run_off: TEAM][scratch: 64 (16 uints, 16 ints, 16 uints, 8 doubles)];
// the workgroup's two 256-entry code tables follow the last team.
__host__ __device__ inline uint32_t team_lds_words(uint32_t rows, uint32_t team, uint32_t rec_cap, uint32_t out_cap,
                                                   uint32_t nsync, uint32_t nblk)
{
    uint32_t w = rows * team + (rec_cap + 1u) / 2u + out_cap + 1u + nsync + nblk + 1u + team;
    w = (w + 1u) & ~1u;   // keep the scratch 8-byte aligned
    return w + 64u;
}

// Front of the fused kernels: the bucket's coordinates into registers (v is read once), its norm (written to
// norms_out), the quantizer, level|sign bytes into the team's LDS words qb32[rows * TEAM].
template <int TEAM, int VPT>
__device__ __forceinline__ void front_quantize_to_lds(const EncodeParams &P, const EncodeWorker &W, uint64_t b,
                                                      bool active, uint64_t base, uint32_t nbk, uint32_t tid,
                                                      uint32_t *qb32, uint32_t *scratch)
{
    const float *vb = W.v + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(vb) & 15u) == 0;
    float4 x[VPT];
    if (aligned && nbk == (uint32_t)VPT * TEAM * 4u) {   // a full bucket that fills every row: plain vector loads
#pragma unroll
        for (int i = 0; i < VPT; ++i)
            x[i] = TEAM >= 64 ? load_once4(reinterpret_cast<const float4 *>(vb) + ((uint32_t)i * TEAM + tid))
                              : reinterpret_cast<const float4 *>(vb)[(uint32_t)i * TEAM + tid];
    } else {
#pragma unroll
        for (int i = 0; i < VPT; ++i)
            x[i] = load_vec4(vb, (uint32_t)i * TEAM + tid, nbk, aligned);
    }
    auto row = [&](int i) { return x[i]; };
    const float nrm = team_uniform_f32<TEAM>(team_norm<TEAM, VPT>(row, reinterpret_cast<double *>(scratch + 32)));
    const bool finite = nrm < __builtin_huge_valf();   // false for NaN too
    if (active && tid == 0) {
        W.norms_out[b] = nrm;
        if (!finite)
            atomicOr(P.flags, kFlagNonfinite);
    }
    const BucketScale B = make_scale(nrm, (int)P.s);
    const BucketKey key = bucket_key(W.seed, b);
    if (B.prescale != 1.0f) {   // tiny norm: work on the bucket scaled by a power of two
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            x[i].x *= B.prescale;
            x[i].y *= B.prescale;
            x[i].z *= B.prescale;
            x[i].w *= B.prescale;
        }
    }
    const uint32_t x0 = (key.k0 + 4u * tid) * kRngC1;      // row i starts 4 * TEAM * i coordinates further on
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        if ((uint32_t)i < P.rows) {
            const uint32_t vi = (uint32_t)i * TEAM + tid;
            qb32[vi] = B.dead ? 0u : quantize_vec4(x[i], x0 + (uint32_t)i * (4u * TEAM * kRngC1), key.k1, B);
        }
    }
}

// Front of the kernels that start from level|sign bytes: q_in into the team's LDS words.
template <int TEAM>
__device__ __forceinline__ void front_bytes_to_lds(const EncodeParams &P, const EncodeWorker &W, uint64_t base,
                                                   uint32_t nbk, uint32_t tid, uint32_t *qb32)
{
    const uint8_t *qg = W.q_in + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(qg) & 3u) == 0;
    for (uint32_t i = 0; i < P.rows; ++i) {
        const uint32_t vi = i * TEAM + tid;
        const uint32_t e0 = 4u * vi;
        uint32_t word = 0;
        if (aligned && e0 + 3u < nbk) {
            word = reinterpret_cast<const uint32_t *>(qg)[vi];
        } else {
            for (uint32_t c = 0; c < 4u; ++c)
                if (e0 + c < nbk)
                    word |= (uint32_t)qg[e0 + c] << (8u * c);
        }
        qb32[vi] = word;
    }
}

// Front of the fused kernels for an arbitrary level table T and the norm P.norm_linf selects: as
// front_quantize_to_lds, with quantize_table_vec4 on the bucket's edges l_t * ||v|| (kept in LDS).
template <int TEAM, int VPT>
__device__ __forceinline__ void front_quantize_table_to_lds(const EncodeParams &P, const EncodeWorker &W,
                                                            const LevelTable &T, uint64_t b, bool active, uint64_t base,
                                                            uint32_t nbk, uint32_t tid, uint32_t *qb32, uint32_t *scratch)
{
    __shared__ double edges_all[TeamGeom<TEAM>::kTeamsPerWG][16];
    double *edges = edges_all[threadIdx.x / TEAM];
    const float *vb = W.v + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(vb) & 15u) == 0;
    float4 x[VPT];
    if (aligned && nbk == (uint32_t)VPT * TEAM * 4u) {   // a full bucket that fills every row (as in the main front)
#pragma unroll
        for (int i = 0; i < VPT; ++i)
            x[i] = TEAM >= 64 ? load_once4(reinterpret_cast<const float4 *>(vb) + ((uint32_t)i * TEAM + tid))
                              : reinterpret_cast<const float4 *>(vb)[(uint32_t)i * TEAM + tid];
    } else {
#pragma unroll
        for (int i = 0; i < VPT; ++i)
            x[i] = load_vec4(vb, (uint32_t)i * TEAM + tid, nbk, aligned);
    }
    float nrm;
    if (P.norm_linf) {
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            m = max(max(m, f2u(x[i].x) & 0x7fffffffu), f2u(x[i].y) & 0x7fffffffu);
            m = max(max(m, f2u(x[i].z) & 0x7fffffffu), f2u(x[i].w) & 0x7fffffffu);
        }
        nrm = u2f(team_max_u32<TEAM>(m, scratch));
    } else {
        auto row = [&](int i) { return x[i]; };
        nrm = team_norm<TEAM, VPT>(row, reinterpret_cast<double *>(scratch + 32));
    }
    nrm = team_uniform_f32<TEAM>(nrm);
    const bool finite = nrm < __builtin_huge_valf();   // false for NaN too
    if (active && tid == 0) {
        W.norms_out[b] = nrm;
        if (!finite)
            atomicOr(P.flags, kFlagNonfinite);
    }
    const bool dead = !(nrm > 0.0f) || !finite;
    if (tid < 16u)
        edges[tid] = (double)T.lev[tid] * (double)nrm;
    team_barrier<TEAM>();
    const double e1 = edges[1];
    const BucketKey key = bucket_key(W.seed, b);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        if ((uint32_t)i < P.rows) {
            const uint32_t vi = (uint32_t)i * TEAM + tid;
            qb32[vi] = quantize_table_vec4(x[i], key.k0 + 4u * vi, key.k1, edges, e1, P.s, dead);
        }
    }
}

// MODE 0: fused norms + quantize + encode from v.  MODE 1: encode from level/sign bytes.  MODE 2: as 0 for the level
// table T and the norm P.norm_linf selects (T is ignored in the other modes).
template <int TEAM, int VPT, int MODE>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_encode(EncodeParams P, EncodeBatch Wk, LevelTable T)
{
    extern __shared__ __align__(16) uint32_t smem[];
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t tid = threadIdx.x % TEAM;
    const uint32_t team = team_uniform_u32<TEAM>(threadIdx.x / TEAM);   // a scalar unless a wave holds four teams
    uint32_t *lds = smem + team * P.lds_words;
    uint32_t *qb32 = lds;
    uint16_t *rec = reinterpret_cast<uint16_t *>(qb32 + P.rows * TEAM);
    uint32_t *out = qb32 + P.rows * TEAM + (P.rec_cap + 1u) / 2u;
    uint32_t *sync_l = out + P.out_cap + 1u;
    uint32_t *blk = sync_l + P.nsync;
    uint32_t *run_off = blk + P.nblk + 1u;
    uint32_t *scratch = lds + P.lds_words - 64u;
    uint32_t *erc_lut = smem + TeamGeom<TEAM>::kTeamsPerWG * P.lds_words;
    uint32_t *tail_lut = erc_lut + 256;
    if (threadIdx.x < 256u) {
        erc_lut[threadIdx.x] = kErcTable.v[threadIdx.x];
        tail_lut[threadIdx.x] = kTailTable.v[threadIdx.x];
    }

    const uint64_t b = (uint64_t)blockIdx.x * TeamGeom<TEAM>::kTeamsPerWG + team;
    const bool active = b < P.nb;
    const uint64_t base = active ? b * P.bucket : 0;
    const uint32_t nbk = active ? (uint32_t)min((uint64_t)P.bucket, P.d - base) : 0u;

    if constexpr (MODE == 2) {
        front_quantize_table_to_lds<TEAM, VPT>(P, W, T, b, active, base, nbk, tid, qb32, scratch);
    } else if constexpr (MODE == 0) {
        front_quantize_to_lds<TEAM, VPT>(P, W, b, active, base, nbk, tid, qb32, scratch);
    } else {
        front_bytes_to_lds<TEAM>(P, W, base, nbk, tid, qb32);
    }
    __syncthreads();
    encode_from_lds<TEAM, VPT>(P, W, active, b, qb32, out, rec, erc_lut, tail_lut, sync_l, blk, run_off, scratch);
}

// ------------------------------------------------- offsets and gather of the slots
//
// wc_b = ceil(len_b / 32) words per bucket; start word of bucket b = sum of wc over the worker's
// earlier buckets; bit_off[b+1] = 32 * start_b + len_b.  One "finish" kernel per batch: a
// workgroup owns FB consecutive buckets of one worker (16, or 64 where buckets are small, so
// that a workgroup still has a few thousand words to move), sums the word counts before them
// (directly, or from per-chunk prefix sums when the worker has many buckets), writes their
// offsets and copies their staging slots to their place in `words`, one word per thread at
// a time, the word's bucket found by bisection.

constexpr uint32_t kChunk = 1024;          // buckets per chunk of the two-level sum
constexpr uint64_t kDirectSumMax = 8192;   // up to this many buckets every workgroup sums directly

__device__ __forceinline__ uint64_t block_sum_u64(uint64_t x, uint64_t *scratch /* 4 */)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        x += __shfl_xor((unsigned long long)x, off, kWave);
    __syncthreads();
    if ((threadIdx.x & 63u) == 0)
        scratch[threadIdx.x >> 6] = x;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// chunk_sums[k * (nchunks + 1) + c] = words of worker k's buckets [c*1024, (c+1)*1024)
__global__ __launch_bounds__(256) void k_chunk_sums(const uint32_t *lens, uint64_t nb, uint64_t nb_stride,
                                                    uint64_t nchunks, uint64_t *chunk_sums)
{
    __shared__ uint64_t scratch[4];
    const uint32_t *l = lens + (uint64_t)blockIdx.y * nb_stride;
    const uint64_t i0 = (uint64_t)blockIdx.x * kChunk;
    uint64_t s = 0;
    for (uint32_t k = threadIdx.x; k < kChunk; k += 256u)
        if (i0 + k < nb)
            s += (l[i0 + k] + 31u) >> 5;
    s = block_sum_u64(s, scratch);
    if (threadIdx.x == 0)
        chunk_sums[(uint64_t)blockIdx.y * (nchunks + 1) + blockIdx.x] = s;
}

// One workgroup per worker: chunk_sums[c] <- sum of chunk_sums[0..c) (in place).
__global__ __launch_bounds__(256) void k_chunk_scan(uint64_t *chunk_sums, uint64_t nchunks)
{
    __shared__ uint64_t carry;
    __shared__ uint64_t wave_tot[4];
    uint64_t *cs = chunk_sums + (uint64_t)blockIdx.x * (nchunks + 1);
    if (threadIdx.x == 0)
        carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint64_t i0 = 0; i0 < nchunks; i0 += 256) {
        const uint64_t i = i0 + threadIdx.x;
        const uint64_t v = i < nchunks ? cs[i] : 0ull;
        uint64_t inc = v;
        for (int off = 1; off < 64; off <<= 1) {
            const uint64_t t = __shfl_up((unsigned long long)inc, off, 64);
            if (lane >= off)
                inc += t;
        }
        if (lane == 63)
            wave_tot[wave] = inc;
        __syncthreads();
        uint64_t before = carry;
        for (int w = 0; w < wave; ++w)
            before += wave_tot[w];
        if (i < nchunks)
            cs[i] = before + inc - v;
        __syncthreads();
        if (threadIdx.x == 255)
            carry = before + inc;
        __syncthreads();
    }
}

// Buckets per workgroup of k_finish.
__host__ __device__ inline uint32_t finish_buckets(uint32_t bucket) { return bucket <= 1024u ? 64u : 16u; }

// grid (ceil(nb / FB), K), FB = 16 or 64.  chunk_prefix == nullptr: sum the lengths of all earlier buckets directly.
template <uint32_t FB, uint32_t WG>
__global__ __launch_bounds__(WG) void k_finish(EncodeParams P, EncodeBatch Wk, const uint64_t *chunk_prefix,
                                                uint64_t nchunks, uint32_t groups)
{
    static_assert(FB == 16 || FB == 64, "one wave scans the workgroup's word counts");
    static_assert(WG == 64 || WG == 256, "block_sum_u64 adds four waves");
    __shared__ uint64_t scratch[4];
    __shared__ uint32_t wstart[FB + 1];   // first word of each bucket, relative to the group's first
    __shared__ uint32_t skip[FB];
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t *__restrict__ lens = P.lens + (uint64_t)blockIdx.y * P.nb_stride;
    const uint32_t tid = threadIdx.x;

    // A workgroup takes `groups` consecutive groups of FB buckets: the words before its first bucket are summed once
    // (from the chunk's start), after that the running total carries over from group to group.
    uint64_t b_first = (uint64_t)blockIdx.x * groups * FB;
    uint64_t lo = 0, base = 0;
    if (chunk_prefix) {
        const uint64_t c = b_first / kChunk;
        lo = c * kChunk;
        base = chunk_prefix[(uint64_t)blockIdx.y * (nchunks + 1) + c];
    }
    uint32_t part = 0;     // < 2^32: at most 8192 lengths of < 2^21 bits each are summed here
    {
        // lo and b_first are multiples of 16, so the range splits into aligned groups of four lengths
        const uint4 *__restrict__ l4 = reinterpret_cast<const uint4 *>(lens + lo);
        const uint32_t n4 = (uint32_t)((b_first - lo) >> 2);
#pragma unroll 4
        for (uint32_t i = tid; i < n4; i += WG) {
            const uint4 v = l4[i];
            part += ((v.x + 31u) >> 5) + ((v.y + 31u) >> 5) + ((v.z + 31u) >> 5) + ((v.w + 31u) >> 5);
        }
    }
    if constexpr (WG == 64u) {            // one wave
        uint64_t x = part;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1)
            x += __shfl_xor((unsigned long long)x, off, kWave);
        base += x;
    } else {
        base += block_sum_u64(part, scratch);
    }

    for (uint32_t g = 0; g < groups && b_first < P.nb; ++g, b_first += FB) {
        uint32_t my_len = 0;
        if (tid < FB && b_first + tid < P.nb)
            my_len = lens[b_first + tid];
        if (tid < kWave) {                      // the first wave: inclusive scan of the word counts
            uint32_t inc = tid < FB ? (my_len + 31u) >> 5 : 0u;
#pragma unroll
            for (int off = 1; off < (int)FB; off <<= 1) {
                const uint32_t t = (uint32_t)__shfl_up((int)inc, off, kWave);
                if ((int)tid >= off)
                    inc += t;
            }
            if (tid < FB)
                wstart[tid + 1] = inc;
            if (tid == 0)
                wstart[0] = 0;
        }
        __syncthreads();
        if (tid < FB && b_first + tid < P.nb) {
            const uint64_t start = base + wstart[tid];
            W.bit_off[b_first + tid + 1] = 32ull * start + my_len;
            if (b_first + tid == 0)
                W.bit_off[0] = 0;
            const bool over = base + wstart[tid + 1] > W.words_cap;
            skip[tid] = over;
            if (over && my_len)
                atomicOr(P.flags, kFlagCapacity);
        }
        __syncthreads();

        // copy the staging slots: word w of the group's run belongs to the bucket found by bisection
        const uint32_t total = wstart[FB];
        const uint32_t *__restrict__ staging = P.staging + ((uint64_t)blockIdx.y * P.nb + b_first) * P.slot_words;
        uint32_t *__restrict__ dst = W.words + base;
#pragma unroll 4
        for (uint32_t w = tid; w < total; w += WG) {
            uint32_t j = 0;
#pragma unroll
            for (uint32_t step = FB / 2; step >= 1; step >>= 1)
                j += (wstart[j + step] <= w) ? step : 0u;
            if (!skip[j])
                dst[w] = staging[(uint64_t)j * P.slot_words + (w - wstart[j])];
        }
        base += total;
        __syncthreads();          // wstart and skip are read to the end before the next group overwrites them
    }
}

}  // namespace nuq
