// Fixed-width coding (Sec. 5: the "4-bit" and "8-bit" variants; 3 bits in Table 1): every coordinate sends its sign
// and level index in b bits.  Layout: coordinate i of a bucket is the code  sign << (b-1) | level index  at bits
// [i*b, i*b + b) of the bucket's field, most significant bit first, in 32-bit words; every bucket's field is
// wpb = ceil(bucket * b / 32) words, so bucket k starts at word k * wpb.  No offsets, no index: both directions are
// plain streaming kernels.
#pragma once

#include "nuq_encode_kernels.hpp"

namespace nuq {

struct FixedParams {
    uint32_t b;     // bits per coordinate, 3..8
    uint32_t wpb;   // words per bucket field
};

// LDS words per team of k_pack_fixed: [qb32: rows * TEAM][field: wpb][scratch: 64]
__host__ __device__ inline uint32_t fixed_lds_words(uint32_t rows, uint32_t team, uint32_t wpb)
{
    const uint32_t w = (rows * team + wpb + 1u) & ~1u;
    return w + 64u;
}

// MODE 0: norms + quantizer + packing from v (read once).  MODE 1: packing of level|sign bytes.  MODE 2: as 0 for the
// level table T and the norm P.norm_linf selects (T is ignored in the other modes).  One bucket per team.
template <int TEAM, int VPT, int MODE>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_pack_fixed(EncodeParams P, EncodeBatch Wk, FixedParams F,
                                                                    LevelTable T)
{
    extern __shared__ __align__(16) uint32_t smem[];
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t tid = threadIdx.x % TEAM;
    const uint32_t team = team_uniform_u32<TEAM>(threadIdx.x / TEAM);
    uint32_t *lds = smem + team * P.lds_words;
    uint32_t *qb32 = lds;
    uint32_t *field = qb32 + P.rows * TEAM;
    uint32_t *scratch = lds + P.lds_words - 64u;
    const uint64_t b = (uint64_t)blockIdx.x * TeamGeom<TEAM>::kTeamsPerWG + team;
    const bool active = b < P.nb;
    const uint64_t base = active ? b * P.bucket : 0;
    const uint32_t nbk = active ? (uint32_t)min((uint64_t)P.bucket, P.d - base) : 0u;

    for (uint32_t i = tid; i < F.wpb; i += TEAM)
        field[i] = 0u;
    if constexpr (MODE == 2)
        front_quantize_table_to_lds<TEAM, VPT>(P, W, T, b, active, base, nbk, tid, qb32, scratch);
    else if constexpr (MODE == 0)
        front_quantize_to_lds<TEAM, VPT>(P, W, b, active, base, nbk, tid, qb32, scratch);
    else
        front_bytes_to_lds<TEAM>(P, W, base, nbk, tid, qb32);
    __syncthreads();

    // Each thread packs a contiguous chunk of rows * 4 coordinates.  Codes are shifted into a 64-bit register and
    // leave it 32 bits at a time; a chunk's first and last words may be shared with its neighbours, so words are
    // OR-ed into the (zeroed) field.
    const uint32_t per = P.rows * 4u;
    const uint32_t c0 = tid * per;
    const uint32_t c1 = min(c0 + per, nbk);
    if (c0 < c1) {
        const uint8_t *qbytes = reinterpret_cast<const uint8_t *>(qb32);
        const uint32_t bit0 = c0 * F.b;
        uint32_t wi = bit0 >> 5, fill = bit0 & 31u;
        uint64_t acc = 0;
        for (uint32_t c = c0; c < c1; ++c) {
            const uint32_t byte = qbytes[c];
            const uint32_t code = ((byte >> 7) << (F.b - 1u)) | (byte & 0x7fu);
            acc = (acc << F.b) | code;
            fill += F.b;
            if (fill >= 32u) {
                fill -= 32u;
                atomicOr(&field[wi++], (uint32_t)(acc >> fill));
                acc &= (1ull << fill) - 1ull;
            }
        }
        if (fill)
            atomicOr(&field[wi], (uint32_t)(acc << (32u - fill)));
    }
    team_barrier<TEAM>();
    if (active) {
        uint32_t *dst = W.words + b * F.wpb;
        for (uint32_t i = tid; i < F.wpb; i += TEAM)
            dst[i] = field[i];
    }
}

struct UnpackParams {
    const float *norms[kMaxBatch];
    const uint32_t *packed[kMaxBatch];
    float *out;
    uint32_t *flags;
    uint64_t d;
    uint32_t K;
    uint32_t bucket;
    uint32_t s;
    uint32_t b;
    uint32_t wpb;
    uint32_t lut_tabs;          // table variant: buckets a workgroup can touch (tables per worker in LDS)
    float scale;
    int accumulate;
    uint32_t use_levels;        // 1: level j has the value lev[j] (a level table), 0: 2^(j - 1 - s)
    float lev[16];
};

// norm * l_level, exact in fp64 either way (level 1..s+1).
__device__ __forceinline__ double fixed_level_value(const UnpackParams &P, double nrm, uint32_t level)
{
    return P.use_levels ? nrm * (double)P.lev[level] : ldexp(nrm, (int)level - 1 - (int)P.s);
}

// out[i] = [out[i] +] scale * sum_k norms_k[bucket] * sign * 2^(level - 1 - s): fp64 sum in worker order, rounded to
// fp32 (the prior, when there is one, is added in fp32 after that).  A level index above s + 1, or a signed zero,
// raises the malformed flag.
//
// Buckets that are multiples of 32 coordinates: a thread owns 32 consecutive coordinates, i.e. exactly B whole words
// of every worker's field (one contiguous load per worker, coalesced over the wave), and the workgroup's 8192 results
// go through LDS so that the stores are whole lines too.
//
// kLut: the value of every code, norm * sign * 2^(level - 1 - s) in fp64 (0 for level 0 and for codes that are not
// valid), is tabulated in LDS once per (bucket the workgroup touches, worker); a code then costs a bit-field extract,
// an LDS read and an fp64 add instead of the exponent arithmetic.  A table of 16 entries is 128 bytes = all 32 banks
// once, so lanes that read one table never conflict whatever their codes.  Codes wider than 5 bits index 32 entries
// by (sign, low four level bits): levels stop at 15.  `lut_tabs` tables per worker are laid out bucket-major.
constexpr uint32_t fixed_lut_entries(uint32_t b) { return b <= 5u ? 1u << b : 32u; }

template <int B>
__device__ __forceinline__ uint32_t fixed_lut_index(uint32_t code)
{
    if constexpr (B <= 5)
        return code;
    else
        return ((code >> (B - 1)) << 4) | (code & 15u);
}

// Whole words of codes that never straddle a word (B = 4, 8): true if some code has a level above s + 1 or is a
// signed zero.  Per field: level + (2^(B-1) - 1) sets the top bit iff level >= 1; level + (2^(B-1) - 2 - s) sets it
// iff level >= s + 2; neither sum leaves its field.
template <int B>
__device__ __forceinline__ bool fixed_word_invalid(uint32_t w, uint32_t s)
{
    static_assert(B == 4 || B == 8, "fields must tile the word");
    constexpr uint32_t kOnes = B == 4 ? 0x11111111u : 0x01010101u;
    constexpr uint32_t kTop = kOnes << (B - 1), kLevels = kTop - kOnes;
    const uint32_t lv = w & kLevels;
    const uint32_t nonzero = (lv + kLevels) & kTop;
    const uint32_t above = (lv + ((1u << (B - 1)) - 2u - s) * kOnes) & kTop;
    return (above | (w & kTop & ~nonzero)) != 0u;
}

template <int B, bool kLut>
__global__ __launch_bounds__(256) void k_unpack_accumulate_fixed32(UnpackParams P)
{
    __shared__ float tile[256 * 33];                          // a thread's 32 results in a row of 33: no bank conflicts
    extern __shared__ __align__(128) double lut[];            // kLut: [lut_tabs][K][entries]
    constexpr uint32_t kEntries = fixed_lut_entries(B);
    constexpr uint32_t kLevelMask = (1u << (B - 1)) - 1u;
    const uint64_t chunk = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const uint64_t i0 = chunk * 32u;
    const uint64_t wg0 = (uint64_t)blockIdx.x * 8192u;
    const uint64_t bk_first = P.d <= 0xffffffffull ? (uint64_t)((uint32_t)wg0 / P.bucket) : wg0 / P.bucket;
    if constexpr (kLut) {
        const uint64_t nb = (P.d + P.bucket - 1) / P.bucket;
        const uint32_t total = P.lut_tabs * P.K * kEntries;
        for (uint32_t e = threadIdx.x; e < total; e += 256u) {
            const uint32_t idx = e % kEntries, k = (e / kEntries) % P.K, tab = e / (kEntries * P.K);
            const uint32_t level = B <= 5 ? idx & kLevelMask : idx & 15u, neg = B <= 5 ? idx >> (B - 1) : idx >> 4;
            double val = 0.0;
            if (bk_first + tab < nb && level >= 1u && level <= P.s + 1u) {
                val = fixed_level_value(P, (double)P.norms[k][bk_first + tab], level);
                val = neg ? -val : val;
            }
            lut[e] = val;
        }
        __syncthreads();
    }
    double sum[32];
#pragma unroll
    for (int c = 0; c < 32; ++c)
        sum[c] = 0.0;
    bool bad = false;
    if (i0 < P.d) {
        const uint64_t bk = P.d <= 0xffffffffull ? (uint64_t)((uint32_t)i0 / P.bucket) : i0 / P.bucket;
        const uint32_t j0 = (uint32_t)(i0 - bk * P.bucket);
        const uint64_t word0 = bk * P.wpb + (uint64_t)(j0 / 32u) * B;
        const double *tab = lut + (uint32_t)(bk - bk_first) * P.K * kEntries;
        for (uint32_t k = 0; k < P.K; ++k) {
            const uint32_t *f = P.packed[k] + word0;
            uint32_t w[B];
#pragma unroll
            for (int t = 0; t < B; ++t)
                w[t] = f[t];
            double nrm = 0.0;
            if constexpr (!kLut)
                nrm = (double)P.norms[k][bk];
            if constexpr (kLut && 32 % B == 0) {
#pragma unroll
                for (int t = 0; t < B; ++t)
                    bad |= fixed_word_invalid<B>(w[t], P.s);
            }
#pragma unroll
            for (int c = 0; c < 32; ++c) {
                // code c occupies bits [c*B, c*B + B) of the B words, most significant bit first
                const int bit = c * B, wi = bit >> 5, off = bit & 31;
                uint32_t code;
                if (off + B <= 32)
                    code = (w[wi] >> (32 - off - B)) & ((1u << B) - 1u);
                else
                    code = ((w[wi] << (off + B - 32)) | (w[wi + 1 < B ? wi + 1 : wi] >> (64 - off - B))) & ((1u << B) - 1u);
                if constexpr (kLut) {
                    if constexpr (32 % B != 0) {
                        const uint32_t level = code & kLevelMask;
                        bad |= level > P.s + 1u || code == (1u << (B - 1));
                    }
                    sum[c] += tab[k * kEntries + fixed_lut_index<B>(code)];
                } else {
                    const uint32_t level = code & kLevelMask, neg = code >> (B - 1);
                    bad |= level > P.s + 1u || (level == 0u && neg);
                    if (level) {
                        const double val = fixed_level_value(P, nrm, min(level, 15u));
                        sum[c] += neg ? -val : val;
                    }
                }
            }
        }
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
    const double sc = (double)P.scale;
#pragma unroll
    for (int c = 0; c < 32; ++c)
        tile[threadIdx.x * 33u + (uint32_t)c] = (float)(sc * sum[c]);
    __syncthreads();
    const uint64_t base = (uint64_t)blockIdx.x * 8192u;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const uint32_t e = ((uint32_t)it * 256u + threadIdx.x) * 4u;          // element of the workgroup's 8192
        const uint64_t i = base + e;
        if (i >= P.d)
            continue;
        const float *row = tile + (e >> 5) * 33u + (e & 31u);
        float4 o{row[0], row[1], row[2], row[3]};
        if (i + 3u < P.d) {
            if (P.accumulate) {
                const float4 prev = *reinterpret_cast<const float4 *>(P.out + i);
                o.x += prev.x;
                o.y += prev.y;
                o.z += prev.z;
                o.w += prev.w;
            }
            *reinterpret_cast<float4 *>(P.out + i) = o;
        } else {
            const float r[4] = {o.x, o.y, o.z, o.w};
            for (uint32_t c = 0; c < 4u && i + c < P.d; ++c)
                P.out[i + c] = P.accumulate ? P.out[i + c] + r[c] : r[c];
        }
    }
}

// Any bucket size: one coordinate per thread.
__global__ __launch_bounds__(256) void k_unpack_accumulate_fixed1(UnpackParams P)
{
    const uint64_t i0 = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (i0 >= P.d)
        return;
    const uint64_t bk = i0 / P.bucket;
    const uint32_t j0 = (uint32_t)(i0 - bk * P.bucket);
    const uint32_t bit0 = j0 * P.b;
    const uint32_t wi = bit0 >> 5, sh = bit0 & 31u;
    const bool two = sh + P.b > 32u;                        // the code straddles a word boundary
    const uint32_t mask_level = (1u << (P.b - 1u)) - 1u;
    double sum = 0.0;
    bool bad = false;
    for (uint32_t k = 0; k < P.K; ++k) {
        const uint32_t *f = P.packed[k] + bk * P.wpb + wi;
        const uint32_t w0 = f[0];
        const uint32_t w1 = two ? f[1] : 0u;
        const uint64_t win = (((uint64_t)w0 << 32) | w1) << sh;     // the code on top
        const uint32_t code = (uint32_t)(win >> (64u - P.b));
        const uint32_t level = code & mask_level, neg = code >> (P.b - 1u);
        bad |= level > P.s + 1u || (level == 0u && neg);
        if (level) {
            const double val = fixed_level_value(P, (double)P.norms[k][bk], min(level, 15u));
            sum += neg ? -val : val;
        }
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
    const float r = (float)((double)P.scale * sum);
    P.out[i0] = P.accumulate ? P.out[i0] + r : r;
}

}  // namespace nuq
