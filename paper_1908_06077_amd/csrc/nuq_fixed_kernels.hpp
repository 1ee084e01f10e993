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

// MODE 0: norms + quantizer + packing from v (read once).  MODE 1: packing of level|sign bytes.  One bucket per team.
template <int TEAM, int VPT, int MODE>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_pack_fixed(EncodeParams P, EncodeBatch Wk, FixedParams F)
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
    if constexpr (MODE == 0)
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
    float scale;
    int accumulate;
};

// out[i] = [out[i] +] scale * sum_k norms_k[bucket] * sign * 2^(level - 1 - s): fp64 sum in worker order, one
// rounding.  A thread owns four consecutive coordinates (one 16-byte store) when buckets are multiples of four,
// else one.  A level index above s + 1, or a signed zero, raises the malformed flag.
template <int VEC>
__global__ __launch_bounds__(256) void k_unpack_accumulate_fixed(UnpackParams P)
{
    const uint64_t i0 = ((uint64_t)blockIdx.x * 256u + threadIdx.x) * VEC;
    if (i0 >= P.d)
        return;
    const uint64_t bk = i0 / P.bucket;
    const uint32_t j0 = (uint32_t)(i0 - bk * P.bucket);
    const uint32_t bit0 = j0 * P.b;
    const uint32_t nbits = VEC * P.b;                       // <= 32
    const uint32_t wi = bit0 >> 5, sh = bit0 & 31u;
    const bool two = sh + nbits > 32u;                      // the codes straddle a word boundary
    const uint32_t mask_level = (1u << (P.b - 1u)) - 1u;
    double sum[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c)
        sum[c] = 0.0;
    bool bad = false;
    for (uint32_t k = 0; k < P.K; ++k) {
        const uint32_t *f = P.packed[k] + bk * P.wpb + wi;
        const uint32_t w0 = f[0];
        const uint32_t w1 = two ? f[1] : 0u;
        const uint64_t win = (((uint64_t)w0 << 32) | w1) << sh;     // the VEC codes on top
        const double nrm = (double)P.norms[k][bk];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const uint32_t code = (uint32_t)(win >> (64u - (uint32_t)(c + 1) * P.b)) & ((1u << P.b) - 1u);
            const uint32_t level = code & mask_level, neg = code >> (P.b - 1u);
            bad |= level > P.s + 1u || (level == 0u && neg);
            if (level) {
                const double val = ldexp(nrm, (int)level - 1 - (int)P.s);
                sum[c] += neg ? -val : val;
            }
        }
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
    const double sc = (double)P.scale;
    if constexpr (VEC == 4) {
        float4 o;
        const bool whole = i0 + 3u < P.d;
        if (whole) {
            float4 prev = P.accumulate ? *reinterpret_cast<const float4 *>(P.out + i0) : float4{0.f, 0.f, 0.f, 0.f};
            o.x = (float)((double)prev.x + sc * sum[0]);
            o.y = (float)((double)prev.y + sc * sum[1]);
            o.z = (float)((double)prev.z + sc * sum[2]);
            o.w = (float)((double)prev.w + sc * sum[3]);
            *reinterpret_cast<float4 *>(P.out + i0) = o;
        } else {
            for (uint32_t c = 0; c < 4u && i0 + c < P.d; ++c)
                P.out[i0 + c] = (float)((P.accumulate ? (double)P.out[i0 + c] : 0.0) + sc * sum[c]);
        }
    } else {
        P.out[i0] = (float)((P.accumulate ? (double)P.out[i0] : 0.0) + sc * sum[0]);
    }
}

}  // namespace nuq
