// Level-table quantizer and maximum norm: Def. 1 for an arbitrary level sequence 0 = l_0 < l_1 < ... < l_{s+1} = 1
// (Sec. 3.1 before the special case; Sec. 4.1 "Generally spaced levels": the exponential family (0, p^s, ..., p, 1),
// uniform levels = QSGD) and the normalization of QSGDinf (Sec. 1, Sec. 2).  Everything else of the path (ENCODE,
// DECODE) is shared: a level index is coded the same way whatever its value.
#pragma once

#include "nuq_encode_kernels.hpp"

namespace nuq {

struct LevelTable {
    float lev[16];   // lev[0] = 0 ... lev[s+1] = 1; entries above s+1 are 0
};

// Maximum of x over the team; every thread returns it.  scratch: 16 words of LDS per workgroup (teams of several waves).
template <int TEAM>
__device__ __forceinline__ uint32_t team_max_u32(uint32_t x, uint32_t *scratch)
{
    constexpr int kLanes = TEAM < kWave ? TEAM : kWave;
#pragma unroll
    for (int off = kLanes / 2; off >= 1; off >>= 1)
        x = max(x, (uint32_t)__shfl_xor((int)x, off, kWave));
    if constexpr (TEAM > kWave) {
        const uint32_t wave = threadIdx.x / kWave;
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0)
            scratch[wave] = x;
        __syncthreads();
        x = scratch[0];
#pragma unroll
        for (int w = 1; w < TEAM / kWave; ++w)
            x = max(x, scratch[w]);
    }
    return x;
}

// norms_out[b] = max_i |v_i| over bucket b: exact.  Bit patterns of non-negative floats order like the floats, and a
// NaN's pattern lies above every number's, so a NaN coordinate makes the norm NaN.
template <int TEAM, int VPT>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_bucket_norms_linf(EncodeParams P, EncodeBatch Wk)
{
    __shared__ uint32_t scratch[16];
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t tid = threadIdx.x % TEAM;
    const uint64_t b = (uint64_t)blockIdx.x * TeamGeom<TEAM>::kTeamsPerWG + threadIdx.x / TEAM;
    const bool active = b < P.nb;
    const uint64_t base = active ? b * P.bucket : 0;
    const uint32_t nbk = active ? (uint32_t)min((uint64_t)P.bucket, P.d - base) : 0u;
    const float *vb = W.v + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(vb) & 15u) == 0;
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const float4 x = load_vec4(vb, (uint32_t)i * TEAM + tid, nbk, aligned);
        m = max(max(m, f2u(x.x) & 0x7fffffffu), f2u(x.y) & 0x7fffffffu);
        m = max(max(m, f2u(x.z) & 0x7fffffffu), f2u(x.w) & 0x7fffffffu);
    }
    m = team_max_u32<TEAM>(m, scratch);
    if (active && tid == 0)
        W.norms_out[b] = u2f(m);
}

// q bytes for an arbitrary level table.  The decision is the outcome of this sequence of IEEE fp64 operations (each
// rounded to nearest; the products of two fp32 values are exact):
//   e_t = l_t * ||v||;  j = largest t with e_t <= |v_i| (s+1: the top level, no draw);
//   tau = e_{j+1} - e_j;  x = |v_i| - e_j;  up iff u * tau < x * 2^24.
// On levels that are powers of two nothing rounds and this is the rule of the main quantizer.
template <int TEAM, int VPT>
__global__ __launch_bounds__(TeamGeom<TEAM>::kWG) void k_quantize_table(EncodeParams P, EncodeBatch Wk, LevelTable T)
{
    __shared__ double edges_all[TeamGeom<TEAM>::kTeamsPerWG][16];
    const EncodeWorker &W = Wk.w[blockIdx.y];
    const uint32_t tid = threadIdx.x % TEAM;
    const uint32_t team = threadIdx.x / TEAM;
    double *edges = edges_all[team];
    const uint64_t b = (uint64_t)blockIdx.x * TeamGeom<TEAM>::kTeamsPerWG + team;
    const bool active = b < P.nb;
    const uint64_t base = active ? b * P.bucket : 0;
    const uint32_t nbk = active ? (uint32_t)min((uint64_t)P.bucket, P.d - base) : 0u;
    const float *vb = W.v + base;
    uint8_t *qb = W.q_out + base;
    const bool aligned = (reinterpret_cast<uintptr_t>(vb) & 15u) == 0;
    const bool qaligned = (reinterpret_cast<uintptr_t>(qb) & 3u) == 0;
    const float nf = active ? W.norms_in[b] : 0.0f;
    const bool dead = !(nf > 0.0f) || !(nf < __builtin_huge_valf());
    if (tid < 16u)
        edges[tid] = (double)T.lev[tid] * (double)nf;
    team_barrier<TEAM>();
    const double e1 = edges[1];
    const BucketKey key = bucket_key(W.seed, b);
#pragma unroll 1
    for (uint32_t i = 0; i < P.rows; ++i) {
        const uint32_t vi = i * TEAM + tid;
        const uint32_t e0 = 4u * vi;
        const bool mine = e0 < nbk;                     // lanes beyond the bucket's end run along with zeros
        const float4 x = mine ? load_vec4(vb, vi, nbk, aligned) : float4{0.f, 0.f, 0.f, 0.f};
        const float xs[4] = {x.x, x.y, x.z, x.w};
        const float big = fmaxf(fmaxf(fabsf(xs[0]), fabsf(xs[1])), fmaxf(fabsf(xs[2]), fabsf(xs[3])));
        uint32_t levels = 0;
        if (!dead) {
            if (__all(!((double)big >= e1))) {          // every coordinate of every lane below the first level
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t u = draw24((key.k0 + e0 + (uint32_t)c) * kRngC1, key.k1);
                    const double a = (double)fabsf(xs[c]);
                    levels |= ((double)u * e1 < a * 16777216.0 ? 1u : 0u) << (8 * c);
                }
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t u = draw24((key.k0 + e0 + (uint32_t)c) * kRngC1, key.k1);
                    const double a = (double)fabsf(xs[c]);
                    uint32_t j = 0;
                    for (uint32_t t = 1; t <= P.s + 1u; ++t)
                        j += edges[t] <= a ? 1u : 0u;   // the levels increase: the count is the largest index
                    if (j <= P.s) {
                        const double lo = edges[j], hi = edges[j + 1u];
                        const double tau = hi - lo;
                        const double over = a - lo;
                        j += (double)u * tau < over * 16777216.0 ? 1u : 0u;
                    }
                    levels |= j << (8 * c);
                }
            }
        }
        const uint32_t v01 = __builtin_amdgcn_perm(f2u(xs[1]), f2u(xs[0]), 0x0c0c0703u);
        const uint32_t v23 = __builtin_amdgcn_perm(f2u(xs[3]), f2u(xs[2]), 0x0c0c0703u);
        const uint32_t sg = __builtin_amdgcn_perm(v23, v01, 0x05040100u);
        const uint32_t nz7 = (levels + 0x7f7f7f7fu) & 0x80808080u;
        const uint32_t packed = (sg & nz7) | levels;
        if (mine) {
            if (qaligned && e0 + 3u < nbk) {
                reinterpret_cast<uint32_t *>(qb)[vi] = packed;
            } else {
                for (uint32_t c = 0; c < 4u && e0 + c < nbk; ++c)
                    qb[e0 + c] = (uint8_t)(packed >> (8 * c));
            }
        }
    }
}

}  // namespace nuq
