// Level-table quantizer and maximum norm: Def. 1 for an arbitrary level sequence 0 = l_0 < l_1 < ... < l_{s+1} = 1
// (Sec. 3.1 before the special case; Sec. 4.1 "Generally spaced levels": the exponential family (0, p^s, ..., p, 1),
// uniform levels = QSGD) and the normalization of QSGDinf (Sec. 1, Sec. 2).  Everything else of the path (ENCODE,
// DECODE) is shared: a level index is coded the same way whatever its value.
#pragma once

#include "nuq_encode_kernels.hpp"

namespace nuq {

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

// q bytes for an arbitrary level table (quantize_table_vec4), one bucket per team.
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
        const uint32_t packed = quantize_table_vec4(x, key.k0 + e0, key.k1, edges, e1, P.s, dead);
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
