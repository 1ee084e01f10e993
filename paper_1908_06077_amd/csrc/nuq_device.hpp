// Device-side building blocks of the NUQSGD compression kernels (gfx950, wave64).
//
//   - counter hash for the rounding draws
//   - the exact nonuniform stochastic rounding rule (Def. 1, Sec. 3.1; App. B)
//   - Elias recursive coding of gaps and level indices (App. A, Alg. 2)
//   - team-wide reductions and scans (a "team" is the group of threads that owns one bucket)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace nuq {

constexpr int kWave = 64;

__device__ __forceinline__ uint32_t f2u(float x) { return __float_as_uint(x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __uint_as_float(x); }

// ---------------------------------------------------------------- rounding draws
//
// One 24-bit uniform integer per coordinate.  Per bucket the 64-bit mixer below turns
// (seed, bucket index) into two key words; per coordinate x = (k0 + i) * C1 is advanced by
// adding C1, then one xor-shift/multiply/xor-shift round absorbs k1.

constexpr uint32_t kRngC1 = 0x9E3779B1u;
constexpr uint32_t kRngC2 = 0x85EBCA6Bu;

struct BucketKey {
    uint32_t k0, k1;
};

__device__ __forceinline__ BucketKey bucket_key(uint64_t seed, uint64_t bucket_index)
{
    uint64_t z = seed + (bucket_index + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return BucketKey{(uint32_t)z, (uint32_t)(z >> 32)};
}

// x = (k0 + index) * C1 on entry.
__device__ __forceinline__ uint32_t draw24(uint32_t x, uint32_t k1)
{
    x = x ^ (x >> 15) ^ k1;
    x *= kRngC2;
    x ^= x >> 16;
    return x >> 8;
}

// ------------------------------------------------------------------- quantizer
//
// Levels l_0 = 0, l_j = 2^(j-1-s).  For a = |v_i| and the fp32 bucket norm N the rule is
//   j = largest index with l_j * N <= a;  a >= N -> s+1;
//   up to j+1  iff  u * (l_{j+1} - l_j) * N  <  (a - l_j * N) * 2^24   (real numbers).
// Integer view: with nS = N * 2^-s (a float, exponent field lowered by s), the bin of a
// is m = floor((bits(a) - bits(nS)) / 2^23): m < 0 is the bin below the first level,
// m >= s means a >= N.  lo = nS * 2^m and x = a - lo are exact floats, w = lo * 2^-24 (or
// nS * 2^-24 in the lowest bin) is an exact float, and one fused multiply-add
// t = fma(u, w, -x) rounds the exact value u*w - x once: rounding never changes the sign
// of a nonzero value (fp32 denormals are kept: the kernels run in IEEE denormal mode), so
// "up" is exactly "t < 0".  w must be a normal float for the scaling to be exact; norms
// below 2^-60 are handled by scaling the whole bucket by 2^100 first (a power of two:
// ratios are unchanged).  The same test without per-bin scales: a2 = a * 2^-m (the bits of
// nS plus the low 23 bits of the difference) lies in [nS, 2 nS), a2 - nS is exact, and
// t = fma(u, nS * 2^-24, -(a2 - nS)) is the t above divided by 2^m.

struct BucketScale {
    uint32_t ns_bits;  // bits of (prescaled) N * 2^-s
    uint32_t c_bits;   // bits of (prescaled) N * 2^(-s-24)
    float ns;          // the same as floats
    float ns2;         // 2 * ns (finite whenever s >= 1)
    float c;
    float prescale;    // 1 or 2^100
    int s;
    bool dead;         // zero or non-finite norm: every level is 0
};

__device__ __forceinline__ BucketScale make_scale(float norm, int s)
{
    BucketScale B;
    B.s = s;
    B.dead = !(norm > 0.0f) || !(norm < __builtin_huge_valf());
    B.prescale = 1.0f;
    if (norm < 0x1p-60f) {
        B.prescale = 0x1p100f;
        norm *= 0x1p100f;
    }
    B.ns_bits = f2u(norm) - ((uint32_t)s << 23);
    B.c_bits = B.ns_bits - (24u << 23);
    B.ns = u2f(B.ns_bits);
    B.ns2 = u2f(B.ns_bits + (1u << 23));
    B.c = u2f(B.c_bits);
    return B;
}

// ------------------------------------------------------------------------- ERC
//
// Alg. 2 for 1 <= N <= 65535: groups binary(N), binary(bits(N)-1), ... (values >= 2 only),
// last computed first, then one 0.  At most three groups, at most 23 bits.
// Returns the code right-aligned; `len` receives its length.
__device__ __forceinline__ uint32_t erc_code(uint32_t N, uint32_t &len)
{
    const uint32_t w0 = 32u - (uint32_t)__clz((int)N);
    uint32_t code = N, l = w0;
    if (w0 >= 3u) {
        const uint32_t n1 = w0 - 1u, w1 = 32u - (uint32_t)__clz((int)n1);
        code |= n1 << l;
        l += w1;
        if (w1 >= 3u) {
            code |= (w1 - 1u) << l;
            l += 2u;
        }
    }
    if (N == 1u) {
        len = 1u;
        return 0u;
    }
    len = l + 1u;
    return code << 1;
}

// Decoder of Alg. 2 on a 32-bit window (MSB first) holding `avail` valid bits.
// Consumes the code from the window.  Returns false if the code does not end inside the
// window or a group is wider than 24 bits.
__device__ __forceinline__ bool erc_decode_window(uint32_t &win, int &avail, uint32_t &N)
{
    N = 1u;
#pragma unroll 1
    for (int it = 0; it < 6; ++it) {
        if (avail < 1)
            return false;
        if ((win >> 31) == 0u) {
            win <<= 1;
            avail -= 1;
            return true;
        }
        const int k = (int)N + 1;
        if (k > avail || k > 24)
            return false;
        N = win >> (32 - k);
        win <<= k;
        avail -= k;
    }
    return false;
}

// ------------------------------------------------------- team reductions / scans
//
// TEAM threads (16, 64, 256 or 1024) own one bucket.  A workgroup holds max(256, TEAM) threads,
// i.e. 16 teams of a quarter wave (a DPP row) each, 4 one-wave teams or a single multi-wave team.
// Multi-wave variants use a small LDS scratch and __syncthreads(); every thread of the workgroup must
// call them.  A quarter-wave team serves small buckets: the per-bucket work that a wave does once
// (norm reduction, scale, hash key, scans) then serves four buckets at a time.
constexpr int kRow = 16;   // lanes of a DPP row

// A value that is the same in every thread of a team, as a scalar when the team is at least a wave.
template <int TEAM>
__device__ __forceinline__ uint32_t team_uniform_u32(uint32_t x)
{
    if constexpr (TEAM >= 64)
        return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
    else
        return x;
}
template <int TEAM>
__device__ __forceinline__ float team_uniform_f32(float x)
{
    return u2f(team_uniform_u32<TEAM>(f2u(x)));
}

// The value lane 15 of each DPP row holds, in every lane of that row.
__device__ __forceinline__ uint32_t row_last_u32(uint32_t x)
{
    return (uint32_t)__shfl((int)x, (int)((threadIdx.x & (kWave - 1)) | (kRow - 1)), kWave);
}

// Value of a wave-uniform quantity as a scalar (lets the compiler keep what derives from it in
// scalar registers and branch on it without touching the exec mask).
__device__ __forceinline__ uint32_t uniform_u32(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
}
__device__ __forceinline__ uint64_t uniform_u64(uint64_t x)
{
    return ((uint64_t)uniform_u32((uint32_t)(x >> 32)) << 32) | uniform_u32((uint32_t)x);
}
__device__ __forceinline__ float uniform_f32(float x) { return u2f(uniform_u32(f2u(x))); }

// Sum of x over the 64 lanes of a wave, returned in every lane: DPP row shifts and row
// broadcasts leave the total in lane 63, which is then read as a scalar.
__device__ __forceinline__ double wave_sum_f64(double x)
{
    auto step = [](double v, auto ctrl, auto row_mask, auto bound) {
        const uint64_t b = (uint64_t)__double_as_longlong(v);
        const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, decltype(ctrl)::value,
                                                                  decltype(row_mask)::value, 0xf, decltype(bound)::value);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), decltype(ctrl)::value,
                                                                  decltype(row_mask)::value, 0xf, decltype(bound)::value);
        return v + __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
    };
    using std::integral_constant;
    x = step(x, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});
    x = step(x, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});
    x = step(x, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});
    x = step(x, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{});
    x = step(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{}, integral_constant<bool, false>{});
    x = step(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{}, integral_constant<bool, false>{});
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, kWave - 1);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), kWave - 1);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// Sum of x over each row of 16 lanes, returned in every lane of the row: four row shifts leave the total in the
// row's last lane (the same summation order for every bucket), which is then handed to the others.
__device__ __forceinline__ double row_sum_f64(double x)
{
    auto step = [](double v, auto ctrl) {
        const uint64_t b = (uint64_t)__double_as_longlong(v);
        const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, decltype(ctrl)::value, 0xf, 0xf, true);
        const uint32_t hi =
            (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), decltype(ctrl)::value, 0xf, 0xf, true);
        return v + __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
    };
    using std::integral_constant;
    x = step(x, integral_constant<int, 0x111>{});
    x = step(x, integral_constant<int, 0x112>{});
    x = step(x, integral_constant<int, 0x114>{});
    x = step(x, integral_constant<int, 0x118>{});
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = row_last_u32((uint32_t)b), hi = row_last_u32((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

template <int TEAM>
__device__ __forceinline__ double team_sum_f64(double x, double *scratch /* TEAM/64 doubles */)
{
    if constexpr (TEAM == kRow)
        return row_sum_f64(x);
    x = wave_sum_f64(x);
    if constexpr (TEAM > kWave) {
        constexpr int NW = TEAM / kWave;
        const int wave = (threadIdx.x % TEAM) / kWave;
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0)
            scratch[wave] = x;
        __syncthreads();
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w)
            t += scratch[w];
        x = t;
    }
    return x;
}

// Inclusive prefix sum across the 64 lanes of a wave with DPP moves: four row-shift steps scan
// each row of 16 lanes, two row-broadcast steps carry the row totals forward.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2, 3
    return v;
}

// Exclusive prefix sum over the team in thread order; `total` receives the team sum.
template <int TEAM>
__device__ __forceinline__ uint32_t team_exclusive_sum(uint32_t v, uint32_t *scratch /* TEAM/64 */,
                                                       uint32_t &total)
{
    if constexpr (TEAM == kRow) {
        uint32_t inc = v;
        inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x111, 0xf, 0xf, true);   // row_shr:1
        inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x112, 0xf, 0xf, true);   // row_shr:2
        inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x114, 0xf, 0xf, true);   // row_shr:4
        inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x118, 0xf, 0xf, true);   // row_shr:8
        total = row_last_u32(inc);
        return inc - v;
    }
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t inc = wave_inclusive_sum(v);
    if constexpr (TEAM == kWave) {
        total = (uint32_t)__builtin_amdgcn_readlane((int)inc, kWave - 1);
        return inc - v;
    } else {
        constexpr int NW = TEAM / kWave;
        const int wave = (threadIdx.x % TEAM) / kWave;
        __syncthreads();
        if (lane == kWave - 1)
            scratch[wave] = inc;
        __syncthreads();
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t t = scratch[w];
            before += (w < wave) ? t : 0u;
            all += t;
        }
        total = all;
        return before + inc - v;
    }
}

// Exclusive running maximum over the team in thread order (identity = `ident`).
template <int TEAM>
__device__ __forceinline__ int team_exclusive_max(int v, int ident, int *scratch /* TEAM/64 */)
{
    if constexpr (TEAM == kRow) {
        const int l = threadIdx.x & (kRow - 1);
        int inc = v;
#pragma unroll
        for (int off = 1; off < kRow; off <<= 1) {
            const int t = __shfl_up(inc, off, kRow);
            if (l >= off)
                inc = max(inc, t);
        }
        const int exc = __shfl_up(inc, 1, kRow);
        return l == 0 ? ident : exc;
    }
    const int lane = threadIdx.x & (kWave - 1);
    int inc = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(inc, off, kWave);
        if (lane >= off)
            inc = max(inc, t);
    }
    int exc = __shfl_up(inc, 1, kWave);
    if (lane == 0)
        exc = ident;
    if constexpr (TEAM > kWave) {
        constexpr int NW = TEAM / kWave;
        const int wave = (threadIdx.x % TEAM) / kWave;
        __syncthreads();
        if (lane == kWave - 1)
            scratch[wave] = inc;
        __syncthreads();
        int before = ident;
#pragma unroll
        for (int w = 0; w < NW; ++w)
            before = (w < wave) ? max(before, scratch[w]) : before;
        exc = max(exc, before);
    }
    return exc;
}

// --------------------------------------------------------- level tables (arbitrary level sequences)
//
// Def. 1 for any 0 = l_0 < l_1 < ... < l_{s+1} = 1 (Sec. 3.1 before the special case; Sec. 4.1 "Generally spaced
// levels").  With e_t = l_t * ||v|| (a product of two fp32 values: exact in fp64) and j = the largest t with
// e_t <= |v_i| (s+1: the top level, no draw), the coordinate goes up iff u (e_{j+1} - e_j) < (|v_i| - e_j) 2^24
// over the real numbers (table_round_up).  On levels that are powers of two this is the rule of the main quantizer.

struct LevelTable {
    float lev[16];   // lev[0] = 0 ... lev[s+1] = 1; entries above s+1 are 0
};

// Maximum of x over the team; every thread returns it.  scratch: 16 words of LDS (teams of several waves).
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

// The rounding decision of Def. 1 for a coordinate a in [lo, hi), lo = l_j ||v||, hi = l_{j+1} ||v|| (both exact
// in fp64), and the draw u: up iff u (hi - lo) < (a - lo) 2^24 over the real numbers.  The two differences and the
// product round once each in fp64 (relative error below 2^-52 on the left, 2^-53 on the right), so the rounded
// comparison is the real one unless the sides agree to within 2^-49; only then (about one coordinate in 2^49) is
// the sign of  a 2^24 - lo 2^24 - u hi + u lo  worked out exactly: each product as a pair (rounded value, fma
// remainder), the six terms added one by one to a list of nonoverlapping doubles by error-free additions, whose
// leading nonzero entry has the sign of the sum.
__device__ __forceinline__ void exact_add(double x, double y, double &hi, double &lo)
{
    hi = x + y;
    const double yv = hi - x;
    lo = (x - (hi - yv)) + (y - yv);
}

__device__ inline bool table_round_up_exact(double ud, double lo, double hi, double a)
{
    double t[6];
    t[0] = a * 16777216.0;
    t[1] = -lo * 16777216.0;
    t[2] = -ud * hi;
    t[3] = __builtin_fma(-ud, hi, -t[2]);
    t[4] = ud * lo;
    t[5] = __builtin_fma(ud, lo, -t[4]);
    // after step i the entries t[0..i] sum to the same value as before and do not overlap, smallest first
#pragma unroll
    for (int i = 1; i < 6; ++i) {
        double carry = t[i];
#pragma unroll
        for (int k = 0; k < i; ++k)
            exact_add(carry, t[k], carry, t[k]);
        t[i] = carry;
    }
    double lead = 0.0;
#pragma unroll
    for (int k = 0; k < 6; ++k)
        lead = t[k] != 0.0 ? t[k] : lead;
    return lead > 0.0;
}

__device__ __forceinline__ bool table_round_up(uint32_t u, double lo, double hi, double a)
{
    const double ud = (double)u;
    const double rhs = (a - lo) * 16777216.0;           // >= 0, and 0 or above 2^-300: a sits in [lo, hi)
    const double diff = ud * (hi - lo) - rhs;
    bool up = diff < 0.0;
    // near-tie: the exponent of the difference is 49 or more below the right-hand side's, read off the high words
    // (a gap of 49 exponents exceeds 48 << 20 whatever the mantissa bits beside them; a zero difference has high
    // word 0; a zero right-hand side, an exact a = lo, is never flagged and stays down as it should)
    const int hd = __double2hiint(diff) & 0x7fffffff, hr = __double2hiint(rhs);
    if (__builtin_expect(hr - hd >= (48 << 20), 0))
        up = table_round_up_exact(ud, lo, hi, a);
    return up;
}

// Level|sign bytes of four coordinates whose first has in-bucket index idx0 (+ k0), for the bucket whose edges
// e_t = l_t * ||v|| lie in LDS (e1 = edges[1]).  Called by whole waves: the first-bin route is chosen per wave.
__device__ __forceinline__ uint32_t quantize_table_vec4(const float4 &x, uint32_t counter0, uint32_t k1,
                                                        const double *edges, double e1, uint32_t s, bool dead)
{
    const float xs[4] = {x.x, x.y, x.z, x.w};
    const float big = fmaxf(fmaxf(fabsf(xs[0]), fabsf(xs[1])), fmaxf(fabsf(xs[2]), fabsf(xs[3])));
    uint32_t levels = 0;
    if (!dead) {
        if (__all(!((double)big >= e1))) {          // every coordinate of every lane below the first level
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t u = draw24((counter0 + (uint32_t)c) * kRngC1, k1);
                const double a = (double)fabsf(xs[c]);
                levels |= (table_round_up(u, 0.0, e1, a) ? 1u : 0u) << (8 * c);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t u = draw24((counter0 + (uint32_t)c) * kRngC1, k1);
                const double a = (double)fabsf(xs[c]);
                uint32_t j = 0;
                for (uint32_t t = 1; t <= s + 1u; ++t)
                    j += edges[t] <= a ? 1u : 0u;   // the levels increase: the count is the largest index
                if (j <= s) {
                    j += table_round_up(u, edges[j], edges[j + 1u], a) ? 1u : 0u;
                }
                levels |= j << (8 * c);
            }
        }
    }
    // sign bytes of the four coordinates, kept where the level is not zero (a level is below 128)
    const uint32_t v01 = __builtin_amdgcn_perm(f2u(xs[1]), f2u(xs[0]), 0x0c0c0703u);
    const uint32_t v23 = __builtin_amdgcn_perm(f2u(xs[3]), f2u(xs[2]), 0x0c0c0703u);
    const uint32_t sg = __builtin_amdgcn_perm(v23, v01, 0x05040100u);
    const uint32_t nz7 = (levels + 0x7f7f7f7fu) & 0x80808080u;
    return (sg & nz7) | levels;
}

}  // namespace nuq
