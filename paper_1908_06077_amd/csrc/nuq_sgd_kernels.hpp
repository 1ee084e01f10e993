// Parameter update of Alg. 1 with the momentum rule of Sec. 4.2 and the moment sums behind the mean normalized
// variance of App. J.  The plain aggregate step of Alg. 1 (w <- w - (alpha/K) sum_k Q_k) needs no kernel of its own:
// it is the decoder's accumulate mode with scale = -alpha/K and out = w.  All three kernels here are streaming,
// HBM-bound passes: 16-byte accesses when the pointers allow, one rounding per stored value.
#pragma once

#include <cstdint>
#include <hip/hip_runtime.h>

namespace nuq {

struct MomentumParams {
    float *w;        // [d] parameters, updated in place
    float *yl;       // [d] y^l of the previous step, replaced by this step's
    const float *g;  // [d] averaged gradient
    uint64_t d;
    double alpha, mu, l;
};

// y = w - alpha g;  y^l = w - l alpha g;  w <- y + mu (y^l - y^l_prev);  y^l_prev <- y^l  (Sec. 4.2).
// Evaluated in fp64 in that order from the fp32 inputs, each result rounded to fp32 once.
__device__ __forceinline__ void momentum_one(float &w, float &yl, float g, double alpha, double la, double mu)
{
    const double wd = (double)w, gd = (double)g;
    const double y = wd - alpha * gd;
    const double ylv = wd - la * gd;
    w = (float)(y + mu * (ylv - (double)yl));
    yl = (float)ylv;
}

template <bool kVec>
__global__ __launch_bounds__(256) void k_momentum_step(MomentumParams P)
{
    const double la = P.l * P.alpha;
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if constexpr (kVec) {
        const uint64_t i = t * 4u;
        if (i + 4u <= P.d) {
            float4 w = *reinterpret_cast<const float4 *>(P.w + i);
            float4 yl = *reinterpret_cast<const float4 *>(P.yl + i);
            const float4 g = *reinterpret_cast<const float4 *>(P.g + i);
            momentum_one(w.x, yl.x, g.x, P.alpha, la, P.mu);
            momentum_one(w.y, yl.y, g.y, P.alpha, la, P.mu);
            momentum_one(w.z, yl.z, g.z, P.alpha, la, P.mu);
            momentum_one(w.w, yl.w, g.w, P.alpha, la, P.mu);
            *reinterpret_cast<float4 *>(P.w + i) = w;
            *reinterpret_cast<float4 *>(P.yl + i) = yl;
        } else {
            for (uint64_t j = i; j < P.d; ++j)
                momentum_one(P.w[j], P.yl[j], P.g[j], P.alpha, la, P.mu);
        }
    } else if (t < P.d) {
        momentum_one(P.w[t], P.yl[t], P.g[t], P.alpha, la, P.mu);
    }
}

// sum[i] += g[i], sumsq[i] += g[i]^2 in fp64: the per-coordinate first and second moments over the draws of a
// gradient estimate (App. J).  The products of fp32 values are exact in fp64.
template <bool kVec>
__global__ __launch_bounds__(256) void k_moments_accumulate(const float *g, double *sum, double *sumsq, uint64_t d)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if constexpr (kVec) {
        const uint64_t i = t * 2u;
        if (i + 2u <= d) {
            const float2 x = *reinterpret_cast<const float2 *>(g + i);
            double2 a = *reinterpret_cast<const double2 *>(sum + i);
            double2 b = *reinterpret_cast<const double2 *>(sumsq + i);
            a.x += (double)x.x;
            a.y += (double)x.y;
            b.x += (double)x.x * (double)x.x;
            b.y += (double)x.y * (double)x.y;
            *reinterpret_cast<double2 *>(sum + i) = a;
            *reinterpret_cast<double2 *>(sumsq + i) = b;
        } else if (i < d) {
            const double x = (double)g[i];
            sum[i] += x;
            sumsq[i] += x * x;
        }
    } else if (t < d) {
        const double x = (double)g[t];
        sum[t] += x;
        sumsq[t] += x * x;
    }
}

constexpr uint32_t kVarianceBlocks = 1024;  // partial pairs written by k_variance_partials

// Block p sums, over its grid-stride share of the coordinates, the variance  sumsq_i/M - (sum_i/M)^2  and the second
// moment  sumsq_i/M  across the M draws, and stores the pair at partial[2p], partial[2p+1].
__global__ __launch_bounds__(256) void k_variance_partials(const double *sum, const double *sumsq, uint64_t d,
                                                           double inv_m, double *partial)
{
    __shared__ double red[2][4];
    double var = 0.0, sec = 0.0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < d; i += (uint64_t)gridDim.x * 256u) {
        const double m1 = sum[i] * inv_m, m2 = sumsq[i] * inv_m;
        var += m2 - m1 * m1;
        sec += m2;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        var += __shfl_down(var, off, 64);
        sec += __shfl_down(sec, off, 64);
    }
    if (threadIdx.x % 64u == 0) {
        red[0][threadIdx.x / 64u] = var;
        red[1][threadIdx.x / 64u] = sec;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        partial[2u * blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        partial[2u * blockIdx.x + 1u] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

// out2[0] = sum of the variance partials, out2[1] = sum of the second-moment partials, in a fixed order
// (one workgroup, tree over 256 lanes), so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void k_variance_finish(const double *partial, uint32_t n, double *out2)
{
    __shared__ double red[2][4];
    double var = 0.0, sec = 0.0;
    for (uint32_t p = threadIdx.x; p < n; p += 256u) {
        var += partial[2u * p];
        sec += partial[2u * p + 1u];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        var += __shfl_down(var, off, 64);
        sec += __shfl_down(sec, off, 64);
    }
    if (threadIdx.x % 64u == 0) {
        red[0][threadIdx.x / 64u] = var;
        red[1][threadIdx.x / 64u] = sec;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        out2[0] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        out2[1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

}  // namespace nuq
