// DECODE + dequantize + aggregate (App. A DECODE; Alg. 1 aggregate line).
//
// A workgroup owns a tile of consecutive output coordinates (whole buckets when the bucket is
// small, a run of sync segments of one bucket when it is large) and keeps the tile's fp32 sum
// in LDS.  Each (worker, bucket, segment) bit string is parsed by one lane, sequentially, as the
// format requires; lanes add their dequantized values into the tile with LDS float atomics;
// the tile is then written out once, coalesced.
#pragma once
#include "nuq_device.hpp"
#include "nuq_encode_kernels.hpp"

namespace nuq {

constexpr uint32_t kMaxWorkers = 32;
constexpr uint32_t kTileMax = 8192;   // coordinates per workgroup tile (32 KB of LDS)

struct DecodeParams {
    const float *norms[kMaxWorkers];
    const uint64_t *bit_off[kMaxWorkers];
    const uint32_t *words[kMaxWorkers];
    const uint32_t *sync[kMaxWorkers];
    float *out;
    uint32_t *flags;
    uint64_t d;
    uint64_t nb;
    uint32_t K;
    uint32_t bucket;
    uint32_t s;
    uint32_t sync_shift;        // log2 stride, 0 = none
    uint32_t nsync;
    uint32_t nseg;              // segments per bucket (nsync + 1)
    uint32_t buckets_per_tile;  // >= 1 when bucket <= kTileMax, else 0
    uint32_t tiles_per_bucket;  // >= 1
    uint32_t tile_coords;       // coordinates a tile spans (full tiles)
    uint32_t segs_per_tile;     // segments of one bucket inside a tile (large buckets)
    float scale;
    int accumulate;
};

// 32 stream bits starting at bit `pos` (MSB first); bits at or after `end` read as zero and
// no word at or after `end` is touched.
__device__ __forceinline__ uint32_t peek32(const uint32_t *words, uint64_t pos, uint64_t end)
{
    const uint64_t wi = pos >> 5;
    const uint32_t bo = (uint32_t)pos & 31u;
    const uint32_t hi = words[wi];
    const uint32_t lo = (bo != 0u && ((wi + 1) << 5) < end) ? words[wi + 1] : 0u;
    return bo ? (hi << bo) | (lo >> (32u - bo)) : hi;
}

// Parse the records of one segment of one worker's bucket and add their values into `tile`.
//   seg_lo/seg_hi : in-bucket index range this lane is responsible for
//   tile_lo       : in-bucket index of tile[0]
__device__ __forceinline__ void decode_segment(const DecodeParams &P, uint32_t k, uint64_t b,
                                               uint32_t g, uint32_t nbk, uint32_t seg_lo,
                                               uint32_t seg_hi, float *tile, int tile_lo)
{
    const uint64_t start = (P.bit_off[k][b] + 31ull) & ~31ull;
    const uint64_t end = P.bit_off[k][b + 1];
    if (end <= start)
        return;
    uint64_t pos = start;
    int prev = -1;
    int forced = -1;   // position of the first record when entering through a sync entry
    if (g > 0u) {
        if (P.sync_shift) {
            const uint32_t e = P.sync[k][b * P.nsync + g - 1u];
            if (e == kSyncEmpty)
                return;
            pos = start + (e & 0x1FFFFFu);
            forced = (int)((g << P.sync_shift) + ((e >> 21) & 0x3FFu));
            if (pos >= end || forced >= (int)nbk) {
                atomicOr(P.flags, kFlagMalformed);
                return;
            }
        }
        // without a sync index the lane walks from the bucket's first record and drops
        // everything below seg_lo
    }
    const float nrm = P.norms[k][b];
    const uint32_t *words = P.words[k];
    while (pos < end) {
        const uint64_t left = end - pos;
        int avail = left < 32 ? (int)left : 32;
        const int avail0 = avail;
        uint32_t win = peek32(words, pos, end);
        uint32_t gap, j;
        bool ok = erc_decode_window(win, avail, gap);
        ok = ok && avail >= 1;
        const uint32_t neg = win >> 31;
        win <<= 1;
        avail -= 1;
        ok = ok && erc_decode_window(win, avail, j);
        int idx = prev + (int)gap;
        if (forced >= 0) {
            idx = forced;
            forced = -1;
        }
        if (!ok || idx >= (int)nbk || idx <= prev || j < 1u || j > P.s + 1u) {
            atomicOr(P.flags, kFlagMalformed);
            return;
        }
        if ((uint32_t)idx >= seg_hi)
            return;
        if ((uint32_t)idx >= seg_lo) {
            // ||v|| * l_j with l_j = 2^(j-1-s): an exact power-of-two scaling
            float val = ldexpf(nrm, (int)j - 1 - (int)P.s);
            atomicAdd(&tile[idx - tile_lo], neg ? -val : val);
        }
        pos += (uint64_t)(avail0 - avail);
        prev = idx;
    }
}

__global__ __launch_bounds__(256) void k_decode_accumulate(DecodeParams P)
{
    extern __shared__ __align__(16) float tile[];
    // Which coordinates does this tile cover?
    uint64_t b0;        // first bucket of the tile
    uint32_t nbuck;     // buckets in the tile (small buckets) or 1
    uint32_t in_lo;     // in-bucket index where the tile starts (large buckets)
    if (P.buckets_per_tile) {
        b0 = (uint64_t)blockIdx.x * P.buckets_per_tile;
        nbuck = (uint32_t)min((uint64_t)P.buckets_per_tile, P.nb - b0);
        in_lo = 0;
    } else {
        b0 = blockIdx.x / P.tiles_per_bucket;
        nbuck = 1;
        in_lo = (blockIdx.x % P.tiles_per_bucket) * P.tile_coords;
    }
    const uint64_t c_lo = b0 * P.bucket + in_lo;                       // first coordinate
    const uint64_t c_hi = P.buckets_per_tile
                              ? min(P.d, (b0 + nbuck) * (uint64_t)P.bucket)
                              : min(P.d, min(c_lo + P.tile_coords, (b0 + 1) * (uint64_t)P.bucket));
    if (c_hi <= c_lo)   // a tile of the (short) last bucket that starts beyond the vector's end
        return;
    const uint32_t span = (uint32_t)(c_hi - c_lo);
    for (uint32_t i = threadIdx.x; i < span; i += blockDim.x)
        tile[i] = 0.0f;
    __syncthreads();

    // Parse units: (bucket in tile, segment in tile, worker).
    const uint32_t segs = P.buckets_per_tile ? P.nseg : P.segs_per_tile;
    const uint32_t units = nbuck * segs * P.K;
    for (uint32_t u = threadIdx.x; u < units; u += blockDim.x) {
        const uint32_t k = u % P.K;
        const uint32_t r = u / P.K;
        const uint32_t sg = r % segs;
        const uint64_t b = b0 + r / segs;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        uint32_t g, seg_lo, seg_hi;
        if (P.sync_shift) {
            g = (in_lo >> P.sync_shift) + sg;
            seg_lo = g << P.sync_shift;
            seg_hi = min(nbk, (g + 1u) << P.sync_shift);
        } else if (P.buckets_per_tile) {
            g = 0;
            seg_lo = 0;
            seg_hi = nbk;
        } else {                          // large bucket without an index: walk from the start
            g = in_lo ? 1u : 0u;
            seg_lo = in_lo;
            seg_hi = min(nbk, in_lo + P.tile_coords);
        }
        if (seg_lo >= nbk)
            continue;
        const int tile_lo = P.buckets_per_tile ? -(int)((b - b0) * P.bucket) : (int)in_lo;
        decode_segment(P, k, b, g, nbk, seg_lo, seg_hi, tile, tile_lo);
    }
    __syncthreads();
    float *o = P.out + c_lo;
    for (uint32_t i = threadIdx.x; i < span; i += blockDim.x) {
        const float val = P.scale * tile[i];
        o[i] = P.accumulate ? o[i] + val : val;
    }
}

}  // namespace nuq
