// DECODE + dequantize + aggregate (App. A DECODE; Alg. 1 aggregate line).
//
// A workgroup owns a tile of consecutive output coordinates: whole buckets when the bucket is
// small, a run of sync segments of one bucket when it is large.  The tile's sum lives in LDS
// as fp64 (LDS fp64 atomic adds run ~20x faster than fp32 ones on this chip, and a sum of
// <= 32 fp32 values scaled by powers of two is exact in fp64 unless their exponents span
// more than 2^29).  The bit strings the tile needs are first copied to LDS with coalesced
// loads.  Each (worker, bucket, segment) bit string is then parsed by one lane, sequentially,
// as the format requires; the tile is finally scaled, rounded to fp32 and written out once.
//
// The parse loop is bound by instruction issue, so it is kept short: a 128-entry table indexed
// by the next seven stream bits resolves every Elias code of up to seven bits (values 1..15:
// all level indices and two thirds of the gaps) in one LDS read and gives the position and
// width of the last group of longer codes; format checks are accumulated and tested once.
#pragma once
#include "nuq_device.hpp"
#include "nuq_encode_kernels.hpp"

namespace nuq {

constexpr uint32_t kMaxWorkers = 32;
constexpr uint32_t kDecodeWG = 128;        // threads per workgroup
constexpr uint32_t kTileCoords = 2048;     // coordinates per workgroup tile (16 KB of fp64)
constexpr uint32_t kStageWords = 704;      // LDS words for staged bit strings
constexpr uint32_t kMaxStreams = 128;      // (bucket, worker) bit strings per tile
constexpr uint32_t kNoStage = 0xFFFFFFFFu;

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
    uint32_t buckets_per_tile;  // >= 1: the tile is this many whole buckets; 0: part of one bucket
    uint32_t tiles_per_bucket;  // >= 1
    uint32_t tile_coords;       // coordinates a full tile spans
    uint32_t segs_per_tile;     // segments of one bucket inside a tile
    float scale;
    int accumulate;
};

// Branch-free decoder of Alg. 2 for values below 65536 on a 32-bit window (MSB first).
// Code shapes: "0" -> 1;  "1x0" -> 2..3;  "1x 1y..y 0" -> 4..15 (group of x+1 bits);
// "1x 1y..y 1z..z 0" -> 16..65535 (group of y+1 bits).  `len` receives the code length
// (<= 23); returns false if the shape is none of these (a fourth group would follow).
__device__ __forceinline__ bool erc_decode_bits(uint32_t w, uint32_t &N, uint32_t &len)
{
    const uint32_t g1 = w >> 30;                       // 2 or 3 when the first bit is set
    const uint32_t k2 = g1 + 1u;                       // width of the second group
    const uint32_t o2 = 30u - k2;
    const uint32_t g2 = (w >> o2) & ((1u << k2) - 1u); // second group (leading bit set if present)
    const uint32_t k3 = g2 + 1u;                       // width of the third group (<= 16)
    const uint32_t o3 = o2 - min(k3, o2);
    const uint32_t g3 = (w >> o3) & ((1u << min(k3, 16u)) - 1u);
    const bool one = (w >> 31) == 0u;
    const bool two = ((w >> 29) & 1u) == 0u;           // terminator right after the first group
    const bool three = ((w >> (o2 - 1u)) & 1u) == 0u;  // terminator right after the second group
    N = one ? 1u : two ? g1 : three ? g2 : g3;
    len = one ? 1u : two ? 3u : three ? 3u + k2 : 3u + k2 + k3;
    const bool term_ok = one || two || three || (k3 <= 16u && o3 >= 1u && ((w >> (o3 - 1u)) & 1u) == 0u);
    return term_ok;
}

// Bit reader over a word array (LDS or global), MSB first, 64-bit buffer.
template <class WordPtr>
struct BitReader {
    WordPtr words;      // word 0 holds stream bit 0 of this reader's frame
    uint32_t next;      // next word to load
    uint32_t limit;     // words at or beyond this index read as zero
    uint64_t buf;       // upcoming bits, MSB aligned
    uint32_t cnt;       // valid bits in buf

    __device__ __forceinline__ void init(WordPtr w, uint32_t bit_pos, uint32_t limit_words)
    {
        words = w;
        limit = limit_words;
        next = bit_pos >> 5;
        const uint32_t bo = bit_pos & 31u;
        buf = 0;
        cnt = 0;
        refill();
        buf <<= bo;
        cnt -= bo;
        refill();
    }
    __device__ __forceinline__ void refill()
    {
        if (cnt <= 32u) {
            const uint32_t w = next < limit ? words[next] : 0u;
            ++next;
            buf |= (uint64_t)w << (32u - cnt);
            cnt += 32u;
        }
    }
    __device__ __forceinline__ uint32_t peek() const { return (uint32_t)(buf >> 32); }
    __device__ __forceinline__ void skip(uint32_t n)
    {
        buf <<= n;
        cnt -= n;
    }
};

// Parse one unit: the records of worker k's bucket b whose bits lie in [bit_lo, bit_hi)
// (offsets from the bucket's first bit), and add their values into the tile.
//   forced   : in-bucket index of the first record (>= 0 when entered through a sync entry,
//              whose gap code is then skipped), or -1 to start from the bucket's beginning
//   idx_lo/idx_hi : records below idx_lo are dropped (walks without an index), a record at or
//              above idx_hi is a format error
template <class WordPtr>
__device__ __forceinline__ void decode_unit(const DecodeParams &P, WordPtr words, uint32_t limit_words,
                                            uint32_t bit_lo, uint32_t bit_hi, int forced, uint32_t idx_lo,
                                            uint32_t idx_hi, double wnorm, double *tile, int tile_lo)
{
    BitReader<WordPtr> br;
    br.init(words, bit_lo, limit_words);
    uint32_t pos = bit_lo;
    int prev = -1;
    while (pos < bit_hi) {
        br.refill();
        uint32_t w = br.peek();
        uint32_t gap, lg, j, lj;
        bool ok = erc_decode_bits(w, gap, lg);
        w <<= lg;
        const uint32_t neg = w >> 31;
        w <<= 1;
        ok = erc_decode_bits(w, j, lj) && ok;
        const uint32_t len = lg + 1u + lj;
        int idx = prev + (int)gap;
        if (forced >= 0) {
            idx = forced;
            forced = -1;
        }
        if (!ok || len > 31u || pos + len > bit_hi || idx <= prev || (uint32_t)idx >= idx_hi || j < 1u ||
            j > P.s + 1u) {
            atomicOr(P.flags, kFlagMalformed);
            return;
        }
        if ((uint32_t)idx >= idx_lo) {
            // ||v|| * l_j = (||v|| * 2^(-1-s)) * 2^j, exact in fp64
            double val = ldexp(wnorm, (int)j);
            atomicAdd(&tile[idx - tile_lo], neg ? -val : val);
        }
        br.skip(len);
        pos += len;
        prev = idx;
    }
}

struct GlobalWords {
    const uint32_t *p;
    __device__ __forceinline__ uint32_t operator[](uint32_t i) const { return p[i]; }
};

// ---- seven-bit code table -------------------------------------------------------------
// Entry for the next seven stream bits p (MSB first):
//   short code (complete within the seven bits): bits 0..4 = code length, bits 5..9 = value
//   long code (three groups): bit 15 set, bits 0..4 = bits before the last group (5 or 6),
//   bits 5..9 = width of the last group (5..16); the value is that group, one 0 follows.
__device__ __forceinline__ uint32_t code_table_entry(uint32_t p)
{
    const uint32_t w = p << 25;
    uint32_t N, len;
    erc_decode_bits(w, N, len);
    if (len <= 7u)
        return len | (N << 5);
    const uint32_t k2 = (w >> 30) + 1u;                         // second group's width (3 or 4)
    const uint32_t g2 = (w >> (30u - k2)) & ((1u << k2) - 1u);  // second group = last group's width - 1
    return 0x8000u | (2u + k2) | ((g2 + 1u) << 5);
}

// Decode one Elias code from the window w with the table; returns the value, `len` its length.
__device__ __forceinline__ uint32_t table_decode(const uint16_t *lut, uint32_t w, uint32_t &len)
{
    const uint32_t e = lut[w >> 25];
    const uint32_t a = e & 31u;              // length, or bits before the last group
    const uint32_t v = (e >> 5) & 31u;       // value, or width of the last group
    const uint32_t big = ((w << a) >> 1) >> (31u - v);   // last group of a long code (v >= 5)
    const bool is_long = (e & 0x8000u) != 0u;
    len = is_long ? a + v + 1u : a;
    return is_long ? big : v;
}

// Fast parse of one unit from words held in `words` (LDS or global through the accessor).
// Reads are clamped to word index `last_word`; format violations set *bad and never leave
// [idx_lo, idx_hi) of the tile.
template <class WordPtr>
__device__ __forceinline__ void decode_unit_fast(WordPtr words, uint32_t last_word, const uint16_t *lut,
                                                 uint32_t bit_lo, uint32_t bit_hi, int forced, uint32_t idx_hi,
                                                 uint32_t smax, double wnorm, double *tile_at0, bool &bad)
{
    uint32_t next = bit_lo >> 5;
    const uint32_t bo = bit_lo & 31u;
    uint64_t buf = ((uint64_t)words[min(next, last_word)] << 32) | words[min(next + 1u, last_word)];
    next += 2u;
    buf <<= bo;
    uint32_t cnt = 64u - bo;
    int remaining = (int)(bit_hi - bit_lo);
    int prev = -1;
    if (forced >= 0 && remaining > 0) {       // entered through a sync entry: the first gap is replaced
        uint32_t lg;
        const uint32_t gap = table_decode(lut, (uint32_t)(buf >> 32), lg);
        prev = forced - (int)gap;
    }
    while (remaining > 0) {
        if (cnt <= 32u) {
            const uint32_t wd = words[min(next, last_word)];
            ++next;
            buf |= (uint64_t)wd << (32u - cnt);
            cnt += 32u;
        }
        const uint32_t w = (uint32_t)(buf >> 32);
        uint32_t lg, lj;
        const uint32_t gap = table_decode(lut, w, lg);
        const uint32_t w2 = w << lg;                      // sign bit on top
        const uint32_t j = table_decode(lut, w2 << 1, lj);
        const uint32_t len = lg + 1u + lj;
        uint32_t idx = (uint32_t)(prev + (int)gap);
        bad |= (idx >= idx_hi) | (j - 1u >= smax) | (len > 31u);
        idx = min(idx, idx_hi - 1u);
        // ||v|| * l_j = (||v|| * 2^(-1-s)) * 2^j, exact in fp64; the sign goes into the top bit
        const double mag = ldexp(wnorm, (int)min(j, 15u));
        const uint64_t vb = (uint64_t)__double_as_longlong(mag) ^ ((uint64_t)(w2 & 0x80000000u) << 32);
        atomicAdd(tile_at0 + idx, __longlong_as_double((long long)vb));
        buf <<= len;
        cnt -= len;
        remaining -= (int)len;
        prev = (int)idx;
    }
    bad |= remaining != 0;
}

__global__ __launch_bounds__(kDecodeWG) void k_decode_accumulate(DecodeParams P)
{
    __shared__ __align__(16) double tile[kTileCoords];
    __shared__ uint32_t stage[kStageWords];
    __shared__ uint32_t st_off[kMaxStreams + 1];  // exclusive prefix of staged words per stream
    __shared__ uint32_t st_bit0[kMaxStreams];     // first staged bit (multiple of 32), from the bucket's first bit
    __shared__ uint64_t st_src[kMaxStreams];      // global address of the first staged word
    __shared__ uint16_t lut[128];
    __shared__ uint32_t scan_scratch[2];

    // ---- which coordinates does this tile cover?
    uint64_t b0;        // first bucket of the tile
    uint32_t nbuck;     // buckets in the tile
    uint32_t in_lo;     // in-bucket index where the tile starts (tiles that are part of a bucket)
    if (P.buckets_per_tile) {
        b0 = (uint64_t)blockIdx.x * P.buckets_per_tile;
        nbuck = (uint32_t)min((uint64_t)P.buckets_per_tile, P.nb - b0);
        in_lo = 0;
    } else {
        b0 = blockIdx.x / P.tiles_per_bucket;
        nbuck = 1;
        in_lo = (blockIdx.x % P.tiles_per_bucket) * P.tile_coords;
    }
    const uint64_t c_lo = b0 * P.bucket + in_lo;
    const uint64_t c_hi = P.buckets_per_tile ? min(P.d, (b0 + nbuck) * (uint64_t)P.bucket)
                                             : min(P.d, min(c_lo + P.tile_coords, (b0 + 1) * (uint64_t)P.bucket));
    if (c_hi <= c_lo)   // a tile of the (short) last bucket that starts beyond the vector's end
        return;
    const uint32_t span = (uint32_t)(c_hi - c_lo);
    const uint32_t g0 = P.sync_shift ? (in_lo >> P.sync_shift) : 0u;                // first segment of the tile
    const bool partial = !P.buckets_per_tile;                                        // part of one bucket
    const bool walk = partial && !P.sync_shift;                                      // no index: walk from the start
    const uint32_t g1 = partial && P.sync_shift ? min(P.nseg, g0 + P.segs_per_tile) : P.nseg;   // one past the last
    const uint32_t tid = threadIdx.x;

    for (uint32_t i = tid; i < (span + 1u) / 2u; i += kDecodeWG)
        reinterpret_cast<double2 *>(tile)[i] = double2{0.0, 0.0};
    lut[tid] = (uint16_t)code_table_entry(tid);

    // ---- which words does each stream = (bucket in tile, worker) need?
    const uint32_t nstreams = nbuck * P.K;
    uint32_t my_words = 0;
    if (tid < nstreams) {
        const uint32_t k = tid % P.K;
        const uint64_t b = b0 + tid / P.K;
        const uint64_t start = (P.bit_off[k][b] + 31ull) & ~31ull;
        const uint64_t end = P.bit_off[k][b + 1];
        const uint32_t len = end > start ? (uint32_t)(end - start) : 0u;
        uint32_t lo = 0, hi = len;
        if (partial && P.sync_shift) {
            const uint32_t *sy = P.sync[k] + b * P.nsync;
            if (g0 > 0u)
                lo = min(sy[g0 - 1u] & 0x1FFFFFu, len);
            if (g1 < P.nseg)
                hi = min(sy[g1 - 1u] & 0x1FFFFFu, len);
        }
        const uint32_t w0 = lo >> 5;
        my_words = (hi > lo && !walk) ? ((hi + 31u) >> 5) - w0 : 0u;
        st_bit0[tid] = w0 << 5;
        st_src[tid] = reinterpret_cast<uint64_t>(P.words[k] + (start >> 5) + w0);
    }
    uint32_t total_words;
    const uint32_t my_off = team_exclusive_sum<kDecodeWG>(my_words, scan_scratch, total_words);
    if (tid < nstreams)
        st_off[tid] = my_off;
    if (tid == 0)
        st_off[nstreams] = total_words;
    __syncthreads();

    // ---- copy them to LDS: word i of the concatenation belongs to the stream found by bisection
    const uint32_t staged_words = min(total_words, kStageWords);
    for (uint32_t i = tid; i < staged_words; i += kDecodeWG) {
        uint32_t lo = 0, hi = nstreams;          // st_off[lo] <= i < st_off[hi]
        while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (st_off[mid] <= i)
                lo = mid;
            else
                hi = mid;
        }
        stage[i] = reinterpret_cast<const uint32_t *>(st_src[lo])[i - st_off[lo]];
    }
    __syncthreads();

    // ---- parse units: (bucket in tile, segment in tile, worker)
    const uint32_t segs = g1 - g0;
    const uint32_t units = nbuck * segs * P.K;
    const double wscale = ldexp(1.0, -1 - (int)P.s);
    bool bad = false;
    for (uint32_t u = tid; u < units; u += kDecodeWG) {
        const uint32_t k = u % P.K;
        const uint32_t r = u / P.K;
        const uint32_t g = g0 + r % segs;
        const uint32_t bi = r / segs;
        const uint64_t b = b0 + bi;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        const uint32_t sidx = bi * P.K + k;
        const uint64_t start = (P.bit_off[k][b] + 31ull) & ~31ull;
        const uint64_t end = P.bit_off[k][b + 1];
        const uint32_t len = end > start ? (uint32_t)(end - start) : 0u;
        uint32_t bit_lo = 0, bit_hi = len, idx_lo = 0, idx_hi = nbk;
        int forced = -1;
        if (P.sync_shift) {
            const uint32_t *sy = P.sync[k] + b * P.nsync;
            idx_lo = g << P.sync_shift;
            idx_hi = min(nbk, (g + 1u) << P.sync_shift);
            if (idx_lo >= nbk)
                continue;
            if (g > 0u) {
                const uint32_t e = sy[g - 1u];
                if (e & kSyncEmpty)
                    continue;
                bit_lo = e & 0x1FFFFFu;
                forced = (int)(idx_lo + ((e >> 21) & 0x3FFu));
            }
            if (g + 1u < P.nseg)
                bit_hi = sy[g] & 0x1FFFFFu;
            if (bit_lo > bit_hi || bit_hi > len || (forced >= 0 && (uint32_t)forced >= idx_hi)) {
                bad = true;
                continue;
            }
        } else if (walk) {
            idx_lo = in_lo;
            if (idx_lo >= nbk)
                continue;
        }
        if (bit_hi <= bit_lo)
            continue;
        const double wnorm = (double)P.norms[k][b] * wscale;
        const int tile_lo = partial ? (int)in_lo : -(int)(bi * P.bucket);
        if (walk) {
            // no index: parse the bucket from its first record in global memory, keep what lands in the tile
            GlobalWords gw{P.words[k] + (start >> 5)};
            const uint32_t hi_idx = min(nbk, in_lo + P.tile_coords);
            BitReader<GlobalWords> br;
            br.init(gw, 0, (len + 31u) >> 5);
            uint32_t pos = 0;
            int prev = -1;
            while (pos < len) {
                br.refill();
                uint32_t w = br.peek(), gap, lg, j, lj;
                bool ok = erc_decode_bits(w, gap, lg);
                w <<= lg;
                const uint32_t neg = w >> 31;
                w <<= 1;
                ok = erc_decode_bits(w, j, lj) && ok;
                const uint32_t rl = lg + 1u + lj;
                const int idx = prev + (int)gap;
                if (!ok || rl > 31u || pos + rl > len || (uint32_t)idx >= nbk || j < 1u || j > P.s + 1u) {
                    bad = true;
                    break;
                }
                if ((uint32_t)idx >= hi_idx)
                    break;
                if ((uint32_t)idx >= idx_lo) {
                    const double val = ldexp(wnorm, (int)j);
                    atomicAdd(&tile[idx - tile_lo], neg ? -val : val);
                }
                br.skip(rl);
                pos += rl;
                prev = idx;
            }
            continue;
        }
        const uint32_t so = st_off[sidx], se = st_off[sidx + 1u];
        const uint32_t bit0 = st_bit0[sidx];
        if (bit_lo < bit0 || bit_hi > bit0 + ((se - so) << 5)) {   // a sync index that is not monotone
            bad = true;
            continue;
        }
        double *tile_at0 = tile - tile_lo;       // address of in-bucket index 0 (never dereferenced outside the tile)
        if (se <= kStageWords) {
            decode_unit_fast(stage + so, se - so - 1u, lut, bit_lo - bit0, bit_hi - bit0, forced, idx_hi, P.s + 1u,
                             wnorm, tile_at0, bad);
        } else {                                  // did not fit in LDS: read the words from global memory
            GlobalWords gw{reinterpret_cast<const uint32_t *>(st_src[sidx])};
            decode_unit_fast(gw, se - so - 1u, lut, bit_lo - bit0, bit_hi - bit0, forced, idx_hi, P.s + 1u, wnorm,
                             tile_at0, bad);
        }
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
    __syncthreads();

    // ---- scale, round to fp32, write
    float *o = P.out + c_lo;
    const double sc = (double)P.scale;
    const bool vec = (reinterpret_cast<uintptr_t>(o) & 15u) == 0;
    if (vec) {
        const uint32_t n4 = span >> 2;
        for (uint32_t i = tid; i < n4; i += kDecodeWG) {
            const double2 a = reinterpret_cast<const double2 *>(tile)[2u * i];
            const double2 c = reinterpret_cast<const double2 *>(tile)[2u * i + 1u];
            float4 r;
            r.x = (float)(sc * a.x);
            r.y = (float)(sc * a.y);
            r.z = (float)(sc * c.x);
            r.w = (float)(sc * c.y);
            float4 *dst = reinterpret_cast<float4 *>(o) + i;
            if (P.accumulate) {
                const float4 old = *dst;
                r.x += old.x;
                r.y += old.y;
                r.z += old.z;
                r.w += old.w;
            }
            *dst = r;
        }
        for (uint32_t i = (n4 << 2) + tid; i < span; i += kDecodeWG) {
            const float r = (float)(sc * tile[i]);
            o[i] = P.accumulate ? o[i] + r : r;
        }
    } else {
        for (uint32_t i = tid; i < span; i += kDecodeWG) {
            const float r = (float)(sc * tile[i]);
            o[i] = P.accumulate ? o[i] + r : r;
        }
    }
}

}  // namespace nuq
