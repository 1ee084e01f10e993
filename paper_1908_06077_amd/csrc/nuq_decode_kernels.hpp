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
// The parse loop is bound by instruction issue and by the latency of its dependent LDS reads,
// so it is kept short: the window at the current bit position comes from one two-word LDS
// read, a 128-entry table indexed by the next seven stream bits resolves every gap code of up
// to seven bits (values 1..15) and gives position and width of the last group of longer ones,
// the level code is taken apart with byte permutes, and format checks are accumulated and
// tested once.  Every metadata load of a tile (offsets, sync entries, norms) is issued before
// the first wait.
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

struct WalkWords {
    const uint32_t *p;
    __device__ __forceinline__ uint32_t operator[](uint32_t i) const { return p[i]; }
};

struct GlobalWords {
    const uint32_t *p;
    uint32_t last;      // highest readable word index
    __device__ __forceinline__ void pair(uint32_t i, uint32_t &hi, uint32_t &lo) const
    {
        hi = p[min(i, last)];
        lo = p[min(i + 1u, last)];
    }
};

// Words staged in LDS; the staging area is padded so that word i + 1 of any staged word i exists.
struct StagedWords {
    const uint32_t *p;
    __device__ __forceinline__ void pair(uint32_t i, uint32_t &hi, uint32_t &lo) const
    {
        hi = p[i];
        lo = p[i + 1u];
    }
};

// ---- gap code table --------------------------------------------------------------------
// Entry for the next seven stream bits p (MSB first), as fields of five bits each:
//   bits  0..4   length of the whole code
//   bits  5..9   position (from the LSB of a 32-bit window) of the last group of a three-group code
//   bits 10..14  width of that group (5..16), 0 for a code complete within the seven bits
//   bits 15..19  value of a code complete within the seven bits (1..15), else 0
// so that value = field3 + bitfield(window, field1, field2) for every code of up to three groups.
__device__ __forceinline__ uint32_t gap_table_entry(uint32_t p)
{
    const uint32_t w = p << 25;
    uint32_t N, len;
    erc_decode_bits(w, N, len);
    if (len <= 7u)
        return len | (N << 15);
    const uint32_t k2 = (w >> 30) + 1u;                         // second group's width (3 or 4)
    const uint32_t g2 = (w >> (30u - k2)) & ((1u << k2) - 1u);  // second group = last group's width - 1
    const uint32_t a = 2u + k2, v = g2 + 1u;
    return (a + v + 1u) | ((32u - a - v) << 5) | (v << 10);
}

// Parse the records in bits [bit_lo, bit_hi) of a unit's frame and add their values into the tile.
//   forced : in-bucket index of the first record when the unit was entered through a sync entry
//            (its gap code is then only skipped), or -1 to start from the bucket's beginning
//   idx_hi : a record at or above this index is a format error; smax = s + 1
// Format violations set `bad`; nothing is ever added outside [0, idx_hi) of the bucket.
//
// One iteration per record, kept short because the loop is bound by instruction issue: the
// 32-bit window at the current position is rebuilt from two adjacent words, the gap comes from
// one table read, and the level code (at most seven bits: 0 | 1x0 | 101yy0 | 111yyy0) is taken
// apart with byte-permute lookups on its first three bits.
template <class Words>
__device__ __forceinline__ void decode_unit_fast(const Words &words, const uint32_t *lut, uint32_t bit_lo,
                                                 uint32_t bit_hi, int forced, uint32_t idx_hi, uint32_t smax,
                                                 double wnorm, double *tile_at0, bool &bad)
{
    uint32_t pos = bit_lo;
    int prev = -1;
    if (forced >= 0 && pos < bit_hi) {
        uint32_t hi, lo;
        words.pair(pos >> 5, hi, lo);
        const uint32_t w = (uint32_t)(((((uint64_t)hi << 32) | lo) << (pos & 31u)) >> 32);
        const uint32_t e = lut[w >> 25];
        const uint32_t gap = (e >> 15) + __builtin_amdgcn_ubfe(w, (e >> 5) & 31u, (e >> 10) & 31u);
        prev = forced - (int)gap;
    }
    while (pos < bit_hi) {
        uint32_t hi, lo;
        words.pair(pos >> 5, hi, lo);
        const uint32_t w = (uint32_t)(((((uint64_t)hi << 32) | lo) << (pos & 31u)) >> 32);
        const uint32_t e = lut[w >> 25];
        const uint32_t lg = e & 31u;
        const uint32_t gap = (e >> 15) + __builtin_amdgcn_ubfe(w, (e >> 5) & 31u, (e >> 10) & 31u);
        const uint32_t w2 = w << lg;                 // sign bit on top, level code below
        const uint32_t c = w2 << 1;
        const uint32_t sel = (c >> 29) | 0x0c0c0c00u;
        const uint32_t lj = __builtin_amdgcn_perm(0x07030603u, 0x01010101u, sel);    // code length
        const uint32_t off = __builtin_amdgcn_perm(0x1a1e1b1eu, 0u, sel);            // where its last group sits
        const uint32_t wd = __builtin_amdgcn_perm(0x04020302u, 0u, sel);             // and how wide it is
        const uint32_t j1 = __builtin_amdgcn_perm(0u, 0x01010101u, sel);             // the code "0"
        const uint32_t j = j1 | __builtin_amdgcn_ubfe(c, off, wd);
        const uint32_t unterminated = __builtin_amdgcn_ubfe(c, (off - 1u) & 31u, 1u);   // a third group would follow
        uint32_t idx = (uint32_t)(prev + (int)gap);
        bad |= (idx >= idx_hi) | (j > smax) | (unterminated != 0u);
        idx = min(idx, idx_hi - 1u);
        // ||v|| * l_j = (||v|| * 2^(-1-s)) * 2^j, exact in fp64; the sign goes into the top bit
        const double mag = ldexp(wnorm, (int)j);
        const uint32_t mh = (uint32_t)((uint64_t)__double_as_longlong(mag) >> 32);
        const uint32_t vh = (mh & 0x7fffffffu) | (w2 & 0x80000000u);
        const uint64_t vb = ((uint64_t)vh << 32) | (uint32_t)__double_as_longlong(mag);
        atomicAdd(tile_at0 + idx, __longlong_as_double((long long)vb));
        pos += lg + 1u + lj;
        prev = (int)idx;
    }
    bad |= pos != bit_hi;
}

// Metadata of one parse unit = (bucket in tile, segment, worker), as loaded from memory.
struct UnitRaw {
    uint64_t bo0, bo1;      // bit_off[b], bit_off[b + 1]
    uint32_t e_lo, e_hi;    // sync entries that bound the segment (0 when not applicable)
    float norm;
};

__global__ __launch_bounds__(kDecodeWG) void k_decode_accumulate(DecodeParams P)
{
    __shared__ __align__(16) double tile[kTileCoords];
    __shared__ uint32_t stage[kStageWords + 2];
    __shared__ uint32_t st_off[kMaxStreams + 1];  // exclusive prefix of staged words per stream
    __shared__ uint32_t st_bit0[kMaxStreams];     // first staged bit (multiple of 32), from the bucket's first bit
    __shared__ uint64_t st_src[kMaxStreams];      // global address of the first staged word
    __shared__ uint32_t lut[128];
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
    const uint32_t nstreams = nbuck * P.K;        // stream = (bucket in tile, worker)
    const uint32_t segs = g1 - g0;
    const uint32_t units = nstreams * segs;       // unit = (bucket in tile, segment, worker)

    // Unit u's worker, bucket and segment, and its metadata loads (all independent of each other).
    auto unit_coords = [&](uint32_t u, uint32_t &k, uint32_t &bi, uint32_t &g) {
        k = u % P.K;
        const uint32_t r = u / P.K;
        g = g0 + r % segs;
        bi = r / segs;
    };
    auto load_unit = [&](uint32_t u) {
        uint32_t k, bi, g;
        unit_coords(u, k, bi, g);
        const uint64_t b = b0 + bi;
        UnitRaw r;
        r.bo0 = P.bit_off[k][b];
        r.bo1 = P.bit_off[k][b + 1];
        r.norm = P.norms[k][b];
        r.e_lo = r.e_hi = 0;
        if (P.sync_shift) {
            const uint32_t *sy = P.sync[k] + b * P.nsync;
            if (g > 0u)
                r.e_lo = sy[g - 1u];
            if (g + 1u < P.nseg)
                r.e_hi = sy[g];
        }
        return r;
    };

    // ---- issue this thread's metadata loads: its stream's extent and its first unit
    uint64_t s_bo0 = 0, s_bo1 = 0;
    uint32_t s_e0 = 0, s_e1 = 0;
    uint32_t s_k = 0;
    uint64_t s_b = 0;
    if (tid < nstreams) {
        s_k = tid % P.K;
        s_b = b0 + tid / P.K;
        s_bo0 = P.bit_off[s_k][s_b];
        s_bo1 = P.bit_off[s_k][s_b + 1];
        if (partial && P.sync_shift) {
            const uint32_t *sy = P.sync[s_k] + s_b * P.nsync;
            if (g0 > 0u)
                s_e0 = sy[g0 - 1u];
            if (g1 < P.nseg)
                s_e1 = sy[g1 - 1u];
        }
    }
    UnitRaw first{};
    if (tid < units)
        first = load_unit(tid);

    for (uint32_t i = tid; i < (span + 1u) / 2u; i += kDecodeWG)
        reinterpret_cast<double2 *>(tile)[i] = double2{0.0, 0.0};
    lut[tid] = gap_table_entry(tid);

    // ---- which words does each stream need?
    uint32_t my_words = 0;
    if (tid < nstreams) {
        const uint64_t start = (s_bo0 + 31ull) & ~31ull;
        const uint32_t len = s_bo1 > start ? (uint32_t)(s_bo1 - start) : 0u;
        uint32_t lo = 0, hi = len;
        if (partial && P.sync_shift) {
            if (g0 > 0u)
                lo = min(s_e0 & 0x1FFFFFu, len);
            if (g1 < P.nseg)
                hi = min(s_e1 & 0x1FFFFFu, len);
        }
        const uint32_t w0 = lo >> 5;
        my_words = (hi > lo && !walk) ? ((hi + 31u) >> 5) - w0 : 0u;
        st_bit0[tid] = w0 << 5;
        st_src[tid] = reinterpret_cast<uint64_t>(P.words[s_k] + (start >> 5) + w0);
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
    if (tid < 2u)
        stage[staged_words + tid] = 0u;          // the parser reads one word past the one it is in
    __syncthreads();

    // ---- parse units
    const double wscale = ldexp(1.0, -1 - (int)P.s);
    bool bad = false;
    for (uint32_t u = tid; u < units; u += kDecodeWG) {
        const UnitRaw m = u == tid ? first : load_unit(u);
        uint32_t k, bi, g;
        unit_coords(u, k, bi, g);
        const uint64_t b = b0 + bi;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        const uint32_t sidx = bi * P.K + k;
        const uint64_t start = (m.bo0 + 31ull) & ~31ull;
        const uint32_t len = m.bo1 > start ? (uint32_t)(m.bo1 - start) : 0u;
        uint32_t bit_lo = 0, bit_hi = len, idx_lo = 0, idx_hi = nbk;
        int forced = -1;
        if (P.sync_shift) {
            idx_lo = g << P.sync_shift;
            idx_hi = min(nbk, (g + 1u) << P.sync_shift);
            if (idx_lo >= nbk)
                continue;
            if (g > 0u) {
                if (m.e_lo & kSyncEmpty)
                    continue;
                bit_lo = m.e_lo & 0x1FFFFFu;
                forced = (int)(idx_lo + ((m.e_lo >> 21) & 0x3FFu));
            }
            if (g + 1u < P.nseg)
                bit_hi = m.e_hi & 0x1FFFFFu;
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
        const double wnorm = (double)m.norm * wscale;
        const int tile_lo = partial ? (int)in_lo : -(int)(bi * P.bucket);
        if (walk) {
            // no index: parse the bucket from its first record in global memory, keep what lands in the tile
            WalkWords gw{P.words[k] + (start >> 5)};
            const uint32_t hi_idx = min(nbk, in_lo + P.tile_coords);
            BitReader<WalkWords> br;
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
            decode_unit_fast(StagedWords{stage + so}, lut, bit_lo - bit0, bit_hi - bit0, forced, idx_hi, P.s + 1u,
                             wnorm, tile_at0, bad);
        } else {                                  // did not fit in LDS: read the words from global memory
            GlobalWords gw{reinterpret_cast<const uint32_t *>(st_src[sidx]), se - so - 1u};
            decode_unit_fast(gw, lut, bit_lo - bit0, bit_hi - bit0, forced, idx_hi, P.s + 1u, wnorm, tile_at0, bad);
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
