// DECODE + dequantize + aggregate (App. A DECODE; Alg. 1 aggregate line).
//
// The output is cut into tiles of consecutive coordinates: whole buckets when the bucket is
// small, a run of sync segments of one bucket when it is large.  A tile's sum lives in LDS as
// fp64 (LDS fp64 atomic adds run ~20x faster than fp32 ones on this chip, and a sum of <= 32
// fp32 values scaled by powers of two is exact in fp64 unless their exponents span more than
// 2^29).  The bit strings a tile needs are copied to LDS, each (worker, bucket, segment) bit
// string -- a unit -- is parsed by one lane, sequentially, as the format requires, and the
// tile is finally scaled, rounded to fp32 and written out once.
//
// LDS capacity bounds the number of tiles in flight, a lone wave issues a dependent
// instruction only every nine cycles or so, and a tile's life would mostly be spent waiting on
// memory (offsets and sync entries first, then the words they point to) and on bookkeeping.  So
// a workgroup is persistent, walks a strided sequence of tiles, and its two waves have
// different jobs: the first parses tile t while the second prepares tile t+1 -- works out
// which words each unit needs, fetches them into registers, leaves a three-word plan per unit
// in LDS -- and has the metadata loads of tile t+2 in flight.  When the parse is over the
// fetched words go to the LDS staging area and both waves write tile t out and clear it.  The critical path of a tile is its
// parse and its write-out.
#pragma once
#include "nuq_device.hpp"
#include "nuq_encode_kernels.hpp"
#include "nuq_sgd_kernels.hpp"

namespace nuq {

constexpr uint32_t kMaxWorkers = 32;
constexpr uint32_t kDecodeWG = 128;        // threads per workgroup: a parsing wave and a preparing wave
constexpr uint32_t kTileCoords = 2048;     // coordinates per tile (16 KB of fp64) ...
constexpr uint32_t kTileCoordsBig = 4096;  // ... or, for few workers and large buckets, twice that (see the launcher)
constexpr uint32_t kWordsPerLane = 8;      // staged words each lane of the preparing wave carries
constexpr uint32_t kStageWords = kWave * kWordsPerLane;   // LDS words per staging buffer
constexpr uint32_t kMaxStreams = 64;       // (bucket, worker) bit strings per tile
constexpr uint32_t kPlanned = 2 * kWave;   // units of a tile that are planned ahead (two per preparing lane)

struct DecodeParams {
    const float *norms[kMaxWorkers];
    const uint64_t *bit_off[kMaxWorkers];
    const uint32_t *words[kMaxWorkers];
    uint64_t words_bits[kMaxWorkers];   // 32 * the words each message holds: no offset may point beyond
    const uint32_t *sync[kMaxWorkers];
    float *out;
    uint32_t *flags;
    uint64_t d;
    uint64_t nb;
    uint32_t ntiles;
    uint32_t K;
    uint32_t bucket;
    uint32_t s;
    uint32_t sync_shift;        // Huffman-coded messages: log2 of the coordinates per piece
    uint32_t pieces_shift;      // log2 of the index pieces per 2048-coordinate block
    uint32_t nsync;             // index entries per bucket, 0 = no index
    uint32_t nseg;              // units per bucket and worker: the pieces of the index (nsync), or 1 without one
    uint32_t buckets_per_tile;  // >= 1: the tile is this many whole buckets; 0: part of one bucket
    uint32_t tiles_per_bucket;  // >= 1
    uint32_t tile_coords;       // coordinates a full tile spans
    uint32_t segs_per_tile;     // pieces of one bucket inside a tile
    uint32_t xcd_base, xcd_rem; // ntiles / 8, ntiles % 8: see xcd_tile
    uint32_t lanes_shift;       // log2 of the lanes that copy one stream's words
    uint32_t stream_cap;        // words the lanes of a stream carry = kWordsPerLane << lanes_shift
    uint32_t stream_stride;     // LDS words per stream: stream_cap, or stream_cap - 1 (odd) for tiles of many streams
    float scale;
    float *yl;                  // kUpdateMomentum: y^l of the previous step, replaced by this step's
    double alpha, la, mu;       // kUpdateMomentum: step size, l * step size, momentum parameter
    float lev[16];              // level-table variant: l_0 = 0 .. l_{s+1} = 1
};

// Workgroup w walks the sequence w, w + grid, w + 2 grid, ... of [0, ntiles).  Workgroups are handed to the eight
// XCDs (each with an L2 of its own) in turn, and the grid is a multiple of eight whenever a workgroup takes more
// than one tile, so every element v of a workgroup's sequence has v mod 8 = the workgroup's XCD.  Element v is
// therefore mapped to tile number (v / 8) of the (v mod 8)'th of eight contiguous runs of tiles: neighbouring tiles,
// which share the cache lines at the ends of their parts of a bit string and their bucket's offsets and sync
// entries, are decoded under the same L2.  A bijection of [0, ntiles) whatever the placement really is.
__device__ __forceinline__ uint32_t xcd_tile(const DecodeParams &P, uint32_t v)
{
    const uint32_t x = v & 7u;
    return x * P.xcd_base + min(x, P.xcd_rem) + (v >> 3);
}

// What the decoder (template parameter UPDATE) does with r = fp32(scale * sum over workers) of a coordinate:
//   kUpdateWrite     out = r
//   kUpdateAdd       out = out + r   (the aggregate step of Alg. 1 when out = w and scale = -alpha/K)
//   kUpdateMomentum  (out, yl) <- momentum rule of Sec. 4.2 with g = r (out = w)
constexpr int kUpdateWrite = 0, kUpdateAdd = 1, kUpdateMomentum = 2;

// A full, 16-byte aligned tile of TC coordinates: every thread handles TC/4/kDecodeWG float4 groups, two at a time, with the
// loads of the old values issued before the LDS reads so that their latencies overlap.
template <int UPDATE, uint32_t TC, uint32_t WG = kDecodeWG>
__device__ __forceinline__ void apply_full_tile(const DecodeParams &P, double *tile, float *o, float *y, uint32_t tid)
{
    constexpr uint32_t kFull = TC / 4u / WG;                      // float4 groups per thread
    const double sc = (double)P.scale;
#pragma unroll
    for (uint32_t r0 = 0; r0 < kFull; r0 += 2u) {
        float4 w[2], yv[2];
        double2 a[2], c[2];
#pragma unroll
        for (uint32_t r = 0; r < 2u; ++r) {
            const uint32_t i = tid + (r0 + r) * WG;
            if constexpr (UPDATE != kUpdateWrite)
                w[r] = reinterpret_cast<const float4 *>(o)[i];
            if constexpr (UPDATE == kUpdateMomentum)
                yv[r] = reinterpret_cast<const float4 *>(y)[i];
        }
#pragma unroll
        for (uint32_t r = 0; r < 2u; ++r) {
            double2 *src = reinterpret_cast<double2 *>(tile) + 2u * (tid + (r0 + r) * WG);
            a[r] = src[0];
            c[r] = src[1];
            src[0] = double2{0.0, 0.0};
            src[1] = double2{0.0, 0.0};
        }
#pragma unroll
        for (uint32_t r = 0; r < 2u; ++r) {
            const uint32_t i = tid + (r0 + r) * WG;
            const float4 v{(float)(sc * a[r].x), (float)(sc * a[r].y), (float)(sc * c[r].x), (float)(sc * c[r].y)};
            if constexpr (UPDATE == kUpdateWrite) {
                store_once4(reinterpret_cast<float4 *>(o) + i, v);     // written once, not read here again
            } else if constexpr (UPDATE == kUpdateAdd) {
                reinterpret_cast<float4 *>(o)[i] = float4{v.x + w[r].x, v.y + w[r].y, v.z + w[r].z, v.w + w[r].w};
            } else {
                momentum_one(w[r].x, yv[r].x, v.x, P.alpha, P.la, P.mu);
                momentum_one(w[r].y, yv[r].y, v.y, P.alpha, P.la, P.mu);
                momentum_one(w[r].z, yv[r].z, v.z, P.alpha, P.la, P.mu);
                momentum_one(w[r].w, yv[r].w, v.w, P.alpha, P.la, P.mu);
                reinterpret_cast<float4 *>(o)[i] = w[r];
                reinterpret_cast<float4 *>(y)[i] = yv[r];
            }
        }
    }
}

template <int UPDATE>
__device__ __forceinline__ void apply4(const DecodeParams &P, float4 r, float4 *dst, float4 *ydst)
{
    if constexpr (UPDATE == kUpdateWrite) {
        *dst = r;
        return;
    }
    float4 w = *dst;
    if constexpr (UPDATE == kUpdateAdd) {
        w.x = r.x + w.x;
        w.y = r.y + w.y;
        w.z = r.z + w.z;
        w.w = r.w + w.w;
    } else {
        float4 yv = *ydst;
        momentum_one(w.x, yv.x, r.x, P.alpha, P.la, P.mu);
        momentum_one(w.y, yv.y, r.y, P.alpha, P.la, P.mu);
        momentum_one(w.z, yv.z, r.z, P.alpha, P.la, P.mu);
        momentum_one(w.w, yv.w, r.w, P.alpha, P.la, P.mu);
        *ydst = yv;
    }
    *dst = w;
}


// Output stage of a tile: scale the sums, round to fp32, apply to the output (write, add, or momentum rule), and
// leave the tile zeroed.  Called by all WG threads of the workgroup.
template <int UPDATE, uint32_t TC, uint32_t WG>
__device__ __forceinline__ void tile_output(const DecodeParams &P, double *tile, uint64_t c_lo, uint32_t span, uint32_t tid)
{
    float *o = P.out + c_lo;
    float *y = UPDATE == kUpdateMomentum ? P.yl + c_lo : o;      // (read only under kUpdateMomentum)
    const bool vec = ((reinterpret_cast<uintptr_t>(o) | reinterpret_cast<uintptr_t>(y)) & 15u) == 0;
    const uint32_t n4 = vec ? span >> 2 : 0u;
    if (n4 == TC / 4u) {
        apply_full_tile<UPDATE, TC, WG>(P, tile, o, y, tid);
    } else {
        const double sc = (double)P.scale;
        for (uint32_t i = tid; i < n4; i += WG) {
            double2 *src = reinterpret_cast<double2 *>(tile) + 2u * i;
            const double2 a = src[0], c = src[1];
            src[0] = double2{0.0, 0.0};
            src[1] = double2{0.0, 0.0};
            const float4 r{(float)(sc * a.x), (float)(sc * a.y), (float)(sc * c.x), (float)(sc * c.y)};
            apply4<UPDATE>(P, r, reinterpret_cast<float4 *>(o) + i, reinterpret_cast<float4 *>(y) + i);
        }
    }
    for (uint32_t i = (n4 << 2) + tid; i < span; i += WG) {      // (n4 = 0 without 16-byte alignment)
        const float r = (float)((double)P.scale * tile[i]);
        tile[i] = 0.0;
        if constexpr (UPDATE == kUpdateMomentum)
            momentum_one(o[i], y[i], r, P.alpha, P.la, P.mu);
        else
            o[i] = UPDATE == kUpdateAdd ? o[i] + r : r;
    }
}

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

// Word sources for the parser.  at(q) returns word q - 1 of the unit's frame (word 0 holds its bit 0); what it
// returns for a word that does not exist is never looked at.
struct GlobalWords {
    const uint32_t *p;
    uint32_t last;      // highest readable word index
    __device__ __forceinline__ uint32_t at(uint32_t q) const { return p[min(max(q, 1u) - 1u, last)]; }
};

// Words staged in LDS.  `p` points one word before the frame; the staging area is padded at both ends so
// that every word the parser can ask for exists.
struct StagedWords {
    const uint32_t *p;
    __device__ __forceinline__ uint32_t at(uint32_t q) const { return p[q]; }
};

// ---- gap code table --------------------------------------------------------------------
// Entry for the next seven stream bits p (MSB first):
//   bits  0..4   length of the whole code (its first two groups fix it)
//   bits  5..9   width of the last group of a three-group code (5..16), 0 for a code complete within the
//                seven bits; that group ends one bit before the code does
//   bits 10..13  value of a code complete within the seven bits (1..15), else 0
// so that value = field2 + bitfield(window, 33 - length, width) for every code of up to three groups.
__device__ __forceinline__ uint32_t gap_table_entry(uint32_t p)
{
    const uint32_t w = p << 25;
    uint32_t N, len;
    erc_decode_bits(w, N, len);
    if (len <= 7u)
        return len | (N << 10);
    const uint32_t k2 = (w >> 30) + 1u;                         // second group's width (3 or 4)
    const uint32_t g2 = (w >> (30u - k2)) & ((1u << k2) - 1u);  // second group = last group's width - 1
    const uint32_t a = 2u + k2, v = g2 + 1u;
    return (a + v + 1u) | (v << 5);
}

// value of the gap code at the top of window w, given its table entry
__device__ __forceinline__ uint32_t gap_value(uint32_t w, uint32_t e)
{
    return (e >> 10) + __builtin_amdgcn_ubfe(w, 33u - (e & 31u), (e >> 5) & 31u);
}

// Parse the records in bits [bit_lo, bit_hi) of a unit's frame and add their values into the tile.
//   forced : in-bucket index of the first record when the unit was entered through a sync entry
//            (its gap code is then only skipped), or -1 to start from the bucket's beginning
//   idx_hi : a record at or above this index is a format error
// Format violations set `bad`; nothing is ever added outside [0, idx_hi) of the bucket.
//
// ---- level code table ------------------------------------------------------------------
// Entry for the seven stream bits p after a record's sign bit (MSB first): the level index 1..smax (smax = s + 1
// <= 15), or 0 for what the message cannot hold: a larger index, or no code that ends within the seven bits (a
// third group would follow: an index above 15).
__device__ __forceinline__ uint32_t level_table_entry(uint32_t p, uint32_t smax)
{
    uint32_t N, len;
    erc_decode_bits(p << 25, N, len);
    return len <= 7u && N <= smax ? N : 0u;
}

// One iteration per record.  A lone wave issues an instruction every five cycles or so, a dependent one every
// nine, and an LDS read takes ~64, so the loop is kept short (format checks are folded into two running values
// and tested once) and is arranged around its one carried dependency, the bit position.  It is
// software-pipelined by hand so that the two LDS reads on that chain are covered by other work:
//   chain 1 : the 32-bit window at the position from two adjacent words through one funnel shift (position + 31
//             is the loop variable: its word index names the second word of the pair, its complement is the
//             shift); the table read for the gap code is issued.  The two words and the one after them are
//             held in registers: a record is at most 31 bits (gap code <= 23, sign, level code <= 7), so the
//             pair moves on by one word at most, and the word that then enters was requested an iteration
//             ago: no read of stream words is on the chain
//   cover   : level and value of the previous record (its level table entry was requested an iteration ago), its
//             add into the tile
//   chain 2 : gap code's length from the entry; the level table read is issued (nothing on the chain waits for
//             it); level code's length from a byte permute on its first three bits (the code is at most seven
//             bits: 0 | 1x0 | 101yy0 | 111yyy0); next position; the pair moves on if the position's word index
//             did, and the word after the pair is requested
//   cover   : this record's gap value and index, loop control
//
// kTable: the value of level j is wnorm * lev[j] (an arbitrary level sequence, lev in LDS) instead of
// wnorm * 2^j (wnorm = ||v|| * 2^(-1-s)); both are exact in fp64.
// Where a decoded value goes.  TileSink: the fp64 tile in LDS that sums the workers (at0 = address of the
// bucket's index 0).  DirectSink: a single message has nothing to sum: fp32(scale * value), the same rounding the
// tile's output stage applies to a sum of one term, stored or added straight into the output.
struct TileSink {
    double *at0;
    __device__ __forceinline__ void add(uint32_t idx, double v) const { atomicAdd(at0 + idx, v); }
};
template <int UPDATE>
struct DirectSink {
    float *at0;
    double scale;
    __device__ __forceinline__ void add(uint32_t idx, double v) const
    {
        const float r = (float)(scale * v);
        if constexpr (UPDATE == kUpdateAdd)
            at0[idx] = r + at0[idx];
        else
            at0[idx] = r;
    }
};

template <bool kTable, class Words, class Sink>
__device__ __forceinline__ void decode_unit_fast(const Words &words, const uint16_t *lut, const uint8_t *lut_level,
                                                 const float *lev, uint32_t bit_lo, uint32_t bit_hi, int forced,
                                                 uint32_t idx_hi, double wnorm, const Sink &sink, bool &bad)
{
    uint32_t p31 = bit_lo + 31u;
    const uint32_t end31 = bit_hi + 31u;
    if (p31 >= end31) {
        bad |= p31 != end31;
        return;
    }
    uint32_t q = p31 >> 5;
    uint32_t hi = words.at(q), lo = words.at(q + 1u), nx = words.at(q + 2u);
    int prev = -1;
    uint32_t w, e;                  // window, gap entry
    uint32_t idx, w2, e2;           // what an iteration leaves for the first cover step of the next: index, window
                                    // at the sign bit, level entry (in flight)
    uint32_t last_i = 0;            // index before clamping: non-decreasing, so the last one tells if any was too big
    uint32_t min_j = 1;             // smallest table entry met: 0 marks a level code the message cannot hold

    auto chain1 = [&]() {
        w = __builtin_amdgcn_alignbit(hi, lo, ~p31);
        e = lut[w >> 25];
    };
    auto chain2 = [&]() {
        const uint32_t lg = e & 31u;
        w2 = w << lg;                            // sign bit on top, level code below
        e2 = lut_level[(w2 >> 24) & 0x7fu];
        const uint32_t sel = ((w2 >> 28) & 7u) | 0x0c0c0c00u;
        const uint32_t lj1 = __builtin_amdgcn_perm(0x08040704u, 0x02020202u, sel);   // sign bit + level code
        p31 += lg + lj1;                         // by 31 at most
        const uint32_t qn = p31 >> 5;
        const bool moved = qn != q;
        hi = moved ? lo : hi;
        lo = moved ? nx : lo;
        q = qn;
        nx = words.at(qn + 2u);
    };
    auto cover_index = [&]() {
        uint32_t i = (uint32_t)(prev + (int)gap_value(w, e));
        if (forced >= 0) {                       // entered through a sync entry: its index replaces the first gap
            i = (uint32_t)forced;
            forced = -1;
        }
        last_i = i;
        idx = min(i, idx_hi - 1u);
        prev = (int)idx;
    };
    auto cover_value = [&]() {
        const uint32_t j = e2;
        min_j = min(min_j, j);
        // ||v|| * l_j = (||v|| * 2^(-1-s)) * 2^j, exact in fp64; the sign goes into the top bit
        double mag;
        if constexpr (kTable)
            mag = wnorm * (double)lev[j];
        else
            mag = ldexp(wnorm, (int)j);
        const uint32_t mh = (uint32_t)((uint64_t)__double_as_longlong(mag) >> 32);
        const uint32_t vh = (mh & 0x7fffffffu) | (w2 & 0x80000000u);
        const uint64_t vb = ((uint64_t)vh << 32) | (uint32_t)__double_as_longlong(mag);
        sink.add(idx, __longlong_as_double((long long)vb));
    };

    chain1();
    chain2();
    cover_index();
    while (p31 < end31) {
        chain1();
        __builtin_amdgcn_sched_barrier(0);
        cover_value();
        __builtin_amdgcn_sched_barrier(0);
        chain2();
        __builtin_amdgcn_sched_barrier(0);
        cover_index();
    }
    cover_value();
    bad |= (p31 != end31) | (last_i >= idx_hi) | (min_j == 0u);
}

// Where a tile lies.  Everything here is uniform over the workgroup.
struct TileGeom {
    uint64_t b0;        // first bucket
    uint64_t c_lo;      // first coordinate
    uint32_t nbuck;     // buckets in the tile (0 for a tile that starts beyond the vector's end)
    uint32_t in_lo;     // in-bucket index where the tile starts (tiles that are part of a bucket)
    uint32_t span;      // coordinates
    uint32_t g0, g1;    // segments [g0, g1) of each bucket
    uint32_t nstreams;  // stream = (bucket in tile, worker)
    uint32_t units;     // unit = (bucket in tile, segment, worker)
};

__device__ __forceinline__ TileGeom tile_geom(const DecodeParams &P, uint32_t t)
{
    TileGeom G;
    if (P.buckets_per_tile) {
        G.b0 = (uint64_t)t * P.buckets_per_tile;
        G.nbuck = (uint32_t)min((uint64_t)P.buckets_per_tile, P.nb - G.b0);
        G.in_lo = 0;
    } else {
        G.b0 = t / P.tiles_per_bucket;
        G.nbuck = 1;
        G.in_lo = (t % P.tiles_per_bucket) * P.tile_coords;
    }
    G.c_lo = G.b0 * P.bucket + G.in_lo;
    const uint64_t c_hi = P.buckets_per_tile ? min(P.d, (G.b0 + G.nbuck) * (uint64_t)P.bucket)
                                             : min(P.d, min(G.c_lo + P.tile_coords, (G.b0 + 1) * (uint64_t)P.bucket));
    G.span = c_hi > G.c_lo ? (uint32_t)(c_hi - G.c_lo) : 0u;
    if (G.span == 0u)        // a tile of the (short) last bucket that starts beyond the vector's end
        G.nbuck = 0;
    const bool partial = !P.buckets_per_tile;
    G.g0 = P.nsync ? (G.in_lo >> kSyncBlockShift) << P.pieces_shift : 0u;
    G.g1 = partial && P.nsync ? min(P.nseg, G.g0 + P.segs_per_tile) : P.nseg;
    G.nstreams = G.nbuck * P.K;
    G.units = G.nstreams * (G.g1 - G.g0);
    return G;
}

// What a lane loads for the stream whose words it helps to copy.
struct StreamRaw {
    uint64_t bo0, bo1;      // bit_off[b], bit_off[b + 1]
    uint32_t e0, e1;        // sync entries at the tile's first and one-past-last segment (partial tiles)
};

// The part of a stream's bit string a tile needs.
struct StreamPart {
    uint64_t first_word;    // index into the worker's words[] of the first word needed
    uint32_t bit0;          // its first bit, from the bucket's first bit (multiple of 32)
    uint32_t nwords;        // words needed
    uint32_t len;           // the bucket's bit length
};

// Offsets that run backwards, leave the worker's words (limit = 32 * their count) or span 2^21 bits or more set
// `bad` and give an empty part: nothing is then read from words[].
__device__ __forceinline__ StreamPart stream_part(const DecodeParams &P, const TileGeom &G, uint64_t bo0, uint64_t bo1,
                                                  uint32_t e0, uint32_t e1, uint64_t limit, bool &bad)
{
    StreamPart S;
    const uint64_t start = (bo0 + 31ull) & ~31ull;
    const bool wrong = bo1 < bo0 || bo1 > limit || (bo1 > start && bo1 - start > (uint64_t)kSyncOffMask);
    bad |= wrong;
    S.len = bo1 > start && !wrong ? (uint32_t)(bo1 - start) : 0u;
    uint32_t lo = 0, hi = S.len;
    if (!P.buckets_per_tile && P.nsync) {
        lo = min(e0 & kSyncOffMask, S.len);
        if (G.g1 < P.nseg)
            hi = min(e1 & kSyncOffMask, S.len);
    }
    const uint32_t w0 = lo >> 5;
    S.bit0 = w0 << 5;
    S.nwords = hi > lo ? ((hi + 31u) >> 5) - w0 : 0u;
    S.first_word = (start >> 5) + w0;
    return S;
}

// What a lane loads for a unit.
struct UnitRaw {
    uint64_t bo0, bo1;      // bit_off[b], bit_off[b + 1]
    uint32_t e_lo, e_hi;    // sync entries that bound the segment
    uint32_t e0, e1;        // sync entries that bound the tile (as in StreamRaw)
    float norm;
};

// A unit ready to parse.  kind: 0 = nothing to do, 1 = words staged in LDS, 2 = words in global memory.
struct UnitPlan {
    uint64_t first_word;    // kind 2: first word needed, as an index into the worker's words[]
    uint32_t nwords;        // kind 2: words needed
    uint32_t stage_off;     // kind 1: first word in the staging buffer
    uint32_t bit_lo, bit_hi;// records to parse, relative to the first word needed
    uint32_t idx_hi;
    int forced;
    float norm;
    uint32_t kind;
};

// The same for a unit whose words are staged (or that has nothing to do), as it is handed from the preparing
// wave to the parsing wave, in three words (every byte of LDS counts here: an eighth workgroup fits a CU only
// below 20480 bytes each).  Bit positions fit sixteen bits: the staging area holds 2^14 bits; the parser works
// out idx_hi itself.
struct PackedPlan {
    uint32_t bits;          // bit_lo | bit_hi << 16
    uint32_t where;         // stage_off | kind << 12 | (forced + 1) << 16
    float norm;
};

__device__ __forceinline__ PackedPlan pack_plan(const UnitPlan &U)
{
    PackedPlan Q;
    Q.bits = U.bit_lo | (U.bit_hi << 16);
    Q.where = U.stage_off | (U.kind << 12) | ((uint32_t)(U.forced + 1) << 16);
    Q.norm = U.norm;
    return Q;
}

template <bool kTable, int UPDATE, uint32_t TC>
__global__ __launch_bounds__(kDecodeWG, 4) void k_decode_accumulate(DecodeParams P)
{
    __shared__ __align__(16) double tile[TC];
    // words at [1, kStageWords]; the parser may read one word before and three after a stream's region
    __shared__ uint32_t stage[kStageWords + 5];
    __shared__ PackedPlan plans[kPlanned];
    __shared__ TileGeom next_geom;                // of the tile being prepared, for the wave that did not compute it
    __shared__ uint16_t lut[128];
    __shared__ uint8_t lut_level[128];
    float *lev = nullptr;                         // level values (level-table variant only)
    if constexpr (kTable) {
        __shared__ float lev_s[16];
        lev = lev_s;
    }

    // words per stream in the staging area (big tiles have few, long streams and always use the full stride)
    const uint32_t stream_stride = TC == kTileCoordsBig ? P.stream_cap : P.stream_stride;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & (kWave - 1u);
    const bool parser = tid < kWave;                  // first wave parses, second wave prepares
    const bool partial = !P.buckets_per_tile;        // tiles are parts of one bucket
    const bool walk = partial && !P.nsync;           // no index: every tile walks its bucket from the start
    const uint64_t last_bucket = P.nb - 1u;
    const double wscale = kTable ? 1.0 : ldexp(1.0, -1 - (int)P.s);

    // Unit u of a tile is (bucket in tile bi, segment g, worker k), k fastest.
    auto unit_coords = [&](const TileGeom &G, uint32_t u, uint32_t &k, uint32_t &bi, uint32_t &g) {
        const uint32_t segs = max(G.g1 - G.g0, 1u);
        k = u % P.K;
        const uint32_t r = u / P.K;
        g = G.g0 + r % segs;
        bi = r / segs;
    };
    // Loads of a unit's metadata.  Nothing is predicated per lane: a lane without a unit, or a unit without a
    // neighbouring sync entry, loads from a clamped index and ignores the value.
    auto load_unit = [&](const TileGeom &G, uint32_t bi, uint32_t g, const uint64_t *bit_off, const float *norms,
                         const uint32_t *sync) {
        UnitRaw r{};
        const uint64_t b = min(G.b0 + bi, last_bucket);
        r.bo0 = bit_off[b];
        r.bo1 = bit_off[b + 1];
        r.norm = norms[b];
        if (P.nsync) {
            const uint32_t *sy = sync + b * P.nsync;
            const uint32_t last = P.nsync - 1u;
            r.e_lo = sy[min(g, last)];
            r.e_hi = sy[min(g + 1u, last)];       // (not looked at for the bucket's last piece)
            if (partial) {
                r.e0 = sy[min(G.g0, last)];
                r.e1 = sy[min(G.g1, last)];       // (not looked at for the bucket's last tile)
            }
        }
        return r;
    };
    // Turn a unit's loaded metadata into what the parser needs.
    auto plan_unit = [&](const TileGeom &G, bool valid, uint32_t k, uint32_t bi, uint32_t g, const UnitRaw &m,
                         bool &bad) {
        UnitPlan U{};
        U.forced = -1;
        if (!valid)
            return U;
        const uint64_t b = G.b0 + bi;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        const StreamPart S = stream_part(P, G, m.bo0, m.bo1, m.e0, m.e1, P.words_bits[k], bad);
        uint32_t bit_lo = 0, bit_hi = S.len;
        U.idx_hi = nbk;
        if (P.nsync) {
            // piece g of the bucket: from its entry's record (whose index the entry gives) to the next entry's
            const uint32_t blk = g >> P.pieces_shift;
            U.idx_hi = min(nbk, (blk + 1u) << kSyncBlockShift);
            bit_lo = m.e_lo & kSyncOffMask;
            if (g + 1u < P.nseg)
                bit_hi = m.e_hi & kSyncOffMask;
            if (bit_lo > bit_hi || bit_hi > S.len) {
                bad = true;
                return U;
            }
            if (bit_hi == bit_lo)             // an empty piece (its entry's index field means nothing)
                return U;
            U.forced = (int)((blk << kSyncBlockShift) + (m.e_lo >> 21));
            if ((uint32_t)U.forced >= U.idx_hi) {
                bad = true;
                return U;
            }
        }
        if (bit_hi <= bit_lo)
            return U;
        if (bit_lo < S.bit0 || bit_hi > S.bit0 + (S.nwords << 5)) {   // a sync index that is not monotone
            bad = true;
            return U;
        }
        U.bit_lo = bit_lo - S.bit0;
        U.bit_hi = bit_hi - S.bit0;
        U.norm = m.norm;
        const uint32_t sidx = bi * P.K + k;
        if (S.nwords <= stream_stride && sidx < kMaxStreams) {
            U.kind = 1;
            U.stage_off = sidx * stream_stride;
        } else {                                  // did not fit in LDS: read the words from global memory
            U.kind = 2;
            U.first_word = S.first_word;
            U.nwords = S.nwords;
        }
        return U;
    };
    // address of in-bucket index 0 of bucket bi of the tile (never dereferenced outside the tile)
    auto tile_origin = [&](const TileGeom &G, uint32_t bi) {
        return partial ? tile - (int)G.in_lo : tile + bi * P.bucket;
    };
    const uint32_t last_len = (uint32_t)(P.d - last_bucket * P.bucket);     // coordinates of the last bucket
    auto parse_planned = [&](const TileGeom &G, uint32_t bi, uint32_t g, const uint32_t *buf, const PackedPlan &Q,
                             bool &bad) {
        const uint32_t nbk = G.b0 + bi == last_bucket ? last_len : P.bucket;
        const uint32_t idx_hi = P.nsync ? min(nbk, ((g >> P.pieces_shift) + 1u) << kSyncBlockShift) : nbk;
        decode_unit_fast<kTable>(StagedWords{buf + (Q.where & 0xFFFu)}, lut, lut_level, lev, Q.bits & 0xFFFFu, Q.bits >> 16,
                         (int)(Q.where >> 16) - 1, idx_hi, (double)Q.norm * wscale, TileSink{tile_origin(G, bi)}, bad);
    };
    // Any unit, from scratch: units beyond the planned ones and units whose words were not staged.
    auto slow_unit = [&](const TileGeom &G, const uint32_t *buf, uint32_t k, uint32_t bi, uint32_t g, bool report,
                         bool &bad) {
        const UnitRaw m = load_unit(G, bi, g, P.bit_off[k], P.norms[k], P.sync[k]);
        bool plan_bad = false;
        const UnitPlan X = plan_unit(G, true, k, bi, g, m, plan_bad);
        if (report)                               // otherwise whoever planned this unit first has reported
            bad |= plan_bad;
        if (X.kind == 1)
            parse_planned(G, bi, g, buf, pack_plan(X), bad);
        else if (X.kind == 2)
            decode_unit_fast<kTable>(GlobalWords{P.words[k] + X.first_word, X.nwords - 1u}, lut, lut_level, lev, X.bit_lo, X.bit_hi,
                             X.forced,
                             X.idx_hi, (double)X.norm * wscale, TileSink{tile_origin(G, bi)}, bad);
    };
    // Tiles of a large bucket without a sync index: every tile parses the bucket from its first record in
    // global memory and keeps what lands inside.
    auto walk_unit = [&](const TileGeom &G, uint32_t k, bool &bad) {
        const uint64_t b = G.b0;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        if (G.in_lo >= nbk)
            return;
        const uint64_t bo0 = P.bit_off[k][b];
        const uint64_t start = (bo0 + 31ull) & ~31ull;
        const uint64_t end = P.bit_off[k][b + 1];
        if (end < bo0 || end > P.words_bits[k] || (end > start && end - start > (uint64_t)kSyncOffMask)) {
            bad = true;                         // offsets that run backwards, leave the words or span too much
            return;
        }
        const uint32_t len = end > start ? (uint32_t)(end - start) : 0u;
        const double wnorm = (double)P.norms[k][b] * wscale;
        WalkWords gw{P.words[k] + (start >> 5)};
        const uint32_t hi_idx = min(nbk, G.in_lo + P.tile_coords);
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
            if ((uint32_t)idx >= G.in_lo) {
                double val;
                if constexpr (kTable)
                    val = wnorm * (double)lev[j];
                else
                    val = ldexp(wnorm, (int)j);
                atomicAdd(&tile[(uint32_t)idx - G.in_lo], neg ? -val : val);
            }
            br.skip(rl);
            pos += rl;
            prev = idx;
        }
    };

    // ---- the preparing wave's constants: its stream and its two units (lane and lane + 64).  The pointers to
    // their workers' arrays are fetched from the kernel arguments every round rather than kept: this wave has
    // time to spare, registers are what is short.
    const uint32_t my_stream = lane >> P.lanes_shift;
    const uint32_t my_sub = lane & ((1u << P.lanes_shift) - 1u);
    const uint32_t sk = my_stream % P.K, sbi = my_stream / P.K;
    uint32_t uk[2], ubi[2], ugr[2];
#pragma unroll
    for (uint32_t h = 0; h < 2u; ++h) {
        const uint32_t u = lane + h * kWave;
        uk[h] = u % P.K;
        const uint32_t r = u / P.K;
        ubi[h] = partial ? 0u : r / P.nseg;       // multi-bucket tiles hold every segment of a bucket
        ugr[h] = partial ? r : r % P.nseg;        // segment, counted from the tile's first
    }
    auto load_stream = [&](const TileGeom &G) {
        StreamRaw r{};
        if (walk)
            return r;
        const uint64_t b = min(G.b0 + sbi, last_bucket);
        const uint64_t *s_bit_off = P.bit_off[sk];
        r.bo0 = s_bit_off[b];
        r.bo1 = s_bit_off[b + 1];
        if (partial && P.nsync) {
            const uint32_t *sy = P.sync[sk] + b * P.nsync;
            r.e0 = sy[min(G.g0, P.nsync - 1u)];
            r.e1 = sy[min(G.g1, P.nsync - 1u)];
        }
        return r;
    };
    // Prepare a tile whose metadata has arrived: plans to LDS, this lane's share of its words into registers.
    auto prepare = [&](const TileGeom &G, const StreamRaw &sr, const UnitRaw &um, uint32_t (&w)[kWordsPerLane],
                       bool &bad) {
        // words: global -> registers
        uint32_t cnt = 0;
        const uint32_t *const s_words = P.words[sk];
        const uint32_t *src = s_words;
        if (my_stream < G.nstreams && !walk) {
            const StreamPart S = stream_part(P, G, sr.bo0, sr.bo1, sr.e0, sr.e1, P.words_bits[sk], bad);
            cnt = min(S.nwords, stream_stride);
            src = s_words + S.first_word;
        }
#pragma unroll
        for (uint32_t i = 0; i < kWordsPerLane; ++i) {
            const uint32_t wi = my_sub + (i << P.lanes_shift);
            const uint32_t *a = wi < cnt ? src + wi : P.flags;     // beyond the stream's part: any readable word
            w[i] = *a;
        }
        // plans, while the words are in flight.  The metadata of a lane's first unit was requested a round ago; a
        // tile with more units than lanes fetches the second one's here and waits (this wave has time to spare).
        plans[lane] = pack_plan(plan_unit(G, lane < G.units, uk[0], ubi[0], G.g0 + ugr[0], um, bad));
        if (G.units > kWave) {
            const UnitRaw m2 = load_unit(G, ubi[1], G.g0 + ugr[1], P.bit_off[uk[1]], P.norms[uk[1]], P.sync[uk[1]]);
            plans[lane + kWave] =
                pack_plan(plan_unit(G, lane + kWave < G.units, uk[1], ubi[1], G.g0 + ugr[1], m2, bad));
        }
    };
    // ... and from the registers to the staging area, once the parse that read it is over
    auto store_words = [&](const uint32_t (&w)[kWordsPerLane]) {
        const uint32_t base = 1u + my_stream * stream_stride + my_sub;    // + word index < kStageWords for every lane
#pragma unroll
        for (uint32_t i = 0; i + 1u < kWordsPerLane; ++i)
            stage[base + (i << P.lanes_shift)] = w[i];
        // only the very last carried word of a stream can be the one an odd stride has no place for
        constexpr uint32_t kLast = kWordsPerLane - 1u;
        if (TC == kTileCoordsBig || my_sub + (kLast << P.lanes_shift) < stream_stride)
            stage[base + (kLast << P.lanes_shift)] = w[kLast];
    };

    // ---- prologue
    bool bad = false;
    const uint32_t stride = gridDim.x;
    uint32_t t = blockIdx.x;                    // < ntiles by the launch
    TileGeom G = tile_geom(P, xcd_tile(P, t));
    StreamRaw sr{};                             // preparing wave: metadata of the tile after the next, in flight
    UnitRaw um{};
    uint32_t wnext[kWordsPerLane] = {};         // preparing wave: its share of the next tile's words
    if (parser) {
        for (uint32_t i = lane; i < TC / 2u; i += kWave)
            reinterpret_cast<double2 *>(tile)[i] = double2{0.0, 0.0};
        lut[lane] = (uint16_t)gap_table_entry(lane);
        lut[lane + kWave] = (uint16_t)gap_table_entry(lane + kWave);
        if constexpr (kTable) {
            if (lane < 16u)
                lev[lane] = P.lev[lane];
        }
        lut_level[lane] = (uint8_t)level_table_entry(lane, P.s + 1u);
        lut_level[lane + kWave] = (uint8_t)level_table_entry(lane + kWave, P.s + 1u);
        if (lane < 5u)
            stage[lane ? kStageWords + lane : 0u] = 0u;    // the pads
    } else {
        sr = load_stream(G);
        um = load_unit(G, ubi[0], G.g0 + ugr[0], P.bit_off[uk[0]], P.norms[uk[0]], P.sync[uk[0]]);
        prepare(G, sr, um, wnext, bad);
        store_words(wnext);
        if (t + stride < P.ntiles) {
            const TileGeom G1 = tile_geom(P, xcd_tile(P, t + stride));
            sr = load_stream(G1);
            um = load_unit(G1, ubi[0], G1.g0 + ugr[0], P.bit_off[uk[0]], P.norms[uk[0]], P.sync[uk[0]]);
        }
    }
    __syncthreads();
    PackedPlan Q[2] = {};
    if (parser) {
        Q[0] = plans[lane];
        if (G.units > kWave)
            Q[1] = plans[lane + kWave];
    }
    __syncthreads();

    for (;;) {
        const bool has1 = t + stride < P.ntiles;                        // uniform
        const bool has2 = has1 && t + stride < P.ntiles - stride;
        if (parser) {
            // ---- parse this tile's units
            const uint32_t *buf = stage;
            if (walk) {
                for (uint32_t u = lane; u < G.units; u += kWave)
                    walk_unit(G, u, bad);
            } else {
#pragma unroll
                for (uint32_t h = 0; h < 2u; ++h) {
                    if (h == 1u && G.units <= kWave)
                        break;
                    const uint32_t kind = (Q[h].where >> 12) & 3u;
                    if (kind == 1u)
                        parse_planned(G, ubi[h], G.g0 + ugr[h], buf, Q[h], bad);
                    else if (kind == 2u)
                        slow_unit(G, buf, uk[h], ubi[h], G.g0 + ugr[h], false, bad);
                }
                for (uint32_t u = lane + kPlanned; u < G.units; u += kWave) {
                    uint32_t k, bi, g;
                    unit_coords(G, u, k, bi, g);
                    slow_unit(G, buf, k, bi, g, true, bad);
                }
            }
        } else if (has1) {
            // ---- prepare the next tile (its metadata was requested a round ago), request the metadata of the
            // one after it
            const TileGeom GA = tile_geom(P, xcd_tile(P, t + stride));
            prepare(GA, sr, um, wnext, bad);
            if (lane == 0)
                next_geom = GA;
            if (has2) {
                const TileGeom G2 = tile_geom(P, xcd_tile(P, t + 2u * stride));
                sr = load_stream(G2);
                um = load_unit(G2, ubi[0], G2.g0 + ugr[0], P.bit_off[uk[0]], P.norms[uk[0]], P.sync[uk[0]]);
            }
        }
        __syncthreads();
        TileGeom G1{};
        if (has1) {
            G1.b0 = uniform_u64(next_geom.b0);
            G1.c_lo = uniform_u64(next_geom.c_lo);
            G1.nbuck = uniform_u32(next_geom.nbuck);
            G1.in_lo = uniform_u32(next_geom.in_lo);
            G1.span = uniform_u32(next_geom.span);
            G1.g0 = uniform_u32(next_geom.g0);
            G1.g1 = uniform_u32(next_geom.g1);
            G1.nstreams = uniform_u32(next_geom.nstreams);
            G1.units = uniform_u32(next_geom.units);
            if (parser) {
                Q[0] = plans[lane];
                if (G1.units > kWave)
                    Q[1] = plans[lane + kWave];
            } else {
                store_words(wnext);          // the staging area is free: this tile's parse is over
            }
        }

        // ---- scale, round to fp32, apply to the output (write, add, or momentum rule); leave the tile zeroed
        tile_output<UPDATE, TC, kDecodeWG>(P, tile, G.c_lo, G.span, tid);
        if (!has1)
            break;
        __syncthreads();
        t += stride;
        G = G1;
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
}

// ---- the tile decoder as one wave per workgroup --------------------------------------------------------------
// For messages with a decoder index whose tiles hold at most 64 pieces, each stream's pieces within the lanes that copy
// that stream (the usual geometries).  What bounds the two-wave kernel above on such tiles is neither the parse nor
// memory but its own bookkeeping: the preparing wave works through several hundred mostly dependent instructions per
// tile at a lone wave's pace (an instruction every nine cycles), sharing its SIMD's issue slots with the parsing waves,
// and two barriers per tile keep the eight workgroups of a CU in step, so that all of them parse, and then all of them
// write, at the same time.  Here one wave does everything for its tiles, in order and without barriers: the lanes
// that copy a stream's words are the lanes that parse its pieces (so one set of offsets and index entries serves
// both), the words of the next tile and the offsets of the tile after it are in flight in registers while this
// tile is parsed and written (a wave per SIMD pair leaves 256 registers per lane), and the workgroups of a CU drift
// apart, which spreads parse, LDS and store traffic over time.
constexpr uint32_t kWaveWG = 64;

struct WaveMeta {           // what a lane loads for its stream (bucket, worker) and its piece of one tile
    uint64_t bo0, bo1;      // bit_off[b], bit_off[b + 1]
    uint32_t e_lo, e_hi;    // index entries of the piece and of the one after it
    float norm;
};

// The paper's ENCODE (App. A): records ERC(gap) | sign | ERC(level index), pieces of equal record count.
template <bool kTable>
struct ErcCodec {
    static constexpr uint32_t kWordsPerLane = nuq::kWordsPerLane;
    uint16_t *lut;          // LDS: 128 entries (gap_table_entry)
    uint8_t *lut_level;     // LDS: 128 entries (level_table_entry)
    float *lev;             // LDS: 16 level values (level-table variant), else nullptr
    struct Range {
        uint32_t bit_lo, bit_hi;    // from the bucket's first bit
        uint32_t forced, idx_hi;    // index of the piece's first record; records stay below idx_hi
    };
    __device__ __forceinline__ void init(const DecodeParams &P, uint32_t lane) const
    {
        lut[lane] = (uint16_t)gap_table_entry(lane);
        lut[lane + kWave] = (uint16_t)gap_table_entry(lane + kWave);
        lut_level[lane] = (uint8_t)level_table_entry(lane, P.s + 1u);
        lut_level[lane + kWave] = (uint8_t)level_table_entry(lane + kWave, P.s + 1u);
        if constexpr (kTable) {
            if (lane < 16u)
                lev[lane] = P.lev[lane];
        }
    }
    __device__ __forceinline__ void entries(const uint32_t *sy, uint32_t g, const DecodeParams &P, uint32_t &e_lo,
                                            uint32_t &e_hi) const
    {
        const uint32_t last = P.nsync - 1u;
        e_lo = sy[min(g, last)];
        e_hi = sy[min(g + 1u, last)];                                 // (not looked at for the bucket's last piece)
    }
    __device__ __forceinline__ bool range(const DecodeParams &P, uint32_t g, uint32_t nbk, uint32_t e_lo, uint32_t e_hi,
                                          uint32_t len, Range &R, bool &bad) const
    {
        const uint32_t blk = g >> P.pieces_shift;
        R.idx_hi = min(nbk, (blk + 1u) << kSyncBlockShift);
        R.bit_lo = e_lo & kSyncOffMask;
        R.bit_hi = g + 1u < P.nseg ? e_hi & kSyncOffMask : len;
        R.forced = (blk << kSyncBlockShift) + (e_lo >> 21);
        if (R.bit_lo > R.bit_hi || R.bit_hi > len) {
            bad = true;
            return false;
        }
        if (R.bit_hi == R.bit_lo)             // an empty piece (its entry's index field means nothing)
            return false;
        if (R.forced >= R.idx_hi) {
            bad = true;
            return false;
        }
        return true;
    }
    template <class Words>
    __device__ __forceinline__ void parse(const Words &words, const Range &R, uint32_t bit0, float norm,
                                          const TileSink &sink, bool &bad) const
    {
        const double wnorm = (double)norm * (kTable ? 1.0 : ldexp(1.0, -1 - (int)s));
        decode_unit_fast<kTable>(words, lut, lut_level, lev, R.bit_lo - bit0, R.bit_hi - bit0, (int)R.forced, R.idx_hi,
                                 wnorm, sink, bad);
    }
    uint32_t s;
};

// The kernel's body is written once for every code of the level indices.  A Codec supplies
//   kWordsPerLane                    staged words each lane carries (64 x that many per tile)
//   init(P, lane)                    its tables, into LDS that the kernel handed it
//   entries(sy, g, P, e_lo, e_hi)    the index entries that bound piece g of a bucket (sy = the bucket's entries)
//   range(P, g, nbk, e_lo, e_hi, len, R, bad)   piece g's bit range and what else its parse needs; false = nothing to do
//   parse(words, R, bit0, norm, sink, bad)      the parse proper, adding values into the tile
template <class Codec, int UPDATE, uint32_t TC>
__device__ __forceinline__ void decode_wave(const DecodeParams &P, const Codec &codec)
{
    constexpr uint32_t kWordsPerLane = Codec::kWordsPerLane;
    constexpr uint32_t kStageWords = kWave * kWordsPerLane;
    __shared__ __align__(16) double tile[TC];
    __shared__ uint32_t stage[kStageWords + 5];       // words at [1, kStageWords]; pads as in k_decode_accumulate
    const uint32_t lane = threadIdx.x;
    const bool partial = !P.buckets_per_tile;         // tiles are parts of one bucket
    const uint32_t stream_stride = TC == kTileCoordsBig ? P.stream_cap : P.stream_stride;
    const uint64_t last_bucket = P.nb - 1u;
    const uint32_t last_len = (uint32_t)(P.d - last_bucket * P.bucket);

    // this lane's stream (bucket in tile, worker) and piece of it; its pointers into that worker's arrays
    const uint32_t lanes = 1u << P.lanes_shift;
    const uint32_t my_stream = lane >> P.lanes_shift, my_sub = lane & (lanes - 1u);
    const uint32_t sk = my_stream % P.K, sbi = my_stream / P.K;
    const uint64_t *const pb = P.bit_off[sk];
    const float *const pn = P.norms[sk];
    const uint32_t *const ps = P.sync[sk];
    const uint32_t *const pw = P.words[sk];
    const uint64_t words_bits = P.words_bits[sk];
    const uint32_t first_lane = lane & ~(lanes - 1u);

    auto load_meta = [&](const TileGeom &G) {
        WaveMeta m;
        const uint64_t b = min(G.b0 + sbi, last_bucket);              // (a lane without a stream loads and ignores)
        m.bo0 = pb[b];
        m.bo1 = pb[b + 1];
        m.norm = pn[b];
        codec.entries(ps + b * P.nsync, G.g0 + my_sub, P, m.e_lo, m.e_hi);
        return m;
    };
    // the part of the lane's stream that the tile needs: from the entry of the tile's first piece to that of the
    // piece after its last one (held by the stream's first and last lanes)
    auto part_of = [&](const TileGeom &G, const WaveMeta &m, bool &bad) {
        uint32_t e0 = 0, e1 = 0;
        if (partial) {
            const uint32_t pieces = G.g1 - G.g0;                      // >= 1 for a tile with coordinates
            e0 = (uint32_t)__shfl((int)m.e_lo, (int)first_lane, kWave);
            e1 = (uint32_t)__shfl((int)m.e_hi, (int)(first_lane + max(pieces, 1u) - 1u), kWave);
        }
        bool wrong = false;
        const StreamPart S = stream_part(P, G, m.bo0, m.bo1, e0, e1, words_bits, wrong);
        bad |= wrong && my_stream < G.nstreams;                       // (a lane without a stream loaded any bucket's)
        return S;
    };
    auto load_words = [&](const TileGeom &G, const StreamPart &S, uint32_t (&w)[kWordsPerLane]) {
        // lanes beyond the part's end load its last word again (nothing reads what they store); a lane without a
        // stream, or a part without words, loads any readable word
        const uint32_t cnt = my_stream < G.nstreams ? min(S.nwords, stream_stride) : 0u;
        const uint32_t *src = cnt ? pw + S.first_word : P.flags;
        const uint32_t last = max(cnt, 1u) - 1u;
#pragma unroll
        for (uint32_t i = 0; i < kWordsPerLane; ++i)
            w[i] = src[min(my_sub + (i << P.lanes_shift), last)];
    };
    auto store_words = [&](const uint32_t (&w)[kWordsPerLane]) {
        const uint32_t base = 1u + my_stream * stream_stride + my_sub;
#pragma unroll
        for (uint32_t i = 0; i + 1u < kWordsPerLane; ++i)
            stage[base + (i << P.lanes_shift)] = w[i];
        constexpr uint32_t kLast = kWordsPerLane - 1u;                // an odd stride has no place for the very last word
        if (TC == kTileCoordsBig || my_sub + (kLast << P.lanes_shift) < stream_stride)
            stage[base + (kLast << P.lanes_shift)] = w[kLast];
    };
    // LDS traffic of one wave needs no hardware barrier: its operations complete in order.  (No memory fence here: a
    // fence also waits for every global load and store in flight, which is exactly what this kernel keeps in flight.)
    auto lds_fence = [] {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        asm volatile("" ::: "memory");
    };

    // ---- tables, cleared tile
    for (uint32_t i = lane; i < TC / 2u; i += kWaveWG)
        reinterpret_cast<double2 *>(tile)[i] = double2{0.0, 0.0};
    codec.init(P, lane);
    if (lane < 5u)
        stage[lane ? kStageWords + lane : 0u] = 0u;                  // the pads

    // ---- prologue: offsets of the first two tiles, words of the first
    bool bad = false;
    const uint32_t stride = gridDim.x;
    uint32_t t = blockIdx.x;                                          // < ntiles by the launch
    TileGeom G0 = tile_geom(P, xcd_tile(P, t)), G1 = G0;
    WaveMeta M0 = load_meta(G0), M1 = M0;
    if (t + stride < P.ntiles) {
        G1 = tile_geom(P, xcd_tile(P, t + stride));
        M1 = load_meta(G1);
    }
    StreamPart S0 = part_of(G0, M0, bad);
    uint32_t W0[kWordsPerLane];
    load_words(G0, S0, W0);
    store_words(W0);

    // Order of a round, chosen for the one counter that tracks loads and stores alike and in issue order: the next
    // tile's words and the offsets of the tile after it are requested first, this tile is parsed (which takes longer
    // than any of those loads, or the previous tile's stores, need), then the words are moved to the staging area,
    // which the parse no longer reads, and only then is this tile written out: no wait ever stands behind a store
    // that has just been issued.
    for (;;) {
        const bool has1 = t + stride < P.ntiles;                      // uniform
        const bool has2 = has1 && t + stride < P.ntiles - stride;
        StreamPart S1 = S0;
        TileGeom G2 = G1;
        WaveMeta M2 = M1;
        if (has1) {
            S1 = part_of(G1, M1, bad);
            load_words(G1, S1, W0);
        }
        if (has2) {
            G2 = tile_geom(P, xcd_tile(P, t + 2u * stride));
            M2 = load_meta(G2);
        }
        lds_fence();

        // ---- this lane's piece of tile t
        const uint32_t pieces = G0.g1 - G0.g0;
        if (my_stream < G0.nstreams && my_sub < pieces) {
            const uint32_t nbk = G0.b0 + sbi == last_bucket ? last_len : P.bucket;
            typename Codec::Range R;
            if (codec.range(P, G0.g0 + my_sub, nbk, M0.e_lo, M0.e_hi, S0.len, R, bad)) {
                // (an index that is not monotone would leave the part of the stream that was copied)
                if (R.bit_lo < S0.bit0 || R.bit_hi > S0.bit0 + (S0.nwords << 5)) {
                    bad = true;
                } else {
                    const TileSink sink{partial ? tile - (int)G0.in_lo : tile + sbi * P.bucket};
                    if (S0.nwords <= stream_stride)
                        codec.parse(StagedWords{stage + my_stream * stream_stride}, R, S0.bit0, M0.norm, sink, bad);
                    else {                            // the part did not fit the staging area: words from global memory
                        codec.parse(GlobalWords{pw + S0.first_word, S0.nwords - 1u}, R, S0.bit0, M0.norm, sink, bad);
                        // every load of this rare path has landed before the paths join again: otherwise the compiler,
                        // which must assume the worst of the joined paths, waits for all memory traffic wherever the
                        // usual path later touches a register that this one loaded into
                        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
                    }
                }
            }
        }
        lds_fence();
        if (has1)
            store_words(W0);                              // (the parse of this tile is over: the staging area is free)
        tile_output<UPDATE, TC, kWaveWG>(P, tile, G0.c_lo, G0.span, lane);
        if (!has1)
            break;
        lds_fence();
        t += stride;
        G0 = G1;
        G1 = G2;
        M0 = M1;
        M1 = M2;
        S0 = S1;
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
}


template <bool kTable, int UPDATE, uint32_t TC>
__global__ __launch_bounds__(kWaveWG, 2) void k_decode_wave(DecodeParams P)
{
    __shared__ uint16_t lut[128];
    __shared__ uint8_t lut_level[128];
    float *lev = nullptr;
    if constexpr (kTable) {
        __shared__ float lev_s[16];
        lev = lev_s;
    }
    decode_wave<ErcCodec<kTable>, UPDATE, TC>(P, ErcCodec<kTable>{lut, lut_level, lev, P.s});
}

// ---- one message (K = 1), main scheme's levels, output written or added to -------------------------------------
// With a single worker there is nothing to sum, and a 2048-coordinate tile would hold only 2048 / stride units for
// 64 parsing lanes.  Here every lane owns one unit (bucket, sync segment), stages its words in an LDS row of its
// own and stores each value where it belongs; for the write mode the workgroup first clears the contiguous range of
// coordinates its units cover (coalesced), and a coordinate belongs to exactly one unit, so nothing races.
constexpr uint32_t kSingleWG = 128;
constexpr uint32_t kSingleCap = 24;                     // words of a unit that are staged (longer units read global memory)
constexpr uint32_t kSingleRow = kSingleCap + 5;         // pad word before, three after; odd: rows start in different banks

template <int UPDATE>
__global__ __launch_bounds__(kSingleWG) void k_decode_single(DecodeParams P)
{
    static_assert(UPDATE == kUpdateWrite || UPDATE == kUpdateAdd, "the momentum rule touches every coordinate");
    __shared__ uint32_t rows[kSingleWG * kSingleRow];
    __shared__ uint16_t lut[128];
    __shared__ uint8_t lut_level[128];
    const uint32_t tid = threadIdx.x;
    lut[tid] = (uint16_t)gap_table_entry(tid);
    lut_level[tid] = (uint8_t)level_table_entry(tid, P.s + 1u);
    const uint64_t units = P.nb * P.nseg;
    const uint64_t u0 = (uint64_t)blockIdx.x * kSingleWG;

    // ---- this lane's unit: metadata, then its words into the lane's LDS row (before the clearing below, so that
    // the two chains of dependent loads run under it)
    const uint64_t u = u0 + tid;
    const uint64_t b = min(u / P.nseg, P.nb - 1u);                  // (clamped: a lane without a unit loads and ignores)
    const uint32_t g = (uint32_t)(u - (u / P.nseg) * P.nseg);
    const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
    const uint32_t blk = g >> P.pieces_shift;                       // the piece's block of 2048 coordinates (0 without index)
    const uint32_t idx_hi = P.nsync ? min(nbk, (blk + 1u) << kSyncBlockShift) : nbk;
    bool work = u < units;
    const uint64_t bo0 = P.bit_off[0][b], bo1 = P.bit_off[0][b + 1];
    const uint64_t start = (bo0 + 31ull) & ~31ull;
    // offsets run forwards, stay inside the words received, and a bucket's bit string is below 2^21 bits
    bool bad = work && (bo1 < bo0 || bo1 > P.words_bits[0] || (bo1 > start && bo1 - start > 0x1FFFFFull));
    const uint32_t len = bo1 > start && !bad ? (uint32_t)(bo1 - start) : 0u;
    uint32_t bit_lo = 0, bit_hi = len;
    int forced = -1;
    if (P.nsync) {
        const uint32_t *sy = P.sync[0] + b * P.nsync;
        const uint32_t e = sy[g];
        bit_lo = e & kSyncOffMask;
        forced = (int)((blk << kSyncBlockShift) + (e >> 21));
        if (g + 1u < P.nseg)
            bit_hi = sy[g + 1u] & kSyncOffMask;
        if (work && (bit_lo > bit_hi || bit_hi > len || (bit_hi > bit_lo && (uint32_t)forced >= idx_hi))) {
            bad = true;
            work = false;
        }
    }
    work = work && bit_hi > bit_lo;
    const uint32_t w0 = bit_lo >> 5, nw = work ? ((bit_hi + 31u) >> 5) - w0 : 0u;
    const uint32_t *src = P.words[0] + (start >> 5) + w0;
    uint32_t *row = rows + tid * kSingleRow;
    const bool staged = nw <= kSingleCap;
    if (work && staged) {
        row[0] = 0u;
        for (uint32_t j0 = 0; j0 < nw; j0 += 8u) {                   // loads of a group in flight together
            uint32_t x[8];
#pragma unroll
            for (uint32_t j = 0; j < 8u; ++j)
                x[j] = src[min(j0 + j, nw - 1u)];
#pragma unroll
            for (uint32_t j = 0; j < 8u; ++j)
                if (j0 + j < nw)
                    row[1u + j0 + j] = x[j];
        }
        row[nw + 1u] = 0u;
        row[nw + 2u] = 0u;
        row[nw + 3u] = 0u;
    }
    const float nrm = P.norms[0][b];

    // ---- write mode: clear the contiguous range of coordinates that the workgroup's units cover
    if constexpr (UPDATE == kUpdateWrite) {
        // The workgroup's units are whole blocks (the pieces per block divide its size): the coordinates before the
        // first block of the next workgroup are its own.
        auto first_coord = [&](uint64_t v) -> uint64_t {    // first coordinate of the block of unit v; d for v = units
            if (v >= units)
                return P.d;
            const uint64_t vb = v / P.nseg;
            const uint64_t c = vb * P.bucket + (((v - vb * P.nseg) >> P.pieces_shift) << kSyncBlockShift);
            return c < P.d ? c : P.d;
        };
        const uint64_t c0 = first_coord(u0), c1 = first_coord(u0 + kSingleWG);
        float *o = P.out;
        const uint64_t up = (c0 + 3u) & ~3ull, dn = c1 & ~3ull;
        const uint64_t a0 = up < c1 ? up : c1, a1 = dn > a0 ? dn : a0;                  // whole float4 groups in [a0, a1)
        const bool vec = (reinterpret_cast<uintptr_t>(o) & 15u) == 0;
        if (vec) {
            for (uint64_t c = c0 + tid; c < a0; c += kSingleWG)
                o[c] = 0.0f;
            for (uint64_t c = a0 + 4ull * tid; c < a1; c += 4ull * kSingleWG)
                *reinterpret_cast<float4 *>(o + c) = float4{0.0f, 0.0f, 0.0f, 0.0f};
            for (uint64_t c = a1 + tid; c < c1; c += kSingleWG)
                o[c] = 0.0f;
        } else {
            for (uint64_t c = c0 + tid; c < c1; c += kSingleWG)
                o[c] = 0.0f;
        }
    }
    __syncthreads();          // tables in place; the cleared range is ordered before the values stored below

    if (work) {
        const uint32_t rel_lo = bit_lo & 31u, rel_hi = bit_hi - (w0 << 5);
        const double wnorm = (double)nrm * ldexp(1.0, -1 - (int)P.s);
        const DirectSink<UPDATE> sink{P.out + b * P.bucket, (double)P.scale};
        if (staged)
            decode_unit_fast<false>(StagedWords{row}, lut, lut_level, nullptr, rel_lo, rel_hi, forced, idx_hi, wnorm, sink,
                                    bad);
        else
            decode_unit_fast<false>(GlobalWords{src, nw - 1u}, lut, lut_level, nullptr, rel_lo, rel_hi, forced, idx_hi,
                                    wnorm, sink, bad);
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
}

}  // namespace nuq
