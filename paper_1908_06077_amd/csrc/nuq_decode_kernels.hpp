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
// LDS capacity bounds the number of tiles in flight, and a tile's life would mostly be spent
// waiting on memory: offsets and sync entries first, then the words they point to.  So a
// workgroup is persistent and walks a strided sequence of tiles as a software pipeline held in
// registers: while tile t is parsed, the words of tile t+1 are in flight to registers (they go
// to LDS once tile t's parse is over) and the metadata of tile t+2 is in flight too.
//
// The parse loop is bound by instruction issue and by the latency of its dependent LDS reads,
// so it is kept short: the window at the current bit position comes from one two-word LDS
// read, a 128-entry table indexed by the next seven stream bits resolves every gap code of up
// to seven bits (values 1..15) and gives position and width of the last group of longer ones,
// the level code is taken apart with byte permutes, and format checks are accumulated and
// tested once.
#pragma once
#include "nuq_device.hpp"
#include "nuq_encode_kernels.hpp"

namespace nuq {

constexpr uint32_t kMaxWorkers = 32;
constexpr uint32_t kDecodeWG = 128;        // threads per workgroup
constexpr uint32_t kTileCoords = 2048;     // coordinates per tile (16 KB of fp64)
constexpr uint32_t kWordsPerThread = 5;    // staged words each thread carries through the pipeline
constexpr uint32_t kStageWords = kDecodeWG * kWordsPerThread;   // LDS words for staged bit strings
constexpr uint32_t kMaxStreams = 64;       // (bucket, worker) bit strings per tile

struct DecodeParams {
    const float *norms[kMaxWorkers];
    const uint64_t *bit_off[kMaxWorkers];
    const uint32_t *words[kMaxWorkers];
    const uint32_t *sync[kMaxWorkers];
    float *out;
    uint32_t *flags;
    uint64_t d;
    uint64_t nb;
    uint32_t ntiles;
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
    uint32_t lanes_shift;       // log2 of the threads that copy one stream's words
    uint32_t stream_cap;        // LDS words reserved per stream = kWordsPerThread << lanes_shift
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
    G.g0 = P.sync_shift ? (G.in_lo >> P.sync_shift) : 0u;
    G.g1 = partial && P.sync_shift ? min(P.nseg, G.g0 + P.segs_per_tile) : P.nseg;
    G.nstreams = G.nbuck * P.K;
    G.units = G.nstreams * (G.g1 - G.g0);
    return G;
}

// What a thread loads for the stream whose words it helps to copy.
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

__device__ __forceinline__ StreamPart stream_part(const DecodeParams &P, const TileGeom &G, uint64_t bo0, uint64_t bo1,
                                                  uint32_t e0, uint32_t e1)
{
    StreamPart S;
    const uint64_t start = (bo0 + 31ull) & ~31ull;
    S.len = bo1 > start ? (uint32_t)(bo1 - start) : 0u;
    uint32_t lo = 0, hi = S.len;
    if (!P.buckets_per_tile && P.sync_shift) {
        if (G.g0 > 0u)
            lo = min(e0 & 0x1FFFFFu, S.len);
        if (G.g1 < P.nseg)
            hi = min(e1 & 0x1FFFFFu, S.len);
    }
    const uint32_t w0 = lo >> 5;
    S.bit0 = w0 << 5;
    S.nwords = hi > lo ? ((hi + 31u) >> 5) - w0 : 0u;
    S.first_word = (start >> 5) + w0;
    return S;
}

// What a thread loads for the unit it parses.
struct UnitRaw {
    uint64_t bo0, bo1;      // bit_off[b], bit_off[b + 1]
    uint32_t e_lo, e_hi;    // sync entries that bound the segment (0 when not applicable)
    uint32_t e0, e1;        // sync entries that bound the tile (as in StreamRaw)
    float norm;
};

// A unit ready to parse.  kind: 0 = nothing to do, 1 = words staged in LDS, 2 = words in global memory.
struct UnitPlan {
    const uint32_t *gwords; // kind 2: first word needed
    uint32_t glast;         // kind 2: highest readable word index
    uint32_t stage_off;     // kind 1: first word in the staging area
    uint32_t bit_lo, bit_hi;// records to parse, relative to the first word needed
    uint32_t idx_hi;
    int forced;
    int tile_lo;            // in-bucket index of the tile's first coordinate (negative for later buckets of a tile)
    float norm;
    uint32_t kind;
};

__global__ __launch_bounds__(kDecodeWG) void k_decode_accumulate(DecodeParams P)
{
    __shared__ __align__(16) double tile[kTileCoords];
    __shared__ uint32_t stage[kStageWords + 1];
    __shared__ uint32_t lut[128];

    const uint32_t tid = threadIdx.x;
    const bool partial = !P.buckets_per_tile;                                        // tiles are parts of one bucket
    const bool walk = partial && !P.sync_shift;                                      // no index: walk from the start
    const uint32_t my_stream = tid >> P.lanes_shift;                                 // the stream this thread copies
    const uint32_t my_lane = tid & ((1u << P.lanes_shift) - 1u);

    // Unit u of a tile is (bucket in tile bi, segment g, worker k), k fastest.
    auto unit_coords = [&](const TileGeom &G, uint32_t u, uint32_t &k, uint32_t &bi, uint32_t &g) {
        const uint32_t segs = G.g1 - G.g0;
        k = u % P.K;
        const uint32_t r = u / P.K;
        g = G.g0 + r % segs;
        bi = r / segs;
    };
    // The worker of this thread's stream and of its first unit never changes from tile to tile, so the
    // pointers to that worker's arrays are fetched once; a fetch per tile would put a dependent load (and a
    // wait for everything in flight) in front of every metadata load.
    const uint32_t sk = my_stream % P.K, sbi = my_stream / P.K;
    const uint64_t *const s_bit_off = P.bit_off[sk];
    const uint32_t *const s_words = P.words[sk];
    const uint32_t *const s_sync = P.sync[sk];
    const uint32_t uk = tid % P.K, ur = tid / P.K;
    const uint32_t ubi = partial ? 0u : ur / P.nseg;        // multi-bucket tiles hold every segment of a bucket
    const uint32_t ugr = partial ? ur : ur % P.nseg;        // segment, counted from the tile's first
    const uint64_t *const u_bit_off = P.bit_off[uk];
    const float *const u_norms = P.norms[uk];
    const uint32_t *const u_sync = P.sync[uk];
    // ---- loads (all independent of each other, nothing is waited for here)
    auto load_stream = [&](const TileGeom &G) {
        StreamRaw r{};
        if (my_stream < G.nstreams && !walk) {
            const uint64_t b = G.b0 + sbi;
            r.bo0 = s_bit_off[b];
            r.bo1 = s_bit_off[b + 1];
            if (partial && P.sync_shift) {
                const uint32_t *sy = s_sync + b * P.nsync;
                if (G.g0 > 0u)
                    r.e0 = sy[G.g0 - 1u];
                if (G.g1 < P.nseg)
                    r.e1 = sy[G.g1 - 1u];
            }
        }
        return r;
    };
    auto load_unit_at = [&](const TileGeom &G, bool valid, uint32_t bi, uint32_t g, const uint64_t *bit_off,
                            const float *norms, const uint32_t *sync) {
        UnitRaw r{};
        if (valid) {
            const uint64_t b = G.b0 + bi;
            r.bo0 = bit_off[b];
            r.bo1 = bit_off[b + 1];
            r.norm = norms[b];
            if (P.sync_shift) {
                const uint32_t *sy = sync + b * P.nsync;
                if (g > 0u)
                    r.e_lo = sy[g - 1u];
                if (g + 1u < P.nseg)
                    r.e_hi = sy[g];
                if (partial) {
                    if (G.g0 > 0u)
                        r.e0 = sy[G.g0 - 1u];
                    if (G.g1 < P.nseg)
                        r.e1 = sy[G.g1 - 1u];
                }
            }
        }
        return r;
    };
    // the unit with the thread's own number
    auto load_my_unit = [&](const TileGeom &G) {
        return load_unit_at(G, tid < G.units, ubi, G.g0 + ugr, u_bit_off, u_norms, u_sync);
    };
    // ---- this thread's share of the copy of a tile's words: global -> registers, registers -> LDS
    auto plan_words = [&](const TileGeom &G, const StreamRaw &r, const uint32_t *&src, uint32_t &cnt) {
        cnt = 0;
        src = s_words;
        if (my_stream < G.nstreams && !walk) {
            const StreamPart S = stream_part(P, G, r.bo0, r.bo1, r.e0, r.e1);
            cnt = min(S.nwords, P.stream_cap);
            src = s_words + S.first_word;
        }
    };
    auto load_words = [&](const uint32_t *src, uint32_t cnt, uint32_t (&w)[kWordsPerThread]) {
#pragma unroll
        for (uint32_t i = 0; i < kWordsPerThread; ++i) {
            const uint32_t wi = my_lane + (i << P.lanes_shift);
            w[i] = wi < cnt ? src[wi] : 0u;
        }
    };
    auto store_words = [&](const uint32_t (&w)[kWordsPerThread]) {
        const uint32_t base = my_stream * P.stream_cap + my_lane;     // < kStageWords for every thread
#pragma unroll
        for (uint32_t i = 0; i < kWordsPerThread; ++i)
            stage[base + (i << P.lanes_shift)] = w[i];
    };
    // ---- turn a unit's loaded metadata into what the parser needs
    auto plan_unit = [&](const TileGeom &G, bool valid, uint32_t k, uint32_t bi, uint32_t g, const UnitRaw &m,
                         bool &bad) {
        UnitPlan U{};
        if (!valid)
            return U;
        const uint64_t b = G.b0 + bi;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        const StreamPart S = stream_part(P, G, m.bo0, m.bo1, m.e0, m.e1);
        uint32_t bit_lo = 0, bit_hi = S.len, idx_lo = 0;
        U.idx_hi = nbk;
        U.forced = -1;
        if (P.sync_shift) {
            idx_lo = g << P.sync_shift;
            U.idx_hi = min(nbk, (g + 1u) << P.sync_shift);
            if (idx_lo >= nbk)
                return U;
            if (g > 0u) {
                if (m.e_lo & kSyncEmpty)
                    return U;
                bit_lo = m.e_lo & 0x1FFFFFu;
                U.forced = (int)(idx_lo + ((m.e_lo >> 21) & 0x3FFu));
            }
            if (g + 1u < P.nseg)
                bit_hi = m.e_hi & 0x1FFFFFu;
            if (bit_lo > bit_hi || bit_hi > S.len || (U.forced >= 0 && (uint32_t)U.forced >= U.idx_hi)) {
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
        U.tile_lo = partial ? (int)G.in_lo : -(int)(bi * P.bucket);
        const uint32_t sidx = bi * P.K + k;
        if (S.nwords <= P.stream_cap && sidx < kMaxStreams) {
            U.kind = 1;
            U.stage_off = sidx * P.stream_cap;
        } else {                                  // did not fit in LDS: read the words from global memory
            U.kind = 2;
            U.gwords = P.words[k] + S.first_word;     // (a per-lane fetch of the pointer: this path is rare)
            U.glast = S.nwords - 1u;
        }
        return U;
    };
    const double wscale = ldexp(1.0, -1 - (int)P.s);
    auto parse_unit = [&](const UnitPlan &U, bool &bad) {
        const double wnorm = (double)U.norm * wscale;
        double *tile_at0 = tile - U.tile_lo;     // address of in-bucket index 0 (never dereferenced outside the tile)
        if (U.kind == 1)
            decode_unit_fast(StagedWords{stage + U.stage_off}, lut, U.bit_lo, U.bit_hi, U.forced, U.idx_hi, P.s + 1u,
                             wnorm, tile_at0, bad);
        else if (U.kind == 2)
            decode_unit_fast(GlobalWords{U.gwords, U.glast}, lut, U.bit_lo, U.bit_hi, U.forced, U.idx_hi, P.s + 1u,
                             wnorm, tile_at0, bad);
    };
    // Tiles of a large bucket without a sync index: every tile parses the bucket from its first record in
    // global memory and keeps what lands inside.
    auto walk_unit = [&](const TileGeom &G, uint32_t k, bool &bad) {
        const uint64_t b = G.b0;
        const uint32_t nbk = (uint32_t)min((uint64_t)P.bucket, P.d - b * P.bucket);
        if (G.in_lo >= nbk)
            return;
        const uint64_t start = (P.bit_off[k][b] + 31ull) & ~31ull;
        const uint64_t end = P.bit_off[k][b + 1];
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
                const double val = ldexp(wnorm, (int)j);
                atomicAdd(&tile[(uint32_t)idx - G.in_lo], neg ? -val : val);
            }
            br.skip(rl);
            pos += rl;
            prev = idx;
        }
    };

    // ---- pipeline prologue
    bool bad = false;
    const uint32_t stride = gridDim.x;
    uint32_t t = blockIdx.x;                    // < ntiles by the launch
    TileGeom G = tile_geom(P, t);
    uint32_t words_next[kWordsPerThread];
    UnitPlan U;
    {
        const StreamRaw sr = load_stream(G);
        const UnitRaw um = load_my_unit(G);
        const uint32_t *src;
        uint32_t cnt;
        plan_words(G, sr, src, cnt);
        load_words(src, cnt, words_next);
        U = plan_unit(G, tid < G.units, uk, ubi, G.g0 + ugr, um, bad);
    }
    // metadata of the tile after this one, in flight from here on
    TileGeom Gn{};
    StreamRaw sr_n{};
    UnitRaw ur_n{};
    if (t + stride < P.ntiles) {
        Gn = tile_geom(P, t + stride);
        sr_n = load_stream(Gn);
        ur_n = load_my_unit(Gn);
    }
    for (uint32_t i = tid; i < kTileCoords / 2u; i += kDecodeWG)
        reinterpret_cast<double2 *>(tile)[i] = double2{0.0, 0.0};
    lut[tid] = gap_table_entry(tid);
    if (tid == 0)
        stage[kStageWords] = 0u;                 // the parser reads one word past the one it is in
    store_words(words_next);
    __syncthreads();

    for (;;) {
        // ---- start the loads of the metadata of the tile after the next and the copy of the next tile's
        // words, in this order and with every address computed first, so that nothing issued here has to be
        // waited for before the parse below
        const bool have_next = t + stride < P.ntiles;     // uniform
        UnitPlan Un{};
        const uint32_t *src_n = s_words;
        uint32_t cnt_n = 0;
        if (have_next) {
            plan_words(Gn, sr_n, src_n, cnt_n);
            Un = plan_unit(Gn, tid < Gn.units, uk, ubi, Gn.g0 + ugr, ur_n, bad);
        }
        TileGeom Gnn{};
        const bool have_nn = have_next && t + stride < P.ntiles - stride;
        if (have_nn) {
            Gnn = tile_geom(P, t + 2u * stride);
            sr_n = load_stream(Gnn);
            ur_n = load_my_unit(Gnn);
        }
        if (have_next)
            load_words(src_n, cnt_n, words_next);

        // ---- parse this tile's units
        if (walk) {
            for (uint32_t u = tid; u < G.units; u += kDecodeWG)
                walk_unit(G, u, bad);
        } else {
            parse_unit(U, bad);
            for (uint32_t u = tid + kDecodeWG; u < G.units; u += kDecodeWG) {
                uint32_t k, bi, g;
                unit_coords(G, u, k, bi, g);
                const UnitRaw m = load_unit_at(G, true, bi, g, P.bit_off[k], P.norms[k], P.sync[k]);
                const UnitPlan X = plan_unit(G, true, k, bi, g, m, bad);
                parse_unit(X, bad);
            }
        }
        __syncthreads();

        // ---- scale, round to fp32, write; leave the tile zeroed
        {
            float *o = P.out + G.c_lo;
            const double sc = (double)P.scale;
            const uint32_t span = G.span;
            const bool vec = (reinterpret_cast<uintptr_t>(o) & 15u) == 0;
            const uint32_t n4 = vec ? span >> 2 : 0u;
            for (uint32_t i = tid; i < n4; i += kDecodeWG) {
                double2 *src = reinterpret_cast<double2 *>(tile) + 2u * i;
                const double2 a = src[0], c = src[1];
                src[0] = double2{0.0, 0.0};
                src[1] = double2{0.0, 0.0};
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
                tile[i] = 0.0;
                o[i] = P.accumulate ? o[i] + r : r;
            }
        }
        if (!have_next)
            break;
        store_words(words_next);                 // the stage is free: this tile's parse is over
        __syncthreads();
        t += stride;
        G = Gn;
        U = Un;
        Gn = Gnn;
    }
    if (bad)
        atomicOr(P.flags, kFlagMalformed);
}

}  // namespace nuq
