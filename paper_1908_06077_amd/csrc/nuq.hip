// C ABI of the NUQSGD compression path (see include/nuq.h): argument checks, launch
// geometry and workspace layout.  All arithmetic of the method lives in the kernels.
#include "../../include/nuq.h"
#include "../../include/nuq_bench.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <type_traits>
#include <vector>

#include "nuq_decode_kernels.hpp"
#include "nuq_device.hpp"
#include "nuq_encode_kernels.hpp"
#include "nuq_fixed_kernels.hpp"
#include "nuq_huffman_kernels.hpp"
#include "nuq_sgd_kernels.hpp"
#include "nuq_table_kernels.hpp"

// Workspace of nuq_quantize_encode_static, the entry point that allocates nothing: staging slots, bit lengths and
// partial sums of the encoder's kernels.  Each device that loads the library holds its own copy until the process
// ends.  In host code this name only stands for the symbol: the device address comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[NUQ_STATIC_WORKSPACE_BYTES];

namespace {

using namespace nuq;

// Address of `scratch` on the current device, looked up once per device (with that device current) and kept.
void *static_workspace_ptr()
{
    static std::mutex mu;
    static void *ptrs[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return nullptr;
        ptrs[dev] = p;
    }
    return ptrs[dev];
}

// Sticky error flags, one word per device (each device holds its own copy of the symbol).
__device__ uint32_t g_flags;

uint32_t *flags_ptr()
{
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_flags)) != hipSuccess)
        return nullptr;
    return static_cast<uint32_t *>(p);
}

// ---- optional per-launch timing (benchmarks only) ----
struct Timing {
    std::vector<hipEvent_t> start, stop;
    std::vector<int32_t> entry;
    uint32_t cap = 0, used = 0;
} g_timing;

struct ScopedTiming {
    hipStream_t st;
    int slot = -1;
    ScopedTiming(int entry, hipStream_t s) : st(s)
    {
        if (g_timing.used < g_timing.cap) {
            slot = (int)g_timing.used++;
            g_timing.entry[slot] = entry;
            (void)hipEventRecord(g_timing.start[slot], st);
        }
    }
    ~ScopedTiming()
    {
        if (slot >= 0)
            (void)hipEventRecord(g_timing.stop[slot], st);
    }
};

uint32_t erc_len_host(uint32_t N)
{
    uint32_t len = 1;
    while (N > 1) {
        uint32_t w = 0;
        for (uint32_t x = N; x; x >>= 1)
            ++w;
        len += w;
        N = w - 1;
    }
    return len;
}

// A level table: s + 2 finite values, 0 = l_0 < l_1 < ... < l_{s+1} = 1.
bool valid_levels(const float *lev, uint32_t s)
{
    if (lev[0] != 0.0f || lev[s + 1] != 1.0f)
        return false;
    for (uint32_t j = 0; j <= s; ++j)
        if (!(lev[j] < lev[j + 1]))
            return false;
    return true;
}

bool valid_common(uint64_t d, uint32_t bucket, uint32_t s)
{
    return d >= 1 && bucket >= 1 && bucket <= NUQ_MAX_BUCKET && s >= 1 && s <= NUQ_MAX_S;
}

bool valid_sync(uint32_t sync_stride)
{
    return sync_stride == 0 ||
           (sync_stride >= 64 && sync_stride <= 1024 && (sync_stride & (sync_stride - 1)) == 0);
}

uint32_t log2u(uint32_t x)
{
    uint32_t l = 0;
    while ((1u << l) < x)
        ++l;
    return l;
}

// Decoder index of an ERC message: blocks of 2048 coordinates per bucket, and log2 of the pieces per block (the
// smallest power of two that is at least min(bucket, 2048) / sync_stride).
uint32_t sync_blocks(uint32_t bucket)
{
    return (bucket + (1u << kSyncBlockShift) - 1u) >> kSyncBlockShift;
}

uint32_t sync_pieces_shift(uint32_t bucket, uint32_t sync_stride)
{
    const uint32_t span = std::min(bucket, 1u << kSyncBlockShift);
    return log2u((span + sync_stride - 1u) / sync_stride);
}

uint32_t slot_words_for(uint32_t bucket, uint32_t s)
{
    const uint64_t bits = (uint64_t)bucket * (2u + erc_len_host(s + 1));
    return (uint32_t)(((bits + 31) / 32 + 3) & ~3ull);   // 16-byte multiple
}

struct Workspace {
    uint32_t *lens;
    uint64_t *chunk_sums;
    uint32_t *staging;
    uint64_t bytes;
};

Workspace carve(void *base, uint32_t K, uint64_t nb, uint32_t slot_words)
{
    auto up = [](uint64_t x) { return (x + 255) & ~255ull; };
    const uint64_t nchunks = (nb + kChunk - 1) / kChunk;
    uint64_t off = 0;
    Workspace w;
    char *p = static_cast<char *>(base);
    w.lens = reinterpret_cast<uint32_t *>(p + off);
    off += up((uint64_t)K * ((nb + 3) & ~3ull) * 4);
    w.chunk_sums = reinterpret_cast<uint64_t *>(p + off);
    off += up((uint64_t)K * (nchunks + 1) * 8);
    w.staging = reinterpret_cast<uint32_t *>(p + off);
    off += up((uint64_t)K * nb * slot_words * 4);
    w.bytes = off;
    return w;
}

// Team shape per bucket size: (threads per bucket, float4 rows per thread).
template <class F>
int dispatch_team(uint32_t bucket, F &&f)
{
    if (bucket <= 512)   // four buckets per wave
        return f(std::integral_constant<int, 16>{}, std::integral_constant<int, 8>{});
    if (bucket <= 2048)
        return f(std::integral_constant<int, 64>{}, std::integral_constant<int, 8>{});
    if (bucket <= 8192)
        return f(std::integral_constant<int, 256>{}, std::integral_constant<int, 8>{});
    if (bucket <= 16384)
        return f(std::integral_constant<int, 256>{}, std::integral_constant<int, 16>{});
    return f(std::integral_constant<int, 1024>{}, std::integral_constant<int, 8>{});
}

int check_launch()
{
    return hipGetLastError() == hipSuccess ? NUQ_OK : NUQ_EHIP;
}

// Grid of a per-bucket kernel: x = workgroups over the buckets of one worker, y = worker.
template <int TEAM>
bool bucket_grid(uint64_t nb, uint32_t K, dim3 &grid)
{
    const uint64_t gx = (nb + TeamGeom<TEAM>::kTeamsPerWG - 1) / TeamGeom<TEAM>::kTeamsPerWG;
    if (gx > 0x7fffffffull)
        return false;
    grid = dim3((uint32_t)gx, K);
    return true;
}

// Offsets and gather: lens and staging slots of K workers into their bit_off and words.
int launch_finish(const EncodeParams &P, const EncodeBatch &Wk, uint32_t K, const Workspace &w, hipStream_t st)
{
    const uint64_t nb = P.nb;
    const uint64_t nchunks = (nb + kChunk - 1) / kChunk;
    const uint64_t *prefix = nullptr;
    if (nb > kDirectSumMax) {
        hipLaunchKernelGGL(k_chunk_sums, dim3((uint32_t)nchunks, K), dim3(256), 0, st, w.lens, nb, P.nb_stride,
                           nchunks, w.chunk_sums);
        hipLaunchKernelGGL(k_chunk_scan, dim3(K), dim3(256), 0, st, w.chunk_sums, nchunks);
        prefix = w.chunk_sums;
    }
    const uint32_t fb = finish_buckets(P.bucket);
    // groups of fb buckets per workgroup: one where there are few (every workgroup slot of the chip gets work), up
    // to 8 where there are many (the sum of the lengths before a workgroup's first bucket is then paid once per 8)
    const uint64_t ngroups = (nb + fb - 1) / fb;
    const uint32_t per_wg = (uint32_t)std::min<uint64_t>(8, std::max<uint64_t>(1, ngroups * K / 16384));
    const dim3 fgrid((uint32_t)((ngroups + per_wg - 1) / per_wg), K);
    if (fb == 64u && per_wg > 1u)        // many small groups: one wave per workgroup, four times the groups in flight
        hipLaunchKernelGGL((k_finish<64, 64>), fgrid, dim3(64), 0, st, P, Wk, prefix, nchunks, per_wg);
    else if (fb == 64u)
        hipLaunchKernelGGL((k_finish<64, 256>), fgrid, dim3(256), 0, st, P, Wk, prefix, nchunks, per_wg);
    else
        hipLaunchKernelGGL((k_finish<16, 256>), fgrid, dim3(256), 0, st, P, Wk, prefix, nchunks, per_wg);
    return check_launch();
}

// MODE 0: fused norms + quantize + ENCODE from v.  MODE 1: ENCODE from level/sign bytes.  MODE 2: as 0 with the
// level table `levels` (host memory, s + 2 values) and the norm `norm_kind` selects.
template <int MODE>
int encode_batch(uint32_t K, const EncodeBatch &Wk, uint64_t d, uint32_t bucket, uint32_t s, uint32_t sync_stride,
                 void *workspace, uint64_t workspace_bytes, nuq_stream_t stream, const float *levels = nullptr,
                 uint32_t norm_kind = NUQ_NORM_L2)
{
    if (K < 1 || K > kMaxBatch || !valid_common(d, bucket, s) || !valid_sync(sync_stride) || !workspace ||
        (reinterpret_cast<uintptr_t>(workspace) & 15u))
        return NUQ_EINVAL;
    LevelTable T{};
    if (MODE == 2) {
        if (!levels || !valid_levels(levels, s) || (norm_kind != NUQ_NORM_L2 && norm_kind != NUQ_NORM_LINF))
            return NUQ_EINVAL;
        for (uint32_t j = 0; j < s + 2u; ++j)
            T.lev[j] = levels[j];
    }
    const uint32_t nsync = nuq_num_sync(bucket, sync_stride);
    for (uint32_t k = 0; k < K; ++k) {
        const EncodeWorker &w = Wk.w[k];
        if (!w.bit_off || !w.words || (nsync && !w.sync))
            return NUQ_EINVAL;
        if (MODE != 1 && (!w.v || !w.norms_out || (reinterpret_cast<uintptr_t>(w.v) & 3u)))
            return NUQ_EINVAL;
        if (MODE == 1 && !w.q_in)
            return NUQ_EINVAL;
    }
    const uint64_t nb = nuq_num_buckets(d, bucket);
    const uint32_t slot_words = slot_words_for(bucket, s);
    const Workspace w = carve(workspace, K, nb, slot_words);
    if (w.bytes > workspace_bytes)
        return NUQ_ECAPACITY;
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);

    EncodeParams P{};
    P.d = d;
    P.nb = nb;
    P.nb_stride = (nb + 3) & ~3ull;
    P.bucket = bucket;
    P.s = s;
    P.nsync = nsync;
    P.pieces_shift = nsync ? sync_pieces_shift(bucket, sync_stride) : 0;
    P.nblk = sync_blocks(bucket);
    P.slot_words = slot_words;
    P.lens = w.lens;
    P.staging = w.staging;
    P.flags = flags;
    P.norm_linf = norm_kind == NUQ_NORM_LINF ? 1u : 0u;
    int rc = dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        using G = TeamGeom<TEAM>;
        P.rows = (bucket + 4 * TEAM - 1) / (4 * TEAM);
        P.rec_cap = team_rec_cap(bucket);
        P.out_cap = team_out_cap(slot_words);
        P.lds_words = team_lds_words(P.rows, TEAM, P.rec_cap, P.out_cap, nsync, P.nblk);
        const size_t lds_bytes = (size_t)P.lds_words * 4 * G::kTeamsPerWG + 2 * 256 * 4;   // + the two code tables
        if (lds_bytes > 160 * 1024)
            return (int)NUQ_EINVAL;
        auto kern = k_encode<TEAM, VPT, MODE>;
        if (lds_bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return (int)NUQ_EHIP;
        dim3 grid;
        if (!bucket_grid<TEAM>(nb, K, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(MODE == 1 ? NUQ_T_ENCODE : NUQ_T_QUANTIZE_ENCODE, st);
        hipLaunchKernelGGL(kern, grid, dim3(G::kWG), lds_bytes, st, P, Wk, T);
        return check_launch();
    });
    if (rc != NUQ_OK)
        return rc;

    return launch_finish(P, Wk, K, w, st);
}

bool valid_fixed(uint32_t s, uint32_t b)
{
    return b >= 3 && b <= 8 && s + 2u <= (1u << (b - 1u));
}

// MODE 0: norms + quantizer + fixed-width packing from v.  MODE 1: packing of level|sign bytes.  MODE 2: as 0 with
// the level table `levels` (host memory, s + 2 values) and the norm `norm_kind` selects.
template <int MODE>
int pack_fixed_batch(uint32_t K, const EncodeBatch &Wk, uint64_t d, uint32_t bucket, uint32_t s, uint32_t b,
                     nuq_stream_t stream, const float *levels = nullptr, uint32_t norm_kind = NUQ_NORM_L2)
{
    if (K < 1 || K > kMaxBatch || !valid_common(d, bucket, s) || !valid_fixed(s, b))
        return NUQ_EINVAL;
    LevelTable T{};
    if (MODE == 2) {
        if (!levels || !valid_levels(levels, s) || (norm_kind != NUQ_NORM_L2 && norm_kind != NUQ_NORM_LINF))
            return NUQ_EINVAL;
        for (uint32_t j = 0; j < s + 2u; ++j)
            T.lev[j] = levels[j];
    }
    for (uint32_t k = 0; k < K; ++k) {
        const EncodeWorker &w = Wk.w[k];
        if (!w.words)
            return NUQ_EINVAL;
        if (MODE != 1 && (!w.v || !w.norms_out || (reinterpret_cast<uintptr_t>(w.v) & 3u)))
            return NUQ_EINVAL;
        if (MODE == 1 && !w.q_in)
            return NUQ_EINVAL;
    }
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    EncodeParams P{};
    P.d = d;
    P.nb = nuq_num_buckets(d, bucket);
    P.bucket = bucket;
    P.s = s;
    P.flags = flags;
    P.norm_linf = norm_kind == NUQ_NORM_LINF ? 1u : 0u;
    FixedParams F{};
    F.b = b;
    F.wpb = (bucket * b + 31u) / 32u;
    return dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        using G = TeamGeom<TEAM>;
        P.rows = (bucket + 4 * TEAM - 1) / (4 * TEAM);
        P.lds_words = fixed_lds_words(P.rows, TEAM, F.wpb);
        const size_t lds_bytes = (size_t)P.lds_words * 4 * G::kTeamsPerWG;
        if (lds_bytes > 160 * 1024)
            return (int)NUQ_EINVAL;
        auto kern = k_pack_fixed<TEAM, VPT, MODE>;
        if (lds_bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return (int)NUQ_EHIP;
        dim3 grid;
        if (!bucket_grid<TEAM>(P.nb, K, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(MODE == 1 ? NUQ_T_ENCODE : NUQ_T_QUANTIZE_ENCODE, st);
        hipLaunchKernelGGL(kern, grid, dim3(G::kWG), lds_bytes, st, P, Wk, F, T);
        return check_launch();
    });
}

// Canonical code tables from code lengths (host arithmetic).  False unless the lengths describe a complete
// prefix code over the s + 2 level indices with lengths 1..15.
bool huffman_tables(const uint8_t *lengths, uint32_t s, HuffmanCode &H)
{
    H = HuffmanCode{};
    H.nsym = s + 2u;
    uint32_t next = 0, code = 0, prev_len = 0;
    bool any = false;
    for (uint32_t len = 1; len <= 15u; ++len) {
        H.offset[len] = next;
        for (uint32_t j = 0; j < H.nsym; ++j) {
            if (lengths[j] != len)
                continue;
            if (any)
                code = (code + 1u) << (len - prev_len);
            any = true;
            prev_len = len;
            if (!H.count[len])
                H.first[len] = code;
            ++H.count[len];
            H.code[j] = code;
            H.len[j] = len;
            H.sorted[next++] = j;
            H.maxlen = len;
        }
    }
    return any && next == H.nsym && code == (1u << prev_len) - 1u;
}

struct HuffmanWorkspace {
    uint32_t *lens;
    uint64_t *chunk_sums;
    uint64_t bytes;
};

HuffmanWorkspace carve_huffman(void *base, uint64_t nb)
{
    HuffmanWorkspace w{};
    const uint64_t nb_stride = (nb + 3) & ~3ull, nchunks = (nb + kChunk - 1) / kChunk;
    uint8_t *p = static_cast<uint8_t *>(base);
    w.lens = reinterpret_cast<uint32_t *>(p);
    uint64_t off = (nb_stride * 4 + 15) & ~15ull;
    w.chunk_sums = reinterpret_cast<uint64_t *>(p + off);
    off += (nchunks + 1) * 8;
    w.bytes = (off + 15) & ~15ull;
    return w;
}

// Workgroups of the persistent decode kernel that the current device holds at once (0 on error).
// `variant` indexes kDecodeKernels: 2 * (3 * table + update) + big tile.
using DecodeKernel = void (*)(DecodeParams);
constexpr DecodeKernel kDecodeKernels[] = {
    k_decode_accumulate<false, kUpdateWrite, kTileCoords>,    k_decode_accumulate<false, kUpdateWrite, kTileCoordsBig>,
    k_decode_accumulate<false, kUpdateAdd, kTileCoords>,      k_decode_accumulate<false, kUpdateAdd, kTileCoordsBig>,
    k_decode_accumulate<false, kUpdateMomentum, kTileCoords>, k_decode_accumulate<false, kUpdateMomentum, kTileCoordsBig>,
    k_decode_accumulate<true, kUpdateWrite, kTileCoords>,     k_decode_accumulate<true, kUpdateWrite, kTileCoordsBig>,
    k_decode_accumulate<true, kUpdateAdd, kTileCoords>,       k_decode_accumulate<true, kUpdateAdd, kTileCoordsBig>,
};
constexpr uint32_t kDecodeVariants = sizeof(kDecodeKernels) / sizeof(kDecodeKernels[0]);
// the same variants of the one-wave tile decoder
constexpr DecodeKernel kDecodeWaveKernels[kDecodeVariants] = {
    k_decode_wave<false, kUpdateWrite, kTileCoords>,    k_decode_wave<false, kUpdateWrite, kTileCoordsBig>,
    k_decode_wave<false, kUpdateAdd, kTileCoords>,      k_decode_wave<false, kUpdateAdd, kTileCoordsBig>,
    k_decode_wave<false, kUpdateMomentum, kTileCoords>, k_decode_wave<false, kUpdateMomentum, kTileCoordsBig>,
    k_decode_wave<true, kUpdateWrite, kTileCoords>,     k_decode_wave<true, kUpdateWrite, kTileCoordsBig>,
    k_decode_wave<true, kUpdateAdd, kTileCoords>,       k_decode_wave<true, kUpdateAdd, kTileCoordsBig>,
};

uint32_t decode_resident_workgroups(uint32_t variant, bool wave)
{
    static uint32_t cached[2][kDecodeVariants][64] = {};
    int dev = 0;
    if (variant >= kDecodeVariants || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return 0;
    uint32_t &slot = cached[wave ? 1 : 0][variant][dev];
    if (!slot) {
        int per_cu = 0, cus = 0;
        const void *kern = reinterpret_cast<const void *>(wave ? kDecodeWaveKernels[variant] : kDecodeKernels[variant]);
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, (int)(wave ? kWaveWG : kDecodeWG), 0) !=
                hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || per_cu < 1 ||
            cus < 1)
            return 0;
        slot = (uint32_t)per_cu * (uint32_t)cus;
    }
    return slot;
}

}  // namespace

extern "C" {

uint64_t nuq_num_buckets(uint64_t d, uint32_t bucket)
{
    return bucket ? (d + bucket - 1) / bucket : 0;
}

uint32_t nuq_num_sync(uint32_t bucket, uint32_t sync_stride)
{
    if (!bucket || !valid_sync(sync_stride) || !sync_stride)
        return 0;
    return sync_blocks(bucket) << sync_pieces_shift(bucket, sync_stride);
}

uint32_t nuq_huffman_num_sync(uint32_t bucket, uint32_t sync_stride)
{
    return sync_stride ? (bucket + sync_stride - 1) / sync_stride - 1 : 0;
}

uint64_t nuq_max_words(uint64_t d, uint32_t bucket, uint32_t s)
{
    if (!bucket)
        return 0;
    return (d * (2u + erc_len_host(s + 1)) + 31) / 32 + nuq_num_buckets(d, bucket);
}

uint64_t nuq_encode_workspace_bytes(uint32_t K, uint64_t d, uint32_t bucket, uint32_t s)
{
    if (K < 1 || K > kMaxBatch || !valid_common(d, bucket, s))
        return 0;
    return carve(nullptr, K, nuq_num_buckets(d, bucket), slot_words_for(bucket, s)).bytes;
}

uint64_t nuq_workspace_bytes(uint64_t d, uint32_t bucket, uint32_t K)
{
    return nuq_encode_workspace_bytes(K, d, bucket, NUQ_MAX_S);
}

int nuq_bucket_norms(const float *v, uint64_t d, uint32_t bucket, float *norms, nuq_stream_t stream)
{
    if (!v || !norms || !valid_common(d, bucket, 1) || (reinterpret_cast<uintptr_t>(v) & 3u))
        return NUQ_EINVAL;
    EncodeParams P{};
    EncodeBatch Wk{};
    Wk.w[0].v = v;
    Wk.w[0].norms_out = norms;
    P.d = d;
    P.bucket = bucket;
    P.nb = nuq_num_buckets(d, bucket);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        dim3 grid;
        if (!bucket_grid<TEAM>(P.nb, 1, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(NUQ_T_NORMS, st);
        hipLaunchKernelGGL((k_bucket_norms<TEAM, VPT>), grid, dim3(TeamGeom<TEAM>::kWG), 0, st, P, Wk);
        return check_launch();
    });
}

int nuq_quantize(const float *v, uint64_t d, uint32_t bucket, uint32_t s, uint64_t seed, const float *norms,
                 uint8_t *q, nuq_stream_t stream)
{
    if (!v || !norms || !q || !valid_common(d, bucket, s) || (reinterpret_cast<uintptr_t>(v) & 3u))
        return NUQ_EINVAL;
    EncodeParams P{};
    EncodeBatch Wk{};
    Wk.w[0].v = v;
    Wk.w[0].norms_in = norms;
    Wk.w[0].q_out = q;
    Wk.w[0].seed = seed;
    P.d = d;
    P.bucket = bucket;
    P.s = s;
    P.nb = nuq_num_buckets(d, bucket);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        P.rows = (bucket + 4 * TEAM - 1) / (4 * TEAM);
        dim3 grid;
        if (!bucket_grid<TEAM>(P.nb, 1, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(NUQ_T_QUANTIZE, st);
        hipLaunchKernelGGL((k_quantize<TEAM, VPT>), grid, dim3(TeamGeom<TEAM>::kWG), 0, st, P, Wk);
        return check_launch();
    });
}

int nuq_bucket_norms_linf(const float *v, uint64_t d, uint32_t bucket, float *norms, nuq_stream_t stream)
{
    if (!v || !norms || !valid_common(d, bucket, 1) || (reinterpret_cast<uintptr_t>(v) & 3u))
        return NUQ_EINVAL;
    EncodeParams P{};
    EncodeBatch Wk{};
    Wk.w[0].v = v;
    Wk.w[0].norms_out = norms;
    P.d = d;
    P.bucket = bucket;
    P.nb = nuq_num_buckets(d, bucket);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        dim3 grid;
        if (!bucket_grid<TEAM>(P.nb, 1, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(NUQ_T_NORMS, st);
        hipLaunchKernelGGL((k_bucket_norms_linf<TEAM, VPT>), grid, dim3(TeamGeom<TEAM>::kWG), 0, st, P, Wk);
        return check_launch();
    });
}

int nuq_quantize_table(const float *v, uint64_t d, uint32_t bucket, uint32_t s, const float *levels, uint64_t seed,
                       const float *norms, uint8_t *q, nuq_stream_t stream)
{
    if (!v || !norms || !q || !levels || !valid_common(d, bucket, s) || !valid_levels(levels, s) ||
        (reinterpret_cast<uintptr_t>(v) & 3u))
        return NUQ_EINVAL;
    EncodeParams P{};
    EncodeBatch Wk{};
    LevelTable T{};
    for (uint32_t j = 0; j < s + 2u; ++j)
        T.lev[j] = levels[j];
    Wk.w[0].v = v;
    Wk.w[0].norms_in = norms;
    Wk.w[0].q_out = q;
    Wk.w[0].seed = seed;
    P.d = d;
    P.bucket = bucket;
    P.s = s;
    P.nb = nuq_num_buckets(d, bucket);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        P.rows = (bucket + 4 * TEAM - 1) / (4 * TEAM);
        dim3 grid;
        if (!bucket_grid<TEAM>(P.nb, 1, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(NUQ_T_QUANTIZE, st);
        hipLaunchKernelGGL((k_quantize_table<TEAM, VPT>), grid, dim3(TeamGeom<TEAM>::kWG), 0, st, P, Wk, T);
        return check_launch();
    });
}

int nuq_encode(const uint8_t *q, uint64_t d, uint32_t bucket, uint32_t s, uint32_t sync_stride, uint64_t *bit_off,
               uint32_t *words, uint64_t words_cap, uint32_t *sync, void *workspace, uint64_t workspace_bytes,
               nuq_stream_t stream)
{
    EncodeBatch Wk{};
    Wk.w[0].q_in = q;
    Wk.w[0].bit_off = bit_off;
    Wk.w[0].words = words;
    Wk.w[0].words_cap = words_cap;
    Wk.w[0].sync = sync;
    return encode_batch<1>(1, Wk, d, bucket, s, sync_stride, workspace, workspace_bytes, stream);
}

int nuq_quantize_encode(const float *v, uint64_t d, uint32_t bucket, uint32_t s, uint64_t seed,
                        uint32_t sync_stride, float *norms, uint64_t *bit_off, uint32_t *words, uint64_t words_cap,
                        uint32_t *sync, void *workspace, uint64_t workspace_bytes, nuq_stream_t stream)
{
    EncodeBatch Wk{};
    Wk.w[0].v = v;
    Wk.w[0].seed = seed;
    Wk.w[0].norms_out = norms;
    Wk.w[0].bit_off = bit_off;
    Wk.w[0].words = words;
    Wk.w[0].words_cap = words_cap;
    Wk.w[0].sync = sync;
    return encode_batch<0>(1, Wk, d, bucket, s, sync_stride, workspace, workspace_bytes, stream);
}

int nuq_quantize_encode_static(const float *v, uint64_t d, uint32_t bucket, uint32_t s, uint64_t seed,
                               uint32_t sync_stride, float *norms, uint64_t *bit_off, uint32_t *words,
                               uint64_t words_cap, uint32_t *sync, nuq_stream_t stream)
{
    const uint64_t need = nuq_encode_workspace_bytes(1, d, bucket, s);
    if (!need)
        return NUQ_EINVAL;
    if (need > NUQ_STATIC_WORKSPACE_BYTES)
        return NUQ_ECAPACITY;
    void *ws = static_workspace_ptr();
    if (!ws)
        return NUQ_EHIP;
    return nuq_quantize_encode(v, d, bucket, s, seed, sync_stride, norms, bit_off, words, words_cap, sync, ws,
                               NUQ_STATIC_WORKSPACE_BYTES, stream);
}

int nuq_quantize_encode_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d, uint32_t bucket,
                              uint32_t s, uint32_t sync_stride, float *const *norms, uint64_t *const *bit_off,
                              uint32_t *const *words, const uint64_t *words_cap, uint32_t *const *sync,
                              void *workspace, uint64_t workspace_bytes, nuq_stream_t stream)
{
    if (K < 1 || K > kMaxBatch || !v || !seeds || !norms || !bit_off || !words || !words_cap)
        return NUQ_EINVAL;
    EncodeBatch Wk{};
    for (uint32_t k = 0; k < K; ++k) {
        Wk.w[k].v = v[k];
        Wk.w[k].seed = seeds[k];
        Wk.w[k].norms_out = norms[k];
        Wk.w[k].bit_off = bit_off[k];
        Wk.w[k].words = words[k];
        Wk.w[k].words_cap = words_cap[k];
        Wk.w[k].sync = sync ? sync[k] : nullptr;
    }
    return encode_batch<0>(K, Wk, d, bucket, s, sync_stride, workspace, workspace_bytes, stream);
}

// levels: nullptr for the levels 2^(j-1-s), else the s + 2 values of a level table (host memory).
static int decode_accumulate_any(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                                 const uint32_t *const *words, const uint64_t *words_len,
                                 const uint32_t *const *sync, uint64_t d,
                                 uint32_t bucket, uint32_t s, uint32_t sync_stride, const float *levels, float scale,
                                 int accumulate, float *out, nuq_stream_t stream,
                                 const MomentumParams *momentum = nullptr)
{
    if (K < 1 || K > NUQ_MAX_WORKERS || !norms || !bit_off || !words || !words_len || !out ||
        !valid_common(d, bucket, s) ||
        !valid_sync(sync_stride) || (levels && !valid_levels(levels, s)))
        return NUQ_EINVAL;
    const uint32_t nsync = nuq_num_sync(bucket, sync_stride);
    if (nsync && !sync)
        return NUQ_EINVAL;
    DecodeParams P{};
    for (uint32_t k = 0; k < K; ++k) {
        if (!norms[k] || !bit_off[k] || !words[k] || (nsync && !sync[k]))
            return NUQ_EINVAL;
        P.norms[k] = norms[k];
        P.bit_off[k] = bit_off[k];
        P.words[k] = words[k];
        P.words_bits[k] = words_len[k] > (UINT64_MAX >> 5) ? UINT64_MAX : words_len[k] << 5;
        P.sync[k] = nsync ? sync[k] : nullptr;
    }
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    P.out = out;
    P.flags = flags;
    P.d = d;
    P.nb = nuq_num_buckets(d, bucket);
    P.K = K;
    P.bucket = bucket;
    P.s = s;
    P.nsync = nsync;
    P.nseg = nsync ? nsync : 1;                 // units (pieces) per bucket and worker
    P.pieces_shift = nsync ? sync_pieces_shift(bucket, sync_stride) : 0;
    P.scale = scale;
    if (momentum && levels)
        return NUQ_EINVAL;
    if (K == 1 && !levels && !momentum && (nsync || bucket <= 512)) {
        // one message: a lane per (bucket, sync segment), values stored directly (k_decode_single)
        const uint64_t wgs = (P.nb * P.nseg + kSingleWG - 1) / kSingleWG;
        if (wgs > 0x7fffffffull)
            return NUQ_EINVAL;
        ScopedTiming timing(NUQ_T_DECODE, static_cast<hipStream_t>(stream));
        if (accumulate)
            hipLaunchKernelGGL(k_decode_single<kUpdateAdd>, dim3((uint32_t)wgs), dim3(kSingleWG), 0,
                               static_cast<hipStream_t>(stream), P);
        else
            hipLaunchKernelGGL(k_decode_single<kUpdateWrite>, dim3((uint32_t)wgs), dim3(kSingleWG), 0,
                               static_cast<hipStream_t>(stream), P);
        return check_launch();
    }
    // Tiles of 4096 coordinates (32 KB of fp64, four workgroups per CU instead of eight) where the usual 2048 would
    // give the 64 parsing lanes at most 32 units: parts of large buckets of few workers.  The parse is bound by
    // instruction issue, so one full wave per SIMD gets through more records than two half-empty ones.
    const bool big = nsync && bucket >= kTileCoordsBig && (K << P.pieces_shift) <= 32u;
    const uint32_t tile_coords = big ? kTileCoordsBig : kTileCoords;
    const uint32_t variant = 2u * ((levels ? 3u : 0u) + (momentum ? (uint32_t)kUpdateMomentum
                                                                  : accumulate ? (uint32_t)kUpdateAdd
                                                                               : (uint32_t)kUpdateWrite)) + (big ? 1u : 0u);
    if (momentum) {
        P.yl = momentum->yl;
        P.alpha = momentum->alpha;
        P.la = momentum->l * momentum->alpha;
        P.mu = momentum->mu;
    }
    uint64_t ntiles;
    uint32_t max_streams;
    if (bucket <= kTileCoords) {
        const uint32_t by_size = kTileCoords / bucket, by_streams = kMaxStreams / K;
        P.buckets_per_tile = by_size < by_streams ? by_size : by_streams;
        P.tiles_per_bucket = 1;
        P.tile_coords = P.buckets_per_tile * bucket;
        P.segs_per_tile = P.nseg;
        ntiles = (P.nb + P.buckets_per_tile - 1) / P.buckets_per_tile;
        max_streams = P.buckets_per_tile * K;
    } else {
        P.buckets_per_tile = 0;
        P.tile_coords = tile_coords;
        P.tiles_per_bucket = (bucket + tile_coords - 1) / tile_coords;
        P.segs_per_tile = nsync ? (tile_coords >> kSyncBlockShift) << P.pieces_shift : 1;
        ntiles = P.nb * P.tiles_per_bucket;
        max_streams = K;
    }
    if (ntiles > 0x7fffffffull)
        return NUQ_EINVAL;
    P.ntiles = (uint32_t)ntiles;
    P.xcd_base = P.ntiles / 8u;
    P.xcd_rem = P.ntiles % 8u;
    // lanes (of the preparing wave) per stream for the copy of its words: the largest power of two that gives
    // every stream a group
    P.lanes_shift = 0;
    while ((2u << P.lanes_shift) * max_streams <= 64u)
        ++P.lanes_shift;
    P.stream_cap = kWordsPerLane << P.lanes_shift;
    // An odd stride when a tile has many streams (small buckets): lanes of different streams stand at like offsets,
    // and with a stride of 8 or 16 words they would read the same few banks (config 5: -5 %).  With few, long
    // streams the word given up costs more than the conflicts (config 4: +4 %), so those keep the full stride.
    P.stream_stride = max_streams >= 16u ? P.stream_cap - 1u : P.stream_cap;
    // One wave per workgroup where a tile holds at most 64 pieces and each stream's pieces fit the lanes that copy it
    // (every usual geometry with an index); the two-wave kernel takes the rest (no index, many workers, fine strides).
    const bool wave = nsync && max_streams <= 64u && P.segs_per_tile <= (1u << P.lanes_shift);
    uint32_t resident = decode_resident_workgroups(variant, wave);
    if (!resident)
        return NUQ_EHIP;
    resident &= ~7u;                            // a multiple of the eight XCDs (see xcd_tile)
    if (!resident)
        resident = 8u;
    // Every resident workgroup slot is used.  Workgroups walk tiles with stride `grid`, so the first
    // ntiles mod grid of them get one tile more than the rest: those are the workgroups that arrive first on their
    // CUs, whose parsing waves are the oldest on their SIMDs and run faster than the later ones.
    const uint32_t grid = P.ntiles < resident ? P.ntiles : resident;
    ScopedTiming timing(NUQ_T_DECODE, static_cast<hipStream_t>(stream));
    if (levels)
        for (uint32_t j = 0; j < s + 2u; ++j)
            P.lev[j] = levels[j];
    if (wave)
        hipLaunchKernelGGL(kDecodeWaveKernels[variant], dim3(grid), dim3(kWaveWG), 0, static_cast<hipStream_t>(stream), P);
    else
        hipLaunchKernelGGL(kDecodeKernels[variant], dim3(grid), dim3(kDecodeWG), 0, static_cast<hipStream_t>(stream), P);
    return check_launch();
}

int nuq_quantize_encode_table_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                    uint32_t bucket, uint32_t s, const float *levels, uint32_t norm_kind,
                                    uint32_t sync_stride, float *const *norms, uint64_t *const *bit_off,
                                    uint32_t *const *words, const uint64_t *words_cap, uint32_t *const *sync,
                                    void *workspace, uint64_t workspace_bytes, nuq_stream_t stream)
{
    if (K < 1 || K > kMaxBatch || !v || !seeds || !norms || !bit_off || !words || !words_cap || !levels)
        return NUQ_EINVAL;
    EncodeBatch Wk{};
    for (uint32_t k = 0; k < K; ++k) {
        Wk.w[k].v = v[k];
        Wk.w[k].seed = seeds[k];
        Wk.w[k].norms_out = norms[k];
        Wk.w[k].bit_off = bit_off[k];
        Wk.w[k].words = words[k];
        Wk.w[k].words_cap = words_cap[k];
        Wk.w[k].sync = sync ? sync[k] : nullptr;
    }
    return encode_batch<2>(K, Wk, d, bucket, s, sync_stride, workspace, workspace_bytes, stream, levels, norm_kind);
}

int nuq_decode_accumulate(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                          const uint32_t *const *words, const uint64_t *words_len, const uint32_t *const *sync,
                          uint64_t d, uint32_t bucket, uint32_t s, uint32_t sync_stride, float scale, int accumulate,
                          float *out, nuq_stream_t stream)
{
    return decode_accumulate_any(K, norms, bit_off, words, words_len, sync, d, bucket, s, sync_stride, nullptr, scale,
                                 accumulate, out, stream);
}

int nuq_decode_accumulate_table(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                                const uint32_t *const *words, const uint64_t *words_len,
                                const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                                uint32_t sync_stride, const float *levels, float scale, int accumulate, float *out,
                                nuq_stream_t stream)
{
    if (!levels)
        return NUQ_EINVAL;
    return decode_accumulate_any(K, norms, bit_off, words, words_len, sync, d, bucket, s, sync_stride, levels, scale,
                                 accumulate, out, stream);
}

uint64_t nuq_fixed_words(uint64_t d, uint32_t bucket, uint32_t b)
{
    if (!bucket || b < 3 || b > 8)
        return 0;
    return nuq_num_buckets(d, bucket) * (((uint64_t)bucket * b + 31) / 32);
}

int nuq_pack_fixed(const uint8_t *q, uint64_t d, uint32_t bucket, uint32_t s, uint32_t b, uint32_t *packed,
                   nuq_stream_t stream)
{
    EncodeBatch Wk{};
    Wk.w[0].q_in = q;
    Wk.w[0].words = packed;
    return pack_fixed_batch<1>(1, Wk, d, bucket, s, b, stream);
}

int nuq_quantize_pack_fixed_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                  uint32_t bucket, uint32_t s, uint32_t b, float *const *norms,
                                  uint32_t *const *packed, nuq_stream_t stream)
{
    if (K < 1 || K > kMaxBatch || !v || !seeds || !norms || !packed)
        return NUQ_EINVAL;
    EncodeBatch Wk{};
    for (uint32_t k = 0; k < K; ++k) {
        Wk.w[k].v = v[k];
        Wk.w[k].seed = seeds[k];
        Wk.w[k].norms_out = norms[k];
        Wk.w[k].words = packed[k];
    }
    return pack_fixed_batch<0>(K, Wk, d, bucket, s, b, stream);
}

int nuq_quantize_pack_fixed_table_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                        uint32_t bucket, uint32_t s, const float *levels, uint32_t norm_kind, uint32_t b,
                                        float *const *norms, uint32_t *const *packed, nuq_stream_t stream)
{
    if (K < 1 || K > kMaxBatch || !v || !seeds || !norms || !packed || !levels)
        return NUQ_EINVAL;
    EncodeBatch Wk{};
    for (uint32_t k = 0; k < K; ++k) {
        Wk.w[k].v = v[k];
        Wk.w[k].seed = seeds[k];
        Wk.w[k].norms_out = norms[k];
        Wk.w[k].words = packed[k];
    }
    return pack_fixed_batch<2>(K, Wk, d, bucket, s, b, stream, levels, norm_kind);
}

static int unpack_accumulate_fixed_any(uint32_t K, const float *const *norms, const uint32_t *const *packed, uint64_t d,
                                       uint32_t bucket, uint32_t s, const float *levels, uint32_t b, float scale,
                                       int accumulate, float *out, nuq_stream_t stream)
{
    if (K < 1 || K > NUQ_MAX_WORKERS || !norms || !packed || !out || !valid_common(d, bucket, s) ||
        !valid_fixed(s, b) || (levels && !valid_levels(levels, s)))
        return NUQ_EINVAL;
    UnpackParams P{};
    if (levels) {
        P.use_levels = 1u;
        for (uint32_t j = 0; j < s + 2u; ++j)
            P.lev[j] = levels[j];
    }
    for (uint32_t k = 0; k < K; ++k) {
        if (!norms[k] || !packed[k])
            return NUQ_EINVAL;
        P.norms[k] = norms[k];
        P.packed[k] = packed[k];
    }
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    P.out = out;
    P.flags = flags;
    P.d = d;
    P.K = K;
    P.bucket = bucket;
    P.s = s;
    P.b = b;
    P.wpb = (bucket * b + 31u) / 32u;
    P.scale = scale;
    P.accumulate = accumulate;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool wide = bucket % 32u == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
    const uint64_t threads = wide ? (d + 31) / 32 : d;
    const uint64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull)
        return NUQ_EINVAL;
    ScopedTiming timing(NUQ_T_DECODE, st);
    const dim3 grid((uint32_t)blocks);
    if (!wide) {
        hipLaunchKernelGGL(k_unpack_accumulate_fixed1, grid, dim3(256), 0, st, P);
    } else {
        // Tables of code values in LDS when those of the buckets a workgroup (8192 coordinates) can touch fit in
        // 16 KB beside the 33 KB output tile (three workgroups per CU at worst); else the arithmetic variant.
        const uint64_t nb = nuq_num_buckets(d, bucket);
        const bool tiled = 8192u % bucket == 0 || bucket % 8192u == 0;
        const uint64_t tabs = std::min<uint64_t>(nb, tiled ? std::max(1u, 8192u / bucket) : 8192u / bucket + 2u);
        const uint64_t lut_bytes = tabs * K * fixed_lut_entries(b) * sizeof(double);
        const bool lut = lut_bytes <= 16384u;
        P.lut_tabs = (uint32_t)tabs;
        const uint32_t dyn = lut ? (uint32_t)lut_bytes : 0u;
#define NUQ_LAUNCH_UNPACK(B)                                                                                   \
    do {                                                                                                       \
        if (lut)                                                                                               \
            hipLaunchKernelGGL((k_unpack_accumulate_fixed32<B, true>), grid, dim3(256), dyn, st, P);           \
        else                                                                                                   \
            hipLaunchKernelGGL((k_unpack_accumulate_fixed32<B, false>), grid, dim3(256), 0, st, P);            \
    } while (0)
        switch (b) {
        case 3: NUQ_LAUNCH_UNPACK(3); break;
        case 4: NUQ_LAUNCH_UNPACK(4); break;
        case 5: NUQ_LAUNCH_UNPACK(5); break;
        case 6: NUQ_LAUNCH_UNPACK(6); break;
        case 7: NUQ_LAUNCH_UNPACK(7); break;
        default: NUQ_LAUNCH_UNPACK(8); break;
        }
#undef NUQ_LAUNCH_UNPACK
    }
    return check_launch();
}

int nuq_unpack_accumulate_fixed(uint32_t K, const float *const *norms, const uint32_t *const *packed, uint64_t d,
                                uint32_t bucket, uint32_t s, uint32_t b, float scale, int accumulate, float *out,
                                nuq_stream_t stream)
{
    return unpack_accumulate_fixed_any(K, norms, packed, d, bucket, s, nullptr, b, scale, accumulate, out, stream);
}

int nuq_unpack_accumulate_fixed_table(uint32_t K, const float *const *norms, const uint32_t *const *packed, uint64_t d,
                                      uint32_t bucket, uint32_t s, const float *levels, uint32_t b, float scale,
                                      int accumulate, float *out, nuq_stream_t stream)
{
    if (!levels)
        return NUQ_EINVAL;
    return unpack_accumulate_fixed_any(K, norms, packed, d, bucket, s, levels, b, scale, accumulate, out, stream);
}


int nuq_level_histogram(const uint8_t *q, uint64_t d, uint64_t *hist, nuq_stream_t stream)
{
    if (!q || !hist || d < 1)
        return NUQ_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(64), 0, st, reinterpret_cast<unsigned long long *>(hist), 16u);
    const uint64_t blocks = (d + 256ull * 64 - 1) / (256ull * 64);
    hipLaunchKernelGGL(k_level_histogram, dim3((uint32_t)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, st, q, d,
                       reinterpret_cast<unsigned long long *>(hist));
    return check_launch();
}

int nuq_huffman_lengths(const uint64_t *hist, uint32_t s, uint8_t *lengths)
{
    if (!hist || !lengths || s < 1 || s > NUQ_MAX_S)
        return NUQ_EINVAL;
    // Huffman's algorithm on the weights hist[j] + 1 (Sec. 5, "Efficient Encoding"), as a merge of two queues: the
    // leaves sorted by (weight, symbol), and the merged nodes in order of creation, whose weights never decrease.
    // The next smallest node is at the front of one of the queues; of two equal weights the leaf goes first, which
    // is the order (weight, id) with leaves numbered before merged nodes.
    const uint32_t nsym = s + 2u;
    uint32_t leaf[16];                  // symbols, sorted
    for (uint32_t j = 0; j < nsym; ++j)
        leaf[j] = j;
    std::stable_sort(leaf, leaf + nsym, [&](uint32_t x, uint32_t y) { return hist[x] < hist[y]; });
    uint64_t merged_weight[16];
    uint32_t kid[16][2];                // children of merged node m: a symbol, or 16 + a merged node
    uint32_t nl = 0, nm_front = 0, nm = 0;
    auto take = [&](uint64_t &weight) {
        const bool from_leaves =
            nl < nsym && (nm_front == nm || hist[leaf[nl]] + 1u <= merged_weight[nm_front]);
        if (from_leaves) {
            weight = hist[leaf[nl]] + 1u;
            return leaf[nl++];
        }
        weight = merged_weight[nm_front];
        return 16u + nm_front++;
    };
    for (uint32_t m = 0; m + 1u < nsym; ++m) {
        uint64_t w0, w1;
        kid[m][0] = take(w0);
        kid[m][1] = take(w1);
        merged_weight[m] = w0 + w1;
        nm = m + 1u;
    }
    // depths from the root (the last merged node) down
    uint32_t depth[16] = {0};
    for (uint32_t m = nsym - 1u; m-- > 0u;)
        for (uint32_t c = 0; c < 2u; ++c) {
            if (kid[m][c] >= 16u)
                depth[kid[m][c] - 16u] = depth[m] + 1u;
            else
                lengths[kid[m][c]] = (uint8_t)(depth[m] + 1u);
        }
    return NUQ_OK;
}

uint64_t nuq_huffman_max_words(uint64_t d, uint32_t bucket)
{
    if (!bucket)
        return 0;
    return (d * 16 + 31) / 32 + nuq_num_buckets(d, bucket);
}

uint64_t nuq_encode_huffman_workspace_bytes(uint64_t d, uint32_t bucket)
{
    if (!bucket)
        return 0;
    return carve_huffman(nullptr, nuq_num_buckets(d, bucket)).bytes;
}

int nuq_encode_huffman(const uint8_t *q, uint64_t d, uint32_t bucket, uint32_t s, uint32_t sync_stride,
                       const uint8_t *lengths, uint64_t *bit_off, uint32_t *words, uint64_t words_cap,
                       uint32_t *sync, void *workspace, uint64_t workspace_bytes, nuq_stream_t stream)
{
    if (!q || !lengths || !bit_off || !words || !workspace || !valid_common(d, bucket, s) ||
        !valid_sync(sync_stride) || (reinterpret_cast<uintptr_t>(workspace) & 15u))
        return NUQ_EINVAL;
    const uint32_t nsync = nuq_huffman_num_sync(bucket, sync_stride);
    if (nsync && !sync)
        return NUQ_EINVAL;
    HuffmanCode H;
    if (!huffman_tables(lengths, s, H))
        return NUQ_EINVAL;
    const uint64_t nb = nuq_num_buckets(d, bucket);
    const HuffmanWorkspace w = carve_huffman(workspace, nb);
    if (w.bytes > workspace_bytes)
        return NUQ_ECAPACITY;
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    EncodeParams P{};
    EncodeBatch Wk{};
    Wk.w[0].q_in = q;
    Wk.w[0].bit_off = bit_off;
    Wk.w[0].words = words;
    Wk.w[0].words_cap = words_cap;
    Wk.w[0].sync = sync;
    P.d = d;
    P.nb = nb;
    P.nb_stride = (nb + 3) & ~3ull;
    P.bucket = bucket;
    P.s = s;
    P.sync_shift = nsync ? log2u(sync_stride) : 0;
    P.nsync = nsync;
    P.lens = w.lens;
    P.flags = flags;
    const uint64_t nchunks = (nb + kChunk - 1) / kChunk;
    return dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        using G = TeamGeom<TEAM>;
        P.rows = (bucket + 4 * TEAM - 1) / (4 * TEAM);
        P.lds_words = huffman_lds_words(P.rows, TEAM, bucket, nsync);
        const size_t lds_bytes = (size_t)P.lds_words * 4 * G::kTeamsPerWG;
        if (lds_bytes > 160 * 1024)
            return (int)NUQ_EINVAL;
        auto emit = k_huffman_emit<TEAM, VPT>;
        if (lds_bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(emit), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return (int)NUQ_EHIP;
        dim3 grid;
        if (!bucket_grid<TEAM>(nb, 1, grid))
            return (int)NUQ_EINVAL;
        hipLaunchKernelGGL((k_huffman_lens<TEAM, VPT>), grid, dim3(G::kWG), 0, st, P, Wk, H);
        hipLaunchKernelGGL(k_chunk_sums, dim3((uint32_t)nchunks, 1), dim3(256), 0, st, w.lens, nb, P.nb_stride, nchunks,
                           w.chunk_sums);
        hipLaunchKernelGGL(k_chunk_scan, dim3(1), dim3(256), 0, st, w.chunk_sums, nchunks);
        hipLaunchKernelGGL(k_bit_offsets, dim3((uint32_t)nchunks), dim3(256), 0, st, w.lens, nb, w.chunk_sums, bit_off);
        ScopedTiming timing(NUQ_T_ENCODE, st);
        hipLaunchKernelGGL(emit, grid, dim3(G::kWG), lds_bytes, st, P, Wk, H);
        return check_launch();
    });
}

// Staging words per bucket for the fused Huffman encoder: every coordinate at the longest codeword (s + 1 bits) and a
// sign bit.
uint32_t huffman_slot_words(uint32_t bucket, uint32_t s)
{
    const uint64_t bits = (uint64_t)bucket * (s + 2u);
    return (uint32_t)(((bits + 31) / 32 + 3) & ~3ull);
}

uint64_t nuq_encode_huffman_batch_workspace_bytes(uint32_t K, uint64_t d, uint32_t bucket, uint32_t s)
{
    if (K < 1 || K > kMaxBatch || !valid_common(d, bucket, s))
        return 0;
    return carve(nullptr, K, nuq_num_buckets(d, bucket), huffman_slot_words(bucket, s)).bytes;
}

int nuq_quantize_encode_huffman_batch(uint32_t K, const float *const *v, const uint64_t *seeds, uint64_t d,
                                      uint32_t bucket, uint32_t s, uint32_t sync_stride, const uint8_t *lengths,
                                      float *const *norms, uint64_t *const *bit_off, uint32_t *const *words,
                                      const uint64_t *words_cap, uint32_t *const *sync, void *workspace,
                                      uint64_t workspace_bytes, nuq_stream_t stream)
{
    if (K < 1 || K > kMaxBatch || !v || !seeds || !norms || !bit_off || !words || !words_cap || !lengths ||
        !workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || !valid_common(d, bucket, s) ||
        !valid_sync(sync_stride))
        return NUQ_EINVAL;
    const uint32_t nsync = nuq_huffman_num_sync(bucket, sync_stride);
    HuffmanCode H;
    if (!huffman_tables(lengths, s, H))
        return NUQ_EINVAL;
    EncodeBatch Wk{};
    for (uint32_t k = 0; k < K; ++k) {
        if (!v[k] || !norms[k] || !bit_off[k] || !words[k] || (nsync && (!sync || !sync[k])) ||
            (reinterpret_cast<uintptr_t>(v[k]) & 3u))
            return NUQ_EINVAL;
        Wk.w[k].v = v[k];
        Wk.w[k].seed = seeds[k];
        Wk.w[k].norms_out = norms[k];
        Wk.w[k].bit_off = bit_off[k];
        Wk.w[k].words = words[k];
        Wk.w[k].words_cap = words_cap[k];
        Wk.w[k].sync = nsync ? sync[k] : nullptr;
    }
    const uint64_t nb = nuq_num_buckets(d, bucket);
    const uint32_t slot_words = huffman_slot_words(bucket, s);
    const Workspace w = carve(workspace, K, nb, slot_words);
    if (w.bytes > workspace_bytes)
        return NUQ_ECAPACITY;
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    EncodeParams P{};
    P.d = d;
    P.nb = nb;
    P.nb_stride = (nb + 3) & ~3ull;
    P.bucket = bucket;
    P.s = s;
    P.sync_shift = nsync ? log2u(sync_stride) : 0;
    P.nsync = nsync;
    P.slot_words = slot_words;
    P.out_cap = slot_words;
    P.lens = w.lens;
    P.staging = w.staging;
    P.flags = flags;
    int rc = dispatch_team(bucket, [&](auto team_c, auto vpt_c) {
        constexpr int TEAM = decltype(team_c)::value, VPT = decltype(vpt_c)::value;
        using G = TeamGeom<TEAM>;
        P.rows = (bucket + 4 * TEAM - 1) / (4 * TEAM);
        P.lds_words = ((P.rows * TEAM + P.out_cap + 1u + nsync + 1u) & ~1u) + 64u;
        const size_t lds_bytes = (size_t)P.lds_words * 4 * G::kTeamsPerWG;
        if (lds_bytes > 160 * 1024)
            return (int)NUQ_EINVAL;
        auto kern = k_huffman_fused<TEAM, VPT>;
        if (lds_bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return (int)NUQ_EHIP;
        dim3 grid;
        if (!bucket_grid<TEAM>(nb, K, grid))
            return (int)NUQ_EINVAL;
        ScopedTiming timing(NUQ_T_QUANTIZE_ENCODE, st);
        hipLaunchKernelGGL(kern, grid, dim3(G::kWG), lds_bytes, st, P, Wk, H);
        return check_launch();
    });
    if (rc != NUQ_OK)
        return rc;
    return launch_finish(P, Wk, K, w, st);
}

int nuq_decode_huffman_batch(uint32_t K, const uint64_t *const *bit_off, const uint32_t *const *words,
                             const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                             uint32_t sync_stride, const uint8_t *lengths, uint8_t *const *q, nuq_stream_t stream)
{
    if (K < 1 || K > kMaxBatch || !bit_off || !words || !lengths || !q || !valid_common(d, bucket, s) ||
        !valid_sync(sync_stride))
        return NUQ_EINVAL;
    const uint32_t nsync = nuq_huffman_num_sync(bucket, sync_stride);
    if (nsync && !sync)
        return NUQ_EINVAL;
    HuffmanCode H;
    if (!huffman_tables(lengths, s, H))
        return NUQ_EINVAL;
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    HuffmanDecodeParams P{};
    for (uint32_t k = 0; k < K; ++k) {
        if (!bit_off[k] || !words[k] || !q[k] || (nsync && !sync[k]))
            return NUQ_EINVAL;
        P.w[k] = HuffmanStream{bit_off[k], words[k], nsync ? sync[k] : nullptr, q[k]};
    }
    P.flags = flags;
    P.d = d;
    P.nb = nuq_num_buckets(d, bucket);
    P.bucket = bucket;
    P.sync_shift = nsync ? log2u(sync_stride) : 0;
    P.nsync = nsync;
    P.nseg = nsync + 1;
    const uint64_t units = P.nb * P.nseg;
    const uint64_t blocks = nsync ? (units + 63) / 64 : (units + 255) / 256;
    if (blocks > 0x7fffffffull)
        return NUQ_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(NUQ_T_DECODE, st);
    // one staging row per thread: at most 1024 / 16 + 9 words
    const size_t direct_lds = (size_t)kHuffmanDirectWG * huffman_stage_stride(sync_stride) * 4u;
    bool direct = nsync && bucket % 16u == 0 && direct_lds <= 40u * 1024u;
    for (uint32_t k = 0; k < K && direct; ++k)
        direct = (reinterpret_cast<uintptr_t>(q[k]) & 15u) == 0;
    if (direct) {
        const uint64_t wgs = (units + kHuffmanDirectWG - 1) / kHuffmanDirectWG;
        hipLaunchKernelGGL(k_huffman_decode_direct, dim3((uint32_t)wgs, K), dim3(kHuffmanDirectWG), direct_lds, st, P,
                           H);
    } else if (nsync) {
        const size_t lds_bytes = 64u * (sync_stride / 4u + 1u + huffman_stage_stride(sync_stride)) * 4u;
        if (lds_bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(k_huffman_decode_tile),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return NUQ_EHIP;
        hipLaunchKernelGGL(k_huffman_decode_tile, dim3((uint32_t)blocks, K), dim3(64), lds_bytes, st, P, H);
    } else {
        hipLaunchKernelGGL(k_huffman_decode, dim3((uint32_t)blocks, K), dim3(256), 0, st, P, H);
    }
    return check_launch();
}

int nuq_decode_accumulate_huffman(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                                  const uint32_t *const *words, const uint64_t *words_len,
                                  const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                                  uint32_t sync_stride, const uint8_t *lengths, float scale, int accumulate,
                                  float *out, nuq_stream_t stream)
{
    if (K < 1 || K > NUQ_MAX_WORKERS || !norms || !bit_off || !words || !words_len || !sync || !lengths || !out ||
        !valid_common(d, bucket, s) || !valid_sync(sync_stride))
        return NUQ_EINVAL;
    const uint32_t nsync = nuq_huffman_num_sync(bucket, sync_stride);
    HuffmanCode H;
    if (!nsync || !huffman_tables(lengths, s, H))
        return NUQ_EINVAL;
    DecodeParams P{};
    for (uint32_t k = 0; k < K; ++k) {
        if (!norms[k] || !bit_off[k] || !words[k] || !sync[k])
            return NUQ_EINVAL;
        P.norms[k] = norms[k];
        P.bit_off[k] = bit_off[k];
        P.words[k] = words[k];
        P.words_bits[k] = words_len[k] > (UINT64_MAX >> 5) ? UINT64_MAX : words_len[k] << 5;
        P.sync[k] = sync[k];
    }
    P.out = out;
    P.d = d;
    P.nb = nuq_num_buckets(d, bucket);
    P.K = K;
    P.bucket = bucket;
    P.s = s;
    P.scale = scale;
    P.nsync = nsync;
    P.nseg = nsync + 1u;                        // pieces per bucket: ceil(bucket / sync_stride)
    P.sync_shift = log2u(sync_stride);
    P.pieces_shift = log2u(kTileCoords / sync_stride);
    // tiles as for the ERC strings: several whole buckets, or 2048 coordinates of one
    uint64_t ntiles;
    uint32_t max_streams;
    if (bucket <= kTileCoords) {
        const uint32_t by_size = kTileCoords / bucket, by_streams = kMaxStreams / K;
        P.buckets_per_tile = by_size < by_streams ? by_size : by_streams;
        P.tiles_per_bucket = 1;
        P.tile_coords = P.buckets_per_tile * bucket;
        P.segs_per_tile = P.nseg;
        ntiles = (P.nb + P.buckets_per_tile - 1) / P.buckets_per_tile;
        max_streams = P.buckets_per_tile * K;
    } else {
        P.buckets_per_tile = 0;
        P.tile_coords = kTileCoords;
        P.tiles_per_bucket = (bucket + kTileCoords - 1) / kTileCoords;
        P.segs_per_tile = kTileCoords >> P.sync_shift;
        ntiles = P.nb * P.tiles_per_bucket;
        max_streams = K;
    }
    if (ntiles > 0x7fffffffull)
        return NUQ_EINVAL;
    P.ntiles = (uint32_t)ntiles;
    P.xcd_base = P.ntiles / 8u;
    P.xcd_rem = P.ntiles % 8u;
    while ((2u << P.lanes_shift) * max_streams <= 64u)
        ++P.lanes_shift;
    // the lanes that copy a stream's words parse its pieces: a piece per lane
    if (P.segs_per_tile > (1u << P.lanes_shift))
        return NUQ_EINVAL;
    P.stream_cap = HuffmanWaveCodec::kWordsPerLane << P.lanes_shift;
    P.stream_stride = max_streams >= 16u ? P.stream_cap - 1u : P.stream_cap;
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    P.flags = flags;
    auto kern = accumulate ? k_decode_wave_huffman<kUpdateAdd> : k_decode_wave_huffman<kUpdateWrite>;
    static uint32_t cached[2][64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return NUQ_EHIP;
    uint32_t &resident = cached[accumulate ? 1 : 0][dev];
    if (!resident) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kern), (int)kWaveWG,
                                                         0) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || per_cu < 1 ||
            cus < 1)
            return NUQ_EHIP;
        resident = ((uint32_t)per_cu * (uint32_t)cus) & ~7u;          // a multiple of the eight XCDs (see xcd_tile)
        if (!resident)
            resident = 8u;
    }
    const uint32_t grid = P.ntiles < resident ? P.ntiles : resident;
    ScopedTiming timing(NUQ_T_DECODE, static_cast<hipStream_t>(stream));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kWaveWG), 0, static_cast<hipStream_t>(stream), P, H);
    return check_launch();
}

int nuq_decode_huffman(const uint64_t *bit_off, const uint32_t *words, const uint32_t *sync, uint64_t d,
                       uint32_t bucket, uint32_t s, uint32_t sync_stride, const uint8_t *lengths, uint8_t *q,
                       nuq_stream_t stream)
{
    return nuq_decode_huffman_batch(1, &bit_off, &words, &sync, d, bucket, s, sync_stride, lengths, &q, stream);
}

int nuq_average_levels(uint32_t K, const float *const *norms, const uint8_t *const *q, uint64_t d, uint32_t bucket,
                       uint32_t s, float scale, int accumulate, float *out, nuq_stream_t stream)
{
    if (K < 1 || K > NUQ_MAX_WORKERS || !norms || !q || !out || !valid_common(d, bucket, s))
        return NUQ_EINVAL;
    AverageParams P{};
    bool aligned = bucket % 4u == 0;
    for (uint32_t k = 0; k < K; ++k) {
        if (!norms[k] || !q[k])
            return NUQ_EINVAL;
        P.norms[k] = norms[k];
        P.q[k] = q[k];
        aligned = aligned && (reinterpret_cast<uintptr_t>(q[k]) & 3u) == 0;
    }
    P.out = out;
    P.d = d;
    P.K = K;
    P.bucket = bucket;
    P.s = s;
    P.scale = scale;
    P.accumulate = accumulate;
    bool wide = aligned && bucket % 16u == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
    for (uint32_t k = 0; k < K && wide; ++k)
        wide = (reinterpret_cast<uintptr_t>(q[k]) & 15u) == 0;
    const uint64_t threads = wide ? (d + 15) / 16 : aligned ? (d + 3) / 4 : d, blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull)
        return NUQ_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (wide) {
        // value tables in LDS when those of the buckets a workgroup (4096 coordinates) can touch fit in 16 KB
        const uint64_t nb = nuq_num_buckets(d, bucket);
        const bool tiled = 4096u % bucket == 0 || bucket % 4096u == 0;
        const uint64_t tabs = std::min<uint64_t>(nb, tiled ? std::max(1u, 4096u / bucket) : 4096u / bucket + 2u);
        const uint64_t lut_bytes = tabs * K * 32u * sizeof(double);
        P.lut_tabs = (uint32_t)tabs;
        if (lut_bytes <= 16384u)
            hipLaunchKernelGGL(k_average_levels16<true>, dim3((uint32_t)blocks), dim3(256), (uint32_t)lut_bytes, st, P);
        else
            hipLaunchKernelGGL(k_average_levels16<false>, dim3((uint32_t)blocks), dim3(256), 0, st, P);
    }
    else if (aligned)
        hipLaunchKernelGGL(k_average_levels<4>, dim3((uint32_t)blocks), dim3(256), 0, st, P);
    else
        hipLaunchKernelGGL(k_average_levels<1>, dim3((uint32_t)blocks), dim3(256), 0, st, P);
    return check_launch();
}

int nuq_momentum_step(float *w, float *yl, const float *g, uint64_t d, float alpha, float mu, float l,
                      nuq_stream_t stream)
{
    if (!std::isfinite(alpha) || !std::isfinite(mu) || !std::isfinite(l) || mu < 0.0f || !(mu < 1.0f))
        return NUQ_EINVAL;
    if (d == 0)
        return NUQ_OK;
    if (!w || !yl || !g)
        return NUQ_EINVAL;
    const bool vec = ((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(yl) |
                       reinterpret_cast<uintptr_t>(g)) & 15u) == 0;
    const uint64_t threads = vec ? (d + 3) / 4 : d, blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull)
        return NUQ_EINVAL;
    const MomentumParams P{w, yl, g, d, (double)alpha, (double)mu, (double)l};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (vec)
        hipLaunchKernelGGL(k_momentum_step<true>, dim3((uint32_t)blocks), dim3(256), 0, st, P);
    else
        hipLaunchKernelGGL(k_momentum_step<false>, dim3((uint32_t)blocks), dim3(256), 0, st, P);
    return check_launch();
}

int nuq_decode_momentum_step(uint32_t K, const float *const *norms, const uint64_t *const *bit_off,
                             const uint32_t *const *words, const uint64_t *words_len,
                             const uint32_t *const *sync, uint64_t d, uint32_t bucket, uint32_t s,
                             uint32_t sync_stride, float scale, float alpha, float mu, float l, float *w, float *yl,
                             nuq_stream_t stream)
{
    if (!std::isfinite(alpha) || !std::isfinite(mu) || !std::isfinite(l) || mu < 0.0f || !(mu < 1.0f) || !yl)
        return NUQ_EINVAL;
    const MomentumParams M{w, yl, nullptr, d, (double)alpha, (double)mu, (double)l};
    return decode_accumulate_any(K, norms, bit_off, words, words_len, sync, d, bucket, s, sync_stride, nullptr, scale,
                                 0, w, stream, &M);
}

int nuq_moments_accumulate(const float *g, double *sum, double *sumsq, uint64_t d, nuq_stream_t stream)
{
    if (d == 0)
        return NUQ_OK;
    if (!g || !sum || !sumsq)
        return NUQ_EINVAL;
    const bool vec = (reinterpret_cast<uintptr_t>(g) & 7u) == 0 &&
                     ((reinterpret_cast<uintptr_t>(sum) | reinterpret_cast<uintptr_t>(sumsq)) & 15u) == 0;
    const uint64_t threads = vec ? (d + 1) / 2 : d, blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull)
        return NUQ_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (vec)
        hipLaunchKernelGGL(k_moments_accumulate<true>, dim3((uint32_t)blocks), dim3(256), 0, st, g, sum, sumsq, d);
    else
        hipLaunchKernelGGL(k_moments_accumulate<false>, dim3((uint32_t)blocks), dim3(256), 0, st, g, sum, sumsq, d);
    return check_launch();
}

int nuq_normalized_variance(const double *sum, const double *sumsq, uint64_t d, uint64_t M, void *workspace,
                            uint64_t workspace_bytes, double *out2, nuq_stream_t stream)
{
    static_assert(NUQ_VARIANCE_WORKSPACE_BYTES == kVarianceBlocks * 2u * sizeof(double), "workspace size");
    if (M < 1 || !out2 || !workspace || workspace_bytes < NUQ_VARIANCE_WORKSPACE_BYTES ||
        (reinterpret_cast<uintptr_t>(workspace) & 7u) != 0 || (d > 0 && (!sum || !sumsq)))
        return NUQ_EINVAL;
    double *partial = static_cast<double *>(workspace);
    const uint32_t blocks = (uint32_t)std::min<uint64_t>(kVarianceBlocks, std::max<uint64_t>(1, (d + 255) / 256));
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_variance_partials, dim3(blocks), dim3(256), 0, st, sum, sumsq, d, 1.0 / (double)M, partial);
    hipLaunchKernelGGL(k_variance_finish, dim3(1), dim3(256), 0, st, partial, blocks, out2);
    return check_launch();
}

int nuq_last_error_flags(uint32_t *host_flags, nuq_stream_t stream)
{
    if (!host_flags)
        return NUQ_EINVAL;
    uint32_t *flags = flags_ptr();
    if (!flags)
        return NUQ_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(host_flags, flags, sizeof(uint32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return NUQ_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess)
        return NUQ_EHIP;
    const uint32_t zero = 0;
    if (hipMemcpyAsync(flags, &zero, sizeof(uint32_t), hipMemcpyHostToDevice, st) != hipSuccess)
        return NUQ_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess)
        return NUQ_EHIP;
    return NUQ_OK;
}

int nuq_timing_begin(uint32_t max_launches)
{
    if (max_launches > 4096 || g_timing.cap != 0)
        return NUQ_EINVAL;
    g_timing.start.resize(max_launches);
    g_timing.stop.resize(max_launches);
    g_timing.entry.assign(max_launches, 0);
    for (uint32_t i = 0; i < max_launches; ++i)
        if (hipEventCreate(&g_timing.start[i]) != hipSuccess || hipEventCreate(&g_timing.stop[i]) != hipSuccess)
            return NUQ_EHIP;
    g_timing.used = 0;
    g_timing.cap = max_launches;
    return NUQ_OK;
}

int nuq_timing_collect(float *ms, int32_t *entry, uint32_t cap, uint32_t *count)
{
    if (!ms || !entry || !count)
        return NUQ_EINVAL;
    int rc = NUQ_OK;
    uint32_t n = 0;
    for (uint32_t i = 0; i < g_timing.used; ++i) {
        if (hipEventSynchronize(g_timing.stop[i]) != hipSuccess)
            rc = NUQ_EHIP;
        float t = 0.f;
        if (hipEventElapsedTime(&t, g_timing.start[i], g_timing.stop[i]) != hipSuccess)
            rc = NUQ_EHIP;
        if (n < cap) {
            ms[n] = t;
            entry[n] = g_timing.entry[i];
            ++n;
        }
    }
    for (uint32_t i = 0; i < g_timing.cap; ++i) {
        (void)hipEventDestroy(g_timing.start[i]);
        (void)hipEventDestroy(g_timing.stop[i]);
    }
    g_timing = Timing{};
    *count = n;
    return rc;
}

}  // extern "C"
