// Device side of libzipmoe: zm_decode_experts and its gfx950 kernels.
//
// One launch decodes every tensor of the experts a MoE layer's gate selected
// (ZipMoE, arXiv 2601.21198, Sec. 3.1 "Real-time Inference"): each wavefront
// takes one stream of one E-chunk, entropy-decodes its exponent bytes and merges
// them with the raw sign-mantissa bytes into bf16 words (the tensor recovery
// step of Sec. 3.3) without the exponents ever leaving registers.
//
// Work decomposition
//   grid    x: workgroups of kWaves consecutive streams, y: tensor
//   wave    one stream: stream_values consecutive values, tiles of 512
//   lane j  owns values 8j..8j+7 of every tile: one 64-bit load of
//           sign-mantissa bytes and one 128-bit store of bf16 words per tile,
//           both contiguous across the wave (512 B and 1 KiB per instruction)
//
// Per wave
//   1. one read of the chunk's table entry locates the stream; its words are
//      requested with 128-bit loads (a4) -- first, because decoding can not start
//      without them -- and go to LDS;
//   2. the sign-mantissa bytes of the stream's first eight tiles are requested;
//   3. the decode table goes to LDS (a3) as two byte tables (code length, symbol)
//      at fixed LDS addresses, replicated to the full index width;
//   4. lock-step decode (a5): every lane keeps two words (lo, hi) of its own
//      bitstream and a bit position; per round it extracts a 32-bit window with
//      one funnel shift and decodes R symbols by table lookup;
//   5. after a round the lanes whose position passed 32 bits take the next
//      words of the stream: a ballot marks them, a prefix count over the ballot
//      (mbcnt) gives each its word (a6);
//   6. the eight decoded exponent bytes are merged with the sign-mantissa bytes
//      by byte-parallel bit operations and stored (a8).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "zipmoe.h"

namespace {

constexpr int kMaxTasks = 48;     // tensors per launch; 80 B each keeps the kernel arguments under 4 KiB
constexpr uint32_t kTile = 512;
constexpr int kGroup = 8;         // tiles whose sign-mantissa loads are in flight together

// One tensor to decode.  Its parts may live in separate allocations (a cache may keep only some of them
// resident), so each has a pointer of its own.
struct Task {
    const uint8_t *lut;       // decode table: 2^max_len entries of 16 bits
    const uint8_t *sm;        // sign-mantissa section
    const uint8_t *echunks;   // E-chunk region (what the blob holds from e_offset on)
    const uint64_t *table;    // chunk table (entries of 8 + 4*(streams_per_chunk+1) bytes, rounded up to 8); offsets count from the start of the blob
    uint16_t *out;
    uint64_t n_values;
    uint64_t e_offset;        // blob offset of the E-chunk region
    uint64_t e_size;          // bytes in the E-chunk region
    uint32_t stream_values;
    uint32_t streams_per_chunk;
    uint32_t n_streams;
    uint32_t max_len;
};

struct Launch {
    uint32_t n_tasks;
    uint32_t stream_cap_words;   // LDS words reserved per wave for its stream
    uint32_t pad[2];
    Task task[kMaxTasks];        // blockIdx.y selects the task
};
static_assert(sizeof(Launch) <= 4096, "kernel arguments must stay under 4 KiB");

// base + number of set bits of `mask` below this lane (the exclusive prefix count of a ballot)
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, uint32_t base)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), base));
}

// Sec. 3.3 recovery of four values at once: e4 and sm4 hold four exponent bytes
// and four sign-mantissa bytes; the results are the four bf16 words, two per register.
__device__ __forceinline__ void recover4(uint32_t e4, uint32_t sm4, uint32_t &w01, uint32_t &w23)
{
    const uint32_t hi4 = (sm4 & 0x80808080u) | ((e4 >> 1) & 0x7F7F7F7Fu);   // s eeeeeee
    const uint32_t lo4 = ((e4 << 7) & 0x80808080u) | (sm4 & 0x7F7F7F7Fu);   // e mmmmmmm
    w01 = __builtin_amdgcn_perm(hi4, lo4, 0x05010400u);
    w23 = __builtin_amdgcn_perm(hi4, lo4, 0x07030602u);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// kStreaming: the output of the launch is larger than the last-level cache, so the stores are marked
// non-temporal; smaller outputs are written normally and tend to stay cached for their consumer.
template <bool kStreaming = false>
__device__ __forceinline__ void recover_and_store(uint16_t *dst, uint2 e, uint2 sm)
{
    uint4 w;
    recover4(e.x, sm.x, w.x, w.y);
    recover4(e.y, sm.y, w.z, w.w);
    if constexpr (kStreaming) __builtin_nontemporal_store((u32x4){w.x, w.y, w.z, w.w}, reinterpret_cast<u32x4 *>(dst));
    else *reinterpret_cast<uint4 *>(dst) = w;
}

// Same for a lane that owns fewer than eight values of the tile.
__device__ __forceinline__ void recover_and_store_partial(uint16_t *dst, uint2 e, uint2 sm, int32_t left)
{
    uint32_t ws[4];
    recover4(e.x, sm.x, ws[0], ws[1]);
    recover4(e.y, sm.y, ws[2], ws[3]);
#pragma unroll
    for (int q = 0; q < 8; ++q)
        if (q < left) dst[q] = static_cast<uint16_t>(ws[q >> 1] >> (16 * (q & 1)));
}

template <int R>
struct Code {
    static constexpr int kIndexBits = R == 4 ? 8 : 12;     // R = 4 iff the longest code has at most 8 bits
    static constexpr uint32_t kEntries = 1u << kIndexBits;
};

// Lock-step decoder state of one lane (a5, a6).  len_tab / sym_tab are the workgroup's byte tables.
template <int R>
struct Decoder {
    const uint32_t *words;
    uint32_t last_word;
    uint32_t lo = 0, hi = 0;      // words q and q+1 of this lane's bitstream
    uint32_t pos = 0;             // bits of lo already used (< 32 at the start of a round)
    uint32_t next = 128;          // next unread word of the stream (uniform over the wave)

    // Decodes this lane's eight exponent bytes of one tile.
    __device__ __forceinline__ uint2 tile(const uint8_t *len_tab, const uint8_t *sym_tab)
    {
        constexpr uint32_t kMask = Code<R>::kEntries - 1u;
        uint32_t e[2] = {0u, 0u};
#pragma unroll
        for (int r = 0; r < 8 / R; ++r) {
            // R symbols out of one 32-bit window; `used` is the bit offset of the next code in it
            const uint32_t win = __builtin_amdgcn_alignbit(hi, lo, pos);
            uint32_t used = 0;
            uint32_t s[R];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const uint32_t idx = (win >> used) & kMask;
                s[k] = sym_tab[idx];
                used += len_tab[idx];
            }
            pos += used;
            // byte 0 of each symbol register, packed with byte permutes (0x0c selects a zero byte)
            if constexpr (R == 4) {
                const uint32_t s01 = __builtin_amdgcn_perm(s[1], s[0], 0x0c0c0400u);
                e[r] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(s[3], s[2], 0x0c0c0400u), s01, 0x05040100u);
            } else {
                const uint32_t s01 = __builtin_amdgcn_perm(s[1], s[0], 0x0c0c0400u);
                e[r >> 1] = (r & 1) ? __builtin_amdgcn_perm(s01, e[r >> 1], 0x05040100u) : s01;
            }
            // a6: lanes that crossed a word boundary take the stream's next words, in lane order: the
            // ballot's prefix count is each taker's offset.  Written without branches (every lane reads
            // a word, only the takers keep it) so that the whole tile is one basic block.  After the
            // stream's last round the word read here is never used.
            const bool take = pos >= 32u;
            const uint64_t takers = __ballot(take);
            const uint32_t fresh = words[min(lanes_below(takers, next), last_word)];
            lo = take ? hi : lo;
            hi = take ? fresh : hi;
            pos &= 31u;
            next += static_cast<uint32_t>(__builtin_popcountll(takers));
        }
        return make_uint2(e[0], e[1]);
    }
};

// R: symbols per round; kWaves: waves (streams) per workgroup; kStreaming: non-temporal stores
template <int R, int kWaves, bool kStreaming>
__global__ void __launch_bounds__(64 * kWaves) zm_decode_kernel(const Launch P)
{
    // Byte tables of the workgroup's tensor, at fixed LDS addresses so that a lookup is one LDS read with
    // an immediate offset.  The lookups of a wave hit random words of a 64-word table and do collide on
    // banks (the counters show conflicts in 45 % of the LDS-active cycles), but waves spend about 1 % of
    // their cycles waiting for LDS: confining the lookups to 32- or 16-word tables changed nothing.
    __shared__ __align__(16) uint8_t len_tab[Code<R>::kEntries];
    __shared__ __align__(16) uint8_t sym_tab[Code<R>::kEntries];
    extern __shared__ __align__(16) uint32_t stream_lds[];

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // grid: x = workgroup inside the tensor, y = tensor.  The task is copied with one batch of scalar loads.
    const Task t = P.task[blockIdx.y];
    uint32_t *words = stream_lds + wave * P.stream_cap_words;

    const uint32_t g = blockIdx.x * kWaves + wave;
    bool active = g < t.n_streams;
    const uint32_t W = t.stream_values;
    const uint64_t v0 = static_cast<uint64_t>(g) * W;              // first value of the stream in the tensor
    uint32_t sn = 0, mode = ZM_MODE_RAW, tiles = 0;
    const uint8_t *raw = nullptr;
    if (active) {
        const uint64_t rest = t.n_values - v0;
        sn = rest < W ? static_cast<uint32_t>(rest) : W;
        tiles = (sn + kTile - 1) / kTile;
    }
    const bool full = sn != 0 && sn % (kGroup * kTile) == 0;       // the common shape: whole groups of eight tiles
    const uint8_t *sm_base = t.sm + v0 + lane * 8u;
    const int32_t mine = static_cast<int32_t>(sn) - static_cast<int32_t>(lane * 8u);   // values left from this lane's first one

    uint4 held_a = make_uint4(0u, 0u, 0u, 0u), held_b = held_a;   // first 2 KiB of the stream
    uint32_t n_held = 0;
    if (active) {
        const uint32_t c = g / t.streams_per_chunk, s = g % t.streams_per_chunk;
        // one read of the chunk's table entry gives the chunk's place and mode and this stream's extent
        const uint32_t stride = (8u + 4u * (t.streams_per_chunk + 1u) + 7u) & ~7u;
        const uint8_t *entry = reinterpret_cast<const uint8_t *>(t.table) + static_cast<uint64_t>(c) * stride;
        const uint64_t ent = *reinterpret_cast<const uint64_t *>(entry);
        const uint32_t o0 = reinterpret_cast<const uint32_t *>(entry + 8)[s];
        const uint32_t o1 = reinterpret_cast<const uint32_t *>(entry + 8)[s + 1];
        const uint64_t at = (ent & ~15ull) - t.e_offset;            // offset inside the E-chunk region
        mode = static_cast<uint32_t>(ent & 15ull);
        if ((ent & ~15ull) < t.e_offset) {
            active = false;
        } else if (mode == ZM_MODE_CODED) {
            // a4: the stream's words, 128 bits per lane per load.  They are requested before the (larger)
            // sign-mantissa bytes because decoding can not start without them; the first 2 KiB (two
            // vectors per lane, more than a typical stream) wait in registers until the other requests
            // are out, longer streams are copied here.
            if (o1 < o0 || at + o1 > t.e_size) {
                active = false;
            } else {
                const uint32_t nvec = min((o1 - o0) >> 4, P.stream_cap_words >> 2);
                const uint4 *src = reinterpret_cast<const uint4 *>(t.echunks + at + o0);
                uint4 *dst = reinterpret_cast<uint4 *>(words);
                n_held = min(nvec, 128u);
                if (lane < n_held) held_a = src[lane];
                if (lane + 64 < n_held) held_b = src[lane + 64];
                for (uint32_t i = 128 + lane; i < nvec; i += 64) dst[i] = src[i];
            }
        } else {
            raw = t.echunks + at + static_cast<uint64_t>(s) * W;
            if (mode != ZM_MODE_RAW || at + static_cast<uint64_t>(s) * W + ((sn + 15u) & ~15u) > t.e_size) active = false;
        }
    }
    // Next in the request order: the sign-mantissa bytes of the first kGroup tiles.  They stay in flight
    // while the stream is staged and decoding starts.
    uint2 sm[kGroup];
    if (full) {
#pragma unroll
        for (int k = 0; k < kGroup; ++k) sm[k] = *reinterpret_cast<const uint2 *>(sm_base + k * kTile);
    } else {
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            sm[k] = make_uint2(0u, 0u);
            if (static_cast<uint32_t>(k) < tiles && mine - static_cast<int32_t>(k * kTile) > 0)
                sm[k] = *reinterpret_cast<const uint2 *>(sm_base + k * kTile);
        }
    }

    // a3: decode table -> LDS, split into a length table and a symbol table and replicated over the
    // index bits above the longest code.  Every wave of the workgroup writes the same bytes (LDS word
    // writes are atomic), so a wave may read as soon as its own writes are done: no workgroup barrier.
    {
        const uint16_t *src = reinterpret_cast<const uint16_t *>(t.lut);
        const uint32_t mask = (1u << t.max_len) - 1u;
        if (R == 4) {
            // 256 entries, four per lane, all loads issued before the first is used
            const uint32_t i = 4u * lane;
            const uint32_t a = src[i & mask], b = src[(i + 1) & mask], c = src[(i + 2) & mask], d = src[(i + 3) & mask];
            const uint32_t ab = a | (b << 16), cd = c | (d << 16);
            reinterpret_cast<uint32_t *>(sym_tab)[lane] = __builtin_amdgcn_perm(cd, ab, 0x06040200u);
            reinterpret_cast<uint32_t *>(len_tab)[lane] = __builtin_amdgcn_perm(cd, ab, 0x07050301u);
        } else {
            // 4096 entries; R = 2 implies max_len >= 9, so any 16 consecutive entries stay consecutive under the mask
            for (uint32_t i = 16u * lane; i < Code<R>::kEntries; i += 16u * 64u) {
                const uint4 *v = reinterpret_cast<const uint4 *>(src + (i & mask));
                const uint4 x = v[0], y = v[1];
                uint4 sy, le;
                sy.x = __builtin_amdgcn_perm(x.y, x.x, 0x06040200u); le.x = __builtin_amdgcn_perm(x.y, x.x, 0x07050301u);
                sy.y = __builtin_amdgcn_perm(x.w, x.z, 0x06040200u); le.y = __builtin_amdgcn_perm(x.w, x.z, 0x07050301u);
                sy.z = __builtin_amdgcn_perm(y.y, y.x, 0x06040200u); le.z = __builtin_amdgcn_perm(y.y, y.x, 0x07050301u);
                sy.w = __builtin_amdgcn_perm(y.w, y.z, 0x06040200u); le.w = __builtin_amdgcn_perm(y.w, y.z, 0x07050301u);
                *reinterpret_cast<uint4 *>(sym_tab + i) = sy;
                *reinterpret_cast<uint4 *>(len_tab + i) = le;
            }
        }
    }

    if (n_held) {
        uint4 *dst = reinterpret_cast<uint4 *>(words);
        if (lane < n_held) dst[lane] = held_a;
        if (lane + 64 < n_held) dst[lane + 64] = held_b;
    }
    // LDS written by some lanes of this wave is read by others: order the LDS accesses only
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
    if (!active) return;

    uint16_t *out_base = t.out + v0 + lane * 8u;

    Decoder<R> dec;
    dec.words = words; dec.last_word = P.stream_cap_words - 1u;
    if (mode == ZM_MODE_CODED) {
        const uint2 first = reinterpret_cast<const uint2 *>(words)[lane];
        dec.lo = first.x; dec.hi = first.y;
    }

    // Common case, straight-line: a coded stream of whole groups of kGroup tiles (one group at the default
    // stream length).  The first group's loads were issued above; from here on the wave only computes and
    // stores, and asks for the next group's sign-mantissa bytes when a group is done.
    if (mode == ZM_MODE_CODED && full) {
        const uint32_t groups = sn / (kGroup * kTile);
        for (uint32_t gi = 0;;) {
#pragma unroll
            for (int k = 0; k < kGroup; ++k)
                recover_and_store<kStreaming>(out_base + (gi * kGroup + k) * kTile, dec.tile(len_tab, sym_tab), sm[k]);
            if (++gi == groups) break;
            // longer streams: the next eight tiles' sign-mantissa bytes
#pragma unroll
            for (int k = 0; k < kGroup; ++k) sm[k] = *reinterpret_cast<const uint2 *>(sm_base + (gi * kGroup + k) * kTile);
        }
        return;
    }

    // General case: raw chunks, short last streams, streams that are not whole groups of kGroup tiles.
    for (uint32_t g0 = 0; g0 < tiles; g0 += kGroup) {
        if (g0) {
#pragma unroll
            for (int k = 0; k < kGroup; ++k) {
                sm[k] = make_uint2(0u, 0u);
                if (g0 + k < tiles && mine - static_cast<int32_t>((g0 + k) * kTile) > 0)
                    sm[k] = *reinterpret_cast<const uint2 *>(sm_base + (g0 + k) * kTile);
            }
        }
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            const uint32_t tile = g0 + k;
            if (tile < tiles) {
                const int32_t left = mine - static_cast<int32_t>(tile * kTile);
                uint2 ev = make_uint2(0u, 0u);
                if (mode == ZM_MODE_CODED) ev = dec.tile(len_tab, sym_tab);
                else if (left > 0) ev = *reinterpret_cast<const uint2 *>(raw + tile * kTile + lane * 8u);
                if (left >= 8) recover_and_store<kStreaming>(out_base + tile * kTile, ev, sm[k]);
                else if (left > 0) recover_and_store_partial(out_base + tile * kTile, ev, sm[k], left);
            }
        }
    }
}


// Stand-alone tensor recovery (Sec. 3.3): one tile of 512 values per wave; lane j merges values
// 8j..8j+7 -- a 64-bit load from each input, one 128-bit store, all contiguous across the wave.
constexpr int kRecoverTilesPerWave = 1;   // measured on 58.7 M-value tensors: 1 tile 68.9 %, 2: 68.3 %, 4: 67.4 %, 8: 65.7 % of 8 TB/s

__global__ void __launch_bounds__(256) zm_recover_kernel(const uint8_t *__restrict__ e, const uint8_t *__restrict__ sm,
                                                         uint16_t *__restrict__ out, uint64_t n)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = static_cast<uint64_t>(blockIdx.x) * 4u + (threadIdx.x >> 6);
    const uint64_t base = wave * (kRecoverTilesPerWave * kTile) + lane * 8u;
    uint2 ev[kRecoverTilesPerWave], sv[kRecoverTilesPerWave];
#pragma unroll
    for (int k = 0; k < kRecoverTilesPerWave; ++k) {
        const uint64_t i = base + static_cast<uint64_t>(k) * kTile;
        ev[k] = sv[k] = make_uint2(0u, 0u);
        if (i + 8 <= n) {
            ev[k] = *reinterpret_cast<const uint2 *>(e + i);
            sv[k] = *reinterpret_cast<const uint2 *>(sm + i);
        } else if (i < n) {                       // the tensor's last, partial group of eight
            uint32_t eb[2] = {0u, 0u}, sb[2] = {0u, 0u};
            for (uint32_t q = 0; q < n - i; ++q) {
                eb[q >> 2] |= static_cast<uint32_t>(e[i + q]) << (8 * (q & 3));
                sb[q >> 2] |= static_cast<uint32_t>(sm[i + q]) << (8 * (q & 3));
            }
            ev[k] = make_uint2(eb[0], eb[1]); sv[k] = make_uint2(sb[0], sb[1]);
        }
    }
#pragma unroll
    for (int k = 0; k < kRecoverTilesPerWave; ++k) {
        const uint64_t i = base + static_cast<uint64_t>(k) * kTile;
        if (i + 8 <= n) recover_and_store(out + i, ev[k], sv[k]);
        else if (i < n) recover_and_store_partial(out + i, ev[k], sv[k], static_cast<int32_t>(n - i));
    }
}

inline size_t stream_cap_words(uint32_t stream_values, uint32_t max_len_bound)
{
    const size_t syms = static_cast<size_t>(stream_values / kTile) * 8;
    const size_t words = 64 * (2 + (syms * max_len_bound + 31) / 32) + 4;
    return (words + 3) & ~static_cast<size_t>(3);
}

constexpr size_t kLdsLimit = 64 * 1024;
constexpr uint64_t kLastLevelCacheBytes = 256ull << 20;   // MI355X Infinity Cache

template <int R, int kWaves>
int launch_tasks(Launch &L, size_t cap, hipStream_t stream)
{
    const size_t lds = 4 * kWaves * cap;                       // dynamic part: the streams
    if (lds + 2 * Code<R>::kEntries > kLdsLimit) {
        if constexpr (kWaves > 1) return launch_tasks<R, kWaves / 2>(L, cap, stream);
        else return ZM_E_ARG;                   // stream too long to stage in LDS
    }
    uint32_t blocks = 0;            // of the largest tensor; workgroups past a smaller tensor's end exit at once
    for (uint32_t k = 0; k < L.n_tasks; ++k) {
        const uint32_t b = (L.task[k].n_streams + kWaves - 1) / kWaves;
        blocks = b > blocks ? b : blocks;
    }
    if (!blocks) return ZM_OK;
    uint64_t out_bytes = 0;
    for (uint32_t k = 0; k < L.n_tasks; ++k) out_bytes += 2 * L.task[k].n_values;
    if (out_bytes > kLastLevelCacheBytes)
        hipLaunchKernelGGL((zm_decode_kernel<R, kWaves, true>), dim3(blocks, L.n_tasks), dim3(64 * kWaves), lds, stream, L);
    else
        hipLaunchKernelGGL((zm_decode_kernel<R, kWaves, false>), dim3(blocks, L.n_tasks), dim3(64 * kWaves), lds, stream, L);
    return hipGetLastError() == hipSuccess ? ZM_OK : ZM_E_HIP;
}

template <int R>
int launch_group(const Task *tasks, int n, hipStream_t stream)
{
    constexpr uint32_t kLenBound = R == 4 ? 8 : ZM_MAX_CODE_LEN;
    int done = 0;
    while (done < n) {
        Launch L{};
        uint32_t max_stream = 0;
        int k = 0;
        for (; k < kMaxTasks && done + k < n; ++k) {
            L.task[k] = tasks[done + k];
            max_stream = max_stream > L.task[k].stream_values ? max_stream : L.task[k].stream_values;
        }
        L.n_tasks = static_cast<uint32_t>(k);
        const size_t cap = stream_cap_words(max_stream, kLenBound);
        L.stream_cap_words = static_cast<uint32_t>(cap);
        // two streams per workgroup: measured on one MoE layer call of 118 MB, 1 / 2 / 4 / 8 waves per
        // workgroup reach 63.1 / 63.2 / 61.9 / 58.2 % of the HBM roofline (1.2 GB calls: 72.5 / 72.9 / 73.2 / 72.0 %).
        // With long codes a workgroup stages 8 KiB of tables, so four streams share them: 2 / 4 / 8 waves reach
        // 41.9 / 45.6 / 45.6 % on a 170 MB call and 52.2 / 53.8 / 52.9 % on 1.2 GB calls.
        const int rc = launch_tasks<R, R == 4 ? 2 : 4>(L, cap, stream);
        if (rc != ZM_OK) return rc;
        done += k;
    }
    return ZM_OK;
}



// Checks one tensor's description and appends its task to the group of its round length.
int add_task(const zm_tensor_parts &pt, const zm_tensor_info &ti, void *out, Task *t4, int &n4, Task *t2, int &n2)
{
    if (ti.n_values == 0) return ZM_OK;
    if (!pt.table || !pt.chunk_offsets || !pt.sm || !pt.echunks || !out) return ZM_E_ARG;
    if ((reinterpret_cast<uintptr_t>(pt.table) & 15) || (reinterpret_cast<uintptr_t>(pt.chunk_offsets) & 7) ||
        (reinterpret_cast<uintptr_t>(pt.sm) & 15) || (reinterpret_cast<uintptr_t>(pt.echunks) & 15) ||
        (reinterpret_cast<uintptr_t>(out) & 15)) return ZM_E_ARG;
    if (ti.stream_values == 0 || ti.stream_values % kTile || ti.chunk_values % ti.stream_values) return ZM_E_ARG;
    if (ti.max_len < 1 || ti.max_len > ZM_MAX_CODE_LEN) return ZM_E_ARG;
    if (ti.round_symbols != (ti.max_len <= 8 ? 4u : 2u)) return ZM_E_ARG;
    if (ti.e_offset > ti.blob_size || ti.sm_offset + ((ti.n_values + 255) & ~255ull) > ti.e_offset) return ZM_E_ARG;
    if (ti.table_stride != ((8u + 4u * (ti.chunk_values / ti.stream_values + 1u) + 7u) & ~7u)) return ZM_E_ARG;
    const uint64_t n_streams = (ti.n_values + ti.stream_values - 1) / ti.stream_values;
    if (n_streams > 0x7FFFFFFFull) return ZM_E_ARG;
    Task t;
    t.lut = static_cast<const uint8_t *>(pt.table);
    t.sm = static_cast<const uint8_t *>(pt.sm);
    t.echunks = static_cast<const uint8_t *>(pt.echunks);
    t.table = static_cast<const uint64_t *>(pt.chunk_offsets);
    t.out = static_cast<uint16_t *>(out);
    t.n_values = ti.n_values;
    t.e_offset = ti.e_offset;
    t.e_size = ti.blob_size - ti.e_offset;
    t.stream_values = ti.stream_values;
    t.streams_per_chunk = ti.chunk_values / ti.stream_values;
    t.n_streams = static_cast<uint32_t>(n_streams);
    t.max_len = ti.max_len;
    if (ti.round_symbols == 4) t4[n4++] = t; else t2[n2++] = t;
    return ZM_OK;
}

constexpr int kMaxTensorsPerCall = 256;

}  // namespace

extern "C" int zm_decode_tensors(const zm_tensor_parts *parts, const zm_tensor_info *infos, int n_tensors,
                                 void *const *out_bf16, void *stream)
{
    if (n_tensors == 0) return ZM_OK;
    if (!parts || !infos || !out_bf16 || n_tensors < 0 || n_tensors > kMaxTensorsPerCall) return ZM_E_ARG;
    Task t4[kMaxTensorsPerCall], t2[kMaxTensorsPerCall];
    int n4 = 0, n2 = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const int rc = add_task(parts[i], infos[i], out_bf16[i], t4, n4, t2, n2);
        if (rc != ZM_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int rc = launch_group<4>(t4, n4, s);
    if (rc != ZM_OK) return rc;
    return launch_group<2>(t2, n2, s);
}

extern "C" int zm_decode_experts(const void *const *blobs, const uint64_t *const *chunk_offsets,
                                 const zm_tensor_info *infos, int n_experts, int tensors_per_expert,
                                 const int32_t *expert_ids, int n_selected,
                                 void *const *out_bf16, void *stream)
{
    if (n_selected == 0) return ZM_OK;
    if (!blobs || !chunk_offsets || !infos || !expert_ids || !out_bf16) return ZM_E_ARG;
    if (n_experts <= 0 || tensors_per_expert <= 0 || n_selected < 0) return ZM_E_ARG;
    if (static_cast<long>(n_selected) * tensors_per_expert > kMaxTensorsPerCall) return ZM_E_ARG;
    Task t4[kMaxTensorsPerCall], t2[kMaxTensorsPerCall];
    int n4 = 0, n2 = 0;
    for (int j = 0; j < n_selected; ++j) {
        const int e = expert_ids[j];
        if (e < 0 || e >= n_experts) return ZM_E_ARG;
        for (int m = 0; m < tensors_per_expert; ++m) {
            const size_t src = static_cast<size_t>(e) * tensors_per_expert + m;
            const size_t dst = static_cast<size_t>(j) * tensors_per_expert + m;
            const zm_tensor_info &ti = infos[src];
            if (ti.n_values == 0) continue;
            if (!blobs[src]) return ZM_E_ARG;
            const uint8_t *blob = static_cast<const uint8_t *>(blobs[src]);
            const zm_tensor_parts pt{blob + ti.lut_offset, chunk_offsets[src], blob + ti.sm_offset, blob + ti.e_offset};
            const int rc = add_task(pt, ti, out_bf16[dst], t4, n4, t2, n2);
            if (rc != ZM_OK) return rc;
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int rc = launch_group<4>(t4, n4, s);
    if (rc != ZM_OK) return rc;
    return launch_group<2>(t2, n2, s);
}

extern "C" int zm_recover(const void *exponents, const void *sign_mantissa, size_t n_values, void *out_bf16, void *stream)
{
    if (n_values == 0) return ZM_OK;
    if (!exponents || !sign_mantissa || !out_bf16) return ZM_E_ARG;
    if ((reinterpret_cast<uintptr_t>(exponents) & 7) || (reinterpret_cast<uintptr_t>(sign_mantissa) & 7) ||
        (reinterpret_cast<uintptr_t>(out_bf16) & 15)) return ZM_E_ARG;
    const uint64_t per_block = 4ull * kRecoverTilesPerWave * kTile;
    const uint64_t blocks = (n_values + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFFull) return ZM_E_ARG;
    hipLaunchKernelGGL(zm_recover_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t *>(exponents), static_cast<const uint8_t *>(sign_mantissa),
                       static_cast<uint16_t *>(out_bf16), static_cast<uint64_t>(n_values));
    return hipGetLastError() == hipSuccess ? ZM_OK : ZM_E_HIP;
}
