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
//   1. one read of the chunk's table entry locates the stream; its bytes (64 lane-length bytes, then the 64
//      lane bitstreams back to back) are requested with 128-bit loads (a4) -- first, because decoding can not
//      start without them -- and go to LDS;
//   2. the sign-mantissa bytes of the stream's tiles are requested: all eight of a group with non-temporal
//      stores, the first four with ordinary stores (the others as tiles are finished);
//   3. the decode table's first 256 entries go to LDS (a3) as 16-bit entries, code length in the low byte and
//      symbol in the high byte, at a fixed LDS address, replicated to the full index width; longer codes
//      are resolved from the tensor's full table in device memory;
//   4. a wavefront prefix sum over the 64 lane-length bytes gives every lane the first and the last bit of
//      its own bitstream (a6): what varies from lane to lane is where its input lies, its output positions
//      are fixed;
//   5. lock-step decode (a5): a lane's bitstream holds the first half of its symbols from its first bit upwards
//      and the second half, last symbol first, from its last bit downwards, so every lane runs two independent
//      decode chains at once (the lookups of one overlap the latency of the other).  Per chain it keeps two
//      words of the bitstream, a bit position and the index of its next word; per round it extracts a 32-bit
//      window with one funnel shift (bit-reversed for the downward chain) and decodes R symbols by table
//      lookup; the next word is requested at the start of the round, so that a chain that crosses a word
//      boundary finds it there;
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
    uint32_t code;            // longest code length | lane quantum << 8
};

struct Launch {
    uint32_t n_tasks;
    uint32_t stream_cap_words;   // LDS words reserved per wave for its stream
    uint32_t pad[2];
    Task task[kMaxTasks];        // blockIdx.y selects the task
};
static_assert(sizeof(Launch) <= 4096, "kernel arguments must stay under 4 KiB");

constexpr uint32_t kLaneBytes = 64;   // a stream opens with one length byte per lane

// Exclusive prefix sum of x over the 64 lanes of the wave (a6), by data-parallel primitives: an inclusive
// scan inside each row of 16 lanes (shifts by 1, 2, 4, 8), then lane 15 of row 0 and 2 is added to the next
// row, then lane 31 to rows 2 and 3.  Lanes with no source keep the `old` operand, zero.
__device__ __forceinline__ uint32_t wave_exclusive_sum(uint32_t x)
{
    uint32_t v = x;
    v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v - x;
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

// kStreaming: the stores are marked non-temporal (the output is larger than the last-level cache, or the
// caller said that its buffers are not cache-resident); else they are ordinary stores, whose lines tend to
// stay cached for a consumer or for the next call that rewrites the same buffers.
template <bool kStreaming = false>
__device__ __forceinline__ void recover_and_store(uint16_t *dst, uint2 e, uint2 sm)
{
    uint4 w;
    recover4(e.x, sm.x, w.x, w.y);
    recover4(e.y, sm.y, w.z, w.w);
    if constexpr (kStreaming) {
        // four adjacent word stores that the compiler merges into one 128-bit non-temporal store; written as a
        // vector store the same code needs 11 more registers and loses two waves per SIMD
        uint32_t *p = reinterpret_cast<uint32_t *>(__builtin_assume_aligned(dst, 16));
        __builtin_nontemporal_store(w.x, p); __builtin_nontemporal_store(w.y, p + 1);
        __builtin_nontemporal_store(w.z, p + 2); __builtin_nontemporal_store(w.w, p + 3);
    } else {
        *reinterpret_cast<uint4 *>(dst) = w;
    }
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

constexpr uint32_t kTableEntries = 256;   // the LDS table resolves the first eight bits of a code
constexpr uint32_t kLongSlots = 16;       // eight-bit beginnings of longer codes that get a block of the second LDS table
constexpr uint32_t kLongFlag = 0x80u;     // set in the length byte of a first-table entry whose code has more than eight bits

// Lock-step decoder state of one lane (a5): two chains, one reading the lane's bitstream upwards from its
// first bit (the first half of the lane's symbols, in order), one reading it downwards from its last bit (the
// second half, last symbol first).
// R = 4: every code has at most 8 bits, four symbols per 32-bit window.  R = 2: codes of up to ZM_MAX_CODE_LEN
// bits, two symbols per window; the LDS table still resolves eight bits, and a lane that meets a longer code
// (its table entry carries a length above 8: no code of at most 8 bits begins with these bits) takes its entry
// from a second LDS table that holds, for each eight-bit beginning of longer codes, the 16 entries its further
// bits select -- or, when a tensor has more than kLongSlots such beginnings, from the tensor's full decode table in
// device memory.  Long codes are the rare ones by construction and sit together at the end of the code space.
template <int R>
struct Decoder {
    const uint32_t *words;        // the stream as staged in LDS (length bytes included)
    uint32_t last_word;           // highest index a read may use
    // upward chain: words q and q+1 of the bitstream, bits of lo already used (< 32 at the start of a round), index of word q+2
    uint32_t lo = 0, hi = 0, pos = 0, next = 0;
    // downward chain: dhi is the word that holds the bits just below the read position, of which its low dpos
    // bits (0..31) are still unread, dlo the word below it, dnext the index of the word below that
    uint32_t dlo = 0, dhi = 0, dpos = 0, dnext = 0;
    // R = 2 only: the LDS table of the codes longer than eight bits (kLongSlots blocks of 16 entries, one block per
    // eight-bit beginning that such codes share) and the bits it resolves beyond the first eight; 0 = the tensor has
    // more such beginnings than blocks, and long codes are looked up in device memory
    const uint16_t *sub = nullptr;
    uint32_t sub_bits = 0;

    // first_bit, end_bit: where this lane's bitstream starts and ends, counted from the first payload bit
    __device__ __forceinline__ void start(uint32_t first_bit, uint32_t end_bit)
    {
        const uint32_t q = kLaneBytes / 4 + (first_bit >> 5);
        pos = first_bit & 31u;
        lo = words[min(q, last_word)];
        hi = words[min(q + 1u, last_word)];
        next = q + 2u;
        const uint32_t w = min(kLaneBytes / 4 + (end_bit >> 5), last_word);     // >= 16, so the indices below stay >= 14
        dpos = end_bit & 31u;
        dhi = words[w];
        dlo = words[w - 1u];
        dnext = w - 2u;
    }

    // R = 2: the entry of a code longer than eight bits, whose first-table entry v carries kLongFlag.
    __device__ __forceinline__ uint32_t long_code(const uint16_t *full_table, uint32_t max_len, uint32_t win, uint32_t acc,
                                                  uint32_t v) const
    {
        if (sub_bits) {
            // the entry's high byte names the block of this beginning; the code's further bits index it
            const uint32_t more = __builtin_amdgcn_ubfe(win, acc + 8u, 4) & ((1u << sub_bits) - 1u);
            return sub[((v >> 8) & (kLongSlots - 1u)) * 16u + more];
        }
        const uint32_t full = full_table[(win >> (acc & 31u)) & ((1u << max_len) - 1u)];
        return __builtin_amdgcn_perm(0u, full, 0x0c0c0001u);      // symbol | length << 8  ->  length | symbol << 8
    }

    // One round: R symbols of each chain.  up / down receive the R entries in the order read.
    __device__ __forceinline__ void round(const uint16_t *tab, const uint16_t *full_table, uint32_t max_len,
                                          uint32_t (&up)[R], uint32_t (&down)[R])
    {
        // the words the chains take if the round crosses a word boundary: asked for now, used after the round
        const uint32_t fresh = words[min(next, last_word)];
        const uint32_t dfresh = words[min(dnext, last_word)];
        // R symbols out of one 32-bit window per chain.  acc sums the entries: its low byte is the bit offset of
        // the next code in the window (at most 32), the bytes above hold a sum of symbols that nothing reads.
        // The field extract takes the low five bits of acc as its offset; when they wrap (32 bits used) no
        // further code is extracted.  The downward window is reversed so that its next bit is bit 0 too.
        const uint32_t win = __builtin_amdgcn_alignbit(hi, lo, pos);
        const uint32_t dwin = __builtin_bitreverse32(__builtin_amdgcn_alignbit(dhi, dlo, dpos));
        uint32_t acc = 0, dacc = 0;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            // the entries (length | symbol << 8) of the codes that start at bit (acc & 31) of the two windows
            uint32_t v = tab[__builtin_amdgcn_ubfe(win, acc, 8)];
            uint32_t dv = tab[__builtin_amdgcn_ubfe(dwin, dacc, 8)];
            if constexpr (R == 2) {
                // both look-ups are out before either is tested: one branch per step, rarely taken
                if ((v | dv) & kLongFlag) {
                    if (v & kLongFlag) v = long_code(full_table, max_len, win, acc, v);
                    if (dv & kLongFlag) dv = long_code(full_table, max_len, dwin, dacc, dv);
                }
            }
            up[k] = v;
            down[k] = dv;
            acc += v;
            dacc += dv;
        }
        // written without branches so that (with short codes) a whole tile pair is one basic block
        pos += acc & 0xffu;
        const bool take = pos >= 32u;
        lo = take ? hi : lo;
        hi = take ? fresh : hi;
        next += take ? 1u : 0u;
        pos &= 31u;
        const int32_t left = static_cast<int32_t>(dpos) - static_cast<int32_t>(dacc & 0xffu);    // -32..31
        const bool dtake = left < 0;
        dhi = dtake ? dlo : dhi;
        dlo = dtake ? dfresh : dlo;
        dnext -= dtake ? 1u : 0u;
        dpos = static_cast<uint32_t>(left) & 31u;
    }

    // Four symbols of each chain: .x = the upward chain's, .y = the downward chain's, both packed in value order
    // (byte 0 = the symbol with the lowest index), i.e. half a tile's exponent bytes for this lane each.
    __device__ __forceinline__ uint2 quad(const uint16_t *tab, const uint16_t *full_table, uint32_t max_len)
    {
        // byte 1 (the symbol) of each entry, packed with byte permutes (0x0c selects a zero byte)
        if constexpr (R == 4) {
            uint32_t up[4], down[4];
            round(tab, full_table, max_len, up, down);
            const uint32_t u01 = __builtin_amdgcn_perm(up[1], up[0], 0x0c0c0501u), u23 = __builtin_amdgcn_perm(up[3], up[2], 0x0c0c0501u);
            const uint32_t d01 = __builtin_amdgcn_perm(down[2], down[3], 0x0c0c0501u), d23 = __builtin_amdgcn_perm(down[0], down[1], 0x0c0c0501u);
            return make_uint2(__builtin_amdgcn_perm(u23, u01, 0x05040100u), __builtin_amdgcn_perm(d23, d01, 0x05040100u));
        } else {
            uint32_t ua[2], da[2], ub[2], db[2];
            round(tab, full_table, max_len, ua, da);
            round(tab, full_table, max_len, ub, db);
            const uint32_t u01 = __builtin_amdgcn_perm(ua[1], ua[0], 0x0c0c0501u), u23 = __builtin_amdgcn_perm(ub[1], ub[0], 0x0c0c0501u);
            const uint32_t d01 = __builtin_amdgcn_perm(db[0], db[1], 0x0c0c0501u), d23 = __builtin_amdgcn_perm(da[0], da[1], 0x0c0c0501u);
            return make_uint2(__builtin_amdgcn_perm(u23, u01, 0x05040100u), __builtin_amdgcn_perm(d23, d01, 0x05040100u));
        }
    }
};

// R: symbols per round; kWaves: waves (streams) per workgroup; kStreaming: non-temporal stores
template <int R, int kWaves, bool kStreaming>
__global__ void __launch_bounds__(64 * kWaves) zm_decode_kernel(const Launch P)
{
    // The decode table of the workgroup's tensor for the first eight bits of a code, at a fixed LDS address:
    // one 16-bit read gives a code's length and its symbol.  (Two byte tables, one read each, were 2-4 % slower:
    // twice the LDS instructions, whose random accesses collide on banks.)
    __shared__ __align__(16) uint16_t tab[kTableEntries];
    // second table for codes longer than eight bits (R = 2): kLongSlots blocks of 16 entries, and the eight-bit
    // beginning each block belongs to
    __shared__ __align__(16) uint16_t sub[R == 2 ? kLongSlots * 16 : 4];
    __shared__ uint16_t long_prefix[R == 2 ? kLongSlots : 2];
    extern __shared__ __align__(16) uint32_t stream_lds[];

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // grid: x = workgroup inside the tensor, y = tensor.  The task is copied with one batch of scalar loads.
    const Task t = P.task[blockIdx.y];
    uint32_t *words = stream_lds + wave * P.stream_cap_words;
    const uint32_t W = t.stream_values;
    const uint32_t max_len = t.code & 0xffu, quantum = t.code >> 8;
    const uint32_t stride = (8u + 4u * (t.streams_per_chunk + 1u) + 7u) & ~7u;     // bytes of a chunk-table entry

    const uint32_t g = blockIdx.x * kWaves + wave;
    bool active = g < t.n_streams;
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
        const uint8_t *entry = reinterpret_cast<const uint8_t *>(t.table) + static_cast<uint64_t>(c) * stride;
        const uint64_t ent = *reinterpret_cast<const uint64_t *>(entry);
        const uint32_t o0 = reinterpret_cast<const uint32_t *>(entry + 8)[s];
        const uint32_t o1 = reinterpret_cast<const uint32_t *>(entry + 8)[s + 1];
        const uint64_t at = (ent & ~15ull) - t.e_offset;            // offset inside the E-chunk region
        mode = static_cast<uint32_t>(ent & 15ull);
        if ((ent & ~15ull) < t.e_offset) {
            active = false;
        } else if (mode == ZM_MODE_CODED) {
            // a4: the stream's bytes, 128 bits per lane per load.  They are requested before the (larger)
            // sign-mantissa bytes because decoding can not start without them; the first 2 KiB (two
            // vectors per lane, more than a typical stream) wait in registers until the other requests
            // are out, longer streams are copied here.
            if (o1 < o0 + kLaneBytes || at + o1 > t.e_size) {
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
    // Next in the request order: the sign-mantissa bytes of the first tiles.  They stay in flight while the
    // stream is staged and decoding starts.  A straight-line stream is decoded from both ends: pair i is tile i
    // (upward chain) and tile 7 - i of the group (downward chain); up[i] / down[i] hold their bytes.
    // With ordinary stores the first kAhead pairs are asked for here and pair i + kAhead when pair i is done:
    // the requests of the thousands of waves that start together are spread out and everyone's first tiles
    // arrive sooner.  A wave waits for such a later load behind its own earlier stores, though, and non-temporal
    // stores take long to be acknowledged: with them all eight tiles are asked for up front.  So they are with
    // long codes, whose look-ups in device memory would wait behind the later requests as well.
    constexpr int kPairs = kGroup / 2;
    constexpr int kAhead = (kStreaming || R == 2) ? kPairs : 2;
    const bool straight = full && mode == ZM_MODE_CODED;
    uint2 up[kPairs], down[kPairs];
    if (straight) {
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            up[i] = *reinterpret_cast<const uint2 *>(sm_base + i * kTile);
            down[i] = *reinterpret_cast<const uint2 *>(sm_base + (tiles - 1u - i) * kTile);
        }
    }

    // a3: decode table -> LDS, its first 256 entries with the two bytes of an entry swapped (length low),
    // replicated over the index bits above the longest code.  Four entries per lane, all loads issued before the
    // first is used.  Every wave of the workgroup writes the same bytes (LDS word writes are atomic), so a wave may
    // read as soon as its own writes are done: no workgroup barrier.
    uint32_t sub_bits = 0;
    {
        const uint16_t *src = reinterpret_cast<const uint16_t *>(t.lut);
        const uint32_t mask = (1u << max_len) - 1u;
        const uint32_t i = 4u * lane;
        uint32_t a = src[i & mask], b = src[(i + 1) & mask], c = src[(i + 2) & mask], d = src[(i + 3) & mask];
        if constexpr (R == 2) {
            // Entries with a length above eight mark the eight-bit beginnings of longer codes.  They are numbered in
            // index order; if there are at most kLongSlots of them, entry number s gets block s of the second table
            // (its symbol byte is replaced by s) and the block is filled with the 2^(max_len - 8) entries of the
            // full table that share these eight bits.
            const uint32_t la = (a >> 8) > 8u, lb = (b >> 8) > 8u, lc = (c >> 8) > 8u, ld = (d >> 8) > 8u;
            const uint64_t ma = __builtin_amdgcn_ballot_w64(la), mb = __builtin_amdgcn_ballot_w64(lb),
                           mc = __builtin_amdgcn_ballot_w64(lc), md = __builtin_amdgcn_ballot_w64(ld);
            const uint32_t n_long = __builtin_popcountll(ma) + __builtin_popcountll(mb) + __builtin_popcountll(mc) + __builtin_popcountll(md);
            // every such entry is flagged in its length byte (lengths stay below 16)
            a |= la ? kLongFlag << 8 : 0u; b |= lb ? kLongFlag << 8 : 0u; c |= lc ? kLongFlag << 8 : 0u; d |= ld ? kLongFlag << 8 : 0u;
            if (n_long != 0 && n_long <= kLongSlots && max_len > 8u) {
                const uint64_t below = (1ull << lane) - 1ull;
                const uint32_t sa = __builtin_popcountll(ma & below) + __builtin_popcountll(mb & below) +
                                    __builtin_popcountll(mc & below) + __builtin_popcountll(md & below);
                const uint32_t sb = sa + la, sc = sb + lb, sd = sc + lc;
                if (la) { long_prefix[sa] = static_cast<uint16_t>(i); a = (a & 0xff00u) | sa; }
                if (lb) { long_prefix[sb] = static_cast<uint16_t>(i + 1u); b = (b & 0xff00u) | sb; }
                if (lc) { long_prefix[sc] = static_cast<uint16_t>(i + 2u); c = (c & 0xff00u) | sc; }
                if (ld) { long_prefix[sd] = static_cast<uint16_t>(i + 3u); d = (d & 0xff00u) | sd; }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
                sub_bits = max_len - 8u;
                // lane l fills entries 4l..4l+3 of the second table: block (4l)/16, further bits (4l)%16 + 0..3
                const uint32_t block = lane >> 2, first = (lane & 3u) * 4u;
                uint32_t e[4];
#pragma unroll
                for (uint32_t j = 0; j < 4; ++j) {
                    const uint32_t more = first + j;
                    e[j] = 0u;
                    if (block < n_long && more < (1u << sub_bits))
                        e[j] = src[(static_cast<uint32_t>(long_prefix[block]) + (more << 8)) & mask];
                }
                const uint32_t e01 = e[0] | (e[1] << 16), e23 = e[2] | (e[3] << 16);
                reinterpret_cast<uint2 *>(sub)[lane] = make_uint2(__builtin_amdgcn_perm(e01, e01, 0x02030001u), __builtin_amdgcn_perm(e23, e23, 0x02030001u));
            }
        }
        const uint32_t ab = a | (b << 16), cd = c | (d << 16);
        reinterpret_cast<uint2 *>(tab)[lane] = make_uint2(__builtin_amdgcn_perm(ab, ab, 0x02030001u), __builtin_amdgcn_perm(cd, cd, 0x02030001u));
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

    const uint16_t *full_table = reinterpret_cast<const uint16_t *>(t.lut);
    Decoder<R> dec;
    dec.words = words; dec.last_word = P.stream_cap_words - 1u;
    dec.sub = sub; dec.sub_bits = sub_bits;
    if (mode == ZM_MODE_CODED) {
        // a6: this lane's bitstream has 8 * tiles + quantum * (its length byte) bits and starts where
        // the bitstreams of the lanes below it end
        const uint32_t units = reinterpret_cast<const uint8_t *>(words)[lane];
        const uint32_t bits = 8u * tiles + quantum * units;
        const uint32_t first = wave_exclusive_sum(bits);
        dec.start(first, first + bits);
    }

    if (straight) {
        // Common case, straight-line: a coded stream of whole groups of kGroup tiles (one group at the
        // default stream length).  Group number q is the tiles 4q..4q+3 (upward chain) and, from the other
        // end, tiles - 1 - 4q down to tiles - 4 - 4q (downward chain).  The first group's loads were issued
        // above; from here on the wave only computes and stores, and asks for the next group's sign-mantissa
        // bytes when a group is done.
        const uint32_t groups = tiles / kGroup;
        for (uint32_t q = 0;;) {
            const uint32_t lo_tile = q * kPairs, hi_tile = tiles - 1u - q * kPairs;
#pragma unroll
            for (int i = 0; i < kPairs; ++i) {
                // a tile's eight symbols come in two quads: the upward chain gives values 0..3 first, the
                // downward chain values 4..7 first
                const uint2 a = dec.quad(tab, full_table, max_len), b = dec.quad(tab, full_table, max_len);
                recover_and_store<kStreaming>(out_base + (lo_tile + i) * kTile, make_uint2(a.x, b.x), up[i]);
                recover_and_store<kStreaming>(out_base + (hi_tile - i) * kTile, make_uint2(b.y, a.y), down[i]);
                if (q == 0 && i + kAhead < kPairs) {
                    up[i + kAhead] = *reinterpret_cast<const uint2 *>(sm_base + (i + kAhead) * kTile);
                    down[i + kAhead] = *reinterpret_cast<const uint2 *>(sm_base + (tiles - 1u - (i + kAhead)) * kTile);
                }
            }
            if (++q == groups) break;
#pragma unroll
            for (int i = 0; i < kPairs; ++i) {
                up[i] = *reinterpret_cast<const uint2 *>(sm_base + (q * kPairs + i) * kTile);
                down[i] = *reinterpret_cast<const uint2 *>(sm_base + (tiles - 1u - q * kPairs - i) * kTile);
            }
        }
    } else {
        // General case: raw chunks, short last streams, streams that are not whole groups of kGroup tiles.
        // Pair p is tile p and tile tiles - 1 - p; with an odd number of tiles the last pair is the middle
        // tile alone, whose low half comes from the upward and whose high half from the downward chain.
        auto load_sm = [&](uint32_t tile) {
            return mine - static_cast<int32_t>(tile * kTile) > 0 ? *reinterpret_cast<const uint2 *>(sm_base + tile * kTile)
                                                                   : make_uint2(0u, 0u);
        };
        auto finish = [&](uint32_t tile, uint2 ev, uint2 smv) {
            const int32_t left = mine - static_cast<int32_t>(tile * kTile);
            if (mode != ZM_MODE_CODED) ev = left > 0 ? *reinterpret_cast<const uint2 *>(raw + tile * kTile + lane * 8u) : make_uint2(0u, 0u);
            if (left >= 8) recover_and_store<kStreaming>(out_base + tile * kTile, ev, smv);
            else if (left > 0) recover_and_store_partial(out_base + tile * kTile, ev, smv, left);
        };
        for (uint32_t p = 0; 2u * p < tiles; ++p) {
            const uint32_t lo_tile = p, hi_tile = tiles - 1u - p;
            const uint2 sm_lo = load_sm(lo_tile), sm_hi = load_sm(hi_tile);
            uint2 a = make_uint2(0u, 0u), b = a;
            if (mode == ZM_MODE_CODED) {
                a = dec.quad(tab, full_table, max_len);
                if (lo_tile != hi_tile) b = dec.quad(tab, full_table, max_len);
            }
            if (lo_tile != hi_tile) {
                finish(lo_tile, make_uint2(a.x, b.x), sm_lo);
                finish(hi_tile, make_uint2(b.y, a.y), sm_hi);
            } else {
                finish(lo_tile, make_uint2(a.x, a.y), sm_lo);
            }
        }
    }
}


// Stand-alone tensor recovery (Sec. 3.3): one tile of 512 values per wave; lane j merges values
// 8j..8j+7 -- a 64-bit load from each input, one 128-bit store, all contiguous across the wave.
constexpr int kRecoverTilesPerWave = 1;   // measured on 58.7 M-value tensors: 1 tile 68.9 %, 2: 68.3 %, 4: 67.4 %, 8: 65.7 % of 8 TB/s

template <bool kStreaming>
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
        if (i + 8 <= n) recover_and_store<kStreaming>(out + i, ev[k], sv[k]);
        else if (i < n) recover_and_store_partial(out + i, ev[k], sv[k], static_cast<int32_t>(n - i));
    }
}

// LDS words a wave reserves for one stream of the launch's longest kind: the length bytes, the code bits
// of a lane bounded by the longest code, the rounding of every lane to the quantum, the padding to 16 bytes,
// and two words a lane may read past its last one.
inline size_t stream_cap_words(uint32_t stream_values, uint32_t max_len_bound, uint32_t quantum)
{
    const size_t syms = static_cast<size_t>(stream_values / kTile) * 8;
    const size_t bytes = kLaneBytes + (64 * (syms * max_len_bound + quantum) + 7) / 8 + 16 + 8;
    return ((bytes + 15) & ~static_cast<size_t>(15)) / 4;
}

constexpr size_t kLdsLimit = 64 * 1024;
// LDS a workgroup holds beside its streams: the first table, and with long codes the second one and its index
template <int R>
constexpr size_t kStaticLds = 2 * kTableEntries + (R == 2 ? 2 * kLongSlots * 16 + 2 * kLongSlots : 0);
constexpr uint64_t kLastLevelCacheBytes = 256ull << 20;   // MI355X Infinity Cache

template <int R, int kWaves, bool kStreaming>
int launch_kernel(const Launch &L, uint32_t blocks, size_t lds, hipStream_t stream)
{
    void *args[] = {const_cast<Launch *>(&L)};
    const void *fn = reinterpret_cast<const void *>(&zm_decode_kernel<R, kWaves, kStreaming>);
    // the launch's own status: an error left behind by an earlier, unrelated call is not this call's
    return hipLaunchKernel(fn, dim3(blocks, L.n_tasks), dim3(64 * kWaves), args, lds, stream) == hipSuccess ? ZM_OK : ZM_E_HIP;
}

// Where the shapes of a call's launches go when they are asked for instead of launched.
struct Recorder {
    zm_launch_shape *out;
    int cap;
    int n = 0;
};

template <int R, int kWaves>
int launch_tasks(Launch &L, size_t cap, int stores, hipStream_t stream, Recorder *rec)
{
    const size_t lds = 4 * kWaves * cap;                       // dynamic part: the streams
    if (lds + kStaticLds<R> > kLdsLimit) {
        if constexpr (kWaves > 1) return launch_tasks<R, kWaves / 2>(L, cap, stores, stream, rec);
        else return ZM_E_ARG;                   // stream too long to stage in LDS
    }
    uint32_t blocks = 0;            // of the largest tensor; workgroups past a smaller tensor's end exit at once
    uint64_t out_bytes = 0;
    for (uint32_t k = 0; k < L.n_tasks; ++k) {
        const uint32_t b = (L.task[k].n_streams + kWaves - 1) / kWaves;
        blocks = b > blocks ? b : blocks;
        out_bytes += 2 * L.task[k].n_values;
    }
    if (!blocks) return ZM_OK;
    const bool streaming = stores == ZM_STORES_STREAMING || (stores == ZM_STORES_AUTO && out_bytes > kLastLevelCacheBytes);
    if (rec) {
        if (rec->n < rec->cap)
            rec->out[rec->n] = zm_launch_shape{static_cast<uint32_t>(R), static_cast<uint32_t>(kWaves), streaming ? 1u : 0u, blocks,
                                               L.n_tasks, static_cast<uint32_t>(lds + kStaticLds<R>)};
        ++rec->n;
        return ZM_OK;
    }
    return streaming ? launch_kernel<R, kWaves, true>(L, blocks, lds, stream) : launch_kernel<R, kWaves, false>(L, blocks, lds, stream);
}

// Collects the tensors of one round length and launches them, at most kMaxTasks per launch.
template <int R>
struct Group {
    static constexpr uint32_t kLenBound = R == 4 ? 8 : ZM_MAX_CODE_LEN;
    Launch L{};
    uint32_t max_stream = 0, max_quantum = 1;
    int stores;
    hipStream_t stream;
    Recorder *rec;

    Group(int store_policy, hipStream_t s, Recorder *r) : stores(store_policy), stream(s), rec(r) {}

    int add(const Task &t)
    {
        L.task[L.n_tasks++] = t;
        max_stream = max_stream > t.stream_values ? max_stream : t.stream_values;
        max_quantum = max_quantum > (t.code >> 8) ? max_quantum : (t.code >> 8);
        return L.n_tasks == kMaxTasks ? flush() : ZM_OK;
    }

    int flush()
    {
        if (!L.n_tasks) return ZM_OK;
        const size_t cap = stream_cap_words(max_stream, kLenBound, max_quantum);
        L.stream_cap_words = static_cast<uint32_t>(cap);
        // two streams per workgroup: on one MoE layer call of 118 MB one, two and four waves per workgroup are
        // within 1 % of each other, eight are 5 % slower
        const int rc = launch_tasks<R, 2>(L, cap, stores, stream, rec);
        L.n_tasks = 0; max_stream = 0; max_quantum = 1;
        return rc;
    }
};

// Checks one tensor's description and fills its task.  skip: the tensor is empty.
int make_task(const zm_tensor_parts &pt, const zm_tensor_info &ti, void *out, Task &t, bool &skip)
{
    skip = ti.n_values == 0;
    if (skip) return ZM_OK;
    if (!pt.table || !pt.chunk_offsets || !pt.sm || !pt.echunks || !out) return ZM_E_ARG;
    if ((reinterpret_cast<uintptr_t>(pt.table) & 15) || (reinterpret_cast<uintptr_t>(pt.chunk_offsets) & 7) ||
        (reinterpret_cast<uintptr_t>(pt.sm) & 15) || (reinterpret_cast<uintptr_t>(pt.echunks) & 15) ||
        (reinterpret_cast<uintptr_t>(out) & 15)) return ZM_E_ARG;
    if (ti.stream_values == 0 || ti.stream_values % kTile || ti.chunk_values % ti.stream_values) return ZM_E_ARG;
    if (ti.max_len < 1 || ti.max_len > ZM_MAX_CODE_LEN) return ZM_E_ARG;
    const uint32_t span = (ti.max_len - 1) * (ti.stream_values / 64);
    if (ti.lane_quantum != (span + 254) / 255 + (span == 0)) return ZM_E_ARG;
    if (ti.e_offset > ti.blob_size || ti.sm_offset + ((ti.n_values + 255) & ~255ull) > ti.e_offset) return ZM_E_ARG;
    if (ti.table_stride != ((8u + 4u * (ti.chunk_values / ti.stream_values + 1u) + 7u) & ~7u)) return ZM_E_ARG;
    const uint64_t n_streams = (ti.n_values + ti.stream_values - 1) / ti.stream_values;
    if (n_streams > 0x7FFFFFFFull) return ZM_E_ARG;
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
    t.code = ti.max_len | ti.lane_quantum << 8;
    return ZM_OK;
}

constexpr int kMaxTensorsPerCall = 256;

// Tensor i of a call, as make_task wants it; implemented by the two entry points.
template <typename Describe>
int decode_call(int n_tensors, Describe describe, int stores, hipStream_t stream, Recorder *rec = nullptr)
{
    if (stores != ZM_STORES_AUTO && stores != ZM_STORES_CACHED && stores != ZM_STORES_STREAMING) return ZM_E_ARG;
    // first pass: every tensor is checked before anything is launched
    for (int i = 0; i < n_tensors; ++i) {
        Task t; bool skip;
        const int rc = describe(i, t, skip);
        if (rc != ZM_OK) return rc;
    }
    Group<4> short_codes(stores, stream, rec);
    Group<2> long_codes(stores, stream, rec);
    for (int i = 0; i < n_tensors; ++i) {
        Task t; bool skip;
        describe(i, t, skip);
        if (skip) continue;
        const int rc = (t.code & 0xffu) <= 8 ? short_codes.add(t) : long_codes.add(t);
        if (rc != ZM_OK) return rc;
    }
    const int rc = short_codes.flush();
    return rc != ZM_OK ? rc : long_codes.flush();
}

}  // namespace

extern "C" int zm_decode_tensors(const zm_tensor_parts *parts, const zm_tensor_info *infos, int n_tensors,
                                 void *const *out_bf16, void *stream)
{
    if (n_tensors == 0) return ZM_OK;
    if (!parts || !infos || !out_bf16 || n_tensors < 0 || n_tensors > kMaxTensorsPerCall) return ZM_E_ARG;
    return decode_call(n_tensors, [&](int i, Task &t, bool &skip) { return make_task(parts[i], infos[i], out_bf16[i], t, skip); },
                       ZM_STORES_AUTO, static_cast<hipStream_t>(stream));
}

extern "C" int zm_decode_launch_shapes(const zm_tensor_info *infos, int n_tensors, int stores,
                                       zm_launch_shape *shapes_out, int shapes_cap, int *n_shapes)
{
    if (!infos || n_tensors < 0 || n_tensors > kMaxTensorsPerCall || shapes_cap < 0 || (shapes_cap && !shapes_out) || !n_shapes) return ZM_E_ARG;
    // the same path as a decode call, with placeholder addresses and a recorder in place of the launches
    uint8_t *const somewhere = reinterpret_cast<uint8_t *>(uintptr_t{4096});
    const zm_tensor_parts pt{somewhere, somewhere, somewhere, somewhere};
    Recorder rec{shapes_out, shapes_cap};
    const int rc = decode_call(n_tensors, [&](int i, Task &t, bool &skip) { return make_task(pt, infos[i], somewhere, t, skip); },
                               stores, nullptr, &rec);
    *n_shapes = rec.n;
    return rc;
}

extern "C" int zm_decode_experts_stores(const void *const *blobs, const uint64_t *const *chunk_offsets,
                                        const zm_tensor_info *infos, int n_experts, int tensors_per_expert,
                                        const int32_t *expert_ids, int n_selected,
                                        void *const *out_bf16, int stores, void *stream)
{
    if (n_selected == 0) return ZM_OK;
    if (!blobs || !chunk_offsets || !infos || !expert_ids || !out_bf16) return ZM_E_ARG;
    if (n_experts <= 0 || tensors_per_expert <= 0 || n_selected < 0) return ZM_E_ARG;
    if (static_cast<long>(n_selected) * tensors_per_expert > kMaxTensorsPerCall) return ZM_E_ARG;
    for (int j = 0; j < n_selected; ++j)
        if (expert_ids[j] < 0 || expert_ids[j] >= n_experts) return ZM_E_ARG;
    auto describe = [&](int i, Task &t, bool &skip) {
        const int j = i / tensors_per_expert, m = i % tensors_per_expert;
        const size_t src = static_cast<size_t>(expert_ids[j]) * tensors_per_expert + m;
        const zm_tensor_info &ti = infos[src];
        skip = ti.n_values == 0;
        if (skip) return ZM_OK;
        if (!blobs[src]) return ZM_E_ARG;
        const uint8_t *blob = static_cast<const uint8_t *>(blobs[src]);
        const zm_tensor_parts pt{blob + ti.lut_offset, chunk_offsets[src], blob + ti.sm_offset, blob + ti.e_offset};
        return make_task(pt, ti, out_bf16[i], t, skip);
    };
    return decode_call(n_selected * tensors_per_expert, describe, stores, static_cast<hipStream_t>(stream));
}

extern "C" int zm_decode_experts(const void *const *blobs, const uint64_t *const *chunk_offsets,
                                 const zm_tensor_info *infos, int n_experts, int tensors_per_expert,
                                 const int32_t *expert_ids, int n_selected,
                                 void *const *out_bf16, void *stream)
{
    return zm_decode_experts_stores(blobs, chunk_offsets, infos, n_experts, tensors_per_expert, expert_ids, n_selected,
                                    out_bf16, ZM_STORES_AUTO, stream);
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
    const uint8_t *e = static_cast<const uint8_t *>(exponents), *sm = static_cast<const uint8_t *>(sign_mantissa);
    uint16_t *out = static_cast<uint16_t *>(out_bf16);
    uint64_t n = n_values;
    void *args[] = {&e, &sm, &out, &n};
    // A launch that moves more than half of the last-level cache (four bytes per value) writes with non-temporal
    // stores: measured on 58.7 M-value tensors 71.6 against 68.9 % of the HBM roofline; on 2.9 M-value tensors,
    // whose buffers stay cached between calls, ordinary stores are the faster ones (43.3 against 40.4 %).
    const void *fn = 4 * n > kLastLevelCacheBytes / 2 ? reinterpret_cast<const void *>(&zm_recover_kernel<true>)
                                                  : reinterpret_cast<const void *>(&zm_recover_kernel<false>);
    return hipLaunchKernel(fn, dim3(static_cast<uint32_t>(blocks)), dim3(256),
                           args, 0, static_cast<hipStream_t>(stream)) == hipSuccess ? ZM_OK : ZM_E_HIP;
}
