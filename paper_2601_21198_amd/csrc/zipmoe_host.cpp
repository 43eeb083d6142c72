// Host side of libzipmoe: codebook construction, encoder, blob inspection.
//
// Follows ZipMoE (arXiv 2601.21198) Sec. 3.1, offline initialisation: bit-field
// decomposition of bf16 words (fields as in Sec. 2.2), sharding of the exponent
// bytes into independently coded E-chunks, byte-packed sign-mantissa section,
// serialisation with metadata.  The E-chunk backend (Sec. 6, "Other
// Compressors") is a canonical length-limited prefix code; the layout of the
// serialised tensor is described in include/zipmoe.h.
#include "zipmoe.h"

#include <algorithm>
#include <array>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <new>
#include <thread>
#include <vector>

namespace {

constexpr uint32_t kMagic = 0x454F4D5Au;   // "ZMOE"
constexpr uint32_t kVersion = 4;
constexpr uint32_t kHeaderBytes = 128;
constexpr uint32_t kLanes = 64;
constexpr uint32_t kRun = 8;               // consecutive values per lane per tile
constexpr uint32_t kTile = kLanes * kRun;  // 512

// header field positions
struct Hdr {
    static constexpr size_t magic = 0, version = 4, n_values = 8, chunk = 16, stream = 20, n_chunks = 24,
                            max_len = 28, quantum = 32, n_present = 36, pad_sym = 40, table_stride = 44, len_off = 48,
                            lut_off = 56, table_off = 64, sm_off = 72, e_off = 80, blob_size = 88;
};

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) & ~(a - 1); }

template <typename T> inline void store_le(uint8_t *p, T v) { std::memcpy(p, &v, sizeof(T)); }   // x86-64 host: little-endian
template <typename T> inline T load_le(const uint8_t *p) { T v; std::memcpy(&v, p, sizeof(T)); return v; }

inline bool geometry_ok(uint32_t chunk_values, uint32_t stream_values)
{
    return stream_values != 0 && chunk_values != 0 && stream_values % kTile == 0 && chunk_values % stream_values == 0;
}

// bytes of one chunk-table entry: the 64-bit offset|mode word and the offsets of the chunk's streams plus its length
inline uint32_t table_stride_for(uint32_t chunk_values, uint32_t stream_values)
{
    return static_cast<uint32_t>(align_up(8 + 4ull * (chunk_values / stream_values + 1), 8));
}

// Unit of the per-lane length bytes: the smallest q >= 1 for which (L - 1) * (W / 64) <= 255 * q, so that
// the byte of a lane whose every code has the longest length still fits.
inline uint32_t lane_quantum_for(uint32_t max_len, uint32_t stream_values)
{
    const uint32_t span = (max_len - 1) * (stream_values / kLanes);
    return std::max(1u, (span + 254) / 255);
}

// Canonical code table derived from code lengths.
struct Book {
    uint8_t len[256];
    uint16_t wire[256];   // code with its first wire bit in bit 0 (ready for LSB-first packing)
    uint16_t canon[256];  // the same code with its first wire bit in its top bit (the canonical code value)
    uint32_t max_len = 1;
    uint32_t n_present = 0;
    uint32_t pad = 0;
    uint32_t kraft = 0;   // in units of 2^-ZM_MAX_CODE_LEN
};

bool make_book(const uint8_t code_len[256], Book &b)
{
    uint32_t count[ZM_MAX_CODE_LEN + 2] = {0};
    b.n_present = 0; b.kraft = 0; b.max_len = 1; b.pad = 0;
    for (int s = 0; s < 256; ++s) {
        const uint32_t l = code_len[s];
        if (l > ZM_MAX_CODE_LEN) return false;
        b.len[s] = static_cast<uint8_t>(l);
        b.wire[s] = 0; b.canon[s] = 0;
        if (l) { ++count[l]; ++b.n_present; b.kraft += 1u << (ZM_MAX_CODE_LEN - l); b.max_len = std::max(b.max_len, l); }
    }
    if (b.kraft > (1u << ZM_MAX_CODE_LEN)) return false;
    // first canonical code of each length: codes of length l follow those of length l-1
    uint32_t first[ZM_MAX_CODE_LEN + 2] = {0};
    uint32_t code = 0;
    for (uint32_t l = 1; l <= ZM_MAX_CODE_LEN; ++l) { code = (code + count[l - 1]) << 1; first[l] = code; }
    bool pad_set = false;
    for (uint32_t l = 1; l <= ZM_MAX_CODE_LEN; ++l) {
        uint32_t c = first[l];
        for (int s = 0; s < 256; ++s) {
            if (b.len[s] != l) continue;
            uint32_t rev = 0;
            for (uint32_t k = 0; k < l; ++k) rev |= ((c >> k) & 1u) << (l - 1 - k);
            b.wire[s] = static_cast<uint16_t>(rev);
            b.canon[s] = static_cast<uint16_t>(c);
            if (!pad_set) { b.pad = static_cast<uint32_t>(s); pad_set = true; }
            ++c;
        }
    }
    return true;
}

void fill_decode_table(const Book &b, uint8_t *lut /* 2 << max_len bytes */)
{
    const uint32_t entries = 1u << b.max_len;
    for (uint32_t x = 0; x < entries; ++x) { lut[2 * x] = static_cast<uint8_t>(b.pad); lut[2 * x + 1] = 1; }
    for (int s = 0; s < 256; ++s) {
        const uint32_t l = b.len[s];
        if (!l) continue;
        for (uint32_t x = b.wire[s]; x < entries; x += 1u << l) { lut[2 * x] = static_cast<uint8_t>(s); lut[2 * x + 1] = static_cast<uint8_t>(l); }
    }
}

// Upper bound on the bytes of one coded stream: 64 length bytes, the code bits, the rounding of every lane
// to the quantum, the padding to 16 bytes.
size_t stream_byte_bound(uint32_t stream_values)
{
    const size_t syms = static_cast<size_t>(stream_values / kTile) * kRun;
    return align_up(kLanes + (kLanes * (syms * ZM_MAX_CODE_LEN + 255) + 7) / 8, 16);
}

// Packs exponents e[0..n) of one stream: 64 length bytes, then the lanes' bitstreams back to back (LSB first),
// zero bits to a multiple of 16 bytes.  A lane's bitstream holds the codes of its first half of symbols from its
// first bit upwards and those of its second half, last symbol first, from its last bit downwards; the unused
// bits sit in the middle.  Returns the bytes written.
size_t pack_stream(const uint8_t *e, uint32_t n, const Book &b, uint32_t quantum, uint8_t *out)
{
    const uint32_t tiles = (n + kTile - 1) / kTile;
    const uint32_t syms = tiles * kRun;                 // per lane
    uint8_t *payload = out + kLanes;
    uint64_t acc = 0;                                    // bits not yet written, lowest first
    uint32_t fill = 0;
    size_t at = 0;                                       // payload bytes written
    auto put = [&](uint32_t bits, uint32_t count) {      // count <= 32
        acc |= static_cast<uint64_t>(bits) << fill;
        fill += count;
        while (fill >= 8) { payload[at++] = static_cast<uint8_t>(acc); acc >>= 8; fill -= 8; }
    };
    auto symbol = [&](uint32_t lane, uint32_t j) -> uint32_t {
        const uint32_t idx = (j / kRun) * kTile + lane * kRun + (j % kRun);
        return idx < n ? e[idx] : b.pad;
    };
    for (uint32_t lane = 0; lane < kLanes; ++lane) {
        uint32_t used = 0;
        for (uint32_t j = 0; j < syms; ++j) used += b.len[symbol(lane, j)];
        const uint32_t units = (used - syms + quantum - 1) / quantum;
        out[lane] = static_cast<uint8_t>(units);
        // in ascending bit order: the first half's codes, first bit lowest; the zero bits in the middle; the
        // second half's codes from the half's first symbol (read last) to the lane's last symbol (read first),
        // each with its first bit highest
        for (uint32_t j = 0; j < syms / 2; ++j) { const uint32_t s = symbol(lane, j); put(b.wire[s], b.len[s]); }
        for (uint32_t fillers = syms + quantum * units - used; fillers; ) {
            const uint32_t k = std::min(fillers, 32u);
            put(0, k);
            fillers -= k;
        }
        for (uint32_t j = syms / 2; j < syms; ++j) { const uint32_t s = symbol(lane, j); put(b.canon[s], b.len[s]); }
    }
    if (fill) put(0, 8 - fill);
    const size_t total = align_up(kLanes + at, 16);
    std::memset(payload + at, 0, total - kLanes - at);
    return total;
}

int read_info(const uint8_t *p, size_t size, zm_tensor_info *info, Book *book_out)
{
    if (size < kHeaderBytes + 256) return ZM_E_FORMAT;
    if (load_le<uint32_t>(p + Hdr::magic) != kMagic || load_le<uint32_t>(p + Hdr::version) != kVersion) return ZM_E_FORMAT;
    zm_tensor_info t{};
    t.n_values = load_le<uint64_t>(p + Hdr::n_values);
    t.chunk_values = load_le<uint32_t>(p + Hdr::chunk);
    t.stream_values = load_le<uint32_t>(p + Hdr::stream);
    t.n_chunks = load_le<uint32_t>(p + Hdr::n_chunks);
    t.max_len = load_le<uint32_t>(p + Hdr::max_len);
    t.lane_quantum = load_le<uint32_t>(p + Hdr::quantum);
    t.n_present = load_le<uint32_t>(p + Hdr::n_present);
    t.lut_offset = load_le<uint64_t>(p + Hdr::lut_off);
    t.table_offset = load_le<uint64_t>(p + Hdr::table_off);
    t.sm_offset = load_le<uint64_t>(p + Hdr::sm_off);
    t.e_offset = load_le<uint64_t>(p + Hdr::e_off);
    t.blob_size = load_le<uint64_t>(p + Hdr::blob_size);
    if (!geometry_ok(t.chunk_values, t.stream_values)) return ZM_E_FORMAT;
    if (t.max_len < 1 || t.max_len > ZM_MAX_CODE_LEN) return ZM_E_FORMAT;
    const uint64_t chunks = (t.n_values + t.chunk_values - 1) / t.chunk_values;
    if (chunks != t.n_chunks) return ZM_E_FORMAT;
    if (load_le<uint64_t>(p + Hdr::len_off) != kHeaderBytes || t.lut_offset != kHeaderBytes + 256) return ZM_E_FORMAT;
    if (t.table_offset != align_up(t.lut_offset + (2ull << t.max_len), 16)) return ZM_E_FORMAT;
    t.table_stride = load_le<uint32_t>(p + Hdr::table_stride);
    if (t.table_stride != table_stride_for(t.chunk_values, t.stream_values)) return ZM_E_FORMAT;
    if (t.sm_offset != align_up(t.table_offset + static_cast<uint64_t>(t.table_stride) * (chunks + 1), 256)) return ZM_E_FORMAT;
    if (t.e_offset != align_up(t.sm_offset + t.n_values, 256)) return ZM_E_FORMAT;
    if (t.blob_size < t.e_offset || (t.blob_size & 255)) return ZM_E_FORMAT;
    Book b;
    if (!make_book(p + kHeaderBytes, b)) return ZM_E_FORMAT;
    if (b.max_len != t.max_len || b.n_present != t.n_present) return ZM_E_FORMAT;
    if (t.lane_quantum != lane_quantum_for(t.max_len, t.stream_values)) return ZM_E_FORMAT;
    if (load_le<uint32_t>(p + Hdr::pad_sym) != b.pad) return ZM_E_FORMAT;
    if (b.n_present >= 2 && b.kraft != (1u << ZM_MAX_CODE_LEN)) return ZM_E_FORMAT;   // decode table must be total
    if (t.n_values > 0 && b.n_present == 0) return ZM_E_FORMAT;
    if (info) *info = t;
    if (book_out) *book_out = b;
    return ZM_OK;
}

// Length-limited optimal prefix code by package-merge (Larmore & Hirschberg 1990).
// weight[i] ascending; returns lengths for the n sorted items.
void package_merge(const std::vector<uint64_t> &weight, int max_len, std::vector<uint8_t> &length)
{
    const size_t n = weight.size();
    length.assign(n, 0);
    if (n == 1) { length[0] = 1; return; }
    struct Node { uint64_t w; std::vector<uint8_t> uses; };   // uses[i]: how often item i is inside
    std::vector<Node> level;                                   // current list, ascending
    level.reserve(2 * n);
    for (size_t i = 0; i < n; ++i) { Node nd{weight[i], std::vector<uint8_t>(n, 0)}; nd.uses[i] = 1; level.push_back(std::move(nd)); }
    for (int depth = 2; depth <= max_len; ++depth) {
        std::vector<Node> packs;
        for (size_t i = 0; i + 1 < level.size(); i += 2) {
            Node nd{level[i].w + level[i + 1].w, level[i].uses};
            for (size_t k = 0; k < n; ++k) nd.uses[k] = static_cast<uint8_t>(nd.uses[k] + level[i + 1].uses[k]);
            packs.push_back(std::move(nd));
        }
        std::vector<Node> merged;
        merged.reserve(n + packs.size());
        size_t a = 0, b = 0;
        while (a < n || b < packs.size()) {
            // on equal weight a plain item goes first
            if (b >= packs.size() || (a < n && weight[a] <= packs[b].w)) {
                Node nd{weight[a], std::vector<uint8_t>(n, 0)}; nd.uses[a] = 1; merged.push_back(std::move(nd)); ++a;
            } else merged.push_back(std::move(packs[b++]));
        }
        level.swap(merged);
    }
    for (size_t i = 0; i < 2 * n - 2; ++i)
        for (size_t k = 0; k < n; ++k) length[k] = static_cast<uint8_t>(length[k] + level[i].uses[k]);
}


// Table-driven decode of one stream on the host: the prefix sum over the length bytes gives every lane's
// first and last bit; each lane is decoded on its own, its first half of symbols upwards through one 64-bit
// buffer and its second half downwards through another, a symbol of each per step.
// lut: 2^max_len entries (symbol, length) indexed by the next max_len bits with the first bit lowest, followed by
// 2^max_len entries indexed with the first bit highest.  Returns false if a lane's halves would run into each other.
bool unpack_stream(const uint8_t *stream, size_t n_bytes, uint32_t n, const uint8_t *lut, uint32_t max_len,
                   uint32_t quantum, uint8_t *e)
{
    const uint32_t tiles = (n + kTile - 1) / kTile;
    const uint32_t syms = tiles * kRun;
    const uint32_t mask = (1u << max_len) - 1u;
    const uint8_t *mirror = lut + (2u << max_len);
    if (n_bytes < kLanes) return false;
    const uint8_t *payload = stream + kLanes;
    const size_t payload_words = (n_bytes - kLanes) / 4;
    const uint64_t payload_bits = payload_words * 32ull;
    auto word = [&](size_t i) -> uint64_t { return i < payload_words ? load_le<uint32_t>(payload + 4 * i) : 0u; };   // zeros outside
    auto place = [&](uint32_t lane, uint32_t j, uint32_t sym) {
        const uint32_t idx = (j / kRun) * kTile + lane * kRun + (j % kRun);
        if (idx < n) e[idx] = static_cast<uint8_t>(sym);
    };
    uint64_t start = 0;
    for (uint32_t lane = 0; lane < kLanes; ++lane) {
        const uint64_t span = syms + static_cast<uint64_t>(quantum) * stream[lane];
        if (start + span > payload_bits) return false;
        // upwards: the next bit is bit 0 of `up`; at least 32 valid bits before a lookup
        size_t next_up = start >> 5;
        uint64_t up = (word(next_up) | word(next_up + 1) << 32) >> (start & 31);
        uint32_t up_valid = 64 - static_cast<uint32_t>(start & 31);
        next_up += 2;
        // downwards: the next bit is bit 63 of `down`
        const uint64_t end = start + span;
        size_t next_down = end >> 5;                       // the word that holds the bits just below `end`, if end is not word-aligned
        uint32_t down_valid = static_cast<uint32_t>(end & 31);
        uint64_t down = down_valid ? word(next_down) << (64 - down_valid) : 0;
        --next_down;                                       // wraps past zero to an index outside the payload: reads as zero
        while (down_valid <= 32) { down |= word(next_down--) << (32 - down_valid); down_valid += 32; }
        uint64_t used = 0;
        for (uint32_t step = 0; step < syms / 2; ++step) {
            const uint32_t a = static_cast<uint32_t>(up) & mask;
            const uint32_t z = static_cast<uint32_t>(down >> (64 - max_len));
            place(lane, step, lut[2 * a]);
            place(lane, syms - 1 - step, mirror[2 * z]);
            const uint32_t la = lut[2 * a + 1], lz = mirror[2 * z + 1];
            up >>= la; up_valid -= la;
            down <<= lz; down_valid -= lz;
            used += la + lz;
            if (up_valid <= 32) { up |= word(next_up++) << up_valid; up_valid += 32; }
            if (down_valid <= 32) { down |= word(next_down--) << (32 - down_valid); down_valid += 32; }
        }
        if (used > span) return false;
        start += span;
    }
    return true;
}

// lut: the decode table built from the blob's code lengths (not the blob's own copy, which a caller may not
// have validated: its lengths bound the shifts below)
int decode_chunk_exponents(const uint8_t *p, const zm_tensor_info &t, const uint8_t *lut, uint64_t c, uint8_t *e_out)
{
    const uint8_t *entry = p + t.table_offset + static_cast<uint64_t>(t.table_stride) * c;
    const uint64_t ent = load_le<uint64_t>(entry);
    const uint64_t nxt = load_le<uint64_t>(entry + t.table_stride);
    const uint64_t at = ent & ~15ull, end = nxt & ~15ull, mode = ent & 15;
    if (at < t.e_offset || end < at || end > t.blob_size) return ZM_E_FORMAT;
    const uint64_t first = c * t.chunk_values;
    const uint32_t cn = static_cast<uint32_t>(std::min<uint64_t>(t.chunk_values, t.n_values - first));
    uint8_t *e = e_out + first;
    if (mode == ZM_MODE_RAW) {
        if (end - at < cn) return ZM_E_FORMAT;
        std::memcpy(e, p + at, cn);
        return ZM_OK;
    }
    if (mode != ZM_MODE_CODED) return ZM_E_FORMAT;
    const uint32_t streams = (cn + t.stream_values - 1) / t.stream_values;
    const uint8_t *h = p + at;
    for (uint32_t s = 0; s < streams; ++s) {
        const uint32_t o0 = load_le<uint32_t>(entry + 8 + 4 * s), o1 = load_le<uint32_t>(entry + 8 + 4 * (s + 1));
        if ((o0 & 3) || o1 < o0 || o1 > end - at) return ZM_E_FORMAT;
        const uint32_t sn = std::min(t.stream_values, cn - s * t.stream_values);
        if (!unpack_stream(h + o0, o1 - o0, sn, lut, t.max_len, t.lane_quantum, e + static_cast<size_t>(s) * t.stream_values))
            return ZM_E_FORMAT;
    }
    return ZM_OK;
}

}  // namespace

extern "C" {

int zm_version(void) { return 20000; }    // 2.0.0: serialised format 3

const char *zm_strerror(int status)
{
    switch (status) {
        case ZM_OK: return "ok";
        case ZM_E_ARG: return "invalid argument";
        case ZM_E_SIZE: return "output buffer too small";
        case ZM_E_FORMAT: return "malformed serialised tensor";
        case ZM_E_HIP: return "HIP runtime error";
        case ZM_E_NOMEM: return "out of host memory";
        default: return "unknown status";
    }
}

int zm_exponent_histogram(const uint16_t *bf16, size_t n_values, uint64_t hist[256])
{
    if ((!bf16 && n_values) || !hist) return ZM_E_ARG;
    uint64_t h[4][256] = {};
    size_t i = 0;
    for (; i + 4 <= n_values; i += 4) {
        ++h[0][(bf16[i] >> 7) & 0xFF]; ++h[1][(bf16[i + 1] >> 7) & 0xFF];
        ++h[2][(bf16[i + 2] >> 7) & 0xFF]; ++h[3][(bf16[i + 3] >> 7) & 0xFF];
    }
    for (; i < n_values; ++i) ++h[0][(bf16[i] >> 7) & 0xFF];
    for (int s = 0; s < 256; ++s) hist[s] = h[0][s] + h[1][s] + h[2][s] + h[3][s];
    return ZM_OK;
}

int zm_build_codebook(const uint64_t hist[256], int max_len, uint8_t code_len_out[256])
{
    if (!hist || !code_len_out || max_len < 1 || max_len > ZM_MAX_CODE_LEN) return ZM_E_ARG;
    try {
        std::vector<std::pair<uint64_t, int>> present;
        for (int s = 0; s < 256; ++s) { code_len_out[s] = 0; if (hist[s]) present.emplace_back(hist[s], s); }
        if (present.empty()) return ZM_OK;
        if (present.size() > (1ull << max_len)) return ZM_E_ARG;
        std::sort(present.begin(), present.end());
        std::vector<uint64_t> weight;
        for (auto &p : present) weight.push_back(p.first);
        std::vector<uint8_t> length;
        package_merge(weight, max_len, length);
        for (size_t i = 0; i < present.size(); ++i) code_len_out[present[i].second] = length[i];
    } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    return ZM_OK;
}

size_t zm_encode_bound(size_t n_values, uint32_t chunk_values, uint32_t stream_values)
{
    if (!geometry_ok(chunk_values, stream_values)) return 0;
    const size_t chunks = (n_values + chunk_values - 1) / chunk_values;
    // header + code lengths + widest decode table + chunk table + SM section + E-chunks stored raw, each with padding
    return 384 + (2u << ZM_MAX_CODE_LEN) + 16 + static_cast<size_t>(table_stride_for(chunk_values, stream_values)) * (chunks + 1) +
           256 + (n_values + 256) + (n_values + 16 * chunks) + 256;
}

int zm_encode(const uint16_t *bf16, size_t n_values, uint32_t chunk_values, uint32_t stream_values,
              const uint8_t code_len[256], uint8_t *blob, size_t blob_cap, size_t *blob_size,
              uint64_t *chunk_offsets, size_t chunk_offsets_cap, size_t *n_chunks)
{
    if ((!bf16 && n_values) || !code_len || !blob || !blob_size) return ZM_E_ARG;
    if (!geometry_ok(chunk_values, stream_values)) return ZM_E_ARG;
    Book book;
    if (!make_book(code_len, book)) return ZM_E_ARG;
    if (book.n_present >= 2 && book.kraft != (1u << ZM_MAX_CODE_LEN)) return ZM_E_ARG;   // the decode table must be total
    const size_t chunks = (n_values + chunk_values - 1) / chunk_values;
    if (blob_cap < zm_encode_bound(n_values, chunk_values, stream_values)) return ZM_E_SIZE;
    const uint32_t stride = table_stride_for(chunk_values, stream_values);
    if (chunk_offsets && chunk_offsets_cap < (chunks + 1) * (stride / 8)) return ZM_E_SIZE;

    const uint32_t L = book.max_len;
    const uint64_t lut_off = kHeaderBytes + 256;
    const uint64_t table_off = align_up(lut_off + (2ull << L), 16);
    const uint64_t sm_off = align_up(table_off + static_cast<uint64_t>(stride) * (chunks + 1), 256);
    const uint64_t e_off = align_up(sm_off + n_values, 256);
    try {
        std::memset(blob, 0, e_off);
        std::memcpy(blob + kHeaderBytes, book.len, 256);
        fill_decode_table(book, blob + lut_off);

        // split (Sec. 3.1): sign-mantissa bytes go straight to their section, exponent bytes to scratch
        std::vector<uint8_t> expo(n_values ? n_values : 1);
        uint8_t *sm = blob + sm_off;
        for (size_t i = 0; i < n_values; ++i) {
            const uint32_t w = bf16[i];
            const uint32_t ex = (w >> 7) & 0xFF;
            if (!book.len[ex]) return ZM_E_ARG;
            expo[i] = static_cast<uint8_t>(ex);
            sm[i] = static_cast<uint8_t>(((w >> 8) & 0x80) | (w & 0x7F));
        }

        const uint32_t quantum = lane_quantum_for(L, stream_values);
        const uint32_t max_streams = chunk_values / stream_values;
        std::vector<uint8_t> coded(static_cast<size_t>(max_streams) * stream_byte_bound(stream_values));
        uint64_t pos = e_off;
        for (size_t c = 0; c < chunks; ++c) {
            const size_t first = c * static_cast<size_t>(chunk_values);
            const uint32_t cn = static_cast<uint32_t>(std::min<size_t>(chunk_values, n_values - first));
            const uint32_t streams = (cn + stream_values - 1) / stream_values;
            const uint64_t raw_bytes = align_up(cn, 16);
            uint8_t *entry = blob + table_off + static_cast<uint64_t>(stride) * c;      // zero so far
            size_t at = 0;                                                               // bytes
            bool smaller = true;
            for (uint32_t s = 0; s < streams; ++s) {
                store_le<uint32_t>(entry + 8 + 4 * s, static_cast<uint32_t>(at));
                const uint32_t sn = std::min(stream_values, cn - s * stream_values);
                at += pack_stream(&expo[first + static_cast<size_t>(s) * stream_values], sn, book, quantum, &coded[at]);
                if (at >= raw_bytes) { smaller = false; break; }
            }
            uint64_t mode;
            if (smaller) {
                store_le<uint32_t>(entry + 8 + 4 * streams, static_cast<uint32_t>(at));
                std::memcpy(blob + pos, coded.data(), at);
                mode = ZM_MODE_CODED;
            } else {
                std::memset(entry, 0, stride);
                std::memset(blob + pos, 0, raw_bytes);
                std::memcpy(blob + pos, &expo[first], cn);
                mode = ZM_MODE_RAW;
            }
            store_le<uint64_t>(entry, pos | mode);
            pos += smaller ? at : raw_bytes;
        }
        store_le<uint64_t>(blob + table_off + static_cast<uint64_t>(stride) * chunks, pos);
        const uint64_t total = align_up(pos, 256);
        std::memset(blob + pos, 0, total - pos);

        store_le<uint32_t>(blob + Hdr::magic, kMagic);
        store_le<uint32_t>(blob + Hdr::version, kVersion);
        store_le<uint64_t>(blob + Hdr::n_values, n_values);
        store_le<uint32_t>(blob + Hdr::chunk, chunk_values);
        store_le<uint32_t>(blob + Hdr::stream, stream_values);
        store_le<uint32_t>(blob + Hdr::n_chunks, static_cast<uint32_t>(chunks));
        store_le<uint32_t>(blob + Hdr::max_len, L);
        store_le<uint32_t>(blob + Hdr::quantum, quantum);
        store_le<uint32_t>(blob + Hdr::n_present, book.n_present);
        store_le<uint32_t>(blob + Hdr::pad_sym, book.pad);
        store_le<uint32_t>(blob + Hdr::table_stride, stride);
        store_le<uint64_t>(blob + Hdr::len_off, kHeaderBytes);
        store_le<uint64_t>(blob + Hdr::lut_off, lut_off);
        store_le<uint64_t>(blob + Hdr::table_off, table_off);
        store_le<uint64_t>(blob + Hdr::sm_off, sm_off);
        store_le<uint64_t>(blob + Hdr::e_off, e_off);
        store_le<uint64_t>(blob + Hdr::blob_size, total);
        *blob_size = total;
        if (n_chunks) *n_chunks = chunks;
        if (chunk_offsets) std::memcpy(chunk_offsets, blob + table_off, static_cast<size_t>(stride) * (chunks + 1));
    } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    return ZM_OK;
}

int zm_blob_info(const void *blob_host, size_t size, zm_tensor_info *info)
{
    if (!blob_host || !info) return ZM_E_ARG;
    return read_info(static_cast<const uint8_t *>(blob_host), size, info, nullptr);
}

int zm_validate_blob(const void *blob_host, size_t size)
{
    if (!blob_host) return ZM_E_ARG;
    const uint8_t *p = static_cast<const uint8_t *>(blob_host);
    zm_tensor_info t; Book book;
    const int rc = read_info(p, size, &t, &book);
    if (rc != ZM_OK) return rc;
    if (t.blob_size > size) return ZM_E_FORMAT;
    for (size_t i = Hdr::blob_size + 8; i < kHeaderBytes; ++i) if (p[i]) return ZM_E_FORMAT;
    // decode table must be the one the code lengths define
    std::vector<uint8_t> lut(2u << t.max_len);
    fill_decode_table(book, lut.data());
    if (std::memcmp(lut.data(), p + t.lut_offset, lut.size())) return ZM_E_FORMAT;
    // chunk table and chunk structure
    uint64_t expect = t.e_offset;
    const uint64_t byte_cap = stream_byte_bound(t.stream_values);
    for (uint64_t c = 0; c < t.n_chunks; ++c) {
        const uint8_t *entry = p + t.table_offset + static_cast<uint64_t>(t.table_stride) * c;
        const uint64_t ent = load_le<uint64_t>(entry);
        const uint64_t nxt = load_le<uint64_t>(entry + t.table_stride);
        const uint64_t at = ent & ~15ull, end = nxt & ~15ull, mode = ent & 15;
        if (at != expect || end < at || end > t.blob_size) return ZM_E_FORMAT;
        const uint64_t cn = std::min<uint64_t>(t.chunk_values, t.n_values - c * t.chunk_values);
        uint64_t used_slots = 0;                     // 32-bit offset slots of the entry that carry data
        if (mode == ZM_MODE_RAW) {
            if (end - at != align_up(cn, 16)) return ZM_E_FORMAT;
        } else if (mode == ZM_MODE_CODED) {
            const uint64_t streams = (cn + t.stream_values - 1) / t.stream_values;
            used_slots = streams + 1;
            if (load_le<uint32_t>(entry + 8) != 0 || load_le<uint32_t>(entry + 8 + 4 * streams) != end - at) return ZM_E_FORMAT;
            for (uint64_t s = 0; s < streams; ++s) {
                const uint32_t o0 = load_le<uint32_t>(entry + 8 + 4 * s), o1 = load_le<uint32_t>(entry + 8 + 4 * (s + 1));
                if ((o0 & 15) || (o1 & 15) || o1 < o0 || o1 > end - at) return ZM_E_FORMAT;
                if (o1 - o0 < kLanes || o1 - o0 > byte_cap) return ZM_E_FORMAT;
                // the lanes' bit counts must fit the stream: a decoder reads no lane past the stream's end
                const uint64_t sn = std::min<uint64_t>(t.stream_values, cn - s * t.stream_values);
                const uint64_t syms = (sn + kTile - 1) / kTile * kRun;
                const uint8_t *lane_bytes = p + at + o0;
                uint64_t bits = 0;
                for (uint32_t lane = 0; lane < kLanes; ++lane) bits += syms + static_cast<uint64_t>(t.lane_quantum) * lane_bytes[lane];
                if (align_up(kLanes + (bits + 7) / 8, 16) != o1 - o0) return ZM_E_FORMAT;
            }
        } else return ZM_E_FORMAT;
        for (uint64_t j = 8 + 4 * used_slots; j < t.table_stride; j += 4) if (load_le<uint32_t>(entry + j)) return ZM_E_FORMAT;
        expect = end;
    }
    const uint8_t *last_entry = p + t.table_offset + static_cast<uint64_t>(t.table_stride) * t.n_chunks;
    const uint64_t last = load_le<uint64_t>(last_entry);
    if (last != expect || align_up(last, 256) != t.blob_size) return ZM_E_FORMAT;
    for (uint64_t j = 8; j < t.table_stride; j += 4) if (load_le<uint32_t>(last_entry + j)) return ZM_E_FORMAT;
    return ZM_OK;
}


int zm_decode_exponents_host(const void *blob_host, size_t size, uint32_t chunk_begin, uint32_t chunk_end,
                             uint8_t *e_out, int n_threads)
{
    if (!blob_host || !e_out) return ZM_E_ARG;
    const uint8_t *p = static_cast<const uint8_t *>(blob_host);
    zm_tensor_info t; Book book;
    const int rc = read_info(p, size, &t, &book);
    if (rc != ZM_OK) return rc;
    if (t.blob_size > size) return ZM_E_FORMAT;
    if (chunk_begin > chunk_end || chunk_end > t.n_chunks) return ZM_E_ARG;
    if (chunk_begin == chunk_end) return ZM_OK;
    const uint32_t workers = std::min<uint32_t>(std::max(n_threads, 1), chunk_end - chunk_begin);
    std::atomic<uint32_t> next_chunk{chunk_begin};
    std::atomic<int> status{ZM_OK};
    std::vector<std::thread> pool;
    try {
        // two tables: the blob's (indexed by the next max_len bits, first bit lowest) for the upward chain and its
        // mirror (first bit highest) for the downward chain
        std::vector<uint8_t> lut(4u << t.max_len);
        fill_decode_table(book, lut.data());
        for (uint32_t x = 0; x < (1u << t.max_len); ++x) {
            const uint32_t y = __builtin_bitreverse32(x) >> (32 - t.max_len);
            lut[(2u << t.max_len) + 2 * x] = lut[2 * y];
            lut[(2u << t.max_len) + 2 * x + 1] = lut[2 * y + 1];
        }
        auto work = [&]() {
            for (;;) {
                const uint32_t c = next_chunk.fetch_add(1);
                if (c >= chunk_end || status.load() != ZM_OK) return;
                const int r = decode_chunk_exponents(p, t, lut.data(), c, e_out);
                if (r != ZM_OK) status.store(r);
            }
        };
        try {
            pool.reserve(workers);
            for (uint32_t i = 1; i < workers; ++i) pool.emplace_back(work);
        } catch (...) {
            status.store(ZM_E_NOMEM);                  // the threads that did start see it and stop
        }
        work();
        for (auto &th : pool) th.join();
    } catch (...) {
        for (auto &th : pool) if (th.joinable()) th.join();
        return ZM_E_NOMEM;
    }
    return status.load();
}

}  // extern "C"
