/*
 * zm_oracle.c -- reference codec for compressed bf16 expert weights.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain checker that the
 * tests, the smoke check and the benchmark's CPU-baseline leg run; the
 * product library never includes, links or calls it, and it shares no code,
 * table or header with the product library.
 *
 * What it follows (ZipMoE, arXiv 2601.21198):
 *   - Sec. 2.2 "BF16 Parameters": a bf16 word is 1 sign, 8 exponent and 7
 *     mantissa bits.
 *   - Sec. 3.1 "Offline Initialization": bit-field decomposition into
 *     exponent bits and sign-mantissa bits; the exponent bits are cut into
 *     K shards that are compressed one by one (E-chunks); the sign-mantissa
 *     bits are packed one byte per value (SM-chunks); everything plus the
 *     metadata is serialised into one binary object.
 *   - Sec. 3.3 "Memory-Coalesced Tensor Recovery Kernel": the inverse step,
 *     exponent byte + sign-mantissa byte -> bf16 word.
 *   - Sec. 6 "Other Compressors": the compressor that turns exponent bytes
 *     into an E-chunk is pluggable.  The backend defined here is a canonical,
 *     length-limited prefix code (one codebook per tensor).  Its bitstream
 *     layout is not in the paper; it is fixed by this file and described in
 *     the comments below, step by step.
 *
 * Every function is written for readability, one step at a time: bits are
 * handled one at a time, the code-length optimiser is an exhaustive dynamic
 * programme over the Kraft budget, and nothing is blocked, fused or
 * table-accelerated.
 *
 * Parity status: every function here is pinned by tests that do not go
 * through this file's own arithmetic (closed forms, brute force, the exact
 * round-trip property, the entropy bound of Sec. 2.2); nothing is unpinned.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* ---- layout constants of the serialised object ------------------------- */

#define ZO_MAGIC        0x454F4D5Au   /* bytes 'Z','M','O','E' */
#define ZO_VERSION      4u
#define ZO_HEADER_BYTES 128u
#define ZO_LANES        64u   /* per-stream lanes                              */
#define ZO_RUN          8u    /* consecutive values one lane owns in a tile     */
#define ZO_TILE         512u  /* ZO_LANES * ZO_RUN values                       */
#define ZO_MAX_LEN      12    /* longest code the format admits                 */

enum { ZO_OK = 0, ZO_E_ARG = -1, ZO_E_SIZE = -2, ZO_E_FORMAT = -3, ZO_E_NOMEM = -4 };

enum { ZO_MODE_CODED = 0, ZO_MODE_RAW = 1 };

/* header field offsets (bytes) */
enum {
    H_MAGIC = 0, H_VERSION = 4, H_NVALUES = 8, H_CHUNK = 16, H_STREAM = 20,
    H_NCHUNKS = 24, H_L = 28, H_QUANTUM = 32, H_NPRESENT = 36, H_PADSYM = 40, H_TABLE_STRIDE = 44,
    H_LEN_OFF = 48, H_LUT_OFF = 56, H_TABLE_OFF = 64, H_SM_OFF = 72,
    H_E_OFF = 80, H_BLOB_SIZE = 88
};

static uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

static void put32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void put64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static uint32_t get32(const uint8_t *p) { uint32_t v = 0; for (int i = 0; i < 4; i++) v |= (uint32_t)p[i] << (8 * i); return v; }
static uint64_t get64(const uint8_t *p) { uint64_t v = 0; for (int i = 0; i < 8; i++) v |= (uint64_t)p[i] << (8 * i); return v; }

/* ---- Sec. 2.2 / Sec. 3.1: bit-field decomposition ---------------------- */

/* word = s eeeeeeee mmmmmmm (bit 15 .. bit 0).
 * exponent byte  = the 8 e bits;
 * sign-mantissa byte = s in bit 7, the 7 m bits in bits 6..0.               */
void zo_split(const uint16_t *w, size_t n, uint8_t *e, uint8_t *sm)
{
    for (size_t i = 0; i < n; i++) {
        unsigned sign = (w[i] >> 15) & 1u;
        unsigned expo = (w[i] >> 7) & 0xFFu;
        unsigned mant = w[i] & 0x7Fu;
        e[i] = (uint8_t)expo;
        sm[i] = (uint8_t)((sign << 7) | mant);
    }
}

/* Sec. 3.3: the recovery step, the inverse of zo_split. */
void zo_merge(const uint8_t *e, const uint8_t *sm, size_t n, uint16_t *w)
{
    for (size_t i = 0; i < n; i++) {
        unsigned sign = (sm[i] >> 7) & 1u;
        unsigned mant = sm[i] & 0x7Fu;
        unsigned expo = e[i];
        w[i] = (uint16_t)((sign << 15) | (expo << 7) | mant);
    }
}

void zo_histogram(const uint8_t *e, size_t n, uint64_t hist[256])
{
    for (int s = 0; s < 256; s++) hist[s] = 0;
    for (size_t i = 0; i < n; i++) hist[e[i]]++;
}

/* ---- codebook: optimal length-limited prefix-code lengths -------------- */

/* Definition used: among all assignments len[s] in 1..max_len for the
 * symbols with hist[s] > 0 that satisfy the Kraft inequality
 *      sum_s 2^(-len[s]) <= 1,
 * pick one that minimises sum_s hist[s]*len[s].  A prefix code with those
 * lengths exists exactly when Kraft holds, so this is the optimal
 * length-limited prefix code.  The search is an exact dynamic programme:
 * symbols are taken one by one, the state is the Kraft budget spent so far
 * in units of 2^(-max_len).  Absent symbols get length 0.
 * Returns ZO_E_ARG if max_len is outside 1..ZO_MAX_LEN or the present
 * symbols cannot fit (more than 2^max_len of them).                        */
int zo_code_lengths(const uint64_t hist[256], int max_len, uint8_t len[256])
{
    if (max_len < 1 || max_len > ZO_MAX_LEN) return ZO_E_ARG;
    int sym[256], n = 0;
    for (int s = 0; s < 256; s++) { len[s] = 0; if (hist[s] > 0) sym[n++] = s; }
    if (n == 0) return ZO_OK;
    const uint32_t budget = 1u << max_len;
    if ((uint32_t)n > budget) return ZO_E_ARG;

    const uint64_t INF = UINT64_MAX;
    /* cost[i][k]: least sum of hist*len over the first i present symbols
     * whose Kraft terms add up to exactly k units; pick[i][k]: the length
     * given to symbol i-1 on that best path.                                */
    size_t row = (size_t)budget + 1;
    uint64_t *cost = (uint64_t *)malloc((size_t)(n + 1) * row * sizeof(uint64_t));
    uint8_t *pick = (uint8_t *)malloc((size_t)(n + 1) * row);
    if (!cost || !pick) { free(cost); free(pick); return ZO_E_NOMEM; }
    for (size_t j = 0; j < (size_t)(n + 1) * row; j++) { cost[j] = INF; pick[j] = 0; }
    cost[0] = 0;
    for (int i = 0; i < n; i++) {
        for (uint32_t k = 0; k <= budget; k++) {
            uint64_t c = cost[(size_t)i * row + k];
            if (c == INF) continue;
            for (int l = 1; l <= max_len; l++) {
                uint32_t k2 = k + (1u << (max_len - l));
                if (k2 > budget) continue;
                uint64_t c2 = c + hist[sym[i]] * (uint64_t)l;
                size_t j = (size_t)(i + 1) * row + k2;
                if (c2 < cost[j]) { cost[j] = c2; pick[j] = (uint8_t)l; }
            }
        }
    }
    uint32_t best_k = 0; uint64_t best = INF;
    for (uint32_t k = 0; k <= budget; k++)
        if (cost[(size_t)n * row + k] < best) { best = cost[(size_t)n * row + k]; best_k = k; }
    uint32_t k = best_k;
    for (int i = n; i >= 1; i--) {
        int l = pick[(size_t)i * row + k];
        len[sym[i - 1]] = (uint8_t)l;
        k -= 1u << (max_len - l);
    }
    free(cost); free(pick);
    return ZO_OK;
}

/* Canonical code assignment.  Present symbols are ordered by (length
 * ascending, symbol value ascending); the first gets code 0, each next one
 * gets (previous code + 1) shifted left by the increase in length.  code[s]
 * holds the code as a number whose most significant of len[s] bits is the
 * first bit on the wire.  Returns the number of present symbols.           */
int zo_canonical(const uint8_t len[256], uint16_t code[256])
{
    int n = 0;
    uint32_t next = 0; int prev_len = 0;
    for (int s = 0; s < 256; s++) code[s] = 0;
    for (int l = 1; l <= ZO_MAX_LEN; l++) {
        for (int s = 0; s < 256; s++) {
            if (len[s] != l) continue;
            if (n > 0) next = (next + 1) << (l - prev_len);
            code[s] = (uint16_t)next;
            prev_len = l;
            n++;
        }
    }
    return n;
}

/* Integer Kraft sum in units of 2^(-ZO_MAX_LEN); a complete code gives
 * exactly 2^ZO_MAX_LEN.  Lengths outside 0..ZO_MAX_LEN give UINT32_MAX.    */
uint32_t zo_kraft_units(const uint8_t len[256])
{
    uint32_t k = 0;
    for (int s = 0; s < 256; s++) {
        if (len[s] > ZO_MAX_LEN) return UINT32_MAX;
        if (len[s]) k += 1u << (ZO_MAX_LEN - len[s]);
    }
    return k;
}

static int max_code_len(const uint8_t len[256])
{
    int L = 1;
    for (int s = 0; s < 256; s++) if (len[s] > L) L = len[s];
    return L;
}

/* the symbol that fills positions past the end of a stream: the first one in
 * canonical order, whose code is all zero bits                              */
static int pad_symbol(const uint8_t len[256])
{
    for (int l = 1; l <= ZO_MAX_LEN; l++)
        for (int s = 0; s < 256; s++) if (len[s] == l) return s;
    return 0;
}

/* ---- one stream: at most stream_values consecutive values -------------- */
/*
 * A stream is cut into tiles of 512 values.  In every tile lane j (0..63)
 * owns values 8j .. 8j+7, so over the stream a lane owns 8*tiles symbols,
 * taken tile after tile.  Positions at or past the stream's end hold the pad
 * symbol.
 *
 * Each lane has a bitstream of its own, D = m + q*b bits long (m = 8*tiles
 * symbols, T code bits, q the "quantum", a constant of the tensor kept in the
 * header, and the byte b = ceil((T - m) / q), which makes D the smallest such
 * number >= T).  It is filled from both ends, so that a decoder can work on
 * two independent halves at once:
 *   - the codes of the lane's first m/2 symbols, in order, from the lane's
 *     first bit upwards, the first bit of a code first;
 *   - the codes of its last m/2 symbols, in reverse order (symbol m-1 first),
 *     from the lane's last bit downwards, the first bit of a code at the
 *     higher position;
 *   - the D - T bits left in the middle are zero.
 * (Every code has at least one bit, so T >= m; q is the smallest integer
 * >= 1 for which b fits a byte whatever the symbols are:
 * q >= (L - 1) * (W / 64) / 255, L the longest code of the book, W the stream
 * length of the tensor.)
 *
 * The stream is
 *   bytes 0..63   b of lane 0, lane 1, ..., lane 63
 *   then          the 64 lane bitstreams one right after the other, lane 0
 *                 first, with no gap: lane j starts at bit D_0 + .. + D_(j-1).
 *                 Bit k of this payload is bit (k mod 32) of its 32-bit
 *                 little-endian word k / 32, i.e. bit (k mod 8) of byte k / 8.
 *   then          zero bits up to a multiple of 16 bytes.
 * A decoder finds every lane's first and last bit with a prefix sum over the
 * 64 bytes and then reads each lane's bits independently of the others.
 */

/* the quantum q of a tensor whose longest code has L bits and whose streams
 * hold W values                                                            */
static uint32_t lane_quantum(int L, uint32_t W)
{
    uint32_t span = (uint32_t)(L - 1) * (W / ZO_LANES);
    uint32_t q = (span + 254) / 255;
    return q ? q : 1;
}

/* worst-case number of bytes of one coded stream */
static size_t stream_bytes_bound(uint32_t stream_values)
{
    size_t tiles = (stream_values + ZO_TILE - 1) / ZO_TILE;
    size_t bits = (size_t)ZO_LANES * (tiles * ZO_RUN * ZO_MAX_LEN + 255);   /* code bits + rounding to the quantum */
    return round_up(ZO_LANES + (bits + 7) / 8, 16);
}

/* symbol number j of a lane: value i = j mod 8 of the lane's run in tile j / 8 */
static int lane_symbol(const uint8_t *e, uint32_t n, int pad, uint32_t lane, uint32_t j)
{
    uint32_t idx = (j / ZO_RUN) * ZO_TILE + lane * ZO_RUN + (j % ZO_RUN);
    return idx < n ? e[idx] : pad;
}

static void put_bit(uint8_t *payload, uint64_t k, uint32_t bit)
{
    payload[k / 8] |= (uint8_t)(bit << (k % 8));
}

static uint32_t get_bit(const uint8_t *payload, uint64_t k)
{
    return (payload[k / 8] >> (k % 8)) & 1u;
}

/* Encodes exponents e[0..n) (n <= stream_values) into out[], which must be
 * zero on entry; returns bytes written (a multiple of 16).                 */
static size_t encode_stream(const uint8_t *e, uint32_t n, const uint8_t len[256],
                            const uint16_t code[256], uint32_t q, int pad, uint8_t *out)
{
    const uint32_t tiles = (n + ZO_TILE - 1) / ZO_TILE;
    const uint32_t m = tiles * ZO_RUN;           /* symbols per lane */
    uint8_t *payload = out + ZO_LANES;
    uint64_t at = 0;                             /* payload bit where the current lane starts */
    for (uint32_t lane = 0; lane < ZO_LANES; lane++) {
        /* the lane's symbols in decode order, and its code bits */
        uint32_t T = 0;
        for (uint32_t j = 0; j < m; j++) T += len[lane_symbol(e, n, pad, lane, j)];
        uint32_t units = (T - m + q - 1) / q;                /* at most 255 by the choice of q */
        uint64_t D = m + (uint64_t)q * units;
        out[lane] = (uint8_t)units;
        /* first half: upwards from the lane's first bit */
        uint64_t k = at;
        for (uint32_t j = 0; j < m / 2; j++) {
            int s = lane_symbol(e, n, pad, lane, j);
            for (int b = len[s] - 1; b >= 0; b--)            /* first wire bit = top bit of the code */
                put_bit(payload, k++, (code[s] >> b) & 1u);
        }
        /* second half, last symbol first: downwards from the lane's last bit */
        k = at + D;
        for (uint32_t j = m; j-- > m / 2; ) {
            int s = lane_symbol(e, n, pad, lane, j);
            for (int b = len[s] - 1; b >= 0; b--)
                put_bit(payload, --k, (code[s] >> b) & 1u);
        }
        at += D;
    }
    return round_up(ZO_LANES + (at + 7) / 8, 16);
}

/* Decodes one stream of n_bytes bytes as stored.  Writes n exponent bytes.
 * Checks everything it can: that every bit it reads lies inside the lane's
 * own D bits, that every code is a code of the book, that pad positions hold
 * the pad symbol, that the lane's byte is the smallest that fits its codes,
 * that the bits between a lane's last code and the next lane are zero, and
 * that the stream ends, after zero bits only, at the first multiple of 16
 * bytes.                                                                   */
static int decode_stream(const uint8_t *stream, size_t n_bytes, uint32_t n,
                         const uint8_t len[256], const uint16_t code[256],
                         int L, uint32_t q, int pad, uint8_t *e)
{
    const uint32_t tiles = (n + ZO_TILE - 1) / ZO_TILE;
    const uint32_t m = tiles * ZO_RUN;
    if (n_bytes < ZO_LANES || n_bytes % 16) return ZO_E_FORMAT;
    const uint8_t *payload = stream + ZO_LANES;
    const uint64_t payload_bits = (uint64_t)(n_bytes - ZO_LANES) * 8;
    uint64_t at = 0;
    for (uint32_t lane = 0; lane < ZO_LANES; lane++) {
        const uint64_t D = m + (uint64_t)q * stream[lane];
        if (at + D > payload_bits) return ZO_E_FORMAT;
        /* lo: next bit of the first half (moving up); hi: one past the next bit of the second half (moving down) */
        uint64_t lo = at, hi = at + D;
        for (uint32_t step = 0; step < m; step++) {
            const int up = step < m / 2;
            const uint32_t j = up ? step : m - 1 - (step - m / 2);
            /* walk the code one bit at a time until it equals a code of the book */
            uint32_t acc = 0; int l = 0, found = -1;
            while (found < 0 && l < L) {
                if (lo >= hi) return ZO_E_FORMAT;             /* the two halves may not run into each other */
                acc = (acc << 1) | get_bit(payload, up ? lo++ : --hi);
                l++;
                for (int s = 0; s < 256; s++)
                    if (len[s] == l && code[s] == acc) { found = s; break; }
            }
            if (found < 0) return ZO_E_FORMAT;
            uint32_t idx = (j / ZO_RUN) * ZO_TILE + lane * ZO_RUN + (j % ZO_RUN);
            if (idx < n) e[idx] = (uint8_t)found;
            else if (found != pad) return ZO_E_FORMAT;
        }
        if (hi - lo >= q) return ZO_E_FORMAT;                /* a smaller byte would have done */
        for (uint64_t k = lo; k < hi; k++) if (get_bit(payload, k)) return ZO_E_FORMAT;
        at += D;
    }
    if (n_bytes != round_up(ZO_LANES + (at + 7) / 8, 16)) return ZO_E_FORMAT;
    for (uint64_t k = at; k < payload_bits; k++) if (get_bit(payload, k)) return ZO_E_FORMAT;
    return ZO_OK;
}

/* ---- the serialised tensor --------------------------------------------- */
/*
 * byte 0    header, 128 bytes (fields at the H_* offsets, the rest zero)
 * byte 128  code_len[256]: code length of every exponent value, 0 = absent
 *           (canonical codes follow from the lengths)
 * byte 384  decode table: 2^L entries of 16 bits, L = longest code length
 *           (at least 1).  Entry x describes the code that the L stream bits
 *           x (bit 0 = first wire bit) begin with: low byte = symbol, high
 *           byte = its length.  Bit patterns that begin with no code (only
 *           when fewer than two symbols are present) name the pad symbol
 *           with length 1.
 * then      chunk table, 16-byte aligned: n_chunks+1 entries of `stride`
 *           bytes, stride = 8 + 4*(C/W + 1) rounded up to a multiple of 8.
 *           Entry c: a 64-bit word = byte offset of E-chunk c from the start
 *           of the object (a multiple of 16) + the chunk's mode in the low 4
 *           bits; then 32-bit stream_off[0..S], the byte offsets of the
 *           chunk's S streams from the chunk start and, in stream_off[S], the
 *           chunk's length (all zero for a RAW chunk); then zeros.  The last
 *           entry holds the end offset of the last E-chunk, mode bits 0, and
 *           zeros.  One read of a table entry tells a decoder where a stream
 *           starts and ends.
 * then      SM section, 256-byte aligned: n_values sign-mantissa bytes in
 *           tensor order
 * then      E-chunks, the first 256-byte aligned, each 16-byte aligned.
 *           Chunk c covers values [c*C, min(n, (c+1)*C)).
 *             mode RAW:   the chunk's exponent bytes, zero padded to 16
 *             mode CODED: the chunk's S streams one after the other;
 *                         stream s covers values [s*W, (s+1)*W) of the chunk
 *           A chunk is stored RAW when its coded form would not be smaller.
 * The object's total size is a multiple of 256.
 */

/* bytes of one chunk-table entry */
static uint64_t table_stride(uint32_t C, uint32_t W) { return round_up(8 + 4 * ((uint64_t)(C / W) + 1), 8); }

size_t zo_encode_bound(size_t n_values, uint32_t chunk_values, uint32_t stream_values)
{
    size_t chunks = chunk_values ? (n_values + chunk_values - 1) / chunk_values : 0;
    size_t stride = (chunk_values && stream_values && chunk_values % stream_values == 0) ? (size_t)table_stride(chunk_values, stream_values) : 8;
    return 384 + 2 * 4096 + 16 + stride * (chunks + 1) + 256 + n_values + 256 + n_values + 16 * chunks + 512;
}

static int check_geometry(uint32_t C, uint32_t W)
{
    if (W == 0 || C == 0) return 0;
    if (W % ZO_TILE) return 0;
    if (C % W) return 0;
    return 1;
}

int zo_encode(const uint16_t *w, size_t n, uint32_t C, uint32_t W,
              const uint8_t len[256], uint8_t *blob, size_t cap, size_t *size_out)
{
    if (!check_geometry(C, W)) return ZO_E_ARG;
    if (zo_kraft_units(len) > (1u << ZO_MAX_LEN)) return ZO_E_ARG;
    if (cap < zo_encode_bound(n, C, W)) return ZO_E_SIZE;

    uint8_t *e = (uint8_t *)malloc(n ? n : 1), *sm = (uint8_t *)malloc(n ? n : 1);
    if (!e || !sm) { free(e); free(sm); return ZO_E_NOMEM; }
    zo_split(w, n, e, sm);
    for (size_t i = 0; i < n; i++) if (len[e[i]] == 0) { free(e); free(sm); return ZO_E_ARG; }

    uint16_t code[256];
    int n_present = zo_canonical(len, code);
    int L = max_code_len(len);
    int pad = pad_symbol(len);
    size_t K = (n + C - 1) / C;

    uint64_t len_off = ZO_HEADER_BYTES;
    uint64_t lut_off = len_off + 256;
    uint64_t table_off = round_up(lut_off + 2 * ((uint64_t)1 << L), 16);
    const uint64_t stride = table_stride(C, W);
    uint64_t sm_off = round_up(table_off + stride * (K + 1), 256);
    uint64_t e_off = round_up(sm_off + n, 256);

    memset(blob, 0, e_off);
    memcpy(blob + len_off, len, 256);
    /* decode table, by its definition: for every L-bit pattern find the code it begins with */
    for (uint32_t x = 0; x < (1u << L); x++) {
        int sym = pad, sl = 1;
        for (int s = 0; s < 256; s++) {
            if (!len[s]) continue;
            int match = 1;
            for (int b = 0; b < len[s]; b++) {
                uint32_t wire_bit = (x >> b) & 1u;
                uint32_t code_bit = (code[s] >> (len[s] - 1 - b)) & 1u;
                if (wire_bit != code_bit) { match = 0; break; }
            }
            if (match) { sym = s; sl = len[s]; break; }
        }
        blob[lut_off + 2 * x] = (uint8_t)sym;
        blob[lut_off + 2 * x + 1] = (uint8_t)sl;
    }
    memcpy(blob + sm_off, sm, n);

    const uint32_t q = lane_quantum(L, W);
    const size_t tmp_bytes = stream_bytes_bound(W);
    uint8_t *tmp = (uint8_t *)malloc(tmp_bytes);
    uint64_t pos = e_off;
    for (size_t c = 0; c < K; c++) {
        uint32_t cn = (uint32_t)((n - c * C) < C ? (n - c * C) : C);
        uint32_t S = (cn + W - 1) / W;
        uint64_t raw_bytes = round_up(cn, 16);
        /* coded form, built in place; the stream offsets go to the chunk's table entry */
        uint8_t *entry = blob + table_off + stride * c;
        uint64_t at = 0;
        uint8_t *base = blob + pos;
        int fits = 1;
        memset(entry, 0, stride);
        for (uint32_t s = 0; s < S && fits; s++) {
            uint32_t sn = (cn - s * W) < W ? (cn - s * W) : W;
            memset(tmp, 0, tmp_bytes);
            size_t nb = encode_stream(e + c * C + (size_t)s * W, sn, len, code, q, pad, tmp);
            put32(entry + 8 + 4 * s, (uint32_t)at);
            if (at + nb >= raw_bytes) { fits = 0; break; }
            memcpy(base + at, tmp, nb);
            at += nb;
        }
        if (fits && at < raw_bytes) {
            put32(entry + 8 + 4 * S, (uint32_t)at);
            put64(entry, pos | ZO_MODE_CODED);
            pos += at;
        } else {
            memset(entry, 0, stride);
            memset(base, 0, raw_bytes);
            memcpy(base, e + c * C, cn);
            put64(entry, pos | ZO_MODE_RAW);
            pos += raw_bytes;
        }
    }
    memset(blob + table_off + stride * K, 0, stride);
    put64(blob + table_off + stride * K, pos);
    uint64_t total = round_up(pos, 256);
    memset(blob + pos, 0, total - pos);

    put32(blob + H_MAGIC, ZO_MAGIC); put32(blob + H_VERSION, ZO_VERSION);
    put64(blob + H_NVALUES, n); put32(blob + H_CHUNK, C); put32(blob + H_STREAM, W);
    put32(blob + H_NCHUNKS, (uint32_t)K); put32(blob + H_L, (uint32_t)L);
    put32(blob + H_QUANTUM, q); put32(blob + H_NPRESENT, (uint32_t)n_present);
    put32(blob + H_PADSYM, (uint32_t)pad); put32(blob + H_TABLE_STRIDE, (uint32_t)stride);
    put64(blob + H_LEN_OFF, len_off); put64(blob + H_LUT_OFF, lut_off);
    put64(blob + H_TABLE_OFF, table_off); put64(blob + H_SM_OFF, sm_off);
    put64(blob + H_E_OFF, e_off); put64(blob + H_BLOB_SIZE, total);
    *size_out = total;
    free(tmp); free(e); free(sm);
    return ZO_OK;
}

/* number of values stored in a serialised tensor, or 0 if the header is bad */
uint64_t zo_blob_values(const uint8_t *blob, size_t size)
{
    if (size < ZO_HEADER_BYTES || get32(blob + H_MAGIC) != ZO_MAGIC) return 0;
    return get64(blob + H_NVALUES);
}

/* Decodes chunks [c0, c1) of a serialised tensor into out (indexed from the
 * tensor's first value: chunk c lands at out[c*C ...]).  Validates the
 * header, the codebook and every structure it walks.                       */
int zo_decode_chunks(const uint8_t *blob, size_t size, size_t c0, size_t c1, uint16_t *out)
{
    if (size < ZO_HEADER_BYTES) return ZO_E_FORMAT;
    if (get32(blob + H_MAGIC) != ZO_MAGIC || get32(blob + H_VERSION) != ZO_VERSION) return ZO_E_FORMAT;
    uint64_t n = get64(blob + H_NVALUES);
    uint32_t C = get32(blob + H_CHUNK), W = get32(blob + H_STREAM);
    uint64_t K = get32(blob + H_NCHUNKS);
    int L = (int)get32(blob + H_L);
    uint64_t len_off = get64(blob + H_LEN_OFF), lut_off = get64(blob + H_LUT_OFF);
    uint64_t table_off = get64(blob + H_TABLE_OFF), sm_off = get64(blob + H_SM_OFF);
    uint64_t e_off = get64(blob + H_E_OFF), total = get64(blob + H_BLOB_SIZE);
    if (!check_geometry(C, W)) return ZO_E_FORMAT;
    if (K != (n + C - 1) / C) return ZO_E_FORMAT;
    if (total > size || total % 256) return ZO_E_FORMAT;
    if (len_off != ZO_HEADER_BYTES || lut_off != len_off + 256) return ZO_E_FORMAT;
    if (L < 1 || L > ZO_MAX_LEN) return ZO_E_FORMAT;
    if (table_off != round_up(lut_off + 2 * ((uint64_t)1 << L), 16)) return ZO_E_FORMAT;
    const uint64_t stride = table_stride(C, W);
    if (get32(blob + H_TABLE_STRIDE) != stride) return ZO_E_FORMAT;
    if (sm_off != round_up(table_off + stride * (K + 1), 256)) return ZO_E_FORMAT;
    if (e_off != round_up(sm_off + n, 256) || e_off > total) return ZO_E_FORMAT;
    if (c0 > c1 || c1 > K) return ZO_E_ARG;

    const uint8_t *len = blob + len_off;
    if (zo_kraft_units(len) > (1u << ZO_MAX_LEN)) return ZO_E_FORMAT;
    if (max_code_len(len) != L) return ZO_E_FORMAT;
    const uint32_t q = lane_quantum(L, W);
    if (get32(blob + H_QUANTUM) != q) return ZO_E_FORMAT;
    uint16_t code[256];
    int n_present = zo_canonical(len, code);
    int pad = pad_symbol(len);
    if ((uint32_t)n_present != get32(blob + H_NPRESENT) || (uint32_t)pad != get32(blob + H_PADSYM)) return ZO_E_FORMAT;

    const uint8_t *sm = blob + sm_off;
    uint8_t *e = (uint8_t *)malloc(C);
    int rc = ZO_OK;
    for (uint64_t c = c0; c < c1 && rc == ZO_OK; c++) {
        const uint8_t *entry = blob + table_off + stride * c;
        uint64_t ent = get64(entry), nxt = get64(entry + stride);
        uint64_t at = ent & ~(uint64_t)15, end = nxt & ~(uint64_t)15;
        unsigned mode = (unsigned)(ent & 15);
        uint32_t cn = (uint32_t)((n - c * C) < C ? (n - c * C) : C);
        uint32_t S = (cn + W - 1) / W;
        if (at < e_off || end < at || end > total) { rc = ZO_E_FORMAT; break; }
        if (c == 0 && at != e_off) { rc = ZO_E_FORMAT; break; }
        const uint8_t *base = blob + at;
        /* unused offset slots of the entry are zero */
        for (uint64_t j = 8 + 4 * ((uint64_t)(mode == ZO_MODE_CODED ? S : 0) + (mode == ZO_MODE_CODED)); j < stride && rc == ZO_OK; j += 4)
            if (get32(entry + j) != 0) rc = ZO_E_FORMAT;
        if (rc != ZO_OK) break;
        if (mode == ZO_MODE_RAW) {
            if (end - at != round_up(cn, 16)) { rc = ZO_E_FORMAT; break; }
            memcpy(e, base, cn);
        } else if (mode == ZO_MODE_CODED) {
            if (get32(entry + 8) != 0 || get32(entry + 8 + 4 * S) != end - at) { rc = ZO_E_FORMAT; break; }
            for (uint32_t s = 0; s < S && rc == ZO_OK; s++) {
                uint32_t o0 = get32(entry + 8 + 4 * s), o1 = get32(entry + 8 + 4 * (s + 1));
                if (o0 % 16 || o1 % 16 || o1 < o0 || o1 > end - at) { rc = ZO_E_FORMAT; break; }
                uint32_t sn = (cn - s * W) < W ? (cn - s * W) : W;
                rc = decode_stream(base + o0, o1 - o0, sn, len, code, L, q, pad, e + (size_t)s * W);
            }
        } else rc = ZO_E_FORMAT;
        if (rc == ZO_OK) zo_merge(e, sm + c * C, cn, out + c * C);
    }
    if (rc == ZO_OK && c1 == K && get64(blob + table_off + stride * K) > total) rc = ZO_E_FORMAT;
    free(e);
    return rc;
}

int zo_decode(const uint8_t *blob, size_t size, uint16_t *out, size_t out_cap)
{
    if (size < ZO_HEADER_BYTES || get32(blob + H_MAGIC) != ZO_MAGIC) return ZO_E_FORMAT;
    if (out_cap < get64(blob + H_NVALUES)) return ZO_E_SIZE;
    return zo_decode_chunks(blob, size, 0, get32(blob + H_NCHUNKS), out);
}

/* Checks that the stored decode table is the one the code lengths define. */
int zo_check_table(const uint8_t *blob, size_t size)
{
    if (size < 384 || get32(blob + H_MAGIC) != ZO_MAGIC) return ZO_E_FORMAT;
    if (get64(blob + H_LEN_OFF) != ZO_HEADER_BYTES || get64(blob + H_LUT_OFF) != ZO_HEADER_BYTES + 256) return ZO_E_FORMAT;
    const uint8_t *len = blob + ZO_HEADER_BYTES;
    int L = (int)get32(blob + H_L);
    uint64_t lut_off = ZO_HEADER_BYTES + 256;
    if (L < 1 || L > ZO_MAX_LEN || lut_off + 2 * ((uint64_t)1 << L) > size) return ZO_E_FORMAT;
    uint16_t code[256];
    zo_canonical(len, code);
    int pad = pad_symbol(len);
    for (uint32_t x = 0; x < (1u << L); x++) {
        /* walk the bits of x as the decoder would */
        uint32_t acc = 0; int found = -1, l = 0;
        while (found < 0 && l < L) {
            acc = (acc << 1) | ((x >> l) & 1u); l++;
            for (int s = 0; s < 256; s++) if (len[s] == l && code[s] == acc) { found = s; break; }
        }
        int sym = found >= 0 ? found : pad, sl = found >= 0 ? l : 1;
        if (blob[lut_off + 2 * x] != sym || blob[lut_off + 2 * x + 1] != sl) return ZO_E_FORMAT;
    }
    return ZO_OK;
}
