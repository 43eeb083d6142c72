/*
 * zipmoe.h -- C ABI of libzipmoe: lossless compression of bf16 MoE expert
 * weights on the host, and their decompression on an MI355X (gfx950).
 *
 * The method is that of ZipMoE (arXiv 2601.21198):
 *   Sec. 2.2  a bf16 word is 1 sign bit, 8 exponent bits, 7 mantissa bits; the
 *             exponent field has only about 2.6 bits of entropy.
 *   Sec. 3.1  offline initialisation: every tensor is split into exponent bits
 *             and sign-mantissa bits; the exponent bits are cut into shards that
 *             are compressed one by one ("E-chunks"); the sign-mantissa bits are
 *             packed one byte per value ("SM-chunks"); all of it, plus metadata,
 *             is serialised into one binary object.
 *   Sec. 3.3  "Memory-Coalesced Tensor Recovery Kernel": exponent bytes and
 *             sign-mantissa bytes are merged back into bf16 words with
 *             vectorised, coalesced loads and stores.
 *   Sec. 6    "Other Compressors": the E-chunk compressor is a pluggable
 *             backend.  The backend of this library is a canonical prefix code
 *             with one codebook per tensor whose decoder runs on the GPU, so
 *             decompression and recovery are one kernel launch.
 *
 * Conventions
 *   - Every function returns an int status: ZM_OK or a negative ZM_E_* code,
 *     unless stated otherwise.  No function throws, none keeps global state,
 *     and none but the zm_cache object (which says so) keeps a pointer it was
 *     given.  Functions are thread-safe as long as concurrent calls write
 *     distinct outputs.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device memory of the current device.  The caller owns every buffer.
 *   - bf16 values are passed as their 16-bit patterns (uint16_t), row-major.
 *
 * Serialised tensor ("blob"), all integers little-endian:
 *   byte 0     header, 128 bytes (see zm_tensor_info for the fields it carries)
 *   byte 128   code_len[256]: code length of every exponent value, 0 = absent
 *   byte 384   decode table, 2^L 16-bit entries (L = longest code length): the
 *              entry for an L-bit stream window is symbol | length << 8
 *   then       chunk table: n_chunks+1 entries of table_stride bytes
 *              (8 + 4*(chunk_values/stream_values + 1), rounded up to a
 *              multiple of 8): a 64-bit word = byte offset of the E-chunk in
 *              the blob (multiple of 16) | mode in the low 4 bits, then the
 *              32-bit byte offsets of the chunk's streams from the chunk start
 *              followed by the chunk's length (zeros for a raw chunk); the last
 *              entry holds the end offset
 *   then       SM section (256-byte aligned): n_values sign-mantissa bytes
 *              (sign in bit 7, mantissa in bits 6..0), tensor order
 *   then       E-chunks (first one 256-byte aligned, each 16-byte aligned);
 *              chunk c covers values [c*chunk_values, (c+1)*chunk_values).
 *              mode 1 (raw): the exponent bytes.  mode 0 (coded): the chunk's
 *              streams one after the other.
 *              A stream covers stream_values consecutive values, cut into
 *              tiles of 512; in every tile lane j of 64 owns values 8j..8j+7.
 *              A lane has m symbols (8 per tile, tile after tile; positions
 *              past the stream's end hold the first symbol in canonical order)
 *              and a bitstream of D = m + q*b bits, b the smallest byte that
 *              fits their codes.  The bitstream is filled from both ends: the
 *              codes of symbols 0..m/2-1 upwards from its first bit, first
 *              code bit first; the codes of symbols m-1 down to m/2 downwards
 *              from its last bit (symbol m-1's first code bit is the lane's
 *              last bit, the next code bit the one below it); the bits in
 *              between are zero.  A decoder can so run two independent chains
 *              per lane.  The stream is the 64 bytes b (lane 0 first),
 *              then the 64 bitstreams back to back with no gap (payload bit k
 *              is bit k%32 of the little-endian 32-bit word k/32), then zero
 *              bits to a multiple of 16 bytes.  A prefix sum over the 64 bytes
 *              gives every lane's first bit and, with it, the lane before's
 *              last.  q, the header's lane_quantum, is
 *              the smallest integer >= 1 with (L-1)*(stream_values/64) <= 255*q.
 */
#ifndef ZIPMOE_H
#define ZIPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZM_OK        0
#define ZM_E_ARG    (-1)   /* null pointer, size or alignment that the call does not admit */
#define ZM_E_SIZE   (-2)   /* an output buffer is too small                                */
#define ZM_E_FORMAT (-3)   /* the blob is not a well-formed serialised tensor              */
#define ZM_E_HIP    (-4)   /* the HIP runtime reported an error (kept for hipGetLastError)  */
#define ZM_E_NOMEM  (-5)   /* host allocation failed                                       */

#define ZM_MAX_CODE_LEN 12   /* longest code length the format admits */
#define ZM_TILE_VALUES  512  /* stream_values must be a multiple of this */
#define ZM_MODE_CODED 0
#define ZM_MODE_RAW   1

/* What a decoder needs to know about one serialised tensor; filled by
 * zm_blob_info from the blob's header (the "metadata" of Sec. 3.1). */
typedef struct zm_tensor_info {
    uint64_t n_values;       /* bf16 values in the tensor                         */
    uint64_t blob_size;      /* bytes, a multiple of 256                          */
    uint64_t lut_offset;     /* byte offset of the decode table                   */
    uint64_t table_offset;   /* byte offset of the chunk table                    */
    uint64_t sm_offset;      /* byte offset of the SM section                     */
    uint64_t e_offset;       /* byte offset of the first E-chunk                  */
    uint32_t chunk_values;   /* values per E-chunk (the last chunk may be short)  */
    uint32_t stream_values;  /* values per stream inside a chunk                  */
    uint32_t n_chunks;
    uint32_t max_len;        /* L, longest code length in use (>= 1)              */
    uint32_t lane_quantum;   /* q: unit, in bits, of the per-lane length bytes    */
    uint32_t n_present;      /* exponent values that occur                        */
    uint32_t table_stride;   /* bytes of one chunk-table entry                    */
    uint32_t reserved;
} zm_tensor_info;

/* Library version as major*10000 + minor*100 + patch. Never fails. */
int zm_version(void);

/* Static, human-readable text for a status code. Never returns NULL. */
const char *zm_strerror(int status);

/* Histogram of the exponent field (Sec. 2.2) of n_values bf16 words.
 * host in: bf16; host out: hist[256].  ZM_E_ARG on null pointers. */
int zm_exponent_histogram(const uint16_t *bf16, size_t n_values, uint64_t hist[256]);

/* Codebook for the E-chunk backend (Sec. 3.1 "compressed", Sec. 6).
 * host in: hist[256], the exponent histogram of the tensor the codebook serves.
 * host out: code_len_out[256]: 0 for absent symbols, else 1..max_len, such that
 * sum 2^-len <= 1 and sum hist*len is the minimum possible under the limit
 * (an optimal length-limited prefix code).  One present symbol gets length 1.
 * max_len must be in 1..ZM_MAX_CODE_LEN and 2^max_len >= number of present
 * symbols, else ZM_E_ARG. */
int zm_build_codebook(const uint64_t hist[256], int max_len, uint8_t code_len_out[256]);

/* Upper bound on the size of the serialised object of Sec. 3.1 (all components plus their
 * metadata in one binary object) that zm_encode can produce for a tensor of n_values. 0 if the
 * geometry is not admissible (see zm_encode). */
size_t zm_encode_bound(size_t n_values, uint32_t chunk_values, uint32_t stream_values);

/* Offline initialisation of one tensor (Sec. 3.1): split, shard, encode, pack,
 * serialise.  Everything is host memory.
 *   bf16, n_values    the tensor, flattened row-major
 *   chunk_values      values per E-chunk; a multiple of stream_values
 *   stream_values     values per stream; a multiple of ZM_TILE_VALUES
 *   code_len          codebook from zm_build_codebook (must cover every
 *                     exponent value that occurs; sum 2^-len must be exactly 1
 *                     when two or more symbols are present, so that every bit
 *                     pattern decodes)
 *   blob, blob_cap    output buffer, at least zm_encode_bound(...) bytes
 *   blob_size         out: bytes written (a multiple of 256)
 *   chunk_offsets, chunk_offsets_cap   optional (may be NULL/0) copy of the
 *                     blob's chunk table, (n_chunks+1) * table_stride/8 64-bit
 *                     words (capacity counted in such words)
 *   n_chunks          out (may be NULL)
 * The output is a function of the inputs alone: equal inputs give equal bytes.
 * ZM_E_ARG for bad geometry, bad codebook or a symbol without a code;
 * ZM_E_SIZE if a buffer is too small; ZM_E_NOMEM. */
int zm_encode(const uint16_t *bf16, size_t n_values, uint32_t chunk_values, uint32_t stream_values,
              const uint8_t code_len[256], uint8_t *blob, size_t blob_cap, size_t *blob_size,
              uint64_t *chunk_offsets, size_t chunk_offsets_cap, size_t *n_chunks);

/* The metadata that Sec. 3.1 serialises with the compressed components: reads and
 * checks the header and codebook of a blob in host memory (size may be just the first
 * 384 bytes or the whole blob) and fills *info.
 * ZM_E_FORMAT if magic, version, geometry, section offsets or codebook are
 * not consistent. */
int zm_blob_info(const void *blob_host, size_t size, zm_tensor_info *info);

/* Full structural check of a serialised tensor (the binary object of Sec. 3.1) in host
 * memory, to be run once when a blob is registered, before it is uploaded: header, codebook, decode table against
 * the codebook, chunk table, every chunk header and stream offset, every
 * address a decoder will touch inside blob_size.  ZM_E_FORMAT on any
 * violation.  It does not decode the streams. */
int zm_validate_blob(const void *blob_host, size_t size);

/* The hot call (Sec. 3.1 "Real-time Inference", steps 5-8, for experts whose
 * compressed form is resident; Sec. 3.3 recovery): decode the experts a MoE
 * layer's gate selected, in one kernel launch per 48 tensors of a code-table width class (codes of at most 8
 * bits, longer codes).
 *
 *   blobs             host array [n_experts * tensors_per_expert] of DEVICE
 *                     pointers; entry e*tensors_per_expert + m is tensor m of
 *                     expert e; each 16-byte aligned, uploaded unchanged from
 *                     zm_encode's output
 *   chunk_offsets     host array, same shape, of DEVICE pointers to each
 *                     tensor's chunk table ((n_chunks+1) * table_stride bytes;
 *                     may point into the blob at table_offset)
 *   infos             host array, same shape, from zm_blob_info
 *   n_experts, tensors_per_expert
 *   expert_ids        host array [n_selected], each in [0, n_experts);
 *                     duplicates are legal and are decoded twice
 *   out_bf16          host array [n_selected * tensors_per_expert] of DEVICE
 *                     pointers; entry j*tensors_per_expert + m receives the
 *                     n_values bf16 words of tensor m of expert expert_ids[j];
 *                     each 16-byte aligned and distinct
 *   stream            a hipStream_t (NULL = the default stream)
 *
 * Asynchronous: enqueues the launches on `stream` and returns; allocates
 * nothing, copies nothing, does not synchronise.  All arguments travel as
 * kernel arguments, so host arrays may be reused as soon as the call returns;
 * device buffers must stay valid until the stream has passed the call.  For
 * the same reason the call may be recorded on a capturing stream and replayed
 * from the HIP graph: it records kernel launches and nothing else.
 * Blobs must have passed zm_validate_blob: the kernel confines every access to
 * the sizes in `infos`, it does not re-validate the streams.
 * At most 256 tensors (n_selected * tensors_per_expert) per call.
 * ZM_E_ARG for null pointers, ids out of range, misaligned pointers, too many
 * tensors or a stream length the decoder cannot stage; ZM_E_HIP if a launch
 * fails. */
int zm_decode_experts(const void *const *blobs, const uint64_t *const *chunk_offsets,
                      const zm_tensor_info *infos, int n_experts, int tensors_per_expert,
                      const int32_t *expert_ids, int n_selected,
                      void *const *out_bf16, void *stream);


/* The same call with the store policy chosen by the caller, who knows what becomes of the output buffers:
 *   ZM_STORES_AUTO       what zm_decode_experts does: non-temporal stores iff one launch writes more than the
 *                        256 MB last-level cache holds
 *   ZM_STORES_CACHED     ordinary stores: right when the same buffers are rewritten call after call (the lines
 *                        are still in the last-level cache and never travel to HBM) or are read at once
 *   ZM_STORES_STREAMING  non-temporal stores: right when the buffers are not cache-resident (fresh or rotating
 *                        buffers): nothing is left in the L2 caches to be written back when the kernel ends
 * ZM_E_ARG for any other value. */
#define ZM_STORES_AUTO      0
#define ZM_STORES_CACHED    1
#define ZM_STORES_STREAMING 2
int zm_decode_experts_stores(const void *const *blobs, const uint64_t *const *chunk_offsets,
                             const zm_tensor_info *infos, int n_experts, int tensors_per_expert,
                             const int32_t *expert_ids, int n_selected,
                             void *const *out_bf16, int stores, void *stream);


/* ---- A layer's resident experts as one handle (Sec. 3.1: the serialised objects made offline are what the
 * run-time system keeps).  The handle holds what zm_decode_experts takes as arrays, so the hot call names
 * expert ids and output buffers only.  It owns no device memory. ---- */
typedef struct zm_layer zm_layer;

/* Device bytes the blobs of a layer occupy: their sizes, each rounded up to 256.  blob_sizes: host array
 * [n_tensors].  ZM_E_ARG on null pointers, n_tensors <= 0 or overflow. */
int zm_layer_arena_bytes(const size_t *blob_sizes, int n_tensors, size_t *bytes);

/* Registers a layer: checks every blob with zm_validate_blob, then copies them into `arena` (DEVICE memory of at
 * least zm_layer_arena_bytes bytes, 256-byte aligned, owned by the caller and in use until zm_layer_destroy)
 * with synchronous copies.  host_blobs, blob_sizes: host arrays [n_experts * tensors_per_expert], entry
 * e*tensors_per_expert + m is tensor m of expert e; the host blobs are not needed after the call.
 * ZM_E_ARG, ZM_E_SIZE (arena too small), ZM_E_FORMAT (a blob fails the check; nothing was uploaded),
 * ZM_E_NOMEM, ZM_E_HIP. */
int zm_layer_create(const void *const *host_blobs, const size_t *blob_sizes, int n_experts, int tensors_per_expert,
                    void *arena, size_t arena_bytes, zm_layer **layer_out);

/* Description of tensor `tensor` of expert `expert` and, if device_blob_out is not NULL, the device address
 * of its blob.  ZM_E_ARG on bad indices. */
int zm_layer_tensor_info(const zm_layer *layer, int expert, int tensor, zm_tensor_info *info_out,
                         const void **device_blob_out);

/* zm_decode_experts_stores on the layer's experts: expert_ids, n_selected, out_bf16, stores and stream as
 * there, same limits and errors; asynchronous, allocates nothing. */
int zm_layer_decode(const zm_layer *layer, const int32_t *expert_ids, int n_selected, void *const *out_bf16,
                    int stores, void *stream);

/* Frees the handle's host memory; the arena goes back to the caller (who waits for pending decodes before
 * reusing it).  NULL is allowed. */
void zm_layer_destroy(zm_layer *layer);


/* What a decode call for the tensors infos[0..n_tensors) would launch, by the rule the decode calls use
 * themselves and without launching anything (for benchmarks and profiles that have to name the kernel):
 * one entry per kernel launch, in launch order.  Host only. */
typedef struct zm_launch_shape {
    uint32_t round_symbols;        /* symbols a lane decodes per 32-bit window: 4 (codes <= 8 bits) or 2   */
    uint32_t waves_per_workgroup;  /* streams that share a workgroup                                       */
    uint32_t streaming_stores;     /* 1: non-temporal stores                                               */
    uint32_t workgroups;           /* grid x: workgroups of the largest tensor of the launch               */
    uint32_t tensors;              /* grid y                                                               */
    uint32_t lds_bytes;            /* LDS of one workgroup                                                 */
} zm_launch_shape;
/* shapes_out holds shapes_cap entries (may be NULL with 0); *n_shapes receives the number of launches, which
 * may exceed shapes_cap.  ZM_E_ARG as for the decode calls. */
int zm_decode_launch_shapes(const zm_tensor_info *infos, int n_tensors, int stores,
                            zm_launch_shape *shapes_out, int shapes_cap, int *n_shapes);


/* One tensor given by its parts instead of by one blob, for callers that keep
 * only some parts of a tensor resident (Sec. 3.2 "Compression States": the
 * E-chunks and the SM-chunks of an expert may be cached separately).  All four
 * are DEVICE pointers to verbatim copies of byte ranges of the blob. */
typedef struct zm_tensor_parts {
    const void *table;          /* decode table: blob bytes [lut_offset, table_offset); 16-byte aligned  */
    const void *chunk_offsets;  /* chunk table: blob bytes [table_offset, table_offset + table_stride*(n_chunks+1)) */
    const void *sm;             /* SM section: blob bytes [sm_offset, e_offset); 16-byte aligned          */
    const void *echunks;        /* E-chunks: blob bytes [e_offset, blob_size); 16-byte aligned            */
} zm_tensor_parts;

/* Same decode as zm_decode_experts for an explicit list of tensors:
 * parts[i], infos[i] (host arrays) describe tensor i, out_bf16[i] (host array
 * of DEVICE pointers, 16-byte aligned) receives its n_values bf16 words.
 * At most 256 tensors per call.  Asynchronous on `stream`, allocates nothing.
 * ZM_E_ARG for null or misaligned pointers or inconsistent infos; ZM_E_HIP. */
int zm_decode_tensors(const zm_tensor_parts *parts, const zm_tensor_info *infos, int n_tensors,
                      void *const *out_bf16, void *stream);

/* Measurement aid (no part of the decode path): a plain streaming kernel that reads read_bytes from src
 * and writes write_bytes to dst (both DEVICE, 16-byte aligned, sizes multiples of 16, write_bytes >= 16)
 * with 128-bit vectors, ordinary or non-temporal stores.  pieces_per_lane = 1: one vector per lane and
 * direction, the finest grain; 8: eight per lane, all loads before the first store, which is what one
 * wavefront of the decode kernel moves for a stream of 4096 values.  Timed on a launch of the decode call's
 * size and read/write mix it gives the practical ceiling of this machine's memory system that the decode
 * kernel's fraction of the HBM roofline is set against.  Asynchronous on `stream`.
 * ZM_E_ARG for null or misaligned pointers, bad sizes or another pieces_per_lane; ZM_E_HIP if the launch
 * fails. */
int zm_mover_probe(const void *src, void *dst, size_t read_bytes, size_t write_bytes, int pieces_per_lane,
                   int streaming_stores, void *stream);

/* For callers that can not allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc -- and have the serialised tensors in HOST memory: the same decode as
 * zm_decode_tensors, with the compressed bytes staged in a fixed device array that belongs to the library
 * (ZM_STAGING_BYTES bytes per device, held from the first call on that device until the process ends)
 * instead of a caller-provided arena as in zm_cache_fetch.
 *   host_blobs  host array [n_tensors] of HOST pointers to validated blobs (pinned memory makes the copies
 *               asynchronous); infos[i] from zm_blob_info; out_bf16[i] a DEVICE pointer, 16-byte aligned,
 *               that receives tensor i's n_values bf16 words.  At most 256 tensors.
 * On `stream` it enqueues one host-to-device copy per tensor (the blob from its decode table on) and the
 * decode launches; it calls no allocating routine.  The host blobs must stay unchanged until the stream
 * has passed the call.  All calls on one device share that device's staging area: calls on different
 * streams (or threads) that can overlap in time race and must be serialised by the caller; calls on one
 * stream are ordered by the stream.  Nothing in the area needs clearing: every byte a launch reads was
 * written by that call's copies.
 * ZM_E_SIZE if the blobs of one call add up to more than ZM_STAGING_BYTES; ZM_E_ARG for null pointers,
 * inconsistent infos or too many tensors; ZM_E_HIP if the runtime refuses the symbol lookup, a copy or a
 * launch. */
#define ZM_STAGING_BYTES (32u << 20)
int zm_decode_host_tensors(const void *const *host_blobs, const zm_tensor_info *infos, int n_tensors,
                           void *const *out_bf16, void *stream);

/* ---- Compression-aware expert cache (Sec. 3.2, Sec. 3.4, Sec. 6) --------------
 * One cache serves one MoE layer.  HBM is partitioned into four pools, ordered
 * F < C < S < E: F keeps recovered bf16 tensors, C keeps E-chunks and SM-chunks,
 * S keeps SM-chunks, E keeps E-chunks.  Whatever an expert's pool does not hold
 * is fetched from the host copy of its blobs (Sec. 6: host memory is the tier
 * below device memory) with asynchronous copies that overlap the decode of the
 * experts that need none.  Every fetch counts one activation of each named
 * expert; an expert whose rank r in the activation counts (0 = most activated,
 * ties to the lower id) satisfies r < tau_i = slots[0] + .. + slots[i] +
 * tolerance is dispatched to the first such pool i (pools of capacity 0 are
 * skipped); if that pool is better than the one it is in, it moves there, taking
 * a free slot or evicting the pool's least activated member (never one named by
 * the same fetch, never one activated more often than itself); an expert that
 * qualifies for no pool is not kept.  An access never demotes. */
#define ZM_POOL_FULL       0
#define ZM_POOL_COMPRESSED 1
#define ZM_POOL_SM         2
#define ZM_POOL_E          3
#define ZM_POOL_NONE       4

typedef struct zm_cache zm_cache;

typedef struct zm_cache_config {
    int32_t n_experts;
    int32_t tensors_per_expert;
    int32_t slots[4];        /* capacities S_F, S_C, S_S, S_E in experts (Sec. 3.4)              */
    int32_t tolerance;       /* the tolerance margin delta of the rank thresholds (Sec. 3.4)       */
    int32_t max_selected;    /* most experts one fetch may name; max_selected*tensors_per_expert <= 256 */
} zm_cache_config;

/* The pool the dispatch rule assigns to `expert` given the activation counts
 * (host array of n_experts): ZM_POOL_FULL .. ZM_POOL_E, or ZM_POOL_NONE.  A pure
 * function of its arguments.  ZM_E_ARG (negative) on bad arguments. */
int zm_cache_dispatch(const uint64_t *counts, int n_experts, const int32_t slots[4], int tolerance, int expert);

/* Bytes of device memory a cache with this configuration needs.  infos: host
 * array [n_experts * tensors_per_expert] from zm_blob_info. */
int zm_cache_arena_bytes(const zm_cache_config *config, const zm_tensor_info *infos, size_t *bytes);

/* Bytes of one expert's packed host image (below). */
int zm_cache_image_bytes(const zm_cache_config *config, const zm_tensor_info *infos, size_t *bytes);

/* Packs what the cache ever copies of one expert -- the SM sections of its
 * tensors, then their E-chunk regions, laid out as in a pool slot -- into
 * `image` (HOST memory of zm_cache_image_bytes bytes, pinned for asynchronous
 * copies).  With such images a fetch moves an expert's missing parts with one
 * copy (both parts) or one per part instead of one per tensor and part; each
 * host-to-device copy has a fixed cost of some 10 us.  host_blobs: as for
 * zm_cache_create.  ZM_E_ARG, ZM_E_SIZE. */
int zm_cache_pack_expert(const zm_cache_config *config, const zm_tensor_info *infos, const void *const *host_blobs,
                         int expert, void *image, size_t image_bytes);

/* Creates a cache.  host_blobs: host array [n_experts * tensors_per_expert] of
 * HOST pointers to the validated blobs.  host_images: NULL, or host array
 * [n_experts] of images made by zm_cache_pack_expert.  Without images the blobs
 * are what fetches copy from (pinned memory makes the copies asynchronous) and
 * must stay valid for the life of the cache; with images the images must, and
 * the blobs are only read during this call.  arena: DEVICE
 * memory of at least zm_cache_arena_bytes bytes, 256-byte aligned, owned by the
 * caller and used by the cache until zm_cache_destroy.  The decode tables and
 * chunk tables of all tensors are uploaded at once (the call returns when they
 * are resident); all pools start empty.  The cache creates one HIP stream and two
 * events of its own and allocates no device memory.
 * ZM_E_ARG, ZM_E_SIZE (arena too small), ZM_E_NOMEM, ZM_E_HIP. */
int zm_cache_create(const zm_cache_config *config, const void *const *host_blobs, const void *const *host_images,
                    const zm_tensor_info *infos,
                    void *arena, size_t arena_bytes, zm_cache **out);

/* Makes the bf16 tensors of the named experts available and tells where they are.
 *   expert_ids   host array [n_selected] of distinct ids, n_selected <= max_selected
 *   out_bf16     host array [n_selected * tensors_per_expert], receives DEVICE
 *                pointers (16-byte aligned) to each tensor's n_values bf16 words
 *   found_in     optional host array [n_selected]: the pool each expert was found
 *                in (ZM_POOL_*), before this fetch moved it
 *   stream       the hipStream_t the caller will read the tensors on
 * Asynchronous: the tensors are complete once `stream` has passed the call.
 * Pointers into the F pool stay valid until a later fetch evicts that expert;
 * all other pointers are valid until the next fetch on this cache.  Work the
 * caller queued on `stream` before the call (readers of earlier results) is
 * waited for before anything is overwritten.  Not thread-safe per cache.
 * ZM_E_ARG for bad ids, duplicates or too many experts (the cache is unchanged);
 * ZM_E_HIP if a copy, an event or a launch fails: the pools may then disagree
 * with the bookkeeping, so every later fetch on this cache returns ZM_E_HIP too
 * and the cache can only be destroyed. */
int zm_cache_fetch(zm_cache *cache, const int32_t *expert_ids, int n_selected, void **out_bf16,
                   int32_t *found_in, void *stream);

/* The pool `expert` is in now (ZM_POOL_*), or ZM_E_ARG. */
int zm_cache_pool_of(const zm_cache *cache, int expert);

/* Waits for the cache's own stream, destroys it and the events, frees host
 * bookkeeping.  The arena goes back to the caller.  NULL is allowed. */
void zm_cache_destroy(zm_cache *cache);

/* ---- Cache-pool planning (Sec. 3.4 "Hierarchical Cache Planning", App. C, App. D) ----
 * Host only, double precision.  Ranks are 0-based here: entry 0 of a rank-based
 * list belongs to the most activated expert. */

/* Profiled delays and shape constants of the makespan estimate (App. C, Alg. 3). */
typedef struct zm_plan_costs {
    double decompress_delay;   /* c: decompression of one E-chunk                 */
    double e_read_delay;       /* v: read of one E-chunk from the tier below      */
    double sm_read_delay;      /* u: read of one SM-chunk (one tensor's SM bytes) */
    int32_t threads;           /* L: parallel decompression workers               */
    int32_t shards_per_tensor; /* K                                               */
    int32_t tensors_per_expert;/* n                                               */
} zm_plan_costs;

/* App. D, modified iterative proportional fitting.  f[n]: rank-based inclusion
 * probabilities (each in [0,1], sum = k).  q_out[n]: selection probabilities of
 * independent draws whose distribution, conditioned on exactly k selections,
 * includes rank i with probability f[i].  Starts from weights w = f and
 * multiplies w_i by f_i / f_i(w) until max |f_i(w) - f_i| < tol or max_iters;
 * iters_out (may be NULL) receives the iterations used.  ZM_E_ARG, ZM_E_NOMEM. */
int zm_plan_selection_probabilities(const double *f, int n, int k, int max_iters, double tol, double *q_out, int *iters_out);

/* App. C, Alg. 2: phi_out[h], h = 0..n: probability that exactly h of n
 * independent selections with probabilities q[n] occur. */
int zm_plan_hit_distribution(const double *q, int n, double *phi_out);

/* App. C, Alg. 3: estimated makespan of a sparse layer that activates k experts
 * of which hits[0..3] are found in pools F, C, S, E:
 * max(SM reads * u + E reads * v, (E reads * v + decompressions * c) / L). */
int zm_plan_makespan(int k, const int32_t hits[4], const zm_plan_costs *costs, double *makespan_out);

/* Expected makespan when the pools hold the rank intervals of sizes slots[0..3]
 * one after the other (the remaining ranks are misses), under the hit-pattern
 * distribution of Sec. 3.4 conditioned on exactly k selections. */
int zm_plan_expected_makespan(const double *q, int n_experts, const int32_t slots[4], int k, const zm_plan_costs *costs,
                              double *cost_out);

/* App. C, Alg. 4: grid search over the memory ratios of the pools (step 1/grid,
 * ratios sum to 1, only pools whose bit is set in pool_mask -- bit 0 = F .. bit 3
 * = E -- may get memory).  A pool with ratio r holds floor(r * memory_bytes /
 * bytes_per_expert[pool]) experts, at most the ranks left by the pools before
 * it.  Configurations are visited in lexicographic order of the (F, C, S, E) grid
 * counts and replace the best one only if strictly cheaper.  Outputs the best
 * ratios, their slot counts (ready for zm_cache_config.slots) and the expected
 * makespan. */
int zm_plan_pools(const double *f, int n_experts, int k, const zm_plan_costs *costs, double memory_bytes,
                  const double bytes_per_expert[4], int grid, int pool_mask,
                  double ratios_out[4], int32_t slots_out[4], double *cost_out);

/* ---- The paper's own split of the work (Sec. 3.1 step 7, Sec. 3.3): E-chunks
 * are decompressed by L CPU worker threads, the GPU only runs the recovery
 * kernel.  These two calls provide that path next to the fused one. ---- */

/* Decompresses E-chunks [chunk_begin, chunk_end) of a blob in host memory into
 * exponent bytes, one per value, with n_threads worker threads (the paper's L;
 * values < 1 are taken as 1).  e_out (host) is indexed from the tensor's first
 * value: chunk c is written to e_out[c*chunk_values ...]; it must hold
 * n_values bytes.  The blob must have passed zm_validate_blob.
 * ZM_E_ARG for null pointers or a bad chunk range, ZM_E_FORMAT if the header
 * or a chunk is malformed, ZM_E_NOMEM. */
int zm_decode_exponents_host(const void *blob_host, size_t size, uint32_t chunk_begin, uint32_t chunk_end,
                             uint8_t *e_out, int n_threads);

/* Tensor recovery kernel (Sec. 3.3): merges n_values exponent bytes and
 * n_values sign-mantissa bytes (both DEVICE, 8-byte aligned) into n_values bf16
 * words (DEVICE, 16-byte aligned) with vector loads and stores:
 * word = sign << 15 | exponent << 7 | mantissa.  Asynchronous on `stream`
 * (a hipStream_t), allocates nothing.  Tensors of more than 32 Mi values are
 * written with non-temporal stores (they do not stay in the last-level cache).  ZM_E_ARG for null or misaligned
 * pointers, ZM_E_HIP if the launch fails. */
int zm_recover(const void *exponents, const void *sign_mantissa, size_t n_values, void *out_bf16, void *stream);

/* ---- Cache-affinity scheduling of one sparse layer's reconstruction tasks
 * (Sec. 3.3 "Cache-Affinity Scheduler", App. A; analysis in App. B).  Host only,
 * double precision.  The machine model is the paper's: one I/O thread, L
 * decompression threads, one GPU stream.  A task is one tensor of one selected
 * expert; it reads K E-chunks (each `e_read`) and/or one SM-chunk (`sm_read`)
 * if they are not in memory, decompresses K E-chunks (each `decompress`, one
 * thread each, ready when that E-chunk has arrived), is recovered on the GPU
 * stream (`recover`) when all of that is done, and the expert runs for
 * expert_time[expert] on the GPU stream once all its tensors are recovered.
 * The makespan is the end of the last execution. ---- */

typedef struct zm_sched_task {
    int32_t expert;        /* n(j): index into expert_time */
    int32_t needs_sm;      /* the SM-chunk must be read: the task is Type-I */
    int32_t needs_e;       /* the E-chunks must be read */
    int32_t needs_decode;  /* 0: the tensor is held in full, no operation but the execution */
} zm_sched_task;

typedef struct zm_sched_costs {
    double sm_read;        /* u */
    double e_read;         /* rho * u / K */
    double decompress;     /* c */
    double recover;        /* per tensor on the GPU stream; 0 gives the paper's model */
    int32_t threads;       /* L >= 1 */
    int32_t shards;        /* K >= 1 */
} zm_sched_costs;

#define ZM_OP_E_READ 0
#define ZM_OP_SM_READ 1
#define ZM_OP_DECOMPRESS 2
#define ZM_OP_RECOVER 3
#define ZM_OP_EXECUTE 4

typedef struct zm_sched_event {
    int32_t kind;          /* ZM_OP_* */
    int32_t task;          /* task index; the expert index for ZM_OP_EXECUTE */
    int32_t chunk;         /* E-chunk index for reads of E-chunks and decompressions, else 0 */
    int32_t unit;          /* decompression thread for ZM_OP_DECOMPRESS, else 0 */
    double start;
    double end;
} zm_sched_event;

typedef struct zm_sched_result {
    double makespan;       /* end of the last operation on the GPU stream */
    double io_end;         /* end of the last read */
    double charge;         /* App. B: total idle time in front of decompressions on their threads */
} zm_sched_result;

/* App. A, Alg. 1: builds the blocks.  Type-I and Type-II tasks are each sorted
 * by non-increasing expert_time (ties: expert index, then task index).  A block
 * starts with the first Type-I task left; until it is compute-dominant (the l-th
 * earliest decompression thread ends at least l * e_read after the I/O thread,
 * l = 1..min(L, K)) the next task of (Type-II, then Type-I) goes to the earliest
 * position that does not increase the total charge, else behind the last task of
 * the block of the preferred class (Type-II if the block has one, else Type-I)
 * whose expert_time is not smaller, else to the end.  Type-II tasks left at the
 * end form a last block.  order_out[n_tasks]: task indices, highest priority
 * first; block b covers positions [block_end_out[b-1], block_end_out[b]) with
 * block_end_out[-1] = 0; block_end_out needs n_tasks entries.
 * ZM_E_ARG for null pointers, expert indices outside [0, n_experts), costs that
 * are negative or not finite, threads or shards < 1; ZM_E_NOMEM. */
int zm_sched_build(const zm_sched_task *tasks, int n_tasks, const double *expert_time, int n_experts,
                   const zm_sched_costs *costs, int32_t *order_out, int32_t *block_end_out, int *n_blocks_out);

/* App. A: runs the tasks named by order[0 .. block_end[n_blocks-1]) (distinct
 * task indices; tasks not named take no part) under work-conserving list
 * scheduling in that priority order.  The I/O thread reads, block after block,
 * the block's E-chunks in task order and then its SM-chunks in task order; a free
 * decompression thread (the lowest-numbered of those free) takes the first
 * decompression in (position, chunk) order whose E-chunk has arrived; the GPU
 * stream takes the first ready recovery or execution, an execution ranking right
 * behind its expert's last task.  result (may not be NULL) receives the totals,
 * worker_end_out (may be NULL, L entries) each thread's last end, events_out
 * (may be NULL) up to events_cap events in the order they were placed and
 * n_events_out (may be NULL) how many there are in all.
 * ZM_E_ARG as above and for a bad order; ZM_E_NOMEM. */
int zm_sched_simulate(const zm_sched_task *tasks, int n_tasks, const double *expert_time, int n_experts,
                      const zm_sched_costs *costs, const int32_t *order, const int32_t *block_end, int n_blocks,
                      zm_sched_result *result, double *worker_end_out,
                      zm_sched_event *events_out, size_t events_cap, size_t *n_events_out);

/* App. B, lower bounds on the makespan of any schedule: bounds_out[0] = total
 * read time, [1] = total decompression time / L, [2] = total execution time,
 * [3] = longest chain of one task (reads, decompression on min(L, K) threads,
 * recovery, its expert's execution). */
int zm_sched_lower_bounds(const zm_sched_task *tasks, int n_tasks, const double *expert_time, int n_experts,
                          const zm_sched_costs *costs, double bounds_out[4]);

#ifdef __cplusplus
}
#endif
#endif /* ZIPMOE_H */
