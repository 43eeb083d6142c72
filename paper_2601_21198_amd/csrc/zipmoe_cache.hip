// Compression-aware expert cache of one MoE layer on a discrete-memory GPU.
//
// Follows ZipMoE (arXiv 2601.21198):
//   Sec. 3.2  compression states: the E-chunks, the SM-chunks and the full tensors
//             of an expert are cached separately.
//   Sec. 3.4  cache pools F (full tensors) < C (E-chunks and SM-chunks) <
//             S (SM-chunks) < E (E-chunks); an expert whose activation-count rank
//             r satisfies r < tau_i = (capacities of the pools up to i) + delta
//             is dispatched to the first such pool i; a pool that overflows
//             evicts its least frequently activated member; an expert whose
//             rank passes every threshold is dropped right after execution.
//   Sec. 6    systems with dedicated device memory: host memory is the tier
//             below the pools, reached with asynchronous host-to-device copies.
//   App. C    which parts an expert in each state still has to fetch: SM-chunks
//             unless it is in F, C or S; E-chunks unless it is in F, C or E;
//             decompression unless it is in F.
//
// On MI355X the tier below HBM is (pinned) host memory.  Copies run on a stream
// of their own and overlap the decode of the experts that need none; the decode
// itself is zm_decode_tensors.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "zipmoe.h"

namespace {

constexpr int kPools = 4;                     // F, C, S, E
constexpr int kUncached = ZM_POOL_NONE;
inline size_t up256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }
inline size_t up16(size_t x) { return (x + 15) & ~static_cast<size_t>(15); }

struct Layout {
    // per tensor index m of an expert: offsets of its parts inside a slot of each kind
    std::vector<size_t> full_off, sm_off, e_off;
    size_t full_bytes = 0, sm_bytes = 0, e_bytes = 0;      // per expert
    std::vector<size_t> meta_off;                          // per (expert, tensor): decode table, then chunk table
    std::vector<size_t> meta_table_off;
    size_t meta_bytes = 0;
    size_t slot_bytes[kPools] = {0, 0, 0, 0};
    size_t pool_off[kPools] = {0, 0, 0, 0};
    size_t transient_off = 0, transient_bytes = 0;         // per selected expert: SM + E + full
    size_t total = 0;
};

bool make_layout(const zm_cache_config &c, const zm_tensor_info *infos, Layout &L)
{
    const int T = c.tensors_per_expert;
    L.full_off.assign(T, 0); L.sm_off.assign(T, 0); L.e_off.assign(T, 0);
    std::vector<size_t> full_cap(T, 0), sm_cap(T, 0), e_cap(T, 0);
    const size_t n = static_cast<size_t>(c.n_experts) * T;
    L.meta_off.assign(n, 0); L.meta_table_off.assign(n, 0);
    size_t meta = 0;
    for (size_t i = 0; i < n; ++i) {
        const zm_tensor_info &t = infos[i];
        if (t.e_offset > t.blob_size || t.sm_offset > t.e_offset || t.table_offset > t.sm_offset || t.lut_offset > t.table_offset)
            return false;
        const int m = static_cast<int>(i % T);
        full_cap[m] = std::max(full_cap[m], up256(2 * t.n_values));
        sm_cap[m] = std::max(sm_cap[m], up256(t.e_offset - t.sm_offset));
        e_cap[m] = std::max(e_cap[m], up256(t.blob_size - t.e_offset));
        L.meta_off[i] = meta;
        meta += up16(t.table_offset - t.lut_offset);
        L.meta_table_off[i] = meta;
        meta += up16(static_cast<size_t>(t.table_stride) * (t.n_chunks + 1));
    }
    L.meta_bytes = up256(meta);
    for (int m = 0; m < T; ++m) {
        L.full_off[m] = L.full_bytes; L.full_bytes += full_cap[m];
        L.sm_off[m] = L.sm_bytes; L.sm_bytes += sm_cap[m];
        L.e_off[m] = L.e_bytes; L.e_bytes += e_cap[m];
    }
    L.slot_bytes[ZM_POOL_FULL] = L.full_bytes;
    L.slot_bytes[ZM_POOL_COMPRESSED] = L.sm_bytes + L.e_bytes;      // SM parts first, then E parts
    L.slot_bytes[ZM_POOL_SM] = L.sm_bytes;
    L.slot_bytes[ZM_POOL_E] = L.e_bytes;
    size_t at = L.meta_bytes;
    for (int p = 0; p < kPools; ++p) { L.pool_off[p] = at; at += L.slot_bytes[p] * static_cast<size_t>(c.slots[p]); }
    L.transient_off = at;
    L.transient_bytes = L.sm_bytes + L.e_bytes + L.full_bytes;
    at += L.transient_bytes * static_cast<size_t>(c.max_selected);
    L.total = at;
    return true;
}

bool config_ok(const zm_cache_config *c)
{
    if (!c || c->n_experts <= 0 || c->tensors_per_expert <= 0 || c->max_selected <= 0 || c->tolerance < 0) return false;
    if (static_cast<long>(c->max_selected) * c->tensors_per_expert > 256) return false;
    for (int p = 0; p < kPools; ++p) if (c->slots[p] < 0) return false;
    return true;
}

// rank of `expert` in the activation counts: how many experts come before it when sorted by
// count, highest first, ties by lower id first
int rank_of(const uint64_t *counts, int n, int expert)
{
    int r = 0;
    for (int x = 0; x < n; ++x)
        if (counts[x] > counts[expert] || (counts[x] == counts[expert] && x < expert)) ++r;
    return r;
}

int dispatch_rank(int rank, const int32_t slots[kPools], int tolerance)
{
    long cum = 0;
    for (int p = 0; p < kPools; ++p) {
        cum += slots[p];
        if (slots[p] > 0 && rank < cum + tolerance) return p;
    }
    return kUncached;
}

}  // namespace

struct zm_cache {
    zm_cache_config cfg;
    Layout lay;
    std::vector<zm_tensor_info> infos;
    std::vector<const uint8_t *> host;         // per tensor: the blob (used by fetches only when there are no images)
    std::vector<const uint8_t *> image;        // per expert: packed SM sections then E-chunk regions, or empty
    uint8_t *arena = nullptr;
    std::vector<uint64_t> count;
    std::vector<int8_t> pool_of;               // per expert: pool or kUncached
    std::vector<int32_t> slot_of;
    std::vector<int32_t> owner[kPools];        // per pool, per slot: expert or -1
    std::vector<int32_t> limbo[kPools];        // slots released by the current fetch, reusable from the next one
    hipStream_t copy_stream = nullptr;
    hipEvent_t ev_start = nullptr, ev_copied = nullptr;
    bool broken = false;                       // a fetch failed half-way: slots and bookkeeping may disagree
    // work lists of a fetch (sized at creation for max_selected experts; a fetch is not re-entrant anyway)
    struct Plan { int expert, found, target, slot; };
    std::vector<Plan> plan;
    std::vector<zm_tensor_parts> parts_now, parts_later;
    std::vector<zm_tensor_info> infos_now, infos_later;
    std::vector<void *> out_now, out_later;

    uint8_t *slot_ptr(int pool, int slot) const { return arena + lay.pool_off[pool] + lay.slot_bytes[pool] * static_cast<size_t>(slot); }
    uint8_t *transient_ptr(int j) const { return arena + lay.transient_off + lay.transient_bytes * static_cast<size_t>(j); }
};

extern "C" {

int zm_cache_dispatch(const uint64_t *counts, int n_experts, const int32_t slots[4], int tolerance, int expert)
{
    if (!counts || !slots || n_experts <= 0 || expert < 0 || expert >= n_experts || tolerance < 0) return ZM_E_ARG;
    return dispatch_rank(rank_of(counts, n_experts, expert), slots, tolerance);
}

int zm_cache_arena_bytes(const zm_cache_config *config, const zm_tensor_info *infos, size_t *bytes)
{
    if (!config_ok(config) || !infos || !bytes) return ZM_E_ARG;
    Layout L;
    try { if (!make_layout(*config, infos, L)) return ZM_E_ARG; } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    *bytes = L.total;
    return ZM_OK;
}

int zm_cache_image_bytes(const zm_cache_config *config, const zm_tensor_info *infos, size_t *bytes)
{
    if (!config_ok(config) || !infos || !bytes) return ZM_E_ARG;
    Layout L;
    try { if (!make_layout(*config, infos, L)) return ZM_E_ARG; } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    *bytes = L.sm_bytes + L.e_bytes;
    return ZM_OK;
}

int zm_cache_pack_expert(const zm_cache_config *config, const zm_tensor_info *infos, const void *const *host_blobs,
                         int expert, void *image, size_t image_bytes)
{
    if (!config_ok(config) || !infos || !host_blobs || !image || expert < 0 || expert >= config->n_experts) return ZM_E_ARG;
    Layout L;
    try { if (!make_layout(*config, infos, L)) return ZM_E_ARG; } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    if (image_bytes < L.sm_bytes + L.e_bytes) return ZM_E_SIZE;
    uint8_t *dst = static_cast<uint8_t *>(image);
    std::memset(dst, 0, L.sm_bytes + L.e_bytes);
    for (int m = 0; m < config->tensors_per_expert; ++m) {
        const size_t i = static_cast<size_t>(expert) * config->tensors_per_expert + m;
        const zm_tensor_info &t = infos[i];
        if (!host_blobs[i]) return ZM_E_ARG;
        const uint8_t *src = static_cast<const uint8_t *>(host_blobs[i]);
        std::memcpy(dst + L.sm_off[m], src + t.sm_offset, t.e_offset - t.sm_offset);
        std::memcpy(dst + L.sm_bytes + L.e_off[m], src + t.e_offset, t.blob_size - t.e_offset);
    }
    return ZM_OK;
}

int zm_cache_create(const zm_cache_config *config, const void *const *host_blobs, const void *const *host_images,
                    const zm_tensor_info *infos,
                    void *arena, size_t arena_bytes, zm_cache **out)
{
    if (!config_ok(config) || !host_blobs || !infos || !arena || !out) return ZM_E_ARG;
    if (reinterpret_cast<uintptr_t>(arena) & 255) return ZM_E_ARG;
    zm_cache *c = nullptr;
    try {
        c = new zm_cache();
        c->cfg = *config;
        if (!make_layout(*config, infos, c->lay)) { delete c; return ZM_E_ARG; }
        if (arena_bytes < c->lay.total) { delete c; return ZM_E_SIZE; }
        const size_t n = static_cast<size_t>(config->n_experts) * config->tensors_per_expert;
        c->infos.assign(infos, infos + n);
        c->host.resize(n);
        for (size_t i = 0; i < n; ++i) {
            if (!host_blobs[i]) { delete c; return ZM_E_ARG; }
            c->host[i] = static_cast<const uint8_t *>(host_blobs[i]);
        }
        if (host_images) {
            c->image.resize(config->n_experts);
            for (int e = 0; e < config->n_experts; ++e) {
                if (!host_images[e]) { delete c; return ZM_E_ARG; }
                c->image[e] = static_cast<const uint8_t *>(host_images[e]);
            }
        }
        c->arena = static_cast<uint8_t *>(arena);
        c->count.assign(config->n_experts, 0);
        const size_t most = static_cast<size_t>(config->max_selected) * config->tensors_per_expert;
        c->plan.resize(config->max_selected);
        c->parts_now.resize(most); c->parts_later.resize(most);
        c->infos_now.resize(most); c->infos_later.resize(most);
        c->out_now.resize(most); c->out_later.resize(most);
        c->pool_of.assign(config->n_experts, static_cast<int8_t>(kUncached));
        c->slot_of.assign(config->n_experts, -1);
        for (int p = 0; p < kPools; ++p) c->owner[p].assign(config->slots[p], -1);
    } catch (const std::bad_alloc &) { delete c; return ZM_E_NOMEM; }
    if (hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_start, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_copied, hipEventDisableTiming) != hipSuccess) {
        zm_cache_destroy(c);
        return ZM_E_HIP;
    }
    // decode tables and chunk tables of every tensor stay resident: a few KB per tensor
    const size_t n = c->infos.size();
    for (size_t i = 0; i < n; ++i) {
        const zm_tensor_info &t = c->infos[i];
        if (hipMemcpyAsync(c->arena + c->lay.meta_off[i], c->host[i] + t.lut_offset, t.table_offset - t.lut_offset,
                           hipMemcpyHostToDevice, c->copy_stream) != hipSuccess ||
            hipMemcpyAsync(c->arena + c->lay.meta_table_off[i], c->host[i] + t.table_offset, static_cast<size_t>(t.table_stride) * (t.n_chunks + 1),
                           hipMemcpyHostToDevice, c->copy_stream) != hipSuccess) {
            zm_cache_destroy(c);
            return ZM_E_HIP;
        }
    }
    if (hipStreamSynchronize(c->copy_stream) != hipSuccess) { zm_cache_destroy(c); return ZM_E_HIP; }
    *out = c;
    return ZM_OK;
}

void zm_cache_destroy(zm_cache *c)
{
    if (!c) return;
    if (c->copy_stream) { (void)hipStreamSynchronize(c->copy_stream); (void)hipStreamDestroy(c->copy_stream); }
    if (c->ev_start) (void)hipEventDestroy(c->ev_start);
    if (c->ev_copied) (void)hipEventDestroy(c->ev_copied);
    delete c;
}

int zm_cache_pool_of(const zm_cache *c, int expert)
{
    if (!c || expert < 0 || expert >= c->cfg.n_experts) return ZM_E_ARG;
    return c->pool_of[expert];
}

int zm_cache_fetch(zm_cache *c, const int32_t *expert_ids, int n_selected, void **out_bf16, int32_t *found_in,
                   void *stream)
{
    if (!c || !expert_ids || !out_bf16 || n_selected < 0 || n_selected > c->cfg.max_selected) return ZM_E_ARG;
    if (c->broken) return ZM_E_HIP;
    if (n_selected == 0) return ZM_OK;
    const int T = c->cfg.tensors_per_expert, N = c->cfg.n_experts;
    for (int j = 0; j < n_selected; ++j) {
        if (expert_ids[j] < 0 || expert_ids[j] >= N) return ZM_E_ARG;
        for (int i = 0; i < j; ++i) if (expert_ids[i] == expert_ids[j]) return ZM_E_ARG;    // a gate selects distinct experts
    }
    hipStream_t main_stream = static_cast<hipStream_t>(stream);
    // slots released by the previous fetch may be reused now
    for (int p = 0; p < kPools; ++p) {
        for (int s : c->limbo[p]) c->owner[p][s] = -1;
        c->limbo[p].clear();
    }
    // copies of this fetch must not overtake what the caller still has queued on its stream
    // (the previous fetch's outputs may live in the transient buffers)
    if (hipEventRecord(c->ev_start, main_stream) != hipSuccess ||
        hipStreamWaitEvent(c->copy_stream, c->ev_start, 0) != hipSuccess) return ZM_E_HIP;

    for (int j = 0; j < n_selected; ++j) ++c->count[expert_ids[j]];

    using Plan = zm_cache::Plan;
    Plan *plan = c->plan.data();
    auto selected = [&](int e) { for (int j = 0; j < n_selected; ++j) if (expert_ids[j] == e) return true; return false; };
    for (int j = 0; j < n_selected; ++j) {
        const int e = expert_ids[j];
        Plan &pl = plan[j];
        pl.expert = e; pl.found = c->pool_of[e]; pl.slot = c->slot_of[e];
        int target = dispatch_rank(rank_of(c->count.data(), N, e), c->cfg.slots, c->cfg.tolerance);
        if (target >= pl.found) target = pl.found;            // an access never demotes (pools are ordered F < C < S < E < none)
        if (target != pl.found) {
            // take a free slot of the target pool, else evict its least frequently activated member
            // that this call does not use
            int slot = -1;
            std::vector<int32_t> &own = c->owner[target];
            for (size_t s = 0; s < own.size() && slot < 0; ++s) if (own[s] == -1) slot = static_cast<int>(s);
            if (slot < 0) {
                int victim_slot = -1;
                for (size_t s = 0; s < own.size(); ++s) {
                    const int x = own[s];
                    if (x < 0 || selected(x)) continue;        // x < 0: a slot in limbo
                    if (victim_slot < 0 || c->count[x] < c->count[own[victim_slot]] ||
                        (c->count[x] == c->count[own[victim_slot]] && x > own[victim_slot])) victim_slot = static_cast<int>(s);
                }
                if (victim_slot >= 0 && c->count[own[victim_slot]] <= c->count[e]) {
                    const int x = own[victim_slot];
                    c->pool_of[x] = static_cast<int8_t>(kUncached); c->slot_of[x] = -1;
                    slot = victim_slot;
                }
            }
            if (slot < 0) target = pl.found;                    // nowhere to go: stays where it is
            else {
                own[slot] = e;
                if (pl.found != kUncached) { c->owner[pl.found][pl.slot] = -2; c->limbo[pl.found].push_back(pl.slot); }
                c->pool_of[e] = static_cast<int8_t>(target); c->slot_of[e] = slot;
            }
        }
        pl.target = target;
        if (found_in) found_in[j] = pl.found;
    }

    // data movement and decode lists
    zm_tensor_parts *parts_now = c->parts_now.data(), *parts_later = c->parts_later.data();
    zm_tensor_info *infos_now = c->infos_now.data(), *infos_later = c->infos_later.data();
    void **out_now = c->out_now.data(), **out_later = c->out_later.data();
    int n_now = 0, n_later = 0;
    bool any_copy = false;
    for (int j = 0; j < n_selected; ++j) {
        const Plan &pl = plan[j];
        const int e = pl.expert;
        uint8_t *tr = c->transient_ptr(j);
        uint8_t *tr_sm = tr, *tr_e = tr + c->lay.sm_bytes, *tr_full = tr + c->lay.sm_bytes + c->lay.e_bytes;
        const int new_slot = c->slot_of[e];
        // where the parts are now (device) -- from the pool the expert was found in
        const uint8_t *have_sm = nullptr, *have_e = nullptr;
        if (pl.found == ZM_POOL_COMPRESSED) { have_sm = c->slot_ptr(pl.found, pl.slot); have_e = have_sm + c->lay.sm_bytes; }
        else if (pl.found == ZM_POOL_SM) have_sm = c->slot_ptr(pl.found, pl.slot);
        else if (pl.found == ZM_POOL_E) have_e = c->slot_ptr(pl.found, pl.slot);
        // where they have to be kept (device) -- in the pool the expert goes to, if that pool keeps them
        uint8_t *keep_sm = nullptr, *keep_e = nullptr, *keep_full = nullptr;
        if (pl.target != pl.found) {
            uint8_t *dst = c->slot_ptr(pl.target, new_slot);
            if (pl.target == ZM_POOL_FULL) keep_full = dst;
            else if (pl.target == ZM_POOL_COMPRESSED) { keep_sm = dst; keep_e = dst + c->lay.sm_bytes; }
            else if (pl.target == ZM_POOL_SM) keep_sm = dst;
            else if (pl.target == ZM_POOL_E) keep_e = dst;
        }
        // With packed images the parts of an expert move as whole regions: one copy when both regions come
        // from the host and land next to each other (a C slot, or the transient buffer), else one per region.
        const bool by_region = !c->image.empty() && pl.found != ZM_POOL_FULL;
        bool region_copied = false;
        if (by_region) {
            uint8_t *sm_to = keep_sm ? keep_sm : (have_sm ? nullptr : tr_sm);
            uint8_t *e_to = keep_e ? keep_e : (have_e ? nullptr : tr_e);
            const uint8_t *img = c->image[e];
            hipError_t rc = hipSuccess;
            if (sm_to && e_to && !have_sm && !have_e && e_to == sm_to + c->lay.sm_bytes) {
                rc = hipMemcpyAsync(sm_to, img, c->lay.sm_bytes + c->lay.e_bytes, hipMemcpyHostToDevice, c->copy_stream);
            } else {
                if (sm_to) rc = have_sm ? hipMemcpyAsync(sm_to, have_sm, c->lay.sm_bytes, hipMemcpyDeviceToDevice, c->copy_stream)
                                        : hipMemcpyAsync(sm_to, img, c->lay.sm_bytes, hipMemcpyHostToDevice, c->copy_stream);
                if (rc == hipSuccess && e_to)
                    rc = have_e ? hipMemcpyAsync(e_to, have_e, c->lay.e_bytes, hipMemcpyDeviceToDevice, c->copy_stream)
                                : hipMemcpyAsync(e_to, img + c->lay.sm_bytes, c->lay.e_bytes, hipMemcpyHostToDevice, c->copy_stream);
            }
            if (rc != hipSuccess) { c->broken = true; return ZM_E_HIP; }
            region_copied = sm_to || e_to;
        }
        for (int m = 0; m < T; ++m) {
            const size_t i = static_cast<size_t>(e) * T + m;
            const zm_tensor_info &ti = c->infos[i];
            void *&out = out_bf16[static_cast<size_t>(j) * T + m];
            if (pl.found == ZM_POOL_FULL) { out = c->slot_ptr(ZM_POOL_FULL, pl.slot) + c->lay.full_off[m]; continue; }
            bool copied = region_copied;
            const size_t sm_len = ti.e_offset - ti.sm_offset, e_len = ti.blob_size - ti.e_offset;
            // SM part: already in place, or moved device-to-device into its new pool, or fetched from the host
            const uint8_t *sm_src = have_sm ? have_sm + c->lay.sm_off[m] : nullptr;
            uint8_t *sm_dst = keep_sm ? keep_sm + c->lay.sm_off[m] : (sm_src ? nullptr : tr_sm + c->lay.sm_off[m]);
            if (sm_dst && !by_region) {
                const hipError_t rc = sm_src ? hipMemcpyAsync(sm_dst, sm_src, sm_len, hipMemcpyDeviceToDevice, c->copy_stream)
                                             : hipMemcpyAsync(sm_dst, c->host[i] + ti.sm_offset, sm_len, hipMemcpyHostToDevice, c->copy_stream);
                if (rc != hipSuccess) { c->broken = true; return ZM_E_HIP; }
                copied = true;
            }
            const uint8_t *e_src = have_e ? have_e + c->lay.e_off[m] : nullptr;
            uint8_t *e_dst = keep_e ? keep_e + c->lay.e_off[m] : (e_src ? nullptr : tr_e + c->lay.e_off[m]);
            if (e_dst && !by_region) {
                const hipError_t rc = e_src ? hipMemcpyAsync(e_dst, e_src, e_len, hipMemcpyDeviceToDevice, c->copy_stream)
                                            : hipMemcpyAsync(e_dst, c->host[i] + ti.e_offset, e_len, hipMemcpyHostToDevice, c->copy_stream);
                if (rc != hipSuccess) { c->broken = true; return ZM_E_HIP; }
                copied = true;
            }
            zm_tensor_parts pt;
            pt.table = c->arena + c->lay.meta_off[i];
            pt.chunk_offsets = c->arena + c->lay.meta_table_off[i];
            pt.sm = sm_dst ? sm_dst : sm_src;
            pt.echunks = e_dst ? e_dst : e_src;
            out = keep_full ? keep_full + c->lay.full_off[m] : tr_full + c->lay.full_off[m];
            if (copied) { parts_later[n_later] = pt; infos_later[n_later] = ti; out_later[n_later++] = out; any_copy = true; }
            else { parts_now[n_now] = pt; infos_now[n_now] = ti; out_now[n_now++] = out; }
        }
    }
    // experts whose parts are all resident decode while the copies for the others are in flight
    int rc = zm_decode_tensors(parts_now, infos_now, n_now, out_now, stream);
    if (rc == ZM_OK && any_copy) {
        if (hipEventRecord(c->ev_copied, c->copy_stream) != hipSuccess ||
            hipStreamWaitEvent(main_stream, c->ev_copied, 0) != hipSuccess) rc = ZM_E_HIP;
        else rc = zm_decode_tensors(parts_later, infos_later, n_later, out_later, stream);
    }
    if (rc != ZM_OK) c->broken = true;
    return rc;
}

}  // extern "C"
