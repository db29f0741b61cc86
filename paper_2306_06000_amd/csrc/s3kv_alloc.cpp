// Host bookkeeping of libs3kv: the slot table and the free-extent list of one arena, and the
// entry points that are pure integer work.  No HIP call is made from this file except through
// the launchers declared in s3kv_internal.h, and none at all for a metadata-only arena.
//
// Policy (S3 paper, arXiv 2306.06000): a sequence reserves its PREDICTED length rounded up to
// the granule (sections 1, 2.3), sequences are admitted in caller order while they fit in what
// is left (section 3, scheduler paragraph), a sequence that used up its reservation gets twice
// the room (section 3, supervisor paragraph), and the free space is reported back (ibid.).
// Where the paper is silent: placement is first fit at the lowest offset, a grown slot is placed
// before the old one is released, and capacities never exceed max_len.
#include <string.h>

#include <new>
#include <string>

#include <algorithm>

#include "s3kv_internal.h"

static thread_local std::string g_hip_error;

void s3i_set_hip_error(const char *what, int code, const char *text) {
    g_hip_error = std::string(what) + ": " + (text ? text : "?") + " (" + std::to_string(code) + ")";
}

extern "C" const char *s3_last_hip_error(void) { return g_hip_error.c_str(); }

extern "C" const char *s3_status_str(int status) {
    switch (status) {
        case S3_OK: return "S3_OK";
        case S3_ERR_INVALID: return "S3_ERR_INVALID";
        case S3_ERR_NOMEM: return "S3_ERR_NOMEM";
        case S3_ERR_SLOT_FULL: return "S3_ERR_SLOT_FULL";
        case S3_ERR_MAXLEN: return "S3_ERR_MAXLEN";
        case S3_ERR_HIP: return "S3_ERR_HIP";
        case S3_ERR_SCRATCH: return "S3_ERR_SCRATCH";
        default: return status > 0 ? "count" : "unknown";
    }
}

static bool config_ok(const s3_kv_config *c) {
    if (!c) return false;
    if (c->n_layers <= 0 || c->n_heads <= 0) return false;
    if (c->head_dim != 64 && c->head_dim != 96 && c->head_dim != 128 && c->head_dim != 256) return false;
    if (c->kv_dtype != S3_F16 && c->kv_dtype != S3_BF16 && c->kv_dtype != S3_E4M3) return false;
    if (c->kv_dtype == S3_E4M3 && c->act_dtype != S3_F16 && c->act_dtype != S3_BF16) return false;  // 16-bit activations
    if (c->granule <= 0 || c->max_len <= 0 || c->max_len % c->granule != 0) return false;
    if (c->n_kv_heads < 0 || (c->n_kv_heads > 0 && (c->n_kv_heads > c->n_heads || c->n_heads % c->n_kv_heads))) return false;
    // 96-wide heads (the 64 x 96 model of the paper's table 1): multi-head 16-bit caches only
    if (c->head_dim == 96 && (c->kv_dtype == S3_E4M3 || (c->n_kv_heads > 0 && c->n_kv_heads != c->n_heads))) return false;
    return true;
}

extern "C" int64_t s3_kv_bytes_per_token(const s3_kv_config *cfg) {
    if (!config_ok(cfg)) return S3_ERR_INVALID;
    // K and V, every layer, H*D two-byte numbers: 4*l*d_h bytes (section 2.1)
    const int kv_heads = cfg->n_kv_heads > 0 ? cfg->n_kv_heads : cfg->n_heads;
    return (int64_t)2 * cfg->n_layers * kv_heads * cfg->head_dim * (cfg->kv_dtype == S3_E4M3 ? 1 : 2);
}

extern "C" int s3_kv_arena_init(s3_arena **out, const s3_kv_config *cfg, void *dev_base, size_t dev_bytes) {
    if (!out || !config_ok(cfg)) return S3_ERR_INVALID;
    if (dev_base && ((uintptr_t)dev_base & 255u)) return S3_ERR_INVALID;
    s3_arena *a = new (std::nothrow) s3_arena();
    if (!a) return S3_ERR_NOMEM;
    a->cfg = *cfg;
    a->base = (char *)dev_base;
    a->dev_bytes = dev_bytes;
    a->elem_bytes = cfg->kv_dtype == S3_E4M3 ? 1 : 2;
    if (a->cfg.n_kv_heads == 0) a->cfg.n_kv_heads = cfg->n_heads;
    if (cfg->kv_dtype != S3_E4M3) a->cfg.act_dtype = cfg->kv_dtype;
    a->row_bytes = (int64_t)a->cfg.n_kv_heads * cfg->head_dim * a->elem_bytes;
    a->n_tokens = (int64_t)(dev_bytes / (size_t)s3_kv_bytes_per_token(cfg));
    a->plane_bytes = a->n_tokens * a->row_bytes;
    if (a->n_tokens > 0) a->free_ext[0] = a->n_tokens;
    if (dev_base) {
        int rc = s3i_device_cus(&a->num_cus);
        if (rc == S3_OK) rc = s3i_static_scratch_setup();
        if (rc != S3_OK) {
            delete a;
            return rc;
        }
    }
    *out = a;
    return S3_OK;
}

extern "C" int32_t s3_kv_capacity_for(const s3_kv_config *cfg, int32_t predicted_len) {
    if (!config_ok(cfg) || predicted_len < 0) return S3_ERR_INVALID;
    const int64_t g = cfg->granule;
    int64_t cap = ((int64_t)predicted_len + g - 1) / g * g;
    if (cap < g) cap = g;
    if (cap > cfg->max_len) cap = cfg->max_len;
    return (int32_t)cap;
}

extern "C" int32_t s3_kv_grown_capacity(const s3_kv_config *cfg, int32_t cap) {
    if (!config_ok(cfg) || cap < 0) return S3_ERR_INVALID;
    const int64_t twice = 2 * (int64_t)cap;
    return (int32_t)(twice > cfg->max_len ? cfg->max_len : twice);
}

int32_t s3i_capacity_for(const s3_arena *a, int32_t predicted_len) { return s3_kv_capacity_for(&a->cfg, predicted_len); }

int64_t s3i_carve(s3_arena *a, int64_t cap) {
    for (auto it = a->free_ext.begin(); it != a->free_ext.end(); ++it) {
        if (it->second >= cap) {
            const int64_t off = it->first, size = it->second;
            a->free_ext.erase(it);
            if (size > cap) a->free_ext[off + cap] = size - cap;
            return off;
        }
    }
    return -1;
}

void s3i_release(s3_arena *a, int64_t off, int64_t cap) {
    auto next = a->free_ext.lower_bound(off);
    if (next != a->free_ext.end() && off + cap == next->first) {
        cap += next->second;
        next = a->free_ext.erase(next);
    }
    if (next != a->free_ext.begin()) {
        auto prev = std::prev(next);
        if (prev->first + prev->second == off) {
            prev->second += cap;
            return;
        }
    }
    a->free_ext[off] = cap;
}

const s3_slot *s3i_live_slot(const s3_arena *a, int32_t id) {
    if (!a || id < 0 || (size_t)id >= a->slots.size() || !a->slots[id].live) return nullptr;
    return &a->slots[id];
}

extern "C" int s3_kv_alloc(s3_arena *a, int32_t n, const int32_t *predicted_len, int32_t *slot_id,
                           int64_t *slot_off, int32_t *slot_cap) {
    if (!a || n < 0 || (n > 0 && (!predicted_len || !slot_id || !slot_off || !slot_cap))) return S3_ERR_INVALID;
    for (int32_t i = 0; i < n; i++)
        if (predicted_len[i] < 0) return S3_ERR_INVALID;
    int admitted = 0;
    for (int32_t i = 0; i < n; i++) {
        const int32_t cap = s3i_capacity_for(a, predicted_len[i]);
        const int64_t off = s3i_carve(a, cap);
        if (off < 0) {
            slot_id[i] = -1;
            slot_off[i] = -1;
            slot_cap[i] = 0;
            continue;
        }
        int32_t id;
        if (!a->dead_ids.empty()) {
            id = *a->dead_ids.begin();
            a->dead_ids.erase(a->dead_ids.begin());
        } else {
            id = (int32_t)a->slots.size();
            a->slots.emplace_back();
        }
        a->slots[id].off = off;
        a->slots[id].cap = cap;
        a->slots[id].live = true;
        a->used_tokens += cap;
        slot_id[i] = id;
        slot_off[i] = off;
        slot_cap[i] = cap;
        admitted++;
    }
    return admitted;
}

extern "C" int s3_kv_free(s3_arena *a, int32_t slot_id) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s) return S3_ERR_INVALID;
    s3i_release(a, s->off, s->cap);
    a->used_tokens -= s->cap;
    a->slots[slot_id] = s3_slot();
    a->dead_ids.insert(slot_id);
    return S3_OK;
}

extern "C" int s3_kv_slot_info(const s3_arena *a, int32_t slot_id, int64_t *off, int32_t *cap) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s) return S3_ERR_INVALID;
    if (off) *off = s->off;
    if (cap) *cap = s->cap;
    return S3_OK;
}

extern "C" int s3_kv_grow(s3_arena *a, int32_t slot_id, int32_t len, int64_t *new_off, int32_t *new_cap,
                          void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || len < 0 || len > s->cap) return S3_ERR_INVALID;
    if (s->cap >= a->cfg.max_len) return S3_ERR_MAXLEN;
    const int64_t old_off = s->off;
    const int32_t old_cap = s->cap;
    const int64_t cap2 = s3_kv_grown_capacity(&a->cfg, old_cap);
    const int64_t off2 = s3i_carve(a, cap2);  // the old extent is still reserved: no overlap possible
    if (off2 < 0) return S3_ERR_NOMEM;
    if (a->base && len > 0) {
        const int rc = s3i_launch_copy_planes(a->base + old_off * a->row_bytes, a->base + off2 * a->row_bytes,
                                              (size_t)len * (size_t)a->row_bytes, (size_t)a->plane_bytes,
                                              (size_t)a->plane_bytes, 2 * a->cfg.n_layers, stream);
        if (rc != S3_OK) {
            s3i_release(a, off2, cap2);
            return rc;
        }
    }
    s3i_release(a, old_off, old_cap);
    a->slots[slot_id].off = off2;
    a->slots[slot_id].cap = (int32_t)cap2;
    a->used_tokens += cap2 - old_cap;
    a->n_grows++;
    if (new_off) *new_off = off2;
    if (new_cap) *new_cap = (int32_t)cap2;
    return S3_OK;
}

// Compaction (section 3, supervisor paragraph: after sequences have left, the rows below a blank are
// shifted so that everything is stored contiguously again).  Live slots keep their order by offset and
// slide down to close every hole; the free space becomes one extent at the end.
extern "C" int s3_kv_compact(s3_arena *a, int32_t n, const int32_t *slot_id, const int32_t *len, int64_t *new_off,
                             int32_t *n_moved, void *stream) {
    if (!a || n < 0 || (n > 0 && (!slot_id || !len))) return S3_ERR_INVALID;
    std::vector<int32_t> rows(a->slots.size(), -1);  // rows to preserve per id; -1: the whole capacity
    for (int32_t i = 0; i < n; i++) {
        const s3_slot *s = s3i_live_slot(a, slot_id[i]);
        if (!s || len[i] < 0 || len[i] > s->cap) return S3_ERR_INVALID;
        rows[slot_id[i]] = len[i];
    }
    std::map<int64_t, int32_t> by_off;  // offset -> id
    for (size_t id = 0; id < a->slots.size(); id++)
        if (a->slots[id].live) by_off[a->slots[id].off] = (int32_t)id;
    int64_t cursor = 0;
    int32_t moved = 0;
    for (const auto &e : by_off) {
        s3_slot &s = a->slots[e.second];
        const int64_t gap = s.off - cursor;
        const int64_t keep = rows[e.second] >= 0 ? rows[e.second] : s.cap;
        if (gap > 0) {
            if (a->base) {
                // source and destination overlap when gap < keep: move pieces of `gap` rows in stream order,
                // each piece lands on rows that the previous piece has already left
                for (int64_t r = 0; r < keep; r += gap) {
                    const int64_t piece = keep - r < gap ? keep - r : gap;
                    const int rc = s3i_launch_copy_planes(
                        a->base + (s.off + r) * a->row_bytes, a->base + (cursor + r) * a->row_bytes,
                        (size_t)piece * (size_t)a->row_bytes, (size_t)a->plane_bytes, (size_t)a->plane_bytes,
                        2 * a->cfg.n_layers, stream);
                    if (rc != S3_OK) return rc;  // rows already moved stay moved; the table below is not updated
                }
            }
            moved++;
        }
        cursor += s.cap;
    }
    // every copy is enqueued: now the table
    cursor = 0;
    for (const auto &e : by_off) {
        a->slots[e.second].off = cursor;
        cursor += a->slots[e.second].cap;
    }
    a->free_ext.clear();
    if (cursor < a->n_tokens) a->free_ext[cursor] = a->n_tokens - cursor;
    for (int32_t i = 0; i < n && new_off; i++) new_off[i] = a->slots[slot_id[i]].off;
    if (n_moved) *n_moved = moved;
    return S3_OK;
}

extern "C" int s3_kv_stats(const s3_arena *a, int64_t *used_tok, int64_t *free_tok, int64_t *largest_free_tok,
                           int64_t *capacity_tok) {
    if (!a) return S3_ERR_INVALID;
    int64_t free_sum = 0, largest = 0;
    for (const auto &e : a->free_ext) {
        free_sum += e.second;
        if (e.second > largest) largest = e.second;
    }
    if (used_tok) *used_tok = a->used_tokens;
    if (free_tok) *free_tok = free_sum;
    if (largest_free_tok) *largest_free_tok = largest;
    if (capacity_tok) *capacity_tok = a->n_tokens;
    return S3_OK;
}

// The attention kernel family an arena uses depends on whether its key/value heads are shared.
static int s3i_variants_of(const s3_arena *a) {
    if (a->cfg.kv_dtype == S3_E4M3) return a->cfg.n_kv_heads < a->cfg.n_heads ? 1 : s3i_num_fp8_shapes();
    return a->cfg.n_kv_heads < a->cfg.n_heads ? s3i_num_gqa_shapes() + 1 : s3i_num_variants();  // + the matrix-core kernel
}

int s3i_kernel_kind(const s3_arena *a) {
    if (a->cfg.kv_dtype == S3_E4M3) return a->cfg.n_kv_heads < a->cfg.n_heads ? 4 : 3;
    if (a->cfg.n_kv_heads >= a->cfg.n_heads) return 0;
    const int group = a->cfg.n_heads / a->cfg.n_kv_heads;
    return (a->variant == s3i_num_gqa_shapes() || (a->variant < 0 && group >= 4)) ? 2 : 1;
}

extern "C" int s3_kv_set_param(s3_arena *a, const char *name, int64_t value) {
    if (!a || !name) return S3_ERR_INVALID;
    if (!strcmp(name, "chunk")) {
        if (value != 0 && (value < 32 || value > 2048 || value % 32)) return S3_ERR_INVALID;
        a->chunk = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "classes")) {
        if (value < 0 || value > 8) return S3_ERR_INVALID;
        a->ncls = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "grid_blocks")) {
        if (value < 0 || value > (1 << 20)) return S3_ERR_INVALID;
        a->grid_blocks = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "variant")) {
        if (value < -1 || value >= s3i_variants_of(a)) return S3_ERR_INVALID;
        a->variant = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "gqa_merge")) {
        if (value != 0 && value != 1) return S3_ERR_INVALID;
        a->gqa_merge = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "gqa_dynamic")) {
        if (value < -1 || value > 100) return S3_ERR_INVALID;
        a->gqa_dynamic = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "gqa_stream")) {
        if (value < -1 || value > 1) return S3_ERR_INVALID;
        a->gqa_stream = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "merge_sync")) {
        if (value != 0 && value != 1) return S3_ERR_INVALID;
        a->merge_sync = (int32_t)value;
        return S3_OK;
    }
    if (!strcmp(name, "profile")) {  // k > 0: time every k-th attention launch with events; 0: off; both reset
        if (value < 0 || value > 1000000) return S3_ERR_INVALID;
        if (!a->base) return S3_ERR_INVALID;
        s3i_profile_reset(a);
        a->profile = (int32_t)value;
        a->prof_tick = 0;
        return S3_OK;
    }
    return S3_ERR_INVALID;
}

extern "C" int s3_kv_get_param(const s3_arena *a, const char *name, int64_t *value) {
    if (!a || !name || !value) return S3_ERR_INVALID;
    if (!strcmp(name, "chunk")) *value = a->chunk;
    else if (!strcmp(name, "grid_blocks")) *value = a->grid_blocks;
    else if (!strcmp(name, "classes")) *value = a->ncls;
    else if (!strcmp(name, "variant")) *value = a->variant;
    else if (!strcmp(name, "merge_sync")) *value = a->merge_sync;
    else if (!strcmp(name, "gqa_merge")) *value = a->gqa_merge;
    else if (!strcmp(name, "gqa_stream")) *value = a->gqa_stream;
    else if (!strcmp(name, "gqa_dynamic")) *value = a->gqa_dynamic;
    else if (!strcmp(name, "n_variants")) *value = s3i_variants_of(a);
    else if (!strcmp(name, "default_variant")) *value = s3i_kernel_kind(a) == 0 ? s3i_default_variant() : -1;
    else if (!strcmp(name, "kernel_kind")) *value = s3i_kernel_kind(a);
    else if (!strcmp(name, "n_grows")) *value = a->n_grows;
    else if (!strcmp(name, "live_slots")) *value = (int64_t)a->slots.size() - (int64_t)a->dead_ids.size();
    else if (!strcmp(name, "scratch_bytes")) *value = (int64_t)a->scratch_bytes;
    else if (!strcmp(name, "num_cus")) *value = a->num_cus;
    else if (!strncmp(name, "profile_", 8)) {
        const int rc = s3i_profile_collect(const_cast<s3_arena *>(a));
        if (rc != S3_OK) return rc;
        if (!strcmp(name, "profile_launches")) *value = a->prof_launches;
        else if (!strcmp(name, "profile_partial_ns")) *value = (int64_t)(a->prof_partial_ms * 1e6);
        else if (!strcmp(name, "profile_merge_ns")) *value = (int64_t)(a->prof_merge_ms * 1e6);
        else if (!strcmp(name, "profile_p10_ns") || !strcmp(name, "profile_p50_ns") || !strcmp(name, "profile_p90_ns")) {
            // nearest-rank percentile of the timed launches' first interval (the attention kernel)
            std::vector<float> d = a->prof_durations_ms;
            if (d.empty()) { *value = 0; return S3_OK; }
            std::sort(d.begin(), d.end());
            const int pct = name[9] == '1' ? 10 : name[9] == '5' ? 50 : 90;
            size_t k = (d.size() * pct + 99) / 100;
            if (k > 0) k--;
            *value = (int64_t)(d[k] * 1e6);
        }
        else return S3_ERR_INVALID;
    }
    else return S3_ERR_INVALID;
    return S3_OK;
}
