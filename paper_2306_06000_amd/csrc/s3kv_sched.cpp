// Length-aware scheduler of libs3kv (host integers only): a request pool and the decreasing-first-fit
// admission pass of the S3 paper (section 3, scheduler paragraph): the pool is sorted by the size of the
// KV cache each request would reserve, largest first, and walked once; a request is put into the batch
// iff its reservation still fits in the arena, until nothing is left of the memory or the pool has been
// walked.  Called again at every iteration with whatever the finished sequences have freed
// (iteration-level scheduling, same section).  Ties keep arrival order.
#include <algorithm>
#include <new>
#include <vector>

#include "s3kv_internal.h"

struct s3_request {
    int64_t id;
    int32_t predicted_len;
    int64_t arrival;
};

struct s3_sched {
    s3_arena *arena = nullptr;
    std::vector<s3_request> pool;  // arrival order
    int64_t next_arrival = 0;
};

extern "C" int s3_sched_create(s3_sched **out, s3_arena *a) {
    if (!out || !a) return S3_ERR_INVALID;
    s3_sched *s = new (std::nothrow) s3_sched();
    if (!s) return S3_ERR_NOMEM;
    s->arena = a;
    *out = s;
    return S3_OK;
}

extern "C" void s3_sched_destroy(s3_sched *s) { delete s; }

extern "C" int s3_sched_submit(s3_sched *s, int64_t request_id, int32_t predicted_len) {
    if (!s || predicted_len < 0) return S3_ERR_INVALID;
    s->pool.push_back({request_id, predicted_len, s->next_arrival++});
    return S3_OK;
}

extern "C" int s3_sched_pool_size(const s3_sched *s) { return s ? (int)s->pool.size() : S3_ERR_INVALID; }

extern "C" int s3_sched_admit(s3_sched *s, int32_t max_out, int64_t *request_id, int32_t *slot_id, int64_t *slot_off,
                              int32_t *slot_cap) {
    if (!s || max_out < 0 || (max_out > 0 && (!request_id || !slot_id || !slot_off || !slot_cap))) return S3_ERR_INVALID;
    // decreasing order of reserved size; stable, so equal sizes stay in arrival order
    std::vector<size_t> order(s->pool.size());
    for (size_t i = 0; i < order.size(); i++) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) {
        return s3i_capacity_for(s->arena, s->pool[x].predicted_len) > s3i_capacity_for(s->arena, s->pool[y].predicted_len);
    });
    std::vector<char> taken(s->pool.size(), 0);
    int admitted = 0;
    for (size_t k = 0; k < order.size() && admitted < max_out; k++) {
        int64_t free_tok = 0;
        s3_kv_stats(s->arena, nullptr, &free_tok, nullptr, nullptr);
        if (free_tok <= 0) break;  // no memory left: stop walking the pool
        const s3_request &r = s->pool[order[k]];
        int32_t id = -1, cap = 0;
        int64_t off = -1;
        const int rc = s3_kv_alloc(s->arena, 1, &r.predicted_len, &id, &off, &cap);
        if (rc < 0) return rc;
        if (rc == 0) continue;  // does not fit: go on to the next (smaller) request
        request_id[admitted] = r.id;
        slot_id[admitted] = id;
        slot_off[admitted] = off;
        slot_cap[admitted] = cap;
        taken[order[k]] = 1;
        admitted++;
    }
    size_t w = 0;
    for (size_t i = 0; i < s->pool.size(); i++)
        if (!taken[i]) s->pool[w++] = s->pool[i];
    s->pool.resize(w);
    return admitted;
}
