/*
 * s3kv - prediction-sized ragged KV cache and decode-step attention for AMD MI355X (gfx950).
 *
 * C ABI of libs3kv.so.  Plain pointers and sizes only.  Every pointer is marked
 * HOST or DEVICE; DEVICE pointers are HIP device memory owned by the caller.
 *
 * The library implements the memory-management idea of the S3 paper (arXiv 2306.06000):
 * every sequence reserves KV-cache room for its PREDICTED length instead of the
 * maximum sequence length (sections 1, 2.2, 2.3), rows are filled append-only
 * (section 2.2), each sequence attends to its own rows without padding
 * (section 2.1 equation; section 3, scheduler paragraph on irregular batches), and
 * a sequence that outgrows its reservation gets twice the room (section 3,
 * supervisor paragraph).
 *
 * Units.  Slot offsets, capacities, lengths and positions are in TOKEN ROWS.  One
 * token row holds, for every layer, one key and one value vector of
 * n_heads*head_dim elements: bytes_per_token = 2*n_layers*n_heads*head_dim*elem
 * (= the paper's 4*l*d_h bytes for two-byte elements, section 2.1); with fewer K/V heads than query
 * heads (multi-query attention, which the paper's related-work section names as a complementary way to
 * shrink the cache) n_kv_heads takes the place of n_heads in that count.  How rows are
 * placed inside the arena is private to the library.
 *
 * Conventions.  Every call returns an s3_status (or a non-negative count where
 * stated).  Nothing aborts or throws.  No call synchronises the device unless
 * stated.  Kernels are enqueued on the `stream` argument (a hipStream_t passed as
 * void*; NULL is the default stream).  Host-side bookkeeping (slot table, free
 * list) changes immediately; device work is ordered by the stream.  An arena is
 * not thread-safe: serialise calls on one arena (different arenas may be used from
 * different threads); attention launches of one arena share its scratch and must not
 * overlap on the device either (one stream, or ordered streams).
 *
 * Graphs.  s3_decode_attention / s3_decode_step only enqueue kernels once the library's
 * scratch is large enough for the batch (it grows, with a device synchronisation and an
 * allocation, on the first call with a larger batch): after one eager call with the same
 * arguments' shapes the launches may be recorded into a HIP graph and replayed.
 *
 * Error behaviour of device arrays.  slot_off/pos/cur_len live in device memory
 * and cannot be checked by the host without a sync, so the kernels themselves
 * skip any entry that would address rows outside the arena (off < 0, len < 0,
 * len > max_len or off+len > arena capacity): append writes nothing for such an
 * entry, attention returns an all-zero row.  No access ever leaves the arena.
 */
#ifndef S3KV_H
#define S3KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct s3_arena s3_arena; /* opaque; host-side metadata owned by the library */

/* S3_E4M3: 8-bit float, 1 sign / 4 exponent (bias 7) / 3 fraction bits, no infinities, largest 448
 * (cache rows only; related work: quantisation as a complementary way to shrink the cache). */
typedef enum { S3_F16 = 0, S3_BF16 = 1, S3_F32 = 2, S3_E4M3 = 3 } s3_dtype;

typedef enum {
    S3_OK = 0,
    S3_ERR_INVALID = -1,   /* null pointer, bad shape, unknown id, misaligned base, unsupported type */
    S3_ERR_NOMEM = -2,     /* the arena cannot fit the request; state unchanged */
    S3_ERR_SLOT_FULL = -3, /* append at pos == capacity; nothing written, nothing launched */
    S3_ERR_MAXLEN = -4,    /* grow of a slot whose capacity already is max_len */
    S3_ERR_HIP = -5,       /* a HIP call failed; see s3_last_hip_error() */
    S3_ERR_SCRATCH = -6    /* s3_decode_step_static: the call needs more chunk-partial scratch than the
                              library's fixed device buffer holds; nothing launched */
} s3_status;

typedef struct {
    int32_t n_layers;  /* l: transformer layers whose K and V the arena holds            */
    int32_t n_heads;   /* H                                                              */
    int32_t head_dim;  /* D: 64, 128 or 256; 96 for multi-head 16-bit caches (n_kv_heads 0 or
                          n_heads, kv_dtype S3_F16 / S3_BF16)                            */
    int32_t kv_dtype;  /* s3_dtype of the cache rows (and, if 16-bit, of q, k_new, v_new):
                          S3_F16, S3_BF16 or S3_E4M3                                     */
    int32_t granule;   /* G: capacities are multiples of G tokens (> 0)                  */
    int32_t max_len;   /* M: largest capacity, tokens; a multiple of G                   */
    int32_t n_kv_heads; /* heads of K and V: 0 or n_heads = one per query head; a divisor of n_heads =
                           grouped-query, 1 = multi-query attention (each K/V head serves
                           n_heads / n_kv_heads query heads; q and out keep n_heads)       */
    int32_t act_dtype; /* kv_dtype == S3_E4M3 only: type of q, k_new, v_new, S3_F16 or S3_BF16 (append
                          rounds a new row to the nearest e4m3 code, ties to even, saturating at
                          +-448, NaN -> 0x7f; attention widens the codes exactly).  Ignored for 16-bit
                          caches.  s3_kv_fill and s3_kv_read_rows move codes (one byte per
                          element).                                                       */
} s3_kv_config;

/* KV-cache bytes one token occupies: 2 * n_layers * n_kv_heads * head_dim * sizeof(element)
 * (section 2.1: 4*l*d_h bytes in half precision).  Returns the byte count, or
 * S3_ERR_INVALID (< 0) for a bad config. */
int64_t s3_kv_bytes_per_token(const s3_kv_config *cfg /*HOST*/);

/* The reservation rules as plain functions of a configuration (HOST integers; no arena needed).
 *   s3_kv_capacity_for     tokens reserved for a sequence predicted to reach predicted_len tokens in total
 *                          (sections 1 and 2.3: reserve what is predicted, not the maximum):
 *                          min(M, max(G, round_up(predicted_len, G)))
 *   s3_kv_grown_capacity   reservation owed to a sequence that used up `cap` tokens and is not finished
 *                          (section 3, supervisor paragraph: twice the memory): min(2*cap, M).  It is what
 *                          s3_kv_grow reserves, and what an evicted sequence is re-admitted with.
 * Both return S3_ERR_INVALID (< 0) for a bad config or a negative argument. */
int32_t s3_kv_capacity_for(const s3_kv_config *cfg /*HOST*/, int32_t predicted_len);
int32_t s3_kv_grown_capacity(const s3_kv_config *cfg /*HOST*/, int32_t cap);

/* Create the bookkeeping for one arena over caller-owned device memory.
 *   dev_base  DEVICE, 256-byte aligned, dev_bytes long; stays owned by the caller and must
 *             outlive the arena.  NULL = metadata-only arena: alloc/free/grow/stats work
 *             as integers (grow copies nothing), every call that touches rows returns
 *             S3_ERR_INVALID.  No HIP call is made for a metadata-only arena.
 *   capacity  = floor(dev_bytes / bytes_per_token) token rows.
 * The arena contents are not cleared.  *out receives the handle. */
int s3_kv_arena_init(s3_arena **out /*HOST*/, const s3_kv_config *cfg /*HOST*/, void *dev_base /*DEVICE*/,
                     size_t dev_bytes);

/* Frees host metadata and the library's own split-K scratch (synchronises the device
 * if such scratch exists).  Never touches dev_base.  NULL is allowed. */
void s3_kv_arena_destroy(s3_arena *a);

/* Reserve a slot per sequence by predicted length (sections 1 and 2.3; admission loop of
 * section 3, scheduler paragraph): in caller order, sequence i gets capacity
 *   cap = min(M, max(G, round_up(predicted_len[i], G)))
 * at the lowest-offset free extent that holds it (first fit), iff one exists; otherwise
 * slot_id[i] = -1, slot_off[i] = -1, slot_cap[i] = 0 and the loop goes on to i+1.
 *   predicted_len  HOST [n]  predicted TOTAL tokens (prompt + predicted output), >= 0
 *   slot_id        HOST [n]  out: id (smallest unused non-negative integer) or -1
 *   slot_off       HOST [n]  out: first token row of the slot
 *   slot_cap       HOST [n]  out: capacity in tokens
 * Returns the number admitted (>= 0), or S3_ERR_INVALID with state unchanged (n < 0, null
 * pointer, a negative prediction). */
int s3_kv_alloc(s3_arena *a, int32_t n, const int32_t *predicted_len, int32_t *slot_id, int64_t *slot_off,
                int32_t *slot_cap);

/* The sequence finished (iteration-level check of section 3): return its extent to the
 * free list, merging with free neighbours.  S3_ERR_INVALID for an id that is not live. */
int s3_kv_free(s3_arena *a, int32_t slot_id);

/* Offset and capacity of a live slot.  S3_ERR_INVALID if not live. */
int s3_kv_slot_info(const s3_arena *a, int32_t slot_id, int64_t *off /*HOST*/, int32_t *cap /*HOST*/);

/* Append-only fill of the reserved rows (section 2.2): for b in [0, n), write the new token's key
 * and value for `layer` into row pos[b] of the slot starting at slot_off[b].
 *   slot_id   HOST [n] or NULL, pos_host HOST [n] or NULL: when both are given the host checks
 *             BEFORE launching that every id is live, 0 <= pos_host[b], and pos_host[b] <
 *             capacity; pos_host[b] == capacity gives S3_ERR_SLOT_FULL (the sequence used up
 *             its reservation: call s3_kv_grow), anything else bad gives S3_ERR_INVALID; in
 *             both cases nothing is written.  When NULL the caller vouches for the positions.
 *   slot_off  DEVICE [n] int64, pos DEVICE [n] int32
 *   k_new, v_new  DEVICE [n][H][D] elements of kv_dtype (8-bit caches: of act_dtype, quantised here;
 *                 shared K/V heads: [n][n_kv_heads][D]), 16-byte aligned */
int s3_kv_append(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                 const int64_t *slot_off, const int32_t *pos, const void *k_new, const void *v_new,
                 void *stream);

/* Decode-step attention (section 2.1 equation, per head): for b in [0, n), h in [0, H)
 *   out[b][h][:] = softmax_j( scale * q[b][h][:] . K_b[j][h][:] ) . V_b[:][h][:],  j in [0, cur_len[b])
 * over the sequence's own rows only (no padding).  cur_len[b] == 0 gives a zero row.
 * Arithmetic is fp32 (dot products, max-subtracted softmax, weighted sum); contexts are
 * cut into chunks whose partial (max, sum, weighted sum) are merged by a second kernel.
 *   q         DEVICE [n][H][D] kv_dtype (8-bit caches: act_dtype), 16-byte aligned
 *   slot_off  DEVICE [n] int64, cur_len DEVICE [n] int32
 *   out       DEVICE [n][H][D] of out_dtype (S3_F32, S3_F16 or S3_BF16), 16-byte aligned
 *   scale     <= 0 means 1/sqrt(D)
 * May grow the library's scratch buffer with hipMalloc (which synchronises) the first time a
 * larger batch is seen; n <= 4095. */
int s3_decode_attention(s3_arena *a, int32_t layer, int32_t n, const void *q, const int64_t *slot_off,
                        const int32_t *cur_len, void *out, int32_t out_dtype, float scale, void *stream);

/* One layer-step (multi-head caches, 16-bit or 8-bit rows: in ONE kernel launch): exactly s3_kv_append(pos) followed by s3_decode_attention over
 * cur_len[b] = pos[b] + 1 rows (the new token attends to itself as well; section 2.1), same results,
 * same host-side checks (slot_id / pos_host as in s3_kv_append), same treatment of bad device entries.
 * The wave that owns the new row takes it from k_new / v_new and writes it into the arena; the
 * workgroup that delivers the last chunk of a context merges the chunks, so no second kernel runs.
 *   len_out   DEVICE [n] int32 or NULL: receives pos[b] + 1, the positions of the next step; must not
 *             be the same array as pos (S3_ERR_INVALID) - alternate between two arrays. */
/* (Shared key/value heads: the same call, results and checks, as two or three launches on `stream`: the
 * append (folded into the attention kernel when the matrix-core kernel runs over 16-bit rows), the
 * attention kernel, and a merge of chunk partials.  An 8-bit cache rounds the new row to codes in the
 * same kernel that attends over it.) */
int s3_decode_step(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                   const int64_t *slot_off, const int32_t *pos, const void *q, const void *k_new,
                   const void *v_new, void *out, int32_t out_dtype, float scale, int32_t *len_out, void *stream);

/* For callers that cannot allocate device memory: code recorded into a HIP graph, serving loops that must
 * never synchronise, harnesses that forbid hipMalloc.  Exactly s3_decode_step (same arguments, checks,
 * kernels and results), except that the chunk partials and arrival counters live in a fixed buffer that is
 * part of the library's device image (S3_STATIC_SCRATCH_BYTES = 32 MiB, held by every GPU the library runs
 * on until the process ends) instead of the arena's scratch: the call makes no hipMalloc, hipFree or other
 * allocating call and never synchronises.  A call that needs more - about
 * n * ceil(max_len / chunk) * n_heads * (4 * head_dim + 8) bytes plus the counters; 32 MiB hold the
 * 28-layer, 721-sequence GPT-J batch at the default chunk - returns S3_ERR_SCRATCH and launches nothing.
 * The "profile" parameter does not time these launches (its events are allocated).  All calls on one GPU,
 * from every arena, share the buffer and it keeps the last call's contents: the counters are left at zero
 * by every launch (and are cleared by a small kernel on `stream` whenever the previous call on this GPU laid
 * the buffer out differently), partials are always written before they are read; calls that overlap on one
 * GPU (two streams, two threads) race on it. */
int s3_decode_step_static(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                          const int64_t *slot_off, const int32_t *pos, const void *q, const void *k_new,
                          const void *v_new, void *out, int32_t out_dtype, float scale, int32_t *len_out,
                          void *stream);
#define S3_STATIC_SCRATCH_BYTES (32u << 20)

/* Size the arena's own scratch (chunk partials, arrival counters) once, for batches of up to max_batch
 * sequences at the current "chunk" setting, so that s3_decode_attention / s3_decode_step never allocate or
 * synchronise afterwards (they still grow it on demand for a larger batch or a smaller chunk).  Allocates
 * with hipMalloc and synchronises the device if the scratch must grow.  max_batch in [1, 4095]. */
int s3_kv_reserve_scratch(s3_arena *a, int32_t max_batch);

/* A sequence used up its reservation and is not finished: double it (section 3, supervisor
 * paragraph).  new capacity = min(2*cap, M); the new slot is placed first-fit while the old one is
 * still reserved (they never overlap); rows [0, len) of K and V of every layer are copied on
 * `stream`; the old extent is then released and the id keeps naming the sequence.
 *   S3_ERR_MAXLEN if cap == M, S3_ERR_NOMEM if no extent fits (state unchanged in both),
 *   S3_ERR_INVALID for a dead id or len outside [0, cap]. */
int s3_kv_grow(s3_arena *a, int32_t slot_id, int32_t len, int64_t *new_off /*HOST*/,
               int32_t *new_cap /*HOST*/, void *stream);

/* Compaction (section 3, supervisor paragraph: rows below a blank are shifted up so that everything is
 * stored contiguously again): every live slot slides down, in order of offset, to close the holes that
 * finished and relocated sequences left; afterwards the free space is one extent at the end.  Capacities
 * and ids do not change.
 *   slot_id, len  HOST [n]: slots whose first len[i] rows are to be preserved (the others' rows beyond
 *                 len are not copied); live slots that are not listed are moved whole
 *   new_off       HOST [n] out (may be NULL): offsets of the listed slots after compaction; use
 *                 s3_kv_slot_info for the rest.  The caller must refresh its device slot_off[] arrays.
 *   n_moved       HOST out (may be NULL): slots that changed place
 * Copies run on `stream` in order (overlapping moves are cut into pieces that never overwrite rows not
 * yet moved).  S3_ERR_INVALID (nothing changed) for a dead id or len outside [0, cap]. */
int s3_kv_compact(s3_arena *a, int32_t n, const int32_t *slot_id, const int32_t *len, int64_t *new_off,
                  int32_t *n_moved, void *stream);

/* Eviction to the host and reload (the paper's own handling of a sequence that used up its reservation,
 * section 3, supervisor paragraph; its cost is the "penalty" of section 4.3).  Use when s3_kv_grow
 * answers S3_ERR_NOMEM, or to make room for others.
 *   s3_kv_evict_bytes  bytes of host memory needed for len rows of every plane (< 0: bad argument)
 *   s3_kv_evict        copies rows [0, len) of K and V of every layer to host_buf (HOST, pinned memory
 *                      makes the copies asynchronous; layout [2*n_layers][len][H][D]) on `stream`, then
 *                      frees the slot.  host_buf is complete once the stream has passed the copies.
 *   s3_kv_restore      reserves a slot for predicted_len (>= len; the paper doubles the old reservation),
 *                      copies the rows back on `stream`; returns the new id / offset / capacity.
 *                      S3_ERR_NOMEM if nothing fits (state unchanged). */
int64_t s3_kv_evict_bytes(const s3_arena *a, int32_t len);
int s3_kv_evict(s3_arena *a, int32_t slot_id, int32_t len, void *host_buf /*HOST*/, void *stream);
int s3_kv_restore(s3_arena *a, int32_t predicted_len, int32_t len, const void *host_buf /*HOST*/,
                  int32_t *slot_id /*HOST out*/, int64_t *slot_off /*HOST out*/, int32_t *slot_cap /*HOST out*/,
                  void *stream);

/* The device-side halves of the same eviction and re-admission (section 3, supervisor paragraph), for callers
 * that keep the host link off the decode stream: the rows are first gathered into a contiguous DEVICE buffer
 * (one kernel; the slot can be freed right behind it in stream order and its room reused at once), cross the
 * link in one copy on another stream, and come back the same way.
 *   s3_kv_gather_rows   rows [0, len) of K and V of every layer of a live slot -> dev_buf (DEVICE, 16-byte
 *                       aligned, s3_kv_evict_bytes(len) bytes, layout [2*n_layers][len][H][D] as host_buf of
 *                       s3_kv_evict); the slot stays live (free it with s3_kv_free)
 *   s3_kv_scatter_rows  the inverse: dev_buf -> rows [0, len) of every plane of a live slot (reserve it with
 *                       s3_kv_alloc for the reservation the sequence is owed, see s3_kv_grown_capacity)
 * S3_ERR_INVALID for a dead id, len outside [0, cap] or a misaligned buffer. */
int s3_kv_gather_rows(s3_arena *a, int32_t slot_id, int32_t len, void *dev_buf /*DEVICE*/, void *stream);
int s3_kv_scatter_rows(s3_arena *a, int32_t slot_id, int32_t len, const void *dev_buf /*DEVICE*/, void *stream);

/* The link half of a staged eviction or re-admission: copy `bytes` (a multiple of 16; both pointers 16-byte
 * aligned) between a DEVICE buffer and pinned HOST memory that the device can address (memory from hipHostMalloc,
 * which torch's pinned tensors are), in either direction, with a kernel of `workgroups` workgroups (1..1024) on
 * `stream`.  Each workgroup takes a whole compute unit (it reserves the unit's LDS).  Few workgroups keep few
 * writes queued for the link at once, which is what lets decode steps run beside the copy undisturbed: two reach
 * about 30 GB/s and leave an attention kernel at full speed, eight reach the link's 55 GB/s and slow whatever runs
 * beside the copy's first milliseconds several times over (as the runtime's own copy kernels do).
 * The caller vouches for both ranges (they cannot be checked here). */
int s3_kv_link_copy(void *dst /*DEVICE or pinned HOST*/, const void *src /*DEVICE or pinned HOST*/, size_t bytes,
                    int32_t workgroups, void *stream);

/* The supervisor's report of available memory (section 3), in tokens.  Any out pointer may be NULL. */
int s3_kv_stats(const s3_arena *a, int64_t *used_tok, int64_t *free_tok, int64_t *largest_free_tok,
                int64_t *capacity_tok);

/* Bulk write of rows [first_row, first_row+n_rows) of a live slot for one layer: the stand-in for
 * the prompt phase.  k_rows, v_rows: DEVICE [n_rows][H][D] kv_dtype, 16-byte aligned.
 * S3_ERR_SLOT_FULL if first_row + n_rows > capacity. */
int s3_kv_fill(s3_arena *a, int32_t slot_id, int32_t layer, int32_t first_row, int32_t n_rows,
               const void *k_rows, const void *v_rows, void *stream);

/* Admission of several newcomers in one launch (iteration-level scheduling, section 3: finished
 * sequences are replaced between two decode steps): exactly n_new s3_kv_fill calls with first_row 0
 * and, if slot_off / len are given, the s3_kv_batch_patch that puts newcomer i into entry
 * batch_idx[i] of the running batch (its slot's offset, its n_rows[i] as the length).  All arguments
 * are checked before anything is enqueued.
 *   slot_id, n_rows HOST [n_new]; k_rows, v_rows HOST [n_new] arrays of DEVICE pointers to
 *   [n_rows[i]][H][D] rows of the cache type, 16-byte aligned
 *   slot_off DEVICE [batch_n] int64 and len DEVICE [batch_n] int32, or both NULL; batch_idx HOST [n_new] */
int s3_kv_fill_batch(s3_arena *a, int32_t layer, int32_t n_new, const int32_t *slot_id, const int32_t *n_rows,
                     const void *const *k_rows, const void *const *v_rows, int32_t batch_n, int64_t *slot_off,
                     int32_t *len, const int32_t *batch_idx, void *stream);

/* For callers that keep slot_off[] / len[] of the running batch in device memory: rewrite n_updates
 * entries (a grown slot's new offset, a newcomer that took a finished sequence's place) without a
 * host-to-device copy; the values travel as kernel arguments.  Stream-ordered like everything else.
 *   slot_off DEVICE [n] int64 or NULL, len DEVICE [n] int32 or NULL (at least one given)
 *   idx HOST [n_updates] entries in [0, n); new_off / new_len HOST [n_updates] (needed for the array given) */
int s3_kv_batch_patch(int32_t n, int64_t *slot_off, int32_t *len, int32_t n_updates, const int32_t *idx,
                      const int64_t *new_off, const int32_t *new_len, void *stream);

/* Copy rows [first_row, first_row+n_rows) of K (which = 0) or V (which = 1) of a live slot into
 * dst, DEVICE [n_rows][H][D] kv_dtype, 16-byte aligned.  For bit-exact checks of append / grow. */
int s3_kv_read_rows(s3_arena *a, int32_t slot_id, int32_t layer, int32_t which, int32_t first_row,
                    int32_t n_rows, void *dst, void *stream);

/* Length-aware scheduler (section 3, scheduler paragraph; host integers only).  A request pool plus the
 * decreasing-first-fit pass: the pool is ordered by the capacity each request would reserve, largest
 * first (equal sizes in arrival order), and walked once; a request joins the batch iff s3_kv_alloc
 * finds room for it; the walk ends when no token of the arena is free, when max_out requests have been
 * admitted, or at the end of the pool.  Call s3_sched_admit again at every iteration, after the finished
 * sequences were freed (iteration-level scheduling, same section).
 *   s3_sched_submit    put a request (caller's id, predicted TOTAL length) into the pool
 *   s3_sched_admit     request_id / slot_id / slot_off / slot_cap: HOST [max_out] out; returns the number
 *                      admitted (they leave the pool), or an error (< 0)
 *   s3_sched_pool_size requests still waiting */
typedef struct s3_sched s3_sched;
int s3_sched_create(s3_sched **out /*HOST*/, s3_arena *a);
void s3_sched_destroy(s3_sched *s);
int s3_sched_submit(s3_sched *s, int64_t request_id, int32_t predicted_len);
int s3_sched_admit(s3_sched *s, int32_t max_out, int64_t *request_id, int32_t *slot_id, int64_t *slot_off,
                   int32_t *slot_cap);
int s3_sched_pool_size(const s3_sched *s);

/* Measurement aid: the rate a plain streaming kernel reaches over the first `bytes` of the arena
 * (mode 0: 128-bit reads only, in the attention kernels' pattern - 1 KiB pieces of 8 KiB rows -, `bytes`
 * rounded down to a multiple of 1 MiB and at least that; mode 1: copy of the first `bytes` onto the next
 * `bytes`, counted as 2*bytes moved), averaged over `reps` back-to-back launches on the default stream, in GB/s.
 * DESTROYS arena contents in mode 1.  Synchronises the device.  Says what fraction of the nominal
 * HBM peak is attainable at all, next to the attention kernel's own figure. */
int s3_kv_probe_bandwidth(s3_arena *a, size_t bytes, int32_t mode, int32_t reps, double *gbps /*HOST*/);

/* Launch-shape knobs of the attention kernels and measurement switches.  set names:
 *   "chunk"        tokens per split-K chunk (multiple of 32, 32..2048; 0 = library default)
 *   "classes"      length classes of the longest-first work order (1..8; 0 = library default); a batch of
 *                  thousands of sequences keeps as many as fit the workgroup's memory
 *   "grid_blocks"  workgroups launched (0 = library default)
 *   "variant"      kernel variant index, -1 = default (see get "n_variants"; arenas with shared
 *                  key/value heads have their own, shorter, list)
 *   "merge_sync"   how chunks of one context that meet inside ONE launch (s3_decode_step on multi-head
 *                  caches, 8-bit rows) are ordered across workgroups: 0 (default) write-through partial
 *                  stores, a drained memory counter and a relaxed counter increment; 1 device-scope
 *                  release / acquire fences around the increment (slower; same results)
 *   "gqa_merge"    shared key/value heads, matrix-core kernel: 1 = multi-chunk contexts are finished inside the
 *                  attention launch (arrival counters, write-through partials), 0 (default) = by a merge launch;
 *                  same results; the launch-saving form measured slower (its partials bypass the caches)
 *   "gqa_dynamic"  shared key/value heads, matrix-core kernel: per cent of the work list that is dealt by stride
 *                  before the waves claim the remaining positions from a device-wide counter (1..99; 0, 100 or -1,
 *                  the default = all by stride: claims pay only on very long lists of long items); same results
 *   "gqa_stream"   shared key/value heads, matrix-core kernel: how K rows are read: 1 = with the streaming hint
 *                  (whole rows per load, operand layout through LDS), 0 = plain loads straight into operand layout,
 *                  -1 (default) = 1 if the launch's K rows exceed the 256 MB memory-side cache, else 0; same results
 *   "profile"      k > 0: every k-th attention launch (counted from this call) carries HIP events that
 *                  take the kernel's own start and end times (hipExtLaunchKernel); 0: off; both reset the sums
 * get names: the above plus "default_variant", "kernel_kind" (0 multi-head kernels, 1 shared-K/V vector-ALU kernel,
 * 2 shared-K/V matrix-core kernel, 3 kernel for 8-bit rows, 4 matrix-core kernel over 8-bit rows with
 * shared heads: what the next attention launch uses), "n_variants", "n_grows",
 * "live_slots", "scratch_bytes", "num_cus" and,
 * after "profile" k, "profile_launches", "profile_partial_ns", "profile_merge_ns" (sums over the
 * timed launches since the last reset) and "profile_p10_ns", "profile_p50_ns", "profile_p90_ns"
 * (nearest-rank percentiles of the attention kernel's duration); reading them waits for
 * the recorded events.
 * Returns S3_ERR_INVALID for an unknown name or a value out of range. */
int s3_kv_set_param(s3_arena *a, const char *name /*HOST*/, int64_t value);
int s3_kv_get_param(const s3_arena *a, const char *name /*HOST*/, int64_t *value /*HOST*/);

/* Text of the last HIP error seen by this thread's calls ("" if none), and of a status code. */
const char *s3_last_hip_error(void);
const char *s3_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* S3KV_H */
