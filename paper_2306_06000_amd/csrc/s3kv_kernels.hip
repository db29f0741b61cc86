// Launch code of libs3kv for gfx950 (MI355X) and its small kernels: append, plane copies (grow / fill /
// read-back), batch patches, the bandwidth probe, and the host side of every attention call.  The attention
// kernels live in s3kv_attn.h (multi-head 16-bit caches; instantiated per head dimension by
// s3kv_attn_inst.hip), s3kv_gqa.hip, s3kv_gqa_mfma.hip (shared key/value heads) and s3kv_fp8.hip (8-bit
// rows) and are launched from here; the device helpers all of them share are in s3kv_device.h.
//
// Arena layout.  Plane p = 2*layer + (0: K, 1: V) holds N token rows of H*D elements (H = cached
// heads), token-major: element (token t, head h, d) of a plane sits at ((t*H + h)*D + d).  A slot
// is the row range [off, off+cap) in EVERY plane, so one sequence's rows of one plane are one
// contiguous run and the attention kernels stream them with 128-bit loads.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <map>
#include <mutex>

#include "s3kv_internal.h"

#include "s3kv_device.h"

static int hip_fail(const char *what, hipError_t e) {
    s3i_set_hip_error(what, (int)e, hipGetErrorString(e));
    return S3_ERR_HIP;
}
#define HIP_TRY(call)                                     \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) return hip_fail(#call, e_); \
    } while (0)

int s3i_device_cus(int32_t *cus) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    int n = 0;
    HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    *cus = n;
    return S3_OK;
}

// ------------------------------------------------------------------------------------------
// plane copies
// ------------------------------------------------------------------------------------------
// blockIdx.y = plane; each thread moves 16-byte pieces; nbytes is a multiple of 16.
__global__ void __launch_bounds__(256) copy_planes_kernel(const char *src, char *dst, size_t n16,
                                                          size_t src_plane_stride, size_t dst_plane_stride) {
    const u32x4 *s = (const u32x4 *)(src + (size_t)blockIdx.y * src_plane_stride);
    u32x4 *d = (u32x4 *)(dst + (size_t)blockIdx.y * dst_plane_stride);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) d[i] = s[i];
}

// Two independent copies in one launch (blockIdx.y picks the pair): the K and V rows of a fill.
__global__ void __launch_bounds__(256) copy_pair_kernel(const char *src0, char *dst0, const char *src1, char *dst1,
                                                        size_t n16) {
    const u32x4 *s = (const u32x4 *)(blockIdx.y ? src1 : src0);
    u32x4 *d = (u32x4 *)(blockIdx.y ? dst1 : dst0);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) d[i] = s[i];
}

// Rewrite a few entries of the per-batch device arrays; the new values travel as kernel arguments.
#define S3_PATCH_MAX 32
struct PatchArgs {
    int64_t off[S3_PATCH_MAX];
    int32_t idx[S3_PATCH_MAX];
    int32_t len[S3_PATCH_MAX];
    int32_t count;
};
__global__ void __launch_bounds__(64) batch_patch_kernel(int64_t *slot_off, int32_t *len, const PatchArgs p) {
    const int i = threadIdx.x;
    if (i < p.count) {
        if (slot_off) slot_off[p.idx[i]] = p.off[i];
        if (len) len[p.idx[i]] = p.len[i];
    }
}

extern "C" int s3_kv_batch_patch(int32_t n, int64_t *slot_off, int32_t *len, int32_t n_updates, const int32_t *idx,
                                 const int64_t *new_off, const int32_t *new_len, void *stream) {
    if (n < 0 || n_updates < 0 || (!slot_off && !len)) return S3_ERR_INVALID;
    if (n_updates == 0) return S3_OK;
    if (!idx || (slot_off && !new_off) || (len && !new_len)) return S3_ERR_INVALID;
    for (int32_t i = 0; i < n_updates; i++)
        if (idx[i] < 0 || idx[i] >= n) return S3_ERR_INVALID;
    for (int32_t first = 0; first < n_updates; first += S3_PATCH_MAX) {
        PatchArgs p;
        p.count = n_updates - first < S3_PATCH_MAX ? n_updates - first : S3_PATCH_MAX;
        for (int32_t i = 0; i < p.count; i++) {
            p.idx[i] = idx[first + i];
            p.off[i] = new_off ? new_off[first + i] : 0;
            p.len[i] = new_len ? new_len[first + i] : 0;
        }
        hipLaunchKernelGGL(batch_patch_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, slot_off, len, p);
        HIP_TRY(hipGetLastError());
    }
    return S3_OK;
}

// Admission of several newcomers in one launch: their prompt rows (K and V of one layer) and, optionally,
// their entries of the running batch's device arrays.  Everything travels as kernel arguments.
#define S3_FILL_MAX 16
struct FillArgs {
    const char *ksrc[S3_FILL_MAX];
    const char *vsrc[S3_FILL_MAX];
    char *kdst[S3_FILL_MAX];
    char *vdst[S3_FILL_MAX];
    int64_t off[S3_FILL_MAX];
    uint64_t n16[S3_FILL_MAX];  // 16-byte pieces of one plane's rows (max_len rows of up to 64 KiB reach 2^32)
    int32_t idx[S3_FILL_MAX];
    int32_t rows[S3_FILL_MAX];
};
// grid (x, 2, entries): blockIdx.z picks the newcomer, blockIdx.y K or V, the x blocks stride over its rows.
__global__ void __launch_bounds__(256) fill_batch_kernel(const FillArgs f, int64_t *slot_off, int32_t *len) {
    const int z = blockIdx.z;
    const u32x4 *s = (const u32x4 *)(blockIdx.y ? f.vsrc[z] : f.ksrc[z]);
    u32x4 *d = (u32x4 *)(blockIdx.y ? f.vdst[z] : f.kdst[z]);
    const size_t n16 = f.n16[z], stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) d[i] = s[i];
    if (slot_off && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        slot_off[f.idx[z]] = f.off[z];
        len[f.idx[z]] = f.rows[z];
    }
}

extern "C" int s3_kv_fill_batch(s3_arena *a, int32_t layer, int32_t n_new, const int32_t *slot_id, const int32_t *n_rows,
                                const void *const *k_rows, const void *const *v_rows, int32_t batch_n,
                                int64_t *slot_off, int32_t *len, const int32_t *batch_idx, void *stream) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n_new < 0) return S3_ERR_INVALID;
    if (n_new == 0) return S3_OK;
    if (!slot_id || !n_rows || !k_rows || !v_rows) return S3_ERR_INVALID;
    const bool patch = slot_off || len;
    if (patch && (!slot_off || !len || !batch_idx || batch_n <= 0)) return S3_ERR_INVALID;
    for (int32_t i = 0; i < n_new; i++) {  // everything is checked before anything is enqueued
        const s3_slot *s = s3i_live_slot(a, slot_id[i]);
        if (!s || n_rows[i] < 0) return S3_ERR_INVALID;
        if (n_rows[i] > s->cap) return S3_ERR_SLOT_FULL;
        if (n_rows[i] > 0 && (!k_rows[i] || !v_rows[i] || ((uintptr_t)k_rows[i] & 15) || ((uintptr_t)v_rows[i] & 15)))
            return S3_ERR_INVALID;
        if (patch && (batch_idx[i] < 0 || batch_idx[i] >= batch_n)) return S3_ERR_INVALID;
    }
    for (int32_t first = 0; first < n_new; first += S3_FILL_MAX) {
        FillArgs f;
        memset(&f, 0, sizeof(f));
        const int count = n_new - first < S3_FILL_MAX ? n_new - first : S3_FILL_MAX;
        size_t most = 1;
        for (int i = 0; i < count; i++) {
            const s3_slot *s = s3i_live_slot(a, slot_id[first + i]);
            const size_t n16 = (size_t)n_rows[first + i] * a->row_bytes / 16;
            f.ksrc[i] = (const char *)k_rows[first + i];
            f.vsrc[i] = (const char *)v_rows[first + i];
            f.kdst[i] = a->plane(layer, 0) + s->off * a->row_bytes;
            f.vdst[i] = a->plane(layer, 1) + s->off * a->row_bytes;
            f.n16[i] = n16;
            f.off[i] = s->off;
            f.idx[i] = patch ? batch_idx[first + i] : 0;
            f.rows[i] = n_rows[first + i];
            if (n16 > most) most = n16;
        }
        size_t blocks = (most + 1023) / 1024;
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(fill_batch_kernel, dim3((unsigned)blocks, 2, (unsigned)count), dim3(256), 0, (hipStream_t)stream,
                           f, patch ? slot_off : nullptr, patch ? len : nullptr);
        HIP_TRY(hipGetLastError());
    }
    return S3_OK;
}

int s3i_launch_copy_planes(const char *src, char *dst, size_t nbytes, size_t src_plane_stride,
                           size_t dst_plane_stride, int planes, void *stream) {
    if (nbytes == 0 || planes <= 0) return S3_OK;
    if ((nbytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return S3_ERR_INVALID;
    const size_t n16 = nbytes / 16;
    size_t blocks = (n16 + 1023) / 1024;  // four pieces per thread
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(copy_planes_kernel, dim3((unsigned)blocks, (unsigned)planes), dim3(256), 0,
                       (hipStream_t)stream, src, dst, n16, src_plane_stride, dst_plane_stride);
    HIP_TRY(hipGetLastError());
    return S3_OK;
}

// ------------------------------------------------------------------------------------------
// bandwidth probe: what a plain streaming kernel reaches on this device, to put the attention
// kernel's number next to (the attainable HBM rate is below the nominal peak)
// ------------------------------------------------------------------------------------------
static int ensure_scratch(s3_arena *a, size_t need);

// The buffer is read as the attention kernels read a cache: rows of 8 KiB, a wave streams one 1 KiB piece of 128
// consecutive rows, eight non-temporal 128-bit loads per lane in flight; neighbouring waves take neighbouring pieces
// of the same rows.  (A grid-stride loop over the whole buffer, four loads in flight, read 20 % slower here.)
#define S3_PROBE_ROW 8192
#define S3_PROBE_ROWS 128
__global__ void __launch_bounds__(256) read_probe_kernel(const char *src, size_t n_items, unsigned int *sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t item = (size_t)blockIdx.x * 4 + wave; item < n_items; item += (size_t)gridDim.x * 4) {
        const char *base = src + (item / 8) * ((size_t)S3_PROBE_ROWS * S3_PROBE_ROW) + (item % 8) * 1024 + lane * 16;
        for (int r = 0; r < S3_PROBE_ROWS; r += 8) {
            u32x4 v[8];
#pragma unroll
            for (int i = 0; i < 8; i++) v[i] = __builtin_nontemporal_load((const u32x4 *)(base + (size_t)(r + i) * S3_PROBE_ROW));
#pragma unroll
            for (int i = 0; i < 8; i++) acc ^= v[i];
        }
    }
    const unsigned int x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9E3779B9u) *sink = x;  // practically never: keeps the loads alive
}

extern "C" int s3_kv_probe_bandwidth(s3_arena *a, size_t bytes, int32_t mode, int32_t reps, double *gbps) {
    if (!a || !a->base || !gbps || reps <= 0 || (mode != 0 && mode != 1)) return S3_ERR_INVALID;
    // mode 0 reads whole blocks of 128 rows of 8 KiB (1 MiB); a smaller request reads nothing and is refused
    bytes = mode == 0 ? bytes / ((size_t)S3_PROBE_ROWS * S3_PROBE_ROW) * ((size_t)S3_PROBE_ROWS * S3_PROBE_ROW) : bytes & ~(size_t)15;
    if (bytes == 0 || (mode == 0 ? bytes : 2 * bytes) > a->dev_bytes) return S3_ERR_INVALID;
    const int rc = ensure_scratch(a, 256);
    if (rc != S3_OK) return rc;
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    HIP_TRY(hipEventCreate(&e1));
    const size_t n16 = bytes / 16;
    const int cus = a->num_cus > 0 ? a->num_cus : 256;
    for (int r = -2; r < reps; r++) {  // two untimed warm-up passes
        if (r == 0) HIP_TRY(hipEventRecord(e0, nullptr));
        if (mode == 0) {
            hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)(cus * 2)), dim3(256), 0, nullptr, a->base,
                               bytes / ((size_t)S3_PROBE_ROWS * 1024), (unsigned int *)((char *)a->scratch + 128));
        } else {
            hipLaunchKernelGGL(copy_planes_kernel, dim3((unsigned)(cus * 8), 1), dim3(256), 0, nullptr, a->base,
                               a->base + bytes, n16, (size_t)0, (size_t)0);
        }
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipEventRecord(e1, nullptr));
    HIP_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *gbps = (double)(mode == 0 ? bytes : 2 * bytes) * reps / (ms * 1e-3) / 1e9;
    return S3_OK;
}

// ------------------------------------------------------------------------------------------
// append
// ------------------------------------------------------------------------------------------
// grid (n, 2): block (b, which) copies one row of H*D elements into row off+pos of the plane.
__global__ void __launch_bounds__(256) append_kernel(char *kplane, char *vplane, const int64_t *slot_off,
                                                     const int32_t *pos, const char *k_new, const char *v_new,
                                                     int64_t row_bytes, int64_t n_tokens, int32_t max_len) {
    const int b = blockIdx.x;
    const int64_t off = slot_off[b];
    const int64_t p = pos[b];
    if (off < 0 || p < 0 || p >= max_len || off + p >= n_tokens) return;  // never leave the arena
    const u32x4 *s = (const u32x4 *)((blockIdx.y ? v_new : k_new) + (int64_t)b * row_bytes);
    u32x4 *d = (u32x4 *)((blockIdx.y ? vplane : kplane) + (off + p) * row_bytes);
    const int n16 = (int)(row_bytes >> 4);
    for (int i = threadIdx.x; i < n16; i += 256) d[i] = s[i];
}

// ------------------------------------------------------------------------------------------
// attention: kernel choice and launchers
// ------------------------------------------------------------------------------------------
// Multi-head kernels, one translation unit per head dimension (s3kv_attn_inst.hip).
attn_fn s3i_pick_mha_d64(int dt, int variant, bool fused);
attn_fn s3i_pick_mha_d96(int dt, int variant, bool fused);
attn_fn s3i_pick_mha_d128(int dt, int variant, bool fused);
attn_fn s3i_pick_mha_d256(int dt, int variant, bool fused);
attn_fn s3i_pick_merge_d64();
attn_fn s3i_pick_merge_d96();
attn_fn s3i_pick_merge_d128();
attn_fn s3i_pick_merge_d256();
int s3i_default_variant();
int s3i_default_variant_large();
int s3i_variant_threads(int variant, bool fused);
int s3i_variant_ring_bytes(int variant);
int s3i_variant_dynamic(int variant);
int s3i_variant_stream(int variant);

static attn_fn pick_kernel(int dt, int d, int variant, bool fused) {
    switch (d) {
        case 64: return s3i_pick_mha_d64(dt, variant, fused);
        case 96: return s3i_pick_mha_d96(dt, variant, fused);
        case 128: return s3i_pick_mha_d128(dt, variant, fused);
        case 256: return s3i_pick_mha_d256(dt, variant, fused);
        default: return nullptr;
    }
}

static attn_fn pick_merge(int d) {
    return d == 64 ? s3i_pick_merge_d64() : d == 96 ? s3i_pick_merge_d96() : d == 128 ? s3i_pick_merge_d128()
                                                                                       : s3i_pick_merge_d256();
}

// Heads that one 128-bit wave load of 16-bit elements covers: 512/D, except that a 96-wide head takes a
// group of sixteen lanes of which twelve are used (four heads per load).
static int heads_per_load(int d) { return d == 96 ? 4 : 512 / d; }

static int ensure_scratch(s3_arena *a, size_t need) {
    if (need <= a->scratch_bytes) return S3_OK;
    if (a->scratch) {
        HIP_TRY(hipDeviceSynchronize());
        HIP_TRY(hipFree(a->scratch));
        a->scratch = nullptr;
        a->scratch_bytes = 0;
    }
    HIP_TRY(hipMalloc(&a->scratch, need));
    a->scratch_bytes = need;
    HIP_TRY(hipMemset(a->scratch, 0, need));  // the arrival counters at its head must start at zero
    return S3_OK;
}

// ---- the fixed scratch of s3_decode_step_static ------------------------------------------
// Part of the library's device image: every GPU that loads the library holds its own copy at its own
// address until the process ends.  In host code the array's name is only a handle for the runtime; the
// device address is asked for once per device (with that device current) and only that address is ever
// handed to kernels.
static __device__ __align__(256) unsigned char s3_static_scratch[S3_STATIC_SCRATCH_BYTES];

#define S3_MAX_DEVICES 64
struct StaticScratch {
    void *ptr = nullptr;      // device address of s3_static_scratch on this device
    size_t counter_bytes = 0; // counter region of the last call on this device (0: none yet)
};
static StaticScratch g_static[S3_MAX_DEVICES];
static std::mutex g_static_guard;

__global__ void __launch_bounds__(256) zero_words_kernel(unsigned int *p, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

// The current device's entry, with the buffer's device address resolved (once per device).  Caller holds the guard.
static int static_scratch_entry(StaticScratch **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= S3_MAX_DEVICES) return S3_ERR_INVALID;
    StaticScratch &st = g_static[dev];
    if (!st.ptr) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(s3_static_scratch)));
        if (!p || ((uintptr_t)p & 255)) return S3_ERR_INVALID;
        st.ptr = p;
    }
    *out = &st;
    return S3_OK;
}

// Called when an arena is created over device memory: the address is then known before the first decode step
// (which may run where no runtime query is wanted, e.g. under graph capture).
int s3i_static_scratch_setup() {
    std::lock_guard<std::mutex> lock(g_static_guard);
    StaticScratch *st = nullptr;
    return static_scratch_entry(&st);
}

// Address of the current device's fixed scratch, laid out with cnt_bytes of arrival counters at its head.
// The counters must be zero before a launch.  Every launch leaves them at zero, but the region may hold
// partials of a call that laid the buffer out with fewer counter bytes (another arena kind): whenever the
// counter region differs from the last call's on this device (the first call included) it is cleared by a
// kernel on `stream` (a kernel, not a memset, so that the call can be recorded into a graph).
static int static_scratch_for_call(size_t cnt_bytes, void *stream, char **out) {
    std::lock_guard<std::mutex> lock(g_static_guard);
    StaticScratch *entry = nullptr;
    const int src = static_scratch_entry(&entry);
    if (src != S3_OK) return src;
    StaticScratch &st = *entry;
    if (cnt_bytes != st.counter_bytes) {
        const size_t clear = cnt_bytes > st.counter_bytes ? cnt_bytes : st.counter_bytes;
        if (clear > 0) {
            const size_t words = clear / sizeof(unsigned int);
            hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((words + 1023) / 1024)), dim3(256), 0,
                               (hipStream_t)stream, (unsigned int *)st.ptr, words);
            HIP_TRY(hipGetLastError());
        }
        st.counter_bytes = cnt_bytes;
    }
    *out = (char *)st.ptr;
    return S3_OK;
}

// ---- optional event timing of the attention kernels -------------------------------------
static int prof_next_event(s3_arena *a, hipEvent_t *ev) {
    if (a->prof_used == a->prof_events.size()) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        a->prof_events.push_back((void *)e);
    }
    *ev = (hipEvent_t)a->prof_events[a->prof_used++];
    return S3_OK;
}

int s3i_profile_collect(s3_arena *a) {
    for (size_t i = 0; i + 2 < a->prof_used; i += 3) {
        hipEvent_t e0 = (hipEvent_t)a->prof_events[i], e1 = (hipEvent_t)a->prof_events[i + 1],
                   e2 = (hipEvent_t)a->prof_events[i + 2];
        HIP_TRY(hipEventSynchronize(e2));
        float p = 0.f, m = 0.f;
        HIP_TRY(hipEventElapsedTime(&p, e0, e1));
        HIP_TRY(hipEventElapsedTime(&m, e1, e2));
        a->prof_partial_ms += p;
        a->prof_merge_ms += m;
        a->prof_launches++;
        a->prof_durations_ms.push_back(p);
    }
    a->prof_used = 0;
    return S3_OK;
}

void s3i_profile_reset(s3_arena *a) {
    (void)s3i_profile_collect(a);
    a->prof_partial_ms = a->prof_merge_ms = 0.0;
    a->prof_launches = 0;
    a->prof_durations_ms.clear();
    // events are created here, not at the first timed launch: creating one costs tens of microseconds
    while (a->prof_events.size() < 3 * 64) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) break;
        a->prof_events.push_back((void *)e);
    }
}

extern "C" void s3_kv_arena_destroy(s3_arena *a) {
    if (!a) return;
    if (!a->prof_events.empty()) {
        (void)hipDeviceSynchronize();
        for (void *e : a->prof_events) (void)hipEventDestroy((hipEvent_t)e);
    }
    if (a->scratch) {
        (void)hipDeviceSynchronize();
        (void)hipFree(a->scratch);
    }
    delete a;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// The append of one layer: a bit copy of the new rows, or, for 8-bit caches, their quantisation.
static int launch_append(s3_arena *a, int32_t layer, int32_t n, const int64_t *slot_off, const int32_t *pos,
                         const void *k_new, const void *v_new, void *stream) {
    if (a->cfg.kv_dtype == S3_E4M3) {
        append_fp8_fn fn = s3i_pick_append_fp8(a->cfg.act_dtype);
        if (!fn) return S3_ERR_INVALID;
        hipLaunchKernelGGL(fn, dim3((unsigned)n, 2), dim3(256), 0, (hipStream_t)stream, a->plane(layer, 0),
                           a->plane(layer, 1), slot_off, pos, (const char *)k_new, (const char *)v_new,
                           (int32_t)a->row_bytes, a->n_tokens, a->cfg.max_len);
    } else {
        hipLaunchKernelGGL(append_kernel, dim3((unsigned)n, 2), dim3(256), 0, (hipStream_t)stream, a->plane(layer, 0),
                           a->plane(layer, 1), slot_off, pos, (const char *)k_new, (const char *)v_new, a->row_bytes,
                           a->n_tokens, a->cfg.max_len);
    }
    HIP_TRY(hipGetLastError());
    return S3_OK;
}
static int check_slots_host(const s3_arena *a, int32_t n, const int32_t *slot_id, const int32_t *pos_host);

extern "C" int s3_kv_append(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                            const int64_t *slot_off, const int32_t *pos, const void *k_new, const void *v_new,
                            void *stream) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n < 0) return S3_ERR_INVALID;
    if (n == 0) return S3_OK;
    if (!slot_off || !pos || !k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return S3_ERR_INVALID;
    const int rc = check_slots_host(a, n, slot_id, pos_host);
    if (rc != S3_OK) return rc;
    return launch_append(a, layer, n, slot_off, pos, k_new, v_new, stream);
}

static int check_slots_host(const s3_arena *a, int32_t n, const int32_t *slot_id, const int32_t *pos_host) {
    if (!slot_id || !pos_host) return S3_OK;  // the caller vouches for the positions
    bool full = false;
    for (int32_t b = 0; b < n; b++) {
        const s3_slot *s = s3i_live_slot(a, slot_id[b]);
        if (!s || pos_host[b] < 0 || pos_host[b] > s->cap) return S3_ERR_INVALID;
        if (pos_host[b] == s->cap) full = true;
    }
    return full ? S3_ERR_SLOT_FULL : S3_OK;
}

// Workgroups of `fn` (threads per workgroup, dynamic LDS bytes) that one CU holds at once.  Asked
// from the runtime once per kernel and LDS size class (4 KiB steps).
static int resident_per_cu(const void *fn, int threads, size_t dyn_lds, int *per_cu) {
    static std::map<std::pair<const void *, size_t>, int> resident;  // (kernel, LDS in 4 KiB) -> workgroups per CU
    static std::mutex guard;  // shared by all arenas, which may live on different threads
    std::lock_guard<std::mutex> lock(guard);
    const std::pair<const void *, size_t> key(fn, (dyn_lds + 4095) / 4096);
    auto it = resident.find(key);
    if (it == resident.end()) {
        if (dyn_lds > 16384)
            HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(key.second * 4096)));
        int got = 0;
        HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&got, fn, threads, key.second * 4096));
        if (got < 1) return S3_ERR_INVALID;  // does not fit the device at all
        it = resident.emplace(key, got).first;
    }
    *per_cu = it->second;
    return S3_OK;
}

// One attention call as the entry points hand it over.  with_append: s3_decode_step (len_or_pos is the
// append position, the kernels attend over pos + 1 rows and publish len_out).
struct AttnCall {
    int32_t layer, n;
    const void *q;
    const int64_t *slot_off;
    const int32_t *len_or_pos;
    void *out;
    int32_t out_dtype;
    float scale;
    void *stream;
    bool with_append;
    const void *k_new, *v_new;
    int32_t *len_out;
    bool static_scratch;  // s3_decode_step_static: partials and counters in the library's fixed device buffer
};

static size_t batch_view_lds(int n, int ncls);

// Kernel arguments every attention kernel shares.  row_heads: heads of a cached row; q_heads: heads of q / out.
static AttnArgs common_args(const s3_arena *a, const AttnCall &c, int row_heads, int q_heads, int chunk) {
    AttnArgs args;
    memset(&args, 0, sizeof(args));
    args.kplane = a->plane(c.layer, 0);
    args.vplane = a->plane(c.layer, 1);
    args.q = (const char *)c.q;
    args.k_new = (const char *)c.k_new;
    args.v_new = (const char *)c.v_new;
    args.slot_off = c.slot_off;
    args.cur_len = c.len_or_pos;
    args.out = c.out;
    args.n_tokens = a->n_tokens;
    args.n = c.n;
    args.H = row_heads;
    args.Hq = q_heads;
    args.chunk = chunk;
    args.max_chunks = (a->cfg.max_len + chunk - 1) / chunk;
    // length classes of the longest-first work order: small batches gain from it (their kernels are
    // short, the tail matters); for large batches the extra prologue work per class costs more than
    // the order gains.  Measured on MI355X.
    args.ncls = a->ncls > 0 ? a->ncls : c.n <= 128 ? 4 : c.n <= 256 ? 2 : 1;
    // the view must fit LDS beside the kernels' own buffers (up to 67 KiB) whatever the caller asked for:
    // a batch of thousands keeps fewer classes
    while (args.ncls > 1 && batch_view_lds(c.n, args.ncls) > (size_t)96 * 1024) args.ncls--;
    args.out_dtype = c.out_dtype;
    args.max_len = a->cfg.max_len;
    args.len_add = c.with_append ? 1 : 0;
    const float scale = c.scale > 0.f ? c.scale : 1.0f / sqrtf((float)a->cfg.head_dim);
    args.scale_log2e = scale * 1.4426950408889634f;
    args.len_out = c.with_append ? c.len_out : nullptr;
    args.merge_sync = a->merge_sync;
    return args;
}

// Library scratch: [arrival counters: cnt_bytes, fixed per arena kind, zero between launches]
// [partial sums][partial (max, sum)], one partial per (sequence, chunk, head of q).
static int place_scratch(s3_arena *a, AttnArgs &args, size_t cnt_bytes, const AttnCall &c) {
    const size_t n_part = (size_t)args.n * args.max_chunks * args.Hq;
    const size_t acc_bytes = n_part * a->cfg.head_dim * sizeof(float);
    const size_t need = cnt_bytes + acc_bytes + n_part * sizeof(float2);
    char *base = nullptr;
    if (c.static_scratch) {  // no allocation on this path: the fixed buffer holds the call, or the call is refused
        if (need > (size_t)S3_STATIC_SCRATCH_BYTES) return S3_ERR_SCRATCH;
        const int rc = static_scratch_for_call(cnt_bytes, c.stream, &base);
        if (rc != S3_OK) return rc;
    } else {
        const int rc = ensure_scratch(a, need);
        if (rc != S3_OK) return rc;
        base = (char *)a->scratch;
    }
    args.arrivals = (unsigned int *)base;
    args.queue = cnt_bytes >= 256 ? (unsigned int *)(base + cnt_bytes - 256) : nullptr;  // the last 256 bytes of the counter region
    args.part_acc = (float *)(base + cnt_bytes);
    args.part_ml = (float2 *)(base + cnt_bytes + acc_bytes);
    return S3_OK;
}

// Bytes of the arrival counters at the head of the scratch: one per (sequence, head group), for the largest
// batch a call takes, so that the partials behind them never move with the batch size.
static size_t counters_bytes(int n_hg) {
    return ((((size_t)(S3_MAX_BATCH + 1) * n_hg * sizeof(unsigned int)) + 255) & ~(size_t)255) + 256;  // + the work-list counters
}

// Scratch an attention call over n sequences needs at most: the launchers' layout with the smallest chunk
// they may choose for any batch size (or the chunk the caller fixed).
static size_t scratch_need(const s3_arena *a, int n) {
    const int D = a->cfg.head_dim, Hq = a->cfg.n_heads;
    const int kind = s3i_kernel_kind(a);
    int chunk = a->chunk;
    size_t cnt_bytes = 0;
    if (kind == 0 || kind == 3) {  // kernels that merge chunks themselves carry counters
        if (chunk <= 0) chunk = 1024;
        const int gh = kind == 3 ? 1024 / D : heads_per_load(D);
        cnt_bytes = counters_bytes((Hq + gh - 1) / gh);
    } else {
        if (chunk <= 0) chunk = (kind == 2 || kind == 4) ? 128 : 256;
        if (kind == 2 || kind == 4)  // arrival counters (if chunks merge inside the launch) and the work-list counters
            cnt_bytes = counters_bytes(a->cfg.n_kv_heads * ((Hq / a->cfg.n_kv_heads + 15) / 16));
    }
    const size_t max_chunks = (size_t)(a->cfg.max_len + chunk - 1) / chunk;
    const size_t n_part = (size_t)n * max_chunks * Hq;
    return cnt_bytes + n_part * ((size_t)D * sizeof(float) + sizeof(float2));
}

extern "C" int s3_kv_reserve_scratch(s3_arena *a, int32_t max_batch) {
    if (!a || !a->base || max_batch < 1 || max_batch > S3_MAX_BATCH) return S3_ERR_INVALID;
    return ensure_scratch(a, scratch_need(a, max_batch));
}

static size_t batch_view_lds(int n, int ncls) {
    return (size_t)n * 8 + (size_t)((n + 1) & ~1) * 4 + (size_t)ncls * (n + 1) * 4;
}

// Grid of a kernel that walks the work list with a stride: the workgroups that are resident at once
// (every workgroup pays the batch-view prologue once), times `rounds`; or what the caller set.
static int stride_grid(const s3_arena *a, const void *fn, int threads, size_t dyn_lds, int rounds, int *blocks,
                       int max_per_cu = 0) {
    if (a->grid_blocks > 0) {
        *blocks = a->grid_blocks;
        return S3_OK;
    }
    int per_cu = 0;
    const int rc = resident_per_cu(fn, threads, dyn_lds, &per_cu);
    if (rc != S3_OK) return rc;
    if (max_per_cu > 0 && per_cu > max_per_cu) per_cu = max_per_cu;
    *blocks = (a->num_cus > 0 ? a->num_cus : 256) * per_cu * rounds;
    return S3_OK;
}

// Launch the attention kernel and, if merge_heads > 0, attn_merge_kernel over that many heads of q / out
// (it finishes multi-chunk contexts and writes the zero rows of empty ones).  Every k-th call (the
// "profile" parameter) is bracketed with events: before, after the attention kernel, after the merge.
static int launch_attn_kernels(s3_arena *a, attn_fn fn, int blocks, int threads, size_t dyn_lds, void *stream,
                               const AttnArgs &args, int merge_heads, bool may_time) {
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    const bool timed = may_time && a->profile > 0 && (a->prof_tick++ % a->profile) == 0;
    if (timed) {
        for (int i = 0; i < 3; i++) {
            const int prc = prof_next_event(a, &ev[i]);
            if (prc != S3_OK) return prc;
        }
        // the events take the kernel's own start and end times (not the times at which markers around it
        // pass through the queue), so the duration is the one a profiler reports for the dispatch
        AttnArgs copy = args;
        void *kargs[] = {(void *)&copy};
        HIP_TRY(hipExtLaunchKernel((const void *)fn, dim3((unsigned)blocks), dim3((unsigned)threads), kargs, dyn_lds,
                                   (hipStream_t)stream, ev[0], ev[1], 0));
    } else {
        hipLaunchKernelGGL(fn, dim3((unsigned)blocks), dim3((unsigned)threads), dyn_lds, (hipStream_t)stream, args);
        HIP_TRY(hipGetLastError());
    }
    if (merge_heads > 0) {
        const int D = a->cfg.head_dim;
        AttnArgs margs = args;
        margs.H = merge_heads;  // the merge kernel indexes partials and output by head of q
        const int GH = heads_per_load(D);
        const unsigned mblocks = (unsigned)(((int64_t)args.n * ((merge_heads + GH - 1) / GH) + 3) / 4);
        attn_fn mfn = pick_merge(D);
        if (timed) {
            void *kargs[] = {(void *)&margs};
            HIP_TRY(hipExtLaunchKernel((const void *)mfn, dim3(mblocks), dim3(256), kargs, 0, (hipStream_t)stream, nullptr,
                                       ev[2], 0));
        } else {
            hipLaunchKernelGGL(mfn, dim3(mblocks), dim3(256), 0, (hipStream_t)stream, margs);
            HIP_TRY(hipGetLastError());
        }
    } else if (timed) {
        HIP_TRY(hipEventRecord(ev[2], (hipStream_t)stream));
    }
    return S3_OK;
}

// Shared key/value heads.  Vector-ALU kernel: append as its own launch, attention, merge.  Matrix-core
// kernel: attention (which appends the new row itself), merge; over 8-bit rows: quantising append launch,
// attention, merge.
static int launch_gqa(s3_arena *a, const AttnCall &c) {
    const int D = a->cfg.head_dim, Hq = a->cfg.n_heads, Hkv = a->cfg.n_kv_heads;
    const int group = Hq / Hkv;
    const int gq = group % 8 == 0 ? 8 : group % 4 == 0 ? 4 : group % 2 == 0 ? 2 : 1;
    // Variant indices of a shared-K/V arena: the shapes of the vector-ALU kernel, then the matrix-core kernel.
    const int kind = s3i_kernel_kind(a);
    const bool mfma = kind == 2 || kind == 4, eight_bit = kind == 4;
    int threads = 256;
    attn_fn fn = eight_bit ? s3i_pick_gqa_mfma8(a->cfg.act_dtype, D)
                 : mfma    ? s3i_pick_gqa_mfma(a->cfg.kv_dtype, D)
                           : s3i_pick_gqa(a->cfg.kv_dtype, D, gq, a->variant, &threads);
    if (!fn) return S3_ERR_INVALID;
    if (c.with_append && (!mfma || eight_bit)) {  // 16-bit rows: the matrix-core kernel appends by itself
        const int arc = launch_append(a, c.layer, c.n, c.slot_off, c.len_or_pos, c.k_new, c.v_new, c.stream);
        if (arc != S3_OK) return arc;
    }
    const int GH = 512 / D;
    // work items per chunk: (K/V head groups x query sub-blocks), or for the matrix-core kernel
    // (K/V heads x blocks of 16 query heads), there one item per wave
    const int per_seq = mfma ? Hkv * ((group + 15) / 16) : ((Hkv + GH - 1) / GH) * (group / gq);
    // Few (sequence, head group) pairs: cut contexts finer so that the chip still has work everywhere.
    const int chunk = a->chunk > 0 ? a->chunk
                      : mfma     ? ((int64_t)c.n * per_seq >= 4096 ? 256 : 128)  // one wave per item: short items keep every SIMD busy
                      : (int64_t)c.n * per_seq >= 2048 ? 1024 : (int64_t)c.n * per_seq >= 512 ? 512 : 256;
    AttnArgs args = common_args(a, c, Hkv, Hq, chunk);
    if (mfma && a->ncls <= 0) args.ncls = 1;  // items of at most 128 rows are all alike: no order to gain from (measured)
    // matrix-core kernel: chunks of a context may meet inside the launch (one counter per sequence and item slot)
    const bool ink = mfma && a->gqa_merge != 0;
    args.merge_in_kernel = ink ? 1 : 0;
    args.stream_k = a->gqa_stream;
    args.dyn_list = mfma && a->gqa_dynamic > 0 ? a->gqa_dynamic : 0;
    int rc = place_scratch(a, args, mfma ? counters_bytes(per_seq) : 0, c);
    if (rc != S3_OK) return rc;
    const size_t dyn_lds = batch_view_lds(c.n, args.ncls);
    int blocks = 0;
    rc = stride_grid(a, (const void *)fn, threads, dyn_lds, 1, &blocks);
    if (rc != S3_OK) return rc;
    return launch_attn_kernels(a, fn, blocks, threads, dyn_lds, c.stream, args, ink ? 0 : Hq, !c.static_scratch);
}

// 8-bit cache rows: one kernel, which in a decode step also quantises and appends the new row, merges
// chunks and publishes the new lengths.
static int launch_fp8(s3_arena *a, const AttnCall &c) {
    const int D = a->cfg.head_dim, H = a->cfg.n_heads;
    int threads = 0;
    attn_fn fn = s3i_pick_fp8(a->cfg.act_dtype, D, a->variant, &threads);
    if (!fn) return S3_ERR_INVALID;
    AttnArgs args = common_args(a, c, H, H, a->chunk > 0 ? a->chunk : 1024);
    const int n_hg = (H + 1024 / D - 1) / (1024 / D);  // head groups: 1024/D heads per 128-bit wave load of bytes
    int rc = place_scratch(a, args, counters_bytes(n_hg), c);
    if (rc != S3_OK) return rc;
    const size_t dyn_lds = batch_view_lds(c.n, args.ncls);
    int blocks = 0;
    rc = stride_grid(a, (const void *)fn, threads, dyn_lds, c.n > 128 ? 2 : 1, &blocks);
    if (rc != S3_OK) return rc;
    return launch_attn_kernels(a, fn, blocks, threads, dyn_lds, c.stream, args, 0, !c.static_scratch);  // the kernel merges by itself
}

// Shared by s3_decode_attention (partial kernel + merge kernel) and s3_decode_step (with_append: one
// kernel that also appends, merges and publishes the new lengths).
static int launch_attention(s3_arena *a, const AttnCall &c) {
    if (a->cfg.n_kv_heads < a->cfg.n_heads) return launch_gqa(a, c);
    if (a->cfg.kv_dtype == S3_E4M3) return launch_fp8(a, c);
    const int D = a->cfg.head_dim, H = a->cfg.n_heads;
    // Defaults from sweeps on MI355X: large chunks keep most contexts in one piece (no cross-workgroup
    // merge), eight waves share an item's rows evenly, each with two batches of two rows in flight
    // alternately (1 % ahead of one batch of four rows on the ragged batch of 64, level on the others).
    const int variant = a->variant >= 0 ? a->variant : c.n > 128 ? s3i_default_variant_large() : s3i_default_variant();
    const bool fused = c.with_append;
    attn_fn fn = pick_kernel(a->cfg.kv_dtype, D, variant, fused);
    if (!fn) return S3_ERR_INVALID;
    const int GH = heads_per_load(D);
    const int n_hg = (H + GH - 1) / GH;
    AttnArgs args = common_args(a, c, H, H, a->chunk > 0 ? a->chunk : 1024);
    args.len_out = c.len_out;
    // a dynamic work list is a longest-processing-time schedule only if the long items come first: four length
    // classes whatever the batch size (with a fixed stride, large batches did better without the classes' prologue)
    if (a->ncls <= 0 && fused && s3i_variant_dynamic(variant)) {
        args.ncls = 4;
        while (args.ncls > 1 && batch_view_lds(c.n, args.ncls) > (size_t)96 * 1024) args.ncls--;
    }
    int rc = place_scratch(a, args, counters_bytes(n_hg), c);
    if (rc != S3_OK) return rc;
    const int threads = s3i_variant_threads(variant, fused);  // the fused kernel adds an epilogue wave
    const size_t view = batch_view_lds(c.n, args.ncls);
    const size_t dyn_lds = fused && s3i_variant_ring_bytes(variant) ? ((view + 15) & ~(size_t)15) + s3i_variant_ring_bytes(variant) : view;
    int blocks = 0;
    // fixed stride: large batches balance better over two rounds of resident workgroups; a dynamic work list
    // needs exactly the resident ones
    const int rounds = (fused && s3i_variant_dynamic(variant)) ? 1 : c.n > 128 ? 2 : 1;
    // the shapes that carry the row stream across items keep a compute unit's memory pipeline full from one
    // workgroup; a second resident one (their register count admits it) measured 2 % slower
    rc = stride_grid(a, (const void *)fn, threads, dyn_lds, rounds, &blocks, fused && s3i_variant_stream(variant) ? 1 : 0);
    if (rc != S3_OK) return rc;
    return launch_attn_kernels(a, fn, blocks, threads, dyn_lds, c.stream, args, fused ? 0 : H, !c.static_scratch);
}

extern "C" int s3_decode_attention(s3_arena *a, int32_t layer, int32_t n, const void *q, const int64_t *slot_off,
                                   const int32_t *cur_len, void *out, int32_t out_dtype, float scale, void *stream) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n < 0 || n > S3_MAX_BATCH) return S3_ERR_INVALID;
    if (n == 0) return S3_OK;
    if (!q || !slot_off || !cur_len || !out || !aligned16(q) || !aligned16(out)) return S3_ERR_INVALID;
    if (out_dtype != S3_F32 && out_dtype != S3_F16 && out_dtype != S3_BF16) return S3_ERR_INVALID;
    const AttnCall c = {layer, n, q, slot_off, cur_len, out, out_dtype, scale, stream, false, nullptr, nullptr, nullptr, false};
    return launch_attention(a, c);
}

static int decode_step(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                       const int64_t *slot_off, const int32_t *pos, const void *q, const void *k_new, const void *v_new,
                       void *out, int32_t out_dtype, float scale, int32_t *len_out, void *stream, bool static_scratch) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n < 0 || n > S3_MAX_BATCH) return S3_ERR_INVALID;
    if (n == 0) return S3_OK;
    if (!q || !k_new || !v_new || !slot_off || !pos || !out) return S3_ERR_INVALID;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return S3_ERR_INVALID;
    if (len_out == pos) return S3_ERR_INVALID;  // other workgroups still read pos while len_out is written
    if (out_dtype != S3_F32 && out_dtype != S3_F16 && out_dtype != S3_BF16) return S3_ERR_INVALID;
    const int rc = check_slots_host(a, n, slot_id, pos_host);
    if (rc != S3_OK) return rc;
    const AttnCall c = {layer, n, q, slot_off, pos, out, out_dtype, scale, stream, true, k_new, v_new, len_out, static_scratch};
    return launch_attention(a, c);
}

extern "C" int s3_decode_step(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                              const int64_t *slot_off, const int32_t *pos, const void *q, const void *k_new,
                              const void *v_new, void *out, int32_t out_dtype, float scale, int32_t *len_out,
                              void *stream) {
    return decode_step(a, layer, n, slot_id, pos_host, slot_off, pos, q, k_new, v_new, out, out_dtype, scale, len_out,
                       stream, false);
}

extern "C" int s3_decode_step_static(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id,
                                     const int32_t *pos_host, const int64_t *slot_off, const int32_t *pos, const void *q,
                                     const void *k_new, const void *v_new, void *out, int32_t out_dtype, float scale,
                                     int32_t *len_out, void *stream) {
    return decode_step(a, layer, n, slot_id, pos_host, slot_off, pos, q, k_new, v_new, out, out_dtype, scale, len_out,
                       stream, true);
}

extern "C" int s3_kv_fill(s3_arena *a, int32_t slot_id, int32_t layer, int32_t first_row, int32_t n_rows,
                          const void *k_rows, const void *v_rows, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || layer < 0 || layer >= a->cfg.n_layers || first_row < 0 || n_rows < 0) return S3_ERR_INVALID;
    if ((int64_t)first_row + n_rows > s->cap) return S3_ERR_SLOT_FULL;
    if (n_rows == 0) return S3_OK;
    if (!k_rows || !v_rows) return S3_ERR_INVALID;
    const size_t nbytes = (size_t)n_rows * a->row_bytes;
    const int64_t row0 = s->off + first_row;
    if (((uintptr_t)k_rows & 15) || ((uintptr_t)v_rows & 15)) return S3_ERR_INVALID;
    const size_t n16 = nbytes / 16;
    size_t blocks = (n16 + 1023) / 1024;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(copy_pair_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, (hipStream_t)stream,
                       (const char *)k_rows, a->plane(layer, 0) + row0 * a->row_bytes, (const char *)v_rows,
                       a->plane(layer, 1) + row0 * a->row_bytes, n16);
    HIP_TRY(hipGetLastError());
    return S3_OK;
}

// ---- evict to / restore from host memory (the paper's own misprediction path, section 3 and 4.3) ----
extern "C" int64_t s3_kv_evict_bytes(const s3_arena *a, int32_t len) {
    if (!a || len < 0 || len > a->cfg.max_len) return S3_ERR_INVALID;
    return (int64_t)2 * a->cfg.n_layers * len * a->row_bytes;
}

extern "C" int s3_kv_evict(s3_arena *a, int32_t slot_id, int32_t len, void *host_buf, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || len < 0 || len > s->cap || (len > 0 && !host_buf)) return S3_ERR_INVALID;
    const size_t piece = (size_t)len * (size_t)a->row_bytes;
    const int planes = 2 * a->cfg.n_layers;
    for (int p = 0; p < planes && piece; p++)
        HIP_TRY(hipMemcpyAsync((char *)host_buf + (size_t)p * piece,
                               a->base + (int64_t)p * a->plane_bytes + s->off * a->row_bytes, piece,
                               hipMemcpyDeviceToHost, (hipStream_t)stream));
    return s3_kv_free(a, slot_id);
}

extern "C" int s3_kv_restore(s3_arena *a, int32_t predicted_len, int32_t len, const void *host_buf, int32_t *slot_id,
                             int64_t *slot_off, int32_t *slot_cap, void *stream) {
    if (!a || !a->base || !slot_id || len < 0 || predicted_len < len || (len > 0 && !host_buf)) return S3_ERR_INVALID;
    if (len > a->cfg.max_len) return S3_ERR_INVALID;
    int32_t id = -1, cap = 0;
    int64_t off = -1;
    const int admitted = s3_kv_alloc(a, 1, &predicted_len, &id, &off, &cap);
    if (admitted < 0) return admitted;
    if (admitted == 0) return S3_ERR_NOMEM;
    const size_t piece = (size_t)len * (size_t)a->row_bytes;
    const int planes = 2 * a->cfg.n_layers;
    for (int p = 0; p < planes && piece; p++) {
        const hipError_t e = hipMemcpyAsync(a->base + (int64_t)p * a->plane_bytes + off * a->row_bytes,
                                            (const char *)host_buf + (size_t)p * piece, piece, hipMemcpyHostToDevice,
                                            (hipStream_t)stream);
        if (e != hipSuccess) {
            (void)s3_kv_free(a, id);
            return hip_fail("hipMemcpyAsync(restore)", e);
        }
    }
    *slot_id = id;
    if (slot_off) *slot_off = off;
    if (slot_cap) *slot_cap = cap;
    return S3_OK;
}

// Rows [0, len) of every plane of a live slot to / from one contiguous device buffer laid out like the host
// buffer of s3_kv_evict: the device-side halves of an eviction and of a re-admission that cross the host link
// off the decode stream.  One launch each.
extern "C" int s3_kv_gather_rows(s3_arena *a, int32_t slot_id, int32_t len, void *dev_buf, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || len < 0 || len > s->cap || (len > 0 && (!dev_buf || ((uintptr_t)dev_buf & 15)))) return S3_ERR_INVALID;
    const size_t piece = (size_t)len * (size_t)a->row_bytes;
    return s3i_launch_copy_planes(a->base + s->off * a->row_bytes, (char *)dev_buf, piece, (size_t)a->plane_bytes, piece,
                                  2 * a->cfg.n_layers, stream);
}

extern "C" int s3_kv_scatter_rows(s3_arena *a, int32_t slot_id, int32_t len, const void *dev_buf, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || len < 0 || len > s->cap || (len > 0 && (!dev_buf || ((uintptr_t)dev_buf & 15)))) return S3_ERR_INVALID;
    const size_t piece = (size_t)len * (size_t)a->row_bytes;
    return s3i_launch_copy_planes((const char *)dev_buf, a->base + s->off * a->row_bytes, piece, piece, (size_t)a->plane_bytes,
                                  2 * a->cfg.n_layers, stream);
}

// A copy that deliberately occupies few compute units, and occupies them alone: `workgroups` workgroups of 1024
// threads move `bytes` with four 16-byte pieces in flight per thread, and every workgroup reserves nearly all of a
// compute unit's LDS so that no attention workgroup shares the unit with waves that wait on the host link.  For
// transfers between device memory and mapped pinned host memory beside the decode steps.  How many workgroups
// is the caller's trade: the copy's rate grows with them (measured device -> host: 1: 17 GB/s, 2: 31, 4: 43,
// 8: 55 = the link's rate), but so does the number of writes queued for the link at once, and beyond four the
// queue hurts everything else that runs - with eight, whatever kernel was running when a copy started (an
// attention launch, a doubling's copy) took 3-5 times as long for the copy's first milliseconds (attention
// launches of the 28-layer workload under a kernel trace: average 769-780 us, up to 3.5 ms; the runtime's own
// copy kernels, which spread over every unit: 821 us, up to 5.5 ms), with one, two or four: 746-748 us, none above
// 1.0 ms.  The decode loop uses two.
#define S3_LINK_THREADS 1024
#define S3_LINK_LDS (152 * 1024)
__global__ void __launch_bounds__(S3_LINK_THREADS) link_copy_kernel(const char *src, char *dst, size_t n16) {
    const u32x4 *s = (const u32x4 *)src;
    u32x4 *d = (u32x4 *)dst;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = s[i], b = s[i + stride], c = s[i + 2 * stride], e = s[i + 3 * stride];
        d[i] = a;
        d[i + stride] = b;
        d[i + 2 * stride] = c;
        d[i + 3 * stride] = e;
    }
    for (; i < n16; i += stride) d[i] = s[i];
}

extern "C" int s3_kv_link_copy(void *dst, const void *src, size_t bytes, int32_t workgroups, void *stream) {
    if (bytes == 0) return S3_OK;
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return S3_ERR_INVALID;
    if (workgroups < 1 || workgroups > 1024) return S3_ERR_INVALID;
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute((const void *)link_copy_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, S3_LINK_LDS);
    });
    if (attr != hipSuccess) return hip_fail("hipFuncSetAttribute(link_copy_kernel)", attr);
    hipLaunchKernelGGL(link_copy_kernel, dim3((unsigned)workgroups), dim3(S3_LINK_THREADS), S3_LINK_LDS, (hipStream_t)stream,
                       (const char *)src, (char *)dst, bytes / 16);
    HIP_TRY(hipGetLastError());
    return S3_OK;
}

extern "C" int s3_kv_read_rows(s3_arena *a, int32_t slot_id, int32_t layer, int32_t which, int32_t first_row,
                               int32_t n_rows, void *dst, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || layer < 0 || layer >= a->cfg.n_layers || first_row < 0 || n_rows < 0 ||
        (which != 0 && which != 1))
        return S3_ERR_INVALID;
    if ((int64_t)first_row + n_rows > s->cap) return S3_ERR_INVALID;
    if (n_rows == 0) return S3_OK;
    if (!dst) return S3_ERR_INVALID;
    return s3i_launch_copy_planes(a->plane(layer, which) + (s->off + first_row) * a->row_bytes, (char *)dst,
                                  (size_t)n_rows * a->row_bytes, 0, 0, 1, stream);
}
