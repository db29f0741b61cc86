// Internal declarations shared by the host bookkeeping and the HIP launchers of libs3kv.
#pragma once
#include <stdint.h>

#include <map>
#include <set>
#include <vector>

#include "s3kv.h"

struct s3_slot {
    int64_t off = -1;
    int32_t cap = 0;
    bool live = false;
};

struct s3_arena {
    s3_kv_config cfg{};
    char *base = nullptr;      // device memory owned by the caller (nullptr: metadata only)
    size_t dev_bytes = 0;
    int64_t n_tokens = 0;      // N: token rows the arena holds
    int64_t elem_bytes = 2;
    int64_t row_bytes = 0;     // kv heads * D * elem
    int64_t plane_bytes = 0;   // N * row_bytes; plane p = 2*layer + (0: K, 1: V)

    std::map<int64_t, int64_t> free_ext;  // offset -> size, disjoint, coalesced
    std::vector<s3_slot> slots;           // indexed by id
    std::set<int32_t> dead_ids;           // ids below slots.size() that are not live
    int64_t used_tokens = 0;
    int64_t n_grows = 0;

    // split-K partials owned by the library
    void *scratch = nullptr;
    size_t scratch_bytes = 0;

    // optional timing of the attention kernels with events on the launch stream
    int32_t profile = 0;       // k > 0: bracket every k-th attention launch with events
    int64_t prof_tick = 0;     // attention launches since profiling was switched on
    std::vector<void *> prof_events;  // triples: before partial, after partial, after merge
    size_t prof_used = 0;             // events handed out since the last collect
    double prof_partial_ms = 0.0, prof_merge_ms = 0.0;
    int64_t prof_launches = 0;
    std::vector<float> prof_durations_ms;  // first interval of every timed launch since the last reset

    // launch-shape knobs (0 = default)
    int32_t chunk = 0;
    int32_t ncls = 0;  // length classes of the work order (0: library default)
    int32_t grid_blocks = 0;
    int32_t variant = -1;
    int32_t gqa_merge = 0;   // matrix-core kernel for shared heads: 1 = chunks merge inside the launch, 0 = merge launch
    int32_t gqa_stream = -1; // matrix-core kernel: K rows read with the streaming hint (1), with plain loads (0), by launch size (-1)
    int32_t gqa_dynamic = -1; // matrix-core kernel: per cent of the work list dealt by stride before waves claim positions (0, 100 or -1, the default: all by stride)
    int32_t merge_sync = 0;  // ordering of chunks that meet inside one launch (0: write-through partials, 1: fences)
    int32_t num_cus = 0;

    char *plane(int32_t layer, int32_t which) const {
        return base + (int64_t)(2 * layer + which) * plane_bytes;
    }
};

// host bookkeeping (s3kv_alloc.cpp)
int32_t s3i_capacity_for(const s3_arena *a, int32_t predicted_len);
int64_t s3i_carve(s3_arena *a, int64_t cap);          // first fit; -1 if nothing fits
void s3i_release(s3_arena *a, int64_t off, int64_t cap);
const s3_slot *s3i_live_slot(const s3_arena *a, int32_t id);
void s3i_set_hip_error(const char *what, int code, const char *text);

// device work (s3kv_kernels.hip); each returns an s3_status
int s3i_launch_copy_planes(const char *src, char *dst, size_t nbytes, size_t src_plane_stride,
                           size_t dst_plane_stride, int planes, void *stream);
int s3i_num_variants();    // kernel variants of the multi-head attention kernels
int s3i_default_variant(); // the one an arena uses unless told otherwise
int s3i_num_gqa_shapes();  // shapes of the shared-K/V (grouped-query) attention kernel
int s3i_num_fp8_shapes();  // shapes of the attention kernel for 8-bit cache rows
// Which attention kernel family the arena's next launch uses: 0 multi-head, 1 shared-K/V on the vector
// ALU, 2 shared-K/V on the matrix cores (variant index = number of shapes, or the default from four
// query heads per cached head; measured on MI355X), 3 the kernel for 8-bit cache rows, 4 the matrix-core
// kernel over 8-bit rows (shared K/V heads with an 8-bit cache).
int s3i_kernel_kind(const s3_arena *a);
int s3i_profile_collect(s3_arena *a);  // synchronises on the recorded events and accumulates the sums
void s3i_profile_reset(s3_arena *a);
int s3i_device_cus(int32_t *cus);
int s3i_static_scratch_setup();  // resolves the device address of the fixed scratch of s3_decode_step_static
