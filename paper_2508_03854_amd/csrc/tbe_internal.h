// Internal declarations shared by the translation units of libtbe355 (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "tbe355.h"

namespace tbe {

// ---- tunables that fix the workspace layout -------------------------------------------------
constexpr int kSegChunk = 512;         // a unique row with more lookups than this is split into chunks of this size
constexpr int kRadixTile = 4096;  // elements per radix-sort tile (256 threads x items per thread)
constexpr int kRadixMaxBlocks = 8192;  // each radix block owns one contiguous slice of the input
constexpr int kRleTile = 2048;  // elements per run-length tile (at most 4096: one wavefront scans its runs of 64)
constexpr int kLinTile = 2048;         // positions per linearize tile
constexpr int kMaxSlices = 64;         // sub-slices of one table's gradient block (8 XCDs x up to 8 sweeps)
constexpr int kMaxSortSegments = 4096;  // tables beyond this are sorted as one segment on the linearised key
constexpr int kDenseRows = 16;   // rows per table that the dense-row kernel reduces (multiple of 4)
constexpr int kDenseChunks = 32;            // bag chunks (= partial sums) per dense row
constexpr int kFwdGroupMaxLanes = 32;   // rows of at most this many lanes use one bag per lane group
constexpr int kHotRows = 256;           // rows per table that the forward may hold in LDS (the handle's hot-row list)
constexpr int kMaxReplicas = 16;        // replicas of one buffer that tbe_replica_mean averages in one call
constexpr int kTicketStride = 32;       // words between two ticket counters: each sits in a 128-byte line of its own
constexpr int kTicketWords = (kMaxSlices / 8) * 8 * kTicketStride;  // one counter per (sweep, XCD)
constexpr int kCounterWords = 64;      // device counters: [0]=U [1]=long rows [3]=units

struct TimingSlot {
    const char* name;
    hipEvent_t beg, end;
};

}  // namespace tbe

struct tbe_handle {
    int32_t T = 0;
    tbe_dtype dtype = TBE_F32;
    int device = 0;
    int64_t total_rows = 0;
    int64_t total_elems = 0;
    int32_t sumD = 0;
    int32_t maxD = 0;
    int32_t minD = 0;
    bool seg_mostly_wavefront_rows = false;  // most rows of the tables up to 256 columns need all 64 lanes (D > 128)
    int key_bits = 1;  // bits needed to hold the value total_rows (the key given to invalid ids)
    // Sort plan.  Positions arrive grouped by table, so sorting every table's run of positions on its table-local id
    // alone gives the same order as sorting all of them on the linearised key, with fewer key bits whenever
    // bits(max rows of one table) needs fewer radix passes than bits(sum of rows).
    bool segmented = false;  // true: one sort segment per table, local keys; false: one segment, linearised keys
    int sort_bits = 1;       // key bits the radix passes cover
    int sort_passes = 1;
    std::vector<int64_t> rows, row_base, w_off;
    std::vector<int32_t> D, D_off;
    // device metadata, one allocation
    void* d_meta = nullptr;
    int32_t* d_D_off = nullptr;     // [T+1]
    int64_t* d_row_base = nullptr;  // [T+1]
    int64_t* d_w_off = nullptr;     // [T+1]
    void* static_scratch = nullptr; // device address, on this handle's device, of the library's fixed scratch array
    int32_t* d_err = nullptr;       // sticky invalid-id flag
    // Forward classes: 0, 5, 6 = one wavefront per bag, rows of at most 64 / 128 / 256 sixteen-byte fragments;
    // 1..4 = narrow rows (32 / 16 / 8 / <=4 lanes per row), where every lane group of a wavefront takes a bag of its
    // own (2 / 4 / 8 / 16 bags per wavefront).  d_fwd_tables lists the tables class by class.
    int32_t* d_fwd_tables = nullptr;  // [T]
    // Hot-row hint: the table-local ids of the rows of every table that had the most lookups in the last backward
    // call (at most kHotRows each), written by that call's kernels and read by the next forward.  Any contents give
    // the same forward result; null when the handle has too many tables to keep one.
    uint32_t* d_hot_ids = nullptr;    // [T][kHotRows]
    uint32_t* d_hot_n = nullptr;      // [T]
    int64_t hot_min_workgroups = 256; // the forward stages hot rows in LDS when a width class fills this many workgroups; < 0: never
    int fwd_first[7] = {0, 0, 0, 0, 0, 0, 0};
    int fwd_count[7] = {0, 0, 0, 0, 0, 0, 0};
    // timing
    bool timing = false;
    std::vector<tbe::TimingSlot> slots;  // pool of event pairs
    int n_used = 0;                      // slots used by the calls since timing was (re)enabled
};

namespace tbe {

// Workspace carving for a batch of N lookups (all offsets in bytes, 256-byte aligned).
struct Workspace {
    // keys/vals: radix double buffers of N+1 words each.  The payload of a key is the linear bag id of its lookup
    // (pooled calls) or its position (non-pooled calls), so vals[sorted] is the per-lookup stream the gradient
    // kernels read.  After the sort vals[spare] receives unique_rows.
    size_t keys[2], vals[2], bag_of_pos, seg_start, radix_hist, bin_tot, rle_counts, counters, long_tables, tickets, seq_gbase, seg_bounds,
        seg_chunk0, chunk_desc, dense_rows, dense_n, dense_bounds, tile_long, tile_slots,
        long_list, unit_list, bounds, partial, total;
    int radix_blocks;     // blocks a single segment of N keys would need
    int radix_maxc;       // chunk descriptors: radix_blocks + number of segments (every segment may end in a partial chunk)
    int nseg;             // sort segments
    int64_t radix_chunk;  // elements per radix block (multiple of kRadixTile)
    int rle_blocks;
    int64_t cap_long, cap_main, cap_chunks, cap_units;   // long rows; slots before the dense region; all slots; units
    int long_tiles;       // tiles of unique rows that the long-row passes walk
    int64_t n;            // number of lookups the workspace was carved for
};
Workspace carve(const tbe_handle* h, int64_t N);

// RAII-free helper: brackets one kernel launch with events when timing is on.
struct LaunchTimer {
    tbe_handle* h;
    hipStream_t s;
    int slot = -1;
    LaunchTimer(const tbe_handle* h_, hipStream_t s_, const char* name);
    void done();
};

// launchers (each returns hipGetLastError() after its launches).  idx32: ids and offsets are int32 instead of
// int64; out_io / grad_io: 0 float, 1 binary16, 2 bfloat16.
hipError_t launch_forward(const tbe_handle* h, const void* tables, const int32_t* d_D_off, const void* indices,
                          const void* offsets, int idx32, int32_t B, int64_t nnz, tbe_pooling pooling, void* out,
                          int out_io, hipStream_t s);
// every replicas[m] (device pointers, M <= kMaxReplicas) becomes the element-wise mean; count elements each
hipError_t launch_replica_mean(const tbe_handle* h, void* const* replicas, int M, size_t count, bool f32, hipStream_t s);
hipError_t launch_linearize(const tbe_handle* h, const void* indices, const void* offsets, int idx32, int32_t B, int64_t N,
                            uint32_t* keys, uint32_t* bag_of_pos, hipStream_t s);
// sorts keys[0] of the workspace segment by segment (see tbe_handle::segmented); the payload that travels with a key
// is payload[p] (nullptr: its position p).  The keys written by the last pass are linearised row keys in either
// mode.  Returns in *result_buf which buffer pair (0/1) holds the sorted keys and payloads.
hipError_t launch_radix_sort(const tbe_handle* h, const Workspace& w, char* ws, int64_t N, const uint32_t* payload,
                             const void* offsets, int idx32, int32_t B, int* result_buf, hipStream_t s);
// `sorted` is the buffer index (0/1) that holds the sorted pairs; vals of the other pair receive unique_rows
hipError_t launch_run_lengths(const tbe_handle* h, const Workspace& w, char* ws, int sorted, int64_t N, hipStream_t s);
// state == nullptr: plain SGD step.  seq != 0: grad_out is the non-pooled layout (one [n_t, D_t] block per table),
// offsets has T+1 entries and B is 1.
hipError_t launch_segment_update(const tbe_handle* h, const Workspace& w, char* ws, int spare, const void* grad_out,
                                 int grad_io, const void* offsets, int idx32, int32_t B, tbe_pooling pooling, float lr,
                                 float eps, float c, void* tables, float* state, int seq, int64_t grad_elems, hipStream_t s);
// non-pooled lookup: out block of table t = rows indices[offsets[t] .. offsets[t+1]) of table t, one after the other
hipError_t launch_lookup_seq(const tbe_handle* h, const void* tables, const void* indices, const void* offsets, int idx32,
                             int64_t nnz, void* out, int out_io, int64_t out_elems, hipStream_t s);

}  // namespace tbe
