// Floating-point half of the backward pass: per unique row, sum the upstream gradient slices of the
// row's segment and apply one moment-scaled row-wise AdaGrad step in place (Algorithm 1, steps 5-6).
//
// Every unique row has exactly one owner (a group of lanes, a wavefront, or the wavefront that combines
// a hot row's partial sums), so weights and moments have a single writer and the result does not depend
// on scheduling.  A row of D floats is covered by LPR = D/4 lanes (one float4 each), which leaves
// G = 64/LPR lane groups per wavefront.  Rows are binned by the number of lookups that hit them:
//   - short  (a run of <= G consecutive rows with <= 64 lookups in total): one row per lane group, the
//     lookups' bag ids arrive with one coalesced load and are handed out with cross-lane reads;
//   - medium (65 .. kSegChunk lookups): the whole wavefront walks the row, groups interleaved;
//   - long   (> kSegChunk lookups, the head of the Zipf distribution): cut into chunks that separate
//     wavefronts reduce into a partial buffer, combined in chunk order by the row's owner.
// Row metadata (segment bounds, key, table, moment) is fetched for 64 rows at a time, one row per lane.
#include "tbe_device.h"
#include "tbe_internal.h"

namespace tbe {

constexpr int kSegThreads = 256;
constexpr int kSegBlocks = 2048;  // persistent grids: waves stride over blocks of 64 unique rows, or over rows
// Gradient fragments in flight per lane while a row is reduced: as many as the registers of the variant allow
// without spilling at the WAVES wavefronts per SIMD its kernel is compiled for.  Measured at the largest workload with
// 32-bit gradients: 2 / 4 / 6 / 8 in flight give 21.6 / 20.4 / 20.2 / 19.8 ms for the row updates; 8 needs more than
// the 64 registers of 8 wavefronts per SIMD, which is why seg_update runs 7 (6: 20.7 ms); 16-bit fragments are half
// the size.
template <int NC, bool MEAN, typename GT, int WAVES>
__device__ __host__ constexpr int seg_unroll() {
    return NC > 1 ? 4 : (sizeof(GT) == 4 ? (WAVES < 8 ? (MEAN ? 6 : 8) : (MEAN ? 4 : 6)) : 8);
}


struct RowGeom {
    int D, LPR, G, sub, lc;
};

__device__ __forceinline__ RowGeom row_geom(int D) {
    RowGeom g;
    const int lane = lane_id();
    const int nl = (D + 3) >> 2;
    g.D = D;
    g.LPR = nl >= kWave ? kWave : pow2ceil64(nl);
    const int lpr_log2 = __builtin_ctz((unsigned)g.LPR);   // LPR is a power of two: shifts, not divisions
    g.G = kWave >> lpr_log2;
    g.sub = lane >> lpr_log2;
    g.lc = (lane & (g.LPR - 1)) * 4;
    return g;
}

// table of a linearised row key: the t with row_base[t] <= key < row_base[t+1]
__device__ __forceinline__ int table_of_key(const int64_t* __restrict__ row_base, int T, uint32_t key) {
    int lo = 0, hi = T;  // first t in [0, T] with row_base[t] > key, minus 1
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (row_base[mid] > (int64_t)key) hi = mid;
        else lo = mid + 1;
    }
    return lo - 1;
}

struct SegArgs {
    const uint32_t* keys_unique;  // unique_rows
    const uint32_t* seg_start;
    const uint32_t* counters;     // [0]=U, [1]=long rows, [3]=work units
    const uint32_t* bag_sorted;   // the sorted payload: linear bag id of every sorted lookup
    IdxView offsets;
    const void* grad_out;         // [B, sum(D)] float / binary16 / bfloat16, per the kernel's GT (or the sequence layout)
    const int64_t* seq_gbase;     // non-pooled mode only: element offset of table t's gradient block minus start_t * D_t
    int seq;                      // 1: non-pooled; bag_sorted then holds the original positions
    const int32_t* D_off;
    const int64_t* row_base;
    const int64_t* w_off;
    int32_t T, B, sumD, maxD;
    int32_t mixed;         // 1: both row-update kernels run, each on the rows of its own width class
    uint32_t total_rows;
    float lr, eps, inv_c;
    void* tables;
    float* state;          // nullptr: plain SGD step, no moments
    uint32_t* long_list;   // [cap_long][4]  (u, first slot, parts | sliced flag, table)
    float* partial;        // [cap_chunks][maxD] partial sums of long rows
    uint32_t* tile_long;   // [tiles + 1] long rows per tile of kLongTile unique rows, then their exclusive scan
    uint32_t* tile_slots;  // [tiles + 1] partial-sum slots those rows need, then the exclusive scan
    uint32_t dense_slot0;  // first slot of the region reserved for dense rows (kDenseChunks per row, kDenseRows per table)
    uint32_t* tcount;      // [T+1] long rows per table (then tbase [T+1], tfill [T+1] behind it)
    uint2* unit_list;      // [cap_units] (position in long_list, unit index)
    uint32_t* bounds;      // [cap_long][kMaxSlices + 1] sub-slice borders inside a sliced row's segment
    uint32_t* dense_rows;  // [T][kDenseRows] position in long_list of the table's dense rows
    uint32_t* dense_n;     // [T] number of dense rows (0: the table does not take the dense path)
    uint32_t* dense_bounds;  // [T][kDenseRows][kDenseChunks + 1] borders of the bag chunks inside each dense row's segment
    uint32_t* tickets;     // [sweep][XCD] counters, kTicketStride words apart, zero before the first sweep
    uint32_t cap_units;
    uint32_t cap_long, cap_chunks;
};

template <bool MEAN>
__device__ __forceinline__ float bag_scale(const IdxView offsets, uint32_t bag) {
    if (!MEAN) return 1.f;
    const int64_t L = offsets[(int64_t)bag + 1] - offsets[bag];
    return L > 0 ? 1.f / (float)L : 0.f;
}

// Where the upstream gradient of a lookup of table t lives: element base + (row - row0) * pitch (+ column).
// Pooled: row = bag id, one [B, sum(D)] matrix.  Non-pooled: row = original position, one [n_t, D_t] block per table.
struct GradAddr {
    int64_t base, pitch, row0;
};
__device__ __forceinline__ GradAddr grad_addr(const SegArgs& a, const int t, const int D) {
    GradAddr ga;
    if (a.seq) {
        ga.base = a.seq_gbase[t]; ga.pitch = D; ga.row0 = 0;
    } else {
        ga.base = a.D_off[t]; ga.pitch = a.sumD; ga.row0 = (int64_t)t * a.B;
    }
    return ga;
}

// Whole-wavefront reduction of sorted positions [s, e) of ONE row:
// acc += sum of scale(bag) * grad_out[b, d0 + col .. col+3]; the groups take interleaved positions and
// fold_groups() completes the sum.  NC = 256-column chunks per row.
template <int NC, bool MEAN, typename GT, int WAVES = 8>
__device__ __forceinline__ void segment_reduce(float (&acc)[NC][4], const RowGeom& g, const GT* __restrict__ gcol,
                                               const int64_t sumD, const int64_t bag0,
                                               const uint32_t* __restrict__ bag_sorted, const IdxView offsets,
                                               const uint32_t s, const uint32_t e) {
    constexpr int kSegUnroll = seg_unroll<NC, MEAN, GT, WAVES>();
    const int lane = lane_id();
    for (uint32_t base = s; base < e; base += kWave) {
        const int n = (int)((e - base) < (uint32_t)kWave ? (e - base) : (uint32_t)kWave);
        uint32_t my_b = 0;
        float my_s = 1.f;
        if (lane < n) {
            const uint32_t bag = bag_sorted[base + lane];
            my_b = (uint32_t)((int64_t)bag - bag0);
            my_s = bag_scale<MEAN>(offsets, bag);
        }
        for (int k0 = 0; k0 < n; k0 += kSegUnroll * g.G) {
            typename GradIO<GT>::raw_t x[kSegUnroll][NC];
            float sc[kSegUnroll];
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u) {
                const int k = k0 + u * g.G + g.sub;
                const uint32_t b = __shfl(my_b, k & (kWave - 1), kWave);
                sc[u] = MEAN ? __shfl(my_s, k & (kWave - 1), kWave) : 1.f;
                const bool on = k < n;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int col = g.lc + c * kWave * 4;
                    x[u][c] = (on && col < g.D) ? GradIO<GT>::load(gcol + (int64_t)b * sumD + col) : GradIO<GT>::zero();
                }
            }
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const float4 f = GradIO<GT>::to_float(x[u][c]);
                    if (MEAN) {
                        acc[c][0] = fmaf(sc[u], f.x, acc[c][0]);
                        acc[c][1] = fmaf(sc[u], f.y, acc[c][1]);
                        acc[c][2] = fmaf(sc[u], f.z, acc[c][2]);
                        acc[c][3] = fmaf(sc[u], f.w, acc[c][3]);
                    } else {
                        acc[c][0] += f.x;
                        acc[c][1] += f.y;
                        acc[c][2] += f.z;
                        acc[c][3] += f.w;
                    }
                }
        }
    }
}

template <int NC>
__device__ __forceinline__ void fold_groups(float (&acc)[NC][4], const RowGeom& g) {
    for (int o = g.LPR; o < kWave; o <<= 1) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (o == 32) acc[c][v] = pair_sum<32>(acc[c][v]);        // the two halves / odd and even rows: in place
                else if (o == 16) acc[c][v] = pair_sum<16>(acc[c][v]);
                else acc[c][v] += __shfl_xor(acc[c][v], o, kWave);
            }
    }
}

// the step size of Algorithm 1, step 6: lr / (sqrt(v / c) + eps), from the hardware square root and reciprocal (one
// unit in the last place each); v == 0 means the row's gradient is zero and nothing is applied
__device__ __forceinline__ float adagrad_step(const float v_new, const float lr, const float eps, const float inv_c) {
    const float denom = __builtin_amdgcn_sqrtf(v_new * inv_c) + eps;
    return v_new > 0.f ? lr * __builtin_amdgcn_rcpf(denom) : 0.f;
}

// The optimizer step for one row.  acc holds the complete row gradient in the LPR lanes that `on`
// marks (all groups after fold_groups, or each group its own row).  v_old is the row's moment.
//   v <- v + ||g||^2 ;  w <- w - lr / (sqrt(v / c) + eps) * g      (updated v; v stored unscaled)
// Lanes with write == true store their 4 columns; the lane with lc == 0 among them stores the moment.
// With sgd == true the step is plain SGD instead, w <- w - lr * g, and the moment is neither read nor written.
template <typename WT, int NC>
__device__ __forceinline__ void adagrad_row(const float (&acc)[NC][4], const RowGeom& g, WT* __restrict__ wrow,
                                            float* __restrict__ vptr, const float v_old, const bool write,
                                            const float lr, const float eps, const float inv_c, const bool sgd = false) {
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int col = g.lc + c * kWave * 4;
        if (col < g.D) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sq = fmaf(acc[c][v], acc[c][v], sq);
        }
    }
    sq = group_sum(sq, g.LPR);  // within the LPR lanes that cover the row
    const float v_new = v_old + sq;
    const float step = sgd ? lr : adagrad_step(v_new, lr, eps, inv_c);
    if (write) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int col = g.lc + c * kWave * 4;
            if (col < g.D) {
                float w[4];
                RowIO<WT>::load4(wrow + col, w);
#pragma unroll
                for (int v = 0; v < 4; ++v) w[v] = fmaf(-step, acc[c][v], w[v]);
                RowIO<WT>::store4(wrow + col, w);
            }
        }
        if (g.lc == 0 && !sgd) *vptr = v_new;
    }
}

// ---- long rows (> kSegChunk lookups): the head of the Zipf distribution ------------------------------
// The upstream gradient block of one table (B x D_t floats, 16-32 MB at large batch sizes) is several times
// one XCD's 4 MB L2, so the slices that hot rows gather would stream through the L2 again and again
// (measured: random 1 KB reads run at ~28 TB/s from an L2-resident set, ~8 TB/s otherwise).  For such tables
// every XCD owns one eighth of the bags (workgroup id mod 8 is the XCD the dispatcher picks) and walks it in
// sub-slices of at most ~0.5 MB of gradient, one sub-slice per sweep over the list of hot rows; the hot rows are
// listed table by table, so at any time an XCD works on one sub-slice of one or two tables, which stays
// resident in its L2 while all hot rows of the table pass over it.  The stable sort left a row's lookups in
// ascending bag order, so the lookups of a sub-slice are one contiguous range found by binary search.
// A hot row thus has 8 partial sums, one per XCD, accumulated over the sweeps.
// Hot rows of tables whose gradient block fits the L2 anyway are cut into up to 16 equal parts instead.
constexpr int kMaxParts = 16;
constexpr int kMaxPartsSeq = 1024;
constexpr uint32_t kSliceBytes = (uint32_t)512 << 10;

constexpr uint32_t kSlicedFlag = 0x80000000u;
constexpr uint32_t kDenseFlag = 0x40000000u;   // the row is reduced by the dense-row kernel: no units, kDenseChunks partial sums
constexpr uint32_t kDenseDiv = 8;   // a dense row has at least B / kDenseDiv lookups (and at least kDenseMin)
constexpr uint32_t kDenseMin = 4096;
constexpr int kDenseMaxCand = 1024;            // candidates per table the selection can rank

// number of sub-slices of a table's gradient block (power of two); >= 8 means "bag-sliced over the XCDs"
__device__ __host__ __forceinline__ uint32_t slices_for(uint32_t B, uint32_t D) {
    const uint64_t bytes = (uint64_t)B * D * 4u;
    uint32_t S = 1;
    while (S < kMaxSlices && bytes > (uint64_t)S * kSliceBytes) S <<= 1;
    return S;
}

// first i in [lo, hi) with a[i] >= x (a ascending), or hi
__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t* __restrict__ a, uint32_t lo, uint32_t hi, uint32_t x) {
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// How a long row is worked on.  Bag-sliced rows (tables whose gradient block is >= 8 sub-slices): every XCD
// reduces the row's lookups that fall into its bags, sub-slice by sub-slice (one per sweep); rows with at least
// kHeavyMin lookups are additionally cut into C units per (XCD, sweep) so that all units are of similar size -
// otherwise the few heaviest rows would keep their workgroups busy long after the others have moved on to later
// tables, and the XCD's working set would no longer be one sub-slice.  Other long rows: C equal shares.
constexpr uint32_t kHeavyMin = 8192;
constexpr uint32_t kUnitLookups = 256;
struct LongPlan {
    bool sliced;
    uint32_t nsub;    // sub-slices per XCD (sweeps that touch the row)
    uint32_t C;       // units per (XCD, sweep) if sliced, else number of equal shares
    uint32_t nslots;  // partial sums of the row
};
__device__ __forceinline__ LongPlan long_plan(uint32_t B, uint32_t D, uint32_t len, bool seq) {
    LongPlan p;
    const uint32_t S = slices_for(B, D);
    if (S >= 8u) {
        p.sliced = true;
        p.nsub = S / 8u;
        p.C = len >= kHeavyMin ? len / (8u * p.nsub * kUnitLookups) + 2u : 1u;
        p.nslots = p.C == 1u ? 8u : 8u * p.nsub * p.C;   // light: one per XCD, summed over the sweeps in place
    } else {
        p.sliced = false;
        p.nsub = 1;
        p.C = (len + kSegChunk - 1) / kSegChunk;
        // non-pooled: every lookup has a gradient row of its own, nothing to keep in a cache, so just more parts
        const uint32_t cap = seq ? (uint32_t)kMaxPartsSeq : (uint32_t)kMaxParts;
        if (p.C > cap) p.C = cap;
        p.nslots = p.C;
    }
    return p;
}

// ---- 1a. the long rows: found, counted and given their partial-sum slots in row order ---------------------------
// Three small passes over the unique rows, kLongTile rows per workgroup:
//   count : long rows and the slots they need per tile, long rows per table
//   scan  : exclusive scans of the per-tile and per-table counts (one workgroup)
//   fill  : every long row gets its slots - the running sum in ROW order, so that which rows still find room in
//           the slot area does not depend on timing - and its place in the list, grouped by table
// A row that finds no room (the area is sized for skewed batches, not for the worst case of every lookup sitting in
// a row just above the threshold) is marked: the kernel that applies the steps then reduces it itself, slowly.
// long_list entry: (u, first slot, C | flags, table).  Order inside a table is arrival order; it only decides the
// order in which units are handed out, never an order of additions.
constexpr int kLongTile = 1024;
constexpr uint32_t kOverflowFlag = 0x20000000u;   // no slots: reduced inside seg_long_update_kernel
constexpr uint32_t kCountMask = 0x1FFFFFFFu;

struct LongRow {
    bool is_long;
    int t;
    LongPlan p;
};
// (s0 = seg_start[u], len = the row's number of lookups, anything for u >= U: loaded by the caller, for all of a
// thread's rows before any is looked at)
__device__ __forceinline__ LongRow long_row(const SegArgs& a, const uint32_t u, const uint32_t U, const uint32_t s0,
                                            const uint32_t len) {
    LongRow r;
    r.is_long = false;
    r.t = 0;
    r.p.sliced = false; r.p.nsub = 1; r.p.C = 0; r.p.nslots = 0;
    if (u >= U) return r;
    if (len <= (uint32_t)kSegChunk) return r;
    const uint32_t key = a.keys_unique[u];
    if (key >= a.total_rows) return r;   // the pseudo-row of invalid ids
    r.is_long = true;
    // the table: from the bag of the row's first lookup where the payload is a bag (one load instead of a search)
    r.t = a.seq ? table_of_key(a.row_base, a.T, key) : (int)(a.bag_sorted[s0] / (uint32_t)a.B);
    r.p = long_plan((uint32_t)a.B, (uint32_t)(a.D_off[r.t + 1] - a.D_off[r.t]), len, a.seq != 0);
    return r;
}

__global__ __launch_bounds__(256) void seg_long_count_kernel(const SegArgs a) {
    __shared__ uint32_t s_n, s_slots;
    const uint32_t U = a.counters[0];
    const uint32_t ntiles = (U + kLongTile - 1) / kLongTile;
    for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (threadIdx.x == 0) s_n = s_slots = 0u;
        __syncthreads();
        uint32_t n = 0, slots = 0;
        uint32_t start[kLongTile / 256], len[kLongTile / 256];
#pragma unroll
        for (int k = 0; k < kLongTile / 256; ++k) {
            const uint32_t u = tile * kLongTile + k * 256 + threadIdx.x;
            // unconditional loads, so that they overlap: a row behind the last reads row 0 (seg_start always has two
            // entries), and long_row looks at no length of a row that does not exist
            const uint32_t uc = u < U ? u : 0u;
            start[k] = a.seg_start[uc];
            len[k] = a.seg_start[uc + 1] - start[k];
        }
#pragma unroll
        for (int k = 0; k < kLongTile / 256; ++k) {
            const uint32_t u = tile * kLongTile + k * 256 + threadIdx.x;
            const LongRow r = long_row(a, u, U, start[k], len[k]);
            if (r.is_long) {
                ++n;
                slots += r.p.nslots;
                atomicAdd(&a.tcount[r.t], 1u);
            }
        }
        if (n) {
            atomicAdd(&s_n, n);
            atomicAdd(&s_slots, slots);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            a.tile_long[tile] = s_n;
            a.tile_slots[tile] = s_slots;
        }
        __syncthreads();
    }
}

// exclusive scan of v[0 .. n) in place (one workgroup of 1024 threads, four entries per thread and round); returns
// the total
__device__ __forceinline__ uint32_t scan_in_place_1024(uint32_t* __restrict__ v, const int n, uint32_t* smem) {
    uint32_t carry = 0;
    for (int base = 0; base < n; base += 4 * 1024) {
        const int i = base + 4 * (int)threadIdx.x;
        uint32_t x[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = (i + q < n) ? v[i + q] : 0u;
        uint32_t tot;
        uint32_t run = carry + block_excl_scan<1024>(x[0] + x[1] + x[2] + x[3], smem, &tot);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i + q < n) v[i + q] = run;
            run += x[q];
        }
        carry += tot;
    }
    return carry;
}

__global__ __launch_bounds__(1024) void seg_long_scan_kernel(const SegArgs a, uint32_t* __restrict__ tbase,
                                                             uint32_t* __restrict__ tfill,
                                                             uint32_t* __restrict__ counters) {
    __shared__ uint32_t smem[1024 / kWave];
    const int ntiles = (int)((counters[0] + kLongTile - 1) / kLongTile);   // the tiles that hold rows
    for (int i = threadIdx.x; i <= a.T; i += 1024) {
        tbase[i] = i < a.T ? a.tcount[i] : 0u;
        tfill[i] = 0u;
    }
    __syncthreads();
    const uint32_t nlong = scan_in_place_1024(tbase, a.T + 1, smem);   // tbase[T] = number of long rows
    scan_in_place_1024(a.tile_long, ntiles, smem);
    scan_in_place_1024(a.tile_slots, ntiles, smem);
    if (threadIdx.x == 0) counters[1] = nlong;
}

__global__ __launch_bounds__(256) void seg_long_fill_kernel(const SegArgs a, const uint32_t* __restrict__ tbase,
                                                            uint32_t* __restrict__ tfill) {
    __shared__ uint32_t smem[256 / kWave];
    const uint32_t U = a.counters[0];
    const uint32_t ntiles = (U + kLongTile - 1) / kLongTile;
    for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (a.tile_long[tile + 1 < ntiles ? tile + 1 : tile] == a.tile_long[tile] && tile + 1 < ntiles) continue;   // no long row here
        uint32_t slot_run = a.tile_slots[tile];       // slots of the long rows before this tile
        uint32_t start[kLongTile / 256], len[kLongTile / 256];
#pragma unroll
        for (int k = 0; k < kLongTile / 256; ++k) {
            const uint32_t u = tile * kLongTile + k * 256 + threadIdx.x;
            // unconditional loads, so that they overlap: a row behind the last reads row 0 (seg_start always has two
            // entries), and long_row looks at no length of a row that does not exist
            const uint32_t uc = u < U ? u : 0u;
            start[k] = a.seg_start[uc];
            len[k] = a.seg_start[uc + 1] - start[k];
        }
#pragma unroll
        for (int k = 0; k < kLongTile / 256; ++k) {   // (rows k*256 .. k*256+255 of the tile, in row order)
            const uint32_t u = tile * kLongTile + k * 256 + threadIdx.x;
            const LongRow r = long_row(a, u, U, start[k], len[k]);
            uint32_t tot;
            const uint32_t slot = slot_run + block_excl_scan<256>(r.is_long ? r.p.nslots : 0u, smem, &tot);
            slot_run += tot;
            if (!r.is_long) continue;
            const uint32_t pos = tbase[r.t] + atomicAdd(&tfill[r.t], 1u);
            if (pos >= a.cap_long) continue;   // (cannot happen: at most nnz / (kSegChunk + 1) rows are long)
            const uint32_t flags = r.p.sliced ? kSlicedFlag : 0u;
            uint4* e = reinterpret_cast<uint4*>(a.long_list) + pos;
            if (slot + r.p.nslots <= a.dense_slot0) *e = make_uint4(u, slot, r.p.C | flags, (uint32_t)r.t);
            else *e = make_uint4(u, 0u, flags | kOverflowFlag, (uint32_t)r.t);   // no room: no units, C = 0
        }
    }
}

// ---- 1c. the hot-row hint for the next forward: per table the kHotRows rows with the most lookups ------------------
// One workgroup per table ranks the table's long rows by their number of lookups (ties: smaller key first) and
// leaves the table-local ids of the first kHotRows in the handle.  With more long rows than can be ranked the first
// kHotRows of the list serve: the list is a hint, the forward gives the same result whatever it holds.
constexpr int kHotMaxCand = 1024;
__global__ __launch_bounds__(256) void hot_select_kernel(const SegArgs a, const uint32_t* __restrict__ tbase,
                                                         uint32_t* __restrict__ hot_ids, uint32_t* __restrict__ hot_n) {
    __shared__ uint32_t c_len[kHotMaxCand], c_key[kHotMaxCand];
    const int t = blockIdx.x;
    const uint4* list = reinterpret_cast<const uint4*>(a.long_list);
    const uint32_t nlong = a.counters[1] < a.cap_long ? a.counters[1] : a.cap_long;
    const uint32_t i0 = tbase[t] < nlong ? tbase[t] : nlong, i1 = tbase[t + 1] < nlong ? tbase[t + 1] : nlong;
    const uint32_t n = i1 - i0;
    const uint32_t rb = (uint32_t)a.row_base[t];
    uint32_t* ids = hot_ids + (size_t)t * kHotRows;
    if (threadIdx.x == 0) hot_n[t] = n < (uint32_t)kHotRows ? n : (uint32_t)kHotRows;
    if (n > (uint32_t)kHotMaxCand) {
        for (uint32_t k = threadIdx.x; k < (uint32_t)kHotRows; k += blockDim.x) ids[k] = a.keys_unique[list[i0 + k].x] - rb;
        return;
    }
    for (uint32_t k = threadIdx.x; k < n; k += blockDim.x) {
        const uint32_t u = list[i0 + k].x;
        c_len[k] = a.seg_start[u + 1] - a.seg_start[u];
        c_key[k] = a.keys_unique[u];
    }
    __syncthreads();
    for (uint32_t k = threadIdx.x; k < n; k += blockDim.x) {
        uint32_t rank = 0;
        for (uint32_t j = 0; j < n; ++j)
            rank += (c_len[j] > c_len[k] || (c_len[j] == c_len[k] && c_key[j] < c_key[k])) ? 1u : 0u;
        if (rank < (uint32_t)kHotRows) ids[rank] = c_key[k] - rb;
    }
}

// ---- 1d. work units in list (= table) order: unit (pos, c) for c < C(pos); one workgroup -------------
__global__ __launch_bounds__(1024) void seg_long_units_kernel(const SegArgs a, uint32_t* __restrict__ counters) {
    __shared__ uint32_t smem[1024 / kWave];
    const uint32_t nlong = counters[1] < a.cap_long ? counters[1] : a.cap_long;
    const uint4* list = reinterpret_cast<const uint4*>(a.long_list);
    uint32_t carry = 0;
    for (uint32_t base = 0; base < nlong; base += 1024) {
        const uint32_t pos = base + threadIdx.x;
        const uint32_t z = pos < nlong ? list[pos].z : 0u;
        const uint32_t C = (z & kDenseFlag) ? 0u : (z & kCountMask);   // dense rows and rows without slots have no units
        uint32_t tot;
        const uint32_t ex = block_excl_scan<1024>(C, smem, &tot);
        for (uint32_t c = 0; c < C; ++c) {
            const uint32_t e = carry + ex + c;
            if (e < a.cap_units) a.unit_list[e] = make_uint2(pos, c);
        }
        carry += tot;
    }
    if (threadIdx.x == 0) counters[3] = carry < a.cap_units ? carry : a.cap_units;  // number of units
}

// ---- 1e. bag-sliced rows: where each sub-slice starts in the row's segment (one wavefront per row) ------
// bounds[pos][k] = first sorted position of the row whose bag is >= start of sub-slice k, k = 0 .. S; the
// sub-slices of XCD x are k = x*nsub .. (x+1)*nsub - 1.
__global__ __launch_bounds__(kSegThreads) void seg_long_bounds_kernel(const SegArgs a) {
    const int lane = lane_id();
    const uint32_t nlong = a.counters[1] < a.cap_long ? a.counters[1] : a.cap_long;
    const uint4* list = reinterpret_cast<const uint4*>(a.long_list);
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    const uint32_t W8 = ((uint32_t)a.B + 7u) / 8u;
    for (uint32_t pos = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); pos < nlong; pos += nwaves) {
        const uint4 ent = list[pos];
        if (!(ent.z & kSlicedFlag)) continue;
        const int t = (int)ent.w;
        const uint32_t nsub = slices_for((uint32_t)a.B, (uint32_t)(a.D_off[t + 1] - a.D_off[t])) / 8u;
        const uint32_t S = 8u * nsub;  // <= 64
        const uint32_t Wsub = (W8 + nsub - 1) / nsub;
        const uint32_t s = a.seg_start[ent.x];
        const uint32_t e = a.seg_start[ent.x + 1];
        const uint32_t bag0 = (uint32_t)t * (uint32_t)a.B;
        for (uint32_t k = lane; k <= S; k += kWave) {
            uint32_t r;
            if (k == 0) r = s;
            else if (k == S) r = e;
            else {
                const uint32_t x = k / nsub, j = k - x * nsub;
                uint32_t b_lo = x * W8 + j * Wsub;
                if (b_lo > (x + 1) * W8) b_lo = (x + 1) * W8;
                r = lower_bound_u32(a.bag_sorted, s, e, bag0 + b_lo);
            }
            a.bounds[(size_t)pos * (kMaxSlices + 1) + k] = r;
        }
    }
}

// ---- 2. one wavefront per unit (and XCD); one launch per sweep ------------------------------------------
// partial[slot] (+)= sum of a range of the row's lookups.  A light row's partial sum is accumulated over the
// sweeps; the kernel boundary between two sweeps orders those updates.
// One unit on one XCD in one sweep: partial[slot] (+)= sum over a range of the row's lookups (whole wavefront).
template <int NC, bool MEAN, typename GT>
__device__ __forceinline__ void long_unit(const SegArgs& a, const uint32_t sweep, const uint32_t xcd, const uint32_t e) {
    const uint2 un = a.unit_list[e];
    const uint4 ent = reinterpret_cast<const uint4*>(a.long_list)[un.x];
    const uint32_t C = ent.z & kCountMask;
    const uint32_t c = un.y;
    const int t = (int)ent.w;
    const int d0 = a.D_off[t];
    const RowGeom g = row_geom(a.D_off[t + 1] - d0);
    uint32_t lo, hi, slot;
    bool accumulate = false;
    if (ent.z & kSlicedFlag) {
        const uint32_t nsub = slices_for((uint32_t)a.B, (uint32_t)g.D) / 8u;
        if (sweep >= nsub) return;
        const uint32_t* bd = a.bounds + (size_t)un.x * (kMaxSlices + 1) + xcd * nsub + sweep;
        const uint32_t r_lo = bd[0], r_hi = bd[1];            // this XCD's lookups of the sub-slice
        const uint32_t q = (r_hi - r_lo + C - 1) / C;          // ... cut into C units
        lo = r_lo + c * q < r_hi ? r_lo + c * q : r_hi;
        hi = lo + q < r_hi ? lo + q : r_hi;
        if (C == 1u) {
            slot = ent.y + xcd;
            accumulate = sweep > 0;  // the earlier sweep's launch has finished: plain read-add-write
        } else {
            slot = ent.y + (xcd * nsub + sweep) * C + c;
        }
    } else {
        if (sweep != 0u || (e & 7u) != xcd) return;  // every XCD sees every unit; each takes every eighth
        const uint32_t s = a.seg_start[ent.x];
        const uint64_t len = a.seg_start[ent.x + 1] - s;
        lo = s + (uint32_t)(len * c / C);
        hi = s + (uint32_t)(len * (c + 1) / C);
        slot = ent.y + c;
    }
    float acc[NC][4];
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) acc[cc][0] = acc[cc][1] = acc[cc][2] = acc[cc][3] = 0.f;
    const GradAddr ga = grad_addr(a, t, g.D);
    segment_reduce<NC, MEAN, GT>(acc, g, static_cast<const GT*>(a.grad_out) + ga.base, ga.pitch, ga.row0,
                                 a.bag_sorted, a.offsets, lo, hi);
    fold_groups<NC>(acc, g);
    if (g.sub == 0) {
        float* dst = a.partial + (size_t)slot * a.maxD;
#pragma unroll
        for (int cc = 0; cc < NC; ++cc) {
            const int col = g.lc + cc * kWave * 4;
            if (col < g.D) {
                float4 r = make_float4(acc[cc][0], acc[cc][1], acc[cc][2], acc[cc][3]);
                if (accumulate) {
                    const float4 o = *reinterpret_cast<const float4*>(dst + col);
                    r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w;
                }
                *reinterpret_cast<float4*>(dst + col) = r;
            }
        }
    }
}

// Units are handed out in list order, kTicketUnits per wavefront and ticket, through one counter per (sweep, XCD):
// the units in flight on an XCD are then neighbours in the list (the hot rows of one or two tables), whatever the
// individual units cost, and the sub-slices they gather from stay in that XCD's L2.  (Walking the list with a
// fixed stride lets the workgroups drift apart: measured L2 hit rate 34% against 90% in list order.)
template <int NC, bool MEAN, typename GT>
__global__ __launch_bounds__(kSegThreads, NC == 1 ? 8 : 4) void seg_long_partial_kernel(const SegArgs a, const uint32_t sweep) {
    constexpr uint32_t kWpb = kSegThreads / kWave;
    constexpr uint32_t kTicketUnits = 1;
    __shared__ uint32_t s_ticket;
    const uint32_t nunits = a.counters[3];
    const uint32_t xcd = blockIdx.x & 7u;
    uint32_t* const ticket = a.tickets + (sweep * 8u + xcd) * kTicketStride;
    for (;;) {
        if (threadIdx.x == 0) s_ticket = atomicAdd(ticket, 1u);
        __syncthreads();
        const uint32_t first = s_ticket * (kWpb * kTicketUnits);
        __syncthreads();   // everyone has read the ticket before the next one overwrites it
        if (first >= nunits) break;
#pragma unroll 1
        for (uint32_t k = 0; k < kTicketUnits; ++k) {
            const uint32_t e = first + k * kWpb + (threadIdx.x >> 6);
            if (e < nunits) long_unit<NC, MEAN, GT>(a, sweep, xcd, e);   // the last ticket may be partly empty
        }
    }
}

// ---- 2b. dense rows ------------------------------------------------------------------------------------------
// The few hottest rows of a table appear in a large share of its bags (at Zipf exponents around 1.1 a dozen rows
// take a third of all lookups).  Reducing them lookup by lookup reads every bag's gradient row once per hot row that
// the bag holds; instead, the table's gradient block is streamed ONCE, bag by bag, and every gradient row is added
// to the accumulators of all the table's dense rows, weighted by how often the bag holds that row (mostly 0 or 1).
// A wavefront owns one bag chunk of one table: it keeps kDenseRows x D accumulators in registers, walks its bags in
// blocks of 64, builds the 64 x kDenseRows count table of a block in LDS from the rows' sorted bag lists (a cursor
// per row; the lists are ascending), and ends with one partial sum per dense row.  seg_long_update adds the
// kDenseChunks partial sums of a row in chunk order, so the result does not depend on scheduling.
// (Gradients are taken to be finite: count * fragment with a count of zero and an infinite element is NaN, so a
// non-finite element of one bag's gradient makes every dense row of that table non-finite, not only the rows the
// bag holds.  Guarding the product costs a third of this kernel's time - measured 1.6 -> 2.2 ms at the largest
// workload - for inputs that have already lost the training run.)
// Selection (one workgroup per table): rows with at least max(kDenseMin, B/kDenseDiv) lookups, the kDenseRows longest (ties:
// smaller key first), and only if together they hold at least 2*B lookups - otherwise streaming the whole block
// costs more than the lookups it saves.  Only bag-sliced tables qualify (others fit the L2 anyway).
__global__ __launch_bounds__(256) void seg_dense_select_kernel(const SegArgs a, const uint32_t* __restrict__ tbase) {
    __shared__ uint32_t c_len[kDenseMaxCand], c_key[kDenseMaxCand], c_pos[kDenseMaxCand], c_rank[kDenseMaxCand];
    __shared__ uint32_t s_n, s_sum;
    const int t = blockIdx.x;
    uint4* list = reinterpret_cast<uint4*>(a.long_list);
    const uint32_t D = (uint32_t)(a.D_off[t + 1] - a.D_off[t]);
    if (threadIdx.x == 0) {
        s_n = 0u;
        s_sum = 0u;
        a.dense_n[t] = 0u;
    }
    __syncthreads();
    if (a.seq || D > 256u || slices_for((uint32_t)a.B, D) < 8u) return;
    const uint32_t nlong = a.counters[1] < a.cap_long ? a.counters[1] : a.cap_long;
    const uint32_t i0 = tbase[t] < nlong ? tbase[t] : nlong, i1 = tbase[t + 1] < nlong ? tbase[t + 1] : nlong;
    const uint32_t thr = (uint32_t)a.B / kDenseDiv > kDenseMin ? (uint32_t)a.B / kDenseDiv : kDenseMin;
    for (uint32_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) {
        const uint4 ent = list[i];
        if (!(ent.z & kSlicedFlag)) continue;
        const uint32_t len = a.seg_start[ent.x + 1] - a.seg_start[ent.x];
        if (len < thr) continue;
        const uint32_t j = atomicAdd(&s_n, 1u);
        if (j < (uint32_t)kDenseMaxCand) {
            c_len[j] = len;
            c_key[j] = a.keys_unique[ent.x];
            c_pos[j] = i;
        }
    }
    __syncthreads();
    const uint32_t n = s_n;
    if (n == 0u || n > (uint32_t)kDenseMaxCand) return;   // (more candidates than can be ranked: all stay sparse)
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) {
        uint32_t rank = 0;
        for (uint32_t j = 0; j < n; ++j)
            rank += (c_len[j] > c_len[i] || (c_len[j] == c_len[i] && c_key[j] < c_key[i])) ? 1u : 0u;
        c_rank[i] = rank;
        if (rank < (uint32_t)kDenseRows) atomicAdd(&s_sum, c_len[i] < 0x08000000u ? c_len[i] : 0x08000000u);
    }
    __syncthreads();
    if (s_sum < 2u * (uint32_t)a.B) return;
    // every selected row gets the kDenseChunks slots that the reserved region holds for (table, rank)
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) {
        if (c_rank[i] < (uint32_t)kDenseRows) {
            a.dense_rows[t * kDenseRows + c_rank[i]] = c_pos[i];
            a.long_list[4 * (size_t)c_pos[i] + 1] = a.dense_slot0 + ((uint32_t)t * kDenseRows + c_rank[i]) * (uint32_t)kDenseChunks;
            a.long_list[4 * (size_t)c_pos[i] + 2] = kDenseFlag;
        }
    }
    if (threadIdx.x == 0) a.dense_n[t] = n < (uint32_t)kDenseRows ? n : (uint32_t)kDenseRows;
}

// borders of the bag chunks inside every dense row's segment: one wavefront per row, one border per lane
__global__ __launch_bounds__(kSegThreads) void seg_dense_bounds_kernel(const SegArgs a) {
    const int t = blockIdx.x;
    const uint32_t n = a.dense_n[t];
    if (n == 0u) return;
    const int lane = lane_id();
    const uint4* list = reinterpret_cast<const uint4*>(a.long_list);
    const uint32_t CB = ((uint32_t)a.B + kDenseChunks - 1) / kDenseChunks;
    const uint32_t bag0 = (uint32_t)t * (uint32_t)a.B;
    for (uint32_t h = threadIdx.x >> 6; h < n; h += kSegThreads / kWave) {
        const uint4 ent = list[a.dense_rows[t * kDenseRows + h]];
        const uint32_t s = a.seg_start[ent.x], e = a.seg_start[ent.x + 1];
        for (int c = lane; c <= kDenseChunks; c += kWave) {
            uint32_t r;
            if (c == 0) r = s;
            else if (c == kDenseChunks) r = e;
            else {
                const uint32_t b = (uint32_t)c * CB < (uint32_t)a.B ? (uint32_t)c * CB : (uint32_t)a.B;
                r = lower_bound_u32(a.bag_sorted, s, e, bag0 + b);
            }
            a.dense_bounds[((size_t)t * kDenseRows + h) * (kDenseChunks + 1) + c] = r;
        }
    }
}

constexpr int kDenseU = 3;   // gradient rows in flight per lane group
template <bool MEAN, typename GT>
__global__ __launch_bounds__(kSegThreads, kDenseRows <= 16 ? 3 : 2) void seg_dense_partial_kernel(const SegArgs a) {
    __shared__ uint32_t s_cnt[kSegThreads / kWave][kWave][kDenseRows];   // per wavefront: counts of a block of 64 bags
    const int lane = lane_id();
    const int wv = threadIdx.x >> 6;
    const uint32_t wid = blockIdx.x * (kSegThreads / kWave) + (uint32_t)wv;
    const int t = (int)(wid / kDenseChunks);
    const uint32_t c = wid % kDenseChunks;
    if (t >= a.T) return;
    const uint32_t n = a.dense_n[t];
    if (n == 0u) return;   // (wavefronts leave on their own: the kernel uses no workgroup barrier)
    const int d0 = a.D_off[t];
    const RowGeom g = row_geom(a.D_off[t + 1] - d0);
    const uint32_t B = (uint32_t)a.B;
    const uint32_t CB = (B + kDenseChunks - 1) / kDenseChunks;
    const uint32_t b_lo = c * CB < B ? c * CB : B;
    const uint32_t b_hi = b_lo + CB < B ? b_lo + CB : B;
    const uint32_t bag0 = (uint32_t)t * B;
    const uint4* list = reinterpret_cast<const uint4*>(a.long_list);
    // lane h < n: cursor into dense row h's sorted bag list, the end of this chunk's part, the row's first slot
    uint32_t cur = 0, end = 0, slot0 = 0;
    if ((uint32_t)lane < n) {
        const size_t o = ((size_t)t * kDenseRows + lane) * (kDenseChunks + 1) + c;
        cur = a.dense_bounds[o];
        end = a.dense_bounds[o + 1];
        slot0 = list[a.dense_rows[t * kDenseRows + lane]].y;
    }
    float acc[kDenseRows][4];
#pragma unroll
    for (int h = 0; h < kDenseRows; ++h) acc[h][0] = acc[h][1] = acc[h][2] = acc[h][3] = 0.f;
    const GT* gcol = static_cast<const GT*>(a.grad_out) + d0 + g.lc;
    const bool col_on = g.lc < g.D;
    uint32_t* cnt = &s_cnt[wv][0][0];
    for (uint32_t sb = b_lo; sb < b_hi; sb += kWave) {
        const uint32_t nb = b_hi - sb < (uint32_t)kWave ? b_hi - sb : (uint32_t)kWave;
        // ---- the block's count table: zero, then one pass per dense row over the part of its list inside the block
#pragma unroll
        for (int q = 0; q < kDenseRows; q += 4)
            *reinterpret_cast<uint4*>(&cnt[lane * kDenseRows + q]) = make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        for (uint32_t h = 0; h < n; ++h) {
            uint32_t ch = __shfl(cur, (int)h, kWave);
            const uint32_t eh = __shfl(end, (int)h, kWave);
            for (;;) {   // the list is ascending, so the entries of this block are a prefix of what is left
                const uint32_t ei = ch + (uint32_t)lane;
                const uint32_t v = ei < eh ? a.bag_sorted[ei] - bag0 - sb : 0xFFFFFFFFu;
                const bool inb = v < nb;
                if (inb) atomicAdd(&cnt[v * kDenseRows + h], 1u);
                const uint32_t k = (uint32_t)__popcll(__ballot(inb));
                ch += k;
                if (k < (uint32_t)kWave) break;
            }
            if ((uint32_t)lane == h) cur = ch;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        float my_s = 1.f;
        if (MEAN && (uint32_t)lane < nb) my_s = bag_scale<true>(a.offsets, bag0 + sb + (uint32_t)lane);
        // ---- stream the block's gradient rows; every lane group takes every G-th bag
        for (uint32_t k0 = 0; k0 < nb; k0 += kDenseU * g.G) {
            typename GradIO<GT>::raw_t x[kDenseU];
            uint32_t kk[kDenseU];
#pragma unroll
            for (int u = 0; u < kDenseU; ++u) {
                kk[u] = k0 + (uint32_t)(u * g.G + g.sub);
                const bool on = kk[u] < nb && col_on;
                x[u] = on ? GradIO<GT>::load(gcol + (int64_t)(sb + kk[u]) * a.sumD) : GradIO<GT>::zero();
            }
#pragma unroll
            for (int u = 0; u < kDenseU; ++u) {
                const uint32_t k = kk[u] & (kWave - 1);   // (a bag beyond nb has a zero gradient fragment and zero counts)
                float4 f = GradIO<GT>::to_float(x[u]);
                if (MEAN) {
                    const float sc = __shfl(my_s, (int)k, kWave);
                    f.x *= sc; f.y *= sc; f.z *= sc; f.w *= sc;
                }
                uint32_t w[kDenseRows];
#pragma unroll
                for (int q = 0; q < kDenseRows; q += 4) {
                    const uint4 r = *reinterpret_cast<const uint4*>(&cnt[k * kDenseRows + q]);
                    w[q] = r.x; w[q + 1] = r.y; w[q + 2] = r.z; w[q + 3] = r.w;
                }
#pragma unroll
                for (int h = 0; h < kDenseRows; ++h) {
                    const float m = (float)w[h];
                    acc[h][0] = fmaf(m, f.x, acc[h][0]);
                    acc[h][1] = fmaf(m, f.y, acc[h][1]);
                    acc[h][2] = fmaf(m, f.z, acc[h][2]);
                    acc[h][3] = fmaf(m, f.w, acc[h][3]);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the reads above precede the next block's zeroing
    }
    // ---- one partial sum per dense row: fold the lane groups, then the first group stores
#pragma unroll
    for (int h = 0; h < kDenseRows; ++h) {
        float one[1][4] = {{acc[h][0], acc[h][1], acc[h][2], acc[h][3]}};
        fold_groups<1>(one, g);
        const uint32_t slot = __shfl(slot0, h, kWave) + c;
        if ((uint32_t)h < n && g.sub == 0 && col_on)
            *reinterpret_cast<float4*>(a.partial + (size_t)slot * a.maxD + g.lc) = make_float4(one[0][0], one[0][1], one[0][2], one[0][3]);
    }
}

// ---- 3a. rows with at most kSegChunk lookups, all tables at most 256 columns wide ------------------
// kSegWaves = wavefronts per SIMD the kernel is compiled and launched for: 8, or 7 with more fragments in flight; the
// host picks (see the launch).
template <typename WT, bool MEAN, typename GT, int kSegWaves>
__global__ __launch_bounds__(kSegThreads, kSegWaves) void seg_update_kernel(const SegArgs a) {
    constexpr int kSegUnroll = seg_unroll<1, MEAN, GT, kSegWaves>();
    const int lane = lane_id();
    const uint32_t U = a.counters[0];
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    // rows per wavefront pass: 64 when there is plenty of work, fewer when the batch touches so few rows that
    // whole wavefronts would otherwise go idle while others walk 64 rows one round after the other
    uint32_t rpw = kWave;
    while (rpw > 8u && U / rpw < 2u * nwaves) rpw >>= 1;
    const uint32_t nblk = (U + rpw - 1) / rpw;
    WT* tables = static_cast<WT*>(a.tables);
    for (uint32_t blk = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); blk < nblk; blk += nwaves) {
        // ---- one row per lane: bounds, key, table, width, moment
        const uint32_t u = (uint32_t)lane < rpw ? blk * rpw + lane : U;
        uint32_t s = 0, e = 0, key = 0;
        if (u < U) {
            s = a.seg_start[u];
            e = a.seg_start[u + 1];
            key = a.keys_unique[u];
        }
        const uint32_t len = e - s;
        bool live = (u < U) && len >= 1 && len <= (uint32_t)kSegChunk && key < a.total_rows;
        int t = 0, D = 4;
        float v = 0.f;
        if (live) {
            t = table_of_key(a.row_base, a.T, key);
            D = a.D_off[t + 1] - a.D_off[t];
            if (D > 256) {   // a wider table's row: the one-wavefront-per-row kernel takes it
                live = false;
                D = 4;
            } else {
                v = a.state ? a.state[key] : 0.f;
            }
        }
        int r = 0;
        while (r < (int)rpw) {
            if (!bcast_lane((int)live, r)) {
                ++r;
                continue;
            }
            const RowGeom g = row_geom(bcast_lane(D, r));   // r is the same in all lanes: scalar reads
            const uint32_t s_r = bcast_lane(s, r);
            const uint32_t len_r = bcast_lane(len, r);
            if (len_r > (uint32_t)kWave) {
                // ---- medium row: the whole wavefront reduces it
                const uint32_t key_r = bcast_lane(key, r);
                const int t_r = bcast_lane(t, r);
                const float v_r = bcast_lane(v, r);
                float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
                const GradAddr ga = grad_addr(a, t_r, g.D);
                segment_reduce<1, MEAN, GT, kSegWaves>(acc, g, static_cast<const GT*>(a.grad_out) + ga.base, ga.pitch, ga.row0,
                                            a.bag_sorted, a.offsets, s_r, s_r + len_r);
                fold_groups<1>(acc, g);
                WT* wrow = tables + a.w_off[t_r] + ((int64_t)key_r - a.row_base[t_r]) * g.D;
                adagrad_row<WT, 1>(acc, g, wrow, a.state + key_r, v_r, g.sub == 0, a.lr, a.eps, a.inv_c, a.state == nullptr);
                ++r;
                continue;
            }
            if (g.G == 1) {
                // ---- a short row as wide as the wavefront (more than 128 columns): one row per round, so its
                // bookkeeping is the same in all lanes and stays on the scalar unit (key, table, bag ids, addresses)
                const uint32_t key_r = bcast_lane(key, r);
                const int t_r = bcast_lane(t, r);
                const float v_r = bcast_lane(v, r);
                uint32_t my_bag = 0;
                float my_s = 1.f;
                if ((uint32_t)lane < len_r) {
                    my_bag = a.bag_sorted[s_r + lane];
                    my_s = bag_scale<MEAN>(a.offsets, my_bag);
                }
                const bool col_on = g.lc < g.D;
                const GradAddr ga = grad_addr(a, t_r, g.D);
                const GT* gcol = static_cast<const GT*>(a.grad_out) + ga.base + g.lc;
                float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
                for (uint32_t q0 = 0; q0 < len_r; q0 += kSegUnroll) {
                    typename GradIO<GT>::raw_t x[kSegUnroll];
                    float sc[kSegUnroll];
#pragma unroll
                    for (int uu = 0; uu < kSegUnroll; ++uu) {
                        const uint32_t qi = q0 + uu;                                  // < 64 wherever it is used
                        const uint32_t bag = bcast_lane(my_bag, (int)(qi & (kWave - 1)));
                        sc[uu] = MEAN ? bcast_lane(my_s, (int)(qi & (kWave - 1))) : 1.f;
                        const bool on = qi < len_r && col_on;
                        x[uu] = on ? GradIO<GT>::load(gcol + ((int64_t)bag - ga.row0) * ga.pitch) : GradIO<GT>::zero();
                    }
#pragma unroll
                    for (int uu = 0; uu < kSegUnroll; ++uu) {
                        const float4 f = GradIO<GT>::to_float(x[uu]);
                        if (MEAN) {
                            acc[0][0] = fmaf(sc[uu], f.x, acc[0][0]);
                            acc[0][1] = fmaf(sc[uu], f.y, acc[0][1]);
                            acc[0][2] = fmaf(sc[uu], f.z, acc[0][2]);
                            acc[0][3] = fmaf(sc[uu], f.w, acc[0][3]);
                        } else {
                            acc[0][0] += f.x;
                            acc[0][1] += f.y;
                            acc[0][2] += f.z;
                            acc[0][3] += f.w;
                        }
                    }
                }
                WT* wrow = tables + a.w_off[t_r] + ((int64_t)key_r - a.row_base[t_r]) * g.D;
                adagrad_row<WT, 1>(acc, g, wrow, a.state + key_r, v_r, true, a.lr, a.eps, a.inv_c, a.state == nullptr);
                ++r;
                continue;
            }
            // ---- short rows: rows r .. r+k-1 share the width of row r and have at most 64 lookups in total
            const bool q = live && D == g.D && lane >= r && lane < r + g.G && (e - s_r) <= (uint32_t)kWave;
            const uint64_t m = __ballot(q) >> r;                       // bit j: row r+j qualifies
            const int k = (~m == 0ull) ? kWave : (__ffsll((unsigned long long)(~m)) - 1);  // trailing ones, >= 1
            const uint32_t tot = bcast_lane(e, r + k - 1) - s_r;   // lookups of the k rows, <= 64
            uint32_t my_bag = 0;
            float my_s = 1.f;
            if ((uint32_t)lane < tot) {
                my_bag = a.bag_sorted[s_r + lane];
                my_s = bag_scale<MEAN>(a.offsets, my_bag);
            }
            // this lane group's row
            const bool gon = g.sub < k;
            const int gi = (r + g.sub) & (kWave - 1);
            const uint32_t gs = __shfl(s, gi, kWave);
            // cross-lane reads stay outside any lane-dependent condition: a lane that sits out cannot be read from
            const uint32_t glen_any = __shfl(len, gi, kWave);
            const uint32_t glen = gon ? glen_any : 0u;
            const uint32_t gkey = __shfl(key, gi, kWave);
            const int gt = __shfl(t, gi, kWave);
            const float gv = __shfl(v, gi, kWave);
            const int goff = (int)(gs - s_r);
            const bool col_on = g.lc < g.D;
            const GradAddr ga = grad_addr(a, gt, g.D);
            const GT* gcol = static_cast<const GT*>(a.grad_out) + ga.base + g.lc;
            const int64_t bag0 = ga.row0;
            WT* wrow = tables + a.w_off[gt] + ((int64_t)gkey - a.row_base[gt]) * g.D;
            uint32_t lmax = glen;  // longest row of the round (wave-uniform loop bound)
            for (int o = g.LPR; o < kWave; o <<= 1) {
                const uint32_t other = __shfl_xor(lmax, o, kWave);
                lmax = other > lmax ? other : lmax;
            }
            float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
            for (uint32_t q0 = 0; q0 < lmax; q0 += kSegUnroll) {
                typename GradIO<GT>::raw_t x[kSegUnroll];
                float sc[kSegUnroll];
#pragma unroll
                for (int uu = 0; uu < kSegUnroll; ++uu) {
                    const uint32_t qi = q0 + uu;
                    const int src = (goff + (int)qi) & (kWave - 1);
                    const uint32_t bag = __shfl(my_bag, src, kWave);
                    sc[uu] = MEAN ? __shfl(my_s, src, kWave) : 1.f;
                    const bool on = qi < glen && col_on;
                    x[uu] = on ? GradIO<GT>::load(gcol + ((int64_t)bag - bag0) * ga.pitch) : GradIO<GT>::zero();
                }
#pragma unroll
                for (int uu = 0; uu < kSegUnroll; ++uu) {
                    const float4 f = GradIO<GT>::to_float(x[uu]);
                    if (MEAN) {
                        acc[0][0] = fmaf(sc[uu], f.x, acc[0][0]);
                        acc[0][1] = fmaf(sc[uu], f.y, acc[0][1]);
                        acc[0][2] = fmaf(sc[uu], f.z, acc[0][2]);
                        acc[0][3] = fmaf(sc[uu], f.w, acc[0][3]);
                    } else {
                        acc[0][0] += f.x;
                        acc[0][1] += f.y;
                        acc[0][2] += f.z;
                        acc[0][3] += f.w;
                    }
                }
            }
            adagrad_row<WT, 1>(acc, g, wrow, a.state + gkey, gv, gon, a.lr, a.eps, a.inv_c, a.state == nullptr);
            r += k;
        }
    }
}

// ---- 3b. same rows, any width up to 1024 columns: one wavefront per row ----------------------------
template <typename WT, bool MEAN, typename GT>
__global__ __launch_bounds__(kSegThreads, 4) void seg_update_wide_kernel(const SegArgs a) {
    const uint32_t U = a.counters[0];
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    WT* tables = static_cast<WT*>(a.tables);
    for (uint32_t u = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); u < U; u += nwaves) {
        const uint32_t s = a.seg_start[u];
        const uint32_t e = a.seg_start[u + 1];
        const uint32_t key = a.keys_unique[u];
        if (key >= a.total_rows) continue;  // invalid ids: no row
        if (e - s > (uint32_t)kSegChunk) continue;   // long rows are left to the long-row kernels
        const int t = table_of_key(a.row_base, a.T, key);
        const int d0 = a.D_off[t];
        if (a.mixed && a.D_off[t + 1] - d0 <= 256) continue;   // done by the 64-rows-per-wavefront kernel
        const RowGeom g = row_geom(a.D_off[t + 1] - d0);
        WT* wrow = tables + a.w_off[t] + ((int64_t)key - a.row_base[t]) * g.D;
        float acc[4][4];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        const GradAddr ga = grad_addr(a, t, g.D);
        segment_reduce<4, MEAN, GT>(acc, g, static_cast<const GT*>(a.grad_out) + ga.base, ga.pitch, ga.row0, a.bag_sorted,
                                    a.offsets, s, e);
        fold_groups<4>(acc, g);
        adagrad_row<WT, 4>(acc, g, wrow, a.state + key, a.state ? a.state[key] : 0.f, g.sub == 0, a.lr, a.eps, a.inv_c,
                           a.state == nullptr);
    }
}

// ---- 4. one workgroup per long row: add its partial sums, then the step ----------------------------------
// Wavefront w adds slots w, w+4, ... in ascending order, the four sums are added in wavefront order, and
// wavefront 0 applies the step: a fixed order, so the result does not depend on scheduling.
template <typename WT, bool MEAN, typename GT>
__global__ __launch_bounds__(kSegThreads) void seg_long_update_kernel(const SegArgs a) {
    __shared__ float s_sum[kSegThreads / kWave][1024];
    const uint32_t nlong = a.counters[1] < a.cap_long ? a.counters[1] : a.cap_long;
    WT* tables = static_cast<WT*>(a.tables);
    const int wv = threadIdx.x >> 6;
    for (uint32_t li = blockIdx.x; li < nlong; li += gridDim.x) {
        const uint4 ent = reinterpret_cast<const uint4*>(a.long_list)[li];
        const uint32_t u = ent.x;
        const uint32_t slot = ent.y;
        const uint32_t key = a.keys_unique[u];
        const int t = (int)ent.w;
        const int D = a.D_off[t + 1] - a.D_off[t];
        const uint32_t C = ent.z & kCountMask;
        uint32_t nch = C;  // partial sums of the row
        if (ent.z & kDenseFlag) nch = kDenseChunks;
        else if (ent.z & kOverflowFlag) nch = 0u;
        else if (ent.z & kSlicedFlag) nch = C == 1u ? 8u : C * (slices_for((uint32_t)a.B, (uint32_t)D));
        // here all 64 lanes cover the row (or a 256-column part of it); groups are not used
        RowGeom g;
        g.D = D; g.LPR = kWave; g.G = 1; g.sub = 0; g.lc = lane_id() * 4;
        float acc[4][4];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        if ((ent.z & (kOverflowFlag | kDenseFlag)) == kOverflowFlag) {
            // a row that found no room in the slot area: its lookups are reduced here, a quarter per wavefront in
            // ascending order (slow - one gradient fragment in flight - but only batches far from the skew the area
            // is sized for come here)
            const uint32_t s0 = a.seg_start[u], len = a.seg_start[u + 1] - s0;
            const uint32_t q = (len + kSegThreads / kWave - 1) / (kSegThreads / kWave);
            const uint32_t lo = s0 + ((uint32_t)wv * q < len ? (uint32_t)wv * q : len);
            const uint32_t hi = s0 + ((uint32_t)(wv + 1) * q < len ? (uint32_t)(wv + 1) * q : len);
            const GradAddr ga = grad_addr(a, t, D);
            const GT* gcol = static_cast<const GT*>(a.grad_out) + ga.base;
            for (uint32_t i = lo; i < hi; ++i) {
                const uint32_t bag = a.bag_sorted[i];
                const float sc = bag_scale<MEAN>(a.offsets, bag);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int col = g.lc + c * 256;
                    if (col < D) {
                        const float4 f = GradIO<GT>::to_float(GradIO<GT>::load(gcol + ((int64_t)bag - ga.row0) * ga.pitch + col));
                        acc[c][0] = fmaf(sc, f.x, acc[c][0]); acc[c][1] = fmaf(sc, f.y, acc[c][1]);
                        acc[c][2] = fmaf(sc, f.z, acc[c][2]); acc[c][3] = fmaf(sc, f.w, acc[c][3]);
                    }
                }
            }
        }
        for (uint32_t k = (uint32_t)wv; k < nch; k += kSegThreads / kWave) {
            const float* src = a.partial + (size_t)(slot + k) * a.maxD;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int col = g.lc + c * 256;
                if (col < D) {
                    const float4 v = *reinterpret_cast<const float4*>(src + col);
                    acc[c][0] += v.x; acc[c][1] += v.y; acc[c][2] += v.z; acc[c][3] += v.w;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int col = g.lc + c * 256;
            if (col < D) *reinterpret_cast<float4*>(&s_sum[wv][col]) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
        }
        __syncthreads();
        if (wv == 0) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int col = g.lc + c * 256;
                if (col < D) {
#pragma unroll
                    for (int w2 = 1; w2 < kSegThreads / kWave; ++w2) {
                        const float4 o = *reinterpret_cast<const float4*>(&s_sum[w2][col]);
                        acc[c][0] += o.x; acc[c][1] += o.y; acc[c][2] += o.z; acc[c][3] += o.w;
                    }
                }
            }
            WT* wrow = tables + a.w_off[t] + ((int64_t)key - a.row_base[t]) * D;
            adagrad_row<WT, 4>(acc, g, wrow, a.state + key, a.state ? a.state[key] : 0.f, true, a.lr, a.eps, a.inv_c,
                               a.state == nullptr);
        }
        __syncthreads();
    }
}

// Head of every row-update pass: clears what the kernels below count and hand out (hot-row counters, per-table
// counts, unit tickets), so that the pass can be run again on the same sorted batch.  counters[0], the number of
// unique rows, belongs to the sort and stays.
__global__ __launch_bounds__(1024) void seg_reset_kernel(uint32_t* __restrict__ counters, uint32_t* __restrict__ zero,
                                                         const int zero_words) {
    for (int i = threadIdx.x; i < zero_words; i += 1024) zero[i] = 0u;
    if (threadIdx.x >= 1 && threadIdx.x < kCounterWords) counters[threadIdx.x] = 0u;
}

// the two row-update kernels and the hot-row reduction for one gradient element type
template <typename GT>
static void launch_row_updates(const tbe_handle* h, const SegArgs& a, bool mean, bool narrow, bool wide,
                               hipStream_t s) {
    const bool f32 = h->dtype == TBE_F32;
    if (narrow) {
        // every CU filled once; 7 wavefronts per SIMD for 32-bit gradients on binary16 tables when most of their rows
        // are as wide as the wavefront (measured: 20.2 -> 19.8 ms there, but 2.43 -> 2.55 ms on fp32 tables of the
        // same widths, which therefore keep 8)
        if (sizeof(GT) == 4 && !f32 && h->seg_mostly_wavefront_rows) {
            const unsigned grid = 256u * 7u;
            if (mean) seg_update_kernel<__half, true, GT, 7><<<grid, kSegThreads, 0, s>>>(a);
            else seg_update_kernel<__half, false, GT, 7><<<grid, kSegThreads, 0, s>>>(a);
        } else {
            const unsigned grid = 256u * 8u;
            if (f32) {
                if (mean) seg_update_kernel<float, true, GT, 8><<<grid, kSegThreads, 0, s>>>(a);
                else seg_update_kernel<float, false, GT, 8><<<grid, kSegThreads, 0, s>>>(a);
            } else {
                if (mean) seg_update_kernel<__half, true, GT, 8><<<grid, kSegThreads, 0, s>>>(a);
                else seg_update_kernel<__half, false, GT, 8><<<grid, kSegThreads, 0, s>>>(a);
            }
        }
    }
    if (wide) {
        if (f32) {
            if (mean) seg_update_wide_kernel<float, true, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            else seg_update_wide_kernel<float, false, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        } else {
            if (mean) seg_update_wide_kernel<__half, true, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            else seg_update_wide_kernel<__half, false, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        }
    }
}

template <typename GT>
static void launch_long_partial(const SegArgs& a, uint32_t sweep, bool mean, bool narrow, hipStream_t s) {
    if (narrow) {
        if (mean) seg_long_partial_kernel<1, true, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a, sweep);
        else seg_long_partial_kernel<1, false, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a, sweep);
    } else {
        if (mean) seg_long_partial_kernel<4, true, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a, sweep);
        else seg_long_partial_kernel<4, false, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a, sweep);
    }
}

// non-pooled mode: element offset of every table's gradient block, minus start_t * D_t, so that the kernels address
// a lookup by its original position alone
// If offsets is not ascending from 0 to nnz, or the blocks do not fit grad_elems, no gradient address can be
// trusted: the batch is then flagged as an index error and the number of unique rows set to zero, which turns the
// update kernels that follow into no-ops.
__global__ void seq_gbase_kernel(const IdxView offsets, const int32_t* __restrict__ D_off, const int T, const int64_t nnz,
                                 const int64_t grad_elems, int64_t* __restrict__ gbase, uint32_t* __restrict__ counters,
                                 int32_t* __restrict__ err) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int64_t acc = 0;
    bool ok = offsets[0] == 0 && offsets[T] == nnz;
    for (int t = 0; t < T; ++t) {
        const int64_t s0 = offsets[t], s1 = offsets[t + 1];
        const int64_t D = D_off[t + 1] - D_off[t];
        ok = ok && s1 >= s0;
        gbase[t] = acc - s0 * D;
        acc += (s1 > s0 ? s1 - s0 : 0) * D;
    }
    if (!ok || acc > grad_elems) {
        counters[0] = 0u;
        atomicOr(err, 1);
    }
}

template <typename GT>
static void launch_long_update(const SegArgs& a, bool f32, bool mean, hipStream_t s) {
    if (f32) {
        if (mean) seg_long_update_kernel<float, true, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        else seg_long_update_kernel<float, false, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
    } else {
        if (mean) seg_long_update_kernel<__half, true, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        else seg_long_update_kernel<__half, false, GT><<<kSegBlocks, kSegThreads, 0, s>>>(a);
    }
}

template <typename GT>
static void launch_dense_partial(const SegArgs& a, unsigned grid, bool mean, hipStream_t s) {
    if (mean) seg_dense_partial_kernel<true, GT><<<grid, kSegThreads, 0, s>>>(a);
    else seg_dense_partial_kernel<false, GT><<<grid, kSegThreads, 0, s>>>(a);
}

hipError_t launch_segment_update(const tbe_handle* h, const Workspace& w, char* ws, int spare, const void* grad_out,
                                 int grad_io, const void* offsets, int idx32, int32_t B, tbe_pooling pooling, float lr,
                                 float eps, float c, void* tables, float* state, int seq, int64_t grad_elems, hipStream_t s) {
    SegArgs a;
    a.seq = seq;
    a.seq_gbase = reinterpret_cast<const int64_t*>(ws + w.seq_gbase);

    a.keys_unique = reinterpret_cast<const uint32_t*>(ws + w.vals[spare]);
    a.seg_start = reinterpret_cast<const uint32_t*>(ws + w.seg_start);
    uint32_t* counters = reinterpret_cast<uint32_t*>(ws + w.counters);
    a.counters = counters;
    seg_reset_kernel<<<1, 1024, 0, s>>>(counters, reinterpret_cast<uint32_t*>(ws + w.long_tables),
                                        (int)((w.tickets - w.long_tables) / 4) + kTicketWords);
    if (seq)
        seq_gbase_kernel<<<1, 64, 0, s>>>(IdxView{offsets, idx32}, h->d_D_off, h->T, (int64_t)w.n, grad_elems,
                                          reinterpret_cast<int64_t*>(ws + w.seq_gbase), counters, h->d_err);
    a.bag_sorted = reinterpret_cast<const uint32_t*>(ws + w.vals[spare ^ 1]);   // the sorted payload stream
    a.offsets = IdxView{offsets, idx32};
    a.grad_out = grad_out;
    a.D_off = h->d_D_off;
    a.row_base = h->d_row_base;
    a.w_off = h->d_w_off;
    a.T = h->T;
    a.B = B;
    a.sumD = h->sumD;
    a.maxD = h->maxD;
    a.total_rows = (uint32_t)h->total_rows;
    a.lr = lr;
    a.eps = eps;
    a.inv_c = 1.0f / c;
    a.tables = tables;
    a.state = state;
    a.long_list = reinterpret_cast<uint32_t*>(ws + w.long_list);
    a.partial = reinterpret_cast<float*>(ws + w.partial);
    a.unit_list = reinterpret_cast<uint2*>(ws + w.unit_list);
    a.bounds = reinterpret_cast<uint32_t*>(ws + w.bounds);
    a.tickets = reinterpret_cast<uint32_t*>(ws + w.tickets);
    a.dense_rows = reinterpret_cast<uint32_t*>(ws + w.dense_rows);
    a.dense_n = reinterpret_cast<uint32_t*>(ws + w.dense_n);
    a.dense_bounds = reinterpret_cast<uint32_t*>(ws + w.dense_bounds);
    a.cap_units = (uint32_t)w.cap_units;
    a.cap_long = (uint32_t)w.cap_long;
    a.cap_chunks = (uint32_t)w.cap_chunks;
    const bool mean = pooling == TBE_MEAN;
    const bool f32 = h->dtype == TBE_F32;
    // Rows of tables up to 256 columns wide go to the kernel that keeps 64 rows per wavefront, rows of wider tables
    // to the one-wavefront-per-row kernel; a handle that holds both kinds runs both, each skipping the other's rows.
    const bool narrow = h->minD <= 256;
    const bool wide = h->maxD > 256;
    a.mixed = narrow && wide ? 1 : 0;
    // the dense-row path: tables up to 256 columns, and only when some such table's gradient block is bag-sliced
    const bool dense = narrow && !seq && slices_for((uint32_t)B, (uint32_t)(h->maxD < 256 ? h->maxD : 256)) >= 8u;
    uint32_t* tcount = reinterpret_cast<uint32_t*>(ws + w.long_tables);
    uint32_t* tbase = tcount + (h->T + 1);
    uint32_t* tfill = tbase + (h->T + 1);
    a.tcount = tcount;
    a.tile_long = reinterpret_cast<uint32_t*>(ws + w.tile_long);
    a.tile_slots = reinterpret_cast<uint32_t*>(ws + w.tile_slots);
    a.dense_slot0 = (uint32_t)w.cap_main;
    {   // rows with at most kSegChunk lookups; the others are noted for the long-row path
        LaunchTimer tm(h, s, "seg_update");
        if (grad_io == 0) launch_row_updates<float>(h, a, mean, narrow, wide, s);
        else if (grad_io == 1) launch_row_updates<__half>(h, a, mean, narrow, wide, s);
        else launch_row_updates<bf16_t>(h, a, mean, narrow, wide, s);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_long_list");
        const unsigned lgrid = (unsigned)(w.long_tiles < 4096 ? w.long_tiles : 4096);
        seg_long_count_kernel<<<lgrid, 256, 0, s>>>(a);
        seg_long_scan_kernel<<<1, 1024, 0, s>>>(a, tbase, tfill, counters);
        seg_long_fill_kernel<<<lgrid, 256, 0, s>>>(a, tbase, tfill);
        if (h->d_hot_ids && !seq) hot_select_kernel<<<h->T, 256, 0, s>>>(a, tbase, h->d_hot_ids, h->d_hot_n);
        if (dense) seg_dense_select_kernel<<<h->T, 256, 0, s>>>(a, tbase);
        seg_long_units_kernel<<<1, 1024, 0, s>>>(a, counters);
        if (slices_for((uint32_t)B, (uint32_t)h->maxD) >= 8u) seg_long_bounds_kernel<<<kSegBlocks, kSegThreads, 0, s>>>(a);   // (a chain of ~17 dependent loads per row: many waves)
        if (dense) seg_dense_bounds_kernel<<<h->T, kSegThreads, 0, s>>>(a);
        tm.done();
    }
    if (dense) {
        LaunchTimer tm(h, s, "seg_dense_partial");
        const unsigned grid = (unsigned)(((int64_t)h->T * kDenseChunks + kSegThreads / kWave - 1) / (kSegThreads / kWave));
        if (grad_io == 0) launch_dense_partial<float>(a, grid, mean, s);
        else if (grad_io == 1) launch_dense_partial<__half>(a, grid, mean, s);
        else launch_dense_partial<bf16_t>(a, grid, mean, s);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_long_partial");
        // one launch per sub-slice of an XCD's bags (as many as the widest table has; at least one for the shares)
        uint32_t nsweeps = slices_for((uint32_t)B, (uint32_t)h->maxD) / 8u;
        if (nsweeps < 1u) nsweeps = 1u;
        for (uint32_t sw = 0; sw < nsweeps; ++sw) {
            if (grad_io == 0) launch_long_partial<float>(a, sw, mean, !wide, s);
            else if (grad_io == 1) launch_long_partial<__half>(a, sw, mean, !wide, s);
            else launch_long_partial<bf16_t>(a, sw, mean, !wide, s);
        }
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_long_update");
        // one row per workgroup and round, a dependent chain of loads each: enough workgroups to fill every CU's slots
        if (grad_io == 0) launch_long_update<float>(a, f32, mean, s);
        else if (grad_io == 1) launch_long_update<__half>(a, f32, mean, s);
        else launch_long_update<bf16_t>(a, f32, mean, s);
        tm.done();
    }
    return hipGetLastError();
}

}  // namespace tbe
