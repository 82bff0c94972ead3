// Forward: pooled lookup, one wavefront per bag.
//
// A bag's rows are D_t * sizeof(weight) contiguous bytes each (128 B .. 1 KB for the shapes of interest),
// so a 64-lane wavefront would waste most lanes on one row.  The wavefront is therefore split into
// G = 64 / LPR groups of LPR lanes, LPR = D_t / kVec lanes covering one row with one 16-byte load per
// lane; the groups walk the bag in an interleaved fashion, four rows per group in flight, and a
// butterfly over the groups folds the partial sums at the end.  The bag's ids are read with one
// coalesced 64-wide load and handed to the groups with cross-lane reads.
#include "tbe_device.h"
#include "tbe_internal.h"

namespace tbe {

constexpr int kFwdThreads = 256;

// Lane-group classes: a bag with more ids than this is walked by a whole wavefront instead of one lane group.  The
// more bags share a wavefront, the more lanes one long bag keeps waiting, so the bound falls with the lanes per row
// (measured at lognormal bag lengths, 8 bags per wavefront: 2.28 ms without, 2.07 / 2.01 / 1.94 / 1.86 ms at 96 / 64 /
// 48 / 32; a bound below the typical length would send ordinary bags the slower way).
__device__ __host__ __forceinline__ int long_bag_min(const int lanes_per_row) {
    return lanes_per_row > 16 ? 64 : (lanes_per_row > 8 ? 48 : 32);
}

// NC = number of 64-lane column chunks a row needs (1 when D <= 64 * kVec); U = rows in flight per group.
// The pooled value that is stored: the sum, or for mean pooling sum / L - the product with the reciprocal, corrected
// once by its exact residual (the usual refinement step of a division), so that a mean that is exactly representable
// (a bag whose ids are all equal, say) comes out exact and a 16-bit `out` rounds it the way the definition does.
// An empty bag has L = 0 and inv = 0: the result is the (zero) sum.
template <bool MEAN>
__device__ __forceinline__ float pooled(const float sum, const float L, const float inv) {
    if (!MEAN) return sum;
    const float q = sum * inv;
    return fmaf(fmaf(-q, L, sum), inv, q);
}

template <typename WT, int NC, int U, bool MEAN>
__device__ __forceinline__ void forward_bag(const WT* __restrict__ table, const int D, const int64_t R,
                                            const IdxView indices, const int64_t start, const int64_t end,
                                            void* __restrict__ out, const int out_io, const int64_t out_elem,
                                            int32_t* err) {
    constexpr int V = RowIO<WT>::kVec;
    using raw_t = typename RowIO<WT>::raw_t;
    const int lane = lane_id();
    const int nl = (D + V - 1) / V;  // lanes needed by one row
    const int LPR = nl >= kWave ? kWave : pow2ceil64(nl);
    const int G = kWave / LPR;
    const int sub = lane / LPR;
    const int lc = (lane & (LPR - 1)) * V;

    float acc[NC][V];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[c][v] = 0.f;

    for (int64_t base = start; base < end; base += kWave) {
        const int n = (int)((end - base) < (int64_t)kWave ? (end - base) : (int64_t)kWave);
        int32_t my = -1;
        if (lane < n) {
            const int64_t id = indices[base + lane];
            if (id >= 0 && id < R) my = (int32_t)id;
            else atomicOr(err, 1);
        }
        for (int k0 = 0; k0 < n; k0 += U * G) {
            raw_t x[U][NC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = k0 + u * G + sub;
                const int32_t got = __shfl(my, k & (kWave - 1), kWave);
                const int32_t id = (k < n) ? got : -1;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int col = lc + c * kWave * V;
                    x[u][c] = (id >= 0 && col < D) ? RowIO<WT>::load_raw(table + (int64_t)id * D + col)
                                                   : RowIO<WT>::zero_raw();
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < NC; ++c) RowIO<WT>::accumulate(x[u][c], acc[c]);
        }
    }
    // fold the groups
    for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[c][v] += __shfl_xor(acc[c][v], o, kWave);
    }
    float scale = 1.f, lenf = 0.f;
    if (MEAN) {
        const int64_t L = end - start;
        lenf = (float)L;
        scale = L > 0 ? 1.f / lenf : 0.f;
    }
    if (sub == 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int col = lc + c * kWave * V;
            if (col < D) {
#pragma unroll
                for (int v4 = 0; v4 < V; v4 += 4) {
                    store4_from_float(out, out_io, out_elem + col + v4, pooled<MEAN>(acc[c][v4], lenf, scale),
                                      pooled<MEAN>(acc[c][v4 + 1], lenf, scale), pooled<MEAN>(acc[c][v4 + 2], lenf, scale),
                                      pooled<MEAN>(acc[c][v4 + 3], lenf, scale));
                }
            }
        }
    }
}

// One kernel per NC so that the common narrow-row case (NC = 1) keeps its register count low enough for
// 8 wavefronts per SIMD; the host launches one per width class that has tables.  `tables_of_class` lists the
// tables this launch covers (those whose rows need more than 64 * (NC / 2) and at most 64 * NC lanes).
template <typename WT, int NC, int U, bool MEAN>
__global__ __launch_bounds__(kFwdThreads, NC == 1 ? 8 : 4) void forward_kernel(
    const WT* __restrict__ weights, const IdxView indices, const IdxView offsets,
    const int32_t* __restrict__ D_off, const int64_t* __restrict__ w_off, const int64_t* __restrict__ row_base,
    const int32_t* __restrict__ tables_of_class, const int32_t n_tables, const int32_t B, const int64_t nnz,
    const int32_t sumD, void* __restrict__ out, const int out_io, int32_t* err) {
    const int64_t q = (int64_t)blockIdx.x * (kFwdThreads / kWave) + (threadIdx.x >> 6);
    const int64_t i = q / B;
    if (i >= n_tables) return;
    const int32_t t = tables_of_class[i];
    const int32_t b = (int32_t)(q - i * B);
    const int64_t bag = (int64_t)t * B + b;
    const int32_t d0 = D_off[t];
    const int D = D_off[t + 1] - d0;
    const int64_t R = row_base[t + 1] - row_base[t];
    // clamped so that a malformed offsets array can never take a read outside indices[0, nnz)
    int64_t start = offsets[bag];
    int64_t end = offsets[bag + 1];
    start = start < 0 ? 0 : (start > nnz ? nnz : start);
    end = end < start ? start : (end > nnz ? nnz : end);
    forward_bag<WT, NC, U, MEAN>(weights + w_off[t], D, R, indices, start, end, out, out_io, (int64_t)b * sumD + d0, err);
}

// Narrow rows (at most 16 lanes per row): every lane group of the wavefront takes a bag of its own, G = 64 / LPR
// consecutive bags of one table per wavefront.  A bag of a dozen narrow rows is a few hundred bytes; with one
// wavefront per bag the step is bound by the latency of the offsets -> ids -> rows chain, not by bandwidth.
// A group reads LPR ids with one coalesced load, then walks them U rows at a time.
template <typename WT, int U, bool MEAN>
__global__ __launch_bounds__(kFwdThreads, 8) void forward_groups_kernel(
    const WT* __restrict__ weights, const IdxView indices, const IdxView offsets,
    const int32_t* __restrict__ D_off, const int64_t* __restrict__ w_off, const int64_t* __restrict__ row_base,
    const int32_t* __restrict__ tables_of_class, const int32_t n_tables, const int lpr_log2, const int32_t B,
    const int64_t nnz, const int32_t sumD, void* __restrict__ out, const int out_io, int32_t* err) {
    constexpr int V = RowIO<WT>::kVec;
    using raw_t = typename RowIO<WT>::raw_t;
    const int lane = lane_id();
    const int LPR = 1 << lpr_log2;
    const int G = kWave >> lpr_log2;
    const int64_t per_table = ((int64_t)B + G - 1) / G;   // wavefronts per table
    const int64_t wid = (int64_t)blockIdx.x * (kFwdThreads / kWave) + (threadIdx.x >> 6);
    const int64_t i = wid / per_table;
    if (i >= n_tables) return;
    const int32_t t = tables_of_class[i];
    const int sub = lane >> lpr_log2;
    const int li = lane & (LPR - 1);        // lane inside its group
    const int lc = li * V;
    const int64_t b = (wid - i * per_table) * G + sub;
    const bool has_bag = b < B;
    const int32_t d0 = D_off[t];
    const int D = D_off[t + 1] - d0;
    const int64_t R = row_base[t + 1] - row_base[t];
    const WT* table = weights + w_off[t];
    int64_t start = 0, end = 0;
    if (has_bag) {   // clamped so that a malformed offsets array can never take a read outside indices[0, nnz)
        const int64_t bag = (int64_t)t * B + b;
        start = offsets[bag];
        end = offsets[bag + 1];
        start = start < 0 ? 0 : (start > nnz ? nnz : start);
        end = end < start ? start : (end > nnz ? nnz : end);
    }
    const int full_len = (int)((end - start) < (int64_t)0x7FFFFFFF ? (end - start) : (int64_t)0x7FFFFFFF);
    // a bag far longer than its neighbours would keep the other groups of the wavefront waiting: such bags are left to
    // forward_long_bags_kernel, where a whole wavefront walks one bag
    const bool is_long = full_len > long_bag_min(LPR);
    const int len = is_long ? 0 : full_len;
    const int maxlen = wave_max_i32(len);   // longest bag of the wavefront: the loop bounds below are wave-uniform
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    const bool col_on = lc < D;
    for (int base = 0; base < maxlen; base += LPR) {
        int32_t my = -1;
        if (base + li < len) {
            const int64_t id = indices[start + base + li];
            if (id >= 0 && id < R) my = (int32_t)id;
            else atomicOr(err, 1);
        }
        const int nk = maxlen - base < LPR ? maxlen - base : LPR;
        for (int k0 = 0; k0 < nk; k0 += U) {
            raw_t x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // cross-lane read outside any lane-dependent condition; lanes of a finished bag read -1
                const int32_t id = __shfl(my, (sub << lpr_log2) + ((k0 + u) & (LPR - 1)), kWave);
                const bool on = (k0 + u) < nk && id >= 0 && col_on;
                x[u] = on ? RowIO<WT>::load_raw(table + (int64_t)id * D + lc) : RowIO<WT>::zero_raw();
            }
#pragma unroll
            for (int u = 0; u < U; ++u) RowIO<WT>::accumulate(x[u], acc);
        }
    }
    const float lenf = (float)len;
    float scale = 1.f;
    if (MEAN) scale = len > 0 ? 1.f / lenf : 0.f;
    if (has_bag && col_on && !is_long) {
        const int64_t out_elem = b * (int64_t)sumD + d0 + lc;
#pragma unroll
        for (int v4 = 0; v4 < V; v4 += 4)
            store4_from_float(out, out_io, out_elem + v4, pooled<MEAN>(acc[v4], lenf, scale),
                              pooled<MEAN>(acc[v4 + 1], lenf, scale), pooled<MEAN>(acc[v4 + 2], lenf, scale),
                              pooled<MEAN>(acc[v4 + 3], lenf, scale));
    }
}

// ---- the lane-group classes with the tables' hottest rows held in LDS --------------------------------------------
// In a skewed batch a hundred rows of a table take half of its lookups.  Their rows come from the L2, but every read
// that leaves a compute unit's vector L1 occupies one of its few dozen miss slots for the length of the trip, and it
// is those slots times the trip time that bound this kernel.  A workgroup of 16 wavefronts therefore takes a long run of
// consecutive bags of ONE table, copies the rows that the handle lists as the table's hottest (the rows that had the
// most lookups in the last backward call - a hint: any list of valid ids gives the same result) into LDS once, and
// serves every lookup of one of those rows from there.  A lookup finds out through a small open-addressing table of
// ids in LDS.  Per round of LPR ids a lane group first walks its cold ids (global loads, U rows in flight), then its
// hot ones (LDS reads); the two lists are compacted through an LDS stage, so that no lane issues a load it does not
// need.  The sum is taken in that order, which is fixed, so results do not depend on timing.
constexpr int kHotThreads = 1024;
constexpr int kHotWaves = kHotThreads / kWave;
constexpr int kHotTab = 1024;                // slots of the id table (at most kHotRows ids: a quarter full)
constexpr int kHotRowBytes = 64 << 10;       // LDS bytes for rows
constexpr int kHotPasses = 8;               // rounds of kHotWaves * G bags per workgroup
constexpr uint32_t kHotEmpty = 0xFFFFFFFFu;

__device__ __forceinline__ uint32_t hot_hash(const uint32_t id) { return (id * 0x9E3779B1u) >> 22; }   // 10 bits

template <typename WT, int U, bool MEAN>
__global__ __launch_bounds__(kHotThreads, 8) void forward_hot_kernel(
    const WT* __restrict__ weights, const IdxView indices, const IdxView offsets,
    const int32_t* __restrict__ D_off, const int64_t* __restrict__ w_off, const int64_t* __restrict__ row_base,
    const int32_t* __restrict__ tables_of_class, const int32_t n_tables, const int lpr_log2, const int32_t B,
    const int64_t nnz, const int32_t sumD, void* __restrict__ out, const int out_io, int32_t* err,
    const uint32_t* __restrict__ hot_ids, const uint32_t* __restrict__ hot_n, const int32_t chunks_per_table) {
    constexpr int V = RowIO<WT>::kVec;
    using raw_t = typename RowIO<WT>::raw_t;
    __shared__ raw_t s_rows[kHotRowBytes / 16];
    __shared__ uint32_t s_tab_id[kHotTab];
    __shared__ uint16_t s_tab_slot[kHotTab];
    __shared__ uint32_t s_cold[kHotWaves][kWave];
    __shared__ uint16_t s_hot[kHotWaves][kWave];
    const int lane = lane_id();
    const int wv = threadIdx.x >> 6;
    const int LPR = 1 << lpr_log2;
    const int G = kWave >> lpr_log2;
    const int32_t i = (int32_t)(blockIdx.x / (uint32_t)chunks_per_table);
    const int32_t chunk = (int32_t)(blockIdx.x - (uint32_t)i * (uint32_t)chunks_per_table);
    if (i >= n_tables) return;
    const int32_t t = tables_of_class[i];
    const int sub = lane >> lpr_log2;
    const int li = lane & (LPR - 1);        // lane inside its group
    const int lc = li * V;
    const int32_t d0 = D_off[t];
    const int D = D_off[t + 1] - d0;
    const int64_t R = row_base[t + 1] - row_base[t];
    const WT* table = weights + w_off[t];
    const bool col_on = lc < D;
    // ---- the table's hot rows: id table, then the rows themselves (one lane group per row)
    int nh = (int)hot_n[t];
    const int cap = (kHotRowBytes / 16) >> lpr_log2;
    nh = nh > kHotRows ? kHotRows : nh;
    nh = nh > cap ? cap : nh;
    for (int k = threadIdx.x; k < kHotTab; k += kHotThreads) s_tab_id[k] = kHotEmpty;
    __syncthreads();
    if ((int)threadIdx.x < nh) {
        const uint32_t id = hot_ids[(size_t)t * kHotRows + threadIdx.x];
        if ((int64_t)id < R) {
            uint32_t hsh = hot_hash(id);
            for (;;) {   // ends: the table is at most a quarter full
                const uint32_t old = atomicCAS(&s_tab_id[hsh], kHotEmpty, id);
                if (old == kHotEmpty) {
                    s_tab_slot[hsh] = (uint16_t)threadIdx.x;
                    break;
                }
                if (old == id) break;   // listed twice: the first entry serves
                hsh = (hsh + 1u) & (kHotTab - 1u);
            }
        }
    }
    for (int k = (int)(threadIdx.x >> lpr_log2); k < nh; k += kHotThreads >> lpr_log2) {
        const uint32_t id = hot_ids[(size_t)t * kHotRows + k];
        s_rows[(k << lpr_log2) + li] = ((int64_t)id < R && col_on) ? RowIO<WT>::load_raw(table + (int64_t)id * D + lc)
                                                                     : RowIO<WT>::zero_raw();
    }
    __syncthreads();
    // ---- the bags
    const uint32_t gmask = LPR >= 32 ? 0xFFFFFFFFu : ((1u << LPR) - 1u);   // (LPR <= 32 in these classes)
    const uint32_t below = (1u << li) - 1u;
    uint32_t* const cold = &s_cold[wv][sub << lpr_log2];
    uint16_t* const hot = &s_hot[wv][sub << lpr_log2];
    for (int pass = 0; pass < kHotPasses; ++pass) {
        const int64_t b = (((int64_t)chunk * kHotPasses + pass) * kHotWaves + wv) * G + sub;
        if ((((int64_t)chunk * kHotPasses + pass) * kHotWaves + wv) * G >= B) break;   // (the same for all lanes)
        const bool has_bag = b < B;
        int64_t start = 0, end = 0;
        if (has_bag) {   // clamped so that a malformed offsets array can never take a read outside indices[0, nnz)
            const int64_t bag = (int64_t)t * B + b;
            start = offsets[bag];
            end = offsets[bag + 1];
            start = start < 0 ? 0 : (start > nnz ? nnz : start);
            end = end < start ? start : (end > nnz ? nnz : end);
        }
        const int full_len = (int)((end - start) < (int64_t)0x7FFFFFFF ? (end - start) : (int64_t)0x7FFFFFFF);
        const bool is_long = full_len > long_bag_min(LPR);   // left to forward_long_bags_kernel
        const int len = is_long ? 0 : full_len;
        const int maxlen = wave_max_i32(len);
        float acc[V];
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = 0.f;
        for (int base = 0; base < maxlen; base += LPR) {
            int32_t my = -1;
            if (base + li < len) {
                const int64_t id = indices[start + base + li];
                if (id >= 0 && id < R) my = (int32_t)id;
                else atomicOr(err, 1);
            }
            int slot = -1;
            if (my >= 0 && nh > 0) {
                uint32_t hsh = hot_hash((uint32_t)my);
                for (;;) {
                    const uint32_t tid = s_tab_id[hsh];
                    if (tid == kHotEmpty) break;
                    if (tid == (uint32_t)my) {
                        slot = (int)s_tab_slot[hsh];
                        break;
                    }
                    hsh = (hsh + 1u) & (kHotTab - 1u);
                }
            }
            // this lane group's cold ids and hot slots, each list in bag order
            const bool is_cold = my >= 0 && slot < 0, is_hot = slot >= 0;
            const uint32_t mc = (uint32_t)(__ballot(is_cold) >> (sub << lpr_log2)) & gmask;
            const uint32_t mh = (uint32_t)(__ballot(is_hot) >> (sub << lpr_log2)) & gmask;
            if (is_cold) cold[__popc(mc & below)] = (uint32_t)my;
            if (is_hot) hot[__popc(mh & below)] = (uint16_t)slot;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            const int nc = __popc(mc), nhh = __popc(mh);
            const int ncmax = wave_max_i32(nc), nhmax = wave_max_i32(nhh);
            for (int k0 = 0; k0 < ncmax; k0 += U) {
                raw_t x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t id = cold[(k0 + u) & (LPR - 1)];
                    const bool on = (k0 + u) < nc && col_on;
                    x[u] = on ? RowIO<WT>::load_raw(table + (int64_t)id * D + lc) : RowIO<WT>::zero_raw();
                }
#pragma unroll
                for (int u = 0; u < U; ++u) RowIO<WT>::accumulate(x[u], acc);
            }
            for (int k0 = 0; k0 < nhmax; k0 += 4) {
                raw_t x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int sl = hot[(k0 + u) & (LPR - 1)];
                    const bool on = (k0 + u) < nhh;
                    x[u] = on ? s_rows[(sl << lpr_log2) + li] : RowIO<WT>::zero_raw();
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) RowIO<WT>::accumulate(x[u], acc);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the lists are free for the next round
        }
        const float lenf = (float)len;
        float scale = 1.f;
        if (MEAN) scale = len > 0 ? 1.f / lenf : 0.f;
        if (has_bag && col_on && !is_long) {
            const int64_t out_elem = b * (int64_t)sumD + d0 + lc;
#pragma unroll
            for (int v4 = 0; v4 < V; v4 += 4)
                store4_from_float(out, out_io, out_elem + v4, pooled<MEAN>(acc[v4], lenf, scale),
                                  pooled<MEAN>(acc[v4 + 1], lenf, scale), pooled<MEAN>(acc[v4 + 2], lenf, scale),
                                  pooled<MEAN>(acc[v4 + 3], lenf, scale));
        }
    }
}

// The long bags of the lane-group classes.  A wavefront looks at kLongScan x 64 consecutive bags of one table, 64 at
// a time with one bag per lane, and walks every bag with more than long_bag_min ids with all of its lanes
// (forward_bag, as for wide rows).  A kernel of its own: inside the lane-group kernel the second phase pushed the
// binary16 variant over its 64 registers (8.0 -> 9.3 ms at the largest workload).
constexpr int kLongScan = 4;
template <typename WT, bool MEAN>
__global__ __launch_bounds__(kFwdThreads, 4) void forward_long_bags_kernel(
    const WT* __restrict__ weights, const IdxView indices, const IdxView offsets,
    const int32_t* __restrict__ D_off, const int64_t* __restrict__ w_off, const int64_t* __restrict__ row_base,
    const int32_t* __restrict__ tables_of_class, const int32_t n_tables, const int32_t B, const int64_t nnz,
    const int32_t sumD, void* __restrict__ out, const int out_io, int32_t* err) {
    constexpr int V = RowIO<WT>::kVec;
    const int lane = lane_id();
    const int64_t per_table = ((int64_t)B + kLongScan * kWave - 1) / (kLongScan * kWave);   // wavefronts per table
    const int64_t wid = (int64_t)blockIdx.x * (kFwdThreads / kWave) + (threadIdx.x >> 6);
    const int64_t i = wid / per_table;
    if (i >= n_tables) return;
    const int32_t t = tables_of_class[i];
    const int32_t d0 = D_off[t];
    const int D = D_off[t + 1] - d0;
    // the bound of the table's class: lanes per row as the host classifies them (power of two, at least 4)
    const int nl = (D + V - 1) / V;
    const int bound = long_bag_min(nl > 16 ? 32 : (nl > 8 ? 16 : (nl > 4 ? 8 : 4)));
    for (int q = 0; q < kLongScan; ++q) {
        const int64_t b0 = ((wid - i * per_table) * kLongScan + q) * kWave;   // first bag of this round (wave-uniform)
        if (b0 >= B) break;
        const int64_t b = b0 + lane;
        int64_t start = 0, end = 0;
        if (b < B) {   // clamped as in the lane-group kernel
            const int64_t bag = (int64_t)t * B + b;
            start = offsets[bag];
            end = offsets[bag + 1];
            start = start < 0 ? 0 : (start > nnz ? nnz : start);
            end = end < start ? start : (end > nnz ? nnz : end);
        }
        uint64_t todo = __ballot(end - start > (int64_t)bound);
        while (todo != 0ull) {
            const int src = __ffsll((unsigned long long)todo) - 1;
            todo &= todo - 1ull;
            const int64_t s = (int64_t)(((uint64_t)bcast_lane((uint32_t)((uint64_t)start >> 32), src) << 32) |
                                        (uint64_t)bcast_lane((uint32_t)((uint64_t)start & 0xFFFFFFFFull), src));
            const int64_t e = (int64_t)(((uint64_t)bcast_lane((uint32_t)((uint64_t)end >> 32), src) << 32) |
                                        (uint64_t)bcast_lane((uint32_t)((uint64_t)end & 0xFFFFFFFFull), src));
            forward_bag<WT, 1, 4, MEAN>(weights + w_off[t], D, row_base[t + 1] - row_base[t], indices, s, e, out,
                                                out_io, (b0 + src) * (int64_t)sumD + d0, err);
        }
    }
}

template <typename WT, int NC, int U>
static void launch_forward_nc(const tbe_handle* h, int cls, const void* tables, const int32_t* d_D_off,
                              const IdxView indices, const IdxView offsets, int32_t B, int64_t nnz, bool mean, void* out,
                              int out_io, hipStream_t s) {
    const int n = h->fwd_count[cls];
    if (n == 0) return;
    const int32_t* list = h->d_fwd_tables + h->fwd_first[cls];
    const int wpb = kFwdThreads / kWave;
    const dim3 grid((unsigned)(((int64_t)n * B + wpb - 1) / wpb));
    const WT* w = static_cast<const WT*>(tables);
    if (mean)
        forward_kernel<WT, NC, U, true><<<grid, kFwdThreads, 0, s>>>(w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base,
                                                                     list, n, B, nnz, h->sumD, out, out_io, h->d_err);
    else
        forward_kernel<WT, NC, U, false><<<grid, kFwdThreads, 0, s>>>(w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base,
                                                                      list, n, B, nnz, h->sumD, out, out_io, h->d_err);
}

// the narrow-row classes: 32, 16, 8 and 4 lanes per row
template <typename WT>
static void launch_forward_groups(const tbe_handle* h, const void* tables, const int32_t* d_D_off, const IdxView indices,
                                  const IdxView offsets, int32_t B, int64_t nnz, bool mean, void* out, int out_io,
                                  hipStream_t s) {
    const WT* w = static_cast<const WT*>(tables);
    const int wpb = kFwdThreads / kWave;
    for (int c = 1; c < 5; ++c) {
        const int n = h->fwd_count[c];
        if (n == 0) continue;
        const int lpr_log2 = 6 - c;              // 32, 16, 8, 4 lanes per row
        const int G = kWave >> lpr_log2;
        const int64_t waves = (int64_t)n * (((int64_t)B + G - 1) / G);
        const dim3 grid((unsigned)((waves + wpb - 1) / wpb));
        const int32_t* list = h->d_fwd_tables + h->fwd_first[c];
        // with a hot-row list in the handle, and enough bags per table to fill a workgroup's rounds
        const int64_t bags_per_wg = (int64_t)kHotPasses * kHotWaves * G;
        const int cpt = (int)(((int64_t)B + bags_per_wg - 1) / bags_per_wg);
        if (h->d_hot_ids && h->hot_min_workgroups >= 0 && (int64_t)n * cpt >= h->hot_min_workgroups) {
            const dim3 hgrid((unsigned)((int64_t)n * cpt));
            if (mean)
                forward_hot_kernel<WT, 8, true><<<hgrid, kHotThreads, 0, s>>>(
                    w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base, list, n, lpr_log2, B, nnz, h->sumD, out, out_io,
                    h->d_err, h->d_hot_ids, h->d_hot_n, cpt);
            else
                forward_hot_kernel<WT, 8, false><<<hgrid, kHotThreads, 0, s>>>(
                    w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base, list, n, lpr_log2, B, nnz, h->sumD, out, out_io,
                    h->d_err, h->d_hot_ids, h->d_hot_n, cpt);
            continue;
        }
        if (mean)
            forward_groups_kernel<WT, 8, true><<<grid, kFwdThreads, 0, s>>>(
                w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base, list, n, lpr_log2, B, nnz, h->sumD, out, out_io, h->d_err);
        else
            forward_groups_kernel<WT, 8, false><<<grid, kFwdThreads, 0, s>>>(
                w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base, list, n, lpr_log2, B, nnz, h->sumD, out, out_io, h->d_err);
    }
    // the bags those launches left out (the four classes' tables follow one another in the list)
    const int n_all = h->fwd_count[1] + h->fwd_count[2] + h->fwd_count[3] + h->fwd_count[4];
    if (n_all > 0) {
        const int64_t waves = (int64_t)n_all * (((int64_t)B + kLongScan * kWave - 1) / (kLongScan * kWave));
        const dim3 grid((unsigned)((waves + wpb - 1) / wpb));
        const int32_t* list = h->d_fwd_tables + h->fwd_first[1];
        if (mean)
            forward_long_bags_kernel<WT, true><<<grid, kFwdThreads, 0, s>>>(
                w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base, list, n_all, B, nnz, h->sumD, out, out_io, h->d_err);
        else
            forward_long_bags_kernel<WT, false><<<grid, kFwdThreads, 0, s>>>(
                w, indices, offsets, d_D_off, h->d_w_off, h->d_row_base, list, n_all, B, nnz, h->sumD, out, out_io, h->d_err);
    }
}

hipError_t launch_forward(const tbe_handle* h, const void* tables, const int32_t* d_D_off, const void* indices_p,
                          const void* offsets_p, int idx32, int32_t B, int64_t nnz, tbe_pooling pooling, void* out,
                          int out_io, hipStream_t s) {
    const IdxView indices{indices_p, idx32}, offsets{offsets_p, idx32};
    const int64_t nbags = (int64_t)h->T * B;
    if (nbags == 0) return hipSuccess;
    LaunchTimer tm(h, s, "forward_pool");
    const bool mean = pooling == TBE_MEAN;
    if (h->dtype == TBE_F32) {
        launch_forward_nc<float, 1, 4>(h, 0, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
        launch_forward_nc<float, 2, 4>(h, 5, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
        launch_forward_nc<float, 4, 2>(h, 6, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
        launch_forward_groups<float>(h, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
    } else {
        launch_forward_nc<__half, 1, 4>(h, 0, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
        launch_forward_nc<__half, 2, 4>(h, 5, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
        launch_forward_groups<__half>(h, tables, d_D_off, indices, offsets, B, nnz, mean, out, out_io, s);
    }
    tm.done();
    return hipGetLastError();
}

// ---- non-pooled lookup -------------------------------------------------------------------------------------
// out block of table t = [n_t, D_t], row i = W_t[indices[offsets[t] + i]]; the blocks follow one another.
// A wavefront takes 64 consecutive positions: every lane resolves one lookup (table, source row, destination),
// then the 16-byte fragments of all 64 rows are copied lane-parallel, four in flight per lane.
__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)(v & 0xFFFFFFFFll), o, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)((uint64_t)v >> 32), o, kWave);
        v += (int64_t)(((uint64_t)hi << 32) | lo);
    }
    return v;
}

template <typename WT>
__device__ __forceinline__ void copy_fragment(const WT* __restrict__ src, void* __restrict__ out, const int out_io,
                                              const int64_t elem, const bool zero) {
    constexpr int V = RowIO<WT>::kVec;
    float x[V];
    if (zero) {
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = 0.f;
    } else {
        RowIO<WT>::load(src, x);
    }
#pragma unroll
    for (int v4 = 0; v4 < V; v4 += 4) store4_from_float(out, out_io, elem + v4, x[v4], x[v4 + 1], x[v4 + 2], x[v4 + 3]);
}

template <typename WT>
__global__ __launch_bounds__(kFwdThreads, 8) void lookup_seq_kernel(
    const WT* __restrict__ weights, const IdxView indices, const IdxView offsets, const int32_t* __restrict__ D_off,
    const int64_t* __restrict__ w_off, const int64_t* __restrict__ row_base, const int T, const int64_t nnz,
    void* __restrict__ out, const int out_io, const int64_t out_elems, int32_t* err) {
    constexpr int V = RowIO<WT>::kVec;
    const int lane = lane_id();
    const int64_t p0 = ((int64_t)blockIdx.x * (kFwdThreads / kWave) + (threadIdx.x >> 6)) * kWave;
    if (p0 >= nnz) return;
    const int64_t p = p0 + lane;
    const bool valid = p < nnz;
    // table of the position: the last t with offsets[t] <= p (empty tables are skipped by construction)
    int t = 0;
    {
        const int64_t q = valid ? p : p0;
        int lo = 0, hi = T;  // invariant: offsets[lo] <= q, answer in [lo, hi)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (offsets[mid] <= q) lo = mid;
            else hi = mid;
        }
        t = lo;
    }
    // element offset of the table's block: sum over earlier tables of n_t' * D_t'
    const int t0 = __shfl(t, 0, kWave);
    int64_t part = 0;
    for (int tt = lane; tt < t0; tt += kWave) {
        const int64_t n = offsets[tt + 1] - offsets[tt];
        part += (n > 0 ? n : 0) * (int64_t)(D_off[tt + 1] - D_off[tt]);
    }
    int64_t base = wave_sum_i64(part);
    for (int tt = t0; tt < t; ++tt) {
        const int64_t n = offsets[tt + 1] - offsets[tt];
        base += (n > 0 ? n : 0) * (int64_t)(D_off[tt + 1] - D_off[tt]);
    }
    const int D = D_off[t + 1] - D_off[t];
    int64_t id = valid ? indices[p] : 0;
    const int64_t R = row_base[t + 1] - row_base[t];
    bool bad = false;
    if (valid && (id < 0 || id >= R)) {
        atomicOr(err, 1);   // as in the pooled forward: flagged, and the row reads as zeros
        bad = true;
        id = 0;
    }
    const int64_t src_elem = w_off[t] + id * D;
    int64_t dst_elem = base + (p - offsets[t]) * D;
    // a malformed offsets array (not ascending from 0 to nnz) must never take a store outside out[0, out_elems)
    if (valid && (dst_elem < 0 || dst_elem + D > out_elems)) {
        atomicOr(err, 1);
        dst_elem = -1;
    }
    const int n = (int)((nnz - p0) < (int64_t)kWave ? (nnz - p0) : (int64_t)kWave);
    const int F = D / V;  // fragments per row
    const bool uniform = __all(!valid || D == __shfl(D, 0, kWave));
    if (uniform) {
        const int F0 = __shfl(F, 0, kWave);
        const int total = n * F0;
        for (int q0 = 0; q0 < total; q0 += 4 * kWave) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + u * kWave + lane;
                const int k = q / F0, f = q - k * F0;
                const int ks = k < n ? k : 0;
                const uint32_t s_lo = __shfl((uint32_t)(src_elem & 0xFFFFFFFFll), ks, kWave);
                const uint32_t s_hi = __shfl((uint32_t)((uint64_t)src_elem >> 32), ks, kWave);
                const uint32_t d_lo = __shfl((uint32_t)(dst_elem & 0xFFFFFFFFll), ks, kWave);
                const uint32_t d_hi = __shfl((uint32_t)((uint64_t)dst_elem >> 32), ks, kWave);
                const int zb = __shfl((int)bad, ks, kWave);
                const int64_t d0 = (int64_t)(((uint64_t)d_hi << 32) | d_lo);
                if (q < total && d0 >= 0) {
                    const int64_t se = (int64_t)(((uint64_t)s_hi << 32) | s_lo) + (int64_t)f * V;
                    copy_fragment<WT>(weights + se, out, out_io, d0 + (int64_t)f * V, zb != 0);
                }
            }
        }
    } else {  // a table boundary inside the 64 positions: row by row
        for (int k = 0; k < n; ++k) {
            const uint32_t s_lo = __shfl((uint32_t)(src_elem & 0xFFFFFFFFll), k, kWave);
            const uint32_t s_hi = __shfl((uint32_t)((uint64_t)src_elem >> 32), k, kWave);
            const uint32_t d_lo = __shfl((uint32_t)(dst_elem & 0xFFFFFFFFll), k, kWave);
            const uint32_t d_hi = __shfl((uint32_t)((uint64_t)dst_elem >> 32), k, kWave);
            const int zb = __shfl((int)bad, k, kWave);
            const int Fk = __shfl(F, k, kWave);
            const int64_t d0 = (int64_t)(((uint64_t)d_hi << 32) | d_lo);
            for (int f = lane; f < Fk && d0 >= 0; f += kWave) {
                const int64_t se = (int64_t)(((uint64_t)s_hi << 32) | s_lo) + (int64_t)f * V;
                copy_fragment<WT>(weights + se, out, out_io, d0 + (int64_t)f * V, zb != 0);
            }
        }
    }
}

hipError_t launch_lookup_seq(const tbe_handle* h, const void* tables, const void* indices_p, const void* offsets_p,
                             int idx32, int64_t nnz, void* out, int out_io, int64_t out_elems, hipStream_t s) {
    if (nnz == 0) return hipSuccess;
    const IdxView indices{indices_p, idx32}, offsets{offsets_p, idx32};
    const int64_t per_block = (int64_t)(kFwdThreads / kWave) * kWave;
    const dim3 grid((unsigned)((nnz + per_block - 1) / per_block));
    LaunchTimer tm(h, s, "lookup_seq");
    if (h->dtype == TBE_F32)
        lookup_seq_kernel<float><<<grid, kFwdThreads, 0, s>>>(static_cast<const float*>(tables), indices, offsets, h->d_D_off,
                                                              h->d_w_off, h->d_row_base, h->T, nnz, out, out_io, out_elems, h->d_err);
    else
        lookup_seq_kernel<__half><<<grid, kFwdThreads, 0, s>>>(static_cast<const __half*>(tables), indices, offsets,
                                                               h->d_D_off, h->d_w_off, h->d_row_base, h->T, nnz, out, out_io,
                                                               out_elems, h->d_err);
    tm.done();
    return hipGetLastError();
}

}  // namespace tbe
