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
#include "tbe_device.cuh"
#include "tbe_internal.h"

namespace tbe {

constexpr int kSegThreads = 256;
constexpr int kSegBlocks = 2048;  // persistent grid: waves stride over blocks of 64 unique rows
#ifndef TBE_SEG_U
#define TBE_SEG_U 4
#endif
constexpr int kSegUnroll = TBE_SEG_U;

struct RowGeom {
    int D, LPR, G, sub, lc;
};

__device__ __forceinline__ RowGeom row_geom(int D) {
    RowGeom g;
    const int lane = lane_id();
    const int nl = (D + 3) >> 2;
    g.D = D;
    g.LPR = nl >= kWave ? kWave : pow2ceil64(nl);
    g.G = kWave / g.LPR;
    g.sub = lane / g.LPR;
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
    const uint32_t* counters;     // [0]=U, [1]=n_long, [2]=n_chunks
    const uint32_t* bag_sorted;   // linear bag id of every sorted position
    const int64_t* offsets;
    const float* grad_out;
    const int32_t* D_off;
    const int64_t* row_base;
    const int64_t* w_off;
    int32_t T, B, sumD, maxD;
    uint32_t total_rows;
    float lr, eps, inv_c;
    void* tables;
    float* state;
    uint32_t* long_list;   // [cap_long][3]  (u, slot, nchunks)
    uint32_t* chunk_desc;  // [cap_chunks][2] (u, k)
    float* partial;        // [cap_chunks][maxD]
    uint32_t cap_long, cap_chunks;
};

template <bool MEAN>
__device__ __forceinline__ float bag_scale(const int64_t* __restrict__ offsets, uint32_t bag) {
    if (!MEAN) return 1.f;
    const int64_t L = offsets[(int64_t)bag + 1] - offsets[bag];
    return L > 0 ? 1.f / (float)L : 0.f;
}

// Whole-wavefront reduction of sorted positions [s, e) of ONE row:
// acc += sum of scale(bag) * grad_out[b, d0 + col .. col+3]; the groups take interleaved positions and
// fold_groups() completes the sum.  NC = 256-column chunks per row.
template <int NC, bool MEAN>
__device__ __forceinline__ void segment_reduce(float (&acc)[NC][4], const RowGeom& g, const float* __restrict__ gcol,
                                               const int64_t sumD, const int64_t bag0,
                                               const uint32_t* __restrict__ bag_sorted,
                                               const int64_t* __restrict__ offsets, const uint32_t s, const uint32_t e) {
    const int lane = lane_id();
    for (uint32_t base = s; base < e; base += kWave) {
        const int n = (int)((e - base) < (uint32_t)kWave ? (e - base) : (uint32_t)kWave);
        int32_t my_b = 0;
        float my_s = 1.f;
        if (lane < n) {
            const uint32_t bag = bag_sorted[base + lane];
            my_b = (int32_t)((int64_t)bag - bag0);
            my_s = bag_scale<MEAN>(offsets, bag);
        }
        for (int k0 = 0; k0 < n; k0 += kSegUnroll * g.G) {
            float4 x[kSegUnroll][NC];
            float sc[kSegUnroll];
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u) {
                const int k = k0 + u * g.G + g.sub;
                const int32_t b = __shfl(my_b, k & (kWave - 1), kWave);
                sc[u] = MEAN ? __shfl(my_s, k & (kWave - 1), kWave) : 1.f;
                const bool on = k < n;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int col = g.lc + c * kWave * 4;
                    x[u][c] = (on && col < g.D) ? *reinterpret_cast<const float4*>(gcol + (int64_t)b * sumD + col)
                                                : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if (MEAN) {
                        acc[c][0] = fmaf(sc[u], x[u][c].x, acc[c][0]);
                        acc[c][1] = fmaf(sc[u], x[u][c].y, acc[c][1]);
                        acc[c][2] = fmaf(sc[u], x[u][c].z, acc[c][2]);
                        acc[c][3] = fmaf(sc[u], x[u][c].w, acc[c][3]);
                    } else {
                        acc[c][0] += x[u][c].x;
                        acc[c][1] += x[u][c].y;
                        acc[c][2] += x[u][c].z;
                        acc[c][3] += x[u][c].w;
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
            for (int v = 0; v < 4; ++v) acc[c][v] += __shfl_xor(acc[c][v], o, kWave);
    }
}

// The optimizer step for one row.  acc holds the complete row gradient in the LPR lanes that `on`
// marks (all groups after fold_groups, or each group its own row).  v_old is the row's moment.
//   v <- v + ||g||^2 ;  w <- w - lr / (sqrt(v / c) + eps) * g      (updated v; v stored unscaled)
// Lanes with write == true store their 4 columns; the lane with lc == 0 among them stores the moment.
template <typename WT, int NC>
__device__ __forceinline__ void adagrad_row(const float (&acc)[NC][4], const RowGeom& g, WT* __restrict__ wrow,
                                            float* __restrict__ vptr, const float v_old, const bool write,
                                            const float lr, const float eps, const float inv_c) {
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int col = g.lc + c * kWave * 4;
        if (col < g.D) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sq = fmaf(acc[c][v], acc[c][v], sq);
        }
    }
    for (int o = 1; o < g.LPR; o <<= 1) sq += __shfl_xor(sq, o, kWave);  // within the LPR lanes that cover the row
    const float v_new = v_old + sq;
    const float denom = sqrtf(v_new * inv_c) + eps;
    const float step = v_new > 0.f ? lr / denom : 0.f;  // v_new == 0 means g == 0: nothing to apply
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
        if (g.lc == 0) *vptr = v_new;
    }
}

// ---- 1. find the long rows and give each of their chunks a slot in the partial buffer ------------
__global__ __launch_bounds__(256) void seg_schedule_kernel(const SegArgs a, uint32_t* __restrict__ counters) {
    const uint32_t U = counters[0];
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t u = blockIdx.x * blockDim.x + threadIdx.x; u < U; u += stride) {
        const uint32_t len = a.seg_start[u + 1] - a.seg_start[u];
        if (len > (uint32_t)kSegChunk && a.keys_unique[u] < a.total_rows) {
            const uint32_t nch = (len + kSegChunk - 1) / kSegChunk;
            const uint32_t li = atomicAdd(&counters[1], 1u);
            const uint32_t slot = atomicAdd(&counters[2], nch);
            if (li < a.cap_long && slot + nch <= a.cap_chunks) {  // always true by construction of the capacities
                a.long_list[3 * li + 0] = u;
                a.long_list[3 * li + 1] = slot;
                a.long_list[3 * li + 2] = nch;
                for (uint32_t k = 0; k < nch; ++k) {
                    a.chunk_desc[2 * (slot + k) + 0] = u;
                    a.chunk_desc[2 * (slot + k) + 1] = k;
                }
            }
        }
    }
}

// ---- 2. one wavefront per chunk of a long row: partial[slot] = sum of the chunk's gradient slices --
template <int NC, bool MEAN>
__global__ __launch_bounds__(kSegThreads, NC == 1 ? 8 : 4) void seg_long_partial_kernel(const SegArgs a) {
    const uint32_t nchunks = a.counters[2] < a.cap_chunks ? a.counters[2] : a.cap_chunks;
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    for (uint32_t w = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); w < nchunks; w += nwaves) {
        const uint32_t u = a.chunk_desc[2 * w + 0];
        const uint32_t k = a.chunk_desc[2 * w + 1];
        const uint32_t key = a.keys_unique[u];
        const int t = table_of_key(a.row_base, a.T, key);
        const int d0 = a.D_off[t];
        const RowGeom g = row_geom(a.D_off[t + 1] - d0);
        const uint32_t s = a.seg_start[u] + k * kSegChunk;
        const uint32_t e_row = a.seg_start[u + 1];
        const uint32_t e = (s + kSegChunk < e_row) ? s + kSegChunk : e_row;
        float* dst = a.partial + (size_t)w * a.maxD;
        float acc[NC][4];
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        segment_reduce<NC, MEAN>(acc, g, a.grad_out + d0, a.sumD, (int64_t)t * a.B, a.bag_sorted, a.offsets, s, e);
        fold_groups<NC>(acc, g);
        if (g.sub == 0) {
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int col = g.lc + c * kWave * 4;
                if (col < g.D) *reinterpret_cast<float4*>(dst + col) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
            }
        }
    }
}

// ---- 3a. rows with at most kSegChunk lookups, all tables at most 256 columns wide ------------------
template <typename WT, bool MEAN>
__global__ __launch_bounds__(kSegThreads, 8) void seg_update_kernel(const SegArgs a) {
    const int lane = lane_id();
    const uint32_t U = a.counters[0];
    const uint32_t nblk = (U + kWave - 1) / kWave;
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    WT* tables = static_cast<WT*>(a.tables);
    for (uint32_t blk = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); blk < nblk; blk += nwaves) {
        // ---- one row per lane: bounds, key, table, width, moment
        const uint32_t u = blk * kWave + lane;
        uint32_t s = 0, e = 0, key = 0;
        if (u < U) {
            s = a.seg_start[u];
            e = a.seg_start[u + 1];
            key = a.keys_unique[u];
        }
        const uint32_t len = e - s;
        const bool live = (u < U) && len >= 1 && len <= (uint32_t)kSegChunk && key < a.total_rows;
        int t = 0, D = 4;
        float v = 0.f;
        if (live) {
            t = table_of_key(a.row_base, a.T, key);
            D = a.D_off[t + 1] - a.D_off[t];
            v = a.state[key];
        }
        int r = 0;
        while (r < kWave) {
            if (!__shfl((int)live, r, kWave)) {
                ++r;
                continue;
            }
            const RowGeom g = row_geom(__shfl(D, r, kWave));
            const uint32_t s_r = __shfl(s, r, kWave);
            const uint32_t len_r = __shfl(len, r, kWave);
            if (len_r > (uint32_t)kWave) {
                // ---- medium row: the whole wavefront reduces it
                const uint32_t key_r = __shfl(key, r, kWave);
                const int t_r = __shfl(t, r, kWave);
                const float v_r = __shfl(v, r, kWave);
                float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
                segment_reduce<1, MEAN>(acc, g, a.grad_out + a.D_off[t_r], a.sumD, (int64_t)t_r * a.B, a.bag_sorted,
                                        a.offsets, s_r, s_r + len_r);
                fold_groups<1>(acc, g);
                WT* wrow = tables + a.w_off[t_r] + ((int64_t)key_r - a.row_base[t_r]) * g.D;
                adagrad_row<WT, 1>(acc, g, wrow, a.state + key_r, v_r, g.sub == 0, a.lr, a.eps, a.inv_c);
                ++r;
                continue;
            }
            // ---- short rows: rows r .. r+k-1 share the width of row r and have at most 64 lookups in total
            const bool q = live && D == g.D && lane >= r && lane < r + g.G && (e - s_r) <= (uint32_t)kWave;
            const uint64_t m = __ballot(q) >> r;                       // bit j: row r+j qualifies
            const int k = (~m == 0ull) ? kWave : (__ffsll((unsigned long long)(~m)) - 1);  // trailing ones, >= 1
            const uint32_t tot = __shfl(e, r + k - 1, kWave) - s_r;   // lookups of the k rows, <= 64
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
            const float* gcol = a.grad_out + a.D_off[gt] + g.lc;
            const int64_t bag0 = (int64_t)gt * a.B;
            WT* wrow = tables + a.w_off[gt] + ((int64_t)gkey - a.row_base[gt]) * g.D;
            uint32_t lmax = glen;  // longest row of the round (wave-uniform loop bound)
            for (int o = g.LPR; o < kWave; o <<= 1) {
                const uint32_t other = __shfl_xor(lmax, o, kWave);
                lmax = other > lmax ? other : lmax;
            }
            float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
            for (uint32_t q0 = 0; q0 < lmax; q0 += kSegUnroll) {
                float4 x[kSegUnroll];
                float sc[kSegUnroll];
#pragma unroll
                for (int uu = 0; uu < kSegUnroll; ++uu) {
                    const uint32_t qi = q0 + uu;
                    const int src = (goff + (int)qi) & (kWave - 1);
                    const uint32_t bag = __shfl(my_bag, src, kWave);
                    sc[uu] = MEAN ? __shfl(my_s, src, kWave) : 1.f;
                    const bool on = qi < glen && col_on;
                    x[uu] = on ? *reinterpret_cast<const float4*>(gcol + ((int64_t)bag - bag0) * a.sumD)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int uu = 0; uu < kSegUnroll; ++uu) {
                    if (MEAN) {
                        acc[0][0] = fmaf(sc[uu], x[uu].x, acc[0][0]);
                        acc[0][1] = fmaf(sc[uu], x[uu].y, acc[0][1]);
                        acc[0][2] = fmaf(sc[uu], x[uu].z, acc[0][2]);
                        acc[0][3] = fmaf(sc[uu], x[uu].w, acc[0][3]);
                    } else {
                        acc[0][0] += x[uu].x;
                        acc[0][1] += x[uu].y;
                        acc[0][2] += x[uu].z;
                        acc[0][3] += x[uu].w;
                    }
                }
            }
            adagrad_row<WT, 1>(acc, g, wrow, a.state + gkey, gv, gon, a.lr, a.eps, a.inv_c);
            r += k;
        }
    }
}

// ---- 3b. same rows, any width up to 1024 columns: one wavefront per row ----------------------------
template <typename WT, bool MEAN>
__global__ __launch_bounds__(kSegThreads, 4) void seg_update_wide_kernel(const SegArgs a) {
    const uint32_t U = a.counters[0];
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    WT* tables = static_cast<WT*>(a.tables);
    for (uint32_t u = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); u < U; u += nwaves) {
        const uint32_t s = a.seg_start[u];
        const uint32_t e = a.seg_start[u + 1];
        const uint32_t key = a.keys_unique[u];
        if (e - s > (uint32_t)kSegChunk || key >= a.total_rows) continue;  // long rows: kernel 4; invalid ids: no row
        const int t = table_of_key(a.row_base, a.T, key);
        const int d0 = a.D_off[t];
        const RowGeom g = row_geom(a.D_off[t + 1] - d0);
        WT* wrow = tables + a.w_off[t] + ((int64_t)key - a.row_base[t]) * g.D;
        float acc[4][4];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        segment_reduce<4, MEAN>(acc, g, a.grad_out + d0, a.sumD, (int64_t)t * a.B, a.bag_sorted, a.offsets, s, e);
        fold_groups<4>(acc, g);
        adagrad_row<WT, 4>(acc, g, wrow, a.state + key, a.state[key], g.sub == 0, a.lr, a.eps, a.inv_c);
    }
}

// ---- 4. one wavefront per long row: add its chunks' partial sums in chunk order, then step --------
template <typename WT>
__global__ __launch_bounds__(kSegThreads) void seg_long_update_kernel(const SegArgs a) {
    const uint32_t nlong = a.counters[1] < a.cap_long ? a.counters[1] : a.cap_long;
    const uint32_t nwaves = gridDim.x * (kSegThreads / kWave);
    WT* tables = static_cast<WT*>(a.tables);
    for (uint32_t li = blockIdx.x * (kSegThreads / kWave) + (threadIdx.x >> 6); li < nlong; li += nwaves) {
        const uint32_t u = a.long_list[3 * li + 0];
        const uint32_t slot = a.long_list[3 * li + 1];
        const uint32_t nch = a.long_list[3 * li + 2];
        const uint32_t key = a.keys_unique[u];
        const int t = table_of_key(a.row_base, a.T, key);
        const int D = a.D_off[t + 1] - a.D_off[t];
        // here all 64 lanes cover the row (or a 256-column part of it); groups are not used
        RowGeom g;
        g.D = D; g.LPR = kWave; g.G = 1; g.sub = 0; g.lc = lane_id() * 4;
        WT* wrow = tables + a.w_off[t] + ((int64_t)key - a.row_base[t]) * D;
        float acc[4][4];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        for (uint32_t k = 0; k < nch; ++k) {
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
        adagrad_row<WT, 4>(acc, g, wrow, a.state + key, a.state[key], true, a.lr, a.eps, a.inv_c);
    }
}

hipError_t launch_segment_update(const tbe_handle* h, const Workspace& w, char* ws, int spare, const float* grad_out,
                                 const int64_t* offsets, int32_t B, tbe_pooling pooling, float lr, float eps, float c,
                                 void* tables, float* state, hipStream_t s) {
    SegArgs a;
    a.keys_unique = reinterpret_cast<const uint32_t*>(ws + w.vals[spare]);
    a.seg_start = reinterpret_cast<const uint32_t*>(ws + w.seg_start);
    uint32_t* counters = reinterpret_cast<uint32_t*>(ws + w.counters);
    a.counters = counters;
    a.bag_sorted = reinterpret_cast<const uint32_t*>(ws + w.keys[spare]);
    a.offsets = offsets;
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
    a.chunk_desc = reinterpret_cast<uint32_t*>(ws + w.chunk_desc);
    a.partial = reinterpret_cast<float*>(ws + w.partial);
    a.cap_long = (uint32_t)w.cap_long;
    a.cap_chunks = (uint32_t)w.cap_chunks;
    const bool mean = pooling == TBE_MEAN;
    const bool f32 = h->dtype == TBE_F32;
    const bool narrow = h->maxD <= 256;
    {
        LaunchTimer tm(h, s, "seg_schedule");
        seg_schedule_kernel<<<512, 256, 0, s>>>(a, counters);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_long_partial");
        if (narrow) {
            if (mean) seg_long_partial_kernel<1, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            else seg_long_partial_kernel<1, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        } else {
            if (mean) seg_long_partial_kernel<4, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            else seg_long_partial_kernel<4, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        }
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_update");
        if (narrow) {
            if (f32) {
                if (mean) seg_update_kernel<float, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
                else seg_update_kernel<float, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            } else {
                if (mean) seg_update_kernel<__half, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
                else seg_update_kernel<__half, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            }
        } else {
            if (f32) {
                if (mean) seg_update_wide_kernel<float, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
                else seg_update_wide_kernel<float, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            } else {
                if (mean) seg_update_wide_kernel<__half, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
                else seg_update_wide_kernel<__half, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            }
        }
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_long_update");
        if (f32) seg_long_update_kernel<float><<<256, kSegThreads, 0, s>>>(a);
        else seg_long_update_kernel<__half><<<256, kSegThreads, 0, s>>>(a);
        tm.done();
    }
    return hipGetLastError();
}

}  // namespace tbe
