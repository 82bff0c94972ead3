// Floating-point half of the backward pass: per unique row, sum the upstream gradient slices of the
// row's segment and apply one moment-scaled row-wise AdaGrad step in place (Algorithm 1, steps 5-6).
//
// One wavefront owns one unique row, so every row and every moment has exactly one writer and the
// result does not depend on scheduling.  A row of D floats is covered by LPR = D/4 lanes (one float4
// each); the 64/LPR groups of the wavefront walk the segment interleaved, four gradient slices per
// group in flight, and a butterfly folds the groups.  Rows with more than kSegChunk lookups (the head
// of the Zipf distribution) are cut into chunks that are reduced by separate wavefronts into a partial
// buffer and then combined, in chunk order, by the row's single owner.
#include "tbe_device.cuh"
#include "tbe_internal.h"

namespace tbe {

constexpr int kSegThreads = 256;
constexpr int kSegBlocks = 2048;  // persistent grid: waves stride over the unique rows
constexpr int kSegUnroll = 4;

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

// acc += sum over sorted positions [s, e) of  scale(bag) * grad_out[b, d0 + col .. col+3]; every group of
// the wavefront accumulates a different subset, fold_groups() completes the sum.
template <int NC, bool MEAN>
__device__ __forceinline__ void segment_reduce(float (&acc)[NC][4], const RowGeom& g, const float* __restrict__ gcol,
                                               const int64_t sumD, const int64_t bag0,
                                               const uint32_t* __restrict__ vals_sorted,
                                               const uint32_t* __restrict__ bag_of_pos,
                                               const int64_t* __restrict__ offsets, const uint32_t s, const uint32_t e) {
    const int lane = lane_id();
    for (uint32_t base = s; base < e; base += kWave) {
        const int n = (int)((e - base) < (uint32_t)kWave ? (e - base) : (uint32_t)kWave);
        int32_t my_b = 0;
        float my_s = 1.f;
        if (lane < n) {
            const uint32_t p = vals_sorted[base + lane];
            const int64_t bag = (int64_t)bag_of_pos[p];
            my_b = (int32_t)(bag - bag0);
            if (MEAN) {
                const int64_t L = offsets[bag + 1] - offsets[bag];
                my_s = L > 0 ? 1.f / (float)L : 0.f;
            }
        }
        for (int k0 = 0; k0 < n; k0 += kSegUnroll * g.G) {
            float x[kSegUnroll][NC][4];
            float sc[kSegUnroll];
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u) {
                const int k = k0 + u * g.G + g.sub;
                const int32_t b = __shfl(my_b, k & (kWave - 1), kWave);
                sc[u] = MEAN ? __shfl(my_s, k & (kWave - 1), kWave) : 1.f;
                const bool on = k < n;
                if (!on) sc[u] = 0.f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int col = g.lc + c * kWave * 4;
                    if (on && col < g.D) {
                        const float4 v = *reinterpret_cast<const float4*>(gcol + (int64_t)b * sumD + col);
                        x[u][c][0] = v.x; x[u][c][1] = v.y; x[u][c][2] = v.z; x[u][c][3] = v.w;
                    } else {
                        x[u][c][0] = x[u][c][1] = x[u][c][2] = x[u][c][3] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u)
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[c][v] = MEAN ? fmaf(sc[u], x[u][c][v], acc[c][v]) : acc[c][v] + x[u][c][v];
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

// The optimizer step for one row; acc holds the complete row gradient in every group of the wavefront.
//   v <- v + ||g||^2 ;  w <- w - lr / (sqrt(v / c) + eps) * g      (updated v; v stored unscaled)
template <typename WT, int NC>
__device__ __forceinline__ void adagrad_row(const float (&acc)[NC][4], const RowGeom& g, WT* __restrict__ wrow,
                                            float* __restrict__ vptr, const float lr, const float eps,
                                            const float inv_c) {
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
    const float v_new = *vptr + sq;
    const float denom = sqrtf(v_new * inv_c) + eps;
    const float step = v_new > 0.f ? lr / denom : 0.f;  // v_new == 0 means g == 0: nothing to apply
    if (g.sub == 0) {
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
    }
    if (lane_id() == 0) *vptr = v_new;
}

struct SegArgs {
    const uint32_t* keys_unique;   // unique_rows
    const uint32_t* seg_start;
    const uint32_t* counters;      // [0]=U, [1]=n_long, [2]=n_chunks
    const uint32_t* vals_sorted;
    const uint32_t* bag_of_pos;
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
template <bool MEAN>
__global__ __launch_bounds__(kSegThreads) void seg_long_partial_kernel(const SegArgs a) {
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
        const float* gcol = a.grad_out + d0;
        const int64_t bag0 = (int64_t)t * a.B;
        float* dst = a.partial + (size_t)w * a.maxD;
        if (g.D <= 256) {
            float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
            segment_reduce<1, MEAN>(acc, g, gcol, a.sumD, bag0, a.vals_sorted, a.bag_of_pos, a.offsets, s, e);
            fold_groups<1>(acc, g);
            if (g.sub == 0 && g.lc < g.D) *reinterpret_cast<float4*>(dst + g.lc) = make_float4(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
        } else {
            float acc[4][4];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
            segment_reduce<4, MEAN>(acc, g, gcol, a.sumD, bag0, a.vals_sorted, a.bag_of_pos, a.offsets, s, e);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int col = g.lc + c * 256;
                if (col < g.D) *reinterpret_cast<float4*>(dst + col) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
            }
        }
    }
}

// ---- 3. one wavefront per unique row with at most kSegChunk lookups: reduce + step ----------------
template <typename WT, bool MEAN>
__global__ __launch_bounds__(kSegThreads) void seg_update_kernel(const SegArgs a) {
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
        const float* gcol = a.grad_out + d0;
        const int64_t bag0 = (int64_t)t * a.B;
        WT* wrow = tables + a.w_off[t] + ((int64_t)key - a.row_base[t]) * g.D;
        if (g.D <= 256) {
            float acc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
            segment_reduce<1, MEAN>(acc, g, gcol, a.sumD, bag0, a.vals_sorted, a.bag_of_pos, a.offsets, s, e);
            fold_groups<1>(acc, g);
            adagrad_row<WT, 1>(acc, g, wrow, a.state + key, a.lr, a.eps, a.inv_c);
        } else {
            float acc[4][4];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
            segment_reduce<4, MEAN>(acc, g, gcol, a.sumD, bag0, a.vals_sorted, a.bag_of_pos, a.offsets, s, e);
            adagrad_row<WT, 4>(acc, g, wrow, a.state + key, a.lr, a.eps, a.inv_c);
        }
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
        adagrad_row<WT, 4>(acc, g, wrow, a.state + key, a.lr, a.eps, a.inv_c);
    }
}

hipError_t launch_segment_update(const tbe_handle* h, const Workspace& w, char* ws, const uint32_t* keys_sorted,
                                 const uint32_t* vals_sorted, const float* grad_out, const int64_t* offsets, int32_t B,
                                 int64_t N, tbe_pooling pooling, float lr, float eps, float c, void* tables, float* state,
                                 hipStream_t s) {
    (void)keys_sorted;
    (void)N;
    SegArgs a;
    a.keys_unique = reinterpret_cast<const uint32_t*>(ws + w.unique_rows);
    a.seg_start = reinterpret_cast<const uint32_t*>(ws + w.seg_start);
    uint32_t* counters = reinterpret_cast<uint32_t*>(ws + w.counters);
    a.counters = counters;
    a.vals_sorted = vals_sorted;
    a.bag_of_pos = reinterpret_cast<const uint32_t*>(ws + w.bag_of_pos);
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
    {
        LaunchTimer tm(h, s, "seg_schedule");
        seg_schedule_kernel<<<512, 256, 0, s>>>(a, counters);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_long_partial");
        if (mean) seg_long_partial_kernel<true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        else seg_long_partial_kernel<false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "seg_update");
        if (f32) {
            if (mean) seg_update_kernel<float, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            else seg_update_kernel<float, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
        } else {
            if (mean) seg_update_kernel<__half, true><<<kSegBlocks, kSegThreads, 0, s>>>(a);
            else seg_update_kernel<__half, false><<<kSegBlocks, kSegThreads, 0, s>>>(a);
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
