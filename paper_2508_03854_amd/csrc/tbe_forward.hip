// Forward: pooled lookup, one wavefront per bag.
//
// A bag's rows are D_t * sizeof(weight) contiguous bytes each (128 B .. 1 KB for the shapes of interest),
// so a 64-lane wavefront would waste most lanes on one row.  The wavefront is therefore split into
// G = 64 / LPR groups of LPR lanes, LPR = D_t / kVec lanes covering one row with one 16-byte load per
// lane; the groups walk the bag in an interleaved fashion, four rows per group in flight, and a
// butterfly over the groups folds the partial sums at the end.  The bag's ids are read with one
// coalesced 64-wide load and handed to the groups with cross-lane reads.
#include "tbe_device.cuh"
#include "tbe_internal.h"

namespace tbe {

constexpr int kFwdThreads = 256;
#ifndef TBE_FWD_U
#define TBE_FWD_U 4
#endif
#ifndef TBE_FWD_WAVES
#define TBE_FWD_WAVES 8
#endif

// NC = number of 64-lane column chunks a row needs (1 when D <= 64 * kVec); U = rows in flight per group.
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
    float scale = 1.f;
    if (MEAN) {
        const int64_t L = end - start;
        scale = L > 0 ? 1.f / (float)L : 0.f;
    }
    if (sub == 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int col = lc + c * kWave * V;
            if (col < D) {
#pragma unroll
                for (int v4 = 0; v4 < V; v4 += 4) {
                    store4_from_float(out, out_io, out_elem + col + v4, acc[c][v4] * scale, acc[c][v4 + 1] * scale,
                                      acc[c][v4 + 2] * scale, acc[c][v4 + 3] * scale);
                }
            }
        }
    }
}

// One kernel per NC so that the common narrow-row case (NC = 1) keeps its register count low enough for
// 8 wavefronts per SIMD; the host picks the kernel from the widest table of the handle.
template <typename WT, int NC, int U, bool MEAN>
__global__ __launch_bounds__(kFwdThreads, NC == 1 ? TBE_FWD_WAVES : 4) void forward_kernel(
    const WT* __restrict__ weights, const IdxView indices, const IdxView offsets,
    const int32_t* __restrict__ D_off, const int64_t* __restrict__ w_off, const int64_t* __restrict__ row_base,
    const int32_t B, const int64_t nbags, const int64_t nnz, const int32_t sumD, void* __restrict__ out,
    const int out_io, int32_t* err) {
    const int64_t bag = (int64_t)blockIdx.x * (kFwdThreads / kWave) + (threadIdx.x >> 6);
    if (bag >= nbags) return;
    const int32_t t = (int32_t)(bag / B);
    const int32_t b = (int32_t)(bag - (int64_t)t * B);
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

template <typename WT, int NC, int U>
static void launch_forward_nc(const tbe_handle* h, const void* tables, const int32_t* d_D_off, const IdxView indices,
                              const IdxView offsets, int32_t B, int64_t nbags, int64_t nnz, bool mean, void* out,
                              int out_io, dim3 grid, hipStream_t s) {
    const WT* w = static_cast<const WT*>(tables);
    if (mean)
        forward_kernel<WT, NC, U, true><<<grid, kFwdThreads, 0, s>>>(w, indices, offsets, d_D_off, h->d_w_off,
                                                                     h->d_row_base, B, nbags, nnz, h->sumD, out, out_io, h->d_err);
    else
        forward_kernel<WT, NC, U, false><<<grid, kFwdThreads, 0, s>>>(w, indices, offsets, d_D_off, h->d_w_off,
                                                                      h->d_row_base, B, nbags, nnz, h->sumD, out, out_io, h->d_err);
}

hipError_t launch_forward(const tbe_handle* h, const void* tables, const int32_t* d_D_off, const void* indices_p,
                          const void* offsets_p, int idx32, int32_t B, int64_t nnz, tbe_pooling pooling, void* out,
                          int out_io, hipStream_t s) {
    const IdxView indices{indices_p, idx32}, offsets{offsets_p, idx32};
    const int64_t nbags = (int64_t)h->T * B;
    if (nbags == 0) return hipSuccess;
    const int wpb = kFwdThreads / kWave;
    const dim3 grid((unsigned)((nbags + wpb - 1) / wpb));
    LaunchTimer tm(h, s, "forward_pool");
    const bool mean = pooling == TBE_MEAN;
    if (h->dtype == TBE_F32) {
        if (h->maxD <= 256) launch_forward_nc<float, 1, TBE_FWD_U>(h, tables, d_D_off, indices, offsets, B, nbags, nnz, mean, out, out_io, grid, s);
        else if (h->maxD <= 512) launch_forward_nc<float, 2, 4>(h, tables, d_D_off, indices, offsets, B, nbags, nnz, mean, out, out_io, grid, s);
        else launch_forward_nc<float, 4, 2>(h, tables, d_D_off, indices, offsets, B, nbags, nnz, mean, out, out_io, grid, s);
    } else {
        if (h->maxD <= 512) launch_forward_nc<__half, 1, TBE_FWD_U>(h, tables, d_D_off, indices, offsets, B, nbags, nnz, mean, out, out_io, grid, s);
        else launch_forward_nc<__half, 2, 4>(h, tables, d_D_off, indices, offsets, B, nbags, nnz, mean, out, out_io, grid, s);
    }
    tm.done();
    return hipGetLastError();
}

}  // namespace tbe
