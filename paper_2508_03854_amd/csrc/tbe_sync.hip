// Replica synchronisation of Algorithm 1 (weight sync and moment sync) for replicas that live on ONE device:
// every replica's buffer is replaced by the element-wise mean over the replicas.  Across devices this step is
// an all-reduce; that is outside this library.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "tbe_device.h"
#include "tbe_internal.h"

namespace tbe {

__device__ __forceinline__ float elem_to_float(float x) { return x; }
__device__ __forceinline__ float elem_to_float(__half x) { return __half2float(x); }
__device__ __forceinline__ void elem_from_float(float* p, float x) { *p = x; }
__device__ __forceinline__ void elem_from_float(__half* p, float x) { *p = __float2half_rn(x); }

struct ReplicaPtrs {
    void* p[kMaxReplicas];
};

// 16 bytes per thread and iteration: the sum runs over the replicas in index order, in fp32, and is divided by M
// (a true division, so the result is the correctly rounded quotient of the fp32 sum).
template <typename WT>
__global__ __launch_bounds__(256) void replica_mean_kernel(const ReplicaPtrs r, const int M, const size_t nvec,
                                                           const size_t count) {
    constexpr int V = RowIO<WT>::kVec;
    const float fm = (float)M;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        float sum[V];
#pragma unroll
        for (int v = 0; v < V; ++v) sum[v] = 0.f;
        for (int m = 0; m < M; ++m) {
            float x[V];
            RowIO<WT>::load(static_cast<const WT*>(r.p[m]) + i * V, x);
#pragma unroll
            for (int v = 0; v < V; ++v) sum[v] += x[v];
        }
#pragma unroll
        for (int v = 0; v < V; ++v) sum[v] /= fm;
        for (int m = 0; m < M; ++m) {
            WT* dst = static_cast<WT*>(r.p[m]) + i * V;
#pragma unroll
            for (int v4 = 0; v4 < V; v4 += 4) {
                const float q[4] = {sum[v4], sum[v4 + 1], sum[v4 + 2], sum[v4 + 3]};
                RowIO<WT>::store4(dst + v4, q);
            }
        }
    }
    // the last count % V elements, one thread each
    const size_t tail0 = nvec * V;
    if (blockIdx.x == 0 && tail0 + threadIdx.x < count) {
        const size_t e = tail0 + threadIdx.x;
        float s = 0.f;
        for (int m = 0; m < M; ++m) s += elem_to_float(static_cast<const WT*>(r.p[m])[e]);
        s /= fm;
        for (int m = 0; m < M; ++m) elem_from_float(static_cast<WT*>(r.p[m]) + e, s);
    }
}

hipError_t launch_replica_mean(const tbe_handle* h, void* const* replicas, int M, size_t count, bool f32, hipStream_t s) {
    ReplicaPtrs r;
    for (int m = 0; m < kMaxReplicas; ++m) r.p[m] = m < M ? replicas[m] : nullptr;
    LaunchTimer tm(h, s, "replica_mean");
    if (f32) {
        const size_t nvec = count / RowIO<float>::kVec;
        replica_mean_kernel<float><<<256 * 8, 256, 0, s>>>(r, M, nvec, count);
    } else {
        const size_t nvec = count / RowIO<__half>::kVec;
        replica_mean_kernel<__half><<<256 * 8, 256, 0, s>>>(r, M, nvec, count);
    }
    tm.done();
    return hipGetLastError();
}

}  // namespace tbe
