// Measurement aids: kernels of known traffic.  Not steps of the method.
//   - a streaming copy (what the memory system delivers for the friendliest pattern, and the kernel that the
//     hardware byte counters of a profile are scaled by);
//   - a gather of fixed-size slices from pseudo-random places of a window of chosen size, optionally written back
//     (what it delivers for the access pattern of the embedding kernels: one row or one gradient slice per lookup,
//     from a working set that does or does not fit a cache level).
#include "tbe_device.h"
#include "tbe_internal.h"

namespace tbe {

// four 16-byte loads in flight per lane, streaming (non-temporal) loads and stores
__global__ __launch_bounds__(256) void calibration_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                               const size_t n) {
    constexpr size_t kU = 4;
    const size_t span = (size_t)gridDim.x * blockDim.x * kU;
    for (size_t base = (size_t)blockIdx.x * blockDim.x * kU + threadIdx.x; base < n; base += span) {
        uint4 x[kU];
#pragma unroll
        for (size_t u = 0; u < kU; ++u) {
            const size_t i = base + u * blockDim.x;
            if (i < n) x[u] = nt_load16(src + i);
        }
#pragma unroll
        for (size_t u = 0; u < kU; ++u) {
            const size_t i = base + u * blockDim.x;
            if (i < n) nt_store16(dst + i, x[u]);
        }
    }
}

// A bijection of [0, 2^k), k <= 32: odd multiplications modulo 2^k and right xor-shifts are each invertible, so
// `count` consecutive inputs (count <= 2^k) give `count` distinct, scattered outputs.
__device__ __forceinline__ uint32_t scatter_bits(uint32_t x, const int k) {
    const uint32_t mask = (k >= 32) ? 0xFFFFFFFFu : ((1u << k) - 1u);
    const int s1 = k / 2 > 0 ? k / 2 : 1, s2 = k / 3 > 0 ? k / 3 : 1;
    x &= mask;
    x = (x * 0x9E3779B1u) & mask;
    x ^= x >> s1;
    x = (x * 0x85EBCA6Bu) & mask;
    x ^= x >> s2;
    x = (x * 0xC2B2AE35u) & mask;
    x ^= x >> s1;
    return x;
}

// LPR = 16-byte fragments per slice (lanes per slice).  Workgroup id mod 8 = XCD x; XCD x draws the slices
// i = x, x+8, ... (its eighth of the `gathers`) from window x (per_xcd) or window 0.  A wavefront takes 64 slices
// at a time: every lane works out the place of one of them, then the lane groups fetch them, kU per group in flight.
template <int LPR, bool RMW>
__global__ __launch_bounds__(256, 8) void calibration_gather_kernel(uint4* __restrict__ buf, const uint64_t window_frags,
                                                                    const int per_xcd, const int log2_slices,
                                                                    const uint64_t gathers, uint32_t* __restrict__ sink) {
    constexpr int G = kWave / LPR;        // lane groups per wavefront
    constexpr int kU = G >= 8 ? 8 : 4;    // slices in flight per lane group
    const int lane = lane_id();
    const int sub = lane / LPR, frag = lane % LPR;
    const uint32_t xcd = blockIdx.x & 7u;
    const uint64_t per = (gathers + 7u - xcd) / 8u;   // slices of this XCD
    const uint64_t waves_in_xcd = (uint64_t)(gridDim.x / 8u) * (blockDim.x / kWave);
    const uint64_t my_wave = (uint64_t)(blockIdx.x / 8u) * (blockDim.x / kWave) + (threadIdx.x >> 6);
    uint4* win = buf + (per_xcd ? (uint64_t)xcd * window_frags : 0ull);
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (uint64_t j0 = my_wave * kWave; j0 < per; j0 += waves_in_xcd * kWave) {
        const uint64_t j = j0 + (uint64_t)lane;                       // this lane's slice
        // a shared window: read-only gathers of every XCD range over the whole window (each starts elsewhere in the
        // sequence); written-back ones are numbered globally, so that no two land on one slice
        const uint32_t place = scatter_bits((uint32_t)(per_xcd ? j : (RMW ? j * 8u + xcd : j + xcd * 0x9E3779u)), log2_slices);
        const int n = per - j0 < (uint64_t)kWave ? (int)(per - j0) : kWave;
        for (int k0 = 0; k0 < n; k0 += kU * G) {
            uint4 x[kU];
            uint4* p[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int k = k0 + u * G + sub;
                p[u] = win + (uint64_t)__shfl(place, k & (kWave - 1), kWave) * LPR + frag;
                x[u] = k < n ? *p[u] : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                if (RMW) {
                    if (k0 + u * G + sub < n) *p[u] = make_uint4(x[u].x + 1u, x[u].y, x[u].z, x[u].w);
                } else {
                    acc.x ^= x[u].x; acc.y ^= x[u].y; acc.z ^= x[u].z; acc.w ^= x[u].w;
                }
            }
        }
    }
    if (!RMW) {   // keeps the loads alive; one word per lane
        const uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
        sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = v;
    }
}

constexpr unsigned kGatherGrid = 256u * 8u;   // every compute unit filled once at 8 wavefronts per SIMD

template <int LPR>
static void launch_gather(bool rmw, uint4* buf, uint64_t window_frags, int per_xcd, int log2_slices, uint64_t gathers,
                          uint32_t* sink, hipStream_t s) {
    if (rmw) calibration_gather_kernel<LPR, true><<<kGatherGrid, 256, 0, s>>>(buf, window_frags, per_xcd, log2_slices, gathers, sink);
    else calibration_gather_kernel<LPR, false><<<kGatherGrid, 256, 0, s>>>(buf, window_frags, per_xcd, log2_slices, gathers, sink);
}

}  // namespace tbe

using namespace tbe;

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" {

tbe_status tbe_calibration_copy(tbe_handle* h, void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!h || !dst || !src || (bytes & 15) != 0 || !aligned16(dst) || !aligned16(src)) return TBE_EINVAL;
    if (bytes == 0) return TBE_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    LaunchTimer tm(h, s, "calibration_copy");
    calibration_copy_kernel<<<256 * 8, 256, 0, s>>>(static_cast<uint4*>(dst), static_cast<const uint4*>(src), bytes / 16);
    tm.done();
    return hipGetLastError() == hipSuccess ? TBE_OK : TBE_EHIP;
}

tbe_status tbe_calibration_gather(tbe_handle* h, void* buf, size_t buf_bytes, size_t window_bytes, int32_t per_xcd,
                                  int32_t slice_bytes, int64_t gathers, int32_t write_back, void* sink,
                                  size_t sink_bytes, void* hip_stream) {
    if (!h || !buf || !sink || !aligned16(buf) || !aligned16(sink) || gathers < 0) return TBE_EINVAL;
    if (slice_bytes < 16 || slice_bytes > 1024 || (slice_bytes & (slice_bytes - 1)) != 0) return TBE_ESHAPE;
    if (window_bytes < (size_t)slice_bytes || (window_bytes & (window_bytes - 1)) != 0) return TBE_ESHAPE;
    if (buf_bytes < window_bytes * (per_xcd ? 8u : 1u)) return TBE_ESHAPE;
    if (sink_bytes < (size_t)kGatherGrid * 256u * 4u) return TBE_ESHAPE;
    const uint64_t slices = window_bytes / (size_t)slice_bytes;
    // written-back slices must be distinct (two lane groups on one slice would race): the place of slice i is a
    // bijection of i, so at most `slices` of them per window
    if (write_back && (per_xcd ? ((uint64_t)gathers + 7u) / 8u : (uint64_t)gathers) > slices) return TBE_ESHAPE;
    if (slices > (1ull << 32) || (uint64_t)gathers > (1ull << 32)) return TBE_ESHAPE;   // places are 32-bit
    if (gathers == 0) return TBE_OK;
    int log2_slices = 0;
    while ((1ull << log2_slices) < slices) ++log2_slices;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    uint4* b = static_cast<uint4*>(buf);
    uint32_t* k = static_cast<uint32_t*>(sink);
    const uint64_t wf = window_bytes / 16u;
    LaunchTimer tm(h, s, "calibration_gather");
    switch (slice_bytes / 16) {
        case 1: launch_gather<1>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
        case 2: launch_gather<2>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
        case 4: launch_gather<4>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
        case 8: launch_gather<8>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
        case 16: launch_gather<16>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
        case 32: launch_gather<32>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
        default: launch_gather<64>(write_back != 0, b, wf, per_xcd, log2_slices, (uint64_t)gathers, k, s); break;
    }
    tm.done();
    return hipGetLastError() == hipSuccess ? TBE_OK : TBE_EHIP;
}

}  // extern "C"
