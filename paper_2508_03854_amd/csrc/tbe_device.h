// Device-side helpers for gfx950 (64-lane wavefronts).
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbe {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() {
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

__device__ __forceinline__ uint64_t lanemask_lt() { return (1ull << lane_id()) - 1ull; }

// smallest power of two >= x, for 1 <= x <= 64
__device__ __forceinline__ int pow2ceil64(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Inclusive prefix sum across the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    const int l = lane_id();
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        uint32_t n = __shfl_up(v, o, kWave);
        if (l >= o) v += n;
    }
    return v;
}

// Exclusive prefix sum across a block of NT threads (NT multiple of 64). smem: NT/64 words.
// Returns the exclusive prefix of this thread; *total is the block sum (same in every thread).
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* smem, uint32_t* total) {
    const int l = lane_id();
    const int w = threadIdx.x >> 6;
    const uint32_t inc = wave_incl_scan(v);
    if (l == kWave - 1) smem[w] = inc;
    __syncthreads();
    uint32_t wbase = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NT / kWave; ++i) {
        const uint32_t s = smem[i];
        if (i < w) wbase += s;
        tot += s;
    }
    __syncthreads();  // smem may be reused by the caller after this
    *total = tot;
    return wbase + inc - v;
}

// ---- streaming (non-temporal) 16-byte accesses: data that is used once should not displace what a cache is kept for
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load16(const void* p) {
    const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store16(void* p, const uint4 v) {
    u32x4_t x;
    x.x = v.x; x.y = v.y; x.z = v.z; x.w = v.w;
    __builtin_nontemporal_store(x, static_cast<u32x4_t*>(p));
}

// ---- ids and offsets: int64 or int32 at the boundary --------------------------------------------------
struct IdxView {
    const void* p;
    int is32;
    __device__ __forceinline__ int64_t operator[](int64_t i) const {
        return is32 ? (int64_t)static_cast<const int32_t*>(p)[i] : static_cast<const int64_t*>(p)[i];
    }
};

// ---- pooled output / upstream gradient element types: float, IEEE binary16, bfloat16 ---------------------
struct bf16_t { unsigned short bits; };  // bfloat16 = the upper half of a binary32

__device__ __forceinline__ float bf16_to_float(unsigned short b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ unsigned short float_to_bf16_rn(float x) {  // round to nearest even; NaN stays NaN
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (unsigned short)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// Four consecutive elements of the upstream gradient.  A fragment stays in its raw form between the load
// and its use, so that several loads can be in flight before the first conversion needs its data.
template <typename GT>
struct GradIO;
template <>
struct GradIO<float> {
    using raw_t = float4;
    static __device__ __forceinline__ raw_t load(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ raw_t zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ float4 to_float(const raw_t& r) { return r; }
};
template <>
struct GradIO<__half> {
    using raw_t = uint2;
    static __device__ __forceinline__ raw_t load(const __half* p) { return *reinterpret_cast<const uint2*>(p); }
    static __device__ __forceinline__ raw_t zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ float4 to_float(const raw_t& r) {
        return make_float4(__half2float(__ushort_as_half((unsigned short)(r.x & 0xFFFFu))),
                           __half2float(__ushort_as_half((unsigned short)(r.x >> 16))),
                           __half2float(__ushort_as_half((unsigned short)(r.y & 0xFFFFu))),
                           __half2float(__ushort_as_half((unsigned short)(r.y >> 16))));
    }
};
template <>
struct GradIO<bf16_t> {
    using raw_t = uint2;
    static __device__ __forceinline__ raw_t load(const bf16_t* p) { return *reinterpret_cast<const uint2*>(p); }
    static __device__ __forceinline__ raw_t zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ float4 to_float(const raw_t& r) {
        return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                           __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
    }
};

// store four consecutive elements; io = 0 float, 1 binary16, 2 bfloat16 (one rounding to nearest even)
__device__ __forceinline__ void store4_from_float(void* base, int io, int64_t elem, float a, float b, float c, float d) {
    if (io == 0) {
        *reinterpret_cast<float4*>(static_cast<float*>(base) + elem) = make_float4(a, b, c, d);
    } else {
        unsigned short h0, h1, h2, h3;
        if (io == 1) {
            h0 = __half_as_ushort(__float2half_rn(a)); h1 = __half_as_ushort(__float2half_rn(b));
            h2 = __half_as_ushort(__float2half_rn(c)); h3 = __half_as_ushort(__float2half_rn(d));
        } else {
            h0 = float_to_bf16_rn(a); h1 = float_to_bf16_rn(b); h2 = float_to_bf16_rn(c); h3 = float_to_bf16_rn(d);
        }
        *reinterpret_cast<uint2*>(static_cast<unsigned short*>(base) + elem) =
            make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
    }
}

// ---- 16-byte row fragments ---------------------------------------------------------------------
// RowIO<WT>::kVec elements of a table row travel in one 16-byte load.
// Sum over the aligned group of LPR lanes (a power of two up to 64) that a lane belongs to, in every lane of the group.
// Groups of up to 16 lanes lie inside one 16-lane row, where the data-parallel-primitive lane patterns exchange
// values without a trip through the LDS crossbar: neighbours, pairs of a quad, the mirrored half row, the mirrored
// row; only the steps across rows (16, 32) take the general shuffle.  All 64 lanes must be active.  The order of the
// additions is fixed, so the result does not depend on timing.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(const float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// x[lane] + x[lane ^ O] for O = 16 or 32, the same bits in both partners: the gfx950 row-swap instructions exchange
// the odd and even 16-lane rows (or the two 32-lane halves) of two registers in place, again without the LDS crossbar
// (lane layout checked on the device: result 0 keeps the lower partner's value, result 1 the upper partner's).
template <int O>
__device__ __forceinline__ float pair_sum(const float x) {
    const unsigned u = __float_as_uint(x);
    if (O == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
}
__device__ __forceinline__ float group_sum(float x, const int LPR) {
    if (LPR >= 2) x += dpp_lane<0xB1>(x);     // quad_perm [1,0,3,2]
    if (LPR >= 4) x += dpp_lane<0x4E>(x);     // quad_perm [2,3,0,1]
    if (LPR >= 8) x += dpp_lane<0x141>(x);    // row_half_mirror: lane i <- lane 7-i of its half row
    if (LPR >= 16) x += dpp_lane<0x140>(x);   // row_mirror: lane i <- lane 15-i of its row
    if (LPR >= 32) x = pair_sum<16>(x);
    if (LPR >= 64) x = pair_sum<32>(x);
    return x;
}

// Maximum over the wavefront, as a wavefront-uniform value: inside the 16-lane rows by DPP lane patterns, across
// the four rows by scalar lane reads.  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ int dpp_lane_i32(const int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ int wave_max_i32(int x) {
    int o = dpp_lane_i32<0xB1>(x);  x = o > x ? o : x;    // quad_perm [1,0,3,2]
    o = dpp_lane_i32<0x4E>(x);      x = o > x ? o : x;    // quad_perm [2,3,0,1]
    o = dpp_lane_i32<0x141>(x);     x = o > x ? o : x;    // row_half_mirror
    o = dpp_lane_i32<0x140>(x);     x = o > x ? o : x;    // row_mirror: every lane holds its row's maximum
    const int a = __builtin_amdgcn_readlane(x, 0), b = __builtin_amdgcn_readlane(x, 16);
    const int c = __builtin_amdgcn_readlane(x, 32), d = __builtin_amdgcn_readlane(x, 48);
    const int ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

// The value a given lane holds, for all lanes, when that lane is the same for the whole wavefront: a scalar read
// (the result is wavefront-uniform, so what is computed from it stays on the scalar unit) instead of a trip through
// the LDS crossbar.
__device__ __forceinline__ int bcast_lane(const int x, const int src) { return __builtin_amdgcn_readlane(x, src); }
__device__ __forceinline__ uint32_t bcast_lane(const uint32_t x, const int src) {
    return (uint32_t)__builtin_amdgcn_readlane((int)x, src);
}
__device__ __forceinline__ float bcast_lane(const float x, const int src) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src));
}

template <typename WT>
struct RowIO;

template <>
struct RowIO<float> {
    static constexpr int kVec = 4;
    using raw_t = float4;  // a fragment as it sits in registers between the load and its use
    static __device__ __forceinline__ raw_t load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ raw_t zero_raw() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ void accumulate(const raw_t& r, float (&acc)[4]) {
        acc[0] += r.x; acc[1] += r.y; acc[2] += r.z; acc[3] += r.w;
    }
    static __device__ __forceinline__ void load(const float* p, float (&x)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    // 4-element fragment used by the optimizer step (one lane owns 4 columns)
    static __device__ __forceinline__ void load4(const float* p, float (&x)[4]) { load(p, x); }
    static __device__ __forceinline__ void store4(float* p, const float (&x)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    }
};

template <>
struct RowIO<__half> {
    static constexpr int kVec = 8;
    using raw_t = uint4;
    static __device__ __forceinline__ raw_t load_raw(const __half* p) { return *reinterpret_cast<const uint4*>(p); }
    static __device__ __forceinline__ raw_t zero_raw() { return make_uint4(0u, 0u, 0u, 0u); }
    // acc += float(half): the mixed-precision FMA reads the binary16 operand straight from one half of the 32-bit
    // register (x * 1.0 + acc, one rounding, the same value as convert-then-add), one instruction instead of two.
    // The forward is bound by vector-ALU issue at 16-bit rows, so this is its inner loop's main cost.
    static __device__ __forceinline__ void accumulate(const raw_t& r, float (&acc)[8]) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel_hi:[1,0,0]" : "+v"(acc[2 * i]) : "v"(w[i]));
            asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc[2 * i + 1]) : "v"(w[i]));
        }
    }
    static __device__ __forceinline__ void load(const __half* p, float (&x)[8]) {
        const uint4 raw = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xFFFFu)));
            x[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
        }
    }
    static __device__ __forceinline__ void load4(const __half* p, float (&x)[4]) {
        const uint2 raw = *reinterpret_cast<const uint2*>(p);
        x[0] = __half2float(__ushort_as_half((unsigned short)(raw.x & 0xFFFFu)));
        x[1] = __half2float(__ushort_as_half((unsigned short)(raw.x >> 16)));
        x[2] = __half2float(__ushort_as_half((unsigned short)(raw.y & 0xFFFFu)));
        x[3] = __half2float(__ushort_as_half((unsigned short)(raw.y >> 16)));
    }
    // one rounding, to nearest even, from the fp32 result to the stored binary16
    static __device__ __forceinline__ void store4(__half* p, const float (&x)[4]) {
        uint2 raw;
        raw.x = (uint32_t)__half_as_ushort(__float2half_rn(x[0])) | ((uint32_t)__half_as_ushort(__float2half_rn(x[1])) << 16);
        raw.y = (uint32_t)__half_as_ushort(__float2half_rn(x[2])) | ((uint32_t)__half_as_ushort(__float2half_rn(x[3])) << 16);
        *reinterpret_cast<uint2*>(p) = raw;
    }
};

}  // namespace tbe
