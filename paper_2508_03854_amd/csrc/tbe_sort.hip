// Integer half of the backward pass: linearise ids into row keys, stable LSD radix sort of (key, payload) with the
// lookup's bag id (pooled calls) or position (non-pooled calls) as payload, run-length segmentation into unique rows.  Everything here is exact integer work.
#include "tbe_device.h"
#include "tbe_internal.h"

namespace tbe {

// =================================================================================================
// linearize: key[p] = row_base[t(p)] + indices[p] (or the table-local id alone when the sort is segmented),
// bag_of_pos[p] = linear bag id of p, the payload a pooled call sorts along with the key
// =================================================================================================
constexpr int kLinThreads = 256;

// first i in [lo, hi] with a[i] > x   (caller guarantees a[hi] > x)
__device__ __forceinline__ int64_t upper_bound_i64(const IdxView a, int64_t lo, int64_t hi, int64_t x) {
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] > x) hi = mid;
        else lo = mid + 1;
    }
    return lo;
}

// The same search by a whole wavefront: 64 probes per round cut the range 64-fold, so 8 M offsets take 4 dependent
// loads instead of 23.  Every lane returns the result.  Terminates for any contents of a (the range shrinks every
// round) and never reads outside [lo, hi).
__device__ __forceinline__ int64_t wave_upper_bound_i64(const IdxView a, int64_t lo, int64_t hi, const int64_t x) {
    const int lane = lane_id();
    while (lo < hi) {
        const int64_t step = (hi - lo + kWave - 1) / kWave;
        const int64_t i = lo + (int64_t)(lane + 1) * step - 1;   // lane's probe; the last lane's is >= hi - 1
        const bool gt = i < hi ? (a[i] > x) : true;
        const uint64_t m = __ballot(gt);                         // (a probe beyond hi counts as greater)
        if (m == 0ull) return hi;                                // all of [lo, hi) is <= x
        const int f = __ffsll((unsigned long long)m) - 1;        // first probe above x
        const int64_t i_f = lo + (int64_t)(f + 1) * step - 1;
        lo += (int64_t)f * step;                                 // the probe before it was <= x
        hi = i_f < hi ? i_f : hi;
    }
    return lo;
}

// A block owns kLinTile consecutive positions.  It finds the bags that own its first and last position
// with two binary searches in the global offsets and stages that offsets segment in LDS (relative to the
// tile start).  Every bag that starts inside the tile then marks its first position, and a running maximum
// over the positions gives each position the last bag that starts at or before it, i.e. its owner (empty bags
// start where the next one does and lose against it).
__global__ __launch_bounds__(kLinThreads) void linearize_kernel(const IdxView indices, const IdxView offsets,
                                                                const int64_t nbags, const int32_t B,
                                                                const int64_t* __restrict__ row_base,
                                                                const uint32_t invalid_key, const bool local_keys,
                                                                const int64_t N, uint32_t* __restrict__ keys,
                                                                uint32_t* __restrict__ bag_of_pos, int32_t* err) {
    constexpr int kItems = kLinTile / kLinThreads;   // positions per thread: kItems rows of 64 per wavefront
    __shared__ int32_t s_off[kLinTile + 2];
    __shared__ int32_t s_own[kLinTile];
    __shared__ int32_t s_wmax[kLinThreads / kWave];
    __shared__ int64_t s_lo, s_hi;
    const int64_t p0 = (int64_t)blockIdx.x * kLinTile;
    const int64_t p1 = (p0 + kLinTile < N) ? p0 + kLinTile : N;
    if (p0 >= N) return;
    // owner of p: the bag with offsets[bag] <= p < offsets[bag+1]  ==  (first i with offsets[i] > p) - 1.
    // Searching i in [0, nbags] and clamping keeps every later access in range even for malformed offsets.
    // Wavefront 0 searches for the tile's first position, wavefront 1 for its last.
    if ((threadIdx.x >> 6) < 2) {
        const bool first = (threadIdx.x >> 6) == 0;
        const int64_t r = wave_upper_bound_i64(offsets, 0, nbags, first ? p0 : p1 - 1) - 1;
        if ((threadIdx.x & (kWave - 1)) == 0) *(first ? &s_lo : &s_hi) = r;
    }
    for (int i = threadIdx.x; i < kLinTile; i += kLinThreads) s_own[i] = 0;
    __syncthreads();
    int64_t lo = s_lo, hi = s_hi;
    lo = lo < 0 ? 0 : (lo > nbags - 1 ? nbags - 1 : lo);
    hi = hi < lo ? lo : (hi > nbags - 1 ? nbags - 1 : hi);
    const int64_t nb = hi - lo + 1;             // bags touched by this tile (>= 1)
    const bool staged = nb + 1 <= kLinTile + 2;  // nb+1 offsets entries fit in LDS
    if (staged) {
        for (int i = threadIdx.x; i <= (int)nb; i += kLinThreads) {
            int64_t rel = offsets[lo + i] - p0;
            rel = rel < -1 ? -1 : (rel > kLinTile ? kLinTile : rel);
            s_off[i] = (int32_t)rel;
            if (i >= 1 && i < (int)nb && rel >= 0 && rel < kLinTile) atomicMax(&s_own[rel], i);   // bag lo+i starts here
        }
    }
    __syncthreads();
    const int lane = lane_id();
    const int w = threadIdx.x >> 6;
    int32_t own[kItems];
    if (staged) {
        // running maximum: along each row of 64 by shuffles, carried from row to row, then across the wavefronts
        int32_t carry = 0;
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            int32_t v = s_own[w * (kWave * kItems) + k * kWave + lane];
            for (int o = 1; o < kWave; o <<= 1) {
                const int32_t up = __shfl_up(v, o, kWave);
                if (lane >= o) v = up > v ? up : v;
            }
            v = v > carry ? v : carry;
            own[k] = v;
            carry = __shfl(v, kWave - 1, kWave);
        }
        if (lane == 0) s_wmax[w] = carry;
        __syncthreads();
        int32_t prev = 0;
        for (int ww = 0; ww < w; ++ww) prev = s_wmax[ww] > prev ? s_wmax[ww] : prev;
#pragma unroll
        for (int k = 0; k < kItems; ++k) own[k] = own[k] > prev ? own[k] : prev;
    }
    // The ids and the row ranges of all of a thread's positions first (a position behind the tile's end reads the
    // tile's last one), pinned in registers here: left to itself the compiler moves every load into the branch that
    // uses it and waits for it there, one position after the other.
    int64_t idv[kItems], bagv[kItems], rbv[kItems], rev[kItems];
    if (indices.is32) {
        const int32_t* q = static_cast<const int32_t*>(indices.p);
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            const int64_t p = p0 + w * (kWave * kItems) + k * kWave + lane;
            idv[k] = (int64_t)q[p < p1 ? p : p1 - 1];
        }
    } else {
        const int64_t* q = static_cast<const int64_t*>(indices.p);
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            const int64_t p = p0 + w * (kWave * kItems) + k * kWave + lane;
            idv[k] = q[p < p1 ? p : p1 - 1];
        }
    }
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int64_t p = p0 + w * (kWave * kItems) + k * kWave + lane;
        int64_t bag;
        if (staged) bag = lo + own[k];
        else bag = upper_bound_i64(offsets, lo, hi + 1, p < p1 ? p : p1 - 1) - 1;   // a tile spanning more than kLinTile bags (runs of empty bags)
        bag = bag < lo ? lo : (bag > hi ? hi : bag);
        bagv[k] = bag;
        const int32_t t = (int32_t)(bag / B);
        rbv[k] = row_base[t];
        rev[k] = row_base[t + 1];
    }
#pragma unroll
    for (int k = 0; k < kItems; ++k) asm volatile("" : "+v"(idv[k]), "+v"(rbv[k]), "+v"(rev[k]));
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int64_t p = p0 + w * (kWave * kItems) + k * kWave + lane;
        if (p >= p1) continue;
        const int64_t bag = bagv[k];
        const int64_t rb = rbv[k];
        const int64_t R = rev[k] - rb;
        const int64_t id = idv[k];
        // local_keys: the table-local id (an invalid id gets R, one past the table's last row); the sort's last
        // pass turns it into the linearised key
        uint32_t key;
        if (id >= 0 && id < R) {
            key = local_keys ? (uint32_t)id : (uint32_t)(rb + id);
        } else {
            key = local_keys ? (uint32_t)R : invalid_key;
            atomicOr(err, 1);
        }
        keys[p] = key;
        bag_of_pos[p] = (uint32_t)bag;
    }
}

hipError_t launch_linearize(const tbe_handle* h, const void* indices_p, const void* offsets_p, int idx32, int32_t B,
                            int64_t N, uint32_t* keys, uint32_t* bag_of_pos, hipStream_t s) {
    const IdxView indices{indices_p, idx32}, offsets{offsets_p, idx32};
    const int64_t nbags = (int64_t)h->T * B;
    const unsigned grid = (unsigned)((N + kLinTile - 1) / kLinTile);
    LaunchTimer tm(h, s, "linearize");
    linearize_kernel<<<grid, kLinThreads, 0, s>>>(indices, offsets, nbags, B, h->d_row_base, (uint32_t)h->total_rows,
                                                  h->segmented, N, keys, bag_of_pos, h->d_err);
    tm.done();
    return hipGetLastError();
}

// =================================================================================================
// Segmented LSD radix sort, <= 8 bits per pass.  The positions are cut into segments (one per table, or a single
// one) and every segment into chunks of at most `chunk` positions; a chunk never crosses a segment border.
//   plan    : segment borders from offsets, chunk descriptors (once per sort)
//   hist    : block k counts the digits of chunk k                                   -> ghist[digit][k]
//   binscan : block d turns ghist[d][*] into an exclusive scan per segment, in place -> bin_tot[segment][d]
//   scatter : block k ranks its chunk tile by tile and writes (key, val) to its final place inside the segment
// Chunk k precedes chunk k+1, and the scatter ranks elements in input order, so the sort is stable.
// The last pass turns table-local keys into linearised ones as it writes them.
// =================================================================================================
constexpr int kRsThreads = 256;
constexpr int kRsWaves = kRsThreads / kWave;
constexpr int kRsItems = kRadixTile / kRsThreads;  // 16 keys per thread and tile
constexpr int kRsBins = 256;

struct SortPlan {
    const uint32_t* bounds;   // [nseg + 1] first position of every segment; bounds[nseg] = N
    const uint32_t* chunk0;   // [nseg + 1] first chunk of every segment; chunk0[nseg] = number of chunks
    const uint4* desc;        // [chunks] (first position, end position, segment, -)
    int nseg;
    int G;                    // row length of ghist (> number of chunks)
};

// One workgroup.  Segment borders: offsets[t * B], forced into [0, N] and made ascending, so that the chunks
// always tile [0, N) exactly, whatever the offsets array holds.
__global__ __launch_bounds__(1024) void radix_plan_kernel(const IdxView offsets, const int32_t B, const int nseg,
                                                          const int64_t N, const int64_t chunk,
                                                          uint32_t* __restrict__ bounds, uint32_t* __restrict__ chunk0,
                                                          uint4* __restrict__ desc, const int maxc) {
    __shared__ uint32_t s_b[kMaxSortSegments + 1];
    __shared__ uint32_t s_c[kMaxSortSegments + 1];
    for (int t = threadIdx.x; t <= nseg; t += 1024) {
        int64_t b = (t == 0) ? 0 : (t == nseg ? N : offsets[(int64_t)t * B]);
        b = b < 0 ? 0 : (b > N ? N : b);
        s_b[t] = (uint32_t)b;
    }
    __syncthreads();
    if (threadIdx.x == 0) {   // running maximum (ascending borders) and chunk counts; nseg is small
        uint32_t run = 0, c = 0;
        for (int t = 0; t <= nseg; ++t) {
            const uint32_t b = s_b[t] > run ? s_b[t] : run;
            if (t > 0) c += (uint32_t)(((int64_t)b - run + chunk - 1) / chunk);
            run = b;
            s_b[t] = b;
            s_c[t] = c;   // chunks of the segments before t
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t <= nseg; t += 1024) {
        bounds[t] = s_b[t];
        chunk0[t] = s_c[t];
    }
    // chunk c belongs to the last segment t with chunk0[t] <= c (segments without chunks are skipped by this rule)
    const uint32_t total = s_c[nseg] < (uint32_t)maxc ? s_c[nseg] : (uint32_t)maxc;
    for (uint32_t c = threadIdx.x; c < total; c += 1024) {
        int lo = 0, hi = nseg;   // invariant: s_c[lo] <= c, answer in [lo, hi)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_c[mid] <= c) lo = mid;
            else hi = mid;
        }
        const int64_t s = (int64_t)s_b[lo] + (int64_t)(c - s_c[lo]) * chunk;
        const int64_t s1 = s_b[lo + 1];
        const int64_t e = s + chunk < s1 ? s + chunk : s1;
        desc[c] = make_uint4((uint32_t)s, (uint32_t)e, (uint32_t)lo, 0u);
    }
}

// One digit count into the wavefront's private histogram.  When every active lane holds the same digit (the
// common case for the high digits, because ids arrive grouped by table) one lane adds the whole count instead of
// 64 lanes queueing on one LDS word.
__device__ __forceinline__ void hist_add(uint32_t* __restrict__ hw, const uint32_t d, const bool valid) {
    const uint64_t act = __ballot(valid);
    if (act == 0ull) return;
    const uint32_t d0 = bcast_lane(d, __ffsll((unsigned long long)act) - 1);   // (the first active lane's digit)
    const uint64_t same = __ballot(valid && d == d0);
    if (same == act) {
        if (lane_id() == __ffsll((unsigned long long)act) - 1) atomicAdd(&hw[d0], (uint32_t)__popcll(act));
    } else if (valid) {
        atomicAdd(&hw[d], 1u);
    }
}

// Private histograms per wavefront: lanes are spread over kHistCopies of them, which divides the number of lanes
// that meet on one LDS word or bank (the kernel is bound by these LDS additions, not by the key stream: 1.04 ms with
// one copy, 0.83 ms with two, for the three passes of the largest workload).
constexpr int kHistCopies = 2;
__global__ __launch_bounds__(kRsThreads) void radix_hist_kernel(const uint32_t* __restrict__ keys, const SortPlan pl,
                                                                const int shift, const uint32_t mask, const int nbins,
                                                                uint32_t* __restrict__ ghist) {
    __shared__ uint32_t h[kHistCopies * kRsWaves][kRsBins];
    const uint32_t nchunks = pl.chunk0[pl.nseg];
    if (blockIdx.x >= nchunks) {   // unused column: zeros, so that the scan can run over the whole row
        for (int d = threadIdx.x; d < nbins; d += kRsThreads) ghist[(size_t)d * pl.G + blockIdx.x] = 0u;
        return;
    }
    for (int i = threadIdx.x; i < kHistCopies * kRsWaves * kRsBins; i += kRsThreads) (&h[0][0])[i] = 0u;
    __syncthreads();
    uint32_t* hw = h[kHistCopies * (threadIdx.x >> 6) + (threadIdx.x & (kHistCopies - 1))];
    const uint4 ds = pl.desc[blockIdx.x];
    const int64_t s = ds.x, e = ds.y;
    // leading elements up to the next 16-byte boundary, whole uint4 groups, then up to 3 trailing elements
    int64_t lead = (4 - (s & 3)) & 3;
    if (lead > e - s) lead = e - s;
    {
        const int64_t i = s + threadIdx.x;
        const bool valid = (int64_t)threadIdx.x < lead;
        const uint32_t k = valid ? keys[i] : 0u;
        hist_add(hw, (k >> shift) & mask, valid);
    }
    const int64_t s4 = s + lead;
    const int64_t n4 = (e - s4) >> 2;
    const uint4* k4 = reinterpret_cast<const uint4*>(keys + s4);
    for (int64_t base = 0; base < n4; base += kRsThreads) {
        const int64_t i = base + threadIdx.x;
        const bool valid = i < n4;
        uint4 k = make_uint4(0u, 0u, 0u, 0u);
        if (valid) k = k4[i];
        hist_add(hw, (k.x >> shift) & mask, valid);
        hist_add(hw, (k.y >> shift) & mask, valid);
        hist_add(hw, (k.z >> shift) & mask, valid);
        hist_add(hw, (k.w >> shift) & mask, valid);
    }
    {
        const int64_t i = s4 + 4 * n4 + threadIdx.x;
        const bool valid = i < e;
        const uint32_t k = valid ? keys[i] : 0u;
        hist_add(hw, (k >> shift) & mask, valid);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < nbins; d += kRsThreads) {
        uint32_t c = 0;
#pragma unroll
        for (int ww = 0; ww < kHistCopies * kRsWaves; ++ww) c += h[ww][d];
        ghist[(size_t)d * pl.G + blockIdx.x] = c;
    }
}

// grid = nbins blocks; block d scans row d of ghist in place: first over all chunks, then every segment's part is
// re-based to start at zero; bin_tot[segment][d] = number of keys with digit d in the segment
__global__ __launch_bounds__(kRsThreads) void radix_binscan_kernel(uint32_t* __restrict__ ghist, const SortPlan pl,
                                                                   uint32_t* __restrict__ bin_tot) {
    __shared__ uint32_t smem[kRsWaves];
    __shared__ uint32_t s_b0[kMaxSortSegments];
    uint32_t* row = ghist + (size_t)blockIdx.x * pl.G;
    const int nchunks = (int)pl.chunk0[pl.nseg];   // < G; row[nchunks] is an unused column holding zero
    uint32_t carry = 0;
    for (int base = 0; base <= nchunks; base += 4 * kRsThreads) {   // four counts per thread and round
        const int i = base + 4 * (int)threadIdx.x;
        uint32_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (i + q <= nchunks) ? row[i + q] : 0u;
        uint32_t tot;
        uint32_t run = carry + block_excl_scan<kRsThreads>(v[0] + v[1] + v[2] + v[3], smem, &tot);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i + q <= nchunks) row[i + q] = run;     // row[nchunks] = total
            run += v[q];
        }
        carry += tot;
    }
    __syncthreads();
    for (int t = threadIdx.x; t < pl.nseg; t += kRsThreads) {
        const uint32_t b0 = row[pl.chunk0[t]], b1 = row[pl.chunk0[t + 1]];
        s_b0[t] = b0;
        bin_tot[(size_t)t * kRsBins + blockIdx.x] = b1 - b0;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nchunks; i += kRsThreads) row[i] -= s_b0[pl.desc[i].z];
}

// One tile of a chunk.  FULL: all kRadixTile positions exist, so nothing is predicated (all but a chunk's last tile).
template <bool FULL>
__device__ __forceinline__ uint32_t scatter_tile(
    const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in, uint32_t* __restrict__ keys_out,
    uint32_t* __restrict__ vals_out, const int64_t tile, const int64_t e, const int shift, const uint32_t mask,
    const bool iota_vals, const int globalize, const int64_t* __restrict__ row_base, const int32_t B,
    const uint32_t invalid_key, const int seg, uint32_t (*s_cnt)[kRsBins], uint32_t* s_base, uint32_t* s_dstart,
    uint32_t* s_keys, uint32_t* s_vals, uint32_t* s_scan) {
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = tid >> 6;
    const uint64_t lt = lanemask_lt();
    for (int i = tid; i < kRsWaves * kRsBins; i += kRsThreads) (&s_cnt[0][0])[i] = 0u;
    __syncthreads();  // also orders the s_base update / s_keys reads of the previous tile

    uint32_t key[kRsItems], val[kRsItems], off[kRsItems];
    const int64_t wbase = tile + (int64_t)w * (kWave * kRsItems);
    if (iota_vals) {   // the payload is the position itself (the branch sits outside the loop: inside it the compiler
                       // waits for every key before it goes on to the next)
#pragma unroll
        for (int k = 0; k < kRsItems; ++k) {
            const int64_t i = wbase + k * kWave + lane;
            const bool valid = FULL || i < e;
            key[k] = valid ? keys_in[i] : 0xFFFFFFFFu;
            val[k] = valid ? (uint32_t)i : 0u;
        }
    } else {
#pragma unroll
        for (int k = 0; k < kRsItems; ++k) {
            const int64_t i = wbase + k * kWave + lane;
            const bool valid = FULL || i < e;
            key[k] = valid ? keys_in[i] : 0xFFFFFFFFu;
            val[k] = valid ? vals_in[i] : 0u;
        }
    }
    // Rank inside the wave, item by item in input order.  peers = the valid lanes that hold the same digit: per digit
    // bit one ballot, and the lanes that agree with this lane's bit are  ~(ballot ^ (all ones if the bit is set)).
#pragma unroll
    for (int k = 0; k < kRsItems; ++k) {
        const int64_t i = wbase + k * kWave + lane;
        const bool valid = FULL || i < e;
        const uint32_t d = (key[k] >> shift) & mask;
        const uint64_t vmask = FULL ? ~0ull : __builtin_amdgcn_ballot_w64(valid);
        uint32_t plo = (uint32_t)vmask, phi = (uint32_t)(vmask >> 32);
        const uint32_t dv = (FULL || valid) ? d : 0u;   // lanes without an element vote in no ballot
#pragma unroll
        for (int b = 0; b < 8; ++b) {   // (bits above the digit's width are zero in every lane: those rounds change nothing)
            const uint64_t m = __builtin_amdgcn_uicmp(dv & (1u << b), 0u, 33 /* != */);   // lanes whose digit has bit b
            const uint32_t sel = (uint32_t)__builtin_amdgcn_sbfe((int)d, b, 1);           // all ones if this lane's has
            plo &= ~((uint32_t)m ^ sel);
            phi &= ~((uint32_t)(m >> 32) ^ sel);
        }
        const uint64_t peers = ((uint64_t)phi << 32) | plo;   // never empty for a valid lane: it holds the lane itself
        uint32_t old = 0;
        const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : 0;
        if (valid && lane == leader) old = atomicAdd(&s_cnt[w][d], (uint32_t)__popcll(peers));
        old = __shfl(old, leader, kWave);
        off[k] = old + (uint32_t)__popcll(peers & lt);
    }
    __syncthreads();
    // per digit: exclusive offsets over the waves, tile total, exclusive scan over the digits
    uint32_t my_tot = 0;
    {
        uint32_t run = 0;
#pragma unroll
        for (int ww = 0; ww < kRsWaves; ++ww) {
            const uint32_t c = s_cnt[ww][tid];
            s_cnt[ww][tid] = run;
            run += c;
        }
        my_tot = run;
        uint32_t tot;
        const uint32_t ex = block_excl_scan<kRsThreads>(my_tot, s_scan, &tot);
        s_dstart[tid] = ex;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kRsItems; ++k) {
        const int64_t i = wbase + k * kWave + lane;
        if (FULL || i < e) {
            const uint32_t d = (key[k] >> shift) & mask;
            const uint32_t pos = s_dstart[d] + s_cnt[w][d] + off[k];
            s_keys[pos] = key[k];
            s_vals[pos] = val[k];
        }
    }
    __syncthreads();
    const int cnt = FULL ? kRadixTile : (int)(e - tile);
    for (int j = tid; j < cnt; j += kRsThreads) {
        const uint32_t kk = s_keys[j];
        const uint32_t d = (kk >> shift) & mask;
        const uint32_t dst = s_base[d] + ((uint32_t)j - s_dstart[d]);
        const uint32_t vv = s_vals[j];
        uint32_t ko = kk;
        if (globalize) {   // last pass of a segmented sort: table-local id -> linearised row key
            // the table comes from the lookup's bag where the payload is one (so that key and bag always agree),
            // else from the segment
            const int t = globalize == 1 ? (int)(vv / (uint32_t)B) : seg;
            const int64_t rb = row_base[t];
            ko = ((int64_t)kk >= row_base[t + 1] - rb) ? invalid_key : (uint32_t)(rb + kk);
        }
        keys_out[dst] = ko;
        vals_out[dst] = vv;
    }
    __syncthreads();
    return my_tot;
}

__global__ __launch_bounds__(kRsThreads) void radix_scatter_kernel(const uint32_t* __restrict__ keys_in,
                                                                   const uint32_t* __restrict__ vals_in,
                                                                   uint32_t* __restrict__ keys_out,
                                                                   uint32_t* __restrict__ vals_out, const SortPlan pl,
                                                                   const int shift, const uint32_t mask, const int nbins,
                                                                   const uint32_t* __restrict__ ghist,
                                                                   const uint32_t* __restrict__ bin_tot,
                                                                   const bool iota_vals, const int globalize,
                                                                   const int64_t* __restrict__ row_base, const int32_t B,
                                                                   const uint32_t invalid_key) {
    __shared__ uint32_t s_cnt[kRsWaves][kRsBins];  // per-wave digit counts, then per-wave exclusive offsets
    __shared__ uint32_t s_base[kRsBins];           // where this block's next element of digit d goes
    __shared__ uint32_t s_dstart[kRsBins];         // start of digit d inside the locally sorted tile
    __shared__ uint32_t s_keys[kRadixTile];
    __shared__ uint32_t s_vals[kRadixTile];
    __shared__ uint32_t s_scan[kRsWaves];

    const int tid = threadIdx.x;
    if (blockIdx.x >= pl.chunk0[pl.nseg]) return;
    const uint4 ds = pl.desc[blockIdx.x];
    const int64_t s = ds.x, e = ds.y;
    const int seg = (int)ds.z;
    {   // base of every digit for this chunk: segment start + (digits below d, whole segment) + (digit d, the
        // segment's chunks before this one)
        const uint32_t t = (tid < nbins) ? bin_tot[(size_t)seg * kRsBins + tid] : 0u;
        uint32_t tot;
        const uint32_t ex = block_excl_scan<kRsThreads>(t, s_scan, &tot);
        s_base[tid] = (tid < nbins) ? pl.bounds[seg] + ex + ghist[(size_t)tid * pl.G + blockIdx.x] : 0u;
    }
    for (int64_t tile = s; tile < e; tile += kRadixTile) {
        uint32_t my_tot;
        if (e - tile >= (int64_t)kRadixTile)
            my_tot = scatter_tile<true>(keys_in, vals_in, keys_out, vals_out, tile, e, shift, mask, iota_vals,
                                        globalize, row_base, B, invalid_key, seg, s_cnt, s_base, s_dstart, s_keys, s_vals, s_scan);
        else
            my_tot = scatter_tile<false>(keys_in, vals_in, keys_out, vals_out, tile, e, shift, mask, iota_vals,
                                         globalize, row_base, B, invalid_key, seg, s_cnt, s_base, s_dstart, s_keys, s_vals, s_scan);
        s_base[tid] += my_tot;
    }
}

hipError_t launch_radix_sort(const tbe_handle* h, const Workspace& w, char* ws, int64_t N, const uint32_t* payload,
                             const void* offsets, int idx32, int32_t B, int* result_buf, hipStream_t s) {
    const int passes = h->sort_passes;
    const int bits = (h->sort_bits + passes - 1) / passes;  // <= 8
    const int nbins = 1 << bits;
    const uint32_t mask = (uint32_t)nbins - 1u;
    uint32_t* ghist = reinterpret_cast<uint32_t*>(ws + w.radix_hist);
    uint32_t* bin_tot = reinterpret_cast<uint32_t*>(ws + w.bin_tot);
    SortPlan pl;
    pl.bounds = reinterpret_cast<const uint32_t*>(ws + w.seg_bounds);
    pl.chunk0 = reinterpret_cast<const uint32_t*>(ws + w.seg_chunk0);
    pl.desc = reinterpret_cast<const uint4*>(ws + w.chunk_desc);
    pl.nseg = w.nseg;
    pl.G = w.radix_maxc + 1;
    {
        LaunchTimer tm(h, s, "radix_plan");
        radix_plan_kernel<<<1, 1024, 0, s>>>(IdxView{offsets, idx32}, B, w.nseg, N, w.radix_chunk,
                                             reinterpret_cast<uint32_t*>(ws + w.seg_bounds),
                                             reinterpret_cast<uint32_t*>(ws + w.seg_chunk0),
                                             reinterpret_cast<uint4*>(ws + w.chunk_desc), w.radix_maxc);
        tm.done();
    }
    const int grid = w.radix_maxc;
    int cur = 0;
    for (int p = 0; p < passes; ++p) {
        const uint32_t* kin = reinterpret_cast<const uint32_t*>(ws + w.keys[cur]);
        const uint32_t* vin = (p == 0 && payload) ? payload : reinterpret_cast<const uint32_t*>(ws + w.vals[cur]);
        uint32_t* kout = reinterpret_cast<uint32_t*>(ws + w.keys[cur ^ 1]);
        uint32_t* vout = reinterpret_cast<uint32_t*>(ws + w.vals[cur ^ 1]);
        const int shift = p * bits;
        {
            LaunchTimer tm(h, s, "radix_hist");
            radix_hist_kernel<<<grid + 1, kRsThreads, 0, s>>>(kin, pl, shift, mask, nbins, ghist);
            tm.done();
        }
        {
            LaunchTimer tm(h, s, "radix_binscan");
            radix_binscan_kernel<<<nbins, kRsThreads, 0, s>>>(ghist, pl, bin_tot);
            tm.done();
        }
        {
            LaunchTimer tm(h, s, "radix_scatter");
            // the last pass of a segmented sort writes linearised keys: table from the bag id (pooled) or the segment
            const int globalize = (h->segmented && p == passes - 1) ? (payload ? 1 : 2) : 0;
            radix_scatter_kernel<<<grid, kRsThreads, 0, s>>>(kin, vin, kout, vout, pl, shift, mask, nbins, ghist, bin_tot,
                                                             p == 0 && !payload, globalize, h->d_row_base, B,
                                                             (uint32_t)h->total_rows);
            tm.done();
        }
        cur ^= 1;
    }
    *result_buf = cur;
    return hipGetLastError();
}

// =================================================================================================
// run-length segmentation of the sorted keys: unique_rows, seg_start, num_unique
// Element order inside a tile: 8 rows of 256, row k / wave w / lane l is element k*256 + w*64 + l, so
// every (k, w) pair is a run of 64 consecutive elements and ballots give exact ranks.
// =================================================================================================
constexpr int kRleThreads = 256;
constexpr int kRleItems = kRleTile / kRleThreads;            // 8
constexpr int kRleRuns = kRleItems * (kRleThreads / kWave);  // runs of 64 elements per tile
static_assert(kRleRuns <= kWave, "one wavefront scans the run counts of a tile");

// Head flags of a thread's kRleItems elements (element k*kRleThreads + tid of the tile): element i is a head if it
// exists and its key differs from its predecessor's.  The loads are unconditional (indices clamped into the array,
// which always holds at least one element) and all issued before the first comparison, so that they overlap.
__device__ __forceinline__ void head_flags(const uint32_t* __restrict__ keys, const int64_t base, const int64_t N,
                                           bool (&head)[kRleItems]) {
    uint32_t cur[kRleItems], prev[kRleItems];
#pragma unroll
    for (int k = 0; k < kRleItems; ++k) {
        const int64_t i = base + k * kRleThreads + threadIdx.x;
        const bool in = i < N;
        cur[k] = keys[in ? i : 0];
        prev[k] = keys[(in && i > 0) ? i - 1 : 0];
    }
#pragma unroll
    for (int k = 0; k < kRleItems; ++k) {
        const int64_t i = base + k * kRleThreads + threadIdx.x;
        head[k] = i < N && (i == 0 || cur[k] != prev[k]);
    }
}

__global__ __launch_bounds__(kRleThreads) void rle_count_kernel(const uint32_t* __restrict__ keys, const int64_t N,
                                                                uint32_t* __restrict__ block_counts) {
    __shared__ uint32_t s_w[kRleThreads / kWave];
    const int64_t base = (int64_t)blockIdx.x * kRleTile;
    uint32_t c = 0;   // heads seen by this wavefront: one ballot and one population count per run of 64 keys
    bool head[kRleItems];
    head_flags(keys, base, N, head);
#pragma unroll
    for (int k = 0; k < kRleItems; ++k) c += (uint32_t)__popcll(__ballot(head[k]));
    if (lane_id() == 0) s_w[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tot = 0;
#pragma unroll
        for (int w = 0; w < kRleThreads / kWave; ++w) tot += s_w[w];
        block_counts[blockIdx.x] = tot;
    }
}

// single block: exclusive scan of the per-tile head counts in place; writes num_unique and the closing
// seg_start entry.
__global__ __launch_bounds__(1024) void rle_scan_kernel(uint32_t* __restrict__ block_counts, const int nblocks,
                                                        const int64_t N, uint32_t* __restrict__ seg_start,
                                                        uint32_t* __restrict__ counters) {
    __shared__ uint32_t smem[1024 / kWave];
    uint32_t carry = 0;
    for (int base = 0; base < nblocks; base += 4 * 1024) {   // four counts per thread and round: a quarter of the barriers
        const int i = base + 4 * (int)threadIdx.x;
        uint32_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (i + q < nblocks) ? block_counts[i + q] : 0u;
        uint32_t tot;
        uint32_t run = carry + block_excl_scan<1024>(v[0] + v[1] + v[2] + v[3], smem, &tot);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i + q < nblocks) block_counts[i + q] = run;
            run += v[q];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) {
        counters[0] = carry;  // num_unique
        seg_start[carry] = (uint32_t)N;
    }
}

// Writes unique_rows and seg_start: element i is a head if its key differs from its predecessor's.
__global__ __launch_bounds__(kRleThreads) void rle_write_kernel(const uint32_t* __restrict__ keys, const int64_t N,
                                                                const int ntiles,
                                                                const uint32_t* __restrict__ block_base,
                                                                uint32_t* __restrict__ unique_rows,
                                                                uint32_t* __restrict__ seg_start) {
    __shared__ uint32_t s_run[kRleRuns];
    const int lane = lane_id();
    const int w = threadIdx.x >> 6;
    const uint64_t lt = lanemask_lt();
    const uint32_t tile = blockIdx.x;
    if (tile >= (uint32_t)ntiles) return;
    const int64_t base = (int64_t)tile * kRleTile;
    uint64_t heads[kRleItems];
    bool head[kRleItems];
    head_flags(keys, base, N, head);
#pragma unroll
    for (int k = 0; k < kRleItems; ++k) {
        heads[k] = __ballot(head[k]);
        if (lane == 0) s_run[k * (kRleThreads / kWave) + w] = (uint32_t)__popcll(heads[k]);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {  // one wavefront scans the 32 run counts
        const uint32_t v = (threadIdx.x < kRleRuns) ? s_run[threadIdx.x] : 0u;
        const uint32_t inc = wave_incl_scan(v);
        if (threadIdx.x < kRleRuns) s_run[threadIdx.x] = inc - v;
    }
    __syncthreads();
    const uint32_t bb = block_base[tile];
#pragma unroll
    for (int k = 0; k < kRleItems; ++k) {
        if ((heads[k] >> lane) & 1ull) {
            const int64_t i = base + k * kRleThreads + threadIdx.x;
            const uint32_t u = bb + s_run[k * (kRleThreads / kWave) + w] + (uint32_t)__popcll(heads[k] & lt);
            unique_rows[u] = keys[i];
            seg_start[u] = (uint32_t)i;
        }
    }
}

hipError_t launch_run_lengths(const tbe_handle* h, const Workspace& w, char* ws, int sorted, int64_t N, hipStream_t s) {
    const uint32_t* keys_sorted = reinterpret_cast<const uint32_t*>(ws + w.keys[sorted]);
    uint32_t* counts = reinterpret_cast<uint32_t*>(ws + w.rle_counts);
    uint32_t* counters = reinterpret_cast<uint32_t*>(ws + w.counters);
    uint32_t* unique_rows = reinterpret_cast<uint32_t*>(ws + w.vals[sorted ^ 1]);
    uint32_t* seg_start = reinterpret_cast<uint32_t*>(ws + w.seg_start);
    {
        LaunchTimer tm(h, s, "rle_count");
        rle_count_kernel<<<w.rle_blocks, kRleThreads, 0, s>>>(keys_sorted, N, counts);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "rle_scan");
        rle_scan_kernel<<<1, 1024, 0, s>>>(counts, w.rle_blocks, N, seg_start, counters);
        tm.done();
    }
    {
        LaunchTimer tm(h, s, "rle_write");
        rle_write_kernel<<<w.rle_blocks, kRleThreads, 0, s>>>(keys_sorted, N, w.rle_blocks, counts, unique_rows, seg_start);
        tm.done();
    }
    return hipGetLastError();
}

}  // namespace tbe
