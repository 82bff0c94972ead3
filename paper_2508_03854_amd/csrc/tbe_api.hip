// C ABI of libtbe355: argument checks, table metadata, workspace carving, stream plumbing, timing.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>

#include "tbe_internal.h"

namespace tbe {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

Workspace carve(const tbe_handle* h, int64_t N) {
    Workspace w;
    memset(&w, 0, sizeof(w));
    const size_t n = (size_t)(N > 0 ? N : 1);
    w.n = N;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align256(off + bytes);
        return at;
    };
    w.keys[0] = take(4 * (n + 1));
    w.keys[1] = take(4 * (n + 1));
    w.vals[0] = take(4 * (n + 1));
    w.vals[1] = take(4 * (n + 1));
    w.bag_of_pos = w.vals[0];   // read by the first radix pass only, which writes keys[1] / vals[1]: no buffer of its own
    w.seg_start = take(4 * (n + 1));
    // radix: G blocks, each owning a contiguous slice that is a whole number of tiles
    int64_t tiles = ((int64_t)n + kRadixTile - 1) / kRadixTile;
    int64_t G = tiles < kRadixMaxBlocks ? tiles : kRadixMaxBlocks;
    int64_t tiles_per_block = (tiles + G - 1) / G;
    w.radix_chunk = tiles_per_block * kRadixTile;
    w.radix_blocks = (int)(((int64_t)n + w.radix_chunk - 1) / w.radix_chunk);
    w.nseg = h->segmented ? h->T : 1;
    w.radix_maxc = w.radix_blocks + w.nseg;
    w.radix_hist = take(4 * (size_t)256 * (size_t)(w.radix_maxc + 1));
    w.bin_tot = take(4 * 256 * (size_t)w.nseg);
    w.seg_bounds = take(4 * (size_t)(w.nseg + 1));
    w.seg_chunk0 = take(4 * (size_t)(w.nseg + 1));
    w.chunk_desc = take(16 * (size_t)w.radix_maxc);
    w.rle_blocks = (int)(((int64_t)n + kRleTile - 1) / kRleTile);
    w.rle_counts = take(4 * (size_t)(w.rle_blocks + 1));
    w.counters = take(4 * kCounterWords);
    // Rows with more than kSegChunk lookups (at most n / (kSegChunk + 1) of them) are reduced into partial sums of
    // maxD floats each.  In the worst case - every lookup in a row just above a threshold - they would need n / 51
    // slots (16 to 20 bytes per lookup at 256 columns); the area holds n / 192 + 4096 (a skewed batch's few hundred
    // thousand hot rows use a fifth of that at the largest workload), slots are given out in row order, and a row
    // that finds none left is reduced by the kernel that applies its step.  Behind it: kDenseChunks slots for each of
    // the at most kDenseRows dense rows of every table.
    w.cap_long = (int64_t)n / (kSegChunk + 1) + 1;
    w.cap_main = (int64_t)n / 192 + 4096;
    w.cap_chunks = w.cap_main + (int64_t)kDenseChunks * kDenseRows * h->T;
    // work units: one per long row, or len/(8*256) + 2 <= len/1024 for the heaviest, or ceil(len/512) <= len/256 shares
    w.cap_units = w.cap_long + (int64_t)n / 1024 + (int64_t)n / 256 + 2;
    w.long_tiles = (int)(((int64_t)n + 1023) / 1024);   // unique rows <= lookups
    w.tile_long = take(4 * (size_t)(w.long_tiles + 1));
    w.tile_slots = take(4 * (size_t)(w.long_tiles + 1));
    w.unit_list = take(8 * (size_t)w.cap_units);
    w.bounds = take(4 * (size_t)(kMaxSlices + 1) * (size_t)w.cap_long);
    w.long_tables = take(4 * 3 * (size_t)(h->T + 1));
    w.tickets = take(4 * (size_t)kTicketWords);   // directly behind long_tables: one loop clears both
    w.seq_gbase = take(8 * (size_t)(h->T + 1));
    w.dense_rows = take(4 * (size_t)kDenseRows * (size_t)h->T);
    w.dense_n = take(4 * (size_t)h->T);
    w.dense_bounds = take(4 * (size_t)kDenseRows * (kDenseChunks + 1) * (size_t)h->T);
    w.long_list = take(16 * (size_t)w.cap_long);
    w.partial = take(4 * (size_t)w.cap_chunks * (size_t)h->maxD);
    w.total = off;
    return w;
}

LaunchTimer::LaunchTimer(const tbe_handle* h_, hipStream_t s_, const char* name) : h(const_cast<tbe_handle*>(h_)), s(s_) {
    if (!h->timing) return;
    if (h->n_used == (int)h->slots.size()) {
        TimingSlot t;
        t.name = name;
        if (hipEventCreate(&t.beg) != hipSuccess || hipEventCreate(&t.end) != hipSuccess) return;
        h->slots.push_back(t);
    }
    slot = h->n_used++;
    h->slots[slot].name = name;
    (void)hipEventRecord(h->slots[slot].beg, s);
}

void LaunchTimer::done() {
    if (slot >= 0) (void)hipEventRecord(h->slots[slot].end, s);
}

// ---- scratch memory for the entry point that allocates nothing ------------------------------------------------------
// A fixed array in the library's device image, one copy per GPU at that GPU's own address.  In host code the array's
// name is only a handle for the runtime: its device address is looked up once per device, with that device current,
// and kept; kernels, copies and fills always get that address, never the name.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[TBE_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, once looked up

// address of `scratch` on the CURRENT device (which is `device`), or nullptr if the runtime cannot give it
static void* static_scratch_address(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}

static int bits_for(uint64_t v) {  // number of bits needed to represent v (>= 1)
    int b = 1;
    while ((v >> b) != 0) ++b;
    return b;
}

}  // namespace tbe

using namespace tbe;

extern "C" {

#ifndef TBE_SOURCE_DIGEST
#define TBE_SOURCE_DIGEST "unknown"
#endif
const char* tbe_build_info(void) { return "tbe355 gfx950 " TBE_SOURCE_DIGEST; }

const char* tbe_status_string(tbe_status s) {
    switch (s) {
        case TBE_OK: return "ok";
        case TBE_EINVAL: return "invalid argument";
        case TBE_ESHAPE: return "size outside the supported limits";
        case TBE_EDTYPE: return "unknown dtype or pooling mode";
        case TBE_EWORKSPACE: return "workspace too small";
        case TBE_EINDEX: return "an id outside its table was seen";
        case TBE_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

tbe_status tbe_create(int32_t T, const int64_t* rows, const int32_t* D, tbe_dtype weight_dtype, tbe_handle** out) {
    if (!out) return TBE_EINVAL;
    *out = nullptr;
    if (!rows || !D) return TBE_EINVAL;
    if (weight_dtype != TBE_F32 && weight_dtype != TBE_F16) return TBE_EDTYPE;
    if (T < 1 || T > (1 << 20)) return TBE_ESHAPE;
    const int dmul = weight_dtype == TBE_F16 ? 8 : 4;
    tbe_handle* h = new (std::nothrow) tbe_handle;
    if (!h) return TBE_EHIP;
    h->T = T;
    h->dtype = weight_dtype;
    h->rows.assign(rows, rows + T);
    h->D.assign(D, D + T);
    h->row_base.assign(T + 1, 0);
    h->w_off.assign(T + 1, 0);
    h->D_off.assign(T + 1, 0);
    int64_t sumD = 0;
    for (int t = 0; t < T; ++t) {
        if (rows[t] < 1 || rows[t] >= ((int64_t)1 << 31) || D[t] < 4 || D[t] > 1024 || D[t] % dmul != 0) {
            delete h;
            return TBE_ESHAPE;
        }
        h->row_base[t + 1] = h->row_base[t] + rows[t];
        h->w_off[t + 1] = h->w_off[t] + rows[t] * (int64_t)D[t];
        sumD += D[t];
        h->D_off[t + 1] = (int32_t)sumD;
        if (D[t] > h->maxD) h->maxD = D[t];
        if (t == 0 || D[t] < h->minD) h->minD = D[t];
        if (h->row_base[t + 1] >= (int64_t)0xFFFFFFFFll || sumD > (int64_t)0x7FFFFFF0ll) {
            delete h;
            return TBE_ESHAPE;
        }
    }
    h->total_rows = h->row_base[T];
    h->total_elems = h->w_off[T];
    h->sumD = (int32_t)sumD;
    h->key_bits = bits_for((uint64_t)h->total_rows);
    {
        int64_t max_rows = 0;
        for (int t = 0; t < T; ++t) max_rows = rows[t] > max_rows ? rows[t] : max_rows;
        const int local_bits = bits_for((uint64_t)max_rows);  // the local key of an invalid id is rows[t] itself
        h->segmented = T > 1 && T <= kMaxSortSegments && (local_bits + 7) / 8 < (h->key_bits + 7) / 8;
        h->sort_bits = h->segmented ? local_bits : h->key_bits;
        h->sort_passes = (h->sort_bits + 7) / 8;
    }
    {   // row-weighted share of the rows as wide as a wavefront (129..256 columns) among the tables up to 256 columns
        double wide = 0.0, all = 0.0;
        for (int t = 0; t < T; ++t) {
            if (D[t] > 256) continue;
            all += (double)rows[t];
            if (D[t] > 128) wide += (double)rows[t];
        }
        h->seg_mostly_wavefront_rows = all > 0.0 && wide >= 0.5 * all;
    }
    if (hipGetDevice(&h->device) != hipSuccess) {
        delete h;
        return TBE_EHIP;
    }
    h->static_scratch = static_scratch_address(h->device);   // (null: the entry point that needs it reports TBE_EHIP)
    const size_t b_doff = align256(4 * (size_t)(T + 1)), b_rb = align256(8 * (size_t)(T + 1)), b_wo = b_rb;
    const size_t b_cls = align256(4 * (size_t)T);
    const bool keep_hot = T <= kMaxSortSegments;
    const size_t b_hot = keep_hot ? align256(4 * (size_t)T * kHotRows) + align256(4 * (size_t)T) : 0;
    const size_t total = b_doff + b_rb + b_wo + 256 + b_cls + b_hot;
    std::vector<int32_t> cls_tables;
    {   // forward classes by lanes per row (D / elements per 16-byte fragment, rounded up to a power of two)
        const int vec = weight_dtype == TBE_F16 ? 8 : 4;
        std::vector<int32_t> lists[7];
        for (int t = 0; t < T; ++t) {
            const int nl = (D[t] + vec - 1) / vec;
            const int c = nl > 128 ? 6 : (nl > 64 ? 5 : (nl > kFwdGroupMaxLanes ? 0 : (nl > 16 ? 1 : (nl > 8 ? 2 : (nl > 4 ? 3 : 4)))));
            lists[c].push_back(t);
        }
        for (int c = 0; c < 7; ++c) {
            h->fwd_first[c] = (int)cls_tables.size();
            h->fwd_count[c] = (int)lists[c].size();
            cls_tables.insert(cls_tables.end(), lists[c].begin(), lists[c].end());
        }
    }
    if (hipMalloc(&h->d_meta, total) != hipSuccess) {
        delete h;
        return TBE_EHIP;
    }
    char* base = static_cast<char*>(h->d_meta);
    h->d_D_off = reinterpret_cast<int32_t*>(base);
    h->d_row_base = reinterpret_cast<int64_t*>(base + b_doff);
    h->d_w_off = reinterpret_cast<int64_t*>(base + b_doff + b_rb);
    h->d_err = reinterpret_cast<int32_t*>(base + b_doff + b_rb + b_wo);
    h->d_fwd_tables = reinterpret_cast<int32_t*>(base + b_doff + b_rb + b_wo + 256);
    if (keep_hot) {   // (zeroed below: no hot rows until a backward call has listed some)
        h->d_hot_ids = reinterpret_cast<uint32_t*>(base + b_doff + b_rb + b_wo + 256 + b_cls);
        h->d_hot_n = h->d_hot_ids + align256(4 * (size_t)T * kHotRows) / 4;
    }
    bool ok = hipMemset(h->d_meta, 0, total) == hipSuccess;
    ok = ok && hipMemcpy(h->d_fwd_tables, cls_tables.data(), 4 * (size_t)T, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(h->d_D_off, h->D_off.data(), 4 * (size_t)(T + 1), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(h->d_row_base, h->row_base.data(), 8 * (size_t)(T + 1), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(h->d_w_off, h->w_off.data(), 8 * (size_t)(T + 1), hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
        (void)hipFree(h->d_meta);
        delete h;
        return TBE_EHIP;
    }
    *out = h;
    return TBE_OK;
}

tbe_status tbe_destroy(tbe_handle* h) {
    if (!h) return TBE_OK;
    for (auto& t : h->slots) {
        (void)hipEventDestroy(t.beg);
        (void)hipEventDestroy(t.end);
    }
    if (h->d_meta) (void)hipFree(h->d_meta);
    delete h;
    return TBE_OK;
}

static tbe_status check_batch(const tbe_handle* h, int32_t B, int64_t nnz) {
    if (B < 1) return TBE_ESHAPE;
    // positions are 32-bit; the margin keeps every strided position loop (steps of at most one tile) from wrapping
    if (nnz < 0 || nnz > (int64_t)0xFFFF0000ll) return TBE_ESHAPE;
    if ((int64_t)h->T * B >= ((int64_t)1 << 31)) return TBE_ESHAPE;
    return TBE_OK;
}

tbe_status tbe_workspace_bytes(const tbe_handle* h, int32_t B, int64_t max_nnz, size_t* bytes) {
    if (!h || !bytes) return TBE_EINVAL;
    const tbe_status st = check_batch(h, B, max_nnz);
    if (st != TBE_OK) return st;
    *bytes = carve(h, max_nnz).total;
    return TBE_OK;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static bool io_ok(int io) { return io == TBE_IO_F32 || io == TBE_IO_F16 || io == TBE_IO_BF16; }
static bool idx_ok(int d) { return d == TBE_I64 || d == TBE_I32; }

tbe_status tbe_forward_ex(const tbe_handle* h, const void* tables, const int32_t* D_offsets, const void* indices,
                          const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz, tbe_pooling pooling,
                          void* out, tbe_io_dtype out_dtype, void* hip_stream) {
    if (!h || !tables || !offsets || !out || (!indices && nnz > 0)) return TBE_EINVAL;
    if (pooling != TBE_SUM && pooling != TBE_MEAN) return TBE_EDTYPE;
    if (!io_ok(out_dtype) || !idx_ok(index_dtype)) return TBE_EDTYPE;
    const tbe_status st = check_batch(h, B, nnz);
    if (st != TBE_OK) return st;
    const size_t ia = index_dtype == TBE_I32 ? 4 : 8;
    if (!aligned(tables, 16) || !aligned(out, 16) || !aligned(indices, ia) || !aligned(offsets, ia)) return TBE_EINVAL;
    const hipError_t e = launch_forward(h, tables, D_offsets ? D_offsets : h->d_D_off, indices, offsets,
                                        index_dtype == TBE_I32, B, nnz, pooling, out, (int)out_dtype,
                                        static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TBE_OK : TBE_EHIP;
}

tbe_status tbe_forward(const tbe_handle* h, const void* tables, const int32_t* D_offsets, const int64_t* indices,
                       const int64_t* offsets, int32_t B, int64_t nnz, tbe_pooling pooling, float* out,
                       void* hip_stream) {
    return tbe_forward_ex(h, tables, D_offsets, indices, offsets, TBE_I64, B, nnz, pooling, out, TBE_IO_F32, hip_stream);
}

// phases of the backward: steps a2-a4 need the ids only, steps a5-a6 need what a2-a4 left in the workspace
constexpr int kPrepare = 1, kApply = 2;

// shared body of the backward entry points; state == nullptr selects the plain SGD step
// seq != 0: the non-pooled layout (B is 1, offsets has T+1 entries, grad_out holds grad_elems elements)
static tbe_status backward_impl(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype, const void* indices,
                                const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz,
                                tbe_pooling pooling, float lr, float eps, float momentum_scale, void* tables, float* state,
                                void* workspace, size_t workspace_bytes, void* hip_stream, int seq = 0,
                                int64_t grad_elems = 0, int phases = kPrepare | kApply) {
    const bool prep = (phases & kPrepare) != 0, apply = (phases & kApply) != 0;
    if (!h || !offsets || (apply && !tables)) return TBE_EINVAL;
    if (nnz > 0 && ((prep && !indices) || (apply && !grad_out))) return TBE_EINVAL;
    if (pooling != TBE_SUM && pooling != TBE_MEAN) return TBE_EDTYPE;
    if (!io_ok(grad_dtype) || !idx_ok(index_dtype)) return TBE_EDTYPE;
    if (!isfinite(lr) || !isfinite(eps) || eps < 0.f || !isfinite(momentum_scale) || !(momentum_scale > 0.f))
        return TBE_EINVAL;
    const tbe_status st = check_batch(h, B, nnz);
    if (st != TBE_OK) return st;
    const size_t ia = index_dtype == TBE_I32 ? 4 : 8;
    if (!aligned(tables, 16) || !aligned(grad_out, 16) || !aligned(state, 4) || !aligned(indices, ia) ||
        !aligned(offsets, ia))
        return TBE_EINVAL;
    if (nnz == 0) return TBE_OK;  // no id appears in the batch: no row has a gradient
    if (!workspace || !aligned(workspace, 256)) return TBE_EINVAL;
    const Workspace w = carve(h, nnz);
    if (workspace_bytes < w.total) return TBE_EWORKSPACE;
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int idx32 = index_dtype == TBE_I32;
    hipError_t e = hipSuccess;
    int buf = h->sort_passes & 1;  // every pass flips the double buffer, starting from 0
    if (prep) {
        e = launch_linearize(h, indices, offsets, idx32, B, nnz, reinterpret_cast<uint32_t*>(ws + w.keys[0]),
                             reinterpret_cast<uint32_t*>(ws + w.bag_of_pos), s);
        if (e != hipSuccess) return TBE_EHIP;
        // pooled: the bag id of every position travels with its key; non-pooled: the position itself
        e = launch_radix_sort(h, w, ws, nnz, seq ? nullptr : reinterpret_cast<const uint32_t*>(ws + w.bag_of_pos),
                              offsets, idx32, B, &buf, s);
        if (e != hipSuccess) return TBE_EHIP;
        e = launch_run_lengths(h, w, ws, buf, nnz, s);
        if (e != hipSuccess) return TBE_EHIP;
    }
    if (!apply) return TBE_OK;
    e = launch_segment_update(h, w, ws, buf ^ 1, grad_out, (int)grad_dtype, offsets, idx32, B, pooling, lr, eps,
                              momentum_scale, tables, state, seq, grad_elems, s);
    return e == hipSuccess ? TBE_OK : TBE_EHIP;
}

tbe_status tbe_backward_rowwise_adagrad_ex(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype,
                                           const void* indices, const void* offsets, tbe_index_dtype index_dtype,
                                           int32_t B, int64_t nnz, tbe_pooling pooling, float lr, float eps,
                                           float momentum_scale, void* tables, float* state, void* workspace,
                                           size_t workspace_bytes, void* hip_stream) {
    if (!state) return TBE_EINVAL;
    return backward_impl(h, grad_out, grad_dtype, indices, offsets, index_dtype, B, nnz, pooling, lr, eps, momentum_scale,
                         tables, state, workspace, workspace_bytes, hip_stream);
}

tbe_status tbe_backward_rowwise_adagrad_static(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype,
                                               const void* indices, const void* offsets, tbe_index_dtype index_dtype,
                                               int32_t B, int64_t nnz, tbe_pooling pooling, float lr, float eps,
                                               float momentum_scale, void* tables, float* state, void* hip_stream) {
    if (!h || !state) return TBE_EINVAL;
    const tbe_status st = check_batch(h, B, nnz);
    if (st != TBE_OK) return st;
    if (carve(h, nnz).total > (size_t)TBE_STATIC_SCRATCH_BYTES) return TBE_EWORKSPACE;   // beyond the fixed array
    if (!h->static_scratch) return TBE_EHIP;
    // per-kernel timing creates events and grows a host-side list on first use: not in a call that allocates nothing
    tbe_handle* hm = const_cast<tbe_handle*>(h);
    const bool timing = hm->timing;
    hm->timing = false;
    const tbe_status r = backward_impl(h, grad_out, grad_dtype, indices, offsets, index_dtype, B, nnz, pooling, lr, eps,
                                       momentum_scale, tables, state, h->static_scratch, (size_t)TBE_STATIC_SCRATCH_BYTES,
                                       hip_stream);
    hm->timing = timing;
    return r;
}

tbe_status tbe_backward_prepare(const tbe_handle* h, const void* indices, const void* offsets,
                                tbe_index_dtype index_dtype, int32_t B, int64_t nnz, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
    return backward_impl(h, nullptr, TBE_IO_F32, indices, offsets, index_dtype, B, nnz, TBE_SUM, 0.f, 0.f, 1.f, nullptr,
                         nullptr, workspace, workspace_bytes, hip_stream, 0, 0, kPrepare);
}

tbe_status tbe_backward_apply_rowwise_adagrad(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype,
                                              const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz,
                                              tbe_pooling pooling, float lr, float eps, float momentum_scale,
                                              void* tables, float* state, void* workspace, size_t workspace_bytes,
                                              void* hip_stream) {
    if (!state) return TBE_EINVAL;
    return backward_impl(h, grad_out, grad_dtype, nullptr, offsets, index_dtype, B, nnz, pooling, lr, eps, momentum_scale,
                         tables, state, workspace, workspace_bytes, hip_stream, 0, 0, kApply);
}

tbe_status tbe_lookup_seq(const tbe_handle* h, const void* tables, const void* indices, const void* offsets,
                          tbe_index_dtype index_dtype, int64_t nnz, void* out, tbe_io_dtype out_dtype, int64_t out_elems,
                          void* hip_stream) {
    if (!h || !tables || !offsets || (!indices && nnz > 0) || (!out && out_elems > 0) || out_elems < 0) return TBE_EINVAL;
    if (!io_ok(out_dtype) || !idx_ok(index_dtype)) return TBE_EDTYPE;
    const tbe_status st = check_batch(h, 1, nnz);
    if (st != TBE_OK) return st;
    const size_t ia = index_dtype == TBE_I32 ? 4 : 8;
    if (!aligned(tables, 16) || !aligned(out, 16) || !aligned(indices, ia) || !aligned(offsets, ia)) return TBE_EINVAL;
    const hipError_t e = launch_lookup_seq(h, tables, indices, offsets, index_dtype == TBE_I32, nnz, out, (int)out_dtype,
                                           out_elems, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TBE_OK : TBE_EHIP;
}

tbe_status tbe_backward_seq_rowwise_adagrad(const tbe_handle* h, const void* grad_seq, tbe_io_dtype grad_dtype,
                                            int64_t grad_elems, const void* indices, const void* offsets,
                                            tbe_index_dtype index_dtype, int64_t nnz, float lr, float eps,
                                            float momentum_scale, void* tables, float* state, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
    if (!state || grad_elems < 0) return TBE_EINVAL;
    return backward_impl(h, grad_seq, grad_dtype, indices, offsets, index_dtype, 1, nnz, TBE_SUM, lr, eps, momentum_scale,
                         tables, state, workspace, workspace_bytes, hip_stream, 1, grad_elems);
}

tbe_status tbe_backward_sgd(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype, const void* indices,
                            const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz, tbe_pooling pooling,
                            float lr, void* tables, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return backward_impl(h, grad_out, grad_dtype, indices, offsets, index_dtype, B, nnz, pooling, lr, 0.f, 1.f, tables,
                         nullptr, workspace, workspace_bytes, hip_stream);
}

tbe_status tbe_backward_apply_sgd(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype, const void* offsets,
                                  tbe_index_dtype index_dtype, int32_t B, int64_t nnz, tbe_pooling pooling, float lr,
                                  void* tables, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return backward_impl(h, grad_out, grad_dtype, nullptr, offsets, index_dtype, B, nnz, pooling, lr, 0.f, 1.f, tables,
                         nullptr, workspace, workspace_bytes, hip_stream, 0, 0, kApply);
}

tbe_status tbe_backward_rowwise_adagrad(const tbe_handle* h, const float* grad_out, const int64_t* indices,
                                        const int64_t* offsets, int32_t B, int64_t nnz, tbe_pooling pooling, float lr,
                                        float eps, float momentum_scale, void* tables, float* state, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
    return tbe_backward_rowwise_adagrad_ex(h, grad_out, TBE_IO_F32, indices, offsets, TBE_I64, B, nnz, pooling, lr, eps,
                                           momentum_scale, tables, state, workspace, workspace_bytes, hip_stream);
}

tbe_status tbe_debug_sorted(const tbe_handle* h, void* workspace, int32_t B, int64_t nnz, const uint32_t** keys_sorted,
                            const uint32_t** vals_sorted, const uint32_t** unique_rows, const uint32_t** seg_start,
                            const uint32_t** num_unique) {
    if (!h || !workspace) return TBE_EINVAL;
    const tbe_status st = check_batch(h, B, nnz);
    if (st != TBE_OK) return st;
    const Workspace w = carve(h, nnz);
    const int buf = h->sort_passes & 1;  // every pass flips the double buffer, starting from 0
    char* ws = static_cast<char*>(workspace);
    if (keys_sorted) *keys_sorted = reinterpret_cast<const uint32_t*>(ws + w.keys[buf]);
    if (vals_sorted) *vals_sorted = reinterpret_cast<const uint32_t*>(ws + w.vals[buf]);
    if (unique_rows) *unique_rows = reinterpret_cast<const uint32_t*>(ws + w.vals[buf ^ 1]);
    if (seg_start) *seg_start = reinterpret_cast<const uint32_t*>(ws + w.seg_start);
    if (num_unique) *num_unique = reinterpret_cast<const uint32_t*>(ws + w.counters);
    return TBE_OK;
}

tbe_status tbe_poll_index_error(tbe_handle* h) {
    if (!h) return TBE_EINVAL;
    int32_t flag = 0;
    if (hipDeviceSynchronize() != hipSuccess) return TBE_EHIP;
    if (hipMemcpy(&flag, h->d_err, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess) return TBE_EHIP;
    if (flag) {
        if (hipMemset(h->d_err, 0, sizeof(flag)) != hipSuccess) return TBE_EHIP;
        return TBE_EINDEX;
    }
    return TBE_OK;
}

tbe_status tbe_replica_mean(tbe_handle* h, void* const* replicas, int32_t M, size_t count, tbe_dtype dtype,
                            void* hip_stream) {
    if (!h || !replicas || M < 1 || M > kMaxReplicas) return TBE_EINVAL;
    if (dtype != TBE_F32 && dtype != TBE_F16) return TBE_EDTYPE;
    const size_t bytes = count * (dtype == TBE_F32 ? 4u : 2u);
    for (int m = 0; m < M; ++m) {
        if (!replicas[m] || !aligned(replicas[m], 16)) return TBE_EINVAL;
        const uintptr_t a0 = reinterpret_cast<uintptr_t>(replicas[m]);
        for (int k = 0; k < m; ++k) {   // two replicas that share bytes would race (equal pointers, or ranges that overlap)
            const uintptr_t b0 = reinterpret_cast<uintptr_t>(replicas[k]);
            if (a0 == b0 || (a0 < b0 + bytes && b0 < a0 + bytes)) return TBE_EINVAL;
        }
    }
    if (count == 0 || M == 1) return TBE_OK;   // the mean over one replica is that replica
    const hipError_t e = launch_replica_mean(h, replicas, M, count, dtype == TBE_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TBE_OK : TBE_EHIP;
}

tbe_status tbe_set_tunable(tbe_handle* h, tbe_tunable which, int64_t value) {
    if (!h) return TBE_EINVAL;
    switch (which) {
        case TBE_TUNE_HOT_ROWS_MIN_WORKGROUPS: h->hot_min_workgroups = value; return TBE_OK;
    }
    return TBE_EINVAL;
}

tbe_status tbe_timing_enable(tbe_handle* h, int enable) {
    if (!h) return TBE_EINVAL;
    h->timing = enable != 0;
    h->n_used = 0;
    return TBE_OK;
}

tbe_status tbe_timing_count(tbe_handle* h, int32_t* n) {
    if (!h || !n) return TBE_EINVAL;
    *n = h->n_used;
    return TBE_OK;
}

tbe_status tbe_timing_read(tbe_handle* h, int32_t i, const char** name, float* ms) {
    if (!h || !name || !ms || i < 0 || i >= h->n_used) return TBE_EINVAL;
    TimingSlot& t = h->slots[i];
    if (hipEventSynchronize(t.end) != hipSuccess) return TBE_EHIP;
    if (hipEventElapsedTime(ms, t.beg, t.end) != hipSuccess) return TBE_EHIP;
    *name = t.name;
    return TBE_OK;
}

}  // extern "C"
