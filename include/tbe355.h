/*
 * tbe355 - table-batched embedding forward and fused sparse backward with moment-scaled row-wise
 * AdaGrad, for one MI355X (gfx950).  C ABI: plain pointers and sizes, status codes, no exceptions.
 *
 * The operation is the per-GPU embedding step of a sharded recommendation model: every GPU looks up
 * the ids of the batch in the table shards it hosts and, in the backward pass, turns the gradients of
 * the rows that appeared in the batch into an immediate optimizer step, so that no gradient tensor is
 * ever materialised (paper, Section 2.1 and Section 3.1: the backward pass and the optimizer of the
 * sparse tables are fused).  The optimizer is the paper's moment-scaled row-wise AdaGrad
 * (Algorithm 1, steps 5 and 6).
 *
 * Conventions
 *   - T tables; table t has rows[t] rows of D[t] columns.  All tables live in ONE flat device buffer,
 *     table after table, each row-major; element offset of table t is sum_{u<t} rows[u]*D[u].
 *   - A batch has B samples.  Bag (t, b) is the list of ids of table t for sample b.  Ids are
 *     table-local, in [0, rows[t]).  Layout is table-major CSR: bag (t, b) owns
 *     indices[offsets[t*B + b] .. offsets[t*B + b + 1]).  offsets has T*B + 1 entries, offsets[0] = 0,
 *     offsets[T*B] = nnz.  The same id may occur several times in a bag and counts every time.
 *   - Pooled output / upstream gradient: float32 [B, sum(D)] row-major; bag (t, b) maps to columns
 *     D_offsets[t] .. D_offsets[t+1]-1 of row b.
 *   - Every pointer argument marked DEVICE is device memory owned by the caller; HOST pointers are read
 *     during the call only.  The library allocates device memory only in tbe_create (table metadata: a few KB,
 *     plus 1 KB per table for the forward's hot-row hint) and never in the hot calls; its device image also
 *     holds the TBE_STATIC_SCRATCH_BYTES array of tbe_backward_rowwise_adagrad_static.
 *   - The hot calls enqueue kernels on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and return without synchronising.  They are safe to capture into a HIP graph.
 *   - Limits: 4 <= D[t] <= 1024 and D[t] % 4 == 0 (% 8 for fp16 weights); rows[t] < 2^31;
 *     sum(rows) < 2^32 - 1; nnz <= 2^32 - 2^16; T*B < 2^31.
 *   - Errors are returned as tbe_status; nothing is launched when an argument check fails.  An id
 *     outside its table never causes an out-of-bounds access: the forward skips it, the backward gives
 *     it to no row, and both raise a sticky device flag that tbe_poll_index_error reads back.
 */
#ifndef TBE355_H
#define TBE355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tbe_handle tbe_handle; /* opaque: table shapes + small device-side metadata + timing events */

typedef enum {
    TBE_OK = 0,
    TBE_EINVAL = 1,     /* NULL / misaligned pointer, non-finite or out-of-range scalar */
    TBE_ESHAPE = 2,     /* a size outside the limits above */
    TBE_EDTYPE = 3,     /* unknown dtype or pooling code */
    TBE_EWORKSPACE = 4, /* workspace smaller than tbe_workspace_bytes says */
    TBE_EINDEX = 5,     /* an id outside its table was seen (reported by tbe_poll_index_error) */
    TBE_EHIP = 6        /* a HIP runtime call failed */
} tbe_status;

typedef enum { TBE_F32 = 0, TBE_F16 = 1 } tbe_dtype;    /* storage type of the tables; math is fp32 */
typedef enum { TBE_SUM = 0, TBE_MEAN = 1 } tbe_pooling; /* mean divides a bag's sum by its length */
typedef enum { TBE_I64 = 0, TBE_I32 = 1 } tbe_index_dtype;                   /* type of indices AND offsets */
typedef enum { TBE_IO_F32 = 0, TBE_IO_F16 = 1, TBE_IO_BF16 = 2 } tbe_io_dtype; /* pooled output / upstream gradient */

/* Describe the table set.  rows, D: HOST arrays of T entries.  Builds D_offsets / row_base / table
 * offsets on the current device.  One host thread at a time may make calls on a handle; calls on different
 * streams may overlap on the device as long as they do not share a workspace or write the same tables (all they
 * share in the handle is read-only metadata and the sticky invalid-id flag). */
tbe_status tbe_create(int32_t T, const int64_t* rows, const int32_t* D, tbe_dtype weight_dtype, tbe_handle** out);
tbe_status tbe_destroy(tbe_handle* h);

/* Bytes of scratch that tbe_backward_rowwise_adagrad needs for a batch of B samples and at most
 * max_nnz lookups (sort double buffers, segment lists, partial sums of very hot rows). */
tbe_status tbe_workspace_bytes(const tbe_handle* h, int32_t B, int64_t max_nnz, size_t* bytes);

/* Forward: pooled lookup (paper Section 2.1: an id selects a row of its table; the problem statement
 * pools a bag of rows by sum or mean).
 *   out[b, D_offsets[t] + j] = s * sum_{p in bag (t,b)} tables_t[indices[p], j],  s = 1 (sum) or 1/len (mean);
 * an empty bag gives zeros.  fp32 accumulation.
 *   tables    DEVICE  flat weights (float or IEEE binary16 per the handle's dtype), 16-byte aligned
 *   D_offsets DEVICE  int32 [T+1], or NULL to use the handle's own copy
 *   indices   DEVICE  int64 [nnz];  offsets DEVICE int64 [T*B+1]
 *   out       DEVICE  float [B, sum(D)], 16-byte aligned, fully overwritten
 * Order of the additions inside a bag: fixed for given inputs and a given hot-row hint in the handle (see
 * tbe_set_tunable); the hint is rewritten by every backward call on the handle. */
tbe_status tbe_forward(const tbe_handle* h, const void* tables, const int32_t* D_offsets, const int64_t* indices,
                       const int64_t* offsets, int32_t B, int64_t nnz, tbe_pooling pooling, float* out,
                       void* hip_stream);

/* Backward + optimizer, in place (paper Section 2.1: only rows whose ids appear in the batch get a
 * gradient; Section 3.2: a row's gradient is the sum over the samples that hit it; Algorithm 1 steps 5-6).
 * Steps: key[p] = row_base[table of p] + indices[p]; stable ascending radix sort of the keys (equal keys keep
 * the order of their positions p);
 * run-length segmentation into unique rows; per unique row u of table t
 *   g      = sum over the row's segment of  s_bag * grad_out[b, D_offsets[t] : D_offsets[t+1]]
 *   v_u    = v_u + ||g||_2^2                       (state, stored unscaled)
 *   w_u   -= lr / (sqrt(v_u / momentum_scale) + eps) * g      (uses the updated v_u)
 * exactly once per unique row; every other row of tables/state keeps its bits.  momentum_scale is the
 * paper's scaling factor c (> 0); c = 1 is plain row-wise AdaGrad.  Results do not depend on timing:
 * no floating-point atomics are used, so two runs on the same inputs agree bit for bit.
 *   grad_out  DEVICE float [B, sum(D)], 16-byte aligned; finite values (a non-finite element makes the rows it
 *             reaches non-finite, and may do so to other hot rows of the same table)
 *   tables    DEVICE in/out;  state DEVICE float [sum(rows)] in/out, indexed by linearised row key
 *   workspace DEVICE, 256-byte aligned, >= tbe_workspace_bytes(h, B, nnz); contents are scratch */
tbe_status tbe_backward_rowwise_adagrad(const tbe_handle* h, const float* grad_out, const int64_t* indices,
                                        const int64_t* offsets, int32_t B, int64_t nnz, tbe_pooling pooling, float lr,
                                        float eps, float momentum_scale, void* tables, float* state, void* workspace,
                                        size_t workspace_bytes, void* hip_stream);

/* Variants with narrower streams (the id, output and gradient streams are the dominant compulsory bytes when
 * few distinct rows are touched).  Same operations as the two calls above, which are the (TBE_I64, TBE_IO_F32)
 * case.  index_dtype gives the element type of BOTH indices and offsets (int32 needs nnz < 2^31).  out_dtype /
 * grad_dtype give the element type of the [B, sum(D)] matrix: float, IEEE binary16 or bfloat16.  Arithmetic is
 * unchanged (fp32 accumulation): the forward rounds each pooled value once, to nearest even, when it stores it;
 * the backward converts each gradient element exactly to fp32 when it loads it. */
tbe_status tbe_forward_ex(const tbe_handle* h, const void* tables, const int32_t* D_offsets, const void* indices,
                          const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz, tbe_pooling pooling,
                          void* out, tbe_io_dtype out_dtype, void* hip_stream);
tbe_status tbe_backward_rowwise_adagrad_ex(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype,
                                           const void* indices, const void* offsets, tbe_index_dtype index_dtype,
                                           int32_t B, int64_t nnz, tbe_pooling pooling, float lr, float eps,
                                           float momentum_scale, void* tables, float* state, void* workspace,
                                           size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory or size a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): tbe_backward_rowwise_adagrad_ex with its scratch memory in a fixed array
 * of TBE_STATIC_SCRATCH_BYTES bytes that is part of the library's device image (every GPU the library runs on holds
 * one copy until the process ends).  Same arguments otherwise, same kernels, bit-identical results.  Allocates
 * nothing, frees nothing.  A batch that needs more than the array holds - tbe_workspace_bytes(h, B, nnz) >
 * TBE_STATIC_SCRATCH_BYTES - is refused with TBE_EWORKSPACE before anything is launched.  All calls on one GPU share
 * that GPU's array, whatever the handle: two such calls that overlap in time on one GPU (different streams or
 * threads) race, so serialise them; the array keeps the last call's contents, and the kernels clear what they need
 * cleared themselves.  tbe_debug_sorted does not apply to it, and its kernels are not recorded by tbe_timing_* (the
 * first recording of a kernel creates its events). */
#define TBE_STATIC_SCRATCH_BYTES (64u << 20)
tbe_status tbe_backward_rowwise_adagrad_static(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype,
                                               const void* indices, const void* offsets, tbe_index_dtype index_dtype,
                                               int32_t B, int64_t nnz, tbe_pooling pooling, float lr, float eps,
                                               float momentum_scale, void* tables, float* state, void* hip_stream);

/* The backward in two calls, so that the part that needs only the ids can leave the critical path.
 * tbe_backward_prepare runs the linearise / sort / run-length steps (Section 2.1: which rows appear in the batch
 * is known from the ids alone) and leaves their result in `workspace`; it may be enqueued on another stream as soon
 * as the batch's ids are on the device, concurrently with tbe_forward or with the dense part of the model.
 * tbe_backward_apply_rowwise_adagrad then does the per-row reduction and the step (Section 3.2, Algorithm 1 steps
 * 5-6) from grad_out and that workspace.  prepare followed by apply equals tbe_backward_rowwise_adagrad_ex bit for
 * bit.  The caller orders the two (same stream, or an event), passes the same h, offsets, index_dtype, B, nnz and
 * workspace to both and leaves the workspace untouched in between.  apply may be called again on the same prepared
 * workspace (every call is one more step on the same batch).  Argument rules and errors as for the one-call form. */
tbe_status tbe_backward_prepare(const tbe_handle* h, const void* indices, const void* offsets,
                                tbe_index_dtype index_dtype, int32_t B, int64_t nnz, void* workspace,
                                size_t workspace_bytes, void* hip_stream);
tbe_status tbe_backward_apply_rowwise_adagrad(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype,
                                              const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz,
                                              tbe_pooling pooling, float lr, float eps, float momentum_scale,
                                              void* tables, float* state, void* workspace, size_t workspace_bytes,
                                              void* hip_stream);

/* Same backward with the plain SGD step the paper names as the conventional alternative to row-wise AdaGrad
 * (Section 3.2, first paragraph):  w_u -= lr * g  once per unique row, g the row's summed gradient as above.
 * No optimizer state.  Same workspace, argument rules and determinism as the row-wise AdaGrad call. */
tbe_status tbe_backward_sgd(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype, const void* indices,
                            const void* offsets, tbe_index_dtype index_dtype, int32_t B, int64_t nnz, tbe_pooling pooling,
                            float lr, void* tables, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The plain SGD step on a workspace that tbe_backward_prepare filled: prepare + this call equal tbe_backward_sgd bit
 * for bit (Section 3.2, first paragraph, for the step; rules as for tbe_backward_apply_rowwise_adagrad). */
tbe_status tbe_backward_apply_sgd(const tbe_handle* h, const void* grad_out, tbe_io_dtype grad_dtype, const void* offsets,
                                  tbe_index_dtype index_dtype, int32_t B, int64_t nnz, tbe_pooling pooling, float lr,
                                  void* tables, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Non-pooled lookup and its backward (Section 2.1: the forward maps categorical ids to embedding rows; this is
 * that map without pooling, as needed by features that are a long sequence of event ids per sample).
 *   offsets  DEVICE [T+1], ascending from 0 to nnz: the ids of table t are indices[offsets[t] .. offsets[t+1])
 *            (this is the pooled layout with B = 1); same element type as indices
 *   out / grad_seq  DEVICE, 16-byte aligned: one row-major [n_t, D_t] block per table, n_t = offsets[t+1]-offsets[t],
 *            the blocks one after the other (a single [nnz, D] matrix when all tables have the same D);
 *            out_elems / grad_elems = number of elements the caller's buffer holds, >= sum_t n_t * D_t
 * tbe_lookup_seq:  out row of position p = W_t[indices[p], :], converted to out_dtype (one rounding).
 * tbe_backward_seq_rowwise_adagrad: as tbe_backward_rowwise_adagrad_ex with the row gradient
 *   g = sum over the positions p that hold the row's id of grad_seq row p;  workspace >= tbe_workspace_bytes(h, 1, nnz).
 * An id outside its table reads as a zero row in the lookup, gets no update in the backward, and is reported by
 * tbe_poll_index_error; so is an offsets array that is not ascending from 0 to nnz or does not fit the buffer (the
 * lookup then skips the affected rows, the backward updates nothing). */
tbe_status tbe_lookup_seq(const tbe_handle* h, const void* tables, const void* indices, const void* offsets,
                          tbe_index_dtype index_dtype, int64_t nnz, void* out, tbe_io_dtype out_dtype, int64_t out_elems,
                          void* hip_stream);
tbe_status tbe_backward_seq_rowwise_adagrad(const tbe_handle* h, const void* grad_seq, tbe_io_dtype grad_dtype,
                                            int64_t grad_elems, const void* indices, const void* offsets,
                                            tbe_index_dtype index_dtype, int64_t nnz, float lr, float eps,
                                            float momentum_scale, void* tables, float* state, void* workspace,
                                            size_t workspace_bytes, void* hip_stream);

/* Replica synchronisation (Algorithm 1, the weight-sync and moment-sync steps after the local update) for M
 * replicas that live on this one device:  x^(j) <- (1/M) * sum_m x^(m)  for every replica j, element by element.
 * Call it once on the replicas' `tables` buffers (dtype of the handle) and once on their `state` buffers
 * (TBE_F32).  Across devices this step is an all-reduce and is not part of this library.
 *   replicas  HOST array of M DEVICE pointers (1 <= M <= 16), each 16-byte aligned, `count` elements of `dtype`,
 *             no two of the M buffers sharing a byte; read and overwritten in place
 * The sum runs over the replicas in index order in fp32 and is divided by M; binary16 buffers are rounded once,
 * to nearest even.  M == 1 leaves the buffer untouched.  TBE_EINVAL for a null or misaligned pointer, a repeated one, or buffers
 * that overlap. */
tbe_status tbe_replica_mean(tbe_handle* h, void* const* replicas, int32_t M, size_t count, tbe_dtype dtype,
                            void* hip_stream);

/* Parity hooks: DEVICE pointers into `workspace` holding the integer by-products of the last backward
 * call made with the same (h, workspace, B, nnz); valid until the next backward on that workspace.
 *   keys_sorted[nnz]  linearised row keys, ascending
 *   vals_sorted[nnz]  what travelled with each key through the stable sort: after a pooled call the linear bag id
 *                     t*B+b of the lookup (non-decreasing inside a run of equal keys, because positions are
 *                     bag-major and the sort is stable); after a non-pooled call the original position p
 *                     (ascending inside a run of equal keys)
 *   unique_rows[*num_unique] ascending, seg_start[*num_unique + 1] (seg_start[U] = nnz), num_unique[1].
 * Invalid ids, if any, carry the key sum(rows) and form pseudo-rows that no kernel updates: one trailing pseudo-row,
 * or - when the handle sorts table by table, which tbe_create decides from the table sizes - one at the end of
 * every table's run that has invalid ids (keys_sorted is then ascending among the valid ids only).
 * Non-pooled calls: pass B = 1. */
tbe_status tbe_debug_sorted(const tbe_handle* h, void* workspace, int32_t B, int64_t nnz,
                            const uint32_t** keys_sorted, const uint32_t** vals_sorted, const uint32_t** unique_rows,
                            const uint32_t** seg_start, const uint32_t** num_unique);

/* Synchronises the device, reads and clears the sticky invalid-id flag.  Returns TBE_EINDEX if it was set. */
tbe_status tbe_poll_index_error(tbe_handle* h);

/* Tunables of a handle (host-side settings read by later calls; none changes any result beyond the order of
 * floating-point additions).
 *   TBE_TUNE_HOT_ROWS_MIN_WORKGROUPS  The forward keeps, for every table, a copy of the rows that had the most lookups
 *       in the LAST backward call on this handle in on-chip memory (the handle remembers their ids: a hint, the
 *       pooled sums are the same whatever it holds) and serves their lookups from there.  That path runs for a group
 *       of tables of one width when it fills at least `value` workgroups (default 256, one per compute unit; 0:
 *       whenever the width allows it; negative: never). */
typedef enum { TBE_TUNE_HOT_ROWS_MIN_WORKGROUPS = 0 } tbe_tunable;
tbe_status tbe_set_tunable(tbe_handle* h, tbe_tunable which, int64_t value);

/* Per-kernel timing with HIP events on the stream the kernels run on.  tbe_timing_enable(h, 1) clears
 * the record and turns timing on: from then on every kernel that a forward/backward call launches is
 * bracketed by two events and appended to the record, in launch order.  tbe_timing_count gives the
 * number of recorded launches; tbe_timing_read synchronises on launch i's events and returns the
 * kernel's name (a static string) and its duration in milliseconds.  tbe_timing_enable(h, 0) turns it
 * off.  Do not enable while capturing a graph. */
tbe_status tbe_timing_enable(tbe_handle* h, int enable);
tbe_status tbe_timing_count(tbe_handle* h, int32_t* n);
tbe_status tbe_timing_read(tbe_handle* h, int32_t i, const char** name, float* ms);

/* Measurement aid, not a step of the method: a plain streaming copy of `bytes` bytes (multiple of 16, both
 * pointers DEVICE and 16-byte aligned) on `hip_stream`.  Profiles use it as the kernel of known traffic
 * that hardware byte counters are scaled by, and the benchmark reports its rate as the achievable
 * streaming bandwidth next to the published peak.  Recorded by the timing facility as "calibration_copy". */
tbe_status tbe_calibration_copy(tbe_handle* h, void* dst, const void* src, size_t bytes, void* hip_stream);

/* Measurement aid, not a step of the method: `gathers` slices of `slice_bytes` bytes each (a power of two, 16 ..
 * 1024) are read from pseudo-random, slice-aligned places of a window of `window_bytes` bytes (a power of two) of
 * `buf`; with write_back != 0 every slice is written back changed (a read-modify-write, as the row update does).
 * This is the access pattern of the embedding kernels - one table row or one gradient slice per lookup - with the
 * traffic known by construction: gathers * slice_bytes read (and as much written).  The compute die is made of 8
 * partitions with a level-2 cache each, and workgroup i runs on partition i mod 8: with per_xcd != 0 partition x
 * draws its eighth of the slices from a window of its own, buf + x * window_bytes, so that `window_bytes` is the
 * working set of one level-2 cache; with per_xcd == 0 all draw from the one window at buf.  Places are a bijection
 * of the slice number, so up to window_bytes / slice_bytes slices per window are distinct; reads may exceed that
 * (they then repeat, which is what a window smaller than a cache is for), written-back slices may not (TBE_ESHAPE).
 *   buf   DEVICE, 16-byte aligned, buf_bytes >= window_bytes * (per_xcd ? 8 : 1); contents are scratch
 *   sink  DEVICE, 16-byte aligned, sink_bytes >= 2 MiB; receives one checksum word per lane
 * Recorded by the timing facility as "calibration_gather". */
tbe_status tbe_calibration_gather(tbe_handle* h, void* buf, size_t buf_bytes, size_t window_bytes, int32_t per_xcd,
                                  int32_t slice_bytes, int64_t gathers, int32_t write_back, void* sink,
                                  size_t sink_bytes, void* hip_stream);

const char* tbe_status_string(tbe_status s);

/* "tbe355 gfx950 <digest>": the digest names the sources and build settings this library was compiled from (twelve
 * hex digits; "unknown" if the build did not supply one).  Profiles record it next to the byte counts they measured. */
const char* tbe_build_info(void);

#ifdef __cplusplus
}
#endif
#endif /* TBE355_H */
