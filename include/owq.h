/*
 * owq.h - C ABI of the OWQ mixed-precision linear layer for AMD MI355X (gfx950).
 *
 * The layer is the one the OWQ paper (arxiv 2306.02272) stores and runs at
 * inference time: a full-size matrix of 3- or 4-bit codes whose weak-column
 * positions are zero-filled, a step size and zero point per output channel or
 * per group of input columns, k "weak" input columns kept in fp16, and one
 * integer index per weak column (section "Outlier-Aware Weight Quantization",
 * storage paragraph; appendix B.2, latency-favoured format).  One call
 * evaluates, for every row n of a batch of fp16 activations,
 *
 *     y[n, i] = sum_{j not weak} s[i, g(j)] * (q[i, j] - z[i, g(j)]) * x[n, j]
 *             + sum_{t < k}      Ww[i, t] * x[n, weak_idx[t]]
 *
 * which is the dequantised dense matrix-vector product plus the product of
 * the fp16 weak columns with the activations gathered at their indices
 * (section "Acceleration on Real Device").  Shapes follow Eq. (3): W is
 * d_out x d_in; the activations are passed transposed, one row per token.
 *
 * All functions return a status code; none throws, aborts or prints.
 * Pointers are marked HOST or DEVICE.  Streams are hipStream_t passed as
 * void* (NULL = the default stream).
 */
#ifndef OWQ_H
#define OWQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct owq_layer_s *owq_handle_t; /* opaque; owned by the library until owq_free_layer */

typedef enum {
  OWQ_OK = 0,
  OWQ_ERR_NULL = 1,       /* a required pointer is NULL */
  OWQ_ERR_SHAPE = 2,      /* d_out < 1, d_in < 1, the packed layer would reach 4 GiB, or a launch shape does not fit */
  OWQ_ERR_BITS = 3,       /* bits is neither 3 nor 4 */
  OWQ_ERR_GROUP = 4,      /* group_size is neither 0 nor a positive multiple of 128 */
  OWQ_ERR_CODE_RANGE = 5, /* a code at a non-weak column is >= 2^bits */
  OWQ_ERR_INDEX = 6,      /* k out of [0, d_in], weak_idx not strictly ascending in [0, d_in), or n_sets out of range */
  OWQ_ERR_BUFFER = 7,     /* a buffer is too small or misaligned */
  OWQ_ERR_BATCH = 8,      /* batch < 0 or above OWQ_MAX_BATCH */
  OWQ_ERR_HANDLE = 9,     /* not a live handle */
  OWQ_ERR_HIP = 10,       /* a HIP call failed; see owq_layer_info_t.last_hip_error */
  OWQ_ERR_UNSUPPORTED = 11, /* the layer needs more on-chip memory than one workgroup may use */
  OWQ_ERR_LAYOUT = 12,     /* layout is none of OWQ_LAYOUT_GEMV, OWQ_LAYOUT_TILE, OWQ_LAYOUT_COMPACT */
  OWQ_ERR_SCRATCH = 13     /* owq_linear_static: the layer needs more than OWQ_STATIC_SCRATCH_BYTES of scratch memory */
} owq_status_t;

#define OWQ_MAX_BATCH 65535
#define OWQ_MAX_WEAK_SETS 65536
#define OWQ_FORMAT_VERSION 1
#define OWQ_STATIC_SCRATCH_BYTES (32u << 20) /* the library's own scratch array, one per GPU, see owq_linear_static */

/*
 * Plain description of a layer.  Every pointer is HOST memory, borrowed for the
 * duration of the call only.
 *   codes     [d_out][d_in], one code per byte, row-major.  Values at weak
 *             columns are ignored and stored as 0 (the zero-filled positions).
 *   scale     fp16 bit patterns, [d_out][G]; G = 1 if group_size == 0, else
 *             ceil(d_in / group_size).  Groups are runs of group_size
 *             consecutive input columns of a row.
 *   zero      fp16 bit patterns, [d_out][G] (any finite fp16 value).
 *   weak_idx  [k], strictly ascending, each in [0, d_in).  May be NULL if k == 0.
 *   weak_w    fp16 bit patterns, [d_out][k] row-major; column t belongs to input
 *             column weak_idx[t].  May be NULL if k == 0.
 */
typedef struct {
  int32_t d_out, d_in;
  int32_t bits;       /* 3 or 4 */
  int32_t group_size; /* 0 = per output channel; else a multiple of 128 */
  int32_t k;
  const uint8_t *codes;
  const uint16_t *scale;
  const uint16_t *zero;
  const int32_t *weak_idx;
  const uint16_t *weak_w;
  int32_t layout;     /* OWQ_LAYOUT_GEMV (0), OWQ_LAYOUT_TILE (1) or OWQ_LAYOUT_COMPACT (2), see below */
} owq_layer_desc_t;

/*
 * Two packed layouts hold the same content.  OWQ_LAYOUT_GEMV is built for single tokens
 * (one lane streams 128 columns of one row; a batch is one pass over the weights per two tokens, where the shape allows, else per token).
 * OWQ_LAYOUT_TILE is built for batches: 32 rows by 256 columns per tile, unpacked straight
 * into matrix-core operands, one pass over the weights per 64 tokens (half the matrix work
 * for 32 tokens or fewer).  Either layout accepts any batch and gives the same result up to
 * rounding; they differ in speed only.  The blob of the tile layout ends in a scratch area
 * (staged activations, sums, fp32 partial results) that owq_linear uses at run time, so that
 * the call needs neither an allocation nor a workspace argument.
 * OWQ_LAYOUT_COMPACT is the storage-favoured format of the paper's appendix B.2 for the
 * single-token kernel: the weak columns are taken out of the low-bit matrix (d_in - k columns
 * are stored, in their original order, blocked as in OWQ_LAYOUT_GEMV), which saves
 * bits * k * d_out / 8 bytes; the kernel moves the activations of the remaining columns
 * together while it stages them.  One scale per row only (group_size = 0, else
 * OWQ_ERR_GROUP).  One more section follows the weak indices: one dword per 8 input columns,
 * low byte = which of them are weak (bit e = column 8i+e), upper 24 bits = the number of weak
 * columns before column 8i; owq_layer_info_t.off_wmask is its offset.
 */
#define OWQ_LAYOUT_GEMV 0
#define OWQ_LAYOUT_TILE 1
#define OWQ_LAYOUT_COMPACT 2

/*
 * Geometry of the packed blob (format version 1) and the launch shape in use.
 * A block is 128 consecutive input columns of one row; a tile is r rows by cw
 * blocks; the blob is four 256-byte-aligned sections (codes, scale/zero pairs,
 * weak weights, weak indices).
 */
typedef struct {
  int32_t format_version;
  int32_t d_out, d_in, bits, group_size, k;
  int32_t nblk, cw, r, nact, nslab, n_rt, d_out_pad, chunks, n_groups, kp;
  uint64_t off_codes, off_sz, off_weak_w, off_weak_idx, total_bytes;
  /* tile layout only: block pairs per row, weak-column bit mask, run-time scratch area;
     scale/zero pairs are stored [group][row] in this layout, [row][group] in the other */
  int32_t layout, nbp;
  uint64_t off_wmask, off_scratch;
  /* launch shape (filled for handles only) */
  int32_t row_tiles_per_wg, row_splits, waves_per_wg, prefetch_depth;
  int32_t workgroups, lds_bytes;
  int32_t last_hip_error;
  int32_t reserved;
} owq_layer_info_t;

/* Geometry for a description; needs no GPU.  Only the shape fields of desc are read. */
owq_status_t owq_geometry(const owq_layer_desc_t *desc, owq_layer_info_t *info);

/* Bytes of DEVICE (or host) memory the packed blob of this layer needs. */
owq_status_t owq_packed_bytes(const owq_layer_desc_t *desc, size_t *bytes);

/*
 * Validate desc and write the packed blob into HOST memory host_buf (at least
 * owq_packed_bytes bytes; every byte of the blob is written).  Needs no GPU.
 */
owq_status_t owq_pack_host(const owq_layer_desc_t *desc, void *host_buf, size_t bytes);

/*
 * Inverse of the code packing: read the codes section of a HOST blob laid out as
 * info describes and write codes [d_out][d_in], one per byte, to HOST memory.
 */
owq_status_t owq_unpack_codes(const void *host_packed, const owq_layer_info_t *info, uint8_t *codes);

/*
 * Validate, pack on the host and upload into DEVICE memory dev_buf (256-byte
 * aligned, at least owq_packed_bytes bytes, owned by the caller, who keeps it
 * alive and unmodified until owq_free_layer).  The copy is enqueued on stream
 * and the call returns after it has completed.  On success *out is a new handle.
 */
owq_status_t owq_pack_layer(const owq_layer_desc_t *desc, void *dev_buf, size_t dev_bytes,
                            void *stream, owq_handle_t *out);

/*
 * Make a handle over a blob that already sits in DEVICE memory dev_buf in packed
 * form (written earlier by owq_pack_host / owq_pack_layer / owq_export_packed for
 * a layer of the same shape, e.g. read back from a file or copied on the device).
 * Only the shape fields of desc are read; the blob's contents are not checked.
 * dev_buf: 256-byte aligned, at least owq_packed_bytes bytes, owned by the caller.
 */
owq_status_t owq_open_packed(const owq_layer_desc_t *desc, void *dev_buf, size_t dev_bytes,
                             owq_handle_t *out);

/*
 * y = layer(x) for a batch of activations.
 *   x  DEVICE, fp16, [batch][d_in] row-major
 *   y  DEVICE, fp16, [batch][d_out] row-major, written in full; must not overlap x
 * Products are accumulated in fp32 and rounded once to fp16 (nearest even).
 * The work is enqueued on stream; the call does not wait, allocate or copy.
 * batch == 0 is a no-op.  The device of dev_buf must be current.
 * Handles of the GEMV layout are immutable: concurrent calls on different streams are
 * allowed.  A handle of the tile layout keeps intermediate results in the scratch area of
 * its blob: calls on one such handle must not overlap in time.
 */
owq_status_t owq_linear(owq_handle_t h, const void *x, void *y, int32_t batch, void *stream);

/*
 * owq_linear with the intermediate results of a tile-layout call in caller-owned DEVICE memory
 * instead of the blob's scratch area: calls on ONE handle may then run on several streams at
 * once, each with a workspace of its own (the same relaxation of section "Weak Column Tuning"'s
 * shared dense matrix to concurrent requests).  workspace: 256-byte aligned, at least
 * owq_workspace_bytes bytes (0 for the other layouts, which need none and ignore it), contents
 * undefined before and after; calls that share a workspace must not overlap.  Same result as
 * owq_linear, bit for bit.  Errors as owq_linear, and OWQ_ERR_BUFFER for a workspace that is
 * too small or misaligned.
 */
owq_status_t owq_workspace_bytes(owq_handle_t h, size_t *bytes);
owq_status_t owq_linear_ws(owq_handle_t h, const void *x, void *y, int32_t batch, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * owq_linear for callers that cannot allocate and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The intermediate
 * results of a tile-layout call go to a static DEVICE array inside the library, of
 * OWQ_STATIC_SCRATCH_BYTES bytes, one per GPU, held from the library's load until the process
 * ends; the blob is only read.  The call allocates nothing and frees nothing.  The work is split
 * so that its partial results fit the array (fewer workgroups than owq_linear may use for large
 * layers); the result equals owq_linear's to rounding (the order of the partial sums may
 * differ).  A layer whose staged activations and one partial result per 256 rows do not fit the
 * array is rejected with OWQ_ERR_SCRATCH.  Every call on a GPU shares that GPU's array and
 * finds the previous call's contents in it (nothing in it has to start at zero: every kernel
 * writes what it later reads); calls that overlap in time on one GPU race.  Handles of the
 * other layouts use no scratch memory and run as owq_linear does.
 */
owq_status_t owq_linear_static(owq_handle_t h, const void *x, void *y, int32_t batch, void *stream);

/*
 * Measurement aids for benchmarks (the context lines beside the layer's own figures; the paper's
 * section "Acceleration on Real Device" compares kernel times): owq_probe_read enqueues one
 * launch that reads `bytes` bytes (a multiple of 16) of DEVICE memory dev_buf (16-byte aligned)
 * once with 128-bit loads from `workgroups` workgroups of 256 threads and computes nothing;
 * owq_probe_read_write does the same and then writes out_bytes bytes (a multiple of 16) of DEVICE
 * memory out (16-byte aligned), each workgroup its share, as a layer call ends on the store of y;
 * owq_probe_empty enqueues a launch of 256 workgroups that does nothing; owq_probe_alu enqueues
 * one launch of `workgroups` workgroups of 256 threads in which every thread issues, `trips`
 * times, 32 runs of the five fp32 instructions that owq_search_config spends per weight and grid
 * point (multiply, round, clamp, two fused multiply-adds) on registers only: 160 * trips
 * instructions per thread; dev_word = 4 bytes of DEVICE memory, 4-byte aligned, which it never
 * writes in practice; owq_probe_mfma, with the same arguments and limits, has every wave issue
 * `trips` times 16 of the 32x32x16 fp16 matrix instructions of the batched path into four
 * independent accumulator tiles on registers only (two workgroups per compute unit as there):
 * workgroups * 4 * trips * 16 * 32768 flops.  Errors: OWQ_ERR_NULL, OWQ_ERR_BUFFER (alignment, size), OWQ_ERR_SHAPE
 * (workgroups out of [1, 65536], trips out of [1, 2^20], 64 GiB or more), OWQ_ERR_HIP.
 */
owq_status_t owq_probe_read(const void *dev_buf, size_t bytes, int32_t workgroups, void *stream);
owq_status_t owq_probe_read_write(const void *dev_buf, size_t bytes, int32_t workgroups, void *out, size_t out_bytes,
                                  void *stream);
owq_status_t owq_probe_empty(void *stream);
owq_status_t owq_probe_alu(void *dev_word, int32_t workgroups, int32_t trips, void *stream);
owq_status_t owq_probe_mfma(void *dev_word, int32_t workgroups, int32_t trips, void *stream);

/*
 * Weak-column tuning (section "Weak Column Tuning" of the paper: after quantisation only the
 * fp16 weak columns are trained, per task; the low-bit matrix and the weak indices are shared).
 *
 * owq_update_weak replaces the layer's own weak columns in place: weak_w HOST, fp16 bit
 * patterns [d_out][k] row-major (may be NULL if k == 0).  The copy is enqueued on stream and
 * the call returns after it has completed; no owq_linear on this handle may be in flight.
 *
 * owq_weak_set_bytes / owq_pack_weak_set make a further set of weak columns for the same layer
 * (same k, same indices) in caller-owned DEVICE memory dev_buf (16-byte aligned, at least
 * owq_weak_set_bytes bytes, kept alive and unmodified while calls use it).
 *
 * owq_linear_multi: as owq_linear, but token n takes its weak columns from
 * weak_sets[task_id[n]] when 0 <= task_id[n] < n_sets, and the layer's own otherwise:
 *     y[n, i] = dense part of x[n] + sum_t Ww[task_id[n]][i, t] * x[n, weak_idx[t]]
 *   weak_sets  DEVICE array of n_sets DEVICE pointers, each written by owq_pack_weak_set for
 *              this layer; 1 <= n_sets <= OWQ_MAX_WEAK_SETS; only entries that some token
 *              selects are read
 *   task_id    DEVICE int32 [batch]
 * Same rounding, stream and overlap rules as owq_linear.
 */
owq_status_t owq_update_weak(owq_handle_t h, const uint16_t *weak_w, void *stream);
owq_status_t owq_weak_set_bytes(owq_handle_t h, size_t *bytes);
owq_status_t owq_pack_weak_set(owq_handle_t h, const uint16_t *weak_w, void *dev_buf, size_t dev_bytes, void *stream);
owq_status_t owq_linear_multi(owq_handle_t h, const void *const *weak_sets, int32_t n_sets, const int32_t *task_id,
                              const void *x, void *y, int32_t batch, void *stream);

/* Release the handle (the host-side record only; dev_buf stays with the caller). */
owq_status_t owq_free_layer(owq_handle_t h);

/* Geometry, launch shape and last HIP error of a handle. */
owq_status_t owq_layer_info(owq_handle_t h, owq_layer_info_t *info);

/* Copy the packed blob back from the device into HOST memory; waits for the copy. */
owq_status_t owq_export_packed(owq_handle_t h, void *host_buf, size_t bytes);

/*
 * Tuning hook for benchmarks: override the launch shape.  A value of 0 keeps the current
 * setting; rejected shapes leave the handle unchanged.  Not thread-safe against concurrent
 * owq_linear on the same handle.
 *   GEMV layout: row_tiles_per_wg >= 1; row_splits divides row_tiles_per_wg; waves_per_wg in
 *     [1, 8] divides nslab * row_splits; prefetch_depth in {2, 4, 8} (8 only with at most 4
 *     waves).
 *   Tile layout: waves_per_wg = 4 or 8 (layers with group-wise scales: 4 only).  row_splits = S > 0: every
 *     group of 64 * waves_per_wg rows is cut into S column ranges, one workgroup each
 *     (S <= d_in / 256; row_tiles_per_wg must be 0 or that number of workgroups).
 *     row_splits = 0 and row_tiles_per_wg = P > 0: the flattened (row group, 256-column step)
 *     sequence is cut into P equal ranges.  Both 0: the default for the chosen waves_per_wg.
 *     The number of workgroups is limited by the partial-result slots of the scratch area.
 *     These three shape the three-launch path, which takes passes of more than 16 tokens.
 *     prefetch_depth shapes the one-launch kernel for passes of few tokens: 0 = the library
 *     uses it for passes of 16 tokens or fewer and chooses its work split; -1 = never use it;
 *     S + 100 c with S in [1, 99], c in [0, 3] = use it for every pass of 32 tokens or fewer,
 *     with every row tile's columns cut into S ranges (S <= d_in / 128) and, for c = 1, 2, 3,
 *     1, 2 or 4 row tiles per workgroup (c = 0: the library chooses).  A shape that does not
 *     fit a later call's number of tokens (the activations of a range must fit LDS) makes
 *     that owq_linear return OWQ_ERR_SHAPE.  The kernel needs x 16-byte aligned, d_in a
 *     multiple of 128, a group size of 128 * 2^n or none, and one task; other calls take the
 *     three-launch path.
 */
owq_status_t owq_set_launch(owq_handle_t h, int32_t row_tiles_per_wg, int32_t row_splits,
                            int32_t waves_per_wg, int32_t prefetch_depth);

/*
 * Quantization configuration search (paper, section "Quantization Configuration Search"): for
 * every output row and every group of its input columns, choose the step size and the zero
 * point from a two-dimensional grid of narrowed ranges so that rounding to nearest with
 * clamping changes the fp16 weights least.  The weak columns take no part: they are neither in
 * the range nor in the error, and their codes are written as 0.  The outputs are what
 * owq_layer_desc_t takes (after a copy to the host).
 *
 * The paper names the search and its objective; the grid is this library's reading.  With C the
 * non-weak columns of the group, lo and hi the least and greatest weight over C, R = hi - lo:
 *     grid       i in [0, n_lo), j in [0, n_hi):  lo_i = lo + a_i R,  hi_j = hi - b_j R,
 *                a_i = shrink i / (n_lo - 1),  b_j = shrink j / (n_hi - 1)   (0 when n = 1)
 *     candidate  s = fp16(max((hi_j - lo_i) / (2^bits - 1), 2^-14)),
 *                z = clamp(rint(-lo_i (1 / s)), -2048, 2048)
 *     codes      q = clamp(rint(w (1 / s)) + z, 0, 2^bits - 1)
 *     error      E = sum over C of (w - s (q - z))^2
 *     choice     least E; among equal E the least i n_hi + j
 * R = 0: the range is widened to reach 0; still 0, or C empty: s = 1, z = 0, every code 0,
 * E = 0, choice 0.  Every step that decides s, z or q is one IEEE binary32 operation (round
 * half to even); E is summed in binary32, so that among candidates whose errors differ by less
 * than that sum's rounding, either may be chosen.  Weights must be finite.
 */
typedef struct {
  int32_t d_out, d_in;
  int32_t bits;       /* 3 or 4 */
  int32_t group_size; /* 0 = one group per row; else a multiple of 128 (the last group may be shorter) */
  int32_t k;          /* number of weak columns, 0 <= k <= d_in */
  int32_t n_lo, n_hi; /* grid points for the lower and the upper end of the range, 1..16 each */
  float shrink;       /* largest fraction of R cut from one end, 0 <= shrink < 0.5 */
} owq_search_desc_t;

/*
 * desc HOST.  DEVICE, owned by the caller, row-major: w fp16 bit patterns [d_out][d_in] (read);
 * weak_idx [k] ascending column indices (read; may be NULL if k == 0; not checked: entries out
 * of order or out of range give a wrong result, never an access out of bounds); written:
 * scale, zero fp16 bit patterns [d_out][G], codes [d_out][d_in], and, unless NULL, err [d_out][G]
 * (E of the choice) and choice [d_out][G] (i n_hi + j).  G = 1 if group_size == 0, else
 * ceil(d_in / group_size).  One launch on `stream`, no allocation, no synchronisation.
 * Errors: OWQ_ERR_NULL, OWQ_ERR_SHAPE (sizes below 1, d_out G above 2^31 - 1, grid or shrink out
 * of range), OWQ_ERR_BITS, OWQ_ERR_GROUP, OWQ_ERR_INDEX (k out of range), OWQ_ERR_UNSUPPORTED (d_in above
 * 385024: the weak-column bit mask of a row must fit 47 KiB of LDS), OWQ_ERR_HIP.
 */
owq_status_t owq_search_config(const owq_search_desc_t *desc, const uint16_t *w, const int32_t *weak_idx,
                               uint16_t *scale, uint16_t *zero, uint8_t *codes, float *err, int32_t *choice,
                               void *stream);

/*
 * Backward of the layer for weak-column tuning (paper, section "PEFT with Weak Column Tuning":
 * after quantisation only the fp16 weak columns are trained, the low-bit matrix stays as it
 * is).  The layer is linear, so its derivatives are its transposes.  With dy = dL/dy:
 *
 *     dx[n, j]            = sum_i dy[n, i] s[i, g(j)] (q[i, j] - z[i, g(j)])      j not weak
 *     dx[n, weak_idx[t]]  = sum_i dy[n, i] Ww[i, t]
 *     dww[i, t]           = sum_n dy[n, i] x[n, weak_idx[t]]
 *
 * Handles of OWQ_LAYOUT_TILE only (else OWQ_ERR_LAYOUT): the codes go from the packed tiles
 * through the matrix cores twice, once to turn them (rows into the contraction axis), once for
 * the product.  DEVICE pointers, owned by the caller, row-major, 16-byte aligned: dy fp16
 * [batch][d_out] (read), x fp16 [batch][d_in] (read; only its weak columns; may be NULL if dww
 * is NULL), dx fp16 [batch][d_in] (written; NULL = not wanted), dww fp32 [d_out][k] (written,
 * summed over the whole batch; NULL = not wanted), workspace of at least
 * owq_backward_workspace_bytes bytes for this batch, 256-byte aligned (contents undefined before and after;
 * calls that share a workspace must not overlap).  fp32 accumulation; dy is first scaled by the
 * power of two that brings its largest magnitude into [512, 1024) (exact, undone on the sums), then
 * dy times the step size is rounded to fp16 once before the product: relative 2^-11 per term whatever
 * the magnitude of the gradients, except for terms whose scaled product falls below 2^-14 (with step
 * sizes of 1e-3: dy more than ten thousand times smaller than the largest one), whose absolute error
 * stays below 2^-25, against largest terms of about 1; step sizes above 64 may overflow the product;
 * dx is rounded to fp16 once.  Work is queued on `stream`, nothing is allocated, nothing synchronises.
 * Errors: OWQ_ERR_HANDLE, OWQ_ERR_LAYOUT, OWQ_ERR_NULL, OWQ_ERR_BATCH, OWQ_ERR_BUFFER (workspace
 * too small, a pointer misaligned), OWQ_ERR_HIP.  batch == 0 is a no-op.
 */
owq_status_t owq_backward_workspace_bytes(owq_handle_t h, int32_t batch, size_t *bytes);
owq_status_t owq_linear_backward(owq_handle_t h, const void *dy, const void *x, void *dx, float *dww,
                                 int32_t batch, void *workspace, size_t workspace_bytes, void *stream);

const char *owq_status_str(owq_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* OWQ_H */
