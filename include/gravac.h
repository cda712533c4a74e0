/*
 * gravac.h - C ABI of the MI355X (gfx950) gradient-compression library.
 *
 * The library implements the per-worker compression path that GraVAC
 * (arxiv 2305.12201) runs on every training iteration:
 *
 *   error feedback      acc = residual + grad                   Sec. III-B (g_ef), Alg. 1 error-feedback step
 *   Top-k at factor CF  keep the k = ceil(n/CF) largest |acc|,  Sec. II-C (CF definition, Top-k: values
 *                       send (index, value) pairs                 and indices are sent, the rest is zero)
 *   residual update     residual = acc - compressed             Alg. 1 residual-update step, Sec. III-B
 *   compression gain    ||g_c||^2 / ||g_ef||^2 for one or       Sec. III-B compression-gain equation,
 *                       several candidate CFs on the same acc     Alg. 1 gain steps (theta_min and theta_s*theta_min)
 *   layerwise mode      the same, independently per tensor      Sec. III-A (layerwise compression)
 *   decompression       rebuild to the dense dimension and      Sec. III-A (t_decompress), Alg. 1 Aggregate
 *                       sum W workers' messages
 *
 * Conventions
 *   - "device pointer": memory of the current HIP device (any allocator).  "host pointer":
 *     ordinary host memory, read before the call returns.
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream).  Outputs are valid once the stream has been synchronised.
 *   - The library never allocates device memory: scratch space comes from the caller's
 *     `workspace`.  Calls that overlap in time must use different workspaces.
 *   - The library keeps no state between calls, with one exception: layerwise calls pass their segment tables
 *     through a ring of up to eight pinned host staging buffers that the library allocates on first use
 *     (hipHostMalloc, grown when a larger table arrives, kept until the process ends) and that are shared by all
 *     callers of the process; the call's first kernel reads the buffer and copies the tables into the workspace.
 *     A caller that issues layerwise calls faster than the GPU runs them is held, once two
 *     buffers exist, until the table copy of an earlier layerwise call (on whatever stream it was queued) has run:
 *     the host then stays at most a call or two ahead.  More buffers are only allocated while others are in the
 *     hands of concurrent callers.  Flat-mode calls touch no such state.
 *   - HIP graphs: a flat-mode compression (gravac_compress, gravac_randomk_compress, gravac_recompress with
 *     n_seg == 0), gravac_commit and gravac_decompress_accumulate consist of kernel launches only (no copies, no
 *     memsets, no host synchronisation), so they can be recorded into a graph and replayed; the host tables
 *     (cf_list, counts) are read at capture time.  Layerwise calls on a capturing stream return GRAVAC_ERR_CAPTURE.
 *   - Return value: GRAVAC_OK (0) or a negative GRAVAC_ERR_* code.  GRAVAC_ERR_INVALID_ARG, GRAVAC_ERR_CAPACITY,
 *     GRAVAC_ERR_WORKSPACE, GRAVAC_ERR_CAPTURE and GRAVAC_ERR_STATIC_LIMIT are found before anything is queued: no
 *     kernel has been launched and no buffer has been touched.  GRAVAC_ERR_HIP means a HIP runtime call failed;
 *     part of the work may have been queued by then, and residual, outputs and workspace are unspecified.
 */
#ifndef GRAVAC_H
#define GRAVAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GRAVAC_OK 0
#define GRAVAC_ERR_INVALID_ARG (-1) /* null pointer, size or CF out of range, bad segment table, misaligned buffer */
#define GRAVAC_ERR_CAPACITY (-2)    /* out_capacity smaller than the number of pairs the call will emit */
#define GRAVAC_ERR_WORKSPACE (-3)   /* workspace missing or smaller than gravac_workspace_bytes() */
#define GRAVAC_ERR_HIP (-4)         /* a HIP runtime call failed (launch, copy) */
#define GRAVAC_ERR_CAPTURE (-5)     /* the stream is being captured into a HIP graph and the call cannot be replayed:
                                       a layerwise call (its segment tables travel through a host staging buffer
                                       that later calls rewrite) */

#define GRAVAC_ERR_STATIC_LIMIT (-6) /* gravac_decompress_accumulate_static: W and n need more than GRAVAC_STATIC_SCRATCH_BYTES */

#define GRAVAC_MAX_CF 8             /* candidate CFs per call */
#define GRAVAC_STATS_PER_CF 4       /* doubles per (segment, CF) in out_stats */

/* flags of the compression calls (0 = none; any other bit is refused) */
#define GRAVAC_FLAG_FORCE_FALLBACK 1u /* a testing aid: skip the sampled threshold estimate, so that every segment takes
                                         the exact-histogram route (same results, more passes over memory) */
#define GRAVAC_FLAG_NO_COMMIT 2u      /* gravac_compress, gravac_randomk_compress: nothing is removed from the residual, which
                                         receives acc = residual + grad as it is; message and statistics are the same.  For
                                         a caller that evaluates two CFs and decides afterwards which message to send
                                         (Alg. 1): compress at theta_min with this flag, derive the candidate CF's message
                                         from that message (gravac_recompress with residual == NULL), then remove the
                                         message that is sent with gravac_commit.  Not accepted by the other calls. */

/*
 * Number of pairs a call will emit for a tensor of n elements at compression factor cf:
 * k = ceil(n / cf) clamped to [1, n]  (Sec. II-C: keeping 10 % is CF 10x, 1 % is CF 100x).
 * Integral cf uses exact integer arithmetic.  Returns -1 for n <= 0 or cf < 1 or non-finite cf.
 */
int64_t gravac_topk_count(int64_t n, double cf);

/*
 * Workspace size in bytes for a gravac_compress call on n elements with n_cf candidate CFs
 * and n_seg segments (0 or 1 = one flat tensor).  The size depends only on these three
 * numbers (it covers any segment table with n_seg entries).  About 16 bytes per element (two index / value lists
 * with a slot per element, so that no list can overflow), plus 56 KB per (segment, CF) and per 65,536 elements for
 * histograms and gather lists, plus 8 KB per sample block (the size allows 64 of them per tensor in layerwise mode,
 * 128 for a flat call).  Examples: 44,549,160 elements flat, one CF: 716 MB; the same as 314 tensors: 986 MB;
 * 138,357,544 elements flat: 2.22 GB.
 */
int gravac_workspace_bytes(int64_t n, int n_cf, int n_seg, size_t* bytes_out);

/*
 * One compression step of Alg. 1 for one worker.
 *
 *   grad        device, float[n], read only.
 *   residual    device, float[n].  In: the leftover of earlier iterations.
 *               Out: acc with the committed selection's slots set to +0.0f (with GRAVAC_FLAG_NO_COMMIT: acc).
 *               (Both may start at any float boundary; the fast path, 16-byte accesses, is taken when both are
 *               16-byte aligned, as every allocator's buffers are.)
 *   n           1 <= n <= 2^31 - 1 (indices are int32).
 *   cf_list     host, double[n_cf], every entry finite and >= 1.  1 <= n_cf <= GRAVAC_MAX_CF.
 *   commit      position in cf_list of the CF whose selection is emitted into out_idx/out_val
 *               and removed from the residual.  Every CF of the list gets its statistics.
 *   seg_offsets host, int64[n_seg + 1], strictly increasing from 0 to n: tensor boundaries for
 *               layerwise mode (independent Top-k per tensor with k_t = ceil(n_t / CF)).
 *               NULL with n_seg == 0 means one flat tensor.
 *   out_idx     device, int32[out_capacity]; out_val device, float[out_capacity].
 *               The message: pairs (global index, acc value) in ascending index order
 *               (segment-major in layerwise mode).  Ties in |acc| go to the lower index.
 *   out_capacity  must be >= sum over segments of gravac_topk_count(n_t, cf_list[commit]).
 *   out_count   device, int64 scalar or NULL: number of pairs written.
 *   out_stats   device, double[max(n_seg,1)][n_cf][4]:
 *               { ||g_c||^2, ||g_ef||^2, gain = ratio (1 if ||g_ef||^2 == 0),
 *                 |acc| of the smallest selected entry }.
 *   workspace   device, 256-byte aligned, at least gravac_workspace_bytes(n, n_cf, n_seg) bytes.
 *               Contents on entry are irrelevant; contents on exit are unspecified.
 *   flags       0, or GRAVAC_FLAG_FORCE_FALLBACK and / or GRAVAC_FLAG_NO_COMMIT.
 */
int gravac_compress(const float* grad, float* residual, int64_t n,
                    const double* cf_list, int n_cf, int commit,
                    const int64_t* seg_offsets, int n_seg,
                    int32_t* out_idx, float* out_val, int64_t out_capacity,
                    int64_t* out_count, double* out_stats,
                    void* workspace, size_t workspace_bytes,
                    unsigned flags, void* stream);

/*
 * Random-k with error feedback (Sec. II-C names it as the sparsifier with negligible compression
 * overhead; the paper runs the controller on top of it in Sec. IV-B).  Everything is as in gravac_compress
 * (error feedback, k = ceil(n_t / CF) per tensor, message layout, residual update, gain for every CF of
 * the list, layerwise mode, workspace, flags) except which k entries are kept: every index i of the flat
 * gradient gets a priority P(seed, i), a keyed bijection of the 31-bit integers, and a tensor keeps its
 * k entries of highest priority.  No two indices share a priority; selections for several CFs under one
 * seed are nested; the draw does not depend on how the gradient is split into tensors.  The caller
 * changes the seed from iteration to iteration (and uses the same seed on every worker if all workers
 * should keep the same indices).
 *
 *   P(seed, i):  z = seed + 0x9E3779B97F4A7C15; z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9;
 *                z = (z ^ (z >> 27)) * 0x94D049BB133111EB; z ^= z >> 31        (64-bit: SplitMix64's first output)
 *                s0 = z mod 2^31, s1 = (z >> 32) mod 2^31, M = 2^31 - 1, then on 32-bit unsigned arithmetic
 *                x = (i + s0) & M;  x ^= x >> 16; x = (x * 0x7FEB352D) & M;  x ^= x >> 15; x = (x * 0x046CA68B) & M;
 *                x ^= x >> 16; x = (x + s1) & M;  x ^= x >> 14; x = (x * 0x2C1B3C6D) & M;
 *                x ^= x >> 15; x = (x * 0x297A2D39) & M;  x ^= x >> 15;  P = x
 *
 *   out_stats   device, double[max(n_seg,1)][n_cf][4]: { ||g_c||^2, ||g_ef||^2, gain, lowest selected priority }.
 */
int gravac_randomk_compress(const float* grad, float* residual, int64_t n,
                            const double* cf_list, int n_cf, int commit, uint64_t seed,
                            const int64_t* seg_offsets, int n_seg,
                            int32_t* out_idx, float* out_val, int64_t out_capacity,
                            int64_t* out_count, double* out_stats,
                            void* workspace, size_t workspace_bytes,
                            unsigned flags, void* stream);

/*
 * Threshold sparsifier with error feedback: what Sec. II-C says of DGC's selection, entries below a threshold are
 * discarded (DGC's momentum correction and gradient clipping are named there but not defined, and are not part of
 * this).  acc = residual + grad (Sec. III-B); entry i is kept iff |acc[i]| >= tau, magnitudes compared as bit
 * patterns with the sign cleared, so an entry equal to tau is kept and a NaN ranks above every tau; the message is
 * the kept (index, acc) pairs in ascending index order, the residual acc with the kept slots set to +0.0f (Alg. 1),
 * the gain ||message||^2 / ||acc||^2 (1 if 0 / 0).  One flat tensor.
 *
 *   grad, residual, n   as for gravac_compress.
 *   tau            positive and finite.
 *   out_idx, out_val   device, int32 / float [out_capacity] (may be NULL if out_capacity is 0).
 *   out_capacity   >= 0.  The number of kept entries depends on the data: if it exceeds out_capacity NOTHING is
 *                  emitted and nothing is removed (the residual holds acc), while out_count and out_stats still
 *                  describe the full selection; the caller sees out_count > out_capacity and calls again with
 *                  larger buffers (on the residual as it is, with a zero gradient) or a higher tau.
 *   out_count      device, int64 scalar, required: the number of entries at or above tau.
 *   out_stats      device, double[4]: { ||g_c||^2, ||g_ef||^2, gain, tau }.
 *   workspace      device, 256-byte aligned, at least gravac_workspace_bytes(n, 1, 0) bytes.
 */
int gravac_threshold_compress(const float* grad, float* residual, int64_t n, float tau,
                              int32_t* out_idx, float* out_val, int64_t out_capacity,
                              int64_t* out_count, double* out_stats,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Multi-level compression (Sec. IV-C): the second-level Top-k.  Given the level-1 message
 * (idx1, val1) that gravac_compress emitted at CF theta1, select the k2 = ceil(k1 / cf_rel) entries of
 * largest |val1| (ties to the lower index, i.e. the earlier position), which is the message a direct
 * compression at CF theta1 * cf_rel would have produced when k2 equals its k.  The commit is deferred:
 * the level-1 entries NOT selected here are written back into the residual, so that after this call
 * the residual is the one a direct compression at the higher CF would have left.
 *
 *   idx1, val1  device, int32[k1] / float[k1], read only: the level-1 message, indices
 *               ascending within a segment (as gravac_compress emits them).
 *   k1          1 <= k1 <= 2^31 - 1.
 *   cf_rel      finite, >= 1: the ratio theta2 / theta1.
 *   seg_counts  host, int64[n_seg], pairs per tensor of a layerwise level-1 message (each >= 1, sum k1);
 *               NULL with n_seg == 0 for a flat message.  Every tensor gets its own k2_t = ceil(k1_t / cf_rel).
 *   residual    device, float[n], or NULL.  In: the residual left by the level-1 commit (0 in the idx1 slots).
 *               Out: residual[idx1[i]] = val1[i] for the entries not selected, +0.0f for the selected.
 *               Entries of idx1 outside [0, n) are not written.  NULL: nothing is restored.
 *   n           length of residual (ignored when residual is NULL).
 *   out_idx, out_val, out_capacity, out_count   as for gravac_compress; the pairs keep idx1's order.
 *               Must not overlap idx1 / val1.
 *   out_stats   device, double[max(n_seg,1)][4]: { ||level-2 message||^2, ||level-1 message||^2, their
 *               ratio (1 if the denominator is 0), |val| of the smallest selected entry }.  The ratio
 *               times the level-1 gain is the gain at theta2 (Sec. IV-C).
 *   workspace   device, 256-byte aligned, at least gravac_workspace_bytes(k1, 1, n_seg) bytes.
 *   flags       0, or GRAVAC_FLAG_FORCE_FALLBACK.
 * Putting the unselected values back costs a scattered store per level-1 entry (most of the call's time for a
 * level-1 message that holds a tenth of the gradient).  A caller that has not committed the level-1 message
 * (gravac_compress with GRAVAC_FLAG_NO_COMMIT) passes residual == NULL here and commits the message it sends with
 * gravac_commit.
 */
int gravac_recompress(const int32_t* idx1, const float* val1, int64_t k1, double cf_rel,
                      const int64_t* seg_counts, int n_seg,
                      float* residual, int64_t n,
                      int32_t* out_idx, float* out_val, int64_t out_capacity,
                      int64_t* out_count, double* out_stats,
                      void* workspace, size_t workspace_bytes,
                      unsigned flags, void* stream);

/*
 * Commit of a message into the residual (Alg. 1, residual update of the branch taken): residual[idx[i]] =
 * +0.0f for i < count.  After a level-1 call with GRAVAC_FLAG_NO_COMMIT it removes the message that is sent, level 1
 * or level 2, from a residual that still holds acc.  With it the controller can also take back the deferred commit of gravac_recompress:
 * after gravac_compress at theta_min and gravac_recompress on its message the residual is the one of the
 * candidate CF; committing the level-1 message's indices makes it the residual of theta_min again.
 * (For the dense branch, gravac_decompress_accumulate of the level-2 message into the residual gives back
 * the error-fed gradient, exactly except that a selected -0.0 comes back as +0.0.)
 *
 *   idx       device, int32[count], read only; entries outside [0, n) are ignored.  count >= 0.
 *   residual  device, float[n].
 */
int gravac_commit(const int32_t* idx, int64_t count, float* residual, int64_t n, void* stream);

/*
 * Decompression with aggregation (Sec. III-A t_decompress; what a worker does with the
 * messages it received): dense_out[idx] += val for workers w = 0 .. W-1 in that order.
 *
 *   idx, val    device, the W messages back to back; worker w's pairs start at
 *               counts[0] + ... + counts[w-1].  Within one worker the indices must be
 *               strictly ascending (as gravac_compress emits them).  Indices outside
 *               [0, n) are ignored.
 *   counts      host, int64[W], pairs per worker (>= 0).  W >= 1.
 *   dense_out   device, float[n]; it is added to, not cleared.
 * Adds are binary32, one per pair, in worker order, so the result does not depend on
 * scheduling.
 *   workspace   device, 256-byte aligned, at least gravac_decompress_workspace_bytes(W, n) bytes, or NULL.
 *               With a workspace the tile boundaries of every message are computed once (one thread per
 *               pair) instead of being searched for tile by tile: up to twice as fast, for messages spread
 *               thinly over dense_out as for dense ones (either way a stretch of 8192 entries that few pairs
 *               name is updated entry by entry, not rewritten whole; without a workspace only for W <= 8); the
 *               result is the same.  Contents on entry are irrelevant.
 */
int gravac_decompress_workspace_bytes(int W, int64_t n, size_t* bytes_out);
int gravac_decompress_accumulate(const int32_t* idx, const float* val,
                                 const int64_t* counts, int W,
                                 int64_t n, float* dense_out,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * The update step of Alg. 1 (w_{i+1} = w_i - eta * g~, g~ the aggregate of the workers' compressed gradients;
 * Eq. (1) for the 1/N of the mean) applied straight from the W messages, without a dense gradient in between:
 * for workers w = 0 .. W-1 in that order and every pair of the message
 *     params[idx] = params[idx] + alpha * val
 * with the product rounded to binary32 first and the sum rounded to binary32 after it (no fused multiply-add).
 * With alpha = -eta / W this is the plain SGD step on the mean of the decompressed messages; what momentum,
 * weight decay or another optimizer needs is gravac_decompress_accumulate into a zeroed buffer instead.
 * alpha = 1 gives gravac_decompress_accumulate bit for bit.  Only entries that a pair names are written, and
 * with a workspace a stretch of 8192 entries that few pairs name is not read whole either.
 *
 *   alpha       any finite or non-finite binary32 value; it is applied as given.
 *   params      device, float[n]; updated in place.
 * All other arguments, the order of the adds and the error behaviour as for gravac_decompress_accumulate
 * (same workspace size).
 */
int gravac_decompress_update(const int32_t* idx, const float* val,
                             const int64_t* counts, int W,
                             int64_t n, float alpha, float* params,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * gravac_decompress_accumulate for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result
 * (bit for bit) and same kernels as gravac_decompress_accumulate with a workspace, but the tile boundaries of the
 * messages live in a buffer of GRAVAC_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy on
 * every GPU the library is used on, held until the process ends).  The call allocates nothing and frees nothing.
 *
 *   limit     gravac_decompress_workspace_bytes(W, n) <= GRAVAC_STATIC_SCRATCH_BYTES, i.e.
 *             min(W, 64) * (ceil(n / 8192) + 1) <= 2^20 (W = 8: n up to about 1.07e9); beyond that the call returns
 *             GRAVAC_ERR_STATIC_LIMIT and launches nothing.
 *   sharing   all calls on one GPU use that GPU's one buffer, which keeps the previous call's contents; every entry a
 *             call reads it has written itself before, so nothing needs clearing.  Calls that overlap in time on one
 *             GPU (different streams or threads) race on the buffer: give such callers gravac_decompress_accumulate
 *             with workspaces of their own.
 */
#define GRAVAC_STATIC_SCRATCH_BYTES (4u << 20)
int gravac_decompress_accumulate_static(const int32_t* idx, const float* val,
                                        const int64_t* counts, int W,
                                        int64_t n, float* dense_out, void* stream);

/*
 * Diagnostics of the last gravac_compress call that used `workspace`: synchronises `stream`
 * and copies 8 int32 to the host pointer out8:
 *   [0] 1 if any segment took the exact-histogram fallback, [1] number of such segments,
 *   [2] internal-error flag (must be 0), [3] number of segments, [4] how many of [1] needed no second
 *   pass over the gradient (the located histogram bin was too coarse and too full and was binned again from the
 *   lists the pass had collected), [5..7] reserved.
 */
int gravac_read_status(const void* workspace, void* stream, int32_t* out8);

const char* gravac_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* GRAVAC_H */
