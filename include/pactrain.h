/* pactrain.h - C ABI of the PacTrain per-step gradient compression path on one AMD GPU.
 *
 * The path (paper Sec. III-B/III-C, Alg. 1): a pruning mask derived from weight magnitudes is
 * known to every data-parallel worker; each worker uses it to pack its flat gradient into a
 * shorter dense buffer; the packed buffers are summed by an ordinary floating-point all-reduce
 * (the sum of Eq. 1); the reduced buffer is scattered back into a dense gradient whose pruned
 * positions are zero (Eq. 2).  This library holds the four operations as GPU kernels:
 *
 *     pac_build_mask -> pac_compress (once per worker) -> pac_reduce_local -> pac_decompress
 *
 * and, further down, what the paper puts around them: the Mask Tracker (Sec. III-B), the weight
 * update of Eq. 1 fused into the decompression, and the ternary payload of Sec. III-D.
 *
 * Conventions
 *  - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller owns every data
 *    buffer.  The context owns only scratch (histograms, tile records, scan state), sized in
 *    pac_create; no call on the path allocates.
 *  - Every path call enqueues its kernels on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and returns without synchronising.  (pac_build_mask runs part of its work
 *    on a stream of the context, forked from and joined back to `hip_stream` with events; see there
 *    for the one case in which it copies a scope table to the device first.)  Calls on one context
 *    must be issued on one stream at a time: they share the context's scratch.
 *  - A call returns PAC_OK or a negative pac_status; argument errors are found on the host before
 *    anything is launched and leave the outputs untouched.  The text of the last error is kept in
 *    the context (pac_last_error).  Nothing throws or aborts.
 *  - What only the device can see (a count that does not match the mask, a bounded wait that gave up)
 *    cannot be returned by a call that does not wait for the device: the kernels raise bits in a status
 *    word of the context, which stays as it is until pac_device_status reads and clears it.
 *  - Layout: bit b of mask word j stands for flat element 64*j + b; bits at or beyond n in the last
 *    word are zero.  prefix[j] is the number of set bits in words 0..j-1 over the whole flat set,
 *    so the element at set bit b of word j lives in compact slot
 *    prefix[j] + popcount(mask[j] & ((1 << b) - 1)): ascending flat index.
 *  - Data buffers need element alignment only (4 bytes for PAC_F32, 2 for PAC_BF16); buffers
 *    aligned to 16 bytes take the wide-access kernels.  d_mask needs 8-byte, d_prefix 4-byte
 *    alignment.
 *  - Limits: n < 2^32 elements, at most PAC_MAX_WORKERS buffers per reduction.
 */
#ifndef PACTRAIN_H
#define PACTRAIN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t pac_status;
enum {
    PAC_OK = 0,
    PAC_ERR_ARG = -1,   /* NULL pointer, bad dtype, bad segment table                         */
    PAC_ERR_ALIGN = -2, /* pointer not aligned to its element size                            */
    PAC_ERR_RANGE = -3, /* n >= 2^32 or > context capacity, sparsity outside [0,1], W out of range */
    PAC_ERR_COUNT = -4, /* nnz passed exceeds n (a count that disagrees with the mask itself is only
                           visible on the device: PAC_DEV_COUNT_MISMATCH)                          */
    PAC_ERR_HIP = -5,   /* a HIP runtime call failed; pac_last_error holds its text           */
    PAC_ERR_NOMEM = -6  /* scratch allocation failed in pac_create                            */
};

typedef enum { PAC_F32 = 0, PAC_BF16 = 1 } pac_dtype;

#define PAC_MAX_WORKERS 64u
#define PAC_TABLE_SLOTS 4u

typedef struct pac_ctx pac_ctx;

/* Bits of the context's device status word (pac_device_status).  The low byte holds conditions
 * under which an output is NOT what this header promises; the bits above it only tell which of the
 * slower, equally exact code paths ran. */
enum {
    PAC_DEV_SCAN_STALLED = 0x01,    /* the prefix scan's bounded wait for an earlier tile gave up: d_prefix
                                       (and a count derived from it) is wrong                              */
    PAC_DEV_COUNT_MISMATCH = 0x02,  /* the number of set mask bits is not the nnz the call was given (or, in
                                       pac_build_mask, not the sum of the scopes' keep counts)             */
    PAC_DEV_META_MISMATCH = 0x04,   /* mask, prefix and nnz passed to a gather / scatter do not fit together:
                                       the tile was skipped (gather) or zero-filled (scatter)              */
    PAC_DEV_RETRY_TAKEN = 0x100,    /* a sampled threshold bracket missed and pac_build_mask ran its
                                       full-count pass                                                     */
    PAC_DEV_SLOW_PATH = 0x200       /* very many equal magnitudes: pac_build_mask resolved a scope from its
                                       weights instead of its candidate lists                              */
};

/* Create a context on HIP device `hip_device` able to build masks over up to `max_elems` flat
 * elements split into up to `max_segments` prune scopes.  Allocates all scratch.  *out is NULL on
 * failure. */
pac_status pac_create(pac_ctx** out, int hip_device, uint64_t max_elems, uint32_t max_segments);

/* Synchronises the device and frees the scratch.  NULL is accepted. */
pac_status pac_destroy(pac_ctx* ctx);

/* Text of the last error of this context ("" if none).  Owned by the context.  With ctx == NULL,
 * the text of the last failed pac_create of this thread. */
const char* pac_last_error(const pac_ctx* ctx);

/* Reads the context's device status word (PAC_DEV_* bits, raised by the kernels of earlier calls on
 * this context and sticky until cleared).  Enqueued on `hip_stream` behind those calls.
 *   d_flags_out (DEVICE uint32, may be NULL): receives the word, in stream order; no host wait.
 *   h_flags_out (HOST uint32, may be NULL): receives the word; the call then waits for the stream.
 *   clear != 0: the word is reset to zero by the same read.
 * With both pointers NULL and clear == 0 the call does nothing. */
pac_status pac_device_status(pac_ctx* ctx, uint32_t* d_flags_out, uint32_t* h_flags_out, int clear,
                             void* hip_stream);

/* Keep count of one prune scope of n elements at a target sparsity (the pruning ratio of Alg. 1):
 * k = ceil((1 - s) * n), evaluated in integers with s rounded to the nearest 1e-6.  Pure host
 * arithmetic; the same rule pac_build_mask applies to each segment.  Returns 0 for s outside
 * [0,1]. */
uint64_t pac_keep_count(uint64_t n, double sparsity);

/* Number of 64-bit mask words (and of prefix entries) for n elements: ceil(n / 64). */
uint64_t pac_mask_words(uint64_t n);

/* (1) Magnitude-pruning mask (paper Sec. II-B: importance = |weight|; Sec. III-B: the selection is a
 * function of the weights alone, hence identical on all workers; Sec. III-C step 1 / Alg. 1 Prune).
 *
 * The flat weights d_weights[0..n) are split into nseg prune scopes [h_seg_offsets[s],
 * h_seg_offsets[s+1]) (h_seg_offsets[0] = 0, [nseg] = n, ascending, empty scopes allowed); scope s
 * keeps k_s = pac_keep_count(len_s, h_sparsity[s]) elements: those first in the order
 * "|w| descending, flat index ascending", where |w| is compared through the bit pattern with the
 * sign cleared (so -0 ties +0, denormals count, NaN ranks above infinity).  nseg = 1 is a global
 * prune, one segment per tensor a per-layer prune.  Weights are not modified.
 *
 * Writes d_mask[ceil(n/64)] and d_prefix[ceil(n/64)]; *h_nnz_out (may be NULL) receives
 * sum_s k_s, which is known on the host without waiting for the device.  n = 0 is allowed
 * (nothing is written).
 *
 * Scope tables: the context keeps the last PAC_TABLE_SLOTS distinct (offsets, sparsity) tables it was
 * given resident on the device.  A call whose table is among them enqueues kernels only.  A call with
 * a new table first copies it to the device (an asynchronous copy from pinned memory of the context,
 * on `hip_stream`; it replaces the least recently used table, and waits on the host only if that
 * slot's previous upload, many calls ago, has still not run).  While `hip_stream` is being captured
 * into a graph a new table is refused with PAC_ERR_ARG: run the call once outside the capture first;
 * a table used under capture then stays resident for the life of the context.
 * Device-side checks: PAC_DEV_COUNT_MISMATCH if the mask it wrote does not hold sum_s k_s bits,
 * PAC_DEV_SCAN_STALLED, and the two informational bits. */
pac_status pac_build_mask(pac_ctx* ctx, const float* d_weights, uint64_t n,
                          const uint64_t* h_seg_offsets, uint32_t nseg, const double* h_sparsity,
                          uint64_t* d_mask, uint32_t* d_prefix, uint64_t* h_nnz_out,
                          void* hip_stream);

/* (2) Compress one worker's flat gradient (paper Sec. I / III-B: the shared mask reformats the
 * sparse gradient into a low-dimensional dense tensor; Alg. 1 compress(update)):
 * d_compact[slot(i)] = d_grad[i] for every set bit i, bit-exact copies, ascending flat index.
 * nnz must be the number of set bits (the value pac_build_mask returned); the kernel never writes
 * at or beyond d_compact[nnz].  A different nnz raises PAC_DEV_COUNT_MISMATCH, metadata that does not
 * fit together PAC_DEV_META_MISMATCH, in the context's device status word. */
pac_status pac_compress(pac_ctx* ctx, const void* d_grad, pac_dtype dtype, uint64_t n,
                        const uint64_t* d_mask, const uint32_t* d_prefix,
                        void* d_compact, uint64_t nnz, void* hip_stream);

/* (3) Element-wise sum of W compact buffers held in this GPU's memory: the payload arithmetic of
 * the all-reduce over workers (the sum in Eq. 1; no 1/n, no learning rate).
 * out[j] = (((c_0[j] + c_1[j]) + c_2[j]) + ... + c_{W-1}[j]) in IEEE single precision, in that
 * order.  PAC_BF16: every input is widened to single, the same adds, one round-to-nearest-even
 * back to bf16 (NaN stays NaN).  h_d_compact is a HOST array of W device pointers, read before
 * the call returns.  d_out may alias one of the inputs.  1 <= W <= PAC_MAX_WORKERS. */
pac_status pac_reduce_local(pac_ctx* ctx, const void* const* h_d_compact, uint32_t W,
                            pac_dtype dtype, uint64_t nnz, void* d_out, void* hip_stream);

/* (4) Decompress (paper Eq. 2 read as a selection): d_dense_out[i] = d_compact[slot(i)] where the
 * mask bit is set, the all-zero bit pattern (+0.0) elsewhere.  Every one of the n outputs is
 * written.  No read at or beyond d_compact[nnz].  Device-side checks as in pac_compress. */
pac_status pac_decompress(pac_ctx* ctx, const void* d_compact, pac_dtype dtype, uint64_t nnz,
                          const uint64_t* d_mask, const uint32_t* d_prefix,
                          void* d_dense_out, uint64_t n, void* hip_stream);

/* (2)+(3) in one pass, for W workers whose dense gradients all lie in THIS GPU's memory: the gather
 * of pac_compress for each worker and the sum of pac_reduce_local, without the W compact buffers in
 * between (Sec. III-B / Alg. 1 compress step, the sum of Eq. 1):
 *   d_reduced[slot(i)] = (((g_0[i] + g_1[i]) + g_2[i]) + ... + g_{W-1}[i])   for every set bit i,
 * same order, same IEEE single adds, same single rounding for PAC_BF16: bit for bit what
 * pac_reduce_local gives on the outputs of W pac_compress calls.  It saves writing and re-reading
 * W * nnz elements and reading the mask and prefix W - 1 times.
 * This call has no counterpart on a real cluster, where the workers' gradients lie on different GPUs
 * and the compact buffers are what travels: it measures an upper bound of the single-GPU stand-in
 * and is reported apart from the four-call path.
 * h_d_grads is a HOST array of W device pointers (n elements each), read before the call returns.
 * Device-side checks as in pac_compress.  1 <= W <= PAC_MAX_WORKERS. */
pac_status pac_step_fused(pac_ctx* ctx, const void* const* h_d_grads, uint32_t W, pac_dtype dtype, uint64_t n,
                          const uint64_t* d_mask, const uint32_t* d_prefix, void* d_reduced, uint64_t nnz,
                          void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Around the hot path: Mask Tracker and weight update.
 * ------------------------------------------------------------------------------------------ */

/* Mask of the non-zero elements of a flat tensor: the (Weight != 0) of paper Eq. 2, which is how the
 * Mask Tracker (Sec. III-B, Mask Tracker paragraph) reads the sparsity pattern off a flattened
 * bucket.  Bit i is set iff d_values[i] != 0 as an IEEE comparison (both zeros are zero; NaN and
 * denormals are not).  Writes d_mask[ceil(n/64)] (bits >= n zero), d_prefix[ceil(n/64)] and, if
 * d_nnz_out is not NULL, the number of set bits to that DEVICE location (the count depends on the
 * data, so the host learns it only by copying it back).  n must not exceed the context's max_elems.
 * Uses the context's scratch, like pac_build_mask. */
pac_status pac_mask_from_nonzero(pac_ctx* ctx, const void* d_values, pac_dtype dtype, uint64_t n,
                                 uint64_t* d_mask, uint32_t* d_prefix, uint64_t* d_nnz_out,
                                 void* hip_stream);

/* pac_mask_from_nonzero for callers that cannot allocate device memory or create a context: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same outputs as
 * pac_mask_from_nonzero, bit for bit.  It takes no context; the scratch of its prefix scan is a 32 KiB
 * array inside the library's device image, which every GPU the library runs on holds until the process
 * ends.  The call allocates nothing, frees nothing and never waits for the device.
 *   - Runs on the CURRENT HIP device; every pointer must belong to it.
 *   - n at most 2^32 - 1 (PAC_ERR_RANGE beyond; the array is sized for that maximum).
 *   - d_flags_out (DEVICE uint32, may be NULL) receives this call's PAC_DEV_* bits (only
 *     PAC_DEV_SCAN_STALLED can occur), in stream order.
 *   - All calls on one GPU share the one array, which keeps the last call's contents (each call clears
 *     what it needs first, on the stream): calls that may run at the same time on one GPU - from two
 *     streams or two threads - race; issue them on one stream, or order the streams with events.
 *   - The first call on a device looks up the array's address (no allocation); make that call, with
 *     any n, n = 0 included, before capturing a stream.
 * Error text: pac_last_error(NULL), per thread. */
pac_status pac_mask_from_nonzero_noalloc(const void* d_values, pac_dtype dtype, uint64_t n, uint64_t* d_mask,
                                         uint32_t* d_prefix, uint64_t* d_nnz_out, uint32_t* d_flags_out,
                                         void* hip_stream);

/* Mask Tracker comparison (Sec. III-B: the mask of this iteration against the previous one):
 * *d_diff_bits_out (DEVICE) = number of positions below n at which the two bitmasks differ;
 * 0 means the sparsity pattern is unchanged.  Bits at and beyond n are ignored. */
pac_status pac_mask_equal(pac_ctx* ctx, const uint64_t* d_mask_a, const uint64_t* d_mask_b, uint64_t n,
                          uint64_t* d_diff_bits_out, void* hip_stream);

/* Mask Tracker bookkeeping (Sec. III-B; Alg. 1, the mask-update step and the stability test that
 * chooses between the two synchronisations): keeps the previous iteration's mask on the device and
 * counts consecutive comparisons that found no difference.  The pattern counts as stable once that
 * count reaches `patience` (the paper asks for an unchanged pattern over several iterations without
 * giving a number: the caller chooses, >= 1).  The first mask a tracker sees, and a mask of another
 * length n, count as a change.
 * pac_tracker_update enqueues compare + copy on the stream and writes {unchanged, stable} to
 * d_state_out (DEVICE uint32[2], may be NULL).  The caller decides between the compressed and the
 * dense synchronisation from that state (for the dense one, pac_reduce_local sums W dense buffers
 * of n elements just as it sums compact ones).  Calls on one tracker must be issued in stream order.
 * The tracker belongs to the context and must be destroyed before it. */
typedef struct pac_tracker pac_tracker;
pac_status pac_tracker_create(pac_ctx* ctx, uint64_t max_elems, uint32_t patience, pac_tracker** out);
pac_status pac_tracker_update(pac_tracker* tracker, const uint64_t* d_mask, uint64_t n,
                              uint32_t* d_state_out, void* hip_stream);
pac_status pac_tracker_destroy(pac_tracker* tracker);

/* Weight update of paper Eq. 1 on the sparse model, fused with pac_decompress: for every set bit i,
 * d_weights[i] <- d_weights[i] - alpha * d_reduced[slot(i)] (alpha = eta / n of Eq. 1, computed by
 * the caller; one IEEE single multiply, then one subtract, each rounded to nearest; bf16 sums are
 * widened exactly; a NaN result is some NaN, its sign and payload are the hardware's); for every
 * clear bit, d_weights[i] <- +0 (the pruned weights stay zero, Eq. 2).
 * The dense gradient is never materialised.  No read at or beyond d_reduced[nnz]. */
pac_status pac_decompress_update(pac_ctx* ctx, const void* d_reduced, pac_dtype dtype, uint64_t nnz,
                                 const uint64_t* d_mask, const uint32_t* d_prefix, float alpha,
                                 float* d_weights, uint64_t n, void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Ternary payload (paper Sec. III-D: ternarize(g) quantises
 * the gradient at random into {-1, 0, +1} times a scale, unbiased in expectation, Eq. 3).  The
 * quantiser is the TernGrad one the section names: with a scale s >= max|g| shared by the workers,
 * element -> s * sign(g) * b, b ~ Bernoulli(|g| / s).  It is applied to the compact buffers; the
 * workers' ternaries are then summed as integers and scaled once.
 *   random bits  Philox4x32-10 (Salmon et al., SC'11), key = (seed, seed >> 32), counter =
 *                (j / 4, (j / 4) >> 32, stream_id, stream_id >> 32); output word j % 4 serves
 *                element j.  A worker passes its own stream_id; a step its own seed.
 *   decision     u = (word >> 8) * 2^-24; kept iff u < |g| / s (one IEEE single division)
 *   codes        0 = 0, 1 = +1, 2 = -1; element j in bits 2*(j%4).. of byte j/4; unused bits zero
 *   degenerate   a scale that is zero, negative, infinite or NaN, and NaN elements, give code 0
 * Packed buffers hold ceil(count / 4) bytes and must be 4-byte aligned.
 * ------------------------------------------------------------------------------------------ */

/* *d_scale (DEVICE float) = max |x| over the buffer, NaN elements ignored (0 for an empty buffer).
 * With accumulate != 0 the result is max(old *d_scale, max|x|): one call per worker builds the
 * shared scale (the old value must be a non-negative number). */
pac_status pac_absmax(pac_ctx* ctx, const void* d_values, pac_dtype dtype, uint64_t count, int accumulate,
                      float* d_scale_inout, void* hip_stream);

pac_status pac_ternarize(pac_ctx* ctx, const void* d_values, pac_dtype dtype, uint64_t count,
                         const float* d_scale, uint64_t seed, uint64_t stream_id, uint8_t* d_packed_out,
                         void* hip_stream);

/* d_out[j] = *d_scale * (float)(t_0[j] + ... + t_{W-1}[j]): exact integer sum, one single-precision
 * multiply, one round-to-nearest-even for a PAC_BF16 output.  h_d_packed is a HOST array of W device
 * pointers, read before the call returns.  1 <= W <= PAC_MAX_WORKERS. */
pac_status pac_ternary_reduce_local(pac_ctx* ctx, const uint8_t* const* h_d_packed, uint32_t W, uint64_t count,
                                    const float* d_scale, pac_dtype out_dtype, void* d_out, void* hip_stream);

/* Test hook: lower the number of undecided elements pac_build_mask lists between its selection passes
 * (elements in total; each 4096-element tile gets its share, at most 128).  Tiles whose undecided
 * elements do not fit are re-read from the weights by the later passes; results are identical.
 * Exists so that tests can reach that branch with small inputs. */
pac_status pac_debug_set_candidate_capacity(pac_ctx* ctx, uint64_t capacity);

/* Test hook: the number of polls after which a workgroup of the prefix scan stops waiting for an
 * earlier tile (default 2^22; 0 = give up on the first value that is not there yet).  A workgroup that
 * gives up still finishes normally and raises PAC_DEV_SCAN_STALLED.  Exists so that a test can see
 * that flag without a kernel that hangs. */
pac_status pac_debug_set_scan_spin_limit(pac_ctx* ctx, uint32_t polls);

#ifdef __cplusplus
}
#endif
#endif /* PACTRAIN_H */
