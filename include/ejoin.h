/*
 * ejoin -- brute-force Euclidean-distance epsilon self-join on AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "Fast and Scalable Mixed Precision Euclidean Distance Calculations
 * Using GPU Tensor Cores" (arXiv 2508.21230): every pair of points of a data set is compared,
 * and the pairs whose Euclidean distance is <= epsilon are returned (Section 2.1, Eq. 1;
 * Section 2.2.1 "Scenario 1").  The distance is evaluated in the expanded form
 *     dist^2(p_i, p_j) = s_i + s_j - 2 a_ij ,   s_i = sum_k p_ik^2 ,   a_ij = sum_k p_ik p_jk
 * (Section 3.1, Steps 1-3) with FP16 inputs and FP32 accumulation on the matrix cores.
 *
 * Conventions shared by all calls
 *   - Every pointer below except `ejoin_ctx**`, `ejoin_ctx*`, `float* ms` and the strings is a
 *     DEVICE pointer owned by the caller.  The library never frees or reallocates them.
 *   - X holds FP16 bit patterns, row-major: point i occupies X[i*ld .. i*ld + d - 1].
 *     `ld` (elements) must be a multiple of 64 and >= d rounded up to a multiple of 64; the
 *     columns d .. roundup(d,64)-1 must hold zeros (the paper pads d to a multiple of 64 with
 *     zeros, Section 4.2).  X must be 128-byte aligned (Section 3.3.6: each point 128 B aligned).
 *     Values must be finite.
 *   - 1 <= n < 2^32 - 256, 1 <= d <= 65536.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work and return;
 *     results are valid once the caller has synchronised the stream.  A call must not overlap
 *     another call on the same context.
 *   - Return value: EJOIN_OK or a negative error code; nothing is enqueued on error.
 *   - The squared distance the library works with is, in FP32,
 *         acc' = a_ij - s_i/2 - s_j/2,    d2 = max(0, -2 acc'),    pass  <=>  acc' >= -fl(eps * eps) / 2,
 *     where a_ij and s_i are accumulated over k in ascending order on the matrix cores in steps
 *     of 32 coordinates, and the two norm terms are added by one more matrix-core step (Step 3 of
 *     Section 3.1 folded into the accumulation).  The self pair (i, i) is always reported, with
 *     d2 = 0.  Duplicates of a point are at distance exactly 0 whenever the point's s_i is at least
 *     max(2^-16 s_max, 2^-14), s_max the largest s of the data (the norm term is then carried exactly;
 *     below that it is carried to about 2^-41 s_max).  "<= epsilon" is the paper's comparison
 *     (Section 2.2.1).
 *   - Data range: every s_i = sum_k x_ik^2 must be finite and below 2^31 (the paper's method
 *     assumes data commensurate with the FP16 range, Section 4.5).  This is detected on the
 *     device: a join over data outside the range reports zero pairs / zero counts and
 *     ejoin_status returns a non-zero status.
 */
#ifndef EJOIN_H
#define EJOIN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EJOIN_OK 0
#define EJOIN_EINVAL (-1)       /* null pointer, size out of range, misaligned X or ld */
#define EJOIN_EUNSUPPORTED (-2) /* device is not gfx950 / shape outside the supported range */
#define EJOIN_EHIP (-3)         /* a HIP runtime call failed; see ejoin_last_hip_error */
#define EJOIN_ENOMEM (-4)       /* the context's workspace could not be allocated */
#define EJOIN_ESCRATCH (-5)     /* ejoin_selfjoin_pairs_noalloc: the problem does not fit the static scratch */

typedef struct ejoin_ctx ejoin_ctx;

/* Create a context on HIP device `device`.  The context owns a few hundred bytes of device
 * status words and a workspace: 20 bytes per point (the norms s_i and their FP16 split) plus, for
 * the join calls, a re-laid-out copy of X (roundup(n,256) * (roundup(d,64) + 32) * 2 bytes).  The workspace
 * is grown on demand with hipMalloc, or ahead of time by ejoin_reserve.  A call that has to grow the
 * workspace frees the old one first, which waits for the device to be idle: only calls that find the
 * workspace large enough "enqueue and return".  Host pointer out. */
int ejoin_create(ejoin_ctx** out, int device);

/* Free the context and its device memory.  The caller must have synchronised its streams. */
int ejoin_destroy(ejoin_ctx* ctx);

/* Grow the workspace so that joins of up to n points in total (both sets of a two-set join
 * together) of up to d coordinates allocate nothing. */
int ejoin_reserve(ejoin_ctx* ctx, int64_t n, int32_t d);

/* Static, human-readable text for a return code. */
const char* ejoin_strerror(int code);

/* Text of the last HIP error seen by this context ("" if none). */
const char* ejoin_last_hip_error(const ejoin_ctx* ctx);

/* Ingestion: converts FP32 rows to the FP16 layout the joins take.  X32 (device, n rows of d floats,
 * row stride ld32 >= d elements) -> X16 (device, 128-byte aligned, row stride ld16: a multiple of 64,
 * >= roundup(d,64)):
 *     X16[i][k] = fp16( scale * (X32[i][k] - center[k]) ),   k < d,
 * every operation rounded to nearest even in FP32 before the final rounding to FP16; columns
 * d .. ld16-1 are set to zero (the zero padding of Section 4.2).  `center` (device, d floats) may be
 * NULL (no shift).  A shift leaves distances unchanged and a scale multiplies them by `scale` (so
 * epsilon must be scaled too); together they move the data into the part of the FP16 range where
 * its spacing is fine -- the remedy the paper suggests for data that converts badly (Section 5).
 * Values that overflow FP16 become Inf and make the join report status EJOIN_STATUS_NONFINITE. */
int ejoin_convert_f32(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, const float* center, float scale,
                      uint16_t* X16, int64_t ld16, void* stream);

/* Step 1 of Section 3.1: s[i] = sum_k x_ik^2 for i < n, FP32, written to the device array s (n floats).
 * Accumulated on the matrix cores in the same order as the Gram products of the join. */
int ejoin_norms(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float* s, void* stream);

/* Per-point neighbour counts (the quantity behind the paper's selectivity, Section 4.1.3).
 *   counts[i]     (device, n x u32, overwritten)  = #{ j != i : dist(x_i, x_j) <= eps }
 *   *total_pairs  (device, u64, overwritten)      = #{ (i, j), i < j : dist <= eps }
 * The paper's |R| is 2 * total_pairs + n and its selectivity S is 2 * total_pairs / n. */
int ejoin_selfjoin_count(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps,
                         uint32_t* counts, uint64_t* total_pairs, void* stream);

/* The result set of the self-join (Section 2.2.1): every (i, j), i < j, with dist <= eps, once,
 * plus the self pair (i, i) of every point; in no particular order, without duplicates.
 *   pairs    (device, capacity x 2 x u32): pair p is (pairs[2p], pairs[2p+1]) with i <= j
 *   dist2    (device, capacity x f32, or NULL): d2 of pair p (0 for self pairs)
 *   *n_pairs (device, u64, overwritten): number of pairs FOUND.  If it exceeds `capacity`, exactly
 *            `capacity` pairs were written and the rest dropped: run again with a larger buffer
 *            (or size it with ejoin_selfjoin_count: needed = total_pairs + n). */
int ejoin_selfjoin_pairs(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps,
                         uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream);

/* The self-join with its result returned to host memory in batches, for the end-to-end response time the paper
 * measures (Section 4.1: all overheads included, "storing the results in main memory"; result sets are returned
 * from the GPU to the host in batches).  The join is cut into `batches` launches (at most EJOIN_MAX_BATCHES; by rows
 * of 4096 x 4096-point blocks of the distance matrix, about the same work each); while launch b + 1 computes, the
 * pairs launch b found are copied to the host on a second stream.  Unlike the other calls this one BLOCKS: it
 * returns when every pair is in host memory.
 *   pairs, dist2    (device, capacity x 2 x u32 / capacity x f32 or NULL): where the kernels collect the result
 *   host_pairs, host_dist2 (HOST, same sizes; pinned memory for full copy speed; host_dist2 NULL iff dist2 NULL)
 *   *host_n_pairs   (HOST): number of pairs FOUND; if it exceeds capacity, exactly capacity pairs were returned
 * Result set and conventions otherwise as ejoin_selfjoin_pairs (same pairs, in another order). */
#define EJOIN_MAX_BATCHES 32
int ejoin_selfjoin_pairs_to_host(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps,
                                 uint32_t* pairs, float* dist2, uint64_t capacity, int32_t batches,
                                 uint32_t* host_pairs, float* host_dist2, uint64_t* host_n_pairs, void* stream);

/* For callers that cannot allocate device memory while they run -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: ejoin_selfjoin_pairs with the workspace taken from a
 * static device array of EJOIN_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU
 * the library runs on holds it from load to process end) instead of the context's workspace.  The call
 * allocates and frees nothing, whatever its arguments.  Arguments, results and conventions are those
 * of ejoin_selfjoin_pairs, and so are the results, bit for bit.  The problem must fit:
 *     256 + roundup(20 * npad, 512) + npad * (roundup(d,64) + 32) * 2  <=  EJOIN_STATIC_SCRATCH_BYTES,
 * npad = roundup(n,256) (n = 100,000 at d = 128 does; so does n = 20,000 at d = 960); otherwise
 * EJOIN_ESCRATCH is returned and nothing is enqueued.  All contexts of a GPU share the one array, which
 * keeps the last call's contents (the call clears what it needs zero): calls of this entry point that
 * overlap on one GPU race, also from different contexts or streams. */
#define EJOIN_STATIC_SCRATCH_BYTES (40u << 20)
int ejoin_selfjoin_pairs_noalloc(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps,
                                 uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream);

/* Higher-accuracy variant for FP32 data: the self-join of n FP32 rows (device, row stride ld32 >= d
 * elements, no padding or alignment required) with every coordinate carried as two FP16 numbers,
 * x ~ hi + lo, hi = fp16(x), lo = fp16(x - hi) -- 22 significant bits instead of 11, which removes the
 * FP16 conversion of the inputs as a source of error (the paper names the limited accuracy of FP16
 * inputs and possible remedies as future work, Section 5).  The inner products are taken as
 * hi.hi + lo.hi + hi.lo on the matrix cores (FP32 accumulation, 3 x the work of the FP16 join); norms,
 * threshold, result conventions, capacity / n_pairs / dist2 / counts and the data-range rule
 * (|x| <= 65504, s < 2^31) are those of ejoin_selfjoin_pairs / ejoin_selfjoin_count.  d <= 16384.
 * The workspace holds two re-laid-out copies of the split data, 12 * roundup(n,256) * roundup(d,64) bytes;
 * ejoin_reserve(ctx, 2 * n, 3 * roundup(d,64)) sizes it ahead of time. */
int ejoin_selfjoin_pairs_f32(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, float eps,
                             uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream);
int ejoin_selfjoin_count_f32(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, float eps,
                             uint32_t* counts, uint64_t* total_pairs, void* stream);

/* Two-set join: "points" P (np x d) against "query points" Q (nq x d), the general form of the
 * distance computation of Section 3.1 (fragments of points and of query points; the paper offers
 * the method as a subroutine for such searches, Section 1).  Same layout rules for P and Q as for X
 * (own row strides ldp, ldq; same d).  Result: every (i, j), i < np, j < nq, with dist(p_i, q_j) <= eps,
 * once, as pairs[2p] = i (index into P), pairs[2p+1] = j (index into Q); no symmetry is assumed and
 * there are no self pairs.  capacity / n_pairs / dist2 as for ejoin_selfjoin_pairs.
 * The data-range rule (s < 2^31) applies to both sets. */
int ejoin_join_pairs(ejoin_ctx* ctx, const uint16_t* P, int64_t np, int64_t ldp, const uint16_t* Q, int64_t nq, int64_t ldq,
                     int32_t d, float eps, uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream);

/* Counts of the two-set join:
 *   counts_p[i] (device, np x u32, overwritten) = #{ j : dist(p_i, q_j) <= eps }
 *   counts_q[j] (device, nq x u32, overwritten; may be NULL) = #{ i : dist(p_i, q_j) <= eps }
 *   *total      (device, u64, overwritten)      = number of matching (i, j) */
int ejoin_join_count(ejoin_ctx* ctx, const uint16_t* P, int64_t np, int64_t ldp, const uint16_t* Q, int64_t nq, int64_t ldq,
                     int32_t d, float eps, uint32_t* counts_p, uint32_t* counts_q, uint64_t* total, void* stream);

/* Prepared point set, for joining many batches of query points against the same points (the use as a
 * subroutine of searches the paper names, Section 1): ejoin_set_create computes the norms of X and its
 * re-laid-out copy once (work enqueued on `stream`; X may be released once that work has completed),
 * ejoin_set_join_pairs / _count then do per call only the work that depends on the query points.
 * The set owns its device memory (roundup(n,256) * (roundup(d,64) * 2 + 84) bytes) until
 * ejoin_set_destroy, which the caller invokes after synchronising, and before destroying the context.
 * Results, arguments and conventions are those of ejoin_join_pairs / ejoin_join_count with P = the set
 * (d is the set's).  A join writes a small part of the set (the norm terms, rescaled to the larger of
 * the two sets' largest norms), so calls that use the same set must not overlap.  *out is a host pointer. */
typedef struct ejoin_set ejoin_set;
int ejoin_set_create(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, void* stream, ejoin_set** out);
int ejoin_set_destroy(ejoin_set* set);
int ejoin_set_join_pairs(ejoin_ctx* ctx, ejoin_set* P, const uint16_t* Q, int64_t nq, int64_t ldq, float eps,
                         uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream);
int ejoin_set_join_count(ejoin_ctx* ctx, ejoin_set* P, const uint16_t* Q, int64_t nq, int64_t ldq, float eps,
                         uint32_t* counts_p, uint32_t* counts_q, uint64_t* total, void* stream);

/* Dense block of squared distances, for checking Steps 2-3 of Section 3.1 element by element:
 *   out[r * cols + c] = d2(i0 + r, j0 + c),  0 <= r < rows, 0 <= c < cols   (device, rows*cols f32)
 * computed with exactly the arithmetic of the join (so it is bit-identical to the dist2 the join
 * reports for the same pair).  Requires i0 + rows <= n, j0 + cols <= n. */
int ejoin_dist2_tile(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, int64_t i0, int64_t j0,
                     int32_t rows, int32_t cols, float* out, void* stream);

/* Waits for the stream of the context's last join or dense-tile call (which must still exist), reads
 * that call's status word and stores it in *status (host pointer):
 *   0 = ok, 1 = some s_i >= 2^31 (outside the supported data range), 2 = Inf/NaN in the input. */
#define EJOIN_STATUS_OK 0
#define EJOIN_STATUS_NORM_RANGE 1
#define EJOIN_STATUS_NONFINITE 2
int ejoin_status(ejoin_ctx* ctx, int* status);

/* Number of 256 x 256 output tiles the Gram kernel evaluates for n points (upper triangle,
 * diagonal included): the executed matrix-core work is 2 * 256 * 256 * roundup(d,64) FLOP per tile. */
int64_t ejoin_tiles_evaluated(int64_t n);
/* ... and for a two-set join of np x nq points (the full grid of tiles). */
int64_t ejoin_tiles_evaluated2(int64_t np, int64_t nq);

#ifdef __cplusplus
}
#endif
#endif /* EJOIN_H */
