/*
 * libtng -- the per-iteration data-parallel step of Trajectory Normalized Gradients (TNG,
 * arXiv 1901.08227) for M simulated workers on one AMD MI355X (gfx950).
 *
 * One iteration is Algorithm 1 of the paper with the normalisation of Eqs. 1-2:
 *   every worker m: local gradient g^m(w_t); normalise against the shared reference g~
 *   (v = g - g~, Eq. 1; v = g ./ g~, Eq. 2; v = (g - g~) ./ g~', the combined form given
 *   after Eq. 2; or against the worker's own scalar reference mean(g^m) 1, first entry of the
 *   list in "Reference Vectors"); scale R_m = max_d |v_d|; stochastic low-bit code of v/R_m (section
 *   "Gradient Compression"); pack;  server: decode, average over m, undo the
 *   normalisation, w <- w - eta v (Background, Eq. "qsgd"), refresh g~ from the decoded
 *   average (sections "Reference Vectors", "Convex Problems").
 *
 * General conventions
 *   - C ABI, no exceptions, no exit(); every call returns a tng_status.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library allocates no device memory: scratch space is the
 *     caller's workspace handed to tng_create.  tng_ctx is a small host object.
 *   - All device work is enqueued on the hipStream_t given to tng_create and is
 *     asynchronous; outputs are valid once the caller has synchronised that stream.
 *     Only tng_set_logreg_dense / tng_set_logreg_csr block (a small host-to-device copy).
 *   - float = IEEE binary32.  The normalise / threshold / decode arithmetic is evaluated
 *     with one rounding per operation (no fused multiply-add, subnormals kept) so that
 *     codes are reproducible bit for bit; for fixed (config, inputs, iter) the outputs of
 *     encode and decode do not depend on launch geometry or on earlier calls.
 *   - Layout: g is row-major [M][d] with row pitch d; codes is row-major [M][words] with
 *     words = tng_words_per_row(d, bits); element e of a row sits in word e / (32/bits) at
 *     bit offset (e % (32/bits)) * bits; code = level | sign << (bits-1); unused high bits
 *     of the last word are zero.  g, gref, gref2, w, vbar, noise must be 16-byte aligned,
 *     codes and scales 4-byte aligned.
 *   - Inputs are assumed finite; non-finite gradients give unspecified codes.
 *   - Errors: a NULL pointer, misalignment or an out-of-range field gives
 *     TNG_ERR_INVALID_ARG and enqueues nothing; a call that needs problem data that was
 *     not set gives TNG_ERR_BAD_STATE; a workspace smaller than tng_workspace_bytes gives
 *     TNG_ERR_WORKSPACE; a failed launch gives TNG_ERR_HIP; tng_create gives TNG_ERR_HOST_MEMORY when
 *     the host cannot hold the context.
 */
#ifndef TNG_H
#define TNG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tng_ctx tng_ctx;

typedef enum {
  TNG_OK = 0,
  TNG_ERR_INVALID_ARG = 1,
  TNG_ERR_BAD_STATE = 2,
  TNG_ERR_WORKSPACE = 3,
  TNG_ERR_UNSUPPORTED = 4,
  TNG_ERR_HIP = 5,
  TNG_ERR_TOO_LARGE = 6,
  TNG_ERR_HOST_MEMORY = 7
} tng_status;

/* How the gradient is normalised before coding (section "Normalized Gradients"). */
typedef enum {
  TNG_NORM_NONE = 0, /* v = g: zero reference, plain compressed SGD (remark after Proposition 2) */
  TNG_NORM_SUB = 1,  /* Eq. 1: v = g - g~,         decoded as g~ + r                           */
  TNG_NORM_QUOT = 2, /* Eq. 2: v = g ./ g~,        decoded as g~ (.) r                         */
  TNG_NORM_COMB = 3, /* combined: v = (g - g~) ./ g~', decoded as g~' (.) r + g~               */
  TNG_NORM_MEAN = 4  /* per-worker reference mean(g^m) 1 ("Reference Vectors", first entry):
                        v = g^m - mu_m, mu_m = float(sum_e g^m_e / d) sent along with R_m (32 more
                        bits per worker); decoded as mu_m + r per worker before averaging.  The
                        shared reference g~ is not used by the coder.                             */
} tng_norm;

/* The coder's scale R (section "Gradient Compression": R = max_d |v_d|; the same coder with the
 * l2 norm as R is the one of the QSGD/TernGrad family the section builds on). */
typedef enum {
  TNG_SCALE_MAX = 0, /* R = max_d |v_d|                                                          */
  TNG_SCALE_L2 = 1   /* R = float(sqrt(sum_d v_d^2)); |v_d| / R <= 1 still holds                  */
} tng_scale;

/* How the reference is refreshed (section "Reference Vectors"; "Convex Problems"). */
typedef enum {
  TNG_REF_ZERO = 0,    /* never: g~ keeps the caller's initial value (zeros in Algorithm 1)     */
  TNG_REF_LAST_AVG = 1, /* g~ <- decoded average of this iteration when (iter+1) % period == 0  */
  TNG_REF_WINDOW_AVG = 2 /* g~ <- mean of the last ref_window decoded averages (second entry of the
                            list of reference choices), refreshed on the same schedule            */
} tng_ref_policy;

typedef enum {
  TNG_PROB_EXTERNAL = 0,     /* caller fills g; tng_local_grad is not available                 */
  TNG_PROB_LOGREG_DENSE = 1, /* logistic regression, dense row-major features                   */
  TNG_PROB_LOGREG_CSR = 2,   /* logistic regression, CSR features                               */
  TNG_PROB_ROSENBROCK = 3    /* chain Rosenbrock function + additive noise                      */
} tng_problem;

typedef struct {
  uint64_t d;          /* dimension of w, 1 <= d <= 2^34 (CSR problem: d <= 65535 * 2^14)       */
  uint32_t M;          /* number of simulated workers, >= 1                                     */
  uint32_t bits;       /* 2: ternary {-1,0,1} x R; 4: sign + 3-bit level, 7 levels              */
  int32_t norm;        /* tng_norm                                                              */
  float quot_eps;      /* > 0: reference entries with |g~| < eps are replaced by +-eps (Eq. 2)  */
  int32_t ref_policy;  /* tng_ref_policy                                                        */
  uint32_t ref_period; /* K >= 1                                                                */
  uint64_t seed;       /* Philox key                                                            */
  float lr;            /* eta, finite                                                           */
  float l2;            /* l2 regularisation of the logistic problems, finite                    */
  uint32_t batch;      /* minibatch rows per worker (logistic problems), >= 1 there             */
  int32_t problem;     /* tng_problem                                                           */
  uint32_t ref_window; /* tau_max >= 1 of TNG_REF_WINDOW_AVG (ignored by the other policies)            */
  int32_t scale;       /* tng_scale                                                             */
} tng_config;

/* ceil(d * bits / 32); 0 if bits is not 2 or 4. */
uint64_t tng_words_per_row(uint64_t d, uint32_t bits);

/* Device scratch bytes tng_create needs for this configuration; 0 if the configuration is invalid.
 * (For 2-bit codes with the largest-magnitude scale and TNG_NORM_NONE / TNG_NORM_SUB over 2^26 elements or
 * more, d a multiple of 1024, this includes M * d / 2 bytes: tng_normalize_encode then reads g once and
 * keeps the few elements that can code non-zero there between its two passes; same codes, bit for bit.) */
size_t tng_workspace_bytes(const tng_config* cfg);

/* Creates a context.  cfg: host.  workspace: device, 256-byte aligned, at least
 * tng_workspace_bytes(cfg) bytes, owned by the caller and kept alive until tng_destroy.
 * hip_stream: a hipStream_t (NULL = the default stream).  *out receives the context. */
tng_status tng_create(const tng_config* cfg, void* workspace, size_t workspace_bytes,
                      void* hip_stream, tng_ctx** out);
tng_status tng_destroy(tng_ctx* ctx);
const char* tng_status_string(tng_status s); /* static storage */

/* Problem data (Background: worker m holds its own shard Omega_m).  X, y, rowptr, col, val:
 * host arrays of M device pointers; n_rows: host array of M row counts (1 <= n < 2^32).
 * Dense shards are row-major [n_rows[m]][d], 16-byte aligned; labels are 0/1 floats.
 * CSR: rowptr int64[n_rows+1], col int32 in [0, d) ascending within each row, fewer than 2^32
 * entries per row, val float.  The device data must outlive
 * the context or the next tng_set_* call.  These two calls copy the pointer tables into the
 * workspace and block until that copy is done. */
tng_status tng_set_logreg_dense(tng_ctx* ctx, const float* const* X, const float* const* y,
                                const uint64_t* n_rows);
tng_status tng_set_logreg_csr(tng_ctx* ctx, const int64_t* const* rowptr,
                              const int32_t* const* col, const float* const* val,
                              const float* const* y, const uint64_t* n_rows);
/* The same shards with the stored entries of a row as (column, value) pairs in one array instead of two
 * parallel arrays: entries[m] is a device array of tng_csr_entry, 8-byte aligned, entry k of row i at
 * rowptr[i] + k, columns ascending within each row as above.  The gradient kernels read the entries of a
 * row in short runs (the part of the row that falls into one column tile); with pairs such a run is one
 * contiguous piece of memory instead of two, which is what their speed depends on: prefer this layout
 * (faster per iteration at d = 2^24, 0.1 % density).  The two layouts give the same results.
 * Everything said for tng_set_logreg_csr applies. */
typedef struct {
  int32_t col;
  float val;
} tng_csr_entry;
tng_status tng_set_logreg_csr_pairs(tng_ctx* ctx, const int64_t* const* rowptr, const tng_csr_entry* const* entries,
                                    const float* const* y, const uint64_t* n_rows);
/* Optional, CSR problem: checks the shards given to the last tng_set_logreg_csr against what the
 * gradient kernels assume and cannot check on the hot path: row pointers non-negative and
 * non-decreasing, ending within the nnz[m] entries stored for worker m (nnz: host array of M counts =
 * the lengths of the col / val arrays), fewer than 2^32 entries per row; column ids in [0, d) and
 * strictly ascending within each row.  One pass over the row pointers and, only if they are sound, one
 * over the column ids; blocks until done.  TNG_OK, or TNG_ERR_INVALID_ARG if any check fails (the
 * kernels index on-chip tiles with col - tile start: shards that fail must not be used). */
tng_status tng_validate_csr(tng_ctx* ctx, const uint64_t* nnz);
/* Optional, CSR problem: a per-row index of where each stored row enters each column tile of the
 * gradient kernels (the columns are processed in tiles of 2^14 coordinates held in on-chip memory).
 * Without it every tng_local_grad / tng_step re-derives these offsets with a pass over the column ids
 * of its minibatch rows; with it that pass becomes a small gather.  The index depends on the shards
 * only, costs 4 (ceil(d / 2^14) + 1) bytes per row (about 3 % of a row at 0.1 % density) and is built
 * once: tng_set_csr_index enqueues the build on the context's stream for the shards given to the last
 * tng_set_logreg_csr (a later tng_set_logreg_csr drops it).  index: device, 256-byte aligned, at least
 * tng_csr_index_bytes(cfg, n_rows) bytes (0 = not available for this configuration: not the CSR
 * problem, or a shard of 2^31 rows or more), owned by the caller and kept alive while it is in use. */
size_t tng_csr_index_bytes(const tng_config* cfg, const uint64_t* n_rows);
tng_status tng_set_csr_index(tng_ctx* ctx, void* index, size_t bytes);
/* Rosenbrock: additive noise of the coming iteration, device [M][d], or NULL for none
 * ("Nonconvex Problems": the stochastic gradient is the exact gradient plus Gaussian noise). */
tng_status tng_set_noise(tng_ctx* ctx, const float* noise);
/* Rosenbrock: Gaussian noise N(0, variance) made on the device instead of read from a tensor
 * (variance > 0; 0 switches it off; the later of tng_set_noise / tng_set_noise_variance wins).
 * Element e of worker m at iteration iter is sigma * z with sigma = sqrtf(variance) and z from the
 * Box-Muller transform of the Philox4x32-10 block with counter (e >> 2, m, iter, 2): output words 0, 1
 * serve e & 3 = 0 (cosine branch) and 1 (sine branch), words 2, 3 serve e & 3 = 2 and 3;
 * u1 = ((word >> 8) + 1) 2^-24, u2 = (word >> 8) 2^-24, z = sqrt(-2 ln u1) {cos, sin}(2 pi u2).
 * Evaluated in binary32 (a few units in the last place of the float64 value; not bit-pinned). */
tng_status tng_set_noise_variance(tng_ctx* ctx, float variance);
/* History of TNG_REF_WINDOW_AVG: device [ref_window][d], zero-filled by the caller before the first
 * iteration (missing history counts as zeros) and then owned by the library: the decoded average of
 * iteration iter is kept in slot iter % ref_window.  Must be set before tng_update_reference / tng_step. */
tng_status tng_set_reference_history(tng_ctx* ctx, float* history);
/* Second reference g~' of TNG_NORM_COMB, device [d]; must be set before encode / decode. */
tng_status tng_set_second_reference(tng_ctx* ctx, const float* gref2);
/* Per-worker means of TNG_NORM_MEAN, device float[M], 4-byte aligned, owned by the caller: written
 * by tng_normalize_encode (and the encode part of tng_step), read by tng_decode_aggregate; the third
 * array, next to codes and scales, that travels from the workers to the server.  Must be set before
 * encode / decode / step in that mode.
 * Sums over a row (this mean, and the l2 scale) are taken in binary64 in a fixed order, so that their
 * float32 rounding is reproducible: chunks of 4096 elements; inside a chunk 256 lanes, lane j adding
 * elements 256 k + j for k = 0..15 in order, then the lanes in order; chunk sums in order inside
 * groups of 256 chunks; group sums in order. */
tng_status tng_set_worker_means(tng_ctx* ctx, float* means);

/* Raw 32-bit draws first .. first+count-1 of the sequence (seed, iter, worker, stream) of the
 * counter-based generator Philox4x32-10 (Salmon et al., SC'11): draw j is output word j & 3 of
 * the block with counter (j >> 2, worker, iter, stream) and key (seed low, seed high).
 * Stream 0 feeds the rounding decisions (element e of worker m uses draw e), stream 1 the
 * minibatch row ids.  out: device uint32[count]. */
tng_status tng_rng_draws(tng_ctx* ctx, uint32_t iter, uint32_t worker, uint32_t stream,
                         uint64_t first, uint64_t count, uint32_t* out);

/* Minibatch row ids of iteration iter, idx[m][j] = (draw_j * n_rows[m]) >> 32, uniform with
 * replacement (Background: "uniformly sampled").  idx: device uint32[M][batch]. */
tng_status tng_minibatch_indices(tng_ctx* ctx, uint32_t iter, uint32_t* idx);

/* Algorithm 1, local gradient of every worker at w.  w: device [d]; g: device [M][d] (out).
 * Logistic problems: g_m = (1/B) sum_{i in batch_m(iter)} (sigma(x_i . w) - y_i) x_i + l2 w.
 * Rosenbrock: g_m = grad f(w) + noise_m, f(x) = sum_i 100 (x_{i+1} - x_i^2)^2 + (1 - x_i)^2. */
tng_status tng_local_grad(tng_ctx* ctx, uint32_t iter, const float* w, float* g);

/* Workers' side of Algorithm 1 (normalise, R_m, sample, pack).  g: device [M][d]; gref: device
 * [d] (ignored, may be NULL, for TNG_NORM_NONE); codes: device [M][words] (out); scales:
 * device [M] (out), scales[m] = R_m of worker m (max_d |v_d|, or the l2 norm for TNG_SCALE_L2),
 * taken as 0 below FLT_MIN. */
tng_status tng_normalize_encode(tng_ctx* ctx, uint32_t iter, const float* g, const float* gref,
                                uint32_t* codes, float* scales);

/* tng_normalize_encode for callers that cannot allocate device memory or hold a context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same kernels, same
 * outputs, bit for bit, as tng_normalize_encode of a context created from *cfg; what that call keeps in
 * the caller's workspace (the per-workgroup partial maxima of the scale pass) lives in a fixed 1 MiB
 * array in device memory inside the library, which every GPU the library has run on holds until the
 * process ends.  No hipMalloc / hipFree, no context, no workspace; the first call on a device looks up
 * the array's address there.
 *   cfg: host; only d, M, bits, norm, quot_eps, seed are used (the rest must still be valid).
 *   hip_stream: a hipStream_t of the current device (NULL = the default stream); the call is asynchronous.
 *   g, gref, codes, scales: device, as for tng_normalize_encode.
 * Limits: M <= 64 (TNG_ERR_TOO_LARGE beyond); scale = TNG_SCALE_MAX and norm in {NONE, SUB, QUOT}
 * (TNG_ERR_UNSUPPORTED otherwise: the other modes need a second reference, per-worker means or the
 * ordered-sum scratch).  All calls on one GPU share the one array: calls that overlap in time on the
 * same GPU (different streams, different threads) race; calls on one stream are safe.  Nothing in the
 * array has to be cleared between calls. */
tng_status tng_normalize_encode_static(const tng_config* cfg, void* hip_stream, uint32_t iter, const float* g,
                                       const float* gref, uint32_t* codes, float* scales);

/* Server's side: vbar[e] = denorm( (sum_m decode(codes[m][e]) in worker order) * (1/M) ).
 * codes, scales, gref as above; vbar: device [d] (out). */
tng_status tng_decode_aggregate(tng_ctx* ctx, const uint32_t* codes, const float* scales,
                                const float* gref, float* vbar);

/* Reference rule.  TNG_REF_LAST_AVG: if (iter+1) % ref_period == 0, gref <- vbar, else no-op.
 * TNG_REF_WINDOW_AVG: history[iter % ref_window] <- vbar at every iteration, and on a refresh
 * iteration gref <- (sum of the ref_window slots, oldest first) * (1 / ref_window).  TNG_REF_ZERO: no-op. */
tng_status tng_update_reference(tng_ctx* ctx, uint32_t iter, const float* vbar, float* gref);

/* One whole iteration: local_grad (unless TNG_PROB_EXTERNAL, where g is an input),
 * normalize_encode, decode_aggregate, w <- w - lr * vbar, update_reference.
 * w, gref: device [d], updated in place; g, codes, scales, vbar: device, as above. */
tng_status tng_step(tng_ctx* ctx, uint32_t iter, float* w, float* gref, float* g,
                    uint32_t* codes, float* scales, float* vbar);

/* Timing hook for benchmarks and profilers (no counterpart in the paper).  events: host array of
 * 5 * slots hipEvent_t created by the caller with timing enabled, or NULL to switch the hook off;
 * the array is copied.  Encode call number c (tng_normalize_encode or the encode part of tng_step,
 * counted from this call on) records, on the context's stream, events[5 (c % slots) + 0] before
 * the scale pass, + 1 between the scale pass and the quantise pass, + 2 after the quantise pass;
 * decode call number c records + 3 before and + 4 after the decode kernel.  The events stay owned
 * by the caller and must outlive the calls that record them. */
tng_status tng_set_profile_events(tng_ctx* ctx, void* const* events, uint32_t slots);

#ifdef __cplusplus
}
#endif
#endif /* TNG_H */
