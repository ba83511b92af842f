/*
 * lgreco.h - C ABI of the MI355X-native L-GreCo hot path (liblgreco.so).
 *
 * L-GreCo (layer-wise adaptive gradient compression) picks, for every layer of a model,
 * one compression parameter out of a candidate list so that the total compressed size is
 * minimal while the total squared-L2 compression error stays below the error of a uniform
 * default setting (paper: sections "Problem Setup" and "The L-GreCo Framework",
 * Algorithm 1).  This library is the data-parallel hot path of that method on one GPU:
 *
 *   lgreco_profile   error(l, c) and size(l, c) for every layer l and candidate c
 *                    (Algorithm 1: the Costs and Errors matrices; "Implementation":
 *                    simulated compress -> decompress, squared L2 distance)
 *   lgreco_emax      E_max = total error of the uniform default (Algorithm 1, step 2)
 *   lgreco_solve     the layer x discretised-error dynamic program and its back-trace
 *                    (Algorithm 1, the DP and PD tables)
 *   lgreco_profile_solve  the three calls above as one, without a host round trip between
 *                    the profile's kernels and the solver's
 *   lgreco_compress  apply the chosen per-layer setting, produce the payload and update
 *                    the error-feedback buffer (what the paper's communication engine does
 *                    with the mapping, section "Implementation")
 *
 * Three compression families (section "Experimental Validation"): bucketed quantization
 * with b bits per value, layer-wise Top-K with density d, PowerSGD-style low rank with rank r.
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers (HIP global memory on the current device);
 *     every other pointer is HOST memory.  The caller owns all of them.  The handle owns
 *     only scratch memory sized at lgreco_create().
 *   - All kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream).  Host outputs are valid when the call returns (the call waits for them, not
 *     necessarily for the stream to drain); a call without host outputs (lgreco_compress) does
 *     not wait.  Calls on one handle must not
 *     overlap: use one stream per handle, or order the streams yourself.
 *   - Every function returns an lgreco status: 0 on success, negative on error.  Nothing
 *     throws, nothing prints.  Inputs must be finite; NaN/Inf gradients give undefined
 *     numerical results (never a fault).
 *   - Gradients of all layers live in one flat fp32 buffer; layer l is the range
 *     [offset, offset + numel).  Ranges must not overlap.  16-byte aligned layer starts
 *     (offset % 4 == 0 with a 16-byte aligned buffer) take the fast path; other offsets work
 *     through a slower path.
 */
#ifndef LGRECO_H
#define LGRECO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LGRECO_OK            0
#define LGRECO_EINVAL       (-1)  /* null pointer, negative/zero size, unknown family, bad layer table */
#define LGRECO_ENOSPACE     (-2)  /* exceeds the limits given to lgreco_create */
#define LGRECO_EINFEASIBLE  (-3)  /* no assignment fits the error budget */
#define LGRECO_EHIP         (-4)  /* HIP runtime error (text via lgreco_last_hip_error) */
#define LGRECO_EUNSUPPORTED (-5)  /* valid request this build does not implement */

#define LGRECO_QUANT   0   /* param = bits per value, integer in [1, 8] */
#define LGRECO_TOPK    1   /* param = density in (0, 1] */
#define LGRECO_LOWRANK 2   /* param = rank, integer in [1, r_max] */

#define LGRECO_MAX_CANDS 128
#define LGRECO_MAX_BINS  16384

typedef struct lgreco_handle lgreco_handle_t;

/* One layer of the flat gradient buffer.  rows*cols == numel gives the matrix view used by
 * LOWRANK (rows = first tensor dimension, cols = product of the others, row-major);
 * rows == 0 marks a tensor with no matrix view (LOWRANK candidates are then rejected). */
typedef struct {
    int64_t offset;   /* first element in the flat buffer */
    int64_t numel;    /* > 0, < 2^31 */
    int32_t rows;
    int32_t cols;
} lgreco_layer_t;

typedef struct {
    int32_t family;   /* LGRECO_QUANT | LGRECO_TOPK | LGRECO_LOWRANK */
    int32_t reserved; /* must be 0 */
    double  param;
} lgreco_cand_t;

typedef struct {
    int32_t  bucket;       /* quantization bucket size in elements; this build: 128 */
    int32_t  stochastic;   /* 0: round to nearest (floor(t + 0.5)); 1: floor(t + u), u from
                              Philox4x32-10 keyed by seed with counter (index/4, layer) */
    uint64_t seed;
    int32_t  power_iters;  /* LOWRANK power-iteration steps per call (appendix "Low-rank error
                            * computation", "Power Iteration Steps"): 1..16; every step is P = XQ, Phat = orth(P),
                            * Q = X^T Phat, with Q feeding the next step */
    int32_t  r_max;        /* columns of the warm-start Q per layer; this build: <= 64 */
    int32_t  reuse_thresholds; /* TOPK: 1 = a call with the same layer table and the same k as the
                            * previous call of its kind (profile / compress) starts its single
                            * pass from the thresholds found then, a margin lower, instead of
                            * sampling the data first.  Results do not depend on it: a layer
                            * whose data moved past the margin is collected again. */
    int32_t  dp_groups;    /* solver: 0 = decide per solve from its size; 1 = always one sequential
                            * sweep; 2, 4, 8 = sweep the layers in that many groups side by side and
                            * join the groups' tables (results are the same in every case,
                            * Algorithm 1's tie-breaks included) */
    int32_t  strict_budget; /* solver: 0 = Algorithm 1's constraint on the discretised errors, sum of
                            * bins <= n_bins, under which the real errors may exceed e_max by up to
                            * L steps (see lgreco_solve); 1 = only assignments whose bins sum to at
                            * most n_bins - L are accepted, which keeps the sum of the real errors
                            * below e_max (section "The Constrained Optimization Problem") */
    int32_t  keep_ef_on_failure; /* lgreco_profile_solve_compress with quantization / Top-K candidates
                            * only: 0 = the profile leaves x = fl32(g + e) in d_ef as it forms it and
                            * the compression reads x there (less memory traffic: g is read once,
                            * and the Top-K layers are compressed from the candidates the profile
                            * recorded, with no further pass over their data); a
                            * call that fails after its profile ran then leaves d_ef = x.  1 = d_ef
                            * is written by the compression only and is untouched when the call
                            * fails.  Results of a successful call are the same either way. */
} lgreco_config_t;

/* Create a handle for problems of at most max_elems gradient elements (sum of numel),
 * max_layers layers and max_cands candidates.  Allocates the scratch memory on the current
 * device (about 16 bytes per element of max_elems for the Top-K candidate buffers, the rest is
 * small beside it; the low-rank buffers grow with the first call that needs them); the handle
 * must be used on that device only, by one thread at a time. */
int lgreco_create(lgreco_handle_t** out, const lgreco_config_t* cfg, int64_t max_elems,
                  int32_t max_layers, int32_t max_cands);
int lgreco_destroy(lgreco_handle_t* h);

/* size(l, c) in bytes, host arithmetic only (Algorithm 1, the Costs matrix):
 *   QUANT   sum over the layer's buckets of ceil(count*bits/8) + 8   (codes + fp32 min, unit)
 *   TOPK    8*k, k = min(n, max(1, floor(d*n + 0.5)))               (fp32 value + u32 index)
 *   LOWRANK 4*(rows + cols)*r
 * sizes is [L x P] row-major. */
int lgreco_sizes(const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                 int32_t bucket, int64_t* sizes);

/* Profile: errors[l][c] = || C_c(x) - x ||^2 with x = fl32(g + e) for every layer and
 * candidate, the squared L2 distance between the vector and its compress -> decompress image
 * (section "Implementation"; additive over layers, section "The Constrained Optimization
 * Problem").  The error-feedback buffer is read, never updated.
 *   d_grads  fp32 flat gradient buffer, read only
 *   d_ef     fp32 error-feedback buffer of the same layout, or NULL (= zeros)
 *   d_q0     LOWRANK only (else NULL): warm-start Q of every layer, fp32, layer l at element
 *            offset r_max * (sum of cols of layers before l), [cols x r_max] row-major; rank r
 *            uses its first r columns
 *   errors   host [L x P] row-major, fp64
 *   sizes    host [L x P] row-major, bytes, or NULL to skip */
int lgreco_profile(lgreco_handle_t* h, const float* d_grads, const float* d_ef,
                   const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                   const float* d_q0, double* errors, int64_t* sizes, void* stream);

/* Candidate list from a default parameter, the rule of the paper's experiments (section
 * "Experimental setup", "Parameter ranges"): bits and ranks [D/2, 2 D] in steps of 1 (D/2
 * rounded down, at least 1; bits at most 8, ranks at most r_max when r_max > 0), densities
 * [D/10, 10 D] in steps of D/10 (at most 1).  Host arithmetic.
 *   cands          receives up to cap candidates in increasing parameter order
 *   count          number of candidates of the range (LGRECO_ENOSPACE if it exceeds cap)
 *   default_index  position of the default parameter in the list (may be NULL) */
int lgreco_candidate_range(int32_t family, double default_param, int32_t r_max,
                           lgreco_cand_t* cands, int32_t cap, int32_t* count,
                           int32_t* default_index);

/* E_max: sum over layers, in layer order, of errors[l][default_cand] (Algorithm 1, step 2;
 * section "The Error Bound").  Host arithmetic. */
int lgreco_emax(const double* errors, int32_t L, int32_t P, int32_t default_cand, double* e_max);

/* Solve: minimise sum size(l, c_l) subject to sum bin(l, c_l) <= n_bins, where
 * bin = floor((error * n_bins) / e_max) in fp64 (discretisation step e_max / n_bins,
 * section "The L-GreCo Framework"); candidates with bin > n_bins are unusable.  The table is
 * swept layer by layer with a strict '<' over candidates in index order and the back-trace
 * starts from the lowest-error minimum of the last row (Algorithm 1).
 *   choice       host [L]: candidate index per layer
 *   total_size   sum of the chosen sizes (may be NULL)
 *   total_error  sum of the chosen real errors (may be NULL)
 * The constraint is on the discretised errors: every bin rounds its error down by less than one
 * step, so an assignment the solver accepts has total_error < e_max * (1 + L / n_bins), not
 * total_error <= e_max.  The return value is still LGRECO_OK then (the paper's algorithm accepts
 * the same assignments); a caller that needs total_error <= e_max creates the handle with
 * strict_budget = 1: the bins of an accepted assignment then sum to at most n_bins - L.  That
 * tighter budget may leave no assignment (LGRECO_EINFEASIBLE) where the plain one has some;
 * lgreco_profile_solve and lgreco_profile_solve_compress, which know the uniform default, return
 * the default then (its total error is e_max itself).
 * Returns LGRECO_EINFEASIBLE if no assignment fits; choice then holds each layer's
 * minimum-error candidate.  n_bins <= LGRECO_MAX_BINS. */
int lgreco_solve(lgreco_handle_t* h, const double* errors, const int64_t* sizes, int32_t L,
                 int32_t P, double e_max, int32_t n_bins, int32_t* choice, int64_t* total_size,
                 double* total_error, void* stream);

/* Solve with the time-based objective: minimise sum size(l, c_l) * T(l) under the same
 * constraint (section "Time optimization": per-bucket coefficients T applied to the layers of
 * the bucket; appendix "Buckets prioritization": T = index of the bucket the layer travels in).
 * The coefficients are non-negative integers, so the table stays exact: a caller with real
 * regression coefficients scales and rounds them.  Everything else is as in lgreco_solve,
 * with size * T in place of size, tie-breaks included.
 *   weights     host [L], 0 <= T(l); every size(l,c) * T(l) must stay below 2^45
 *   total_size  sum of the chosen sizes in bytes, unweighted (may be NULL)
 *   total_cost  sum of the chosen size * T (may be NULL) */
int lgreco_solve_weighted(lgreco_handle_t* h, const double* errors, const int64_t* sizes,
                          const int64_t* weights, int32_t L, int32_t P, double e_max,
                          int32_t n_bins, int32_t* choice, int64_t* total_size,
                          int64_t* total_cost, double* total_error, void* stream);

/* lgreco_emax + lgreco_solve for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  No handle: every intermediate
 * table (candidate lists, the arg-min table PD) lives in one array in the library's device image,
 * LGRECO_STATIC_MAX_PD_BYTES + 82432 bytes (4.08 MiB) per GPU the library runs on, held until the
 * process ends.  The call allocates nothing, copies nothing to or from the host and does not wait:
 * its three kernels are queued on `stream` and the outputs are complete in stream order.
 *   d_errors      device [L x P] fp64, row-major, 16-byte aligned (e.g. the table a profile left)
 *   d_sizes       device [L x P] int64 bytes, 16-byte aligned; every size in [0, 2^30) and the sum
 *                 over layers of each layer's largest size below 2^30 (else d_result[0] = 3)
 *   default_cand  E_max = sum over layers, in layer order, of d_errors[l][default_cand]
 *   d_choice      device out [L]: candidate per layer; each layer's minimum-error candidate when
 *                 no assignment fits; -1 on invalid input
 *   d_result      device out [4] int64: [0] 0 ok, 1 no assignment fits the budget, 2 internal
 *                 inconsistency, 3 invalid table (a NaN, a size out of range); [1] total size;
 *                 [2] bit pattern of the fp64 total error; [3] bit pattern of the fp64 E_max
 * Limits (beyond them: LGRECO_ENOSPACE, nothing queued): L <= 1024, P <= 16, L * P <= 4096,
 * n_bins <= LGRECO_MAX_BINS and L * ((n_bins + 4) & ~3) <= LGRECO_STATIC_MAX_PD_BYTES.
 * Results equal lgreco_emax + lgreco_solve on the same tables, tie-breaks included.  All calls on
 * one GPU share that GPU's array: calls that overlap in time on one GPU (different streams
 * without ordering, several threads) race.  The array keeps the last call's contents; the call
 * rewrites every word it later reads, nothing needs clearing. */
#define LGRECO_STATIC_MAX_PD_BYTES (4 << 20)
int lgreco_solve_static(const double* d_errors, const int64_t* d_sizes, int32_t L, int32_t P,
                        int32_t default_cand, int32_t n_bins, int32_t* d_choice, int64_t* d_result,
                        void* stream);

/* lgreco_profile, lgreco_emax and lgreco_solve in one call (Algorithm 1 from the Errors matrix to
 * the traced-back assignment): the solve follows the profile on the stream without the host round
 * trip in between - E_max, the discretised errors and the solver's candidate lists are formed on
 * the device from the error table the profile kernels just wrote.  Arguments as in the three
 * calls; results are the same as theirs, tie-breaks included.
 *   default_cand  candidate index whose uniform use defines E_max
 *   errors        host out [L x P] (required)
 *   sizes         host out [L x P] (required here: the solver needs them)
 *   e_max         host out (required)
 *   choice        host out [L]
 * Returns LGRECO_EINFEASIBLE with the minimum-error choice as lgreco_solve does.  Problems the
 * device-side step does not take (more than 1024 layers, more than 16 candidates, more than 4096
 * table entries, total size of 2^30 bytes or more) go through the three calls internally. */
int lgreco_profile_solve(lgreco_handle_t* h, const float* d_grads, const float* d_ef,
                         const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands,
                         int32_t P, const float* d_q0, int32_t default_cand, int32_t n_bins,
                         double* errors, int64_t* sizes, double* e_max, int32_t* choice,
                         int64_t* total_size, double* total_error, void* stream);

/* Byte offset of every layer's payload for a given choice, host arithmetic only.
 * offsets has L+1 entries; layer l's payload is [offsets[l], offsets[l] + size(l, choice[l]))
 * and offsets[L] is the buffer size to allocate.  Layer starts are rounded up to 16 bytes. */
int lgreco_payload_layout(const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands,
                          int32_t P, const int32_t* choice, int32_t bucket, int64_t* offsets);

/* Compress every layer with its chosen candidate.
 *   d_ef       in: error feedback e; out: e' = x - decompress(compress(x)), x = fl32(g + e).
 *              Required (not NULL).
 *   d_q        LOWRANK only (else NULL): in: warm-start Q (layout as d_q0); out: the first r
 *              columns of each layer's block hold the new Q (next warm start)
 *   d_payload  out, layouts:
 *     QUANT   per bucket (fp32 min, fp32 unit) for all buckets, then each bucket's codes as
 *             an LSB-first bit stream (element i at bits [i*b, (i+1)*b)) padded to a byte
 *     TOPK    fp32 values[k] then uint32 indices[k] (index within the layer), ascending
 *             index; among equal magnitudes the lower index is kept
 *     LOWRANK Phat [rows x r] then Q [cols x r], fp32 row-major
 *   offsets    host [L+1] from lgreco_payload_layout
 * The call has no host output and returns with its kernels queued on `stream`: d_payload, d_ef
 * and d_q are complete in stream order (for the next call on this stream, or after the caller
 * waits on the stream).  The host arrays are read before the call returns.  An error of the
 * queued work surfaces at the next call that waits.  A call whose layer table, choice or offsets
 * differ from the previous call's uploads them first and waits for that copy, hence for whatever
 * was queued on `stream` before it; a loop that repeats them does not wait. */
int lgreco_compress(lgreco_handle_t* h, const float* d_grads, float* d_ef,
                    const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                    const int32_t* choice, float* d_q, uint8_t* d_payload, const int64_t* offsets,
                    void* stream);

/* One pass of the whole path as one call: lgreco_profile_solve, lgreco_payload_layout and
 * lgreco_compress with the choice just found (Algorithm 1 followed by the step that applies its
 * result, section "Implementation"), so that no time passes in the caller between the solver's
 * result and the compression kernels.  Arguments as in those calls, except:
 *   d_ef      required: read by the profile, then updated by the compression
 *   d_q       LOWRANK (else NULL): warm start of the profile, then in/out of the compression
 *   d_payload device buffer of payload_capacity bytes; the layout depends on the choice, so it must
 *             hold the largest total any choice gives (sum over layers of the largest size, plus
 *             16 bytes of padding per layer); a choice that does not fit: LGRECO_ENOSPACE, nothing
 *             compressed
 *   offsets   host out [L+1], the layout used
 * Host outputs of the profile and the solve are valid on return; the compression kernels are
 * queued as with lgreco_compress.  LGRECO_EINFEASIBLE: as lgreco_solve, nothing compressed.
 * Whenever nothing is compressed (a failed solve, a payload buffer too small, a table that is not
 * finite) d_ef holds either what it held before or, with keep_ef_on_failure = 0 and no low-rank
 * candidate, x = fl32(g + e): the gradient an uncompressed step would send, with the error
 * feedback already added.
 * With quantization and Top-K candidates in one list part of the compression is queued on a
 * stream the handle owns (default priority); it starts behind the solver's kernel on `stream` and
 * `stream` waits for it before the call returns, so for the caller everything is in `stream`'s
 * order as before. */
int lgreco_profile_solve_compress(lgreco_handle_t* h, const float* d_grads, float* d_ef,
                                  const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands,
                                  int32_t P, float* d_q, int32_t default_cand, int32_t n_bins,
                                  double* errors, int64_t* sizes, double* e_max, int32_t* choice,
                                  int64_t* total_size, double* total_error, uint8_t* d_payload,
                                  int64_t payload_capacity, int64_t* offsets, void* stream);

/* Receiver side of the codec: turn the payloads written by lgreco_compress (same layer table,
 * candidate list, choice and offsets) back into dense gradients, the step that follows the
 * exchange of compressed gradients in the paper's pipeline (section "Implementation": the
 * communication engine applies the chosen per-layer parameters on every worker).
 *   d_payload   device buffer holding every layer's payload at offsets[l]
 *   d_out       fp32 device buffer with the layout of the gradient buffer; layer l's region
 *               receives the image of its payload: fma(code, unit, min) per element (QUANT),
 *               the kept values at their indices and zero elsewhere (TOPK), Phat Q^T (LOWRANK)
 *   accumulate  0: the image replaces the region; 1: it is added to what the region holds
 *               (fp32, one rounding per element), as when summing the workers' gradients
 * Elements of d_out outside the layers are not touched.  A Top-K index at or beyond the
 * layer's size (a corrupt payload) is skipped. */
int lgreco_decompress(lgreco_handle_t* h, const uint8_t* d_payload, const int64_t* offsets,
                      const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands,
                      int32_t P, const int32_t* choice, float* d_out, int32_t accumulate,
                      void* stream);

/* Gradient accumulation between two runs of the algorithm (section "Implementation": in
 * between runs, per-layer gradients are accumulated in auxiliary buffers; the error table is
 * then built on the accumulated gradients).  d_acc[i] = d_grads[i] when reset != 0 (first step
 * of a window), else d_acc[i] += d_grads[i]; fp32, n elements, both buffers 16-byte aligned. */
int lgreco_accumulate(lgreco_handle_t* h, float* d_acc, const float* d_grads, int64_t n,
                      int32_t reset, void* stream);

/* Timing of the kernels launched by the last profile / solve / compress call on this handle.
 * lgreco_set_timing(h, level) makes every call time its kernels with HIP events on the call's
 * stream: level 1 the main kernels only (the streaming passes, the contractions, the DP), whose
 * events ride on the kernel launches themselves (the kernel's own begin and end timestamps);
 * level 2 every section, each further bracket a pair of recorded events; 0 none.  Either kind of
 * event costs a few microseconds of the stream's time.  Setting the level also clears the totals below.
 * lgreco_get_timing returns the number of sections recorded by the last call and
 * fills names (static strings) and milliseconds for up to `cap` of them. */
int lgreco_set_timing(lgreco_handle_t* h, int32_t level);
/* Time only every `every`-th call of each kind, counted from the last lgreco_set_timing (the
 * first call after it is timed); 1 = every call, the default.  A kernel that carries events
 * leaves a few microseconds of the stream idle on either side of it, so a loop that wants its
 * own throughput undisturbed samples. */
int lgreco_set_timing_stride(lgreco_handle_t* h, int32_t every);
int lgreco_get_timing(lgreco_handle_t* h, const char** names, float* ms, int32_t cap);
/* The same for the last call of one kind (the handle keeps one set of events per kind, so a
 * lgreco_compress that returned with its kernels still queued can be read after a later profile
 * or solve call).  Both functions wait for the events they read.  The library itself reads a
 * call's events out when the next call of that kind starts (which therefore waits for the
 * earlier one while timing is on) or when a call of another kind is about to wait for the
 * stream anyway, whichever comes first. */
#define LGRECO_CALL_PROFILE  0
#define LGRECO_CALL_SOLVE    1
#define LGRECO_CALL_COMPRESS 2
#define LGRECO_CALL_RECEIVE  3   /* lgreco_decompress, lgreco_accumulate */
int lgreco_get_timing_of(lgreco_handle_t* h, int32_t call, const char** names, float* ms, int32_t cap);
/* Totals per section over all calls of one kind since lgreco_set_timing: names, summed
 * milliseconds and how many calls contributed, for up to `cap` sections; returns the number of
 * sections.  A loop can run untouched and be read once at its end. */
int lgreco_get_timing_totals(lgreco_handle_t* h, int32_t call, const char** names, double* total_ms,
                             int64_t* count, int32_t cap);

/* A promise about d_ef of lgreco_profile_solve_compress, kept until changed: while `on` is not 0 the
 * caller guarantees that the buffer holds zeros on entry of every such call (the first step of a
 * run, or a caller that keeps no error feedback between calls and hands in a cleared buffer).  The
 * profile then does not read it (x = fl32(g + 0) = g: 4 bytes per element less to fetch, which the
 * memory-bound contractions of the low-rank profile feel most), nor does the low-rank layers'
 * compression of the same call, which writes the new error feedback without fetching the old;
 * the other families' compression reads and updates it as ever, and every result is the one the
 * call gives without the promise.  A buffer that is not zero under the promise gives results
 * that ignore part or all of its content: not an error the library can see.  Off at creation. */
int lgreco_set_ef_zero_on_entry(lgreco_handle_t* h, int32_t on);

/* How many solves on this handle found the solver's result block incomplete when its sequence
 * number had already arrived in host memory (the block's check words caught it and the call went
 * on waiting until the block was whole).  Diagnostics only. */
int64_t lgreco_late_handovers(const lgreco_handle_t* h);

/* How the last successful solve on this handle swept its table: 0 sequentially, G > 0 in G layer
 * groups, 1000 + G in G groups where ties between ways of sharing the error bins among the groups
 * had to be resolved by Algorithm 1's tie-breaks, -G sequentially after that resolution gave up.
 * Diagnostics only. */
int lgreco_last_solve_groups(const lgreco_handle_t* h);

const char* lgreco_strerror(int status);
/* Text of the last HIP error seen by this handle ("" if none). */
const char* lgreco_last_hip_error(const lgreco_handle_t* h);

#ifdef __cplusplus
}
#endif
#endif /* LGRECO_H */
