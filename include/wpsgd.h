/*
 * wpsgd.h -- C ABI of the WP-SGD hot path on AMD MI355X (gfx950).
 *
 * The library runs k independent sequential SGD chains of unequal length on an
 * L2-regularised linear loss and then forms one weighted model average, as in
 * Algorithm 1 ("WP-SGD") of arXiv 1708.04801.
 *
 * Conventions for every entry point
 *   - Return value: WPSGD_OK (0) or a negative wpsgd_status.  Nothing throws.
 *   - "DEVICE" pointers are HIP device addresses on the current device, owned by
 *     the caller; "HOST" pointers are ordinary host memory.  The library never
 *     frees or keeps a caller pointer past the call.  (HOST inputs are copied
 *     before the call returns.)
 *   - GPU work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and is NOT synchronised: device outputs are complete
 *     when the stream reaches that point.  HOST outputs are complete on return.
 *     HOST inputs travel through pinned staging buffers that belong to the call,
 *     so a call that takes HOST arrays cannot be recorded into a HIP graph.
 *   - Step counts: n_steps[i] is the number of SGD steps chain i runs.  In the
 *     paper's notation the fastest node consumes t = max_i n_steps[i] samples
 *     and node i is T_i = t - n_steps[i] steps behind it (Algorithm 1; Table I).
 *   - The library allocates no device memory; scratch space is a caller-provided
 *     workspace whose size the *_workspace functions report.
 */
#ifndef WPSGD_H
#define WPSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WPSGD_OK = 0,
    WPSGD_INVALID_ARG = -1,        /* NULL pointer, size out of range, bad enum, eta*lambda >= 1 ... */
    WPSGD_HIP_ERROR = -2,          /* a HIP call failed; see wpsgd_last_hip_error()                  */
    WPSGD_WORKSPACE_TOO_SMALL = -3,
    WPSGD_UNSUPPORTED = -4,        /* a forced plan that no kernel implements                        */
    WPSGD_INCOMPLETE = -5          /* reported by wpsgd_chains_status: some chains could not finish  */
} wpsgd_status;

/* L(x, y, yhat) of Eq. 4, a convex function of yhat = w.x:
 *   hinge    max(0, 1 - y*yhat)      slope -y where y*yhat < 1, 0 elsewhere (0 at the kink)
 *   logistic log(1 + exp(-y*yhat))   slope -y / (1 + exp(y*yhat))                            */
typedef enum { WPSGD_HINGE = 0, WPSGD_LOGISTIC = 1 } wpsgd_loss;

/* Which examples a chain visits.
 *   STREAM  row = floor(word0 * m / 2^32) of a Philox4x32-10 stream keyed by (seed, chain, step):
 *           independent draws with replacement from the whole data set (wpsgd_sample_indices).
 *   SHARDS  Algorithm 1 as written: the examples are randomly partitioned among the k nodes and
 *           each node walks its own part in random order, without replacement
 *           (wpsgd_shard_indices).                                                             */
typedef enum { WPSGD_SAMPLE_STREAM = 0, WPSGD_SAMPLE_SHARDS = 1 } wpsgd_sampling;

/* Storage type of dense rows.  bfloat16 values are widened exactly to fp32 on load. */
typedef enum { WPSGD_F32 = 0, WPSGD_BF16 = 1 } wpsgd_dtype;

/* The data set {x^1..x^m} of Eq. 3, one example per row.  Exactly one of `dense`
 * and the CSR triple is non-NULL.  All pointers are DEVICE pointers.            */
typedef struct wpsgd_matrix {
    int64_t m;                 /* rows (examples), 1 <= m < 2^32                             */
    int64_t d;                 /* columns (model dimension), d >= 1                          */
    const void *dense;         /* row-major m x d, element (j,c) at dense[j*ld + c]; or NULL */
    int64_t ld;                /* row stride in elements, ld >= d (ignored for CSR)          */
    wpsgd_dtype dtype;         /* storage of `dense` (CSR values are always fp32)            */
    const int64_t *row_ptr;    /* CSR: m+1 offsets, row j is [row_ptr[j], row_ptr[j+1])      */
    const int32_t *col_idx;    /* CSR: column of each entry, strictly ascending in a row, < d */
    const float *vals;         /* CSR: value of each entry                                   */
} wpsgd_matrix;

/* Optional kernel plan for wpsgd_run_chains; zero in a field means "choose for me".
 * Used by the tests and the tuner to reach every kernel variant at any size.      */
typedef struct wpsgd_plan {
    int threads;         /* workgroup size of a chain: 64, 256, 512 or 1024 (dense); 64 or 192 (CSR)    */
    int block_steps;     /* dense: SGD steps folded into one reduction round: 1, 2, 4 or 8              */
    int prefetch;        /* dense: rounds of sample rows kept in flight ahead of the one being consumed.
                            CSR: selects the kernel - 1 plain gather/scatter; 4 one wave per chain, hot
                            columns in LDS, cold model values fetched 4 steps ahead; 8 the same with two
                            more waves per chain that prepare the rows (the default)                  */
    int state_in_hbm;    /* 1: keep the model vector in the workspace (HBM) instead of registers        */
    int rows;            /* where a dense row waits between its dot product and its update:
                            1 registers, requested `prefetch` rounds ahead; 2 registers, with the next
                            row landing in LDS meanwhile (rows up to 128 KiB); 3 nowhere: the row is
                            streamed twice (rows too long for 1 and 2)                                 */
    int helpers;         /* dense, 256 threads, k a multiple of 8: workgroups per chain that run ahead of
                            it on otherwise idle compute units and pull its rows into the L2 cache the
                            chain's compute unit shares.  0: choose (2 when compute units are to spare
                            and rows are 8 KiB or longer); -1: none; 1..3: that many, room permitting  */
    int slices;          /* dense, 256 threads, rows in registers: compute units per chain.  Each takes a
                            slice of 256 x (elements per thread) columns of the model vector and of every
                            row; the slices add their partial sums through global memory once per round
                            (logistic: up to 4 steps per round; hinge: up to 2).  k*slices must not exceed
                            the compute units.  0: choose (chains whose rows need more than 256
                            threads, compute units permitting); 1: a chain is one workgroup; 2..8: that
                            many, which must be what some 256-thread shape needs to cover d.
                            The slices of a chain wait for each other, so all k*slices workgroups must
                            be running at once.  The library sees to it where it can: a sliced launch
                            never has more workgroups than the device has compute units, and within one
                            process sliced launches run one after the other whatever streams they are
                            queued on.  What it cannot see (another process that keeps the device busy)
                            can still seat some slices late; a slice that has waited slice_wait_us in
                            vain ends, the chain's row of W is NaN, and wpsgd_chains_status reports
                            WPSGD_INCOMPLETE.                                                          */
    int slice_wait_us;   /* about how long a column slice waits for the others' sums before it gives up, in
                            microseconds, at most 60 s (the kernel counts polls: it waits at least this long
                            and at most about twice as long).  0: two seconds.  -1: not at all, so that every
                            sliced chain gives up at its first exchange (a test of that path)          */
} wpsgd_plan;

/* ---- per-chain SGD (Algorithm 1, the loop over n = 1..t-T_i; Eq. 5 with Eq. 4) ----
 *
 * Chain i (i = 0..k-1) starts from w = 0 (Algorithm 1) and performs n_steps[i] updates
 *     w <- (1 - eta*lambda) * w  -  eta * dL/dyhat(y_j, w.x_j) * x_j
 * where j is the row its own sample stream names at that step (see
 * wpsgd_sample_indices).  The result of chain i is written to W[i*d .. i*d+d).
 *
 *   X, y        DEVICE; y holds m labels, each -1 or +1
 *   k           number of chains, 1 <= k <= 2^31-1
 *   n_steps     HOST, k entries, each >= 0 (0: the chain does nothing, its row of W is 0)
 *   eta, lambda eta > 0, lambda >= 0, eta*lambda < 1
 *   seed        key of the sample stream
 *   W           DEVICE out, k x d row-major fp32
 *   workspace   DEVICE scratch of at least wpsgd_run_chains_workspace(...) bytes, 256-byte
 *               aligned; contents on entry are ignored, contents on exit are unspecified
 *   plan        NULL or a forced kernel plan
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, UNSUPPORTED (forced plan), HIP_ERROR.
 * Two calls that share a workspace must be ordered on one stream.                        */
size_t wpsgd_run_chains_workspace(const wpsgd_matrix *X, int k, wpsgd_loss loss,
                                  const wpsgd_plan *plan);
int wpsgd_run_chains(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_steps,
                     double eta, double lambda, wpsgd_loss loss, uint64_t seed,
                     float *W, void *workspace, size_t workspace_bytes,
                     const wpsgd_plan *plan, void *stream);

/* The same from a common start vector and from inside the sample streams: chain i starts from
 * w_start (DEVICE, d entries fp32; NULL means zero) and takes the rows its stream names at steps
 * step_offsets[i] .. step_offsets[i] + n_steps[i] - 1 (HOST, k entries >= 0; NULL means zero).
 * With both NULL and sampling = WPSGD_SAMPLE_STREAM this is wpsgd_run_chains.  WPSGD_SAMPLE_SHARDS
 * needs k <= m.  The experiments of the paper start every node from a
 * constant vector; restarting all chains from the weighted average every so many steps, each chain
 * continuing its own stream, is the periodic averaging of Section III (Deduction 2).            */
int wpsgd_run_chains_from(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_steps,
                          double eta, double lambda, wpsgd_loss loss, uint64_t seed, wpsgd_sampling sampling,
                          const float *w_start, const int64_t *step_offsets, float *W,
                          void *workspace, size_t workspace_bytes, const wpsgd_plan *plan, void *stream);

/* Did every chain of the last wpsgd_run_chains, wpsgd_run_chains_from or wpsgd_run_spans call on
 * this workspace (all spans of it) finish?  Waits for `stream`, on which that call was queued, and
 * reads the status word the kernels keep at the start of the workspace.
 * Returns WPSGD_OK, or WPSGD_INCOMPLETE if chains that were cut into column slices gave up waiting
 * for each other (their rows of W, and whatever was computed from them, are NaN), or an error.   */
int wpsgd_chains_status(const void *workspace, void *stream);

/* ---- delay SGD under the Check function (Section IV, Algorithm 3 phase 1, Algorithm 4; Lemma 4) ----
 * Server i (i = 0..k-1) receives n_samples[i] samples, the rows its own sample stream names (see
 * wpsgd_sample_indices), and keeps the iterates w_0, w_1, .. w_J it has accepted.  For a sample (x, y)
 * the gradient was taken tau iterates ago:
 *     candidate = w_J - eta*lambda*w_{J-tau} - eta * dL/dyhat(y, w_{J-tau}.x) * x
 * (an index below 0 means w_0).  With check != 0 the candidate becomes w_{J+1} only if Algorithm 4
 * accepts, first, every triple of consecutive iterates among w_{J-tau} .. w_J and then the triple
 * (w_{J-1}, w_J, candidate), all measured along x: with L_w = w.x, beta^2 = x.x,
 *     rate = (eta*lambda + eta*beta^2)^(1/max(tau,1))      (c* = 1 bounds the slope of both losses)
 *     Length_min = (L_b - rate*L_a) / (1 - rate)
 * a triple (a, b, c) passes if rate < 1, L_c lies between L_b and Length_min (ends included) and
 * |b|^2 - L_b^2/beta^2 <= |a|^2 - L_a^2/beta^2 (the part across the sample does not grow, as the proof
 * of Lemma 4 requires).  Triples that would reach before w_0 are not tested.  A rejected candidate is
 * dropped, its sample is spent, and the server is as it was.  With check == 0 every candidate is kept:
 * plain delay SGD.  All arithmetic is fp64.
 *   X            DEVICE, dense rows only (CSR: UNSUPPORTED)
 *   n_samples    HOST, k entries >= 0
 *   tau          delay, 0 <= tau <= 16 (more: UNSUPPORTED)
 *   w_start      DEVICE, d entries fp32: w_0 of every server; NULL means zero (Algorithm 3)
 *   W            DEVICE out, k x d row-major fp32: the last accepted iterate of each server
 *   accepted     DEVICE out, k entries: J of each server.  Phase 2 of Algorithm 3 is wpsgd_weights_rate
 *                on these counts followed by wpsgd_combine.
 *   workspace    DEVICE scratch of at least wpsgd_run_delay_chains_workspace(X, k, tau) bytes (0 is
 *                returned for arguments the call would refuse), 256-byte aligned: the sample counts, room
 *                for the servers' iterates, and 32 bytes per row of X for what the test needs of a row
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR.                              */
size_t wpsgd_run_delay_chains_workspace(const wpsgd_matrix *X, int k, int tau);
int wpsgd_run_delay_chains(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_samples,
                           double eta, double lambda, wpsgd_loss loss, uint64_t seed, int tau, int check,
                           const float *w_start, float *W, int64_t *accepted,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---- weights (Eq. 6; Eq. 8 for a chosen contraction rate r) ----
 *   a[i] = rate^{T_i} / sum_j rate^{T_j},  T_i = max_j n_steps[j] - n_steps[i],
 *   rate = 1 - eta*lambda (wpsgd_weights) or r in (0, 1] (wpsgd_weights_rate).
 * Pure host code, fp64.  a is HOST out, k entries.  Equal step counts give exactly 1/k
 * (the plain average of SimuParallel SGD, Algorithm 2).                                   */
int wpsgd_weights(int k, const int64_t *n_steps, double eta, double lambda, double *a);
int wpsgd_weights_rate(int k, const int64_t *n_steps, double rate, double *a);

/* Benefit condition of Eq. 7 / Eq. 9 (Corollary 3 / 4): *margin receives
 * 2*sum_i rate^{T_i} - (sqrt(k) + k); positive means the condition holds.  HOST only.  */
int wpsgd_benefit_margin(int k, const int64_t *n_steps, double rate, double *margin);

/* ---- weighted model average (Algorithm 1, the aggregation line; Lemma 3) ----
 *   w_out[c] = sum_{i=0}^{k-1} a[i] * W[i*d + c],  accumulated in fp64, rounded once to fp32.
 *   W       DEVICE k x d row-major fp32        a      HOST, k entries
 *   w_out   DEVICE out, d entries fp32
 *   workspace DEVICE scratch of at least wpsgd_combine_workspace(k, d) bytes, 256-byte aligned */
size_t wpsgd_combine_workspace(int k, int64_t d);
int wpsgd_combine(const float *W, const double *a, int k, int64_t d, float *w_out,
                  void *workspace, size_t workspace_bytes, void *stream);

/* ---- periodic weighted averaging (Section III, Deduction 2) ----
 * n_spans times over: every chain i takes steps_per_span[i] steps from the common vector v (w_start,
 * or zero, the first time), continuing its own sample stream where the previous span left it, and v
 * becomes sum_i a_i w_i with the weights of Eq. 6 for steps_per_span.  The largest entry of
 * steps_per_span is the paper's `span`, counted on the fastest node.  One span is Algorithm 1.
 * Everything is queued on `stream`; the call may wait for earlier spans' small host-to-device
 * copies (step counts, weights), never for a kernel it has queued itself.
 *   steps_per_span  HOST, k entries >= 0, at least one > 0; steps_per_span[i] * n_spans <= 2^62
 *   w_start         DEVICE, d entries fp32, or NULL for zero
 *   w_out           DEVICE out, d entries fp32: v after the last span (may be w_start)
 *   workspace       DEVICE scratch of at least wpsgd_run_spans_workspace(...) bytes, 256-byte aligned
 *                   (the chains' models, and what wpsgd_run_chains and wpsgd_combine need)
 * Errors: as wpsgd_run_chains_from and wpsgd_combine; INVALID_ARG for n_spans < 1.             */
size_t wpsgd_run_spans_workspace(const wpsgd_matrix *X, int k, wpsgd_loss loss, const wpsgd_plan *plan);
int wpsgd_run_spans(const wpsgd_matrix *X, const float *y, int k, const int64_t *steps_per_span, int64_t n_spans,
                    double eta, double lambda, wpsgd_loss loss, uint64_t seed, wpsgd_sampling sampling,
                    const float *w_start, float *w_out, void *workspace, size_t workspace_bytes,
                    const wpsgd_plan *plan, void *stream);

/* The expression the text below Deduction 2 asks to keep under 1 for averaging every span to be
 * valid:  *value = k / (sum_j rate^{T_j}) * rate^{span},  span = max_j steps_per_span[j],
 * T_j = span - steps_per_span[j].  (It equals k / sum_j rate^{-steps_per_span[j]}, so as printed it
 * is below 1 whenever rate < 1 and some chain moves.)  HOST only, fp64.                         */
int wpsgd_span_condition(int k, const int64_t *steps_per_span, double rate, double *value);

/* ---- objective and prediction error of a model (Eq. 3 with the loss of Eq. 4) ----
 *   out[0] = lambda/2 * |w|^2 + (1/m) * sum_j L(x_j, y_j, w.x_j)
 *   out[1] = fraction of rows with y_j * (w.x_j) <= 0     (the error rate the experiments report)
 * Dot products, losses and sums are carried in fp64; the result does not depend on timing.
 *   X, y     DEVICE, as for wpsgd_run_chains (to evaluate on part of a data set, pass a matrix
 *            that describes those rows: an offset `dense` or `row_ptr` pointer and their count)
 *   w        DEVICE, d entries fp32 (for instance the output of wpsgd_combine)
 *   out      DEVICE, two doubles, 8-byte aligned
 *   workspace DEVICE scratch of at least wpsgd_objective_workspace(X) bytes, 256-byte aligned
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, UNSUPPORTED (d >= 2^29), HIP_ERROR.                    */
size_t wpsgd_objective_workspace(const wpsgd_matrix *X);
int wpsgd_objective(const wpsgd_matrix *X, const float *y, const float *w, double lambda, wpsgd_loss loss,
                    double *out, void *workspace, size_t workspace_bytes, void *stream);

/* The same for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The partial sums live in an area
 * of 192 KiB that the library owns on every device it runs on (a static device array, held until
 * the process ends), which is enough for any m; a data set that would need more is refused with
 * WPSGD_UNSUPPORTED, as is d >= 2^29.  The call allocates nothing and the result is bit for bit
 * that of wpsgd_objective.  All calls on one device share the area: calls that may overlap there
 * (two streams, two host threads) race on it and must be ordered by the caller; nothing in it has
 * to be cleared between calls.                                                                    */
int wpsgd_objective_static(const wpsgd_matrix *X, const float *y, const float *w, double lambda, wpsgd_loss loss,
                           double *out, void *stream);

/* ---- sample stream (stands for the per-node shuffle and n-th-example fetch of Algorithm 1) ----
 * Row visited by chain `chain` at step n (0-based):
 *   (r0,..) = Philox4x32-10(counter = (n mod 2^32, n div 2^32, chain, 0),
 *                           key = (seed mod 2^32, seed div 2^32));   j = floor(r0 * m / 2^32).
 * Writes rows for steps n0 .. n0+count-1.  The HOST variant runs the generator on the CPU;
 * the DEVICE variant runs the same generator the chain kernels use and writes to DEVICE memory. */
int wpsgd_sample_indices(uint64_t seed, int chain, int64_t n0, int64_t count, int64_t m,
                         int64_t *out_host);
int wpsgd_sample_indices_device(uint64_t seed, int chain, int64_t n0, int64_t count, int64_t m,
                                int64_t *out_device, void *stream);

/* ---- sample order of Algorithm 1: random partition among k nodes, each node shuffles its part ----
 * One keyed permutation pi of [0, m) shuffles all rows: a four-round Feistel network over 2h bits
 * (h = max(1, ceil(bits(m-1)/2))), round r mapping (L, R) to (R, L xor (F_r(R) mod 2^h)) with
 * F_r(R) = word 0 of Philox4x32-10(counter = (R, r, 0x5348524D, 0xFFFFFFFF), key = seed), applied
 * again while the result is >= m.  Node i owns the permuted positions [floor(i*m/k), floor((i+1)*m/k))
 * and visits them in order, starting over when it has seen them all:
 *     row(i, n) = pi(lo_i + n mod m_i).
 * Needs 1 <= k <= m < 2^32 and 0 <= chain < k.  HOST and DEVICE variants as above.             */
int wpsgd_shard_indices(uint64_t seed, int chain, int k, int64_t n0, int64_t count, int64_t m,
                        int64_t *out_host);
int wpsgd_shard_indices_device(uint64_t seed, int chain, int k, int64_t n0, int64_t count, int64_t m,
                               int64_t *out_device, void *stream);

/* ---- diagnostics ---- */
/* Streaming ceiling probe (not a step of the method): `groups` workgroups of 256 threads each read
 * `rows_per_group` rows of the dense matrix X, in the order the sample stream of chain = group index
 * names them, with 64 to 128 KiB in flight and no arithmetic.  Timed by the caller, it tells how fast
 * that many compute units can pull rows out of HBM, i.e. the ceiling of any kernel that gives one
 * chain to one workgroup.  sink: DEVICE, groups*256 floats (written, content meaningless).
 * Rows must be 16-byte aligned and a multiple of 16 bytes long, else UNSUPPORTED.             */
int wpsgd_stream_rows(const wpsgd_matrix *X, int groups, int64_t rows_per_group, uint64_t seed,
                      float *sink, void *stream);

const char *wpsgd_strerror(int status);
int wpsgd_last_hip_error(void);           /* hipError_t of the last failed HIP call on this thread */
/* Writes a short description of the kernel the given problem would run (for logs and the
 * tuner), e.g. "dense_reg f32 logistic nt=256 ept=16 vec=4 B=4 P=2".  HOST.                */
int wpsgd_describe_plan(const wpsgd_matrix *X, int k, wpsgd_loss loss, const wpsgd_plan *plan,
                        char *buf, size_t buf_bytes);

#ifdef __cplusplus
}
#endif
#endif /* WPSGD_H */
