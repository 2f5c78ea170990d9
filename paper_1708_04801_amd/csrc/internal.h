// Host-side plumbing shared by the translation units of libwpsgd: the argument block every
// chain kernel receives, the resolved kernel plan, and the launcher entry of each kernel family.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "wpsgd.h"

namespace wpsgd {

// Arguments common to all chain kernels.  Workgroup b runs chain order[b] for nsteps[b] steps
// (the host sorts chains longest first so that a late workgroup never holds the longest chain).
struct ChainArgs {
    // data set
    const void *dense;        // row-major, ld elements per row (fp32 or bfloat16 bits)
    int64_t ld;
    const int64_t *row_ptr;   // CSR
    const int32_t *col_idx;
    const float *vals;
    const float *y;
    int64_t m, d;
    // chains
    int k;
    const int32_t *order;     // DEVICE, k entries: chain id run by workgroup b
    const int64_t *nsteps;    // DEVICE, k entries: steps of that chain
    const int64_t *step0;     // DEVICE, k entries: position in that chain's sample stream of its first step
    const double *pow_tab;    // DEVICE, 128 entries: (1-eta*lambda)^l for l = 0..63, then (1-eta*lambda)^-(l+1)
    const float *w_start;     // DEVICE, d entries: every chain starts from this vector; NULL: from zero
    const uint32_t *perm;     // DEVICE, m entries: shuffled row order for partition-and-shuffle sampling;
                              // NULL: the with-replacement stream
    const uint32_t *shard;    // DEVICE, 3k entries when perm is set: for workgroup b, its chain's first
                              // position shard[b], share size shard[k+b], and step0 mod size shard[2k+b]
    // hyper-parameters (fp64 on purpose: (1-eta*lambda)^n must not be compounded in fp32)
    double eta, rho;          // rho = 1 - eta*lambda
    uint32_t seed_lo, seed_hi;
    // Helper workgroups (dense register kernels): workgroups k .. k+helpers-1 run ahead of the
    // chains and pull their rows into the L2 cache; helpers is a multiple of k (or 0, and only
    // for k <= 128).
    int helpers;
    uint32_t *progress;       // DEVICE, 2k+16 entries, zero at launch: [b] steps workgroup b has completed
                              // (low 32 bits), [k+b] its XCD number plus one, [2k+x] helper seats taken on XCD x
    // Column slices (dense register kernel): workgroup b + s*k runs slice s of the chain of workgroup b;
    // xchg is the table the slices add their partial sums through (zero at launch), else unused.
    int slices;               // 1: a chain is one workgroup
    void *xchg;               // DEVICE, k * 8 * 2 slots of 128 bytes, then k * 8 words (the slices' XCD numbers)
    uint32_t slice_max_polls; // how often a slice polls for the others' sums before it gives up (a poll takes
                              // 600 to 1200 cycles); 0: it does not poll at all
    uint32_t *status;         // DEVICE, first word of the workspace: bit 0 is set by a slice that gave up
    // outputs / scratch
    float *W;                 // k x d
    void *state;              // k x d model vectors in HBM (state_in_hbm plans), else unused
};

// Arguments of the delay-SGD servers (Section IV, Algorithms 3 and 4): workgroup i is server i.
constexpr int kDelayMaxTau = 16;
struct DelayArgs {
    const void *dense;        // row-major, ld elements per row (fp32 or bfloat16 bits)
    int64_t ld;
    const float *y;
    int64_t m, d;
    int k;
    const int64_t *n_samples; // DEVICE, k entries: samples server i receives
    const float *w_start;     // DEVICE, d entries, or NULL for zero
    double eta, lambda;
    int loss, tau, check;
    uint32_t seed_lo, seed_hi;
    double *ring;             // DEVICE, k x (max(tau,1)+2) x d: the iterates each server keeps
    void *row_table;          // DEVICE, m x 32 bytes: room for what the Check function needs of each row, or
                              // NULL when the servers visit too few rows for such a table to pay
    float *W;                 // k x d out
    int64_t *accepted;        // k out: updates each server has made
};

enum class Family { DenseReg, DenseMem, Csr };

// A fully resolved plan (every field chosen).
struct Plan {
    Family family;
    int dtype;       // WPSGD_F32 / WPSGD_BF16 (dense)
    int loss;
    int threads;     // workgroup size
    int ept;         // model elements per thread (DenseReg)
    int vec;         // elements per global load instruction
    int block_steps; // B
    int prefetch;    // P: rounds in flight
    int rows;        // DenseReg: 1 rows wait in registers, 2 next row staged in LDS, 3 rows streamed twice
    int slices;      // DenseReg, rows = 1: workgroups (column slices) per chain
    size_t state_bytes_per_elem;   // 0 when the state lives in registers
};

// Launchers: return hipSuccess, or hipErrorInvalidValue when no instantiation matches the plan.
hipError_t launch_dense_reg(const Plan &p, const ChainArgs &a, hipStream_t s);
hipError_t launch_dense_mem(const Plan &p, const ChainArgs &a, hipStream_t s);
hipError_t launch_csr(const Plan &p, const ChainArgs &a, hipStream_t s);
hipError_t launch_csr_pair(const Plan &p, const ChainArgs &a, hipStream_t s);   // two waves per chain
bool dense_reg_has(const Plan &p);   // is (dtype, loss, threads, ept, vec, B, P) instantiated?

hipError_t launch_delay_servers(const DelayArgs &a, int dtype, int vec, hipStream_t s);
hipError_t launch_zero_words(uint32_t *p, size_t words, hipStream_t s);
hipError_t launch_combine(const float *W, const double *a_dev, int k, int64_t d, float *w_out,
                          hipStream_t s);
hipError_t launch_stream_rows(const void *X, int64_t row_stride, uint32_t row_bytes, uint32_t m,
                              int groups, int64_t rows_per_group, uint32_t seed_lo, uint32_t seed_hi,
                              float *sink, hipStream_t s);
// Objective / error-rate evaluator: ChainArgs carries the matrix, the labels and m, d only.
int64_t objective_grid(int64_t m);
size_t objective_partials_bytes(int64_t m);
// the library's own partial-sum area on the current device (a file-scope device array) and its size
hipError_t objective_static_partials(double **partials, size_t *bytes);
hipError_t launch_objective(const ChainArgs &a, int dtype, int vec, int loss, const float *w, double lambda,
                            double *partials, double *out, hipStream_t s);
hipError_t launch_permute_rows(uint32_t seed_lo, uint32_t seed_hi, uint32_t m, uint32_t *perm, hipStream_t s);
hipError_t launch_sample_rows(uint32_t seed_lo, uint32_t seed_hi, uint32_t chain, int64_t n0,
                              int64_t count, uint32_t m, uint32_t shard_k, int64_t *out, hipStream_t s);

}  // namespace wpsgd
