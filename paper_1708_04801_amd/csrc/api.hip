// The C ABI of libwpsgd (see wpsgd.h): argument checks, the kernel planner, the host-side
// weights of Eq. 6 / Eq. 8, and the small host->device hand-overs the kernels need.
#include <algorithm>
#include <atomic>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <numeric>
#include <vector>

#include "device_utils.h"
#include "internal.h"

namespace wpsgd {

hipError_t dense_reg_dispatch_f32_loss0(Plan &, const ChainArgs *, hipStream_t);
hipError_t dense_reg_dispatch_f32_loss1(Plan &, const ChainArgs *, hipStream_t);
hipError_t dense_reg_dispatch_bf16_loss0(Plan &, const ChainArgs *, hipStream_t);
hipError_t dense_reg_dispatch_bf16_loss1(Plan &, const ChainArgs *, hipStream_t);
bool dense_reg_shape_f32_loss0(int, int, int);
bool dense_reg_shape_f32_loss1(int, int, int);
bool dense_reg_shape_bf16_loss0(int, int, int);
bool dense_reg_shape_bf16_loss1(int, int, int);

static thread_local int g_last_hip_error = 0;

static int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return WPSGD_HIP_ERROR;
}

static hipError_t dense_reg_dispatch(Plan &p, const ChainArgs *a, hipStream_t s)
{
    if (p.dtype == WPSGD_BF16)
        return p.loss == WPSGD_HINGE ? dense_reg_dispatch_bf16_loss0(p, a, s)
                                     : dense_reg_dispatch_bf16_loss1(p, a, s);
    return p.loss == WPSGD_HINGE ? dense_reg_dispatch_f32_loss0(p, a, s)
                                 : dense_reg_dispatch_f32_loss1(p, a, s);
}

static bool dense_reg_shape(int dtype, int loss, int threads, int ept, int vec)
{
    if (dtype == WPSGD_BF16)
        return loss == WPSGD_HINGE ? dense_reg_shape_bf16_loss0(threads, ept, vec)
                                   : dense_reg_shape_bf16_loss1(threads, ept, vec);
    return loss == WPSGD_HINGE ? dense_reg_shape_f32_loss0(threads, ept, vec)
                               : dense_reg_shape_f32_loss1(threads, ept, vec);
}

static size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

static int check_matrix(const wpsgd_matrix *X)
{
    if (!X) return WPSGD_INVALID_ARG;
    if (X->m < 1 || X->m > 0xFFFFFFFFLL || X->d < 1) return WPSGD_INVALID_ARG;
    const bool has_csr = X->row_ptr || X->col_idx || X->vals;
    if (X->dense) {
        if (has_csr) return WPSGD_INVALID_ARG;
        if (X->ld < X->d) return WPSGD_INVALID_ARG;
        if (X->dtype != WPSGD_F32 && X->dtype != WPSGD_BF16) return WPSGD_INVALID_ARG;
    } else {
        if (!(X->row_ptr && X->col_idx && X->vals)) return WPSGD_INVALID_ARG;
    }
    return WPSGD_OK;
}

// Widest load the rows allow: every row start and every fragment must be 16-byte aligned.
static int dense_vec(const wpsgd_matrix *X)
{
    const int wide = X->dtype == WPSGD_BF16 ? 8 : 4;
    const bool ok = ((uintptr_t)X->dense % 16 == 0) && (X->ld % wide == 0) && (X->d % wide == 0);
    return ok ? wide : 1;
}

// Chooses the kernel family and its parameters.  Dense rows go to the register kernel when
// some instantiated shape holds d elements, else to the HBM-state kernel.
static int compute_units()
{
    static std::atomic<int> cached{0};          // (asking twice is harmless)
    int cus = cached.load(std::memory_order_relaxed);
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
            (void)hipGetLastError();
            return 256;                 // no device to ask (planning on a host without one): the target's count
        }
        cus = n;
        cached.store(cus, std::memory_order_relaxed);
    }
    return cus;
}

static int resolve_plan(const wpsgd_matrix *X, int k, wpsgd_loss loss, const wpsgd_plan *force, Plan *out,
                        double rho = 1.0, int64_t max_steps = 0)
{
    Plan p{};
    p.loss = (int)loss;
    p.dtype = X->dense ? (int)X->dtype : WPSGD_F32;
    const size_t state_elem = (loss == WPSGD_HINGE) ? sizeof(double) : sizeof(float);
    const wpsgd_plan f = force ? *force : wpsgd_plan{0, 0, 0, 0, 0, 0, 0, 0};
    if (f.threads < 0 || f.block_steps < 0 || f.prefetch < 0 || f.rows < 0 || f.rows > 3 || f.helpers < -1 || f.helpers > 3 || f.slices < 0 || f.slices > 8) return WPSGD_INVALID_ARG;
    if (f.slice_wait_us < -1 || f.slice_wait_us > 60 * 1000 * 1000) return WPSGD_INVALID_ARG;

    if (!X->dense) {
        if (f.threads && f.threads != kWave && f.threads != 3 * kWave) return WPSGD_UNSUPPORTED;
        if (f.block_steps > 1 || (f.prefetch > 1 && f.prefetch != 4 && f.prefetch != 8) || f.rows || f.slices > 1) return WPSGD_UNSUPPORTED;
        p.family = Family::Csr;
        p.threads = kWave;
        p.vec = 1;
        p.block_steps = 1;
        // The LDS-cached kernels (prefetch 4: one wave per chain, 8: three) never fold their lazy scale
        // back into the vector, so they need (1-eta*lambda)^steps to stay well inside fp32 range.
        // They park unused lanes on scratch columns at the start of the vector, and the two-wave
        // kernel addresses the vector with 32-bit byte offsets.
        const bool no_fold = (double)max_steps * std::log(rho) > -55.0;       // scale > 2^-80
        const bool cached_ok = X->d >= 64 && no_fold;
        const bool pair_ok = X->d >= 128 && no_fold && (uint64_t)X->d * state_elem < (1ull << 32);
        if (f.prefetch == 4 && !cached_ok) return WPSGD_UNSUPPORTED;
        if (f.prefetch == 8 && !pair_ok) return WPSGD_UNSUPPORTED;
        p.prefetch = f.prefetch ? f.prefetch : (pair_ok ? 8 : (cached_ok ? 4 : 1));
        if (p.prefetch == 8) p.threads = 3 * kWave;
        p.state_bytes_per_elem = state_elem;
        *out = p;
        return WPSGD_OK;
    }

    const int wide = dense_vec(X);
    p.vec = wide;
    // The register kernel folds its lazy scale once per 64 steps, which needs
    // (1-eta*lambda)^64 to stay far inside fp32 range; a harsher shrink takes the HBM kernel,
    // which checks every step.
    const bool mild_shrink = rho >= 0.55;
    if (!f.state_in_hbm && mild_shrink) {
        static const int kThreads[] = {64, 256, 512, 1024};
        static const int kEpt[] = {1, 2, 4, 8, 16, 32, 64, 128};
        // smallest workgroup first, then the smallest fragment that covers d; fragments much
        // narrower than one wide load use scalar loads so that all lanes carry data
        auto search = [&](int slices, Plan *found) -> bool {
        for (int nt : kThreads) {
            if (f.threads && f.threads != nt) continue;
            if (slices > 1 && nt != 256) continue;
            for (int ept : kEpt) {
                // the shape covers d, or one slice of it with no slice left empty
                if ((int64_t)nt * ept * slices < X->d) continue;
                if (slices > 1 && (int64_t)nt * ept * (slices - 1) >= X->d) break;
                int vec = wide;
                if (wide > 1 && ept * 4 <= wide) vec = 1;
                if (ept % vec != 0) continue;
                if (!dense_reg_shape(p.dtype, p.loss, nt, ept, vec)) continue;
                Plan q = p;
                q.vec = vec;
                q.family = Family::DenseReg;
                q.threads = nt;
                q.ept = ept;
                q.block_steps = f.block_steps;
                q.prefetch = f.prefetch;
                q.rows = f.rows;
                q.slices = slices;
                q.state_bytes_per_elem = 0;
                if (slices > 1) {
                    // the slices' exchange carries twelve words: ten fp32 sums (4 steps per round) or three fp64 sums (2 steps)
                    q.rows = 1;
                    if (f.rows > 1 || vec == 1 || k * slices > compute_units()) continue;
                    if ((size_t)X->d * state_elem < 2304) continue;       // the exchange table borrows the HBM-state area: 2080 bytes a chain
                    if (!q.block_steps) q.block_steps = 2;             // one exchange per two steps
                    if (q.block_steps > (p.loss == WPSGD_LOGISTIC ? 4 : 2)) continue;
                }
                // Few chains of 16 KiB fp32 rows, each alone on a compute unit, are bound by the
                // latency of a step: two steps per reduction round (three sums instead of two, one
                // exchange instead of two) are 8 % faster there.  With more chains than compute
                // units the extra Gram products would only cost throughput.
                if (!f.block_steps && !f.prefetch && !f.rows && nt == 256 && ept == 16 && vec == 4 &&
                    p.loss == WPSGD_LOGISTIC && p.dtype == WPSGD_F32 && k <= compute_units()) {
                    Plan two = q;
                    two.block_steps = 2;
                    two.prefetch = 4;
                    if (dense_reg_dispatch(two, nullptr, nullptr) == hipSuccess) {
                        *found = two;
                        return true;
                    }
                }
                if (dense_reg_dispatch(q, nullptr, nullptr) == hipSuccess) {
                    *found = q;
                    return true;
                }
            }
        }
        return false;
        };
        Plan found;
        bool have = search(f.slices > 1 ? f.slices : 1, &found);
        // Rows too long for 256 threads (or for any one workgroup), few chains: rather than one chain
        // per 1024-thread workgroup, cut each chain into as many column slices as there are compute
        // units for (the widest workload: 8 slices of 8192 columns run 3 times as fast as one
        // workgroup of 1024; with fp64 state that row length has no one-workgroup shape at all).
        if (f.slices == 0 && !f.threads && !f.block_steps && !f.prefetch && !f.rows && (!have || found.threads == 1024)) {
            for (int c = 8; c >= 2; --c) {
                Plan cut;
                if (k * c <= compute_units() && search(c, &cut)) {
                    found = cut;
                    have = true;
                    break;
                }
            }
        }
        if (have) {
            *out = found;
            return WPSGD_OK;
        }
        if (f.threads || f.block_steps || f.prefetch || f.rows || f.slices > 1) return WPSGD_UNSUPPORTED;
    }
    if (f.rows || f.slices > 1) return WPSGD_UNSUPPORTED;
    p.family = Family::DenseMem;
    p.threads = f.threads ? f.threads : (X->d >= 16384 ? 1024 : 256);
    if (p.threads != 256 && p.threads != 1024) return WPSGD_UNSUPPORTED;
    if (f.block_steps > 1 || f.prefetch > 1) return WPSGD_UNSUPPORTED;
    p.block_steps = 1;
    p.prefetch = 1;
    p.state_bytes_per_elem = state_elem;
    *out = p;
    return WPSGD_OK;
}


// shuffled row order of partition-and-shuffle sampling (always reserved: the workspace query does
// not know which sampling a call will ask for)
static size_t perm_bytes(int64_t m) { return align256((size_t)m * sizeof(uint32_t)); }

static size_t state_elem_bytes(wpsgd_loss loss)
{
    return loss == WPSGD_HINGE ? sizeof(double) : sizeof(float);
}

// Workspace header.  First a status block (word 0: bit 0 set by chains that could not finish, see
// wpsgd_chains_status); then the chain order; then, in that order, step counts, stream offsets,
// three 32-bit numbers per chain describing its share under partition-and-shuffle sampling, and a
// progress counter per chain (zero at launch) that helper workgroups watch; last, the powers
// (1-eta*lambda)^l and (1-eta*lambda)^-(l+1), l = 0..63, in fp64.  Every part is 256-byte aligned.
constexpr size_t kStatusBytes = 256;
constexpr int kSliceWaitDefaultUs = 2 * 1000 * 1000;      // two seconds
constexpr size_t kPowTabBytes = 2 * 64 * sizeof(double);
struct HeaderLayout {
    size_t order, steps, offsets, shard, progress, pow_tab, total;
};
static HeaderLayout header_layout(int k)
{
    HeaderLayout h;
    h.order = kStatusBytes;
    h.steps = h.order + align256((size_t)k * sizeof(int32_t));
    h.offsets = h.steps + align256((size_t)k * sizeof(int64_t));
    h.shard = h.offsets + align256((size_t)k * sizeof(int64_t));
    h.progress = h.shard + align256((size_t)k * 3 * sizeof(uint32_t));
    h.pow_tab = h.progress + align256(((size_t)k * 2 + 16) * sizeof(uint32_t));
    h.total = h.pow_tab + kPowTabBytes;
    return h;
}
static size_t header_bytes(int k) { return header_layout(k).total; }

// 32-bit words of the table the column slices of k chains exchange their sums through: per chain
// 8 slices x 2 round parities x 32 words of records, then 8 words (the slices' XCD numbers)
static size_t slice_table_words(int k) { return (size_t)k * (8 * 2 * 32 + 8); }

// Helper workgroups per chain for a resolved plan: only the 256-thread register kernels have
// them, and only on compute units no chain occupies (at most 128 chains).
static int helpers_per_chain(const Plan &p, const wpsgd_matrix *X, int k, const wpsgd_plan *force)
{
    if (p.family != Family::DenseReg || p.threads != 256 || p.rows != 1 || k > 128 || p.slices > 1) return 0;
    const int asked = force ? force->helpers : 0;
    if (asked < 0) return 0;
    const int room = (compute_units() - k) / k;
    const int64_t row_bytes = X->d * (X->dtype == WPSGD_BF16 ? 2 : 4);
    const int want = asked > 0 ? asked : (row_bytes >= 8192 ? 2 : 0);      // a third helper only adds L2 traffic
    return std::max(0, std::min(want, std::min(room, 3)));
}

// Host arrays (chain order, step counts, weights) reach the device through a small ring of pinned
// staging buffers per host thread.  An event marks the last copy out of a buffer; it is rewritten
// only after that copy has finished, so the caller's arrays can be released as soon as a call returns.
struct StagingSlot {
    void *host = nullptr;
    size_t capacity = 0;
    hipEvent_t last_copy = nullptr;
    bool pending = false;
};
constexpr int kStagingSlots = 4;     // copies that may be queued before a call has to wait
struct StagingRing {
    StagingSlot slot[kStagingSlots];
    int next = 0;
    // A host thread that ends gives its buffers back (once their last copies have finished).  If the
    // runtime is already shutting down the calls fail and the process's exit reclaims everything.
    ~StagingRing()
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) {
            (void)hipGetLastError();
            return;
        }
        for (StagingSlot &st : slot) {
            if (st.pending && st.last_copy) (void)hipEventSynchronize(st.last_copy);
            if (st.last_copy) (void)hipEventDestroy(st.last_copy);
            if (st.host) (void)hipHostFree(st.host);
            st = StagingSlot{};
        }
        (void)hipGetLastError();
    }
};
static thread_local StagingRing g_staging;

static int upload(void *dst, const void *src, size_t bytes, hipStream_t s)
{
    StagingSlot &st = g_staging.slot[g_staging.next];
    g_staging.next = (g_staging.next + 1) % kStagingSlots;
    hipError_t e;
    if (st.pending) {
        e = hipEventSynchronize(st.last_copy);
        if (e != hipSuccess) return hip_fail(e);
        st.pending = false;
    }
    if (st.capacity < bytes) {
        if (st.host) (void)hipHostFree(st.host);
        st.host = nullptr;
        st.capacity = 0;
        const size_t want = std::max<size_t>(bytes, 1 << 16);
        e = hipHostMalloc(&st.host, want, hipHostMallocDefault);
        if (e != hipSuccess) return hip_fail(e);
        st.capacity = want;
    }
    if (!st.last_copy) {
        e = hipEventCreateWithFlags(&st.last_copy, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(e);
    }
    std::memcpy(st.host, src, bytes);
    e = hipMemcpyAsync(dst, st.host, bytes, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventRecord(st.last_copy, s);
    if (e != hipSuccess) return hip_fail(e);
    st.pending = true;
    return WPSGD_OK;
}

static int check_steps(int k, const int64_t *n_steps)
{
    if (k < 1 || !n_steps) return WPSGD_INVALID_ARG;
    for (int i = 0; i < k; ++i)
        if (n_steps[i] < 0) return WPSGD_INVALID_ARG;
    return WPSGD_OK;
}

static const char *family_name(Family f)
{
    switch (f) {
    case Family::DenseReg: return "dense_reg";
    case Family::DenseMem: return "dense_mem";
    default: return "csr";
    }
}

}  // namespace wpsgd

using namespace wpsgd;

extern "C" {

size_t wpsgd_run_chains_workspace(const wpsgd_matrix *X, int k, wpsgd_loss loss, const wpsgd_plan *plan)
{
    if (check_matrix(X) != WPSGD_OK || k < 1) return 0;
    if (loss != WPSGD_HINGE && loss != WPSGD_LOGISTIC) return 0;
    Plan p;
    if (resolve_plan(X, k, loss, plan, &p) != WPSGD_OK) return 0;
    // Always room for the model vectors in HBM: which kernel runs also depends on eta*lambda,
    // which this query does not see.
    return header_bytes(k) + perm_bytes(X->m) + align256((size_t)k * (size_t)X->d * state_elem_bytes(loss));
}

int wpsgd_describe_plan(const wpsgd_matrix *X, int k, wpsgd_loss loss, const wpsgd_plan *plan,
                        char *buf, size_t buf_bytes)
{
    if (!buf || buf_bytes == 0 || k < 1) return WPSGD_INVALID_ARG;
    int rc = check_matrix(X);
    if (rc != WPSGD_OK) return rc;
    if (loss != WPSGD_HINGE && loss != WPSGD_LOGISTIC) return WPSGD_INVALID_ARG;
    Plan p;
    rc = resolve_plan(X, k, loss, plan, &p);
    if (rc != WPSGD_OK) return rc;
    static const char *const kRows[] = {"", " rows=registers", " rows=lds", " rows=twice"};
    char helped[32] = "";
    const int hp = helpers_per_chain(p, X, k, plan);
    if (hp > 0) std::snprintf(helped, sizeof(helped), " helpers=%d", hp);
    if (p.family == Family::DenseReg && p.slices > 1) std::snprintf(helped, sizeof(helped), " slices=%d", p.slices);
    std::snprintf(buf, buf_bytes, "%s %s %s nt=%d ept=%d vec=%d B=%d P=%d state=%s%s%s",
                  family_name(p.family), p.dtype == WPSGD_BF16 ? "bf16" : "f32",
                  p.loss == WPSGD_HINGE ? "hinge" : "logistic", p.threads, p.ept, p.vec,
                  p.block_steps, p.prefetch,
                  p.state_bytes_per_elem == 0 ? "registers" : (p.state_bytes_per_elem == 8 ? "hbm-f64" : "hbm-f32"),
                  p.family == Family::DenseReg ? kRows[p.rows] : "", helped);
    return WPSGD_OK;
}

int wpsgd_run_chains(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_steps,
                     double eta, double lambda, wpsgd_loss loss, uint64_t seed, float *W,
                     void *workspace, size_t workspace_bytes, const wpsgd_plan *plan, void *stream)
{
    return wpsgd_run_chains_from(X, y, k, n_steps, eta, lambda, loss, seed, WPSGD_SAMPLE_STREAM, nullptr, nullptr, W,
                                 workspace, workspace_bytes, plan, stream);
}

// Chains cut into column slices wait for each other's workgroups.  Two such launches seated half and
// half on the device would each wait for workgroups that cannot start before the other launch's have
// ended, so within this process they run one after the other: a launch first makes its stream wait
// for the previous sliced launch on the device (on whatever stream that was queued).
struct SlicedLaunchOrder {
    static constexpr int kMaxDevices = 64;
    std::mutex lock;
    hipEvent_t last[kMaxDevices] = {};
    bool queued[kMaxDevices] = {};
};
static SlicedLaunchOrder g_sliced;

// keep_status: leave the status word as earlier launches on this workspace left it (later spans of
// wpsgd_run_spans); otherwise it is cleared along with the header.
static int run_chains_from(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_steps,
                           double eta, double lambda, wpsgd_loss loss, uint64_t seed, wpsgd_sampling sampling,
                           const float *w_start, const int64_t *step_offsets, float *W,
                           void *workspace, size_t workspace_bytes, const wpsgd_plan *plan, void *stream, bool keep_status)
{
    int rc = check_matrix(X);
    if (rc != WPSGD_OK) return rc;
    if (!y || !W) return WPSGD_INVALID_ARG;
    if (sampling != WPSGD_SAMPLE_STREAM && sampling != WPSGD_SAMPLE_SHARDS) return WPSGD_INVALID_ARG;
    if (sampling == WPSGD_SAMPLE_SHARDS && (int64_t)k > X->m) return WPSGD_INVALID_ARG;     // a node without examples
    rc = check_steps(k, n_steps);
    if (rc != WPSGD_OK) return rc;
    if (step_offsets)
        for (int i = 0; i < k; ++i)
            if (step_offsets[i] < 0 || step_offsets[i] > INT64_MAX - n_steps[i]) return WPSGD_INVALID_ARG;
    if (!(eta > 0.0) || !(lambda >= 0.0) || !(eta * lambda < 1.0)) return WPSGD_INVALID_ARG;
    if (loss != WPSGD_HINGE && loss != WPSGD_LOGISTIC) return WPSGD_INVALID_ARG;
    Plan p;
    int64_t max_steps = 0;
    for (int i = 0; i < k; ++i) max_steps = std::max(max_steps, n_steps[i]);
    rc = resolve_plan(X, k, loss, plan, &p, 1.0 - eta * lambda, max_steps);
    if (rc != WPSGD_OK) return rc;
    // behind the header and the shuffled order: the model vectors of the HBM-state kernels, or the
    // table the column slices of a chain exchange their sums through
    const bool sliced = p.family == Family::DenseReg && p.slices > 1;
    const size_t behind = sliced ? slice_table_words(k) * sizeof(uint32_t) : (size_t)k * (size_t)X->d * p.state_bytes_per_elem;
    const HeaderLayout h = header_layout(k);
    const size_t need = h.total + perm_bytes(X->m) + align256(behind);
    if (!workspace || ((uintptr_t)workspace % 256) != 0) return WPSGD_INVALID_ARG;
    if (workspace_bytes < need) return WPSGD_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);

    // longest chain first (stable, so equal lengths keep their order); order and step counts
    // travel in one copy, laid out exactly as the workspace header
    std::vector<int32_t> order(k);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t x, int32_t z) { return n_steps[x] > n_steps[z]; });
    std::vector<char> header(h.total, 0);
    std::memcpy(header.data() + h.order, order.data(), (size_t)k * sizeof(int32_t));
    int64_t *sorted_steps = reinterpret_cast<int64_t *>(header.data() + h.steps);
    int64_t *sorted_offsets = reinterpret_cast<int64_t *>(header.data() + h.offsets);
    uint32_t *shard = reinterpret_cast<uint32_t *>(header.data() + h.shard);
    for (int b = 0; b < k; ++b) {
        sorted_steps[b] = n_steps[order[b]];
        sorted_offsets[b] = step_offsets ? step_offsets[order[b]] : 0;
        if (sampling == WPSGD_SAMPLE_SHARDS) {
            const uint64_t lo = (uint64_t)order[b] * (uint64_t)X->m / (uint64_t)k;
            const uint64_t hi = ((uint64_t)order[b] + 1) * (uint64_t)X->m / (uint64_t)k;
            shard[b] = (uint32_t)lo;
            shard[k + b] = (uint32_t)(hi - lo);
            shard[2 * k + b] = (uint32_t)((uint64_t)sorted_offsets[b] % (hi - lo));
        }
    }

    double *pow_tab = reinterpret_cast<double *>(header.data() + h.pow_tab);
    {
        const double rho = 1.0 - eta * lambda, inv_rho = 1.0 / rho;
        double up = 1.0, down = inv_rho;
        for (int l = 0; l < 64; ++l) {
            pow_tab[l] = up;
            pow_tab[64 + l] = down;
            up *= rho;
            down *= inv_rho;
        }
    }
    char *ws = static_cast<char *>(workspace);
    uint32_t *perm_dev = reinterpret_cast<uint32_t *>(ws + h.total);
    void *state_dev = ws + h.total + perm_bytes(X->m);
    const size_t from = keep_status ? kStatusBytes : 0;           // (the status block is zero in `header`)
    rc = upload(ws + from, header.data() + from, header.size() - from, s);
    if (rc != WPSGD_OK) return rc;

    ChainArgs a{};
    a.dense = X->dense;
    a.ld = X->ld;
    a.row_ptr = X->row_ptr;
    a.col_idx = X->col_idx;
    a.vals = X->vals;
    a.y = y;
    a.m = X->m;
    a.d = X->d;
    a.k = k;
    a.status = reinterpret_cast<uint32_t *>(ws);
    a.order = reinterpret_cast<const int32_t *>(ws + h.order);
    a.nsteps = reinterpret_cast<const int64_t *>(ws + h.steps);
    a.step0 = reinterpret_cast<const int64_t *>(ws + h.offsets);
    a.w_start = w_start;
    a.pow_tab = reinterpret_cast<const double *>(ws + h.pow_tab);
    a.progress = reinterpret_cast<uint32_t *>(ws + h.progress);
    a.helpers = helpers_per_chain(p, X, k, plan) * k;
    a.slices = sliced ? p.slices : 1;
    a.xchg = state_dev;
    // how long a slice waits for the others before it gives up, as a number of polls: a poll takes 600 to
    // 1200 cycles of a 2.4 GHz clock, so four polls per microsecond are at least the time asked for and
    // at most twice that; 0: no poll at all (the plan's test hook)
    const int wait_us = plan ? plan->slice_wait_us : 0;
    a.slice_max_polls = wait_us < 0 ? 0u : (uint32_t)std::min<int64_t>((int64_t)(wait_us > 0 ? wait_us : kSliceWaitDefaultUs) * 4, INT32_MAX);
    if (a.slices > 1) {
        hipError_t ze = launch_zero_words(static_cast<uint32_t *>(state_dev), slice_table_words(k), s);
        if (ze != hipSuccess) return hip_fail(ze);
    }
    a.eta = eta;
    a.rho = 1.0 - eta * lambda;
    a.seed_lo = (uint32_t)(seed & 0xFFFFFFFFu);
    a.seed_hi = (uint32_t)(seed >> 32);
    a.perm = nullptr;
    if (sampling == WPSGD_SAMPLE_SHARDS) {
        hipError_t pe = launch_permute_rows(a.seed_lo, a.seed_hi, (uint32_t)X->m, perm_dev, s);
        if (pe != hipSuccess) return hip_fail(pe);
        a.perm = perm_dev;
        a.shard = reinterpret_cast<const uint32_t *>(ws + h.shard);
    }
    a.W = W;
    a.state = state_dev;

    hipError_t e;
    if (a.slices > 1) {
        int dev = 0;
        e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        if (dev < 0 || dev >= SlicedLaunchOrder::kMaxDevices) return hip_fail(hipErrorInvalidDevice);
        std::lock_guard<std::mutex> guard(g_sliced.lock);
        if (!g_sliced.last[dev]) {
            e = hipEventCreateWithFlags(&g_sliced.last[dev], hipEventDisableTiming);
            if (e != hipSuccess) return hip_fail(e);
        }
        if (g_sliced.queued[dev]) {
            e = hipStreamWaitEvent(s, g_sliced.last[dev], 0);
            if (e != hipSuccess) return hip_fail(e);
        }
        e = dense_reg_dispatch(p, &a, s);
        if (e == hipSuccess) {
            e = hipEventRecord(g_sliced.last[dev], s);
            g_sliced.queued[dev] = e == hipSuccess;
        }
    } else {
        switch (p.family) {
        case Family::DenseReg: e = dense_reg_dispatch(p, &a, s); break;
        case Family::DenseMem: e = launch_dense_mem(p, a, s); break;
        default: e = launch_csr(p, a, s); break;
        }
    }
    if (e == hipErrorInvalidValue) return WPSGD_UNSUPPORTED;
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

int wpsgd_run_chains_from(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_steps,
                          double eta, double lambda, wpsgd_loss loss, uint64_t seed, wpsgd_sampling sampling,
                          const float *w_start, const int64_t *step_offsets, float *W,
                          void *workspace, size_t workspace_bytes, const wpsgd_plan *plan, void *stream)
{
    return run_chains_from(X, y, k, n_steps, eta, lambda, loss, seed, sampling, w_start, step_offsets, W, workspace,
                           workspace_bytes, plan, stream, false);
}

static size_t delay_ring_bytes(const wpsgd_matrix *X, int k, int tau)
{
    return (size_t)k * (size_t)(std::max(tau, 1) + 2) * (size_t)X->d * sizeof(double);
}

// a table of 32 bytes per row: what the Check function needs of a row and not of the model
static size_t delay_table_bytes(const wpsgd_matrix *X) { return align256((size_t)X->m * 32); }

size_t wpsgd_run_delay_chains_workspace(const wpsgd_matrix *X, int k, int tau)
{
    if (check_matrix(X) != WPSGD_OK || !X->dense || k < 1 || tau < 0 || tau > kDelayMaxTau) return 0;
    return align256((size_t)k * sizeof(int64_t)) + align256(delay_ring_bytes(X, k, tau)) + delay_table_bytes(X);
}

int wpsgd_run_delay_chains(const wpsgd_matrix *X, const float *y, int k, const int64_t *n_samples,
                           double eta, double lambda, wpsgd_loss loss, uint64_t seed, int tau, int check,
                           const float *w_start, float *W, int64_t *accepted,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_matrix(X);
    if (rc != WPSGD_OK) return rc;
    if (!y || !W || !accepted || tau < 0) return WPSGD_INVALID_ARG;
    rc = check_steps(k, n_samples);
    if (rc != WPSGD_OK) return rc;
    if (!(eta > 0.0) || !(lambda >= 0.0) || !(eta * lambda < 1.0)) return WPSGD_INVALID_ARG;
    if (loss != WPSGD_HINGE && loss != WPSGD_LOGISTIC) return WPSGD_INVALID_ARG;
    if (!X->dense || tau > kDelayMaxTau) return WPSGD_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace % 256) != 0) return WPSGD_INVALID_ARG;
    if (workspace_bytes < wpsgd_run_delay_chains_workspace(X, k, tau)) return WPSGD_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(workspace);
    rc = upload(base, n_samples, (size_t)k * sizeof(int64_t), s);
    if (rc != WPSGD_OK) return rc;
    DelayArgs a{};
    a.dense = X->dense;
    a.ld = X->ld;
    a.y = y;
    a.m = X->m;
    a.d = X->d;
    a.k = k;
    a.n_samples = reinterpret_cast<const int64_t *>(base);
    a.w_start = w_start;
    a.eta = eta;
    a.lambda = lambda;
    a.loss = (int)loss;
    a.tau = tau;
    a.check = check != 0;
    a.seed_lo = (uint32_t)seed;
    a.seed_hi = (uint32_t)(seed >> 32);
    a.ring = reinterpret_cast<double *>(base + align256((size_t)k * sizeof(int64_t)));
    a.W = W;
    a.accepted = accepted;
    // The row table costs a pass over the whole data set: it pays when the servers together visit a
    // good part of the rows (the kernel that uses it is only chosen under the Check function).
    int64_t visits = 0;
    for (int i = 0; i < k; ++i) visits += std::min<int64_t>(n_samples[i], INT64_MAX / 2 / k);
    a.row_table = (check != 0 && visits >= X->m / 4)
                      ? base + align256((size_t)k * sizeof(int64_t)) + align256(delay_ring_bytes(X, k, tau))
                      : nullptr;
    const bool start_ok = !w_start || (uintptr_t)w_start % 4 == 0;
    if (!start_ok) return WPSGD_INVALID_ARG;
    hipError_t e = launch_delay_servers(a, (int)X->dtype, dense_vec(X), s);
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

int wpsgd_chains_status(const void *workspace, void *stream)
{
    if (!workspace) return WPSGD_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t word = 0;
    hipError_t e = hipMemcpyAsync(&word, workspace, sizeof(word), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e);
    return (word & 1u) ? WPSGD_INCOMPLETE : WPSGD_OK;
}

int wpsgd_weights_rate(int k, const int64_t *n_steps, double rate, double *a)
{
    int rc = check_steps(k, n_steps);
    if (rc != WPSGD_OK) return rc;
    if (!a || !(rate > 0.0) || !(rate <= 1.0)) return WPSGD_INVALID_ARG;
    int64_t t = 0;
    for (int i = 0; i < k; ++i) t = std::max(t, n_steps[i]);
    // rate^T = exp(T * log(rate)); the fastest chain has T = 0, so the sum is at least 1
    const double log_rate = std::log(rate);
    double total = 0.0;
    for (int i = 0; i < k; ++i) {
        a[i] = std::exp((double)(t - n_steps[i]) * log_rate);
        total += a[i];
    }
    for (int i = 0; i < k; ++i) a[i] /= total;
    return WPSGD_OK;
}

int wpsgd_weights(int k, const int64_t *n_steps, double eta, double lambda, double *a)
{
    if (!(eta > 0.0) || !(lambda >= 0.0) || !(eta * lambda < 1.0)) return WPSGD_INVALID_ARG;
    int rc = check_steps(k, n_steps);
    if (rc != WPSGD_OK) return rc;
    if (!a) return WPSGD_INVALID_ARG;
    int64_t t = 0;
    for (int i = 0; i < k; ++i) t = std::max(t, n_steps[i]);
    const double log_rate = std::log1p(-eta * lambda);    // log(1 - eta*lambda) without cancellation
    double total = 0.0;
    for (int i = 0; i < k; ++i) {
        a[i] = std::exp((double)(t - n_steps[i]) * log_rate);
        total += a[i];
    }
    for (int i = 0; i < k; ++i) a[i] /= total;
    return WPSGD_OK;
}

int wpsgd_benefit_margin(int k, const int64_t *n_steps, double rate, double *margin)
{
    int rc = check_steps(k, n_steps);
    if (rc != WPSGD_OK) return rc;
    if (!margin || !(rate > 0.0) || !(rate <= 1.0)) return WPSGD_INVALID_ARG;
    int64_t t = 0;
    for (int i = 0; i < k; ++i) t = std::max(t, n_steps[i]);
    const double log_rate = std::log(rate);
    double total = 0.0;
    for (int i = 0; i < k; ++i) total += std::exp((double)(t - n_steps[i]) * log_rate);
    *margin = 2.0 * total - (std::sqrt((double)k) + (double)k);
    return WPSGD_OK;
}

size_t wpsgd_combine_workspace(int k, int64_t d)
{
    (void)d;
    return k < 1 ? 0 : align256((size_t)k * sizeof(double));
}

int wpsgd_combine(const float *W, const double *a, int k, int64_t d, float *w_out, void *workspace,
                  size_t workspace_bytes, void *stream)
{
    if (!W || !a || !w_out || k < 1 || d < 1) return WPSGD_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace % 256) != 0) return WPSGD_INVALID_ARG;
    if (workspace_bytes < wpsgd_combine_workspace(k, d)) return WPSGD_WORKSPACE_TOO_SMALL;
    for (int i = 0; i < k; ++i)
        if (!std::isfinite(a[i])) return WPSGD_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = upload(workspace, a, (size_t)k * sizeof(double), s);
    if (rc != WPSGD_OK) return rc;
    hipError_t e = launch_combine(W, static_cast<const double *>(workspace), k, d, w_out, s);
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

size_t wpsgd_run_spans_workspace(const wpsgd_matrix *X, int k, wpsgd_loss loss, const wpsgd_plan *plan)
{
    const size_t chains = wpsgd_run_chains_workspace(X, k, loss, plan);
    if (chains == 0) return 0;
    return chains + align256((size_t)k * (size_t)X->d * sizeof(float)) + wpsgd_combine_workspace(k, X->d);
}

int wpsgd_run_spans(const wpsgd_matrix *X, const float *y, int k, const int64_t *steps_per_span, int64_t n_spans,
                    double eta, double lambda, wpsgd_loss loss, uint64_t seed, wpsgd_sampling sampling,
                    const float *w_start, float *w_out, void *workspace, size_t workspace_bytes,
                    const wpsgd_plan *plan, void *stream)
{
    int rc = check_matrix(X);
    if (rc != WPSGD_OK) return rc;
    rc = check_steps(k, steps_per_span);
    if (rc != WPSGD_OK) return rc;
    if (!w_out || n_spans < 1) return WPSGD_INVALID_ARG;
    int64_t span = 0;
    for (int i = 0; i < k; ++i) span = std::max(span, steps_per_span[i]);
    if (span < 1 || span > ((int64_t)1 << 62) / n_spans) return WPSGD_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace % 256) != 0) return WPSGD_INVALID_ARG;
    // the chains' workspace comes first, so that its status word is the first word of this one too
    const size_t chains = wpsgd_run_chains_workspace(X, k, loss, plan);
    const size_t models = align256((size_t)k * (size_t)X->d * sizeof(float));
    const size_t average = wpsgd_combine_workspace(k, X->d);
    if (chains == 0) return WPSGD_UNSUPPORTED;
    if (workspace_bytes < chains + models + average) return WPSGD_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    float *W = reinterpret_cast<float *>(ws + chains);
    std::vector<double> a(k);
    rc = wpsgd_weights(k, steps_per_span, eta, lambda, a.data());
    if (rc != WPSGD_OK) return rc;
    std::vector<int64_t> first(k);
    for (int64_t sp = 0; sp < n_spans; ++sp) {
        for (int i = 0; i < k; ++i) first[i] = sp * steps_per_span[i];
        rc = run_chains_from(X, y, k, steps_per_span, eta, lambda, loss, seed, sampling, sp == 0 ? w_start : w_out,
                             first.data(), W, ws, chains, plan, stream, sp > 0);
        if (rc != WPSGD_OK) return rc;
        if (sp == 0) {          // (this call also carries the weights to the device; they stay there for the spans to come)
            rc = wpsgd_combine(W, a.data(), k, X->d, w_out, ws + chains + models, average, stream);
            if (rc != WPSGD_OK) return rc;
        } else {
            hipError_t e = launch_combine(W, reinterpret_cast<const double *>(ws + chains + models), k, X->d, w_out,
                                          static_cast<hipStream_t>(stream));
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    return WPSGD_OK;
}

int wpsgd_span_condition(int k, const int64_t *steps_per_span, double rate, double *value)
{
    int rc = check_steps(k, steps_per_span);
    if (rc != WPSGD_OK) return rc;
    if (!value || !(rate > 0.0) || !(rate <= 1.0)) return WPSGD_INVALID_ARG;
    int64_t span = 0;
    for (int i = 0; i < k; ++i) span = std::max(span, steps_per_span[i]);
    const double log_rate = std::log(rate);
    double total = 0.0;
    for (int i = 0; i < k; ++i) total += std::exp((double)(span - steps_per_span[i]) * log_rate);
    *value = (double)k / total * std::exp((double)span * log_rate);
    return WPSGD_OK;
}

size_t wpsgd_objective_workspace(const wpsgd_matrix *X)
{
    if (check_matrix(X) != WPSGD_OK) return 0;
    return align256(objective_partials_bytes(X->m));
}

static int objective_check(const wpsgd_matrix *X, const float *y, const float *w, double lambda, wpsgd_loss loss,
                           const double *out)
{
    int rc = check_matrix(X);
    if (rc != WPSGD_OK) return rc;
    if (!y || !w || !out || !(lambda >= 0.0)) return WPSGD_INVALID_ARG;
    if (loss != WPSGD_HINGE && loss != WPSGD_LOGISTIC) return WPSGD_INVALID_ARG;
    if ((uintptr_t)out % sizeof(double) != 0) return WPSGD_INVALID_ARG;
    if (X->d >= (1ll << 29)) return WPSGD_UNSUPPORTED;           // 32-bit byte offsets into a row and into w
    return WPSGD_OK;
}

static int objective_launch(const wpsgd_matrix *X, const float *y, const float *w, double lambda, wpsgd_loss loss,
                            double *out, double *partials, hipStream_t s)
{
    ChainArgs a{};
    a.dense = X->dense;
    a.ld = X->ld;
    a.row_ptr = X->row_ptr;
    a.col_idx = X->col_idx;
    a.vals = X->vals;
    a.y = y;
    a.m = X->m;
    a.d = X->d;
    int vec = 1;
    if (X->dense && (uintptr_t)w % 16 == 0) vec = dense_vec(X);
    hipError_t e = launch_objective(a, X->dense ? (int)X->dtype : WPSGD_F32, vec, (int)loss, w, lambda, partials, out, s);
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

int wpsgd_objective(const wpsgd_matrix *X, const float *y, const float *w, double lambda, wpsgd_loss loss,
                    double *out, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = objective_check(X, y, w, lambda, loss, out);
    if (rc != WPSGD_OK) return rc;
    if (!workspace || ((uintptr_t)workspace % 256) != 0) return WPSGD_INVALID_ARG;
    if (workspace_bytes < wpsgd_objective_workspace(X)) return WPSGD_WORKSPACE_TOO_SMALL;
    return objective_launch(X, y, w, lambda, loss, out, static_cast<double *>(workspace), static_cast<hipStream_t>(stream));
}

int wpsgd_objective_static(const wpsgd_matrix *X, const float *y, const float *w, double lambda, wpsgd_loss loss,
                           double *out, void *stream)
{
    int rc = objective_check(X, y, w, lambda, loss, out);
    if (rc != WPSGD_OK) return rc;
    double *partials = nullptr;          // the library's own area on this device, in place of a workspace
    size_t room = 0;
    hipError_t e = objective_static_partials(&partials, &room);
    if (e != hipSuccess) return hip_fail(e);
    if (objective_partials_bytes(X->m) > room) return WPSGD_UNSUPPORTED;     // more partial sums than that area holds
    return objective_launch(X, y, w, lambda, loss, out, partials, static_cast<hipStream_t>(stream));
}

int wpsgd_sample_indices(uint64_t seed, int chain, int64_t n0, int64_t count, int64_t m,
                         int64_t *out_host)
{
    if (chain < 0 || n0 < 0 || count < 0 || m < 1 || m > 0xFFFFFFFFLL) return WPSGD_INVALID_ARG;
    if (count > 0 && !out_host) return WPSGD_INVALID_ARG;
    for (int64_t t = 0; t < count; ++t)
        out_host[t] = (int64_t)sample_row((uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32),
                                          (uint32_t)chain, (uint64_t)(n0 + t), (uint32_t)m);
    return WPSGD_OK;
}

int wpsgd_sample_indices_device(uint64_t seed, int chain, int64_t n0, int64_t count, int64_t m,
                                int64_t *out_device, void *stream)
{
    if (chain < 0 || n0 < 0 || count < 0 || m < 1 || m > 0xFFFFFFFFLL) return WPSGD_INVALID_ARG;
    if (count > 0 && !out_device) return WPSGD_INVALID_ARG;
    hipError_t e = launch_sample_rows((uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32),
                                      (uint32_t)chain, n0, count, (uint32_t)m, 0u, out_device,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

int wpsgd_shard_indices(uint64_t seed, int chain, int k, int64_t n0, int64_t count, int64_t m,
                        int64_t *out_host)
{
    if (chain < 0 || k < 1 || chain >= k || n0 < 0 || count < 0 || m < 1 || m > 0xFFFFFFFFLL || (int64_t)k > m)
        return WPSGD_INVALID_ARG;
    if (count > 0 && !out_host) return WPSGD_INVALID_ARG;
    for (int64_t t = 0; t < count; ++t)
        out_host[t] = (int64_t)shard_row((uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32), (uint32_t)chain,
                                         (uint32_t)k, (uint64_t)(n0 + t), (uint32_t)m);
    return WPSGD_OK;
}

int wpsgd_shard_indices_device(uint64_t seed, int chain, int k, int64_t n0, int64_t count, int64_t m,
                               int64_t *out_device, void *stream)
{
    if (chain < 0 || k < 1 || chain >= k || n0 < 0 || count < 0 || m < 1 || m > 0xFFFFFFFFLL || (int64_t)k > m)
        return WPSGD_INVALID_ARG;
    if (count > 0 && !out_device) return WPSGD_INVALID_ARG;
    hipError_t e = launch_sample_rows((uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32),
                                      (uint32_t)chain, n0, count, (uint32_t)m, (uint32_t)k, out_device,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

int wpsgd_stream_rows(const wpsgd_matrix *X, int groups, int64_t rows_per_group, uint64_t seed,
                      float *sink, void *stream)
{
    int rc = check_matrix(X);
    if (rc != WPSGD_OK) return rc;
    if (!X->dense || !sink || groups < 1 || rows_per_group < 1) return WPSGD_INVALID_ARG;
    const int64_t elem = X->dtype == WPSGD_BF16 ? 2 : 4;
    const int64_t row_bytes = X->d * elem;
    // 16-byte loads: rows must start on 16-byte boundaries and be a whole number of them
    if ((uintptr_t)X->dense % 16 != 0 || (X->ld * elem) % 16 != 0 || row_bytes % 16 != 0 ||
        row_bytes > 0x7FFFFFFF)
        return WPSGD_UNSUPPORTED;
    hipError_t e = launch_stream_rows(X->dense, X->ld * elem, (uint32_t)row_bytes, (uint32_t)X->m, groups,
                                      rows_per_group, (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32),
                                      sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? WPSGD_OK : hip_fail(e);
}

const char *wpsgd_strerror(int status)
{
    switch (status) {
    case WPSGD_OK: return "ok";
    case WPSGD_INVALID_ARG: return "invalid argument";
    case WPSGD_HIP_ERROR: return "HIP call failed (see wpsgd_last_hip_error)";
    case WPSGD_WORKSPACE_TOO_SMALL: return "workspace too small";
    case WPSGD_UNSUPPORTED: return "no kernel implements the forced plan";
    case WPSGD_INCOMPLETE: return "chains cut into column slices gave up waiting for each other; their rows of W are NaN";
    default: return "unknown status";
    }
}

int wpsgd_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
