// Sparse-row (CSR) SGD chains.  One wavefront runs one chain; the model vector lives in HBM
// (the workspace) because a text-like feature space (d ~ 10^6) fits no on-chip store.  The
// lambda-shrink of Eq. 5 never touches the vector: w = s*v with the fp64 scalar s absorbing
// (1 - eta*lambda) each step, so a step costs O(nnz of the row): gather v at the row's
// columns, reduce, scatter the rank-one update back.
#include "device_utils.h"
#include "internal.h"

namespace wpsgd {

constexpr int kCsrChunks = 4;   // entries of a row kept in registers between gather and scatter: 4*64

template <int LOSS>
__global__ __launch_bounds__(kWave) void chain_csr_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    const int lane = threadIdx.x;
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const int64_t d = a.d;
    TV *v = static_cast<TV *>(a.state) + (int64_t)chain * d;

    for (int64_t col = lane; col < d; col += kWave) v[col] = a.w_start ? (TV)a.w_start[col] : (TV)0;
    __syncthreads();   // the start values must be visible to whichever lane gathers them later
    const int64_t step0 = a.step0[blockIdx.x];

    RowWindow win;
    win.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m, a.perm, (uint32_t)a.k);
    double s = 1.0, inv_s = 1.0;
    const double rho = a.rho, inv_rho = 1.0 / a.rho, eta = a.eta;

    for (int64_t step = 0; step < n; ++step) {
        const uint32_t row = win.get(step0 + step);
        const int64_t lo = a.row_ptr[row], hi = a.row_ptr[(int64_t)row + 1];
        const double y = (double)a.y[row];

        int32_t col[kCsrChunks];
        float val[kCsrChunks];
        TV acc = (TV)0;
#pragma unroll
        for (int c = 0; c < kCsrChunks; ++c) {
            const int64_t p = lo + c * kWave + lane;
            col[c] = 0;
            val[c] = 0.0f;
            if (p < hi) {
                col[c] = a.col_idx[p];
                val[c] = a.vals[p];
                acc += v[col[c]] * (TV)val[c];
            }
        }
        for (int64_t p = lo + kCsrChunks * kWave + lane; p < hi; p += kWave)   // very long rows
            acc += v[a.col_idx[p]] * (TV)a.vals[p];
        acc = wave_sum(acc);

        const double slope = loss_slope<LOSS>(y, s * (double)acc);
        s *= rho;
        inv_s *= inv_rho;
        const TV coef = (TV)(-eta * slope * inv_s);
        if (coef != (TV)0) {
#pragma unroll
            for (int c = 0; c < kCsrChunks; ++c) {
                const int64_t p = lo + c * kWave + lane;
                if (p < hi) v[col[c]] += coef * (TV)val[c];     // columns are distinct inside a row
            }
            for (int64_t p = lo + kCsrChunks * kWave + lane; p < hi; p += kWave)
                v[a.col_idx[p]] += coef * (TV)a.vals[p];
            __syncthreads();   // another lane may gather these columns at the next step
        }
        if (s < 0x1p-30) {
            for (int64_t c2 = lane; c2 < d; c2 += kWave) v[c2] *= (TV)s;
            s = 1.0;
            inv_s = 1.0;
            __syncthreads();
        }
    }

    float *out = a.W + (int64_t)chain * d;
    for (int64_t c2 = lane; c2 < d; c2 += kWave) out[c2] = (float)(s * (double)v[c2]);
}

// ---------------------------------------------------------------------------------------------
// The fast CSR kernel.  Same recursion; what changes is where the model vector is read from.
//
//  * Columns below kHead (the hot head of a Zipf-like feature space) live in LDS for the whole
//    chain: one wavefront's LDS accesses are ordered, so a step sees the previous step's update
//    without waiting for memory.
//  * The other columns stay in HBM.  The rows a chain visits are known ahead of time, so their
//    entries (column, value) are requested 2Q steps ahead and the model values at their tail
//    columns Q steps ahead; both wait in registers.  A value fetched early is stale if one of
//    the steps in between wrote the same column.  Every tail write leaves the step number in
//    two small LDS tables, indexed by two different hashes of the column; a step whose tail
//    column finds a recent step number in both (a real conflict, or - rarely - two unrelated
//    aliases at once) drains the memory queue and reads its tail values again.  No false
//    negatives: a write always leaves both stamps.
//  * Nothing in the loop is conditional on data except that re-read, which is written with
//    inline memory instructions so that the compiler's count of outstanding loads - and with it
//    the partial waits that keep the prefetch alive - is the same on both paths.
//
// When is a prefetched value safe?  Loads and stores of one wave complete in issue order.  The
// entry loads of step t+2Q are issued after the stores of step t and are waited for at step
// t+Q (when the tail values of step t+2Q are requested), so at any step i all stores of steps
// <= i-Q are complete, and a tail value requested at step i for step i+Q can only miss writes
// of steps i-Q+1 .. i+Q-1: the 2Q-1 steps before the one that uses it.  The stamp test covers
// exactly those.
// ---------------------------------------------------------------------------------------------
constexpr int kHead = 8192;            // columns kept in LDS
constexpr int kStamps = 16384;         // entries of each of the two stamp tables (16-bit step numbers)
constexpr int kQ = 4;                  // prefetch distance of tail values, in steps
constexpr int kRing = 2 * kQ;          // prefetch distance of row entries
constexpr int kRowChunks = 2;          // entries of a row held in registers: 2*64

// Memory instructions the compiler does not see.  Each one drains the queue, so the value is
// there (or the store is done) when the statement ends; used only off the fast path.
__device__ inline uint32_t hidden_load_u32(const void *p)
{
    uint32_t r;
    asm volatile("s_waitcnt vmcnt(0)\n\tglobal_load_dword %0, %1, off\n\ts_waitcnt vmcnt(0)"
                 : "=v"(r) : "v"(p) : "memory");
    return r;
}
__device__ inline float hidden_load(const float *p) { return __uint_as_float(hidden_load_u32(p)); }
__device__ inline double hidden_load(const double *p)
{
    double r;
    asm volatile("s_waitcnt vmcnt(0)\n\tglobal_load_dwordx2 %0, %1, off\n\ts_waitcnt vmcnt(0)"
                 : "=v"(r) : "v"(p) : "memory");
    return r;
}
__device__ inline void hidden_store(float *p, float x)
{
    asm volatile("global_store_dword %0, %1, off\n\ts_waitcnt vmcnt(0)" : : "v"(p), "v"(x) : "memory");
}
__device__ inline void hidden_store(double *p, double x)
{
    asm volatile("global_store_dwordx2 %0, %1, off\n\ts_waitcnt vmcnt(0)" : : "v"(p), "v"(x) : "memory");
}

template <int LOSS>
__global__ __launch_bounds__(kWave) void chain_csr_cached_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    __shared__ TV head[kHead];
    __shared__ uint16_t stamps[2][kStamps];

    const int lane = threadIdx.x;
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const int64_t d = a.d;
    TV *v = static_cast<TV *>(a.state) + (int64_t)chain * d;
    float *out = a.W + (int64_t)chain * d;
    const int64_t nnz = a.row_ptr[a.m];

    const int64_t step0 = a.step0[blockIdx.x];
    if (nnz == 0) {                     // no entries at all: every step only shrinks the start vector
        double s_all = 1.0, pw = a.rho;
        for (int64_t e = n; e > 0; e >>= 1) {
            if (e & 1) s_all *= pw;
            pw *= pw;
        }
        for (int64_t c = lane; c < d; c += kWave) out[c] = a.w_start ? (float)(s_all * (double)a.w_start[c]) : 0.0f;
        return;
    }
    if (n == 0) {                       // no steps: the chain returns its start vector
        for (int64_t c = lane; c < d; c += kWave) out[c] = a.w_start ? a.w_start[c] : 0.0f;
        return;
    }
    for (int c = lane; c < kHead; c += kWave) head[c] = (a.w_start && c < d) ? (TV)a.w_start[c] : (TV)0;
    for (int c = lane; c < 2 * kStamps; c += kWave) (&stamps[0][0])[c] = 0;
    for (int64_t c = kHead + lane; c < d; c += kWave) v[c] = a.w_start ? (TV)a.w_start[c] : (TV)0;
    TV *dump = v + lane;                // per-lane scratch target for stores that must not count
                                        // (head columns of v are unused while the chain runs)
    __syncthreads();

    const uint32_t seed_lo = a.seed_lo, seed_hi = a.seed_hi, m32 = (uint32_t)a.m;
    const double rho = a.rho, inv_rho = 1.0 / a.rho;
    double rho_pow = 1.0, inv_rho_pow1 = inv_rho, rho64 = rho, inv_rho64 = inv_rho;
#pragma unroll
    for (int bit = 0; bit < 6; ++bit) {
        if ((lane >> bit) & 1) {
            rho_pow *= rho64;
            inv_rho_pow1 *= inv_rho64;
        }
        rho64 *= rho64;
        inv_rho64 *= inv_rho64;
    }
    double s_w = 1.0, eos_w = a.eta;

    // per-lane tables of the current window (a) and the next one (b): first entry and length of
    // the row each step visits; labels and scale factors of the current window only
    int64_t lo_a, lo_b;
    int len_a, len_b;
    float y_b;
    TV zs_tab = (TV)0, cs_tab = (TV)0;
    auto load_window = [&](int64_t w, int64_t &lo, int &len, float &y) {
        const uint32_t row = sample_window(seed_lo, seed_hi, (uint32_t)chain, step0 + w * kWave, m32, a.perm, (uint32_t)a.k);
        const int64_t p0 = a.row_ptr[row], p1 = a.row_ptr[(int64_t)row + 1];
        lo = p0;
        len = (int)(p1 - p0);
        y = a.y[row];
    };
    float y_a;
    load_window(0, lo_a, len_a, y_a);
    load_window(1, lo_b, len_b, y_b);

    int32_t colr[kRing][kRowChunks];
    float valr[kRing][kRowChunks];
    TV vr[kQ][kRowChunks];

    // entries of the row visited at in-window position jj (0..127) -> ring slot
    auto request_entries = [&](int slot, int jj) {
        const int64_t lo = jj < kWave ? lane_read_i64(lo_a, jj) : lane_read_i64(lo_b, jj - kWave);
        const int len = jj < kWave ? __builtin_amdgcn_readlane(len_a, jj) : __builtin_amdgcn_readlane(len_b, jj - kWave);
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) {
            const int e = c * kWave + lane;
            const int64_t p = e < len ? lo + e : 0;       // past the row: re-read entry 0 (discarded)
            colr[slot][c] = a.col_idx[p];
            valr[slot][c] = a.vals[p];
        }
    };
    auto row_len = [&](int jj) {
        return jj < kWave ? __builtin_amdgcn_readlane(len_a, jj) : __builtin_amdgcn_readlane(len_b, jj - kWave);
    };
    // tail values of the row whose entries sit in ring slot `slot`
    auto request_tail = [&](int vslot, int slot, int len) {
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) {
            const int e = c * kWave + lane;
            const int32_t col = colr[slot][c];
            const bool tail = e < len && col >= kHead;
            vr[vslot][c] = tail ? v[col] : dump[0];
        }
    };

    const uint16_t kWindowSteps = 2 * kQ;
    // the two stamp slots of a column: columns that share the first differ in the second
    auto slot_a = [](int32_t col) { return col & (kStamps - 1); };
    auto slot_b = [](int32_t col) { return (int)(((uint32_t)col + ((uint32_t)col >> 14) * 2731u) & (kStamps - 1)); };
    // One step at in-window position j, absolute step number `step`.
    auto do_step = [&](int slot, int vslot, int j, int64_t step) {
        const int len = row_len(j);
        const uint16_t now = (uint16_t)step;
        int32_t col[kRowChunks];
        float val[kRowChunks];
        TV vv[kRowChunks];
        bool is_head[kRowChunks], is_tail[kRowChunks];
        bool stale = false;
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) {
            const int e = c * kWave + lane;
            const bool in = e < len;
            col[c] = colr[slot][c];
            val[c] = in ? valr[slot][c] : 0.0f;
            is_head[c] = in && col[c] < kHead;
            is_tail[c] = in && col[c] >= kHead;
            const TV hv = head[is_head[c] ? col[c] : 0];
            const uint16_t sa = stamps[0][is_tail[c] ? slot_a(col[c]) : 0];
            const uint16_t sb = stamps[1][is_tail[c] ? slot_b(col[c]) : 0];
            vv[c] = is_head[c] ? hv : (is_tail[c] ? vr[vslot][c] : (TV)0);
            stale = stale || (is_tail[c] && (uint16_t)(now - sa) < kWindowSteps && (uint16_t)(now - sb) < kWindowSteps);
        }
        if (__any(stale)) {             // drain, then read this step's tail values again
#pragma unroll
            for (int c = 0; c < kRowChunks; ++c) {
                const TV fresh = hidden_load(is_tail[c] ? v + col[c] : dump);
                if (is_tail[c]) vv[c] = fresh;
            }
        }
        TV acc = (TV)0;
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) acc += vv[c] * (TV)val[c];
        // rows longer than the register window: the rest of the row, one entry per lane at a time
        for (int e0 = kRowChunks * kWave; e0 < len; e0 += kWave) {
            const int e = e0 + lane;
            const int64_t lo = lane_read_i64(lo_a, j);
            const bool in = e < len;
            const int32_t xc = (int32_t)hidden_load_u32(a.col_idx + (in ? lo + e : 0));
            const float xv = hidden_load(a.vals + (in ? lo + e : 0));
            const TV cur = (in && xc < kHead) ? head[xc] : hidden_load(in ? v + xc : dump);
            if (in) acc += cur * (TV)xv;
        }
        const TV zs = lane_read(zs_tab, j), cs = lane_read(cs_tab, j);      // label folded in
        TV coef;
        if constexpr (LOSS == kLossHinge) {
            coef = lane63_below_one(zs, wave_sum_lane63(acc)) ? cs : 0.0;
        } else {
            acc = wave_sum(acc);
            coef = cs * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(zs * acc));
        }
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) {
            const TV nv = vv[c] + coef * (TV)val[c];
            if (is_head[c]) head[col[c]] = nv;
            if (is_tail[c]) {
                stamps[0][slot_a(col[c])] = now;
                stamps[1][slot_b(col[c])] = now;
            }
            *(is_tail[c] ? v + col[c] : dump) = nv;       // one store per chunk, whatever the data
        }
        for (int e0 = kRowChunks * kWave; e0 < len; e0 += kWave) {
            const int e = e0 + lane;
            const int64_t lo = lane_read_i64(lo_a, j);
            const bool in = e < len;
            const int32_t xc = (int32_t)hidden_load_u32(a.col_idx + (in ? lo + e : 0));
            const float xv = hidden_load(a.vals + (in ? lo + e : 0));
            if (in && xc < kHead) {
                head[xc] += coef * (TV)xv;
            } else {
                const TV cur = hidden_load(in ? v + xc : dump);
                hidden_store(in ? v + xc : dump, in ? cur + coef * (TV)xv : cur);
                if (in) {
                    stamps[0][slot_a(xc)] = now;
                    stamps[1][slot_b(xc)] = now;
                }
            }
        }
    };

    // prologue: entries of steps 0..2Q-1, tail values of steps 0..Q-1
#pragma unroll
    for (int t = 0; t < kRing; ++t) request_entries(t, t);
#pragma unroll
    for (int t = 0; t < kQ; ++t) request_tail(t, t, row_len(t));
    __builtin_amdgcn_s_waitcnt(0x0F70);

    const int64_t ngroups = (n + kRing - 1) / kRing;
    int j0 = 0;
    for (int64_t g = 0; g < ngroups; ++g) {
        if (j0 == 0) {      // new window of 64 steps
            const int64_t w = g * kRing / kWave;
            if (w > 0) {
                s_w *= rho64;
                eos_w *= inv_rho64;
                lo_a = lo_b;
                len_a = len_b;
                y_a = y_b;
                load_window(w + 1, lo_b, len_b, y_b);
            }
            const double sl = s_w * rho_pow, el = eos_w * inv_rho_pow1;
            const bool live = w * kWave + lane < n;
            const double yd = (double)y_a;
            if constexpr (LOSS == kLossHinge) {
                zs_tab = yd * sl;
                cs_tab = live ? yd * el : 0.0;
            } else {
                zs_tab = (float)(yd * sl * 1.4426950408889634);
                cs_tab = live ? (float)(yd * el) : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
            const int j = j0 + u;
            do_step(u, u % kQ, j, g * kRing + u);
            request_entries(u, j + kRing);                                     // step +2Q
            request_tail(u % kQ, (u + kQ) % kRing, row_len(j + kQ));           // step +Q
        }
        j0 = (j0 + kRing) & (kWave - 1);
    }

    __syncthreads();        // all tail stores done before the vector is read back
    const int64_t last_w = (n - 1) / kWave;
    const int rem = (int)(n - last_w * kWave);
    const double s_end = s_w * lane_read(rho_pow, rem - 1) * rho;
    for (int c = lane; c < kHead && c < d; c += kWave) out[c] = (float)(s_end * (double)head[c]);
    for (int64_t c = kHead + lane; c < d; c += kWave) out[c] = (float)(s_end * (double)v[c]);
}

hipError_t launch_csr(const Plan &p, const ChainArgs &a, hipStream_t s)
{
    if (p.prefetch == 8) return launch_csr_pair(p, a, s);
    if (p.prefetch > 1) {       // the cached kernel (its lazy scale is never folded: see the planner)
        if (p.loss == WPSGD_HINGE)
            hipLaunchKernelGGL((chain_csr_cached_kernel<kLossHinge>), dim3(a.k), dim3(kWave), 0, s, a);
        else
            hipLaunchKernelGGL((chain_csr_cached_kernel<kLossLogistic>), dim3(a.k), dim3(kWave), 0, s, a);
        return hipGetLastError();
    }
    if (p.loss == WPSGD_HINGE)
        hipLaunchKernelGGL((chain_csr_kernel<kLossHinge>), dim3(a.k), dim3(kWave), 0, s, a);
    else
        hipLaunchKernelGGL((chain_csr_kernel<kLossLogistic>), dim3(a.k), dim3(kWave), 0, s, a);
    return hipGetLastError();
}

}  // namespace wpsgd
