// Delay SGD under the Check function (Section IV, Algorithms 3 and 4; Lemma 4): one workgroup is one
// server.  It keeps the accepted iterates w_{J-reach} .. w_J (reach = max(tau, 1)) and room for one
// candidate as a ring of fp64 vectors in the workspace.  Every thread owns the same columns of every
// vector in every pass, so the ring needs no synchronisation of its own; it is re-read every sample
// and stays in the cache of the compute unit's XCD.
//
// Per sample x (one row of the data set), one pass over the row forms beta^2 = x.x and the projections
// L_t = w_t.x of the iterates the delayed gradient spans.  From those scalars alone every thread takes
// the same decision: the slope u at w_{J-tau}, the triples of the first call of Check, and the triple
// (w_{J-1}, w_J, candidate) of the second call, whose third projection follows from the update rule,
//     L_c = L_J - eta*lambda*L_{J-tau} - eta*u*beta^2,
// so a sample that is thrown away costs no second pass.  Only an accepted candidate is written:
//     w_{J+1} = w_J - eta*lambda*w_{J-tau} - eta*u*x          (the recurrence in the proof of Lemma 4)
// together with its squared length, which later tests need for the part across a sample,
// |w|^2 - L^2/beta^2.  All arithmetic is fp64; the result is rounded to fp32 once, at the end.
//
// Four kernels.  delay_server_reg_kernel holds the ring in registers, newest iterate first, and shifts
// it when a candidate is accepted; the rows of the next samples (which do not depend on what is
// accepted) are requested PF samples ahead, so a sample costs the pass over its row, one exchange of
// sums and the decision.  It covers rows of up to 256 x EPT aligned elements and delays up to 4.
// For the same shapes, delay_server_batch_kernel decides B samples per exchange under the Check
// function, where nearly every sample is thrown away, and delay_server_plain_kernel takes tau + 1 samples
// per exchange without it, where the delay makes their gradients independent; both stage rows in LDS.
// delay_server_kernel keeps the ring in the workspace and covers everything else.
#include <atomic>

#include "dense_rows.h"
#include "device_utils.h"
#include "internal.h"

namespace wpsgd {
namespace {

constexpr int kDelayThreads = 256;
constexpr int kDelayWaves = kDelayThreads / kWave;

template <typename TX, int VEC> struct DelayRow;
template <> struct DelayRow<float, 1> {
    double x[1];
    __device__ void load(const float *p) { x[0] = (double)p[0]; }
};
template <> struct DelayRow<float, 4> {
    double x[4];
    __device__ void load(const float *p)
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        x[0] = (double)q.x; x[1] = (double)q.y; x[2] = (double)q.z; x[3] = (double)q.w;
    }
};
template <> struct DelayRow<uint16_t, 1> {
    double x[1];
    __device__ void load(const uint16_t *p) { x[0] = (double)bf16_one(p[0]); }
};
template <> struct DelayRow<uint16_t, 8> {
    double x[8];
    __device__ void load(const uint16_t *p)
    {
        const uint4 q = *reinterpret_cast<const uint4 *>(p);
        x[0] = (double)bf16_lo(q.x); x[1] = (double)bf16_hi(q.x); x[2] = (double)bf16_lo(q.y); x[3] = (double)bf16_hi(q.y);
        x[4] = (double)bf16_lo(q.z); x[5] = (double)bf16_hi(q.z); x[6] = (double)bf16_lo(q.w); x[7] = (double)bf16_hi(q.w);
    }
};

// N fp64 wave sums at once, level by level: the moves of one level are independent of each other, so
// none has to wait for the addition before it (a DPP operand written by the instruction just before
// costs idle slots).  Per value the additions and their order are those of wave_sum_lane63; the
// totals are valid in lane 63.
template <int CTRL, int N>
__device__ inline void wave_sums_level(double (&v)[N], int count)
{
    double moved[N];
#pragma unroll
    for (int t = 0; t < N; ++t)
        if (t < count) moved[t] = dpp_move<CTRL, 0xF>(v[t]);
#pragma unroll
    for (int t = 0; t < N; ++t)
        if (t < count) v[t] += moved[t];
}
template <int N>
__device__ inline void wave_sums_lane63(double (&v)[N], int count)
{
    wave_sums_level<0xB1>(v, count);
    wave_sums_level<0x4E>(v, count);
    wave_sums_level<0x141>(v, count);
    wave_sums_level<0x140>(v, count);
    wave_sums_level<0x142>(v, count);
    wave_sums_level<0x143>(v, count);
}

// One triple of Algorithm 4: the newest projection must lie between the middle one and
// Length_min = (L_b - rate*L_a)/(1 - rate), ends included, and the part of the middle iterate across
// the sample (squared length pb) must not be longer than that of the oldest (pa).
__device__ inline bool check_triple(double La, double Lb, double Lc, double pa, double pb, double rate)
{
    if (!(rate < 1.0)) return false;
    const double Lmin = (Lb - rate * La) / (1.0 - rate);
    const double lo = Lmin < Lb ? Lmin : Lb, hi = Lmin < Lb ? Lb : Lmin;
    return lo <= Lc && Lc <= hi && !(pb > pa);
}

// The two halves of that test without a division, as the register kernel takes them (rate < 1 and
// beta2 > 0 are the caller's business; only comparisons that sit within rounding of a tie can differ).
// Between L_b and Length_min: multiply the three numbers by 1 - rate > 0.
__device__ inline bool inside_interval(double La, double Lb, double Lc, double rate)
{
    const double s = 1.0 - rate;
    const double e0 = s * Lb, e1 = Lb - rate * La, c = s * Lc;
    const double lo = e1 < e0 ? e1 : e0, hi = e1 < e0 ? e0 : e1;
    return (lo <= c) & (c <= hi);
}
// |b|^2 - L_b^2/beta2 <= |a|^2 - L_a^2/beta2, multiplied by beta2.
__device__ inline bool across_does_not_grow(double La, double Lb, double na2, double nb2, double beta2)
{
    return !((nb2 - na2) * beta2 > Lb * Lb - La * La);
}

// base^(1/REACH) for the delays the register kernel covers, by square and cube roots.
template <int REACH>
__device__ inline double delay_root(double base)
{
    if constexpr (REACH == 1) return base;
    else if constexpr (REACH == 2) return sqrt(base);
    else if constexpr (REACH == 3) return cbrt(base);
    else if constexpr (REACH == 4) return sqrt(sqrt(base));
    else return pow(base, 1.0 / (double)REACH);
}

// MAXW: how many iterates one pass can project (reach + 1 are needed).
template <typename TX, int VEC, int MAXW>
__global__ __launch_bounds__(kDelayThreads) void delay_server_kernel(DelayArgs a)
{
    constexpr int NT = kDelayThreads, NW = kDelayWaves;
    __shared__ double red[2][NW][MAXW + 1];
    __shared__ double nrm[MAXW + 1];               // squared lengths of the ring's vectors, by slot

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int chain = blockIdx.x;
    const int64_t n = a.n_samples[chain];
    const int64_t d = a.d;
    const int reach = a.tau > 1 ? a.tau : 1;
    const int slots = reach + 2;
    const TX *X = static_cast<const TX *>(a.dense);
    double *ring = a.ring + (int64_t)chain * slots * d;
    const double eta = a.eta, eta_lambda = a.eta * a.lambda;
    int parity = 0;

    // sums `count` values per thread over the workgroup; every thread receives the same totals
    auto block_sums = [&](double(&v)[MAXW + 1], int count) {
#pragma unroll
        for (int t = 0; t <= MAXW; ++t)
            if (t < count) {
                const double w = wave_sum_lane63(v[t]);
                if (lane == kWave - 1) red[parity][wave][t] = w;
            }
        __syncthreads();
#pragma unroll
        for (int t = 0; t <= MAXW; ++t)
            if (t < count) {
                double sum = red[parity][0][t];
#pragma unroll
                for (int w = 1; w < NW; ++w) sum += red[parity][w][t];
                v[t] = sum;
            }
        parity ^= 1;
    };

    {   // w_0 and its squared length
        double v[MAXW + 1];
        v[0] = 0.0;
        for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC)
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const double w = a.w_start ? (double)a.w_start[col + j] : 0.0;
                ring[col + j] = w;
                v[0] += w * w;
            }
        block_sums(v, 1);
        if (tid == 0) nrm[0] = v[0];
    }

    RowWindow win;
    win.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m);
    int64_t J = 0;                                  // accepted updates so far

    for (int64_t s = 0; s < n; ++s) {
        const uint32_t row = win.get(s);
        const TX *xr = X + (int64_t)row * a.ld;
        const double y = (double)a.y[row];
        const int64_t at = J - a.tau > 0 ? J - a.tau : 0;          // where the gradient is evaluated
        // iterates to project: w_{J-reach} .. w_J under Check, w_{J-tau} alone without it
        const int64_t first = a.check ? (J - reach > 0 ? J - reach : 0) : at;
        const int nwin = a.check ? (int)(J - first) + 1 : 1;
        int64_t off[MAXW];
#pragma unroll
        for (int t = 0; t < MAXW; ++t) off[t] = (int64_t)((first + t) % slots) * d;

        double v[MAXW + 1];                          // v[t] = w_{first+t}.x, v[MAXW] = x.x
#pragma unroll
        for (int t = 0; t <= MAXW; ++t) v[t] = 0.0;
        for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC) {
            DelayRow<TX, VEC> c;
            c.load(xr + col);
#pragma unroll
            for (int j = 0; j < VEC; ++j) v[MAXW] += c.x[j] * c.x[j];
#pragma unroll
            for (int t = 0; t < MAXW; ++t)
                if (t < nwin) {
                    const double *w = ring + off[t] + col;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) v[t] += w[j] * c.x[j];
                }
        }
        // the totals are wanted in v[0..nwin) and v[MAXW]; move x.x next to the projections
        {
            const double b = v[MAXW];
#pragma unroll
            for (int t = 0; t < MAXW; ++t)
                if (t == nwin) v[t] = b;
            if (nwin == MAXW) v[MAXW] = b;
        }
        block_sums(v, nwin + 1);
        double beta2 = v[MAXW], L_new = 0.0, L_prev = 0.0;
#pragma unroll
        for (int t = 0; t < MAXW; ++t) {
            if (t == nwin) beta2 = v[t];
            if (t == nwin - 1) L_new = v[t];             // w_J.x (without Check: w_{J-tau}.x)
            if (t == nwin - 2) L_prev = v[t];            // w_{J-1}.x
        }
        const double yhat = (a.check && a.tau == 0) ? L_new : v[0];
        const double g = a.loss == kLossHinge ? loss_slope<kLossHinge>(y, yhat) : loss_slope<kLossLogistic>(y, yhat);

        bool keep = true;
        if (a.check) {
            const double base = eta_lambda + eta * beta2;
            const double rate = reach == 1 ? base : pow(base, 1.0 / (double)reach);
            auto across2 = [&](int64_t t, double L) {
                const double n2 = nrm[t % slots];
                return beta2 > 0.0 ? n2 - L * L / beta2 : n2;
            };
#pragma unroll
            for (int t = 2; t < MAXW; ++t)
                if (t < nwin && keep)
                    keep = check_triple(v[t - 2], v[t - 1], v[t], across2(first + t - 2, v[t - 2]),
                                        across2(first + t - 1, v[t - 1]), rate);
            if (keep && J >= 1) {
                const double L_cand = L_new - eta_lambda * yhat - eta * g * beta2;
                keep = check_triple(L_prev, L_new, L_cand, across2(J - 1, L_prev), across2(J, L_new), rate);
            }
        }
        if (keep) {
            const double *wj = ring + (int64_t)(J % slots) * d;
            const double *wd = ring + (int64_t)(at % slots) * d;
            double *dst = ring + (int64_t)((J + 1) % slots) * d;
            const double eg = eta * g;
            double u[MAXW + 1];
            u[0] = 0.0;
            for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC) {
                DelayRow<TX, VEC> c;
                c.load(xr + col);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const double w = wj[col + j] - eta_lambda * wd[col + j] - eg * c.x[j];
                    dst[col + j] = w;
                    u[0] += w * w;
                }
            }
            block_sums(u, 1);
            ++J;
            if (tid == 0) nrm[J % slots] = u[0];
        }
    }

    const double *last = ring + (int64_t)(J % slots) * d;
    float *out = a.W + (int64_t)chain * d;
    for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC)
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[col + j] = (float)last[col + j];
    if (tid == 0) a.accepted[chain] = J;
}

// The ring in registers.  R1 = max(tau, 1) + 1 iterates are kept: r[i] is w_{J-i}; before J reaches i
// the slot holds w_0, which is what an index below zero means.  n2[i] is |w_{J-i}|^2.
template <typename TX, int EPT, int VEC, int R1, int PF>
__global__ __launch_bounds__(kDelayThreads) void delay_server_reg_kernel(DelayArgs a)
{
    constexpr int NT = kDelayThreads, NW = kDelayWaves;
    using Frag = RowFrag<TX, NT, EPT, VEC>;
    __shared__ double red[2][NW][R1 + 1];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int chain = blockIdx.x;
    const int64_t n = a.n_samples[chain];
    const uint32_t d = (uint32_t)a.d;
    const char *X = static_cast<const char *>(a.dense);
    const int64_t row_stride = a.ld * (int64_t)sizeof(TX);
    const uint32_t row_bytes = d * (uint32_t)sizeof(TX);
    const double eta = a.eta, eta_lambda = a.eta * a.lambda;
    const bool no_delay = R1 == 2 && a.tau == 0;    // with three or more iterates kept the delay is R1 - 1
    int parity = 0;

    // element e of this thread is column col0[e / VEC] + e % VEC; columns from d on do not exist
    uint32_t off[Frag::kChunks];
#pragma unroll
    for (int c = 0; c < Frag::kChunks; ++c) off[c] = (uint32_t)((c * NT + tid) * VEC) * (uint32_t)sizeof(TX);
    auto column = [&](int e) { return (uint32_t)(((e / VEC) * NT + tid) * VEC + e % VEC); };

    auto block_sums = [&](auto &v, auto count_tag) {
        constexpr int COUNT = decltype(count_tag)::value;
        wave_sums_lane63(v, COUNT);
#pragma unroll
        for (int t = 0; t < COUNT; ++t)
            if (lane == kWave - 1) red[parity][wave][t] = v[t];
        __syncthreads();
#pragma unroll
        for (int t = 0; t < COUNT; ++t) {
            double sum = red[parity][0][t];
#pragma unroll
            for (int w = 1; w < NW; ++w) sum += red[parity][w][t];
            v[t] = sum;
        }
        parity ^= 1;
    };

    double r[R1][EPT], n2[R1];
    {
        double v[1] = {0.0};
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const uint32_t col = column(e);
            const double w = (a.w_start && col < d) ? (double)a.w_start[col] : 0.0;
#pragma unroll
            for (int i = 0; i < R1; ++i) r[i][e] = w;
            v[0] += w * w;
        }
        block_sums(v, std::integral_constant<int, 1>{});
#pragma unroll
        for (int i = 0; i < R1; ++i) n2[i] = v[0];
    }

    RowWindow win;
    win.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m);
    Frag x[PF];
    float ys[PF];
    auto request = [&](int u, int64_t s) {
        const uint32_t row = win.get(s);
        const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + (int64_t)row * row_stride, row_bytes);
#pragma unroll
        for (int c = 0; c < Frag::kChunks; ++c) x[u].load_chunk(c, rx, off[c]);
        ys[u] = a.y[row];
    };
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < n) request(u, u);

    int64_t J = 0;
    for (int64_t s0 = 0; s0 < n; s0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int64_t s = s0 + u;
            if (s >= n) break;
            double xe[EPT];
#pragma unroll
            for (int e = 0; e < EPT; ++e) xe[e] = (double)x[u].at(e);
            const double y = (double)ys[u];
            if (s + PF < n) request(u, s + PF);

            double v[R1 + 1];                        // v[i] = w_{J-i}.x, v[R1] = x.x
#pragma unroll
            for (int i = 0; i <= R1; ++i) v[i] = 0.0;
            if (a.check) {
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
                    v[R1] += xe[e] * xe[e];
#pragma unroll
                    for (int i = 0; i < R1; ++i) v[i] += r[i][e] * xe[e];
                }
                block_sums(v, std::integral_constant<int, R1 + 1>{});
            } else {                                 // only the projection the gradient needs
#pragma unroll
                for (int e = 0; e < EPT; ++e) v[0] += (no_delay ? r[0][e] : r[R1 - 1][e]) * xe[e];
                block_sums(v, std::integral_constant<int, 1>{});
                v[R1 - 1] = v[0];
            }
            const double beta2 = v[R1];
            const double yhat = no_delay ? v[0] : v[R1 - 1];           // the gradient is taken at w_{J-tau}

            // The cheapest tests come first and a failed one ends the sample: the parts across x (no root,
            // no slope), then the intervals of the first call (the root), then the candidate's (the slope).
            bool keep = true;
            double g = 0.0;
            if (a.check) {
                if (beta2 > 0.0) {
#pragma unroll
                    for (int i = 0; i + 1 < R1; ++i)      // pairs (w_{J-i-1}, w_{J-i}) that some triple holds
                        if (J >= i + 1) keep = keep && across_does_not_grow(v[i + 1], v[i], n2[i + 1], n2[i], beta2);
                } else {
#pragma unroll
                    for (int i = 0; i + 1 < R1; ++i)
                        if (J >= i + 1) keep = keep && !(n2[i] > n2[i + 1]);
                }
                if (keep) {
                    const double rate = delay_root<R1 - 1>(eta_lambda + eta * beta2);
                    keep = rate < 1.0 || J == 0;          // with no triple to test nothing is rejected
#pragma unroll
                    for (int i = 0; i + 2 < R1; ++i)
                        if (J >= i + 2) keep = keep && inside_interval(v[i + 2], v[i + 1], v[i], rate);
                    if (keep && J >= 1) {
                        g = a.loss == kLossHinge ? loss_slope<kLossHinge>(y, yhat) : loss_slope<kLossLogistic>(y, yhat);
                        const double L_cand = v[0] - eta_lambda * yhat - eta * g * beta2;
                        keep = inside_interval(v[1], v[0], L_cand, rate);
                    } else if (keep) {
                        g = a.loss == kLossHinge ? loss_slope<kLossHinge>(y, yhat) : loss_slope<kLossLogistic>(y, yhat);
                    }
                }
            } else {
                g = a.loss == kLossHinge ? loss_slope<kLossHinge>(y, yhat) : loss_slope<kLossLogistic>(y, yhat);
            }
            if (keep) {
                const double eg = eta * g;
                double u2[1] = {0.0};
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
                    const double old = no_delay ? r[0][e] : r[R1 - 1][e];
                    const double w = r[0][e] - eta_lambda * old - eg * xe[e];
#pragma unroll
                    for (int i = R1 - 1; i >= 1; --i) r[i][e] = r[i - 1][e];
                    r[0][e] = w;
                    u2[0] += w * w;
                }
                block_sums(u2, std::integral_constant<int, 1>{});
#pragma unroll
                for (int i = R1 - 1; i >= 1; --i) n2[i] = n2[i - 1];
                n2[0] = u2[0];
                ++J;
            }
        }
    }

    float *out = a.W + (int64_t)chain * a.d;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const uint32_t col = column(e);
        if (col < d) out[col] = (float)r[0][e];
    }
    if (tid == 0) a.accepted[chain] = J;
}

// Rows on their way from HBM into LDS.  A ring of S row slots (sample s in slot s mod S), filled by loads
// that land in LDS directly and need no registers while in flight; behind the slots, S pads that
// receive, the same way, a small record per sample: SIDE dwords from an array indexed by the sample's
// row (SIDE = 1: its label; SIDE = 8: its entry of the row table, see DelayRowEntry).  Every wave requests, and later reads back, only its own
// part of a row (the columns its lanes own), so the slots need no barrier.  The compiler does not see
// these loads; a wave's loads complete in issue order, so waiting until at most (S - B) samples' worth of
// them are outstanding means the B oldest samples have landed.  Samples past the end of the stream are
// requested all the same (the last valid row again), which keeps that count a constant.  The record goes
// out before its row, so it has landed when the row has; fetched by an ordinary load inside the loop it
// would queue behind the rows on their way and wait for all of them.
template <typename TX, int EPT, int VEC, int S, int SIDE>
struct LdsRows {
    static_assert(SIDE >= 1 && SIDE <= kWave && (SIDE & (SIDE - 1)) == 0, "a power of two of dwords");
    static constexpr int NT = kDelayThreads, NW = kDelayWaves;
    using Frag = RowFrag<TX, NT, EPT, VEC>;
    static_assert(VEC * sizeof(TX) == 16, "16-byte loads only");
    static constexpr int CHUNKS = EPT / VEC;
    static_assert(Frag::kWords == 4 * CHUNKS, "four words per chunk");
    static constexpr uint32_t kWaveBytes = CHUNKS * kWave * 16;          // what one wave holds of one row
    static constexpr uint32_t kSlotBytes = NW * kWaveBytes;
    static constexpr uint32_t kLabelBytes = kWave * 4;                   // a wave's copy of one record (64 / SIDE times)
    static constexpr int kLoadsPerSample = CHUNKS + 1;                   // the row's chunks and its record
    static constexpr size_t kBytes = (size_t)S * (kSlotBytes + NW * kLabelBytes);
    typedef __attribute__((address_space(3))) uint32_t *lds_words;

    lds_words stage;            // S slots, then S x NW record pads
    uint32_t slot0, labels0;    // LDS byte addresses of this wave's part of slot 0 and of its pad 0
    uint32_t voff, lane, wave, side_lane;
    u32x4 ry;                   // the records as a buffer
    const char *X;
    int64_t row_stride, n;
    uint32_t row_bytes;
    RowWindow ahead;

    // clears the slots (lanes whose columns lie beyond the row are out of the buffer's range: whether such
    // a load writes zeros or nothing, the slots read as zero there afterwards); ends with a barrier
    __device__ void init(lds_words lds, const DelayArgs &a, int chain, int64_t samples, const void *records)
    {
        const int tid = threadIdx.x;
        stage = lds;
        lane = (uint32_t)(tid & (kWave - 1));
        wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid / kWave);
        slot0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(size_t)lds + wave * kWaveBytes));
        labels0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(size_t)lds + (uint32_t)S * kSlotBytes + wave * kLabelBytes));
        voff = (uint32_t)(tid * 16);                 // this lane's bytes of chunk 0; chunk c adds c*NT*16
        const uint64_t ybase = (uint64_t)(uintptr_t)records;
        ry[0] = (uint32_t)ybase;
        ry[1] = (uint32_t)(ybase >> 32) & 0xffffu;
        ry[2] = (uint32_t)a.m * (uint32_t)(SIDE * 4);
        ry[3] = 0x00020000u;
        side_lane = (lane & (uint32_t)(SIDE - 1)) * 4u;
        X = static_cast<const char *>(a.dense);
        row_stride = a.ld * (int64_t)sizeof(TX);
        row_bytes = (uint32_t)a.d * (uint32_t)sizeof(TX);
        n = samples;
        ahead.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m);
        for (uint32_t i = (uint32_t)tid; i < (uint32_t)S * (kSlotBytes / 4); i += NT) stage[i] = 0u;
        __syncthreads();
    }
    // the record and the row of sample s (of the last sample, beyond the end) into slot s mod S
    __device__ void request(int64_t s)
    {
        const uint32_t row = ahead.get(s < n ? s : n - 1);
        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                     :
                     : "s"(labels0 + (uint32_t)(s % S) * (NW * kLabelBytes)), "v"(row * (uint32_t)(SIDE * 4) + side_lane), "s"(ry)
                     : "memory", "m0");
        const uint64_t base = (uint64_t)(uintptr_t)(X + (int64_t)row * row_stride);
        u32x4 rx;
        rx[0] = (uint32_t)base;
        rx[1] = (uint32_t)(base >> 32) & 0xffffu;
        rx[2] = row_bytes;
        rx[3] = 0x00020000u;
        const uint32_t slot = slot0 + (uint32_t)(s % S) * kSlotBytes;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c)
            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :
                         : "s"(slot + c * (kWave * 16)), "v"(voff), "s"(rx), "s"(c * (NT * 16))
                         : "memory", "m0");
    }
    // waits until the B oldest of the S samples requested last have landed
    // (gfx9 encoding: vmcnt split over bits 3:0 and 15:14; expcnt and lgkmcnt left open)
    template <int B>
    __device__ static void wait_for_oldest()
    {
        constexpr int kLater = (S - B) * kLoadsPerSample;
        static_assert(kLater >= 0 && kLater < 64, "the counter holds 63");
        __builtin_amdgcn_s_waitcnt(((kLater & 0xF) | ((kLater >> 4) << 14)) | 0x0F70);
        __builtin_amdgcn_sched_barrier(0);
    }
    // this thread's elements of the row of sample s
    __device__ void take(int64_t s, Frag &x) const
    {
        const lds_words src = stage + (size_t)(s % S) * (kSlotBytes / 4) + (size_t)wave * (kWaveBytes / 4) + lane * 4;
        typedef __attribute__((address_space(3))) const u32x4 *lds_quads;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const u32x4 q = *(lds_quads)(src + c * (kWave * 4));
            x.w[4 * c + 0] = q[0];
            x.w[4 * c + 1] = q[1];
            x.w[4 * c + 2] = q[2];
            x.w[4 * c + 3] = q[3];
        }
    }
    // dword j of sample s's record (the same address in every lane)
    __device__ uint32_t side(int64_t s, int j) const
    {
        return stage[(size_t)S * (kSlotBytes / 4) + (size_t)(s % S) * (NW * kLabelBytes / 4) + (size_t)wave * (kLabelBytes / 4) + j];
    }
    __device__ double side_f64(int64_t s, int j) const
    {
        return __longlong_as_double((long long)(((uint64_t)side(s, j + 1) << 32) | side(s, j)));
    }
    // every LDS read of a slot must have returned before the slot is requested again
    __device__ static void reads_done() { __builtin_amdgcn_s_waitcnt(0xC07F); }
    // nothing may still be landing when the wave ends
    __device__ static void drain() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }
};

// What the Check function needs of a row and not of the model: computed once per row of the data set
// instead of once per visit.  32 bytes, read as eight dwords.
struct DelayRowEntry {
    double beta2;       // x.x
    double rate;        // (eta*lambda + eta*beta2)^(1/reach)
    float y;            // the label
    float pad[3];
};
static_assert(sizeof(DelayRowEntry) == 32, "eight dwords");

template <typename TX, int VEC>
__global__ __launch_bounds__(kDelayThreads) void delay_row_table_kernel(DelayArgs a, DelayRowEntry *table, int reach)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * kDelayWaves + threadIdx.x / kWave;       // one wave per row
    if (row >= a.m) return;
    const TX *xr = static_cast<const TX *>(a.dense) + row * a.ld;
    double acc = 0.0;
    for (int64_t col = (int64_t)lane * VEC; col < a.d; col += (int64_t)kWave * VEC) {
        DelayRow<TX, VEC> c;
        c.load(xr + col);
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc += c.x[j] * c.x[j];
    }
    const double beta2 = wave_sum(acc);
    if (lane == 0) {
        const double base = a.eta * a.lambda + a.eta * beta2;
        DelayRowEntry e;
        e.beta2 = beta2;
        e.rate = reach == 1 ? base : reach == 2 ? delay_root<2>(base) : reach == 3 ? delay_root<3>(base) : delay_root<4>(base);
        e.y = a.y[row];
        e.pad[0] = e.pad[1] = e.pad[2] = 0.0f;
        table[row] = e;
    }
}

// All tests of the Check function for one sample, from its scalars alone and without branches on the
// data: L[i] = w_{J-i}.x; n2[i] = |w_{J-i}|^2; beta2 = x.x and rate from the row table; yhat and g
// belong to w_{J-tau}.
template <int R1>
__device__ inline bool window_passes(const double *L, const double (&n2)[R1], double beta2, double rate, int64_t J,
                                     double eta, double eta_lambda, double yhat, double g)
{
    // (bitwise and/or on purpose: nothing here is worth a branch, and without branches the tests of
    // several samples can be interleaved)
    bool ok = true;
#pragma unroll
    for (int i = 0; i + 1 < R1; ++i) {          // pairs (w_{J-i-1}, w_{J-i}) that some triple holds
        const bool along = across_does_not_grow(L[i + 1], L[i], n2[i + 1], n2[i], beta2);
        const bool plain = !(n2[i] > n2[i + 1]);
        ok = ok & ((J < i + 1) | (beta2 > 0.0 ? along : plain));
    }
    ok = ok & ((rate < 1.0) | (J == 0));        // with no triple to test nothing is rejected
#pragma unroll
    for (int i = 0; i + 2 < R1; ++i) ok = ok & ((J < i + 2) | inside_interval(L[i + 2], L[i + 1], L[i], rate));
    const double L_cand = L[0] - eta_lambda * yhat - eta * g * beta2;
    ok = ok & ((J < 1) | inside_interval(L[1], L[0], L_cand, rate));
    return ok;
}

// Under the Check function nearly every sample is thrown away, and a sample that is thrown away leaves
// the ring as it was.  This kernel therefore looks at B samples at once: it projects the ring on all B
// rows, exchanges the B x R1 sums in one round and takes the B decisions side by side in
// straight-line code (so that their dependent fp64 chains overlap), each as if the samples before it had
// been rejected.  The decisions up to and including the first acceptance are then the sequential ones;
// that sample's candidate is written and the samples behind it are looked at again, against the new ring,
// as the next batch.
//
// Rows come through LdsRows: the rows of samples pos .. pos+S-1 are always in LDS or on their way, so a
// batch's rows were asked for at least S-B samples earlier, and the row of an accepted sample is still in
// its slot when the candidate is formed.
template <typename TX, int EPT, int VEC, int R1, int B, int S>
__global__ __launch_bounds__(kDelayThreads) void delay_server_batch_kernel(DelayArgs a)
{
    constexpr int NT = kDelayThreads, NW = kDelayWaves, NV = B * R1;
    using Rows = LdsRows<TX, EPT, VEC, S, 8>;       // with each row its entry of the row table
    using Frag = typename Rows::Frag;
    extern __shared__ __attribute__((aligned(16))) uint32_t stage[];     // Rows::kBytes
    __shared__ double red[2][NW][NV];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int chain = blockIdx.x;
    const int64_t n = a.n_samples[chain];
    const uint32_t d = (uint32_t)a.d;
    const double eta = a.eta, eta_lambda = a.eta * a.lambda;
    const bool no_delay = R1 == 2 && a.tau == 0;
    int parity = 0;

    auto column = [&](int e) { return (uint32_t)(((e / VEC) * NT + tid) * VEC + e % VEC); };

    auto block_sums = [&](auto &v, auto count_tag) {
        constexpr int COUNT = decltype(count_tag)::value;
        wave_sums_lane63(v, COUNT);
#pragma unroll
        for (int t = 0; t < COUNT; ++t)
            if (lane == kWave - 1) red[parity][wave][t] = v[t];
        __syncthreads();
#pragma unroll
        for (int t = 0; t < COUNT; ++t) {
            double sum = red[parity][0][t];
#pragma unroll
            for (int w = 1; w < NW; ++w) sum += red[parity][w][t];
            v[t] = sum;
        }
        parity ^= 1;
    };

    double r[R1][EPT], n2[R1];
    {
        double v[1] = {0.0};
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const uint32_t col = column(e);
            const double w = (a.w_start && col < d) ? (double)a.w_start[col] : 0.0;
#pragma unroll
            for (int i = 0; i < R1; ++i) r[i][e] = w;
            v[0] += w * w;
        }
        block_sums(v, std::integral_constant<int, 1>{});
#pragma unroll
        for (int i = 0; i < R1; ++i) n2[i] = v[0];
    }
    if (n <= 0) {
        float *out0 = a.W + (int64_t)chain * a.d;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const uint32_t col = column(e);
            if (col < d) out0[col] = (float)r[0][e];
        }
        if (tid == 0) a.accepted[chain] = 0;
        return;
    }

    Rows rows;
    rows.init((typename Rows::lds_words)&stage[0], a, chain, n, a.row_table);
    for (int64_t s = 0; s < S; ++s) rows.request(s);
    int64_t J = 0, pos = 0;
    while (pos < n) {
        Rows::template wait_for_oldest<B>();        // samples pos .. pos+B-1 have landed
        double y[B], beta2[B], rate[B];             // DelayRowEntry of each sample's row
#pragma unroll
        for (int b = 0; b < B; ++b) {
            beta2[b] = rows.side_f64(pos + b, 0);
            rate[b] = rows.side_f64(pos + b, 2);
            y[b] = (double)__uint_as_float(rows.side(pos + b, 4));
        }
        double v[NV];                               // v[b*R1 + i] = w_{J-i}.x_b
#pragma unroll
        for (int t = 0; t < NV; ++t) v[t] = 0.0;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            Frag x;
            rows.take(pos + b, x);
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const double xe = (double)x.at(e);
#pragma unroll
                for (int i = 0; i < R1; ++i) v[b * R1 + i] += r[i][e] * xe;
            }
        }
        block_sums(v, std::integral_constant<int, NV>{});

        bool keep[B];
        double slope[B], yhat[B];
#pragma unroll
        for (int b = 0; b < B; ++b) yhat[b] = no_delay ? v[b * R1] : v[b * R1 + R1 - 1];
        if (a.loss == kLossHinge) {                 // (one branch for the batch, so that the B slopes share a block)
#pragma unroll
            for (int b = 0; b < B; ++b) slope[b] = loss_slope<kLossHinge>(y[b], yhat[b]);
        } else {
#pragma unroll
            for (int b = 0; b < B; ++b) slope[b] = loss_slope<kLossLogistic>(y[b], yhat[b]);
        }
#pragma unroll
        for (int b = 0; b < B; ++b)
            keep[b] = (pos + b < n) & window_passes<R1>(v + b * R1, n2, beta2[b], rate[b], J, eta, eta_lambda, yhat[b], slope[b]);
        int taken = B;                              // the first sample of the batch that is accepted
#pragma unroll
        for (int b = B - 1; b >= 0; --b) taken = keep[b] ? b : taken;
        taken = __builtin_amdgcn_readfirstlane(taken);     // (every lane holds the same sums, hence the same verdict)
        int advance = B;
        if (__builtin_expect(taken < B, 0)) {
            // w_{J+1} = w_J - eta*lambda*w_{J-tau} - eta*u*x; the row is still in its slot
            double eg = 0.0;
#pragma unroll
            for (int b = 0; b < B; ++b)
                if (b == taken) eg = eta * slope[b];
            Frag x;
            rows.take(pos + taken, x);
            double u2[1] = {0.0};
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const double old = no_delay ? r[0][e] : r[R1 - 1][e];
                const double w = r[0][e] - eta_lambda * old - eg * (double)x.at(e);
#pragma unroll
                for (int i = R1 - 1; i >= 1; --i) r[i][e] = r[i - 1][e];
                r[0][e] = w;
                u2[0] += w * w;
            }
            block_sums(u2, std::integral_constant<int, 1>{});
#pragma unroll
            for (int i = R1 - 1; i >= 1; --i) n2[i] = n2[i - 1];
            n2[0] = u2[0];
            ++J;
            advance = taken + 1;
        }
        // the slots of the samples left behind take the rows that follow the ones on their way
        Rows::reads_done();
#pragma unroll
        for (int i = 0; i < B; ++i)
            if (i < advance) rows.request(pos + S + i);
        pos += advance;
    }
    Rows::drain();

    float *out = a.W + (int64_t)chain * a.d;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const uint32_t col = column(e);
        if (col < d) out[col] = (float)r[0][e];
    }
    if (tid == 0) a.accepted[chain] = J;
}

// f(integral_constant<int, 0>) .. f(integral_constant<int, N-1>): a loop whose index is a constant
// expression in its body (register arrays indexed through it are never indexed at run time).
template <int N, typename F, int I = 0>
__device__ inline void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, F, I + 1>(static_cast<F &&>(f));
    }
}

// Without the Check function every sample is an update, and the delay itself gives the parallelism: the
// gradients of the next tau + 1 samples are taken at w_{J-tau} .. w_J, which all exist already.  One
// batch is R1 = tau + 1 samples: R1 projections (sample i on the iterate tau - i back) cross the workgroup
// in one exchange, then R1 updates follow, element by element, with no further exchange.  The ring holds
// exactly R1 iterates, so an update overwrites the oldest one - the very iterate its gradient was taken
// at - and after a whole batch every iterate is back in the registers it started in: slot (i + 1) mod R1
// is both where sample i's gradient is taken and where w_{J+i+1} goes; no register is ever moved.  (Slots
// start as w_0, which is what an iterate before the start means.)  Rows come through LdsRows.
template <typename TX, int EPT, int VEC, int R1, int S>
__global__ __launch_bounds__(kDelayThreads) void delay_server_plain_kernel(DelayArgs a)
{
    constexpr int NT = kDelayThreads, NW = kDelayWaves, B = R1;
    static_assert(R1 >= 2, "a delay of at least one");
    using Rows = LdsRows<TX, EPT, VEC, S, 1>;       // with each row its label
    using Frag = typename Rows::Frag;
    extern __shared__ __attribute__((aligned(16))) uint32_t stage[];     // Rows::kBytes
    __shared__ double red[2][NW][B];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int chain = blockIdx.x;
    const int64_t n = a.n_samples[chain];
    const uint32_t d = (uint32_t)a.d;
    const double eta = a.eta, eta_lambda = a.eta * a.lambda;
    int parity = 0;
    auto column = [&](int e) { return (uint32_t)(((e / VEC) * NT + tid) * VEC + e % VEC); };

    double r[R1][EPT];                              // r[p]: the iterate w_t with t mod R1 = p (w_0 before that)
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const uint32_t col = column(e);
        const double w = (a.w_start && col < d) ? (double)a.w_start[col] : 0.0;
#pragma unroll
        for (int p = 0; p < R1; ++p) r[p][e] = w;
    }
    int newest = 0;                                 // slot of w_J when the loop ends
    if (n > 0) {
        Rows rows;
        rows.init((typename Rows::lds_words)&stage[0], a, chain, n, a.y);
        for (int64_t s = 0; s < S; ++s) rows.request(s);
        for (int64_t pos = 0; pos < n; pos += B) {  // J = pos is a multiple of R1 here: w_J sits in slot 0
            Rows::template wait_for_oldest<B>();
            double y[B], v[B];
            Frag x[B];
            static_for<B>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                y[i] = (double)__uint_as_float(rows.side(pos + i, 0));
                rows.take(pos + i, x[i]);
                v[i] = 0.0;
#pragma unroll
                for (int e = 0; e < EPT; ++e) v[i] += r[(i + 1) % R1][e] * (double)x[i].at(e);
            });
            wave_sums_lane63(v, B);
#pragma unroll
            for (int i = 0; i < B; ++i)
                if (lane == kWave - 1) red[parity][wave][i] = v[i];
            __syncthreads();
            double eg[B];
            if (a.loss == kLossHinge) {
#pragma unroll
                for (int i = 0; i < B; ++i) {
                    double sum = red[parity][0][i];
#pragma unroll
                    for (int w = 1; w < NW; ++w) sum += red[parity][w][i];
                    eg[i] = eta * loss_slope<kLossHinge>(y[i], sum);
                }
            } else {
#pragma unroll
                for (int i = 0; i < B; ++i) {
                    double sum = red[parity][0][i];
#pragma unroll
                    for (int w = 1; w < NW; ++w) sum += red[parity][w][i];
                    eg[i] = eta * loss_slope<kLossLogistic>(y[i], sum);
                }
            }
            parity ^= 1;
            // w_{J+i+1} = w_{J+i} - eta*lambda*w_{J+i-tau} - eta*u*x_i, for the samples that exist
            static_for<B>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                if (pos + i < n) {
#pragma unroll
                    for (int e = 0; e < EPT; ++e)
                        r[(i + 1) % R1][e] = r[i % R1][e] - eta_lambda * r[(i + 1) % R1][e] - eg[i] * (double)x[i].at(e);
                    newest = (i + 1) % R1;
                }
            });
            Rows::reads_done();
#pragma unroll
            for (int i = 0; i < B; ++i) rows.request(pos + S + i);
        }
        Rows::drain();
    }

    float *out = a.W + (int64_t)chain * a.d;
    static_for<R1>([&](auto pc) {                   // (a branch per slot: the ring is never indexed at run time)
        constexpr int p = decltype(pc)::value;
        if (newest == p) {
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const uint32_t col = column(e);
                if (col < d) out[col] = (float)r[p][e];
            }
        }
    });
    if (tid == 0) a.accepted[chain] = n > 0 ? n : 0;
}

constexpr int kDelayRegMaxTau = 4;
constexpr int kDelayAhead = 4;          // samples whose rows are in flight
constexpr int kDelayBatch = 4;          // samples looked at side by side under Check
constexpr int kDelaySlots = 8;          // rows in LDS or on their way there

// The batch kernel claims S row slots of LDS, which is more than a kernel may have without asking.
template <typename TX, int EPT, int VEC, int R1>
bool launch_batch(const DelayArgs &a, hipStream_t s)
{
    auto kernel = delay_server_batch_kernel<TX, EPT, VEC, R1, kDelayBatch, kDelaySlots>;
    constexpr size_t bytes = LdsRows<TX, EPT, VEC, kDelaySlots, 8>::kBytes;
    static std::atomic<int> allowed{0};             // 0 not asked yet, 1 granted, -1 refused (asking twice is harmless)
    int may = allowed.load(std::memory_order_relaxed);
    if (may == 0) {
        may = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)bytes) == hipSuccess ? 1 : -1;
        if (may < 0) (void)hipGetLastError();
        allowed.store(may, std::memory_order_relaxed);
    }
    if (may < 0) return false;                      // the per-sample kernel serves instead
    // what depends on a row alone, once per row
    hipLaunchKernelGGL((delay_row_table_kernel<TX, VEC>), dim3((unsigned)((a.m + kDelayWaves - 1) / kDelayWaves)), dim3(kDelayThreads),
                       0, s, a, static_cast<DelayRowEntry *>(a.row_table), R1 - 1);
    hipLaunchKernelGGL(kernel, dim3(a.k), dim3(kDelayThreads), bytes, s, a);
    return true;
}

template <typename TX, int EPT, int VEC, int R1>
bool launch_plain(const DelayArgs &a, hipStream_t s)
{
    auto kernel = delay_server_plain_kernel<TX, EPT, VEC, R1, kDelaySlots>;
    constexpr size_t bytes = LdsRows<TX, EPT, VEC, kDelaySlots, 1>::kBytes;
    static std::atomic<int> allowed{0};
    int may = allowed.load(std::memory_order_relaxed);
    if (may == 0) {
        may = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)bytes) == hipSuccess ? 1 : -1;
        if (may < 0) (void)hipGetLastError();
        allowed.store(may, std::memory_order_relaxed);
    }
    if (may < 0) return false;
    hipLaunchKernelGGL(kernel, dim3(a.k), dim3(kDelayThreads), bytes, s, a);
    return true;
}

// Launches the register kernel if one is built for this shape; *done tells.
template <typename TX, int VEC>
hipError_t launch_reg(const DelayArgs &a, hipStream_t s, bool *done)
{
    const int r1 = (a.tau > 1 ? a.tau : 1) + 1;
    *done = true;
#define WPSGD_DELAY_REG(EPT, R1)                                                                                 \
    if (a.d <= (int64_t)kDelayThreads * EPT && r1 == R1) {                                                       \
        if (a.check && a.row_table && a.m < (1 << 27) && launch_batch<TX, EPT, VEC, R1>(a, s))                   \
            return hipGetLastError();                                                                            \
        else if (!a.check && a.tau >= 1 && a.m < (1 << 30) && launch_plain<TX, EPT, VEC, R1>(a, s))              \
            return hipGetLastError();                                                                            \
        else                                                                                                     \
            hipLaunchKernelGGL((delay_server_reg_kernel<TX, EPT, VEC, R1, kDelayAhead>), dim3(a.k), dim3(kDelayThreads), 0, s, a); \
        return hipGetLastError();                                                                                \
    }
    WPSGD_DELAY_REG(8, 2) WPSGD_DELAY_REG(8, 3) WPSGD_DELAY_REG(8, 4) WPSGD_DELAY_REG(8, 5)
    WPSGD_DELAY_REG(16, 2) WPSGD_DELAY_REG(16, 3) WPSGD_DELAY_REG(16, 4) WPSGD_DELAY_REG(16, 5)
#undef WPSGD_DELAY_REG
    *done = false;
    return hipSuccess;
}

template <typename TX, int VEC>
hipError_t launch_reach(const DelayArgs &a, hipStream_t s)
{
    const int need = (a.tau > 1 ? a.tau : 1) + 1;
#define WPSGD_DELAY_TRY(MAXW)                                                                                   \
    if (need <= MAXW) {                                                                                         \
        hipLaunchKernelGGL((delay_server_kernel<TX, VEC, MAXW>), dim3(a.k), dim3(kDelayThreads), 0, s, a);      \
        return hipGetLastError();                                                                               \
    }
    WPSGD_DELAY_TRY(3)
    WPSGD_DELAY_TRY(5)
    WPSGD_DELAY_TRY(kDelayMaxTau + 1)
#undef WPSGD_DELAY_TRY
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_delay_servers(const DelayArgs &a, int dtype, int vec, hipStream_t s)
{
    if (vec > 1 && a.tau <= kDelayRegMaxTau && a.d * (dtype == WPSGD_BF16 ? 2 : 4) < (int64_t)1 << 31) {
        bool done = false;
        const hipError_t e = dtype == WPSGD_BF16 ? launch_reg<uint16_t, 8>(a, s, &done) : launch_reg<float, 4>(a, s, &done);
        if (done) return e;
    }
    if (dtype == WPSGD_BF16) return vec > 1 ? launch_reach<uint16_t, 8>(a, s) : launch_reach<uint16_t, 1>(a, s);
    return vec > 1 ? launch_reach<float, 4>(a, s) : launch_reach<float, 1>(a, s);
}

}  // namespace wpsgd
