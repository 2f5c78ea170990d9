// Dense-row SGD chains with the model vector held in registers.
//
// One workgroup runs one chain (Algorithm 1, the inner loop of node i): NT threads own EPT model
// elements each, so the vector never leaves the register file between the first and the last
// step.  The step  w <- (1-eta*lambda) w - eta*g*x  (Eq. 5 with Eq. 4) is carried as w = s*v:
// the shrink only touches the fp64 scalar s, the gradient part touches v.
//
// Because the rows a chain visits depend on (seed, chain, step) only, never on w, rows are
// requested P rounds before they are consumed and wait in registers.  A round folds B steps into
// one workgroup-wide reduction: with the rows x_0..x_{B-1} of the round and the vector v at its
// start, the threads reduce p_b = v.x_b and G_ab = x_a.x_b (a<b) together; the B dependent
// steps are then a scalar recursion
//     v_b.x_b = p_b + sum_{a<b} c_a G_ab,   yhat_b = s_b * (v_b.x_b),   c_b = -eta*g_b / s_{b+1}
// and the round ends with the rank-B update v += sum_b c_b x_b.  This is the same arithmetic as
// B single steps up to summation order; B = 1 is the plain step.
//
// This file is compiled once per (row storage, loss) pair; WPSGD_TX_BF16 and WPSGD_LOSS select it.
#include "device_utils.h"
#include "internal.h"

namespace wpsgd {

#if WPSGD_TX_BF16
using RowElem = uint16_t;
#else
using RowElem = float;
#endif
constexpr int kLoss = WPSGD_LOSS;

// The EPT elements of one row that a thread owns.  Element e of the fragment is column
//   ((e / VEC) * NT + tid) * VEC + e % VEC
// so that every load instruction of a wave covers one contiguous 64*VEC-element span.
// Loads are unconditional (a lane past the end of the row re-reads the row's first elements and
// discards them): a load that may or may not be issued would force the wait before each use to
// drain every outstanding load, and the prefetch with it.  FULL says NT*EPT == d, i.e. no lane
// is ever past the end and the discard is compiled out.
template <typename TX, int NT, int EPT, int VEC, bool FULL>
struct RowFrag {
    static constexpr bool kPacked = (sizeof(TX) == 2) && (VEC == 8);
    static constexpr int kWords = kPacked ? EPT / 2 : EPT;
    uint32_t w[kWords];     // fp32 bit patterns, or pairs of bfloat16 when packed

    __device__ inline void load(const TX *row, int64_t d, int tid)
    {
        static_assert(EPT % VEC == 0, "fragment must be whole loads");
#pragma unroll
        for (int c = 0; c < EPT / VEC; ++c) {
            const int64_t col = ((int64_t)c * NT + tid) * VEC;
            const bool in = FULL || col < d;        // d is a multiple of VEC whenever VEC > 1
            const TX *p = row + (in ? col : 0);
            if constexpr (VEC == 1) {
                uint32_t q;
                if constexpr (sizeof(TX) == 2) {
                    q = (uint32_t)p[0] << 16;
                } else {
                    q = __float_as_uint(p[0]);
                }
                w[c] = in ? q : 0u;
            } else {
                static_assert(kPacked || (sizeof(TX) == 4 && VEC == 4), "16-byte loads only");
                const uint4 q = *reinterpret_cast<const uint4 *>(p);
                w[4 * c + 0] = in ? q.x : 0u;
                w[4 * c + 1] = in ? q.y : 0u;
                w[4 * c + 2] = in ? q.z : 0u;
                w[4 * c + 3] = in ? q.w : 0u;
            }
        }
    }
    __device__ inline float at(int e) const
    {
        if constexpr (kPacked) {
            return (e & 1) ? bf16_hi(w[e >> 1]) : bf16_lo(w[e >> 1]);
        } else {
            return __uint_as_float(w[e]);
        }
    }
};

// TX and LOSS are template parameters (not just per-file constants) so that the four builds of
// this file produce four distinct sets of kernel symbols.
template <typename TX, int LOSS, int NT, int EPT, int VEC, int B, int P, bool FULL>
__global__ __launch_bounds__(NT) void chain_dense_reg_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;     // state, dot products and the step recursion
    constexpr int NW = NT / kWave;
    constexpr int NG = B * (B - 1) / 2;
    constexpr int NR = B + NG;
    constexpr int NACC = EPT >= 4 ? 4 : EPT;       // independent partial sums per dot product
    __shared__ TV red[2][NR][NW];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const TX *X = static_cast<const TX *>(a.dense);

    TV v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) v[e] = (TV)0;
    // w = s*v.  s and eta/s are fp64 and advance independently of the data.
    double s = 1.0, eta_over_s = a.eta;
    const double rho = a.rho, inv_rho = 1.0 / a.rho;

    RowFrag<TX, NT, EPT, VEC, FULL> x[P][B];
    float yv[P][B];
    RowWindow win;
    win.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m);

    // Request the rows of round `blk` into slot u.  Steps past the end of the chain re-request
    // the chain's last row (a cache hit) so that the loop body has no data-dependent branches.
    auto request = [&](int u, int64_t blk) {
#pragma unroll
        for (int b = 0; b < B; ++b) {
            int64_t step = blk * B + b;
            step = step < n ? step : n - 1;
            const uint32_t row = win.get(step);
            x[u][b].load(X + (int64_t)row * a.ld, a.d, tid);
            // The label travels with the row through the vector-memory queue.  As a scalar
            // load it would be re-issued right before its use (scalar registers are scarce
            // here) and put a cache miss on the dependent path of every step.
            uint32_t row_v = row;
            asm volatile("" : "+v"(row_v));
            yv[u][b] = a.y[row_v];
        }
    };

    int parity = 0;
    auto consume = [&](int u, int64_t blk) {
        // p_b = v.x_b and G_qb = x_q.x_b, each as NACC interleaved partial sums
        TV acc[NR][NACC];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int j = 0; j < NACC; ++j) acc[r][j] = (TV)0;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            TV xe[B];
#pragma unroll
            for (int b = 0; b < B; ++b) xe[b] = (TV)x[u][b].at(e);
#pragma unroll
            for (int b = 0; b < B; ++b) acc[b][e % NACC] += v[e] * xe[b];
            int g = B;
#pragma unroll
            for (int q = 0; q < B; ++q)
#pragma unroll
                for (int b = q + 1; b < B; ++b) acc[g++][e % NACC] += xe[q] * xe[b];
        }
        TV tot[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            TV t = acc[r][0];
#pragma unroll
            for (int j = 1; j < NACC; ++j) t += acc[r][j];
            tot[r] = wave_sum_lane63(t);
        }
        if constexpr (NW > 1) {
            if (lane == kWave - 1) {
#pragma unroll
                for (int r = 0; r < NR; ++r) red[parity][r][wave] = tot[r];
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                TV t = red[parity][r][0];
#pragma unroll
                for (int w = 1; w < NW; ++w) t += red[parity][r][w];
                tot[r] = t;
            }
            parity ^= 1;
        } else {
#pragma unroll
            for (int r = 0; r < NR; ++r) tot[r] = read_lane63(tot[r]);
        }
        // the B dependent steps, as scalars
        TV c[B];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            TV dot = tot[b];
            int g = B;
#pragma unroll
            for (int q = 0; q < B; ++q)
#pragma unroll
                for (int bb = q + 1; bb < B; ++bb) {
                    if (bb == b) dot += c[q] * tot[g];
                    ++g;
                }
            const bool live = blk * B + b < n;
            const double s_next = live ? s * rho : s;
            const double eos_next = live ? eta_over_s * inv_rho : 0.0;     // eta / s_next
            if constexpr (LOSS == kLossHinge) {
                c[b] = step_coef_hinge((double)yv[u][b], dot, s, eos_next);
            } else {
                c[b] = step_coef_logistic(yv[u][b], dot, (float)s, (float)eos_next);
            }
            if (live) {
                s = s_next;
                eta_over_s = eos_next;
            }
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
#pragma unroll
            for (int b = 0; b < B; ++b) v[e] += c[b] * (TV)x[u][b].at(e);
        }
        if (s < 0x1p-30) {          // fold the scale into v long before eta/s leaves fp32 range
#pragma unroll
            for (int e = 0; e < EPT; ++e) v[e] *= (TV)s;
            s = 1.0;
            eta_over_s = a.eta;
        }
    };

    if (n > 0) {
        const int64_t nblk = (n + B - 1) / B;
#pragma unroll
        for (int u = 0; u < P; ++u) request(u, u);
        int64_t blk0 = 0;
        for (; blk0 + P <= nblk; blk0 += P) {
#pragma unroll
            for (int u = 0; u < P; ++u) {
                consume(u, blk0 + u);
                request(u, blk0 + u + P);
            }
        }
#pragma unroll
        for (int u = 0; u < P; ++u) {
            if (blk0 + u < nblk) consume(u, blk0 + u);
        }
    }

    float *out = a.W + (int64_t)chain * a.d;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        if (FULL || col < a.d) out[col] = (float)(s * (double)v[e]);
    }
}

// ---------------------------------------------------------------------------------------------
// Instantiated variants: V(threads, elements per thread, load width, B, P).  Within one
// (threads, ept, vec) shape the first entry is the default; the others are reachable through a
// forced plan.  Register budget per thread: 512 at 256 threads, 256 at 512, 128 at 1024.
// ---------------------------------------------------------------------------------------------
#define WPSGD_VARIANTS_ANY(V)                                                                  \
    V(64, 1, 1, 1, 8) V(64, 2, 1, 1, 8) V(64, 4, 1, 1, 8)                                      \
    V(64, 1, 1, 4, 2) V(64, 4, 1, 2, 4)                                                        \
    V(256, 4, 1, 1, 4) V(256, 8, 1, 1, 4) V(256, 16, 1, 1, 4) V(256, 32, 1, 1, 2)              \
    V(256, 4, 1, 4, 2) V(256, 16, 1, 4, 2)                                                     \
    V(1024, 16, 1, 1, 2) V(1024, 32, 1, 1, 1)

#if WPSGD_TX_BF16
#define WPSGD_VARIANTS_VEC(V)                                                                  \
    V(64, 8, 8, 1, 8) V(64, 8, 8, 4, 2)                                                        \
    V(256, 8, 8, 1, 8) V(256, 16, 8, 1, 8) V(256, 32, 8, 4, 2) V(256, 32, 8, 1, 4)             \
    V(256, 8, 8, 4, 2) V(256, 16, 8, 4, 2)                                                     \
    V(1024, 16, 8, 1, 4) V(1024, 32, 8, 1, 2) V(1024, 16, 8, 2, 2)
#if WPSGD_LOSS == 1
#define WPSGD_VARIANTS_WIDE(V) V(1024, 64, 8, 1, 1) V(512, 128, 8, 1, 1)
#else
#define WPSGD_VARIANTS_WIDE(V)
#endif
#else
#define WPSGD_VARIANTS_VEC(V)                                                                  \
    V(64, 4, 4, 1, 8) V(64, 4, 4, 1, 16) V(64, 4, 4, 2, 4) V(64, 4, 4, 4, 2)                   \
    V(256, 4, 4, 1, 8) V(256, 8, 4, 1, 8) V(256, 16, 4, 4, 2) V(256, 32, 4, 1, 4)              \
    V(256, 4, 4, 4, 2) V(256, 8, 4, 4, 2) V(256, 16, 4, 1, 8) V(256, 16, 4, 1, 4)              \
    V(256, 16, 4, 2, 2) V(256, 16, 4, 2, 4) V(256, 16, 4, 4, 3) V(256, 32, 4, 4, 2)            \
    V(512, 8, 4, 1, 8) V(512, 8, 4, 4, 2) V(512, 8, 4, 2, 4)                                   \
    V(1024, 4, 4, 1, 8) V(1024, 4, 4, 4, 2) V(1024, 4, 4, 2, 4)                                \
    V(1024, 16, 4, 1, 2) V(1024, 16, 4, 2, 1) V(1024, 32, 4, 1, 1)
#define WPSGD_VARIANTS_WIDE(V)
#endif

#define WPSGD_ALL_VARIANTS(V) WPSGD_VARIANTS_VEC(V) WPSGD_VARIANTS_ANY(V) WPSGD_VARIANTS_WIDE(V)

#define WPSGD_CAT2(a, b) a##b
#define WPSGD_CAT(a, b) WPSGD_CAT2(a, b)
#if WPSGD_TX_BF16
#define WPSGD_SUFFIX WPSGD_CAT(bf16_loss, WPSGD_LOSS)
#else
#define WPSGD_SUFFIX WPSGD_CAT(f32_loss, WPSGD_LOSS)
#endif

// find(plan, launch?): walks the table; exact match on (threads, ept, vec, B, P) where the plan
// gives B and P, else the first entry of the shape.
hipError_t WPSGD_CAT(dense_reg_dispatch_, WPSGD_SUFFIX)(Plan &p, const ChainArgs *a, hipStream_t s)
{
#define WPSGD_TRY(NT, EPT, VEC, BB, PP)                                                        \
    if (p.threads == NT && p.ept == EPT && p.vec == VEC && (p.block_steps == 0 || p.block_steps == BB) && \
        (p.prefetch == 0 || p.prefetch == PP)) {                                               \
        p.block_steps = BB;                                                                    \
        p.prefetch = PP;                                                                       \
        if (a) {                                                                               \
            if ((int64_t)NT * EPT == a->d)                                                     \
                hipLaunchKernelGGL((chain_dense_reg_kernel<RowElem, kLoss, NT, EPT, VEC, BB, PP, true>),  \
                                   dim3(a->k), dim3(NT), 0, s, *a);                            \
            else                                                                               \
                hipLaunchKernelGGL((chain_dense_reg_kernel<RowElem, kLoss, NT, EPT, VEC, BB, PP, false>), \
                                   dim3(a->k), dim3(NT), 0, s, *a);                            \
            return hipGetLastError();                                                          \
        }                                                                                      \
        return hipSuccess;                                                                     \
    }
    WPSGD_ALL_VARIANTS(WPSGD_TRY)
#undef WPSGD_TRY
    return hipErrorInvalidValue;
}

// shape table for the planner: does (threads, ept, vec) exist for this storage/loss?
bool WPSGD_CAT(dense_reg_shape_, WPSGD_SUFFIX)(int threads, int ept, int vec)
{
#define WPSGD_TRY(NT, EPT, VEC, BB, PP) if (threads == NT && ept == EPT && vec == VEC) return true;
    WPSGD_ALL_VARIANTS(WPSGD_TRY)
#undef WPSGD_TRY
    return false;
}

}  // namespace wpsgd
