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

    for (int64_t col = lane; col < d; col += kWave) v[col] = (TV)0;
    __syncthreads();   // the zeros must be visible to whichever lane gathers them later

    RowWindow win;
    win.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m);
    double s = 1.0, inv_s = 1.0;
    const double rho = a.rho, inv_rho = 1.0 / a.rho, eta = a.eta;

    for (int64_t step = 0; step < n; ++step) {
        const uint32_t row = win.get(step);
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

hipError_t launch_csr(const Plan &p, const ChainArgs &a, hipStream_t s)
{
    if (p.loss == WPSGD_HINGE)
        hipLaunchKernelGGL((chain_csr_kernel<kLossHinge>), dim3(a.k), dim3(kWave), 0, s, a);
    else
        hipLaunchKernelGGL((chain_csr_kernel<kLossLogistic>), dim3(a.k), dim3(kWave), 0, s, a);
    return hipGetLastError();
}

}  // namespace wpsgd
