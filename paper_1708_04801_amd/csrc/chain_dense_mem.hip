// Dense-row SGD chains with the model vector in HBM (the workspace), for dimensions that do
// not fit the register file of one workgroup.  Same recursion as the register kernel
// (Eq. 5 with Eq. 4, carried as w = s*v), one step per reduction round: a first pass over the
// row forms v.x, a second pass (the row is then an L2 hit) applies v += c*x.  Every thread
// touches the same columns in every pass, so the vector needs no synchronisation of its own.
#include "device_utils.h"
#include "internal.h"

namespace wpsgd {

template <typename TX, int VEC> struct RowChunk;
template <> struct RowChunk<float, 1> {
    float x[1];
    __device__ void load(const float *p) { x[0] = p[0]; }
};
template <> struct RowChunk<float, 4> {
    float x[4];
    __device__ void load(const float *p)
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
    }
};
template <> struct RowChunk<uint16_t, 1> {
    float x[1];
    __device__ void load(const uint16_t *p) { x[0] = bf16_one(p[0]); }
};
template <> struct RowChunk<uint16_t, 8> {
    float x[8];
    __device__ void load(const uint16_t *p)
    {
        const uint4 q = *reinterpret_cast<const uint4 *>(p);
        x[0] = bf16_lo(q.x); x[1] = bf16_hi(q.x); x[2] = bf16_lo(q.y); x[3] = bf16_hi(q.y);
        x[4] = bf16_lo(q.z); x[5] = bf16_hi(q.z); x[6] = bf16_lo(q.w); x[7] = bf16_hi(q.w);
    }
};

template <typename TX, int LOSS, int NT, int VEC>
__global__ __launch_bounds__(NT) void chain_dense_mem_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    constexpr int NW = NT / kWave;
    __shared__ TV red[2][NW];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const int64_t d = a.d;
    const TX *X = static_cast<const TX *>(a.dense);
    TV *v = static_cast<TV *>(a.state) + (int64_t)chain * d;

    for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC)
#pragma unroll
        for (int j = 0; j < VEC; ++j) v[col + j] = a.w_start ? (TV)a.w_start[col + j] : (TV)0;
    const int64_t step0 = a.step0[blockIdx.x];

    RowWindow win;
    win.init(a.seed_lo, a.seed_hi, (uint32_t)chain, (uint32_t)a.m, a.perm, (uint32_t)a.k);
    double s = 1.0, inv_s = 1.0;
    const double rho = a.rho, inv_rho = 1.0 / a.rho, eta = a.eta;
    int parity = 0;

    for (int64_t step = 0; step < n; ++step) {
        const uint32_t row = win.get(step0 + step);
        const TX *xr = X + (int64_t)row * a.ld;
        const double y = (double)a.y[row];
        TV acc = (TV)0;
        for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC) {
            RowChunk<TX, VEC> c;
            c.load(xr + col);
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc += v[col + j] * (TV)c.x[j];
        }
        acc = wave_sum(acc);
        if constexpr (NW > 1) {
            if (lane == 0) red[parity][wave] = acc;
            __syncthreads();
            TV t = red[parity][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) t += red[parity][w];
            acc = t;
            parity ^= 1;
        }
        const double slope = loss_slope<LOSS>(y, s * (double)acc);
        s *= rho;
        inv_s *= inv_rho;
        const TV coef = (TV)(-eta * slope * inv_s);
        if (coef != (TV)0) {
            for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC) {
                RowChunk<TX, VEC> c;
                c.load(xr + col);
#pragma unroll
                for (int j = 0; j < VEC; ++j) v[col + j] += coef * (TV)c.x[j];
            }
        }
        if (s < 0x1p-30) {
            for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC)
#pragma unroll
                for (int j = 0; j < VEC; ++j) v[col + j] *= (TV)s;
            s = 1.0;
            inv_s = 1.0;
        }
    }

    float *out = a.W + (int64_t)chain * d;
    for (int64_t col = (int64_t)tid * VEC; col < d; col += (int64_t)NT * VEC)
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[col + j] = (float)(s * (double)v[col + j]);
}

template <typename TX, int LOSS>
static hipError_t launch_tx_loss(const Plan &p, const ChainArgs &a, hipStream_t s)
{
    constexpr int WIDE = sizeof(TX) == 2 ? 8 : 4;
#define WPSGD_MEM_TRY(NT, VEC)                                                                 \
    if (p.threads == NT && p.vec == VEC) {                                                     \
        hipLaunchKernelGGL((chain_dense_mem_kernel<TX, LOSS, NT, VEC>), dim3(a.k), dim3(NT), 0, s, a); \
        return hipGetLastError();                                                              \
    }
    WPSGD_MEM_TRY(256, 1)
    WPSGD_MEM_TRY(256, WIDE)
    WPSGD_MEM_TRY(1024, 1)
    WPSGD_MEM_TRY(1024, WIDE)
#undef WPSGD_MEM_TRY
    return hipErrorInvalidValue;
}

hipError_t launch_dense_mem(const Plan &p, const ChainArgs &a, hipStream_t s)
{
    if (p.dtype == WPSGD_BF16)
        return p.loss == WPSGD_HINGE ? launch_tx_loss<uint16_t, kLossHinge>(p, a, s)
                                     : launch_tx_loss<uint16_t, kLossLogistic>(p, a, s);
    return p.loss == WPSGD_HINGE ? launch_tx_loss<float, kLossHinge>(p, a, s)
                                 : launch_tx_loss<float, kLossLogistic>(p, a, s);
}

}  // namespace wpsgd
