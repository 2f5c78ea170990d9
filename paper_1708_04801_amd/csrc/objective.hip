// Regularised objective and prediction error of a model on a data set (Eq. 3 with Eq. 4):
//     c(w) = lambda/2 |w|^2 + (1/m) sum_j L(x_j, y_j, w.x_j),   error = #{ j : y_j (w.x_j) <= 0 } / m.
//
// A pure stream over the data: one wavefront takes one row at a time (lanes across the row's
// columns or entries), accumulates w.x in fp64 (the products of two fp32 numbers are exact in
// fp64, so the only rounding is in the order of the sum), reduces across the wave and adds the
// row's loss to its own running total.  Which rows a wave takes, and the order in which the
// waves' totals are added, are fixed by the launch shape, so the result does not depend on
// timing.  The model vector is read through the cache hierarchy (it is at most a few MiB).
#include <atomic>

#include "device_utils.h"
#include "internal.h"

namespace wpsgd {
namespace {

constexpr int kObjThreads = 256;
constexpr int kObjWaves = kObjThreads / kWave;
typedef uint32_t ou32x4 __attribute__((ext_vector_type(4)));

// loss and "wrong side" indicator of one row from z = y * yhat, both in fp64
__device__ inline void row_loss(int loss, double z, double &l, double &wrong)
{
    if (loss == kLossHinge) {
        l = (z < 1.0) ? 1.0 - z : 0.0;
    } else {
        l = (z > 0.0) ? log1p(exp(-z)) : -z + log1p(exp(z));     // log(1 + exp(-z)) without overflow
    }
    wrong = (z <= 0.0) ? 1.0 : 0.0;
}

// Every wave also adds up the squares of its share of the model vector (for the regulariser): one
// workgroup doing that alone took 0.27 ms at d = 2^20, two thirds as long as the rows themselves.
__device__ inline double squares_of_my_share(const float *w, int64_t d, int64_t wave_id, int64_t nwaves, int lane)
{
    const int64_t per = (d + nwaves - 1) / nwaves;
    const int64_t c0 = wave_id * per, c1 = c0 + per < d ? c0 + per : d;
    double sq = 0.0;
    for (int64_t c = c0 + lane; c < c1; c += kWave) sq += (double)w[c] * (double)w[c];
    return wave_sum(sq);
}

// Rows are read once and the model vector over and over: the rows' loads carry the non-temporal
// hint (cache-policy bit 1 of a buffer load), which keeps them from displacing it (+4 % at 16 KiB rows).
constexpr int kReadOnce = 2;

// VEC elements per lane and load (16 bytes when VEC > 1); RB rows in flight per wave.
template <typename TX, int VEC, int RB>
__global__ __launch_bounds__(kObjThreads) void objective_dense_kernel(const char *X, int64_t row_stride, int64_t m,
                                                                     int64_t d, const float *y, const float *w, int loss,
                                                                     double *partials)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave_id = (int64_t)blockIdx.x * kObjWaves + threadIdx.x / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * kObjWaves;
    const uint32_t row_bytes = (uint32_t)(d * (int64_t)sizeof(TX));
    const __amdgpu_buffer_rsrc_t wres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(w), 0, (int)(uint32_t)(d * 4), 0x00020000);
    const int64_t span = (int64_t)kWave * VEC;                 // columns one wave covers per load
    double loss_sum = 0.0, wrong_sum = 0.0;

    for (int64_t row0 = wave_id * RB; row0 < m; row0 += nwaves * RB) {
        double acc[RB];
        __amdgpu_buffer_rsrc_t xres[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            acc[r] = 0.0;
            const int64_t row = row0 + r < m ? row0 + r : m - 1;          // past the end: a row that is ignored below
            xres[r] = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(X + row * row_stride), 0, (int)row_bytes, 0x00020000);
        }
#pragma unroll 2
        for (int64_t c0 = 0; c0 < d; c0 += span) {
            const uint32_t col = (uint32_t)(c0 + (int64_t)lane * VEC);
            float wv[VEC];
            if constexpr (VEC == 1) {
                wv[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(wres, col * 4u, 0, 0));
            } else {
#pragma unroll
                for (int q = 0; q < VEC / 4; ++q) {
                    const ou32x4 t = __builtin_amdgcn_raw_buffer_load_b128(wres, col * 4u + q * 16u, 0, 0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) wv[q * 4 + i] = __uint_as_float(t[i]);
                }
            }
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                float xv[VEC];
                if constexpr (VEC == 1) {
                    if constexpr (sizeof(TX) == 2)
                        xv[0] = bf16_one((uint16_t)__builtin_amdgcn_raw_buffer_load_b16(xres[r], col * 2u, 0, kReadOnce));
                    else
                        xv[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(xres[r], col * 4u, 0, kReadOnce));
                } else {
                    const ou32x4 t = __builtin_amdgcn_raw_buffer_load_b128(xres[r], col * (uint32_t)sizeof(TX), 0, kReadOnce);
                    if constexpr (sizeof(TX) == 2) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            xv[2 * i] = bf16_lo(t[i]);
                            xv[2 * i + 1] = bf16_hi(t[i]);
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) xv[i] = __uint_as_float(t[i]);
                    }
                }
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[r] += (double)wv[i] * (double)xv[i];
            }
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const double yhat = wave_sum(acc[r]);
            if (row0 + r < m) {                                 // uniform
                double l, wr;
                row_loss(loss, (double)y[row0 + r] * yhat, l, wr);
                loss_sum += l;
                wrong_sum += wr;
            }
        }
    }
    const double sq = squares_of_my_share(w, d, wave_id, nwaves, lane);
    if (lane == 0) {
        partials[3 * wave_id] = loss_sum;
        partials[3 * wave_id + 1] = wrong_sum;
        partials[3 * wave_id + 2] = sq;
    }
}

__global__ __launch_bounds__(kObjThreads) void objective_csr_kernel(const int64_t *row_ptr, const int32_t *col_idx,
                                                                   const float *vals, int64_t m, int64_t d, const float *y,
                                                                   const float *w, int loss, double *partials)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave_id = (int64_t)blockIdx.x * kObjWaves + threadIdx.x / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * kObjWaves;
    double loss_sum = 0.0, wrong_sum = 0.0;
    for (int64_t row = wave_id; row < m; row += nwaves) {
        const int64_t p0 = row_ptr[row], p1 = row_ptr[row + 1];
        double acc = 0.0;
        for (int64_t p = p0 + lane; p < p1; p += kWave) acc += (double)w[col_idx[p]] * (double)vals[p];
        const double yhat = wave_sum(acc);
        double l, wr;
        row_loss(loss, (double)y[row] * yhat, l, wr);
        loss_sum += l;
        wrong_sum += wr;
    }
    const double sq = squares_of_my_share(w, d, wave_id, nwaves, lane);
    if (lane == 0) {
        partials[3 * wave_id] = loss_sum;
        partials[3 * wave_id + 1] = wrong_sum;
        partials[3 * wave_id + 2] = sq;
    }
}

// One workgroup: adds the waves' totals (losses, wrong predictions, squares) in wave order and writes the two results.
constexpr int kFinishThreads = 1024;
__global__ __launch_bounds__(kFinishThreads) void objective_finish_kernel(const double *partials, int64_t nwaves,
                                                                         int64_t m, double lambda, double *out)
{
    __shared__ double red[3][kFinishThreads];
    const int t = threadIdx.x;
    double a = 0.0, b = 0.0, sq = 0.0;
    for (int64_t i = t; i < nwaves; i += kFinishThreads) {
        a += partials[3 * i];
        b += partials[3 * i + 1];
        sq += partials[3 * i + 2];
    }
    red[0][t] = a;
    red[1][t] = b;
    red[2][t] = sq;
    __syncthreads();
    for (int s = kFinishThreads / 2; s > 0; s >>= 1) {
        if (t < s) {
            red[0][t] += red[0][t + s];
            red[1][t] += red[1][t + s];
            red[2][t] += red[2][t + s];
        }
        __syncthreads();
    }
    if (t == 0) {
        out[0] = 0.5 * lambda * red[2][0] + red[0][0] / (double)m;
        out[1] = red[1][0] / (double)m;
    }
}

// The workgroups walk the rows with a stride of the whole grid, so the grid should be exactly what the
// device holds at once: with more, the surplus runs as a second, thinly occupied round (2048
// workgroups where 1536 fit cost 14 % at 16 KiB rows, 2048 where 1280 fit 11 % at 1 KiB rows).
// Asked once per kernel.
template <auto kernel>
unsigned resident_grid(unsigned most)
{
    static std::atomic<unsigned> cached{0};        // (one instance per kernel; working it out twice is harmless)
    unsigned resident = cached.load(std::memory_order_relaxed);
    if (resident == 0) {
        // a workgroup is one wave on each of a compute unit's four SIMDs; a SIMD has 512 registers
        // per lane, handed out in blocks of eight, and room for eight waves
        hipFuncAttributes attr;
        int dev = 0, cus = 0;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(kernel)) != hipSuccess || hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || attr.numRegs < 1 || cus < 1) {
            (void)hipGetLastError();
            return most;
        }
        const int blocks = (attr.numRegs + 7) / 8 * 8;
        const int per_cu = blocks >= 512 ? 1 : (512 / blocks < 8 ? 512 / blocks : 8);
        resident = (unsigned)per_cu * (unsigned)cus;
        cached.store(resident, std::memory_order_relaxed);
    }
    return resident < most ? resident : most;
}

template <typename TX, int VEC>
unsigned launch_dense_rows(int rb, unsigned most, hipStream_t s, const char *X, int64_t stride, int64_t m, int64_t d,
                           const float *y, const float *w, int loss, double *partials)
{
    unsigned grid;
    if (rb == 4) {
        grid = resident_grid<objective_dense_kernel<TX, VEC, 4>>(most);
        hipLaunchKernelGGL((objective_dense_kernel<TX, VEC, 4>), dim3(grid), dim3(kObjThreads), 0, s, X, stride, m, d, y, w, loss, partials);
    } else {
        grid = resident_grid<objective_dense_kernel<TX, VEC, 1>>(most);
        hipLaunchKernelGGL((objective_dense_kernel<TX, VEC, 1>), dim3(grid), dim3(kObjThreads), 0, s, X, stride, m, d, y, w, loss, partials);
    }
    return grid;
}

}  // namespace

int64_t objective_grid(int64_t m)
{
    const int64_t want = (m + kObjWaves - 1) / kObjWaves;
    return want < 2048 ? want : 2048;          // at most eight workgroups per compute unit (the launch takes what fits)
}

size_t objective_partials_bytes(int64_t m) { return (size_t)objective_grid(m) * kObjWaves * 3 * sizeof(double); }

// Partial sums for callers that cannot allocate (wpsgd_objective_static): room for the largest launch,
// 2048 workgroups of four waves with three sums each - 192 KiB that every device the library runs
// on holds until the process ends.  Host code never uses the array's name as an address: it asks for
// the device address once per device and passes that to the kernels, as it passes a workspace.
constexpr size_t kStaticPartials = (size_t)2048 * kObjWaves * 3;
static __device__ __align__(256) double scratch[kStaticPartials];

hipError_t objective_static_partials(double **partials, size_t *bytes)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<double *> address[kMaxDevices];      // (two threads asking at once get the same answer)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    double *p = address[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        address[dev].store(p, std::memory_order_release);
    }
    *partials = p;
    *bytes = kStaticPartials * sizeof(double);
    return hipSuccess;
}

hipError_t launch_objective(const ChainArgs &a, int dtype, int vec, int loss, const float *w, double lambda,
                            double *partials, double *out, hipStream_t s)
{
    const unsigned most = (unsigned)objective_grid(a.m);      // what the partial sums have room for
    unsigned grid = most;
    if (a.dense) {
        const char *X = static_cast<const char *>(a.dense);
        const int elem = dtype == WPSGD_BF16 ? 2 : 4;
        const int64_t stride = a.ld * elem;
        const int rb = a.d <= (int64_t)kWave * vec * 2 ? 4 : 1;     // short rows: several in flight per wave
        if (dtype == WPSGD_BF16) {
            if (vec > 1) grid = launch_dense_rows<uint16_t, 8>(rb, most, s, X, stride, a.m, a.d, a.y, w, loss, partials);
            else grid = launch_dense_rows<uint16_t, 1>(rb, most, s, X, stride, a.m, a.d, a.y, w, loss, partials);
        } else {
            if (vec > 1) grid = launch_dense_rows<float, 4>(rb, most, s, X, stride, a.m, a.d, a.y, w, loss, partials);
            else grid = launch_dense_rows<float, 1>(rb, most, s, X, stride, a.m, a.d, a.y, w, loss, partials);
        }
    } else {
        grid = resident_grid<objective_csr_kernel>(most);
        hipLaunchKernelGGL(objective_csr_kernel, dim3(grid), dim3(kObjThreads), 0, s, a.row_ptr, a.col_idx, a.vals, a.m,
                           a.d, a.y, w, loss, partials);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t nwaves = (int64_t)grid * kObjWaves;
    hipLaunchKernelGGL(objective_finish_kernel, dim3(1), dim3(kFinishThreads), 0, s, partials, nwaves, a.m, lambda, out);
    return hipGetLastError();
}

}  // namespace wpsgd
