// Weighted model average  w_out[c] = sum_i a_i W[i,c]  (the aggregation line of Algorithm 1;
// Lemma 3) and the device-side view of the sample stream.
//
// The average is a pure stream over the k x d matrix W: every column is owned by one thread
// (four adjacent columns when alignment allows), rows are walked in ascending order with
// several loads in flight, and the sum is kept in fp64 and rounded once.  When there are too
// few columns to fill the chip, the rows are split over RS slices of a workgroup whose partial
// sums are added in slice order through LDS, so the result does not depend on timing.
#include "device_utils.h"
#include "internal.h"

namespace wpsgd {

constexpr int kCombineThreads = 256;

template <int VEC, int RS, int THREADS = kCombineThreads>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(6))) void combine_kernel(const float *__restrict__ W,
                                                                  const double *__restrict__ a,
                                                                  int k, int64_t d,
                                                                  float *__restrict__ out)
{
    constexpr int CT = THREADS / RS;                  // column-owning threads per workgroup
    constexpr int UNROLL = 16;                        // rows requested before the first is used
    constexpr int TAIL = 4;                           // the same for the rows left over
    __shared__ double part[RS][CT][VEC];
    const int cx = threadIdx.x % CT;
    const int slice = threadIdx.x / CT;
    const int64_t col = ((int64_t)blockIdx.x * CT + cx) * VEC;
    const bool in = col < d;

    double acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = 0.0;

    if (in) {
        // slice r owns rows [r*per, min(k, (r+1)*per))
        const int per = (k + RS - 1) / RS;
        const int i0 = slice * per;
        const int i1 = (i0 + per < k) ? i0 + per : k;
        int i = i0;
        for (; i + UNROLL <= i1; i += UNROLL) {
            float x[UNROLL][VEC];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const float *p = W + (int64_t)(i + u) * d + col;
                // every element of W is read once: non-temporal loads keep it from displacing anything
                // (16 rows in flight and this hint: 4.3 -> 5.5 TB/s at k = 128, d = 2^20; the kernel
                // must stay under 80 registers for that: at 94 it fell back to 4.5)
                if constexpr (VEC == 4) {
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    const f32x4 q = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
                    x[u][0] = q[0]; x[u][1] = q[1]; x[u][2] = q[2]; x[u][3] = q[3];
                } else {
                    x[u][0] = __builtin_nontemporal_load(p);
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const double w = a[i + u];
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] += w * (double)x[u][j];
            }
        }
        for (; i < i1; i += TAIL) {
            const int left = i1 - i;
            float x[TAIL][VEC];
#pragma unroll
            for (int u = 0; u < TAIL; ++u) {
                if (u < left) {
                    const float *p = W + (int64_t)(i + u) * d + col;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) x[u][j] = p[j];
                }
            }
#pragma unroll
            for (int u = 0; u < TAIL; ++u) {
                if (u < left) {
                    const double w = a[i + u];
#pragma unroll
                    for (int j = 0; j < VEC; ++j) acc[j] += w * (double)x[u][j];
                }
            }
        }
    }

    if constexpr (RS > 1) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) part[slice][cx][j] = acc[j];
        __syncthreads();
        if (slice == 0 && in) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                double t = part[0][cx][j];
                for (int r = 1; r < RS; ++r) t += part[r][cx][j];
                acc[j] = t;
            }
        }
    }
    if (slice == 0 && in) {
        if constexpr (VEC == 4) {
            *reinterpret_cast<float4 *>(out + col) =
                make_float4((float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]);
        } else {
            out[col] = (float)acc[0];
        }
    }
}

template <int VEC>
static hipError_t launch_combine_vec(const float *W, const double *a, int k, int64_t d, float *out,
                                     hipStream_t s)
{
    const int64_t col_threads = (d + VEC - 1) / VEC;
    // enough workgroups to cover the chip several times over -> no row split
    int rs = 1;
    if (col_threads < 256 * 1024 && k >= 64) rs = 4;
    if (col_threads < 64 * 1024 && k >= 256) rs = 16;
    // Very few columns, very many rows (2048 chains of 256 columns): 1024 threads, 64 slices of the
    // rows per workgroup, so that a thread walks 32 rows instead of 128 (one dependent batch of
    // loads instead of eight).
    if (col_threads <= 1024 && k >= 1024) {
        const unsigned grid64 = (unsigned)((col_threads + 15) / 16);
        hipLaunchKernelGGL((combine_kernel<VEC, 64, 1024>), dim3(grid64), dim3(1024), 0, s, W, a, k, d, out);
        return hipGetLastError();
    }
    const int ct = kCombineThreads / rs;
    const unsigned grid = (unsigned)((col_threads + ct - 1) / ct);
    if (rs == 1)
        hipLaunchKernelGGL((combine_kernel<VEC, 1>), dim3(grid), dim3(kCombineThreads), 0, s, W, a, k, d, out);
    else if (rs == 4)
        hipLaunchKernelGGL((combine_kernel<VEC, 4>), dim3(grid), dim3(kCombineThreads), 0, s, W, a, k, d, out);
    else
        hipLaunchKernelGGL((combine_kernel<VEC, 16>), dim3(grid), dim3(kCombineThreads), 0, s, W, a, k, d, out);
    return hipGetLastError();
}

hipError_t launch_combine(const float *W, const double *a_dev, int k, int64_t d, float *w_out,
                          hipStream_t s)
{
    const bool wide = (d % 4 == 0) && ((uintptr_t)W % 16 == 0) && ((uintptr_t)w_out % 16 == 0);
    return wide ? launch_combine_vec<4>(W, a_dev, k, d, w_out, s)
                : launch_combine_vec<1>(W, a_dev, k, d, w_out, s);
}

// Rows visited by one chain at steps n0 .. n0+count-1, produced by the same per-wave window the
// chain kernels read (so this kernel checks their generator, not a copy of it).
__global__ __launch_bounds__(kWave) void sample_rows_kernel(uint32_t seed_lo, uint32_t seed_hi,
                                                            uint32_t chain, int64_t n0,
                                                            int64_t count, uint32_t m, uint32_t shard_k,
                                                            int64_t *out)
{
    const int64_t per = (count + gridDim.x - 1) / gridDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * per;
    const int64_t t1 = (t0 + per < count) ? t0 + per : count;
    if (shard_k) {     // partition-and-shuffle order, evaluated directly
        for (int64_t t = t0 + threadIdx.x; t < t1; t += kWave)
            out[t] = (int64_t)shard_row(seed_lo, seed_hi, chain, shard_k, (uint64_t)(n0 + t), m);
        return;
    }
    RowWindow win;
    win.init(seed_lo, seed_hi, chain, m);
    for (int64_t t = t0; t < t1; ++t) {
        const uint32_t row = win.get(n0 + t);
        if (threadIdx.x == 0) out[t] = (int64_t)row;
    }
}

// The shuffled row order pi(0), .., pi(m-1) of partition-and-shuffle sampling, one entry per thread.
__global__ __launch_bounds__(256) void permute_rows_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t m,
                                                           uint32_t half, uint32_t *perm)
{
    const uint64_t pos = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (pos < m) perm[pos] = permute_row((uint32_t)pos, m, half, seed_lo, seed_hi);
}

hipError_t launch_permute_rows(uint32_t seed_lo, uint32_t seed_hi, uint32_t m, uint32_t *perm, hipStream_t s)
{
    const unsigned grid = (unsigned)(((uint64_t)m + 255) / 256);
    hipLaunchKernelGGL(permute_rows_kernel, dim3(grid), dim3(256), 0, s, seed_lo, seed_hi, m, feistel_half_bits(m), perm);
    return hipGetLastError();
}

// Streaming ceiling probe: `groups` workgroups each read `rows_per_group` rows of a dense matrix
// in the order the sample stream of chain `blockIdx.x` names them, with 64 to 128 KiB in flight, and do
// nothing else.  It measures how fast that many compute units can pull rows out of HBM at all,
// which bounds any kernel that gives one chain to one workgroup.
constexpr int kProbeThreads = 256;
constexpr int kProbeDepth = 4;
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kProbeThreads) void stream_rows_kernel(const char *X, int64_t row_stride,
                                                                    uint32_t row_bytes, uint32_t m,
                                                                    int64_t rows_per_group,
                                                                    uint32_t seed_lo, uint32_t seed_hi,
                                                                    float *sink)
{
    constexpr int kSeg = 4;                              // load instructions per segment
    RowWindow win;
    win.init(seed_lo, seed_hi, blockIdx.x, m);
    const uint32_t lane_off = threadIdx.x * 16u;
    constexpr uint32_t kSegBytes = kSeg * kProbeThreads * 16u;      // 16 KiB
    const uint32_t segs_per_row = (row_bytes + kSegBytes - 1) / kSegBytes;
    const int64_t segments = rows_per_group * segs_per_row;
    float acc = 0.0f;
    // A row is cut into 16 KiB segments; kProbeDepth segments are in flight, each slot being
    // consumed and re-requested in turn.
    probe_u32x4 q[kProbeDepth][kSeg];
    int64_t next_row = 0;
    uint32_t next_seg = 0;
    auto issue = [&](int u) {
        const int64_t r = next_row < rows_per_group ? next_row : rows_per_group - 1;
        const uint32_t row = win.get(r);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(X + (int64_t)row * row_stride), 0, (int)row_bytes, 0x00020000);
        const uint32_t base = next_seg * kSegBytes + lane_off;
#pragma unroll
        for (int c = 0; c < kSeg; ++c)
            q[u][c] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, base + c * kProbeThreads * 16u, 0, 0);
        if (++next_seg == segs_per_row) {
            next_seg = 0;
            ++next_row;
        }
    };
#pragma unroll
    for (int u = 0; u < kProbeDepth; ++u) issue(u);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    for (int64_t done = 0; done < segments; done += kProbeDepth) {
#pragma unroll
        for (int u = 0; u < kProbeDepth; ++u) {
#pragma unroll
            for (int c = 0; c < kSeg; ++c) acc += __uint_as_float(q[u][c][0]);
            issue(u);
        }
    }
    sink[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = acc;
}

hipError_t launch_stream_rows(const void *X, int64_t row_stride, uint32_t row_bytes, uint32_t m,
                              int groups, int64_t rows_per_group, uint32_t seed_lo, uint32_t seed_hi,
                              float *sink, hipStream_t s)
{
    hipLaunchKernelGGL(stream_rows_kernel, dim3(groups), dim3(kProbeThreads), 0, s,
                       static_cast<const char *>(X), row_stride, row_bytes, m, rows_per_group, seed_lo,
                       seed_hi, sink);
    return hipGetLastError();
}

__global__ void zero_words_kernel(uint32_t *p, size_t words)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// a fill kernel rather than a memset: the call may sit inside a captured graph
hipError_t launch_zero_words(uint32_t *p, size_t words, hipStream_t s)
{
    if (words == 0) return hipSuccess;
    const unsigned grid = (unsigned)((words + 255) / 256 < 256 ? (words + 255) / 256 : 256);
    hipLaunchKernelGGL(zero_words_kernel, dim3(grid), dim3(256), 0, s, p, words);
    return hipGetLastError();
}

hipError_t launch_sample_rows(uint32_t seed_lo, uint32_t seed_hi, uint32_t chain, int64_t n0,
                              int64_t count, uint32_t m, uint32_t shard_k, int64_t *out, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    const unsigned grid = (unsigned)((count + 255) / 256 < 1024 ? (count + 255) / 256 : 1024);
    hipLaunchKernelGGL(sample_rows_kernel, dim3(grid), dim3(kWave), 0, s, seed_lo, seed_hi, chain, n0,
                       count, m, shard_k, out);
    return hipGetLastError();
}

}  // namespace wpsgd
