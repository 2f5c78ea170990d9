// Device-side building blocks shared by the chain kernels: the counter-based sample stream,
// wavefront reductions, bfloat16 unpacking and the loss slope.  gfx950 only (64-wide waves).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wpsgd {

constexpr int kWave = 64;
constexpr int kLossHinge = 0;
constexpr int kLossLogistic = 1;

// ---------------------------------------------------------------------------------------------
// Sample stream.  Philox4x32-10 (Salmon et al., SC'11): ten rounds of
//   (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
// with the key advanced by the two Weyl constants after every round.  Only output word 0 is
// used: row = floor(word0 * m / 2^32).  Counter = (step lo, step hi, chain, 0), key = seed.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline uint32_t mul_hi_u32(uint32_t a, uint32_t b)
{
    return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);   // lowers to v_mul_hi_u32 on the GPU
}

__host__ __device__ inline uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = mul_hi_u32(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = mul_hi_u32(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    return c0;
}

__host__ __device__ inline uint32_t sample_row(uint32_t seed_lo, uint32_t seed_hi, uint32_t chain,
                                               uint64_t step, uint32_t m)
{
    const uint32_t r0 = philox4x32_10_word0((uint32_t)step, (uint32_t)(step >> 32), chain, 0u,
                                            seed_lo, seed_hi);
    return mul_hi_u32(r0, m);
}

// One wave's window onto a chain's sample stream: lane l holds the row of step base+l.
// get(step) must be called with a wave-uniform step; it refills the window (64 Philox
// evaluations, one per lane) whenever the step leaves it.
struct RowWindow {
    uint32_t seed_lo, seed_hi, chain, m;
    int64_t base;
    uint32_t rows;

    __device__ void init(uint32_t slo, uint32_t shi, uint32_t c, uint32_t mm)
    {
        seed_lo = slo; seed_hi = shi; chain = c; m = mm;
        base = -1;
        rows = 0;
    }
    __device__ uint32_t get(int64_t step)
    {
        const int64_t b = step & ~(int64_t)(kWave - 1);
        if (b != base) {
            base = b;
            rows = sample_row(seed_lo, seed_hi, chain, (uint64_t)(b + (int)(threadIdx.x & (kWave - 1))), m);
        }
        return (uint32_t)__builtin_amdgcn_readlane((int)rows, (int)(step & (kWave - 1)));
    }
};

// ---------------------------------------------------------------------------------------------
// Wavefront sum, result in every lane.  Butterfly over lane ^ 1, 2, 4, 8, 16, 32.
// ---------------------------------------------------------------------------------------------
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ inline double wave_sum(double v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// bfloat16 is the upper half of a binary32: widening is a shift.
__device__ inline float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ inline float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }
__device__ inline float bf16_one(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// dL/dyhat (Eq. 4 with the two losses this library offers).
template <int LOSS>
__device__ inline double loss_slope(double y, double yhat)
{
    if constexpr (LOSS == kLossHinge) {
        return (y * yhat < 1.0) ? -y : 0.0;
    } else {
        return -y / (1.0 + exp(y * yhat));
    }
}

// Model-vector precision by loss: the hinge slope is discontinuous in yhat, so a rounding-size
// error in w can flip a step and displace the chain by eta*|x|; its state and dot products are
// carried in fp64.  The logistic slope is smooth and fp32 state is accurate to ~1e-6.
template <int LOSS> struct StateType { using type = float; };
template <> struct StateType<kLossHinge> { using type = double; };

}  // namespace wpsgd
