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

// ---------------------------------------------------------------------------------------------
// Sampling as Algorithm 1 writes it: the examples are randomly partitioned among the k nodes and
// every node walks its own part in random order.  Kept counter-based: one keyed permutation pi
// of [0, m) (a four-round Feistel network over 2*half bits whose round function is Philox, with
// cycle walking to stay inside [0, m)) shuffles all rows; node i owns the permuted positions
// [floor(i*m/k), floor((i+1)*m/k)) and visits them in order, starting over when it has seen them
// all.  Row of node i at step n:  pi(lo_i + n mod m_i).
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline uint32_t feistel_half_bits(uint32_t m)
{
    uint32_t bits = 0;                       // bits needed for m-1
    for (uint32_t x = m - 1; x != 0; x >>= 1) ++bits;
    const uint32_t half = (bits + 1) / 2;
    return half == 0 ? 1u : half;
}

__host__ __device__ inline uint32_t permute_row(uint32_t x, uint32_t m, uint32_t half, uint32_t seed_lo,
                                                uint32_t seed_hi)
{
    const uint32_t mask = (1u << half) - 1u;
    do {
        uint32_t L = x >> half, Rr = x & mask;
#pragma unroll
        for (uint32_t r = 0; r < 4; ++r) {
            const uint32_t f = philox4x32_10_word0(Rr, r, 0x5348524Du, 0xFFFFFFFFu, seed_lo, seed_hi) & mask;
            const uint32_t t = L ^ f;
            L = Rr;
            Rr = t;
        }
        x = (L << half) | Rr;
    } while (x >= m);                        // the network permutes [0, 4^half); walk the cycle back into [0, m)
    return x;
}

__host__ __device__ inline uint32_t shard_row(uint32_t seed_lo, uint32_t seed_hi, uint32_t chain, uint32_t k,
                                              uint64_t step, uint32_t m)
{
    const uint64_t lo = ((uint64_t)chain * m) / k, hi = ((uint64_t)(chain + 1) * m) / k;
    const uint64_t len = hi - lo;            // >= 1 because k <= m
    return permute_row((uint32_t)(lo + step % len), m, feistel_half_bits(m), seed_lo, seed_hi);
}

// Position in the shuffled order of the row node `chain` of k visits at `step` (see above).
__host__ __device__ inline uint32_t shard_position(uint32_t chain, uint32_t k, uint64_t step, uint32_t m)
{
    const uint64_t lo = ((uint64_t)chain * m) / k, hi = ((uint64_t)(chain + 1) * m) / k;
    return (uint32_t)(lo + step % (hi - lo));
}

// Rows of the 64 steps starting at `base`, one per lane.  perm == nullptr: the with-replacement
// stream.  Otherwise partition-and-shuffle sampling over k nodes, with perm the shuffled order
// pi(0..m-1) tabulated beforehand (the chain kernels read it instead of evaluating pi).  Kept out
// of line: it runs once per 64 steps, and inlining its integer code at every use bloats the loops
// around it.
__device__ __attribute__((noinline)) inline uint32_t sample_window(uint32_t seed_lo, uint32_t seed_hi,
                                                                   uint32_t chain, int64_t base,
                                                                   uint32_t m, const uint32_t *perm = nullptr,
                                                                   uint32_t k = 1)
{
    const uint64_t step = (uint64_t)(base + (int)(threadIdx.x & (kWave - 1)));
    if (perm) return perm[shard_position(chain, k, step, m)];
    return sample_row(seed_lo, seed_hi, chain, step, m);
}

// One wave's window onto a chain's sample stream: lane l holds the row of step base+l.
// get(step) must be called with a wave-uniform step; it refills the window (64 Philox
// evaluations, one per lane) whenever the step leaves it.
struct RowWindow {
    uint32_t seed_lo, seed_hi, chain, m, k;
    const uint32_t *perm;
    int64_t base;
    uint32_t rows;

    __device__ void init(uint32_t slo, uint32_t shi, uint32_t c, uint32_t mm, const uint32_t *pm = nullptr,
                         uint32_t kk = 1)
    {
        seed_lo = slo; seed_hi = shi; chain = c; m = mm; perm = pm; k = kk;
        base = -1;
        rows = 0;
    }
    __device__ uint32_t get(int64_t step)
    {
        const int64_t b = step & ~(int64_t)(kWave - 1);
        if (b != base) {
            base = b;
            rows = sample_window(seed_lo, seed_hi, chain, b, m, perm, k);
        }
        return (uint32_t)__builtin_amdgcn_readlane((int)rows, (int)(step & (kWave - 1)));
    }
};

// ---------------------------------------------------------------------------------------------
// Wavefront sums on the DPP cross-lane network (no LDS traffic).
//
// dpp_move<CTRL, ROW_MASK>(x): every lane of an enabled 16-lane row receives x from the lane
// CTRL names; lanes of disabled rows receive 0.  Controls used (GFX9 encodings):
//   0xB1 quad_perm[1,0,3,2] (lane^1)   0x4E quad_perm[2,3,0,1] (lane^2)
//   0x141 row_half_mirror (7 - lane%8) 0x140 row_mirror (15 - lane%16)
//   0x142 row_bcast15: lane 15 of each row to every lane of the next row
//   0x143 row_bcast31: lane 31 to every lane of rows 2 and 3
// After the four in-row steps all 16 lanes of a row hold the row sum; bcast15 adds each row's sum
// to the next row, then bcast31 adds row 1's to rows 2 and 3: the wave total is in row 3, i.e. in
// lane 63 (and only there).
// ---------------------------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_move_bits(int x)
{
    if constexpr (ROW_MASK == 0xF) {
        // every lane has a valid source for the in-row controls: no fill value is needed
        return __builtin_amdgcn_mov_dpp(x, CTRL, 0xF, 0xF, true);
    } else {
        return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xF, false);
    }
}

template <int CTRL, int ROW_MASK>
__device__ inline float dpp_move(float x)
{
    return __int_as_float(dpp_move_bits<CTRL, ROW_MASK>(__float_as_int(x)));
}

template <int CTRL, int ROW_MASK>
__device__ inline double dpp_move(double x)
{
    const long long bits = __double_as_longlong(x);
    const int lo = dpp_move_bits<CTRL, ROW_MASK>((int)(bits & 0xFFFFFFFFLL));
    const int hi = dpp_move_bits<CTRL, ROW_MASK>((int)(bits >> 32));
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}

// Sum over the 64 lanes; the result is valid in lane 63 only.
template <typename T>
__device__ inline T wave_sum_lane63(T v)
{
    v += dpp_move<0xB1, 0xF>(v);
    v += dpp_move<0x4E, 0xF>(v);
    v += dpp_move<0x141, 0xF>(v);
    v += dpp_move<0x140, 0xF>(v);
    // The cross-row steps run unmasked: lanes without a source lane receive 0, rows 1 and 2 end up
    // with sums nobody reads, and row 3 - lane 63 - adds (r3 + r2) + (r1 + r0) as it should.  (Masked
    // to the rows that matter, each step would first need a zero moved into the other rows.)
    v += dpp_move<0x142, 0xF>(v);
    v += dpp_move<0x143, 0xF>(v);
    return v;
}

// fp32: the two cross-row steps as single fused instructions (the masked rows keep their value,
// so no zero has to be moved in first).  The same additions in the same order as above.  A DPP
// operand written by the preceding VALU instruction needs two wait states.
template <>
__device__ inline float wave_sum_lane63<float>(float v)
{
    v += dpp_move<0xB1, 0xF>(v);
    v += dpp_move<0x4E, 0xF>(v);
    v += dpp_move<0x141, 0xF>(v);
    v += dpp_move<0x140, 0xF>(v);
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf"
                 : "+v"(v));
    return v;
}

// Three fp32 sums at once, level by level: each value's next level is two instructions behind its
// previous one, which is exactly the distance a DPP operand needs, so no idle slots are spent.
// Per value the additions and their order are those of wave_sum_lane63.
__device__ inline void wave_sum3_lane63(float &a, float &b, float &c)
{
#define WPSGD_DPP3(CTRL)                                                       \
    "v_add_f32_dpp %0, %0, %0 " CTRL "\n\t"                                     \
    "v_add_f32_dpp %1, %1, %1 " CTRL "\n\t"                                     \
    "v_add_f32_dpp %2, %2, %2 " CTRL "\n\t"
    asm volatile("s_nop 1\n\t"
                 WPSGD_DPP3("quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1")
                 WPSGD_DPP3("quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1")
                 WPSGD_DPP3("row_half_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1")
                 WPSGD_DPP3("row_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1")
                 WPSGD_DPP3("row_bcast:15 row_mask:0xa bank_mask:0xf")
                 WPSGD_DPP3("row_bcast:31 row_mask:0xc bank_mask:0xf")
                 : "+v"(a), "+v"(b), "+v"(c));
#undef WPSGD_DPP3
}

__device__ inline float read_lane63(float v)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), kWave - 1));
}

__device__ inline double read_lane63(double v)
{
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)(bits & 0xFFFFFFFFLL), kWave - 1);
    const int hi = __builtin_amdgcn_readlane((int)(bits >> 32), kWave - 1);
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}

// Is zs * (value in lane 63) < 1?  The hinge step of a one-wave chain needs only this one bit of the
// wave's sum, so the sum is not broadcast first: every lane compares, lane 63's answer counts.
__device__ inline bool lane63_below_one(double zs, double sum_in_lane63)
{
    return (__builtin_amdgcn_ballot_w64(zs * sum_in_lane63 < 1.0) >> (kWave - 1)) != 0;
}

// Sum over the 64 lanes, result in every lane.
template <typename T>
__device__ inline T wave_sum(T v)
{
    return read_lane63(wave_sum_lane63(v));
}

// Wave-uniform read of lane j of a per-lane value.
__device__ inline float lane_read(float t, int j)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), j));
}
__device__ inline int64_t lane_read_i64(int64_t t, int j)
{
    const int lo = __builtin_amdgcn_readlane((int)(t & 0xFFFFFFFFLL), j);
    const int hi = __builtin_amdgcn_readlane((int)(t >> 32), j);
    return ((int64_t)hi << 32) | (int64_t)(unsigned int)lo;
}
__device__ inline double lane_read(double t, int j)
{
    return __longlong_as_double(lane_read_i64(__double_as_longlong(t), j));
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
