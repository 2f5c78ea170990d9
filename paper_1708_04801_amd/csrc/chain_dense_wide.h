// Dense chains whose rows are too long to wait in registers beside the model vector: rows
// streamed twice, or the next row staged in LDS.  Included by chain_dense_reg.hip, which
// instantiates and dispatches them.
#pragma once
#include "dense_rows.h"

namespace wpsgd {

// Wide rows: the model vector still lives in registers (1024 threads x EPT elements), but a row
// no longer fits beside it, so a step streams its row twice and keeps none of it: the first
// pass (from HBM) forms v.x, the second (the row is then in L2) applies v += c*x.  Same
// recursion, same per-window scalar tables, one step per round.
template <typename TX, int LOSS, int NT, int EPT, int VEC>
__global__ __launch_bounds__(NT) void chain_dense_wide_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    using Frag = RowFrag<TX, NT, VEC, VEC>;        // one chunk: VEC elements
    constexpr int NW = NT / kWave;
    constexpr int CHUNKS = EPT / VEC;
    constexpr int GROUP = CHUNKS >= 4 ? 4 : CHUNKS;    // chunks requested together
    constexpr int NGROUPS = CHUNKS / GROUP;
    static_assert(CHUNKS % GROUP == 0, "whole groups");
    __shared__ TV red[2][NW];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const char *X = static_cast<const char *>(a.dense);
    const int64_t row_stride = a.ld * (int64_t)sizeof(TX);
    const uint32_t row_bytes = (uint32_t)(a.d * (int64_t)sizeof(TX));
    float *out = a.W + (int64_t)chain * a.d;

    TV v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        v[e] = (a.w_start && col < a.d) ? (TV)a.w_start[col] : (TV)0;
    }
    const int64_t step0 = a.step0[blockIdx.x];

    if (n > 0) {
        const uint32_t off0 = (uint32_t)((tid * VEC) * sizeof(TX));          // chunk c adds c*NT*VEC elements
        constexpr uint32_t kChunkStride = (uint32_t)(NT * VEC * sizeof(TX));
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
        uint32_t rows = 0;
        TV zs_tab = (TV)0, cs_tab = (TV)0;
        int parity = 0;

        // Streams the row behind rx through f(e, x_e), GROUP chunks in flight ahead of their use.
        auto stream_row = [&](__amdgpu_buffer_rsrc_t rx, auto &&f) {
            Frag buf[2][GROUP];
#pragma unroll
            for (int c = 0; c < GROUP; ++c) buf[0][c].load_chunk(0, rx, off0 + c * kChunkStride);
#pragma unroll
            for (int g = 0; g < NGROUPS; ++g) {
                if (g + 1 < NGROUPS) {
#pragma unroll
                    for (int c = 0; c < GROUP; ++c)
                        buf[(g + 1) & 1][c].load_chunk(0, rx, off0 + ((g + 1) * GROUP + c) * kChunkStride);
                }
#pragma unroll
                for (int c = 0; c < GROUP; ++c)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) f((g * GROUP + c) * VEC + i, buf[g & 1][c].at(i));
            }
        };

        for (int64_t step = 0; step < n; ++step) {
            const int j = (int)(step & (kWave - 1));
            if (j == 0) {       // a new window of 64 steps
                if (step > 0) {
                    s_w *= rho64;
                    eos_w *= inv_rho64;
                    if (s_w < 0x1p-30) {
#pragma unroll
                        for (int e = 0; e < EPT; ++e) v[e] *= (TV)s_w;
                        s_w = 1.0;
                        eos_w = a.eta;
                    }
                }
                rows = sample_window(a.seed_lo, a.seed_hi, (uint32_t)chain, step0 + step, (uint32_t)a.m, a.perm, (uint32_t)a.k);
                const double sl = s_w * rho_pow, el = eos_w * inv_rho_pow1;
                if constexpr (LOSS == kLossHinge) {
                    zs_tab = sl;
                    cs_tab = el;
                } else {
                    zs_tab = (float)(sl * 1.4426950408889634);
                    cs_tab = (float)el;
                }
            }
            const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)rows, j);
            const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + (int64_t)row * row_stride, row_bytes);
            const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y + row, 4u);
            const TV y = (TV)__uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(ry, 0, 0, 0));

            TV acc[4] = {(TV)0, (TV)0, (TV)0, (TV)0};
            stream_row(rx, [&](int e, float xe) { acc[e & 3] += v[e] * (TV)xe; });
            TV tot = wave_sum_lane63((acc[0] + acc[1]) + (acc[2] + acc[3]));
            if (lane == kWave - 1) red[parity][wave] = tot;
            const TV zy = lane_read(zs_tab, j) * y, cy = lane_read(cs_tab, j) * y;
            __syncthreads();
            tot = red[parity][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) tot += red[parity][w];
            parity ^= 1;
            TV c;
            if constexpr (LOSS == kLossHinge) {
                c = (zy * tot < 1.0) ? cy : 0.0;
            } else {
                c = cy * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(zy * tot));
            }
            if (c != (TV)0)      // uniform: every thread holds the same c
                stream_row(rx, [&](int e, float xe) { v[e] += c * (TV)xe; });
        }
        const int64_t last_w = (n - 1) / kWave;
        const int rem = (int)(n - last_w * kWave);
        const double s_end = s_w * lane_read(rho_pow, rem - 1) * rho;
#pragma unroll
        for (int e = 0; e < EPT; ++e) v[e] = (TV)(s_end * (double)v[e]);
    }

#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        if (col < a.d) out[col] = (float)v[e];
    }
}

// Long rows that fit in LDS once (up to 128 KiB): the row of the current step sits in registers
// beside the model vector, the row of the next step travels from HBM straight into LDS (loads that
// land in LDS need no registers while they are in flight), and the dot product and the update both
// read the register copy, so a row crosses the memory system once.  Each wave owns the LDS slots of
// the chunks it loads and is the only one to read them, so the transfer needs no barrier: when a
// step is done the wave moves the next row, 1 KiB chunk by chunk, from LDS to registers and
// requests the same chunk of the row after that into the slot just freed.  Loads complete in
// issue order, so "at most CHUNKS-1 outstanding" means the oldest chunk has landed.
template <typename TX, int LOSS, int NT, int EPT, int VEC>
__global__ __launch_bounds__(NT) void chain_dense_lds_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    using Frag = RowFrag<TX, NT, EPT, VEC>;
    static_assert(VEC * sizeof(TX) == 16, "16-byte loads only");
    constexpr int NW = NT / kWave;
    constexpr int CHUNKS = EPT / VEC;
    static_assert(Frag::kWords == 4 * CHUNKS, "four words per chunk");
    static_assert(CHUNKS >= 1 && CHUNKS <= 8, "the wait below encodes CHUNKS-1 in four bits");
    __shared__ __attribute__((aligned(16))) uint32_t stage[NW][CHUNKS][kWave * 4];
    __shared__ TV red[2][NW];
    static_assert(sizeof(stage) <= 128 * 1024, "row must fit in LDS");

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);      // a scalar: registers are scarce here
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const char *X = static_cast<const char *>(a.dense);
    const int64_t row_stride = a.ld * (int64_t)sizeof(TX);
    const uint32_t row_bytes = (uint32_t)(a.d * (int64_t)sizeof(TX));
    float *out = a.W + (int64_t)chain * a.d;

    TV v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        v[e] = (a.w_start && col < a.d) ? (TV)a.w_start[col] : (TV)0;
    }
    const int64_t step0 = a.step0[blockIdx.x];

    if (n > 0) {
        const uint32_t off0 = (uint32_t)(tid * 16);                           // chunk c adds c*NT*16 bytes
        constexpr uint32_t kChunkStride = (uint32_t)(NT * 16);
        // Registers are what this kernel runs out of, so nothing that is only needed once per
        // window of 64 steps stays in one: (1-eta*lambda)^lane and its inverse are read from a
        // small table at every window start, and the next window's rows are computed when the
        // look-ahead first reaches into it.
        const double rho = a.rho;
        const double rho64 = a.pow_tab[kWave - 1] * rho, inv_rho64 = a.pow_tab[2 * kWave - 1];
        auto lane_powers = [&](double &rho_pow, double &inv_rho_pow1) {
            rho_pow = a.pow_tab[lane];
            inv_rho_pow1 = a.pow_tab[kWave + lane];
        };
        double s_w = 1.0, eos_w = a.eta;
        const uint32_t seed_lo = a.seed_lo, seed_hi = a.seed_hi, m32 = (uint32_t)a.m;
        // out of line: the registers are full of model and row here, and this runs once per 64 steps
        auto window_rows = [&](int64_t w) {
            return sample_window(seed_lo, seed_hi, (uint32_t)chain, step0 + w * kWave, m32, a.perm, (uint32_t)a.k);
        };
        uint32_t rows_a = window_rows(0), rows_b = window_rows(1);   // this window; the next (valid from position 62 on)
        TV zs_tab = (TV)0, cs_tab = (TV)0;     // per lane, label folded in: y*s_l (*log2 e), y*eta/s_{l+1}
        int parity = 0;
        Frag xr;                               // the row of the current step

        // descriptor of the row visited at in-window position jj (0 <= jj < 128), as four dwords:
        // base address, stride 0, bytes, dword-typed (reads past the end return 0)
        auto row_at = [&](int jj) {
            const uint32_t ra = (uint32_t)__builtin_amdgcn_readlane((int)rows_a, jj & (kWave - 1));
            const uint32_t rb = (uint32_t)__builtin_amdgcn_readlane((int)rows_b, jj & (kWave - 1));
            const uint32_t row = jj < kWave ? ra : rb;
            const uint64_t base = (uint64_t)(uintptr_t)(X + (int64_t)row * row_stride);
            u32x4 r;
            r[0] = (uint32_t)base;
            r[1] = (uint32_t)(base >> 32) & 0xffffu;
            r[2] = row_bytes;
            r[3] = 0x00020000u;
            return r;
        };
        // Chunk c of that row straight into this wave's LDS slot c: lane l's 16 bytes land at slot
        // base + 16*l.  Written as an instruction the compiler does not model, so that it neither
        // counts these loads in its own waits nor drains them in front of every LDS access; the
        // waits that matter are placed by hand below.
        typedef __attribute__((address_space(3))) uint32_t *lds_ptr;
        const uint32_t slot0 = (uint32_t)__builtin_amdgcn_readfirstlane(
            (int)((uint32_t)(size_t)(lds_ptr)&stage[0][0][0] + (uint32_t)wave * (CHUNKS * kWave * 16)));
        auto request_chunk = [&](int c, u32x4 rx) {
            // the chunk's offset in the row rides in a scalar, so one vector register serves all chunks
            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :
                         : "s"(slot0 + c * (kWave * 16)), "v"(off0), "s"(rx), "s"(c * kChunkStride)
                         : "memory", "m0");
        };
        auto take_chunk = [&](int c) {
            const u32x4 q = *reinterpret_cast<const u32x4 *>(&stage[wave][c][lane * 4]);
            xr.w[4 * c + 0] = q[0];
            xr.w[4 * c + 1] = q[1];
            xr.w[4 * c + 2] = q[2];
            xr.w[4 * c + 3] = q[3];
        };

        {   // row 0 into registers, row 1 on its way
            const u32x4 r0 = row_at(0), r1 = row_at(1);
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) request_chunk(c, r0);
            __builtin_amdgcn_s_waitcnt(0x0F70);                               // vmcnt(0)
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) take_chunk(c);
            __builtin_amdgcn_s_waitcnt(0xC07F);                               // lgkmcnt(0)
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) request_chunk(c, r1);
        }

        for (int64_t step = 0; step < n; ++step) {
            const int j = (int)(step & (kWave - 1));
            if (j == 0) {       // a new window of 64 steps
                if (step > 0) {
                    s_w *= rho64;
                    eos_w *= inv_rho64;
                    if (s_w < 0x1p-30) {
#pragma unroll
                        for (int e = 0; e < EPT; ++e) v[e] *= (TV)s_w;
                        s_w = 1.0;
                        eos_w = a.eta;
                    }
                    rows_a = rows_b;
                }
                double rho_pow, inv_rho_pow1;
                lane_powers(rho_pow, inv_rho_pow1);
                const double yl = (double)a.y[rows_a];
                const double sl = s_w * rho_pow * yl, el = eos_w * inv_rho_pow1 * yl;
                if constexpr (LOSS == kLossHinge) {
                    zs_tab = sl;
                    cs_tab = el;
                } else {
                    zs_tab = (float)(sl * 1.4426950408889634);
                    cs_tab = (float)el;
                }
            }

            TV acc[2] = {(TV)0, (TV)0};         // two partial sums: registers are scarce here
#pragma unroll
            for (int e = 0; e < EPT; ++e) acc[e & 1] += v[e] * (TV)xr.at(e);
            TV tot = wave_sum_lane63(acc[0] + acc[1]);
            if (lane == kWave - 1) red[parity][wave] = tot;
            const TV zy = lane_read(zs_tab, j), cy = lane_read(cs_tab, j);
            __syncthreads();
            tot = red[parity][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) tot += red[parity][w];
            parity ^= 1;
            TV c;
            if constexpr (LOSS == kLossHinge) {
                c = (zy * tot < 1.0) ? cy : 0.0;
            } else {
                c = cy * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(zy * tot));
            }
            // The widened elements of the dot product must not stay alive until the update (there
            // is no room for them beside v and the row): make the row words opaque here.
#pragma unroll
            for (int q = 0; q < Frag::kWords; ++q) asm volatile("" : "+v"(xr.w[q]));
            if (c != (TV)0) {    // uniform: every thread holds the same c
#pragma unroll
                for (int e = 0; e < EPT; ++e) v[e] += c * (TV)xr.at(e);
            }

            // row(step+1): LDS -> registers; row(step+2): HBM -> the slots just read
            if (j == kWave - 2 && step > 0) rows_b = window_rows(step / kWave + 1);    // the look-ahead enters the next window
            const u32x4 r2 = row_at(j + 2);
#pragma unroll
            for (int cidx = 0; cidx < CHUNKS; ++cidx) {
                __builtin_amdgcn_s_waitcnt(0x0F70 | (CHUNKS - 1));            // vmcnt(CHUNKS-1)
                take_chunk(cidx);
                __builtin_amdgcn_s_waitcnt(0xC07F);                           // lgkmcnt(0): slot read before it is refilled
                request_chunk(cidx, r2);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);     // nothing may still be landing in LDS when the wave ends

        const int64_t last_w = (n - 1) / kWave;
        const int rem = (int)(n - last_w * kWave);
        double rho_pow, inv_rho_pow1;
        lane_powers(rho_pow, inv_rho_pow1);
        const double s_end = s_w * lane_read(rho_pow, rem - 1) * rho;
#pragma unroll
        for (int e = 0; e < EPT; ++e) v[e] = (TV)(s_end * (double)v[e]);
    }

#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        if (col < a.d) out[col] = (float)v[e];
    }
}

}  // namespace wpsgd
