// Dense chains whose rows reach the computing waves through a ring of LDS slots that waves of
// their own fill.  Included by chain_dense_reg.hip, which instantiates and dispatches it.
#pragma once
#include "dense_rows.h"

namespace wpsgd {

// Rows fed through LDS by waves of their own.  A wave that issues vector memory loads pays for
// them in its own instruction stream (a 16 KiB row costs the four waves of a chain some 200 cycles
// per step that nothing hides), while other waves of the same SIMD are not slowed down by those
// loads at all.  So the workgroup is split: NT threads ("workers") hold the model vector and run
// the recursion exactly as in the register kernel, and as many threads again ("movers") do nothing
// but bring rows from HBM straight into a ring of LDS slots (loads that land in LDS need no
// registers while in flight).  A worker copies the rows of the next round from the ring into
// registers while the partial sums of the current round cross the workgroup.
//
// One barrier per round synchronises everything.  With rounds r = 0, 1, ... of B steps each and
// a ring of R rows, barrier r separates
//   workers: rows of round r read from the ring and consumed | rows of round r+1 read from the ring
//   movers : rows of round r+1 have landed (loads complete in issue order, so "at most
//            (R-2B) rows' worth outstanding" says so) | the slots of round r are refilled with
//            the rows of the steps R ahead.
template <typename TX, int LOSS, int NT, int EPT, int VEC, int B>
__global__ __launch_bounds__(2 * NT) void chain_dense_fed_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    using Frag = RowFrag<TX, NT, EPT, VEC>;
    static_assert(VEC * sizeof(TX) == 16, "16-byte loads only");
    constexpr int NW = NT / kWave;
    constexpr int NG = B * (B - 1) / 2;
    constexpr int NR = B + NG;
    constexpr int NACC = EPT >= 4 ? 4 : EPT;
    constexpr int CHUNKS = EPT / VEC;                       // 16-byte pieces of a row per worker = loads per mover wave and row
    constexpr int kSlotBytes = NT * EPT * (int)sizeof(TX);  // a row, padded to what the workers span
    constexpr int kRingMax = (144 * 1024) / kSlotBytes;
    constexpr int R = ((kRingMax > 16 ? 16 : kRingMax) / B) * B;    // rows in the ring: a whole number of rounds
    static_assert(R >= 4 * B, "the ring holds the round in use, the next two and one in flight");
    static_assert((R - 2 * B) * CHUNKS <= 63, "the mover's waits must be encodable");
    static_assert(kWave % (2 * B) == 0 && R < kWave, "windows hold whole pairs of rounds");
    __shared__ __attribute__((aligned(16))) uint32_t ring[R * kSlotBytes / 4];
    __shared__ TV red[2][NR][NW];
    __shared__ float ylab[NW][2][kWave];

    if ((int)blockIdx.x >= a.k) {       // a helper workgroup: see run_ahead_of_chain
        run_ahead_of_chain<TX>(a, reinterpret_cast<uint32_t *>(&ylab[0][0][0]));
        return;
    }
    const int tid = threadIdx.x;
    if (a.helpers > 0 && tid == 0) announce_chain_workgroup(a);
    const int lane = tid & (kWave - 1);
    const int wave_all = __builtin_amdgcn_readfirstlane(tid / kWave);
    const bool mover = wave_all >= NW;
    const int wave = mover ? wave_all - NW : wave_all;
    const int wtid = tid & (NT - 1);                        // index among the workers (or among the movers)
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const char *X = static_cast<const char *>(a.dense);
    const int64_t row_stride = a.ld * (int64_t)sizeof(TX);
    const uint32_t row_bytes = (uint32_t)(a.d * (int64_t)sizeof(TX));
    float *out = a.W + (int64_t)chain * a.d;
    const int64_t step0 = a.step0[blockIdx.x];

    // Columns past d are never loaded (the loads stop at the end of the row), so their ring bytes
    // keep the zeros written here and contribute nothing.
    for (int i = tid * 4; i < R * kSlotBytes / 4; i += 2 * NT * 4) {
        ring[i + 0] = 0u;
        ring[i + 1] = 0u;
        ring[i + 2] = 0u;
        ring[i + 3] = 0u;
    }
    __syncthreads();

    TV v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) v[e] = (TV)0;

    // rounds both kinds of wave run: whole pairs (the workers alternate between two register sets)
    const int64_t nblk = (n + B - 1) / B;
    const int64_t npairs = (nblk + 1) / 2;

    const uint32_t seed_lo = a.seed_lo, seed_hi = a.seed_hi, m32 = (uint32_t)a.m;
    uint32_t shard_lo = 0, shard_len = 1, shard_inc = 0, shard_pos = 0;
    if (a.perm) {
        shard_lo = a.shard[blockIdx.x];
        shard_len = a.shard[a.k + blockIdx.x];
        const uint32_t pos0 = a.shard[2 * a.k + blockIdx.x], room = shard_len - pos0;
        shard_inc = (uint32_t)kWave % shard_len;
        shard_pos = (uint32_t)lane < room ? pos0 + (uint32_t)lane : ((uint32_t)lane - room) % shard_len;
    }
    // rows visited in window w, one step per lane; windows are asked for in order 0, 1, 2, ...
    auto window_rows = [&](int64_t w) {
        if (a.perm) {
            const uint32_t *p = a.perm + ((uint64_t)shard_lo + shard_pos);
            uint32_t r;
            asm volatile("global_load_dword %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(r) : "v"(p) : "memory");
            const uint32_t t = shard_pos + shard_inc;
            shard_pos = (t < shard_pos || t >= shard_len) ? t - shard_len : t;
            return r;
        }
        return sample_row(seed_lo, seed_hi, (uint32_t)chain, (uint64_t)(step0 + w * kWave + lane), m32);
    };
    typedef __attribute__((address_space(3))) uint32_t *lds_ptr;
    const uint32_t ring_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(size_t)(lds_ptr)&ring[0]);

    if (n > 0 && mover) {
        uint32_t rows_a = window_rows(0), rows_b = window_rows(1);
        // lane l: address of the row of step l + R of the window
        uint32_t req_lo = 0, req_hi = 0;
        auto tabulate_requests = [&]() {
            const int src = ((lane + R) & (kWave - 1)) * 4;
            const uint32_t ra = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)rows_a);
            const uint32_t rb = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)rows_b);
            const uint32_t row = lane + R < kWave ? ra : rb;
            const uint64_t base = (uint64_t)(uintptr_t)X + (uint64_t)row * (uint64_t)row_stride;
            req_lo = (uint32_t)base;
            req_hi = (uint32_t)(base >> 32) & 0xffffu;
        };
        const uint32_t voff = (uint32_t)(lane * 16);
        // this wave's share of the row at `base` (16 bits of stride field zero, reads past the end
        // dropped) into the ring slot at byte position `pos`
        auto fetch = [&](uint32_t lo, uint32_t hi, uint32_t pos) {
            u32x4 rx;
            rx[0] = lo;
            rx[1] = hi;
            rx[2] = row_bytes;
            rx[3] = 0x00020000u;
#pragma unroll
            for (int q = 0; q < CHUNKS; ++q) {
                const uint32_t piece = (uint32_t)((q * NW + wave) * (kWave * 16));
                // (the descriptor words may come straight from lane reads: leave the scalar
                // registers time to settle before a memory instruction reads them)
                asm volatile("s_nop 4\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                             :
                             : "s"(ring_base + pos + piece), "v"(voff), "s"(rx), "s"(piece)
                             : "memory", "m0");
            }
        };
        // the whole ring first: rows 0 .. R-1
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)rows_a, r);
            const uint64_t base = (uint64_t)(uintptr_t)X + (uint64_t)row * (uint64_t)row_stride;
            fetch((uint32_t)base, (uint32_t)(base >> 32) & 0xffffu, (uint32_t)(r * kSlotBytes));
        }
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"((R - 2 * B) * CHUNKS) : "memory");     // rounds 0 and 1 have landed
        __syncthreads();
        uint32_t pos = 0;                           // ring position of the round whose slots are refilled next
        int j = 0;                                  // its in-window position
        for (int64_t r = 0; r < 2 * npairs; ++r) {
            if (j == 0) {
                const int64_t w = (r * B) / kWave;
                if (w > 0) {
                    rows_a = rows_b;
                    rows_b = window_rows(w + 1);
                }
                tabulate_requests();
            }
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"((R - 3 * B) * CHUNKS) : "memory");  // round r+2 has landed
            __syncthreads();
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)req_lo, j + b);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)req_hi, j + b);
                fetch(lo, hi, pos + (uint32_t)(b * kSlotBytes));
            }
            pos += (uint32_t)(B * kSlotBytes);
            if (pos == (uint32_t)(R * kSlotBytes)) pos = 0;
            j = (j + B) & (kWave - 1);
        }
        asm volatile("s_waitcnt vmcnt(0)" : : : "memory");      // nothing may still be landing when the wave ends
        return;
    }
    if (mover) return;

#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + wtid) * VEC + (e % VEC);
        v[e] = (a.w_start && col < a.d) ? (TV)a.w_start[col] : (TV)0;
    }

    if (n > 0) {
        Frag x[2][B];
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
        uint32_t rows_b = 0;
        TV zs_tab = (TV)0, cs_tab = (TV)0;

        // labels of a window: one gather per wave that lands in LDS, asked for a window ahead
        typedef __attribute__((address_space(3))) float *lds_fptr;
        const uint32_t ylab_base = (uint32_t)(size_t)(lds_fptr)&ylab[0][0][0] + (uint32_t)wave * (2 * kWave * 4);
        auto request_labels = [&](int64_t w, uint32_t rows) {
            const float *py = a.y + rows;
            const uint32_t slot = (uint32_t)__builtin_amdgcn_readfirstlane((int)(ylab_base + (uint32_t)(w & 1) * (kWave * 4)));
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" : : "s"(slot), "v"(py) : "memory", "m0");
        };
        request_labels(0, window_rows(0));
        rows_b = window_rows(1);
        request_labels(1, rows_b);

        // rows of a round from the ring (byte position pos) into register set u
        const uint32_t my_off = (uint32_t)(wtid * 16);
        auto take = [&](int u, uint32_t pos) {
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int c = 0; c < CHUNKS; ++c) {
                    const u32x4 q = *reinterpret_cast<const u32x4 *>(
                        reinterpret_cast<const char *>(ring) + (pos + my_off) + (b * kSlotBytes + c * NT * 16));
                    x[u][b].w[4 * c + 0] = q[0];
                    x[u][b].w[4 * c + 1] = q[1];
                    x[u][b].w[4 * c + 2] = q[2];
                    x[u][b].w[4 * c + 3] = q[3];
                }
        };

        int parity = 0;
        uint32_t pos_next = (uint32_t)(B * kSlotBytes);     // ring position of the round after the current one
        auto round = [&](int u, int j) {
            TV acc[NR][NACC];
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int q = 0; q < NACC; ++q) acc[r][q] = (TV)0;
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
                for (int q = 1; q < NACC; ++q) t += acc[r][q];
                tot[r] = t;
            }
            if constexpr (NR == 3 && sizeof(TV) == 4) {
                wave_sum3_lane63(tot[0], tot[1], tot[2]);
            } else {
#pragma unroll
                for (int r = 0; r < NR; ++r) tot[r] = wave_sum_lane63(tot[r]);
            }
            if (lane == kWave - 1) {
#pragma unroll
                for (int r = 0; r < NR; ++r) red[parity][r][wave] = tot[r];
            }
            // The rows of the next round move from the ring to registers while this wave waits at
            // the barrier: a wave cannot issue while data returns into its registers, and here it
            // has nothing to issue anyway.  LDS operations of a wave complete in order, so once
            // at most the B*CHUNKS reads are outstanding the partial sums above are in LDS.
            asm volatile("" : : : "memory");
            take(u ^ 1, pos_next);
            pos_next += (uint32_t)(B * kSlotBytes);
            if (pos_next == (uint32_t)(R * kSlotBytes)) pos_next = 0;
            TV zy[B], cy[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                zy[b] = lane_read(zs_tab, j + b);
                cy[b] = lane_read(cs_tab, j + b);
            }
            asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(B * CHUNKS) : "memory");
            __builtin_amdgcn_s_barrier();
            TV part[NR][NW];
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int w = 0; w < NW; ++w) part[r][w] = red[parity][r][w];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                TV t = part[r][0];
#pragma unroll
                for (int w = 1; w < NW; ++w) t += part[r][w];
                tot[r] = t;
            }
            parity ^= 1;
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
                if constexpr (LOSS == kLossHinge) {
                    c[b] = (zy[b] * dot < 1.0) ? cy[b] : 0.0;
                } else {
                    c[b] = cy[b] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(zy[b] * dot));
                }
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
#pragma unroll
                for (int b = 0; b < B; ++b) v[e] += c[b] * (TV)x[u][b].at(e);
            }
        };

        __syncthreads();            // round 0 has landed in the ring
        take(0, 0u);

        int j0 = 0;
        for (int64_t g = 0; g < npairs; ++g) {
            if (a.helpers > 0 && tid == 0 && (j0 & 7) == 0) a.progress[blockIdx.x] = (uint32_t)(g * 2 * B);   // for the helpers to see
            if (j0 == 0) {      // a new window of 64 steps begins
                const int64_t w = (g * 2 * B) / kWave;
                if (w > 0) {
                    s_w *= rho64;
                    eos_w *= inv_rho64;
                    if (s_w < 0x1p-30) {
#pragma unroll
                        for (int e = 0; e < EPT; ++e) v[e] *= (TV)s_w;
                        s_w = 1.0;
                        eos_w = a.eta;
                    }
                    rows_b = window_rows(w + 1);
                }
                // the labels of this window were asked for a window ago; the workers issue no
                // other vector memory operation, so the queue is simply drained here
                __builtin_amdgcn_s_waitcnt(0x0F70);
                if (w > 0) request_labels(w + 1, rows_b);
                const double yl = (double)ylab[wave][w & 1][lane];
                const double sl = s_w * rho_pow * yl, el = eos_w * inv_rho_pow1 * yl;
                const bool live = w * kWave + lane < n;
                if constexpr (LOSS == kLossHinge) {
                    zs_tab = sl;
                    cs_tab = live ? el : 0.0;
                } else {
                    zs_tab = (float)(sl * 1.4426950408889634);
                    cs_tab = live ? (float)el : 0.0f;
                }
            }
            round(0, j0);
            round(1, j0 + B);
            j0 = (j0 + 2 * B) & (kWave - 1);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        if (a.helpers > 0 && tid == 0) a.progress[blockIdx.x] = kChainDone;
        const int64_t last_w = (n - 1) / kWave;
        const int rem = (int)(n - last_w * kWave);
        const double s_end = s_w * lane_read(rho_pow, rem - 1) * rho;
#pragma unroll
        for (int e = 0; e < EPT; ++e) v[e] = (TV)(s_end * (double)v[e]);
    }

#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = ((int64_t)(e / VEC) * NT + wtid) * VEC + (e % VEC);
        if (col < a.d) out[col] = (float)v[e];
    }
}

}  // namespace wpsgd
