// Dense-row SGD chains with the model vector held in registers.
//
// One workgroup runs one chain (Algorithm 1, the inner loop of node i): NT threads own EPT model
// elements each, so the vector never leaves the register file between the first and the last
// step.  The step  w <- (1-eta*lambda) w - eta*g*x  (Eq. 5 with Eq. 4) is carried as w = s*v:
// the shrink only touches a scalar, the gradient part touches v.
//
// Because the rows a chain visits depend on (seed, chain, step) only, never on w, rows are
// requested P-1 rounds before they are consumed and wait in registers.  A round folds B steps
// into one workgroup-wide reduction: with the rows x_0..x_{B-1} of the round and the vector v at
// its start, the threads reduce p_b = v.x_b and G_ab = x_a.x_b (a<b) together; the B dependent
// steps are then a scalar recursion
//     v_b.x_b = p_b + sum_{a<b} c_a G_ab,   yhat_b = s_b * (v_b.x_b),   c_b = -eta*g_b / s_{b+1}
// and the round ends with the rank-B update v += sum_b c_b x_b.  This is the same arithmetic as
// B single steps up to summation order; B = 1 is the plain step.
//
// What does not depend on w is prepared once per window of 64 steps, one step per lane: the
// visited rows (Philox) and the two per-step scalars of the recursion, s_l and eta/s_{l+1} with
// s_l = s_window * (1-eta*lambda)^l in fp64.  Inside a window a step fetches them with a lane
// read, so its dependent path holds no integer hashing and no fp64 scale arithmetic.  Steps
// past the end of the chain have eta/s = 0 in their lane and therefore change nothing: the loop
// always runs whole groups of P rounds and needs no tail code.
//
// Rows are fetched with raw buffer loads: the row's address sits in a scalar descriptor, each
// lane adds a fixed 32-bit offset, and lanes past the end of the row read zeros.
//
// Two things reach beyond the one workgroup (both in dense_rows.h): helper workgroups that run
// ahead of a chain and pull its rows into L2, and column slices - a chain whose rows are too long
// for one workgroup runs as several, each with NT*EPT columns, that add their sums once per round.
//
// This file is compiled once per (row storage, loss) pair; WPSGD_TX_BF16 and WPSGD_LOSS select it.
#include <atomic>

#include "dense_rows.h"
#include "chain_dense_wide.h"

namespace wpsgd {

#if WPSGD_TX_BF16
using RowElem = uint16_t;
#else
using RowElem = float;
#endif
constexpr int kLoss = WPSGD_LOSS;


// TX and LOSS are template parameters (not just per-file constants) so that the four builds of
// this file produce four distinct sets of kernel symbols.
// SLICED: the launch cuts every chain into a.slices column slices (a kernel of its own, so that the
// one-workgroup chain carries none of the slices' exchange, not even as a branch not taken: the
// mere presence of that branch between the barrier and the row requests cost 15 % at d = 4096).
template <typename TX, int LOSS, int NT, int EPT, int VEC, int B, int P, bool SLICED>
__global__ __launch_bounds__(NT) void chain_dense_reg_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;     // state, dot products and the step recursion
    using Frag = RowFrag<TX, NT, EPT, VEC>;
    constexpr int NW = NT / kWave;
    constexpr int NG = B * (B - 1) / 2;
    constexpr int NR = B + NG;
    // independent partial sums per dot product: enough chains of dependent FMAs in flight to hide their
    // latency.  A round of two or more steps forms three or more sums side by side, which are chains
    // enough: one accumulator each (nine additions fewer per round than with four: 4.5 % of a round at
    // d = 4096, where two accumulators gave 2.5 %; sliced chains of 128 KiB rows showed no difference
    // and keep four).
    constexpr int NACC = EPT < 4 ? EPT : (NR >= 3 && !SLICED ? 1 : 4);
    constexpr int D = B * P;                       // steps per group of P rounds
    static_assert(kWave % D == 0, "a 64-step window must hold whole groups");
    __shared__ TV red[2][NR][NW];
    // Labels of a whole window, gathered straight into LDS one window ahead (per wave, two windows)
    __shared__ float ylab[NW][2][kWave];
    // Sliced chains: the workgroup's verdict at the end of the chain (did a wave give up waiting for
    // the other slices?), reached by one vote behind the loop.
    __shared__ uint32_t gave_up_word;
    typedef __attribute__((address_space(3))) volatile uint32_t *lds_flag_ptr;      // (LDS-typed: no flat accesses)
    const lds_flag_ptr gave_up = (lds_flag_ptr)&gave_up_word;
    if constexpr (SLICED) {
        if (threadIdx.x == 0) *gave_up = 0u;
        __syncthreads();
    }

    if constexpr (!SLICED) {
        if ((int)blockIdx.x >= a.k) {              // a helper workgroup: see run_ahead_of_chain
            run_ahead_of_chain<TX>(a, reinterpret_cast<uint32_t *>(&ylab[0][0][0]));
            return;
        }
    }
    const int tid = threadIdx.x;
    if constexpr (!SLICED) {
        if (a.helpers > 0 && tid == 0) announce_chain_workgroup(a);
    }
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    // Workgroup cb + s*k runs column slice s of the chain of workgroup cb: columns
    // [s*NT*EPT, (s+1)*NT*EPT) of the model vector and of every row.  One slice is the whole chain.
    const int cb = SLICED ? (int)(blockIdx.x % (unsigned)a.k) : (int)blockIdx.x;
    const int slice = SLICED ? (int)(blockIdx.x / (unsigned)a.k) : 0;
    const int64_t col0 = (int64_t)slice * (NT * EPT);
    const int chain = a.order[cb];
    const int64_t n = a.nsteps[cb];
    const char *X = static_cast<const char *>(a.dense);
    const int64_t row_stride = a.ld * (int64_t)sizeof(TX);
    const uint32_t row_bytes = (uint32_t)(a.d * (int64_t)sizeof(TX));
    float *out = a.W + (int64_t)chain * a.d;
    bool lost = false;                  // set when the other slices of the chain did not show up

    TV v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = col0 + ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        v[e] = (a.w_start && col < a.d) ? (TV)a.w_start[col] : (TV)0;
    }
    const int64_t step0 = a.step0[cb];

    if (n > 0) {
        uint32_t off[Frag::kChunks];               // this lane's byte offset of each chunk
#pragma unroll
        for (int c = 0; c < Frag::kChunks; ++c)
            off[c] = (uint32_t)((col0 + (c * NT + tid) * VEC) * (int64_t)sizeof(TX));
        Frag x[P][B];

        // (1-eta*lambda)^lane and (1-eta*lambda)^-(lane+1), by binary powering in fp64
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
        double s_w = 1.0, eos_w = a.eta;     // scale and eta/scale at the start of the window

        const uint32_t seed_lo = a.seed_lo, seed_hi = a.seed_hi, m32 = (uint32_t)a.m;
        // Partition-and-shuffle sampling reads the tabulated shuffled order; the lane's position in
        // its chain's share advances by 64 (mod the share size) from window to window, so no
        // division sits in the loop.  Windows are asked for in order: 0, 1, 2, ...
        uint32_t shard_lo = 0, shard_len = 1, shard_inc = 0, shard_pos = 0;
        if (a.perm) {
            shard_lo = a.shard[cb];
            shard_len = a.shard[a.k + cb];
            const uint32_t pos0 = a.shard[2 * a.k + cb], room = shard_len - pos0;
            shard_inc = (uint32_t)kWave % shard_len;
            shard_pos = (uint32_t)lane < room ? pos0 + (uint32_t)lane : ((uint32_t)lane - room) % shard_len;
        }
        auto window_rows = [&](int64_t w) {
            if (a.perm) {
                const uint32_t *p = a.perm + ((uint64_t)shard_lo + shard_pos);
                uint32_t r;   // a load the compiler does not count: nothing outside this branch may wait for it
                asm volatile("global_load_dword %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(r) : "v"(p) : "memory");
                const uint32_t t = shard_pos + shard_inc;                 // may wrap past 2^32: then it is past the share too
                shard_pos = (t < shard_pos || t >= shard_len) ? t - shard_len : t;
                return r;
            }
            return sample_row(seed_lo, seed_hi, (uint32_t)chain, (uint64_t)(step0 + w * kWave + lane), m32);
        };
        uint32_t rows_a = window_rows(0), rows_b = window_rows(1);   // this window and the next
        TV zs_tab = (TV)0, cs_tab = (TV)0;   // per lane: s_l (times log2(e) for logistic), eta/s_{l+1}

        // Descriptors of the B rows of the round at in-window position j (0 <= j < 128; positions
        // >= 64 lie in the next window), straight from the row numbers: used before the loop only.
        auto describe = [&](int j, __amdgpu_buffer_rsrc_t (&rx)[B]) {
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int jj = j + b;
                const uint32_t ra = (uint32_t)__builtin_amdgcn_readlane((int)rows_a, jj & (kWave - 1));
                const uint32_t rb = (uint32_t)__builtin_amdgcn_readlane((int)rows_b, jj & (kWave - 1));
                const uint32_t row = jj < kWave ? ra : rb;
                rx[b] = make_rsrc(X + (int64_t)row * row_stride, row_bytes);
            }
        };
        // Inside the loop a round requests the rows of the round kAhead steps later.  Their
        // addresses are tabulated once per window, one step per lane: lane l holds the address of
        // the row of step l + kAhead of the window (the upper lanes reach into the next window), so
        // that a request costs two lane reads instead of a 64-bit multiply-add on the scalar unit.
        constexpr int kAhead = (P == 1 ? 1 : P - 1) * B;
        static_assert(kAhead < kWave, "the look-ahead stays within one window");
        uint32_t req_lo = 0, req_hi = 0;
        auto tabulate_requests = [&]() {
            const int src = ((lane + kAhead) & (kWave - 1)) * 4;
            const uint32_t ra = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)rows_a);
            const uint32_t rb = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)rows_b);
            const uint32_t row = lane + kAhead < kWave ? ra : rb;
            const uint64_t base = (uint64_t)(uintptr_t)X + (uint64_t)row * (uint64_t)row_stride;
            req_lo = (uint32_t)base;
            req_hi = (uint32_t)(base >> 32);
        };
        // descriptors of the rows to request while the round at position j (0 <= j < 64) runs
        auto describe_ahead = [&](int j, __amdgpu_buffer_rsrc_t (&rx)[B]) {
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const uint64_t lo = (uint32_t)__builtin_amdgcn_readlane((int)req_lo, j + b);
                const uint64_t hi = (uint32_t)__builtin_amdgcn_readlane((int)req_hi, j + b);
                rx[b] = make_rsrc(reinterpret_cast<const void *>((hi << 32) | lo), row_bytes);
            }
        };
        // requests rows b_lo .. b_hi-1 of a round into slot u
        auto issue_rows = [&](int u, const __amdgpu_buffer_rsrc_t (&rx)[B], int b_lo, int b_hi) {
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int c = 0; c < Frag::kChunks; ++c)
                    if (b >= b_lo && b < b_hi) x[u][b].load_chunk(c, rx[b], off[c]);
        };
        auto issue = [&](int u, const __amdgpu_buffer_rsrc_t (&rx)[B]) { issue_rows(u, rx, 0, B); };
        // A round's requests are issued in two halves, the first while the workgroup's sums travel
        // back, the second after the update: the four waves' requests for one row keep the CU's
        // address path busy for 256 cycles, and a wave that wants to issue behind a longer queue
        // than that stands still (two rows at once cost 17 % at d = 4096).
        constexpr int kFirstHalf = (B + 1) / 2;
        auto request = [&](int u, int j) {
            __amdgpu_buffer_rsrc_t rx[B];
            describe(j, rx);
            issue(u, rx);
        };
        // Labels: the 64 labels of a window are gathered with one load per wave that lands in LDS
        // (each lane's dword at slot + 4*lane), a whole window before they are read.  The compiler
        // does not see that load, and nothing waits for it: memory operations of a wave complete
        // in order and at most 63 can be outstanding, so after the hundreds of row loads of one
        // window it has landed.  (A scalar load would be drained at every LDS wait, a per-step
        // vector load costs a descriptor and an instruction per step.)
        typedef __attribute__((address_space(3))) float *lds_fptr;
        const uint32_t ylab_base = (uint32_t)(size_t)(lds_fptr)&ylab[0][0][0] + (uint32_t)wave * (2 * kWave * 4);
        auto request_labels = [&](int64_t w, uint32_t rows) {
            const float *py = a.y + rows;
            const uint32_t slot = (uint32_t)__builtin_amdgcn_readfirstlane((int)(ylab_base + (uint32_t)(w & 1) * (kWave * 4)));
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" : : "s"(slot), "v"(py) : "memory", "m0");
        };
        request_labels(0, rows_a);
        request_labels(1, rows_b);

        uint32_t round_no = 0;              // rounds done, as the slices of a chain count them
        // who publishes a slice's sums; nobody when slices are told not to wait at all (then no record
        // ever shows up and every wave of every slice gives up at its first exchange)
        const bool publisher = tid == 0 && a.slice_max_polls != 0;
        uint32_t max_polls = a.slice_max_polls;        // how long an exchange may wait for the other slices
        bool near_slices = false;
        if constexpr (SLICED) near_slices = slices_share_an_xcd(a, cb, slice, tid == 0);
        int parity = 0;
        // One round: steps at in-window positions j .. j+B-1, rows in slot u.  While the partial
        // sums cross the workgroup, slot u_prev (consumed one round ago) is requested again for
        // the round kAhead steps from here.
        auto round = [&](int u, int j, int u_prev) {
            if constexpr (P >= 3 && !SLICED && NW > 1) {
                // One wait for all chunks of this round's rows, which were requested P-1 rounds ago, instead
                // of one in front of each chunk's first use (four instructions fewer per round: -1 %).  The
                // loads issued since then may stay in flight.  (gfx9 encoding: vmcnt split over bits 3:0 and
                // 15:14, expcnt and lgkmcnt left open.)
                constexpr int kLater = (P - 2) * B * Frag::kChunks;
                static_assert(kLater < 64, "the counter holds 63");
                __builtin_amdgcn_s_waitcnt(((kLater & 0xF) | ((kLater >> 4) << 14)) | 0x0F70);
                __builtin_amdgcn_sched_barrier(0);          // nothing that reads the rows moves in front of it
            }
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
            if constexpr (NW > 1) {
                if (lane == kWave - 1) {
#pragma unroll
                    for (int r = 0; r < NR; ++r) red[parity][r][wave] = tot[r];
                }
            }
            // The next rows are described (scalar arithmetic) while the partial sums travel to LDS
            // and requested while the workgroup's sums travel back: both waits hide something.
            __amdgpu_buffer_rsrc_t next_rows[B];
            if constexpr (P > 1) describe_ahead(j, next_rows);
            // per-step scalars with the label folded in, ready before the sums arrive
            TV zy[B], cy[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                zy[b] = lane_read(zs_tab, j + b);
                cy[b] = lane_read(cs_tab, j + b);
            }
            if constexpr (NW > 1) {
                __syncthreads();
                TV part[NR][NW];
#pragma unroll
                for (int r = 0; r < NR; ++r)
#pragma unroll
                    for (int w = 0; w < NW; ++w) part[r][w] = red[parity][r][w];
                // (A sliced chain requests its rows after the slices' exchange instead: loads return
                // in order, so the exchange's polls would wait behind rows just requested from HBM.)
                if constexpr (P > 1 && !SLICED) issue_rows(u_prev, next_rows, 0, kFirstHalf);
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    TV t = part[r][0];
#pragma unroll
                    for (int w = 1; w < NW; ++w) t += part[r][w];
                    tot[r] = t;
                }
                parity ^= 1;
            } else {
                if constexpr (P > 1) issue_rows(u_prev, next_rows, 0, kFirstHalf);
                // One wave: the sums sit in lane 63.  The hinge only needs one bit of them, which
                // is read off the comparison below; the logistic slope needs the value in every lane.
                if constexpr (LOSS != kLossHinge) {
#pragma unroll
                    for (int r = 0; r < NR; ++r) tot[r] = read_lane63(tot[r]);
                }
            }
            // several slices: add up the slices' sums (every wave of every slice ends with the same totals)
            static_assert(!SLICED || (NW > 1 && NR * sizeof(TV) <= kSliceMaxWords * 4), "the slices' exchange carries twelve words");
            if constexpr (SLICED) {
                uint32_t w[kSliceMaxWords];
#pragma unroll
                for (int q = 0; q < kSliceMaxWords; ++q) w[q] = 0u;
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    if constexpr (sizeof(TV) == 8) {
                        const uint64_t bits = (uint64_t)__double_as_longlong((double)tot[r]);
                        w[2 * r] = (uint32_t)bits;
                        w[2 * r + 1] = (uint32_t)(bits >> 32);
                    } else {
                        w[r] = __float_as_uint((float)tot[r]);
                    }
                }
                const bool met = near_slices ? slices_all_reduce<sizeof(TV) == 8, NR, true>(a, cb, slice, publisher, round_no, max_polls, w)
                                             : slices_all_reduce<sizeof(TV) == 8, NR, false>(a, cb, slice, publisher, round_no, max_polls, w);
                if (__builtin_expect(!met, 0)) {
                    // The wait for the other slices ran out.  The wave tells the host, waits no more in the
                    // rounds left of its group, and leaves the chain at the group's end (see there).
                    lost = true;
                    max_polls = 0;
#pragma unroll
                    for (int q = 0; q < kSliceMaxWords; ++q) w[q] = 0x7ff80000u;      // NaN as a float, and as either half of a double
                    if (lane == kWave - 1) __hip_atomic_fetch_or(a.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if constexpr (P > 1) issue_rows(u_prev, next_rows, 0, kFirstHalf);
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    if constexpr (sizeof(TV) == 8) {
                        tot[r] = (TV)__longlong_as_double((long long)(((uint64_t)w[2 * r + 1] << 32) | w[2 * r]));
                    } else {
                        tot[r] = (TV)__uint_as_float(w[r]);
                    }
                }
                ++round_no;
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
                if constexpr (LOSS == kLossHinge) {
                    // -eta*g/s_next, g = -y or 0
                    if constexpr (SLICED) {
                        // (dot - dot is 0 for every number and NaN for NaN: a chain whose slices lost each
                        // other must not turn NaN sums into steps not taken)
                        c[b] = (zy[b] * dot < 1.0) ? cy[b] : dot - dot;
                    } else if constexpr (NW > 1) {
                        c[b] = (zy[b] * dot < 1.0) ? cy[b] : 0.0;
                    } else {
                        c[b] = lane63_below_one(zy[b], dot) ? cy[b] : 0.0;
                    }
                } else {
                    // -eta*g/s_next with g = -y/(1+exp(y*yhat)); exp as 2^(log2(e)*y*s*dot)
                    c[b] = cy[b] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(zy[b] * dot));
                }
            }
            if constexpr (SLICED && P > 1 && B == 2) {
                // A slice's next poll waits for these requests (loads return in order): they go out
                // between the two halves of the update rather than behind it (fp64 state on 128 KiB
                // rows: -4 %; fp32 state: no difference).  Per element the additions keep their order.
#pragma unroll
                for (int e = 0; e < EPT; ++e) v[e] += c[0] * (TV)x[u][0].at(e);
                __builtin_amdgcn_sched_barrier(0);
                issue_rows(u_prev, next_rows, kFirstHalf, B);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < EPT; ++e) v[e] += c[1] * (TV)x[u][1].at(e);
            } else {
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
#pragma unroll
                    for (int b = 0; b < B; ++b) v[e] += c[b] * (TV)x[u][b].at(e);
                }
                if constexpr (P > 1 && kFirstHalf < B) {
                    __builtin_amdgcn_sched_barrier(0);        // keep these requests behind the update
                    issue_rows(u_prev, next_rows, kFirstHalf, B);
                }
            }
            if constexpr (P == 1) {                       // a single slot: refill once it is free
                __amdgpu_buffer_rsrc_t rx[B];
                describe_ahead(j, rx);
                issue(u, rx);
            }
        };

        // Slots 0..P-2 hold rounds 0..P-2 on entry to the loop; round r refills the slot of
        // round r-1 with round r+P-1.
#pragma unroll
        for (int u = 0; u + 1 < P; ++u) request(u, u * B);
        if constexpr (P == 1) request(0, 0);
        // Let the first rows land before the loop starts.  With loads pending on entry, the wait
        // in front of the loop's first use must cover the entry path too and is placed as a full
        // drain that every iteration then pays; entering with an empty queue leaves only the
        // partial waits of the steady state.  (gfx9 encoding: vmcnt = 0, expcnt and lgkmcnt open.)
        __builtin_amdgcn_s_waitcnt(0x0F70);

        const int64_t nblk = (n + B - 1) / B;
        const int64_t ngroups = (nblk + P - 1) / P;
        int j0 = 0;                                 // in-window position of the group's first step
        for (int64_t g = 0; g < ngroups; ++g) {
            if constexpr (!SLICED) {
                if (a.helpers > 0 && tid == 0) a.progress[cb] = (uint32_t)(g * D);   // for the helpers to see
            }
            if (j0 == 0) {      // a new window of 64 steps begins (never in the middle of a group)
                const int64_t w = (g * D) / kWave;
                if (w > 0) {
                    s_w *= rho64;
                    eos_w *= inv_rho64;
                    if (s_w < 0x1p-30) {    // fold the scale into v long before eta/s leaves fp32 range
#pragma unroll
                        for (int e = 0; e < EPT; ++e) v[e] *= (TV)s_w;
                        s_w = 1.0;
                        eos_w = a.eta;
                    }
                    rows_a = rows_b;
                    rows_b = window_rows(w + 1);
                    request_labels(w + 1, rows_b);
                }
                tabulate_requests();
                const double yl = (double)ylab[wave][w & 1][lane];      // requested a window ago (or before the loop)
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
#pragma unroll
            for (int u = 0; u < P; ++u)
                round(u, j0 + u * B, (u + P - 1) % P);
            j0 = (j0 + D) & (kWave - 1);
            if (lost) break;                        // (uniform within a wave)
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);      // no label load may still be on its way to LDS when the wave ends
        if constexpr (!SLICED) {
            if (a.helpers > 0 && tid == 0) a.progress[cb] = kChainDone;
        }
        if constexpr (SLICED) {
            // A wave that gave up turns its partial sums into NaN for good before it goes (nobody else
            // writes those words): from the next round on every sum of this slice is NaN, so is the
            // record it publishes, and so are the totals, the steps and the model of every slice of
            // the chain.  The failure travels with the data; a round that goes well carries no check
            // for it.  Then one verdict for the workgroup: if any of its waves gave up, all of its
            // columns are NaN, also when that happened in the chain's last rounds.  (A wave that left
            // the loop early may meet the others at this barrier while they are still at a round's.)
            if (lost && lane == kWave - 1) {
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    red[0][r][wave] = (TV)__builtin_nanf("");
                    red[1][r][wave] = (TV)__builtin_nanf("");
                }
                *gave_up = 1u;
            }
            __syncthreads();
            if (*gave_up != 0u) lost = true;
        }
        // scale at the chain's end: s_w covers the steps before the last window
        const int64_t last_w = (n - 1) / kWave;
        const int rem = (int)(n - last_w * kWave);                          // 1..64 steps in it
        const double s_end = s_w * lane_read(rho_pow, rem - 1) * rho;
#pragma unroll
        for (int e = 0; e < EPT; ++e) v[e] = (TV)(s_end * (double)v[e]);
    }

#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int64_t col = col0 + ((int64_t)(e / VEC) * NT + tid) * VEC + (e % VEC);
        if (col < a.d) out[col] = lost ? __builtin_nanf("") : (float)v[e];
    }
}

// ---------------------------------------------------------------------------------------------
// Instantiated variants: V(threads, elements per thread, load width, B, P).  Within one
// (threads, ept, vec) shape the first entry is the default; the others are reachable through a
// forced plan.  Register budget per thread: 512 at 256 threads, 256 at 512, 128 at 1024.
// P > 0: rows wait in registers, P rounds requested ahead.  P = -1: the next row is staged in LDS.
// P = 0: rows are streamed twice.
// ---------------------------------------------------------------------------------------------
// 64 elements per thread only with fp32 state (logistic): 64 fp64 values would fill the registers
#if WPSGD_LOSS == 1
#define WPSGD_WIDEST(V, VEC) V(1024, 64, VEC, 1, 0)
#define WPSGD_WIDEST_LDS(V, VEC) V(1024, 64, VEC, 1, -1)
#else
#define WPSGD_WIDEST(V, VEC)
#define WPSGD_WIDEST_LDS(V, VEC)
#endif

#define WPSGD_VARIANTS_ANY(V)                                                                  \
    V(64, 1, 1, 1, 8) V(64, 2, 1, 1, 8) V(64, 4, 1, 1, 8)                                      \
    V(64, 1, 1, 4, 2) V(64, 4, 1, 2, 4)                                                        \
    V(256, 4, 1, 1, 4) V(256, 8, 1, 1, 4) V(256, 16, 1, 1, 4) V(256, 32, 1, 1, 2)              \
    V(256, 4, 1, 4, 2) V(256, 16, 1, 4, 2)                                                     \
    V(1024, 16, 1, 1, 0) V(1024, 32, 1, 1, 0) WPSGD_WIDEST(V, 1)

#if WPSGD_TX_BF16
#define WPSGD_VARIANTS_VEC(V)                                                                  \
    V(64, 8, 8, 1, 8) V(64, 8, 8, 4, 2)                                                        \
    V(256, 8, 8, 1, 8) V(256, 16, 8, 1, 8) V(256, 32, 8, 1, 4) V(256, 32, 8, 4, 2)             \
    V(256, 8, 8, 4, 2) V(256, 16, 8, 4, 2)                                                     \
    V(256, 8, 8, 2, 4) V(256, 16, 8, 2, 4) V(256, 32, 8, 2, 4) V(256, 64, 8, 2, 2) V(256, 64, 8, 1, 4) \
    V(256, 64, 8, 4, 2)                                                                        \
    V(1024, 16, 8, 1, -1) V(1024, 32, 8, 1, -1) WPSGD_WIDEST_LDS(V, 8)                          \
    V(1024, 16, 8, 1, 0) V(1024, 32, 8, 1, 0) WPSGD_WIDEST(V, 8)
#define WPSGD_VARIANTS_WIDE(V)
#else
#define WPSGD_VARIANTS_VEC(V)                                                                  \
    V(64, 4, 4, 1, 8) V(64, 4, 4, 1, 16) V(64, 4, 4, 2, 4) V(64, 4, 4, 4, 2)                   \
    V(256, 4, 4, 1, 8) V(256, 8, 4, 1, 8) V(256, 16, 4, 1, 8) V(256, 32, 4, 1, 4) V(256, 16, 4, 1, 16) V(256, 8, 4, 1, 16)             \
    V(256, 4, 4, 4, 2) V(256, 8, 4, 4, 2) V(256, 16, 4, 4, 2) V(256, 16, 4, 1, 4)              \
    V(256, 16, 4, 2, 2) V(256, 16, 4, 2, 4) V(256, 16, 4, 2, 8) V(256, 32, 4, 4, 2)            \
    V(256, 4, 4, 2, 4) V(256, 8, 4, 2, 4) V(256, 32, 4, 2, 2)                                  \
    V(512, 8, 4, 1, 8) V(512, 8, 4, 4, 2) V(512, 8, 4, 2, 4)                                   \
    V(1024, 4, 4, 1, 8) V(1024, 4, 4, 4, 2) V(1024, 4, 4, 2, 4)                                \
    V(1024, 16, 4, 1, -1) V(1024, 32, 4, 1, -1)                                                \
    V(1024, 16, 4, 1, 0) V(1024, 32, 4, 1, 0) WPSGD_WIDEST(V, 4)
#define WPSGD_VARIANTS_WIDE(V)
#endif

#define WPSGD_ALL_VARIANTS(V) WPSGD_VARIANTS_VEC(V) WPSGD_VARIANTS_ANY(V) WPSGD_VARIANTS_WIDE(V)

// Which variants also exist as a kernel for column slices: four waves, vector loads, rows in
// registers, and sums that fit the slices' records (twelve 32-bit words).
constexpr bool can_slice(int nt, int vec, int bb, int pp)
{
    return nt == 256 && vec > 1 && pp > 0 &&
           (bb + bb * (bb - 1) / 2) * sizeof(typename StateType<kLoss>::type) <= (size_t)kSliceMaxWords * 4;
}

template <int NT, int EPT, int VEC, int BB, int PP>
static void launch_variant(const ChainArgs &a, hipStream_t s)
{
    if constexpr (PP < 0) {
        hipLaunchKernelGGL((chain_dense_lds_kernel<RowElem, kLoss, NT, EPT, VEC>), dim3(a.k), dim3(NT), 0, s, a);
    } else if constexpr (PP == 0) {
        hipLaunchKernelGGL((chain_dense_wide_kernel<RowElem, kLoss, NT, EPT, VEC>), dim3(a.k), dim3(NT), 0, s, a);
    } else {
        if (a.slices > 1) {
            if constexpr (can_slice(NT, VEC, BB, PP)) {       // (the dispatch offers no other variant to a sliced plan)
                hipLaunchKernelGGL((chain_dense_reg_kernel<RowElem, kLoss, NT, EPT, VEC, BB, PP, true>), dim3(a.k * a.slices), dim3(NT), 0, s, a);
            }
            return;
        }
        auto kernel = chain_dense_reg_kernel<RowElem, kLoss, NT, EPT, VEC, BB, PP, false>;
        size_t claim = 0;
        if (a.helpers > 0) {
            // more than half of a compute unit's LDS per workgroup: chains and helpers each get a unit of their own
            static std::atomic<int> allowed{0};         // 0 not asked yet, 1 granted, -1 refused (asking twice is harmless)
            int may = allowed.load(std::memory_order_relaxed);
            if (may == 0) {
                may = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 84 * 1024) == hipSuccess ? 1 : -1;
                if (may < 0) (void)hipGetLastError();
                allowed.store(may, std::memory_order_relaxed);
            }
            if (may > 0) claim = 84 * 1024;
        }
        ChainArgs b = a;
        if (claim == 0) b.helpers = 0;
        hipLaunchKernelGGL(kernel, dim3(b.k + b.helpers), dim3(NT), claim, s, b);
    }
}

#define WPSGD_CAT2(a, b) a##b
#define WPSGD_CAT(a, b) WPSGD_CAT2(a, b)
#if WPSGD_TX_BF16
#define WPSGD_SUFFIX WPSGD_CAT(bf16_loss, WPSGD_LOSS)
#else
#define WPSGD_SUFFIX WPSGD_CAT(f32_loss, WPSGD_LOSS)
#endif

constexpr int rows_kind(int pp) { return pp > 0 ? 1 : (pp == -1 ? 2 : 3); }

// find(plan, launch?): walks the table; exact match on (threads, ept, vec, B, P, rows) where the
// plan gives them, else the first entry of the shape.
hipError_t WPSGD_CAT(dense_reg_dispatch_, WPSGD_SUFFIX)(Plan &p, const ChainArgs *a, hipStream_t s)
{
#define WPSGD_TRY(NT, EPT, VEC, BB, PP)                                                        \
    if (p.threads == NT && p.ept == EPT && p.vec == VEC && (p.block_steps == 0 || p.block_steps == BB) && \
        (p.rows == 0 || p.rows == rows_kind(PP)) && (p.prefetch == 0 || p.prefetch == (PP < 0 ? 1 : PP)) && \
        (p.slices <= 1 || can_slice(NT, VEC, BB, PP))) {                                        \
        p.block_steps = BB;                                                                    \
        p.prefetch = PP < 0 ? 1 : PP;                                                          \
        p.rows = rows_kind(PP);                                                                \
        if (a) {                                                                               \
            launch_variant<NT, EPT, VEC, BB, PP>(*a, s);                                        \
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

