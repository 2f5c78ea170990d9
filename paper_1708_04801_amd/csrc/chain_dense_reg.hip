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

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor over [base, base+bytes): dword-typed, reads past the end return 0.
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// The EPT elements of one row that a thread owns.  Element e of the fragment is column
//   ((e / VEC) * NT + tid) * VEC + e % VEC
// so that every load instruction of a wave covers one contiguous 64*VEC-element span.
template <typename TX, int NT, int EPT, int VEC>
struct RowFrag {
    static constexpr bool kPacked = (sizeof(TX) == 2) && (VEC == 8);
    static constexpr int kWords = kPacked ? EPT / 2 : EPT;
    static constexpr int kChunks = EPT / VEC;
    static_assert(EPT % VEC == 0, "fragment must be whole loads");
    uint32_t w[kWords];     // fp32 bit patterns, or pairs of bfloat16 when packed

    // chunk c of the row behind `row`; off = this lane's byte offset of the chunk in a row
    __device__ inline void load_chunk(int c, __amdgpu_buffer_rsrc_t row, uint32_t off)
    {
        if constexpr (VEC == 1) {
            if constexpr (sizeof(TX) == 2) {
                w[c] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(row, off, 0, 0) << 16;
            } else {
                w[c] = __builtin_amdgcn_raw_buffer_load_b32(row, off, 0, 0);
            }
        } else {
            static_assert(kPacked || (sizeof(TX) == 4 && VEC == 4), "16-byte loads only");
            const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(row, off, 0, 0);
            w[4 * c + 0] = q[0];
            w[4 * c + 1] = q[1];
            w[4 * c + 2] = q[2];
            w[4 * c + 3] = q[3];
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

// A helper workgroup (one whose index is k or more) runs ahead of a chain and touches one dword
// of every 128-byte line of the rows the chain will visit, so that they sit in the L2 cache of the
// chain's XCD when the chain asks for them.  One compute unit draws some 55-60 GB/s from HBM however
// many loads it keeps in flight, which for 16 KiB rows is no faster than a chain can consume them;
// out of L2 it draws more than twice that.  Workgroups are handed to the XCDs in turn, so with k a
// multiple of 8 helper k*q + b and chain workgroup b share an XCD; the q-th of a chain's Q helpers
// takes the steps t with t mod Q = q.  The chain publishes how far it has come; a helper stays
// between kLeadMin and kLeadMax steps ahead of that (far enough to beat the chain's own requests,
// close enough that the lines are still cached when they are used), stops when the chain says it
// has finished, and gives up when the chain does not move, so it ends whatever the chain does.  The touched data lands in a scratch corner
// of LDS and is never read.
constexpr int kLeadMin = 10, kLeadMax = 26;
constexpr uint32_t kChainDone = 0xFFFFFFFFu;      // published by a chain that has finished

template <typename TX>
__device__ inline void run_ahead_of_chain(const ChainArgs &a, uint32_t *lds_sink)
{
    if (threadIdx.x >= kWave) return;                    // one wave does it
    const int lane = (int)threadIdx.x;
    const int h = (int)blockIdx.x - a.k;
    const int b = h % a.k, q = h / a.k, Q = a.helpers / a.k;
    const int chain = a.order[b];
    const int64_t n = a.nsteps[b];
    const int64_t step0 = a.step0[b];
    const char *X = static_cast<const char *>(a.dense);
    const int64_t row_stride = a.ld * (int64_t)sizeof(TX);
    const uint32_t row_bytes = (uint32_t)(a.d * (int64_t)sizeof(TX));
    const uint32_t *progress = a.progress + b;
    const uint32_t voff = (uint32_t)(lane * 128);        // an instruction touches 64 lines: 8 KiB of a row
    typedef __attribute__((address_space(3))) uint32_t *lds_ptr;
    const uint32_t sink = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(size_t)(lds_ptr)lds_sink);
    uint32_t seen = 0;                                   // steps the chain has completed, as last read
    int64_t polls = n / 4 + (1 << 15);                   // every wait below draws on this
    bool alive = true;
    for (int64_t w0 = 0; w0 < n && alive; w0 += kWave) {
        const uint32_t rows = sample_window(a.seed_lo, a.seed_hi, (uint32_t)chain, step0 + w0, (uint32_t)a.m, a.perm,
                                            (uint32_t)a.k);
        for (int j = (int)((q + Q - (int)(w0 % Q)) % Q); j < kWave && w0 + j < n; j += Q) {
            const uint32_t t = (uint32_t)(w0 + j);
            while (seen != kChainDone && (int32_t)(t - seen) > kLeadMax && polls > 0) {
                seen = __hip_atomic_load(progress, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                --polls;
                if (seen != kChainDone && (int32_t)(t - seen) > kLeadMax) __builtin_amdgcn_s_sleep(16);
            }
            if (polls <= 0 || seen == kChainDone) {      // the chain does not move, or has finished
                alive = false;
                break;
            }
            if ((int32_t)(t - seen) < kLeadMin) continue;        // the chain has asked for this row itself by now
            const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)rows, j);
            const uint64_t base = (uint64_t)(uintptr_t)X + (uint64_t)row * (uint64_t)row_stride;
            u32x4 rx;
            rx[0] = (uint32_t)base;
            rx[1] = (uint32_t)(base >> 32) & 0xffffu;
            rx[2] = row_bytes;
            rx[3] = 0x00020000u;
            for (uint32_t piece = 0; piece < row_bytes; piece += 64 * 128) {
                asm volatile("s_nop 4\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                             :
                             : "s"(sink), "v"(voff), "s"(rx), "s"(piece)
                             : "memory", "m0");
            }
            asm volatile("s_waitcnt vmcnt(12)" : : : "memory");
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");          // nothing may still be landing when the wave ends
}

// TX and LOSS are template parameters (not just per-file constants) so that the four builds of
// this file produce four distinct sets of kernel symbols.
template <typename TX, int LOSS, int NT, int EPT, int VEC, int B, int P>
__global__ __launch_bounds__(NT) void chain_dense_reg_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;     // state, dot products and the step recursion
    using Frag = RowFrag<TX, NT, EPT, VEC>;
    constexpr int NW = NT / kWave;
    constexpr int NG = B * (B - 1) / 2;
    constexpr int NR = B + NG;
    constexpr int NACC = EPT >= 4 ? 4 : EPT;       // independent partial sums per dot product
    constexpr int D = B * P;                       // steps per group of P rounds
    static_assert(kWave % D == 0, "a 64-step window must hold whole groups");
    __shared__ TV red[2][NR][NW];
    // Labels of a whole window, gathered straight into LDS one window ahead (per wave, two windows)
    __shared__ float ylab[NW][2][kWave];

    if ((int)blockIdx.x >= a.k) {       // a helper workgroup: see run_ahead_of_chain
        run_ahead_of_chain<TX>(a, reinterpret_cast<uint32_t *>(&ylab[0][0][0]));
        return;
    }
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
        uint32_t off[Frag::kChunks];               // this lane's byte offset of each chunk
#pragma unroll
        for (int c = 0; c < Frag::kChunks; ++c) off[c] = (uint32_t)(((c * NT + tid) * VEC) * sizeof(TX));
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
            shard_lo = a.shard[blockIdx.x];
            shard_len = a.shard[a.k + blockIdx.x];
            const uint32_t pos0 = a.shard[2 * a.k + blockIdx.x], room = shard_len - pos0;
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

        int parity = 0;
        // One round: steps at in-window positions j .. j+B-1, rows in slot u.  While the partial
        // sums cross the workgroup, slot u_prev (consumed one round ago) is requested again for
        // the round kAhead steps from here.
        auto round = [&](int u, int j, int u_prev) {
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
                if constexpr (P > 1) issue_rows(u_prev, next_rows, 0, kFirstHalf);
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
                    if constexpr (NW > 1) {
                        c[b] = (zy[b] * dot < 1.0) ? cy[b] : 0.0;
                    } else {
                        const bool inside = (__builtin_amdgcn_ballot_w64(zy[b] * dot < 1.0) >> (kWave - 1)) != 0;   // lane 63's verdict
                        c[b] = inside ? cy[b] : 0.0;
                    }
                } else {
                    // -eta*g/s_next with g = -y/(1+exp(y*yhat)); exp as 2^(log2(e)*y*s*dot)
                    c[b] = cy[b] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(zy[b] * dot));
                }
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
#pragma unroll
                for (int b = 0; b < B; ++b) v[e] += c[b] * (TV)x[u][b].at(e);
            }
            if constexpr (P > 1 && kFirstHalf < B) {
                __builtin_amdgcn_sched_barrier(0);        // keep these requests behind the update
                issue_rows(u_prev, next_rows, kFirstHalf, B);
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
            if (a.helpers > 0 && tid == 0) a.progress[blockIdx.x] = (uint32_t)(g * D);   // for the helpers to see
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
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);      // no label load may still be on its way to LDS when the wave ends
        if (a.helpers > 0 && tid == 0) a.progress[blockIdx.x] = kChainDone;
        // scale at the chain's end: s_w covers the steps before the last window
        const int64_t last_w = (n - 1) / kWave;
        const int rem = (int)(n - last_w * kWave);                          // 1..64 steps in it
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

// ---------------------------------------------------------------------------------------------
// Instantiated variants: V(threads, elements per thread, load width, B, P).  Within one
// (threads, ept, vec) shape the first entry is the default; the others are reachable through a
// forced plan.  Register budget per thread: 512 at 256 threads, 256 at 512, 128 at 1024.
// P > 0: rows wait in registers, P rounds requested ahead.  P = -1: the next row is staged in LDS.
// P = 0: rows are streamed twice.  P = -2: rows are fed through an LDS ring by mover waves.
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
    V(256, 8, 8, 1, -2) V(256, 16, 8, 1, -2) V(256, 32, 8, 1, -2)                              \
    V(256, 8, 8, 2, -2) V(256, 16, 8, 2, -2) V(256, 32, 8, 2, -2)                              \
    V(1024, 16, 8, 1, -1) V(1024, 32, 8, 1, -1) WPSGD_WIDEST_LDS(V, 8)                          \
    V(1024, 16, 8, 1, 0) V(1024, 32, 8, 1, 0) WPSGD_WIDEST(V, 8)
#define WPSGD_VARIANTS_WIDE(V)
#else
#define WPSGD_VARIANTS_VEC(V)                                                                  \
    V(64, 4, 4, 1, 8) V(64, 4, 4, 1, 16) V(64, 4, 4, 2, 4) V(64, 4, 4, 4, 2)                   \
    V(256, 4, 4, 1, 8) V(256, 8, 4, 1, 8) V(256, 16, 4, 1, 8) V(256, 32, 4, 1, 4) V(256, 16, 4, 1, 16) V(256, 8, 4, 1, 16)             \
    V(256, 4, 4, 4, 2) V(256, 8, 4, 4, 2) V(256, 16, 4, 4, 2) V(256, 16, 4, 1, 4)              \
    V(256, 16, 4, 2, 2) V(256, 16, 4, 2, 4) V(256, 16, 4, 2, 8) V(256, 32, 4, 4, 2)            \
    V(256, 4, 4, 1, -2) V(256, 8, 4, 1, -2) V(256, 16, 4, 1, -2) V(256, 32, 4, 1, -2)          \
    V(256, 4, 4, 2, -2) V(256, 8, 4, 2, -2) V(256, 16, 4, 2, -2)                               \
    V(512, 8, 4, 1, 8) V(512, 8, 4, 4, 2) V(512, 8, 4, 2, 4)                                   \
    V(1024, 4, 4, 1, 8) V(1024, 4, 4, 4, 2) V(1024, 4, 4, 2, 4)                                \
    V(1024, 16, 4, 1, -1) V(1024, 32, 4, 1, -1)                                                \
    V(1024, 16, 4, 1, 0) V(1024, 32, 4, 1, 0) WPSGD_WIDEST(V, 4)
#define WPSGD_VARIANTS_WIDE(V)
#endif

#define WPSGD_ALL_VARIANTS(V) WPSGD_VARIANTS_VEC(V) WPSGD_VARIANTS_ANY(V) WPSGD_VARIANTS_WIDE(V)

template <int NT, int EPT, int VEC, int BB, int PP>
static void launch_variant(const ChainArgs &a, hipStream_t s)
{
    if constexpr (PP == -2) {
        // (its LDS ring leaves room for one workgroup per compute unit, helpers included)
        hipLaunchKernelGGL((chain_dense_fed_kernel<RowElem, kLoss, NT, EPT, VEC, BB>), dim3(a.k + a.helpers), dim3(2 * NT), 0, s, a);
    } else if constexpr (PP < 0) {
        hipLaunchKernelGGL((chain_dense_lds_kernel<RowElem, kLoss, NT, EPT, VEC>), dim3(a.k), dim3(NT), 0, s, a);
    } else if constexpr (PP == 0) {
        hipLaunchKernelGGL((chain_dense_wide_kernel<RowElem, kLoss, NT, EPT, VEC>), dim3(a.k), dim3(NT), 0, s, a);
    } else {
        auto kernel = chain_dense_reg_kernel<RowElem, kLoss, NT, EPT, VEC, BB, PP>;
        size_t claim = 0;
        if (a.helpers > 0) {
            // more than half of a compute unit's LDS per workgroup: chains and helpers each get a unit of their own
            static int allowed = 0;         // 0 not asked yet, 1 granted, -1 refused
            if (allowed == 0) {
                allowed = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, 84 * 1024) == hipSuccess ? 1 : -1;
                if (allowed < 0) (void)hipGetLastError();
            }
            if (allowed > 0) claim = 84 * 1024;
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

constexpr int rows_kind(int pp) { return pp > 0 ? 1 : (pp == -1 ? 2 : (pp == 0 ? 3 : 4)); }

// find(plan, launch?): walks the table; exact match on (threads, ept, vec, B, P, rows) where the
// plan gives them, else the first entry of the shape.
hipError_t WPSGD_CAT(dense_reg_dispatch_, WPSGD_SUFFIX)(Plan &p, const ChainArgs *a, hipStream_t s)
{
#define WPSGD_TRY(NT, EPT, VEC, BB, PP)                                                        \
    if (p.threads == NT && p.ept == EPT && p.vec == VEC && (p.block_steps == 0 || p.block_steps == BB) && \
        (p.rows == 0 || p.rows == rows_kind(PP)) && (p.prefetch == 0 || p.prefetch == (PP < 0 ? 1 : PP))) { \
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
