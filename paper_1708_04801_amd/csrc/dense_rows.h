// What the dense register kernels share: the per-thread fragment of a row, raw buffer descriptors,
// and the helper workgroups that run ahead of a chain.
#pragma once
#include "device_utils.h"
#include "internal.h"

namespace wpsgd {

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
// out of L2 it draws more than twice that.
//
// Who helps whom is settled on the device, because only there is it known which XCD a workgroup
// landed on.  Every chain workgroup writes its XCD number (plus one) next to its progress counter.
// A helper reads its own, waits (within a budget) until every chain has written, takes the next
// free seat of its XCD with an atomic increment, and serves the chains of that XCD in turn: seat
// r goes to chain r mod (chains on this XCD) as that chain's (r div chains)-th helper, and the
// q-th of a chain's Q helpers takes the steps t with t mod Q = q.  Helpers beyond Q per chain
// leave.  The chain publishes how far it has come; a helper stays between kLeadMin and kLeadMax
// steps ahead of that (far enough to beat the chain's own requests, close enough that the lines
// are still cached when they are used), stops when the chain says it has finished, and gives up
// when the chain does not move, so it ends whatever the chain does.  The touched data lands in a
// scratch corner of LDS and is never read.
//
// Header words used (all zero at launch): progress[b] for chain workgroup b, progress[k + b] its
// XCD number plus one, progress[2k + x] the seats taken on XCD x.
constexpr int kLeadMin = 10, kLeadMax = 26;
constexpr uint32_t kChainDone = 0xFFFFFFFFu;      // published by a chain that has finished
constexpr int kMaxXcds = 16;

__device__ inline uint32_t xcd_of_this_wave()
{
    uint32_t x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    return x & 0xfu;
}

// called by thread 0 of a chain workgroup before its first step.  Helpers on every XCD read this
// word and each XCD has an L2 cache of its own, so it is stored at device scope (written through);
// the progress counter is only read by helpers of the same XCD and takes plain stores.
__device__ inline void announce_chain_workgroup(const ChainArgs &a)
{
    __hip_atomic_store(a.progress + a.k + blockIdx.x, xcd_of_this_wave() + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// index of the n-th set bit (n counted from 0) of a mask that has more than n bits set
__device__ inline int nth_set_bit(uint64_t mask, int n)
{
    for (int i = 0; i < n; ++i) mask &= mask - 1;
    return __builtin_ctzll(mask);
}

template <typename TX>
__device__ inline void run_ahead_of_chain(const ChainArgs &a, uint32_t *lds_sink)
{
    if (threadIdx.x >= kWave) return;                    // one wave does it
    const int lane = (int)threadIdx.x;
    const int Q = a.helpers / a.k;
    // which chains run on this XCD?  (k <= 128: two header words per lane)
    const uint32_t here = xcd_of_this_wave() + 1u;
    const uint32_t *where = a.progress + a.k;
    uint64_t on0 = 0, on1 = 0;
    bool all = false;
    for (int tries = 0; tries < (1 << 14) && !all; ++tries) {
        const uint32_t x0 = lane < a.k ? __hip_atomic_load(where + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ~0u;
        const uint32_t x1 = lane + kWave < a.k
                                ? __hip_atomic_load(where + lane + kWave, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                : ~0u;
        all = __builtin_amdgcn_ballot_w64(x0 != 0u && x1 != 0u) == ~0ull;
        on0 = __builtin_amdgcn_ballot_w64(x0 == here);
        on1 = __builtin_amdgcn_ballot_w64(x1 == here);
        if (!all) __builtin_amdgcn_s_sleep(16);
    }
    const int n_here = __builtin_popcountll(on0) + __builtin_popcountll(on1);
    if (!all || n_here == 0) return;                     // chains not running yet, or none of them here
    uint32_t seat = 0;
    if (lane == 0) seat = atomicAdd(a.progress + 2 * a.k + (here - 1u), 1u);
    seat = (uint32_t)__builtin_amdgcn_readfirstlane((int)seat);
    const int q = (int)seat / n_here, which = (int)seat % n_here;
    if (q >= Q) return;                                  // this XCD's chains have their helpers
    const int first = __builtin_popcountll(on0);
    const int b = which < first ? nth_set_bit(on0, which) : kWave + nth_set_bit(on1, which - first);
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

}  // namespace wpsgd
