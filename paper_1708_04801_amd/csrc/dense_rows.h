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

__device__ inline uint32_t xcd_of_this_wave()
{
    uint32_t x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    return x & 0xfu;
}

// ---------------------------------------------------------------------------------------------
// A chain cut into column slices, one workgroup (and compute unit) per slice: every slice holds
// its part of the model vector and reads its part of each row, and once per round the slices add
// up their partial sums.  The sums travel through a small table in global memory, 2 KiB per chain:
// for each round parity up to four record blocks of 256 bytes.  The first 128-byte line of a block
// holds one 16-byte record {w0, w1, w2, stamp} per slice, the second line each record's mirror
// image {stamp, w2, w1, w0}; stamp = round number + 1 (the table is zero at launch), and twelve
// 32-bit words of sums fit in the four blocks.  Lane s of every wave reads slice s's records, so one
// poll of a wave touches two lines per block.  A reader accepts a slice's records when each and its
// mirror carry the stamp it waits for and agree word for word, so it never uses half of one
// round's record and half of another's.  The same parity's records are written again only two
// rounds later, after their writer has read every slice's record of the round in between, which
// those slices published after reading this one: nobody still reads a record when it is
// overwritten.  Every wait has a budget; a slice that loses the others says so in the workspace's
// status word, fills its part of the result with NaN and ends.
//
// The accepted sums sit in lanes 0..7 (zero beyond the last slice) and are added by three
// exchange levels among those lanes: one fixed tree, the same in every wave of every slice, so all
// slices continue with identical bits.  (Reading them lane by lane into scalars and adding in
// slice order cost a seventh of the whole pass on the widest workload.)
//
// NEAR: all slices of the chain run on one XCD and meet in its L2: plain stores end up there, and
// device-scope loads skip the reader's own first-level cache and find them (measured between two
// compute units of one XCD: 580 cycles one way, against 1000-1200 with device-scope stores, which
// are what slices on different XCDs need; loads of narrower scope are served from the reader's
// own first-level cache and never see the other side's store).
// ---------------------------------------------------------------------------------------------
constexpr int kMaxSlices = 8;
constexpr int kSliceSlotWords = 32;
constexpr int kSliceMaxWords = 12;

__device__ inline uint32_t *slice_slot(const ChainArgs &a, int chain_block, int slice, int parity)
{
    return static_cast<uint32_t *>(a.xchg) + (size_t)chain_block * (kMaxSlices * 2 * kSliceSlotWords) + parity * (4 * 64) + slice * 4;
}

template <bool NEAR, int NWORDS>
__device__ inline void slice_publish(uint32_t *slot, const uint32_t (&w)[kSliceMaxWords], uint32_t stamp)
{
#pragma unroll
    for (int q = 0; q < (NWORDS + 2) / 3; ++q) {
        u32x4 rec, mirror;
        rec[0] = w[3 * q]; rec[1] = w[3 * q + 1]; rec[2] = w[3 * q + 2]; rec[3] = stamp;
        mirror[0] = stamp; mirror[1] = w[3 * q + 2]; mirror[2] = w[3 * q + 1]; mirror[3] = w[3 * q];
        uint32_t *at = slot + 64 * q;
        if constexpr (NEAR) {
            asm volatile("global_store_dwordx4 %0, %1, off\n\tglobal_store_dwordx4 %0, %2, off offset:128"
                         :
                         : "v"(at), "v"(rec), "v"(mirror)
                         : "memory");
        } else {
            asm volatile("global_store_dwordx4 %0, %1, off sc1\n\tglobal_store_dwordx4 %0, %2, off offset:128 sc1"
                         :
                         : "v"(at), "v"(rec), "v"(mirror)
                         : "memory");
        }
    }
}

// One slice's words if its records are complete for `stamp`.  All loads and the wait for them sit
// in one assembly statement: their results are ordinary registers when it ends.
template <int NWORDS>
__device__ inline bool slice_read(const uint32_t *slot, uint32_t stamp, uint32_t (&w)[kSliceMaxWords])
{
    constexpr int NQ = (NWORDS + 2) / 3;
    static_assert(NQ >= 1 && NQ <= 4, "one to four records");
    u32x4 rec[NQ], mirror[NQ];
    if constexpr (NQ == 1) {
        asm volatile("global_load_dwordx4 %0, %2, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %2, off offset:128 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(rec[0]), "=&v"(mirror[0])
                     : "v"(slot)
                     : "memory");
    } else if constexpr (NQ == 2) {
        asm volatile("global_load_dwordx4 %0, %4, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %4, off offset:128 sc1\n\t"
                     "global_load_dwordx4 %2, %4, off offset:256 sc1\n\t"
                     "global_load_dwordx4 %3, %4, off offset:384 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(rec[0]), "=&v"(mirror[0]), "=&v"(rec[1]), "=&v"(mirror[1])
                     : "v"(slot)
                     : "memory");
    } else if constexpr (NQ == 3) {
        asm volatile("global_load_dwordx4 %0, %6, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %6, off offset:128 sc1\n\t"
                     "global_load_dwordx4 %2, %6, off offset:256 sc1\n\t"
                     "global_load_dwordx4 %3, %6, off offset:384 sc1\n\t"
                     "global_load_dwordx4 %4, %6, off offset:512 sc1\n\t"
                     "global_load_dwordx4 %5, %6, off offset:640 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(rec[0]), "=&v"(mirror[0]), "=&v"(rec[1]), "=&v"(mirror[1]), "=&v"(rec[2]), "=&v"(mirror[2])
                     : "v"(slot)
                     : "memory");
    } else {
        asm volatile("global_load_dwordx4 %0, %8, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %8, off offset:128 sc1\n\t"
                     "global_load_dwordx4 %2, %8, off offset:256 sc1\n\t"
                     "global_load_dwordx4 %3, %8, off offset:384 sc1\n\t"
                     "global_load_dwordx4 %4, %8, off offset:512 sc1\n\t"
                     "global_load_dwordx4 %5, %8, off offset:640 sc1\n\t"
                     "global_load_dwordx4 %6, %8, off offset:768 sc1\n\t"
                     "global_load_dwordx4 %7, %8, off offset:896 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(rec[0]), "=&v"(mirror[0]), "=&v"(rec[1]), "=&v"(mirror[1]), "=&v"(rec[2]), "=&v"(mirror[2]), "=&v"(rec[3]), "=&v"(mirror[3])
                     : "v"(slot)
                     : "memory");
    }
    bool ok = true;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        ok = ok && rec[q][3] == stamp && mirror[q][0] == stamp && rec[q][0] == mirror[q][3] && rec[q][1] == mirror[q][2] &&
             rec[q][2] == mirror[q][1];
        w[3 * q] = rec[q][0];
        w[3 * q + 1] = rec[q][1];
        w[3 * q + 2] = rec[q][2];
    }
    return ok;
}

// Do all slices of this chain run on one XCD?  Every slice writes its XCD number (plus one) behind
// the slots, at device scope, and reads the others'; if they do not all show up in time the answer
// is no, which is always safe.
__device__ inline bool slices_share_an_xcd(const ChainArgs &a, int chain_block, int slice, bool announcer)
{
    uint32_t *words = static_cast<uint32_t *>(a.xchg) + (size_t)a.k * kMaxSlices * 2 * kSliceSlotWords +
                      (size_t)chain_block * kMaxSlices;
    const uint32_t mine = xcd_of_this_wave() + 1u;
    if (announcer) __hip_atomic_store(words + slice, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int lane = (int)(threadIdx.x & (kWave - 1));
    bool all = false, same = false;
    for (int tries = 0; tries < (1 << 14) && !all; ++tries) {
        const uint32_t x = lane < a.slices ? __hip_atomic_load(words + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : mine;
        all = __builtin_amdgcn_ballot_w64(x != 0u) == ~0ull;
        same = __builtin_amdgcn_ballot_w64(x == mine) == ~0ull;
        if (!all) __builtin_amdgcn_s_sleep(8);
    }
    return all && same;
}

// the value a lane pattern (a DPP control word) brings from another lane of the same row of 16
template <int CTRL>
__device__ inline float from_other_lane(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ inline double from_other_lane(double v)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)bits, CTRL, 0xf, 0xf, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(bits >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// Adds the slices' sums for this round, in one fixed tree.  w holds NVAL values of this slice (fp32:
// one word each; fp64: two), identical in every wave of the slice; lane 0 of wave 0 publishes them.
// Returns false if the other slices did not show up within max_polls polls.
template <bool IS_F64, int NVAL, bool NEAR>
__device__ inline bool slices_all_reduce(const ChainArgs &a, int chain_block, int slice, bool publisher, uint32_t round,
                                         uint32_t max_polls, uint32_t (&w)[kSliceMaxWords])
{
    constexpr int NWORDS = IS_F64 ? 2 * NVAL : NVAL;
    static_assert(NWORDS <= kSliceMaxWords, "a slot holds twelve words");
    const int lane = (int)(threadIdx.x & (kWave - 1));
    const int parity = (int)(round & 1u);
    const uint32_t stamp = round + 1u;
    if (publisher) slice_publish<NEAR, NWORDS>(slice_slot(a, chain_block, slice, parity), w, stamp);
    // The slices reach this point within a few hundred cycles of each other, and a poll takes some
    // 600 (it also waits for the row requests made before it: loads return in order).  One sent at
    // once is answered just before the other records land and a second has to follow; sent ~400
    // cycles later, the first usually finds them (measured: 2.05 polls per round without the
    // pause, 4 % of the pass).
    __builtin_amdgcn_s_sleep(6);
    const int src = lane < a.slices ? lane : 0;                   // lanes beyond the slices repeat slice 0
    const uint32_t *slot = slice_slot(a, chain_block, src, parity);
    uint32_t got[kSliceMaxWords];
    // The first poll usually finds every record.  The wait is bounded by a number of polls the host has
    // worked out from the time it allows (a poll takes 600 to 1200 cycles).  (A clock read in this loop,
    // or a second copy of the poll behind the first, cost 3 % of a pass although neither is ever reached
    // when all goes well: the loop keeps the shape it was tuned in.)
    bool all = false;
    for (uint32_t tries = 0; tries < max_polls && !all; ++tries)
        all = __builtin_amdgcn_ballot_w64(slice_read<NWORDS>(slot, stamp, got)) == ~0ull;
    if (!all) return false;
    if constexpr (IS_F64) {
        // as below, on the two halves of each fp64 sum
#pragma unroll
        for (int r = 0; r < NVAL; ++r) {
            double t = lane < a.slices ? __longlong_as_double((long long)(((uint64_t)got[2 * r + 1] << 32) | got[2 * r])) : 0.0;
            t += from_other_lane<0xB1>(t);
            t += from_other_lane<0x4E>(t);
            t += from_other_lane<0x141>(t);
            const uint64_t bits = (uint64_t)__double_as_longlong(t);
            w[2 * r] = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)bits);
            w[2 * r + 1] = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(bits >> 32));
        }
    } else {
        // lanes 0..7 hold the slices' sums (zero beyond the last slice); three exchange levels among
        // those eight lanes add them in one fixed tree, the same in every slice and wave
        if constexpr (NVAL == 3) {
            // three sums level by level: each one's next level is two instructions behind its last
            float t0 = lane < a.slices ? __uint_as_float(got[0]) : 0.0f;
            float t1 = lane < a.slices ? __uint_as_float(got[1]) : 0.0f;
            float t2 = lane < a.slices ? __uint_as_float(got[2]) : 0.0f;
#define WPSGD_DPP3(CTRL)                                                       \
    "v_add_f32_dpp %0, %0, %0 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t" \
    "v_add_f32_dpp %1, %1, %1 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t" \
    "v_add_f32_dpp %2, %2, %2 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            asm volatile("s_nop 1\n\t" WPSGD_DPP3("quad_perm:[1,0,3,2]") WPSGD_DPP3("quad_perm:[2,3,0,1]") WPSGD_DPP3("row_half_mirror")
                         : "+v"(t0), "+v"(t1), "+v"(t2));
#undef WPSGD_DPP3
            w[0] = (uint32_t)__builtin_amdgcn_readfirstlane(__float_as_int(t0));
            w[1] = (uint32_t)__builtin_amdgcn_readfirstlane(__float_as_int(t1));
            w[2] = (uint32_t)__builtin_amdgcn_readfirstlane(__float_as_int(t2));
        } else {
#pragma unroll
            for (int r = 0; r < NVAL; ++r) {
                float t = lane < a.slices ? __uint_as_float(got[r]) : 0.0f;
                t += from_other_lane<0xB1>(t);      // quad_perm [1,0,3,2]
                t += from_other_lane<0x4E>(t);      // quad_perm [2,3,0,1]
                t += from_other_lane<0x141>(t);     // row_half_mirror
                w[r] = (uint32_t)__builtin_amdgcn_readfirstlane(__float_as_int(t));
            }
        }
    }
    return true;
}

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
