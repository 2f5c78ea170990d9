// Sparse-row (CSR) SGD chains, three wavefronts per chain.
//
// A step of a sparse chain is a short dependent recursion (gather the model at the row's columns,
// reduce, decide, scatter), and one wavefront issues one instruction at a time: with a single
// wave the step is bound by the number of instructions in it, and most of those do not depend on
// the model at all - finding the row, fetching its entries, sorting columns into "kept in LDS"
// and "kept in HBM", computing addresses, deciding whether an early fetch can be stale.  This
// kernel gives that part to two more waves, each on a SIMD of its own:
//
//   record scout  walks the chain's sample stream ahead of the worker.  For every step it fetches
//           the row's entries (last entry first, so that the HBM-resident columns of a row, its
//           highest, share the first load) and writes one 16-byte record per entry into an LDS
//           ring: the value, the LDS address of the model element (or of a scratch slot), the
//           offset of the model element in the HBM-resident part of the vector (or an offset past
//           its end, which the hardware turns into no access at all), and whether it is one.  It
//           also writes the per-step scalars of the recursion.
//   stamp scout   walks the same stream, keeps the stamp tables described below and marks the
//           steps that must read their values again.
//   worker  runs the recursion of Eq. 5 (w = s*v, the shrink carried by the scalar s) from the
//           records: all its loads, stores and LDS accesses are unconditional and their
//           addresses come ready-made.
//
// The model vector's HBM-resident part is prepared before this kernel and turned into W after it
// by two wide kernels (csr_state_start_kernel, csr_state_finish_kernel), so a chain does no work
// proportional to d.
//
// The ring has three sections of kG steps.  One barrier per section keeps the waves in step:
// the scouts pass barrier i after writing section i, the worker passes it before it starts
// section i-1, whose steps read records of sections i-1 and i; so the scouts are always writing
// the one section the worker is not reading.  All waves execute the same number of barriers.
//
// Model values: columns below kPHead live in LDS; the others stay in HBM and are requested kTQ
// steps ahead.  A value fetched early is stale if a step in between wrote the same column.  Whether
// that can have happened depends on the rows alone, not on the model, so the stamp scout decides it: it
// keeps two LDS stamp tables (two different hashes of the column) with the step number of the last
// write to each slot, and a step that finds recent numbers in both slots of one of its columns is
// marked; the worker drains the memory queue and reads that step's values again.  A write always
// leaves both stamps, so a conflict is never missed; two unrelated aliases at once cost a needless
// re-read.  The worker carries no stamp traffic at all.
//
// Which writes can an early fetch miss?  Memory operations of one wave complete in issue order.
// The values for step t+kTQ are requested at the end of step t, after step t has waited for its
// own values, which were requested at the end of step t-kTQ, after that step's stores.  So all
// stores of steps <= t-kTQ are complete by then, and the fetch for step t+kTQ can only miss the
// writes of steps t-kTQ+1 .. t+kTQ-1: the 2*kTQ-1 steps before the one that uses it.
#include <algorithm>
#include <type_traits>

#include "device_utils.h"
#include "internal.h"

namespace wpsgd {
namespace {

typedef uint32_t pu32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t pu32x2 __attribute__((ext_vector_type(2)));

constexpr int kPHead = 8192;       // columns whose model values live in LDS
constexpr int kPStamps = 8192;     // entries of each stamp table (16-bit step numbers)
constexpr int kG = 8;              // steps per ring section
constexpr int kSections = 3;
constexpr int kLead = 16;          // scout: entries are requested this many steps before their records are written
constexpr int kTQ = 4;             // worker: HBM-resident model values are requested this many steps ahead
constexpr int kChunks = 2;         // entries of a row that go through records: kChunks * 64
constexpr int kSlots = kChunks * kWave;
constexpr int kPairThreads = 3 * kWave;     // the worker and two scouts
constexpr uint32_t kRecordBytes = kSlots * 16;              // the records of one step ...
constexpr uint32_t kStepBytes = kRecordBytes + 32;          // ... followed by its scalars (StepScalars, StepRow)
constexpr uint32_t kSectionBytes = kG * kStepBytes;
constexpr uint16_t kRecent = 2 * kTQ;
constexpr int kWideTail = 1 << 30;  // flag in a step's row length: HBM-resident columns also outside chunk 0
static_assert(kTQ + 1 < kG, "record and value rings are indexed modulo kG");
static_assert(kLead == 2 * kG, "the scout's entry ring is two sections deep");

// Byte offsets inside the one LDS block.
template <typename TV>
struct Lds {
    static constexpr uint32_t head = 0;                                           // kPHead model values
    static constexpr uint32_t head_scratch = head + kPHead * sizeof(TV);          // one per record slot
    static constexpr uint32_t stamp_a = head_scratch + kSlots * sizeof(TV);       // kPStamps + scratch slots
    static constexpr uint32_t stamp_b = stamp_a + (kPStamps + kSlots) * 2;
    static constexpr uint32_t ring = (stamp_b + (kPStamps + kSlots) * 2 + 15u) & ~15u;
    static constexpr uint32_t bytes = ring + kSections * kSectionBytes;
};

// per-step scalars, written by the scout behind the step's records
template <typename TV>
struct __attribute__((aligned(16))) StepScalars {
    TV zs, cs;            // y*s_l (times log2 e for the logistic loss) and y*eta/s_{l+1}; cs = 0 past the chain's end
};
struct __attribute__((aligned(16))) StepRow {
    int64_t lo;           // first entry of the row
    int32_t len;          // entries in the row
    int32_t pad;
};

__device__ inline void wait_lds_then_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Memory instructions the compiler does not see; each drains the queue, so the value is there (or
// the store is done) when the statement ends.  Used off the fast path only, so that the compiler's
// count of outstanding loads, and with it the partial waits of the fast path, is the same whether
// or not the slow path ran.
__device__ inline double drained_buffer_load(pu32x4 rsrc, uint32_t off, double)
{
    double r;
    asm volatile("s_waitcnt vmcnt(0)\n\tbuffer_load_dwordx2 %0, %1, %2, 0 offen\n\ts_waitcnt vmcnt(0)"
                 : "=v"(r) : "v"(off), "s"(rsrc) : "memory");
    return r;
}
__device__ inline float drained_buffer_load(pu32x4 rsrc, uint32_t off, float)
{
    float r;
    asm volatile("s_waitcnt vmcnt(0)\n\tbuffer_load_dword %0, %1, %2, 0 offen\n\ts_waitcnt vmcnt(0)"
                 : "=v"(r) : "v"(off), "s"(rsrc) : "memory");
    return r;
}
__device__ inline void drained_buffer_store(pu32x4 rsrc, uint32_t off, double x)
{
    asm volatile("buffer_store_dwordx2 %0, %1, %2, 0 offen\n\ts_waitcnt vmcnt(0)" : : "v"(x), "v"(off), "s"(rsrc) : "memory");
}
__device__ inline void drained_buffer_store(pu32x4 rsrc, uint32_t off, float x)
{
    asm volatile("buffer_store_dword %0, %1, %2, 0 offen\n\ts_waitcnt vmcnt(0)" : : "v"(x), "v"(off), "s"(rsrc) : "memory");
}
__device__ inline uint32_t drained_global_load_u32(const void *p)
{
    uint32_t r;
    asm volatile("s_waitcnt vmcnt(0)\n\tglobal_load_dword %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(r) : "v"(p) : "memory");
    return r;
}

__device__ inline pu32x4 descriptor(const void *base, uint32_t bytes)
{
    const uint64_t b = (uint64_t)(uintptr_t)base;
    pu32x4 r;
    r[0] = (uint32_t)b;
    r[1] = (uint32_t)(b >> 32) & 0xffffu;
    r[2] = bytes;
    r[3] = 0x00020000u;      // dword-typed raw buffer: reads past `bytes` return 0, writes are dropped
    return r;
}

__device__ inline double load_state(__amdgpu_buffer_rsrc_t r, uint32_t off, double)
{
    const pu32x2 q = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
    return __longlong_as_double(((long long)q[1] << 32) | (long long)q[0]);
}
__device__ inline float load_state(__amdgpu_buffer_rsrc_t r, uint32_t off, float)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
}
__device__ inline void store_state(__amdgpu_buffer_rsrc_t r, uint32_t off, double x)
{
    const long long b = __double_as_longlong(x);
    pu32x2 q;
    q[0] = (uint32_t)b;
    q[1] = (uint32_t)(b >> 32);
    __builtin_amdgcn_raw_buffer_store_b64(q, r, off, 0, 0);
}
__device__ inline void store_state(__amdgpu_buffer_rsrc_t r, uint32_t off, float x)
{
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(x), r, off, 0, 0);
}

__device__ inline uint32_t stamp_slot_a(uint32_t col) { return col & (kPStamps - 1); }
__device__ inline uint32_t stamp_slot_b(uint32_t col) { return (col + (col >> 13) * 2731u) & (kPStamps - 1); }

template <int LOSS>
__global__ __launch_bounds__(kPairThreads) void chain_csr_pair_kernel(ChainArgs a)
{
    using TV = typename StateType<LOSS>::type;
    using L = Lds<TV>;
    static_assert(L::bytes <= 160 * 1024, "LDS block too large");
    __shared__ __attribute__((aligned(16))) char lds[L::bytes];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int chain = a.order[blockIdx.x];
    const int64_t n = a.nsteps[blockIdx.x];
    const int64_t d = a.d;
    TV *v = static_cast<TV *>(a.state) + (int64_t)chain * d;
    const int64_t nnz = a.row_ptr[a.m];

    const int64_t step0 = a.step0[blockIdx.x];
    // The vector in the workspace holds the chain's start vector on entry (csr_state_start_kernel)
    // and is scaled into W after the launch (csr_state_finish_kernel): the chain itself touches
    // only what its rows touch.  A chain without steps, or a matrix without entries (every step
    // then only shrinks the vector), has nothing to do here.
    if (nnz == 0 || n == 0) return;
    TV *head = reinterpret_cast<TV *>(lds + L::head);
    for (int c = tid; c < kPHead + kSlots; c += kPairThreads)                             // values and scratch slots
        head[c] = (a.w_start && c < kPHead && c < d) ? (TV)a.w_start[c] : (TV)0;
    for (int c = tid; c < 2 * (kPStamps + kSlots); c += kPairThreads) reinterpret_cast<uint16_t *>(lds + L::stamp_a)[c] = 0;
    __syncthreads();

    const int64_t ngroups = (n + kG - 1) / kG;       // the worker runs groups 0..ngroups-1, the scout writes 0..ngroups
    const double rho = a.rho;

    if (wave != 0) {
        // ------------------------------------------------------------------------- scouts
        // Wave 1 writes the records and the step scalars; wave 2 keeps the stamps and marks the steps
        // that must re-read their values.  Both walk the sample stream the same way, kLead steps ahead
        // of what they write, and both write into the section the worker is not reading.
        const uint32_t seed_lo = a.seed_lo, seed_hi = a.seed_hi, m32 = (uint32_t)a.m;
        const double inv_rho = 1.0 / rho;
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

        // per-lane tables of the window being written (a) and the next one (b)
        int64_t lo_a, lo_b;
        int len_a, len_b;
        float y_a, y_b;
        auto load_window = [&](int64_t w, int64_t &lo, int &len, float &y) {
            // (The sampler is written out here rather than called: after a call the compiler no longer knows
            // which loads are outstanding and drains the whole queue at the top of every iteration of the loop
            // below, rows requested kLead steps ahead included.)
            const uint64_t step = (uint64_t)(step0 + w * kWave + lane);
            const uint32_t row = a.perm ? a.perm[shard_position((uint32_t)chain, (uint32_t)a.k, step, m32)]
                                        : sample_row(seed_lo, seed_hi, (uint32_t)chain, step, m32);
            const int64_t p0 = a.row_ptr[row], p1 = a.row_ptr[(int64_t)row + 1];
            lo = p0;
            len = (int)(p1 - p0);
            y = a.y[row];
        };
        load_window(0, lo_a, len_a, y_a);
        load_window(1, lo_b, len_b, y_b);
        StepScalars<TV> sc_tab;          // per lane: the scalars of step (window start + lane)

        auto scout = [&](auto role_tag) {
            constexpr bool MARKS = decltype(role_tag)::value;          // false: records, true: stamps and marks
            int64_t redo_until = -1;         // steps up to this one re-read their values (they follow a very long row)
            struct { bool tail, forced; uint16_t now, sa, sb; char *h; } prev = {false, false, 0, 0, 0, nullptr};      // (stamp scout) the step before
            uint32_t er_col[kLead][kChunks], er_val[kLead][kChunks];
            // Entries of a row into ring slot `slot`, last entry first: slot position e (lane e % 64 of
            // chunk e / 64) holds entry len-1-e.  Columns ascend within a row, so the HBM-resident ones
            // (the large ones) end up at the front and chunk 0 holds them all unless the row has more
            // than 64 of them: the worker then needs one load and one store to HBM per step, not two of
            // each.  Positions past the row's start get an offset past the end and read zeros.
            auto request = [&](int slot, int64_t lo, int len) {
                const uint32_t bytes = (uint32_t)len * 4u;
                const __amdgpu_buffer_rsrc_t rc =
                    __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(a.col_idx + lo), 0, (int)bytes, 0x00020000);
#pragma unroll
                for (int c = 0; c < kChunks; ++c)
                    er_col[slot][c] = __builtin_amdgcn_raw_buffer_load_b32(rc, (uint32_t)(len - 1 - (c * kWave + lane)) * 4u, 0, 0);
                if constexpr (!MARKS) {
                    const __amdgpu_buffer_rsrc_t rv =
                        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.vals + lo), 0, (int)bytes, 0x00020000);
#pragma unroll
                    for (int c = 0; c < kChunks; ++c)
                        er_val[slot][c] = __builtin_amdgcn_raw_buffer_load_b32(rv, (uint32_t)(len - 1 - (c * kWave + lane)) * 4u, 0, 0);
                }
            };
#pragma unroll
            for (int t = 0; t < kLead; ++t) request(t, lane_read_i64(lo_a, t), __builtin_amdgcn_readlane(len_a, t));
            // Enter the loop with an empty queue: with loads pending on entry the compiler covers the entry
            // path by a full drain in front of the loop's first use, which every iteration then pays.
            __builtin_amdgcn_s_waitcnt(0x0F70);

            // One section: steps kG*i .. kG*i+kG-1.  HALF = i & 1 selects the entry-ring slots.
            auto write_group = [&](int64_t i, auto half_tag) {
                constexpr int HALF = decltype(half_tag)::value;
                const int j0 = (int)((i * kG) & (kWave - 1));
                const int64_t w = (i * kG) / kWave;
                if (j0 == 0) {                       // a new window: rotate the tables, publish its scalars
                    if (w > 0) {
                        s_w *= rho64;
                        eos_w *= inv_rho64;
                        lo_a = lo_b;
                        len_a = len_b;
                        y_a = y_b;
                        load_window(w + 1, lo_b, len_b, y_b);
                    }
                    if constexpr (!MARKS) {
                        const double yd = (double)y_a;
                        const double sl = yd * s_w * rho_pow, el = yd * eos_w * inv_rho_pow1;
                        const bool live = w * kWave + lane < n;
                        if constexpr (LOSS == kLossHinge) {
                            sc_tab.zs = sl;
                            sc_tab.cs = live ? el : 0.0;
                        } else {
                            sc_tab.zs = (float)(sl * 1.4426950408889634);
                            sc_tab.cs = live ? (float)el : 0.0f;
                        }
                    }
                }
                // the rows requested now lie kLead steps ahead: in this window while j0 + u + kLead < 64
                const bool ahead_in_next = j0 + kLead >= kWave;
                const int64_t lo_t = ahead_in_next ? lo_b : lo_a;
                const int len_t = ahead_in_next ? len_b : len_a;
                char *sec0 = lds + L::ring + (uint32_t)(i % kSections) * kSectionBytes;
                char *sec = sec0 + lane * 16;
#pragma unroll
                for (int u = 0; u < kG; ++u) {
                    const int slot = HALF * kG + u;
                    const int len = __builtin_amdgcn_readlane(len_a, j0 + u);
                    char *h = sec0 + u * kStepBytes + kRecordBytes;          // the step's scalars
                    if constexpr (MARKS) {
                        // Stamps: the step numbers of the last writes to the two slots of an HBM-resident
                        // column (lanes without one use a slot of their own), read, compared and rewritten
                        // in step order.  What is written does not depend on what was read, so a step's reads
                        // and writes go out back to back and the comparison is made one step later, when the
                        // values have arrived: the wave never waits for LDS.  Chunk 0 holds all HBM-resident
                        // columns of a row unless there are more than 64 (then the others are done on the spot).
                        const int64_t t = i * kG + u;
                        const uint16_t now = (uint16_t)t;
                        const int e0 = lane;
                        const uint32_t col0 = er_col[slot][0];
                        const bool tail0 = e0 < len && col0 >= (uint32_t)kPHead;
                        uint16_t *const pa = reinterpret_cast<uint16_t *>(lds + L::stamp_a) + (tail0 ? stamp_slot_a(col0) : (uint32_t)(kPStamps + e0));
                        uint16_t *const pb = reinterpret_cast<uint16_t *>(lds + L::stamp_b) + (tail0 ? stamp_slot_b(col0) : (uint32_t)(kPStamps + e0));
                        const uint16_t sa = *pa, sb = *pb;
                        *pa = now;
                        *pb = now;
                        bool more = false;           // recent writes to HBM-resident columns outside chunk 0
#pragma unroll
                        for (int c = 1; c < kChunks; ++c) {
                            const int e = c * kWave + lane;
                            const uint32_t col = er_col[slot][c];
                            const bool tl = e < len && col >= (uint32_t)kPHead;
                            if (__builtin_expect(__any(tl), 0)) {
                                uint16_t *const qa = reinterpret_cast<uint16_t *>(lds + L::stamp_a) + (tl ? stamp_slot_a(col) : (uint32_t)(kPStamps + e));
                                uint16_t *const qb = reinterpret_cast<uint16_t *>(lds + L::stamp_b) + (tl ? stamp_slot_b(col) : (uint32_t)(kPStamps + e));
                                const uint16_t ta = *qa, tb = *qb;
                                more |= __any(tl & ((uint16_t)(now - ta) < kRecent) & ((uint16_t)(now - tb) < kRecent));
                                *qa = now;
                                *qb = now;
                            }
                        }
                        // a row too long for the records writes its excess columns without stamps: the steps
                        // that could have fetched such a column early re-read instead
                        if (len > kSlots) redo_until = t + kRecent - 1;
                        const bool forced = more || t <= redo_until;
                        // the verdict on the step before this one (its stamps have arrived by now)
                        if (u > 0) {                 // (a section's last step was settled before its barrier)
                            const bool stale = __any(prev.tail & ((uint16_t)(prev.now - prev.sa) < kRecent) & ((uint16_t)(prev.now - prev.sb) < kRecent)) || prev.forced;
                            if (lane == 0) reinterpret_cast<StepRow *>(prev.h + 16)->pad = stale ? 1 : 0;
                        }
                        prev.tail = tail0; prev.now = now; prev.sa = sa; prev.sb = sb; prev.forced = forced; prev.h = h;
                        if (u == kG - 1) {           // the section's last step is settled before the barrier
                            const bool stale = __any(tail0 & ((uint16_t)(now - sa) < kRecent) & ((uint16_t)(now - sb) < kRecent)) || forced;
                            if (lane == 0) reinterpret_cast<StepRow *>(h + 16)->pad = stale ? 1 : 0;
                        }
                    } else {
                        bool far_tail = false;       // an HBM-resident column outside chunk 0?
#pragma unroll
                        for (int c = 0; c < kChunks; ++c) {
                            const int e = c * kWave + lane;
                            const uint32_t col = er_col[slot][c];
                            const bool in = e < len;
                            const bool is_head = in && col < (uint32_t)kPHead;
                            const bool is_tail = in && col >= (uint32_t)kPHead;
                            if (c > 0) far_tail |= is_tail;
                            pu32x4 rec;
                            rec[0] = er_val[slot][c];
                            rec[1] = is_head ? L::head + col * (uint32_t)sizeof(TV) : L::head_scratch + e * (uint32_t)sizeof(TV);
                            // lanes without an HBM-resident column point past the end of the vector: their
                            // loads return zero and their stores are dropped, so they cause no traffic
                            rec[2] = is_tail ? col * (uint32_t)sizeof(TV) : 0xFFFFFFF0u;
                            rec[3] = is_tail ? 0x80000000u : 0u;
                            *reinterpret_cast<pu32x4 *>(sec + u * kStepBytes + c * (kWave * 16)) = rec;
                        }
                        const bool wide = __any(far_tail);
                        if (lane == j0 + u) {        // the lane that holds this step's scalars publishes them
                            *reinterpret_cast<StepScalars<TV> *>(h) = sc_tab;
                            reinterpret_cast<StepRow *>(h + 16)->lo = lo_a;
                            reinterpret_cast<StepRow *>(h + 16)->len = len_a | (wide ? kWideTail : 0);
                        }
                    }
                    const int jj = (j0 + u + kLead) & (kWave - 1);
                    request(slot, lane_read_i64(lo_t, jj), __builtin_amdgcn_readlane(len_t, jj));
                }
            };
            for (int64_t i = 0; i <= ngroups; i += 2) {
                write_group(i, std::integral_constant<int, 0>{});
                wait_lds_then_barrier();
                if (i + 1 <= ngroups) {
                    write_group(i + 1, std::integral_constant<int, 1>{});
                    wait_lds_then_barrier();
                }
            }
        };
        if (wave == 1) scout(std::false_type{});
        else scout(std::true_type{});
    } else {
        // ------------------------------------------------------------------------- worker
        const __amdgpu_buffer_rsrc_t vres =
            __builtin_amdgcn_make_buffer_rsrc(v, 0, (int)(uint32_t)(d * (int64_t)sizeof(TV)), 0x00020000);
        const pu32x4 vdesc = descriptor(v, (uint32_t)(d * (int64_t)sizeof(TV)));
        pu32x4 rec[kG][kChunks];
        TV vr[kG];                    // HBM-resident values of chunk 0 (the other chunks hold none, or the step is flagged)
        StepScalars<TV> scr[kG];
        int lenr[kG], staler[kG];
        const char *ring0 = lds + L::ring;
        const char *ring = ring0 + lane * 16;

        wait_lds_then_barrier();      // section 0 written
        wait_lds_then_barrier();      // section 1 written
#pragma unroll
        for (int q = 0; q <= kTQ; ++q)
#pragma unroll
            for (int c = 0; c < kChunks; ++c)
                rec[q][c] = *reinterpret_cast<const pu32x4 *>(ring + q * kStepBytes + c * (kWave * 16));
#pragma unroll
        for (int q = 0; q <= kTQ; ++q) {
            scr[q] = *reinterpret_cast<const StepScalars<TV> *>(ring0 + q * kStepBytes + kRecordBytes);
            lenr[q] = reinterpret_cast<const StepRow *>(ring0 + q * kStepBytes + kRecordBytes + 16)->len;
            staler[q] = reinterpret_cast<const StepRow *>(ring0 + q * kStepBytes + kRecordBytes + 16)->pad;
        }
#pragma unroll
        for (int q = 0; q < kTQ; ++q) vr[q] = load_state(vres, rec[q][0][2], TV{});
        __builtin_amdgcn_s_waitcnt(0x0F70);      // enter the loop with an empty queue

        for (int64_t g = 0; g < ngroups; ++g) {
            if (g > 0) wait_lds_then_barrier();  // section g+1 written
            const uint32_t off_cur = (uint32_t)(g % kSections) * kSectionBytes;
            const uint32_t off_nxt = (uint32_t)((g + 1) % kSections) * kSectionBytes;
#pragma unroll
            for (int u = 0; u < kG; ++u) {
                const int64_t t = g * kG + u;
                const char *hdr_t = ring0 + off_cur + u * kStepBytes + kRecordBytes;      // scalars of step t
                // Model values and stamps of step t first: they queue right behind the previous
                // step's LDS writes and everything below waits for them.
                TV hv[kChunks];
#pragma unroll
                for (int c = 0; c < kChunks; ++c) hv[c] = *reinterpret_cast<const TV *>(lds + rec[u][c][1]);
                {   // records and scalars of step t+kTQ+1
                    const int uu = u + kTQ + 1;
                    const uint32_t src = (uu < kG ? off_cur : off_nxt) + (uu % kG) * kStepBytes;
#pragma unroll
                    for (int c = 0; c < kChunks; ++c)
                        rec[uu % kG][c] = *reinterpret_cast<const pu32x4 *>(ring + src + c * (kWave * 16));
                    scr[uu % kG] = *reinterpret_cast<const StepScalars<TV> *>(ring0 + src + kRecordBytes);
                    lenr[uu % kG] = reinterpret_cast<const StepRow *>(ring0 + src + kRecordBytes + 16)->len;
                    staler[uu % kG] = reinterpret_cast<const StepRow *>(ring0 + src + kRecordBytes + 16)->pad;
                }
                // (Steps past the chain's end run like any other: their step scalar is zero, so they write
                // back what they read.  A branch around them would keep the compiler from moving the reads
                // above to the front of the step.)
                {
                    const StepScalars<TV> sc = scr[u];
                    const int len_word = __builtin_amdgcn_readfirstlane(lenr[u]);
                    const int len = len_word & (kWideTail - 1);
                    const bool wide = (len_word & kWideTail) != 0;
                    TV vv[kChunks];
                    float val[kChunks];
                    bool tail[kChunks];
#pragma unroll
                    for (int c = 0; c < kChunks; ++c) {
                        const pu32x4 r = rec[u][c];
                        val[c] = __uint_as_float(r[0]);
                        tail[c] = (int32_t)r[3] < 0;
                        vv[c] = hv[c];
                    }
                    vv[0] = tail[0] ? vr[u] : hv[0];
                    if (__builtin_expect(__builtin_amdgcn_readfirstlane(staler[u]) != 0, 0)) {      // (the scout's verdict) drain, then read this step's HBM-resident values again
                        const TV fresh = drained_buffer_load(vdesc, rec[u][0][2], TV{});
                        if (tail[0]) vv[0] = fresh;
                    }
                    if (__builtin_expect(wide, 0)) {        // more than 64 HBM-resident columns: the others are read here, after everything before
#pragma unroll
                        for (int c = 1; c < kChunks; ++c) {
                            const TV fresh = drained_buffer_load(vdesc, rec[u][c][2], TV{});
                            if (tail[c]) vv[c] = fresh;
                        }
                    }
                    TV acc = (TV)0;
#pragma unroll
                    for (int c = 0; c < kChunks; ++c) acc += vv[c] * (TV)val[c];
                    if (__builtin_expect(len > kSlots, 0)) {             // the rest of a very long row, one entry per lane at a time
                        const int64_t lo = reinterpret_cast<const StepRow *>(hdr_t + 16)->lo;
                        for (int e0 = 0; e0 < len - kSlots; e0 += kWave) {      // (the records hold the row's last kSlots entries)
                            const int e = e0 + lane;
                            const bool in = e < len - kSlots;
                            const uint32_t xc = drained_global_load_u32(a.col_idx + (in ? lo + e : lo));
                            const float xv = __uint_as_float(drained_global_load_u32(a.vals + (in ? lo + e : lo)));
                            const bool hd = xc < (uint32_t)kPHead;
                            const TV cur = (in && hd) ? head[xc]
                                                      : drained_buffer_load(vdesc, in ? xc * (uint32_t)sizeof(TV) : 0xFFFFFFF0u, TV{});
                            if (in) acc += cur * (TV)xv;
                        }
                    }
                    TV coef;
                    if constexpr (LOSS == kLossHinge) {
                        coef = lane63_below_one(sc.zs, wave_sum_lane63(acc)) ? sc.cs : 0.0;
                    } else {
                        acc = wave_sum(acc);
                        coef = sc.cs * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc.zs * acc));
                    }
#pragma unroll
                    for (int c = 0; c < kChunks; ++c) {
                        const pu32x4 r = rec[u][c];
                        const TV nv = vv[c] + coef * (TV)val[c];
                        *reinterpret_cast<TV *>(lds + r[1]) = nv;
                        if (c == 0) store_state(vres, r[2], nv);
                        else if (__builtin_expect(wide, 0)) drained_buffer_store(vdesc, r[2], nv);
                    }
                    if (__builtin_expect(len > kSlots, 0)) {
                        const int64_t lo = reinterpret_cast<const StepRow *>(hdr_t + 16)->lo;
                        for (int e0 = 0; e0 < len - kSlots; e0 += kWave) {
                            const int e = e0 + lane;
                            const bool in = e < len - kSlots;
                            const uint32_t xc = drained_global_load_u32(a.col_idx + (in ? lo + e : lo));
                            const float xv = __uint_as_float(drained_global_load_u32(a.vals + (in ? lo + e : lo)));
                            if (in && xc < (uint32_t)kPHead) {
                                head[xc] += coef * (TV)xv;
                            } else {
                                const uint32_t off = in ? xc * (uint32_t)sizeof(TV) : 0xFFFFFFF0u;      // (past the end: no access)
                                const TV cur = drained_buffer_load(vdesc, off, TV{});
                                drained_buffer_store(vdesc, off, in ? cur + coef * (TV)xv : cur);
                            }
                        }
                    }
                }
                // HBM-resident values of step t+kTQ (its records arrived one step ago)
                vr[(u + kTQ) % kG] = load_state(vres, rec[(u + kTQ) % kG][0][2], TV{});
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);      // all stores done before the vector is read back
    }
    __syncthreads();

    // the columns kept in LDS go back to the vector in the workspace
    for (int c = tid; c < kPHead && c < d; c += kPairThreads) v[c] = head[c];
}

// Before the chains: every chain's vector in the workspace starts as the common start vector (or
// zero).  Grid row y is chain row0 + y; the workgroups of a row share its columns.
template <typename TV>
__global__ __launch_bounds__(256) void csr_state_start_kernel(TV *state, const float *w_start, int64_t d, int row0)
{
    TV *v = state + (int64_t)(row0 + (int)blockIdx.y) * d;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < d; c += (int64_t)gridDim.x * 256)
        v[c] = w_start ? (TV)w_start[c] : (TV)0;
}

// After the chains: W[chain,:] = (1-eta*lambda)^n * v, the lazy scale applied once, in fp64.  Grid row
// y is the chain that workgroup row0 + y of the chain kernel ran.
template <typename TV>
__global__ __launch_bounds__(256) void csr_state_finish_kernel(const TV *state, float *W, const int32_t *order,
                                                                const int64_t *nsteps, double rho, int64_t d, int row0)
{
    const int b = row0 + (int)blockIdx.y;
    const int chain = order[b];
    double s_end = 1.0, p = rho;
    for (int64_t e = nsteps[b]; e > 0; e >>= 1) {       // (uniform over the workgroup)
        if (e & 1) s_end *= p;
        p *= p;
    }
    const TV *v = state + (int64_t)chain * d;
    float *out = W + (int64_t)chain * d;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < d; c += (int64_t)gridDim.x * 256)
        out[c] = (float)(s_end * (double)v[c]);
}

template <typename TV, int LOSS>
static hipError_t launch_pair(const ChainArgs &a, hipStream_t s)
{
    TV *state = static_cast<TV *>(a.state);
    constexpr int kRows = 32768;                // chains per launch of the start and finish kernels (a grid's y extent is 16 bits)
    // enough workgroups per chain to fill the device, not more than a chain has 256-column strips
    const int rows_at_once = a.k < kRows ? a.k : kRows;
    const unsigned across = (unsigned)std::max<int64_t>(1, std::min<int64_t>((a.d + 255) / 256, (4096 + rows_at_once - 1) / rows_at_once));
    for (int row0 = 0; row0 < a.k; row0 += kRows) {
        const unsigned rows = (unsigned)std::min(kRows, a.k - row0);
        hipLaunchKernelGGL((csr_state_start_kernel<TV>), dim3(across, rows), dim3(256), 0, s, state, a.w_start, a.d, row0);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((chain_csr_pair_kernel<LOSS>), dim3(a.k), dim3(kPairThreads), 0, s, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int row0 = 0; row0 < a.k; row0 += kRows) {
        const unsigned rows = (unsigned)std::min(kRows, a.k - row0);
        hipLaunchKernelGGL((csr_state_finish_kernel<TV>), dim3(across, rows), dim3(256), 0, s, state, a.W, a.order, a.nsteps, a.rho,
                           a.d, row0);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_csr_pair(const Plan &p, const ChainArgs &a, hipStream_t s)
{
    return p.loss == WPSGD_HINGE ? launch_pair<double, kLossHinge>(a, s) : launch_pair<float, kLossLogistic>(a, s);
}

}  // namespace wpsgd
