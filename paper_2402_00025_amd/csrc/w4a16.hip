// Kernels and C ABI of the fused W4A16 skinny GEMM for gfx950.  See include/w4a16.h for the
// contract and w4a16_device.hpp for the per-wave routines.
//
// Paper: "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference with SplitK work
// decomposition".  Algorithm 1 is the SplitK kernel; Section 3 (first paragraph) describes the
// data-parallel tiling it is compared with; Section 2.1 the atomic reduction.
#include "w4a16_device.hpp"
#include "w4a16_stream.hpp"

#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "../../include/w4a16.h"

namespace w4a16 {

struct GemmArgs {
    // what every wave needs before its first load, packed at the front so that it arrives with
    // one batch of scalar loads
    const _Float16* A;
    const uint32_t* qweight;
    const _Float16* scales;
    const uint32_t* qzeros;
    _Float16* C;
    float* scratch;     // split-k: fp32 sums [16, n] (atomic) or partial tiles [split_k, m, n] (workspace)
    int m, n, k;
    int tiles;            // column tiles = ceil(n / (16 V))
    int split_k;
    // The compute groups (32 * IPG consecutive k each) are dealt to the split_k * waves k parts
    // in order: part i = slice * waves + wave gets groups_base of them, the first groups_rem
    // parts one more (k need not divide evenly; every part stays a whole number of groups).
    int groups_base;
    int groups_rem;
    int param_shift;      // log2(compute groups per quantisation group)
    int lds_wave_bytes;   // LDS region of one wave
    int waves;            // working waves per workgroup (the launch has one more in service mode)
    int spin_limit;     // phase mode: bound on polls of a flag
    int probe_delay;    // phase mode: 64-cycle sleeps before the early sample of the flag
    uint32_t* tickets;  // split-k: one arrival counter per column tile
    uint32_t* flags;    // phase mode: zeroings so far, per tile origin
    uint32_t* counts;   // phase mode: calls so far, per (tile origin, slice)
    uint32_t* errors;   // phase mode: count of waits that ran out
    uint32_t* err_host; // phase mode: word in pinned host memory set to 1 by a wait that ran out (may be null)
};

enum : int {
    kDirect = 0, kAtomicF32 = 1, kAtomicPkF16 = 2, kWorkspace = 3, kAtomicFixed = 4, kAtomicPkF16Phase = 5,
    kAtomicPkF16Service = 6  // the phase protocol run by one extra wavefront per workgroup (internal)
};

// kAtomicFixed: one 64-bit integer atomic add per output element and workgroup.
//   bits 58..63  arrivals before this one (0..63: split_k <= 64; the last add may carry out of
//                the word, which is then reset anyway)
//   bits 52..57  how many of the contributions so far were NaN (they add nothing to the sum)
//   bits  0..51  sum of (partial * 2^28 + 2^45): fixed point, biased so it never goes negative;
//                every term is below 2^46 (|partial| is clamped below 2^17, beyond fp16's range),
//                so 64 of them stay below 2^52.  2^-28 resolves every product of an fp16 value
//                with a small integer exactly and is finer than the fp32 partial sums' own
//                last place from 1/16 on.
// The add returns the previous word, so the workgroup that sees split_k - 1 earlier arrivals
// holds the complete sum (previous + its own) and finishes the element: one memory round trip,
// no separate ticket, and a sum that does not depend on arrival order (integer addition).  A NaN
// among the partial sums makes the result NaN, as with every other reduction; an infinite or
// huge one is clamped and comes out as an fp16 infinity.
constexpr int kFixedFracBits = 28;
constexpr uint64_t kFixedBias = 1ull << 45;
constexpr int kFixedNanShift = 52;
constexpr int kFixedArrivalShift = 58;
constexpr uint64_t kFixedArrival = 1ull << kFixedArrivalShift;
constexpr uint64_t kFixedSumMask = (1ull << kFixedNanShift) - 1;
constexpr uint64_t kFixedNanMask = (kFixedArrival - 1) & ~kFixedSumMask;
constexpr float kFixedClamp = 131071.0f;  // |partial| < 2^17 keeps partial * 2^28 inside the bias

__device__ __forceinline__ uint64_t fixed_contribution(float v)
{
    const bool nan = v != v;
    v = nan ? 0.f : fminf(fmaxf(v, -kFixedClamp), kFixedClamp);
    const long long q = __double2ll_rn((double)v * (double)(1ull << kFixedFracBits));
    return (uint64_t)(q + (long long)kFixedBias) + kFixedArrival + (nan ? 1ull << kFixedNanShift : 0ull);
}

// The total of the word before the last add (`old`) and the last contribution (`mine`); the
// fields are read from each on its own, so a NaN count of 64 cannot wrap to "none".
__device__ __forceinline__ float fixed_total(uint64_t old, uint64_t mine, int split_k)
{
    const long long q =
        (long long)((old & kFixedSumMask) + (mine & kFixedSumMask)) - (long long)split_k * (long long)kFixedBias;
    const float sum = (float)((double)q * (1.0 / (double)(1ull << kFixedFracBits)));
    return ((old | mine) & kFixedNanMask) ? __builtin_nanf("") : sum;
}

// After `old = fetch_add(word, mine)`: if this was the last of split_k arrivals, returns true
// with the total in *total and resets the word to zero for the next call.
__device__ __forceinline__ bool fixed_finish(uint64_t* word, uint64_t old, uint64_t mine, int split_k, float* total)
{
    if ((int)(old >> kFixedArrivalShift) != split_k - 1) return false;
    *total = fixed_total(old, mine, split_k);
    __hip_atomic_store(word, (uint64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Results and protocol words are stored write-through (the sc1 bit of a buffer store, an
// agent-scope atomic store elsewhere).  A plain store leaves a dirty line in the die's L2 that
// the release at the end of the kernel has to find and write back: 0.16 us per launch on the
// headline shape for a single dirty word per workgroup, which is as much as the whole sum over
// the waves costs.  Written through, nothing is dirty when the kernel ends.
constexpr int kWriteThrough = 16;  // aux bits of a buffer store: sc1

__device__ __forceinline__ void store_through(uint32_t* word, uint32_t value)
{
    __hip_atomic_store(word, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t pack_half2(float lo, float hi)
{
    const half2_t h = {(_Float16)lo, (_Float16)hi};  // v_cvt_f16_f32: round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// Everything this thread has sent to memory (atomics, write-through stores) has been performed
// before it goes on.  On gfx9-family hardware the vector memory counter also covers stores and
// atomics without return.  The "memory" clobber keeps the compiler from moving accesses across.
__device__ __forceinline__ void wait_memory_ops() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// A wait of the phase protocol ran out (one lane calls this): count it, raise the sticky word the
// host looks at before its next call, and add NaN to the first column pair of the tile, so that
// the output cannot pass for a result.  `c_off` is a byte offset inside C.
__device__ __forceinline__ void phase_wait_failed(uint32_t* errors, uint32_t* err_host, rsrc_t rs_c, uint32_t c_off)
{
    __hip_atomic_fetch_add(errors, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (err_host) __hip_atomic_store(err_host, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    const half2_t poison = {(_Float16)__builtin_nanf(""), (_Float16)__builtin_nanf("")};
    __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(poison, rs_c, c_off, 0, 0);
}

// One workgroup = WAVES wavefronts that share one output tile [m, 16 V] and divide the
// workgroup's k range between them; blockIdx = (tile, slice), dispatched as slice * tiles + tile.
//
// MODE kDirect       the workgroup owns the tile alone (data-parallel kernel, or split_k == 1):
//                    its sum is rounded once to fp16 and stored.
// MODE kAtomicF32    Algorithm 1's final step with fp32 atomic adds into scratch; the workgroup
//                    that arrives last at the tile's ticket swaps the sums out (leaving zeros
//                    for the next call), rounds once and stores C.
// MODE kAtomicPkF16  packed-fp16 atomic adds straight into a C that a fill kernel zeroed.
// MODE kWorkspace    partial tiles are written through to memory; the last workgroup adds them
//                    in slice order (bit-reproducible).
// MODE kAtomicFixed  64-bit fixed-point atomic adds that also count arrivals (see above);
//                    bit-reproducible, one round trip.
// MODE kAtomicPkF16Phase  packed-fp16 atomic adds straight into C with no launch before this one:
//                    the slice-0 workgroup of a tile zeroes the tile as its first action and
//                    publishes that in the tile's flag; the others add once they have seen it.
//
// Synchronisation of the ticketed modes.  Every access that one workgroup makes and another
// reads is a device-scope atomic operation (add, exchange, write-through store, cache-bypassing
// load), so it is performed at the level where all compute dies see it; none of it sits dirty
// in a die-local L2.  What is left to order is time: a workgroup waits until its own
// contributions have been performed (wait_memory_ops + barrier) before one of its threads takes
// the ticket, and the last workgroup reads only after its ticket came back.  A device-scope
// release fence would do the same but also write back the whole L2 of the die, which costs
// more than the GEMM itself.
//
// The phase protocol (kAtomicPkF16Phase) uses no atomic operation besides the adds into C
// (atomics of several workgroups on one word are served one after the other, at about a
// memory round trip each).  State, per split_k and per tile origin e = n0 / 16:
//   counts[e][slice]  how many calls this (tile, slice) workgroup has run; only it writes it
//   flags[e]          how many times the tile has been zeroed; only the slice-0 workgroup writes it
// Every call that touches a tile runs all split_k of its workgroups, so before a call these
// words are all equal (= c) and after it all are c + 1.  Wave 0 of the slice-0 workgroup stores
// zeros (write-through) to the tile before it issues any load.  Then wave 0 of every workgroup
// loads its own count c.  Vector memory operations of a wave complete in issue order, so when c
// has arrived the zeros are in memory: the slice-0 workgroup stores c + 1 into flags[e] (and every
// workgroup stores c + 1 into its own count).  Every wave samples flags[e] during its last
// compute group and, after the workgroup's barrier, adds only when it has seen c + 1; otherwise
// it polls (bounded by spin_limit; a wait that runs out is counted in `errors` and the wave goes
// on).  The slice-0 workgroup never waits for anyone and has the lowest block index of the
// tile's workgroups, so the wait ends.
// MODE kAtomicPkF16Service is the same protocol with the roles moved out of the working waves:
// the workgroup has one wavefront more, which stores the zeros (slice 0), loads the count,
// publishes, samples the flag until it has seen this call's value, and only then joins the
// workgroup's barrier.  The working waves neither issue the protocol's memory operations (whose
// in-order completion would hold back their weight data) nor look at the flag: passing the
// barrier means the zeros are in memory.  Used where a wave needs few registers (one compute
// group per wave), so that the extra wave costs no occupancy.
// WMAX (4 or 16) is the largest number of working waves the instantiation may be launched with;
// the small one lets the compiler use more than 128 registers per lane.
constexpr int kPhaseMaxSplit = 64;          // largest split_k of the phase protocol
constexpr uint32_t kPhaseOrigins = 1u << 12;  // tile origins n0 / 16 it covers: n <= 65536

// GC: 1 = every wave has exactly one compute group, 2 = at least two, 0 = decided at run time.
// BITS: width of the packed fields, 4 (the paper's), 2, 3 or 8 (Section 2: the method carries
// over to other n-bit schemes; qweight is then int32 [k BITS / 32, n] and qzeros int32
// [k / g, n BITS / 32]; 3-bit fields: 32 of them in a stream of three words).
// NS: strips of 16 V columns per wave.  2 (only with GC = 1): the wave multiplies the same
// activations with the weights of two adjacent strips, which halves the activation traffic per
// weight byte and the number of waves.
template <int V, int IPG, int MODE, int WMAX, int GC, int BITS = 4, int NS = 1>
__device__ __forceinline__ void gemm_body(const GemmArgs& p)
{
    static_assert(NS == 1 || (NS == 2 && GC == 1), "two strips per wave: one compute group per wave");
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    constexpr int BN = 16 * V * NS;
    constexpr bool kService = MODE == kAtomicPkF16Service;

    const int tid = threadIdx.x;
    const int nthreads = p.waves * kWave;  // threads of the working waves (not read from the launch: an argument arrives with the others)
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // uniform: keeps offsets scalar
    const int waves = nthreads / kWave;
    // grid = (tiles, split_k): the same dispatch order as slice * tiles + tile, without a division
    // at the head of every wave
    const int tile = blockIdx.x;
    const int slice = blockIdx.y;
    const int n0 = tile * BN;
    const int m = p.m, n = p.n, k = p.k;
    // (the host has checked the shape: divisions by constants become single shifts)
    __builtin_assume(m > 0 && n > 0 && k > 0);

    if constexpr (kService) {
        if (wave == waves) {
            // ---- the service wave (see the protocol above)
            constexpr uint32_t kOutside = 0xFFFFFF00u;
            const uint32_t origin_s = (uint32_t)n0 / 16u;
            const rsrc_t rs_c = make_rsrc(p.C, (uint32_t)m * (uint32_t)n * 2u);
#pragma unroll
            for (int i = 0; i < 2 * NS; ++i) {
                const int u = lane + kWave * i;
                const int row = u / (BN / 8), col = n0 + 8 * (u % (BN / 8));
                const bool inside = slice == 0 && row < m && col < n;
                const uint32_t off = inside ? ((uint32_t)row * (uint32_t)n + (uint32_t)col) * 2u : kOutside;
                __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{0u, 0u, 0u, 0u}, rs_c, off, 0, 16);
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            uint32_t* my_count = p.counts + origin_s * (uint32_t)p.split_k + (uint32_t)slice;
            uint32_t count_s = *(volatile uint32_t*)my_count;  // issued after the stores: its arrival means they are done
            asm volatile("" : "+v"(count_s)::"memory");
            const uint32_t now = __builtin_amdgcn_readfirstlane(count_s) + 1u;
            if (lane == 0) {
                store_through(my_count, now);
                if (slice == 0)
                    __hip_atomic_store(p.flags + origin_s, now, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            uint32_t seen = now - 1u;
            int polls = 0;
            do {
                for (int i = 0; i < p.probe_delay; ++i) __builtin_amdgcn_s_sleep(1);
                seen = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(p.flags + origin_s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                ++polls;
            } while (seen != now && polls < p.spin_limit);
            if (seen != now && lane == 0) phase_wait_failed(p.errors, p.err_host, rs_c, (uint32_t)n0 * 2u);
            __syncthreads();  // the working waves' one barrier
            return;
        }
    }

    // ---- phase protocol, first part (wave 0): the zeros of slice 0, then this workgroup's call
    // count.  Buffer instructions whose offset lies outside the buffer are dropped by the
    // hardware, so the lanes and waves that take no part get such an offset instead of a branch:
    // the count stays an ordinary value that is waited for only where it is used.
    uint32_t count = 0, early = 0;
    const uint32_t origin = (uint32_t)n0 / 16u;
    if constexpr (MODE == kAtomicPkF16Phase) {
        constexpr uint32_t kOutside = 0xFFFFFF00u;
        // 16-byte units of the tile: unit u = (row, 8 columns); n % 8 == 0 keeps a unit either
        // inside or outside the matrix.  m * BN / 8 <= 128 units: two per lane of wave 0.
        const rsrc_t rs_c = make_rsrc(p.C, (uint32_t)m * (uint32_t)n * 2u);
        const bool zeroer = slice == 0 && wave == 0;
#pragma unroll
        for (int i = 0; i < 2 * NS; ++i) {
            const int u = lane + kWave * i;
            const int row = u / (BN / 8), col = n0 + 8 * (u % (BN / 8));
            const bool inside = zeroer && row < m && col < n;
            const uint32_t off = inside ? ((uint32_t)row * (uint32_t)n + (uint32_t)col) * 2u : kOutside;
            // aux 16 = sc1: written through to memory, where every compute die sees it
            __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{0u, 0u, 0u, 0u}, rs_c, off, 0, 16);
        }
        // the count is the first load after the zero stores, and no load is issued ahead of it
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        const rsrc_t rs_counts = make_rsrc(p.counts, kPhaseOrigins * (uint32_t)p.split_k * 4u);
        count = __builtin_amdgcn_raw_buffer_load_b32(
            rs_counts, wave == 0 ? (origin * (uint32_t)p.split_k + (uint32_t)slice) * 4u : kOutside, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

    const LaneMap lm = make_lane_map<V, BITS>(lane, n0, m, n, k);
    const uint32_t qgroups = (uint32_t)(k / (32 * IPG)) >> p.param_shift;
    Tensors tensors;
    tensors.A = make_rsrc(p.A, (uint32_t)m * (uint32_t)k * 2u);
    // (k and n times BITS / 32, written per width so that each keeps its shortest form; 3-bit: k, n % 32 == 0)
    constexpr int kFields = BITS == 3 ? 1 : 32 / BITS;
    tensors.qweight = make_rsrc(p.qweight, (uint32_t)(BITS == 3 ? k / 32 * 3 : k / kFields) * (uint32_t)n * 4u);
    tensors.scales = make_rsrc(p.scales, qgroups * (uint32_t)n * 2u);
    tensors.qzeros = make_rsrc(p.qzeros, qgroups * (uint32_t)(BITS == 3 ? n / 32 * 3 : n / kFields) * 4u);
    tensors.m = m;
    tensors.n = n;
    tensors.k = k;
    tensors.param_shift = p.param_shift;

    float4_t acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int part = slice * p.waves + wave;
    const int g_begin = part * p.groups_base + (part < p.groups_rem ? part : p.groups_rem);
    const int g_count = p.groups_base + (part < p.groups_rem ? 1 : 0);
    // LDS: [0] the flag value this call waits for, [1] wave 0's early sample of the flag; from byte 16 on one [m][BN] fp32 tile per wave
    uint32_t* lds_phase = (uint32_t*)lds_raw;
    char* lds_tiles = lds_raw + 16;
    FlagProbe probe;
    probe.addr = p.flags + origin;
    probe.value = 0;
    Ring<V, IPG, BITS> ring;
    wave_prime<V, IPG, GC, BITS>(ring, tensors, lm, g_begin, g_count, [&]() {
        if constexpr (MODE == kAtomicPkF16Phase) {
            if (wave == 0) {
                // wait for the count (the asm makes it a used value here)
                asm volatile("" : "+v"(count)::"memory");
                const uint32_t now = __builtin_amdgcn_readfirstlane(count) + 1u;
                if (lane == 0) {
                    lds_phase[0] = now;
                    store_through(p.counts + origin * (uint32_t)p.split_k + (uint32_t)slice, now);
                    if (slice == 0)
                        __hip_atomic_store(p.flags + origin, now, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                // Early sample of the flag for the whole workgroup.  The slice-0 workgroup of
                // the tile publishes at about this moment, so the sample is taken a little
                // later; this wave has nothing to do but wait for its weights anyway.  A sample
                // that comes too early only means that the late sample below is used instead.
                for (int i = 0; i < p.probe_delay; ++i) __builtin_amdgcn_s_sleep(1);
                early = __hip_atomic_load(p.flags + origin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    });
    // second strip: its parameters and weights are requested behind the first strip's, so they
    // arrive while the first strip is being computed; the activations are the first strip's
    Ring<V, IPG, BITS> ring1;
    float4_t acc1[V];
    if constexpr (NS == 2) {
        const LaneMap lm1 = make_lane_map<V, BITS>(lane, n0 + 16 * V, m, n, k);
        issue_params<V, BITS>(ring1.par[0], lm1, tensors, g_begin);
#pragma unroll
        for (int it = 0; it < IPG; ++it)
        {
            if constexpr (BITS == 4)
                ring1.step[0][it].w.load(tensors.qweight, lm1.off_w, ((uint32_t)g_begin * IPG + it) * 16u * (uint32_t)n);
            else
                issue_step_weights<V, BITS>(ring1.step[0][it], lm1, tensors, (uint32_t)g_begin * IPG + it);
        }
#pragma unroll
        for (int j = 0; j < V; ++j) acc1[j] = float4_t{0.f, 0.f, 0.f, 0.f};
        wave_run<V, IPG, MODE == kAtomicPkF16Phase, GC, BITS>(ring, tensors, lm, g_begin, g_count, acc, probe);
#pragma unroll
        for (int it = 0; it < IPG; ++it) ring1.step[0][it].a = ring.step[0][it].a;
        FlagProbe none{nullptr, 0};
        if constexpr (BITS == 8)
            compute_group<V, IPG, 0, false, false, BITS>(ring1, lm1, tensors, magic_64x4(), 0, acc1, none);
        else
            compute_group<V, IPG, 0, false, false, BITS>(ring1, lm1, tensors, magic_1024x2(), 0, acc1, none);
    } else {
        wave_run<V, IPG, MODE == kAtomicPkF16Phase, GC, BITS>(ring, tensors, lm, g_begin, g_count, acc, probe);
    }

    if constexpr (MODE == kAtomicPkF16Phase) {
        if (wave == 0 && lane == 0) lds_phase[1] = early;
    }

    // ---- two strips per wave, four waves (the launch the plan uses): the sum over the waves and
    // the adds into C in as few instructions as possible behind the barrier, because one wave per
    // SIMD runs them with nothing to overlap them with.  Every wave writes its whole [16][128]
    // tile (rows >= m hold copies of row m - 1 and are never added); thread t then owns the column
    // pair 2 (t % 64) of rows t / 64 + 4 i, i = 0..3: eight bytes at 8 t + 2048 i of every wave's
    // tile, so all sixteen reads share one address register, and consecutive lanes add to
    // consecutive words of one row of C.  The offsets into C are worked out before the barrier
    // (the asm pins them there); rows >= m and columns >= n get an offset outside the buffer.
    if constexpr (NS == 2 && kService) {
        if (waves == 4) {
            constexpr int kTileBytes = 16 * BN * 4;
            constexpr uint32_t kOutside = 0xFFFFFF00u;
            char* mine = lds_tiles + wave * kTileBytes + ((4 * (lane >> 4)) * BN + V * (lane & 15)) * 4;
            uint32_t their_offset = 8u * (uint32_t)tid;
            const rsrc_t rs_c = make_rsrc(p.C, (uint32_t)m * (uint32_t)n * 2u);
            const int col = n0 + 2 * (tid & 63);
            uint32_t off[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (tid >> 6) + 4 * i;
                off[i] = (row < m && col < n) ? ((uint32_t)row * (uint32_t)n + (uint32_t)col) * 2u : kOutside;
            }
            asm volatile("" : "+v"(off[0]), "+v"(off[1]), "+v"(off[2]), "+v"(off[3]), "+v"(their_offset));
            const char* theirs = lds_tiles + their_offset;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                *(float4_t*)(mine + r * BN * 4) = float4_t{acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
                *(float4_t*)(mine + r * BN * 4 + 16 * V * 4) = float4_t{acc1[0][r], acc1[1][r], acc1[2][r], acc1[3][r]};
            }
            __syncthreads();
            float2 part[4][4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) part[i][q] = *(const float2*)(theirs + q * kTileBytes + i * 2048);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float sx = (part[i][0].x + part[i][1].x) + (part[i][2].x + part[i][3].x);
                const float sy = (part[i][0].y + part[i][1].y) + (part[i][2].y + part[i][3].y);
                const half2_t h = {(_Float16)sx, (_Float16)sy};
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(h, rs_c, off[i], 0, 0);
            }
            return;
        }
    }

    // ---- sum the waves' tiles through LDS.  acc[j][r] is row 4*(lane/16)+r, column V*(lane%16)+j.
    float* red = (float*)(lds_tiles + wave * p.lds_wave_bytes);  // [m][BN]
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * (lane >> 4) + r;
        if (row < m) {
            float* dst = red + row * BN + V * (lane & 15);
            if constexpr (NS == 2) {
                static_assert(NS == 1 || V == 4, "two strips per wave: 128-bit loads");
                *(float4_t*)(dst + 16 * V) = float4_t{acc1[0][r], acc1[1][r], acc1[2][r], acc1[3][r]};
            }
            if constexpr (V == 4) {
                *(float4_t*)dst = float4_t{acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
            } else if constexpr (V == 2) {
                *(float2*)dst = float2{acc[0][r], acc[1][r]};
            } else {
                *dst = acc[0][r];
            }
        }
    }

    // A unit is one element (modes whose atomics are per element) or two adjacent columns.
    // Consecutive threads take consecutive units, so an atomic instruction of a wave touches the
    // fewest cache lines (the L2 charges atomics per line).  A thread's first two units are
    // handled in straight-line code whose addresses are worked out before the barrier and whose
    // LDS reads (two units x up to four waves) are in flight together; the modes that write C
    // itself use buffer instructions, which drop lanes whose offset lies outside the buffer, so
    // there is no branch between the barrier and the adds.  Further units (few threads, many
    // rows) go through the loop behind.
    constexpr int EPU = (MODE == kAtomicF32 || MODE == kAtomicFixed) ? 1 : 2;
    constexpr bool kBufferOut =
        MODE == kDirect || MODE == kAtomicPkF16 || MODE == kAtomicPkF16Phase || MODE == kAtomicPkF16Service;
    constexpr uint32_t kOutsideC = 0xFFFFFF00u;
    const int units = m * BN / EPU;
    const int wave_floats = p.lds_wave_bytes / 4;
    const float* red0 = (const float*)lds_tiles;
    const rsrc_t rs_out = make_rsrc(p.C, (uint32_t)m * (uint32_t)n * 2u);

    struct Unit {
        bool ok;        // inside the tile and the matrix
        int lds;        // float index inside a wave's tile
        int row, col;
        uint32_t off;   // byte offset into C, or kOutsideC
    };
    auto make_unit = [&](int u) {
        Unit x;
        const int uc = u < units ? u : 0;
        const int e = uc * EPU;
        x.lds = e;
        x.row = e / BN;
        x.col = n0 + e % BN;
        x.ok = u < units && x.col < n;
        x.off = x.ok ? ((uint32_t)x.row * (uint32_t)n + (uint32_t)x.col) * 2u : kOutsideC;
        return x;
    };
    // `base` = wave index of the first of four tiles to read; tiles past the last wave are read
    // from the last wave (a valid address) and left out of the sum
    auto read_unit = [&](const Unit& x, int base, float (&v)[4][EPU]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int wq = base + q < waves ? base + q : waves - 1;
            const float* src = red0 + wq * wave_floats + x.lds;
            if constexpr (EPU == 2) {
                const float2 t2 = *(const float2*)src;
                v[q][0] = t2.x;
                v[q][1] = t2.y;
            } else {
                v[q][0] = *src;
            }
        }
    };
    auto add_unit = [&](int base, const float (&v)[4][EPU], float (&sum)[EPU]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float keep = base + q < waves ? 1.f : 0.f;
#pragma unroll
            for (int e = 0; e < EPU; ++e) sum[e] = q == 0 ? sum[e] + v[q][e] : sum[e] + keep * v[q][e];
        }
    };
    auto emit_pair = [&](const Unit& xa, const float (&sa)[EPU], const Unit& xb, const float (&sb)[EPU]) {
        if constexpr (MODE == kDirect) {
            __builtin_amdgcn_raw_buffer_store_b32(pack_half2(sa[0], sa[1]), rs_out, xa.off, 0, kWriteThrough);
            __builtin_amdgcn_raw_buffer_store_b32(pack_half2(sb[0], sb[1]), rs_out, xb.off, 0, kWriteThrough);
        } else if constexpr (MODE == kAtomicPkF16 || MODE == kAtomicPkF16Phase || MODE == kAtomicPkF16Service) {
            const half2_t ha = {(_Float16)sa[0], (_Float16)sa[1]};
            const half2_t hb = {(_Float16)sb[0], (_Float16)sb[1]};
            __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(ha, rs_out, xa.off, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(hb, rs_out, xb.off, 0, 0);
        } else if constexpr (MODE == kAtomicFixed) {
            const Unit* xs[2] = {&xa, &xb};
            const float vs[2] = {sa[0], sb[0]};
            uint64_t mine[2], old[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                mine[i] = fixed_contribution(vs[i]);
                old[i] = 0;
                if (xs[i]->ok)
                    old[i] = __hip_atomic_fetch_add((uint64_t*)p.scratch + (size_t)xs[i]->row * n + xs[i]->col, mine[i],
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                float total = 0.f;
                const size_t idx = (size_t)xs[i]->row * n + xs[i]->col;
                if (xs[i]->ok && fixed_finish((uint64_t*)p.scratch + idx, old[i], mine[i], p.split_k, &total)) {
                    const _Float16 h = (_Float16)total;
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(uint16_t, h), rs_out, xs[i]->off, 0, kWriteThrough);
                }
            }
        } else if constexpr (MODE == kAtomicF32) {
            if (xa.ok)
                __hip_atomic_fetch_add(p.scratch + (size_t)xa.row * n + xa.col, sa[0], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            if (xb.ok)
                __hip_atomic_fetch_add(p.scratch + (size_t)xb.row * n + xb.col, sb[0], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        } else {  // kWorkspace
            const Unit* xs[2] = {&xa, &xb};
            const float* ss[2] = {sa, sb};
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if (!xs[i]->ok) continue;
                const uint64_t bits = (uint64_t)__builtin_bit_cast(uint32_t, ss[i][0]) |
                                      ((uint64_t)__builtin_bit_cast(uint32_t, ss[i][EPU - 1]) << 32);
                __hip_atomic_store((uint64_t*)(p.scratch + ((size_t)slice * m + xs[i]->row) * n + xs[i]->col), bits,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };
    (void)kBufferOut;

    const Unit first_a = make_unit(tid), first_b = make_unit(tid + nthreads);
    const bool has_units = tid < units;  // a workgroup of many waves on a narrow tile has idle threads
    __syncthreads();
    float va[4][EPU], vb[4][EPU];
    if (has_units) {
        read_unit(first_a, 0, va);
        read_unit(first_b, 0, vb);
    }

    if constexpr (MODE == kAtomicPkF16Phase) {
        // wait until this call's zeros of the tile are in memory (normally already seen)
        const uint32_t expect = lds_phase[0];
        uint32_t seen = lds_phase[1];
        if (seen != expect) seen = __builtin_amdgcn_readfirstlane(probe.value);
        int polls = 0;
        while (seen != expect && polls < p.spin_limit) {
            __builtin_amdgcn_s_sleep(4);
            seen = __builtin_amdgcn_readfirstlane(
                __hip_atomic_load(p.flags + origin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            ++polls;
        }
        if (seen != expect && lane == 0) phase_wait_failed(p.errors, p.err_host, rs_out, (uint32_t)n0 * 2u);
    }

    if (has_units) {
        float sa[EPU], sb[EPU];
#pragma unroll
        for (int e = 0; e < EPU; ++e) sa[e] = sb[e] = 0.f;
        add_unit(0, va, sa);
        add_unit(0, vb, sb);
        for (int base = 4; base < waves; base += 4) {
            read_unit(first_a, base, va);
            read_unit(first_b, base, vb);
            add_unit(base, va, sa);
            add_unit(base, vb, sb);
        }
        emit_pair(first_a, sa, first_b, sb);
    }
    for (int u0 = tid + 2 * nthreads; u0 < units; u0 += 2 * nthreads) {
        const Unit xa = make_unit(u0), xb = make_unit(u0 + nthreads);
        float sa[EPU], sb[EPU];
#pragma unroll
        for (int e = 0; e < EPU; ++e) sa[e] = sb[e] = 0.f;
        for (int base = 0; base < waves; base += 4) {
            read_unit(xa, base, va);
            read_unit(xb, base, vb);
            add_unit(base, va, sa);
            add_unit(base, vb, sb);
        }
        emit_pair(xa, sa, xb, sb);
    }

    if constexpr (MODE == kAtomicF32 || MODE == kWorkspace) {
        // ticket: the workgroup that arrives last at this tile finishes it
        __shared__ uint32_t last_flag;
        wait_memory_ops();
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t old = __hip_atomic_fetch_add(p.tickets + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last_flag = (old == (uint32_t)(p.split_k - 1));
        }
        __syncthreads();
        if (last_flag) {
            const int pairs = m * (BN / 2);
            if constexpr (MODE == kAtomicF32) {
                const int elems = m * BN;
                for (int e = threadIdx.x; e < elems; e += blockDim.x) {
                    const int row = e / BN;
                    const int col = n0 + e % BN;
                    if (col >= n) continue;
                    const size_t idx = (size_t)row * n + col;
                    const float v = __hip_atomic_exchange(p.scratch + idx, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    p.C[idx] = (_Float16)v;
                }
            } else {
                for (int e = threadIdx.x; e < pairs; e += blockDim.x) {
                    const int row = e / (BN / 2);
                    const int col = n0 + 2 * (e % (BN / 2));
                    if (col >= n) continue;
                    float v0 = 0.f, v1 = 0.f;
                    for (int s = 0; s < p.split_k; ++s) {
                        const uint64_t bits = __hip_atomic_load(
                            (const uint64_t*)(p.scratch + ((size_t)s * m + row) * n + col), __ATOMIC_RELAXED,
                            __HIP_MEMORY_SCOPE_AGENT);
                        v0 += __builtin_bit_cast(float, (uint32_t)bits);
                        v1 += __builtin_bit_cast(float, (uint32_t)(bits >> 32));
                    }
                    *(uint32_t*)(p.C + (size_t)row * n + col) = pack_half2(v0, v1);
                }
            }
            if (threadIdx.x == 0)
                __hip_atomic_store(p.tickets + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Kernel entry.  The first 14 dwords of the argument list (five pointers, four integers) are
// what a wave needs before it can issue its first load; the build asks the compiler to have
// them preloaded into scalar registers at wave launch (kernarg preload), so that no round trip
// to the kernarg segment (about 0.3 us) precedes the loads.  Everything else comes in `rest`
// and is fetched by one batch of scalar loads while the first vector loads are in flight.
//   packed = m | param_shift << 5 | waves << 7 | groups_base << 12
//   tiles_rem = tiles | groups_rem << 20
struct GemmRest {
    float* scratch;
    uint32_t* tickets;
    uint32_t* flags;
    uint32_t* counts;
    uint32_t* errors;
    uint32_t* err_host;
    int split_k;
    int lds_wave_bytes;
    int spin_limit;
    int probe_delay;
};

template <int V, int IPG, int MODE, int WMAX, int GC, int BITS = 4, int NS = 1>
__global__ void __launch_bounds__(kWave * (WMAX + (MODE == kAtomicPkF16Service ? 1 : 0)))
gemm_kernel(const _Float16* A, const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros, _Float16* C,
            int packed, int n, int k, int tiles_rem, const GemmRest rest)
{
    GemmArgs p;
    p.A = A;
    p.qweight = qweight;
    p.scales = scales;
    p.qzeros = qzeros;
    p.C = C;
    p.m = packed & 31;
    p.param_shift = (packed >> 5) & 3;
    p.waves = (packed >> 7) & 31;
    p.groups_base = (int)((unsigned)packed >> 12);
    p.groups_rem = (int)((unsigned)tiles_rem >> 20);
    p.n = n;
    p.k = k;
    p.tiles = tiles_rem & ((1 << 20) - 1);
    p.scratch = rest.scratch;
    p.tickets = rest.tickets;
    p.flags = rest.flags;
    p.counts = rest.counts;
    p.errors = rest.errors;
    p.err_host = rest.err_host;
    p.split_k = rest.split_k;
    p.lds_wave_bytes = rest.lds_wave_bytes;
    p.spin_limit = rest.spin_limit;
    p.probe_delay = rest.probe_delay;
    gemm_body<V, IPG, MODE, WMAX, GC, BITS, NS>(p);
}

// Streaming SplitK kernel: the four column strips of a workgroup share their activations
// through LDS (see w4a16_stream.hpp).  blockIdx = (slice, tile), dispatched as tile * split_k + slice: consecutive
// workgroups go to consecutive compute dies, so with split_k a multiple of 8 every die reads
// only its own k slices of A.
//
// MODE kDirect            split_k == 1: round once, store.
// MODE kAtomicPkF16       packed-fp16 atomic adds into a C that a fill kernel zeroed beforehand.
// MODE kAtomicPkF16Phase  packed-fp16 atomic adds, C zeroed inside this kernel by the phase
//                         protocol of gemm_kernel, run by wave 0 of the workgroup.  Its memory
//                         operations (zero stores of slice 0, load of the call count) are issued
//                         behind the prologue's loads, so their completion holds back none of
//                         the data the wave needs first; it publishes after the first round of
//                         the steady loop, when a load issued after the count has been consumed,
//                         samples the flag before the last groups and does not join the last
//                         barrier, behind which all waves add into C, before it has seen it.
// BITS: width of the packed fields, as in gemm_body.
template <int D, int MODE, int MT, int BITS = 4>
__device__ __forceinline__ void stream_body(const StreamArgs& p)
{
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    constexpr bool kPhase = MODE == kAtomicPkF16Phase;
    constexpr uint32_t kOutside = 0xFFFFFF00u;

    const int tid = threadIdx.x;
    const int nthreads = kStreamStrips * p.wk * kWave;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    // grid = (split_k, tiles): the same dispatch order as tile * split_k + slice, without a division
    // at the head of every wave
    const int slice = blockIdx.x;
    const int tile = blockIdx.y;
    const int m = p.m, n = p.n, k = p.k;
    // (the host has checked the shape: divisions by constants become single shifts)
    __builtin_assume(m > 0 && n > 0 && k > 0);

    const int strip = wave & (kStreamStrips - 1);
    const int kpart = wave / kStreamStrips;
    // k part of this wave, its first compute group and its group count (the same for every wave
    // of the workgroup: the host allows a remainder only with one k part per workgroup)
    const int part = slice * p.wk + kpart;
    const int g_begin = part * p.groups_base + (part < p.groups_rem ? part : p.groups_rem);
    const int G_real = p.groups_base + (part < p.groups_rem ? 1 : 0);
    // Ring depth 2 walks the groups in pairs.  An odd count is evened out by a phantom group
    // behind the last one: it is loaded (the next part's data, or zeros behind the end of k) and
    // multiplied like the others, and its product is dropped (a second drain path for odd
    // counts made the compiler wait for every load in flight before either drain).
    const int G = D == 2 ? (G_real + 1) & ~1 : G_real;
    const float last_keep = G == G_real ? 1.f : 0.f;
    const int n0 = (tile * kStreamStrips + strip) * 64;

    const LaneMap lm = make_lane_map<4, BITS>(lane, n0, m, n, k);
    const uint32_t qgroups = (uint32_t)(k / 128) >> p.param_shift;
    Tensors tensors;
    tensors.A = make_rsrc(p.A, (uint32_t)m * (uint32_t)k * 2u);
    constexpr int kFields = BITS == 3 ? 1 : 32 / BITS;  // sizes written per width, as in gemm_body
    tensors.qweight = make_rsrc(p.qweight, (uint32_t)(BITS == 3 ? k / 32 * 3 : k / kFields) * (uint32_t)n * 4u);
    tensors.scales = make_rsrc(p.scales, qgroups * (uint32_t)n * 2u);
    tensors.qzeros = make_rsrc(p.qzeros, qgroups * (uint32_t)(BITS == 3 ? n / 32 * 3 : n / kFields) * 4u);
    tensors.m = m;
    tensors.n = n;
    tensors.k = k;
    tensors.param_shift = p.param_shift;
    const rsrc_t rs_c = make_rsrc(p.C, (uint32_t)m * (uint32_t)n * 2u);

    // this wave's quarter of a chunk: rows 4 strip .. 4 strip + 3 of every row tile, 16 lanes
    // (256 bytes) per row; rows >= m are not fetched (an offset outside the buffer returns zeros)
    StreamLane<MT> sl;
    const int prow = 4 * strip + (lane >> 4);
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        const int arow = 16 * rt + prow;
        sl.a_voff[rt] = arow < m ? ((uint32_t)arow * (uint32_t)k + 8u * (uint32_t)(lane & 15)) * 2u : kOutside;
    }
    sl.a_soff0 = (uint32_t)g_begin * 256u;
    sl.wslot = chunk_slot_bytes(lane & 15, prow);
#pragma unroll
    for (int it = 0; it < 4; ++it) sl.roff[it] = chunk_slot_bytes(4 * it + (lane >> 4), lane & 15);
    sl.ring = lds_raw + kpart * 2 * (MT * kChunkBytes);

    // ---- prologue: the first D chunk quarters, then the first D groups of weights; chunk 0 goes
    // to LDS.  The compute unit returns the loads of all its waves in one issue order, and
    // nobody can start before all four quarters of chunk 0 are there: the barrier between the
    // two kinds of loads keeps every quarter ahead of every weight load of the workgroup
    // (otherwise the last wave's quarter queues behind the other waves' weights, tens of KiB).
    u32x4_t a_in[D][MT];
#pragma unroll
    for (int h = 0; h < D; ++h)
#pragma unroll
        for (int rt = 0; rt < MT; ++rt)
            a_in[h][rt] = __builtin_amdgcn_raw_buffer_load_b128(tensors.A, sl.a_voff[rt],
                                                                sl.a_soff0 + (uint32_t)h * 256u, 0);
    __builtin_amdgcn_sched_barrier(0);
    // (the bare barrier: nothing in LDS is handed over here, and the fence of __syncthreads would
    // wait for every scalar load in flight, the second batch of kernel arguments among them)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    WeightRing<D, BITS> ring;
    ring_prime<D, 0>(ring, lm, tensors, g_begin);

    // ---- phase protocol, first part (wave 0), behind the prologue's loads: zeros of slice 0 (the
    // lanes of every other wave get offsets outside the buffer), then the workgroup's call count
    const uint32_t origin = (uint32_t)tile * (kStreamTileCols / 16);
    uint32_t count = 0;
    if constexpr (kPhase) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        // 16-byte units of the tile: m rows x 32 units; n % 8 == 0 keeps a unit inside or outside
#pragma unroll
        for (int i = 0; i < 8 * MT; ++i) {
            const int u = lane + kWave * i;
            const int row = u >> 5, col = tile * kStreamTileCols + 8 * (u & 31);
            const bool inside = wave == 0 && slice == 0 && row < m && col < n;
            const uint32_t off = inside ? ((uint32_t)row * (uint32_t)n + (uint32_t)col) * 2u : kOutside;
            __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{0u, 0u, 0u, 0u}, rs_c, off, 0, 16);  // 16 = sc1
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        const rsrc_t rs_counts = make_rsrc(p.counts, kPhaseOrigins * (uint32_t)p.split_k * 4u);
        count = __builtin_amdgcn_raw_buffer_load_b32(
            rs_counts, wave == 0 ? (origin * (uint32_t)p.split_k + (uint32_t)slice) * 4u : kOutside, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
        *(half8_t*)(sl.ring + rt * kChunkBytes + sl.wslot) = order_activations<BITS>(a_in[0][rt]);
    __syncthreads();
    u32x4_t a[MT][4];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int it = 0; it < 4; ++it) a[rt][it] = *(const u32x4_t*)(sl.ring + rt * kChunkBytes + sl.roff[it]);

    float4_t acc[MT][4];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[rt][j] = float4_t{0.f, 0.f, 0.f, 0.f};
    const uint32_t magic = unpack_magic<BITS>();

    uint32_t now = 0, sample = 0;
    bool published = !(kPhase && wave == 0);
    auto publish = [&]() {
        // the count was issued before weights that have been consumed by now: it has arrived,
        // and with it the zero stores issued before it have completed
        now = __builtin_amdgcn_readfirstlane(count) + 1u;
        if (lane == 0) {
            store_through(p.counts + origin * (uint32_t)p.split_k + (uint32_t)slice, now);
            if (slice == 0) __hip_atomic_store(p.flags + origin, now, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        published = true;
    };
    // steady state: D groups are consumed and the next D requested, as long as those exist
    int c = 0;
    for (; c + 2 * D <= G; c += D) {
        stream_groups<D, 0, true, MT>(ring, a_in, a, sl, lm, tensors, magic, c, g_begin, acc, 1.f);
        if constexpr (kPhase) {
            if (!published && c >= D) publish();
        }
    }
    if constexpr (kPhase) {
        if (wave == 0) {
            if (!published) publish();
            sample = __hip_atomic_load(p.flags + origin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    stream_groups<D, 0, false, MT>(ring, a_in, a, sl, lm, tensors, magic, c, g_begin, acc, last_keep);

    // ---- up to 16 rows: the tiles go to LDS and come back with consecutive lanes on consecutive
    // column pairs, in as few instructions as possible behind the barrier (one wave per SIMD
    // runs them with nothing to overlap them with).  Every wave stores its whole [16][64] tile
    // (rows >= m are never added); thread t owns the column pair 2 (t % 128) of the workgroup's
    // 256 columns and the rows t / 128 + (threads / 128) i, so its LDS reads share one address
    // register with constant offsets and its offsets into C advance by a constant.  Rows >= m
    // lie behind the end of the buffer by themselves; columns >= n get an offset that does.
    if constexpr (MT == 1) {
        constexpr int kWaveTile = 16 * 64 * 4;
        constexpr uint32_t kFarOutside = 0x80000000u;  // stays outside when the row steps are added
        char* tiles = lds_raw + p.wk * 2 * kChunkBytes;
        char* mine = tiles + wave * kWaveTile + ((4 * (lane >> 4)) * 64 + 4 * (lane & 15)) * 4;
        const int cp = tid & 127;
        const int col = tile * kStreamTileCols + 2 * cp;
        uint32_t src = (uint32_t)((cp >> 5) * kWaveTile + 8 * (cp & 31) + (tid >> 7) * 256);
        uint32_t off0 = col < n ? ((uint32_t)(tid >> 7) * (uint32_t)n + (uint32_t)col) * 2u : kFarOutside;
        asm volatile("" : "+v"(src), "+v"(off0));
#pragma unroll
        for (int r = 0; r < 4; ++r)
            *(float4_t*)(mine + r * 256) = float4_t{acc[0][0][r], acc[0][1][r], acc[0][2][r], acc[0][3][r]};
        if constexpr (kPhase) {
            if (wave == 0) {
                // wave 0 holds the barrier until this call's zeros of the tile are in memory
                bool seen = __builtin_amdgcn_readfirstlane(sample) == now;
                int polls = 0;
                while (!seen && polls < p.spin_limit) {
                    for (int i = 0; i < p.probe_delay; ++i) __builtin_amdgcn_s_sleep(1);
                    seen = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.flags + origin, __ATOMIC_RELAXED,
                                                                            __HIP_MEMORY_SCOPE_AGENT)) == now;
                    ++polls;
                }
                if (!seen && lane == 0)
                    phase_wait_failed(p.errors, p.err_host, rs_c, (uint32_t)tile * (uint32_t)kStreamTileCols * 2u);
            }
        }
        __syncthreads();
        const char* theirs = tiles + src;
        auto emit = [&](float2 v, uint32_t off) {
            if constexpr (MODE == kDirect) {
                __builtin_amdgcn_raw_buffer_store_b32(pack_half2(v.x, v.y), rs_c, off, 0, kWriteThrough);
            } else {
                const half2_t h = {(_Float16)v.x, (_Float16)v.y};
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(h, rs_c, off, 0, 0);
            }
        };
        if (p.wk == 1) {
            // 256 threads: rows t / 128 + 2 i
            const uint32_t step = 4u * (uint32_t)n;
            float2 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = *(const float2*)(theirs + 512 * i);
#pragma unroll
            for (int i = 0; i < 8; ++i) emit(v[i], off0 + (uint32_t)i * step);
        } else {
            // 512 threads, two k parts: rows t / 128 + 4 i, the second part's tiles 16 KiB further on
            const uint32_t step = 8u * (uint32_t)n;
            float2 v[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = *(const float2*)(theirs + 1024 * i);
                w[i] = *(const float2*)(theirs + 1024 * i + kStreamStrips * kWaveTile);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) emit(float2{v[i].x + w[i].x, v[i].y + w[i].y}, off0 + (uint32_t)i * step);
        }
        return;
    }

    // ---- more rows: every wave's tile -> LDS (behind the chunks); after the barrier the sums
    // leave with consecutive lanes on consecutive column pairs
    float* red_all = (float*)(lds_raw + p.wk * 2 * (MT * kChunkBytes));
    float* red = red_all + (size_t)wave * m * 64;  // [m][64]
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 16 * rt + 4 * (lane >> 4) + r;
            if (row < m)
                *(float4_t*)(red + row * 64 + 4 * (lane & 15)) =
                    float4_t{acc[rt][0][r], acc[rt][1][r], acc[rt][2][r], acc[rt][3][r]};
        }
    if constexpr (kPhase) {
        if (wave == 0) {
            // wave 0 holds the barrier until this call's zeros of the tile are in memory
            bool seen = __builtin_amdgcn_readfirstlane(sample) == now;
            int polls = 0;
            while (!seen && polls < p.spin_limit) {
                for (int i = 0; i < p.probe_delay; ++i) __builtin_amdgcn_s_sleep(1);
                seen = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.flags + origin, __ATOMIC_RELAXED,
                                                                        __HIP_MEMORY_SCOPE_AGENT)) == now;
                ++polls;
            }
            if (!seen && lane == 0)
                phase_wait_failed(p.errors, p.err_host, rs_c, (uint32_t)tile * (uint32_t)kStreamTileCols * 2u);
        }
    }
    __syncthreads();
    // A thread keeps one pair of adjacent columns (cp = tid % 128: strip cp / 32, columns
    // 2 (cp % 32) ..) and walks down the rows nthreads / 128 at a time, so per row it needs one
    // LDS read per k part, one conversion and one add whose address advances by a constant;
    // consecutive lanes sit on consecutive pairs (an atomic instruction touches the fewest cache
    // lines).  Four rows are in flight together; rows >= m and columns >= n get offsets outside
    // the buffer, which the hardware drops.
    const int cp = tid & 127;
    const int st = cp >> 5, c2 = 2 * (cp & 31);
    const int col = tile * kStreamTileCols + st * 64 + c2;
    const int rows_per_pass = nthreads >> 7;
    const int strip_floats = m * 64;
    const float* src0 = red_all + st * strip_floats + c2;
    const int second_part = (p.wk - 1) * kStreamStrips * strip_floats;  // wk is 1 or 2
    const bool col_ok = col < n;
    for (int row0 = tid >> 7; row0 < m; row0 += 4 * rows_per_pass) {
        float2 v[4];
        uint32_t off[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = row0 + i * rows_per_pass;
            const int rc = row < m ? row : row0;
            off[i] = (row < m && col_ok) ? ((uint32_t)row * (uint32_t)n + (uint32_t)col) * 2u : kOutside;
            v[i] = *(const float2*)(src0 + rc * 64);
            if (p.wk > 1) {
                const float2 t1 = *(const float2*)(src0 + rc * 64 + second_part);
                v[i].x += t1.x;
                v[i].y += t1.y;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (MODE == kDirect) {
                __builtin_amdgcn_raw_buffer_store_b32(pack_half2(v[i].x, v[i].y), rs_c, off[i], 0, kWriteThrough);
            } else {
                const half2_t h = {(_Float16)v[i].x, (_Float16)v[i].y};
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(h, rs_c, off[i], 0, 0);
            }
        }
    }
}

// Kernel entry of the streaming kernel; the leading 14 dwords are preloaded as for gemm_kernel.
//   packed = m | param_shift << 7 | wk << 9 | groups_base << 12
//   split_rem = split_k | groups_rem << 16
// Up to 16 rows: 4 or 8 waves, at most 256 registers each.  More rows (MT row tiles): 4 waves,
// which may then use the whole register file of their SIMDs for the MT x 4 accumulator tiles.
struct StreamRest {
    uint32_t* flags;
    uint32_t* counts;
    uint32_t* errors;
    uint32_t* err_host;
    int spin_limit;
    int probe_delay;
};

template <int D, int MODE, int MT, int BITS = 4>
__global__ void __launch_bounds__(kWave * (MT > 1 ? 4 : 8))
gemm_stream_kernel(const _Float16* A, const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros,
                   _Float16* C, int packed, int n, int k, int split_rem, const StreamRest rest)
{
    StreamArgs p;
    p.A = A;
    p.qweight = qweight;
    p.scales = scales;
    p.qzeros = qzeros;
    p.C = C;
    p.m = packed & 127;
    p.param_shift = (packed >> 7) & 3;
    p.wk = (packed >> 9) & 7;
    p.groups_base = (int)((unsigned)packed >> 12);
    p.groups_rem = (int)((unsigned)split_rem >> 16);
    p.n = n;
    p.k = k;
    p.split_k = split_rem & 0xFFFF;
    p.tiles = 0;  // only the launch needs it
    p.flags = rest.flags;
    p.counts = rest.counts;
    p.errors = rest.errors;
    p.err_host = rest.err_host;
    p.spin_limit = rest.spin_limit;
    p.probe_delay = rest.probe_delay;
    stream_body<D, MODE, MT, BITS>(p);
}

// StreamK decomposition (the paper's Conclusion names it as the successor of SplitK to explore):
// a fixed number of persistent workgroups, about one or two per compute unit, divide the
// iteration space evenly.  An iteration is one compute group (128 k) of one 256-column tile;
// iterations are numbered tile-major, and workgroup w takes [w T / W, (w + 1) T / W) of the
// T = tiles x groups iterations: a run that may end one tile and begin the next.  Every piece
// of a tile (a "segment") is computed like a k slice of the streaming SplitK kernel and added
// to C with packed-fp16 atomics (C zeroed by the fill kernel); a segment that is a whole tile
// is stored.  Segments have any length >= 1; an odd one runs a phantom group more, as in
// stream_body.
template <int BITS>
__device__ __forceinline__ void streamk_segment(const StreamArgs& p, char* lds_raw, int tile, int g_begin, int G,
                                                int groups)
{
    constexpr int D = 2;
    constexpr uint32_t kOutside = 0xFFFFFF00u;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int strip = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int m = p.m, n = p.n, k = p.k;
    // (the host has checked the shape: divisions by constants become single shifts)
    __builtin_assume(m > 0 && n > 0 && k > 0);
    const int n0 = (tile * kStreamStrips + strip) * 64;

    const LaneMap lm = make_lane_map<4, BITS>(lane, n0, m, n, k);
    const uint32_t qgroups = (uint32_t)groups >> p.param_shift;
    Tensors tensors;
    tensors.A = make_rsrc(p.A, (uint32_t)m * (uint32_t)k * 2u);
    constexpr int kFields = BITS == 3 ? 1 : 32 / BITS;  // sizes written per width, as in gemm_body
    tensors.qweight = make_rsrc(p.qweight, (uint32_t)(BITS == 3 ? k / 32 * 3 : k / kFields) * (uint32_t)n * 4u);
    tensors.scales = make_rsrc(p.scales, qgroups * (uint32_t)n * 2u);
    tensors.qzeros = make_rsrc(p.qzeros, qgroups * (uint32_t)(BITS == 3 ? n / 32 * 3 : n / kFields) * 4u);
    tensors.m = m;
    tensors.n = n;
    tensors.k = k;
    tensors.param_shift = p.param_shift;
    const rsrc_t rs_c = make_rsrc(p.C, (uint32_t)m * (uint32_t)n * 2u);

    StreamLane<1> sl;
    const int prow = 4 * strip + (lane >> 4);
    sl.a_voff[0] = prow < m ? ((uint32_t)prow * (uint32_t)k + 8u * (uint32_t)(lane & 15)) * 2u : kOutside;
    sl.a_soff0 = (uint32_t)g_begin * 256u;
    sl.wslot = chunk_slot_bytes(lane & 15, prow);
#pragma unroll
    for (int it = 0; it < 4; ++it) sl.roff[it] = chunk_slot_bytes(4 * it + (lane >> 4), lane & 15);
    sl.ring = lds_raw;

    // prologue as in stream_body.  The ring is primed with two groups even when the segment has
    // one: the second then is the phantom group.
    u32x4_t a_in[D][1];
#pragma unroll
    for (int h = 0; h < D; ++h)
        a_in[h][0] = __builtin_amdgcn_raw_buffer_load_b128(tensors.A, sl.a_voff[0], sl.a_soff0 + (uint32_t)h * 256u, 0);
    __builtin_amdgcn_sched_barrier(0);
    // (the bare barrier: nothing in LDS is handed over here, and the fence of __syncthreads would
    // wait for every scalar load in flight, the second batch of kernel arguments among them)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    WeightRing<D, BITS> ring;
    ring_prime<D, 0>(ring, lm, tensors, g_begin);
    *(half8_t*)(sl.ring + sl.wslot) = order_activations<BITS>(a_in[0][0]);
    __syncthreads();
    u32x4_t a[1][4];
#pragma unroll
    for (int it = 0; it < 4; ++it) a[0][it] = *(const u32x4_t*)(sl.ring + sl.roff[it]);
    float4_t acc[1][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[0][j] = float4_t{0.f, 0.f, 0.f, 0.f};
    const uint32_t magic = unpack_magic<BITS>();

    // an odd count is evened out by a phantom group whose product is dropped (see stream_body)
    const int Ge = (G + 1) & ~1;
    const float last_keep = Ge == G ? 1.f : 0.f;
    int c = 0;
    for (; c + 2 * D <= Ge; c += D)
        stream_groups<D, 0, true, 1>(ring, a_in, a, sl, lm, tensors, magic, c, g_begin, acc, 1.f);
    stream_groups<D, 0, false, 1>(ring, a_in, a, sl, lm, tensors, magic, c, g_begin, acc, last_keep);

    // the tile -> LDS; column pairs leave as in stream_body
    float* red_all = (float*)(lds_raw + 2 * kChunkBytes);
    float* red = red_all + (size_t)strip * m * 64;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * (lane >> 4) + r;
        if (row < m)
            *(float4_t*)(red + row * 64 + 4 * (lane & 15)) = float4_t{acc[0][0][r], acc[0][1][r], acc[0][2][r], acc[0][3][r]};
    }
    __syncthreads();
    const bool whole_tile = G == groups;
    const int cp = tid & 127;
    const int st = cp >> 5, c2 = 2 * (cp & 31);
    const int col = tile * kStreamTileCols + st * 64 + c2;
    constexpr int rows_per_pass = kStreamStrips * kWave >> 7;
    const float* src0 = red_all + st * (m * 64) + c2;
    const bool col_ok = col < n;
    for (int row0 = tid >> 7; row0 < m; row0 += 4 * rows_per_pass) {
        float2 v[4];
        uint32_t off[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = row0 + i * rows_per_pass;
            const int rc = row < m ? row : row0;
            off[i] = (row < m && col_ok) ? ((uint32_t)row * (uint32_t)n + (uint32_t)col) * 2u : kOutside;
            v[i] = *(const float2*)(src0 + rc * 64);
        }
        if (whole_tile) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_raw_buffer_store_b32(pack_half2(v[i].x, v[i].y), rs_c, off[i], 0, kWriteThrough);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const half2_t h = {(_Float16)v[i].x, (_Float16)v[i].y};
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_v2f16(h, rs_c, off[i], 0, 0);
            }
        }
    }
}

// Kernel entry of the StreamK variant: 4 waves (one 256-column tile wide); `workgroups` is the
// launch's grid size (an argument, so that no launch-geometry read is needed).
//   packed = m | param_shift << 7
template <int BITS>
__global__ void __launch_bounds__(kWave* kStreamStrips)
gemm_streamk_kernel(const _Float16* A, const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros,
                    _Float16* C, int packed, int n, int k, int workgroups)
{
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    StreamArgs p;
    p.A = A;
    p.qweight = qweight;
    p.scales = scales;
    p.qzeros = qzeros;
    p.C = C;
    p.m = packed & 127;
    p.param_shift = (packed >> 7) & 3;
    p.n = n;
    p.k = k;
    const int groups = k / 128;
    const long long total = (long long)((n + kStreamTileCols - 1) / kStreamTileCols) * groups;
    const long long w = blockIdx.x;
    long long it = w * total / workgroups;
    const long long end = (w + 1) * total / workgroups;
    while (it < end) {
        const int tile = (int)(it / groups);
        const int g_begin = (int)(it - (long long)tile * groups);
        const long long rest = end - it;
        const int G = rest < groups - g_begin ? (int)rest : groups - g_begin;
        streamk_segment<BITS>(p, lds_raw, tile, g_begin, G, groups);
        it += G;
        __syncthreads();  // the next segment reuses the chunks and the tile in LDS
    }
}

// C <- 0 for the packed-fp16 atomic mode (a kernel, not a memset, so the call can be captured
// in a HIP graph).
__global__ void fill_zero_kernel(uint32_t* p, size_t words)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// ---- activation ordering (GPTQ's act-order; outside the paper, whose groups are contiguous) ----
// The group of row kk is g_idx[kk].  Such a map comes from quantising the rows in some order and
// cutting that order into runs of g, so sorting the rows by group (stably) makes the groups
// contiguous again: with perm = the sorted order, C = sum_i A[:, perm[i]] W[perm[i], :], which is
// the plain product of the gathered activations with the reordered weight rows.  The weights are
// static, so they are reordered once (prepare); a call gathers the activations (m x k fp16, one
// small kernel) and runs the ordinary GEMM.

// perm[b * g + i] = the i-th row (in ascending row order) whose group is b.  One workgroup per
// group walks all rows 256 at a time; a group that does not have exactly g rows sets *status.
__global__ void __launch_bounds__(256)
actorder_perm_kernel(const int32_t* __restrict__ g_idx, int32_t* __restrict__ perm, int32_t* status, int k, int g)
{
    __shared__ int wave_total[4];
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int count = 0;  // rows of this group found so far (uniform)
    for (int base = 0; base < k; base += 256) {
        const int r = base + tid;
        const bool mine = r < k && g_idx[r] == b;
        const unsigned long long ballot = __ballot(mine);
        const int rank = __popcll(ballot & ((1ull << lane) - 1ull));
        if (lane == 0) wave_total[wave] = __popcll(ballot);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) before += wave_total[w];
            total += wave_total[w];
        }
        const int pos = count + before + rank;
        if (mine && pos < g) perm[(size_t)b * g + pos] = r;
        count += total;
        __syncthreads();
    }
    if (tid == 0 && count != g) atomicOr(status, 1);
}

// Row i of the reordered matrix is row perm[i] of the given one: every output word gathers its
// eight 4-bit fields.  Entries of perm outside [0, k) (only possible when *status was set) are
// clamped, so the kernel stays inside its buffers whatever g_idx held.
__global__ void actorder_repack_kernel(const uint32_t* __restrict__ qweight, const int32_t* __restrict__ perm,
                                       uint32_t* __restrict__ out, int n, int k)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t words = (size_t)(k / 8) * n;
    if (idx >= words) return;
    const int R = (int)(idx / n), j = (int)(idx % n);
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int src = perm[8 * R + i];
        src = src < 0 ? 0 : (src >= k ? k - 1 : src);
        word |= field(qweight[(size_t)(src >> 3) * n + j], src & 7) << (4 * i);
    }
    out[idx] = word;
}

// A_work[i][t] = A[i][perm[t]].
__global__ void actorder_gather_kernel(const _Float16* __restrict__ A, const int32_t* __restrict__ perm,
                                       _Float16* __restrict__ A_work, int m, int k)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)m * k) return;
    const int i = (int)(idx / k), t = (int)(idx % k);
    int src = perm[t];
    src = src < 0 ? 0 : (src >= k ? k - 1 : src);
    A_work[idx] = A[(size_t)i * k + src];
}

// ---- measurement probe: a plain coalesced read of a buffer (U 16-byte loads in flight per
// lane, grid-stride), the ceiling any kernel that has to read those bytes can reach.  NT: with
// the non-temporal hint that the GEMM kernels' weight loads carry.
template <int U, bool NT = false>
__global__ void __launch_bounds__(512) read_probe_kernel(const u32x4_t* __restrict__ p, size_t vecs, uint32_t* sink)
{
    auto fetch = [&](size_t at) {
        if constexpr (NT) return __builtin_nontemporal_load(p + at);
        else return p[at];
    };
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (; i + (U - 1) * stride < vecs; i += U * stride) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = fetch(i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < vecs; i += stride) acc ^= fetch(i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && sink) sink[0] = acc.x;  // keeps the loads alive
}

// ---- test probes: the same unpack_shift / zero_const / field routines as the GEMM ----------
// q_u8[kk][j] and z_u8[gi][j]; one thread per packed word.
__global__ void unpack_kernel(const uint32_t* qweight, const uint32_t* qzeros, uint8_t* q_u8, uint8_t* z_u8,
                              int n, int k, int groups)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nw = (size_t)(k / 8) * n;
    if (i < nw) {
        const int r = (int)(i / n), j = (int)(i % n);
        const half8_t h = unpack_shift(qweight[i], zero_const(0), magic_1024x2());
#pragma unroll
        for (int s = 0; s < 8; ++s) q_u8[(size_t)(8 * r + slot_to_field(s)) * n + j] = (uint8_t)(int)(float)h[s];
    }
    const size_t nz = (size_t)groups * (n / 8);
    if (i < nz) {
        const int gi = (int)(i / (n / 8)), c = (int)(i % (n / 8));
        const uint32_t w = qzeros[i];
#pragma unroll
        for (int f = 0; f < 8; ++f) z_u8[(size_t)gi * n + 8 * c + f] = (uint8_t)field(w, f);
    }
}

// W[kk][j] = fp16((q - z) * s); one thread per packed word.
__global__ void dequant_kernel(const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros,
                               _Float16* W, int n, int k, int group_size)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nw = (size_t)(k / 8) * n;
    if (i >= nw) return;
    const int r = (int)(i / n), j = (int)(i % n);
    const int gi = (8 * r) / group_size;
    const uint32_t z = field(qzeros[(size_t)gi * (n / 8) + j / 8], j % 8);
    const float s = (float)scales[(size_t)gi * n + j];
    const half8_t h = unpack_shift(qweight[i], zero_const(z), magic_1024x2());
#pragma unroll
    for (int t = 0; t < 8; ++t) W[(size_t)(8 * r + slot_to_field(t)) * n + j] = (_Float16)((float)h[t] * s);
}

// ------------------------------------------------------------------------------------------
// Host side
struct Buffer {
    void* ptr = nullptr;
    size_t bytes = 0;
};
// Split-k state of one device, owned by the library.  Buffers only ever grow, and a buffer that
// is outgrown is kept until w4a16_release_scratch: a HIP graph captured earlier still holds its
// address and must find it alive (and consistent: every call leaves its words as it found them).
struct DeviceScratch {
    Buffer sums;      // atomic mode: fp32 [16, n]; all zero whenever no call is running
    Buffer partials;  // workspace mode: fp32 [split_k, m, n]; no invariant
    Buffer fixed;     // fixed-point mode: uint64 [16, n]; all zero whenever no call is running
    Buffer tickets;   // uint32 per column tile; all zero whenever no call is running
    // phase mode, uint32: one buffer per split_k in use (2..kPhaseMaxSplit), allocated on the first
    // call with that split_k: flags [kPhaseOrigins], then counts [kPhaseOrigins][split_k]
    Buffer phase_level[kPhaseMaxSplit + 1];
    Buffer phase_err;  // the error count [1]
    uint32_t* err_host = nullptr;  // pinned host word that a wait which ran out sets to 1
    void* retired[64] = {};        // outgrown buffers, freed by w4a16_release_scratch
    int retired_count = 0;
};
// Where one call's split-k state lives: the library's own buffers, a workspace the caller bound
// to the stream, or the static array of the entry point that allocates nothing.
struct ScratchView {
    float* sums = nullptr;
    float* partials = nullptr;
    uint64_t* fixed = nullptr;
    uint32_t* tickets = nullptr;
    uint32_t* flags = nullptr;
    uint32_t* counts = nullptr;
    uint32_t* errors = nullptr;
    uint32_t* err_host = nullptr;
};
struct ScratchNeed {
    size_t sums_floats = 0, partial_floats = 0, fixed_words = 0, ticket_count = 0;
    int phase_split = 0;  // 0, or the split_k whose flags and counts the call needs
    int n = 0;            // columns of the call (the phase words cover tile origins n0 / 16)
};
enum : int { kScratchLibrary = 0, kScratchStatic = 1 };
// Word offset of the counts inside a level's buffer, and the buffer's size in words.
static size_t phase_counts_offset() { return kPhaseOrigins; }
static size_t phase_level_words(int split_k) { return (size_t)kPhaseOrigins * (1 + (size_t)split_k); }

// ---- the static array of w4a16_gemm_static (callers that cannot allocate) --------------------
// Limits of that entry point: n <= kStaticMaxN, m * n <= kStaticFixedWords for the fixed-point
// adds (up to four rows at the largest n), split_k <= kStaticPhaseMaxSplit for the in-kernel
// zeroing.  Layout, in 32-bit words: [0] the count of waits that ran out (64 words reserved);
// the fixed-point words; then for every split_k from 2 on a level of flags [kStaticOrigins] and
// counts [kStaticOrigins][split_k].  Zero at load time, and every call leaves it as it found it
// (the fixed-point words return to zero, the phase words count calls).
constexpr int kStaticMaxN = 16384;
constexpr size_t kStaticFixedWords = (size_t)4 * kStaticMaxN;  // 64-bit words
constexpr int kStaticPhaseMaxSplit = 32;
constexpr uint32_t kStaticOrigins = kStaticMaxN / 16;
constexpr size_t kStaticHeadWords = 64;
constexpr size_t static_level_offset(int split_k)  // in 32-bit words; levels 2 .. split_k - 1 lie before it
{
    return kStaticHeadWords + 2 * kStaticFixedWords +
           (size_t)kStaticOrigins * ((size_t)(split_k - 2) + ((size_t)(split_k - 1) * split_k / 2 - 1));
}
constexpr size_t kStaticWords = static_level_offset(kStaticPhaseMaxSplit + 1);
static __device__ __align__(256) uint32_t scratch[kStaticWords];
// Text of the last failed HIP call on this host thread (for W4A16_ERR_HIP diagnostics).
static thread_local char g_hip_detail[256] = "";

static bool hip_ok(hipError_t e, const char* what)
{
    if (e == hipSuccess) return true;
    snprintf(g_hip_detail, sizeof(g_hip_detail), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
    return false;
}
#define W4A16_HIP(call) hip_ok((call), #call)

constexpr int kMaxDevices = 64;
// Polls of a tile flag before a wave gives up (each poll is a round trip to memory, about a
// microsecond): far longer than any call takes, short enough that a broken state cannot hang
// the device.
constexpr int kSpinLimit = 1 << 17;
static int g_spin_limit = kSpinLimit;  // w4a16_set_phase_spin_limit (tests of the failure path)
// 64-cycle sleeps before a sample of the tile flag (service wave: before every sample; in-wave
// protocol: between learning the call count and the early sample).  Measured flat from 0 to 16
// with a slight optimum at 8-16 (fewer polls on the way to memory), worse from 32 on.
static int g_probe_delay = 8;
// Deepest weight ring (compute groups in flight per wave) the streaming kernel may use: 1 or 2.
static int g_stream_depth = 2;
// Persistent workgroups of the StreamK variant when the caller leaves the choice to the library.
static int g_streamk_blocks = 256;
// Fewest workgroups that the plan accepts for a launch whose waves each take a long run of groups.
static int g_stream_min_blocks = 160;
static DeviceScratch g_scratch[kMaxDevices];
static uint32_t* g_static_ptr[kMaxDevices];  // device address of `scratch` on each device (hipGetSymbolAddress)
// A workspace that the caller bound to a stream (w4a16_set_workspace): calls on that stream keep
// their split-k state there, so calls on different streams no longer share anything.
struct Binding {
    int dev = -1;
    hipStream_t stream = nullptr;
    uint32_t* base = nullptr;
    int n_max = 0;
};
constexpr int kMaxBindings = 64;
static Binding g_bindings[kMaxBindings];
static std::mutex g_mutex;

// Layout of a caller's workspace, in 32-bit words: 64 words head ([0] = waits that ran out), one
// ticket per 16 columns, the phase levels of split_k 2..64, fp32 sums [16, n_max], fixed-point
// words [16, n_max].
static size_t workspace_level_offset(int n_max, int split_k)
{
    return 64 + (size_t)n_max / 16 + (size_t)kPhaseOrigins * ((size_t)(split_k - 2) + ((size_t)(split_k - 1) * split_k / 2 - 1));
}
static size_t workspace_sums_offset(int n_max) { return (workspace_level_offset(n_max, kPhaseMaxSplit + 1) + 63) & ~(size_t)63; }
static size_t workspace_fixed_offset(int n_max) { return workspace_sums_offset(n_max) + (size_t)16 * n_max; }
static size_t workspace_words(int n_max) { return workspace_fixed_offset(n_max) + (size_t)32 * n_max; }

// `even_split`: a requested split_k must cut k into equal shares of whole quantisation groups
// (Algorithm 1 as printed); otherwise it only has to be positive, and the shares are whole
// compute groups whose counts differ by at most one.
static int check_args(int m, int n, int k, int group_size, int split_k, bool even_split = true)
{
    if (m < 1 || n < 8 || (n % 8) != 0 || group_size < 8 || (group_size % 8) != 0 || k < group_size ||
        (k % group_size) != 0)
        return W4A16_ERR_SHAPE;
    if (split_k < 0) return W4A16_ERR_SPLIT;
    if (even_split && split_k > 0 && ((k % split_k) != 0 || ((k / split_k) % group_size) != 0))
        return W4A16_ERR_SPLIT;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256) return W4A16_ERR_UNSUPPORTED;
    return W4A16_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Largest w in {16, 8, 4, 2, 1}, w <= cap, that leaves every one of `parts_before * w` k parts
// at least one of the `groups` compute groups.
static int largest_wave_split(int groups, int parts_before, int cap)
{
    for (int w = 16; w > 1; w >>= 1)
        if (w <= cap && (long long)parts_before * w <= groups) return w;
    return 1;
}

struct Plan {
    int split_k, tile_cols, waves, reduce;
};

// The phase protocol keeps one set of words per split_k, for any split_k up to kPhaseMaxSplit.
static bool phase_split_ok(int split_k) { return split_k >= 2 && split_k <= kPhaseMaxSplit; }

// Launch shape, from sweeps on MI355X (256 compute units, 1024 SIMDs).
//
// SplitK: 64-column tiles (128-bit weight loads).  The kernel is bound by how fast a burst of
// loads can be put in flight, so the plan aims at about 2048 short-lived waves when the whole
// weight matrix is small enough to be requested at once (<= 8 MiB packed), and otherwise at
// 160 or more workgroups of long-running waves.  Up to four waves of a workgroup divide its k
// range (their tiles are added in LDS, which keeps the atomic traffic down); the rest of the k
// parallelism is split_k.
// Data-parallel: the only source of workgroups is the column tiling, so tiles shrink (64, 32,
// 16 columns) until there are at least 160 of them, and four or eight waves of a workgroup
// divide k.
static int make_plan(int m, int n, int k, int group_size, bool dp, int split_k, int tile_cols, int waves,
                     int reduce, Plan* out, int bits = 4)
{
    const int reduce_asked = reduce;
    // compute groups: the units (32, 64 or 128 consecutive k) that the k parts are made of
    const int cgroups = k / (group_size >= 128 ? 128 : group_size);
    const long long packed_bytes = (long long)k * n * bits / 8;
    const long long weights_half = (long long)k * n / 2;  // the packed bytes of 4-bit fields: size rules count weights
    bool bits_choice = false;
    if (bits != 4) {
        // 2-bit, 3-bit and 8-bit fields: the per-wave kernel with 64-column tiles, with two strips per
        // wave or the streaming kernel where the rules below find them, and narrow tiles for the
        // launches that do not split k
        if (tile_cols != 0 && tile_cols != 64) return W4A16_ERR_UNSUPPORTED;
        // more than 16 rows: the streaming kernel's row tiles (a SplitK launch with the library's tile and waves)
        if (m > 16 && (dp || tile_cols != 0 || waves != 0 || m > 16 * kStreamMaxRowTiles)) return W4A16_ERR_UNSUPPORTED;
        bits_choice = !dp && tile_cols == 0 && waves == 0 && split_k == 0 && m <= 16;
        const bool narrow = dp && tile_cols == 0;
        tile_cols = 64;
        if (narrow) {
            // the data-parallel launch narrows its tiles as the 4-bit one does (further down)
            while (tile_cols > 16 && (n + tile_cols - 1) / tile_cols < g_stream_min_blocks &&
                   (n + tile_cols / 2 - 1) / (tile_cols / 2) <= 256)
                tile_cols /= 2;
        }
    }
    // The rules below come from a sweep of 246 shapes (n 2048..28672, k 1024..14336, m 1, 4, 16)
    // over every launch shape the kernels offer; the plan lands within 1 % (geometric mean, 9 %
    // at worst) of the best candidate of each shape.
    const bool library_choice = !dp && bits == 4 && tile_cols == 0 && waves == 0 && split_k == 0 && m <= 16;
    const int tiles64 = (n + 63) / 64;
    // Short k (up to 1024, or up to 2048 when the column tiles alone fill the machine once):
    // no split at all.  The call is a latency chain of a few microseconds, and zeroing, atomics
    // and further waves only add to it.
    // A random-shape audit added: also up to k = 1536 when the data-parallel tiling gives 130-256
    // workgroups, up to k = 2176 from 130 tiles of 64 columns on (n = 8848, k = 1792, m = 16:
    // 5.6 us against 7.5 with two slices); with five rows or more (where a
    // split costs the zeroing protocol) up to k = 3072 at 190-256 tiles, and, up to twelve rows,
    // up to k = 6400 there.
    int dp_cols = 64;  // the data-parallel kernel's tile width: narrower until 160 workgroups, never past 256
    while (dp_cols > 16 && (n + dp_cols - 1) / dp_cols < g_stream_min_blocks && (n + dp_cols / 2 - 1) / (dp_cols / 2) <= 256)
        dp_cols /= 2;
    const int dp_tiles = (n + dp_cols - 1) / dp_cols;
    const bool fills_once = tiles64 >= 190 && tiles64 <= 256;
    // Whether the two-strip launch further down is to be had for this shape (its conditions
    // other than who is asking).
    // (beyond split_k = 8: 22 MiB since the streaming kernel's epilogue was shortened; n = 8184, k = 6144, m = 4:
    // 8.2 us with two strips, 7.7 with 256 workgroups of the streaming kernel)
    const long long two_strip_limit = bits == 4   ? (cgroups / 4 > 8 ? (22ll << 20) : (32ll << 20))
                                      : bits == 2 ? (cgroups / 4 > 8 ? (24ll << 20) : (32ll << 20))
                                                  : (20ll << 20);
    // (from one row on since the sum over the waves was shortened: 3 % ahead of the fixed-point launch at m = 1)
    // (up to four rows only up to twelve slices: n = 3072, k = 8192: sixteen slices 5.5-5.6 us, one group per wave with
    // fixed-point adds 5.0-5.3)
    const bool two_strip_ok = m >= (bits == 4 ? 1 : 2) && group_size >= 128 && !(tiles64 >= 200 && tiles64 <= 256) &&
                              (reduce == W4A16_REDUCE_AUTO || reduce == W4A16_REDUCE_ATOMIC_PK_F16_PHASE) &&
                              cgroups % 4 == 0 && phase_split_ok(cgroups / 4) && cgroups / 4 <= (m <= 4 ? 12 : 16) &&
                              // (from 132 workgroups on: 140-144 of them are 10-22 % ahead of the single-strip launches
                              // on n = 6144, k = 1536; n = 4608, k = 2048; n = 3584, k = 2560; n = 2304, k = 4096 at
                              // m = 2..16; with 120-128 the single-strip launch with one group per wave is 3-7 % ahead)
                              (long long)((n + 127) / 128) * (cgroups / 4) >= 132 &&
                              // (not just over one workgroup per compute unit where the per-wave kernel with its
                              // service wavefront fills the machine once: n = 2560, k = 8192: 320 workgroups of
                              // two strips take 5.1-5.7 us, six slices of 40 tiles 4.7-5.3)
                              // (with five to twelve rows up to 128 tiles: nine shapes with 264-320 such workgroups, e.g. n = 5120,
                              // k = 4096: the per-wave launch 3-10 % ahead at m = 6, 8 (4.64 us against 5.12) and 1-8 % at
                              // m = 12; from -5 to +6 % at m = 16, two strips ahead at m = 2)
                              // (where that launch gets runs of three groups or fewer: n = 6144, k = 3584, m = 8 would leave it two
                              // slices with 3.5 groups per wave, 5.7 us against 5.2 for 336 workgroups of two strips)
                              !(bits == 4 && m >= 5 && (tiles64 <= 48 || (m <= 12 && tiles64 <= 128 && cgroups <= 12 * (256 / tiles64))) &&
                                (long long)((n + 127) / 128) * (cgroups / 4) > 256 &&
                                (long long)((n + 127) / 128) * (cgroups / 4) < 352) &&
                              (long long)k * n / 2 < two_strip_limit && (size_t)n <= 16 * (size_t)kPhaseOrigins;
    // A fourth audit (40 random shapes, then grids around its misses) added two more cases of no
    // split.  130-256 tiles of 64 columns up to k = 3584: one workgroup per tile over all of k
    // beats the streaming kernel by 13-35 % (n = 10048 or 11520, k = 2304 or 2816, m = 8, 16) and
    // is level with or ahead of everything else, except two strips per wave where they are to be
    // had and the tiles are few (under 170, under 150 up to eight rows: 2-15 % for two strips at
    // 130 tiles, 7 % at 147 with four rows, 2-10 % against them at 157-180).  And 130-256 tiles of 16 columns (n up to 4096) up
    // to k = 3328 where two strips are not to be had: eight waves per 16-column tile beat the
    // split launches by 4-46 % (most at five to twelve rows).
    const bool short_k_tiles_fill = cgroups <= 28 && tiles64 >= 130 && tiles64 <= 256;
    // (a later grid, n = 9728..12288 x k = 1536..3072: two strips 3-15 % ahead up to 168 tiles at m = 2, 6 and,
    // from k = 2048 on, 3-13 % ahead up to 192 tiles at m = 16; level or behind at 176 tiles and more with few rows)
    const bool two_strips_there = two_strip_ok && (tiles64 < 170 || (m > 8 && cgroups >= 16));
    // (4-bit fields only: n = 2880, k = 2944 is 5-7 % slower that way at the other widths)
    // (from five rows on: n = 2304, k = 3072, m = 1 takes 4.2 us that way and 3.5 with six slices of 64-column tiles)
    // (the same on 170-256 tiles of 32 columns up to k = 3200: a grid of n = 5600..8000, k = 2304..3200 where k / 128
    // is no multiple of four, m = 6, 16 has eight waves per tile 5-32 % ahead of what was chosen before, and within
    // 3 % of the best launch except at n = 5600, m = 16 from k = 2816 on, 6-7 %)
    // Since the per-wave kernel's zeroing protocol runs in a service wavefront, its split launches beat the
    // unsplit narrow tiles with five rows or more from ten groups on (n = 1704, k = 1280, m = 8, 16: 3.2-3.5 us
    // against 3.45-3.9; n = 7000, k = 2176, m = 16: 5.0 against 6.1; n = 3072, k = 3328, m = 16: 4.6 against 6.3):
    // the rules on narrow tiles below then hold for up to four rows.  The other field widths, whose per-wave
    // launches use the same wavefront, from sixteen groups on (n = 8192, k = 2048, m = 16: two slices 4.3-5.8 us
    // against 5.4-6.6 unsplit on 32-column tiles; at k = 1536 the unsplit tiles are 2-9 % ahead).
    const bool narrow_ok = !(m >= 5 && cgroups >= (bits == 4 ? 10 : 16) && group_size >= 128);
    const bool narrow_tiles_fill = narrow_ok &&
        bits == 4 && m >= 5 && dp_tiles <= 256 && !two_strip_ok &&
        // (the 32-column case only up to k = 2176 since the per-wave kernel's zeroing protocol runs in a service
        // wavefront: from k = 2304 on two slices of 64-column tiles are 9-26 % ahead on the same grid)
        ((dp_cols == 16 && cgroups <= 26 && dp_tiles >= 130) || (dp_cols == 32 && cgroups <= 17 && dp_tiles >= 170));
    // (the first of them up to k = 2176 from two rows on: a grid of n = 4608..8000, k = 1792 and 2176,
    // m = 2..16 has eight waves per 32-column tile 2-10 % ahead at m = 2, 4 and 18-35 % at m = 8, 16;
    // from k = 2560 on two strips per wave win where they are to be had)
    // (the other field widths: k = 2176 on 249 tiles of 32 columns is 15-42 % slower unsplit at 3 and 8 bits)
    // (two strips per wave first where they are to be had, as above: n = 6144..8192, k = 1536 or 2048, m = 2:
    // 3.55-4.2 us against 3.95-4.65 on unsplit 32-column tiles; n = 9216, k = 1536, m = 2..16: 3.8-4.3 against
    // 4.25-4.9 on unsplit 64-column tiles)
    const bool strips_first = two_strips_there && (bits == 4 || cgroups / 4 >= 4);
    const bool no_split = cgroups <= 8 ||
                          (cgroups <= (m >= 2 && bits == 4 ? 17 : 12) && dp_tiles >= 130 && dp_tiles <= 256 && (narrow_ok || dp_cols == 64) &&
                           !strips_first) ||
                          // (from 120 tiles on: n = 8216, k = 1920, m = 4, 16: 129 tiles unsplit are 17 % ahead of two slices)
                          // (where that launch would use narrow tiles, only while those are in use: n = 8192,
                          // k = 2048, m = 16: 256 tiles of 32 columns unsplit 5.5 us, two strips in four slices 4.5)
                          (cgroups <= 17 && tiles64 >= 120 && tiles64 <= 256 && (narrow_ok || dp_cols == 64) && !strips_first) ||
                          // (k up to 1408 from 100 narrow tiles on: n = 1704..2000, m = 1..16: 27-45 % ahead of two slices)
                          (cgroups <= 11 && dp_tiles >= 100 && dp_tiles <= 256 && (narrow_ok || dp_cols == 64)) ||
                          // (up to k = 3072 only since the streaming kernel's epilogue was shortened: n = 13936,
                          // k = 6144, m = 12 and n = 15672, k = 4992, m = 6 are 7-9 % faster with four slices of it)
                          (m >= 5 && ((cgroups <= 24 && fills_once) || (bits != 4 && m <= 12 && cgroups <= 50 && fills_once))) ||
                          (short_k_tiles_fill && !two_strips_there) || narrow_tiles_fill ||
                          // (more than 256 tiles up to k = 1664: level or up to 25 % ahead on n = 17280..28672)
                          (cgroups <= 13 && tiles64 > 256);
    if ((library_choice || bits_choice) && group_size >= 128 && no_split) {
        // the launch of the data-parallel kernel (the other field widths as well: on 36 random shapes
        // with k up to 3712 their launches became 3-5 % faster on average, up to 35 % on narrow tiles)
        const int tc = dp_cols;
        // (eight waves per narrow tile beyond twelve rows too once k is long: 3-5 % at k = 2304..2816, m = 16)
        const int wv = tc < 64 && (m <= 12 || cgroups >= 18) ? 8 : 4;
        out->split_k = 1;
        out->tile_cols = tc;
        out->waves = cgroups < wv ? largest_wave_split(cgroups, 1, wv) : wv;
        out->reduce = reduce == W4A16_REDUCE_AUTO ? W4A16_REDUCE_ATOMIC_PK_F16_PHASE : reduce;  // not used: split_k == 1
        return W4A16_OK;
    }
    // Two strips per wave (128-column tiles, one compute group per wave, in-kernel zeroing by the
    // service wavefront): when k is short enough for that (k / 128 = 4 split_k with split_k up
    // to 16, i.e. k <= 8192), there is more than one row, at least 160 workgroups, and less
    // than 32 MiB of packed 4-bit weights (25 MiB beyond split_k = 8).  The other field widths go
    // by the number of weights too (what counts is the number of waves and of loads in flight),
    // with their own bounds from a sweep of 11 shapes at m = 2..16: 2-bit fields as 4-bit ones but
    // 24 MiB beyond split_k = 8 (n = k = 7168 loses 5 %), 3-bit and 8-bit fields, which issue two
    // loads per step, 20 MiB (n = 11008 or 12288 with k = 4096 lose 3-9 %, n = k = 8192 8-30 %);
    // inside the bounds two strips gain 5-30 % over the single-strip launch.  0-7 % faster than the
    // single-strip launch with fixed-point adds at m = 2..4, 1-4 % at m = 8..16, and up to 19 %
    // faster than the streaming kernel on matrices of 16-25 MiB.
    // (not where the 64-column tiles alone give 200-256 workgroups: one workgroup per tile over
    // all of k, stored without atomics, is 4-7 % faster there)
    // (the other widths: from split_k = 4 on; with 2 or 3 slices of a short k the tiles alone fill
    // the machine and the unsplit launch is 5-25 % faster, n = 26656, k = 1536 and n = 21952, k = 1024)
    if ((library_choice || (bits_choice && cgroups / 4 >= 4)) && two_strip_ok) {
        out->split_k = cgroups / 4;
        out->tile_cols = 128;
        out->waves = 4;
        out->reduce = W4A16_REDUCE_ATOMIC_PK_F16_PHASE;
        return W4A16_OK;
    }
    // Streaming kernel (256-column tiles, activations shared through LDS): asked for by
    // tile_cols = 256, or chosen when the activation operand is large (m >= 5) and the weight
    // matrix is too big to be requested in one burst, provided the launch has enough workgroups.
    if (!dp && ((bits == 4 && (tile_cols == kStreamTileCols || (tile_cols == 0 && waves == 0))) || bits_choice ||
                (bits != 4 && m > 16))) {
        // more than 16 rows come here only when the streaming kernel can take them
        const bool asked = (bits == 4 && tile_cols == kStreamTileCols) || m > 16;
        const int stiles = (n + kStreamTileCols - 1) / kStreamTileCols;
        const bool shape_ok = group_size == 128 || group_size == 256;
        const bool reduce_ok = reduce == W4A16_REDUCE_AUTO || reduce == W4A16_REDUCE_ATOMIC_PK_F16 ||
                               reduce == W4A16_REDUCE_ATOMIC_PK_F16_PHASE;
        int S = split_k;
        const int S0 = split_k;  // 0: the split is the library's
        int stream_waves = waves;
        if (S == 0) {
            // about one workgroup per compute unit (160 to 319 of them), at least two groups each
            // (at most 32 slices: the packed-fp16 adds round once per slice)
            S = 1;
            while (S * 2 <= 32 && cgroups / (S * 2) >= 2 && stiles * S * 2 <= 256) S *= 2;
            // (never past 256: n = 11008, k = 4096, m = 32: 19.2 us with 258 workgroups against 11.9
            // with 215; n = 16576, k = 1664, m = 8: 8.8 us with 260 against 7.1 without a split)
            if (stiles * S < g_stream_min_blocks && S * 2 <= 32 && cgroups / (S * 2) >= 2 && stiles * S * 2 <= 256)
                S *= 2;
            // A split_k that is no power of two fills the machine where the powers of two leave it
            // under-filled or spill over it: the largest one with at most 256 workgroups, if that
            // gives 192 or more and runs of two groups or more (n = 5120, k = 13824: 12 slices, 240
            // workgroups, 11.6 us against 12.8 with 8 slices; n = 4800, k = 4864, m = 8: 12 slices of
            // three groups, 6.7 us, against 7.2 from the per-wave kernel).
            const int s_fill = 256 / stiles < 32 ? 256 / stiles : 32;
            const bool fill = s_fill >= 3 && (s_fill & (s_fill - 1)) != 0 && stiles * s_fill >= 192 &&
                              (stiles * S < 224 || stiles * S > 256) && cgroups / s_fill >= 2;
            if (fill) S = s_fill;
            // Where that count sits badly on 256 compute units (under 200 or over 256), 128-192
            // workgroups of eight waves do better, if each of their two k parts gets a long run
            // (eight groups or more): twice the loads in flight per compute unit.
            if (!fill && waves == 0 && m <= 16 && (stiles * S < 200 || stiles * S > 256)) {
                int S8 = 1;
                while (stiles * S8 * 2 <= 192) S8 *= 2;
                if (stiles * S8 >= 128 && cgroups % (2 * S8) == 0 && cgroups / (2 * S8) >= 8) {
                    S = S8;
                    stream_waves = 2 * kStreamStrips;
                }
            }
        }
        // Where the count stays under 208 and eight waves (below) are not to be had, close to two
        // workgroups per compute unit (416-512) is the next good place, from 40 MiB of packed weights on:
        // n = 23752, k = 3840, m = 12: 465 workgroups take 12.6 us, 186 take 14.1 and 372 take 13.7;
        // n = 16624, k = 14720, m = 16: 455 take 27.3, 195 take 28.7, 520 take 33.0; n = 22232, k = 7808
        // or 11136, m = 4..16: 435 are 10 % ahead of 174.  (n = 16960, k = 4352, 35 MiB, m = 12: 469 take
        // 12.5 us, 201 take 11.4.)
        bool two_per_unit = false;
        // (not from 208 on: n = 18432, k = 7168 would gain 3-8 % with 504 workgroups instead of 216, but fifteen
        // shapes of four audits with 208-223 lose 2-11 % that way)
        if (bits == 4 && S0 == 0 && stream_waves != 2 * kStreamStrips && waves == 0 && m <= 16 && stiles * S < 208 &&
            weights_half >= (40ll << 20)) {
            const bool eight_to_be_had = bits != 8 && cgroups % (2 * S) == 0 && cgroups / (2 * S) >= 8;
            int s2 = 512 / stiles < 32 ? 512 / stiles : 32;
            if (!eight_to_be_had && s2 > S && stiles * s2 >= 416 && cgroups / s2 >= 4) {
                S = s2;
                two_per_unit = true;
            }
        }
        // Eight waves with the split as chosen, where that leaves compute units idle: a grid of 105
        // launches (43-125 column tiles, 150-256 workgroups, 8-16 groups per k part, m = 1, 6, 16) has
        // eight waves 7-17 % ahead of four at 156-180 workgroups, 4-13 % at 196-198, 0-7 % at 208,
        // 4-5 % at 219-220 with twelve groups or more per part (level with eight), and 1-6 % behind
        // from 240 on.
        // (2-bit and 3-bit fields gain the same way, 7-17 % on eight launches; 8-bit fields, whose waves
        // have twice the bytes in flight already, lose 2-5 %)
        if (bits != 8 && S0 == 0 && stream_waves != 2 * kStreamStrips && waves == 0 && m <= 16 && S >= 1 &&
            cgroups % (2 * S) == 0) {
            const int part_groups = cgroups / (2 * S);
            // (up to 224 with sixteen groups or more per part: n = 28672, k = 8192, m = 16: 23.6 us against 24.9-25.4;
            // n = 28256, k = 11264, m = 1: 28.5 against 30.2)
            // Since the weight loads carry the non-temporal hint eight waves lead further up: 57 launches with
            // 232-256 workgroups (n = 7424..31744, m = 1, 6, 16) have them 2-11 % ahead at 232-236 (29 of 30), 0-10 % at
            // 240 (one of twelve 1 % behind), at 248 3-9 % ahead with twelve groups per part and level or 1.5 %
            // behind with eight, and 5-8 % behind at 256.
            if (part_groups >= 8 && (stiles * S <= 240 || (stiles * S <= 248 && part_groups >= 12)))
                stream_waves = 2 * kStreamStrips;
        }
        const int min_blocks = stream_waves == 2 * kStreamStrips ? 128 : g_stream_min_blocks;
        // Fewer rows: only with a count that sits well, and only on large matrices or where the
        // per-wave kernel's own count (64-column tiles x its split) exceeds the 256 compute units
        // and one group per wave is not to be had (n = 18584, k = 12032, m = 2: 291 workgroups of the per-wave
        // kernel take 35.2 us, 219 of the streaming kernel 24.1).
        int pw_parts = cgroups < 4 ? cgroups : 4;
        while (pw_parts >= 4 && pw_parts * 2 <= cgroups && tiles64 * (pw_parts / 4) < g_stream_min_blocks &&
               tiles64 * (pw_parts / 2) <= 256)
            pw_parts *= 2;
        const int pw_blocks = tiles64 * (pw_parts >= 4 ? pw_parts / 4 : 1);
        // (one group per wave: below 96 MiB; n = 21192, k = 11264, 113 MiB, m = 1, 2: 7300 workgroups
        // of it take 28-29 us, 249 of the streaming kernel 23.6)
        // (below 40 MiB since the streaming epilogue was shortened: n = 23064, k = 8192, 90 MiB, m = 1: 22.6 us
        // against 19.9 with 182 workgroups of eight waves; n = 25112, k = 4096, 49 MiB, m = 2: 14.7 against
        // 12.5; n = 12288, k = 4096, 24 MiB, m = 1 is the largest shape seen where one group per wave leads)
        const bool pw_one_group = bits == 4 && m <= 4 && cgroups % 4 == 0 && cgroups / 4 <= 64 && weights_half < (40ll << 20);
        // (or stays under 160 while the streaming kernel's slices keep five groups or more)
        const bool pw_bad = (pw_blocks > 256 || (pw_blocks < g_stream_min_blocks && cgroups / S >= 5)) && !pw_one_group;
        const bool few_rows_ok = (stream_waves == 2 * kStreamStrips || (stiles * S >= 192 && stiles * S <= 256) || two_per_unit) &&
                                 ((m >= 3 && weights_half >= (48ll << 20)) ||
                                  // (any row count from 16 MiB on when 224-256 workgroups are to be had: 6-13 %
                                  // ahead of one group per wave on six shapes of 44-73 MiB at m = 1, 2, 4; 2-7 % on
                                  // n = k = 8192 at m = 1, 4 and n = 8184, k = 6144 at m = 4 since the epilogue was shortened)
                                  // (from three rows on below 40 MiB: at one row the fixed-point launches stay 1-9 % ahead)
                                  // (at one or two rows as well where k / 128 is no multiple of four, so that one group per
                                  // wave is not to be had: n = 10216, k = 4352, m = 1: 7.4 us against 8.0; n = 3352,
                                  // k = 14592, m = 2: 8.1 against 8.8)
                                  // (not where the 64-column tiles fill the machine once: n = 14160, k = 5504, m = 2: 10.2 us
                                  // unsplit, 10.7 with four slices of the streaming kernel)
                                  // (and from 22 tiles of 256 columns on: with fewer the many slices cost more than they gain,
                                  // n = 4096, k = 11008, m = 1: 7.2 us against 7.0; n = 5120, k = 13696, m = 2: 9.6 against 9.1)
                                  (weights_half >= (((m >= 3 || (cgroups % 4 != 0 && !fills_once && stiles >= 22)) ? 16ll : 40ll) << 20) &&
                                   stream_waves != 2 * kStreamStrips && stiles * S >= 224 && stiles * S <= 256) ||
                                  (weights_half >= (40ll << 20) && two_per_unit) ||
                                  (weights_half > (8ll << 20) && pw_bad &&
                                   // (n = 16984, k = 3200, m = 4: 201 workgroups take 9.5 us, 266 unsplit tiles 11.9;
                                   // n = 16824, k = 3712, m = 1: 198 workgroups 9.6 us, 263 unsplit tiles 12.7)
                                   (stream_waves == 2 * kStreamStrips || stiles * S >= 192)));
        // (from five rows on the per-wave kernel has to use the in-wave zeroing protocol instead
        // of the fixed-point adds, and the streaming kernel wins by up to 22 % at m = 6)
        // The other field widths take the same rules: with the streaming kernel allowed wherever the 4-bit
        // plan allows it, 102 shapes per width (n = 8192..28672 x k = 2048..16384 at m = 2, 6, 16 and 30
        // seeded random ones) are within 0.6-1.1 % (geometric mean) of the best per-wave launch with an
        // explicit split_k, and the shapes this changes are 14-16 % faster on average than under the narrower
        // rules fitted to earlier versions of the two kernels (3-bit fields, n = 16896, k = 12288, m = 6:
        // 23.5 us against 32.4; 2-bit fields, n = 28672, k = 4096, m = 16: 14.0 against 20.3); behind by more
        // than 3 % only at m = 2 (four shapes, up to 7 %) and on n = 22304, k = 3200, m = 6 at 2 bits (5 %).
        // Few column tiles (n up to 2560, up to 3072 with at most eight rows) with five rows or more stay
        // with the per-wave kernel: its slices are 64 columns wide, so a quarter of the streaming kernel's
        // split fills the machine (a quarter of the atomic requests), and with the zeroing protocol in a
        // service wavefront its longer runs no longer lose: n = 1536, k = 12288, m = 6: 4.6 us with ten
        // slices against 6.3 with the streaming kernel's 32; n = 2048, k = 16384, m = 16: 7.3 against 8.9;
        // level from n = 3072 (m = 16) or 4096 (m = 6) on.
        // (and up to n = 4096 while k stays at 9216 or below: n = 3776, k = 8448, m = 16: 6.9 us against 7.6)
        // (and up to n = 8192 while k stays at 4096 or below: n = 6016, k = 3712, m = 12: two slices 5.9 us against 6.6)
        // (every field width: n = 2048, k = 16384, m = 16: 8-bit fields 9.0 us against 10.0, 2-bit 6.1 against 7.2)
        const bool few_tiles = m >= 5 && (stiles <= 10 || (stiles <= 12 && m <= 8) || (stiles <= 16 && cgroups <= 72) ||
                                          (stiles <= 32 && cgroups <= 40));
        // (3-bit fields, whose lanes fetch two word rows per step of which they need one and a half: not with
        // up to eight rows where the 64-column tiles alone give 190-256 workgroups: n = 14144, k = 15488, m = 2, 6:
        // 24.5 us unsplit against 26.7; n = k = 16384: 25.8-26.0 against 27.0-27.1; level at m = 16)
        const bool width_ok = !(bits == 3 && m <= 8 && fills_once);
        const bool worth = S <= cgroups && !few_tiles && width_ok &&
                           ((m >= 5 && weights_half > (8ll << 20) && stiles * S >= min_blocks) || few_rows_ok);
        if (asked || (shape_ok && reduce_ok && worth)) {
            if (!shape_ok || !reduce_ok) return W4A16_ERR_UNSUPPORTED;
            waves = stream_waves;
            if (waves == 0) waves = kStreamStrips;
            if (waves != kStreamStrips && waves != 2 * kStreamStrips) return W4A16_ERR_UNSUPPORTED;
            if (m > 16 * kStreamMaxRowTiles || (m > 16 && waves != kStreamStrips)) return W4A16_ERR_UNSUPPORTED;
            const int wk = waves / kStreamStrips;
            // the two k parts of an 8-wave workgroup meet at one barrier per group: equal counts
            if (S < 1 || S >= (1 << 16) || (long long)S * wk > cgroups || (wk > 1 && cgroups % (S * wk) != 0))
                return W4A16_ERR_SPLIT;
            if (reduce == W4A16_REDUCE_AUTO)
                reduce = phase_split_ok(S) && (size_t)n <= 16 * (size_t)kPhaseOrigins ? W4A16_REDUCE_ATOMIC_PK_F16_PHASE
                                                                                      : W4A16_REDUCE_ATOMIC_PK_F16;
            if (S > 1 && reduce == W4A16_REDUCE_ATOMIC_PK_F16_PHASE &&
                (!phase_split_ok(S) || (size_t)n > 16 * (size_t)kPhaseOrigins))
                return W4A16_ERR_UNSUPPORTED;
            out->split_k = S;
            out->tile_cols = kStreamTileCols;
            out->waves = waves;
            out->reduce = reduce;
            return W4A16_OK;
        }
    }
    if (tile_cols == 0) {
        tile_cols = 64;
        if (dp && bits == 4) {
            // narrower tiles until there are 160 workgroups (sweeps: 160-256 workgroups beat both
            // fewer, wider tiles and more than 256 narrow ones)
            // ... but never beyond 256 (n = 8848: 139 tiles of 64 take 5.6 us, 277 of 32 take 7.4)
            while (tile_cols > 16 && (n + tile_cols - 1) / tile_cols < g_stream_min_blocks &&
                   (n + tile_cols / 2 - 1) / (tile_cols / 2) <= 256)
                tile_cols /= 2;
        }
    }
    // 128 columns: two 64-column strips per wave, one compute group per wave, in-kernel zeroing
    const bool two_strips = tile_cols == 128;
    if (two_strips && (dp || group_size < 128)) return W4A16_ERR_UNSUPPORTED;
    if (tile_cols != 16 && tile_cols != 32 && tile_cols != 64 && !two_strips) return W4A16_ERR_UNSUPPORTED;
    const int tiles = (n + tile_cols - 1) / tile_cols;
    if (dp) {
        split_k = 1;
    } else if (split_k == 0) {
        // Measured on MI355X: a wave either takes exactly one group (little state per wave, many
        // resident waves, every load of the launch in flight at once) or a long run of them
        // (few workgroups, about one per compute unit); runs of two to four groups lose to both.
        int parts = 1;  // k parts of a column tile = split_k * waves
        int own_waves = 4;
        if (m >= 5 && group_size >= 128 && tiles <= 128 && cgroups >= 8) {
            // Five rows or more (packed-fp16 adds, zeroing protocol in a service wavefront): about one
            // workgroup of four waves per compute unit, whatever run length that gives the waves, never
            // less than one group each (n = 1024, k = 16384: 16 slices, 4.4-4.7 us, against 4.8-5.7 with
            // 32; n = k = 4096 without two strips: four slices of two groups per wave 4.65 us, eight
            // slices of one group 5.03).  The other field widths alike (44 seeded shapes with n up to 9600 at
            // m = 6 and 16: 8-bit fields 4-6 % faster in the geometric mean over the shapes this changes, 3-bit
            // and 2-bit fields 12-17 %).
            const int s_max = 256 / tiles < 64 ? 256 / tiles : 64;
            int s = s_max;
            while (s > 1 && 4 * s > cgroups) --s;
            if (tiles * s < 160) {
                // a short k leaves that launch under-filled: two waves per slice with about three groups
                // for the pair (n = 2048, k = 2816: six slices of two waves 3.7 us, five of four 4.3)
                // (one group per wave up to twelve groups: n = 1704, k = 1280: five slices 3.2-3.6 us, four 3.9-4.3)
                const int s2_want = cgroups <= 12 ? cgroups / 2 : (cgroups + 2) / 3;
                const int s2 = s_max < s2_want ? s_max : s2_want;
                // (not where every wave of the four has exactly one group and there are 100 workgroups or more:
                // n = 1408, k = 2560, m = 16: five slices of four waves 3.4 us, seven of two 3.8; 3-bit fields
                // 3.5 against 4.3; n = 1024, k = 4096: eight slices of four 3.6 us, eleven of two 4.05)
                const bool one_each = 4 * s == cgroups && tiles * s >= 100;
                if (s2 > s && !one_each) {
                    s = s2;
                    own_waves = 2;
                }
            } else {
                // ... and of the splits with the same longest run, the smallest that still gives 160 workgroups
                // (k = 12288 on 16 tiles: twelve slices of two groups per wave take 4.2-4.7 us, sixteen slices,
                // half of whose waves take two groups and half one, 4.8-5.6)
                // (one or two groups beyond an even share do not count as a longer run: the one or two waves that
                // have them finish while the machine empties.  k = 12416 (97 groups) on 29 or 32 tiles: eight
                // slices 4.9-5.2 us at m = 6 and 5.8-6.0 at m = 16, seven slices, where every workgroup has a
                // wave with four groups, 5.2-5.5 and 6.25-6.6; k = 8320 (65 groups) on 16 tiles, m = 16: sixteen
                // slices 4.6 us, ten 5.05)
                const int counted = cgroups > 3 ? cgroups - 2 : 1;
                const int longest = (counted + 4 * s - 1) / (4 * s);
                const int s_top = s;
                while (s > 1 && tiles * (s - 1) >= 160 && (counted + 4 * (s - 1) - 1) / (4 * (s - 1)) == longest) --s;
                // ... but first the largest split with at least 128 workgroups whose waves all get the same count, give
                // or take two groups (k = 6272, 49 groups, on 24 tiles: six slices, two groups per wave and one wave
                // with three, 4.2-4.6 us; seven to ten slices 4.4-5.1; k = 4096 on 36 tiles: four slices 4.1 us, five 4.35)
                // (runs of up to three groups only: with longer ones a group more or less weighs little and the
                // number of workgroups decides: k = 3968 on 65 tiles at 8, 3 and 2 bits: three slices 4.6-6.3 us,
                // two slices of four groups per wave 5.3-7.4)
                for (int e = s_top; e >= 2 && tiles * e >= 128; --e) {
                    const int over = cgroups % (4 * e);
                    if ((over <= 2 || over >= 4 * e - 3) && (cgroups + 2) / (4 * e) <= 3) {
                        s = e;
                        break;
                    }
                }
            }
            parts = own_waves * s;
        } else if (packed_bytes <= (8ll << 20)) {
            while (parts * 2 <= cgroups && tiles * parts * 2 <= 2048) parts *= 2;
            // one group per wave where that fits although no power of two gets there (n = 2304, k = 3072,
            // m = 1: six slices of four waves take 3.5 us, four slices with two groups per wave 4.3)
            if (cgroups % 4 == 0 && tiles * cgroups <= 2048) parts = cgroups;
        } else {
            // four waves per workgroup and the fewest k slices that give 160 workgroups
            // (group sizes below 128 make the groups short and the parameter traffic large: sweeps
            // put their optimum at about 450 workgroups or more, and never at one group per wave)
            const int want_blocks = group_size < 128 ? 448 : g_stream_min_blocks;
            parts = cgroups < 4 ? cgroups : 4;
            // (never past 256 workgroups for the long groups: 140 beat 280)
            while (parts >= 4 && parts * 2 <= cgroups && tiles * (parts / 4) < want_blocks &&
                   (group_size < 128 || tiles * (parts / 2) <= 256))
                parts *= 2;
            // Few rows make the atomic traffic of many slices small: where the count above sits
            // badly on 256 compute units, one group per wave does better; and where that is not
            // to be had and there are more workgroups than fit at once, shorter runs (four groups
            // or more) even out the load.
            // a split of any value where the powers of two leave the machine under-filled (the
            // fixed-point adds and the zeroing protocol take any split_k up to 64): n = 2232,
            // k = 14592, m = 4: six slices, 210 workgroups, 6.95 us against 8.0 with four
            if (group_size >= 128 && parts >= 4 && tiles * (parts / 4) < 192) {
                const int s_any = 256 / tiles < 64 ? 256 / tiles : 64;
                if (s_any > parts / 4 && tiles * s_any >= 192 && s_any * 8 <= cgroups) parts = 4 * s_any;
            }
            const int blocks = tiles * (parts >= 4 ? parts / 4 : 1);
            if (group_size < 128) {
                // as chosen above
            } else if (bits == 4 && m <= 4 && cgroups % 4 == 0 && cgroups / 4 <= 64 && packed_bytes < (40ll << 20) &&
                       (blocks < 200 || blocks > 256)) {
                parts = cgroups;
            } else if (blocks > 256) {
                while (parts * 2 <= cgroups && cgroups / (parts * 2) >= 4) parts *= 2;
            }
        }
        int w = waves != 0 ? waves : parts < own_waves ? parts : own_waves;
        if (w > parts) w = parts;
        split_k = parts / w;
        // The library's own choice stays where the reduction is accurate: every packed-fp16 add
        // rounds, so the error grows like sqrt(split_k) * 2e-4 (1.1e-3 at 32, against the
        // tolerance of 2e-3); the fixed-point adds used for up to four rows take 64 slices.
        const int split_cap = m <= 4 ? 64 : 32;
        if (split_k > split_cap) split_k = split_cap;
        if (waves == 0) waves = w;
    }
    if (split_k < 1 || split_k > cgroups) return W4A16_ERR_SPLIT;
    // data-parallel, narrow tiles: eight waves divide k for up to twelve rows, four beyond (sweeps)
    if (waves == 0) waves = largest_wave_split(cgroups, split_k, dp && tile_cols < 64 && m <= 12 ? 8 : 4);
    if (waves < 1 || waves > 16 || (long long)split_k * waves > cgroups) return W4A16_ERR_UNSUPPORTED;
    if (reduce == W4A16_REDUCE_AUTO) {
        // few rows: the arrival-counting fixed-point adds finish in one round trip with no
        // zero-fill launch.  Many rows: returning 64-bit atomics cost more than the fill launch
        // that the packed-fp16 adds need.
        reduce = (m <= 4 && split_k <= 64) ? W4A16_REDUCE_ATOMIC_FIXED
                 : phase_split_ok(split_k)  ? W4A16_REDUCE_ATOMIC_PK_F16_PHASE
                                            : W4A16_REDUCE_ATOMIC_PK_F16;
    }
    if (two_strips) {
        if (split_k * waves != cgroups || waves > 4 || split_k < 2) return W4A16_ERR_UNSUPPORTED;
        // the only reduction of this launch; an explicit request for another one is refused, not rewritten
        if (reduce_asked == W4A16_REDUCE_AUTO) reduce = W4A16_REDUCE_ATOMIC_PK_F16_PHASE;
        if (reduce != W4A16_REDUCE_ATOMIC_PK_F16_PHASE) return W4A16_ERR_UNSUPPORTED;
    }
    if (reduce < W4A16_REDUCE_ATOMIC_F32 || reduce > W4A16_REDUCE_ATOMIC_PK_F16_PHASE) return W4A16_ERR_UNSUPPORTED;
    if (reduce == W4A16_REDUCE_ATOMIC_FIXED && split_k > 64) return W4A16_ERR_UNSUPPORTED;
    // (a launch that does not split k stores directly: whatever reduction is named is not used,
    // so a plan that this function reported can be passed back as it is)
    if (split_k > 1 && reduce == W4A16_REDUCE_ATOMIC_PK_F16_PHASE && !phase_split_ok(split_k)) return W4A16_ERR_UNSUPPORTED;
    out->split_k = split_k;
    out->tile_cols = tile_cols;
    out->waves = waves;
    out->reduce = reduce;
    return W4A16_OK;
}

// Grow-only device buffer.  Growth happens on the first call that needs the size, outside any
// timed region (allocation and a synchronous clear), never while `stream` is being captured into
// a graph, and never frees: the outgrown buffer is retired (see DeviceScratch).
static int grow(DeviceScratch& s, Buffer& b, size_t bytes, size_t floor_bytes, hipStream_t stream, bool* grew)
{
    if (b.bytes >= bytes) return W4A16_OK;
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (!W4A16_HIP(hipStreamIsCapturing(stream, &capturing))) return W4A16_ERR_HIP;
    if (capturing != hipStreamCaptureStatusNone) {
        snprintf(g_hip_detail, sizeof(g_hip_detail),
                 "split-k scratch has to be allocated before a capture: run the call once eagerly, or use "
                 "w4a16_reserve_scratch or w4a16_set_workspace");
        return W4A16_ERR_STATE;
    }
    if (b.ptr) {
        if (s.retired_count >= (int)(sizeof(s.retired) / sizeof(s.retired[0]))) return W4A16_ERR_UNSUPPORTED;
        s.retired[s.retired_count++] = b.ptr;
    }
    if (bytes < floor_bytes) bytes = floor_bytes;
    if (bytes < 2 * b.bytes) bytes = 2 * b.bytes;  // few retirements
    b.ptr = nullptr;
    b.bytes = 0;
    if (!W4A16_HIP(hipMalloc(&b.ptr, bytes))) return W4A16_ERR_HIP;
    if (!W4A16_HIP(hipMemset(b.ptr, 0, bytes))) return W4A16_ERR_HIP;
    b.bytes = bytes;
    *grew = true;
    return W4A16_OK;
}

// Has a wait of the phase protocol run out on this device since the scratch was last released?
// (a read of pinned host memory: no synchronisation)
static bool sticky_error(const DeviceScratch& s) { return s.err_host && *(volatile uint32_t*)s.err_host != 0u; }

static Binding* find_binding(int dev, hipStream_t stream)
{
    for (Binding& b : g_bindings)
        if (b.base && b.dev == dev && b.stream == stream) return &b;
    return nullptr;
}

// The pointers a call needs, from the source `kind` names.  kScratchLibrary: the workspace bound
// to `stream` if there is one, else the library's own buffers (allocated here on first need).
// kScratchStatic: the static array; nothing is allocated, sizes beyond it are W4A16_ERR_LIMIT.
static int resolve_scratch(int kind, hipStream_t stream, const ScratchNeed& need, ScratchView* out)
{
    if (need.phase_split < 0 || need.phase_split > kPhaseMaxSplit) return W4A16_ERR_UNSUPPORTED;
    int dev = 0;
    if (!W4A16_HIP(hipGetDevice(&dev))) return W4A16_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return W4A16_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    *out = ScratchView{};
    if (kind == kScratchStatic) {
        if (need.sums_floats || need.partial_floats || need.ticket_count) return W4A16_ERR_UNSUPPORTED;
        if (need.n > kStaticMaxN || need.fixed_words > kStaticFixedWords || need.phase_split > kStaticPhaseMaxSplit)
            return W4A16_ERR_LIMIT;
        if (!g_static_ptr[dev]) {
            // once per device, with that device current: the array's name is a host-side stand-in,
            // its address on this device comes from the runtime
            uint32_t* ptr = nullptr;
            if (!W4A16_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)))) return W4A16_ERR_HIP;
            if (!ptr) return W4A16_ERR_HIP;
            g_static_ptr[dev] = ptr;
        }
        uint32_t* base = g_static_ptr[dev];
        out->errors = base;
        out->fixed = (uint64_t*)(base + kStaticHeadWords);
        if (need.phase_split) {
            out->flags = base + static_level_offset(need.phase_split);
            out->counts = out->flags + kStaticOrigins;
        }
        return W4A16_OK;
    }
    DeviceScratch& s = g_scratch[dev];
    if (sticky_error(s)) return W4A16_ERR_STATE;
    if (const Binding* b = find_binding(dev, stream)) {
        if (need.n > b->n_max) return W4A16_ERR_LIMIT;
        out->errors = b->base;
        out->err_host = s.err_host;
        out->tickets = b->base + 64;
        if (need.phase_split) {
            out->flags = b->base + workspace_level_offset(b->n_max, need.phase_split);
            out->counts = out->flags + phase_counts_offset();
        }
        out->sums = (float*)(b->base + workspace_sums_offset(b->n_max));
        out->fixed = (uint64_t*)(b->base + workspace_fixed_offset(b->n_max));
        if (need.partial_floats) {
            // the partial tiles of the workspace flavour have no bound: they stay in the library's buffer
            bool grew_partials = false;
            const int rcp = grow(s, s.partials, need.partial_floats * sizeof(float), 0, stream, &grew_partials);
            if (rcp != W4A16_OK) return rcp;
            if (grew_partials && !W4A16_HIP(hipDeviceSynchronize())) return W4A16_ERR_HIP;
            out->partials = (float*)s.partials.ptr;
        }
        return W4A16_OK;
    }
    bool grew = false;
    // sized for sixteen rows whatever m is, and at first for n = 16384, so that the usual shapes
    // never grow a buffer twice
    const size_t rows16 = (size_t)16 * (size_t)need.n;
    const size_t sums_floats = need.sums_floats ? (need.sums_floats > rows16 ? need.sums_floats : rows16) : 0;
    const size_t fixed_words = need.fixed_words ? (need.fixed_words > rows16 ? need.fixed_words : rows16) : 0;
    int rc = grow(s, s.sums, sums_floats * sizeof(float), (size_t)16 * 16384 * sizeof(float), stream, &grew);
    if (rc == W4A16_OK) rc = grow(s, s.partials, need.partial_floats * sizeof(float), 0, stream, &grew);
    if (rc == W4A16_OK) rc = grow(s, s.fixed, fixed_words * sizeof(uint64_t), (size_t)16 * 16384 * sizeof(uint64_t), stream, &grew);
    if (rc == W4A16_OK) rc = grow(s, s.tickets, need.ticket_count * sizeof(uint32_t), 4096 * sizeof(uint32_t), stream, &grew);
    if (rc == W4A16_OK && need.phase_split) {
        rc = grow(s, s.phase_level[need.phase_split], phase_level_words(need.phase_split) * sizeof(uint32_t), 0, stream, &grew);
        if (rc == W4A16_OK) rc = grow(s, s.phase_err, sizeof(uint32_t), 256, stream, &grew);
        if (rc == W4A16_OK && !s.err_host) {
            if (!W4A16_HIP(hipHostMalloc((void**)&s.err_host, 256, hipHostMallocMapped))) return W4A16_ERR_HIP;
            *s.err_host = 0u;
        }
    }
    if (rc != W4A16_OK) return rc;
    if (grew && !W4A16_HIP(hipDeviceSynchronize())) return W4A16_ERR_HIP;
    out->sums = (float*)s.sums.ptr;
    out->partials = (float*)s.partials.ptr;
    out->fixed = (uint64_t*)s.fixed.ptr;
    out->tickets = (uint32_t*)s.tickets.ptr;
    if (need.phase_split) {
        out->flags = (uint32_t*)s.phase_level[need.phase_split].ptr;
        out->counts = out->flags + phase_counts_offset();
    }
    out->errors = (uint32_t*)s.phase_err.ptr;
    out->err_host = s.err_host;
    return W4A16_OK;
}

template <int V, int IPG, int MODE, int WMAX, int GC, int BITS = 4, int NS = 1>
static int launch_bound(const GemmArgs& a, int waves, size_t lds_bytes, hipStream_t stream)
{
    auto kern = gemm_kernel<V, IPG, MODE, WMAX, GC, BITS, NS>;
    if (lds_bytes > 64 * 1024) {
        if (!W4A16_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes)))
            return W4A16_ERR_HIP;
    }
    const unsigned threads = (unsigned)(waves + (MODE == kAtomicPkF16Service ? 1 : 0)) * kWave;
    // (the second grid dimension holds at most 65535)
    if (a.m > 31 || a.param_shift > 3 || a.waves > 31 || a.groups_base >= (1 << 20) || a.tiles >= (1 << 20) ||
        a.groups_rem >= (1 << 11) || a.split_k < 1 || a.split_k >= (1 << 16))
        return W4A16_ERR_UNSUPPORTED;
    const int packed = a.m | a.param_shift << 5 | a.waves << 7 | (int)((unsigned)a.groups_base << 12);
    const int tiles_rem = a.tiles | a.groups_rem << 20;
    GemmRest rest;
    rest.scratch = a.scratch;
    rest.tickets = a.tickets;
    rest.flags = a.flags;
    rest.counts = a.counts;
    rest.errors = a.errors;
    rest.err_host = a.err_host;
    rest.split_k = a.split_k;
    rest.lds_wave_bytes = a.lds_wave_bytes;
    rest.spin_limit = a.spin_limit;
    rest.probe_delay = a.probe_delay;
    hipLaunchKernelGGL(kern, dim3((unsigned)a.tiles, (unsigned)a.split_k), dim3(threads), lds_bytes, stream, a.A,
                       a.qweight, a.scales, a.qzeros, a.C, packed, a.n, a.k, tiles_rem, rest);
    return W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

template <int V, int IPG, int MODE>
static int launch_one(const GemmArgs& a, int waves, size_t lds_bytes, hipStream_t stream)
{
    if (waves <= 4) {
        // the tuned shape (128-bit loads, group of 128) knows its group count at compile time
        if constexpr (V == 4 && IPG == 4) {
            if (a.groups_base == 1 && a.groups_rem == 0) {
                // few registers per wave: the phase protocol gets a wave of its own
                if constexpr (MODE == kAtomicPkF16Phase)
                    return launch_bound<V, IPG, kAtomicPkF16Service, 4, 1>(a, waves, lds_bytes, stream);
                else
                    return launch_bound<V, IPG, MODE, 4, 1>(a, waves, lds_bytes, stream);
            }
            // (longer runs too: run inside wave 0, the protocol puts a wait for the second batch of kernel
            // arguments and the zero stores ahead of every wave's first load)
            if constexpr (MODE == kAtomicPkF16Phase) {
                if (a.groups_base >= 2) return launch_bound<V, IPG, kAtomicPkF16Service, 4, 2>(a, waves, lds_bytes, stream);
                return launch_bound<V, IPG, kAtomicPkF16Service, 4, 0>(a, waves, lds_bytes, stream);
            } else {
                if (a.groups_base >= 2) return launch_bound<V, IPG, MODE, 4, 2>(a, waves, lds_bytes, stream);
                return launch_bound<V, IPG, MODE, 4, 0>(a, waves, lds_bytes, stream);
            }
        } else {
            return launch_bound<V, IPG, MODE, 4, 0>(a, waves, lds_bytes, stream);
        }
    }
    if constexpr (V == 4 && IPG == 4) {
        // one group per wave needs few registers, so large workgroups lose nothing
        if (a.groups_base == 1 && a.groups_rem == 0) return launch_bound<V, IPG, MODE, 16, 1>(a, waves, lds_bytes, stream);
    }
    return launch_bound<V, IPG, MODE, 16, 0>(a, waves, lds_bytes, stream);
}

template <int V, int IPG>
static int launch_mode(const GemmArgs& a, int waves, size_t lds_bytes, int mode, hipStream_t stream)
{
    switch (mode) {
    case kDirect: return launch_one<V, IPG, kDirect>(a, waves, lds_bytes, stream);
    case kAtomicF32: return launch_one<V, IPG, kAtomicF32>(a, waves, lds_bytes, stream);
    case kAtomicPkF16: return launch_one<V, IPG, kAtomicPkF16>(a, waves, lds_bytes, stream);
    case kWorkspace: return launch_one<V, IPG, kWorkspace>(a, waves, lds_bytes, stream);
    case kAtomicFixed: return launch_one<V, IPG, kAtomicFixed>(a, waves, lds_bytes, stream);
    default: return launch_one<V, IPG, kAtomicPkF16Phase>(a, waves, lds_bytes, stream);
    }
}

template <int V>
static int launch_ipg(const GemmArgs& a, int ipg, int waves, size_t lds_bytes, int mode, hipStream_t stream)
{
    switch (ipg) {
    case 1: return launch_mode<V, 1>(a, waves, lds_bytes, mode, stream);
    case 2: return launch_mode<V, 2>(a, waves, lds_bytes, mode, stream);
    default: return launch_mode<V, 4>(a, waves, lds_bytes, mode, stream);
    }
}

// ---- 2-bit, 3-bit and 8-bit fields, per-wave kernel with a split: 64-column tiles, at most four waves per workgroup
template <int IPG, int MODE, int BITS>
static int launchn_one(const GemmArgs& a, int waves, size_t lds_bytes, hipStream_t stream)
{
    if (waves > 4) return W4A16_ERR_UNSUPPORTED;
    // (groups of 128: the phase protocol in a wavefront of its own, as for 4-bit fields)
    constexpr int kMode = MODE == kAtomicPkF16Phase && IPG == 4 ? kAtomicPkF16Service : MODE;
    if (a.groups_base >= 2) return launch_bound<4, IPG, kMode, 4, 2, BITS>(a, waves, lds_bytes, stream);
    return launch_bound<4, IPG, kMode, 4, 0, BITS>(a, waves, lds_bytes, stream);
}

template <int IPG, int BITS>
static int launchn_mode(const GemmArgs& a, int waves, size_t lds_bytes, int mode, hipStream_t stream)
{
    switch (mode) {
    case kDirect: return launchn_one<IPG, kDirect, BITS>(a, waves, lds_bytes, stream);
    // (the entry points of these widths take no `reduce`: the plan's three flavours only)
    case kAtomicF32: return W4A16_ERR_UNSUPPORTED;
    case kWorkspace: return W4A16_ERR_UNSUPPORTED;
    case kAtomicPkF16: return launchn_one<IPG, kAtomicPkF16, BITS>(a, waves, lds_bytes, stream);
    case kAtomicFixed: return launchn_one<IPG, kAtomicFixed, BITS>(a, waves, lds_bytes, stream);
    default: return launchn_one<IPG, kAtomicPkF16Phase, BITS>(a, waves, lds_bytes, stream);
    }
}

template <int BITS>
static int launchn_ipg(const GemmArgs& a, int ipg, int waves, size_t lds_bytes, int mode, hipStream_t stream)
{
    switch (ipg) {
    case 1: return launchn_mode<1, BITS>(a, waves, lds_bytes, mode, stream);
    case 2: return launchn_mode<2, BITS>(a, waves, lds_bytes, mode, stream);
    default: return launchn_mode<4, BITS>(a, waves, lds_bytes, mode, stream);
    }
}

// ---- the other field widths, data-parallel launch with narrow tiles (16 or 32 columns, up to 16 waves)
template <int V, int BITS>
static int launchn_direct_narrow(const GemmArgs& a, int ipg, int waves, size_t lds_bytes, hipStream_t stream)
{
    if (waves <= 4) {
        switch (ipg) {
        case 1: return launch_bound<V, 1, kDirect, 4, 0, BITS>(a, waves, lds_bytes, stream);
        case 2: return launch_bound<V, 2, kDirect, 4, 0, BITS>(a, waves, lds_bytes, stream);
        default: return launch_bound<V, 4, kDirect, 4, 0, BITS>(a, waves, lds_bytes, stream);
        }
    }
    switch (ipg) {
    case 1: return launch_bound<V, 1, kDirect, 16, 0, BITS>(a, waves, lds_bytes, stream);
    case 2: return launch_bound<V, 2, kDirect, 16, 0, BITS>(a, waves, lds_bytes, stream);
    default: return launch_bound<V, 4, kDirect, 16, 0, BITS>(a, waves, lds_bytes, stream);
    }
}

template <int BITS>
static int launchn_direct_narrow_v(const GemmArgs& a, int V, int ipg, int waves, size_t lds_bytes, hipStream_t stream)
{
    if (V == 1) return launchn_direct_narrow<1, BITS>(a, ipg, waves, lds_bytes, stream);
    return launchn_direct_narrow<2, BITS>(a, ipg, waves, lds_bytes, stream);
}

// ---- launch of the streaming SplitK kernel
template <int D, int MODE, int MT, int BITS = 4>
static int launch_stream_one(const StreamArgs& a, size_t lds_bytes, hipStream_t stream)
{
    auto kern = gemm_stream_kernel<D, MODE, MT, BITS>;
    if (lds_bytes > 64 * 1024) {
        if (!W4A16_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes)))
            return W4A16_ERR_HIP;
    }
    // (the second grid dimension holds at most 65535)
    if (a.m > 16 * MT || (MT > 1 && a.wk != 1) || a.wk > 2 || a.groups_base >= (1 << 20) || a.split_k < 1 ||
        a.split_k >= (1 << 16) || a.groups_rem >= (1 << 15) || a.tiles < 1 || a.tiles >= (1 << 16))
        return W4A16_ERR_UNSUPPORTED;
    const int packed = a.m | a.param_shift << 7 | a.wk << 9 | (int)((unsigned)a.groups_base << 12);
    const int split_rem = a.split_k | a.groups_rem << 16;
    StreamRest rest;
    rest.flags = a.flags;
    rest.counts = a.counts;
    rest.errors = a.errors;
    rest.err_host = a.err_host;
    rest.spin_limit = a.spin_limit;
    rest.probe_delay = a.probe_delay;
    hipLaunchKernelGGL(kern, dim3((unsigned)a.split_k, (unsigned)a.tiles), dim3((unsigned)(kStreamStrips * a.wk) * kWave), lds_bytes, stream, a.A,
                       a.qweight, a.scales, a.qzeros, a.C, packed, a.n, a.k, split_rem, rest);
    return W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

template <int D, int MT, int BITS = 4>
static int launch_stream_mode(const StreamArgs& a, size_t lds_bytes, int mode, hipStream_t stream)
{
    if (mode == kDirect) return launch_stream_one<D, kDirect, MT, BITS>(a, lds_bytes, stream);
    if (mode == kAtomicPkF16) return launch_stream_one<D, kAtomicPkF16, MT, BITS>(a, lds_bytes, stream);
    return launch_stream_one<D, kAtomicPkF16Phase, MT, BITS>(a, lds_bytes, stream);
}

template <int MT, int BITS = 4>
static int launch_stream_tiles(const StreamArgs& a, size_t lds_bytes, int mode, hipStream_t stream)
{
    // ring depth: two groups in flight per wave when every k part has at least two
    if (a.groups_base >= 2 && g_stream_depth >= 2) return launch_stream_mode<2, MT, BITS>(a, lds_bytes, mode, stream);
    return launch_stream_mode<1, MT, BITS>(a, lds_bytes, mode, stream);
}

// mt row tiles of 16 activation rows share one pass over the weights, at every field width
template <int BITS>
static int launch_stream_rows(const StreamArgs& a, int mt, size_t lds_bytes, int mode, hipStream_t stream)
{
    switch (mt) {
    case 1: return launch_stream_tiles<1, BITS>(a, lds_bytes, mode, stream);
    case 2: return launch_stream_tiles<2, BITS>(a, lds_bytes, mode, stream);
    case 3: return launch_stream_tiles<3, BITS>(a, lds_bytes, mode, stream);
    default: return launch_stream_tiles<4, BITS>(a, lds_bytes, mode, stream);
    }
}

// tile_cols = 256; waves = 4 * (k parts per workgroup), 4 or 8.  group_size 128 or 256.
// m <= 64; more than 16 rows need waves = 4.
static int run_stream(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                      int n, int k, int group_size, int split_k, int waves, int reduce, hipStream_t stream, int bits = 4,
                      int scratch_kind = kScratchLibrary)
{
    if (group_size != 128 && group_size != 256) return W4A16_ERR_UNSUPPORTED;
    if (waves == 0) waves = kStreamStrips;
    if (waves != kStreamStrips && waves != 2 * kStreamStrips) return W4A16_ERR_UNSUPPORTED;
    const int wk = waves / kStreamStrips;
    const int mt = (m + 15) / 16;  // row tiles
    if (mt > kStreamMaxRowTiles || (mt > 1 && wk != 1)) return W4A16_ERR_UNSUPPORTED;
    const int groups = k / 128;
    // the two k parts of an 8-wave workgroup meet at one barrier per group: equal counts
    if (split_k < 1 || (long long)split_k * wk > groups || (wk > 1 && groups % (split_k * wk) != 0))
        return W4A16_ERR_SPLIT;
    if (reduce == W4A16_REDUCE_AUTO)
        reduce = phase_split_ok(split_k) && (size_t)n <= 16 * (size_t)kPhaseOrigins ? W4A16_REDUCE_ATOMIC_PK_F16_PHASE
                                                                                  : W4A16_REDUCE_ATOMIC_PK_F16;
    if (reduce != W4A16_REDUCE_ATOMIC_PK_F16 && reduce != W4A16_REDUCE_ATOMIC_PK_F16_PHASE)
        return W4A16_ERR_UNSUPPORTED;
    StreamArgs a;
    a.A = (const _Float16*)A;
    a.qweight = (const uint32_t*)qweight;
    a.scales = (const _Float16*)scales;
    a.qzeros = (const uint32_t*)qzeros;
    a.C = (_Float16*)C;
    a.flags = a.counts = a.errors = a.err_host = nullptr;
    a.m = m;
    a.n = n;
    a.k = k;
    a.tiles = (n + kStreamTileCols - 1) / kStreamTileCols;
    a.split_k = split_k;
    a.wk = wk;
    a.groups_base = groups / (split_k * wk);
    a.groups_rem = groups % (split_k * wk);
    a.param_shift = group_size == 256 ? 1 : 0;
    a.spin_limit = g_spin_limit;
    a.probe_delay = g_probe_delay;
    // (one row tile: whole 16-row tiles whatever m is, which the epilogue indexes with constants)
    const size_t lds_bytes = (size_t)wk * 2 * mt * kChunkBytes + (size_t)waves * (mt == 1 ? 16 : m) * 64 * 4;
    int mode = kDirect;
    if (split_k > 1) {
        if (reduce == W4A16_REDUCE_ATOMIC_PK_F16_PHASE) {
            if (!phase_split_ok(split_k) || (size_t)n > 16 * (size_t)kPhaseOrigins) return W4A16_ERR_UNSUPPORTED;
            ScratchNeed need;
            need.phase_split = split_k;
            need.n = n;
            ScratchView view;
            const int rc = resolve_scratch(scratch_kind, stream, need, &view);
            if (rc != W4A16_OK) return rc;
            a.flags = view.flags;
            a.counts = view.counts;
            a.errors = view.errors;
            a.err_host = view.err_host;
            mode = kAtomicPkF16Phase;
        } else {
            const size_t words = (size_t)m * n / 2;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                               (uint32_t*)C, words);
            if (!W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
            mode = kAtomicPkF16;
        }
    }
    switch (bits) {
    case 8: return launch_stream_rows<8>(a, mt, lds_bytes, mode, stream);
    case 3: return launch_stream_rows<3>(a, mt, lds_bytes, mode, stream);
    case 2: return launch_stream_rows<2>(a, mt, lds_bytes, mode, stream);
    default: return launch_stream_rows<4>(a, mt, lds_bytes, mode, stream);
    }
}

// Can a call with these knobs use the streaming kernel with more than one row tile?
static bool stream_rows_ok(int group_size, bool dp, int tile_cols, int waves, int reduce)
{
    return !dp && (group_size == 128 || group_size == 256) && (tile_cols == 0 || tile_cols == kStreamTileCols) &&
           (waves == 0 || waves == kStreamStrips) &&
           (reduce == W4A16_REDUCE_AUTO || reduce == W4A16_REDUCE_ATOMIC_PK_F16 ||
            reduce == W4A16_REDUCE_ATOMIC_PK_F16_PHASE);
}

// StreamK variant: `workgroups` persistent workgroups (0 = one per compute unit, the best count
// in sweeps; capped by the number of iterations).  group_size 128 or 256; m <= 16 per launch.
static int run_streamk(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                       int n, int k, int group_size, int workgroups, hipStream_t stream, int bits = 4)
{
    if (group_size != 128 && group_size != 256) return W4A16_ERR_UNSUPPORTED;
    if ((unsigned long long)k * (unsigned long long)n * (unsigned)bits / 8 >= (1ull << 31)) return W4A16_ERR_UNSUPPORTED;
    const int groups = k / 128;
    const int tiles = (n + kStreamTileCols - 1) / kStreamTileCols;
    const long long total = (long long)tiles * groups;
    if (workgroups < 0) return W4A16_ERR_UNSUPPORTED;
    if (workgroups == 0) workgroups = g_streamk_blocks;
    if (workgroups > total) workgroups = (int)total;
    // no tile is shared between workgroups: nothing to add up, nothing to zero
    const bool whole_tiles = total % workgroups == 0 && (total / workgroups) % groups == 0;
    if (!whole_tiles) {
        const size_t words = (size_t)m * n / 2;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                           (uint32_t*)C, words);
        if (!W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
    }
    const int packed = m | (group_size == 256 ? 1 : 0) << 7;
    const size_t lds_bytes = 2 * kChunkBytes + (size_t)kStreamStrips * m * 64 * 4;
    auto launch = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3((unsigned)workgroups), dim3(kStreamStrips * kWave), lds_bytes, stream,
                           (const _Float16*)A, (const uint32_t*)qweight, (const _Float16*)scales,
                           (const uint32_t*)qzeros, (_Float16*)C, packed, n, k, workgroups);
    };
    switch (bits) {
    case 8: launch(gemm_streamk_kernel<8>); break;
    case 3: launch(gemm_streamk_kernel<3>); break;
    case 2: launch(gemm_streamk_kernel<2>); break;
    default: launch(gemm_streamk_kernel<4>); break;
    }
    return W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

static void read_tuning_env()
{
    static bool done = false;
    if (done) return;
    done = true;
    // a value outside its range is ignored (the default stays)
    auto read = [](const char* name, int lo, int hi, int* value) {
        const char* e = getenv(name);
        if (!e || !*e) return;
        char* end = nullptr;
        const long v = strtol(e, &end, 10);
        if (end && *end == '\0' && v >= lo && v <= hi) *value = (int)v;
    };
    read("W4A16_PROBE_DELAY", 0, 64, &g_probe_delay);
    read("W4A16_STREAM_DEPTH", 1, 2, &g_stream_depth);
    read("W4A16_STREAM_MIN_BLOCKS", 1, 1024, &g_stream_min_blocks);
    read("W4A16_STREAMK_BLOCKS", 1, 65535, &g_streamk_blocks);
}

static int run_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                    int n, int k, int group_size, bool dp, int split_k, int tile_cols, int waves, int reduce,
                    bool even_split, void* stream_v, int bits = 4, int scratch_kind = kScratchLibrary)
{
    if (!A || !qweight || !scales || !qzeros || !C) return W4A16_ERR_NULL;
    read_tuning_env();
    int rc = check_args(m, n, k, group_size, dp ? 1 : split_k, even_split);
    if (rc != W4A16_OK) return rc;
    if (!aligned16(A) || !aligned16(qweight) || !aligned16(scales) || !aligned16(qzeros) || !aligned16(C))
        return W4A16_ERR_UNSUPPORTED;
    if ((unsigned long long)k * (unsigned long long)n * (unsigned)bits / 8 >= (1ull << 31)) return W4A16_ERR_UNSUPPORTED;
    if (bits == 2 && (n % 16) != 0) return W4A16_ERR_SHAPE;  // a zero word holds sixteen columns
    if (bits == 3 && (n % 32) != 0) return W4A16_ERR_SHAPE;  // three zero words hold thirty-two columns
    // More than 16 rows (beyond the paper's regime): the streaming kernel takes up to 64 rows as
    // row tiles of one launch, so the weights stream once per 64 rows; whatever it does not
    // cover (data-parallel kernel, group sizes below 128, the other tile widths and reductions)
    // runs as one launch per 16 rows.
    const int rows_per_launch = stream_rows_ok(group_size, dp, tile_cols, waves, reduce) ? 16 * kStreamMaxRowTiles : 16;
    if (m > rows_per_launch) {
        for (int r = 0; r < m; r += rows_per_launch) {
            const int mm = m - r < rows_per_launch ? m - r : rows_per_launch;
            rc = run_gemm((const _Float16*)A + (size_t)r * k, qweight, scales, qzeros, (_Float16*)C + (size_t)r * n, mm,
                          n, k, group_size, dp, split_k, tile_cols, waves, reduce, even_split, stream_v, bits,
                          scratch_kind);
            if (rc != W4A16_OK) return rc;
        }
        return W4A16_OK;
    }
    Plan plan;
    rc = make_plan(m, n, k, group_size, dp, split_k, tile_cols, waves, reduce, &plan, bits);
    if (rc != W4A16_OK) return rc;
    if (plan.tile_cols == kStreamTileCols) {
        if ((unsigned long long)k * (unsigned long long)n / 2 >= (1ull << 31)) return W4A16_ERR_UNSUPPORTED;
        return run_stream(A, qweight, scales, qzeros, C, m, n, k, group_size, plan.split_k, plan.waves, plan.reduce,
                          (hipStream_t)stream_v, bits, scratch_kind);
    }

    hipStream_t stream = (hipStream_t)stream_v;
    const int ipg = group_size >= 128 ? 4 : group_size / 32;  // MFMA steps (32 k each) per compute group
    const int param_shift = group_size == 256 ? 1 : 0;
    const bool two_strips = plan.tile_cols == 128;
    const int V = two_strips ? 4 : plan.tile_cols / 16;
    GemmArgs a;
    a.A = (const _Float16*)A;
    a.qweight = (const uint32_t*)qweight;
    a.scales = (const _Float16*)scales;
    a.qzeros = (const uint32_t*)qzeros;
    a.C = (_Float16*)C;
    a.scratch = nullptr;
    a.tickets = nullptr;
    a.m = m;
    a.n = n;
    a.k = k;
    a.tiles = (n + plan.tile_cols - 1) / plan.tile_cols;
    a.split_k = plan.split_k;
    const int cgroups = k / (32 * ipg), kparts = plan.split_k * plan.waves;
    a.groups_base = cgroups / kparts;
    a.groups_rem = cgroups % kparts;
    a.waves = plan.waves;
    a.param_shift = param_shift;
    // LDS: 16 bytes for the phase word, then one [m, tile_cols] fp32 tile per wave, for the sum
    // over the workgroup's waves
    // (two strips per wave: whole 16-row tiles whatever m is, which the four-wave epilogue indexes with constants)
    a.lds_wave_bytes = two_strips ? 16 * 128 * 4 : (m * plan.tile_cols * 4 + 15) & ~15;
    const size_t lds_bytes = 16 + (size_t)a.lds_wave_bytes * plan.waves;
    a.flags = nullptr;
    a.counts = nullptr;
    a.errors = nullptr;
    a.err_host = nullptr;
    a.spin_limit = g_spin_limit;
    a.probe_delay = g_probe_delay;
    if (lds_bytes > 160 * 1024) return W4A16_ERR_UNSUPPORTED;

    int mode = kDirect;
    if (plan.split_k > 1) {
        mode = plan.reduce;  // W4A16_REDUCE_* values equal the kernel modes
        if (mode != kAtomicPkF16) {
            if (mode == kAtomicPkF16Phase && (size_t)n > 16 * (size_t)kPhaseOrigins) return W4A16_ERR_UNSUPPORTED;
            ScratchNeed need;
            need.n = n;
            need.sums_floats = mode == kAtomicF32 ? (size_t)m * n : 0;
            need.partial_floats = mode == kWorkspace ? (size_t)plan.split_k * m * n : 0;
            need.fixed_words = mode == kAtomicFixed ? (size_t)m * n : 0;
            need.ticket_count = mode == kAtomicF32 || mode == kWorkspace ? (size_t)a.tiles : 0;
            need.phase_split = mode == kAtomicPkF16Phase ? plan.split_k : 0;
            ScratchView view;
            rc = resolve_scratch(scratch_kind, stream, need, &view);
            if (rc != W4A16_OK) return rc;
            a.scratch = mode == kAtomicF32 ? view.sums : mode == kWorkspace ? view.partials : (float*)view.fixed;
            a.tickets = view.tickets;
            if (mode == kAtomicPkF16Phase) {
                a.flags = view.flags;
                a.counts = view.counts;
                a.errors = view.errors;
                a.err_host = view.err_host;
            }
        } else {
            const size_t words = (size_t)m * n / 2;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                               (uint32_t*)C, words);
            if (!W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
        }
    }
    if (two_strips) {
        if (ipg != 4 || mode != kAtomicPkF16Phase || a.groups_base != 1 || a.groups_rem != 0 || plan.waves > 4)
            return W4A16_ERR_UNSUPPORTED;
        switch (bits) {
        case 8: return launch_bound<4, 4, kAtomicPkF16Service, 4, 1, 8, 2>(a, plan.waves, lds_bytes, stream);
        case 3: return launch_bound<4, 4, kAtomicPkF16Service, 4, 1, 3, 2>(a, plan.waves, lds_bytes, stream);
        case 2: return launch_bound<4, 4, kAtomicPkF16Service, 4, 1, 2, 2>(a, plan.waves, lds_bytes, stream);
        default: return launch_bound<4, 4, kAtomicPkF16Service, 4, 1, 4, 2>(a, plan.waves, lds_bytes, stream);
        }
    }
    if (bits != 4 && V < 4) {
        // narrow tiles: the data-parallel launch only
        if (mode != kDirect) return W4A16_ERR_UNSUPPORTED;
        if (bits == 8) return launchn_direct_narrow_v<8>(a, V, ipg, plan.waves, lds_bytes, stream);
        if (bits == 3) return launchn_direct_narrow_v<3>(a, V, ipg, plan.waves, lds_bytes, stream);
        return launchn_direct_narrow_v<2>(a, V, ipg, plan.waves, lds_bytes, stream);
    }
    if (bits == 8) return launchn_ipg<8>(a, ipg, plan.waves, lds_bytes, mode, stream);
    if (bits == 2) return launchn_ipg<2>(a, ipg, plan.waves, lds_bytes, mode, stream);
    if (bits == 3) return launchn_ipg<3>(a, ipg, plan.waves, lds_bytes, mode, stream);
    switch (V) {
    case 1: return launch_ipg<1>(a, ipg, plan.waves, lds_bytes, mode, stream);
    case 2: return launch_ipg<2>(a, ipg, plan.waves, lds_bytes, mode, stream);
    default: return launch_ipg<4>(a, ipg, plan.waves, lds_bytes, mode, stream);
    }
}

}  // namespace w4a16

// ------------------------------------------------------------------------------------------
extern "C" {

int w4a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
               int k, int group_size, int split_k, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, 0, 0,
                           W4A16_REDUCE_AUTO, true, stream);
}

int w4a16_gemm_static(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                      int n, int k, int group_size, int split_k, void* stream)
{
    // the limits that do not depend on the launch; resolve_scratch checks the rest against the plan
    if (m > 16 || n > w4a16::kStaticMaxN) {
        const int rc = w4a16::check_args(m, n, k, group_size, split_k, true);
        return rc != W4A16_OK ? rc : W4A16_ERR_LIMIT;
    }
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, 0, 0,
                           W4A16_REDUCE_AUTO, true, stream, 4, w4a16::kScratchStatic);
}

int w4a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, 0, 0, W4A16_REDUCE_AUTO,
                           true, stream);
}

int w4a16_gemm_streamk_bits(int bits, const void* A, const void* qweight, const void* scales, const void* qzeros,
                            void* C, int m, int n, int k, int group_size, int workgroups, void* stream)
{
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return W4A16_ERR_UNSUPPORTED;
    if (!A || !qweight || !scales || !qzeros || !C) return W4A16_ERR_NULL;
    w4a16::read_tuning_env();
    int rc = w4a16::check_args(m, n, k, group_size, 1);
    if (rc != W4A16_OK) return rc;
    if ((bits == 2 && (n % 16) != 0) || (bits == 3 && (n % 32) != 0)) return W4A16_ERR_SHAPE;
    if (!w4a16::aligned16(A) || !w4a16::aligned16(qweight) || !w4a16::aligned16(scales) || !w4a16::aligned16(qzeros) ||
        !w4a16::aligned16(C))
        return W4A16_ERR_UNSUPPORTED;
    for (int r = 0; r < m; r += 16) {
        const int mm = m - r < 16 ? m - r : 16;
        rc = w4a16::run_streamk((const _Float16*)A + (size_t)r * k, qweight, scales, qzeros,
                                (_Float16*)C + (size_t)r * n, mm, n, k, group_size, workgroups, (hipStream_t)stream,
                                bits);
        if (rc != W4A16_OK) return rc;
    }
    return W4A16_OK;
}

int w4a16_gemm_streamk(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                       int n, int k, int group_size, int workgroups, void* stream)
{
    return w4a16_gemm_streamk_bits(4, A, qweight, scales, qzeros, C, m, n, k, group_size, workgroups, stream);
}

int w8a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
               int k, int group_size, int split_k, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, 0, 0,
                           W4A16_REDUCE_AUTO, true, stream, 8);
}

int w8a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, 0, 0, W4A16_REDUCE_AUTO,
                           true, stream, 8);
}

int w2a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
               int k, int group_size, int split_k, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, 0, 0,
                           W4A16_REDUCE_AUTO, true, stream, 2);
}

int w2a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, 0, 0, W4A16_REDUCE_AUTO,
                           true, stream, 2);
}

int w3a16_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
               int k, int group_size, int split_k, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, 0, 0,
                           W4A16_REDUCE_AUTO, true, stream, 3);
}

int w3a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, 0, 0, W4A16_REDUCE_AUTO,
                           true, stream, 3);
}

long long w3a16_algorithmic_bytes(int m, int n, int k, int group_size)
{
    if (m < 1 || n < 32 || group_size < 32 || k < group_size) return 0;
    const long long g = k / group_size;
    return (long long)k / 32 * 3 * n * 4 + g * n * 2 + g * (n / 32 * 3) * 4 + (long long)m * k * 2 + (long long)m * n * 2;
}

long long w2a16_algorithmic_bytes(int m, int n, int k, int group_size)
{
    if (m < 1 || n < 16 || group_size < 16 || k < group_size) return 0;
    const long long g = k / group_size;
    return (long long)k * n / 4 + g * n * 2 + g * (n / 16) * 4 + (long long)m * k * 2 + (long long)m * n * 2;
}

long long w8a16_algorithmic_bytes(int m, int n, int k, int group_size)
{
    if (m < 1 || n < 8 || group_size < 8 || k < group_size) return 0;
    const long long g = k / group_size;
    return (long long)k * n + g * n * 2 + g * (n / 4) * 4 + (long long)m * k * 2 + (long long)m * n * 2;
}

int w4a16_actorder_prepare(const void* qweight, const void* g_idx, void* qweight_sorted, void* perm, void* status,
                           int n, int k, int group_size, void* stream)
{
    if (!qweight || !g_idx || !qweight_sorted || !perm || !status) return W4A16_ERR_NULL;
    int rc = w4a16::check_args(1, n, k, group_size, 1);
    if (rc != W4A16_OK) return rc;
    if (qweight == qweight_sorted) return W4A16_ERR_UNSUPPORTED;  // not in place
    hipStream_t st = (hipStream_t)stream;
    // a fill kernel rather than an asynchronous memset, so that the call can be captured into a graph
    hipLaunchKernelGGL(w4a16::fill_zero_kernel, dim3(1), dim3(64), 0, st, (uint32_t*)status, (size_t)1);
    if (!w4a16::W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
    hipLaunchKernelGGL(w4a16::actorder_perm_kernel, dim3((unsigned)(k / group_size)), dim3(256), 0, st,
                       (const int32_t*)g_idx, (int32_t*)perm, (int32_t*)status, k, group_size);
    if (!w4a16::W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
    const size_t words = (size_t)(k / 8) * n;
    hipLaunchKernelGGL(w4a16::actorder_repack_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st,
                       (const uint32_t*)qweight, (const int32_t*)perm, (uint32_t*)qweight_sorted, n, k);
    return w4a16::W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

int w4a16_gemm_actorder(const void* A, const void* qweight_sorted, const void* scales, const void* qzeros,
                        const void* perm, void* A_work, void* C, int m, int n, int k, int group_size, int split_k,
                        void* stream)
{
    if (!A || !qweight_sorted || !scales || !qzeros || !perm || !A_work || !C) return W4A16_ERR_NULL;
    int rc = w4a16::check_args(m, n, k, group_size, split_k);
    if (rc != W4A16_OK) return rc;
    if (!w4a16::aligned16(A_work) || A_work == A) return W4A16_ERR_UNSUPPORTED;
    const size_t elems = (size_t)m * k;
    hipLaunchKernelGGL(w4a16::actorder_gather_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, (const _Float16*)A, (const int32_t*)perm, (_Float16*)A_work, m, k);
    if (!w4a16::W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
    return w4a16::run_gemm(A_work, qweight_sorted, scales, qzeros, C, m, n, k, group_size, false, split_k, 0, 0,
                           W4A16_REDUCE_AUTO, true, stream);
}

int w4a16_gemm_ex(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, int split_k, int tile_cols, int waves, int reduce, void* stream)
{
    if (tile_cols < 0 || waves < 0 || reduce < 0) return W4A16_ERR_UNSUPPORTED;
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, tile_cols, waves,
                           reduce, false, stream);
}

int w4a16_gemm_dp_ex(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                     int n, int k, int group_size, int tile_cols, int waves, void* stream)
{
    if (tile_cols < 0 || waves < 0) return W4A16_ERR_UNSUPPORTED;
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, tile_cols, waves,
                           W4A16_REDUCE_AUTO, true, stream);
}

int w4a16_plan(int m, int n, int k, int group_size, int dp, int* split_k, int* tile_cols, int* waves, int* reduce)
{
    const int req = split_k ? *split_k : 0;
    int rc = w4a16::check_args(m, n, k, group_size, dp ? 1 : req, false);
    if (rc != W4A16_OK) return rc;
    w4a16::Plan plan;
    // more rows than one launch takes: the plan of each launch
    const int rows = w4a16::stream_rows_ok(group_size, dp != 0, tile_cols ? *tile_cols : 0, waves ? *waves : 0,
                                           reduce ? *reduce : 0)
                         ? 16 * w4a16::kStreamMaxRowTiles
                         : 16;
    rc = w4a16::make_plan(m < rows ? m : rows, n, k, group_size, dp != 0, req, tile_cols ? *tile_cols : 0,
                          waves ? *waves : 0, reduce ? *reduce : 0, &plan);
    if (rc != W4A16_OK) return rc;
    if (split_k) *split_k = plan.split_k;
    if (tile_cols) *tile_cols = plan.tile_cols;
    if (waves) *waves = plan.waves;
    if (reduce) *reduce = plan.reduce;
    return W4A16_OK;
}

int w4a16_plan_bits(int bits, int m, int n, int k, int group_size, int dp, int* split_k, int* tile_cols, int* waves,
                    int* reduce)
{
    if (bits == 4) return w4a16_plan(m, n, k, group_size, dp, split_k, tile_cols, waves, reduce);
    if (bits != 2 && bits != 3 && bits != 8) return W4A16_ERR_UNSUPPORTED;
    const int req = split_k ? *split_k : 0;
    int rc = w4a16::check_args(m, n, k, group_size, dp ? 1 : req, true);
    if (rc != W4A16_OK) return rc;
    if ((bits == 2 && n % 16 != 0) || (bits == 3 && n % 32 != 0)) return W4A16_ERR_SHAPE;
    w4a16::Plan plan;
    // more rows than one launch takes (64 for SplitK with group_size 128 or 256, else 16): the plan of each launch
    const int rows = w4a16::stream_rows_ok(group_size, dp != 0, 0, 0, W4A16_REDUCE_AUTO) ? 16 * w4a16::kStreamMaxRowTiles : 16;
    rc = w4a16::make_plan(m < rows ? m : rows, n, k, group_size, dp != 0, dp ? 1 : req, 0, 0, W4A16_REDUCE_AUTO, &plan, bits);
    if (rc != W4A16_OK) return rc;
    if (split_k) *split_k = plan.split_k;
    if (tile_cols) *tile_cols = plan.tile_cols;
    if (waves) *waves = plan.waves;
    if (reduce) *reduce = plan.reduce;
    return W4A16_OK;
}

int w4a16_check(int m, int n, int k, int group_size, int split_k)
{
    return w4a16::check_args(m, n, k, group_size, split_k);
}

int w4a16_unpack(const void* qweight, const void* qzeros, void* q_u8, void* z_u8, int n, int k, int group_size,
                 void* stream)
{
    if (!qweight || !qzeros || !q_u8 || !z_u8) return W4A16_ERR_NULL;
    if (n < 8 || (n % 8) != 0 || group_size < 8 || (group_size % 8) != 0 || k < group_size || (k % group_size) != 0)
        return W4A16_ERR_SHAPE;
    const size_t nw = (size_t)(k / 8) * n;
    hipLaunchKernelGGL(w4a16::unpack_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const uint32_t*)qweight, (const uint32_t*)qzeros, (uint8_t*)q_u8, (uint8_t*)z_u8, n, k,
                       k / group_size);
    return w4a16::W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

int w4a16_dequant(const void* qweight, const void* scales, const void* qzeros, void* W, int n, int k, int group_size,
                  void* stream)
{
    if (!qweight || !scales || !qzeros || !W) return W4A16_ERR_NULL;
    if (n < 8 || (n % 8) != 0 || group_size < 8 || (group_size % 8) != 0 || k < group_size || (k % group_size) != 0)
        return W4A16_ERR_SHAPE;
    const size_t nw = (size_t)(k / 8) * n;
    hipLaunchKernelGGL(w4a16::dequant_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const uint32_t*)qweight, (const _Float16*)scales, (const uint32_t*)qzeros, (_Float16*)W, n,
                       k, group_size);
    return w4a16::W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

int w4a16_read_probe(const void* buffer, long long bytes, int shape, void* stream)
{
    if (!buffer) return W4A16_ERR_NULL;
    if (bytes < 16 || (bytes % 16) != 0 || !w4a16::aligned16(buffer)) return W4A16_ERR_SHAPE;
    const size_t vecs = (size_t)bytes / 16;
    const w4a16::u32x4_t* p = (const w4a16::u32x4_t*)buffer;
    hipStream_t st = (hipStream_t)stream;
    uint32_t* none = nullptr;
    switch (shape) {
    case 0: {  // one pass: every lane issues its eight loads and is done
        const size_t blocks = (vecs + 256 * 8 - 1) / (256 * 8);
        hipLaunchKernelGGL(w4a16::read_probe_kernel<8>, dim3((unsigned)(blocks < 65535 ? blocks : 65535)), dim3(256), 0, st,
                           p, vecs, none);
        break;
    }
    case 1: hipLaunchKernelGGL(w4a16::read_probe_kernel<8>, dim3(2048), dim3(256), 0, st, p, vecs, none); break;
    case 2: hipLaunchKernelGGL(w4a16::read_probe_kernel<4>, dim3(2048), dim3(512), 0, st, p, vecs, none); break;
    case 3: hipLaunchKernelGGL(w4a16::read_probe_kernel<2>, dim3(8192), dim3(256), 0, st, p, vecs, none); break;
    case 4: hipLaunchKernelGGL(w4a16::read_probe_kernel<1>, dim3(16384), dim3(256), 0, st, p, vecs, none); break;
    // 5..9: the same five with the non-temporal hint
    case 5: {
        const size_t blocks = (vecs + 256 * 8 - 1) / (256 * 8);
        hipLaunchKernelGGL((w4a16::read_probe_kernel<8, true>), dim3((unsigned)(blocks < 65535 ? blocks : 65535)), dim3(256), 0,
                           st, p, vecs, none);
        break;
    }
    case 6: hipLaunchKernelGGL((w4a16::read_probe_kernel<8, true>), dim3(2048), dim3(256), 0, st, p, vecs, none); break;
    case 7: hipLaunchKernelGGL((w4a16::read_probe_kernel<4, true>), dim3(2048), dim3(512), 0, st, p, vecs, none); break;
    case 8: hipLaunchKernelGGL((w4a16::read_probe_kernel<2, true>), dim3(8192), dim3(256), 0, st, p, vecs, none); break;
    case 9: hipLaunchKernelGGL((w4a16::read_probe_kernel<1, true>), dim3(16384), dim3(256), 0, st, p, vecs, none); break;
    default: return W4A16_ERR_UNSUPPORTED;
    }
    return w4a16::W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

long long w4a16_algorithmic_bytes(int m, int n, int k, int group_size)
{
    if (m < 1 || n < 8 || group_size < 8 || k < group_size) return 0;
    const long long g = k / group_size;
    return (long long)k * n / 2 + g * n * 2 + g * (n / 8) * 4 + (long long)m * k * 2 + (long long)m * n * 2;
}

const char* w4a16_strerror(int code)
{
    switch (code) {
    case W4A16_OK: return "ok";
    case W4A16_ERR_NULL: return "a required pointer is NULL";
    case W4A16_ERR_SHAPE: return "bad shape: need m >= 1, n % 8 == 0, group_size % 8 == 0, k % group_size == 0";
    case W4A16_ERR_SPLIT:
        return "bad split_k: need split_k >= 0; w4a16_gemm: k % split_k == 0 and (k / split_k) % group_size == 0; "
               "w4a16_gemm_ex: no more k parts than compute groups";
    case W4A16_ERR_UNSUPPORTED:
        return "unsupported: group_size not in {32,64,128,256}, pointer not 16-byte aligned, or bad tuning value";
    case W4A16_ERR_HIP: return "a HIP runtime call failed";
    case W4A16_ERR_STATE:
        return "split-k scratch unusable: a wait of the in-kernel zeroing ran out earlier on this device (release "
               "the scratch to go on), or scratch would have to be allocated while the stream is being captured";
    case W4A16_ERR_LIMIT:
        return "beyond a fixed capacity: w4a16_gemm_static takes m <= 16, n <= 16384, m * n <= 65536 with up to "
               "four rows and split_k <= 32 beyond; a bound workspace takes n up to the n_max it was sized for";
    default: return "unknown w4a16 error code";
    }
}

const char* w4a16_last_hip_error(void) { return w4a16::g_hip_detail; }

long long w4a16_phase_timeouts(void)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return W4A16_ERR_HIP;
    if (dev < 0 || dev >= w4a16::kMaxDevices) return W4A16_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(w4a16::g_mutex);
    const w4a16::DeviceScratch& s = w4a16::g_scratch[dev];
    // the counters of the library's own scratch, of the static array and of every bound workspace
    const uint32_t* words[2 + w4a16::kMaxBindings];
    int count = 0;
    if (s.phase_err.ptr) words[count++] = (const uint32_t*)s.phase_err.ptr;
    if (w4a16::g_static_ptr[dev]) words[count++] = w4a16::g_static_ptr[dev];
    for (const w4a16::Binding& b : w4a16::g_bindings)
        if (b.base && b.dev == dev) words[count++] = b.base;
    if (count == 0) return 0;
    if (hipDeviceSynchronize() != hipSuccess) return W4A16_ERR_HIP;
    long long total = 0;
    for (int i = 0; i < count; ++i) {
        uint32_t v = 0;
        if (hipMemcpy(&v, words[i], sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return W4A16_ERR_HIP;
        total += v;
    }
    return total;
}

int w4a16_set_phase_spin_limit(int polls)
{
    if (polls < 0) return W4A16_ERR_UNSUPPORTED;
    w4a16::g_spin_limit = polls == 0 ? w4a16::kSpinLimit : polls;
    return W4A16_OK;
}

long long w4a16_workspace_bytes(int n_max)
{
    if (n_max < 8 || (n_max % 8) != 0 || (size_t)n_max > 16 * (size_t)w4a16::kPhaseOrigins) return 0;
    return (long long)(w4a16::workspace_words(n_max) * sizeof(uint32_t));
}

int w4a16_set_workspace(void* workspace, long long bytes, int n_max, void* stream_v)
{
    int dev = 0;
    if (!w4a16::W4A16_HIP(hipGetDevice(&dev))) return W4A16_ERR_HIP;
    if (dev < 0 || dev >= w4a16::kMaxDevices) return W4A16_ERR_UNSUPPORTED;
    hipStream_t stream = (hipStream_t)stream_v;
    if (workspace) {
        const long long want = w4a16_workspace_bytes(n_max);
        if (want == 0) return W4A16_ERR_SHAPE;
        if (bytes < want) return W4A16_ERR_LIMIT;
        if (((uintptr_t)workspace & 255u) != 0) return W4A16_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(w4a16::g_mutex);
    w4a16::DeviceScratch& s = w4a16::g_scratch[dev];
    w4a16::Binding* slot = w4a16::find_binding(dev, stream);
    if (!workspace) {  // unbind
        if (slot) *slot = w4a16::Binding{};
        return W4A16_OK;
    }
    if (!slot)
        for (w4a16::Binding& b : w4a16::g_bindings)
            if (!b.base) {
                slot = &b;
                break;
            }
    if (!slot) return W4A16_ERR_LIMIT;
    if (!s.err_host) {
        if (!w4a16::W4A16_HIP(hipHostMalloc((void**)&s.err_host, 256, hipHostMallocMapped))) return W4A16_ERR_HIP;
        *s.err_host = 0u;
    }
    // every word starts at zero; cleared on the stream the workspace serves (a kernel, not a memset node)
    const size_t words = w4a16::workspace_words(n_max);
    hipLaunchKernelGGL(w4a16::fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                       (uint32_t*)workspace, words);
    if (!w4a16::W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
    slot->dev = dev;
    slot->stream = stream;
    slot->base = (uint32_t*)workspace;
    slot->n_max = n_max;
    return W4A16_OK;
}

int w4a16_reserve_scratch(int n_max)
{
    if (n_max < 8 || (n_max % 8) != 0) return W4A16_ERR_SHAPE;
    // everything the library's own plan can ask for at this n: fixed-point words and every phase level
    for (int split_k = 0; split_k <= w4a16::kPhaseMaxSplit; split_k = split_k == 0 ? 2 : split_k + 1) {
        w4a16::ScratchNeed need;
        need.n = n_max;
        need.fixed_words = (size_t)16 * n_max;
        need.phase_split = (size_t)n_max <= 16 * (size_t)w4a16::kPhaseOrigins ? split_k : 0;
        w4a16::ScratchView view;
        const int rc = w4a16::resolve_scratch(w4a16::kScratchLibrary, nullptr, need, &view);
        if (rc != W4A16_OK) return rc;
    }
    return W4A16_OK;
}

int w4a16_release_scratch(void)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return W4A16_ERR_HIP;
    if (dev < 0 || dev >= w4a16::kMaxDevices) return W4A16_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(w4a16::g_mutex);
    w4a16::DeviceScratch& s = w4a16::g_scratch[dev];
    if (hipDeviceSynchronize() != hipSuccess) return W4A16_ERR_HIP;
    if (s.sums.ptr) (void)hipFree(s.sums.ptr);
    if (s.partials.ptr) (void)hipFree(s.partials.ptr);
    if (s.fixed.ptr) (void)hipFree(s.fixed.ptr);
    if (s.tickets.ptr) (void)hipFree(s.tickets.ptr);
    for (w4a16::Buffer& level : s.phase_level)
        if (level.ptr) (void)hipFree(level.ptr);
    if (s.phase_err.ptr) (void)hipFree(s.phase_err.ptr);
    for (int i = 0; i < s.retired_count; ++i) (void)hipFree(s.retired[i]);
    if (s.err_host) (void)hipHostFree(s.err_host);
    s = w4a16::DeviceScratch{};
    // bound workspaces belong to their callers: forget them; the static array starts over at zero
    for (w4a16::Binding& b : w4a16::g_bindings)
        if (b.dev == dev) b = w4a16::Binding{};
    if (w4a16::g_static_ptr[dev] &&
        hipMemset(w4a16::g_static_ptr[dev], 0, w4a16::kStaticWords * sizeof(uint32_t)) != hipSuccess)
        return W4A16_ERR_HIP;
    return W4A16_OK;
}

}  // extern "C"
