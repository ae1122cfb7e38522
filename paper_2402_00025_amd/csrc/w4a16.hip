// Kernels and C ABI of the fused W4A16 skinny GEMM for gfx950.  See include/w4a16.h for the
// contract and w4a16_device.hpp for the per-wave routines.
//
// Paper: "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference with SplitK work
// decomposition".  Algorithm 1 is the SplitK kernel; Section 3 (first paragraph) describes the
// data-parallel tiling it is compared with; Section 2.1 the atomic reduction.
#include "w4a16_device.hpp"

#include <cstdio>
#include <mutex>

#include "../../include/w4a16.h"

namespace w4a16 {

struct GemmArgs {
    const _Float16* A;
    const uint32_t* qweight;
    const _Float16* scales;
    const uint32_t* qzeros;
    _Float16* C;
    float* scratch;     // split-k: fp32 sums [16, n] (atomic) or partial tiles [split_k, m, n] (workspace)
    uint32_t* tickets;  // split-k: one arrival counter per column tile
    int m, n, k;
    int tiles;            // column tiles = ceil(n / (16 V))
    int split_k;
    int groups_per_block; // compute groups (32 * IPG consecutive k) per workgroup
    int groups_per_wave;  // groups_per_block / waves
    int param_shift;      // log2(compute groups per quantisation group)
    int lds_wave_bytes;   // LDS region of one wave
};

enum : int { kDirect = 0, kAtomicF32 = 1, kAtomicPkF16 = 2, kWorkspace = 3, kAtomicFixed = 4 };

// kAtomicFixed: one 64-bit integer atomic add per output element and workgroup.
//   bits 56..63  arrivals so far (split_k <= 64)
//   bits  0..55  sum of (partial * 2^33 + 2^50): fixed point, biased so it never goes negative
// The add returns the previous word, so the workgroup that sees split_k - 1 earlier arrivals
// holds the complete sum (previous + its own) and finishes the element: one memory round trip,
// no separate ticket, and a sum that does not depend on arrival order (integer addition).
constexpr int kFixedFracBits = 33;
constexpr uint64_t kFixedBias = 1ull << 50;
constexpr uint64_t kFixedArrival = 1ull << 56;
constexpr uint64_t kFixedSumMask = kFixedArrival - 1;
constexpr float kFixedClamp = 131071.0f;  // |partial| < 2^17 keeps partial * 2^33 inside the bias

__device__ __forceinline__ uint64_t fixed_contribution(float v)
{
    v = fminf(fmaxf(v, -kFixedClamp), kFixedClamp);
    const long long q = __double2ll_rn((double)v * (double)(1ull << kFixedFracBits));
    return (uint64_t)(q + (long long)kFixedBias) + kFixedArrival;
}

__device__ __forceinline__ float fixed_total(uint64_t word, int split_k)
{
    const long long q = (long long)(word & kFixedSumMask) - (long long)split_k * (long long)kFixedBias;
    return (float)((double)q * (1.0 / (double)(1ull << kFixedFracBits)));
}

// After `old = fetch_add(word, mine)`: if this was the last of split_k arrivals, returns true
// with the total in *total and resets the word to zero for the next call.
__device__ __forceinline__ bool fixed_finish(uint64_t* word, uint64_t old, uint64_t mine, int split_k, float* total)
{
    if ((int)(old >> 56) != split_k - 1) return false;
    *total = fixed_total(old + mine, split_k);
    __hip_atomic_store(word, (uint64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
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

// One workgroup = WAVES wavefronts that share one output tile [m, 16 V] and divide the
// workgroup's k range between them; blockIdx.x = slice * tiles + tile.
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
//
// Synchronisation of the ticketed modes.  Every access that one workgroup makes and another
// reads is a device-scope atomic operation (add, exchange, write-through store, cache-bypassing
// load), so it is performed at the level where all compute dies see it; none of it sits dirty
// in a die-local L2.  What is left to order is time: a workgroup waits until its own
// contributions have been performed (wait_memory_ops + barrier) before one of its threads takes
// the ticket, and the last workgroup reads only after its ticket came back.  A device-scope
// release fence would do the same but also write back the whole L2 of the die, which costs
// more than the GEMM itself.
// WMAX (4 or 16) is the largest number of waves the instantiation may be launched with; the
// small one lets the compiler use more than 128 registers per lane.
template <int V, int IPG, int MODE, int WMAX>
__global__ void __launch_bounds__(kWave * WMAX) gemm_kernel(const GemmArgs p)
{
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    constexpr int BN = 16 * V;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: keeps offsets scalar
    const int waves = blockDim.x / kWave;
    const int tile = blockIdx.x % p.tiles;
    const int slice = blockIdx.x / p.tiles;
    const int n0 = tile * BN;
    const int m = p.m, n = p.n, k = p.k;

    const LaneMap lm = make_lane_map<V>(lane, n0, m, n, k);
    const uint32_t qgroups = (uint32_t)(k / (32 * IPG)) >> p.param_shift;
    Tensors tensors;
    tensors.A = make_rsrc(p.A, (uint32_t)m * (uint32_t)k * 2u);
    tensors.qweight = make_rsrc(p.qweight, (uint32_t)(k / 8) * (uint32_t)n * 4u);
    tensors.scales = make_rsrc(p.scales, qgroups * (uint32_t)n * 2u);
    tensors.qzeros = make_rsrc(p.qzeros, qgroups * (uint32_t)(n / 8) * 4u);
    tensors.m = m;
    tensors.n = n;
    tensors.k = k;
    tensors.param_shift = p.param_shift;

    float4_t acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int g_begin = slice * p.groups_per_block + wave * p.groups_per_wave;
    wave_mainloop<V, IPG>(tensors, lm, g_begin, p.groups_per_wave, acc);

    // ---- sum the waves' tiles through LDS.  acc[j][r] is row 4*(lane/16)+r, column V*(lane%16)+j.
    float* red = (float*)(lds_raw + wave * p.lds_wave_bytes);  // [m][BN]
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * (lane >> 4) + r;
        if (row < m) {
#pragma unroll
            for (int j = 0; j < V; ++j) red[row * BN + V * (lane & 15) + j] = acc[j][r];
        }
    }
    __syncthreads();

    const int pairs = m * (BN / 2);
    const int wave_floats = p.lds_wave_bytes / 4;
    const float* red0 = (const float*)lds_raw;

    if constexpr (MODE == kAtomicF32 || MODE == kAtomicFixed) {
        // one element per lane, consecutive lanes on consecutive columns: an atomic instruction
        // of a wave then touches the fewest cache lines, and the L2 charges atomics per line.
        // Up to kBatch elements per thread are in flight at once so that the returning atomics
        // of the fixed-point mode cost one memory round trip, not one per element.
        constexpr int kBatch = 4;
        const int elems = m * BN;
        for (int e0 = threadIdx.x; e0 < elems; e0 += kBatch * blockDim.x) {
            size_t idx[kBatch];
            bool ok[kBatch];
            float v[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int e = e0 + u * blockDim.x;
                const int row = e / BN;
                const int c = e % BN;
                ok[u] = e < elems && n0 + c < n;
                idx[u] = ok[u] ? (size_t)row * n + n0 + c : 0;
                v[u] = 0.f;
                if (ok[u])
                    for (int w = 0; w < waves; ++w) v[u] += red0[w * wave_floats + row * BN + c];
            }
            if constexpr (MODE == kAtomicF32) {
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (ok[u])
                        __hip_atomic_fetch_add(p.scratch + idx[u], v[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                uint64_t mine[kBatch], old[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    mine[u] = fixed_contribution(v[u]);
                    old[u] = 0;
                    if (ok[u])
                        old[u] = __hip_atomic_fetch_add((uint64_t*)p.scratch + idx[u], mine[u], __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    float total = 0.f;
                    if (ok[u] && fixed_finish((uint64_t*)p.scratch + idx[u], old[u], mine[u], p.split_k, &total))
                        p.C[idx[u]] = (_Float16)total;
                }
            }
        }
    } else {
        for (int e = threadIdx.x; e < pairs; e += blockDim.x) {
            const int row = e / (BN / 2);
            const int c2 = 2 * (e % (BN / 2));
            const int col = n0 + c2;
            if (col >= n) continue;
            float v0 = 0.f, v1 = 0.f;
            for (int w = 0; w < waves; ++w) {
                const float2 t = *(const float2*)(red0 + w * wave_floats + row * BN + c2);
                v0 += t.x;
                v1 += t.y;
            }
            const size_t idx = (size_t)row * n + col;
            if constexpr (MODE == kDirect) {
                *(uint32_t*)(p.C + idx) = pack_half2(v0, v1);
            } else if constexpr (MODE == kAtomicPkF16) {
                const half2_t h = {(_Float16)v0, (_Float16)v1};
                __builtin_amdgcn_global_atomic_fadd_v2f16((__attribute__((address_space(1))) half2_t*)(p.C + idx), h);
            } else {
                const uint64_t bits = (uint64_t)__builtin_bit_cast(uint32_t, v0) |
                                      ((uint64_t)__builtin_bit_cast(uint32_t, v1) << 32);
                __hip_atomic_store((uint64_t*)(p.scratch + ((size_t)slice * m + row) * n + col), bits,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
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

// C <- 0 for the packed-fp16 atomic mode (a kernel, not a memset, so the call can be captured
// in a HIP graph).
__global__ void fill_zero_kernel(uint32_t* p, size_t words)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
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
struct DeviceScratch {
    Buffer sums;      // atomic mode: fp32 [16, n]; all zero whenever no call is running
    Buffer partials;  // workspace mode: fp32 [split_k, m, n]; no invariant
    Buffer fixed;     // fixed-point mode: uint64 [16, n]; all zero whenever no call is running
    Buffer tickets;   // uint32 per column tile; all zero whenever no call is running
};
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
static DeviceScratch g_scratch[kMaxDevices];
static std::mutex g_mutex;

static int check_args(int m, int n, int k, int group_size, int split_k)
{
    if (m < 1 || n < 8 || (n % 8) != 0 || group_size < 8 || (group_size % 8) != 0 || k < group_size ||
        (k % group_size) != 0)
        return W4A16_ERR_SHAPE;
    if (split_k < 0) return W4A16_ERR_SPLIT;
    if (split_k > 0 && ((k % split_k) != 0 || ((k / split_k) % group_size) != 0)) return W4A16_ERR_SPLIT;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256) return W4A16_ERR_UNSUPPORTED;
    return W4A16_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Largest w in {16, 8, 4, 2, 1}, w <= cap, that divides `groups`.
static int largest_wave_split(int groups, int cap)
{
    for (int w = 16; w >= 1; w >>= 1)
        if (w <= cap && groups % w == 0) return w;
    return 1;
}

struct Plan {
    int split_k, tile_cols, waves, reduce;
};

// Launch shape, from sweeps on MI355X (256 compute units, 1024 SIMDs).
//
// SplitK: 64-column tiles (128-bit weight loads).  The kernel is bound by how fast a burst of
// loads can be put in flight, so the plan aims at one to two resident waves per SIMD: about
// 2048 waves when the whole weight matrix is small enough to be requested at once (<= 8 MiB
// packed), about 1024 longer-running waves otherwise.  Up to four waves of a workgroup divide
// its k range (their tiles are added in LDS, which keeps the atomic traffic down); the rest of
// the k parallelism is split_k.
// Data-parallel: the only source of workgroups is the column tiling, so tiles shrink (64, 32,
// 16 columns) until there are about 256 of them, and the waves of a workgroup divide k.
static int make_plan(int m, int n, int k, int group_size, bool dp, int split_k, int tile_cols, int waves,
                     int reduce, Plan* out)
{
    const int groups = k / group_size;
    if (tile_cols == 0) {
        tile_cols = 64;
        if (dp) {
            while (tile_cols > 16 && (n + tile_cols - 1) / tile_cols < 256) tile_cols /= 2;
        }
    }
    if (tile_cols != 16 && tile_cols != 32 && tile_cols != 64) return W4A16_ERR_UNSUPPORTED;
    const int tiles = (n + tile_cols - 1) / tile_cols;
    // 64-column tiles need more than 128 registers per lane, so at most 4 waves per workgroup
    const int wave_cap = tile_cols == 64 ? 4 : 16;
    if (dp) {
        split_k = 1;
    } else if (split_k == 0) {
        const long long packed_bytes = (long long)k * n / 2;
        const int target_waves = packed_bytes <= (8ll << 20) ? 2048 : 1024;
        int want = 1;  // split_k * waves
        while (want * 2 <= groups && groups % (want * 2) == 0 && tiles * want * 2 <= target_waves) want *= 2;
        const int w = want < 4 ? want : 4;
        split_k = want / w;
        if (waves == 0) waves = w;
    }
    if (split_k < 1 || groups % split_k != 0) return W4A16_ERR_SPLIT;
    const int gpb = groups / split_k;
    if (waves == 0) waves = largest_wave_split(gpb, dp ? wave_cap : 4);
    if (waves < 1 || waves > 16 || gpb % waves != 0) return W4A16_ERR_UNSUPPORTED;
    if (reduce == W4A16_REDUCE_AUTO) {
        // few rows: the arrival-counting fixed-point adds finish in one round trip with no
        // zero-fill launch.  Many rows: returning 64-bit atomics cost more than the fill launch
        // that the packed-fp16 adds need.
        reduce = (m <= 4 && split_k <= 64) ? W4A16_REDUCE_ATOMIC_FIXED : W4A16_REDUCE_ATOMIC_PK_F16;
    }
    if (reduce < W4A16_REDUCE_ATOMIC_F32 || reduce > W4A16_REDUCE_ATOMIC_FIXED) return W4A16_ERR_UNSUPPORTED;
    if (reduce == W4A16_REDUCE_ATOMIC_FIXED && split_k > 64) return W4A16_ERR_UNSUPPORTED;
    out->split_k = split_k;
    out->tile_cols = tile_cols;
    out->waves = waves;
    out->reduce = reduce;
    return W4A16_OK;
}

// Grow-only device buffer.  Growth happens on the first call for a shape, outside any timed
// region; it frees (which waits for the device), allocates, clears and synchronises.
static int grow(Buffer& b, size_t bytes, bool* grew)
{
    if (b.bytes >= bytes) return W4A16_OK;
    if (b.ptr) (void)hipFree(b.ptr);
    b.ptr = nullptr;
    b.bytes = 0;
    if (!W4A16_HIP(hipMalloc(&b.ptr, bytes))) return W4A16_ERR_HIP;
    if (!W4A16_HIP(hipMemset(b.ptr, 0, bytes))) return W4A16_ERR_HIP;
    b.bytes = bytes;
    *grew = true;
    return W4A16_OK;
}

static int ensure_scratch(size_t sums_floats, size_t partial_floats, size_t fixed_words, size_t ticket_count,
                          float** sums, float** partials, uint64_t** fixed, uint32_t** tickets)
{
    int dev = 0;
    if (!W4A16_HIP(hipGetDevice(&dev))) return W4A16_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return W4A16_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceScratch& s = g_scratch[dev];
    bool grew = false;
    int rc = grow(s.sums, sums_floats * sizeof(float), &grew);
    if (rc == W4A16_OK) rc = grow(s.partials, partial_floats * sizeof(float), &grew);
    if (rc == W4A16_OK) rc = grow(s.fixed, fixed_words * sizeof(uint64_t), &grew);
    if (rc == W4A16_OK) rc = grow(s.tickets, ticket_count * sizeof(uint32_t), &grew);
    if (rc != W4A16_OK) return rc;
    if (grew && !W4A16_HIP(hipDeviceSynchronize())) return W4A16_ERR_HIP;
    *sums = (float*)s.sums.ptr;
    *partials = (float*)s.partials.ptr;
    *fixed = (uint64_t*)s.fixed.ptr;
    *tickets = (uint32_t*)s.tickets.ptr;
    return W4A16_OK;
}

template <int V, int IPG, int MODE, int WMAX>
static int launch_bound(const GemmArgs& a, int waves, size_t lds_bytes, hipStream_t stream)
{
    auto kern = gemm_kernel<V, IPG, MODE, WMAX>;
    if (lds_bytes > 64 * 1024) {
        if (!W4A16_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes)))
            return W4A16_ERR_HIP;
    }
    const unsigned grid = (unsigned)(a.tiles * a.split_k);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(waves * kWave), lds_bytes, stream, a);
    return W4A16_HIP(hipGetLastError()) ? W4A16_OK : W4A16_ERR_HIP;
}

template <int V, int IPG, int MODE>
static int launch_one(const GemmArgs& a, int waves, size_t lds_bytes, hipStream_t stream)
{
    if (waves <= 4) return launch_bound<V, IPG, MODE, 4>(a, waves, lds_bytes, stream);
    return launch_bound<V, IPG, MODE, 16>(a, waves, lds_bytes, stream);
}

template <int V, int IPG>
static int launch_mode(const GemmArgs& a, int waves, size_t lds_bytes, int mode, hipStream_t stream)
{
    switch (mode) {
    case kDirect: return launch_one<V, IPG, kDirect>(a, waves, lds_bytes, stream);
    case kAtomicF32: return launch_one<V, IPG, kAtomicF32>(a, waves, lds_bytes, stream);
    case kAtomicPkF16: return launch_one<V, IPG, kAtomicPkF16>(a, waves, lds_bytes, stream);
    case kWorkspace: return launch_one<V, IPG, kWorkspace>(a, waves, lds_bytes, stream);
    default: return launch_one<V, IPG, kAtomicFixed>(a, waves, lds_bytes, stream);
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

static int run_gemm(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                    int n, int k, int group_size, bool dp, int split_k, int tile_cols, int waves, int reduce,
                    void* stream_v)
{
    if (!A || !qweight || !scales || !qzeros || !C) return W4A16_ERR_NULL;
    int rc = check_args(m, n, k, group_size, dp ? 1 : split_k);
    if (rc != W4A16_OK) return rc;
    if (!aligned16(A) || !aligned16(qweight) || !aligned16(scales) || !aligned16(qzeros) || !aligned16(C))
        return W4A16_ERR_UNSUPPORTED;
    if (m > 16) {
        // more than one MFMA row tile: one launch per 16 rows (each streams the weights again;
        // the paper's regime is m <= 16, larger m is served for completeness)
        for (int r = 0; r < m; r += 16) {
            const int mm = m - r < 16 ? m - r : 16;
            rc = run_gemm((const _Float16*)A + (size_t)r * k, qweight, scales, qzeros, (_Float16*)C + (size_t)r * n, mm,
                          n, k, group_size, dp, split_k, tile_cols, waves, reduce, stream_v);
            if (rc != W4A16_OK) return rc;
        }
        return W4A16_OK;
    }
    Plan plan;
    rc = make_plan(m, n, k, group_size, dp, split_k, tile_cols, waves, reduce, &plan);
    if (rc != W4A16_OK) return rc;

    hipStream_t stream = (hipStream_t)stream_v;
    const int ipg = group_size >= 128 ? 4 : group_size / 32;  // MFMA steps (32 k each) per compute group
    const int param_shift = group_size == 256 ? 1 : 0;
    const int V = plan.tile_cols / 16;
    if ((unsigned long long)k * (unsigned long long)n / 2 >= (1ull << 31)) return W4A16_ERR_UNSUPPORTED;
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
    a.groups_per_block = (k / (32 * ipg)) / plan.split_k;
    a.groups_per_wave = a.groups_per_block / plan.waves;
    a.param_shift = param_shift;
    // LDS: one [m, tile_cols] fp32 tile per wave, for the sum over the workgroup's waves
    a.lds_wave_bytes = (m * plan.tile_cols * 4 + 15) & ~15;
    const size_t lds_bytes = (size_t)a.lds_wave_bytes * plan.waves;
    if (lds_bytes > 160 * 1024) return W4A16_ERR_UNSUPPORTED;

    int mode = kDirect;
    if (plan.split_k > 1) {
        mode = plan.reduce;  // W4A16_REDUCE_* values equal the kernel modes
        if (mode != kAtomicPkF16) {
            float *sums = nullptr, *partials = nullptr;
            uint64_t* fixed = nullptr;
            rc = ensure_scratch(mode == kAtomicF32 ? (size_t)16 * n : 0,
                                mode == kWorkspace ? (size_t)plan.split_k * m * n : 0,
                                mode == kAtomicFixed ? (size_t)16 * n : 0, (size_t)a.tiles, &sums, &partials, &fixed,
                                &a.tickets);
            if (rc != W4A16_OK) return rc;
            a.scratch = mode == kAtomicF32 ? sums : mode == kWorkspace ? partials : (float*)fixed;
        } else {
            const size_t words = (size_t)m * n / 2;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                               (uint32_t*)C, words);
            if (!W4A16_HIP(hipGetLastError())) return W4A16_ERR_HIP;
        }
    }
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
                           W4A16_REDUCE_AUTO, stream);
}

int w4a16_gemm_dp(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, void* stream)
{
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, 0, 0, W4A16_REDUCE_AUTO,
                           stream);
}

int w4a16_gemm_ex(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m, int n,
                  int k, int group_size, int split_k, int tile_cols, int waves, int reduce, void* stream)
{
    if (tile_cols < 0 || waves < 0 || reduce < 0) return W4A16_ERR_UNSUPPORTED;
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, false, split_k, tile_cols, waves,
                           reduce, stream);
}

int w4a16_gemm_dp_ex(const void* A, const void* qweight, const void* scales, const void* qzeros, void* C, int m,
                     int n, int k, int group_size, int tile_cols, int waves, void* stream)
{
    if (tile_cols < 0 || waves < 0) return W4A16_ERR_UNSUPPORTED;
    return w4a16::run_gemm(A, qweight, scales, qzeros, C, m, n, k, group_size, true, 1, tile_cols, waves,
                           W4A16_REDUCE_AUTO, stream);
}

int w4a16_plan(int m, int n, int k, int group_size, int dp, int* split_k, int* tile_cols, int* waves, int* reduce)
{
    const int req = split_k ? *split_k : 0;
    int rc = w4a16::check_args(m, n, k, group_size, dp ? 1 : req);
    if (rc != W4A16_OK) return rc;
    w4a16::Plan plan;
    rc = w4a16::make_plan(m, n, k, group_size, dp != 0, req, tile_cols ? *tile_cols : 0, waves ? *waves : 0,
                          reduce ? *reduce : 0, &plan);
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
    case W4A16_ERR_SPLIT: return "bad split_k: need split_k >= 0, k % split_k == 0, (k / split_k) % group_size == 0";
    case W4A16_ERR_UNSUPPORTED:
        return "unsupported: group_size not in {32,64,128,256}, pointer not 16-byte aligned, or bad tuning value";
    case W4A16_ERR_HIP: return "a HIP runtime call failed";
    default: return "unknown w4a16 error code";
    }
}

const char* w4a16_last_hip_error(void) { return w4a16::g_hip_detail; }

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
    s = w4a16::DeviceScratch{};
    return W4A16_OK;
}

}  // extern "C"
