// SplitK kernel whose workgroup shares its activation slice through LDS (gfx950, wave64).
//
// Paper: "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference with SplitK work
// decomposition", Algorithm 1: every program owns an output tile and a 1/split_k share of k,
// loads and dequantises tiles of both operands, multiplies with an fp32 accumulator and adds
// its partial tile into C.
//
// Workgroup = wn x wk wavefronts.  The wn waves of one k part own adjacent 64-column strips, so
// the workgroup's tile is 64*wn columns wide; the wk k parts divide the workgroup's k range.
// All waves read the same activation slice A[0:m, k range], which is fetched from memory once
// per workgroup, reordered to the field order of the unpack and kept in LDS in the layout of the
// MFMA A operand: one 16-byte slot per (8 consecutive k, row).  The weight stream goes
// HBM -> registers -> MFMA exactly as in the per-wave kernel (w4a16_device.hpp), but the
// register ring holds weights only, so it can be D quantisation groups deep.
#pragma once
#include "w4a16_device.hpp"

namespace w4a16 {

struct SharedArgs {
    const _Float16* A;
    const uint32_t* qweight;
    const _Float16* scales;
    const uint32_t* qzeros;
    _Float16* C;
    uint32_t* flags;      // one word per workgroup tile (modes that order zeroing and adding)
    int m, n, k;
    int tiles;            // workgroup column tiles = ceil(n / (64 * wn))
    int split_k;
    int wn, wk;           // waves of a workgroup: wn column strips x wk k parts
    int groups_per_wave;  // compute groups (128 consecutive k) per wave; a multiple of D
    int param_shift;      // log2(compute groups per quantisation group)
    int a_bytes;          // LDS bytes of the activation slice
    int spin_limit;       // bound on polls of a tile flag (the wait always ends)
};

template <int D>
struct WeightRing {
    Words<4> w[D][4];
    ParamRegs<4> par[D];
};

template <int D, int H>
__device__ __forceinline__ void ring_issue_group(WeightRing<D>& ring, const LaneMap& lm, const Tensors& t, int gi)
{
    issue_params<4>(ring.par[H], lm, t, gi);
#pragma unroll
    for (int it = 0; it < 4; ++it)
        ring.w[H][it].load(t.qweight, lm.off_w, ((uint32_t)gi * 4u + it) * 16u * (uint32_t)t.n);
}

// One compute group (128 k) out of ring slot H.  `a` holds the activation operands of its four
// MFMA steps; each is replaced by the same step of the next group as soon as it has been used
// (NEXT_A), and each weight register set by the same step of group `refill` (REFILL).
template <int D, int H, bool REFILL, bool NEXT_A>
__device__ __forceinline__ void shared_compute_group(WeightRing<D>& ring, const LaneMap& lm, const Tensors& t,
                                                     uint32_t magic, int refill, const char* a_next,
                                                     int a_step_bytes, u32x4_t (&a)[4], float4_t (&acc)[4])
{
    ZeroConst zc[4];
    float sc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        zc[j] = zero_const((ring.par[H].zword >> (lm.zshift + 4 * j)) & 0xFu);
        sc[j] = scale_of<4>(ring.par[H].s, j);
    }
    if constexpr (REFILL) {
        __builtin_amdgcn_sched_barrier(0);
        issue_params<4>(ring.par[H], lm, t, refill);
        __builtin_amdgcn_sched_barrier(0);
    }
    float4_t tile[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) tile[j] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const half8_t a8 = __builtin_bit_cast(half8_t, a[it]);
        half8_t b8[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) b8[j] = unpack_shift(ring.w[H][it].v[j], zc[j], magic);
        if constexpr (REFILL) {
            __builtin_amdgcn_sched_barrier(0);
            ring.w[H][it].load(t.qweight, lm.off_w, ((uint32_t)refill * 4u + it) * 16u * (uint32_t)t.n);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) tile[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a8, b8[j], tile[j], 0, 0, 0);
        if constexpr (NEXT_A) a[it] = *(const u32x4_t*)(a_next + it * a_step_bytes);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] += sc[j] * tile[j];
}

template <int D, int H, bool REFILL>
__device__ __forceinline__ void shared_compute_slots(WeightRing<D>& ring, const LaneMap& lm, const Tensors& t,
                                                     uint32_t magic, int g_next, const char*& a_ptr,
                                                     int a_step_bytes, u32x4_t (&a)[4], float4_t (&acc)[4])
{
    if constexpr (H < D) {
        // the very last group of the wave has no successor to prefetch activations for
        constexpr bool kNextA = REFILL || (H + 1 < D);
        a_ptr += 4 * a_step_bytes;
        shared_compute_group<D, H, REFILL, kNextA>(ring, lm, t, magic, g_next + H, a_ptr, a_step_bytes, a, acc);
        shared_compute_slots<D, H + 1, REFILL>(ring, lm, t, magic, g_next, a_ptr, a_step_bytes, a, acc);
    }
}

template <int D, int H>
__device__ __forceinline__ void ring_prime(WeightRing<D>& ring, const LaneMap& lm, const Tensors& t, int g_begin)
{
    if constexpr (H < D) {
        ring_issue_group<D, H>(ring, lm, t, g_begin + H);
        ring_prime<D, H + 1>(ring, lm, t, g_begin);
    }
}

}  // namespace w4a16
