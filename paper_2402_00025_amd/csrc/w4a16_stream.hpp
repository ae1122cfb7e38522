// Device routines of the streaming SplitK kernel, whose workgroup shares its activations through
// LDS (gfx950, wave64).
//
// Paper: "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference with SplitK work
// decomposition", Algorithm 1: every program owns an output tile and a 1/split_k share of k,
// loads and dequantises tiles of both operands, multiplies with an fp32 accumulator and adds
// its partial tile into C.
//
// Workgroup = 4 x wk wavefronts.  The four waves of one k part own adjacent 64-column strips
// (a 256-column tile) and walk the same k range, one quantisation group (128 k) at a time, so
// they need the same activations A[0:16, 128 k]: a 4 KiB chunk.  Each of the four waves fetches
// a quarter of every chunk (four rows, full cache lines), reorders it to the field order of the
// unpack and writes it to LDS in the layout of the MFMA A operand; after the workgroup's barrier
// every wave reads its operands from there.  That divides the activation traffic through the
// vector memory pipe by four; what remains is a per-group barrier.
//
// A compute unit returns vector-memory data in issue order, so a load issued now arrives only
// after the D groups of weight loads that are already in flight.  A chunk quarter is therefore
// requested D groups ahead (into a register ring of D quarters) and written to LDS at the end of
// the group before the one that uses it; by then it has long arrived and the wait costs nothing.
// LDS holds two chunks per k part (the one being read and the next one).
//
// More than 16 activation rows (up to 64) are row tiles of the same workgroup: a chunk grows to
// one 4 KiB block per row tile, and the weights a wave has unpacked for an MFMA step are used
// once per row tile, so the weight stream and the unpacking are paid once for all rows.
#pragma once
#include "w4a16_device.hpp"

namespace w4a16 {

struct StreamArgs {
    const _Float16* A;
    const uint32_t* qweight;
    const _Float16* scales;
    const uint32_t* qzeros;
    _Float16* C;
    uint32_t* flags;      // phase protocol: zeroings so far, per tile origin (n0 / 16)
    uint32_t* counts;     // phase protocol: calls so far, per (tile origin, slice)
    uint32_t* errors;     // phase protocol: count of waits that ran out
    uint32_t* err_host;   // phase protocol: word in pinned host memory set by a wait that ran out (may be null)
    int m, n, k;
    int tiles;            // 256-column workgroup tiles = ceil(n / 256)
    int split_k;
    int wk;               // k parts per workgroup; working waves = 4 * wk (2 only with m <= 16)
    // compute groups (128 consecutive k) per k part: part i = slice * wk + kpart gets groups_base,
    // the first groups_rem parts one more (groups_rem > 0 only with wk == 1); groups_base >= D.
    // At ring depth 2 a part with an odd count runs one phantom group more, whose product is dropped.
    int groups_base;
    int groups_rem;
    int param_shift;      // log2(compute groups per quantisation group)
    int spin_limit;       // phase protocol: bound on samples of a flag
    int probe_delay;      // phase protocol: 64-cycle sleeps before a sample
};

constexpr int kStreamStrips = 4;
constexpr int kStreamTileCols = 64 * kStreamStrips;
constexpr int kChunkBytes = 16 * 128 * 2;  // one row tile of an activation chunk in LDS: 16 rows x 128 k, fp16
constexpr int kStreamMaxRowTiles = 4;      // row tiles of 16 activation rows per workgroup

// LDS layout of a chunk: one 16-byte slot per (kc = 8 consecutive k, row): slot kc * 16 + (row ^ kc).
// The xor makes both access patterns conflict-free: a writing wave has, in every 16 lanes, one
// row and kc = 0..15; a reading wave has one kc and rows 0..15.
__device__ __forceinline__ int chunk_slot_bytes(int kc, int row) { return (kc * 16 + (row ^ kc)) * 16; }

// BITS: width of the packed fields (4, or 8, 3, 2 as in the per-wave kernel); the activation
// slot of a step's registers is not used here (the activations come from LDS).
template <int D, int BITS = 4>
struct WeightRing {
    StepRegs<4, BITS> w[D][4];
    ParamRegs<4, BITS> par[D];
};

template <int D, int H, int BITS>
__device__ __forceinline__ void ring_issue_group(WeightRing<D, BITS>& ring, const LaneMap& lm, const Tensors& t, int gi)
{
    issue_params<4, BITS>(ring.par[H], lm, t, gi);
#pragma unroll
    for (int it = 0; it < 4; ++it) issue_step_weights<4, BITS>(ring.w[H][it], lm, t, (uint32_t)gi * 4u + it);
}

template <int D, int H, int BITS>
__device__ __forceinline__ void ring_prime(WeightRing<D, BITS>& ring, const LaneMap& lm, const Tensors& t, int g_begin)
{
    if constexpr (H < D) {
        ring_issue_group<D, H, BITS>(ring, lm, t, g_begin + H);
        ring_prime<D, H + 1, BITS>(ring, lm, t, g_begin);
    }
}

// What stays fixed for a lane while it streams: where its quarter of a chunk comes from and goes
// to, and where its MFMA operands of the four steps of a group lie in a chunk.  MT = row tiles
// of 16 activation rows (m <= 16 MT): a chunk then is MT blocks of 4 KiB, one per row tile, and
// every wave fetches its quarter (four rows) of each.
template <int MT>
struct StreamLane {
    uint32_t a_voff[MT];  // per row tile: byte offset of its 16 bytes of A inside a chunk quarter's row, or outside the buffer
    uint32_t a_soff0;     // byte offset of chunk 0 of this wave's k range
    int wslot;            // LDS byte offset (inside a row tile's block) of the slot it writes
    int roff[4];          // LDS byte offsets (inside a row tile's block) of the slots it reads, per MFMA step
    char* ring;           // the k part's two chunks in LDS
};

// One compute group (128 k) of a wave out of ring slot H; `cc` is its index inside the wave's
// range.  REFILL: request the weights and the chunk quarters of group cc + D.  NEXT: there is a
// group cc + 1: publish its chunk quarters, meet the other waves, fetch the next operands.
// The unpacked weights of a step serve all MT row tiles.
// `last_keep` says whether the contribution of a wave's last group (the one without NEXT) counts:
// 1, or 0 when that group is a phantom that only evens out an odd count (its loads read the
// next part's data or, behind the end of k, zeros; its product is dropped).
template <int D, int H, bool REFILL, bool NEXT, int MT, int BITS>
__device__ __forceinline__ void stream_group(WeightRing<D, BITS>& ring, u32x4_t (&a_in)[D][MT], u32x4_t (&a)[MT][4],
                                             const StreamLane<MT>& sl, const LaneMap& lm, const Tensors& t,
                                             uint32_t magic, int cc, int g_begin, float4_t (&acc)[MT][4],
                                             float last_keep)
{
    typename ZeroOf<BITS>::type zc[4];
    float sc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        zc[j] = zero_of_column<4, BITS>(ring.par[H], lm, j);
        sc[j] = scale_of<4>(ring.par[H].s, j);
    }
    if constexpr (REFILL) {
        __builtin_amdgcn_sched_barrier(0);
        issue_params<4, BITS>(ring.par[H], lm, t, g_begin + cc + D);
#pragma unroll
        for (int rt = 0; rt < MT; ++rt)
            a_in[H][rt] = __builtin_amdgcn_raw_buffer_load_b128(t.A, sl.a_voff[rt],
                                                                sl.a_soff0 + (uint32_t)(cc + D) * 256u, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    float4_t tile[MT][4];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int j = 0; j < 4; ++j) tile[rt][j] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        half8_t b8[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) b8[j] = unpack_column<4, BITS>(ring.w[H][it], j, lm, zc[j], magic);
        if constexpr (REFILL) {
            __builtin_amdgcn_sched_barrier(0);
            issue_step_weights<4, BITS>(ring.w[H][it], lm, t, (uint32_t)(g_begin + cc + D) * 4u + it);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) {
            const half8_t a8 = __builtin_bit_cast(half8_t, a[rt][it]);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                tile[rt][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a8, b8[j], tile[rt][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (NEXT) {
                acc[rt][j] += sc[j] * tile[rt][j];
            } else {
                // a select, not a product with 0: the phantom's operands are someone else's data
                // and need not be finite
                const float4_t add = sc[j] * tile[rt][j];
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[rt][j][r] += last_keep != 0.f ? add[r] : 0.f;
            }
        }
    if constexpr (NEXT) {
        char* buf = sl.ring + ((cc + 1) & 1) * (MT * kChunkBytes);
#pragma unroll
        for (int rt = 0; rt < MT; ++rt)
            *(half8_t*)(buf + rt * kChunkBytes + sl.wslot) = order_activations<BITS>(a_in[(H + 1) % D][rt]);
        __syncthreads();
#pragma unroll
        for (int rt = 0; rt < MT; ++rt)
#pragma unroll
            for (int it = 0; it < 4; ++it) a[rt][it] = *(const u32x4_t*)(buf + rt * kChunkBytes + sl.roff[it]);
    }
}

template <int D, int H, bool REFILL, int MT, int BITS>
__device__ __forceinline__ void stream_groups(WeightRing<D, BITS>& ring, u32x4_t (&a_in)[D][MT], u32x4_t (&a)[MT][4],
                                              const StreamLane<MT>& sl, const LaneMap& lm, const Tensors& t,
                                              uint32_t magic, int c0, int g_begin, float4_t (&acc)[MT][4],
                                              float last_keep)
{
    if constexpr (H < D) {
        // the last group of the wave has no successor
        constexpr bool kNext = REFILL || (H + 1 < D);
        stream_group<D, H, REFILL, kNext, MT, BITS>(ring, a_in, a, sl, lm, t, magic, c0 + H, g_begin, acc, last_keep);
        stream_groups<D, H + 1, REFILL, MT, BITS>(ring, a_in, a, sl, lm, t, magic, c0, g_begin, acc, last_keep);
    }
}

}  // namespace w4a16
