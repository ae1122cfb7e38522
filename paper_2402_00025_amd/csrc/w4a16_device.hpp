// Device routines of the fused W4A16 skinny GEMM for gfx950 (CDNA4, wave64).
//
// Paper: "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference with SplitK work
// decomposition".  Section 2 (first paragraph) defines the inputs and the dequantisation,
// Algorithm 1 the SplitK loop, Section 3 (first paragraph) the data-parallel variant.
//
// One wavefront walks a strip of 16*V output columns over a range of quantisation groups.
// Lane l owns columns V*(l%16) .. V*(l%16)+V-1 of the strip for everything that is per column
// (packed weight words, zero points, scales, output), and packed row (l/16) of every four.
//
//   * one 32-bit qweight word = 8 consecutive k of one column = exactly one lane's share of the
//     B operand of v_mfma_f32_16x16x32_f16, so a V-word vector load feeds V MFMAs with no
//     cross-lane movement;
//   * fields are turned into fp16 integers (q - z) with two mask-or operations per pair and one
//     packed fp16 add/fma, all exact;
//   * the scale is applied in fp32 to the 16x16 result of a whole group, so the weight is never
//     rounded to fp16;
//   * the activation slice of the group is staged through wave-private LDS, permuted to the
//     field order the unpack produces.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace w4a16 {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// ------------------------------------------------------------------------------------------
// Unpack + zero-point shift (Section 2: "dequantized, scaled and shifted using bitwise
// operations").  fp16 1024.0 is 0x6400 and has a unit in the last place of 1, so OR-ing a
// 4-bit field into its mantissa gives 1024 + q exactly; a field left at bit 4 gives
// 1024 + 16 q.  Subtracting 1024 + z, or multiplying by 1/16 and subtracting 64 + z, are
// exact in fp16 and leave the integer q - z.
struct ZeroConst {
    uint32_t lo;  // two copies of fp16 -(1024 + z)
    uint32_t hi;  // two copies of fp16 -(64 + z)
};

__device__ __forceinline__ ZeroConst zero_const(uint32_t z)
{
    ZeroConst c;
    const uint32_t zz = z | (z << 16);
    c.lo = 0xE400E400u | zz;          // -(1024 + z): ulp 1 -> z in the low mantissa bits
    c.hi = 0xD400D400u | (zz << 4);   // -(64 + z):   ulp 1/16 -> z shifted by 4
    return c;
}

// Field i of a packed word: bits [4i, 4i+3].
__device__ __forceinline__ uint32_t field(uint32_t word, int i) { return (word >> (4 * i)) & 0xFu; }

// The eight fields of `word` minus the zero point as fp16, in slot order
// [f0, f4, f1, f5, f2, f6, f3, f7] (the order in which the masks deliver them).
__device__ __forceinline__ half8_t unpack_shift(uint32_t word, ZeroConst c)
{
    const half2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t clo = __builtin_bit_cast(half2_t, c.lo);
    const half2_t chi = __builtin_bit_cast(half2_t, c.hi);
    const uint32_t w8 = word >> 8;
    const uint32_t t0 = (word & 0x000F000Fu) | 0x64006400u;  // 1024 + {f0, f4}
    const uint32_t t1 = (word & 0x00F000F0u) | 0x64006400u;  // 1024 + 16 {f1, f5}
    const uint32_t t2 = (w8 & 0x000F000Fu) | 0x64006400u;    // 1024 + {f2, f6}
    const uint32_t t3 = (w8 & 0x00F000F0u) | 0x64006400u;    // 1024 + 16 {f3, f7}
    const half2_t h0 = __builtin_bit_cast(half2_t, t0) + clo;
    const half2_t h1 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t1), sixteenth, chi);
    const half2_t h2 = __builtin_bit_cast(half2_t, t2) + clo;
    const half2_t h3 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t3), sixteenth, chi);
    u32x4_t packed = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                      __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3)};
    return __builtin_bit_cast(half8_t, packed);
}

// k offset (0..7) inside a packed word of the value held in slot s of unpack_shift's result.
__device__ __forceinline__ int slot_to_field(int s) { return (s >> 1) + 4 * (s & 1); }

// ------------------------------------------------------------------------------------------
// Global reads go through buffer instructions: the tensor's base and size sit in a scalar
// resource descriptor, the per-lane byte offset is a 32-bit register that never changes, and
// the per-group advance is a scalar offset, so the loop spends no vector ALU on addresses.
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    // word 3 = 0x00020000: raw buffer, 32-bit data format (the CDNA3/CDNA4 value)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// V consecutive 32-bit words.
template <int V> struct Words;
template <> struct Words<1> {
    uint32_t v[1];
    __device__ __forceinline__ void load(rsrc_t r, uint32_t voff, uint32_t soff)
    {
        v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
    }
};
template <> struct Words<2> {
    uint32_t v[2];
    __device__ __forceinline__ void load(rsrc_t r, uint32_t voff, uint32_t soff)
    {
        u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        v[0] = t.x; v[1] = t.y;
    }
};
template <> struct Words<4> {
    uint32_t v[4];
    __device__ __forceinline__ void load(rsrc_t r, uint32_t voff, uint32_t soff)
    {
        u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
};

// V consecutive fp16 scales as raw bits (two per 32-bit register).
template <int V> struct ScaleBits;
template <> struct ScaleBits<1> {
    uint32_t r[1];
    __device__ __forceinline__ void load(rsrc_t rs, uint32_t voff, uint32_t soff)
    {
        r[0] = __builtin_amdgcn_raw_buffer_load_b16(rs, voff, soff, 0);
    }
};
template <> struct ScaleBits<2> {
    uint32_t r[1];
    __device__ __forceinline__ void load(rsrc_t rs, uint32_t voff, uint32_t soff)
    {
        r[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, 0);
    }
};
template <> struct ScaleBits<4> {
    uint32_t r[2];
    __device__ __forceinline__ void load(rsrc_t rs, uint32_t voff, uint32_t soff)
    {
        u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, 0);
        r[0] = t.x; r[1] = t.y;
    }
};
template <int V>
__device__ __forceinline__ float scale_of(const ScaleBits<V>& s, int j)
{
    uint16_t bits = (uint16_t)(s.r[j >> 1] >> (16 * (j & 1)));
    return (float)__builtin_bit_cast(_Float16, bits);
}

// ------------------------------------------------------------------------------------------
// What one lane fetches for one quantisation group of its strip: IPG x V weight words
// (IPG = group_size / 32 MFMA steps), one qzeros word and V scales.
template <int V, int IPG>
struct GroupRegs {
    Words<V> w[IPG];
    uint32_t zword;
    ScaleBits<V> s;
};

// The lane's share of the group's activation slice: up to IPG 16-byte pieces.
template <int IPG>
struct ActRegs {
    u32x4_t a[IPG];
};

// Addressing that stays fixed for a lane during the whole kernel: 32-bit byte offsets into
// the four tensors.  A lane whose columns lie beyond n (a strip may overhang the matrix) reads
// the columns of lane 0 instead; its results are private to it and are never stored.
template <int V, int IPG>
struct LaneMap {
    static constexpr int CH = 4 * IPG;        // 16-byte pieces per activation row per compute group
    static constexpr int RPP = kWave / CH;    // activation rows fetched per pass
    static constexpr int RS = 64 * IPG + 16;  // LDS row stride in bytes (+16 spreads rows over banks)

    uint32_t off_w;   // ((lane / 16) * n + col0) * 4   into qweight
    uint32_t off_z;   // (col0 / 8) * 4                 into a qzeros row
    uint32_t off_s;   // col0 * 2                       into a scales row
    uint32_t off_a;   // (a_row * k + 8 * a_ch) * 2     into A
    int zshift;       // 4 * (col0 % 8)
    int a_row;        // staging role: activation row of the first pass
    int lds_wr;       // byte offset of the lane's staging store (first pass)
    int lds_rd;       // byte offset of the lane's MFMA operand read (step 0)
};

// Scalar view of the problem.  A "compute group" is 32 * IPG consecutive k; a quantisation
// group is (1 << param_shift) compute groups (group_size 256 runs as two halves of 128).
struct Tensors {
    rsrc_t A, qweight, scales, qzeros;
    int m, n, k;
    int param_shift;
};

template <int V, int IPG>
__device__ __forceinline__ void issue_weight_loads(GroupRegs<V, IPG>& r, const LaneMap<V, IPG>& lm,
                                                   const Tensors& t, int gi)
{
    const uint32_t gp = (uint32_t)gi >> t.param_shift;
    r.zword = __builtin_amdgcn_raw_buffer_load_b32(t.qzeros, lm.off_z, gp * (uint32_t)(t.n / 8) * 4u, 0);
    r.s.load(t.scales, lm.off_s, gp * (uint32_t)t.n * 2u);
#pragma unroll
    for (int it = 0; it < IPG; ++it)
        r.w[it].load(t.qweight, lm.off_w, ((uint32_t)gi * IPG + it) * 16u * (uint32_t)t.n);
}

template <int V, int IPG>
__device__ __forceinline__ void issue_act_loads(ActRegs<IPG>& r, const LaneMap<V, IPG>& lm, const Tensors& t, int gi)
{
    using LM = LaneMap<V, IPG>;
#pragma unroll
    for (int p = 0; p < IPG; ++p) {
        if (lm.a_row + p * LM::RPP < t.m)
            r.a[p] = __builtin_amdgcn_raw_buffer_load_b128(
                t.A, lm.off_a, ((uint32_t)gi * (32 * IPG) + (uint32_t)p * LM::RPP * (uint32_t)t.k) * 2u, 0);
    }
}

// Write the lane's share of the group's activation slice to the wave's LDS region, each
// 8-value piece permuted to the slot order of unpack_shift.
template <int V, int IPG>
__device__ __forceinline__ void stage_activations(const ActRegs<IPG>& r, const LaneMap<V, IPG>& lm, char* lds, int m)
{
    using LM = LaneMap<V, IPG>;
#pragma unroll
    for (int t = 0; t < IPG; ++t) {
        if (lm.a_row + t * LM::RPP < m) {
            const u32x4_t d = r.a[t];  // d.x = {a0,a1}, d.y = {a2,a3}, d.z = {a4,a5}, d.w = {a6,a7}
            u32x4_t e;
            e.x = (d.x & 0xFFFFu) | (d.z << 16);         // {a0, a4}
            e.y = (d.x >> 16) | (d.z & 0xFFFF0000u);     // {a1, a5}
            e.z = (d.y & 0xFFFFu) | (d.w << 16);         // {a2, a6}
            e.w = (d.y >> 16) | (d.w & 0xFFFF0000u);     // {a3, a7}
            *(u32x4_t*)(lds + lm.lds_wr + t * LM::RPP * LM::RS) = e;
        }
    }
}

// One quantisation group: IPG MFMA steps into a fresh 16x16 tile per column set, then
// acc += scale * tile in fp32.
template <int V, int IPG>
__device__ __forceinline__ void compute_group(const GroupRegs<V, IPG>& r, const LaneMap<V, IPG>& lm,
                                              const char* lds, float4_t (&acc)[V])
{
    ZeroConst zc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) zc[j] = zero_const((r.zword >> (lm.zshift + 4 * j)) & 0xFu);
    float4_t tile[V];
#pragma unroll
    for (int j = 0; j < V; ++j) tile[j] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < IPG; ++it) {
        const half8_t a8 = *(const half8_t*)(lds + lm.lds_rd + it * 64);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const half8_t b8 = unpack_shift(r.w[it].v[j], zc[j]);
            tile[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a8, b8, tile[j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const float s = scale_of<V>(r.s, j);
        acc[j] += s * tile[j];
    }
}

// Make LDS writes of this wave visible to the other lanes of the same wave, and keep the
// compiler from moving LDS accesses across this point.  LDS operations of one wave execute
// in program order, so no hardware barrier is needed.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The loop of Algorithm 1 for one wave: compute groups [g_begin, g_begin + g_count) of its
// strip.  While group i is computed, the weight words and activations of group i+1 are in
// flight (weights double-buffered in registers; activations single-buffered, because the
// staging store consumes them before the next fetch is issued).
template <int V, int IPG>
__device__ __forceinline__ void wave_mainloop(const Tensors& t, const LaneMap<V, IPG>& lm, char* lds, int g_begin,
                                              int g_count, float4_t (&acc)[V])
{
    GroupRegs<V, IPG> r0, r1;
    ActRegs<IPG> ar;
    issue_weight_loads<V, IPG>(r0, lm, t, g_begin);
    issue_act_loads<V, IPG>(ar, lm, t, g_begin);
    for (int i = 0; i < g_count; i += 2) {
        stage_activations<V, IPG>(ar, lm, lds, t.m);
        const bool has1 = (i + 1 < g_count);
        if (has1) {
            issue_weight_loads<V, IPG>(r1, lm, t, g_begin + i + 1);
            issue_act_loads<V, IPG>(ar, lm, t, g_begin + i + 1);
        }
        wave_lds_sync();
        compute_group<V, IPG>(r0, lm, lds, acc);
        wave_lds_sync();
        if (!has1) break;
        stage_activations<V, IPG>(ar, lm, lds, t.m);
        if (i + 2 < g_count) {
            issue_weight_loads<V, IPG>(r0, lm, t, g_begin + i + 2);
            issue_act_loads<V, IPG>(ar, lm, t, g_begin + i + 2);
        }
        wave_lds_sync();
        compute_group<V, IPG>(r1, lm, lds, acc);
        wave_lds_sync();
    }
}

template <int V, int IPG>
__device__ __forceinline__ LaneMap<V, IPG> make_lane_map(int lane, int n0, int m, int n, int k)
{
    using LM = LaneMap<V, IPG>;
    LM lm;
    const int col0 = n0 + V * (lane & 15);
    const int colc = col0 < n ? col0 : V * (lane & 15) % n;  // an overhanging lane reads valid columns
    lm.off_w = ((uint32_t)(lane >> 4) * (uint32_t)n + (uint32_t)colc) * 4u;
    lm.off_z = (uint32_t)(colc >> 3) * 4u;
    lm.off_s = (uint32_t)colc * 2u;
    lm.zshift = 4 * (colc & 7);
    const int a_ch = lane % LM::CH;
    lm.a_row = lane / LM::CH;
    lm.off_a = ((uint32_t)lm.a_row * (uint32_t)k + 8u * (uint32_t)a_ch) * 2u;
    lm.lds_wr = lm.a_row * LM::RS + a_ch * 16;
    const int mrow = lane & 15;
    const int arow = mrow < m ? mrow : m;  // row m of the region holds zeros
    lm.lds_rd = arow * LM::RS + (lane >> 4) * 16;
    return lm;
}

}  // namespace w4a16
