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
//   * the activation operand is fetched straight into MFMA layout (row l%16, eight consecutive
//     k per lane) and permuted in registers to the field order the unpack produces; LDS is used
//     only to add up the tiles of the waves of a workgroup;
//   * loads are issued one MFMA step (32 k) at a time into a register ring two groups deep, so
//     a wave keeps about two groups of weights in flight while it computes.
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

// fp16 1024.0 twice.  Kept in a vector register (the asm hides the constant from the
// optimiser) so that "(word & mask) | magic" becomes one v_and_or_b32: on gfx9 a VOP3
// instruction can take only one scalar/literal operand, and the mask already is one.
__device__ __forceinline__ uint32_t magic_1024x2()
{
    uint32_t v;
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(v));
    return v;
}

// The eight fields of `word` minus the zero point as fp16, in slot order
// [f0, f4, f1, f5, f2, f6, f3, f7] (the order in which the masks deliver them).
__device__ __forceinline__ half8_t unpack_shift(uint32_t word, ZeroConst c, uint32_t magic)
{
    const half2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t clo = __builtin_bit_cast(half2_t, c.lo);
    const half2_t chi = __builtin_bit_cast(half2_t, c.hi);
    const uint32_t w8 = word >> 8;
    const uint32_t t0 = (word & 0x000F000Fu) | magic;  // 1024 + {f0, f4}
    const uint32_t t1 = (word & 0x00F000F0u) | magic;  // 1024 + 16 {f1, f5}
    const uint32_t t2 = (w8 & 0x000F000Fu) | magic;    // 1024 + {f2, f6}
    const uint32_t t3 = (w8 & 0x00F000F0u) | magic;    // 1024 + 16 {f3, f7}
    const half2_t h0 = __builtin_bit_cast(half2_t, t0) + clo;
    const half2_t h1 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t1), sixteenth, chi);
    const half2_t h2 = __builtin_bit_cast(half2_t, t2) + clo;
    const half2_t h3 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t3), sixteenth, chi);
    u32x4_t packed = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                      __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3)};
    return __builtin_bit_cast(half8_t, packed);
}

// 8-bit fields (Section 2 remarks that the method carries over to other n-bit schemes): a word
// holds four consecutive k of a column, so a lane's B operand is two words.  A byte OR-ed
// into the mantissa of fp16 1024.0 is 1024 + q exactly (q <= 255 < 2^10); v_perm_b32 builds
// two such halves per instruction from the word and a register of 0x64 bytes, in the order
// of k, so the activation operand needs no reordering.
struct ZeroConst8 {
    uint32_t lo;  // two copies of fp16 -(1024 + z), z <= 255
};

__device__ __forceinline__ ZeroConst8 zero_const8(uint32_t z)
{
    ZeroConst8 c;
    c.lo = 0xE400E400u | z | (z << 16);
    return c;
}

// 0x64 in every byte, kept in a vector register (see magic_1024x2: one literal per VOP3).
__device__ __forceinline__ uint32_t magic_64x4()
{
    uint32_t v;
    asm volatile("v_mov_b32 %0, 0x64646464" : "=v"(v));
    return v;
}

// Fields 0..3 of w0 and 0..3 of w1 (k = 8 consecutive values) minus the zero point, as fp16.
__device__ __forceinline__ half8_t unpack_shift8(uint32_t w0, uint32_t w1, ZeroConst8 c, uint32_t magic64)
{
    const half2_t clo = __builtin_bit_cast(half2_t, c.lo);
    const uint32_t t0 = __builtin_amdgcn_perm(magic64, w0, 0x04010400u);  // 1024 + {f0, f1}
    const uint32_t t1 = __builtin_amdgcn_perm(magic64, w0, 0x04030402u);  // 1024 + {f2, f3}
    const uint32_t t2 = __builtin_amdgcn_perm(magic64, w1, 0x04010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(magic64, w1, 0x04030402u);
    const half2_t h0 = __builtin_bit_cast(half2_t, t0) + clo;
    const half2_t h1 = __builtin_bit_cast(half2_t, t1) + clo;
    const half2_t h2 = __builtin_bit_cast(half2_t, t2) + clo;
    const half2_t h3 = __builtin_bit_cast(half2_t, t3) + clo;
    u32x4_t packed = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                      __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3)};
    return __builtin_bit_cast(half8_t, packed);
}

// 2-bit fields: a word holds sixteen consecutive k of a column, a lane's B operand is one half
// of it (`half_shift` = 0 or 16).  With y = h | h << 14 the pairs {f0,f1}, {f2,f3}, {f4,f5} sit
// at bits (0,16), (4,20), (8,24) of y, inside the mantissa of fp16 1024.0 in both halves, and
// {f6,f7} at bits (0,16) of y >> 12: a mask-or gives 1024 + q, 1024 + 16 q or 1024 + 256 q, and a
// packed add or fma (by 1/16 or 1/256) leaves q - z exactly, in the order of k.
struct ZeroConst2 {
    uint32_t c0;  // two copies of fp16 -(1024 + z)
    uint32_t c4;  // two copies of fp16 -(64 + z)
    uint32_t c8;  // two copies of fp16 -(4 + z)
};

__device__ __forceinline__ ZeroConst2 zero_const2(uint32_t z)
{
    ZeroConst2 c;
    const uint32_t zz = z | (z << 16);
    c.c0 = 0xE400E400u | zz;         // ulp 1
    c.c4 = 0xD400D400u | (zz << 4);  // ulp 1/16
    c.c8 = 0xC400C400u | (zz << 8);  // ulp 1/256
    return c;
}

__device__ __forceinline__ half8_t unpack_shift2(uint32_t word, int half_shift, ZeroConst2 c, uint32_t magic)
{
    const half2_t k16 = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t k256 = {(_Float16)0.00390625f, (_Float16)0.00390625f};
    const uint32_t h = (word >> half_shift) & 0xFFFFu;
    const uint32_t y = h | (h << 14);
    const uint32_t y2 = y >> 12;
    const uint32_t t0 = (y & 0x00030003u) | magic;   // 1024 + {f0, f1}
    const uint32_t t1 = (y & 0x00300030u) | magic;   // 1024 + 16 {f2, f3}
    const uint32_t t2 = (y & 0x03000300u) | magic;   // 1024 + 256 {f4, f5}
    const uint32_t t3 = (y2 & 0x00030003u) | magic;  // 1024 + {f6, f7}
    const half2_t h0 = __builtin_bit_cast(half2_t, t0) + __builtin_bit_cast(half2_t, c.c0);
    const half2_t h1 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t1), k16, __builtin_bit_cast(half2_t, c.c4));
    const half2_t h2 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t2), k256, __builtin_bit_cast(half2_t, c.c8));
    const half2_t h3 = __builtin_bit_cast(half2_t, t3) + __builtin_bit_cast(half2_t, c.c0);
    u32x4_t packed = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                      __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3)};
    return __builtin_bit_cast(half8_t, packed);
}

// 3-bit fields: 32 consecutive k of a column are a stream of 96 bits in three consecutive word
// rows, value u at stream bits [3u, 3u + 2].  A lane's eight k are 24 consecutive stream bits that
// start at a multiple of 24: inside one word or across two (`lo`, `hi`), brought down to bits
// 0..23 by one funnel shift.  y keeps f0..f3 in its low half and f4..f7 in its high half at bits
// 0, 3, 6, 9; fields at bits 0, 3, 6 lie inside the mantissa of fp16 1024.0, and f3 / f7 come from
// y >> 6: a mask-or gives 1024 + q, 1024 + 8 q or 1024 + 64 q, and a packed add or fma (by 1/8 or
// 1/64) leaves q - z exactly, in the slot order of unpack_shift.
struct ZeroConst3 {
    uint32_t c0;  // two copies of fp16 -(1024 + z)
    uint32_t c3;  // two copies of fp16 -(128 + z)
    uint32_t c6;  // two copies of fp16 -(16 + z)
};

__device__ __forceinline__ ZeroConst3 zero_const3(uint32_t z)
{
    ZeroConst3 c;
    const uint32_t zz = z | (z << 16);
    c.c0 = 0xE400E400u | zz;         // ulp 1
    c.c3 = 0xD800D800u | (zz << 3);  // ulp 1/8
    c.c6 = 0xCC00CC00u | (zz << 6);  // ulp 1/64
    return c;
}

__device__ __forceinline__ half8_t unpack_shift3(uint32_t lo, uint32_t hi, int funnel, ZeroConst3 c, uint32_t magic)
{
    const half2_t k8 = {(_Float16)0.125f, (_Float16)0.125f};
    const half2_t k64 = {(_Float16)0.015625f, (_Float16)0.015625f};
    const uint32_t x = __builtin_amdgcn_alignbit(hi, lo, (uint32_t)funnel);  // bits 0..23: f0..f7
    const uint32_t y = (x & 0x00000FFFu) | ((x << 4) & 0x0FFF0000u);
    const uint32_t y6 = y >> 6;
    const uint32_t t0 = (y & 0x00070007u) | magic;   // 1024 + {f0, f4}
    const uint32_t t1 = (y & 0x00380038u) | magic;   // 1024 + 8 {f1, f5}
    const uint32_t t2 = (y & 0x01C001C0u) | magic;   // 1024 + 64 {f2, f6}
    const uint32_t t3 = (y6 & 0x00380038u) | magic;  // 1024 + 8 {f3, f7}
    const half2_t h0 = __builtin_bit_cast(half2_t, t0) + __builtin_bit_cast(half2_t, c.c0);
    const half2_t h1 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t1), k8, __builtin_bit_cast(half2_t, c.c3));
    const half2_t h2 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t2), k64, __builtin_bit_cast(half2_t, c.c6));
    const half2_t h3 = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, t3), k8, __builtin_bit_cast(half2_t, c.c3));
    u32x4_t packed = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                      __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3)};
    return __builtin_bit_cast(half8_t, packed);
}

// Eight consecutive activations {a0..a7} (four registers, two per register) reordered to the
// slot order of unpack_shift: {a0,a4}, {a1,a5}, {a2,a6}, {a3,a7}.
__device__ __forceinline__ half8_t permute_activations(u32x4_t d)
{
    u32x4_t e;
    e.x = __builtin_amdgcn_perm(d.z, d.x, 0x05040100u);
    e.y = __builtin_amdgcn_perm(d.z, d.x, 0x07060302u);
    e.z = __builtin_amdgcn_perm(d.w, d.y, 0x05040100u);
    e.w = __builtin_amdgcn_perm(d.w, d.y, 0x07060302u);
    return __builtin_bit_cast(half8_t, e);
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

// Cache policy of the weight loads: the non-temporal hint.  Every packed word is read once per call, so
// it should not displace the activations and group parameters that the other workgroups of a compute
// die re-read from its L2 (same box, library plan, us per call: m = 8, n = k = 16384: 24.4-24.9 -> 23.2-23.5;
// n = 28672, k = 8192, m = 16: 23.6 -> 22.6; m = 16, n = k = 8192: 9.54 -> 9.35; n = k = 4096: 4.44 -> 4.38).
// Only on the 128-bit loads: a 16-column tile's 64 bytes of a word row share their cache line with the
// neighbouring tile's, which then has to fetch it again (n = 3480, k = 2176, m = 4, unsplit 16-column tiles: 4.2 -> 4.5).
constexpr int kWeightLoadAux = 2;  // the builtin's aux bit 1: `nt` on gfx950

// V consecutive 32-bit words of the weight stream.
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
        u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, kWeightLoadAux);
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
// One MFMA step (32 consecutive k) of a lane: V weight words (BITS = 4: eight k each) or twice
// V words (BITS = 8: word rows 2 kg and 2 kg + 1 of the step's eight, four k each) and its 8
// activations.
template <int V, int BITS = 4>
struct StepRegs {
    Words<V> w;
    u32x4_t a;
};
template <int V>
struct StepRegs<V, 8> {
    Words<V> w, w1;
    u32x4_t a;
};
// BITS = 3: the one or two word rows (of the step's three) that hold the lane's 24 stream bits
template <int V>
struct StepRegs<V, 3> {
    Words<V> w, w1;
    u32x4_t a;
};

// Per-group parameters of a lane: one qzeros word (3-bit fields: two, the lane's 3 V bits may lie
// across them) and V scales.
template <int V, int BITS = 4>
struct ParamRegs {
    uint32_t zword;
    ScaleBits<V> s;
};
template <int V>
struct ParamRegs<V, 3> {
    uint32_t zword, zword1;
    ScaleBits<V> s;
};

// Addressing that stays fixed for a lane during the whole kernel: 32-bit byte offsets into
// the four tensors.  A lane whose columns lie beyond n (a strip may overhang the matrix) reads
// valid columns of the matrix instead, and a lane whose activation row is >= m reads row m-1;
// in both cases what it computes lands in accumulator entries that are never stored.
struct LaneMap {
    uint32_t off_w;   // ((lane / 16) * n + col0) * 4       into qweight (8-bit fields: twice the row)
    uint32_t off_w1;  // 3-bit fields only: the word row that holds the upper part of the lane's 24 bits
    uint32_t off_z;   // (col0 / 8) * 4                     into a qzeros row
    uint32_t off_z1;  // 3-bit fields only: the next word when the lane's 3 V bits go across, else off_z
    uint32_t off_s;   // col0 * 2                           into a scales row
    uint32_t off_a;   // (row * k + 8 * (lane / 16)) * 2    into A, row = min(lane % 16, m - 1)
    int zshift;       // 4 * (col0 % 8)
    int half_shift;   // 2-bit fields: which half of the word the lane's eight k are (0 or 16);
                      // 3-bit fields: the funnel shift that brings the lane's 24 bits down (0, 24, 16, 8)
};

// Scalar view of the problem.  A "compute group" is 32 * IPG consecutive k; a quantisation
// group is (1 << param_shift) compute groups (group_size 256 runs as two halves of 128).
struct Tensors {
    rsrc_t A, qweight, scales, qzeros;
    int m, n, k;
    int param_shift;
};

// The weight words of MFMA step `step` along k (k = 32 * step) of a lane.
template <int V, int BITS = 4>
__device__ __forceinline__ void issue_step_weights(StepRegs<V, BITS>& r, const LaneMap& lm, const Tensors& t, uint32_t step)
{
    if constexpr (BITS == 8) {
        // eight word rows per step
        r.w.load(t.qweight, lm.off_w, step * 32u * (uint32_t)t.n);
        r.w1.load(t.qweight, lm.off_w, (step * 32u + 4u) * (uint32_t)t.n);
    } else if constexpr (BITS == 2) {
        // two word rows per step, each shared by two lane groups
        r.w.load(t.qweight, lm.off_w, step * 8u * (uint32_t)t.n);
    } else if constexpr (BITS == 3) {
        // three word rows per step
        r.w.load(t.qweight, lm.off_w, step * 12u * (uint32_t)t.n);
        r.w1.load(t.qweight, lm.off_w1, step * 12u * (uint32_t)t.n);
    } else {
        r.w.load(t.qweight, lm.off_w, step * 16u * (uint32_t)t.n);
    }
}

template <int V, int IPG, int BITS = 4>
__device__ __forceinline__ void issue_step(StepRegs<V, BITS>& r, const LaneMap& lm, const Tensors& t, int gi, int it)
{
    const uint32_t step = (uint32_t)gi * IPG + it;  // MFMA step index along k: k = 32 * step
    r.a = __builtin_amdgcn_raw_buffer_load_b128(t.A, lm.off_a, step * 64u, 0);
    issue_step_weights<V, BITS>(r, lm, t, step);
}

template <int V, int BITS = 4>
__device__ __forceinline__ void issue_params(ParamRegs<V, BITS>& r, const LaneMap& lm, const Tensors& t, int gi)
{
    const uint32_t gp = (uint32_t)gi >> t.param_shift;
    // a qzeros row is n * BITS / 32 words (written per width so that each keeps its shortest form)
    if constexpr (BITS == 3) {
        const uint32_t zrow = gp * (uint32_t)(t.n / 32 * 3) * 4u;
        r.zword = __builtin_amdgcn_raw_buffer_load_b32(t.qzeros, lm.off_z, zrow, 0);
        r.zword1 = __builtin_amdgcn_raw_buffer_load_b32(t.qzeros, lm.off_z1, zrow, 0);
    } else {
        r.zword = __builtin_amdgcn_raw_buffer_load_b32(t.qzeros, lm.off_z, gp * (uint32_t)(t.n / (32 / BITS)) * 4u, 0);
    }
    r.s.load(t.scales, lm.off_s, gp * (uint32_t)t.n * 2u);
}

// The unpack stage as functions of the field width, for kernels that keep rings of their own:
// the zero-point constant of the lane's column j, the B operand of that column for one step,
// the constant register the unpack needs, and the activations in the order of the fields.
template <int BITS> struct ZeroOf { using type = ZeroConst; };
template <> struct ZeroOf<8> { using type = ZeroConst8; };
template <> struct ZeroOf<3> { using type = ZeroConst3; };
template <> struct ZeroOf<2> { using type = ZeroConst2; };

template <int V, int BITS>
__device__ __forceinline__ typename ZeroOf<BITS>::type zero_of_column(const ParamRegs<V, BITS>& par, const LaneMap& lm, int j)
{
    if constexpr (BITS == 8) {
        return zero_const8((par.zword >> (lm.zshift + 8 * j)) & 0xFFu);
    } else if constexpr (BITS == 2) {
        return zero_const2((par.zword >> (lm.zshift + 2 * j)) & 0x3u);
    } else if constexpr (BITS == 3) {
        const uint32_t zbits = __builtin_amdgcn_alignbit(par.zword1, par.zword, (uint32_t)lm.zshift);
        return zero_const3((zbits >> (3 * j)) & 0x7u);
    } else {
        return zero_const((par.zword >> (lm.zshift + 4 * j)) & 0xFu);
    }
}

template <int V, int BITS>
__device__ __forceinline__ half8_t unpack_column(const StepRegs<V, BITS>& r, int j, const LaneMap& lm,
                                                 typename ZeroOf<BITS>::type zc, uint32_t magic)
{
    if constexpr (BITS == 8) return unpack_shift8(r.w.v[j], r.w1.v[j], zc, magic);
    else if constexpr (BITS == 2) return unpack_shift2(r.w.v[j], lm.half_shift, zc, magic);
    else if constexpr (BITS == 3) return unpack_shift3(r.w.v[j], r.w1.v[j], lm.half_shift, zc, magic);
    else return unpack_shift(r.w.v[j], zc, magic);
}

template <int BITS>
__device__ __forceinline__ uint32_t unpack_magic()
{
    if constexpr (BITS == 8) return magic_64x4();
    else return magic_1024x2();
}

// 4-bit and 3-bit fields come out in the slot order of unpack_shift, 8-bit and 2-bit ones in the order of k
template <int BITS>
__device__ __forceinline__ half8_t order_activations(u32x4_t d)
{
    if constexpr (BITS == 4 || BITS == 3) return permute_activations(d);
    else return __builtin_bit_cast(half8_t, d);
}

// Ring of two compute groups: half h holds the IPG steps and the parameters of one group.
template <int V, int IPG, int BITS = 4>
struct Ring {
    StepRegs<V, BITS> step[2][IPG];
    ParamRegs<V, BITS> par[2];
};

template <int V, int IPG, int H, int BITS = 4>
__device__ __forceinline__ void issue_group(Ring<V, IPG, BITS>& ring, const LaneMap& lm, const Tensors& t, int gi)
{
    issue_params<V, BITS>(ring.par[H], lm, t, gi);
#pragma unroll
    for (int it = 0; it < IPG; ++it) issue_step<V, IPG, BITS>(ring.step[H][it], lm, t, gi, it);
}

// A word in memory that the last compute group of a wave samples while it still has work to
// do, so that the round trip to memory is hidden (used by the split-k mode whose workgroups
// wait for the zeroing of their output tile; see the kernel).
struct FlagProbe {
    const uint32_t* addr;
    uint32_t value;
};

// One compute group out of ring half H: IPG MFMA steps into a fresh 16x16 tile per column
// set, then acc += scale * tile in fp32.  Each step's registers are refilled with the same
// step of group `refill` (two groups ahead) as soon as they have been consumed.  With PROBE the
// flag is sampled once the second step's weights have arrived.
template <int V, int IPG, int H, bool REFILL, bool PROBE, int BITS = 4>
__device__ __forceinline__ void compute_group(Ring<V, IPG, BITS>& ring, const LaneMap& lm, const Tensors& t,
                                              uint32_t magic, int refill, float4_t (&acc)[V], FlagProbe& probe)
{
    ZeroConst zc[V];
    ZeroConst8 zc8[V];
    ZeroConst2 zc2[V];
    ZeroConst3 zc3[V];
    float sc[V];
    uint32_t zbits3 = 0;
    if constexpr (BITS == 3)
        zbits3 = __builtin_amdgcn_alignbit(ring.par[H].zword1, ring.par[H].zword, (uint32_t)lm.zshift);
#pragma unroll
    for (int j = 0; j < V; ++j) {
        if constexpr (BITS == 8) zc8[j] = zero_const8((ring.par[H].zword >> (lm.zshift + 8 * j)) & 0xFFu);
        else if constexpr (BITS == 2) zc2[j] = zero_const2((ring.par[H].zword >> (lm.zshift + 2 * j)) & 0x3u);
        else if constexpr (BITS == 3) zc3[j] = zero_const3((zbits3 >> (3 * j)) & 0x7u);
        else zc[j] = zero_const((ring.par[H].zword >> (lm.zshift + 4 * j)) & 0xFu);
        sc[j] = scale_of<V>(ring.par[H].s, j);
    }
    if constexpr (REFILL) {
        // sched_barrier: keep the instruction scheduler from sinking the refill loads to the
        // end of the loop body (it would serialise load latency and compute)
        __builtin_amdgcn_sched_barrier(0);
        issue_params<V, BITS>(ring.par[H], lm, t, refill);
        __builtin_amdgcn_sched_barrier(0);
    }
    float4_t tile[V];
#pragma unroll
    for (int j = 0; j < V; ++j) tile[j] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < IPG; ++it) {
        half8_t a8, b8[V];
        if constexpr (BITS == 8) {
            // `magic` is the register of 0x64 bytes here; the fields come out in the order of k
            a8 = __builtin_bit_cast(half8_t, ring.step[H][it].a);
#pragma unroll
            for (int j = 0; j < V; ++j)
                b8[j] = unpack_shift8(ring.step[H][it].w.v[j], ring.step[H][it].w1.v[j], zc8[j], magic);
        } else if constexpr (BITS == 2) {
            a8 = __builtin_bit_cast(half8_t, ring.step[H][it].a);
#pragma unroll
            for (int j = 0; j < V; ++j) b8[j] = unpack_shift2(ring.step[H][it].w.v[j], lm.half_shift, zc2[j], magic);
        } else if constexpr (BITS == 3) {
            a8 = permute_activations(ring.step[H][it].a);
#pragma unroll
            for (int j = 0; j < V; ++j)
                b8[j] = unpack_shift3(ring.step[H][it].w.v[j], ring.step[H][it].w1.v[j], lm.half_shift, zc3[j], magic);
        } else {
            a8 = permute_activations(ring.step[H][it].a);
#pragma unroll
            for (int j = 0; j < V; ++j) b8[j] = unpack_shift(ring.step[H][it].w.v[j], zc[j], magic);
        }
        if constexpr (REFILL) {
            __builtin_amdgcn_sched_barrier(0);
            issue_step<V, IPG, BITS>(ring.step[H][it], lm, t, refill, it);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (PROBE) {
            if (it == (IPG > 1 ? 1 : 0)) {
                __builtin_amdgcn_sched_barrier(0);
                probe.value = __hip_atomic_load(probe.addr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int j = 0; j < V; ++j) tile[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a8, b8[j], tile[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] += sc[j] * tile[j];
}

// The loop of Algorithm 1 for one wave: compute groups [g_begin, g_begin + g_count) of its
// strip, with up to two groups of loads in flight.  wave_prime issues the first one or two
// groups; wave_run consumes them.  The steady-state loop refills without any branch, so the
// compiler's wait counts stay exact; the last one to three groups drain the ring.
// `primed()` runs once, after the loads have been issued, inside the branch that issued them:
// a wait it contains then counts exactly the loads of that branch.  GC is what is known about
// g_count at compile time: 1 = exactly one group, 2 = at least two, 0 = nothing.
template <int V, int IPG, int GC, int BITS = 4, class F>
__device__ __forceinline__ void wave_prime(Ring<V, IPG, BITS>& ring, const Tensors& t, const LaneMap& lm, int g_begin,
                                           int g_count, F&& primed)
{
    issue_group<V, IPG, 0, BITS>(ring, lm, t, g_begin);
    if constexpr (GC == 1) {
        primed();
    } else if constexpr (GC == 2) {
        issue_group<V, IPG, 1, BITS>(ring, lm, t, g_begin + 1);
        primed();
    } else {
        if (g_count > 1) {
            issue_group<V, IPG, 1, BITS>(ring, lm, t, g_begin + 1);
            primed();
        } else {
            primed();
        }
    }
}

template <int V, int IPG, bool PROBE, int GC, int BITS = 4>
__device__ __forceinline__ void wave_run(Ring<V, IPG, BITS>& ring, const Tensors& t, const LaneMap& lm, int g_begin,
                                         int g_count, float4_t (&acc)[V], FlagProbe& probe)
{
    uint32_t magic;
    if constexpr (BITS == 8) magic = magic_64x4();
    else magic = magic_1024x2();
    if constexpr (GC == 1) {
        compute_group<V, IPG, 0, false, PROBE, BITS>(ring, lm, t, magic, 0, acc, probe);
        return;
    }
    int i = 0;
    for (; i + 3 < g_count; i += 2) {
        compute_group<V, IPG, 0, true, false, BITS>(ring, lm, t, magic, g_begin + i + 2, acc, probe);
        compute_group<V, IPG, 1, true, false, BITS>(ring, lm, t, magic, g_begin + i + 3, acc, probe);
    }
    const int left = g_count - i;  // 1, 2 or 3 groups; half 0 holds group i, half 1 group i + 1
    if (left == 3) {
        compute_group<V, IPG, 0, true, false, BITS>(ring, lm, t, magic, g_begin + i + 2, acc, probe);
        compute_group<V, IPG, 1, false, false, BITS>(ring, lm, t, magic, 0, acc, probe);
        compute_group<V, IPG, 0, false, PROBE, BITS>(ring, lm, t, magic, 0, acc, probe);
    } else if (left == 2) {
        compute_group<V, IPG, 0, false, false, BITS>(ring, lm, t, magic, 0, acc, probe);
        compute_group<V, IPG, 1, false, PROBE, BITS>(ring, lm, t, magic, 0, acc, probe);
    } else if (left == 1) {
        compute_group<V, IPG, 0, false, PROBE, BITS>(ring, lm, t, magic, 0, acc, probe);
    }
}

template <int V, int BITS = 4>
__device__ __forceinline__ LaneMap make_lane_map(int lane, int n0, int m, int n, int k)
{
    LaneMap lm;
    lm.half_shift = 0;
    lm.off_w1 = 0;
    lm.off_z1 = 0;
    const int col0 = n0 + V * (lane & 15);
    const int colc = col0 < n ? col0 : 0;  // an overhanging lane reads the first columns (n >= 8 >= V)
    if constexpr (BITS == 8) {
        // lane group kg = lane / 16 takes word rows 2 kg and 2 kg + 1 of a step; four columns per zero word
        lm.off_w = (2u * (uint32_t)(lane >> 4) * (uint32_t)n + (uint32_t)colc) * 4u;
        lm.off_z = (uint32_t)(colc >> 2) * 4u;
        lm.zshift = 8 * (colc & 3);
    } else if constexpr (BITS == 2) {
        // lane groups 0, 1 take the two halves of word row 0 of a step, lane groups 2, 3 of row 1;
        // sixteen columns per zero word
        lm.off_w = ((uint32_t)(lane >> 5) * (uint32_t)n + (uint32_t)colc) * 4u;
        lm.off_z = (uint32_t)(colc >> 4) * 4u;
        lm.zshift = 2 * (colc & 15);
        lm.half_shift = 16 * ((lane >> 4) & 1);
    } else if constexpr (BITS == 3) {
        // lane group kg takes stream bits [24 kg, 24 kg + 24) of the step's 96: word rows
        // {0, 0}, {0, 1}, {1, 2}, {2, 2} and funnel shifts 0, 24, 16, 8; thirty-two columns per
        // three zero words
        const int kg = lane >> 4;
        const int row_lo = kg == 0 ? 0 : kg - 1, row_hi = kg == 3 ? 2 : kg;
        lm.off_w = ((uint32_t)row_lo * (uint32_t)n + (uint32_t)colc) * 4u;
        lm.off_w1 = ((uint32_t)row_hi * (uint32_t)n + (uint32_t)colc) * 4u;
        lm.half_shift = (32 - 8 * kg) & 31;
        lm.off_z = (uint32_t)((3 * colc) >> 5) * 4u;
        lm.zshift = (3 * colc) & 31;
        // V divides 32, so the lane's columns stay inside one stream of three words
        lm.off_z1 = lm.off_z + (lm.zshift + 3 * V > 32 ? 4u : 0u);
    } else {
        lm.off_w = ((uint32_t)(lane >> 4) * (uint32_t)n + (uint32_t)colc) * 4u;
        lm.off_z = (uint32_t)(colc >> 3) * 4u;
        lm.zshift = 4 * (colc & 7);
    }
    lm.off_s = (uint32_t)colc * 2u;
    const int mrow = lane & 15;
    const int arow = mrow < m ? mrow : m - 1;
    lm.off_a = ((uint32_t)arow * (uint32_t)k + 8u * (uint32_t)(lane >> 4)) * 2u;
    return lm;
}

}  // namespace w4a16
