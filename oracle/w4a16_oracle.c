/*
 * CPU oracle for the fused W4A16 skinny GEMM  C[m,n] = A[m,k] . dequant(Wq)[k,n].
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP kernels are
 * checked against.  Nothing in the product path may call it; it shares no code, header,
 * table or helper with the HIP sources.
 *
 * What it follows (paper: "Accelerating a Triton Fused Kernel for W4A16 Quantized Inference
 * with SplitK work decomposition"):
 *   - Section 2, first paragraph: inputs are an fp16 activation matrix, a packed int32
 *     weight matrix and scale / zero parameters; the weights are unpacked with bitwise
 *     operations, shifted by the zero point and scaled (GPTQ-style int4).
 *   - Algorithm 1: an fp32 accumulator tile, a loop over k-blocks that adds dot products,
 *     and one final addition of every program's partial tile into C.  SplitK and the
 *     data-parallel tiling only change where and in which order partial sums are formed,
 *     so the result is the plain matrix product; this file is that product written out.
 *
 * Readings of points the paper leaves open (each is exercised by a test):
 *   - field i of a packed word is bits [4i, 4i+3]; in qweight field i of word row r is
 *     k = 8r + i; in qzeros field i of word column c is output column 8c + i;
 *   - w[kk][j] = (q[kk][j] - z[kk/g][j]) * s[kk/g][j], no "+1" zero-point offset;
 *   - groups are contiguous runs of g rows along k;
 *   - fp32 -> fp16 conversion rounds to nearest, ties to even.
 *
 * w4a16_oracle_gemm, the function every parity test calls, is the definition one output element
 * at a time: three nested loops (column, row, k), nothing cached, nothing blocked.
 * w4a16_oracle_gemm_blocked is the same arithmetic arranged in column blocks for the timed CPU
 * baseline only, held to the definition bit for bit by a test.
 *
 * Accumulation modes: 0 = fp64 accumulator (every product a*w is exact in fp64, so this is
 * the definition up to one rounding per addition at 2^-53), 1 = fp32 accumulator with fp32
 * products, the precision Algorithm 1 names.  Summation order is ascending k inside each
 * partial sum and ascending partition index across partial sums.
 *
 * Parity status: all functions below are pinned by tests/test_oracle_*.py against closed
 * forms, exact-rational brute force, numpy's float16 and matmul, and pack/unpack bijection;
 * which k index enters which partial sum by a hand-worked cancellation case in fp32;
 * the functions for other field widths (end of the file) by hand-written words, numpy byte
 * views, exact rationals, closed forms, numpy's matmul and, at 4 bits, the 4-bit functions;
 * the product with a group index per row by the contiguous case, numpy's matmul over a
 * gathered dense weight, invariance under reordering of the rows, and exact rationals;
 * the 3-bit functions (last section) by hand-written words with the two values that lie
 * across words, numpy's unpackbits over a little-endian byte view, bijection, the 4-bit
 * product on the same field values, numpy's matmul, exact rationals and one-hot rows.
 * Unpinned: agreement with the bit layout of the authors' own kernel and with real GPTQ
 * checkpoints (the paper prints neither).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- fp16 <-> fp32/fp64 */

float w4a16_oracle_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t f = h & 0x3FFu;
    uint32_t bits;
    if (e == 0) {
        if (f == 0) {
            bits = sign;
        } else { /* subnormal: value = f * 2^-24, normalise */
            int shift = 0;
            while (!(f & 0x400u)) { f <<= 1; ++shift; }
            f &= 0x3FFu;
            bits = sign | ((uint32_t)(127 - 15 + 1 - shift) << 23) | (f << 13);
        }
    } else if (e == 31) {
        bits = sign | 0x7F800000u | (f << 13);
    } else {
        bits = sign | ((e + 127 - 15) << 23) | (f << 13);
    }
    float out;
    memcpy(&out, &bits, 4);
    return out;
}

/* Round a double to the nearest fp16, ties to even, in one rounding. */
uint16_t w4a16_oracle_double_to_half(double x)
{
    uint64_t bits;
    memcpy(&bits, &x, 8);
    uint16_t sign = (uint16_t)((bits >> 63) << 15);
    int exp = (int)((bits >> 52) & 0x7FF);
    uint64_t man = bits & ((1ULL << 52) - 1);
    if (exp == 0x7FF) return (uint16_t)(sign | (man ? 0x7E00 : 0x7C00));
    if (exp == 0) return sign; /* zero or double subnormal: far below half's range */
    int e = exp - 1023;
    if (e > 15) return (uint16_t)(sign | 0x7C00);
    uint64_t sig = (1ULL << 52) | man; /* value = sig * 2^(e-52) */
    int shift = 42;                     /* keep 11 significant bits */
    if (e < -14) shift += (-14 - e);    /* half subnormal: fixed exponent -14 */
    if (shift > 63) return sign;
    uint64_t q = sig >> shift;
    uint64_t rem = sig & ((1ULL << shift) - 1);
    uint64_t halfway = 1ULL << (shift - 1);
    if (rem > halfway || (rem == halfway && (q & 1))) ++q;
    uint32_t out;
    if (e < -14) out = (uint32_t)q;                            /* q == 1024 becomes the least normal */
    else out = ((uint32_t)(e + 15) << 10) + (uint32_t)(q - 1024); /* q == 2048 carries into the exponent */
    return (uint16_t)(sign | out);
}

uint16_t w4a16_oracle_float_to_half(float x) { return w4a16_oracle_double_to_half((double)x); }

/* ---------------------------------------------------------------- pack / unpack */

/* q[kk][j] = field (kk % 8) of qweight[kk / 8][j];  q is uint8 [k, n]. */
void w4a16_oracle_unpack_qweight(const int32_t* qweight, uint8_t* q, int n, int k)
{
    for (int kk = 0; kk < k; ++kk)
        for (int j = 0; j < n; ++j) {
            uint32_t word = (uint32_t)qweight[(size_t)(kk / 8) * n + j];
            q[(size_t)kk * n + j] = (uint8_t)((word >> (4 * (kk % 8))) & 0xFu);
        }
}

/* z[gi][j] = field (j % 8) of qzeros[gi][j / 8];  z is uint8 [groups, n]. */
void w4a16_oracle_unpack_qzeros(const int32_t* qzeros, uint8_t* z, int n, int groups)
{
    for (int gi = 0; gi < groups; ++gi)
        for (int j = 0; j < n; ++j) {
            uint32_t word = (uint32_t)qzeros[(size_t)gi * (n / 8) + j / 8];
            z[(size_t)gi * n + j] = (uint8_t)((word >> (4 * (j % 8))) & 0xFu);
        }
}

void w4a16_oracle_pack_qweight(const uint8_t* q, int32_t* qweight, int n, int k)
{
    for (int r = 0; r < k / 8; ++r)
        for (int j = 0; j < n; ++j) {
            uint32_t word = 0;
            for (int i = 0; i < 8; ++i)
                word |= (uint32_t)(q[(size_t)(8 * r + i) * n + j] & 0xFu) << (4 * i);
            qweight[(size_t)r * n + j] = (int32_t)word;
        }
}

void w4a16_oracle_pack_qzeros(const uint8_t* z, int32_t* qzeros, int n, int groups)
{
    for (int gi = 0; gi < groups; ++gi)
        for (int c = 0; c < n / 8; ++c) {
            uint32_t word = 0;
            for (int i = 0; i < 8; ++i)
                word |= (uint32_t)(z[(size_t)gi * n + 8 * c + i] & 0xFu) << (4 * i);
            qzeros[(size_t)gi * (n / 8) + c] = (int32_t)word;
        }
}

/* ---------------------------------------------------------------- dequantisation */

static inline int field_of(const int32_t* words, size_t word_index, int field)
{
    return (int)(((uint32_t)words[word_index] >> (4 * field)) & 0xFu);
}

/* W[kk][j] = (q - z) * s as fp32; exact: |q - z| <= 15 and an fp16 scale has 11 bits. */
void w4a16_oracle_dequant(const int32_t* qweight, const uint16_t* scales, const int32_t* qzeros,
                          float* W, int n, int k, int group_size)
{
    for (int kk = 0; kk < k; ++kk) {
        int gi = kk / group_size;
        for (int j = 0; j < n; ++j) {
            int q = field_of(qweight, (size_t)(kk / 8) * n + j, kk % 8);
            int z = field_of(qzeros, (size_t)gi * (n / 8) + j / 8, j % 8);
            float s = w4a16_oracle_half_to_float(scales[(size_t)gi * n + j]);
            W[(size_t)kk * n + j] = (float)(q - z) * s;
        }
    }
}

/* ---------------------------------------------------------------- the product */

/* Which partial sum a k index belongs to.
 * block_k == 0: split_k contiguous chunks of k / split_k.
 * block_k  > 0: Algorithm 1's walk: program pid_k starts at k-block pid_k and advances by
 *               block_k * split_k, so k-block b belongs to partial sum b % split_k. */
static inline int partition_of(int kk, int k, int split_k, int block_k)
{
    if (split_k == 1) return 0;
    if (block_k == 0) return kk / (k / split_k);
    return (kk / block_k) % split_k;
}

/*
 * Cref (fp64 [m,n], required) and C16 (fp16 [m,n], may be NULL) <- A . dequant(Wq): the
 * definition, one output element at a time.
 * acc_mode 0: fp64 accumulators; 1: fp32 products and accumulators (Algorithm 1's accumulator).
 * split_k >= 1 partial sums are formed separately, each from zero over its own k indices in
 * ascending order, and then added in ascending partition order, as the final additions into C
 * of Algorithm 1 do in some order.
 * threads: OpenMP threads over output columns (every output element is computed by one thread,
 * by the loops below and nothing else); <= 0 means the runtime default.
 * Returns the number of threads used, or a negative number on bad arguments.
 */
int w4a16_oracle_gemm(const uint16_t* A, const int32_t* qweight, const uint16_t* scales,
                      const int32_t* qzeros, double* Cref, uint16_t* C16,
                      int m, int n, int k, int group_size,
                      int split_k, int block_k, int acc_mode, int threads)
{
    if (!A || !qweight || !scales || !qzeros || !Cref) return -1;
    if (m < 1 || n < 8 || n % 8 || group_size < 8 || group_size % 8 || k < group_size || k % group_size) return -2;
    if (split_k < 1 || (block_k == 0 && k % split_k) || block_k < 0) return -3;
    if (acc_mode != 0 && acc_mode != 1) return -4;

    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif

#pragma omp parallel for schedule(static)
    for (int j = 0; j < n; ++j) {
        for (int i = 0; i < m; ++i) {
            double total64 = 0.0;
            float total32 = 0.0f;
            for (int p = 0; p < split_k; ++p) {
                double part64 = 0.0;
                float part32 = 0.0f;
                for (int kk = 0; kk < k; ++kk) {
                    if (partition_of(kk, k, split_k, block_k) != p) continue;
                    const int grp = kk / group_size;
                    const int qd = field_of(qweight, (size_t)(kk / 8) * n + j, kk % 8);
                    const int zd = field_of(qzeros, (size_t)grp * (n / 8) + j / 8, j % 8);
                    const float sd = w4a16_oracle_half_to_float(scales[(size_t)grp * n + j]);
                    const float wd = (float)(qd - zd) * sd; /* exact */
                    const float ad = w4a16_oracle_half_to_float(A[(size_t)i * k + kk]);
                    if (acc_mode == 0) {
                        part64 += (double)ad * (double)wd;
                    } else {
                        const float prod = ad * wd;
                        part32 += prod;
                    }
                }
                total64 += part64;
                total32 += part32;
            }
            const double total = acc_mode == 0 ? total64 : (double)total32;
            Cref[(size_t)i * n + j] = total;
            if (C16) C16[(size_t)i * n + j] = w4a16_oracle_double_to_half(total);
        }
    }
    return used;
}

/*
 * The same product arranged for speed, for the timed CPU baseline only: blocks of 128 output
 * columns, one dequantised weight row kept per k index and used by all m activation rows, one
 * array of partial sums per block.  Per output element the operations and their order are those
 * of w4a16_oracle_gemm (ascending k inside a partial sum, ascending partition order), so the
 * results are the same bit for bit; a test holds it to that on several blocks and a ragged last
 * one.  No parity test uses this function.
 */
int w4a16_oracle_gemm_blocked(const uint16_t* A, const int32_t* qweight, const uint16_t* scales,
                              const int32_t* qzeros, double* Cref, uint16_t* C16,
                              int m, int n, int k, int group_size,
                              int split_k, int block_k, int acc_mode, int threads)
{
    if (!A || !qweight || !scales || !qzeros || !Cref) return -1;
    if (m < 1 || n < 8 || n % 8 || group_size < 8 || group_size % 8 || k < group_size || k % group_size) return -2;
    if (split_k < 1 || (block_k == 0 && k % split_k) || block_k < 0) return -3;
    if (acc_mode != 0 && acc_mode != 1) return -4;

    const int col_block = 128;
    const int n_blocks = (n + col_block - 1) / col_block;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif

#pragma omp parallel for schedule(static)
    for (int blk = 0; blk < n_blocks; ++blk) {
        const int j0 = blk * col_block;
        const int j1 = (j0 + col_block < n) ? j0 + col_block : n;
        const int w = j1 - j0;
        /* part[p][i][jj]: partial sum p of output (i, j0 + jj) */
        double* part64 = NULL;
        float* part32 = NULL;
        if (acc_mode == 0) part64 = (double*)calloc((size_t)split_k * m * w, sizeof(double));
        else part32 = (float*)calloc((size_t)split_k * m * w, sizeof(float));
        float* wrow = (float*)malloc((size_t)w * sizeof(float));

        for (int kk = 0; kk < k; ++kk) {
            const int gi = kk / group_size;
            const int p = partition_of(kk, k, split_k, block_k);
            for (int jj = 0; jj < w; ++jj) {
                const int j = j0 + jj;
                int q = field_of(qweight, (size_t)(kk / 8) * n + j, kk % 8);
                int z = field_of(qzeros, (size_t)gi * (n / 8) + j / 8, j % 8);
                float s = w4a16_oracle_half_to_float(scales[(size_t)gi * n + j]);
                wrow[jj] = (float)(q - z) * s; /* exact */
            }
            for (int i = 0; i < m; ++i) {
                const float a = w4a16_oracle_half_to_float(A[(size_t)i * k + kk]);
                if (acc_mode == 0) {
                    double* acc = part64 + ((size_t)p * m + i) * w;
                    for (int jj = 0; jj < w; ++jj) acc[jj] += (double)a * (double)wrow[jj];
                } else {
                    float* acc = part32 + ((size_t)p * m + i) * w;
                    for (int jj = 0; jj < w; ++jj) {
                        float prod = a * wrow[jj];
                        acc[jj] += prod;
                    }
                }
            }
        }
        for (int i = 0; i < m; ++i)
            for (int jj = 0; jj < w; ++jj) {
                double total;
                if (acc_mode == 0) {
                    double t = 0.0;
                    for (int p = 0; p < split_k; ++p) t += part64[((size_t)p * m + i) * w + jj];
                    total = t;
                } else {
                    float t = 0.0f;
                    for (int p = 0; p < split_k; ++p) t += part32[((size_t)p * m + i) * w + jj];
                    total = (double)t;
                }
                Cref[(size_t)i * n + j0 + jj] = total;
                if (C16) C16[(size_t)i * n + j0 + jj] = w4a16_oracle_double_to_half(total);
            }
        free(part64);
        free(part32);
        free(wrow);
    }
    return used;
}

/* ---------------------------------------------------------------- other field widths
 *
 * Section 2 of the paper remarks that the method carries over to other n-bit quantisation
 * schemes.  The same layout with fields of `bits` bits (2, 4 or 8), f = 32 / bits per word:
 *     q[kk][j]  = field (kk % f) of qweight[kk / f][j],   qweight int32 [k / f, n]
 *     z[gi][j]  = field (j % f)  of qzeros[gi][j / f],    qzeros  int32 [k / g, n / f]
 * field i = bits [bits * i, bits * i + bits - 1];  W = (q - z) * s as before.
 * Written on their own (they share nothing with the 4-bit functions above), so that
 * bits = 4 can be checked against those. */

static inline int bits_ok(int bits) { return bits == 2 || bits == 4 || bits == 8; }

static inline int field_of_width(const int32_t* words, size_t word_index, int field, int bits)
{
    const uint32_t mask = (1u << bits) - 1u;
    return (int)(((uint32_t)words[word_index] >> (bits * field)) & mask);
}

int w4a16_oracle_unpack_qweight_bits(const int32_t* qweight, uint8_t* q, int n, int k, int bits)
{
    if (!bits_ok(bits)) return -1;
    const int f = 32 / bits;
    for (int kk = 0; kk < k; ++kk)
        for (int j = 0; j < n; ++j)
            q[(size_t)kk * n + j] = (uint8_t)field_of_width(qweight, (size_t)(kk / f) * n + j, kk % f, bits);
    return 0;
}

int w4a16_oracle_unpack_qzeros_bits(const int32_t* qzeros, uint8_t* z, int n, int groups, int bits)
{
    if (!bits_ok(bits)) return -1;
    const int f = 32 / bits;
    for (int gi = 0; gi < groups; ++gi)
        for (int j = 0; j < n; ++j)
            z[(size_t)gi * n + j] = (uint8_t)field_of_width(qzeros, (size_t)gi * (n / f) + j / f, j % f, bits);
    return 0;
}

int w4a16_oracle_pack_qweight_bits(const uint8_t* q, int32_t* qweight, int n, int k, int bits)
{
    if (!bits_ok(bits)) return -1;
    const int f = 32 / bits;
    const uint32_t mask = (1u << bits) - 1u;
    for (int r = 0; r < k / f; ++r)
        for (int j = 0; j < n; ++j) {
            uint32_t word = 0;
            for (int i = 0; i < f; ++i) word |= ((uint32_t)q[(size_t)(f * r + i) * n + j] & mask) << (bits * i);
            qweight[(size_t)r * n + j] = (int32_t)word;
        }
    return 0;
}

int w4a16_oracle_pack_qzeros_bits(const uint8_t* z, int32_t* qzeros, int n, int groups, int bits)
{
    if (!bits_ok(bits)) return -1;
    const int f = 32 / bits;
    const uint32_t mask = (1u << bits) - 1u;
    for (int gi = 0; gi < groups; ++gi)
        for (int c = 0; c < n / f; ++c) {
            uint32_t word = 0;
            for (int i = 0; i < f; ++i) word |= ((uint32_t)z[(size_t)gi * n + f * c + i] & mask) << (bits * i);
            qzeros[(size_t)gi * (n / f) + c] = (int32_t)word;
        }
    return 0;
}

/* Cref (fp64 [m, n], required) and C16 (fp16 [m, n], may be NULL) <- A . W, the definition:
 * every product exact in fp64 ((q - z) * s is exact in fp32: at most 9 + 11 significant bits),
 * summed over k in ascending order in an fp64 accumulator.  Returns the OpenMP threads used or
 * a negative number on bad arguments. */
int w4a16_oracle_gemm_bits(const uint16_t* A, const int32_t* qweight, const uint16_t* scales,
                           const int32_t* qzeros, double* Cref, uint16_t* C16,
                           int m, int n, int k, int group_size, int bits, int threads)
{
    if (!A || !qweight || !scales || !qzeros || !Cref) return -1;
    if (!bits_ok(bits)) return -5;
    const int f = 32 / bits;
    if (m < 1 || n < f || n % f || group_size < f || group_size % f || k < group_size || k % group_size) return -2;

    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif

#pragma omp parallel for schedule(static)
    for (int j = 0; j < n; ++j) {
        for (int i = 0; i < m; ++i) {
            double sum = 0.0;
            for (int kk = 0; kk < k; ++kk) {
                const int gi = kk / group_size;
                const int qv = field_of_width(qweight, (size_t)(kk / f) * n + j, kk % f, bits);
                const int zv = field_of_width(qzeros, (size_t)gi * (n / f) + j / f, j % f, bits);
                const float sv = w4a16_oracle_half_to_float(scales[(size_t)gi * n + j]);
                const float wv = (float)(qv - zv) * sv; /* exact */
                const float av = w4a16_oracle_half_to_float(A[(size_t)i * k + kk]);
                sum += (double)av * (double)wv;
            }
            Cref[(size_t)i * n + j] = sum;
            if (C16) C16[(size_t)i * n + j] = w4a16_oracle_double_to_half(sum);
        }
    }
    return used;
}

/* ---------------------------------------------------------------- group index per row
 *
 * GPTQ's activation ordering (outside the paper, which has contiguous groups): the group of row
 * kk is g_idx[kk], any value in [0, groups), instead of kk / g.  4-bit fields as in Section 2:
 *     W[kk][j] = (q[kk][j] - z[g_idx[kk]][j]) * s[g_idx[kk]][j]
 * Written on its own; with g_idx[kk] = kk / g it must reproduce w4a16_oracle_gemm.
 * Returns the OpenMP threads used or a negative number on bad arguments (-6: a g_idx entry
 * outside [0, groups)). */
int w4a16_oracle_gemm_gidx(const uint16_t* A, const int32_t* qweight, const uint16_t* scales,
                           const int32_t* qzeros, const int32_t* g_idx, double* Cref, uint16_t* C16,
                           int m, int n, int k, int groups, int threads)
{
    if (!A || !qweight || !scales || !qzeros || !g_idx || !Cref) return -1;
    if (m < 1 || n < 8 || n % 8 || k < 8 || k % 8 || groups < 1) return -2;
    for (int kk = 0; kk < k; ++kk)
        if (g_idx[kk] < 0 || g_idx[kk] >= groups) return -6;

    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif

#pragma omp parallel for schedule(static)
    for (int j = 0; j < n; ++j) {
        for (int i = 0; i < m; ++i) {
            double sum = 0.0;
            for (int kk = 0; kk < k; ++kk) {
                const int row_group = g_idx[kk];
                const int qf = (int)(((uint32_t)qweight[(size_t)(kk / 8) * n + j] >> (4 * (kk % 8))) & 0xFu);
                const int zf = (int)(((uint32_t)qzeros[(size_t)row_group * (n / 8) + j / 8] >> (4 * (j % 8))) & 0xFu);
                const float sf = w4a16_oracle_half_to_float(scales[(size_t)row_group * n + j]);
                const float wf = (float)(qf - zf) * sf; /* exact */
                const float af = w4a16_oracle_half_to_float(A[(size_t)i * k + kk]);
                sum += (double)af * (double)wf;
            }
            Cref[(size_t)i * n + j] = sum;
            if (C16) C16[(size_t)i * n + j] = w4a16_oracle_double_to_half(sum);
        }
    }
    return used;
}

/* ---------------------------------------------------------------- 3-bit fields
 *
 * Section 2's remark again, for a width that does not divide 32.  Reading used here (the one
 * GPTQ checkpoints have): 32 consecutive values form a stream of 96 bits, value u at stream
 * bits [3u, 3u + 2], low bit first; stream bit b is bit (b % 32) of word (b / 32) of three
 * consecutive words.  Values 10 and 21 therefore lie across two words.
 *     qweight int32 [3 k / 32, n]:  word rows 3 t, 3 t + 1, 3 t + 2 of column j are the stream of
 *                                   k = 32 t .. 32 t + 31 of that column
 *     qzeros  int32 [k / g, 3 n / 32]: words 3 t, 3 t + 1, 3 t + 2 of a row are the stream of
 *                                   columns 32 t .. 32 t + 31
 * W = (q - z) * s as before.  Everything below goes bit by bit through that definition. */

static inline int stream3_bit(const int32_t* words, size_t first_word, size_t word_stride, int b)
{
    return (int)(((uint32_t)words[first_word + (size_t)(b / 32) * word_stride] >> (b % 32)) & 1u);
}

/* value u (0..31) of the 96-bit stream whose three words are first_word + {0, 1, 2} * word_stride */
static inline int stream3_value(const int32_t* words, size_t first_word, size_t word_stride, int u)
{
    int v = 0;
    for (int t = 0; t < 3; ++t) v |= stream3_bit(words, first_word, word_stride, 3 * u + t) << t;
    return v;
}

static inline void stream3_store(int32_t* words, size_t first_word, size_t word_stride, int u, int value)
{
    for (int t = 0; t < 3; ++t) {
        const int b = 3 * u + t;
        uint32_t w = (uint32_t)words[first_word + (size_t)(b / 32) * word_stride];
        w &= ~(1u << (b % 32));
        w |= (uint32_t)((value >> t) & 1) << (b % 32);
        words[first_word + (size_t)(b / 32) * word_stride] = (int32_t)w;
    }
}

void w4a16_oracle_unpack_qweight_3bit(const int32_t* qweight, uint8_t* q, int n, int k)
{
    for (int kk = 0; kk < k; ++kk)
        for (int j = 0; j < n; ++j)
            q[(size_t)kk * n + j] = (uint8_t)stream3_value(qweight, (size_t)(kk / 32) * 3 * n + j, (size_t)n, kk % 32);
}

void w4a16_oracle_unpack_qzeros_3bit(const int32_t* qzeros, uint8_t* z, int n, int groups)
{
    const size_t row_words = (size_t)n / 32 * 3;
    for (int gi = 0; gi < groups; ++gi)
        for (int j = 0; j < n; ++j)
            z[(size_t)gi * n + j] = (uint8_t)stream3_value(qzeros, (size_t)gi * row_words + (size_t)(j / 32) * 3, 1, j % 32);
}

void w4a16_oracle_pack_qweight_3bit(const uint8_t* q, int32_t* qweight, int n, int k)
{
    memset(qweight, 0, (size_t)k / 32 * 3 * n * sizeof(int32_t));
    for (int kk = 0; kk < k; ++kk)
        for (int j = 0; j < n; ++j)
            stream3_store(qweight, (size_t)(kk / 32) * 3 * n + j, (size_t)n, kk % 32, q[(size_t)kk * n + j] & 7);
}

void w4a16_oracle_pack_qzeros_3bit(const uint8_t* z, int32_t* qzeros, int n, int groups)
{
    const size_t row_words = (size_t)n / 32 * 3;
    memset(qzeros, 0, (size_t)groups * row_words * sizeof(int32_t));
    for (int gi = 0; gi < groups; ++gi)
        for (int j = 0; j < n; ++j)
            stream3_store(qzeros, (size_t)gi * row_words + (size_t)(j / 32) * 3, 1, j % 32, z[(size_t)gi * n + j] & 7);
}

/* Cref (fp64 [m, n], required) and C16 (fp16 [m, n], may be NULL) <- A . W, the definition,
 * summed over k in ascending order in an fp64 accumulator ((q - z) * s is exact in fp32).
 * Returns the OpenMP threads used or a negative number on bad arguments. */
int w4a16_oracle_gemm_3bit(const uint16_t* A, const int32_t* qweight, const uint16_t* scales,
                           const int32_t* qzeros, double* Cref, uint16_t* C16,
                           int m, int n, int k, int group_size, int threads)
{
    if (!A || !qweight || !scales || !qzeros || !Cref) return -1;
    if (m < 1 || n < 32 || n % 32 || group_size < 32 || group_size % 32 || k < group_size || k % group_size) return -2;

    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif

    const size_t zero_row_words = (size_t)n / 32 * 3;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < n; ++j) {
        for (int i = 0; i < m; ++i) {
            double sum = 0.0;
            for (int kk = 0; kk < k; ++kk) {
                const int group = kk / group_size;
                const int q3 = stream3_value(qweight, (size_t)(kk / 32) * 3 * n + j, (size_t)n, kk % 32);
                const int z3 = stream3_value(qzeros, (size_t)group * zero_row_words + (size_t)(j / 32) * 3, 1, j % 32);
                const float s3 = w4a16_oracle_half_to_float(scales[(size_t)group * n + j]);
                const float w3 = (float)(q3 - z3) * s3; /* exact */
                const float a3 = w4a16_oracle_half_to_float(A[(size_t)i * k + kk]);
                sum += (double)a3 * (double)w3;
            }
            Cref[(size_t)i * n + j] = sum;
            if (C16) C16[(size_t)i * n + j] = w4a16_oracle_double_to_half(sum);
        }
    }
    return used;
}
