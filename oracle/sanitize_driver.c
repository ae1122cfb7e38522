/*
 * Host sanitizer driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY (CPU, no GPU code).
 *
 * Built together with w4a16_oracle.c under -fsanitize=address,undefined by tests/test_oracle_sanitize.py
 * and run once: every oracle function is called on small ragged shapes whose buffers are
 * allocated at their exact sizes, so that any index outside an input or output, any signed
 * overflow or bad shift in the oracle ends the run with a report.  Values are not checked here
 * (the pins do that); a checksum is printed so that the calls cannot be optimised away.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

float w4a16_oracle_half_to_float(uint16_t h);
uint16_t w4a16_oracle_double_to_half(double x);
void w4a16_oracle_unpack_qweight(const int32_t* qweight, uint8_t* q, int n, int k);
void w4a16_oracle_unpack_qzeros(const int32_t* qzeros, uint8_t* z, int n, int groups);
void w4a16_oracle_pack_qweight(const uint8_t* q, int32_t* qweight, int n, int k);
void w4a16_oracle_pack_qzeros(const uint8_t* z, int32_t* qzeros, int n, int groups);
void w4a16_oracle_dequant(const int32_t* qweight, const uint16_t* scales, const int32_t* qzeros, float* W, int n,
                          int k, int group_size);
int w4a16_oracle_gemm(const uint16_t* A, const int32_t* qweight, const uint16_t* scales, const int32_t* qzeros,
                      double* Cref, uint16_t* C16, int m, int n, int k, int group_size, int split_k, int block_k,
                      int acc_mode, int threads);
int w4a16_oracle_gemm_blocked(const uint16_t* A, const int32_t* qweight, const uint16_t* scales,
                              const int32_t* qzeros, double* Cref, uint16_t* C16, int m, int n, int k,
                              int group_size, int split_k, int block_k, int acc_mode, int threads);
int w4a16_oracle_unpack_qweight_bits(const int32_t* qweight, uint8_t* q, int n, int k, int bits);
int w4a16_oracle_unpack_qzeros_bits(const int32_t* qzeros, uint8_t* z, int n, int groups, int bits);
int w4a16_oracle_pack_qweight_bits(const uint8_t* q, int32_t* qweight, int n, int k, int bits);
int w4a16_oracle_pack_qzeros_bits(const uint8_t* z, int32_t* qzeros, int n, int groups, int bits);
int w4a16_oracle_gemm_bits(const uint16_t* A, const int32_t* qweight, const uint16_t* scales, const int32_t* qzeros,
                           double* Cref, uint16_t* C16, int m, int n, int k, int group_size, int bits, int threads);
int w4a16_oracle_gemm_gidx(const uint16_t* A, const int32_t* qweight, const uint16_t* scales, const int32_t* qzeros,
                           const int32_t* g_idx, double* Cref, uint16_t* C16, int m, int n, int k, int groups,
                           int threads);
void w4a16_oracle_unpack_qweight_3bit(const int32_t* qweight, uint8_t* q, int n, int k);
void w4a16_oracle_unpack_qzeros_3bit(const int32_t* qzeros, uint8_t* z, int n, int groups);
void w4a16_oracle_pack_qweight_3bit(const uint8_t* q, int32_t* qweight, int n, int k);
void w4a16_oracle_pack_qzeros_3bit(const uint8_t* z, int32_t* qzeros, int n, int groups);
int w4a16_oracle_gemm_3bit(const uint16_t* A, const int32_t* qweight, const uint16_t* scales, const int32_t* qzeros,
                           double* Cref, uint16_t* C16, int m, int n, int k, int group_size, int threads);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (uint32_t)(state >> 16);
}
static int32_t* words(size_t count)
{
    int32_t* p = (int32_t*)malloc(count * sizeof(int32_t));
    for (size_t i = 0; i < count; ++i) p[i] = (int32_t)next_u32();
    return p;
}
/* fp16 bit patterns of finite values of moderate size (exponent field 8..17) */
static uint16_t* halves(size_t count)
{
    uint16_t* p = (uint16_t*)malloc(count * sizeof(uint16_t));
    for (size_t i = 0; i < count; ++i) {
        const uint32_t r = next_u32();
        p[i] = (uint16_t)((r & 0x8000u) | ((8u + (r >> 16) % 10u) << 10) | (r & 0x3FFu));
    }
    return p;
}

static double run_width(int bits, int m, int n, int k, int g)
{
    const int f = bits == 3 ? 0 : 32 / bits;
    const size_t wrows = bits == 3 ? (size_t)k / 32 * 3 : (size_t)k / f;
    const size_t zcols = bits == 3 ? (size_t)n / 32 * 3 : (size_t)n / f;
    const int groups = k / g;
    int32_t* qw = words(wrows * n);
    int32_t* qz = words((size_t)groups * zcols);
    uint16_t* s = halves((size_t)groups * n);
    uint16_t* A = halves((size_t)m * k);
    double* C = (double*)malloc((size_t)m * n * sizeof(double));
    uint16_t* C16 = (uint16_t*)malloc((size_t)m * n * sizeof(uint16_t));
    uint8_t* q = (uint8_t*)malloc((size_t)k * n);
    uint8_t* z = (uint8_t*)malloc((size_t)groups * n);
    int32_t* qw2 = (int32_t*)malloc(wrows * n * sizeof(int32_t));
    int32_t* qz2 = (int32_t*)malloc((size_t)groups * zcols * sizeof(int32_t));
    double sum = 0.0;
    if (bits == 3) {
        w4a16_oracle_unpack_qweight_3bit(qw, q, n, k);
        w4a16_oracle_unpack_qzeros_3bit(qz, z, n, groups);
        w4a16_oracle_pack_qweight_3bit(q, qw2, n, k);
        w4a16_oracle_pack_qzeros_3bit(z, qz2, n, groups);
        if (w4a16_oracle_gemm_3bit(A, qw, s, qz, C, C16, m, n, k, g, 2) < 0) exit(3);
    } else {
        if (w4a16_oracle_unpack_qweight_bits(qw, q, n, k, bits) || w4a16_oracle_unpack_qzeros_bits(qz, z, n, groups, bits) ||
            w4a16_oracle_pack_qweight_bits(q, qw2, n, k, bits) || w4a16_oracle_pack_qzeros_bits(z, qz2, n, groups, bits))
            exit(4);
        if (w4a16_oracle_gemm_bits(A, qw, s, qz, C, C16, m, n, k, g, bits, 2) < 0) exit(5);
    }
    for (size_t i = 0; i < (size_t)m * n; ++i) sum += C[i] + C16[i];
    for (size_t i = 0; i < wrows * n; ++i) sum += (double)(qw2[i] == qw[i]);
    free(qw); free(qz); free(s); free(A); free(C); free(C16); free(q); free(z); free(qw2); free(qz2);
    return sum;
}

static double run_4bit(int m, int n, int k, int g)
{
    const int groups = k / g;
    int32_t* qw = words((size_t)k / 8 * n);
    int32_t* qz = words((size_t)groups * (n / 8));
    uint16_t* s = halves((size_t)groups * n);
    uint16_t* A = halves((size_t)m * k);
    double* C = (double*)malloc((size_t)m * n * sizeof(double));
    uint16_t* C16 = (uint16_t*)malloc((size_t)m * n * sizeof(uint16_t));
    uint8_t* q = (uint8_t*)malloc((size_t)k * n);
    uint8_t* z = (uint8_t*)malloc((size_t)groups * n);
    int32_t* qw2 = (int32_t*)malloc((size_t)k / 8 * n * sizeof(int32_t));
    int32_t* qz2 = (int32_t*)malloc((size_t)groups * (n / 8) * sizeof(int32_t));
    float* W = (float*)malloc((size_t)k * n * sizeof(float));
    int32_t* g_idx = (int32_t*)malloc((size_t)k * sizeof(int32_t));
    double sum = 0.0;
    w4a16_oracle_unpack_qweight(qw, q, n, k);
    w4a16_oracle_unpack_qzeros(qz, z, n, groups);
    w4a16_oracle_pack_qweight(q, qw2, n, k);
    w4a16_oracle_pack_qzeros(z, qz2, n, groups);
    w4a16_oracle_dequant(qw, s, qz, W, n, k, g);
    for (int acc = 0; acc < 2; ++acc)
        for (int variant = 0; variant < 4; ++variant) {
            const int split_k = variant == 0 ? 1 : 2, block_k = variant == 2 ? 8 : variant == 3 ? g : 0;
            if (w4a16_oracle_gemm(A, qw, s, qz, C, C16, m, n, k, g, split_k, block_k, acc, 2) < 0) exit(6);
            for (size_t i = 0; i < (size_t)m * n; ++i) sum += C[i] + C16[i];
            if (w4a16_oracle_gemm_blocked(A, qw, s, qz, C, variant & 1 ? C16 : NULL, m, n, k, g, split_k, block_k, acc, 2) < 0)
                exit(7);
            for (size_t i = 0; i < (size_t)m * n; ++i) sum -= C[i];
        }
    for (int kk = 0; kk < k; ++kk) g_idx[kk] = (int)(next_u32() % (uint32_t)groups);
    if (w4a16_oracle_gemm_gidx(A, qw, s, qz, g_idx, C, C16, m, n, k, groups, 2) < 0) exit(8);
    for (size_t i = 0; i < (size_t)m * n; ++i) sum += C[i];
    for (size_t i = 0; i < (size_t)k * n; ++i) sum += W[i];
    free(qw); free(qz); free(s); free(A); free(C); free(C16); free(q); free(z); free(qw2); free(qz2); free(W); free(g_idx);
    return sum;
}

int main(void)
{
    double sum = 0.0;
    for (uint32_t h = 0; h < 65536u; ++h) {
        const float f = w4a16_oracle_half_to_float((uint16_t)h);
        sum += (double)w4a16_oracle_double_to_half((double)f);
    }
    const double specials[] = {0.0, -0.0, 1e-320, 5.9e-8, 6.1e-5, 65504.0, 65520.0, 1e300, -1e300, 1.0 / 3.0};
    for (size_t i = 0; i < sizeof(specials) / sizeof(specials[0]); ++i) sum += w4a16_oracle_double_to_half(specials[i]);
    sum += run_4bit(1, 8, 32, 32);
    sum += run_4bit(3, 200, 256, 128);   /* ragged against the blocked arrangement's 128 columns */
    sum += run_4bit(16, 136, 128, 64);
    sum += run_width(2, 2, 48, 128, 64);
    sum += run_width(4, 5, 40, 128, 32);
    sum += run_width(8, 3, 36, 64, 32);
    sum += run_width(3, 4, 96, 128, 64);
    printf("oracle sanitizer run finished, checksum %.17g\n", sum);
    return 0;
}
