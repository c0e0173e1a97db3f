/*
 * CPU oracle for the group-wise 4-bit-weight / fp16-activation (W4A16) linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or call this file;
 * it exists so that tests, the smoke check and the benchmark's cpu_baseline leg have a slow,
 * plainly written definition to compare the GPU library against.  It shares no code with the
 * GPU library.
 *
 * What is computed (paper section 2.2, "W4A16": weights quantised to 4 bits with a group size
 * of 128, activations kept at 16 bits; the linear layer is y = x . dequant(W)):
 *   1. unpack   q[k,n] = 4-bit field k%8 of qweight[k/8, n];  z[g,n] = field n%8 of qzeros[g, n/8]
 *   2. dequant  w[k,n] = (float)(q[k,n] - z[k/G,n]) * (float)s[k/G,n]           (exact in fp32)
 *   3. matmul   y32[m,n] = sum_{k=0..K-1} (float)x[m,k] * w[k,n], fp32 multiply then fp32 add,
 *               k ascending; an fp64 shadow y64 of the same sum is kept to size the fp32 error
 *   4. round    y16 = round-to-nearest-even fp16 of y32
 * The paper prints no storage layout and no worked numerical example; the layout is the
 * canonical one described in the input generator, and every function is pinned by the CPU tests
 * (round trips, closed forms, brute force in rational arithmetic, library cross-checks).
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC  (no fast-math: order of the
 * k-sum is part of the definition).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- IEEE binary16 <-> binary32, written out (gcc 11 on x86 has no _Float16) ---- */

float orc_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t bits;
    if (exp == 0) {
        if (man == 0) {
            bits = sign;
        } else { /* subnormal: value = man * 2^-24; normalise */
            int e = -1;
            do { man <<= 1; e++; } while (!(man & 0x400u));
            man &= 0x3FFu;
            bits = sign | ((uint32_t)(127 - 15 - e) << 23) | (man << 13);
        }
    } else if (exp == 31) {
        bits = sign | 0x7F800000u | (man << 13);
    } else {
        bits = sign | ((exp + 127 - 15) << 23) | (man << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

uint16_t orc_f32_to_f16(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t absx = x & 0x7FFFFFFFu;
    if (absx >= 0x7F800000u) { /* inf or nan */
        if (absx == 0x7F800000u) return sign | 0x7C00u;
        return sign | 0x7E00u | (uint16_t)((absx >> 13) & 0x3FFu);
    }
    if (absx >= 0x477FF000u) { /* >= 65520 rounds to inf */
        return sign | 0x7C00u;
    }
    if (absx < 0x33000001u) { /* <= 2^-25: rounds to zero (ties-to-even at exactly 2^-25) */
        return sign;
    }
    int32_t e = (int32_t)(absx >> 23) - 127; /* unbiased */
    uint32_t m = (absx & 0x7FFFFFu) | 0x800000u; /* 24-bit significand */
    int shift;          /* bits dropped from the 24-bit significand */
    uint32_t hexp;
    if (e < -14) {      /* result subnormal: value = m * 2^(e-23), unit 2^-24 */
        shift = -e - 1; /* 13 + (-14 - e) */
        hexp = 0;
    } else {
        shift = 13;
        hexp = (uint32_t)(e + 15);
    }
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept++;
    uint32_t out;
    if (hexp == 0) {
        out = kept; /* kept may reach 0x400 -> smallest normal, encoding still right */
    } else {
        out = (hexp << 10) + (kept - 0x400u); /* carry out of kept bumps the exponent */
    }
    return sign | (uint16_t)out;
}

void orc_f16_to_f32_array(const uint16_t *h, float *f, size_t n)
{
    for (size_t i = 0; i < n; i++) f[i] = orc_f16_to_f32(h[i]);
}

void orc_f32_to_f16_array(const float *f, uint16_t *h, size_t n)
{
    for (size_t i = 0; i < n; i++) h[i] = orc_f32_to_f16(f[i]);
}

/* ---- step 1: unpack ---- */

void orc_unpack_codes(const int32_t *qweight, uint8_t *q, int K, int N)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++) {
            uint32_t word = (uint32_t)qweight[(size_t)(k >> 3) * N + n];
            q[(size_t)k * N + n] = (uint8_t)((word >> (4 * (k & 7))) & 0xFu);
        }
}

void orc_unpack_zeros(const int32_t *qzeros, uint8_t *z, int groups, int N)
{
    for (int g = 0; g < groups; g++)
        for (int n = 0; n < N; n++) {
            uint32_t word = (uint32_t)qzeros[(size_t)g * (N / 8) + (n >> 3)];
            z[(size_t)g * N + n] = (uint8_t)((word >> (4 * (n & 7))) & 0xFu);
        }
}

/* ---- step 2: dequantise to fp32, W[k,n] row-major ---- */

void orc_dequant(const int32_t *qweight, const uint16_t *scales, const int32_t *qzeros,
                 float *W, int N, int K, int G)
{
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; k++) {
        int g = k / G;
        for (int n = 0; n < N; n++) {
            uint32_t cw = (uint32_t)qweight[(size_t)(k >> 3) * N + n];
            uint32_t zw = (uint32_t)qzeros[(size_t)g * (N / 8) + (n >> 3)];
            int q = (int)((cw >> (4 * (k & 7))) & 0xFu);
            int z = (int)((zw >> (4 * (n & 7))) & 0xFu);
            float s = orc_f16_to_f32(scales[(size_t)g * N + n]);
            W[(size_t)k * N + n] = (float)(q - z) * s;
        }
    }
}

/* ---- steps 3 and 4: y32[m,n] = sum_k x[m,k] * W[k,n] (k ascending), fp64 shadow, fp16 rounding.
 * The loops run m, k, n so that the inner loop walks a row of W; each y[m,n] still receives its
 * K terms one at a time in ascending k, which is the definition.  y64 and y16 may be NULL. ---- */

void orc_matmul(const uint16_t *x, const float *W, float *y32, double *y64, uint16_t *y16,
                int M, int N, int K)
{
    const int chunk = 512; /* columns per parallel task; has no effect on any y[m,n] */
    int nchunks = (N + chunk - 1) / chunk;
#pragma omp parallel for schedule(dynamic)
    for (int c = 0; c < nchunks; c++) {
        int n0 = c * chunk;
        int n1 = n0 + chunk < N ? n0 + chunk : N;
        for (int m = 0; m < M; m++) {
            float *yr = y32 + (size_t)m * N;
            double *yd = y64 ? y64 + (size_t)m * N : NULL;
            for (int n = n0; n < n1; n++) yr[n] = 0.0f;
            if (yd) for (int n = n0; n < n1; n++) yd[n] = 0.0;
            for (int k = 0; k < K; k++) {
                float xv = orc_f16_to_f32(x[(size_t)m * K + k]);
                const float *wr = W + (size_t)k * N;
                for (int n = n0; n < n1; n++) {
                    float prod = xv * wr[n];
                    yr[n] = yr[n] + prod;
                }
                if (yd) {
                    double xd = (double)xv;
                    for (int n = n0; n < n1; n++) yd[n] += xd * (double)wr[n];
                }
            }
            if (y16) for (int n = n0; n < n1; n++) y16[(size_t)m * N + n] = orc_f32_to_f16(yr[n]);
        }
    }
}

/* whole layer in one call; W is caller-provided scratch of K*N floats */
void orc_gemm(const uint16_t *x, const int32_t *qweight, const uint16_t *scales,
              const int32_t *qzeros, float *W, float *y32, double *y64, uint16_t *y16,
              int M, int N, int K, int G)
{
    orc_dequant(qweight, scales, qzeros, W, N, K, G);
    orc_matmul(x, W, y32, y64, y16, M, N, K);
}

int orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}
