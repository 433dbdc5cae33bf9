/*
 * CPU oracle for ABFT-protected matrix multiplication -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision / 64-bit-integer definitions of everything the
 * protected GEMM path computes.  Nothing in the product (the HIP library, its
 * Python binding) may include, link or call this file; it exists so that tests,
 * the smoke check and the benchmark's CPU-baseline leg have an independent
 * answer to compare with.  It shares no code, header, table or constant with
 * the GPU path.
 *
 * Notation follows the paper (Sec. 2.1): A is M x K (activations), B is K x N
 * (weights), C = A.B is M x N.  All matrices here are dense row-major arrays
 * with no padding (leading dimension = number of columns).
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC abft_oracle.c -o libabft_oracle.so
 * (-ffp-contract=off keeps every multiply and add a separately rounded fp64
 * operation, so the result does not depend on whether the host has FMA).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* number of host threads the parallel loops below will use */
int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- *
 * Storage formats -> double.  Inputs of the method are *already rounded*
 * fp16 / bf16 / int8 values; widening them is exact, so input rounding is
 * never an error source in the comparison.
 * ------------------------------------------------------------------------- */

/* IEEE 754 binary16 bit pattern -> double (exact). */
double orc_f16_bits_to_f64(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400), e - 25); /* (1024+m) * 2^(e-15-10) */
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double (exact): bf16 is the top half of a binary32. */
double orc_bf16_bits_to_f64(uint16_t b) {
    uint32_t w = (uint32_t)b << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

void orc_widen_f16(const uint16_t *src, size_t n, double *dst) {
    for (size_t i = 0; i < n; ++i) dst[i] = orc_f16_bits_to_f64(src[i]);
}

void orc_widen_bf16(const uint16_t *src, size_t n, double *dst) {
    for (size_t i = 0; i < n; ++i) dst[i] = orc_bf16_bits_to_f64(src[i]);
}

/* ------------------------------------------------------------------------- *
 * C = A.B by the definition C[i][j] = sum_k A[i][k] B[k][j]  (Sec. 2.1).
 * The k loop is the middle loop so that B is walked along rows; each C[i][j]
 * still receives its K products in ascending k, one rounded fp64 add at a
 * time, exactly as the textbook i-j-k dot-product order would.
 * ------------------------------------------------------------------------- */
void orc_gemm_f64(int M, int N, int K, const double *A, const double *B, double *C) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double *c = C + (size_t)i * N;
        for (int j = 0; j < N; ++j) c[j] = 0.0;
        for (int k = 0; k < K; ++k) {
            double a = A[(size_t)i * K + k];
            const double *b = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

/* int8 x int8 -> exact 64-bit integer result. */
void orc_gemm_i8(int M, int N, int K, const int8_t *A, const int8_t *B, int64_t *C) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        int64_t *c = C + (size_t)i * N;
        for (int j = 0; j < N; ++j) c[j] = 0;
        for (int k = 0; k < K; ++k) {
            int64_t a = A[(size_t)i * K + k];
            const int8_t *b = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) c[j] += a * (int64_t)b[j];
        }
    }
}

/* Selected rows of C only (for spot checks at sizes where all of C is too
 * slow): out[r][j] = sum_k A[rows[r]][k] B[k][j]. */
void orc_gemm_rows_f64(int nrows, const int *rows, int N, int K, const double *A, const double *B,
                       double *out) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < nrows; ++r) {
        const double *a = A + (size_t)rows[r] * K;
        double *c = out + (size_t)r * N;
        for (int j = 0; j < N; ++j) c[j] = 0.0;
        for (int k = 0; k < K; ++k) {
            const double *b = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) c[j] += a[k] * b[j];
        }
    }
}

void orc_gemm_rows_i8(int nrows, const int *rows, int N, int K, const int8_t *A, const int8_t *B,
                      int64_t *out) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < nrows; ++r) {
        const int8_t *a = A + (size_t)rows[r] * K;
        int64_t *c = out + (size_t)r * N;
        for (int j = 0; j < N; ++j) c[j] = 0;
        for (int k = 0; k < K; ++k) {
            const int8_t *b = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) c[j] += (int64_t)a[k] * (int64_t)b[j];
        }
    }
}

/* Running value of one accumulator after the products k = 0 .. k_after-1
 * (the quantity a mid-loop fault corrupts, Sec. 2.3). */
double orc_partial_dot_f64(int N, int K, const double *A, const double *B, int i, int j, int k_begin,
                           int k_end) {
    double s = 0.0;
    for (int k = k_begin; k < k_end; ++k) s += A[(size_t)i * K + k] * B[(size_t)k * N + j];
    return s;
}

int64_t orc_partial_dot_i8(int N, int K, const int8_t *A, const int8_t *B, int i, int j, int k_begin,
                           int k_end) {
    int64_t s = 0;
    for (int k = k_begin; k < k_end; ++k)
        s += (int64_t)A[(size_t)i * K + k] * (int64_t)B[(size_t)k * N + j];
    return s;
}

/* ------------------------------------------------------------------------- *
 * The four steps of ABFT for a matrix product (Sec. 2.4):
 *   (1) column checksum of A  alpha[k] = sum_i A[i][k]   (1 x K)
 *       row    checksum of B  beta[k]  = sum_j B[k][j]   (K x 1)
 *   (2) their dot product     s_AB = sum_k alpha[k] beta[k]
 *   (3) output summation      s_C  = sum_ij C[i][j]
 *   (4) compare (2) with (3).
 * ------------------------------------------------------------------------- */
void orc_col_checksum_f64(int M, int K, const double *A, double *alpha) {
    for (int k = 0; k < K; ++k) alpha[k] = 0.0;
    for (int i = 0; i < M; ++i)
        for (int k = 0; k < K; ++k) alpha[k] += A[(size_t)i * K + k];
}

void orc_row_checksum_f64(int K, int N, const double *B, double *beta) {
    for (int k = 0; k < K; ++k) {
        double s = 0.0;
        for (int j = 0; j < N; ++j) s += B[(size_t)k * N + j];
        beta[k] = s;
    }
}

void orc_col_checksum_i8(int M, int K, const int8_t *A, int64_t *alpha) {
    for (int k = 0; k < K; ++k) alpha[k] = 0;
    for (int i = 0; i < M; ++i)
        for (int k = 0; k < K; ++k) alpha[k] += A[(size_t)i * K + k];
}

void orc_row_checksum_i8(int K, int N, const int8_t *B, int64_t *beta) {
    for (int k = 0; k < K; ++k) {
        int64_t s = 0;
        for (int j = 0; j < N; ++j) s += B[(size_t)k * N + j];
        beta[k] = s;
    }
}

double orc_dot_f64(int K, const double *x, const double *y) {
    double s = 0.0;
    for (int k = 0; k < K; ++k) s += x[k] * y[k];
    return s;
}

int64_t orc_dot_i64(int K, const int64_t *x, const int64_t *y) {
    int64_t s = 0;
    for (int k = 0; k < K; ++k) s += x[k] * y[k];
    return s;
}

/* Sum of the r0..r1 x c0..c1 sub-block of a row-major M x N matrix
 * (whole matrix: r0=0, r1=M, c0=0, c1=N). */
double orc_block_sum_f64(int N, const double *C, int r0, int r1, int c0, int c1) {
    double s = 0.0;
    for (int i = r0; i < r1; ++i)
        for (int j = c0; j < c1; ++j) s += C[(size_t)i * N + j];
    return s;
}

int64_t orc_block_sum_i64(int N, const int64_t *C, int r0, int r1, int c0, int c1) {
    int64_t s = 0;
    for (int i = r0; i < r1; ++i)
        for (int j = c0; j < c1; ++j) s += C[(size_t)i * N + j];
    return s;
}

/* Scale of the operands that enters the floating-point comparison tolerance
 * of the global check:
 *   Phi = sqrt( sum_k ||A[:,k]||_2^2 * ||B[k,:]||_2^2 )
 * (the expected Frobenius norm of C when the columns of A / rows of B are
 * uncorrelated).  The paper states no tolerance; this is this build's reading. */
double orc_phi_f64(int M, int N, int K, const double *A, const double *B) {
    double acc = 0.0;
    for (int k = 0; k < K; ++k) {
        double a2 = 0.0, b2 = 0.0;
        for (int i = 0; i < M; ++i) a2 += A[(size_t)i * K + k] * A[(size_t)i * K + k];
        for (int j = 0; j < N; ++j) b2 += B[(size_t)k * N + j] * B[(size_t)k * N + j];
        acc += a2 * b2;
    }
    return sqrt(acc);
}

/* Worst-case scale S_abs = sum_k (sum_i |A[i][k]|)(sum_j |B[k][j]|): every
 * partial sum that can occur while forming C or either checksum is bounded by
 * it, so gamma * S_abs is a rigorous (if loose) bound on |s_C - s_AB|. */
double orc_sabs_f64(int M, int N, int K, const double *A, const double *B) {
    double acc = 0.0;
    for (int k = 0; k < K; ++k) {
        double a1 = 0.0, b1 = 0.0;
        for (int i = 0; i < M; ++i) a1 += fabs(A[(size_t)i * K + k]);
        for (int j = 0; j < N; ++j) b1 += fabs(B[(size_t)k * N + j]);
        acc += a1 * b1;
    }
    return acc;
}

/* ------------------------------------------------------------------------- *
 * Thread-level one-sided ABFT (Sec. 5.2.2, Table 1, right column), evaluated
 * for one register tile T = rows r0..r1-1, columns c0..c1-1 of C:
 *   chi[k]  = sum_{j in T} B[k][j]            checksum of the tile's B_t only
 *   rho[i]  = sum_k A[i][k] chi[k]            all of A_t times that checksum
 *   lhs     = sum_{(i,j) in T} C[i][j]        tile-local output summation
 *   rhs     = sum_{i in T} rho[i]
 * The tile passes when lhs == rhs (up to the tolerance for floating point).
 * C is passed in so that a corrupted C can be checked.
 * ------------------------------------------------------------------------- */
void orc_tile_one_sided_f64(int N, int K, const double *A, const double *B, const double *C, int r0,
                            int r1, int c0, int c1, double *lhs, double *rhs) {
    double sum_rho = 0.0;
    for (int i = r0; i < r1; ++i) {
        double rho = 0.0;
        for (int k = 0; k < K; ++k) {
            double chi = 0.0;
            for (int j = c0; j < c1; ++j) chi += B[(size_t)k * N + j];
            rho += A[(size_t)i * K + k] * chi;
        }
        sum_rho += rho;
    }
    *lhs = orc_block_sum_f64(N, C, r0, r1, c0, c1);
    *rhs = sum_rho;
}

void orc_tile_one_sided_i8(int N, int K, const int8_t *A, const int8_t *B, const int64_t *C, int r0,
                           int r1, int c0, int c1, int64_t *lhs, int64_t *rhs) {
    int64_t sum_rho = 0;
    for (int i = r0; i < r1; ++i) {
        int64_t rho = 0;
        for (int k = 0; k < K; ++k) {
            int64_t chi = 0;
            for (int j = c0; j < c1; ++j) chi += B[(size_t)k * N + j];
            rho += (int64_t)A[(size_t)i * K + k] * chi;
        }
        sum_rho += rho;
    }
    *lhs = orc_block_sum_i64(N, C, r0, r1, c0, c1);
    *rhs = sum_rho;
}

/* Two-sided variant (Sec. 5.2.2, Table 1, middle column): checksums of both
 * A_t and B_t, one product per k. */
void orc_tile_two_sided_f64(int N, int K, const double *A, const double *B, const double *C, int r0,
                            int r1, int c0, int c1, double *lhs, double *rhs) {
    double acc = 0.0;
    for (int k = 0; k < K; ++k) {
        double a = 0.0, chi = 0.0;
        for (int i = r0; i < r1; ++i) a += A[(size_t)i * K + k];
        for (int j = c0; j < c1; ++j) chi += B[(size_t)k * N + j];
        acc += a * chi;
    }
    *lhs = orc_block_sum_f64(N, C, r0, r1, c0, c1);
    *rhs = acc;
}

void orc_tile_two_sided_i8(int N, int K, const int8_t *A, const int8_t *B, const int64_t *C, int r0,
                           int r1, int c0, int c1, int64_t *lhs, int64_t *rhs) {
    int64_t acc = 0;
    for (int k = 0; k < K; ++k) {
        int64_t a = 0, chi = 0;
        for (int i = r0; i < r1; ++i) a += A[(size_t)i * K + k];
        for (int j = c0; j < c1; ++j) chi += B[(size_t)k * N + j];
        acc += a * chi;
    }
    *lhs = orc_block_sum_i64(N, C, r0, r1, c0, c1);
    *rhs = acc;
}

/* ------------------------------------------------------------------------- *
 * Fault model (Sec. 2.3): one wrong value in C, produced by processing logic.
 * Modelled as one flipped bit in the stored representation of an accumulator:
 * binary32 for the floating-point paths, two's-complement int32 for int8.
 * ------------------------------------------------------------------------- */
double orc_flip_bit_f32(double value, int bit) {
    float f = (float)value; /* the accumulator holds a binary32 */
    uint32_t w;
    memcpy(&w, &f, sizeof w);
    w ^= (uint32_t)1u << bit;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

int64_t orc_flip_bit_i32(int64_t value, int bit) {
    uint32_t w = (uint32_t)(int32_t)value;
    w ^= (uint32_t)1u << bit;
    return (int64_t)(int32_t)w;
}

/* ------------------------------------------------------------------------- *
 * Arithmetic intensity and the roofline test (Sec. 3.1, Eq. 1).
 *   FLOPs = 2 M N K,  Bytes = sA*M*K + sB*K*N + sC*M*N
 * with each dimension first rounded up to a multiple of pad_to (the paper pads
 * to multiples of 8 for its MMA shape, Sec. 6.2; pad_to = 1 means no padding).
 * ------------------------------------------------------------------------- */
static double pad_up(double x, int pad_to) {
    return pad_to > 1 ? ceil(x / pad_to) * pad_to : x;
}

double orc_flops(double M, double N, double K, int pad_to) {
    return 2.0 * pad_up(M, pad_to) * pad_up(N, pad_to) * pad_up(K, pad_to);
}

double orc_bytes(double M, double N, double K, double sA, double sB, double sC, int pad_to) {
    double m = pad_up(M, pad_to), n = pad_up(N, pad_to), k = pad_up(K, pad_to);
    return sA * m * k + sB * k * n + sC * m * n;
}

double orc_arithmetic_intensity(double M, double N, double K, double sA, double sB, double sC,
                                int pad_to) {
    return orc_flops(M, N, K, pad_to) / orc_bytes(M, N, K, sA, sB, sC, pad_to);
}

/* compute-to-memory-bandwidth ratio of a device: peak op/s over bytes/s */
double orc_cmr(double peak_ops_per_s, double bytes_per_s) { return peak_ops_per_s / bytes_per_s; }

/* Eq. 1: compute bound iff intensity > CMR (strictly). */
int orc_compute_bound(double intensity, double cmr) { return intensity > cmr; }

/* Intensity-guided choice (Sec. 5.3): 1 = global ABFT for compute-bound
 * layers, 2 = thread-level ABFT otherwise (ties go to thread-level because
 * Eq. 1 is a strict inequality). */
int orc_select(double intensity, double cmr) { return orc_compute_bound(intensity, cmr) ? 1 : 2; }

/* ------------------------------------------------------------------------- *
 * Convolution lowered to a matrix product (Sec. 2.1: layers are executed as
 * matrix multiplications).  x is NHWC (batch, H, W, Cin); row m of the
 * lowered matrix is output pixel (n, oh, ow) and column k is filter tap
 * (kh, kw, c); taps that fall in the zero padding contribute 0.
 * out is (batch*OH*OW) x (KH*KW*Cin), row-major.
 * ------------------------------------------------------------------------- */
void orc_im2col_f64(int batch, int H, int W, int Cin, int KH, int KW, int stride, int pad,
                    const double *x, double *out) {
    int OH = (H + 2 * pad - KH) / stride + 1;
    int OW = (W + 2 * pad - KW) / stride + 1;
    size_t Kdim = (size_t)KH * KW * Cin;
    for (int n = 0; n < batch; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                size_t m = ((size_t)n * OH + oh) * OW + ow;
                for (int kh = 0; kh < KH; ++kh)
                    for (int kw = 0; kw < KW; ++kw) {
                        int h = oh * stride - pad + kh;
                        int w = ow * stride - pad + kw;
                        for (int c = 0; c < Cin; ++c) {
                            size_t k = ((size_t)kh * KW + kw) * Cin + c;
                            double v = 0.0;
                            if (h >= 0 && h < H && w >= 0 && w < W)
                                v = x[(((size_t)n * H + h) * W + w) * Cin + c];
                            out[m * Kdim + k] = v;
                        }
                    }
            }
}
