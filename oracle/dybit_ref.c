/* Plain C oracle for DyBit.  TEST INFRASTRUCTURE ONLY.
 *
 * Scalar loops, float64 / int64 arithmetic, OpenMP across rows, no BLAS, no
 * intrinsics.  Written from the definitions in Sec. III-A (Eq. 1, Table I) and
 * the datapath description of Sec. III-B; shares no code with the HIP library.
 * It exists (a) as a second, independently typed statement of the definitions
 * that the numpy oracle is cross-checked against and (b) as the CPU baseline
 * that the benchmark times on the host cores.
 *
 * Codes are handled unpacked (one byte per code) except in ref_pack/ref_unpack.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int mag_bits(int bits, int is_signed) { return is_signed ? bits - 1 : bits; }

/* Eq. 1 with the Table I reading: zero, all-ones = 2^(m-1), start bit 0 =
 * fraction only, otherwise 2^(i-1) (1 + x / 2^k) with i leading ones. */
double ref_magnitude(int c, int m)
{
    if (c == 0) return 0.0;
    if (c == (1 << m) - 1) return ldexp(1.0, m - 1);
    if (((c >> (m - 1)) & 1) == 0) return ldexp((double)c, -(m - 1));
    int i = 0;
    for (int pos = m - 1; pos >= 0 && ((c >> pos) & 1); --pos) ++i;
    int k = m - i - 1;
    int x = c & ((1 << k) - 1);
    return ldexp(1.0 + ldexp((double)x, -k), i - 1);
}

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* values_out[code] for all 2^bits codes; sign-magnitude, sign=1/mag=0 -> +0. */
void ref_codebook(int bits, int is_signed, double *values_out)
{
    int m = mag_bits(bits, is_signed);
    for (int c = 0; c < (1 << m); ++c) {
        double v = ref_magnitude(c, m);
        values_out[c] = v;
        if (is_signed) values_out[(1 << m) | c] = (c == 0) ? 0.0 : -v;
    }
}

float ref_absmax_scale(const float *x, size_t n, int bits, int is_signed)
{
    float mx = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > mx) mx = a;            /* NaN compares false: ignored */
    }
    if (mx == 0.0f) return 1.0f;
    return mx / (float)ldexp(1.0, mag_bits(bits, is_signed) - 1);
}

/* Nearest code in exact arithmetic: rank of |x| among T_j = s * mid_j (exact in
 * double), ties to the even magnitude code. */
void ref_quantize(const float *x, size_t n, float scale, int bits, int is_signed,
                  uint8_t *codes_out)
{
    int m = mag_bits(bits, is_signed);
    int nmid = (1 << m) - 1;
    double T[256];
    for (int j = 0; j < nmid; ++j)
        T[j] = (double)scale * 0.5 * (ref_magnitude(j, m) + ref_magnitude(j + 1, m));
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < (long long)n; ++i) {
        float xv = x[i];
        if (xv != xv) { codes_out[i] = 0; continue; }
        double ax = fabs((double)xv);
        int lo = 0, hi = nmid;         /* rank = #{j : T_j < ax} */
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (T[mid] < ax) lo = mid + 1; else hi = mid;
        }
        int rank = lo;
        if (rank < nmid && T[rank] == ax && (rank & 1)) rank += 1;
        int neg = signbit(xv) ? 1 : 0;
        int code;
        if (is_signed) code = (neg && rank != 0) ? (rank | (1 << (bits - 1))) : rank;
        else code = neg ? 0 : rank;
        codes_out[i] = (uint8_t)code;
    }
}

void ref_dequantize(const uint8_t *codes, size_t n, float scale, int bits, int is_signed,
                    float *y_out)
{
    double cb[256];
    ref_codebook(bits, is_signed, cb);
    for (size_t i = 0; i < n; ++i) y_out[i] = scale * (float)cb[codes[i]];
}

/* Little-endian bit stream, code j in bits [j*bits, (j+1)*bits). */
void ref_pack(const uint8_t *codes, size_t n, int bits, uint8_t *out)
{
    size_t nbytes = (n * (size_t)bits + 7) / 8;
    memset(out, 0, nbytes);
    for (size_t j = 0; j < n; ++j) {
        size_t bit = j * (size_t)bits;
        unsigned v = (unsigned)codes[j] << (bit & 7);
        out[bit >> 3] |= (uint8_t)(v & 0xff);
        if (v >> 8) out[(bit >> 3) + 1] |= (uint8_t)(v >> 8);
    }
}

void ref_unpack(const uint8_t *buf, size_t n, int bits, uint8_t *codes_out)
{
    for (size_t j = 0; j < n; ++j) {
        size_t bit = j * (size_t)bits;
        unsigned v = buf[bit >> 3];
        if ((bit & 7) + (size_t)bits > 8) v |= (unsigned)buf[(bit >> 3) + 1] << 8;
        codes_out[j] = (uint8_t)((v >> (bit & 7)) & ((1u << bits) - 1));
    }
}

static void int_table(int bits, int is_signed, long long *tab)
{
    double cb[256];
    ref_codebook(bits, is_signed, cb);
    int m = mag_bits(bits, is_signed);
    for (int c = 0; c < (1 << bits); ++c) tab[c] = (long long)ldexp(cb[c], m - 1);
}

/* C[i][j] = sA*sW * sum_k vA[i][k] vW[j][k] (+bias[j]) (ReLU); D = the same sum
 * over absolute values (+|bias|).  Accumulates exact integers in int64. */
void ref_gemm(long long M, long long N, long long K,
              const uint8_t *a_codes, int a_bits, int a_signed, float a_scale,
              const uint8_t *w_codes, int w_bits, int w_signed, float w_scale,
              const float *bias, int relu, double *C, double *D)
{
    long long ta[256], tw[256];
    int_table(a_bits, a_signed, ta);
    int_table(w_bits, w_signed, tw);
    double unit = (double)a_scale * (double)w_scale *
                  ldexp(1.0, -(mag_bits(a_bits, a_signed) - 1) - (mag_bits(w_bits, w_signed) - 1));
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < M; ++i) {
        for (long long j = 0; j < N; ++j) {
            long long acc = 0, den = 0;
            for (long long k = 0; k < K; ++k) {
                long long p = ta[a_codes[i * K + k]] * tw[w_codes[j * K + k]];
                acc += p;
                den += p < 0 ? -p : p;
            }
            double c = (double)acc * unit, d = (double)den * unit;
            if (bias) { c += (double)bias[j]; d += fabs((double)bias[j]); }
            if (relu && c < 0.0) c = 0.0;
            C[i * N + j] = c;
            if (D) D[i * N + j] = d;
        }
    }
}

/* Direct convolution, x [B][H][W][Cin], w [Cout][kh][kw][Cin], y [B][Ho][Wo][Cout];
 * taps outside the image contribute exactly zero. */
void ref_conv2d(long long B, long long H, long long W, long long Cin, long long Cout,
                int kh, int kw, int stride, int pad,
                const uint8_t *x_codes, int x_bits, int x_signed, float x_scale,
                const uint8_t *w_codes, int w_bits, int w_signed, float w_scale,
                const float *bias, int relu, double *Y, double *D)
{
    long long tx[256], tw[256];
    int_table(x_bits, x_signed, tx);
    int_table(w_bits, w_signed, tw);
    long long Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    double unit = (double)x_scale * (double)w_scale *
                  ldexp(1.0, -(mag_bits(x_bits, x_signed) - 1) - (mag_bits(w_bits, w_signed) - 1));
#pragma omp parallel for schedule(static) collapse(2)
    for (long long b = 0; b < B; ++b)
        for (long long ho = 0; ho < Ho; ++ho)
            for (long long wo = 0; wo < Wo; ++wo)
                for (long long co = 0; co < Cout; ++co) {
                    long long acc = 0, den = 0;
                    for (int r = 0; r < kh; ++r) {
                        long long hi = ho * stride - pad + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int s = 0; s < kw; ++s) {
                            long long wi = wo * stride - pad + s;
                            if (wi < 0 || wi >= W) continue;
                            const uint8_t *xp = x_codes + ((b * H + hi) * W + wi) * Cin;
                            const uint8_t *wp = w_codes + ((co * kh + r) * kw + s) * Cin;
                            for (long long c = 0; c < Cin; ++c) {
                                long long p = tx[xp[c]] * tw[wp[c]];
                                acc += p;
                                den += p < 0 ? -p : p;
                            }
                        }
                    }
                    double v = (double)acc * unit, d = (double)den * unit;
                    if (bias) { v += (double)bias[co]; d += fabs((double)bias[co]); }
                    if (relu && v < 0.0) v = 0.0;
                    long long o = ((b * Ho + ho) * Wo + wo) * Cout + co;
                    Y[o] = v;
                    if (D) D[o] = d;
                }
}
