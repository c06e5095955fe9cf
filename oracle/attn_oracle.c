/*
 * CPU oracle for scaled dot-product attention, O = softmax(Q K^T * scale) V  (paper Sec. 2.2, Eq. 1).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition written out in fp64: the score row is
 * materialised in full, the softmax is the two-pass textbook form (max, exp, sum, divide), and the
 * output is the plain weighted sum of the V rows.  There is no tiling, no online rescaling and no
 * reordering; nothing here is shared with, or derived from, the GPU library.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Query rows are independent in Eq. 1, so the N x N matrices S and P are produced one row at a time;
 * a caller may ask for any subset of rows (used to spot-check very long sequences) and may ask for
 * the rows of P themselves.
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC attn_oracle.c -o libattn_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* IEEE binary16 bit pattern -> double, exactly (every binary16 value is a double). */
static double f16_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0)        v = ldexp((double)mant, -24);              /* zero and subnormals: mant * 2^-24 */
    else if (expo == 31)  v = mant ? NAN : INFINITY;
    else                  v = ldexp((double)(mant | 0x400), expo - 25); /* (1024+mant) * 2^(expo-15-10) */
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exactly: a bfloat16 is the top half of a binary32. */
static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static void widen(const void* src, int dtype, long count, double* dst) {
    long t;
    if (dtype == ORACLE_F64) {
        memcpy(dst, src, (size_t)count * sizeof(double));
    } else if (dtype == ORACLE_F16) {
        const uint16_t* s = (const uint16_t*)src;
        for (t = 0; t < count; ++t) dst[t] = f16_bits_to_double(s[t]);
    } else {
        const uint16_t* s = (const uint16_t*)src;
        for (t = 0; t < count; ++t) dst[t] = bf16_bits_to_double(s[t]);
    }
}

/* Exposed so that the decoders can be pinned against an independent implementation. */
double attn_oracle_decode_f16(uint16_t h)  { return f16_bits_to_double(h); }
double attn_oracle_decode_bf16(uint16_t b) { return bf16_bits_to_double(b); }

/*
 * One (batch, head) slice.  Q, K, V: N x d row-major, element type `dtype`.
 * rows: indices of the query rows wanted (NULL = all N rows in order, n_rows is then ignored).
 * O: n_rows x d doubles.  rowsum (optional): sum_j P[i][j] after the division, per requested row.
 * P (optional): n_rows x N doubles, the softmax rows.
 * causal != 0: key j is visible to query i iff j <= i.
 * Returns 0, or 1 on bad arguments / allocation failure.
 */
int attn_oracle_head(const void* Q, const void* K, const void* V, int dtype,
                     long N, int d, double scale, int causal,
                     const long* rows, long n_rows,
                     double* O, double* rowsum, double* P, int n_threads) {
    if (!Q || !K || !V || !O || N <= 0 || d <= 0) return 1;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!rows) n_rows = N;
    if (n_rows < 0) return 1;
    {
        long r;
        if (rows) for (r = 0; r < n_rows; ++r) if (rows[r] < 0 || rows[r] >= N) return 1;
    }
    double* Qd = (double*)malloc((size_t)N * d * sizeof(double));
    double* Kd = (double*)malloc((size_t)N * d * sizeof(double));
    double* Vd = (double*)malloc((size_t)N * d * sizeof(double));
    if (!Qd || !Kd || !Vd) { free(Qd); free(Kd); free(Vd); return 1; }
    widen(Q, dtype, N * d, Qd);
    widen(K, dtype, N * d, Kd);
    widen(V, dtype, N * d, Vd);
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
#else
    n_threads = 1;
#endif
    int failed = 0;
#pragma omp parallel num_threads(n_threads)
    {
        double* s = (double*)malloc((size_t)N * sizeof(double));   /* one row of S, then of P */
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
        long r;
#pragma omp for schedule(dynamic, 4)
        for (r = 0; r < n_rows; ++r) {
            if (!s) continue;
            long i = rows ? rows[r] : r;
            const double* q = Qd + (size_t)i * d;
            long j; int c;
            /* S[i][j] = scale * <Q_i, K_j>;  masked entries are -inf */
            for (j = 0; j < N; ++j) {
                if (causal && j > i) { s[j] = -INFINITY; continue; }
                const double* k = Kd + (size_t)j * d;
                double dot = 0.0;
                for (c = 0; c < d; ++c) dot += q[c] * k[c];
                s[j] = scale * dot;
            }
            /* P[i][:] = softmax(S[i][:]) */
            double mx = -INFINITY;
            for (j = 0; j < N; ++j) if (s[j] > mx) mx = s[j];
            double Z = 0.0;
            for (j = 0; j < N; ++j) { s[j] = exp(s[j] - mx); Z += s[j]; }
            for (j = 0; j < N; ++j) s[j] /= Z;
            if (rowsum) { double t = 0.0; for (j = 0; j < N; ++j) t += s[j]; rowsum[r] = t; }
            if (P) memcpy(P + (size_t)r * N, s, (size_t)N * sizeof(double));
            /* O[i][:] = sum_j P[i][j] V[j][:] */
            double* o = O + (size_t)r * d;
            for (c = 0; c < d; ++c) o[c] = 0.0;
            for (j = 0; j < N; ++j) {
                const double* v = Vd + (size_t)j * d;
                double p = s[j];
                for (c = 0; c < d; ++c) o[c] += p * v[c];
            }
        }
        free(s);
    }
    free(Qd); free(Kd); free(Vd);
    return failed;
}

int attn_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
