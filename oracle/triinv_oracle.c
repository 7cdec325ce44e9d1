/*
 * fp64 CPU oracle for the batched triangular inversion T = (I + A)^{-1}.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the hot path
 * computes.  It shares no code, header, table or constant with the HIP library; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * What is computed (paper, Sec. 1, Eq. 3 and Table 1; sign convention T = (I + A)^{-1}):
 *   A_ij = beta_i * exp(g_i - g_j) * <k_i, k_j>                     scalar gate   (GDN row)
 *   A_ij = beta_i * sum_c k_ic * k_jc * exp(g_ic - g_jc)            per-channel   (KDA row)
 *   A_ij = beta_i * <k_i, k_j>                                      no gate       (DeltaNet row)
 *   for i > j inside one chunk of C tokens, A_ij = 0 for i <= j (the strictly-lower mask L^-),
 * and T is the unique solution of (I + A) T = I, obtained by row-oriented forward
 * substitution:   T = I;  T[i,c] = - sum_{j=c}^{i-1} A[i,j] * T[j,c]   for c < i.
 * Every stored input value (fp32, fp16 or bf16) is widened exactly to fp64 first; all
 * arithmetic is IEEE fp64.
 *
 * Parity pins: every entry point is pinned by tests (closed forms, library inverse, brute
 * force, nilpotent Neumann sum, gate similarity); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2 };
enum { ORC_GATE_SCALAR = 0, ORC_GATE_PER_CHANNEL = 1, ORC_GATE_NONE = 2 };

static double widen_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* subnormal or zero */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

static double widen_bf16(uint16_t b)
{
    uint32_t bits = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double widen(const void *p, int64_t idx, int dtype)
{
    switch (dtype) {
    case ORC_F32: return (double)((const float *)p)[idx];
    case ORC_F16: return widen_f16(((const uint16_t *)p)[idx]);
    default: return widen_bf16(((const uint16_t *)p)[idx]);
    }
}

static int set_threads(int n_threads)
{
#ifdef _OPENMP
    int hw = omp_get_num_procs();
    if (n_threads <= 0 || n_threads > hw) n_threads = hw;
    return n_threads;
#else
    (void)n_threads;
    return 1;
#endif
}

int oracle_hw_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* One matrix: A (fp64, C x C, entries with i <= j ignored) -> T (fp64, C x C, dense). */
static void forward_substitution(const double *A, double *T, int C)
{
    for (int i = 0; i < C; ++i)
        for (int c = 0; c < C; ++c) T[(int64_t)i * C + c] = (i == c) ? 1.0 : 0.0;
    for (int i = 1; i < C; ++i)
        for (int c = 0; c < i; ++c) {
            double s = 0.0;
            for (int j = c; j < i; ++j) s += A[(int64_t)i * C + j] * T[(int64_t)j * C + c];
            T[(int64_t)i * C + c] = -s;
        }
}

/* T = (I + strict_lower(A))^{-1} for n_mat matrices already held in fp64. */
int oracle_tri_inv_f64(const double *A, double *T, int64_t n_mat, int C, int n_threads)
{
    if (n_mat < 0 || C <= 0) return -1;
    if (n_mat == 0) return 0;
    if (!A || !T) return -2;
    int nt = set_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int64_t m = 0; m < n_mat; ++m)
        forward_substitution(A + m * C * C, T + m * C * C, C);
    return 0;
}

/* Same, reading the matrices as stored (fp32 / fp16 / bf16), widening exactly. */
int oracle_tri_inv(const void *A, int in_dtype, double *T, int64_t n_mat, int C, int n_threads)
{
    if (n_mat < 0 || C <= 0 || in_dtype < 0 || in_dtype > 2) return -1;
    if (n_mat == 0) return 0;
    if (!A || !T) return -2;
    int nt = set_threads(n_threads);
    int rc = 0;
#pragma omp parallel num_threads(nt)
    {
        double *Ad = (double *)malloc(sizeof(double) * (size_t)C * C);
        if (!Ad) {
#pragma omp atomic write
            rc = -3;
        } else {
#pragma omp for schedule(static)
            for (int64_t m = 0; m < n_mat; ++m) {
                for (int i = 0; i < C; ++i)
                    for (int j = 0; j < C; ++j)
                        Ad[i * C + j] = (i > j) ? widen(A, m * C * C + (int64_t)i * C + j, in_dtype) : 0.0;
                forward_substitution(Ad, T + m * C * C, C);
            }
            free(Ad);
        }
    }
    return rc;
}

/*
 * Build A (fp64) for every chunk from the stored keys, beta and chunk-local cumulative
 * log-decay g.  K is [B, Tlen, H, d_k]; beta [B, Tlen, H]; g [B, Tlen, H] (scalar gate),
 * [B, Tlen, H, d_k] (per-channel gate) or unused.  Output matrix index
 * m = (b * (Tlen / C) + chunk) * H + h, each C x C row-major, zeros for i <= j.
 * The exponential is evaluated on the difference g_i - g_j, as the definition is written.
 * If sel != NULL only the n_sel matrices sel[0..n_sel) are built, written densely in that order
 * (used to check sampled outputs of workloads too large to redo entirely on the host).
 */
int oracle_build_A(const void *K, int k_dtype, const float *beta, const float *g, int gate_kind,
                   double *A, int B, int64_t Tlen, int H, int d_k, int C,
                   const int64_t *sel, int64_t n_sel, int n_threads)
{
    if (B <= 0 || H <= 0 || d_k <= 0 || C <= 0 || Tlen < 0 || Tlen % C) return -1;
    if (k_dtype < 0 || k_dtype > 2 || gate_kind < 0 || gate_kind > 2) return -1;
    if (!K || !beta || !A || (gate_kind != ORC_GATE_NONE && !g)) return -2;
    int64_t n_chunk = Tlen / C;
    int64_t n_all = (int64_t)B * n_chunk * H;
    int64_t n_out = sel ? n_sel : n_all;
    if (n_out < 0) return -1;
    for (int64_t s = 0; sel && s < n_sel; ++s)
        if (sel[s] < 0 || sel[s] >= n_all) return -1;
    int nt = set_threads(n_threads);
    int rc = 0;
#pragma omp parallel num_threads(nt)
    {
        double *kc = (double *)malloc(sizeof(double) * (size_t)C * d_k);
        double *gc = (double *)malloc(sizeof(double) * (size_t)C * d_k);
        if (!kc || !gc) {
#pragma omp atomic write
            rc = -3;
        } else {
#pragma omp for schedule(static)
            for (int64_t o = 0; o < n_out; ++o) {
                int64_t m = sel ? sel[o] : o;
                int h = (int)(m % H);
                int64_t chunk = (m / H) % n_chunk;
                int64_t b = m / ((int64_t)H * n_chunk);
                for (int i = 0; i < C; ++i) {
                    int64_t tok = (b * Tlen + chunk * C + i) * H + h; /* index into [B,Tlen,H] */
                    for (int c = 0; c < d_k; ++c) {
                        kc[i * d_k + c] = widen(K, tok * d_k + c, k_dtype);
                        if (gate_kind == ORC_GATE_PER_CHANNEL) gc[i * d_k + c] = (double)g[tok * d_k + c];
                    }
                    if (gate_kind == ORC_GATE_SCALAR) gc[i] = (double)g[tok];
                }
                double *Am = A + o * C * C;
                for (int i = 0; i < C; ++i) {
                    int64_t tok = (b * Tlen + chunk * C + i) * H + h;
                    double bi = (double)beta[tok];
                    for (int j = 0; j < C; ++j) {
                        double v = 0.0;
                        if (i > j) {
                            double s = 0.0;
                            if (gate_kind == ORC_GATE_PER_CHANNEL) {
                                for (int c = 0; c < d_k; ++c)
                                    s += kc[i * d_k + c] * kc[j * d_k + c] * exp(gc[i * d_k + c] - gc[j * d_k + c]);
                            } else {
                                for (int c = 0; c < d_k; ++c) s += kc[i * d_k + c] * kc[j * d_k + c];
                                if (gate_kind == ORC_GATE_SCALAR) s *= exp(gc[i] - gc[j]);
                            }
                            v = bi * s;
                        }
                        Am[i * C + j] = v;
                    }
                }
            }
        }
        free(kc);
        free(gc);
    }
    return rc;
}

/* Fused flavour: build A as above, then invert.  T is fp64 [n_mat or n_sel, C, C]. */
int oracle_gdn_chunk_tri_inv(const void *K, int k_dtype, const float *beta, const float *g, int gate_kind,
                             double *T, int B, int64_t Tlen, int H, int d_k, int C,
                             const int64_t *sel, int64_t n_sel, int n_threads)
{
    if (C <= 0 || Tlen < 0 || (C > 0 && Tlen % C)) return -1;
    int64_t n_mat = sel ? n_sel : (int64_t)B * (Tlen / C) * H;
    if (n_mat == 0) return 0;
    double *A = (double *)malloc(sizeof(double) * (size_t)n_mat * C * C);
    if (!A) return -3;
    int rc = oracle_build_A(K, k_dtype, beta, g, gate_kind, A, B, Tlen, H, d_k, C, sel, n_sel, n_threads);
    if (rc == 0) rc = oracle_tri_inv_f64(A, T, n_mat, C, n_threads);
    free(A);
    return rc;
}
