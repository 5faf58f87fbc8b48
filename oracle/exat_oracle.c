/*
 * exat_oracle.c -- CPU oracle for the multi-replica tensor compression step.
 *
 * THIS IS TEST INFRASTRUCTURE, not the product.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or constant generator with the HIP library; the only
 * thing the two sides have in common is the written definition of the
 * operation (paper Sec. 3 "Compression", Eq. 3) and of the synthetic-noise
 * function documented below, each implemented independently.
 *
 * Everything here is deliberately plain: one replica at a time, mode by mode,
 * one scalar fp64 accumulator per output element, no blocking, no fusion.
 * OpenMP is used only to spread independent output elements over cores.
 *
 * Layouts (paper Sec. 4.1: tensors are column-major):
 *   X[i + I*(j + J*k)]            third-order tensor, fp32
 *   U[l*ldU + i]  (L x I)         compression matrices, reduction index contiguous
 *   Y[l + L*(m + M*n)]            one proxy tensor, fp64 here
 *   A[i + I*r]    (I x R)         CP factor matrices of the synthetic input
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the OpenMP loops below will use (1 without OpenMP) */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Eq. 3 written out literally: six nested loops.  Tiny inputs only.   */
/* ------------------------------------------------------------------ */
void orc_comp_brute(const float *X, int64_t I, int64_t J, int64_t K,
                    const float *U, int64_t ldU, int64_t L,
                    const float *V, int64_t ldV, int64_t M,
                    const float *W, int64_t ldW, int64_t N, double *Y)
{
    for (int64_t n = 0; n < N; n++)
        for (int64_t m = 0; m < M; m++)
            for (int64_t l = 0; l < L; l++) {
                double s = 0.0;
                for (int64_t k = 0; k < K; k++)
                    for (int64_t j = 0; j < J; j++)
                        for (int64_t i = 0; i < I; i++)
                            s += (double)U[l * ldU + i] * (double)V[m * ldV + j] *
                                 (double)W[n * ldW + k] * (double)X[i + I * (j + J * k)];
                Y[l + L * (m + M * n)] = s;
            }
}

/* ------------------------------------------------------------------ */
/* One tensor-times-matrix product along `mode` (0,1,2), the building  */
/* block of "compress each dimension respectively" (Sec. 4.3).         */
/* T is d[0] x d[1] x d[2] column-major (fp32 if t_is_f32 else fp64);  */
/* Mat is rows x d[mode]; out has d[mode] replaced by rows, fp64.      */
/* ------------------------------------------------------------------ */
void orc_ttm(const void *T, int t_is_f32, const int64_t *d, int mode,
             const float *Mat, int64_t ld, int64_t rows, double *out)
{
    const int64_t s[3] = {1, d[0], d[0] * d[1]};
    int64_t od[3] = {d[0], d[1], d[2]};
    od[mode] = rows;
    const int64_t os[3] = {1, od[0], od[0] * od[1]};
    const int64_t ext = d[mode], st = s[mode];
    const float *Tf = (const float *)T;
    const double *Td = (const double *)T;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t a2 = 0; a2 < od[2]; a2++)
        for (int64_t a1 = 0; a1 < od[1]; a1++)
            for (int64_t a0 = 0; a0 < od[0]; a0++) {
                int64_t a[3] = {a0, a1, a2};
                const int64_t r = a[mode];
                a[mode] = 0;
                const int64_t base = a[0] * s[0] + a[1] * s[1] + a[2] * s[2];
                const float *row = Mat + r * ld;
                double acc = 0.0;
                if (t_is_f32)
                    for (int64_t t = 0; t < ext; t++) acc += (double)row[t] * (double)Tf[base + t * st];
                else
                    for (int64_t t = 0; t < ext; t++) acc += (double)row[t] * Td[base + t * st];
                out[a0 * os[0] + a1 * os[1] + a2 * os[2]] = acc;
            }
}

/* ------------------------------------------------------------------ */
/* Y = Comp(X, U, V, W) (Eq. 3) as three successive orc_ttm calls in   */
/* the order order[0], order[1], order[2] (a permutation of 0,1,2);    */
/* the paper's order is 0,1,2.  Returns 0, or -1 if out of memory.     */
/* ------------------------------------------------------------------ */
int orc_comp(const float *X, int64_t I, int64_t J, int64_t K,
             const float *U, int64_t ldU, int64_t L,
             const float *V, int64_t ldV, int64_t M,
             const float *W, int64_t ldW, int64_t N,
             const int *order, double *Y)
{
    const float *mats[3] = {U, V, W};
    const int64_t lds[3] = {ldU, ldV, ldW};
    const int64_t rows[3] = {L, M, N};
    int64_t d[3] = {I, J, K};
    const void *cur = X;
    int cur_f32 = 1;
    double *owned = NULL;
    for (int s = 0; s < 3; s++) {
        const int mode = order[s];
        int64_t od[3] = {d[0], d[1], d[2]};
        od[mode] = rows[mode];
        double *out = (s == 2) ? Y : (double *)malloc(sizeof(double) * (size_t)(od[0] * od[1] * od[2]));
        if (!out) { free(owned); return -1; }
        orc_ttm(cur, cur_f32, d, mode, mats[mode], lds[mode], rows[mode], out);
        free(owned);
        owned = (s == 2) ? NULL : out;
        cur = out;
        cur_f32 = 0;
        d[mode] = rows[mode];
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Closed form for an exactly rank-R input X = sum_r a_r o b_r o c_r   */
/* (Eq. 1): Comp(X,U,V,W) = sum_r (U a_r) o (V b_r) o (W c_r), which    */
/* is the identity A_p = U_p A behind the decomposition stage (Sec. 3). */
/* ------------------------------------------------------------------ */
int orc_closed_form(const float *A, const float *B, const float *C,
                    int64_t I, int64_t J, int64_t K, int64_t R,
                    const float *U, int64_t ldU, int64_t L,
                    const float *V, int64_t ldV, int64_t M,
                    const float *W, int64_t ldW, int64_t N, double *Y)
{
    double *UA = (double *)malloc(sizeof(double) * (size_t)(L * R));
    double *VB = (double *)malloc(sizeof(double) * (size_t)(M * R));
    double *WC = (double *)malloc(sizeof(double) * (size_t)(N * R));
    if (!UA || !VB || !WC) { free(UA); free(VB); free(WC); return -1; }
    for (int64_t r = 0; r < R; r++) {
        for (int64_t l = 0; l < L; l++) {
            double s = 0.0;
            for (int64_t i = 0; i < I; i++) s += (double)U[l * ldU + i] * (double)A[i + I * r];
            UA[l + L * r] = s;
        }
        for (int64_t m = 0; m < M; m++) {
            double s = 0.0;
            for (int64_t j = 0; j < J; j++) s += (double)V[m * ldV + j] * (double)B[j + J * r];
            VB[m + M * r] = s;
        }
        for (int64_t n = 0; n < N; n++) {
            double s = 0.0;
            for (int64_t k = 0; k < K; k++) s += (double)W[n * ldW + k] * (double)C[k + K * r];
            WC[n + N * r] = s;
        }
    }
    for (int64_t n = 0; n < N; n++)
        for (int64_t m = 0; m < M; m++)
            for (int64_t l = 0; l < L; l++) {
                double s = 0.0;
                for (int64_t r = 0; r < R; r++) s += UA[l + L * r] * VB[m + M * r] * WC[n + N * r];
                Y[l + L * (m + M * n)] = s;
            }
    free(UA); free(VB); free(WC);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Synthetic noise g(seed; i,j,k): a counter-based standard normal.    */
/* The paper's synthetic tensors are exactly low rank (Sec. 5.1); the  */
/* additive noise and its generator are this project's definition:     */
/*                                                                     */
/*  mixA(x): x^=x>>16; x*=0x7feb352d; x^=x>>15; x*=0x846ca68b; x^=x>>16 */
/*  mixB(x): x^=x>>16; x*=0x21f0aaad; x^=x>>15; x*=0x735a2d97; x^=x>>15 */
/*  s    = mixA(mixA(lo32(seed) ^ 0x243f6a88) ^ hi32(seed))             */
/*  ck   = mixA(mixA(s ^ k) ^ j)                 (key of fibre (:,j,k)) */
/*  x    = ck ^ (i >> 2)                          (four i share a draw) */
/*  w    = (i & 2) ? mixB(x) : mixA(x)            (two i share a word)  */
/*  u1   = ((w >> 16) + 0.5) / 65536,  u2 = ((w & 0xffff) + 0.5)/65536  */
/*  g    = sqrt(-2 ln u1) * ((i & 1) ? sin(2 pi u2) : cos(2 pi u2))     */
/*                                                                     */
/* (Box-Muller on 16-bit uniforms; all integer arithmetic mod 2^32.)   */
/* It depends on the global coordinates only, never on the tiling.     */
/* Requires 0 <= i,j,k < 2^31.                                          */
/* mixA / mixB use two published public-domain constant sets of the     */
/* multiply-xorshift hash family ("lowbias32" and a second result of    */
/* the same hash-prospector search); 0x243f6a88 = fractional bits of pi.*/
/* ------------------------------------------------------------------ */
static inline uint32_t mixA(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
static inline uint32_t mixB(uint32_t x)
{
    x ^= x >> 16; x *= 0x21f0aaadu; x ^= x >> 15; x *= 0x735a2d97u; x ^= x >> 15;
    return x;
}
uint32_t orc_noise_word(uint64_t seed, int64_t i, int64_t j, int64_t k)
{
    const uint32_t s = mixA(mixA((uint32_t)seed ^ 0x243f6a88u) ^ (uint32_t)(seed >> 32));
    const uint32_t ck = mixA(mixA(s ^ (uint32_t)k) ^ (uint32_t)j);
    const uint32_t x = ck ^ (uint32_t)(i >> 2);
    return (i & 2) ? mixB(x) : mixA(x);
}
double orc_noise(uint64_t seed, int64_t i, int64_t j, int64_t k)
{
    const uint32_t w = orc_noise_word(seed, i, j, k);
    const double u1 = ((double)(w >> 16) + 0.5) / 65536.0;
    const double u2 = ((double)(w & 0xffffu) + 0.5) / 65536.0;
    const double rad = sqrt(-2.0 * log(u1));
    const double ang = 6.283185307179586476925286766559 * u2;
    return rad * ((i & 1) ? sin(ang) : cos(ang));
}
void orc_noise_box(uint64_t seed, int64_t i0, int64_t i1, int64_t j0, int64_t j1,
                   int64_t k0, int64_t k1, double *out)
{
    const int64_t di = i1 - i0, dj = j1 - j0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t k = k0; k < k1; k++)
        for (int64_t j = j0; j < j1; j++)
            for (int64_t i = i0; i < i1; i++)
                out[(i - i0) + di * ((j - j0) + dj * (k - k0))] = orc_noise(seed, i, j, k);
}

/* round-to-nearest-even fp32 -> bf16, returned as the fp32 it represents */
float orc_round_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&v, &u, 4);
    return v;
}
void orc_round_bf16_array(const float *in, float *out, int64_t n)
{
    for (int64_t t = 0; t < n; t++) out[t] = orc_round_bf16(in[t]);
}

/* ------------------------------------------------------------------ */
/* Synthetic input of the dense experiments (Sec. 5.1, Eq. 1) plus the */
/* project's noise term, on the half-open box [i0,i1)x[j0,j1)x[k0,k1): */
/*   X[i,j,k] = fl32( sum_r A[i,r] B[j,r] C[k,r] + sigma*g(seed;i,j,k) )*/
/* evaluated in fp64 and rounded once to fp32 (then, if to_bf16, once   */
/* more to bf16 by round-to-nearest-even).  out is column-major on the  */
/* box.  A,B,C are column-major I x R, J x R, K x R.                    */
/* ------------------------------------------------------------------ */
void orc_gen_box(const float *A, const float *B, const float *C,
                 int64_t I, int64_t J, int64_t K, int64_t R,
                 uint64_t seed, double sigma,
                 int64_t i0, int64_t i1, int64_t j0, int64_t j1, int64_t k0, int64_t k1,
                 int to_bf16, float *out)
{
    const int64_t di = i1 - i0, dj = j1 - j0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t k = k0; k < k1; k++)
        for (int64_t j = j0; j < j1; j++)
            for (int64_t i = i0; i < i1; i++) {
                double s = 0.0;
                for (int64_t r = 0; r < R; r++)
                    s += (double)A[i + I * r] * (double)B[j + J * r] * (double)C[k + K * r];
                if (sigma != 0.0) s += sigma * orc_noise(seed, i, j, k);
                float v = (float)s;
                if (to_bf16) v = orc_round_bf16(v);
                out[(i - i0) + di * ((j - j0) + dj * (k - k0))] = v;
            }
}
