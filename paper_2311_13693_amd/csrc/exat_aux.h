// Small kernels around the fused mode-1/2 kernel: operand packing (stacking, padding,
// bf16 rounding), the mode-3 contraction, the block merge and the stand-alone block generator.
#pragma once
#include "exat_device.h"

namespace exat {

// round a value through the plan's element type (identity for fp32)
template <typename T> __device__ __forceinline__ float round_through(float v) { return (float)elem<T>::from_f32(v); }

// Stacked fp32 matrix (rows x cols, leading dimension ld) -> zero-padded [rowspad][colspad] of T.
template <typename T>
__global__ void k_pack_u(const float *src, int64_t ld, int rows, int64_t cols, T *dst, int rowspad, int64_t colspad)
{
    const int64_t n = (int64_t)rowspad * colspad;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / colspad, c = idx % colspad;
        const float v = (r < rows && c < cols) ? src[r * ld + c] : 0.0f;
        dst[idx] = elem<T>::from_f32(v);
    }
}

// Stacked fp32 V (P*M x J) -> fp32 [P][Mpad][Jpad], zero padded, values rounded through T.
template <typename T>
__global__ void k_pack_v(const float *src, int64_t ld, int P, int M, int64_t J, float *dst, int Mpad, int64_t Jpad)
{
    const int64_t n = (int64_t)P * Mpad * Jpad;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = idx % Jpad, pm = idx / Jpad;
        const int m = (int)(pm % Mpad), pr = (int)(pm / Mpad);
        const float v = (m < M && j < J) ? src[((int64_t)pr * M + m) * ld + j] : 0.0f;
        dst[idx] = round_through<T>(v);
    }
}

// Stacked fp32 W (P*N x K) -> dense fp32 [P*N][K], values rounded through T.
template <typename T>
__global__ void k_pack_w(const float *src, int64_t ld, int rows, int64_t K, float *dst)
{
    const int64_t n = (int64_t)rows * K;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / K, c = idx % K;
        dst[idx] = round_through<T>(src[r * ld + c]);
    }
}

// Mode 3: Y[p,l,m,n] (=|+=) sum_{k in [k0,k1)} W_p[n,k] Q[k-k0][p*L+l][m], accumulated in fp64
// in ascending k.  One thread per (q, m) position and NT consecutive n.
struct Mode3Params {
    const float *Q;  // [nk][PLpad][Mpad]
    const float *W;  // [P*N][K]
    float *Y;        // [P][N][M][L] i.e. Y[l + L*(m + M*(n + N*p))]
    int L, M, N, PL, PLpad, Mpad;
    int64_t K, k0, k1;
    int accumulate;
};

template <int NT>
__global__ __launch_bounds__(256) void k_mode3(const Mode3Params p)
{
    const int64_t pos = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int q = (int)(pos / p.Mpad), m = (int)(pos % p.Mpad);
    if (q >= p.PL || m >= p.M) return;
    const int pr = q / p.L, l = q % p.L;
    const int n0 = blockIdx.y * NT;
    const float *wrow[NT];
#pragma unroll
    for (int n = 0; n < NT; n++) {
        const int nn = (n0 + n < p.N) ? n0 + n : p.N - 1;
        wrow[n] = p.W + ((int64_t)pr * p.N + nn) * p.K + p.k0;
    }
    double acc[NT];
#pragma unroll
    for (int n = 0; n < NT; n++) acc[n] = 0.0;
    const int64_t nk = p.k1 - p.k0, qs = (int64_t)p.PLpad * p.Mpad;
    const float *qp = p.Q + (int64_t)q * p.Mpad + m;
    for (int64_t kk = 0; kk < nk; kk++) {
        const double qv = (double)qp[kk * qs];
#pragma unroll
        for (int n = 0; n < NT; n++) acc[n] = __builtin_fma((double)wrow[n][kk], qv, acc[n]);
    }
#pragma unroll
    for (int n = 0; n < NT; n++) {
        if (n0 + n < p.N) {
            float *dst = p.Y + l + (int64_t)p.L * (m + (int64_t)p.M * (n0 + n + (int64_t)p.N * pr));
            const float v = (float)acc[n];
            *dst = p.accumulate ? *dst + v : v;
        }
    }
}

// Block merge (Fig. 2a): Y = sum over partial slots in ascending slot order (fp64 running sum).
__global__ void k_merge(const float *slots, const unsigned char *used, int nslots, int64_t n, float *Y)
{
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        double s = 0.0;
        for (int t = 0; t < nslots; t++)
            if (used[t]) s += (double)slots[(int64_t)t * n + idx];
        Y[idx] = (float)s;
    }
}

// Stand-alone generator of one box of the synthetic tensor, column-major on the box.
struct GenParams {
    const float *A, *B, *C;
    int64_t ldA, ldB, ldC;
    int R;
    uint32_t skey;
    float amp2_ln2;
    int64_t i0, i1, j0, j1, k0, k1;
};

template <typename T>
__global__ __launch_bounds__(256) void k_gen_box(const GenParams p, T *out)
{
    const int64_t q0 = p.i0 >> 2, nq = ((p.i1 - 1) >> 2) - q0 + 1;
    const int64_t di = p.i1 - p.i0, dj = p.j1 - p.j0, dk = p.k1 - p.k0;
    const int64_t n = nq * dj * dk;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t iq = q0 + idx % nq, jk = idx / nq;
        const int64_t j = p.j0 + jk % dj, k = p.k0 + jk / dj;
        float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int r = 0; r < p.R; r++) {
            const float bc = p.B[j + p.ldB * r] * p.C[k + p.ldC * r];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int64_t i = 4 * iq + e;
                if (i >= p.i0 && i < p.i1) x[e] = __builtin_fmaf(p.A[i + p.ldA * r], bc, x[e]);
            }
        }
        if (p.amp2_ln2 != 0.0f) {
            float z[4];
            noise_quad(fibre_key(p.skey, (uint32_t)j, (uint32_t)k), (uint32_t)iq, p.amp2_ln2, z);
#pragma unroll
            for (int e = 0; e < 4; e++) x[e] += z[e];
        }
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int64_t i = 4 * iq + e;
            if (i >= p.i0 && i < p.i1) out[(i - p.i0) + di * ((j - p.j0) + dj * (k - p.k0))] = elem<T>::from_f32(x[e]);
        }
    }
}

}  // namespace exat
