// Batched CP-ALS on the P proxy tensors (paper Alg. 1; Sec. 3 "Decomposition").  Declarations and contracts in
// include/exat.h.
//
// The P problems are independent and small (L, M, N, R <= 64), so one workgroup owns one replica for all sweeps
// and everything but the tensor itself lives in LDS: the three factor matrices, the R x R normal matrix and the
// MTTKRP result.  One update, e.g. of A:
//   MTTKRP  Mx[l,r] = sum_n C[n,r] * (sum_m Y[l,m,n] * B[m,r])       lanes along l, a quarter of the r per wave
//   Gram    G = (C^T C) * (B^T B)                                    Hadamard product of the two Gram matrices
//   solve   A = Mx G^{-1} by Cholesky (G = L L^T in LDS) and one forward/backward substitution per row of Mx
// The tensor is read from three copies, one per mode, each with the updated mode's index contiguous, so that
// every MTTKRP reads coalesced.  fp32 throughout; every sum has a fixed order.
#include "../../include/exat.h"

#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr int CP_MAX = 64;   // largest L, M, N and R

struct CpParams {
    const float *Y1, *Y2, *Y3;   // per replica D0*D1*D2 floats: [l + L(m + Mn)], [m + M(l + Ln)], [n + N(l + Lm)]
    float *A, *B, *C;            // per replica column-major L x R, M x R, N x R
    int L, M, N, R, sweeps;
};

// Y2[m + M(l + Ln)] and Y3[n + N(l + Lm)] from Y[l + L(m + Mn)], all replicas
__global__ __launch_bounds__(256) void k_cpals_permute(const float *Y, float *Y2, float *Y3, int L, int M, int N, int64_t total)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int64_t lmn = (int64_t)L * M * N, p = t / lmn, e = t % lmn;
    const int l = (int)(e % L), m = (int)((e / L) % M), n = (int)(e / ((int64_t)L * M));
    const float y = Y[t];
    Y2[p * lmn + m + (int64_t)M * (l + (int64_t)L * n)] = y;
    Y3[p * lmn + n + (int64_t)N * (l + (int64_t)L * m)] = y;
}

// RW = columns r per wave (R <= 4*RW); factor rows in LDS are RS = 4*RW floats long, zero beyond R
template <int RW>
__global__ __launch_bounds__(256) void k_cpals(const CpParams p)
{
    constexpr int RS = 4 * RW;
    extern __shared__ float smem[];
    float *FA = smem, *FB = FA + CP_MAX * RS, *FC = FB + CP_MAX * RS;   // factors, [d][RS]
    float *G = FC + CP_MAX * RS;                                         // [R][R+1]: normal matrix, then its Cholesky factor
    float *Mx = G + CP_MAX * (CP_MAX + 1);                               // [64][R+1]: MTTKRP result, then the solution
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int R = p.R, GS = R + 1;
    const int64_t rep = blockIdx.x;
    const int64_t lmn = (int64_t)p.L * p.M * p.N;

    // start values: column-major in memory, [d][RS] in LDS
    auto load_factor = [&](float *F, const float *src, int D) {
        for (int e = tid; e < CP_MAX * RS; e += 256) {
            const int d = e / RS, r = e % RS;
            F[e] = (d < D && r < R) ? src[d + (int64_t)D * r] : 0.0f;
        }
    };
    load_factor(FA, p.A + rep * p.L * R, p.L);
    load_factor(FB, p.B + rep * p.M * R, p.M);
    load_factor(FC, p.C + rep * p.N * R, p.N);
    __syncthreads();

    // F0 (D0 x R) <- least-squares update from the tensor copy Yp[d0 + D0(d1 + D1 d2)] and the factors F1, F2
    auto update = [&](float *F0, const float *Yp, const float *F1, const float *F2, int D0, int D1, int D2) {
        // MTTKRP
        float acc[RW];
#pragma unroll
        for (int x = 0; x < RW; x++) acc[x] = 0.0f;
        const int r0 = w * RW;
        const bool on = lane < D0;
        const float *yl = Yp + (on ? lane : 0);
        for (int d2 = 0; d2 < D2; d2++) {
            float s[RW];
#pragma unroll
            for (int x = 0; x < RW; x++) s[x] = 0.0f;
            const float *yd = yl + (int64_t)D0 * D1 * d2;
            int d1 = 0;
            for (; d1 + 4 <= D1; d1 += 4) {   // four loads in flight
                const float y0 = yd[(int64_t)D0 * d1], y1 = yd[(int64_t)D0 * (d1 + 1)];
                const float y2 = yd[(int64_t)D0 * (d1 + 2)], y3 = yd[(int64_t)D0 * (d1 + 3)];
#pragma unroll
                for (int x = 0; x < RW; x++) {
                    s[x] = fmaf(y0, F1[d1 * RS + r0 + x], s[x]);
                    s[x] = fmaf(y1, F1[(d1 + 1) * RS + r0 + x], s[x]);
                    s[x] = fmaf(y2, F1[(d1 + 2) * RS + r0 + x], s[x]);
                    s[x] = fmaf(y3, F1[(d1 + 3) * RS + r0 + x], s[x]);
                }
            }
            for (; d1 < D1; d1++) {
                const float y0 = yd[(int64_t)D0 * d1];
#pragma unroll
                for (int x = 0; x < RW; x++) s[x] = fmaf(y0, F1[d1 * RS + r0 + x], s[x]);
            }
#pragma unroll
            for (int x = 0; x < RW; x++) acc[x] = fmaf(s[x], F2[d2 * RS + r0 + x], acc[x]);
        }
        if (on) {
#pragma unroll
            for (int x = 0; x < RW; x++)
                if (r0 + x < R) Mx[lane * GS + r0 + x] = acc[x];
        }
        // normal matrix G = (F2^T F2) * (F1^T F1)
        for (int e = tid; e < R * R; e += 256) {
            const int r = e / R, c = e % R;
            float g1 = 0.0f, g2 = 0.0f;
            for (int d = 0; d < D1; d++) g1 = fmaf(F1[d * RS + r], F1[d * RS + c], g1);
            for (int d = 0; d < D2; d++) g2 = fmaf(F2[d * RS + r], F2[d * RS + c], g2);
            G[r * GS + c] = g1 * g2;
        }
        __syncthreads();
        // Cholesky factor in the lower triangle of G, right-looking: per column, scale it, then every thread
        // updates its share of the trailing triangle (two barriers per column, no serial sums)
        for (int j = 0; j < R; j++) {
            const float inv = 1.0f / sqrtf(G[j * GS + j]);
            __syncthreads();   // everyone has read the pivot
            for (int t = j + tid; t < R; t += 256) G[t * GS + j] *= inv;   // t = j: the pivot becomes its square root
            __syncthreads();
            const int n = R - 1 - j;   // trailing triangle: rows t > j, columns j < c <= t
            for (int e = tid; e < n * n; e += 256) {
                const int t = j + 1 + e / n, c = j + 1 + e % n;
                if (c <= t) G[t * GS + c] = fmaf(-G[t * GS + j], G[c * GS + j], G[t * GS + c]);
            }
            __syncthreads();
        }
        // one row of Mx per thread, held in registers: L z = m, then L^T o = z.  The loops are unrolled to the
        // instantiation's largest rank, so the row is indexed statically and the reads of the factor (the same
        // address for every thread) do not depend on the data.
        if (tid < D0) {
            float m[RS];
#pragma unroll
            for (int i = 0; i < RS; i++) m[i] = i < R ? Mx[tid * GS + i] : 0.0f;
#pragma unroll
            for (int i = 0; i < RS; i++) {
                if (i < R) {
                    float v = m[i];
#pragma unroll
                    for (int k = 0; k < i; k++) v = fmaf(-G[i * GS + k], m[k], v);
                    m[i] = v / G[i * GS + i];
                }
            }
#pragma unroll
            for (int i = RS - 1; i >= 0; i--) {
                if (i < R) {
                    float v = m[i];
#pragma unroll
                    for (int k = i + 1; k < RS; k++)
                        if (k < R) v = fmaf(-G[k * GS + i], m[k], v);
                    m[i] = v / G[i * GS + i];
                }
            }
#pragma unroll
            for (int r = 0; r < RS; r++)
                if (r < R) F0[tid * RS + r] = m[r];
        }
        __syncthreads();
    };

    const float *Y1 = p.Y1 + rep * lmn, *Y2 = p.Y2 + rep * lmn, *Y3 = p.Y3 + rep * lmn;
    for (int t = 0; t < p.sweeps; t++) {
        update(FA, Y1, FB, FC, p.L, p.M, p.N);   // A <- Y_(1) (C kr B) [(C^T C) * (B^T B)]^-1
        update(FB, Y2, FA, FC, p.M, p.L, p.N);   // B <- Y_(2) (C kr A) [(C^T C) * (A^T A)]^-1
        update(FC, Y3, FA, FB, p.N, p.L, p.M);   // C <- Y_(3) (B kr A) [(B^T B) * (A^T A)]^-1
    }
    auto store_factor = [&](const float *F, float *dst, int D) {
        for (int e = tid; e < D * R; e += 256) {
            const int d = e % D, r = e / D;
            dst[d + (int64_t)D * r] = F[d * RS + r];
        }
    };
    store_factor(FA, p.A + rep * p.L * R, p.L);
    store_factor(FB, p.B + rep * p.M * R, p.M);
    store_factor(FC, p.C + rep * p.N * R, p.N);
}

template <int RW>
int launch_cpals(const CpParams &p, int P, hipStream_t st)
{
    const size_t lds = (size_t)(3 * CP_MAX * 4 * RW + 2 * CP_MAX * (CP_MAX + 1)) * sizeof(float);
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_cpals<RW>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return EXAT_ERR_HIP;
    hipLaunchKernelGGL(k_cpals<RW>, dim3((unsigned)P), dim3(256), lds, st, p);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

}  // namespace

extern "C" {

int64_t exat_cpals_workspace_floats(int32_t L, int32_t M, int32_t N, int32_t P)
{
    if (L < 1 || M < 1 || N < 1 || P < 1) return 0;
    return 2 * (int64_t)L * M * N * P;
}

int exat_cpals(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps, float *A, float *B,
               float *C, float *work, void *stream)
{
    if (!Y || !A || !B || !C || !work) return EXAT_ERR_NULL;
    if (L < 1 || M < 1 || N < 1 || R < 1 || P < 1 || sweeps < 0) return EXAT_ERR_SHAPE;
    if (L > CP_MAX || M > CP_MAX || N > CP_MAX || R > CP_MAX || P > (1 << 20)) return EXAT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = (int64_t)L * M * N * P;
    float *Y2 = work, *Y3 = work + total;
    hipLaunchKernelGGL(k_cpals_permute, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, Y, Y2, Y3, L, M, N, total);
    if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    CpParams p;
    p.Y1 = Y; p.Y2 = Y2; p.Y3 = Y3; p.A = A; p.B = B; p.C = C;
    p.L = L; p.M = M; p.N = N; p.R = R; p.sweeps = sweeps;
    if (R <= 16) return launch_cpals<4>(p, P, st);
    if (R <= 32) return launch_cpals<8>(p, P, st);
    return launch_cpals<16>(p, P, st);
}

}  // extern "C"
