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

// Stacked fp32 W (P*N x K) -> transposed fp32 [P][K][Npad] (n contiguous, zero padded), values
// rounded through T: the layout the mode-3 MFMA reads its B operand from with coalesced loads.
template <typename T>
__global__ void k_pack_w(const float *src, int64_t ld, int P, int N, int64_t K, float *dst, int Npad)
{
    const int64_t n_all = (int64_t)P * K * Npad;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n_all; idx += (int64_t)gridDim.x * blockDim.x) {
        const int n = (int)(idx % Npad);
        const int64_t pk = idx / Npad, k = pk % K, pr = pk / K;
        const float v = (n < N) ? src[(pr * N + n) * ld + k] : 0.0f;
        dst[idx] = round_through<T>(v);
    }
}

// Mode 3: Y[p,l,m,n] (=|+=) sum_{k in [k0,k1)} W_p[n,k] Q[k-k0][p*L+l][m].
// One wave owns 32 consecutive (q, m) positions of one stacked row q (so one replica) and up
// to 64 values of n; it runs fp32 MFMAs over k in ascending order, flushing the fp32 partial
// sums into fp64 totals every KFLUSH values of k so that the summation error does not grow
// with the extent of K.
struct Mode3Params {
    const float *Q;  // [nk][PLpad][Mpad]
    const float *W;  // [P][K][Npad]
    float *Y;        // Y[l + L*(m + M*(n + N*p))]
    int L, M, N, PL, PLpad, Mpad, Npad;
    int64_t K, k0, k1;
    int accumulate;
    unsigned char *flag;  // if not null, set to 1 by the launch (block streaming: "this slot holds a partial result")
};

// One workgroup per 32 (q, m) positions x <= 64 columns n; its M3_WAVES waves split the k range into contiguous
// slabs (the outputs are few and the k range long, so k is where the parallelism is) and wave 0 adds the partial
// sums in wave order, which keeps the result independent of timing.
constexpr int M3_WAVES = 4;

// NT = 32-column tiles of n per workgroup (1 or 2).  LONGK: a wave's slab of k may exceed KFLUSH values, so the
// fp32 MFMA accumulators are flushed into fp64 sums every KFLUSH values; without it the accumulators themselves
// are the slab's result and no fp64 registers are alive during the loop.
template <int NT, bool LONGK>
__global__ __launch_bounds__(64 * M3_WAVES, LONGK ? 1 : 2) void k_mode3(const Mode3Params p)
{
    constexpr int KFLUSH = 512;
    __shared__ float part[M3_WAVES - 1][NT][16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, hi = lane >> 5;
    if (p.flag != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *p.flag = 1;
    const int64_t pos0 = (int64_t)blockIdx.x * 32;
    if (pos0 >= (int64_t)p.PL * p.Mpad) return;  // whole workgroup
    const int q = (int)(pos0 / p.Mpad), m0 = (int)(pos0 % p.Mpad);
    if (m0 >= p.M) return;                       // a tile made of padding columns only (whole workgroup)
    const int pr = q / p.L, l = q % p.L;
    const int n0 = blockIdx.y * 32 * NT;
    const int64_t nkall = p.k1 - p.k0, qs = (int64_t)p.PLpad * p.Mpad;
    const int64_t slab = (((nkall + M3_WAVES - 1) / M3_WAVES) + 1) & ~(int64_t)1;  // even: lanes 32..63 take odd k
    const int64_t kbeg = wave * slab;
    const int64_t nk = (kbeg >= nkall) ? 0 : ((kbeg + slab < nkall) ? slab : nkall - kbeg);
    const float *qp = p.Q + kbeg * qs + pos0 + l32;                                    // + kk*qs
    const float *wp = p.W + ((int64_t)pr * p.K + p.k0 + kbeg) * p.Npad + n0 + l32;     // + kk*Npad (+32 for tile 1)
    double totl[LONGK ? NT : 1][16];   // LONGK only
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
            acc[t][e] = 0.0f;
            if (LONGK) totl[t][e] = 0.0;
        }
    for (int64_t kc = 0; kc < nk; kc += LONGK ? KFLUSH : nk) {
        const int64_t kend = (LONGK && kc + KFLUSH < nk) ? kc + KFLUSH : nk;
        // 16 values of k per batch, two register sets: the loads of the next batch are issued before the MFMAs
        // of the current one (the kernel runs at well under one wave per SIMD, so nothing else hides the latency)
        constexpr int KB = 16, NS = KB / 2;
        float a0[NS], b00[NS], b10[NS], a1[NS], b01[NS], b11[NS];  // b1* unused when NT == 1
        auto load_batch = [&](float *a, float *b0, float *b1, int64_t kk) {
#pragma unroll
            for (int t = 0; t < NS; t++) {
                const int64_t kx = kk + 2 * t + hi;
                const bool ok = kx < kend;
                a[t] = ok ? qp[kx * qs] : 0.0f;
                b0[t] = ok ? wp[kx * p.Npad] : 0.0f;
                if (NT == 2) b1[t] = ok ? wp[kx * p.Npad + 32] : 0.0f;
            }
        };
        auto mma_batch = [&](const float *a, const float *b0, const float *b1) {
#pragma unroll
            for (int t = 0; t < NS; t++) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b0[t], acc[0], 0, 0, 0);
                if (NT == 2) acc[NT - 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b1[t], acc[1], 0, 0, 0);
            }
        };
        load_batch(a0, b00, b10, kc);
        for (int64_t kk = kc; kk < kend; kk += 2 * KB) {
            load_batch(a1, b01, b11, kk + KB);       // zeros beyond kend
            __builtin_amdgcn_sched_barrier(0);
            mma_batch(a0, b00, b10);
            load_batch(a0, b00, b10, kk + 2 * KB);
            __builtin_amdgcn_sched_barrier(0);
            mma_batch(a1, b01, b11);
        }
        if (LONGK) {
#pragma unroll
            for (int t = 0; t < NT; t++)
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    totl[t][e] += (double)acc[t][e];
                    acc[t][e] = 0.0f;
                }
        }
    }
    double tot[NT][16];
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) tot[t][e] = LONGK ? totl[t][e] : (double)acc[t][e];
    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int e = 0; e < 16; e++) part[wave - 1][t][e][lane] = (float)tot[t][e];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < M3_WAVES - 1; w++)
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int e = 0; e < 16; e++) tot[t][e] += (double)part[w][t][e][lane];
    // C layout: element 4b+r of the accumulator is row (position) 8b + 4*hi + r, column n = l32
#pragma unroll
    for (int t = 0; t < NT; t++) {
        const int n = n0 + 32 * t + l32;
        if (n < p.N) {
#pragma unroll
            for (int b4 = 0; b4 < 4; b4++)
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int m = m0 + 8 * b4 + 4 * hi + r;
                    if (m < p.M) {
                        float *dst = p.Y + l + (int64_t)p.L * (m + (int64_t)p.M * (n + (int64_t)p.N * pr));
                        const float v = (float)tot[t][4 * b4 + r];
                        *dst = p.accumulate ? *dst + v : v;
                    }
                }
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
