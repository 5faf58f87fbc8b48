// Batched CP-ALS on the P proxy tensors (paper Alg. 1; Sec. 3 "Decomposition").  Declarations and contracts in
// include/exat.h.
//
// The P problems are independent and small (L, M, N, R <= 64).  One update, e.g. of A, is two launches:
//   k_cpals_mttkrp  Mx[l,r] = sum_n C[n,r] * (sum_m Y[l,m,n] * B[m,r]): the n range of every replica is cut into
//                   slabs, one workgroup per (replica, slab), so that the P small problems fill the chip; lanes
//                   along l, a quarter of the r per wave, the two factor matrices in LDS.  Partial results per slab.
//   k_cpals_solve   one workgroup per replica: adds the slabs' partial results in slab order, forms the normal
//                   matrix G = (C^T C) * (B^T B) (Hadamard product of the Gram matrices), factors it (Cholesky,
//                   right-looking, in LDS) and solves A = Mx G^{-1}, one row of Mx per thread.
// The tensor is read from three copies, one per mode, each with the updated mode's index contiguous, so that
// every MTTKRP reads coalesced.  fp32 throughout; every sum has a fixed order.
#include "../../include/exat.h"

#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr int CP_MAX = 64;   // largest L, M, N and R

struct CpUpdate {
    const float *Yp;        // the copy of Y with the updated mode contiguous: per replica [d0 + D0(d1 + D1 d2)]
    const float *F1, *F2;   // the two fixed factors, per replica column-major D1 x R, D2 x R
    float *F0;              // the updated factor, per replica column-major D0 x R
    float *part;            // [replica][slab][d0][R] partial MTTKRP results
    int D0, D1, D2, R, NS, DS;   // NS slabs of DS values of d2
    int32_t *status;        // optional, [replica]: incremented by every update whose normal matrix has a non-positive pivot
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

// column-major D x R in memory -> [d][RS] in LDS, zero beyond D and R
template <int RS>
__device__ inline void load_factor(float *F, const float *src, int D, int R, int tid)
{
    for (int e = tid; e < CP_MAX * RS; e += 256) F[e] = 0.0f;
    __syncthreads();
    for (int e = tid; e < D * R; e += 256) F[(e % D) * RS + e / D] = src[e];
}

// RW = columns r per wave (R <= 4*RW); factor rows in LDS are RS = 4*RW floats long
template <int RW>
__global__ __launch_bounds__(256) void k_cpals_mttkrp(const CpUpdate p)
{
    constexpr int RS = 4 * RW;
    __shared__ float F1[CP_MAX * RS], F2[CP_MAX * RS];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t rep = blockIdx.x;
    const int slab = blockIdx.y, D0 = p.D0, D1 = p.D1, R = p.R;
    load_factor<RS>(F1, p.F1 + rep * D1 * R, D1, R, tid);
    load_factor<RS>(F2, p.F2 + rep * p.D2 * R, p.D2, R, tid);
    __syncthreads();
    float acc[RW];
#pragma unroll
    for (int x = 0; x < RW; x++) acc[x] = 0.0f;
    const int r0 = w * RW;
    const bool on = lane < D0;
    const float *yl = p.Yp + rep * D0 * D1 * p.D2 + (on ? lane : 0);
    const int d2a = slab * p.DS, d2b = (d2a + p.DS < p.D2) ? d2a + p.DS : p.D2;
    for (int d2 = d2a; d2 < d2b; d2++) {
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
        float *dst = p.part + ((rep * p.NS + slab) * D0 + lane) * R;
#pragma unroll
        for (int x = 0; x < RW; x++)
            if (r0 + x < R) dst[r0 + x] = acc[x];
    }
}

template <int RW>
__global__ __launch_bounds__(256) void k_cpals_solve(const CpUpdate p)
{
    constexpr int RS = 4 * RW;
    __shared__ float F1[CP_MAX * RS], F2[CP_MAX * RS];
    __shared__ float G[RS * (RS + 1)];        // normal matrix, updated in place by the factorisation (row stride R+1)
    __shared__ float Lf[RS * (RS + 1)];       // its Cholesky factor
    __shared__ float Mx[CP_MAX * (RS + 1)];   // MTTKRP result (row stride R+1)
    const int tid = threadIdx.x;
    const int64_t rep = blockIdx.x;
    const int D0 = p.D0, D1 = p.D1, D2 = p.D2, R = p.R, GS = R + 1;
    load_factor<RS>(F1, p.F1 + rep * D1 * R, D1, R, tid);
    load_factor<RS>(F2, p.F2 + rep * D2 * R, D2, R, tid);
    // MTTKRP result: the slabs' partial results in slab order
    for (int e = tid; e < D0 * R; e += 256) {
        const float *src = p.part + rep * p.NS * D0 * R + e;
        const int64_t st = (int64_t)D0 * R;
        float v = 0.0f;
        int sl = 0;
        for (; sl + 32 <= p.NS; sl += 32) {   // 32 loads in flight (a round trip to memory each), added in slab order
            float t[32];
#pragma unroll
            for (int u = 0; u < 32; u++) t[u] = src[(sl + u) * st];
#pragma unroll
            for (int u = 0; u < 32; u++) v += t[u];
        }
        for (; sl + 8 <= p.NS; sl += 8) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; u++) t[u] = src[(sl + u) * st];
#pragma unroll
            for (int u = 0; u < 8; u++) v += t[u];
        }
        for (; sl < p.NS; sl++) v += src[sl * st];
        Mx[(e / R) * GS + e % R] = v;
    }
    __syncthreads();
    // normal matrix G = (F2^T F2) * (F1^T F1)
    for (int e = tid; e < R * R; e += 256) {
        const int r = e / R, c = e % R;
        float g1 = 0.0f, g2 = 0.0f;
        for (int d = 0; d < D1; d++) g1 = fmaf(F1[d * RS + r], F1[d * RS + c], g1);
        for (int d = 0; d < D2; d++) g2 = fmaf(F2[d * RS + r], F2[d * RS + c], g2);
        G[r * GS + c] = g1 * g2;
    }
    __syncthreads();
    // Cholesky factor, right-looking, one barrier per column: every thread scales the entries of column j that it
    // needs by the pivot's inverse square root on the fly for its share of the trailing triangle, and the scaled
    // column goes to a second matrix Lf (nobody reads column j of G again), so reading and scaling do not collide.
    bool bad = false;   // the same in every thread: all read the same pivots
    for (int j = 0; j < R; j++) {
        const float piv = G[j * GS + j];
        bad = bad || !(piv > 0.0f);   // zero, negative or NaN: the normal matrix is not positive definite in fp32
        const float inv = 1.0f / sqrtf(piv);
        for (int t = j + tid; t < R; t += 256) Lf[t * GS + j] = G[t * GS + j] * inv;   // t = j: the pivot's square root
        const int n = R - 1 - j;   // trailing triangle: rows t > j, columns j < c <= t
        for (int e = tid; e < n * n; e += 256) {
            const int t = j + 1 + e / n, c = j + 1 + e % n;
            if (c <= t) G[t * GS + c] = fmaf(-(G[t * GS + j] * inv), G[c * GS + j] * inv, G[t * GS + c]);
        }
        __syncthreads();
    }
    // one row of Mx per thread, held in registers: L z = m, then L^T o = z.  The loops are unrolled to the
    // instantiation's largest rank, so the row is indexed statically and the reads of the factor (the same
    // address for every thread) do not depend on the data.
    if (bad && tid == 0 && p.status) p.status[rep] += 1;   // launches on one stream: nothing else touches this word now
    if (tid < D0) {
        float m[RS];
#pragma unroll
        for (int i = 0; i < RS; i++) m[i] = i < R ? Mx[tid * GS + i] : 0.0f;
#pragma unroll
        for (int i = 0; i < RS; i++) {
            if (i < R) {
                float v = m[i];
#pragma unroll
                for (int k = 0; k < i; k++) v = fmaf(-Lf[i * GS + k], m[k], v);
                m[i] = v / Lf[i * GS + i];
            }
        }
#pragma unroll
        for (int i = RS - 1; i >= 0; i--) {
            if (i < R) {
                float v = m[i];
#pragma unroll
                for (int k = i + 1; k < RS; k++)
                    if (k < R) v = fmaf(-Lf[k * GS + i], m[k], v);
                m[i] = v / Lf[i * GS + i];
            }
        }
        float *dst = p.F0 + rep * D0 * R + tid;   // column-major D0 x R
#pragma unroll
        for (int r = 0; r < RS; r++)
            if (r < R) dst[(int64_t)D0 * r] = m[r];
    }
}

// slabs per replica: enough workgroups for about four per compute unit, at most one slab per value of d2
inline int slabs_for(int D2, int P)
{
    int ns = (1024 + P - 1) / P;
    return ns < 1 ? 1 : (ns > D2 ? D2 : ns);
}

template <int RW>
int launch_update(CpUpdate u, int P, hipStream_t st)
{
    u.NS = slabs_for(u.D2, P);
    u.DS = (u.D2 + u.NS - 1) / u.NS;
    u.NS = (u.D2 + u.DS - 1) / u.DS;
    hipLaunchKernelGGL(k_cpals_mttkrp<RW>, dim3((unsigned)P, (unsigned)u.NS), dim3(256), 0, st, u);
    hipLaunchKernelGGL(k_cpals_solve<RW>, dim3((unsigned)P), dim3(256), 0, st, u);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

}  // namespace

extern "C" {

int64_t exat_cpals_workspace_floats(int32_t L, int32_t M, int32_t N, int32_t P)
{
    if (L < 1 || M < 1 || N < 1 || P < 1) return 0;
    // two permuted copies of Y + the slabs' partial MTTKRP results (at most 64 slabs of 64 x 64 per replica)
    const int maxd = L > M ? (L > N ? L : N) : (M > N ? M : N);
    return 2 * (int64_t)L * M * N * P + (int64_t)P * slabs_for(maxd, P) * CP_MAX * CP_MAX;
}

__global__ void k_cpals_clear_status(int32_t *status, int P)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < P) status[t] = 0;
}

int exat_cpals(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps, float *A, float *B,
               float *C, float *work, void *stream)
{
    return exat_cpals_checked(Y, L, M, N, P, R, sweeps, A, B, C, work, nullptr, stream);
}

int exat_cpals_checked(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps, float *A, float *B,
                       float *C, float *work, int32_t *status, void *stream)
{
    if (!Y || !A || !B || !C || !work) return EXAT_ERR_NULL;
    if (L < 1 || M < 1 || N < 1 || R < 1 || P < 1 || sweeps < 0) return EXAT_ERR_SHAPE;
    if (L > CP_MAX || M > CP_MAX || N > CP_MAX || R > CP_MAX || P > (1 << 20)) return EXAT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = (int64_t)L * M * N * P;
    float *Y2 = work, *Y3 = work + total, *part = work + 2 * total;
    if (status) {   // a fill kernel, not a memset: the call may be recorded into a graph
        hipLaunchKernelGGL(k_cpals_clear_status, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, status, P);
        if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    }
    if (sweeps > 0) {
        hipLaunchKernelGGL(k_cpals_permute, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, Y, Y2, Y3, L, M, N, total);
        if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    }
    auto update = [&](const float *Yp, float *F0, const float *F1, const float *F2, int D0, int D1, int D2) {
        CpUpdate u;
        u.Yp = Yp; u.F0 = F0; u.F1 = F1; u.F2 = F2; u.part = part; u.status = status; u.D0 = D0; u.D1 = D1; u.D2 = D2; u.R = R; u.NS = 1; u.DS = D2;
        if (R <= 16) return launch_update<4>(u, P, st);
        if (R <= 32) return launch_update<8>(u, P, st);
        return launch_update<16>(u, P, st);
    };
    for (int t = 0; t < sweeps; t++) {
        int rc;
        if ((rc = update(Y, A, B, C, L, M, N)) != EXAT_OK) return rc;    // A <- Y_(1) (C kr B) [(C^T C) * (B^T B)]^-1
        if ((rc = update(Y2, B, A, C, M, L, N)) != EXAT_OK) return rc;   // B <- Y_(2) (C kr A) [(C^T C) * (A^T A)]^-1
        if ((rc = update(Y3, C, A, B, N, L, M)) != EXAT_OK) return rc;   // C <- Y_(3) (B kr A) [(B^T B) * (A^T A)]^-1
    }
    return EXAT_OK;
}

}  // extern "C"

// ---- exat_cpals for callers that cannot allocate: the workspace is a static device array ----
namespace {
constexpr int64_t kScratchFloats = 4LL << 20;   // 16 MiB per GPU, held until the process ends
constexpr int kMaxDevices = 64;
float *g_scratch_ptr[kMaxDevices] = {};         // device address of `scratch` on each GPU (each holds its own copy)
}  // namespace
static __device__ __align__(256) float scratch[kScratchFloats];

extern "C" {

int exat_cpals_noalloc(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps, float *A, float *B,
                       float *C, void *stream)
{
    if (!Y || !A || !B || !C) return EXAT_ERR_NULL;
    if (L < 1 || M < 1 || N < 1 || R < 1 || P < 1 || sweeps < 0) return EXAT_ERR_SHAPE;
    if (L > CP_MAX || M > CP_MAX || N > CP_MAX || R > CP_MAX || P > (1 << 20)) return EXAT_ERR_SHAPE;
    if (exat_cpals_workspace_floats(L, M, N, P) > kScratchFloats) return EXAT_ERR_SHAPE;   // beyond the static workspace
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EXAT_ERR_HIP;
    if (!g_scratch_ptr[dev]) {
        // in host code the array's name is a stand-in, not a device address: ask the runtime for this GPU's copy, once
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return EXAT_ERR_HIP; }
        g_scratch_ptr[dev] = (float *)ptr;
    }
    // nothing of the workspace has to start at zero: every sweep writes the permuted copies and the slab sums before
    // it reads them
    return exat_cpals(Y, L, M, N, P, R, sweeps, A, B, C, g_scratch_ptr[dev], stream);
}

}  // extern "C"
