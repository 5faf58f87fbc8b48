// Joining the replicas: the stacked least-squares problem of the paper's Eq. 4 (Sec. 3 "Decomposition"),
//   [A_1; ...; A_P] = [U_1; ...; U_P] X,     (PL x R) = (PL x I)(I x R),
// solved for X by conjugate gradients on the normal equations (CGLS), all R columns at once, each with its own
// step lengths.  Declarations and contracts in include/exat.h.
//
// The stacked matrix is the array the compression was set up with; it is only read, never factored or copied.
// One iteration is two launches, each a tall-and-skinny product on the fp32 matrix cores (32x32x2):
//   k_ls_up    q = U p      one workgroup per 32 rows of U; p = s + beta p_old is formed on the fly
//   k_ls_down  s = U^T r    one workgroup per 32 columns of U; r = r_old - alpha q is formed on the fly, and the
//                           workgroup updates its 32 rows of x
// Every workgroup also writes its share of the new p (r) into the other of two buffers, so no launch reads what
// it writes.  The squared column norms that alpha and beta need are left as per-workgroup partial sums and added
// in workgroup order by whoever needs them: no atomics, every sum has a fixed order.
// In fp32 the iteration must not run on past convergence (the step lengths become ratios of rounding noise and the
// iterates drift away again), so a column whose normal-equation residual has fallen to `tol` times its start value
// is frozen: its alpha and beta are zero from then on, which every workgroup decides alike from the same sums.
#include "../../include/exat.h"

#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int LS_MAXR = 64;

struct LsParams {
    const float *U;       // rows x I, row-major, leading dimension ldU
    int64_t ldU;
    int rows, I, R;
    int Rp, rowsP, IP;    // R, rows and I rounded up to multiples of 32; the work arrays are padded with zeros
    int nbA, nbB;         // workgroups of k_ls_up (rowsP / 32) and k_ls_down (IP / 32)
    int vec4;             // rows of U may be read 16 bytes at a time
    float tol2;           // a column whose gamma has fallen to tol2 * gamma_0 is left as it is
    float *x, *s, *p[2];  // IP x Rp, row-major
    float *q, *r[2];      // rowsP x Rp, row-major
    float *partA;         // [nbA][64]    column sums of q^2 per workgroup
    float *partB[3];      // [nbB][64]    column sums of s^2 per workgroup: initial, then two alternating
};

// stacked replica factors A[l + L*(c + R*p)] -> r[row][c], row = p*L + l, padded with zeros
__global__ void k_ls_init(LsParams P, const float *Astack, int L)
{
    const int64_t n = (int64_t)P.rowsP * P.Rp;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % P.Rp);
        const int64_t row = idx / P.Rp;
        float v = 0.0f;
        if (row < P.rows && c < P.R) v = Astack[row % L + (int64_t)L * (c + (int64_t)P.R * (row / L))];
        P.r[0][idx] = v;
    }
}

// Adds the partial tiles of waves 1..3 to wave 0's, in wave order.  After it wave 0 holds the workgroup's
// 32 x (32 NT) tile: register v of lane (m, h) is element [8 (v / 4) + 4 h + v % 4][m] of column tile nt.
template <int NT>
__device__ __forceinline__ void reduce_waves(f32x16 (&acc)[NT], float (*red)[NT][16][64], int w, int lane)
{
    if (w > 0) {
#pragma unroll
        for (int nt = 0; nt < NT; nt++)
#pragma unroll
            for (int v = 0; v < 16; v++) red[w - 1][nt][v][lane] = acc[nt][v];
    }
    __syncthreads();
    if (w == 0) {
        for (int ww = 0; ww < 3; ww++)
#pragma unroll
            for (int nt = 0; nt < NT; nt++)
#pragma unroll
                for (int v = 0; v < 16; v++) acc[nt][v] += red[ww][nt][v][lane];
    }
}

// wave 0: stores the tile to out (rows row0.., leading dimension Rp) and the tile's column sums of squares
template <int NT>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[NT], float *out, int Rp, int row0, float *part, int m, int h)
{
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        float ss = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int row = row0 + 8 * (v / 4) + 4 * h + (v % 4);
            out[(int64_t)row * Rp + 32 * nt + m] = acc[nt][v];
            ss += acc[nt][v] * acc[nt][v];
        }
        ss += __shfl_xor(ss, 32);
        if (h == 0) part[32 * nt + m] = ss;
    }
    if (NT == 1 && h == 1) part[32 + m] = 0.0f;
}

// q = U p_t with p_t = s + beta_t p_{t-1} (p_0 = s); beta_t = gamma_t / gamma_{t-1}, gamma = column sums of s^2
template <int NT>
__global__ __launch_bounds__(256) void k_ls_up(LsParams P, int t, int cur, int prev)
{
    __shared__ float red[3][NT][16][64];
    __shared__ float beta_s[64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, m = lane & 31, h = lane >> 5;
    const int b = blockIdx.x;
    if (tid < 64) {
        float bt = 0.0f;
        if (t > 0) {
            float g1 = 0.0f, g0 = 0.0f, gz = 0.0f;
            for (int i = 0; i < P.nbB; i++) {
                g1 += P.partB[cur][i * 64 + tid];
                g0 += P.partB[prev][i * 64 + tid];
                gz += P.partB[0][i * 64 + tid];
            }
            bt = (g0 > 0.0f && g1 > P.tol2 * gz) ? g1 / g0 : 0.0f;
        }
        beta_s[tid] = bt;
    }
    __syncthreads();
    const float *s = P.s, *pold = P.p[(t + 1) & 1];
    float *pnew = P.p[t & 1];
    // this workgroup's share of p_t
    const int64_t n = (int64_t)P.IP * P.Rp;
    for (int64_t idx = (int64_t)b * 256 + tid; idx < n; idx += (int64_t)gridDim.x * 256) {
        float v = s[idx];
        if (t > 0) v += beta_s[idx % P.Rp] * pold[idx];
        pnew[idx] = v;
    }
    float bet[NT];
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        bet[nt] = beta_s[32 * nt + m];
#pragma unroll
        for (int v = 0; v < 16; v++) acc[nt][v] = 0.0f;
    }
    const int row = 32 * b + m;
    const bool rok = row < P.rows;
    const float *urow = P.U + (int64_t)(rok ? row : P.rows - 1) * P.ldU;
    // 8 values of k per step (lane half h takes 4 consecutive ones); wave w takes steps w, w + 4, ...
    for (int k0 = 8 * w; k0 < P.IP; k0 += 32) {
        const int k = k0 + 4 * h;
        float u[4];
        if (P.vec4 && k + 3 < P.I) {
            const float4 v = *(const float4 *)(urow + k);
            u[0] = v.x; u[1] = v.y; u[2] = v.z; u[3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; e++) u[e] = (k + e < P.I) ? urow[k + e] : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const float ue = rok ? u[e] : 0.0f;
#pragma unroll
            for (int nt = 0; nt < NT; nt++) {
                const int64_t o = (int64_t)(k + e) * P.Rp + 32 * nt + m;
                float pv = s[o];
                if (t > 0) pv += bet[nt] * pold[o];
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(ue, pv, acc[nt], 0, 0, 0);
            }
        }
    }
    reduce_waves<NT>(acc, red, w, lane);
    if (w == 0) store_tile<NT>(acc, P.q, P.Rp, 32 * b, P.partA + (int64_t)b * 64, m, h);
}

// s = U^T r_{t+1} with r_{t+1} = r_t - alpha_t q_t, x += alpha_t p_t; alpha_t = gamma_t / (column sums of q_t^2).
// t = -1 is the start: r is taken as it stands, x is cleared.
template <int NT>
__global__ __launch_bounds__(256) void k_ls_down(LsParams P, int t, int cur, int nxt)
{
    __shared__ float red[3][NT][16][64];
    __shared__ float alpha_s[64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, m = lane & 31, h = lane >> 5;
    const int b = blockIdx.x;
    if (tid < 64) {
        float a = 0.0f;
        if (t >= 0) {
            float g = 0.0f, gz = 0.0f, d = 0.0f;
            for (int i = 0; i < P.nbB; i++) {
                g += P.partB[cur][i * 64 + tid];
                gz += P.partB[0][i * 64 + tid];
            }
            for (int i = 0; i < P.nbA; i++) d += P.partA[i * 64 + tid];
            a = (d > 0.0f && g > P.tol2 * gz) ? g / d : 0.0f;
        }
        alpha_s[tid] = a;
    }
    __syncthreads();
    const float *rold = P.r[t < 0 ? 0 : (t + 1) & 1], *q = P.q;
    float *rnew = P.r[t < 0 ? 1 : t & 1];
    const int64_t n = (int64_t)P.rowsP * P.Rp;
    for (int64_t idx = (int64_t)b * 256 + tid; idx < n; idx += (int64_t)gridDim.x * 256) {
        float v = rold[idx];
        if (t >= 0) v -= alpha_s[idx % P.Rp] * q[idx];
        rnew[idx] = v;
    }
    // the 32 rows of x that belong to this workgroup's columns of U
    const float *pt = P.p[t & 1];
    for (int e = tid; e < 32 * P.Rp; e += 256) {
        const int64_t o = (int64_t)32 * b * P.Rp + e;
        P.x[o] = t >= 0 ? P.x[o] + alpha_s[e % P.Rp] * pt[o] : 0.0f;
    }
    float al[NT];
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        al[nt] = alpha_s[32 * nt + m];
#pragma unroll
        for (int v = 0; v < 16; v++) acc[nt][v] = 0.0f;
    }
    const int i = 32 * b + m;
    const bool iok = i < P.I;
    const float *ucol = P.U + (iok ? i : P.I - 1);
    // 16 rows of U per step (lane half h takes every second one); wave w takes steps w, w + 4, ...
    for (int k0 = 16 * w; k0 < P.rowsP; k0 += 64) {
        float u[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int pl = k0 + 2 * e + h;
            const float v = ucol[(int64_t)(pl < P.rows ? pl : P.rows - 1) * P.ldU];
            u[e] = (iok && pl < P.rows) ? v : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int pl = k0 + 2 * e + h;
#pragma unroll
            for (int nt = 0; nt < NT; nt++) {
                const int64_t o = (int64_t)pl * P.Rp + 32 * nt + m;
                float rv = rold[o];
                if (t >= 0) rv -= al[nt] * q[o];
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(u[e], rv, acc[nt], 0, 0, 0);
            }
        }
    }
    reduce_waves<NT>(acc, red, w, lane);
    if (w == 0) store_tile<NT>(acc, P.s, P.Rp, 32 * b, P.partB[nxt] + (int64_t)b * 64, m, h);
}

// X[i + I*c] = x[i][c]; relres[c] = sqrt(gamma_last / gamma_0), the norm of column c of U^T (A - U X) relative to
// that of U^T A
__global__ void k_ls_finish(LsParams P, int last, float *X, float *relres)
{
    const int64_t n = (int64_t)P.I * P.R;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t c = idx / P.I, i = idx % P.I;
        X[idx] = P.x[i * P.Rp + c];
    }
    if (relres && blockIdx.x == 0 && (int)threadIdx.x < P.R) {
        float g1 = 0.0f, g0 = 0.0f;
        for (int i = 0; i < P.nbB; i++) {
            g1 += P.partB[last][i * 64 + threadIdx.x];
            g0 += P.partB[0][i * 64 + threadIdx.x];
        }
        relres[threadIdx.x] = g0 > 0.0f ? sqrtf(g1 / g0) : 0.0f;
    }
}

inline int up32(int v) { return 32 * ((v + 31) / 32); }

bool shape_ok(int32_t P, int32_t L, int32_t I, int32_t R)
{
    return P >= 1 && L >= 1 && I >= 1 && R >= 1 && R <= LS_MAXR && (int64_t)P * L <= (1 << 24) && I <= (1 << 24);
}

}  // namespace

extern "C" {

int64_t exat_ls_workspace_floats(int32_t P, int32_t L, int32_t I, int32_t R)
{
    if (!shape_ok(P, L, I, R)) return 0;
    const int64_t rowsP = up32(P * L), IP = up32(I), Rp = up32(R);
    return 4 * IP * Rp + 3 * rowsP * Rp + (rowsP / 32) * 64 + 3 * (IP / 32) * 64;
}

int exat_ls(const float *U, int64_t ldU, int32_t P, int32_t L, int32_t I, const float *Astack, int32_t R, int32_t iters,
            float tol, float *X, float *relres, float *work, void *stream)
{
    if (!U || !Astack || !X || !work) return EXAT_ERR_NULL;
    if (!shape_ok(P, L, I, R) || ldU < I || iters < 0 || !(tol >= 0.0f)) return EXAT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    LsParams p;
    p.U = U; p.ldU = ldU; p.rows = P * L; p.I = I; p.R = R;
    p.Rp = up32(R); p.rowsP = up32(p.rows); p.IP = up32(I);
    p.nbA = p.rowsP / 32; p.nbB = p.IP / 32;
    p.tol2 = tol * tol;
    p.vec4 = (ldU % 4 == 0 && ((uintptr_t)U & 15) == 0) ? 1 : 0;
    const int64_t nx = (int64_t)p.IP * p.Rp, nr = (int64_t)p.rowsP * p.Rp;
    float *w = work;
    p.x = w; w += nx; p.s = w; w += nx; p.p[0] = w; w += nx; p.p[1] = w; w += nx;
    p.q = w; w += nr; p.r[0] = w; w += nr; p.r[1] = w; w += nr;
    p.partA = w; w += (int64_t)p.nbA * 64;
    for (int t = 0; t < 3; t++) { p.partB[t] = w; w += (int64_t)p.nbB * 64; }
    const bool two = p.Rp == 64;
    auto down = [&](int t, int cur, int nxt) {
        if (two) hipLaunchKernelGGL(k_ls_down<2>, dim3((unsigned)p.nbB), dim3(256), 0, st, p, t, cur, nxt);
        else hipLaunchKernelGGL(k_ls_down<1>, dim3((unsigned)p.nbB), dim3(256), 0, st, p, t, cur, nxt);
    };
    auto up = [&](int t, int cur, int prev) {
        if (two) hipLaunchKernelGGL(k_ls_up<2>, dim3((unsigned)p.nbA), dim3(256), 0, st, p, t, cur, prev);
        else hipLaunchKernelGGL(k_ls_up<1>, dim3((unsigned)p.nbA), dim3(256), 0, st, p, t, cur, prev);
    };
    // gamma_t (the column sums of s_t^2) lives in partB[cur(t)]: gamma_0 stays in buffer 0 for the final ratio
    auto cur_of = [](int t) { return t == 0 ? 0 : 1 + ((t - 1) & 1); };
    const unsigned g_init = (unsigned)((nr + 255) / 256 < 4096 ? (nr + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_ls_init, dim3(g_init), dim3(256), 0, st, p, Astack, (int)L);
    down(-1, 0, 0);
    for (int t = 0; t < iters; t++) {
        up(t, cur_of(t), t > 0 ? cur_of(t - 1) : 0);
        down(t, cur_of(t), cur_of(t + 1));
    }
    const int64_t nout = (int64_t)I * R;
    const unsigned g_fin = (unsigned)((nout + 255) / 256 < 4096 ? (nout + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_ls_finish, dim3(g_fin), dim3(256), 0, st, p, cur_of(iters), X, relres);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

}  // extern "C"
