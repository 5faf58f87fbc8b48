// Joining the replicas: the stacked least-squares problem of the paper's Eq. 4 (Sec. 3 "Decomposition"),
//   [A_1; ...; A_P] = [U_1; ...; U_P] X,     (PL x R) = (PL x I)(I x R),
// solved for X by conjugate gradients on the normal equations (CGLS), all R columns at once, each with its own
// step lengths.  Declarations and contracts in include/exat.h.
//
// The stacked matrix is the array the compression was set up with; it is only read, never factored or copied.
// One iteration is two launches, each a tall-and-skinny product on the fp32 matrix cores (32x32x2):
//   k_ls_up    q = U p      one workgroup per 32 rows of U and 32 right-hand sides; p = s + beta p_old is formed
//                           on the fly
//   k_ls_down  s = U^T r    one workgroup per 32 columns of U and 32 right-hand sides; r = r_old - alpha q is
//                           formed on the fly, and the workgroup updates its block of x
// The eight waves of a workgroup split the contraction range and add their tiles in wave order.
// A small problem has too few output tiles to fill the chip; then several workgroups share a tile, each takes part
// of the contraction range, and k_ls_join adds their partial products in a fixed order.
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
    float *join;          // [group][rows][Rp] partial products when several workgroups share an output tile
};

constexpr int LS_MAXJOIN = 512;   // output tiles x groups never exceeds this when there is more than one group

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

constexpr int LS_NW = 8;   // waves per workgroup; they split the contraction range

// Adds the partial tiles of waves 1.. to wave 0's, in wave order.  After it wave 0 holds the workgroup's 32 x 32
// tile: register v of lane (m, h) is element [8 (v / 4) + 4 h + v % 4][m].
__device__ __forceinline__ void reduce_waves(f32x16 &acc, float (*red)[16][64], int w, int lane)
{
    if (w > 0) {
#pragma unroll
        for (int v = 0; v < 16; v++) red[w - 1][v][lane] = acc[v];
    }
    __syncthreads();
    if (w == 0) {
        for (int ww = 0; ww < LS_NW - 1; ww++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[v] += red[ww][v][lane];
    }
}

// Column sums of three [n][64] arrays of per-workgroup partial sums at once (so that their loads are in flight
// together): wave g adds the entries g, g + LS_NW, ... of column tid % 64, the first 64 threads then add the waves'
// results in wave order and hold the sums.  All threads of the workgroup must call it.
__device__ __forceinline__ void colsum3(const float *__restrict__ pa, int na, const float *__restrict__ pb, int nb,
                                        const float *__restrict__ pc, int nc, float (*tmp)[LS_NW][64], int tid,
                                        float &ra, float &rb, float &rc)
{
    const int c = tid & 63, g = tid >> 6;
    const int nmax = na > nb ? (na > nc ? na : nc) : (nb > nc ? nb : nc);
    float a = 0.0f, b = 0.0f, d = 0.0f;
#pragma unroll 4
    for (int i = g; i < nmax; i += LS_NW) {
        const float va = i < na ? pa[i * 64 + c] : 0.0f;
        const float vb = i < nb ? pb[i * 64 + c] : 0.0f;
        const float vc = i < nc ? pc[i * 64 + c] : 0.0f;
        a += va; b += vb; d += vc;
    }
    tmp[0][g][c] = a; tmp[1][g][c] = b; tmp[2][g][c] = d;
    __syncthreads();
    ra = rb = rc = 0.0f;
    if (tid < 64)
        for (int w = 0; w < LS_NW; w++) { ra += tmp[0][w][c]; rb += tmp[1][w][c]; rc += tmp[2][w][c]; }
}

// wave 0: stores the tile to out (rows row0.., columns col0.., leading dimension Rp) and the tile's column sums
// of squares
__device__ __forceinline__ void store_tile(const f32x16 &acc, float *out, int Rp, int row0, int col0, float *part, int m, int h)
{
    float ss = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; v++) {
        const int row = row0 + 8 * (v / 4) + 4 * h + (v % 4);
        out[(int64_t)row * Rp + col0 + m] = acc[v];
        ss += acc[v] * acc[v];
    }
    if (!part) return;
    ss += __shfl_xor(ss, 32);
    if (h == 0) part[col0 + m] = ss;
    if (Rp == 32 && h == 1) part[32 + m] = 0.0f;
}

// Adds the G partial products of the workgroups that shared an output tile, in group order, into `out` and leaves
// the column sums of squares of the 32 rows of workgroup b in part[b][64].  256 threads: a thread keeps one column.
__global__ __launch_bounds__(256) void k_ls_join(const float *__restrict__ src, int G, int64_t gstride, float *__restrict__ out,
                                                 float *__restrict__ part, int Rp)
{
    __shared__ float col[8][64];
    const int tid = threadIdx.x, c = tid & (Rp - 1), r0 = tid / Rp, nr = 256 / Rp;   // nr row groups: 8 or 4
    const int64_t base = (int64_t)blockIdx.x * 32 * Rp;
    float ss = 0.0f;
    for (int r = r0; r < 32; r += nr) {
        const int64_t off = base + (int64_t)r * Rp + c;
        float v = 0.0f;
        for (int g = 0; g < G; g++) v += src[g * gstride + off];
        out[off] = v;
        ss += v * v;
    }
    col[r0][c] = ss;
    __syncthreads();
    if (tid < 64) {
        float t = 0.0f;
        if (tid < Rp)
            for (int g = 0; g < nr; g++) t += col[g][tid];
        part[(int64_t)blockIdx.x * 64 + tid] = t;
    }
}

constexpr int LS_D = 4;   // steps whose operands a wave loads in one batch; two batches are in flight

// q = U p_t with p_t = s + beta_t p_{t-1} (p_0 = s); beta_t = gamma_t / gamma_{t-1}, gamma = column sums of s^2.
// Workgroup (b, nt): rows 32 b .. 32 b + 31 of U, columns 32 nt .. 32 nt + 31 of p.
__global__ __launch_bounds__(64 * LS_NW) void k_ls_up(LsParams P, int t, int cur, int prev)
{
    __shared__ float red[LS_NW - 1][16][64];
    __shared__ float beta_s[64];
    __shared__ float tmp[3][LS_NW][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, m = lane & 31, h = lane >> 5;
    const int b = blockIdx.x, col0 = 32 * blockIdx.y;
    const float *__restrict__ s = P.s, *__restrict__ pold = P.p[(t + 1) & 1];
    float *__restrict__ pnew = P.p[t & 1];
    const int row = 32 * b + m;
    const bool rok = row < P.rows;
    const float *urow = P.U + (int64_t)(rok ? row : P.rows - 1) * P.ldU;
    // 8 values of k per step (lane half h takes 4 consecutive ones); wave w takes steps w, w + LS_NW, ..., LS_D
    // of them per batch
    struct Ops { float u[4], sv[4], pv[4]; };
    Ops oa[LS_D], ob[LS_D];
    auto load_batch = [&](Ops *o, int k0) {
#pragma unroll
        for (int d = 0; d < LS_D; d++) {
            const int k = k0 + d * 8 * LS_NW + 4 * h;
            if (k - 4 * h < P.IP) {
                if (P.vec4 && k + 3 < P.I) {
                    const float4 v = *(const float4 *)(urow + k);
                    o[d].u[0] = v.x; o[d].u[1] = v.y; o[d].u[2] = v.z; o[d].u[3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; e++) o[d].u[e] = (k + e < P.I) ? urow[k + e] : 0.0f;
                }
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const unsigned off = (unsigned)(k + e) * (unsigned)P.Rp + (unsigned)(col0 + m);   // < 2^30
                    o[d].sv[e] = s[off];
                    o[d].pv[e] = t > 0 ? pold[off] : 0.0f;
                }
            }
        }
    };
    auto mac_batch = [&](const Ops *o, int k0, float bet, f32x16 &acc) {
#pragma unroll
        for (int d = 0; d < LS_D; d++) {
            if (k0 + d * 8 * LS_NW < P.IP) {
#pragma unroll
                for (int e = 0; e < 4; e++)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(rok ? o[d].u[e] : 0.0f, o[d].sv[e] + bet * o[d].pv[e], acc, 0, 0, 0);
            }
        }
    };
    constexpr int BK = LS_D * 8 * LS_NW;   // values of k per batch of the workgroup
    const int GK = BK * (int)gridDim.z;    // the groups of an output tile take the batches in turn
    const int kw = 8 * w + BK * (int)blockIdx.z;
    load_batch(oa, kw);                    // in flight while the step length is worked out
    load_batch(ob, kw + GK);
    if (t > 0) {
        float g1, g0, gz;
        colsum3(P.partB[cur], P.nbB, P.partB[prev], P.nbB, P.partB[0], P.nbB, tmp, tid, g1, g0, gz);
        if (tid < 64) beta_s[tid] = (g0 > 0.0f && g1 > P.tol2 * gz) ? g1 / g0 : 0.0f;
    } else if (tid < 64)
        beta_s[tid] = 0.0f;
    __syncthreads();
    const float bet = beta_s[col0 + m];
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = 0.0f;
    for (int k0 = kw; k0 < P.IP; k0 += 2 * GK) {
        mac_batch(oa, k0, bet, acc);
        load_batch(oa, k0 + 2 * GK);
        mac_batch(ob, k0 + GK, bet, acc);
        load_batch(ob, k0 + 3 * GK);
    }
    // this workgroup's share of p_t
    const int64_t n = (int64_t)P.IP * P.Rp;
    const int64_t wg = b + (int64_t)gridDim.x * (blockIdx.y + (int64_t)gridDim.y * blockIdx.z), nwg = (int64_t)gridDim.x * gridDim.y * gridDim.z;
#pragma unroll 4
    for (int64_t idx = wg * (64 * LS_NW) + tid; idx < n; idx += nwg * (64 * LS_NW)) {
        float v = s[idx];
        if (t > 0) v += beta_s[idx & (P.Rp - 1)] * pold[idx];
        pnew[idx] = v;
    }
    reduce_waves(acc, red, w, lane);
    if (w == 0) {
        if (gridDim.z == 1) store_tile(acc, P.q, P.Rp, 32 * b, col0, P.partA + (int64_t)b * 64, m, h);
        else store_tile(acc, P.join + (int64_t)blockIdx.z * P.rowsP * P.Rp, P.Rp, 32 * b, col0, nullptr, m, h);
    }
}

// s = U^T r_{t+1} with r_{t+1} = r_t - alpha_t q_t, x += alpha_t p_t; alpha_t = gamma_t / (column sums of q_t^2).
// t = -1 is the start: r is taken as it stands, x is cleared.
// Workgroup (b, nt): columns 32 b .. 32 b + 31 of U, columns 32 nt .. 32 nt + 31 of r.
__global__ __launch_bounds__(64 * LS_NW) void k_ls_down(LsParams P, int t, int cur, int nxt)
{
    __shared__ float red[LS_NW - 1][16][64];
    __shared__ float alpha_s[64];
    __shared__ float tmp[3][LS_NW][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, m = lane & 31, h = lane >> 5;
    const int b = blockIdx.x, col0 = 32 * blockIdx.y;
    const float *__restrict__ rold = P.r[t < 0 ? 0 : (t + 1) & 1], *__restrict__ q = P.q;
    float *__restrict__ rnew = P.r[t < 0 ? 1 : t & 1];
    const int i = 32 * b + m;
    const bool iok = i < P.I;
    const unsigned ucol = (unsigned)(iok ? i : P.I - 1), ldu = (unsigned)P.ldU;   // rows * ldU < 2^30
    // 8 rows of U per step (lane half h takes every second one); wave w takes steps w, w + LS_NW, ..., LS_D of them
    // per batch
    struct Ops { float u[4], rv[4], qv[4]; };
    Ops oa[LS_D], ob[LS_D];
    auto load_batch = [&](Ops *o, int k0) {
#pragma unroll
        for (int d = 0; d < LS_D; d++) {
            if (k0 + d * 8 * LS_NW < P.rowsP) {
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int pl = k0 + d * 8 * LS_NW + 2 * e + h;
                    const float v = P.U[(unsigned)(pl < P.rows ? pl : P.rows - 1) * ldu + ucol];
                    o[d].u[e] = (iok && pl < P.rows) ? v : 0.0f;
                    const unsigned off = (unsigned)pl * (unsigned)P.Rp + (unsigned)(col0 + m);   // < 2^30
                    o[d].rv[e] = rold[off];
                    o[d].qv[e] = t >= 0 ? q[off] : 0.0f;
                }
            }
        }
    };
    auto mac_batch = [&](const Ops *o, int k0, float al, f32x16 &acc) {
#pragma unroll
        for (int d = 0; d < LS_D; d++) {
            if (k0 + d * 8 * LS_NW < P.rowsP) {
#pragma unroll
                for (int e = 0; e < 4; e++)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o[d].u[e], o[d].rv[e] - al * o[d].qv[e], acc, 0, 0, 0);
            }
        }
    };
    constexpr int BK = LS_D * 8 * LS_NW;   // rows of U per batch of the workgroup
    const int GK = BK * (int)gridDim.z;    // the groups of an output tile take the batches in turn
    const int kw = 8 * w + BK * (int)blockIdx.z;
    load_batch(oa, kw);                    // in flight while the step length is worked out
    load_batch(ob, kw + GK);
    if (t >= 0) {
        float g, gz, d;
        colsum3(P.partB[cur], P.nbB, P.partB[0], P.nbB, P.partA, P.nbA, tmp, tid, g, gz, d);
        if (tid < 64) alpha_s[tid] = (d > 0.0f && g > P.tol2 * gz) ? g / d : 0.0f;
    } else if (tid < 64)
        alpha_s[tid] = 0.0f;
    __syncthreads();
    const float al = alpha_s[col0 + m];
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = 0.0f;
    for (int k0 = kw; k0 < P.rowsP; k0 += 2 * GK) {
        mac_batch(oa, k0, al, acc);
        load_batch(oa, k0 + 2 * GK);
        mac_batch(ob, k0 + GK, al, acc);
        load_batch(ob, k0 + 3 * GK);
    }
    const int64_t n = (int64_t)P.rowsP * P.Rp;
    const int64_t wg = b + (int64_t)gridDim.x * (blockIdx.y + (int64_t)gridDim.y * blockIdx.z), nwg = (int64_t)gridDim.x * gridDim.y * gridDim.z;
#pragma unroll 4
    for (int64_t idx = wg * (64 * LS_NW) + tid; idx < n; idx += nwg * (64 * LS_NW)) {
        float v = rold[idx];
        if (t >= 0) v -= alpha_s[idx & (P.Rp - 1)] * q[idx];
        rnew[idx] = v;
    }
    // the 32 x 32 block of x that belongs to this workgroup's columns of U and of r
    const float *__restrict__ pt = P.p[t & 1];
#pragma unroll 2
    for (int e = tid; e < 32 * 32 && blockIdx.z == 0; e += 64 * LS_NW) {
        const int64_t off = (int64_t)(32 * b + e / 32) * P.Rp + col0 + e % 32;
        P.x[off] = t >= 0 ? P.x[off] + alpha_s[col0 + e % 32] * pt[off] : 0.0f;
    }
    reduce_waves(acc, red, w, lane);
    if (w == 0) {
        if (gridDim.z == 1) store_tile(acc, P.s, P.Rp, 32 * b, col0, P.partB[nxt] + (int64_t)b * 64, m, h);
        else store_tile(acc, P.join + (int64_t)blockIdx.z * P.IP * P.Rp, P.Rp, 32 * b, col0, nullptr, m, h);
    }
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
    return P >= 1 && L >= 1 && I >= 1 && R >= 1 && R <= LS_MAXR && (int64_t)P * L <= (1 << 22) && I <= (1 << 22);
}

}  // namespace

extern "C" {

int64_t exat_ls_workspace_floats(int32_t P, int32_t L, int32_t I, int32_t R)
{
    if (!shape_ok(P, L, I, R)) return 0;
    const int64_t rowsP = up32(P * L), IP = up32(I), Rp = up32(R);
    return 4 * IP * Rp + 3 * rowsP * Rp + (rowsP / 32) * 64 + 3 * (IP / 32) * 64 + LS_MAXJOIN * 1024;
}

int exat_ls(const float *U, int64_t ldU, int32_t P, int32_t L, int32_t I, const float *Astack, int32_t R, int32_t iters,
            float tol, float *X, float *relres, float *work, void *stream)
{
    if (!U || !Astack || !X || !work) return EXAT_ERR_NULL;
    if (!shape_ok(P, L, I, R) || ldU < I || iters < 0 || !(tol >= 0.0f)) return EXAT_ERR_SHAPE;
    if ((int64_t)P * L * ldU > ((int64_t)1 << 30)) return EXAT_ERR_SHAPE;   // the kernels index U with 32 bits
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
    p.join = w;
    const unsigned nct = (unsigned)(p.Rp / 32);   // column tiles of 32 right-hand sides
    // A single workgroup draws little bandwidth from memory, so small problems are spread further: up to 16 groups of
    // workgroups share an output tile (one per batch of the contraction range at most), each leaves a partial
    // product, and k_ls_join adds them in group order.
    auto groups = [&](int64_t tiles, int64_t len) {
        const int64_t bk = (int64_t)LS_D * 8 * LS_NW, batches = (len + bk - 1) / bk;
        int64_t g = LS_MAXJOIN / tiles;
        if (g > 16) g = 16;
        if (g > batches) g = batches;
        return (unsigned)(g < 1 ? 1 : g);
    };
    const unsigned ga = groups((int64_t)p.nbA * nct, p.IP), gb = groups((int64_t)p.nbB * nct, p.rowsP);
    auto down = [&](int t, int cur, int nxt) {
        hipLaunchKernelGGL(k_ls_down, dim3((unsigned)p.nbB, nct, gb), dim3(64 * LS_NW), 0, st, p, t, cur, nxt);
        if (gb > 1)
            hipLaunchKernelGGL(k_ls_join, dim3((unsigned)p.nbB), dim3(256), 0, st, (const float *)p.join, (int)gb, nx, p.s, p.partB[nxt], p.Rp);
    };
    auto up = [&](int t, int cur, int prev) {
        hipLaunchKernelGGL(k_ls_up, dim3((unsigned)p.nbA, nct, ga), dim3(64 * LS_NW), 0, st, p, t, cur, prev);
        if (ga > 1)
            hipLaunchKernelGGL(k_ls_join, dim3((unsigned)p.nbA), dim3(256), 0, st, (const float *)p.join, (int)ga, nr, p.q, p.partA, p.Rp);
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
