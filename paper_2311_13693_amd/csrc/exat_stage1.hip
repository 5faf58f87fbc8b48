// First stage of the two-stage compression (paper Sec. 4.4): X1 = X x1 U x2 V x3 W with sparse U, V, W
// shared by all replicas.  Declarations and contracts in include/exat.h.
//
// The stage is bound by reading X once from HBM (4 bytes per element against 2*nnz_per_column flops), so the
// kernels are organised around that stream and use no matrix cores:
//   k_stage1_mode12  one workgroup per frontal slice k.  It walks the slice in 64-column x 128-row tiles that
//                    go HBM -> registers -> LDS (each element once, the next tile's loads in flight while the
//                    current one is used).  Mode 1: a lane owns a column j of the tile and a wave a set of
//                    output rows a; for every non-zero (a, i) of U inside the tile the wave does one LDS read
//                    and one FMA, the non-zero itself coming through the scalar cache (it is the same for all
//                    lanes).  When the column tile's rows are finished the 64 x A1 result is turned through
//                    LDS and mode 2 runs the same way with lanes along a.  The A1 x B1 slice result goes to
//                    Q[k][b][a].
//   k_stage1_mode3   X1[a,b,c] = sum_k W[c,k] Q[k][b][a], a thread per (a,b,c), the non-zeros of row c in
//                    stored order.
// Every sum has a fixed order, so results are bit-identical from run to run.
#include "../../include/exat.h"

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

namespace {

constexpr int S1_IT = 128;     // rows i per tile
constexpr int S1_JT = 64;      // columns j per tile (one per lane)
constexpr int S1_XS = S1_IT + 1;  // LDS row stride of the X tile (odd: lanes reading one i of 64 columns hit 64 banks)
constexpr int S1_MAXROWS = 128;   // largest A1 and B1
constexpr int64_t kMaxExtent1 = 2147483647LL - 64;

struct SEnt { int c; float v; };  // one non-zero: column inside its tile, value

struct S1Params {
    const float *X;
    int64_t I, J, K;
    int A1, B1;
    const int *Utp;    // [nit][A1+1] offsets into Uent; every (tile,row) range is a multiple of 4 entries
    const SEnt *Uent;
    const int *Vtp;    // [njt][B1+1]
    const SEnt *Vent;
    float *Q;          // [K][B1][A1]
};

// AR = output rows a per wave in mode 1 (A1 <= 4*AR), AT = 64-lane tiles of a in mode 2 (A1 <= 64*AT),
// BR = output rows b per wave in mode 2 (B1 <= 4*BR)
template <int AR, int AT, int BR>
__global__ __launch_bounds__(256) void k_stage1_mode12(const S1Params p)
{
    extern __shared__ float smem[];
    constexpr int ZS = 64 * AT + 1;
    float *xs = smem;                    // [64 j][S1_XS]
    float *zs = smem + S1_JT * S1_XS;    // [64 j][ZS]: mode-1 result of the current column tile
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t k = blockIdx.x;
    const float *Xk = p.X + k * p.I * p.J;
    const int nit = (int)((p.I + S1_IT - 1) / S1_IT), njt = (int)((p.J + S1_JT - 1) / S1_JT);
    const int li = tid & 127, lj = tid >> 7;   // this thread's element of the tile: row li, columns lj + 2*jj

    float acc2[AT][BR];
#pragma unroll
    for (int at = 0; at < AT; at++)
#pragma unroll
        for (int x = 0; x < BR; x++) acc2[at][x] = 0.0f;

    float pre[32];
    auto gload = [&](int jt, int it) {
        const int64_t i = (int64_t)it * S1_IT + li;
        const float *src = Xk + i + p.I * ((int64_t)jt * S1_JT + lj);
        const int64_t jleft = p.J - ((int64_t)jt * S1_JT + lj);   // columns lj + 2*jj with 2*jj < jleft exist
#pragma unroll
        for (int jj = 0; jj < 32; jj++)
            pre[jj] = (i < p.I && 2 * jj < jleft) ? src[p.I * 2 * jj] : 0.0f;
    };
    gload(0, 0);
    for (int jt = 0; jt < njt; jt++) {
        float acc1[AR];
#pragma unroll
        for (int x = 0; x < AR; x++) acc1[x] = 0.0f;
        for (int it = 0; it < nit; it++) {
            __syncthreads();   // the previous tile's readers are done
#pragma unroll
            for (int jj = 0; jj < 32; jj++) xs[(2 * jj + lj) * S1_XS + li] = pre[jj];
            __syncthreads();
            if (it + 1 < nit) gload(jt, it + 1);
            else if (jt + 1 < njt) gload(jt + 1, 0);
            const int *tp = p.Utp + (int64_t)it * (p.A1 + 1);
            const float *xl = xs + lane * S1_XS;
#pragma unroll
            for (int x = 0; x < AR; x++) {
                const int a = w + 4 * x;
                if (a < p.A1) {
                    const int e1 = tp[a + 1];
                    float s = acc1[x];
                    for (int e = tp[a]; e < e1; e += 4) {
                        const SEnt n0 = p.Uent[e], n1 = p.Uent[e + 1], n2 = p.Uent[e + 2], n3 = p.Uent[e + 3];
                        s = fmaf(n0.v, xl[n0.c], s);
                        s = fmaf(n1.v, xl[n1.c], s);
                        s = fmaf(n2.v, xl[n2.c], s);
                        s = fmaf(n3.v, xl[n3.c], s);
                    }
                    acc1[x] = s;
                }
            }
        }
        // turn the 64 x A1 result: zs[j][a]
#pragma unroll
        for (int x = 0; x < AR; x++) {
            const int a = w + 4 * x;
            if (a < p.A1) zs[lane * ZS + a] = acc1[x];
        }
        __syncthreads();
        const int *vp = p.Vtp + (int64_t)jt * (p.B1 + 1);
#pragma unroll
        for (int x = 0; x < BR; x++) {
            const int b = w + 4 * x;
            if (b < p.B1) {
                const int e1 = vp[b + 1];
                for (int e = vp[b]; e < e1; e += 4) {
#pragma unroll
                    for (int u = 0; u < 4; u++) {
                        const SEnt n = p.Vent[e + u];
#pragma unroll
                        for (int at = 0; at < AT; at++) acc2[at][x] = fmaf(n.v, zs[n.c * ZS + 64 * at + lane], acc2[at][x]);
                    }
                }
            }
        }
        // the next column tile's first barrier separates these reads of zs from its next writes
    }
    float *Qk = p.Q + k * p.B1 * p.A1;
#pragma unroll
    for (int x = 0; x < BR; x++) {
        const int b = w + 4 * x;
        if (b < p.B1) {
#pragma unroll
            for (int at = 0; at < AT; at++) {
                const int a = 64 * at + lane;
                if (a < p.A1) Qk[(int64_t)b * p.A1 + a] = acc2[at][x];
            }
        }
    }
}

struct S1Mode3Params {
    const float *Q;   // [K][AB]
    const int *rp;    // [C1+1]
    const int *ci;
    const float *val;
    float *X1;        // [C1][AB]: X1[a + A1*(b + B1*c)]
    int64_t AB;
};

__global__ __launch_bounds__(256) void k_stage1_mode3(const S1Mode3Params p)
{
    const int64_t ab = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y;
    if (ab >= p.AB) return;
    const int e1 = p.rp[c + 1];
    float s = 0.0f;
    for (int e = p.rp[c]; e < e1; e++) s = fmaf(p.val[e], p.Q[(int64_t)p.ci[e] * p.AB + ab], s);
    p.X1[ab + p.AB * c] = s;
}

// Splits a CSR matrix into column tiles of width `tile`: per tile a row-pointer array and entries with
// tile-local columns, every (tile,row) range padded with zero entries to a multiple of 4.
bool tile_csr(const exat_csr_t &m, int tile, std::vector<int> &tp, std::vector<SEnt> &ent)
{
    const int nt = (int)((m.cols + tile - 1) / tile);
    std::vector<std::vector<SEnt>> rows((size_t)nt * m.rows);
    for (int r = 0; r < m.rows; r++)
        for (int64_t e = m.rowptr[r]; e < m.rowptr[r + 1]; e++) {
            const int c = m.colidx[e];
            rows[(size_t)(c / tile) * m.rows + r].push_back(SEnt{c % tile, m.val[e]});
        }
    tp.assign((size_t)nt * (m.rows + 1), 0);
    ent.clear();
    for (int t = 0; t < nt; t++) {
        for (int r = 0; r < m.rows; r++) {
            tp[(size_t)t * (m.rows + 1) + r] = (int)ent.size();
            const auto &v = rows[(size_t)t * m.rows + r];
            ent.insert(ent.end(), v.begin(), v.end());
            while (ent.size() % 4) ent.push_back(SEnt{0, 0.0f});
            if (ent.size() > 0x7fffff00u) return false;
        }
        tp[(size_t)t * (m.rows + 1) + m.rows] = (int)ent.size();
    }
    return true;
}

int check_csr(const exat_csr_t *m, int64_t cols, int maxrows)
{
    if (!m || !m->rowptr) return EXAT_ERR_NULL;
    if (m->rows < 1 || m->rows > maxrows || m->cols != cols) return EXAT_ERR_SHAPE;
    if (m->rowptr[0] != 0) return EXAT_ERR_SHAPE;
    for (int r = 0; r < m->rows; r++)
        if (m->rowptr[r + 1] < m->rowptr[r]) return EXAT_ERR_SHAPE;
    const int64_t nnz = m->rowptr[m->rows];
    if (nnz > 0x7fffff00LL) return EXAT_ERR_SHAPE;
    if (nnz > 0 && (!m->colidx || !m->val)) return EXAT_ERR_NULL;
    for (int64_t e = 0; e < nnz; e++)
        if (m->colidx[e] < 0 || m->colidx[e] >= cols) return EXAT_ERR_SHAPE;
    return EXAT_OK;
}

template <typename T>
int upload(const std::vector<T> &h, T **d)
{
    const size_t bytes = (h.size() ? h.size() : 1) * sizeof(T);
    if (hipMalloc((void **)d, bytes) != hipSuccess) { *d = nullptr; return EXAT_ERR_ALLOC; }
    if (h.size() && hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return EXAT_ERR_HIP;
    return EXAT_OK;
}

template <int AR, int AT, int BR>
int launch12(const S1Params &p, dim3 grid, size_t lds, hipStream_t st)
{
    // more than 64 KiB of dynamic LDS has to be allowed per kernel (once per process is enough: the size is fixed by AT)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_stage1_mode12<AR, AT, BR>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return EXAT_ERR_HIP;
    hipLaunchKernelGGL((k_stage1_mode12<AR, AT, BR>), grid, dim3(256), lds, st, p);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

}  // namespace

struct exat_stage1_s {
    int64_t I, J, K;
    int A1, B1, C1;
    int *Utp = nullptr, *Vtp = nullptr, *Wrp = nullptr, *Wci = nullptr;
    SEnt *Uent = nullptr, *Vent = nullptr;
    float *Wval = nullptr, *Q = nullptr;
    bool timing = false, timing_valid = false;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
};

extern "C" {

int exat_stage1_destroy(exat_stage1_t s)
{
    if (!s) return EXAT_OK;
    void *bufs[] = {s->Utp, s->Vtp, s->Wrp, s->Wci, s->Uent, s->Vent, s->Wval, s->Q};
    for (void *b : bufs)
        if (b) (void)hipFree(b);
    for (auto &e : s->ev)
        if (e) (void)hipEventDestroy(e);
    delete s;
    return EXAT_OK;
}

int exat_stage1_create(exat_stage1_t *out, int64_t I, int64_t J, int64_t K, const exat_csr_t *U, const exat_csr_t *V,
                       const exat_csr_t *W)
{
    if (!out) return EXAT_ERR_NULL;
    *out = nullptr;
    if (I < 1 || J < 1 || K < 1 || I > kMaxExtent1 || J > kMaxExtent1 || K > kMaxExtent1) return EXAT_ERR_SHAPE;
    int rc;
    if ((rc = check_csr(U, I, S1_MAXROWS)) != EXAT_OK) return rc;
    if ((rc = check_csr(V, J, S1_MAXROWS)) != EXAT_OK) return rc;
    if ((rc = check_csr(W, K, 65535)) != EXAT_OK) return rc;
    exat_stage1_s *s = new (std::nothrow) exat_stage1_s;
    if (!s) return EXAT_ERR_ALLOC;
    s->I = I; s->J = J; s->K = K;
    s->A1 = U->rows; s->B1 = V->rows; s->C1 = W->rows;
    try {
        std::vector<int> tp;
        std::vector<SEnt> ent;
        if (!tile_csr(*U, S1_IT, tp, ent)) { exat_stage1_destroy(s); return EXAT_ERR_SHAPE; }
        if ((rc = upload(tp, &s->Utp)) == EXAT_OK) rc = upload(ent, &s->Uent);
        if (rc == EXAT_OK) {
            if (!tile_csr(*V, S1_JT, tp, ent)) { exat_stage1_destroy(s); return EXAT_ERR_SHAPE; }
            if ((rc = upload(tp, &s->Vtp)) == EXAT_OK) rc = upload(ent, &s->Vent);
        }
        if (rc == EXAT_OK) {
            const int64_t nnz = W->rowptr[W->rows];
            std::vector<int> rp(W->rows + 1), ci(W->colidx, W->colidx + nnz);
            for (int r = 0; r <= W->rows; r++) rp[r] = (int)W->rowptr[r];
            std::vector<float> val(W->val, W->val + nnz);
            if ((rc = upload(rp, &s->Wrp)) == EXAT_OK && (rc = upload(ci, &s->Wci)) == EXAT_OK) rc = upload(val, &s->Wval);
        }
    } catch (const std::bad_alloc &) {
        rc = EXAT_ERR_ALLOC;
    }
    if (rc == EXAT_OK && hipMalloc((void **)&s->Q, (size_t)K * s->A1 * s->B1 * sizeof(float)) != hipSuccess) {
        s->Q = nullptr;
        rc = EXAT_ERR_ALLOC;
    }
    if (rc != EXAT_OK) { exat_stage1_destroy(s); return rc; }
    *out = s;
    return EXAT_OK;
}

int exat_stage1_dims(exat_stage1_t s, int32_t *A1, int32_t *B1, int32_t *C1)
{
    if (!s || !A1 || !B1 || !C1) return EXAT_ERR_NULL;
    *A1 = s->A1; *B1 = s->B1; *C1 = s->C1;
    return EXAT_OK;
}

int exat_stage1_apply(exat_stage1_t s, const float *X, float *X1, void *stream)
{
    if (!s || !X || !X1) return EXAT_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    S1Params p;
    p.X = X; p.I = s->I; p.J = s->J; p.K = s->K; p.A1 = s->A1; p.B1 = s->B1;
    p.Utp = s->Utp; p.Uent = s->Uent; p.Vtp = s->Vtp; p.Vent = s->Vent; p.Q = s->Q;
    const int AT = s->A1 > 64 ? 2 : 1;
    const size_t lds = (size_t)(S1_JT * S1_XS + S1_JT * (64 * AT + 1)) * sizeof(float);
    const dim3 grid((unsigned)s->K);
    if (s->timing && hipEventRecord(s->ev[0], st) != hipSuccess) return EXAT_ERR_HIP;
    int rc;
    if (s->A1 <= 64 && s->B1 <= 64) rc = launch12<16, 1, 16>(p, grid, lds, st);
    else if (s->A1 <= 64) rc = launch12<16, 1, 32>(p, grid, lds, st);
    else if (s->B1 <= 64) rc = launch12<32, 2, 16>(p, grid, lds, st);
    else rc = launch12<32, 2, 32>(p, grid, lds, st);
    if (rc != EXAT_OK) return rc;
    if (s->timing && hipEventRecord(s->ev[1], st) != hipSuccess) return EXAT_ERR_HIP;
    S1Mode3Params m;
    m.Q = s->Q; m.rp = s->Wrp; m.ci = s->Wci; m.val = s->Wval; m.X1 = X1; m.AB = (int64_t)s->A1 * s->B1;
    hipLaunchKernelGGL(k_stage1_mode3, dim3((unsigned)((m.AB + 255) / 256), (unsigned)s->C1), dim3(256), 0, st, m);
    if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    if (s->timing) {
        if (hipEventRecord(s->ev[2], st) != hipSuccess) return EXAT_ERR_HIP;
        s->timing_valid = true;
    }
    return EXAT_OK;
}

int exat_stage1_set_timing(exat_stage1_t s, int enable)
{
    if (!s) return EXAT_ERR_NULL;
    if (enable && !s->ev[0])
        for (auto &e : s->ev)
            if (hipEventCreate(&e) != hipSuccess) return EXAT_ERR_HIP;
    s->timing = enable != 0;
    s->timing_valid = false;
    return EXAT_OK;
}

int exat_stage1_last_timing(exat_stage1_t s, float *ms_mode12, float *ms_mode3)
{
    if (!s || !ms_mode12 || !ms_mode3) return EXAT_ERR_NULL;
    if (!s->timing || !s->timing_valid) return EXAT_ERR_STATE;
    if (hipEventSynchronize(s->ev[2]) != hipSuccess) return EXAT_ERR_HIP;
    if (hipEventElapsedTime(ms_mode12, s->ev[0], s->ev[1]) != hipSuccess) return EXAT_ERR_HIP;
    if (hipEventElapsedTime(ms_mode3, s->ev[1], s->ev[2]) != hipSuccess) return EXAT_ERR_HIP;
    return EXAT_OK;
}

}  // extern "C"
