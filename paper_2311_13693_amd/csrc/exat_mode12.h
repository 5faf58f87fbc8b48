// Fused mode-1 + mode-2 kernel of the compression chain (paper Sec. 4.3: "compress each
// dimension respectively"), for all replicas at once.
//
// One workgroup owns one frontal slice k of the (sub-box of the) tensor and one group of
// ROWS stacked rows q = p*L + l of the stacked mode-1 operand [U_1; ...; U_P] (the stacked
// matrix of Eq. 4).  It walks the slice in column chunks of COLS = 32*CT fibres; for each
// chunk it
//   mode 1:  Z[q, j] = sum_i U[q, i] X[i, j, k]   over the whole i extent (MFMA, fp32 acc),
//            X tiles of 32 x COLS staged through LDS (loaded from HBM, or generated on chip),
//   mode 2:  Q[q, m] += sum_{j in chunk} Z[q, j] V_{p(q)}[m, j]   (fp32 MFMA on the
//            LDS-transposed Z; rows of a 32-row tile that belong to different replicas are
//            multiplied by their own V_p and selected by row),
// and keeps Q (ROWS x M, this slice) in HBM/L2 between chunks.  Because the i reduction is
// complete before mode 2 runs, mode 2 is executed exactly once per (q, j, k): no work is
// repeated per block.  Mode 3 (over k) is a separate small kernel.
#pragma once
#include "exat_device.h"
#include "exat_common.h"
#include "exat_mode2.h"

namespace exat {

template <typename T, int RT, int CT>
struct Mode12Cfg {
    static constexpr int ROWS = 128 * RT;
    static constexpr int COLS = 32 * CT;
    static constexpr int EI = 32;                            // i extent of one LDS stage
    static constexpr int E16 = elem<T>::per16;               // elements per 16-byte fragment
    static constexpr int FPR = EI / E16;                     // fragments per tile row
    static constexpr int ROWB = EI * (int)sizeof(T) + 16;    // LDS row stride in bytes (odd multiple of 16)
    static constexpr int ZST = COLS + 4;                     // floats per row of the transposed Z tile
    static constexpr int STAGE_BYTES = (ROWS + COLS) * ROWB;
    static constexpr int EPI_BYTES = 4 * 32 * ZST * 4;
    static constexpr int LDS_BYTES = STAGE_BYTES > EPI_BYTES ? STAGE_BYTES : EPI_BYTES;
};

// Slow, fully guarded staging of the X tile straight into LDS (box edges, unaligned tensors).
template <typename T, int COLS, int ROWB>
__device__ __forceinline__ void stage_x_guarded(const Mode12Params &p, unsigned char *Xs, int64_t ib, int64_t jc, int64_t k, int tid)
{
    const T *Xp = (const T *)p.X;
    for (int pc = tid; pc < COLS * 32; pc += 256) {
        const int c = pc >> 5, e = pc & 31;
        const int64_t j = jc + c, i = ib + e;
        T v = elem<T>::from_f32(0.0f);
        if (j >= p.j0 && j < p.j1 && i >= p.i0 && i < p.i1)
            v = Xp[(i - p.xo_i) + (j - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk];
        ((T *)(Xs + c * ROWB))[e] = v;
    }
}

// On-chip generation of 16 consecutive i of one fibre (j,k):
//   X = sum_r A[i,r] B[j,r] C[k,r] + sigma g(seed;i,j,k), zero outside the box.
// Indices are clamped for the loads and the result is masked, so there are no branches.
template <bool TAIL>
__device__ __forceinline__ void gen_run16(const Mode12Params &p, int64_t i, int64_t j, int64_t k, float x[16])
{
    const bool colok = (j >= p.j0) && (j < p.j1);
    const int64_t jj = colok ? j : p.j0;
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = 0.0f;
    const float *bp = p.B + jj, *cp = p.C + k;
    if (!TAIL) {
        const float *ap = p.A + i;
        for (int r = 0; r < p.R; r++) {
            const float bc = bp[p.ldB * r] * cp[p.ldC * r];
            const f32x4 *a4 = (const f32x4 *)(ap + p.ldA * r);
            if (p.a_vec) {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const f32x4 av = a4[q];
#pragma unroll
                    for (int e = 0; e < 4; e++) x[4 * q + e] = __builtin_fmaf(av[e], bc, x[4 * q + e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = __builtin_fmaf(ap[p.ldA * r + e], bc, x[e]);
            }
        }
    } else {
        for (int r = 0; r < p.R; r++) {
            const float bc = bp[p.ldB * r] * cp[p.ldC * r];
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int64_t ii = (i + e < p.I) ? i + e : p.I - 1;
                x[e] = __builtin_fmaf(p.A[ii + p.ldA * r], bc, x[e]);
            }
        }
    }
    if (p.amp2_ln2 != 0.0f) {
        const uint32_t ck = fibre_key(p.skey, (uint32_t)jj, (uint32_t)k);
#pragma unroll
        for (int q = 0; q < 4; q++) {
            float z[4];
            noise_quad(ck, (uint32_t)(i >> 2) + q, p.amp2_ln2, z);
#pragma unroll
            for (int e = 0; e < 4; e++) x[4 * q + e] += z[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 16; e++)
        if (!colok || i + e < p.i0 || i + e >= p.i1) x[e] = 0.0f;
}

template <typename T, int RT, int CT, int SRC>
__global__ __launch_bounds__(256) void k_mode12(const Mode12Params p)
{
    typedef Mode12Cfg<T, RT, CT> cfg;
    typedef typename mma_frag<T>::type frag_t;
    constexpr int ROWS = cfg::ROWS, COLS = cfg::COLS, EI = cfg::EI, E16 = cfg::E16, FPR = cfg::FPR,
                  ROWB = cfg::ROWB, ZST = cfg::ZST;
    constexpr int UPT = ROWS * FPR / 256;  // 16-byte pieces of the U tile per thread
    constexpr int XPT = COLS * FPR / 256;  // 16-byte pieces of the X tile per thread (materialised)
    constexpr int GPT = COLS * 2 / 256;    // 16-element runs of the X tile per thread (generated)
    static_assert(ROWS * FPR % 256 == 0 && COLS * FPR % 256 == 0 && COLS * 2 % 256 == 0, "tile/thread mismatch");
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *Us = smem;
    unsigned char *Xs = smem + ROWS * ROWB;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    // unit decode: consecutive workgroup ids go round-robin over the 8 XCDs, so the G row
    // groups that read the same slice k land on the same XCD (and share its L2).
    const int nk = (int)(p.k1 - p.k0);
    const int bid = blockIdx.x, xcd = bid & 7, t = bid >> 3;
    const int g = t % p.G, kidx = (t / p.G) * 8 + xcd;
    if (kidx >= nk) return;
    const int64_t k = p.k0 + kidx;
    const int row0 = g * ROWS;
    const int wrow0 = row0 + wave * (RT * 32);
    const int64_t ia0 = p.i0 & ~(int64_t)(EI - 1);
    const int nstage = (int)((p.i1 - ia0 + EI - 1) / EI);
    const int64_t ja0 = (p.j0 / COLS) * COLS;

    // per-thread piece coordinates (tile row/column r, 16-byte fragment f); piece u is r + u*(256/FPR)
    const int pr0 = tid / FPR, pf = tid % FPR;
    const unsigned u_voff = (unsigned)pr0 * (unsigned)p.Ipad + (unsigned)pf * E16;  // elements, < 2^31 by the plan's limits
    const unsigned u_vstep = (unsigned)(256 / FPR) * (unsigned)p.Ipad;
    const T *Ug = (const T *)p.U + (int64_t)row0 * p.Ipad;  // + ib: uniform
    unsigned char *us_w = Us + pr0 * ROWB + pf * 16;         // + u*(256/FPR)*ROWB
    unsigned char *xs_w = Xs + pr0 * ROWB + pf * 16;
    const unsigned char *us_r = Us + (wave * (RT * 32) + l32) * ROWB + hi * 16;  // + rt*32*ROWB + g2*32
    const unsigned char *xs_r = Xs + l32 * ROWB + hi * 16;                       // + ct*32*ROWB + g2*32

    u32x4 upre[UPT];               // next stage of U, in flight from global memory
    u32x4 xpre[SRC == SRC_MATERIALISED ? XPT : 1];
    float xgen[SRC == SRC_GENERATED ? GPT : 1][16];

    for (int64_t jc = ja0; jc < p.j1; jc += COLS) {
        f32x16 acc[RT][CT];
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < CT; ct++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[rt][ct][e] = 0.0f;

        const bool jfull = (jc >= p.j0) && (jc + COLS <= p.j1);
        // materialised source: per-thread element offset of piece 0 of this chunk inside X
        const int64_t x_off = (pf * E16 - p.xo_i) + (jc + pr0 - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk;
        const int64_t x_step = (int64_t)(256 / FPR) * p.x_sj;

        // a stage takes the fast path when the whole 32 x COLS tile lies inside the box
        auto is_fast = [&](int s) -> bool {
            const int64_t ib = ia0 + (int64_t)s * EI;
            if (SRC == SRC_MATERIALISED) return p.x_vec && jfull && ib >= p.i0 && ib + EI <= p.i1;
            return ib + EI <= p.I;
        };
        // fetches (or generates) the operands of stage s into registers
        auto fetch = [&](int s) {
            const int64_t ib = ia0 + (int64_t)s * EI;
            const T *ub = Ug + ib;
#pragma unroll
            for (int u = 0; u < UPT; u++) upre[u] = *(const u32x4 *)(ub + (u_voff + u * u_vstep));
            if constexpr (SRC == SRC_MATERIALISED) {
                if (is_fast(s)) {
                    const T *xb = (const T *)p.X + ib;
#pragma unroll
                    for (int u = 0; u < XPT; u++) xpre[u] = *(const u32x4 *)(xb + (x_off + u * x_step));
                }
            } else {
#pragma unroll
                for (int u = 0; u < GPT; u++) {
                    const int pc = tid + u * 256, c = pc >> 1, h = pc & 1;
                    if (is_fast(s)) gen_run16<false>(p, ib + 16 * h, jc + c, k, xgen[u]);
                    else gen_run16<true>(p, ib + 16 * h, jc + c, k, xgen[u]);
                }
            }
        };
        // writes the fetched stage into the LDS tiles
        auto commit = [&](int s) {
#pragma unroll
            for (int u = 0; u < UPT; u++) *(u32x4 *)(us_w + u * (256 / FPR) * ROWB) = upre[u];
            if constexpr (SRC == SRC_MATERIALISED) {
                if (is_fast(s)) {
#pragma unroll
                    for (int u = 0; u < XPT; u++) *(u32x4 *)(xs_w + u * (256 / FPR) * ROWB) = xpre[u];
                } else {
                    stage_x_guarded<T, COLS, ROWB>(p, Xs, ia0 + (int64_t)s * EI, jc, k, tid);
                }
            } else {
#pragma unroll
                for (int u = 0; u < GPT; u++) {
                    const int pc = tid + u * 256, c = pc >> 1, h = pc & 1;
                    T *dst = (T *)(Xs + c * ROWB) + 16 * h;
#pragma unroll
                    for (int e = 0; e < 16; e++) dst[e] = elem<T>::from_f32(xgen[u][e]);
                }
            }
        };

        fetch(0);
        for (int s = 0; s < nstage; s++) {
            __syncthreads();  // the previous stage's MFMAs (or the epilogue) are done with the LDS
            commit(s);
            __syncthreads();
            if (s + 1 < nstage) fetch(s + 1);  // in flight while the MFMAs below run
            // ---- mode-1 MFMAs on the staged tiles ----
            // Both operands use the same lane -> i assignment (fragment 2*g2 + hi of the row),
            // so the order in which the 32 i of the stage are consumed is irrelevant.
            // Fragments are double-buffered in registers: the LDS reads of step g2+1 are issued
            // before the MFMAs of step g2, and the scheduling barriers keep them from moving further.
            frag_t a[2][RT], bx[2][CT];
#pragma unroll
            for (int rt = 0; rt < RT; rt++) a[0][rt] = *(const frag_t *)(us_r + rt * 32 * ROWB);
#pragma unroll
            for (int ct = 0; ct < CT; ct++) bx[0][ct] = *(const frag_t *)(xs_r + ct * 32 * ROWB);
#pragma unroll
            for (int g2 = 0; g2 < FPR / 2; g2++) {
                __builtin_amdgcn_sched_barrier(0);
                if (g2 + 1 < FPR / 2) {
#pragma unroll
                    for (int rt = 0; rt < RT; rt++) a[(g2 + 1) & 1][rt] = *(const frag_t *)(us_r + rt * 32 * ROWB + (g2 + 1) * 32);
#pragma unroll
                    for (int ct = 0; ct < CT; ct++) bx[(g2 + 1) & 1][ct] = *(const frag_t *)(xs_r + ct * 32 * ROWB + (g2 + 1) * 32);
                }
#pragma unroll
                for (int rt = 0; rt < RT; rt++)
#pragma unroll
                    for (int ct = 0; ct < CT; ct++) mma_frag<T>::mma(acc[rt][ct], a[g2 & 1][rt], bx[g2 & 1][ct]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- mode 2 on the finished Z chunk ----
        __syncthreads();  // staging LDS is free now
        float *Zs = (float *)smem + wave * (32 * ZST);
        const bool first_chunk = (jc == ja0);
        if (p.MT == 2) mode2_chunk<RT, CT, 2, VM_F32, 4>(p, nullptr, Zs, acc, wrow0, kidx, jc, first_chunk, lane);
        else mode2_chunk<RT, CT, 1, VM_F32, 4>(p, nullptr, Zs, acc, wrow0, kidx, jc, first_chunk, lane);
    }
}

}  // namespace exat
