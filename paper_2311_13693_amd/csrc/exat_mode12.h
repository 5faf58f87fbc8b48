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

namespace exat {

struct Mode12Params {
    const void *U;   // packed [PLpad][Ipad] of T, zero padded
    const float *V;  // packed [P][Mpad][Jpad] fp32, zero padded (bf16-rounded values for bf16 plans)
    float *Q;        // [k1-k0][PLpad][Mpad] fp32
    // materialised source: element (i,j,k) at X[(i-xo_i) + (j-xo_j)*x_sj + (k-xo_k)*x_sk]
    const void *X;
    int64_t x_sj, x_sk, xo_i, xo_j, xo_k;
    int x_vec;  // 16-byte loads of X are aligned
    // generated source
    const float *A, *B, *C;
    int64_t ldA, ldB, ldC;
    int R;
    uint32_t skey;
    float amp2_ln2;  // -2 ln2 sigma^2, 0 when sigma == 0
    int64_t I, Ipad, Jpad;
    int L, PL, PLpad, Mpad, MT, G;
    int64_t i0, i1, j0, j1, k0, k1;
};

enum { SRC_MATERIALISED = 0, SRC_GENERATED = 1 };

template <typename T> struct mma_frag;
template <> struct mma_frag<float> {
    typedef f32x4 type;
    __device__ static __forceinline__ void mma(f32x16 &c, const f32x4 &a, const f32x4 &b)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], c, 0, 0, 0);
    }
};
template <> struct mma_frag<__bf16> {
    typedef bf16x8 type;
    __device__ static __forceinline__ void mma(f32x16 &c, const bf16x8 &a, const bf16x8 &b)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

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

template <typename T, int RT, int CT, int SRC>
__global__ __launch_bounds__(256) void k_mode12(const Mode12Params p)
{
    typedef Mode12Cfg<T, RT, CT> cfg;
    typedef typename mma_frag<T>::type frag_t;
    constexpr int ROWS = cfg::ROWS, COLS = cfg::COLS, EI = cfg::EI, E16 = cfg::E16, FPR = cfg::FPR,
                  ROWB = cfg::ROWB, ZST = cfg::ZST;
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
    const T *Up = (const T *)p.U;

    for (int64_t jc = ja0; jc < p.j1; jc += COLS) {
        f32x16 acc[RT][CT];
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < CT; ct++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[rt][ct][e] = 0.0f;

        for (int s = 0; s < nstage; s++) {
            const int64_t ib = ia0 + (int64_t)s * EI;
            __syncthreads();
            // ---- stage the U tile: ROWS x EI, rows contiguous in i ----
            for (int pc = tid; pc < ROWS * FPR; pc += 256) {
                const int r = pc / FPR, f = pc % FPR;
                const uint4 v = *(const uint4 *)(Up + (int64_t)(row0 + r) * p.Ipad + ib + f * E16);
                *(uint4 *)(Us + r * ROWB + f * 16) = v;
            }
            // ---- stage the X tile: COLS fibres x EI ----
            if (SRC == SRC_MATERIALISED) {
                const T *Xp = (const T *)p.X;
                for (int pc = tid; pc < COLS * FPR; pc += 256) {
                    const int c = pc / FPR, f = pc % FPR;
                    const int64_t j = jc + c, i = ib + f * E16;
                    union { uint4 v; T e[E16]; } u;
                    u.v = make_uint4(0, 0, 0, 0);
                    if (j >= p.j0 && j < p.j1) {
                        const T *src = Xp + (i - p.xo_i) + (j - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk;
                        if (p.x_vec && i >= p.i0 && i + E16 <= p.i1) {
                            u.v = *(const uint4 *)src;
                        } else {
#pragma unroll
                            for (int e = 0; e < E16; e++)
                                if (i + e >= p.i0 && i + e < p.i1) u.e[e] = src[e];
                        }
                    }
                    *(uint4 *)(Xs + c * ROWB + f * 16) = u.v;
                }
            } else {
                // on-chip generation: X = sum_r A[i,r] B[j,r] C[k,r] + sigma g(seed;i,j,k)
                for (int pc = tid; pc < COLS * 2; pc += 256) {
                    const int c = pc >> 1, h = pc & 1;
                    const int64_t j = jc + c, i = ib + 16 * h;
                    float x[16];
#pragma unroll
                    for (int e = 0; e < 16; e++) x[e] = 0.0f;
                    if (j >= p.j0 && j < p.j1 && i < p.i1 && i + 16 > p.i0) {
                        if (i + 16 <= p.I) {
                            for (int r = 0; r < p.R; r++) {
                                const float bc = p.B[j + p.ldB * r] * p.C[k + p.ldC * r];
                                const float *a = p.A + i + p.ldA * r;
#pragma unroll
                                for (int e = 0; e < 16; e++) x[e] = __builtin_fmaf(a[e], bc, x[e]);
                            }
                        } else {
                            for (int r = 0; r < p.R; r++) {
                                const float bc = p.B[j + p.ldB * r] * p.C[k + p.ldC * r];
                                const float *a = p.A + i + p.ldA * r;
#pragma unroll
                                for (int e = 0; e < 16; e++)
                                    if (i + e < p.I) x[e] = __builtin_fmaf(a[e], bc, x[e]);
                            }
                        }
                        if (p.amp2_ln2 != 0.0f) {
                            const uint32_t ck = fibre_key(p.skey, (uint32_t)j, (uint32_t)k);
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
                            if (i + e < p.i0 || i + e >= p.i1) x[e] = 0.0f;
                    }
                    T *dst = (T *)(Xs + c * ROWB) + 16 * h;
#pragma unroll
                    for (int e = 0; e < 16; e++) dst[e] = elem<T>::from_f32(x[e]);
                }
            }
            __syncthreads();
            // ---- mode-1 MFMAs on the staged tiles ----
            // Both operands use the same lane -> i assignment (fragment 2*g2 + hi of the row),
            // so the order in which the 32 i of the stage are consumed is irrelevant.
#pragma unroll
            for (int g2 = 0; g2 < FPR / 2; g2++) {
                frag_t a[RT], bx[CT];
#pragma unroll
                for (int rt = 0; rt < RT; rt++)
                    a[rt] = *(const frag_t *)(Us + (wave * (RT * 32) + rt * 32 + l32) * ROWB + (2 * g2 + hi) * 16);
#pragma unroll
                for (int ct = 0; ct < CT; ct++)
                    bx[ct] = *(const frag_t *)(Xs + (ct * 32 + l32) * ROWB + (2 * g2 + hi) * 16);
#pragma unroll
                for (int rt = 0; rt < RT; rt++)
#pragma unroll
                    for (int ct = 0; ct < CT; ct++) mma_frag<T>::mma(acc[rt][ct], a[rt], bx[ct]);
            }
        }

        // ---- mode 2 on the finished Z chunk ----
        __syncthreads();  // staging LDS is free now
        float *Zs = (float *)smem + wave * (32 * ZST);
        const bool first_chunk = (jc == ja0);
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const int q0 = wrow0 + rt * 32;  // wave-uniform
            if (q0 < p.PL) {
                // C layout of the 32x32 MFMA: acc[4b + r] is row 8b + 4*hi + r, column l32
#pragma unroll
                for (int ct = 0; ct < CT; ct++)
#pragma unroll
                    for (int b4 = 0; b4 < 4; b4++)
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            Zs[(8 * b4 + 4 * hi + r) * ZST + ct * 32 + l32] = acc[rt][ct][4 * b4 + r];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int qlast = (q0 + 31 < p.PL - 1) ? q0 + 31 : p.PL - 1;
                const int pfirst = q0 / p.L, plast = qlast / p.L;
                for (int pp = pfirst; pp <= plast; pp++) {
                    f32x16 qa[2];
#pragma unroll
                    for (int mt = 0; mt < 2; mt++)
#pragma unroll
                        for (int e = 0; e < 16; e++) qa[mt][e] = 0.0f;
                    const float *Vp = p.V + (int64_t)pp * p.Mpad * p.Jpad + jc;
#pragma unroll 4
                    for (int g8 = 0; g8 < COLS / 8; g8++) {
                        const f32x4 a = *(const f32x4 *)(Zs + l32 * ZST + 8 * g8 + 4 * hi);
#pragma unroll
                        for (int mt = 0; mt < 2; mt++) {
                            if (mt < p.MT) {
                                const f32x4 bv = *(const f32x4 *)(Vp + (int64_t)(mt * 32 + l32) * p.Jpad + 8 * g8 + 4 * hi);
                                mma_frag<float>::mma(qa[mt], a, bv);
                            }
                        }
                    }
                    const int rlo = pp * p.L, rhi = rlo + p.L;  // rows of replica pp
#pragma unroll
                    for (int mt = 0; mt < 2; mt++) {
                        if (mt < p.MT) {
#pragma unroll
                            for (int b4 = 0; b4 < 4; b4++)
#pragma unroll
                                for (int r = 0; r < 4; r++) {
                                    const int row = q0 + 8 * b4 + 4 * hi + r;
                                    if (row >= rlo && row < rhi) {
                                        float *dst = p.Q + ((int64_t)kidx * p.PLpad + row) * p.Mpad + mt * 32 + l32;
                                        float v = qa[mt][4 * b4 + r];
                                        if (!first_chunk) v += *dst;
                                        *dst = v;
                                    }
                                }
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
}

}  // namespace exat
