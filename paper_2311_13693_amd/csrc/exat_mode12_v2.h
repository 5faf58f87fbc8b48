// Fused mode-1 + mode-2 kernel, software-pipelined variant with the U tile staged through LDS.  The host uses
// it for the fp32 generated source (two waves per SIMD); every other aligned case runs k_mode12_v3, which
// includes this header for the pieces the two share (generator operand splitting, geometry).
//
// Same decomposition as k_mode12 (one workgroup = one slice k x one group of ROWS stacked rows,
// full i reduction per 128-fibre column chunk, mode 2 on the finished Z chunk), with
//   * two LDS stage buffers of 64-byte tile rows (16 fp32 or 32 bf16 values of i), so that a
//     stage costs one barrier and the next stage is written while the current one is multiplied;
//   * U tiles prefetched from L2 into registers one stage ahead;
//   * for the generated source, the low-rank part of the X tile produced by MFMA instead of
//     vector FMAs: X[i, j] = sum_r A[i,r] (B[j,r] C[k,r]) is a (32 x R)(R x 128) product per
//     stage.  To keep fp32 accuracy on the bf16 matrix cores both operands are split into
//     16-bit pieces (a = a_h + a_m; see gen_piece) and the three significant cross terms are accumulated in
//     fp32: 6 terms (error ~2^-23) on the fp32 path, 3 terms (error ~2^-16, below the bf16
//     rounding of the tile) on the bf16 path.  The noise term is added to the accumulator
//     layout directly: each lane holds aligned quads of 4 consecutive i, the unit of the
//     counter-based generator.
#pragma once
#include "exat_mode12.h"
#include "exat_mode2.h"


namespace exat {

struct GenSplitParams {
    const __bf16 *Asp;  // [NV][Irows][Rpad] bf16 pieces of A, zero padded (rows >= I and columns >= R)
    int64_t Irows;
    int Rpad;
};

// MFMA 16x16x32 bf16: A lane (row l%16, k 8*(l/16)+e), B lane (col l%16, k 8*(l/16)+e),
// C lane (col l%16, rows 4*(l/16)+r).
typedef float f32x4v __attribute__((ext_vector_type(4)));
#ifndef V2_VB
#define V2_VB 4
#endif

template <typename T> struct v2geom;
template <> struct v2geom<float> { static constexpr int EI = 16, NV = 2, NTERM = 3, SUBI = 1; };
template <> struct v2geom<__bf16> { static constexpr int EI = 32, NV = 2, NTERM = 3, SUBI = 2; };

template <int NW, int RT>
struct Mode12V2Cfg {
    static constexpr int ROWS = 32 * NW * RT, COLS = 128, ROWB = 80;
    static constexpr int BUF_BYTES = (ROWS + COLS) * ROWB;
    static constexpr int ZST = COLS + 4;
    static constexpr int EPI_BYTES = NW * 32 * ZST * 4;
    static constexpr int LDS_BYTES = 2 * BUF_BYTES > EPI_BYTES ? 2 * BUF_BYTES : EPI_BYTES;
};

// The generator's low-rank product runs on the 16x16x32 matrix instruction with every operand value taken as
// the sum of two 16-bit pieces, v = h + m, and the three significant cross terms accumulated in fp32.
// bf16 plans: bf16 pieces (16 significand bits together, below the bf16 rounding of the tile).
// fp32 plans: fp16 pieces (22 significand bits together; the dropped term is 2^-22 of a product; the factors and
// their products are O(1..100), far inside the fp16 range).  Pieces travel as raw 16-bit patterns in bf16x8
// registers whatever their format.
template <typename T> struct gen_piece;
template <> struct gen_piece<__bf16> {
    static constexpr int FMT = 0;
    __device__ static __forceinline__ void split(float v, __bf16 &h, __bf16 &m)
    {
        h = (__bf16)v;
        m = (__bf16)(v - (float)h);
    }
    __device__ static __forceinline__ f32x4v mfma(const bf16x8 &a, const bf16x8 &b, const f32x4v &c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct gen_piece<float> {
    static constexpr int FMT = 1;
    __device__ static __forceinline__ void split(float v, __bf16 &h, __bf16 &m)
    {
        const _Float16 fh = (_Float16)v;
        const _Float16 fm = (_Float16)(v - (float)fh);
        h = __builtin_bit_cast(__bf16, fh);
        m = __builtin_bit_cast(__bf16, fm);
    }
    __device__ static __forceinline__ f32x4v mfma(const bf16x8 &a, const bf16x8 &b, const f32x4v &c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// BOXED: the box is a proper sub-range in i, so elements outside [i0,i1) must be forced to zero
// (for the full extent the zero padding of U already removes them).
template <typename T, int NW, int RT, int SRC, int KS, bool BOXED>
__global__ __launch_bounds__(64 * NW) void k_mode12_v2(const Mode12Params p, const GenSplitParams gs)
{
    typedef Mode12V2Cfg<NW, RT> cfg;
    typedef typename mma_frag<T>::type frag_t;
    constexpr int CT = 4, ROWS = cfg::ROWS, COLS = cfg::COLS, ROWB = cfg::ROWB, ZST = cfg::ZST;
    constexpr int EI = v2geom<T>::EI, NV = v2geom<T>::NV, SUBI = v2geom<T>::SUBI;
    constexpr int E16 = elem<T>::per16;
    constexpr int NT = 64 * NW;         // threads
    constexpr int PSTEP = NT / 4;       // tile rows covered by one round of 16-byte pieces
    constexpr int UPT = ROWS * 4 / NT;  // 16-byte pieces of the U tile per thread
    constexpr int XPT = COLS * 4 / NT;  // 16-byte pieces of the X tile per thread (materialised)
    constexpr int NSJ = 8 / NW;         // 16-column sub-tiles of the generated tile per wave
    constexpr int WCOLS = COLS / NW;    // columns of the generated tile owned by one wave
    extern __shared__ __align__(16) unsigned char smem[];

    // the wave index is the same for all lanes of a wave: say so, which keeps everything derived from it scalar
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int l16 = lane & 15, q16 = lane >> 4;
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

    const int pr0 = tid >> 2, pf = tid & 3;  // piece coordinates: tile row, 16-byte fragment
    const unsigned u_voff = (unsigned)pr0 * (unsigned)p.Ipad + (unsigned)pf * E16;
    const unsigned u_vstep = (unsigned)PSTEP * (unsigned)p.Ipad;
    const T *Ug = (const T *)p.U + (int64_t)row0 * p.Ipad;
    const int us_w = pr0 * ROWB + pf * 16;                              // + u*PSTEP*ROWB
    const int xs_w = ROWS * ROWB + pr0 * ROWB + pf * 16;
    const int us_r = (wave * (RT * 32) + l32) * ROWB + hi * 16;         // + rt*32*ROWB + g2*32
    const int xs_r = ROWS * ROWB + l32 * ROWB + hi * 16;                // + ct*32*ROWB + g2*32
    // generated tile: this wave owns columns [WCOLS*wave, WCOLS*(wave+1)) of the chunk; a lane holds, for
    // sj < NSJ and si < SUBI, the quad of rows 16*si + 4*q16 .. +3 of column WCOLS*wave + 16*sj + l16
    const int xg_w = ROWS * ROWB + (WCOLS * wave + l16) * ROWB + (4 * q16) * (int)sizeof(T);  // + sj*16*ROWB + si*16*sizeof(T)

    u32x4 upre[UPT];
    u32x4 xpre[SRC == SRC_MATERIALISED ? XPT : 1];
    bf16x8 afrag[SRC == SRC_GENERATED ? NV * KS * SUBI : 1];
    bf16x8 bfrag[SRC == SRC_GENERATED ? NV * KS * NSJ : 1];
    f32x4v accx[SRC == SRC_GENERATED ? SUBI * NSJ : 1];
    uint32_t ckey[NSJ];
    float amp[NSJ];

    for (int64_t jc = ja0; jc < p.j1; jc += COLS) {
        f32x16 acc[RT][CT];
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < CT; ct++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[rt][ct][e] = 0.0f;

        // ---- per-chunk set-up ----
        int64_t x_off[XPT];
        bool x_ok[XPT];
        if constexpr (SRC == SRC_MATERIALISED) {
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                const int64_t j = jc + pr0 + PSTEP * u;
                x_ok[u] = (j >= p.j0) && (j < p.j1);
                x_off[u] = (pf * E16 - p.xo_i) + (j - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk;
            }
        } else {
            // B operand of the generator: bc[j, r] = B[j,r] C[k,r] for this lane's two columns, split in bf16 pieces
#pragma unroll
            for (int sj = 0; sj < NSJ; sj++) {
                const int64_t j = jc + WCOLS * wave + 16 * sj + l16;
                const bool colok = (j >= p.j0) && (j < p.j1);
                const int64_t jj = colok ? j : p.j0;
                ckey[sj] = fibre_key(p.skey, (uint32_t)jj, (uint32_t)k);
                amp[sj] = colok ? p.amp2_ln2 : 0.0f;
#pragma unroll
                for (int ks = 0; ks < KS; ks++) {
                    bf16x8 bh, bm;
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        // clamped, unconditional loads (no branch per element), masked afterwards
                        const int r = 32 * ks + 8 * q16 + e, rr = r < p.R ? r : p.R - 1;
                        float bc = *(p.B + jj + p.ldB * rr) * *(p.C + k + p.ldC * rr);
                        bc = (colok && r < p.R) ? bc : 0.0f;
                        __bf16 h, m;
                        gen_piece<T>::split(bc, h, m);
                        bh[e] = h; bm[e] = m;
                    }
                    bfrag[(0 * KS + ks) * NSJ + sj] = bh;
                    bfrag[(1 * KS + ks) * NSJ + sj] = bm;
                }
            }
        }

        auto stage_i = [&](int s) -> int64_t { return ia0 + (int64_t)(s < nstage ? s : nstage - 1) * EI; };
        auto load_u = [&](int s) {
            const T *ub = Ug + stage_i(s);
#pragma unroll
            for (int u = 0; u < UPT; u++) upre[u] = *((const u32x4 *)(ub + (u_voff + u * u_vstep)));
        };
        auto load_x = [&](int s) {
            if constexpr (SRC == SRC_MATERIALISED) {
                const T *xb = (const T *)p.X + stage_i(s);
#pragma unroll
                for (int u = 0; u < XPT; u++) {
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (x_ok[u]) v = *(const u32x4 *)(xb + x_off[u]);
                    xpre[u] = v;
                }
            }
        };
        auto load_a = [&](int s) {
            if constexpr (SRC == SRC_GENERATED) {
                const int64_t ib = stage_i(s);
#pragma unroll
                for (int v = 0; v < NV; v++)
#pragma unroll
                    for (int ks = 0; ks < KS; ks++)
#pragma unroll
                        for (int si = 0; si < SUBI; si++)
                            afrag[(v * KS + ks) * SUBI + si] = *((const bf16x8 *)(gs.Asp + ((int64_t)v * gs.Irows + ib + 16 * si + l16) * gs.Rpad + 32 * ks + 8 * q16));
            }
        };
        // low-rank part of the tile of the stage whose A fragments are loaded: accx = A_tile * bc^T
        auto gen_x = [&]() {
            if constexpr (SRC == SRC_GENERATED) {
#pragma unroll
                for (int si = 0; si < SUBI; si++)
#pragma unroll
                    for (int sj = 0; sj < NSJ; sj++) {
                        f32x4v c = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                        for (int ks = 0; ks < KS; ks++) {
                            const bf16x8 ah = afrag[(0 * KS + ks) * SUBI + si], am = afrag[(1 * KS + ks) * SUBI + si];
                            const bf16x8 bh = bfrag[(0 * KS + ks) * NSJ + sj], bm = bfrag[(1 * KS + ks) * NSJ + sj];
                            // smallest terms first
                            c = gen_piece<T>::mfma(am, bh, c);
                            c = gen_piece<T>::mfma(ah, bm, c);
                            c = gen_piece<T>::mfma(ah, bh, c);
                        }
                        accx[si * NSJ + sj] = c;
                    }
            }
        };
        // writes the stage held in registers (U, and X loaded or generated) into LDS buffer `buf`
        auto commit = [&](int s, int buf) {
            unsigned char *base = smem + buf * cfg::BUF_BYTES;
#pragma unroll
            for (int u = 0; u < UPT; u++) *(u32x4 *)(base + us_w + u * PSTEP * ROWB) = upre[u];
            if constexpr (SRC == SRC_MATERIALISED) {
#pragma unroll
                for (int u = 0; u < XPT; u++) *(u32x4 *)(base + xs_w + u * PSTEP * ROWB) = xpre[u];
            } else {
                const int64_t ib = stage_i(s);
#pragma unroll
                for (int si = 0; si < SUBI; si++)
#pragma unroll
                    for (int sj = 0; sj < NSJ; sj++) {
                        const int64_t i = ib + 16 * si + 4 * q16;
                        float z[4];
                        noise_quad(ckey[sj], (uint32_t)(i >> 2), amp[sj], z);
                        float x[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            x[e] = accx[si * NSJ + sj][e] + z[e];
                            if (BOXED && (i + e < p.i0 || i + e >= p.i1)) x[e] = 0.0f;
                        }
                        unsigned char *dst = base + xg_w + sj * 16 * ROWB + si * 16 * (int)sizeof(T);
                        if constexpr (sizeof(T) == 4) {
                            f32x4 v = {x[0], x[1], x[2], x[3]};
                            *(f32x4 *)dst = v;
                        } else {
                            bf16x4 v = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
                            *(bf16x4 *)dst = v;
                        }
                    }
            }
        };

        // ---- prologue: stage 0 into buffer 0, stage 1 in registers, A fragments of stage 2 in flight ----
        load_u(0); load_x(0); load_a(0);
        gen_x();
        __syncthreads();  // the previous chunk's epilogue is done with the LDS
        commit(0, 0);
        load_u(1); load_x(1); load_a(1);
        gen_x();
        load_a(2);
        __syncthreads();

        // One iteration = "fill" (write stage s+1 from registers into the other LDS buffer, start the loads of
        // stage s+2, generate the tile of stage s+2: vector + memory work) and "multiply" (MFMAs of stage s from
        // the current buffer).  The two parts touch different LDS buffers and different registers.
        auto fill = [&](int s) {
            commit(s + 1, (s + 1) & 1);
            load_u(s + 2); load_x(s + 2);
            gen_x();        // tile of stage s+2 from the A fragments loaded one iteration ago
            load_a(s + 3);
        };
        auto multiply = [&](int s) {
            const unsigned char *base = smem + (s & 1) * cfg::BUF_BYTES;
            frag_t a[2][RT], bx[2][CT];
#pragma unroll
            for (int rt = 0; rt < RT; rt++) a[0][rt] = *(const frag_t *)(base + us_r + rt * 32 * ROWB);
#pragma unroll
            for (int ct = 0; ct < CT; ct++) bx[0][ct] = *(const frag_t *)(base + xs_r + ct * 32 * ROWB);
#pragma unroll
            for (int rt = 0; rt < RT; rt++) a[1][rt] = *(const frag_t *)(base + us_r + rt * 32 * ROWB + 32);
#pragma unroll
            for (int ct = 0; ct < CT; ct++) bx[1][ct] = *(const frag_t *)(base + xs_r + ct * 32 * ROWB + 32);
#pragma unroll
            for (int g2 = 0; g2 < 2; g2++)
#pragma unroll
                for (int rt = 0; rt < RT; rt++)
#pragma unroll
                    for (int ct = 0; ct < CT; ct++) mma_frag<T>::mma(acc[rt][ct], a[g2][rt], bx[g2][ct]);
        };
        for (int s = 0; s < nstage; s++) {
            fill(s);
            multiply(s);
            __syncthreads();
        }

        // ---- mode 2 on the finished Z chunk ----
        float *Zs = (float *)smem + wave * (32 * ZST);
        const bool first_chunk = (jc == ja0);
        // the generator's registers leave less room for V fragments in flight
        constexpr int VB = SRC == SRC_GENERATED ? V2_VB : 16;
        if (p.MT == 2) mode2_chunk<RT, CT, 2, VM_F32, VB>(p, nullptr, Zs, acc, wrow0, kidx, jc, first_chunk, lane);
        else mode2_chunk<RT, CT, 1, VM_F32, VB>(p, nullptr, Zs, acc, wrow0, kidx, jc, first_chunk, lane);
    }
}

// A (I x R, column-major, fp32) -> the generator's two 16-bit pieces [2][Irows][Rpad] (bf16 pieces for bf16 plans,
// fp16 pieces for fp32 plans), zero padded
template <typename T>
__global__ void k_split_a(const float *A, int64_t I, int R, __bf16 *out, int64_t Irows, int Rpad)
{
    const int64_t n = Irows * Rpad;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = idx / Rpad;
        const int r = (int)(idx % Rpad);
        const float v = (i < I && r < R) ? A[i + I * r] : 0.0f;
        __bf16 h, m;
        gen_piece<T>::split(v, h, m);
        out[idx] = h;
        out[n + idx] = m;
    }
}

}  // namespace exat
