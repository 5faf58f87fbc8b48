// Fused mode-1 + mode-2 kernel for fp32 data on the fp16 matrix cores (the residual split of the paper's Eq. 5).
//
// X and the stacked U stay fp32 in memory.  Every operand element is taken as the sum of two fp16 pieces,
// x = x_h + x_l with x_h = fl16(x), x_l = fl16(x - x_h) (22 significand bits together), and a product u*x as the
// three cross terms u_h x_h + u_h x_l + u_l x_h accumulated in fp32; the dropped term u_l x_l is 2^-22 of the
// product.  (The X tile is split on the fly with the packed round-toward-zero conversion, x_h = rtz16(x),
// x_l = rtz16(x - x_h): x - x_h is exact, and the pair still carries 21 bits.)  One 32x32x16 block then costs three fp16 MFMAs (96 clk) instead of eight fp32 MFMAs (512 clk).
// Magnitudes must stay inside the fp16 range (|x|, |u|, |Z| < 65504); pieces below 2^-24 are lost.
//
// Same decomposition, tile shape and fragment-ordered U as k_mode12_v3 (materialised source only): U is split
// once at operand preparation (two fragment arrays), the X tile is split when it moves from registers to LDS
// (two tiles of 64-byte rows per stage), the finished Z tile and V_p are split in the mode-2 phase.
#pragma once
#include "exat_mode12_v3.h"

namespace exat {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

struct SplitParams {
    const _Float16 *Ufh, *Ufl;  // high / low pieces of U, [PLpad/32][nig][64 lanes][8]: lane l of fragment (rt, ig)
                                // holds row 32*rt + l%32, i = 16*ig + 8*(l/32) .. +7
    int64_t nig;                // Ipad / 16
    const _Float16 *Vfh, *Vfl;  // high / low pieces of V, [P][Jpad/16][2][64 lanes][8] (see mode2_chunk)
};

template <int NW, int RT>
struct Mode12SplitCfg {
    static constexpr int ROWS = 32 * NW * RT, COLS = 128, ROWB = 80;
    static constexpr int XBUF_BYTES = COLS * ROWB;        // one piece of one stage
    static constexpr int STAGE_BYTES = 2 * XBUF_BYTES;    // high tile, low tile
    static constexpr int ZST = COLS + 4;
    static constexpr int EPI_BYTES = NW * 32 * ZST * 4;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES > EPI_BYTES ? 2 * STAGE_BYTES : EPI_BYTES;
};

// DU: register sets of U fragments, DX: register sets of the X tile (as in k_mode12_v3)
// TAB: X is a slab of separate blocks addressed through Mode12Params::xtab, as in k_mode12_v3.
template <int NW, int RT, int DU, int DX, bool TAB = false>
__global__ __launch_bounds__(64 * NW) void k_mode12_split(const Mode12Params p, const SplitParams sp)
{
    typedef Mode12SplitCfg<NW, RT> cfg;
    constexpr int CT = 4, ROWS = cfg::ROWS, COLS = cfg::COLS, ROWB = cfg::ROWB, ZST = cfg::ZST, XBUF = cfg::XBUF_BYTES, STAGE = cfg::STAGE_BYTES;
    constexpr int EI = 32, GI = 16;            // i per stage, i per U fragment
    constexpr int NT = 64 * NW, PCOLS = NT / 4, XPT = COLS / PCOLS;  // 4 threads x 8 floats cover the 32 i of one column
    constexpr int NMAIN = 2 * RT * CT;
    constexpr int UNR = lcm_i(lcm_i(2, DU), DX);
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nk = (int)(p.k1 - p.k0);
    const int bid = blockIdx.x, xcd = bid & 7, t = bid >> 3;
    // the row groups of one slice sit next to each other on one XCD and share the X tiles through its L2
    const int g = t % p.G, kidx = (t / p.G) * 8 + xcd;
    if (kidx >= nk) return;
    const int64_t k = p.k0 + kidx;
    const int row0 = p.row_base + g * ROWS;
    const int wrow0 = row0 + wave * (RT * 32);
    const int64_t ia0 = p.i0 & ~(int64_t)(EI - 1);
    const int nstage = (int)((p.i1 - ia0 + EI - 1) / EI);
    const int64_t ja0 = (p.j0 / COLS) * COLS;
    const int64_t u_rt_step = sp.nig * (64 * 8);

    f16x8 uh[DU][RT][2], ul[DU][RT][2];
    f32x4 xpre[DX][2 * XPT];

    for (int64_t jc = ja0; jc < p.j1; jc += COLS) {
        // per-lane offsets derived again in every chunk (keeps them out of registers during the mode-2 phase)
        int tidc = tid;
        asm volatile("" : "+v"(tidc));
        const int lane = tidc & 63, l32 = lane & 31, hi = lane >> 5;
        const int64_t ufo = ((int64_t)(wrow0 >> 5) * sp.nig) * (64 * 8) + lane * 8;
        const _Float16 *ufh = sp.Ufh + ufo, *ufl = sp.Ufl + ufo;
        const int pr0 = tidc >> 2, pf = tidc & 3;
        const int xs_w = pr0 * ROWB + pf * 16;      // + u*PCOLS*ROWB; low tile at + XBUF
        const int xs_r = l32 * ROWB + hi * 16;      // + ct*32*ROWB + g2*32; low tile at + XBUF
        f32x16 acc[RT][CT];
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < CT; ct++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[rt][ct][e] = 0.0f;
        int64_t x_off[XPT];
        bool x_ok[XPT];
        const void *const *tabrow = nullptr;   // TAB: the block pointers of this chunk's column, indexed by bi
        if constexpr (TAB) {
            // the chunk lies inside block column (bj, bk): offsets are relative to the start of a block of that column
            const int64_t bj = jc / p.x_dJ, bk = k / p.x_dK;
            const int64_t jb0 = bj * p.x_dJ, djb = (p.j1 - jb0 < p.x_dJ) ? p.j1 - jb0 : p.x_dJ;
            tabrow = p.xtab + (bk * p.tab_nbj + bj) * p.tab_nbi;
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                const int64_t j = jc + pr0 + PCOLS * u;
                x_ok[u] = (j >= p.j0) && (j < p.j1);
                x_off[u] = pf * 8 + (j - jb0) * p.x_dI + (k - bk * p.x_dK) * p.x_dI * djb;
            }
        } else {
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                const int64_t j = jc + pr0 + PCOLS * u;
                x_ok[u] = (j >= p.j0) && (j < p.j1);
                x_off[u] = (pf * 8 - p.xo_i) + (j - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk;
            }
        }

        auto stage_i = [&](int s) -> int64_t { return ia0 + (int64_t)(s < nstage ? s : nstage - 1) * EI; };
        auto load_u = [&](int d, int rt, int g2, int64_t ig) {
            const int64_t o = rt * u_rt_step + (ig + g2) * (64 * 8);
            uh[d][rt][g2] = *(const f16x8 *)(ufh + o);
            ul[d][rt][g2] = *(const f16x8 *)(ufl + o);
        };
        // TAB: start of stage s inside its block; the pointer is read from the table a whole stage before the loads
        // that use it are issued (the calls of load_x come in the order of the stages, from stage 0)
        auto gptr = [](const float *q) { return (const __attribute__((address_space(1))) f32x4 *)(uintptr_t)q; };
        const float *tab_next = nullptr;
        auto tab_fetch = [&](int s) {
            if constexpr (TAB) {
                const int ii = (int)stage_i(s), bi = ii / (int)p.x_dI;
                tab_next = (const float *)tabrow[bi] + (ii - bi * (int)p.x_dI);
            }
        };
        tab_fetch(0);
        auto load_x = [&](int s, f32x4 *slot) {
            const float *xb;
            if constexpr (TAB) xb = tab_next;
            else xb = (const float *)p.X + stage_i(s);
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                f32x4 v0 = {0.0f, 0.0f, 0.0f, 0.0f}, v1 = v0;
                if (x_ok[u]) {
                    v0 = *gptr(xb + x_off[u]);
                    v1 = *gptr(xb + x_off[u] + 4);
                }
                slot[2 * u] = v0;
                slot[2 * u + 1] = v1;
            }
            tab_fetch(s + 1);
        };
        // splits the tile pieces held in `slot` and writes the two fp16 tiles of a stage into LDS at `base`
        auto commit = [&](const f32x4 *slot, unsigned char *base) {
            typedef __fp16 h2 __attribute__((ext_vector_type(2)));
            typedef unsigned int u32x4w __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                u32x4w hw, lw;
#pragma unroll
                for (int e = 0; e < 4; e++) {  // pairs (2e, 2e+1) of the 8 values of this lane
                    const float a = slot[2 * u + (e >> 1)][2 * (e & 1)], b = slot[2 * u + (e >> 1)][2 * (e & 1) + 1];
                    const h2 h = __builtin_amdgcn_cvt_pkrtz(a, b);
                    const h2 l = __builtin_amdgcn_cvt_pkrtz(a - (float)h[0], b - (float)h[1]);
                    hw[e] = __builtin_bit_cast(unsigned int, h);
                    lw[e] = __builtin_bit_cast(unsigned int, l);
                }
                *(u32x4w *)(base + xs_w + u * PCOLS * ROWB) = hw;
                *(u32x4w *)(base + XBUF + xs_w + u * PCOLS * ROWB) = lw;
            }
        };
        // one stage: MFMAs of stage s (tiles in LDS buffer s&1, U fragments in register set s%DU) while the tile of
        // stage s+1 is split into the other buffer and the loads of later stages are issued
        auto stage = [&](auto sic, int s) {
            constexpr int SI = decltype(sic)::value;
            constexpr int PH = SI & 1, US = SI % DU, XS = (SI + 1) % DX;
            const unsigned char *cur = smem + PH * STAGE;
            unsigned char *oth = smem + (PH ^ 1) * STAGE;
            const int64_t ig2 = stage_i(s + DU) / GI;
            f16x8 bh[2][CT], bl[2][CT];
#pragma unroll
            for (int g2 = 0; g2 < 2; g2++)
#pragma unroll
                for (int ct = 0; ct < CT; ct++) {
                    bh[g2][ct] = *(const f16x8 *)(cur + xs_r + ct * 32 * ROWB + g2 * 32);
                    bl[g2][ct] = *(const f16x8 *)(cur + XBUF + xs_r + ct * 32 * ROWB + g2 * 32);
                }
            commit(xpre[XS], oth);
            load_x(s + 1 + DX, xpre[XS]);
            __builtin_amdgcn_sched_barrier(0);
            static_for<NMAIN>([&](auto mc) {
                constexpr int m = decltype(mc)::value, g2 = m / (RT * CT), rt = (m / CT) % RT, ct = m % CT;
                // smallest terms first
                acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ul[US][rt][g2], bh[g2][ct], acc[rt][ct], 0, 0, 0);
                acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_f16(uh[US][rt][g2], bl[g2][ct], acc[rt][ct], 0, 0, 0);
                acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_f16(uh[US][rt][g2], bh[g2][ct], acc[rt][ct], 0, 0, 0);
                if constexpr (ct == CT - 1) load_u(US, rt, g2, ig2);  // last use this stage: refill for stage s+DU
            });
        };

        // ---- prologue ----
#pragma unroll
        for (int d = 0; d < DU; d++) {
            const int64_t igd = stage_i(d) / GI;
#pragma unroll
            for (int rt = 0; rt < RT; rt++)
#pragma unroll
                for (int g2 = 0; g2 < 2; g2++) load_u(d, rt, g2, igd);
        }
#pragma unroll
        for (int d = 0; d < DX; d++) load_x(d, xpre[d]);
        __syncthreads();  // the previous chunk's mode-2 phase is done with the LDS
        commit(xpre[0], smem);
        load_x(DX, xpre[0]);
        __syncthreads();

        int s = 0;
        for (; s + UNR <= nstage; s += UNR)
            static_for<UNR>([&](auto c) {
                stage(c, s + decltype(c)::value);
                __syncthreads();
            });
        static_for<UNR - 1>([&](auto c) {
            if (s + decltype(c)::value < nstage) {
                stage(c, s + decltype(c)::value);
                __syncthreads();
            }
        });

        // ---- mode 2 on the finished Z chunk ----
        float *Zs = (float *)smem + wave * (32 * ZST);
        const bool first_chunk = (jc == ja0);
        if (p.MT == 2) mode2_chunk<RT, CT, 2, VM_F16X2>(p, sp.Vfh, Zs, acc, wrow0, kidx, jc, first_chunk, tid & 63, sp.Vfl);
        else mode2_chunk<RT, CT, 1, VM_F16X2>(p, sp.Vfh, Zs, acc, wrow0, kidx, jc, first_chunk, tid & 63, sp.Vfl);
    }
}

// Stacked fp32 U (rows x cols, leading dimension ld) -> two fp16 piece arrays in MFMA fragment order
// [rows/32][nig][64 lanes][8], zero padded (see SplitParams).
__global__ void k_pack_u_split(const float *src, int64_t ld, int rows, int64_t cols, _Float16 *dh, _Float16 *dl, int rowtiles, int64_t nig)
{
    const int64_t n = (int64_t)rowtiles * nig * 64 * 8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int e = (int)(idx & 7), l = (int)((idx >> 3) & 63);
        const int64_t f = idx >> 9, ig = f % nig, rt = f / nig;
        const int64_t r = rt * 32 + (l & 31), c = ig * 16 + (l >> 5) * 8 + e;
        const float v = (r < rows && c < cols) ? src[r * ld + c] : 0.0f;
        const _Float16 h = (_Float16)v;
        dh[idx] = h;
        dl[idx] = (_Float16)(v - (float)h);
    }
}

// Stacked fp32 V (P*M x J) -> two fp16 piece arrays in B-fragment order [P][Jpad/16][2][64 lanes][8], zero padded.
__global__ void k_pack_v_split(const float *src, int64_t ld, int P, int M, int64_t J, _Float16 *dh, _Float16 *dl, int64_t Jpad)
{
    const int64_t n = (int64_t)P * Jpad * 64;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int e = (int)(idx & 7), l = (int)((idx >> 3) & 63), mt = (int)((idx >> 9) & 1);
        const int64_t f = idx >> 10, j16 = f % (Jpad / 16), pr = f / (Jpad / 16);
        const int m = 32 * mt + (l & 31);
        const int64_t j = 16 * j16 + 8 * (l >> 5) + e;
        const float v = (m < M && j < J) ? src[(pr * M + m) * ld + j] : 0.0f;
        const _Float16 h = (_Float16)v;
        dh[idx] = h;
        dl[idx] = (_Float16)(v - (float)h);
    }
}

}  // namespace exat
