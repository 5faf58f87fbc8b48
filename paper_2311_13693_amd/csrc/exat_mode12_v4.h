// Fused mode-1 + mode-2 kernel for the bf16 generated source (the trillion-element configuration), fourth variant.
//
// Same decomposition as the other mode-1/2 kernels (one workgroup = one slice k x one group of ROWS stacked rows,
// full i reduction per 128-fibre column chunk, mode 2 on the finished Z chunk) and the same numerics as
// k_mode12_v3<__bf16, ..., SRC_GENERATED> (identical X tiles, identical accumulation order: results are bit-identical).
// What differs is how a stage is laid out for the hardware:
//   * A SIMD runs matrix and vector instructions side by side as long as the instruction stream offers both: an MFMA
//     occupies the matrix pipe for 32 cycles but the issue port for 4, and independent vector instructions issued
//     behind it run under it, from the same wave or from the second wave of the SIMD.  The stage is therefore written
//     as plain straight-line code -- all of the stage's MFMAs, the generator's low-rank MFMAs of the tile after next,
//     the noise of the next tile -- and the compiler is given the issue pattern "one MFMA, then a few vector
//     instructions" through scheduling-group hints instead of a hand-cut sequence of slots.
//   * Row groups are 512 stacked rows (8 waves x 2 row tiles, two waves per SIMD at 256 registers each, or 4 waves x 4
//     row tiles): the tile is generated once per row group, and its generation costs as much vector time as 400 rows
//     of MFMA work, so groups below that size are bound by the vector units whatever the schedule.
//   * A wave generates column blocks of ONE 16-row half of the tile, so that it needs the generator's A pieces of that
//     half only (half the A traffic of a wave that owns a full-height strip).
#pragma once
#include "exat_mode12_v3.h"

namespace exat {

template <int NW, int RT>
struct Mode12V4Cfg {
    static constexpr int ROWS = 32 * NW * RT, COLS = 128, ROWB = 80;
    static constexpr int XBUF_BYTES = COLS * ROWB;
    static constexpr int MAX_XBUFS = 8;
    static constexpr int LDS_BYTES = MAX_XBUFS * XBUF_BYTES;   // the ring of X tiles is all the LDS the kernel uses
};

// KS: 32-wide steps of the factor rank (R <= 32*KS); BOXED: the box is a proper sub-range in i; DU: register sets of
// U fragments (requested DU stages ahead); SCHED: 0 = leave the stage to the compiler's scheduler, 1 = interleave
// matrix and vector instructions through scheduling-group hints; NXB: X tiles in the LDS ring (2, 4 or 8).  A stage
// reads tile s from slot s mod NXB and writes tile s + NXB/2, and the workgroup meets at a barrier only after every
// NXB/2-th stage: between two barriers the slots read and the slots written are disjoint.
template <int NW, int RT, int KS, bool BOXED, int DU, int SCHED, int NXB = 2>
__global__ __launch_bounds__(64 * NW, NW / 4) void k_mode12_v4(const Mode12Params p, const GenSplitParams gs, const UFragParams uf)
{
    typedef Mode12V4Cfg<NW, RT> cfg;
    typedef __bf16 T;
    constexpr int CT = 4, ROWS = cfg::ROWS, COLS = cfg::COLS, ROWB = cfg::ROWB, XBUF = cfg::XBUF_BYTES;
    constexpr int EI = 32, GI = 16, E16 = 8;
    constexpr int SJW = 16 / NW;            // 16-column blocks of the generated tile per wave (all in one 16-row half)
    constexpr int NQ = SJW;                 // quads of 4 consecutive i per lane and stage
    constexpr int NTERM = 3;                // a_m b_h + a_h b_m + a_h b_h
    constexpr int W = NXB / 2;              // a stage produces the tile W stages ahead
    constexpr int UNR = lcm_i(lcm_i(2, DU), NXB);
    static_assert(NW == 4 || NW == 8, "4 or 8 waves");
    static_assert((NXB == 2 || NXB == 4 || NXB == 8) && NXB <= cfg::MAX_XBUFS && (SCHED == 1 || NXB == 2), "ring of 2, 4 or 8 X tiles");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nk = (int)(p.k1 - p.k0);
    const int bid = blockIdx.x, xcd = bid & 7, t = bid >> 3;
    // neighbours on an XCD take the same row group (and different slices): they share the U stream through its L2
    const int nkx = (nk + 7) >> 3;
    const int g = t / nkx;
    const int kidx = (t % nkx) * 8 + xcd;
    if (kidx >= nk) return;
    const int64_t k = p.k0 + kidx;
    const int row0 = p.row_base + g * ROWS;
    // row tile rt of wave w is tile w + NW*rt of the group: when the group's last tiles lie beyond the stacked rows (cfg5's
    // fifth group has 11 of 16), the waves that lose a tile are spread over all four SIMDs
    const int wrow0 = row0 + wave * 32;
    const bool two_tiles = RT == 2 && wrow0 + NW * 32 < p.PL;   // wave-uniform: this wave's second tile holds stacked rows
    const int64_t ia0 = p.i0 & ~(int64_t)(EI - 1);
    const int nstage = (int)((p.i1 - ia0 + EI - 1) / EI);
    const int64_t ja0 = (p.j0 / COLS) * COLS;
    const int64_t u_rt_step = uf.nig * (64 * E16);
    const int si = wave & 1, sj0 = (wave >> 1) * SJW;   // this wave generates rows 16*si.. of column blocks sj0 .. sj0+SJW-1

    bf16x8 ufr[DU][RT][2];
    bf16x8 afrag[2][2 * KS];             // A pieces (h, m) of the tiles s+2, s+3: [tile parity][piece, rank step]
    bf16x8 bfrag[2 * KS * SJW];          // B pieces (h, m) of this wave's column blocks: constant over a chunk
    f32x4v lr[2][NQ];                    // low-rank part of the tiles s+1, s+2: [tile parity][quad]
    uint32_t ckey[SJW];
    float amp[SJW];

    for (int64_t jc = ja0; jc < p.j1; jc += COLS) {
        int tidc = tid;
        asm volatile("" : "+v"(tidc));   // per-lane offsets are derived again in every chunk (not kept live over mode 2)
        const int lane = tidc & 63, l32 = lane & 31, hi = lane >> 5, l16 = lane & 15, q16 = lane >> 4;
        // Global addresses are a wave-uniform 64-bit base (scalar registers) plus a 32-bit per-lane byte offset: no
        // 64-bit per-lane pointer is kept in vector registers and no vector instruction is spent on address arithmetic
        const unsigned u_lane = (unsigned)lane * 16u;                                           // U fragments: 16 bytes per lane
        const unsigned a_lane = ((unsigned)l16 * (unsigned)gs.Rpad + 8u * (unsigned)q16) * 2u;  // A pieces: row l16, 8 ranks from 8*q16
        // buffer addressing: the descriptor holds the base, a scalar register the wave-uniform part of the offset, and the
        // one vector register u_lane / a_lane the per-lane part, so that a request costs no vector instruction at all
        const __amdgpu_buffer_rsrc_t urs = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const char *)uf.Uf + ((int64_t)(wrow0 >> 5) * uf.nig) * 1024), 0, (int)(((RT - 1) * NW + 1) * u_rt_step * 2), 0x00020000);
        const __amdgpu_buffer_rsrc_t ars = __builtin_amdgcn_make_buffer_rsrc((void *)gs.Asp, 0, (int)(2 * gs.Irows * gs.Rpad * 2), 0x00020000);
        const uint32_t iq_lane = 4u * (unsigned)si + (unsigned)q16;                             // quad of i within a stage
        const int xs_r = l32 * ROWB + hi * 16;                                          // + ct*32*ROWB + g2*32
        const int xg_w = (16 * sj0 + l16) * ROWB + (16 * si + 4 * q16) * (int)sizeof(T); // + b*16*ROWB
        f32x16 acc[RT][CT];
        float zero = 0.0f;
        asm volatile("" : "+v"(zero));   // a zero the compiler cannot keep as a 16-register vector across the chunks
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < CT; ct++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[rt][ct][e] = zero;

        // ---- per-chunk set-up: the generator's B operand bc[j, r] = B[j,r] C[k,r] of this lane's columns ----
#pragma unroll
        for (int b = 0; b < SJW; b++) {
            const int64_t j = jc + 16 * (sj0 + b) + l16;
            const bool colok = (j >= p.j0) && (j < p.j1);
            const int64_t jj = colok ? j : p.j0;
            ckey[b] = fibre_key(p.skey, (uint32_t)jj, (uint32_t)k);
            amp[b] = colok ? p.amp2_ln2 : 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                bf16x8 bh, bm;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const int r = 32 * ks + 8 * q16 + e, rr = r < p.R ? r : p.R - 1;   // clamped load, masked value
                    float bc = p.B[jj + p.ldB * rr] * p.C[k + p.ldC * rr];
                    bc = (colok && r < p.R) ? bc : 0.0f;
                    __bf16 h, m;
                    gen_piece<T>::split(bc, h, m);
                    bh[e] = h; bm[e] = m;
                }
                bfrag[(0 * KS + ks) * SJW + b] = bh;
                bfrag[(1 * KS + ks) * SJW + b] = bm;
            }
        }

        auto stage_i = [&](int s) -> int64_t { return ia0 + (int64_t)(s < nstage ? s : nstage - 1) * EI; };
        auto load_uf = [&](int rt, int64_t ig) -> bf16x8 {
            return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(urs, (int)u_lane, (int)((rt * NW * u_rt_step + ig * (64 * E16)) * 2), 0));
        };
        // A pieces of rows 16*si .. 16*si+15 of tile s
        auto load_a = [&](int s, bf16x8 *af) {
            const int64_t ib = stage_i(s);
#pragma unroll
            for (int v = 0; v < 2; v++)
#pragma unroll
                for (int ks = 0; ks < KS; ks++)
                    af[v * KS + ks] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                        ars, (int)a_lane, (int)((((int64_t)v * gs.Irows + ib + 16 * si) * gs.Rpad + 32 * ks) * 2), 0));
        };
        // low-rank part of the tile whose A pieces are in af: smallest terms first
        auto gen_lr = [&](f32x4v *dst, const bf16x8 *af) {
#pragma unroll
            for (int b = 0; b < SJW; b++) {
                f32x4v c = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++) {
                    c = gen_piece<T>::mfma(af[1 * KS + ks], bfrag[(0 * KS + ks) * SJW + b], c);
                    c = gen_piece<T>::mfma(af[0 * KS + ks], bfrag[(1 * KS + ks) * SJW + b], c);
                    c = gen_piece<T>::mfma(af[0 * KS + ks], bfrag[(0 * KS + ks) * SJW + b], c);
                }
                dst[b] = c;
            }
        };
        // tile s = low rank + noise, masked, rounded to bf16, into LDS buffer `base`
        auto noise_store = [&](int s, unsigned char *base, const f32x4v *lrs) {
            const int64_t i = stage_i(s) + 16 * si + 4 * q16;
#pragma unroll
            for (int b = 0; b < SJW; b++) {
                float z[4];
                noise_quad(ckey[b], (uint32_t)(i >> 2), amp[b], z);
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    x[e] = lrs[b][e] + z[e];
                    if (BOXED && (i + e < p.i0 || i + e >= p.i1)) x[e] = 0.0f;
                }
                const bf16x4 v = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
                *(bf16x4 *)(base + xg_w + b * 16 * ROWB) = v;
            }
        };

        // ---- the noise of one quad (4 consecutive i of one fibre) cut into NSTEP short steps, so that a stage can deal
        //      them out between its MFMAs.  State of quad b: nw[2b], nw[2b+1] (the two hash words), then the uniforms,
        //      radii and angles of the two Box-Muller pairs.  Same arithmetic as noise_quad. ----
        constexpr int NSTEP = 13;
        uint32_t nw[2 * NQ];
        float nu1[2 * NQ], nu2[2 * NQ], ncs[2 * NQ];
        auto nstep = [&](auto uc, int64_t ib1, unsigned char *oth, const f32x4v *lrs) {
            constexpr int u = decltype(uc)::value, st = u / NQ, b = u % NQ, w0 = 2 * b, w1 = 2 * b + 1;
            if constexpr (st == 0) {
                const uint32_t x = ckey[b] ^ ((uint32_t)(ib1 >> 2) + iq_lane);
                nw[w0] = x ^ (x >> 16);
            } else if constexpr (st == 1) {
                nw[w1] = nw[w0] * 0x21f0aaadu; nw[w0] *= 0x7feb352du;
            } else if constexpr (st == 2) {
                nw[w0] ^= nw[w0] >> 15; nw[w1] ^= nw[w1] >> 15;
            } else if constexpr (st == 3) {
                nw[w0] *= 0x846ca68bu; nw[w1] *= 0x735a2d97u;
            } else if constexpr (st == 4) {
                nw[w0] ^= nw[w0] >> 16; nw[w1] ^= nw[w1] >> 15;
            } else if constexpr (st == 5) {
                nu1[w0] = __builtin_fmaf((float)(nw[w0] >> 16), 0x1p-16f, 0x1p-17f);
                nu1[w1] = __builtin_fmaf((float)(nw[w1] >> 16), 0x1p-16f, 0x1p-17f);
            } else if constexpr (st == 6) {
                nu2[w0] = __builtin_fmaf((float)(nw[w0] & 0xffffu), 0x1p-16f, 0x1p-17f);
                nu2[w1] = __builtin_fmaf((float)(nw[w1] & 0xffffu), 0x1p-16f, 0x1p-17f);
            } else if constexpr (st == 7) {
                nu1[w0] = __builtin_amdgcn_logf(nu1[w0]); nu1[w1] = __builtin_amdgcn_logf(nu1[w1]);
            } else if constexpr (st == 8) {
                nu1[w0] = __builtin_amdgcn_sqrtf(amp[b] * nu1[w0]); nu1[w1] = __builtin_amdgcn_sqrtf(amp[b] * nu1[w1]);
            } else if constexpr (st == 9) {
                ncs[w0] = __builtin_amdgcn_cosf(nu2[w0]); ncs[w1] = __builtin_amdgcn_cosf(nu2[w1]);
            } else if constexpr (st == 10) {
                nu2[w0] = __builtin_amdgcn_sinf(nu2[w0]); nu2[w1] = __builtin_amdgcn_sinf(nu2[w1]);
            } else if constexpr (st == 11) {
                ncs[w0] *= nu1[w0]; nu2[w0] *= nu1[w0]; ncs[w1] *= nu1[w1]; nu2[w1] *= nu1[w1];
            } else {
                const int64_t i = ib1 + 16 * si + 4 * q16;
                float x[4] = {lrs[b][0] + ncs[w0], lrs[b][1] + nu2[w0], lrs[b][2] + ncs[w1], lrs[b][3] + nu2[w1]};
#pragma unroll
                for (int e = 0; e < 4; e++)
                    if (BOXED && (i + e < p.i0 || i + e >= p.i1)) x[e] = 0.0f;
                const bf16x4 v = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
                *(bf16x4 *)(oth + xg_w + b * 16 * ROWB) = v;
            }
        };

        // One stage: the MFMAs of stage s (X tile in LDS buffer s&1), the tile of stage s+1 produced into the other
        // buffer, the low-rank part of tile s+2, and the operand requests of later stages.
        // SCHED == 1 fixes the issue order.  A wave issues in order and an MFMA waits for the matrix pipe, so two MFMAs in
        // a row stall the wave, and the vector instructions behind them, for the first one's duration, while vector
        // instructions placed behind an MFMA run under it.  The stage is a sequence of slots "one MFMA, then a share of
        // the noise steps in proportion to the MFMA's duration"; the generator's MFMAs sit between the main ones of the
        // first two thirds; a request for operands of a later stage follows the last MFMA that reads the registers it
        // refills; the first steps run ahead of the first MFMA, under the latency of the LDS reads.
        auto stage = [&](auto sic, auto rac, int s) __attribute__((always_inline)) {
            constexpr int SI = decltype(sic)::value;  // s mod UNR
            constexpr int RA = decltype(rac)::value;  // row tiles of this wave that hold stacked rows (1 .. RT)
            constexpr int PH = SI & 1, US = SI % DU;
            constexpr int PN = (PH + W) & 1, PG = PN ^ 1;   // parities of the tile whose noise / whose low-rank part this stage makes
            const unsigned char *cur = smem + (SI % NXB) * XBUF;
            unsigned char *oth = smem + ((SI + W) % NXB) * XBUF;
            const int64_t ig2 = stage_i(s + DU) / GI;
            constexpr int NGEN = NTERM * KS * SJW, NMAIN = 2 * RA * CT;
            // X fragment f = g2*CT + ct: columns 32 ct .. 32 ct + 31, i group g2
            auto load_bx = [&](int f) -> bf16x8 { return *(const bf16x8 *)(cur + xs_r + (f % CT) * 32 * ROWB + (f / CT) * 32); };
            if constexpr (SCHED == 0) {
                bf16x8 bx[2][CT];
#pragma unroll
                for (int f = 0; f < 2 * CT; f++) bx[f / CT][f % CT] = load_bx(f);
                noise_store(s + 1, oth, lr[PH ^ 1]);
                gen_lr(lr[PH], afrag[PH]);   // tile s+2 from the A pieces requested two stages ago
                load_a(s + 4, afrag[PH]);
#pragma unroll
                for (int g2 = 0; g2 < 2; g2++)
#pragma unroll
                    for (int rt = 0; rt < RA; rt++) {
#pragma unroll
                        for (int ct = 0; ct < CT; ct++) acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[g2][ct], ufr[US][rt][g2], acc[rt][ct], 0, 0, 0);
                        ufr[US][rt][g2] = load_uf(rt, ig2 + g2);   // refill for stage s+DU
                    }
            } else {
                const int64_t ib1 = stage_i(s + W);
                constexpr int NU = NSTEP * NQ, NFRONT = NU / 6;
                constexpr int MG = (NMAIN * 2) / 3;                 // the generator's MFMAs follow main MFMAs 0 .. MG-1
                constexpr int WT = 2 * NMAIN + NGEN;                // total weight: main 2, generator 1
                auto gens_before = [](int m) constexpr { return (m * NGEN + MG - 1) / MG < NGEN ? (m * NGEN + MG - 1) / MG : NGEN; };
                auto step_at = [](int w) constexpr { return NFRONT + w * (NU - NFRONT) / WT; };
                // main MFMA m = (g2*CT + ct)*RT + rt: an X fragment serves RT consecutive MFMAs and is requested BXA
                // fragments ahead (a ring of BXA + 1 register sets)
                constexpr int BXA = 2;
                bf16x8 bx[BXA + 1];
#pragma unroll
                for (int f = 0; f < BXA; f++) bx[f] = load_bx(f);
                __builtin_amdgcn_sched_barrier(0);
                static_for<NFRONT>([&](auto uc) { nstep(uc, ib1, oth, lr[PN]); });
                __builtin_amdgcn_sched_barrier(0);
                static_for<NMAIN>([&](auto mc) {
                    constexpr int m = decltype(mc)::value, f = m / RA, rt = m % RA, g2 = f / CT, ct = f % CT;
                    if constexpr (rt == 0 && f + BXA < 2 * CT) bx[(f + BXA) % (BXA + 1)] = load_bx(f + BXA);
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[f % (BXA + 1)], ufr[US][rt][g2], acc[rt][ct], 0, 0, 0);
                    if constexpr (ct == CT - 1) ufr[US][rt][g2] = load_uf(rt, ig2 + g2);   // last use this stage: refill for stage s+DU
                    __builtin_amdgcn_sched_barrier(0);
                    constexpr int g0 = gens_before(m), g1 = gens_before(m + 1), wb = 2 * m + g0;
                    static_for<step_at(wb + 2) - step_at(wb)>([&](auto uc) { nstep(ic<step_at(wb) + decltype(uc)::value>(), ib1, oth, lr[PN]); });
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<g1 - g0>([&](auto gc) {
                        constexpr int n = g0 + decltype(gc)::value, term = n % NTERM, ks = (n / NTERM) % KS, b = n / (NTERM * KS);
                        constexpr int av = term == 0 ? 1 : 0, bv = term == 1 ? 1 : 0;   // a_m b_h, a_h b_m, a_h b_h
                        const f32x4v zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
                        lr[PG][b] = gen_piece<T>::mfma(afrag[PG][av * KS + ks], bfrag[(bv * KS + ks) * SJW + b], (term == 0 && ks == 0) ? zero4 : lr[PG][b]);
                        if constexpr (n == NGEN - 1) load_a(s + W + 3, afrag[PG]);         // these A pieces are free now
                        __builtin_amdgcn_sched_barrier(0);
                        constexpr int v0 = step_at(wb + 2 + n - g0), v1 = step_at(wb + 3 + n - g0);
                        static_for<v1 - v0>([&](auto uc) { nstep(ic<v0 + decltype(uc)::value>(), ib1, oth, lr[PN]); });
                        __builtin_amdgcn_sched_barrier(0);
                    });
                });
            }
        };

        // ---- prologue ----
        // (the stage loop exists twice: for waves with RT row tiles, and for waves whose second tile lies beyond the stacked
        //  rows, which then run half the main MFMAs and request half the U fragments; the choice is wave-uniform)
        auto run = [&](auto rac) __attribute__((always_inline)) {
            constexpr int RA = decltype(rac)::value;
        // Tiles 0 .. W-1 go to the ring, the low-rank part of tile W to its register set, and the A pieces of tiles W+1 and
        // W+2 to theirs.  Order of the requests: all A pieces first, the U fragments last.  The compiler derives the wait in
        // front of a stage's first generator MFMA from the smaller of two counts of requests issued after the A pieces it
        // reads, the one on the way in from here and the one around the loop; with the U requests ahead of the A pieces that
        // count made every other stage wait for requests issued a fraction of a stage before.
        {
            bf16x8 at[W + 3][2 * KS];
#pragma unroll
            for (int t = 0; t < W + 3; t++) load_a(t, at[t]);
#pragma unroll
            for (int d = 0; d < DU; d++) {
                const int64_t igd = stage_i(d) / GI;
#pragma unroll
                for (int rt = 0; rt < RA; rt++)
#pragma unroll
                    for (int g2 = 0; g2 < 2; g2++) ufr[d][rt][g2] = load_uf(rt, igd + g2);
            }
            __syncthreads();  // every wave is done with the ring slots of the previous chunk's last stages
#pragma unroll
            for (int t = 0; t < W; t++) {
                f32x4v l0[NQ];
                gen_lr(l0, at[t]);
                noise_store(t, smem + t * XBUF, l0);
            }
            gen_lr(lr[W & 1], at[W]);
#pragma unroll
            for (int q = 0; q < 2 * KS; q++) { afrag[(W + 1) & 1][q] = at[W + 1][q]; afrag[W & 1][q] = at[W + 2][q]; }
            __syncthreads();
        }

        int s = 0;
        for (; s + UNR <= nstage; s += UNR)
            static_for<UNR>([&](auto c) {
                stage(c, rac, s + decltype(c)::value);
                if constexpr ((decltype(c)::value + 1) % W == 0) __syncthreads();
            });
        static_for<UNR - 1>([&](auto c) {
            if (s + decltype(c)::value < nstage) {
                stage(c, rac, s + decltype(c)::value);
                if constexpr ((decltype(c)::value + 1) % W == 0) __syncthreads();
            }
        });

        };
        if (two_tiles) run(ic<RT>()); else run(ic<1>());

        // ---- mode 2 on the finished chunk, straight from the accumulators (they hold Z^T: the MFMAs above take the X
        //      fragment as first and the U fragment as second operand) ----
        const bool first_chunk = (jc == ja0);
        if (p.MT == 2) mode2_direct_bf16<RT, CT, 2, NW * 32>(p, uf.Vz, acc, wrow0, kidx, jc, first_chunk, tid & 63);
        else mode2_direct_bf16<RT, CT, 1, NW * 32>(p, uf.Vz, acc, wrow0, kidx, jc, first_chunk, tid & 63);
    }
}

}  // namespace exat
