// Mode 2 of the compression chain on a finished Z chunk, shared by the pipelined mode-1/2 kernels:
// per 32-row tile of a wave and per replica p the tile touches,
//     Q[k][rows of p in the tile, 0..M) += Z_tile[rows, chunk columns] * V_p[:, chunk columns]^T.
// Each wave passes its tile through a private LDS region (Zs) to turn the MFMA accumulator layout into
// A-operand layout.  Nothing in the loops is conditional per element: the Q block is read and written whole
// (its rows exist up to PLpad), V and B/C gathers are unconditional, the rows of a replica are picked with a
// select.  Per-element branches here cost a scratch reload and a full memory wait each.
#pragma once
#include "exat_common.h"

namespace exat {

template <int V> struct ic { static constexpr int value = V; };

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// MTC: 32-column tiles of M (1 or 2).  VM selects the arithmetic:
//   VM_F32   fp32 MFMA, V_p from p.V;
//   VM_BF16  bf16 matrix cores, Z split into two bf16 pieces (error 2^-17), V_p (bf16) from Vf in fragment
//            order, [P][Jpad/16][2][64 lanes][8], lane l of fragment (p, j16, mt) holding
//            V_p[m = 32*mt + l%32, j = 16*j16 + 8*(l/32) .. +7];
//   VM_F16X2 fp16 matrix cores, Z and V_p each split into two fp16 pieces (Vf: high pieces, Vf2: low pieces,
//            same fragment order), the three significant cross terms accumulated in fp32 (error 2^-22).
// VB: V fragments (of 8 columns) requested together on the fp32 path; 16 = a whole chunk, fewer where registers are short.
enum { VM_F32 = 0, VM_BF16 = 1, VM_F16X2 = 2 };
template <int RT, int CT, int MTC, int VM, int VB = 16>
__device__ __forceinline__ void mode2_chunk(const Mode12Params &p, const void *Vf, float *Zs, const f32x16 (&acc)[RT][CT],
                                            int wrow0, int kidx, int64_t jc, bool first_chunk, int lane, const void *Vf2 = nullptr)
{
    constexpr int COLS = 32 * CT, ZST = COLS + 4;
    constexpr int MP = 32 * MTC;  // = p.Mpad; a constant here so that the 32 Q accesses of a tile differ by immediates
#pragma unroll
    for (int rt = 0; rt < RT; rt++) {
        const int q0 = wrow0 + rt * 32;  // wave-uniform
        if (q0 < p.PL) {
            // The lane number is made opaque here, so that every per-lane address below is derived after the stage loop,
            // where registers are free.  Left visible, the addresses of the Q rows and V fragments are loop invariants: the
            // compiler computes them once per workgroup, spills them, and reloads each in front of its access behind a full
            // memory wait -- some forty dependent round trips to memory per tile and chunk.
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int l32 = ln & 31, hi = ln >> 5;
            lane = ln;
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
            // The 32 x Mpad block of Q this tile adds to: requested before the MFMAs that produce the addends,
            // all of it and without conditions (the rows exist up to PLpad; rows of the padding hold zeros)
            float *Qt = p.Q + ((int64_t)kidx * p.PLpad + q0 + 4 * hi) * MP + l32;  // + (8*b4 + r)*Mpad + 32*mt
            float qsum[MTC][16];
#pragma unroll
            for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                for (int e = 0; e < 16; e++) qsum[mt][e] = 0.0f;
            if (!first_chunk) {
#pragma unroll
                for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                    for (int e = 0; e < 16; e++)
                        qsum[mt][e] = *((const float *)(Qt + (8 * (e >> 2) + (e & 3)) * MP + 32 * mt));
            }
            for (int pp = pfirst; pp <= plast; pp++) {
                const int rlo = pp * p.L, rhi = rlo + p.L;
                f32x16 qa[MTC];
#pragma unroll
                for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                    for (int e = 0; e < 16; e++) qa[mt][e] = 0.0f;
                if constexpr (VM == VM_F16X2) {
                    const int64_t fo = (((int64_t)pp * (p.Jpad / 16) + jc / 16) * 2) * 64 + lane;
                    const f16x8 *vh = (const f16x8 *)Vf + fo, *vl = (const f16x8 *)Vf2 + fo;
                    constexpr int GB = 4;  // 16-column groups per batch of V fragments
#pragma unroll
                    for (int g0 = 0; g0 < COLS / 16; g0 += GB) {
                        f16x8 bh[GB][MTC], bl[GB][MTC];
#pragma unroll
                        for (int g = 0; g < GB; g++)
#pragma unroll
                            for (int mt = 0; mt < MTC; mt++) {
                                bh[g][mt] = vh[((g0 + g) * 2 + mt) * 64];
                                bl[g][mt] = vl[((g0 + g) * 2 + mt) * 64];
                            }
                        __builtin_amdgcn_sched_barrier(0);  // keeps the requests together, ahead of the first MFMA
#pragma unroll
                        for (int g = 0; g < GB; g++) {
                            const f32x4 z0 = *(const f32x4 *)(Zs + l32 * ZST + 16 * (g0 + g) + 8 * hi);
                            const f32x4 z1 = *(const f32x4 *)(Zs + l32 * ZST + 16 * (g0 + g) + 8 * hi + 4);
                            f16x8 zh, zl;
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                zh[e] = (_Float16)z0[e]; zl[e] = (_Float16)(z0[e] - (float)zh[e]);
                                zh[4 + e] = (_Float16)z1[e]; zl[4 + e] = (_Float16)(z1[e] - (float)zh[4 + e]);
                            }
#pragma unroll
                            for (int mt = 0; mt < MTC; mt++) {
                                qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl, bh[g][mt], qa[mt], 0, 0, 0);
                                qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, bl[g][mt], qa[mt], 0, 0, 0);
                                qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, bh[g][mt], qa[mt], 0, 0, 0);
                            }
                        }
                    }
                } else if constexpr (VM == VM_BF16) {
                    // bf16 matrix cores: Z = zh + zl (bf16 pieces), V_p in fragment order
                    const bf16x8 *vf = (const bf16x8 *)Vf + (((int64_t)pp * (p.Jpad / 16) + jc / 16) * 2) * 64 + lane;
                    bf16x8 bv[COLS / 16][MTC];
#pragma unroll
                    for (int g16 = 0; g16 < COLS / 16; g16++)
#pragma unroll
                        for (int mt = 0; mt < MTC; mt++) bv[g16][mt] = *(vf + (g16 * 2 + mt) * 64);
                    __builtin_amdgcn_sched_barrier(0);  // keeps the requests together, ahead of the first MFMA
#pragma unroll
                    for (int g16 = 0; g16 < COLS / 16; g16++) {
                        const f32x4 z0 = *(const f32x4 *)(Zs + l32 * ZST + 16 * g16 + 8 * hi);
                        const f32x4 z1 = *(const f32x4 *)(Zs + l32 * ZST + 16 * g16 + 8 * hi + 4);
                        bf16x8 zh, zl;
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            zh[e] = (__bf16)z0[e]; zl[e] = (__bf16)(z0[e] - (float)zh[e]);
                            zh[4 + e] = (__bf16)z1[e]; zl[4 + e] = (__bf16)(z1[e] - (float)zh[4 + e]);
                        }
#pragma unroll
                        for (int mt = 0; mt < MTC; mt++) {
                            qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zl, bv[g16][mt], qa[mt], 0, 0, 0);
                            qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, bv[g16][mt], qa[mt], 0, 0, 0);
                        }
                    }
                } else {
                    // all V fragments of one 32-column tile of M are requested together, then multiplied: left
                    // to itself the compiler waits for each 16-byte load before its four MFMAs
                    const float *Vp = p.V + (int64_t)pp * MP * p.Jpad + jc + (int64_t)l32 * p.Jpad + 4 * hi;
#pragma unroll
                    for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                        for (int g0 = 0; g0 < COLS / 8; g0 += VB) {
                            f32x4 bv[VB];
#pragma unroll
                            for (int g8 = 0; g8 < VB; g8++)
                                bv[g8] = *((const f32x4 *)(Vp + (int64_t)(mt * 32) * p.Jpad + 8 * (g0 + g8)));
                            __builtin_amdgcn_sched_barrier(0);  // keeps the requests together, ahead of the first MFMA
#pragma unroll
                            for (int g8 = 0; g8 < VB; g8++) {
                                const f32x4 av = *(const f32x4 *)(Zs + l32 * ZST + 8 * (g0 + g8) + 4 * hi);
                                mma_frag<float>::mma(qa[mt], av, bv[g8]);
                            }
                        }
                }
                // rows of replica pp take this product (a select, not a branch)
#pragma unroll
                for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        const int row = q0 + 8 * (e >> 2) + 4 * hi + (e & 3);
                        qsum[mt][e] += (row >= rlo && row < rhi) ? qa[mt][e] : 0.0f;
                    }
            }
#pragma unroll
            for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                for (int e = 0; e < 16; e++)
                    *(Qt + (8 * (e >> 2) + (e & 3)) * MP + 32 * mt) = qsum[mt][e];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// Mode 2 straight from the accumulators, for kernels that ran mode 1 with the MFMA operands swapped, so that a
// tile's accumulator holds Z^T (rows: 32 fibres j, columns: 32 stacked rows q).  Register 4b+r of lane l is then
// Z^T[j = 8b + 4(l/32) + r][q = l%32], which is exactly what the 32x32x2 MFMA wants as its second operand for
// the pair of contraction indices (8b + r, 8b + 4 + r): Q^T[m, q] += sum_j V_p[m, j] Z^T[j, q] takes 16 MFMAs per
// tile with no trip through LDS.  V comes in the matching order (k_pack_v_direct): [p][mt][j/32][b][lane][r] holds
// V_p[32 mt + l%32][32 (j/32) + 8b + 4(l/32) + r].  Requires L % 32 == 0 (a tile of 32 rows q lies in one
// replica) and fp32 data.  Q keeps its layout [k][q][m]: a lane owns one row q and writes 16-byte pieces of it.
// The RT * MTC output tiles are taken one after the other in steps of one column tile ct (16 MFMAs); the V
// fragments of a step are requested three steps ahead (a ring of four register sets), so that after the first
// step the requests are always in flight behind the matrix instructions, also across the stores of a finished tile.
// Q between the chunks: the rows a wave adds to are its own for the whole launch, so the running sums stay in a
// wave-private piece of LDS (qlds: RT * MTC * 4 pieces of 64 lanes x 16 bytes, each lane reading back exactly what it
// wrote: no bank conflicts, no barrier) and only the last chunk's result goes to memory; Q is written once and never read.
template <int RT, int CT, int MTC>
__device__ __forceinline__ void mode2_direct(const Mode12Params &p, const float *Vd, const f32x16 (&acc)[RT][CT], int wrow0, int kidx,
                                             int64_t jc, bool first_chunk, bool last_chunk, f32x4 *qlds, int lane)
{
    constexpr int MP = 32 * MTC;   // = p.Mpad
    constexpr int NS = RT * MTC * CT, AHEAD = 3;
    const int l32 = lane & 31, hi = lane >> 5;
    const int64_t nj32 = p.Jpad / 32;
    f32x4 v[AHEAD + 1][4];
    f32x4 qold[4];
    f32x16 d;
    // step s = ((rt * MTC + mt) * CT + ct); a row tile beyond the stacked rows is skipped (wave-uniform)
    auto load_step = [&](int s) {
        const int rt = s / (MTC * CT), mt = (s / CT) % MTC, ct = s % CT;
        const int q0 = wrow0 + rt * 32;
        if (q0 < p.PL) {
            const int pr = q0 / p.L;
            const f32x4 *vf = (const f32x4 *)Vd + (((int64_t)pr * MTC + mt) * nj32 + jc / 32) * (4 * 64) + lane;
#pragma unroll
            for (int b = 0; b < 4; b++) v[s % (AHEAD + 1)][b] = vf[(ct * 4 + b) * 64];
        }
    };
#pragma unroll
    for (int s = 0; s < AHEAD && s < NS; s++) load_step(s);
#pragma unroll
    for (int s = 0; s < NS; s++) {
        const int rt = s / (MTC * CT), mt = (s / CT) % MTC, ct = s % CT;
        const int q0 = wrow0 + rt * 32;
        // this lane's 16 values of row q of Q (4 pieces of 4 consecutive m)
        float *Qt = p.Q + ((int64_t)kidx * p.PLpad + q0 + l32) * MP + 32 * mt + 4 * hi;   // + 8*b
        if (s + AHEAD < NS) load_step(s + AHEAD);
        if (ct == 0 && q0 < p.PL) {
#pragma unroll
            for (int b = 0; b < 4; b++) qold[b] = first_chunk ? f32x4{0.0f, 0.0f, 0.0f, 0.0f} : qlds[(((rt * MTC + mt) * 4) + b) * 64 + lane];
#pragma unroll
            for (int e = 0; e < 16; e++) d[e] = 0.0f;
        }
        __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the MFMAs
        if (q0 < p.PL) {
#pragma unroll
            for (int b = 0; b < 4; b++)
#pragma unroll
                for (int r = 0; r < 4; r++)
                    d = __builtin_amdgcn_mfma_f32_32x32x2f32(v[s % (AHEAD + 1)][b][r], acc[rt][ct][4 * b + r], d, 0, 0, 0);
            if (ct == CT - 1) {
                // d: register 4b+r of lane l is Q^T[m = 32 mt + 8b + 4(l/32) + r][q = q0 + l%32]
#pragma unroll
                for (int b = 0; b < 4; b++) {
                    f32x4 o;
#pragma unroll
                    for (int r = 0; r < 4; r++) o[r] = d[4 * b + r] + qold[b][r];
                    if (last_chunk) *(f32x4 *)(Qt + 8 * b) = o;
                    else qlds[(((rt * MTC + mt) * 4) + b) * 64 + lane] = o;
                }
            }
        }
    }
}

// Mode 2 straight from the accumulators on the bf16 matrix cores, for kernels that ran mode 1 with the MFMA operands
// swapped (a tile's accumulator holds Z^T: rows 32 fibres j, columns 32 stacked rows q).  Registers 8t .. 8t+7 of lane l
// are Z^T[j = 16t + 4(l/32) + e%4 + 8(e/4)][q = l%32], e = 0..7: converted to bf16 they are the second operand of a
// 32x32x16 MFMA whose 16 contraction slots stand for the 16 fibres 16t .. 16t+15 in that order, and V comes packed in
// the same order (UFragParams::Vz), so Q^T[m, q] += sum_j V_p[m, j] Z^T[j, q] needs no trip through LDS and no wave
// barrier.  Z goes in as two bf16 pieces (error 2^-17), as in mode2_chunk<VM_BF16>.  A tile of 32 rows q may touch two
// replicas: both products are formed and each lane keeps the one of its row's replica.  Q keeps its layout [k][q][m]: a
// lane owns one row q and reads and writes 16-byte pieces of it.
template <int RT, int CT, int MTC, int RSTRIDE = 32>
__device__ __forceinline__ void mode2_direct_bf16(const Mode12Params &p, const void *Vz, const f32x16 (&acc)[RT][CT], int wrow0, int kidx,
                                                  int64_t jc, bool first_chunk, int lane)
{
    constexpr int MP = 32 * MTC;   // = p.Mpad
#pragma unroll
    for (int rt = 0; rt < RT; rt++) {
        const int q0 = wrow0 + rt * RSTRIDE;   // wave-uniform
        if (q0 < p.PL) {
            int ln = lane;
            asm volatile("" : "+v"(ln));       // per-lane addresses are derived here, after the stage loop (see mode2_chunk)
            const int l32 = ln & 31, hi = ln >> 5;
            const int q = q0 + l32;
            const int qlast = (q0 + 31 < p.PL - 1) ? q0 + 31 : p.PL - 1;
            const int pfirst = q0 / p.L, plast = qlast / p.L;
            const float *Qt = p.Q + ((int64_t)kidx * p.PLpad + q) * MP + 4 * hi;   // + 32*mt + 8*b
            f32x4 qsum[MTC][4];
#pragma unroll
            for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                for (int b = 0; b < 4; b++) qsum[mt][b] = first_chunk ? f32x4{0.0f, 0.0f, 0.0f, 0.0f} : *(const f32x4 *)(Qt + 32 * mt + 8 * b);
            for (int pp = pfirst; pp <= plast; pp++) {
                const bool mine = q >= pp * p.L && q < (pp + 1) * p.L;
                // fragment (ct, t, mt) of this chunk: j16 = jc/16 + 2 ct + t
                const bf16x8 *vz = (const bf16x8 *)Vz + (((int64_t)pp * (p.Jpad / 16) + jc / 16) * 2) * 64 + ln;
                f32x16 qa[MTC];   // started by the first MFMA (its addend is the constant zero)
                const f32x16 zero16 = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
                // step st = 2 ct + t takes the fragments (st, mt); they are requested two steps ahead (a ring of three sets)
                bf16x8 bv[3][MTC];
#pragma unroll
                for (int st = 0; st < 2; st++)
#pragma unroll
                    for (int mt = 0; mt < MTC; mt++) bv[st][mt] = vz[(st * 2 + mt) * 64];
#pragma unroll
                for (int st = 0; st < 2 * CT; st++) {
                    const int ct = st >> 1, t = st & 1;
                    if (st + 2 < 2 * CT) {
#pragma unroll
                        for (int mt = 0; mt < MTC; mt++) bv[(st + 2) % 3][mt] = vz[((st + 2) * 2 + mt) * 64];
                    }
                    __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the MFMAs
                    bf16x8 zh, zl;
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const float z = acc[rt][ct][8 * t + e];
                        zh[e] = (__bf16)z;
                        zl[e] = (__bf16)(z - (float)zh[e]);
                    }
#pragma unroll
                    for (int mt = 0; mt < MTC; mt++) {
                        qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[st % 3][mt], zl, st == 0 ? zero16 : qa[mt], 0, 0, 0);
                        qa[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[st % 3][mt], zh, qa[mt], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                    for (int b = 0; b < 4; b++)
#pragma unroll
                        for (int r = 0; r < 4; r++) qsum[mt][b][r] += mine ? qa[mt][4 * b + r] : 0.0f;
            }
            // (the row's address is derived a second time rather than kept across the loop above, where registers are short)
            int ls = lane;
            asm volatile("" : "+v"(ls));
            float *Qs = p.Q + ((int64_t)kidx * p.PLpad + q0 + (ls & 31)) * MP + 4 * (ls >> 5);
#pragma unroll
            for (int mt = 0; mt < MTC; mt++)
#pragma unroll
                for (int b = 0; b < 4; b++) *(f32x4 *)(Qs + 32 * mt + 8 * b) = qsum[mt][b];
        }
    }
}

}  // namespace exat
