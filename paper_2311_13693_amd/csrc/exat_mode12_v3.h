// Fused mode-1 + mode-2 kernel, third variant: the stacked U operand never touches LDS.
//
// Same decomposition as k_mode12 / k_mode12_v2 (one workgroup = one slice k x one group of ROWS stacked rows,
// full i reduction per 128-fibre column chunk, mode 2 on the finished Z chunk).  Differences:
//   * Every element of a U tile is consumed by exactly one wave, so staging it through LDS buys nothing and
//     costs an LDS write (64 B/clk/CU measured) plus an LDS read (128 B/clk/CU) per element.  Operand
//     preparation therefore also stores U in MFMA fragment order -- [row tile][i group][lane][16 bytes] -- and
//     each wave loads its A fragments straight from L2 into registers with fully coalesced 1 KiB loads, two
//     stages ahead (the stage loop is unrolled by two so that the two register sets are addressed statically).
//     LDS only holds the X tile (two 10 KiB stage buffers), which all waves share.
//   * A wave issues in order, and an MFMA cannot issue before the previous one has left the matrix pipe: two
//     MFMAs in a row stall the wave, and every vector instruction behind them, for the first one's duration,
//     while vector instructions placed between two MFMAs run under the first.  The generated-source stage is
//     therefore emitted as a fixed sequence of slots "one MFMA, then a share of the stage's vector work":
//     the noise of the next X tile is cut into 13 pipeline steps per quad of elements, and the steps are
//     dealt out over the main MFMAs (weight 2) and the generator's low-rank MFMAs (weight 1) in proportion
//     to their duration.
//   * bf16 plans run mode 2 on the bf16 matrix cores as well: the finished fp32 Z tile is split into two
//     bf16 pieces (error 2^-17) and multiplied with V, which bf16 plans round to bf16 anyway, stored in
//     fragment order.  The Q rows a tile adds to are requested before the mode-2 MFMAs, not after them.
#pragma once
#include <utility>

#include "exat_mode12_v2.h"

namespace exat {

struct UFragParams {
    const void *Uf;  // [PLpad/32][nig][64][16 bytes]: lane l of fragment (rt, ig) holds row 32*rt + l%32,
                     // i = ig*GI + (l/32)*E16 .. +E16-1   (GI = 2*E16: 16 for bf16, 8 for fp32)
    int64_t nig;     // Ipad / GI
    const void *Vf;  // bf16 plans: [P][Jpad/16][2][64][8 bf16]: lane l of fragment (p, j16, mt) holds
                     // V_p[m = 32*mt + l%32, j = 16*j16 + 8*(l/32) .. +7]
    const void *Vz;  // bf16 plans: the same fragments with the 16 columns of a fragment in the order in which the
                     // accumulators of a transposed mode 1 hold them (mode2_direct_bf16): element e of lane l is
                     // V_p[m = 32*mt + l%32, j = 16*j16 + 4*(l/32) + e%4 + 8*(e/4)]
};

template <int NW, int RT>
struct Mode12V3Cfg {
    static constexpr int ROWS = 32 * NW * RT, COLS = 128, ROWB = 80;
    static constexpr int XBUF_BYTES = COLS * ROWB;
    static constexpr int ZST = COLS + 4;
    static constexpr int EPI_BYTES = NW * 32 * ZST * 4;
    static constexpr int LDS_BYTES = 2 * XBUF_BYTES > EPI_BYTES ? 2 * XBUF_BYTES : EPI_BYTES;
    // kernels that take mode 2 straight from the accumulators (ZT): the two X buffers and the running sums of Q
    static constexpr int zt_lds_bytes(int MT) { return 2 * XBUF_BYTES + NW * RT * MT * 4 * 64 * 16; }
};

template <typename T> struct gen_terms;
// a = a_h + a_m: index 0 = h, 1 = m (bf16 pieces for bf16 plans, fp16 pieces for fp32 plans: gen_piece).  Smallest products first.
template <> struct gen_terms<__bf16> {
    static constexpr int N = 3;
    static constexpr int A[3] = {1, 0, 0};
    static constexpr int B[3] = {0, 1, 0};
};
template <> struct gen_terms<float> {
    static constexpr int N = 3;
    static constexpr int A[3] = {1, 0, 0};
    static constexpr int B[3] = {0, 1, 0};
};

template <int... Ms, typename F>
__device__ __forceinline__ void static_for_seq(std::integer_sequence<int, Ms...>, F &&f) { (f(ic<Ms>()), ...); }
// f(ic<0>()), ..., f(ic<N-1>()): a loop whose index is a compile-time constant in the body
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f) { static_for_seq(std::make_integer_sequence<int, N>(), f); }

// Slot plan of one generated-source stage.  Main MFMA m (0..NMAIN-1) is followed by the generator MFMAs
// g with g*MG/NGEN == m (they sit in the first MG main slots so that the A pieces can be reloaded in time);
// a main slot has weight 2, a generator slot weight 1, and the NUOP vector steps are dealt out by weight.
// The first NFRONT vector steps run before the first MFMA, while the stage's LDS fragment reads are in flight.
template <int NMAIN, int NGEN, int NUOP>
struct slot_plan {
    static constexpr int MG = (NMAIN * 2) / 3;
    static constexpr int W = 2 * NMAIN + NGEN;
    static constexpr int NFRONT = NUOP / 5;
    static constexpr int gens_before(int m) { return (m * NGEN + MG - 1) / MG < NGEN ? (m * NGEN + MG - 1) / MG : NGEN; }
    static constexpr int weight_before(int m) { return 2 * m + gens_before(m); }
    static constexpr int uop_at(int w) { return NFRONT + w * (NUOP - NFRONT) / W; }
};

constexpr int gcd_i(int a, int b) { return b == 0 ? a : gcd_i(b, a % b); }
constexpr int lcm_i(int a, int b) { return a / gcd_i(a, b) * b; }

// DU: register sets of U fragments (fragments are requested DU stages ahead); DX: register sets of the
// materialised X tile (requested DX + 1 stages ahead).  The stage loop is unrolled by lcm(2, DU, DX) so that
// every set is addressed statically.
// WPS: waves per SIMD the register allocation must allow (2 with NW = 4 lets two workgroups share a compute unit,
// so that one's chunk set-up and mode-2 phases run under the other's MFMA phase).
// ZT: mode 1 with the MFMA operands swapped (accumulators hold Z^T) and mode 2 straight from the accumulators
// (mode2_direct; fp32 materialised source, L % 32 == 0).
// TAB: the materialised X is a set of separate blocks addressed through Mode12Params::xtab (a slab of streamed blocks
// compressed in one launch: the box covers the whole i extent, its j and k ranges are whole blocks); needs whole stages
// of i and whole 128-fibre chunks inside every block.
template <typename T, int NW, int RT, int SRC, int KS, bool BOXED, int DU = 2, int DX = 1, int WPS = (NW + 3) / 4, bool ZT = false, bool TAB = false>
__global__ __launch_bounds__(64 * NW, WPS) void k_mode12_v3(const Mode12Params p, const GenSplitParams gs, const UFragParams uf)
{
    typedef Mode12V3Cfg<NW, RT> cfg;
    typedef typename mma_frag<T>::type frag_t;
    constexpr int CT = 4, ROWS = cfg::ROWS, COLS = cfg::COLS, ROWB = cfg::ROWB, ZST = cfg::ZST, XBUF = cfg::XBUF_BYTES;
    constexpr int EI = v2geom<T>::EI, NV = v2geom<T>::NV, SUBI = v2geom<T>::SUBI;
    constexpr int E16 = elem<T>::per16, GI = 2 * E16;
    constexpr int NT = 64 * NW, PSTEP = NT / 4, XPT = COLS * 4 / NT;
    constexpr int NSJ = 8 / NW, WCOLS = COLS / NW, NQ = SUBI * NSJ, NWD = 2 * NQ;
    constexpr int NMAIN = 2 * RT * CT;                       // main mma slots per stage
    constexpr int NTERM = gen_terms<T>::N, NGEN = NQ * KS * NTERM, NUOP = 13 * NQ;
    typedef slot_plan<NMAIN, NGEN, NUOP> plan;
    constexpr int UNR = lcm_i(lcm_i(2, DU), SRC == SRC_MATERIALISED ? DX : 1);
    static_assert(DU >= 2 && DX >= 1, "prefetch depths");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nk = (int)(p.k1 - p.k0);
    const int bid = blockIdx.x, xcd = bid & 7, t = bid >> 3;
    // Workgroup ids go round-robin over the 8 XCDs.  Materialised source: the G row groups of one slice sit
    // next to each other on one XCD and share the X tiles through its L2.  Generated source: nothing of X is
    // shared, so neighbours take the same row group g (and different slices) and share the U tiles instead,
    // which at 24 KiB per stage are the larger stream.
    const int nkx = (nk + 7) >> 3;
    const int g = SRC == SRC_GENERATED ? t / nkx : t % p.G;
    const int kidx = (SRC == SRC_GENERATED ? t % nkx : t / p.G) * 8 + xcd;
    if (kidx >= nk) return;
    const int64_t k = p.k0 + kidx;
    const int row0 = p.row_base + g * ROWS;
    const int wrow0 = row0 + wave * (RT * 32);
    const int64_t ia0 = p.i0 & ~(int64_t)(EI - 1);
    const int nstage = (int)((p.i1 - ia0 + EI - 1) / EI);
    const int64_t ja0 = (p.j0 / COLS) * COLS;

    const int64_t u_rt_step = uf.nig * (64 * E16);

    frag_t ufr[DU][RT][2];
    u32x4 xpre[SRC == SRC_MATERIALISED ? DX : 1][SRC == SRC_MATERIALISED ? XPT : 1];
    // A pieces of the stages whose low-rank tiles are next.  With one wave per SIMD there is room for two sets
    // (requested two stages ahead, [stage parity]); with two waves per SIMD one set, requested one stage ahead.
    constexpr int NAB = NW == 4 ? 2 : 1;
    bf16x8 afrag[NAB][SRC == SRC_GENERATED ? NV * KS * SUBI : 1];
    bf16x8 bfrag[SRC == SRC_GENERATED ? NV * KS * NSJ : 1];
    f32x4v accg[2][SRC == SRC_GENERATED ? NQ : 1];  // low-rank part of the X tiles of stages s+1, s+2: [stage parity][quad]
    uint32_t nw[SRC == SRC_GENERATED ? NWD : 1];
    float nu1[SRC == SRC_GENERATED ? NWD : 1], nu2[SRC == SRC_GENERATED ? NWD : 1], ncs[SRC == SRC_GENERATED ? NWD : 1];
    uint32_t ckey[NSJ];
    float amp[NSJ];

    // materialised source: the X tile of the next chunk's first stage, requested before the mode-2 phase of this
    // chunk so that the memory latency of the chunk start lies behind it (the second tile of the prologue as well
    // measured no faster and cost registers)
    u32x4 xnext[SRC == SRC_MATERIALISED ? XPT : 1];
    bool have_next = false;
    for (int64_t jc = ja0; jc < p.j1; jc += COLS) {
        // Per-lane offsets and pointers of the stage loop are derived again in every chunk from a copy of the
        // thread id the compiler cannot see through.  Kept live across chunks they would sit in registers during
        // the mode-2 phase, which then spills, and every reload of a spilled value is a full memory wait.
        int tidc = tid;
        asm volatile("" : "+v"(tidc));
        const int lane = tidc & 63, l32 = lane & 31, hi = lane >> 5, l16 = lane & 15, q16 = lane >> 4;
        // A fragments of this wave: row tiles (row0/32 + wave*RT + rt), i group ig
        const T *ufl = (const T *)uf.Uf + ((int64_t)(wrow0 >> 5) * uf.nig) * (64 * E16) + lane * E16;
        const int pr0 = tidc >> 2, pf = tidc & 3;
        const int xs_w = pr0 * ROWB + pf * 16;                                        // materialised tile: + u*PSTEP*ROWB
        const int xs_r = l32 * ROWB + hi * 16;                                        // + ct*32*ROWB + g2*32
        const int xg_w = (WCOLS * wave + l16) * ROWB + (4 * q16) * (int)sizeof(T);    // generated tile: + sj*16*ROWB + si*16*sizeof(T)
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
        const void *const *tabrow = nullptr;   // TAB: the block pointers of this chunk's column, indexed by bi
        if constexpr (SRC == SRC_MATERIALISED && TAB) {
            // the chunk lies inside block column (bj, bk): offsets are relative to the start of a block of that column
            const int64_t bj = jc / p.x_dJ, bk = k / p.x_dK;
            const int64_t jb0 = bj * p.x_dJ, djb = (p.j1 - jb0 < p.x_dJ) ? p.j1 - jb0 : p.x_dJ;
            tabrow = p.xtab + (bk * p.tab_nbj + bj) * p.tab_nbi;
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                const int64_t j = jc + pr0 + PSTEP * u;
                x_ok[u] = (j >= p.j0) && (j < p.j1);
                x_off[u] = pf * E16 + (j - jb0) * p.x_dI + (k - bk * p.x_dK) * p.x_dI * djb;
            }
        } else if constexpr (SRC == SRC_MATERIALISED) {
#pragma unroll
            for (int u = 0; u < XPT; u++) {
                const int64_t j = jc + pr0 + PSTEP * u;
                x_ok[u] = (j >= p.j0) && (j < p.j1);
                x_off[u] = (pf * E16 - p.xo_i) + (j - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk;
            }
        } else {
            // B operand of the generator: bc[j, r] = B[j,r] C[k,r] for this lane's columns, split in bf16 pieces
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
        auto load_uf = [&](int rt, int64_t ig) -> frag_t {
            return *((const frag_t *)(ufl + rt * u_rt_step + ig * (64 * E16)));
        };
        // TAB: start of stage s inside its block (block bi of the chunk's column).  The pointer is read from the table a
        // whole stage before the loads that use it are issued, behind the loads of the stage before.
        // a pointer that came out of the table is a pointer to device memory: say so, or every load through it is a flat load
        auto gptr = [](const T *q) { return (const __attribute__((address_space(1))) u32x4 *)(uintptr_t)q; };
        const T *tab_next = nullptr;
        auto tab_fetch = [&](int s) {
            if constexpr (TAB) {
                const int ii = (int)stage_i(s), bi = ii / (int)p.x_dI;
                tab_next = (const T *)tabrow[bi] + (ii - bi * (int)p.x_dI);
            }
        };
        if constexpr (TAB) {
            tab_fetch(have_next ? 1 : 0);   // the first load of the prologue: stage 0, or stage 1 when tile 0 was prefetched
        }
        auto load_x = [&](int s, u32x4 *slot) {
            if constexpr (SRC == SRC_MATERIALISED) {
                const T *xb;
                if constexpr (TAB) xb = tab_next;   // fetched behind the previous call's loads
                else xb = (const T *)p.X + stage_i(s);
#pragma unroll
                for (int u = 0; u < XPT; u++) {
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (x_ok[u]) v = *gptr(xb + x_off[u]);
                    slot[u] = v;
                }
                if constexpr (TAB) tab_fetch(s + 1);   // the calls come in the order of the stages
            }
        };
        auto load_a = [&](int s, bf16x8 *af) {
            if constexpr (SRC == SRC_GENERATED) {
                const int64_t ib = stage_i(s);
#pragma unroll
                for (int v = 0; v < NV; v++)
#pragma unroll
                    for (int ks = 0; ks < KS; ks++)
#pragma unroll
                        for (int si = 0; si < SUBI; si++)
                            af[(v * KS + ks) * SUBI + si] = *((const bf16x8 *)(gs.Asp + ((int64_t)v * gs.Irows + ib + 16 * si + l16) * gs.Rpad + 32 * ks + 8 * q16));
            }
        };
        // one low-rank MFMA of the tile whose A pieces are in af: term n of accumulator `dst`
        auto gen_one = [&](int n, f32x4v *dst, const bf16x8 *af) {
            const int term = n % NTERM, ks = (n / NTERM) % KS, sub = n / (NTERM * KS), si = sub / NSJ, sj = sub % NSJ;
            const bf16x8 av = af[(gen_terms<T>::A[term] * KS + ks) * SUBI + si];
            const bf16x8 bv = bfrag[(gen_terms<T>::B[term] * KS + ks) * NSJ + sj];
            const f32x4v zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
            const f32x4v c = (term == 0 && ks == 0) ? zero4 : dst[sub];
            dst[sub] = gen_piece<T>::mfma(av, bv, c);
        };
        // quad q of stage s: X = low rank (in xin) + noise, masked, converted and written to LDS buffer `base`
        auto store_quad = [&](unsigned char *base, int q, int64_t ib, const float *z, const f32x4v &lr) {
            const int64_t i = ib + 16 * (q / NSJ) + 4 * q16;
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                x[e] = lr[e] + z[e];
                if (BOXED && (i + e < p.i0 || i + e >= p.i1)) x[e] = 0.0f;
            }
            unsigned char *dst = base + xg_w + (q % NSJ) * 16 * ROWB + (q / NSJ) * 16 * (int)sizeof(T);
            if constexpr (sizeof(T) == 4) {
                f32x4 v = {x[0], x[1], x[2], x[3]};
                *(f32x4 *)dst = v;
            } else {
                bf16x4 v = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
                *(bf16x4 *)dst = v;
            }
        };
        // un-woven commit of stage s (prologue only)
        auto commit_plain = [&](int s, unsigned char *base, const f32x4v *lr) {
            if constexpr (SRC == SRC_MATERIALISED) {
#pragma unroll
                for (int u = 0; u < XPT; u++) *(u32x4 *)(base + xs_w + u * PSTEP * ROWB) = xpre[0][u];
            } else {
                const int64_t ib = stage_i(s);
#pragma unroll
                for (int q = 0; q < NQ; q++) {
                    float z[4];
                    noise_quad(ckey[q % NSJ], (uint32_t)((ib + 16 * (q / NSJ) + 4 * q16) >> 2), amp[q % NSJ], z);
                    store_quad(base, q, ib, z, lr[q]);
                }
            }
        };

        // vector step u = 13*? of the noise of stage s+1: step u / NQ of quad u % NQ (two hash words, four elements)
        auto uop = [&](auto uc, int64_t ib1, unsigned char *oth, const f32x4v *lr) {
            constexpr int u = decltype(uc)::value, st = u / NQ, q = u % NQ, w0 = 2 * q, w1 = 2 * q + 1;
            if constexpr (st == 0) {
                const uint32_t x = ckey[q % NSJ] ^ (uint32_t)((ib1 + 16 * (q / NSJ) + 4 * q16) >> 2);
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
                nu1[w0] = __builtin_amdgcn_sqrtf(amp[q % NSJ] * nu1[w0]); nu1[w1] = __builtin_amdgcn_sqrtf(amp[q % NSJ] * nu1[w1]);
            } else if constexpr (st == 9) {
                ncs[w0] = __builtin_amdgcn_cosf(nu2[w0]); ncs[w1] = __builtin_amdgcn_cosf(nu2[w1]);
            } else if constexpr (st == 10) {
                nu2[w0] = __builtin_amdgcn_sinf(nu2[w0]); nu2[w1] = __builtin_amdgcn_sinf(nu2[w1]);
            } else if constexpr (st == 11) {
                ncs[w0] *= nu1[w0]; nu2[w0] *= nu1[w0]; ncs[w1] *= nu1[w1]; nu2[w1] *= nu1[w1];
            } else {
                const float z[4] = {ncs[w0], nu2[w0], ncs[w1], nu2[w1]};
                store_quad(oth, q, ib1, z, lr[q]);
            }
        };

        // one stage: MFMAs of stage s (X tile in LDS buffer PH, A fragments in register set PH) interleaved with
        // the production of the X tile of stage s+1 (into the other buffer), the low-rank MFMAs of stage s+2 and
        // the reload of the A fragment registers for stage s+2
        // fp32 sources: the stage barrier sits mid-stage (see stage); the bf16 build of that form spills.  The fp32 generated
        // source qualifies with two waves per SIMD: its stage holds 64 fp32 MFMAs per wave and one quad of noise per lane,
        // so the whole tile of stage s+1 is produced under the first half of the MFMAs.
        constexpr bool MIDBAR_GEN = SRC == SRC_GENERATED && sizeof(T) == 4 && NW == 8;
        constexpr bool MIDBAR = (SRC == SRC_MATERIALISED && sizeof(T) == 4) || MIDBAR_GEN;
        frag_t bx0[MIDBAR ? CT : 1];   // first-group X fragments of the stage about to run
        auto stage = [&](auto sic, int s) {
            constexpr int SI = decltype(sic)::value;  // s mod UNR
            constexpr int PH = SI & 1, US = SI % DU, XS = (SI + 1) % DX;
            const unsigned char *cur = smem + PH * XBUF;
            unsigned char *oth = smem + (PH ^ 1) * XBUF;
            const int64_t ib1 = stage_i(s + 1);
            const int64_t ig2 = stage_i(s + DU) / GI;
            if constexpr (MIDBAR_GEN) {
                // As below, for the generated source: the noise steps and the generator's MFMAs of the stage all sit in the
                // first half (the MFMAs of the first i group), so that every wave has stored its part of the tile of stage
                // s+1 when it reaches the barrier between the two halves.
                frag_t bx1[CT];
#pragma unroll
                for (int ct = 0; ct < CT; ct++) bx1[ct] = *(const frag_t *)(cur + xs_r + ct * 32 * ROWB + 32);
                __builtin_amdgcn_sched_barrier(0);
                constexpr int NH = NMAIN / 2;
                static_for<NMAIN>([&](auto mc) {
                    constexpr int m = decltype(mc)::value, g2 = m / (RT * CT), rt = (m / CT) % RT, ct = m % CT;
                    if constexpr (m == NH) {
                        __syncthreads();
#pragma unroll
                        for (int c2 = 0; c2 < CT; c2++) bx0[c2] = *(const frag_t *)(oth + xs_r + c2 * 32 * ROWB);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const frag_t &bxe = g2 == 0 ? bx0[ct] : bx1[ct];
                    if constexpr (ZT) mma_frag<T>::mma(acc[rt][ct], bxe, ufr[US][rt][g2]);
                    else mma_frag<T>::mma(acc[rt][ct], ufr[US][rt][g2], bxe);
                    if constexpr (ct == CT - 1) ufr[US][rt][g2] = load_uf(rt, ig2 + g2);  // last use this stage: refill for stage s+DU
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (m < NH) {
                        // steps u0..u1 of the NUOP noise steps and generator MFMAs g0..g1 of NGEN behind main MFMA m
                        constexpr int u0 = m * NUOP / NH, u1 = (m + 1) * NUOP / NH, g0 = m * NGEN / NH, g1 = (m + 1) * NGEN / NH;
                        static_for<u1 - u0>([&](auto uc) { uop(ic<u0 + decltype(uc)::value>(), ib1, oth, accg[PH ^ 1]); });
                        __builtin_amdgcn_sched_barrier(0);
                        static_for<g1 - g0>([&](auto gc) {
                            gen_one(g0 + decltype(gc)::value, accg[PH], afrag[PH % NAB]);
                            __builtin_amdgcn_sched_barrier(0);
                        });
                        if constexpr (g1 == NGEN && g0 < NGEN) load_a(s + 2 + NAB, afrag[PH % NAB]);  // these A pieces are free now
                    }
                });
                return;
            }
            if constexpr (MIDBAR) {
                // Materialised fp32 source: the tile of stage s+1 is complete in LDS as soon as every wave has stored its
                // part at the start of stage s, so the stage's barrier sits between its two halves (the MFMAs of the
                // first and of the second i group): the first-group fragments of stage s+1 are read right after it,
                // behind the second half's MFMAs, and a wave that waits at the barrier leaves the matrix pipe to the
                // other wave of its SIMD.  bx0 holds the first-group fragments of the current stage on entry.
                frag_t bx1[CT];
#pragma unroll
                for (int ct = 0; ct < CT; ct++) bx1[ct] = *(const frag_t *)(cur + xs_r + ct * 32 * ROWB + 32);
#pragma unroll
                for (int u = 0; u < XPT; u++) *(u32x4 *)(oth + xs_w + u * PSTEP * ROWB) = xpre[XS][u];
                load_x(s + 1 + DX, xpre[XS]);
                __builtin_amdgcn_sched_barrier(0);
                static_for<NMAIN>([&](auto mc) {
                    constexpr int m = decltype(mc)::value, g2 = m / (RT * CT), rt = (m / CT) % RT, ct = m % CT;
                    if constexpr (m == NMAIN / 2) {
                        __syncthreads();
#pragma unroll
                        for (int c2 = 0; c2 < CT; c2++) bx0[c2] = *(const frag_t *)(oth + xs_r + c2 * 32 * ROWB);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const frag_t &bxe = g2 == 0 ? bx0[ct] : bx1[ct];
                    if constexpr (ZT) mma_frag<T>::mma(acc[rt][ct], bxe, ufr[US][rt][g2]);
                    else mma_frag<T>::mma(acc[rt][ct], ufr[US][rt][g2], bxe);
                    if constexpr (ct == CT - 1) ufr[US][rt][g2] = load_uf(rt, ig2 + g2);  // last use this stage: refill for stage s+DU
                    __builtin_amdgcn_sched_barrier(0);
                });
                return;
            }
            frag_t bx[2][CT];
#pragma unroll
            for (int g2 = 0; g2 < 2; g2++)
#pragma unroll
                for (int ct = 0; ct < CT; ct++) bx[g2][ct] = *(const frag_t *)(cur + xs_r + ct * 32 * ROWB + g2 * 32);
            if constexpr (SRC == SRC_MATERIALISED) {
#pragma unroll
                for (int u = 0; u < XPT; u++) *(u32x4 *)(oth + xs_w + u * PSTEP * ROWB) = xpre[XS][u];
                load_x(s + 1 + DX, xpre[XS]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (SRC == SRC_GENERATED) {
                static_for<plan::NFRONT>([&](auto uc) { uop(uc, ib1, oth, accg[PH ^ 1]); });
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<NMAIN>([&](auto mc) {
                constexpr int m = decltype(mc)::value, g2 = m / (RT * CT), rt = (m / CT) % RT, ct = m % CT;
                if constexpr (ZT) mma_frag<T>::mma(acc[rt][ct], bx[g2][ct], ufr[US][rt][g2]);
                else mma_frag<T>::mma(acc[rt][ct], ufr[US][rt][g2], bx[g2][ct]);
                if constexpr (ct == CT - 1) ufr[US][rt][g2] = load_uf(rt, ig2 + g2);  // last use this stage: refill for stage s+DU
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (SRC == SRC_GENERATED) {
                    constexpr int g0 = plan::gens_before(m), g1 = plan::gens_before(m + 1), wb = plan::weight_before(m);
                    constexpr int u0 = plan::uop_at(wb), u1 = plan::uop_at(wb + 2);
                    static_for<u1 - u0>([&](auto uc) { uop(ic<u0 + decltype(uc)::value>(), ib1, oth, accg[PH ^ 1]); });
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<g1 - g0>([&](auto gc) {
                        constexpr int g = g0 + decltype(gc)::value;
                        gen_one(g, accg[PH], afrag[PH % NAB]);
                        __builtin_amdgcn_sched_barrier(0);
                        constexpr int v0 = plan::uop_at(wb + 2 + g - g0), v1 = plan::uop_at(wb + 3 + g - g0);
                        static_for<v1 - v0>([&](auto uc) { uop(ic<v0 + decltype(uc)::value>(), ib1, oth, accg[PH ^ 1]); });
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    if constexpr (g1 == NGEN && g0 < NGEN) load_a(s + 2 + NAB, afrag[PH % NAB]);  // these A pieces are free now
                }
            });
        };

        // ---- prologue: A fragments of stages 0 and 1 in registers, X tile of stage 0 in buffer 0, of stage 1 in
        //      registers, generator pieces of stage 2 in flight ----
#pragma unroll
        for (int d = 0; d < DU; d++) {
            const int64_t igd = stage_i(d) / GI;
#pragma unroll
            for (int rt = 0; rt < RT; rt++)
#pragma unroll
                for (int g2 = 0; g2 < 2; g2++) ufr[d][rt][g2] = load_uf(rt, igd + g2);
        }
        if constexpr (SRC == SRC_MATERIALISED) {
#pragma unroll
            for (int d = 0; d < DX; d++) {
                if (d == 0 && have_next) {
#pragma unroll
                    for (int u = 0; u < XPT; u++) xpre[0][u] = xnext[u];
                } else
                    load_x(d, xpre[d]);
            }
        }
        load_a(0, afrag[0]);
        if constexpr (NAB == 2) load_a(1, afrag[1]);
        if constexpr (SRC == SRC_GENERATED) {
#pragma unroll
            for (int n = 0; n < NGEN; n++) gen_one(n, accg[0], afrag[0]);
        }
        __syncthreads();  // the previous chunk's epilogue is done with the LDS
        commit_plain(0, smem, accg[0]);
        load_x(DX, xpre[0]);
        load_a(NAB == 2 ? 2 : 1, afrag[0]);
        if constexpr (SRC == SRC_GENERATED) {
#pragma unroll
            for (int n = 0; n < NGEN; n++) gen_one(n, accg[1], afrag[NAB - 1]);
        }
        load_a(NAB == 2 ? 3 : 2, afrag[NAB - 1]);
        __syncthreads();

        if constexpr (MIDBAR) {
#pragma unroll
            for (int ct = 0; ct < CT; ct++) bx0[ct] = *(const frag_t *)(smem + xs_r + ct * 32 * ROWB);
        }
        int s = 0;
        for (; s + UNR <= nstage; s += UNR)
            static_for<UNR>([&](auto c) {
                stage(c, s + decltype(c)::value);
                if constexpr (!MIDBAR) __syncthreads();   // otherwise the stage has its barrier inside
            });
        static_for<UNR - 1>([&](auto c) {
            if (s + decltype(c)::value < nstage) {
                stage(c, s + decltype(c)::value);
                if constexpr (!MIDBAR) __syncthreads();
            }
        });
        if constexpr (MIDBAR) __syncthreads();   // every wave is done with the X tiles in LDS

        if constexpr (SRC == SRC_MATERIALISED) {
            have_next = jc + COLS < p.j1;
            if (have_next) {
                if constexpr (TAB) {
                    const int64_t jn = jc + COLS, bj = jn / p.x_dJ, bk = k / p.x_dK;
                    const int64_t jb0 = bj * p.x_dJ, djb = (p.j1 - jb0 < p.x_dJ) ? p.j1 - jb0 : p.x_dJ;
                    const T *xb = (const T *)p.xtab[(bk * p.tab_nbj + bj) * p.tab_nbi];   // block bi = 0 of the next chunk's column
#pragma unroll
                    for (int u = 0; u < XPT; u++) {
                        const int64_t j = jn + pr0 + PSTEP * u;
                        u32x4 v = {0u, 0u, 0u, 0u};
                        if (j >= p.j0 && j < p.j1) v = *gptr(xb + pf * E16 + (j - jb0) * p.x_dI + (k - bk * p.x_dK) * p.x_dI * djb);
                        xnext[u] = v;
                    }
                } else {
                const T *xb = (const T *)p.X + stage_i(0);
#pragma unroll
                for (int u = 0; u < XPT; u++) {
                    const int64_t j = jc + COLS + pr0 + PSTEP * u;
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (j >= p.j0 && j < p.j1) v = *(const u32x4 *)(xb + (pf * E16 - p.xo_i) + (j - p.xo_j) * p.x_sj + (k - p.xo_k) * p.x_sk);
                    xnext[u] = v;
                }
                }
            }
        }
        // ---- mode 2 on the finished Z chunk ----
        float *Zs = (float *)smem + wave * (32 * ZST);
        const bool first_chunk = (jc == ja0);
        if constexpr (ZT) {
            static_assert(!ZT || sizeof(T) == 4, "ZT: fp32 only");
            // running sums of Q: behind the two X buffers, RT * MT * 4 KiB per wave (Mode12V3Cfg::zt_lds_bytes)
            f32x4 *qlds = (f32x4 *)(smem + 2 * XBUF) + wave * (RT * p.MT * 4 * 64);
            const bool last_chunk = jc + COLS >= p.j1;
            if (p.MT == 2) mode2_direct<RT, CT, 2>(p, p.Vd, acc, wrow0, kidx, jc, first_chunk, last_chunk, qlds, tid & 63);
            else mode2_direct<RT, CT, 1>(p, p.Vd, acc, wrow0, kidx, jc, first_chunk, last_chunk, qlds, tid & 63);
        } else if (p.MT == 2) mode2_chunk<RT, CT, 2, sizeof(T) == 2 ? VM_BF16 : VM_F32>(p, uf.Vf, Zs, acc, wrow0, kidx, jc, first_chunk, tid & 63);
        else mode2_chunk<RT, CT, 1, sizeof(T) == 2 ? VM_BF16 : VM_F32>(p, uf.Vf, Zs, acc, wrow0, kidx, jc, first_chunk, tid & 63);
    }
}

// Stacked fp32 U (rows x cols, leading dimension ld) -> MFMA fragment order [rows/32][nig][64 lanes][E16] of T,
// zero padded: lane l of fragment (rt, ig) holds row 32*rt + l%32, columns ig*2*E16 + (l/32)*E16 .. +E16-1.
template <typename T>
__global__ void k_pack_u_frag(const float *src, int64_t ld, int rows, int64_t cols, T *dst, int rowtiles, int64_t nig)
{
    constexpr int E16 = elem<T>::per16;
    const int64_t n = (int64_t)rowtiles * nig * 64 * E16;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int e = (int)(idx % E16);
        const int l = (int)((idx / E16) % 64);
        const int64_t f = idx / (64 * E16), ig = f % nig, rt = f / nig;
        const int64_t r = rt * 32 + (l & 31), c = ig * (2 * E16) + (l >> 5) * E16 + e;
        const float v = (r < rows && c < cols) ? src[r * ld + c] : 0.0f;
        dst[idx] = elem<T>::from_f32(v);
    }
}

// Stacked fp32 V (P*M x J) -> bf16 B fragments of the 32x32x16 MFMA, [P][Jpad/16][2][64 lanes][8], zero padded:
// lane l of fragment (p, j16, mt) holds V_p[m = 32*mt + l%32, j = 16*j16 + 8*(l/32) .. +7].
// perm: the column order of mode2_direct_bf16 (UFragParams::Vz) instead.
__global__ void k_pack_v_frag(const float *src, int64_t ld, int P, int M, int64_t J, __bf16 *dst, int64_t Jpad, int perm)
{
    const int64_t n = (int64_t)P * Jpad * 64;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int e = (int)(idx & 7), l = (int)((idx >> 3) & 63), mt = (int)((idx >> 9) & 1);
        const int64_t f = idx >> 10, j16 = f % (Jpad / 16), pr = f / (Jpad / 16);
        const int m = 32 * mt + (l & 31);
        const int64_t j = perm ? 16 * j16 + 4 * (l >> 5) + (e & 3) + 8 * (e >> 2) : 16 * j16 + 8 * (l >> 5) + e;
        const float v = (m < M && j < J) ? src[(pr * M + m) * ld + j] : 0.0f;
        dst[idx] = (__bf16)v;
    }
}

// Stacked fp32 V (P*M x J) in the order mode2_direct consumes: [P][Mpad/32][Jpad/32][4 b][64 lanes][4 r] holds
// V_p[m = 32*mt + l%32][j = 32*jt + 8*b + 4*(l/32) + r], zero padded.
__global__ void k_pack_v_direct(const float *src, int64_t ld, int P, int M, int64_t J, float *dst, int Mpad, int64_t Jpad)
{
    const int64_t n = (int64_t)P * Mpad * Jpad;
    const int64_t nj32 = Jpad / 32;
    const int mtc = Mpad / 32;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int r = (int)(idx & 3), l = (int)((idx >> 2) & 63), b = (int)((idx >> 8) & 3);
        const int64_t f = idx >> 10, jt = f % nj32, mt = (f / nj32) % mtc, pr = f / (nj32 * mtc);
        const int m = 32 * (int)mt + (l & 31);
        const int64_t j = 32 * jt + 8 * b + 4 * (l >> 5) + r;
        dst[idx] = (m < M && j < J) ? src[(pr * M + m) * ld + j] : 0.0f;
    }
}

}  // namespace exat
