// First stage of the two-stage compression (paper Sec. 4.4): X1 = X x1 U x2 V x3 W with sparse U, V, W
// shared by all replicas.  Declarations and contracts in include/exat.h.
//
// The stage reads X once from HBM (4 bytes per element against 2*nnz_per_column flops):
//   k_stage1_mode12  one workgroup per (frontal slice k, range of column tiles).  It walks its part of the slice
//                    in 64-column x 128-row tiles that go HBM -> registers -> LDS, each element once.  Mode 1: a
//                    lane owns a column j of the tile; the non-zeros of U inside the row tile are dealt to the
//                    waves row by row, as streams of 64-byte chunks (8 non-zeros of one output row a).  For every
//                    non-zero the wave does one LDS read and one multiply-add; the row's sum over the row tiles
//                    is kept in LDS.  When the column tile's rows are finished mode 2 runs over the 64 x A1 result
//                    with lanes along a, and the A1 x B1 partial result of the column range goes to Q.
//   k_stage1_sum_ranges  adds the partial results of the column ranges (only when a slice was split).
//   k_stage1_mode3   X1[a,b,c] = sum_k W[c,k] Q[k][b][a], a thread per (a,b,c), the non-zeros of row c in
//                    stored order.
//   k_stage1_mfma    the same two modes on the matrix cores, which are otherwise idle in this read-bound stage, when every
//                    value of U and V is exactly representable in bf16 (sign matrices are) and I is a multiple of 4: U and V
//                    are taken as DENSE bf16 matrices, X is read along its columns in whole cache lines, transposed through
//                    wave-private LDS slots and split on the fly into three truncated bf16 pieces (an exact split, so the
//                    products are exact too); described at the kernel.  16 times the arithmetic of the sparse form on a unit
//                    with nothing else to do; the sparse form's per-non-zero instruction streams and dependent scalar loads
//                    are what kept it below half of the HBM peak.
// Every sum has a fixed order, so results are bit-identical from run to run.
#include "../../include/exat.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

namespace {

constexpr int S1_IT = 128;     // rows i per tile
constexpr int S1_JT = 64;      // columns j per tile (one per lane)
constexpr int S1_NW = 8;       // waves per workgroup (each owns a chunk stream per row tile)
constexpr int S1_NT = 64 * S1_NW;
constexpr int S1_XS = S1_IT + 1;  // LDS row stride of the X tile (odd: lanes reading one i of 64 columns hit 64 banks)
constexpr int S1_MAXROWS = 128;   // largest A1 and B1
constexpr int64_t S1_MAXI = (1 << 23) - 1;   // 64 tile columns of I floats must stay below 2 GiB (buffer offsets)
constexpr int64_t kMaxExtent1 = 2147483647LL - 64;

struct SEnt { int c; float v; };  // one non-zero: column inside its tile, value

// Mode-1 work of one wave on one row tile: a stream of 64-byte chunks, each holding up to 8 non-zeros of ONE
// output row as (word, value) pairs.  A word's low 9 bits are the non-zero's byte offset in an LDS tile row
// (4 * local column); the first word of a chunk also carries the output row (bits 9..16), whether this is
// the row's last chunk in the tile (bit 17) and whether pairs 4..7 are only padding (bit 18).  Padding pairs
// are (0, 0.0f).
constexpr int CH_LAST = 1 << 17, CH_HALF = 1 << 18;

struct S1Params {
    const float *X;
    int64_t I, J, K;
    int A1, B1;
    const int2 *Uoc;   // [nit][S1_NW waves]: (first chunk, number of chunks) of the wave's stream
    const int *Uch;    // chunks, 16 ints each; two padding chunks at the very end
    const int *Vtp;    // [njt][B1+1] offsets into Vent; every (tile,row) range is a multiple of 4 entries
    const SEnt *Vent;
    float *Q;          // [JS][K][B1][A1]: partial sums over the column range of each workgroup
    int jt_per;        // column tiles per workgroup (blockIdx.y selects the range)
    int64_t k0;        // slice index of X[0] (X may be a slab of slices of the tensor): Q is indexed by k0 + blockIdx.x
    int64_t qstride;   // floats between the partial results of consecutive column ranges
};

typedef int i32x4 __attribute__((ext_vector_type(4)));

// The operator's tables are never written while a kernel runs.  Reading them through the constant address
// space tells the compiler so: wave-uniform reads then go through the scalar cache into SGPRs even in loops
// that contain LDS atomics (which it otherwise takes for possible writers).
#define S1_CONST __attribute__((address_space(4)))
template <typename T>
__device__ inline const S1_CONST T *as_const(const T *p) { return (const S1_CONST T *)(uintptr_t)p; }

// AT = 64-lane tiles of a (A1 <= 64*AT), BR = output rows b per wave in mode 2 (B1 <= S1_NW*BR)
template <int AT, int BR>
__global__ __launch_bounds__(S1_NT, 6) void k_stage1_mode12(const S1Params p)
{
    extern __shared__ float smem[];
    constexpr int ZS = 64 * AT + 1;
    constexpr int CG = S1_NT / S1_IT;     // column groups: a thread holds row li of columns lj + CG*jj
    constexpr int NPRE = S1_JT / CG;
    float *xs = smem;                    // [64 j][S1_XS]
    float *zs = smem + S1_JT * S1_XS;    // [64 j][ZS]: mode-1 result of the current column tile
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t k = blockIdx.x;
    const float *Xk = p.X + k * p.I * p.J;
    const int nit = (int)((p.I + S1_IT - 1) / S1_IT), njt = (int)((p.J + S1_JT - 1) / S1_JT);
    const int li = tid & (S1_IT - 1);
    const int lj = w / (S1_IT / 64);     // the same for the whole wave: tile addresses are wave-uniform + 4*li

    float acc2[AT][BR];
#pragma unroll
    for (int at = 0; at < AT; at++)
#pragma unroll
        for (int x = 0; x < BR; x++) acc2[at][x] = 0.0f;

    float pre[NPRE];
    // Tile loads go through a buffer descriptor rebuilt per tile (scalar work only): the address of a load is
    // descriptor base (the wave's first column of the tile) + a per-load scalar offset (the column) + one
    // per-lane offset (the row), so no per-load address lives in vector registers, and the descriptor's
    // range check returns 0 for columns past J; lanes whose row is past I get an offset outside any range.
    auto gload = [&](int jt, int it) {
        const int64_t i0 = (int64_t)it * S1_IT, j0 = (int64_t)jt * S1_JT + lj;
        const int64_t org = i0 + p.I * j0;
        int64_t rem = (p.I * p.J - org) * 4;
        rem = rem < 0 ? 0 : (rem > 0x7fffffff ? 0x7fffffff : rem);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(Xk + org), 0, (int)rem, 0x00020000);
        const int voff = (i0 + li < p.I) ? 4 * li : (int)0x80000000;
#pragma unroll
        for (int jj = 0; jj < NPRE; jj++)
            pre[jj] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, (int)(p.I * CG * jj * 4), 0));
    };
    gload(blockIdx.y * p.jt_per, 0);
    const char *xl = (const char *)(xs + lane * S1_XS);
    float *zl = zs + lane * ZS;
    const int jt0 = blockIdx.y * p.jt_per, jt1 = (jt0 + p.jt_per < njt) ? jt0 + p.jt_per : njt;
    for (int jt = jt0; jt < jt1; jt++) {
        for (int t = tid; t < S1_JT * ZS; t += S1_NT) zs[t] = 0.0f;
        for (int it = 0; it < nit; it++) {
            __syncthreads();   // the previous tile's readers are done (and zs is cleared)
#pragma unroll
            for (int jj = 0; jj < NPRE; jj++) xs[(CG * jj + lj) * S1_XS + li] = pre[jj];
            __syncthreads();
            // mode 1: the wave's chunk stream, the next chunk requested before the current one is used
            const S1_CONST int *ocp = as_const((const int *)p.Uoc) + 2 * (it * S1_NW + w);
            const int nch = ocp[1];
            // Lane l holds words 4*(l&3) .. 4*(l&3)+3 of a chunk, so every quad of lanes has the whole chunk and a
            // quad broadcast (folded into the consuming add / multiply-add as a DPP operand) hands any word to
            // all lanes.  Chunks are requested two ahead.
            const i32x4 *cpv = (const i32x4 *)(p.Uch + 16 * (int64_t)ocp[0]) + (lane & 3);
            float s = 0.0f;
            // acc += (word of quad lane q) * x in one instruction.  The compiler does not see inside the asm, so the two
            // wait states a DPP read needs after a VALU write of the same register are put in by hand (S1_FMAC0
            // opens each group; nothing writes the chunk registers between the members of a group)
#define S1_BC(v, q) __builtin_amdgcn_update_dpp(0, v, (q) * 0x55, 0xf, 0xf, true)
#define S1_FMAC(word, x, q) S1_FMAC_(word, x, q, "")
#define S1_FMAC0(word, x, q) S1_FMAC_(word, x, q, "s_nop 1\n\t")
#define S1_FMAC_(word, x, q, pre)                                                                                       \
    asm(pre "v_fmac_f32_dpp %0, %1, %2 quad_perm:[" #q "," #q "," #q "," #q "] row_mask:0xf bank_mask:0xf bound_ctrl:1"    \
        : "+v"(s) : "v"(word), "v"(x))
            auto use = [&](const i32x4 &c) {
                const int h = __builtin_amdgcn_readfirstlane(c.x);
                // the row's running sum over the row tiles lives in zs; its read is issued with the tile reads so
                // that its latency is not waited out separately (LDS atomic adds would not return anything either,
                // but they take a cycle per lane)
                const bool last = (h & CH_LAST) != 0;
                float *za = zl + ((h >> 9) & 0xff);
                const float zold = last ? *za : 0.0f;
                const float x0 = *(const float *)(xl + (S1_BC(c.x, 0) & 0x1ff)), x1 = *(const float *)(xl + S1_BC(c.z, 0));
                const float x2 = *(const float *)(xl + S1_BC(c.x, 1)), x3 = *(const float *)(xl + S1_BC(c.z, 1));
                if (!(h & CH_HALF)) {
                    const float x4 = *(const float *)(xl + S1_BC(c.x, 2)), x5 = *(const float *)(xl + S1_BC(c.z, 2));
                    const float x6 = *(const float *)(xl + S1_BC(c.x, 3)), x7 = *(const float *)(xl + S1_BC(c.z, 3));
                    S1_FMAC0(c.y, x4, 2);
                    S1_FMAC(c.w, x5, 2);
                    S1_FMAC(c.y, x6, 3);
                    S1_FMAC(c.w, x7, 3);
                }
                S1_FMAC0(c.y, x0, 0);
                S1_FMAC(c.w, x1, 0);
                S1_FMAC(c.y, x2, 1);
                S1_FMAC(c.w, x3, 1);
                if (last) {
                    *za = s + zold;
                    s = 0.0f;
                }
            };
            // three chunk registers in rotation (no register copies), requests two chunks ahead
            i32x4 cA = cpv[0], cB = cpv[4], cC;
            for (int ch = 0; ch < nch; ch += 3) {
                cC = cpv[4 * (ch + 2)];
                use(cA);
                if (ch + 1 >= nch) break;
                cA = cpv[4 * (ch + 3)];
                use(cB);
                if (ch + 2 >= nch) break;
                cB = cpv[4 * (ch + 4)];
                use(cC);
            }
#undef S1_BC
#undef S1_FMAC
#undef S1_FMAC0
#undef S1_FMAC_
            // The next tile is requested only now: a wave's loads complete in issue order, so chunk requests queued
            // behind a tile request would wait out the HBM latency.  Other workgroups on the CU cover this one's wait.
            if (it + 1 < nit) gload(jt, it + 1);
            else if (jt + 1 < jt1) gload(jt + 1, 0);
        }
        __syncthreads();   // zs complete
        const S1_CONST int *vp = as_const(p.Vtp) + (int64_t)jt * (p.B1 + 1);
        const S1_CONST int *vent = as_const((const int *)p.Vent);
#pragma unroll
        for (int x = 0; x < BR; x++) {
            const int b = w + S1_NW * x;
            if (b < p.B1) {
                const int e1 = vp[b + 1];
                for (int e = vp[b]; e < e1; e += 4) {
#pragma unroll
                    for (int u = 0; u < 4; u++) {
                        const SEnt n{vent[2 * (e + u)], __int_as_float(vent[2 * (e + u) + 1])};
#pragma unroll
                        for (int at = 0; at < AT; at++) acc2[at][x] = fmaf(n.v, zs[n.c * ZS + 64 * at + lane], acc2[at][x]);
                    }
                }
            }
        }
        __syncthreads();   // zs may be cleared again
    }
    float *Qk = p.Q + blockIdx.y * p.qstride + (p.k0 + k) * p.B1 * p.A1;
#pragma unroll
    for (int x = 0; x < BR; x++) {
        const int b = w + S1_NW * x;
        if (b < p.B1) {
#pragma unroll
            for (int at = 0; at < AT; at++) {
                const int a = 64 * at + lane;
                if (a < p.A1) Qk[(int64_t)b * p.A1 + a] = acc2[at][x];
            }
        }
    }
}


// ---- mode 1 on the matrix cores (U dense in bf16), mode 2 as above -------------------------------------------------
constexpr int SM_NW = 4;            // waves per workgroup
constexpr int SM_CT = 2;            // 32-column tiles per wave
constexpr int SM_TJ = 32 * SM_CT * SM_NW;   // columns per workgroup tile (256)
constexpr int SM_GI = 32;           // rows i per step (two MFMA contraction lengths)

typedef __bf16 s1_bf16x8 __attribute__((ext_vector_type(8)));
typedef float s1_f32x16 __attribute__((ext_vector_type(16)));
typedef float s1_f32x4 __attribute__((ext_vector_type(4)));
typedef s1_f32x4 s1_f32x4_u __attribute__((aligned(4)));   // a column of X starts at a multiple of 4 bytes, not of 16
typedef unsigned int s1_u32x4 __attribute__((ext_vector_type(4)));

struct S1MParams {
    const float *X;
    int64_t I, J;
    int A1, B1;
    const __bf16 *Ud;  // [RT][nks + 1][64 lanes][8]: lane l of fragment (rt, ks) holds U[32 rt + l%32][16 ks + 8 (l/32) .. +7], zero
                       // padded; fragment nks is all zeros (the padding steps of a tile multiply with it)
    const __bf16 *Vd;  // [MT][16 ntile][64 lanes][8]: element e of lane l of fragment (mt, j16) holds
                       // V[32 mt + l%32][16 j16 + 4 (l/32) + e%4 + 8 (e/4)] (the order in which a transposed accumulator holds
                       // its 16 columns), zero padded
    float *Q;          // [K][B1][A1]
    int64_t k0;
};

template <int N, typename F> __device__ __forceinline__ void s1_static_for_(F &&f, std::integral_constant<int, N>, std::integral_constant<int, N>) {}
template <int N, int I_, typename F> __device__ __forceinline__ void s1_static_for_(F &&f, std::integral_constant<int, I_>, std::integral_constant<int, N> n)
{
    f(std::integral_constant<int, I_>());
    s1_static_for_(f, std::integral_constant<int, I_ + 1>(), n);
}
template <int N, typename F> __device__ __forceinline__ void s1_static_for(F &&f) { s1_static_for_(f, std::integral_constant<int, 0>(), std::integral_constant<int, N>()); }

// RT, MT = 32-row tiles of a and of b (A1 <= 32 RT, B1 <= 32 MT), D = steps of X a wave keeps in flight, RAGGED: I is no
// multiple of 32 (what a request reads past the end of a column is set to zero).
//
// Mode 1.  A wave owns 64 columns of the workgroup's 256-column tile and walks down them in steps of 32 rows.  A step's
// 8 KiB are requested with eight 16-byte-per-lane loads that run ALONG the columns (eight lanes cover the 128 bytes of one
// column, a load covers eight columns: every request is a whole cache line), D steps ahead, together with the U fragments
// of the same step -- a wave's loads come back in issue order, so a request with a shorter lead would wait behind the long
// ones and cut their lead to its own.  When a step arrives the wave writes it into its private LDS slot (column-major, the
// 16-byte pieces of a column XOR-swizzled with the column number so that neither the writes along the columns nor the
// fragment reads across them collide on a bank), reads it back as MFMA operands (lane l: column l%32 of a 32-column tile,
// eight consecutive rows), splits each value into three truncated bf16 pieces (8 + 8 + 8 significand bits: the split is
// exact, so are the products with the bf16 U) and issues three MFMAs per row tile, X as first operand: the accumulators
// hold Z^T (rows: columns j, columns: rows a).  Nothing in the step loop waits for another wave: no barrier, no branch
// (steps past the end of a tile are made harmless instead: they multiply a valid step of the same columns with the
// all-zero U fragment).
// Mode 2, at the end of a tile, is on the matrix cores as well: the waves put their Z^T tiles into LDS in operand order
// (registers 8t .. 8t+7 of a transposed accumulator are the 16 columns 16t .. 16t+15 in the order Vd is packed in), and the
// RT x MT blocks of the slice's B1 x A1 result are dealt out to the four waves (block b = mt RT + rt to wave b mod 4), each
// of which adds, over the tile's 16 column blocks, V fragment x split Z^T fragment to the blocks it owns, in registers,
// for the whole slice.  No two waves add to the same number, so every sum has a fixed order.
template <int RT, int MT, int D, bool RAGGED, int WPC = 1>
__global__ __launch_bounds__(64 * SM_NW, WPC) void k_stage1_mfma(const S1MParams p)
{
    extern __shared__ float smem[];
    constexpr int DL = 2;                           // LDS slots per wave
    constexpr int UN = D % DL == 0 ? D : D * DL;    // steps per unrolled group: ring slots are compile-time constants
    constexpr int SLOT = 64 * SM_GI;                // floats per slot: 64 columns x 32 rows
    constexpr int NBW = (RT * MT + SM_NW - 1) / SM_NW;   // result blocks per wave
    constexpr bool ONE_RT = SM_NW % RT == 0;        // all blocks of a wave lie in one row tile rt: its Z fragments are split once
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *xs = smem + w * (DL * SLOT);
    float *zt = smem;                               // Z^T fragments of a finished tile: [16 jb][RT][2 halves][64 lanes][4]
    const int64_t k = blockIdx.x;
    const float *Xk = p.X + k * p.I * p.J;
    const int nks = (int)((p.I + 15) / 16);         // U fragments per row tile (plus the zero fragment)
    const int ng = (int)((p.I + SM_GI - 1) / SM_GI);
    const int ntile = (int)((p.J + SM_TJ - 1) / SM_TJ);
    const int ngp = (ng + UN - 1) / UN * UN;        // steps per tile, padded to whole groups

    s1_f32x16 acc[RT][SM_CT];
#pragma unroll
    for (int rt = 0; rt < RT; rt++)
#pragma unroll
        for (int ct = 0; ct < SM_CT; ct++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[rt][ct][e] = 0.0f;
    s1_f32x16 qacc[NBW];                            // block w + 4 i of the slice's result, transposed: rows b, columns a
#pragma unroll
    for (int i = 0; i < NBW; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) qacc[i][e] = 0.0f;

    // the slice as a buffer: a request past its end (columns past J) returns zeros
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void *)Xk, 0, (int)(p.I * p.J * 4), 0x00020000);
    const int x_lane = (int)(((lane >> 3) * p.I + 4 * (lane & 7)) * 4);        // column lane/8 of a load's eight, piece lane%8
    const int f_lane = lane * 16;
    const __amdgpu_buffer_rsrc_t urs = __builtin_amdgcn_make_buffer_rsrc((void *)p.Ud, 0, (int)((int64_t)RT * (nks + 1) * 1024), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc((void *)p.Vd, 0, (int)((int64_t)MT * 16 * ntile * 1024), 0x00020000);
    // LDS offset (floats) of piece q (4 rows) of column c in a slot
    auto swz = [](int c, int q) { return c * SM_GI + 4 * (q ^ ((c >> 1) & 7)); };

    s1_f32x4 xr[D][8];             // ring of steps of X as requested: xr[d][m] = this lane's piece of load m
    s1_bf16x8 ur[D][2][RT];        // the U fragments of the same steps: [half-step][row tile]

    // requests of padded step n = tile * ngp + g: X of the step itself if it exists, else of the last step of the tile
    // (or of the last tile), which is then multiplied with the zero fragment
    auto request_x = [&](int n, s1_f32x4 (&dst)[8]) {
        int tile = n / ngp, g = n - tile * ngp;
        tile = tile < ntile ? tile : ntile - 1;
        g = g < ng ? g : ng - 1;
        const int soff = (int)((((int64_t)tile * SM_TJ + 64 * w) * p.I + (int64_t)SM_GI * g) * 4);
#pragma unroll
        for (int m = 0; m < 8; m++) {
            s1_f32x4 v = __builtin_bit_cast(s1_f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrs, x_lane, soff + (int)(8 * m * p.I * 4), 0));
            if (RAGGED) {
                const bool in = (int64_t)SM_GI * g + 4 * (lane & 7) < p.I;   // I is a multiple of 4: a piece is inside or outside
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = in ? v[e] : 0.0f;
            }
            dst[m] = v;
        }
    };
    auto request_u = [&](int n, s1_bf16x8 (&dst)[2][RT]) {
        const int tile = n / ngp, g = n - tile * ngp;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            int ks = 2 * g + h;
            ks = (g < ng && ks < nks) ? ks : nks;      // the zero fragment for what lies past the end
#pragma unroll
            for (int rt = 0; rt < RT; rt++)
                dst[h][rt] = __builtin_bit_cast(s1_bf16x8, __builtin_amdgcn_raw_buffer_load_b128(urs, f_lane, (rt * (nks + 1) + ks) * 1024, 0));
        }
    };
    // x = h + m + l with h, m, l the three 8-bit slices of the significand, each a bf16 value (truncation: the residuals
    // are exact); two values per register
    auto split3 = [&](const s1_f32x4 (&x)[2], s1_bf16x8 &h, s1_bf16x8 &m, s1_bf16x8 &l) {
        s1_u32x4 ph, pm, pl;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const float x0 = x[q >> 1][2 * (q & 1)], x1 = x[q >> 1][2 * (q & 1) + 1];
            const unsigned b0 = __builtin_bit_cast(unsigned, x0), b1 = __builtin_bit_cast(unsigned, x1);
            const float r0 = x0 - __builtin_bit_cast(float, b0 & 0xffff0000u), r1 = x1 - __builtin_bit_cast(float, b1 & 0xffff0000u);
            const unsigned c0 = __builtin_bit_cast(unsigned, r0), c1 = __builtin_bit_cast(unsigned, r1);
            const float s0 = r0 - __builtin_bit_cast(float, c0 & 0xffff0000u), s1 = r1 - __builtin_bit_cast(float, c1 & 0xffff0000u);
            ph[q] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
            pm[q] = __builtin_amdgcn_perm(c1, c0, 0x07060302u);
            pl[q] = __builtin_amdgcn_perm(__builtin_bit_cast(unsigned, s1), __builtin_bit_cast(unsigned, s0), 0x07060302u);
        }
        h = __builtin_bit_cast(s1_bf16x8, ph); m = __builtin_bit_cast(s1_bf16x8, pm); l = __builtin_bit_cast(s1_bf16x8, pl);
    };
    // mode 2 on the finished tile
    auto finish_tile = [&](int tile) {
        __syncthreads();   // every wave is done with its slots: the Z^T fragments take the LDS over
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < SM_CT; ct++)
#pragma unroll
                for (int t = 0; t < 2; t++) {
                    const int jb = 4 * w + 2 * ct + t;      // 16-column block of the tile
                    float *dst = zt + ((jb * RT + rt) * 2) * 256 + lane * 4;
                    s1_f32x4 lo, up;
#pragma unroll
                    for (int e = 0; e < 4; e++) { lo[e] = acc[rt][ct][8 * t + e]; up[e] = acc[rt][ct][8 * t + 4 + e]; }
                    *(s1_f32x4 *)dst = lo;
                    *(s1_f32x4 *)(dst + 256) = up;
                }
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int ct = 0; ct < SM_CT; ct++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[rt][ct][e] = 0.0f;
        __syncthreads();
        // V fragments of column block jb for the wave's blocks, requested one block ahead
        s1_bf16x8 vr[2][NBW];
        auto request_v = [&](int jb, s1_bf16x8 (&dst)[NBW]) {
#pragma unroll
            for (int i = 0; i < NBW; i++) {
                const int blk = w + SM_NW * i, mt = blk / RT;    // past the last block: a request past the buffer, zeros
                dst[i] = __builtin_bit_cast(s1_bf16x8, __builtin_amdgcn_raw_buffer_load_b128(vrs, f_lane, (mt * 16 * ntile + 16 * tile + jb) * 1024, 0));
            }
        };
        request_v(0, vr[0]);
#pragma unroll
        for (int jb = 0; jb < 16; jb++) {
            if (jb + 1 < 16) request_v(jb + 1, vr[(jb + 1) & 1]);
            s1_bf16x8 zh, zm, zl;
            if constexpr (ONE_RT) {
                const int rt = w % RT;
                const float *src = zt + ((jb * RT + rt) * 2) * 256 + lane * 4;
                s1_f32x4 x[2];
                x[0] = *(const s1_f32x4 *)src; x[1] = *(const s1_f32x4 *)(src + 256);
                split3(x, zh, zm, zl);
            }
            if constexpr (ONE_RT) {
                // pieces outside, blocks inside: consecutive MFMAs go to different accumulators
#pragma unroll
                for (int i = 0; i < NBW; i++) qacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[jb & 1][i], zl, qacc[i], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < NBW; i++) qacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[jb & 1][i], zm, qacc[i], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < NBW; i++) qacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[jb & 1][i], zh, qacc[i], 0, 0, 0);
            } else {
#pragma unroll
                for (int i = 0; i < NBW; i++) {
                    const int rt = (w + SM_NW * i) % RT;
                    const float *src = zt + ((jb * RT + rt) * 2) * 256 + lane * 4;
                    s1_f32x4 x[2];
                    x[0] = *(const s1_f32x4 *)src; x[1] = *(const s1_f32x4 *)(src + 256);
                    split3(x, zh, zm, zl);
                    qacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[jb & 1][i], zl, qacc[i], 0, 0, 0);
                    qacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[jb & 1][i], zm, qacc[i], 0, 0, 0);
                    qacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[jb & 1][i], zh, qacc[i], 0, 0, 0);
                }
            }
        }
        __syncthreads();   // the slots take the LDS back
    };

    s1_static_for<D>([&](auto dc) {
        constexpr int d = decltype(dc)::value;
        request_x(d, xr[d]);
        request_u(d, ur[d]);
    });
    for (int tile = 0; tile < ntile; tile++) {
        for (int g0 = 0; g0 < ngp; g0 += UN) {
            s1_static_for<UN>([&](auto dc) {
                constexpr int dd = decltype(dc)::value, d = dd % D, sl = dd % DL;
                const int n = tile * ngp + g0 + dd;
                float *slot = xs + sl * SLOT;
                // the step that has arrived goes to the wave's LDS slot, and its registers out again for step n + D
#pragma unroll
                for (int m = 0; m < 8; m++) *(s1_f32x4 *)(slot + swz(8 * m + (lane >> 3), lane & 7)) = xr[d][m];
                request_x(n + D, xr[d]);
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    s1_bf16x8 xp[3][SM_CT];   // pieces l, m, h of the two column tiles
#pragma unroll
                    for (int ct = 0; ct < SM_CT; ct++) {
                        const int j = 32 * ct + l32;
                        s1_f32x4 x[2];
                        x[0] = *(const s1_f32x4 *)(slot + swz(j, 4 * h + 2 * hi));
                        x[1] = *(const s1_f32x4 *)(slot + swz(j, 4 * h + 2 * hi + 1));
                        split3(x, xp[2][ct], xp[1][ct], xp[0][ct]);
                    }
                    // smallest pieces first; consecutive MFMAs go to different accumulators (one that adds to the result of
                    // the instruction before it waits for that result)
#pragma unroll
                    for (int pc = 0; pc < 3; pc++)
#pragma unroll
                        for (int ct = 0; ct < SM_CT; ct++)
#pragma unroll
                            for (int rt = 0; rt < RT; rt++)
                                acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xp[pc][ct], ur[d][h][rt], acc[rt][ct], 0, 0, 0);
                }
                request_u(n + D, ur[d]);
            });
        }
        finish_tile(tile);
    }
    // block (mt, rt) of the wave: register 4 b4 + r of lane l is Q[b = 32 mt + 8 b4 + 4 (l/32) + r][a = 32 rt + l%32]
    float *Qk = p.Q + (p.k0 + k) * p.B1 * p.A1;
#pragma unroll
    for (int i = 0; i < NBW; i++) {
        const int blk = w + SM_NW * i, mt = blk / RT, rt = blk % RT;
        const int a = 32 * rt + l32;
        if (blk < RT * MT && a < p.A1) {
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int b = 32 * mt + 8 * (e >> 2) + 4 * hi + (e & 3);
                if (b < p.B1) Qk[(int64_t)b * p.A1 + a] = qacc[i][e];
            }
        }
    }
}

// Q[0][..] += Q[1][..] + ... + Q[JS-1][..] (the column ranges in order), four floats per thread; n4 = K*A1*B1/4
// rounded up, the allocation is padded accordingly.
__global__ __launch_bounds__(256) void k_stage1_sum_ranges(float *Q, int JS, int64_t stride, int64_t n4)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n4) return;
    float4 a = ((const float4 *)Q)[t];
    for (int js = 1; js < JS; js++) {
        const float4 b = ((const float4 *)(Q + js * stride))[t];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    ((float4 *)Q)[t] = a;
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
    auto qsum = [&](int e) { return p.Q[(int64_t)p.ci[e] * p.AB + ab]; };
    float s = 0.0f;
    int e = p.rp[c];
    for (; e + 4 <= e1; e += 4) {   // four entries' loads in flight together; the sum keeps the stored order
        const float t0 = qsum(e), t1 = qsum(e + 1), t2 = qsum(e + 2), t3 = qsum(e + 3);
        s = fmaf(p.val[e], t0, s);
        s = fmaf(p.val[e + 1], t1, s);
        s = fmaf(p.val[e + 2], t2, s);
        s = fmaf(p.val[e + 3], t3, s);
    }
    for (; e < e1; e++) s = fmaf(p.val[e], qsum(e), s);
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

// Builds the mode-1 chunk streams: per row tile the rows are dealt to the waves longest first (each to the
// wave with the least work so far), and every row's non-zeros inside the tile are cut into chunks of 8.
bool chunk_csr(const exat_csr_t &m, std::vector<int2> &oc, std::vector<int> &ch)
{
    const int nt = (int)((m.cols + S1_IT - 1) / S1_IT);
    std::vector<std::vector<SEnt>> rows((size_t)nt * m.rows);
    for (int r = 0; r < m.rows; r++)
        for (int64_t e = m.rowptr[r]; e < m.rowptr[r + 1]; e++) {
            const int c = m.colidx[e];
            rows[(size_t)(c / S1_IT) * m.rows + r].push_back(SEnt{c % S1_IT, m.val[e]});
        }
    oc.assign((size_t)nt * S1_NW, int2{0, 0});
    ch.clear();
    std::vector<int> order(m.rows);
    for (int t = 0; t < nt; t++) {
        const std::vector<SEnt> *tr = &rows[(size_t)t * m.rows];
        for (int r = 0; r < m.rows; r++) order[r] = r;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return tr[a].size() > tr[b].size(); });
        std::vector<int> mine[S1_NW];
        size_t load[S1_NW] = {};
        for (int r : order) {
            if (tr[r].empty()) continue;
            int best = 0;
            for (int w = 1; w < S1_NW; w++)
                if (load[w] < load[best]) best = w;
            mine[best].push_back(r);
            load[best] += (tr[r].size() + 7) / 8 * 8 + 2;
        }
        for (int w = 0; w < S1_NW; w++) {
            const size_t first = ch.size() / 16;
            for (int r : mine[w]) {
                const auto &v = tr[r];
                for (size_t e = 0; e < v.size(); e += 8) {
                    const size_t n = std::min<size_t>(8, v.size() - e);
                    int word[16];
                    for (size_t u = 0; u < 8; u++) {
                        word[2 * u] = u < n ? 4 * v[e + u].c : 0;
                        const float val = u < n ? v[e + u].v : 0.0f;
                        memcpy(&word[2 * u + 1], &val, 4);
                    }
                    word[0] |= r << 9;
                    if (e + 8 >= v.size()) word[0] |= CH_LAST;
                    if (n <= 4) word[0] |= CH_HALF;
                    ch.insert(ch.end(), word, word + 16);
                }
            }
            if (ch.size() / 16 > 0x7ffffff0u / 16) return false;
            oc[(size_t)t * S1_NW + w] = int2{(int)first, (int)(ch.size() / 16 - first)};
        }
    }
    ch.insert(ch.end(), 32, 0);   // the two chunks the last prefetches of the last stream read
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

template <int AT, int BR>
int launch12(const S1Params &p, dim3 grid, size_t lds, hipStream_t st)
{
    // more than 64 KiB of dynamic LDS has to be allowed per kernel (once per process is enough: the size is fixed by AT)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_stage1_mode12<AT, BR>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return EXAT_ERR_HIP;
    hipLaunchKernelGGL((k_stage1_mode12<AT, BR>), grid, dim3(S1_NT), lds, st, p);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

template <int RT, int MT, int D, bool RAGGED, int WPC = 1>
int launch_mfma_inst(const S1MParams &p, unsigned nk, hipStream_t st)
{
    const size_t zt = (size_t)16 * RT * 2 * 256 * sizeof(float), slots = (size_t)SM_NW * 2 * 64 * SM_GI * sizeof(float);
    const size_t lds = zt > slots ? zt : slots;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_stage1_mfma<RT, MT, D, RAGGED, WPC>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return EXAT_ERR_HIP;
    hipLaunchKernelGGL((k_stage1_mfma<RT, MT, D, RAGGED, WPC>), dim3(nk), dim3(64 * SM_NW), lds, st, p);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}
template <int RT, int MT, int D, int WPC>
int launch_mfma(const S1MParams &p, unsigned nk, hipStream_t st)
{
    return (p.I % SM_GI) ? launch_mfma_inst<RT, MT, D, true, WPC>(p, nk, st) : launch_mfma_inst<RT, MT, D, false, WPC>(p, nk, st);
}
template <int RT, int D, int WPC>
int launch_mfma_rt(const S1MParams &p, unsigned nk, hipStream_t st)
{
    switch ((p.B1 + 31) / 32) {
    case 1: return launch_mfma<RT, 1, D, WPC>(p, nk, st);
    case 2: return launch_mfma<RT, 2, D, WPC>(p, nk, st);
    case 3: return launch_mfma<RT, 3, D, WPC>(p, nk, st);
    default: return launch_mfma<RT, 4, D, WPC>(p, nk, st);
    }
}

// Dense bf16 copy of U in MFMA fragment order, if every value (duplicates summed) is a bf16 value; false otherwise
bool dense_bf16_frags(const exat_csr_t &m, int64_t I, std::vector<uint16_t> &frag)
{
    const int RT = (m.rows + 31) / 32;
    const int64_t nks = (I + 15) / 16;
    std::vector<float> acc((size_t)RT * (nks + 1) * 64 * 8, 0.0f);   // one more fragment per row tile, all zeros
    for (int r = 0; r < m.rows; r++)
        for (int64_t e = m.rowptr[r]; e < m.rowptr[r + 1]; e++) {
            const int64_t i = m.colidx[e];
            const int64_t ks = i / 16;
            const int lane = (r % 32) + 32 * (int)((i % 16) / 8);
            acc[(((size_t)(r / 32) * (nks + 1) + ks) * 64 + lane) * 8 + (size_t)(i % 8)] += m.val[e];
        }
    frag.resize(acc.size());
    for (size_t t = 0; t < acc.size(); t++) {
        uint32_t b;
        memcpy(&b, &acc[t], 4);
        if (b & 0xffffu) return false;
        frag[t] = (uint16_t)(b >> 16);
    }
    return true;
}

// Dense bf16 copy of V in the fragment order of k_stage1_mfma's mode 2 (S1MParams::Vd), if every value is a bf16 value
bool dense_bf16_frags_v(const exat_csr_t &m, int64_t J, std::vector<uint16_t> &frag)
{
    const int MT = (m.rows + 31) / 32;
    const int64_t nj16 = 16 * ((J + SM_TJ - 1) / SM_TJ);
    std::vector<float> acc((size_t)MT * nj16 * 64 * 8, 0.0f);
    for (int r = 0; r < m.rows; r++)
        for (int64_t e = m.rowptr[r]; e < m.rowptr[r + 1]; e++) {
            const int64_t j = m.colidx[e];
            const int c = (int)(j % 16);                            // column inside its block of 16: c = 4 half + e%4 + 8 (e/4)
            const int half = (c >> 2) & 1, el = (c & 3) + 4 * (c >> 3);
            acc[(((size_t)(r / 32) * nj16 + j / 16) * 64 + (r % 32) + 32 * half) * 8 + el] += m.val[e];
        }
    frag.resize(acc.size());
    for (size_t t = 0; t < acc.size(); t++) {
        uint32_t b;
        memcpy(&b, &acc[t], 4);
        if (b & 0xffffu) return false;
        frag[t] = (uint16_t)(b >> 16);
    }
    return true;
}

}  // namespace

struct exat_stage1_s {
    int64_t I, J, K;
    int A1, B1, C1;
    int2 *Uoc = nullptr;
    int *Uch = nullptr, *Vtp = nullptr, *Wrp = nullptr, *Wci = nullptr;
    SEnt *Vent = nullptr;
    float *Wval = nullptr, *Q = nullptr;
    uint16_t *Ud = nullptr;   // dense bf16 U and V in fragment order when the first two modes run on the matrix cores
    uint16_t *Vd = nullptr;   // (k_stage1_mfma), else null
    int JS = 1, jt_per = 1;   // column ranges per slice (more workgroups when K alone would not fill the chip)
    bool timing = false, timing_valid = false;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    // host-streamed application: ring of device buffers holding slabs of frontal slices, a copy stream, and per
    // buffer the events "copied" (copy stream) and "consumed" (compute stream)
    static constexpr int kRing = 3;
    float *ring[kRing] = {nullptr, nullptr, nullptr};
    int64_t slab = 0;   // slices per slab
    hipStream_t copy_stream = nullptr;
    hipEvent_t ev_copied[kRing] = {nullptr, nullptr, nullptr}, ev_free[kRing] = {nullptr, nullptr, nullptr};
    bool ring_used[kRing] = {false, false, false};
};

namespace {
inline int64_t qstride_of(const exat_stage1_s *s) { return ((int64_t)s->K * s->A1 * s->B1 + 3) / 4 * 4; }
}  // namespace

extern "C" {

int exat_stage1_destroy(exat_stage1_t s)
{
    if (!s) return EXAT_OK;
    void *bufs[] = {s->Uoc, s->Uch, s->Vtp, s->Wrp, s->Wci, s->Vent, s->Wval, s->Q, s->Ud, s->Vd};
    for (void *b : bufs)
        if (b) (void)hipFree(b);
    for (auto &e : s->ev)
        if (e) (void)hipEventDestroy(e);
    for (int b = 0; b < exat_stage1_s::kRing; b++) {
        if (s->ring[b]) (void)hipFree(s->ring[b]);
        if (s->ev_copied[b]) (void)hipEventDestroy(s->ev_copied[b]);
        if (s->ev_free[b]) (void)hipEventDestroy(s->ev_free[b]);
    }
    if (s->copy_stream) (void)hipStreamDestroy(s->copy_stream);
    delete s;
    return EXAT_OK;
}

int exat_stage1_create(exat_stage1_t *out, int64_t I, int64_t J, int64_t K, const exat_csr_t *U, const exat_csr_t *V,
                       const exat_csr_t *W)
{
    if (!out) return EXAT_ERR_NULL;
    *out = nullptr;
    if (I < 1 || J < 1 || K < 1 || I > S1_MAXI || J > kMaxExtent1 || K > kMaxExtent1) return EXAT_ERR_SHAPE;
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
        std::vector<int2> oc;
        std::vector<int> ch;
        if (!chunk_csr(*U, oc, ch)) { exat_stage1_destroy(s); return EXAT_ERR_SHAPE; }
        if ((rc = upload(oc, &s->Uoc)) == EXAT_OK) rc = upload(ch, &s->Uch);
        // modes 1 and 2 on the matrix cores when U and V are bf16 matrices (EXAT_STAGE1_MFMA=0 keeps the sparse form: a
        // testing aid).  The kernel reads columns 16 bytes at a time and addresses a slice with 32-bit byte offsets.
        const char *env = getenv("EXAT_STAGE1_MFMA");
        std::vector<uint16_t> fragu, fragv;
        if (rc == EXAT_OK && !(env && atoi(env) == 0) && I % 4 == 0 && I * J * 4 < 2147483647LL && dense_bf16_frags(*U, I, fragu) &&
            dense_bf16_frags_v(*V, J, fragv)) {
            if ((rc = upload(fragu, &s->Ud)) == EXAT_OK) rc = upload(fragv, &s->Vd);
        }
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
    {
        // Column ranges per slice: the workgroups all take about the same time, so the kernel runs in
        // ceil(workgroups / resident workgroups) rounds of ceil(njt / JS) column tiles each; take the smallest JS
        // that minimises the product.
        const int64_t njt = (J + S1_JT - 1) / S1_JT;
        const int64_t slots = 256 * (s->A1 > 64 ? 2 : 3);   // LDS allows 3 (A1 <= 64) or 2 workgroups per CU
        int64_t best = 1, best_cost = -1;
        for (int64_t js = 1; js <= njt && js <= 64; js++) {
            const int64_t per = (njt + js - 1) / js, njs = (njt + per - 1) / per;
            const int64_t cost = ((K * njs + slots - 1) / slots) * per;
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = njs; }
        }
        s->jt_per = (int)((njt + best - 1) / best);
        s->JS = (int)((njt + s->jt_per - 1) / s->jt_per);
        if (s->Ud) { s->JS = 1; s->jt_per = (int)njt; }   // k_stage1_mfma: one workgroup per slice, all its columns
    }
    if (rc == EXAT_OK && hipMalloc((void **)&s->Q, (size_t)s->JS * qstride_of(s) * sizeof(float)) != hipSuccess) {
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

namespace {

// modes 1 and 2 over the nk frontal slices starting at X (slices k0 .. k0+nk-1 of the tensor)
int run_mode12(exat_stage1_s *s, const float *X, int64_t k0, int64_t nk, hipStream_t st)
{
    if (s->Ud) {
        S1MParams m;
        m.X = X; m.I = s->I; m.J = s->J; m.A1 = s->A1; m.B1 = s->B1; m.Ud = (const __bf16 *)s->Ud; m.Vd = (const __bf16 *)s->Vd;
        m.Q = s->Q; m.k0 = k0;
        // Two steps in flight per wave measured best at every size (three or more cost registers and gain nothing: the
        // waves of a compute unit together keep 64 to 128 KiB on their way).  Up to 64 rows a the registers allow two
        // workgroups per compute unit, which is worth more than depth (cfg2: 0.116 -> 0.101 ms).
        switch ((s->A1 + 31) / 32) {
        case 1: return launch_mfma_rt<1, 2, 2>(m, (unsigned)nk, st);
        case 2: return launch_mfma_rt<2, 2, 2>(m, (unsigned)nk, st);
        case 3: return launch_mfma_rt<3, 2, 1>(m, (unsigned)nk, st);
        default: return launch_mfma_rt<4, 2, 1>(m, (unsigned)nk, st);
        }
    }
    S1Params p;
    p.X = X; p.I = s->I; p.J = s->J; p.K = s->K; p.A1 = s->A1; p.B1 = s->B1; p.k0 = k0;
    p.Uoc = s->Uoc; p.Uch = s->Uch; p.Vtp = s->Vtp; p.Vent = s->Vent; p.Q = s->Q; p.jt_per = s->jt_per; p.qstride = qstride_of(s);
    const int AT = s->A1 > 64 ? 2 : 1;
    const size_t lds = (size_t)(S1_JT * S1_XS + S1_JT * (64 * AT + 1)) * sizeof(float);
    const dim3 grid((unsigned)nk, (unsigned)s->JS);
    constexpr int BR1 = 64 / S1_NW, BR2 = 128 / S1_NW;
    if (s->A1 <= 64 && s->B1 <= 64) return launch12<1, BR1>(p, grid, lds, st);
    if (s->A1 <= 64) return launch12<1, BR2>(p, grid, lds, st);
    if (s->B1 <= 64) return launch12<2, BR1>(p, grid, lds, st);
    return launch12<2, BR2>(p, grid, lds, st);
}

// sum of the column ranges, then mode 3
int run_mode3(exat_stage1_s *s, float *X1, hipStream_t st)
{
    if (s->JS > 1) {
        const int64_t n4 = qstride_of(s) / 4;
        hipLaunchKernelGGL(k_stage1_sum_ranges, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, s->Q, s->JS, qstride_of(s), n4);
        if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    }
    S1Mode3Params m;
    m.Q = s->Q; m.rp = s->Wrp; m.ci = s->Wci; m.val = s->Wval; m.X1 = X1; m.AB = (int64_t)s->A1 * s->B1;
    hipLaunchKernelGGL(k_stage1_mode3, dim3((unsigned)((m.AB + 255) / 256), (unsigned)s->C1), dim3(256), 0, st, m);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

}  // namespace

int exat_stage1_apply(exat_stage1_t s, const float *X, float *X1, void *stream)
{
    if (!s || !X || !X1) return EXAT_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (s->timing && hipEventRecord(s->ev[0], st) != hipSuccess) return EXAT_ERR_HIP;
    int rc = run_mode12(s, X, 0, s->K, st);
    if (rc != EXAT_OK) return rc;
    if (s->timing && hipEventRecord(s->ev[1], st) != hipSuccess) return EXAT_ERR_HIP;
    if ((rc = run_mode3(s, X1, st)) != EXAT_OK) return rc;
    if (s->timing) {
        if (hipEventRecord(s->ev[2], st) != hipSuccess) return EXAT_ERR_HIP;
        s->timing_valid = true;
    }
    return EXAT_OK;
}

int exat_stage1_apply_host(exat_stage1_t s, const float *Xhost, float *X1, void *stream)
{
    if (!s || !Xhost || !X1) return EXAT_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const int64_t slice = s->I * s->J;   // elements per frontal slice; slices are contiguous in a column-major tensor
    if (!s->copy_stream) {
        // about 128 MiB per slab; EXAT_STAGE1_SLAB_BYTES overrides the size (testing aid: several slabs on small tensors)
        const char *env = getenv("EXAT_STAGE1_SLAB_BYTES");
        const int64_t target = env && atoll(env) > 0 ? atoll(env) : (int64_t)(128u << 20);
        int64_t slab = target / (slice * 4);
        slab = slab < 1 ? 1 : (slab > s->K ? s->K : slab);
        // default priority: streams of different priorities are never mixed in this library
        if (hipStreamCreateWithFlags(&s->copy_stream, hipStreamNonBlocking) != hipSuccess) { s->copy_stream = nullptr; return EXAT_ERR_HIP; }
        s->slab = slab;
        for (int b = 0; b < exat_stage1_s::kRing; b++) {
            if (hipMalloc((void **)&s->ring[b], (size_t)slab * slice * 4) != hipSuccess) { s->ring[b] = nullptr; (void)hipGetLastError(); return EXAT_ERR_ALLOC; }
            if (hipEventCreateWithFlags(&s->ev_copied[b], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&s->ev_free[b], hipEventDisableTiming) != hipSuccess) return EXAT_ERR_HIP;
        }
    }
    for (int b = 0; b < exat_stage1_s::kRing; b++)
        if (!s->ring[b] || !s->ev_copied[b] || !s->ev_free[b]) return EXAT_ERR_ALLOC;   // an earlier set-up failed half way
    int64_t n = 0;
    for (int64_t k0 = 0; k0 < s->K; k0 += s->slab, n++) {
        const int b = (int)(n % exat_stage1_s::kRing);
        const int64_t nk = k0 + s->slab <= s->K ? s->slab : s->K - k0;
        if (s->ring_used[b] && hipStreamWaitEvent(s->copy_stream, s->ev_free[b], 0) != hipSuccess) return EXAT_ERR_HIP;
        if (hipMemcpyAsync(s->ring[b], Xhost + k0 * slice, (size_t)nk * slice * 4, hipMemcpyHostToDevice, s->copy_stream) != hipSuccess) return EXAT_ERR_HIP;
        if (hipEventRecord(s->ev_copied[b], s->copy_stream) != hipSuccess) return EXAT_ERR_HIP;
        if (hipStreamWaitEvent(st, s->ev_copied[b], 0) != hipSuccess) return EXAT_ERR_HIP;
        const int rc = run_mode12(s, s->ring[b], k0, nk, st);
        if (rc != EXAT_OK) return rc;
        if (hipEventRecord(s->ev_free[b], st) != hipSuccess) return EXAT_ERR_HIP;
        s->ring_used[b] = true;
    }
    return run_mode3(s, X1, st);
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
