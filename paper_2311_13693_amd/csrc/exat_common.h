// Parameter block and MFMA wrappers shared by the mode-1/2 kernels and their common mode-2 phase.
#pragma once
#include "exat_device.h"

namespace exat {

struct Mode12Params {
    const void *U;   // packed [PLpad][Ipad] of T, zero padded
    const float *V;  // packed [P][Mpad][Jpad] fp32, zero padded (bf16-rounded values for bf16 plans)
    const float *Vd; // fp32 plans: V in the order mode2_direct consumes (k_pack_v_direct), else unused
    float *Q;        // [k1-k0][PLpad][Mpad] fp32
    // materialised source: element (i,j,k) at X[(i-xo_i) + (j-xo_j)*x_sj + (k-xo_k)*x_sk]
    const void *X;
    int64_t x_sj, x_sk, xo_i, xo_j, xo_k;
    int x_vec;  // 16-byte loads of X are aligned
    // materialised source held as separate blocks (k_mode12_v3 with TAB): xtab[bi + tab_nbi*(bj + tab_nbj*bk)] is the
    // column-major x_dI x dj x dk block (bi, bj, bk) of X (dj, dk shorter in the last block of an axis); X is unused
    const void *const *xtab;
    int64_t x_dI, x_dJ, x_dK;
    int tab_nbi, tab_nbj;
    // generated source
    const float *A, *B, *C;
    int64_t ldA, ldB, ldC;
    int R, a_vec;  // a_vec: 16-byte loads of A rows are aligned
    uint32_t skey;
    float amp2_ln2;  // -2 ln2 sigma^2, 0 when sigma == 0
    int64_t I, Ipad, Jpad;
    int L, PL, PLpad, Mpad, MT, G;
    int row_base;  // first stacked row of row group 0 of this launch (k_mode12_v3; a multiple of 32, else 0)
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

}  // namespace exat
