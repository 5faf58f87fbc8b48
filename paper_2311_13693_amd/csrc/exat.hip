// C ABI of the exat library (declarations and contracts in include/exat.h): argument
// validation, plan/workspace management and kernel launches.  No compute happens on the host.
#include "../../include/exat.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "exat_aux.h"
#include "exat_mode12.h"
#include "exat_mode12_v2.h"
#include "exat_mode12_v3.h"
#include "exat_mode12_v4.h"
#include "exat_mode12_split.h"

using namespace exat;

namespace {

constexpr int64_t kMaxExtent = 2147483647LL - 64;
constexpr int64_t kSlotBudgetBytes = 4LL << 30;

}  // namespace

struct exat_plan_s {
    exat_desc_t d;
    int PL, PLpad, Mpad, MT, Npad;
    int64_t Ipad, Jpad;
    void *Upack = nullptr;
    void *Ufrag = nullptr;  // U in MFMA fragment order (k_pack_u_frag), same size as Upack
    void *Vfragz = nullptr; // bf16 plans: V in the fragment order of mode2_direct_bf16 (k_pack_v_frag with perm = 1)
    void *Vfrag = nullptr;  // bf16 plans: V in bf16 MFMA fragment order (k_pack_v_frag); fp32 plans: V in the order
                            // mode2_direct consumes (k_pack_v_direct)
    _Float16 *Ufh = nullptr, *Ufl = nullptr, *Vfh = nullptr, *Vfl = nullptr;  // split plans: fp16 pieces in fragment order
    float *Vpack = nullptr, *Wpack = nullptr, *Q = nullptr;
    bool factors_set = false;
    // block-streamed state
    float *slots = nullptr;
    unsigned char *used_dev = nullptr;
    int nslots = 0;
    int64_t nblocks = 0, ysize = 0;
    std::vector<unsigned char> submitted, slot_used;
    int64_t nsubmitted = 0;
    const void **xtab = nullptr;   // device: one pointer per block of X (exat_compress_blocks), [nbk][nbj][nbi]
    // host-streamed compression: ring of device block buffers, a copy stream, and per buffer an event "copy done"
    // (recorded on the copy stream) and an event "buffer consumed" (recorded on the compute stream)
    static constexpr int kRing = 3;
    void *ring[kRing] = {nullptr, nullptr, nullptr};
    hipStream_t copy_stream = nullptr;
    hipEvent_t ev_copied[kRing] = {nullptr, nullptr, nullptr}, ev_free[kRing] = {nullptr, nullptr, nullptr};
    bool ring_used[kRing] = {false, false, false};
    // optional per-kernel timing
    // a ring of event triples, one per compress call, so that a caller can time many calls without waiting in between
    static constexpr int kTimeRing = 128;
    bool timing = false;
    int64_t timed_calls = 0;
    hipEvent_t evr[kTimeRing][3] = {};
    __bf16 *Asplit = nullptr;  // the two 16-bit pieces of the generator's A factor (bf16 or fp16 bit patterns), [2][Ipad][64]
    size_t ub = 0, vb = 0, qb = 0, ab = 0;  // byte sizes of Upack, Vpack, Q, Asplit
};

namespace {

inline int64_t ceil_to(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
// extent of block b along an axis of length n cut into pieces of d (the last piece may be shorter)
inline int64_t blk_ext(int64_t n, int64_t d, int64_t b) { return (b + 1) * d <= n ? d : n - b * d; }
inline size_t esize(int dt) { return dt == EXAT_BF16 ? 2 : 4; }

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return s ? atoi(s) : dflt;
}

// row-tile count per wave of the mode-1/2 kernel (workgroup rows = 128*rt)
int choose_rt(const exat_plan_s *pl, bool generated)
{
    const int forced = env_int("EXAT_RT", 0);
    if (pl->d.in_dtype == EXAT_BF16) {
        if (forced == 2 || forced == 5) return forced;
        return pl->PL > 512 ? 5 : 2;
    }
    if (forced == 1 || forced == 2 || forced == 4) return forced;
    if (pl->PL <= 128) return 1;
    if (generated && pl->PL >= 512) return 4;
    return 2;
}

int validate_desc(const exat_desc_t *d)
{
    if (!d) return EXAT_ERR_NULL;
    if (d->in_dtype != EXAT_F32 && d->in_dtype != EXAT_BF16 && d->in_dtype != EXAT_F32_SPLIT) return EXAT_ERR_DTYPE;
    if (d->I < 1 || d->J < 1 || d->K < 1 || d->I > kMaxExtent || d->J > kMaxExtent || d->K > kMaxExtent) return EXAT_ERR_SHAPE;
    if (d->L < 1 || d->M < 1 || d->N < 1 || d->P < 1 || d->M > 64) return EXAT_ERR_SHAPE;
    if ((int64_t)d->P * d->L >= (1 << 24) || (int64_t)d->P * d->N >= (1 << 24)) return EXAT_ERR_SHAPE;
    if (d->dI < 1 || d->dJ < 1 || d->dK < 1) return EXAT_ERR_SHAPE;
    if (d->dI > d->I || d->dJ > d->J || d->dK > d->K) return EXAT_ERR_SHAPE;
    return EXAT_OK;
}

int validate_gen(const exat_gen_t *g)
{
    if (!g || !g->A || !g->B || !g->C) return EXAT_ERR_NULL;
    if (g->R < 1 || g->R > 256) return EXAT_ERR_SHAPE;
    if (!(g->sigma >= 0.0f) || !(g->sigma < 1e18f)) return EXAT_ERR_SHAPE;
    return EXAT_OK;
}

unsigned grid_for(int64_t n) { int64_t g = (n + 255) / 256; return (unsigned)(g > 65536 ? 65536 : (g < 1 ? 1 : g)); }

float amp2_ln2_of(float sigma) { return sigma == 0.0f ? 0.0f : (float)(-2.0 * 0.69314718055994530942 * (double)sigma * (double)sigma); }

template <typename T, int RT, int CT, int SRC>
int launch_mode12_inst(const Mode12Params &mp, int nk, hipStream_t st)
{
    typedef Mode12Cfg<T, RT, CT> cfg;
    auto kern = k_mode12<T, RT, CT, SRC>;
    static bool attr_done = false;  // per instantiation; setting it twice is harmless
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, cfg::LDS_BYTES) != hipSuccess) return EXAT_ERR_HIP;
        attr_done = true;
    }
    const int64_t grid = 8LL * ((nk + 7) / 8) * mp.G;
    if (grid > 2147483647LL) return EXAT_ERR_SHAPE;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), cfg::LDS_BYTES, st, mp);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

template <int SRC>
int launch_mode12_f32(int rt, const Mode12Params &mp, int nk, hipStream_t st)
{
    switch (rt) {
    case 1: return launch_mode12_inst<float, 1, 4, SRC>(mp, nk, st);
    case 2: return launch_mode12_inst<float, 2, 4, SRC>(mp, nk, st);
    default: return launch_mode12_inst<float, 4, 4, SRC>(mp, nk, st);
    }
}
template <int SRC>
int launch_mode12_bf16(int rt, const Mode12Params &mp, int nk, hipStream_t st)
{
    switch (rt) {
    case 2: return launch_mode12_inst<__bf16, 2, 4, SRC>(mp, nk, st);
    default: return launch_mode12_inst<__bf16, 5, 4, SRC>(mp, nk, st);
    }
}

template <typename T, int NW, int RT, int SRC, int KS, bool BOXED>
int launch_v2_inst(const Mode12Params &mp, const GenSplitParams &gs, int nk, hipStream_t st)
{
    typedef Mode12V2Cfg<NW, RT> cfg;
    auto kern = k_mode12_v2<T, NW, RT, SRC, KS, BOXED>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, cfg::LDS_BYTES) != hipSuccess) return EXAT_ERR_HIP;
        attr_done = true;
    }
    const int64_t grid = 8LL * ((nk + 7) / 8) * mp.G;
    if (grid > 2147483647LL) return EXAT_ERR_SHAPE;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * NW), cfg::LDS_BYTES, st, mp, gs);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

// fp32 generated source (LDS-staged U)
template <int NW, int RT>
int launch_v2_gen_f32(const Mode12Params &mp, const GenSplitParams &gs, int ks, bool boxed, int nk, hipStream_t st)
{
    if (ks == 1) return boxed ? launch_v2_inst<float, NW, RT, SRC_GENERATED, 1, true>(mp, gs, nk, st) : launch_v2_inst<float, NW, RT, SRC_GENERATED, 1, false>(mp, gs, nk, st);
    return boxed ? launch_v2_inst<float, NW, RT, SRC_GENERATED, 2, true>(mp, gs, nk, st) : launch_v2_inst<float, NW, RT, SRC_GENERATED, 2, false>(mp, gs, nk, st);
}

template <typename T, int NW, int RT, int SRC, int KS, bool BOXED, int DU, int DX, int WPS = (NW + 3) / 4, bool ZT = false, bool TAB = false>
int launch_v3_inst(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, int nk, hipStream_t st)
{
    typedef Mode12V3Cfg<NW, RT> cfg;
    auto kern = k_mode12_v3<T, NW, RT, SRC, KS, BOXED, DU, DX, WPS, ZT, TAB>;
    static bool attr_done = false;
    constexpr int lds_max = ZT ? cfg::zt_lds_bytes(2) : cfg::LDS_BYTES;
    static_assert(lds_max <= 160 * 1024, "LDS of a compute unit");
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max) != hipSuccess) return EXAT_ERR_HIP;
        attr_done = true;
    }
    const int64_t grid = 8LL * ((nk + 7) / 8) * mp.G;
    if (grid > 2147483647LL) return EXAT_ERR_SHAPE;
    if (ZT && (mp.MT < 1 || mp.MT > 2)) return EXAT_ERR_SHAPE;
    const int lds = ZT ? cfg::zt_lds_bytes(mp.MT) : cfg::LDS_BYTES;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * NW), lds, st, mp, gs, uf);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

// materialised source: fp32 stages are long (fp32 MFMA), two register sets suffice; bf16 stages are 16 times
// shorter and want the tiles requested further ahead
template <typename T, int NW, int RT, bool TAB = false>
int launch_v3_mat(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, int nk, hipStream_t st)
{
    constexpr int D = sizeof(T) == 2 ? 3 : 2, DXV = sizeof(T) == 2 ? 3 : 1;
    return launch_v3_inst<T, NW, RT, SRC_MATERIALISED, 1, false, D, DXV, (NW + 3) / 4, false, TAB>(mp, gs, uf, nk, st);
}

// fp32 materialised source with mode 2 straight from the (transposed) accumulators; needs L % 32 == 0
template <int NW, int RT>
int launch_v3_mat_zt(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, int nk, hipStream_t st)
{
    return launch_v3_inst<float, NW, RT, SRC_MATERIALISED, 1, false, 2, 1, (NW + 3) / 4, true>(mp, gs, uf, nk, st);
}

// the same over a slab of separate blocks (Mode12Params::xtab)
template <int NW, int RT>
int launch_v3_mat_zt_tab(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, int nk, hipStream_t st)
{
    return launch_v3_inst<float, NW, RT, SRC_MATERIALISED, 1, false, 2, 1, (NW + 3) / 4, true, true>(mp, gs, uf, nk, st);
}

// bf16 generated source, 4 waves
template <int RT>
int launch_v3_gen_bf16(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, int ks, bool boxed, int nk, hipStream_t st)
{
    if (ks == 1) return boxed ? launch_v3_inst<__bf16, 4, RT, SRC_GENERATED, 1, true, 2, 1>(mp, gs, uf, nk, st) : launch_v3_inst<__bf16, 4, RT, SRC_GENERATED, 1, false, 2, 1>(mp, gs, uf, nk, st);
    return boxed ? launch_v3_inst<__bf16, 4, RT, SRC_GENERATED, 2, true, 2, 1>(mp, gs, uf, nk, st) : launch_v3_inst<__bf16, 4, RT, SRC_GENERATED, 2, false, 2, 1>(mp, gs, uf, nk, st);
}

// bf16 generated source, 8 waves x 2 row tiles (512 stacked rows per group), k_mode12_v4
template <bool BOXED>
int launch_v4_inst(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, int nk, hipStream_t st)
{
    typedef Mode12V4Cfg<8, 2> cfg;
    auto kern = k_mode12_v4<8, 2, 1, BOXED, 2, 1, 8>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, cfg::LDS_BYTES) != hipSuccess) return EXAT_ERR_HIP;
        attr_done = true;
    }
    const int64_t grid = 8LL * ((nk + 7) / 8) * mp.G;
    if (grid > 2147483647LL) return EXAT_ERR_SHAPE;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), cfg::LDS_BYTES, st, mp, gs, uf);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}
int launch_v4_gen_bf16(const Mode12Params &mp, const GenSplitParams &gs, const UFragParams &uf, bool boxed, int nk, hipStream_t st)
{
    return boxed ? launch_v4_inst<true>(mp, gs, uf, nk, st) : launch_v4_inst<false>(mp, gs, uf, nk, st);
}

// fp32 data on the fp16 matrix cores (two-piece split), materialised source, 4 waves x RT row tiles
template <int RT, bool TAB = false>
int launch_split(const Mode12Params &mp, const SplitParams &sp, int nk, hipStream_t st)
{
    typedef Mode12SplitCfg<4, RT> cfg;
    auto kern = k_mode12_split<4, RT, 2, 4, TAB>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, cfg::LDS_BYTES) != hipSuccess) return EXAT_ERR_HIP;
        attr_done = true;
    }
    const int64_t grid = 8LL * ((nk + 7) / 8) * mp.G;
    if (grid > 2147483647LL) return EXAT_ERR_SHAPE;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), cfg::LDS_BYTES, st, mp, sp);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

// fills the plan-dependent part of the parameters and launches mode 1+2 followed by mode 3
int run_chain(exat_plan_s *pl, Mode12Params mp, bool generated, float *Yout, int accumulate, hipStream_t st, unsigned char *flag = nullptr)
{
    // The pipelined kernels need whole 64-byte stages of i inside the box (materialised source) or a factor
    // rank that fits their generator (generated source); everything else takes the generic kernel.
    // EXAT_PIPELINED=0 forces the generic kernel (a testing aid).
    const bool bf = pl->d.in_dtype == EXAT_BF16;
    const int ei = bf ? 32 : 16;
    bool pipelined = env_int("EXAT_PIPELINED", 1) != 0;
    if (generated) pipelined = pipelined && mp.R <= 64;
    else pipelined = pipelined && mp.x_vec && (mp.i0 % ei == 0) && ((mp.i1 - mp.i0) % ei == 0);
    // only k_mode12_v3<..., TAB> and k_mode12_split<..., TAB> read the block table
    if (mp.xtab && (generated || (pl->d.in_dtype == EXAT_F32_SPLIT ? (mp.i0 % 32 != 0 || (mp.i1 - mp.i0) % 32 != 0) : !pipelined))) return EXAT_ERR_STATE;
    int rt = choose_rt(pl, generated);
    if (pipelined) {
        // rt = 128-row units of the workgroup tile: 2 = 4 waves x 2 row tiles, 3 = 4 waves x 3, 4 = 8 waves x 2
        const int forced = env_int("EXAT_RT", 0);
        rt = (forced == 2 || forced == 4) ? forced : (pl->PL > 256 ? 4 : 2);
        // bf16 generated source: 4 waves x 3 row tiles (384 stacked rows), one wave per SIMD, unless told otherwise
        if (bf && generated && pl->PL > 256 && forced != 2 && forced != 4) rt = 3;
        // the bf16 generator has no 8-wave build
        if (bf && generated && rt == 4) rt = 3;
        // bf16 materialised source: the 8-wave build spills around its mode-2 phase and measured 2.5 times slower than the
        // 4-wave one on a 10000 x 10000 x 256 slab (621 against 251 ms)
        if (bf && !generated && forced == 0) rt = 2;
        // a small box (one streamed block) with 512-row groups would not give every compute unit a workgroup
        if (!generated && rt == 4 && forced == 0 && (mp.k1 - mp.k0) * ((pl->PL + 511) / 512) < 256) rt = 2;
    }
    // the LDS-staged fp32 generator kernel (k_mode12_v2) addresses its U tile with 32-bit element offsets of up to
    // 255 rows: beyond 2^23 padded columns the generic kernel takes over
    const bool f32_gen_v3 = rt == 4 && pl->d.L % 32 == 0 && env_int("EXAT_F32_GEN_V3", 1);
    if (pipelined && generated && !bf && !f32_gen_v3 && pl->Ipad > (1LL << 23)) { pipelined = false; rt = choose_rt(pl, generated); }
    // fp32 data on the fp16 matrix cores: materialised sources with whole 32-value stages of i inside the box
    const bool split = pl->d.in_dtype == EXAT_F32_SPLIT && !generated && mp.x_vec && (mp.i0 % 32 == 0) && ((mp.i1 - mp.i0) % 32 == 0);
    const int rows = 128 * rt;
    mp.U = pl->Upack; mp.V = pl->Vpack; mp.Q = pl->Q;
    mp.Vd = pl->d.in_dtype == EXAT_BF16 ? nullptr : (const float *)pl->Vfrag;
    mp.I = pl->d.I; mp.Ipad = pl->Ipad; mp.Jpad = pl->Jpad;
    mp.L = pl->d.L; mp.PL = pl->PL; mp.PLpad = pl->PLpad; mp.Mpad = pl->Mpad; mp.MT = pl->MT;
    mp.G = (pl->PL + rows - 1) / rows;
    const int nk = (int)(mp.k1 - mp.k0);
    int rc;
    GenSplitParams gs;
    gs.Asp = pl->Asplit; gs.Irows = pl->Ipad; gs.Rpad = 32 * ((mp.R + 31) / 32);
    if (pipelined && generated) {
        const int64_t n = gs.Irows * gs.Rpad;
        if (bf) hipLaunchKernelGGL(k_split_a<__bf16>, dim3(grid_for(n)), dim3(256), 0, st, mp.A, pl->d.I, mp.R, pl->Asplit, gs.Irows, gs.Rpad);
        else hipLaunchKernelGGL(k_split_a<float>, dim3(grid_for(n)), dim3(256), 0, st, mp.A, pl->d.I, mp.R, pl->Asplit, gs.Irows, gs.Rpad);
        if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    }
    hipEvent_t *ev = pl->evr[pl->timed_calls % exat_plan_s::kTimeRing];
    if (pl->timing && hipEventRecord(ev[0], st) != hipSuccess) return EXAT_ERR_HIP;
    if (split) {
        SplitParams sp;
        sp.Ufh = pl->Ufh; sp.Ufl = pl->Ufl; sp.nig = pl->Ipad / 16; sp.Vfh = pl->Vfh; sp.Vfl = pl->Vfl;
        // 256-row groups (one wave per SIMD, 2 row tiles; measured a little faster than 384-row groups); a
        // remainder of at most 128 rows gets a launch of its own with one row tile per wave
        const int full = pl->PL / 256, rem = pl->PL - 256 * full;
        rc = EXAT_OK;
        if (full > 0 || rem > 128) { mp.G = rem > 128 ? full + 1 : full; rc = mp.xtab ? launch_split<2, true>(mp, sp, nk, st) : launch_split<2>(mp, sp, nk, st); }
        if (rc == EXAT_OK && rem > 0 && rem <= 128) {
            mp.row_base = 256 * full; mp.G = 1;
            rc = mp.xtab ? launch_split<1, true>(mp, sp, nk, st) : launch_split<1>(mp, sp, nk, st);
        }
    } else if (pipelined) {
        const bool boxed = generated && (mp.i0 != 0 || mp.i1 != pl->d.I);
        const int ks = gs.Rpad / 32;
        UFragParams uf;
        uf.Uf = pl->Ufrag; uf.nig = pl->Ipad / (bf ? 16 : 8); uf.Vf = pl->Vfrag; uf.Vz = pl->Vfragz;
        if (!generated) {
            if (mp.xtab) {   // a slab of blocks (exat_compress_blocks has checked that these kernels apply)
                if (bf) rc = rt == 4 ? launch_v3_mat<__bf16, 8, 2, true>(mp, gs, uf, nk, st) : launch_v3_mat<__bf16, 4, 2, true>(mp, gs, uf, nk, st);
                else if (pl->d.L % 32 == 0 && env_int("EXAT_ZT", 1))
                    rc = rt == 4 ? launch_v3_mat_zt_tab<8, 2>(mp, gs, uf, nk, st) : launch_v3_mat_zt_tab<4, 2>(mp, gs, uf, nk, st);
                else rc = rt == 4 ? launch_v3_mat<float, 8, 2, true>(mp, gs, uf, nk, st) : launch_v3_mat<float, 4, 2, true>(mp, gs, uf, nk, st);
            } else if (bf) rc = rt == 4 ? launch_v3_mat<__bf16, 8, 2>(mp, gs, uf, nk, st) : launch_v3_mat<__bf16, 4, 2>(mp, gs, uf, nk, st);
            else if (pl->d.L % 32 == 0 && env_int("EXAT_ZT", 1))
                rc = rt == 4 ? launch_v3_mat_zt<8, 2>(mp, gs, uf, nk, st) : launch_v3_mat_zt<4, 2>(mp, gs, uf, nk, st);
            else rc = rt == 4 ? launch_v3_mat<float, 8, 2>(mp, gs, uf, nk, st) : launch_v3_mat<float, 4, 2>(mp, gs, uf, nk, st);
        } else if (bf && pl->PL > 256 && ks == 1 && env_int("EXAT_RT", 0) == 0 && pl->Ipad < (1LL << 21)) {
            // 512-row groups, two waves per SIMD (k_mode12_v4): the tile is generated once per group, so large groups
            // are what keeps the generator's vector work below the MFMA work.  Factor ranks above 32 would need twice
            // the generator registers, which this build does not have: they take the 384-row kernel below.  The kernel
            // addresses U and the generator's A pieces with 32-bit byte offsets (a wave's two row tiles are 8 tiles, 576
            // bytes per padded column, apart): 2^21 padded columns and more take the 384-row kernel as well.
            mp.G = (pl->PL + 511) / 512;
            rc = launch_v4_gen_bf16(mp, gs, uf, boxed, nk, st);
        } else if (bf) {
            if (rt == 3) {
                // 384-row groups; a remainder of at most 256 rows gets a launch of its own with a smaller tile
                // instead of a mostly empty group (the generator's vector work per group does not shrink with
                // the rows, the MFMA work does)
                const int full = pl->PL / 384, rem = pl->PL - 384 * full;
                rc = EXAT_OK;
                if (full > 0 && (rem == 0 || rem <= 256)) {
                    mp.G = full;
                    rc = launch_v3_gen_bf16<3>(mp, gs, uf, ks, boxed, nk, st);
                    if (rc == EXAT_OK && rem > 0) {
                        mp.row_base = 384 * full; mp.G = 1;
                        rc = rem <= 128 ? launch_v3_gen_bf16<1>(mp, gs, uf, ks, boxed, nk, st) : launch_v3_gen_bf16<2>(mp, gs, uf, ks, boxed, nk, st);
                    }
                } else
                    rc = launch_v3_gen_bf16<3>(mp, gs, uf, ks, boxed, nk, st);
            } else rc = launch_v3_gen_bf16<2>(mp, gs, uf, ks, boxed, nk, st);
        } else if (f32_gen_v3) {
            // fp32 generator, 8 waves x 2 row tiles, U fragments straight into registers and mode 2 straight from the
            // accumulators (the register-hungry LDS transposition of mode 2 was what made this build spill in its stage
            // loop); EXAT_F32_GEN_V3=0 selects the LDS-staged kernel below
            if (ks == 1) rc = boxed ? launch_v3_inst<float, 8, 2, SRC_GENERATED, 1, true, 2, 1, 2, true>(mp, gs, uf, nk, st)
                                    : launch_v3_inst<float, 8, 2, SRC_GENERATED, 1, false, 2, 1, 2, true>(mp, gs, uf, nk, st);
            else rc = boxed ? launch_v3_inst<float, 8, 2, SRC_GENERATED, 2, true, 2, 1, 2, true>(mp, gs, uf, nk, st)
                            : launch_v3_inst<float, 8, 2, SRC_GENERATED, 2, false, 2, 1, 2, true>(mp, gs, uf, nk, st);
        } else {
            // LDS-staged fp32 generator kernel, 4 waves x 2 row tiles (256-row groups) only: its 8-wave build is not
            // instantiated (the bf16 build of that shape once faulted at the 10000^3 size, cause unknown)
            mp.G = (pl->PL + 255) / 256;
            rc = launch_v2_gen_f32<4, 2>(mp, gs, ks, boxed, nk, st);
        }
    } else if (pl->d.in_dtype == EXAT_BF16)
        rc = generated ? launch_mode12_bf16<SRC_GENERATED>(rt, mp, nk, st) : launch_mode12_bf16<SRC_MATERIALISED>(rt, mp, nk, st);
    else
        rc = generated ? launch_mode12_f32<SRC_GENERATED>(rt, mp, nk, st) : launch_mode12_f32<SRC_MATERIALISED>(rt, mp, nk, st);
    if (rc != EXAT_OK) return rc;
    if (pl->timing && hipEventRecord(ev[1], st) != hipSuccess) return EXAT_ERR_HIP;
    Mode3Params m3;
    m3.Q = pl->Q; m3.W = pl->Wpack; m3.Y = Yout;
    m3.L = pl->d.L; m3.M = pl->d.M; m3.N = pl->d.N; m3.PL = pl->PL; m3.PLpad = pl->PLpad; m3.Mpad = pl->Mpad;
    m3.Npad = pl->Npad;
    m3.K = pl->d.K; m3.k0 = mp.k0; m3.k1 = mp.k1; m3.accumulate = accumulate; m3.flag = flag;
    const int64_t ntile = ((int64_t)pl->PL * pl->Mpad + 31) / 32;
    dim3 grid((unsigned)ntile, (unsigned)((pl->Npad + 63) / 64));
    const bool longk = (m3.k1 - m3.k0) > 512LL * M3_WAVES - 8;   // a wave's slab (rounded up to even) may exceed 512
    if (pl->Npad % 64 == 0) {
        if (longk) hipLaunchKernelGGL((k_mode3<2, true>), grid, dim3(64 * M3_WAVES), 0, st, m3);
        else hipLaunchKernelGGL((k_mode3<2, false>), grid, dim3(64 * M3_WAVES), 0, st, m3);
    } else {  // 32-column tiles, so that no launch carries an idle second tile
        grid.y = (unsigned)(pl->Npad / 32);
        if (longk) hipLaunchKernelGGL((k_mode3<1, true>), grid, dim3(64 * M3_WAVES), 0, st, m3);
        else hipLaunchKernelGGL((k_mode3<1, false>), grid, dim3(64 * M3_WAVES), 0, st, m3);
    }
    if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    if (pl->timing) {
        if (hipEventRecord(ev[2], st) != hipSuccess) return EXAT_ERR_HIP;
        pl->timed_calls++;
    }
    return EXAT_OK;
}

__global__ void k_clear_flags(unsigned char *flags, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) flags[i] = 0;
}

// up to 32 entries of the block-pointer table per launch, carried in the kernel arguments
struct PtrChunk { const void *p[32]; int64_t idx[32]; };
__global__ void k_set_ptrs(const void **tab, PtrChunk c, int n)
{
    const int t = threadIdx.x;
    if (t < n) tab[c.idx[t]] = c.p[t];
}

// the partial-result slots of the block-streamed calls, allocated at their first use with a plan
int ensure_slots(exat_plan_s *pl, hipStream_t st)
{
    if (pl->slots) return EXAT_OK;
    int64_t ns = kSlotBudgetBytes / (pl->ysize * 4);
    if (ns < 1) ns = 1;
    if (ns > pl->nblocks) ns = pl->nblocks;
    if (ns > (1 << 20)) ns = 1 << 20;
    if (hipMalloc((void **)&pl->slots, (size_t)ns * pl->ysize * 4) != hipSuccess || hipMalloc((void **)&pl->used_dev, (size_t)ns) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(pl->slots); (void)hipFree(pl->used_dev);
        pl->slots = nullptr; pl->used_dev = nullptr;
        return EXAT_ERR_ALLOC;
    }
    pl->nslots = (int)ns;
    pl->submitted.assign((size_t)pl->nblocks, 0);
    pl->slot_used.assign((size_t)ns, 0);
    pl->nsubmitted = 0;
    hipLaunchKernelGGL(k_clear_flags, dim3(grid_for(ns)), dim3(256), 0, st, pl->used_dev, (int)ns);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

}  // namespace

extern "C" {

int exat_plan_create(exat_plan_t *plan, const exat_desc_t *desc)
{
    if (!plan) return EXAT_ERR_NULL;
    *plan = nullptr;
    int rc = validate_desc(desc);
    if (rc != EXAT_OK) return rc;
    exat_plan_s *pl = new (std::nothrow) exat_plan_s();
    if (!pl) return EXAT_ERR_ALLOC;
    pl->d = *desc;
    pl->PL = desc->P * desc->L;
    pl->MT = (desc->M + 31) / 32;
    pl->Mpad = 32 * pl->MT;
    pl->Npad = 32 * ((desc->N + 31) / 32);
    pl->Ipad = ceil_to(desc->I, 32);
    pl->Jpad = ceil_to(desc->J, 256);
    // every kernel variant the plan may pick must find its row groups inside the padding
    int64_t plpad = 0;
    const int rts_f32[] = {1, 2, 3, 4}, rts_bf16[] = {2, 3, 4, 5};
    if (desc->in_dtype == EXAT_BF16) { for (int rt : rts_bf16) { int64_t v = ceil_to(pl->PL, 128 * rt); if (v > plpad) plpad = v; } }
    else { for (int rt : rts_f32) { int64_t v = ceil_to(pl->PL, 128 * rt); if (v > plpad) plpad = v; } }
    pl->PLpad = (int)plpad;
    const size_t es = esize(desc->in_dtype);
    const size_t ub = (size_t)pl->PLpad * pl->Ipad * es;
    const size_t vb = (size_t)desc->P * pl->Mpad * pl->Jpad * 4;
    const size_t wb = (size_t)desc->P * desc->K * pl->Npad * 4;
    const size_t qb = (size_t)desc->K * pl->PLpad * pl->Mpad * 4;
    pl->ub = ub; pl->vb = vb; pl->qb = qb; pl->ab = (size_t)3 * pl->Ipad * 64 * 2;
    if (hipMalloc((void **)&pl->Asplit, pl->ab) != hipSuccess ||
        hipMalloc(&pl->Upack, ub) != hipSuccess || hipMalloc(&pl->Ufrag, ub) != hipSuccess ||
        (desc->in_dtype == EXAT_BF16 && (hipMalloc(&pl->Vfrag, (size_t)desc->P * pl->Jpad * 64 * 2) != hipSuccess ||
                                         hipMalloc(&pl->Vfragz, (size_t)desc->P * pl->Jpad * 64 * 2) != hipSuccess)) ||
        (desc->in_dtype != EXAT_BF16 && hipMalloc(&pl->Vfrag, (size_t)desc->P * pl->Mpad * pl->Jpad * 4) != hipSuccess) ||
        (desc->in_dtype == EXAT_F32_SPLIT &&
         (hipMalloc((void **)&pl->Ufh, (size_t)pl->PLpad * pl->Ipad * 2) != hipSuccess || hipMalloc((void **)&pl->Ufl, (size_t)pl->PLpad * pl->Ipad * 2) != hipSuccess ||
          hipMalloc((void **)&pl->Vfh, (size_t)desc->P * pl->Jpad * 64 * 2) != hipSuccess || hipMalloc((void **)&pl->Vfl, (size_t)desc->P * pl->Jpad * 64 * 2) != hipSuccess)) || hipMalloc((void **)&pl->Vpack, vb) != hipSuccess ||
        hipMalloc((void **)&pl->Wpack, wb) != hipSuccess || hipMalloc((void **)&pl->Q, qb) != hipSuccess) {
        (void)hipGetLastError();
        exat_plan_destroy(pl);
        return EXAT_ERR_ALLOC;
    }
    pl->nblocks = cdiv(desc->I, desc->dI) * cdiv(desc->J, desc->dJ) * cdiv(desc->K, desc->dK);
    pl->ysize = (int64_t)desc->P * desc->L * desc->M * desc->N;
    *plan = pl;
    return EXAT_OK;
}

int exat_plan_destroy(exat_plan_t pl)
{
    if (pl) {
        for (int b = 0; b < exat_plan_s::kRing; b++) {
            if (pl->ring[b]) (void)hipFree(pl->ring[b]);
            if (pl->ev_copied[b]) (void)hipEventDestroy(pl->ev_copied[b]);
            if (pl->ev_free[b]) (void)hipEventDestroy(pl->ev_free[b]);
        }
        if (pl->copy_stream) (void)hipStreamDestroy(pl->copy_stream);
    }
    if (!pl) return EXAT_OK;
    (void)hipFree(pl->Upack); (void)hipFree(pl->Ufrag); (void)hipFree(pl->Vfrag); (void)hipFree(pl->Vfragz);
    (void)hipFree(pl->Ufh); (void)hipFree(pl->Ufl); (void)hipFree(pl->Vfh); (void)hipFree(pl->Vfl); (void)hipFree(pl->Vpack); (void)hipFree(pl->Wpack); (void)hipFree(pl->Q);
    (void)hipFree(pl->slots); (void)hipFree(pl->used_dev); (void)hipFree(pl->Asplit); (void)hipFree((void *)pl->xtab);
    for (auto &tr : pl->evr)
        for (hipEvent_t e : tr) if (e) (void)hipEventDestroy(e);
    delete pl;
    return EXAT_OK;
}

int exat_set_factors(exat_plan_t pl, const float *U, int64_t ldU, const float *V, int64_t ldV,
                     const float *W, int64_t ldW, void *stream)
{
    if (!pl || !U || !V || !W) return EXAT_ERR_NULL;
    const exat_desc_t &d = pl->d;
    if (ldU < d.I || ldV < d.J || ldW < d.K) return EXAT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const int64_t nu = (int64_t)pl->PLpad * pl->Ipad, nv = (int64_t)d.P * pl->Mpad * pl->Jpad, nw = (int64_t)d.P * d.K * pl->Npad;
    if (d.in_dtype == EXAT_BF16) {
        hipLaunchKernelGGL(k_pack_u<__bf16>, dim3(grid_for(nu)), dim3(256), 0, st, U, ldU, pl->PL, d.I, (__bf16 *)pl->Upack, pl->PLpad, pl->Ipad);
        hipLaunchKernelGGL(k_pack_u_frag<__bf16>, dim3(grid_for(nu)), dim3(256), 0, st, U, ldU, pl->PL, d.I, (__bf16 *)pl->Ufrag, pl->PLpad / 32, pl->Ipad / 16);
        hipLaunchKernelGGL(k_pack_v_frag, dim3(grid_for((int64_t)d.P * pl->Jpad * 64)), dim3(256), 0, st, V, ldV, d.P, d.M, d.J, (__bf16 *)pl->Vfrag, pl->Jpad, 0);
        hipLaunchKernelGGL(k_pack_v_frag, dim3(grid_for((int64_t)d.P * pl->Jpad * 64)), dim3(256), 0, st, V, ldV, d.P, d.M, d.J, (__bf16 *)pl->Vfragz, pl->Jpad, 1);
        hipLaunchKernelGGL(k_pack_v<__bf16>, dim3(grid_for(nv)), dim3(256), 0, st, V, ldV, d.P, d.M, d.J, pl->Vpack, pl->Mpad, pl->Jpad);
        hipLaunchKernelGGL(k_pack_w<__bf16>, dim3(grid_for(nw)), dim3(256), 0, st, W, ldW, d.P, d.N, d.K, pl->Wpack, pl->Npad);
    } else {
        if (d.in_dtype == EXAT_F32_SPLIT) {
            hipLaunchKernelGGL(k_pack_u_split, dim3(grid_for(nu)), dim3(256), 0, st, U, ldU, pl->PL, d.I, pl->Ufh, pl->Ufl, pl->PLpad / 32, pl->Ipad / 16);
            hipLaunchKernelGGL(k_pack_v_split, dim3(grid_for((int64_t)d.P * pl->Jpad * 64)), dim3(256), 0, st, V, ldV, d.P, d.M, d.J, pl->Vfh, pl->Vfl, pl->Jpad);
        }
        hipLaunchKernelGGL(k_pack_u<float>, dim3(grid_for(nu)), dim3(256), 0, st, U, ldU, pl->PL, d.I, (float *)pl->Upack, pl->PLpad, pl->Ipad);
        hipLaunchKernelGGL(k_pack_u_frag<float>, dim3(grid_for(nu)), dim3(256), 0, st, U, ldU, pl->PL, d.I, (float *)pl->Ufrag, pl->PLpad / 32, pl->Ipad / 8);
        hipLaunchKernelGGL(k_pack_v<float>, dim3(grid_for(nv)), dim3(256), 0, st, V, ldV, d.P, d.M, d.J, pl->Vpack, pl->Mpad, pl->Jpad);
        hipLaunchKernelGGL(k_pack_v_direct, dim3(grid_for(nv)), dim3(256), 0, st, V, ldV, d.P, d.M, d.J, (float *)pl->Vfrag, pl->Mpad, pl->Jpad);
        hipLaunchKernelGGL(k_pack_w<float>, dim3(grid_for(nw)), dim3(256), 0, st, W, ldW, d.P, d.N, d.K, pl->Wpack, pl->Npad);
    }
    if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    pl->factors_set = true;
    return EXAT_OK;
}

int exat_compress(exat_plan_t pl, const void *X, float *Y, void *stream)
{
    if (!pl || !X || !Y) return EXAT_ERR_NULL;
    if (!pl->factors_set) return EXAT_ERR_STATE;
    const exat_desc_t &d = pl->d;
    Mode12Params mp;
    memset(&mp, 0, sizeof(mp));
    mp.X = X; mp.x_sj = d.I; mp.x_sk = d.I * d.J;
    const int e16 = 16 / (int)esize(d.in_dtype);
    mp.x_vec = (d.I % e16 == 0) && (((uintptr_t)X & 15) == 0);
    mp.i0 = 0; mp.i1 = d.I; mp.j0 = 0; mp.j1 = d.J; mp.k0 = 0; mp.k1 = d.K;
    return run_chain(pl, mp, false, Y, 0, (hipStream_t)stream);
}

int exat_compress_gen(exat_plan_t pl, const exat_gen_t *gen, const exat_box_t *box, float *Y, void *stream)
{
    if (!pl || !Y) return EXAT_ERR_NULL;
    int rc = validate_gen(gen);
    if (rc != EXAT_OK) return rc;
    if (!pl->factors_set) return EXAT_ERR_STATE;
    const exat_desc_t &d = pl->d;
    exat_box_t b = {0, d.I, 0, d.J, 0, d.K};
    if (box) b = *box;
    if (b.i0 < 0 || b.j0 < 0 || b.k0 < 0 || b.i1 > d.I || b.j1 > d.J || b.k1 > d.K || b.i0 >= b.i1 || b.j0 >= b.j1 || b.k0 >= b.k1)
        return EXAT_ERR_SHAPE;
    Mode12Params mp;
    memset(&mp, 0, sizeof(mp));
    mp.A = gen->A; mp.B = gen->B; mp.C = gen->C; mp.ldA = d.I; mp.ldB = d.J; mp.ldC = d.K; mp.R = gen->R;
    mp.a_vec = (d.I % 4 == 0) && (((uintptr_t)gen->A & 15) == 0);
    mp.skey = seed_key(gen->seed);
    mp.amp2_ln2 = amp2_ln2_of(gen->sigma);
    mp.i0 = b.i0; mp.i1 = b.i1; mp.j0 = b.j0; mp.j1 = b.j1; mp.k0 = b.k0; mp.k1 = b.k1;
    return run_chain(pl, mp, true, Y, 0, (hipStream_t)stream);
}

int exat_compress_block(exat_plan_t pl, const void *Xblk, int32_t bi, int32_t bj, int32_t bk, void *stream)
{
    if (!pl || !Xblk) return EXAT_ERR_NULL;
    if (!pl->factors_set) return EXAT_ERR_STATE;
    const exat_desc_t &d = pl->d;
    const int64_t nbi = cdiv(d.I, d.dI), nbj = cdiv(d.J, d.dJ), nbk = cdiv(d.K, d.dK);
    if (bi < 0 || bj < 0 || bk < 0 || bi >= nbi || bj >= nbj || bk >= nbk) return EXAT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const int rcs = ensure_slots(pl, st);
    if (rcs != EXAT_OK) return rcs;
    const int64_t blk = bi + nbi * (bj + nbj * (int64_t)bk);
    if (pl->submitted[(size_t)blk]) return EXAT_ERR_STATE;
    const int slot = (int)(blk % pl->nslots);
    Mode12Params mp;
    memset(&mp, 0, sizeof(mp));
    const int64_t di = blk_ext(d.I, d.dI, bi), dj = blk_ext(d.J, d.dJ, bj), dk = blk_ext(d.K, d.dK, bk);
    mp.X = Xblk; mp.x_sj = di; mp.x_sk = di * dj;
    mp.xo_i = (int64_t)bi * d.dI; mp.xo_j = (int64_t)bj * d.dJ; mp.xo_k = (int64_t)bk * d.dK;
    const int e16 = 16 / (int)esize(d.in_dtype);
    mp.x_vec = (di % e16 == 0) && (mp.xo_i % e16 == 0) && (((uintptr_t)Xblk & 15) == 0);
    mp.i0 = mp.xo_i; mp.i1 = mp.xo_i + di; mp.j0 = mp.xo_j; mp.j1 = mp.xo_j + dj; mp.k0 = mp.xo_k; mp.k1 = mp.xo_k + dk;
    // the mode-3 launch of the block marks its slot as holding a partial result (the merge adds marked slots only)
    int rc = run_chain(pl, mp, false, pl->slots + (int64_t)slot * pl->ysize, pl->slot_used[(size_t)slot] ? 1 : 0, st,
                       pl->slot_used[(size_t)slot] ? nullptr : pl->used_dev + slot);
    if (rc != EXAT_OK) return rc;
    pl->slot_used[(size_t)slot] = 1;
    pl->submitted[(size_t)blk] = 1;
    pl->nsubmitted++;
    return EXAT_OK;
}

int exat_compress_blocks(exat_plan_t pl, const void *const *Xblk, int32_t bj0, int32_t bj1, int32_t bk0, int32_t bk1, void *stream)
{
    if (!pl || !Xblk) return EXAT_ERR_NULL;
    if (!pl->factors_set) return EXAT_ERR_STATE;
    const exat_desc_t &d = pl->d;
    const int64_t nbi = cdiv(d.I, d.dI), nbj = cdiv(d.J, d.dJ), nbk = cdiv(d.K, d.dK);
    if (bj0 < 0 || bk0 < 0 || bj0 >= bj1 || bk0 >= bk1 || bj1 > nbj || bk1 > nbk) return EXAT_ERR_SHAPE;
    const int64_t n = nbi * (bj1 - bj0) * (int64_t)(bk1 - bk0);
    for (int64_t q = 0; q < n; q++)
        if (!Xblk[q]) return EXAT_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const int rcs = ensure_slots(pl, st);
    if (rcs != EXAT_OK) return rcs;
    for (int64_t bk = bk0; bk < bk1; bk++)
        for (int64_t bj = bj0; bj < bj1; bj++)
            for (int64_t bi = 0; bi < nbi; bi++)
                if (pl->submitted[(size_t)(bi + nbi * (bj + nbj * bk))]) return EXAT_ERR_STATE;
    // One launch over the slab needs the kernels that read X through a table of block pointers: whole stages of i
    // (16 values for fp32 plans, 32 for bf16 and split-fp16 plans) and whole 128-fibre chunks inside every block,
    // 16-byte aligned blocks.  Any other slab is compressed block by block.
    const int ei = d.in_dtype == EXAT_F32 ? 16 : 32;
    bool one_launch = d.I % d.dI == 0 && d.dI % ei == 0 && d.dJ % 128 == 0 &&
                      (d.in_dtype == EXAT_F32_SPLIT || env_int("EXAT_PIPELINED", 1) != 0) && env_int("EXAT_SLAB", 1) != 0;
    for (int64_t q = 0; q < n && one_launch; q++)
        if ((uintptr_t)Xblk[q] & 15) one_launch = false;
    if (!one_launch) {
        int64_t q = 0;
        for (int64_t bk = bk0; bk < bk1; bk++)
            for (int64_t bj = bj0; bj < bj1; bj++)
                for (int64_t bi = 0; bi < nbi; bi++, q++) {
                    const int rc = exat_compress_block(pl, Xblk[q], (int32_t)bi, (int32_t)bj, (int32_t)bk, stream);
                    if (rc != EXAT_OK) return rc;
                }
        return EXAT_OK;
    }
    if (!pl->xtab) {
        if (pl->nblocks > (1LL << 24)) return EXAT_ERR_SHAPE;
        if (hipMalloc((void **)&pl->xtab, (size_t)pl->nblocks * sizeof(void *)) != hipSuccess) { (void)hipGetLastError(); pl->xtab = nullptr; return EXAT_ERR_ALLOC; }
    }
    // the slab's entries of the table (the kernel indexes it by global block coordinates)
    {
        PtrChunk c;
        int m = 0;
        int64_t q = 0;
        for (int64_t bk = bk0; bk < bk1; bk++)
            for (int64_t bj = bj0; bj < bj1; bj++)
                for (int64_t bi = 0; bi < nbi; bi++, q++) {
                    c.p[m] = Xblk[q]; c.idx[m] = bi + nbi * (bj + nbj * bk);
                    if (++m == 32 || q == n - 1) {
                        hipLaunchKernelGGL(k_set_ptrs, dim3(1), dim3(64), 0, st, pl->xtab, c, m);
                        m = 0;
                    }
                }
        if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    }
    Mode12Params mp;
    memset(&mp, 0, sizeof(mp));
    mp.xtab = pl->xtab; mp.x_dI = d.dI; mp.x_dJ = d.dJ; mp.x_dK = d.dK; mp.tab_nbi = (int)nbi; mp.tab_nbj = (int)nbj;
    mp.x_vec = 1;
    mp.i0 = 0; mp.i1 = d.I;
    mp.j0 = (int64_t)bj0 * d.dJ; mp.j1 = std::min<int64_t>(d.J, (int64_t)bj1 * d.dJ);
    mp.k0 = (int64_t)bk0 * d.dK; mp.k1 = std::min<int64_t>(d.K, (int64_t)bk1 * d.dK);
    // the slab's partial result goes to the slot of its first block
    const int64_t first = nbi * (bj0 + nbj * (int64_t)bk0);
    const int slot = (int)(first % pl->nslots);
    const int rc = run_chain(pl, mp, false, pl->slots + (int64_t)slot * pl->ysize, pl->slot_used[(size_t)slot] ? 1 : 0, st,
                             pl->slot_used[(size_t)slot] ? nullptr : pl->used_dev + slot);
    if (rc != EXAT_OK) return rc;
    pl->slot_used[(size_t)slot] = 1;
    for (int64_t bk = bk0; bk < bk1; bk++)
        for (int64_t bj = bj0; bj < bj1; bj++)
            for (int64_t bi = 0; bi < nbi; bi++) pl->submitted[(size_t)(bi + nbi * (bj + nbj * bk))] = 1;
    pl->nsubmitted += n;
    return EXAT_OK;
}

int exat_finalize(exat_plan_t pl, float *Y, void *stream)
{
    if (!pl || !Y) return EXAT_ERR_NULL;
    if (!pl->slots || pl->nsubmitted == 0) return EXAT_ERR_STATE;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_merge, dim3(grid_for(pl->ysize)), dim3(256), 0, st, pl->slots, pl->used_dev, pl->nslots, pl->ysize, Y);
    hipLaunchKernelGGL(k_clear_flags, dim3(grid_for(pl->nslots)), dim3(256), 0, st, pl->used_dev, pl->nslots);
    if (hipGetLastError() != hipSuccess) return EXAT_ERR_HIP;
    std::fill(pl->submitted.begin(), pl->submitted.end(), 0);
    std::fill(pl->slot_used.begin(), pl->slot_used.end(), 0);
    pl->nsubmitted = 0;
    return EXAT_OK;
}

int exat_compress_host(exat_plan_t pl, const void *Xhost, float *Y, void *stream)
{
    if (!pl || !Xhost || !Y) return EXAT_ERR_NULL;
    if (!pl->factors_set) return EXAT_ERR_STATE;
    if (pl->nsubmitted != 0) return EXAT_ERR_STATE;   // a block sequence of the caller's is open
    const exat_desc_t &d = pl->d;
    const size_t es = esize(d.in_dtype);
    const size_t blk_bytes = (size_t)d.dI * d.dJ * d.dK * es;
    hipStream_t st = (hipStream_t)stream;
    if (!pl->copy_stream) {
        // default priority: streams of different priorities are never mixed in this library
        if (hipStreamCreateWithFlags(&pl->copy_stream, hipStreamNonBlocking) != hipSuccess) { pl->copy_stream = nullptr; return EXAT_ERR_HIP; }
        for (int b = 0; b < exat_plan_s::kRing; b++) {
            if (hipMalloc(&pl->ring[b], blk_bytes) != hipSuccess) { pl->ring[b] = nullptr; (void)hipGetLastError(); return EXAT_ERR_ALLOC; }
            if (hipEventCreateWithFlags(&pl->ev_copied[b], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&pl->ev_free[b], hipEventDisableTiming) != hipSuccess) return EXAT_ERR_HIP;
        }
    }
    for (int b = 0; b < exat_plan_s::kRing; b++)
        if (!pl->ring[b] || !pl->ev_copied[b] || !pl->ev_free[b]) return EXAT_ERR_ALLOC;   // an earlier set-up failed half way
    const int nbi = (int)cdiv(d.I, d.dI), nbj = (int)cdiv(d.J, d.dJ), nbk = (int)cdiv(d.K, d.dK);
    int64_t n = 0;
    for (int bk = 0; bk < nbk; bk++)
        for (int bj = 0; bj < nbj; bj++)
            for (int bi = 0; bi < nbi; bi++, n++) {
                const int b = (int)(n % exat_plan_s::kRing);
                // the copy into buffer b may start once the block that used it last has been consumed
                if (pl->ring_used[b] && hipStreamWaitEvent(pl->copy_stream, pl->ev_free[b], 0) != hipSuccess) return EXAT_ERR_HIP;
                hipMemcpy3DParms cp;
                memset(&cp, 0, sizeof(cp));
                cp.srcPtr = make_hipPitchedPtr(const_cast<void *>(Xhost), (size_t)d.I * es, (size_t)d.I * es, (size_t)d.J);
                cp.srcPos = make_hipPos((size_t)bi * d.dI * es, (size_t)bj * d.dJ, (size_t)bk * d.dK);
                const size_t di = (size_t)blk_ext(d.I, d.dI, bi), dj = (size_t)blk_ext(d.J, d.dJ, bj), dk = (size_t)blk_ext(d.K, d.dK, bk);
                cp.dstPtr = make_hipPitchedPtr(pl->ring[b], di * es, di * es, dj);
                cp.dstPos = make_hipPos(0, 0, 0);
                cp.extent = make_hipExtent(di * es, dj, dk);
                cp.kind = hipMemcpyHostToDevice;
                if (hipMemcpy3DAsync(&cp, pl->copy_stream) != hipSuccess) return EXAT_ERR_HIP;
                if (hipEventRecord(pl->ev_copied[b], pl->copy_stream) != hipSuccess) return EXAT_ERR_HIP;
                if (hipStreamWaitEvent(st, pl->ev_copied[b], 0) != hipSuccess) return EXAT_ERR_HIP;
                const int rc = exat_compress_block(pl, pl->ring[b], bi, bj, bk, stream);
                if (rc != EXAT_OK) {
                    // leave no half-finished block sequence behind
                    hipLaunchKernelGGL(k_clear_flags, dim3(grid_for(pl->nslots)), dim3(256), 0, st, pl->used_dev, pl->nslots);
                    std::fill(pl->submitted.begin(), pl->submitted.end(), 0);
                    std::fill(pl->slot_used.begin(), pl->slot_used.end(), 0);
                    pl->nsubmitted = 0;
                    return rc;
                }
                if (hipEventRecord(pl->ev_free[b], st) != hipSuccess) return EXAT_ERR_HIP;
                pl->ring_used[b] = true;
            }
    return exat_finalize(pl, Y, stream);
}

int exat_gen_block(const exat_desc_t *desc, const exat_gen_t *gen, int32_t bi, int32_t bj, int32_t bk, void *out, void *stream)
{
    int rc = validate_desc(desc);
    if (rc != EXAT_OK) return rc;
    rc = validate_gen(gen);
    if (rc != EXAT_OK) return rc;
    if (!out) return EXAT_ERR_NULL;
    const exat_desc_t &d = *desc;
    if (bi < 0 || bj < 0 || bk < 0 || bi >= cdiv(d.I, d.dI) || bj >= cdiv(d.J, d.dJ) || bk >= cdiv(d.K, d.dK)) return EXAT_ERR_SHAPE;
    GenParams gp;
    gp.A = gen->A; gp.B = gen->B; gp.C = gen->C; gp.ldA = d.I; gp.ldB = d.J; gp.ldC = d.K; gp.R = gen->R;
    gp.skey = seed_key(gen->seed);
    gp.amp2_ln2 = amp2_ln2_of(gen->sigma);
    gp.i0 = (int64_t)bi * d.dI; gp.i1 = gp.i0 + blk_ext(d.I, d.dI, bi);
    gp.j0 = (int64_t)bj * d.dJ; gp.j1 = gp.j0 + blk_ext(d.J, d.dJ, bj);
    gp.k0 = (int64_t)bk * d.dK; gp.k1 = gp.k0 + blk_ext(d.K, d.dK, bk);
    const int64_t nq = ((gp.i1 - 1) >> 2) - (gp.i0 >> 2) + 1;
    const int64_t n = nq * (gp.j1 - gp.j0) * (gp.k1 - gp.k0);
    hipStream_t st = (hipStream_t)stream;
    if (d.in_dtype == EXAT_BF16)
        hipLaunchKernelGGL(k_gen_box<__bf16>, dim3(grid_for(n)), dim3(256), 0, st, gp, (__bf16 *)out);
    else
        hipLaunchKernelGGL(k_gen_box<float>, dim3(grid_for(n)), dim3(256), 0, st, gp, (float *)out);
    return hipGetLastError() == hipSuccess ? EXAT_OK : EXAT_ERR_HIP;
}

int exat_plan_set_timing(exat_plan_t pl, int enable)
{
    if (!pl) return EXAT_ERR_NULL;
    if (enable && !pl->evr[0][0]) {
        for (auto &tr : pl->evr)
            for (hipEvent_t &e : tr)
                if (hipEventCreate(&e) != hipSuccess) return EXAT_ERR_HIP;
    }
    pl->timing = enable != 0;
    pl->timed_calls = 0;
    return EXAT_OK;
}

int exat_plan_timing_of(exat_plan_t pl, int32_t age, float *ms_mode12, float *ms_mode3)
{
    if (!pl || !ms_mode12 || !ms_mode3) return EXAT_ERR_NULL;
    if (!pl->timing || age < 0 || age >= exat_plan_s::kTimeRing || age >= pl->timed_calls) return EXAT_ERR_STATE;
    hipEvent_t *ev = pl->evr[(pl->timed_calls - 1 - age) % exat_plan_s::kTimeRing];
    if (hipEventSynchronize(ev[2]) != hipSuccess) return EXAT_ERR_HIP;
    if (hipEventElapsedTime(ms_mode12, ev[0], ev[1]) != hipSuccess) return EXAT_ERR_HIP;
    if (hipEventElapsedTime(ms_mode3, ev[1], ev[2]) != hipSuccess) return EXAT_ERR_HIP;
    return EXAT_OK;
}

int exat_plan_last_timing(exat_plan_t pl, float *ms_mode12, float *ms_mode3)
{
    return exat_plan_timing_of(pl, 0, ms_mode12, ms_mode3);
}

const char *exat_strerror(int status)
{
    switch (status) {
    case EXAT_OK: return "success";
    case EXAT_ERR_NULL: return "a required pointer is NULL";
    case EXAT_ERR_SHAPE: return "invalid shape, block, box or leading dimension";
    case EXAT_ERR_DTYPE: return "unknown element type";
    case EXAT_ERR_STATE: return "call not valid in the plan's current state";
    case EXAT_ERR_ALLOC: return "allocation failed";
    case EXAT_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

}  // extern "C"
