/*
 * exat.h -- C ABI of the MI355X (gfx950) multi-replica tensor compression library.
 *
 * The operation is the compression stage of the Exascale-Tensor scheme
 * (paper Sec. 3 "Compression", Eq. 3; Alg. 2 lines 1-2): for p = 0..P-1
 *
 *     Y_p[l,m,n] = sum_{i,j,k} U_p[l,i] * V_p[m,j] * W_p[n,k] * X[i,j,k]
 *
 * i.e. Y_p = X x1 U_p x2 V_p x3 W_p, computed block by block (Sec. 4.3, Fig. 2)
 * with all P replicas' U_p stacked into one (P*L) x I operand (the stacked
 * matrix of Eq. 4), so that X is traversed once for all replicas.
 *
 * Conventions
 *   - Every pointer named "device" is a HIP device pointer on the current device;
 *     descriptors (exat_desc_t, exat_gen_t, exat_box_t) are host structs.
 *   - X is column-major (Sec. 4.1): element (i,j,k) at X[i + I*(j + J*k)].
 *   - U, V, W are stacked and row-major with the reduction index contiguous:
 *     U[(p*L + l)*ldU + i], V[(p*M + m)*ldV + j], W[(p*N + n)*ldW + k]; fp32.
 *   - Y is fp32, column-major per replica, replicas outermost:
 *     Y[l + L*(m + M*(n + N*p))].
 *   - `stream` is a borrowed hipStream_t (NULL = default stream).  All work is
 *     enqueued asynchronously on it; no call synchronises the device (the
 *     measurement aids that wait for their own events say so).
 *   - The caller owns every buffer it passes.  A plan owns only its workspace
 *     (packed operand copies, the mode-2 intermediate, block partials).
 *   - Every function returns EXAT_OK (0) or a negative exat_status_t; nothing is
 *     printed, thrown or aborted across this boundary.
 *   - Calls on one plan must not overlap in time (they share the plan's workspace).
 */
#ifndef EXAT_H
#define EXAT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct exat_plan_s *exat_plan_t; /* opaque */

typedef enum {
    EXAT_OK = 0,
    EXAT_ERR_NULL = -1,   /* a required pointer is NULL                                    */
    EXAT_ERR_SHAPE = -2,  /* non-positive or too large extent, block edge larger than the   */
                          /* tensor, box not inside the tensor, ld too small               */
    EXAT_ERR_DTYPE = -3,  /* unknown in_dtype                                              */
    EXAT_ERR_STATE = -4,  /* factors not set, block submitted twice, finalize with nothing */
    EXAT_ERR_ALLOC = -5,  /* device or host allocation failed                              */
    EXAT_ERR_HIP = -6     /* a HIP runtime call or kernel launch failed                    */
} exat_status_t;

/* Type in which the kernels consume the X tile and U, V, W.  Products are always
 * accumulated in fp32 and Y is always fp32.  With EXAT_BF16 the elements of X, U, V, W
 * are rounded to bf16 (round-to-nearest-even) before use; the intermediates of the
 * mode-1 and mode-2 contractions stay fp32. */
typedef enum { EXAT_F32 = 0, EXAT_BF16 = 1, EXAT_F32_SPLIT = 2 } exat_dtype_t;
/* EXAT_F32_SPLIT (the residual split of Eq. 5): X, U, V, W are fp32 in memory exactly as with EXAT_F32,
 * but exat_compress / exat_compress_block run the mode-1 and mode-2 contractions on the fp16 matrix
 * cores: every operand element is used as the sum of two fp16 pieces, x = fl16(x) + fl16(x - fl16(x)),
 * and every product as its three significant cross terms accumulated in fp32 (the dropped term is
 * 2^-22 of the product).  Results agree with EXAT_F32 to fp32 rounding level provided |X|, |U|, |V| and
 * the mode-1 intermediate stay below the fp16 maximum (65504); nothing checks that.  Sources the
 * split kernel does not cover (exat_compress_gen, unaligned blocks) run the EXAT_F32 kernels. */

/* Problem statement: the inputs of Alg. 2 plus the block edge of Sec. 4.3. */
typedef struct {
    int64_t I, J, K;     /* X is I x J x K; each extent in [1, 2^31 - 64]                  */
    int32_t L, M, N, P;  /* each Y_p is L x M x N; P replicas; M <= 64; P*L < 2^24          */
    int32_t dI, dJ, dK;  /* block edges, 1 <= dI <= I etc. (Sec. 4.3 assumes they divide    */
                         /* the extents; here the last block of an axis may be shorter)    */
    int32_t in_dtype;    /* exat_dtype_t                                                    */
} exat_desc_t;

/* Synthetic input of the dense experiments (Sec. 5.1, Eq. 1) plus additive noise:
 *   X[i,j,k] = sum_{r<R} A[i,r] B[j,r] C[k,r] + sigma * g(seed; i,j,k)
 * A, B, C: device, fp32, column-major I x R, J x R, K x R (A[i + I*r]).
 * g is the library's counter-based standard-normal function of the GLOBAL coordinates
 * (so X does not depend on how it is tiled): with 32-bit mixers
 *   mixA(x): x^=x>>16; x*=0x7feb352d; x^=x>>15; x*=0x846ca68b; x^=x>>16
 *   mixB(x): x^=x>>16; x*=0x21f0aaad; x^=x>>15; x*=0x735a2d97; x^=x>>15
 *   s  = mixA(mixA(lo32(seed) ^ 0x243f6a88) ^ hi32(seed));  ck = mixA(mixA(s ^ k) ^ j)
 *   w  = (i & 2) ? mixB(ck ^ (i>>2)) : mixA(ck ^ (i>>2))
 *   u1 = ((w>>16) + 0.5)/65536, u2 = ((w & 0xffff) + 0.5)/65536
 *   g  = sqrt(-2 ln u1) * ((i & 1) ? sin(2 pi u2) : cos(2 pi u2))
 * evaluated in fp32 with the hardware log2/sqrt/sin/cos.
 * The multiplier/shift sets of mixA and mixB are two published, public-domain 32-bit integer hash
 * finalisers of the multiply-xorshift family (the "lowbias32" constants found by Chris Wellons'
 * hash-prospector search and a second set from the same search); 0x243f6a88 is the first 32 fractional
 * bits of pi.  The composition into a stream key, a fibre key and a quad counter is this library's own. */
typedef struct {
    const float *A, *B, *C; /* device */
    int32_t R;              /* 1 <= R <= 256 */
    uint64_t seed;
    float sigma;
} exat_gen_t;

/* Half-open sub-box [i0,i1) x [j0,j1) x [k0,k1) of X; any non-empty box inside X. */
typedef struct { int64_t i0, i1, j0, j1, k0, k1; } exat_box_t;

/* Creates a plan for `desc` on the current device and allocates the workspace of the one-shot calls
 * (packed U/V/W copies and the mode-2 intermediate of P*L x M x K floats).  exat_compress and
 * exat_compress_gen allocate nothing afterwards.  Two calls allocate on their FIRST use with a plan and
 * must therefore not be the first such call inside a stream capture: exat_compress_block (the block
 * partials, at most 4 GiB) and exat_compress_host (three device block buffers, a copy stream, events).
 * Errors: NULL, SHAPE, DTYPE, ALLOC. */
int exat_plan_create(exat_plan_t *plan, const exat_desc_t *desc);

/* Frees the plan's workspace.  The caller must have synchronised the streams the plan
 * was used on.  NULL is accepted. */
int exat_plan_destroy(exat_plan_t plan);

/* Operand preparation: copies the stacked fp32 U (P*L x I), V (P*M x J), W (P*N x K)
 * (device, leading dimensions ldU >= I, ldV >= J, ldW >= K in elements) into the plan's
 * padded tile layout, rounding to bf16 when in_dtype is EXAT_BF16.  The shared first S
 * rows of Alg. 2 line 1 are a property of the caller's matrices; the library is agnostic.
 * Must be called before any compress call; may be called again to replace the matrices.
 * Errors: NULL, SHAPE, HIP. */
int exat_set_factors(exat_plan_t plan, const float *U, int64_t ldU, const float *V, int64_t ldV,
                     const float *W, int64_t ldW, void *stream);

/* Y_p = Comp(X, U_p, V_p, W_p) for all p over a fully materialised X (Eq. 3).
 * X: device, column-major I x J x K, fp32 (EXAT_F32) or bf16 (EXAT_BF16).
 * Y: device, P*L*M*N floats, overwritten.  Bit-identical from run to run.
 * Errors: NULL, STATE (factors not set), HIP. */
int exat_compress(exat_plan_t plan, const void *X, float *Y, void *stream);

/* Block-streamed compression (Sec. 4.3, Fig. 2a): compresses the block
 * T^{bi,bj,bk} = X(bi*dI:(bi+1)*dI, bj*dJ:.., bk*dK:..) (cut off at the tensor's edge when the block
 * edges do not divide the extents; there are ceil(I/dI) x ceil(J/dJ) x ceil(K/dK) blocks) given as its own
 * column-major device array of the block's actual extents (in_dtype) with the matching column slices of U, V, W and
 * adds the result to the plan's partial sums.  Xblk may be reused as soon as the work
 * enqueued on `stream` has completed.  Each block is accepted once (a second
 * submission returns STATE); exat_finalize merges the partials in a fixed order, so Y
 * does not depend on the submission order whenever the plan could give every block its
 * own partial (it can for up to 4 GiB of partials; beyond that, blocks that share a
 * partial are summed in submission order).  The first call with a plan allocates the partials.
 * Errors: NULL, SHAPE (block index out of range), STATE, ALLOC (first call only), HIP. */
int exat_compress_block(exat_plan_t plan, const void *Xblk, int32_t bi, int32_t bj, int32_t bk,
                        void *stream);

/* Block-streamed compression with several blocks resident at once (Sec. 4.3, Fig. 2: the blocks are independent,
 * so as many as the memory holds can be taken together): one call compresses the SLAB of blocks
 * { (bi, bj, bk) : 0 <= bi < ceil(I/dI), bj0 <= bj < bj1, bk0 <= bk < bk1 }, i.e. whole block columns along i.
 * Xblk: HOST array of ceil(I/dI)*(bj1-bj0)*(bk1-bk0) device pointers, bi fastest, then bj, then bk; each block
 * column-major in its actual extents as for exat_compress_block.  The array is read before the call returns; the
 * blocks must stay valid until the work on `stream` has completed.
 * A slab is compressed as one sub-tensor: mode 1 runs over the whole i extent before mode 2 is applied and mode 2
 * over the slab's j range before mode 3, so every mode is applied once per element (a lone block repeats modes 2
 * and 3) and one launch fills the chip.  The slab leaves one partial result, which exat_finalize merges with those
 * of the other slabs and single blocks of the pass in a fixed order: Y does not depend on the order of the calls,
 * only on how the blocks were grouped into slabs (rounding).  Requirements of the one-launch form: dI a
 * multiple of 16 (EXAT_BF16 and EXAT_F32_SPLIT: 32) that divides I, dJ a multiple of 128, 16-byte aligned
 * blocks; any other slab is compressed block by block, as by exat_compress_block.  Allocates on its first use with a plan (the block
 * partials and a table of one pointer per block).
 * Errors: NULL, STATE (factors not set, a block of the slab submitted twice), SHAPE, ALLOC, HIP. */
int exat_compress_blocks(exat_plan_t plan, const void *const *Xblk, int32_t bj0, int32_t bj1, int32_t bk0,
                         int32_t bk1, void *stream);

/* Merges the block partials into Y (overwritten) and resets the plan's block state so
 * that a new sequence of exat_compress_block calls can start.
 * Errors: NULL, STATE (no block submitted), HIP. */
int exat_finalize(exat_plan_t plan, float *Y, void *stream);

/* Block-streamed compression of a tensor that lives in HOST memory (Sec. 4.3 with the tensor outside the
 * accelerator's memory): every block T^{bi,bj,bk} is copied into one of three device buffers the plan owns
 * (allocated on first use, dI*dJ*dK elements each) on an internal copy stream and compressed on `stream` as by
 * exat_compress_block, copies running ahead of the compute by up to two blocks; exat_finalize ends the pass.
 * The blocks are taken in the fixed order bi fastest, bk slowest, so Y is bit-identical to the same sequence of
 * exat_compress_block calls.  Xhost: host, column-major I x J x K in in_dtype; page-locked memory
 * (hipHostMalloc) is needed for the copies to overlap the compute, pageable memory works but serialises.
 * Asynchronous: returns when everything is enqueued; Xhost must stay valid until the work on `stream` has
 * completed.  Must not be interleaved with a block sequence of the caller's on the same plan.
 * Errors: NULL, STATE (factors not set, block sequence open), ALLOC, HIP. */
int exat_compress_host(exat_plan_t plan, const void *Xhost, float *Y, void *stream);

/* Compression of the synthetic tensor of exat_gen_t without ever materialising it: the
 * kernels generate each X tile on chip.  box == NULL means the whole tensor; otherwise
 * only the elements of X inside the box contribute (the merge of Fig. 2a over a sub-box).
 * Y: device, P*L*M*N floats, overwritten.
 * Errors: NULL, SHAPE (bad R or box), STATE, HIP. */
int exat_compress_gen(exat_plan_t plan, const exat_gen_t *gen, const exat_box_t *box, float *Y,
                      void *stream);

/* Writes block (bi,bj,bk) of the synthetic tensor into `out` (device, column-major in the block's actual
 * extents, dI x dJ x dK except at a ragged edge, fp32 or bf16 according to desc->in_dtype): the same element function the
 * fused kernels evaluate on chip.
 * Errors: NULL, SHAPE, DTYPE, HIP. */
int exat_gen_block(const exat_desc_t *desc, const exat_gen_t *gen, int32_t bi, int32_t bj, int32_t bk,
                   void *out, void *stream);

/* Measurement aid (not part of the paper's method): with timing enabled, every compress
 * call records HIP events on its stream around the fused mode-1/2 kernel and around the
 * mode-3 kernel.  exat_plan_last_timing waits for the most recent call's events and returns
 * the two kernel durations in milliseconds (these are the calls in this API that block).  The plan keeps
 * the events of its last 128 calls: exat_plan_timing_of returns those of the call `age` calls back
 * (0 = the most recent), so that a caller can enqueue many calls back to back and read their kernel
 * times afterwards.  Errors: NULL, STATE (timing off, no such call since it was enabled, age >= 128), HIP. */
int exat_plan_set_timing(exat_plan_t plan, int enable);
int exat_plan_last_timing(exat_plan_t plan, float *ms_mode12, float *ms_mode3);
int exat_plan_timing_of(exat_plan_t plan, int32_t age, float *ms_mode12, float *ms_mode3);

/* Measurement aid (not part of the paper's method): what the matrix cores of this GPU sustain when a kernel issues
 * nothing but MFMAs -- the ceiling a compression kernel could reach at best on the box it runs on, next to the
 * published peak its roofline fraction is quoted against.  Launches `workgroups` workgroups of eight waves (two per
 * SIMD) that each issue iters * 64 independent MFMAs, kind 0: 32x32x16 bf16, kind 1: 32x32x2 fp32, on operands that
 * are all 0.5 (random_operands == 0) or pseudo-random in [-1, 1) and different for consecutive MFMAs; runs the launch
 * twice on the default stream and times the second.  tflops: the measured rate; core_ghz: the core clock during the
 * launch (core-clock ticks over 100 MHz wall-clock ticks of one workgroup).  Blocks until done; allocates and frees
 * two small buffers.  Errors: NULL, SHAPE, ALLOC, HIP. */
int exat_probe_mfma(int32_t kind, int32_t random_operands, int32_t iters, int32_t workgroups, double *tflops,
                    double *core_ghz);

/* ---- Two-stage compression (Sec. 4.4) --------------------------------------------------------------
 * The paper builds the compression matrices as U_p = U'_p U, V_p = V'_p V, W_p = W'_p W with sparse
 * U (A1 x I), V (B1 x J), W (C1 x K) shared by all replicas (A1 = alpha L etc., alpha > 1), which turns
 * the compression into I x J x K -> A1 x B1 x C1 -> L x M x N.  The first stage,
 *
 *     X1[a,b,c] = sum_{i,j,k} U[a,i] V[b,j] W[c,k] X[i,j,k],
 *
 * is what exat_stage1_apply computes: one pass over X that is bound by reading it.  When every entry of U and
 * of V (repeated entries added) is a bf16 number, as the entries of sign matrices are, and I is a multiple of 4,
 * the first two modes run on the matrix cores with X split exactly into three bf16 pieces (same result up to
 * the order of the fp32 additions); otherwise, or with EXAT_STAGE1_MFMA=0 in the environment at creation, a
 * sparse form runs that uses the vector units only.
 * The second stage is the dense multi-replica compression of X1: an ordinary plan with I,J,K = A1,B1,C1
 * and U', V', W' as its factors, fed with X1 through exat_compress.
 *
 * A sparse matrix is handed over in CSR form in HOST memory and copied at creation: rowptr[rows+1]
 * (rowptr[0] = 0, non-decreasing), colidx/val[rowptr[rows]] (0 <= colidx < cols; any order inside a row;
 * repeated entries add).  The paper fixes neither pattern nor density; any CSR matrix is accepted. */
typedef struct {
    int32_t rows;           /* U, V: 1..128; W: 1..65535                         */
    int64_t cols;           /* must equal I, J, K respectively                   */
    const int64_t *rowptr;  /* host */
    const int32_t *colidx;  /* host */
    const float *val;       /* host */
} exat_csr_t;

typedef struct exat_stage1_s *exat_stage1_t; /* opaque */

/* Creates the first-stage operator for an I x J x K tensor on the current device: validates and copies
 * the three matrices (re-tiled for the kernels) and allocates the K x B1 x A1 float intermediate.
 * Synchronous (blocking host-to-device copies).  Errors: NULL, SHAPE (extents, rows out of range, cols
 * mismatch, malformed CSR, more than 2^31-256 entries), ALLOC, HIP. */
int exat_stage1_create(exat_stage1_t *s, int64_t I, int64_t J, int64_t K, const exat_csr_t *U,
                       const exat_csr_t *V, const exat_csr_t *W);

/* Frees the operator; the caller must have synchronised the streams it was used on.  NULL is accepted. */
int exat_stage1_destroy(exat_stage1_t s);

/* Output extents A1, B1, C1 (the row counts of U, V, W).  Errors: NULL. */
int exat_stage1_dims(exat_stage1_t s, int32_t *A1, int32_t *B1, int32_t *C1);

/* X1 = X x1 U x2 V x3 W.  X: device, fp32, column-major I x J x K.  X1: device, A1*B1*C1 floats,
 * column-major (X1[a + A1*(b + B1*c)]), overwritten.  fp32 arithmetic with a fixed summation order
 * (bit-identical from run to run).  Asynchronous on `stream`; calls on one operator must not overlap
 * (they share its intermediate).  Errors: NULL, HIP. */
int exat_stage1_apply(exat_stage1_t s, const float *X, float *X1, void *stream);

/* The same for a tensor in HOST memory: slabs of frontal slices (contiguous in a column-major tensor, about
 * 128 MiB each) are copied into three device buffers the operator owns (allocated on first use) on an internal
 * copy stream, up to two slabs ahead of the kernels on `stream`.  Same result as exat_stage1_apply, bit for
 * bit.  Page-locked memory is needed for the copies to overlap the kernels.  Asynchronous; Xhost must stay
 * valid until the work on `stream` has completed.  Errors: NULL, ALLOC, HIP. */
int exat_stage1_apply_host(exat_stage1_t s, const float *Xhost, float *X1, void *stream);

/* Measurement aid, as exat_plan_set_timing / exat_plan_last_timing: durations of the fused mode-1/2
 * kernel and of the mode-3 kernel of the most recent exat_stage1_apply. */
int exat_stage1_set_timing(exat_stage1_t s, int enable);
int exat_stage1_last_timing(exat_stage1_t s, float *ms_mode12, float *ms_mode3);

/* ---- CP-ALS on the proxy tensors (Alg. 1) ----------------------------------------------------------
 * The decomposition stage applies the alternating-least-squares algorithm to each of the P small tensors
 * Y_p (L x M x N) that the compression produced.  exat_cpals runs `sweeps` sweeps of the loop body of Alg. 1
 * (update A, then B, then C; each the least-squares solution with the other two fixed,
 * A <- Y_(1) (C kr B) [(C^T C) * (B^T B)]^{-1}, solved by Cholesky factorisation of the R x R normal matrix)
 * for all P replicas at once, one workgroup per replica, in fp32.  There is no convergence test: the caller
 * chooses the number of sweeps.
 *   Y      device, P*L*M*N floats in the layout exat_compress writes: Y[l + L*(m + M*(n + N*p))]; not modified
 *   A,B,C  device, in: start values, out: result; per replica column-major L x R, M x R, N x R:
 *          A[l + L*(r + R*p)] etc.
 *   work   device scratch of exat_cpals_workspace_floats(L,M,N,P) floats (two permuted copies of Y), caller-owned
 * Limits: L, M, N, R <= 64.  The normal matrices must be positive definite (they are for generic data): Alg. 1
 * writes a pseudo-inverse, which this solve does not provide, so a replica whose normal matrix loses rank ends in
 * NaN or meaningless factors.  exat_cpals_checked reports that: `status` (device, P int32, written by the call)
 * counts, per replica, the factor updates whose R x R normal matrix showed a zero, negative or NaN pivot in the
 * Cholesky factorisation (0 = every update was positive definite); the caller restarts such a replica from other
 * start values (or drops it), as the restart loop of Alg. 2 does with replicas that fail.  The arithmetic is that of
 * exat_cpals, bit for bit.  Asynchronous on `stream`.  Errors: NULL, SHAPE, HIP. */
int64_t exat_cpals_workspace_floats(int32_t L, int32_t M, int32_t N, int32_t P);
int exat_cpals(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps,
               float *A, float *B, float *C, float *work, void *stream);
int exat_cpals_checked(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps,
                       float *A, float *B, float *C, float *work, int32_t *status, void *stream);

/* exat_cpals for callers that cannot allocate device memory and have no workspace to hand over (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same sweeps, with the workspace taken
 * from a static device array of 4194304 floats (16 MiB) that every GPU the library runs on
 * holds until the process ends.  The call allocates nothing; its first use on a device looks the array's address up.
 * Problems whose exat_cpals_workspace_floats(L,M,N,P) exceeds that size are rejected with SHAPE (cfg1's and cfg2's
 * proxy tensors fit, cfg3's do not).  All calls on one GPU share the one array: calls that overlap in time on the
 * same GPU (different streams, different host threads) race and must be serialised by the caller.
 * Same arguments, results (bit for bit) and limits as exat_cpals.  Errors: NULL, SHAPE, HIP. */
int exat_cpals_noalloc(const float *Y, int32_t L, int32_t M, int32_t N, int32_t P, int32_t R, int32_t sweeps,
                       float *A, float *B, float *C, void *stream);

/* ---- joining the replicas: the stacked least-squares problem (Eq. 4) -------------------------------------
 * After the P decompositions and the alignment of their columns, the factor of the full tensor (up to one common
 * permutation and scaling, A Pi Sigma in the paper's notation) is the least-squares solution X (I x R) of
 *   [A_1; ...; A_P] = [U_1; ...; U_P] X
 * with the stacked P*L x I compression matrix of that mode.  exat_ls runs `iters` iterations of the conjugate
 * gradient method on the normal equations (CGLS) from X = 0, in fp32, all columns at once, reading the stacked
 * matrix in place.  A column is left as it is once its normal-equation residual ||U^T (A - U X)|| has fallen to
 * `tol` times its start value ||U^T A|| (in fp32 the iteration drifts away again if it runs on past convergence;
 * 1e-6 is a good value, below about 3e-7 the test never triggers; 0 switches it off).  The host never waits: all
 * `iters` iterations are launched, the caller may read back `relres`.
 *   U       device, the stacked matrix as exat_set_factors takes it: row p*L + l is row l of U_p; row-major,
 *           leading dimension ldU >= I in elements; not modified
 *   Astack  device, P*L x R in the layout exat_cpals writes: A[l + L*(r + R*p)]; not modified
 *   X       device, out: I x R column-major, X[i + I*r]
 *   relres  device, out, R floats, or NULL: per column ||U^T (A - U X)|| / ||U^T A|| after the last iteration
 *   work    device scratch of exat_ls_workspace_floats(P, L, I, R) floats, caller-owned
 * The system must have full column rank (P*L >= I); the iteration count for a given accuracy grows with the
 * condition number of the stacked matrix (about 30 iterations to tol = 1e-6 at P*L = 2 I with Gaussian
 * matrices; a square system, P*L = I, is out of reach of fp32).  Limits: R <= 64, P*L and I <= 2^22, P*L*ldU <= 2^30.
 * Asynchronous on `stream`.  Errors: NULL, SHAPE, HIP. */
int64_t exat_ls_workspace_floats(int32_t P, int32_t L, int32_t I, int32_t R);
int exat_ls(const float *U, int64_t ldU, int32_t P, int32_t L, int32_t I, const float *Astack, int32_t R,
            int32_t iters, float tol, float *X, float *relres, float *work, void *stream);

/* Static description of a status code (never NULL). */
const char *exat_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* EXAT_H */
