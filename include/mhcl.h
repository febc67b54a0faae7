/*
 * mhcl.h -- C ABI of libmhcl: the per-token hyper-connection path of mHC-lite
 * (and of the Sinkhorn-Knopp mHC variant it is compared with) for AMD gfx950.
 *
 * One layer of the network updates n residual streams x in R^{n x C} as
 *
 *     x_out = H_res x + H_post^T f(H_pre x)                      (Eq. 1)
 *
 * where the coefficients are computed per token from the flattened streams
 * x_hat in R^{1 x nC} (Sec. 3.2, the lines above Eq. 4, Eq. 4 and Eq. 5):
 *
 *     x_hat' = RMSNorm(x_hat)
 *     H_pre  = sigmoid(alpha_pre  x_hat' W_pre  + b_pre)          in R^{1 x n}
 *     H_post = 2 sigmoid(alpha_post x_hat' W_post + b_post)       in R^{1 x n}
 *     a      = softmax(alpha_res x_hat' W_res + b_res)            in R^{n!}
 *     H_res  = sum_k a_k P_k                                      in R^{n x n}
 *
 * (P_k: the n! permutation matrices, Theorem 3.1), or, in the Sinkhorn-Knopp
 * variant (Sec. 2, Eq. 2), H_res = SK(exp(mat(alpha_res x_hat' W_res + b_res)))
 * with W_res in R^{nC x n^2} and SK repeated sk_iters times.  A third form
 * keeps only K chosen permutations (Sec. 5, the paragraph on larger n):
 * a = softmax over K logits, H_res = sum over the K given P_k; still doubly
 * stochastic, n up to 8.
 *
 * f (attention / MLP) is the caller's: the library hands back h = H_pre x, the
 * caller computes y = f(h) and hands y in.  Backward likewise: the caller
 * provides the gradient on x_out and on h and receives the gradient on x, y
 * and the parameters.
 *
 * Conventions (they hold for every entry point unless it says otherwise)
 *  - Every tensor pointer is a DEVICE pointer owned by the caller, dense,
 *    row-major, 16-byte aligned.  The library never allocates, frees or
 *    synchronises; every call only enqueues kernels on `stream` (a
 *    hipStream_t passed as void*; NULL is the default stream).  Scratch memory
 *    comes from the caller as `ws` / `ws_bytes`, sized by
 *    mhcl_workspace_bytes(); its contents are undefined before and after a
 *    call.  Calls on different streams with disjoint outputs and workspaces
 *    may overlap.  The library keeps two pieces of state, each named where it
 *    is used: the per-host-thread arming of mhcl_profile_next_call, and the
 *    per-GPU static scratch array of mhcl_fwd_coeffs_pre_static.
 *  - Placement (performance only, never correctness): mhcl_bwd_fused runs
 *    about 5 % faster in its second pass when x, g_xout and g_x start at
 *    three different offsets modulo 1 KiB, in steps of 256 bytes (say 0, 256
 *    and 512 past a 1 KiB boundary), than when they are equally aligned.
 *  - Stream tensors (x, y, h, x_out and their gradients) have the element
 *    type desc->io_dtype.  Coefficients, parameters and parameter gradients
 *    are always fp32.  All arithmetic accumulates in fp32; bf16 results are
 *    rounded to nearest-even once, from the fp32 value.
 *  - x is [T, n, C] and is flattened stream-major: x_hat[j*C + c] = x[j][c].
 *  - W is one [n*C, M] matrix, b is [M]; columns are [res | pre | post] with
 *    M = n! + 2n (MHCL_RES_LITE; res column k belongs to permutation k) or
 *    M = n*n + 2n (MHCL_RES_SK; res column i*n + j is entry (i, j)), or
 *    M = K + 2n (MHCL_RES_SUBSET; res column k belongs to row k of desc->perm).
 *    alpha is [3] = {alpha_res, alpha_pre, alpha_post}, in device memory.
 *  - Permutations are ordered lexicographically as tuples
 *    (sigma(0), ..., sigma(n-1)); k = 0 is the identity; P_k[i][sigma_k(i)] = 1.
 *  - RMSNorm has no gain: x_hat' = x_hat / sqrt(mean(x_hat^2) + eps).
 *  - One SK iteration rescales all columns to sum 1, then all rows.
 *  - H_res is [T, n, n], H_pre and H_post are [T, n].
 *  - Every function returns an mhcl_status.  Arguments are validated before
 *    anything is enqueued, so a non-OK status means nothing ran.  T == 0 is
 *    valid: per-token tensors may then be null, nothing is read, and the
 *    sums over tokens (g_W, g_b, g_alpha) are written as zeros.  Errors of the HIP runtime at launch are
 *    reported as MHCL_ERR_HIP.  Nothing aborts or throws.
 */
#ifndef MHCL_H
#define MHCL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MHCL_OK = 0,
  MHCL_ERR_INVALID_ARG = 1, /* null pointer, misaligned pointer, bad enum, n/C/T out of range */
  MHCL_ERR_UNSUPPORTED = 2, /* a valid description the library has no kernel for */
  MHCL_ERR_WORKSPACE = 3,   /* ws is null or smaller than mhcl_workspace_bytes() */
  MHCL_ERR_HIP = 4          /* a kernel launch was rejected by the runtime */
} mhcl_status;

enum { MHCL_BF16 = 0, MHCL_F32 = 1 };          /* io_dtype */
enum { MHCL_RES_LITE = 0, MHCL_RES_SK = 1, MHCL_RES_SUBSET = 2 };   /* res_mode */

/* operations that need workspace, for mhcl_workspace_bytes() */
enum {
  MHCL_OP_COEFFS = 0,
  MHCL_OP_COEFFS_BWD = 1,
  MHCL_OP_FWD_COEFFS_PRE = 2,
  MHCL_OP_BWD_FUSED = 3
};

typedef struct {
  int32_t n;        /* residual streams, 1..5 (1..8 for MHCL_RES_SUBSET)           */
  int32_t C;        /* width of one stream; a positive multiple of 8               */
  int64_t T;        /* tokens, >= 0                                                */
  int32_t io_dtype; /* MHCL_BF16 | MHCL_F32                                        */
  int32_t res_mode; /* MHCL_RES_LITE | MHCL_RES_SK | MHCL_RES_SUBSET               */
  int32_t sk_iters; /* SK repetitions (1..32) for MHCL_RES_SK; else ignored         */
  float eps;        /* RMSNorm epsilon, >= 0, added to the mean square             */
  int32_t n_perm;   /* MHCL_RES_SUBSET: K, number of permutations, 1..128; else ignored */
  const int8_t *perm; /* MHCL_RES_SUBSET: DEVICE pointer, [K][n], perm[k][i] = column
                       * of the 1 in row i of P_k.  Every row must be a permutation of
                       * 0..n-1 (the caller's responsibility: device memory is not
                       * inspected on the host); it must stay valid while kernels of a
                       * call using this descriptor run.  Else ignored.           */
} mhcl_desc;

const char *mhcl_status_string(int status);

/* Checks a descriptor (host only; touches no GPU). */
int mhcl_validate(const mhcl_desc *desc);

/* M: number of logits / columns of W for this descriptor; -1 if invalid. */
int32_t mhcl_logit_count(const mhcl_desc *desc);

/* Bytes of workspace `op` needs for `desc`; 0 if desc or op is invalid.
 * Host only. */
size_t mhcl_workspace_bytes(const mhcl_desc *desc, int op);

/* Host helper: writes the permutation table the library uses (Theorem 3.1;
 * lexicographic order) into HOST memory sigma[n!][n], sigma[k][i] = column of
 * the 1 in row i of P_k.  n in 1..5. */
int mhcl_perm_table(int32_t n, int8_t *sigma);

/* ---- forward ----------------------------------------------------------- */

/* Coefficients of one layer (Sec. 3.2 Eqs. 4-5, or Sec. 2 Eq. 2 in SK mode).
 * in : x [T,n,C] io, W [nC,M] f32, b [M] f32, alpha [3] f32
 * out: H_res [T,n,n], H_pre [T,n], H_post [T,n] f32 */
int mhcl_coeffs(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                const float *alpha, float *H_res, float *H_pre, float *H_post,
                void *ws, size_t ws_bytes, void *stream);

/* Pre-aggregate, the argument of f in Eq. 1: h[c] = sum_j H_pre[j] x[j][c].
 * in : x [T,n,C] io, H_pre [T,n] f32;  out: h [T,C] io */
int mhcl_pre(const mhcl_desc *desc, const void *x, const float *H_pre, void *h, void *stream);

/* Residual update, Eq. 1 with y = f(h) supplied:
 * x_out[i][c] = sum_j H_res[i][j] x[j][c] + H_post[i] y[c].
 * in : x [T,n,C], y [T,C] io; H_res, H_post f32;  out: x_out [T,n,C] io.
 * x_out must not alias x. */
int mhcl_post(const mhcl_desc *desc, const void *x, const void *y, const float *H_res,
              const float *H_post, void *x_out, void *stream);

/* mhcl_coeffs and mhcl_pre in one call (one validation, one workspace).
 * bf16 streams with at most 32 logits, C a multiple of 256 from 1024 to 8192
 * and at least 512 * floor(65536 / C) tokens: ONE kernel reads x from HBM once and produces the
 * projection, H_pre and h from the same register tile (groups of 16 tokens
 * shared by C / 256 thread blocks that exchange their partial sums; needs the
 * 256 compute units of the device free for its 256 blocks, see the source).
 * Its workspace holds one slice of the projection per 256 columns,
 * (C / 256) * T * (M + 1) * 4 bytes (6 % of x at n = 4, C = 4096).
 * The projection's sum over n C terms is then split differently from
 * mhcl_coeffs, so H_* agree with it to fp32 rounding of the logits and h to
 * one bf16 step.  Every other shape, or a device that cannot hold the 256
 * blocks at once: mhcl_coeffs followed by mhcl_pre, bit for bit (x is then
 * read twice: h needs H_pre, which needs the token's whole row).
 * Results are reproducible bit for bit from call to call either way.
 * MHCL_FWD_ONCE=0 in the environment keeps the two-kernel form everywhere (for
 * a process that shares the device with other long-running work: the one
 * kernel wants a compute unit per block, waits for blocks that have none yet
 * for about a second at most, and returns NaN in the outputs if that was not
 * enough); it is read at every call and by mhcl_workspace_bytes. */
int mhcl_fwd_coeffs_pre(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                        const float *alpha, float *H_res, float *H_pre, float *H_post, void *h,
                        void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): mhcl_fwd_coeffs_pre without
 * a workspace argument.  Its scratch is a static device array of
 * MHCL_STATIC_SCRATCH_BYTES that every GPU the library runs on holds from the
 * first use of the library on it until the process ends; the call allocates
 * and frees nothing (no hipMalloc, no library allocator).  It always runs the
 * kernels of mhcl_coeffs followed by mhcl_pre, with their results bit for bit
 * (the single-read kernel needs more scratch than the array at the shapes where
 * it pays).  Returns MHCL_ERR_WORKSPACE, and enqueues nothing, when
 * mhcl_workspace_bytes(desc, MHCL_OP_COEFFS) exceeds the array (at
 * n = 4, bf16 streams that is about T * 132 bytes + 2 MiB: the array covers
 * n = 4, C = 4096 up to 100 000 tokens).  The first call on a GPU looks up the
 * array's device address (hipGetSymbolAddress; make that call outside graph
 * capture).  All calls on one GPU share the array: two such calls that overlap
 * in time on one GPU (different streams or host threads) race; calls on one
 * stream are ordered and safe.  The array's contents between calls are
 * undefined; nothing in it has to be cleared. */
#define MHCL_STATIC_SCRATCH_BYTES (16u << 20)
int mhcl_fwd_coeffs_pre_static(const mhcl_desc *desc, const void *x, const float *W,
                               const float *b, const float *alpha, float *H_res, float *H_pre,
                               float *H_post, void *h, void *stream);

/* ---- backward (chain rule on the definitions above) -------------------- */

/* Backward of mhcl_post, with x, y, H_res, H_post independent inputs.
 * in : x, y, H_res, H_post as in mhcl_post; g_xout [T,n,C] io
 * out: g_x [T,n,C] io, OVERWRITTEN with H_res^T g_xout;  g_y [T,C] io;
 *      g_H_res [T,n,n], g_H_post [T,n] f32 */
int mhcl_post_bwd(const mhcl_desc *desc, const void *x, const void *y, const float *H_res,
                  const float *H_post, const void *g_xout, void *g_x, void *g_y,
                  float *g_H_res, float *g_H_post, void *stream);

/* Backward of mhcl_pre.  g_x is ACCUMULATED into (g_x[j] += H_pre[j] g_h) in
 * the io type; g_H_pre [T,n] is overwritten. */
int mhcl_pre_bwd(const mhcl_desc *desc, const void *x, const float *H_pre, const void *g_h,
                 void *g_x, float *g_H_pre, void *stream);

/* Backward of mhcl_coeffs.  Recomputes the forward from x (nothing is saved
 * between forward and backward).  g_x is ACCUMULATED into in the io type;
 * g_W [nC,M], g_b [M], g_alpha [3] (f32) are overwritten with the sums over
 * all T tokens, added in a fixed order (results are bitwise reproducible). */
int mhcl_coeffs_bwd(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                    const float *alpha, const float *g_H_res, const float *g_H_pre,
                    const float *g_H_post, void *g_x, float *g_W, float *g_b, float *g_alpha,
                    void *ws, size_t ws_bytes, void *stream);

/* Whole backward of one layer for the loss <g_xout, x_out> + <g_h, h> with y
 * an independent input: equals mhcl_post_bwd, mhcl_pre_bwd, mhcl_coeffs_bwd
 * chained, but g_x is summed in fp32 and rounded once, and x is read in fewer
 * passes.  Coefficients are recomputed from x.
 * in : x, y, W, b, alpha as in forward; g_xout [T,n,C], g_h [T,C] io
 * out: g_x [T,n,C], g_y [T,C] io; g_W [nC,M], g_b [M], g_alpha [3] f32; all
 *      overwritten.  g_y may be NULL (a caller that needed it before g_h
 *      existed has it already): it is then neither computed nor written.
 * For n >= 5 with bf16 streams and C a multiple of 64 (any form; with a
 * permutation subset only while n * ceil(M / 32) * 4 KiB of W plus the
 * per-token records fit the 160 KiB of LDS) the product W vr inside g_x uses
 * W rounded to 11 significant bits (fp16 of W times a power of two chosen per
 * call from max |W|, so any magnitude is fine); the change is far below the
 * bf16 rounding of g_x. */
int mhcl_bwd_fused(const mhcl_desc *desc, const void *x, const void *y, const float *W,
                   const float *b, const float *alpha, const void *g_xout, const void *g_h,
                   void *g_x, void *g_y, float *g_W, float *g_b, float *g_alpha,
                   void *ws, size_t ws_bytes, void *stream);

/* ---- diagnostics of doubly stochasticity (Sec. 3.1, Sec. 4.3) ------------ */

/* The logits of one layer, z = alpha_g (RMSNorm(x_hat) W) + b (Sec. 3.2, the
 * three lines above Eq. 4; Sec. 2 Eq. 2 in SK mode), and per token the
 * relative range of Eq. 3 for the matrix exp(mat(z_res)) that Sinkhorn-Knopp
 * starts from, as log(1/nu) = max z_res - min z_res (natural log; every entry
 * of exp(.) is positive, so the minimum over positive entries is the minimum).
 * in : x [T,n,C] io, W [nC,M] f32, b [M] f32, alpha [3] f32
 * out: z [T,M] f32, columns [res | pre | post]; log_inv_nu [T] f32.  Either
 *      output may be null, not both.
 * Workspace as for MHCL_OP_COEFFS. */
int mhcl_logits(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                const float *alpha, float *z, float *log_inv_nu, void *ws, size_t ws_bytes,
                void *stream);

/* Column sums and l1 errors of L layers' per-token residual matrices and of
 * their running product over the layers (Sec. 3.1 footnote 1 and last
 * paragraph; Sec. 4.3, "per-matrix" and "prod").  n in 1..8, L >= 1, T >= 0.
 * in : H [L,T,n,n] f32 (e.g. L calls of mhcl_coeffs into one buffer)
 * out, each nullable (not all):
 *   colsum      [L,T,n]  colsum[l][t][j] = sum_i H[l][t][i][j]
 *   l1          [L,T]    ||H 1 - 1||_1 + ||H^T 1 - 1||_1
 *   prod        [T,n,n]  Q_L, with Q_l = H_l Q_{l-1}, Q_0 = I: later layers
 *                        multiply on the left, the order Eq. 1 applies them
 *                        (the paper's product sign fixes no order)
 *   prod_colsum [L,T,n]  column sums of Q_l
 *   prod_l1     [L,T]    l1 error of Q_l
 * fp32 throughout; needs no workspace. */
int mhcl_ds_chain(int32_t n, int32_t L, int64_t T, const float *H, float *colsum, float *l1,
                  float *prod, float *prod_colsum, float *prod_l1, void *stream);

/* ---- measurement aids (no part of the method) --------------------------- */

/* Kernel stages that can be bracketed with events. */
enum {
  MHCL_STAGE_NONE = 0,
  MHCL_STAGE_FWD_PROJ = 1,   /* projection + coefficients kernel of the forward          */
  MHCL_STAGE_FWD_PRE = 2,    /* h = H_pre x                                              */
  MHCL_STAGE_POST = 3,       /* x_out = H_res x + H_post y                               */
  MHCL_STAGE_BWD_REDUCE = 4, /* backward pass 1: all per-token reductions + coefficients */
  MHCL_STAGE_BWD_OUT = 5,    /* backward pass 2: g_x and g_y                             */
  MHCL_STAGE_BWD_GW = 6      /* backward: g_W, the reduction over tokens                 */
};

/* Arms the NEXT library call made by this host thread: it records the
 * hipEvent_t `ev_start` on its stream right before the first kernel of `stage`
 * and `ev_stop` right after the last one, then disarms.  Both events are the
 * caller's (created with timing enabled).  State is per host thread. */
int mhcl_profile_next_call(int stage, void *ev_start, void *ev_stop);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both
 * pointers 16-byte aligned): the yardstick for achievable HBM bandwidth and
 * for calibrating hardware byte counters. */
int mhcl_debug_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MHCL_H */
