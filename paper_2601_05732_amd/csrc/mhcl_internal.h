// Host-side declarations shared by the translation units of libmhcl.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mhcl.h"

namespace mhcl {

inline int host_factorial(int n) { return n <= 1 ? 1 : n * host_factorial(n - 1); }
inline int res_logits(const mhcl_desc &d) {
  if (d.res_mode == MHCL_RES_LITE) return host_factorial(d.n);
  if (d.res_mode == MHCL_RES_SUBSET) return d.n_perm;
  return d.n * d.n;
}
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Carves a caller-provided workspace into 256-byte aligned pieces.
struct WsCursor {
  char *base;
  size_t off = 0;
  explicit WsCursor(void *p) : base(static_cast<char *>(p)) {}
  template <typename T>
  T *take(size_t count) {
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += align_up(count * sizeof(T));
    return p;
  }
};

// Per-token results of the backward's coefficient stage, all [T, ...] fp32.
struct BwdTokenBufs {
  float *H_res;   // [T, n*n]
  float *H_pre;   // [T, n]
  float *H_post;  // [T, n]
  float *vr;      // [T, M]   r * alpha_g * g_z   (the vector multiplied with W and x)
  float *coefx;   // [T]      (r^2 / nC) <vr, u_raw>
  float *gz;      // [T, M+3] g_z, then the three per-group sums of g_z * u
};

// ---- generic (plain ALU) kernels: any n in 1..5, bf16 or f32 streams -----
hipError_t launch_proj_generic(const mhcl_desc &d, int M, const void *x, const float *W,
                               float *u_raw, float *sumsq, hipStream_t s);
hipError_t launch_coeffs_epilogue(const mhcl_desc &d, int parts, const float *u_raw,
                                  const float *sumsq, const float *b, const float *alpha, float *H_res, float *H_pre,
                                  float *H_post, hipStream_t s);
hipError_t launch_pre(const mhcl_desc &d, const void *x, const float *H_pre, void *h, hipStream_t s);
hipError_t launch_post(const mhcl_desc &d, const void *x, const void *y, const float *H_res,
                       const float *H_post, void *x_out, hipStream_t s);
hipError_t launch_post_bwd(const mhcl_desc &d, const void *x, const void *y, const float *H_res,
                           const float *H_post, const void *g_xout, void *g_x, void *g_y,
                           float *g_H_res, float *g_H_post, hipStream_t s);
hipError_t launch_pre_bwd(const mhcl_desc &d, const void *x, const float *H_pre, const void *g_h,
                          void *g_x, float *g_H_pre, hipStream_t s);
// dots only: g_H_res = <g_xout[i], x[j]>, g_H_post = <g_xout[i], y>, g_H_pre = <g_h, x[j]>
hipError_t launch_bwd_dots(const mhcl_desc &d, const void *x, const void *y, const void *g_xout,
                           const void *g_h, float *g_H_res, float *g_H_post, float *g_H_pre,
                           hipStream_t s);
hipError_t launch_coeffs_bwd_epilogue(const mhcl_desc &d, int parts, const float *u_raw,
                                      const float *sumsq,
                                      const float *b, const float *alpha, const float *g_H_res,
                                      const float *g_H_pre, const float *g_H_post,
                                      const BwdTokenBufs &o, hipStream_t s);
// fused == true : g_x = H_res^T g_xout + H_pre g_h + W vr - x coefx ; g_y = H_post g_xout
// fused == false: g_x += W vr - x coefx
hipError_t launch_gx_generic(const mhcl_desc &d, int M, bool fused, const void *x, const float *W,
                             const void *g_xout, const void *g_h, const BwdTokenBufs &o, void *g_x,
                             void *g_y, hipStream_t s);
int gw_chunks_generic(const mhcl_desc &d);
hipError_t launch_gw_generic(const mhcl_desc &d, int M, const void *x, const float *vr,
                             float *partials, float *g_W, hipStream_t s);
hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
// a fill kernel (safe under graph capture, unlike a memset node)
hipError_t launch_fill_zero(float *p, size_t count, hipStream_t s);
// g_b [M] and g_alpha [3] from gz [T, M+3]; part is scratch of
// param_sum_blocks(d) * (M+3) floats
int param_sum_blocks(const mhcl_desc &d);
hipError_t launch_param_sums(const mhcl_desc &d, int M, const float *gz, float *g_b, float *g_alpha,
                             float *part, hipStream_t s);
// the same over `rows` rows of [M+3] (rows <= T: `part` as above is large enough)
hipError_t launch_param_sums_rows(int64_t rows, int M, const float *src, float *g_b,
                                  float *g_alpha, float *part, hipStream_t s);

// ---- permutation-subset form (run-time table d.perm, n up to 8) --------------
// eight lanes per token: permutation subsets and the full form at n = 5
bool coeffs_group_ok(const mhcl_desc &d);
hipError_t launch_coeffs_group(const mhcl_desc &d, int parts, const float *u_raw,
                               const float *sumsq, const float *b, const float *alpha,
                               float *H_res, float *H_pre, float *H_post, hipStream_t s);
hipError_t launch_coeffs_bwd_subset(const mhcl_desc &d, int parts, const float *u_raw,
                                    const float *sumsq, const float *b, const float *alpha,
                                    const float *g_H_res, const float *g_H_pre,
                                    const float *g_H_post, const BwdTokenBufs &o, hipStream_t s);

// ---- diagnostics ----------------------------------------------------------
// z [T,M] and spread [T] (max - min of the residual logits); either may be null
hipError_t launch_logits(const mhcl_desc &d, int M, int parts, const float *u_raw,
                         const float *sumsq, const float *b, const float *alpha, float *z,
                         float *spread, hipStream_t s);
hipError_t launch_ds_chain(int n, int L, int64_t T, const float *H, float *colsum, float *l1,
                           float *prod, float *prod_colsum, float *prod_l1, hipStream_t s);

// ---- bf16 fast path (MFMA projections); needs fast_path_ok(desc) ---------
bool fast_path_ok(const mhcl_desc &d);
// The MFMA projection may split K over up to kMaxKSplit blocks per token tile;
// u_raw and sumsq then hold that many slices ([parts][T][M], [parts][T]).
constexpr int kMaxKSplit = 4;
int proj_ksplit(const mhcl_desc &d);
size_t packed_w_b_bytes(const mhcl_desc &d, int M);
// packs W (B layout) and, in the same launch, clears `nzero` floats at `zero`
hipError_t launch_pack_w_b(const mhcl_desc &d, int M, const float *W, void *Wp, hipStream_t s,
                           float *zero = nullptr, size_t nzero = 0);
hipError_t launch_proj_mfma(const mhcl_desc &d, int M, const void *x, const void *Wp, float *u_raw,
                            float *sumsq, hipStream_t s);

// Single-read forward (projection slices, H_pre and h from one read of x): bf16 fast path
// with at most 32 logits, C a multiple of 256 from 1024 to 8192, enough tokens to fill the pipeline.
bool fwd_once_ok(const mhcl_desc &d);
struct OnceWs {
  float *u_part, *sumsq_part;   // [parts][T][M], [parts][T]: one slice per 256-column part
  char *Wp;                     // packed W (B layout)
  unsigned long long *xchg;     // exchange rings of the kernel (zeroed by its launcher)
  size_t xchg_words, bytes;
  int parts;
  OnceWs(const mhcl_desc &d, void *ws);
};
// *usable == false on return with hipSuccess: this device cannot hold the kernel's grid at
// once (the caller then takes the two-kernel path).
hipError_t prepare_fwd_once(const mhcl_desc &d, int M, bool *usable);
// the kernel itself; w.Wp must hold the packed W and the w.xchg_words words at w.xchg must be
// zero (tags count from 1 in every launch)
hipError_t launch_fwd_once(const mhcl_desc &d, int M, const void *x, const float *b,
                           const float *alpha, const OnceWs &w, void *h, hipStream_t s);

// fused backward on the fast path (needs fast_bwd_ok(desc))
bool fast_bwd_ok(const mhcl_desc &d);
bool fast_bwd_whi(const mhcl_desc &d);    // wide case, n >= 5, where W fits LDS as one fp16 part: that pass 2 as one kernel
bool fast_bwd_wide(const mhcl_desc &d);   // n >= 5 or a subset: pass 2 split into W vr and the mixing
int gw_chunks_fast(const mhcl_desc &d);
struct FastBwdWs {
  // gz: [ceil(T/64)][M+3] sums of g_z and g_z u over each 64 tokens
  // wmax_part: partial maxima of |W|; wscale: {scale, 1 / scale} of the fp16 copy of W
  float *u_raw, *sumsq, *gH_res, *gH_pre, *gH_post, *cpk, *gz, *partials, *psum, *D, *wmax_part, *wscale;
  uint16_t *vr_hi, *vr_lo, *vrT_hi, *vrT_lo;
  char *Wp, *Wa;
  int CP, MP32, MP16, parts;
  size_t bytes;
  FastBwdWs(const mhcl_desc &d, void *ws);
};
hipError_t launch_pack_w_ab(const mhcl_desc &d, int M, const float *W, const FastBwdWs &w,
                            hipStream_t s);
hipError_t launch_bwd_reduce(const mhcl_desc &d, int M, const void *x, const void *y,
                             const void *g_xout, const void *g_h, const FastBwdWs &w,
                             hipStream_t s);
hipError_t launch_bwd_dots_fast(const mhcl_desc &d, const void *x, const void *y, const void *g_xout,
                                const void *g_h, const FastBwdWs &w, hipStream_t s);
hipError_t launch_bwd_epilogue_fast(const mhcl_desc &d, const float *b, const float *alpha,
                                    const FastBwdWs &w, hipStream_t s);
// the same stage for the permutation-subset form (run-time table)
hipError_t launch_bwd_epilogue_group(const mhcl_desc &d, const float *b, const float *alpha,
                                     const FastBwdWs &w, hipStream_t s);
hipError_t launch_bwd_out_wide(const mhcl_desc &d, int M, const void *x, const void *g_xout,
                               const void *g_h, const FastBwdWs &w, void *g_x, void *g_y,
                               hipStream_t s);
hipError_t launch_bwd_out_gw(const mhcl_desc &d, int M, const void *x, const void *g_xout,
                             const void *g_h, const FastBwdWs &w, void *g_x, void *g_y, float *g_W,
                             hipStream_t s);
hipError_t launch_bwd_gw(const mhcl_desc &d, int M, const void *x, const FastBwdWs &w, float *g_W,
                         hipStream_t s);
// g_W from the chunks' partial sums (none if chunks == 1) and g_b, g_alpha from the
// [rows, M+3] per-64-token sums of g_z, in one launch
hipError_t launch_bwd_finish(const float *partials, size_t size, int chunks, float *g_W,
                             const float *gz_rows, int64_t rows, int M, float *g_b, float *g_alpha,
                             hipStream_t s);
int fast_gw_chunks(const mhcl_desc &d);

}  // namespace mhcl
