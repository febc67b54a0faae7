// C ABI of libmhcl: validation, workspace layout, dispatch.  See include/mhcl.h.
#include "mhcl_common.h"
#include "mhcl_internal.h"

#include <mutex>

using namespace mhcl;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_desc(const mhcl_desc *d) {
  if (!d) return MHCL_ERR_INVALID_ARG;
  if (d->res_mode != MHCL_RES_LITE && d->res_mode != MHCL_RES_SK && d->res_mode != MHCL_RES_SUBSET)
    return MHCL_ERR_INVALID_ARG;
  if (d->n < 1 || d->n > (d->res_mode == MHCL_RES_SUBSET ? kMaxNSubset : kMaxN))
    return MHCL_ERR_INVALID_ARG;
  if (d->res_mode == MHCL_RES_SUBSET && (d->n_perm < 1 || d->n_perm > kMaxPerm || !d->perm))
    return MHCL_ERR_INVALID_ARG;
  if (d->C < 8 || d->C % 8 != 0) return MHCL_ERR_INVALID_ARG;
  if (d->T < 0) return MHCL_ERR_INVALID_ARG;
  if (d->io_dtype != MHCL_BF16 && d->io_dtype != MHCL_F32) return MHCL_ERR_INVALID_ARG;
  if (d->res_mode == MHCL_RES_SK && (d->sk_iters < 1 || d->sk_iters > kMaxSkIters))
    return MHCL_ERR_INVALID_ARG;
  if (!(d->eps >= 0.f)) return MHCL_ERR_INVALID_ARG;
  // index arithmetic: one launch addresses at most 2^31 - 1 blocks, and a
  // token's flattened row must fit an int
  if (static_cast<int64_t>(d->n) * d->C > (1 << 24)) return MHCL_ERR_UNSUPPORTED;
  if (d->T > (static_cast<int64_t>(1) << 31) - 1) return MHCL_ERR_UNSUPPORTED;
  if (d->T * (d->C / 4) / 256 > (static_cast<int64_t>(1) << 31) - 1) return MHCL_ERR_UNSUPPORTED;
  return MHCL_OK;
}

template <typename... P>
bool all_ok(P... p) {
  return ((p != nullptr && aligned16(p)) && ...);
}

int logits(const mhcl_desc &d) { return res_logits(d) + 2 * d.n; }

// ---- workspace layouts -----------------------------------------------------
struct CoeffsWs {
  float *u_raw, *sumsq;
  char *Wp;   // packed W (fast path only)
  size_t bytes;
  CoeffsWs(const mhcl_desc &d, void *ws) {
    WsCursor c(ws);
    const size_t T = static_cast<size_t>(d.T);
    const size_t parts = static_cast<size_t>(proj_ksplit(d));
    u_raw = c.take<float>(parts * T * logits(d));
    sumsq = c.take<float>(parts * T);
    Wp = fast_path_ok(d) ? c.take<char>(packed_w_b_bytes(d, logits(d))) : nullptr;
    bytes = c.off;
  }
};

struct BwdWs {
  float *u_raw, *sumsq, *gH_res, *gH_pre, *gH_post, *partials, *psum;
  char *Wp;
  BwdTokenBufs tok;
  size_t bytes;
  BwdWs(const mhcl_desc &d, void *ws, bool need_dots) {
    WsCursor c(ws);
    const size_t T = static_cast<size_t>(d.T);
    const int M = logits(d), n = d.n;
    const size_t parts = static_cast<size_t>(proj_ksplit(d));
    u_raw = c.take<float>(parts * T * M);
    sumsq = c.take<float>(parts * T);
    tok.H_res = c.take<float>(T * n * n);
    tok.H_pre = c.take<float>(T * n);
    tok.H_post = c.take<float>(T * n);
    tok.vr = c.take<float>(T * M);
    tok.coefx = c.take<float>(T);
    tok.gz = c.take<float>(T * (M + 3));
    gH_res = gH_pre = gH_post = nullptr;
    if (need_dots) {
      gH_res = c.take<float>(T * n * n);
      gH_pre = c.take<float>(T * n);
      gH_post = c.take<float>(T * n);
    }
    const int chunks = gw_chunks_generic(d);
    partials = chunks > 1 ? c.take<float>(static_cast<size_t>(chunks) * n * d.C * M) : nullptr;
    Wp = fast_path_ok(d) ? c.take<char>(packed_w_b_bytes(d, M)) : nullptr;
    psum = c.take<float>(static_cast<size_t>(param_sum_blocks(d)) * (M + 3));
    bytes = c.off;
  }
};

// Per-thread arming of event brackets around one stage (mhcl_profile_next_call).
thread_local int t_stage = MHCL_STAGE_NONE;
thread_local hipEvent_t t_ev_start = nullptr, t_ev_stop = nullptr;

struct StageBracket {
  bool on;
  hipStream_t s;
  StageBracket(int stage, hipStream_t stream) : on(stage == t_stage && t_ev_start), s(stream) {
    if (on) (void)hipEventRecord(t_ev_start, s);
  }
  ~StageBracket() {
    if (on) (void)hipEventRecord(t_ev_stop, s);
  }
};
struct Disarm {
  ~Disarm() { t_stage = MHCL_STAGE_NONE; }
};

#define MHCL_HIP(expr)                              \
  do {                                              \
    if ((expr) != hipSuccess) return MHCL_ERR_HIP;  \
  } while (0)

// u_raw, sumsq of every token: MFMA kernel when the shape allows, else plain ALU
hipError_t run_projection(const mhcl_desc &d, const void *x, const float *W, float *u_raw,
                          float *sumsq, char *Wp, int stage, hipStream_t s) {
  const int M = logits(d);
  if (fast_path_ok(d)) {
    hipError_t e = launch_pack_w_b(d, M, W, Wp, s);
    if (e != hipSuccess) return e;
    StageBracket br(stage, s);
    return launch_proj_mfma(d, M, x, Wp, u_raw, sumsq, s);
  }
  StageBracket br(stage, s);
  return launch_proj_generic(d, M, x, W, u_raw, sumsq, s);
}

// per-token coefficients from the projection: compile-time tables for the full
// permutation and Sinkhorn-Knopp forms, the run-time table for a subset
hipError_t run_coeffs_epilogue(const mhcl_desc &d, int parts, const float *u_raw,
                               const float *sumsq, const float *b, const float *alpha,
                               float *H_res, float *H_pre, float *H_post, hipStream_t s) {
  if (coeffs_group_ok(d))
    return launch_coeffs_group(d, parts, u_raw, sumsq, b, alpha, H_res, H_pre, H_post, s);
  return launch_coeffs_epilogue(d, parts, u_raw, sumsq, b, alpha, H_res, H_pre, H_post, s);
}
hipError_t run_coeffs_bwd_epilogue(const mhcl_desc &d, const float *u_raw, const float *sumsq,
                                   const float *b, const float *alpha, const float *g_H_res,
                                   const float *g_H_pre, const float *g_H_post,
                                   const BwdTokenBufs &o, hipStream_t s) {
  if (d.res_mode == MHCL_RES_SUBSET)
    return launch_coeffs_bwd_subset(d, proj_ksplit(d), u_raw, sumsq, b, alpha, g_H_res, g_H_pre,
                                    g_H_post, o, s);
  return launch_coeffs_bwd_epilogue(d, proj_ksplit(d), u_raw, sumsq, b, alpha, g_H_res, g_H_pre,
                                    g_H_post, o, s);
}

// argument checks of mhcl_fwd_coeffs_pre and its allocation-free variant
int check_fwd_coeffs_pre(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                         const float *alpha, const float *H_res, const float *H_pre,
                         const float *H_post, const void *h) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, (const void *)W, (const void *)b, (const void *)alpha, (const void *)H_res,
              (const void *)H_pre, (const void *)H_post, h))
    return MHCL_ERR_INVALID_ARG;
  return MHCL_OK;
}

// scratch of mhcl_fwd_coeffs_pre: the larger of the two layouts where the single-read kernel applies
size_t fwd_coeffs_pre_ws_bytes(const mhcl_desc &d) {
  const size_t two = CoeffsWs(d, nullptr).bytes;
  if (!fwd_once_ok(d)) return two;
  const size_t one = OnceWs(d, nullptr).bytes;
  return one > two ? one : two;
}

// projection, coefficients, pre-aggregate with `ws` as the scratch (aligned; large enough for
// the single-read layout if `once`, else for the two-kernel layout)
int run_fwd_coeffs_pre(const mhcl_desc &d, const void *x, const float *W, const float *b,
                       const float *alpha, float *H_res, float *H_pre, float *H_post, void *h,
                       void *ws, bool once, hipStream_t s) {
  Disarm disarm;
  if (once && fwd_once_ok(d)) {
    OnceWs w(d, ws);
    bool usable = false;
    MHCL_HIP(prepare_fwd_once(d, logits(d), &usable));
    if (usable) {
      // (the exchange rings are zeroed by the launch that packs W)
      MHCL_HIP(launch_pack_w_b(d, logits(d), W, w.Wp, s, reinterpret_cast<float *>(w.xchg),
                               w.xchg_words * 2));
      {
        StageBracket br(MHCL_STAGE_FWD_PROJ, s);
        MHCL_HIP(launch_fwd_once(d, logits(d), x, b, alpha, w, h, s));
      }
      MHCL_HIP(run_coeffs_epilogue(d, w.parts, w.u_part, w.sumsq_part, b, alpha, H_res, H_pre,
                                   H_post, s));
      return MHCL_OK;
    }
  }
  CoeffsWs w(d, ws);
  MHCL_HIP(run_projection(d, x, W, w.u_raw, w.sumsq, w.Wp, MHCL_STAGE_FWD_PROJ, s));
  MHCL_HIP(run_coeffs_epilogue(d, proj_ksplit(d), w.u_raw, w.sumsq, b, alpha, H_res, H_pre, H_post, s));
  {
    StageBracket br(MHCL_STAGE_FWD_PRE, s);
    MHCL_HIP(launch_pre(d, x, H_pre, h, s));
  }
  return MHCL_OK;
}

// Scratch of mhcl_fwd_coeffs_pre_static: one array per GPU, resident from the moment the
// code object is loaded on that GPU until the process ends.  `scratch` itself is only a
// host-side handle of the symbol; the array's device address is looked up once per device
// and kernels are given that address.
__device__ __align__(256) unsigned char scratch[MHCL_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MHCL_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MHCL_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MHCL_OK;
}

}  // namespace

extern "C" {

const char *mhcl_status_string(int status) {
  switch (status) {
    case MHCL_OK: return "ok";
    case MHCL_ERR_INVALID_ARG: return "invalid argument";
    case MHCL_ERR_UNSUPPORTED: return "unsupported configuration";
    case MHCL_ERR_WORKSPACE: return "workspace missing or too small";
    case MHCL_ERR_HIP: return "HIP runtime error at launch";
  }
  return "unknown status";
}

int mhcl_validate(const mhcl_desc *desc) { return check_desc(desc); }

int32_t mhcl_logit_count(const mhcl_desc *desc) {
  if (check_desc(desc) != MHCL_OK) return -1;
  return logits(*desc);
}

size_t mhcl_workspace_bytes(const mhcl_desc *desc, int op) {
  if (check_desc(desc) != MHCL_OK) return 0;
  size_t b = 0;
  switch (op) {
    case MHCL_OP_COEFFS: b = CoeffsWs(*desc, nullptr).bytes; break;
    case MHCL_OP_FWD_COEFFS_PRE: b = fwd_coeffs_pre_ws_bytes(*desc); break;
    case MHCL_OP_COEFFS_BWD: b = BwdWs(*desc, nullptr, false).bytes; break;
    case MHCL_OP_BWD_FUSED:
      b = fast_bwd_ok(*desc) ? FastBwdWs(*desc, nullptr).bytes : BwdWs(*desc, nullptr, true).bytes;
      break;
    default: return 0;
  }
  return b < 256 ? 256 : b;
}

int mhcl_perm_table(int32_t n, int8_t *sigma) {
  if (!sigma || n < 1 || n > kMaxN) return MHCL_ERR_INVALID_ARG;
  auto copy = [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    for (int k = 0; k < factorial(N); ++k)
      for (int i = 0; i < N; ++i) sigma[k * N + i] = Perm<N>::tab.s[k][i];
  };
  switch (n) {
    case 1: copy(std::integral_constant<int, 1>{}); break;
    case 2: copy(std::integral_constant<int, 2>{}); break;
    case 3: copy(std::integral_constant<int, 3>{}); break;
    case 4: copy(std::integral_constant<int, 4>{}); break;
    case 5: copy(std::integral_constant<int, 5>{}); break;
  }
  return MHCL_OK;
}

int mhcl_profile_next_call(int stage, void *ev_start, void *ev_stop) {
  if (stage < MHCL_STAGE_NONE || stage > MHCL_STAGE_BWD_GW) return MHCL_ERR_INVALID_ARG;
  if (stage != MHCL_STAGE_NONE && (!ev_start || !ev_stop)) return MHCL_ERR_INVALID_ARG;
  t_stage = stage;
  t_ev_start = static_cast<hipEvent_t>(ev_start);
  t_ev_stop = static_cast<hipEvent_t>(ev_stop);
  return MHCL_OK;
}

int mhcl_debug_copy(void *dst, const void *src, size_t bytes, void *stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0)
    return MHCL_ERR_INVALID_ARG;
  MHCL_HIP(launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
  return MHCL_OK;
}

int mhcl_coeffs(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                const float *alpha, float *H_res, float *H_pre, float *H_post, void *ws,
                size_t ws_bytes, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, (const void *)W, (const void *)b, (const void *)alpha, (const void *)H_res,
              (const void *)H_pre, (const void *)H_post))
    return MHCL_ERR_INVALID_ARG;
  if (!ws || !aligned16(ws) || ws_bytes < mhcl_workspace_bytes(desc, MHCL_OP_COEFFS))
    return MHCL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CoeffsWs w(*desc, ws);
  Disarm disarm;
  MHCL_HIP(run_projection(*desc, x, W, w.u_raw, w.sumsq, w.Wp, MHCL_STAGE_FWD_PROJ, s));
  MHCL_HIP(run_coeffs_epilogue(*desc, proj_ksplit(*desc), w.u_raw, w.sumsq, b, alpha, H_res, H_pre,
                               H_post, s));
  return MHCL_OK;
}

int mhcl_logits(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                const float *alpha, float *z, float *log_inv_nu, void *ws, size_t ws_bytes,
                void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, (const void *)W, (const void *)b, (const void *)alpha))
    return MHCL_ERR_INVALID_ARG;
  if ((!z && !log_inv_nu) || !aligned16(z) || !aligned16(log_inv_nu)) return MHCL_ERR_INVALID_ARG;
  if (!ws || !aligned16(ws) || ws_bytes < mhcl_workspace_bytes(desc, MHCL_OP_COEFFS))
    return MHCL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CoeffsWs w(*desc, ws);
  Disarm disarm;
  MHCL_HIP(run_projection(*desc, x, W, w.u_raw, w.sumsq, w.Wp, MHCL_STAGE_FWD_PROJ, s));
  MHCL_HIP(launch_logits(*desc, mhcl_logit_count(desc), proj_ksplit(*desc), w.u_raw, w.sumsq, b,
                         alpha, z, log_inv_nu, s));
  return MHCL_OK;
}

int mhcl_ds_chain(int32_t n, int32_t L, int64_t T, const float *H, float *colsum, float *l1,
                  float *prod, float *prod_colsum, float *prod_l1, void *stream) {
  if (n < 1 || n > kMaxNSubset || L < 1 || T < 0) return MHCL_ERR_INVALID_ARG;
  if (T == 0) return MHCL_OK;
  if (!H || !aligned16(H)) return MHCL_ERR_INVALID_ARG;
  if (!colsum && !l1 && !prod && !prod_colsum && !prod_l1) return MHCL_ERR_INVALID_ARG;
  if (!aligned16(colsum) || !aligned16(l1) || !aligned16(prod) || !aligned16(prod_colsum) ||
      !aligned16(prod_l1))
    return MHCL_ERR_INVALID_ARG;
  Disarm disarm;
  MHCL_HIP(launch_ds_chain(n, L, T, H, colsum, l1, prod, prod_colsum, prod_l1,
                           static_cast<hipStream_t>(stream)));
  return MHCL_OK;
}

int mhcl_pre(const mhcl_desc *desc, const void *x, const float *H_pre, void *h, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, (const void *)H_pre, (const void *)h)) return MHCL_ERR_INVALID_ARG;
  Disarm disarm;
  StageBracket br(MHCL_STAGE_FWD_PRE, static_cast<hipStream_t>(stream));
  MHCL_HIP(launch_pre(*desc, x, H_pre, h, static_cast<hipStream_t>(stream)));
  return MHCL_OK;
}

int mhcl_post(const mhcl_desc *desc, const void *x, const void *y, const float *H_res,
              const float *H_post, void *x_out, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, y, (const void *)H_res, (const void *)H_post, (const void *)x_out))
    return MHCL_ERR_INVALID_ARG;
  if (x_out == x) return MHCL_ERR_INVALID_ARG;
  Disarm disarm;
  StageBracket br(MHCL_STAGE_POST, static_cast<hipStream_t>(stream));
  MHCL_HIP(launch_post(*desc, x, y, H_res, H_post, x_out, static_cast<hipStream_t>(stream)));
  return MHCL_OK;
}

int mhcl_fwd_coeffs_pre(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                        const float *alpha, float *H_res, float *H_pre, float *H_post, void *h,
                        void *ws, size_t ws_bytes, void *stream) {
  if (int e = check_fwd_coeffs_pre(desc, x, W, b, alpha, H_res, H_pre, H_post, h)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!ws || !aligned16(ws) || ws_bytes < mhcl_workspace_bytes(desc, MHCL_OP_FWD_COEFFS_PRE))
    return MHCL_ERR_WORKSPACE;
  return run_fwd_coeffs_pre(*desc, x, W, b, alpha, H_res, H_pre, H_post, h, ws, true,
                            static_cast<hipStream_t>(stream));
}

int mhcl_fwd_coeffs_pre_static(const mhcl_desc *desc, const void *x, const float *W,
                               const float *b, const float *alpha, float *H_res, float *H_pre,
                               float *H_post, void *h, void *stream) {
  if (int e = check_fwd_coeffs_pre(desc, x, W, b, alpha, H_res, H_pre, H_post, h)) return e;
  if (desc->T == 0) return MHCL_OK;
  if (CoeffsWs(*desc, nullptr).bytes > MHCL_STATIC_SCRATCH_BYTES)
    return MHCL_ERR_WORKSPACE;   // the shape needs more scratch than the static array holds
  void *ws = nullptr;
  if (int e = static_scratch(&ws)) return e;
  // every word of the workspace this call reads is written by its own kernels first, so
  // what the previous call left in the array does not matter
  return run_fwd_coeffs_pre(*desc, x, W, b, alpha, H_res, H_pre, H_post, h, ws, false,
                            static_cast<hipStream_t>(stream));
}

int mhcl_post_bwd(const mhcl_desc *desc, const void *x, const void *y, const float *H_res,
                  const float *H_post, const void *g_xout, void *g_x, void *g_y, float *g_H_res,
                  float *g_H_post, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, y, (const void *)H_res, (const void *)H_post, g_xout, (const void *)g_x,
              (const void *)g_y, (const void *)g_H_res, (const void *)g_H_post))
    return MHCL_ERR_INVALID_ARG;
  Disarm disarm;
  MHCL_HIP(launch_post_bwd(*desc, x, y, H_res, H_post, g_xout, g_x, g_y, g_H_res, g_H_post,
                           static_cast<hipStream_t>(stream)));
  return MHCL_OK;
}

int mhcl_pre_bwd(const mhcl_desc *desc, const void *x, const float *H_pre, const void *g_h,
                 void *g_x, float *g_H_pre, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) return MHCL_OK;   // per-token tensors may then be null
  if (!all_ok(x, (const void *)H_pre, g_h, (const void *)g_x, (const void *)g_H_pre))
    return MHCL_ERR_INVALID_ARG;
  Disarm disarm;
  MHCL_HIP(launch_pre_bwd(*desc, x, H_pre, g_h, g_x, g_H_pre, static_cast<hipStream_t>(stream)));
  return MHCL_OK;
}

int mhcl_coeffs_bwd(const mhcl_desc *desc, const void *x, const float *W, const float *b,
                    const float *alpha, const float *g_H_res, const float *g_H_pre,
                    const float *g_H_post, void *g_x, float *g_W, float *g_b, float *g_alpha,
                    void *ws, size_t ws_bytes, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) {   // sums over no tokens; per-token tensors may be null
    if (!all_ok((const void *)g_W, (const void *)g_b, (const void *)g_alpha))
      return MHCL_ERR_INVALID_ARG;
    hipStream_t s0 = static_cast<hipStream_t>(stream);
    const int M0 = logits(*desc);
    MHCL_HIP(launch_fill_zero(g_W, static_cast<size_t>(desc->n) * desc->C * M0, s0));
    MHCL_HIP(launch_fill_zero(g_b, M0, s0));
    MHCL_HIP(launch_fill_zero(g_alpha, 3, s0));
    return MHCL_OK;
  }
  if (!all_ok(x, (const void *)W, (const void *)b, (const void *)alpha, (const void *)g_H_res,
              (const void *)g_H_pre, (const void *)g_H_post, (const void *)g_x, (const void *)g_W,
              (const void *)g_b, (const void *)g_alpha))
    return MHCL_ERR_INVALID_ARG;
  if (!ws || !aligned16(ws) || ws_bytes < mhcl_workspace_bytes(desc, MHCL_OP_COEFFS_BWD))
    return MHCL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int M = logits(*desc);
  BwdWs w(*desc, ws, false);
  Disarm disarm;
  MHCL_HIP(run_projection(*desc, x, W, w.u_raw, w.sumsq, w.Wp, MHCL_STAGE_BWD_REDUCE, s));
  MHCL_HIP(run_coeffs_bwd_epilogue(*desc, w.u_raw, w.sumsq, b, alpha, g_H_res, g_H_pre, g_H_post,
                                   w.tok, s));
  MHCL_HIP(launch_gx_generic(*desc, M, false, x, W, nullptr, nullptr, w.tok, g_x, nullptr, s));
  MHCL_HIP(launch_gw_generic(*desc, M, x, w.tok.vr, w.partials, g_W, s));
  MHCL_HIP(launch_param_sums(*desc, M, w.tok.gz, g_b, g_alpha, w.psum, s));
  return MHCL_OK;
}

int mhcl_bwd_fused(const mhcl_desc *desc, const void *x, const void *y, const float *W,
                   const float *b, const float *alpha, const void *g_xout, const void *g_h,
                   void *g_x, void *g_y, float *g_W, float *g_b, float *g_alpha, void *ws,
                   size_t ws_bytes, void *stream) {
  if (int e = check_desc(desc)) return e;
  if (desc->T == 0) {   // sums over no tokens; per-token tensors may be null
    if (!all_ok((const void *)g_W, (const void *)g_b, (const void *)g_alpha))
      return MHCL_ERR_INVALID_ARG;
    hipStream_t s0 = static_cast<hipStream_t>(stream);
    const int M0 = logits(*desc);
    MHCL_HIP(launch_fill_zero(g_W, static_cast<size_t>(desc->n) * desc->C * M0, s0));
    MHCL_HIP(launch_fill_zero(g_b, M0, s0));
    MHCL_HIP(launch_fill_zero(g_alpha, 3, s0));
    return MHCL_OK;
  }
  if (!all_ok(x, y, (const void *)W, (const void *)b, (const void *)alpha, g_xout, g_h,
              (const void *)g_x, (const void *)g_W, (const void *)g_b, (const void *)g_alpha))
    return MHCL_ERR_INVALID_ARG;
  if (g_y && !aligned16(g_y)) return MHCL_ERR_INVALID_ARG;   // g_y is optional
  if (!ws || !aligned16(ws) || ws_bytes < mhcl_workspace_bytes(desc, MHCL_OP_BWD_FUSED))
    return MHCL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int M = logits(*desc);
  Disarm disarm;
  if (fast_bwd_ok(*desc)) {
    FastBwdWs f(*desc, ws);
    const bool wide = fast_bwd_wide(*desc);
    MHCL_HIP(launch_pack_w_ab(*desc, M, W, f, s));
    {
      StageBracket br(MHCL_STAGE_BWD_REDUCE, s);
      if (wide) {
        MHCL_HIP(launch_proj_mfma(*desc, M, x, f.Wp, f.u_raw, f.sumsq, s));
        MHCL_HIP(launch_bwd_dots_fast(*desc, x, y, g_xout, g_h, f, s));
      } else {
        MHCL_HIP(launch_bwd_reduce(*desc, M, x, y, g_xout, g_h, f, s));
      }
    }
    if (coeffs_group_ok(*desc))
      MHCL_HIP(launch_bwd_epilogue_group(*desc, b, alpha, f, s));
    else
      MHCL_HIP(launch_bwd_epilogue_fast(*desc, b, alpha, f, s));
    if (wide) {
      {
        StageBracket br(MHCL_STAGE_BWD_OUT, s);
        MHCL_HIP(launch_bwd_out_wide(*desc, M, x, g_xout, g_h, f, g_x, g_y, s));
      }
      StageBracket br(MHCL_STAGE_BWD_GW, s);
      MHCL_HIP(launch_bwd_gw(*desc, M, x, f, g_W, s));
    } else {
      StageBracket br(MHCL_STAGE_BWD_OUT, s);
      MHCL_HIP(launch_bwd_out_gw(*desc, M, x, g_xout, g_h, f, g_x, g_y, g_W, s));
    }
    MHCL_HIP(launch_bwd_finish(f.partials, static_cast<size_t>(desc->n) * desc->C * M,
                               fast_gw_chunks(*desc), g_W, f.gz, (desc->T + 63) / 64, M, g_b, g_alpha,
                               s));
    return MHCL_OK;
  }
  BwdWs w(*desc, ws, true);
  MHCL_HIP(run_projection(*desc, x, W, w.u_raw, w.sumsq, w.Wp, MHCL_STAGE_BWD_REDUCE, s));
  MHCL_HIP(launch_bwd_dots(*desc, x, y, g_xout, g_h, w.gH_res, w.gH_post, w.gH_pre, s));
  MHCL_HIP(run_coeffs_bwd_epilogue(*desc, w.u_raw, w.sumsq, b, alpha, w.gH_res, w.gH_pre,
                                   w.gH_post, w.tok, s));
  {
    StageBracket br(MHCL_STAGE_BWD_OUT, s);
    MHCL_HIP(launch_gx_generic(*desc, M, true, x, W, g_xout, g_h, w.tok, g_x, g_y, s));
  }
  MHCL_HIP(launch_gw_generic(*desc, M, x, w.tok.vr, w.partials, g_W, s));
  MHCL_HIP(launch_param_sums(*desc, M, w.tok.gz, g_b, g_alpha, w.psum, s));
  return MHCL_OK;
}

}  // extern "C"
