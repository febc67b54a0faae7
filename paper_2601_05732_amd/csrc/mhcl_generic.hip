// Generic kernels of libmhcl: plain fp32 ALU arithmetic, any n in 1..5, bf16
// or f32 streams.  They serve f32 streams, shapes the MFMA kernels do not
// cover, and the separable entry points.  Every reduction runs in a fixed
// order, so results are bitwise reproducible.
#include "mhcl_common.h"
#include "mhcl_internal.h"

namespace mhcl {

namespace {

constexpr int kBlock = 256;

// n = 1..5: kernels that unroll the compile-time permutation table
template <typename F>
hipError_t dispatch_n5(int n, F &&f) {
  switch (n) {
    case 1: return f(std::integral_constant<int, 1>{});
    case 2: return f(std::integral_constant<int, 2>{});
    case 3: return f(std::integral_constant<int, 3>{});
    case 4: return f(std::integral_constant<int, 4>{});
    case 5: return f(std::integral_constant<int, 5>{});
  }
  return hipErrorInvalidValue;
}
// n = 1..8: the stream kernels (the permutation-subset form goes up to 8)
template <typename F>
hipError_t dispatch_n(int n, F &&f) {
  switch (n) {
    case 6: return f(std::integral_constant<int, 6>{});
    case 7: return f(std::integral_constant<int, 7>{});
    case 8: return f(std::integral_constant<int, 8>{});
  }
  return dispatch_n5(n, f);
}
template <typename F>
hipError_t dispatch_io(int io, F &&f) {
  if (io == MHCL_BF16) return f(BF16{});
  return f(F32{});
}
template <typename F>
hipError_t dispatch_mode(int mode, F &&f) {
  if (mode == MHCL_RES_LITE) return f(std::integral_constant<int, MHCL_RES_LITE>{});
  return f(std::integral_constant<int, MHCL_RES_SK>{});
}

// Sum over the block of CNT per-thread values (CNT <= 256); the totals land in
// red[0..cnt).  Fixed order: butterfly inside each wave, then waves 0..3.
template <int CNT>
__device__ __forceinline__ void block_sum(float (&v)[CNT], float *red /* [4*CNT] */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < CNT; ++i) {
    const float s = wave_sum(v[i]);
    if (lane == 0) red[wave * CNT + i] = s;
  }
  __syncthreads();
  if (threadIdx.x < CNT) {
    const int i = threadIdx.x;
    red[i] = ((red[i] + red[CNT + i]) + red[2 * CNT + i]) + red[3 * CNT + i];
  }
  __syncthreads();
}

// ------------------------------------------------------------ projection
// u_raw[t][m] = sum_k x_hat[t][k] W[k][m] and sumsq[t] = sum_k x_hat[t][k]^2
// (the two reductions over nC behind RMSNorm and the linear maps of Sec. 3.2).
// One block per kTok tokens; thread (m lane 0..31, k slice 0..7).
constexpr int kTok = 4;

template <typename IO>
__global__ __launch_bounds__(kBlock) void proj_generic_kernel(const void *__restrict__ x,
                                                              const float *__restrict__ W, int nC,
                                                              int M, int64_t T,
                                                              float *__restrict__ u_raw,
                                                              float *__restrict__ sumsq) {
  __shared__ float red[8][kTok][32];
  __shared__ float red2[4 * kTok];
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kTok;
  const int ml = threadIdx.x & 31, ks = threadIdx.x >> 5;
  int64_t row[kTok];
#pragma unroll
  for (int i = 0; i < kTok; ++i) row[i] = (t0 + i < T ? t0 + i : T - 1) * nC;

  float ss[kTok];
#pragma unroll
  for (int i = 0; i < kTok; ++i) ss[i] = 0.f;
  for (int k = threadIdx.x; k < nC; k += kBlock) {
#pragma unroll
    for (int i = 0; i < kTok; ++i) {
      const float v = IO::load1(x, row[i] + k);
      ss[i] += v * v;
    }
  }
  block_sum<kTok>(ss, red2);
  if (threadIdx.x < kTok && t0 + threadIdx.x < T) sumsq[t0 + threadIdx.x] = red2[threadIdx.x];

  for (int m0 = 0; m0 < M; m0 += 32) {
    const int m = m0 + ml;
    // nC / 8 terms per thread (2048 at n C = 16384): carried in fp64 so that this path,
    // the one f32 streams take, keeps its logits to fp32 rounding at any width
    double acc[kTok];
#pragma unroll
    for (int i = 0; i < kTok; ++i) acc[i] = 0.0;
    if (m < M) {
      for (int k = ks; k < nC; k += 8) {
        const double w = W[static_cast<size_t>(k) * M + m];
#pragma unroll
        for (int i = 0; i < kTok; ++i) acc[i] += static_cast<double>(IO::load1(x, row[i] + k)) * w;
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kTok; ++i) red[ks][i][ml] = static_cast<float>(acc[i]);
    __syncthreads();
    if (threadIdx.x < kTok * 32) {
      const int i = threadIdx.x >> 5;
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) s += red[q][i][ml];
      if (m < M && t0 + i < T) u_raw[(t0 + i) * M + m] = s;
    }
  }
}

// ------------------------------------------------------------ coefficients
template <int N, int MODE>
__global__ __launch_bounds__(128) void coeffs_epilogue_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha, int nC, float eps, int sk_iters,
    int64_t T, float *__restrict__ H_res, float *__restrict__ H_pre, float *__restrict__ H_post) {
  constexpr int R = Dims<N, MODE>::R, M = Dims<N, MODE>::M;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 128 + threadIdx.x;
  if (t >= T) return;
  float u[M], bb[M], a[R], Hr[N * N], Hp[N], Hq[N];
  float ssq = sumsq[t];
#pragma unroll
  for (int m = 0; m < M; ++m) { u[m] = u_raw[t * M + m]; bb[m] = b[m]; }
  for (int pt = 1; pt < parts; ++pt) {   // K-split slices, added in order
    ssq += sumsq[pt * T + t];
#pragma unroll
    for (int m = 0; m < M; ++m) u[m] += u_raw[(pt * T + t) * M + m];
  }
  const TokenParams p{alpha[0], alpha[1], alpha[2], eps, sk_iters};
  token_coeffs<N, MODE>(u, ssq, nC, bb, p, Hr, Hp, Hq, a);
#pragma unroll
  for (int e = 0; e < N * N; ++e) H_res[t * N * N + e] = Hr[e];
#pragma unroll
  for (int j = 0; j < N; ++j) { H_pre[t * N + j] = Hp[j]; H_post[t * N + j] = Hq[j]; }
}

// The same for many slices (at most 32 logits, M a multiple of 4): one thread per token would
// read them in as many dependent rounds, one logit at a time.  Here eight lanes share a token,
// lane c adds logits 4c..4c+3 of all slices in order (16-byte loads, a token's row of a slice
// is one contiguous request), the sums meet in LDS and one thread per token goes on: the 64
// tokens of a block in ONE full wave, a different one from block to block (a half-filled wave
// costs the same issue slots as a full one, and wave w of every block sits on the same SIMD:
// with 32 tokens per block in wave 0 this stage took 17 of the kernel's 22 us, now 4).
// Same order of additions as coeffs_epilogue_kernel, so the same bits.
template <int N, int MODE>
__global__ __launch_bounds__(512) void coeffs_epilogue_sliced_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha, int nC, float eps, int sk_iters,
    int64_t T, float *__restrict__ H_res, float *__restrict__ H_pre, float *__restrict__ H_post) {
  constexpr int R = Dims<N, MODE>::R, M = Dims<N, MODE>::M;
  static_assert(M % 4 == 0 && M <= 32, "rows of 16-byte pieces, eight lanes per token");
  __shared__ float su[64][M + 1];   // 64 tokens per block: M sums and the sum of squares
  const int tl = threadIdx.x >> 3, c = threadIdx.x & 7;
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * 64;
  int64_t t = t0 + tl;
  if (t > T - 1) t = T - 1;
  if (c < M / 4) {
    const float4 *row = reinterpret_cast<const float4 *>(u_raw + t * M) + c;
    const size_t stride = static_cast<size_t>(T) * M / 4;   // float4 per slice
    // (eight slices requested at a time, added in order: a loop of one load and one addition
    //  pays a memory round trip per slice)
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p0 = 0; p0 < parts; p0 += 8) {
      float4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = row[(p0 + i < parts ? p0 + i : parts - 1) * stride];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (p0 + i == 0) acc = v[0];
        else if (p0 + i < parts) { acc.x += v[i].x; acc.y += v[i].y; acc.z += v[i].z; acc.w += v[i].w; }
      }
    }
    su[tl][4 * c + 0] = acc.x; su[tl][4 * c + 1] = acc.y;
    su[tl][4 * c + 2] = acc.z; su[tl][4 * c + 3] = acc.w;
  }
  if (c == 7) {   // (the lane with the fewest logits to add, or none)
    float ssq = 0.f;
    for (int p0 = 0; p0 < parts; p0 += 8) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = sumsq[(p0 + i < parts ? p0 + i : parts - 1) * T + t];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (p0 + i == 0) ssq = v[0];
        else if (p0 + i < parts) ssq += v[i];
      }
    }
    su[tl][M] = ssq;
  }
  __syncthreads();
  if ((threadIdx.x >> 6) != (blockIdx.x & 7)) return;
  const int tk = threadIdx.x & 63;
  t = t0 + tk;
  if (t >= T) return;
  float u[M], bb[M], a[R], Hr[N * N], Hp[N], Hq[N];
#pragma unroll
  for (int m = 0; m < M; ++m) { u[m] = su[tk][m]; bb[m] = b[m]; }
  const float ssq = su[tk][M];
  const TokenParams p{alpha[0], alpha[1], alpha[2], eps, sk_iters};
  token_coeffs<N, MODE>(u, ssq, nC, bb, p, Hr, Hp, Hq, a);
#pragma unroll
  for (int e = 0; e < N * N; ++e) H_res[t * N * N + e] = Hr[e];
#pragma unroll
  for (int j = 0; j < N; ++j) { H_pre[t * N + j] = Hp[j]; H_post[t * N + j] = Hq[j]; }
}

template <int N, int MODE>
__global__ __launch_bounds__(128) void coeffs_bwd_epilogue_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha, const float *__restrict__ gH_res,
    const float *__restrict__ gH_pre, const float *__restrict__ gH_post, int nC, float eps,
    int sk_iters, int64_t T, BwdTokenBufs o) {
  constexpr int R = Dims<N, MODE>::R, M = Dims<N, MODE>::M;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 128 + threadIdx.x;
  if (t >= T) return;
  float u[M], bb[M], a[R], Hr[N * N], Hp[N], Hq[N], gz[M];
  float gr[N * N], gp[N], gq[N];
  float sums[(MODE == MHCL_RES_SK) ? 2 * kMaxSkIters * N : 1];
  float ssq = sumsq[t];
#pragma unroll
  for (int m = 0; m < M; ++m) { u[m] = u_raw[t * M + m]; bb[m] = b[m]; }
  for (int pt = 1; pt < parts; ++pt) {
    ssq += sumsq[pt * T + t];
#pragma unroll
    for (int m = 0; m < M; ++m) u[m] += u_raw[(pt * T + t) * M + m];
  }
#pragma unroll
  for (int e = 0; e < N * N; ++e) gr[e] = gH_res[t * N * N + e];
#pragma unroll
  for (int j = 0; j < N; ++j) { gp[j] = gH_pre[t * N + j]; gq[j] = gH_post[t * N + j]; }
  const TokenParams p{alpha[0], alpha[1], alpha[2], eps, sk_iters};
  const float r = token_coeffs<N, MODE>(u, ssq, nC, bb, p, Hr, Hp, Hq, a,
                                        (MODE == MHCL_RES_SK) ? sums : nullptr);
#pragma unroll
  for (int e = 0; e < N * N; ++e) o.H_res[t * N * N + e] = Hr[e];
#pragma unroll
  for (int j = 0; j < N; ++j) { o.H_pre[t * N + j] = Hp[j]; o.H_post[t * N + j] = Hq[j]; }
  token_coeffs_bwd<N, MODE>(gr, gp, gq, a, Hr, Hp, Hq, sums, sk_iters, gz);
  // z_m = alpha_g (r u_raw_m) + b_m
  float ga[3] = {0.f, 0.f, 0.f}, dot = 0.f;
#pragma unroll
  for (int m = 0; m < M; ++m) {
    const int g = m < R ? 0 : (m < R + N ? 1 : 2);
    const float al = g == 0 ? p.alpha_res : (g == 1 ? p.alpha_pre : p.alpha_post);
    const float vr = r * al * gz[m];
    o.gz[t * (M + 3) + m] = gz[m];
    o.vr[t * M + m] = vr;
    ga[g] += gz[m] * (r * u[m]);
    dot += vr * u[m];
  }
#pragma unroll
  for (int g = 0; g < 3; ++g) o.gz[t * (M + 3) + M + g] = ga[g];
  o.coefx[t] = (r * r / static_cast<float>(nC)) * dot;
}

// ------------------------------------------------------------ stream mixing
// h = H_pre x   (Eq. 1, argument of f): one thread per 16-byte chunk of h.
template <typename IO, int N>
__global__ __launch_bounds__(kBlock) void pre_kernel(const void *__restrict__ x,
                                                     const float *__restrict__ H_pre,
                                                     void *__restrict__ h, int C, int64_t T) {
  constexpr int V = IO::kVec;
  const int vpr = C / V;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= T * vpr) return;
  const int64_t t = idx / vpr;
  const int c = static_cast<int>(idx % vpr) * V;
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
#pragma unroll
  for (int j = 0; j < N; ++j) {
    float v[V];
    IO::load(x, (t * N + j) * C + c, v);
    const float w = H_pre[t * N + j];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] += w * v[e];
  }
  IO::store(h, t * C + c, acc);
}

// x_out = H_res x + H_post^T y   (Eq. 1)
template <typename IO, int N>
__global__ __launch_bounds__(kBlock) void post_kernel(const void *__restrict__ x,
                                                      const void *__restrict__ y,
                                                      const float *__restrict__ H_res,
                                                      const float *__restrict__ H_post,
                                                      void *__restrict__ x_out, int C, int64_t T) {
  constexpr int V = IO::kVec;
  const int vpr = C / V;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= T * vpr) return;
  const int64_t t = idx / vpr;
  const int c = static_cast<int>(idx % vpr) * V;
  float xv[N][V], yv[V];
#pragma unroll
  for (int j = 0; j < N; ++j) IO::load(x, (t * N + j) * C + c, xv[j]);
  IO::load(y, t * C + c, yv);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const float w = H_res[(t * N + i) * N + j];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += w * xv[j][e];
    }
    const float wp = H_post[t * N + i];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] += wp * yv[e];
    IO::store(x_out, (t * N + i) * C + c, acc);
  }
}

// Backward of post: one block per token.
//   g_y = sum_i H_post[i] g_xout[i];  g_x[j] = sum_i H_res[i][j] g_xout[i]
//   g_H_post[i] = <g_xout[i], y>;     g_H_res[i][j] = <g_xout[i], x[j]>
template <typename IO, int N>
__global__ __launch_bounds__(kBlock) void post_bwd_kernel(
    const void *__restrict__ x, const void *__restrict__ y, const float *__restrict__ H_res,
    const float *__restrict__ H_post, const void *__restrict__ g_xout, void *__restrict__ g_x,
    void *__restrict__ g_y, float *__restrict__ g_H_res, float *__restrict__ g_H_post, int C) {
  constexpr int V = IO::kVec;
  constexpr int D = N * N + N;
  __shared__ float red[4 * D];
  const int64_t t = blockIdx.x;
  float Hr[N * N], Hq[N], dots[D];
#pragma unroll
  for (int e = 0; e < N * N; ++e) Hr[e] = H_res[t * N * N + e];
#pragma unroll
  for (int i = 0; i < N; ++i) Hq[i] = H_post[t * N + i];
#pragma unroll
  for (int e = 0; e < D; ++e) dots[e] = 0.f;
  for (int c = threadIdx.x * V; c < C; c += kBlock * V) {
    float xv[N][V], gv[N][V], yv[V];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      IO::load(x, (t * N + j) * C + c, xv[j]);
      IO::load(g_xout, (t * N + j) * C + c, gv[j]);
    }
    IO::load(y, t * C + c, yv);
    float gy[V];
#pragma unroll
    for (int e = 0; e < V; ++e) gy[e] = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        gy[e] += Hq[i] * gv[i][e];
        dots[N * N + i] += gv[i][e] * yv[e];
      }
#pragma unroll
      for (int j = 0; j < N; ++j)
#pragma unroll
        for (int e = 0; e < V; ++e) dots[i * N + j] += gv[i][e] * xv[j][e];
    }
    IO::store(g_y, t * C + c, gy);
#pragma unroll
    for (int j = 0; j < N; ++j) {
      float gx[V];
#pragma unroll
      for (int e = 0; e < V; ++e) gx[e] = 0.f;
#pragma unroll
      for (int i = 0; i < N; ++i)
#pragma unroll
        for (int e = 0; e < V; ++e) gx[e] += Hr[i * N + j] * gv[i][e];
      IO::store(g_x, (t * N + j) * C + c, gx);
    }
  }
  block_sum<D>(dots, red);
  if (threadIdx.x < N * N) g_H_res[t * N * N + threadIdx.x] = red[threadIdx.x];
  if (threadIdx.x < N) g_H_post[t * N + threadIdx.x] = red[N * N + threadIdx.x];
}

// Backward of pre: g_x[j] += H_pre[j] g_h ; g_H_pre[j] = <g_h, x[j]>
template <typename IO, int N>
__global__ __launch_bounds__(kBlock) void pre_bwd_kernel(const void *__restrict__ x,
                                                         const float *__restrict__ H_pre,
                                                         const void *__restrict__ g_h,
                                                         void *__restrict__ g_x,
                                                         float *__restrict__ g_H_pre, int C) {
  constexpr int V = IO::kVec;
  __shared__ float red[4 * N];
  const int64_t t = blockIdx.x;
  float Hp[N], dots[N];
#pragma unroll
  for (int j = 0; j < N; ++j) { Hp[j] = H_pre[t * N + j]; dots[j] = 0.f; }
  for (int c = threadIdx.x * V; c < C; c += kBlock * V) {
    float gh[V];
    IO::load(g_h, t * C + c, gh);
#pragma unroll
    for (int j = 0; j < N; ++j) {
      float xv[V], gx[V];
      IO::load(x, (t * N + j) * C + c, xv);
      IO::load(g_x, (t * N + j) * C + c, gx);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        dots[j] += gh[e] * xv[e];
        gx[e] += Hp[j] * gh[e];
      }
      IO::store(g_x, (t * N + j) * C + c, gx);
    }
  }
  block_sum<N>(dots, red);
  if (threadIdx.x < N) g_H_pre[t * N + threadIdx.x] = red[threadIdx.x];
}

// The n^2 + 2n reductions over C that the backward needs, without outputs.
template <typename IO, int N>
__global__ __launch_bounds__(kBlock) void bwd_dots_kernel(
    const void *__restrict__ x, const void *__restrict__ y, const void *__restrict__ g_xout,
    const void *__restrict__ g_h, float *__restrict__ g_H_res, float *__restrict__ g_H_post,
    float *__restrict__ g_H_pre, int C) {
  constexpr int V = IO::kVec;
  constexpr int D = N * N + 2 * N;
  __shared__ float red[4 * D];
  const int64_t t = blockIdx.x;
  float dots[D];
#pragma unroll
  for (int e = 0; e < D; ++e) dots[e] = 0.f;
  for (int c = threadIdx.x * V; c < C; c += kBlock * V) {
    float xv[N][V], gv[N][V], yv[V], gh[V];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      IO::load(x, (t * N + j) * C + c, xv[j]);
      IO::load(g_xout, (t * N + j) * C + c, gv[j]);
    }
    IO::load(y, t * C + c, yv);
    IO::load(g_h, t * C + c, gh);
#pragma unroll
    for (int i = 0; i < N; ++i) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        dots[N * N + i] += gv[i][e] * yv[e];
        dots[N * N + N + i] += gh[e] * xv[i][e];
      }
#pragma unroll
      for (int j = 0; j < N; ++j)
#pragma unroll
        for (int e = 0; e < V; ++e) dots[i * N + j] += gv[i][e] * xv[j][e];
    }
  }
  block_sum<D>(dots, red);
  if (threadIdx.x < N * N) g_H_res[t * N * N + threadIdx.x] = red[threadIdx.x];
  if (threadIdx.x < N) {
    g_H_post[t * N + threadIdx.x] = red[N * N + threadIdx.x];
    g_H_pre[t * N + threadIdx.x] = red[N * N + N + threadIdx.x];
  }
}

// Gradient on x.  With vr = r alpha g_z and coefx = (r^2/nC) <vr, u_raw>, the
// RMSNorm + projection part is  W vr - x_hat coefx.
//   FUSED: g_x = H_res^T g_xout + H_pre g_h + (that part), rounded once;
//          g_y = sum_i H_post[i] g_xout[i]
//   else : g_x += (that part)
// One block per (token, 256 chunks of C); vr of the token sits in LDS.
template <typename IO, int N, bool FUSED>
__global__ __launch_bounds__(kBlock) void gx_generic_kernel(
    const void *__restrict__ x, const float *__restrict__ W, const void *__restrict__ g_xout,
    const void *__restrict__ g_h, BwdTokenBufs o, int M, int C, void *__restrict__ g_x,
    void *__restrict__ g_y) {
  constexpr int V = IO::kVec;
  __shared__ float sv[160];
  const int64_t t = blockIdx.y;
  for (int m = threadIdx.x; m < M; m += kBlock) sv[m] = o.vr[t * M + m];
  __syncthreads();
  const int c = (blockIdx.x * kBlock + threadIdx.x) * V;
  if (c >= C) return;
  const float cx = o.coefx[t];
  float gv[N][V], gh[V];
  if constexpr (FUSED) {
#pragma unroll
    for (int i = 0; i < N; ++i) IO::load(g_xout, (t * N + i) * C + c, gv[i]);
    IO::load(g_h, t * C + c, gh);
    if (g_y != nullptr) {   // (optional output)
      float gy[V];
#pragma unroll
      for (int e = 0; e < V; ++e) gy[e] = 0.f;
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float w = o.H_post[t * N + i];
#pragma unroll
        for (int e = 0; e < V; ++e) gy[e] += w * gv[i][e];
      }
      IO::store(g_y, t * C + c, gy);
    }
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    float xv[V], acc[V];
    IO::load(x, (t * N + j) * C + c, xv);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float *wr = W + static_cast<size_t>(j * C + c + e) * M;
      float s = 0.f;
      for (int m = 0; m < M; ++m) s += wr[m] * sv[m];
      acc[e] = s - xv[e] * cx;
    }
    if constexpr (FUSED) {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float w = o.H_res[(t * N + i) * N + j];
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += w * gv[i][e];
      }
      const float wp = o.H_pre[t * N + j];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += wp * gh[e];
    } else {
      float old[V];
      IO::load(g_x, (t * N + j) * C + c, old);
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += old[e];
    }
    IO::store(g_x, (t * N + j) * C + c, acc);
  }
}

// g_W[k][m] = sum_t x_hat[t][k] vr[t][m]: the one reduction over tokens.
// Block (k block of 8, token chunk); thread (m lane, k); partial sums per
// chunk, then added over chunks in order.
template <typename IO>
__global__ __launch_bounds__(kBlock) void gw_generic_kernel(const void *__restrict__ x,
                                                            const float *__restrict__ vr, int nC,
                                                            int M, int64_t T, int64_t chunk,
                                                            float *__restrict__ out) {
  const int ml = threadIdx.x & 31, kk = threadIdx.x >> 5;
  const int k = blockIdx.x * 8 + kk;
  const int64_t tb = static_cast<int64_t>(blockIdx.y) * chunk;
  const int64_t te = tb + chunk < T ? tb + chunk : T;
  float *dst = out + static_cast<size_t>(blockIdx.y) * nC * M;
  if (k >= nC) return;
  for (int m0 = 0; m0 < M; m0 += 32) {
    const int m = m0 + ml;
    if (m >= M) break;
    float acc = 0.f;
    for (int64_t t = tb; t < te; ++t) acc += IO::load1(x, t * nC + k) * vr[t * M + m];
    dst[static_cast<size_t>(k) * M + m] = acc;
  }
}

// out[i] = sum over chunks of part[c][i], in a fixed association: the four waves of a
// block each add every fourth chunk for the same 64 elements (several independent
// loads in flight), then ((s0 + s1) + s2) + s3.
__global__ __launch_bounds__(kBlock) void sum_partials_kernel(const float *__restrict__ part,
                                                              size_t size, int chunks,
                                                              float *__restrict__ out) {
  __shared__ float red[4][64];
  const int el = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const size_t i = static_cast<size_t>(blockIdx.x) * 64 + el;
  float s = 0.f;
  if (i < size) {
#pragma unroll 4
    for (int c = grp; c < chunks; c += 4) s += part[c * size + i];
  }
  red[grp][el] = s;
  __syncthreads();
  if (grp == 0 && i < size) out[i] = ((red[0][el] + red[1][el]) + red[2][el]) + red[3][el];
}

// Column sums of a [T, ld] matrix in two fixed-order stages.  Stage 1: block b
// sums rows [b*rows_per_block, ...) of every column (4 row lanes x 64 column
// lanes) into part[b][ld].  Stage 2: one block adds the partials in block order;
// column c goes to dstA[c] if c < nA, else to dstB[c - nA].
__global__ __launch_bounds__(kBlock) void colsum_stage1_kernel(const float *__restrict__ src,
                                                               int64_t T, int ld,
                                                               int64_t rows_per_block,
                                                               float *__restrict__ part) {
  __shared__ float red[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rows_per_block;
  int64_t r1 = r0 + rows_per_block;
  if (r1 > T) r1 = T;
  for (int c0 = 0; c0 < ld; c0 += 64) {
    const int c = c0 + cl;
    float s = 0.f;
    if (c < ld)
      for (int64_t t = r0 + rl; t < r1; t += 4) s += src[t * ld + c];
    __syncthreads();
    red[rl][cl] = s;
    __syncthreads();
    if (rl == 0 && c < ld)
      part[static_cast<size_t>(blockIdx.x) * ld + c] = ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
  }
}

__global__ __launch_bounds__(kBlock) void colsum_stage2_kernel(const float *__restrict__ part,
                                                               int nblocks, int ld, int nA,
                                                               float *__restrict__ dstA,
                                                               float *__restrict__ dstB) {
  __shared__ float red[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  for (int c0 = 0; c0 < ld; c0 += 64) {
    const int c = c0 + cl;
    float s = 0.f;
    if (c < ld) {
#pragma unroll 8
      for (int b = rl; b < nblocks; b += 4) s += part[static_cast<size_t>(b) * ld + c];
    }
    __syncthreads();
    red[rl][cl] = s;
    __syncthreads();
    if (rl == 0 && c < ld) {
      const float v = ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
      if (c < nA) dstA[c] = v;
      else dstB[c - nA] = v;
    }
  }
}

// The end of the fused backward in one launch.  Blocks [0, nbW): g_W = sum over the token
// chunks' partial sums (as sum_partials_kernel).  Block nbW + c: column c of the
// [rows, ld] matrix of per-64-token g_z sums, added in a fixed order (thread i takes rows
// i, i + 256, ... in turn, then a pairwise tree over the threads); columns below nA go to
// dstA (g_b), the others to dstB (g_alpha).
__global__ __launch_bounds__(kBlock) void bwd_finish_kernel(const float *__restrict__ part,
                                                            size_t size, int chunks, int nbW,
                                                            float *__restrict__ out,
                                                            const float *__restrict__ src,
                                                            int64_t rows, int ld, int nA,
                                                            float *__restrict__ dstA,
                                                            float *__restrict__ dstB) {
  __shared__ float red[kBlock];
  if (static_cast<int>(blockIdx.x) < nbW) {
    const int el = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const size_t i = static_cast<size_t>(blockIdx.x) * 64 + el;
    float s = 0.f;
    if (i < size) {
#pragma unroll 4
      for (int c = grp; c < chunks; c += 4) s += part[c * size + i];
    }
    red[grp * 64 + el] = s;
    __syncthreads();
    if (grp == 0 && i < size) out[i] = ((red[el] + red[64 + el]) + red[128 + el]) + red[192 + el];
    return;
  }
  const int c = static_cast<int>(blockIdx.x) - nbW;
  float s = 0.f;
#pragma unroll 4
  for (int64_t r = threadIdx.x; r < rows; r += kBlock) s += src[r * ld + c];
  red[threadIdx.x] = s;
  __syncthreads();
#pragma unroll
  for (int w = kBlock / 2; w > 0; w >>= 1) {
    if (static_cast<int>(threadIdx.x) < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (c < nA) dstA[c] = red[0];
    else dstB[c - nA] = red[0];
  }
}

__global__ __launch_bounds__(kBlock) void fill_zero_kernel(float *__restrict__ p, size_t count) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (i < count) p[i] = 0.f;
}

// 16 bytes per thread and iteration, grid-stride
__global__ __launch_bounds__(kBlock) void copy_kernel(uint4 *__restrict__ dst,
                                                      const uint4 *__restrict__ src, size_t n16) {
  for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x; i < n16;
       i += static_cast<size_t>(gridDim.x) * kBlock)
    dst[i] = src[i];
}

inline unsigned blocks_for(int64_t items, int per) {
  return static_cast<unsigned>((items + per - 1) / per);
}

}  // namespace

// ================================================================ launchers
hipError_t launch_proj_generic(const mhcl_desc &d, int M, const void *x, const float *W,
                               float *u_raw, float *sumsq, hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    using IO = decltype(io);
    hipLaunchKernelGGL(proj_generic_kernel<IO>, dim3(blocks_for(d.T, kTok)), dim3(kBlock), 0, s, x,
                       W, d.n * d.C, M, d.T, u_raw, sumsq);
    return hipGetLastError();
  });
}

hipError_t launch_coeffs_epilogue(const mhcl_desc &d, int parts, const float *u_raw,
                                  const float *sumsq, const float *b, const float *alpha, float *H_res, float *H_pre,
                                  float *H_post, hipStream_t s) {
  return dispatch_n5(d.n, [&](auto nn) {
    return dispatch_mode(d.res_mode, [&](auto mm) {
      constexpr int N = decltype(nn)::value, MODE = decltype(mm)::value;
      constexpr int M = Dims<N, MODE>::M;
      if constexpr (M % 4 == 0 && M <= 32) {
        if (parts >= 8) {
          hipLaunchKernelGGL((coeffs_epilogue_sliced_kernel<N, MODE>), dim3(blocks_for(d.T, 64)),
                             dim3(512), 0, s, u_raw, sumsq, parts, b, alpha, d.n * d.C, d.eps,
                             d.sk_iters, d.T, H_res, H_pre, H_post);
          return hipGetLastError();
        }
      }
      hipLaunchKernelGGL((coeffs_epilogue_kernel<N, MODE>), dim3(blocks_for(d.T, 128)), dim3(128),
                         0, s, u_raw, sumsq, parts, b, alpha, d.n * d.C, d.eps, d.sk_iters, d.T,
                         H_res, H_pre, H_post);
      return hipGetLastError();
    });
  });
}

hipError_t launch_coeffs_bwd_epilogue(const mhcl_desc &d, int parts, const float *u_raw,
                                      const float *sumsq,
                                      const float *b, const float *alpha, const float *g_H_res,
                                      const float *g_H_pre, const float *g_H_post,
                                      const BwdTokenBufs &o, hipStream_t s) {
  return dispatch_n5(d.n, [&](auto nn) {
    return dispatch_mode(d.res_mode, [&](auto mm) {
      constexpr int N = decltype(nn)::value, MODE = decltype(mm)::value;
      hipLaunchKernelGGL((coeffs_bwd_epilogue_kernel<N, MODE>), dim3(blocks_for(d.T, 128)),
                         dim3(128), 0, s, u_raw, sumsq, parts, b, alpha, g_H_res, g_H_pre,
                         g_H_post, d.n * d.C, d.eps, d.sk_iters, d.T, o);
      return hipGetLastError();
    });
  });
}

hipError_t launch_pre(const mhcl_desc &d, const void *x, const float *H_pre, void *h, hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    return dispatch_n(d.n, [&](auto nn) {
      using IO = decltype(io);
      constexpr int N = decltype(nn)::value;
      hipLaunchKernelGGL((pre_kernel<IO, N>), dim3(blocks_for(d.T * (d.C / IO::kVec), kBlock)),
                         dim3(kBlock), 0, s, x, H_pre, h, d.C, d.T);
      return hipGetLastError();
    });
  });
}

hipError_t launch_post(const mhcl_desc &d, const void *x, const void *y, const float *H_res,
                       const float *H_post, void *x_out, hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    return dispatch_n(d.n, [&](auto nn) {
      using IO = decltype(io);
      constexpr int N = decltype(nn)::value;
      hipLaunchKernelGGL((post_kernel<IO, N>), dim3(blocks_for(d.T * (d.C / IO::kVec), kBlock)),
                         dim3(kBlock), 0, s, x, y, H_res, H_post, x_out, d.C, d.T);
      return hipGetLastError();
    });
  });
}

hipError_t launch_post_bwd(const mhcl_desc &d, const void *x, const void *y, const float *H_res,
                           const float *H_post, const void *g_xout, void *g_x, void *g_y,
                           float *g_H_res, float *g_H_post, hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    return dispatch_n(d.n, [&](auto nn) {
      using IO = decltype(io);
      constexpr int N = decltype(nn)::value;
      hipLaunchKernelGGL((post_bwd_kernel<IO, N>), dim3(static_cast<unsigned>(d.T)), dim3(kBlock),
                         0, s, x, y, H_res, H_post, g_xout, g_x, g_y, g_H_res, g_H_post, d.C);
      return hipGetLastError();
    });
  });
}

hipError_t launch_pre_bwd(const mhcl_desc &d, const void *x, const float *H_pre, const void *g_h,
                          void *g_x, float *g_H_pre, hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    return dispatch_n(d.n, [&](auto nn) {
      using IO = decltype(io);
      constexpr int N = decltype(nn)::value;
      hipLaunchKernelGGL((pre_bwd_kernel<IO, N>), dim3(static_cast<unsigned>(d.T)), dim3(kBlock), 0,
                         s, x, H_pre, g_h, g_x, g_H_pre, d.C);
      return hipGetLastError();
    });
  });
}

hipError_t launch_bwd_dots(const mhcl_desc &d, const void *x, const void *y, const void *g_xout,
                           const void *g_h, float *g_H_res, float *g_H_post, float *g_H_pre,
                           hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    return dispatch_n(d.n, [&](auto nn) {
      using IO = decltype(io);
      constexpr int N = decltype(nn)::value;
      hipLaunchKernelGGL((bwd_dots_kernel<IO, N>), dim3(static_cast<unsigned>(d.T)), dim3(kBlock),
                         0, s, x, y, g_xout, g_h, g_H_res, g_H_post, g_H_pre, d.C);
      return hipGetLastError();
    });
  });
}

hipError_t launch_gx_generic(const mhcl_desc &d, int M, bool fused, const void *x, const float *W,
                             const void *g_xout, const void *g_h, const BwdTokenBufs &o, void *g_x,
                             void *g_y, hipStream_t s) {
  return dispatch_io(d.io_dtype, [&](auto io) {
    return dispatch_n(d.n, [&](auto nn) {
      using IO = decltype(io);
      constexpr int N = decltype(nn)::value;
      // grid.y carries the token index: at most 65535 per launch
      const unsigned gx = blocks_for(d.C / IO::kVec, kBlock);
      for (int64_t t0 = 0; t0 < d.T; t0 += 65535) {
        const unsigned gy = static_cast<unsigned>(d.T - t0 < 65535 ? d.T - t0 : 65535);
        BwdTokenBufs oo = o;
        oo.H_res += t0 * N * N; oo.H_pre += t0 * N; oo.H_post += t0 * N;
        oo.vr += t0 * M; oo.coefx += t0;
        const size_t so = static_cast<size_t>(t0) * N * d.C * IO::kBytes;
        const size_t ro = static_cast<size_t>(t0) * d.C * IO::kBytes;
        const char *xo = static_cast<const char *>(x) + so;
        const char *go = g_xout ? static_cast<const char *>(g_xout) + so : nullptr;
        const char *gh = g_h ? static_cast<const char *>(g_h) + ro : nullptr;
        char *gxo = static_cast<char *>(g_x) + so;
        char *gyo = g_y ? static_cast<char *>(g_y) + ro : nullptr;
        if (fused)
          hipLaunchKernelGGL((gx_generic_kernel<IO, N, true>), dim3(gx, gy), dim3(kBlock), 0, s,
                             (const void *)xo, W, (const void *)go, (const void *)gh, oo, M, d.C,
                             (void *)gxo, (void *)gyo);
        else
          hipLaunchKernelGGL((gx_generic_kernel<IO, N, false>), dim3(gx, gy), dim3(kBlock), 0, s,
                             (const void *)xo, W, (const void *)go, (const void *)gh, oo, M, d.C,
                             (void *)gxo, (void *)gyo);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    });
  });
}

int gw_chunks_generic(const mhcl_desc &d) {
  int64_t c = (d.T + 1023) / 1024;
  if (c < 1) c = 1;
  if (c > 32) c = 32;
  return static_cast<int>(c);
}

hipError_t launch_gw_generic(const mhcl_desc &d, int M, const void *x, const float *vr,
                             float *partials, float *g_W, hipStream_t s) {
  const int chunks = gw_chunks_generic(d);
  const int nC = d.n * d.C;
  const int64_t chunk = (d.T + chunks - 1) / chunks;
  return dispatch_io(d.io_dtype, [&](auto io) {
    using IO = decltype(io);
    float *dst = chunks == 1 ? g_W : partials;
    hipLaunchKernelGGL(gw_generic_kernel<IO>, dim3(blocks_for(nC, 8), chunks), dim3(kBlock), 0, s,
                       x, vr, nC, M, d.T, chunk, dst);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || chunks == 1) return e;
    const size_t size = static_cast<size_t>(nC) * M;
    hipLaunchKernelGGL(sum_partials_kernel, dim3(blocks_for(size, 64)), dim3(kBlock), 0, s,
                       (const float *)partials, size, chunks, g_W);
    return hipGetLastError();
  });
}

hipError_t launch_bwd_finish(const float *partials, size_t size, int chunks, float *g_W,
                             const float *gz_rows, int64_t rows, int M, float *g_b, float *g_alpha,
                             hipStream_t s) {
  const int nbW = chunks > 1 ? static_cast<int>(blocks_for(size, 64)) : 0;
  hipLaunchKernelGGL(bwd_finish_kernel, dim3(nbW + M + 3), dim3(kBlock), 0, s, partials, size, chunks,
                     nbW, g_W, gz_rows, rows, M + 3, M, g_b, g_alpha);
  return hipGetLastError();
}

hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + kBlock - 1) / kBlock;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s,
                     static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), n16);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float *p, size_t count, hipStream_t s) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for(count, kBlock)), dim3(kBlock), 0, s, p, count);
  return hipGetLastError();
}

hipError_t launch_param_sums_rows(int64_t rows, int M, const float *src, float *g_b,
                                  float *g_alpha, float *part, hipStream_t s) {
  const int ld = M + 3;
  int64_t nb = (rows + 15) / 16;     // short per-thread chains; stage 2 adds at most 256 rows
  if (nb > 256) nb = 256;
  if (nb < 1) nb = 1;
  const int nblocks = static_cast<int>(nb);
  const int64_t rpb = (rows + nblocks - 1) / nblocks;
  hipLaunchKernelGGL(colsum_stage1_kernel, dim3(nblocks), dim3(kBlock), 0, s, src, rows, ld, rpb,
                     part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_stage2_kernel, dim3(1), dim3(kBlock), 0, s, (const float *)part,
                     nblocks, ld, M, g_b, g_alpha);
  return hipGetLastError();
}

hipError_t launch_param_sums(const mhcl_desc &d, int M, const float *gz, float *g_b, float *g_alpha,
                             float *part, hipStream_t s) {
  return launch_param_sums_rows(d.T, M, gz, g_b, g_alpha, part, s);
}

// upper bound of the stage-1 block count of launch_param_sums_rows for any rows <= T
int param_sum_blocks(const mhcl_desc &d) {
  int64_t b = (d.T + 15) / 16;
  if (b > 256) b = 256;
  if (b < 1) b = 1;
  return static_cast<int>(b);
}

}  // namespace mhcl
