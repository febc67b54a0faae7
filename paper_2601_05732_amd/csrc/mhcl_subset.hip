// Per-token coefficients of the permutation-subset form (Sec. 5, the paragraph
// on larger n): a = softmax over K logits, H_res = sum_k a_k P_k over the K
// permutations of a run-time table (device memory, [K][n]); gates as in
// Sec. 3.2.  n up to 8, K up to 128.  One token per thread; the K weights of
// each thread sit in LDS (a register array indexed by a run-time k would go
// to scratch memory), the table is staged in LDS once per block.
#include "mhcl_common.h"
#include "mhcl_internal.h"

namespace mhcl {

namespace {

constexpr int kThreads = 64;

// Entries are clamped to 0..n-1 so that a malformed table cannot index outside
// the n x n arrays (the result is then simply not doubly stochastic).
__device__ __forceinline__ void stage_table(const int8_t *__restrict__ sigma, int count, int n,
                                            int8_t *dst) {
  for (int i = threadIdx.x; i < count; i += kThreads) {
    int v = sigma[i];
    v = v < 0 ? 0 : (v > n - 1 ? n - 1 : v);
    dst[i] = static_cast<int8_t>(v);
  }
  __syncthreads();
}

// logits of token t summed over the K-split slices, in slice order
__device__ __forceinline__ float raw_logit(const float *__restrict__ u_raw, int parts, int64_t T,
                                           int64_t t, int M, int m) {
  float u = u_raw[t * M + m];
  for (int pt = 1; pt < parts; ++pt) u += u_raw[(pt * T + t) * M + m];
  return u;
}

// softmax weights of the residual logits into a_s[k][thread]; returns r
template <int N>
__device__ __forceinline__ float subset_weights(const float *__restrict__ u_raw,
                                                const float *__restrict__ sumsq, int parts,
                                                const float *__restrict__ b, float alpha_res,
                                                int nC, float eps, int64_t T, int64_t t, int K,
                                                int M, float (*a_s)[kThreads]) {
  float ssq = sumsq[t];
  for (int pt = 1; pt < parts; ++pt) ssq += sumsq[pt * T + t];
  const float r = 1.f / sqrtf(ssq / static_cast<float>(nC) + eps);
  float zmax = -INFINITY;
  for (int k = 0; k < K; ++k) {
    const float z = alpha_res * (r * raw_logit(u_raw, parts, T, t, M, k)) + b[k];
    a_s[k][threadIdx.x] = z;
    zmax = fmaxf(zmax, z);
  }
  float sum = 0.f;
  for (int k = 0; k < K; ++k) {
    const float e = expf(a_s[k][threadIdx.x] - zmax);
    a_s[k][threadIdx.x] = e;
    sum += e;
  }
  for (int k = 0; k < K; ++k) a_s[k][threadIdx.x] = a_s[k][threadIdx.x] / sum;
  return r;
}

// H[i][j] = sum over the given permutations with sigma_k(i) = j of a_k
template <int N>
__device__ __forceinline__ void subset_mix(const float (*a_s)[kThreads], const int8_t *sig, int K,
                                           float (&H)[N * N]) {
#pragma unroll
  for (int e = 0; e < N * N; ++e) H[e] = 0.f;
  for (int k = 0; k < K; ++k) {
    const float w = a_s[k][threadIdx.x];
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int sj = sig[k * N + i];
#pragma unroll
      for (int j = 0; j < N; ++j) H[i * N + j] += (j == sj) ? w : 0.f;
    }
  }
}

template <int N>
__global__ __launch_bounds__(kThreads) void coeffs_subset_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha, int nC, float eps, int64_t T,
    int K, const int8_t *__restrict__ sigma, float *__restrict__ H_res, float *__restrict__ H_pre,
    float *__restrict__ H_post) {
  __shared__ float a_s[kMaxPerm][kThreads];
  __shared__ int8_t sig[kMaxPerm * N];
  stage_table(sigma, K * N, N, sig);
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= T) return;
  const int M = K + 2 * N;
  const float r = subset_weights<N>(u_raw, sumsq, parts, b, alpha[0], nC, eps, T, t, K, M, a_s);
  float H[N * N];
  subset_mix<N>(a_s, sig, K, H);
#pragma unroll
  for (int e = 0; e < N * N; ++e) H_res[t * N * N + e] = H[e];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const float zp = alpha[1] * (r * raw_logit(u_raw, parts, T, t, M, K + j)) + b[K + j];
    const float zq = alpha[2] * (r * raw_logit(u_raw, parts, T, t, M, K + N + j)) + b[K + N + j];
    H_pre[t * N + j] = sigmoidf(zp);
    H_post[t * N + j] = 2.f * sigmoidf(zq);
  }
}

// Backward: g_a[k] = sum_i g_H_res[i][sigma_k(i)], g_z_res = a (g_a - <a, g_a>),
// gates through the logistic function; then the operands of the projection's
// backward as in the other forms: vr = r alpha_g g_z, coefx, and gz | sums of
// g_z u per group.
template <int N>
__global__ __launch_bounds__(kThreads) void coeffs_bwd_subset_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha,
    const float *__restrict__ gH_res, const float *__restrict__ gH_pre,
    const float *__restrict__ gH_post, int nC, float eps, int64_t T, int K,
    const int8_t *__restrict__ sigma, BwdTokenBufs o) {
  __shared__ float a_s[kMaxPerm][kThreads];
  __shared__ float g_s[N * N][kThreads];
  __shared__ int8_t sig[kMaxPerm * N];
  stage_table(sigma, K * N, N, sig);
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= T) return;
  const int M = K + 2 * N;
  const float a0 = alpha[0], a1 = alpha[1], a2 = alpha[2];
  const float r = subset_weights<N>(u_raw, sumsq, parts, b, a0, nC, eps, T, t, K, M, a_s);
  float H[N * N];
  subset_mix<N>(a_s, sig, K, H);
#pragma unroll
  for (int e = 0; e < N * N; ++e) {
    o.H_res[t * N * N + e] = H[e];
    g_s[e][threadIdx.x] = gH_res[t * N * N + e];
  }
  auto g_a = [&](int k) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) s += g_s[i * N + sig[k * N + i]][threadIdx.x];
    return s;
  };
  float mean = 0.f;
  for (int k = 0; k < K; ++k) mean += a_s[k][threadIdx.x] * g_a(k);
  float ga[3] = {0.f, 0.f, 0.f}, dot = 0.f;
  float *gz = o.gz + t * (M + 3);
  float *vr = o.vr + t * M;
  for (int k = 0; k < K; ++k) {
    const float g = a_s[k][threadIdx.x] * (g_a(k) - mean);
    const float u = raw_logit(u_raw, parts, T, t, M, k);
    const float v = r * a0 * g;
    gz[k] = g;
    vr[k] = v;
    ga[0] += g * (r * u);
    dot += v * u;
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const float up = raw_logit(u_raw, parts, T, t, M, K + j);
    const float uq = raw_logit(u_raw, parts, T, t, M, K + N + j);
    const float hp = sigmoidf(a1 * (r * up) + b[K + j]);
    const float hq = 2.f * sigmoidf(a2 * (r * uq) + b[K + N + j]);
    o.H_pre[t * N + j] = hp;
    o.H_post[t * N + j] = hq;
    const float gp = gH_pre[t * N + j] * hp * (1.f - hp);
    const float gq = gH_post[t * N + j] * hq * (1.f - 0.5f * hq);
    gz[K + j] = gp;
    gz[K + N + j] = gq;
    const float vp = r * a1 * gp, vq = r * a2 * gq;
    vr[K + j] = vp;
    vr[K + N + j] = vq;
    ga[1] += gp * (r * up);
    ga[2] += gq * (r * uq);
    dot += vp * up + vq * uq;
  }
#pragma unroll
  for (int g = 0; g < 3; ++g) gz[M + g] = ga[g];
  o.coefx[t] = (r * r / static_cast<float>(nC)) * dot;
}

// The same backward stage for the MFMA kernels of the wide backward path: its
// results go out in the layouts those kernels read (see FastBwdWs):
//   cpk [T][CP] : H_res | H_pre | H_post | coefx
//   vr  [Tpad][MP32] bf16 hi, lo (row per token), vrT [Tpad/32][MP16][32] (tokens innermost)
//   gzs [Tpad/64][M+3] : sums over each 64 tokens of g_z and of the per-group g_z u
// One wave per block; lanes past T recompute the last token and contribute zeros.
__device__ __forceinline__ float wave_total(float v) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
  return v;
}

template <int N>
__global__ __launch_bounds__(kThreads) void bwd_epilogue_subset_fast_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha,
    const float *__restrict__ gH_res, const float *__restrict__ gH_pre,
    const float *__restrict__ gH_post, int nC, float eps, int64_t T, int K,
    const int8_t *__restrict__ sigma, int CP, int MP32, int MP16, float *__restrict__ cpk,
    uint16_t *__restrict__ vr_hi, uint16_t *__restrict__ vr_lo, uint16_t *__restrict__ vrT_hi,
    uint16_t *__restrict__ vrT_lo, float *__restrict__ gz_sums) {
  __shared__ float a_s[kMaxPerm][kThreads];
  __shared__ float g_s[N * N][kThreads];
  __shared__ int8_t sig[kMaxPerm * N];
  stage_table(sigma, K * N, N, sig);
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;   // < Tpad
  const bool live = t < T;
  const int64_t tl = live ? t : T - 1;
  const int64_t blk = t >> 5;
  const int tin = static_cast<int>(t & 31);
  const int M = K + 2 * N;
  const float a0 = alpha[0], a1 = alpha[1], a2 = alpha[2];
  const float r = subset_weights<N>(u_raw, sumsq, parts, b, a0, nC, eps, T, tl, K, M, a_s);
  float H[N * N];
  subset_mix<N>(a_s, sig, K, H);
#pragma unroll
  for (int e = 0; e < N * N; ++e) {
    if (live) cpk[t * CP + e] = H[e];
    g_s[e][threadIdx.x] = gH_res[tl * N * N + e];
  }
  auto g_a = [&](int k) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) s += g_s[i * N + sig[k * N + i]][threadIdx.x];
    return s;
  };
  auto emit = [&](int m, float g, float al, float u, float &dot, float &ga) {
    // g_z of logit m -> vr (both layouts), running sums, and the 64-token total of g_z
    if (!live) g = 0.f;
    const float v = r * al * g;
    ga += g * (r * u);
    dot += v * u;
    uint16_t hi = f32_to_bf16(v);
    uint16_t lo = f32_to_bf16(v - bf16_to_f32(hi));
    vr_hi[t * MP32 + m] = hi;
    vr_lo[t * MP32 + m] = lo;
    vrT_hi[(blk * MP16 + m) * 32 + tin] = hi;
    vrT_lo[(blk * MP16 + m) * 32 + tin] = lo;
    const float tot = wave_total(g);
    if (threadIdx.x == 0) gz_sums[static_cast<int64_t>(blockIdx.x) * (M + 3) + m] = tot;
  };
  float mean = 0.f;
  for (int k = 0; k < K; ++k) mean += a_s[k][threadIdx.x] * g_a(k);
  float ga[3] = {0.f, 0.f, 0.f}, dot = 0.f;
  for (int k = 0; k < K; ++k)
    emit(k, a_s[k][threadIdx.x] * (g_a(k) - mean), a0, raw_logit(u_raw, parts, T, tl, M, k), dot, ga[0]);
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const float up = raw_logit(u_raw, parts, T, tl, M, K + j);
    const float hp = sigmoidf(a1 * (r * up) + b[K + j]);
    if (live) cpk[t * CP + N * N + j] = hp;
    emit(K + j, gH_pre[tl * N + j] * hp * (1.f - hp), a1, up, dot, ga[1]);
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const float uq = raw_logit(u_raw, parts, T, tl, M, K + N + j);
    const float hq = 2.f * sigmoidf(a2 * (r * uq) + b[K + N + j]);
    if (live) cpk[t * CP + N * N + N + j] = hq;
    emit(K + N + j, gH_post[tl * N + j] * hq * (1.f - 0.5f * hq), a2, uq, dot, ga[2]);
  }
  for (int m = M; m < MP32; ++m) { vr_hi[t * MP32 + m] = 0; vr_lo[t * MP32 + m] = 0; }
  for (int m = M; m < MP16; ++m) {
    vrT_hi[(blk * MP16 + m) * 32 + tin] = 0;
    vrT_lo[(blk * MP16 + m) * 32 + tin] = 0;
  }
#pragma unroll
  for (int g = 0; g < 3; ++g) {
    const float tot = wave_total(ga[g]);
    if (threadIdx.x == 0) gz_sums[static_cast<int64_t>(blockIdx.x) * (M + 3) + M + g] = tot;
  }
  if (live) cpk[t * CP + N * N + 2 * N] = (r * r / static_cast<float>(nC)) * dot;
}

template <typename F>
hipError_t dispatch_n8(int n, F &&f) {
  switch (n) {
    case 1: return f(std::integral_constant<int, 1>{});
    case 2: return f(std::integral_constant<int, 2>{});
    case 3: return f(std::integral_constant<int, 3>{});
    case 4: return f(std::integral_constant<int, 4>{});
    case 5: return f(std::integral_constant<int, 5>{});
    case 6: return f(std::integral_constant<int, 6>{});
    case 7: return f(std::integral_constant<int, 7>{});
    case 8: return f(std::integral_constant<int, 8>{});
  }
  return hipErrorInvalidValue;
}

inline unsigned blocks_of(int64_t T) { return static_cast<unsigned>((T + kThreads - 1) / kThreads); }

}  // namespace

hipError_t launch_coeffs_subset(const mhcl_desc &d, int parts, const float *u_raw,
                                const float *sumsq, const float *b, const float *alpha,
                                float *H_res, float *H_pre, float *H_post, hipStream_t s) {
  if (d.n_perm < 1 || d.n_perm > kMaxPerm || !d.perm) return hipErrorInvalidValue;
  return dispatch_n8(d.n, [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    hipLaunchKernelGGL(coeffs_subset_kernel<N>, dim3(blocks_of(d.T)), dim3(kThreads), 0, s, u_raw,
                       sumsq, parts, b, alpha, d.n * d.C, d.eps, d.T, d.n_perm, d.perm, H_res,
                       H_pre, H_post);
    return hipGetLastError();
  });
}

hipError_t launch_coeffs_bwd_subset(const mhcl_desc &d, int parts, const float *u_raw,
                                    const float *sumsq, const float *b, const float *alpha,
                                    const float *g_H_res, const float *g_H_pre,
                                    const float *g_H_post, const BwdTokenBufs &o, hipStream_t s) {
  if (d.n_perm < 1 || d.n_perm > kMaxPerm || !d.perm) return hipErrorInvalidValue;
  return dispatch_n8(d.n, [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    hipLaunchKernelGGL(coeffs_bwd_subset_kernel<N>, dim3(blocks_of(d.T)), dim3(kThreads), 0, s,
                       u_raw, sumsq, parts, b, alpha, g_H_res, g_H_pre, g_H_post, d.n * d.C, d.eps,
                       d.T, d.n_perm, d.perm, o);
    return hipGetLastError();
  });
}

hipError_t launch_bwd_epilogue_subset_fast(const mhcl_desc &d, const float *b, const float *alpha,
                                           const FastBwdWs &w, hipStream_t s) {
  if (d.n_perm < 1 || d.n_perm > kMaxPerm || !d.perm) return hipErrorInvalidValue;
  const int64_t Tpad = (d.T + 63) / 64 * 64;
  return dispatch_n8(d.n, [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    hipLaunchKernelGGL(bwd_epilogue_subset_fast_kernel<N>, dim3(static_cast<unsigned>(Tpad / 64)),
                       dim3(kThreads), 0, s, w.u_raw, w.sumsq, w.parts, b, alpha, w.gH_res,
                       w.gH_pre, w.gH_post, d.n * d.C, d.eps, d.T, d.n_perm, d.perm, w.CP, w.MP32,
                       w.MP16, w.cpk, w.vr_hi, w.vr_lo, w.vrT_hi, w.vrT_lo, w.gz);
    return hipGetLastError();
  });
}

}  // namespace mhcl
