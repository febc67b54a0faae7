// Diagnostics kernels of libmhcl: the logits of a layer with the relative
// range of the Sinkhorn-Knopp input (Sec. 3.1, Eq. 3), and column sums / l1
// errors of single residual matrices and of their product over the layers
// (Sec. 3.1, footnote 1; Sec. 4.3).  Per-token work on a few floats: one
// thread per token, plain fp32.
#include "mhcl_common.h"
#include "mhcl_internal.h"

namespace mhcl {

namespace {

// z[t][m] = alpha_g (r u_raw[t][m]) + b[m], the same expression the coefficient
// kernels evaluate; spread[t] = max - min of the residual logits, which is
// log(1/nu) of exp(z_res) (every entry of exp(.) is positive).
__global__ __launch_bounds__(128) void logits_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha, int nC, float eps, int64_t T,
    int M, int R, int n, float *__restrict__ z, float *__restrict__ spread) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 128 + threadIdx.x;
  if (t >= T) return;
  float ssq = sumsq[t];
  for (int pt = 1; pt < parts; ++pt) ssq += sumsq[pt * T + t];
  const float r = 1.f / sqrtf(ssq / static_cast<float>(nC) + eps);
  const float a0 = alpha[0], a1 = alpha[1], a2 = alpha[2];
  float zmax = -INFINITY, zmin = INFINITY;
  for (int m = 0; m < M; ++m) {
    float u = u_raw[t * M + m];
    for (int pt = 1; pt < parts; ++pt) u += u_raw[(pt * T + t) * M + m];
    const float al = m < R ? a0 : (m < R + n ? a1 : a2);
    const float v = al * (r * u) + b[m];
    if (z) z[t * M + m] = v;
    if (m < R) { zmax = fmaxf(zmax, v); zmin = fminf(zmin, v); }
  }
  if (spread) spread[t] = zmax - zmin;
}

template <int N>
__device__ __forceinline__ float l1_error(const float (&Q)[N * N], float (&cs)[N]) {
  float e = 0.f;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < N; ++j) s += Q[i * N + j];
    e += fabsf(s - 1.f);
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) s += Q[i * N + j];
    cs[j] = s;
    e += fabsf(s - 1.f);
  }
  return e;
}

// Q_l = H_l Q_{l-1}, Q_0 = I: later layers multiply on the left, the order in
// which Eq. 1 applies them.
template <int N>
__global__ __launch_bounds__(128) void ds_chain_kernel(
    const float *__restrict__ H, int L, int64_t T, float *__restrict__ colsum,
    float *__restrict__ l1, float *__restrict__ prod, float *__restrict__ prod_colsum,
    float *__restrict__ prod_l1) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 128 + threadIdx.x;
  if (t >= T) return;
  float Q[N * N], Hl[N * N], Qn[N * N], cs[N];
#pragma unroll
  for (int e = 0; e < N * N; ++e) Q[e] = (e / N == e % N) ? 1.f : 0.f;
  for (int l = 0; l < L; ++l) {
    const int64_t lt = static_cast<int64_t>(l) * T + t;
#pragma unroll
    for (int e = 0; e < N * N; ++e) Hl[e] = H[lt * N * N + e];
    const float e1 = l1_error<N>(Hl, cs);
    if (l1) l1[lt] = e1;
    if (colsum) {
#pragma unroll
      for (int j = 0; j < N; ++j) colsum[lt * N + j] = cs[j];
    }
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
      for (int j = 0; j < N; ++j) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < N; ++k) s += Hl[i * N + k] * Q[k * N + j];
        Qn[i * N + j] = s;
      }
#pragma unroll
    for (int e = 0; e < N * N; ++e) Q[e] = Qn[e];
    const float e2 = l1_error<N>(Q, cs);
    if (prod_l1) prod_l1[lt] = e2;
    if (prod_colsum) {
#pragma unroll
      for (int j = 0; j < N; ++j) prod_colsum[lt * N + j] = cs[j];
    }
  }
  if (prod) {
#pragma unroll
    for (int e = 0; e < N * N; ++e) prod[t * N * N + e] = Q[e];
  }
}

inline unsigned blocks128(int64_t items) { return static_cast<unsigned>((items + 127) / 128); }

}  // namespace

hipError_t launch_logits(const mhcl_desc &d, int M, int parts, const float *u_raw,
                         const float *sumsq, const float *b, const float *alpha, float *z,
                         float *spread, hipStream_t s) {
  hipLaunchKernelGGL(logits_kernel, dim3(blocks128(d.T)), dim3(128), 0, s, u_raw, sumsq, parts, b,
                     alpha, d.n * d.C, d.eps, d.T, M, M - 2 * d.n, d.n, z, spread);
  return hipGetLastError();
}

hipError_t launch_ds_chain(int n, int L, int64_t T, const float *H, float *colsum, float *l1,
                           float *prod, float *prod_colsum, float *prod_l1, hipStream_t s) {
  auto go = [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    hipLaunchKernelGGL(ds_chain_kernel<N>, dim3(blocks128(T)), dim3(128), 0, s, H, L, T, colsum,
                       l1, prod, prod_colsum, prod_l1);
    return hipGetLastError();
  };
  switch (n) {
    case 1: return go(std::integral_constant<int, 1>{});
    case 2: return go(std::integral_constant<int, 2>{});
    case 3: return go(std::integral_constant<int, 3>{});
    case 4: return go(std::integral_constant<int, 4>{});
    case 5: return go(std::integral_constant<int, 5>{});
    case 6: return go(std::integral_constant<int, 6>{});
    case 7: return go(std::integral_constant<int, 7>{});
    case 8: return go(std::integral_constant<int, 8>{});
  }
  return hipErrorInvalidValue;
}

}  // namespace mhcl
