// Shared device-side building blocks of libmhcl (gfx950 only).
//
//  * stream element traits (bf16 / f32) and 16-byte vector access
//  * the permutation table of Theorem 3.1, generated at compile time
//  * the per-token coefficient math of Sec. 3.2 (Eqs. 4-5) and Sec. 2 (Eq. 2),
//    forward and backward, on register arrays
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <utility>

#include "../../include/mhcl.h"

namespace mhcl {

constexpr int kMaxN = 5;          // full permutation form and Sinkhorn-Knopp form
constexpr int kMaxNSubset = 8;    // permutation-subset form
constexpr int kMaxPerm = 128;     // permutations in a subset
constexpr int kMaxSkIters = 32;

// ------------------------------------------------------------------ bf16
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ float bf16lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

// A 16-byte chunk of a stream tensor held as fp32 lanes.
struct BF16 {
  static constexpr int kVec = 8;      // elements per 16 bytes
  static constexpr int kBytes = 2;
  __device__ static __forceinline__ void load(const void *p, size_t elem, float (&v)[8]) {
    const uint4 q = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(p) + elem);
    v[0] = bf16lo(q.x); v[1] = bf16hi(q.x); v[2] = bf16lo(q.y); v[3] = bf16hi(q.y);
    v[4] = bf16lo(q.z); v[5] = bf16hi(q.z); v[6] = bf16lo(q.w); v[7] = bf16hi(q.w);
  }
  __device__ static __forceinline__ void store(void *p, size_t elem, const float (&v)[8]) {
    uint4 q;
    q.x = pack_bf16x2(v[0], v[1]); q.y = pack_bf16x2(v[2], v[3]);
    q.z = pack_bf16x2(v[4], v[5]); q.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(p) + elem) = q;
  }
  __device__ static __forceinline__ float load1(const void *p, size_t elem) {
    return bf16_to_f32(static_cast<const uint16_t *>(p)[elem]);
  }
};
struct F32 {
  static constexpr int kVec = 4;
  static constexpr int kBytes = 4;
  __device__ static __forceinline__ void load(const void *p, size_t elem, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4 *>(static_cast<const float *>(p) + elem);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  }
  __device__ static __forceinline__ void store(void *p, size_t elem, const float (&v)[4]) {
    *reinterpret_cast<float4 *>(static_cast<float *>(p) + elem) = make_float4(v[0], v[1], v[2], v[3]);
  }
  __device__ static __forceinline__ float load1(const void *p, size_t elem) {
    return static_cast<const float *>(p)[elem];
  }
};

// ------------------------------------------------- permutation table
constexpr int factorial(int n) { return n <= 1 ? 1 : n * factorial(n - 1); }

template <int N>
struct PermTab {
  signed char s[factorial(N)][N];
};

// k-th permutation in lexicographic order by unranking k in the factorial
// number system: digit i selects the d-th smallest value not yet used.
template <int N>
constexpr PermTab<N> make_perm_tab() {
  PermTab<N> t{};
  for (int k = 0; k < factorial(N); ++k) {
    bool used[N] = {};
    int rem = k;
    for (int i = 0; i < N; ++i) {
      const int f = factorial(N - 1 - i);
      const int d = rem / f;
      rem %= f;
      int seen = 0;
      for (int j = 0; j < N; ++j) {
        if (used[j]) continue;
        if (seen == d) { t.s[k][i] = static_cast<signed char>(j); used[j] = true; break; }
        ++seen;
      }
    }
  }
  return t;
}

template <int N>
struct Perm {
  static constexpr PermTab<N> tab = make_perm_tab<N>();
};
// sigma_K(I) as a compile-time constant
template <int N, int K, int I>
inline constexpr int kSigma = Perm<N>::tab.s[K][I];

template <int N, int I, int J, int... K>
__device__ __forceinline__ float perm_cell_sum(const float *a, std::integer_sequence<int, K...>) {
  float s = 0.f;
  ((kSigma<N, K, I> == J ? (void)(s += a[K]) : (void)0), ...);
  return s;
}
// H[i][j] = sum over the (n-1)! permutations with sigma_k(i) = j of a_k   (Eq. 5)
template <int N, int... IJ>
__device__ __forceinline__ void perm_mix(const float *a, float *H, std::integer_sequence<int, IJ...>) {
  ((H[IJ] = perm_cell_sum<N, IJ / N, IJ % N>(a, std::make_integer_sequence<int, factorial(N)>{})), ...);
}
template <int N, int K, int... I>
__device__ __forceinline__ float perm_gather(const float *gH, std::integer_sequence<int, I...>) {
  return (gH[I * N + kSigma<N, K, I>] + ...);
}
// g_a[k] = <g_H, P_k> = sum_i g_H[i][sigma_k(i)]
template <int N, int... K>
__device__ __forceinline__ void perm_mix_bwd(const float *gH, float *ga, std::integer_sequence<int, K...>) {
  ((ga[K] = perm_gather<N, K>(gH, std::make_integer_sequence<int, N>{})), ...);
}

// ------------------------------------------------- per-token coefficients
template <int N, int MODE>
struct Dims {
  static constexpr int R = (MODE == MHCL_RES_LITE) ? factorial(N) : N * N;   // residual logits
  static constexpr int M = R + 2 * N;                                         // all logits
};

__device__ __forceinline__ float sigmoidf(float t) { return 1.f / (1.f + expf(-t)); }

struct TokenParams {
  float alpha_res, alpha_pre, alpha_post, eps;
  int sk_iters;
};

// Forward coefficients of one token from the raw projection u_raw = x_hat W
// (not yet normalised) and sum(x_hat^2).  RMSNorm's scale r commutes with the
// projection, so z = alpha (r u_raw) + b.
//   H_res [N*N], H_pre [N], H_post [N]; a [R] (lite: softmax weights; SK:
//   exp(z - max), the SK input); returns r.
// If sums != nullptr (SK mode) it receives the 2*sk_iters*N divisors.
template <int N, int MODE>
__device__ __forceinline__ float token_coeffs(const float *u_raw, float sumsq, int nC,
                                              const float *b, const TokenParams &p, float *H_res,
                                              float *H_pre, float *H_post, float *a,
                                              float *sums = nullptr) {
  constexpr int R = Dims<N, MODE>::R;
  const float r = 1.f / sqrtf(sumsq / static_cast<float>(nC) + p.eps);
  float zmax = -INFINITY;
#pragma unroll
  for (int k = 0; k < R; ++k) {
    a[k] = p.alpha_res * (r * u_raw[k]) + b[k];
    zmax = fmaxf(zmax, a[k]);
  }
  if constexpr (MODE == MHCL_RES_LITE) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < R; ++k) { a[k] = expf(a[k] - zmax); s += a[k]; }
#pragma unroll
    for (int k = 0; k < R; ++k) a[k] = a[k] / s;
    perm_mix<N>(a, H_res, std::make_integer_sequence<int, N * N>{});
  } else {
    // SK is invariant to a global scale of its input after the first
    // normalisation, so exp(z - max) replaces exp(z).
#pragma unroll
    for (int k = 0; k < R; ++k) { a[k] = expf(a[k] - zmax); H_res[k] = a[k]; }
    for (int it = 0; it < p.sk_iters; ++it) {
#pragma unroll
      for (int j = 0; j < N; ++j) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < N; ++i) s += H_res[i * N + j];
        const float inv = 1.f / s;   // one division per line; the entries are scaled by its result
#pragma unroll
        for (int i = 0; i < N; ++i) H_res[i * N + j] = H_res[i * N + j] * inv;
        if (sums) sums[(2 * it) * N + j] = s;
      }
#pragma unroll
      for (int i = 0; i < N; ++i) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < N; ++j) s += H_res[i * N + j];
        const float inv = 1.f / s;
#pragma unroll
        for (int j = 0; j < N; ++j) H_res[i * N + j] = H_res[i * N + j] * inv;
        if (sums) sums[(2 * it + 1) * N + i] = s;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    H_pre[j] = sigmoidf(p.alpha_pre * (r * u_raw[R + j]) + b[R + j]);
    H_post[j] = 2.f * sigmoidf(p.alpha_post * (r * u_raw[R + N + j]) + b[R + N + j]);
  }
  return r;
}

// Backward of token_coeffs: from g_H_res, g_H_pre, g_H_post and the forward
// values produce g_z [M], the gradient on the logits z = alpha_g u + b.
//   lite: g_a[k] = <g_H_res, P_k>, g_z_res = a (g_a - <a, g_a>)
//   SK  : walk the 2*sk_iters normalisations in reverse; for Y = X / s,
//         g_X = (g_Y - sum_axis(g_Y Y)) / s, and X = Y s rebuilds the
//         previous iterate from the stored divisors; then g_z = g_X0 X0.
// H_res is clobbered in SK mode.
template <int N, int MODE>
__device__ __forceinline__ void token_coeffs_bwd(const float *gH_res, const float *gH_pre,
                                                 const float *gH_post, const float *a,
                                                 float *H_res, const float *H_pre,
                                                 const float *H_post, const float *sums,
                                                 int sk_iters, float *g_z) {
  constexpr int R = Dims<N, MODE>::R;
  if constexpr (MODE == MHCL_RES_LITE) {
    perm_mix_bwd<N>(gH_res, g_z, std::make_integer_sequence<int, R>{});
    float mean = 0.f;
#pragma unroll
    for (int k = 0; k < R; ++k) mean += a[k] * g_z[k];
#pragma unroll
    for (int k = 0; k < R; ++k) g_z[k] = a[k] * (g_z[k] - mean);
  } else {
    float g[R];
#pragma unroll
    for (int e = 0; e < R; ++e) g[e] = gH_res[e];
    for (int it = sk_iters - 1; it >= 0; --it) {
#pragma unroll
      for (int i = 0; i < N; ++i) {   // undo the row step
        const float s = sums[(2 * it + 1) * N + i];
        const float inv = 1.f / s;
        float d = 0.f;
#pragma unroll
        for (int j = 0; j < N; ++j) d += g[i * N + j] * H_res[i * N + j];
#pragma unroll
        for (int j = 0; j < N; ++j) {
          g[i * N + j] = (g[i * N + j] - d) * inv;
          H_res[i * N + j] *= s;
        }
      }
#pragma unroll
      for (int j = 0; j < N; ++j) {   // undo the column step
        const float s = sums[(2 * it) * N + j];
        const float inv = 1.f / s;
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < N; ++i) d += g[i * N + j] * H_res[i * N + j];
#pragma unroll
        for (int i = 0; i < N; ++i) {
          g[i * N + j] = (g[i * N + j] - d) * inv;
          H_res[i * N + j] *= s;
        }
      }
    }
#pragma unroll
    for (int e = 0; e < R; ++e) g_z[e] = g[e] * a[e];   // a = exp(z - max) = SK input
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    g_z[R + j] = gH_pre[j] * H_pre[j] * (1.f - H_pre[j]);
    g_z[R + N + j] = gH_post[j] * H_post[j] * (1.f - 0.5f * H_post[j]);
  }
}

// ------------------------------------------------- block reduction
// Sum of `v` over the 256 threads of a block, result valid in every thread.
// `red` is shared scratch of at least 4 floats (one per wave).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

}  // namespace mhcl
