// Per-token coefficients of the table forms: a = softmax over K logits,
// H_res = sum_k a_k P_k over the K permutations of a table [K][n] (Sec. 5, the
// paragraph on larger n: a run-time subset, n up to 8, K up to 128; also the
// full form at n = 5, whose 120 permutations make the unrolled compile-time
// sums too large for the registers); gates as in Sec. 3.2.
//   coeffs_group_kernel     : eight lanes per token; forward coefficients and
//                             the stage between the two passes of the fused backward
//   coeffs_bwd_subset_kernel: one token per thread, for the separable
//                             mhcl_coeffs_bwd (weights in LDS: a register array
//                             indexed by a run-time k would go to scratch memory)
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

// ---------------------------------------------------------------------------
// The same per-token work with eight lanes per token (block = 64 tokens, 512
// threads), for the table forms with many logits (a permutation subset, or
// the full form at n = 5 with its 120 permutations): one token per lane left
// a single wave per CU walking K-long dependent loops over strided global
// loads.  Here the block first stages its tokens' logits, summed over the
// K-split slices, with contiguous loads into LDS; lane l of a token then owns
// the logits k = l, l + 8, ... (softmax, g_a, g_z) and row l of H_res.
//   BWD = false: H_res, H_pre, H_post                       (forward)
//   BWD = true : the stage between the two backward passes, outputs as
//                bwd_epilogue_fast_kernel writes them (cpk, vr, vrT, gz sums);
//                F16ROWS as there.
// The table comes from device memory (`sigma`) or, if `use_tab`, by value.
struct TableArg {
  int8_t s[kMaxPerm * kMaxNSubset];
};
constexpr int kGTok = 64, kGThreads = 512, kOwn = kMaxPerm / 8;

__device__ __forceinline__ float group_sum(float v) {
  v += __shfl_xor(v, 1, 64);
  v += __shfl_xor(v, 2, 64);
  v += __shfl_xor(v, 4, 64);
  return v;
}
__device__ __forceinline__ float group_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 1, 64));
  v = fmaxf(v, __shfl_xor(v, 2, 64));
  v = fmaxf(v, __shfl_xor(v, 4, 64));
  return v;
}

// floats of dynamic LDS the kernel needs (plus K * N table bytes)
inline size_t group_lds_bytes(int N, int K, bool bwd) {
  const int M = K + 2 * N, ld = M | 1;
  size_t fl = 2 * static_cast<size_t>(kGTok) * ld + kGTok;
  if (bwd) fl += static_cast<size_t>(kGTok) * (N * N + 1) + 4 * kGTok;
  return fl * sizeof(float) + static_cast<size_t>(K) * N;
}

template <int N, bool BWD, bool F16ROWS>
__global__ __launch_bounds__(kGThreads) void coeffs_group_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha,
    const float *__restrict__ gH_res, const float *__restrict__ gH_pre,
    const float *__restrict__ gH_post, int nC, float eps, int64_t T, int K,
    const int8_t *__restrict__ sigma, const TableArg tab, int use_tab,
    float *__restrict__ H_res, float *__restrict__ H_pre, float *__restrict__ H_post, int CP,
    int MP32, int MP16, float *__restrict__ cpk, uint16_t *__restrict__ vr_hi,
    uint16_t *__restrict__ vr_lo, uint16_t *__restrict__ vrT_hi, uint16_t *__restrict__ vrT_lo,
    float *__restrict__ gz_sums) {
  extern __shared__ float smem[];
  const int M = K + 2 * N, ld = M | 1;
  constexpr int NN = N * N, gld = NN + 1;
  float *u_s = smem;                              // [64][ld]  raw logits
  float *a_s = u_s + kGTok * ld;                  // [64][ld]  softmax weights, later g_z
  float *g_s = a_s + kGTok * ld;                  // [64][gld] g_H_res            (BWD)
  float *r_s = g_s + (BWD ? kGTok * gld : 0);     // [64]      RMSNorm scale
  float *t_s = r_s + kGTok;                       // [64][4]   sums of g_z u per group, row scale (BWD)
  int8_t *sig = reinterpret_cast<int8_t *>(t_s + (BWD ? 4 * kGTok : 0));   // [K][N]
  const int tid = threadIdx.x;
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kGTok;

  // stage: table (entries clamped to 0..N-1), logits, scale, g_H_res
  for (int i = tid; i < K * N; i += kGThreads) {
    int v = use_tab ? tab.s[i] : sigma[i];
    v = v < 0 ? 0 : (v > N - 1 ? N - 1 : v);
    sig[i] = static_cast<int8_t>(v);
  }
  // (four elements per thread at a time: their loads, one per K-split slice, are all
  // requested before the first sum; the block is alone on its CU when T is small)
  for (int e0 = tid; e0 < kGTok * M; e0 += 4 * kGThreads) {
    float u[4];
    int64_t src[4];
    int dst[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      int e = e0 + v * kGThreads;
      if (e > kGTok * M - 1) e = kGTok * M - 1;   // surplus threads repeat the last element
      const int tk = e / M, m = e - tk * M;
      int64_t tt = t0 + tk;
      if (tt > T - 1) tt = T - 1;
      src[v] = tt * M + m;
      dst[v] = tk * ld + m;
      u[v] = u_raw[src[v]];
    }
    for (int pt = 1; pt < parts; ++pt) {
      float w[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) w[v] = u_raw[static_cast<int64_t>(pt) * T * M + src[v]];
#pragma unroll
      for (int v = 0; v < 4; ++v) u[v] += w[v];
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) u_s[dst[v]] = u[v];
  }
  if (tid < kGTok) {
    int64_t tt = t0 + tid;
    if (tt > T - 1) tt = T - 1;
    float ssq = sumsq[tt];
    for (int pt = 1; pt < parts; ++pt) ssq += sumsq[pt * T + tt];
    r_s[tid] = 1.f / sqrtf(ssq / static_cast<float>(nC) + eps);
  }
  if constexpr (BWD) {
    for (int e = tid; e < kGTok * NN; e += kGThreads) {
      const int tk = e / NN, c = e - tk * NN;
      int64_t tt = t0 + tk;
      if (tt > T - 1) tt = T - 1;
      g_s[tk * gld + c] = gH_res[tt * NN + c];
    }
  }
  __syncthreads();

  const int tok = tid >> 3, l = tid & 7;
  const int64_t t = t0 + tok;
  const bool live = t < T;
  const int64_t tl = live ? t : T - 1;
  const float r = r_s[tok];
  const float a0 = alpha[0], a1 = alpha[1], a2 = alpha[2];
  const float *ut = u_s + tok * ld;
  float *at = a_s + tok * ld;

  // softmax over the K residual logits; own[] = this lane's weights
  float own[kOwn];
  float zmax = -INFINITY;
#pragma unroll
  for (int kk = 0; kk < kOwn; ++kk) {
    const int k = l + 8 * kk;
    own[kk] = -INFINITY;
    if (k < K) {
      own[kk] = a0 * (r * ut[k]) + b[k];
      zmax = fmaxf(zmax, own[kk]);
    }
  }
  zmax = group_max(zmax);
  float sum = 0.f;
#pragma unroll
  for (int kk = 0; kk < kOwn; ++kk) {
    const int k = l + 8 * kk;
    own[kk] = k < K ? expf(own[kk] - zmax) : 0.f;
    sum += own[kk];
  }
  sum = group_sum(sum);
#pragma unroll
  for (int kk = 0; kk < kOwn; ++kk) {
    const int k = l + 8 * kk;
    own[kk] = own[kk] / sum;
    if (k < K) at[k] = own[kk];
  }
  __syncthreads();

  // row l of H_res = sum_k a_k P_k, k ascending
  if (l < N) {
    float row[N];
#pragma unroll
    for (int j = 0; j < N; ++j) row[j] = 0.f;
    for (int k = 0; k < K; ++k) {
      const float w = at[k];
      const int sj = sig[k * N + l];
#pragma unroll
      for (int j = 0; j < N; ++j) row[j] += (j == sj) ? w : 0.f;
    }
    if (live) {
      float *dst = BWD ? cpk + t * CP + l * N : H_res + t * NN + l * N;
#pragma unroll
      for (int j = 0; j < N; ++j) dst[j] = row[j];
    }
  }

  if constexpr (!BWD) {
    if (l < N && live) {
      H_pre[t * N + l] = sigmoidf(a1 * (r * ut[K + l]) + b[K + l]);
      H_post[t * N + l] = 2.f * sigmoidf(a2 * (r * ut[K + N + l]) + b[K + N + l]);
    }
    return;
  } else {
    // g_a[k] = sum_i g_H_res[i][sigma_k(i)], g_z = a (g_a - <a, g_a>)
    const float *gt = g_s + tok * gld;
    float gown[kOwn];
    float meanp = 0.f;
#pragma unroll
    for (int kk = 0; kk < kOwn; ++kk) {
      const int k = l + 8 * kk;
      gown[kk] = 0.f;
      if (k < K) {
        float sg = 0.f;
#pragma unroll
        for (int i = 0; i < N; ++i) sg += gt[i * N + sig[k * N + i]];
        gown[kk] = sg;
        meanp += own[kk] * sg;
      }
    }
    const float mean = group_sum(meanp);
    __syncthreads();   // the weights in a_s are no longer needed: it now takes g_z
    float dotp = 0.f, gap[3] = {0.f, 0.f, 0.f}, vmaxp = 0.f;
#pragma unroll
    for (int kk = 0; kk < kOwn; ++kk) {
      const int k = l + 8 * kk;
      if (k < K) {
        const float g = live ? own[kk] * (gown[kk] - mean) : 0.f;
        const float u = ut[k];
        const float v = r * a0 * g;
        at[k] = g;
        gap[0] += g * (r * u);
        dotp += v * u;
        vmaxp = fmaxf(vmaxp, fabsf(v));
      }
    }
    if (l < N) {
      const float up = ut[K + l], uq = ut[K + N + l];
      const float hp = sigmoidf(a1 * (r * up) + b[K + l]);
      const float hq = 2.f * sigmoidf(a2 * (r * uq) + b[K + N + l]);
      float gp = gH_pre[tl * N + l] * hp * (1.f - hp);
      float gq = gH_post[tl * N + l] * hq * (1.f - 0.5f * hq);
      if (live) {
        cpk[t * CP + NN + l] = hp;
        cpk[t * CP + NN + N + l] = hq;
      } else {
        gp = 0.f;
        gq = 0.f;
      }
      at[K + l] = gp;
      at[K + N + l] = gq;
      const float vp = r * a1 * gp, vq = r * a2 * gq;
      gap[1] = gp * (r * up);
      gap[2] = gq * (r * uq);
      dotp += vp * up + vq * uq;
      vmaxp = fmaxf(vmaxp, fmaxf(fabsf(vp), fabsf(vq)));
    }
    const float dot = group_sum(dotp);
    const float vmax = group_max(vmaxp);
#pragma unroll
    for (int g = 0; g < 3; ++g) gap[g] = group_sum(gap[g]);
    if (l == 0) {
      const float sc = (F16ROWS && vmax > 0.f) ? vmax : 1.f;
      t_s[tok * 4 + 0] = gap[0];
      t_s[tok * 4 + 1] = gap[1];
      t_s[tok * 4 + 2] = gap[2];
      t_s[tok * 4 + 3] = 1.f / sc;
      if (live) {
        cpk[t * CP + NN + 2 * N] = (r * r / static_cast<float>(nC)) * dot;
        if constexpr (F16ROWS) cpk[t * CP + NN + 2 * N + 1] = sc;
      }
    }
    __syncthreads();

    // vr = r alpha_g g_z of logit m of block token tk (zero past the last logit)
    auto vr_of = [&](int tk, int m) {
      if (m >= M) return 0.f;
      const float al = m < K ? a0 : (m < K + N ? a1 : a2);
      return r_s[tk] * al * a_s[tk * ld + m];
    };
    auto split = [](float v, bool f16, uint16_t &hi, uint16_t &lo) {
      if (f16) {
        const _Float16 h16 = static_cast<_Float16>(v);
        const _Float16 l16 = static_cast<_Float16>(v - static_cast<float>(h16));
        hi = __builtin_bit_cast(uint16_t, h16);
        lo = __builtin_bit_cast(uint16_t, l16);
      } else {
        hi = f32_to_bf16(v);
        lo = f32_to_bf16(v - bf16_to_f32(hi));
      }
    };
    auto pack8 = [](const uint16_t (&h)[8]) {
      uint4 v;
      v.x = h[0] | (uint32_t(h[1]) << 16); v.y = h[2] | (uint32_t(h[3]) << 16);
      v.z = h[4] | (uint32_t(h[5]) << 16); v.w = h[6] | (uint32_t(h[7]) << 16);
      return v;
    };
    // rows [Tpad][MP32]: eight consecutive logits of one token per thread
    const int nvec = MP32 / 8;
    for (int e = tid; e < kGTok * nvec; e += kGThreads) {
      const int tk = e / nvec, v8 = e - tk * nvec;
      const float inv = F16ROWS ? t_s[tk * 4 + 3] : 1.f;
      uint16_t hi[8], lo[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) split(vr_of(tk, 8 * v8 + i) * inv, F16ROWS, hi[i], lo[i]);
      const size_t off = static_cast<size_t>(t0 + tk) * MP32 + 8 * v8;
      *reinterpret_cast<uint4 *>(vr_hi + off) = pack8(hi);
      *reinterpret_cast<uint4 *>(vr_lo + off) = pack8(lo);
    }
    // tokens innermost [Tpad/32][MP16][32]: eight consecutive tokens of one logit per thread
    const int64_t blk0 = t0 >> 5;
    for (int e = tid; e < 2 * MP16 * 4; e += kGThreads) {
      const int half = e / (MP16 * 4), rem = e - half * (MP16 * 4);
      const int m = rem >> 2, tg = rem & 3;
      uint16_t hi[8], lo[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) split(vr_of(half * 32 + tg * 8 + i, m), false, hi[i], lo[i]);
      const size_t off = (static_cast<size_t>(blk0 + half) * MP16 + m) * 32 + tg * 8;
      *reinterpret_cast<uint4 *>(vrT_hi + off) = pack8(hi);
      *reinterpret_cast<uint4 *>(vrT_lo + off) = pack8(lo);
    }
    // sums over the block's 64 tokens, token order
    if (tid < M + 3) {
      float sacc = 0.f;
      if (tid < M) {
        for (int tk = 0; tk < kGTok; ++tk) sacc += a_s[tk * ld + tid];
      } else {
        for (int tk = 0; tk < kGTok; ++tk) sacc += t_s[tk * 4 + (tid - M)];
      }
      gz_sums[static_cast<int64_t>(blockIdx.x) * (M + 3) + tid] = sacc;
    }
  }
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


// table of the launch: the caller's subset, or all 120 permutations of n = 5 in
// lexicographic order (full form), passed by value
struct GroupTable {
  int K = 0, use_tab = 0;
  const int8_t *sigma = nullptr;
  TableArg tab{};
};
bool group_table(const mhcl_desc &d, GroupTable &g) {
  if (d.res_mode == MHCL_RES_SUBSET) {
    if (d.n_perm < 1 || d.n_perm > kMaxPerm || !d.perm) return false;
    g.K = d.n_perm;
    g.sigma = d.perm;
    return true;
  }
  if (d.res_mode == MHCL_RES_LITE && d.n == 5) {
    g.K = factorial(5);
    g.use_tab = 1;
    for (int k = 0; k < g.K; ++k)
      for (int i = 0; i < 5; ++i) g.tab.s[k * 5 + i] = Perm<5>::tab.s[k][i];
    return true;
  }
  return false;
}

template <typename Kern>
hipError_t allow_lds(Kern kern, size_t lds) {
  if (lds <= 64 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
}

}  // namespace

bool coeffs_group_ok(const mhcl_desc &d) {
  return d.res_mode == MHCL_RES_SUBSET || (d.res_mode == MHCL_RES_LITE && d.n == 5);
}

hipError_t launch_coeffs_group(const mhcl_desc &d, int parts, const float *u_raw,
                               const float *sumsq, const float *b, const float *alpha,
                               float *H_res, float *H_pre, float *H_post, hipStream_t s) {
  GroupTable g;
  if (!group_table(d, g)) return hipErrorInvalidValue;
  return dispatch_n8(d.n, [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    auto kern = coeffs_group_kernel<N, false, false>;
    const size_t lds = group_lds_bytes(N, g.K, false);
    hipError_t e = allow_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>((d.T + kGTok - 1) / kGTok)),
                       dim3(kGThreads), lds, s, u_raw, sumsq, parts, b, alpha, nullptr, nullptr,
                       nullptr, d.n * d.C, d.eps, d.T, g.K, g.sigma, g.tab, g.use_tab, H_res, H_pre,
                       H_post, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
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

hipError_t launch_bwd_epilogue_group(const mhcl_desc &d, const float *b, const float *alpha,
                                     const FastBwdWs &w, hipStream_t s) {
  GroupTable g;
  if (!group_table(d, g)) return hipErrorInvalidValue;
  const int64_t Tpad = (d.T + 63) / 64 * 64;
  const int M = g.K + 2 * d.n;
  if (w.MP32 != (M + 31) / 32 * 32 || w.MP16 != (M + 15) / 16 * 16) return hipErrorInvalidValue;
  const bool f16 = fast_bwd_whi(d);   // rows for bwd_out_w16_kernel
  if (f16 && w.CP < d.n * d.n + 2 * d.n + 2) return hipErrorInvalidValue;
  return dispatch_n8(d.n, [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    auto launch = [&](auto kern) {
      const size_t lds = group_lds_bytes(N, g.K, true);
      hipError_t e = allow_lds(kern, lds);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(Tpad / kGTok)), dim3(kGThreads), lds, s,
                         w.u_raw, w.sumsq, w.parts, b, alpha, w.gH_res, w.gH_pre, w.gH_post,
                         d.n * d.C, d.eps, d.T, g.K, g.sigma, g.tab, g.use_tab, nullptr, nullptr,
                         nullptr, w.CP, w.MP32, w.MP16, w.cpk, w.vr_hi, w.vr_lo, w.vrT_hi, w.vrT_lo,
                         w.gz);
      return hipGetLastError();
    };
    if constexpr (N >= 5) {
      if (f16) return launch(coeffs_group_kernel<N, true, true>);
    }
    return launch(coeffs_group_kernel<N, true, false>);
  });
}

}  // namespace mhcl
