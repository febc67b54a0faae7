// bf16 fast path of libmhcl for gfx950: the thin projections run on the MFMA
// units (v_mfma_f32_16x16x32_bf16, fp32 accumulate), everything else streams.
//
// x is exactly bf16; W is fp32 and is split into two bf16 parts (hi + lo), so
// x_hat W carries ~16 mantissa bits of W at twice the MFMA work, which stays a
// small fraction of the time the HBM stream needs.
#include "mhcl_common.h"
#include "mhcl_internal.h"
#include "mhcl_mfma.h"

namespace mhcl {

namespace {

__device__ __forceinline__ void split_bf16(float w, uint16_t &hi, uint16_t &lo) {
  hi = f32_to_bf16(w);
  lo = f32_to_bf16(w - bf16_to_f32(hi));
}

// W [K, M] fp32 -> B layout (see mhcl_mfma.h).  One thread per (block pair, lane).
__device__ __forceinline__ void pack_w_b_thread(int idx, const float *__restrict__ W, int K, int M,
                                                int NT, uint4 *__restrict__ Wp) {
  const int lane = idx & 63, blk = idx >> 6;   // blk = s*NT + j
  if (blk >= (K / 32) * NT) return;
  const int s = blk / NT, j = blk % NT, r = lane & 15, q = lane >> 4;
  const int col = 16 * j + r;
  uint16_t hi[8], lo[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k = 32 * s + 8 * q + e;
    const float w = col < M ? W[static_cast<size_t>(k) * M + col] : 0.f;
    split_bf16(w, hi[e], lo[e]);
  }
  uint4 vh, vl;
  vh.x = hi[0] | (uint32_t(hi[1]) << 16); vh.y = hi[2] | (uint32_t(hi[3]) << 16);
  vh.z = hi[4] | (uint32_t(hi[5]) << 16); vh.w = hi[6] | (uint32_t(hi[7]) << 16);
  vl.x = lo[0] | (uint32_t(lo[1]) << 16); vl.y = lo[2] | (uint32_t(lo[3]) << 16);
  vl.z = lo[4] | (uint32_t(lo[5]) << 16); vl.w = lo[6] | (uint32_t(lo[7]) << 16);
  Wp[(static_cast<size_t>(blk) * 2 + 0) * 64 + lane] = vh;
  Wp[(static_cast<size_t>(blk) * 2 + 1) * 64 + lane] = vl;
}

// Also clears `nzero` floats at `zero` (grid-stride): scratch that the kernel launched after
// this one expects to start from zero, without a launch of its own.
__global__ __launch_bounds__(256) void pack_w_b_kernel(const float *__restrict__ W, int K, int M,
                                                       int NT, uint4 *__restrict__ Wp,
                                                       float *__restrict__ zero, unsigned nzero) {
  pack_w_b_thread(blockIdx.x * 256 + threadIdx.x, W, K, M, NT, Wp);
  for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < nzero; i += gridDim.x * 256) zero[i] = 0.f;
}

// ---------------------------------------------------------------------------
// Forward projection: u_raw[t][m] = sum_k x_hat[t][k] W[k][m], sumsq[t] = sum_k
// x_hat[t][k]^2 (RMSNorm's statistic), both from ONE read of x.
//
// Block = 8 waves, each wave owns one or two 16-token A tiles and walks
// the whole K = nC range; the block's waves share each chunk of packed W
// through LDS (double buffered).  A tiles come straight from HBM in MFMA lane
// order: lane (r, q) reads 16 bytes of token r at column 32 s + 8 q, several
// consecutive steps s back to back.
// sum(x^2) is the diagonal of the tile's Gram matrix A A^T, one more MFMA with
// the A tile as both operands.
template <int NT>
struct ProjCfg {
  static constexpr int KC = NT >= 4 ? 2 : 4;        // K steps per chunk
  static constexpr int TG = NT <= 3 ? 1 : 2;        // 16-token A tiles per wave
  // eight waves share each W chunk: one block per CU, half the W traffic from L2 of two
  // four-wave blocks (0.23 -> 0.21 ms at n = 4, C = 4096)
  static constexpr int WAVES = 8;
  static constexpr int kThreads = 64 * WAVES;
  static constexpr int kTokens = 16 * WAVES * TG;              // tokens per block
  static constexpr int kChunkVec = KC * NT * 2 * 64;           // u32x4 per chunk
  static constexpr int kLdsBytes = 2 * kChunkVec * 16;
};

template <int NT>
__global__ __launch_bounds__(ProjCfg<NT>::kThreads, 1) void proj_mfma_kernel(const uint16_t *__restrict__ x,
                                                           const u32x4 *__restrict__ Wp, int K,
                                                           int M, int64_t T,
                                                           float *__restrict__ u_raw,
                                                           float *__restrict__ sumsq) {
  // gridDim.y blocks share the K range of the same tokens (K split): block
  // (bx, part) walks K steps [part * nsteps, (part + 1) * nsteps) and writes its
  // partial u_raw / sumsq to slice `part`; the consumer adds the slices in order.
  using Cfg = ProjCfg<NT>;
  constexpr int KC = Cfg::KC, TG = Cfg::TG;
  extern __shared__ u32x4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int64_t tw = static_cast<int64_t>(blockIdx.x) * Cfg::kTokens + wave * (16 * TG);
  const uint16_t *row[TG];
#pragma unroll
  for (int g = 0; g < TG; ++g) {
    int64_t t = tw + g * 16 + r;
    if (t > T - 1) t = T - 1;
    row[g] = x + t * K + q * 8;
  }
  const int nsteps = K / 32 / gridDim.y;          // K steps of this block
  const int step0 = blockIdx.y * nsteps;
#pragma unroll
  for (int g = 0; g < TG; ++g) row[g] += static_cast<size_t>(step0) * 32;
  Wp += static_cast<size_t>(step0) * NT * 2 * 64;
  u_raw += static_cast<size_t>(blockIdx.y) * T * M;
  sumsq += static_cast<size_t>(blockIdx.y) * T;
  const int nchunks = (nsteps + KC - 1) / KC;

  f32x4 acc[TG][NT], ss[TG];
#pragma unroll
  for (int g = 0; g < TG; ++g) {
    ss[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[g][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  constexpr int WV = (Cfg::kChunkVec + Cfg::kThreads - 1) / Cfg::kThreads;   // u32x4 of W each thread stages per chunk
  constexpr bool kWholeW = Cfg::kChunkVec % Cfg::kThreads == 0;
  u32x4 a[2][TG][KC], wst[WV];
  const int wlim = nsteps * NT * 2 * 64 - 1;   // last valid u32x4 of packed W

  // Loads never branch: a step past the end re-reads the last step (address
  // clamped); compute() zeroes such a tile where it is consumed, so it adds
  // nothing and the load itself is never waited for early.
  // (All blocks walk K in the same order: they then read the same W chunk at about the
  // same time, which keeps W in L2; starting each block elsewhere, as bwd_reduce_kernel
  // does, cost 20 % with nine logit tiles and gained nothing with two.)
  auto load_a = [&](u32x4 (&dst)[TG][KC], int c) {
#pragma unroll
    for (int s = 0; s < KC; ++s) {
      const int step = c * KC + s;
      const int sc = step < nsteps ? step : nsteps - 1;
#pragma unroll
      for (int g = 0; g < TG; ++g)
        dst[g][s] = *reinterpret_cast<const u32x4 *>(row[g] + sc * 32);
    }
  };
  auto load_w = [&](int c) {
    const int base = c * Cfg::kChunkVec;
#pragma unroll
    for (int i = 0; i < WV; ++i) {
      int o = i * Cfg::kThreads + threadIdx.x;
      if (!kWholeW && o > Cfg::kChunkVec - 1) o = Cfg::kChunkVec - 1;   // surplus threads repeat the last word
      const int e = base + o;
      wst[i] = Wp[e < wlim ? e : wlim];
    }
  };
  auto store_w = [&](int buf) {
#pragma unroll
    for (int i = 0; i < WV; ++i) {
      int o = i * Cfg::kThreads + threadIdx.x;
      if (!kWholeW && o > Cfg::kChunkVec - 1) o = Cfg::kChunkVec - 1;
      lds[buf * Cfg::kChunkVec + o] = wst[i];
    }
  };
  // `tail`: the chunk may run past the last K step; such steps get a zero A tile
  auto compute = [&](const u32x4 (&av)[TG][KC], int buf, int c, auto tail) {
    const u32x4 *wb = lds + buf * Cfg::kChunkVec;
#pragma unroll
    for (int s = 0; s < KC; ++s) {
      u32x4 at[TG];
#pragma unroll
      for (int g = 0; g < TG; ++g) {
        if constexpr (decltype(tail)::value)
          at[g] = c * KC + s < nsteps ? av[g][s] : u32x4{0, 0, 0, 0};
        else
          at[g] = av[g][s];
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const u32x4 bh = wb[((s * NT + j) * 2 + 0) * 64 + lane];
        const u32x4 bl = wb[((s * NT + j) * 2 + 1) * 64 + lane];
#pragma unroll
        for (int g = 0; g < TG; ++g) {
          acc[g][j] = mfma16(at[g], bh, acc[g][j]);
          acc[g][j] = mfma16(at[g], bl, acc[g][j]);
        }
      }
#pragma unroll
      for (int g = 0; g < TG; ++g) ss[g] = mfma16(at[g], at[g], ss[g]);
    }
  };
  constexpr std::false_type kFull{};
  constexpr std::true_type kTail{};

  // W is requested before the A tiles of the same chunk: loads return in order,
  // so staging W into LDS only has to wait for the W loads and leaves the A
  // loads of the next chunk in flight across the barrier.
  load_w(0);
  load_a(a[0], 0);
  store_w(0);
  __syncthreads();
  int c = 0;
  for (; c + 2 < nchunks; c += 2) {
    load_w(c + 1); load_a(a[1], c + 1);
    __builtin_amdgcn_sched_barrier(0);   // keep the whole next chunk in flight during compute
    compute(a[0], 0, c, kFull);
    store_w(1);
    __syncthreads();
    load_w(c + 2); load_a(a[0], c + 2);
    __builtin_amdgcn_sched_barrier(0);
    compute(a[1], 1, c + 1, kFull);
    store_w(0);
    __syncthreads();
  }
  if (c + 1 < nchunks) {
    load_w(c + 1); load_a(a[1], c + 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(a[0], 0, c, kFull);
    store_w(1);
    __syncthreads();
    compute(a[1], 1, c + 1, kTail);
  } else {
    compute(a[0], 0, c, kTail);
  }

  // D layout: lane (r, q) holds logit 16 j + r for tokens 4 q + i
#pragma unroll
  for (int g = 0; g < TG; ++g) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t t = tw + g * 16 + 4 * q + i;
      if (t < T) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int col = 16 * j + r;
          if (col < M) u_raw[t * M + col] = acc[g][j][i];
        }
      }
    }
    // Gram diagonal: token r sits at row r = 4 q + i  <=>  q == r / 4, i == r % 4
    if ((r >> 2) == q) {
      const int i = r & 3;
      const float v = i == 0 ? ss[g][0] : (i == 1 ? ss[g][1] : (i == 2 ? ss[g][2] : ss[g][3]));
      const int64_t t = tw + g * 16 + r;
      if (t < T) sumsq[t] = v;
    }
  }
}


// W [K, M] fp32 -> A layout (see mhcl_mfma.h).  One thread per (block pair, lane).
__device__ __forceinline__ void pack_w_a_thread(int idx, const float *__restrict__ W, int K, int M,
                                                int MS, uint4 *__restrict__ Wa) {
  const int lane = idx & 63, blk = idx >> 6;   // blk = (S*4 + h)*MS + ms
  if (blk >= (K / 64) * 4 * MS) return;
  const int ms = blk % MS, h = (blk / MS) & 3, S = blk / (4 * MS);
  const int r = lane & 15, q = lane >> 4;
  const int k = 64 * S + 32 * (h >> 1) + 8 * (r >> 2) + 4 * (h & 1) + (r & 3);
  uint16_t hi[8], lo[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int col = 32 * ms + 8 * q + e;
    const float w = col < M ? W[static_cast<size_t>(k) * M + col] : 0.f;
    split_bf16(w, hi[e], lo[e]);
  }
  uint4 vh, vl;
  vh.x = hi[0] | (uint32_t(hi[1]) << 16); vh.y = hi[2] | (uint32_t(hi[3]) << 16);
  vh.z = hi[4] | (uint32_t(hi[5]) << 16); vh.w = hi[6] | (uint32_t(hi[7]) << 16);
  vl.x = lo[0] | (uint32_t(lo[1]) << 16); vl.y = lo[2] | (uint32_t(lo[3]) << 16);
  vl.z = lo[4] | (uint32_t(lo[5]) << 16); vl.w = lo[6] | (uint32_t(lo[7]) << 16);
  Wa[(static_cast<size_t>(blk) * 2 + 0) * 64 + lane] = vh;
  Wa[(static_cast<size_t>(blk) * 2 + 1) * 64 + lane] = vl;
}

// W [K, M] fp32 -> A layout with ONE fp16 part per block (11 significant bits): for the
// single-kernel wide pass 2, whose LDS holds one part only.  Block index (S*4 + h)*MS + ms.
// Entries are multiplied by `scale`, a power of two chosen from max |W| so that the largest
// entry lands in [2^13, 2^14): weights of any magnitude fit fp16, and the consumer multiplies
// the MFMA result by 1 / scale (exact).
__device__ __forceinline__ void pack_w_a16_thread(int idx, const float *__restrict__ W, int K, int M,
                                                  int MS, float scale, uint4 *__restrict__ Wa) {
  const int lane = idx & 63, blk = idx >> 6;
  if (blk >= (K / 64) * 4 * MS) return;
  const int ms = blk % MS, h = (blk / MS) & 3, S = blk / (4 * MS);
  const int r = lane & 15, q = lane >> 4;
  const int k = 64 * S + 32 * (h >> 1) + 8 * (r >> 2) + 4 * (h & 1) + (r & 3);
  float w[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int col = 32 * ms + 8 * q + e;
    w[e] = col < M ? W[static_cast<size_t>(k) * M + col] * scale : 0.f;
  }
  uint4 v;
  v.x = cvt_pk_f16(w[0], w[1]); v.y = cvt_pk_f16(w[2], w[3]);
  v.z = cvt_pk_f16(w[4], w[5]); v.w = cvt_pk_f16(w[6], w[7]);
  Wa[static_cast<size_t>(blk) * 64 + lane] = v;
}

// max |W| in two stages without atomics: each of kWmaxBlocks blocks writes the maximum over
// its grid-stride share of W; readers take the maximum of those.
constexpr int kWmaxBlocks = 256;
__global__ __launch_bounds__(256) void w_absmax_kernel(const float4 *__restrict__ W4, size_t count4,
                                                       float *__restrict__ part) {
  // count4 16-byte vectors (K is a multiple of 64, so K * M is a multiple of 4); four loads in
  // flight per lane
  __shared__ float red[4];
  float m = 0.f;
  const size_t stride = static_cast<size_t>(gridDim.x) * 256;
  size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  auto take = [&](const float4 &v) {
    // (a NaN entry never wins: it poisons the products downstream anyway)
    m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
  };
  for (; i + 3 * stride < count4; i += 4 * stride) {
    const float4 a = W4[i], b = W4[i + stride], c = W4[i + 2 * stride], d = W4[i + 3 * stride];
    take(a); take(b); take(c); take(d);
  }
  for (; i < count4; i += stride) take(W4[i]);
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) part[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
// the power of two that brings `wmax` into [2^13, 2^14) (1 for zero, infinite or NaN maxima)
__device__ __forceinline__ float fp16_fit_scale(float wmax) {
  if (!(wmax > 0.f) || !(wmax < 3.0e38f)) return 1.f;
  int e;
  (void)frexpf(wmax, &e);            // wmax = f * 2^e, f in [0.5, 1)
  int k = 14 - e;                    // wmax * 2^k in [2^13, 2^14)
  k = k > 126 ? 126 : (k < -126 ? -126 : k);
  return ldexpf(1.f, k);
}

// Both layouts the backward needs in one launch: blocks [0, nb_b) write the B layout
// (pass 1's projection), the rest the A layout (pass 2), with one fp16 part if `a16`;
// then `wmax_part` holds kWmaxBlocks partial maxima of |W| and `wscale[0..1]` receives the
// scale applied to the fp16 part and its inverse.
__global__ __launch_bounds__(256) void pack_w_ab_kernel(const float *__restrict__ W, int K, int M,
                                                        int NT, int MS, int nb_b, int a16,
                                                        const float *__restrict__ wmax_part,
                                                        float *__restrict__ wscale,
                                                        uint4 *__restrict__ Wp,
                                                        uint4 *__restrict__ Wa) {
  const int b = blockIdx.x;
  if (b < nb_b) {
    pack_w_b_thread(b * 256 + threadIdx.x, W, K, M, NT, Wp);
  } else if (a16) {
    __shared__ float red[4];
    static_assert(kWmaxBlocks == 256, "one partial maximum per thread");
    float m = wmax_part[threadIdx.x];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    const float scale = fp16_fit_scale(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])));
    if (b == nb_b && threadIdx.x == 0) {
      wscale[0] = scale;
      wscale[1] = 1.f / scale;
    }
    pack_w_a16_thread((b - nb_b) * 256 + threadIdx.x, W, K, M, MS, scale, Wa);
  } else {
    pack_w_a_thread((b - nb_b) * 256 + threadIdx.x, W, K, M, MS, Wa);
  }
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b),
                                         acc, false);
}
// (the words are passed by value: a bit cast applied directly to a vector
// element expression reads element 0 whatever the index)
__device__ __forceinline__ float dot8_bf16(const u32x4 &a, const u32x4 &b, float acc) {
  acc = dot2_bf16(a.x, b.x, acc);
  acc = dot2_bf16(a.y, b.y, acc);
  acc = dot2_bf16(a.z, b.z, acc);
  acc = dot2_bf16(a.w, b.w, acc);
  return acc;
}

// ---------------------------------------------------------------------------
// Backward pass 1: every per-token reduction of the backward from ONE read of
// x, g_xout, y, g_h:
//   u_raw, sumsq                      (recomputed projection, as in forward)
//   g_H_res[i][j] = <g_xout[i], x[j]>, g_H_post[i] = <g_xout[i], y>,
//   g_H_pre[j]    = <g_h, x[j]>       (reductions over C)
// Block = WAVES (4 or 8) waves x 16 tokens.  The loop runs over 64-column steps of C; at
// each step a lane holds, for its token, 2 x 8 columns (two loads issued back
// to back, so that four lanes consume a whole 128-byte line per visit) of all n streams of x and
// g_xout and of y and g_h, feeds the x tiles to the MFMA projection (W blocks
// of that step staged in LDS, double buffered) and the dot products to
// v_dot2_f32_bf16.  The four lanes that share a token are summed at the end.
template <int N, int NT, int WAVES>
struct ReduceCfg {
  static constexpr int kStageVec = N * 2 * NT * 2 * 64;        // 16-byte words of W per step
  static constexpr int kThreads = 64 * WAVES;
  static constexpr int WV = (kStageVec + kThreads - 1) / kThreads;
  static constexpr int kLdsBytes = 2 * kStageVec * 16;
};

template <int N, int NT, int WAVES>
__global__ __launch_bounds__(64 * WAVES, (WAVES == 4 || N <= 3) ? 2 : 1) void bwd_reduce_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ y,
    const uint16_t *__restrict__ g, const uint16_t *__restrict__ gh,
    const u32x4 *__restrict__ Wp, int C, int M, int64_t T, float *__restrict__ u_raw,
    float *__restrict__ sumsq, float *__restrict__ gH_res, float *__restrict__ gH_post,
    float *__restrict__ gH_pre) {
  using Cfg = ReduceCfg<N, NT, WAVES>;
  constexpr int D = N * N + 2 * N;
  extern __shared__ u32x4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int64_t tw = static_cast<int64_t>(blockIdx.x) * (16 * WAVES) + wave * 16;
  int64_t tl = tw + r;
  if (tl > T - 1) tl = T - 1;
  const uint16_t *xr = x + tl * N * C + q * 8;
  const uint16_t *gr = g + tl * N * C + q * 8;
  const uint16_t *yr = y + tl * C + q * 8;
  const uint16_t *hr = gh + tl * C + q * 8;
  const int ncs = C / 64;   // 64-column steps; also per-stream stride of W in such steps

  struct Tile { u32x4 X[N][2], G[N][2], Y[2], H[2]; };
  u32x4 wst[Cfg::WV];
  f32x4 acc[NT], ss = f32x4{0.f, 0.f, 0.f, 0.f};
  float dots[D];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < D; ++e) dots[e] = 0.f;

  auto load_tile = [&](Tile &tile, int cs) {
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        tile.X[j][u] = *reinterpret_cast<const u32x4 *>(xr + j * C + cs * 64 + u * 32);
        tile.G[j][u] = *reinterpret_cast<const u32x4 *>(gr + j * C + cs * 64 + u * 32);
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      tile.Y[u] = *reinterpret_cast<const u32x4 *>(yr + cs * 64 + u * 32);
      tile.H[u] = *reinterpret_cast<const u32x4 *>(hr + cs * 64 + u * 32);
    }
  };
  // W blocks of step cs: for stream j the 2 K steps 2 (j ncs + cs) + u, NT tiles, hi/lo
  auto load_w = [&](int cs) {
#pragma unroll
    for (int i = 0; i < Cfg::WV; ++i) {
      int e = i * Cfg::kThreads + threadIdx.x;
      if (e > Cfg::kStageVec - 1) e = Cfg::kStageVec - 1;   // surplus threads repeat the last one
      const int j = e / (NT * 256), rem = e % (NT * 256);
      wst[i] = Wp[static_cast<size_t>(j * ncs + cs) * (NT * 256) + rem];
    }
  };
  auto store_w = [&](int buf) {
#pragma unroll
    for (int i = 0; i < Cfg::WV; ++i) {
      int e = i * Cfg::kThreads + threadIdx.x;
      if (e > Cfg::kStageVec - 1) e = Cfg::kStageVec - 1;
      lds[buf * Cfg::kStageVec + e] = wst[i];
    }
  };
  auto compute = [&](const Tile &tile, int buf) {
    const u32x4 *wb = lds + buf * Cfg::kStageVec;
#pragma unroll
    for (int j = 0; j < N; ++j) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
          acc[jt] = mfma16(tile.X[j][u], wb[(((j * 2 + u) * NT + jt) * 2 + 0) * 64 + lane], acc[jt]);
          acc[jt] = mfma16(tile.X[j][u], wb[(((j * 2 + u) * NT + jt) * 2 + 1) * 64 + lane], acc[jt]);
        }
        ss = mfma16(tile.X[j][u], tile.X[j][u], ss);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int i = 0; i < N; ++i)
          dots[i * N + j] = dot8_bf16(tile.G[i][u], tile.X[j][u], dots[i * N + j]);
        dots[N * N + j] = dot8_bf16(tile.G[j][u], tile.Y[u], dots[N * N + j]);
        dots[N * N + N + j] = dot8_bf16(tile.H[u], tile.X[j][u], dots[N * N + N + j]);
      }
      // keeps the W operands of one stream at a time in registers
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // One tile at a time per wave; the block's second resident copy and the other
  // waves keep HBM busy while this wave computes.  Per step: request W of the
  // next step, then this step's stream tile; park W in the idle LDS buffer as
  // soon as it is there (loads return in order, the tile stays in flight);
  // then compute on the tile.  The barrier both publishes the new W buffer and
  // frees the one just read.
  // Each block starts its walk along the rows at another column step (the sums are then
  // taken in a rotated order): with every block at the same columns at the same time, all
  // requests differ only in address bits above the row length and crowd a few memory
  // channels (0.62 -> 0.52 ms at n = 4, C = 4096; W, 2 MiB, stays in L2 either way).
  const int rot = static_cast<int>((blockIdx.x * 13u) % static_cast<unsigned>(ncs));
  auto turn = [&](int c) { const int v = c + rot; return v >= ncs ? v - ncs : v; };
  load_w(turn(0));
  store_w(0);
  __syncthreads();
  if constexpr (WAVES == 8 && N >= 4) {
    // One block per CU: nothing else keeps HBM busy while the block's waves, held in step by the
    // barrier, compute.  So the NEXT step's tile is requested before this step's arithmetic
    // (two tiles in registers); requests go out in the order W(next), tile(next), so that parking
    // W in LDS waits for the W loads alone and computing on the current tile waits for nothing.
    Tile ta, tb2;
    load_tile(ta, turn(0));
    auto step = [&](const Tile &cur, Tile &nxt, int cs) {
      const int nx = cs + 1 < ncs ? cs + 1 : cs;   // the last step re-requests itself (unused)
      load_w(turn(nx));
      load_tile(nxt, turn(nx));
      __builtin_amdgcn_sched_barrier(0);
      store_w((cs + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      compute(cur, cs & 1);
      __syncthreads();
    };
    int cs = 0;
    for (; cs + 1 < ncs; cs += 2) {
      step(ta, tb2, cs);
      step(tb2, ta, cs + 1);
    }
    if (cs < ncs) step(ta, tb2, cs);
  } else {
    Tile tile;
    for (int cs = 0; cs < ncs; ++cs) {
      const int nx = cs + 1 < ncs ? cs + 1 : cs;   // last step re-stages itself (unused)
      load_w(turn(nx));
      load_tile(tile, turn(cs));
      __builtin_amdgcn_sched_barrier(0);
      store_w((cs + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      compute(tile, cs & 1);
      __syncthreads();
    }
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t t = tw + 4 * q + i;
    if (t < T) {
#pragma unroll
      for (int jt = 0; jt < NT; ++jt) {
        const int col = 16 * jt + r;
        if (col < M) u_raw[t * M + col] = acc[jt][i];
      }
    }
  }
  const int64_t t = tw + r;
  if ((r >> 2) == q) {
    const int i = r & 3;
    const float v = i == 0 ? ss[0] : (i == 1 ? ss[1] : (i == 2 ? ss[2] : ss[3]));
    if (t < T) sumsq[t] = v;
  }
  // the four lanes (q = 0..3) of a token hold disjoint column subsets
#pragma unroll
  for (int e = 0; e < D; ++e) {
    dots[e] += __shfl_xor(dots[e], 16, 64);
    dots[e] += __shfl_xor(dots[e], 32, 64);
  }
  if (q == 0 && t < T) {
#pragma unroll
    for (int e = 0; e < N * N; ++e) gH_res[t * N * N + e] = dots[e];
#pragma unroll
    for (int i = 0; i < N; ++i) {
      gH_post[t * N + i] = dots[N * N + i];
      gH_pre[t * N + i] = dots[N * N + N + i];
    }
  }
}

// ---------------------------------------------------------------------------
// The dot products of pass 1 alone (wide case, where the projection runs in
// proj_mfma_kernel): g_H_res, g_H_post, g_H_pre from one read of x, g_xout, y, g_h.
// Same tiles, lane ownership and v_dot2_f32_bf16 arithmetic as bwd_reduce_kernel; no
// W, no LDS, no barrier.  Block = 4 waves x 16 tokens.
template <int N>
__global__ __launch_bounds__(256) void bwd_dots_fast_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ y,
    const uint16_t *__restrict__ g, const uint16_t *__restrict__ gh, int C, int64_t T,
    float *__restrict__ gH_res, float *__restrict__ gH_post, float *__restrict__ gH_pre) {
  constexpr int D = N * N + 2 * N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int64_t tw = static_cast<int64_t>(blockIdx.x) * 64 + wave * 16;
  int64_t tl = tw + r;
  if (tl > T - 1) tl = T - 1;
  const uint16_t *xr = x + tl * N * C + q * 8;
  const uint16_t *gr = g + tl * N * C + q * 8;
  const uint16_t *yr = y + tl * C + q * 8;
  const uint16_t *hr = gh + tl * C + q * 8;
  const int ncs = C / 64;
  float dots[D];
#pragma unroll
  for (int e = 0; e < D; ++e) dots[e] = 0.f;
  const int rot = static_cast<int>((blockIdx.x * 13u) % static_cast<unsigned>(ncs));   // as in bwd_reduce_kernel
  for (int cl = 0; cl < ncs; ++cl) {
    const int cs = cl + rot >= ncs ? cl + rot - ncs : cl + rot;
    u32x4 X[N][2], G[N][2], Y[2], H[2];
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        X[j][u] = *reinterpret_cast<const u32x4 *>(xr + j * C + cs * 64 + u * 32);
        G[j][u] = *reinterpret_cast<const u32x4 *>(gr + j * C + cs * 64 + u * 32);
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      Y[u] = *reinterpret_cast<const u32x4 *>(yr + cs * 64 + u * 32);
      H[u] = *reinterpret_cast<const u32x4 *>(hr + cs * 64 + u * 32);
    }
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int i = 0; i < N; ++i) dots[i * N + j] = dot8_bf16(G[i][u], X[j][u], dots[i * N + j]);
        dots[N * N + j] = dot8_bf16(G[j][u], Y[u], dots[N * N + j]);
        dots[N * N + N + j] = dot8_bf16(H[u], X[j][u], dots[N * N + N + j]);
      }
  }
  // the four lanes (q = 0..3) of a token hold disjoint column subsets
#pragma unroll
  for (int e = 0; e < D; ++e) {
    dots[e] += __shfl_xor(dots[e], 16, 64);
    dots[e] += __shfl_xor(dots[e], 32, 64);
  }
  const int64_t t = tw + r;
  if (q == 0 && t < T) {
#pragma unroll
    for (int e = 0; e < N * N; ++e) gH_res[t * N * N + e] = dots[e];
#pragma unroll
    for (int i = 0; i < N; ++i) {
      gH_post[t * N + i] = dots[N * N + i];
      gH_pre[t * N + i] = dots[N * N + N + i];
    }
  }
}

// ---------------------------------------------------------------------------
// Per-token stage between the two backward passes: coefficients (recomputed),
// g_z, and the operands pass 2 needs, in the layouts its MFMAs read:
//   cpk  [T][CP] f32 : H_res (N*N) | H_pre (N) | H_post (N) | coefx
//   vr   [Tpad][MP32] bf16 hi, lo : vr = r alpha g_z, row per token
//   vrT  [Tpad/32][MP16][32] bf16 hi, lo : the same, tokens innermost
//   gzs  [Tpad/64][M+3] f32 : per 64 tokens, the sums of g_z and of the per-group
//        g_z u (what g_b and g_alpha are summed from), in a fixed butterfly order
// Tokens T..Tpad-1 get zero vr so that padded tiles add nothing to g_W.
// One wave per block, one token per lane.
// F16ROWS (the single-kernel wide pass 2): the vr ROWS hold fp16 hi, lo parts of
// vr / s with s = max_m |vr_m| of the token (1 if that is 0), so that any gradient
// scale fits fp16; s goes to cpk[N*N + 2N + 1].  vrT stays bf16 in either case.
template <int N, int MODE, bool F16ROWS>
__global__ __launch_bounds__(64) void bwd_epilogue_fast_kernel(
    const float *__restrict__ u_raw, const float *__restrict__ sumsq, int parts,
    const float *__restrict__ b, const float *__restrict__ alpha, const float *__restrict__ gH_res,
    const float *__restrict__ gH_pre, const float *__restrict__ gH_post, int nC, float eps,
    int sk_iters, int64_t T, int CP, float *__restrict__ cpk, uint16_t *__restrict__ vr_hi,
    uint16_t *__restrict__ vr_lo, uint16_t *__restrict__ vrT_hi, uint16_t *__restrict__ vrT_lo,
    float *__restrict__ gz_sums) {
  constexpr int R = Dims<N, MODE>::R, M = Dims<N, MODE>::M;
  constexpr int MP32 = (M + 31) / 32 * 32, MP16 = (M + 15) / 16 * 16;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 64 + threadIdx.x;   // < Tpad
  const int64_t blk = t >> 5;
  const int tin = static_cast<int>(t & 31);
  const bool live = t < T;
  const int64_t tl = live ? t : T - 1;   // padded lanes recompute the last token and discard it
  float u[M], a[R], Hr[N * N], Hp[N], Hq[N], gz[M + 3];
  float gr[N * N], gp[N], gq[N];
  float sums[(MODE == MHCL_RES_SK) ? 2 * kMaxSkIters * N : 1];
  float ssq = sumsq[tl];
#pragma unroll
  for (int m = 0; m < M; ++m) u[m] = u_raw[tl * M + m];
  for (int pt = 1; pt < parts; ++pt) {   // K-split slices of the projection, added in order
    ssq += sumsq[pt * T + tl];
#pragma unroll
    for (int m = 0; m < M; ++m) u[m] += u_raw[(pt * T + tl) * M + m];
  }
#pragma unroll
  for (int e = 0; e < N * N; ++e) gr[e] = gH_res[tl * N * N + e];
#pragma unroll
  for (int j = 0; j < N; ++j) { gp[j] = gH_pre[tl * N + j]; gq[j] = gH_post[tl * N + j]; }
  const TokenParams p{alpha[0], alpha[1], alpha[2], eps, sk_iters};
  const float r = token_coeffs<N, MODE>(u, ssq, nC, b, p, Hr, Hp, Hq, a,
                                        (MODE == MHCL_RES_SK) ? sums : nullptr);
  if (live) {
    float *cp = cpk + t * CP;
#pragma unroll
    for (int e = 0; e < N * N; ++e) cp[e] = Hr[e];
#pragma unroll
    for (int j = 0; j < N; ++j) { cp[N * N + j] = Hp[j]; cp[N * N + N + j] = Hq[j]; }
  }
  token_coeffs_bwd<N, MODE>(gr, gp, gq, a, Hr, Hp, Hq, sums, sk_iters, gz);
  float ga[3] = {0.f, 0.f, 0.f}, dot = 0.f;
  uint32_t ph[MP32 / 2], pl[MP32 / 2];   // the token's vr row, two 16-bit parts per word
#pragma unroll
  for (int i = 0; i < MP32 / 2; ++i) { ph[i] = 0; pl[i] = 0; }
  float inv_s = 1.f;
  if constexpr (F16ROWS) {
    float vmax = 0.f;
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const int g = m < R ? 0 : (m < R + N ? 1 : 2);
      const float al = g == 0 ? p.alpha_res : (g == 1 ? p.alpha_pre : p.alpha_post);
      vmax = fmaxf(vmax, fabsf(r * al * (live ? gz[m] : 0.f)));
    }
    const float sc = vmax > 0.f ? vmax : 1.f;
    inv_s = 1.f / sc;
    if (live) cpk[t * CP + N * N + 2 * N + 1] = sc;
  }
#pragma unroll
  for (int m = 0; m < M; ++m) {
    const int g = m < R ? 0 : (m < R + N ? 1 : 2);
    const float al = g == 0 ? p.alpha_res : (g == 1 ? p.alpha_pre : p.alpha_post);
    if (!live) gz[m] = 0.f;
    const float vr = r * al * gz[m];
    ga[g] += gz[m] * (r * u[m]);
    dot += vr * u[m];
    uint16_t hi, lo;
    split_bf16(vr, hi, lo);
    vrT_hi[(blk * MP16 + m) * 32 + tin] = hi;
    vrT_lo[(blk * MP16 + m) * 32 + tin] = lo;
    if constexpr (F16ROWS) {
      const float vs = vr * inv_s;
      const _Float16 h16 = static_cast<_Float16>(vs);
      const _Float16 l16 = static_cast<_Float16>(vs - static_cast<float>(h16));
      hi = __builtin_bit_cast(uint16_t, h16);
      lo = __builtin_bit_cast(uint16_t, l16);
    }
    ph[m / 2] |= static_cast<uint32_t>(hi) << (16 * (m & 1));
    pl[m / 2] |= static_cast<uint32_t>(lo) << (16 * (m & 1));
  }
#pragma unroll
  for (int m = M; m < MP16; ++m) {
    vrT_hi[(blk * MP16 + m) * 32 + tin] = 0;
    vrT_lo[(blk * MP16 + m) * 32 + tin] = 0;
  }
  u32x4 *rh = reinterpret_cast<u32x4 *>(vr_hi + t * MP32);
  u32x4 *rl = reinterpret_cast<u32x4 *>(vr_lo + t * MP32);
#pragma unroll
  for (int i = 0; i < MP32 / 8; ++i) {
    rh[i] = u32x4{ph[4 * i], ph[4 * i + 1], ph[4 * i + 2], ph[4 * i + 3]};
    rl[i] = u32x4{pl[4 * i], pl[4 * i + 1], pl[4 * i + 2], pl[4 * i + 3]};
  }
  if (live) cpk[t * CP + N * N + 2 * N] = (r * r / static_cast<float>(nC)) * dot;
#pragma unroll
  for (int g = 0; g < 3; ++g) gz[M + g] = ga[g];   // zero for padded lanes
  // sum over the 64 tokens of the wave: butterfly, the same order in every run
#pragma unroll
  for (int m = 0; m < M + 3; ++m) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) gz[m] += __shfl_xor(gz[m], off, 64);
  }
  if (threadIdx.x == 0) {
#pragma unroll
    for (int m = 0; m < M + 3; ++m) gz_sums[static_cast<int64_t>(blockIdx.x) * (M + 3) + m] = gz[m];
  }
}

// ---------------------------------------------------------------------------
// Backward pass 2 (n <= 4): the stream outputs AND g_W from one read of x.
//   g_x[j] = sum_i H_res[i][j] g_xout[i] + H_pre[j] g_h + (W vr)[j] - x[j] coefx
//   g_y    = sum_i H_post[i] g_xout[i]
// summed in fp32 and rounded to bf16 once.  A block owns one 64-column step of C
// (all n streams) and a chunk of tokens; its slice of W (A layout, hi + lo)
// sits in LDS for the whole walk.  A lane owns 2 x 8 columns of its token
// (columns 32 u + 8 q + 0..7, u = 0, 1: four lanes read and write whole
// 128-byte lines in two back to back accesses).  (W vr) comes out of the MFMAs
// already in that ownership: lane (token, q), quarter h = 2 u + hh gets rows
// 32 u + 8 q + 4 hh + 0..3.
// Per block iteration the four waves load the tiles of 4 x 16 tokens, publish
// their x tiles in LDS, and wave w (one wave per stream) then accumulates the
// g_W rows of stream w for all 64 tokens:
//   D[m][k] += vrT[m][token] * x^T[token][k]
// with x^T obtained by an MFMA against a 0/1 selection matrix (exact) as in
// bwd_gw_kernel.  Accumulators stay in registers over the block's token chunk;
// partial sums per chunk go to `gw_part` and are added in chunk order.
template <int N, int NT, int SLABS>
__global__ __launch_bounds__(256 * SLABS, SLABS == 1 ? 2 : 1) void bwd_out_gw_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ g,
    const uint16_t *__restrict__ gh, const u32x4 *__restrict__ Wa, const float *__restrict__ cpk,
    const uint16_t *__restrict__ vr_hi, const uint16_t *__restrict__ vr_lo,
    const uint16_t *__restrict__ vrT_hi, const uint16_t *__restrict__ vrT_lo, int MP16, int M, int C,
    int64_t T, int tokens_per_block, int CP, uint16_t *__restrict__ g_x,
    uint16_t *__restrict__ g_y, float *__restrict__ gw_part) {
  constexpr int NCP = N * N + 2 * N + 1;
  constexpr int NCP4 = (NCP + 3) / 4;
  constexpr int kSliceVec = N * 4 * 2 * 64;   // 16-byte words of W per 64-column step
  // SLABS adjacent 64-column steps per block, four waves each, all on the same tokens at
  // the same time: a row visit of the block then covers SLABS x 128 contiguous bytes
  extern __shared__ u32x4 lds_all[];
  const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3, slab = threadIdx.x >> 8;
  u32x4 *lds = lds_all + slab * (2 * kSliceVec);
  u32x4 *xch = lds + kSliceVec;               // x tiles of one iteration: [stream][wave][u][lane]
  const int r = lane & 15, q = lane >> 4;
  const int S = blockIdx.x * SLABS + slab;
  const int c0 = S * 64 + q * 8;
  const int nS = C / 64;
  for (int e = threadIdx.x & 255; e < kSliceVec; e += 256) {
    const int j = e / 512, rem = e % 512;
    lds[e] = Wa[static_cast<size_t>(j * nS + S) * 512 + rem];
  }
  const u32x4 *wl = lds + lane;

  const int64_t tb = static_cast<int64_t>(blockIdx.y) * tokens_per_block;   // multiple of 64
  int64_t te = tb + tokens_per_block;
  if (te > T) te = T;

  u32x4 sel[2];   // selection operands: column c of half h picks row 16 h + c
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int k0 = 8 * q + 2 * e2, k1 = k0 + 1;
      w[e2] = (k0 == 16 * h + r ? 0x3F80u : 0u) | (k1 == 16 * h + r ? 0x3F800000u : 0u);
    }
    sel[h] = u32x4{w[0], w[1], w[2], w[3]};
  }
  f32x4 acc[2][2][NT];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int mt = 0; mt < NT; ++mt) acc[u][h][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto unpack = [](const u32x4 &v, float (&o)[8]) {
    o[0] = bf16lo(v.x); o[1] = bf16hi(v.x); o[2] = bf16lo(v.y); o[3] = bf16hi(v.y);
    o[4] = bf16lo(v.z); o[5] = bf16hi(v.z); o[6] = bf16lo(v.w); o[7] = bf16hi(v.w);
  };
  auto pack = [](const float (&o)[8]) {
    u32x4 v;
    v.x = cvt_pk_bf16(o[0], o[1]); v.y = cvt_pk_bf16(o[2], o[3]);
    v.z = cvt_pk_bf16(o[4], o[5]); v.w = cvt_pk_bf16(o[6], o[7]);
    return v;
  };

  struct In {
    u32x4 X[N][2], G[N][2], H[2], vbh, vbl;
    float4 cp[NCP4];
  };
  auto load_x = [&](In &in, int64_t t0) {
    int64_t tl = t0 + r;
    if (tl > te - 1) tl = te - 1;
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u)
        in.X[j][u] = *reinterpret_cast<const u32x4 *>(x + (tl * N + j) * C + c0 + u * 32);
  };
  auto load_rest = [&](In &in, int64_t t0) {
    int64_t tl = t0 + r;
    if (tl > te - 1) tl = te - 1;
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u)
        in.G[j][u] = *reinterpret_cast<const u32x4 *>(g + (tl * N + j) * C + c0 + u * 32);
#pragma unroll
    for (int u = 0; u < 2; ++u)
      in.H[u] = *reinterpret_cast<const u32x4 *>(gh + tl * C + c0 + u * 32);
    in.vbh = *reinterpret_cast<const u32x4 *>(vr_hi + tl * 32 + q * 8);
    in.vbl = *reinterpret_cast<const u32x4 *>(vr_lo + tl * 32 + q * 8);
    const float4 *cpp = reinterpret_cast<const float4 *>(cpk + tl * CP);
#pragma unroll
    for (int e = 0; e < NCP4; ++e) in.cp[e] = cpp[e];
  };
  auto process = [&](const In &in, int64_t t0) {
    const int64_t t = t0 + r;
    const bool live = t < te;
    float cp[NCP4 * 4];
#pragma unroll
    for (int e = 0; e < NCP4; ++e) {
      cp[4 * e] = in.cp[e].x; cp[4 * e + 1] = in.cp[e].y;
      cp[4 * e + 2] = in.cp[e].z; cp[4 * e + 3] = in.cp[e].w;
    }
    const float cx = cp[N * N + 2 * N];
    float gv[2][N][8], hv[2][8];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int i = 0; i < N; ++i) unpack(in.G[i][u], gv[u][i]);
      unpack(in.H[u], hv[u]);
    }
    if (g_y != nullptr) {   // (optional output)
      u32x4 ov[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float sacc = 0.f;
#pragma unroll
          for (int i = 0; i < N; ++i) sacc += cp[N * N + N + i] * gv[u][i][e];
          o[e] = sacc;
        }
        ov[u] = pack(o);
      }
      if (live) {
        *reinterpret_cast<u32x4 *>(g_y + t * C + c0) = ov[0];
        *reinterpret_cast<u32x4 *>(g_y + t * C + c0 + 32) = ov[1];
      }
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
      u32x4 ov[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        f32x4 wv[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int h = 2 * u + hh;
          const u32x4 wh = wl[((j * 4 + h) * 2 + 0) * 64], wlo = wl[((j * 4 + h) * 2 + 1) * 64];
          wv[hh] = mfma16(wh, in.vbh, f32x4{0.f, 0.f, 0.f, 0.f});
          wv[hh] = mfma16(wlo, in.vbh, wv[hh]);
          wv[hh] = mfma16(wh, in.vbl, wv[hh]);
        }
        float xv[8], o[8];
        unpack(xch[((j * 4 + wave) * 2 + u) * 64 + lane], xv);   // this wave's own tile, parked in LDS
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float sacc = wv[e >> 2][e & 3] - xv[e] * cx;
#pragma unroll
          for (int i = 0; i < N; ++i) sacc += cp[i * N + j] * gv[u][i][e];
          sacc += cp[N * N + j] * hv[u][e];
          o[e] = sacc;
        }
        ov[u] = pack(o);
      }
      if (live) {
        *reinterpret_cast<u32x4 *>(g_x + (t * N + j) * C + c0) = ov[0];
        *reinterpret_cast<u32x4 *>(g_x + (t * N + j) * C + c0 + 32) = ov[1];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // g_W rows of stream `wave` from the 64 tokens whose x tiles sit in LDS.  The vrT operands
  // (two 32-token blocks: wave pairs (0,1) and (2,3)) are fetched by gw_fetch, which the main
  // loop issues BEFORE the next iteration's x tiles: loads return in order, so requested after
  // them these small L2 hits would wait for a whole HBM round trip.
  auto gw_fetch = [&](int64_t t0blk, u32x4 (&va)[2][NT][2]) {
    const int64_t blk0 = t0blk >> 5;
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
#pragma unroll
      for (int mt = 0; mt < NT; ++mt) {
        const size_t row = (static_cast<size_t>(blk0 + pr) * MP16 + mt * 16 + r) * 32;
        const u32x2 h0 = *reinterpret_cast<const u32x2 *>(vrT_hi + row + 4 * q);
        const u32x2 h1 = *reinterpret_cast<const u32x2 *>(vrT_hi + row + 16 + 4 * q);
        const u32x2 l0 = *reinterpret_cast<const u32x2 *>(vrT_lo + row + 4 * q);
        const u32x2 l1 = *reinterpret_cast<const u32x2 *>(vrT_lo + row + 16 + 4 * q);
        va[pr][mt][0] = u32x4{h0.x, h0.y, h1.x, h1.y};
        va[pr][mt][1] = u32x4{l0.x, l0.y, l1.x, l1.y};
      }
    }
  };
  auto gw_accumulate = [&](const u32x4 (&va)[2][NT][2]) {
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {   // one 32-token block each
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const u32x4 xa = xch[((wave * 4 + 2 * pr + 0) * 2 + u) * 64 + lane];
        const u32x4 xb = xch[((wave * 4 + 2 * pr + 1) * 2 + u) * 64 + lane];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
          const f32x4 ta = mfma16(xa, sel[h], z);   // tokens 4q+i of the pair's first 16
          const f32x4 tb2 = mfma16(xb, sel[h], z);  // tokens 4q+i of its second 16
          u32x4 bt;
          bt.x = cvt_pk_bf16(ta[0], ta[1]); bt.y = cvt_pk_bf16(ta[2], ta[3]);
          bt.z = cvt_pk_bf16(tb2[0], tb2[1]); bt.w = cvt_pk_bf16(tb2[2], tb2[3]);
#pragma unroll
          for (int mt = 0; mt < NT; ++mt) {
            acc[u][h][mt] = mfma16(va[pr][mt][0], bt, acc[u][h][mt]);
            acc[u][h][mt] = mfma16(va[pr][mt][1], bt, acc[u][h][mt]);
          }
        }
      }
    }
  };

  // Per iteration: the x tiles go to LDS as soon as they arrive, which frees
  // their registers for the NEXT iteration's x tiles; those are requested right
  // away and fly while this iteration's g_W and mixing work runs.
  In in;
  const int niter = static_cast<int>((te - tb + 63) / 64);   // same for all four waves
  load_x(in, tb + wave * 16);
  for (int it = 0; it < niter; ++it) {
    const int64_t t0 = tb + static_cast<int64_t>(it) * 64 + wave * 16;
    load_rest(in, t0);
    __syncthreads();   // everyone is done with the previous iteration's x tiles (and W is staged)
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) xch[((j * 4 + wave) * 2 + u) * 64 + lane] = in.X[j][u];
    __syncthreads();
    u32x4 va[2][NT][2];
    if (wave < N) gw_fetch(tb + static_cast<int64_t>(it) * 64, va);
    __builtin_amdgcn_sched_barrier(0);
    load_x(in, t0 + 64);   // clamped to the block's last token when past the end
    __builtin_amdgcn_sched_barrier(0);
    if (wave < N) gw_accumulate(va);
    __builtin_amdgcn_sched_barrier(0);
    process(in, t0);
  }

  if (wave < N) {
    float *dst = gw_part + static_cast<size_t>(blockIdx.y) * (static_cast<size_t>(N) * C) * M;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = wave * C + S * 64 + u * 32 + 16 * h + r;
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + 4 * q + i;
            if (m < M) dst[static_cast<size_t>(k) * M + m] = acc[u][h][mt][i];
          }
      }
  }
}

// ---------------------------------------------------------------------------
// Wide case (more than 32 logits, n = 5): the W slice of a 64-column step no
// longer fits on chip next to the stream tiles, so pass 2 is split in two.
// First D[t][k] = (W vr_t)[k] as a plain MFMA product with the W rows of one
// 64-row step resident in LDS (A layout, MS logit steps, hi + lo) and the
// per-token vectors vr as B operands; D is fp32 [T, nC] in the workspace.
template <int MS>
__global__ __launch_bounds__(256, 2) void wv_kernel(const u32x4 *__restrict__ Wa,
                                                    const uint16_t *__restrict__ vr_hi,
                                                    const uint16_t *__restrict__ vr_lo, int MP32,
                                                    int K, int64_t T, int tokens_per_block,
                                                    float *__restrict__ D) {
  constexpr int kSliceVec = 4 * MS * 2 * 64;
  extern __shared__ u32x4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int S = blockIdx.x;
  for (int e = threadIdx.x; e < kSliceVec; e += 256) lds[e] = Wa[static_cast<size_t>(S) * kSliceVec + e];
  __syncthreads();
  const u32x4 *wl = lds + lane;
  const int64_t tb = static_cast<int64_t>(blockIdx.y) * tokens_per_block;
  int64_t te = tb + tokens_per_block;
  if (te > T) te = T;
  for (int64_t t0 = tb + wave * 16; t0 < te; t0 += 64) {
    const int64_t t = t0 + r;
    const bool live = t < te;
    const int64_t tl = live ? t : te - 1;
    u32x4 vbh[MS], vbl[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
      vbh[ms] = *reinterpret_cast<const u32x4 *>(vr_hi + tl * MP32 + ms * 32 + q * 8);
      vbl[ms] = *reinterpret_cast<const u32x4 *>(vr_lo + tl * MP32 + ms * 32 + q * 8);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      f32x4 acc[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int h = 2 * u + hh;
        acc[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
          const u32x4 wh = wl[((h * MS + ms) * 2 + 0) * 64], wlo = wl[((h * MS + ms) * 2 + 1) * 64];
          acc[hh] = mfma16(wh, vbh[ms], acc[hh]);
          acc[hh] = mfma16(wlo, vbh[ms], acc[hh]);
          acc[hh] = mfma16(wh, vbl[ms], acc[hh]);
        }
      }
      if (live) {   // rows 64 S + 32 u + 8 q + 0..7 of token t
        float4 *dst = reinterpret_cast<float4 *>(D + t * K + 64 * S + 32 * u + 8 * q);
        dst[0] = make_float4(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
        dst[1] = make_float4(acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
      }
    }
  }
}

// Pass 2 of the wide case in one kernel, for slices that fit on chip when W is kept
// as ONE 16-bit part (n = 5, 130 logits: 100 KiB per 64-column step; the bf16 pair would be 200):
//   g_x[j] = sum_i H_res[i][j] g_xout[i] + H_pre[j] g_h + (W16 vr)[j] - x[j] coefx
//   g_y    = sum_i H_post[i] g_xout[i]
// W16 = fp16(W * 2^k) (11 significant bits; the power of two is chosen per call from max |W|,
// so weights of any magnitude fit), and vr enters as fp16 hi + lo parts of vr / s with the
// token's own scale s (F16ROWS of the per-token stage), so gradients of any magnitude fit; the
// MFMA result is multiplied by s / 2^k.  Rounding W to fp16 changes (W vr) by about 2^-12 of its
// size, far below the rounding of g_x to bf16 that follows.  Nothing is written between
// the passes (the two-kernel variant stores W vr as fp32 [T, nC] and reads it back).
// One block of eight waves per CU, each wave 16 tokens per iteration; lane ownership
// as in bwd_out_gw_kernel.
// The per-token coefficient record (n^2 + 2n + 2 floats, 82 at n = 8) does not fit the
// registers next to the stream tiles, so each wave parks the records of its 16 tokens
// in its own LDS region and reads the column of H_res it needs stream by stream.
// LDS: N x MS x 4 KiB of W16 plus 8 x 16 x (CP + 4) floats; the launcher falls back to
// the two-kernel form when that exceeds 160 KiB.
template <int N, int MS>
struct OutW16Cfg {
  static constexpr int kStreamVec = 4 * MS * 64;
  static constexpr int CP = (N * N + 2 * N + 2 + 7) / 8 * 8;   // as FastBwdWs::CP
  static constexpr int CPS = CP + 4;                           // LDS row stride (floats)
  static constexpr int kLdsBytes = N * kStreamVec * 16 + 8 * 16 * CPS * 4;
  static constexpr bool kFits = kLdsBytes <= 160 * 1024;
};

template <int N, int MS>
__global__ __launch_bounds__(512, 1) void bwd_out_w16_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ g,
    const uint16_t *__restrict__ gh, const u32x4 *__restrict__ Wa, const float *__restrict__ cpk,
    const uint16_t *__restrict__ vr_hi, const uint16_t *__restrict__ vr_lo,
    const float *__restrict__ wscale, int MP32, int C,
    int64_t T, int tokens_per_block, uint16_t *__restrict__ g_x, uint16_t *__restrict__ g_y) {
  using Cfg = OutW16Cfg<N, MS>;
  constexpr int NN = N * N, CP = Cfg::CP, CPS = Cfg::CPS, CP4 = CP / 4;
  constexpr int kStreamVec = Cfg::kStreamVec;
  constexpr int NV = (16 * CP4 + 63) / 64;     // float4 of the records each lane fetches
  extern __shared__ u32x4 lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int S = blockIdx.x;
  const int c0 = S * 64 + q * 8;
  const int nS = C / 64;
  for (int e = threadIdx.x; e < N * kStreamVec; e += 512) {
    const int j = e / kStreamVec, rem = e % kStreamVec;
    const int blk = rem >> 6, ln = rem & 63;     // blk = h * MS + ms of step j nS + S
    lds[e] = Wa[(static_cast<size_t>(j * nS + S) * 4 * MS + blk) * 64 + ln];
  }
  __syncthreads();
  const u32x4 *wl = lds + lane;
  const float inv_wscale = wscale[1];
  float *cps = reinterpret_cast<float *>(lds + N * kStreamVec) + wave * 16 * CPS;   // this wave's records
  const float *cpr = cps + r * CPS;                                                 // this lane's token

  const int64_t tb = static_cast<int64_t>(blockIdx.y) * tokens_per_block;   // multiple of 128
  int64_t te = tb + tokens_per_block;
  if (te > T) te = T;

  auto unpack = [](const u32x4 &v, float (&o)[8]) {
    o[0] = bf16lo(v.x); o[1] = bf16hi(v.x); o[2] = bf16lo(v.y); o[3] = bf16hi(v.y);
    o[4] = bf16lo(v.z); o[5] = bf16hi(v.z); o[6] = bf16lo(v.w); o[7] = bf16hi(v.w);
  };
  auto pack = [](const float (&o)[8]) {
    u32x4 v;
    v.x = cvt_pk_bf16(o[0], o[1]); v.y = cvt_pk_bf16(o[2], o[3]);
    v.z = cvt_pk_bf16(o[4], o[5]); v.w = cvt_pk_bf16(o[6], o[7]);
    return v;
  };

  for (int64_t t0 = tb + wave * 16; t0 < te; t0 += 128) {
    const int64_t t = t0 + r;
    const bool live = t < te;
    const int64_t tl = live ? t : te - 1;
    u32x4 X[N][2], G[N][2], H[2], vbh[MS], vbl[MS];
    float4 rec[NV];
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        G[j][u] = *reinterpret_cast<const u32x4 *>(g + (tl * N + j) * C + c0 + u * 32);
        X[j][u] = *reinterpret_cast<const u32x4 *>(x + (tl * N + j) * C + c0 + u * 32);
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) H[u] = *reinterpret_cast<const u32x4 *>(gh + tl * C + c0 + u * 32);
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
      vbh[ms] = *reinterpret_cast<const u32x4 *>(vr_hi + tl * MP32 + ms * 32 + q * 8);
      vbl[ms] = *reinterpret_cast<const u32x4 *>(vr_lo + tl * MP32 + ms * 32 + q * 8);
    }
    // the 16 records of the wave's tokens, CP4 float4 each, spread over the lanes
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int idx = lane + 64 * i;
      if (idx > 16 * CP4 - 1) idx = 16 * CP4 - 1;   // surplus lanes repeat the last piece
      const int tk = idx / CP4, part = idx - tk * CP4;
      int64_t tt = t0 + tk;
      if (tt > te - 1) tt = te - 1;
      rec[i] = *reinterpret_cast<const float4 *>(cpk + tt * CP + 4 * part);
    }
    __builtin_amdgcn_wave_barrier();   // (LDS requests of a wave are served in order)
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int idx = lane + 64 * i;
      if (idx > 16 * CP4 - 1) idx = 16 * CP4 - 1;
      const int tk = idx / CP4, part = idx - tk * CP4;
      *reinterpret_cast<float4 *>(cps + tk * CPS + 4 * part) = rec[i];
    }
    __builtin_amdgcn_wave_barrier();
    // W16 holds W * wscale[0] and the vr rows hold vr / (the token's scale): undo both
    const float cx = cpr[NN + 2 * N], vscale = cpr[NN + 2 * N + 1] * inv_wscale;
    float hq[N];
#pragma unroll
    for (int i = 0; i < N; ++i) hq[i] = cpr[NN + N + i];
    if constexpr (N <= 5) {
      // Stream by stream, both 64-byte halves of a line computed and stored together; the
      // g_xout and g_h tiles stay packed and are unpacked at each use (registers).
      if (g_y != nullptr) {   // (optional output)
        u32x4 ov[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
          for (int i = 0; i < N; ++i) {
            float gv[8];
            unpack(G[i][u], gv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += hq[i] * gv[e];
          }
          ov[u] = pack(o);
        }
        if (live) {
          *reinterpret_cast<u32x4 *>(g_y + t * C + c0) = ov[0];
          *reinterpret_cast<u32x4 *>(g_y + t * C + c0 + 32) = ov[1];
        }
      }
#pragma unroll
      for (int j = 0; j < N; ++j) {
        float hr[N];
#pragma unroll
        for (int i = 0; i < N; ++i) hr[i] = cpr[i * N + j];
        const float hp = cpr[NN + j];
        u32x4 ov[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          f32x4 wv[2];
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const int h = 2 * u + hh;
            wv[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
              const u32x4 wh = wl[((j * 4 + h) * MS + ms) * 64];
              wv[hh] = mfma16h(wh, vbh[ms], wv[hh]);
              wv[hh] = mfma16h(wh, vbl[ms], wv[hh]);
            }
          }
          float xv[8], hv[8], o[8];
          unpack(X[j][u], xv);
          unpack(H[u], hv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = vscale * wv[e >> 2][e & 3] - xv[e] * cx + hp * hv[e];
#pragma unroll
          for (int i = 0; i < N; ++i) {
            float gv[8];
            unpack(G[i][u], gv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += hr[i] * gv[e];
          }
          ov[u] = pack(o);
        }
        if (live) {
          *reinterpret_cast<u32x4 *>(g_x + (t * N + j) * C + c0) = ov[0];
          *reinterpret_cast<u32x4 *>(g_x + (t * N + j) * C + c0 + 32) = ov[1];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      // One 64-byte half of the lines at a time: the g_xout tile of that half is unpacked
      // once and serves g_y and all n output streams (unpacking per stream made the kernel
      // ALU bound at n = 8).
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float gv[N][8], hv[8];
#pragma unroll
        for (int i = 0; i < N; ++i) unpack(G[i][u], gv[i]);
        unpack(H[u], hv);
        if (g_y != nullptr) {   // (optional output)
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
          for (int i = 0; i < N; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += hq[i] * gv[i][e];
          if (live) *reinterpret_cast<u32x4 *>(g_y + t * C + c0 + 32 * u) = pack(o);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) {
          f32x4 wv[2];
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const int h = 2 * u + hh;
            wv[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
              const u32x4 wh = wl[((j * 4 + h) * MS + ms) * 64];
              wv[hh] = mfma16h(wh, vbh[ms], wv[hh]);
              wv[hh] = mfma16h(wh, vbl[ms], wv[hh]);
            }
          }
          const float hp = cpr[NN + j];
          float xv[8], o[8];
          unpack(X[j][u], xv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = vscale * wv[e >> 2][e & 3] - xv[e] * cx + hp * hv[e];
#pragma unroll
          for (int i = 0; i < N; ++i) {
            const float hr = cpr[i * N + j];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += hr * gv[i][e];
          }
          if (live) *reinterpret_cast<u32x4 *>(g_x + (t * N + j) * C + c0 + 32 * u) = pack(o);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();   // the records are overwritten in the next iteration
  }
}

// Then the stream outputs in row order (one thread per 8 columns of a token):
//   g_x[j] = sum_i H_res[i][j] g_xout[i] + H_pre[j] g_h + D[j] - x[j] coefx
//   g_y    = sum_i H_post[i] g_xout[i]
template <int N>
__global__ __launch_bounds__(256) void mix_wide_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ g,
    const uint16_t *__restrict__ gh, const float *__restrict__ D, const float *__restrict__ cpk,
    int CP, int C, int64_t T, uint16_t *__restrict__ g_x, uint16_t *__restrict__ g_y) {
  const int vpr = C / 8;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= T * vpr) return;
  const int64_t t = idx / vpr;
  const int c = static_cast<int>(idx % vpr) * 8;
  const float *cp = cpk + t * CP;
  auto unpack = [](const u32x4 &v, float (&o)[8]) {
    o[0] = bf16lo(v.x); o[1] = bf16hi(v.x); o[2] = bf16lo(v.y); o[3] = bf16hi(v.y);
    o[4] = bf16lo(v.z); o[5] = bf16hi(v.z); o[6] = bf16lo(v.w); o[7] = bf16hi(v.w);
  };
  auto pack = [](const float (&o)[8]) {
    u32x4 v;
    v.x = cvt_pk_bf16(o[0], o[1]); v.y = cvt_pk_bf16(o[2], o[3]);
    v.z = cvt_pk_bf16(o[4], o[5]); v.w = cvt_pk_bf16(o[6], o[7]);
    return v;
  };
  float gv[N][8], hv[8];
#pragma unroll
  for (int i = 0; i < N; ++i)
    unpack(*reinterpret_cast<const u32x4 *>(g + (t * N + i) * C + c), gv[i]);
  unpack(*reinterpret_cast<const u32x4 *>(gh + t * C + c), hv);
  if (g_y != nullptr) {   // (optional output)
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float sacc = 0.f;
#pragma unroll
      for (int i = 0; i < N; ++i) sacc += cp[N * N + N + i] * gv[i][e];
      o[e] = sacc;
    }
    *reinterpret_cast<u32x4 *>(g_y + t * C + c) = pack(o);
  }
  const float cx = cp[N * N + 2 * N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    float xv[8], o[8];
    unpack(*reinterpret_cast<const u32x4 *>(x + (t * N + j) * C + c), xv);
    const float4 d0 = *reinterpret_cast<const float4 *>(D + (t * N + j) * C + c);
    const float4 d1 = *reinterpret_cast<const float4 *>(D + (t * N + j) * C + c + 4);
    const float dv[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float sacc = dv[e] - xv[e] * cx;
#pragma unroll
      for (int i = 0; i < N; ++i) sacc += cp[i * N + j] * gv[i][e];
      sacc += cp[N * N + j] * hv[e];
      o[e] = sacc;
    }
    *reinterpret_cast<u32x4 *>(g_x + (t * N + j) * C + c) = pack(o);
  }
}

// ---------------------------------------------------------------------------
// Backward pass 2b: g_W[k][m] = sum_t x_hat[t][k] vr[t][m], the one reduction
// over tokens.  A wave owns CSW K steps (32 rows of g_W each) and walks a chunk
// of tokens 32 at a time.  x arrives with tokens across lanes, but the
// contraction runs over tokens, so each x tile is first transposed by an MFMA
// against a 0/1 selection matrix (exact: the values are bf16), which leaves
// lane (k, q) holding 4 + 4 tokens of column k: the B operand of
//   D[m][k] += vrT[m][token] * x^T[token][k].
// Partial sums per token chunk go to `out`; they are added in chunk order.
template <int NT, int CSW>
__global__ __launch_bounds__(256, 2) void bwd_gw_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ vrT_hi,
    const uint16_t *__restrict__ vrT_lo, int K, int M, int MP16, int64_t T, int64_t nblk,
    int blks_per_chunk, float *__restrict__ out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int s0 = (blockIdx.x * 4 + wave) * CSW;     // first K step of this wave
  const int nsteps = K / 32;
  if (s0 >= nsteps) return;
  // selection operands: column c of half h picks row 16 h + c
  u32x4 sel[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int k0 = 8 * q + 2 * e2, k1 = k0 + 1;
      w[e2] = (k0 == 16 * h + r ? 0x3F80u : 0u) | (k1 == 16 * h + r ? 0x3F800000u : 0u);
    }
    sel[h] = u32x4{w[0], w[1], w[2], w[3]};
  }
  f32x4 acc[CSW][2][NT];
#pragma unroll
  for (int c = 0; c < CSW; ++c)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int mt = 0; mt < NT; ++mt) acc[c][h][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int64_t b0 = static_cast<int64_t>(blockIdx.y) * blks_per_chunk;
  int64_t b1 = b0 + blks_per_chunk;
  if (b1 > nblk) b1 = nblk;
  // (a chunk past the last token block still writes its zeros: the partial sums of every
  // chunk are added afterwards)

  struct In {
    u32x4 X[CSW][2];
    u32x2 v[NT][4];   // hi: tokens 4q.., 16+4q.. ; lo: the same
  };
  auto load = [&](In &in, int64_t blk) {
#pragma unroll
    for (int gI = 0; gI < 2; ++gI) {
      int64_t t = blk * 32 + gI * 16 + r;
      if (t > T - 1) t = T - 1;
#pragma unroll
      for (int c = 0; c < CSW; ++c) {
        const int s = s0 + c < nsteps ? s0 + c : nsteps - 1;
        in.X[c][gI] = *reinterpret_cast<const u32x4 *>(x + t * K + s * 32 + q * 8);
      }
    }
#pragma unroll
    for (int mt = 0; mt < NT; ++mt) {
      const size_t row = (static_cast<size_t>(blk) * MP16 + mt * 16 + r) * 32;
      in.v[mt][0] = *reinterpret_cast<const u32x2 *>(vrT_hi + row + 4 * q);
      in.v[mt][1] = *reinterpret_cast<const u32x2 *>(vrT_hi + row + 16 + 4 * q);
      in.v[mt][2] = *reinterpret_cast<const u32x2 *>(vrT_lo + row + 4 * q);
      in.v[mt][3] = *reinterpret_cast<const u32x2 *>(vrT_lo + row + 16 + 4 * q);
    }
  };
  auto process = [&](const In &in) {
#pragma unroll
    for (int c = 0; c < CSW; ++c) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
        const f32x4 t0 = mfma16(in.X[c][0], sel[h], z);   // tokens 4q+i of the first 16
        const f32x4 t1 = mfma16(in.X[c][1], sel[h], z);   // tokens 4q+i of the second 16
        u32x4 bt;
        bt.x = cvt_pk_bf16(t0[0], t0[1]); bt.y = cvt_pk_bf16(t0[2], t0[3]);
        bt.z = cvt_pk_bf16(t1[0], t1[1]); bt.w = cvt_pk_bf16(t1[2], t1[3]);
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) {
          const u32x4 vh = u32x4{in.v[mt][0].x, in.v[mt][0].y, in.v[mt][1].x, in.v[mt][1].y};
          const u32x4 vl = u32x4{in.v[mt][2].x, in.v[mt][2].y, in.v[mt][3].x, in.v[mt][3].y};
          acc[c][h][mt] = mfma16(vh, bt, acc[c][h][mt]);
          acc[c][h][mt] = mfma16(vl, bt, acc[c][h][mt]);
        }
      }
    }
  };
  if (b0 < b1) {
    In cur, nxt;
    load(cur, b0);
    int64_t blk = b0;
    for (; blk + 1 < b1; ++blk) {
      load(nxt, blk + 1);
      __builtin_amdgcn_sched_barrier(0);
      process(cur);
      cur = nxt;
    }
    process(cur);
  }

  float *dst = out + static_cast<size_t>(blockIdx.y) * K * M;
#pragma unroll
  for (int c = 0; c < CSW; ++c) {
    if (s0 + c < nsteps) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = (s0 + c) * 32 + 16 * h + r;
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + 4 * q + i;
            if (m < M) dst[static_cast<size_t>(k) * M + m] = acc[c][h][mt][i];
          }
      }
    }
  }
}

// The same reduction for many logit tiles (n = 5: NT = 9).  Every wave of a block
// needs the whole vrT block of the 32 tokens at hand (18 KiB), so the block (eight
// waves, one block per CU) stages it in LDS once instead of each wave fetching it
// from L2.  Both vrT and the waves' own x rows arrive by direct global->LDS loads
// (lane l of a wave lands at the wave's base + 16 l), requested TWO token blocks
// ahead: vrT into a ring of three buffers, x into two slots per wave (a slot is free
// again once its rows are in registers).  Every wave issues the same number of loads
// per batch (kBatch), so "all but the newest batch have landed" is one
// s_waitcnt vmcnt(kBatch), and no register waits on memory across iterations.
// (The count relies on one vector-memory instruction per to_lds() call and no other
// vector-memory access inside the loop; the compiled loop holds exactly kBatch.)
template <int NT, int CSW>
struct GwLdsCfg {
  static constexpr int kThreads = 512;
  static constexpr int kPartVec = NT * 16 * 4;                   // 16-byte words of one part of a vrT block
  static constexpr int kBufVec = 2 * kPartVec;
  static constexpr int WV = (kBufVec + kThreads - 1) / kThreads;  // rounds of the block per buffer
  static constexpr int kBufPad = WV * kThreads;                  // whole rounds (the surplus lands in padding)
  static constexpr int kXSlot = 2 * CSW * 64;                    // words of one wave's x rows of a token block
  static constexpr int kBatch = WV + 2 * CSW;                    // vector-memory instructions per wave and batch
  static constexpr int kLdsBytes = (3 * kBufPad + 2 * 8 * kXSlot) * 16;
};

template <int NT, int CSW>
__global__ __launch_bounds__(512, 1) void bwd_gw_lds_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ vrT_hi,
    const uint16_t *__restrict__ vrT_lo, int K, int M, int64_t T, int64_t nblk,
    int blks_per_chunk, float *__restrict__ out) {
  using Cfg = GwLdsCfg<NT, CSW>;
  constexpr int kPartVec = Cfg::kPartVec, kBufVec = Cfg::kBufVec, kBufPad = Cfg::kBufPad;
  constexpr int kBatch = Cfg::kBatch;
  static_assert(kBatch <= 15, "the wait below encodes the count in four bits");
  extern __shared__ u32x4 lds[];
  u32x4 *xring = lds + 3 * kBufPad;             // [slot][wave][c][gI][lane]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int s0 = (blockIdx.x * 8 + wave) * CSW;
  const int nsteps = K / 32;
  u32x4 sel[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int k0 = 8 * q + 2 * e2, k1 = k0 + 1;
      w[e2] = (k0 == 16 * h + r ? 0x3F80u : 0u) | (k1 == 16 * h + r ? 0x3F800000u : 0u);
    }
    sel[h] = u32x4{w[0], w[1], w[2], w[3]};
  }
  f32x4 acc[CSW][2][NT];
#pragma unroll
  for (int c = 0; c < CSW; ++c)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int mt = 0; mt < NT; ++mt) acc[c][h][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int64_t b0 = static_cast<int64_t>(blockIdx.y) * blks_per_chunk;
  int64_t b1 = b0 + blks_per_chunk;
  if (b1 > nblk) b1 = nblk;

  const u32x4 *vh = reinterpret_cast<const u32x4 *>(vrT_hi);
  const u32x4 *vl = reinterpret_cast<const u32x4 *>(vrT_lo);
  auto to_lds = [](const void *src, u32x4 *dst) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
  };
  // one batch: vrT block `blk` -> ring buffer `vbuf`, this wave's x rows of it -> slot `xs`
  auto request = [&](int64_t blk, int vbuf, int xs) {
#pragma unroll
    for (int i = 0; i < Cfg::WV; ++i) {
      int e = i * Cfg::kThreads + threadIdx.x;
      if (e > kBufVec - 1) e = kBufVec - 1;     // surplus lanes re-read the last word (into padding)
      // LDS word e of a part = 16-byte piece (e & 3) ^ ((row >> 2) & 3) of row e >> 2: the
      // 64-byte rows r, r + 4, r + 8, r + 12 would otherwise share their banks
      const int ep = e < kPartVec ? e : e - kPartVec;
      const int eg = (ep & ~3) | ((ep & 3) ^ ((ep >> 4) & 3));
      const u32x4 *src = (e < kPartVec ? vh : vl) + blk * kPartVec + eg;
      to_lds(src, lds + vbuf * kBufPad + i * Cfg::kThreads + wave * 64);
    }
#pragma unroll
    for (int c = 0; c < CSW; ++c) {
      const int s = s0 + c < nsteps ? s0 + c : nsteps - 1;
#pragma unroll
      for (int gI = 0; gI < 2; ++gI) {
        int64_t t = blk * 32 + gI * 16 + r;
        if (t > T - 1) t = T - 1;
        to_lds(x + t * K + s * 32 + q * 8, xring + (xs * 8 + wave) * Cfg::kXSlot + (c * 2 + gI) * 64);
      }
    }
  };

  if (b0 < b1) {   // uniform over the block; an empty chunk still writes its zeros
    request(b0, 0, 0);
    request(b0 + 1 < b1 ? b0 + 1 : b0, 1, 1);
    for (int64_t blk = b0; blk < b1; ++blk) {
      const int i = static_cast<int>(blk - b0);
      // Everything but the newest batch has landed (vmcnt(kBatch)), this wave's LDS
      // reads of the previous block are done (lgkmcnt(0)), then the barrier.  Written
      // out because __syncthreads() carries a release fence that waits for ALL
      // outstanding vector-memory operations, the prefetched batch included.
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(kBatch) : "memory");
      __builtin_amdgcn_sched_barrier(0);
      const u32x4 *xs = xring + ((i & 1) * 8 + wave) * Cfg::kXSlot + lane;
      u32x4 bt[CSW][2];
#pragma unroll
      for (int c = 0; c < CSW; ++c) {
        const u32x4 x0 = xs[(c * 2 + 0) * 64], x1 = xs[(c * 2 + 1) * 64];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
          const f32x4 t0 = mfma16(x0, sel[h], z);
          const f32x4 t1 = mfma16(x1, sel[h], z);
          bt[c][h].x = cvt_pk_bf16(t0[0], t0[1]); bt[c][h].y = cvt_pk_bf16(t0[2], t0[3]);
          bt[c][h].z = cvt_pk_bf16(t1[0], t1[1]); bt[c][h].w = cvt_pk_bf16(t1[2], t1[3]);
        }
      }
      // the x slot has been read into registers (the products above used it): refill it,
      // and the vrT buffer that was read two blocks ago
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
      request(blk + 2 < b1 ? blk + 2 : b1 - 1, (i + 2) % 3, i & 1);   // past the end: the last block again
      __builtin_amdgcn_sched_barrier(0);
      // lane (logit row r, q) takes tokens 4q..4q+3 and 16+4q..: two 8-byte pieces of its 64-byte row
      const uint32_t *base = reinterpret_cast<const uint32_t *>(lds + (i % 3) * kBufPad);
#pragma unroll
      for (int mt = 0; mt < NT; ++mt) {
        // pieces (q >> 1) and 2 + (q >> 1) of the row, at their swizzled places; in 4-byte words
        const int sw = (r >> 2) & 3;
        const int row = (mt * 16 + r) * 16 + (q & 1) * 2;
        const int p0 = row + (((q >> 1) ^ sw) << 2), p1 = row + (((2 + (q >> 1)) ^ sw) << 2);
        const u32x2 h0 = *reinterpret_cast<const u32x2 *>(base + p0);
        const u32x2 h1 = *reinterpret_cast<const u32x2 *>(base + p1);
        const u32x2 l0 = *reinterpret_cast<const u32x2 *>(base + kPartVec * 4 + p0);
        const u32x2 l1 = *reinterpret_cast<const u32x2 *>(base + kPartVec * 4 + p1);
        const u32x4 ah = u32x4{h0.x, h0.y, h1.x, h1.y}, al = u32x4{l0.x, l0.y, l1.x, l1.y};
#pragma unroll
        for (int c = 0; c < CSW; ++c)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            acc[c][h][mt] = mfma16(ah, bt[c][h], acc[c][h][mt]);
            acc[c][h][mt] = mfma16(al, bt[c][h], acc[c][h][mt]);
          }
      }
    }
    // nothing may still be writing LDS when the block ends
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
  }

  float *dst = out + static_cast<size_t>(blockIdx.y) * K * M;
#pragma unroll
  for (int c = 0; c < CSW; ++c) {
    if (s0 + c < nsteps) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = (s0 + c) * 32 + 16 * h + r;
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + 4 * q + i;
            if (m < M) dst[static_cast<size_t>(k) * M + m] = acc[c][h][mt][i];
          }
      }
    }
  }
}

// logit tiles of the full permutation and Sinkhorn-Knopp forms (n <= 5)
template <typename F>
hipError_t dispatch_nt(int NT, F &&f) {
  switch (NT) {
    case 1: return f(std::integral_constant<int, 1>{});
    case 2: return f(std::integral_constant<int, 2>{});
    case 3: return f(std::integral_constant<int, 3>{});
    case 9: return f(std::integral_constant<int, 9>{});
  }
  return hipErrorInvalidValue;
}
// any count up to 9 (the permutation-subset form): projection only
template <typename F>
hipError_t dispatch_nt_proj(int NT, F &&f) {
  switch (NT) {
    case 4: return f(std::integral_constant<int, 4>{});
    case 5: return f(std::integral_constant<int, 5>{});
    case 6: return f(std::integral_constant<int, 6>{});
    case 7: return f(std::integral_constant<int, 7>{});
    case 8: return f(std::integral_constant<int, 8>{});
  }
  return dispatch_nt(NT, f);
}

}  // namespace

bool fast_path_ok(const mhcl_desc &d) {
  if (d.io_dtype != MHCL_BF16 || d.C % 64 != 0) return false;
  const int NT = logit_tiles(res_logits(d) + 2 * d.n);
  return NT >= 1 && NT <= 9;
}

size_t packed_w_b_bytes(const mhcl_desc &d, int M) { return packed_b_bytes(d.n * d.C, M); }

hipError_t launch_pack_w_b(const mhcl_desc &d, int M, const float *W, void *Wp, hipStream_t s,
                           float *zero, size_t nzero) {
  const int K = d.n * d.C, NT = logit_tiles(M);
  const int threads = (K / 32) * NT * 64;
  if (nzero > 0xffffffffu) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_w_b_kernel, dim3((threads + 255) / 256), dim3(256), 0, s, W, K, M, NT,
                     static_cast<uint4 *>(Wp), zero, static_cast<unsigned>(nzero));
  return hipGetLastError();
}

int proj_ksplit(const mhcl_desc &d) {
  if (!fast_path_ok(d)) return 1;
  const int M = res_logits(d) + 2 * d.n;
  int kc = 4, tok = 128;
  const int want = 256;   // one block per CU
  (void)dispatch_nt_proj(logit_tiles(M), [&](auto nt) {
    kc = ProjCfg<decltype(nt)::value>::KC;
    tok = ProjCfg<decltype(nt)::value>::kTokens;
    return hipSuccess;
  });
  const int nsteps = d.n * d.C / 32;
  const int64_t blocks = (d.T + tok - 1) / tok;
  int ks = 1;   // enough blocks for one per CU, each part a whole number of chunk pairs
  while (ks < kMaxKSplit && blocks * ks < want && nsteps % (ks * 2 * 2 * kc) == 0) ks *= 2;
  return ks;
}

hipError_t launch_proj_mfma(const mhcl_desc &d, int M, const void *x, const void *Wp, float *u_raw,
                            float *sumsq, hipStream_t s) {
  const int K = d.n * d.C;
  const int ks = proj_ksplit(d);
  return dispatch_nt_proj(logit_tiles(M), [&](auto nt) {
    constexpr int NT = decltype(nt)::value;
    auto kern = proj_mfma_kernel<NT>;
    constexpr int lds = ProjCfg<NT>::kLdsBytes;
    if (lds > 64 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      if (e != hipSuccess) return e;
    }
    constexpr int kTok = ProjCfg<NT>::kTokens;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>((d.T + kTok - 1) / kTok), ks),
                       dim3(ProjCfg<NT>::kThreads),
                       lds, s, static_cast<const uint16_t *>(x), static_cast<const u32x4 *>(Wp), K,
                       M, d.T, u_raw, sumsq);
    return hipGetLastError();
  });
}


// ---- fused backward, bf16, n <= 4 -------------------------------------------
// n <= 4 (at most 32 logits): fused passes; n = 5: the wide variant of pass 2
bool fast_bwd_ok(const mhcl_desc &d) { return fast_path_ok(d); }
// the single-kernel pass 2 exists for the (n, logit tiles) pairs of the full forms with
// n <= 4; everything else (n >= 5, any permutation subset) takes the wide pass 2
bool fast_bwd_wide(const mhcl_desc &d) { return d.n > 4 || d.res_mode == MHCL_RES_SUBSET; }
// n = 5 of the full forms: wide pass 2 in one kernel with W as one fp16 part in LDS
bool fast_bwd_whi(const mhcl_desc &d) {
  if (!fast_bwd_wide(d) || d.n < 5) return false;
  const int MS = logit_steps(res_logits(d) + 2 * d.n);
  const int CP = (d.n * d.n + 2 * d.n + 2 + 7) / 8 * 8;
  return d.n * MS * 4096 + 8 * 16 * (CP + 4) * 4 <= 160 * 1024;   // OutW16Cfg::kLdsBytes
}

namespace {
// K steps per wave of bwd_gw_kernel: bounded by its accumulators (2 * NT * 4 registers per step)
int gw_csw(const mhcl_desc &d) {
  return logit_tiles(res_logits(d) + 2 * d.n) <= 3 ? 4 : 2;
}
int gw_xblocks(const mhcl_desc &d) {
  const bool lds_kernel = logit_tiles(res_logits(d) + 2 * d.n) > 3;   // eight waves per block there
  const int per_block = (lds_kernel ? 8 : 4) * gw_csw(d);
  return (d.n * d.C / 32 + per_block - 1) / per_block;
}
}  // namespace

int out_gw_tokens_per_block(const mhcl_desc &d) {
  // Token chunks: as many as make the grid one round of resident blocks (all blocks
  // then start together and the blocks of a chunk walk down the same rows side by
  // side), never more than 64 MiB of partial g_W copies, and blocks of a whole
  // number of 64-token iterations (at least 256 tokens, to amortise staging W).
  const int64_t M = res_logits(d) + 2 * d.n;
  const int64_t copy_bytes = static_cast<int64_t>(d.n) * d.C * M * 4;
  const bool pair = (d.C / 64) % 2 == 0;            // two 64-column steps per block
  const int64_t resident = pair ? 256 : 512;        // blocks the chip holds at once
  const int64_t xblocks = pair ? d.C / 128 : d.C / 64;
  int64_t chunks = resident / xblocks;
  if (chunks < 1) chunks = 1;
  const int64_t cap = (64ll << 20) / copy_bytes;
  if (chunks > cap) chunks = cap < 1 ? 1 : cap;
  int64_t tpb = ((d.T + chunks - 1) / chunks + 63) / 64 * 64;
  if (tpb < 256) tpb = 256;
  return static_cast<int>(tpb);
}

int gw_chunks_fast(const mhcl_desc &d) {
  const int64_t nblk = (d.T + 31) / 32;
  // the largest chunk count that keeps the grid at one round of resident blocks (one
  // eight-wave block per compute unit in the LDS kernel, two four-wave blocks otherwise)
  const bool lds_kernel = logit_tiles(res_logits(d) + 2 * d.n) > 3;
  int64_t c = (lds_kernel ? 256 : 512) / gw_xblocks(d);
  if (c > 64) c = 64;
  if (c > nblk) c = nblk;
  if (c < 1) c = 1;
  return static_cast<int>(c);
}

FastBwdWs::FastBwdWs(const mhcl_desc &d, void *ws) {
  WsCursor c(ws);
  const size_t T = static_cast<size_t>(d.T), Tpad = (T + 63) / 64 * 64;
  const int n = d.n, M = res_logits(d) + 2 * d.n, K = d.n * d.C;
  CP = (n * n + 2 * n + 2 + 7) / 8 * 8;   // H_res | H_pre | H_post | coefx | scale of the vr row, padded
  MP32 = logit_steps(M) * 32;
  MP16 = logit_tiles(M) * 16;
  parts = fast_bwd_wide(d) ? proj_ksplit(d) : 1;   // the wide path recomputes with proj_mfma_kernel
  u_raw = c.take<float>(static_cast<size_t>(parts) * T * M);
  sumsq = c.take<float>(static_cast<size_t>(parts) * T);
  gH_res = c.take<float>(T * n * n);
  gH_pre = c.take<float>(T * n);
  gH_post = c.take<float>(T * n);
  cpk = c.take<float>(T * CP);
  gz = c.take<float>((Tpad / 64) * (M + 3));
  vr_hi = c.take<uint16_t>(Tpad * MP32);
  vr_lo = c.take<uint16_t>(Tpad * MP32);
  vrT_hi = c.take<uint16_t>(Tpad * MP16);
  vrT_lo = c.take<uint16_t>(Tpad * MP16);
  Wp = c.take<char>(packed_b_bytes(K, M));
  Wa = c.take<char>(packed_a_bytes(K, M));
  wmax_part = c.take<float>(256);   // kWmaxBlocks
  wscale = c.take<float>(2);
  {
    const int64_t tpb = out_gw_tokens_per_block(d);
    const size_t fused_chunks = static_cast<size_t>((d.T + tpb - 1) / tpb);
    const size_t chunks = fused_chunks > static_cast<size_t>(gw_chunks_fast(d)) ? fused_chunks : gw_chunks_fast(d);
    partials = c.take<float>(chunks * K * M);
  }
  psum = c.take<float>(static_cast<size_t>(param_sum_blocks(d)) * (M + 3));
  D = fast_bwd_wide(d) ? c.take<float>(T * K) : nullptr;
  bytes = c.off;
}

hipError_t launch_pack_w_ab(const mhcl_desc &d, int M, const float *W, const FastBwdWs &w,
                            hipStream_t s) {
  const int K = d.n * d.C, NT = logit_tiles(M), MS = logit_steps(M);
  const int nb_b = ((K / 32) * NT * 64 + 255) / 256;
  const int nb_a = ((K / 64) * 4 * MS * 64 + 255) / 256;
  // one fp16 part where the only reader is bwd_out_w16_kernel; its scale needs max |W| first
  const bool a16 = fast_bwd_whi(d);
  if (a16) {
    hipLaunchKernelGGL(w_absmax_kernel, dim3(kWmaxBlocks), dim3(256), 0, s,
                       reinterpret_cast<const float4 *>(W), static_cast<size_t>(K) * M / 4,
                       w.wmax_part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(pack_w_ab_kernel, dim3(nb_b + nb_a), dim3(256), 0, s, W, K, M, NT, MS, nb_b,
                     a16 ? 1 : 0, w.wmax_part, w.wscale, reinterpret_cast<uint4 *>(w.Wp),
                     reinterpret_cast<uint4 *>(w.Wa));
  return hipGetLastError();
}

hipError_t launch_bwd_reduce(const mhcl_desc &d, int M, const void *x, const void *y,
                             const void *g_xout, const void *g_h, const FastBwdWs &w,
                             hipStream_t s) {
  auto go = [&](auto nn, auto nt) {
    constexpr int N = decltype(nn)::value, NT = decltype(nt)::value;
    auto launch = [&](auto wv) {
      constexpr int WAVES = decltype(wv)::value;
      auto kern = bwd_reduce_kernel<N, NT, WAVES>;
      hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>((d.T + 16 * WAVES - 1) / (16 * WAVES))),
                         dim3(64 * WAVES), (ReduceCfg<N, NT, WAVES>::kLdsBytes), s,
                         static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(y),
                         static_cast<const uint16_t *>(g_xout), static_cast<const uint16_t *>(g_h),
                         reinterpret_cast<const u32x4 *>(w.Wp), d.C, M, d.T, w.u_raw, w.sumsq,
                         w.gH_res, w.gH_post, w.gH_pre);
      return hipGetLastError();
    };
    // 128-token blocks halve the W traffic from L2 (0.52 -> 0.48 ms at n = 4, C = 4096,
    // T = 32768) but need enough tokens to put a block on every CU
    return (d.T + 127) / 128 >= 256 ? launch(std::integral_constant<int, 8>{})
                                    : launch(std::integral_constant<int, 4>{});
  };
  const int NT = logit_tiles(M);
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  using I4 = std::integral_constant<int, 4>;
  switch (d.n * 10 + NT) {   // the (n, logit tiles) pairs that occur for n <= 4
    case 11: return go(I1{}, I1{});   // lite M=3, SK M=3
    case 21: return go(I2{}, I1{});   // lite M=6, SK M=8
    case 31: return go(I3{}, I1{});   // lite M=12, SK M=15
    case 42: return go(I4{}, I2{});   // lite M=32, SK M=24
  }
  return hipErrorInvalidValue;
}

// pass 1 of the wide case without the projection: the dot products alone
hipError_t launch_bwd_dots_fast(const mhcl_desc &d, const void *x, const void *y, const void *g_xout,
                                const void *g_h, const FastBwdWs &w, hipStream_t s) {
  auto go = [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    hipLaunchKernelGGL(bwd_dots_fast_kernel<N>, dim3(static_cast<unsigned>((d.T + 63) / 64)),
                       dim3(256), 0, s, static_cast<const uint16_t *>(x),
                       static_cast<const uint16_t *>(y), static_cast<const uint16_t *>(g_xout),
                       static_cast<const uint16_t *>(g_h), d.C, d.T, w.gH_res, w.gH_post, w.gH_pre);
    return hipGetLastError();
  };
  switch (d.n) {
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

hipError_t launch_bwd_epilogue_fast(const mhcl_desc &d, const float *b, const float *alpha,
                                    const FastBwdWs &w, hipStream_t s) {
  const int64_t Tpad = (d.T + 63) / 64 * 64;
  auto go = [&](auto nn, auto mm) {
    constexpr int N = decltype(nn)::value, MODE = decltype(mm)::value;
    if (w.MP32 != (Dims<N, MODE>::M + 31) / 32 * 32 || w.MP16 != (Dims<N, MODE>::M + 15) / 16 * 16)
      return hipErrorInvalidValue;
    constexpr bool kF16 = N == 5;   // the widths of fast_bwd_whi(): rows for bwd_out_w16_kernel
    if (kF16 != fast_bwd_whi(d) || (kF16 && w.CP < N * N + 2 * N + 2)) return hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_epilogue_fast_kernel<N, MODE, kF16>),
                       dim3(static_cast<unsigned>(Tpad / 64)), dim3(64), 0, s, w.u_raw, w.sumsq,
                       w.parts, b, alpha, w.gH_res, w.gH_pre, w.gH_post, d.n * d.C, d.eps,
                       d.sk_iters, d.T, w.CP, w.cpk, w.vr_hi, w.vr_lo, w.vrT_hi, w.vrT_lo, w.gz);
    return hipGetLastError();
  };
  using L = std::integral_constant<int, MHCL_RES_LITE>;
  using S = std::integral_constant<int, MHCL_RES_SK>;
  const bool lite = d.res_mode == MHCL_RES_LITE;
  switch (d.n) {
    case 1: return lite ? go(std::integral_constant<int, 1>{}, L{}) : go(std::integral_constant<int, 1>{}, S{});
    case 2: return lite ? go(std::integral_constant<int, 2>{}, L{}) : go(std::integral_constant<int, 2>{}, S{});
    case 3: return lite ? go(std::integral_constant<int, 3>{}, L{}) : go(std::integral_constant<int, 3>{}, S{});
    case 4: return lite ? go(std::integral_constant<int, 4>{}, L{}) : go(std::integral_constant<int, 4>{}, S{});
    // the full permutation form at n = 5 (120 permutations) takes the eight-lanes-per-token kernel
    case 5: return lite ? hipErrorInvalidValue : go(std::integral_constant<int, 5>{}, S{});
  }
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_gw(const mhcl_desc &d, int M, const void *x, const FastBwdWs &w, float *g_W,
                         hipStream_t s) {
  const int K = d.n * d.C;
  const int64_t nblk = (d.T + 31) / 32;
  const int chunks = gw_chunks_fast(d);
  const int bpc = static_cast<int>((nblk + chunks - 1) / chunks);
  float *dst = chunks == 1 ? g_W : w.partials;
  hipError_t e = dispatch_nt_proj(logit_tiles(M), [&](auto nt) {
    constexpr int NT = decltype(nt)::value;
    if constexpr (NT <= 3) {
      hipLaunchKernelGGL((bwd_gw_kernel<NT, 4>), dim3(gw_xblocks(d), chunks), dim3(256), 0, s,
                         static_cast<const uint16_t *>(x), w.vrT_hi, w.vrT_lo, K, M, w.MP16, d.T,
                         nblk, bpc, dst);
    } else {
      auto kern = bwd_gw_lds_kernel<NT, 2>;
      constexpr int lds = GwLdsCfg<NT, 2>::kLdsBytes;
      if (lds > 64 * 1024) {
        hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e1 != hipSuccess) return e1;
      }
      hipLaunchKernelGGL(kern, dim3(gw_xblocks(d), chunks), dim3(512), lds, s,
                         static_cast<const uint16_t *>(x), w.vrT_hi, w.vrT_lo, K, M, d.T, nblk, bpc,
                         dst);
    }
    return hipGetLastError();
  });
  return e;   // the chunks' partial sums are added by launch_bwd_finish
}

// wide pass 2: D = W vr, then g_x and g_y
hipError_t launch_bwd_out_wide(const mhcl_desc &d, int M, const void *x, const void *g_xout,
                               const void *g_h, const FastBwdWs &w, void *g_x, void *g_y,
                               hipStream_t s) {
  const int K = d.n * d.C, MS = logit_steps(M);
  if (fast_bwd_whi(d)) {
    // one kernel, W as one fp16 part resident in LDS; one round of one block per CU
    const int64_t xb = d.C / 64;
    int64_t chunks = 256 / xb;
    if (chunks < 1) chunks = 1;
    int64_t tpb1 = ((d.T + chunks - 1) / chunks + 127) / 128 * 128;
    if (tpb1 < 256) tpb1 = 256;
    while ((d.T + tpb1 - 1) / tpb1 > 32768) tpb1 *= 2;
    const dim3 grid1(static_cast<unsigned>(xb), static_cast<unsigned>((d.T + tpb1 - 1) / tpb1));
    auto fused = [&](auto nn, auto ms) {
      constexpr int kN = decltype(nn)::value, kMS = decltype(ms)::value;
      using Cfg = OutW16Cfg<kN, kMS>;
      if constexpr (!Cfg::kFits) {
        return hipErrorInvalidValue;
      } else {
        if (w.CP != Cfg::CP) return hipErrorInvalidValue;
        auto kern = bwd_out_w16_kernel<kN, kMS>;
        if (Cfg::kLdsBytes > 64 * 1024) {
          hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                              hipFuncAttributeMaxDynamicSharedMemorySize,
                                              Cfg::kLdsBytes);
          if (e1 != hipSuccess) return e1;
        }
        hipLaunchKernelGGL(kern, grid1, dim3(512), Cfg::kLdsBytes, s,
                           static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(g_xout),
                           static_cast<const uint16_t *>(g_h), reinterpret_cast<const u32x4 *>(w.Wa),
                           w.cpk, w.vr_hi, w.vr_lo, w.wscale, w.MP32, d.C, d.T, static_cast<int>(tpb1),
                           static_cast<uint16_t *>(g_x), static_cast<uint16_t *>(g_y));
        return hipGetLastError();
      }
    };
    auto by_ms = [&](auto nn) {
      switch (MS) {
        case 1: return fused(nn, std::integral_constant<int, 1>{});
        case 2: return fused(nn, std::integral_constant<int, 2>{});
        case 3: return fused(nn, std::integral_constant<int, 3>{});
        case 4: return fused(nn, std::integral_constant<int, 4>{});
        case 5: return fused(nn, std::integral_constant<int, 5>{});
      }
      return hipErrorInvalidValue;
    };
    switch (d.n) {
      case 5: return by_ms(std::integral_constant<int, 5>{});
      case 6: return by_ms(std::integral_constant<int, 6>{});
      case 7: return by_ms(std::integral_constant<int, 7>{});
      case 8: return by_ms(std::integral_constant<int, 8>{});
    }
    return hipErrorInvalidValue;
  }
  // 1024 tokens per block, more once that would exceed the grid's second dimension
  int64_t tpb = 1024;
  while ((d.T + tpb - 1) / tpb > 32768) tpb *= 2;
  const int kTokensPerBlock = static_cast<int>(tpb);
  const dim3 grid(K / 64, static_cast<unsigned>((d.T + kTokensPerBlock - 1) / kTokensPerBlock));
  auto wv = [&](auto ms) {
    constexpr int kMS = decltype(ms)::value;
    hipLaunchKernelGGL(wv_kernel<kMS>, grid, dim3(256), 4 * kMS * 2 * 64 * 16, s,
                       reinterpret_cast<const u32x4 *>(w.Wa), w.vr_hi, w.vr_lo, w.MP32, K, d.T,
                       kTokensPerBlock, w.D);
    return hipGetLastError();
  };
  hipError_t e = hipErrorInvalidValue;
  switch (MS) {
    case 1: e = wv(std::integral_constant<int, 1>{}); break;
    case 2: e = wv(std::integral_constant<int, 2>{}); break;
    case 3: e = wv(std::integral_constant<int, 3>{}); break;
    case 4: e = wv(std::integral_constant<int, 4>{}); break;
    case 5: e = wv(std::integral_constant<int, 5>{}); break;
  }
  if (e != hipSuccess) return e;
  const int64_t vecs = d.T * (d.C / 8);
  auto mix = [&](auto nn) {
    constexpr int N = decltype(nn)::value;
    hipLaunchKernelGGL(mix_wide_kernel<N>, dim3(static_cast<unsigned>((vecs + 255) / 256)),
                       dim3(256), 0, s, static_cast<const uint16_t *>(x),
                       static_cast<const uint16_t *>(g_xout), static_cast<const uint16_t *>(g_h),
                       w.D, w.cpk, w.CP, d.C, d.T, static_cast<uint16_t *>(g_x),
                       static_cast<uint16_t *>(g_y));
    return hipGetLastError();
  };
  switch (d.n) {
    case 1: return mix(std::integral_constant<int, 1>{});
    case 2: return mix(std::integral_constant<int, 2>{});
    case 3: return mix(std::integral_constant<int, 3>{});
    case 4: return mix(std::integral_constant<int, 4>{});
    case 5: return mix(std::integral_constant<int, 5>{});
    case 6: return mix(std::integral_constant<int, 6>{});
    case 7: return mix(std::integral_constant<int, 7>{});
    case 8: return mix(std::integral_constant<int, 8>{});
  }
  return hipErrorInvalidValue;
}

// g_x, g_y and g_W from one pass (n <= 4)
hipError_t launch_bwd_out_gw(const mhcl_desc &d, int M, const void *x, const void *g_xout,
                             const void *g_h, const FastBwdWs &w, void *g_x, void *g_y, float *g_W,
                             hipStream_t s) {
  const int tpb = out_gw_tokens_per_block(d);
  const int chunks = static_cast<int>((d.T + tpb - 1) / tpb);
  float *dst = chunks == 1 ? g_W : w.partials;
  // two adjacent 64-column steps per block where C allows it
  const bool pair = (d.C / 64) % 2 == 0;
  auto go = [&](auto nn, auto nt) {
    constexpr int N = decltype(nn)::value, NT = decltype(nt)::value;
    constexpr int lds = (N * 4 * 2 * 64) * 2 * 16;
    auto launch = [&](auto sl) {
      constexpr int SL = decltype(sl)::value;
      auto kern = bwd_out_gw_kernel<N, NT, SL>;
      if (lds * SL > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds * SL);
        if (e != hipSuccess) return e;
      }
      hipLaunchKernelGGL(kern, dim3(d.C / 64 / SL, chunks), dim3(256 * SL), lds * SL, s,
                         static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(g_xout),
                         static_cast<const uint16_t *>(g_h), reinterpret_cast<const u32x4 *>(w.Wa),
                         w.cpk, w.vr_hi, w.vr_lo, w.vrT_hi, w.vrT_lo, w.MP16, M, d.C, d.T, tpb,
                         w.CP, static_cast<uint16_t *>(g_x), static_cast<uint16_t *>(g_y), dst);
      return hipGetLastError();
    };
    return pair ? launch(std::integral_constant<int, 2>{}) : launch(std::integral_constant<int, 1>{});
  };
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  using I4 = std::integral_constant<int, 4>;
  hipError_t e = hipErrorInvalidValue;
  switch (d.n * 10 + logit_tiles(M)) {
    case 11: e = go(I1{}, I1{}); break;
    case 21: e = go(I2{}, I1{}); break;
    case 31: e = go(I3{}, I1{}); break;
    case 42: e = go(I4{}, I2{}); break;
  }
  return e;   // the chunks' partial sums are added by launch_bwd_finish
}

// number of token chunks whose g_W partial sums the backward leaves in the workspace
int fast_gw_chunks(const mhcl_desc &d) {
  if (fast_bwd_wide(d)) return gw_chunks_fast(d);
  const int tpb = out_gw_tokens_per_block(d);
  return static_cast<int>((d.T + tpb - 1) / tpb);
}

}  // namespace mhcl
