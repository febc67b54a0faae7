// Forward of the bf16 fast path with ONE read of x: the projection u_raw = x_hat W with
// sum(x_hat^2) (Sec. 3.2, the lines above Eq. (4)), the gate H_pre (Eq. (5)) and the
// pre-aggregate h = H_pre x (Eq. (1), argument of f) from the same register tile.
//
// A token's n x C streams (32 KiB at n = 4, C = 4096) do not fit one compute unit next to
// its neighbours, so the columns are split: a CLUSTER of `parts` blocks shares groups of 16
// tokens, block `part` owns 256 columns of every stream.  Per group a block
//   A  multiplies its piece (16 tokens x n x 256 columns, kept in registers) with its slice
//      of W (resident in LDS for the block's whole life) and writes the partial logits and
//      the partial sum of squares as slice `part` of u_raw / sumsq (the coefficient stage
//      adds the slices in order, as it does for a K split),
//      publishes its partial pre-logits and sum of squares to the cluster,
//   B  three groups later, adds those of ITS share of the group's tokens (token t belongs to
//      part t mod parts) over all parts, in part order, and publishes H_pre of those tokens,
//   C  another three groups later, reads H_pre of all 16 tokens and writes its 256 columns of
//      h from the piece it still holds (eight pieces in registers, 16 registers each at n = 4).
// The blocks of a cluster exchange those few values through memory as 64-bit words that carry
// a tag (the group's number + 1) next to the value, written and read with relaxed agent-scope
// atomics: a word is either the old one or the complete new one, so no fence is needed and
// nothing is ever read before it is valid.  Exchange rings are zeroed before the launch.
// The blocks of a cluster must be resident together: 256 blocks, one per compute unit.
// Every wait is bounded: a lane that does not see its tag after kOnceSpin polls gives up for
// good and its results become NaN, so a lost block shows up in the outputs instead of hanging.
#include "mhcl_common.h"
#include "mhcl_internal.h"
#include "mhcl_mfma.h"
#include <atomic>
#include <cstdlib>

namespace mhcl {

namespace {

typedef unsigned long long u64;
constexpr int kOnceCB = 256;      // columns of every stream per block
constexpr int kOnceGT = 16;       // tokens per group: one MFMA row tile
// Schedule of a step `it`: the piece of group it + PF is requested, group it goes through A,
// group it - DB through B, group it - DC through C.  A published word is polled for the first
// time one and a half steps after it was written (the first try for step it goes out at the
// start of step it - 1), which is more than the exchange takes, so polls rarely repeat.
constexpr int kOncePF = 1, kOnceDB = 3, kOnceDC = 6;
// Slots of the exchange rings.  A block can only publish group g + 8 after every block of its
// cluster has consumed what was published for group g (it needs their H_pre of group
// g + 7 - DC to get that far, and they publish that only after their own step g + 4).
constexpr int kOnceXR = 8;
constexpr int kOnceSpin = 1 << 20;
constexpr int kOnceBlocks = 256;
constexpr int kOnceMaxDevices = 64;

template <int N, int NT>
struct OnceCfg {
  static constexpr int NV = N + 1;                                 // values per token and part: sumsq, N pre-logits
  static constexpr int kSteps = N * (kOnceCB / 32);                // K steps of the block's W slice
  static constexpr int kWVec = kSteps * NT * 2 * 64;               // u32x4
  static constexpr int kRedVec = 8 * (NT + 1) * 64;                // f32x4: [wave][tile][lane]
  // exchange words of a step: at most 64 (token, part) pairs of NV values (a block's tokens
  // times the parts, 4 to 32 of them: 32 at most) and the group's 16 N values of H_pre
  static constexpr int kXwFloats = 64 * NV + kOnceGT * N;
  static constexpr int kLdsBytes = (kWVec + kRedVec) * 16 + (kXwFloats + kOnceGT * NV) * 4;
};

__device__ __forceinline__ void put_word(u64 *p, float v, unsigned tag) {
  __hip_atomic_store(p, (static_cast<u64>(tag) << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 get_word(const u64 *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// `w` holds a first try at p[0..K-1]; polls until every word carries `tag` (bounded), then
// v = the values, or NaN once this lane has given up.
template <int K>
__device__ __forceinline__ void finish_words(const u64 *p, unsigned tag, u64 (&w)[K], float (&v)[K],
                                             bool &bad) {
  auto all_tagged = [&]() {
    bool ok = true;
#pragma unroll
    for (int k = 0; k < K; ++k) ok = ok && static_cast<unsigned>(w[k] >> 32) == tag;
    return ok;
  };
  if (!bad && !all_tagged()) {
    bad = true;
#pragma unroll 1
    for (int spins = 0; spins < kOnceSpin; ++spins) {
      __builtin_amdgcn_s_sleep(1);
#pragma unroll
      for (int k = 0; k < K; ++k) w[k] = get_word(p + k);
      if (all_tagged()) { bad = false; break; }
    }
  }
#pragma unroll
  for (int k = 0; k < K; ++k) v[k] = bad ? NAN : __uint_as_float(static_cast<unsigned>(w[k]));
}

// Barrier for data exchanged through LDS only: this wave's LDS operations are done, its
// outstanding loads and stores stay in flight.  (Written out so that no fence on global memory
// can come with it; for this kernel the compiler emits the same two instructions for
// __syncthreads().)
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory");
  __builtin_amdgcn_sched_barrier(0);
}

template <int N, int NT>
__global__ __launch_bounds__(512, 1) void fwd_once_kernel(
    const uint16_t *__restrict__ x, const u32x4 *__restrict__ Wp, int C, int M, int R, int64_t T,
    const float *__restrict__ b, const float *__restrict__ alpha, float eps, int parts,
    float *__restrict__ u_part, float *__restrict__ sumsq_part, uint16_t *__restrict__ h,
    u64 *__restrict__ l1, u64 *__restrict__ l2) {
  constexpr int PF = kOncePF, DB = kOnceDB, DC = kOnceDC, kOnceRing = PF + 1 + DC;
  using Cfg = OnceCfg<N, NT>;
  constexpr int NV = Cfg::NV;
  extern __shared__ u32x4 lds[];
  u32x4 *wl = lds;                                                  // [kSteps][NT][2][64]
  f32x4 *red = reinterpret_cast<f32x4 *>(lds + Cfg::kWVec);         // [8 waves][NT + 1][64]
  float *xw = reinterpret_cast<float *>(red + Cfg::kRedVec);        // exchange words of the step: [16][NV], then H_pre [16][N]
  float *pub = xw + Cfg::kXwFloats;                                  // [16][NV]: this block's sums of the step's group
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;       // wave = column group of 32
  const int r = lane & 15, q = lane >> 4;
  const int part = blockIdx.x % parts, cluster = blockIdx.x / parts;
  const int nclusters = gridDim.x / parts;
  const int64_t ngroups = (T + kOnceGT - 1) / kOnceGT;
  const int niter = cluster < ngroups ? static_cast<int>((ngroups - 1 - cluster) / nclusters) + 1 : 0;
  if (niter == 0) return;   // (the whole cluster: its blocks exchange only with each other)
  const int col0 = part * kOnceCB + wave * 32 + q * 8;
  const float nC = static_cast<float>(N) * static_cast<float>(C);

  // the block's slice of packed W: rows part*256 .. +255 of every stream
  for (int i = threadIdx.x; i < Cfg::kWVec; i += 512) {
    const int ls = i / (NT * 128), rem = i % (NT * 128);
    const int gstep = ((ls >> 3) * C + part * kOnceCB) / 32 + (ls & 7);
    wl[i] = Wp[static_cast<size_t>(gstep) * (NT * 128) + rem];
  }
  __syncthreads();

  auto group_of = [&](int it) { return cluster + static_cast<int64_t>(it) * nclusters; };
  auto load_piece = [&](u32x4 (&P)[N], int it) {
    int64_t t = group_of(it) * kOnceGT + r;
    if (t > T - 1) t = T - 1;
#pragma unroll
    for (int j = 0; j < N; ++j)
      P[j] = *reinterpret_cast<const u32x4 *>(x + (t * N + j) * C + col0);
  };
  // exchange rings: l1 [slot][cluster][part][token][NV] (what one block publishes per group is
  // one contiguous run: whole lines, two store instructions), l2 [slot][cluster][token][N]
  auto l1_at = [&](int it, int tok, int p) {
    return l1 + (((static_cast<size_t>(it % kOnceXR) * nclusters + cluster) * parts + p) * kOnceGT + tok) * NV;
  };
  auto l2_at = [&](int it, int tok) {
    return l2 + ((static_cast<size_t>(it % kOnceXR) * nclusters + cluster) * kOnceGT + tok) * N;
  };
  // B: block `part` reduces the tokens t of a group with t % parts == part: `nown` of them
  // (none for part >= 16).  Wave 7, lane o N + j -> H_pre[j] of its o-th token.
  constexpr int kPubWords = kOnceGT * NV;                 // what a block publishes per group
  const int nown = part < kOnceGT ? (kOnceGT - 1 - part) / parts + 1 : 0;
  const int bo = (lane / N) < nown ? lane / N : 0, bj = lane % N;
  const bool bpub = lane < nown * N;
  const int btok = part + bo * parts;
  // Polling: what a block reads per step is nown * parts * NV words of l1 (its tokens from
  // every part) and 16 N words of l2 (H_pre of the group); the waves poll equal shares, ONE
  // word per lane, so each wave issues exactly one poll load per step.
  const int kBWords = nown * parts * NV, kWords = kBWords + kOnceGT * N;
  const int kPerWave = (kWords + 7) / 8;                  // <= 64 lanes: parts <= 32
  const int pwi = wave * kPerWave + (lane < kPerWave ? lane : kPerWave - 1);
  const bool pw_live = lane < kPerWave && pwi < kWords;
  const int pw = pwi < kWords ? pwi : kWords - 1;         // this lane's word (past the end: the last one again)
  const bool pw_b = pw < kBWords;
  // word pw < kBWords is value k of part p for the o-th token of this block: pw = (o parts + p) NV + k
  const int pw_k = pw % NV, pw_p = (pw / NV) % parts, pw_tok = part + (pw / (NV * parts)) * parts;

  const float alpha_pre = alpha[1], b_pre = b[R + bj];
  u32x4 P[kOnceRing][N];
  bool bad = false;
  u64 nw[1] = {};            // first try of the word this lane consumes in the next step
  const u64 *np = l1;
  bool nvalid = false;
#pragma unroll
  for (int k = 0; k < PF; ++k) load_piece(P[k], k);   // (clamped re-reads past the cluster's last group)

  auto step = [&](int it, u32x4 (&Pn)[N], const u32x4 (&Pa)[N], const u32x4 (&Pc)[N]) {
    const int ib = it - DB, ic = it - DC;
    const bool doA = it < niter, doB = ib >= 0 && ib < niter, doC = ic >= 0 && ic < niter;
    // The word consumed in this step was requested one step ago; the first try for the NEXT
    // step goes out now, BEFORE this step's loads: results come back in request order, so
    // behind the loads a poll would wait for a whole HBM round trip.  Every lane of every
    // wave issues it (an unused one re-reads word 0), so that the number of loads in flight
    // is the same on every path and the compiler's wait counts stay exact.
    u64 w[1] = {nw[0]};
    const u64 *wp = np;
    const bool wvalid = nvalid;
    {
      const int nb = ib + 1, nc = ic + 1;
      nvalid = pw_b ? (nb >= 0 && nb < niter) : (nc >= 0 && nc < niter);
      np = !nvalid ? l1 : (pw_b ? l1_at(nb, pw_tok, pw_p) + pw_k : l2_at(nc, 0) + (pw - kBWords));
      nw[0] = get_word(np);
    }
    load_piece(Pn, it + PF);   // unconditional (past the last group: clamped re-reads, never used)
    __builtin_amdgcn_sched_barrier(0);

    // ---- A: partial logits and sum of squares of this wave's 32 columns of every stream
    if (doA) {
      f32x4 acc[NT], ss = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < NT; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const int ls = j * 8 + wave;
#pragma unroll
        for (int k = 0; k < NT; ++k) {
          const u32x4 bh = wl[((ls * NT + k) * 2 + 0) * 64 + lane];
          const u32x4 blo = wl[((ls * NT + k) * 2 + 1) * 64 + lane];
          acc[k] = mfma16(Pa[j], bh, acc[k]);
          acc[k] = mfma16(Pa[j], blo, acc[k]);
        }
        ss = mfma16(Pa[j], Pa[j], ss);
      }
#pragma unroll
      for (int k = 0; k < NT; ++k) red[(wave * (NT + 1) + k) * 64 + lane] = acc[k];
      red[(wave * (NT + 1) + NT) * 64 + lane] = ss;
    }
    // this lane's exchange word (requested a step ago) goes to LDS for the block
    {
      float v[1] = {0.f};
      if (wvalid)
        finish_words<1>(wp, static_cast<unsigned>(pw_b ? ib : ic) + 1u, w, v, bad);
      if (pw_live) xw[pw] = v[0];
    }
    lds_barrier();
    if (doA && wave < NT + 1) {   // wave k adds tile k over the eight column groups, in order
      f32x4 v = red[wave * 64 + lane];
#pragma unroll
      for (int c = 1; c < 8; ++c) v += red[(c * (NT + 1) + wave) * 64 + lane];
      const int64_t g0 = group_of(it) * kOnceGT;
      if (wave < NT) {   // D layout: lane (r, q) holds logit 16 wave + r of tokens 4 q + i
        const int m = 16 * wave + r;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = 4 * q + i;
          const int64_t t = g0 + tok;
          if (t < T && m < M) u_part[(static_cast<size_t>(part) * T + t) * M + m] = v[i];
          if (m >= R && m < R + N) pub[tok * NV + 1 + (m - R)] = v[i];
        }
      } else if ((r >> 2) == q) {   // Gram diagonal: token r sits at row 4 q + i
        const int i = r & 3;
        const float s = i == 0 ? v[0] : (i == 1 ? v[1] : (i == 2 ? v[2] : v[3]));
        const int64_t t = g0 + r;
        if (t < T) sumsq_part[static_cast<size_t>(part) * T + t] = s;
        pub[r * NV] = s;
      }
    }
    // ---- B: H_pre of this block's share of group ib from the parts' sums, in part order
    if (wave == 7 && doB) {
      // (in part order, as the coefficient stage adds the slices: that is what makes h agree
      //  with the H_pre the call returns; four parts are read from LDS at a time so that the
      //  reads overlap, the additions stay one chain.  This stage is on the step's critical
      //  path, the other waves wait for it at the barrier below: with one read per part and
      //  addition the kernel took 0.07 ms longer; moving the parts' values between lanes with
      //  DPP row shifts instead of re-reading LDS was slower again.)
      const float *mine = xw + bo * parts * NV;   // [parts][NV] of this lane's token
      float ssq = 0.f, u = 0.f;
      for (int p0 = 0; p0 < parts; p0 += 4) {
        float vs[4], vu[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int pp = p0 + i < parts ? p0 + i : parts - 1;
          vs[i] = mine[pp * NV];
          vu[i] = mine[pp * NV + 1 + bj];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (p0 + i == 0) { ssq = vs[0]; u = vu[0]; }
          else if (p0 + i < parts) { ssq += vs[i]; u += vu[i]; }
        }
      }
      if (bpub) {
        const float rr = 1.f / sqrtf(ssq / nC + eps);
        const float hv = sigmoidf(alpha_pre * (rr * u) + b_pre);
        put_word(l2_at(ib, btok) + bj, hv, static_cast<unsigned>(ib) + 1u);
      }
    }
    // ---- C: h of group ic from the piece loaded DC groups ago
    if (doC) {
      const float *hp = xw + kBWords;   // [16 tokens][N]
      float acc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const float w = hp[r * N + j];
        const u32x4 pv = Pc[j];
        const float v[8] = {bf16lo(pv.x), bf16hi(pv.x), bf16lo(pv.y), bf16hi(pv.y),
                            bf16lo(pv.z), bf16hi(pv.z), bf16lo(pv.w), bf16hi(pv.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += w * v[e];
      }
      const int64_t t = group_of(ic) * kOnceGT + r;
      if (t < T) {
        u32x4 o;
        o.x = pack_bf16x2(acc[0], acc[1]); o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]); o.w = pack_bf16x2(acc[6], acc[7]);
        *reinterpret_cast<u32x4 *>(h + t * C + col0) = o;
      }
    }
    lds_barrier();   // red and xw are rewritten by the next step
    // what this block tells its cluster about group `it`: 16 NV words, contiguous
    if (doA && wave >= 3 && wave < 3 + (kPubWords + 63) / 64) {
      const int i = (wave - 3) * 64 + lane;
      if (i < kPubWords) put_word(l1_at(it, 0, part) + i, pub[i], static_cast<unsigned>(it) + 1u);
    }
  };

  const int total = niter + DC;
#pragma unroll 1
  for (int base = 0; base < total; base += kOnceRing) {
#pragma unroll
    for (int k = 0; k < kOnceRing; ++k) {
      if (base + k < total)
        step(base + k, P[(k + PF) % kOnceRing], P[k], P[(k + PF + 1) % kOnceRing]);
    }
  }
}

template <typename F>
hipError_t dispatch_once(int n, int NT, F &&f) {
  switch (n * 10 + NT) {
    case 21: return f(std::integral_constant<int, 2>{}, std::integral_constant<int, 1>{});
    case 31: return f(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{});
    case 32: return f(std::integral_constant<int, 3>{}, std::integral_constant<int, 2>{});
    case 41: return f(std::integral_constant<int, 4>{}, std::integral_constant<int, 1>{});
    case 42: return f(std::integral_constant<int, 4>{}, std::integral_constant<int, 2>{});
  }
  return hipErrorInvalidValue;
}

// Whether the current device holds 256 blocks of the kernel at once; asked once per device
// and kernel (the answer is cached: 0 unknown, 1 yes, 2 no).
bool device_takes_once(const void *kern, int lds, std::atomic<int> (&cache)[kOnceMaxDevices]) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kOnceMaxDevices) return false;
  // (every time: the attribute belongs to the function on the current device)
  if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
    return false;
  int known = cache[dev].load(std::memory_order_relaxed);
  if (known == 0) {
    int cus = 0, per_cu = 0;
    const bool ok =
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 512, lds) == hipSuccess &&
        static_cast<int64_t>(per_cu) * cus >= kOnceBlocks;
    known = ok ? 1 : 2;
    cache[dev].store(known, std::memory_order_relaxed);
  }
  return known == 1;
}

}  // namespace

bool fwd_once_ok(const mhcl_desc &d) {
  if (!fast_path_ok(d)) return false;
  // the caller's switch: a process that shares the device with other work for long stretches
  // (the kernel wants a compute unit per block) can keep the two-kernel forward
  if (const char *e = getenv("MHCL_FWD_ONCE"); e && e[0] == '0' && e[1] == 0) return false;
  const int M = res_logits(d) + 2 * d.n;
  if (d.n < 2 || d.n > 4 || logit_tiles(M) > 2) return false;
  // 4 to 32 parts (with 64, C = 16384, the per-token stage adds 64 parts' sums per step and
  // the kernel is slower than the two it replaces: 0.57 against 0.45 ms at 8192 tokens)
  if (d.C % kOnceCB != 0 || d.C < 4 * kOnceCB || d.C > 32 * kOnceCB) return false;
  // at least 32 groups per cluster: with fewer the pipeline's fill and drain (DC steps each)
  // cost more than the second read of x (measured at C = 1024: slower at 16 groups, faster at 64)
  return d.T >= 32 * static_cast<int64_t>(kOnceGT) * (kOnceBlocks / (d.C / kOnceCB));
}

OnceWs::OnceWs(const mhcl_desc &d, void *ws) {
  WsCursor c(ws);
  const size_t T = static_cast<size_t>(d.T);
  const int M = res_logits(d) + 2 * d.n;
  parts = d.C / kOnceCB;
  const size_t nclusters = kOnceBlocks / parts;
  u_part = c.take<float>(static_cast<size_t>(parts) * T * M);
  sumsq_part = c.take<float>(static_cast<size_t>(parts) * T);
  Wp = c.take<char>(packed_w_b_bytes(d, M));
  xchg_words = static_cast<size_t>(kOnceXR) * nclusters * kOnceGT * (parts * (d.n + 1) + d.n);
  xchg = c.take<unsigned long long>(xchg_words);
  bytes = c.off;
}

hipError_t prepare_fwd_once(const mhcl_desc &d, int M, bool *usable) {
  *usable = false;
  return dispatch_once(d.n, logit_tiles(M), [&](auto nn, auto nt) {
    constexpr int N = decltype(nn)::value, NT = decltype(nt)::value;
    const void *kern = reinterpret_cast<const void *>(fwd_once_kernel<N, NT>);
    static std::atomic<int> cache[kOnceMaxDevices];   // zero-initialised
    if (!device_takes_once(kern, OnceCfg<N, NT>::kLdsBytes, cache)) return hipSuccess;
    *usable = true;
    return hipSuccess;
  });
}

hipError_t launch_fwd_once(const mhcl_desc &d, int M, const void *x, const float *b,
                           const float *alpha, const OnceWs &w, void *h, hipStream_t s) {
  const int parts = w.parts, nclusters = kOnceBlocks / parts;
  return dispatch_once(d.n, logit_tiles(M), [&](auto nn, auto nt) {
    constexpr int N = decltype(nn)::value, NT = decltype(nt)::value;
    const void *kern = reinterpret_cast<const void *>(fwd_once_kernel<N, NT>);
    constexpr int lds = OnceCfg<N, NT>::kLdsBytes;
    const uint16_t *xa = static_cast<const uint16_t *>(x);
    const u32x4 *wp = reinterpret_cast<const u32x4 *>(w.Wp);
    int C = d.C, Ma = M, R = res_logits(d), pa = parts;
    int64_t T = d.T;
    float eps = d.eps;
    float *up = w.u_part, *sp = w.sumsq_part;
    uint16_t *ha = static_cast<uint16_t *>(h);
    u64 *l1 = w.xchg;
    u64 *l2 = w.xchg + static_cast<size_t>(kOnceXR) * nclusters * kOnceGT * parts * (N + 1);
    const float *ba = b, *aa = alpha;
    void *args[] = {&xa, &wp, &C, &Ma, &R, &T, &ba, &aa, &eps, &pa, &up, &sp, &ha, &l1, &l2};
    // An ordinary launch: with one block per compute unit and nothing else on the device
    // every block is resident at once.  Only the blocks of one cluster depend on each other,
    // and blocks start in index order, so when other work holds compute units the clusters
    // that are complete run to the end and make room; a cluster that is half resident waits
    // for its other half within the bound of its polls (about a second, against well under a
    // millisecond for the whole kernel).  (A cooperative launch would state the requirement
    // to the runtime; it costs 20 us per launch here.)
    return hipLaunchKernel(kern, dim3(nclusters * parts), dim3(512), args, lds, s);
  });
}

}  // namespace mhcl
