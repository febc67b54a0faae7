// Memory-system probe for the hyper-connection path at n = 4, C = 4096, bf16, T = 32768 on gfx950:
// pure traffic skeletons (loads, XORs, stores; no arithmetic of the method) that answer
//   (1) what a read stream reaches by working-set size (L2, memory-side cache, HBM);
//   (2) what the two backward passes' access patterns reach: pass 1 (R: reads x, g_xout, y, g_h,
//       10 rows of C per token), pass 2 (P: reads x, g_xout, g_h, writes g_x, g_y: 9 + 5 rows) as
//       column windows in MFMA lane order, and fully coalesced in row order;
//   (3) whether a token-chunked schedule, in which pass 2 of a chunk re-reads what pass 1 of the
//       same chunk just read (so that the re-read could come from the 256 MB memory-side cache),
//       beats one pass over all tokens followed by the other: as two launches per chunk (SEQ), as
//       one launch per chunk holding pass-1 blocks of chunk j and pass-2 blocks of chunk j-1
//       (MIX), and as one persistent launch in which every block alternates between the two
//       (PERS); the same for the forward (R: reads x; P: reads x, writes h);
//   (4) pass 2 when its reads are warm in the memory-side cache and its writes go to cold HBM.
// Every loop is bounded, there are no waits between blocks, every access is in bounds by
// construction (tokens are clamped to the range, columns are derived from the block index).
//
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 memsys_probe.hip -o memsys_probe
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                        \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
      exit(1);                                                                       \
    }                                                                                \
  } while (0)

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int N = 4, C = 4096, RV = C / 8;   // RV: 16-byte vectors per row of C
constexpr long T = 32768;

struct Bufs {
  const u32x4 *x, *g, *y, *h;
  u32x4 *gx, *gy;
  unsigned *sink;
};

__device__ __forceinline__ void keep(const u32x4 &acc, unsigned *sink) {
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) sink[0] = acc.y;   // never true for these fills
}

// ---- (1) read stream over a buffer of n16 vectors, `passes` times, 8 loads in flight per lane
__global__ __launch_bounds__(256) void read_stream(const u32x4 *__restrict__ p, size_t n16,
                                                    int passes, unsigned *sink) {
  u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * 256;
  for (int ps = 0; ps < passes; ++ps) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
      u32x4 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = p[i + k * stride];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc ^= v[k];
    }
    for (; i < n16; i += stride) acc ^= p[i];
  }
  keep(acc, sink);
}

// ---- pass-1 piece: 128 tokens from t0 (8 waves x 16), columns [kp * C/parts, +C/parts) of every
// row; lane (r, q) reads token r, 16 bytes at 8 q within each 32-column step, two steps back to back
__device__ __forceinline__ void piece_R(const Bufs &b, long t0, long tend, int kp, int parts,
                                        int bwd, u32x4 &acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 15, q = lane >> 4;
  long t = t0 + wave * 16 + r;
  if (t > tend - 1) t = tend - 1;
  const int cw = C / parts, steps = cw / 64;
  const int c0 = (kp * cw) / 8 + q;
  for (int s = 0; s < steps; ++s) {
    // all loads of the step are issued before any is consumed
    u32x4 X[N][2], G[N][2], Y[2], H[2];
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        X[j][u] = b.x[(t * N + j) * RV + c0 + s * 8 + u * 4];
        G[j][u] = bwd ? b.g[(t * N + j) * RV + c0 + s * 8 + u * 4] : acc;
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      Y[u] = bwd ? b.y[t * RV + c0 + s * 8 + u * 4] : acc;
      H[u] = bwd ? b.h[t * RV + c0 + s * 8 + u * 4] : acc;
    }
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) acc ^= X[j][u] ^ G[j][u];
    acc ^= Y[0] ^ Y[1] ^ H[0] ^ H[1];
  }
}

// ---- pass-2 piece, column window of 128 columns (two 64-column slabs x four 16-token waves),
// tokens [ta, tb); reads at token offset rs, writes at token offset ws (to aim at a warm chunk)
__device__ __forceinline__ void piece_P(const Bufs &b, long ta, long tb, long rs, long ws, int win,
                                        int bwd, int rd, int wr, u32x4 &acc) {
  const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3, slab = threadIdx.x >> 8;
  const int r = lane & 15, q = lane >> 4;
  const int cv = (win * 128 + slab * 64) / 8 + q;
  for (long t0 = ta + wave * 16; t0 < tb; t0 += 64) {
    long t = t0 + r;
    const bool live = t < tb;
    if (!live) t = tb - 1;
    u32x4 X[N][2], G[N][2], H[2];
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        X[j][u] = rd ? b.x[((t + rs) * N + j) * RV + cv + u * 4] : acc;
        G[j][u] = (rd && bwd) ? b.g[((t + rs) * N + j) * RV + cv + u * 4] : acc;
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) H[u] = (rd && bwd) ? b.h[(t + rs) * RV + cv + u * 4] : acc;
    if (wr && live) {
      if (bwd) {
#pragma unroll
        for (int j = 0; j < N; ++j)
#pragma unroll
          for (int u = 0; u < 2; ++u) b.gx[((t + ws) * N + j) * RV + cv + u * 4] = X[j][u] ^ G[j][u] ^ H[u];
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) b.gy[(t + ws) * RV + cv + u * 4] = X[0][u] ^ X[1][u] ^ G[2][u] ^ G[3][u];
    }
    if (!wr) {
#pragma unroll
      for (int j = 0; j < N; ++j)
#pragma unroll
        for (int u = 0; u < 2; ++u) acc ^= X[j][u] ^ G[j][u];
      acc ^= H[0] ^ H[1];
    }
  }
}

// One launch: blocks [0, nR) are pass-1 pieces of tokens [r0, r1) (token group = block / parts,
// column part = block % parts); the next nP blocks are pass-2 pieces of tokens [p0, p1), 32
// windows x psub token ranges.  `persist`: every block instead loops over chunks j of Tc tokens,
// doing its pass-1 pieces of chunk j and then its pass-2 pieces of chunk j - 1.
__global__ __launch_bounds__(512, 1) void sched(Bufs b, long r0, long r1, int nR, int parts, long p0,
                                                long p1, int psub, int bwd, int rd, int wr,
                                                long warm, int persist, long Tc) {
  extern __shared__ unsigned pad[];   // sized by the host so that one block fits a compute unit
  pad[threadIdx.x] = threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  if (!persist) {
    int blk = blockIdx.x;
    if (blk < nR) {
      piece_R(b, r0 + (long)(blk / parts) * 128, r1, blk % parts, parts, bwd, acc);
    } else {
      blk -= nR;
      const long per = ((p1 - p0 + psub - 1) / psub + 63) / 64 * 64;
      const long ta = p0 + (blk / 32) * per, tb = ta + per > p1 ? p1 : ta + per;
      // warm >= 0: read (and, if wr == 2, write) the fixed chunk starting at token `warm` instead
      const long rs = warm >= 0 ? warm - p0 : 0;
      if (ta < tb) piece_P(b, ta, tb, rs, wr == 2 ? rs : 0, blk % 32, bwd, rd, wr, acc);
    }
  } else {
    const int nch = (int)((T + Tc - 1) / Tc);
    const int rpieces = (int)((Tc + 127) / 128) * parts, ppieces = 32 * psub;
    const long per = ((Tc + psub - 1) / psub + 63) / 64 * 64;
    for (int j = 0; j <= nch; ++j) {
      if (j < nch) {
        const long a = (long)j * Tc, e = a + Tc > T ? T : a + Tc;
        for (int p = blockIdx.x; p < rpieces; p += gridDim.x) {
          const long t0 = a + (long)(p / parts) * 128;
          if (t0 < e) piece_R(b, t0, e, p % parts, parts, bwd, acc);
        }
      }
      if (j > 0) {
        const long a = (long)(j - 1) * Tc, e = a + Tc > T ? T : a + Tc;
        for (int p = blockIdx.x; p < ppieces; p += gridDim.x) {
          const long ta = a + (p / 32) * per, tb = ta + per > e ? e : ta + per;
          if (ta < tb) piece_P(b, ta, tb, 0, 0, p % 32, bwd, 1, 1, acc);
        }
      }
    }
  }
  keep(acc, b.sink);
  if (pad[(threadIdx.x + 1) & 255] == 0xFFFFFFFFu) b.sink[1] = 1;
}

// ---- pass 2, fully coalesced in row order: one thread per 16-byte vector of a token's row
__global__ __launch_bounds__(256) void pass2_flat(Bufs b, int wr) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * RV) return;
  const long t = idx / RV;
  const int c = (int)(idx % RV);
  u32x4 X[N], G[N], H = b.h[t * RV + c];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    X[j] = b.x[(t * N + j) * RV + c];
    G[j] = b.g[(t * N + j) * RV + c];
  }
  if (wr) {
#pragma unroll
    for (int j = 0; j < N; ++j) b.gx[(t * N + j) * RV + c] = X[j] ^ G[j] ^ H;
    b.gy[t * RV + c] = G[0] ^ G[1] ^ G[2] ^ G[3];
  } else {
    u32x4 acc = H;
#pragma unroll
    for (int j = 0; j < N; ++j) acc ^= X[j] ^ G[j];
    keep(acc, b.sink);
  }
}

int main() {
  const size_t xb = (size_t)T * N * C * 2, yb = (size_t)T * C * 2, slack = 4096;
  char *px, *pg, *py, *ph, *pgx, *pgy;
  unsigned *sink;
  CK(hipMalloc(&px, xb + slack)); CK(hipMalloc(&pg, xb + slack)); CK(hipMalloc(&py, yb + slack));
  CK(hipMalloc(&ph, yb + slack)); CK(hipMalloc(&pgx, xb + slack)); CK(hipMalloc(&pgy, yb + slack));
  CK(hipMalloc(&sink, 64));
  CK(hipMemset(px, 1, xb + slack)); CK(hipMemset(pg, 2, xb + slack)); CK(hipMemset(py, 3, yb + slack));
  CK(hipMemset(ph, 4, yb + slack)); CK(hipMemset(pgx, 0, xb + slack)); CK(hipMemset(pgy, 0, yb + slack));
  // placed as the library's Python layer places them: g_xout 256 B, g_x 512 B past a 1 KiB boundary
  Bufs b;
  b.x = (const u32x4 *)px; b.g = (const u32x4 *)(pg + 256); b.y = (const u32x4 *)py;
  b.h = (const u32x4 *)ph; b.gx = (u32x4 *)(pgx + 512); b.gy = (u32x4 *)(pgy + 768); b.sink = sink;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  auto best_ms = [&](auto &&f) {
    f();
    CK(hipDeviceSynchronize());
    float best = 1e9f;
    for (int rep = 0; rep < 5; ++rep) {
      CK(hipEventRecord(e0)); f(); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      best = ms < best ? ms : best;
    }
    CK(hipGetLastError());
    return best;
  };
  const int lds = 96 * 1024;
  CK(hipFuncSetAttribute((const void *)sched, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  const double U = (double)T * C * 2;   // bytes of one row of C over all tokens

  printf("## 1. read stream by working-set size (GB/s; 2048 blocks x 256 lanes, 8 x 16 B in flight per lane)\n");
  for (size_t mb : {8, 16, 32, 64, 128, 192, 256, 512, 1024}) {
    const size_t bytes = mb << 20;
    const int passes = (int)(((size_t)4 << 30) / bytes);
    const float ms = best_ms([&] {
      hipLaunchKernelGGL(read_stream, dim3(2048), dim3(256), 0, 0, (const u32x4 *)px, bytes / 16, passes, sink);
    });
    printf("working set %5zu MiB: %8.0f GB/s\n", mb, (double)bytes * passes / ms / 1e6);
    fflush(stdout);
  }

  auto one = [&](int nR, int parts, long r0, long r1, int nP, int psub, long p0, long p1, int bwd, int rd,
                 int wr, long warm) {
    hipLaunchKernelGGL(sched, dim3(nR + nP), dim3(512), lds, 0, b, r0, r1, nR, parts, p0, p1, psub, bwd, rd, wr,
                       warm, 0, 0L);
  };
  for (int bwd : {1, 0}) {
    const double ru = bwd ? 10 : 4, pr = bwd ? 9 : 4, pw = bwd ? 5 : 1;
    printf("\n## 2%s. %s: pass 1 reads %gU, pass 2 reads %gU and writes %gU (U = %.0f MiB)\n", bwd ? "b" : "f",
           bwd ? "backward" : "forward", ru, pr, pw, U / 1048576);
    const float r_ms = best_ms([&] { one((int)(T / 128), 1, 0, T, 0, 1, 0, 0, bwd, 1, 1, -1); });
    printf("pass 1, 128-token blocks walking whole rows            : %.3f ms  %5.0f GB/s\n", r_ms, ru * U / r_ms / 1e6);
    const float p_ms = best_ms([&] { one(0, 1, 0, 0, 256, 8, 0, T, bwd, 1, 1, -1); });
    printf("pass 2, column windows (32 x 8 token ranges)            : %.3f ms  %5.0f GB/s\n", p_ms, (pr + pw) * U / p_ms / 1e6);
    const float pr_ms = best_ms([&] { one(0, 1, 0, 0, 256, 8, 0, T, bwd, 1, 0, -1); });
    printf("pass 2, reads only                                      : %.3f ms  %5.0f GB/s\n", pr_ms, pr * U / pr_ms / 1e6);
    const float pw_ms = best_ms([&] { one(0, 1, 0, 0, 256, 8, 0, T, bwd, 0, 1, -1); });
    printf("pass 2, writes only                                     : %.3f ms  %5.0f GB/s\n", pw_ms, pw * U / pw_ms / 1e6);
    if (bwd) {
      const float f_ms = best_ms([&] { hipLaunchKernelGGL(pass2_flat, dim3((unsigned)(T * RV / 256)), dim3(256), 0, 0, b, 1); });
      printf("pass 2, fully coalesced row order                       : %.3f ms  %5.0f GB/s\n", f_ms, 14 * U / f_ms / 1e6);
      const float fr_ms = best_ms([&] { hipLaunchKernelGGL(pass2_flat, dim3((unsigned)(T * RV / 256)), dim3(256), 0, 0, b, 0); });
      printf("pass 2, fully coalesced row order, reads only           : %.3f ms  %5.0f GB/s\n", fr_ms, 9 * U / fr_ms / 1e6);
    }
    // (4) reads warm in the memory-side cache: 32 launches that all read tokens 0..1023, writes walk on
    const float w_ms = best_ms([&] {
      for (int j = 0; j < 32; ++j) one(0, 1, 0, 0, 256, 8, j * 1024L, (j + 1) * 1024L, bwd, 1, 1, 0);
    });
    const float c_ms = best_ms([&] {
      for (int j = 0; j < 32; ++j) one(0, 1, 0, 0, 256, 8, j * 1024L, (j + 1) * 1024L, bwd, 1, 1, -1);
    });
    printf("pass 2 as 32 launches of 1024 tokens, all cold          : %.3f ms\n", c_ms);
    printf("pass 2 as 32 launches, reads of one warm 1024-token chunk: %.3f ms\n", w_ms);
    printf("one pass after the other over all tokens (the baseline) : %.3f ms\n", r_ms + p_ms);
    fflush(stdout);
    // (3) chunked schedules
    for (long Tc : {1024L, 2048L}) {
      const int nch = (int)(T / Tc);
      for (int parts : {16, 32}) {
        const int nR = (int)(Tc / 128) * parts, nP = 256, psub = 8;
        const float seq = best_ms([&] {
          for (int j = 0; j < nch; ++j) {
            one(nR, parts, j * Tc, (j + 1) * Tc, 0, 1, 0, 0, bwd, 1, 1, -1);
            one(0, 1, 0, 0, nP, psub, j * Tc, (j + 1) * Tc, bwd, 1, 1, -1);
          }
        });
        const float mix = best_ms([&] {
          for (int j = 0; j <= nch; ++j)
            one(j < nch ? nR : 0, parts, j < nch ? j * Tc : 0, j < nch ? (j + 1) * Tc : 0, j > 0 ? nP : 0, psub,
                j > 0 ? (j - 1) * Tc : 0, j > 0 ? j * Tc : 0, bwd, 1, 1, -1);
        });
        const float pers = best_ms([&] {
          hipLaunchKernelGGL(sched, dim3(256), dim3(512), lds, 0, b, 0L, 0L, 0, parts, 0L, 0L, psub, bwd, 1, 1, -1L, 1, Tc);
        });
        printf("chunks of %4ld tokens, pass 1 split in %2d column parts    : SEQ %.3f  MIX %.3f  PERS %.3f ms\n", Tc,
               parts, seq, mix, pers);
        fflush(stdout);
      }
    }
  }
  return 0;
}
