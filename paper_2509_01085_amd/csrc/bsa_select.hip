// Sparse-KV selection (Sec. 3.2.3, Eq. 4): block logits -> per-row descending sort ->
// cumulative softmax mass -> minimal prefix reaching the threshold -> CSR block lists
// (the paper's q2k_num / q2k_index of Sec. 3.3) plus the transposed lists that give every
// KV block a single owner in the backward pass.
//
// Pipeline (all on one stream, no host round trip; nnz stays on the device):
//   1. scores_kernel       s[r][j] = score_scale * <Qbar_r, Kbar_j>, fp64, channel-ascending,
//                          multiply and add rounded separately (the order another
//                          implementation must follow to reproduce every comparison)
//   2. row_select_kernel   one workgroup per row: bitonic sort in LDS on (s desc, j asc),
//                          e = exp(s - s_max), scan, k* = 1 + #{c_k < p*Z}; marks the k*
//                          leading blocks in a bit mask, writes k*
//   3. scan_kernel         exclusive scan of the counts -> q2k_ptr, nnz
//   4. expand_kernel       bit mask -> ascending block ids at q2k_ptr[r]
//   5-7. transpose         per (head, 32 columns): ballot-count, scan, ballot-fill -> k2q
#include <math.h>

#include "bsa_common.h"

namespace bsa {

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct SelectWs {
  double* scores;   // [rows][N]
  uint32_t* mask;   // [rows][W]
  int32_t* cnt;     // [rows]  q2k counts
  int32_t* kcnt;    // [rows]  k2q counts
  size_t bytes;
};

static SelectWs carve(const Geom& g, void* base) {
  SelectWs w;
  const size_t W = (g.N + 31) / 32;
  size_t off = 0;
  uint8_t* p = static_cast<uint8_t*>(base);
  w.scores = reinterpret_cast<double*>(p + off); off += align256((size_t)g.rows * g.N * sizeof(double));
  w.mask = reinterpret_cast<uint32_t*>(p + off); off += align256((size_t)g.rows * W * 4);
  w.cnt = reinterpret_cast<int32_t*>(p + off); off += align256((size_t)g.rows * 4);
  w.kcnt = reinterpret_cast<int32_t*>(p + off); off += align256((size_t)g.rows * 4);
  w.bytes = off;
  return w;
}

size_t select_workspace_bytes(const Geom& g) { return carve(g, nullptr).bytes; }

// ---------------------------------------------------------------- 1. block logits
constexpr int TI = 32, TJ = 64, KC = 16;

__global__ __launch_bounds__(256) void scores_kernel(Geom g, const double* Qbar, const double* Kbar,
                                                     double scale, double* S) {
  __shared__ double qs[KC][TI + 1];
  __shared__ double ks[KC][TJ + 1];
  const int bh = blockIdx.z;
  const int i0 = blockIdx.y * TI, j0 = blockIdx.x * TJ;
  const int tid = threadIdx.x;
  const int ti = tid / 16, tj = tid % 16;  // outputs: rows i0 + 2*ti + {0,1}, cols j0 + tj + 16*{0..3}
  const double* Qh = Qbar + (int64_t)bh * g.N * g.d;
  const double* Kh = Kbar + (int64_t)bh * g.N * g.d;
  double acc[2][4] = {};
  for (int c0 = 0; c0 < g.d; c0 += KC) {
    __syncthreads();
    for (int e = tid; e < TI * KC; e += 256) {
      const int r = e / KC, c = e % KC;
      qs[c][r] = (i0 + r < g.N && c0 + c < g.d) ? Qh[(int64_t)(i0 + r) * g.d + c0 + c] : 0.0;
    }
    for (int e = tid; e < TJ * KC; e += 256) {
      const int r = e / KC, c = e % KC;
      ks[c][r] = (j0 + r < g.N && c0 + c < g.d) ? Kh[(int64_t)(j0 + r) * g.d + c0 + c] : 0.0;
    }
    __syncthreads();
    const int kc = min(KC, g.d - c0);
    for (int c = 0; c < kc; ++c) {
      const double q0 = qs[c][2 * ti], q1 = qs[c][2 * ti + 1];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const double k = ks[c][tj + 16 * u];
        acc[0][u] = __dadd_rn(acc[0][u], __dmul_rn(q0, k));
        acc[1][u] = __dadd_rn(acc[1][u], __dmul_rn(q1, k));
      }
    }
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 2 * ti + a, j = j0 + tj + 16 * u;
      if (i < g.N && j < g.N) S[((int64_t)bh * g.N + i) * g.N + j] = __dmul_rn(acc[a][u], scale);
    }
}

// ---------------------------------------------------------------- 2. per-row selection
__device__ inline bool before(double sa, int ja, double sb, int jb) {
  return sa > sb || (sa == sb && ja < jb);
}

__global__ __launch_bounds__(256) void row_select_kernel(Geom g, const double* S, double p, int P,
                                                         uint32_t* mask, int32_t* cnt) {
  extern __shared__ __align__(16) uint8_t smem[];
  double* key = reinterpret_cast<double*>(smem);        // [P]
  int* idx = reinterpret_cast<int*>(key + P);           // [P]
  __shared__ double tot[256];
  __shared__ uint32_t bits[256];
  __shared__ int below;
  const int row = blockIdx.x, tid = threadIdx.x;
  const double* s = S + (int64_t)row * g.N;
  for (int k = tid; k < P; k += 256) {
    key[k] = k < g.N ? s[k] : -INFINITY;
    idx[k] = k;
  }
  bits[tid] = 0;
  if (tid == 0) below = 0;
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < P / 2; t += 256) {
        const int lo = (t / j) * 2 * j + (t % j), hi = lo + j;
        const bool up = (lo & k) == 0;
        const double sl = key[lo], sh = key[hi];
        const int jl = idx[lo], jh = idx[hi];
        const bool hi_first = before(sh, jh, sl, jl);
        if (hi_first == up) {
          key[lo] = sh; key[hi] = sl;
          idx[lo] = jh; idx[hi] = jl;
        }
      }
      __syncthreads();
    }
  }
  // masses relative to the row maximum, in sorted order; padding carries no mass
  const double smax = key[0];
  __syncthreads();
  const int seg = P / 256 > 0 ? P / 256 : 1;  // P is a power of two >= 256
  const int k0 = tid * seg;
  double run = 0.0;
  for (int k = k0; k < k0 + seg; ++k) {
    const double e = k < g.N ? exp(key[k] - smax) : 0.0;
    run = __dadd_rn(run, e);
    key[k] = run;  // inclusive sum inside the segment
  }
  tot[tid] = run;
  __syncthreads();
  double off = 0.0, Z = 0.0;
  for (int u = 0; u < 256; ++u) {
    const double v = tot[u];
    if (u < tid) off = __dadd_rn(off, v);
    Z = __dadd_rn(Z, v);
  }
  int kstar = g.N;
  if (p < 1.0) {
    const double target = __dmul_rn(p, Z);
    int mine = 0;
    for (int k = k0; k < k0 + seg; ++k)
      if (k < g.N && __dadd_rn(off, key[k]) < target) ++mine;
    if (mine) atomicAdd(&below, mine);
    __syncthreads();
    kstar = min(below + 1, g.N);
  }
  for (int k = tid; k < kstar; k += 256) {
    const int j = idx[k];
    atomicOr(&bits[j >> 5], 1u << (j & 31));
  }
  __syncthreads();
  const int W = (g.N + 31) / 32;
  if (tid < W) mask[(int64_t)row * W + tid] = bits[tid];
  if (tid == 0) cnt[row] = kstar;
}

// ---------------------------------------------------------------- 3. exclusive scan
__global__ __launch_bounds__(1024) void scan_kernel(const int32_t* cnt, int n, int32_t* ptr, int64_t* total) {
  __shared__ int part[1024];
  const int tid = threadIdx.x;
  const int seg = (n + 1023) / 1024;
  const int a = min(n, tid * seg), b = min(n, a + seg);
  int s = 0;
  for (int k = a; k < b; ++k) s += cnt[k];
  part[tid] = s;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {  // inclusive Hillis-Steele over the 1024 partials
    const int v = tid >= o ? part[tid - o] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  int run = part[tid] - s;
  for (int k = a; k < b; ++k) {
    ptr[k] = run;
    run += cnt[k];
  }
  if (tid == 1023) {
    ptr[n] = part[1023];
    if (total) *total = part[1023];
  }
}

// ---------------------------------------------------------------- 4. mask -> ascending ids
__global__ __launch_bounds__(256) void expand_kernel(Geom g, const uint32_t* mask, const int32_t* ptr,
                                                     int32_t* out) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= g.rows) return;
  const int W = (g.N + 31) / 32;
  int base = ptr[row];
  for (int w0 = 0; w0 < W; w0 += 64) {
    const int w = w0 + lane;
    uint32_t word = w < W ? mask[(int64_t)row * W + w] : 0u;
    const int pc = __popc(word);
    int incl = pc;
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    int pos = base + incl - pc;
    while (word) {
      const int b = __ffs(word) - 1;
      out[pos++] = w * 32 + b;
      word &= word - 1;
    }
    base += __shfl(incl, 63);
  }
}

// ---------------------------------------------------------------- 5-7. transpose
// One wavefront per (head, group of 32 KV blocks).  FILL=false counts the listing query
// blocks of each column; FILL=true writes them, ascending, at k2q_ptr[column].
template <bool FILL>
__global__ __launch_bounds__(256) void transpose_kernel(Geom g, const uint32_t* mask, int32_t* kcnt,
                                                        const int32_t* kptr, int32_t* kidx) {
  const int lane = threadIdx.x & 63;
  const int W = (g.N + 31) / 32;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= g.B * g.H * W) return;
  const int bh = unit / W, w = unit % W;
  const int col = w * 32 + (lane & 31);
  int acc = 0;  // lane b < 32: running count (or write cursor) of column w*32 + b
  if (FILL && lane < 32 && col < g.N) acc = kptr[(int64_t)bh * g.N + col];
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int i0 = 0; i0 < g.N; i0 += 64) {
    const int i = i0 + lane;
    const uint32_t word = i < g.N ? mask[((int64_t)bh * g.N + i) * W + w] : 0u;
#pragma unroll 4
    for (int b = 0; b < 32; ++b) {
      const bool set = (word >> b) & 1u;
      const unsigned long long m = __ballot(set);
      if (FILL) {
        const int cursor = __shfl(acc, b);
        if (set) kidx[cursor + __popcll(m & lt)] = i;
      }
      if (lane == b) acc += __popcll(m);
    }
  }
  if (!FILL && lane < 32 && col < g.N) kcnt[(int64_t)bh * g.N + col] = acc;
}

int launch_select(const Geom& g, const double* Qbar, const double* Kbar, double threshold,
                  double score_scale, int32_t* q2k_ptr, int32_t* q2k_idx, int32_t* k2q_ptr,
                  int32_t* k2q_idx, int64_t* nnz_dev, void* ws, hipStream_t st) {
  SelectWs w = carve(g, ws);
  const int BH = g.B * g.H;
  hipLaunchKernelGGL(scores_kernel, dim3((g.N + TJ - 1) / TJ, (g.N + TI - 1) / TI, BH), dim3(256), 0, st,
                     g, Qbar, Kbar, score_scale, w.scores);
  int P = 256;
  while (P < g.N) P <<= 1;
  const size_t lds = (size_t)P * (sizeof(double) + sizeof(int));
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(row_select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return BSA_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(row_select_kernel, dim3(g.rows), dim3(256), lds, st, g, w.scores, threshold, P,
                     w.mask, w.cnt);
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, st, w.cnt, g.rows, q2k_ptr, nnz_dev);
  hipLaunchKernelGGL(expand_kernel, dim3((g.rows + 3) / 4), dim3(256), 0, st, g, w.mask, q2k_ptr, q2k_idx);
  if (k2q_ptr) {
    const int W = (g.N + 31) / 32;
    const int units = BH * W;
    hipLaunchKernelGGL(transpose_kernel<false>, dim3((units + 3) / 4), dim3(256), 0, st, g, w.mask, w.kcnt,
                       (const int32_t*)nullptr, (int32_t*)nullptr);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, st, w.kcnt, g.rows, k2q_ptr, (int64_t*)nullptr);
    hipLaunchKernelGGL(transpose_kernel<true>, dim3((units + 3) / 4), dim3(256), 0, st, g, w.mask, w.kcnt,
                       k2q_ptr, k2q_idx);
  }
  return check_launch();
}

}  // namespace bsa
