// Sparse-KV selection (Sec. 3.2.3, Eq. 4): block logits -> per-row order (score descending) ->
// cumulative softmax mass -> minimal prefix reaching the threshold -> CSR block lists
// (the paper's q2k_num / q2k_index of Sec. 3.3) plus the transposed lists that give every
// KV block a single owner in the backward pass.
//
// Pipeline (all on one stream, no host round trip; nnz stays on the device):
//   1. scores_kernel       s[r][j] = score_scale * <Qbar_r, Kbar_j>, fp64, channel-ascending,
//                          multiply and add rounded separately (the order another
//                          implementation must follow to reproduce every comparison)
//   2. row_select_kernel   one workgroup per row: e = exp(s - s_max), Z, then a bisection for
//                          the key of the last block of the minimal prefix (no sort); marks
//                          the k* selected blocks in a bit mask, writes k*
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

// ---- library-owned scratch for callers that cannot allocate (bsa_select_kv_static) ----------
// One copy per GPU, resident from module load until the process ends.  `scratch` names the
// array only towards hipGetSymbolAddress: in host code the identifier is a host-side stand-in,
// not a device address, so everything below that needs the memory uses the looked-up pointer.
constexpr size_t kStaticScratchBytes = BSA_STATIC_SELECT_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_select_scratch(void** ptr, size_t* bytes) {
  constexpr int kMaxDev = 64;
  static void* dev_ptr[kMaxDev] = {};  // each device holds its own copy at its own address
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return BSA_ERR_LAUNCH;
  if (!dev_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BSA_ERR_LAUNCH;
    dev_ptr[dev] = p;
  }
  *ptr = dev_ptr[dev];
  *bytes = kStaticScratchBytes;
  return BSA_OK;
}

// ---------------------------------------------------------------- 1. block logits
constexpr int TI = 64, TJ = 64, KC = 16;
// A 64 x 64 tile of scores per workgroup, 4 x 4 per thread (rows i0 + 4 ti .., columns
// j0 + 4 tj ..): per channel a thread reads 4 + 4 operands from LDS for 16 multiply-adds.
// Every output is accumulated over the channels in ascending order, multiply and add rounded
// separately, whatever the tiling.
__global__ __launch_bounds__(256) void scores_kernel(Geom g, const double* Qbar, const double* Kbar,
                                                     double scale, double* S) {
  __shared__ __align__(16) double qs[KC][TI + 2];  // +2: conflict-free staging stores, rows stay 16-byte aligned
  __shared__ __align__(16) double ks[KC][TJ + 2];
  const int bh = blockIdx.z;
  const int i0 = blockIdx.y * TI, j0 = blockIdx.x * TJ;
  const int tid = threadIdx.x;
  const int ti = tid / 16, tj = tid % 16;
  const double* Qh = Qbar + (int64_t)bh * g.N * g.d;
  const double* Kh = Kbar + (int64_t)bh * g.N * g.d;
  double acc[4][4] = {};
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
      double q[4], k[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        q[u] = qs[c][4 * ti + u];
        k[u] = ks[c][4 * tj + u];
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[a][u] = __dadd_rn(acc[a][u], __dmul_rn(q[a], k[u]));
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 4 * ti + a, j = j0 + 4 * tj + u;
      if (i < g.N && j < g.N) S[((int64_t)bh * g.N + i) * g.N + j] = __dmul_rn(acc[a][u], scale);
    }
}

// ---------------------------------------------------------------- 2. per-row selection
// Eq. 4 without a sort.  In the order (score descending, block id ascending) the selected set
// is a prefix, so it is fixed by the key of its last element.  Scores map to 64-bit integers
// that order the same way; with G(t) = sum of e_j over keys >= t (non-increasing in t) the
// last selected key is the largest t with G(t) >= p*Z.  It is found by bisection over the
// bits of t, keeping the bracket [lo, hi) with G(lo) >= p*Z > G(hi) and the number of keys
// inside it; the search stops as soon as one key is left (about log2 N steps past the keys'
// common prefix).  More than one key left after the last bit means equal scores: those are
// taken in ascending block id while the mass is short.  Sums run in a fixed order (per lane
// ascending, butterfly across lanes, wavefronts in order), so the result is reproducible;
// it equals the sequential-prefix definition whenever no comparison is within rounding of a
// tie, which the callers' margin check establishes.
__device__ inline unsigned long long order_key(double s) {
  if (s == 0.0) s = 0.0;  // -0 and +0 compare equal
  const unsigned long long u = (unsigned long long)__double_as_longlong(s);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m > 0; m >>= 1) v = __dadd_rn(v, __shfl_xor(v, m));
  return v;
}

template <int NW, int MAXE>
__global__ __launch_bounds__(64 * NW) void row_select_kernel(Geom g, const double* S, double p, double zq,
                                                            uint32_t* mask, int32_t* cnt) {
  constexpr int NT = 64 * NW;
  extern __shared__ __align__(16) uint8_t smem[];
  unsigned long long* lkey = reinterpret_cast<unsigned long long*>(smem);  // [N], for the equal-score path
  __shared__ double red[NW];
  __shared__ int redc[NW];
  __shared__ unsigned long long rk[2][NW];
  __shared__ uint32_t bits[256];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* s = S + (int64_t)row * g.N;
  const int ept = (g.N + NT - 1) / NT;  // elements per thread actually used (<= MAXE): j = e*NT + tid
  const int W = (g.N + 31) / 32;

  auto block_sum = [&](double v) -> double {  // the same value in every thread
    v = wave_sum(v);
    if (NW == 1) return v;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    double t = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t = __dadd_rn(t, red[w]);
    return t;
  };
  // both at once (one pair of barriers): the sum in the same order as block_sum
  auto block_sum_count = [&](double v, int c, double& vs, int& cs) {
    v = wave_sum(v);
    if (NW == 1) {
      vs = v;
      cs = c;
      return;
    }
    __syncthreads();
    if (lane == 0) {
      red[wave] = v;
      redc[wave] = c;
    }
    __syncthreads();
    double t = red[0];
    int tc = redc[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
      t = __dadd_rn(t, red[w]);
      tc += redc[w];
    }
    vs = t;
    cs = tc;
  };
  auto block_max = [&](double v) -> double {
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) v = fmax(v, __shfl_xor(v, m));
    if (NW == 1) return v;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) v = fmax(v, red[w]);
    return v;
  };
  auto block_count = [&](int c) -> int {  // c is wave-uniform
    if (NW == 1) return c;
    __syncthreads();
    if (lane == 0) redc[wave] = c;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += redc[w];
    return t;
  };

  double sv[MAXE];
  double smax = -INFINITY;
#pragma unroll
  for (int e = 0; e < MAXE; ++e) {
    const int j = e * NT + tid;
    sv[e] = (e < ept && j < g.N) ? s[j] : -INFINITY;
    smax = fmax(smax, sv[e]);
  }
  smax = block_max(smax);
  for (int k = tid; k < 256; k += NT) bits[k] = 0u;

  unsigned long long key[MAXE];
  double ev[MAXE];
  double zl = 0.0;
  unsigned long long kmin = ~0ull, kmax = 0ull;
#pragma unroll
  for (int e = 0; e < MAXE; ++e) {
    const int j = e * NT + tid;
    const bool live = e < ept && j < g.N;
    key[e] = live ? order_key(sv[e]) : 0ull;  // padding: below every real key, no mass
    ev[e] = live ? exp(sv[e] - smax) : 0.0;
    zl = __dadd_rn(zl, ev[e]);
    if (live) {
      lkey[j] = key[e];
      kmin = key[e] < kmin ? key[e] : kmin;
      kmax = key[e] > kmax ? key[e] : kmax;
    }
  }
  const double Z = block_sum(zl);
  // smallest and largest key of the row
#pragma unroll
  for (int m = 32; m > 0; m >>= 1) {
    const unsigned long long a = __shfl_xor(kmin, m), b = __shfl_xor(kmax, m);
    kmin = a < kmin ? a : kmin;
    kmax = b > kmax ? b : kmax;
  }
  if (NW > 1) {
    __syncthreads();
    if (lane == 0) { rk[0][wave] = kmin; rk[1][wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      kmin = rk[0][w] < kmin ? rk[0][w] : kmin;
      kmax = rk[1][w] > kmax ? rk[1][w] : kmax;
    }
  }
  auto count_where = [&](unsigned long long lo_incl, bool equal_only) -> int {  // keys >= lo (or == lo)
    int cl = 0;
#pragma unroll
    for (int e = 0; e < MAXE; ++e)
      if (e < ept) cl += __popcll(__ballot(equal_only ? key[e] == lo_incl : key[e] >= lo_incl));
    return block_count(cl);
  };

  // The selection is "every key above `last`, plus the first `need` blocks (ascending id)
  // whose key equals `last`"; `tie` says that several blocks share that key.
  int kstar = g.N, need = 1;
  bool all = true, tie = false;
  unsigned long long last = 0ull;
  if (p < 1.0) {
    all = false;
    const double target = __dmul_rn(p, Z);
    const unsigned long long diff = kmin ^ kmax;
    int b = diff ? 63 - __builtin_clzll(diff) : -1;  // highest bit in which two keys differ
    unsigned long long lo = b >= 0 ? (kmin >> b >> 1 << 1 << b) : kmin;  // keys' common prefix, lower bits zero
    int cnt_lo = g.N, cnt_hi = 0;  // keys >= lo; keys >= hi, hi = lo + 2^(b+1)
    for (; b >= 0 && cnt_lo - cnt_hi > 1; --b) {
      const unsigned long long cand = lo | (1ull << b);
      double gl = 0.0;
      int cl = 0;
#pragma unroll
      for (int e = 0; e < MAXE; ++e) {
        if (e < ept) {
          const bool ge = key[e] >= cand;
          gl = __dadd_rn(gl, ge ? ev[e] : 0.0);
          cl += __popcll(__ballot(ge));
        }
      }
      double G;
      int c;
      block_sum_count(gl, cl, G, c);
      if (G >= target) {
        lo = cand;
        cnt_lo = c;
      } else {
        cnt_hi = c;
      }
    }
    // the keys still inside the bracket [lo, lo + span) are all equal (one key, unless scores tie exactly)
    const unsigned long long span = b >= 0 ? (1ull << b << 1) : 1ull;  // 0 stands for 2^64
    tie = cnt_lo - cnt_hi > 1;
    if (tie) {  // equal scores: add them one at a time, as the sorted prefix would
      double gl = 0.0, el = 0.0;
#pragma unroll
      for (int e = 0; e < MAXE; ++e) {
        if (e < ept) {
          gl = __dadd_rn(gl, key[e] > lo ? ev[e] : 0.0);
          if (key[e] == lo) el = ev[e];
        }
      }
      double c = block_sum(gl);
      el = block_max(el);  // the mass of one tied element (identical in all of them)
      const int tied = cnt_lo - cnt_hi;
      need = 0;
      do {
        c = __dadd_rn(c, el);
        ++need;
      } while (c < target && need < tied);
    }
    kstar = cnt_hi + need;
    // the last selected key: the one key value inside the bracket
    unsigned long long lk = 0ull;
#pragma unroll
    for (int e = 0; e < MAXE; ++e)
      if (e < ept && key[e] >= lo && (span == 0ull || key[e] - lo < span) && key[e] > lk) lk = key[e];
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) {
      const unsigned long long o = __shfl_xor(lk, m);
      lk = o > lk ? o : lk;
    }
    if (NW > 1) {
      __syncthreads();
      if (lane == 0) rk[0][wave] = lk;
      __syncthreads();
#pragma unroll
      for (int w = 0; w < NW; ++w) lk = rk[0][w] > lk ? rk[0][w] : lk;
    }
    last = lk;
  }

  // Eq. 3 (statistical dynamic threshold): only blocks whose score reaches
  // tau = mean + std * zq are candidates; they are a prefix of the same order, so the filter
  // can only shorten the selection.  No candidate: the best block alone.
  if (zq == zq && zq != -INFINITY) {
    double sl = 0.0;
#pragma unroll
    for (int e = 0; e < MAXE; ++e)
      if (e < ept && e * NT + tid < g.N) sl = __dadd_rn(sl, sv[e]);
    const double mean = __ddiv_rn(block_sum(sl), (double)g.N);
    double dl = 0.0;
#pragma unroll
    for (int e = 0; e < MAXE; ++e)
      if (e < ept && e * NT + tid < g.N) {
        const double dvn = __dadd_rn(sv[e], -mean);
        dl = __dadd_rn(dl, __dmul_rn(dvn, dvn));
      }
    const double var = g.N > 1 ? __ddiv_rn(block_sum(dl), (double)(g.N - 1)) : 0.0;
    const double tau = __dadd_rn(mean, __dmul_rn(__dsqrt_rn(var), zq));
    const unsigned long long ktau = order_key(tau);
    const int ncand = tau == tau ? count_where(ktau, false) : 0;
    if (ncand < kstar) {
      all = false;
      if (ncand >= 1) {
        kstar = ncand;
        last = ktau;  // "above last, or equal to it": every key >= ktau
        tie = false;
        need = 1;
      } else {
        kstar = 1;
        last = kmax;
        need = 1;
        tie = count_where(kmax, true) > 1;
      }
    }
  }

  if (!all) {
    if (NW > 1) __syncthreads();  // bits[] cleared by everyone
#pragma unroll
    for (int e = 0; e < MAXE; ++e) {
      const int j = e * NT + tid;
      if (e < ept && j < g.N && (key[e] > last || (!tie && key[e] == last))) atomicOr(&bits[j >> 5], 1u << (j & 31));
    }
    if (tie && tid == 0) {  // equal scores: ascending block id, one thread (rare)
      int left = need;
      for (int j = 0; j < g.N && left > 0; ++j)
        if (lkey[j] == last) {
          atomicOr(&bits[j >> 5], 1u << (j & 31));
          --left;
        }
    }
  }
  __syncthreads();
  for (int w = tid; w < W; w += NT) {
    uint32_t v = bits[w];
    if (all) v = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
    mask[(int64_t)row * W + w] = v;
  }
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

int launch_select(const Geom& g, const double* Qbar, const double* Kbar, double threshold, double stat_z,
                  double score_scale, int32_t* q2k_ptr, int32_t* q2k_idx, int32_t* k2q_ptr,
                  int32_t* k2q_idx, int64_t* nnz_dev, void* ws, hipStream_t st) {
  SelectWs w = carve(g, ws);
  const int BH = g.B * g.H;
  const size_t lds = (size_t)g.N * sizeof(unsigned long long);  // <= 64 KB
  if (g.N > 4096)
    if (int rc = allow_dynamic_lds<row_select_kernel<4, 32>>(lds)) return rc;
  hipLaunchKernelGGL(scores_kernel, dim3((g.N + TJ - 1) / TJ, (g.N + TI - 1) / TI, BH), dim3(256), 0, st,
                     g, Qbar, Kbar, score_scale, w.scores);
  if (g.N <= 1024)
    hipLaunchKernelGGL((row_select_kernel<1, 16>), dim3(g.rows), dim3(64), lds, st, g, w.scores, threshold, stat_z, w.mask, w.cnt);
  else if (g.N <= 4096)
    hipLaunchKernelGGL((row_select_kernel<4, 16>), dim3(g.rows), dim3(256), lds, st, g, w.scores, threshold, stat_z, w.mask, w.cnt);
  else
    hipLaunchKernelGGL((row_select_kernel<4, 32>), dim3(g.rows), dim3(256), lds, st, g, w.scores, threshold, stat_z, w.mask, w.cnt);
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
