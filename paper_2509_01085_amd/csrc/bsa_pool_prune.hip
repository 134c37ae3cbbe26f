// Streaming kernels of the index-preparation stage: block mean pooling (Sec. 3.2.3) and
// query pruning by cosine similarity to the block center (Sec. 3.2.2, Eq. 2).
//
// Both are one pass over a [B,H,L,d] tensor and are bound by HBM bandwidth: a wavefront
// owns one 3D block (Bk token rows in Cw-token runs of contiguous memory) and does the fp64
// decision arithmetic on it.
//
// Bit-exactness contract with any other implementation of the same definition: sums run
// in ascending index order (tokens for pooling, channels for dot products) in fp64.  The
// inputs are fp32 or bf16, so every product of two inputs is exact in fp64 and a fused
// multiply-add rounds exactly like multiply-then-add; cos = dot / sqrt(|a|^2 * |c|^2) uses
// IEEE fp64 multiply, sqrt and divide.
#include "bsa_common.h"

namespace bsa {

// One wavefront per 3D block in both kernels, no workgroup barriers: many independent
// wavefronts per CU keep enough loads in flight to stream at HBM rate.

constexpr int kWaves = 4;  // wavefronts (= blocks) per workgroup

template <int ES>
__device__ inline void unpack(uint32_t w, double& lo, double& hi) {  // ES == 2: two bf16 channels of a word
  lo = (double)__uint_as_float(w << 16);
  hi = (double)__uint_as_float(w & 0xffff0000u);
}

// ------------------------------------------------------------------------------ pooling
// Lane l owns the 32-bit words l, l + 64, ... of a token row (two bf16 channels or one fp32
// channel each): every load instruction of the wavefront reads one token's row segment,
// contiguous in memory, and the per-channel sums run over the tokens in ascending
// intra-block id, in registers.  No LDS.
template <int ES>
__global__ __launch_bounds__(64 * kWaves) void pool_kernel(Geom g, const uint8_t* X, double* Xbar) {
  constexpr int TB = 16;                // token rows loaded ahead of the additions
  __shared__ int koff[256];
  for (int t = threadIdx.x; t < g.Bk; t += 64 * kWaves) koff[t] = intra_offset(g, t);
  __syncthreads();  // the only workgroup barrier
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);  // (b*H + h)*N + i
  if (row >= g.rows) return;
  const int64_t bh = row / g.N;
  const int i = (int)(row % g.N);
  const int words = g.d * ES / 4;
  const int nk = (words + 63) / 64;  // words per lane in use
  const uint32_t* base = reinterpret_cast<const uint32_t*>(X) + (bh * g.L + block_origin(g, i)) * (int64_t)words;
#pragma unroll 1
  for (int k = 0; k < nk; ++k) {  // (one pass for d <= 128 bf16 / d <= 64 fp32)
    const int w = lane + 64 * k;
    const bool live = w < words;
    double a0 = 0.0, a1 = 0.0;
    for (int r0 = 0; r0 < g.Bk; r0 += TB) {
      uint32_t v[TB];
#pragma unroll
      for (int u = 0; u < TB; ++u)
        v[u] = (live && r0 + u < g.Bk) ? base[(int64_t)koff[min(r0 + u, g.Bk - 1)] * words + w] : 0u;
#pragma unroll
      for (int u = 0; u < TB; ++u) {
        if (r0 + u < g.Bk) {  // ascending intra-block id
          if (ES == 4) {
            a0 = __dadd_rn(a0, (double)__uint_as_float(v[u]));
          } else {
            double lo, hi;
            unpack<ES>(v[u], lo, hi);
            a0 = __dadd_rn(a0, lo);
            a1 = __dadd_rn(a1, hi);
          }
        }
      }
    }
    if (live) {
      const double bk = (double)g.Bk;
      if (ES == 4) {
        Xbar[row * g.d + w] = __ddiv_rn(a0, bk);
      } else {
        double2 o;
        o.x = __ddiv_rn(a0, bk);
        o.y = __ddiv_rn(a1, bk);
        *reinterpret_cast<double2*>(Xbar + row * g.d + 2 * w) = o;
      }
    }
  }
}

// ------------------------------------------------------------------------------ pruning
// Lane t owns token t of the block (Bk > 64: several passes).  The token rows pass through a
// per-wavefront LDS tile in groups of up to 8 sixteen-byte chunks: loaded row-contiguous
// (coalesced), read back one row per lane; the dot product with the center of the token's
// window and the two squared norms accumulate over the channels in ascending order across the
// groups.  Ranking and quota are per window (Sec. 3.2.2, "Critical Token"); one window per
// block is the single-center method.
constexpr int kGroup = 8;                          // chunks of a row staged at a time
constexpr int kRowStride = kGroup * 16 + 16;       // LDS bytes per staged row (padded: lanes 16 apart share banks, the b128 minimum)
constexpr int kTileBytes = 64 * kRowStride;

__device__ inline void wave_lds_sync() {  // LDS written by other lanes of this wavefront becomes readable
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int ES>
__global__ __launch_bounds__(64 * kWaves) void prune_kernel(Geom g, const uint8_t* Q, int kw,
                                                           int32_t* keep_idx) {
  __shared__ __align__(16) uint8_t tiles[kWaves][kTileBytes];
  __shared__ double cosv[kWaves][256];
  __shared__ int koff[256];
  __shared__ short wid[256];   // window of every intra-block token
  __shared__ short wcen[256];  // critical token of that window (intra-block id)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t = threadIdx.x; t < g.Bk; t += 64 * kWaves) {
    koff[t] = intra_offset(g, t);
    const int w = window_of(g, t);
    wid[t] = (short)w;
    wcen[t] = (short)window_center(g, w);
  }
  __syncthreads();  // the only workgroup barrier; wavefronts are independent from here on
  const int64_t row = (int64_t)blockIdx.x * kWaves + wave;
  if (row >= g.rows) return;
  const int64_t bh = row / g.N;
  const int i = (int)(row % g.N);
  const int row_bytes = g.d * ES, cpr = row_bytes / 16;
  const int n_keep = kw * g.nwin;
  const uint8_t* base = Q + (bh * g.L + block_origin(g, i)) * (int64_t)row_bytes;
  uint8_t* tile = tiles[wave];

  for (int t0 = 0; t0 < g.Bk; t0 += 64) {
    const int nt = min(64, g.Bk - t0);
    const int cen = wcen[min(t0 + lane, g.Bk - 1)];  // this lane's window center
    const bool cen_staged = cen >= t0 && cen < t0 + nt;  // its row is part of this pass's tile
    double dot = 0.0, na2 = 0.0, nc2 = 0.0;  // <q, q_c>, |q|^2, |q_c|^2: channels ascending
    for (int q0 = 0; q0 < cpr; q0 += kGroup) {
      const int nq = min(kGroup, cpr - q0);
      wave_lds_sync();  // everyone is done reading the previous group
      {  // all loads of the group first (at most 64 * kGroup / 64 = kGroup per lane), then the LDS writes
        uint4 val[kGroup];
#pragma unroll
        for (int n = 0; n < kGroup; ++n) {
          const int v = lane + 64 * n, r = min(v / nq, nt - 1), q = v - (v / nq) * nq;
          val[n] = *reinterpret_cast<const uint4*>(base + (int64_t)koff[t0 + r] * row_bytes + 16 * (q0 + q));
        }
#pragma unroll
        for (int n = 0; n < kGroup; ++n) {
          const int v = lane + 64 * n, r = v / nq, q = v - r * nq;
          if (v < nt * nq) *reinterpret_cast<uint4*>(tile + r * kRowStride + 16 * q) = val[n];
        }
      }
      wave_lds_sync();
      if (lane < nt) {
        for (int q = 0; q < nq; ++q) {
          const uint4 xv = *reinterpret_cast<const uint4*>(tile + lane * kRowStride + 16 * q);
          const uint4 cv = cen_staged
                               ? *reinterpret_cast<const uint4*>(tile + (cen - t0) * kRowStride + 16 * q)
                               : *reinterpret_cast<const uint4*>(base + (int64_t)koff[cen] * row_bytes + 16 * (q0 + q));
          const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w}, cw[4] = {cv.x, cv.y, cv.z, cv.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (ES == 4) {
              const double x = (double)__uint_as_float(xw[e]), c = (double)__uint_as_float(cw[e]);
              dot = fma(x, c, dot);
              na2 = fma(x, x, na2);
              nc2 = fma(c, c, nc2);
            } else {
              double xl, xh, cl, ch;
              unpack<ES>(xw[e], xl, xh);
              unpack<ES>(cw[e], cl, ch);
              dot = fma(xl, cl, dot);
              na2 = fma(xl, xl, na2);
              nc2 = fma(cl, cl, nc2);
              dot = fma(xh, ch, dot);
              na2 = fma(xh, xh, na2);
              nc2 = fma(ch, ch, nc2);
            }
          }
        }
      }
    }
    if (lane < nt) {
      const double den = __dsqrt_rn(__dmul_rn(na2, nc2));
      cosv[wave][t0 + lane] = den > 0.0 ? __ddiv_rn(dot, den) : 0.0;
    }
  }
  wave_lds_sync();

  int base_pos = 0;  // retained tokens with a smaller id, over the passes so far
  for (int t0 = 0; t0 < g.Bk; t0 += 64) {
    const int t = t0 + lane;
    bool keep = false;
    if (t < g.Bk) {
      const int w = wid[t], cen = wcen[t];
      if (t == cen) {
        keep = true;
      } else {
        const double ct = cosv[wave][t];
        int rank = 0;  // tokens of the window (center excluded) ordered before t: smaller cosine, then smaller id
        for (int u = 0; u < g.Bk; ++u) {
          const double cu = cosv[wave][u];
          rank += (wid[u] == w && u != cen && u != t) && ((cu < ct) || (cu == ct && u < t));
        }
        keep = rank < kw - 1;
      }
    }
    const unsigned long long m = __ballot(keep);
    if (keep) keep_idx[row * n_keep + base_pos + __popcll(m & ((1ull << lane) - 1ull))] = t;
    base_pos += __popcll(m);
  }
}

int launch_pool(const Geom& g, int dtype, const void* X, double* Xbar, hipStream_t st) {
  const uint8_t* x = static_cast<const uint8_t*>(X);
  const dim3 grid((g.rows + kWaves - 1) / kWaves), block(64 * kWaves);
  if (dtype == BSA_F32)
    hipLaunchKernelGGL(pool_kernel<4>, grid, block, 0, st, g, x, Xbar);
  else
    hipLaunchKernelGGL(pool_kernel<2>, grid, block, 0, st, g, x, Xbar);
  return check_launch();
}

int launch_prune(const Geom& g, int dtype, const void* Q, int window_quota, int32_t* keep_idx, hipStream_t st) {
  const uint8_t* q = static_cast<const uint8_t*>(Q);
  const dim3 grid((g.rows + kWaves - 1) / kWaves), block(64 * kWaves);
  if (dtype == BSA_F32)
    hipLaunchKernelGGL(prune_kernel<4>, grid, block, 0, st, g, q, window_quota, keep_idx);
  else
    hipLaunchKernelGGL(prune_kernel<2>, grid, block, 0, st, g, q, window_quota, keep_idx);
  return check_launch();
}

}  // namespace bsa
