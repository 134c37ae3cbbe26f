// Streaming kernels of the index-preparation stage: block mean pooling (Sec. 3.2.3) and
// query pruning by cosine similarity to the block center (Sec. 3.2.2, Eq. 2).
//
// Both are one pass over a [B,H,L,d] tensor and are bound by HBM bandwidth: a workgroup
// owns one 3D block, pulls its Bk token rows (Cw-token runs of contiguous memory) into LDS
// with 16-byte loads and does the fp64 decision arithmetic from LDS.
//
// Bit-exactness contract with any other implementation of the same definition: sums run
// in ascending index order (tokens for pooling, channels for dot products) in fp64.  The
// inputs are fp32 or bf16, so every product of two inputs is exact in fp64 and a fused
// multiply-add rounds exactly like multiply-then-add; cos = dot / sqrt(|a|^2 * |c|^2) uses
// IEEE fp64 multiply, sqrt and divide.
#include "bsa_common.h"

namespace bsa {

constexpr int kThreads = 256;
constexpr int kChunkBytes = 32 * 1024;  // token rows staged in LDS per pass

// Stage rows [c0, c0+nc) of block i of head bh into LDS, row stride `ldw` 32-bit words.
template <int ES>
__device__ inline void stage_rows(const Geom& g, const uint8_t* X, int64_t bh, int i, int c0, int nc,
                                  uint32_t* tile, int ldw) {
  const int vec_per_row = g.d * ES / 16;
  const int64_t row_bytes = (int64_t)g.d * ES;
  const int origin = block_origin(g, i);
  for (int v = threadIdx.x; v < nc * vec_per_row; v += kThreads) {
    const int r = v / vec_per_row, q = v % vec_per_row;
    const int64_t tok = origin + intra_offset(g, c0 + r);
    const uint4 val = *reinterpret_cast<const uint4*>(X + (bh * g.L + tok) * row_bytes + 16 * q);
    uint32_t* dst = tile + r * ldw + 4 * q;
    dst[0] = val.x; dst[1] = val.y; dst[2] = val.z; dst[3] = val.w;
  }
}

template <int ES>
__device__ inline double elem(const uint32_t* row, int c) {
  if (ES == 4) return (double)__uint_as_float(row[c]);
  const uint32_t w = row[c >> 1];
  return (double)__uint_as_float((c & 1) ? (w & 0xffff0000u) : (w << 16));
}

template <int ES>
__global__ __launch_bounds__(kThreads) void pool_kernel(Geom g, const uint8_t* X, double* Xbar) {
  __shared__ uint32_t tile[kChunkBytes / 4 + 256];
  const int row = blockIdx.x;  // (b*H + h)*N + i
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const int ldw = g.d * ES / 4 + 1;
  const int chunk = min(g.Bk, kChunkBytes / (g.d * ES));
  double acc = 0.0;
  for (int c0 = 0; c0 < g.Bk; c0 += chunk) {
    const int nc = min(chunk, g.Bk - c0);
    __syncthreads();
    stage_rows<ES>(g, X, bh, i, c0, nc, tile, ldw);
    __syncthreads();
    if (threadIdx.x < g.d)
      for (int r = 0; r < nc; ++r) acc = __dadd_rn(acc, elem<ES>(tile + r * ldw, threadIdx.x));
  }
  if (threadIdx.x < g.d) Xbar[(int64_t)row * g.d + threadIdx.x] = __ddiv_rn(acc, (double)g.Bk);
}

template <int ES>
__global__ __launch_bounds__(kThreads) void prune_kernel(Geom g, const uint8_t* Q, int n_keep,
                                                        int32_t* keep_idx) {
  __shared__ uint32_t tile[kChunkBytes / 4 + 256];
  __shared__ uint32_t center_row[256];
  __shared__ double cosv[256];
  __shared__ int kept[256];
  const int row = blockIdx.x;
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const int ldw = g.d * ES / 4 + 1;
  const int chunk = min(g.Bk, kChunkBytes / (g.d * ES));

  stage_rows<ES>(g, Q, bh, i, g.center, 1, center_row, ldw);
  __syncthreads();
  double nc2 = 0.0;  // |q_c|^2, same channel order in every thread
  for (int c = 0; c < g.d; ++c) {
    const double x = elem<ES>(center_row, c);
    nc2 = fma(x, x, nc2);
  }
  for (int c0 = 0; c0 < g.Bk; c0 += chunk) {
    const int nc = min(chunk, g.Bk - c0);
    __syncthreads();
    stage_rows<ES>(g, Q, bh, i, c0, nc, tile, ldw);
    __syncthreads();
    if (threadIdx.x < nc) {
      const uint32_t* r = tile + threadIdx.x * ldw;
      double dot = 0.0, na2 = 0.0;
      for (int c = 0; c < g.d; ++c) {
        const double x = elem<ES>(r, c);
        dot = fma(x, elem<ES>(center_row, c), dot);
        na2 = fma(x, x, na2);
      }
      const double den = __dsqrt_rn(__dmul_rn(na2, nc2));
      cosv[c0 + threadIdx.x] = den > 0.0 ? __ddiv_rn(dot, den) : 0.0;
    }
  }
  __syncthreads();
  const int t = threadIdx.x;
  int keep = 0;
  if (t < g.Bk) {
    if (t == g.center) {
      keep = 1;
    } else {
      const double ct = cosv[t];
      int rank = 0;  // tokens (center excluded) ordered before t: smaller cosine, then smaller id
      for (int u = 0; u < g.Bk; ++u) {
        if (u == g.center || u == t) continue;
        const double cu = cosv[u];
        rank += (cu < ct) || (cu == ct && u < t);
      }
      keep = rank < n_keep - 1;
    }
  }
  kept[t] = keep;
  __syncthreads();
  if (keep) {
    int pos = 0;
    for (int u = 0; u < t; ++u) pos += kept[u];
    keep_idx[(int64_t)row * n_keep + pos] = t;
  }
}

int launch_pool(const Geom& g, int dtype, const void* X, double* Xbar, hipStream_t st) {
  const uint8_t* x = static_cast<const uint8_t*>(X);
  if (dtype == BSA_F32)
    hipLaunchKernelGGL(pool_kernel<4>, dim3(g.rows), dim3(kThreads), 0, st, g, x, Xbar);
  else
    hipLaunchKernelGGL(pool_kernel<2>, dim3(g.rows), dim3(kThreads), 0, st, g, x, Xbar);
  return check_launch();
}

int launch_prune(const Geom& g, int dtype, const void* Q, int n_keep, int32_t* keep_idx, hipStream_t st) {
  const uint8_t* q = static_cast<const uint8_t*>(Q);
  if (dtype == BSA_F32)
    hipLaunchKernelGGL(prune_kernel<4>, dim3(g.rows), dim3(kThreads), 0, st, g, q, n_keep, keep_idx);
  else
    hipLaunchKernelGGL(prune_kernel<2>, dim3(g.rows), dim3(kThreads), 0, st, g, q, n_keep, keep_idx);
  return check_launch();
}

}  // namespace bsa
