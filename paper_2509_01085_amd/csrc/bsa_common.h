// Internal definitions shared by the HIP translation units of libbsa (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bsa.h"

namespace bsa {

// Geometry of one call, derived on the host from bsa_shape_t and passed to kernels by value.
struct Geom {
  int B, H, T, Hs, Ws, Ct, Ch, Cw, d;
  int Nt, Nh, Nw;  // blocks per axis
  int Bk;          // tokens per block
  int N;           // blocks per head
  int L;           // tokens per head
  int rows;        // B*H*N
  int Wt, Wh, Ww;  // window of the critical-token mechanism (Sec. 3.2.2); the whole block when one center per block
  int nwin, Wk;    // windows per block, tokens per window
  int tiled;       // 1: the Bk tokens of block i are the consecutive rows i*Bk .. i*Bk+Bk-1 (block-major layout)
  int dense;       // 1: dense baseline: every pair listed, nothing pruned (implies tiled)
  uint32_t inv_Nw, inv_NwNh;  // floor(2^32 / x) + 1 (0 when x == 1): n / x == umulhi(n, inv) for n < 2^16
};

// Raster index (Sec. 3.1) of intra-block token c of block i (Sec. 3.2.1).
__host__ __device__ inline int token_of(const Geom& g, int i, int c) {
  if (g.tiled) return i * g.Bk + c;
  const int bw = i % g.Nw, bh = (i / g.Nw) % g.Nh, bt = i / (g.Nw * g.Nh);
  const int cw = c % g.Cw, ch = (c / g.Cw) % g.Ch, ct = c / (g.Cw * g.Ch);
  return ((bt * g.Ct + ct) * g.Hs + (bh * g.Ch + ch)) * g.Ws + (bw * g.Cw + cw);
}

// Raster index of the first token (intra-block id 0) of block i.
__host__ __device__ inline int block_origin(const Geom& g, int i) {
  if (g.tiled) return i * g.Bk;
  const int bw = i % g.Nw, bh = (i / g.Nw) % g.Nh, bt = i / (g.Nw * g.Nh);
  return ((bt * g.Ct) * g.Hs + bh * g.Ch) * g.Ws + bw * g.Cw;
}

// Same, division-free (block ids are < 2^16): for per-tile use inside pipelined loops.
__device__ inline int block_origin_fast(const Geom& g, int i) {
  if (g.tiled) return i * g.Bk;
  const int bt = g.inv_NwNh ? (int)__umulhi((uint32_t)i, g.inv_NwNh) : i;
  const int rem = i - bt * g.Nw * g.Nh;
  const int bh = g.inv_Nw ? (int)__umulhi((uint32_t)rem, g.inv_Nw) : rem;
  const int bw = rem - bh * g.Nw;
  return ((bt * g.Ct) * g.Hs + bh * g.Ch) * g.Ws + bw * g.Cw;
}

// Offset of intra-block token c from the block origin, in tokens.
__host__ __device__ inline int intra_offset(const Geom& g, int c) {
  if (g.tiled) return c;
  const int cw = c % g.Cw, ch = (c / g.Cw) % g.Ch, ct = c / (g.Cw * g.Ch);
  return (ct * g.Hs + ch) * g.Ws + cw;
}

// Window (numbered raster-wise over the block's window grid) of intra-block token c.
__host__ __device__ inline int window_of(const Geom& g, int c) {
  if (g.nwin == 1) return 0;
  const int cw = c % g.Cw, ch = (c / g.Cw) % g.Ch, ct = c / (g.Cw * g.Ch);
  return ((ct / g.Wt) * (g.Ch / g.Wh) + ch / g.Wh) * (g.Cw / g.Ww) + cw / g.Ww;
}

// Intra-block id of the critical token of window w: local coordinate (Wt/2, Wh/2, Ww/2).
__host__ __device__ inline int window_center(const Geom& g, int w) {
  const int nw = g.Cw / g.Ww, nh = g.Ch / g.Wh;
  const int c = w % nw, b = (w / nw) % nh, a = w / (nw * nh);
  return ((a * g.Wt + g.Wt / 2) * g.Ch + b * g.Wh + g.Wh / 2) * g.Cw + c * g.Ww + g.Ww / 2;
}

// Critical token of the window that holds intra-block token c.
__host__ __device__ inline int center_of(const Geom& g, int c) { return window_center(g, window_of(g, c)); }

int make_geom(const bsa_shape_t* s, Geom* g);  // validates; returns bsa_status

inline int check_launch() {
  return hipGetLastError() == hipSuccess ? BSA_OK : BSA_ERR_LAUNCH;
}

// Lets `Kernel` be launched with `bytes` of dynamic LDS.  The attribute call is made only when a
// launch needs more than any earlier one of the same kernel on the same device did, i.e. once per
// kernel in steady state; callers run it before they launch anything, so a failure leaves the
// stream untouched.
template <auto Kernel>
inline int allow_dynamic_lds(size_t bytes) {
  constexpr int kMaxDev = 64;
  static size_t granted[kMaxDev] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return BSA_ERR_LAUNCH;
  if (bytes <= granted[dev]) return BSA_OK;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)bytes) != hipSuccess)
    return BSA_ERR_LAUNCH;
  granted[dev] = bytes;
  return BSA_OK;
}

// bf16 <-> fp32 (round to nearest even), bit-level.
__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ inline uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> __device__ inline float load_f32(const T* p);
template <> __device__ inline float load_f32<float>(const float* p) { return *p; }
template <> __device__ inline float load_f32<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void store_f32(T* p, float v);
template <> __device__ inline void store_f32<float>(float* p, float v) { *p = v; }
template <> __device__ inline void store_f32<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

// ---- entry points implemented per translation unit (all enqueue on `st`) ----
int launch_pool(const Geom& g, int dtype, const void* X, double* Xbar, hipStream_t st);
int launch_prune(const Geom& g, int dtype, const void* Q, int window_quota, int32_t* keep_idx, hipStream_t st);
size_t select_workspace_bytes(const Geom& g);
int static_select_scratch(void** ptr, size_t* bytes);  // this device's copy of the library-owned selection scratch
int launch_select(const Geom& g, const double* Qbar, const double* Kbar, double threshold,
                  double stat_z /* Eq. 3 quantile; NaN or -inf: no candidate filter */, double score_scale, int32_t* q2k_ptr, int32_t* q2k_idx, int32_t* k2q_ptr,
                  int32_t* k2q_idx, int64_t* nnz_dev, void* ws, hipStream_t st);

struct AttnArgs {
  const void *Q, *K, *V, *O, *dO;
  const float* LSE_in;
  const int32_t *q2k_ptr, *q2k_idx, *k2q_ptr, *k2q_idx, *keep_idx;
  int n_keep;
  float sm_scale;
  void *O_out, *dQ, *dK, *dV;
  float* LSE_out;
  void* ws;
  unsigned stages;  // backward only: which of its kernels to launch (bsa_bwd_stage bits)
  // tail splitting (MFMA path): on every XCD the last split_n units of a launch are walked in
  // split_S segments by separate workgroups, which leave fp32 partial results in `part` for a
  // combine launch; split_n == 0 turns it off.  fwd_ws: the forward's own workspace.
  int split_S, split_n;
  float* part;
  void* fwd_ws;
  int kv_split_S, kv_split_n;  // the same for the dK/dV launch
  float* kv_part;
  int pack;  // backward records hold two query blocks of at most 16 retained queries each
};

// plain-ALU fp32-accumulate kernels: any supported shape, fp32 or bf16 storage
int launch_fwd_generic(const Geom& g, int dtype, const AttnArgs& a, hipStream_t st);
int launch_bwd_generic(const Geom& g, int dtype, const AttnArgs& a, hipStream_t st);
size_t bwd_workspace_generic(const Geom& g, int n_keep);

// bf16 MFMA kernels: Bk == 64, d == 128 (or 64), n_keep <= 64
bool mfma_supported(const Geom& g, int dtype, int n_keep);  // shapes the bf16 MFMA kernels cover
int launch_fwd_pipe(const Geom& g, const AttnArgs& a, hipStream_t st);
int launch_bwd_pipe(const Geom& g, const AttnArgs& a, hipStream_t st);
size_t bwd_workspace_pipe(const Geom& g, int n_keep);
size_t fwd_workspace_pipe(const Geom& g, int n_keep);

}  // namespace bsa
