// Shape-generic sparse attention forward / backward on the vector ALUs (Eq. 5 with token
// filling, and its backward with the index sets held constant).  fp32 arithmetic throughout,
// storage fp32 or bf16.  This is the path for shapes the MFMA kernels do not cover and for
// true-fp32 inputs; it is written for clarity and any supported (Bk, d, n_keep), not speed.
//
// Work split: 16 queries x 16 keys per workgroup step.  Thread (qi, kt) of 256 owns one
// logit; the 16 lanes sharing qi reduce the row maximum / sum with shuffles (online
// softmax); the same 16 lanes then own channels c = lane, lane+16, ... of that query's
// accumulator.  dK/dV of a KV block are owned by workgroups of that block, which walk the
// block's k2q list: no atomics, fixed summation order.
#include <math.h>

#include "bsa_common.h"

namespace bsa {

constexpr int QT = 16, KT = 16, MAXC = 16;  // MAXC = 256 / 16 channels per lane

struct GenericWs {
  float* g;      // [rows][n_keep][d]  upstream gradient with the fill copies folded in
  float* delta;  // [rows][n_keep]     <g, o>
  size_t bytes;
};
static GenericWs carve(const Geom& g, int n_keep, void* base) {
  GenericWs w;
  uint8_t* p = static_cast<uint8_t*>(base);
  size_t off = 0;
  w.g = reinterpret_cast<float*>(p + off);
  off += (((size_t)g.rows * n_keep * g.d * 4) + 255) & ~(size_t)255;
  w.delta = reinterpret_cast<float*>(p + off);
  off += (((size_t)g.rows * n_keep * 4) + 255) & ~(size_t)255;
  w.bytes = off;
  return w;
}
size_t bwd_workspace_generic(const Geom& g, int n_keep) { return carve(g, n_keep, nullptr).bytes; }

__device__ inline float group16_max(float v) {
  for (int o = 1; o < 16; o <<= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float group16_sum(float v) {
  for (int o = 1; o < 16; o <<= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename T>
__device__ inline void load_rows(float* dst, int ld, const T* head, const int* tok, int n_rows, int n_valid, int d) {
  for (int e = threadIdx.x; e < n_rows * d; e += 256) {
    const int r = e / d, c = e % d;
    dst[r * ld + c] = r < n_valid ? load_f32<T>(head + (int64_t)tok[r] * d + c) : 0.f;
  }
}

__device__ inline int kept_id(const Geom& g, const int32_t* keep_idx, int64_t row, int n_keep, int pos) {
  // clamped: a malformed keep list must not turn into an out-of-bounds access
  return g.dense ? pos : min(max(keep_idx[row * n_keep + pos], 0), g.Bk - 1);
}
__device__ inline int listed_block(const Geom& g, const int32_t* idx, int beg, int t) {
  return g.dense ? t : min(max(idx[beg + t], 0), g.N - 1);
}

// ---------------------------------------------------------------------------- forward
template <typename T>
__global__ __launch_bounds__(256) void fwd_generic_kernel(Geom g, AttnArgs a) {
  extern __shared__ float sm[];
  const int ld = g.d + 1;
  float* qs = sm;                 // [QT][ld]
  float* ks = qs + QT * ld;       // [KT][ld]
  float* vs = ks + KT * ld;       // [KT][ld]
  float* ps = vs + KT * ld;       // [QT][KT+1]
  __shared__ int qtok[QT], ktok[KT];
  __shared__ int keeppos[256];  // position of an intra-block token among the retained rows, -1 if pruned
  __shared__ float lse_s[QT];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const int q0 = blockIdx.y * QT;
  const int nq = min(QT, a.n_keep - q0);
  const T* Qh = static_cast<const T*>(a.Q) + bh * g.L * g.d;
  const T* Kh = static_cast<const T*>(a.K) + bh * g.L * g.d;
  const T* Vh = static_cast<const T*>(a.V) + bh * g.L * g.d;
  T* Oh = static_cast<T*>(a.O_out) + bh * g.L * g.d;
  float* Lh = a.LSE_out + bh * g.L;

  keeppos[tid] = -1;
  __syncthreads();
  if (tid < a.n_keep) keeppos[kept_id(g, a.keep_idx, row, a.n_keep, tid)] = tid;
  if (tid < QT) qtok[tid] = tid < nq ? token_of(g, i, kept_id(g, a.keep_idx, row, a.n_keep, q0 + tid)) : 0;
  __syncthreads();
  load_rows<T>(qs, ld, Qh, qtok, QT, nq, g.d);

  const int beg = g.dense ? 0 : a.q2k_ptr[row];
  const int cnt = g.dense ? g.N : a.q2k_ptr[row + 1] - beg;
  const int qi = tid / 16, kt = tid % 16;
  float m = -INFINITY, l = 0.f, o[MAXC];
#pragma unroll
  for (int cc = 0; cc < MAXC; ++cc) o[cc] = 0.f;

  for (int t = 0; t < cnt; ++t) {
    const int jb = listed_block(g, a.q2k_idx, beg, t);
    for (int k0 = 0; k0 < g.Bk; k0 += KT) {
      const int nk = min(KT, g.Bk - k0);
      __syncthreads();
      if (tid < KT) ktok[tid] = tid < nk ? token_of(g, jb, k0 + tid) : 0;
      __syncthreads();
      load_rows<T>(ks, ld, Kh, ktok, KT, nk, g.d);
      load_rows<T>(vs, ld, Vh, ktok, KT, nk, g.d);
      __syncthreads();
      float s = 0.f;
      for (int c = 0; c < g.d; ++c) s += qs[qi * ld + c] * ks[kt * ld + c];
      s = kt < nk ? s * a.sm_scale : -INFINITY;
      const float mnew = fmaxf(m, group16_max(s));
      const float p = expf(s - mnew);  // exp(-inf) = 0 for the padding keys
      const float alpha = expf(m - mnew);
      l = l * alpha + group16_sum(p);
      m = mnew;
      ps[qi * (KT + 1) + kt] = p;
      __syncthreads();
#pragma unroll
      for (int cc = 0; cc < MAXC; ++cc) {
        const int c = kt + 16 * cc;
        if (c < g.d) {
          float acc = o[cc] * alpha;
          for (int k = 0; k < KT; ++k) acc += ps[qi * (KT + 1) + k] * vs[k * ld + c];
          o[cc] = acc;
        }
      }
    }
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;
  const float lse = l > 0.f ? m + logf(l) : -INFINITY;
  __syncthreads();
  if (qi < nq) {
#pragma unroll
    for (int cc = 0; cc < MAXC; ++cc) {
      const int c = kt + 16 * cc;
      if (c < g.d) {
        const float val = o[cc] * inv;
        store_f32<T>(Oh + (int64_t)qtok[qi] * g.d + c, val);
        qs[qi * ld + c] = val;  // output rows parked in LDS (over the query rows) for the fill
      }
    }
    if (kt == 0) {
      Lh[qtok[qi]] = lse;
      lse_s[qi] = lse;
    }
  }
  __syncthreads();
  // token filling: a pruned token takes the row of its window's critical token; the workgroup
  // whose query tile holds that row writes it
  if (!g.dense) {
    for (int e = tid; e < g.Bk * g.d; e += 256) {
      const int c = e / g.d, ch = e % g.d;
      if (keeppos[c] >= 0) continue;
      const int p = keeppos[center_of(g, c)] - q0;
      if (p >= 0 && p < nq && keeppos[center_of(g, c)] >= 0)
        store_f32<T>(Oh + (int64_t)token_of(g, i, c) * g.d + ch, qs[p * ld + ch]);
    }
    if (tid < g.Bk && keeppos[tid] < 0) {
      const int p = keeppos[center_of(g, tid)] - q0;
      if (p >= 0 && p < nq && keeppos[center_of(g, tid)] >= 0) Lh[token_of(g, i, tid)] = lse_s[p];
    }
  }
}

// ------------------------------------------------------------- backward: preprocess
// g = dO of the retained row (+ for a window's critical token the dO of every pruned token of
// that window, ascending id);
// delta = <g, o>.  One wavefront per retained row, lanes over channels.
template <typename T>
__global__ __launch_bounds__(256) void bwd_pre_generic_kernel(Geom g, AttnArgs a, GenericWs w) {
  __shared__ int keepflag[256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x;
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const T* dOh = static_cast<const T*>(a.dO) + bh * g.L * g.d;
  const T* Oh = static_cast<const T*>(a.O) + bh * g.L * g.d;
  keepflag[tid] = 0;
  __syncthreads();
  if (tid < a.n_keep) keepflag[kept_id(g, a.keep_idx, row, a.n_keep, tid)] = 1;
  __syncthreads();
  for (int kp = wave; kp < a.n_keep; kp += 4) {
    const int c = kept_id(g, a.keep_idx, row, a.n_keep, kp);
    const int64_t tok = token_of(g, i, c);
    float part = 0.f;
    for (int ch = lane; ch < g.d; ch += 64) {
      float gv = load_f32<T>(dOh + tok * g.d + ch);
      if (!g.dense && c == center_of(g, c))  // a critical token: plus the dO of its window's pruned tokens
        for (int u = 0; u < g.Bk; ++u)
          if (!keepflag[u] && window_of(g, u) == window_of(g, c)) gv += load_f32<T>(dOh + (int64_t)token_of(g, i, u) * g.d + ch);
      w.g[(row * a.n_keep + kp) * g.d + ch] = gv;
      part += gv * load_f32<T>(Oh + tok * g.d + ch);
    }
    for (int o = 1; o < 64; o <<= 1) part += __shfl_xor(part, o);
    if (lane == 0) w.delta[row * a.n_keep + kp] = part;
  }
}

// ------------------------------------------------------------------- backward: dQ
template <typename T>
__global__ __launch_bounds__(256) void bwd_dq_generic_kernel(Geom g, AttnArgs a, GenericWs w) {
  extern __shared__ float sm[];
  const int ld = g.d + 1;
  float* qs = sm;                 // [QT][ld]
  float* gs = qs + QT * ld;       // [QT][ld]
  float* ks = gs + QT * ld;       // [KT][ld]
  float* vs = ks + KT * ld;       // [KT][ld]
  float* ds = vs + KT * ld;       // [QT][KT+1]
  __shared__ int qtok[QT], ktok[KT];
  __shared__ int keepflag[256];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const int q0 = blockIdx.y * QT;
  const int nq = min(QT, a.n_keep - q0);
  const T* Qh = static_cast<const T*>(a.Q) + bh * g.L * g.d;
  const T* Kh = static_cast<const T*>(a.K) + bh * g.L * g.d;
  const T* Vh = static_cast<const T*>(a.V) + bh * g.L * g.d;
  T* dQh = static_cast<T*>(a.dQ) + bh * g.L * g.d;
  const float* Lh = a.LSE_in + bh * g.L;

  keepflag[tid] = 0;
  __syncthreads();
  if (tid < a.n_keep) keepflag[kept_id(g, a.keep_idx, row, a.n_keep, tid)] = 1;
  if (tid < QT) qtok[tid] = tid < nq ? token_of(g, i, kept_id(g, a.keep_idx, row, a.n_keep, q0 + tid)) : 0;
  __syncthreads();
  load_rows<T>(qs, ld, Qh, qtok, QT, nq, g.d);
  for (int e = tid; e < QT * g.d; e += 256) {
    const int r = e / g.d, c = e % g.d;
    gs[r * ld + c] = r < nq ? w.g[(row * a.n_keep + q0 + r) * g.d + c] : 0.f;
  }
  const int qi = tid / 16, kt = tid % 16;
  const bool qvalid = qi < nq;
  const float lse = qvalid ? Lh[qtok[qi]] : 0.f;
  const float delta = qvalid ? w.delta[row * a.n_keep + q0 + qi] : 0.f;
  const int beg = g.dense ? 0 : a.q2k_ptr[row];
  const int cnt = g.dense ? g.N : a.q2k_ptr[row + 1] - beg;
  float dq[MAXC];
#pragma unroll
  for (int cc = 0; cc < MAXC; ++cc) dq[cc] = 0.f;

  for (int t = 0; t < cnt; ++t) {
    const int jb = listed_block(g, a.q2k_idx, beg, t);
    for (int k0 = 0; k0 < g.Bk; k0 += KT) {
      const int nk = min(KT, g.Bk - k0);
      __syncthreads();
      if (tid < KT) ktok[tid] = tid < nk ? token_of(g, jb, k0 + tid) : 0;
      __syncthreads();
      load_rows<T>(ks, ld, Kh, ktok, KT, nk, g.d);
      load_rows<T>(vs, ld, Vh, ktok, KT, nk, g.d);
      __syncthreads();
      float s = 0.f, dp = 0.f;
      for (int c = 0; c < g.d; ++c) {
        s += qs[qi * ld + c] * ks[kt * ld + c];
        dp += gs[qi * ld + c] * vs[kt * ld + c];
      }
      const float p = (qvalid && kt < nk) ? expf(s * a.sm_scale - lse) : 0.f;
      ds[qi * (KT + 1) + kt] = p * (dp - delta);
      __syncthreads();
#pragma unroll
      for (int cc = 0; cc < MAXC; ++cc) {
        const int c = kt + 16 * cc;
        if (c < g.d) {
          float acc = dq[cc];
          for (int k = 0; k < KT; ++k) acc += ds[qi * (KT + 1) + k] * ks[k * ld + c];
          dq[cc] = acc;
        }
      }
    }
  }
  if (qvalid) {
#pragma unroll
    for (int cc = 0; cc < MAXC; ++cc) {
      const int c = kt + 16 * cc;
      if (c < g.d) store_f32<T>(dQh + (int64_t)qtok[qi] * g.d + c, dq[cc] * a.sm_scale);
    }
  }
  if (blockIdx.y == 0) {  // pruned queries take no part in the forward: zero gradient
    for (int e = tid; e < g.Bk * g.d; e += 256) {
      const int c = e / g.d, ch = e % g.d;
      if (!keepflag[c]) store_f32<T>(dQh + (int64_t)token_of(g, i, c) * g.d + ch, 0.f);
    }
  }
}

// --------------------------------------------------------------- backward: dK, dV
template <typename T>
__global__ __launch_bounds__(256) void bwd_dkv_generic_kernel(Geom g, AttnArgs a, GenericWs w) {
  extern __shared__ float sm[];
  const int ld = g.d + 1;
  float* qs = sm;                 // [QT][ld]
  float* gs = qs + QT * ld;       // [QT][ld]
  float* ks = gs + QT * ld;       // [KT][ld]
  float* vs = ks + KT * ld;       // [KT][ld]
  float* ps = vs + KT * ld;       // [QT][KT+1]
  float* ds = ps + QT * (KT + 1); // [QT][KT+1]
  __shared__ int qtok[QT], ktok[KT];
  __shared__ float lse_s[QT], delta_s[QT];
  const int tid = threadIdx.x;
  const int64_t col = blockIdx.x;  // (b*H + h)*N + j
  const int64_t bh = col / g.N;
  const int j = col % g.N;
  const int k0 = blockIdx.y * KT;
  const int nk = min(KT, g.Bk - k0);
  const T* Qh = static_cast<const T*>(a.Q) + bh * g.L * g.d;
  const T* Kh = static_cast<const T*>(a.K) + bh * g.L * g.d;
  const T* Vh = static_cast<const T*>(a.V) + bh * g.L * g.d;
  T* dKh = static_cast<T*>(a.dK) + bh * g.L * g.d;
  T* dVh = static_cast<T*>(a.dV) + bh * g.L * g.d;
  const float* Lh = a.LSE_in + bh * g.L;

  if (tid < KT) ktok[tid] = tid < nk ? token_of(g, j, k0 + tid) : 0;
  __syncthreads();
  load_rows<T>(ks, ld, Kh, ktok, KT, nk, g.d);
  load_rows<T>(vs, ld, Vh, ktok, KT, nk, g.d);
  const int beg = g.dense ? 0 : a.k2q_ptr[col];
  const int cnt = g.dense ? g.N : a.k2q_ptr[col + 1] - beg;
  const int qi = tid / 16, kt = tid % 16;  // logit phase: (query, key); sum phase: (key = qi, lane = kt)
  float dk[MAXC], dv[MAXC];
#pragma unroll
  for (int cc = 0; cc < MAXC; ++cc) dk[cc] = dv[cc] = 0.f;

  for (int t = 0; t < cnt; ++t) {
    const int ib = listed_block(g, a.k2q_idx, beg, t);
    const int64_t qrow = bh * g.N + ib;
    for (int q0 = 0; q0 < a.n_keep; q0 += QT) {
      const int nq = min(QT, a.n_keep - q0);
      __syncthreads();
      if (tid < QT) {
        const int tk = tid < nq ? token_of(g, ib, kept_id(g, a.keep_idx, qrow, a.n_keep, q0 + tid)) : 0;
        qtok[tid] = tk;
        lse_s[tid] = tid < nq ? Lh[tk] : 0.f;
        delta_s[tid] = tid < nq ? w.delta[qrow * a.n_keep + q0 + tid] : 0.f;
      }
      __syncthreads();
      load_rows<T>(qs, ld, Qh, qtok, QT, nq, g.d);
      for (int e = tid; e < QT * g.d; e += 256) {
        const int r = e / g.d, c = e % g.d;
        gs[r * ld + c] = r < nq ? w.g[(qrow * a.n_keep + q0 + r) * g.d + c] : 0.f;
      }
      __syncthreads();
      float s = 0.f, dp = 0.f;
      for (int c = 0; c < g.d; ++c) {
        s += qs[qi * ld + c] * ks[kt * ld + c];
        dp += gs[qi * ld + c] * vs[kt * ld + c];
      }
      const float p = (qi < nq && kt < nk) ? expf(s * a.sm_scale - lse_s[qi]) : 0.f;
      ps[qi * (KT + 1) + kt] = p;
      ds[qi * (KT + 1) + kt] = p * (dp - delta_s[qi]);
      __syncthreads();
      const int key = qi;
#pragma unroll
      for (int cc = 0; cc < MAXC; ++cc) {
        const int c = kt + 16 * cc;
        if (c < g.d) {
          float av = dv[cc], ak = dk[cc];
          for (int r = 0; r < QT; ++r) {
            av += ps[r * (KT + 1) + key] * gs[r * ld + c];
            ak += ds[r * (KT + 1) + key] * qs[r * ld + c];
          }
          dv[cc] = av;
          dk[cc] = ak;
        }
      }
    }
  }
  const int key = qi;
  if (key < nk) {
#pragma unroll
    for (int cc = 0; cc < MAXC; ++cc) {
      const int c = kt + 16 * cc;
      if (c < g.d) {
        store_f32<T>(dKh + (int64_t)ktok[key] * g.d + c, dk[cc] * a.sm_scale);
        store_f32<T>(dVh + (int64_t)ktok[key] * g.d + c, dv[cc]);
      }
    }
  }
}

template <typename T>
static int fwd_t(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const size_t lds = (size_t)((QT + 2 * KT) * (g.d + 1) + QT * (KT + 1)) * 4;
  if (int rc = allow_dynamic_lds<fwd_generic_kernel<T>>(lds)) return rc;
  hipLaunchKernelGGL(fwd_generic_kernel<T>, dim3(g.rows, (a.n_keep + QT - 1) / QT), dim3(256), lds, st, g, a);
  return check_launch();
}

template <typename T>
static int bwd_t(const Geom& g, const AttnArgs& a, hipStream_t st) {
  GenericWs w = carve(g, a.n_keep, a.ws);
  const size_t lds = (size_t)((2 * QT + 2 * KT) * (g.d + 1) + 2 * QT * (KT + 1)) * 4;
  if (int rc = allow_dynamic_lds<bwd_dq_generic_kernel<T>>(lds)) return rc;
  if (int rc = allow_dynamic_lds<bwd_dkv_generic_kernel<T>>(lds)) return rc;
  if (a.stages & BSA_BWD_PRE) hipLaunchKernelGGL(bwd_pre_generic_kernel<T>, dim3(g.rows), dim3(256), 0, st, g, a, w);
  if (a.stages & BSA_BWD_DQ) hipLaunchKernelGGL(bwd_dq_generic_kernel<T>, dim3(g.rows, (a.n_keep + QT - 1) / QT), dim3(256), lds, st, g, a, w);
  if (a.stages & BSA_BWD_DKV) hipLaunchKernelGGL(bwd_dkv_generic_kernel<T>, dim3(g.rows, (g.Bk + KT - 1) / KT), dim3(256), lds, st, g, a, w);
  return check_launch();
}

int launch_fwd_generic(const Geom& g, int dtype, const AttnArgs& a, hipStream_t st) {
  return dtype == BSA_F32 ? fwd_t<float>(g, a, st) : fwd_t<uint16_t>(g, a, st);
}
int launch_bwd_generic(const Geom& g, int dtype, const AttnArgs& a, hipStream_t st) {
  return dtype == BSA_F32 ? bwd_t<float>(g, a, st) : bwd_t<uint16_t>(g, a, st);
}

}  // namespace bsa
