// bf16 MFMA kernels for the flagship tile shape: Bk = 64 tokens per block, d = 128 (or 64).
//
// Forward (Eq. 5 + token filling).  A workgroup of four wavefronts owns four consecutive query
// blocks of one head, one block per wavefront (its <= 64 retained queries sit on the MFMA
// column index).  The workgroup walks the UNION of the four KV lists in ascending block
// order; every K/V tile is gathered from the raster layout into LDS once and each wavefront
// uses it only if its own list contains it.  Per tile and wavefront:
//     S^T = K Q^T          (A = K rows from LDS, B = Q^T fragments held in registers)
//     online softmax       (row statistics per lane pair, exp2 domain)
//     O^T += V^T P^T       (A = V^T from LDS, stored transposed + slot-permuted at staging;
//                           B = P^T straight from the S^T accumulator registers)
// K/V tiles are double-buffered: the global loads of tile t+1 are in flight while tile t is
// being multiplied.
#include <math.h>

#include "bsa_mfma.h"

namespace bsa {

constexpr int G = 4;             // query blocks (= wavefronts) per workgroup
constexpr int BK = 64;           // tokens per block on this path
constexpr int VLD = BK + 8;      // V^T row stride in LDS, bf16 elements

bool mfma_supported(const Geom& g, int dtype, int n_keep) {
  return dtype == BSA_BF16 && g.Bk == BK && (g.d == 128 || g.d == 64) && n_keep <= BK;
}

template <int D>
struct Stage {
  static constexpr int KLD = D + 8;               // K row stride in LDS, bf16 elements
  static constexpr int KV = BK * (D / 8) / 256;   // 16-byte K loads per thread
  static constexpr int VUNITS = 16 * (D / 8);     // (4 keys x 8 channels) V units per tile
  u32x4 k[KV];
  u32x4 v[4];

  // issue the global loads of KV block jb
  __device__ inline void load(const Geom& g, const uint16_t* Kh, const uint16_t* Vh, int jb, const int* koff) {
    const int tid = threadIdx.x;
    const int64_t origin = block_origin(g, jb);
#pragma unroll
    for (int n = 0; n < KV; ++n) {
      const int u = tid + 256 * n, row = u / (D / 8), cg = u % (D / 8);
      k[n] = *reinterpret_cast<const u32x4*>(Kh + (origin + koff[row]) * D + 8 * cg);
    }
    if (tid < VUNITS) {
      const int kq = tid % 16, dc = tid / 16;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        v[r] = *reinterpret_cast<const u32x4*>(Vh + (origin + koff[4 * kq + r]) * D + 8 * dc);
    }
  }

  // write them to LDS: K row-major, V transposed with slot-permuted key positions
  __device__ inline void store(uint16_t* Ks, uint16_t* Vs) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int n = 0; n < KV; ++n) {
      const int u = tid + 256 * n, row = u / (D / 8), cg = u % (D / 8);
      *reinterpret_cast<u32x4*>(Ks + row * KLD + 8 * cg) = k[n];
    }
    if (tid < VUNITS) {
      const int kq = tid % 16, dc = tid / 16;
      u32x2 t[8];
      transpose_4x8(v, t);
      const int pos = slot_pos(4 * kq);
#pragma unroll
      for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x2*>(Vs + (8 * dc + c) * VLD + pos) = t[c];
    }
  }
};

// Ascending walk over the union of the workgroup's KV lists, kept as bit masks in LDS.
struct UnionWalk {
  const uint32_t* masks;  // [G][W]
  int W, wave, word;
  uint32_t u, own;
  __device__ inline UnionWalk(const uint32_t* m, int W_, int wave_) : masks(m), W(W_), wave(wave_), word(-1), u(0), own(0) {}
  // next KV block id or -1; `mine` tells whether this wavefront's list contains it
  __device__ inline int next(bool& mine) {
    while (u == 0) {
      if (++word >= W) return -1;
      u = masks[word] | masks[W + word] | masks[2 * W + word] | masks[3 * W + word];
      own = masks[wave * W + word];
    }
    const int b = __ffs(u) - 1;
    u &= u - 1;
    mine = (own >> b) & 1u;
    return word * 32 + b;
  }
};

template <int D, int NQT>
__global__ __launch_bounds__(256, (NQT == 1 ? 2 : 1)) void fwd_mfma_kernel(Geom g, AttnArgs a) {
  constexpr int KLD = Stage<D>::KLD;
  constexpr int DT = D / 32;   // 32-row tiles of the O^T accumulator
  constexpr int DS = D / 16;   // k-steps of the QK^T contraction
  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);              // [2][BK*KLD]
  uint16_t* Vs = Ks + 2 * BK * KLD;                              // [2][D*VLD]
  uint32_t* masks = reinterpret_cast<uint32_t*>(Vs + 2 * D * VLD);  // [G][W]
  __shared__ int koff[BK];
  __shared__ __align__(16) uint16_t cen_row[G][D];
  __shared__ float cen_lse[G];
  __shared__ uint32_t keepbits[G][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int64_t bh = blockIdx.y;
  const int i = blockIdx.x * G + wave;  // this wavefront's query block
  const bool valid = i < g.N;
  const int64_t row = bh * g.N + i;
  const int W = (g.N + 31) / 32;
  const uint16_t* Qh = static_cast<const uint16_t*>(a.Q) + bh * g.L * D;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* Oh = static_cast<uint16_t*>(a.O_out) + bh * g.L * D;
  float* Lh = a.LSE_out + bh * g.L;

  if (tid < BK) koff[tid] = intra_offset(g, tid);
  for (int k = tid; k < G * W; k += 256) masks[k] = 0u;
  if (tid < 2 * G) keepbits[tid >> 1][tid & 1] = 0u;
  __syncthreads();
  if (valid) {
    if (g.dense) {
      for (int w = lane; w < W; w += 64)
        masks[wave * W + w] = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
    } else {
      const int beg = a.q2k_ptr[row], cnt = a.q2k_ptr[row + 1] - beg;
      for (int t = lane; t < cnt; t += 64) {
        const int j = a.q2k_idx[beg + t];
        if ((unsigned)j < (unsigned)g.N) atomicOr(&masks[wave * W + (j >> 5)], 1u << (j & 31));
      }
    }
  }

  // Q^T fragments: lane (col, grp) holds channels 16*step + 8*grp .. +7 of retained query 32*qt + col
  bf16x8 qf[NQT][DS];
  int qtok[NQT];
  int qid[NQT];  // intra-block id of the lane's query, -1 if the column is padding
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int pos = 32 * qt + col;
    qid[qt] = -1;
    qtok[qt] = 0;
    if (valid && pos < a.n_keep) {
      const int c = g.dense ? pos : min(max(a.keep_idx[row * a.n_keep + pos], 0), BK - 1);
      qid[qt] = c;
      qtok[qt] = block_origin(g, i) + koff[c];
      atomicOr(&keepbits[wave][c >> 5], 1u << (c & 31));
    }
#pragma unroll
    for (int s = 0; s < DS; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (qid[qt] >= 0) v = *reinterpret_cast<const u32x4*>(Qh + (int64_t)qtok[qt] * D + 16 * s + 8 * grp);
      qf[qt][s] = as_frag(v);
    }
  }
  __syncthreads();

  f32x16 o[NQT][DT];
  float m[NQT], l[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    m[qt] = -INFINITY;
    l[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[qt][dt][r] = 0.f;
  }
  const float c2 = a.sm_scale * kLog2e;

  UnionWalk walk(masks, W, wave);
  Stage<D> st;
  bool mine = false, mine_next = false;
  int jb = walk.next(mine);
  if (jb >= 0) {
    st.load(g, Kh, Vh, jb, koff);
    st.store(Ks, Vs);
  }
  __syncthreads();
  int buf = 0;
  while (jb >= 0) {
    const int jn = walk.next(mine_next);
    if (jn >= 0) st.load(g, Kh, Vh, jn, koff);
    if (mine) {
      const uint16_t* Kb = Ks + buf * BK * KLD;
      const uint16_t* Vb = Vs + buf * D * VLD;
      f32x16 s[NQT][2];
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qt][kt][r] = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int sp = 0; sp < DS; ++sp) {
          const bf16x8 kfrag = lds_frag(Kb + (32 * kt + col) * KLD + 16 * sp + 8 * grp);
#pragma unroll
          for (int qt = 0; qt < NQT; ++qt) s[qt][kt] = mfma32(kfrag, qf[qt][sp], s[qt][kt]);
        }
      bf16x8 pf[NQT][4];
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) {
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            s[qt][kt][r] *= c2;
            mx = fmaxf(mx, s[qt][kt][r]);
          }
        mx = fmaxf(mx, xor32(mx));
        const float mnew = fmaxf(m[qt], mx);
        const float alpha = __builtin_amdgcn_exp2f(m[qt] - mnew);
        float sum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(s[qt][kt][r] - mnew);
            s[qt][kt][r] = p;
            sum += p;
          }
        l[qt] = l[qt] * alpha + sum;  // per-lane partial; the lane pair is summed at the end
        m[qt] = mnew;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[qt][dt][r] *= alpha;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) pf[qt][ks] = d_to_b(s[qt][ks >> 1], ks & 1);
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 vfrag = lds_frag(Vb + (32 * dt + col) * VLD + 16 * ks + 8 * grp);
#pragma unroll
          for (int qt = 0; qt < NQT; ++qt) o[qt][dt] = mfma32(vfrag, pf[qt][ks], o[qt][dt]);
        }
    }
    if (jn >= 0) st.store(Ks + (buf ^ 1) * BK * KLD, Vs + (buf ^ 1) * D * VLD);
    __syncthreads();
    buf ^= 1;
    jb = jn;
    mine = mine_next;
  }

  // epilogue: normalise, store retained rows, park the center row for the fill
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const float ltot = l[qt] + xor32(l[qt]);
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    const float lse = ltot > 0.f ? (m[qt] + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
    if (qid[qt] >= 0) {
      const bool is_center = !g.dense && qid[qt] == g.center;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 v;
          v.x = pack_bf16(o[qt][dt][4 * r4 + 0] * inv, o[qt][dt][4 * r4 + 1] * inv);
          v.y = pack_bf16(o[qt][dt][4 * r4 + 2] * inv, o[qt][dt][4 * r4 + 3] * inv);
          const int ch = 32 * dt + 8 * r4 + 4 * grp;
          *reinterpret_cast<u32x2*>(Oh + (int64_t)qtok[qt] * D + ch) = v;
          if (is_center) *reinterpret_cast<u32x2*>(&cen_row[wave][ch]) = v;
        }
      if (grp == 0) {
        Lh[qtok[qt]] = lse;
        if (is_center) cen_lse[wave] = lse;
      }
    }
  }
  __syncthreads();
  // token filling: lane c owns intra-block token c; pruned tokens copy the center's row
  if (valid && !g.dense) {
    const bool kept = (keepbits[wave][lane >> 5] >> (lane & 31)) & 1u;
    if (!kept) {
      const int64_t tok = block_origin(g, i) + koff[lane];
#pragma unroll
      for (int q = 0; q < D / 8; ++q)
        *reinterpret_cast<u32x4*>(Oh + tok * D + 8 * q) = *reinterpret_cast<const u32x4*>(&cen_row[wave][8 * q]);
      Lh[tok] = cen_lse[wave];
    }
  }
}

template <int D, int NQT>
static int launch_fwd_t(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const int W = (g.N + 31) / 32;
  const size_t lds = (size_t)2 * BK * Stage<D>::KLD * 2 + (size_t)2 * D * VLD * 2 + (size_t)G * W * 4;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(fwd_mfma_kernel<D, NQT>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return BSA_ERR_LAUNCH;
  hipLaunchKernelGGL((fwd_mfma_kernel<D, NQT>), dim3((g.N + G - 1) / G, g.B * g.H), dim3(256), lds, st, g, a);
  return check_launch();
}

int launch_fwd_mfma(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const bool two = a.n_keep > 32;
  if (g.d == 128) return two ? launch_fwd_t<128, 2>(g, a, st) : launch_fwd_t<128, 1>(g, a, st);
  return two ? launch_fwd_t<64, 2>(g, a, st) : launch_fwd_t<64, 1>(g, a, st);
}

// The MFMA backward is not written yet: the shape-generic kernels serve meanwhile.
int launch_bwd_mfma(const Geom& g, const AttnArgs& a, hipStream_t st) { return launch_bwd_generic(g, BSA_BF16, a, st); }
size_t bwd_workspace_mfma(const Geom& g, int n_keep) { return bwd_workspace_generic(g, n_keep); }

}  // namespace bsa
