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

// Workgroups are dispatched round-robin over the 8 XCDs (id n runs on XCD n % 8), each with its
// own L2.  Remap the linear id so that every XCD works through one contiguous range of
// (head, group) units in order: workgroups that run side by side on an XCD then belong to the
// same head and walk the same K/V tiles in step, which is what lets that L2 serve the re-reads.
__device__ inline int xcd_remap(int n, int total) {
  const int q = total >> 3, r = total & 7, x = n & 7;
  return x * q + min(x, r) + (n >> 3);
}

#define BSA_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

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
  const int ngroups = (g.N + G - 1) / G;
  const int unit = xcd_remap(blockIdx.x, gridDim.x);
  const int64_t bh = unit / ngroups;
  const int i = (unit % ngroups) * G + wave;  // this wavefront's query block
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
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
    for (int s = 0; s < DS; ++s) settle(qf[qt][s]);
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
#ifndef BSA_EXP_NOLOAD
    if (jn >= 0) st.load(g, Kh, Vh, jn, koff);
#endif
#ifdef BSA_EXP_NOCOMPUTE
    mine = false;
#endif
    if (mine) {
      // The 4*DS A fragments of a tile (K rows for both key halves, then V^T) are read from
      // LDS through a ring of RING registers-fragments, RING MFMAs ahead of their use, so the
      // read latency overlaps matrix work instead of preceding every single MFMA.
      constexpr int RING = 8, NF = 4 * DS;
      const uint16_t* kp = Ks + buf * BK * KLD + col * KLD + 8 * grp;
      const uint16_t* vp = Vs + buf * D * VLD + col * VLD + 8 * grp;
      auto frag = [&](int f) -> bf16x8 {
        if (f < 2 * DS) return lds_frag(kp + (32 * (f / DS)) * KLD + 16 * (f % DS));
        const int v = f - 2 * DS;
        return lds_frag(vp + (32 * (v / 4)) * VLD + 16 * (v % 4));
      };
      bf16x8 ring[RING];
#pragma unroll
      for (int f = 0; f < RING; ++f) ring[f] = frag(f);
      BSA_SCHED_FENCE();
      f32x16 s[NQT][2];
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qt][kt][r] = 0.f;
#pragma unroll
      for (int f = 0; f < 2 * DS; ++f) {
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) s[qt][f / DS] = mfma32(ring[f % RING], qf[qt][f % DS], s[qt][f / DS]);
        if (f + RING < NF) ring[f % RING] = frag(f + RING);
        if (f & 1) BSA_SCHED_FENCE();
      }
      bf16x8 pf[NQT][4];
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) {
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qt][kt][r]);
        mx = fmaxf(mx, xor32(mx));
        const float mnew = fmaxf(m[qt], mx * c2);  // c2 > 0: the maximum commutes with the scaling
        const float alpha = __builtin_amdgcn_exp2f(m[qt] - mnew);
        float sum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qt][kt][r], c2, -mnew));
            s[qt][kt][r] = p;
            sum += p;
          }
        l[qt] = l[qt] * alpha + sum;  // per-lane partial; the lane pair is summed at the end
        m[qt] = mnew;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {  // rescale only when some row's maximum moved
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qt][dt][r] *= alpha;
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) pf[qt][ks] = d_to_b(s[qt][ks >> 1], ks & 1);
      }
      BSA_SCHED_FENCE();
#pragma unroll
      for (int f = 2 * DS; f < NF; ++f) {
        const int v = f - 2 * DS;
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) o[qt][v / 4] = mfma32(ring[f % RING], pf[qt][v % 4], o[qt][v / 4]);
        if (f + RING < NF) ring[f % RING] = frag(f + RING);
        if (f & 1) BSA_SCHED_FENCE();
      }
    }
#ifndef BSA_EXP_NOLOAD
    if (jn >= 0) st.store(Ks + (buf ^ 1) * BK * KLD, Vs + (buf ^ 1) * D * VLD);
#endif
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
  hipLaunchKernelGGL((fwd_mfma_kernel<D, NQT>), dim3(((g.N + G - 1) / G) * g.B * g.H), dim3(256), lds, st, g, a);
  return check_launch();
}

int launch_fwd_mfma(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const bool two = a.n_keep > 32;
  if (g.d == 128) return two ? launch_fwd_t<128, 2>(g, a, st) : launch_fwd_t<128, 1>(g, a, st);
  return two ? launch_fwd_t<64, 2>(g, a, st) : launch_fwd_t<64, 1>(g, a, st);
}

// =====================================================================================
// Backward.  Three kernels, no floating-point atomics:
//   pre   per query block: gather the retained Q rows and the folded upstream gradient
//         g (dO of the row; for the center row plus the dO of every pruned token, the
//         gradient of the fill copy), delta = <g, O>, LSE in the exp2 domain; written
//         to the workspace as compact bf16 tiles in the two layouts the MFMA operands need
//         (row-major, and transposed with slot-permuted query positions).
//   dQ    same walk as the forward (four query blocks per workgroup, union of KV lists):
//         S^T = K Q^T, dP^T = V G^T, dS^T = P^T (dP^T - delta), dQ^T += K^T dS^T.
//   dKV   a workgroup owns two adjacent KV blocks (a wavefront owns 32 keys) and walks the
//         union of their k2q lists; the query-block tiles are streamed from the workspace:
//         S = Qc K^T, dP = Gc V^T, dV^T += Gc^T P, dK^T += Qc^T dS.
// =====================================================================================

template <int D, int NQT>
struct BwdTile {  // byte layout of one query block's tile in the workspace and in LDS
  static constexpr int NK = 32 * NQT;
  static constexpr int RLD = D + 8;    // row stride of the row-major parts (bf16 elements)
  static constexpr int TLD = NK + 8;   // row stride of the transposed parts
  static constexpr int QC = 0;
  static constexpr int GC = QC + NK * RLD * 2;
  static constexpr int QT = GC + NK * RLD * 2;
  static constexpr int GT = QT + D * TLD * 2;
  static constexpr int LS = GT + D * TLD * 2;   // float lse2[NK]
  static constexpr int DL = LS + NK * 4;        // float delta[NK]
  static constexpr int BYTES = ((DL + NK * 4) + 255) & ~255;
};

template <int D, int NQT>
__global__ __launch_bounds__(256) void bwd_pre_mfma_kernel(Geom g, AttnArgs a) {
  using T = BwdTile<D, NQT>;
  __shared__ __align__(16) uint16_t qs[T::NK][D];
  __shared__ __align__(16) uint16_t gs[T::NK][D];
  __shared__ float dpart[T::NK][4];
  __shared__ int keepflag[BK];
  __shared__ int qtok[T::NK];
  __shared__ int koff[BK];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const uint16_t* Qh = static_cast<const uint16_t*>(a.Q) + bh * g.L * D;
  const uint16_t* Oh = static_cast<const uint16_t*>(a.O) + bh * g.L * D;
  const uint16_t* dOh = static_cast<const uint16_t*>(a.dO) + bh * g.L * D;
  const float* Lh = a.LSE_in + bh * g.L;
  uint8_t* tile = static_cast<uint8_t*>(a.ws) + row * (int64_t)T::BYTES;
  const int origin = block_origin(g, i);

  if (tid < BK) {
    koff[tid] = intra_offset(g, tid);
    keepflag[tid] = 0;
  }
  __syncthreads();
  int cpos = -1;  // position of the center among the retained rows (same in every thread)
  if (tid < T::NK) {
    int c = -1;
    if (tid < a.n_keep) c = g.dense ? tid : min(max(a.keep_idx[row * a.n_keep + tid], 0), BK - 1);
    qtok[tid] = c >= 0 ? origin + koff[c] : -1;
    if (c >= 0) keepflag[c] = 1;
  }
  __syncthreads();
  if (!g.dense)
    for (int q = 0; q < a.n_keep; ++q)
      if (qtok[q] == origin + koff[g.center]) cpos = q;

  // thread (q = tid / 4 + 64 * pass, quarter = tid % 4) handles D/4 channels of row q
  constexpr int CH = D / 4;
  for (int q = tid >> 2; q < T::NK; q += 64) {
    const int part = tid & 3;
    const int tok = qtok[q];
    float dsum = 0.f;
    for (int c8 = 0; c8 < CH; c8 += 8) {
      const int ch = part * CH + c8;
      u32x4 qv = {0u, 0u, 0u, 0u}, gv = {0u, 0u, 0u, 0u};
      if (tok >= 0) {
        qv = *reinterpret_cast<const u32x4*>(Qh + (int64_t)tok * D + ch);
        gv = *reinterpret_cast<const u32x4*>(dOh + (int64_t)tok * D + ch);
        const u32x4 ov = *reinterpret_cast<const u32x4*>(Oh + (int64_t)tok * D + ch);
        float gf[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          gf[2 * e] = __uint_as_float(gv[e] << 16);
          gf[2 * e + 1] = __uint_as_float(gv[e] & 0xffff0000u);
        }
        if (q == cpos) {  // fold the fill copies: pruned tokens, ascending intra-block id
          for (int u = 0; u < BK; ++u) {
            if (keepflag[u]) continue;
            const u32x4 pv = *reinterpret_cast<const u32x4*>(dOh + (int64_t)(origin + koff[u]) * D + ch);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              gf[2 * e] += __uint_as_float(pv[e] << 16);
              gf[2 * e + 1] += __uint_as_float(pv[e] & 0xffff0000u);
            }
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) gv[e] = pack_bf16(gf[2 * e], gf[2 * e + 1]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          dsum += gf[2 * e] * __uint_as_float(ov[e] << 16);
          dsum += gf[2 * e + 1] * __uint_as_float(ov[e] & 0xffff0000u);
        }
      }
      *reinterpret_cast<u32x4*>(&qs[q][ch]) = qv;
      *reinterpret_cast<u32x4*>(&gs[q][ch]) = gv;
      *reinterpret_cast<u32x4*>(tile + T::QC + (q * T::RLD + ch) * 2) = qv;
      *reinterpret_cast<u32x4*>(tile + T::GC + (q * T::RLD + ch) * 2) = gv;
    }
    dpart[q][part] = dsum;
  }
  __syncthreads();
  if (tid < T::NK) {
    const int tok = qtok[tid];
    float* ls = reinterpret_cast<float*>(tile + T::LS);
    float* dl = reinterpret_cast<float*>(tile + T::DL);
    ls[tid] = tok >= 0 ? Lh[tok] * kLog2e : INFINITY;  // padding rows: exp2(x - inf) = 0
    dl[tid] = tok >= 0 ? (dpart[tid][0] + dpart[tid][1]) + (dpart[tid][2] + dpart[tid][3]) : 0.f;
  }
  // transposed tiles: element (d, slot_pos(q)) = row q, channel d; 8 positions per 16-byte store
  for (int u = tid; u < D * (T::NK / 8); u += 256) {
    const int dch = u / (T::NK / 8), p8 = (u % (T::NK / 8)) * 8;
    uint32_t qo[4], go[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // positions p8 + 2e, p8 + 2e + 1 hold queries x with slot_pos(x) = position (slot_pos is an involution)
      const int x0 = slot_pos(p8 + 2 * e), x1 = slot_pos(p8 + 2 * e + 1);
      qo[e] = (uint32_t)qs[x0][dch] | ((uint32_t)qs[x1][dch] << 16);
      go[e] = (uint32_t)gs[x0][dch] | ((uint32_t)gs[x1][dch] << 16);
    }
    const u32x4 qv = {qo[0], qo[1], qo[2], qo[3]}, gv = {go[0], go[1], go[2], go[3]};
    *reinterpret_cast<u32x4*>(tile + T::QT + (dch * T::TLD + p8) * 2) = qv;
    *reinterpret_cast<u32x4*>(tile + T::GT + (dch * T::TLD + p8) * 2) = gv;
  }
}

// ------------------------------------------------------------------------------- dQ
template <int D, int NQT>
__global__ __launch_bounds__(256) void bwd_dq_mfma_kernel(Geom g, AttnArgs a) {
  using T = BwdTile<D, NQT>;
  constexpr int KLD = Stage<D>::KLD;
  constexpr int DT = D / 32, DS = D / 16;
  constexpr int BUF = (2 * BK * KLD + D * VLD);  // K rows, V rows, K^T : bf16 elements per buffer
  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* base = reinterpret_cast<uint16_t*>(smem);           // [2][BUF]
  uint32_t* masks = reinterpret_cast<uint32_t*>(base + 2 * BUF);  // [G][W]
  __shared__ int koff[BK];
  __shared__ uint32_t keepbits[G][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int64_t bh = blockIdx.y;
  const int i = blockIdx.x * G + wave;
  const bool valid = i < g.N;
  const int64_t row = bh * g.N + i;
  const int W = (g.N + 31) / 32;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* dQh = static_cast<uint16_t*>(a.dQ) + bh * g.L * D;
  const uint8_t* tile = static_cast<const uint8_t*>(a.ws) + row * (int64_t)T::BYTES;

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
  bf16x8 qf[NQT][DS], gf[NQT][DS];
  float lse2[NQT], delta[NQT];
  int qtok[NQT], qid[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int pos = 32 * qt + col;
    qid[qt] = -1;
    qtok[qt] = 0;
    lse2[qt] = INFINITY;
    delta[qt] = 0.f;
    if (valid && pos < a.n_keep) {
      const int c = g.dense ? pos : min(max(a.keep_idx[row * a.n_keep + pos], 0), BK - 1);
      qid[qt] = c;
      qtok[qt] = block_origin(g, i) + koff[c];
      atomicOr(&keepbits[wave][c >> 5], 1u << (c & 31));
      lse2[qt] = reinterpret_cast<const float*>(tile + T::LS)[pos];
      delta[qt] = reinterpret_cast<const float*>(tile + T::DL)[pos];
    }
#pragma unroll
    for (int s = 0; s < DS; ++s) {
      u32x4 qv = {0u, 0u, 0u, 0u}, gv = {0u, 0u, 0u, 0u};
      if (qid[qt] >= 0) {
        qv = *reinterpret_cast<const u32x4*>(tile + T::QC + (pos * T::RLD + 16 * s + 8 * grp) * 2);
        gv = *reinterpret_cast<const u32x4*>(tile + T::GC + (pos * T::RLD + 16 * s + 8 * grp) * 2);
      }
      qf[qt][s] = as_frag(qv);
      gf[qt][s] = as_frag(gv);
    }
  }
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    settle(lse2[qt]);
    settle(delta[qt]);
#pragma unroll
    for (int s = 0; s < DS; ++s) {
      settle(qf[qt][s]);
      settle(gf[qt][s]);
    }
  }
  __syncthreads();

  f32x16 dq[NQT][DT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[qt][dt][r] = 0.f;
  const float c2 = a.sm_scale * kLog2e;

  UnionWalk walk(masks, W, wave);
  Stage<D> sk;   // K rows + K^T
  u32x4 vreg[Stage<D>::KV];  // V rows
  auto load_v = [&](int jb) {
    const int64_t origin = block_origin(g, jb);
#pragma unroll
    for (int n = 0; n < Stage<D>::KV; ++n) {
      const int u = tid + 256 * n, r = u / (D / 8), cg = u % (D / 8);
      vreg[n] = *reinterpret_cast<const u32x4*>(Vh + (origin + koff[r]) * D + 8 * cg);
    }
  };
  auto store_v = [&](uint16_t* Vr) {
#pragma unroll
    for (int n = 0; n < Stage<D>::KV; ++n) {
      const int u = tid + 256 * n, r = u / (D / 8), cg = u % (D / 8);
      *reinterpret_cast<u32x4*>(Vr + r * KLD + 8 * cg) = vreg[n];
    }
  };
  bool mine = false, mine_next = false;
  int jb = walk.next(mine);
  if (jb >= 0) {
    sk.load(g, Kh, Kh, jb, koff);
    load_v(jb);
    sk.store(base, base + 2 * BK * KLD);
    store_v(base + BK * KLD);
  }
  __syncthreads();
  int buf = 0;
  while (jb >= 0) {
    const int jn = walk.next(mine_next);
    if (jn >= 0) {
      sk.load(g, Kh, Kh, jn, koff);
      load_v(jn);
    }
    if (mine) {
      const uint16_t* Kb = base + buf * BUF;
      const uint16_t* Vb = Kb + BK * KLD;
      const uint16_t* Kt = Kb + 2 * BK * KLD;
      bf16x8 dsf[NQT][4];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        f32x16 s[NQT], dp[NQT];
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qt][r] = dp[qt][r] = 0.f;
#pragma unroll
        for (int sp = 0; sp < DS; ++sp) {
          const bf16x8 kfrag = lds_frag(Kb + (32 * kt + col) * KLD + 16 * sp + 8 * grp);
          const bf16x8 vfrag = lds_frag(Vb + (32 * kt + col) * KLD + 16 * sp + 8 * grp);
#pragma unroll
          for (int qt = 0; qt < NQT; ++qt) {
            s[qt] = mfma32(kfrag, qf[qt][sp], s[qt]);
            dp[qt] = mfma32(vfrag, gf[qt][sp], dp[qt]);
          }
        }
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(s[qt][r] * c2 - lse2[qt]);
            s[qt][r] = p * (dp[qt][r] - delta[qt]);
          }
          dsf[qt][2 * kt] = d_to_b(s[qt], 0);
          dsf[qt][2 * kt + 1] = d_to_b(s[qt], 1);
        }
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 ktfrag = lds_frag(Kt + (32 * dt + col) * VLD + 16 * ks + 8 * grp);
#pragma unroll
          for (int qt = 0; qt < NQT; ++qt) dq[qt][dt] = mfma32(ktfrag, dsf[qt][ks], dq[qt][dt]);
        }
    }
    if (jn >= 0) {
      uint16_t* nb = base + (buf ^ 1) * BUF;
      sk.store(nb, nb + 2 * BK * KLD);
      store_v(nb + BK * KLD);
    }
    __syncthreads();
    buf ^= 1;
    jb = jn;
    mine = mine_next;
  }
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    if (qid[qt] < 0) continue;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 v;
        v.x = pack_bf16(dq[qt][dt][4 * r4 + 0] * a.sm_scale, dq[qt][dt][4 * r4 + 1] * a.sm_scale);
        v.y = pack_bf16(dq[qt][dt][4 * r4 + 2] * a.sm_scale, dq[qt][dt][4 * r4 + 3] * a.sm_scale);
        *reinterpret_cast<u32x2*>(dQh + (int64_t)qtok[qt] * D + 32 * dt + 8 * r4 + 4 * grp) = v;
      }
  }
  // pruned queries take no part in the forward: zero gradient rows
  if (valid && !g.dense) {
    const bool kept = (keepbits[wave][lane >> 5] >> (lane & 31)) & 1u;
    if (!kept) {
      const int64_t tok = block_origin(g, i) + koff[lane];
      const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int q = 0; q < D / 8; ++q) *reinterpret_cast<u32x4*>(dQh + tok * D + 8 * q) = z;
    }
  }
}

// ------------------------------------------------------------------------------ dK, dV
// Ascending walk over the union of two k2q lists (bit masks in LDS).
struct PairWalk {
  const uint32_t* masks;  // [2][W]
  int W, which, word;
  uint32_t u, own;
  __device__ inline PairWalk(const uint32_t* m, int W_, int which_) : masks(m), W(W_), which(which_), word(-1), u(0), own(0) {}
  __device__ inline int next(bool& mine) {
    while (u == 0) {
      if (++word >= W) return -1;
      u = masks[word] | masks[W + word];
      own = masks[which * W + word];
    }
    const int b = __ffs(u) - 1;
    u &= u - 1;
    mine = (own >> b) & 1u;
    return word * 32 + b;
  }
};

template <int D, int NQT>
__global__ __launch_bounds__(256) void bwd_dkv_mfma_kernel(Geom g, AttnArgs a) {
  using T = BwdTile<D, NQT>;
  constexpr int DT = D / 32, DS = D / 16;
  constexpr int NV = (T::BYTES + 4095) / 4096;  // 16-byte loads per thread per tile
  extern __shared__ __align__(16) uint8_t smem[];
  uint8_t* tiles = smem;                                              // [2][T::BYTES]
  uint32_t* masks = reinterpret_cast<uint32_t*>(smem + 2 * T::BYTES);  // [2][W]
  __shared__ int koff[BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int64_t bh = blockIdx.y;
  const int which = wave >> 1, half = wave & 1;
  const int j = blockIdx.x * 2 + which;  // this wavefront's KV block; it owns keys 32*half .. +31
  const bool valid = j < g.N;
  const int64_t colrow = bh * g.N + j;
  const int W = (g.N + 31) / 32;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* dKh = static_cast<uint16_t*>(a.dK) + bh * g.L * D;
  uint16_t* dVh = static_cast<uint16_t*>(a.dV) + bh * g.L * D;
  const uint8_t* ws = static_cast<const uint8_t*>(a.ws) + bh * g.N * (int64_t)T::BYTES;

  if (tid < BK) koff[tid] = intra_offset(g, tid);
  for (int k = tid; k < 2 * W; k += 256) masks[k] = 0u;
  __syncthreads();
  if (valid && half == 0) {
    if (g.dense) {
      for (int w = lane; w < W; w += 64)
        masks[which * W + w] = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
    } else {
      const int beg = a.k2q_ptr[colrow], cnt = a.k2q_ptr[colrow + 1] - beg;
      for (int t = lane; t < cnt; t += 64) {
        const int ib = a.k2q_idx[beg + t];
        if ((unsigned)ib < (unsigned)g.N) atomicOr(&masks[which * W + (ib >> 5)], 1u << (ib & 31));
      }
    }
  }
  // stationary B operands: K^T and V^T fragments of the lane's key
  const int64_t ktok = valid ? block_origin(g, j) + koff[32 * half + col] : 0;
  bf16x8 kf[DS], vf[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s) {
    u32x4 kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
    if (valid) {
      kv = *reinterpret_cast<const u32x4*>(Kh + ktok * D + 16 * s + 8 * grp);
      vv = *reinterpret_cast<const u32x4*>(Vh + ktok * D + 16 * s + 8 * grp);
    }
    kf[s] = as_frag(kv);
    vf[s] = as_frag(vv);
  }
#pragma unroll
  for (int s = 0; s < DS; ++s) {
    settle(kf[s]);
    settle(vf[s]);
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[dt][r] = dv[dt][r] = 0.f;
  const float c2 = a.sm_scale * kLog2e;
  __syncthreads();

  PairWalk walk(masks, W, which);
  u32x4 pre[NV];
  auto load_tile = [&](int ib) {
    const uint8_t* src = ws + ib * (int64_t)T::BYTES;
#pragma unroll
    for (int n = 0; n < NV; ++n) {
      const int off = (tid + 256 * n) * 16;
      if (off < T::BYTES) pre[n] = *reinterpret_cast<const u32x4*>(src + off);
    }
  };
  auto store_tile = [&](uint8_t* dst) {
#pragma unroll
    for (int n = 0; n < NV; ++n) {
      const int off = (tid + 256 * n) * 16;
      if (off < T::BYTES) *reinterpret_cast<u32x4*>(dst + off) = pre[n];
    }
  };
  bool mine = false, mine_next = false;
  int ib = walk.next(mine);
  if (ib >= 0) {
    load_tile(ib);
    store_tile(tiles);
  }
  __syncthreads();
  int buf = 0;
  while (ib >= 0) {
    const int in = walk.next(mine_next);
    if (in >= 0) load_tile(in);
    if (mine) {
      const uint8_t* tb = tiles + buf * T::BYTES;
      const uint16_t* Qc = reinterpret_cast<const uint16_t*>(tb + T::QC);
      const uint16_t* Gc = reinterpret_cast<const uint16_t*>(tb + T::GC);
      const uint16_t* Qt = reinterpret_cast<const uint16_t*>(tb + T::QT);
      const uint16_t* Gt = reinterpret_cast<const uint16_t*>(tb + T::GT);
      const float* ls = reinterpret_cast<const float*>(tb + T::LS);
      const float* dl = reinterpret_cast<const float*>(tb + T::DL);
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
        for (int sp = 0; sp < DS; ++sp) {
          s = mfma32(lds_frag(Qc + (32 * qt + col) * T::RLD + 16 * sp + 8 * grp), kf[sp], s);
          dp = mfma32(lds_frag(Gc + (32 * qt + col) * T::RLD + 16 * sp + 8 * grp), vf[sp], dp);
        }
        // D layout: lane = key column, register r = query row 32*qt + 8*(r/4) + 4*grp + r%4
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(ls + 32 * qt + 8 * r4 + 4 * grp);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(dl + 32 * qt + 8 * r4 + 4 * grp);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p = __builtin_amdgcn_exp2f(s[4 * r4 + e] * c2 - l4[e]);
            s[4 * r4 + e] = p;
            dp[4 * r4 + e] = p * (dp[4 * r4 + e] - d4[e]);
          }
        }
        const bf16x8 pf0 = d_to_b(s, 0), pf1 = d_to_b(s, 1), df0 = d_to_b(dp, 0), df1 = d_to_b(dp, 1);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const uint16_t* gt = Gt + (32 * dt + col) * T::TLD + 32 * qt + 8 * grp;
          const uint16_t* qtp = Qt + (32 * dt + col) * T::TLD + 32 * qt + 8 * grp;
          dv[dt] = mfma32(lds_frag(gt), pf0, dv[dt]);
          dv[dt] = mfma32(lds_frag(gt + 16), pf1, dv[dt]);
          dk[dt] = mfma32(lds_frag(qtp), df0, dk[dt]);
          dk[dt] = mfma32(lds_frag(qtp + 16), df1, dk[dt]);
        }
      }
    }
    if (in >= 0) store_tile(tiles + (buf ^ 1) * T::BYTES);
    __syncthreads();
    buf ^= 1;
    ib = in;
    mine = mine_next;
  }
  if (valid) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 kv, vv;
        kv.x = pack_bf16(dk[dt][4 * r4 + 0] * a.sm_scale, dk[dt][4 * r4 + 1] * a.sm_scale);
        kv.y = pack_bf16(dk[dt][4 * r4 + 2] * a.sm_scale, dk[dt][4 * r4 + 3] * a.sm_scale);
        vv.x = pack_bf16(dv[dt][4 * r4 + 0], dv[dt][4 * r4 + 1]);
        vv.y = pack_bf16(dv[dt][4 * r4 + 2], dv[dt][4 * r4 + 3]);
        const int ch = 32 * dt + 8 * r4 + 4 * grp;
        *reinterpret_cast<u32x2*>(dKh + ktok * D + ch) = kv;
        *reinterpret_cast<u32x2*>(dVh + ktok * D + ch) = vv;
      }
  }
}

template <int D, int NQT>
static int launch_bwd_t(const Geom& g, const AttnArgs& a, hipStream_t st) {
  using T = BwdTile<D, NQT>;
  const int W = (g.N + 31) / 32;
  if (a.stages & BSA_BWD_PRE) hipLaunchKernelGGL((bwd_pre_mfma_kernel<D, NQT>), dim3(g.rows), dim3(256), 0, st, g, a);
  const size_t lds_q = (size_t)2 * (2 * BK * Stage<D>::KLD + D * VLD) * 2 + (size_t)G * W * 4;
  const size_t lds_kv = (size_t)2 * T::BYTES + (size_t)2 * W * 4;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_mfma_kernel<D, NQT>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_q) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dkv_mfma_kernel<D, NQT>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_kv) != hipSuccess)
    return BSA_ERR_LAUNCH;
  if (a.stages & BSA_BWD_DQ) hipLaunchKernelGGL((bwd_dq_mfma_kernel<D, NQT>), dim3((g.N + G - 1) / G, g.B * g.H), dim3(256), lds_q, st, g, a);
  if (a.stages & BSA_BWD_DKV) hipLaunchKernelGGL((bwd_dkv_mfma_kernel<D, NQT>), dim3((g.N + 1) / 2, g.B * g.H), dim3(256), lds_kv, st, g, a);
  return check_launch();
}

int launch_bwd_mfma(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const bool two = a.n_keep > 32;
  if (g.d == 128) return two ? launch_bwd_t<128, 2>(g, a, st) : launch_bwd_t<128, 1>(g, a, st);
  return two ? launch_bwd_t<64, 2>(g, a, st) : launch_bwd_t<64, 1>(g, a, st);
}

size_t bwd_workspace_mfma(const Geom& g, int n_keep) {
  const bool two = n_keep > 32;
  const size_t per_row = g.d == 128 ? (two ? BwdTile<128, 2>::BYTES : BwdTile<128, 1>::BYTES)
                                    : (two ? BwdTile<64, 2>::BYTES : BwdTile<64, 1>::BYTES);
  return per_row * (size_t)g.rows;
}

}  // namespace bsa
