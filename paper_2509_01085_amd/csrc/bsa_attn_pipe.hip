// Pipelined bf16 MFMA forward for the flagship tile shape (Bk = 64, d = 128 or 64).
//
// A workgroup owns four consecutive query blocks of a head and walks the union of their KV
// lists in ascending order (Eq. 5: each query block multiplies only the tiles on its own
// list).  K/V tiles stream from the raster layout straight into an LDS ring by global->LDS
// DMA (no staging registers, no transposition pass: the tile format of bsa_mfma.h serves both
// the row fragments of K and the transposed fragments of V) while earlier tiles are being
// multiplied; one barrier per tile.  Per tile and wavefront (32 queries on the MFMA column
// index): S^T = K Q^T, online softmax in the exp2 domain, O^T += V^T P^T.
//
//   n_keep <= 32 : four wavefronts (one per query block), two tiles in the ring, two
//                  workgroups per CU: while one waits at its barrier the other multiplies;
//   n_keep  > 32 : eight wavefronts, two per query block splitting its queries, four tiles
//                  in the ring, one workgroup per CU (also the dense baseline's shape).
// Token filling (Sec. 3.2.2) happens in the epilogue: the center's row is parked in LDS and
// copied to the block's pruned positions.
#include <math.h>

#include "bsa_mfma.h"

namespace bsa {

constexpr int PG = 4;     // query blocks per workgroup
constexpr int PBK = 64;   // tokens per block on this path

__device__ inline int xcd_remap8(int n, int total) {
  // workgroup n runs on XCD n % 8; give every XCD one contiguous range of units
  const int q = total >> 3, r = total & 7, x = n & 7;
  return x * q + min(x, r) + (n >> 3);
}

// Ascending walk over the union of four block lists kept as bit masks in LDS.  Every value
// is wave-uniform; readfirstlane moves the words to scalar registers so the bit scanning
// costs scalar, not vector, instructions.
struct Walk4 {
  const uint32_t* masks;  // [4][W]
  int W, own_list, word;
  uint32_t u, own;
  __device__ inline Walk4(const uint32_t* m, int W_, int own_) : masks(m), W(W_), own_list(own_), word(-1), u(0), own(0) {}
  __device__ inline int next(bool& mine) {
    while (u == 0) {
      if (++word >= W) return -1;
      const uint32_t all = masks[word] | masks[W + word] | masks[2 * W + word] | masks[3 * W + word];
      u = __builtin_amdgcn_readfirstlane(all);
      own = __builtin_amdgcn_readfirstlane(masks[own_list * W + word]);
    }
    const int b = __builtin_ctz(u);
    u &= u - 1;
    mine = (own >> b) & 1u;
    return word * 32 + b;
  }
};

#define BSA_FENCE() __builtin_amdgcn_sched_barrier(0)
#define BSA_WAIT_VM(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")

template <int D, bool SPLITQ>
__global__ __launch_bounds__(SPLITQ ? 512 : 256, 2) void fwd_pipe_kernel(Geom g, AttnArgs a) {
  constexpr int NT = SPLITQ ? 512 : 256;  // threads
  constexpr int NB = SPLITQ ? 4 : 2;      // LDS ring depth (tiles)
  constexpr int RB = D * 2;               // bytes per tile row
  constexpr int CPR = D / 8;              // 16-byte chunks per row
  constexpr int TILE = PBK * RB;          // bytes of one K (or V) tile
  constexpr int NI = PBK * CPR / NT;      // DMA instructions per thread per K (or V) tile
  constexpr int DT = D / 32, DS = D / 16;
  extern __shared__ __align__(16) uint8_t smem[];
  uint8_t* ring = smem;                                                  // [NB][K tile | V tile]
  uint32_t* masks = reinterpret_cast<uint32_t*>(smem + NB * 2 * TILE);   // [PG][W]
  __shared__ int koff[PBK];
  __shared__ __align__(16) uint16_t cen_row[PG][D];
  __shared__ float cen_lse[PG];
  __shared__ uint32_t keepbits[PG][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int qb = wave & 3, sub = wave >> 2;  // sub: which 32 queries of the block (always 0 with four wavefronts)
  const int ngroups = (g.N + PG - 1) / PG;
  const int unit = xcd_remap8(blockIdx.x, gridDim.x);
  const int64_t bh = unit / ngroups;
  const int i = (unit % ngroups) * PG + qb;  // this wavefront's query block
  const bool valid = i < g.N;
  const int64_t row = bh * g.N + i;
  const int W = (g.N + 31) / 32;
  const uint16_t* Qh = static_cast<const uint16_t*>(a.Q) + bh * g.L * D;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* Oh = static_cast<uint16_t*>(a.O_out) + bh * g.L * D;
  float* Lh = a.LSE_out + bh * g.L;

  if (tid < PBK) koff[tid] = intra_offset(g, tid);
  for (int k = tid; k < PG * W; k += NT) masks[k] = 0u;
  if (tid < 2 * PG) keepbits[tid >> 1][tid & 1] = 0u;
  __syncthreads();
  if (valid && sub == 0) {
    if (g.dense) {
      for (int w = lane; w < W; w += 64)
        masks[qb * W + w] = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
    } else {
      const int beg = a.q2k_ptr[row], cnt = a.q2k_ptr[row + 1] - beg;
      for (int t = lane; t < cnt; t += 64) {
        const int j = a.q2k_idx[beg + t];
        if ((unsigned)j < (unsigned)g.N) atomicOr(&masks[qb * W + (j >> 5)], 1u << (j & 31));
      }
    }
  }

  // DMA plan of this thread: LDS slot (tid + NT n) of a tile is position p of row r and
  // receives chunk p ^ swz<D>(r) of that row from global memory.
  int goff[NI];
#pragma unroll
  for (int n = 0; n < NI; ++n) {
    const int slot = tid + NT * n, r = slot / CPR, c = (slot % CPR) ^ swz<D>(r);
    goff[n] = koff[r] * D + c * 8;
  }
  auto issue = [&](int jb, int b) {
    const int64_t origin = (int64_t)block_origin_fast(g, jb) * D;
    uint8_t* kdst = ring + b * 2 * TILE + wave * 1024;
#pragma unroll
    for (int n = 0; n < NI; ++n) dma16(Kh + origin + goff[n], kdst + n * (NT * 16));
#pragma unroll
    for (int n = 0; n < NI; ++n) dma16(Vh + origin + goff[n], kdst + TILE + n * (NT * 16));
  };

  // Q^T fragments (B operand): lane (col, grp) holds channels 16 s + 8 grp .. +7 of its query
  const int qpos = 32 * sub + col;
  int qid = -1, qtok = 0;
  if (valid && qpos < a.n_keep) {
    qid = g.dense ? qpos : min(max(a.keep_idx[row * a.n_keep + qpos], 0), PBK - 1);
    qtok = block_origin(g, i) + koff[qid];
    atomicOr(&keepbits[qb][qid >> 5], 1u << (qid & 31));
  }
  bf16x8 qf[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (qid >= 0) v = *reinterpret_cast<const u32x4*>(Qh + (int64_t)qtok * D + 16 * s + 8 * grp);
    qf[s] = as_frag(v);
  }
#pragma unroll
  for (int s = 0; s < DS; ++s) settle(qf[s]);

  // per-lane LDS offsets of the two fragment kinds
  int koffs[DS];  // row fragment of tile row (32 kt + col): chunk 2 s + grp, swizzled
#pragma unroll
  for (int s = 0; s < DS; ++s) koffs[s] = col * RB + (((2 * s + grp) ^ swz<D>(col)) << 4);
  // transposed fragment (channel tile dt, 16-row step ks, half h): lane L of a 16-lane group
  // points at 8 bytes of tile row 16 ks + 8 h + 4 grp + L/4, channels 32 dt + 16 (q16&1) + 4 (L%4) .. +3
  const int L16 = lane & 15, q16 = lane >> 4, rsub = L16 >> 2, jj = L16 & 3;
  const int cl = 2 * (q16 & 1) + (jj >> 1), rhi = D == 128 ? rsub : (rsub >> 1);
  int voffs[2][DT];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      voffs[h][dt] = (8 * h + 4 * grp + rsub) * RB + ((((dt ^ rhi) << 2) | (cl ^ (2 * h + grp))) << 4) + 8 * (jj & 1);

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float c2 = a.sm_scale * kLog2e;
  __syncthreads();

  Walk4 walk(masks, W, qb);  // runs NB-1 tiles ahead of the multiplication; `pending` remembers
  int issued = 0;            // for the tiles in flight whether this wavefront's list has them
  uint32_t pending = 0;
  {
#pragma unroll
    for (int k = 0; k < NB - 1; ++k) {
      bool mk = false;
      const int jb = walk.next(mk);
      if (jb >= 0) {
        issue(jb, k);
        pending |= (mk ? 1u : 0u) << k;
        ++issued;
      }
    }
  }
  for (int t = 0; t < issued; ++t) {
    // tile t must have landed; up to NB-2 younger tiles may stay in flight (2*NI DMAs each)
    const int ahead = issued - t - 1;
    if (NB >= 4 && ahead >= 2) {
      static_assert(2 * NI == 4 || 2 * NI == 2 || NB < 4, "wait immediates below assume 2 or 4 DMAs per tile");
      if (2 * NI == 4) BSA_WAIT_VM(8); else BSA_WAIT_VM(4);
    } else if (NB >= 3 && ahead == 1) {
      if (2 * NI == 4) BSA_WAIT_VM(4); else BSA_WAIT_VM(2);
    } else {
      BSA_WAIT_VM(0);
    }
    raw_barrier();  // tile t visible to all; everyone is done with tile t-1, whose buffer is refilled now
    {
      bool mn = false;
      const int jn = walk.next(mn);
      if (jn >= 0) {
#ifndef BSA_EXP_NOLOAD
        issue(jn, (t + NB - 1) & (NB - 1));
#endif
        pending |= (mn ? 1u : 0u) << (NB - 1);
        ++issued;
      }
    }
#ifdef BSA_EXP_NOCOMPUTE
    const bool mine = false;
#elif defined(BSA_EXP_ALLMINE)
    const bool mine = true;
#else
    const bool mine = pending & 1u;
#endif
    pending >>= 1;
    if (mine) {
      // 64 keys x this wavefront's 32 queries.  The 4*DS A fragments of the tile (K rows for
      // both key halves, then V^T) are read from LDS through a ring of RING register
      // fragments, RING MFMAs ahead of their use.  Matrix and vector instructions share the
      // register-file bandwidth on this chip and barely co-execute (measured), so the code
      // keeps the vector work per tile minimal rather than trying to hide it.
      const uint8_t* Kb = ring + (t & (NB - 1)) * 2 * TILE;
      const uint8_t* Vb = Kb + TILE;
      constexpr int RING = 8, NF = 2 * DS + 4 * DT;
      auto frag = [&](int f) -> bf16x8 {
        if (f < 2 * DS) return lds_frag(reinterpret_cast<const uint16_t*>(Kb + 32 * (f / DS) * RB + koffs[f % DS]));
        const int v = f - 2 * DS, ks = v / DT, dt = v % DT;
        return lds_frag_tr(Vb + voffs[0][dt] + 16 * ks * RB, Vb + voffs[1][dt] + 16 * ks * RB);
      };
      bf16x8 fr[RING];
#pragma unroll
      for (int f = 0; f < RING; ++f) fr[f] = frag(f);
      BSA_FENCE();
      f32x16 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
      for (int f = 0; f < 2 * DS; ++f) {
        s[f / DS] = mfma32(fr[f % RING], qf[f % DS], s[f / DS]);
        if (f + RING < NF) fr[f % RING] = frag(f + RING);
        if (f & 1) BSA_FENCE();
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      mx = fmaxf(mx, xor32(mx));
      const float mnew = fmaxf(m, mx * c2);  // c2 > 0: the maximum commutes with the scaling
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);
      float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[0][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][r], c2, -mnew));
        s[1][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[1][r], c2, -mnew));
        sum0 += s[0][r];
        sum1 += s[1][r];
      }
      l = l * alpha + (sum0 + sum1);  // per-lane partial; the lane pair is summed at the end
      m = mnew;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {  // rescale only when some row's maximum moved
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
      }
      bf16x8 pf[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) pf[ks] = d_to_b(s[ks >> 1], ks & 1);
      BSA_FENCE();
#pragma unroll
      for (int f = 2 * DS; f < NF; ++f) {
        const int v = f - 2 * DS;  // V^T fragments in (key step, channel tile) order: consecutive MFMAs hit different accumulators
        o[v % DT] = mfma32(fr[f % RING], pf[v / DT], o[v % DT]);
        if (f + RING < NF) fr[f % RING] = frag(f + RING);
        if (f & 1) BSA_FENCE();
      }
    }
  }

  // epilogue: normalise, store the retained rows, park the center's row for the fill
  const float ltot = l + xor32(l);
  const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
  const float lse = ltot > 0.f ? (m + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
  if (qid >= 0) {
    const bool is_center = !g.dense && qid == g.center;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 v;
        v.x = pack_bf16(o[dt][4 * r4 + 0] * inv, o[dt][4 * r4 + 1] * inv);
        v.y = pack_bf16(o[dt][4 * r4 + 2] * inv, o[dt][4 * r4 + 3] * inv);
        const int ch = 32 * dt + 8 * r4 + 4 * grp;
        *reinterpret_cast<u32x2*>(Oh + (int64_t)qtok * D + ch) = v;
        if (is_center) *reinterpret_cast<u32x2*>(&cen_row[qb][ch]) = v;
      }
    if (grp == 0) {
      Lh[qtok] = lse;
      if (is_center) cen_lse[qb] = lse;
    }
  }
  __syncthreads();
  // token filling: lane c of the block's first wavefront owns intra-block token c
  if (valid && !g.dense && sub == 0) {
    const bool kept = (keepbits[qb][lane >> 5] >> (lane & 31)) & 1u;
    if (!kept) {
      const int64_t tok = block_origin(g, i) + koff[lane];
#pragma unroll
      for (int q = 0; q < D / 8; ++q)
        *reinterpret_cast<u32x4*>(Oh + tok * D + 8 * q) = *reinterpret_cast<const u32x4*>(&cen_row[qb][8 * q]);
      Lh[tok] = cen_lse[qb];
    }
  }
}

template <int D, bool SPLITQ>
static int launch_fwd_pipe_t(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const int W = (g.N + 31) / 32;
  const size_t lds = (size_t)(SPLITQ ? 4 : 2) * 2 * PBK * D * 2 + (size_t)PG * W * 4;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(fwd_pipe_kernel<D, SPLITQ>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return BSA_ERR_LAUNCH;
  hipLaunchKernelGGL((fwd_pipe_kernel<D, SPLITQ>), dim3(((g.N + PG - 1) / PG) * g.B * g.H), dim3(SPLITQ ? 512 : 256), lds, st, g, a);
  return check_launch();
}

int launch_fwd_pipe(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const bool splitq = a.n_keep > 32;
  if (g.d == 128) return splitq ? launch_fwd_pipe_t<128, true>(g, a, st) : launch_fwd_pipe_t<128, false>(g, a, st);
  return splitq ? launch_fwd_pipe_t<64, true>(g, a, st) : launch_fwd_pipe_t<64, false>(g, a, st);
}

}  // namespace bsa
