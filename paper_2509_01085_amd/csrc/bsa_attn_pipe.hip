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
//   n_keep <= 16 : as the first, but a wavefront carries two query blocks (16 MFMA columns
//                  each) and the workgroup eight.
// Token filling (Sec. 3.2.2) happens in the epilogue: the rows of the critical tokens (one per
// window of the block) are parked in LDS and copied to their windows' pruned positions.
#include <math.h>

#include "bsa_mfma.h"

namespace bsa {

constexpr int PG = 4;     // query blocks per workgroup
constexpr int PBK = 64;   // tokens per block on this path

bool mfma_supported(const Geom& g, int dtype, int n_keep) {
  return dtype == BSA_BF16 && g.Bk == PBK && (g.d == 128 || g.d == 64) && n_keep <= PBK;
}

// ---- work items -------------------------------------------------------------------------
// A launch covers `units` units of work (four query blocks of a head each).  Workgroups are
// dispatched round-robin over the 8 XCDs, so XCD x is given the contiguous unit range
// [x*q + min(x, r), ...) with q = units / 8, r = units % 8: neighbouring query blocks, whose
// lists overlap, share that XCD's L2.  When the launch is only a few rounds long (units per
// workgroup slot), its tail leaves most of the chip idle; then the last split_n units of every
// XCD's range are walked in split_S segments by separate, shorter workgroups dispatched last,
// and a combine launch merges their partial results.  The dK/dV launch (units = pairs of KV
// blocks, one workgroup per CU) does the same for the units of its last, partly filled round.
constexpr int kCUs = 256;  // compute units of the MI355X


struct SplitPlan {
  int S, n;   // segments per split unit; split units per XCD (0: no splitting)
  int grid;   // workgroups of the main launch
  int units;  // number of split units = workgroups of the combine launch
};

static SplitPlan plan_split(int units, int slots, bool allow) {
  SplitPlan p{1, 0, 0, 0};
  const int q = units / 8, r = units % 8, cmax = q + (r ? 1 : 0);
  if (allow && q >= 5 && units < 12 * slots) {  // short launch: split the last fifth in four
    p.S = 4;
    p.n = (q + 4) / 5;
  }
  p.grid = 8 * (cmax - p.n + p.S * p.n);
  p.units = 8 * p.n;
  return p;
}

struct Item {
  int unit, seg, nseg;
  int sidx;  // ordinal of a split unit (addresses its partial results), -1 for a whole unit
};

__device__ inline bool item_of(int b, int units, int S, int n, Item& it) {
  const int q = units >> 3, r = units & 7, x = b & 7, k = b >> 3;
  const int start = x * q + min(x, r), cnt = q + (x < r ? 1 : 0), whole = cnt - n;
  if (k < whole) {
    it.unit = start + k; it.seg = 0; it.nseg = 1; it.sidx = -1;
    return true;
  }
  const int kk = k - whole, si = kk / S;
  if (si >= n) return false;
  it.unit = start + whole + si; it.seg = kk - si * S; it.nseg = S; it.sidx = x * n + si;
  return true;
}

// the split unit a workgroup of the combine launch finishes
__device__ inline Item split_item_of(int b, int units, int S, int n) {
  const int q = units >> 3, r = units & 7, x = b & 7, si = b >> 3;
  Item it;
  it.unit = x * q + min(x, r) + (q + (x < r ? 1 : 0) - n) + si; it.seg = 0; it.nseg = S; it.sidx = x * n + si;
  return it;
}

// Ascending walk over the union of NL block lists kept as bit masks in LDS.  Every value
// is wave-uniform; readfirstlane moves the words to scalar registers so the bit scanning
// costs scalar, not vector, instructions.
template <int NL, int NOWN>
struct WalkN {
  const uint32_t* masks;  // [NL][W]
  int W, own_list, word, left;
  uint32_t u, own, own2;  // own, own2: the wavefront's own list(s), NOWN of them, own_list and own_list + 1
  __device__ inline WalkN(const uint32_t* m, int W_, int own_)
      : masks(m), W(W_), own_list(own_), word(-1), left(0x7fffffff), u(0), own(0), own2(0) {}
  __device__ inline uint32_t any(int w) const {
    uint32_t all = masks[w];
#pragma unroll
    for (int k = 1; k < NL; ++k) all |= masks[k * W + w];
    return all;
  }
  __device__ inline void load() {
    u = __builtin_amdgcn_readfirstlane(any(word));
    own = __builtin_amdgcn_readfirstlane(masks[own_list * W + word]);
    if (NOWN == 2) own2 = __builtin_amdgcn_readfirstlane(masks[(own_list + 1) * W + word]);
  }
  // next tile of the union; mine: bit 0 = on the first own list, bit 1 = on the second
  __device__ inline int next(uint32_t& mine) {
    if (left <= 0) return -1;
    while (u == 0) {
      if (++word >= W) return -1;
      load();
    }
    const int b = __builtin_ctz(u);
    u &= u - 1;
    mine = ((own >> b) & 1u) | (NOWN == 2 ? ((own2 >> b) & 1u) << 1 : 0u);
    --left;
    return word * 32 + b;
  }
  __device__ inline int next(bool& mine) {
    uint32_t m = 0;
    const int r = next(m);
    mine = m != 0;
    return r;
  }
  // restrict a fresh walk to segment `seg` of `nseg` equal parts of the union
  __device__ inline void restrict_to(int seg, int nseg) {
    int total = 0;
    for (int w = 0; w < W; ++w) total += __builtin_popcount(__builtin_amdgcn_readfirstlane(any(w)));
    int skip = (int)((int64_t)seg * total / nseg);
    left = (int)((int64_t)(seg + 1) * total / nseg) - skip;
    while (++word < W) {
      load();
      const int c = __builtin_popcount(u);
      if (skip < c) break;
      skip -= c;
      u = 0;
    }
    for (; skip > 0; --skip) u &= u - 1;
  }
};

#define BSA_FENCE() __builtin_amdgcn_sched_barrier(0)
#define BSA_WAIT_VM(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")

// COMBINE = false: the walk (a whole unit, or one segment of a split unit, whose unnormalised
// accumulators, running maxima and sums go to a.part).  COMBINE = true: merge the segments of
// a split unit and finish it.  Both end in the same epilogue.
// PACK (n_keep <= 16): a wavefront carries two query blocks, 16 columns of its 32-column MFMA
// tile each, so a workgroup covers eight blocks; a tile that only one of the two lists holds
// is masked (-inf) in the other block's columns.
template <int D, bool SPLITQ, bool COMBINE, bool PACK>
__global__ __launch_bounds__(SPLITQ ? 512 : 256, 2) void fwd_pipe_kernel(Geom g, AttnArgs a) {
  static_assert(!(PACK && SPLITQ), "packing is for short retained sets");
  constexpr int PG = PACK ? 2 * bsa::PG : bsa::PG;  // query blocks per workgroup
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
  __shared__ float cen_lse[PG][PBK];  // per window
  __shared__ uint32_t keepbits[PG][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int sub = wave >> 2;                 // which 32 queries of the block (always 0 with four wavefronts)
  const int qb0 = PACK ? 2 * wave : (wave & 3);            // the wavefront's (first) query block within the workgroup
  const int qb = PACK ? qb0 + (col >> 4) : qb0;            // the lane's
  constexpr int NOWN = PACK ? 2 : 1;
  constexpr int NW = NT / 64;              // wavefronts
  constexpr int NREG = (D / 32) * 16 + 2;  // floats per lane of a partial result: O^T tile, m, l
  const int ngroups = (g.N + PG - 1) / PG;
  Item it;
  if (COMBINE) it = split_item_of(blockIdx.x, ngroups * g.B * g.H, a.split_S, a.split_n);
  else if (!item_of(blockIdx.x, ngroups * g.B * g.H, a.split_S, a.split_n, it)) return;
  const int unit = it.unit;
  const int64_t bh = unit / ngroups;
  const int i0 = (unit % ngroups) * PG + qb0;  // the wavefront's first query block
  const int i = (unit % ngroups) * PG + qb;    // the lane's query block
  const bool valid = i < g.N;
  const int64_t row = bh * g.N + i;
  const int W = (g.N + 31) / 32;
  const uint16_t* Qh = static_cast<const uint16_t*>(a.Q) + bh * g.L * D;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* Oh = static_cast<uint16_t*>(a.O_out) + bh * g.L * D;
  float* Lh = a.LSE_out + bh * g.L;

  if (tid < PBK) koff[tid] = intra_offset(g, tid);
  if (!COMBINE)
    for (int k = tid; k < PG * W; k += NT) masks[k] = 0u;
  if (tid < 2 * PG) keepbits[tid >> 1][tid & 1] = 0u;
  __syncthreads();
  if (!COMBINE && sub == 0) {
#pragma unroll
    for (int o2 = 0; o2 < NOWN; ++o2) {  // the wavefront's own list(s)
      const int ib = i0 + o2, ql = qb0 + o2;
      if (ib >= g.N) continue;
      if (g.dense) {
        for (int w = lane; w < W; w += 64)
          masks[ql * W + w] = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
      } else {
        const int64_t rw = bh * g.N + ib;
        const int beg = a.q2k_ptr[rw], cnt = a.q2k_ptr[rw + 1] - beg;
        for (int t = lane; t < cnt; t += 64) {
          const int j = a.q2k_idx[beg + t];
          if ((unsigned)j < (unsigned)g.N) atomicOr(&masks[ql * W + (j >> 5)], 1u << (j & 31));
        }
      }
    }
  }

  // DMA plan of this thread: LDS slot (tid + NT n) of a tile is position p of row r and
  // receives chunk p ^ swz<D>(r) of that row from global memory.
  uint32_t goff[NI];  // bytes, relative to the block origin
#pragma unroll
  for (int n = 0; n < NI; ++n) {
    const int slot = tid + NT * n, r = slot / CPR, c = (slot % CPR) ^ swz<D>(r);
    goff[n] = (uint32_t)(koff[r] * D + c * 8) * 2u;
  }
  const uint32_t lds_wave = uniform_lds(ring + wave * 1024);
  auto issue = [&](int jb, int b) {  // addresses: scalar base of the block + the lane's offset; nothing vector per instruction
    const int64_t origin = (int64_t)block_origin_fast(g, jb) * D;
    const uint64_t kbase = uniform64(Kh + origin), vbase = uniform64(Vh + origin);
    const uint32_t kdst = lds_wave + b * 2 * TILE;
#pragma unroll
    for (int n = 0; n < NI; ++n) dma16_raw(kbase, goff[n], kdst + n * (NT * 16));
#pragma unroll
    for (int n = 0; n < NI; ++n) dma16_raw(vbase, goff[n], kdst + TILE + n * (NT * 16));
  };

  // Q^T fragments (B operand): lane (col, grp) holds channels 16 s + 8 grp .. +7 of its query
  const int qpos = PACK ? (col & 15) : 32 * sub + col;
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
    if (!COMBINE && qid >= 0) v = *reinterpret_cast<const u32x4*>(Qh + (int64_t)qtok * D + 16 * s + 8 * grp);
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

  // partial results of split unit sidx: [segment][wavefront][NREG][64 lanes] floats
  float* part = it.sidx >= 0 ? a.part + ((int64_t)it.sidx * a.split_S * NW + wave) * (NREG * 64) + lane : nullptr;
  if (COMBINE) {
    // merge the segments in order: m = max m_s, (l, O~) = sum of (l_s, O~_s) 2^(m_s - m)
    for (int sg = 0; sg < it.nseg; ++sg) m = fmaxf(m, part[(int64_t)sg * NW * NREG * 64 + (NREG - 2) * 64]);
    for (int sg = 0; sg < it.nseg; ++sg) {
      const float* ps = part + (int64_t)sg * NW * NREG * 64;
      float v[NREG];  // the segment's values first, all loads in flight together
#pragma unroll
      for (int k = 0; k < NREG; ++k) v[k] = __builtin_nontemporal_load(ps + k * 64);
      const float ms = v[NREG - 2];
      const float w = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - m);
      l += w * v[NREG - 1];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] += w * v[dt * 16 + r];
    }
  }
  WalkN<PG, NOWN> walk(masks, W, qb0);  // runs NB-1 tiles ahead of the multiplication; `pending` remembers
  int issued = 0;                      // for the tiles in flight which of this wavefront's lists have them (2 bits a tile)
  uint32_t pending = 0;
  if (!COMBINE) {
    if (it.nseg > 1) walk.restrict_to(it.seg, it.nseg);
#pragma unroll
    for (int k = 0; k < NB - 1; ++k) {
      uint32_t mk = 0;
      const int jb = walk.next(mk);
      if (jb >= 0) {
        issue(jb, k);
        pending |= mk << (2 * k);
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
      uint32_t mn = 0;
      const int jn = walk.next(mn);
      if (jn >= 0) {
        issue(jn, (t + NB - 1) & (NB - 1));
        pending |= mn << (2 * (NB - 1));
        ++issued;
      }
    }
    const uint32_t mbits = pending & 3u;
    const bool mine = mbits != 0;
    pending >>= 2;
    if (mine) {
      // 64 keys x this wavefront's 32 queries.  The 4*DS A fragments of the tile (K rows for
      // both key halves, then V^T) are read from LDS through a ring of RING register
      // fragments, RING MFMAs ahead of their use.  Matrix, vector and LDS instructions of a
      // SIMD co-execute only in part on this chip (measured: the tile's mix keeps the matrix
      // core at most 62 % busy with two wavefronts that never wait), and the LDS -> MFMA chain is
      // the critical path of a tile, so the vector work per tile is kept minimal.
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
      if (PACK && mbits != 3u && !((mbits >> (col >> 4)) & 1u)) {  // the tile is not on this lane's block's list
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[kt][r] = -INFINITY;
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      mx = pair_max(mx);
      const float mtrue = fmaxf(m, mx * c2);  // c2 > 0: the maximum commutes with the scaling
      // (packed: a query whose block has seen no tile yet stays at -inf; the arithmetic below then uses 0)
      const float mnew = (PACK && mtrue == -INFINITY) ? 0.f : mtrue;
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
      m = mtrue;
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

  if (!COMBINE && it.nseg > 1) {  // a segment: leave the partial result, the combine launch finishes the unit
    float* ps = part + (int64_t)it.seg * NW * NREG * 64;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) ps[(dt * 16 + r) * 64] = o[dt][r];
    ps[(NREG - 2) * 64] = m;
    ps[(NREG - 1) * 64] = l;
    return;
  }
  // epilogue: normalise, store the retained rows, park the rows of the windows' critical tokens
  // (in the tile ring, idle now) for the fill
  uint16_t* cen_rows = reinterpret_cast<uint16_t*>(smem);  // [PG][nwin][D]
  const float ltot = pair_sum(l);
  const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
  const float lse = ltot > 0.f ? (m + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
  __syncthreads();  // every wavefront is done with the ring
  if (qid >= 0) {
    const int win = window_of(g, qid);
    const bool is_center = !g.dense && qid == window_center(g, win);
    uint16_t* park = cen_rows + ((size_t)qb * g.nwin + win) * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 v;
        v.x = pack_bf16(o[dt][4 * r4 + 0] * inv, o[dt][4 * r4 + 1] * inv);
        v.y = pack_bf16(o[dt][4 * r4 + 2] * inv, o[dt][4 * r4 + 3] * inv);
        const int ch = 32 * dt + 8 * r4 + 4 * grp;
        *reinterpret_cast<u32x2*>(Oh + (int64_t)qtok * D + ch) = v;
        if (is_center) *reinterpret_cast<u32x2*>(park + ch) = v;
      }
    if (grp == 0) {
      Lh[qtok] = lse;
      if (is_center) cen_lse[qb][win] = lse;
    }
  }
  __syncthreads();
  // token filling: lane c of the block's first wavefront owns intra-block token c and, if it
  // was pruned, copies the row of its window's critical token
  if (!g.dense && sub == 0) {
#pragma unroll
    for (int o2 = 0; o2 < NOWN; ++o2) {  // the wavefront's own block(s)
      const int ib = i0 + o2, ql = qb0 + o2;
      if (ib >= g.N) continue;
      const bool kept = (keepbits[ql][lane >> 5] >> (lane & 31)) & 1u;
      const int win = window_of(g, lane);
      const bool have = (keepbits[ql][window_center(g, win) >> 5] >> (window_center(g, win) & 31)) & 1u;
      if (!kept && have) {
        const int64_t tok = block_origin(g, ib) + koff[lane];
        const uint16_t* src = cen_rows + ((size_t)ql * g.nwin + win) * D;
#pragma unroll
        for (int q = 0; q < D / 8; ++q)
          *reinterpret_cast<u32x4*>(Oh + tok * D + 8 * q) = *reinterpret_cast<const u32x4*>(src + 8 * q);
        Lh[tok] = cen_lse[ql][win];
      }
    }
  }
}

// =====================================================================================
// Backward, same streaming scheme.  Three kernels, no floating-point atomics:
//   pre   per query block: retained Q rows and the folded upstream gradient g (dO of the
//         row; for the center row plus the dO of every pruned token, the gradient of the
//         fill copy) as bf16 tiles in the swizzled LDS format, delta = <g, O> and LSE in the
//         exp2 domain: one contiguous record per query block in the workspace.
//   dQ    the forward's walk (four query blocks per workgroup, union of their KV lists):
//         S^T = K Q^T, dP^T = V G^T, dS^T = P^T (dP^T - delta), dQ^T += K^T dS^T, one key half
//         at a time; K^T comes from the same K tile through transposed LDS reads.
//   dKV   a workgroup owns two adjacent KV blocks, whose K and V tiles stay in LDS, and walks
//         the union of their k2q lists; the query-block records stream through an LDS ring
//         by DMA.  A wavefront owns 32 keys: S = Qc K^T, dP = Gc V^T, dV^T += Gc^T P,
//         dK^T += Qc^T dS, accumulators in registers for the whole walk.
// =====================================================================================

template <int D, int NQT>
struct BwdRec {  // byte layout of one query block's record (workspace image == LDS image)
  static constexpr int NQ = 32 * NQT;
  static constexpr int RB = D * 2;
  static constexpr int QC = 0;                  // [NQ][D] bf16, swizzled rows
  static constexpr int GC = NQ * RB;            // [NQ][D] bf16, swizzled rows
  static constexpr int LS = 2 * NQ * RB;        // float lse2[NQ]
  static constexpr int DL = LS + NQ * 4;        // float delta[NQ]
  static constexpr int BYTES = DL + NQ * 4;     // multiple of 256
  static constexpr int CHUNKS = BYTES / 16;
};

template <int D, int NQT>
__global__ __launch_bounds__(256) void bwd_pre_pipe_kernel(Geom g, AttnArgs a) {
  using R = BwdRec<D, NQT>;
  constexpr int CPR = D / 8;       // 16-byte chunks per row
  constexpr int RPP = 256 / CPR;   // rows covered by one pass of the workgroup (a row = CPR adjacent lanes)
  extern __shared__ __align__(16) float fold_mem[];
  float* partial = fold_mem;                // [RPP][D] column sums of pruned dO rows, per row group
  float* foldw = fold_mem + RPP * D;        // [nwin][D] the same, complete, per window
  __shared__ int keepflag[PBK];
  __shared__ int qtok[R::NQ];
  __shared__ short qwin[R::NQ];   // window whose critical token the retained row is, or -1
  __shared__ int koff[PBK];
  __shared__ short wtok[PBK];     // tokens grouped by window, ascending id inside a window
  const int tid = threadIdx.x;
  const int c = tid % CPR, rg = tid / CPR;
  const int64_t row = blockIdx.x;
  const int64_t bh = row / g.N;
  const int i = row % g.N;
  const uint16_t* Qh = static_cast<const uint16_t*>(a.Q) + bh * g.L * D;
  const uint16_t* Oh = static_cast<const uint16_t*>(a.O) + bh * g.L * D;
  const uint16_t* dOh = static_cast<const uint16_t*>(a.dO) + bh * g.L * D;
  const float* Lh = a.LSE_in + bh * g.L;
  // a.pack (n_keep <= 16): two query blocks share a record, rows 0..15 the even block's, 16..31 the odd one's
  const int64_t recno = a.pack ? bh * ((g.N + 1) / 2) + (i >> 1) : row;
  const int r0 = a.pack ? 16 * (i & 1) : 0, nrows = a.pack ? 16 : R::NQ;
  uint8_t* rec = static_cast<uint8_t*>(a.ws) + recno * (int64_t)R::BYTES;
  const int origin = block_origin(g, i);

  if (tid < PBK) {
    koff[tid] = intra_offset(g, tid);
    keepflag[tid] = 0;
    if (!g.dense) {  // position of token tid inside its window: raster order of its local coordinates
      const int cw = tid % g.Cw, ch = (tid / g.Cw) % g.Ch, ct = tid / (g.Cw * g.Ch);
      const int k = ((ct % g.Wt) * g.Wh + ch % g.Wh) * g.Ww + cw % g.Ww;
      wtok[window_of(g, tid) * g.Wk + k] = (short)tid;
    }
  }
  __syncthreads();
  if (tid < R::NQ) {
    int k = -1;
    if (tid < a.n_keep) k = g.dense ? tid : min(max(a.keep_idx[row * a.n_keep + tid], 0), PBK - 1);
    qtok[tid] = k >= 0 ? origin + koff[k] : -1;
    qwin[tid] = (short)((k >= 0 && !g.dense && center_of(g, k) == k) ? window_of(g, k) : -1);
    if (k >= 0) keepflag[k] = 1;
  }
  __syncthreads();

  // Gradient of the fill copies: per window, the dO rows of its pruned tokens summed per
  // channel.  G row groups share a window: each adds every G-th token of the window in
  // ascending id, then the groups' sums are added in order.
  if (!g.dense) {
    const int G = g.nwin >= RPP ? 1 : RPP / g.nwin;  // row groups per window
    const int WB = g.nwin >= RPP ? RPP : g.nwin;     // windows per batch
    for (int w0 = 0; w0 < g.nwin; w0 += WB) {
      const int w = w0 + rg / G, sub = rg % G;
      float acc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
      if (rg < WB * G && w < g.nwin) {
        for (int k = sub; k < g.Wk; k += G) {
          const int u = wtok[w * g.Wk + k];
          if (keepflag[u]) continue;
          const u32x4 pv = *reinterpret_cast<const u32x4*>(dOh + (int64_t)(origin + koff[u]) * D + 8 * c);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] += __uint_as_float(pv[e] << 16);
            acc[2 * e + 1] += __uint_as_float(pv[e] & 0xffff0000u);
          }
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) partial[rg * D + 8 * c + e] = acc[e];
      __syncthreads();
      for (int t = tid; t < WB * D; t += 256) {
        const int wl = t / D, ch = t % D;
        if (w0 + wl < g.nwin) {
          float sum = 0.f;
          for (int k = 0; k < G; ++k) sum += partial[(wl * G + k) * D + ch];
          foldw[(w0 + wl) * D + ch] = sum;
        }
      }
      __syncthreads();
    }
  }

  // a last block without a partner also writes the partner's half of the record: padding rows
  const int nwrite = (a.pack && (i & 1) == 0 && i + 1 == g.N) ? 32 : nrows;
  for (int q = rg; q < nwrite; q += RPP) {
    const int tok = q < nrows ? qtok[q] : -1;
    u32x4 qv = {0u, 0u, 0u, 0u}, gv = {0u, 0u, 0u, 0u};
    float dsum = 0.f;
    if (tok >= 0) {
      qv = *reinterpret_cast<const u32x4*>(Qh + (int64_t)tok * D + 8 * c);
      gv = *reinterpret_cast<const u32x4*>(dOh + (int64_t)tok * D + 8 * c);
      const u32x4 ov = *reinterpret_cast<const u32x4*>(Oh + (int64_t)tok * D + 8 * c);
      float gf[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        gf[2 * e] = __uint_as_float(gv[e] << 16);
        gf[2 * e + 1] = __uint_as_float(gv[e] & 0xffff0000u);
      }
      const int w = qwin[q];
      if (w >= 0) {  // a window's critical token: its own dO plus its window's fill copies
#pragma unroll
        for (int e = 0; e < 8; ++e) gf[e] += foldw[w * D + 8 * c + e];
#pragma unroll
        for (int e = 0; e < 4; ++e) gv[e] = pack_bf16(gf[2 * e], gf[2 * e + 1]);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dsum += gf[2 * e] * __uint_as_float(ov[e] << 16);
        dsum += gf[2 * e + 1] * __uint_as_float(ov[e] & 0xffff0000u);
      }
    }
    const int rq = r0 + q;             // row of the record
    const int pos = c ^ swz<D>(rq);    // chunk position inside the swizzled row
    *reinterpret_cast<u32x4*>(rec + R::QC + rq * R::RB + pos * 16) = qv;
    *reinterpret_cast<u32x4*>(rec + R::GC + rq * R::RB + pos * 16) = gv;
#pragma unroll
    for (int msk = 1; msk < CPR; msk <<= 1) dsum += __shfl_xor(dsum, msk);  // the row's CPR lanes
    if (c == 0) {
      // padding rows, and rows whose list was empty (LSE = -inf): +inf, so that exp2(x - inf) = 0
      const float lse = tok >= 0 ? Lh[tok] : INFINITY;
      reinterpret_cast<float*>(rec + R::LS)[rq] = lse == -INFINITY ? INFINITY : lse * kLog2e;
      reinterpret_cast<float*>(rec + R::DL)[rq] = dsum;
    }
  }
}

// ------------------------------------------------------------------------------- dQ
// COMBINE as in the forward: segments of a split unit leave their dQ^T sums in a.part.
// PACK as in the forward: two query blocks per wavefront when n_keep <= 16.
template <int D, bool SPLITQ, bool COMBINE, bool PACK>
__global__ __launch_bounds__(SPLITQ ? 512 : 256, 2) void bwd_dq_pipe_kernel(Geom g, AttnArgs a) {
  static_assert(!(PACK && SPLITQ), "packing is for short retained sets");
  constexpr int PG = PACK ? 2 * bsa::PG : bsa::PG;  // query blocks per workgroup
  using R = BwdRec<D, SPLITQ ? 2 : 1>;
  constexpr int NT = SPLITQ ? 512 : 256;
  constexpr int NB = SPLITQ ? 4 : 2;
  constexpr int RB = D * 2, CPR = D / 8, TILE = PBK * RB, NI = PBK * CPR / NT;
  constexpr int DT = D / 32, DS = D / 16;
  extern __shared__ __align__(16) uint8_t smem[];
  uint8_t* ring = smem;                                                  // [NB][K tile | V tile]
  uint32_t* masks = reinterpret_cast<uint32_t*>(smem + NB * 2 * TILE);   // [PG][W]
  __shared__ int koff[PBK];
  __shared__ uint32_t keepbits[PG][2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int sub = wave >> 2;
  const int qb0 = PACK ? 2 * wave : (wave & 3);  // the wavefront's (first) query block within the workgroup
  const int qb = PACK ? qb0 + (col >> 4) : qb0;  // the lane's
  constexpr int NOWN = PACK ? 2 : 1;
  constexpr int NW = NT / 64;          // wavefronts
  constexpr int NREG = (D / 32) * 16;  // floats per lane of a partial result: the dQ^T tile
  const int ngroups = (g.N + PG - 1) / PG;
  Item it;
  if (COMBINE) it = split_item_of(blockIdx.x, ngroups * g.B * g.H, a.split_S, a.split_n);
  else if (!item_of(blockIdx.x, ngroups * g.B * g.H, a.split_S, a.split_n, it)) return;
  const int unit = it.unit;
  const int64_t bh = unit / ngroups;
  const int i0 = (unit % ngroups) * PG + qb0;
  const int i = (unit % ngroups) * PG + qb;
  const bool valid = i < g.N;
  const int64_t row = bh * g.N + i;
  const int W = (g.N + 31) / 32;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* dQh = static_cast<uint16_t*>(a.dQ) + bh * g.L * D;
  // packed: the wavefront's two blocks (i0 even) share one record, and the lane's row in it is its column
  const uint8_t* rec = static_cast<const uint8_t*>(a.ws) +
                       (PACK ? bh * ((g.N + 1) / 2) + (i0 >> 1) : row) * (int64_t)R::BYTES;

  if (tid < PBK) koff[tid] = intra_offset(g, tid);
  if (!COMBINE)
    for (int k = tid; k < PG * W; k += NT) masks[k] = 0u;
  if (tid < 2 * PG) keepbits[tid >> 1][tid & 1] = 0u;
  __syncthreads();
  if (!COMBINE && sub == 0) {
#pragma unroll
    for (int o2 = 0; o2 < NOWN; ++o2) {  // the wavefront's own list(s)
      const int ib = i0 + o2, ql = qb0 + o2;
      if (ib >= g.N) continue;
      if (g.dense) {
        for (int w = lane; w < W; w += 64)
          masks[ql * W + w] = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
      } else {
        const int64_t rw = bh * g.N + ib;
        const int beg = a.q2k_ptr[rw], cnt = a.q2k_ptr[rw + 1] - beg;
        for (int t = lane; t < cnt; t += 64) {
          const int j = a.q2k_idx[beg + t];
          if ((unsigned)j < (unsigned)g.N) atomicOr(&masks[ql * W + (j >> 5)], 1u << (j & 31));
        }
      }
    }
  }
  uint32_t goff[NI];  // bytes, relative to the block origin
#pragma unroll
  for (int n = 0; n < NI; ++n) {
    const int slot = tid + NT * n, r = slot / CPR, c = (slot % CPR) ^ swz<D>(r);
    goff[n] = (uint32_t)(koff[r] * D + c * 8) * 2u;
  }
  const uint32_t lds_wave = uniform_lds(ring + wave * 1024);
  auto issue = [&](int jb, int b) {  // addresses: scalar base of the block + the lane's offset; nothing vector per instruction
    const int64_t origin = (int64_t)block_origin_fast(g, jb) * D;
    const uint64_t kbase = uniform64(Kh + origin), vbase = uniform64(Vh + origin);
    const uint32_t kdst = lds_wave + b * 2 * TILE;
#pragma unroll
    for (int n = 0; n < NI; ++n) dma16_raw(kbase, goff[n], kdst + n * (NT * 16));
#pragma unroll
    for (int n = 0; n < NI; ++n) dma16_raw(vbase, goff[n], kdst + TILE + n * (NT * 16));
  };

  // Q^T and G^T fragments (B operands) and the row constants, from the query block's record
  const int qpos = PACK ? (col & 15) : 32 * sub + col;
  const int rrow = PACK ? col : qpos;  // row of the record
  int qid = -1, qtok = 0;
  float lse2 = INFINITY, delta = 0.f;
  if (valid && qpos < a.n_keep) {
    qid = g.dense ? qpos : min(max(a.keep_idx[row * a.n_keep + qpos], 0), PBK - 1);
    qtok = block_origin(g, i) + koff[qid];
    atomicOr(&keepbits[qb][qid >> 5], 1u << (qid & 31));
    lse2 = reinterpret_cast<const float*>(rec + R::LS)[rrow];
    delta = reinterpret_cast<const float*>(rec + R::DL)[rrow];
  }
  bf16x8 qf[DS], gf[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s) {
    u32x4 qv = {0u, 0u, 0u, 0u}, gv = {0u, 0u, 0u, 0u};
    if (!COMBINE && qid >= 0) {
      const int off = rrow * RB + (((2 * s + grp) ^ swz<D>(rrow)) << 4);
      qv = *reinterpret_cast<const u32x4*>(rec + R::QC + off);
      gv = *reinterpret_cast<const u32x4*>(rec + R::GC + off);
    }
    qf[s] = as_frag(qv);
    gf[s] = as_frag(gv);
  }
  settle(lse2);
  settle(delta);
#pragma unroll
  for (int s = 0; s < DS; ++s) {
    settle(qf[s]);
    settle(gf[s]);
  }

  int koffs[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s) koffs[s] = col * RB + (((2 * s + grp) ^ swz<D>(col)) << 4);
  const int L16 = lane & 15, q16 = lane >> 4, rsub = L16 >> 2, jj = L16 & 3;
  const int cl = 2 * (q16 & 1) + (jj >> 1), rhi = D == 128 ? rsub : (rsub >> 1);
  int voffs[2][DT];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      voffs[h][dt] = (8 * h + 4 * grp + rsub) * RB + ((((dt ^ rhi) << 2) | (cl ^ (2 * h + grp))) << 4) + 8 * (jj & 1);

  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;
  const float c2 = a.sm_scale * kLog2e;
  __syncthreads();

  // partial results of split unit sidx: [segment][wavefront][NREG][64 lanes] floats
  float* part = it.sidx >= 0 ? a.part + ((int64_t)it.sidx * a.split_S * NW + wave) * (NREG * 64) + lane : nullptr;
  if (COMBINE) {
    for (int sg = 0; sg < it.nseg; ++sg) {
      const float* ps = part + (int64_t)sg * NW * NREG * 64;
      float v[NREG];  // all loads of the segment in flight together
#pragma unroll
      for (int k = 0; k < NREG; ++k) v[k] = __builtin_nontemporal_load(ps + k * 64);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[dt][r] += v[dt * 16 + r];
    }
  }
  WalkN<PG, NOWN> walk(masks, W, qb0);
  int issued = 0;
  uint32_t pending = 0;  // two bits per tile in flight: which of the wavefront's lists hold it
  if (!COMBINE) {
    if (it.nseg > 1) walk.restrict_to(it.seg, it.nseg);
#pragma unroll
    for (int k = 0; k < NB - 1; ++k) {
      uint32_t mk = 0;
      const int jb = walk.next(mk);
      if (jb >= 0) {
        issue(jb, k);
        pending |= mk << (2 * k);
        ++issued;
      }
    }
  }
  for (int t = 0; t < issued; ++t) {
    const int ahead = issued - t - 1;
    if (NB >= 4 && ahead >= 2) {
      if (2 * NI == 4) BSA_WAIT_VM(8); else BSA_WAIT_VM(4);
    } else if (NB >= 3 && ahead == 1) {
      if (2 * NI == 4) BSA_WAIT_VM(4); else BSA_WAIT_VM(2);
    } else {
      BSA_WAIT_VM(0);
    }
    raw_barrier();
    {
      uint32_t mn = 0;
      const int jn = walk.next(mn);
      if (jn >= 0) {
        issue(jn, (t + NB - 1) & (NB - 1));
        pending |= mn << (2 * (NB - 1));
        ++issued;
      }
    }
    const uint32_t mbits = pending & 3u;
    const bool mine = mbits != 0;
    pending >>= 2;
    if (mine) {
      const uint8_t* Kb = ring + (t & (NB - 1)) * 2 * TILE;
      const uint8_t* Vb = Kb + TILE;
      // packed: a tile that is not on this lane's block's list contributes P = 0
      const float lse_t = (PACK && !((mbits >> (col >> 4)) & 1u)) ? INFINITY : lse2;
      // one key half (32 keys) at a time: 2*DS row fragments (K, V alternating), then 2*DT
      // transposed K fragments; a ring of RING register fragments runs ahead of the MFMAs
      constexpr int RING = 8, NF = 2 * DS + 2 * DT;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        auto frag = [&](int f) -> bf16x8 {
          if (f < 2 * DS) {
            const uint8_t* base = (f & 1) ? Vb : Kb;
            return lds_frag(reinterpret_cast<const uint16_t*>(base + 32 * kt * RB + koffs[f >> 1]));
          }
          const int v = f - 2 * DS, h = v / DT, dt = v % DT, ks = 2 * kt + h;
          return lds_frag_tr(Kb + voffs[0][dt] + 16 * ks * RB, Kb + voffs[1][dt] + 16 * ks * RB);
        };
        bf16x8 fr[RING];
#pragma unroll
        for (int f = 0; f < RING; ++f) fr[f] = frag(f);
        BSA_FENCE();
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
        for (int f = 0; f < 2 * DS; ++f) {
          if (f & 1) dp = mfma32(fr[f % RING], gf[f >> 1], dp);
          else s = mfma32(fr[f % RING], qf[f >> 1], s);
          if (f + RING < NF) fr[f % RING] = frag(f + RING);
          if (f & 1) BSA_FENCE();
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c2, -lse_t));
          s[r] = p * (dp[r] - delta);
        }
        const bf16x8 d0 = d_to_b(s, 0), d1 = d_to_b(s, 1);
        BSA_FENCE();
#pragma unroll
        for (int f = 2 * DS; f < NF; ++f) {
          const int v = f - 2 * DS;
          dq[v % DT] = mfma32(fr[f % RING], (v / DT) ? d1 : d0, dq[v % DT]);
          if (f + RING < NF) fr[f % RING] = frag(f + RING);
          if (f & 1) BSA_FENCE();
        }
      }
    }
  }

  if (!COMBINE && it.nseg > 1) {
    float* ps = part + (int64_t)it.seg * NW * NREG * 64;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) ps[(dt * 16 + r) * 64] = dq[dt][r];
    return;
  }
  if (qid >= 0) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 v;
        v.x = pack_bf16(dq[dt][4 * r4 + 0] * a.sm_scale, dq[dt][4 * r4 + 1] * a.sm_scale);
        v.y = pack_bf16(dq[dt][4 * r4 + 2] * a.sm_scale, dq[dt][4 * r4 + 3] * a.sm_scale);
        *reinterpret_cast<u32x2*>(dQh + (int64_t)qtok * D + 32 * dt + 8 * r4 + 4 * grp) = v;
      }
  }
  __syncthreads();
  // pruned queries take no part in the forward: zero gradient rows
  if (!g.dense && sub == 0) {
#pragma unroll
    for (int o2 = 0; o2 < NOWN; ++o2) {  // the wavefront's own block(s)
      const int ib = i0 + o2, ql = qb0 + o2;
      if (ib >= g.N) continue;
      const bool kept = (keepbits[ql][lane >> 5] >> (lane & 31)) & 1u;
      if (!kept) {
        const int64_t tok = block_origin(g, ib) + koff[lane];
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int q = 0; q < D / 8; ++q) *reinterpret_cast<u32x4*>(dQh + tok * D + 8 * q) = z;
      }
    }
  }
}

// ------------------------------------------------------------------------------ dK, dV
// Ascending walk over the union of the two KV blocks' k2q lists (bit masks in LDS), scalar
// state.  PACK: the bits are pairs of query blocks (one shared record), and each KV block has
// two masks: pairs whose even block lists it, pairs whose odd block does.
template <bool PACK>
struct Walk2 {
  const uint32_t* masks;  // [2][W], packed [2][2][W]
  int W, own_list, word, left;
  uint32_t u, own, own2;
  __device__ inline Walk2(const uint32_t* m, int W_, int own_)
      : masks(m), W(W_), own_list(own_), word(-1), left(0x7fffffff), u(0), own(0), own2(0) {}
  __device__ inline uint32_t any(int w) const {
    return PACK ? (masks[w] | masks[W + w] | masks[2 * W + w] | masks[3 * W + w]) : (masks[w] | masks[W + w]);
  }
  __device__ inline void load() {
    u = __builtin_amdgcn_readfirstlane(any(word));
    if (PACK) {
      own = __builtin_amdgcn_readfirstlane(masks[2 * own_list * W + word]);
      own2 = __builtin_amdgcn_readfirstlane(masks[(2 * own_list + 1) * W + word]);
    } else {
      own = __builtin_amdgcn_readfirstlane(masks[own_list * W + word]);
    }
  }
  // mine: bit 0 = on this KV block's list (packed: the pair's even block), bit 1 = the pair's odd block
  __device__ inline int next(uint32_t& mine) {
    if (left <= 0) return -1;
    while (u == 0) {
      if (++word >= W) return -1;
      load();
    }
    const int b = __builtin_ctz(u);
    u &= u - 1;
    mine = ((own >> b) & 1u) | (PACK ? ((own2 >> b) & 1u) << 1 : 0u);
    --left;
    return word * 32 + b;
  }
  // restrict a fresh walk to segment `seg` of `nseg` equal parts of the union
  __device__ inline void restrict_to(int seg, int nseg) {
    int total = 0;
    for (int w = 0; w < W; ++w) total += __builtin_popcount(__builtin_amdgcn_readfirstlane(any(w)));
    int skip = (int)((int64_t)seg * total / nseg);
    left = (int)((int64_t)(seg + 1) * total / nseg) - skip;
    while (++word < W) {
      load();
      const int c = __builtin_popcount(u);
      if (skip < c) break;
      skip -= c;
      u = 0;
    }
    for (; skip > 0; --skip) u &= u - 1;
  }
};

// wait until at most `n` DMA instructions of this wavefront are outstanding (n = per_tile * ahead)
#define BSA_WAIT_CASE(k) case k: BSA_WAIT_VM(k); break;
__device__ inline void wait_vm_upto(int n) {
  switch (n) {
    BSA_WAIT_CASE(0) BSA_WAIT_CASE(1) BSA_WAIT_CASE(2) BSA_WAIT_CASE(3) BSA_WAIT_CASE(4) BSA_WAIT_CASE(5) BSA_WAIT_CASE(6) BSA_WAIT_CASE(8) BSA_WAIT_CASE(9) BSA_WAIT_CASE(10)
    BSA_WAIT_CASE(12) BSA_WAIT_CASE(15) BSA_WAIT_CASE(16) BSA_WAIT_CASE(18) BSA_WAIT_CASE(20) BSA_WAIT_CASE(24)
    BSA_WAIT_CASE(25) BSA_WAIT_CASE(27) BSA_WAIT_CASE(30) BSA_WAIT_CASE(36) BSA_WAIT_CASE(45) BSA_WAIT_CASE(54)
    default: BSA_WAIT_VM(0); break;
  }
}

template <int NQT>
struct DkvRing {  // record ring of the dK/dV kernel
  static constexpr int NB = NQT == 1 ? 5 : 2;   // depth
  static constexpr int PER = NQT == 1 ? 2 : 1;  // records consumed per step
};

template <int D, int NQT, bool PACK>
__global__ __launch_bounds__(512, 1) void bwd_dkv_pipe_kernel(Geom g, AttnArgs a) {
  static_assert(!PACK || NQT == 1, "packed records hold two blocks of at most 16 retained queries");
  using R = BwdRec<D, NQT>;
  constexpr int NT = 512;
  constexpr int RB = D * 2, CPR = D / 8, TILE = PBK * RB, DT = D / 32, DS = D / 16;
  constexpr int NB = DkvRing<NQT>::NB;                 // ring depth (records)
  constexpr int PER = DkvRing<NQT>::PER;               // records consumed per step
  constexpr int NFULL = R::CHUNKS / NT;                // DMA instructions every wavefront issues per record
  constexpr int NTAIL = R::CHUNKS % NT;                // chunks of the last, partial instruction (wavefront 0 only)
  constexpr int NI = PBK * CPR / NT;                   // DMA instructions per thread per stationary K (or V) tile
  static_assert(NTAIL <= 64, "record tail must fit one wavefront");
  static_assert(NB * R::BYTES >= 4 * DT * 16 * 256, "the ring doubles as the reduction buffer");
  extern __shared__ __align__(16) uint8_t smem[];
  uint8_t* kvst = smem;                                                    // [2 KV blocks][K tile | V tile], stationary
  uint8_t* ring = smem + 4 * TILE;                                         // [NB][record]
  uint32_t* masks = reinterpret_cast<uint32_t*>(ring + NB * R::BYTES);     // [2][W]
  __shared__ int koff[PBK];

  // Eight wavefronts: (KV block, key half) x parity.  The two wavefronts of one (block, half)
  // share a SIMD and take alternate records (n_keep <= 32) or the two query sub-tiles of each
  // record (n_keep > 32), each with private accumulators that are summed at the end; while
  // one waits for LDS or runs its softmax arithmetic the other keeps the matrix core busy.
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int par = wave >> 2, which = (wave >> 1) & 1, half = wave & 1;
  const int npairs = (g.N + 1) / 2;
  Item it;
  if (!item_of(blockIdx.x, npairs * g.B * g.H, a.kv_split_S, a.kv_split_n, it)) return;
  const int unit = it.unit;
  const int64_t bh = unit / npairs;
  const int j0 = (unit % npairs) * 2;
  const int j = j0 + which;  // this wavefront's KV block; it owns keys 32*half .. +31
  const bool valid = j < g.N;
  const int64_t colrow = bh * g.N + j;
  const int nrec = PACK ? (g.N + 1) / 2 : g.N;  // records of a head (packed: one per pair of query blocks)
  const int W = (nrec + 31) / 32;
  const uint16_t* Kh = static_cast<const uint16_t*>(a.K) + bh * g.L * D;
  const uint16_t* Vh = static_cast<const uint16_t*>(a.V) + bh * g.L * D;
  uint16_t* dKh = static_cast<uint16_t*>(a.dK) + bh * g.L * D;
  uint16_t* dVh = static_cast<uint16_t*>(a.dV) + bh * g.L * D;
  const uint8_t* ws = static_cast<const uint8_t*>(a.ws) + bh * nrec * (int64_t)R::BYTES;

  if (tid < PBK) koff[tid] = intra_offset(g, tid);
  for (int k = tid; k < (PACK ? 4 : 2) * W; k += NT) masks[k] = 0u;
  __syncthreads();
  if (valid && half == 0 && par == 0) {
    if (g.dense) {
      for (int w = lane; w < W; w += 64)
        masks[which * W + w] = (w * 32 + 32 <= g.N) ? 0xffffffffu : ((1u << (g.N - w * 32)) - 1u);
    } else {
      const int beg = a.k2q_ptr[colrow], cnt = a.k2q_ptr[colrow + 1] - beg;
      for (int t = lane; t < cnt; t += 64) {
        const int ib = a.k2q_idx[beg + t];
        if ((unsigned)ib >= (unsigned)g.N) continue;
        if (PACK) atomicOr(&masks[(2 * which + (ib & 1)) * W + (ib >> 6)], 1u << ((ib >> 1) & 31));
        else atomicOr(&masks[which * W + (ib >> 5)], 1u << (ib & 31));
      }
    }
  }
  // The K and V tiles of the workgroup's two KV blocks stay in LDS for the whole walk (their
  // fragments are the B operands of S and dP); keeping them in registers instead pushes the
  // kernel past 256 VGPRs and the compiler then shuttles accumulators between register files.
  for (int blk = 0; blk < 2; ++blk) {
    const int jb = min(j0 + blk, g.N - 1);
    const int64_t origin = (int64_t)block_origin(g, jb) * D;
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const int slot = tid + NT * n, r = slot / CPR, c = (slot % CPR) ^ swz<D>(r);
      const int off = koff[r] * D + c * 8;
      dma16(Kh + origin + off, kvst + blk * 2 * TILE + wave * 1024 + n * (NT * 16));
      dma16(Vh + origin + off, kvst + blk * 2 * TILE + TILE + wave * 1024 + n * (NT * 16));
    }
  }
  const int64_t ktok = valid ? block_origin(g, j) + koff[32 * half + col] : 0;
  int koffs[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s) koffs[s] = col * RB + (((2 * s + grp) ^ swz<D>(col)) << 4);
  const int L16 = lane & 15, q16 = lane >> 4, rsub = L16 >> 2, jj = L16 & 3;
  const int cl = 2 * (q16 & 1) + (jj >> 1), rhi = D == 128 ? rsub : (rsub >> 1);
  int voffs[2][DT];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      voffs[h][dt] = (8 * h + 4 * grp + rsub) * RB + ((((dt ^ rhi) << 2) | (cl ^ (2 * h + grp))) << 4) + 8 * (jj & 1);

  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[dt][r] = dv[dt][r] = 0.f;
  const float c2 = a.sm_scale * kLog2e;
  const int per_tile = NFULL + (wave == 0 && NTAIL ? 1 : 0);  // DMA instructions of this wavefront per record
  const uint8_t* Kst = kvst + which * 2 * TILE + 32 * half * RB;  // this wavefront's 32 K rows; V rows at + TILE
  const int qt = NQT == 1 ? 0 : par;                              // query sub-tile of a record this wavefront takes
  BSA_WAIT_VM(0);
  __syncthreads();

  auto issue = [&](int ib, int b) {
    const uint8_t* src = ws + ib * (int64_t)R::BYTES + tid * 16;
    uint8_t* dst = ring + b * R::BYTES + wave * 1024;
#pragma unroll
    for (int n = 0; n < NFULL; ++n) dma16(src + n * (NT * 16), dst + n * (NT * 16));
    if (NTAIL && wave == 0 && lane < NTAIL) dma16(src + NFULL * (NT * 16), dst + NFULL * (NT * 16));
  };
  auto modnb = [](int x) { return x >= NB ? x - NB : x; };
  const uint32_t lds_wave = uniform_lds(ring + wave * 1024), tid16 = tid * 16u;
  Walk2<PACK> walk(masks, W, which);
  if (it.nseg > 1) walk.restrict_to(it.seg, it.nseg);
  int issued = 0;        // records requested so far (positions of the union walk)
  uint32_t pending = 0;  // bits 2k, 2k+1: how position PER*s + k is on this wavefront's list (see Walk2::next)
#pragma unroll
  for (int k = 0; k < NB - PER; ++k) {
    uint32_t mk = 0;
    const int ib = walk.next(mk);
    if (ib >= 0) {
      issue(ib, k);
      pending |= mk << (2 * k);
      ++issued;
    }
  }
  int sc = 0;  // ring slot of position PER*s
  for (int s = 0; PER * s < issued; ++s) {
    // the records of this step have landed once at most the later requests are outstanding
    wait_vm_upto(per_tile * max(0, issued - PER * (s + 1)));
    raw_barrier();  // ... for every wavefront; and every wavefront is done with the previous step's slots
    // The requests of this step (the slots freed by the barrier) are not issued here in one
    // burst: right after a barrier all eight wavefronts would queue at the CU's one vector
    // memory port (about 16 cycles per 1 KB instruction).  A wavefront with a tile to multiply
    // spreads them over its first contraction; the others issue them at once.
    constexpr int NDMA = PER * (NFULL + 1);  // instruction slots per step: per record NFULL full ones and the tail
    int dib[PER];  // query block requested for slot sc + NB - PER + k, or -1 (wave-uniform)
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      uint32_t mk = 0;
      dib[k] = walk.next(mk);
      if (dib[k] >= 0) {
        pending |= mk << (2 * (NB - PER + k));
        ++issued;
      }
    }
    auto emit = [&](int q) {  // the q-th instruction slot; every wavefront keeps the same order
      const int k = q / (NFULL + 1), n = q % (NFULL + 1);
      if (dib[k] < 0) return;
      const uint64_t src = uniform64(ws + dib[k] * (int64_t)R::BYTES + n * (NT * 16));  // scalar; the lane adds tid * 16
      const uint32_t dst = lds_wave + modnb(sc + NB - PER + k) * R::BYTES + n * (NT * 16);
      if (n < NFULL) dma16_raw(src, tid16, dst);
      else if (NTAIL && wave == 0 && lane < NTAIL) dma16_raw(src, tid16, dst);
    };
    const int kpos = NQT == 1 ? par : 0;
    const uint32_t mbits = (pending >> (2 * kpos)) & 3u;
    const bool mine = mbits != 0;
    pending >>= 2 * PER;
    constexpr bool SPREAD = NQT == 1;  // (with two query sub-tiles the spread costs registers the kernel does not have)
    if (!SPREAD || !mine) {
#pragma unroll
      for (int q = 0; q < NDMA; ++q) emit(q);
    }
    if (mine) {
      const uint8_t* rb = ring + modnb(sc + kpos) * R::BYTES;
      const uint8_t* Qc = rb + R::QC;
      const uint8_t* Gc = rb + R::GC;
      const float* ls = reinterpret_cast<const float*>(rb + R::LS);
      const float* dl = reinterpret_cast<const float*>(rb + R::DL);
      // fragments in use order: per k-step (Qc row, K row, Gc row, V row), then per
      // (16-query step, channel tile) (Gc^T, Qc^T); a ring of RING fragments runs ahead
      constexpr int RING = 8, NF = 4 * DS + 4 * DT;
      auto frag = [&](int f) -> bf16x8 {
        if (f < 4 * DS) {
          const int sp = f >> 2, kind = f & 3;
          const uint8_t* base = kind == 0 ? Qc + 32 * qt * RB : kind == 1 ? Kst : kind == 2 ? Gc + 32 * qt * RB : Kst + TILE;
          return lds_frag(reinterpret_cast<const uint16_t*>(base + koffs[sp]));
        }
        const int v = f - 4 * DS, dt = (v >> 1) % DT, h = (v >> 1) / DT;
        const uint8_t* base = ((v & 1) ? Qc : Gc) + 16 * (2 * qt + h) * RB;
        return lds_frag_tr(base + voffs[0][dt], base + voffs[1][dt]);
      };
      bf16x8 fr[RING];
#pragma unroll
      for (int f = 0; f < RING; ++f) fr[f] = frag(f);
      BSA_FENCE();
      f32x16 sacc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = dp[r] = 0.f;
      static_assert(!SPREAD || NDMA <= DS, "one DMA slot per k-step of the first contraction");
#pragma unroll
      for (int f = 0; f < 4 * DS; f += 2) {
        if (f & 2) dp = mfma32(fr[f % RING], fr[(f + 1) % RING], dp);
        else sacc = mfma32(fr[f % RING], fr[(f + 1) % RING], sacc);
        if (f + RING < NF) fr[f % RING] = frag(f + RING);
        if (f + 1 + RING < NF) fr[(f + 1) % RING] = frag(f + 1 + RING);
        if (f & 2) {
          if (SPREAD && (f >> 2) < NDMA) emit(f >> 2);
          BSA_FENCE();
        }
      }
      // D layout: lane = key column, register r = query row 32*qt + 8*(r/4) + 4*grp + r%4
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 l4 = *reinterpret_cast<const f32x4*>(ls + 32 * qt + 8 * r4 + 4 * grp);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dl + 32 * qt + 8 * r4 + 4 * grp);
        if (PACK && !((mbits >> (r4 >> 1)) & 1u)) {  // rows 0..15 / 16..31: a block of the pair that does not list this KV block
#pragma unroll
          for (int e = 0; e < 4; ++e) l4[e] = INFINITY;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[4 * r4 + e], c2, -l4[e]));
          sacc[4 * r4 + e] = pv;
          dp[4 * r4 + e] = pv * (dp[4 * r4 + e] - d4[e]);
        }
      }
      const bf16x8 pf0 = d_to_b(sacc, 0), pf1 = d_to_b(sacc, 1), df0 = d_to_b(dp, 0), df1 = d_to_b(dp, 1);
      BSA_FENCE();
#pragma unroll
      for (int f = 4 * DS; f < NF; ++f) {
        const int v = f - 4 * DS, dt = (v >> 1) % DT, h = (v >> 1) / DT;
        if (v & 1) dk[dt] = mfma32(fr[f % RING], h ? df1 : df0, dk[dt]);
        else dv[dt] = mfma32(fr[f % RING], h ? pf1 : pf0, dv[dt]);
        if (f + RING < NF) fr[f % RING] = frag(f + RING);
        if (f & 1) BSA_FENCE();
      }
    }
    sc = modnb(sc + PER);
  }
  // sum the two parities' accumulators (fixed order), dK then dV, through the idle ring
  BSA_WAIT_VM(0);
  f32x4* red = reinterpret_cast<f32x4*>(ring) + (wave & 3) * (DT * 4 * 64) + lane;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    __syncthreads();
    if (par == 1) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x16& acc = pass ? dv[dt] : dk[dt];
          f32x4 v = {acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]};
          red[(dt * 4 + r4) * 64] = v;
        }
    }
    __syncthreads();
    if (par == 0) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 v = red[(dt * 4 + r4) * 64];
          f32x16& acc = pass ? dv[dt] : dk[dt];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[4 * r4 + e] += v[e];
        }
    }
  }
  if (it.sidx >= 0) {  // a segment of a split unit: leave the raw sums for the combine launch
    if (par == 0) {
      f32x4* part = reinterpret_cast<f32x4*>(a.kv_part) +
                    (((int64_t)it.sidx * a.kv_split_S + it.seg) * 4 + (wave & 3)) * (2 * DT * 4 * 64) + lane;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 kq = {dk[dt][4 * r4], dk[dt][4 * r4 + 1], dk[dt][4 * r4 + 2], dk[dt][4 * r4 + 3]};
          f32x4 vq = {dv[dt][4 * r4], dv[dt][4 * r4 + 1], dv[dt][4 * r4 + 2], dv[dt][4 * r4 + 3]};
          __builtin_nontemporal_store(kq, part + (dt * 4 + r4) * 64);
          __builtin_nontemporal_store(vq, part + (DT * 4 + dt * 4 + r4) * 64);
        }
    }
    return;
  }
  if (valid && par == 0) {
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

// Finishes the split units of the dK/dV launch: sums the segments' partial results in segment
// order and stores dK, dV.  Four wavefronts = (KV block of the pair, key half), laid out as the
// main kernel's parity-0 wavefronts.
template <int D>
__global__ __launch_bounds__(256) void bwd_dkv_combine_kernel(Geom g, AttnArgs a) {
  constexpr int DT = D / 32, NV = 2 * DT * 4;  // float4 values per lane: dK then dV
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane >> 5, col = lane & 31;
  const int which = wave >> 1, half = wave & 1;
  const int npairs = (g.N + 1) / 2;
  const Item it = split_item_of(blockIdx.x, npairs * g.B * g.H, a.kv_split_S, a.kv_split_n);
  const int64_t bh = it.unit / npairs;
  const int j = (it.unit % npairs) * 2 + which;
  if (j >= g.N) return;
  const f32x4* part = reinterpret_cast<const f32x4*>(a.kv_part) + ((int64_t)it.sidx * a.kv_split_S * 4 + wave) * (NV * 64) + lane;
  f32x4 acc[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) acc[v] = __builtin_nontemporal_load(part + v * 64);
  for (int sgm = 1; sgm < a.kv_split_S; ++sgm) {
    const f32x4* ps = part + (int64_t)sgm * 4 * (NV * 64);
    f32x4 t[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) t[v] = __builtin_nontemporal_load(ps + v * 64);
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[v][e] += t[v][e];
  }
  const int64_t ktok = block_origin(g, j) + intra_offset(g, 32 * half + col);
  uint16_t* dKh = static_cast<uint16_t*>(a.dK) + bh * g.L * D;
  uint16_t* dVh = static_cast<uint16_t*>(a.dV) + bh * g.L * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const f32x4 kq = acc[dt * 4 + r4], vq = acc[DT * 4 + dt * 4 + r4];
      u32x2 kv, vv;
      kv.x = pack_bf16(kq[0] * a.sm_scale, kq[1] * a.sm_scale);
      kv.y = pack_bf16(kq[2] * a.sm_scale, kq[3] * a.sm_scale);
      vv.x = pack_bf16(vq[0], vq[1]);
      vv.y = pack_bf16(vq[2], vq[3]);
      const int ch = 32 * dt + 8 * r4 + 4 * grp;
      *reinterpret_cast<u32x2*>(dKh + ktok * D + ch) = kv;
      *reinterpret_cast<u32x2*>(dVh + ktok * D + ch) = vv;
    }
}

// floats per lane of one wavefront's partial result
constexpr int fwd_part_regs(int d) { return (d / 32) * 16 + 2; }
constexpr int dq_part_regs(int d) { return (d / 32) * 16; }

// pack: the forward's packed variant (two query blocks per wavefront, eight per workgroup)
static bool fwd_packs(const Geom& g, int n_keep) { return n_keep <= 16 && !g.dense; }
static SplitPlan fwd_plan(const Geom& g, int n_keep, bool allow, bool pack = false) {
  const bool splitq = n_keep > 32;
  const int pg = pack ? 2 * PG : PG;
  return plan_split(((g.N + pg - 1) / pg) * g.B * g.H, kCUs * (splitq ? 1 : 2), allow);
}

// dK/dV: one workgroup per CU and many rounds, so only the units of the last, partly filled
// round of every XCD (and a few more, against the spread of the unit lengths) are split.
static SplitPlan dkv_plan(const Geom& g) {
  const int units = ((g.N + 1) / 2) * g.B * g.H, q = units / 8, r = units % 8, per_xcd = kCUs / 8;
  SplitPlan p{1, 0, 0, 0};
  if (!g.dense && q >= 4 && q < 64 * per_xcd) {
    p.S = 4;
    p.n = min(q % per_xcd + per_xcd / 4, q / 2);
  }
  p.grid = 8 * (q + (r ? 1 : 0) - p.n + p.S * p.n);
  p.units = 8 * p.n;
  return p;
}
constexpr size_t dkv_part_bytes(int d) { return (size_t)4 * 2 * (d / 32) * 16 * 64 * sizeof(float); }  // per segment

template <int D, int NQT, bool PACK>
static int launch_bwd_pipe_t(const Geom& g, AttnArgs a, hipStream_t st) {
  using R = BwdRec<D, NQT>;
  constexpr bool SPLITQ = NQT == 2;
  constexpr int PGK = PACK ? 2 * PG : PG;
  const int W = (g.N + 31) / 32;
  a.pack = PACK ? 1 : 0;
  const size_t lds_q = (size_t)(SPLITQ ? 4 : 2) * 2 * PBK * D * 2 + (size_t)PGK * W * 4;
  const int nrec_head = PACK ? (g.N + 1) / 2 : g.N;
  const size_t nrec = (size_t)g.B * g.H * nrec_head;  // records in the workspace
  const size_t lds_kv = (size_t)4 * PBK * D * 2 + (size_t)DkvRing<NQT>::NB * R::BYTES +
                        (size_t)(PACK ? 4 : 2) * ((nrec_head + 31) / 32) * 4;
  if (int rc = allow_dynamic_lds<bwd_dq_pipe_kernel<D, SPLITQ, false, PACK>>(lds_q)) return rc;
  if (int rc = allow_dynamic_lds<bwd_dkv_pipe_kernel<D, NQT, PACK>>(lds_kv)) return rc;
  if (a.stages & BSA_BWD_PRE)  // LDS: per-row-group partial sums + per-window sums of the fill gradient
    hipLaunchKernelGGL((bwd_pre_pipe_kernel<D, NQT>), dim3(g.rows), dim3(256), (size_t)(256 / (D / 8) + g.nwin) * D * 4, st, g, a);
  if (a.stages & BSA_BWD_DQ) {
    const SplitPlan p = fwd_plan(g, a.n_keep, !g.dense, PACK);  // the dQ walk is the forward's walk
    a.split_S = p.S;
    a.split_n = p.n;
    a.part = reinterpret_cast<float*>(static_cast<uint8_t*>(a.ws) + (size_t)R::BYTES * nrec);  // behind the records
    hipLaunchKernelGGL((bwd_dq_pipe_kernel<D, SPLITQ, false, PACK>), dim3(p.grid), dim3(SPLITQ ? 512 : 256), lds_q, st, g, a);
    if (p.units)
      hipLaunchKernelGGL((bwd_dq_pipe_kernel<D, SPLITQ, true, PACK>), dim3(p.units), dim3(SPLITQ ? 512 : 256), 0, st, g, a);
  }
  if (a.stages & BSA_BWD_DKV) {
    const SplitPlan p = dkv_plan(g);
    const SplitPlan pq = fwd_plan(g, a.n_keep, !g.dense, PACK);
    a.kv_split_S = p.S;
    a.kv_split_n = p.n;
    a.kv_part = reinterpret_cast<float*>(static_cast<uint8_t*>(a.ws) + (size_t)R::BYTES * nrec +
                                         (size_t)pq.units * pq.S * (SPLITQ ? 8 : 4) * dq_part_regs(D) * 64 * sizeof(float));
    hipLaunchKernelGGL((bwd_dkv_pipe_kernel<D, NQT, PACK>), dim3(p.grid), dim3(512), lds_kv, st, g, a);
    if (p.units) hipLaunchKernelGGL((bwd_dkv_combine_kernel<D>), dim3(p.units), dim3(256), 0, st, g, a);
  }
  return check_launch();
}

int launch_bwd_pipe(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const bool two = a.n_keep > 32;
  if (fwd_packs(g, a.n_keep)) return g.d == 128 ? launch_bwd_pipe_t<128, 1, true>(g, a, st) : launch_bwd_pipe_t<64, 1, true>(g, a, st);
  if (g.d == 128) return two ? launch_bwd_pipe_t<128, 2, false>(g, a, st) : launch_bwd_pipe_t<128, 1, false>(g, a, st);
  return two ? launch_bwd_pipe_t<64, 2, false>(g, a, st) : launch_bwd_pipe_t<64, 1, false>(g, a, st);
}

size_t bwd_workspace_pipe(const Geom& g, int n_keep) {
  const bool two = n_keep > 32;
  const size_t per_row = g.d == 128 ? (two ? BwdRec<128, 2>::BYTES : BwdRec<128, 1>::BYTES)
                                    : (two ? BwdRec<64, 2>::BYTES : BwdRec<64, 1>::BYTES);
  const SplitPlan p = fwd_plan(g, n_keep, !g.dense, fwd_packs(g, n_keep));
  const size_t partials = (size_t)p.units * p.S * (two ? 8 : 4) * dq_part_regs(g.d) * 64 * sizeof(float);
  const SplitPlan pk = dkv_plan(g);
  const size_t nrec = fwd_packs(g, n_keep) ? (size_t)g.B * g.H * ((g.N + 1) / 2) : (size_t)g.rows;
  return per_row * nrec + partials + (size_t)pk.units * pk.S * dkv_part_bytes(g.d);  // records | dQ partials | dK/dV partials
}

size_t fwd_workspace_pipe(const Geom& g, int n_keep) {
  if (g.dense) return 0;
  const SplitPlan p = fwd_plan(g, n_keep, true, fwd_packs(g, n_keep));
  return (size_t)p.units * p.S * (n_keep > 32 ? 8 : 4) * fwd_part_regs(g.d) * 64 * sizeof(float);
}

template <int D, bool SPLITQ, bool PACK>
static int launch_fwd_pipe_t(const Geom& g, AttnArgs a, hipStream_t st) {
  constexpr int PGK = PACK ? 2 * PG : PG;
  const int W = (g.N + 31) / 32;
  const size_t lds = (size_t)(SPLITQ ? 4 : 2) * 2 * PBK * D * 2 + (size_t)PGK * W * 4;
  if (int rc = allow_dynamic_lds<fwd_pipe_kernel<D, SPLITQ, false, PACK>>(lds)) return rc;
  if (int rc = allow_dynamic_lds<fwd_pipe_kernel<D, SPLITQ, true, PACK>>((size_t)PGK * g.nwin * D * 2)) return rc;
  const SplitPlan p = fwd_plan(g, a.n_keep, !g.dense && a.fwd_ws != nullptr, PACK);
  a.split_S = p.S;
  a.split_n = p.n;
  a.part = static_cast<float*>(a.fwd_ws);
  hipLaunchKernelGGL((fwd_pipe_kernel<D, SPLITQ, false, PACK>), dim3(p.grid), dim3(SPLITQ ? 512 : 256), lds, st, g, a);
  if (p.units)  // the combine launch needs LDS only for the parked critical-token rows
    hipLaunchKernelGGL((fwd_pipe_kernel<D, SPLITQ, true, PACK>), dim3(p.units), dim3(SPLITQ ? 512 : 256),
                       (size_t)PGK * g.nwin * D * 2, st, g, a);
  return check_launch();
}

int launch_fwd_pipe(const Geom& g, const AttnArgs& a, hipStream_t st) {
  const bool splitq = a.n_keep > 32;
  if (fwd_packs(g, a.n_keep)) return g.d == 128 ? launch_fwd_pipe_t<128, false, true>(g, a, st) : launch_fwd_pipe_t<64, false, true>(g, a, st);
  if (g.d == 128) return splitq ? launch_fwd_pipe_t<128, true, false>(g, a, st) : launch_fwd_pipe_t<128, false, false>(g, a, st);
  return splitq ? launch_fwd_pipe_t<64, true, false>(g, a, st) : launch_fwd_pipe_t<64, false, false>(g, a, st);
}

}  // namespace bsa
