// C-ABI entry points of libbsa: host-side argument validation and dispatch only.
// Every check happens before any launch, so a failed call enqueues nothing.
#include <cmath>

#include "bsa_common.h"

namespace bsa {

int make_geom(const bsa_shape_t* s, Geom* g) {
  if (!s) return BSA_ERR_NULL;
  if (s->dtype != BSA_F32 && s->dtype != BSA_BF16) return BSA_ERR_DTYPE;
  if (s->B <= 0 || s->H <= 0 || s->T <= 0 || s->Hs <= 0 || s->Ws <= 0 || s->Ct <= 0 ||
      s->Ch <= 0 || s->Cw <= 0 || s->d <= 0)
    return BSA_ERR_SHAPE;
  // the paper assumes T/Ct, H/Ch, W/Cw are integers (Sec. 3.2.1)
  if (s->T % s->Ct || s->Hs % s->Ch || s->Ws % s->Cw) return BSA_ERR_SHAPE;
  if (s->d % 8 || s->d > 256) return BSA_ERR_SHAPE;
  const int64_t Bk = (int64_t)s->Ct * s->Ch * s->Cw;
  const int64_t L = (int64_t)s->T * s->Hs * s->Ws;
  if (Bk > 256) return BSA_ERR_SHAPE;
  const int64_t N = L / Bk;
  if (N > 8192) return BSA_ERR_SHAPE;
  const int64_t rows = (int64_t)s->B * s->H * N;
  if (rows * N > 0x7fffffffLL) return BSA_ERR_SHAPE;             // CSR offsets are int32
  if ((int64_t)s->B * s->H * L * s->d > 0x3fffffffffLL) return BSA_ERR_SHAPE;
  g->B = s->B; g->H = s->H; g->T = s->T; g->Hs = s->Hs; g->Ws = s->Ws;
  g->Ct = s->Ct; g->Ch = s->Ch; g->Cw = s->Cw; g->d = s->d;
  g->Nt = s->T / s->Ct; g->Nh = s->Hs / s->Ch; g->Nw = s->Ws / s->Cw;
  g->Bk = (int)Bk; g->N = (int)N; g->L = (int)L; g->rows = (int)rows;
  // windows of the critical-token mechanism must divide the block evenly (Sec. 3.2.2); 0 = the block
  if (s->Wt < 0 || s->Wh < 0 || s->Ww < 0) return BSA_ERR_SHAPE;
  g->Wt = s->Wt ? s->Wt : s->Ct; g->Wh = s->Wh ? s->Wh : s->Ch; g->Ww = s->Ww ? s->Ww : s->Cw;
  if (s->Ct % g->Wt || s->Ch % g->Wh || s->Cw % g->Ww) return BSA_ERR_SHAPE;
  g->Wk = g->Wt * g->Wh * g->Ww;
  g->nwin = g->Bk / g->Wk;
  if (s->layout != BSA_LAYOUT_RASTER && s->layout != BSA_LAYOUT_BLOCK_MAJOR) return BSA_ERR_SHAPE;
  g->tiled = s->layout == BSA_LAYOUT_BLOCK_MAJOR;
  g->dense = 0;
  g->inv_Nw = g->Nw == 1 ? 0u : (uint32_t)(0x100000000ull / (uint32_t)g->Nw) + 1u;
  g->inv_NwNh = g->Nw * g->Nh == 1 ? 0u : (uint32_t)(0x100000000ull / (uint32_t)(g->Nw * g->Nh)) + 1u;
  return BSA_OK;
}

// retained tokens per window, ceil(r * Wk); per block it is nwin times that
static int window_quota(const Geom& g, double r) {
  if (!(r > 0.0) || !(r <= 1.0)) return BSA_ERR_RANGE;
  int n = (int)std::ceil(r * g.Wk - 1e-12);
  if (n < 1) n = 1;
  if (n > g.Wk) n = g.Wk;
  return n;
}

static int n_keep_of(const Geom& g, double r) {
  const int kw = window_quota(g, r);
  return kw < 0 ? kw : kw * g.nwin;
}

}  // namespace bsa

using namespace bsa;

extern "C" {

const char* bsa_strerror(int status) {
  switch (status) {
    case BSA_OK: return "ok";
    case BSA_ERR_NULL: return "a required pointer is NULL";
    case BSA_ERR_SHAPE: return "unsupported shape (extents must be positive, the block must divide the grid, d%8==0, d<=256, Bk<=256, N<=8192)";
    case BSA_ERR_RANGE: return "threshold / keep ratio must lie in (0,1], n_keep in [1,Bk], sm_scale > 0, stages in 1..7";
    case BSA_ERR_CAPACITY: return "index buffer smaller than rows*N";
    case BSA_ERR_DTYPE: return "dtype must be BSA_F32 or BSA_BF16";
    case BSA_ERR_LAUNCH: return "HIP launch error";
    case BSA_ERR_WORKSPACE: return "workspace missing or too small";
    case BSA_ERR_STATIC_LIMIT: return "shape needs more scratch than the library's built-in buffer holds (BSA_STATIC_SELECT_BYTES)";
    default: return "unknown bsa status";
  }
}

int bsa_n_keep(const bsa_shape_t* shape, double keep_ratio) {
  Geom g;
  int rc = make_geom(shape, &g);
  if (rc) return rc;
  return n_keep_of(g, keep_ratio);
}

int bsa_pool_blocks(const bsa_shape_t* shape, const void* X, double* Xbar, void* stream) {
  Geom g;
  int rc = make_geom(shape, &g);
  if (rc) return rc;
  if (!X || !Xbar) return BSA_ERR_NULL;
  return launch_pool(g, shape->dtype, X, Xbar, (hipStream_t)stream);
}

size_t bsa_select_workspace_bytes(const bsa_shape_t* shape) {
  Geom g;
  if (make_geom(shape, &g)) return 0;
  return select_workspace_bytes(g);
}

// use_static: the workspace is this device's copy of the library-owned scratch
static int select_common(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                         double threshold, double stat_z, double score_scale, int32_t* q2k_ptr,
                         int32_t* q2k_idx, int64_t idx_capacity, int32_t* k2q_ptr, int32_t* k2q_idx,
                         int64_t* nnz_dev, void* workspace, size_t workspace_bytes, bool use_static,
                         void* stream) {
  Geom g;
  int rc = make_geom(shape, &g);
  if (rc) return rc;
  if (!Qbar || !Kbar || !q2k_ptr || !q2k_idx) return BSA_ERR_NULL;
  if ((k2q_ptr == nullptr) != (k2q_idx == nullptr)) return BSA_ERR_NULL;
  if (!(threshold > 0.0) || !(threshold <= 1.0)) return BSA_ERR_RANGE;
  if (!std::isfinite(score_scale)) return BSA_ERR_RANGE;
  if (idx_capacity < (int64_t)g.rows * g.N) return BSA_ERR_CAPACITY;
  if (use_static) {
    if (select_workspace_bytes(g) > (size_t)BSA_STATIC_SELECT_BYTES) return BSA_ERR_STATIC_LIMIT;
    if ((rc = static_select_scratch(&workspace, &workspace_bytes)) != BSA_OK) return rc;
  }
  if (!workspace || workspace_bytes < select_workspace_bytes(g)) return BSA_ERR_WORKSPACE;
  return launch_select(g, Qbar, Kbar, threshold, stat_z, score_scale, q2k_ptr, q2k_idx, k2q_ptr, k2q_idx,
                       nnz_dev, workspace, (hipStream_t)stream);
}

int bsa_select_kv(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                  double threshold, double score_scale, int32_t* q2k_ptr, int32_t* q2k_idx,
                  int64_t idx_capacity, int32_t* k2q_ptr, int32_t* k2q_idx, int64_t* nnz_dev,
                  void* workspace, size_t workspace_bytes, void* stream) {
  return select_common(shape, Qbar, Kbar, threshold, (double)NAN, score_scale, q2k_ptr, q2k_idx,
                       idx_capacity, k2q_ptr, k2q_idx, nnz_dev, workspace, workspace_bytes, false, stream);
}

int bsa_select_kv_static(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                         double threshold, double score_scale, int32_t* q2k_ptr, int32_t* q2k_idx,
                         int64_t idx_capacity, int32_t* k2q_ptr, int32_t* k2q_idx, int64_t* nnz_dev,
                         void* stream) {
  return select_common(shape, Qbar, Kbar, threshold, (double)NAN, score_scale, q2k_ptr, q2k_idx,
                       idx_capacity, k2q_ptr, k2q_idx, nnz_dev, nullptr, 0, true, stream);
}

int bsa_select_kv_stat(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                       double threshold, double stat_z, double score_scale, int32_t* q2k_ptr,
                       int32_t* q2k_idx, int64_t idx_capacity, int32_t* k2q_ptr, int32_t* k2q_idx,
                       int64_t* nnz_dev, void* workspace, size_t workspace_bytes, void* stream) {
  if (stat_z != stat_z) return BSA_ERR_RANGE;  // NaN
  return select_common(shape, Qbar, Kbar, threshold, stat_z, score_scale, q2k_ptr, q2k_idx,
                       idx_capacity, k2q_ptr, k2q_idx, nnz_dev, workspace, workspace_bytes, false, stream);
}

int bsa_prune_q(const bsa_shape_t* shape, const void* Q, double keep_ratio, int32_t* keep_idx,
                void* stream) {
  Geom g;
  int rc = make_geom(shape, &g);
  if (rc) return rc;
  if (!Q || !keep_idx) return BSA_ERR_NULL;
  const int kw = window_quota(g, keep_ratio);
  if (kw < 0) return kw;
  return launch_prune(g, shape->dtype, Q, kw, keep_idx, (hipStream_t)stream);
}

size_t bsa_fwd_workspace_bytes(const bsa_shape_t* shape, int n_keep) {
  Geom g;
  if (make_geom(shape, &g)) return 0;
  if (n_keep < 1 || n_keep > g.Bk) return 0;
  return mfma_supported(g, shape->dtype, n_keep) ? fwd_workspace_pipe(g, n_keep) : 0;
}

int bsa_attn_fwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                 const int32_t* q2k_ptr, const int32_t* q2k_idx, const int32_t* keep_idx,
                 int n_keep, float sm_scale, void* O, float* LSE, void* workspace,
                 size_t workspace_bytes, void* stream) {
  Geom g;
  int rc = make_geom(shape, &g);
  if (rc) return rc;
  if (!Q || !K || !V || !q2k_ptr || !q2k_idx || !keep_idx || !O || !LSE) return BSA_ERR_NULL;
  if (n_keep < 1 || n_keep > g.Bk || !(sm_scale > 0.f) || !std::isfinite(sm_scale)) return BSA_ERR_RANGE;
  const size_t need = bsa_fwd_workspace_bytes(shape, n_keep);
  if (need && (!workspace || workspace_bytes < need)) return BSA_ERR_WORKSPACE;
  AttnArgs a{};
  a.fwd_ws = need ? workspace : nullptr;
  a.Q = Q; a.K = K; a.V = V; a.q2k_ptr = q2k_ptr; a.q2k_idx = q2k_idx; a.keep_idx = keep_idx;
  a.n_keep = n_keep; a.sm_scale = sm_scale; a.O_out = O; a.LSE_out = LSE;
  if (mfma_supported(g, shape->dtype, n_keep)) return launch_fwd_pipe(g, a, (hipStream_t)stream);
  return launch_fwd_generic(g, shape->dtype, a, (hipStream_t)stream);
}

size_t bsa_bwd_workspace_bytes(const bsa_shape_t* shape, int n_keep) {
  Geom g;
  if (make_geom(shape, &g)) return 0;
  if (n_keep < 1 || n_keep > g.Bk) return 0;
  if (mfma_supported(g, shape->dtype, n_keep)) return bwd_workspace_pipe(g, n_keep);
  return bwd_workspace_generic(g, n_keep);
}

int bsa_attn_bwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                 const void* O, const float* LSE, const void* dO, const int32_t* q2k_ptr,
                 const int32_t* q2k_idx, const int32_t* k2q_ptr, const int32_t* k2q_idx,
                 const int32_t* keep_idx, int n_keep, float sm_scale, void* dQ, void* dK, void* dV,
                 void* workspace, size_t workspace_bytes, void* stream) {
  return bsa_attn_bwd_stages(shape, Q, K, V, O, LSE, dO, q2k_ptr, q2k_idx, k2q_ptr, k2q_idx, keep_idx,
                             n_keep, sm_scale, dQ, dK, dV, workspace, workspace_bytes,
                             BSA_BWD_PRE | BSA_BWD_DQ | BSA_BWD_DKV, stream);
}

int bsa_attn_bwd_stages(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                        const void* O, const float* LSE, const void* dO, const int32_t* q2k_ptr,
                        const int32_t* q2k_idx, const int32_t* k2q_ptr, const int32_t* k2q_idx,
                        const int32_t* keep_idx, int n_keep, float sm_scale, void* dQ, void* dK,
                        void* dV, void* workspace, size_t workspace_bytes, unsigned stages,
                        void* stream) {
  Geom g;
  int rc = make_geom(shape, &g);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE || !dO || !q2k_ptr || !q2k_idx || !k2q_ptr || !k2q_idx ||
      !keep_idx || !dQ || !dK || !dV)
    return BSA_ERR_NULL;
  if (n_keep < 1 || n_keep > g.Bk || !(sm_scale > 0.f) || !std::isfinite(sm_scale)) return BSA_ERR_RANGE;
  if (!workspace || workspace_bytes < bsa_bwd_workspace_bytes(shape, n_keep)) return BSA_ERR_WORKSPACE;
  AttnArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.LSE_in = LSE; a.dO = dO;
  a.q2k_ptr = q2k_ptr; a.q2k_idx = q2k_idx; a.k2q_ptr = k2q_ptr; a.k2q_idx = k2q_idx;
  a.keep_idx = keep_idx; a.n_keep = n_keep; a.sm_scale = sm_scale;
  a.dQ = dQ; a.dK = dK; a.dV = dV; a.ws = workspace;
  if (stages == 0 || (stages & ~7u)) return BSA_ERR_RANGE;
  a.stages = stages;
  if (mfma_supported(g, shape->dtype, n_keep)) return launch_bwd_pipe(g, a, (hipStream_t)stream);
  return launch_bwd_generic(g, shape->dtype, a, (hipStream_t)stream);
}

// ---- dense baseline (Eq. 1): same kernels, tiles = runs of Bk consecutive tokens, all pairs ----
static int dense_geom(const bsa_shape_t* shape, Geom* g) {
  int rc = make_geom(shape, g);
  if (rc) return rc;
  g->dense = 1;
  g->tiled = 1;
  return BSA_OK;
}

size_t bsa_dense_bwd_workspace_bytes(const bsa_shape_t* shape) {
  Geom g;
  if (dense_geom(shape, &g)) return 0;
  if (mfma_supported(g, shape->dtype, g.Bk)) return bwd_workspace_pipe(g, g.Bk);
  return bwd_workspace_generic(g, g.Bk);
}

int bsa_dense_attn_fwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                       float sm_scale, void* O, float* LSE, void* stream) {
  Geom g;
  int rc = dense_geom(shape, &g);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE) return BSA_ERR_NULL;
  if (!(sm_scale > 0.f) || !std::isfinite(sm_scale)) return BSA_ERR_RANGE;
  AttnArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.n_keep = g.Bk; a.sm_scale = sm_scale; a.O_out = O; a.LSE_out = LSE;
  if (mfma_supported(g, shape->dtype, g.Bk)) return launch_fwd_pipe(g, a, (hipStream_t)stream);
  return launch_fwd_generic(g, shape->dtype, a, (hipStream_t)stream);
}

int bsa_dense_attn_bwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                       const void* O, const float* LSE, const void* dO, float sm_scale, void* dQ,
                       void* dK, void* dV, void* workspace, size_t workspace_bytes, void* stream) {
  Geom g;
  int rc = dense_geom(shape, &g);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV) return BSA_ERR_NULL;
  if (!(sm_scale > 0.f) || !std::isfinite(sm_scale)) return BSA_ERR_RANGE;
  if (!workspace || workspace_bytes < bsa_dense_bwd_workspace_bytes(shape)) return BSA_ERR_WORKSPACE;
  AttnArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.LSE_in = LSE; a.dO = dO; a.n_keep = g.Bk;
  a.sm_scale = sm_scale; a.dQ = dQ; a.dK = dK; a.dV = dV; a.ws = workspace;
  a.stages = BSA_BWD_PRE | BSA_BWD_DQ | BSA_BWD_DKV;
  if (mfma_supported(g, shape->dtype, g.Bk)) return launch_bwd_pipe(g, a, (hipStream_t)stream);
  return launch_bwd_generic(g, shape->dtype, a, (hipStream_t)stream);
}

}  // extern "C"
