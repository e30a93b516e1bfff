// C ABI of the library: host-side argument validation and kernel dispatch.
// Declarations and the meaning of every argument are in include/affmae.h.
#include "../../include/affmae.h"

#include "launch.h"

#include <atomic>

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

struct KnnPlan {
  size_t centroid_off, near_off, members_off, total;
};
KnnPlan knn_plan(int B, int N, int S, int M) {
  KnnPlan p;
  const size_t G = ((size_t)N + S - 1) / S;
  size_t off = 0;
  p.centroid_off = off;
  off += align_up((size_t)B * G * 2 * sizeof(float));
  p.near_off = off;
  off += align_up((size_t)B * G * M * sizeof(int32_t));
  p.members_off = off;
  off += align_up((size_t)B * N * sizeof(int32_t));
  p.total = off;
  return p;
}

int check_knn_shape(int B, int N, int S, int M, int K) {
  if (B < 1 || N < 1 || S < 1 || M < 1 || K < 1) return AFFMAE_ERR_SHAPE;
  const int G = (int)(((long long)N + S - 1) / S);
  if (M > G) return AFFMAE_ERR_SHAPE;
  // every token needs K candidates: the smallest candidate set holds the short last cluster (if there is one)
  const long long last = (long long)N - (long long)(G - 1) * S;
  if ((long long)K > (long long)(M - 1) * S + last) return AFFMAE_ERR_SHAPE;
  if (K > AFFMAE_MAX_K || M > AFFMAE_MAX_NEAR) return AFFMAE_ERR_UNSUPPORTED;
  if ((long long)M * S > 4096) return AFFMAE_ERR_UNSUPPORTED;  // candidate staging: 16 B each in 64 KB of LDS
  return AFFMAE_OK;
}

int check_pla_shape(int B, int N, int H, int d, int K, int dtype) {
  if (dtype != AFFMAE_F32 && dtype != AFFMAE_BF16) return AFFMAE_ERR_DTYPE;
  if (B < 1 || N < 1 || H < 1 || d < 1 || K < 1) return AFFMAE_ERR_SHAPE;
  if (d != 16 && d != 32 && d != 64) return AFFMAE_ERR_UNSUPPORTED;
  if (K > AFFMAE_MAX_K) return AFFMAE_ERR_UNSUPPORTED;
  // per-wave LDS of the gather kernels: (K+1) * (1 + 2H) floats (+ 2*H*d with blanks), four waves
  if ((size_t)4 * ((size_t)(K + 1) * (1 + 2 * (size_t)H) + 2 * (size_t)H * d) * sizeof(float) > 64 * 1024)
    return AFFMAE_ERR_UNSUPPORTED;
  return AFFMAE_OK;
}

// Shapes the cluster-tiled kernels take (storage type and head size are checked by the caller).
bool tiled_shape_ok(int B, int N, int K, int S, int M) {
  affmae::PlaArgs a = {};
  a.B = B; a.N = N; a.K = K; a.S = S; a.M = M; a.d = 32; a.dtype = AFFMAE_BF16;
  static const int32_t dummy = 0;
  a.near_clusters = &dummy;  // only tested for being non-null
  return B >= 1 && N >= 1 && K >= 1 && S >= 1 && M >= 1 && affmae::pla_cluster_supported(a);
}

}  // namespace

extern "C" {

const char* affmae_status_string(int status) {
  switch (status) {
    case AFFMAE_OK: return "ok";
    case AFFMAE_ERR_NULL: return "a required pointer is NULL";
    case AFFMAE_ERR_SHAPE: return "a size is non-positive or inconsistent";
    case AFFMAE_ERR_DTYPE: return "unknown storage type";
    case AFFMAE_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
    case AFFMAE_ERR_UNSUPPORTED: return "request outside the implemented limits";
    case AFFMAE_ERR_DEVICE: return "the HIP runtime refused a launch";
    default: return "unknown status";
  }
}

int affmae_version(void) { return 200; }

#ifndef AFFMAE_BUILD_ID
#define AFFMAE_BUILD_ID "unstamped"
#endif
const char* affmae_build_id(void) { return AFFMAE_BUILD_ID; }

size_t affmae_cluster_workspace_bytes(int B, int N) {
  if (B < 1 || N < 1 || N > (1 << 24)) return 0;
  return align_up(affmae::cluster_workspace_bytes(B, N));
}

int affmae_cluster(const float* coords, int B, int N, int S, double x0, double y0, double w, double h,
                   int32_t* order, int32_t* cluster_id, void* workspace, size_t workspace_bytes, void* stream) {
  if (!coords || !order) return AFFMAE_ERR_NULL;
  if (B < 1 || N < 1 || S < 1) return AFFMAE_ERR_SHAPE;
  if (!(w > 0.0) || !(h > 0.0) || !(w < 1e300) || !(h < 1e300) || !(x0 > -1e300 && x0 < 1e300) ||
      !(y0 > -1e300 && y0 < 1e300))
    return AFFMAE_ERR_SHAPE;  // the frame must be finite and non-empty
  if (N > (1 << 24)) return AFFMAE_ERR_UNSUPPORTED;
  const size_t need = align_up(affmae::cluster_workspace_bytes(B, N));
  if (!workspace || workspace_bytes < need || misaligned(workspace, kAlign)) return AFFMAE_ERR_WORKSPACE;
  return affmae::launch_cluster(coords, B, N, S, x0, y0, w, h, order, cluster_id, workspace,
                                static_cast<hipStream_t>(stream)) == hipSuccess
             ? AFFMAE_OK
             : AFFMAE_ERR_DEVICE;
}

}  // extern "C"

namespace {

int check_vts_shape(int B, int Mq, int Nv, int C, int Hg, int Wg, float x0, float y0, float cell, int Kt) {
  if (B < 1 || Mq < 1 || Nv < 1 || C < 1 || Hg < 1 || Wg < 1 || Kt < 1) return AFFMAE_ERR_SHAPE;
  if (Kt > Nv) return AFFMAE_ERR_SHAPE;
  if (!(cell > 0.f) || !(cell < 3e38f) || !(x0 > -3e38f && x0 < 3e38f) || !(y0 > -3e38f && y0 < 3e38f))
    return AFFMAE_ERR_SHAPE;  // the grid must be finite and non-empty
  if (Kt > AFFMAE_MAX_K) return AFFMAE_ERR_UNSUPPORTED;
  if (C % 2) return AFFMAE_ERR_UNSUPPORTED;  // the kernels move two channels per lane
  if ((long long)B * Hg * Wg > (1ll << 31) - 8 || (long long)B * Mq > (1ll << 31) - 8 ||
      (long long)B * Nv > (1ll << 31) - 8)
    return AFFMAE_ERR_UNSUPPORTED;  // cells, queries and tokens are indexed with int32
  return AFFMAE_OK;
}

affmae::VtsArgs vts_args(const float* query_xy, const float* vis_xy, const void* feat, const int32_t* table, int B,
                         int Mq, int Nv, int C, int Hg, int Wg, float x0, float y0, float cell, int Kt, float p,
                         float eps, int dtype) {
  affmae::VtsArgs a = {};
  a.query_xy = query_xy; a.vis_xy = vis_xy; a.feat = feat; a.table = table;
  a.B = B; a.Mq = Mq; a.Nv = Nv; a.C = C; a.Hg = Hg; a.Wg = Wg; a.Kt = Kt; a.dtype = dtype;
  a.x0 = x0; a.y0 = y0; a.cell = cell; a.p = p; a.eps = eps;
  return a;
}

}  // namespace

extern "C" {

int affmae_vts_table(const float* vis_xy, int B, int Nv, int Hg, int Wg, float x0, float y0, float cell, int Kt,
                     int32_t* table, void* stream) {
  if (!vis_xy || !table) return AFFMAE_ERR_NULL;
  const int rc = check_vts_shape(B, 1, Nv, 2, Hg, Wg, x0, y0, cell, Kt);
  if (rc != AFFMAE_OK) return rc;
  affmae::VtsArgs a = vts_args(nullptr, vis_xy, nullptr, nullptr, B, 1, Nv, 2, Hg, Wg, x0, y0, cell, Kt, 0.f, 0.f, 0);
  a.table_out = table;
  return affmae::launch_vts_table(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}

int affmae_vts_fwd(const float* query_xy, const float* vis_xy, const void* feat, const int32_t* table, int B, int Mq,
                   int Nv, int C, int Hg, int Wg, float x0, float y0, float cell, int Kt, float p, float eps,
                   int dtype, void* out, void* stream) {
  if (!query_xy || !vis_xy || !feat || !table || !out) return AFFMAE_ERR_NULL;
  if (dtype != AFFMAE_F32 && dtype != AFFMAE_BF16) return AFFMAE_ERR_DTYPE;
  const int rc = check_vts_shape(B, Mq, Nv, C, Hg, Wg, x0, y0, cell, Kt);
  if (rc != AFFMAE_OK) return rc;
  if (misaligned(feat, 4) || misaligned(out, 4)) return AFFMAE_ERR_SHAPE;
  affmae::VtsArgs a = vts_args(query_xy, vis_xy, feat, table, B, Mq, Nv, C, Hg, Wg, x0, y0, cell, Kt, p, eps, dtype);
  a.out = out;
  return affmae::launch_vts_fwd(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}

size_t affmae_vts_bwd_workspace_bytes(int B, int Mq, int Nv, int Kt) {
  if (B < 1 || Mq < 1 || Nv < 1 || Kt < 1 || Kt > AFFMAE_MAX_K) return 0;
  if ((long long)B * Mq * Kt > (1ll << 31) - 8 || (long long)B * Nv > (1ll << 31) - 8) return 0;
  return align_up(affmae::vts_bwd_workspace_bytes(B, Mq, Nv, Kt));
}

int affmae_vts_bwd(const float* query_xy, const float* vis_xy, const void* feat, const int32_t* table,
                   const void* dout, int B, int Mq, int Nv, int C, int Hg, int Wg, float x0, float y0, float cell,
                   int Kt, float p, float eps, int dtype, void* dfeat, float* dquery, float* dp, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (!query_xy || !vis_xy || !feat || !table || !dout || !dfeat || !dquery) return AFFMAE_ERR_NULL;
  if (dtype != AFFMAE_F32 && dtype != AFFMAE_BF16) return AFFMAE_ERR_DTYPE;
  const int rc = check_vts_shape(B, Mq, Nv, C, Hg, Wg, x0, y0, cell, Kt);
  if (rc != AFFMAE_OK) return rc;
  if (misaligned(feat, 4) || misaligned(dout, 4) || misaligned(dfeat, 4)) return AFFMAE_ERR_SHAPE;
  if ((long long)B * Mq * Kt > (1ll << 31) - 8 || (long long)B * Nv > (1ll << 31) - 8)
    return AFFMAE_ERR_UNSUPPORTED;  // pairs and tokens are indexed with int32
  const size_t need = align_up(affmae::vts_bwd_workspace_bytes(B, Mq, Nv, Kt));
  if (!workspace || workspace_bytes < need || misaligned(workspace, kAlign)) return AFFMAE_ERR_WORKSPACE;
  affmae::VtsArgs a = vts_args(query_xy, vis_xy, feat, table, B, Mq, Nv, C, Hg, Wg, x0, y0, cell, Kt, p, eps, dtype);
  a.dout = dout; a.dfeat = dfeat; a.dquery = dquery; a.dp = dp; a.workspace = workspace;
  return affmae::launch_vts_bwd(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}

}  // extern "C"

namespace {
int check_merge_shape(int B, int N, int C, int K, int n_keep) {
  if (B < 1 || N < 1 || C < 1 || K < 1 || n_keep < 1 || n_keep > N) return AFFMAE_ERR_SHAPE;
  if (K > AFFMAE_MAX_K) return AFFMAE_ERR_UNSUPPORTED;
  if ((long long)B * N > (1ll << 31) - 8 || (long long)B * n_keep * K > (1ll << 31) - 8)
    return AFFMAE_ERR_UNSUPPORTED;  // tokens and (anchor, neighbour) pairs are indexed with int32
  return AFFMAE_OK;
}
}  // namespace

extern "C" {

int affmae_merge_select(const float* score, const float* coords, int B, int N, int n_keep, int32_t* anchor_idx,
                        float* anchor_xy, void* stream) {
  if (!score || !anchor_idx) return AFFMAE_ERR_NULL;
  if (anchor_xy && !coords) return AFFMAE_ERR_NULL;
  if (B < 1 || N < 1 || n_keep < 1 || n_keep > N) return AFFMAE_ERR_SHAPE;
  if (anchor_xy && (misaligned(coords, 8) || misaligned(anchor_xy, 8))) return AFFMAE_ERR_SHAPE;  // moved as pairs
  if (N > (1 << 24) || (long long)B * N > (1ll << 31) - 8) return AFFMAE_ERR_UNSUPPORTED;
  return affmae::launch_merge_select(score, coords, B, N, n_keep, anchor_idx, anchor_xy,
                                     static_cast<hipStream_t>(stream)) == hipSuccess
             ? AFFMAE_OK
             : AFFMAE_ERR_DEVICE;
}

int affmae_merge_fwd(const void* feat, const float* coords, const float* score, const int32_t* nbr_idx,
                     const int32_t* anchor_idx, int B, int N, int C, int K, int n_keep, float p, int dtype, void* out,
                     void* stream) {
  if (!feat || !coords || !score || !nbr_idx || !anchor_idx || !out) return AFFMAE_ERR_NULL;
  if (dtype != AFFMAE_F32 && dtype != AFFMAE_BF16) return AFFMAE_ERR_DTYPE;
  const int rc = check_merge_shape(B, N, C, K, n_keep);
  if (rc != AFFMAE_OK) return rc;
  if (!(p >= 0.f) || !(p < 3e38f)) return AFFMAE_ERR_SHAPE;
  if (misaligned(coords, 8) || misaligned(feat, dtype == AFFMAE_BF16 ? 2 : 4) || misaligned(out, dtype == AFFMAE_BF16 ? 2 : 4))
    return AFFMAE_ERR_SHAPE;
  affmae::MergeArgs a = {};
  a.feat = feat; a.coords = coords; a.score = score; a.nbr_idx = nbr_idx; a.anchor_idx = anchor_idx;
  a.B = B; a.N = N; a.C = C; a.K = K; a.n_keep = n_keep; a.dtype = dtype; a.p = p; a.out = out;
  return affmae::launch_merge_fwd(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}

size_t affmae_merge_bwd_workspace_bytes(int B, int N, int K, int n_keep) {
  if (check_merge_shape(B, N, 1, K, n_keep) != AFFMAE_OK) return 0;
  return align_up(affmae::merge_bwd_workspace_bytes(B, N, K, n_keep));
}

int affmae_merge_bwd(const void* feat, const float* coords, const float* score, const int32_t* nbr_idx,
                     const int32_t* anchor_idx, const void* dout, int B, int N, int C, int K, int n_keep, float p,
                     int dtype, void* dfeat, float* dscore, float* dp, void* workspace, size_t workspace_bytes,
                     void* stream) {
  if (!feat || !coords || !score || !nbr_idx || !anchor_idx || !dout || !dfeat || !dscore) return AFFMAE_ERR_NULL;
  if (dtype != AFFMAE_F32 && dtype != AFFMAE_BF16) return AFFMAE_ERR_DTYPE;
  const int rc = check_merge_shape(B, N, C, K, n_keep);
  if (rc != AFFMAE_OK) return rc;
  if (!(p >= 0.f) || !(p < 3e38f)) return AFFMAE_ERR_SHAPE;
  const size_t el = dtype == AFFMAE_BF16 ? 2 : 4;
  if (misaligned(coords, 8) || misaligned(feat, el) || misaligned(dout, el) || misaligned(dfeat, el)) return AFFMAE_ERR_SHAPE;
  const size_t need = align_up(affmae::merge_bwd_workspace_bytes(B, N, K, n_keep));
  if (!workspace || workspace_bytes < need || misaligned(workspace, kAlign)) return AFFMAE_ERR_WORKSPACE;
  affmae::MergeArgs a = {};
  a.feat = feat; a.coords = coords; a.score = score; a.nbr_idx = nbr_idx; a.anchor_idx = anchor_idx; a.dout = dout;
  a.B = B; a.N = N; a.C = C; a.K = K; a.n_keep = n_keep; a.dtype = dtype; a.p = p;
  a.dfeat = dfeat; a.dscore = dscore; a.dp = dp; a.workspace = workspace;
  return affmae::launch_merge_bwd(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}

size_t affmae_knn_workspace_bytes(int B, int N, int S, int M, int K) {
  if (check_knn_shape(B, N, S, M, K) != AFFMAE_OK) return 0;
  return knn_plan(B, N, S, M).total;
}

int affmae_knn(const float* coords, const int32_t* cluster_id, int B, int N, int S, int M, int K,
               int32_t* nbr_idx, int32_t* near_clusters, void* workspace, size_t workspace_bytes, void* stream) {
  if (!coords || !nbr_idx) return AFFMAE_ERR_NULL;
  const int rc = check_knn_shape(B, N, S, M, K);
  if (rc != AFFMAE_OK) return rc;
  const KnnPlan plan = knn_plan(B, N, S, M);
  if (!workspace || workspace_bytes < plan.total || misaligned(workspace, kAlign)) return AFFMAE_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  affmae::KnnArgs a;
  a.coords = coords;
  a.cluster_id = cluster_id;
  a.B = B; a.N = N; a.S = S; a.M = M; a.K = K; a.G = (N + S - 1) / S;
  a.nbr_idx = nbr_idx;
  a.near_clusters = near_clusters ? near_clusters : reinterpret_cast<int32_t*>(ws + plan.near_off);
  a.centroid = reinterpret_cast<float*>(ws + plan.centroid_off);
  a.members = reinterpret_cast<int32_t*>(ws + plan.members_off);
  return affmae::launch_knn(a, static_cast<hipStream_t>(stream)) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}

}  // extern "C"

// Scratch of affmae_knn_static: a fixed array in device memory, one copy per GPU, held until the process ends.
// In host code the array's name is only a handle; its device address comes from hipGetSymbolAddress, once per
// device (with that device current), and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[AFFMAE_KNN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, or nullptr when the runtime refuses it.
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // (two first callers store the same address)
  }
  return ptr;
}
}  // namespace

extern "C" {

int affmae_knn_static(const float* coords, const int32_t* cluster_id, int B, int N, int S, int M, int K,
                      int32_t* nbr_idx, int32_t* near_clusters, void* stream) {
  if (!coords || !nbr_idx) return AFFMAE_ERR_NULL;
  const int rc = check_knn_shape(B, N, S, M, K);
  if (rc != AFFMAE_OK) return rc;
  if (knn_plan(B, N, S, M).total > (size_t)AFFMAE_KNN_STATIC_SCRATCH_BYTES) return AFFMAE_ERR_WORKSPACE;
  void* ptr = static_scratch();
  if (!ptr) return AFFMAE_ERR_DEVICE;
  // every word of the scratch that the kernels read is written earlier in the same call: nothing to clear
  return affmae_knn(coords, cluster_id, B, N, S, M, K, nbr_idx, near_clusters, ptr, AFFMAE_KNN_STATIC_SCRATCH_BYTES,
                    stream);
}

size_t affmae_pla_plan_bytes(int B, int N, int K, int S, int M) {
  if (!tiled_shape_ok(B, N, K, S, M)) return 0;
  return affmae::pla_plan_bytes(B, N, K, S, M);
}

int affmae_pla_plan(const int32_t* nbr_idx, const int32_t* near_clusters, int B, int N, int K, int S, int M,
                    void* plan, size_t plan_bytes, void* stream) {
  if (!nbr_idx || !near_clusters || !plan) return AFFMAE_ERR_NULL;
  if (B < 1 || N < 1 || K < 1 || S < 1 || M < 1 || M > (N + S - 1) / S) return AFFMAE_ERR_SHAPE;
  if (!tiled_shape_ok(B, N, K, S, M)) return AFFMAE_ERR_UNSUPPORTED;
  if (plan_bytes < affmae::pla_plan_bytes(B, N, K, S, M) || misaligned(plan, kAlign)) return AFFMAE_ERR_WORKSPACE;
  return affmae::launch_pla_plan(nbr_idx, near_clusters, B, N, K, S, M, plan, static_cast<hipStream_t>(stream)) ==
                 hipSuccess
             ? AFFMAE_OK
             : AFFMAE_ERR_DEVICE;
}

size_t affmae_pla_fwd_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int dtype, int clustered) {
  if (check_pla_shape(B, N, H, d, K, dtype) != AFFMAE_OK) return 0;
  if (clustered && dtype == AFFMAE_BF16 && d == 32 && S > 0) return affmae_pla_plan_bytes(B, N, K, S, M);
  return 0;
}

}  // extern "C"

namespace {
// affmae_pla_fwd: every check, then (with `launch`) the kernels.  Without `launch` it returns the status the call
// would have up to its first launch: entry points that put kernels of their own in front of this one validate
// with it first, so that an error never leaves work enqueued.
int pla_fwd_run(const void* q, const void* k, const void* v, const void* bias, const int32_t* nbr_idx,
                const int32_t* near_clusters, const void* plan, const void* k_blank, const void* v_blank, int B,
                int N, int H, int d, int K, int S, int M, float scale, int dtype, void* out, float* lse,
                void* workspace, size_t workspace_bytes, void* stream, bool launch) {
  if (!q || !k || !v || !nbr_idx || !out || !lse) return AFFMAE_ERR_NULL;
  if ((k_blank == nullptr) != (v_blank == nullptr)) return AFFMAE_ERR_NULL;
  const int rc = check_pla_shape(B, N, H, d, K, dtype);
  if (rc != AFFMAE_OK) return rc;
  if (near_clusters) {
    if (S < 1 || M < 1 || M > (N + S - 1) / S) return AFFMAE_ERR_SHAPE;
  }
  if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(out, 16)) return AFFMAE_ERR_SHAPE;
  if ((k_blank && misaligned(k_blank, 16)) || (v_blank && misaligned(v_blank, 16))) return AFFMAE_ERR_SHAPE;
  affmae::PlaArgs a = {};
  a.q = q; a.k = k; a.v = v; a.bias = bias; a.nbr_idx = nbr_idx; a.near_clusters = near_clusters;
  a.k_blank = k_blank; a.v_blank = v_blank;
  a.B = B; a.N = N; a.H = H; a.d = d; a.K = K; a.S = S; a.M = M; a.scale = scale; a.dtype = dtype;
  a.out = out; a.lse = lse; a.workspace = workspace;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!affmae::pla_cluster_supported(a)) {
    if (!launch) return AFFMAE_OK;
    return affmae::launch_pla_fwd_general(a, st) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
  }
  if (plan && misaligned(plan, kAlign)) return AFFMAE_ERR_WORKSPACE;
  if (!plan) {  // no cached plan: rebuild it in the workspace
    const size_t need = affmae::pla_plan_bytes(B, N, K, S, M);
    if (!workspace || workspace_bytes < need || misaligned(workspace, kAlign)) return AFFMAE_ERR_WORKSPACE;
  }
  if (!launch) return AFFMAE_OK;
  if (!plan) {
    if (affmae::launch_pla_plan(nbr_idx, near_clusters, B, N, K, S, M, workspace, st) != hipSuccess)
      return AFFMAE_ERR_DEVICE;
    plan = workspace;
  }
  return affmae::launch_pla_fwd_cluster(a, plan, st) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}
}  // namespace

extern "C" {

int affmae_pla_fwd(const void* q, const void* k, const void* v, const void* bias, const int32_t* nbr_idx,
                   const int32_t* near_clusters, const void* plan, const void* k_blank, const void* v_blank, int B,
                   int N, int H, int d, int K, int S, int M, float scale, int dtype, void* out, float* lse,
                   void* workspace, size_t workspace_bytes, void* stream) {
  return pla_fwd_run(q, k, v, bias, nbr_idx, near_clusters, plan, k_blank, v_blank, B, N, H, d, K, S, M, scale, dtype,
                     out, lse, workspace, workspace_bytes, stream, true);
}

size_t affmae_pla_bwd_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int dtype, int clustered) {
  if (check_pla_shape(B, N, H, d, K, dtype) != AFFMAE_OK) return 0;
  const size_t gather = align_up(affmae::pla_bwd_general_workspace_bytes(B, N, H, K));
  size_t tiled = 0;
  if (clustered && dtype == AFFMAE_BF16 && d == 32 && S > 0 && tiled_shape_ok(B, N, K, S, M))
    tiled = align_up(affmae::pla_plan_bytes(B, N, K, S, M)) + affmae::pla_bwd_cluster_workspace_bytes(B, N, H, K, S, M);
  return gather > tiled ? gather : tiled;
}

}  // extern "C"

namespace {
// affmae_pla_bwd with the same split as pla_fwd_run.
int pla_bwd_run(const void* q, const void* k, const void* v, const void* bias, const int32_t* nbr_idx,
                const int32_t* near_clusters, const void* plan, const void* k_blank, const void* v_blank,
                const void* out, const float* lse, const void* dout, int B, int N, int H, int d, int K, int S,
                int M, float scale, int dtype, void* dq, void* dk, void* dv, void* dbias, float* dk_blank,
                float* dv_blank, void* workspace, size_t workspace_bytes, void* stream, bool launch) {
  if (!q || !k || !v || !nbr_idx || !lse || !dout || !dq || !dk || !dv) return AFFMAE_ERR_NULL;
  if ((k_blank == nullptr) != (v_blank == nullptr)) return AFFMAE_ERR_NULL;
  if ((dk_blank == nullptr) != (dv_blank == nullptr)) return AFFMAE_ERR_NULL;
  const int rc = check_pla_shape(B, N, H, d, K, dtype);
  if (rc != AFFMAE_OK) return rc;
  if (near_clusters) {
    if (S < 1 || M < 1 || M > (N + S - 1) / S) return AFFMAE_ERR_SHAPE;
  }
  if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(dout, 16) || misaligned(dq, 16) ||
      misaligned(dk, 16) || misaligned(dv, 16))
    return AFFMAE_ERR_SHAPE;
  if ((k_blank && misaligned(k_blank, 16)) || (v_blank && misaligned(v_blank, 16))) return AFFMAE_ERR_SHAPE;
  if (workspace && misaligned(workspace, kAlign)) return AFFMAE_ERR_WORKSPACE;
  affmae::PlaArgs a = {};
  a.q = q; a.k = k; a.v = v; a.bias = bias; a.nbr_idx = nbr_idx; a.near_clusters = near_clusters;
  a.k_blank = k_blank; a.v_blank = v_blank;
  a.B = B; a.N = N; a.H = H; a.d = d; a.K = K; a.S = S; a.M = M; a.scale = scale; a.dtype = dtype;
  a.out = const_cast<void*>(out); a.lse = const_cast<float*>(lse); a.dout = dout;
  a.dq = dq; a.dk = dk; a.dv = dv; a.dbias = dbias; a.dk_blank = dk_blank; a.dv_blank = dv_blank;
  a.workspace = workspace;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (affmae::pla_cluster_supported(a)) {
    if (!out) return AFFMAE_ERR_NULL;
    if (misaligned(out, 16)) return AFFMAE_ERR_SHAPE;
    if (plan && misaligned(plan, kAlign)) return AFFMAE_ERR_WORKSPACE;
    const size_t plan_bytes = plan ? 0 : align_up(affmae::pla_plan_bytes(B, N, K, S, M));
    const size_t need = plan_bytes + affmae::pla_bwd_cluster_workspace_bytes(B, N, H, K, S, M);
    if (!workspace || workspace_bytes < need) return AFFMAE_ERR_WORKSPACE;
    if (!launch) return AFFMAE_OK;
    char* ws = static_cast<char*>(workspace);
    if (!plan) {
      if (affmae::launch_pla_plan(nbr_idx, near_clusters, B, N, K, S, M, ws, st) != hipSuccess)
        return AFFMAE_ERR_DEVICE;
      plan = ws;
    }
    return affmae::launch_pla_bwd_cluster(a, plan, ws + plan_bytes, st) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
  }
  if ((long long)B * N * K >= (1ll << 31)) return AFFMAE_ERR_UNSUPPORTED;  // (query, slot) pairs are numbered in 32 bits
  const size_t need = align_up(affmae::pla_bwd_general_workspace_bytes(B, N, H, K));
  if (!workspace || workspace_bytes < need) return AFFMAE_ERR_WORKSPACE;
  if (!launch) return AFFMAE_OK;
  return affmae::launch_pla_bwd_general(a, st) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
}
}  // namespace

extern "C" {

int affmae_pla_bwd(const void* q, const void* k, const void* v, const void* bias, const int32_t* nbr_idx,
                   const int32_t* near_clusters, const void* plan, const void* k_blank, const void* v_blank,
                   const void* out, const float* lse, const void* dout, int B, int N, int H, int d, int K, int S,
                   int M, float scale, int dtype, void* dq, void* dk, void* dv, void* dbias, float* dk_blank,
                   float* dv_blank, void* workspace, size_t workspace_bytes, void* stream) {
  return pla_bwd_run(q, k, v, bias, nbr_idx, near_clusters, plan, k_blank, v_blank, out, lse, dout, B, N, H, d, K, S, M,
                     scale, dtype, dq, dk, dv, dbias, dk_blank, dv_blank, workspace, workspace_bytes, stream, true);
}

namespace {
// limits of the relative-position table: the gradient kernel keeps H tables in LDS
int check_relpos(const float* coords, const void* table, int B, int N, int H, int K, int R, float rate) {
  if (!coords || !table) return AFFMAE_ERR_NULL;
  if ((long long)B * N * K > (1ll << 31) - 8) return AFFMAE_ERR_UNSUPPORTED;  // pairs are indexed with int32
  if (R < 0 || !(rate > 0.f) || !(rate < 3e38f)) return AFFMAE_ERR_SHAPE;
  if (R > 31 || (long long)H * (2 * R + 1) * (2 * R + 1) > 12288) return AFFMAE_ERR_UNSUPPORTED;
  if (misaligned(coords, 8)) return AFFMAE_ERR_SHAPE;
  return AFFMAE_OK;
}
size_t bias_bytes(int B, int N, int H, int K, int dtype) {
  return align_up((size_t)B * N * H * K * (dtype == AFFMAE_BF16 ? 2 : 4));
}
// Shapes for which the tiled kernels look the bias up themselves (the coordinates' alignment is checked apart).
bool relpos_in_kernel(int B, int N, int d, int K, int S, int M, int dtype, int clustered) {
  return clustered && dtype == AFFMAE_BF16 && d == 32 && K % 8 == 0 && tiled_shape_ok(B, N, K, S, M);
}
}  // namespace

size_t affmae_pla_fwd_relpos_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int dtype,
                                             int clustered) {
  if (check_pla_shape(B, N, H, d, K, dtype) != AFFMAE_OK) return 0;
  if (relpos_in_kernel(B, N, d, K, S, M, dtype, clustered)) return align_up(affmae::pla_plan_bytes(B, N, K, S, M));
  return bias_bytes(B, N, H, K, dtype) + align_up(affmae_pla_fwd_workspace_bytes(B, N, H, d, K, S, M, dtype, clustered));
}

int affmae_pla_fwd_relpos(const void* q, const void* k, const void* v, const float* coords, const void* rel_table,
                          const int32_t* nbr_idx, const int32_t* near_clusters, const void* plan,
                          const void* k_blank, const void* v_blank, int B, int N, int H, int d, int K, int S, int M,
                          float scale, int R, float rate, int dtype, void* out, float* lse, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !nbr_idx || !out || !lse) return AFFMAE_ERR_NULL;
  int rc = check_pla_shape(B, N, H, d, K, dtype);
  if (rc != AFFMAE_OK) return rc;
  rc = check_relpos(coords, rel_table, B, N, H, K, R, rate);
  if (rc != AFFMAE_OK) return rc;
  const size_t bb = bias_bytes(B, N, H, K, dtype);
  if (!workspace || workspace_bytes < affmae_pla_fwd_relpos_workspace_bytes(B, N, H, d, K, S, M, dtype,
                                                                             near_clusters != nullptr) ||
      misaligned(workspace, kAlign))
    return AFFMAE_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (relpos_in_kernel(B, N, d, K, S, M, dtype, near_clusters != nullptr)) {
    // the tiled kernel looks the bias up itself: no bias tensor
    if (M > (N + S - 1) / S) return AFFMAE_ERR_SHAPE;
    affmae::PlaArgs a = {};
    a.q = q; a.k = k; a.v = v; a.nbr_idx = nbr_idx; a.near_clusters = near_clusters;
    a.k_blank = k_blank; a.v_blank = v_blank;
    a.B = B; a.N = N; a.H = H; a.d = d; a.K = K; a.S = S; a.M = M; a.scale = scale; a.dtype = dtype;
    a.out = out; a.lse = lse;
    a.rel_coords = coords; a.rel_table = rel_table; a.rel_R = R; a.rel_rate = rate;
    if (!affmae::pla_cluster_relpos_supported(a)) return AFFMAE_ERR_UNSUPPORTED;  // (the workspace is sized for this path)
    if ((k_blank == nullptr) != (v_blank == nullptr)) return AFFMAE_ERR_NULL;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(out, 16)) return AFFMAE_ERR_SHAPE;
    if ((k_blank && misaligned(k_blank, 16)) || (v_blank && misaligned(v_blank, 16))) return AFFMAE_ERR_SHAPE;
    if (plan && misaligned(plan, kAlign)) return AFFMAE_ERR_WORKSPACE;
    if (!plan) {  // the workspace holds at least a plan (checked above)
      if (affmae::launch_pla_plan(nbr_idx, near_clusters, B, N, K, S, M, ws, st) != hipSuccess)
        return AFFMAE_ERR_DEVICE;
      plan = ws;
    }
    return affmae::launch_pla_fwd_cluster(a, plan, st) == hipSuccess ? AFFMAE_OK : AFFMAE_ERR_DEVICE;
  }
  // the bias is written into the workspace by a kernel of its own: validate the attention call before it
  rc = pla_fwd_run(q, k, v, ws, nbr_idx, near_clusters, plan, k_blank, v_blank, B, N, H, d, K, S, M, scale, dtype, out,
                   lse, ws + bb, workspace_bytes - bb, stream, false);
  if (rc != AFFMAE_OK) return rc;
  const affmae::RelposArgs r = {coords, nbr_idx, rel_table, R, rate};
  if (affmae::launch_relpos_bias(r, B, N, H, K, dtype, ws, st) != hipSuccess) return AFFMAE_ERR_DEVICE;
  return pla_fwd_run(q, k, v, ws, nbr_idx, near_clusters, plan, k_blank, v_blank, B, N, H, d, K, S, M, scale, dtype, out,
                     lse, ws + bb, workspace_bytes - bb, stream, true);
}

size_t affmae_pla_bwd_relpos_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int R, int dtype,
                                             int clustered) {
  if (check_pla_shape(B, N, H, d, K, dtype) != AFFMAE_OK || R < 0 || R > 31) return 0;
  if (relpos_in_kernel(B, N, d, K, S, M, dtype, clustered)) {
    const size_t table = affmae::pla_bwd_cluster_rel_sums(R)
                             ? align_up(affmae::pla_bwd_cluster_rel_workspace_bytes(B, N, H, R))
                             : bias_bytes(B, N, H, K, dtype) + align_up(affmae::relpos_dtable_workspace_bytes(B, N, H, K, R));
    return table + align_up(affmae::pla_plan_bytes(B, N, K, S, M)) +
           align_up(affmae::pla_bwd_cluster_workspace_bytes(B, N, H, K, S, M));
  }
  return 2 * bias_bytes(B, N, H, K, dtype) + align_up(affmae::relpos_dtable_workspace_bytes(B, N, H, K, R)) +
         align_up(affmae_pla_bwd_workspace_bytes(B, N, H, d, K, S, M, dtype, clustered));
}

int affmae_pla_bwd_relpos(const void* q, const void* k, const void* v, const float* coords, const void* rel_table,
                          const int32_t* nbr_idx, const int32_t* near_clusters, const void* plan,
                          const void* k_blank, const void* v_blank, const void* out, const float* lse,
                          const void* dout, int B, int N, int H, int d, int K, int S, int M, float scale, int R,
                          float rate, int dtype, void* dq, void* dk, void* dv, float* drel_table, float* dk_blank,
                          float* dv_blank, void* workspace, size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !nbr_idx || !lse || !dout || !dq || !dk || !dv || !drel_table) return AFFMAE_ERR_NULL;
  int rc = check_pla_shape(B, N, H, d, K, dtype);
  if (rc != AFFMAE_OK) return rc;
  rc = check_relpos(coords, rel_table, B, N, H, K, R, rate);
  if (rc != AFFMAE_OK) return rc;
  const size_t bb = bias_bytes(B, N, H, K, dtype);
  const size_t tb = align_up(affmae::relpos_dtable_workspace_bytes(B, N, H, K, R));
  if (!workspace || workspace_bytes < affmae_pla_bwd_relpos_workspace_bytes(B, N, H, d, K, S, M, R, dtype,
                                                                             near_clusters != nullptr) ||
      misaligned(workspace, kAlign))
    return AFFMAE_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const affmae::RelposArgs r = {coords, nbr_idx, rel_table, R, rate};
  if (relpos_in_kernel(B, N, d, K, S, M, dtype, near_clusters != nullptr)) {
    // the tiled kernels look the bias up themselves; the table's gradient is summed in the query-stationary
    // kernel when the table fits its LDS, else dbias goes through the workspace to the stand-alone kernel
    if (!out) return AFFMAE_ERR_NULL;
    if ((k_blank == nullptr) != (v_blank == nullptr)) return AFFMAE_ERR_NULL;
    if ((dk_blank == nullptr) != (dv_blank == nullptr)) return AFFMAE_ERR_NULL;
    if (M > (N + S - 1) / S) return AFFMAE_ERR_SHAPE;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(dout, 16) || misaligned(dq, 16) ||
        misaligned(dk, 16) || misaligned(dv, 16) || misaligned(out, 16))
      return AFFMAE_ERR_SHAPE;
    if ((k_blank && misaligned(k_blank, 16)) || (v_blank && misaligned(v_blank, 16))) return AFFMAE_ERR_SHAPE;
    if (plan && misaligned(plan, kAlign)) return AFFMAE_ERR_WORKSPACE;
    affmae::PlaArgs a = {};
    a.q = q; a.k = k; a.v = v; a.nbr_idx = nbr_idx; a.near_clusters = near_clusters;
    a.k_blank = k_blank; a.v_blank = v_blank;
    a.B = B; a.N = N; a.H = H; a.d = d; a.K = K; a.S = S; a.M = M; a.scale = scale; a.dtype = dtype;
    a.out = const_cast<void*>(out); a.lse = const_cast<float*>(lse); a.dout = dout;
    a.dq = dq; a.dk = dk; a.dv = dv; a.dk_blank = dk_blank; a.dv_blank = dv_blank;
    a.rel_coords = coords; a.rel_table = rel_table; a.rel_R = R; a.rel_rate = rate;
    if (!affmae::pla_cluster_relpos_supported(a)) return AFFMAE_ERR_UNSUPPORTED;  // (the workspace is sized for this path)
    const bool sums = affmae::pla_bwd_cluster_rel_sums(R);
    size_t off = 0;
    void* parts = nullptr;
    if (sums) {
      a.rel_part = reinterpret_cast<float*>(ws);
      a.rel_dtable = drel_table;
      off += align_up(affmae::pla_bwd_cluster_rel_workspace_bytes(B, N, H, R));
    } else {
      a.dbias = ws;
      parts = ws + bb;
      off += bb + tb;
    }
    if (!plan) {
      if (affmae::launch_pla_plan(nbr_idx, near_clusters, B, N, K, S, M, ws + off, st) != hipSuccess)
        return AFFMAE_ERR_DEVICE;
      plan = ws + off;
    }
    off += align_up(affmae::pla_plan_bytes(B, N, K, S, M));
    if (affmae::launch_pla_bwd_cluster(a, plan, ws + off, st) != hipSuccess) return AFFMAE_ERR_DEVICE;
    if (!sums && affmae::launch_relpos_dtable(r, B, N, H, K, dtype, a.dbias, drel_table, parts, st) != hipSuccess)
      return AFFMAE_ERR_DEVICE;
    return AFFMAE_OK;
  }
  void* bias = ws;
  void* dbias = ws + bb;
  void* parts = ws + 2 * bb;
  char* inner = ws + 2 * bb + tb;
  // validate the attention call before the kernel that writes the bias
  rc = pla_bwd_run(q, k, v, bias, nbr_idx, near_clusters, plan, k_blank, v_blank, out, lse, dout, B, N, H, d, K, S, M,
                   scale, dtype, dq, dk, dv, dbias, dk_blank, dv_blank, inner, workspace_bytes - (2 * bb + tb), stream,
                   false);
  if (rc != AFFMAE_OK) return rc;
  if (affmae::launch_relpos_bias(r, B, N, H, K, dtype, bias, st) != hipSuccess) return AFFMAE_ERR_DEVICE;
  rc = pla_bwd_run(q, k, v, bias, nbr_idx, near_clusters, plan, k_blank, v_blank, out, lse, dout, B, N, H, d, K, S, M,
                   scale, dtype, dq, dk, dv, dbias, dk_blank, dv_blank, inner, workspace_bytes - (2 * bb + tb), stream,
                   true);
  if (rc != AFFMAE_OK) return rc;
  return affmae::launch_relpos_dtable(r, B, N, H, K, dtype, dbias, drel_table, parts, st) == hipSuccess
             ? AFFMAE_OK
             : AFFMAE_ERR_DEVICE;
}

}  // extern "C"
