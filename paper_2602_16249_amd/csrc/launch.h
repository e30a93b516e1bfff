// Internal launcher interface between the C-ABI translation unit and the
// kernel translation units.  Every launcher enqueues on `stream`, performs no
// synchronisation and returns the hipError_t of its last launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace affmae {

struct KnnArgs {
  const float* coords;        // [B,N,2]
  const int32_t* cluster_id;  // [B,N] or nullptr
  int B, N, S, M, K, G;
  int32_t* nbr_idx;        // [B,N,K]
  int32_t* near_clusters;  // [B,G,M] (never null here: points into workspace if the caller passed none)
  float* centroid;         // [B,G,2] workspace
  int32_t* members;        // [B,N] workspace, used only with cluster_id
};
hipError_t launch_knn(const KnnArgs& a, hipStream_t stream);

// Balanced clustering along a Z-order curve.
size_t cluster_workspace_bytes(int B, int N);
hipError_t launch_cluster(const float* coords, int B, int N, int S, double x0, double y0, double w, double h,
                          int32_t* order, int32_t* cluster_id, void* workspace, hipStream_t stream);

// Virtual sampled tokens of the point decoder: nearest-visible-token table over the patch grid, and the
// fused lookup / distance / softmax(-p d) / weighted feature sum, forward and backward.
struct VtsArgs {
  const float* query_xy;  // [B,Mq,2]
  const float* vis_xy;    // [B,Nv,2]
  const void* feat;       // [B,Nv,C]
  const int32_t* table;   // [B,Hg,Wg,Kt]
  const void* dout;       // [B,Mq,C]
  int B, Mq, Nv, C, Hg, Wg, Kt, dtype;
  float x0, y0, cell, p, eps;
  int32_t* table_out;     // table kernel only
  void* out;              // [B,Mq,C]
  void* dfeat;            // [B,Nv,C]
  float* dquery;          // [B,Mq,2]
  float* dp;              // device scalar or nullptr
  void* workspace;
};
hipError_t launch_vts_table(const VtsArgs& a, hipStream_t stream);
hipError_t launch_vts_fwd(const VtsArgs& a, hipStream_t stream);
size_t vts_bwd_workspace_bytes(int B, int Mq, int Nv, int Kt);
hipError_t launch_vts_bwd(const VtsArgs& a, hipStream_t stream);

// Building blocks shared by the gather-style backward passes (vts.hip): a sum of partial results in a fixed order,
// the filing of (query, candidate) pairs per token, and the per-token sum of weighted upstream rows.
size_t sum_parts_scratch_floats(size_t n);
hipError_t launch_sum_parts(const float* part, size_t n, float* part2, float* out, hipStream_t stream);
hipError_t launch_pair_lists(const int32_t* pair_token, int B, int Nv, int pairs_per_image, int32_t* offset,
                             int32_t* list, hipStream_t stream, const int32_t* group_bounds = nullptr,
                             int group_size = 0);
hipError_t launch_pair_gather(const void* dout, const float* weights, const int32_t* offset, const int32_t* list,
                              size_t tokens, int C, int Kt, int dtype, void* dfeat, bool pieces, hipStream_t stream,
                              const float* extra = nullptr, float* extra_sum = nullptr);

// Neighbourhood merging (merge.hip): anchor selection, location-aware aggregation, backward.
struct MergeArgs {
  const void* feat;           // [B,N,C]
  const float* coords;        // [B,N,2]
  const float* score;         // [B,N]
  const int32_t* nbr_idx;     // [B,N,K]
  const int32_t* anchor_idx;  // [B,n_keep]
  const void* dout;           // [B,n_keep,C]
  int B, N, C, K, n_keep, dtype;
  float p;
  void* out;      // [B,n_keep,C]
  void* dfeat;    // [B,N,C]
  float* dscore;  // [B,N]
  float* dp;      // device scalar or nullptr
  void* workspace;
};
hipError_t launch_merge_select(const float* score, const float* coords, int B, int N, int n_keep, int32_t* anchor_idx,
                               float* anchor_xy, hipStream_t stream);
hipError_t launch_merge_fwd(const MergeArgs& a, hipStream_t stream);
size_t merge_bwd_workspace_bytes(int B, int N, int K, int n_keep);
hipError_t launch_merge_bwd(const MergeArgs& a, hipStream_t stream);

// Relative-position bias from a per-head table over quantised offsets (relpos.hip).
struct RelposArgs {
  const float* coords;     // [B,N,2]
  const int32_t* nbr_idx;  // [B,N,K]
  const void* table;       // [H, 2R+1, 2R+1] in the storage type
  int R;
  float rate;              // bins per unit of length
};
hipError_t launch_relpos_bias(const RelposArgs& r, int B, int N, int H, int K, int dtype, void* bias,
                              hipStream_t stream);
size_t relpos_dtable_workspace_bytes(int B, int N, int H, int K, int R);
hipError_t launch_relpos_dtable(const RelposArgs& r, int B, int N, int H, int K, int dtype, const void* dbias,
                                float* dtable, void* workspace, hipStream_t stream);
// dtable[i] = sum over t < tables of part[t][i], i < entries
hipError_t launch_relpos_table_sum(const float* part, int tables, int entries, float* dtable, hipStream_t stream);

struct PlaArgs {
  const void *q, *k, *v, *bias;
  const int32_t* nbr_idx;
  const int32_t* near_clusters;
  const void *k_blank, *v_blank;
  int B, N, H, d, K, S, M;
  float scale;
  int dtype;
  // bias from a relative-position table instead of `bias` (tiled kernels only; null otherwise)
  const float* rel_coords;  // [B,N,2]
  const void* rel_table;    // [H, 2R+1, 2R+1] in the storage type
  int rel_R;
  float rel_rate;
  float* rel_part;    // backward: workspace of pla_bwd_cluster_rel_workspace_bytes, or null (then dbias is written)
  float* rel_dtable;  // backward, with rel_part: [H, 2R+1, 2R+1] gradient of the table
  // forward outputs / backward inputs
  void* out;
  float* lse;
  // backward only
  const void* dout;
  void *dq, *dk, *dv, *dbias;
  float *dk_blank, *dv_blank;
  void* workspace;
};
hipError_t launch_pla_fwd_general(const PlaArgs& a, hipStream_t stream);
hipError_t launch_pla_bwd_general(const PlaArgs& a, hipStream_t stream);
size_t pla_bwd_general_workspace_bytes(int B, int N, int H, int K);

// Cluster-tiled kernels (bf16, d = 32, cluster promise given), driven by a plan.
bool pla_cluster_supported(const PlaArgs& a);
bool pla_cluster_relpos_supported(const PlaArgs& a);  // ... and able to take the bias from a.rel_table themselves
size_t pla_plan_bytes(int B, int N, int K, int S, int M);
hipError_t launch_pla_plan(const int32_t* nbr_idx, const int32_t* near, int B, int N, int K, int S, int M, void* plan,
                           hipStream_t stream);
hipError_t launch_pla_fwd_cluster(const PlaArgs& a, const void* plan, hipStream_t stream);
size_t pla_bwd_cluster_workspace_bytes(int B, int N, int H, int K, int S, int M);
bool pla_bwd_cluster_rel_sums(int R);  // the table is small enough for the backward kernel to sum its gradient itself
size_t pla_bwd_cluster_rel_workspace_bytes(int B, int N, int H, int R);
hipError_t launch_pla_bwd_cluster(const PlaArgs& a, const void* plan, void* workspace, hipStream_t stream);

}  // namespace affmae
