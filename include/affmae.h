/*
 * affmae.h - C ABI of the MI355X (gfx950) neighbourhood-attention library.
 *
 * The library implements the data-parallel hot path of AFFMAE's off-grid
 * hierarchical backbone: balanced clustering of the tokens along a space-filling
 * curve, the batched neighbour search that builds fixed-size neighbourhoods over
 * irregular 2-D token coordinates, local attention, forward and backward, over
 * each token's K neighbours, the neighbourhood merging that downsamples the token
 * set between stages, and the point decoder's virtual sampled tokens.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     never allocates, frees or keeps them.  Tensors are dense, row-major, in
 *     the shapes stated below.  B = images, N = tokens per image, H = heads,
 *     d = channels per head, K = neighbours per token, S = tokens per cluster,
 *     G = ceil(N / S) clusters per image, M = clusters searched per cluster.
 *   - Token and cluster indices are per image (0..N-1, 0..G-1), int32.
 *   - `workspace` is caller-owned device scratch of at least the number of
 *     bytes the matching *_workspace_bytes() call returns (256-byte aligned);
 *     its contents are undefined before and after a call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls validate their arguments on the host, enqueue kernels on `stream`
 *     and return without synchronising.  Calls that share a workspace must be
 *     ordered on one stream.  No call allocates, frees or clears device memory
 *     through the runtime: a caller may record the calls into a HIP graph.
 *     The library keeps no state between calls (the one exception is the fixed
 *     scratch array of affmae_knn_static) and may be called from several threads.
 *   - Return value: AFFMAE_OK (0) or a negative affmae_status.  When an error
 *     is returned nothing has been enqueued.  No exception crosses the ABI.
 *   - Outputs are fully overwritten (never accumulated into).
 *   - The host cannot see tensor contents.  Index values outside their range
 *     (cluster_id, nbr_idx, near_clusters) never cause out-of-bounds accesses,
 *     but the results for the affected tokens are unspecified.
 */
#ifndef AFFMAE_H_
#define AFFMAE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AFFMAE_OK = 0,
  AFFMAE_ERR_NULL = -1,        /* a required pointer is NULL                     */
  AFFMAE_ERR_SHAPE = -2,       /* a size is non-positive or inconsistent         */
  AFFMAE_ERR_DTYPE = -3,       /* unknown storage type                           */
  AFFMAE_ERR_WORKSPACE = -4,   /* workspace missing, too small or misaligned     */
  AFFMAE_ERR_UNSUPPORTED = -5, /* valid request outside the implemented limits   */
  AFFMAE_ERR_DEVICE = -6       /* the HIP runtime refused a launch               */
} affmae_status;

typedef enum { AFFMAE_F32 = 0, AFFMAE_BF16 = 1 } affmae_dtype;

/* Implemented limits (AFFMAE_ERR_UNSUPPORTED beyond them). */
#define AFFMAE_MAX_K 64          /* neighbours per token                         */
#define AFFMAE_MAX_NEAR 64       /* M, clusters searched per cluster             */

/* Human-readable name of a status code; never NULL. */
const char* affmae_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int affmae_version(void);

/* Digest of the sources the library was built from (hex string, never NULL;
 * "unstamped" when built without the package's build script).  Stored profiles
 * carry it so that a reader can tell whether they describe this build. */
const char* affmae_build_id(void);

/*
 * affmae_cluster - balanced clustering (paper, Sec. "AutoFocusFormer": tokens
 * are grouped into equal-size clusters by a space-filling-curve procedure).
 * The paper does not name the curve; this library orders the tokens of an image
 * along the Z-order (Morton) curve of a caller-given frame and cuts the order
 * into consecutive clusters of S tokens (the last one is smaller when S does
 * not divide N).  A coordinate is quantised in double precision to
 * floor((x - x0) / w * 65536) clamped to 0..65535 (likewise y with y0, h); the
 * key of a token interleaves the two 16-bit values, x in the even bits; tokens
 * are ordered by (key, token index), so the result is unique.
 *
 *   coords      in  [B,N,2] fp32 (x, y), finite
 *   x0,y0,w,h   the frame [x0, x0+w) x [y0, y0+h), w, h > 0; points outside it
 *               fall into its border cells
 *   order       out [B,N] int32: order[b][p] = the token at place p of the curve.
 *               Gathering every per-token tensor with it puts the tokens in
 *               cluster order, the layout affmae_knn takes with cluster_id = NULL
 *               and the tiled attention kernels need.
 *   cluster_id  out [B,N] int32 or NULL: the cluster of every token of the
 *               original order (its place / S); usable as affmae_knn's
 *               cluster_id when S divides N.
 *   workspace   affmae_cluster_workspace_bytes(B, N) bytes
 *
 * Errors: AFFMAE_ERR_NULL (coords, order), AFFMAE_ERR_SHAPE (B, N, S < 1; empty
 * or non-finite frame), AFFMAE_ERR_UNSUPPORTED (N > 2^24), AFFMAE_ERR_WORKSPACE.
 */
size_t affmae_cluster_workspace_bytes(int B, int N);
int affmae_cluster(const float* coords, int B, int N, int S, double x0, double y0, double w, double h,
                   int32_t* order, int32_t* cluster_id, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Virtual sampled tokens of the point decoder (paper, Sec. "AFFMAE": a decoder
 * query location q gathers the K nearest visible tokens and aggregates their
 * features with the exponential distance kernel
 *     d_i = |q - x_i| + eps,  w_i = softmax_i(-p d_i),  out = sum_i w_i feat_i;
 * Sec. "Flash-style Cluster Attention and Fast Decoder KNN" and supplement
 * "Point-based decoder": the nearest visible tokens are not searched per query
 * but read from a table cached over the dense Hg x Wg patch grid, the query
 * being rounded to its nearest grid point; lookup, distances, weights and the
 * weighted sum are one kernel).
 *
 * Grid: point (ix, iy) is the patch centre (x0 + (ix + 1/2) cell, y0 + (iy + 1/2)
 * cell), evaluated in fp32 one operation at a time; the nearest grid point of q
 * is the cell that contains it, floor((q.x - x0) / cell) in fp32 clamped to
 * 0..Wg-1 (likewise y), so queries outside the grid use its border cells.
 *
 * affmae_vts_table  table[b][iy][ix][0..Kt-1] = the Kt visible tokens of image b
 *                   nearest to grid point (ix, iy), ascending (fp32 squared
 *                   distance evaluated as in affmae_knn, token index).  Built once
 *                   per mask and reused by every decoder block.
 *   vis_xy  in  [B,Nv,2] fp32, finite       table  out [B,Hg,Wg,Kt] int32
 *
 * affmae_vts_fwd
 *   query_xy in [B,Mq,2] fp32   feat in [B,Nv,C] dtype   out [B,Mq,C] dtype
 *   (several sample points per decoder query are simply more rows of query_xy)
 *
 * affmae_vts_bwd    gradients of L = <dout, out>:
 *   dfeat   out [B,Nv,C] dtype, fully overwritten (summed in fp32 per token over
 *           the queries that use it; the order of the additions, hence the last
 *           bits, may vary run to run)
 *   dquery  out [B,Mq,2] fp32: sum_i dz_i (-p) (q - x_i) / |q - x_i| with
 *           dz_i = w_i (<dout, feat_i> - sum_j w_j <dout, feat_j>); a candidate
 *           that coincides with q contributes no direction
 *   dp      out device scalar fp32 or NULL: sum over all queries of
 *           sum_i dz_i (-(|q - x_i| + eps))
 *   workspace  affmae_vts_bwd_workspace_bytes(B, Mq, Nv, Kt) bytes
 *
 * Limits: 1 <= Kt <= min(Nv, AFFMAE_MAX_K); C even; feat, out, dout, dfeat
 * 4-byte aligned; B*Hg*Wg, B*Mq, B*Nv and (backward) B*Mq*Kt below 2^31 - 8
 * (AFFMAE_ERR_UNSUPPORTED otherwise).  Table entries outside 0..Nv-1 are clamped.
 * The fastest kernels need rows of whole 16-byte pieces (C a multiple of 8 for
 * bf16, of 4 for fp32), 16-byte aligned feature tensors and 8-byte aligned
 * coordinate tensors; other shapes are served by slower kernels, same results.
 * Errors: AFFMAE_ERR_NULL, AFFMAE_ERR_SHAPE (sizes < 1, Kt > Nv, empty or
 * non-finite grid, misaligned tensor), AFFMAE_ERR_DTYPE, AFFMAE_ERR_UNSUPPORTED,
 * AFFMAE_ERR_WORKSPACE.
 */
int affmae_vts_table(const float* vis_xy, int B, int Nv, int Hg, int Wg, float x0, float y0, float cell, int Kt,
                     int32_t* table, void* stream);
int affmae_vts_fwd(const float* query_xy, const float* vis_xy, const void* feat, const int32_t* table, int B, int Mq,
                   int Nv, int C, int Hg, int Wg, float x0, float y0, float cell, int Kt, float p, float eps,
                   int dtype, void* out, void* stream);
size_t affmae_vts_bwd_workspace_bytes(int B, int Mq, int Nv, int Kt);
int affmae_vts_bwd(const float* query_xy, const float* vis_xy, const void* feat, const int32_t* table,
                   const void* dout, int B, int Mq, int Nv, int C, int Hg, int Wg, float x0, float y0, float cell,
                   int Kt, float p, float eps, int dtype, void* dfeat, float* dquery, float* dp, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * Neighbourhood merging (paper, Sec. "AutoFocusFormer": after several local-
 * attention blocks the token set is downsampled; an importance score is learned
 * per token by a one-layer MLP, the top-ranked share d_s of the tokens is kept as
 * anchors, and the remaining tokens are merged into nearby anchors through a
 * differentiable, location-aware aggregation; supplement "AFF architecture": a
 * linear projection follows every merging block).  The paper leaves the operator
 * to the AFF paper; this library takes the following form.  The score layer and
 * the projection are the caller's dense layers.
 *
 * affmae_merge_select  anchors of every image: the n_keep (= d_s N) tokens with the
 *                      largest score, equal scores (-0 and +0 are equal) going to
 *                      the lower token index, listed in ascending token index -
 *                      tokens stored in curve order stay in curve order, so the
 *                      next stage's clusters are again consecutive runs.
 *   score      in  [B,N] fp32, finite      coords     in  [B,N,2] fp32 or NULL
 *   anchor_idx out [B,n_keep] int32        anchor_xy  out [B,n_keep,2] fp32 or NULL:
 *                      the anchors' coordinates, which the merged tokens keep
 *                      (coords and anchor_xy aligned to 8 bytes when both are given)
 *
 * affmae_merge_fwd     out[b,a,:] = sum_j w_j feat[b, n(t,j), :] over the K tokens
 *                      n(t,j) of the neighbourhood of the anchor's token t =
 *                      anchor_idx[b,a] (row t of nbr_idx, the token itself among
 *                      them), w_j = softmax_j(score[b,n(t,j)] - p |x_n(t,j) - x_t|),
 *                      distances in fp32.  A token in no anchor's neighbourhood is
 *                      dropped; one in several contributes to each.
 *   feat   in [B,N,C] dtype     nbr_idx in [B,N,K] int32 (values clamped to 0..N-1)
 *   out    out [B,n_keep,C] dtype, fp32 sums, round to nearest even
 *
 * affmae_merge_bwd     gradients of L = <dout, out>, with g_j = <dout[b,a,:],
 *                      feat[b,n(t,j),:]> and dz_j = w_j (g_j - sum_i w_i g_i):
 *   dfeat  out [B,N,C] dtype: sum over the (anchor, j) pairs with n(t,j) = the token
 *                      of w_j dout[b,a,:] (fp32 sums; 0 for tokens no anchor uses)
 *   dscore out [B,N] fp32: the same sum of dz_j - the gradient that trains the score
 *   dp     out device scalar fp32 or NULL: sum over all pairs of dz_j (-|x_n - x_t|)
 *   workspace  affmae_merge_bwd_workspace_bytes(B, N, K, n_keep) bytes
 *   (the order of the additions into dfeat and dscore, hence their last bits, may
 *   vary from run to run)
 *
 * Limits: 1 <= K <= AFFMAE_MAX_K, 1 <= n_keep <= N <= 2^24, 0 <= p finite, B*N and
 * B*n_keep*K below 2^31 - 8; coords 8-byte aligned.  Rows that are whole 16-byte
 * pieces (C a multiple of 8 for bf16, of 4 for fp32) in 16-byte aligned tensors run
 * the fast kernels, other shapes slower ones, same results.
 * Errors: AFFMAE_ERR_NULL, AFFMAE_ERR_SHAPE, AFFMAE_ERR_DTYPE, AFFMAE_ERR_UNSUPPORTED,
 * AFFMAE_ERR_WORKSPACE.
 */
int affmae_merge_select(const float* score, const float* coords, int B, int N, int n_keep, int32_t* anchor_idx,
                        float* anchor_xy, void* stream);
int affmae_merge_fwd(const void* feat, const float* coords, const float* score, const int32_t* nbr_idx,
                     const int32_t* anchor_idx, int B, int N, int C, int K, int n_keep, float p, int dtype, void* out,
                     void* stream);
size_t affmae_merge_bwd_workspace_bytes(int B, int N, int K, int n_keep);
int affmae_merge_bwd(const void* feat, const float* coords, const float* score, const int32_t* nbr_idx,
                     const int32_t* anchor_idx, const void* dout, int B, int N, int C, int K, int n_keep, float p,
                     int dtype, void* dfeat, float* dscore, float* dp, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * affmae_knn - neighbourhood construction (paper, Sec. "AutoFocusFormer":
 * tokens are grouped into equal-size clusters and every token gets a
 * fixed-size neighbourhood by nearest-neighbour search over 2-D coordinates;
 * the table is built once per encoder stage and reused, Sec. "Limitations").
 *
 *   coords        in  [B,N,2] fp32 (x,y), finite.
 *   cluster_id    in  [B,N] int32 with every cluster holding exactly S tokens
 *                     (the last one, cluster G-1, the N - (G-1) S that are left
 *                     when S does not divide N), or NULL meaning
 *                     cluster_id[b,i] = i / S (tokens stored in cluster order).
 *   B,N,S,M,K         G = ceil(N / S) clusters; 1 <= M <= min(G, AFFMAE_MAX_NEAR);
 *                     1 <= K <= AFFMAE_MAX_K, and K at most the smallest candidate
 *                     set any token can have, (M-1) S + N - (G-1) S (= M*S when S
 *                     divides N); M*S <= 4096.  M == G is exact kNN.
 *   nbr_idx       out [B,N,K]: the K nearest tokens among the members of the M
 *                     clusters nearest to the token's own cluster, ascending in
 *                     (distance, token index).  The token itself takes part.
 *   near_clusters out [B,G,M] or NULL: the M clusters with nearest centroids,
 *                     ascending in (distance, cluster index), the cluster
 *                     itself included.
 *
 * Arithmetic is fixed so that results are unique: distance is the fp32 value
 * fl(fl(dx*dx) + fl(dy*dy)) with dx = fl(ax-bx), dy = fl(ay-by) (no fused
 * multiply-add, no square root); a centroid is the fp32 rounding of the
 * double-precision mean of the members summed in ascending token order.
 */
size_t affmae_knn_workspace_bytes(int B, int N, int S, int M, int K);
int affmae_knn(const float* coords, const int32_t* cluster_id, int B, int N, int S, int M, int K,
               int32_t* nbr_idx, int32_t* near_clusters, void* workspace, size_t workspace_bytes,
               void* stream);

/*
 * affmae_knn_static - affmae_knn for callers that cannot allocate device memory
 * or size a workspace (code recorded into a HIP graph by a harness that forbids
 * allocation, tight serving loops): the same search, same arguments and results,
 * with the scratch (centroids, the near-cluster table when near_clusters is NULL,
 * member lists) in a fixed array of AFFMAE_KNN_STATIC_SCRATCH_BYTES inside the
 * library's device image.  Each GPU the library runs on holds one copy of that
 * array until the process ends.  The call allocates and frees nothing.
 *
 * Errors: as affmae_knn, with AFFMAE_ERR_WORKSPACE when
 * affmae_knn_workspace_bytes(B, N, S, M, K) exceeds AFFMAE_KNN_STATIC_SCRATCH_BYTES
 * (about B * (N * 4 + G * (8 + 4 M)) bytes: a million tokens fit), and
 * AFFMAE_ERR_DEVICE when the runtime cannot give the array's address.
 * All calls on one GPU share the array: calls that may overlap in time (on
 * different streams, or from different threads) race; order them on one stream.
 */
#define AFFMAE_KNN_STATIC_SCRATCH_BYTES (4u << 20)
int affmae_knn_static(const float* coords, const int32_t* cluster_id, int B, int N, int S, int M, int K,
                      int32_t* nbr_idx, int32_t* near_clusters, void* stream);

/*
 * affmae_pla_plan - re-tiles a clustered neighbour table for the cluster-tiled
 * attention kernels (paper, Sec. "Limitations": neighbourhood tables are cached
 * per encoder stage; the plan is that cache in the layout the tiled kernels read,
 * built once per table and passed to every forward and backward call that uses
 * the table).  Optional: without a plan the attention calls rebuild it in their
 * workspace on every call.
 *
 *   nbr_idx, near_clusters  in  as produced by affmae_knn with cluster_id == NULL
 *                               (the promise described under affmae_pla_fwd).
 *   plan                    out caller-owned device buffer of affmae_pla_plan_bytes()
 *                               bytes, 256-byte aligned; opaque.
 * affmae_pla_plan_bytes returns 0, and affmae_pla_plan AFFMAE_ERR_UNSUPPORTED,
 * when the shapes are outside what the tiled kernels take (they need S % 16 == 0
 * - S need not divide N, nor 16: the last cluster, strip and token tile of an
 * image may be short -, M*S <= 1024, N < 2^20 and N*S < 2^31); the attention calls then use the gather
 * kernels and ignore `plan`.
 */
size_t affmae_pla_plan_bytes(int B, int N, int K, int S, int M);
int affmae_pla_plan(const int32_t* nbr_idx, const int32_t* near_clusters, int B, int N, int K, int S,
                    int M, void* plan, size_t plan_bytes, void* stream);

/*
 * affmae_pla_fwd - local attention over each token's neighbourhood (paper,
 * Sec. "Flash-style Cluster Attention and Fast Decoder KNN", the FlashNbhdAttn
 * equation): for every image b, token i and head h
 *     s_j   = scale * <q[b,i,h,:], k[b,n(i,j),h,:]> + bias[b,i,h,j]   (j < K)
 *     s_K   = scale * <q[b,i,h,:], k_blank[h,:]>                      (if given)
 *     p     = softmax(s)
 *     out[b,i,h,:] = sum_j p_j v[b,n(i,j),h,:]  (+ p_K v_blank[h,:])
 *     lse[b,i,h]   = log(sum_j exp(s_j))
 * computed without storing the score matrix, with fp32 softmax statistics and
 * accumulators whatever the storage type.
 *
 *   q,k,v         in  [B,N,H,d] of `dtype`.
 *   bias          in  [B,N,H,K] of `dtype`, or NULL (= 0): one row of K values per
 *                     (token, head), in the order of the token's neighbour list.
 *   nbr_idx       in  [B,N,K] int32, values in [0,N); it need not come from
 *                     affmae_knn and may list a token more than once (each
 *                     slot is its own softmax column) unless near_clusters is
 *                     given.
 *   near_clusters in  [B,G,M] int32 or NULL.  Non-NULL is a promise that
 *                     tokens are stored in cluster order (cluster = i / S),
 *                     that every neighbour of a token of cluster c lies in one
 *                     of near_clusters[b,c,:], and that a token's neighbours
 *                     are pairwise distinct - what affmae_knn produces with
 *                     cluster_id == NULL.  It allows the cluster-tiled kernels
 *                     (bf16 storage, d == 32, S % 16 == 0, any N,
 *                     M*S <= 1024; other shapes, head sizes 16 and 64 among them,
 *                     are served by the slower gather kernels, same results);
 *                     inputs must then be finite.  With NULL, S and M are ignored.
 *   plan          in  NULL, or the buffer affmae_pla_plan filled for this
 *                     nbr_idx / near_clusters and these B,N,K,S,M.
 *   k_blank,v_blank in [H,d] of `dtype`, or both NULL.
 *   d                 16, 32 or 64.  1 <= K <= AFFMAE_MAX_K.
 *   out           out [B,N,H,d] of `dtype` (round to nearest even).
 *   lse           out [B,N,H] fp32.
 */
size_t affmae_pla_fwd_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int dtype,
                                      int clustered);
int affmae_pla_fwd(const void* q, const void* k, const void* v, const void* bias,
                   const int32_t* nbr_idx, const int32_t* near_clusters, const void* plan,
                   const void* k_blank, const void* v_blank, int B, int N, int H, int d, int K, int S,
                   int M, float scale, int dtype, void* out, float* lse, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * affmae_pla_bwd - gradients of affmae_pla_fwd (the paper trains through the
 * attention but prints no backward; this is the chain rule on the equation
 * above).  With p recomputed from lse and g = dout:
 *     dP_j = <g[b,i,h,:], v_j>,  D = sum_j p_j dP_j,  dS_j = p_j (dP_j - D)
 *     dbias[b,i,h,j]  = dS_j
 *     dq[b,i,h,:]     = scale * sum_j dS_j k_j
 *     dk[b,n(i,j),h,:] += scale * dS_j q[b,i,h,:]
 *     dv[b,n(i,j),h,:] += p_j g[b,i,h,:]
 *     dk_blank[h,:]   = scale * sum_{b,i} dS_K q[b,i,h,:]
 *     dv_blank[h,:]   = sum_{b,i} p_K g[b,i,h,:]
 *
 *   inputs as affmae_pla_fwd, plus
 *   out           in  [B,N,H,d] of `dtype`: forward output.  Required by the
 *                     cluster-tiled kernels (they take D = <dout, out>); the
 *                     gather kernels rebuild D from p and dP and accept NULL.
 *   lse           in  [B,N,H] fp32 from the forward call.
 *   dout          in  [B,N,H,d] of `dtype`.
 *   dq,dk,dv      out [B,N,H,d] of `dtype`; sums are formed in fp32.  The order
 *                     of the additions into dk/dv may differ between runs.
 *   dbias         out [B,N,H,K] of `dtype`, or NULL to skip.
 *   dk_blank,dv_blank out [H,d] fp32, or NULL (both required when blanks given
 *                     and their gradients are wanted).
 *   workspace     always required (affmae_pla_bwd_workspace_bytes); the gather
 *                     kernels number the (query, slot) pairs in 32 bits:
 *                     B*N*K < 2^31, else AFFMAE_ERR_UNSUPPORTED.
 */
size_t affmae_pla_bwd_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int dtype,
                                      int clustered);
int affmae_pla_bwd(const void* q, const void* k, const void* v, const void* bias,
                   const int32_t* nbr_idx, const int32_t* near_clusters, const void* plan,
                   const void* k_blank, const void* v_blank, const void* out, const float* lse,
                   const void* dout, int B, int N, int H, int d, int K, int S, int M, float scale,
                   int dtype, void* dq, void* dk, void* dv, void* dbias, float* dk_blank,
                   float* dv_blank, void* workspace, size_t workspace_bytes, void* stream);

/*
 * affmae_pla_fwd_relpos / affmae_pla_bwd_relpos - local attention whose bias is
 * derived inside the library from the token coordinates (paper, Sec.
 * "AutoFocusFormer": within a neighbourhood, attention uses relative position
 * derived directly from the 2-D token coordinates; it is the term B_n of the
 * FlashNbhdAttn equation).  The paper gives no function for it; this library
 * takes a learned table per head over quantised offsets:
 *     B[b,i,h,j] = rel_table[h][by][bx],
 *     bx = clamp(rint((x_n - x_i) * rate), -R, R) + R,  by alike with y,
 * n = nbr_idx[b,i,j]; the offset, the product and the rounding (to nearest, ties
 * to even) are fp32.  The blank column has no bias.  Everything else is as in
 * affmae_pla_fwd / affmae_pla_bwd, whose argument lists these calls follow with
 * `bias` replaced by (coords, rel_table, R, rate) and `dbias` by drel_table.
 *
 * With the cluster promise, bf16, d = 32 and K a multiple of 8 the tiled kernels
 * compute the bias themselves (the coordinates of the token tiles a strip
 * touches are staged in LDS, a cell per (query, neighbour) pair, the value
 * through the cache): no bias or dbias tensor exists, and for tables of at most
 * 128 cells per head (R <= 5) the gradient of the table is summed inside the
 * backward kernel as well.  In every other case the bias is written into the
 * workspace by a kernel of its own and the table's gradient is reduced from
 * dbias by another; the results are the same.
 *
 *   coords      in  [B,N,2] fp32, 8-byte aligned
 *   rel_table   in  [H, 2R+1, 2R+1] in the storage type (row = y bin)
 *   R           bins on each side of zero, 0 <= R <= 31, H*(2R+1)^2 <= 12288
 *   rate        bins per unit of length (> 0), e.g. 1/8 for bins of one 8-px patch
 *   drel_table  out [H, 2R+1, 2R+1] fp32: the bias gradients added up per bin
 *               (fp32 sums; the order of the additions inside a workgroup's
 *               share, hence the last bits, may vary run to run)
 *   workspace   affmae_pla_fwd_relpos_workspace_bytes / affmae_pla_bwd_relpos_workspace_bytes
 *
 * Errors: as affmae_pla_fwd / affmae_pla_bwd, plus AFFMAE_ERR_SHAPE for a negative
 * R or a rate that is not positive and finite, AFFMAE_ERR_UNSUPPORTED beyond the
 * limits of R.
 */
size_t affmae_pla_fwd_relpos_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int dtype,
                                             int clustered);
int affmae_pla_fwd_relpos(const void* q, const void* k, const void* v, const float* coords, const void* rel_table,
                          const int32_t* nbr_idx, const int32_t* near_clusters, const void* plan,
                          const void* k_blank, const void* v_blank, int B, int N, int H, int d, int K, int S, int M,
                          float scale, int R, float rate, int dtype, void* out, float* lse, void* workspace,
                          size_t workspace_bytes, void* stream);
size_t affmae_pla_bwd_relpos_workspace_bytes(int B, int N, int H, int d, int K, int S, int M, int R, int dtype,
                                             int clustered);
int affmae_pla_bwd_relpos(const void* q, const void* k, const void* v, const float* coords, const void* rel_table,
                          const int32_t* nbr_idx, const int32_t* near_clusters, const void* plan,
                          const void* k_blank, const void* v_blank, const void* out, const float* lse,
                          const void* dout, int B, int N, int H, int d, int K, int S, int M, float scale, int R,
                          float rate, int dtype, void* dq, void* dk, void* dv, float* drel_table, float* dk_blank,
                          float* dv_blank, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AFFMAE_H_ */
