/*
 * CPU oracle for the neighbourhood-attention hot path of AFFMAE.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product may call it: only the tests,
 * the smoke check and the benchmark's cpu-baseline leg do.
 *
 * What it follows:
 *   - neighbourhood construction: Sec. "AutoFocusFormer" (tokens carry a 2-D
 *     coordinate, are grouped into equal-size clusters, and every token gets a
 *     fixed-size neighbourhood by nearest-neighbour search over coordinates);
 *   - local attention: the FlashNbhdAttn equation of Sec. "Flash-style Cluster
 *     Attention and Fast Decoder KNN":
 *         softmax(Q_n [K_n K_blank]^T + B_n) [V_n V_blank]
 *     written out per token and head, in double precision, with no tiling;
 *   - backward: the chain rule applied to that equation (the paper does not
 *     print it).
 *
 * Readings taken where the paper is silent (each is listed in the design notes):
 *   - distance = squared Euclidean distance evaluated in fp32 as
 *     fl(fl(dx*dx) + fl(dy*dy)), dx = fl(ax-bx), dy = fl(ay-by); no fused
 *     multiply-add, no square root;
 *   - order = lexicographic (distance, index), lower wins; lists ascending;
 *   - "nearest clusters" = by distance between cluster centroids, a centroid
 *     being the fp32 rounding of the double-precision mean of the members taken
 *     in ascending token order; the cluster itself is included;
 *   - a token is a candidate for its own neighbourhood;
 *   - an explicit logit scale multiplies Q K^T; the blank column has no bias;
 *   - virtual sampled tokens of the point decoder (oracle_vts_*): Sec.
 *     "AFFMAE" (the exponential distance kernel softmax_i(-p d_i), d_i =
 *     |q - x_i| + eps, and the weighted sum of the K nearest visible tokens'
 *     features) and Sec. "Flash-style Cluster Attention and Fast Decoder KNN" /
 *     supplement "Point-based decoder" (a cached table over the dense patch grid
 *     holds, per grid point, the nearest visible tokens; a query is rounded to
 *     its nearest grid point and takes that entry).  Readings: grid points are
 *     the patch centres x0 + (ix + 1/2) cell evaluated in fp32; "nearest grid
 *     point" = the cell that contains the query, floor((qx - x0) / cell) in
 *     fp32, clamped to the grid; the table orders by (fp32 squared distance,
 *     token index) like the neighbour search; the table stores indices only;
 *   - relative-position bias (oracle_relpos_bias / oracle_relpos_dtable): the
 *     paper states that the bias of a neighbourhood is derived from the relative
 *     positions of its tokens and gives no function; reading: a learned table
 *     per head over quantised offsets, bias = table[h][by][bx] with bx = the
 *     offset x_neighbour - x_query times a bin rate, rounded to the nearest
 *     integer (ties to even) in fp32 and clamped to -R..R, plus R; by alike.
 *     The gradient of the table adds up the bias gradients that fall in a bin;
 *   - balanced clustering (oracle_cluster): the paper groups tokens into
 *     equal-size clusters with a space-filling curve it does not name; reading:
 *     Z-order (Morton) curve over coordinates quantised to 16 bits per axis of a
 *     caller-given frame, x in the even key bits, ties by token index, clusters
 *     = consecutive runs of S tokens along the curve (the last may be short);
 *   - neighbourhood merging (oracle_merge_*): Sec. "AutoFocusFormer", the paragraph
 *     on downsampling (a learned importance score per token, the top share d_s of
 *     the tokens kept as anchors, the rest merged into nearby anchors by a
 *     differentiable, location-aware aggregation; the anchors keep their
 *     coordinates); the paper leaves the operator to the AFF paper.  Readings:
 *     the score is an input (the one-layer MLP is the caller's layer); the
 *     n_keep = d_s N tokens with the largest score are the anchors, equal scores
 *     going to the lower index, listed in ascending token index (which keeps the
 *     curve order); an anchor aggregates the K tokens of its own neighbourhood
 *     (itself among them) with the weights softmax_j(score_j - p |x_j - x_anchor|);
 *     the merged token carries the weighted sum of their features and the
 *     anchor's coordinates;
 *
 * Parity pins (tests/test_oracle_*.py): brute force over all pairs with a
 * library sort, hand-derived grid fixtures, exact integer arithmetic on integer
 * coordinates, dense masked softmax attention built from library matmuls,
 * reverse-mode autodiff of that dense form, central finite differences, and
 * the invariants of softmax.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_CLUSTER (-2)
#define ORACLE_ERR_ALLOC (-3)

/* Number of threads the image-parallel loops will use (1 without OpenMP). */
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* fp32 squared distance, every operation rounded on its own. */
static float dist2_f32(float ax, float ay, float bx, float by) {
  float dx = ax - bx;
  float dy = ay - by;
  float xx = dx * dx;
  float yy = dy * dy;
  return xx + yy;
}

typedef struct {
  float d2;
  int32_t idx;
} cand_t;

static int cand_less(const void *pa, const void *pb) {
  const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
  if (a->d2 < b->d2) return -1;
  if (a->d2 > b->d2) return 1;
  if (a->idx < b->idx) return -1;
  if (a->idx > b->idx) return 1;
  return 0;
}

/*
 * Clusters hold S tokens each, except that the last one (cluster G - 1, G = ceil(N / S)) holds the
 * N - (G - 1) S tokens that are left when S does not divide N.
 */
static int cluster_count(int N, int S) { return (N + S - 1) / S; }
static int cluster_size(int c, int N, int S) {
  int G = cluster_count(N, S);
  return c == G - 1 ? N - (G - 1) * S : S;
}

/*
 * Member lists of one image.  cluster_id == NULL means token i belongs to
 * cluster i / S.  members[c*S + r] = r-th token of cluster c in ascending token
 * order (members has room for G*S entries).  Fails unless every cluster has exactly its size in members.
 */
static int build_members(const int32_t *cluster_id, int N, int S, int32_t *members) {
  int G = cluster_count(N, S);
  int *count = (int *)calloc((size_t)G, sizeof(int));
  if (!count) return ORACLE_ERR_ALLOC;
  int rc = ORACLE_OK;
  for (int i = 0; i < N && rc == ORACLE_OK; ++i) {
    int c = cluster_id ? cluster_id[i] : i / S;
    if (c < 0 || c >= G || count[c] >= cluster_size(c, N, S)) {
      rc = ORACLE_ERR_CLUSTER;
      break;
    }
    members[(size_t)c * S + count[c]++] = i;
  }
  for (int c = 0; c < G && rc == ORACLE_OK; ++c)
    if (count[c] != cluster_size(c, N, S)) rc = ORACLE_ERR_CLUSTER;
  free(count);
  return rc;
}

/* Centroid of each cluster: double sum in member order, divide by the number of members, round to fp32. */
static void image_centroids(const float *coords, const int32_t *members, int N, int S, float *centroid) {
  int G = cluster_count(N, S);
  for (int c = 0; c < G; ++c) {
    double sx = 0.0, sy = 0.0;
    int size = cluster_size(c, N, S);
    for (int r = 0; r < size; ++r) {
      int i = members[(size_t)c * S + r];
      sx += (double)coords[2 * (size_t)i + 0];
      sy += (double)coords[2 * (size_t)i + 1];
    }
    centroid[2 * c + 0] = (float)(sx / (double)size);
    centroid[2 * c + 1] = (float)(sy / (double)size);
  }
}

/*
 * oracle_centroids: coords [B,N,2] fp32, cluster_id [B,N] or NULL
 *   -> centroid [B,G,2] fp32, G = ceil(N/S) (the last cluster is short when S does not divide N).
 */
int oracle_centroids(const float *coords, const int32_t *cluster_id, int B, int N, int S,
                     float *centroid) {
  if (!coords || !centroid || B < 0 || N <= 0 || S <= 0) return ORACLE_ERR_ARG;
  int G = cluster_count(N, S);
  int32_t *members = (int32_t *)malloc((size_t)G * S * sizeof(int32_t));
  if (!members) return ORACLE_ERR_ALLOC;
  int rc = ORACLE_OK;
  for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
    rc = build_members(cluster_id ? cluster_id + (size_t)b * N : NULL, N, S, members);
    if (rc == ORACLE_OK)
      image_centroids(coords + (size_t)b * N * 2, members, N, S, centroid + (size_t)b * G * 2);
  }
  free(members);
  return rc;
}

/*
 * oracle_vts_table: for every point of the Hg x Wg patch grid the Kt nearest
 * visible tokens, ascending (fp32 squared distance, token index).
 *   vis_xy [B,Nv,2] fp32; table [B,Hg,Wg,Kt] int32; 1 <= Kt <= Nv.
 */
int oracle_vts_table(const float *vis_xy, int B, int Nv, int Hg, int Wg, float x0, float y0, float cell, int Kt,
                     int32_t *table) {
  if (!vis_xy || !table || B < 0 || Nv <= 0 || Hg <= 0 || Wg <= 0 || Kt < 1 || Kt > Nv || !(cell > 0.f))
    return ORACLE_ERR_ARG;
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    cand_t *cand = (cand_t *)malloc((size_t)Nv * sizeof(cand_t));
    if (!cand) {
#pragma omp critical
      status = ORACLE_ERR_ALLOC;
      continue;
    }
    const float *xy = vis_xy + (size_t)b * Nv * 2;
    for (int iy = 0; iy < Hg; ++iy) {
      for (int ix = 0; ix < Wg; ++ix) {
        const float hx = (float)ix + 0.5f, hy = (float)iy + 0.5f;
        const float sx = hx * cell, sy = hy * cell;
        const float gx = x0 + sx, gy = y0 + sy;
        for (int i = 0; i < Nv; ++i) {
          cand[i].d2 = dist2_f32(gx, gy, xy[2 * i], xy[2 * i + 1]);
          cand[i].idx = i;
        }
        qsort(cand, (size_t)Nv, sizeof(cand_t), cand_less);
        int32_t *row = table + (((size_t)b * Hg + iy) * Wg + ix) * Kt;
        for (int t = 0; t < Kt; ++t) row[t] = cand[t].idx;
      }
    }
    free(cand);
  }
  return status;
}

/* Grid cell of a query coordinate: floor((q - x0) / cell) in fp32, clamped to 0..n-1. */
static int vts_cell(float q, float x0, float cell, int n) {
  const float t = q - x0;
  const float u = t / cell;
  const float f = floorf(u);
  if (!(f >= 0.f)) return 0;
  if (f > (float)(n - 1)) return n - 1;
  return (int)f;
}

/*
 * oracle_vts_fwd: virtual sampled tokens.
 *   query_xy [B,Mq,2] fp32; vis_xy [B,Nv,2] fp32; feat [B,Nv,C] double;
 *   table [B,Hg,Wg,Kt].  For every query: the table entry of its grid cell,
 *   d_i = |q - x_i| + eps, w = softmax_i(-p d_i), out = sum_i w_i feat_i.
 *   out [B,Mq,C]; weights [B,Mq,Kt] may be NULL.
 */
int oracle_vts_fwd(const float *query_xy, const float *vis_xy, const double *feat, const int32_t *table, int B,
                   int Mq, int Nv, int C, int Hg, int Wg, float x0, float y0, float cell, int Kt, double p,
                   double eps, double *out, double *weights) {
  if (!query_xy || !vis_xy || !feat || !table || !out) return ORACLE_ERR_ARG;
  if (B < 0 || Mq <= 0 || Nv <= 0 || C <= 0 || Hg <= 0 || Wg <= 0 || Kt < 1 || !(cell > 0.f)) return ORACLE_ERR_ARG;
  for (size_t t = 0; t < (size_t)B * Hg * Wg * Kt; ++t)
    if (table[t] < 0 || table[t] >= Nv) return ORACLE_ERR_ARG;
  for (int b = 0; b < B; ++b) {
    for (int m = 0; m < Mq; ++m) {
      const float qx = query_xy[((size_t)b * Mq + m) * 2], qy = query_xy[((size_t)b * Mq + m) * 2 + 1];
      const int ix = vts_cell(qx, x0, cell, Wg), iy = vts_cell(qy, y0, cell, Hg);
      const int32_t *row = table + (((size_t)b * Hg + iy) * Wg + ix) * Kt;
      double z[64], zmax = -INFINITY, sum = 0.0;
      if (Kt > 64) return ORACLE_ERR_ARG;
      for (int i = 0; i < Kt; ++i) {
        const double dx = (double)qx - (double)vis_xy[((size_t)b * Nv + row[i]) * 2];
        const double dy = (double)qy - (double)vis_xy[((size_t)b * Nv + row[i]) * 2 + 1];
        z[i] = -p * (sqrt(dx * dx + dy * dy) + eps);
        if (z[i] > zmax) zmax = z[i];
      }
      for (int i = 0; i < Kt; ++i) {
        z[i] = exp(z[i] - zmax);
        sum += z[i];
      }
      double *o = out + ((size_t)b * Mq + m) * C;
      for (int c = 0; c < C; ++c) o[c] = 0.0;
      for (int i = 0; i < Kt; ++i) {
        const double w = z[i] / sum;
        if (weights) weights[((size_t)b * Mq + m) * Kt + i] = w;
        const double *f = feat + ((size_t)b * Nv + row[i]) * C;
        for (int c = 0; c < C; ++c) o[c] += w * f[c];
      }
    }
  }
  return ORACLE_OK;
}

/*
 * oracle_vts_bwd: chain rule on oracle_vts_fwd for L = sum(dout * out).
 *   dfeat [B,Nv,C] += w_i dout;  with g_i = <dout, feat_i>, dz_i = w_i (g_i - sum_j w_j g_j):
 *   dquery [B,Mq,2] = sum_i dz_i (-p) (q - x_i) / |q - x_i|   (0 where q = x_i),
 *   dp (scalar, summed over all queries) = sum_i dz_i (-(|q - x_i| + eps)).
 *   dp_abs (optional, a scale for judging errors of dp, no part of the method): the sum over the queries of the
 *   absolute value of each query's contribution to dp.
 */
int oracle_vts_bwd(const float *query_xy, const float *vis_xy, const double *feat, const int32_t *table,
                   const double *dout, int B, int Mq, int Nv, int C, int Hg, int Wg, float x0, float y0, float cell,
                   int Kt, double p, double eps, double *dfeat, double *dquery, double *dp, double *dp_abs) {
  if (!query_xy || !vis_xy || !feat || !table || !dout || !dfeat || !dquery) return ORACLE_ERR_ARG;
  if (B < 0 || Mq <= 0 || Nv <= 0 || C <= 0 || Hg <= 0 || Wg <= 0 || Kt < 1 || Kt > 64 || !(cell > 0.f))
    return ORACLE_ERR_ARG;
  for (size_t t = 0; t < (size_t)B * Hg * Wg * Kt; ++t)
    if (table[t] < 0 || table[t] >= Nv) return ORACLE_ERR_ARG;
  for (size_t t = 0; t < (size_t)B * Nv * C; ++t) dfeat[t] = 0.0;
  double dp_sum = 0.0, dp_abs_sum = 0.0;
  for (int b = 0; b < B; ++b) {
    for (int m = 0; m < Mq; ++m) {
      const float qx = query_xy[((size_t)b * Mq + m) * 2], qy = query_xy[((size_t)b * Mq + m) * 2 + 1];
      const int ix = vts_cell(qx, x0, cell, Wg), iy = vts_cell(qy, y0, cell, Hg);
      const int32_t *row = table + (((size_t)b * Hg + iy) * Wg + ix) * Kt;
      const double *go = dout + ((size_t)b * Mq + m) * C;
      double w[64], dist[64], dxs[64], dys[64], g[64], zmax = -INFINITY, sum = 0.0, gbar = 0.0;
      for (int i = 0; i < Kt; ++i) {
        dxs[i] = (double)qx - (double)vis_xy[((size_t)b * Nv + row[i]) * 2];
        dys[i] = (double)qy - (double)vis_xy[((size_t)b * Nv + row[i]) * 2 + 1];
        dist[i] = sqrt(dxs[i] * dxs[i] + dys[i] * dys[i]);
        w[i] = -p * (dist[i] + eps);
        if (w[i] > zmax) zmax = w[i];
      }
      for (int i = 0; i < Kt; ++i) {
        w[i] = exp(w[i] - zmax);
        sum += w[i];
      }
      for (int i = 0; i < Kt; ++i) {
        w[i] /= sum;
        const double *f = feat + ((size_t)b * Nv + row[i]) * C;
        double *df = dfeat + ((size_t)b * Nv + row[i]) * C;
        g[i] = 0.0;
        for (int c = 0; c < C; ++c) {
          g[i] += go[c] * f[c];
          df[c] += w[i] * go[c];
        }
        gbar += w[i] * g[i];
      }
      double dqx = 0.0, dqy = 0.0, dp_query = 0.0;
      for (int i = 0; i < Kt; ++i) {
        const double dz = w[i] * (g[i] - gbar);
        if (dist[i] > 0.0) {
          dqx += dz * (-p) * dxs[i] / dist[i];
          dqy += dz * (-p) * dys[i] / dist[i];
        }
        dp_query += dz * (-(dist[i] + eps));
      }
      dp_sum += dp_query;
      dp_abs_sum += fabs(dp_query);
      dquery[((size_t)b * Mq + m) * 2] = dqx;
      dquery[((size_t)b * Mq + m) * 2 + 1] = dqy;
    }
  }
  if (dp) *dp = dp_sum;
  if (dp_abs) *dp_abs = dp_abs_sum;
  return ORACLE_OK;
}

/*
 * Neighbourhood merging (Sec. "AutoFocusFormer": after several local-attention blocks the token set is
 * downsampled; an importance score per token, the top-ranked tokens kept as anchors, the remaining tokens merged
 * into nearby anchors by a differentiable, location-aware aggregation).
 *
 * oracle_merge_select: score [B,N] fp32 (finite) -> anchor_idx [B,n_keep]: the n_keep tokens with the largest
 * score (equal scores: the lower index first), listed in ascending token index.
 */
typedef struct {
  float s;
  int32_t idx;
} score_t;

static int score_before(const void *pa, const void *pb) {
  const score_t *a = (const score_t *)pa, *b = (const score_t *)pb;
  if (a->s > b->s) return -1;
  if (a->s < b->s) return 1;
  if (a->idx < b->idx) return -1;
  if (a->idx > b->idx) return 1;
  return 0;
}

static int int_less(const void *pa, const void *pb) {
  const int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
  return (a > b) - (a < b);
}

int oracle_merge_select(const float *score, int B, int N, int n_keep, int32_t *anchor_idx) {
  if (!score || !anchor_idx || B < 0 || N <= 0 || n_keep < 1 || n_keep > N) return ORACLE_ERR_ARG;
  for (size_t t = 0; t < (size_t)B * N; ++t)
    if (!(score[t] - score[t] == 0.f)) return ORACLE_ERR_ARG; /* NaN or infinite */
  score_t *all = (score_t *)malloc((size_t)N * sizeof(score_t));
  if (!all) return ORACLE_ERR_ALLOC;
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < N; ++i) {
      all[i].s = score[(size_t)b * N + i];
      all[i].idx = i;
    }
    qsort(all, (size_t)N, sizeof(score_t), score_before);
    int32_t *dst = anchor_idx + (size_t)b * n_keep;
    for (int a = 0; a < n_keep; ++a) dst[a] = all[a].idx;
    qsort(dst, (size_t)n_keep, sizeof(int32_t), int_less);
  }
  free(all);
  return ORACLE_OK;
}

/* The aggregation weights of one anchor: w_j = softmax_j(score[n_j] - p |x_{n_j} - x_anchor|), j < K. */
static void merge_weights(const float *xy, const float *score, const int32_t *row, int anchor, int K, double p,
                          double *w, double *dist) {
  double zmax = -INFINITY, sum = 0.0;
  for (int j = 0; j < K; ++j) {
    const double dx = (double)xy[2 * (size_t)row[j]] - (double)xy[2 * (size_t)anchor];
    const double dy = (double)xy[2 * (size_t)row[j] + 1] - (double)xy[2 * (size_t)anchor + 1];
    dist[j] = sqrt(dx * dx + dy * dy);
    w[j] = (double)score[row[j]] - p * dist[j];
    if (w[j] > zmax) zmax = w[j];
  }
  for (int j = 0; j < K; ++j) {
    w[j] = exp(w[j] - zmax);
    sum += w[j];
  }
  for (int j = 0; j < K; ++j) w[j] /= sum;
}

static int merge_check(const int32_t *nbr_idx, const int32_t *anchor_idx, int B, int N, int K, int n_keep) {
  for (size_t t = 0; t < (size_t)B * N * K; ++t)
    if (nbr_idx[t] < 0 || nbr_idx[t] >= N) return ORACLE_ERR_ARG;
  for (size_t t = 0; t < (size_t)B * n_keep; ++t)
    if (anchor_idx[t] < 0 || anchor_idx[t] >= N) return ORACLE_ERR_ARG;
  return ORACLE_OK;
}

/*
 * oracle_merge_fwd: coords [B,N,2] fp32, feat [B,N,C], score [B,N] fp32, nbr_idx [B,N,K] (the stage's neighbour
 * table), anchor_idx [B,n_keep] -> out [B,n_keep,C]: out[a] = sum_j w_j feat[n(anchor_a, j)];
 * weights [B,n_keep,K] may be NULL.  (The merged token's coordinates are the anchor's: nothing to compute.)
 */
int oracle_merge_fwd(const float *coords, const double *feat, const float *score, const int32_t *nbr_idx,
                     const int32_t *anchor_idx, int B, int N, int C, int K, int n_keep, double p, double *out,
                     double *weights) {
  if (!coords || !feat || !score || !nbr_idx || !anchor_idx || !out) return ORACLE_ERR_ARG;
  if (B < 0 || N <= 0 || C <= 0 || K < 1 || K > 64 || n_keep < 1 || n_keep > N) return ORACLE_ERR_ARG;
  if (merge_check(nbr_idx, anchor_idx, B, N, K, n_keep) != ORACLE_OK) return ORACLE_ERR_ARG;
  for (int b = 0; b < B; ++b) {
    const float *xy = coords + (size_t)b * N * 2;
    for (int a = 0; a < n_keep; ++a) {
      const int t = anchor_idx[(size_t)b * n_keep + a];
      const int32_t *row = nbr_idx + ((size_t)b * N + t) * K;
      double w[64], dist[64];
      merge_weights(xy, score + (size_t)b * N, row, t, K, p, w, dist);
      double *o = out + ((size_t)b * n_keep + a) * C;
      for (int c = 0; c < C; ++c) o[c] = 0.0;
      for (int j = 0; j < K; ++j) {
        if (weights) weights[((size_t)b * n_keep + a) * K + j] = w[j];
        const double *f = feat + ((size_t)b * N + row[j]) * C;
        for (int c = 0; c < C; ++c) o[c] += w[j] * f[c];
      }
    }
  }
  return ORACLE_OK;
}

/*
 * oracle_merge_bwd: chain rule on oracle_merge_fwd for L = sum(dout * out).  With g_j = <dout_a, feat_{n_j}> and
 * dz_j = w_j (g_j - sum_i w_i g_i):
 *   dfeat [B,N,C]: dfeat[n_j] += w_j dout_a;   dscore [B,N]: dscore[n_j] += dz_j;
 *   dp (scalar, summed over all anchors) = sum_j dz_j (-|x_{n_j} - x_anchor|);
 *   dp_abs (optional, a scale for judging errors of dp, no part of the method): the sum over the anchors of the
 *   absolute value of each anchor's contribution to dp.
 */
int oracle_merge_bwd(const float *coords, const double *feat, const float *score, const int32_t *nbr_idx,
                     const int32_t *anchor_idx, const double *dout, int B, int N, int C, int K, int n_keep, double p,
                     double *dfeat, double *dscore, double *dp, double *dp_abs) {
  if (!coords || !feat || !score || !nbr_idx || !anchor_idx || !dout || !dfeat || !dscore) return ORACLE_ERR_ARG;
  if (B < 0 || N <= 0 || C <= 0 || K < 1 || K > 64 || n_keep < 1 || n_keep > N) return ORACLE_ERR_ARG;
  if (merge_check(nbr_idx, anchor_idx, B, N, K, n_keep) != ORACLE_OK) return ORACLE_ERR_ARG;
  for (size_t t = 0; t < (size_t)B * N * C; ++t) dfeat[t] = 0.0;
  for (size_t t = 0; t < (size_t)B * N; ++t) dscore[t] = 0.0;
  double dp_sum = 0.0, dp_abs_sum = 0.0;
  for (int b = 0; b < B; ++b) {
    const float *xy = coords + (size_t)b * N * 2;
    for (int a = 0; a < n_keep; ++a) {
      const int t = anchor_idx[(size_t)b * n_keep + a];
      const int32_t *row = nbr_idx + ((size_t)b * N + t) * K;
      const double *go = dout + ((size_t)b * n_keep + a) * C;
      double w[64], dist[64], g[64], gbar = 0.0, dp_anchor = 0.0;
      merge_weights(xy, score + (size_t)b * N, row, t, K, p, w, dist);
      for (int j = 0; j < K; ++j) {
        const double *f = feat + ((size_t)b * N + row[j]) * C;
        double *df = dfeat + ((size_t)b * N + row[j]) * C;
        g[j] = 0.0;
        for (int c = 0; c < C; ++c) {
          g[j] += go[c] * f[c];
          df[c] += w[j] * go[c];
        }
        gbar += w[j] * g[j];
      }
      for (int j = 0; j < K; ++j) {
        const double dz = w[j] * (g[j] - gbar);
        dscore[(size_t)b * N + row[j]] += dz;
        dp_anchor += dz * (-dist[j]);
      }
      dp_sum += dp_anchor;
      dp_abs_sum += fabs(dp_anchor);
    }
  }
  if (dp) *dp = dp_sum;
  if (dp_abs) *dp_abs = dp_abs_sum;
  return ORACLE_OK;
}

/*
 * oracle_cluster: balanced clustering along a Z-order curve (Sec.
 * "AutoFocusFormer": tokens are grouped into equal-size clusters by a
 * space-filling-curve procedure).
 *   coords [B,N,2] fp32; frame = [x0, x0 + w) x [y0, y0 + h), w, h > 0.
 *   A coordinate is quantised in double precision to
 *       floor((x - x0) / w * 65536), clamped to 0..65535,
 *   the key of a token takes bit i of the quantised x as bit 2i and bit i of the
 *   quantised y as bit 2i + 1, and tokens are ordered by (key, token index).
 *   order [B,N]:      order[b][p] = the token at place p along the curve;
 *   cluster_id [B,N]: cluster_id[b][order[b][p]] = p / S  (may be NULL).
 */
typedef struct {
  uint32_t key;
  int32_t idx;
} curve_t;

static int curve_less(const void *pa, const void *pb) {
  const curve_t *a = (const curve_t *)pa, *b = (const curve_t *)pb;
  if (a->key != b->key) return a->key < b->key ? -1 : 1;
  if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
  return 0;
}

static uint32_t quantise16(double x, double x0, double w) {
  double q = floor((x - x0) / w * 65536.0);
  if (q < 0.0) q = 0.0;
  if (q > 65535.0) q = 65535.0;
  return (uint32_t)q;
}

int oracle_cluster(const float *coords, int B, int N, int S, double x0, double y0, double w, double h,
                   int32_t *order, int32_t *cluster_id) {
  if (!coords || !order || B < 0 || N <= 0 || S <= 0 || !(w > 0.0) || !(h > 0.0)) return ORACLE_ERR_ARG;
  int status = ORACLE_OK;
  for (int b = 0; b < B; ++b) {
    curve_t *c = (curve_t *)malloc((size_t)N * sizeof(curve_t));
    if (!c) {
      status = ORACLE_ERR_ALLOC;
      break;
    }
    for (int i = 0; i < N; ++i) {
      const uint32_t qx = quantise16((double)coords[((size_t)b * N + i) * 2 + 0], x0, w);
      const uint32_t qy = quantise16((double)coords[((size_t)b * N + i) * 2 + 1], y0, h);
      uint32_t key = 0;
      for (int bit = 0; bit < 16; ++bit) {
        key |= ((qx >> bit) & 1u) << (2 * bit);
        key |= ((qy >> bit) & 1u) << (2 * bit + 1);
      }
      c[i].key = key;
      c[i].idx = i;
    }
    qsort(c, (size_t)N, sizeof(curve_t), curve_less);
    for (int p = 0; p < N; ++p) {
      order[(size_t)b * N + p] = c[p].idx;
      if (cluster_id) cluster_id[(size_t)b * N + c[p].idx] = p / S;
    }
    free(c);
  }
  return status;
}

/*
 * oracle_knn: clustered neighbour search.
 *   coords [B,N,2] fp32; cluster_id [B,N] int32 or NULL (= i / S);
 *   G = ceil(N/S) clusters of S tokens, the last one short when S does not divide N;
 *   1 <= M <= G; 1 <= K <= the smallest number of candidates any token has.
 *   near_clusters [B,G,M] (may be NULL): for each cluster the M clusters with
 *     nearest centroids, ascending (distance, cluster index); the cluster
 *     itself takes part.
 *   nbr_idx [B,N,K]: for each token the K nearest tokens among the members of
 *     its cluster's M nearest clusters, ascending (distance, token index).
 */
int oracle_knn(const float *coords, const int32_t *cluster_id, int B, int N, int S, int M, int K,
               int32_t *nbr_idx, int32_t *near_clusters) {
  if (!coords || !nbr_idx || B < 0 || N <= 0 || S <= 0) return ORACLE_ERR_ARG;
  int G = cluster_count(N, S);
  if (M < 1 || M > G || K < 1 || (long long)K > (long long)M * S) return ORACLE_ERR_ARG;
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    const float *xy = coords + (size_t)b * N * 2;
    int32_t *members = (int32_t *)malloc((size_t)G * S * sizeof(int32_t));
    int32_t *cluster_of = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    float *centroid = (float *)malloc((size_t)G * 2 * sizeof(float));
    int32_t *near = (int32_t *)malloc((size_t)G * M * sizeof(int32_t));
    cand_t *cand = (cand_t *)malloc((size_t)(M * S > G ? M * S : G) * sizeof(cand_t));
    int rc = (members && cluster_of && centroid && near && cand) ? ORACLE_OK : ORACLE_ERR_ALLOC;
    if (rc == ORACLE_OK) rc = build_members(cluster_id ? cluster_id + (size_t)b * N : NULL, N, S, members);
    if (rc == ORACLE_OK) {
      for (int c = 0; c < G; ++c)
        for (int r = 0; r < cluster_size(c, N, S); ++r) cluster_of[members[(size_t)c * S + r]] = c;
      image_centroids(xy, members, N, S, centroid);
      /* nearest clusters by centroid distance */
      for (int c = 0; c < G; ++c) {
        for (int e = 0; e < G; ++e) {
          cand[e].d2 = dist2_f32(centroid[2 * c], centroid[2 * c + 1], centroid[2 * e], centroid[2 * e + 1]);
          cand[e].idx = e;
        }
        qsort(cand, (size_t)G, sizeof(cand_t), cand_less);
        for (int m = 0; m < M; ++m) near[(size_t)c * M + m] = cand[m].idx;
      }
      if (near_clusters)
        memcpy(near_clusters + (size_t)b * G * M, near, (size_t)G * M * sizeof(int32_t));
      /* per token: all members of the near clusters are candidates */
      for (int i = 0; i < N && rc == ORACLE_OK; ++i) {
        int c = cluster_of[i];
        int n = 0;
        for (int m = 0; m < M; ++m) {
          int e = near[(size_t)c * M + m];
          for (int r = 0; r < cluster_size(e, N, S); ++r) {
            int j = members[(size_t)e * S + r];
            cand[n].d2 = dist2_f32(xy[2 * (size_t)i], xy[2 * (size_t)i + 1], xy[2 * (size_t)j], xy[2 * (size_t)j + 1]);
            cand[n].idx = j;
            ++n;
          }
        }
        if (n < K) {  /* a short last cluster among the near ones left fewer than K candidates */
          rc = ORACLE_ERR_ARG;
          break;
        }
        qsort(cand, (size_t)n, sizeof(cand_t), cand_less);
        int32_t *dst = nbr_idx + ((size_t)b * N + i) * K;
        for (int t = 0; t < K; ++t) dst[t] = cand[t].idx;
      }
    }
    free(members); free(cluster_of); free(centroid); free(near); free(cand);
    if (rc != ORACLE_OK) {
#pragma omp critical
      status = rc;
    }
  }
  return status;
}

/* oracle_knn_bruteforce: every token of the image is a candidate. */
int oracle_knn_bruteforce(const float *coords, int B, int N, int K, int32_t *nbr_idx) {
  if (!coords || !nbr_idx || B < 0 || N <= 0 || K < 1 || K > N) return ORACLE_ERR_ARG;
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    const float *xy = coords + (size_t)b * N * 2;
    cand_t *cand = (cand_t *)malloc((size_t)N * sizeof(cand_t));
    if (!cand) {
#pragma omp critical
      status = ORACLE_ERR_ALLOC;
      continue;
    }
    for (int i = 0; i < N; ++i) {
      for (int j = 0; j < N; ++j) {
        cand[j].d2 = dist2_f32(xy[2 * (size_t)i], xy[2 * (size_t)i + 1], xy[2 * (size_t)j], xy[2 * (size_t)j + 1]);
        cand[j].idx = j;
      }
      qsort(cand, (size_t)N, sizeof(cand_t), cand_less);
      int32_t *dst = nbr_idx + ((size_t)b * N + i) * K;
      for (int t = 0; t < K; ++t) dst[t] = cand[t].idx;
    }
    free(cand);
  }
  return status;
}

/*
 * Softmax row of one (image, token, head): fills s[0..Kt) with the logits and
 * p[0..Kt) with the probabilities, returns log(sum exp(s)).  Kt = K (+1 with a
 * blank column, which is slot K).
 */
static double attention_row(const double *q, const double *k, const double *bias,
                            const int32_t *nbr, const double *k_blank, int b, int i, int h,
                            int N, int H, int d, int K, double scale, double *s, double *p) {
  const double *qi = q + (((size_t)b * N + i) * H + h) * d;
  int Kt = K;
  for (int j = 0; j < K; ++j) {
    int n = nbr[((size_t)b * N + i) * K + j];
    const double *kn = k + (((size_t)b * N + n) * H + h) * d;
    double acc = 0.0;
    for (int t = 0; t < d; ++t) acc += qi[t] * kn[t];
    s[j] = scale * acc + (bias ? bias[(((size_t)b * N + i) * H + h) * K + j] : 0.0);
  }
  if (k_blank) {
    double acc = 0.0;
    for (int t = 0; t < d; ++t) acc += qi[t] * k_blank[(size_t)h * d + t];
    s[K] = scale * acc;
    Kt = K + 1;
  }
  double m = s[0];
  for (int j = 1; j < Kt; ++j)
    if (s[j] > m) m = s[j];
  double z = 0.0;
  for (int j = 0; j < Kt; ++j) {
    p[j] = exp(s[j] - m);
    z += p[j];
  }
  for (int j = 0; j < Kt; ++j) p[j] /= z;
  return m + log(z);
}

static int check_nbr(const int32_t *nbr, size_t count, int N) {
  for (size_t t = 0; t < count; ++t)
    if (nbr[t] < 0 || nbr[t] >= N) return ORACLE_ERR_ARG;
  return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* relative-position bias (Sec. "AutoFocusFormer": within a neighbourhood,    */
/* attention uses relative position derived from the 2-D token coordinates;   */
/* the FlashNbhdAttn equation adds it as B_n).  The function is this build's  */
/* reading: a per-head table over quantised offsets.                          */

/* Bin of one axis: offset (neighbour minus query) times the bin rate, in fp32,
 * rounded to the nearest integer with ties to even, clamped to -R..R, plus R. */
static int relpos_bin(float nbr, float query, float rate, int R) {
  float d = nbr - query;
  float t = d * rate;
  float r = rintf(t); /* default rounding mode: to nearest, ties to even */
  if (!(r >= (float)(-R))) return 0; /* also NaN */
  if (r > (float)R) return 2 * R;
  return (int)r + R;
}

/*
 * oracle_relpos_bias: coords [B,N,2] fp32, nbr_idx [B,N,K], table [H][2R+1][2R+1]
 * (row = y bin, column = x bin) -> bias [B,N,H,K].
 */
int oracle_relpos_bias(const float *coords, const int32_t *nbr_idx, const double *table, int B,
                       int N, int H, int K, int R, float rate, double *bias) {
  if (!coords || !nbr_idx || !table || !bias) return ORACLE_ERR_ARG;
  if (B < 0 || N <= 0 || H <= 0 || K <= 0 || R < 0) return ORACLE_ERR_ARG;
  int W = 2 * R + 1;
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < N; ++i)
      for (int j = 0; j < K; ++j) {
        int n = nbr_idx[((size_t)b * N + i) * K + j];
        if (n < 0 || n >= N) return ORACLE_ERR_ARG;
        const float *ci = coords + ((size_t)b * N + i) * 2;
        const float *cn = coords + ((size_t)b * N + n) * 2;
        int bx = relpos_bin(cn[0], ci[0], rate, R);
        int by = relpos_bin(cn[1], ci[1], rate, R);
        for (int h = 0; h < H; ++h)
          bias[(((size_t)b * N + i) * H + h) * K + j] = table[((size_t)h * W + by) * W + bx];
      }
  return ORACLE_OK;
}

/*
 * oracle_relpos_dtable: the gradient of the table, dtable[h][by][bx] = sum of
 * dbias[b,i,h,j] over every (b,i,j) whose offset falls in bin (by,bx).
 */
int oracle_relpos_dtable(const float *coords, const int32_t *nbr_idx, const double *dbias, int B,
                         int N, int H, int K, int R, float rate, double *dtable) {
  if (!coords || !nbr_idx || !dbias || !dtable) return ORACLE_ERR_ARG;
  if (B < 0 || N <= 0 || H <= 0 || K <= 0 || R < 0) return ORACLE_ERR_ARG;
  int W = 2 * R + 1;
  memset(dtable, 0, (size_t)H * W * W * sizeof(double));
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < N; ++i)
      for (int j = 0; j < K; ++j) {
        int n = nbr_idx[((size_t)b * N + i) * K + j];
        if (n < 0 || n >= N) return ORACLE_ERR_ARG;
        const float *ci = coords + ((size_t)b * N + i) * 2;
        const float *cn = coords + ((size_t)b * N + n) * 2;
        int bx = relpos_bin(cn[0], ci[0], rate, R);
        int by = relpos_bin(cn[1], ci[1], rate, R);
        for (int h = 0; h < H; ++h)
          dtable[((size_t)h * W + by) * W + bx] += dbias[(((size_t)b * N + i) * H + h) * K + j];
      }
  return ORACLE_OK;
}

/*
 * oracle_pla_fwd: q,k,v [B,N,H,d]; bias [B,N,H,K] or NULL; nbr_idx [B,N,K] with
 * values in [0,N) (repeats allowed: every slot is its own softmax column);
 * k_blank,v_blank [H,d] or both NULL.
 *   out [B,N,H,d]; lse [B,N,H] natural log of the softmax denominator;
 *   prob (may be NULL) [B,N,H,K+1] probabilities, slot K = blank (0 if none).
 */
int oracle_pla_fwd(const double *q, const double *k, const double *v, const double *bias,
                   const int32_t *nbr_idx, const double *k_blank, const double *v_blank, int B,
                   int N, int H, int d, int K, double scale, double *out, double *lse,
                   double *prob) {
  if (!q || !k || !v || !nbr_idx || !out || !lse) return ORACLE_ERR_ARG;
  if (B < 0 || N <= 0 || H <= 0 || d <= 0 || K <= 0) return ORACLE_ERR_ARG;
  if ((k_blank == NULL) != (v_blank == NULL)) return ORACLE_ERR_ARG;
  if (check_nbr(nbr_idx, (size_t)B * N * K, N) != ORACLE_OK) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
  for (int b = 0; b < B; ++b) {
    double *s = (double *)malloc((size_t)(K + 1) * sizeof(double));
    double *p = (double *)malloc((size_t)(K + 1) * sizeof(double));
    for (int i = 0; i < N; ++i)
      for (int h = 0; h < H; ++h) {
        double l = attention_row(q, k, bias, nbr_idx, k_blank, b, i, h, N, H, d, K, scale, s, p);
        double *o = out + (((size_t)b * N + i) * H + h) * d;
        for (int t = 0; t < d; ++t) o[t] = 0.0;
        for (int j = 0; j < K; ++j) {
          int n = nbr_idx[((size_t)b * N + i) * K + j];
          const double *vn = v + (((size_t)b * N + n) * H + h) * d;
          for (int t = 0; t < d; ++t) o[t] += p[j] * vn[t];
        }
        if (v_blank)
          for (int t = 0; t < d; ++t) o[t] += p[K] * v_blank[(size_t)h * d + t];
        lse[((size_t)b * N + i) * H + h] = l;
        if (prob) {
          double *pr = prob + (((size_t)b * N + i) * H + h) * (K + 1);
          for (int j = 0; j < K; ++j) pr[j] = p[j];
          pr[K] = k_blank ? p[K] : 0.0;
        }
      }
    free(s);
    free(p);
  }
  return ORACLE_OK;
}

/*
 * oracle_pla_bwd: gradients of L = sum(dout * out) with respect to q, k, v,
 * bias and the blank rows.  With p the softmax row of (b,i,h):
 *   dP_j  = <dout_i, v_j>             (v_j = neighbour row or blank row)
 *   D     = sum_j p_j dP_j
 *   dS_j  = p_j (dP_j - D)
 *   dbias[b,i,h,j]   = dS_j                      (j < K)
 *   dq_i            += scale * dS_j * k_j
 *   dk[n(i,j)]      += scale * dS_j * q_i,   dv[n(i,j)] += p_j * dout_i
 *   dk_blank[h]     += scale * dS_K * q_i,   dv_blank[h] += p_K * dout_i
 * All outputs are overwritten.  dbias, dk_blank, dv_blank may be NULL.
 */
int oracle_pla_bwd(const double *q, const double *k, const double *v, const double *bias,
                   const int32_t *nbr_idx, const double *k_blank, const double *v_blank,
                   const double *dout, int B, int N, int H, int d, int K, double scale, double *dq,
                   double *dk, double *dv, double *dbias, double *dk_blank, double *dv_blank) {
  if (!q || !k || !v || !nbr_idx || !dout || !dq || !dk || !dv) return ORACLE_ERR_ARG;
  if (B < 0 || N <= 0 || H <= 0 || d <= 0 || K <= 0) return ORACLE_ERR_ARG;
  if ((k_blank == NULL) != (v_blank == NULL)) return ORACLE_ERR_ARG;
  if (check_nbr(nbr_idx, (size_t)B * N * K, N) != ORACLE_OK) return ORACLE_ERR_ARG;
  size_t per_image = (size_t)N * H * d;
  memset(dq, 0, (size_t)B * per_image * sizeof(double));
  memset(dk, 0, (size_t)B * per_image * sizeof(double));
  memset(dv, 0, (size_t)B * per_image * sizeof(double));
  if (dk_blank) memset(dk_blank, 0, (size_t)H * d * sizeof(double));
  if (dv_blank) memset(dv_blank, 0, (size_t)H * d * sizeof(double));
  /* blank-row gradients sum over images: one partial per image, added in image order */
  double *blank_part = NULL;
  if (k_blank && (dk_blank || dv_blank)) {
    blank_part = (double *)calloc((size_t)B * 2 * H * d, sizeof(double));
    if (!blank_part) return ORACLE_ERR_ALLOC;
  }
#pragma omp parallel for schedule(static)
  for (int b = 0; b < B; ++b) {
    double *s = (double *)malloc((size_t)(K + 1) * sizeof(double));
    double *p = (double *)malloc((size_t)(K + 1) * sizeof(double));
    double *dP = (double *)malloc((size_t)(K + 1) * sizeof(double));
    for (int i = 0; i < N; ++i)
      for (int h = 0; h < H; ++h) {
        attention_row(q, k, bias, nbr_idx, k_blank, b, i, h, N, H, d, K, scale, s, p);
        int Kt = k_blank ? K + 1 : K;
        size_t qoff = (((size_t)b * N + i) * H + h) * d;
        const double *qi = q + qoff;
        const double *gi = dout + qoff;
        double D = 0.0;
        for (int j = 0; j < Kt; ++j) {
          const double *vn;
          if (j < K) {
            int n = nbr_idx[((size_t)b * N + i) * K + j];
            vn = v + (((size_t)b * N + n) * H + h) * d;
          } else {
            vn = v_blank + (size_t)h * d;
          }
          double acc = 0.0;
          for (int t = 0; t < d; ++t) acc += gi[t] * vn[t];
          dP[j] = acc;
          D += p[j] * acc;
        }
        for (int j = 0; j < Kt; ++j) {
          double dS = p[j] * (dP[j] - D);
          if (j < K) {
            int n = nbr_idx[((size_t)b * N + i) * K + j];
            size_t noff = (((size_t)b * N + n) * H + h) * d;
            if (dbias) dbias[(((size_t)b * N + i) * H + h) * K + j] = dS;
            for (int t = 0; t < d; ++t) {
              dq[qoff + t] += scale * dS * k[noff + t];
              dk[noff + t] += scale * dS * qi[t];
              dv[noff + t] += p[j] * gi[t];
            }
          } else {
            double *pk = blank_part ? blank_part + ((size_t)b * 2 + 0) * H * d + (size_t)h * d : NULL;
            double *pv = blank_part ? blank_part + ((size_t)b * 2 + 1) * H * d + (size_t)h * d : NULL;
            for (int t = 0; t < d; ++t) {
              dq[qoff + t] += scale * dS * k_blank[(size_t)h * d + t];
              if (pk) {
                pk[t] += scale * dS * qi[t];
                pv[t] += p[j] * gi[t];
              }
            }
          }
        }
      }
    free(s);
    free(p);
    free(dP);
  }
  if (blank_part) {
    for (int b = 0; b < B; ++b)
      for (int e = 0; e < H * d; ++e) {
        if (dk_blank) dk_blank[e] += blank_part[((size_t)b * 2 + 0) * H * d + e];
        if (dv_blank) dv_blank[e] += blank_part[((size_t)b * 2 + 1) * H * d + e];
      }
    free(blank_part);
  }
  return ORACLE_OK;
}
