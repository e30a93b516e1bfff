// Balanced clustering along a Z-order curve (paper, Sec. "AutoFocusFormer":
// tokens are grouped into equal-size clusters by a space-filling-curve procedure;
// the curve is not named there - this library takes the Z-order (Morton) curve
// over coordinates quantised to 16 bits per axis of a caller-given frame).
//
// Per image the tokens are sorted by the 64-bit word (curve key << 32 | token
// index): unique words, so the order is exact and ties go to the lower index.
// The sort is a bitonic network over the image's words padded to a power of two
// (pads are all ones and end up last): chunks of up to 2048 words are sorted and
// merged in LDS by one workgroup (many workgroups per image); the compare-exchange
// steps whose partner lies in another chunk run over global memory, up to three
// per pass.  A last kernel writes the order and
// each token's cluster (place along the curve / S).
#include "device_util.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

typedef unsigned long long word_t;
constexpr int kChunk = 2048;       // words sorted in LDS by one workgroup (16 KB): many workgroups per image
constexpr int kSortThreads = 256;

struct ClusterParams {
  const float* coords;  // [B,N,2]
  int N, npad, S;
  double x0, y0, w, h;  // frame
  word_t* words;  // [B][npad]
  int32_t* order;
  int32_t* cluster_id;
};

// floor((x - x0) / w * 65536) clamped to 0..65535, in double precision.
__device__ __forceinline__ uint32_t quantise16(float x, double x0, double w) {
  double q = floor(((double)x - x0) / w * 65536.0);
  q = q < 0.0 ? 0.0 : q;
  q = q > 65535.0 ? 65535.0 : q;
  return (uint32_t)q;
}

// bit i of v -> bit 2i
__device__ __forceinline__ uint32_t spread16(uint32_t v) {
  v = (v | (v << 8)) & 0x00ff00ffu;
  v = (v | (v << 4)) & 0x0f0f0f0fu;
  v = (v | (v << 2)) & 0x33333333u;
  v = (v | (v << 1)) & 0x55555555u;
  return v;
}

__device__ __forceinline__ word_t token_word(const ClusterParams& p, int b, int i) {
  if (i >= p.N) return ~0ull;
  const float* xy = p.coords + ((size_t)b * p.N + i) * 2;
  const uint32_t key = spread16(quantise16(xy[0], p.x0, p.w)) | (spread16(quantise16(xy[1], p.y0, p.h)) << 1);
  return ((word_t)key << 32) | (word_t)(uint32_t)i;
}

// R consecutive compare-exchange steps (k, J), (k, J/2), ... of the bitonic network on a chunk held in LDS, in one
// trip through LDS: a thread takes the 2^R words that these steps connect (strides J .. J >> (R-1)), exchanges
// them in registers and writes them back.  `first` is the global position of the chunk's first word (it
// decides the direction, which is the same for all words of a group because k > J).
// Place of word w in the LDS chunk: the XOR spreads every access pattern of the passes below over all
// banks (a thread's 2^R words with stride 1, 2 or 4 would otherwise fall on a few banks).
__device__ __forceinline__ int lds_place(int w) { return w ^ ((w >> 3) & 31); }

template <int R>
__device__ __forceinline__ void lds_pass(word_t* buf, int n, int first, int k, int J) {
  const int low = J >> (R - 1);
  for (int t = threadIdx.x; t < (n >> R); t += blockDim.x) {
    const int i0 = ((t & ~(low - 1)) << R) | (t & (low - 1));
    word_t v[1 << R];
#pragma unroll
    for (int m = 0; m < (1 << R); ++m) v[m] = buf[lds_place(i0 + m * low)];
    const bool ascending = ((first + i0) & k) == 0;
#pragma unroll
    for (int bit = R - 1; bit >= 0; --bit) {
#pragma unroll
      for (int m = 0; m < (1 << R); ++m) {
        if (!((m >> bit) & 1)) {
          const word_t a = v[m], c = v[m | (1 << bit)];
          const bool swap = (a > c) == ascending;
          v[m] = swap ? c : a;
          v[m | (1 << bit)] = swap ? a : c;
        }
      }
    }
#pragma unroll
    for (int m = 0; m < (1 << R); ++m) buf[lds_place(i0 + m * low)] = v[m];
  }
  __syncthreads();
}

// The steps j = J, J/2, ..., 1 of stage k, three at a time.
__device__ __forceinline__ void lds_steps(word_t* buf, int n, int first, int k, int J) {
  int j = J;
  while (j >= 4) {
    lds_pass<3>(buf, n, first, k, j);
    j >>= 3;
  }
  if (j == 2) lds_pass<2>(buf, n, first, k, 2);
  else if (j == 1) lds_pass<1>(buf, n, first, k, 1);
}

// Builds the words of one chunk and sorts it: all steps with k <= chunk size.
__global__ __launch_bounds__(kSortThreads) void cluster_sort_chunk_kernel(ClusterParams p, int chunk) {
  extern __shared__ word_t buf[];
  const int chunks_per_image = p.npad / chunk;
  const int b = blockIdx.x / chunks_per_image, c = blockIdx.x % chunks_per_image;
  const int first = c * chunk;
  for (int t = threadIdx.x; t < chunk; t += blockDim.x) buf[lds_place(t)] = token_word(p, b, first + t);
  __syncthreads();
  for (int k = 2; k <= chunk; k <<= 1) lds_steps(buf, chunk, first, k, k >> 1);
  word_t* out = p.words + (size_t)b * p.npad + first;
  for (int t = threadIdx.x; t < chunk; t += blockDim.x) out[t] = buf[lds_place(t)];
}

// R consecutive steps (k, J), (k, J/2), ... whose strides are all at least the chunk size: partners sit in
// different chunks, so the 2^R words a thread connects come from and go back to global memory.
template <int R>
__global__ __launch_bounds__(256) void cluster_global_pass_kernel(ClusterParams p, int k, int J) {
  const int groups = p.npad >> R;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (t >= groups) return;
  const int low = J >> (R - 1);
  const int i0 = ((t & ~(low - 1)) << R) | (t & (low - 1));
  word_t* w = p.words + (size_t)b * p.npad;
  word_t v[1 << R];
#pragma unroll
  for (int m = 0; m < (1 << R); ++m) v[m] = w[i0 + m * low];
  const bool ascending = (i0 & k) == 0;
#pragma unroll
  for (int bit = R - 1; bit >= 0; --bit) {
#pragma unroll
    for (int m = 0; m < (1 << R); ++m) {
      if (!((m >> bit) & 1)) {
        const word_t a = v[m], c = v[m | (1 << bit)];
        const bool swap = (a > c) == ascending;
        v[m] = swap ? c : a;
        v[m | (1 << bit)] = swap ? a : c;
      }
    }
  }
#pragma unroll
  for (int m = 0; m < (1 << R); ++m) w[i0 + m * low] = v[m];
}

// The steps j = chunk/2 .. 1 of stage k (k > chunk size), in LDS.
__global__ __launch_bounds__(kSortThreads) void cluster_merge_chunk_kernel(ClusterParams p, int chunk, int k) {
  extern __shared__ word_t buf[];
  const int chunks_per_image = p.npad / chunk;
  const int b = blockIdx.x / chunks_per_image, c = blockIdx.x % chunks_per_image;
  const int first = c * chunk;
  word_t* io = p.words + (size_t)b * p.npad + first;
  for (int t = threadIdx.x; t < chunk; t += blockDim.x) buf[lds_place(t)] = io[t];
  __syncthreads();
  lds_steps(buf, chunk, first, k, chunk >> 1);
  for (int t = threadIdx.x; t < chunk; t += blockDim.x) io[t] = buf[lds_place(t)];
}

__global__ __launch_bounds__(256) void cluster_emit_kernel(ClusterParams p) {
  const int place = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (place >= p.N) return;
  const int tok = (int)(uint32_t)p.words[(size_t)b * p.npad + place];  // pads sort last: the first N are tokens
  p.order[(size_t)b * p.N + place] = tok;
  if (p.cluster_id) p.cluster_id[(size_t)b * p.N + tok] = place / p.S;
}

int next_pow2(int n) {
  int v = 2;
  while (v < n) v <<= 1;
  return v;
}

}  // namespace

size_t cluster_workspace_bytes(int B, int N) { return (size_t)B * next_pow2(N) * sizeof(word_t); }

hipError_t launch_cluster(const float* coords, int B, int N, int S, double x0, double y0, double w, double h,
                          int32_t* order, int32_t* cluster_id, void* workspace, hipStream_t stream) {
  ClusterParams p;
  p.coords = coords; p.N = N; p.npad = next_pow2(N); p.S = S;
  p.x0 = x0; p.y0 = y0; p.w = w; p.h = h;
  p.words = static_cast<word_t*>(workspace);
  p.order = order; p.cluster_id = cluster_id;
  const int chunk = p.npad < kChunk ? p.npad : kChunk;
  const size_t lds = (size_t)chunk * sizeof(word_t);
  const int threads = chunk / 2 < kSortThreads ? (chunk / 2 < 64 ? 64 : chunk / 2) : kSortThreads;
  const dim3 per_chunk(B * (p.npad / chunk));
  AFFMAE_LAUNCH("cluster_sort_chunk_kernel", stream, cluster_sort_chunk_kernel, per_chunk, dim3(threads), lds, stream, p,
                chunk);
  for (int k = chunk * 2; k <= p.npad; k <<= 1) {
    int j = k >> 1;
    while (j >= chunk) {  // up to three steps per pass over global memory
      int steps = 0;
      for (int jj = j; jj >= chunk && steps < 3; jj >>= 1) ++steps;
      const dim3 grid(((p.npad >> steps) + 255) / 256, B);
      if (steps == 3)
        AFFMAE_LAUNCH("cluster_global_pass_kernel", stream, cluster_global_pass_kernel<3>, grid, dim3(256), 0, stream, p, k, j);
      else if (steps == 2)
        AFFMAE_LAUNCH("cluster_global_pass_kernel", stream, cluster_global_pass_kernel<2>, grid, dim3(256), 0, stream, p, k, j);
      else
        AFFMAE_LAUNCH("cluster_global_pass_kernel", stream, cluster_global_pass_kernel<1>, grid, dim3(256), 0, stream, p, k, j);
      j >>= steps;
    }
    AFFMAE_LAUNCH("cluster_merge_chunk_kernel", stream, cluster_merge_chunk_kernel, per_chunk, dim3(threads), lds, stream,
                  p, chunk, k);
  }
  AFFMAE_LAUNCH("cluster_emit_kernel", stream, cluster_emit_kernel, dim3((N + 255) / 256, B), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace affmae
