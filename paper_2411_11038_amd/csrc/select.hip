// Channel importance (Eq. 6) and deterministic Top-K (Sec. 3.2): scores in fp64, selection by exact
// rank under the key (score descending, index ascending), output compacted in ascending index order.
#include "common.hpp"

namespace efqat {

// I[c] = (1/n) sum_j |w[c][j]|, fp64 accumulation, one wavefront per channel, fixed reduction order.
__global__ __launch_bounds__(256) void k_row_importance(const float* __restrict__ w, int64_t c_out, int64_t n,
                                                        int vec, double* __restrict__ scores) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= c_out) return;
  const float* p = w + row * n;
  double acc = 0.0;
  if (vec) {
    const int64_t n4 = n >> 2;
    for (int64_t i = lane; i < n4; i += 64) {
      const float4 v = *reinterpret_cast<const float4*>(p + i * 4);
      acc += (double)fabsf(v.x) + (double)fabsf(v.y) + (double)fabsf(v.z) + (double)fabsf(v.w);
    }
  } else {
    for (int64_t i = lane; i < n; i += 64) acc += (double)fabsf(p[i]);
  }
  acc = wave_sum(acc);
  if (lane == 0) scores[row] = acc / (double)n;
}

// flag[c] = 1 iff fewer than k channels precede c in the order (score desc, index asc).
__global__ __launch_bounds__(256) void k_rank_flags(const double* __restrict__ scores, int64_t n, int64_t k,
                                                    int32_t* __restrict__ flags) {
  __shared__ double tile[1024];
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const double mine = c < n ? scores[c] : 0.0;
  int64_t rank = 0;
  for (int64_t j0 = 0; j0 < n; j0 += 1024) {
    const int64_t cnt = (n - j0) < 1024 ? (n - j0) : 1024;
    __syncthreads();
    for (int64_t t = threadIdx.x; t < cnt; t += blockDim.x) tile[t] = scores[j0 + t];
    __syncthreads();
    if (c < n) {
      for (int64_t t = 0; t < cnt; ++t) {
        const double o = tile[t];
        rank += (o > mine) || (o == mine && (j0 + t) < c);
      }
    }
  }
  if (c < n) flags[c] = rank < k ? 1 : 0;
}

// Ordered compaction of the flagged indices (single block, chunks of 1024 in ascending order).
__global__ __launch_bounds__(1024) void k_compact(const int32_t* __restrict__ flags, int64_t n, int64_t k,
                                                  int32_t* __restrict__ idx) {
  __shared__ int32_t wsum[16];
  __shared__ int32_t s_base;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  if (threadIdx.x == 0) s_base = 0;
  __syncthreads();
  for (int64_t c0 = 0; c0 < n; c0 += 1024) {
    const int64_t c = c0 + threadIdx.x;
    const int f = (c < n) ? flags[c] : 0;
    const unsigned long long b = __ballot(f);
    const int before = __popcll(b & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wv] = __popcll(b);
    __syncthreads();
    int off = s_base;
    for (int i = 0; i < wv; ++i) off += wsum[i];
    if (f) {
      const int64_t pos = (int64_t)off + before;
      if (pos < k) idx[pos] = (int32_t)c;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int i = 0; i < 16; ++i) t += wsum[i];
      s_base += t;
    }
    __syncthreads();
  }
}

// CWPN helpers: per-layer counts of selected channels, and global -> per-layer local indices.
__global__ void k_layer_counts(const int64_t* __restrict__ layer_off, int64_t n_layers,
                               const int32_t* __restrict__ flags, int32_t* __restrict__ k_per_layer) {
  // one wavefront per layer, deterministic integer count
  const int lane = threadIdx.x & 63;
  const int64_t l = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (l >= n_layers) return;
  int cnt = 0;
  for (int64_t c = layer_off[l] + lane; c < layer_off[l + 1]; c += 64) cnt += flags[c];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
  if (lane == 0) k_per_layer[l] = cnt;
}
__global__ void k_localize(const int64_t* __restrict__ layer_off, int64_t n_layers, int64_t k_total,
                            int32_t* __restrict__ idx) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= k_total) return;
  const int64_t g = idx[i];
  int64_t lo = 0, hi = n_layers;
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (layer_off[mid] <= g) lo = mid; else hi = mid;
  }
  idx[i] = (int32_t)(g - layer_off[lo]);
}

}  // namespace efqat

using namespace efqat;

extern "C" int64_t efqat_k_from_ratio(int64_t c_out, int64_t num, int64_t den) {
  if (c_out < 0 || num < 0 || den <= 0 || num > den) return -1;
  return (int64_t)(((__int128)c_out * (__int128)num) / (__int128)den);
}

extern "C" size_t efqat_channel_select_workspace_bytes(int64_t c_out) {
  if (c_out <= 0) return 0;
  return (size_t)(round_up(c_out * (int64_t)sizeof(double), 256) + round_up(c_out * (int64_t)sizeof(int32_t), 256));
}

extern "C" int efqat_channel_select(const float* w, int64_t c_out, int64_t block, int64_t k, double* scores,
                                    int32_t* idx, void* ws, size_t ws_bytes, void* stream) {
  if (c_out <= 0 || block <= 0 || c_out > INT32_MAX || c_out > INT64_MAX / block) return EFQAT_ERR_BAD_SHAPE;
  if (k < 0 || k > c_out) return EFQAT_ERR_BAD_K;
  if (!w || !ws || (k > 0 && !idx)) return EFQAT_ERR_NULL_PTR;
  if (ws_bytes < efqat_channel_select_workspace_bytes(c_out)) return EFQAT_ERR_WORKSPACE;
  if (((uintptr_t)ws % 256) != 0 || ((uintptr_t)w % 4) != 0) return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  WsCarver carve(ws);
  double* sc = (double*)carve.take((size_t)c_out * sizeof(double));
  int32_t* flags = (int32_t*)carve.take((size_t)c_out * sizeof(int32_t));
  double* sc_out = scores ? scores : sc;
  const int vec = (((uintptr_t)w % 16) == 0 && block % 4 == 0) ? 1 : 0;
  hipLaunchKernelGGL(k_row_importance, dim3((unsigned)ceil_div(c_out, 4)), dim3(256), 0, st, w, c_out, block, vec,
                     sc_out);
  EFQAT_LAUNCH_CHECK();
  if (k == 0) return EFQAT_OK;
  hipLaunchKernelGGL(k_rank_flags, dim3((unsigned)ceil_div(c_out, 256)), dim3(256), 0, st, sc_out, c_out, k, flags);
  EFQAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_compact, dim3(1), dim3(1024), 0, st, flags, c_out, k, idx);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

extern "C" size_t efqat_network_select_workspace_bytes(int64_t total) {
  if (total <= 0) return 0;
  return (size_t)round_up(total * (int64_t)sizeof(int32_t), 256);
}

extern "C" int efqat_network_select(const double* scores, const int64_t* layer_off, int64_t n_layers,
                                    int64_t total, int64_t k_total, int32_t* idx, int32_t* k_per_layer, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (n_layers <= 0 || total <= 0 || total > INT32_MAX) return EFQAT_ERR_BAD_SHAPE;
  if (k_total < 0 || k_total > total) return EFQAT_ERR_BAD_K;
  if (!scores || !layer_off || !k_per_layer || !ws || (k_total > 0 && !idx)) return EFQAT_ERR_NULL_PTR;
  if (ws_bytes < efqat_network_select_workspace_bytes(total)) return EFQAT_ERR_WORKSPACE;
  if (((uintptr_t)ws % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  int32_t* flags = (int32_t*)ws;
  hipLaunchKernelGGL(k_rank_flags, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st, scores, total, k_total,
                     flags);
  EFQAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_layer_counts, dim3((unsigned)ceil_div(n_layers, 4)), dim3(256), 0, st, layer_off, n_layers,
                     flags, k_per_layer);
  EFQAT_LAUNCH_CHECK();
  if (k_total > 0) {
    hipLaunchKernelGGL(k_compact, dim3(1), dim3(1024), 0, st, flags, total, k_total, idx);
    EFQAT_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_localize, dim3((unsigned)ceil_div(k_total, 256)), dim3(256), 0, st, layer_off, n_layers,
                       k_total, idx);
    EFQAT_LAUNCH_CHECK();
  }
  return EFQAT_OK;
}
