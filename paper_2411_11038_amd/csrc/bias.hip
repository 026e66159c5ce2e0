// Bias gradient of a quantized linear / convolution layer: db[c] = sum_t dY[t][c].  Biases are never frozen
// (Sec. 3.4; Alg. 1 updates them in every optimizer step), so this runs for all channels whatever the update
// fraction.  HBM bound: dY is read once.  Two deterministic stages: fp32 partial sums per (row chunk, column),
// then a fixed-order double-precision sum of the partials.
#include "common.hpp"

#include <algorithm>

namespace efqat {

constexpr int kBiasCols = 8;        // consecutive channels per lane
constexpr int kBiasRows = 64;       // token rows per block (16 per wavefront, all loads in flight together)

// token-major dY [T][c_out]: a wavefront covers 512 consecutive channels of one token row per step
template <typename T>
__global__ __launch_bounds__(256) void k_bias_partial_tok(const T* __restrict__ dy, int64_t T_rows, int64_t c_out,
                                                          int vec, float* __restrict__ part) {
  __shared__ float red[4][64 * kBiasCols];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = ((int64_t)blockIdx.x * 64 + lane) * kBiasCols;
  float acc[kBiasCols];
#pragma unroll
  for (int j = 0; j < kBiasCols; ++j) acc[j] = 0.0f;
  const int64_t t0 = (int64_t)blockIdx.y * kBiasRows;
  const int64_t t1 = std::min<int64_t>(t0 + kBiasRows, T_rows);
  if (c0 < c_out) {
    if (vec && c0 + kBiasCols <= c_out) {
#pragma unroll
      for (int r = 0; r < kBiasRows / 4; ++r) {
        const int64_t t = t0 + wave + 4 * r;
        if (t >= t1) break;
        float v[kBiasCols];
        if constexpr (sizeof(T) == 2) {
          const uint4 raw = *reinterpret_cast<const uint4*>(dy + t * c_out + c0);
          const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            v[2 * j] = __uint_as_float(w[j] << 16);
            v[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
          }
        } else {
          const float4 a = *reinterpret_cast<const float4*>(dy + t * c_out + c0);
          const float4 b = *reinterpret_cast<const float4*>(dy + t * c_out + c0 + 4);
          v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        }
#pragma unroll
        for (int j = 0; j < kBiasCols; ++j) acc[j] += v[j];
      }
    } else {
      for (int64_t t = t0 + wave; t < t1; t += 4)
#pragma unroll
        for (int j = 0; j < kBiasCols; ++j)
          if (c0 + j < c_out) acc[j] += load_as_f32<T>(dy, t * c_out + c0 + j);
    }
  }
#pragma unroll
  for (int j = 0; j < kBiasCols; ++j) red[wave][lane * kBiasCols + j] = acc[j];
  __syncthreads();
  // 512 columns, 256 threads: two columns each, the four wavefronts' sums added in a fixed order
  for (int q = threadIdx.x; q < 64 * kBiasCols; q += 256) {
    const int64_t c = (int64_t)blockIdx.x * 64 * kBiasCols + q;
    if (c < c_out) part[(int64_t)blockIdx.y * c_out + c] = (red[0][q] + red[1][q]) + (red[2][q] + red[3][q]);
  }
}

// channel-major dY [c_out][T]: one wavefront per (channel, segment of the row)
template <typename T>
__global__ __launch_bounds__(256) void k_bias_partial_chan(const T* __restrict__ dy, int64_t T_rows, int64_t c_out,
                                                           int64_t seg, int nseg, float* __restrict__ part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * 4 + wave;
  if (c >= c_out) return;
  const int64_t t0 = (int64_t)blockIdx.y * seg, t1 = std::min<int64_t>(t0 + seg, T_rows);
  float a = 0.0f;
  for (int64_t t = t0 + lane; t < t1; t += 64) a += load_as_f32<T>(dy, c * T_rows + t);
  a = wave_sum(a);
  if (lane == 0) part[(int64_t)blockIdx.y * c_out + c] = a;
  (void)nseg;
}

// 64 columns per block; the chunks are dealt round-robin to four groups of lanes, whose double-precision sums are
// then added in a fixed order
__global__ __launch_bounds__(256) void k_bias_finish(const float* __restrict__ part, int64_t nchunks, int64_t c_out,
                                                     float* __restrict__ db) {
  __shared__ double red[4][64];
  const int col = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * 64 + col;
  double s = 0.0;
  if (c < c_out) {
    int64_t i = grp;
    for (; i + 28 < nchunks; i += 32) {               // eight independent loads in flight
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = part[(i + 4 * u) * c_out + c];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += (double)v[u];
    }
    for (; i < nchunks; i += 4) s += (double)part[i * c_out + c];
  }
  red[grp][col] = s;
  __syncthreads();
  if (grp == 0 && c < c_out) db[c] = (float)((red[0][col] + red[1][col]) + (red[2][col] + red[3][col]));
}

static int64_t bias_chunks(int64_t T, int64_t c_out, int layout, int64_t* seg_out) {
  if (layout == EFQAT_DY_TOKEN_MAJOR) {
    if (seg_out) *seg_out = kBiasRows;
    return ceil_div(T, kBiasRows);
  }
  // channel major: enough segments to fill the chip when there are few channels, each at least 4096 tokens long
  int64_t nseg = std::max<int64_t>(1, std::min<int64_t>(ceil_div(T, 4096), ceil_div(4096, std::max<int64_t>(c_out / 4, 1))));
  const int64_t seg = round_up(ceil_div(T, nseg), 64);
  nseg = ceil_div(T, seg);
  if (seg_out) *seg_out = seg;
  (void)c_out;
  return nseg;
}

}  // namespace efqat

using namespace efqat;

extern "C" size_t efqat_bias_grad_workspace_bytes(int64_t T, int64_t c_out, int dy_layout) {
  if (T <= 0 || c_out <= 0) return 256;
  return round_up((size_t)bias_chunks(T, c_out, dy_layout, nullptr) * (size_t)c_out * sizeof(float), 256);
}

extern "C" int efqat_bias_grad(const void* dy, int dy_dtype, int dy_layout, int64_t T, int64_t c_out, float* db,
                               void* ws, size_t ws_bytes, void* stream) {
  if (T <= 0 || c_out <= 0 || c_out > INT32_MAX) return EFQAT_ERR_BAD_SHAPE;
  if (dy_dtype != EFQAT_F32 && dy_dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (dy_layout != EFQAT_DY_TOKEN_MAJOR && dy_layout != EFQAT_DY_CHANNEL_MAJOR) return EFQAT_ERR_BAD_LAYOUT;
  if (!dy || !db || !ws) return EFQAT_ERR_NULL_PTR;
  if (ws_bytes < efqat_bias_grad_workspace_bytes(T, c_out, dy_layout)) return EFQAT_ERR_WORKSPACE;
  if (((uintptr_t)ws % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof(PROF_BIAS, st);
  float* part = (float*)ws;
  int64_t seg = 0;
  const int64_t nchunks = bias_chunks(T, c_out, dy_layout, &seg);
  if (nchunks > 65535) return EFQAT_ERR_BAD_SHAPE;
  if (dy_layout == EFQAT_DY_TOKEN_MAJOR) {
    const dim3 grid((unsigned)ceil_div(c_out, 64 * kBiasCols), (unsigned)nchunks);
    const int esz = dy_dtype == EFQAT_F32 ? 4 : 2;
    const int vec = ((c_out % kBiasCols) == 0 && ((uintptr_t)dy % 16) == 0 && (c_out * esz) % 16 == 0) ? 1 : 0;
    if (dy_dtype == EFQAT_F32)
      hipLaunchKernelGGL((k_bias_partial_tok<float>), grid, dim3(256), 0, st, (const float*)dy, T, c_out, vec, part);
    else
      hipLaunchKernelGGL((k_bias_partial_tok<bf16_t>), grid, dim3(256), 0, st, (const bf16_t*)dy, T, c_out, vec, part);
  } else {
    const dim3 grid((unsigned)ceil_div(c_out, 4), (unsigned)nchunks);
    if (dy_dtype == EFQAT_F32)
      hipLaunchKernelGGL((k_bias_partial_chan<float>), grid, dim3(256), 0, st, (const float*)dy, T, c_out, seg,
                         (int)nchunks, part);
    else
      hipLaunchKernelGGL((k_bias_partial_chan<bf16_t>), grid, dim3(256), 0, st, (const bf16_t*)dy, T, c_out, seg,
                         (int)nchunks, part);
  }
  EFQAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_bias_finish, dim3((unsigned)ceil_div(c_out, 64)), dim3(256), 0, st, part, nchunks, c_out, db);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}
