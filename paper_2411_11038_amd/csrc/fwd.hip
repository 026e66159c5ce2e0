// Low-precision forward product of a quantized linear layer (Sec. 3.1: Y = X_q W_q^T computed on integer codes):
// the 8-bit codes go straight to the int8 matrix cores, the quantizer scales and the zero point are applied
// once per output element in the epilogue.
#include "common.hpp"

namespace efqat {

// wsum[c] = sum_i w_codes[c][i]  (exact, int32).  One wavefront per output channel.
__global__ __launch_bounds__(256) void k_row_sum_i8(const int8_t* __restrict__ w, int64_t rows, int64_t cols,
                                                    int64_t ld, int32_t* __restrict__ wsum) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int8_t* p = w + row * ld;
  int acc = 0;
  if ((ld % 4) == 0 && ((uintptr_t)w % 4) == 0) {
    const int64_t n4 = cols >> 2;
    for (int64_t i = lane; i < n4; i += 64) {
      const uint32_t v = *reinterpret_cast<const uint32_t*>(p + i * 4);
      acc += (int)(int8_t)(v & 0xFF) + (int)(int8_t)((v >> 8) & 0xFF) + (int)(int8_t)((v >> 16) & 0xFF) +
             (int)(int8_t)(v >> 24);
    }
    for (int64_t i = (n4 << 2) + lane; i < cols; i += 64) acc += (int)p[i];
  } else {
    for (int64_t i = lane; i < cols; i += 64) acc += (int)p[i];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
  if (lane == 0) wsum[row] = acc;
}

// out[r][0..ldo) = in[r][0..cols) followed by zeros (byte rows; makes K a multiple of 16 for ragged widths)
__global__ __launch_bounds__(256) void k_pad_rows_u8(const uint8_t* __restrict__ in, int64_t rows, int64_t cols,
                                                     uint8_t* __restrict__ out, int64_t ldo) {
  const int64_t total = rows * ldo;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = e / ldo, j = e - r * ldo;
    out[e] = j < cols ? in[r * cols + j] : (uint8_t)0;
  }
}

struct FwdPlan {
  int64_t ldk;       // C_in rounded up to 16
  bool pad;          // operands copied into zero-padded rows
  GemmPlan plan;
  size_t b_wsum, b_xpad, b_wpad, total;
};

static FwdPlan make_fwd_plan(int64_t T, int64_t c_in, int64_t c_out) {
  FwdPlan p{};
  p.ldk = round_up(c_in, 16);
  p.pad = p.ldk != c_in;
  // one stage of the int8 product covers twice the K of a bf16 stage in the same time
  p.plan = gemm_plan(T, c_out, ceil_div(p.ldk, 2), false);
  WsCarver cv(nullptr);
  p.b_wsum = (size_t)c_out * sizeof(int32_t); cv.take(p.b_wsum);
  p.b_xpad = p.pad ? (size_t)T * p.ldk : 0; cv.take(p.b_xpad);
  p.b_wpad = p.pad ? (size_t)c_out * p.ldk : 0; cv.take(p.b_wpad);
  p.total = cv.off;
  return p;
}

}  // namespace efqat

using namespace efqat;

extern "C" size_t efqat_linear_fwd_workspace_bytes(int64_t T, int64_t c_in, int64_t c_out) {
  if (T <= 0 || c_in <= 0 || c_out <= 0) return 0;
  return make_fwd_plan(T, c_in, c_out).total;
}

extern "C" int efqat_linear_fwd(const uint8_t* x_codes, const float* s_x, const float* z_x, const int8_t* w_codes,
                                const float* s_w, int64_t T, int64_t c_in, int64_t c_out, void* y, int y_dtype,
                                void* ws, size_t ws_bytes, void* stream) {
  if (T <= 0 || c_in <= 0 || c_out <= 0 || T > (1 << 30) || c_out > (1 << 30)) return EFQAT_ERR_BAD_SHAPE;
  // (128 - Z_x) * sum_k w must fit the exact 64-bit correction and the int32 accumulators: K <= 2^17 is ample
  if (c_in > (1 << 17)) return EFQAT_ERR_BAD_SHAPE;
  if (y_dtype != EFQAT_F32 && y_dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (!x_codes || !s_x || !z_x || !w_codes || !s_w || !y || !ws) return EFQAT_ERR_NULL_PTR;
  if (((uintptr_t)ws % 256) != 0 || ((uintptr_t)y % (y_dtype == EFQAT_F32 ? 4 : 2)) != 0) return EFQAT_ERR_ALIGNMENT;
  const FwdPlan p = make_fwd_plan(T, c_in, c_out);
  if (ws_bytes < p.total) return EFQAT_ERR_WORKSPACE;
  // the tile loads are 16-byte vectors when the codes are used in place
  if (!p.pad && ((((uintptr_t)x_codes) % 16) != 0 || (((uintptr_t)w_codes) % 16) != 0)) return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  WsCarver cv(ws);
  int32_t* wsum = (int32_t*)cv.take(p.b_wsum);
  uint8_t* xpad = (uint8_t*)cv.take(p.b_xpad);
  uint8_t* wpad = (uint8_t*)cv.take(p.b_wpad);
  hipLaunchKernelGGL(k_row_sum_i8, dim3((unsigned)ceil_div(c_out, 4)), dim3(256), 0, st, w_codes, c_out, c_in, c_in,
                     wsum);
  EFQAT_LAUNCH_CHECK();
  const uint8_t* xa = x_codes;
  const int8_t* wb = w_codes;
  if (p.pad) {
    auto grid = [](int64_t n) { int64_t b = ceil_div(n, 256); return (unsigned)(b > 16384 ? 16384 : b); };
    hipLaunchKernelGGL(k_pad_rows_u8, dim3(grid(T * p.ldk)), dim3(256), 0, st, x_codes, T, c_in, xpad, p.ldk);
    EFQAT_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_pad_rows_u8, dim3(grid(c_out * p.ldk)), dim3(256), 0, st, (const uint8_t*)w_codes, c_out,
                       c_in, wpad, p.ldk);
    EFQAT_LAUNCH_CHECK();
    xa = xpad; wb = (const int8_t*)wpad;
  }
  return launch_gemm_fwd_i8(xa, p.ldk, wb, p.ldk, T, c_out, p.ldk, p.plan, s_x, z_x, s_w, wsum, y, y_dtype, st);
}
