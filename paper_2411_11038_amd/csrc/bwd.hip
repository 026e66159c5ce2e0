// EfQAT backward of one quantized layer (Alg. 1 backward step, Eq. 5): operand preparation,
// the two MFMA contractions, and the fused / second-pass epilogues that apply the straight-through
// clip masks and reduce the quantizer-parameter gradients.
#include "common.hpp"

#include <algorithm>

namespace efqat {

// ------------------------------------------------------------------------------------------------
// element readers
template <typename T> __device__ __forceinline__ float rd(const T* p, int64_t i);
template <> __device__ __forceinline__ float rd<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float rd<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
template <> __device__ __forceinline__ float rd<int8_t>(const int8_t* p, int64_t i) { return (float)p[i]; }
template <> __device__ __forceinline__ float rd<uint8_t>(const uint8_t* p, int64_t i) { return (float)p[i]; }

// Tiled transpose with conversion to bf16:
//   out[j][i] = bf16( (in[i][cm(j)] - sub) * rs(i) ),  i < R, j < Cn;  out[j][i] = 0 for R <= i < i_pad.
//   cm(j) = colmap ? colmap[j] : j     (gather of selected channels when dY is token major)
//   rs(i) = rowscale ? rowscale[i] : 1 (per-output-channel weight scale)
//   sub   = subz ? round(subz[0]) : 0  (activation zero point)
// `out` row j starts at out + j*ldo + out_off (ldo = pitch in elements).
template <typename T> struct Vec4 { };
template <> struct Vec4<float> { typedef float4 type; };
template <> struct Vec4<bf16_t> { typedef uint2 type; };
template <> struct Vec4<int8_t> { typedef uint32_t type; };
template <> struct Vec4<uint8_t> { typedef uint32_t type; };
__device__ __forceinline__ void unpack4(const float4& v, float (&o)[4]) { o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
__device__ __forceinline__ void unpack4(const uint2& v, float (&o)[4]) {
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
}
template <typename T>
__device__ __forceinline__ void unpack4b(uint32_t v, float (&o)[4]) {
#pragma unroll
  for (int t = 0; t < 4; ++t) o[t] = (float)(T)((v >> (8 * t)) & 0xFFu);
}

struct ConvGeom {
  int N, H, W, c_in, c_out, KH, KW, stride, pad, Ho, Wo;
};

// Extras of the transposing copy, all zero / off for a plain 2-D transpose.  blockIdx.z = tap of a convolution:
//   weights:      tap t reads in + t * z_in and writes at column offset out_off + t * z_out;
//   activations:  (conv = 1) source row i is an output pixel (n, ho, wo); tap t reads the input pixel
//                 (n, ho*s + kh - p, wo*s + kw - p), or contributes 0 when that lies outside the image (the
//                 padding is zero in the de-quantised domain), and writes output rows t * z_orow + j.
struct TransposeExtra {
  int64_t z_in, z_out, z_orow;
  int conv;
  ConvGeom g;
};

template <typename T>
__global__ __launch_bounds__(256) void k_transpose_bf16(const T* __restrict__ in, int64_t ld_in, int64_t R,
                                                        int64_t Cn, const int32_t* __restrict__ colmap,
                                                        const float* __restrict__ rowscale,
                                                        const float* __restrict__ subz, bf16_t* __restrict__ out,
                                                        int64_t ldo, int64_t out_off, int64_t i_pad, int vec,
                                                        uint32_t* __restrict__ zero_page, const TransposeExtra ex) {
  __shared__ bf16_t tile[64][66];                     // tile[i][j]
  // optional by-product: 256 bytes of zeros for a later kernel of the same call (saves a launch)
  if (zero_page && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x < 64)
    zero_page[threadIdx.x] = 0u;
  const int64_t i0 = (int64_t)blockIdx.x * 64, j0 = (int64_t)blockIdx.y * 64;
  const float sub = subz ? rintf(subz[0]) : 0.0f;
  const int tap = blockIdx.z;
  in += (int64_t)tap * ex.z_in;
  out += (int64_t)tap * ex.z_out + (int64_t)tap * ex.z_orow * ldo;
  // source row of logical row i, or -1: contributes zeros
  auto src_row = [&](int64_t i) -> int64_t {
    if (i >= R) return -1;
    if (!ex.conv) return i;
    const ConvGeom& g = ex.g;
    const int wo = (int)(i % g.Wo);
    const int ho = (int)((i / g.Wo) % g.Ho);
    const int n = (int)(i / ((int64_t)g.Wo * g.Ho));
    const int h = ho * g.stride + tap / g.KW - g.pad, w = wo * g.stride + tap % g.KW - g.pad;
    if (h < 0 || h >= g.H || w < 0 || w >= g.W) return -1;
    return ((int64_t)n * g.H + h) * g.W + w;
  };
  if (vec && j0 + 64 <= Cn) {
    // dense source, 4 consecutive columns per lane (one 4..16-byte load)
    const int jq = (threadIdx.x & 15) * 4, ib = threadIdx.x >> 4;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int li = ib + 16 * rr;
      const int64_t i = i0 + li;
      const int64_t si = src_row(i);
      float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (si >= 0) {
        const typename Vec4<T>::type raw = *reinterpret_cast<const typename Vec4<T>::type*>(in + si * ld_in + j0 + jq);
        if constexpr (sizeof(T) == 1) unpack4b<T>(raw, v); else unpack4(raw, v);
        const float rs = rowscale ? rowscale[i] : 1.0f;
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = (v[t] - sub) * rs;
      }
      *reinterpret_cast<uint32_t*>(&tile[li][jq]) = pack_bf16x2(v[0], v[1]);
      *reinterpret_cast<uint32_t*>(&tile[li][jq + 2]) = pack_bf16x2(v[2], v[3]);
    }
  } else {
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t j = j0 + tx;
    const int64_t jc = (j < Cn) ? (colmap ? (int64_t)colmap[j] : j) : 0;
#pragma unroll 4
    for (int rr = 0; rr < 16; ++rr) {
      const int li = ty + 4 * rr;
      const int64_t i = i0 + li;
      const int64_t si = src_row(i);
      float v = 0.0f;
      if (si >= 0 && j < Cn) {
        v = rd<T>(in, si * ld_in + jc) - sub;
        if (rowscale) v *= rowscale[i];
      }
      tile[li][tx] = f32_to_bf16(v);
    }
  }
  __syncthreads();
  // out[j][i0 + 8a .. 8a+7]: one 16-byte store per lane, 8 lanes cover the 128 bytes of one output row
  const int a8 = (threadIdx.x & 7) * 8, jb = threadIdx.x >> 3;
#pragma unroll
  for (int ww = 0; ww < 2; ++ww) {
    const int lj = jb + 32 * ww;
    const int64_t jo = j0 + lj, io = i0 + a8;
    if (jo < Cn && io < i_pad) {
      uint32_t w[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) w[t] = (uint32_t)tile[a8 + 2 * t][lj] | ((uint32_t)tile[a8 + 2 * t + 1][lj] << 16);
      *reinterpret_cast<uint4*>(out + jo * ldo + out_off + io) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

// Row-wise cast/copy to bf16 with zero-padded pitch: out[m][j] = bf16(in[rm(m)][j]), j < Cn; 0 up to ldo.
template <typename T>
__global__ __launch_bounds__(256) void k_rows_bf16(const T* __restrict__ in, int64_t ld_in, int64_t R, int64_t Cn,
                                                   const int32_t* __restrict__ rowmap, bf16_t* __restrict__ out,
                                                   int64_t ldo) {
  const int64_t total = R * ldo;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t m = e / ldo, j = e - m * ldo;
    float v = 0.0f;
    if (j < Cn) v = rd<T>(in, (rowmap ? (int64_t)rowmap[m] : m) * ld_in + j);
    out[e] = f32_to_bf16(v);
  }
}

// 256 zero bytes that tile loads read in place of rows / columns outside an operand
__global__ void k_zero_page(uint32_t* __restrict__ p) { p[threadIdx.x] = 0u; }

// Compaction of the selected output channels of a token-major dY (the channel extraction step of Alg. 1, done
// once per call):  out[t][m] = bf16(dY[t][idx[m]]), m < k;  0 for k <= m < kp.
// A lane owns two neighbouring compacted channels (their source columns stay in registers); a wavefront thus
// reads 128 selected channels of one token - a span of a few cache lines, since idx ascends - and writes 256
// contiguous bytes.  The four wavefronts of a block take every fourth token row of the block's row range.
constexpr int kGatherRows = 32;                       // token rows per block
template <typename T>
__global__ __launch_bounds__(256) void k_gather_cols(const T* __restrict__ dy, int64_t ld, int64_t rows,
                                                     const int32_t* __restrict__ idx, int64_t k,
                                                     bf16_t* __restrict__ out, int64_t kp) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t m0 = 2 * ((int64_t)blockIdx.x * 64 + lane);
  if (m0 >= kp) return;
  const int64_t c0 = m0 < k ? (int64_t)idx[m0] : -1, c1 = m0 + 1 < k ? (int64_t)idx[m0 + 1] : -1;
  for (int64_t t0 = (int64_t)blockIdx.y * kGatherRows; t0 < rows; t0 += (int64_t)gridDim.y * kGatherRows) {
    float a[kGatherRows / 4], b[kGatherRows / 4];
#pragma unroll
    for (int r = 0; r < kGatherRows / 4; ++r) {
      const int64_t t = t0 + wave + 4 * r;
      a[r] = (c0 >= 0 && t < rows) ? rd<T>(dy, t * ld + c0) : 0.0f;
      b[r] = (c1 >= 0 && t < rows) ? rd<T>(dy, t * ld + c1) : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < kGatherRows / 4; ++r) {
      const int64_t t = t0 + wave + 4 * r;
      if (t < rows) *reinterpret_cast<uint32_t*>(out + t * kp + m0) = pack_bf16x2(a[r], b[r]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// conv helpers (explicit im2col into workspace; the contractions then run on the same GEMM core)
// dX operand: colA[(n,h,w)][tap*ldc + co] = dYn[(n,ho,wo)][co] with ho*stride + kh - pad = h (else 0).
// dYn is the token-major bf16 copy of dY with pitch ldc (multiple of 8).
__global__ __launch_bounds__(256) void k_im2col_dy(const bf16_t* __restrict__ dyn, int64_t ldc, ConvGeom g,
                                                   bf16_t* __restrict__ col) {
  const int64_t ch = ldc >> 3;                        // 16-byte chunks per tap
  const int taps = g.KH * g.KW;
  const int64_t total = (int64_t)g.N * g.H * g.W * taps * ch;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t c8 = e % ch;
    int64_t r = e / ch;
    const int tap = (int)(r % taps);
    r /= taps;                                        // pixel index (n,h,w)
    const int w = (int)(r % g.W);
    const int h = (int)((r / g.W) % g.H);
    const int n = (int)(r / ((int64_t)g.W * g.H));
    const int kh = tap / g.KW, kw = tap % g.KW;
    const int hn = h + g.pad - kh, wn = w + g.pad - kw;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (hn >= 0 && wn >= 0 && hn % g.stride == 0 && wn % g.stride == 0) {
      const int ho = hn / g.stride, wo = wn / g.stride;
      if (ho < g.Ho && wo < g.Wo)
        v = *reinterpret_cast<const uint4*>(dyn + (((int64_t)n * g.Ho + ho) * g.Wo + wo) * ldc + c8 * 8);
    }
    *reinterpret_cast<uint4*>(col + (r * taps + tap) * ldc + c8 * 8) = v;
  }
}

// ------------------------------------------------------------------------------------------------
// dS_x, dZ_x: ordered sum of the per-block partials written by the dX epilogue.
template <int NTH>
__device__ __forceinline__ void sum_partials_block(const float* __restrict__ part, int64_t n,
                                                   float* __restrict__ ds_x, float* __restrict__ dz_x) {
  constexpr int NW = NTH / 64;
  double a = 0.0, b = 0.0;
  for (int64_t i = threadIdx.x; i < n; i += NTH) { a += (double)part[2 * i]; b += (double)part[2 * i + 1]; }
  a = wave_sum(a); b = wave_sum(b);
  __shared__ double sa[NW], sb[NW];
  if ((threadIdx.x & 63) == 0) { sa[threadIdx.x >> 6] = a; sb[threadIdx.x >> 6] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double ta = 0.0, tb = 0.0;
#pragma unroll
    for (int w = 0; w < NW; w += 4) {                  // fixed order
      ta += (sa[w] + sa[w + 1]) + (sa[w + 2] + sa[w + 3]);
      tb += (sb[w] + sb[w + 1]) + (sb[w + 2] + sb[w + 3]);
    }
    ds_x[0] = (float)ta;
    dz_x[0] = (float)tb;
  }
}

__global__ __launch_bounds__(256) void k_sum_partials(const float* __restrict__ part, int64_t n,
                                                      float* __restrict__ ds_x, float* __restrict__ dz_x) {
  sum_partials_block<256>(part, n, ds_x, dz_x);
}

// Optional optimizer step fused into the second pass (off when w == nullptr), the rule of Alg. 1's optimizer step for
// unfrozen channels.  Weight rows idx: SGD with momentum and weight decay, the optimizer the network parameters keep from
// the full-precision run:  g = dW + wd * W;  buf = mu * buf + g;  W -= lr_w * buf  (buf is skipped when mu == 0).
// Their scales S_w[idx]: Adam, which the quantization parameters are always trained with (Sec. 4 "Setup"), one state
// and step count per channel:  t += 1;  m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;
// S_w -= lr_s * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).
struct StepArgs {
  float* w; float* mom_w;
  float lr_w, mu, wd;
  float* s_w; float* adam_m; float* adam_v; int32_t* adam_t;
  float lr_s, b1, b2, eps;
};

// Second pass of the restricted weight gradient: ordered split-K sum, S_x scaling, straight-through mask
// of the weight quantizer and the per-row scale gradient
//   dW[c][j] = in range ? dW_q : 0,  dS_w[c] = sum_j dW_q * (in range ? code - w/S_w : code),  c = idx[m].
// One block of NTH threads per row: 256, or 1024 for long rows, so that a row is one trip through the loop.
template <int NTH>
__global__ __launch_bounds__(NTH) void k_dw_finish(const float* __restrict__ part, int S, int64_t k, int64_t ncols,
                                                   int vec, const float* __restrict__ s_x,
                                                   const int8_t* __restrict__ w_codes,
                                                   const uint32_t* __restrict__ w_clip, const float* __restrict__ w,
                                                   const float* __restrict__ s_w, const int32_t* __restrict__ idx,
                                                   float* __restrict__ dw, int scatter, float* __restrict__ ds_w,
                                                   const float* __restrict__ part_dx, int64_t n_part_dx,
                                                   float* __restrict__ ds_x, float* __restrict__ dz_x,
                                                   const StepArgs sgd) {
  if ((int64_t)blockIdx.x == k) {                     // one extra block: dS_x, dZ_x from the dX epilogue's partials
    sum_partials_block<NTH>(part_dx, n_part_dx, ds_x, dz_x);
    return;
  }
  const int64_t m = blockIdx.x;
  const int64_t c = idx[m];
  const int64_t wpr = (ncols + 31) >> 5;
  const float sx = s_x[0];
  const float sw = s_w[c];
  const int64_t orow = scatter ? c : m;
  const int64_t slice = k * ncols;
  float acc = 0.0f;
  if (vec) {                                          // ncols % 4 == 0 and 16-byte aligned rows
    for (int64_t j = (int64_t)threadIdx.x * 4; j < ncols; j += 4 * NTH) {
      const float* p = part + m * ncols + j;
      float4 a = *reinterpret_cast<const float4*>(p);
      int s = 1;
      for (; s + 3 < S; s += 4) {                     // four slices in flight; summed in slice order as below
        float4 b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) b[u] = *reinterpret_cast<const float4*>(p + (int64_t)(s + u) * slice);
#pragma unroll
        for (int u = 0; u < 4; ++u) { a.x += b[u].x; a.y += b[u].y; a.z += b[u].z; a.w += b[u].w; }
      }
      for (; s < S; ++s) {
        const float4 b = *reinterpret_cast<const float4*>(p + (int64_t)s * slice);
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
      }
      const float dwq[4] = {sx * a.x, sx * a.y, sx * a.z, sx * a.w};
      const uint32_t bits = w_clip[c * wpr + (j >> 5)] >> (j & 31);
      const uint32_t cw = *reinterpret_cast<const uint32_t*>(w_codes + c * ncols + j);
      const float4 wv = *reinterpret_cast<const float4*>(w + c * ncols + j);
      const float wf[4] = {wv.x, wv.y, wv.z, wv.w};
      float o[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bool inr = (bits >> t) & 1u;
        const float code = (float)(int8_t)((cw >> (8 * t)) & 0xFFu);
        const float gs = inr ? (code - wf[t] / sw) : code;
        acc += dwq[t] * gs;
        o[t] = inr ? dwq[t] : 0.0f;
      }
      if (dw) *reinterpret_cast<float4*>(dw + orow * ncols + j) = make_float4(o[0], o[1], o[2], o[3]);
      if (sgd.w) {
        float gq[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) gq[t] = fmaf(sgd.wd, wf[t], o[t]);
        if (sgd.mom_w) {
          float4 mb = *reinterpret_cast<const float4*>(sgd.mom_w + c * ncols + j);
          mb.x = fmaf(sgd.mu, mb.x, gq[0]); mb.y = fmaf(sgd.mu, mb.y, gq[1]);
          mb.z = fmaf(sgd.mu, mb.z, gq[2]); mb.w = fmaf(sgd.mu, mb.w, gq[3]);
          *reinterpret_cast<float4*>(sgd.mom_w + c * ncols + j) = mb;
          gq[0] = mb.x; gq[1] = mb.y; gq[2] = mb.z; gq[3] = mb.w;
        }
        *reinterpret_cast<float4*>(sgd.w + c * ncols + j) =
            make_float4(fmaf(-sgd.lr_w, gq[0], wf[0]), fmaf(-sgd.lr_w, gq[1], wf[1]), fmaf(-sgd.lr_w, gq[2], wf[2]),
                        fmaf(-sgd.lr_w, gq[3], wf[3]));
      }
    }
  } else {
    for (int64_t j = threadIdx.x; j < ncols; j += NTH) {
      float a = 0.0f;
      for (int s = 0; s < S; ++s) a += part[(int64_t)s * slice + m * ncols + j];
      const float dwq = sx * a;
      const bool inr = (w_clip[c * wpr + (j >> 5)] >> (j & 31)) & 1u;
      const float code = (float)w_codes[c * ncols + j];
      const float wv = w[c * ncols + j];
      const float gs = inr ? (code - wv / sw) : code;
      acc += dwq * gs;
      const float ov = inr ? dwq : 0.0f;
      if (dw) dw[orow * ncols + j] = ov;
      if (sgd.w) {
        float gq = fmaf(sgd.wd, wv, ov);
        if (sgd.mom_w) {
          gq = fmaf(sgd.mu, sgd.mom_w[c * ncols + j], gq);
          sgd.mom_w[c * ncols + j] = gq;
        }
        sgd.w[c * ncols + j] = fmaf(-sgd.lr_w, gq, wv);
      }
    }
  }
  acc = wave_sum(acc);
  __shared__ float red[NTH / 64];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float ds = 0.0f;
#pragma unroll
    for (int w = 0; w < NTH / 64; w += 4) ds += (red[w] + red[w + 1]) + (red[w + 2] + red[w + 3]);   // fixed order
    if (ds_w) ds_w[orow] = ds;
    if (sgd.s_w) {
      // one scalar per row: double precision costs nothing here and leaves only the fp32 storage rounding
      const int t = sgd.adam_t[c] + 1;
      const double g = (double)ds, b1 = (double)sgd.b1, b2 = (double)sgd.b2;
      const double m = b1 * (double)sgd.adam_m[c] + (1.0 - b1) * g;
      const double v = b2 * (double)sgd.adam_v[c] + (1.0 - b2) * g * g;
      const double m_hat = m / (1.0 - pow(b1, (double)t)), v_hat = v / (1.0 - pow(b2, (double)t));
      sgd.adam_t[c] = t;
      sgd.adam_m[c] = (float)m;
      sgd.adam_v[c] = (float)v;
      sgd.s_w[c] = (float)((double)sw - (double)sgd.lr_s * m_hat / (sqrt(v_hat) + (double)sgd.eps));
    }
  }
}

// ------------------------------------------------------------------------------------------------
static inline unsigned grid1d(int64_t total, int per_block = 256) {
  int64_t b = ceil_div(total, per_block);
  if (b > 256 * 64) b = 256 * 64;
  if (b < 1) b = 1;
  return (unsigned)b;
}

template <typename T>
static int transpose_to_bf16(const T* in, int64_t ld_in, int64_t R, int64_t Cn, const int32_t* colmap,
                             const float* rowscale, const float* subz, bf16_t* out, int64_t ldo, int64_t out_off,
                             int64_t i_pad, hipStream_t st, uint32_t* zero_page = nullptr, int taps = 1,
                             const TransposeExtra* extra = nullptr) {
  dim3 grid((unsigned)ceil_div(i_pad, 64), (unsigned)ceil_div(Cn, 64), (unsigned)taps);
  TransposeExtra ex{};
  if (extra) ex = *extra;
  if (grid.y > 65535) return EFQAT_ERR_BAD_SHAPE;
  // 16-byte stores need an 8-element aligned destination; 4-wide loads a dense, 4-element aligned source
  if ((ldo % 8) || (out_off % 8) || (i_pad % 8) || ((uintptr_t)out % 16)) return EFQAT_ERR_ALIGNMENT;
  const int vec = (!colmap && (ld_in % 4) == 0 && ((uintptr_t)in % (4 * sizeof(T))) == 0) ? 1 : 0;
  hipLaunchKernelGGL((k_transpose_bf16<T>), grid, dim3(256), 0, st, in, ld_in, R, Cn, colmap, rowscale, subz, out,
                     ldo, out_off, i_pad, vec, zero_page, ex);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

// Plan of one backward call: sizes of every workspace slice (shared by the size query and the call).
struct BwdPlan {
  int64_t Mx;      // rows of dX as a matrix (T, or N*H*W)
  int64_t Kx;      // contraction length of the dX product (padded C_out, times taps for conv)
  int64_t Nw;      // columns of dW as a matrix (C_in, or KH*KW*C_in)
  int64_t Tw;      // contraction length of the dW product (T, or N*Ho*Wo)
  int64_t ldc;     // C_out rounded up to 8
  int64_t ldt;     // Tw rounded up to 8
  bool need_dyn;   // token-major bf16 copy of dY needed
  bool need_sel;   // gathered dY^T rows materialised (token-major dY, or fp32 / unaligned channel-major)
  bool tn;         // dW product straight from token-major dY columns and the uint8 codes (no transposed copies)
  bool tn_direct;  // ... with dY itself as the A operand (all channels selected)
  bool cmx;        // channel-major dY: dX product straight from dY [C_out][T] and the int8 weight codes
  bool rdw;        // channel-major dY: dW product from the selected rows of dY and the uint8 codes, nothing staged
  bool cdw;        // convolution dW product with the im2col gather of the codes inside the tile loads
  bool cdx;        // convolution dX product with the im2col gather inside the tile loads (no im2col matrix)
  bool dx8;        // dX product with the weight operand read from the int8 codes (no bf16 W_q^T copy)
  bool kk;         // dX product from the bf16 copies by the 192 x 192 kernel with the pinned instruction order
  int dx8_tile;
  int64_t kp;      // k rounded up to 8 (pitch of the compacted dY columns)
  GemmPlan plan_dx, plan_dw;
  size_t b_wqT, b_dyn, b_colA, b_part_dx, b_xcT, b_sel, b_part_dw, b_zero, total;
};

// dxk: the caller's choice of the dX kernel (EFQAT_DX_KERNEL_*); it changes workspace sizes, so the size query takes
// it as well.  io_bf16: x and dX are both bf16 (known at the call, not at the workspace query: nothing it changes
// may change a workspace size).
static BwdPlan make_plan(int64_t T_in, int64_t T_out, int64_t c_in, int64_t c_out, int taps, int64_t k,
                         int dy_dtype, int dy_layout, bool im2col, int dxk, const ConvGeom* cg = nullptr,
                         bool io_bf16 = false) {
  BwdPlan p{};
  p.Mx = T_in; p.Tw = T_out; p.Nw = (int64_t)taps * c_in;
  p.ldc = round_up(c_out, 8); p.ldt = round_up(T_out, 8);
  p.Kx = (int64_t)taps * p.ldc;
  const bool direct_tok = dy_layout == EFQAT_DY_TOKEN_MAJOR && dy_dtype == EFQAT_BF16 && (c_out % 8) == 0;
  p.need_dyn = !direct_tok;
  const bool direct_rows = dy_layout == EFQAT_DY_CHANNEL_MAJOR && dy_dtype == EFQAT_BF16 && (T_out % 8) == 0;
  p.cdw = k > 0 && dy_layout == EFQAT_DY_TOKEN_MAJOR && im2col && cg && (c_in % 128) == 0;
  p.tn = k > 0 && dy_layout == EFQAT_DY_TOKEN_MAJOR && ((!im2col && (c_in % 16) == 0) || p.cdw);
  p.tn_direct = p.tn && direct_tok && k == c_out;
  p.rdw = k > 0 && direct_rows && !im2col && (c_in % 16) == 0;
  p.cmx = direct_rows && !im2col && taps == 1 && (c_in % 16) == 0 && dxk != EFQAT_DX_KERNEL_BF16_PINNED;
  if (p.cmx) p.need_dyn = false;
  p.kp = round_up(k, 8);
  p.need_sel = k > 0 && !direct_rows && !p.tn_direct;
  // stride-1 convolutions whose channel pitch is a multiple of the 64-element K stage gather dY in the tile loads
  p.cdx = im2col && cg && cg->stride == 1 && (p.ldc % 64) == 0 && cg->H <= 65535 && cg->W <= 65535;
  p.plan_dx = gemm_plan(p.Mx, c_in, p.Kx, false, true, !p.cdx);
  p.dx8 = false; p.dx8_tile = 0;
  // Large products (the planner's 256 x 256 case) with a bf16 token-major dY read the weight operand straight
  // from the int8 codes: same speed as the bf16 kernel on these shapes, and no transposed bf16 copy of W_q.
  if (p.cmx) {
    p.plan_dx = gemm_plan(p.Mx, c_in, p.Kx, false, false);
    p.dx8 = true; p.dx8_tile = p.plan_dx.tile;
  } else if (dxk == EFQAT_DX_KERNEL_BF16_PINNED) {
    if (!p.cdx) {
      p.plan_dx.tile = 192; p.plan_dx.split_k = 1;
      p.plan_dx.tiles_m = (int)ceil_div(p.Mx, 192); p.plan_dx.tiles_n = (int)ceil_div(c_in, 192);
    }
  } else if (taps == 1 && !im2col && direct_tok && (c_in % 16) == 0 && dxk != EFQAT_DX_KERNEL_BF16 &&
      (p.plan_dx.tile == 256 || dxk == EFQAT_DX_KERNEL_INT8)) {
    p.dx8 = true; p.dx8_tile = (p.plan_dx.tile == 256 || (p.Mx >= 1024 && c_in >= 512)) ? 256 : 128;
    p.plan_dx.tiles_m = (int)ceil_div(p.Mx, p.dx8_tile); p.plan_dx.tiles_n = (int)ceil_div(c_in, p.dx8_tile);
  }
  // bf16 in and out, whole 192 x 192 tiles: the pinned kernel with its straight-line epilogue changes the ranking of
  // the tiles below 256 (the workspace slices do not depend on the outcome)
  if (!p.dx8 && !p.cdx && io_bf16 && p.plan_dx.tile != 256 && (p.Mx % 192) == 0 && (c_in % 192) == 0 &&
      p.Mx * c_in <= (int64_t)INT32_MAX && dxk != EFQAT_DX_KERNEL_BF16_PINNED)
    p.plan_dx = gemm_plan(p.Mx, c_in, p.Kx, false, true, false, true);
  // 128 x 128 tiles that leave at most one block per compute unit anyway (<= 256 tiles) also take the three-stage
  // ring: a lone block has nothing else to cover the load latency with (1 x 1 convolution of cfg4: 18 -> 14 us)
  p.kk = !p.dx8 && !p.cdx &&
         (p.plan_dx.tile == 192 || (p.plan_dx.tile == 128 && (int64_t)p.plan_dx.tiles_m * p.plan_dx.tiles_n <= 256));
  p.plan_dw = k > 0 ? gemm_plan(k, p.Nw, p.ldt, true, !(p.tn || p.rdw), !p.cdw) : GemmPlan{128, 1, 0, 0};
  WsCarver cv(nullptr);
  p.b_wqT = p.dx8 ? 0 : (size_t)c_in * p.Kx * 2; cv.take(p.b_wqT);
  p.b_dyn = p.need_dyn ? (size_t)T_out * p.ldc * 2 : 0; cv.take(p.b_dyn);
  p.b_colA = (im2col && !p.cdx) ? (size_t)T_in * p.Kx * 2 : 0; cv.take(p.b_colA);
  // one (dS_x, dZ_x) pair per tile: sized for the smallest tile, whichever kernel runs
  p.b_part_dx = (size_t)std::max<int64_t>(ceil_div(p.Mx, 128) * ceil_div(c_in, 128),
                                          (int64_t)p.plan_dx.tiles_m * p.plan_dx.tiles_n) * 2 * sizeof(float);
  cv.take(p.b_part_dx);
  p.b_xcT = (k > 0 && !p.tn && !p.rdw) ? (size_t)p.Nw * p.ldt * 2 : 0; cv.take(p.b_xcT);
  p.b_sel = p.need_sel ? (p.tn ? (size_t)T_out * p.kp * 2 : (size_t)k * p.ldt * 2) : 0; cv.take(p.b_sel);
  p.b_zero = 256; cv.take(p.b_zero);
  p.b_part_dw = k > 0 ? (size_t)p.plan_dw.split_k * k * p.Nw * sizeof(float) : 0; cv.take(p.b_part_dw);
  p.total = cv.off;
  return p;
}

struct BwdIo {
  const void* dy; int dy_dtype; int dy_layout;
  const uint8_t* x_codes; const uint32_t* x_clip; const void* x; int x_dtype; const float* s_x; const float* z_x;
  const int8_t* w_codes; const uint32_t* w_clip; const float* w; const float* s_w; const int32_t* idx; int64_t k;
  void* dx; int dx_dtype; float* dw; int scatter; float* ds_w; float* ds_x; float* dz_x;
  StepArgs sgd;    // fused optimizer step (sgd.w == nullptr: none)
  const void* w_operand = nullptr;   // optional: the bf16 W_q^T matrix (then 256 zero bytes) made beforehand
  hipStream_t side = nullptr;        // optional: second stream for the weight-gradient branch
};

// Fork / join events of the optional second stream: one pair per host thread and device, made at first use and kept
// (recording an event again while an earlier wait on it is still queued is well defined: a wait refers to the
// record that preceded it).
struct SideEvents { hipEvent_t fork, join; };
static int side_events(SideEvents* out) {
  constexpr int kMaxDev = 64;
  thread_local SideEvents ev[kMaxDev];
  thread_local bool have[kMaxDev] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return EFQAT_ERR_HIP;
  if (!have[dev]) {
    if (hipEventCreateWithFlags(&ev[dev].fork, hipEventDisableTiming) != hipSuccess) return EFQAT_ERR_HIP;
    if (hipEventCreateWithFlags(&ev[dev].join, hipEventDisableTiming) != hipSuccess) return EFQAT_ERR_HIP;
    have[dev] = true;
  }
  *out = ev[dev];
  return EFQAT_OK;
}

// Everything that can still fail once the plan is known, checked before the first launch: pointer alignment of the
// operands that the chosen kernels copy 16 bytes at a time, and the grid limits of the staging kernels.
static int check_plan(const BwdPlan& p, const BwdIo& io, int64_t T_out, int64_t c_in, int64_t c_out, bool im2col) {
  if (p.dx8 && ((uintptr_t)io.w_codes % 16) != 0) return EFQAT_ERR_ALIGNMENT;
  if ((p.tn || p.rdw) && ((uintptr_t)io.x_codes % 16) != 0) return EFQAT_ERR_ALIGNMENT;
  const int64_t ymax = 65535 * (int64_t)64;           // the transposing copies put 64 source columns on grid.y
  if (!p.dx8 && !io.w_operand && c_in > ymax) return EFQAT_ERR_BAD_SHAPE;
  if (p.need_dyn && io.dy_layout == EFQAT_DY_CHANNEL_MAJOR && T_out > ymax) return EFQAT_ERR_BAD_SHAPE;
  if (io.k > 0 && !p.tn && !p.rdw && (c_in > ymax || io.k > ymax)) return EFQAT_ERR_BAD_SHAPE;
  // 32-bit per-stage pointer steps of the kernels that read operands as they lie
  if ((p.dx8 || p.tn || p.rdw) && (c_in >= (1 << 24) || c_out >= (1 << 24))) return EFQAT_ERR_BAD_SHAPE;
  if ((p.cmx || p.rdw) && T_out >= (1 << 24)) return EFQAT_ERR_BAD_SHAPE;
  (void)im2col;
  return EFQAT_OK;
}

// Shared driver.  For conv, T_in = N*H*W input pixels, T_out = N*Ho*Wo output pixels; for linear both are T.
static int run_bwd(const BwdIo& io, const BwdPlan& p, int64_t T_in, int64_t T_out, int64_t c_in, int64_t c_out,
                   const ConvGeom* cg, void* ws, hipStream_t st) {
  const int taps = cg ? cg->KH * cg->KW : 1;
  // a 1x1 / stride 1 / no-padding convolution is a linear layer over pixels: no im2col needed
  const bool im2col = cg != nullptr && !(taps == 1 && cg->stride == 1 && cg->pad == 0);
  WsCarver cv(ws);
  bf16_t* wqT = (bf16_t*)cv.take(p.b_wqT);
  bf16_t* dyn = (bf16_t*)cv.take(p.b_dyn);
  bf16_t* colA = (bf16_t*)cv.take(p.b_colA);
  float* part_dx = (float*)cv.take(p.b_part_dx);
  bf16_t* xcT = (bf16_t*)cv.take(p.b_xcT);
  bf16_t* sel = (bf16_t*)cv.take(p.b_sel);
  void* zero_page = cv.take(p.b_zero);
  float* part_dw = (float*)cv.take(p.b_part_dw);
  int rc;

  ProfScope prep(PROF_PREP, st);                       // operand preparation ahead of the dX product
  // ---- W_q^T in bf16:  wqT[ci][tap*ldc + co] = S_w[co] * code[co][tap][ci], zero for co in [c_out, ldc)
  if (!p.dx8 && io.w_operand) {
    // made beforehand by efqat_linear_bwd_weight_operand (same kernel, same bits), with its own zero page behind it
    wqT = (bf16_t*)const_cast<void*>(io.w_operand);
    zero_page = (char*)const_cast<void*>(io.w_operand) + round_up((int64_t)p.b_wqT, 256);
  } else if (p.dx8) {
    hipLaunchKernelGGL(k_zero_page, dim3(1), dim3(64), 0, st, (uint32_t*)zero_page);
    EFQAT_LAUNCH_CHECK();
  } else {
    TransposeExtra ex{};
    ex.z_in = c_in; ex.z_out = p.ldc;                 // one launch for all taps
    rc = transpose_to_bf16<int8_t>(io.w_codes, (int64_t)taps * c_in, c_out, c_in, nullptr, io.s_w, nullptr, wqT,
                                   p.Kx, 0, p.ldc, st, p.b_zero ? (uint32_t*)zero_page : nullptr, taps, &ex);
    if (rc) return rc;
  }

  // ---- optional second stream.  The weight-gradient branch (compaction of the selected columns of dY, dW product)
  // reads the call's inputs and the zero page only, so it may run beside the dX product: blocks of the two products
  // then share the compute units, and neither leaves a partly filled last round behind.  It is forked here, behind
  // everything the caller's stream held before the call and behind the zero page, and joined before the second
  // pass of the weight gradient.
  const bool use_side = io.side && io.side != st && io.k > 0 && (p.tn || p.rdw);
  hipStream_t st2 = st;
  SideEvents ev{};
  if (use_side) {
    rc = side_events(&ev);
    if (rc) return rc;
    if (hipEventRecord(ev.fork, st) != hipSuccess || hipStreamWaitEvent(io.side, ev.fork, 0) != hipSuccess)
      return EFQAT_ERR_HIP;
    st2 = io.side;
  }

  // ---- dY as a token-major bf16 matrix [T_out][ldc] (A operand of the dX product)
  const bf16_t* dy_tok = (const bf16_t*)io.dy;
  if (p.need_dyn) {
    if (io.dy_layout == EFQAT_DY_TOKEN_MAJOR) {
      if (io.dy_dtype == EFQAT_F32)
        hipLaunchKernelGGL((k_rows_bf16<float>), dim3(grid1d(T_out * p.ldc)), dim3(256), 0, st, (const float*)io.dy,
                           c_out, T_out, c_out, nullptr, dyn, p.ldc);
      else
        hipLaunchKernelGGL((k_rows_bf16<bf16_t>), dim3(grid1d(T_out * p.ldc)), dim3(256), 0, st,
                           (const bf16_t*)io.dy, c_out, T_out, c_out, nullptr, dyn, p.ldc);
      EFQAT_LAUNCH_CHECK();
    } else {
      // channel-major [c_out][T_out] -> [T_out][ldc]
      if (io.dy_dtype == EFQAT_F32)
        rc = transpose_to_bf16<float>((const float*)io.dy, T_out, c_out, T_out, nullptr, nullptr, nullptr, dyn,
                                      p.ldc, 0, p.ldc, st);
      else
        rc = transpose_to_bf16<bf16_t>((const bf16_t*)io.dy, T_out, c_out, T_out, nullptr, nullptr, nullptr, dyn,
                                       p.ldc, 0, p.ldc, st);
      if (rc) return rc;
    }
    dy_tok = dyn;
  }

  // ---- dX product with the fused straight-through / qparam epilogue
  const bf16_t* A = dy_tok;
  int64_t lda = p.ldc;
  if (im2col && !p.cdx) {
    hipLaunchKernelGGL(k_im2col_dy, dim3(grid1d(T_in * taps * (p.ldc / 8))), dim3(256), 0, st, dy_tok, p.ldc, *cg,
                       colA);
    EFQAT_LAUNCH_CHECK();
    A = colA; lda = p.Kx;
  }
  prep.close();
  GemmEpilogueDx epi{io.x_codes, io.x_clip, io.x, io.x_dtype, io.s_x, io.z_x, io.dx, io.dx_dtype, part_dx};
  if (p.dx8) {
    if (p.cmx)
      rc = launch_gemm_dx8_cm((const bf16_t*)io.dy, T_out, io.w_codes, c_in, io.s_w, zero_page, p.Mx, c_in, c_out,
                              p.dx8_tile, epi, st);
    else
      rc = launch_gemm_dx8(dy_tok, c_out, io.w_codes, c_in, io.s_w, zero_page, p.Mx, c_in, c_out, p.dx8_tile, epi, st);
  } else if (p.cdx) {
    const ConvDxMap cm{cg->H, cg->W, cg->Ho, cg->Wo, cg->KW, cg->pad, zero_page};
    rc = launch_gemm_nt_conv_dx(dy_tok, p.ldc, wqT, p.Kx, p.Mx, c_in, p.Kx, cm, p.plan_dx, epi, st);
  } else if (p.kk) {
    rc = launch_gemm_kk(A, lda, wqT, p.Kx, zero_page, p.Mx, c_in, p.Kx, p.plan_dx, nullptr, &epi, st);
  } else {
    rc = launch_gemm_nt(A, lda, nullptr, wqT, p.Kx, p.Mx, c_in, p.Kx, p.plan_dx, nullptr, &epi, st);
  }
  if (rc) return rc;
  const int64_t n_part_dx = (int64_t)p.plan_dx.tiles_m * p.plan_dx.tiles_n;
  if (io.k == 0) {
    ProfScope fin(PROF_FINISH, st);
    hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(256), 0, st, part_dx, n_part_dx, io.ds_x, io.dz_x);
    EFQAT_LAUNCH_CHECK();
    return EFQAT_OK;
  }

  if (p.tn) {
    // ---- dW product straight from token-major operands: A = the selected columns of dY (compacted once, or dY
    // itself when every channel is selected), B = the uint8 codes; transposition happens in the LDS reads
    const bf16_t* At = (const bf16_t*)io.dy;
    int64_t ldat = c_out, acols = c_out;
    if (!p.tn_direct) {
      ProfScope gat(PROF_PREP, st2);
      const dim3 ggrid((unsigned)ceil_div(p.kp, 128), (unsigned)std::min<int64_t>(ceil_div(T_out, kGatherRows), 65535));
      if (io.dy_dtype == EFQAT_F32)
        hipLaunchKernelGGL((k_gather_cols<float>), ggrid, dim3(256), 0, st2, (const float*)io.dy, c_out, T_out, io.idx,
                           io.k, sel, p.kp);
      else
        hipLaunchKernelGGL((k_gather_cols<bf16_t>), ggrid, dim3(256), 0, st2, (const bf16_t*)io.dy, c_out, T_out,
                           io.idx, io.k, sel, p.kp);
      EFQAT_LAUNCH_CHECK();
      At = sel; ldat = p.kp; acols = p.kp;
    }
    if (p.cdw) {
      const ConvDwMap cm{cg->H, cg->W, cg->Ho, cg->Wo, cg->KW, cg->stride, cg->pad, (int)c_in};
      rc = launch_gemm_tn_conv(At, ldat, acols, io.x_codes, cm, zero_page, io.z_x, io.k, p.Nw, T_out, p.plan_dw,
                               part_dw, st2);
    } else {
      rc = launch_gemm_tn(At, ldat, acols, io.x_codes, c_in, c_in, zero_page, io.z_x, io.k, p.Nw, T_out, p.plan_dw,
                          part_dw, st2);
    }
    if (rc) return rc;
  } else if (p.rdw) {
    // ---- channel-major dY: the selected rows are gathered by the tile loads, the codes are read as they lie
    rc = launch_gemm_dw_rows((const bf16_t*)io.dy, T_out, io.idx, io.x_codes, c_in, zero_page, io.z_x, io.k, p.Nw,
                             T_out, p.plan_dw, part_dw, st2);
    if (rc) return rc;
  } else {
  ProfScope stg(PROF_PREP, st);                        // staged bf16 operands of the fall-back product
  // ---- B operand of the dW product: (codes - Z_x)^T, exact in bf16
  if (im2col) {
    TransposeExtra ex{};
    ex.z_orow = c_in; ex.conv = 1; ex.g = *cg;        // xcT[(tap, ci)][(n, ho, wo)], one launch for all taps
    rc = transpose_to_bf16<uint8_t>(io.x_codes, c_in, T_out, c_in, nullptr, nullptr, io.z_x, xcT, p.ldt, 0, p.ldt,
                                    st, nullptr, taps, &ex);
    if (rc) return rc;
  } else {
    rc = transpose_to_bf16<uint8_t>(io.x_codes, c_in, T_out, c_in, nullptr, nullptr, io.z_x, xcT, p.ldt, 0, p.ldt, st);
    if (rc) return rc;
  }

  // ---- A operand of the dW product: the selected rows of dY^T
  const bf16_t* Aw; int64_t ldaw; const int32_t* a_rows;
  if (!p.need_sel) {               // channel-major bf16: gather fused into the GEMM's A-tile loads
    Aw = (const bf16_t*)io.dy; ldaw = T_out; a_rows = io.idx;
  } else if (io.dy_layout == EFQAT_DY_CHANNEL_MAJOR) {
    if (io.dy_dtype == EFQAT_F32)
      hipLaunchKernelGGL((k_rows_bf16<float>), dim3(grid1d(io.k * p.ldt)), dim3(256), 0, st, (const float*)io.dy,
                         T_out, io.k, T_out, io.idx, sel, p.ldt);
    else
      hipLaunchKernelGGL((k_rows_bf16<bf16_t>), dim3(grid1d(io.k * p.ldt)), dim3(256), 0, st, (const bf16_t*)io.dy,
                         T_out, io.k, T_out, io.idx, sel, p.ldt);
    EFQAT_LAUNCH_CHECK();
    Aw = sel; ldaw = p.ldt; a_rows = nullptr;
  } else {
    // token major: sel[m][t] = dY[t][idx[m]]
    if (io.dy_dtype == EFQAT_F32)
      rc = transpose_to_bf16<float>((const float*)io.dy, c_out, T_out, io.k, io.idx, nullptr, nullptr, sel, p.ldt, 0,
                                    p.ldt, st);
    else
      rc = transpose_to_bf16<bf16_t>((const bf16_t*)io.dy, c_out, T_out, io.k, io.idx, nullptr, nullptr, sel, p.ldt,
                                     0, p.ldt, st);
    if (rc) return rc;
    Aw = sel; ldaw = p.ldt; a_rows = nullptr;
  }
  const int64_t Kw = p.need_sel ? p.ldt : T_out;
  stg.close();
  rc = launch_gemm_nt(Aw, ldaw, a_rows, xcT, p.ldt, io.k, p.Nw, Kw, p.plan_dw, part_dw, nullptr, st);
  if (rc) return rc;
  }
  if (use_side && (hipEventRecord(ev.join, st2) != hipSuccess || hipStreamWaitEvent(st, ev.join, 0) != hipSuccess))
    return EFQAT_ERR_HIP;
  const int fvec = (p.Nw % 4 == 0 && ((uintptr_t)io.w % 16) == 0 && ((uintptr_t)io.dw % 16) == 0 &&
                    ((uintptr_t)io.w_codes % 4) == 0 && ((uintptr_t)io.sgd.mom_w % 16) == 0) ? 1 : 0;
  ProfScope fin(PROF_FINISH, st);
  // k blocks for the rows of dW plus one that finishes dS_x, dZ_x
  // long rows and few of them: the chain of dependent loads per row, not bandwidth, sets the time
  if (fvec && p.Nw >= 2048 && io.k < 512)
    hipLaunchKernelGGL(k_dw_finish<1024>, dim3((unsigned)io.k + 1), dim3(1024), 0, st, part_dw, p.plan_dw.split_k, io.k,
                       p.Nw, fvec, io.s_x, io.w_codes, io.w_clip, io.w, io.s_w, io.idx, io.dw, io.scatter, io.ds_w,
                       part_dx, n_part_dx, io.ds_x, io.dz_x, io.sgd);
  else
    hipLaunchKernelGGL(k_dw_finish<256>, dim3((unsigned)io.k + 1), dim3(256), 0, st, part_dw, p.plan_dw.split_k, io.k,
                       p.Nw, fvec, io.s_x, io.w_codes, io.w_clip, io.w, io.s_w, io.idx, io.dw, io.scatter, io.ds_w,
                       part_dx, n_part_dx, io.ds_x, io.dz_x, io.sgd);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

static int check_common(const BwdIo& io, int64_t c_out, const void* ws, int dxk) {
  if (io.dy_dtype != EFQAT_F32 && io.dy_dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (io.x_dtype != EFQAT_F32 && io.x_dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (io.dx_dtype != EFQAT_F32 && io.dx_dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (io.dy_layout != EFQAT_DY_TOKEN_MAJOR && io.dy_layout != EFQAT_DY_CHANNEL_MAJOR) return EFQAT_ERR_BAD_LAYOUT;
  if (dxk < EFQAT_DX_KERNEL_AUTO || dxk > EFQAT_DX_KERNEL_BF16_PINNED) return EFQAT_ERR_BAD_LAYOUT;
  if (io.k < 0 || io.k > c_out) return EFQAT_ERR_BAD_K;
  if (io.scatter != 0 && io.scatter != 1) return EFQAT_ERR_BAD_LAYOUT;
  if (!io.dy || !io.x_codes || !io.x_clip || !io.x || !io.s_x || !io.z_x || !io.w_codes || !io.s_w || !io.dx ||
      !io.ds_x || !io.dz_x || !ws)
    return EFQAT_ERR_NULL_PTR;
  if (io.k > 0 && (!io.idx || !io.w_clip || !io.w)) return EFQAT_ERR_NULL_PTR;
  if (io.k > 0 && !io.sgd.w && (!io.dw || !io.ds_w)) return EFQAT_ERR_NULL_PTR;   // gradients may stay unwritten only with the fused step
  if (((uintptr_t)ws % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  const size_t dysz = io.dy_dtype == EFQAT_F32 ? 4 : 2;
  // the dY tile loads are 16-byte vectors when dY is used in place
  if (((uintptr_t)io.dy % 16) != 0 || ((uintptr_t)io.dy % dysz) != 0) return EFQAT_ERR_ALIGNMENT;
  if (((uintptr_t)io.x % (io.x_dtype == EFQAT_F32 ? 4 : 2)) != 0) return EFQAT_ERR_ALIGNMENT;
  if (((uintptr_t)io.dx % (io.dx_dtype == EFQAT_F32 ? 4 : 2)) != 0) return EFQAT_ERR_ALIGNMENT;
  if (((uintptr_t)io.w % 4) != 0 || ((uintptr_t)io.s_w % 4) != 0 || ((uintptr_t)io.dw % 4) != 0 ||
      ((uintptr_t)io.ds_w % 4) != 0 || ((uintptr_t)io.idx % 4) != 0 || ((uintptr_t)io.x_clip % 4) != 0 ||
      ((uintptr_t)io.w_clip % 4) != 0)
    return EFQAT_ERR_ALIGNMENT;
  return EFQAT_OK;
}

static int fill_step(const efqat_opt_step* step, float* w, float* s_w, StepArgs* out) {
  if (!step || !w || !s_w) return EFQAT_ERR_NULL_PTR;
  if (step->momentum != 0.0f && !step->mom_w) return EFQAT_ERR_NULL_PTR;
  if (!step->adam_m || !step->adam_v || !step->adam_t) return EFQAT_ERR_NULL_PTR;
  if (((uintptr_t)step->mom_w % 4) != 0 || ((uintptr_t)step->adam_m % 4) != 0 || ((uintptr_t)step->adam_v % 4) != 0 ||
      ((uintptr_t)step->adam_t % 4) != 0)
    return EFQAT_ERR_ALIGNMENT;
  // 0 <= beta < 1 (the bias correction divides by 1 - beta^t), eps >= 0
  if (!(step->beta1 >= 0.0f && step->beta1 < 1.0f) || !(step->beta2 >= 0.0f && step->beta2 < 1.0f) ||
      !(step->eps >= 0.0f))
    return EFQAT_ERR_BAD_LAYOUT;
  out->w = w; out->s_w = s_w;
  out->mom_w = step->momentum != 0.0f ? step->mom_w : nullptr;
  out->lr_w = step->lr_w; out->mu = step->momentum; out->wd = step->weight_decay;
  out->adam_m = step->adam_m; out->adam_v = step->adam_v; out->adam_t = step->adam_t;
  out->lr_s = step->lr_s; out->b1 = step->beta1; out->b2 = step->beta2; out->eps = step->eps;
  return EFQAT_OK;
}

// Upper limits of the linear entry points: tokens up to 2^30, channel counts below 2^24 (32-bit pointer steps)
static bool linear_shape_ok(int64_t T, int64_t c_in, int64_t c_out) {
  return T > 0 && c_in > 0 && c_out > 0 && T <= (1 << 30) && c_in < (1 << 24) && c_out < (1 << 24);
}

// All linear entry points end here: every check first, then the launches.
static int linear_bwd_entry(BwdIo& io, int64_t T, int64_t c_in, int64_t c_out, const efqat_opt_step* step, float* w_rw,
                            float* s_w_rw, int dxk, void* ws, size_t ws_bytes, void* stream) {
  if (!linear_shape_ok(T, c_in, c_out)) return EFQAT_ERR_BAD_SHAPE;
  int rc;
  if (step) {
    rc = fill_step(step, w_rw, s_w_rw, &io.sgd);
    if (rc) return rc;
  }
  rc = check_common(io, c_out, ws, dxk);
  if (rc) return rc;
  if (io.w_operand && dxk != EFQAT_DX_KERNEL_AUTO) return EFQAT_ERR_BAD_LAYOUT;   // the operand belongs to the default plan
  if (io.w_operand && ((uintptr_t)io.w_operand % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  const BwdPlan p = make_plan(T, T, c_in, c_out, 1, io.k, io.dy_dtype, io.dy_layout, false, dxk, nullptr,
                              io.x_dtype == EFQAT_BF16 && io.dx_dtype == EFQAT_BF16);
  if (ws_bytes < p.total) return EFQAT_ERR_WORKSPACE;
  rc = check_plan(p, io, T, c_in, c_out, false);
  if (rc) return rc;
  return run_bwd(io, p, T, T, c_in, c_out, nullptr, ws, (hipStream_t)stream);
}

}  // namespace efqat

using namespace efqat;

extern "C" size_t efqat_linear_bwd_workspace_bytes_ex(int64_t T, int64_t c_in, int64_t c_out, int64_t k, int dy_dtype,
                                                      int dy_layout, int dx_kernel) {
  if (!linear_shape_ok(T, c_in, c_out) || k < 0 || k > c_out) return 0;
  if (dx_kernel < EFQAT_DX_KERNEL_AUTO || dx_kernel > EFQAT_DX_KERNEL_BF16_PINNED) return 0;
  return make_plan(T, T, c_in, c_out, 1, k, dy_dtype, dy_layout, false, dx_kernel).total;
}

extern "C" size_t efqat_linear_bwd_workspace_bytes(int64_t T, int64_t c_in, int64_t c_out, int64_t k, int dy_dtype,
                                                   int dy_layout) {
  return efqat_linear_bwd_workspace_bytes_ex(T, c_in, c_out, k, dy_dtype, dy_layout, EFQAT_DX_KERNEL_AUTO);
}

extern "C" int efqat_linear_bwd(const void* dy, int dy_dtype, int dy_layout, int64_t T, int64_t c_in, int64_t c_out,
                                const uint8_t* x_codes, const uint32_t* x_clip, const void* x, int x_dtype,
                                const float* s_x, const float* z_x, const int8_t* w_codes, const uint32_t* w_clip,
                                const float* w, const float* s_w, const int32_t* idx, int64_t k, void* dx,
                                int dx_dtype, float* dw, int scatter, float* ds_w, float* ds_x, float* dz_x,
                                void* ws, size_t ws_bytes, void* stream) {
  BwdIo io{dy, dy_dtype, dy_layout, x_codes, x_clip, x, x_dtype, s_x, z_x, w_codes, w_clip, w, s_w, idx, k,
           dx, dx_dtype, dw, scatter, ds_w, ds_x, dz_x};
  return linear_bwd_entry(io, T, c_in, c_out, nullptr, nullptr, nullptr, EFQAT_DX_KERNEL_AUTO, ws, ws_bytes, stream);
}

extern "C" int efqat_linear_bwd_ex(const void* dy, int dy_dtype, int dy_layout, int64_t T, int64_t c_in, int64_t c_out,
                                   const uint8_t* x_codes, const uint32_t* x_clip, const void* x, int x_dtype,
                                   const float* s_x, const float* z_x, const int8_t* w_codes, const uint32_t* w_clip,
                                   float* w, float* s_w, const int32_t* idx, int64_t k, void* dx, int dx_dtype,
                                   float* dw, int scatter, float* ds_w, float* ds_x, float* dz_x,
                                   const void* w_operand, const efqat_opt_step* step, int dx_kernel, void* ws,
                                   size_t ws_bytes, void* stream, void* side_stream) {
  BwdIo io{dy, dy_dtype, dy_layout, x_codes, x_clip, x, x_dtype, s_x, z_x, w_codes, w_clip, w, s_w, idx, k,
           dx, dx_dtype, dw, scatter, ds_w, ds_x, dz_x};
  io.w_operand = w_operand;
  io.side = (hipStream_t)side_stream;
  return linear_bwd_entry(io, T, c_in, c_out, step, w, s_w, dx_kernel, ws, ws_bytes, stream);
}

extern "C" size_t efqat_linear_bwd_weight_operand_bytes(int64_t T, int64_t c_in, int64_t c_out, int dy_dtype,
                                                        int dy_layout) {
  if (!linear_shape_ok(T, c_in, c_out)) return 0;
  const BwdPlan p = make_plan(T, T, c_in, c_out, 1, 0, dy_dtype, dy_layout, false, EFQAT_DX_KERNEL_AUTO);
  return p.dx8 ? 0 : (size_t)round_up((int64_t)p.b_wqT, 256) + 256;
}

extern "C" int efqat_linear_bwd_weight_operand(const int8_t* w_codes, const float* s_w, int64_t T, int64_t c_in,
                                               int64_t c_out, int dy_dtype, int dy_layout, void* operand,
                                               size_t operand_bytes, void* stream) {
  if (!linear_shape_ok(T, c_in, c_out)) return EFQAT_ERR_BAD_SHAPE;
  if (dy_dtype != EFQAT_F32 && dy_dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (dy_layout != EFQAT_DY_TOKEN_MAJOR && dy_layout != EFQAT_DY_CHANNEL_MAJOR) return EFQAT_ERR_BAD_LAYOUT;
  const size_t need = efqat_linear_bwd_weight_operand_bytes(T, c_in, c_out, dy_dtype, dy_layout);
  if (need == 0) return EFQAT_OK;                      // this layer's dX product reads the int8 codes themselves
  if (!w_codes || !s_w || !operand) return EFQAT_ERR_NULL_PTR;
  if (operand_bytes < need) return EFQAT_ERR_WORKSPACE;
  if (((uintptr_t)operand % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  if (c_in > 65535 * (int64_t)64) return EFQAT_ERR_BAD_SHAPE;
  const BwdPlan p = make_plan(T, T, c_in, c_out, 1, 0, dy_dtype, dy_layout, false, EFQAT_DX_KERNEL_AUTO);
  TransposeExtra ex{};
  ex.z_in = c_in; ex.z_out = p.ldc;
  uint32_t* zero_page = (uint32_t*)((char*)operand + round_up((int64_t)p.b_wqT, 256));
  hipStream_t st = (hipStream_t)stream;
  ProfScope prep(PROF_PREP, st);
  return transpose_to_bf16<int8_t>(w_codes, c_in, c_out, c_in, nullptr, s_w, nullptr, (bf16_t*)operand, p.Kx, 0,
                                   p.ldc, st, zero_page, 1, &ex);
}

static int conv_geom(int64_t N, int64_t H, int64_t W, int64_t c_in, int64_t c_out, int64_t KH, int64_t KW,
                     int64_t stride, int64_t pad, ConvGeom* g) {
  if (N <= 0 || H <= 0 || W <= 0 || c_in <= 0 || c_out <= 0 || KH <= 0 || KW <= 0 || stride <= 0 || pad < 0)
    return EFQAT_ERR_BAD_SHAPE;
  if (N > (1 << 24) || H > (1 << 15) || W > (1 << 15) || c_in > (1 << 20) || c_out > (1 << 20) || KH > 64 || KW > 64 ||
      stride > 64 || pad > 64)
    return EFQAT_ERR_BAD_SHAPE;
  if (H + 2 * pad < KH || W + 2 * pad < KW) return EFQAT_ERR_BAD_SHAPE;
  g->N = (int)N; g->H = (int)H; g->W = (int)W; g->c_in = (int)c_in; g->c_out = (int)c_out;
  g->KH = (int)KH; g->KW = (int)KW; g->stride = (int)stride; g->pad = (int)pad;
  g->Ho = (int)((H + 2 * pad - KH) / stride + 1);
  g->Wo = (int)((W + 2 * pad - KW) / stride + 1);
  if ((int64_t)N * H * W > (1 << 30) || (int64_t)N * g->Ho * g->Wo > (1 << 30)) return EFQAT_ERR_BAD_SHAPE;
  return EFQAT_OK;
}

static BwdPlan conv_plan(const ConvGeom& g, int64_t k, int dy_dtype, int dy_layout, int dxk, bool io_bf16) {
  const bool im2col = !(g.KH * g.KW == 1 && g.stride == 1 && g.pad == 0);
  return make_plan((int64_t)g.N * g.H * g.W, (int64_t)g.N * g.Ho * g.Wo, g.c_in, g.c_out, g.KH * g.KW, k, dy_dtype,
                   dy_layout, im2col, dxk, &g, io_bf16);
}

extern "C" size_t efqat_conv_bwd_workspace_bytes_ex(int64_t N, int64_t H, int64_t W, int64_t c_in, int64_t c_out,
                                                    int64_t KH, int64_t KW, int64_t stride, int64_t pad, int64_t k,
                                                    int dy_dtype, int dy_layout, int dx_kernel) {
  ConvGeom g;
  if (conv_geom(N, H, W, c_in, c_out, KH, KW, stride, pad, &g) || k < 0 || k > c_out) return 0;
  if (dx_kernel < EFQAT_DX_KERNEL_AUTO || dx_kernel > EFQAT_DX_KERNEL_BF16_PINNED) return 0;
  return conv_plan(g, k, dy_dtype, dy_layout, dx_kernel, false).total;
}

extern "C" size_t efqat_conv_bwd_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t c_in, int64_t c_out,
                                                 int64_t KH, int64_t KW, int64_t stride, int64_t pad, int64_t k,
                                                 int dy_dtype, int dy_layout) {
  return efqat_conv_bwd_workspace_bytes_ex(N, H, W, c_in, c_out, KH, KW, stride, pad, k, dy_dtype, dy_layout,
                                           EFQAT_DX_KERNEL_AUTO);
}

static int conv_bwd_entry(BwdIo& io, int64_t N, int64_t H, int64_t W, int64_t c_in, int64_t c_out, int64_t KH,
                          int64_t KW, int64_t stride, int64_t pad, const efqat_opt_step* step, float* w_rw,
                          float* s_w_rw, int dxk, void* ws, size_t ws_bytes, void* stream) {
  ConvGeom g;
  int rc = conv_geom(N, H, W, c_in, c_out, KH, KW, stride, pad, &g);
  if (rc) return rc;
  if (step) {
    rc = fill_step(step, w_rw, s_w_rw, &io.sgd);
    if (rc) return rc;
  }
  rc = check_common(io, c_out, ws, dxk);
  if (rc) return rc;
  const BwdPlan p = conv_plan(g, io.k, io.dy_dtype, io.dy_layout, dxk, io.x_dtype == EFQAT_BF16 && io.dx_dtype == EFQAT_BF16);
  if (ws_bytes < p.total) return EFQAT_ERR_WORKSPACE;
  const int64_t T_in = (int64_t)N * H * W, T_out = (int64_t)N * g.Ho * g.Wo;
  rc = check_plan(p, io, T_out, c_in, c_out, true);
  if (rc) return rc;
  return run_bwd(io, p, T_in, T_out, c_in, c_out, &g, ws, (hipStream_t)stream);
}

extern "C" int efqat_conv_bwd(const void* dy, int dy_dtype, int dy_layout, int64_t N, int64_t H, int64_t W,
                              int64_t c_in, int64_t c_out, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                              const uint8_t* x_codes, const uint32_t* x_clip, const void* x, int x_dtype,
                              const float* s_x, const float* z_x, const int8_t* w_codes, const uint32_t* w_clip,
                              const float* w, const float* s_w, const int32_t* idx, int64_t k, void* dx,
                              int dx_dtype, float* dw, int scatter, float* ds_w, float* ds_x, float* dz_x, void* ws,
                              size_t ws_bytes, void* stream) {
  BwdIo io{dy, dy_dtype, dy_layout, x_codes, x_clip, x, x_dtype, s_x, z_x, w_codes, w_clip, w, s_w, idx, k,
           dx, dx_dtype, dw, scatter, ds_w, ds_x, dz_x};
  return conv_bwd_entry(io, N, H, W, c_in, c_out, KH, KW, stride, pad, nullptr, nullptr, nullptr,
                        EFQAT_DX_KERNEL_AUTO, ws, ws_bytes, stream);
}

extern "C" int efqat_conv_bwd_ex(const void* dy, int dy_dtype, int dy_layout, int64_t N, int64_t H, int64_t W,
                                 int64_t c_in, int64_t c_out, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                                 const uint8_t* x_codes, const uint32_t* x_clip, const void* x, int x_dtype,
                                 const float* s_x, const float* z_x, const int8_t* w_codes, const uint32_t* w_clip,
                                 float* w, float* s_w, const int32_t* idx, int64_t k, void* dx, int dx_dtype,
                                 float* dw, int scatter, float* ds_w, float* ds_x, float* dz_x,
                                 const efqat_opt_step* step, int dx_kernel, void* ws, size_t ws_bytes, void* stream,
                                 void* side_stream) {
  BwdIo io{dy, dy_dtype, dy_layout, x_codes, x_clip, x, x_dtype, s_x, z_x, w_codes, w_clip, w, s_w, idx, k,
           dx, dx_dtype, dw, scatter, ds_w, ds_x, dz_x};
  io.side = (hipStream_t)side_stream;
  return conv_bwd_entry(io, N, H, W, c_in, c_out, KH, KW, stride, pad, step, w, s_w, dx_kernel, ws, ws_bytes, stream);
}
