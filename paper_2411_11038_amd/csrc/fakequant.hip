// Fake-quant forward (Eq. 1-4): quantizer statistics, integer codes, straight-through clip masks.
// All kernels are HBM-bound streaming passes built on 64-wide wavefront reductions.
#include "common.hpp"

#include <type_traits>

namespace efqat {

// ----------------------------------------------------------------------------------------------
// 8 consecutive elements as fp32 (vector path: one 16-byte load for bf16, two for fp32)
template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p);
  float4 b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float (&v)[8]) {
  uint4 a = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(w[i] << 16);
    v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

// ----------------------------------------------------------------------------------------------
// Eq. 2 range: alpha = min x, beta = max x over the whole tensor (MinMax observer).
template <typename T>
__global__ __launch_bounds__(256) void k_minmax_partial(const T* __restrict__ x, int64_t n, int vec,
                                                        float* __restrict__ part) {
  float lo = INFINITY, hi = -INFINITY;
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nthreads = (int64_t)gridDim.x * blockDim.x;
  if (vec) {
    const int64_t n8 = n >> 3;
    int64_t i = tid;
    // four 16-byte (bf16) / 32-byte (fp32) loads in flight per lane: with one, a CU has too few bytes outstanding to
    // cover the memory latency at the HBM rate
    for (; i + 3 * nthreads < n8; i += 4 * nthreads) {
      float v[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) load8<T>(x + (i + u * nthreads) * 8, v[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 8; ++j) { lo = fminf(lo, v[u][j]); hi = fmaxf(hi, v[u][j]); }
    }
    for (; i < n8; i += nthreads) {
      float v[8];
      load8<T>(x + i * 8, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) { lo = fminf(lo, v[j]); hi = fmaxf(hi, v[j]); }
    }
    for (i = (n8 << 3) + tid; i < n; i += nthreads) {
      float v = load_as_f32<T>(x, i);
      lo = fminf(lo, v); hi = fmaxf(hi, v);
    }
  } else {
    for (int64_t i = tid; i < n; i += nthreads) {
      float v = load_as_f32<T>(x, i);
      lo = fminf(lo, v); hi = fmaxf(hi, v);
    }
  }
  lo = wave_min(lo); hi = wave_max(hi);
  __shared__ float s_lo[4], s_hi[4];
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_lo[w] = lo; s_hi[w] = hi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    part[2 * blockIdx.x] = fminf(fminf(s_lo[0], s_lo[1]), fminf(s_lo[2], s_lo[3]));
    part[2 * blockIdx.x + 1] = fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3]));
  }
}

// Eq. 2: S_x = (beta - alpha) / (2^b - 1), Z_x = -round(alpha / S_x), each a single-precision op.
__global__ __launch_bounds__(256) void k_act_qparams(const float* __restrict__ part, int nparts, int bits,
                                                     float* __restrict__ scale, float* __restrict__ zp) {
  float lo = INFINITY, hi = -INFINITY;
  for (int i = threadIdx.x; i < nparts; i += blockDim.x) {
    lo = fminf(lo, part[2 * i]); hi = fmaxf(hi, part[2 * i + 1]);
  }
  lo = wave_min(lo); hi = wave_max(hi);
  __shared__ float s_lo[4], s_hi[4];
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_lo[w] = lo; s_hi[w] = hi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const float alpha = fminf(fminf(s_lo[0], s_lo[1]), fminf(s_lo[2], s_lo[3]));
    const float beta = fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3]));
    const float qmax = (float)((1 << bits) - 1);
    float s = __fdiv_rn(__fsub_rn(beta, alpha), qmax);
    if (!(s > 0.0f)) s = 1.0f;                       // zero range
    scale[0] = s;
    zp[0] = 0.0f - rintf(__fdiv_rn(alpha, s));
  }
}

// ----------------------------------------------------------------------------------------------
// round(x / s) as the round-to-nearest-even integer of the correctly rounded quotient.  x * (1/s) is within
// 1.5 ulp of it, so the two round to the same integer unless x/s sits that close to a half-way point; only
// then is the exact (slow) division needed (always for huge quotients, where the tolerance exceeds one half,
// and for a scale so small that its reciprocal overflows).
__device__ __forceinline__ float round_quotient(float x, float s, float inv_s) {
  const float qf = x * inv_s;
  float r = rintf(qf);
  const float tol = 2.5e-7f * fabsf(qf);
  if (!(0.5f - fabsf(qf - r) > tol) || !(inv_s < 3.0e38f)) r = rintf(__fdiv_rn(x, s));
  return r;
}

// ----------------------------------------------------------------------------------------------
// Eq. 1 / Eq. 3: codes + clip-mask bits (+ optional de-quantised bf16 values).
// One wavefront handles one 512-element segment of one row per iteration; a lane owns 8
// consecutive elements, four neighbouring lanes assemble one 32-bit mask word.
// INIT (weights only): the wavefront first takes the row's abs-max and writes its Eq. 4 scale
// S_w[c] = max_j |w[c][j]| / (2^(b-1) - 1), then quantizes the row it has just pulled through the caches.
template <typename T, int MODE, bool INIT>
__global__ __launch_bounds__(256) void k_quantize(const T* __restrict__ x, int64_t rows, int64_t cols, int vec,
                                                  int bits, float* __restrict__ scale,
                                                  const float* __restrict__ zp, uint8_t* __restrict__ codes,
                                                  uint32_t* __restrict__ clip, bf16_t* __restrict__ xq) {
  const int lane = threadIdx.x & 63;
  const int64_t segs = ceil_div(cols, 512);
  const int64_t total = rows * segs;
  const int64_t wpr = ceil_div(cols, 32);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  float lo, hi, z = 0.0f, s_act = 1.0f;
  if (MODE == EFQAT_QUANT_ACT_PER_TENSOR_ASYM) {
    lo = 0.0f; hi = (float)((1 << bits) - 1);
    s_act = scale[0];
    z = rintf(zp[0]);
  } else {
    hi = (float)((1 << (bits - 1)) - 1); lo = -hi;
  }
  // work item = (row, 512-element segment); with INIT a wavefront keeps the whole row (one abs-max scan, then
  // all its segments) so the row is read from HBM once
  const int64_t nitems = INIT ? rows : total;
  for (int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); item < nitems; item += nwaves) {
   const int64_t row = INIT ? item : item / segs;
   float s_row = 1.0f;
   if (INIT) {
     const T* p = x + row * cols;
     float m = 0.0f;
     if (vec) {
       const int64_t n8 = cols >> 3;
       for (int64_t i = lane; i < n8; i += 64) {
         float t8[8];
         load8<T>(p + i * 8, t8);
#pragma unroll
         for (int j = 0; j < 8; ++j) m = fmaxf(m, fabsf(t8[j]));
       }
     } else {
       for (int64_t i = lane; i < cols; i += 64) m = fmaxf(m, fabsf(load_as_f32<T>(p, i)));
     }
     m = wave_max(m);
     s_row = __fdiv_rn(m, hi);
     if (!(s_row > 0.0f)) s_row = 1.0f;             // all-zero row
     if (lane == 0) scale[row] = s_row;
   }
   for (int64_t seg = INIT ? 0 : item - row * segs; seg < (INIT ? segs : item - row * segs + 1); ++seg) {
    const int64_t col0 = seg * 512 + (int64_t)lane * 8;
    float s;
    if (MODE == EFQAT_QUANT_ACT_PER_TENSOR_ASYM) s = s_act;
    else if (INIT) s = s_row;
    else s = scale[row];
    const float inv_s = __fdiv_rn(1.0f, s);
    const int64_t base = row * cols + col0;
    float v[8];
    const bool full = col0 + 8 <= cols;
    if (vec && full) {
      load8<T>(x + base, v);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (col0 + j < cols) ? load_as_f32<T>(x, base + j) : 0.0f;
    }
    uint32_t bits8 = 0;
    uint32_t cw[2] = {0u, 0u};
    float dq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float c = round_quotient(v[j], s, inv_s) + z;   // un-clamped code
      const float cc = __builtin_amdgcn_fmed3f(c, lo, hi);
      const bool inr = (c == cc);                  // closed interval: a code on the bound is not clipped
      if (inr && (col0 + j < cols)) bits8 |= (1u << j);
      if (MODE == EFQAT_QUANT_ACT_PER_TENSOR_ASYM)
        cw[j >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(cc, j & 3, cw[j >> 2]);   // cc is an integer in [0, 255]
      else
        cw[j >> 2] |= ((uint32_t)((int)cc & 0xFF)) << (8 * (j & 3));
      dq[j] = s * (cc - z);
    }
    if (vec && full) {
      *reinterpret_cast<uint2*>(codes + base) = make_uint2(cw[0], cw[1]);
      if (xq) {
        uint4 o = make_uint4(pack_bf16x2(dq[0], dq[1]), pack_bf16x2(dq[2], dq[3]),
                             pack_bf16x2(dq[4], dq[5]), pack_bf16x2(dq[6], dq[7]));
        *reinterpret_cast<uint4*>(xq + base) = o;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (col0 + j < cols) {
          codes[base + j] = (uint8_t)((cw[j >> 2] >> (8 * (j & 3))) & 0xFF);
          if (xq) xq[base + j] = f32_to_bf16(dq[j]);
        }
      }
    }
    uint32_t word = bits8 << (8 * (lane & 3));
    word |= __shfl_xor(word, 1, kWave);
    word |= __shfl_xor(word, 2, kWave);
    const int64_t widx = col0 >> 5;
    if ((lane & 3) == 0 && widx < wpr) clip[row * wpr + widx] = word;
   }
  }
}

// Eq. 1 for a per-tensor quantizer whose rows are a whole number of 32-element mask words (cols % 32 == 0, aligned
// pointers): the tensor is one flat run of 8-element chunks, codes and mask words are flat as well, so no lane idles
// on a ragged segment and nothing is divided.  Each lane handles two chunks a grid-stride apart per iteration, both
// loads issued before either is used.
template <typename T>
__global__ __launch_bounds__(256) void k_quantize_act_flat(const T* __restrict__ x, int64_t nchunks, int bits,
                                                           const float* __restrict__ scale,
                                                           const float* __restrict__ zp, uint8_t* __restrict__ codes,
                                                           uint32_t* __restrict__ clip, bf16_t* __restrict__ xq) {
  const int lane = threadIdx.x & 63;
  const float hi = (float)((1 << bits) - 1);
  const float s = scale[0];
  const float z = rintf(zp[0]);
  const float inv_s = __fdiv_rn(1.0f, s);
  const int64_t stride = (int64_t)gridDim.x * 256;
  auto finish = [&](int64_t c, const float (&v)[8]) {
    uint32_t bits8 = 0;
    uint32_t cw[2] = {0u, 0u};
    float dq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float cu = round_quotient(v[j], s, inv_s) + z;
      const float cc = __builtin_amdgcn_fmed3f(cu, 0.0f, hi);
      if (cu == cc) bits8 |= (1u << j);
      cw[j >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(cc, j & 3, cw[j >> 2]);
      dq[j] = s * (cc - z);
    }
    *reinterpret_cast<uint2*>(codes + c * 8) = make_uint2(cw[0], cw[1]);
    if (xq)
      *reinterpret_cast<uint4*>(xq + c * 8) = make_uint4(pack_bf16x2(dq[0], dq[1]), pack_bf16x2(dq[2], dq[3]),
                                                         pack_bf16x2(dq[4], dq[5]), pack_bf16x2(dq[6], dq[7]));
    // chunks c .. c+3 of lanes 4m .. 4m+3 make one mask word (c of lane 4m is a multiple of 4: see the launch)
    uint32_t word = bits8 << (8 * (lane & 3));
    word |= __shfl_xor(word, 1, kWave);
    word |= __shfl_xor(word, 2, kWave);
    if ((lane & 3) == 0) clip[c >> 2] = word;
  };
  // the grid covers whole groups of four chunks: nchunks % 4 == 0 and the stride is a multiple of 4, so the four
  // lanes of a mask word are in range together
  int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; c + stride < nchunks; c += 2 * stride) {
    float v0[8], v1[8];
    load8<T>(x + c * 8, v0);
    load8<T>(x + (c + stride) * 8, v1);
    finish(c, v0);
    finish(c + stride, v1);
  }
  if (c < nchunks) {
    float v0[8];
    load8<T>(x + c * 8, v0);
    finish(c, v0);
  }
}

// Eq. 4 + Eq. 3 with the row held in registers (weights, min/max initialisation, cols <= 8 * 64 * WPR * NIT <= 16384,
// cols % 32 == 0, aligned pointers): WPR wavefronts per row (1, or the 4 of a block when there are few rows) issue all
// loads of the row at once, take the abs-max, write S_w[c] and quantize from the registers, so the row is read once
// and the reads are not a chain of dependent round trips.
template <int NIT, int WPR>
__global__ __launch_bounds__(256) void k_quantize_w_row_init(const float* __restrict__ w, int64_t rows, int64_t cols,
                                                             int bits, float* __restrict__ scale,
                                                             int8_t* __restrict__ codes, uint32_t* __restrict__ clip,
                                                             double* __restrict__ scores) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = WPR == 4 ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
  const int part = WPR == 4 ? wave : 0;               // which quarter of the row's chunks (interleaved by 64)
  const bool on = row < rows;                         // WPR == 1: whole wavefronts beyond the last row idle
  const float hi = (float)((1 << (bits - 1)) - 1), lo = -hi;
  const int n8 = on ? (int)(cols >> 3) : 0;
  const float* p = w + (on ? row : 0) * cols;
  float v[NIT][8];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * WPR + part) * 64 + lane;
    if (i < n8) load8<float>(p + (int64_t)i * 8, v[it]);
  }
  float m = 0.0f;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    if ((it * WPR + part) * 64 + lane < n8) {
#pragma unroll
      for (int j = 0; j < 8; ++j) m = fmaxf(m, fabsf(v[it][j]));
    }
  }
  m = wave_max(m);
  // optional by-product (Eq. 6): the row's mean |w| in double precision, fixed summation order, from the registers
  double asum = 0.0;
  if (scores) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if ((it * WPR + part) * 64 + lane < n8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) asum += (double)fabsf(v[it][j]);
      }
    }
    asum = wave_sum(asum);
  }
  if (WPR == 4) {
    __shared__ float s_m[4];
    __shared__ double s_a[4];
    if (lane == 0) { s_m[wave] = m; s_a[wave] = asum; }
    __syncthreads();
    m = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    asum = (s_a[0] + s_a[1]) + (s_a[2] + s_a[3]);
  }
  if (scores && on && lane == 0 && part == 0) scores[row] = asum / (double)cols;
  float s = __fdiv_rn(m, hi);
  if (!(s > 0.0f)) s = 1.0f;                          // all-zero row
  if (on && lane == 0 && part == 0) scale[row] = s;
  const float inv_s = __fdiv_rn(1.0f, s);
  const int64_t wpr = cols >> 5;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * WPR + part) * 64 + lane;
    // n8 % 4 == 0: the four lanes of a mask word are in range together
    if (i < n8) {
      uint32_t bits8 = 0;
      uint32_t cw[2] = {0u, 0u};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float cu = round_quotient(v[it][j], s, inv_s);
        const float cc = __builtin_amdgcn_fmed3f(cu, lo, hi);
        if (cu == cc) bits8 |= (1u << j);
        cw[j >> 2] |= ((uint32_t)((int)cc & 0xFF)) << (8 * (j & 3));
      }
      *reinterpret_cast<uint2*>(codes + row * cols + (int64_t)i * 8) = make_uint2(cw[0], cw[1]);
      uint32_t word = bits8 << (8 * (lane & 3));
      word |= __shfl_xor(word, 1, kWave);
      word |= __shfl_xor(word, 2, kWave);
      if ((lane & 3) == 0) clip[row * wpr + (i >> 2)] = word;
    }
  }
}

// ----------------------------------------------------------------------------------------------
static inline bool aligned_to(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// scores (weights with min/max initialisation only): where the row-in-registers kernel runs, it also writes the
// Eq. 6 importance of every row and *scores_done is set; otherwise the caller computes them in a pass of its own.
template <typename T>
static int run_fakequant(const T* x, int64_t rows, int64_t cols, int mode, int bits, int init_minmax,
                         float* scale, float* zp, void* codes, uint32_t* clip, bf16_t* xq, void* ws,
                         hipStream_t st, double* scores = nullptr, bool* scores_done = nullptr) {
  const int64_t n = rows * cols;
  ProfScope prof(mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM ? PROF_QACT : PROF_QW, st);
  const int vec_flat = aligned_to(x, 16) ? 1 : 0;
  const int vec_row = (vec_flat && cols % 8 == 0 && aligned_to(codes, 8) && (!xq || aligned_to(xq, 16))) ? 1 : 0;
  if (init_minmax && mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM) {
    int64_t np64 = ceil_div(n, 256 * 16);
    const int nparts = (int)(np64 < 1024 ? np64 : 1024);
    float* part = (float*)ws;
    hipLaunchKernelGGL((k_minmax_partial<T>), dim3(nparts), dim3(256), 0, st, x, n, vec_flat, part);
    EFQAT_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_act_qparams, dim3(1), dim3(256), 0, st, part, nparts, bits, scale, zp);
    EFQAT_LAUNCH_CHECK();
  }
  const bool row_items = init_minmax && mode == EFQAT_QUANT_W_PER_ROW_SYM;   // one wavefront per row
  const int64_t items = row_items ? rows : rows * ceil_div(cols, 512);
  int64_t blocks = ceil_div(items, 4);
  if (blocks > 256 * 32) blocks = 256 * 32;
  if (mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM && vec_row && (cols % 32) == 0) {
    const int64_t nchunks = n / 8;
    int64_t fb = ceil_div(nchunks, 512);             // two chunks per lane and iteration
    if (fb > 256 * 16) fb = 256 * 16;
    hipLaunchKernelGGL((k_quantize_act_flat<T>), dim3((unsigned)fb), dim3(256), 0, st, x, nchunks, bits, scale, zp,
                       (uint8_t*)codes, clip, xq);
  } else if (mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM)
    hipLaunchKernelGGL((k_quantize<T, EFQAT_QUANT_ACT_PER_TENSOR_ASYM, false>), dim3((unsigned)blocks), dim3(256), 0,
                       st, x, rows, cols, vec_row, bits, scale, zp, (uint8_t*)codes, clip, xq);
  else if (init_minmax && std::is_same<T, float>::value && vec_row && (cols % 32) == 0 && cols <= 8 * 64 * 4 * 8 && !xq) {
    // few rows or long rows: a block per row, so that the chip still holds enough wavefronts to cover the memory
    // latency and a lane holds at most 64 values
    const bool wide = (rows < 4096 && cols > 8 * 64) || cols > 8 * 64 * 8;
    const float* wf = (const float*)x;
    int8_t* cd = (int8_t*)codes;
    const int per_wave = (int)ceil_div(cols, 8 * 64 * (wide ? 4 : 1));     // 8-element chunks per lane
    const dim3 grid((unsigned)(wide ? rows : ceil_div(rows, 4)));
#define EFQAT_ROW_INIT(NIT, WPR) \
  hipLaunchKernelGGL((k_quantize_w_row_init<NIT, WPR>), grid, dim3(256), 0, st, wf, rows, cols, bits, scale, cd, clip, \
                     scores)
    if (wide) {
      if (per_wave <= 1) EFQAT_ROW_INIT(1, 4); else if (per_wave <= 2) EFQAT_ROW_INIT(2, 4);
      else if (per_wave <= 4) EFQAT_ROW_INIT(4, 4); else if (per_wave <= 6) EFQAT_ROW_INIT(6, 4); else EFQAT_ROW_INIT(8, 4);
    } else {
      if (per_wave <= 2) EFQAT_ROW_INIT(2, 1); else if (per_wave <= 4) EFQAT_ROW_INIT(4, 1); else EFQAT_ROW_INIT(8, 1);
    }
#undef EFQAT_ROW_INIT
    if (scores && scores_done) *scores_done = true;
  } else if (init_minmax)
    hipLaunchKernelGGL((k_quantize<T, EFQAT_QUANT_W_PER_ROW_SYM, true>), dim3((unsigned)blocks), dim3(256), 0, st, x,
                       rows, cols, vec_row, bits, scale, zp, (uint8_t*)codes, clip, xq);
  else
    hipLaunchKernelGGL((k_quantize<T, EFQAT_QUANT_W_PER_ROW_SYM, false>), dim3((unsigned)blocks), dim3(256), 0, st, x,
                       rows, cols, vec_row, bits, scale, zp, (uint8_t*)codes, clip, xq);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

}  // namespace efqat

using namespace efqat;

extern "C" size_t efqat_fakequant_fwd_workspace_bytes(int64_t rows, int64_t cols, int mode) {
  (void)rows; (void)cols;
  return mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM ? (size_t)(1024 * 2 * sizeof(float)) : (size_t)256;
}

extern "C" int efqat_fakequant_fwd(const void* x, int dtype, int64_t rows, int64_t cols, int mode, int bits,
                                   int init_minmax, float* scale, float* zero_point, void* codes,
                                   uint32_t* clip_bits, void* xq, void* ws, size_t ws_bytes, void* stream) {
  if (mode != EFQAT_QUANT_ACT_PER_TENSOR_ASYM && mode != EFQAT_QUANT_W_PER_ROW_SYM) return EFQAT_ERR_BAD_LAYOUT;
  if (dtype != EFQAT_F32 && dtype != EFQAT_BF16) return EFQAT_ERR_BAD_DTYPE;
  if (rows <= 0 || cols <= 0 || rows > (INT64_MAX / cols)) return EFQAT_ERR_BAD_SHAPE;
  if (bits < 2 || bits > 8) return EFQAT_ERR_BAD_BITS;
  if (!x || !scale || !codes || !clip_bits) return EFQAT_ERR_NULL_PTR;
  if (mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM && !zero_point) return EFQAT_ERR_NULL_PTR;
  if (init_minmax && mode == EFQAT_QUANT_ACT_PER_TENSOR_ASYM) {
    if (!ws) return EFQAT_ERR_NULL_PTR;
    if (ws_bytes < efqat_fakequant_fwd_workspace_bytes(rows, cols, mode)) return EFQAT_ERR_WORKSPACE;
    if (((uintptr_t)ws % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  }
  const size_t esz = dtype == EFQAT_F32 ? 4 : 2;
  if (((uintptr_t)x % esz) != 0 || ((uintptr_t)clip_bits % 4) != 0 || (xq && ((uintptr_t)xq % 2) != 0))
    return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == EFQAT_F32)
    return run_fakequant<float>((const float*)x, rows, cols, mode, bits, init_minmax, scale, zero_point, codes,
                                clip_bits, (bf16_t*)xq, ws, st);
  return run_fakequant<bf16_t>((const bf16_t*)x, rows, cols, mode, bits, init_minmax, scale, zero_point, codes,
                               clip_bits, (bf16_t*)xq, ws, st);
}

// Weight side of one step in a single call: Eq. 4 + Eq. 3 (codes, clip mask, scales), Eq. 6 and the Top-K.
extern "C" size_t efqat_weight_quant_select_workspace_bytes(int64_t c_out) {
  return efqat_channel_select_workspace_bytes(c_out);
}

extern "C" int efqat_weight_quant_select(const float* w, int64_t c_out, int64_t block, int bits, int init_minmax,
                                         float* scale, int8_t* codes, uint32_t* clip_bits, int64_t k, double* scores,
                                         int32_t* idx, void* ws, size_t ws_bytes, void* stream) {
  if (c_out <= 0 || block <= 0 || c_out > INT32_MAX || c_out > INT64_MAX / block) return EFQAT_ERR_BAD_SHAPE;
  if (bits < 2 || bits > 8) return EFQAT_ERR_BAD_BITS;
  if (k < 0 || k > c_out) return EFQAT_ERR_BAD_K;
  if (!w || !scale || !codes || !clip_bits || !ws || (k > 0 && !idx)) return EFQAT_ERR_NULL_PTR;
  if (ws_bytes < efqat_weight_quant_select_workspace_bytes(c_out)) return EFQAT_ERR_WORKSPACE;
  if (((uintptr_t)ws % 256) != 0 || ((uintptr_t)w % 4) != 0 || ((uintptr_t)clip_bits % 4) != 0 ||
      ((uintptr_t)scale % 4) != 0 || ((uintptr_t)idx % 4) != 0 || ((uintptr_t)scores % 8) != 0)
    return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  double* sc = scores ? scores : (double*)ws;
  bool scores_done = false;
  int rc = run_fakequant<float>(w, c_out, block, EFQAT_QUANT_W_PER_ROW_SYM, bits, init_minmax, scale, nullptr, codes,
                                clip_bits, nullptr, nullptr, st, init_minmax ? sc : nullptr, &scores_done);
  if (rc) return rc;
  if (!scores_done) {                                  // rows too long for the register kernel, or given scales
    rc = launch_row_importance(w, c_out, block, sc, st);
    if (rc) return rc;
  }
  if (k == 0) return EFQAT_OK;
  return launch_topk_profiled(sc, c_out, k, idx, st);
}
