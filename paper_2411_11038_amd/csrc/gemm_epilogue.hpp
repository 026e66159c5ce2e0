// Pieces shared by the product kernels: the argument block and the fused epilogue of the dX product.
#pragma once
#include "common.hpp"

namespace efqat {

typedef float floatx16_t __attribute__((ext_vector_type(16)));

enum { EPI_RAW = 0, EPI_DX = 1, EPI_FWD = 2, EPI_DXF = 3 };   // DXF: epilogue_dx_fast

struct GemmArgs {
  const void* A; int64_t lda; const int32_t* a_rows;   // lda / ldb / K in elements (bf16 or int8)
  const void* B; int64_t ldb;
  int M, N, K;
  int k_per_split;        // multiple of KALIGN
  int tiles_m, tiles_n;
  int group_m;                        // row tiles per group of the tile order (the kernels of gemm_tn.hip)
  float* out;             // raw fp32 [split][M][N]
  // fused dX epilogue
  const uint8_t* x_codes; const uint32_t* x_clip; const void* x; int x_dtype;
  const float* s_x; const float* z_x; void* dx; int dx_dtype; float* partial;
  int epi_vec;            // 8-wide vector accesses allowed in the fused epilogue
  // forward epilogue (int8 product): y = s_x * s_w[n] * (acc + (128 - round(z_x)) * wsum[n])
  const float* s_w; const int32_t* wsum; void* y; int y_dtype;
  // implicit im2col of the A operand (dX product of a stride-1 convolution): row m is the input pixel (n, h, w),
  // K runs over (tap, c_out) with cv_spt 64-channel stages per tap, and the operand element is
  // dY[n][h + pad - kh][w + pad - kw][c_out] or zero outside the output image (read from cv_zero)
  int cv_H, cv_W, cv_Ho, cv_Wo, cv_KW, cv_pad, cv_spt;
  uint64_t cv_m_spt, cv_m_kw;   // floor(2^32 / d) + 1 for d = cv_spt, cv_KW: n / d = (n * m) >> 32 for n * d < 2^32
  const void* cv_zero;
};

// dX product of a stride-1 convolution on 128 x 128 tiles by the kernel with the three-stage ring (gemm_kk.hip)
int launch_gemm_kk_conv128(const GemmArgs& a, bool fast, hipStream_t stream);

// Block barrier that orders LDS traffic only.  __syncthreads() also fences global memory, i.e. waits for every
// outstanding global load and store of the wavefront; between the staging writes and reads of an epilogue that
// would expose a memory round trip per barrier.  Global accesses keep their own dependency tracking.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Fused epilogue of the dX product for a 256-thread block whose wavefront (wm, wn) holds the C::WM x C::WN
// sub-tile at (m0 + wm * C::WM, n0 + wn * C::WN) of an M x N output in C::TM x C::TN 32x32 MFMA accumulators.
// smem: at least 4 * 32 * (C::WN + 8) floats, no longer used by the main loop (the caller has synchronised).
template <class C>
__device__ __forceinline__ void epilogue_dx(const GemmArgs& g, floatx16_t (&acc)[C::TM][C::TN], char* smem, int m0,
                                            int n0, int wm, int wn) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
  // dX = dX_q where the activation was not clipped (straight-through), 0 elsewhere; block partial sums
  // of dS_x = sum dX_q * (in range ? (code - Z) - x/S : code - Z) and dZ_x = sum dX_q * (in range ? 0 : -S).
  // The accumulators go through LDS (32 rows of the wave's tile at a time) so that every lane then owns
  // 8 consecutive columns of one row: 8-byte code loads, 16-byte x loads and 16-byte dX stores.
  constexpr int PITCH = C::WN + 8;                   // floats; 4*PITCH = 32 (mod 64) banks
  constexpr int CPR = C::WN / 8;                     // 8-column chunks per row
  constexpr int RPP = 64 / CPR;                      // rows per pass of the wavefront (lanes beyond RPP*CPR idle)
  constexpr int NPASS = (32 + RPP - 1) / RPP;
  float* stage = reinterpret_cast<float*>(smem) + wave * 32 * PITCH;
  const float s = g.s_x[0];
  const float z = rintf(g.z_x[0]);
  const float ninv_s = -1.0f / s;
  const int64_t wpr = (g.N + 31) >> 5;
  const int row_l0 = lane / CPR, ch = lane % CPR;
  const int gcol = n0 + wn * C::WN + ch * 8;
  float ps = 0.0f, pz = 0.0f;
  const bool lane_on = row_l0 < RPP && gcol < g.N;
  if (g.epi_vec) {
    // Vector path (N % 8 == 0, aligned pointers): a lane's 8-column chunk is entirely inside the matrix.
    // The global inputs of 32-row slab i+1 are fetched while slab i is computed, so their latency is hidden
    // even with a single resident block per CU.
    struct Inputs { uint2 cw; uint4 xa, xb; uint32_t mb; };
    Inputs in[2][NPASS];
    auto fetch = [&](int i, int b) {
#pragma unroll
      for (int p = 0; p < NPASS; ++p) {
        const int row_l = p * RPP + row_l0;
        const int grow = m0 + wm * C::WM + i * 32 + row_l;
        if (lane_on && row_l < 32 && grow < g.M) {
          const int64_t e = (int64_t)grow * g.N + gcol;
          in[b][p].mb = g.x_clip[(int64_t)grow * wpr + (gcol >> 5)] >> (gcol & 31);
          in[b][p].cw = *reinterpret_cast<const uint2*>(g.x_codes + e);
          if (g.x_dtype == EFQAT_F32) {
            in[b][p].xa = *reinterpret_cast<const uint4*>((const float*)g.x + e);
            in[b][p].xb = *reinterpret_cast<const uint4*>((const float*)g.x + e + 4);
          } else {
            in[b][p].xa = *reinterpret_cast<const uint4*>((const bf16_t*)g.x + e);
          }
        }
      }
    };
    fetch(0, 0);
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      const int b = i & 1;
      if (i > 0) __syncthreads();
#pragma unroll
      for (int j = 0; j < C::TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          stage[(8 * (r >> 2) + 4 * fh + (r & 3)) * PITCH + j * 32 + fr] = acc[i][j][r];
      __syncthreads();
      if (i + 1 < C::TM) fetch(i + 1, b ^ 1);
#pragma unroll
      for (int p = 0; p < NPASS; ++p) {
        const int row_l = p * RPP + row_l0;
        const int grow = m0 + wm * C::WM + i * 32 + row_l;
        if (lane_on && row_l < 32 && grow < g.M) {
          const float4 a0 = *reinterpret_cast<const float4*>(stage + row_l * PITCH + ch * 8);
          const float4 a1 = *reinterpret_cast<const float4*>(stage + row_l * PITCH + ch * 8 + 4);
          const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
          const int64_t e = (int64_t)grow * g.N + gcol;
          const Inputs& q8 = in[b][p];
          float xv[8];
          if (g.x_dtype == EFQAT_F32) {
            xv[0] = __uint_as_float(q8.xa.x); xv[1] = __uint_as_float(q8.xa.y);
            xv[2] = __uint_as_float(q8.xa.z); xv[3] = __uint_as_float(q8.xa.w);
            xv[4] = __uint_as_float(q8.xb.x); xv[5] = __uint_as_float(q8.xb.y);
            xv[6] = __uint_as_float(q8.xb.z); xv[7] = __uint_as_float(q8.xb.w);
          } else {
            const uint32_t xw[4] = {q8.xa.x, q8.xa.y, q8.xa.z, q8.xa.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              xv[2 * t] = __uint_as_float(xw[t] << 16);
              xv[2 * t + 1] = __uint_as_float(xw[t] & 0xFFFF0000u);
            }
          }
          float o[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            const uint32_t byte = ((t < 4 ? q8.cw.x : q8.cw.y) >> (8 * (t & 3))) & 0xFFu;
            const float q = (float)byte - z;
            const bool inr = (q8.mb >> t) & 1u;
            const float gs = inr ? fmaf(xv[t], ninv_s, q) : q;
            ps = fmaf(a[t], gs, ps);
            o[t] = inr ? a[t] : 0.0f;
            pz += a[t] - o[t];
          }
          if (g.dx_dtype == EFQAT_F32) {
            *reinterpret_cast<float4*>((float*)g.dx + e) = make_float4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<float4*>((float*)g.dx + e + 4) = make_float4(o[4], o[5], o[6], o[7]);
          } else {
            *reinterpret_cast<uint4*>((bf16_t*)g.dx + e) =
                make_uint4(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]),
                           pack_bf16x2(o[6], o[7]));
          }
        }
      }
    }
  } else {
    // Element-wise path for ragged widths / unaligned pointers.
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      if (i > 0) __syncthreads();
#pragma unroll
      for (int j = 0; j < C::TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          stage[(8 * (r >> 2) + 4 * fh + (r & 3)) * PITCH + j * 32 + fr] = acc[i][j][r];
      __syncthreads();
#pragma unroll
      for (int p = 0; p < NPASS; ++p) {
        const int row_l = p * RPP + row_l0;
        const int grow = m0 + wm * C::WM + i * 32 + row_l;
        if (lane_on && row_l < 32 && grow < g.M) {
          const int64_t e = (int64_t)grow * g.N + gcol;
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            if (gcol + t < g.N) {
              const float av = stage[row_l * PITCH + ch * 8 + t];
              const float q = (float)g.x_codes[e + t] - z;
              const float xv = g.x_dtype == EFQAT_F32 ? ((const float*)g.x)[e + t]
                                                      : bf16_to_f32(((const bf16_t*)g.x)[e + t]);
              const bool inr = (g.x_clip[(int64_t)grow * wpr + ((gcol + t) >> 5)] >> ((gcol + t) & 31)) & 1u;
              const float gs = inr ? fmaf(xv, ninv_s, q) : q;
              ps = fmaf(av, gs, ps);
              const float ov = inr ? av : 0.0f;
              pz += av - ov;
              if (g.dx_dtype == EFQAT_F32) ((float*)g.dx)[e + t] = ov;
              else ((bf16_t*)g.dx)[e + t] = f32_to_bf16(ov);
            }
          }
        }
      }
    }
  }
  ps = wave_sum(ps);
  pz = wave_sum(pz);
  __syncthreads();                                   // staging area is dead: reuse for the block sum
  float* red = reinterpret_cast<float*>(smem);
  if (lane == 0) { red[2 * wave] = ps; red[2 * wave + 1] = pz; }
  __syncthreads();
  if (tid == 0) {
    g.partial[2 * blockIdx.x] = (red[0] + red[2]) + (red[4] + red[6]);
    g.partial[2 * blockIdx.x + 1] = -s * ((red[1] + red[3]) + (red[5] + red[7]));
  }
}

// The same epilogue for the case that needs no decision at run time: bf16 x, bf16 dX, every tile of the block grid
// entirely inside the matrix (M % BM == 0, N % BN == 0), M * N < 2^31 so that element offsets fit 32 bits, 16-byte
// aligned x / dX and 8-byte aligned codes.  Straight-line code: LPR lanes share a row of the 32 x WN slab, each
// taking KC of its 8-column chunks (chunk LPR k + lane % LPR), so a pass covers 64 / LPR rows with all 64 lanes busy
// and every address is one per-lane base plus compile-time offsets; no exec-mask sequence or branch separates the
// passes, the LDS reads of the next pass are issued before the arithmetic of the current one, and the global inputs
// of pass p of the next slab are requested as soon as pass p of this slab has consumed its own (one register set, a
// whole slab of prefetch distance).  With a single resident block per CU the predicated, branching formulation
// above runs at about half this speed.
// Per lane: s1 = sum a gs with gs = in range ? (code - Z) - x / S : code - Z, formed term by term as in epilogue_dx
// (in range |gs| <= 1/2, whereas sum a (code - Z) and sum a x / S taken apart would each be some hundred times larger
// and cancel); sd = sum (a - o) with o = in range ? a : 0.
template <class C>
struct EpiDxFast {
  static constexpr int PITCH = C::WN + 8;            // floats; 4*PITCH = 32 (mod 64) banks
  static constexpr int CPR = C::WN / 8;              // 8-column chunks per row
  static constexpr int LPR = (CPR % 8 == 0) ? 8 : 4;
  static_assert(CPR % LPR == 0, "chunks per row");
  static constexpr int KC = CPR / LPR, RP = 64 / LPR, HP = 32 / RP, NP = HP * KC;
  struct Inputs { uint2 cw; uint4 xa; uint32_t mb; };
  Inputs in[NP];
  uint32_t un, uwpr, row_b, col_b;
  const uint8_t* codes; const uint32_t* clip; const bf16_t* xp; bf16_t* dxp;

  // element offset of pass p = (h, k) of slab i
  __device__ __forceinline__ uint32_t elem(int i, int p) const {
    return (row_b + (uint32_t)(32 * i + RP * (p / KC))) * un + col_b + (uint32_t)(8 * LPR * (p % KC));
  }
  __device__ __forceinline__ void fetch(int i, int p) {
    const uint32_t row = row_b + (uint32_t)(32 * i + RP * (p / KC));
    const uint32_t col = col_b + (uint32_t)(8 * LPR * (p % KC));
    const uint32_t e = row * un + col;
    in[p].mb = clip[row * uwpr + (col >> 5)];        // shifted at use: no arithmetic on a value still in flight
    in[p].cw = *reinterpret_cast<const uint2*>(codes + e);
    in[p].xa = *reinterpret_cast<const uint4*>(xp + e);
  }
  // Addresses of this wavefront's sub-tile, and the requests for the inputs of its first slab.  A kernel may call
  // this before its main loop has ended, provided none of its own global -> LDS copies is still outstanding or
  // issued later (a wavefront's loads complete in order).
  __device__ __forceinline__ void prefetch(const GemmArgs& g, int m0, int n0, int wm, int wn) {
    const int lane = threadIdx.x & 63;
    un = (uint32_t)g.N; uwpr = (uint32_t)((g.N + 31) >> 5);
    row_b = (uint32_t)(m0 + wm * C::WM) + (uint32_t)lane / LPR;
    col_b = (uint32_t)(n0 + wn * C::WN) + ((uint32_t)lane % LPR) * 8u;
    codes = g.x_codes; clip = g.x_clip; xp = (const bf16_t*)g.x; dxp = (bf16_t*)g.dx;
#pragma unroll
    for (int p = 0; p < NP; ++p) fetch(0, p);
  }
  // The epilogue proper; prefetch() has been called.  smem: at least 4 * 32 * (C::WN + 8) floats, no longer used by
  // the main loop (the caller has synchronised).  part_idx: the tile's slot in g.partial.
  __device__ __forceinline__ void run(const GemmArgs& g, floatx16_t (&acc)[C::TM][C::TN], char* smem, int part_idx) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;
    float* stage = reinterpret_cast<float*>(smem) + wave * 32 * PITCH;
    const float s = g.s_x[0];
    const float z = rintf(g.z_x[0]);
    const float ninv_s = -1.0f / s;
    const float* st_b = stage + ((uint32_t)lane / LPR) * PITCH + ((uint32_t)lane % LPR) * 8;
    auto lds_chunk = [&](int p, float4& a0, float4& a1) {
      a0 = *reinterpret_cast<const float4*>(st_b + RP * (p / KC) * PITCH + 8 * LPR * (p % KC));
      a1 = *reinterpret_cast<const float4*>(st_b + RP * (p / KC) * PITCH + 8 * LPR * (p % KC) + 4);
    };
    const uint32_t msh = col_b & 31u;                 // a pass moves by a multiple of 32 columns
    static_assert((8 * LPR) % 32 == 0, "mask bit offset is the same in every pass");
    float s1 = 0.0f, sd = 0.0f;
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      if (i > 0) lds_barrier();
#pragma unroll
      for (int j = 0; j < C::TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          stage[(8 * (r >> 2) + 4 * fh + (r & 3)) * PITCH + j * 32 + fr] = acc[i][j][r];
      lds_barrier();
      float4 n0v, n1v;
      lds_chunk(0, n0v, n1v);
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const float a[8] = {n0v.x, n0v.y, n0v.z, n0v.w, n1v.x, n1v.y, n1v.z, n1v.w};
        if (p + 1 < NP) lds_chunk(p + 1, n0v, n1v);
        const Inputs q8 = in[p];
        if (i + 1 < C::TM) fetch(i + 1, p);
        const uint32_t xw[4] = {q8.xa.x, q8.xa.y, q8.xa.z, q8.xa.w};
        float o[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const float xv = (t & 1) ? __uint_as_float(xw[t >> 1] & 0xFFFF0000u) : __uint_as_float(xw[t >> 1] << 16);
          const uint32_t byte = ((t < 4 ? q8.cw.x : q8.cw.y) >> (8 * (t & 3))) & 0xFFu;
          const bool inr = (q8.mb >> (msh + t)) & 1u;
          const float q = (float)byte - z;
          const float gs = inr ? fmaf(xv, ninv_s, q) : q;   // term by term: |gs| <= 1/2 in range, no cancellation later
          s1 = fmaf(a[t], gs, s1);
          o[t] = inr ? a[t] : 0.0f;
          sd += a[t] - o[t];
        }
        *reinterpret_cast<uint4*>(dxp + elem(i, p)) =
            make_uint4(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]),
                       pack_bf16x2(o[6], o[7]));
        __builtin_amdgcn_sched_barrier(0);            // keeps the passes from piling up in registers
      }
    }
    const float ps = wave_sum(s1);
    const float pz = wave_sum(sd);
    lds_barrier();                                   // staging area is dead: reuse for the block sum
    float* red = reinterpret_cast<float*>(smem);
    if (lane == 0) { red[2 * wave] = ps; red[2 * wave + 1] = pz; }
    lds_barrier();
    if (tid == 0) {
      g.partial[2 * part_idx] = (red[0] + red[2]) + (red[4] + red[6]);
      g.partial[2 * part_idx + 1] = -s * ((red[1] + red[3]) + (red[5] + red[7]));
    }
  }
};

template <class C>
__device__ __forceinline__ void epilogue_dx_fast(const GemmArgs& g, floatx16_t (&acc)[C::TM][C::TN], char* smem,
                                                 int m0, int n0, int wm, int wn) {
  EpiDxFast<C> e;
  e.prefetch(g, m0, n0, wm, wn);
  e.run(g, acc, smem, blockIdx.x);
}

}  // namespace efqat
