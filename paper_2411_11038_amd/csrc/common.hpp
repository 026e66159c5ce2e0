// Shared device/host helpers for the EfQAT gfx950 kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/efqat.h"

namespace efqat {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

constexpr int kWave = 64;

__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 (finite inputs)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_hw_t v = {lo, hi};
  bf16x2_hw_t b = __builtin_convertvector(v, bf16x2_hw_t);
  return *reinterpret_cast<uint32_t*>(&b);
}
// exact when the value is representable in bf16 (small integers): plain truncation
__device__ __forceinline__ uint32_t pack_bf16x2_exact(float lo, float hi) {
  return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
}

template <typename T>
__device__ __forceinline__ float load_as_f32(const T* p, int64_t i);
template <>
__device__ __forceinline__ float load_as_f32<float>(const float* p, int64_t i) { return p[i]; }
template <>
__device__ __forceinline__ float load_as_f32<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }

// Workgroups are handed to the 8 XCDs (each with an L2 of its own) round-robin in dispatch order (x fastest, then
// y).  This maps the dispatch-order id to a logical index under which every XCD owns one contiguous range of
// [0, total): blocks with neighbouring logical indices - the tiles of one split-K slice, which share operand
// tiles - run on the same XCD at the same time, so an operand tile is fetched into one L2 instead of into all.
__device__ __forceinline__ int xcd_contiguous_index(int linear, int total) {
  const int q8 = total >> 3, r8 = total & 7, x = linear & 7, j = linear >> 3;
  return x * q8 + (x < r8 ? x : r8) + j;
}

// ---- wave-level reductions in a fixed butterfly order (deterministic)
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// workspace carving: every sub-buffer starts on a 256-byte boundary
struct WsCarver {
  char* base;
  size_t off;
  __host__ explicit WsCarver(void* p) : base((char*)p), off(0) {}
  __host__ void* take(size_t bytes) {
    void* r = base ? (void*)(base + off) : nullptr;
    off += (size_t)round_up((int64_t)bytes, 256);
    return r;
  }
};

#define EFQAT_LAUNCH_CHECK()                              \
  do {                                                    \
    if (hipGetLastError() != hipSuccess) return EFQAT_ERR_HIP; \
  } while (0)

// ---- internal entry points shared between translation units (host side)
struct GemmEpilogueDx {   // fused STE + activation-qparam partial sums (Eq. 5 left, then Eq. 1's STE)
  const uint8_t* x_codes; // [M][N]
  const uint32_t* x_clip; // [M][ceil(N/32)]
  const void* x;          // [M][N] original activations
  int x_dtype;
  const float* s_x;
  const float* z_x;
  void* dx;               // [M][N]
  int dx_dtype;
  float* partial;         // [grid][2] block partial sums of (dS_x, dZ_x)
};
// true when the fused epilogue may use 8-element vector accesses on x_codes / x / dx
bool gemm_epilogue_vec_ok(const GemmEpilogueDx& e, int64_t N);

// Launch shape of one product: square block tile (256, 192 or 128), split-K factor, tile grid.
struct GemmPlan {
  int tile;
  int split_k;
  int tiles_m, tiles_n;
};
// Pure host function of the problem size (so the workspace query and the call agree).  allow_split = false
// for the product with the fused dX epilogue.
GemmPlan gemm_plan(int64_t M, int64_t N, int64_t K, bool allow_split, bool allow_192 = true, bool allow_256 = true,
                   bool fast192 = false);   // fast192: price the 192 tile as k_gemm_kk with its straight-line epilogue

// C[M][N] = sum_k A[row(m)][k] * B[n][k]; both operands bf16 with K contiguous.
//   a_rows: optional gather, row(m) = a_rows[m]; lda/ldb in elements (multiples of 8), K multiple of 8.
//   plan.split_k > 1: K is cut in contiguous slices, slice s goes to out_partial + s*M*N (raw fp32).
//   epi != nullptr (split_k must be 1): fused dX epilogue instead of the raw store; it writes one
//   (dS_x, dZ_x) partial pair per block, plan.tiles_m * plan.tiles_n pairs in all.
int launch_gemm_nt(const bf16_t* A, int64_t lda, const int32_t* a_rows, const bf16_t* B, int64_t ldb,
                   int64_t M, int64_t N, int64_t K, const GemmPlan& plan, float* out_partial,
                   const GemmEpilogueDx* epi, hipStream_t stream);

// The same product as launch_gemm_nt (no row gather) by the kernel with a hand-pinned instruction order:
// plan.tile 256 or 192; A, B and zero_page (>= 256 zero bytes) 16-byte aligned.
int launch_gemm_kk(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, const void* zero_page, int64_t M,
                   int64_t N, int64_t K, const GemmPlan& plan, float* out_partial, const GemmEpilogueDx* epi,
                   hipStream_t stream);

// Weight-gradient product from token-major operands (no transposed copies):
//   out[s][m][n] = sum over the K-slice s of A[t][m] * (B[t][n] - round(z_x)),  A bf16 [K][lda], B uint8 [K][ldb].
// Columns >= a_cols / b_cols and rows >= K are taken as zero (read from zero_page: 256 zero bytes, 256-byte
// aligned).  plan.tile must be 256 or 128.
int launch_gemm_tn(const bf16_t* A, int64_t lda, int64_t a_cols, const uint8_t* B, int64_t ldb, int64_t b_cols,
                   const void* zero_page, const float* z_x, int64_t M, int64_t N, int64_t K, const GemmPlan& plan,
                   float* out_partial, hipStream_t stream);
// dW product of a convolution without a materialised im2col matrix: A = compacted dY columns [N*Ho*Wo][lda] as in
// launch_gemm_tn, B = the activation codes x_codes NHWC gathered with the tap map inside the tile loads.
// N = KH*KW*c_in, c_in % 128 == 0 (a 128-wide column tile lies inside one tap), plan.tile == 128.
struct ConvDwMap { int H, W, Ho, Wo, KW, stride, pad, c_in; };
int launch_gemm_tn_conv(const bf16_t* A, int64_t lda, int64_t a_cols, const uint8_t* x_codes, const ConvDwMap& cm,
                        const void* zero_page, const float* z_x, int64_t M, int64_t N, int64_t K, const GemmPlan& plan,
                        float* out_partial, hipStream_t stream);
// dX product of a stride-1 convolution without a materialised im2col matrix: row m of the A operand is the input
// pixel (n, h, w); its K = (tap, c_out) elements are gathered from the token-major dY [N*Ho*Wo][ldc] inside the
// tile loads (zero_page, 256 zero bytes, stands in for taps that fall outside the output image).  ldc % 64 == 0,
// K = KH*KW*ldc, plan.tile 192 or 128, no split-K.
struct ConvDxMap { int H, W, Ho, Wo, KW, pad; const void* zero_page; };
int launch_gemm_nt_conv_dx(const bf16_t* dy_tok, int64_t ldc, const bf16_t* wqT, int64_t ldb, int64_t M, int64_t N,
                           int64_t K, const ConvDxMap& cm, const GemmPlan& plan, const GemmEpilogueDx& epi,
                           hipStream_t stream);
// dX product with the weight operand read from the int8 codes (K-major [C_out][ldb]) and scaled by s_w[c] in
// registers, fused dX epilogue.  dy: bf16 [M][lda]; N = C_in multiple of 16; tile 256 or 128.  The partial-sum
// array of the epilogue needs ceil(M / tile) * ceil(N / tile) pairs.
int launch_gemm_dx8(const bf16_t* dy, int64_t lda, const int8_t* w_codes, int64_t ldb, const float* s_w,
                    const void* zero_page, int64_t M, int64_t N, int64_t K, int tile, const GemmEpilogueDx& epi,
                    hipStream_t stream);
// The same product for a channel-major dY [C_out][lda] (lda >= M = T, T % 8 == 0): both operands have the contraction
// index C_out as their row and are transposed by the LDS reads; no copy of dY or W_q is made.
int launch_gemm_dx8_cm(const bf16_t* dy_cm, int64_t lda, const int8_t* w_codes, int64_t ldb, const float* s_w,
                       const void* zero_page, int64_t M, int64_t N, int64_t K, int tile, const GemmEpilogueDx& epi,
                       hipStream_t stream);
// dW product for a channel-major bf16 dY [C_out][lda] (lda >= K = T, K % 8 == 0): row m of the A operand is row
// idx[m] of dY, read through the index list in the tile loads; B = the uint8 codes [K][ldb] as they lie.
//   out[s][m][n] = sum over the K-slice s of dY[idx[m]][t] * (codes[t][n] - round(z_x)),  plan.tile 256 or 128.
int launch_gemm_dw_rows(const bf16_t* dy_cm, int64_t lda, const int32_t* idx, const uint8_t* x_codes, int64_t ldb,
                        const void* zero_page, const float* z_x, int64_t M, int64_t N, int64_t K, const GemmPlan& plan,
                        float* out_partial, hipStream_t stream);
// Event timing of kernel classes (benchmarks only, off by default): a ProfScope brackets the launches made during its
// lifetime with two HIP events on the stream they go to.  Classes = the `which` argument of efqat_profile_read.
enum ProfClass {
  PROF_DX = 0, PROF_DW = 1, PROF_FWD = 2, PROF_PREP = 3, PROF_FINISH = 4, PROF_QACT = 5, PROF_QW = 6,
  PROF_IMPORTANCE = 7, PROF_TOPK = 8, PROF_BIAS = 9, PROF_CLASSES = 10
};
bool prof_begin(int which, hipStream_t st, int* slot);
void prof_end(int which, hipStream_t st, int slot);
struct ProfScope {
  int which, slot;
  hipStream_t st;
  bool on;
  ProfScope(int w, hipStream_t s) : which(w), slot(0), st(s), on(prof_begin(w, s, &slot)) {}
  void close() { if (on) { prof_end(which, st, slot); on = false; } }
  ~ProfScope() { close(); }
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;
};

// Eq. 6 scores of every row of w [c_out][block] (double precision), and the Top-K launch, shared by the select and
// the combined weight-side entry points
int launch_row_importance(const float* w, int64_t c_out, int64_t block, double* scores, hipStream_t st);
void launch_topk(const double* scores, int64_t n, int64_t k, int32_t* idx, hipStream_t st);
int launch_topk_profiled(const double* scores, int64_t n, int64_t k, int32_t* idx, hipStream_t st);

// Forward product on int8 matrix cores: y[m][n] = S_x * S_w[n] * sum_k (x_codes[m][k] - round(Z_x)) * w_codes[n][k].
// K, lda, ldb multiples of 16; wsum[n] = sum_k w_codes[n][k].
int launch_gemm_fwd_i8(const uint8_t* x_codes, int64_t lda, const int8_t* w_codes, int64_t ldb, int64_t M, int64_t N,
                       int64_t K, const GemmPlan& plan, const float* s_x, const float* z_x, const float* s_w,
                       const int32_t* wsum, void* y, int y_dtype, hipStream_t stream);

}  // namespace efqat
