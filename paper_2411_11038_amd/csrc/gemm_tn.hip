// Weight-gradient product straight from token-major operands (Eq. 5 right, restricted as in Alg. 1):
//
//   C[m][n] = sum_t A[t][m] * (B[t][n] - z),   A = selected columns of dY, bf16 [T][lda];  B = activation codes, u8 [T][ldb]
//
// Both operands have the contraction index t as their row index, i.e. they are "transposed" for the matrix
// cores, which want K contiguous per lane.  Instead of transposing them through HBM, tiles are copied as they
// are (global -> LDS, global_load_lds_dwordx4) and the MFMA fragments are read with the gfx950 LDS transpose
// loads: ds_read_b64_tr_b16 for A (4 consecutive t of one m per lane), ds_read_b64_tr_b8 for B (8 consecutive
// t of one n), whose bytes are turned into bf16 (code - z, exact) in registers.  The activation operand thus
// costs one byte per element in HBM, L2 and LDS.
//
// 256 threads = 1 x 4 wavefronts, v_mfma_f32_32x32x16_bf16, K-stage of 64 tokens, two LDS stages, the same
// software pipeline as the K-contiguous kernel.  Rows beyond K / columns beyond the operand widths are read
// from a zero page, so no load needs a predicate.  Output: raw fp32 partial tiles (split-K).
#include "common.hpp"

#include <type_traits>

#include "gemm_epilogue.hpp"
#include "lds_copy.hpp"

namespace efqat {

struct GemmTnArgs {
  const bf16_t* A; int64_t lda;       // [K][lda], lda multiple of 8; columns >= a_cols are not read
  const uint8_t* B; int64_t ldb;      // [K][ldb], ldb multiple of 16
  int a_cols, b_cols;                 // readable widths (multiples of 8 / 16): beyond them the zero page is read
  const void* zero_page;              // >= 256 bytes of zeros, 256-byte aligned
  const float* z_x;
  int M, N, K;
  int k_per_split;                    // multiple of 64
  int tiles_m, tiles_n;
  int group_m;                        // row tiles per group of the tile order (the kernels of gemm_tn.hip)
  float* out;                         // raw fp32 [split][M][N]
  // implicit im2col of the B operand (dW product of a convolution): row t is the output pixel (n, ho, wo), the
  // N-tile at n0 belongs to tap n0 / cv_cin = (kh, kw), and the operand is the code of input pixel
  // (n, ho*s + kh - p, wo*s + kw - p), channel n0 % cv_cin + column.  Outside the image the term is dropped by
  // zeroing the A row of that token in this block (a padded activation is 0 after de-quantisation, which need not
  // be a representable code).  cv_dn / cv_dh / cv_dw: how (n, ho, wo) moves when t advances by 64.
  int cv_H, cv_W, cv_Ho, cv_Wo, cv_KW, cv_stride, cv_pad, cv_cin, cv_dn, cv_dh, cv_dw;
};

template <int T>
struct TnCfg {
  static constexpr int BM = T, BN = T;
  // wavefront grid 1 x 4: every wavefront spans all rows of the tile, so each uint8 fragment of B is converted to
  // bf16 by exactly one wavefront
  static constexpr int WGM = 1, WGN = 4;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int RA = 2 * BM, RB = BN;                 // bytes per LDS row (one token)
  static constexpr int CA = RA / 16, CB = RB / 16;           // 16-byte chunks per row
  static constexpr int A_G = 64 * RA / 1024 / 4, B_G = 64 * RB / 1024 / 4;   // 1-KiB loads per wave and stage
  static constexpr int LDS_A = 64 * RA, LDS_B = 64 * RB;
  static constexpr int LDS_STAGE = LDS_A + LDS_B;
  static constexpr int LDS_BYTES = 2 * LDS_STAGE;
  static constexpr int KSH = RB == 256 ? 0 : 1;              // B swizzle: rows per 256 bytes = 1 << KSH
  // physical 16-byte chunk of logical chunk c in token row k.  A: a 16-lane transpose read touches 4 rows x 32
  // bytes, B: 8 rows x 16 bytes; these XORs spread each half-wave's 256 bytes over all 64 banks.
  __device__ static __forceinline__ int swz_a(int c, int k) { return c ^ (4 * (k & 3)); }
  __device__ static __forceinline__ int swz_b(int c, int k) { return c ^ (2 * ((k >> KSH) & (CB / 2 - 1))); }
};

template <int T, bool CONV = false>
__global__ __launch_bounds__(256) void k_gemm_tn(const GemmTnArgs g) {
#if defined(__HIP_DEVICE_COMPILE__)
  using C = TnCfg<T>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / C::WGN, wn = wave % C::WGN;

  // (tile, split-K slice) of this block: slice-major logical order, one contiguous range per XCD
  const int ntile = gridDim.x;
  const int logical = xcd_contiguous_index(blockIdx.y * ntile + blockIdx.x, ntile * gridDim.y);
  const int split = logical / ntile;
  const int pid = logical - split * ntile;
  const int GM = g.group_m;
  const int per_group = GM * g.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsize = (g.tiles_m - first_m) < GM ? (g.tiles_m - first_m) : GM;
  const int tm = first_m + (pid % per_group) % gsize;
  const int tn = (pid % per_group) / gsize;
  const int m0 = tm * C::BM, n0 = tn * C::BN;

  const int k_begin = split * g.k_per_split;
  const int k_end = (k_begin + g.k_per_split) < g.K ? (k_begin + g.k_per_split) : g.K;
  const int span = k_end - k_begin;
  const int nk = span > 0 ? (span + 63) / 64 : 0;

  const int nfull = span > 0 ? span / 64 : 0;          // stages whose 64 token rows all exist

  // ---- global -> LDS copies.  Load slot j of this wave covers the token rows (wave + 4 j) * RPI .. + RPI - 1 of
  // a stage; lane l lands in row l / chunks-per-row, physical chunk l % chunks-per-row, and therefore fetches the
  // logical chunk that the swizzle maps there.  Every slot keeps a running source pointer that moves on by one
  // stage (64 token rows) after each use; slots whose columns lie outside the operand sit on the zero page with
  // stride 0, so the steady-state loads need no predicate and no multiply.
  constexpr int RPIA = 1024 / C::RA, RPIB = 1024 / C::RB;
  const char* zero = (const char*)g.zero_page;
  const int a_r0 = lane / C::CA, b_r0 = lane / C::CB;
  const char* a_ptr[C::A_G];
  const char* b_ptr[C::B_G];
  uint32_t a_st[C::A_G], b_st[C::B_G];
#pragma unroll
  for (int j = 0; j < C::A_G; ++j) {
    const int kr = (wave + 4 * j) * RPIA + a_r0;
    const int col = m0 + C::swz_a(lane % C::CA, kr) * 8;
    const bool on = col < g.a_cols;
    a_ptr[j] = on ? (const char*)g.A + ((int64_t)(k_begin + kr) * g.lda + col) * 2 : zero;
    a_st[j] = on ? (uint32_t)(g.lda * 128) : 0u;
  }
#pragma unroll
  for (int j = 0; j < C::B_G; ++j) {
    const int kr = (wave + 4 * j) * RPIB + b_r0;
    const int col = n0 + C::swz_b(lane % C::CB, kr) * 16;
    const bool on = col < g.b_cols;
    b_ptr[j] = on ? (const char*)g.B + (int64_t)(k_begin + kr) * g.ldb + col : zero;
    b_st[j] = on ? (uint32_t)(g.ldb * 64) : 0u;
  }
  constexpr int LPS = C::A_G + C::B_G;
  // CONV: output-pixel coordinates of every slot's token row (slots 0 .. A_G-1: A, then B), advanced by 64 tokens
  // after each use; the block's tap; per-lane byte offset of the B column inside a pixel
  int cv_n[CONV ? LPS : 1], cv_ho[CONV ? LPS : 1], cv_wo[CONV ? LPS : 1];
  int cv_kh = 0, cv_kw = 0;
  int64_t cv_bcol[CONV ? C::B_G : 1];
  if constexpr (CONV) {
    const int tap = n0 / g.cv_cin;
    cv_kh = tap / g.cv_KW; cv_kw = tap - cv_kh * g.cv_KW;
    const int hw = g.cv_Ho * g.cv_Wo;
#pragma unroll
    for (int t = 0; t < LPS; ++t) {
      const int kr = t < C::A_G ? (wave + 4 * t) * RPIA + a_r0 : (wave + 4 * (t - C::A_G)) * RPIB + b_r0;
      const int tok = k_begin + kr;
      const int n = tok / hw, rem = tok - n * hw;
      cv_n[t] = n; cv_ho[t] = rem / g.cv_Wo; cv_wo[t] = rem - cv_ho[t] * g.cv_Wo;
    }
#pragma unroll
    for (int j = 0; j < C::B_G; ++j) {
      const int kr = (wave + 4 * j) * RPIB + b_r0;
      const int col = (n0 - tap * g.cv_cin) + C::swz_b(lane % C::CB, kr) * 16;
      cv_bcol[j] = col < g.cv_cin ? (int64_t)col : -1;
    }
  }
  // input pixel of slot t's token under the block's tap, or -1 when it lies outside the image; then step the token
  auto cv_pixel = [&](int t) -> int64_t {
    const int hi = cv_ho[t] * g.cv_stride + cv_kh - g.cv_pad, wi = cv_wo[t] * g.cv_stride + cv_kw - g.cv_pad;
    const bool ok = (unsigned)hi < (unsigned)g.cv_H && (unsigned)wi < (unsigned)g.cv_W;
    const int64_t pix = ((int64_t)cv_n[t] * g.cv_H + hi) * g.cv_W + wi;
    int wo = cv_wo[t] + g.cv_dw;
    const int c1 = wo >= g.cv_Wo ? 1 : 0;
    wo -= c1 * g.cv_Wo;
    int ho = cv_ho[t] + g.cv_dh + c1;
    const int c2 = ho >= g.cv_Ho ? 1 : 0;
    ho -= c2 * g.cv_Ho;
    cv_wo[t] = wo; cv_ho[t] = ho; cv_n[t] += g.cv_dn + c2;
    return ok ? pix : -1;
  };
  using Checked = std::integral_constant<bool, true>;
  using Unchecked = std::integral_constant<bool, false>;
  // issues load slots t0 .. t1-1 of stage kt; every slot must be issued exactly once per stage, in stage order
  auto issue_range = [&](auto checked, int kt, int buf, int t0, int t1) {
    char* sa = smem + buf * C::LDS_STAGE;
    char* sb = sa + C::LDS_A;
    const int kb = kt * 64;
#pragma unroll
    for (int t = t0; t < t1; ++t) {
      if (t < C::A_G) {
        const char* src = a_ptr[t];
        if constexpr (CONV) {
          if (cv_pixel(t) < 0) src = zero;              // this token's tap falls into the padding: drop its term
        }
        if constexpr (decltype(checked)::value) {
          if (kb + (wave + 4 * t) * RPIA + a_r0 >= span) src = zero;
        }
        dma16(src, sa + (wave + 4 * t) * 1024);
        a_ptr[t] += a_st[t];
      } else {
        const int u = t - C::A_G;
        const char* src = b_ptr[u];
        if constexpr (CONV) {
          const int64_t pix = cv_pixel(t);
          src = (pix >= 0 && cv_bcol[u] >= 0) ? (const char*)g.B + pix * g.cv_cin + cv_bcol[u] : zero;
        }
        if constexpr (decltype(checked)::value) {
          if (kb + (wave + 4 * u) * RPIB + b_r0 >= span) src = zero;
        }
        dma16(src, sb + (wave + 4 * u) * 1024);
        b_ptr[u] += b_st[u];
      }
    }
  };

  floatx16_t acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // ---- fragment reads.  16-lane group q = lane / 16: m (n) half mb = 16 (q & 1), K half h = q >> 1; s = lane % 16.
  //   A, transpose read r in {0,1}: lane addresses 8 bytes = 4 m at token 16*sub + 8h + 4r + s/4,
  //      m = 32 i + mb + 4 (s % 4);  result: lane owns m = 32 i + mb + s, tokens 8h + 4r + 0..3.
  //      Its 16-byte chunk is 4 i + c0 (c0 < 4), which the swizzle moves to 4 (i ^ (s/4)) + c0: four base
  //      addresses per LDS buffer (one per i % 4) and compile-time offsets for i / 4, r and the sub-step.
  //   B: lane addresses 8 bytes = 8 n at token 16*sub + 8h + s/2, n = wave_n + 32 j + mb + 8 (s % 2);
  //      result: lane owns n = ... + mb + s, tokens 8h + 0..7.
  static_assert(C::WGM == 1 || C::TM <= 4, "A fragment addressing");
  const int s16 = lane & 15, q = lane >> 4;
  const int mb = 16 * (q & 1), h = q >> 1;
  int a_base[2][4], b_base[2][C::TN];           // LDS byte offsets of sub-step 0, per buffer
  {
    const int k = 8 * h + (s16 >> 2), kk = (s16 >> 2) & 3;
    const int c0 = (mb >> 3) + ((s16 & 3) >> 1);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      a_base[0][u] = k * C::RA + ((4 * ((u + wm * (C::WM / 32)) ^ kk) + c0) << 4) + 8 * (s16 & 1);
      a_base[1][u] = a_base[0][u] + C::LDS_STAGE;
    }
  }
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int k = 8 * h + (s16 >> 1);
    const int nbyte = wn * C::WN + 32 * j + mb + 8 * (s16 & 1);
    b_base[0][j] = C::LDS_A + k * C::RB + (C::swz_b(nbyte >> 4, k) << 4) + (nbyte & 15);
    b_base[1][j] = b_base[0][j] + C::LDS_STAGE;
  }
  const float z = rintf(g.z_x[0]);
  shortx4_t af[2][C::TM][2];
  intx2_t braw[2][C::TN];
  uint32_t bw[2][C::TN][4];                         // converted B fragments: 4 words of two bf16 each
  // LDS read number r of a sub-step: the B codes, then the two halves of every A fragment
  constexpr int NRD = C::TN + 2 * C::TM;
  auto lds_read = [&](auto bufc, int sub, int rb, int r) {
    constexpr int buf = decltype(bufc)::value;
    if (r < C::TN) {
      braw[rb][r] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
          (__attribute__((address_space(3))) intx2_t*)(smem + b_base[buf][r] + sub * 16 * C::RB));
    } else {
      const int i = (r - C::TN) >> 1, hh = (r - C::TN) & 1;
      af[rb][i][hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4_t*)(
          smem + a_base[buf][i & 3] + (i >> 2) * 256 + hh * 4 * C::RA + sub * 16 * C::RA));
    }
  };
  auto load_frags = [&](auto bufc, int sub, int rb) {
#pragma unroll
    for (int r = 0; r < NRD; ++r) lds_read(bufc, sub, rb, r);
  };
  // Activation codes -> (code - z) as bf16: integers of magnitude <= 255 are exact.  Piece p of fragment j makes
  // elements 2p and 2p + 1 (5 VALU operations).
  constexpr int NPIECE = 4 * C::TN;
  auto conv_piece = [&](int rb, int piece) {
    const int j = piece >> 2, pp = piece & 3;
    const uint32_t w = (uint32_t)braw[rb][j][pp >> 1];
    const int sh = 16 * (pp & 1);
    const float f0 = (float)((w >> sh) & 0xFFu) - z;
    const float f1 = (float)((w >> (sh + 8)) & 0xFFu) - z;
    bw[rb][j][pp] = pack_bf16x2(f0, f1);
  };
  auto convert = [&](int rb) {
#pragma unroll
    for (int piece = 0; piece < NPIECE; ++piece) conv_piece(rb, piece);
  };
  auto mfma_one = [&](int rb, int i, int j) {
    struct { shortx4_t lo, hi; } a2 = {af[rb][i][0], af[rb][i][1]};
    const uint4 pk = make_uint4(bw[rb][j][0], bw[rb][j][1], bw[rb][j][2], bw[rb][j][3]);
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a2),
                                                        __builtin_bit_cast(bf16x8_t, pk), acc[i][j], 0, 0, 0);
  };
  auto mfma_all = [&](int rb) {
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int j = 0; j < C::TN; ++j) mfma_one(rb, i, j);
  };

  constexpr int P0 = (LPS + 2) / 3, P1 = (LPS - P0 + 1) / 2, P2 = LPS - P0 - P1;
  auto stage_sync = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- main loop, two LDS stages of 64 tokens, four sub-steps of 16 tokens each.  During the MFMAs of sub-step s
  // the fragments of sub-step s+1 are read and its activation bytes converted; sub-steps 0 and 1 also issue the
  // 2nd and 3rd thirds of the loads of stage kt+1; after sub-step 2 everybody synchronises (stage kt+1 complete,
  // buffer kt free); sub-step 3 reads the first fragments of stage kt+1 and issues the first third of stage kt+2.
  // Invariant: when stage kt starts, the first third of stage kt+1 is in flight iff kt+1 < nfull.
  //
  // A steady-state sub-step has its instruction order pinned, one group per MFMA (the compiler's own interleaving
  // left the conversions of some sub-steps in one clump behind the last MFMA): the MFMAs of fragment set rb; in the
  // first half the LDS reads of the next sub-step (set rb ^ 1), in the second half the conversion of what they
  // returned; the first t1 - t0 groups also issue one global->LDS copy each (stage kt_i into buffer buf_i).
  constexpr int MF = C::TM * C::TN, HF = MF / 2;
  static_assert(HF >= 1 && P0 <= MF && P1 <= MF && P2 <= MF, "copies per sub-step must not exceed its MFMAs");
  auto substep = [&](auto bufn, int sub_next, int rb, int kt_i, int buf_i, int t0, int t1) {
#pragma unroll
    for (int qq = 0; qq < MF; ++qq) {
      mfma_one(rb, qq / C::TN, qq % C::TN);
      if (qq < HF) {
#pragma unroll
        for (int r = (qq * NRD) / HF; r < ((qq + 1) * NRD) / HF; ++r) lds_read(bufn, sub_next, rb ^ 1, r);
      }
      if (qq < t1 - t0) issue_range(Unchecked{}, kt_i, buf_i, t0 + qq, t0 + qq + 1);
      if (qq >= MF - HF) {
        const int q2 = qq - (MF - HF);
#pragma unroll
        for (int piece = (q2 * NPIECE) / HF; piece < ((q2 + 1) * NPIECE) / HF; ++piece) conv_piece(rb ^ 1, piece);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto stage = [&](auto bufc, auto steadyc, int kt) {
    constexpr int cur = decltype(bufc)::value;
    constexpr bool ST = decltype(steadyc)::value;
    using Other = std::integral_constant<int, cur ^ 1>;
    if constexpr (ST) {
      __builtin_amdgcn_sched_barrier(0);
      substep(bufc, 1, 0, kt + 1, cur ^ 1, P0, P0 + P1);
      substep(bufc, 2, 1, kt + 1, cur ^ 1, P0 + P1, LPS);
      substep(bufc, 3, 0, 0, 0, 0, 0);
      stage_sync();
      substep(Other{}, 0, 1, kt + 2, cur, 0, P0);
    } else {
      const bool more1 = kt + 1 < nk;
      if (kt + 1 < nfull) issue_range(Unchecked{}, kt + 1, cur ^ 1, P0, LPS);
      else if (more1) issue_range(Checked{}, kt + 1, cur ^ 1, 0, LPS);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 1, 1);
      mfma_all(0);
      convert(1);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 2, 0);
      mfma_all(1);
      convert(0);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 3, 1);
      mfma_all(0);
      convert(1);
      stage_sync();
      if (more1) load_frags(Other{}, 0, 0);
      if (kt + 2 < nfull) issue_range(Unchecked{}, kt + 2, cur, 0, P0);
      mfma_all(1);
      if (more1) convert(0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  using Steady = std::integral_constant<bool, true>;
  using Drain = std::integral_constant<bool, false>;

  if (nk > 0) issue_range(Checked{}, 0, 0, 0, LPS);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (1 < nfull) issue_range(Unchecked{}, 1, 1, 0, P0);
  if (nk > 0) {
    load_frags(B0{}, 0, 0);
    convert(0);
  }
  int kt = 0;
  for (; kt + 3 < nfull; kt += 2) {                    // stages kt+1 .. kt+3 are full: branch-free pair of stages
    stage(B0{}, Steady{}, kt);
    stage(B1{}, Steady{}, kt + 1);
  }
  for (; kt < nk; kt += 2) {                           // the last (up to four) stages, including a ragged one
    stage(B0{}, Drain{}, kt);
    if (kt + 1 < nk) stage(B1{}, Drain{}, kt + 1);
  }

  // ---- raw fp32 partial tile.  Accumulator layout of the 32x32 MFMA: column lane & 31, rows 8 (r/4) + 4 (lane/32) + r%4.
  const int fr = lane & 31, fh = lane >> 5;
  float* out = g.out + (int64_t)split * g.M * g.N;
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      const int col = n0 + wn * C::WN + j * 32 + fr;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * C::WM + i * 32 + 8 * (r >> 2) + 4 * fh + (r & 3);
        if (row < g.M && col < g.N) out[(int64_t)row * g.N + col] = acc[i][j][r];
      }
    }
#endif
}

// ------------------------------------------------------------------------------------------------
// Input-gradient product with the weight operand taken straight from the int8 codes (Eq. 5 left):
//
//   dX_q[t][i] = sum_c dY[t][c] * (S_w[c] * code[c][i]),   A = dY bf16 [T][lda] (K = c contiguous),
//                                                          B = weight codes int8 [C_out][ldb] (K = c is the row)
//
// A tiles are staged and read like any K-contiguous operand (128-byte rows, 16-byte fragment reads); B tiles are
// copied as they lie and read with ds_read_b64_tr_b8, then turned into bf16(S_w[c] * code) in registers with the
// 64 scales of the stage, which travel through LDS as well.  bf16(S_w * code) is the same rounding a materialised
// bf16 copy of W_q would apply, so results do not depend on which kernel runs.  Compared with that copy the
// weight operand costs half the bytes in L2, L1 and LDS (a 256 x 256 stage is 48 KB instead of 64 KB), and the
// transposed bf16 matrix is never written.  Same wavefront grid (1 x 4), pipeline and load discipline as k_gemm_tn;
// the epilogue is the fused straight-through / dS_x / dZ_x epilogue shared with the K-contiguous kernel.
//
// The same kernel in DW mode is the weight-gradient product for a channel-major dY [C_out][T] (Eq. 5 right,
// restricted):  dW_q[m][i] = sum_t dY[idx[m]][t] * (code[t][i] - Z_x).  The A rows are the selected channels, read
// through the index list in the tile loads (frozen channels are never touched), B = the uint8 activation codes as
// they lie ([T][C_in]; the contraction index is the row), converted as in k_gemm_tn; split-K, raw fp32 partial tiles.
// ATN: the A operand has the contraction index as its row ([K][lda], K-major like B) and is read with
// ds_read_b64_tr_b16 as in k_gemm_tn; otherwise it is K-contiguous ([M][lda]).
template <int T, bool ATN = false>
struct Dx8Cfg {
  static constexpr int BM = T, BN = T;
  static constexpr int WGM = 1, WGN = 4;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int RB = BN;                              // bytes per LDS row of B (one channel c)
  static constexpr int CB = RB / 16;
  static constexpr int RA = 2 * BM, CA = RA / 16;            // ATN: bytes / chunks per LDS row of A (one K index)
  static constexpr int A_G = BM / 8 / 4, B_G = 64 * RB / 1024 / 4;   // 1-KiB loads per wave and stage
  static constexpr int LDS_A = BM * 128, LDS_B = 64 * RB, LDS_S = 4 * 256;   // scales: one copy per wavefront
  static constexpr int LDS_STAGE = LDS_A + LDS_B + LDS_S;
  static constexpr int LDS_LOOP = 2 * LDS_STAGE;
  static constexpr int LDS_EPI = 4 * 32 * (WN + 8) * 4;
  static constexpr int LDS_BYTES = LDS_LOOP > LDS_EPI ? LDS_LOOP : LDS_EPI;
  static constexpr int KSH = RB == 256 ? 0 : 1;
  __device__ static __forceinline__ int swz_a(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }
  __device__ static __forceinline__ int swz_atn(int c, int k) { return c ^ (4 * (k & 3)); }
  __device__ static __forceinline__ int swz_b(int c, int k) { return c ^ (2 * ((k >> KSH) & (CB / 2 - 1))); }
};

struct GemmDx8Args {
  int a_cols;              // ATN: readable width of A (multiple of 8)
  GemmArgs g;              // dX: A = dY, B = weight codes, M = T, N = C_in, K = C_out, fused dX epilogue fields
                           // dW: A = dY channel-major with a_rows = idx, B = activation codes, M = k, N = C_in, K = T
  int b_cols;              // readable width of B (multiple of 16)
  const void* zero_page;   // >= 256 zero bytes
};

// FAST (dX only): the straight-line epilogue for bf16 x / dX and whole tiles (epilogue_dx_fast).
template <int T, bool DW = false, bool ATN = false, bool FAST = false>
__global__ __launch_bounds__(256) void k_gemm_dx8(const GemmDx8Args ga) {
#if defined(__HIP_DEVICE_COMPILE__)
  using C = Dx8Cfg<T, ATN>;
  const GemmArgs& g = ga.g;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = 0, wn = wave;

  const int ntile = gridDim.x;
  const int logical = xcd_contiguous_index(blockIdx.y * ntile + blockIdx.x, ntile * gridDim.y);
  const int split = logical / ntile;                   // split-K slice (0 when there is one)
  const int pid = logical - split * ntile;
  const int GM = g.group_m;
  const int per_group = GM * g.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsize = (g.tiles_m - first_m) < GM ? (g.tiles_m - first_m) : GM;
  const int tm = first_m + (pid % per_group) % gsize;
  const int tn = (pid % per_group) / gsize;
  const int m0 = tm * C::BM, n0 = tn * C::BN;

  // K range of this block: everything for dX, one split-K slice for dW (K below is the length of the slice)
  const int k_begin = DW ? split * g.k_per_split : 0;
  const int k_end_ = DW ? ((k_begin + g.k_per_split) < g.K ? (k_begin + g.k_per_split) : g.K) : g.K;
  const int K = k_end_ > k_begin ? k_end_ - k_begin : 0;
  const int nk = (K + 63) / 64;
  const int nfull = K / 64;
  const char* zero = (const char*)ga.zero_page;

  // ---- global -> LDS copies with running pointers (one 64-bit add per copy; slots outside the operands rest on
  // the zero page with stride 0).  A: slot j covers tile rows (wave + 4 j) * 8 .. + 7, lane l lands in row l / 8,
  // physical chunk l % 8.  B: slot j covers channel rows (wave + 4 j) * RPIB .. of the stage.
  constexpr int RPIB = 1024 / C::RB;
  const int a_lrow = lane >> 3;
  const int a_lch = (lane & 7) ^ (((wave * 8 + a_lrow) >> 1) & 7);   // logical chunk fetched by this lane (same for all j)
  const int b_r0 = lane / C::CB;
  const char* a_ptr[C::A_G];
  const char* b_ptr[C::B_G];
  uint32_t b_st[C::B_G];
  uint32_t a_st[C::A_G];                                // per-stage pointer step of the A slots
  constexpr int RPIA = 1024 / C::RA;                    // ATN: K rows per 1-KiB load
  const int atn_r0 = lane / C::CA;
#pragma unroll
  for (int j = 0; j < C::A_G; ++j) {
    if constexpr (ATN) {
      // slot j covers the K rows (wave + 4 j) * RPIA .. of a stage; lane l lands in row l / CA, physical chunk l % CA
      const int kr = (wave + 4 * j) * RPIA + atn_r0;
      const int col = m0 + C::swz_atn(lane % C::CA, kr) * 8;
      const bool on = col < ga.a_cols;
      a_ptr[j] = on ? (const char*)g.A + ((int64_t)(k_begin + kr) * g.lda + col) * 2 : zero;
      a_st[j] = on ? (uint32_t)(g.lda * 128) : 0u;
    } else {
      int gm = m0 + (wave + 4 * j) * 8 + a_lrow;
      gm = gm < g.M ? gm : g.M - 1;                     // rows past the edge re-read a valid row (outputs discarded)
      const int64_t src_row = (DW && g.a_rows) ? (int64_t)g.a_rows[gm] : (int64_t)gm;
      a_ptr[j] = (const char*)g.A + (src_row * g.lda + k_begin) * 2 + a_lch * 16;
      a_st[j] = 128u;
    }
  }
#pragma unroll
  for (int j = 0; j < C::B_G; ++j) {
    const int kr = (wave + 4 * j) * RPIB + b_r0;
    const int col = n0 + C::swz_b(lane % C::CB, kr) * 16;
    const bool on = col < ga.b_cols;
    b_ptr[j] = on ? (const char*)g.B + (int64_t)(k_begin + kr) * g.ldb + col : zero;
    b_st[j] = on ? (uint32_t)(g.ldb * 64) : 0u;
  }
  const char* s_ptr = DW ? zero : (const char*)g.s_w + lane * 4;   // dX: the scale of channel kt * 64 + lane
  constexpr int LPS = C::A_G + C::B_G + (DW ? 0 : 1);
  using Checked = std::integral_constant<bool, true>;
  using Unchecked = std::integral_constant<bool, false>;
  auto issue_range = [&](auto checked, int kt, int buf, int t0, int t1) {
    char* sa = smem + buf * C::LDS_STAGE;
    char* sb = sa + C::LDS_A;
    char* ss = sb + C::LDS_B;
    const int kb = kt * 64;
#pragma unroll
    for (int t = t0; t < t1; ++t) {
      if (t < C::A_G) {
        const char* src = a_ptr[t];
        if constexpr (decltype(checked)::value) {
          if constexpr (ATN) {
            if (kb + (wave + 4 * t) * RPIA + atn_r0 >= K) src = zero;
          } else {
            if (kb + a_lch * 8 >= K) src = zero;        // K is a multiple of 8: a chunk is all in or all out
          }
        }
        dma16(src, sa + (wave + 4 * t) * 1024);
        a_ptr[t] += a_st[t];
      } else if (t < C::A_G + C::B_G) {
        const int u = t - C::A_G;
        const char* src = b_ptr[u];
        if constexpr (decltype(checked)::value) {
          if (kb + (wave + 4 * u) * RPIB + b_r0 >= K) src = zero;
        }
        dma16(src, sb + (wave + 4 * u) * 1024);
        b_ptr[u] += b_st[u];
      } else {
        // every wavefront fetches its own copy of the stage's 64 scales: no branch in the loop body
        const char* src = s_ptr;
        if constexpr (decltype(checked)::value) {
          if (kb + lane >= K) src = zero;
        }
        dma4(src, ss + wave * 256);
        s_ptr += 256;
      }
    }
  };

  floatx16_t acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // ---- fragment reads.  A (rows = tokens, 16 bytes = 8 channels): lane owns row 32 i + lane % 32, channels
  // 16 sub + 8 (lane / 32) + 0..7.  B (transpose read): lane addresses 8 columns of channel 16 sub + 8 h + s / 2 and
  // ends up with column 32 j + lane % 32, channels 16 sub + 8 h + 0..7, h = lane / 32.
  const int fr = lane & 31, fh = lane >> 5;
  const int s16 = lane & 15, q = lane >> 4;
  const int mb = 16 * (q & 1);
  int b_base[2][C::TN];
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int k = 8 * fh + (s16 >> 1);
    const int nbyte = wn * C::WN + 32 * j + mb + 8 * (s16 & 1);
    b_base[0][j] = C::LDS_A + k * C::RB + (C::swz_b(nbyte >> 4, k) << 4) + (nbyte & 15);
    b_base[1][j] = b_base[0][j] + C::LDS_STAGE;
  }
  typedef int intx4_t __attribute__((ext_vector_type(4)));
  intx4_t af[2][C::TM];
  // ATN: four base addresses per LDS buffer for the transpose reads of A (see k_gemm_tn)
  int atn_base[2][4];
  if constexpr (ATN) {
    const int h = q >> 1;
    const int k = 8 * h + (s16 >> 2), kk = (s16 >> 2) & 3;
    const int c0 = (mb >> 3) + ((s16 & 3) >> 1);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      atn_base[0][u] = k * C::RA + ((4 * (u ^ kk) + c0) << 4) + 8 * (s16 & 1);
      atn_base[1][u] = atn_base[0][u] + C::LDS_STAGE;
    }
  }
  intx2_t braw[2][C::TN];
  float scf[2][8];                                  // the 8 scales of a lane's K positions
  uint32_t bw[2][C::TN][4];                         // converted B fragments: 4 words of two bf16 each
  // LDS read number r of a sub-step: B codes, the scales, then the A fragments
  constexpr int NSC = DW ? 0 : 2;                   // LDS reads of scales per sub-step
  constexpr int NRD = C::TN + NSC + (ATN ? 2 : 1) * C::TM;
  auto lds_read = [&](auto bufc, int sub, int rb, int r) {
    constexpr int buf = decltype(bufc)::value;
    const char* st = smem + buf * C::LDS_STAGE;
    if (r < C::TN) {
      braw[rb][r] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
          (__attribute__((address_space(3))) intx2_t*)(smem + b_base[buf][r] + sub * 16 * C::RB));
    } else if (r < C::TN + NSC) {
      const int hlf = r - C::TN;
      const float4 v = *reinterpret_cast<const float4*>(st + C::LDS_A + C::LDS_B + wave * 256 +
                                                        (16 * sub + 8 * fh + 4 * hlf) * 4);
      scf[rb][4 * hlf] = v.x; scf[rb][4 * hlf + 1] = v.y; scf[rb][4 * hlf + 2] = v.z; scf[rb][4 * hlf + 3] = v.w;
    } else if constexpr (ATN) {
      const int i = (r - C::TN - NSC) >> 1, hh = (r - C::TN - NSC) & 1;
      const shortx4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4_t*)(
          smem + atn_base[buf][i & 3] + (i >> 2) * 256 + hh * 4 * C::RA + sub * 16 * C::RA));
      const intx2_t v2 = __builtin_bit_cast(intx2_t, v);
      af[rb][i][2 * hh] = v2[0]; af[rb][i][2 * hh + 1] = v2[1];
    } else {
      const int i = r - C::TN - NSC;
      af[rb][i] = *reinterpret_cast<const intx4_t*>(st + C::swz_a(32 * i + fr, 2 * sub + fh));
    }
  };
  const float zq = DW ? rintf(g.z_x[0]) : 0.0f;
  auto load_frags = [&](auto bufc, int sub, int rb) {
#pragma unroll
    for (int r = 0; r < NRD; ++r) lds_read(bufc, sub, rb, r);
  };
  // Weight codes -> bf16(S_w[c] * code): the signed byte is converted in one operation (the conversion selects and
  // sign-extends the byte of its source) and multiplied by its scale in fp32, then rounded once like the product
  // itself.  Piece p of fragment j makes elements 2p and 2p + 1 (5 VALU operations).
  constexpr int NPIECE = 4 * C::TN;
  auto conv_piece = [&](int rb, int piece) {
    const int j = piece >> 2, pp = piece & 3;
    const int sh = 16 * (pp & 1);
    if constexpr (DW) {                                // activation codes: (code - Z_x), exact in bf16
      const uint32_t w = (uint32_t)braw[rb][j][pp >> 1];
      bw[rb][j][pp] = pack_bf16x2((float)((w >> sh) & 0xFFu) - zq, (float)((w >> (sh + 8)) & 0xFFu) - zq);
    } else {
      const uint32_t w = (uint32_t)braw[rb][j][pp >> 1];
      const float f0 = (float)(int8_t)((w >> sh) & 0xFFu) * scf[rb][2 * pp];
      const float f1 = (float)(int8_t)((w >> (sh + 8)) & 0xFFu) * scf[rb][2 * pp + 1];
      bw[rb][j][pp] = pack_bf16x2(f0, f1);
    }
  };
  auto convert = [&](int rb) {
#pragma unroll
    for (int piece = 0; piece < NPIECE; ++piece) conv_piece(rb, piece);
  };
  auto mfma_one = [&](int rb, int i, int j) {
    const uint4 pk = make_uint4(bw[rb][j][0], bw[rb][j][1], bw[rb][j][2], bw[rb][j][3]);
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[rb][i]),
                                                        __builtin_bit_cast(bf16x8_t, pk), acc[i][j], 0, 0, 0);
  };
  auto mfma_all = [&](int rb) {
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int j = 0; j < C::TN; ++j) mfma_one(rb, i, j);
  };

  constexpr int P0 = (LPS + 2) / 3, P1 = (LPS - P0 + 1) / 2, P2 = LPS - P0 - P1;
  auto stage_sync = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  // One steady-state sub-step with its instruction order pinned, one group per MFMA: the MFMAs of fragment set rb;
  // in the first half the LDS reads of the next sub-step (set rb ^ 1), in the second half the conversion of what
  // they returned; the first t1 - t0 groups also issue one global->LDS copy each (stage kt_i into buffer buf_i).
  constexpr int MF = C::TM * C::TN, HF = MF / 2;
  static_assert(HF >= 1 && P0 <= MF && P1 <= MF && P2 <= MF, "copies per sub-step must not exceed its MFMAs");
  auto substep = [&](auto bufn, int sub_next, int rb, int kt_i, int buf_i, int t0, int t1) {
#pragma unroll
    for (int qq = 0; qq < MF; ++qq) {
      mfma_one(rb, qq / C::TN, qq % C::TN);
      if (qq < HF) {
#pragma unroll
        for (int r = (qq * NRD) / HF; r < ((qq + 1) * NRD) / HF; ++r) lds_read(bufn, sub_next, rb ^ 1, r);
      }
      if (qq < t1 - t0) issue_range(Unchecked{}, kt_i, buf_i, t0 + qq, t0 + qq + 1);
      if (qq >= MF - HF) {
        const int q2 = qq - (MF - HF);
#pragma unroll
        for (int piece = (q2 * NPIECE) / HF; piece < ((q2 + 1) * NPIECE) / HF; ++piece) conv_piece(rb ^ 1, piece);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- main loop: the schedule of k_gemm_tn (two LDS stages, four sub-steps, loads of the next stage in thirds)
  auto stage = [&](auto bufc, auto steadyc, int kt) {
    constexpr int cur = decltype(bufc)::value;
    constexpr bool ST = decltype(steadyc)::value;
    using Other = std::integral_constant<int, cur ^ 1>;
    if constexpr (ST) {
      __builtin_amdgcn_sched_barrier(0);
      substep(bufc, 1, 0, kt + 1, cur ^ 1, P0, P0 + P1);
      substep(bufc, 2, 1, kt + 1, cur ^ 1, P0 + P1, LPS);
      substep(bufc, 3, 0, 0, 0, 0, 0);
      stage_sync();
      substep(Other{}, 0, 1, kt + 2, cur, 0, P0);
    } else {
      const bool more1 = kt + 1 < nk;
      if (kt + 1 < nfull) issue_range(Unchecked{}, kt + 1, cur ^ 1, P0, LPS);
      else if (more1) issue_range(Checked{}, kt + 1, cur ^ 1, 0, LPS);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 1, 1);
      mfma_all(0);
      convert(1);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 2, 0);
      mfma_all(1);
      convert(0);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 3, 1);
      mfma_all(0);
      convert(1);
      stage_sync();
      if (more1) load_frags(Other{}, 0, 0);
      if (kt + 2 < nfull) issue_range(Unchecked{}, kt + 2, cur, 0, P0);
      mfma_all(1);
      if (more1) convert(0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  using Steady = std::integral_constant<bool, true>;
  using Drain = std::integral_constant<bool, false>;

  if (nk > 0) issue_range(Checked{}, 0, 0, 0, LPS);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (1 < nfull) issue_range(Unchecked{}, 1, 1, 0, P0);
  if (nk > 0) {
    load_frags(B0{}, 0, 0);
    convert(0);
  }
  int kt = 0;
  for (; kt + 3 < nfull; kt += 2) {
    stage(B0{}, Steady{}, kt);
    stage(B1{}, Steady{}, kt + 1);
  }
  for (; kt < nk; kt += 2) {
    stage(B0{}, Drain{}, kt);
    if (kt + 1 < nk) stage(B1{}, Drain{}, kt + 1);
  }
  __syncthreads();

  if constexpr (DW) {
    float* out = g.out + (int64_t)split * g.M * g.N;
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int j = 0; j < C::TN; ++j) {
        const int col = n0 + wn * C::WN + j * 32 + fr;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * C::WM + i * 32 + 8 * (r >> 2) + 4 * fh + (r & 3);
          if (row < g.M && col < g.N) out[(int64_t)row * g.N + col] = acc[i][j][r];
        }
      }
  } else if constexpr (FAST) {
    epilogue_dx_fast<C>(g, acc, smem, m0, n0, wm, wn);
  } else {
    epilogue_dx<C>(g, acc, smem, m0, n0, wm, wn);
  }
#endif
}

// Row tiles per group of the tile order (a group's tiles are walked row-fastest, so the 32 tiles that run on an XCD at
// one time are group_m rows by 32 / group_m columns of tiles and share that many operand panels in its L2).  Measured
// on the LLM-sized products: 2 or 3 for 256 x 256 tiles (dX -1.6 %, dW -3 % against 8); no difference for the
// smaller tiles, which stay at 8.
static int tile_group_m(int tile) { return tile == 256 ? 2 : 8; }

template <int T, bool CONV = false>
static int launch_tn_cfg(const GemmTnArgs& a, int split_k, hipStream_t st) {
  using C = TnCfg<T>;
  // set once per process (initialisation of a function-local static is thread-safe)
  static const hipError_t attr = hipFuncSetAttribute((const void*)k_gemm_tn<T, CONV>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
  if (attr != hipSuccess) return EFQAT_ERR_HIP;
  dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)split_k);
  {
    ProfScope prof(PROF_DW, st);
    hipLaunchKernelGGL((k_gemm_tn<T, CONV>), grid, dim3(256), C::LDS_BYTES, st, a);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

int launch_gemm_tn(const bf16_t* A, int64_t lda, int64_t a_cols, const uint8_t* B, int64_t ldb, int64_t b_cols,
                   const void* zero_page, const float* z_x, int64_t M, int64_t N, int64_t K, const GemmPlan& plan,
                   float* out_partial, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (lda % 8) || (ldb % 16) || (a_cols % 8) || (b_cols % 16)) return EFQAT_ERR_BAD_SHAPE;
  if (lda >= (1 << 24) || ldb >= (1 << 24)) return EFQAT_ERR_BAD_SHAPE;   // 32-bit per-stage pointer strides
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || a_cols > lda || b_cols > ldb) return EFQAT_ERR_BAD_SHAPE;
  if (((uintptr_t)A % 16) || ((uintptr_t)B % 16) || ((uintptr_t)zero_page % 256)) return EFQAT_ERR_ALIGNMENT;
  GemmTnArgs a{};
  a.A = A; a.lda = lda; a.B = B; a.ldb = ldb; a.a_cols = (int)a_cols; a.b_cols = (int)b_cols;
  a.zero_page = zero_page; a.z_x = z_x;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)(ceil_div(ceil_div(K, 64), plan.split_k) * 64);
  a.tiles_m = plan.tiles_m; a.tiles_n = plan.tiles_n; a.group_m = tile_group_m(plan.tile);
  a.out = out_partial;
  switch (plan.tile) {
    case 256: return launch_tn_cfg<256>(a, plan.split_k, stream);
    case 128: return launch_tn_cfg<128>(a, plan.split_k, stream);
    default: return EFQAT_ERR_BAD_SHAPE;
  }
}


template <int T, bool DW = false, bool ATN = false, bool FAST = false>
static int launch_dx8_cfg(const GemmDx8Args& a, int split_k, hipStream_t st) {
  using C = Dx8Cfg<T, ATN>;
  // set once per process (initialisation of a function-local static is thread-safe)
  static const hipError_t attr = hipFuncSetAttribute((const void*)k_gemm_dx8<T, DW, ATN, FAST>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
  if (attr != hipSuccess) return EFQAT_ERR_HIP;
  dim3 grid((unsigned)(a.g.tiles_m * a.g.tiles_n), (unsigned)split_k);
  {
    ProfScope prof(DW ? PROF_DW : PROF_DX, st);
    hipLaunchKernelGGL((k_gemm_dx8<T, DW, ATN, FAST>), grid, dim3(256), C::LDS_BYTES, st, a);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

// nothing left to decide in the epilogue: bf16 in and out, whole tiles, 32-bit element offsets, aligned pointers
static bool dx8_epilogue_fast(const GemmArgs& g, const GemmEpilogueDx& epi, int tile) {
  return g.epi_vec && epi.x_dtype == EFQAT_BF16 && epi.dx_dtype == EFQAT_BF16 && (g.M % tile) == 0 &&
         (g.N % tile) == 0 && (int64_t)g.M * g.N <= (int64_t)INT32_MAX;
}

int launch_gemm_dx8_cm(const bf16_t* dy_cm, int64_t lda, const int8_t* w_codes, int64_t ldb, const float* s_w,
                       const void* zero_page, int64_t M, int64_t N, int64_t K, int tile, const GemmEpilogueDx& epi,
                       hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (M % 8) || (lda % 8) || (ldb % 16) || (N % 16)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || ldb >= (1 << 24) || lda >= (1 << 24)) return EFQAT_ERR_BAD_SHAPE;
  if (((uintptr_t)dy_cm % 16) || ((uintptr_t)w_codes % 16) || ((uintptr_t)s_w % 4) || ((uintptr_t)zero_page % 256))
    return EFQAT_ERR_ALIGNMENT;
  GemmDx8Args a{};
  a.g.A = dy_cm; a.g.lda = lda; a.g.B = w_codes; a.g.ldb = ldb;
  a.g.M = (int)M; a.g.N = (int)N; a.g.K = (int)K;
  a.g.s_w = s_w;
  a.g.x_codes = epi.x_codes; a.g.x_clip = epi.x_clip; a.g.x = epi.x; a.g.x_dtype = epi.x_dtype;
  a.g.s_x = epi.s_x; a.g.z_x = epi.z_x; a.g.dx = epi.dx; a.g.dx_dtype = epi.dx_dtype; a.g.partial = epi.partial;
  a.g.epi_vec = gemm_epilogue_vec_ok(epi, N) ? 1 : 0;
  a.g.tiles_m = (int)ceil_div(M, tile); a.g.tiles_n = (int)ceil_div(N, tile); a.g.group_m = tile_group_m(tile);
  a.a_cols = (int)M; a.b_cols = (int)N;
  a.zero_page = zero_page;
  switch (tile) {
    case 256: return dx8_epilogue_fast(a.g, epi, 256) ? launch_dx8_cfg<256, false, true, true>(a, 1, stream)
                                                      : launch_dx8_cfg<256, false, true>(a, 1, stream);
    case 128: return dx8_epilogue_fast(a.g, epi, 128) ? launch_dx8_cfg<128, false, true, true>(a, 1, stream)
                                                      : launch_dx8_cfg<128, false, true>(a, 1, stream);
    default: return EFQAT_ERR_BAD_SHAPE;
  }
}

int launch_gemm_dw_rows(const bf16_t* dy_cm, int64_t lda, const int32_t* idx, const uint8_t* x_codes, int64_t ldb,
                        const void* zero_page, const float* z_x, int64_t M, int64_t N, int64_t K, const GemmPlan& plan,
                        float* out_partial, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (K % 8) || (lda % 8) || (ldb % 16) || (N % 16)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || ldb >= (1 << 24)) return EFQAT_ERR_BAD_SHAPE;
  if (((uintptr_t)dy_cm % 16) || ((uintptr_t)x_codes % 16) || ((uintptr_t)zero_page % 256)) return EFQAT_ERR_ALIGNMENT;
  GemmDx8Args a{};
  a.g.A = dy_cm; a.g.lda = lda; a.g.a_rows = idx; a.g.B = x_codes; a.g.ldb = ldb;
  a.g.M = (int)M; a.g.N = (int)N; a.g.K = (int)K;
  a.g.k_per_split = (int)(ceil_div(ceil_div(K, 64), plan.split_k) * 64);
  a.g.z_x = z_x; a.g.out = out_partial;
  a.g.tiles_m = plan.tiles_m; a.g.tiles_n = plan.tiles_n; a.g.group_m = tile_group_m(plan.tile);
  a.b_cols = (int)N;
  a.zero_page = zero_page;
  switch (plan.tile) {
    case 256: return launch_dx8_cfg<256, true>(a, plan.split_k, stream);
    case 128: return launch_dx8_cfg<128, true>(a, plan.split_k, stream);
    default: return EFQAT_ERR_BAD_SHAPE;
  }
}

int launch_gemm_tn_conv(const bf16_t* A, int64_t lda, int64_t a_cols, const uint8_t* x_codes, const ConvDwMap& cm,
                        const void* zero_page, const float* z_x, int64_t M, int64_t N, int64_t K, const GemmPlan& plan,
                        float* out_partial, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (lda % 8) || (a_cols % 8) || a_cols > lda || lda >= (1 << 24)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || plan.tile != 128 || (cm.c_in % 128) != 0)
    return EFQAT_ERR_BAD_SHAPE;
  if (((uintptr_t)A % 16) || ((uintptr_t)x_codes % 16) || ((uintptr_t)zero_page % 256)) return EFQAT_ERR_ALIGNMENT;
  GemmTnArgs a{};
  a.A = A; a.lda = lda; a.B = x_codes; a.ldb = 0; a.a_cols = (int)a_cols; a.b_cols = INT32_MAX;
  a.zero_page = zero_page; a.z_x = z_x;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)(ceil_div(ceil_div(K, 64), plan.split_k) * 64);
  a.tiles_m = plan.tiles_m; a.tiles_n = plan.tiles_n; a.group_m = tile_group_m(plan.tile);
  a.out = out_partial;
  a.cv_H = cm.H; a.cv_W = cm.W; a.cv_Ho = cm.Ho; a.cv_Wo = cm.Wo; a.cv_KW = cm.KW; a.cv_stride = cm.stride;
  a.cv_pad = cm.pad; a.cv_cin = cm.c_in;
  const int hw = cm.Ho * cm.Wo, rem = 64 % hw;
  a.cv_dn = 64 / hw; a.cv_dh = rem / cm.Wo; a.cv_dw = rem % cm.Wo;
  return launch_tn_cfg<128, true>(a, plan.split_k, stream);
}

int launch_gemm_dx8(const bf16_t* dy, int64_t lda, const int8_t* w_codes, int64_t ldb, const float* s_w,
                    const void* zero_page, int64_t M, int64_t N, int64_t K, int tile, const GemmEpilogueDx& epi,
                    hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (K % 8) || (lda % 8) || (ldb % 16) || (N % 16)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || ldb >= (1 << 24)) return EFQAT_ERR_BAD_SHAPE;
  if (((uintptr_t)dy % 16) || ((uintptr_t)w_codes % 16) || ((uintptr_t)s_w % 4) || ((uintptr_t)zero_page % 256))
    return EFQAT_ERR_ALIGNMENT;
  GemmDx8Args a{};
  a.g.A = dy; a.g.lda = lda; a.g.B = w_codes; a.g.ldb = ldb;
  a.g.M = (int)M; a.g.N = (int)N; a.g.K = (int)K;
  a.g.s_w = s_w;
  a.g.x_codes = epi.x_codes; a.g.x_clip = epi.x_clip; a.g.x = epi.x; a.g.x_dtype = epi.x_dtype;
  a.g.s_x = epi.s_x; a.g.z_x = epi.z_x; a.g.dx = epi.dx; a.g.dx_dtype = epi.dx_dtype; a.g.partial = epi.partial;
  a.g.epi_vec = gemm_epilogue_vec_ok(epi, N) ? 1 : 0;
  a.g.tiles_m = (int)ceil_div(M, tile); a.g.tiles_n = (int)ceil_div(N, tile); a.g.group_m = tile_group_m(tile);
  a.b_cols = (int)N;
  a.zero_page = zero_page;
  switch (tile) {
    case 256: return dx8_epilogue_fast(a.g, epi, 256) ? launch_dx8_cfg<256, false, false, true>(a, 1, stream)
                                                      : launch_dx8_cfg<256>(a, 1, stream);
    case 128: return dx8_epilogue_fast(a.g, epi, 128) ? launch_dx8_cfg<128, false, false, true>(a, 1, stream)
                                                      : launch_dx8_cfg<128>(a, 1, stream);
    default: return EFQAT_ERR_BAD_SHAPE;
  }
}

}  // namespace efqat
