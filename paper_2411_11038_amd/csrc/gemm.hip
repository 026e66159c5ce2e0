// bf16 MFMA GEMM core for gfx950:  C[M][N] = sum_k A[row(m)][k] * B[n][k]   (both operands K-contiguous).
//
// It serves both contractions of Eq. 5:
//   dX_q = dY . W_q        A = dY [T][C_out],               B = W_q^T [C_in][C_out]
//   dW_q[id] = dY[:,id]^T X_q   A = rows id of dY^T [C_out][T] (gather fused into the A-tile loads),
//                               B = (codes - Z_x)^T [C_in][T]
// 256 threads = 4 wavefronts in a 2x2 grid, v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  Operand tiles
// go global -> LDS directly (global_load_lds_dwordx4, 128-byte row segments = whole cache lines per request)
// into two LDS stages of K = 64 with an XOR swizzle that makes the ds_read_b128 fragment reads conflict free;
// fragments are double-buffered in registers and the loads of the stage after next are spread over three of the
// four MFMA sub-steps.  Split-K writes raw fp32 partial tiles (deterministic second-pass reduction).
#include "common.hpp"

#include <type_traits>

#include "gemm_epilogue.hpp"

namespace efqat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef int intx4_t __attribute__((ext_vector_type(4)));
typedef int intx16_t __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

#ifndef EFQAT_GEMM_GM
#define EFQAT_GEMM_GM 8   // row tiles per group of the block -> tile walk
#endif
constexpr int KALIGN = 64;  // split-K slices start on multiples of this many K elements



// BM x BN output tile per 256-thread block; one LDS stage holds 128 bytes of K per tile row (64 bf16 or 128 int8),
// S stages.
template <int BM, int BN, int S>
struct TileCfg {
  static constexpr int BKT = 64;                        // K in units of 2 bytes
  static constexpr int WM = BM / 2, WN = BN / 2;        // per-wave tile (2 x 2 wavefronts)
  static constexpr int TM = WM / 32, TN = WN / 32;      // MFMA tiles per wave
  static constexpr int PITCH_B = BKT * 2;               // bytes per tile row in LDS
  static constexpr int CPRW = BKT / 8;                  // 16-byte chunks per row
  static constexpr int RPI = 1024 / PITCH_B;            // rows covered by one 1-KiB wave load
  static constexpr int R256 = 256 / PITCH_B;            // rows per 256 bytes (LDS bank period for b128)
  static constexpr int A_G = BM / RPI / 4, B_G = BN / RPI / 4;  // 1-KiB row groups per wave and stage
  static constexpr int NS = BKT / 16;                   // MFMA sub-steps per stage
  static constexpr int LDS_A = BM * PITCH_B, LDS_B = BN * PITCH_B;
  static constexpr int LDS_STAGE = LDS_A + LDS_B;
  static constexpr int LDS_LOOP = S * LDS_STAGE;
  static constexpr int LDS_EPI = 4 * 32 * (WN + 8) * 4;  // staging of the fused dX epilogue
  static constexpr int LDS_BYTES = LDS_LOOP > LDS_EPI ? LDS_LOOP : LDS_EPI;
  // XOR swizzle: 16 consecutive rows read the same logical chunk in one ds_read_b128 quarter-wave; with
  // f(row) = (row / R256) mod CPRW the 16 physical chunks are distinct modulo 256 bytes (64 banks).
  __device__ static __forceinline__ int swz(int row, int chunk) {
    return row * PITCH_B + ((chunk ^ ((row / R256) & (CPRW - 1))) << 4);
  }
};

struct True { static constexpr bool value = true; };
struct False { static constexpr bool value = false; };

// Scheduling hint for one MFMA sub-step: NR groups of (a share of the MF MFMAs, one LDS fragment read), the
// first NL groups followed by one global->LDS load.  The group sizes must be compile-time constants.
template <int MF, int NR, int NL, int Q>
struct SchedPattern {
  static __device__ __forceinline__ void run() {
    if constexpr (Q < NR) {
      __builtin_amdgcn_sched_group_barrier(0x008, ((Q + 1) * MF) / NR - (Q * MF) / NR, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if constexpr (Q < NL) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      SchedPattern<MF, NR, NL, Q + 1>::run();
    }
  }
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// EPI: EPI_RAW fp32 partial tiles (split-K), EPI_DX fused dX epilogue, EPI_FWD forward epilogue.
// I8: operands are int8 codes (A unsigned, re-biased by 128 in registers) on v_mfma_i32_32x32x32_i8; else bf16.
// CONV: the A operand is gathered from a token-major dY with the im2col map of a stride-1 convolution (see GemmArgs).
template <int BM, int BN, int EPI, bool I8, bool CONV = false>
__global__ __launch_bounds__(256) void k_gemm_nt(const GemmArgs g) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only builtins; the host pass needs only the launch stub
  constexpr int S = 2;
  constexpr int ESZ = I8 ? 1 : 2;                       // bytes per K element
  constexpr int BKT = 128 / ESZ;                        // K elements per LDS stage
  static_assert(I8 == (EPI == EPI_FWD), "the int8 product is the forward pass");
  using C = TileCfg<BM, BN, S>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS bases stay scalar
  const int wm = wave >> 1, wn = wave & 1;

  // ---- block -> tile: spread contiguous tile ranges over the 8 XCDs (one L2 each), then walk the
  // range in groups of 8 row-tiles so that concurrently resident blocks share operand panels.
  const int ntile = gridDim.x;
  const int logical = xcd_contiguous_index(blockIdx.y * ntile + blockIdx.x, ntile * gridDim.y);
  const int split = logical / ntile;                   // split-K slice (0 when there is one)
  const int pid = logical - split * ntile;
  const int GM = EFQAT_GEMM_GM;
  const int per_group = GM * g.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsize = (g.tiles_m - first_m) < GM ? (g.tiles_m - first_m) : GM;
  const int tm = first_m + (pid % per_group) % gsize;
  const int tn = (pid % per_group) / gsize;
  const int m0 = tm * BM, n0 = tn * BN;
  const int lm0 = m0, ln0 = n0;

  const int k_begin = split * g.k_per_split;
  const int k_end = (k_begin + g.k_per_split) < g.K ? (k_begin + g.k_per_split) : g.K;

  // ---- operand staging.  One wave instruction of the direct global->LDS load (global_load_lds_dwordx4)
  // fills 1 KiB of contiguous LDS = RPI tile rows: lane l lands in row RPI*grp + l / CPRW, slot l % CPRW, so
  // it must fetch the logical chunk slot ^ f(row) of that row (f is the same for every group of a wave).
  const int lrow = lane / C::CPRW, slot = lane % C::CPRW;
  const int lch = slot ^ (((wave * C::RPI + lrow) / C::R256) & (C::CPRW - 1));
  const char* a_ptr[C::A_G];
  const char* b_ptr[C::B_G];
  int cv_q0[CONV ? C::A_G : 1], cv_hw[CONV ? C::A_G : 1];   // CONV: n * Ho * Wo and (h << 16 | w) of the slot's pixel
#pragma unroll
  for (int j = 0; j < C::A_G; ++j) {
    int gm = lm0 + (wave + 4 * j) * C::RPI + lrow;
    gm = gm < g.M ? gm : g.M - 1;                       // rows past the edge re-read a valid row
    if constexpr (CONV) {
      const int hw = g.cv_H * g.cv_W;
      const int n = gm / hw, rem = gm - n * hw;
      const int h = rem / g.cv_W, w = rem - h * g.cv_W;
      cv_q0[j] = n * g.cv_Ho * g.cv_Wo;
      cv_hw[j] = (h << 16) | w;
      a_ptr[j] = nullptr;
    } else {
      const int64_t src = g.a_rows ? (int64_t)g.a_rows[gm] : (int64_t)gm;
      a_ptr[j] = (const char*)g.A + (src * g.lda + k_begin) * ESZ + lch * 16;
    }
  }
  // source of this lane's 16 bytes of A-slot j in stage kt
  auto a_src = [&](int j, int kt) -> const char* {
    if constexpr (CONV) {
      const int sidx = k_begin / 64 + kt;              // 64-channel stage index along K = (tap, channel)
      const int tap = (int)(((uint64_t)(uint32_t)sidx * g.cv_m_spt) >> 32), cst = sidx - tap * g.cv_spt;
      const int kh = (int)(((uint64_t)(uint32_t)tap * g.cv_m_kw) >> 32), kw = tap - kh * g.cv_KW;
      const int ho = (cv_hw[j] >> 16) + g.cv_pad - kh, wo = (cv_hw[j] & 0xFFFF) + g.cv_pad - kw;
      const bool ok = (unsigned)ho < (unsigned)g.cv_Ho && (unsigned)wo < (unsigned)g.cv_Wo;
      const int64_t pix = (int64_t)cv_q0[j] + ho * g.cv_Wo + wo;
      return ok ? (const char*)g.A + (pix * g.lda + cst * 64) * 2 + lch * 16 : (const char*)g.cv_zero;
    } else {
      return a_ptr[j] + kt * 128;
    }
  };
#pragma unroll
  for (int j = 0; j < C::B_G; ++j) {
    int gn = ln0 + (wave + 4 * j) * C::RPI + lrow;
    gn = gn < g.N ? gn : g.N - 1;
    b_ptr[j] = (const char*)g.B + ((int64_t)gn * g.ldb + k_begin) * ESZ + lch * 16;
  }
  const int span = k_end - k_begin;
  const int nfull = span > 0 ? span / BKT : 0;         // stages that need no predicate
  const int nk = span > 0 ? (span + BKT - 1) / BKT : 0;

  constexpr int LPS = C::A_G + C::B_G;                 // wave-level 1-KiB loads per stage
  auto issue_direct = [&](int kt, int buf) {           // a full, unpredicated stage
    char* sa = smem + buf * C::LDS_STAGE;
    char* sb = sa + C::LDS_A;
    const int koff = kt * 128;                          // bytes
#pragma unroll
    for (int j = 0; j < C::A_G; ++j)
      __builtin_amdgcn_global_load_lds(a_src(j, kt), (lds_ptr_t)(sa + (wave + 4 * j) * 1024), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < C::B_G; ++j)
      __builtin_amdgcn_global_load_lds(b_ptr[j] + koff, (lds_ptr_t)(sb + (wave + 4 * j) * 1024), 16, 0, 0);
  };
  // any stage: a ragged last stage goes through registers.  K is a multiple of 8, so a 16-byte chunk is
  // all in or all out; missing chunks are written as zeros.
  auto issue = [&](int kt, int buf) {
    if (kt < nfull) {
      issue_direct(kt, buf);
    } else {
      char* sa = smem + buf * C::LDS_STAGE;
      char* sb = sa + C::LDS_A;
      const int koff = kt * 128;                          // bytes
      const bool ok = (koff + lch * 16) < span * ESZ;
#pragma unroll
      for (int j = 0; j < C::A_G; ++j) {
        const uint4 v = ok ? *reinterpret_cast<const uint4*>(a_src(j, kt)) : make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(sa + (wave + 4 * j) * 1024 + lane * 16) = v;
      }
#pragma unroll
      for (int j = 0; j < C::B_G; ++j) {
        const uint4 v = ok ? *reinterpret_cast<const uint4*>(b_ptr[j] + koff) : make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(sb + (wave + 4 * j) * 1024 + lane * 16) = v;
      }
    }
  };

  typename std::conditional<I8, intx16_t, floatx16_t>::type acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int fr = lane & 31, fh = lane >> 5;
  const int a_row0 = wm * C::WM + fr, b_row0 = wn * C::WN + fr;
  intx4_t af[2][C::TM], bfr[2][C::TN];                  // 16-byte fragments: 8 bf16 or 16 int8 along K
  auto load_frags = [&](int buf, int s, int rb) {
    const char* sa = smem + buf * C::LDS_STAGE;
    const char* sb = sa + C::LDS_A;
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
      af[rb][i] = *reinterpret_cast<const intx4_t*>(sa + C::swz(a_row0 + i * 32, 2 * s + fh));
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
      bfr[rb][j] = *reinterpret_cast<const intx4_t*>(sb + C::swz(b_row0 + j * 32, 2 * s + fh));
  };
  auto mfma_all = [&](int rb) {
    if constexpr (I8) {
      // activation codes are unsigned: x - 128 fits int8 (flip the top bit of every byte); the epilogue adds
      // 128 * sum_k w back
#pragma unroll
      for (int i = 0; i < C::TM; ++i) af[rb][i] ^= (int)0x80808080;
    }
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int j = 0; j < C::TN; ++j) {
        if constexpr (I8)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[rb][i], bfr[rb][j], acc[i][j], 0, 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[rb][i]),
                                                              __builtin_bit_cast(bf16x8_t, bfr[rb][j]), acc[i][j],
                                                              0, 0, 0);
      }
  };

  // ---- main loop, two LDS stages.  Stage kt computes from buffer kt & 1 in NS = 4 sub-steps of K = 16:
  //   sub-step s < 3: read the fragments of sub-step s+1 while the MFMAs of sub-step s run; sub-steps 0 and 1
  //     also issue the 2nd and 3rd thirds of the loads of stage kt+1 into the other buffer;
  //   then wait for this wave's LDS reads and global->LDS loads, and barrier: stage kt+1 is complete for
  //     everybody and nobody reads this stage's buffer any more;
  //   sub-step 3: read the first fragments of stage kt+1 and issue the 1st third of the loads of stage kt+2
  //     into this stage's (now free) buffer, under the MFMAs of sub-step 3.
  // Every load thus has at least one full sub-step (16 MFMAs per wave) to land, and the texture addresser never
  // sees more than a third of a stage at once.
  static_assert(S == 2 && C::NS == 4, "two-stage schedule");
  constexpr int MF = C::TM * C::TN, NR = C::TM + C::TN;
  constexpr int P0 = (LPS + 2) / 3, P1 = (LPS - P0 + 1) / 2, P2 = LPS - P0 - P1;   // loads per third
  auto issue_range = [&](int kt, int buf, int t0, int t1) {
    char* sa = smem + buf * C::LDS_STAGE;
    char* sb = sa + C::LDS_A;
    const int koff = kt * 128;                          // bytes
#pragma unroll
    for (int t = t0; t < t1; ++t) {
      if (t < C::A_G)
        __builtin_amdgcn_global_load_lds(a_src(t, kt), (lds_ptr_t)(sa + (wave + 4 * t) * 1024), 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds(b_ptr[t - C::A_G] + koff,
                                         (lds_ptr_t)(sb + (wave + 4 * (t - C::A_G)) * 1024), 16, 0, 0);
    }
  };
  auto stage_sync = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  if (nk > 0) issue(0, 0);
  wait_vmcnt<0>();
  __syncthreads();
  if (1 < nfull) issue_range(1, 1, 0, P0);
  if (nk > 0) load_frags(0, 0, 0);
  int kt = 0;
  // steady state: stages kt+1 and kt+2 are full stages -> branch-free body, one scheduling region per sub-step
  for (; kt + 2 < nfull; ++kt) {
    const int cur = kt & 1;
    __builtin_amdgcn_sched_barrier(0);
    load_frags(cur, 1, 1);
    issue_range(kt + 1, cur ^ 1, P0, P0 + P1);
    mfma_all(0);
    SchedPattern<MF, NR, P1, 0>::run();
    __builtin_amdgcn_sched_barrier(0);
    load_frags(cur, 2, 0);
    issue_range(kt + 1, cur ^ 1, P0 + P1, LPS);
    mfma_all(1);
    SchedPattern<MF, NR, P2, 0>::run();
    __builtin_amdgcn_sched_barrier(0);
    load_frags(cur, 3, 1);
    mfma_all(0);
    SchedPattern<MF, NR, 0, 0>::run();
    stage_sync();
    load_frags(cur ^ 1, 0, 0);
    issue_range(kt + 2, cur, 0, P0);
    mfma_all(1);
    SchedPattern<MF, NR, P0, 0>::run();
    __builtin_amdgcn_sched_barrier(0);
  }
  // drain: the last stages, including a ragged one
  for (; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nfull) issue_range(kt + 1, cur ^ 1, P0, LPS);   // its first third is already in flight
    else if (kt + 1 < nk) issue(kt + 1, cur ^ 1);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(cur, 1, 1);
    mfma_all(0);
    SchedPattern<MF, NR, 0, 0>::run();
    __builtin_amdgcn_sched_barrier(0);
    load_frags(cur, 2, 0);
    mfma_all(1);
    SchedPattern<MF, NR, 0, 0>::run();
    __builtin_amdgcn_sched_barrier(0);
    load_frags(cur, 3, 1);
    mfma_all(0);
    SchedPattern<MF, NR, 0, 0>::run();
    stage_sync();
    if (kt + 1 < nk) load_frags(cur ^ 1, 0, 0);
    mfma_all(1);
  }
  __syncthreads();

  // ---- epilogue.  MFMA 32x32 accumulator layout: lane holds column (lane & 31) and rows
  // 8*(r/4) + 4*(lane >> 5) + (r % 4), r = 0..15.
  if constexpr (EPI == EPI_RAW) {
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
  } else if constexpr (EPI == EPI_DX) {
    epilogue_dx<C>(g, acc, smem, m0, n0, wm, wn);
  } else if constexpr (EPI == EPI_DXF) {
    epilogue_dx_fast<C>(g, acc, smem, m0, n0, wm, wn);
  } else {
    // Forward epilogue: the int32 sums are over (code - 128) * w, so
    //   y[m][n] = S_x * S_w[n] * (acc + (128 - round(Z_x)) * sum_k w[n][k]).
    // Accumulators go through LDS so that a lane owns 8 consecutive columns of a row (16/32-byte stores).
    constexpr int PITCH = C::WN + 8;
    constexpr int CPR = C::WN / 8;
    constexpr int RPP = 64 / CPR;
    constexpr int NPASS = (32 + RPP - 1) / RPP;
    int* stage = reinterpret_cast<int*>(smem) + wave * 32 * PITCH;
    const float sx = g.s_x[0];
    const long long zc = 128 - (long long)rintf(g.z_x[0]);
    const int row_l0 = lane / CPR, ch = lane % CPR;
    const int gcol = n0 + wn * C::WN + ch * 8;
    const bool lane_on = row_l0 < RPP && gcol < g.N;
    float scl[8];
    long long corr[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const bool ok = lane_on && gcol + t < g.N;
      scl[t] = ok ? sx * g.s_w[gcol + t] : 0.0f;
      corr[t] = ok ? zc * (long long)g.wsum[gcol + t] : 0;
    }
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
          const int4 a0 = *reinterpret_cast<const int4*>(stage + row_l * PITCH + ch * 8);
          const int4 a1 = *reinterpret_cast<const int4*>(stage + row_l * PITCH + ch * 8 + 4);
          const int a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
          float o[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) o[t] = scl[t] * (float)((long long)a[t] + corr[t]);
          const int64_t e = (int64_t)grow * g.N + gcol;
          if (g.epi_vec && gcol + 8 <= g.N) {
            if (g.y_dtype == EFQAT_F32) {
              *reinterpret_cast<float4*>((float*)g.y + e) = make_float4(o[0], o[1], o[2], o[3]);
              *reinterpret_cast<float4*>((float*)g.y + e + 4) = make_float4(o[4], o[5], o[6], o[7]);
            } else {
              *reinterpret_cast<uint4*>((bf16_t*)g.y + e) =
                  make_uint4(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]),
                             pack_bf16x2(o[6], o[7]));
            }
          } else {
#pragma unroll
            for (int t = 0; t < 8; ++t)
              if (gcol + t < g.N) {
                if (g.y_dtype == EFQAT_F32) ((float*)g.y)[e + t] = o[t];
                else ((bf16_t*)g.y)[e + t] = f32_to_bf16(o[t]);
              }
          }
        }
      }
    }
  }
#endif
}

// ---------------------------------------------------------------------------------------------- host
// Tile / split-K choice: a small cost model in CU clock cycles, evaluated on the host and calibrated on
// measured runs of this kernel (rates in flop per clock per block):
//   - a T x T block runs its K loop at `rate`: 256 -> 2500, 192 -> 2100, 128 -> 1000 with two blocks resident
//     per CU.  The big tiles are bounded by what one CU's vector L1 pulls from L2 (about 19 B/clk) times their
//     flop per byte, the small one additionally by its doubled L2 traffic;
//   - per block: launch/prologue 4000 cycles plus the epilogue, 0.75 cycles per output element for the fused
//     dX epilogue (it streams x, codes, mask and dX through HBM), 0.6 when a second resident block overlaps it,
//     0.3 for the raw fp32 store;
//   - blocks run in rounds of 256 CUs x blocks-per-CU;  split-K adds its fp32 partial tiles, written and read once.
struct TileModel { int t; int bpc; double rate; double epi_dx; };
static const TileModel kTiles[3] = {{256, 1, 2500.0, 0.75}, {192, 1, 2100.0, 0.75}, {128, 2, 1000.0, 0.6}};
// the 192 x 192 kernel with the three-stage ring and the straight-line epilogue (k_gemm_kk, EPI_DXF)
static const TileModel kTileFast192 = {192, 1, 2545.0, 0.45};

GemmPlan gemm_plan(int64_t M, int64_t N, int64_t K, bool allow_split, bool allow_192, bool allow_256, bool fast192) {
  GemmPlan best{};
  double best_t = 1e300;
  const int64_t ksteps = ceil_div(K, KALIGN);
  for (const TileModel& tm0 : kTiles) {
    const TileModel& tm = (tm0.t == 192 && fast192) ? kTileFast192 : tm0;
    if (tm.t == 192 && !allow_192) continue;
    if (tm.t == 256 && !allow_256) continue;
    const int64_t tiles = ceil_div(M, tm.t) * ceil_div(N, tm.t);
    int64_t max_s = allow_split ? ksteps / 8 : 1;
    if (max_s < 1) max_s = 1;
    if (max_s > 32) max_s = 32;
    for (int64_t s = 1; s <= max_s; ++s) {
      const int64_t kslice = ceil_div(ksteps, s) * KALIGN;
      const double per_elem = allow_split ? 0.3 : tm.epi_dx;
      const double block = 2.0 * tm.t * tm.t * (double)kslice / tm.rate + 4000.0 + per_elem * tm.t * tm.t;
      const double rounds = (double)ceil_div(tiles * s, 256 * tm.bpc);
      double t = rounds * block;
      if (allow_split) t += (double)s * (double)M * (double)N * 8.0 / 2400.0;   // partial tiles at ~5 TB/s
      if (t < best_t) {
        best_t = t;
        best.tile = tm.t; best.split_k = (int)s;
        best.tiles_m = (int)ceil_div(M, tm.t); best.tiles_n = (int)ceil_div(N, tm.t);
      }
    }
  }
  return best;
}

bool gemm_epilogue_vec_ok(const GemmEpilogueDx& e, int64_t N) {
  return (N % 8) == 0 && ((uintptr_t)e.x_codes % 8) == 0 && ((uintptr_t)e.x % 16) == 0 && ((uintptr_t)e.dx % 16) == 0;
}

template <int BM, int BN, int EPI, bool I8, bool CONV = false>
static int launch_cfg(const GemmArgs& a, int split_k, hipStream_t st) {
  using C = TileCfg<BM, BN, 2>;
  // set once per process (initialisation of a function-local static is thread-safe)
  static const hipError_t attr = hipFuncSetAttribute((const void*)k_gemm_nt<BM, BN, EPI, I8, CONV>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
  if (attr != hipSuccess) return EFQAT_ERR_HIP;
  dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)split_k);
  constexpr int kProf = (EPI == EPI_DX || EPI == EPI_DXF) ? PROF_DX : (EPI == EPI_RAW ? PROF_DW : PROF_FWD);
  {
    ProfScope prof(kProf, st);
    hipLaunchKernelGGL((k_gemm_nt<BM, BN, EPI, I8, CONV>), grid, dim3(256), C::LDS_BYTES, st, a);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

// nothing left to decide in the dX epilogue: bf16 in and out, whole tiles, 32-bit element offsets, aligned pointers
static bool nt_epilogue_fast(const GemmArgs& g, const GemmEpilogueDx& epi, int tile) {
  return g.epi_vec && epi.x_dtype == EFQAT_BF16 && epi.dx_dtype == EFQAT_BF16 && (g.M % tile) == 0 &&
         (g.N % tile) == 0 && (int64_t)g.M * g.N <= (int64_t)INT32_MAX;
}

int launch_gemm_nt(const bf16_t* A, int64_t lda, const int32_t* a_rows, const bf16_t* B, int64_t ldb, int64_t M,
                   int64_t N, int64_t K, const GemmPlan& plan, float* out_partial, const GemmEpilogueDx* epi,
                   hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (K % 8) || (lda % 8) || (ldb % 8)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return EFQAT_ERR_BAD_SHAPE;
  const int split_k = plan.split_k;
  if (epi && split_k != 1) return EFQAT_ERR_BAD_SHAPE;
  GemmArgs a{};
  a.A = A; a.lda = lda; a.a_rows = a_rows; a.B = B; a.ldb = ldb;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)(ceil_div(ceil_div(K, KALIGN), split_k) * KALIGN);
  a.out = out_partial;
  if (epi) {
    a.x_codes = epi->x_codes; a.x_clip = epi->x_clip; a.x = epi->x; a.x_dtype = epi->x_dtype;
    a.s_x = epi->s_x; a.z_x = epi->z_x; a.dx = epi->dx; a.dx_dtype = epi->dx_dtype; a.partial = epi->partial;
    a.epi_vec = gemm_epilogue_vec_ok(*epi, N) ? 1 : 0;
  }
  a.tiles_m = plan.tiles_m;
  a.tiles_n = plan.tiles_n;
  switch (plan.tile) {
    case 256:
      return epi ? launch_cfg<256, 256, EPI_DX, false>(a, 1, stream)
                 : launch_cfg<256, 256, EPI_RAW, false>(a, split_k, stream);
    case 192:
      return epi ? launch_cfg<192, 192, EPI_DX, false>(a, 1, stream)
                 : launch_cfg<192, 192, EPI_RAW, false>(a, split_k, stream);
    case 128:
      if (epi && nt_epilogue_fast(a, *epi, 128)) return launch_cfg<128, 128, EPI_DXF, false>(a, 1, stream);
      return epi ? launch_cfg<128, 128, EPI_DX, false>(a, 1, stream)
                 : launch_cfg<128, 128, EPI_RAW, false>(a, split_k, stream);
    default:
      return EFQAT_ERR_BAD_SHAPE;
  }
}

int launch_gemm_nt_conv_dx(const bf16_t* dy_tok, int64_t ldc, const bf16_t* wqT, int64_t ldb, int64_t M, int64_t N,
                           int64_t K, const ConvDxMap& cm, const GemmPlan& plan, const GemmEpilogueDx& epi,
                           hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (ldc % 64) || (K % 64) || (ldb % 8) || cm.H > 65535 || cm.W > 65535)
    return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || plan.split_k != 1) return EFQAT_ERR_BAD_SHAPE;
  if (((uintptr_t)cm.zero_page % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  GemmArgs a{};
  a.A = dy_tok; a.lda = ldc; a.a_rows = nullptr; a.B = wqT; a.ldb = ldb;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)(ceil_div(K, KALIGN) * KALIGN);
  a.x_codes = epi.x_codes; a.x_clip = epi.x_clip; a.x = epi.x; a.x_dtype = epi.x_dtype;
  a.s_x = epi.s_x; a.z_x = epi.z_x; a.dx = epi.dx; a.dx_dtype = epi.dx_dtype; a.partial = epi.partial;
  a.epi_vec = gemm_epilogue_vec_ok(epi, N) ? 1 : 0;
  a.tiles_m = plan.tiles_m; a.tiles_n = plan.tiles_n;
  a.cv_H = cm.H; a.cv_W = cm.W; a.cv_Ho = cm.Ho; a.cv_Wo = cm.Wo; a.cv_KW = cm.KW; a.cv_pad = cm.pad;
  a.cv_spt = (int)(ldc / 64); a.cv_zero = cm.zero_page;
  a.cv_m_spt = (1ull << 32) / (uint64_t)a.cv_spt + 1; a.cv_m_kw = (1ull << 32) / (uint64_t)cm.KW + 1;
  switch (plan.tile) {
    case 192: return nt_epilogue_fast(a, epi, 192) ? launch_cfg<192, 192, EPI_DXF, false, true>(a, 1, stream)
                                                   : launch_cfg<192, 192, EPI_DX, false, true>(a, 1, stream);
    case 128:
      // at most one block per compute unit anyway: the three-stage ring hides the load latency a lone block sees
      if ((int64_t)a.tiles_m * a.tiles_n <= 256) return launch_gemm_kk_conv128(a, nt_epilogue_fast(a, epi, 128), stream);
      return nt_epilogue_fast(a, epi, 128) ? launch_cfg<128, 128, EPI_DXF, false, true>(a, 1, stream)
                                           : launch_cfg<128, 128, EPI_DX, false, true>(a, 1, stream);
    default: return EFQAT_ERR_BAD_SHAPE;
  }
}

int launch_gemm_fwd_i8(const uint8_t* x_codes, int64_t lda, const int8_t* w_codes, int64_t ldb, int64_t M, int64_t N,
                       int64_t K, const GemmPlan& plan, const float* s_x, const float* z_x, const float* s_w,
                       const int32_t* wsum, void* y, int y_dtype, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (K % 16) || (lda % 16) || (ldb % 16)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || plan.split_k != 1) return EFQAT_ERR_BAD_SHAPE;
  GemmArgs a{};
  a.A = x_codes; a.lda = lda; a.a_rows = nullptr; a.B = w_codes; a.ldb = ldb;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)(ceil_div(K, 2 * KALIGN) * 2 * KALIGN);
  a.s_x = s_x; a.z_x = z_x; a.s_w = s_w; a.wsum = wsum; a.y = y; a.y_dtype = y_dtype;
  a.epi_vec = ((N % 8) == 0 && ((uintptr_t)y % 16) == 0) ? 1 : 0;
  a.tiles_m = plan.tiles_m;
  a.tiles_n = plan.tiles_n;
  switch (plan.tile) {
    case 256: return launch_cfg<256, 256, EPI_FWD, true>(a, 1, stream);
    case 192: return launch_cfg<192, 192, EPI_FWD, true>(a, 1, stream);
    case 128: return launch_cfg<128, 128, EPI_FWD, true>(a, 1, stream);
    default: return EFQAT_ERR_BAD_SHAPE;
  }
}

}  // namespace efqat
