// Input-gradient product from two K-contiguous bf16 operands with a hand-pinned instruction order (Eq. 5 left):
//
//   C[m][n] = sum_k A[m][k] * B[n][k],   A = dY bf16 [M][lda],  B = de-quantised W_q^T bf16 [N][ldb]
//
// Same arithmetic as k_gemm_nt; what differs is how the loop is laid out.  Tiles are copied global -> LDS as they
// lie (128-byte rows of 64 K-values, 16-byte chunks XOR-swizzled by the row so that fragment reads are free of bank
// conflicts), fragments are plain 16-byte LDS reads, and every sub-step (one K-slice of 16) is written out as one
// group per MFMA: the MFMA, at most two LDS reads of the next sub-step's fragments, and at most one global -> LDS
// copy of the next stage.  With a single block of four wavefronts per CU there is no second wavefront on a SIMD to
// cover a stall, so the order of these three instruction streams decides the speed; left to the compiler's
// scheduler the reads and copies clump and the matrix cores idle for more than half of the loop.
//
// 256 threads; 192 x 192 tile, wavefront grid 2 x 2 (96 x 96 per wavefront, 9 accumulators);
// v_mfma_f32_32x32x16_bf16; K-stage of 64; a ring of three LDS stages (144 KB): the copies of stage kt + 2 are issued
// while stage kt is multiplied and are only waited for at the end of stage kt + 1, so a copy may take more than a
// whole stage (about 1200 cycles of MFMA work) before it stalls anything - with two stages the memory latency under
// load did not fit.  Rows past M / N re-read the last valid row (their outputs are discarded), chunks past K come
// from a zero page, so no copy needs a predicate.
#include "common.hpp"

#include <type_traits>

#include "gemm_epilogue.hpp"
#include "lds_copy.hpp"

namespace efqat {

template <int T, int WGM_, int WGN_>
struct KkCfg {
  static constexpr int BM = T, BN = T;
  static constexpr int WGM = WGM_, WGN = WGN_;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int A_G = BM / 8 / 4, B_G = BN / 8 / 4;       // 1-KiB copies (8 rows) per wavefront and stage
  static constexpr int LDS_A = BM * 128, LDS_B = BN * 128;
  static constexpr int LDS_STAGE = LDS_A + LDS_B;
  static constexpr int NST = 3;                                  // LDS stages in the ring
  static constexpr int LDS_LOOP = NST * LDS_STAGE;
  static constexpr int LDS_EPI = 4 * 32 * (WN + 8) * 4;
  static constexpr int LDS_BYTES = LDS_LOOP > LDS_EPI ? LDS_LOOP : LDS_EPI;
  static_assert(WGM * WGN == 4 && WM % 32 == 0 && WN % 32 == 0 && BM % 32 == 0, "tile / wavefront grid");
};

struct GemmKkArgs {
  GemmArgs g;              // A, lda, B, ldb, M, N, K, k_per_split, tiles, out or the fused dX epilogue fields
  const void* zero_page;   // >= 256 zero bytes
};

// CONV: the A operand is gathered from a token-major dY with the im2col map of a stride-1 convolution, as in
// k_gemm_nt (see GemmArgs): every copy slot keeps (n, h, w) of its input pixel and forms its source address per stage
// from the stage's tap; K = taps * ldc is a whole number of stages.
template <int T, int WGM, int WGN, int EPI, bool CONV = false>
__global__ __launch_bounds__(256) void k_gemm_kk(const GemmKkArgs ga) {
#if defined(__HIP_DEVICE_COMPILE__)
  using C = KkCfg<T, WGM, WGN>;
  const GemmArgs& g = ga.g;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / C::WGN, wn = wave % C::WGN;

  // consecutive block ids land on different XCDs: give each XCD a contiguous range of tiles, then walk the tiles
  // in groups of GM tile rows so that the blocks running together share operand rows in L2
  const int ntile = gridDim.x;
  const int logical = xcd_contiguous_index(blockIdx.y * ntile + blockIdx.x, ntile * gridDim.y);
  const int split = logical / ntile;                   // split-K slice (0 when there is one)
  const int pid = logical - split * ntile;
  const int GM = 8;
  const int per_group = GM * g.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsize = (g.tiles_m - first_m) < GM ? (g.tiles_m - first_m) : GM;
  const int tm = first_m + (pid % per_group) % gsize;
  const int tn = (pid % per_group) / gsize;
  const int m0 = tm * C::BM, n0 = tn * C::BN;

  const int k_begin = split * g.k_per_split;
  const int k_end_ = (k_begin + g.k_per_split) < g.K ? (k_begin + g.k_per_split) : g.K;
  const int K = k_end_ > k_begin ? k_end_ - k_begin : 0;
  const int nk = (K + 63) / 64;
  const int nfull = K / 64;
  const char* zero = (const char*)ga.zero_page;

  // ---- global -> LDS copies with running pointers.  Slot j of an operand covers tile rows (wave + 4 j) * 8 .. + 7;
  // lane l lands in row l / 8, physical chunk l % 8, and fetches the logical chunk that the swizzle puts there.
  const int c_lrow = lane >> 3;
  const int c_lch = (lane & 7) ^ (((wave * 8 + c_lrow) >> 1) & 7);   // same for every slot: 32 j = 0 (mod 16)
  const char* a_ptr[C::A_G];
  const char* b_ptr[C::B_G];
  int cv_q0[CONV ? C::A_G : 1], cv_hw[CONV ? C::A_G : 1];   // CONV: n * Ho * Wo and (h << 16 | w) of the slot's pixel
#pragma unroll
  for (int j = 0; j < C::A_G; ++j) {
    int gm = m0 + (wave + 4 * j) * 8 + c_lrow;
    gm = gm < g.M ? gm : g.M - 1;
    if constexpr (CONV) {
      const int hw = g.cv_H * g.cv_W;
      const int n = gm / hw, rem = gm - n * hw;
      const int h = rem / g.cv_W, w = rem - h * g.cv_W;
      cv_q0[j] = n * g.cv_Ho * g.cv_Wo;
      cv_hw[j] = (h << 16) | w;
      a_ptr[j] = nullptr;
    } else {
      a_ptr[j] = (const char*)g.A + ((int64_t)gm * g.lda + k_begin) * 2 + c_lch * 16;
    }
  }
  // CONV: source of this lane's 16 bytes of A slot j in stage kt (the zero page when the tap falls outside the image)
  auto a_src_conv = [&](int j, int kt) -> const char* {
    const int sidx = k_begin / 64 + kt;                // 64-channel stage index along K = (tap, channel)
    const int tap = (int)(((uint64_t)(uint32_t)sidx * g.cv_m_spt) >> 32), cst = sidx - tap * g.cv_spt;
    const int kh = (int)(((uint64_t)(uint32_t)tap * g.cv_m_kw) >> 32), kw = tap - kh * g.cv_KW;
    const int ho = (cv_hw[j] >> 16) + g.cv_pad - kh, wo = (cv_hw[j] & 0xFFFF) + g.cv_pad - kw;
    const bool ok = (unsigned)ho < (unsigned)g.cv_Ho && (unsigned)wo < (unsigned)g.cv_Wo;
    const int64_t pix = (int64_t)cv_q0[j] + ho * g.cv_Wo + wo;
    return ok ? (const char*)g.A + (pix * g.lda + cst * 64) * 2 + c_lch * 16 : zero;
  };
#pragma unroll
  for (int j = 0; j < C::B_G; ++j) {
    int gn = n0 + (wave + 4 * j) * 8 + c_lrow;
    gn = gn < g.N ? gn : g.N - 1;
    b_ptr[j] = (const char*)g.B + ((int64_t)gn * g.ldb + k_begin) * 2 + c_lch * 16;
  }
  constexpr int LPS = C::A_G + C::B_G;
  using Checked = std::integral_constant<bool, true>;
  using Unchecked = std::integral_constant<bool, false>;
  auto issue_range = [&](auto checked, int kt, int buf, int t0, int t1) {
    char* sa = smem + buf * C::LDS_STAGE;
    char* sb = sa + C::LDS_A;
    const bool off = decltype(checked)::value && (kt * 64 + c_lch * 8 >= K);   // K % 8 == 0: a chunk is all in or out
#pragma unroll
    for (int t = t0; t < t1; ++t) {
      if (t < C::A_G) {
        if constexpr (CONV) {
          dma16(a_src_conv(t, kt), sa + (wave + 4 * t) * 1024);
        } else {
          dma16(off ? zero : a_ptr[t], sa + (wave + 4 * t) * 1024);
          a_ptr[t] += 128;
        }
      } else {
        const int u = t - C::A_G;
        dma16(off ? zero : b_ptr[u], sb + (wave + 4 * u) * 1024);
        b_ptr[u] += 128;
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

  // ---- fragment reads: lane owns row 32 i + lane % 32 of its wavefront's rows, K-values 16 sub + 8 (lane / 32) + 0..7,
  // i.e. logical chunk 2 sub + lane / 32.  Rows 32 i + r share their swizzle term, so one address per (buffer, sub)
  // and operand serves every fragment through the instruction's immediate offset.
  const int fr = lane & 31, fh = lane >> 5;
  int a_addr[C::NST][4], b_addr[C::NST][4];
#pragma unroll
  for (int sub = 0; sub < 4; ++sub) {
    const int ch = ((2 * sub + fh) ^ ((fr >> 1) & 7)) << 4;
    a_addr[0][sub] = (wm * C::WM + fr) * 128 + ch;
    b_addr[0][sub] = C::LDS_A + (wn * C::WN + fr) * 128 + ch;
#pragma unroll
    for (int b = 1; b < C::NST; ++b) {
      a_addr[b][sub] = a_addr[0][sub] + b * C::LDS_STAGE;
      b_addr[b][sub] = b_addr[0][sub] + b * C::LDS_STAGE;
    }
  }
  static_assert((C::WM % 16) == 0 && (C::WN % 16) == 0, "the swizzle term must not depend on the wavefront's origin");
  typedef int intx4_t __attribute__((ext_vector_type(4)));
  intx4_t af[2][C::TM], bf[2][C::TN];
  // LDS read number r of a sub-step, in the order the MFMAs first need them: A0, all of B, then the other A
  constexpr int NRD = C::TM + C::TN;
  auto lds_read = [&](auto bufc, int sub, int rb, int r) {
    constexpr int buf = decltype(bufc)::value;
    if (r == 0) {
      af[rb][0] = *reinterpret_cast<const intx4_t*>(smem + a_addr[buf][sub]);
    } else if (r <= C::TN) {
      bf[rb][r - 1] = *reinterpret_cast<const intx4_t*>(smem + b_addr[buf][sub] + (r - 1) * 4096);
    } else {
      af[rb][r - C::TN] = *reinterpret_cast<const intx4_t*>(smem + a_addr[buf][sub] + (r - C::TN) * 4096);
    }
  };
  auto load_frags = [&](auto bufc, int sub, int rb) {
#pragma unroll
    for (int r = 0; r < NRD; ++r) lds_read(bufc, sub, rb, r);
  };
  auto mfma_one = [&](int rb, int i, int j) {
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[rb][i]),
                                                        __builtin_bit_cast(bf16x8_t, bf[rb][j]), acc[i][j], 0, 0, 0);
  };
  auto mfma_all = [&](int rb) {
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int j = 0; j < C::TN; ++j) mfma_one(rb, i, j);
  };

  // copies of one stage, by the sub-step that issues them: the first P0 go out one stage early (last sub-step of the
  // stage before, right after the barrier that frees their buffer), the rest in sub-steps 0, 1, 2
  constexpr int P0 = LPS / 4, P1 = (LPS - P0 + 2) / 3, P2 = (LPS - P0 - P1 + 1) / 2, P3 = LPS - P0 - P1 - P2;
  // end of a stage: the copies of the next stage have landed (the LPS copies issued after them, which belong to
  // the stage after next, may still be in flight), every wavefront is done reading this stage's buffer
  // `tail`: one of the last two stages - every copy landed before it began and none is issued any more
  auto stage_sync = [&](auto steadyc, bool tail) {
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(steadyc)::value) {
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(LPS) : "memory");   // the LPS copies issued since stay in flight
    } else if (tail) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  // One steady-state sub-step, one group per MFMA: the MFMAs of fragment set rb; spread over the first RG groups
  // the LDS reads of the next sub-step (into set rb ^ 1); the first t1 - t0 groups also issue one global -> LDS copy
  // each (stage kt_i into buffer buf_i).
  constexpr int MF = C::TM * C::TN;
  constexpr int RG = (2 * MF + 2) / 3;
  static_assert(P0 <= MF && P1 <= MF && P2 <= MF && P3 <= MF, "copies per sub-step must not exceed its MFMAs");
  auto substep = [&](auto bufn, int sub_next, int rb, int kt_i, int buf_i, int t0, int t1) {
#pragma unroll
    for (int qq = 0; qq < MF; ++qq) {
      mfma_one(rb, qq / C::TN, qq % C::TN);
      if (qq < RG) {
#pragma unroll
        for (int r = (qq * NRD) / RG; r < ((qq + 1) * NRD) / RG; ++r) lds_read(bufn, sub_next, rb ^ 1, r);
      }
      if (qq < t1 - t0) issue_range(Unchecked{}, kt_i, buf_i, t0 + qq, t0 + qq + 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  EpiDxFast<C> epi;                                   // used by EPI_DXF only
  const int kt_epi = nk >= 2 ? nk - 2 : 0;            // the first of the last two stages

  // ---- main loop.  Stage kt lives in buffer kt % 3.  On entry to stage kt the first P0 copies of stage kt + 2 have
  // been issued if and only if that stage is a full one (kt + 2 < nfull); both variants keep this true for kt + 1.
  auto stage = [&](auto bufc, auto steadyc, int kt) {
    constexpr int cur = decltype(bufc)::value;
    constexpr bool ST = decltype(steadyc)::value;
    constexpr int nxt = (cur + 1) % C::NST, nn = (cur + 2) % C::NST;
    using Next = std::integral_constant<int, nxt>;
    if constexpr (ST) {              // kt + 3 < nfull
      __builtin_amdgcn_sched_barrier(0);
      substep(bufc, 1, 0, kt + 2, nn, P0, P0 + P1);
      substep(bufc, 2, 1, kt + 2, nn, P0 + P1, P0 + P1 + P2);
      substep(bufc, 3, 0, kt + 2, nn, P0 + P1 + P2, LPS);
      stage_sync(steadyc, false);
      substep(Next{}, 0, 1, kt + 3, cur, 0, P0);
    } else {
      const bool more1 = kt + 1 < nk;
      // the last two stages: the preceding barrier was passed with every copy landed (all drain stages before
      // them wait for vmcnt(0)), and nothing more is issued - the moment to request the epilogue's first inputs
      const bool tail = kt + 2 >= nk;
      if (kt + 2 < nfull) issue_range(Unchecked{}, kt + 2, nn, P0, LPS);
      else if (kt + 2 < nk) issue_range(Checked{}, kt + 2, nn, 0, LPS);
      if constexpr (EPI == EPI_DXF) {
        if (kt == kt_epi) epi.prefetch(g, m0, n0, wm, wn);
      }
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 1, 1);
      mfma_all(0);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 2, 0);
      mfma_all(1);
      __builtin_amdgcn_sched_barrier(0);
      load_frags(bufc, 3, 1);
      mfma_all(0);
      stage_sync(steadyc, tail);
      if (more1) load_frags(Next{}, 0, 0);
      if (kt + 3 < nfull) issue_range(Unchecked{}, kt + 3, cur, 0, P0);
      mfma_all(1);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  using B2 = std::integral_constant<int, 2>;
  using Steady = std::integral_constant<bool, true>;
  using Drain = std::integral_constant<bool, false>;

  if (nk > 0) issue_range(Checked{}, 0, 0, 0, LPS);
  if (nk > 1) issue_range(Checked{}, 1, 1, 0, LPS);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (2 < nfull) issue_range(Unchecked{}, 2, 2, 0, P0);
  if (nk > 0) load_frags(B0{}, 0, 0);
  int kt = 0;
  for (; kt + 5 < nfull; kt += 3) {
    stage(B0{}, Steady{}, kt);
    stage(B1{}, Steady{}, kt + 1);
    stage(B2{}, Steady{}, kt + 2);
  }
  for (; kt < nk; kt += 3) {
    stage(B0{}, Drain{}, kt);
    if (kt + 1 < nk) stage(B1{}, Drain{}, kt + 1);
    if (kt + 2 < nk) stage(B2{}, Drain{}, kt + 2);
  }
  __syncthreads();

  if constexpr (EPI == EPI_DX) {
    epilogue_dx<C>(g, acc, smem, m0, n0, wm, wn);
  } else if constexpr (EPI == EPI_DXF) {
    epi.run(g, acc, smem, blockIdx.x);
  } else {
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
  }
#endif
}

template <int T, int WGM, int WGN, int EPI, bool CONV = false>
static int launch_kk_cfg(const GemmKkArgs& a, int split_k, hipStream_t st) {
  using C = KkCfg<T, WGM, WGN>;
  // set once per process (initialisation of a function-local static is thread-safe)
  static const hipError_t attr = hipFuncSetAttribute((const void*)k_gemm_kk<T, WGM, WGN, EPI, CONV>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
  if (attr != hipSuccess) return EFQAT_ERR_HIP;
  dim3 grid((unsigned)(a.g.tiles_m * a.g.tiles_n), (unsigned)split_k);
  {
    ProfScope prof(EPI == EPI_RAW ? PROF_DW : PROF_DX, st);
    hipLaunchKernelGGL((k_gemm_kk<T, WGM, WGN, EPI, CONV>), grid, dim3(256), C::LDS_BYTES, st, a);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

int launch_gemm_kk(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, const void* zero_page, int64_t M,
                   int64_t N, int64_t K, const GemmPlan& plan, float* out_partial, const GemmEpilogueDx* epi,
                   hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || (K % 8) || (lda % 8) || (ldb % 8)) return EFQAT_ERR_BAD_SHAPE;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return EFQAT_ERR_BAD_SHAPE;
  if (!zero_page) return EFQAT_ERR_NULL_PTR;
  if (((uintptr_t)A % 16) || ((uintptr_t)B % 16) || ((uintptr_t)zero_page % 16)) return EFQAT_ERR_ALIGNMENT;
  const int split_k = plan.split_k;
  if (epi && split_k != 1) return EFQAT_ERR_BAD_SHAPE;
  GemmKkArgs ka{};
  GemmArgs& a = ka.g;
  ka.zero_page = zero_page;
  a.A = A; a.lda = lda; a.a_rows = nullptr; a.B = B; a.ldb = ldb;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)(ceil_div(ceil_div(K, 64), split_k) * 64);   // slices start on whole K-stages
  a.out = out_partial;
  if (epi) {
    a.x_codes = epi->x_codes; a.x_clip = epi->x_clip; a.x = epi->x; a.x_dtype = epi->x_dtype;
    a.s_x = epi->s_x; a.z_x = epi->z_x; a.dx = epi->dx; a.dx_dtype = epi->dx_dtype; a.partial = epi->partial;
    a.epi_vec = gemm_epilogue_vec_ok(*epi, N) ? 1 : 0;
  }
  a.tiles_m = plan.tiles_m;
  a.tiles_n = plan.tiles_n;
  switch (plan.tile) {
    case 192: {
      if (!epi) return launch_kk_cfg<192, 2, 2, EPI_RAW>(ka, split_k, stream);
      // nothing to decide at run time: the straight-line epilogue
      const bool fast = a.epi_vec && epi->x_dtype == EFQAT_BF16 && epi->dx_dtype == EFQAT_BF16 && (M % 192) == 0 &&
                        (N % 192) == 0 && M * N <= (int64_t)INT32_MAX;
      return fast ? launch_kk_cfg<192, 2, 2, EPI_DXF>(ka, 1, stream) : launch_kk_cfg<192, 2, 2, EPI_DX>(ka, 1, stream);
    }
    case 128: {
      if (!epi) return launch_kk_cfg<128, 2, 2, EPI_RAW>(ka, split_k, stream);
      const bool fast = a.epi_vec && epi->x_dtype == EFQAT_BF16 && epi->dx_dtype == EFQAT_BF16 && (M % 128) == 0 &&
                        (N % 128) == 0 && M * N <= (int64_t)INT32_MAX;
      return fast ? launch_kk_cfg<128, 2, 2, EPI_DXF>(ka, 1, stream) : launch_kk_cfg<128, 2, 2, EPI_DX>(ka, 1, stream);
    }
    default:
      return EFQAT_ERR_BAD_SHAPE;
  }
}

// dX product of a stride-1 convolution on 128 x 128 tiles with the three-stage ring; `a` as launch_gemm_nt_conv_dx
// fills it (K a whole number of 64-channel stages, no split-K).
int launch_gemm_kk_conv128(const GemmArgs& a, bool fast, hipStream_t stream) {
  if ((a.K % 64) != 0 || !a.cv_zero || ((uintptr_t)a.cv_zero % 16) != 0) return EFQAT_ERR_BAD_SHAPE;
  GemmKkArgs ka{};
  ka.g = a;
  ka.g.k_per_split = a.K;
  ka.zero_page = a.cv_zero;
  return fast ? launch_kk_cfg<128, 2, 2, EPI_DXF, true>(ka, 1, stream) : launch_kk_cfg<128, 2, 2, EPI_DX, true>(ka, 1, stream);
}

}  // namespace efqat
