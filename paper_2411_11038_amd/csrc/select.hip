// Channel importance (Eq. 6) and deterministic Top-K (Sec. 3.2): scores in fp64, exact selection under the
// key (score descending, index ascending) by radix select, output compacted in ascending index order.
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

// Exact Top-K by radix select, one block of NTH threads.  Scores are non-negative doubles, so their bit
// patterns order like the values.  Passes over 8-bit digits of the 64-bit key, from the highest bit on which
// two keys differ downwards, find the key T of the k-th largest score and `need`, the number of scores equal
// to T that still belong to the selection (as soon as at most 64 candidates remain they are ranked directly); then one ordered sweep writes every index whose score is > T, plus the first `need` indices
// (ascending) whose score equals T: ties go to the lower index, output is ascending.  Integer counting only,
// so the result does not depend on thread scheduling.
// Where the keys live between the passes: up to KPT per thread in registers (n <= KPT * NTH); else, with in_lds, in a
// dynamic LDS array of n keys (8 n bytes); else they are re-read from memory in every pass.
template <int NTH, int KPT>
__global__ __launch_bounds__(NTH) void k_topk_radix(const double* __restrict__ scores, int64_t n, int64_t k,
                                                     int32_t* __restrict__ idx, int in_lds) {
  extern __shared__ __attribute__((aligned(16))) unsigned long long lkeys[];
  constexpr int NW = NTH / 64;                        // wavefronts
  __shared__ unsigned int hist[NW][256];              // one histogram per wavefront: less atomic contention
  __shared__ unsigned int total[256];
  __shared__ unsigned long long s_prefix, s_or[NW], s_and[NW];
  __shared__ long long s_need;
  __shared__ int wsum_gt[NW], wsum_eq[NW];
  __shared__ long long s_base_gt, s_base_eq;
  __shared__ unsigned long long cand_key[64];
  __shared__ int cand_idx[64];
  __shared__ int s_bin_count, s_ncand;
  __shared__ int scan_gt[KPT * NW + 64], scan_eq[KPT * NW + 64]; // KPT x wavefronts (cached case), padded to whole lanes
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  // Up to KPT keys per thread stay in registers for all passes (n <= KPT * NTH); longer inputs are re-read.
  constexpr int EPL = (KPT * NW + 63) / 64;           // scan entries per lane of the ordered output
  unsigned long long keys[KPT];
  const bool cached = n <= (int64_t)KPT * NTH;
  // Keys are taken relative to the smallest one (order and equality are unchanged): the scores of a layer lie in a
  // narrow band, and without the offset a band that straddles a power of two would put its highest differing bit
  // in the exponent, so that the first digit window would split the keys into two or three crowded bins.  With it
  // the first window starts at the top bit of (max - min) and spreads the keys over all 256 bins.
  unsigned long long vmin = ~0ull;
  if (cached) {
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      const int64_t i = (int64_t)q * NTH + tid;
      keys[q] = 0ull;
      if (i < n) {
        keys[q] = (unsigned long long)__double_as_longlong(scores[i]);
        vmin = keys[q] < vmin ? keys[q] : vmin;
      }
    }
  } else {
    for (int64_t i = tid; i < n; i += NTH) {
      const unsigned long long key = (unsigned long long)__double_as_longlong(scores[i]);
      if (in_lds) lkeys[i] = key;                      // each thread re-reads only what it wrote until the next barrier
      vmin = key < vmin ? key : vmin;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long t = __shfl_xor(vmin, o, kWave);
    vmin = t < vmin ? t : vmin;
  }
  if (lane == 0) s_and[wv] = vmin;
  __syncthreads();
  vmin = ~0ull;
  for (int i = 0; i < NW; ++i) vmin = s_and[i] < vmin ? s_and[i] : vmin;
  const unsigned long long kmin = vmin;
  // Leading bits on which all (offset) keys agree need no pass: they are the zero bits above the top bit of the OR.
  unsigned long long vor = 0ull;
  if (cached) {
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      const int64_t i = (int64_t)q * NTH + tid;
      if (i < n) { keys[q] -= kmin; vor |= keys[q]; }
    }
  } else if (in_lds) {
    for (int64_t i = tid; i < n; i += NTH) { const unsigned long long key = lkeys[i] - kmin; lkeys[i] = key; vor |= key; }
  } else {
    for (int64_t i = tid; i < n; i += NTH) vor |= (unsigned long long)__double_as_longlong(scores[i]) - kmin;
  }
  // offset key of element i for the passes below (not for the register-resident case)
  auto key_at = [&](int64_t i) -> unsigned long long {
    return in_lds ? lkeys[i] : (unsigned long long)__double_as_longlong(scores[i]) - kmin;
  };
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) vor |= __shfl_xor(vor, o, kWave);
  if (lane == 0) s_or[wv] = vor;
  __syncthreads();
  vor = 0ull;
  for (int i = 0; i < NW; ++i) vor |= s_or[i];
  const unsigned long long diff = vor;                 // the smallest offset key is 0: every set bit differs somewhere
  // The first 8-bit digit window ends at the highest bit on which two keys differ, so the first pass already
  // spreads the keys over the bins; below it the windows follow each other down to bit 0 (the last one may be
  // narrower).  `top` = first bit above the current window; the bits from `top` upwards are the prefix.
  const int hb = diff ? 63 - __clzll((long long)diff) : 7;
  int top = (hb >= 7 ? hb : 7) + 1;
  if (tid == 0) {
    s_prefix = top >= 64 ? 0ull : (vor >> top);         // shared by all keys
    s_need = k;
    s_bin_count = 1 << 30;
  }
  for (int b = tid; b < NW * 256; b += NTH) (&hist[0][0])[b] = 0u;
  __syncthreads();
  while (top > 0) {
    const int width = top < 8 ? top : 8;
    const int shift = top - width;                      // the window is bits [shift, top)
    const unsigned long long dmask = (1ull << width) - 1ull;
    const unsigned long long prefix = s_prefix;
    if (cached) {
#pragma unroll
      for (int q = 0; q < KPT; ++q) {
        const int64_t i = (int64_t)q * NTH + tid;
        const unsigned long long key = keys[q];
        const bool match = (top >= 64) || ((key >> top) == prefix);
        if (i < n && match) atomicAdd(&hist[wv][(key >> shift) & dmask], 1u);
      }
    } else {
      for (int64_t i = tid; i < n; i += NTH) {
        const unsigned long long key = key_at(i);
        const bool match = (top >= 64) || ((key >> top) == prefix);
        if (match) atomicAdd(&hist[wv][(key >> shift) & dmask], 1u);
      }
    }
    __syncthreads();
    if (tid < 256) {                                    // fold the per-wave histograms, clear them for the next pass
      unsigned int t = 0;
      for (int w = 0; w < NW; ++w) { t += hist[w][tid]; hist[w][tid] = 0u; }
      total[tid] = t;
    }
    __syncthreads();
    if (wv == 0) {
      // digit search by the first wavefront: lane l owns bins 4l..4l+3; suffix sums (bins above) by shuffles
      const int need = (int)s_need;                     // counts fit 32 bits: n <= INT32_MAX
      const int h0 = (int)total[4 * lane], h1 = (int)total[4 * lane + 1], h2 = (int)total[4 * lane + 2],
                h3 = (int)total[4 * lane + 3];
      const int tot = h0 + h1 + h2 + h3;
      int inc = tot;                                    // inclusive suffix sum over lanes >= l
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_down(inc, o, kWave);
        if (lane + o < 64) inc += t;
      }
      int a = inc - tot;                                // keys in bins above this lane's four
      if (a < need && need <= a + tot) {                // exactly one lane holds the crossing
        int d;
        if (a + h3 >= need) d = 3;
        else { a += h3; if (a + h2 >= need) d = 2; else { a += h2; if (a + h1 >= need) d = 1; else { a += h1; d = 0; } } }
        s_need = need - a;                              // still to take among keys whose digit equals d
        s_prefix = (prefix << width) | (unsigned long long)(4 * lane + d);
        s_bin_count = d == 3 ? h3 : d == 2 ? h2 : d == 1 ? h1 : h0;
      }
      if (lane == 0) s_ncand = 0;
    }
    __syncthreads();
    // Few keys left under the chosen prefix: finish at once instead of one pass per remaining byte.  The
    // candidates are gathered (in any order) and ranked by one wavefront under (key descending, index ascending).
    top = shift;                                        // the prefix now reaches down to `shift`
    if (top > 0 && s_bin_count <= 64) {
      const unsigned long long np = s_prefix;
      if (cached) {
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
          const int64_t i = (int64_t)q * NTH + tid;
          if (i < n && (keys[q] >> top) == np) {
            const int slot = atomicAdd(&s_ncand, 1);
            cand_key[slot] = keys[q]; cand_idx[slot] = (int)i;
          }
        }
      } else {
        for (int64_t i = tid; i < n; i += NTH) {
          const unsigned long long key = key_at(i);
          if ((key >> top) == np) {
            const int slot = atomicAdd(&s_ncand, 1);
            cand_key[slot] = key; cand_idx[slot] = (int)i;
          }
        }
      }
      __syncthreads();
      if (wv == 0) {
        const int nc = s_ncand;                         // == s_bin_count
        const int need = (int)s_need;                   // 1 .. nc
        const bool on = lane < nc;
        const unsigned long long mk = on ? cand_key[lane] : 0ull;
        const int mi = on ? cand_idx[lane] : 0;
        int rank = 0;
        for (int j = 0; j < nc; ++j) {
          const unsigned long long kj = cand_key[j];
          const int ij = cand_idx[j];
          rank += (kj > mk || (kj == mk && ij < mi)) ? 1 : 0;
        }
        const unsigned long long hit = __ballot(on && rank == need - 1);   // exactly one lane
        const int src = __ffsll((long long)hit) - 1;
        const unsigned int tlo = __shfl((unsigned int)mk, src, kWave), thi = __shfl((unsigned int)(mk >> 32), src, kWave);
        const unsigned long long Tk = ((unsigned long long)thi << 32) | tlo;
        const unsigned long long eqtake = __ballot(on && mk == Tk && rank < need);
        if (lane == 0) { s_prefix = Tk; s_need = __popcll(eqtake); }
      }
      __syncthreads();
      break;
    }
  }
  const unsigned long long T = s_prefix;
  const long long need = s_need;
  if (cached) {
    // Ordered output from the keys still in registers: key q of thread t sits at index NTH q + t.  Every wavefront
    // counts its "greater" and "equal" flags per chunk q, one wavefront turns the KPT x NW counts into exclusive
    // prefixes in index order, then every selected key knows its output position.  Two barriers, no global re-read.
    const unsigned long long below = (1ull << lane) - 1ull;
    // (the flags are formed again in the last loop rather than kept: 2 * KPT wave masks would not fit the registers
    // of a 1024-thread block)
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      const int64_t c = (int64_t)q * NTH + tid;
      const unsigned long long bgq = __ballot(c < n && keys[q] > T);
      const unsigned long long beq = __ballot(c < n && keys[q] == T);
      if (lane == 0) { scan_gt[q * NW + wv] = __popcll(bgq); scan_eq[q * NW + wv] = __popcll(beq); }
    }
    __syncthreads();
    if (wv == 0) {
      // exclusive scan of the KPT * NW counts (EPL consecutive entries per lane; entries beyond the end are zero)
      int g[EPL], e[EPL];
      int gs = 0, es = 0;
#pragma unroll
      for (int u = 0; u < EPL; ++u) {
        const bool in = EPL * lane + u < KPT * NW;
        g[u] = in ? scan_gt[EPL * lane + u] : 0; e[u] = in ? scan_eq[EPL * lane + u] : 0;
        gs += g[u]; es += e[u];
      }
      int gi = gs, ei = es;                             // inclusive prefix over lanes <= l
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int tg = __shfl_up(gi, o, kWave), te = __shfl_up(ei, o, kWave);
        if (lane >= o) { gi += tg; ei += te; }
      }
      int gx = gi - gs, ex = ei - es;
#pragma unroll
      for (int u = 0; u < EPL; ++u) {
        scan_gt[EPL * lane + u] = gx; scan_eq[EPL * lane + u] = ex;
        gx += g[u]; ex += e[u];
      }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      const int64_t c = (int64_t)q * NTH + tid;
      const bool gt = c < n && keys[q] > T, eq = c < n && keys[q] == T;
      const unsigned long long bgq = __ballot(gt), beq = __ballot(eq);
      const long long gt_before = scan_gt[q * NW + wv] + __popcll(bgq & below);
      const long long eq_before = scan_eq[q * NW + wv] + __popcll(beq & below);
      if (gt || (eq && eq_before < need)) {
        const long long pos = gt_before + (eq_before < need ? eq_before : need);
        if (pos < k) idx[pos] = (int32_t)c;
      }
    }
    return;
  }
  if (tid == 0) { s_base_gt = 0; s_base_eq = 0; }
  __syncthreads();
  for (int64_t c0 = 0; c0 < n; c0 += NTH) {
    const int64_t c = c0 + tid;
    unsigned long long key = 0ull;
    if (c < n) key = key_at(c);
    const bool gt = (c < n) && key > T;
    const bool eq = (c < n) && key == T;
    const unsigned long long bg = __ballot(gt), be = __ballot(eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    if (lane == 0) { wsum_gt[wv] = __popcll(bg); wsum_eq[wv] = __popcll(be); }
    __syncthreads();
    long long gt_before = s_base_gt + __popcll(bg & below);
    long long eq_before = s_base_eq + __popcll(be & below);
    for (int i = 0; i < wv; ++i) { gt_before += wsum_gt[i]; eq_before += wsum_eq[i]; }
    const bool take = gt || (eq && eq_before < need);
    if (take) {
      const long long pos = gt_before + (eq_before < need ? eq_before : need);
      if (pos < k) idx[pos] = (int32_t)c;
    }
    __syncthreads();
    if (tid == 0) {
      long long a = 0, e = 0;
      for (int i = 0; i < NW; ++i) { a += wsum_gt[i]; e += wsum_eq[i]; }
      s_base_gt += a; s_base_eq += e;
    }
    __syncthreads();
  }
}

// Short inputs (BERT / ResNet channel counts) fit the registers of four wavefronts, whose barriers are cheaper; the
// number of keys per thread is a template argument so that a short input does not walk through empty slots.  Longer
// inputs (LLM-sized layers) keep their keys in LDS, up to 16384 of them (128 KB); beyond that they are re-read.
constexpr int64_t kTopkLdsKeys = 16384;
void launch_topk(const double* scores, int64_t n, int64_t k, int32_t* idx, hipStream_t st) {
  if (n <= 256) hipLaunchKernelGGL((k_topk_radix<256, 1>), dim3(1), dim3(256), 0, st, scores, n, k, idx, 0);
  else if (n <= 4 * 256) hipLaunchKernelGGL((k_topk_radix<256, 4>), dim3(1), dim3(256), 0, st, scores, n, k, idx, 0);
  else if (n <= 12 * 256) hipLaunchKernelGGL((k_topk_radix<256, 12>), dim3(1), dim3(256), 0, st, scores, n, k, idx, 0);
  else {
    // set once per process (initialisation of a function-local static is thread-safe); a failure leaves the default
    // LDS limit in place and the launch below then reports it
    static const hipError_t attr = hipFuncSetAttribute((const void*)k_topk_radix<1024, 1>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       (int)(kTopkLdsKeys * sizeof(unsigned long long)));
    (void)attr;
    const int in_lds = n <= kTopkLdsKeys ? 1 : 0;
    const size_t lds = in_lds ? (size_t)n * sizeof(unsigned long long) : 0;
    hipLaunchKernelGGL((k_topk_radix<1024, 1>), dim3(1), dim3(1024), lds, st, scores, n, k, idx, in_lds);
  }
}

int launch_topk_profiled(const double* scores, int64_t n, int64_t k, int32_t* idx, hipStream_t st) {
  {
    ProfScope prof(PROF_TOPK, st);
    launch_topk(scores, n, k, idx, st);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

int launch_row_importance(const float* w, int64_t c_out, int64_t block, double* scores, hipStream_t st) {
  const int vec = (((uintptr_t)w % 16) == 0 && block % 4 == 0) ? 1 : 0;
  {
    ProfScope prof(PROF_IMPORTANCE, st);
    hipLaunchKernelGGL(k_row_importance, dim3((unsigned)ceil_div(c_out, 4)), dim3(256), 0, st, w, c_out, block, vec,
                       scores);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

// CWPN helpers: per-layer counts of selected channels, and global -> per-layer local indices.
__global__ void k_layer_counts(const int64_t* __restrict__ layer_off, int64_t n_layers,
                               const int32_t* __restrict__ idx, int64_t k_total,
                               int32_t* __restrict__ k_per_layer) {
  // idx holds ascending global indices: the count of a layer is a difference of two lower bounds
  const int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= n_layers) return;
  auto lower_bound = [&](int64_t v) {
    int64_t lo = 0, hi = k_total;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)idx[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo;
  };
  k_per_layer[l] = (int32_t)(lower_bound(layer_off[l + 1]) - lower_bound(layer_off[l]));
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
  return (size_t)round_up(c_out * (int64_t)sizeof(double), 256);
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
  double* sc_out = scores ? scores : sc;
  const int vec = (((uintptr_t)w % 16) == 0 && block % 4 == 0) ? 1 : 0;
  {
    ProfScope prof(PROF_IMPORTANCE, st);
    hipLaunchKernelGGL(k_row_importance, dim3((unsigned)ceil_div(c_out, 4)), dim3(256), 0, st, w, c_out, block, vec,
                       sc_out);
  }
  EFQAT_LAUNCH_CHECK();
  if (k == 0) return EFQAT_OK;
  {
    ProfScope prof(PROF_TOPK, st);
    launch_topk(sc_out, c_out, k, idx, st);
  }
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

// ------------------------------------------------------------------------------------------------
// efqat_channel_select for callers that cannot allocate device memory: the per-channel scores, which the plain entry
// point keeps in the caller's workspace, live in a file-scope device array of the library instead.
namespace efqat {

constexpr int64_t kStaticSelectMaxChannels = EFQAT_STATIC_SELECT_MAX_CHANNELS;
static __device__ __align__(256) double scratch[kStaticSelectMaxChannels];   // 512 KiB per GPU, for the process' life

// Host code must not pass `scratch` itself to a kernel: here that name is only a handle for the symbol.  The
// array's device address differs per GPU (each holds its own copy) and is looked up once per device, with that
// device current.
constexpr int kMaxDevices = 64;
static double* g_scratch_ptr[kMaxDevices];

static int static_scratch(double** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EFQAT_ERR_HIP;
  if (!g_scratch_ptr[dev]) {
    double* p = nullptr;
    if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return EFQAT_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return EFQAT_OK;
}

}  // namespace efqat

extern "C" int efqat_channel_select_static(const float* w, int64_t c_out, int64_t block, int64_t k, int32_t* idx,
                                           void* stream) {
  if (c_out <= 0 || block <= 0 || c_out > INT64_MAX / block) return EFQAT_ERR_BAD_SHAPE;
  if (c_out > kStaticSelectMaxChannels) return EFQAT_ERR_WORKSPACE;   // more channels than the built-in scratch holds
  if (k < 0 || k > c_out) return EFQAT_ERR_BAD_K;
  if (!w || (k > 0 && !idx)) return EFQAT_ERR_NULL_PTR;
  if (((uintptr_t)w % 4) != 0 || ((uintptr_t)idx % 4) != 0) return EFQAT_ERR_ALIGNMENT;
  double* sc = nullptr;
  const int rc = static_scratch(&sc);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const int vec = (((uintptr_t)w % 16) == 0 && block % 4 == 0) ? 1 : 0;
  // every score that Top-K reads is written by this launch first: nothing in the scratch has to start at zero
  hipLaunchKernelGGL(k_row_importance, dim3((unsigned)ceil_div(c_out, 4)), dim3(256), 0, st, w, c_out, block, vec, sc);
  EFQAT_LAUNCH_CHECK();
  if (k == 0) return EFQAT_OK;
  launch_topk(sc, c_out, k, idx, st);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}

extern "C" size_t efqat_network_select_workspace_bytes(int64_t total) {
  (void)total;
  return 256;   // no scratch needed; kept so callers can treat every entry point alike
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
  // k_per_layer is derived from idx; with k_total == 0 every count is 0 and idx is never read
  if (k_total > 0) {
    launch_topk(scores, total, k_total, idx, st);
    EFQAT_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_layer_counts, dim3((unsigned)ceil_div(n_layers, 256)), dim3(256), 0, st, layer_off, n_layers,
                     idx, k_total, k_per_layer);
  EFQAT_LAUNCH_CHECK();
  if (k_total > 0) {
    hipLaunchKernelGGL(k_localize, dim3((unsigned)ceil_div(k_total, 256)), dim3(256), 0, st, layer_off, n_layers,
                       k_total, idx);
    EFQAT_LAUNCH_CHECK();
  }
  return EFQAT_OK;
}

// ------------------------------------------------------------------------------------------------
// EfQAT-LWPN (Table 2): blocks are whole layers.  Every channel of a layer has the same number of weights, so the
// layer's mean |w| is the mean of its channel means: one block per layer reduces them in double precision in a
// fixed order.
namespace efqat {

__global__ __launch_bounds__(256) void k_layer_means(const double* __restrict__ scores,
                                                     const int64_t* __restrict__ layer_off,
                                                     double* __restrict__ layer_scores) {
  __shared__ double red[256];
  const int64_t b = layer_off[blockIdx.x], e = layer_off[blockIdx.x + 1];
  double s = 0.0;
  for (int64_t i = b + threadIdx.x; i < e; i += 256) s += scores[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) layer_scores[blockIdx.x] = e > b ? red[0] / (double)(e - b) : 0.0;
}

// k_per_layer[l] = channels of layer l if l is among the (ascending) selected layers, else 0
__global__ void k_layer_flags(const int64_t* __restrict__ layer_off, int64_t n_layers,
                              const int32_t* __restrict__ layer_idx, int64_t k_layers,
                              int32_t* __restrict__ k_per_layer) {
  const int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= n_layers) return;
  int64_t lo = 0, hi = k_layers;                      // binary search for l in layer_idx
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (layer_idx[mid] < l) lo = mid + 1; else hi = mid;
  }
  const bool on = lo < k_layers && layer_idx[lo] == l;
  k_per_layer[l] = on ? (int32_t)(layer_off[l + 1] - layer_off[l]) : 0;
}

}  // namespace efqat

using namespace efqat;

extern "C" size_t efqat_layer_select_workspace_bytes(int64_t n_layers) {
  return round_up((size_t)(n_layers > 0 ? n_layers : 1) * sizeof(double), 256);
}

extern "C" int efqat_layer_select(const double* scores, const int64_t* layer_off, int64_t n_layers,
                                  int64_t k_layers, double* layer_scores, int32_t* layer_idx,
                                  int32_t* k_per_layer, void* ws, size_t ws_bytes, void* stream) {
  if (n_layers <= 0 || n_layers > INT32_MAX) return EFQAT_ERR_BAD_SHAPE;
  if (k_layers < 0 || k_layers > n_layers) return EFQAT_ERR_BAD_K;
  if (!scores || !layer_off || !k_per_layer || !ws || (k_layers > 0 && !layer_idx)) return EFQAT_ERR_NULL_PTR;
  if (ws_bytes < efqat_layer_select_workspace_bytes(n_layers)) return EFQAT_ERR_WORKSPACE;
  if (((uintptr_t)ws % 256) != 0) return EFQAT_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  double* ls = layer_scores ? layer_scores : (double*)ws;
  hipLaunchKernelGGL(k_layer_means, dim3((unsigned)n_layers), dim3(256), 0, st, scores, layer_off, ls);
  EFQAT_LAUNCH_CHECK();
  if (k_layers > 0) {
    launch_topk(ls, n_layers, k_layers, layer_idx, st);
    EFQAT_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_layer_flags, dim3((unsigned)ceil_div(n_layers, 256)), dim3(256), 0, st, layer_off, n_layers,
                     layer_idx, k_layers, k_per_layer);
  EFQAT_LAUNCH_CHECK();
  return EFQAT_OK;
}
