// Latent-space neighbourhoods B_k(x) of every code of a VQ codebook (paper
// Sec. 2.2: the k nearest neighbours of a token in latent space; reused by Sec. 4).
//
// The result is defined by the float64 inner product (products added in index
// order) with ties to the lower index, so it does not depend on how the matrix
// cores round.  Three kernels:
//   pack    zero-padded copy of the codebook (rows of DP floats, DP = 16..256 a power of two >= D), row
//           norms and their maximum (for the rounding bound below).
//   select  the dense V x V contraction on the matrix cores, swept twice per block of
//           query codes and never written out: sweep 1 histograms each row's
//           similarities into 1024 bins and finds the bin b* holding the (k-1)-th
//           largest; sweep 2 appends every code whose bin is >= b* - 1 - m to the
//           row's candidate list.  Rows of up to 16 floats: fp32 MFMA 16x16x4, 16
//           queries per block, m = 0.  Longer rows: the sweeps are bound by streaming
//           the codebook out of the last-level cache once per block and sweep, so they
//           run on a bf16 copy of it (half the bytes, MFMA 16x16x32) with 32 queries
//           per block (half the blocks), and m bins of margin make up for the rounding
//           of the copy (see row_eps).
//   rank    per row: exact float64 keys of the candidates (FMA chain in index
//           order), rank by (key desc, index asc) with value buckets in LDS, write the row.
// Why the candidate list is enough: a code that is not a candidate has an
// approximate similarity below the lower edge e of the lowest bin taken, hence an exact
// key below e + eps, eps bounding the rounding of the approximate similarity.  If the (k-1)-th exact key
// among the candidates is >= e + eps, no outsider can belong to the row.  Rows
// that fail this test, or overflow the candidate list, take an exact (slow)
// radix-select path over all V codes instead.
#include <limits.h>
#include <math.h>

#include <type_traits>

#include <atomic>

#include "lpp_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kBins = 1024;                   // the bf16 sweeps: two 16-bit counts per LDS word,
constexpr float kBinScale = 512.0f;           // bin = floor((s + 1) * 512), clamped
constexpr int kBinsF = 512;                   // the fp32 sweeps (rows of up to 16 floats, similarities spread
constexpr float kBinScaleF = 256.0f;          // widely): 32-bit counts, bin = floor((s + 1) * 256), clamped
constexpr int kSelWaves = 4;
constexpr int kSelRows = 16;                  // query codes per select block
constexpr int kSel2Waves = 8;                 // the bf16 sweeps: 8 waves and
constexpr int kSel2Rows = 32;                 // 32 query codes per block
constexpr int kRankThreads = 256;
constexpr int kSlack = 1024;                  // candidate list = k - 1 + slack (rounded); rows of up to 16
constexpr int kSlackShort = 512;              // floats spread their similarities widely: half of it

struct KnnArgs {
  const float* E;
  int32_t V, D, DP, Vp, k, cap;
  float* Ep;            // [Vp][DP]
  uint16_t* Eh;         // [Vp][DP] bf16 (round to nearest even) of Ep, or null: the sweeps run in fp32
  float bin_scale;      // bins per unit of similarity in the sweeps' histograms
  float* norms;         // [Vp]
  uint32_t* maxnorm;    // float bits
  int32_t* bstar;       // [Vp] lowest bin whose codes became candidates
  int32_t* cnt;         // [Vp]
  uint16_t* cand;       // [V][cap]
  int32_t* neigh;       // [V][k]
};

__global__ void knn_init_kernel(KnnArgs a) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *a.maxnorm = 0u;
}

// A wave per row, 16 rows per wave: padded copy, norm; one atomic per block for the max norm.
constexpr int kPackRows = 64;   // rows per block of 4 waves
__global__ __launch_bounds__(256) void knn_pack_kernel(KnnArgs a) {
  __shared__ float s_max[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float mx = 0.f;
  for (int i = 0; i < kPackRows / 4; ++i) {
    const int row = blockIdx.x * kPackRows + 4 * i + wave;
    if (row >= a.Vp) break;
    float ss = 0.f;
    for (int d = lane; d < a.DP; d += 64) {
      float v = 0.f;
      if (row < a.V && d < a.D) v = a.E[(int64_t)row * a.D + d];
      a.Ep[(int64_t)row * a.DP + d] = v;
      if (a.Eh) {
        const uint32_t u = __float_as_uint(v);
        // round to nearest even on the upper 16 bits; NaN stays NaN (quiet bit set)
        const uint32_t h = (u & 0x7FFFFFFFu) > 0x7F800000u ? ((u >> 16) | 0x40u) : ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
        a.Eh[(int64_t)row * a.DP + d] = (uint16_t)h;
      }
      ss += v * v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float n = sqrtf(ss);
    if (lane == 0) a.norms[row] = n;
    if (row < a.V) mx = fmaxf(mx, n);
  }
  if (lane == 0) s_max[wave] = mx;
  __syncthreads();
  if (threadIdx.x == 0)
    atomicMax(a.maxnorm, __float_as_uint(fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]))));
}

// Bound on |approximate - exact| similarity of row i with any code.  fp32 sweeps: the matrix
// core's additions, (DP + 4) roundings of 2^-23 on sums of at most |e_i| |e_j|.  bf16 sweeps: each
// operand carries a relative rounding of 2^-9, so each product one of 2^-8 + 2^-18 (the products
// themselves are exact in fp32), summed: (2^-8 + 2^-18) sum |e_i,t e_j,t| <= that times |e_i| |e_j|;
// plus the additions as before.  2.5e-7 covers the rounding of the bin map.
__device__ __forceinline__ float row_eps(const KnnArgs& a, int i) {
  const float add = (float)(a.DP + 4) * 1.1920929e-07f;
  const float rel = a.Eh ? 0.00390625f * 1.01f + add : add;
  return rel * a.norms[i] * __uint_as_float(*a.maxnorm) * 1.001f + 2.5e-7f;
}
// Bins of margin below b* - 1 that the candidates of row i take in.  The (k-1)-th largest
// approximate similarity lies in bin b*, so the (k-1)-th exact key of the candidates is at least
// b*'s lower edge less eps; the rank kernel's test wants it eps above the lower edge of the lowest
// bin taken, b* - 1 - m: (1 + m) bins >= 2 eps.  (Huge for rows whose eps is: everything is taken.)
__device__ __forceinline__ int row_margin(const KnnArgs& a, int i) {
  if (!a.Eh) return 0;
  const float m = ceilf(2.0f * row_eps(a, i) * a.bin_scale - 1.0f);
  return m < (float)kBins ? (m > 0.f ? (int)m : 0) : kBins;      // (NaN norms: kBins)
}

// b* of one row's histogram (two 16-bit counts per word): the highest bin whose count from the top
// reaches kk, 0 if none does.  One wave; every lane returns it.
__device__ __forceinline__ int find_bstar(const uint32_t* h, int kk, int lane) {
  // lane covers bins [1023 - 16*lane - 15, 1023 - 16*lane], scanned downwards
  int cntv[16];
  int local = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t w = h[(kBins / 2 - 1) - 8 * lane - j];   // bins (hi, lo) = (odd, even)
    cntv[2 * j] = (int)(w >> 16);
    cntv[2 * j + 1] = (int)(w & 0xFFFFu);
    local += cntv[2 * j] + cntv[2 * j + 1];
  }
  int incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  const unsigned long long bal = __ballot(incl >= kk);
  int bs = 0;
  if (bal) {
    const int fl = __ffsll((long long)bal) - 1;
    int run = __shfl(incl - local, fl);
    int found = 0;
    if (lane == fl) {
      found = kBins - 1 - 16 * lane - 15;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        run += cntv[j];
        if (run >= kk) { found = kBins - 1 - 16 * lane - j; break; }
      }
    }
    bs = __shfl(found, fl);
  }
  return bs;
}

// b* of one row's histogram of kBinsF 32-bit counts, as find_bstar.
__device__ __forceinline__ int find_bstar32(const uint32_t* h, int kk, int lane) {
  // lane covers bins [511 - 8*lane - 7, 511 - 8*lane], scanned downwards
  int cntv[8];
  int local = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    cntv[j] = (int)h[(kBinsF - 1) - 8 * lane - j];
    local += cntv[j];
  }
  int incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  const unsigned long long bal = __ballot(incl >= kk);
  int bs = 0;
  if (bal) {
    const int fl = __ffsll((long long)bal) - 1;
    int run = __shfl(incl - local, fl);
    int found = 0;
    if (lane == fl) {
      found = kBinsF - 1 - 8 * lane - 7;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        run += cntv[j];
        if (run >= kk) { found = kBinsF - 1 - 8 * lane - j; break; }
      }
    }
    bs = __shfl(found, fl);
  }
  return bs;
}

// The sweeps in fp32, for rows of up to 16 floats (DP = 16: one float4 per lane and code).
// Contraction slot (step, g) of the 16x16x4 MFMA is dimension 4*g + step on both operands.
// A block owns 16 query codes; its 4 waves take the code tiles (16 codes each) in turn and share
// the rows' histograms in LDS, so that a compute unit holds many waves and the latency of the
// tile loads (served by L2: the codebook is small) is covered.  U tiles are in flight per wave.
// The sweeps are bound by the instructions issued per similarity: tiles that hold neither the
// queries' own codes nor padding (all but two) take a path with no test and no branch per
// similarity, and a similarity costs a multiply-add, a convert, a clamp, an address and the LDS add.
__global__ __launch_bounds__(kSelWaves * 64) void knn_select_f32_kernel(KnnArgs a) {
  constexpr int U = 4;
  extern __shared__ uint32_t s_hist[];          // [kSelRows][kBinsF]
  __shared__ int s_cnt[kSelRows];
  __shared__ int s_low[kSelRows];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (tile numbers stay scalar)
  const int l16 = lane & 15, g4 = lane >> 4;
  const int row0 = blockIdx.x * kSelRows;               // the block's 16 query codes
  const int qrow = row0 + l16;                          // the lane's query code (B operand column)
  const int V = a.V;
  const int kk = a.k - 1;                               // neighbours besides the code itself
  const int ntiles = a.Vp / 16;
  const int own_tile = row0 / 16, full_tiles = (row0 + kSelRows <= V) ? V / 16 : 0;   // plain: t != own_tile && t < full_tiles

  const f32x4 qv = *reinterpret_cast<const f32x4*>(a.Ep + (int64_t)qrow * 16 + 4 * g4);

  for (int i = threadIdx.x; i < kSelRows * kBinsF; i += kSelWaves * 64) s_hist[i] = 0u;
  if (threadIdx.x < kSelRows) s_cnt[threadIdx.x] = 0;
  __syncthreads();

  // second sweep: candidates are the codes with x >= thr (bin >= the lowest bin taken; -inf takes
  // everything that is a number).  x = (s + 1) * 256 is the bin before truncation and the map is
  // monotone, so the second sweep compares floats.
  float thr = -INFINITY;
  const float* lane_row = a.Ep + (int64_t)l16 * 16 + 4 * g4;
  uint32_t* my_hist = s_hist + l16 * kBinsF;
  auto sweep = [&](auto phase_tag) {
    constexpr int PHASE = decltype(phase_tag)::value;
    for (int t0 = wave; t0 < ntiles; t0 += kSelWaves * U) {
      f32x4 av[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int t = min(t0 + kSelWaves * u, ntiles - 1);      // (past the end: a re-read that is not used)
        av[u] = *reinterpret_cast<const f32x4*>(lane_row + (int64_t)t * 256);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][0], qv[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][1], qv[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][2], qv[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][3], qv[3], acc, 0, 0, 0);
        const int t = t0 + kSelWaves * u;
        if (t >= ntiles) continue;
        // lane holds sim(code 16 t + 4*g4 + r, query qrow), r = 0..3
        float x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = __builtin_fmaf(acc[r], kBinScaleF, kBinScaleF);
        const bool plain = t != own_tile && t < full_tiles;    // uniform
        if (PHASE == 0) {
          if (plain) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              atomicAdd(&my_hist[min(max((int)x[r], 0), kBinsF - 1)], 1u);     // (int) truncates and sends NaN to 0
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int code = t * 16 + 4 * g4 + r;
              if (!(code >= V || code == qrow || qrow >= V)) atomicAdd(&my_hist[min(max((int)x[r], 0), kBinsF - 1)], 1u);
            }
          }
        } else {
          bool pass[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) pass[r] = x[r] >= thr;
          if (!plain) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int code = t * 16 + 4 * g4 + r;
              pass[r] = pass[r] && !(code >= V || code == qrow || qrow >= V);
            }
          }
          if (__ballot(pass[0] || pass[1] || pass[2] || pass[3])) {   // about one code in sixteen passes
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (pass[r]) {
                const int pos = atomicAdd(&s_cnt[l16], 1);
                if (pos < a.cap) a.cand[(int64_t)qrow * a.cap + pos] = (uint16_t)(t * 16 + 4 * g4 + r);
              }
          }
        }
      }
    }
  };
  sweep(std::integral_constant<int, 0>());
  __syncthreads();
  // lowest bin taken, per row: b* - 1, b* the highest bin whose count from the top reaches kk; a wave takes 4 rows
  for (int r = wave * (kSelRows / kSelWaves); r < (wave + 1) * (kSelRows / kSelWaves); ++r) {
    const int bs = find_bstar32(s_hist + r * kBinsF, kk, lane);
    if (lane == 0) {
      s_low[r] = bs - 1;
      if (row0 + r < a.Vp) a.bstar[row0 + r] = bs - 1;
    }
  }
  __syncthreads();
  thr = s_low[l16] <= 0 ? -INFINITY : (float)s_low[l16];      // (bin 0 also holds what is below -1)
  sweep(std::integral_constant<int, 1>());
  __syncthreads();
  if (threadIdx.x < kSelRows && row0 + threadIdx.x < a.Vp) a.cnt[row0 + threadIdx.x] = s_cnt[threadIdx.x];
}

// The sweeps on the bf16 copy of the codebook.  KS = contraction steps of 32 (DP = 32 * KS).
// A block owns 32 query codes -- two B operands per wave, so a code tile that was loaded feeds two
// MFMA chains -- and its 8 waves take the code tiles (16 codes each) in turn; U tiles are in flight
// per wave.  Slot (g, e) of a step is dimension 32*step + 8*g + e on both operands.
template <int KS>
__global__ __launch_bounds__(kSel2Waves * 64) void knn_select_bf16_kernel(KnnArgs a) {
  constexpr int U = KS >= 8 ? 2 : 4;
  extern __shared__ uint32_t s_hist[];          // [kSel2Rows][kBins/2], two 16-bit counts per word
  __shared__ int s_cnt[kSel2Rows];
  __shared__ int s_low[kSel2Rows];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (tile numbers stay scalar)
  const int l16 = lane & 15, g4 = lane >> 4;
  const int row0 = blockIdx.x * kSel2Rows;              // the block's 32 query codes (Vp is a multiple of 64)
  const int DP = a.DP, V = a.V;
  const int kk = a.k - 1;
  const int ntiles = a.Vp / 16;

  bf16x8 qv[2][KS];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qv[qt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
          a.Eh + (int64_t)(row0 + 16 * qt + l16) * DP + 32 * ks + 8 * g4));

  for (int i = threadIdx.x; i < kSel2Rows * (kBins / 2); i += kSel2Waves * 64) s_hist[i] = 0u;
  if (threadIdx.x < kSel2Rows) s_cnt[threadIdx.x] = 0;
  __syncthreads();

  float thr[2] = {-INFINITY, -INFINITY};   // second sweep: x >= thr; -inf takes everything that is a number
  const uint16_t* lane_row = a.Eh + (int64_t)l16 * DP + 8 * g4;
  auto sweep = [&](auto phase_tag) {
    constexpr int PHASE = decltype(phase_tag)::value;
    for (int t0 = wave; t0 < ntiles; t0 += kSel2Waves * U) {
      bf16x8 av[U][KS];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int t = min(t0 + kSel2Waves * u, ntiles - 1);     // (past the end: a re-read that is not used)
        const uint16_t* arow = lane_row + (int64_t)t * (16 * DP);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          av[u][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(arow + 32 * ks));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u][ks], qv[0][ks], acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u][ks], qv[1][ks], acc[1], 0, 0, 0);
        }
        const int t = t0 + kSel2Waves * u;
        if (t >= ntiles) continue;
        // tiles without the queries' own codes and without padding take no check per similarity
        const bool plain = (t >> 1) != row0 / 32 && t * 16 + 16 <= V && row0 + kSel2Rows <= V;    // uniform
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
          // lane holds sim(code 16 t + 4*g4 + r, query row0 + 16 qt + l16), r = 0..3
          const int qrow = row0 + 16 * qt + l16;
          float x[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) x[r] = __builtin_fmaf(acc[qt][r], kBinScale, kBinScale);
          if (PHASE == 0) {
            uint32_t* my_hist = s_hist + (16 * qt + l16) * (kBins / 2);
            if (plain) {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int bin = min(max((int)x[r], 0), kBins - 1);      // (int) truncates and sends NaN to 0
                atomicAdd(&my_hist[bin >> 1], 1u << ((bin & 1) << 4));
              }
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int code = t * 16 + 4 * g4 + r;
                const int bin = min(max((int)x[r], 0), kBins - 1);
                if (!(code >= V || code == qrow || qrow >= V)) atomicAdd(&my_hist[bin >> 1], 1u << ((bin & 1) << 4));
              }
            }
          } else {
            bool pass[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) pass[r] = x[r] >= thr[qt];
            if (!plain) {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int code = t * 16 + 4 * g4 + r;
                pass[r] = pass[r] && !(code >= V || code == qrow || qrow >= V);
              }
            }
            if (__ballot(pass[0] || pass[1] || pass[2] || pass[3])) {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (pass[r]) {
                  const int pos = atomicAdd(&s_cnt[16 * qt + l16], 1);
                  if (pos < a.cap) a.cand[(int64_t)qrow * a.cap + pos] = (uint16_t)(t * 16 + 4 * g4 + r);
                }
            }
          }
        }
      }
    }
  };
  sweep(std::integral_constant<int, 0>());
  __syncthreads();
  // lowest bin taken, per row: b* - 1 less the margin for the rounding of the copy; a wave takes 4 rows
  for (int r = wave * (kSel2Rows / kSel2Waves); r < (wave + 1) * (kSel2Rows / kSel2Waves); ++r) {
    const int bs = find_bstar(s_hist + r * (kBins / 2), kk, lane);
    if (lane == 0) {
      const int low = row0 + r < a.Vp ? bs - 1 - row_margin(a, row0 + r) : 0;
      s_low[r] = low;
      if (row0 + r < a.Vp) a.bstar[row0 + r] = low;
    }
  }
  __syncthreads();
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) thr[qt] = s_low[16 * qt + l16] <= 0 ? -INFINITY : (float)s_low[16 * qt + l16];
  sweep(std::integral_constant<int, 1>());
  __syncthreads();
  if (threadIdx.x < kSel2Rows && row0 + threadIdx.x < a.Vp) a.cnt[row0 + threadIdx.x] = s_cnt[threadIdx.x];
}

__device__ __forceinline__ uint64_t orderable(double x) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// exact key of the pair (row i held in LDS as floats, code j): float64 FMA chain in index order
__device__ __forceinline__ uint64_t exact_key(const float* ei, const float* Ep, int DP, int D, int j) {
  const float* ej = Ep + (int64_t)j * DP;
  double acc = 0.0;
  for (int t0 = 0; t0 < D; t0 += 4) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(ej + t0);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (t0 + e < D) acc = __builtin_fma((double)ei[t0 + e], (double)v[e], acc);
  }
  return orderable(acc);
}

// (key desc, idx asc) "a goes before b"
__device__ __forceinline__ bool before(uint64_t ka, uint32_t ia, uint64_t kb, uint32_t ib) {
  return ka > kb || (ka == kb && ia < ib);
}

__device__ __forceinline__ double key_value(uint64_t K) {
  const uint64_t u = (K >> 63) ? (K & 0x7FFFFFFFFFFFFFFFull) : ~K;
  return __longlong_as_double((long long)u);
}


// Rank of each of the n entries of (skey, sidx) in the order (key desc, idx asc), without a
// comparison sort: the keys are spread over NB buckets by a monotone map of their value
// (bucket 0 = largest), bucket sizes are scanned, the entries' ids are scattered bucket by
// bucket, and an entry's rank is its bucket's start plus the number of bucket mates that go
// before it.  The first kk ranks are written to out[1 + rank]; the key of rank kk - 1 is left in
// *kth.  cur[NB] and ord[n] are LDS scratch.  Ends with a barrier.
__device__ void bucket_rank(const uint64_t* skey, const uint16_t* sidx, int n, int NB, uint32_t* cur,
                            uint16_t* ord, uint64_t* s_red, int kk, int32_t* out, uint64_t* kth,
                            int tid) {
  const int lane = tid & 63, wv = tid >> 6;
  uint64_t lo = ~0ull, hi = 0ull;
  for (int c = tid; c < n; c += kRankThreads) {
    const uint64_t K = skey[c];
    lo = K < lo ? K : lo;
    hi = K > hi ? K : hi;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint64_t l2 = __shfl_xor(lo, o), h2 = __shfl_xor(hi, o);
    lo = l2 < lo ? l2 : lo;
    hi = h2 > hi ? h2 : hi;
  }
  if (lane == 0) { s_red[2 * wv] = lo; s_red[2 * wv + 1] = hi; }
  for (int b = tid; b < NB; b += kRankThreads) cur[b] = 0u;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kRankThreads / 64; ++w) {
    lo = s_red[2 * w] < lo ? s_red[2 * w] : lo;
    hi = s_red[2 * w + 1] > hi ? s_red[2 * w + 1] : hi;
  }
  const double xlo = key_value(lo), xhi = key_value(hi);
  const double span = xhi - xlo;
  // span may be 0, inf or NaN (equal, infinite or NaN keys): then everything shares bucket 0
  const double scale = (span > 0.0 && span < 1.0e300) ? (double)NB / span : 0.0;
  auto bucket_of = [&](uint64_t K) -> int {
    const double f = (xhi - key_value(K)) * scale;        // monotone non-increasing in K
    int b = f >= (double)(NB - 1) ? NB - 1 : (int)f;
    return f > 0.0 ? b : 0;                                // NaN and negatives to bucket 0
  };
  for (int c = tid; c < n; c += kRankThreads) atomicAdd(&cur[bucket_of(skey[c])], 1u);
  __syncthreads();
  // exclusive scan of the NB counts: each lane owns NB / kRankThreads consecutive buckets
  {
    const int per = NB / kRankThreads;                     // NB is a multiple of kRankThreads
    uint32_t local = 0u;
    for (int j = 0; j < per; ++j) local += cur[tid * per + j];
    uint32_t incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    uint32_t* s_wt = reinterpret_cast<uint32_t*>(s_red + 8);
    if (lane == 63) s_wt[wv] = incl;
    __syncthreads();
    uint32_t run = incl - local;
    for (int w = 0; w < wv; ++w) run += s_wt[w];
    for (int j = 0; j < per; ++j) {
      const uint32_t cnt = cur[tid * per + j];
      cur[tid * per + j] = run;
      run += cnt;
    }
  }
  __syncthreads();
  for (int c = tid; c < n; c += kRankThreads) {
    const uint32_t pos = atomicAdd(&cur[bucket_of(skey[c])], 1u);
    ord[pos] = (uint16_t)c;
  }
  __syncthreads();
  // cur[b] is now the end of bucket b; its start is the end of bucket b - 1
  for (int c = tid; c < n; c += kRankThreads) {
    const uint64_t K = skey[c];
    const uint32_t I = sidx[c];
    const int b = bucket_of(K);
    const int beg = b ? (int)cur[b - 1] : 0, end = (int)cur[b];
    int rank = beg;
    for (int m = beg; m < end; ++m) {
      const int o = ord[m];
      rank += before(skey[o], sidx[o], K, I) ? 1 : 0;
    }
    if (rank == kk - 1) *kth = K;
    if (rank < kk) out[1 + rank] = (int32_t)I;
  }
  __syncthreads();
}

// CH floats of a codebook row are staged per step: a wave loads 64 candidate rows with 16-byte
// pieces (whole 64- or 128-byte segments per row), parks them in its own LDS tile and every lane
// then runs the float64 chain of its own candidate over the tile row.
template <int CH>
__global__ __launch_bounds__(kRankThreads) void knn_rank_kernel(KnnArgs a, int P) {
  constexpr int LPR = CH / 4;            // lanes per staged row piece
  constexpr int RPI = 64 / LPR;          // rows per load instruction
  constexpr int PITCH = CH + 4;          // floats; 16-byte reads of 16 consecutive rows hit distinct banks
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_hist[256];
  __shared__ int s_misc[8];
  __shared__ uint64_t s_red[12];
  __shared__ uint64_t s_kth;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int i = blockIdx.x;
  const int V = a.V, D = a.D, DP = a.DP, kk = a.k - 1;
  int32_t* out = a.neigh + (int64_t)i * a.k;
  if (tid == 0) out[0] = i;
  if (kk == 0) return;
  uint64_t* skey = reinterpret_cast<uint64_t*>(smem);
  uint16_t* sidx = reinterpret_cast<uint16_t*>(skey + P);     // (V <= 65536; P is a multiple of 256)
  double* eid = reinterpret_cast<double*>(sidx + P);     // the query row as doubles
  float* ei = reinterpret_cast<float*>(eid + DP);         // and as loaded (exact path)
  // scratch: staging tiles while keys are computed, then the buckets of the ranking
  unsigned char* scratch = reinterpret_cast<unsigned char*>(ei + DP);
  float* tile = reinterpret_cast<float*>(scratch) + wv * 64 * PITCH;
  uint32_t* cur = reinterpret_cast<uint32_t*>(scratch);
  uint16_t* ord = reinterpret_cast<uint16_t*>(cur + P);
  for (int d = tid; d < DP; d += kRankThreads) {
    const float v = a.Ep[(int64_t)i * DP + d];
    ei[d] = v;
    eid[d] = (double)v;
  }
  __syncthreads();

  const int n = a.cnt[i];
  bool slow = n > a.cap || n < kk;          // list overflowed: only the exact path is safe
  if (!slow) {
    const uint16_t* crow = a.cand + (int64_t)i * a.cap;
    const int nsteps = (D + CH - 1) / CH;
    for (int base = wv * 64; base < n; base += kRankThreads) {
      const int c = base + lane;
      const int jown = c < n ? (int)crow[c] : i;
      double acc = 0.0;
      if (CH == 16) {
        // rows of 16 floats are one 64-byte segment: every lane reads its own candidate's row, no tile
        // (Dimensions past D are zero in both rows of the padded copy, and a product of zeros added
        // to the chain leaves it as it is -- the chain starts at +0 and can never be -0 -- so whole
        // groups of four are taken with no test per dimension, and only the groups that hold any.)
        const float* er = a.Ep + (int64_t)jown * DP;
        const int nq = (D + 3) >> 2;                     // uniform
        f32x4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (q < nq) v[q] = *reinterpret_cast<const f32x4*>(er + 4 * q);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (q < nq) {
            const f64x2 e0 = *reinterpret_cast<const f64x2*>(eid + 4 * q);
            const f64x2 e1 = *reinterpret_cast<const f64x2*>(eid + 4 * q + 2);
            acc = __builtin_fma(e0[0], (double)v[q][0], acc);
            acc = __builtin_fma(e0[1], (double)v[q][1], acc);
            acc = __builtin_fma(e1[0], (double)v[q][2], acc);
            acc = __builtin_fma(e1[1], (double)v[q][3], acc);
          }
        if (c < n) { skey[c] = orderable(acc); sidx[c] = (uint16_t)jown; }
        continue;
      }
      f32x4 piece[LPR];
#pragma unroll
      for (int q = 0; q < LPR; ++q) {
        const int jr = __shfl(jown, q * RPI + lane / LPR);
        piece[q] = *reinterpret_cast<const f32x4*>(a.Ep + (int64_t)jr * DP + (lane % LPR) * 4);
      }
      for (int st = 0; st < nsteps; ++st) {
#pragma unroll
        for (int q = 0; q < LPR; ++q)
          *reinterpret_cast<f32x4*>(tile + (q * RPI + lane / LPR) * PITCH + (lane % LPR) * 4) = piece[q];
        wave_lds_sync();
        if (st + 1 < nsteps) {
#pragma unroll
          for (int q = 0; q < LPR; ++q) {
            const int jr = __shfl(jown, q * RPI + lane / LPR);
            piece[q] = *reinterpret_cast<const f32x4*>(a.Ep + (int64_t)jr * DP + (st + 1) * CH + (lane % LPR) * 4);
          }
        }
        const double* eq = eid + st * CH;
        if (D - st * CH >= CH) {
#pragma unroll
          for (int t0 = 0; t0 < CH; t0 += 4) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(tile + lane * PITCH + t0);
            const f64x2 e0 = *reinterpret_cast<const f64x2*>(eq + t0);
            const f64x2 e1 = *reinterpret_cast<const f64x2*>(eq + t0 + 2);
            acc = __builtin_fma(e0[0], (double)v[0], acc);
            acc = __builtin_fma(e0[1], (double)v[1], acc);
            acc = __builtin_fma(e1[0], (double)v[2], acc);
            acc = __builtin_fma(e1[1], (double)v[3], acc);
          }
        } else {
          const int lim = D - st * CH;                       // > 0: the ragged last step
          for (int t = 0; t < lim; ++t) acc = __builtin_fma(eq[t], (double)tile[lane * PITCH + t], acc);
        }
        wave_lds_sync();
      }
      if (c < n) { skey[c] = orderable(acc); sidx[c] = (uint16_t)jown; }
    }
    __syncthreads();
    bucket_rank(skey, sidx, n, P, cur, ord, s_red, kk, out, &s_kth, tid);
    // can a code outside the candidate list still belong to the row?
    const int low = a.bstar[i];
    if (low >= 1) {
      const float edge = (float)low / a.bin_scale - 1.0f;         // lower edge of the lowest bin taken
      slow = s_kth < orderable((double)edge + (double)row_eps(a, i));
    }
    if (!slow) return;
    // the row was written from the candidate list and is written again below by other lanes:
    // make the first version reach memory before any lane goes on (rare path)
    __threadfence();
    __syncthreads();
  }
  // ---- exact path over all V codes: radix select of the kk-th largest key
  {
    uint64_t prefix = 0ull;
    int need = kk;
    for (int byte = 7; byte >= 0; --byte) {
      s_hist[tid] = 0;
      __syncthreads();
      for (int j = tid; j < V; j += kRankThreads) {
        if (j == i) continue;
        const uint64_t K = exact_key(ei, a.Ep, DP, D, j);
        const bool match = byte == 7 || (K >> (8 * (byte + 1))) == (prefix >> (8 * (byte + 1)));
        if (match) atomicAdd(&s_hist[(int)((K >> (8 * byte)) & 255ull)], 1);
      }
      __syncthreads();
      if (tid == 0) {
        int cum = 0, bsel = 0;
        for (int bkt = 255; bkt >= 0; --bkt) {
          if (cum + s_hist[bkt] >= need) { bsel = bkt; break; }
          cum += s_hist[bkt];
        }
        s_misc[0] = bsel;
        s_misc[1] = need - cum;
      }
      __syncthreads();
      prefix |= (uint64_t)s_misc[0] << (8 * byte);
      need = s_misc[1];
      __syncthreads();
    }
    // prefix = exact kk-th largest key; keep everything above it plus the `need`
    // lowest-index codes equal to it
    const int n_gt = kk - need;
    if (tid == 0) { s_misc[2] = 0; s_misc[3] = 0; }
    __syncthreads();
    for (int j0 = 0; j0 < V; j0 += kRankThreads) {
      const int j = j0 + tid;
      uint64_t K = 0ull;
      bool gt = false, eq = false;
      if (j < V && j != i) {
        K = exact_key(ei, a.Ep, DP, D, j);
        gt = K > prefix;
        eq = K == prefix;
      }
      if (gt) {
        const int pos = atomicAdd(&s_misc[2], 1);
        skey[pos] = K; sidx[pos] = (uint16_t)j;
      }
      // ordered compaction of the ties (ascending index)
      const unsigned long long bal = __ballot(eq);
      if (lane == 0) s_hist[wv] = __popcll(bal);
      __syncthreads();
      int base = s_misc[3];
      for (int w = 0; w < wv; ++w) base += s_hist[w];
      const int rank = base + __popcll(bal & ((1ull << lane) - 1ull));
      if (eq && rank < need) { skey[n_gt + rank] = K; sidx[n_gt + rank] = (uint16_t)j; }
      __syncthreads();
      if (tid == 0) s_misc[3] += s_hist[0] + s_hist[1] + s_hist[2] + s_hist[3];
      __syncthreads();
    }
    bucket_rank(skey, sidx, kk, P, cur, ord, s_red, kk, out, &s_kth, tid);
  }
}

int32_t cap_for(int32_t k, int32_t DP) {
  return (int32_t)lpp_align_up((size_t)(k - 1) + (DP <= 16 ? kSlackShort : kSlack), 64);
}

struct KnnLayout {
  size_t o_ep, o_eh, o_norms, o_max, o_bstar, o_cnt, o_cand, total;
  int32_t DP, Vp, cap;
};

KnnLayout knn_layout(int32_t V, int32_t D, int32_t k) {
  KnnLayout L;
  L.DP = 16;
  while (L.DP < D) L.DP <<= 1;             // 16, 32, ..., 256
  L.Vp = (int32_t)lpp_align_up((size_t)V, 64);
  L.cap = cap_for(k, L.DP);
  size_t o = 0;
  L.o_ep = o;    o += lpp_align_up((size_t)L.Vp * L.DP * sizeof(float), 256);
  L.o_eh = o;    o += L.DP >= 32 ? lpp_align_up((size_t)L.Vp * L.DP * sizeof(uint16_t), 256) : 0;
  L.o_norms = o; o += lpp_align_up((size_t)L.Vp * sizeof(float), 256);
  L.o_max = o;   o += 256;
  L.o_bstar = o; o += lpp_align_up((size_t)L.Vp * sizeof(int32_t), 256);
  L.o_cnt = o;   o += lpp_align_up((size_t)L.Vp * sizeof(int32_t), 256);
  L.o_cand = o;  o += lpp_align_up((size_t)V * L.cap * sizeof(uint16_t), 256);
  L.total = o;
  return L;
}

template <int KS>
int32_t launch_select_bf16(const KnnArgs& a, hipStream_t s) {
  const size_t lds = (size_t)kSel2Rows * (kBins / 2) * sizeof(uint32_t);
  auto kern = knn_select_bf16_kernel<KS>;
  static LppLdsLimit limit;
  const int32_t st = lpp_ensure_lds(reinterpret_cast<const void*>(kern), limit, lds);
  if (st != LPP_OK) return st;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.Vp / kSel2Rows)), dim3(kSel2Waves * 64), lds, s, a);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}

int32_t launch_select_f32(const KnnArgs& a, hipStream_t s) {
  const size_t lds = (size_t)kSelRows * kBinsF * sizeof(uint32_t);
  static LppLdsLimit limit;
  const int32_t st = lpp_ensure_lds(reinterpret_cast<const void*>(knn_select_f32_kernel), limit, lds);
  if (st != LPP_OK) return st;
  hipLaunchKernelGGL(knn_select_f32_kernel, dim3((unsigned)(a.Vp / kSelRows)), dim3(kSelWaves * 64), lds, s, a);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}

}  // namespace

extern "C" size_t lpp_build_neighbours_workspace(int32_t V, int32_t D, int32_t k) {
  if (V < 1 || D < 1 || k < 1 || k > V || k > LPP_MAX_K || D > 256 || V > 65536) return 0;
  return knn_layout(V, D, k).total;
}

extern "C" int32_t lpp_build_neighbours(const float* E, int32_t V, int32_t D, int32_t k, int32_t* neigh,
                                        void* ws, size_t ws_bytes, void* stream) {
  if (!E || !neigh) return LPP_EINVAL;
  if (V < 1 || D < 1 || k < 1 || k > V) return LPP_EINVAL;
  if (k > LPP_MAX_K || D > 256 || V > 65536) return LPP_EUNSUPPORTED;
  const KnnLayout L = knn_layout(V, D, k);
  if (!ws || ws_bytes < L.total) return LPP_ENOWORKSPACE;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { (void)hipGetLastError(); return LPP_EHIP; }
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  unsigned char* w = reinterpret_cast<unsigned char*>(ws);
  KnnArgs a;
  a.E = E; a.V = V; a.D = D; a.DP = L.DP; a.Vp = L.Vp; a.k = k; a.cap = L.cap;
  a.Ep = reinterpret_cast<float*>(w + L.o_ep);
  a.Eh = L.DP >= 32 ? reinterpret_cast<uint16_t*>(w + L.o_eh) : nullptr;
  a.bin_scale = a.Eh ? kBinScale : kBinScaleF;
  a.norms = reinterpret_cast<float*>(w + L.o_norms);
  a.maxnorm = reinterpret_cast<uint32_t*>(w + L.o_max);
  a.bstar = reinterpret_cast<int32_t*>(w + L.o_bstar);
  a.cnt = reinterpret_cast<int32_t*>(w + L.o_cnt);
  a.cand = reinterpret_cast<uint16_t*>(w + L.o_cand);
  a.neigh = neigh;

  hipLaunchKernelGGL(knn_init_kernel, dim3(1), dim3(64), 0, s, a);
  LPP_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(knn_pack_kernel, dim3((unsigned)((L.Vp + kPackRows - 1) / kPackRows)), dim3(256), 0, s, a);
  LPP_HIP_TRY(hipGetLastError());
  if (k > 1) {
    int32_t st;
    switch (L.DP / 16) {
      case 1: st = launch_select_f32(a, s); break;
      case 2: st = launch_select_bf16<1>(a, s); break;
      case 4: st = launch_select_bf16<2>(a, s); break;
      case 8: st = launch_select_bf16<4>(a, s); break;
      case 16: st = launch_select_bf16<8>(a, s); break;
      default: st = LPP_EUNSUPPORTED; break;
    }
    if (st != LPP_OK) return st;
  }
  const int P = (int)lpp_align_up((size_t)L.cap, kRankThreads);
  const int CH = L.DP < 32 ? 16 : 32;
  // keys + indices + the query row (as doubles and floats) + max(staging tiles, bucket counters and order);
  // rows of 16 floats need no staging tiles
  const size_t stage = CH == 16 ? 0 : (size_t)(kRankThreads / 64) * 64 * (CH + 4) * sizeof(float);
  const size_t sortb = (size_t)P * 6;
  const size_t lds = (size_t)P * 10 + (size_t)L.DP * 12 + (stage > sortb ? stage : sortb);
  if (lds > 150 * 1024) return LPP_EUNSUPPORTED;
  static LppLdsLimit limit[2];   // (zero-initialised) one per kernel
  const void* fn = CH == 16 ? reinterpret_cast<const void*>(knn_rank_kernel<16>)
                            : reinterpret_cast<const void*>(knn_rank_kernel<32>);
  const int32_t st = lpp_ensure_lds(fn, limit[CH == 32], lds);
  if (st != LPP_OK) return st;
  if (CH == 16)
    hipLaunchKernelGGL(knn_rank_kernel<16>, dim3((unsigned)V), dim3(kRankThreads), lds, s, a, P);
  else
    hipLaunchKernelGGL(knn_rank_kernel<32>, dim3((unsigned)V), dim3(kRankThreads), lds, s, a, P);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}
