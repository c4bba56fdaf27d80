// Relaxed acceptance over a static draft tree: per-row vocabulary softmax,
// neighbour gather-sum under the multiplicative bound, ratio / accept test,
// residual update, inverse-CDF draw, and the walk (paper Sec. 4; Sec. 2.2;
// App. A.2 Eq. 1-2).
//
// One workgroup of 1024 lanes owns one tree row of one batch item.  The row's
// target distribution r lives in LDS (unnormalised, with a running scale) and in
// the registers of the lanes that loaded it; the drafter distribution p stays in
// registers only.  The two logit rows are therefore read from HBM exactly once and
// every later pass (gather, prefix scan, residual, CDF search) runs out of LDS and
// registers.  The neighbour rows of the row's first children are fetched while the
// logits are still in flight.  Rows are independent: each is evaluated for the
// outcome "all earlier siblings were rejected", which needs no uniform.  The last
// row of a batch item to finish chases the recorded decisions from the root.
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include "lpp_internal.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kPre = 8;        // children per row whose neighbour lists are staged in LDS
constexpr int kPreK = 1024;    // neighbour slots staged per child

struct TreeTab {               // by-value kernel argument: read through the scalar cache
  uint16_t child_ptr[LPP_MAX_ROWS + 1];
  uint16_t child_idx[LPP_MAX_ROWS];
};

struct VerifyArgs {
  const float* target;
  const float* drafter;
  int64_t ldv;
  int32_t off, V, M, kstride, k, depth;
  float lambda;
  const int32_t* tokens;
  const int32_t* neigh;
  const float* u_accept;
  const float* u_final;
  uint8_t* decision;
  float* ratio;
  float* mass;
  int32_t* n_agg;
  float* q_tok;
  float* p_tok;
  int32_t* final_all;
  int32_t* accept_len;
  int32_t* path;
  int32_t* final_token;
  int32_t* ws_decision;   // [B*M] always written: the walk reads these
  int32_t* ws_final;      // [B*M]
  int32_t* counters;      // [B] zero between calls, or null: walk runs as its own kernel
  int32_t dbg;
};

// ---- wave64 primitives on DPP (row shifts, row broadcasts)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or(float old, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_inclusive_scan(float v) {
  v += dpp_or<0x111, 0xf>(0.f, v);   // row_shr:1
  v += dpp_or<0x112, 0xf>(0.f, v);   // row_shr:2
  v += dpp_or<0x114, 0xf>(0.f, v);   // row_shr:4
  v += dpp_or<0x118, 0xf>(0.f, v);   // row_shr:8
  v += dpp_or<0x142, 0xa>(0.f, v);   // row_bcast:15 into rows 1 and 3
  v += dpp_or<0x143, 0xc>(0.f, v);   // row_bcast:31 into rows 2 and 3
  return v;
}
__device__ __forceinline__ float wave_prev_lane(float v, float first) {   // lane i <- lane i-1
  return dpp_or<0x138, 0xf>(first, v);                                      // wave_shr:1
}
__device__ __forceinline__ float wave_sum(float v) {
  v = wave_inclusive_scan(v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  const float ninf = -INFINITY;
  v = fmaxf(v, dpp_or<0x111, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x112, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x114, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x118, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x142, 0xa>(ninf, v));
  v = fmaxf(v, dpp_or<0x143, 0xc>(ninf, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// exp(x) for x <= 0 through the hardware exp2; the argument is formed in two
// pieces so that its rounding error stays below one ulp of the result.
__device__ __forceinline__ float exp_neg(float x) {
  const float hi = 1.44269502162933349609375f, lo = 1.925963033500011e-08f;   // log2(e) = hi + lo
  return __builtin_amdgcn_exp2f(__builtin_fmaf(x, hi, x * lo));
}

template <bool ALIGNED>
__device__ __forceinline__ float4 load_logits4(const float* row, int e0, int V) {
  const float ninf = -INFINITY;
  if (ALIGNED && e0 + 3 < V) {
    typedef float vec4f __attribute__((ext_vector_type(4)));
    const vec4f x = __builtin_nontemporal_load(reinterpret_cast<const vec4f*>(row + e0));
    return make_float4(x.x, x.y, x.z, x.w);
  }
  float4 v;
  v.x = (e0 + 0 < V) ? __builtin_nontemporal_load(row + e0 + 0) : ninf;
  v.y = (e0 + 1 < V) ? __builtin_nontemporal_load(row + e0 + 1) : ninf;
  v.z = (e0 + 2 < V) ? __builtin_nontemporal_load(row + e0 + 2) : ninf;
  v.w = (e0 + 3 < V) ? __builtin_nontemporal_load(row + e0 + 3) : ninf;
  return v;
}

// Follow the first accepted child per level from the root (App. A.2: accepted
// tokens are kept, everything after the first rejection is discarded).
__device__ __forceinline__ void walk_item(const TreeTab& tt, const int* dec, const int* fin, int depth,
                                          int32_t* accept_len, int32_t* path, int32_t* final_token) {
  int cur = 0, n = 0;
  while (n < depth) {
    int nxt = -1;
    for (int ci = tt.child_ptr[cur]; ci < tt.child_ptr[cur + 1]; ++ci) {
      const int c = tt.child_idx[ci];
      if (dec[c]) { nxt = c; break; }
    }
    if (nxt < 0) break;
    path[n++] = nxt;
    cur = nxt;
  }
  for (int i = n; i < depth; ++i) path[i] = -1;
  *accept_len = n;
  *final_token = fin[cur];
}

// NCH = float4 chunks per lane; a row holds at most NCH * 4096 tokens.  Lane `tid`
// owns tokens 4*(tid + 1024*j) .. +3 for j < NCH.
template <int NCH, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void verify_rows_kernel(VerifyArgs a, TreeTab tt) {
  extern __shared__ float r_lds[];  // NCH * 4096 floats: current r, unnormalised
  __shared__ uint16_t s_neigh[kPre * kPreK];
  __shared__ float s_red[2][kWaves];
  __shared__ float s_seg[NCH][kWaves];
  __shared__ float s_wtot[kWaves];
  __shared__ int s_vidx[kWaves];
  __shared__ float s_vval[kWaves];
  __shared__ int s_lastpos[kWaves];
  __shared__ int s_tok[LPP_MAX_ROWS];
  __shared__ float s_dlog[LPP_MAX_ROWS];
  __shared__ int s_walk[2 * LPP_MAX_ROWS];
  __shared__ int s_ticket;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int P = blockIdx.x % a.M, b = blockIdx.x / a.M;
  const int V = a.V;
  const int64_t nodebase = (int64_t)b * a.M;
  const int64_t rowoff = (nodebase + P) * a.ldv + a.off;
  const float* trow = a.target + rowoff;
  const int cp0 = tt.child_ptr[P];
  const int nchild = tt.child_ptr[P + 1] - cp0;
  const float* drow = nchild > 0 ? a.drafter + rowoff : nullptr;
  const int npre = min(nchild, kPre);
  const int kpre = min(a.k, kPreK);

  // ---- small dependent reads first, so that they are not queued behind the rows
  int my_tok = 0;
  float my_dlog = 0.f;
  if (tid < nchild) {
    my_tok = a.tokens[nodebase + tt.child_idx[cp0 + tid]];
    my_tok = min(max(my_tok, 0), V - 1);
    my_dlog = drow[my_tok];
  }
  int ptok[kPre];
#pragma unroll
  for (int ci = 0; ci < kPre; ++ci) {
    ptok[ci] = 0;
    if (ci < npre) {
      const int t = a.tokens[nodebase + tt.child_idx[cp0 + ci]];
      ptok[ci] = min(max(t, 0), V - 1);
    }
  }

  // ---- every HBM read of the row is issued up front
  float4 tv[NCH], dv[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) tv[j] = load_logits4<ALIGNED>(trow, 4 * (tid + kThreads * j), V);
  if (nchild > 0) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) dv[j] = load_logits4<ALIGNED>(drow, 4 * (tid + kThreads * j), V);
  } else {
#pragma unroll
    for (int j = 0; j < NCH; ++j) dv[j] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  }
  int nreg[kPre];
#pragma unroll
  for (int ci = 0; ci < kPre; ++ci) {
    nreg[ci] = ptok[ci];
    if (ci < npre && tid > 0 && tid < kpre) nreg[ci] = a.neigh[(int64_t)ptok[ci] * a.kstride + tid];
  }

  // ---- softmax statistics of both rows (Sec. 2 notation: q target, p drafter; T = 1)
  float mt = -INFINITY, md = -INFINITY;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    mt = fmaxf(mt, fmaxf(fmaxf(tv[j].x, tv[j].y), fmaxf(tv[j].z, tv[j].w)));
    md = fmaxf(md, fmaxf(fmaxf(dv[j].x, dv[j].y), fmaxf(dv[j].z, dv[j].w)));
  }
  mt = wave_max(mt);
  md = wave_max(md);
  if (lane == 0) { s_red[0][w] = mt; s_red[1][w] = md; }
  if (tid < nchild) { s_tok[tid] = my_tok; s_dlog[tid] = my_dlog; }
  __syncthreads();
  mt = s_red[0][0]; md = s_red[1][0];
#pragma unroll
  for (int i = 1; i < kWaves; ++i) { mt = fmaxf(mt, s_red[0][i]); md = fmaxf(md, s_red[1][i]); }
  if (mt == -INFINITY) mt = 0.f;
  if (md == -INFINITY) md = 0.f;
  __syncthreads();

  float r_reg[NCH][4], p_reg[NCH][4];
  float st = 0.f, sd = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    r_reg[j][0] = exp_neg(tv[j].x - mt); r_reg[j][1] = exp_neg(tv[j].y - mt);
    r_reg[j][2] = exp_neg(tv[j].z - mt); r_reg[j][3] = exp_neg(tv[j].w - mt);
    p_reg[j][0] = exp_neg(dv[j].x - md); p_reg[j][1] = exp_neg(dv[j].y - md);
    p_reg[j][2] = exp_neg(dv[j].z - md); p_reg[j][3] = exp_neg(dv[j].w - md);
    st += (r_reg[j][0] + r_reg[j][1]) + (r_reg[j][2] + r_reg[j][3]);
    sd += (p_reg[j][0] + p_reg[j][1]) + (p_reg[j][2] + p_reg[j][3]);
    *reinterpret_cast<float4*>(&r_lds[4 * (tid + kThreads * j)]) =
        make_float4(r_reg[j][0], r_reg[j][1], r_reg[j][2], r_reg[j][3]);
  }
#pragma unroll
  for (int ci = 0; ci < kPre; ++ci)
    if (ci < npre) s_neigh[ci * kPreK + tid] = (uint16_t)min(max(nreg[ci], 0), V - 1);
  st = wave_sum(st);
  sd = wave_sum(sd);
  if (lane == 0) { s_red[0][w] = st; s_red[1][w] = sd; }
  __syncthreads();
  st = 0.f; sd = 0.f;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) { st += s_red[0][i]; sd += s_red[1][i]; }
  float rs = st > 0.f ? 1.0f / st : 0.f;           // r_true = r_lds * rs
  const float inv_sd = sd > 0.f ? 1.0f / sd : 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) p_reg[j][e] = p_reg[j][e] * inv_sd;

  if (P == 0 && tid == 0) {  // row 0 is no drafted node: defined outputs
    a.ws_decision[nodebase] = 0;
    if (a.decision) a.decision[nodebase] = 0;
    if (a.ratio) a.ratio[nodebase] = 0.f;
    if (a.mass) a.mass[nodebase] = 0.f;
    if (a.n_agg) a.n_agg[nodebase] = 0;
    if (a.q_tok) a.q_tok[nodebase] = 0.f;
    if (a.p_tok) a.p_tok[nodebase] = 0.f;
  }

  if (a.dbg == 1) { if (tid == 0) a.ws_final[nodebase + P] = (int)(rs * 1e6f + p_reg[0][0]); return; }
  // ---- children in static order, each against the current residual r
  for (int ci = 0; ci < (a.dbg == 2 ? 0 : nchild); ++ci) {
    const int c = tt.child_idx[cp0 + ci];
    const int t = s_tok[ci];
    const float rt = r_lds[t];
    const float cap = a.lambda * rt;                 // bound: sum_A r < lambda * r(x^)   (Sec. 4)
    const int32_t* nrow = a.neigh + (int64_t)t * a.kstride;
    const bool staged = ci < kPre;
    float carry = 0.f, mass_u = 0.f;
    int jstar = INT_MAX;
    int n_first = t;
    for (int base = 0; base < a.k; base += kThreads) {
      const int i = base + tid;
      int n = t;
      float v = 0.f;
      if (i < a.k) {
        if (i > 0) {
          if (staged && base == 0) n = s_neigh[ci * kPreK + tid];
          else { n = nrow[i]; n = min(max(n, 0), V - 1); }
        }
        v = r_lds[n];
      }
      if (base == 0) n_first = n;
      const float incl = wave_inclusive_scan(v);
      if (lane == 63) s_wtot[w] = incl;
      __syncthreads();
      float prefix = carry, total = carry;
#pragma unroll
      for (int ww = 0; ww < kWaves; ++ww) {
        if (ww == w) prefix = total;
        total += s_wtot[ww];
      }
      const float C = prefix + incl;                          // prefix sum including slot i
      const float excl = prefix + wave_prev_lane(incl, 0.f);  // = C of slot i-1
      const bool stop = (i >= 1 && i < a.k && !(C < cap)) || (i == a.k);
      const unsigned long long bal = __ballot(stop);
      if (bal) {
        const int fl = __ffsll((long long)bal) - 1;
        if (lane == fl) { s_vidx[w] = i; s_vval[w] = excl; }
      } else if (lane == 0) {
        s_vidx[w] = INT_MAX;
      }
      __syncthreads();
#pragma unroll
      for (int ww = kWaves - 1; ww >= 0; --ww)
        if (s_vidx[ww] != INT_MAX) { jstar = s_vidx[ww]; mass_u = s_vval[ww]; }
      if (jstar != INT_MAX) break;
      carry = total;
    }
    if (jstar == INT_MAX) { jstar = a.k; mass_u = carry; }

    if (tid == 0) {
      const float qt = rt * rs, m = mass_u * rs;
      const float pt = exp_neg(s_dlog[ci] - md) * inv_sd;
      const float u = a.u_accept[nodebase + c];
      const int dec = (u * pt < m) ? 1 : 0;                   // u < min(1, mass / p(x^))
      a.ws_decision[nodebase + c] = dec;
      if (a.decision) a.decision[nodebase + c] = (uint8_t)dec;
      if (a.ratio) a.ratio[nodebase + c] = m / pt;
      if (a.mass) a.mass[nodebase + c] = m;
      if (a.n_agg) a.n_agg[nodebase + c] = jstar;
      if (a.q_tok) a.q_tok[nodebase + c] = qt;
      if (a.p_tok) a.p_tok[nodebase + c] = pt;
    }

    // outcome "rejected": move A's mass onto x^ ...
    for (int base = 0; base < jstar; base += kThreads) {
      const int i = base + tid;
      if (i >= 1 && i < jstar) {
        int n = n_first;
        if (base > 0) { n = nrow[i]; n = min(max(n, 0), V - 1); }
        if (n != t) r_lds[n] = 0.f;
      }
    }
    if (tid == 0) r_lds[t] = mass_u;
    __syncthreads();
    // ... and keep the normalised positive part of (r' - p)    (Eq. 2)
    float res[NCH][4];
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const float4 rv = *reinterpret_cast<const float4*>(&r_lds[4 * (tid + kThreads * j)]);
      res[j][0] = fmaxf(rv.x * rs - p_reg[j][0], 0.f);
      res[j][1] = fmaxf(rv.y * rs - p_reg[j][1], 0.f);
      res[j][2] = fmaxf(rv.z * rs - p_reg[j][2], 0.f);
      res[j][3] = fmaxf(rv.w * rs - p_reg[j][3], 0.f);
      z += (res[j][0] + res[j][1]) + (res[j][2] + res[j][3]);
    }
    z = wave_sum(z);
    if (lane == 0) s_red[0][w] = z;
    __syncthreads();
    z = 0.f;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) z += s_red[0][i];
    if (z > 0.f) {
      rs = 1.0f / z;
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
#pragma unroll
        for (int e = 0; e < 4; ++e) r_reg[j][e] = res[j][e];
        *reinterpret_cast<float4*>(&r_lds[4 * (tid + kThreads * j)]) =
            make_float4(res[j][0], res[j][1], res[j][2], res[j][3]);
      }
    } else {  // r' == p: nothing left to resample from; r stays as it was
#pragma unroll
      for (int j = 0; j < NCH; ++j)
        *reinterpret_cast<float4*>(&r_lds[4 * (tid + kThreads * j)]) =
            make_float4(r_reg[j][0], r_reg[j][1], r_reg[j][2], r_reg[j][3]);
    }
    __syncthreads();
  }

  // ---- draw from the final r by inverse CDF over ascending token index.  The
  // cumulative sum is taken segment by segment (segment j = tokens [4096 j, 4096 j + 4096)),
  // inside a segment chunk by chunk in lane order: the same sums decide which
  // segment, which chunk and which token holds the target.
  float csum[NCH], incl[NCH];
  int lastpos = -1;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    csum[j] = (r_reg[j][0] + r_reg[j][1]) + (r_reg[j][2] + r_reg[j][3]);
    incl[j] = wave_inclusive_scan(csum[j]);
    if (lane == 63) s_seg[j][w] = incl[j];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (r_reg[j][e] > 0.f) lastpos = 4 * (tid + kThreads * j) + e;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, o));
  if (lane == 0) s_lastpos[w] = lastpos;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j)
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) total += s_seg[j][ww];
  const float target = a.u_final[nodebase + P] * total;
  // replay the same running sum: the lane whose chunk crosses the target reports it
  float run = 0.f;
  int found = INT_MAX;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    float prefix = run;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) {
      if (ww == w) prefix = run;
      run += s_seg[j][ww];
    }
    const float cin = prefix + incl[j];                          // cumulative mass after my chunk
    const float cex = prefix + wave_prev_lane(incl[j], 0.f);     // ... and before it
    if (found == INT_MAX && cin > target) {
      const float u0 = cex + r_reg[j][0], u1 = u0 + r_reg[j][1], u2 = u1 + r_reg[j][2];
      int e = u0 > target ? 0 : u1 > target ? 1 : u2 > target ? 2 : 3;
      if (!(r_reg[j][e] > 0.f)) e = r_reg[j][3] > 0.f ? 3 : r_reg[j][2] > 0.f ? 2 : r_reg[j][1] > 0.f ? 1 : 0;
      found = 4 * (tid + kThreads * j) + e;
    }
  }
  // lowest token over the block: chunks are ordered by (segment, wave, lane) = token order
  int best = found;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o));
  if (lane == 0) s_vidx[w] = best;
  __syncthreads();
  if (tid == 0) {
    int x = INT_MAX, lp = -1;
    for (int ww = 0; ww < kWaves; ++ww) { x = min(x, s_vidx[ww]); lp = max(lp, s_lastpos[ww]); }
    if (x == INT_MAX) x = lp >= 0 ? lp : 0;
    x = min(x, V - 1);
    a.ws_final[nodebase + P] = x;
    if (a.final_all) a.final_all[nodebase + P] = x;
    if (a.counters) {
      __threadfence();
      s_ticket = atomicAdd(&a.counters[b], 1);
    }
  }
  if (!a.counters) return;
  __syncthreads();
  if (s_ticket != a.M - 1) return;
  // ---- this row finished last for item b: every decision of the item is visible
  __threadfence();
  if (tid < a.M) {
    s_walk[tid] = __hip_atomic_load(&a.ws_decision[nodebase + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_walk[LPP_MAX_ROWS + tid] = __hip_atomic_load(&a.ws_final[nodebase + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (tid == 0) {
    walk_item(tt, s_walk, s_walk + LPP_MAX_ROWS, a.depth, a.accept_len + b, a.path + (int64_t)b * a.depth,
              a.final_token + b);
    a.counters[b] = 0;    // ready for the next call
  }
}

// Stand-alone walk for batches larger than the counter array.
__global__ void walk_kernel(VerifyArgs a, TreeTab tt, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  walk_item(tt, a.ws_decision + (int64_t)b * a.M, a.ws_final + (int64_t)b * a.M, a.depth, a.accept_len + b,
            a.path + (int64_t)b * a.depth, a.final_token + b);
}

template <int NCH, bool ALIGNED>
int32_t launch_rows(const VerifyArgs& a, const TreeTab& tt, int B, hipStream_t stream) {
  static bool attr_set = false;
  const size_t lds = (size_t)NCH * 4096 * sizeof(float);
  auto kern = verify_rows_kernel<NCH, ALIGNED>;
  if (!attr_set) {
    LPP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(B * a.M)), dim3(kThreads), lds, stream, a, tt);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}

}  // namespace

extern "C" size_t lpp_relaxed_verify_workspace(const lpp_tree* tree, int32_t B, int32_t V, int32_t k) {
  (void)V; (void)k;
  if (!tree || B < 1) return 0;
  const size_t nodes = (size_t)B * tree->M;
  return 2 * lpp_align_up(nodes * sizeof(int32_t), 256);
}

extern "C" int32_t lpp_relaxed_verify(const lpp_tree* tree, const float* target_logits,
                                      const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                      int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                      int32_t kstride, int32_t k, float lambda, const float* u_accept,
                                      const float* u_final, const lpp_verify_out* out, void* ws,
                                      size_t ws_bytes, void* stream) {
  if (!tree || !target_logits || !tokens || !neigh || !u_accept || !u_final || !out) return LPP_EINVAL;
  if (!out->accept_len || !out->path || !out->final_token) return LPP_EINVAL;
  if (tree->M > 1 && !drafter_logits) return LPP_EINVAL;
  if (B < 1 || V < 1 || k < 1 || k > kstride || k > V) return LPP_EINVAL;
  if (vocab_offset < 0 || (int64_t)vocab_offset + V > ldv) return LPP_EINVAL;
  if (lambda != lambda) return LPP_EINVAL;
  if (V > LPP_MAX_VOCAB) return LPP_EUNSUPPORTED;
  if ((int64_t)B * tree->M > INT_MAX) return LPP_EUNSUPPORTED;
  const size_t need = lpp_relaxed_verify_workspace(tree, B, V, k);
  if (!ws || ws_bytes < need) return LPP_ENOWORKSPACE;
  if (!tree->d_counters) return LPP_EHIP;

  VerifyArgs a;
  a.target = target_logits; a.drafter = drafter_logits; a.ldv = ldv; a.off = vocab_offset;
  a.V = V; a.M = tree->M; a.kstride = kstride; a.k = k; a.lambda = lambda;
  a.depth = tree->depth > 0 ? tree->depth : 1;
  a.tokens = tokens; a.neigh = neigh; a.u_accept = u_accept; a.u_final = u_final;
  a.decision = out->decision; a.ratio = out->ratio; a.mass = out->mass; a.n_agg = out->n_agg;
  a.q_tok = out->q_tok; a.p_tok = out->p_tok; a.final_all = out->final_tok_all;
  a.accept_len = out->accept_len; a.path = out->path; a.final_token = out->final_token;
  const size_t nodes = (size_t)B * tree->M;
  a.ws_decision = reinterpret_cast<int32_t*>(ws);
  a.ws_final = reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(ws) +
                                          lpp_align_up(nodes * sizeof(int32_t), 256));
  const bool fused_walk = B <= LPP_COUNTER_SLOTS;
  a.counters = fused_walk ? tree->d_counters : nullptr;
  { const char* e = getenv("LPP_DBG"); a.dbg = e ? atoi(e) : 0; }

  TreeTab tt;
  for (int i = 0; i <= LPP_MAX_ROWS; ++i)
    tt.child_ptr[i] = (uint16_t)(i <= tree->M ? tree->child_ptr[i] : tree->child_ptr[tree->M]);
  for (int i = 0; i < LPP_MAX_ROWS; ++i)
    tt.child_idx[i] = (uint16_t)(i < tree->M - 1 ? tree->child_idx[i] : 0);

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  auto aligned16 = [&](const float* p) {
    return p == nullptr || ((reinterpret_cast<uintptr_t>(p + vocab_offset) % 16 == 0) && (ldv % 4 == 0));
  };
  const bool al = aligned16(target_logits) && aligned16(drafter_logits);
  const int nch = V <= 4096 ? 1 : V <= 8192 ? 2 : V <= 16384 ? 4 : 8;
  int32_t st;
#define LPP_DISPATCH(N) st = al ? launch_rows<N, true>(a, tt, B, s) : launch_rows<N, false>(a, tt, B, s)
  switch (nch) {
    case 1: LPP_DISPATCH(1); break;
    case 2: LPP_DISPATCH(2); break;
    case 4: LPP_DISPATCH(4); break;
    default: LPP_DISPATCH(8); break;
  }
#undef LPP_DISPATCH
  if (st != LPP_OK) return st;
  if (!fused_walk) {
    hipLaunchKernelGGL(walk_kernel, dim3((unsigned)((B + 63) / 64)), dim3(64), 0, s, a, tt, B);
    LPP_HIP_TRY(hipGetLastError());
  }
  return LPP_OK;
}
