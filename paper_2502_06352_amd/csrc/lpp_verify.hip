// Relaxed acceptance over a static draft tree: per-row vocabulary softmax,
// neighbour gather-sum under the multiplicative bound, ratio / accept test,
// residual update, inverse-CDF draw, and the walk (paper Sec. 4; Sec. 2.2;
// App. A.2 Eq. 1-2).
//
// One workgroup of 1024 lanes owns one tree row of one batch item.  The row's
// target distribution r lives in LDS (unnormalised, with a running scale), the
// drafter distribution p stays in registers of the lanes that loaded it, so the
// two logit rows are read from HBM exactly once and every later pass (gather,
// prefix scan, residual, CDF search) runs out of LDS.  Rows are independent: each
// is evaluated for the outcome "all earlier siblings were rejected", which needs
// no uniform, and a second tiny kernel chases the decisions from the root.
#include <limits.h>
#include <math.h>

#include "lpp_internal.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxChildren = LPP_MAX_ROWS;

struct VerifyArgs {
  const float* target;
  const float* drafter;
  int64_t ldv;
  int32_t off, V, M, kstride, k;
  float lambda;
  const int32_t* tokens;
  const int32_t* neigh;
  const float* u_accept;
  const float* u_final;
  const int32_t* child_ptr;
  const int32_t* child_idx;
  uint8_t* decision;
  float* ratio;
  float* mass;
  int32_t* n_agg;
  float* q_tok;
  float* p_tok;
  int32_t* final_all;
  uint8_t* ws_decision;  // always written: the walk reads these
  int32_t* ws_final;
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_inclusive_scan(float v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    float t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
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

// NCH = float4 chunks per lane; a row holds at most NCH * 4096 tokens.
template <int NCH, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void verify_rows_kernel(VerifyArgs a) {
  extern __shared__ float r_lds[];  // NCH * 4096 floats: current r, unnormalised
  __shared__ float s_red[2][kWaves];
  __shared__ float s_wtot[kWaves];
  __shared__ int s_vidx[kWaves];
  __shared__ float s_vval[kWaves];
  __shared__ int s_lastpos[kWaves];
  __shared__ int s_tok[kMaxChildren];
  __shared__ float s_dlog[kMaxChildren];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int P = blockIdx.x % a.M, b = blockIdx.x / a.M;
  const int V = a.V;
  const int64_t rowoff = ((int64_t)b * a.M + P) * a.ldv + a.off;
  const float* trow = a.target + rowoff;
  const int cp0 = a.child_ptr[P], cp1 = a.child_ptr[P + 1];
  const int nchild = cp1 - cp0;
  const float* drow = nchild > 0 ? a.drafter + rowoff : nullptr;

  // ---- issue every HBM read of the row up front
  float4 tv[NCH], dv[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) tv[j] = load_logits4<ALIGNED>(trow, 4 * (tid + kThreads * j), V);
  if (nchild > 0) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) dv[j] = load_logits4<ALIGNED>(drow, 4 * (tid + kThreads * j), V);
    if (tid < nchild) {
      int c = a.child_idx[cp0 + tid];
      int t = a.tokens[(int64_t)b * a.M + c];
      t = min(max(t, 0), V - 1);
      s_tok[tid] = t;
      s_dlog[tid] = drow[t];
    }
  } else {
#pragma unroll
    for (int j = 0; j < NCH; ++j) dv[j] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
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
    r_reg[j][0] = expf(tv[j].x - mt); r_reg[j][1] = expf(tv[j].y - mt);
    r_reg[j][2] = expf(tv[j].z - mt); r_reg[j][3] = expf(tv[j].w - mt);
    p_reg[j][0] = expf(dv[j].x - md); p_reg[j][1] = expf(dv[j].y - md);
    p_reg[j][2] = expf(dv[j].z - md); p_reg[j][3] = expf(dv[j].w - md);
    st += (r_reg[j][0] + r_reg[j][1]) + (r_reg[j][2] + r_reg[j][3]);
    sd += (p_reg[j][0] + p_reg[j][1]) + (p_reg[j][2] + p_reg[j][3]);
    *reinterpret_cast<float4*>(&r_lds[4 * (tid + kThreads * j)]) =
        make_float4(r_reg[j][0], r_reg[j][1], r_reg[j][2], r_reg[j][3]);
  }
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
    for (int e = 0; e < 4; ++e) p_reg[j][e] = __fmul_rn(p_reg[j][e], inv_sd);

  const int64_t nodebase = (int64_t)b * a.M;
  if (P == 0 && tid == 0) {  // row 0 is no drafted node: defined outputs
    if (a.decision) a.decision[nodebase] = 0;
    a.ws_decision[nodebase] = 0;
    if (a.ratio) a.ratio[nodebase] = 0.f;
    if (a.mass) a.mass[nodebase] = 0.f;
    if (a.n_agg) a.n_agg[nodebase] = 0;
    if (a.q_tok) a.q_tok[nodebase] = 0.f;
    if (a.p_tok) a.p_tok[nodebase] = 0.f;
  }

  // ---- children in static order, each against the current residual r
  for (int ci = 0; ci < nchild; ++ci) {
    const int c = a.child_idx[cp0 + ci];
    const int t = s_tok[ci];
    const float rt = r_lds[t];
    const float cap = a.lambda * rt;                 // bound: sum_A r < lambda * r(x^)   (Sec. 4)
    const int32_t* nrow = a.neigh + (int64_t)t * a.kstride;
    float carry = 0.f, mass_u = 0.f;
    int jstar = INT_MAX;
    int n_first = t;
    for (int base = 0; base < a.k; base += kThreads) {
      const int i = base + tid;
      int n = t;
      float v = 0.f;
      if (i < a.k) {
        if (i > 0) { n = nrow[i]; n = min(max(n, 0), V - 1); }
        v = r_lds[n];
      }
      if (base == 0) n_first = n;
      const float incl = wave_inclusive_scan(v, lane);
      if (lane == 63) s_wtot[w] = incl;
      __syncthreads();
      float prefix = carry, total = carry;
#pragma unroll
      for (int ww = 0; ww < kWaves; ++ww) {
        if (ww == w) prefix = total;
        total += s_wtot[ww];
      }
      const float C = prefix + incl;                 // prefix sum including slot i
      float prev = __shfl_up(incl, 1);
      const float excl = lane == 0 ? prefix : prefix + prev;   // = C of slot i-1
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
      const float qt = __fmul_rn(rt, rs), m = __fmul_rn(mass_u, rs);
      const float pt = __fmul_rn(expf(s_dlog[ci] - md), inv_sd);
      const float u = a.u_accept[nodebase + c];
      const uint8_t dec = (__fmul_rn(u, pt) < m) ? 1 : 0;   // u < min(1, mass / p(x^))
      a.ws_decision[nodebase + c] = dec;
      if (a.decision) a.decision[nodebase + c] = dec;
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
      res[j][0] = fmaxf(__fmul_rn(rv.x, rs) - p_reg[j][0], 0.f);
      res[j][1] = fmaxf(__fmul_rn(rv.y, rs) - p_reg[j][1], 0.f);
      res[j][2] = fmaxf(__fmul_rn(rv.z, rs) - p_reg[j][2], 0.f);
      res[j][3] = fmaxf(__fmul_rn(rv.w, rs) - p_reg[j][3], 0.f);
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

  // ---- draw from the final r by inverse CDF over ascending token index
  constexpr int EP = 4 * NCH;  // contiguous tokens per lane for the scan
  float d[EP];
  float local = 0.f;
  int lastpos = -1;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const float4 rv = *reinterpret_cast<const float4*>(&r_lds[tid * EP + 4 * j]);
    d[4 * j + 0] = rv.x; d[4 * j + 1] = rv.y; d[4 * j + 2] = rv.z; d[4 * j + 3] = rv.w;
  }
#pragma unroll
  for (int e = 0; e < EP; ++e) {
    local += d[e];
    if (d[e] > 0.f) lastpos = tid * EP + e;
  }
  const float incl = wave_inclusive_scan(local, lane);
  if (lane == 63) s_wtot[w] = incl;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, o));
  if (lane == 0) s_lastpos[w] = lastpos;
  __syncthreads();
  float prefix = 0.f, total = 0.f;
#pragma unroll
  for (int ww = 0; ww < kWaves; ++ww) {
    if (ww == w) prefix = total;
    total += s_wtot[ww];
  }
  const float target = __fmul_rn(a.u_final[nodebase + P], total);
  const float excl = prefix + incl - local;
  const bool hit = (prefix + incl) > target;
  const unsigned long long bal = __ballot(hit);
  if (bal) {
    const int fl = __ffsll((long long)bal) - 1;
    if (lane == fl) {
      // first token whose cumulative mass exceeds the target
      float run = 0.f;
      int x = tid * EP + EP - 1;
      bool found = false;
#pragma unroll
      for (int e = 0; e < EP; ++e) {
        run += d[e];
        if (!found && (excl + run) > target) { x = tid * EP + e; found = true; }
      }
      s_vidx[w] = x;
    }
  } else if (lane == 0) {
    s_vidx[w] = INT_MAX;
  }
  __syncthreads();
  if (tid == 0) {
    int x = INT_MAX, lp = -1;
    for (int ww = kWaves - 1; ww >= 0; --ww) {
      if (s_vidx[ww] != INT_MAX) x = s_vidx[ww];
      lp = max(lp, s_lastpos[ww]);
    }
    if (x == INT_MAX) x = lp >= 0 ? lp : 0;
    x = min(x, V - 1);
    a.ws_final[nodebase + P] = x;
    if (a.final_all) a.final_all[nodebase + P] = x;
  }
}

// Follow the first accepted child per level from the root (App. A.2: accepted
// tokens are kept, everything after the first rejection is discarded).
__global__ void walk_kernel(int B, int M, int depth, const int32_t* child_ptr, const int32_t* child_idx,
                            const uint8_t* decision, const int32_t* final_all, int32_t* accept_len,
                            int32_t* path, int32_t* final_token) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const uint8_t* dec = decision + (int64_t)b * M;
  int cur = 0, n = 0;
  while (true) {
    int nxt = -1;
    for (int ci = child_ptr[cur]; ci < child_ptr[cur + 1]; ++ci) {
      const int c = child_idx[ci];
      if (dec[c]) { nxt = c; break; }
    }
    if (nxt < 0 || n >= depth) break;
    path[(int64_t)b * depth + n] = nxt;
    ++n;
    cur = nxt;
  }
  for (int i = n; i < depth; ++i) path[(int64_t)b * depth + i] = -1;
  accept_len[b] = n;
  final_token[b] = final_all[(int64_t)b * M + cur];
}

template <int NCH, bool ALIGNED>
int32_t launch_rows(const VerifyArgs& a, int B, hipStream_t stream) {
  static bool attr_set = false;
  const size_t lds = (size_t)NCH * 4096 * sizeof(float);
  auto kern = verify_rows_kernel<NCH, ALIGNED>;
  if (!attr_set) {
    LPP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(B * a.M)), dim3(kThreads), lds, stream, a);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}

}  // namespace

extern "C" size_t lpp_relaxed_verify_workspace(const lpp_tree* tree, int32_t B, int32_t V, int32_t k) {
  (void)V; (void)k;
  if (!tree || B < 1) return 0;
  const size_t nodes = (size_t)B * tree->M;
  return lpp_align_up(nodes * sizeof(int32_t), 256) + lpp_align_up(nodes, 256);
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
  if (!tree->d_child_ptr) return LPP_EHIP;

  VerifyArgs a;
  a.target = target_logits; a.drafter = drafter_logits; a.ldv = ldv; a.off = vocab_offset;
  a.V = V; a.M = tree->M; a.kstride = kstride; a.k = k; a.lambda = lambda;
  a.tokens = tokens; a.neigh = neigh; a.u_accept = u_accept; a.u_final = u_final;
  a.child_ptr = tree->d_child_ptr; a.child_idx = tree->d_child_idx;
  a.decision = out->decision; a.ratio = out->ratio; a.mass = out->mass; a.n_agg = out->n_agg;
  a.q_tok = out->q_tok; a.p_tok = out->p_tok; a.final_all = out->final_tok_all;
  const size_t nodes = (size_t)B * tree->M;
  a.ws_final = reinterpret_cast<int32_t*>(ws);
  a.ws_decision = reinterpret_cast<uint8_t*>(ws) + lpp_align_up(nodes * sizeof(int32_t), 256);

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  auto aligned16 = [&](const float* p) {
    return p == nullptr || ((reinterpret_cast<uintptr_t>(p + vocab_offset) % 16 == 0) && (ldv % 4 == 0));
  };
  const bool al = aligned16(target_logits) && aligned16(drafter_logits);
  const int nch = V <= 4096 ? 1 : V <= 8192 ? 2 : V <= 16384 ? 4 : 8;
  int32_t st;
#define LPP_DISPATCH(N)                                              \
  st = al ? launch_rows<N, true>(a, B, s) : launch_rows<N, false>(a, B, s)
  switch (nch) {
    case 1: LPP_DISPATCH(1); break;
    case 2: LPP_DISPATCH(2); break;
    case 4: LPP_DISPATCH(4); break;
    default: LPP_DISPATCH(8); break;
  }
#undef LPP_DISPATCH
  if (st != LPP_OK) return st;
  const int depth = tree->depth > 0 ? tree->depth : 1;
  hipLaunchKernelGGL(walk_kernel, dim3((unsigned)((B + 63) / 64)), dim3(64), 0, s, B, tree->M, depth,
                     tree->d_child_ptr, tree->d_child_idx, a.ws_decision, a.ws_final, out->accept_len,
                     out->path, out->final_token);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}
