// Relaxed acceptance over a static draft tree: per-row vocabulary softmax,
// neighbour gather-sum under the multiplicative bound, ratio / accept test,
// residual update, inverse-CDF draw, and the walk (paper Sec. 4; Sec. 2.2;
// App. A.2 Eq. 1-2).
//
// One workgroup owns one tree row of one batch item.  The two logit rows are read
// from HBM exactly once, with every load issued before the first use; the row's
// current target distribution r lives in LDS (unnormalised, with a running scale
// rs) and in the registers of the lanes that own its tokens, the drafter
// distribution p in registers only.  Rows are independent: each is evaluated for
// the outcome "all earlier siblings were rejected", which needs no uniform.
//
// Per child the critical path is three workgroup barriers:
//   all      gather r at the child's k neighbours (two slots per lane, nearest first),
//            scan the sums inside each wave
//   barrier
//   all      add the wave totals in order, find the end of A, move A's mass onto x^
//   barrier
//   all      read their tokens of r' back from LDS, form [r' rs - p]_+ in place,
//            reduce its sum
//   barrier
// Barriers wait for LDS traffic only, so global stores stay in flight across
// them; what a child's test leaves behind is written to global memory once, after
// the row's draw.  Rows with the most children are given the lowest block indices.
// The walk: the last row of a batch item to finish (a ticket counter) follows the
// recorded decisions from the root; when the whole grid is resident at once, the
// block of the first row table entry collects the other rows' results instead
// (STAG below) and nobody takes a ticket.
//
// Variants of the same kernel (template switches, so that the plain build pays for none of them):
// FRONT  classifier-free guidance and top-k in front of the target softmax (App. B "Models");
// ALT    the other reading of two points the paper leaves open: A picked by passing over the
//        neighbours that would break the bound instead of stopping at the first one (wave 0 walks
//        the gathered values 64 at a time), and siblings that are distinct draws (a rejected token
//        leaves p, which is rescaled by 1 / (1 - p(x^))).
// STAG   the build for a grid that is resident at once (one row per compute unit): rows hold
//        their logit loads back by chain length, and the walk is done by a wave of the longest
//        row's block beside that row's draw (collect_and_walk).
// The additive bound of the earlier LANTERN method is a run-time choice of the cap.
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "lpp_internal.h"

namespace {

constexpr int kMaxStage = 8;       // neighbour lists of the first children kept in LDS
constexpr int kStageSmall = 4;     // ... when two rows per compute unit have to fit
constexpr float kLog2e = 1.44269504088896340736f;

// By-value kernel argument, indexed by a wave-uniform value only (scalar loads).  Entry i
// describes the row handled by blocks [i B, (i+1) B): rows are sorted by descending number of
// children.  row | nchild << 8 | first child row << 16 | offset into child_idx << 24.
struct TreeTab {
  uint32_t rowinfo[LPP_MAX_ROWS];
};

struct VerifyArgs {
  const float* target;    // with a sampling front end: the text-conditioned rows
  const float* uncond;    // null-conditioned rows of the target, or null (no guidance)
  const float* drafter;
  float cfg_scale;        // guidance scale s: l = u + s (c - u)
  int32_t top_k;          // keep the top_k largest guided logits of a row (0: keep all)
  int64_t ldv;
  int32_t off, V, M, B, kstride, k, depth;
  int32_t nstage;         // child lists whose first pass is staged in LDS (<= kMaxStage)
  int32_t n_parents;      // rows with children (they come first in the row table)
  int32_t wait_parent, wait_leaf;   // what a row holds its loads back per parent / leaf entry ahead of it (1/256 of 1024 clocks)
  float lambda;           // bound factor, or delta when `additive`
  int32_t additive;       // 0: sum_A r < lambda r(x^)   1: sum_A r < delta
  int32_t skip;           // A: 0 longest nearest-first prefix, 1 neighbours that would break the bound are passed over
  int32_t norepl;         // siblings: 0 i.i.d. draws from p, 1 distinct tokens (a rejected token leaves p)
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
  int32_t spin_limit;     // (whole grid resident) how often the walking block asks for the other rows' words
  const int32_t* child_idx;   // [N] children of all rows, grouped by parent (read only if !consecutive)
  int32_t consecutive;    // every row's children are consecutive rows
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
// N scans side by side, step by step: the steps of one scan depend on each other, those of
// different scans do not, so their latencies overlap.
template <int N>
__device__ __forceinline__ void wave_inclusive_scan_n(float (&v)[N]) {
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_or<0x111, 0xf>(0.f, v[j]);
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_or<0x112, 0xf>(0.f, v[j]);
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_or<0x114, 0xf>(0.f, v[j]);
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_or<0x118, 0xf>(0.f, v[j]);
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_or<0x142, 0xa>(0.f, v[j]);
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_or<0x143, 0xc>(0.f, v[j]);
}
// Inclusive scan of non-negative values that is non-decreasing over the lanes.
// The tree above adds in a different order per lane, so neighbouring results can
// be out of order by a rounding; a running maximum puts them back in order.
__device__ __forceinline__ float wave_monotone_scan(float v) {
  v = wave_inclusive_scan(v);
  // (non-negative floats order like their bit patterns: an integer maximum, which the DPP forms take directly)
  uint32_t u = __float_as_uint(v);
  u = max(u, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u, 0x111, 0xf, 0xf, false));
  u = max(u, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u, 0x112, 0xf, 0xf, false));
  u = max(u, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u, 0x114, 0xf, 0xf, false));
  u = max(u, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u, 0x118, 0xf, 0xf, false));
  u = max(u, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u, 0x142, 0xa, 0xf, false));
  u = max(u, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u, 0x143, 0xc, 0xf, false));
  return __uint_as_float(u);
}
__device__ __forceinline__ float wave_prev_lane(float v, float first) {   // lane i <- lane i-1
  return dpp_or<0x138, 0xf>(first, v);                                      // wave_shr:1
}
__device__ __forceinline__ float lane_value(float v, int lane) {           // `lane` is wave-uniform
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float wave_sum(float v) { return lane_value(wave_inclusive_scan(v), 63); }
__device__ __forceinline__ float wave_max(float v) {
  const float ninf = -INFINITY;
  v = fmaxf(v, dpp_or<0x111, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x112, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x114, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x118, 0xf>(ninf, v));
  v = fmaxf(v, dpp_or<0x142, 0xa>(ninf, v));
  v = fmaxf(v, dpp_or<0x143, 0xc>(ninf, v));
  return lane_value(v, 63);
}

// Workgroup barrier that orders LDS traffic only: outstanding global loads and
// stores of the wave are not waited for.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// exp(x - m) as exp2(x * log2(e) + m2), m2 = -m * log2(e): one FMA and the hardware exp2.
__device__ __forceinline__ float exp2_fma(float x, float m2) {
  return __builtin_amdgcn_exp2f(__builtin_fmaf(x, kLog2e, m2));
}

// Four consecutive logits of a row, tokens e0 .. e0+3.  The load is unconditional and in
// bounds (clamped address); mask_logits4 afterwards turns tokens at or past V into -inf.
// The two are separate so that nothing consumes a load while others are still to be issued.
// ALIGNED: 16-byte aligned rows and V % 4 == 0.
template <bool ALIGNED>
__device__ __forceinline__ float4 load_logits4(const float* row, int e0, int V) {
  if (ALIGNED) {
    typedef float vec4f __attribute__((ext_vector_type(4)));
    const vec4f x = __builtin_nontemporal_load(reinterpret_cast<const vec4f*>(row + min(e0, V - 4)));
    return make_float4(x.x, x.y, x.z, x.w);
  }
  float4 v;
  v.x = __builtin_nontemporal_load(row + min(e0 + 0, V - 1));
  v.y = __builtin_nontemporal_load(row + min(e0 + 1, V - 1));
  v.z = __builtin_nontemporal_load(row + min(e0 + 2, V - 1));
  v.w = __builtin_nontemporal_load(row + min(e0 + 3, V - 1));
  return v;
}
__device__ __forceinline__ float4 mask_logits4(float4 v, int e0, int V) {
  const float ninf = -INFINITY;
  return make_float4(e0 + 0 < V ? v.x : ninf, e0 + 1 < V ? v.y : ninf, e0 + 2 < V ? v.z : ninf,
                     e0 + 3 < V ? v.w : ninf);
}

// The tail both walks share: wd[q] = parent << 1 | decision of row lane + 64 q (0 for rows that do
// not exist).  Children are tried in ascending row index, so the child a row hands over to is its
// lowest accepted one: next[parent] = min over accepted children, then one lane follows next[]
// from the root.  Returns (to lane 0) the row the path ends on.
__device__ __forceinline__ int follow_accepted(const int (&wd)[LPP_MAX_ROWS / 64], int M, int depth, int lane, int* s_next,
                                               int32_t* accept_len, int32_t* path) {
#pragma unroll
  for (int q = 0; q < LPP_MAX_ROWS / 64; ++q) {
    const int i = lane + 64 * q;
    if (i >= 1 && i < M && (wd[q] & 1)) atomicMin(&s_next[wd[q] >> 1], i);
  }
  wave_lds_sync();
  int cur = 0;
  if (lane == 0) {
    int n = 0;
    while (n < depth) {
      const int nxt = s_next[cur];
      if (nxt == INT_MAX) break;
      path[n++] = nxt;
      cur = nxt;
    }
    for (int i = n; i < depth; ++i) path[i] = -1;
    *accept_len = n;
  }
  return cur;
}

// Follow the first accepted child per level from the root (App. A.2: accepted
// tokens are kept, everything after the first rejection is discarded).  One wave.
// word[i] = parent(i) << 1 | decision(i) as the row kernels recorded it; s_next is M ints
// of LDS, s_fin another M.  Children are tried in ascending row index, so the child a
// row hands over to is the lowest accepted one.
__device__ __forceinline__ void walk_wave(const int32_t* word, const int32_t* fin, int M, int depth, int lane,
                                          int* s_next, int* s_fin, int32_t* accept_len, int32_t* path,
                                          int32_t* final_token) {
  int wd[LPP_MAX_ROWS / 64];
#pragma unroll
  for (int q = 0; q < LPP_MAX_ROWS / 64; ++q) {
    const int i = lane + 64 * q;
    wd[q] = 0;
    if (i < M) {
      wd[q] = __hip_atomic_load(&word[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_fin[i] = __hip_atomic_load(&fin[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_next[i] = INT_MAX;
    }
  }
  wave_lds_sync();
  const int cur = follow_accepted(wd, M, depth, lane, s_next, accept_len, path);
  if (lane == 0) *final_token = s_fin[cur];
}

// Walk of one item when the whole grid is resident at once (one wave of the block that walks).
// Every other row of the item leaves its words -- (parent << 1 | decision) per child, its draw --
// in `mail` (device-scope stores), this wave asks for them until none is missing and walks as
// above.  Nobody waits for this block, so the wait ends as soon as the other blocks have run; it
// is bounded all the same (`spin_limit` rounds of loads): when the bound is hit the item's
// accept_len, path and final token are set to -1 and the count in mail[kMailGaveUp] goes up.
//
// Words carry a tag in their upper bits (kMailTagShift) that changes from call to call, so a
// word that arrives after its call's walk gave up is not taken for the next call's, and nothing
// has to be cleared between calls.  Every row block, the walking one too, owns one word of the
// mail (its draw's); it reads the tag that word holds when it starts -- the one its own last call
// left there, calls on one handle being ordered on a stream -- and uses the next one (1..1023
// round and round; memory that was zeroed holds tag 0, which no call uses) for everything it
// sends.  All rows of an item therefore step through the same tags, call after call.
// s_own: [M] words of this block's own children, -1 elsewhere; s_next, s_fin: M ints each;
// *s_end: row the path ended on (-1: failed), for the wave that holds this block's own draw.
// The first round of loads is issued by the caller ahead of time (mail_fetch), so that it is in
// flight while this wave still has other work.
constexpr int kMailTagShift = 20;                    // payloads are below 2^20 (row << 1 | decision; a token)
constexpr uint32_t kMailPayload = (1u << kMailTagShift) - 1u;
// The tag that follows the one in `last_word`, in place.
__device__ __forceinline__ uint32_t next_tag(uint32_t last_word) {
  const uint32_t last_tag = last_word >> kMailTagShift;
  return (last_tag >= 1023u ? 1u : last_tag + 1u) << kMailTagShift;
}
struct MailRound {
  int w[LPP_MAX_ROWS / 64], f[LPP_MAX_ROWS / 64];
};
__device__ __forceinline__ void mail_fetch(MailRound& r, const int32_t* mail, int64_t nodebase, int M, int lane) {
#pragma unroll
  for (int q = 0; q < LPP_MAX_ROWS / 64; ++q) {       // all loads of a round in flight together
    const int ic = min(lane + 64 * q, M - 1);
    r.w[q] = __hip_atomic_load(&mail[nodebase + ic], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    r.f[q] = __hip_atomic_load(&mail[LPP_MAX_ROWS + nodebase + ic], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ __forceinline__ void collect_and_walk(MailRound r, int32_t* mail, uint32_t tagw, int64_t nodebase, int M,
                                                 int depth, int P, int spin_limit, int lane, const int* s_own,
                                                 int* s_next, int* s_fin, int* s_end, int32_t* accept_len,
                                                 int32_t* path, int32_t* final_token) {
  constexpr int Q = LPP_MAX_ROWS / 64;
  int wd[Q], fn[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int i = lane + 64 * q;
    wd[q] = (i >= 1 && i < M) ? s_own[i] : 0;
    fn[q] = (i < M && i != P) ? -1 : 0;
  }
  bool ok = false;
  // (a negative limit makes the walk give up at once: the host's way to exercise that path)
  if (spin_limit >= 0) {
    for (int spin = 0;; ++spin) {
      bool missing = false;
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        if (wd[q] == -1 && ((uint32_t)r.w[q] & ~kMailPayload) == tagw) wd[q] = (int)((uint32_t)r.w[q] & kMailPayload);
        if (fn[q] == -1 && ((uint32_t)r.f[q] & ~kMailPayload) == tagw) fn[q] = (int)((uint32_t)r.f[q] & kMailPayload);
        missing = missing || wd[q] == -1 || fn[q] == -1;
      }
      if (!__ballot(missing)) { ok = true; break; }
      if (spin >= spin_limit) break;
      __builtin_amdgcn_s_sleep(4);
      mail_fetch(r, mail, nodebase, M, lane);
    }
  }
  if (!ok) {
    if (lane == 0) {
      __hip_atomic_fetch_add(&mail[kMailGaveUp], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (int i = 0; i < depth; ++i) path[i] = -1;
      *accept_len = -1;
      *final_token = -1;
      *s_end = -1;
    }
    return;
  }
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int i = lane + 64 * q;
    if (i < M) {
      s_fin[i] = fn[q];
      s_next[i] = INT_MAX;
    }
  }
  wave_lds_sync();
  const int cur = follow_accepted(wd, M, depth, lane, s_next, accept_len, path);
  if (lane == 0) {
    if (cur != P) *final_token = s_fin[cur];      // (ended on this block's own row: its draw is with wave 0)
    *s_end = cur;
  }
}

// Sum (max), in wave order, of one float per wave held in LDS; every wave
// computes the same value the same way.
// WIDE: two broadcast reads and seven additions, a shorter chain than the row shifts (for the
// build that has eight registers to spare).
template <int NW, bool WIDE = false>
__device__ __forceinline__ float combine_sum(const float* s_w, int lane) {
  if (WIDE && NW == 8) {
    const float4 a = *reinterpret_cast<const float4*>(s_w), b = *reinterpret_cast<const float4*>(s_w + 4);
    return ((((((a.x + a.y) + a.z) + a.w) + b.x) + b.y) + b.z) + b.w;
  }
  float x = lane < NW ? s_w[lane] : 0.f;
  x += dpp_or<0x111, 0xf>(0.f, x);
  x += dpp_or<0x112, 0xf>(0.f, x);
  x += dpp_or<0x114, 0xf>(0.f, x);
  x += dpp_or<0x118, 0xf>(0.f, x);
  return lane_value(x, NW - 1);
}
template <int NW>
__device__ __forceinline__ float combine_max(const float* s_w, int lane) {
  float x = lane < NW ? s_w[lane] : -INFINITY;
  x = fmaxf(x, dpp_or<0x111, 0xf>(-INFINITY, x));
  x = fmaxf(x, dpp_or<0x112, 0xf>(-INFINITY, x));
  x = fmaxf(x, dpp_or<0x114, 0xf>(-INFINITY, x));
  x = fmaxf(x, dpp_or<0x118, 0xf>(-INFINITY, x));
  return lane_value(x, NW - 1);
}

// NT lanes per block, NCH float4 chunks per lane: a row holds at most NT * NCH * 4
// tokens.  Lane `tid` owns tokens 4*(tid + NT*j) .. +3 for j < NCH.  In token order
// the row is therefore a sequence of NCH * NW cells of 256 tokens, cell j * NW + w
// owned by wave w.  The neighbour list of a child is taken in passes of 2 NT slots,
// lane `tid` holding slots 2 tid and 2 tid + 1 of the pass.
// FRONT: classifier-free guidance and top-k in front of the target softmax (paper App. B "Models").
// ALT: the build that also knows the other readings of A and of the sibling scheme
// (VerifyArgs::skip, ::norepl); the plain build does not carry their registers and LDS.
// STAG: rows hold their logit loads back by their place in the row table (see the kernel body): a
// build of its own, because the waits force another order of the first loads.
template <int NT, int NCH, bool ALIGNED, bool FRONT, bool ALT, bool STAG>
// (The plain build is held to 128 registers -- four waves per SIMD, two rows per compute unit: one
// register more would halve that, which costs far more than a spill.)
__global__ __launch_bounds__(NT, (STAG || ALT || FRONT || NT > 512) ? 1 : 4) void verify_rows_kernel(VerifyArgs a, TreeTab tt) {
  constexpr int NW = NT / 64;
  constexpr int NC = NCH * NW;             // cells
  constexpr int CPL = (NC + 63) / 64;      // cells per lane of wave 0 in the final draw
  constexpr int PASS = 2 * NT;             // neighbour slots per pass
  constexpr int MAXP = (LPP_MAX_K + PASS - 1) / PASS;
  constexpr int ZC = NT * NCH * 4;         // index of a cell of r_lds that always holds 0
  extern __shared__ __align__(16) unsigned char smem[];
  float* r_lds = reinterpret_cast<float*>(smem);                              // current r, then the zero cell
  uint32_t* s_neigh = reinterpret_cast<uint32_t*>(r_lds + ZC + 4);            // [nstage][NT] pairs of 16-bit slots
  float* s_val = reinterpret_cast<float*>(s_neigh + a.nstage * NT);           // ALT: [PASS] gathered values of a pass
  uint32_t* s_incl = reinterpret_cast<uint32_t*>(s_val + PASS);               // ALT: [PASS / 32] membership bits
  __shared__ __align__(16) float s_max[2][NW];
  __shared__ __align__(16) float s_sum[2][NW];
  __shared__ __align__(16) float s_z[2][NW];
  __shared__ float s_wtot[2][NW];
  __shared__ float s_cell[64 * CPL];
  __shared__ int s_tok[LPP_MAX_ROWS];
  __shared__ int s_child[LPP_MAX_ROWS];
  __shared__ float s_dlog[LPP_MAX_ROWS];
  __shared__ float s_u[LPP_MAX_ROWS];
  __shared__ int s_jstar;
  __shared__ int s_ncand;
  __shared__ uint32_t s_tau;
  __shared__ float s_mass;
  // (whole grid resident) the walking block: words of its own children, next[], finals, end of the path
  __shared__ int s_mail[STAG ? 3 * LPP_MAX_ROWS + 1 : 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.x % a.B;
  const uint32_t ri = tt.rowinfo[blockIdx.x / a.B];
  const int P = ri & 255u;
  const int V = a.V, k = a.k;
  const int64_t nodebase = (int64_t)b * a.M;
  const int64_t rowoff = (nodebase + P) * a.ldv + a.off;
  const float* trow = a.target + rowoff;
  const int nchild = (ri >> 8) & 255u;               // < LPP_MAX_ROWS <= NT
  const int first_child = (ri >> 16) & 255u, cp0 = ri >> 24;
  const float* drow = nchild > 0 ? a.drafter + rowoff : nullptr;
  const int nst = min(nchild, a.nstage);
  // When the whole grid is resident at once there are no tickets: the block of the first table
  // entry (most children, as a rule the last to finish) collects the other rows' words itself,
  // in a wave of its own beside the draw, and walks.  The other rows never wait for anybody.
  const bool walker = STAG && blockIdx.x < (unsigned)a.B;
  if (STAG && walker && tid < a.M) s_mail[tid] = -1;        // (read after several barriers)

  int crow[kMaxStage], stok[kMaxStage];
#pragma unroll
  for (int ci = 0; ci < kMaxStage; ++ci) {
    crow[ci] = first_child + ci;
    if (!a.consecutive && ci < nchild) crow[ci] = a.child_idx[cp0 + ci];
  }
  if (STAG) {
    // When the whole grid is resident at once, every row asks for its logits in the same
    // microsecond and the memory system serves them all at the same pace: the row with the longest
    // chain of children then starts as late as a leaf.  Here rows with shorter chains hold their
    // loads back (the host turns the bytes asked for ahead of a row -- the table is sorted by
    // children, parents first -- into a wait), so that the long chains get theirs first.  The wait
    // is a sum of fixed sleeps (units of 1024 clocks): no loop stands before the loads.
    // The drafted tokens, first link of the chain token -> neighbour list, are asked for before the
    // wait as vector loads at one address for all lanes (unconditional, so that they return in
    // order ahead of the rows): behind a sleep the compiler no longer makes them scalar loads, and
    // scalar loads issued before it would have the row loads wait for them.
    const int e_sorted = blockIdx.x / a.B;
    const uint32_t wt = (uint32_t)__builtin_amdgcn_readfirstlane(
        min((min(e_sorted, a.n_parents) * a.wait_parent + max(e_sorted - a.n_parents, 0) * a.wait_leaf) >> 8, 31));
    int lane_zero = 0;
    asm("" : "+v"(lane_zero));       // (opaque to the compiler: keeps these loads on the vector path)
#pragma unroll
    for (int ci = 0; ci < kMaxStage; ++ci) stok[ci] = a.tokens[nodebase + min(crow[ci], a.M - 1) + lane_zero];
    if (wt & 1u) __builtin_amdgcn_s_sleep(16);
    if (wt & 2u) __builtin_amdgcn_s_sleep(32);
    if (wt & 4u) __builtin_amdgcn_s_sleep(64);
    if (wt & 8u) { __builtin_amdgcn_s_sleep(64); __builtin_amdgcn_s_sleep(64); }
    if (wt & 16u) { __builtin_amdgcn_s_sleep(127); __builtin_amdgcn_s_sleep(127); __builtin_amdgcn_s_sleep(2); }
  }
  // ---- every HBM read of the two rows is issued first: nothing else is as long
  float4 tv[NCH], dv[NCH], uv[FRONT ? NCH : 1];
#pragma unroll
  for (int j = 0; j < NCH; ++j) tv[j] = load_logits4<ALIGNED>(trow, 4 * (tid + NT * j), V);
  if (FRONT && a.uncond) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) uv[FRONT ? j : 0] = load_logits4<ALIGNED>(a.uncond + rowoff, 4 * (tid + NT * j), V);
  }
  if (nchild > 0) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) dv[j] = load_logits4<ALIGNED>(drow, 4 * (tid + NT * j), V);
  } else {
#pragma unroll
    for (int j = 0; j < NCH; ++j) dv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // ---- the chain row -> drafted tokens -> neighbour lists.  The tokens of the first
  // children sit at wave-uniform addresses (scalar loads, which do not queue behind the rows).
  const float u_fin = a.u_final[nodebase + P];
#pragma unroll
  for (int ci = 0; ci < kMaxStage; ++ci) {
    if (STAG) {
      stok[ci] = ci < nchild ? min(max(__builtin_amdgcn_readfirstlane(stok[ci]), 0), V - 1) : 0;
    } else {
      stok[ci] = 0;
      if (ci < nchild) stok[ci] = min(max(a.tokens[nodebase + crow[ci]], 0), V - 1);
    }
  }
  int my_tok = 0, my_child = 0;
#pragma unroll
  for (int ci = 0; ci < kMaxStage; ++ci)
    if (tid == ci) { my_tok = stok[ci]; my_child = crow[ci]; }
  if (nchild > kMaxStage && tid >= kMaxStage && tid < nchild) {     // rows with many children: a slower chain
    my_child = a.consecutive ? first_child + tid : a.child_idx[cp0 + tid];
    my_tok = min(max(a.tokens[nodebase + my_child], 0), V - 1);
  }
  float my_u = 0.f, my_dlog = 0.f;
  if (tid < nchild) {
    my_u = a.u_accept[nodebase + my_child];
    my_dlog = drow[my_tok];
  }
  int nreg[kMaxStage][2];      // slots tid and tid + NT of the first pass (lists that are not
#pragma unroll                 // staged re-read the first child's: no branch, no extra traffic)
  for (int ci = 0; ci < kMaxStage; ++ci) {
    const int32_t* nrow = a.neigh + (int64_t)(ci < nst ? stok[ci] : stok[0]) * a.kstride;
    nreg[ci][0] = nrow[min(tid, k - 1)];
    nreg[ci][1] = nrow[min(tid + NT, k - 1)];
  }

  __builtin_amdgcn_sched_barrier(0);   // every load above is issued before anything below waits
  const bool full_row = V == NT * NCH * 4;   // no token of the block's range lies past the vocabulary

  // ---- sampling front end of the target row (App. B "Models": guidance scale, top-k): the
  // guided logit l = u + s (c - u) in float32, difference, product and sum each rounded once; then
  // only the top_k largest of the row stay (ties with the k-th stay too), the rest becomes -inf
  if (FRONT) {
    const bool guide = a.uncond != nullptr;
    uint32_t key[NCH][4];       // order-preserving integer image of the guided logits
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      float c[4] = {tv[j].x, tv[j].y, tv[j].z, tv[j].w};
      const float u[4] = {uv[FRONT ? j : 0].x, uv[FRONT ? j : 0].y, uv[FRONT ? j : 0].z, uv[FRONT ? j : 0].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float l = c[e];
        if (guide) {
          const float g = c[e] - u[e];
          const float sg = a.cfg_scale * g;
          l = u[e] + sg;
          if (c[e] == -INFINITY) l = -INFINITY;
        }
        if (4 * (tid + NT * j) + e >= V) l = -INFINITY;
        c[e] = l;
        const uint32_t b = __float_as_uint(l);
        key[j][e] = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
      }
      tv[j] = make_float4(c[0], c[1], c[2], c[3]);
    }
    if (a.top_k > 0 && a.top_k < V) {
      // The top_k-th largest key.  Fast way: 2048 bins spread evenly over the row's range of values
      // (a monotone map, so whole bins lie above or below the one that holds the answer; spread
      // values mean few collisions in the LDS histogram), then an exact rank among the few keys of
      // that bin.  If that bin is crowded (many equal values), a radix select over the key bits
      // does the same exactly, only slower.  Histograms live in the LDS that r will occupy later.
      uint32_t* hist = reinterpret_cast<uint32_t*>(smem);          // [2048]
      uint32_t* cand = hist + 2048;                                // [kCand]
      constexpr int kCand = 256;
      uint32_t prefix = 0;
      bool done = false;
      {
        float lo = INFINITY, hi = -INFINITY;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
          const float c[4] = {tv[j].x, tv[j].y, tv[j].z, tv[j].w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (c[e] > -INFINITY && c[e] < INFINITY) { lo = fminf(lo, c[e]); hi = fmaxf(hi, c[e]); }
        }
        lo = -wave_max(-lo);
        hi = wave_max(hi);
        if (lane == 0) { s_max[0][w] = -lo; s_max[1][w] = hi; }
        for (int i = tid; i < 2048; i += NT) hist[i] = 0u;
        if (tid == 0) { s_ncand = 0; s_tau = 0u; }
        lds_barrier();
        lo = -combine_max<NW>(s_max[0], lane);
        hi = combine_max<NW>(s_max[1], lane);
        const float scale = hi > lo ? 2047.0f / (hi - lo) : 0.f;
        int bin[NCH][4];
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
          const float c[4] = {tv[j].x, tv[j].y, tv[j].z, tv[j].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float x = (c[e] - lo) * scale;                 // monotone in c; -inf, NaN -> bin 0
            bin[j][e] = x >= 2047.f ? 2047 : (x >= 0.f ? (int)x : 0);
            atomicAdd(&hist[bin[j][e]], 1u);
          }
        }
        lds_barrier();
        int cnt[32];
        int local = 0;
#pragma unroll
        for (int i = 0; i < 32; ++i) { cnt[i] = (int)hist[2047 - 32 * lane - i]; local += cnt[i]; }
        int incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int t = __shfl_up(incl, o);
          if (lane >= o) incl += t;
        }
        const unsigned long long bal = __ballot(incl >= a.top_k);
        const int fl = bal ? __ffsll((long long)bal) - 1 : 63;
        int bstar = 0, above = 0, inbin = 0;
        if (lane == fl) {
          int run = incl - local;
          bstar = max(2047 - 32 * lane - 31, 0);
          above = run;
#pragma unroll
          for (int i = 0; i < 32; ++i) {
            if (run + cnt[i] >= a.top_k) { bstar = 2047 - 32 * lane - i; above = run; inbin = cnt[i]; break; }
            run += cnt[i];
          }
        }
        bstar = __shfl(bstar, fl); above = __shfl(above, fl); inbin = __shfl(inbin, fl);
        const int need = a.top_k - above;                        // rank inside bin bstar, from the top
        if (inbin <= kCand) {                                    // uniform
#pragma unroll
          for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (bin[j][e] == bstar) cand[atomicAdd(&s_ncand, 1)] = key[j][e];
          lds_barrier();
          const int n = s_ncand;
          for (int i = tid; i < n; i += NT) {
            const uint32_t ki = cand[i];
            int gt = 0, ge = 0;
            for (int q = 0; q < n; ++q) { gt += cand[q] > ki; ge += cand[q] >= ki; }
            if (gt < need && need <= ge) s_tau = ki;             // (equal keys write the same value)
          }
          lds_barrier();
          prefix = s_tau;
          done = true;
        }
        lds_barrier();                                           // histogram and list are free again
      }
      if (!done) {
        int need = a.top_k;
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
          const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
          const int bits = pass == 2 ? 10 : 11;
          const int nb = 1 << bits;
          for (int i = tid; i < 2048; i += NT) hist[i] = 0u;
          lds_barrier();
#pragma unroll
          for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const bool in = pass == 0 || (key[j][e] >> (shift + bits)) == (prefix >> (shift + bits));
              if (in) atomicAdd(&hist[(key[j][e] >> shift) & (nb - 1)], 1u);
            }
          lds_barrier();
          // every wave walks the bins from the top (32 per lane) and finds the one holding the need-th key
          int cnt[32];
          int local = 0;
#pragma unroll
          for (int i = 0; i < 32; ++i) {
            const int b = 2047 - 32 * lane - i;
            cnt[i] = b < nb ? (int)hist[b] : 0;
            local += cnt[i];
          }
          int incl = local;
#pragma unroll
          for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
          }
          const unsigned long long bal = __ballot(incl >= need);
          const int fl = bal ? __ffsll((long long)bal) - 1 : 63;
          int found = 0, above = 0;
          if (lane == fl) {
            int run = incl - local;
            found = max(2047 - 32 * lane - 31, 0);
            above = run;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
              if (run + cnt[i] >= need) { found = 2047 - 32 * lane - i; above = run; break; }
              run += cnt[i];
            }
          }
          found = __shfl(found, fl);
          above = __shfl(above, fl);
          prefix |= (uint32_t)found << shift;
          need -= above;
          lds_barrier();            // the histogram is cleared again (or handed over to r) after this
        }
      }
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        if (key[j][0] < prefix) tv[j].x = -INFINITY;
        if (key[j][1] < prefix) tv[j].y = -INFINITY;
        if (key[j][2] < prefix) tv[j].z = -INFINITY;
        if (key[j][3] < prefix) tv[j].w = -INFINITY;
      }
    }
  }

  // ---- softmax statistics of both rows (Sec. 2 notation: q target, p drafter; T = 1)
  float mt = -INFINITY, md = -INFINITY;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    if (!full_row && !FRONT) tv[j] = mask_logits4(tv[j], 4 * (tid + NT * j), V);
    if (!full_row || nchild == 0) dv[j] = mask_logits4(dv[j], 4 * (tid + NT * j), nchild > 0 ? V : 0);
    mt = fmaxf(mt, fmaxf(fmaxf(tv[j].x, tv[j].y), fmaxf(tv[j].z, tv[j].w)));
    md = fmaxf(md, fmaxf(fmaxf(dv[j].x, dv[j].y), fmaxf(dv[j].z, dv[j].w)));
  }
  mt = wave_max(mt);
  md = wave_max(md);
  if (lane == 0) { s_max[0][w] = mt; s_max[1][w] = md; }
  lds_barrier();
  mt = combine_max<NW>(s_max[0], lane);
  md = combine_max<NW>(s_max[1], lane);
  if (mt == -INFINITY) mt = 0.f;
  if (md == -INFINITY) md = 0.f;
  const float mt2 = -mt * kLog2e, md2 = -md * kLog2e;   // exp(x - m) = exp2(x*log2e - m*log2e)

  float p_reg[NCH][4];
  float st = 0.f, sd = 0.f;
  // STAG: the sums of my chunks of the current r, as the last pass over the row left them: the
  // draw's cell sums come from these instead of from another read of the row
  float csum[STAG ? NCH : 1];
  bool csum_valid = STAG;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const float r0 = exp2_fma(tv[j].x, mt2), r1 = exp2_fma(tv[j].y, mt2);
    const float r2 = exp2_fma(tv[j].z, mt2), r3 = exp2_fma(tv[j].w, mt2);
    p_reg[j][0] = exp2_fma(dv[j].x, md2); p_reg[j][1] = exp2_fma(dv[j].y, md2);
    p_reg[j][2] = exp2_fma(dv[j].z, md2); p_reg[j][3] = exp2_fma(dv[j].w, md2);
    if (STAG) csum[j] = (r0 + r1) + (r2 + r3);
    st += (r0 + r1) + (r2 + r3);
    sd += (p_reg[j][0] + p_reg[j][1]) + (p_reg[j][2] + p_reg[j][3]);
    *reinterpret_cast<float4*>(&r_lds[4 * (tid + NT * j)]) = make_float4(r0, r1, r2, r3);
  }
  st = wave_sum(st);
  sd = wave_sum(sd);
  if (lane == 0) { s_sum[0][w] = st; s_sum[1][w] = sd; }
  if (tid == 0) r_lds[ZC] = 0.f;
  // per child: token, row, drafter logit, uniform, and the first pass of its neighbour list
  // as 16-bit indices into r_lds (slot 0 = x^ itself; slots past k point at the zero cell)
  if (tid < nchild) { s_tok[tid] = my_tok; s_child[tid] = my_child; s_dlog[tid] = my_dlog; s_u[tid] = my_u; }
#pragma unroll
  for (int ci = 0; ci < kMaxStage; ++ci)
    if (ci < nst) {
      uint16_t* dst = reinterpret_cast<uint16_t*>(s_neigh + ci * NT);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const int slot = tid + NT * s;
        int n = min(max(nreg[ci][s], 0), V - 1);
        if (slot == 0) n = stok[ci];
        if (slot >= k) n = ZC;
        dst[slot] = (uint16_t)n;
      }
    }
  lds_barrier();
  st = combine_sum<NW>(s_sum[0], lane);
  sd = combine_sum<NW>(s_sum[1], lane);
  float rs = st > 0.f ? 1.0f / st : 0.f;           // r_true = r_lds * rs
  const float inv_sd = sd > 0.f ? 1.0f / sd : 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) p_reg[j][e] = p_reg[j][e] * inv_sd;

  // ---- children in static order, each against the current residual r
  int tog = 0;
  float pscale = 1.f;        // ALT, distinct siblings: p = p_reg * pscale once rejected tokens have left p
  // What a child's test leaves behind is kept by lane `ci` of the block and written out for up to
  // 64 children at once when the loop is over (by wave 0 after the draw; waves that own children
  // 64 and up, before they leave): the per-child chain below then carries no global stores.
  float k_m = 0.f, k_qt = 0.f, k_pt = 0.f;
  int k_j = 0;
  uint32_t tagw = 0;         // (whole grid resident) this call's tag, in place for the mail words
  auto write_children = [&](int first, int count) {
    if (lane < count) {
      const int cc = first + lane;
      const int c = s_child[cc];
      const float pt = ALT ? k_pt : exp2_fma(s_dlog[cc], md2) * inv_sd;   // p(x^): the drafter's probability of the token
      const int dec = (s_u[cc] * pt < k_m) ? 1 : 0;                        // u < min(1, mass / p(x^))
      // what the walk needs of this node: a device-scope store, visible to every compute unit
      // once it has completed (no cache write-back needed before the ticket, or for the block that walks)
      if (!(STAG && walker))
        __hip_atomic_store(&a.ws_decision[nodebase + c], (int)(tagw | (uint32_t)((P << 1) | dec)), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      if (a.decision) a.decision[nodebase + c] = (uint8_t)dec;
      if (a.ratio) a.ratio[nodebase + c] = k_m / pt;
      if (a.mass) a.mass[nodebase + c] = k_m;
      if (a.n_agg) a.n_agg[nodebase + c] = k_j;
      if (a.q_tok) a.q_tok[nodebase + c] = k_qt;
      if (a.p_tok) a.p_tok[nodebase + c] = pt;
    }
  };
  // Token and first-pass operands of the child about to be taken.  They are fetched ahead of its
  // turn: token and slot indices while the previous child's residual is formed, the values of r
  // right behind the barrier that ends it and before that residual's sum is known (r is read
  // again in the rare case that the sum turns out empty and r is put back).
  auto first_slots = [&](int cj, int tj) -> uint32_t {
    if (cj < nst) return s_neigh[cj * NT + tid];
    const int32_t* nrow = a.neigh + (int64_t)tj * a.kstride;
    const int sl0 = 2 * tid;
    const int x0 = nrow[min(sl0, k - 1)], x1 = nrow[min(sl0 + 1, k - 1)];
    int n0 = min(max(x0, 0), V - 1), n1 = min(max(x1, 0), V - 1);
    if (sl0 == 0) n0 = tj;
    if (sl0 >= k) n0 = ZC;
    if (sl0 + 1 >= k) n1 = ZC;
    return (uint32_t)n0 | ((uint32_t)n1 << 16);
  };
  int t_nx = 0;
  uint32_t pk_nx = (uint32_t)ZC | ((uint32_t)ZC << 16);
  float rt_nx = 0.f, v0_nx = 0.f, v1_nx = 0.f;
  if (nchild > 0) {
    t_nx = s_tok[0];
    pk_nx = first_slots(0, t_nx);
    rt_nx = r_lds[t_nx];
    v0_nx = r_lds[pk_nx & 0xFFFFu];
    v1_nx = r_lds[pk_nx >> 16];
  }
  for (int ci = 0; ci < nchild; ++ci) {
    const int t = t_nx;
    const float rt = rt_nx;
    const uint32_t pk_first = pk_nx;
    const float v0_first = v0_nx, v1_first = v1_nx;
    const bool skip_rule = ALT && a.skip;
    float cum_sk = rt;       // (wave 0) mass of A so far under the skip rule: x^ is always a member
    int cnt_sk = 0;          // (wave 0) members besides x^
    // bound: sum_A r < lambda * r(x^)  (Sec. 4), or the additive form sum_A r < delta of the same
    // section, brought to the scale of the unnormalised r
    const float cap = a.additive ? a.lambda / rs : a.lambda * rt;
    const int32_t* nrow = a.neigh + (int64_t)t * a.kstride;

    // A = longest nearest-first prefix whose running sum stays below the cap.  G(i), the sum
    // through the slots of lane i, is non-decreasing over the block by construction (monotone
    // scan inside a wave, wave totals added one after the other), so the lanes wholly inside A,
    // the one lane A ends in and the lanes outside follow each other in that order.
    uint32_t pn[MAXP];       // my two slots of each pass (16-bit indices)
    float pv0[MAXP], pv1[MAXP];
    uint32_t pm[MAXP];       // bit 0 / 1: slot zeroed by me in this pass
    float carry = 0.f;       // sum over the passes already taken
    bool found = false;
#pragma unroll
    for (int ps = 0; ps < MAXP; ++ps) {
      pn[ps] = 0; pv0[ps] = pv1[ps] = 0.f; pm[ps] = 0;
      if (ps * PASS < k && !found) {                 // uniform
        const int sl0 = ps * PASS + 2 * tid;
        uint32_t pk;
        if (ps == 0) {
          pk = pk_first;
        } else {
          const int x0 = nrow[min(sl0, k - 1)], x1 = nrow[min(sl0 + 1, k - 1)];
          int n0 = min(max(x0, 0), V - 1), n1 = min(max(x1, 0), V - 1);
          if (sl0 >= k) n0 = ZC;
          if (sl0 + 1 >= k) n1 = ZC;
          pk = (uint32_t)n0 | ((uint32_t)n1 << 16);
        }
        const int n0 = pk & 0xFFFFu, n1 = pk >> 16;
        const float v0 = ps == 0 ? v0_first : r_lds[n0], v1 = ps == 0 ? v1_first : r_lds[n1];
        bool z0, z1;
        if (skip_rule) {
          // Neighbours are visited nearest first; one whose value would lift the sum to the cap is
          // passed over and the visit goes on.  All waves park their values, wave 0 walks them 64
          // at a time: lanes that cannot fit any more drop out (the sum only grows), a scan over
          // the rest finds the first that breaks the bound, everything before it joins A.
          s_val[2 * tid] = v0;
          s_val[2 * tid + 1] = v1;
          lds_barrier();
          if (w == 0) {
            for (int c = 0; c < PASS / 64; ++c) {
              const int slot = ps * PASS + 64 * c + lane;
              if (ps * PASS + 64 * c >= k) break;                       // uniform
              const float val = s_val[64 * c + lane];
              unsigned long long rem = __ballot(slot < k && slot != 0), inc = 0ull;
              for (int it = 0; it < 64 && rem; ++it) {                  // every turn removes at least one lane
                rem &= __ballot(cum_sk + val < cap);
                if (!rem) break;
                const float S = wave_monotone_scan(((rem >> lane) & 1ull) ? val : 0.f);
                const unsigned long long viol = rem & __ballot(!(cum_sk + S < cap));
                if (!viol) { inc |= rem; cum_sk = cum_sk + lane_value(S, 63); break; }
                const int lv = __builtin_amdgcn_readfirstlane(__ffsll((long long)viol) - 1);
                inc |= rem & ((1ull << lv) - 1ull);
                cum_sk = cum_sk + lane_value(wave_prev_lane(S, 0.f), lv);
                rem &= ~((2ull << lv) - 1ull);
              }
              cnt_sk += __popcll(inc);
              if (lane == 0) { s_incl[2 * c] = (uint32_t)inc; s_incl[2 * c + 1] = (uint32_t)(inc >> 32); }
            }
          }
          lds_barrier();
          const uint32_t bits = s_incl[(2 * tid) >> 5] >> ((2 * tid) & 31);   // (slots of chunks past k: stale bits, masked below)
          z0 = (bits & 1u) && sl0 < k && sl0 != 0 && n0 != t;
          z1 = (bits & 2u) && sl0 + 1 < k && n1 != t;
        } else {
          const float incl = wave_monotone_scan(v0 + v1);
          if (lane == 63) s_wtot[tog][w] = incl;
          lds_barrier();
          float base = carry, mybase = carry;
#pragma unroll
          for (int i = 0; i < NW; ++i) {
            if (i == w) mybase = base;
            base += s_wtot[tog][i];
          }
          tog ^= 1;
          const float G = mybase + incl;                         // through my slots
          const float pc = mybase + wave_prev_lane(incl, 0.f);   // before my slots
          const bool full = G < cap;
          const bool edge = !full && (pc < cap || sl0 == 0);     // A ends in my slots
          const float c0 = pc + v0;
          const bool m0 = full || (edge && (sl0 == 0 || c0 < cap));
          if (edge) {
            s_jstar = min(m0 ? sl0 + 1 : sl0, k);
            s_mass = m0 ? c0 : pc;
            r_lds[t] = m0 ? c0 : pc;                             // A's mass moves onto x^ ...
          }
          z0 = m0 && sl0 != 0 && n0 != t;
          z1 = full && n1 != t;
          carry = base;
          found = !(base < cap);
        }
        if (z0) r_lds[n0] = 0.f;                               // ... and leaves the other members
        if (z1) r_lds[n1] = 0.f;
        pn[ps] = pk; pv0[ps] = v0; pv1[ps] = v1; pm[ps] = (z0 ? 1u : 0u) | (z1 ? 2u : 0u);
      }
    }
    if (skip_rule) {
      if (tid == 0) { s_jstar = 1 + cnt_sk; s_mass = cum_sk; r_lds[t] = cum_sk; }
    } else if (!found && tid == 0) { s_jstar = k; s_mass = carry; r_lds[t] = carry; }
    lds_barrier();
    // p(x^) with distinct siblings: the drafter's probability of the token in what is left of p
    float pt = 0.f;
    if (ALT) {
      pt = exp2_fma(s_dlog[ci], md2) * inv_sd;
      if (a.norepl) {
        pt = pt * pscale;
        for (int cj = 0; cj < ci; ++cj)
          if (s_tok[cj] == t) pt = 0.f;                         // already tried: it has left p
      }
    }
    // outcome "rejected": keep the positive part of (r' - p); its sum is the new normaliser
    // (Eq. 2).  Product and difference are rounded separately: a drafter equal to the target
    // then leaves exactly nothing.  (r' rs - p <= 1, so clamping to [0, 1] is the positive part:
    // it folds into the subtraction.)
    {
      const int cn = min(ci + 1, nchild - 1);                   // (after the last child: its own, unused)
      t_nx = s_tok[cn];
      pk_nx = first_slots(cn, t_nx);
    }
    float4 rv[NCH];
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      float4* own = reinterpret_cast<float4*>(&r_lds[4 * (tid + NT * j)]);
      rv[j] = *own;
      float4 res;
      if (ALT) {
        res.x = __builtin_amdgcn_fmed3f(rv[j].x * rs - p_reg[j][0] * pscale, 0.f, 1.f);
        res.y = __builtin_amdgcn_fmed3f(rv[j].y * rs - p_reg[j][1] * pscale, 0.f, 1.f);
        res.z = __builtin_amdgcn_fmed3f(rv[j].z * rs - p_reg[j][2] * pscale, 0.f, 1.f);
        res.w = __builtin_amdgcn_fmed3f(rv[j].w * rs - p_reg[j][3] * pscale, 0.f, 1.f);
      } else {
        res.x = __builtin_amdgcn_fmed3f(rv[j].x * rs - p_reg[j][0], 0.f, 1.f);
        res.y = __builtin_amdgcn_fmed3f(rv[j].y * rs - p_reg[j][1], 0.f, 1.f);
        res.z = __builtin_amdgcn_fmed3f(rv[j].z * rs - p_reg[j][2], 0.f, 1.f);
        res.w = __builtin_amdgcn_fmed3f(rv[j].w * rs - p_reg[j][3], 0.f, 1.f);
      }
      z += (res.x + res.y) + (res.z + res.w);
      if (STAG) csum[j] = (res.x + res.y) + (res.z + res.w);
      *own = res;
    }
    if (w == (ci >> 6)) {
      const float m = s_mass * rs;
      const int jstar = s_jstar;
      if (tid == ci) { k_m = m; k_j = jstar; k_qt = rt * rs; k_pt = pt; }
    }
    z = wave_sum(z);
    if (lane == 0) s_z[ci & 1][w] = z;
    lds_barrier();
    z = combine_sum<NW, STAG>(s_z[ci & 1], lane);
    rt_nx = r_lds[t_nx];
    v0_nx = r_lds[pk_nx & 0xFFFFu];
    v1_nx = r_lds[pk_nx >> 16];
    if (z > 0.f) {
      rs = __builtin_amdgcn_rcpf(z);       // (1 ulp: the quotient's own rounding is of that size)
      csum_valid = STAG;
    } else {
      csum_valid = false;                  // (the row is put back below: its sums are read again for the draw)
      // r' == p: nothing left to resample from, and r stays as it was before this child:
      // put r' back, then undo the move of A's mass
#pragma unroll
      for (int j = 0; j < NCH; ++j) *reinterpret_cast<float4*>(&r_lds[4 * (tid + NT * j)]) = rv[j];
      lds_barrier();
#pragma unroll
      for (int ps = 0; ps < MAXP; ++ps) {
        if (pm[ps] & 1u) r_lds[pn[ps] & 0xFFFFu] = pv0[ps];
        if (pm[ps] & 2u) r_lds[pn[ps] >> 16] = pv1[ps];
      }
      if (tid == 0) r_lds[t] = rt;
      lds_barrier();
      rt_nx = r_lds[t_nx];
      v0_nx = r_lds[pk_nx & 0xFFFFu];
      v1_nx = r_lds[pk_nx >> 16];
    }
    if (ALT && a.norepl) {
      // the rejected token leaves p; the rest is divided by what it leaves behind
#pragma unroll
      for (int j = 0; j < NCH; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (4 * (tid + NT * j) + e == t) p_reg[j][e] = 0.f;
      const float left = 1.0f - pt;
      pscale = left > 0.f ? pscale / left : 0.f;
    }
  }

  // (whole grid resident) the word this row left in the mail last time holds the last call's tag;
  // this call's is the next one.  Asked for now, looked at after the cell sums: a load still on its
  // way while the children are taken is waited for in there.  (A vector load at one address for
  // all lanes: as a wave-uniform value it would be waited for on the spot.)
  uint32_t last_word = 0;
  if (STAG) {
    int lane_zero = 0;
    asm("" : "+v"(lane_zero));
    last_word = (uint32_t)a.ws_final[nodebase + P + lane_zero];
  }
  MailRound mail_first;      // (the wave that walks) asked for now, looked at after the cell sums
  if (STAG && walker && w == 1) mail_fetch(mail_first, a.ws_decision, nodebase, a.M, lane);
  // ---- draw from the final r by inverse CDF over ascending token index: cell sums by
  // their owners, then wave 0 finds the cell, the lane and the token.
  {
    // (all reads first, then the NCH reductions side by side: their steps are independent)
    float cs[NCH];
    if (STAG && csum_valid) {              // uniform
#pragma unroll
      for (int j = 0; j < NCH; ++j) cs[j] = csum[STAG ? j : 0];
    } else {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const float4 cv = *reinterpret_cast<const float4*>(&r_lds[4 * (tid + NT * j)]);
        cs[j] = (cv.x + cv.y) + (cv.z + cv.w);
      }
    }
    wave_inclusive_scan_n<NCH>(cs);
    float mine = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const float tot = lane_value(cs[j], 63);
      if (lane == j) mine = tot;
    }
    if (lane < NCH) s_cell[lane * NW + w] = mine;
  }
  for (int i = NC + tid; i < 64 * CPL; i += NT) s_cell[i] = 0.f;
  if (w != 0 && nchild > 64 * w) {
    // (rare: more than 64 children)  this wave's stores have to be complete before wave 0 takes
    // the row's ticket, which it does after the barrier below
    tagw = STAG ? next_tag(last_word) : 0u;
    write_children(64 * w, min(nchild - 64 * w, 64));
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
  }
  if (STAG && walker && tid < nchild) {
    // the walking block's own children: their words go to the wave that walks through LDS
    const float pt = ALT ? k_pt : exp2_fma(s_dlog[tid], md2) * inv_sd;
    s_mail[s_child[tid]] = (P << 1) | ((s_u[tid] * pt < k_m) ? 1 : 0);
  }
  lds_barrier();
  if (w != 0) {
    if (!(STAG && walker)) return;
    tagw = STAG ? next_tag(last_word) : 0u;
    if (w == 1)
      collect_and_walk(mail_first, a.ws_decision, tagw, nodebase, a.M, a.depth, P, a.spin_limit, lane, s_mail,
                       s_mail + LPP_MAX_ROWS, s_mail + 2 * LPP_MAX_ROWS, s_mail + 3 * LPP_MAX_ROWS, a.accept_len + b,
                       a.path + (int64_t)b * a.depth, a.final_token + b);
    // (the walking block's own word is read by nobody but itself, next call: it keeps the tags in step)
    if (w == 1 && lane == 0) a.ws_final[nodebase + P] = (int)tagw;
    lds_barrier();           // (met by wave 0 once it holds the draw)
    return;
  }

  float cpre[CPL];           // running sum over my cells
  {
    float run = 0.f;
#pragma unroll
    for (int i = 0; i < CPL; ++i) { run += s_cell[CPL * lane + i]; cpre[i] = run; }
  }
  const float cincl = wave_monotone_scan(cpre[CPL - 1]);
  const float cexcl = wave_prev_lane(cincl, 0.f);
  const float total = lane_value(cincl, 63);
  const float target = u_fin * total;
  // first cell whose cumulative sum exceeds the target, else the last cell with mass
  int cellid = -1;
  float cellbase = 0.f;
  bool exact = true;
  {
    int myc = -1;
    float myb = 0.f;
#pragma unroll
    for (int i = CPL - 1; i >= 0; --i)
      if (cexcl + cpre[i] > target) { myc = CPL * lane + i; myb = i > 0 ? cexcl + cpre[i - 1] : cexcl; }
    const unsigned long long hit = __ballot(myc >= 0);
    if (hit) {
      const int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)hit) - 1);
      cellid = __builtin_amdgcn_readlane(myc, l);
      cellbase = lane_value(myb, l);
    } else {
      exact = false;
      int lastc = -1;
#pragma unroll
      for (int i = 0; i < CPL; ++i)
        if (s_cell[CPL * lane + i] > 0.f) lastc = CPL * lane + i;
      const unsigned long long any = __ballot(lastc >= 0);
      if (any) cellid = __builtin_amdgcn_readlane(lastc, __builtin_amdgcn_readfirstlane(63 - __builtin_clzll(any)));
    }
  }
  int x = 0;
  if (cellid >= 0) {
    const int tb = 4 * (64 * (cellid % NW) + NT * (cellid / NW));      // first token of the cell
    const float4 rv = *reinterpret_cast<const float4*>(&r_lds[tb + 4 * lane]);
    const float cs = (rv.x + rv.y) + (rv.z + rv.w);
    const float incl = wave_monotone_scan(cs);
    const float lbase = cellbase + wave_prev_lane(incl, 0.f);
    const unsigned long long hit = exact ? __ballot(cellbase + incl > target) : 0ull;
    int l;
    if (hit) {
      l = __ffsll((long long)hit) - 1;
    } else {
      const unsigned long long any = __ballot(cs > 0.f);
      l = any ? 63 - __builtin_clzll(any) : 0;
    }
    l = __builtin_amdgcn_readfirstlane(l);
    const float u0 = lbase + rv.x, u1 = u0 + rv.y, u2 = u1 + rv.z;
    int e = 3;
    if (hit) e = u0 > target ? 0 : u1 > target ? 1 : u2 > target ? 2 : 3;
    const float pick = e == 0 ? rv.x : e == 1 ? rv.y : e == 2 ? rv.z : rv.w;
    if (!(pick > 0.f)) e = rv.w > 0.f ? 3 : rv.z > 0.f ? 2 : rv.y > 0.f ? 1 : 0;
    x = __builtin_amdgcn_readlane(tb + 4 * lane + e, l);
  }
  x = min(x, V - 1);
  tagw = STAG ? next_tag(last_word) : 0u;
  write_children(0, min(nchild, 64));
  int ticket = 0;
  if (lane == 0) {
    if (P == 0) {  // row 0 is no drafted node: defined outputs
      if (!STAG) __hip_atomic_store(&a.ws_decision[nodebase], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (a.decision) a.decision[nodebase] = 0;
      if (a.ratio) a.ratio[nodebase] = 0.f;
      if (a.mass) a.mass[nodebase] = 0.f;
      if (a.n_agg) a.n_agg[nodebase] = 0;
      if (a.q_tok) a.q_tok[nodebase] = 0.f;
      if (a.p_tok) a.p_tok[nodebase] = 0.f;
    }
    if (!(STAG && walker))
      __hip_atomic_store(&a.ws_final[nodebase + P], (int)(tagw | (uint32_t)x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (a.final_all) a.final_all[nodebase + P] = x;
    if (!STAG && a.counters) {
      // every store of this row's decisions and draw was issued by this wave: once they have
      // completed they are visible device-wide, and only then the ticket is taken
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      ticket = __hip_atomic_fetch_add(&a.counters[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (STAG) {
    if (walker) {
      lds_barrier();         // the walk is done
      if (lane == 0 && s_mail[3 * LPP_MAX_ROWS] == P) a.final_token[b] = x;
    }
    return;
  }
  if (!a.counters) return;
  ticket = __builtin_amdgcn_readfirstlane(ticket);
  if (ticket != a.M - 1) return;
  // ---- this row finished last for item b: every decision of the item is visible (the walk reads
  // them with device-scope loads)
  int* s_walk = reinterpret_cast<int*>(smem);     // r is dead
  walk_wave(a.ws_decision + nodebase, a.ws_final + nodebase, a.M, a.depth, lane, s_walk, s_walk + a.M,
            a.accept_len + b, a.path + (int64_t)b * a.depth, a.final_token + b);
  if (lane == 0) __hip_atomic_store(&a.counters[b], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);    // ready for the next call
}

// Stand-alone walk for batches larger than the counter array: one wave per item.
__global__ __launch_bounds__(64) void walk_kernel(VerifyArgs a) {
  __shared__ int s_walk[2 * LPP_MAX_ROWS];
  const int b = blockIdx.x;
  const int64_t nodebase = (int64_t)b * a.M;
  walk_wave(a.ws_decision + nodebase, a.ws_final + nodebase, a.M, a.depth, threadIdx.x, s_walk, s_walk + a.M,
            a.accept_len + b, a.path + (int64_t)b * a.depth, a.final_token + b);
}

template <int NT, int NCH, bool ALIGNED, bool FRONT, bool ALT, bool STAG>
int32_t launch_rows(const VerifyArgs& a_in, const TreeTab& tt, hipStream_t stream) {
  static LppLdsLimit limit;   // (zero-initialised) one per instantiation
  VerifyArgs a = a_in;
  auto lds_for = [](int nstage) {
    return ((size_t)NT * NCH * 4 + 4) * sizeof(float) + (size_t)nstage * NT * sizeof(uint32_t) +
           (ALT ? (size_t)2 * NT * sizeof(float) + (size_t)2 * NT / 8 : 0);
  };
  // 160 KB per compute unit, less the kernel's fixed arrays: the widest rows keep fewer lists staged
  while (a.nstage > 0 && lds_for(a.nstage) > 152 * 1024) --a.nstage;
  const size_t lds = lds_for(a.nstage);
  auto kern = verify_rows_kernel<NT, NCH, ALIGNED, FRONT, ALT, STAG>;
  const int32_t st = lpp_ensure_lds(reinterpret_cast<const void*>(kern), limit, lds);
  if (st != LPP_OK) return st;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.M)), dim3(NT), lds, stream, a, tt);
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

namespace {
int32_t relaxed_verify_impl(int32_t additive, int32_t skip, int32_t norepl, bool front,
                            const float* uncond_logits, float cfg_scale,
                            int32_t top_k, const lpp_tree* tree, const float* target_logits,
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
  if (V > LPP_MAX_VOCAB || k > LPP_MAX_K) return LPP_EUNSUPPORTED;
  if ((int64_t)B * tree->M > INT_MAX) return LPP_EUNSUPPORTED;
  const size_t need = lpp_relaxed_verify_workspace(tree, B, V, k);
  if (!ws || ws_bytes < need) return LPP_ENOWORKSPACE;
  if (!tree->d_counters) return LPP_EHIP;

  VerifyArgs a;
  a.target = target_logits; a.uncond = uncond_logits; a.cfg_scale = cfg_scale; a.top_k = top_k;
  a.drafter = drafter_logits; a.ldv = ldv; a.off = vocab_offset;
  a.V = V; a.M = tree->M; a.B = B; a.kstride = kstride; a.k = k; a.lambda = lambda; a.additive = additive;
  a.skip = skip; a.norepl = norepl;
  const bool alt = skip || norepl;
  a.depth = tree->depth > 0 ? tree->depth : 1;
  // Staged lists cost LDS.  When there are several rows per compute unit, two rows resident at
  // once (one computing while the other's loads are in flight) are worth more than staging the
  // lists of a row's fifth and later children: those children read their lists from global memory.
  a.nstage = std::min<int32_t>(tree->max_children, (int64_t)B * tree->M > 2 * 256 ? kStageSmall : kMaxStage);
  a.tokens = tokens; a.neigh = neigh; a.u_accept = u_accept; a.u_final = u_final;
  a.decision = out->decision; a.ratio = out->ratio; a.mass = out->mass; a.n_agg = out->n_agg;
  a.q_tok = out->q_tok; a.p_tok = out->p_tok; a.final_all = out->final_tok_all;
  a.accept_len = out->accept_len; a.path = out->path; a.final_token = out->final_token;
  const size_t nodes = (size_t)B * tree->M;
  a.ws_decision = reinterpret_cast<int32_t*>(ws);
  a.ws_final = reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(ws) +
                                          lpp_align_up(nodes * sizeof(int32_t), 256));
  bool fused_walk = B <= LPP_COUNTER_SLOTS;
  a.counters = fused_walk ? tree->d_counters : nullptr;
  a.spin_limit = 0;

  a.child_idx = tree->d_child_idx;
  a.consecutive = tree->consecutive_children ? 1 : 0;
  TreeTab tt;
  for (int i = 0; i < LPP_MAX_ROWS; ++i) {
    uint32_t ri = 0;
    if (i < tree->M) {
      const int32_t row = tree->heavy_first[i];
      const int32_t c0 = tree->child_ptr[row], nc = tree->child_ptr[row + 1] - c0;
      const int32_t first = nc > 0 ? tree->child_idx[c0] : 0;
      ri = (uint32_t)row | ((uint32_t)nc << 8) | ((uint32_t)first << 16) | ((uint32_t)(nc > 0 ? c0 : 0) << 24);
    }
    tt.rowinfo[i] = ri;
  }
  // Whole grid resident at once (one block per compute unit, the plain step only): rows hold their
  // loads back by chain length and the walk needs no tickets (see the kernel).  With more blocks
  // than compute units the launch order, most children first, already staggers the rows; with a
  // front end every row has a long stretch of its own before its chain, which waits would only
  // push back.
  a.n_parents = tree->n_parents;
  a.wait_parent = a.wait_leaf = 0;
  // (The walk by a resident block assumes that all B * M blocks of the launch are on the device at
  // once: one block per compute unit, the device not shared with other work meanwhile.  If that
  // does not hold the walk may give up, which lpp_tree_walk_status reports.)
  const bool stag = (int64_t)B * tree->M <= std::min<int32_t>(tree->n_cu, LPP_MAX_ROWS) && !front && !alt && tree->d_mail != nullptr;
  if (stag) {
    // Tuned on MI355X (256 compute units): a row waits for 0.8 of the time the memory system needs,
    // at kStaggerBytesPerSecond, for the bytes asked for ahead of it (measured best: 0.7 .. 0.9).
    constexpr double kStagger = 0.8, kStaggerBytesPerSecond = 5.0e12;
    // one logit row of every item, in 1/256 of the kernel's sleep unit (1024 clocks)
    const double ticks_per_row = (double)B * V * 4.0 / kStaggerBytesPerSecond * (tree->clock_khz * 1.0e3) / 1024.0 * 256.0 * kStagger;
    a.wait_parent = (int32_t)(2.0 * ticks_per_row);
    a.wait_leaf = (int32_t)ticks_per_row;
    // the other rows' words reach the walking block through the tree's mail words, not the workspace
    a.ws_decision = tree->d_mail;
    a.ws_final = tree->d_mail + LPP_MAX_ROWS;
    a.counters = nullptr;
    fused_walk = true;
    // about 0.5 us a round: a quarter of a second before the walk gives up (see collect_and_walk)
    a.spin_limit = tree->walk_patience;
  }

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  auto aligned16 = [&](const float* p) {
    return p == nullptr || ((reinterpret_cast<uintptr_t>(p + vocab_offset) % 16 == 0) && (ldv % 4 == 0) && (V % 4 == 0));
  };
  const bool al = aligned16(target_logits) && aligned16(drafter_logits) && aligned16(uncond_logits);
  int32_t st;
#define LPP_DISPATCH2(T, N, ALT)                                                                            \
  st = front ? (al ? launch_rows<T, N, true, true, ALT, false>(a, tt, s) : launch_rows<T, N, false, true, ALT, false>(a, tt, s))   \
             : (al ? launch_rows<T, N, true, false, ALT, false>(a, tt, s) : launch_rows<T, N, false, false, ALT, false>(a, tt, s))
#define LPP_DISPATCH(T, N)                                     \
  do {                                                         \
    if (stag) {                                                \
      st = al ? launch_rows<T, N, true, false, false, true>(a, tt, s) : launch_rows<T, N, false, false, false, true>(a, tt, s); \
    } else if (alt) { LPP_DISPATCH2(T, N, true); } else { LPP_DISPATCH2(T, N, false); } \
  } while (0)
  if (V <= 2048) LPP_DISPATCH(512, 1);
  else if (V <= 4096) LPP_DISPATCH(512, 2);
  else if (V <= 8192) LPP_DISPATCH(512, 4);
  else if (V <= 16384) LPP_DISPATCH(512, 8);
  else LPP_DISPATCH(1024, 8);
#undef LPP_DISPATCH
#undef LPP_DISPATCH2
  if (st != LPP_OK) return st;
  if (!fused_walk) {
    hipLaunchKernelGGL(walk_kernel, dim3((unsigned)B), dim3(64), 0, s, a);
    LPP_HIP_TRY(hipGetLastError());
  }
  return LPP_OK;
}
}  // namespace

extern "C" int32_t lpp_relaxed_verify(const lpp_tree* tree, const float* target_logits,
                                      const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                      int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                      int32_t kstride, int32_t k, float lambda, const float* u_accept,
                                      const float* u_final, const lpp_verify_out* out, void* ws,
                                      size_t ws_bytes, void* stream) {
  return relaxed_verify_impl(0, 0, 0, false, nullptr, 0.f, 0, tree, target_logits, drafter_logits, ldv, vocab_offset, V, B, tokens, neigh,
                             kstride, k, lambda, u_accept, u_final, out, ws, ws_bytes, stream);
}

// ---- the entry point that allocates nothing.  Its walk words (what lpp_relaxed_verify keeps in
// the caller's workspace) live in a file-scope device array.  In host code the array's name is
// only a stand-in for the symbol: the device address is asked for once per device and kept.
#define LPP_STATIC_SCRATCH_BYTES (2 * (size_t)LPP_STATIC_MAX_NODES * sizeof(int32_t))
static __device__ __align__(256) unsigned char scratch[LPP_STATIC_SCRATCH_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kLppMaxDevices] = {};

// Device address of `scratch` on the current device (each device holds its own copy).
int32_t static_scratch(void** out) {
  int dev = -1;
  LPP_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kLppMaxDevices) return LPP_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    LPP_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return LPP_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return LPP_OK;
}
}  // namespace

extern "C" int32_t lpp_relaxed_verify_static(const lpp_tree* tree, const float* target_logits,
                                             const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                             int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                             int32_t kstride, int32_t k, float lambda, const float* u_accept,
                                             const float* u_final, const lpp_verify_out* out, void* stream) {
  if (!tree) return LPP_EINVAL;
  if (B >= 1 && (int64_t)B * tree->M > LPP_STATIC_MAX_NODES) return LPP_EUNSUPPORTED;
  void* ws = nullptr;
  if (tree->d_counters) {       // (a host-only handle goes on to argument validation and fails there with LPP_EHIP)
    const int32_t st = static_scratch(&ws);
    if (st != LPP_OK) return st;
  } else {
    ws = reinterpret_cast<void*>(uintptr_t(256));   // never dereferenced: no device, nothing is launched
  }
  return relaxed_verify_impl(0, 0, 0, false, nullptr, 0.f, 0, tree, target_logits, drafter_logits, ldv, vocab_offset, V, B, tokens, neigh,
                             kstride, k, lambda, u_accept, u_final, out, ws, LPP_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int32_t lpp_relaxed_verify_additive(const lpp_tree* tree, const float* target_logits,
                                               const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                               int32_t V, int32_t B, const int32_t* tokens,
                                               const int32_t* neigh, int32_t kstride, int32_t k, float delta,
                                               const float* u_accept, const float* u_final,
                                               const lpp_verify_out* out, void* ws, size_t ws_bytes,
                                               void* stream) {
  return relaxed_verify_impl(1, 0, 0, false, nullptr, 0.f, 0, tree, target_logits, drafter_logits, ldv, vocab_offset, V, B, tokens, neigh,
                             kstride, k, delta, u_accept, u_final, out, ws, ws_bytes, stream);
}

extern "C" int32_t lpp_relaxed_verify_sampled(const lpp_tree* tree, const float* cond_logits,
                                              const float* uncond_logits, float cfg_scale, int32_t top_k,
                                              const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                              int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                              int32_t kstride, int32_t k, float lambda, const float* u_accept,
                                              const float* u_final, const lpp_verify_out* out, void* ws,
                                              size_t ws_bytes, void* stream) {
  if (cfg_scale != cfg_scale || top_k < 0) return LPP_EINVAL;
  return relaxed_verify_impl(0, 0, 0, true, uncond_logits, cfg_scale, top_k, tree, cond_logits, drafter_logits, ldv,
                             vocab_offset, V, B, tokens, neigh, kstride, k, lambda, u_accept, u_final, out, ws,
                             ws_bytes, stream);
}

extern "C" int32_t lpp_relaxed_verify_opts(const lpp_tree* tree, const float* target_logits,
                                           const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                           int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                           int32_t kstride, int32_t k, const lpp_verify_options* opts,
                                           const float* u_accept, const float* u_final,
                                           const lpp_verify_out* out, void* ws, size_t ws_bytes, void* stream) {
  if (!opts) return LPP_EINVAL;
  if (opts->bound != LPP_BOUND_MULTIPLICATIVE && opts->bound != LPP_BOUND_ADDITIVE) return LPP_EINVAL;
  if (opts->rule != LPP_RULE_PREFIX && opts->rule != LPP_RULE_SKIP) return LPP_EINVAL;
  if (opts->siblings != LPP_SIBLINGS_IID && opts->siblings != LPP_SIBLINGS_DISTINCT) return LPP_EINVAL;
  if (opts->cfg_scale != opts->cfg_scale || opts->top_k < 0) return LPP_EINVAL;
  const bool front = opts->uncond_logits != nullptr || opts->top_k > 0;
  return relaxed_verify_impl(opts->bound == LPP_BOUND_ADDITIVE, opts->rule == LPP_RULE_SKIP,
                             opts->siblings == LPP_SIBLINGS_DISTINCT, front, opts->uncond_logits, opts->cfg_scale,
                             opts->top_k, tree, target_logits, drafter_logits, ldv, vocab_offset, V, B, tokens, neigh,
                             kstride, k, opts->bound_value, u_accept, u_final, out, ws, ws_bytes, stream);
}
