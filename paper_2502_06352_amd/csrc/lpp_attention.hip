// Tree-masked decode attention of the flattened draft tree against the target
// model's KV cache (paper Sec. 2.1; App. A.2 "Tree drafting and decoding": every
// tree row sees the whole prefix plus its ancestors and itself, nothing else).
//
// bf16 path.  Keys are cut into groups of 32 (cache groups first, then tree
// groups).  A wave owns whole groups and all tree rows of its block's row range:
//   S^T[32 keys x rows] = K_group * Q^T       (MFMA 16x16x32 bf16, K straight from HBM
//                                              into the A operand, Q held in registers)
//   online softmax down the key axis, which is mostly lane-local in this layout
//   O^T[Dh x rows]    += V_group^T * P^T       (V transposed through a wave-private LDS
//                                              tile; P never leaves registers)
// The ancestor mask is one 64-bit word per (row, 64 tree keys) and only touches
// tree groups.  Waves of a block merge their (max, sum, O) through LDS; when the
// key range of one (batch, head) is split over several blocks to fill the chip the
// partials go through the workspace and a small merge kernel finishes the softmax.
//
// fp32 path: a plain wave-per-row kernel for small shapes (no matrix cores).
#include <math.h>

#include "lpp_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kAttnWaves = 4;
constexpr int kVPitch = 72;          // bytes per row of the transposed V tile (32 keys + pad)
constexpr float kMasked = -1.0e30f;  // finite stand-in for -inf

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* kc;
  const uint16_t* vc;
  const uint16_t* kt;
  const uint16_t* vt;
  const int32_t* seq_len;
  const uint64_t* anc;
  int32_t B, H, S, M, words;
  int32_t nsplit, msplits, mtiles;   // mtiles = ceil(M / 16)
  float scale_log2;                  // scale * log2(e)
  float* out;                        // [B,H,M,Dh]
  float* ws_o;                       // [BH][nsplit][mtiles*16][Dh]   unnormalised partial O
  float* ws_ml;                      // [BH][nsplit][mtiles*16][2]    (max in log2 units, sum)
};

__device__ __forceinline__ uint4 ld16(const uint16_t* p) {
  return *reinterpret_cast<const uint4*>(p);
}
__device__ __forceinline__ uint32_t bf16_rne(float x) {  // finite inputs only
  uint32_t u = __float_as_uint(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int DH, int NT>
__global__ __launch_bounds__(kAttnWaves * 64) void tree_attn_bf16_kernel(AttnArgs a) {
  constexpr int KS = DH / 32;        // contraction steps of Q K^T
  constexpr int DT = DH / 16;        // Dh tiles of the output
  constexpr int CPR = DH / 8;        // 16-byte chunks per K/V row
  constexpr int QPP = 64 / CPR;      // key quads per V load pass
  constexpr int VP = 8 / QPP;        // V load passes per 32-key group
  constexpr int ROWS = NT * 16;
  constexpr int OPITCH = DH + 4;     // floats per row of the merge buffer
  extern __shared__ unsigned char smem[];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, g4 = lane >> 4;

  // block -> (batch*head, key split, row split); all blocks of one head share an XCD
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per_bh = a.nsplit * a.msplits;
  const int BH = a.B * a.H;
  const int bh = (slot / per_bh) * 8 + xcd;
  if (bh >= BH) return;
  const int split = (slot % per_bh) / a.msplits, ms = (slot % per_bh) % a.msplits;
  const int b = bh / a.H;
  const int M = a.M, S = a.S;
  const int m0 = ms * ROWS;
  int seq = S;
  if (a.seq_len) seq = min(max(a.seq_len[b], 0), S);
  const int GC = (seq + 31) >> 5, GT = (M + 31) >> 5, G = GC + GT;
  const int gbeg = (int)(((long long)split * G) / a.nsplit);
  const int gend = (int)(((long long)(split + 1) * G) / a.nsplit);

  // Q as the B operand: column = tree row, 8 consecutive Dh per lane and step
  bf16x8 qb[NT][KS];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int m = m0 + nt * 16 + l16;
#pragma unroll
    for (int st = 0; st < KS; ++st) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (m < M) v = ld16(a.q + ((int64_t)bh * M + m) * DH + st * 32 + g4 * 8);
      qb[nt][st] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x4 oacc[DT][NT];
  float m_run[NT], l_part[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m_run[nt] = kMasked;
    l_part[nt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  unsigned char* vtile = smem + wave * (DH * kVPitch);
  const int vq = lane / CPR, vc8 = lane % CPR;   // V load role: key quad, 8-wide Dh chunk

  for (int g = gbeg + wave; g < gend; g += kAttnWaves) {
    const bool is_tree = g >= GC;
    const int kbase = is_tree ? (g - GC) * 32 : g * 32;
    const int limit = is_tree ? M : seq;                       // keys [kbase, limit) exist
    const uint16_t* Kp = is_tree ? a.kt + (int64_t)bh * M * DH : a.kc + (int64_t)bh * S * DH;
    const uint16_t* Vp = is_tree ? a.vt + (int64_t)bh * M * DH : a.vc + (int64_t)bh * S * DH;

    bf16x8 ka[2][KS];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const int row = min(kbase + kt * 16 + l16, limit - 1);
#pragma unroll
      for (int st = 0; st < KS; ++st)
        ka[kt][st] = __builtin_bit_cast(bf16x8, ld16(Kp + (int64_t)row * DH + st * 32 + g4 * 8));
    }
    uint4 vr[VP][4];
#pragma unroll
    for (int ps = 0; ps < VP; ++ps)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = kbase + (ps * QPP + vq) * 4 + i;
        vr[ps][i] = make_uint4(0, 0, 0, 0);                    // absent keys contribute exact zeros
        if (row < limit) vr[ps][i] = ld16(Vp + (int64_t)row * DH + vc8 * 8);
      }

    // S^T = K Q^T
    f32x4 sacc[2][NT];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        sacc[kt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < KS; ++st)
          sacc[kt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt][st], qb[nt][st], sacc[kt][nt], 0, 0, 0);
      }

    // online softmax over this group's 32 keys; lane holds keys kt*16 + 4*g4 + r of column l16
    bf16x8 pb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int m = m0 + nt * 16 + l16;
      uint32_t bits;
      if (is_tree) {
        bits = 0;
        if (m < M) bits = (uint32_t)(a.anc[(int64_t)m * a.words + (kbase >> 6)] >> (kbase & 63));
      } else {
        const int left = seq - kbase;
        bits = left >= 32 ? 0xFFFFFFFFu : ((1u << left) - 1u);
      }
      float sv[2][4];
      float mx = m_run[nt];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const bool on = (bits >> (kt * 16 + 4 * g4 + r)) & 1u;
          sv[kt][r] = on ? sacc[kt][nt][r] * a.scale_log2 : kMasked;
          mx = fmaxf(mx, sv[kt][r]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - mx);
      m_run[nt] = mx;
      uint32_t pk[4];
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 4; r += 2) {
          const float p0 = sv[kt][r] > 0.5f * kMasked ? __builtin_amdgcn_exp2f(sv[kt][r] - mx) : 0.f;
          const float p1 = sv[kt][r + 1] > 0.5f * kMasked ? __builtin_amdgcn_exp2f(sv[kt][r + 1] - mx) : 0.f;
          const uint32_t h0 = bf16_rne(p0), h1 = bf16_rne(p1);
          psum += __uint_as_float(h0 << 16) + __uint_as_float(h1 << 16);
          pk[kt * 2 + r / 2] = h0 | (h1 << 16);
        }
      l_part[nt] = l_part[nt] * alpha + psum;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) oacc[dt][nt] *= alpha;
      pb[nt] = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
    }

    // V^T through the wave-private LDS tile: [Dh][32 keys] bf16
    wave_lds_sync();   // the previous group's reads are done
#pragma unroll
    for (int ps = 0; ps < VP; ++ps) {
      const int quad = ps * QPP + vq;
      const uint32_t w0[4] = {vr[ps][0].x, vr[ps][0].y, vr[ps][0].z, vr[ps][0].w};
      const uint32_t w1[4] = {vr[ps][1].x, vr[ps][1].y, vr[ps][1].z, vr[ps][1].w};
      const uint32_t w2[4] = {vr[ps][2].x, vr[ps][2].y, vr[ps][2].z, vr[ps][2].w};
      const uint32_t w3[4] = {vr[ps][3].x, vr[ps][3].y, vr[ps][3].z, vr[ps][3].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint2 lo, hi;   // Dh element 2j and 2j+1 of the chunk, keys quad*4 .. +3
        lo.x = __builtin_amdgcn_perm(w1[j], w0[j], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(w3[j], w2[j], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(w1[j], w0[j], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(w3[j], w2[j], 0x07060302u);
        *reinterpret_cast<uint2*>(vtile + (vc8 * 8 + 2 * j) * kVPitch + quad * 8) = lo;
        *reinterpret_cast<uint2*>(vtile + (vc8 * 8 + 2 * j + 1) * kVPitch + quad * 8) = hi;
      }
    }
    wave_lds_sync();
    // O^T += V^T P^T ; contraction slot (g4, j) is key (j<4 ? 0 : 16) + 4*g4 + j%4 on both sides
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const unsigned char* rowp = vtile + (dt * 16 + l16) * kVPitch + g4 * 8;
      const uint2 a0 = *reinterpret_cast<const uint2*>(rowp);
      const uint2 a1 = *reinterpret_cast<const uint2*>(rowp + 32);
      const bf16x8 va = __builtin_bit_cast(bf16x8, make_uint4(a0.x, a0.y, a1.x, a1.y));
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        oacc[dt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[nt], oacc[dt][nt], 0, 0, 0);
    }
  }

  // ---- merge the waves of this block (fixed order => run-to-run identical)
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    l_part[nt] += __shfl_xor(l_part[nt], 16);
    l_part[nt] += __shfl_xor(l_part[nt], 32);
  }
  __syncthreads();   // every wave is done with its V tile: the buffer is reused below
  float* s_o = reinterpret_cast<float*>(smem);                  // [ROWS][OPITCH]
  float* s_m = s_o + ROWS * OPITCH;                             // [waves][ROWS]
  float* s_l = s_m + kAttnWaves * ROWS;                         // [waves][ROWS]
  if (g4 == 0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      s_m[wave * ROWS + nt * 16 + l16] = m_run[nt];
      s_l[wave * ROWS + nt * 16 + l16] = l_part[nt];
    }
  }
  __syncthreads();
  float mtot[NT], ltot[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int col = nt * 16 + l16;
    float mm = s_m[col];
#pragma unroll
    for (int w = 1; w < kAttnWaves; ++w) mm = fmaxf(mm, s_m[w * ROWS + col]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w)
      ll += __builtin_amdgcn_exp2f(s_m[w * ROWS + col] - mm) * s_l[w * ROWS + col];
    mtot[nt] = mm;
    ltot[nt] = ll;
    const float f = __builtin_amdgcn_exp2f(m_run[nt] - mm);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt][nt] *= f;
  }
  for (int w = 0; w < kAttnWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          float4* dst = reinterpret_cast<float4*>(&s_o[(nt * 16 + l16) * OPITCH + dt * 16 + 4 * g4]);
          float4 v = make_float4(oacc[dt][nt][0], oacc[dt][nt][1], oacc[dt][nt][2], oacc[dt][nt][3]);
          if (w > 0) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
          *dst = v;
        }
    }
    __syncthreads();
  }
  if (wave == 0 && g4 == 0) {   // totals for the write-out below
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      s_m[nt * 16 + l16] = mtot[nt];
      s_l[nt * 16 + l16] = ltot[nt];
    }
  }
  __syncthreads();

  // ---- write: final rows if this block saw every key, else an unnormalised partial
  constexpr int C4 = DH / 4;
  for (int idx = threadIdx.x; idx < ROWS * C4; idx += kAttnWaves * 64) {
    const int r = idx / C4, c4 = idx % C4;
    const int m = m0 + r;
    if (m >= M) continue;
    float4 v = *reinterpret_cast<const float4*>(&s_o[r * OPITCH + c4 * 4]);
    if (a.nsplit == 1) {
      const float inv = 1.0f / s_l[r];
      v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
      *reinterpret_cast<float4*>(a.out + ((int64_t)bh * M + m) * DH + c4 * 4) = v;
    } else {
      const int64_t prow = ((int64_t)bh * a.nsplit + split) * (a.mtiles * 16) + m;
      *reinterpret_cast<float4*>(a.ws_o + prow * DH + c4 * 4) = v;
      if (c4 == 0) { a.ws_ml[prow * 2] = s_m[r]; a.ws_ml[prow * 2 + 1] = s_l[r]; }
    }
  }
}

// Finish the softmax across the key splits of one (batch, head): one lane per 4 output floats.
template <int DH>
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(AttnArgs a) {
  constexpr int C4 = DH / 4;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)a.B * a.H * a.M * C4;
  if (idx >= total) return;
  const int c4 = (int)(idx % C4);
  const int64_t row = idx / C4;
  const int m = (int)(row % a.M);
  const int64_t bh = row / a.M;
  const int rows_pad = a.mtiles * 16;
  float mm = kMasked;
  for (int s = 0; s < a.nsplit; ++s) mm = fmaxf(mm, a.ws_ml[((bh * a.nsplit + s) * rows_pad + m) * 2]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float ll = 0.f;
  for (int s = 0; s < a.nsplit; ++s) {
    const int64_t prow = (bh * a.nsplit + s) * rows_pad + m;
    const float f = __builtin_amdgcn_exp2f(a.ws_ml[prow * 2] - mm);
    ll += f * a.ws_ml[prow * 2 + 1];
    const float4 v = *reinterpret_cast<const float4*>(a.ws_o + prow * DH + c4 * 4);
    acc.x += f * v.x; acc.y += f * v.y; acc.z += f * v.z; acc.w += f * v.w;
  }
  const float inv = 1.0f / ll;
  *reinterpret_cast<float4*>(a.out + row * DH + c4 * 4) =
      make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

// ---------------------------------------------------------------- fp32 path
// One block of 4 waves per (tree row, batch*head); lanes split Dh, waves split keys.
struct AttnArgsF32 {
  const float* q; const float* kc; const float* vc; const float* kt; const float* vt;
  const int32_t* seq_len; const uint64_t* anc;
  int32_t B, H, S, M, words, Dh;
  float scale;
  float* out;
};

__global__ __launch_bounds__(256) void tree_attn_f32_kernel(AttnArgsF32 a) {
  __shared__ float s_m[4], s_l[4];
  __shared__ float s_acc[4][128];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = blockIdx.x, bh = blockIdx.y, b = bh / a.H;
  const int Dh = a.Dh, M = a.M, S = a.S;
  int seq = S;
  if (a.seq_len) seq = min(max(a.seq_len[b], 0), S);
  const float* qrow = a.q + ((int64_t)bh * M + m) * Dh;
  const float q0 = lane < Dh ? qrow[lane] : 0.f;
  const float q1 = lane + 64 < Dh ? qrow[lane + 64] : 0.f;
  float mx = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
  const int nkeys = seq + M;
  for (int j = wave; j < nkeys; j += 4) {
    const float* kr; const float* vr;
    if (j < seq) {
      kr = a.kc + ((int64_t)bh * S + j) * Dh; vr = a.vc + ((int64_t)bh * S + j) * Dh;
    } else {
      const int t = j - seq;
      if (!((a.anc[(int64_t)m * a.words + (t >> 6)] >> (t & 63)) & 1ull)) continue;   // not an ancestor
      kr = a.kt + ((int64_t)bh * M + t) * Dh; vr = a.vt + ((int64_t)bh * M + t) * Dh;
    }
    float part = (lane < Dh ? q0 * kr[lane] : 0.f) + (lane + 64 < Dh ? q1 * kr[lane + 64] : 0.f);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
    const float s = part * a.scale;
    const float mn = fmaxf(mx, s);
    const float alpha = expf(mx - mn), p = expf(s - mn);
    mx = mn;
    l = l * alpha + p;
    acc0 = acc0 * alpha + (lane < Dh ? p * vr[lane] : 0.f);
    acc1 = acc1 * alpha + (lane + 64 < Dh ? p * vr[lane + 64] : 0.f);
  }
  if (lane == 0) { s_m[wave] = mx; s_l[wave] = l; }
  s_acc[wave][lane] = acc0;
  s_acc[wave][lane + 64] = acc1;
  __syncthreads();
  if (wave == 0) {
    float mm = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float ll = 0.f, o0 = 0.f, o1 = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float f = s_m[w] == -INFINITY ? 0.f : expf(s_m[w] - mm);
      ll += f * s_l[w];
      o0 += f * s_acc[w][lane];
      o1 += f * s_acc[w][lane + 64];
    }
    float* orow = a.out + ((int64_t)bh * M + m) * Dh;
    if (lane < Dh) orow[lane] = o0 / ll;
    if (lane + 64 < Dh) orow[lane + 64] = o1 / ll;
  }
}

struct AttnPlan {
  int nt, msplits, nsplit, mtiles;
  size_t lds;
};

AttnPlan plan_attention(const lpp_tree* tree, int B, int H, int S, int Dh) {
  AttnPlan p;
  p.mtiles = (tree->M + 15) / 16;
  const int max_nt = Dh == 64 ? 5 : 4;
  p.msplits = (p.mtiles + max_nt - 1) / max_nt;
  p.nt = (p.mtiles + p.msplits - 1) / p.msplits;
  const int G = (S + 31) / 32 + (tree->M + 31) / 32;
  const int blocks_bh = B * H * p.msplits;
  int ns = (3 * 256 + blocks_bh - 1) / blocks_bh;          // aim at ~3 blocks per CU
  const int max_ns = (G + kAttnWaves - 1) / kAttnWaves;    // at least one group per wave
  if (ns > max_ns) ns = max_ns;
  if (ns < 1) ns = 1;
  p.nsplit = ns;
  const size_t vt = (size_t)kAttnWaves * Dh * kVPitch;
  const size_t mg = ((size_t)p.nt * 16 * (Dh + 4) + 2 * kAttnWaves * p.nt * 16) * sizeof(float);
  p.lds = vt > mg ? vt : mg;
  return p;
}

template <int DH, int NT>
int32_t launch_bf16(const AttnArgs& a, const AttnPlan& p, hipStream_t s) {
  static bool attr_set = false;
  auto kern = tree_attn_bf16_kernel<DH, NT>;
  if (!attr_set && p.lds > 48 * 1024) {
    LPP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds));
    attr_set = true;
  }
  const int BH = a.B * a.H;
  const unsigned blocks = 8u * ((BH + 7) / 8) * p.nsplit * p.msplits;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kAttnWaves * 64), p.lds, s, a);
  LPP_HIP_TRY(hipGetLastError());
  if (p.nsplit > 1) {
    const int64_t total = (int64_t)BH * a.M * (DH / 4);
    hipLaunchKernelGGL(tree_attn_merge_kernel<DH>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
    LPP_HIP_TRY(hipGetLastError());
  }
  return LPP_OK;
}

}  // namespace

extern "C" size_t lpp_tree_attention_workspace(const lpp_tree* tree, int32_t B, int32_t H, int32_t S,
                                               int32_t Dh) {
  if (!tree || B < 1 || H < 1 || S < 0 || (Dh != 64 && Dh != 128)) return 0;
  const AttnPlan p = plan_attention(tree, B, H, S, Dh);
  const size_t rows = (size_t)B * H * p.nsplit * p.mtiles * 16;
  return lpp_align_up(rows * Dh * sizeof(float), 256) + lpp_align_up(rows * 2 * sizeof(float), 256);
}

extern "C" int32_t lpp_tree_attention(const lpp_tree* tree, int32_t dtype, const void* q, const void* k_cache,
                                      const void* v_cache, const void* k_tree, const void* v_tree,
                                      const int32_t* seq_len, int32_t B, int32_t H, int32_t S, int32_t Dh,
                                      float scale, float* out, void* ws, size_t ws_bytes, void* stream) {
  if (!tree || !q || !k_tree || !v_tree || !out) return LPP_EINVAL;
  if (B < 1 || H < 1 || S < 0 || Dh < 1) return LPP_EINVAL;
  if (S > 0 && (!k_cache || !v_cache)) return LPP_EINVAL;
  if (scale != scale) return LPP_EINVAL;
  if (Dh != 64 && Dh != 128) return LPP_EUNSUPPORTED;
  if (dtype != LPP_F32 && dtype != LPP_BF16) return LPP_EUNSUPPORTED;
  if ((int64_t)B * H > (1 << 24)) return LPP_EUNSUPPORTED;
  const size_t need = lpp_tree_attention_workspace(tree, B, H, S, Dh);
  if (!ws || ws_bytes < need) return LPP_ENOWORKSPACE;
  if (!tree->d_anc) return LPP_EHIP;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (scale == 0.f) scale = 1.0f / sqrtf((float)Dh);

  if (dtype == LPP_F32) {
    AttnArgsF32 a;
    a.q = (const float*)q; a.kc = (const float*)k_cache; a.vc = (const float*)v_cache;
    a.kt = (const float*)k_tree; a.vt = (const float*)v_tree; a.seq_len = seq_len; a.anc = tree->d_anc;
    a.B = B; a.H = H; a.S = S; a.M = tree->M; a.words = tree->words; a.Dh = Dh; a.scale = scale; a.out = out;
    hipLaunchKernelGGL(tree_attn_f32_kernel, dim3((unsigned)tree->M, (unsigned)(B * H)), dim3(256), 0, s, a);
    LPP_HIP_TRY(hipGetLastError());
    return LPP_OK;
  }

  const AttnPlan p = plan_attention(tree, B, H, S, Dh);
  AttnArgs a;
  a.q = (const uint16_t*)q; a.kc = (const uint16_t*)k_cache; a.vc = (const uint16_t*)v_cache;
  a.kt = (const uint16_t*)k_tree; a.vt = (const uint16_t*)v_tree; a.seq_len = seq_len; a.anc = tree->d_anc;
  a.B = B; a.H = H; a.S = S; a.M = tree->M; a.words = tree->words;
  a.nsplit = p.nsplit; a.msplits = p.msplits; a.mtiles = p.mtiles;
  a.scale_log2 = scale * 1.44269504088896340736f;
  a.out = out;
  const size_t rows = (size_t)B * H * p.nsplit * p.mtiles * 16;
  a.ws_o = reinterpret_cast<float*>(ws);
  a.ws_ml = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(ws) + lpp_align_up(rows * Dh * sizeof(float), 256));

#define LPP_ATTN(DHV, NTV) return launch_bf16<DHV, NTV>(a, p, s)
  if (Dh == 64) {
    switch (p.nt) {
      case 1: LPP_ATTN(64, 1);
      case 2: LPP_ATTN(64, 2);
      case 3: LPP_ATTN(64, 3);
      case 4: LPP_ATTN(64, 4);
      default: LPP_ATTN(64, 5);
    }
  } else {
    switch (p.nt) {
      case 1: LPP_ATTN(128, 1);
      case 2: LPP_ATTN(128, 2);
      case 3: LPP_ATTN(128, 3);
      default: LPP_ATTN(128, 4);
    }
  }
#undef LPP_ATTN
}
