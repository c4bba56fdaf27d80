// Tree-masked decode attention of the flattened draft tree against the target
// model's KV cache (paper Sec. 2.1; App. A.2 "Tree drafting and decoding": every
// tree row sees the whole prefix plus its ancestors and itself, nothing else).
//
// bf16 path.  Keys are cut into groups of 32 (cache groups first, then tree
// groups).  A wave owns whole groups and all tree rows of its block's row range:
//   S^T[32 keys x rows] = K_group * Q^T       (MFMA 16x16x32 bf16, K straight from HBM
//                                              into the A operand, Q held in registers)
//   softmax down the key axis, which is mostly lane-local in this layout; the
//   reference maximum of a row only moves when a score exceeds it by 2^8, so the
//   accumulators are rarely rescaled
//   O^T[Dh x rows]    += V_group^T * P^T       (V rows go to a wave-private LDS tile as
//                                              they are and come back through the
//                                              transposing LDS read; P stays in registers;
//                                              a tile of ones in place of V^T gives the
//                                              row sums of the rounded P)
// The loads of a wave's next group are issued before it works on the current one.
// The ancestor mask is one 64-bit word per (row, 64 tree keys) and only touches
// tree groups.  Waves of a block merge their (max, sum, O) through LDS; when the
// key range of one (batch, head) is split over several blocks to fill the chip the
// partials go through the workspace and the block that finishes last adds them up
// in split order.
//
// fp32 path: a plain two-pass kernel, one block per row, for small shapes (no matrix cores).
#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "lpp_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr float kMasked = -1.0e30f;  // finite stand-in for -inf
constexpr float kLazy = 8.0f;        // log2 of the largest probability weight before a rescale

// Several layers of one step go out in one launch: block index / blocks_per_layer picks the layer,
// whose tensors are looked up in a table inside the kernel arguments (a wave-uniform index).
constexpr int kLayersPerLaunch = 16;
struct LayerPtrs {
  const void* q; const void* kc; const void* vc; const void* kt; const void* vt;
  void* out;                         // [B,H,M,Dh] float, or bf16 when out_bf16
};

struct AttnArgs {
  LayerPtrs layer[kLayersPerLaunch];
  int32_t n_layers;
  uint32_t blocks_per_layer, rc_bpl;  // (a multiple of 8: every layer maps to the XCDs the same way)
  int64_t layer_rows;                // partial rows per layer in ws_o / ws_ml
  int32_t layer_counters;            // counters per layer
  const int32_t* seq_len;
  const uint64_t* anc;
  int32_t B, H, S, M, words;
  int32_t Hkv, gq;                   // key/value heads and query heads per key/value head (H = Hkv * gq)
  int32_t out_bf16;                  // out holds bf16 instead of float
  int32_t nsplit, msplits, mtiles;   // mtiles = ceil(M / 16)
  uint32_t rc_perbh, rc_msplits, rc_H, rc_nsplit, rc_gq;   // ceil(2^32 / d): n / d = mulhi(n, rc) while n d < 2^32
  float scale_log2;                  // scale * log2(e)
  float* ws_o;                       // [BH][nsplit][mtiles*16][Dh]   unnormalised partial O
  float* ws_ml;                      // [BH][nsplit][mtiles*16][2]    (reference max in log2 units, sum)
  uint32_t ws_o_bytes, ws_ml_bytes;  // sizes of the two (each below 2^31 when `counters` is set)
  int32_t* counters;                 // [BH * msplits] zero between calls, or null: separate merge kernel
};

// n / d for wave-uniform operands through the host's reciprocal: scalar multiplies, no division
__device__ __forceinline__ uint32_t div_rc(uint32_t n, uint32_t d, uint32_t rc) {
  const uint32_t q = (uint32_t)(((uint64_t)n * rc) >> 32);   // (rc = 0 for d = 1)
  return rc == 0 ? n : q;
}
__device__ __forceinline__ uint4 ld16(const uint16_t* p) {
  return *reinterpret_cast<const uint4*>(p);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // round to nearest even (hardware convert)
  const bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// 16- and 8-byte accesses that are visible device-wide once they have completed (the cache policy
// of a device-scope atomic, on whole vectors): what the blocks of one head exchange their partial
// results with inside one launch.  `off` is a byte offset into the buffer behind `rsrc`.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
constexpr int kDeviceScope = 16;     // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t device_buffer(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ void store_dev(__amdgpu_buffer_rsrc_t r, uint32_t off, float4 v) {
  const u32x4 x = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
  __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)off, 0, kDeviceScope);
}
__device__ __forceinline__ void store_dev(__amdgpu_buffer_rsrc_t r, uint32_t off, float2 v) {
  const u32x2 x = {__float_as_uint(v.x), __float_as_uint(v.y)};
  __builtin_amdgcn_raw_buffer_store_b64(x, r, (int)off, 0, kDeviceScope);
}
__device__ __forceinline__ float4 load_dev4(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, kDeviceScope);
  return make_float4(__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w));
}
__device__ __forceinline__ float2 load_dev2(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  const u32x2 x = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, kDeviceScope);
  return make_float2(__uint_as_float(x.x), __uint_as_float(x.y));
}

// four consecutive output elements starting at element index e of the output tensor
__device__ __forceinline__ void store_out4(float* out, bool as_bf16, int64_t e, float4 v) {
  if (as_bf16)
    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + e) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
  else
    *reinterpret_cast<float4*>(out + e) = v;
}

// One key group in flight: K as the A operand of S^T = K Q^T, V as loaded (row-major chunks).
template <int DH>
struct Stage {
  bf16x8 ka[2][DH / 32];
  uint4 vr[DH / 16];     // chunk c = lane + 64 p of the group's 32 x (DH/8) 16-byte chunks
};

// NT = row tiles (of 16 tree rows) per wave, RW = waves along the rows, KW = waves along the keys:
// a block covers NT * RW * 16 tree rows; wave (kw, rw) takes key groups gbeg + kw, + KW, ... for
// rows [rw NT 16, (rw + 1) NT 16).  The RW waves that share a key group load it independently; the
// second read is served by the compute unit's own cache.
template <int DH, int NT, int RW, int KW>
__global__ __launch_bounds__(RW * KW * 64, (RW * KW == 4 && DH == 64 ? (NT == 2 ? 3 : 2) : 1)) void tree_attn_bf16_kernel(AttnArgs a) {
  static_assert(RW == 1, "a block is one row range; its waves split the keys");
  constexpr int W = RW * KW;
  constexpr int KS = DH / 32;        // contraction steps of Q K^T
  constexpr int DT = DH / 16;        // Dh tiles of the output
  constexpr int CPR = DH / 8;        // 16-byte chunks per K/V row
  constexpr int VCH = DH / 16;       // V chunks per lane and group
  constexpr int VPITCH = DH * 2 + 32;   // bytes per key of the LDS V tile: 32 mod 256, so that the
                                        // 16 keys x 32 bytes of a transposing read hit all banks once
  constexpr int VTILE = 32 * VPITCH;
  constexpr int WROWS = NT * 16;     // rows of a wave
  constexpr int ROWS = RW * WROWS;   // rows of the block
  constexpr int OPITCH = DH + 4;     // floats per row of the merge buffer
  // merge slots: one per wave if that fits where the V tiles were (or in 12 KB per wave), else half as many
  constexpr int MS = (KW * NT * 16 * (DH + 4) * 4 <= (KW * 2 * VTILE > KW * 12 * 1024 ? KW * 2 * VTILE : KW * 12 * 1024)) ? KW : KW / 2;
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_ticket;

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;
  const int kw = wave % KW, rw = wave / KW;

  // block -> (batch*head, key split, row split); all blocks of one key/value head (every row range
  // and every query head that reads it) share an XCD and follow each other in launch order
  const uint32_t lyr = div_rc(blockIdx.x, a.blocks_per_layer, a.rc_bpl);
  const uint32_t bid = blockIdx.x - lyr * a.blocks_per_layer;
  const LayerPtrs& L = a.layer[lyr];
  const uint32_t xcd = bid & 7, slot = bid >> 3;
  const uint32_t per_bh = (uint32_t)(a.nsplit * a.msplits);
  const uint32_t hq = div_rc(slot, per_bh, a.rc_perbh), hr = slot - hq * per_bh;
  const uint32_t kvq = div_rc(hq, (uint32_t)a.gq, a.rc_gq), qg = hq - kvq * (uint32_t)a.gq;
  const int KVBH = a.B * a.Hkv;
  // (no early exit for the padding blocks of the last XCD round: a branch here would keep every
  // later argument load behind it; they redo the last head's work and write nothing)
  const bool live = (int)(kvq * 8 + xcd) < KVBH;
  const int kvbh = min((int)(kvq * 8 + xcd), KVBH - 1);     // batch * Hkv + key/value head
  const int bh = kvbh * a.gq + (int)qg;                     // batch * H + query head
  const int split = (int)div_rc(hr, (uint32_t)a.msplits, a.rc_msplits), ms = (int)hr - split * a.msplits;
  const int b = (int)div_rc((uint32_t)bh, (uint32_t)a.H, a.rc_H);
  const int M = a.M, S = a.S;
  const int m0 = ms * ROWS + rw * WROWS;       // first row of this wave
  int seq = S;
  if (a.seq_len) seq = min(max(a.seq_len[b], 0), S);     // (everything below depends on it anyway)
  const int GC = (seq + 31) >> 5, GT = (M + 31) >> 5, G = GC + GT;
  const int gbeg = (int)div_rc((uint32_t)(split * G), (uint32_t)a.nsplit, a.rc_nsplit);
  const int gend = (int)div_rc((uint32_t)((split + 1) * G), (uint32_t)a.nsplit, a.rc_nsplit);
  const uint16_t* kc = reinterpret_cast<const uint16_t*>(L.kc) + (int64_t)kvbh * S * DH;
  const uint16_t* vc = reinterpret_cast<const uint16_t*>(L.vc) + (int64_t)kvbh * S * DH;
  const uint16_t* kt = reinterpret_cast<const uint16_t*>(L.kt) + (int64_t)kvbh * M * DH;
  const uint16_t* vt = reinterpret_cast<const uint16_t*>(L.vt) + (int64_t)kvbh * M * DH;
  const uint16_t* qh = reinterpret_cast<const uint16_t*>(L.q) + (int64_t)bh * M * DH;
  float* const out = reinterpret_cast<float*>(L.out);

  // Key groups [0, GF) lie wholly inside the cache: no mask, no bounds.  The others (the ragged
  // end of the cache and the tree keys) go through the general path after them.
  const int GF = seq >> 5;
  const uint32_t koff = (uint32_t)(l16 * DH + g4 * 8);                      // my K chunk inside a group
  const uint32_t voff = (uint32_t)((lane / CPR) * DH + (lane % CPR) * 8);   // my V chunks: + p * (64 / CPR) rows
  auto load_full = [&](Stage<DH>& st, int g) {
    const uint16_t* Kp = kc + (int64_t)g * (32 * DH);
    const uint16_t* Vp = vc + (int64_t)g * (32 * DH);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        st.ka[t][ks] = __builtin_bit_cast(bf16x8, ld16(Kp + (koff + (uint32_t)(t * 16 * DH + ks * 32))));
#pragma unroll
    for (int p = 0; p < VCH; ++p) st.vr[p] = ld16(Vp + (voff + (uint32_t)(p * (64 / CPR) * DH)));
  };
  // general path: every load is unconditional and in bounds (row index clamped); absent keys are
  // masked out of the scores, and their V rows are zeroed on the way into LDS
  auto load_any = [&](Stage<DH>& st, int g) {
    const bool is_tree = g >= GC;
    const int kbase = is_tree ? (g - GC) * 32 : g * 32;
    const int last = (is_tree ? M : seq) - 1;
    const uint16_t* Kp = is_tree ? kt : kc;
    const uint16_t* Vp = is_tree ? vt : vc;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = min(kbase + t * 16 + l16, last);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        st.ka[t][ks] = __builtin_bit_cast(bf16x8, ld16(Kp + (uint32_t)(row * DH + ks * 32 + g4 * 8)));
    }
#pragma unroll
    for (int p = 0; p < VCH; ++p) {
      const int c = lane + 64 * p;
      const int row = min(kbase + c / CPR, last);
      st.vr[p] = ld16(Vp + (uint32_t)(row * DH + (c % CPR) * 8));
    }
  };

  // Q as the B operand: column = tree row, 8 consecutive Dh per lane and step
  bf16x8 qb[NT][KS];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int m = min(m0 + nt * 16 + l16, M - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qb[nt][ks] = __builtin_bit_cast(bf16x8, ld16(qh + (uint32_t)(m * DH + ks * 32 + g4 * 8)));
  }

  f32x4 oacc[DT][NT], lacc[NT];
  float m_ref[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m_ref[nt] = kMasked;
    lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const uint32_t one2 = 0x3F803F80u;   // two bf16 ones
  const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(one2, one2, one2, one2));

  unsigned char* vtile = smem + wave * (2 * VTILE);
  int buf = 0;
  const uint32_t vst = (uint32_t)((lane / CPR) * VPITCH + (lane % CPR) * 16);           // where my V chunks go
  const uint32_t vld = (uint32_t)((4 * g4 + (l16 >> 2)) * VPITCH + 8 * (l16 & 3));     // what I point the transposing read at

  // Which of the 32 keys of group g row m0 + nt 16 + l16 may see: the ancestor mask for tree
  // keys, the valid length for the ragged end of the cache.  The mask words are fetched here and
  // only looked at inside compute_group, so that the fetch does not hold up what follows.
  auto visibility = [&](uint64_t (&vis)[NT], int g) {
    const bool is_tree = g >= GC;
    const int kbase = is_tree ? (g - GC) * 32 : 0;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int m = min(m0 + nt * 16 + l16, M - 1);   // (rows past M are never written out)
      vis[nt] = a.anc[m * a.words + (kbase >> 6)];     // (a valid word also for cache groups: unused there)
    }
  };

  // One key group.  FULL (compile time): all 32 keys present and visible to every row.
  auto compute_group = [&](const Stage<DH>& st, int g, const uint64_t (&vis)[NT], auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const bool is_tree = g >= GC;
    const int kbase = is_tree ? (g - GC) * 32 : g * 32;
    const int limit = is_tree ? M : seq;                       // keys [kbase, limit) exist

    // S^T = K Q^T
    f32x4 sacc[2][NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        sacc[t][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          sacc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.ka[t][ks], qb[nt][ks], sacc[t][nt], 0, 0, 0);
      }

    // V rows into this wave's LDS tile, as they are
    unsigned char* tile = vtile + buf * VTILE;
#pragma unroll
    for (int p = 0; p < VCH; ++p) {
      uint4 v = st.vr[p];
      if (!FULL && kbase + (lane + 64 * p) / CPR >= limit) v = make_uint4(0, 0, 0, 0);   // absent keys: exact zeros
      *reinterpret_cast<uint4*>(tile + vst + p * (64 / CPR) * VPITCH) = v;
    }

    // softmax weights of the group; lane holds keys t*16 + 4*g4 + r of column l16
    uint32_t bits[NT];
    float mxl[NT];
    bool need = false;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      bits[nt] = 0xFFFFFFFFu;
      if (!FULL) {
        const int left = seq - kbase;
        const uint32_t cache_bits = left >= 32 ? 0xFFFFFFFFu : ((1u << left) - 1u);
        bits[nt] = is_tree ? (uint32_t)(vis[nt] >> (kbase & 63)) : cache_bits;
        bits[nt] >>= 4 * g4;        // bit 16 t + r is now my key (t, r)
      }
      float v = kMasked;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float sc = sacc[t][nt][r];
          if (!FULL && !((bits[nt] >> (16 * t + r)) & 1u)) sc = kMasked;
          v = fmaxf(v, sc);
        }
      mxl[nt] = v > 0.5f * kMasked ? v * a.scale_log2 : kMasked;   // (scale > 0: the maximum commutes with it)
      need = need || (mxl[nt] > m_ref[nt] + kLazy);
    }
    if (__ballot(need)) {   // some row's reference moves: rare after a wave's first group
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        float v = mxl[nt];
        v = fmaxf(v, __shfl_xor(v, 16));
        v = fmaxf(v, __shfl_xor(v, 32));
        const bool up = v > m_ref[nt] + kLazy;                 // decided per row: no row depends on another's scores
        const float nm = up ? v : m_ref[nt];
        const float alpha = __builtin_amdgcn_exp2f(m_ref[nt] - nm);
        m_ref[nt] = nm;
        lacc[nt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) oacc[dt][nt] *= alpha;
      }
    }
    bf16x8 pb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      uint32_t pk[4];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; r += 2) {
          float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[t][nt][r], a.scale_log2, -m_ref[nt]));
          float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[t][nt][r + 1], a.scale_log2, -m_ref[nt]));
          if (!FULL) {
            if (!((bits[nt] >> (16 * t + r)) & 1u)) p0 = 0.f;
            if (!((bits[nt] >> (16 * t + r + 1)) & 1u)) p1 = 0.f;
          }
          pk[t * 2 + r / 2] = pack_bf16(p0, p1);
        }
      pb[nt] = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
      lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[nt], lacc[nt], 0, 0, 0);
    }

    // O^T += V^T P^T.  Contraction slot (g4, j) is key (j < 4 ? 0 : 16) + 4 g4 + j % 4 on both sides.
    // The transposing read hands lane (l16, g4) the four values V[key 4 g4 + j][dt 16 + l16]: within a
    // group of 16 lanes, lane s points at 4 consecutive Dh of key 4 g4 + s / 4 at Dh offset 4 (s % 4).
    wave_lds_sync();
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const unsigned char* src = tile + vld + dt * 32;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(const __attribute__((address_space(3))) unsigned char*)src);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(const __attribute__((address_space(3))) unsigned char*)(src + 16 * VPITCH));
      const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
      const bf16x8 va = __builtin_bit_cast(bf16x8, make_uint4(l2.x, l2.y, h2.x, h2.y));
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        oacc[dt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[nt], oacc[dt][nt], 0, 0, 0);
    }
    buf ^= 1;   // the next group writes the other tile while these reads may still be in flight
  };
  const std::integral_constant<bool, true> kFull;
  const std::integral_constant<bool, false> kAny;

  // ---- this wave's groups.  The full groups go through a ring of D stages: the loads of the next
  // D - 1 groups are in flight while one is worked on, and a stage is refilled as soon as it has
  // been consumed.  The wave's first general group is fetched before them and worked on while
  // the ring's first loads are in flight.
  {
    const int h1 = min(gend, GF);                     // full groups: [gbeg, h1)
    const int c0 = max(gbeg, GF);                     // general groups: [c0, gend)
    const uint64_t novis[NT] = {};
    Stage<DH> cst;
    uint64_t vis[NT];
    int gx = c0 + kw;                                 // next general group of this wave
    if (GF >= 1) {
      constexpr int D = 2;   // (deeper rings were no faster on long caches and slower on short ones: the
                             //  eight waves of a block already have sixteen groups in flight)
      Stage<DH> st[D];
      const bool pre = gx < gend;
      if (pre) { visibility(vis, gx); load_any(cst, gx); }
      // Ring loads are issued unconditionally (a group index past the end is clamped: a re-read
      // that is never used), so that the number of loads in flight is the same on every path and
      // each wait lets the younger loads stay in flight.
      int g = gbeg + kw;
      const int hl = max(h1 - 1, 0);
#pragma unroll
      for (int d = 0; d < D; ++d) load_full(st[d], min(g + d * KW, hl));
      if (pre) { compute_group(cst, gx, vis, kAny); gx += KW; }   // while the ring's loads are in flight
      // whole rounds of the ring, as long as at least the round's first refill is a group of this
      // wave (a round that would refill nothing is left to the tail below: a wave with D groups or
      // fewer would else spend half of the compute unit's load issue on re-reads nobody uses)
      while (g + D * KW < h1) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
          compute_group(st[d], g, novis, kFull);
          load_full(st[d], min(g + D * KW, hl));
          g += KW;
        }
      }
#pragma unroll
      for (int d = 0; d < D; ++d) {               // what is left: up to D groups, already loaded
        if (g < h1) compute_group(st[d], g, novis, kFull);
        g += KW;
      }
    }
    for (; gx < gend; gx += KW) {                 // further general groups: rare, not pipelined
      visibility(vis, gx);
      load_any(cst, gx);
      compute_group(cst, gx, vis, kAny);
    }
  }

  // ---- merge the waves of the block (fixed order => run-to-run identical): every wave brings
  // its O to the block's reference maximum and parks it in LDS; the sum over the waves is taken
  // on the way out
  // (the maxima and sums have a place of their own behind the V tiles, so a wave can leave them
  // there as soon as it is done; O is parked over the V tiles once every wave is done with them)
  constexpr int OBYTES = MS * ROWS * OPITCH * 4, VBYTES = KW * 2 * VTILE;
  float* s_o = reinterpret_cast<float*>(smem);                  // [MS][ROWS][OPITCH]
  float* s_m = reinterpret_cast<float*>(smem + (OBYTES > VBYTES ? OBYTES : VBYTES));   // [W][ROWS], then the block's: [ROWS]
  float* s_l = s_m + (W + 1) * ROWS;                            // [W][ROWS], then the block's: [ROWS]
  const int r0 = rw * WROWS;                                    // my first row inside the block
  if (g4 == 0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      s_m[wave * ROWS + r0 + nt * 16 + l16] = m_ref[nt];
      s_l[wave * ROWS + r0 + nt * 16 + l16] = lacc[nt][0];
    }
  }
  __syncthreads();   // every wave is done with its V tiles too
  float fscale[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int col = r0 + nt * 16 + l16;
    float mm = kMasked;
#pragma unroll
    for (int w = 0; w < KW; ++w) mm = fmaxf(mm, s_m[(rw * KW + w) * ROWS + col]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < KW; ++w)
      ll += __builtin_amdgcn_exp2f(s_m[(rw * KW + w) * ROWS + col] - mm) * s_l[(rw * KW + w) * ROWS + col];
    fscale[nt] = __builtin_amdgcn_exp2f(m_ref[nt] - mm);
    if (kw == 0 && g4 == 0) { s_m[W * ROWS + col] = mm; s_l[W * ROWS + col] = ll; }
  }
  // MS slots of [ROWS][OPITCH] floats: with fewer slots than waves the upper waves park first and
  // the lower ones add themselves on top
#pragma unroll
  for (int round = (MS == KW ? 1 : 0); round < 2; ++round) {
    if (round == 1 && MS != KW) __syncthreads();
    const bool mine = round == 0 ? kw >= MS : kw < MS;
    if (mine) {
      const int sl = kw % MS;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int col = r0 + nt * 16 + l16;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          float4* dst = reinterpret_cast<float4*>(&s_o[(sl * ROWS + col) * OPITCH + dt * 16 + 4 * g4]);
          float4 v = make_float4(oacc[dt][nt][0] * fscale[nt], oacc[dt][nt][1] * fscale[nt],
                                 oacc[dt][nt][2] * fscale[nt], oacc[dt][nt][3] * fscale[nt]);
          if (round == 1 && MS != KW) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
          *dst = v;
        }
      }
    }
  }
  __syncthreads();

  // ---- write: final rows if this block saw every key, else an unnormalised partial
  constexpr int C4 = DH / 4;
  const int rows_pad = a.mtiles * 16;
  const int mb = ms * ROWS;                                     // first row of the block
  const __amdgpu_buffer_rsrc_t dev_o = device_buffer(a.ws_o, a.ws_o_bytes), dev_ml = device_buffer(a.ws_ml, a.ws_ml_bytes);
  for (int idx = threadIdx.x; idx < ROWS * C4; idx += W * 64) {
    const int r = idx / C4, c4 = idx % C4;
    const int m = mb + r;
    if (m >= M || !live) continue;
    float4 v = *reinterpret_cast<const float4*>(&s_o[r * OPITCH + c4 * 4]);
#pragma unroll
    for (int w = 1; w < MS; ++w) {
      const float4 o = *reinterpret_cast<const float4*>(&s_o[(w * ROWS + r) * OPITCH + c4 * 4]);
      v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
    }
    const float bm = s_m[W * ROWS + r], bl = s_l[W * ROWS + r];
    if (a.nsplit == 1) {
      const float inv = 1.0f / bl;
      v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
      store_out4(out, a.out_bf16 != 0, ((int64_t)bh * M + m) * DH + c4 * 4, v);
    } else {
      const int64_t prow = lyr * a.layer_rows + ((int64_t)bh * a.nsplit + split) * rows_pad + m;
      float* dst = a.ws_o + prow * DH + c4 * 4;
      if (a.counters) {   // read by another block of this launch: stores that are visible device-wide when they complete
        store_dev(dev_o, (uint32_t)((prow * DH + c4 * 4) * 4), v);
        if (c4 == 0) store_dev(dev_ml, (uint32_t)(prow * 8), make_float2(bm, bl));
      } else {
        *reinterpret_cast<float4*>(dst) = v;
        if (c4 == 0) { a.ws_ml[prow * 2] = bm; a.ws_ml[prow * 2 + 1] = bl; }
      }
    }
  }
  if (a.nsplit == 1 || !a.counters || !live) return;

  // ---- the block of this (head, row range) that finishes last adds the splits up, in split order
  // Every wave first waits until its own stores of the partial have completed (a device-scope
  // store is visible to every compute unit once it has completed; the workgroup barrier alone
  // waits for LDS traffic only), then the barrier gathers the waves, and only then the ticket is
  // taken.  The ticket and the reads below are device-scope atomics as well, so no cache
  // write-back or invalidate is needed.
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __syncthreads();
  if (threadIdx.x == 0)
    s_ticket = __hip_atomic_fetch_add(&a.counters[lyr * a.layer_counters + bh * a.msplits + ms], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (s_ticket != a.nsplit - 1) return;
  for (int idx = threadIdx.x; idx < ROWS * C4; idx += W * 64) {
    const int r = idx / C4, c4 = idx % C4;
    const int m = mb + r;
    if (m >= M) continue;
    // (four splits at a time: all their loads are in flight together)
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float ll = 0.f, mm = kMasked;
    for (int s0 = 0; s0 < a.nsplit; s0 += 4) {
      float2 ml[4];
      float4 o[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int sp = min(s0 + u, a.nsplit - 1);                // (a split past the end: read again, weight 0)
        const int64_t prow = lyr * a.layer_rows + ((int64_t)bh * a.nsplit + sp) * rows_pad + m;
        ml[u] = load_dev2(dev_ml, (uint32_t)(prow * 8));
        o[u] = load_dev4(dev_o, (uint32_t)((prow * DH + c4 * 4) * 4));
      }
      float nm = mm;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (s0 + u < a.nsplit) nm = fmaxf(nm, ml[u].x);
      const float keep = __builtin_amdgcn_exp2f(mm - nm);       // (the first batch: exp2(-huge) = 0 on zeros)
      acc.x *= keep; acc.y *= keep; acc.z *= keep; acc.w *= keep; ll *= keep;
      mm = nm;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float f = s0 + u < a.nsplit ? __builtin_amdgcn_exp2f(ml[u].x - mm) : 0.f;
        ll += f * ml[u].y;
        acc.x += f * o[u].x; acc.y += f * o[u].y; acc.z += f * o[u].z; acc.w += f * o[u].w;
      }
    }
    const float inv = 1.0f / ll;
    store_out4(out, a.out_bf16 != 0, ((int64_t)bh * M + m) * DH + c4 * 4,
               make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv));
  }
  if (threadIdx.x == 0)   // ready for the next call
    __hip_atomic_store(&a.counters[lyr * a.layer_counters + bh * a.msplits + ms], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
  const int64_t lbase = (int64_t)blockIdx.y * a.layer_rows;      // this layer's partials
  float mm = kMasked;
  for (int s = 0; s < a.nsplit; ++s) mm = fmaxf(mm, a.ws_ml[(lbase + (bh * a.nsplit + s) * rows_pad + m) * 2]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float ll = 0.f;
  for (int s = 0; s < a.nsplit; ++s) {
    const int64_t prow = lbase + (bh * a.nsplit + s) * rows_pad + m;
    const float f = __builtin_amdgcn_exp2f(a.ws_ml[prow * 2] - mm);
    ll += f * a.ws_ml[prow * 2 + 1];
    const float4 v = *reinterpret_cast<const float4*>(a.ws_o + prow * DH + c4 * 4);
    acc.x += f * v.x; acc.y += f * v.y; acc.z += f * v.z; acc.w += f * v.w;
  }
  const float inv = 1.0f / ll;
  store_out4(reinterpret_cast<float*>(a.layer[blockIdx.y].out), a.out_bf16 != 0, row * DH + c4 * 4,
             make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv));
}

// ---------------------------------------------------------------- fp32 path
// One block of 4 waves per (tree row, batch*head); lanes split Dh, waves split keys.
struct AttnArgsF32 {
  LayerPtrs layer[kLayersPerLaunch];     // blockIdx.z picks the layer
  const int32_t* seq_len; const uint64_t* anc;
  int32_t B, H, S, M, words, Dh;
  int32_t gq, out_bf16;     // query heads per key/value head; out holds bf16 instead of float
  float scale;
};

// One block per (tree row, batch*head).  Pass 1: one key per thread, score = scale <q, k>, masked
// keys dropped, block-wide maximum and sum of exp.  Pass 2: lanes split Dh, waves split the keys,
// weights come from LDS.  Every load is independent of the previous one, so they overlap.
__global__ __launch_bounds__(256) void tree_attn_f32_kernel(AttnArgsF32 a) {
  extern __shared__ __align__(16) float s_p[];       // [seq + M] scores, then weights
  __shared__ __align__(16) float s_q[128];
  __shared__ float s_red[2][4];
  __shared__ float s_acc[4][128];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = blockIdx.x, bh = blockIdx.y, b = bh / a.H;
  const int kvbh = bh / a.gq;            // batch * Hkv + key/value head (H = Hkv * gq)
  const int Dh = a.Dh, M = a.M, S = a.S;
  int seq = S;
  if (a.seq_len) seq = min(max(a.seq_len[b], 0), S);     // (everything below depends on it anyway)
  const int nkeys = seq + M;
  const LayerPtrs& L = a.layer[blockIdx.z];
  const float* const lq = reinterpret_cast<const float*>(L.q);
  const float* const lkc = reinterpret_cast<const float*>(L.kc);
  const float* const lvc = reinterpret_cast<const float*>(L.vc);
  const float* const lkt = reinterpret_cast<const float*>(L.kt);
  const float* const lvt = reinterpret_cast<const float*>(L.vt);
  if (tid < Dh) s_q[tid] = lq[((int64_t)bh * M + m) * Dh + tid];
  __syncthreads();

  float mx = -INFINITY;
  for (int j = tid; j < nkeys; j += 256) {
    float sc = -INFINITY;
    const int t = j - seq;
    const bool on = j < seq || ((a.anc[(int64_t)m * a.words + (t >> 6)] >> (t & 63)) & 1ull);
    if (on) {
      const float* kr = j < seq ? lkc + ((int64_t)kvbh * S + j) * Dh : lkt + ((int64_t)kvbh * M + t) * Dh;
      float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
      for (int c = 0; c < Dh; c += 4) {
        const float4 kv = *reinterpret_cast<const float4*>(kr + c);
        const float4 qv = *reinterpret_cast<const float4*>(s_q + c);
        d0 += qv.x * kv.x; d1 += qv.y * kv.y; d2 += qv.z * kv.z; d3 += qv.w * kv.w;
      }
      sc = ((d0 + d1) + (d2 + d3)) * a.scale;
    }
    s_p[j] = sc;
    mx = fmaxf(mx, sc);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if (lane == 0) s_red[0][wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(s_red[0][0], s_red[0][1]), fmaxf(s_red[0][2], s_red[0][3]));   // finite: a row sees itself
  float l = 0.f;
  for (int j = tid; j < nkeys; j += 256) {
    const float sc = s_p[j];
    const float p = sc == -INFINITY ? 0.f : expf(sc - mx);
    s_p[j] = p;
    l += p;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
  if (lane == 0) s_red[1][wave] = l;
  __syncthreads();
  l = (s_red[1][0] + s_red[1][1]) + (s_red[1][2] + s_red[1][3]);

  // (loads are unconditional and eight keys deep; a key with weight 0 -- masked or underflowed --
  // contributes an exact 0 whatever its V row holds)
  float acc0 = 0.f, acc1 = 0.f;
  const bool hi = lane + 64 < Dh;
  for (int j0 = wave; j0 < nkeys; j0 += 32) {
    float pj[8], v0[8], v1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int j = min(j0 + 4 * u, nkeys - 1);
      pj[u] = j0 + 4 * u < nkeys ? s_p[j] : 0.f;
      const float* vr = j < seq ? lvc + ((int64_t)kvbh * S + j) * Dh : lvt + ((int64_t)kvbh * M + (j - seq)) * Dh;
      v0[u] = vr[lane];
      v1[u] = hi ? vr[lane + 64] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc0 += pj[u] != 0.f ? pj[u] * v0[u] : 0.f;
      acc1 += pj[u] != 0.f ? pj[u] * v1[u] : 0.f;
    }
  }
  s_acc[wave][lane] = acc0;
  s_acc[wave][lane + 64] = acc1;
  __syncthreads();
  if (wave == 0) {
    const float o0 = (s_acc[0][lane] + s_acc[1][lane]) + (s_acc[2][lane] + s_acc[3][lane]);
    const float o1 = (s_acc[0][lane + 64] + s_acc[1][lane + 64]) + (s_acc[2][lane + 64] + s_acc[3][lane + 64]);
    const int64_t e = ((int64_t)bh * M + m) * Dh;
    if (a.out_bf16) {
      __bf16* orow = reinterpret_cast<__bf16*>(L.out) + e;
      if (lane < Dh) orow[lane] = (__bf16)(o0 / l);
      if (lane + 64 < Dh) orow[lane + 64] = (__bf16)(o1 / l);
    } else {
      float* orow = reinterpret_cast<float*>(L.out) + e;
      if (lane < Dh) orow[lane] = o0 / l;
      if (lane + 64 < Dh) orow[lane + 64] = o1 / l;
    }
  }
}

struct AttnPlan {
  int nt, kw, msplits, nsplit, mtiles;
  size_t lds;
};

// A block is one range of NT * 16 tree rows of one (batch, head) and one range of key groups;
// its KW waves take the key groups in turn.  The blocks of a head that differ in the row range
// read the same keys at about the same time and sit on the same XCD, so that the second read is
// served by its L2.  Key splits (which cost a pass through the workspace) are only added while
// the launch (all its layers) would leave compute units idle.
AttnPlan plan_attention(const lpp_tree* tree, int B, int H, int S, int Dh, int layers) {
  AttnPlan p;
  p.mtiles = (tree->M + 15) / 16;
  // Up to 64 rows: two tiles per wave and one or two blocks per head (enough blocks to fill the
  // chip at small batch).  More rows: up to five tiles per wave, so that as few blocks as possible
  // stream the same K/V out of L2.
  if (p.mtiles <= 4 || Dh != 64) {
    p.nt = p.mtiles == 1 ? 1 : 2;
    p.msplits = (p.mtiles + p.nt - 1) / p.nt;
    // Few heads (a quarter of the compute units or fewer would get a block): one tile per wave and
    // twice the row ranges fill the chip with blocks that need no more key splits than before.
    // (Head size 64 only: measured slower at 128, where a one-tile wave holds as many registers.)
    if (Dh == 64 && p.nt == 2 &&
        (int64_t)B * H * p.msplits * std::max(1, std::min(layers, kLayersPerLaunch)) * 4 <= tree->n_cu) {
      p.nt = 1;
      p.msplits = p.mtiles;
    }
  } else {
    p.msplits = (p.mtiles + 4) / 5;
    p.nt = (p.mtiles + p.msplits - 1) / p.msplits;
  }
  const int G = (S + 31) / 32 + (tree->M + 31) / 32;
  const int64_t blocks_bh = (int64_t)B * H * p.msplits * std::max(1, std::min(layers, kLayersPerLaunch));
  // Blocks of 8 waves, one per compute unit -- unless the launch has more blocks than compute units
  // and a wave of a 4-wave block still has two groups or more: then two or three such blocks share
  // a compute unit and cover each other's fixed latencies (first bytes, in-block merge, write-out)
  // and stalls, which the waves of one block, in step with each other, cannot.  With three tiles or
  // more per wave (two waves per SIMD either way) that pays from two rounds of blocks on.
  p.kw = 8;
  if (G >= 8 && ((p.nt == 2 && blocks_bh > (int64_t)tree->n_cu) ||
                 (p.nt >= 3 && Dh == 64 && blocks_bh >= 2 * (int64_t)tree->n_cu)))
    p.kw = 4;
  int ns = (int)std::min<int64_t>(tree->n_cu / blocks_bh, 1 << 20);   // key splits only while a compute unit would idle
  const int max_ns = G / (2 * p.kw);              // at least two key groups per wave
  if (ns > max_ns) ns = max_ns;
  if (ns < 1) ns = 1;
  p.nsplit = ns;
  const int rows = p.nt * 16;
  const size_t vt = (size_t)p.kw * 2 * 32 * (Dh * 2 + 32);
  const int ms = (size_t)p.kw * rows * (Dh + 4) * 4 <= std::max<size_t>(vt, (size_t)p.kw * 12 * 1024) ? p.kw : p.kw / 2;
  const size_t og = (size_t)ms * rows * (Dh + 4) * sizeof(float);
  p.lds = (vt > og ? vt : og) + (size_t)2 * (p.kw + 1) * rows * sizeof(float);
  return p;
}

template <int DH, int NT, int RW, int KW>
int32_t launch_bf16(const AttnArgs& a, const AttnPlan& p, hipStream_t s) {
  static LppLdsLimit limit;
  auto kern = tree_attn_bf16_kernel<DH, NT, RW, KW>;
  const int32_t st = lpp_ensure_lds(reinterpret_cast<const void*>(kern), limit, p.lds, 48 * 1024);
  if (st != LPP_OK) return st;
  hipLaunchKernelGGL(kern, dim3(a.blocks_per_layer * (unsigned)a.n_layers), dim3(RW * KW * 64), p.lds, s, a);
  LPP_HIP_TRY(hipGetLastError());
  if (p.nsplit > 1 && !a.counters) {
    const int64_t total = (int64_t)a.B * a.H * a.M * (DH / 4);
    hipLaunchKernelGGL(tree_attn_merge_kernel<DH>, dim3((unsigned)((total + 255) / 256), (unsigned)a.n_layers), dim3(256),
                       0, s, a);
    LPP_HIP_TRY(hipGetLastError());
  }
  return LPP_OK;
}

size_t layer_workspace(const AttnPlan& p, int B, int H, int Dh, size_t* o_bytes) {
  const size_t rows = (size_t)B * H * p.nsplit * p.mtiles * 16;
  if (o_bytes) *o_bytes = lpp_align_up(rows * Dh * sizeof(float), 256);
  return lpp_align_up(rows * Dh * sizeof(float), 256) + lpp_align_up(rows * 2 * sizeof(float), 256);
}

}  // namespace

extern "C" size_t lpp_tree_attention_workspace(const lpp_tree* tree, int32_t B, int32_t H, int32_t S,
                                               int32_t Dh) {
  return lpp_tree_attention_layers_workspace(tree, 1, B, H, S, Dh);
}

extern "C" size_t lpp_tree_attention_layers_workspace(const lpp_tree* tree, int32_t L, int32_t B, int32_t H,
                                                      int32_t S, int32_t Dh) {
  if (!tree || L < 1 || B < 1 || H < 1 || S < 0 || (Dh != 64 && Dh != 128)) return 0;
  const AttnPlan p = plan_attention(tree, B, H, S, Dh, L);
  return (size_t)std::min(L, kLayersPerLaunch) * layer_workspace(p, B, H, Dh, nullptr);
}

namespace {
int32_t tree_attention_impl(const lpp_tree* tree, int32_t dtype, int32_t out_dtype, const lpp_attention_layer* layers,
                            int32_t L, const int32_t* seq_len, int32_t B, int32_t H, int32_t Hkv, int32_t S,
                            int32_t Dh, float scale, void* ws, size_t ws_bytes, void* stream) {
  if (!tree || !layers || L < 1) return LPP_EINVAL;
  if (B < 1 || H < 1 || S < 0 || Dh < 1) return LPP_EINVAL;
  if (Hkv < 1 || Hkv > H || H % Hkv != 0) return LPP_EINVAL;
  for (int32_t l = 0; l < L; ++l) {
    const lpp_attention_layer& y = layers[l];
    if (!y.q || !y.k_tree || !y.v_tree || !y.out) return LPP_EINVAL;
    if (S > 0 && (!y.k_cache || !y.v_cache)) return LPP_EINVAL;
  }
  if (!(scale >= 0.f) || scale == INFINITY) return LPP_EINVAL;   // NaN, negative, infinite
  if (Dh != 64 && Dh != 128) return LPP_EUNSUPPORTED;
  if (dtype != LPP_F32 && dtype != LPP_BF16) return LPP_EUNSUPPORTED;
  if (out_dtype != LPP_F32 && out_dtype != LPP_BF16) return LPP_EUNSUPPORTED;
  if ((int64_t)B * H > (1 << 24) || (int64_t)B * H * H >= (1ll << 32)) return LPP_EUNSUPPORTED;
  if ((int64_t)S * Dh >= (1ll << 31) || (int64_t)tree->M * Dh >= (1ll << 31)) return LPP_EUNSUPPORTED;   // 32-bit offsets inside one head
  const size_t need = lpp_tree_attention_layers_workspace(tree, L, B, H, S, Dh);
  if (!ws || ws_bytes < need) return LPP_ENOWORKSPACE;
  if (!tree->d_anc) return LPP_EHIP;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (scale == 0.f) scale = 1.0f / sqrtf((float)Dh);

  const AttnPlan p = plan_attention(tree, B, H, S, Dh, L);
  // up to kLayersPerLaunch layers per launch; the launches of one call follow each other on the
  // stream and share the workspace
  for (int32_t l0 = 0; l0 < L; l0 += kLayersPerLaunch) {
    const int32_t nl = std::min(L - l0, kLayersPerLaunch);
    if (dtype == LPP_F32) {
      AttnArgsF32 a;
      for (int32_t l = 0; l < kLayersPerLaunch; ++l) {
        const lpp_attention_layer& y = layers[l0 + std::min(l, nl - 1)];
        a.layer[l] = LayerPtrs{y.q, y.k_cache, y.v_cache, y.k_tree, y.v_tree, y.out};
      }
      a.seq_len = seq_len; a.anc = tree->d_anc;
      a.B = B; a.H = H; a.S = S; a.M = tree->M; a.words = tree->words; a.Dh = Dh; a.scale = scale;
      a.gq = H / Hkv; a.out_bf16 = out_dtype == LPP_BF16;
      static LppLdsLimit limit;
      const size_t lds = (size_t)(S + tree->M) * sizeof(float);
      if (lds > 144 * 1024) return LPP_EUNSUPPORTED;     // the scores of one row are kept in LDS
      const int32_t st = lpp_ensure_lds(reinterpret_cast<const void*>(tree_attn_f32_kernel), limit, lds, 48 * 1024);
      if (st != LPP_OK) return st;
      hipLaunchKernelGGL(tree_attn_f32_kernel, dim3((unsigned)tree->M, (unsigned)(B * H), (unsigned)nl), dim3(256), lds,
                         s, a);
      LPP_HIP_TRY(hipGetLastError());
      continue;
    }

    AttnArgs a;
    for (int32_t l = 0; l < kLayersPerLaunch; ++l) {
      const lpp_attention_layer& y = layers[l0 + std::min(l, nl - 1)];
      a.layer[l] = LayerPtrs{y.q, y.k_cache, y.v_cache, y.k_tree, y.v_tree, y.out};
    }
    a.n_layers = nl;
    a.seq_len = seq_len; a.anc = tree->d_anc;
    a.B = B; a.H = H; a.S = S; a.M = tree->M; a.words = tree->words;
    a.Hkv = Hkv; a.gq = H / Hkv; a.out_bf16 = out_dtype == LPP_BF16;
    a.nsplit = p.nsplit; a.msplits = p.msplits; a.mtiles = p.mtiles;
    auto rc = [](uint32_t d) { return d <= 1 ? 0u : (uint32_t)((0x100000000ull + d - 1) / d); };
    a.rc_perbh = rc((uint32_t)(p.nsplit * p.msplits)); a.rc_msplits = rc((uint32_t)p.msplits);
    a.rc_H = rc((uint32_t)H); a.rc_nsplit = rc((uint32_t)p.nsplit); a.rc_gq = rc((uint32_t)(H / Hkv));
    a.scale_log2 = scale * 1.44269504088896340736f;
    const int64_t KVBH = (int64_t)B * Hkv;
    const int64_t bpl = 8 * ((KVBH + 7) / 8) * (H / Hkv) * p.nsplit * p.msplits;
    if (bpl * nl >= (1ll << 31)) return LPP_EUNSUPPORTED;
    a.blocks_per_layer = (uint32_t)bpl; a.rc_bpl = rc((uint32_t)bpl);
    size_t o_layer = 0;
    const size_t ws_layer = layer_workspace(p, B, H, Dh, &o_layer);
    (void)ws_layer;
    a.layer_rows = (int64_t)B * H * p.nsplit * p.mtiles * 16;
    a.layer_counters = B * H * p.msplits;
    const size_t o_bytes = (size_t)nl * a.layer_rows * Dh * sizeof(float), ml_bytes = (size_t)nl * a.layer_rows * 2 * sizeof(float);
    // the in-kernel merge of key splits addresses the partials with 32-bit offsets and needs a
    // counter per (layer, head, row range)
    a.counters = ((int64_t)nl * a.layer_counters <= LPP_COUNTER_SLOTS && o_bytes < (1u << 31))
                     ? tree->d_counters + LPP_COUNTER_SLOTS : nullptr;
    a.ws_o_bytes = (uint32_t)std::min<size_t>(o_bytes, 0x7FFFFFFFu);
    a.ws_ml_bytes = (uint32_t)std::min<size_t>(ml_bytes, 0x7FFFFFFFu);
    a.ws_o = reinterpret_cast<float*>(ws);
    a.ws_ml = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(ws) + (size_t)std::min(L, kLayersPerLaunch) * o_layer);

    int32_t st = LPP_EUNSUPPORTED;
    if (Dh == 64) {
      if (p.nt == 1) st = launch_bf16<64, 1, 1, 8>(a, p, s);
      else if (p.nt == 2) st = p.kw == 4 ? launch_bf16<64, 2, 1, 4>(a, p, s) : launch_bf16<64, 2, 1, 8>(a, p, s);
      else if (p.nt == 3) st = p.kw == 4 ? launch_bf16<64, 3, 1, 4>(a, p, s) : launch_bf16<64, 3, 1, 8>(a, p, s);
      else if (p.nt == 4) st = p.kw == 4 ? launch_bf16<64, 4, 1, 4>(a, p, s) : launch_bf16<64, 4, 1, 8>(a, p, s);
      else st = p.kw == 4 ? launch_bf16<64, 5, 1, 4>(a, p, s) : launch_bf16<64, 5, 1, 8>(a, p, s);
    } else {
      if (p.nt == 1) st = launch_bf16<128, 1, 1, 8>(a, p, s);
      else if (p.nt == 2) st = p.kw == 4 ? launch_bf16<128, 2, 1, 4>(a, p, s) : launch_bf16<128, 2, 1, 8>(a, p, s);
    }
    if (st != LPP_OK) return st;
  }
  return LPP_OK;
}
}  // namespace

extern "C" int32_t lpp_tree_attention(const lpp_tree* tree, int32_t dtype, const void* q, const void* k_cache,
                                      const void* v_cache, const void* k_tree, const void* v_tree,
                                      const int32_t* seq_len, int32_t B, int32_t H, int32_t S, int32_t Dh,
                                      float scale, float* out, void* ws, size_t ws_bytes, void* stream) {
  const lpp_attention_layer y = {q, k_cache, v_cache, k_tree, v_tree, out};
  return tree_attention_impl(tree, dtype, LPP_F32, &y, 1, seq_len, B, H, H, S, Dh, scale, ws, ws_bytes, stream);
}

extern "C" int32_t lpp_tree_attention_gqa(const lpp_tree* tree, int32_t dtype, int32_t out_dtype, const void* q,
                                          const void* k_cache, const void* v_cache, const void* k_tree,
                                          const void* v_tree, const int32_t* seq_len, int32_t B, int32_t H,
                                          int32_t Hkv, int32_t S, int32_t Dh, float scale, void* out, void* ws,
                                          size_t ws_bytes, void* stream) {
  const lpp_attention_layer y = {q, k_cache, v_cache, k_tree, v_tree, out};
  return tree_attention_impl(tree, dtype, out_dtype, &y, 1, seq_len, B, H, Hkv, S, Dh, scale, ws, ws_bytes, stream);
}

extern "C" int32_t lpp_tree_attention_layers(const lpp_tree* tree, int32_t dtype, int32_t out_dtype,
                                             const lpp_attention_layer* layers, int32_t L, const int32_t* seq_len,
                                             int32_t B, int32_t H, int32_t Hkv, int32_t S, int32_t Dh, float scale,
                                             void* ws, size_t ws_bytes, void* stream) {
  return tree_attention_impl(tree, dtype, out_dtype, layers, L, seq_len, B, H, Hkv, S, Dh, scale, ws, ws_bytes, stream);
}
