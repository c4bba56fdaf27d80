// Commit of a verified step to the KV cache (paper App. A.2 "Tree drafting and decoding":
// accepted tokens are kept, what follows the first rejection is discarded): the K/V rows of the
// root and of the accepted path are appended to each item's cache in path order.
//
// Pure data movement, at most (1 + depth) rows of Dh elements per (batch, head): one block per
// (batch*head, slot), 16 bytes per lane.
#include "lpp_internal.h"

namespace {

struct CommitArgs {
  const unsigned char* kt;
  const unsigned char* vt;
  unsigned char* kc;
  unsigned char* vc;
  const int32_t* path;
  const int32_t* accept_len;
  const int32_t* seq_len;
  int32_t* new_len;
  int32_t H, S, M, depth;
  int32_t row_bytes;      // Dh * element size
};

__global__ __launch_bounds__(64) void commit_kv_kernel(CommitArgs a) {
  const int bh = blockIdx.x, slot = blockIdx.y;          // slot 0 = root, slot i = path[i - 1]
  const int b = bh / a.H;
  const int n = min(max(a.accept_len[b], 0), a.depth);
  const int base = min(max(a.seq_len[b], 0), a.S);
  if (slot == 0 && bh % a.H == 0 && threadIdx.x == 0 && a.new_len) a.new_len[b] = min(base + 1 + n, a.S);
  if (slot > n) return;
  const int pos = base + slot;
  if (pos >= a.S) return;                                  // past the capacity: dropped
  int row = 0;
  if (slot > 0) row = min(max(a.path[b * a.depth + slot - 1], 0), a.M - 1);
  const int64_t src = ((int64_t)bh * a.M + row) * a.row_bytes, dst = ((int64_t)bh * a.S + pos) * a.row_bytes;
  for (int o = threadIdx.x * 16; o < a.row_bytes; o += 64 * 16) {
    *reinterpret_cast<uint4*>(a.kc + dst + o) = *reinterpret_cast<const uint4*>(a.kt + src + o);
    *reinterpret_cast<uint4*>(a.vc + dst + o) = *reinterpret_cast<const uint4*>(a.vt + src + o);
  }
}

}  // namespace

extern "C" int32_t lpp_commit_kv(const lpp_tree* tree, int32_t dtype, const void* k_tree, const void* v_tree,
                                 const int32_t* path, const int32_t* accept_len, const int32_t* seq_len,
                                 int32_t B, int32_t H, int32_t S, int32_t Dh, void* k_cache, void* v_cache,
                                 int32_t* new_len, void* stream) {
  if (!tree || !k_tree || !v_tree || !path || !accept_len || !seq_len || !k_cache || !v_cache) return LPP_EINVAL;
  if (B < 1 || H < 1 || S < 1 || Dh < 1) return LPP_EINVAL;
  if (new_len == seq_len) return LPP_EINVAL;                // every head's block reads seq_len
  if (dtype != LPP_F32 && dtype != LPP_BF16) return LPP_EUNSUPPORTED;
  const int esz = dtype == LPP_F32 ? 4 : 2;
  if ((Dh * esz) % 16 != 0) return LPP_EUNSUPPORTED;
  if ((int64_t)B * H > 0x7FFFFFFF) return LPP_EUNSUPPORTED;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { (void)hipGetLastError(); return LPP_EHIP; }
  CommitArgs a;
  a.kt = (const unsigned char*)k_tree; a.vt = (const unsigned char*)v_tree;
  a.kc = (unsigned char*)k_cache; a.vc = (unsigned char*)v_cache;
  a.path = path; a.accept_len = accept_len; a.seq_len = seq_len; a.new_len = new_len;
  a.H = H; a.S = S; a.M = tree->M; a.depth = tree->depth > 0 ? tree->depth : 1;
  a.row_bytes = Dh * esz;
  hipLaunchKernelGGL(commit_kv_kernel, dim3((unsigned)(B * H), (unsigned)(a.depth + 1)), dim3(64), 0,
                     reinterpret_cast<hipStream_t>(stream), a);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}
