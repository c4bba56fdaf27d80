// Static draft-tree handle: validation, derived tables, device upload.
// (paper Sec. 2.1 static tree drafting; App. A.2 ancestors-only mask)
#include <algorithm>
#include <new>

#include "lpp_internal.h"

extern "C" const char* lpp_strerror(int32_t status) {
  switch (status) {
    case LPP_OK: return "ok";
    case LPP_EINVAL: return "invalid argument";
    case LPP_EUNSUPPORTED: return "unsupported size or type";
    case LPP_ENOWORKSPACE: return "workspace missing or too small";
    case LPP_EHIP: return "HIP runtime error (or no device)";
    default: return "unknown status";
  }
}

extern "C" const char* lpp_version(void) { return "lpp 0.1 (gfx950)"; }

extern "C" int32_t lpp_tree_create(const int32_t* parent_host, int32_t M, lpp_tree** out) {
  if (!parent_host || !out) return LPP_EINVAL;
  *out = nullptr;
  if (M < 1 || M > LPP_MAX_ROWS) return LPP_EINVAL;
  if (parent_host[0] != -1) return LPP_EINVAL;
  for (int32_t i = 1; i < M; ++i)
    if (parent_host[i] < 0 || parent_host[i] >= i) return LPP_EINVAL;

  lpp_tree* t = new (std::nothrow) lpp_tree();
  if (!t) return LPP_EHIP;
  t->M = M;
  t->words = (M + 63) / 64;
  t->parent.assign(parent_host, parent_host + M);
  t->row_depth.assign(M, 0);
  t->child_ptr.assign(M + 1, 0);
  t->child_idx.assign(M > 1 ? M - 1 : 1, 0);
  t->anc.assign((size_t)M * t->words, 0);
  std::vector<int32_t> cnt(M, 0);
  for (int32_t i = 1; i < M; ++i) {
    t->row_depth[i] = t->row_depth[t->parent[i]] + 1;
    if (t->row_depth[i] > t->depth) t->depth = t->row_depth[i];
    cnt[t->parent[i]]++;
  }
  for (int32_t i = 0; i < M; ++i) {
    t->child_ptr[i + 1] = t->child_ptr[i] + cnt[i];
    if (cnt[i] > 0) t->n_parents++;
    if (cnt[i] > t->max_children) t->max_children = cnt[i];
  }
  std::vector<int32_t> fill(t->child_ptr.begin(), t->child_ptr.end() - 1);
  for (int32_t i = 1; i < M; ++i) t->child_idx[fill[t->parent[i]]++] = i;  // ascending row index
  for (int32_t i = 0; i < M; ++i)
    for (int32_t ci = t->child_ptr[i] + 1; ci < t->child_ptr[i + 1]; ++ci)
      if (t->child_idx[ci] != t->child_idx[ci - 1] + 1) t->consecutive_children = false;
  t->heavy_first.resize(M);
  for (int32_t i = 0; i < M; ++i) t->heavy_first[i] = i;
  std::stable_sort(t->heavy_first.begin(), t->heavy_first.end(),
                   [&](int32_t x, int32_t y) { return cnt[x] > cnt[y]; });
  for (int32_t i = 0; i < M; ++i) {
    uint64_t* row = &t->anc[(size_t)i * t->words];
    if (i > 0)
      for (int32_t w = 0; w < t->words; ++w) row[w] = t->anc[(size_t)t->parent[i] * t->words + w];
    row[i / 64] |= (uint64_t)1 << (i % 64);
  }

  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    *out = t;  // host-only handle
    return LPP_OK;
  }
  auto fail = [&]() {
    (void)hipGetLastError();
    lpp_tree_destroy(t);
    return (int32_t)LPP_EHIP;
  };
  if (hipGetDevice(&t->device) != hipSuccess) return fail();
  {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, t->device) != hipSuccess) return fail();
    if (v > 0) t->n_cu = v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeClockRate, t->device) != hipSuccess) return fail();
    if (v > 0) t->clock_khz = v;
  }
  size_t b_ptr = sizeof(int32_t) * (M + 1), b_idx = sizeof(int32_t) * t->child_idx.size(),
         b_anc = sizeof(uint64_t) * t->anc.size();
  if (hipMalloc((void**)&t->d_child_ptr, b_ptr) != hipSuccess) return fail();
  if (hipMalloc((void**)&t->d_child_idx, b_idx) != hipSuccess) return fail();
  if (hipMalloc((void**)&t->d_anc, b_anc) != hipSuccess) return fail();
  const size_t b_cnt = sizeof(int32_t) * 2 * LPP_COUNTER_SLOTS;
  if (hipMalloc((void**)&t->d_counters, b_cnt) != hipSuccess) return fail();
  if (hipMemset(t->d_counters, 0, b_cnt) != hipSuccess) return fail();
  const size_t b_mail = sizeof(int32_t) * kMailWords;
  if (hipMalloc((void**)&t->d_mail, b_mail) != hipSuccess) return fail();
  if (hipMemset(t->d_mail, 0, b_mail) != hipSuccess) return fail();
  if (hipMemcpy(t->d_child_ptr, t->child_ptr.data(), b_ptr, hipMemcpyHostToDevice) != hipSuccess) return fail();
  if (hipMemcpy(t->d_child_idx, t->child_idx.data(), b_idx, hipMemcpyHostToDevice) != hipSuccess) return fail();
  if (hipMemcpy(t->d_anc, t->anc.data(), b_anc, hipMemcpyHostToDevice) != hipSuccess) return fail();
  *out = t;
  return LPP_OK;
}

extern "C" int32_t lpp_tree_destroy(lpp_tree* t) {
  if (!t) return LPP_OK;
  if (t->d_child_ptr) (void)hipFree(t->d_child_ptr);
  if (t->d_child_idx) (void)hipFree(t->d_child_idx);
  if (t->d_anc) (void)hipFree(t->d_anc);
  if (t->d_counters) (void)hipFree(t->d_counters);
  if (t->d_mail) (void)hipFree(t->d_mail);
  delete t;
  return LPP_OK;
}

extern "C" int32_t lpp_tree_info(const lpp_tree* t, int32_t* M, int32_t* depth, int32_t* n_parents,
                                 int32_t* max_children) {
  if (!t) return LPP_EINVAL;
  if (M) *M = t->M;
  if (depth) *depth = t->depth;
  if (n_parents) *n_parents = t->n_parents;
  if (max_children) *max_children = t->max_children;
  return LPP_OK;
}

// ---- state of the walk done by a resident block (lpp_relaxed_verify when B * M blocks fit the device)
namespace {
__global__ void mail_reset_kernel(int32_t* mail) {
  for (int i = threadIdx.x; i < kMailWords; i += blockDim.x) mail[i] = 0;
}
}  // namespace

extern "C" int32_t lpp_tree_set_walk_patience(lpp_tree* t, int32_t rounds) {
  if (!t || rounds < -1) return LPP_EINVAL;
  t->walk_patience = rounds > (1 << 19) ? (1 << 19) : rounds;
  return LPP_OK;
}

extern "C" int32_t lpp_tree_walk_status(const lpp_tree* t, int32_t* gave_up) {
  if (!t || !gave_up) return LPP_EINVAL;
  *gave_up = 0;
  if (!t->d_mail) return LPP_EHIP;
  int32_t flag = 0;
  LPP_HIP_TRY(hipMemcpy(&flag, t->d_mail + kMailGaveUp, sizeof(int32_t), hipMemcpyDeviceToHost));
  *gave_up = flag;
  return LPP_OK;
}

extern "C" int32_t lpp_tree_walk_reset(lpp_tree* t, void* stream) {
  if (!t) return LPP_EINVAL;
  if (!t->d_mail) return LPP_EHIP;
  hipLaunchKernelGGL(mail_reset_kernel, dim3(1), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), t->d_mail);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}
