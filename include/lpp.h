/*
 * lpp.h -- C ABI of the static-tree relaxed-verification step (LANTERN++) for one
 * AMD MI355X (gfx950).
 *
 * The step verifies a fixed-topology draft tree against the target model in one
 * pass (paper Sec. 2.1 and App. A.2 "Tree drafting and decoding") and applies the
 * relaxed acceptance rule with the multiplicative bound (paper Sec. 4), falling
 * back to residual resampling on rejection (Sec. 2.2, App. A.2 Eq. 2).
 *
 * Conventions
 *   - Every pointer is tagged [host] or [device] below.  Device buffers are owned
 *     by the caller, must live on the current HIP device and must stay valid
 *     until the work enqueued on `stream` has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise and never allocate device
 *     memory, except lpp_tree_create / lpp_tree_destroy.
 *   - Every call validates its arguments on the host first and returns a status;
 *     nothing is enqueued unless the status is LPP_OK.  No call throws.
 *   - `ws` is caller-provided device scratch of at least the size returned by the
 *     matching *_workspace query (256-byte aligned).  Its contents are undefined
 *     between calls; two calls that share one workspace must be ordered on a stream.
 *   - Rows: a tree has M = N+1 rows; row 0 is the root (the last committed token),
 *     rows 1..N are the drafted nodes.
 */
#ifndef LPP_H_
#define LPP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LPP_OK = 0,
  LPP_EINVAL = 1,        /* bad argument (null pointer, size out of range, malformed tree) */
  LPP_EUNSUPPORTED = 2,  /* well-formed but outside what the kernels implement              */
  LPP_ENOWORKSPACE = 3,  /* ws is NULL or ws_bytes is smaller than the query's answer       */
  LPP_EHIP = 4           /* a HIP runtime call failed (no device, launch failure, ...)      */
};

enum { LPP_F32 = 0, LPP_BF16 = 1 };

/* Limits of this implementation. */
#define LPP_MAX_ROWS   256     /* M                                     */
#define LPP_MAX_VOCAB  32768   /* V of lpp_relaxed_verify               */
#define LPP_MAX_K      4096    /* k of lpp_build_neighbours and verify */

const char* lpp_strerror(int32_t status);   /* static string, never NULL */
const char* lpp_version(void);

/* ------------------------------------------------------------------ tree ---
 * Static draft-tree topology (paper Sec. 2.1 "static tree drafting"; App. B
 * "Static Tree Structures").  parent_host [host]: M entries, parent[0] = -1,
 * 0 <= parent[i] < i for i >= 1.  Children of a row are tried in ascending row
 * index.  The library copies what it needs (child lists, depths, ancestor
 * bitmasks: bit t of row i set iff t == i or t is an ancestor of i) to the
 * current device; with no HIP device present the handle is host-only: it can be
 * queried and passed to argument validation, and compute calls return LPP_EHIP.
 * Errors: LPP_EINVAL (null, M < 1, M > LPP_MAX_ROWS, malformed parent),
 * LPP_EHIP (allocation or copy failed).
 */
typedef struct lpp_tree lpp_tree;
int32_t lpp_tree_create(const int32_t* parent_host, int32_t M, lpp_tree** out);
int32_t lpp_tree_destroy(lpp_tree* tree);
/* Any output pointer may be NULL.  depth = number of levels below the root. */
int32_t lpp_tree_info(const lpp_tree* tree, int32_t* M, int32_t* depth,
                      int32_t* n_parents, int32_t* max_children);

/* The walk of lpp_relaxed_verify when all B * M row blocks of a launch fit the device at once (one
 * per compute unit) is done by one of the item's row blocks, which waits, with a bound, for the other
 * rows' results (see lpp_relaxed_verify).  That presumes the launch's blocks are all resident
 * together: the stream's kernel has the device to itself (no compute-unit mask, no long kernel of
 * another stream or process in the way).  If the wait ever runs out, the item's accept_len, path and
 * final_token are -1 for that call, and for that call only: the rows' results carry the number of
 * their call, so whatever arrives late is not taken for a later call's.  A caller checks
 * accept_len[b] < 0 (lpp_commit_kv commits nothing but the root for such an item) or asks:
 *   lpp_tree_walk_status   [host] gave_up = number of walks that gave up since the handle was made or
 *                          last reset.  Copies one word back from the device: it waits for the device
 *                          (not for use inside a capture).
 *   lpp_tree_walk_reset    enqueues on `stream` the kernel that sets that count (and the handle's other
 *                          walk words) back to zero; never needed for correctness.
 *   lpp_tree_set_walk_patience   rounds (about 0.5 us each) the walking block waits: default and maximum
 *                          2^19; -1 makes the walk give up at once (for tests of the caller's handling).
 * Errors: LPP_EINVAL (null, rounds < -1), LPP_EHIP (host-only handle, copy or launch failed).
 */
int32_t lpp_tree_walk_status(const lpp_tree* tree, int32_t* gave_up);
int32_t lpp_tree_walk_reset(lpp_tree* tree, void* stream);
int32_t lpp_tree_set_walk_patience(lpp_tree* tree, int32_t rounds);

/* ------------------------------------------------------ neighbour build ---
 * Latent-space neighbourhoods B_k(x) of every code: the k codes closest to x in
 * the codebook's embedding space (paper Sec. 2.2; reused by Sec. 4).
 *   E      [device] float32 [V, D] row-major codebook; the caller L2-normalises
 *          the rows, so the inner product used here is the cosine similarity.
 *   neigh  [device] int32 [V, k] out; row x = B_k(x), nearest first, x itself in
 *          slot 0.  Order is by the similarity evaluated in float64 (the D
 *          products added one after the other in index order), ties to the lower
 *          index -- a deterministic, machine-independent result.
 * One-time per codebook.  Errors: LPP_EINVAL (null, V < 1, D < 1, k < 1, k > V),
 * LPP_EUNSUPPORTED (k > LPP_MAX_K, D > 256, V > 65536), LPP_ENOWORKSPACE, LPP_EHIP.
 * A codebook so degenerate that more than k + 1024 codes tie with the k-th
 * neighbour of some code (within the rounding of the filter: float32 for rows of up
 * to 16 floats, bfloat16 operands for longer ones) is still handled exactly by a
 * slower per-row path; so are rows far from unit length.
 */
size_t  lpp_build_neighbours_workspace(int32_t V, int32_t D, int32_t k);
int32_t lpp_build_neighbours(const float* E, int32_t V, int32_t D, int32_t k,
                             int32_t* neigh, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------- tree attention ---
 * One layer of tree-masked decode attention: the drafted tree is laid out as one
 * sequence of rows and checked in a single pass whose mask hides every node that
 * is not an ancestor (paper Sec. 2.1; App. A.2).  For batch item b, head h,
 * row i:  out[b,h,i,:] = softmax_j(scale * <q[b,h,i], K_j>) V_j  over the keys
 * j in { cached positions [0, seq_len[b]) } U { tree rows t : t == i or t is an
 * ancestor of i }.
 *   dtype     LPP_F32 or LPP_BF16: element type of q, k_cache, v_cache, k_tree, v_tree
 *   q, k_tree, v_tree   [device] [B, H, M, Dh] contiguous
 *   k_cache, v_cache    [device] [B, H, S, Dh] contiguous (multi-head: H_kv = H)
 *   seq_len   [device] int32 [B] or NULL (= S for every item); values are clamped to [0, S]
 *   scale     0 selects 1/sqrt(Dh); negative, infinite or NaN is LPP_EINVAL
 *   out       [device] float32 [B, H, M, Dh]
 * Softmax and accumulation are float32; bf16 inputs are multiplied on the matrix
 * cores.  Errors: LPP_EINVAL (null, B/H/S/Dh < 1 -- S = 0 is allowed), LPP_EUNSUPPORTED
 * (Dh not 64 or 128, dtype unknown, LPP_F32 with S + M > 36864), LPP_ENOWORKSPACE, LPP_EHIP.
 */
size_t  lpp_tree_attention_workspace(const lpp_tree* tree, int32_t B, int32_t H,
                                     int32_t S, int32_t Dh);
int32_t lpp_tree_attention(const lpp_tree* tree, int32_t dtype,
                           const void* q, const void* k_cache, const void* v_cache,
                           const void* k_tree, const void* v_tree, const int32_t* seq_len,
                           int32_t B, int32_t H, int32_t S, int32_t Dh, float scale,
                           float* out, void* ws, size_t ws_bytes, void* stream);

/* The same attention (Sec. 2.1; App. A.2) for targets whose key/value heads are shared by
 * groups of query heads, and with a choice of output type:
 *   Hkv       key/value heads; must divide H; query head h reads key/value head
 *             h / (H / Hkv)  (Hkv == H is the call above)
 *   k_tree, v_tree   [device] [B, Hkv, M, Dh];  k_cache, v_cache  [device] [B, Hkv, S, Dh]
 *   out_dtype LPP_F32 or LPP_BF16: element type of out [B, H, M, Dh]; bf16 is rounded to
 *             nearest even from the float32 result
 * Everything else, the workspace query (by H) included, is as for lpp_tree_attention.  The
 * query heads of one key/value head run next to each other on one XCD, so that the shared
 * keys and values leave HBM once.  Errors: as above, plus LPP_EINVAL when Hkv < 1, Hkv > H
 * or H % Hkv != 0, and LPP_EUNSUPPORTED for an unknown out_dtype.
 */
int32_t lpp_tree_attention_gqa(const lpp_tree* tree, int32_t dtype, int32_t out_dtype,
                               const void* q, const void* k_cache, const void* v_cache,
                               const void* k_tree, const void* v_tree, const int32_t* seq_len,
                               int32_t B, int32_t H, int32_t Hkv, int32_t S, int32_t Dh, float scale,
                               void* out, void* ws, size_t ws_bytes, void* stream);

/* Several layers of one step in one launch (paper Sec. 2.1; App. A.2: the target checks the
 * flattened tree in one forward pass, i.e. this attention once per layer; App. B: the targets
 * have tens of layers).  Every layer has its own tensors, all of the shapes of
 * lpp_tree_attention_gqa; tree, seq_len, sizes, scale and types are shared.  The layers' blocks
 * go out together (up to 16 layers per launch, more in consecutive launches on the stream), so that
 * one layer's start-up and merge overlap the streaming of the others.  The call does not order
 * the layers against each other: they must be independent (queries computed beforehand).
 *   layers   [host] L entries of device pointers (read during the call only)
 * Workspace: lpp_tree_attention_layers_workspace.  Errors: as lpp_tree_attention_gqa, plus
 * LPP_EINVAL for L < 1 or a null entry.
 */
typedef struct lpp_attention_layer {
  const void* q;          /* [device] [B, H, M, Dh]   */
  const void* k_cache;    /* [device] [B, Hkv, S, Dh] */
  const void* v_cache;    /* [device] [B, Hkv, S, Dh] */
  const void* k_tree;     /* [device] [B, Hkv, M, Dh] */
  const void* v_tree;     /* [device] [B, Hkv, M, Dh] */
  void*       out;        /* [device] [B, H, M, Dh], float32 or bf16 (out_dtype) */
} lpp_attention_layer;
size_t  lpp_tree_attention_layers_workspace(const lpp_tree* tree, int32_t L, int32_t B, int32_t H,
                                            int32_t S, int32_t Dh);
int32_t lpp_tree_attention_layers(const lpp_tree* tree, int32_t dtype, int32_t out_dtype,
                                  const lpp_attention_layer* layers, int32_t L, const int32_t* seq_len,
                                  int32_t B, int32_t H, int32_t Hkv, int32_t S, int32_t Dh, float scale,
                                  void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------- relaxed verify ---
 * Softmax of every row, relaxed acceptance of every drafted node and the walk
 * down the tree (paper Sec. 4; Sec. 2.2; App. A.2 Eq. 1-2).  For row P with
 * children c_1 < c_2 < ... (tokens x^ = tokens[b, c]):
 *     q = softmax(target_logits[b,P]), p = softmax(drafter_logits[b,P]), r <- q
 *     for each child:  A = longest nearest-first prefix of B_k(x^) with
 *                          sum_{x in A} r(x) < lambda * r(x^)   (x^ always in A)
 *                      mass = sum_A r,  ratio = mass / p(x^),
 *                      decision = (u_accept * p(x^) < mass)
 *                      r <- normalise([r' - p]_+), r' = r with A's mass moved onto x^
 *     final_tok_all[b,P] = inverse-CDF draw from r with u_final[b,P]
 *                          (a leaf draws its bonus token from q)
 * Each row is evaluated for the outcome "all earlier siblings rejected", which
 * involves no uniform; the walk then follows the first accepted child per level.
 *   target_logits, drafter_logits  [device] float32 [B, M, ldv]; image token x is
 *        column vocab_offset + x; columns outside [vocab_offset, vocab_offset+V)
 *        must be -inf by contract and are not read; drafter rows of leaves are
 *        never read (drafter_logits may be NULL if the tree has no drafted node).
 *   tokens    [device] int32 [B, M], values in [0, V) (clamped otherwise); tokens[b,0] ignored
 *   neigh     [device] int32 [V, kstride], first k columns used, slot 0 of row x is x
 *   lambda    bound factor; values <= 1 admit no neighbour (plain speculative sampling)
 *   u_accept, u_final   [device] float32 [B, M] in [0,1), supplied by the caller
 *   out       see lpp_verify_out; accept_len, path and final_token are required,
 *             the per-node arrays may be NULL.
 * Errors: LPP_EINVAL (null, B < 1, V < 1, k < 1, k > kstride, k > V,
 * vocab_offset < 0, vocab_offset + V > ldv, lambda NaN), LPP_EUNSUPPORTED
 * (V > LPP_MAX_VOCAB, k > LPP_MAX_K), LPP_ENOWORKSPACE, LPP_EHIP.
 * The calls keep a few words of state in the tree handle between kernels (tickets, the rows'
 * results on their way to the block that walks): calls that share a handle must be ordered on
 * a stream.  When B * M blocks fit the device at once, the walk of an item is done by one of
 * its row blocks, which waits for the others' results; that wait is bounded, and nobody waits
 * for that block.  Should it ever run out (it cannot unless the other blocks of the launch do
 * not run), accept_len[b], path[b, :] and final_token[b] of that call are set to -1 (later calls
 * are not affected); lpp_tree_walk_status counts such walks.
 */
typedef struct lpp_verify_out {
  int32_t* accept_len;     /* [device] [B]        number of accepted drafted nodes            */
  int32_t* path;           /* [device] [B, depth] accepted rows root-to-leaf, -1 padded       */
  int32_t* final_token;    /* [device] [B]        token emitted after the accepted path       */
  uint8_t* decision;       /* [device] [B, M]     accept test of every node (row 0 unused: 0) */
  float*   ratio;          /* [device] [B, M]     mass / p(x^)                                */
  float*   mass;           /* [device] [B, M]     aggregated target mass                      */
  int32_t* n_agg;          /* [device] [B, M]     |A|                                         */
  float*   q_tok;          /* [device] [B, M]     r(x^) seen by the node                      */
  float*   p_tok;          /* [device] [B, M]     p(x^)                                       */
  int32_t* final_tok_all;  /* [device] [B, M]     draw of every row if the walk stops there   */
} lpp_verify_out;

size_t  lpp_relaxed_verify_workspace(const lpp_tree* tree, int32_t B, int32_t V, int32_t k);
int32_t lpp_relaxed_verify(const lpp_tree* tree, const float* target_logits,
                           const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                           int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                           int32_t kstride, int32_t k, float lambda,
                           const float* u_accept, const float* u_final,
                           const lpp_verify_out* out, void* ws, size_t ws_bytes, void* stream);

/* lpp_relaxed_verify for callers that cannot hand over (or allocate) a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid device allocation.  The walk words that
 * lpp_relaxed_verify keeps in `ws` live in a static device array inside the library instead
 * (2 * LPP_STATIC_MAX_NODES int32 = 512 KiB, held by every GPU the library runs on until the process
 * ends).  The call allocates and frees nothing; everything else -- arguments, outputs, kernels,
 * results bit for bit -- is as for lpp_relaxed_verify.  All calls on one GPU share that array and
 * it keeps the last call's contents (every word a call reads it has written before): two calls
 * whose kernels may overlap on one GPU (different streams, different threads) race; order them.
 * The first call on a device looks the array's address up (no stream work): make it outside a
 * graph capture; later calls may be captured.
 * Errors: as lpp_relaxed_verify (no LPP_ENOWORKSPACE), plus LPP_EUNSUPPORTED when
 * B * M > LPP_STATIC_MAX_NODES or the device index is 64 or more.
 */
#define LPP_STATIC_MAX_NODES 65536
int32_t lpp_relaxed_verify_static(const lpp_tree* tree, const float* target_logits,
                                  const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                  int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                  int32_t kstride, int32_t k, float lambda,
                                  const float* u_accept, const float* u_final,
                                  const lpp_verify_out* out, void* stream);

/* The same step under the additive bound of the earlier LANTERN method, which the paper's Sec. 4
 * states next to its own:  A = longest nearest-first prefix of B_k(x^) with
 *     sum_{x in A} r(x) < delta        (x^ always in A; r normalised),
 * everything else as in lpp_relaxed_verify.  delta <= r(x^) admits no neighbour.  Same arguments,
 * workspace (lpp_relaxed_verify_workspace) and errors; delta NaN is LPP_EINVAL.
 */
int32_t lpp_relaxed_verify_additive(const lpp_tree* tree, const float* target_logits,
                                    const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                    int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                    int32_t kstride, int32_t k, float delta,
                                    const float* u_accept, const float* u_final,
                                    const lpp_verify_out* out, void* ws, size_t ws_bytes, void* stream);

/* The same step with the sampling configuration of the paper's experiments in front of the target
 * softmax (App. B "Models": classifier-free guidance, top-k sampling, temperature 1), fused into the
 * load of the target rows:
 *     l(x) = u(x) + cfg_scale * (c(x) - u(x))     c = cond_logits row, u = uncond_logits row
 *     only the top_k largest l of a row stay (ties with the top_k-th stay too), the rest is -inf
 *     q = softmax(l)
 * computed in float32 with the difference, the product and the sum each rounded once, so that which
 * tokens survive is reproducible.  uncond_logits NULL = no guidance (l = c); top_k 0 or >= V = no
 * filter.  drafter_logits are taken as they are.  Everything else as in lpp_relaxed_verify (same
 * workspace query).  Extra errors: LPP_EINVAL for cfg_scale NaN or top_k < 0.
 */
int32_t lpp_relaxed_verify_sampled(const lpp_tree* tree, const float* cond_logits,
                                   const float* uncond_logits, float cfg_scale, int32_t top_k,
                                   const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                   int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                   int32_t kstride, int32_t k, float lambda,
                                   const float* u_accept, const float* u_final,
                                   const lpp_verify_out* out, void* ws, size_t ws_bytes, void* stream);

/* The same step with every choice in one place: the bound (Sec. 4: LANTERN++'s multiplicative
 * one or the additive one of LANTERN), the front end (App. B "Models"), and the two points the
 * paper leaves open -- how A is picked inside B_k(x^) (Sec. 4 states only the constraint) and
 * how the children of one row were drafted (Sec. 2.1 says only that several are drawn from p):
 *   rule      LPP_RULE_PREFIX   A = the longest nearest-first prefix of B_k(x^) under the bound
 *             LPP_RULE_SKIP     neighbours are visited nearest first; one that would lift the
 *                               sum to the bound or above is passed over and the visit goes on
 *                               (n_agg = |A| then counts members, not a prefix length)
 *   siblings  LPP_SIBLINGS_IID       i.i.d. draws from p: every child is tried against p
 *             LPP_SIBLINGS_DISTINCT  distinct tokens drawn one after the other: a rejected
 *                               child's token leaves p (p(x^) <- 0, the rest / (1 - p(x^))) before
 *                               the next child; p_tok and ratio report that p; a token that is
 *                               handed in twice has p = 0 the second time
 *   bound, bound_value          LPP_BOUND_MULTIPLICATIVE with lambda, LPP_BOUND_ADDITIVE with delta
 *   uncond_logits, cfg_scale, top_k   as in lpp_relaxed_verify_sampled; NULL and 0 = no front end
 * With the zero-initialised struct and bound_value = lambda this is lpp_relaxed_verify.  Both
 * sibling schemes leave the output law equal to the target when A = {x^}.  Same workspace query;
 * errors as above, plus LPP_EINVAL for a null opts or an unknown enumerator.
 */
#define LPP_BOUND_MULTIPLICATIVE 0
#define LPP_BOUND_ADDITIVE       1
#define LPP_RULE_PREFIX          0
#define LPP_RULE_SKIP            1
#define LPP_SIBLINGS_IID         0
#define LPP_SIBLINGS_DISTINCT    1
typedef struct lpp_verify_options {
  int32_t bound;
  float   bound_value;
  int32_t rule;
  int32_t siblings;
  const float* uncond_logits;   /* [device] [B, M, ldv] or NULL */
  float   cfg_scale;
  int32_t top_k;
} lpp_verify_options;
int32_t lpp_relaxed_verify_opts(const lpp_tree* tree, const float* target_logits,
                                const float* drafter_logits, int64_t ldv, int32_t vocab_offset,
                                int32_t V, int32_t B, const int32_t* tokens, const int32_t* neigh,
                                int32_t kstride, int32_t k, const lpp_verify_options* opts,
                                const float* u_accept, const float* u_final,
                                const lpp_verify_out* out, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- commit ---
 * Appends what the step keeps to the KV cache (paper App. A.2: accepted tokens are kept, the rest
 * of the tree is discarded).  For item b the rows r_0 = 0 (the root: the last committed token, not
 * in the cache yet) and r_i = path[b, i-1], 1 <= i <= accept_len[b], of k_tree / v_tree are copied
 * to cache positions seq_len[b] + i of every head; new_len[b] = seq_len[b] + 1 + accept_len[b].
 * Rows that would land at or past S are dropped and new_len is capped at S.
 *   dtype               LPP_F32 or LPP_BF16 (element type of the four K/V tensors)
 *   k_tree, v_tree      [device] [B, H, M, Dh]
 *   path, accept_len    [device] int32 [B, depth] / [B], as written by lpp_relaxed_verify
 *   seq_len             [device] int32 [B] current lengths (clamped to [0, S])
 *   k_cache, v_cache    [device] [B, H, S, Dh], updated in place
 *   new_len             [device] int32 [B] out, or NULL; must not be seq_len itself
 * Errors: LPP_EINVAL (null, sizes < 1, new_len == seq_len), LPP_EUNSUPPORTED (dtype unknown, row
 * size not a multiple of 16 bytes), LPP_EHIP.
 */
int32_t lpp_commit_kv(const lpp_tree* tree, int32_t dtype, const void* k_tree, const void* v_tree,
                      const int32_t* path, const int32_t* accept_len, const int32_t* seq_len,
                      int32_t B, int32_t H, int32_t S, int32_t Dh, void* k_cache, void* v_cache,
                      int32_t* new_len, void* stream);

/* ----------------------------------------------------------------- probe ---
 * Measurement aid, not a step of the method: streams `bytes` (rounded down to a multiple of 16)
 * from src once with `blocks` workgroups of 256 lanes and writes nothing (sink may be NULL; it is
 * only there so that the reads cannot be optimised away).  Timed by the benchmark as the streaming
 * read ceiling of the device, next to the published HBM peak.
 *   src   [device] 16-byte aligned;  sink [device] uint32 or NULL
 * Errors: LPP_EINVAL (null src, bytes < 16, misaligned, blocks < 1 or > 2^20), LPP_EHIP.
 */
int32_t lpp_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, int32_t blocks, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LPP_H_ */
