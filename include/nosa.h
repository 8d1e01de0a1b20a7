/*
 * libnosa — the decode-step hot path of NOSA (native and offloadable sparse attention) on one
 * AMD MI355X (gfx950): block score -> constrained block selection -> load positions -> fetch of
 * offloaded blocks from pinned host memory -> block-sparse attention over the selected blocks.
 *
 * Plain C ABI.  No call allocates or frees device memory; every tensor is owned by the caller.
 * "dev" = device memory, "host" = host memory, "pinned" = page-locked host memory that the GPU
 * can read (hipHostMalloc).  Unless stated, calls only enqueue work on the context's stream and
 * return without synchronising; they never read device memory from the host.
 *
 * Every call returns NOSA_OK (0) or a negative error code; nothing is launched when argument
 * validation fails, and no exception or abort crosses this boundary.  nosa_last_error() returns a
 * description of the last failure on the context (or of the last context-free failure).
 *
 * Notation (paper symbol -> field): block size n_b -> block_size; k/n_b -> k_blocks (K);
 * k_q/n_b -> kq_blocks (Kq); mean-pool kernel / stride l_k, l_s -> pool_kernel, pool_stride;
 * B batch, Hq query heads, Hkv KV heads, G = Hq/Hkv, d head_dim, T tokens in the cache,
 * N = ceil(T/n_b) blocks, C GPU slots per (batch, KV head).  A "unit" is one (batch, KV head).
 *
 * Tensor layouts (row-major, innermost last):
 *   q             [B, Hq, d]                 dtype            dev
 *   k_pooled      [B, Hkv, n_sub_max, d]     dtype            dev   pooled key of sub-block j
 *   se_pooled     [B, Hkv, n_sub_max]        fp32             dev   pooled importance of sub-block j
 *   n_tokens      [B]                        int32            dev   T per batch element (counts the current token)
 *   sq_blk,se_blk [B, Hkv, max_blocks]       fp32             dev   block-level scores, -inf = no score
 *   sel_idx       [B, Hkv, K]                int32            dev   Gamma(t), ascending, -1 padded
 *   n_sel         [B, Hkv]                   int32            dev
 *   slot_of_block [B, Hkv, max_blocks]       int32            dev   GPU slot of a block, -1 = not resident
 *   block_of_slot [B, Hkv, C]                int32            dev   block held by a slot, -1 = empty
 *   load_list     [B, Hkv, K, 2]             int32            dev   (block, slot) pairs to fetch, -1 padded
 *   n_load        [B, Hkv]                   int32            dev
 *   pool_k,pool_v [B, Hkv, C, n_b, d]        dtype            dev   paged GPU KV pool
 *   pool_bias     [B, Hkv, C, n_b]           fp32             dev   attention bias b_j of the pooled tokens
 *   host_k,host_v [B, Hkv, max_blocks, n_b, d] dtype          pinned  every block of the cache
 *   host_bias     [B, Hkv, max_blocks, n_b]  fp32             pinned
 *   out           [B, Hq, d]                 dtype            dev
 *   lse           [B, Hq]                    fp32             dev   natural-log sum of exp of the logits
 */
#ifndef NOSA_H
#define NOSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NOSA_OK 0
#define NOSA_EINVAL (-1) /* NULL / inconsistent argument, call out of order                      */
#define NOSA_ESHAPE (-2) /* a shape or budget this build does not support                       */
#define NOSA_EHIP (-3)   /* a HIP runtime call failed; nosa_last_error() names it               */

#define NOSA_DTYPE_F32 0
#define NOSA_DTYPE_BF16 1

typedef struct nosa_ctx nosa_ctx; /* opaque: parameters, streams, events, workspace */

/* The hyper-parameter bag of Alg. 1 ("params": k, k_e, k_q, block size, pooling strides) plus the
 * tensor geometry.  Budget split as in App. B.2: K = sink + window + Kq + Ke, so
 * Ke = K - sink_blocks - window_blocks - kq_blocks is implied and must be >= 0.               */
typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* B, Hq, Hkv, d; d in {64, 128}; Hq % Hkv == 0  */
  int32_t block_size;                             /* n_b; this build supports 64                   */
  int32_t pool_kernel, pool_stride;               /* l_k, l_s; both == n_b => one pooled key/block  */
  int32_t k_blocks, kq_blocks;                    /* K, Kq (Kq bounds the blocks fetched per step)   */
  int32_t sink_blocks, window_blocks;             /* Ns >= 0, Nw >= 1 (the window holds the tail)    */
  int32_t gpu_slots;                              /* C >= K                                         */
  int32_t max_blocks;                             /* capacity of the per-unit block tables          */
  int32_t n_sub_max;                              /* capacity of k_pooled / se_pooled per unit      */
  int32_t dtype;                                  /* NOSA_DTYPE_F32 or NOSA_DTYPE_BF16 (q, K, V, out) */
  int32_t victim_policy;                          /* which free slots a miss overwrites: 0 ascending slot
                                                     order; 1 empty slots, then the least important block
                                                     (smallest se_blk) first -- matters only when C > K      */
  float softmax_scale;                            /* multiplies q.k only; <= 0 selects 1/sqrt(d)     */
} nosa_params;

/* ---- context ---------------------------------------------------------------------------------*/

/* Pure host check of a parameter set (no GPU needed).  Returns NOSA_OK, NOSA_EINVAL or NOSA_ESHAPE;
 * when msg != NULL a description of the first problem is copied into it (at most msg_len bytes). */
int nosa_validate_params(const nosa_params* p, char* msg, size_t msg_len);

/* Creates a context for one layer shape.  main_stream is a hipStream_t (NULL = the default
 * stream) on which score, select and decode are enqueued; the context creates one more stream of
 * default priority for fetches, and the events that order the two.  The current device at the
 * time of the call is the context's device.                                                      */
int nosa_create(nosa_ctx** out, const nosa_params* p, void* main_stream);
int nosa_destroy(nosa_ctx* ctx); /* synchronises both streams, destroys them; frees no caller memory */

/* Scratch for the split partial results of nosa_sparse_decode.  The caller allocates
 * nosa_workspace_bytes() bytes of device memory (256-byte aligned) and hands them over once; the
 * buffer must stay valid until nosa_destroy and belongs to this context alone (contexts must not
 * share one).  nosa_set_workspace enqueues one small kernel on the context's stream that zeroes the
 * per-unit arrival counters at the start of the buffer.                                           */
size_t nosa_workspace_bytes(const nosa_params* p);
int nosa_set_workspace(nosa_ctx* ctx, void* dev_ws, size_t bytes);

/* Number of partial results per unit in nosa_sparse_decode (1..NOSA_MAX_SPLITS); the default is
 * chosen from the shape so that the launch fills whole rounds of 512 workgroups with as few partial
 * results as possible (1 at 512 units, 4 at 128, 5 at 96).  The workspace is sized for
 * NOSA_MAX_SPLITS.                                                                              */
#define NOSA_MAX_SPLITS 16
int nosa_set_splits(nosa_ctx* ctx, int splits);
int nosa_get_splits(const nosa_ctx* ctx);

/* Which kernel nosa_sparse_decode runs.
 * 2, the matrix-core kernel (bf16 only): the (up to 16) heads of a group are the N dimension of
 * v_mfma_f32_16x16x32_bf16, K feeds the score product straight from global memory, V is transposed
 * through LDS, the softmax weights are rounded to bf16 (nearest even) for the second product while the row
 * sums keep the unrounded ones.  Its cost does not depend on G: it streams K and V at the same rate for
 * G = 1 and for the G = 16 of the paper's own 3B and 8B models (32 query / 2 KV heads).
 * 1, the vector-ALU kernel (fp32 and bf16): K and V stream through registers in full lines, q.k by packed dot
 * products, P.V by fp32 FMAs; 4 G flops per byte, so it falls behind from G = 6 on and spills at G = 16.
 * 0 (default): 2 for bf16, 1 for fp32.  A request for 2 on an fp32 context runs 1.
 * Group sizes G = Hq / Hkv: kernel 2 takes the group as an argument, any G in 1..16; kernel 1 is
 * instantiated for G in {1, 2, 3, 4, 6, 8, 12, 16}.  So bf16 contexts accept every G up to 16 (a request
 * for kernel 1 with another G runs 2), fp32 contexts the listed ones; nosa_validate_params says which. */
int nosa_set_attention_kernel(nosa_ctx* ctx, int which);

/* With several splits, who merges the partial results of a unit: 1 (default) the workgroup of the
 * attention kernel that finds all the others of its unit done (an arrival counter per unit, nobody
 * waits); 0 a separate combine launch.  Same arithmetic in the same order, same result.           */
int nosa_set_merge_in_kernel(nosa_ctx* ctx, int on);

/* overlap = 1: fetches run on the context's own stream; a nosa_sparse_decode that follows
 * a nosa_fetch first attends the selected blocks that are not in that fetch's load list, then waits
 * for the fetch, attends the fetched blocks and merges.  overlap = 0: everything is enqueued on the
 * main stream in call order.  Same selections, outputs equal up to the summation order of the merge.
 * Default: 1 when the selected keys and values of a step (units x K x block x d x 2) are at least
 * 320 MB, else 0 -- the second attention launch and the cross-stream waits cost about 28 us per step,
 * which the hidden attention time has to exceed (8B shape: 1.62 -> 1.50 ms; 1B shape: 0.116 -> 0.144). */
int nosa_set_overlap(nosa_ctx* ctx, int overlap);

/* Size of the gather kernel's persistent grid (default 512, capped by the number of units).  Each
 * workgroup keeps 4 KiB of host reads in flight (16 KiB when there are fewer than 256): more workgroups raise the link throughput (36 GB/s
 * at 16, 52 at 64, 56 at 512 on PCIe Gen5 x16) but slow HBM reads of kernels that run beside it.   */
int nosa_set_fetch_workgroups(nosa_ctx* ctx, int workgroups);

const char* nosa_last_error(const nosa_ctx* ctx); /* ctx may be NULL */

/* ---- the hot path (Alg. 1, one decode step of one layer) -------------------------------------*/

/* Stage 1, scores.  S_c^q = Q K_c^T (Sec. 2.1), summed over the G query heads of each KV head,
 * then the block-level max over the sub-blocks that lie wholly inside a block, applied
 * identically to the query-aware score and to the pooled importance score (mean-pooling and
 * max-pooling Eqs. of Sec. 3.1; "fused_pooling" in Alg. 1).  Sub-block j covers tokens
 * [j*l_s, j*l_s + l_k) and exists once all its tokens do.  Raw dot products: no scale, no softmax.
 * Writes sq_blk and se_blk for every block index < max_blocks (-inf where a block has no complete
 * sub-block).  All pointers dev.                                                                 */
int nosa_block_score(nosa_ctx* ctx, const void* q, const void* k_pooled, const float* se_pooled,
                     const int32_t* n_tokens, float* sq_blk, float* se_blk);

/* Stage 1, selection, and the load positions.
 * Selection (selection Eq. of Sec. 3.1; Alg. 1 select_topk_indices): sink blocks and the last
 * window_blocks blocks are forced (InfLLMv2 mask, Sec. 2.1); among the remaining complete blocks
 * the Kq best by sq_blk are taken, then the Ke best of the rest by se_blk; ties go to the lower
 * block index.  sel_idx receives Gamma(t) in ascending order.
 * Load positions (Sec. 4 "Memory Layout and Block Selection"; Alg. 1 generate_load_positions):
 * the selected blocks without a slot, in ascending order, are paired with the slots (ascending)
 * that are empty or hold a block outside Gamma(t) (with victim_policy 1: of those slots, the empty
 * ones and then the ones whose block has the smallest se_blk are used, handed out in ascending slot
 * order); both residency maps are updated in place and the pairs are written to load_list / n_load.  With C == K and an unchanged cache, n_load <= Kq
 * on every step after the first (Theorem 1).  All pointers dev; nothing is read back.            */
int nosa_select(nosa_ctx* ctx, const float* sq_blk, const float* se_blk, const int32_t* n_tokens,
                int32_t* sel_idx, int32_t* n_sel, int32_t* slot_of_block, int32_t* block_of_slot,
                int32_t* load_list, int32_t* n_load);

/* Host-to-device transfer of the missed blocks (Sec. 4 "Offloading Communication"; Alg. 1
 * host_to_device_communication): a gather kernel reads each listed block's keys, values and bias
 * straight from pinned host memory and writes them into the block's slot.  host_* are pinned host
 * pointers (host_bias and pool_bias may both be NULL); pool_*, load_list, n_load are dev.
 * Ordered after the preceding nosa_select and before the following nosa_sparse_decode.           */
int nosa_fetch(nosa_ctx* ctx, const void* host_k, const void* host_v, const float* host_bias,
               void* pool_k, void* pool_v, float* pool_bias, const int32_t* load_list,
               const int32_t* n_load);

/* Element-wise counterpart of nosa_fetch, for the block-wise versus element-wise comparison of
 * Sec. 3.2 ("Comparison with DMA"): copies single token rows.  token_list [B,Hkv,max_list,2] dev holds
 * (token index in the host cache, row index in the unit's pool viewed as C*n_b rows); n_list [B,Hkv] dev.
 * Runs on the main stream (a study entry point, not part of the decode step).                     */
int nosa_fetch_tokens(nosa_ctx* ctx, const void* host_k, const void* host_v, const float* host_bias,
                      void* pool_k, void* pool_v, float* pool_bias, const int32_t* token_list,
                      const int32_t* n_list, int32_t max_list);

/* Stage 2, attention (output Eq. of Sec. 3.1 "Attention Calculation"): for every query head,
 * softmax over the tokens j < T of the selected blocks of  softmax_scale * q.k_j + b_j, times V;
 * exp(b_j) exp(q k_j + m_j) of the paper is the same thing with the mask m_j realised by visiting
 * only selected blocks.  pool_bias may be NULL (b = 0); lse may be NULL.  Every selected block
 * must have a slot (nosa_select guarantees it).  All pointers dev.                               */
int nosa_sparse_decode(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v,
                       const float* pool_bias, const int32_t* sel_idx, const int32_t* n_sel,
                       const int32_t* slot_of_block, const int32_t* n_tokens, void* out, float* lse);

/* nosa_sparse_decode for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same
 * kernels and same result, but the split partial results live in a scratch array of
 * NOSA_STATIC_SCRATCH_BYTES that is part of the library's device code (one copy per GPU, held until the
 * process ends) instead of in the workspace of nosa_set_workspace, which need not be set.  The call
 * allocates nothing.  The array holds NOSA_STATIC_SCRATCH_UNITS arrival counters (a fixed region, whatever the
 * shape of the context) followed by the partial results, units x splits x G x (d + 2) x 4 bytes; the call
 * returns NOSA_ESHAPE when the context has more units than that or when the partial results do not fit
 * (lower nosa_set_splits, or use nosa_sparse_decode).  The array starts at zero
 * when the library is loaded and only the per-unit arrival counters at its start rely on that: every launch
 * leaves them at zero again; partial results are written before they are read.  All contexts of a process
 * share a GPU's array and it keeps the last call's contents, so two such calls that overlap in time
 * on one GPU (different streams, or a graph replay beside an eager call) race; calls on one stream
 * are ordered.                                                                                     */
#define NOSA_STATIC_SCRATCH_BYTES (8u << 20)
#define NOSA_STATIC_SCRATCH_UNITS 16384
int nosa_sparse_decode_static(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v,
                              const float* pool_bias, const int32_t* sel_idx, const int32_t* n_sel,
                              const int32_t* slot_of_block, const int32_t* n_tokens, void* out, float* lse);

/* One whole decode step of one layer = the four calls above, in the order of Alg. 1, behind one
 * entry point (one boundary crossing per step instead of four).  Every field has the meaning and
 * memory kind of the like-named argument above; host_bias / pool_bias may both be NULL, lse may be
 * NULL.
 * With one pooled key per block (pool_kernel == pool_stride == block_size) and at most 1024 blocks
 * (and slots) per unit, Stage 1 runs as ONE kernel: a workgroup per unit streams the unit's pooled
 * keys, keeps the block scores in LDS and selects from there (same arithmetic and same results as
 * nosa_block_score followed by nosa_select).  sq_blk and se_blk are then optional outputs: pass NULL
 * and the scores never travel through HBM (nosa_append needs se_blk: keep it for a growing context).
 * nosa_set_fused_select(ctx, 0) switches back to the two separate kernels.                        */
typedef struct {
  const void* q;
  const void* k_pooled;
  const float* se_pooled;
  const int32_t* n_tokens;
  float* sq_blk;
  float* se_blk;
  int32_t* sel_idx;
  int32_t* n_sel;
  int32_t* slot_of_block;
  int32_t* block_of_slot;
  int32_t* load_list;
  int32_t* n_load;
  const void* host_k;
  const void* host_v;
  const float* host_bias;
  void* pool_k;
  void* pool_v;
  float* pool_bias;
  void* out;
  float* lse;
} nosa_step_args;
int nosa_decode_step(nosa_ctx* ctx, const nosa_step_args* args);
int nosa_set_fused_select(nosa_ctx* ctx, int on);

/* The same step recorded once into a HIP graph (Sec. 4 "Kernel Fusion": the paper captures the
 * launch-bound part of the step in a graph) and replayed with one launch.  All pointers are baked
 * in: the caller refreshes the contents of q (and of the cache tensors) in place between replays.
 * The graph holds kernel nodes on two branches (gather | attention over resident blocks) joined
 * before the attention over fetched blocks; it contains no memset nodes.  Kernel timing is not
 * recorded for replays.  nosa_graph_launch enqueues on the context's main stream.                 */
typedef struct nosa_graph nosa_graph;
int nosa_graph_create(nosa_ctx* ctx, const nosa_step_args* args, nosa_graph** out);
/* The general form: every libnosa call made on the context between nosa_graph_begin and nosa_graph_end
 * is recorded instead of run (stream capture of the context's main stream; the fetch stream joins and
 * leaves the capture through the context's events), e.g. the step of a growing context,
 * nosa_split_qkv_evict -> nosa_append -> nosa_decode_step, as one graph.  A recorded fetch must be
 * followed by the attention call that waits for it before nosa_graph_end.  Only calls that enqueue
 * kernels belong in between (no nosa_set_workspace, nosa_timing_read, nosa_destroy).               */
int nosa_graph_begin(nosa_ctx* ctx);
int nosa_graph_end(nosa_ctx* ctx, nosa_graph** out);
int nosa_graph_launch(nosa_ctx* ctx, nosa_graph* graph);
int nosa_graph_destroy(nosa_graph* graph);

/* ---- cache maintenance (Alg. 1 update_compressed_k / update_importance_score) ----------------*/

/* Rebuilds k_pooled and se_pooled from a whole cache: K_c[j] = mean of the keys of sub-block j
 * (block compression f_c, Sec. 2.1), S_c^e[j] = mean of the importance score b over it (mean-pooling
 * Eq.).  keys [B,Hkv,max_blocks,n_b,d] and bias [B,Hkv,max_blocks,n_b] may be dev or pinned host
 * memory.  Sums in fp64 in token order and rounds once (K_c to dtype, nearest even; S_c^e to fp32), so
 * the pooled arrays do not depend on any blocking of the sum and two implementations of this
 * definition agree bit for bit.  Sub-blocks not complete at n_tokens are written as zero.  Not part
 * of the timed path.                                                                            */
int nosa_pool_blocks(nosa_ctx* ctx, const void* keys, const float* bias, const int32_t* n_tokens,
                     void* k_pooled, float* se_pooled);

/* Upstream of the cache update (Alg. 1 fused_linear_projection; Sec. 4 "Kernel Fusion": the eviction
 * head is fused with the split of the QKV tensor).  qkv [B, (Hq + 2 Hkv) d] dtype holds, per token,
 * all query heads, then all key heads, then all value heads.  w1 [d, Hkv] and w2 [Hkv] are the fp32
 * eviction-head weights (importance-score Eq., Sec. 3.1; tau = softplus, no final exp: ED-DMA).
 *   mode 0 (table of App. D, one gate per KV head):  b[b,h] = softplus(v_h . w1[:,h]) * w2[h]
 *   mode 1 (the Eq. as printed, shared by the heads): b[b,h] = sum_m softplus(v_h . w1[:,m]) * w2[m]
 * Outputs: q_out [B,Hq,d], k_new, v_new [B,Hkv,d] (bit copies, ready for RoPE and nosa_append) and
 * b_new [B,Hkv] fp32.  All pointers dev.                                                          */
int nosa_split_qkv_evict(nosa_ctx* ctx, const void* qkv, const float* w1, const float* w2, int mode,
                         void* q_out, void* k_new, void* v_new, float* b_new);

/* Appends the current token of every unit (Alg. 1: the cache engine is updated before Stage 1).
 * k_new, v_new [B,Hkv,d] dtype, b_new [B,Hkv] fp32, all dev.  Token t = n_tokens[b] goes to block
 * J = t / n_b, row t % n_b of the host pool (written by the GPU over the host link) and, when block J
 * has a slot, to that slot.  A token that opens a new block first gives the block a slot: the lowest
 * empty slot, else the slot of the resident block with the smallest se_blk (block-level importance
 * as written by the last nosa_block_score; ties: lower slot) among blocks that are neither sink
 * blocks nor among the Nw - 1 blocks before J that stay in the window (the block that leaves the
 * window, J - Nw, is a candidate like any other); if there is none the block stays
 * non-resident and the next nosa_select lists it as a miss.  Evicting the least important candidate
 * keeps the per-step fetch bound of Theorem 1 across block boundaries.  Then every sub-block that
 * this token completes gets its pooled key and pooled importance (same arithmetic as
 * nosa_pool_blocks, read back from the host pool), and n_tokens[b] is incremented.  Tokens beyond
 * max_blocks * n_b are ignored.  Not part of the timed path.                                      */
int nosa_append(nosa_ctx* ctx, const void* k_new, const void* v_new, const float* b_new,
                void* pool_k, void* pool_v, float* pool_bias, void* host_k, void* host_v, float* host_bias,
                void* k_pooled, float* se_pooled, const float* se_blk, int32_t* n_tokens,
                int32_t* slot_of_block, int32_t* block_of_slot);

/* ---- sparse prefill (sparse attention in both stages; results Table, "Sparse Prefill" rows) ---
 *
 * A chunk of lq query positions p0 .. p0+lq-1 per batch element, whose keys, values and biases are
 * already in the cache and whose complete blocks are already pooled (nosa_pool_blocks).  Position t
 * of the chunk behaves like a decode step with n_tokens = p0 + t + 1: the same scores, the same
 * constrained selection (selection Eq., Sec. 3.1), the same biased softmax (Sec. 3.2) over the
 * selected tokens, none of which is in its future.  Nothing is offloaded during prefill, so the
 * cache is addressed by block: cache_k, cache_v [B,Hkv,max_blocks,n_b,d], cache_bias
 * [B,Hkv,max_blocks,n_b] fp32 (the pool layout with slot = block; needs gpu_slots == max_blocks).
 * Restrictions: bf16, p0 and lq multiples of n_b = 64, p0 + lq <= max_blocks * n_b.  All pointers dev.
 *
 * nosa_prefill_select: q_chunk [B,lq,Hq,d] -> sel_idx [B,lq,Hkv,K] (ascending, -1 padded) and n_sel
 * [B,lq,Hkv].  Scratch owned by the caller: n_tok_scratch int32 [B*lq], sq_scratch and se_scratch
 * fp32 [B*lq*Hkv*max_blocks].  Afterwards sq_scratch holds the query-aware block scores of every
 * position for the complete blocks of its prefix (other entries unspecified); se_scratch is only
 * written when the pooling windows differ from the blocks (pool_kernel or pool_stride != n_b).
 *
 * nosa_prefill_attend: out [B,lq,Hq,d] (dtype) and lse [B,lq,Hq] fp32 from the selection above.  */
int nosa_prefill_select(nosa_ctx* ctx, const void* q_chunk, const void* k_pooled, const float* se_pooled,
                        int32_t p0, int32_t lq, int32_t* n_tok_scratch, float* sq_scratch, float* se_scratch,
                        int32_t* sel_idx, int32_t* n_sel);
int nosa_prefill_attend(nosa_ctx* ctx, const void* q_chunk, const void* cache_k, const void* cache_v,
                        const float* cache_bias, const int32_t* sel_idx, const int32_t* n_sel, int32_t p0,
                        int32_t lq, void* out, float* lse);

/* ---- per-kernel timing for benchmarks --------------------------------------------------------*/

#define NOSA_KERNEL_SCORE 0
#define NOSA_KERNEL_SELECT 1
#define NOSA_KERNEL_FETCH 2
#define NOSA_KERNEL_DECODE 3  /* the split attention kernel (dominant) */
#define NOSA_KERNEL_COMBINE 4 /* merge of split results, or the second (fetched blocks + merge) launch */
#define NOSA_KERNEL_EVICT 5   /* nosa_split_qkv_evict                                           */
#define NOSA_KERNEL_APPEND 6  /* the launches of nosa_append together                           */
#define NOSA_KERNEL_PREFILL 7 /* the attention kernel of nosa_prefill_attend                    */
#define NOSA_KERNEL_COUNT 8
/* When enabled, each launch of the kernels above is bracketed by HIP events on the stream it runs
 * on.  nosa_timing_read synchronises those events, returns the summed duration and the number of
 * launches since the last read, and resets the counters.  At most 4096 launches per kernel are
 * kept between reads.                                                                           */
int nosa_timing_enable(nosa_ctx* ctx, int on);

/* Diagnostics: with a trace buffer set (dev, 4 x uint64 per workgroup, capacity in workgroups), every
 * workgroup of the stand-alone attention kernel (nosa_sparse_decode with no fetch in flight) records
 * {start, end} in ticks of the GPU's 100 MHz real-time counter, the XCD it ran on and its index.  A
 * launch with more workgroups (units x splits) than the capacity records nothing.  NULL switches it off. */
int nosa_set_trace(nosa_ctx* ctx, uint64_t* dev_buf, int32_t capacity_workgroups);
int nosa_timing_read(nosa_ctx* ctx, int kernel, double* total_ms, int32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* NOSA_H */
