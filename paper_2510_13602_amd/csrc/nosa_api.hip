// C-ABI entry points of libnosa: argument validation, context, stream ordering, timing.
// Every entry point validates before it launches; the kernels live in the other files.
#include <cmath>
#include <new>

#include "nosa_internal.h"

namespace {
thread_local char g_err[512] = {0};  // errors raised without a context
}

namespace nosa {

int set_error(nosa_ctx* ctx, int code, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 512, fmt, ap);
  va_end(ap);
  return code;
}

TimedLaunch::TimedLaunch(nosa_ctx* c, int k, hipStream_t s) : ctx(c), kernel(k), stream(s) {
  if (!ctx->timing) return;
  Timing& t = ctx->timed[kernel];
  if (t.n >= kMaxTimed) return;
  if (!t.start[t.n]) {
    // timing only: nothing synchronises with the host through these events, so they need no system-scope fence
    // (without it an event pair costs the stream less, and the durations are closer to the kernels' own)
    if (hipEventCreateWithFlags(&t.start[t.n], hipEventDisableSystemFence) != hipSuccess ||
        hipEventCreateWithFlags(&t.stop[t.n], hipEventDisableSystemFence) != hipSuccess)
      return;
  }
  slot = t.n;
  (void)hipEventRecord(t.start[slot], stream);
}

TimedLaunch::~TimedLaunch() {
  if (slot < 0) return;
  Timing& t = ctx->timed[kernel];
  (void)hipEventRecord(t.stop[slot], stream);
  t.n = slot + 1;
}

}  // namespace nosa

using nosa::set_error;

static int failf(char* msg, size_t len, int code, const char* fmt, ...) __attribute__((format(printf, 4, 5)));
static int failf(char* msg, size_t len, int code, const char* fmt, ...) {
  if (msg && len) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(msg, len, fmt, ap);
    va_end(ap);
  }
  return code;
}

static int validate(const nosa_params* p, char* msg, size_t len) {
#define fail(...) failf(msg, len, __VA_ARGS__)
  if (!p) return fail(NOSA_EINVAL, "params is NULL");
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1)
    return fail(NOSA_EINVAL, "batch, n_q_heads, n_kv_heads must be >= 1 (got %d, %d, %d)", p->batch,
                p->n_q_heads, p->n_kv_heads);
  if (p->n_q_heads % p->n_kv_heads != 0)
    return fail(NOSA_EINVAL, "n_q_heads (%d) must be a multiple of n_kv_heads (%d)", p->n_q_heads, p->n_kv_heads);
  if (p->dtype != NOSA_DTYPE_F32 && p->dtype != NOSA_DTYPE_BF16) return fail(NOSA_EINVAL, "unknown dtype %d", p->dtype);
  if (p->victim_policy != 0 && p->victim_policy != 1) return fail(NOSA_EINVAL, "unknown victim_policy %d", p->victim_policy);
  if (p->head_dim != 64 && p->head_dim != 128) return fail(NOSA_ESHAPE, "head_dim %d not in {64, 128}", p->head_dim);
  if (p->block_size != nosa::kBlockTokens) return fail(NOSA_ESHAPE, "block_size %d unsupported (64 only)", p->block_size);
  if (!nosa::decode_supports_group(p->n_q_heads / p->n_kv_heads, p->dtype))
    return fail(NOSA_ESHAPE, "GQA group %d unsupported (bf16: 1..16; fp32: 1, 2, 3, 4, 6, 8, 12, 16)", p->n_q_heads / p->n_kv_heads);
  if (p->pool_kernel < 1 || p->pool_stride < 1 || p->pool_kernel > p->block_size)
    return fail(NOSA_EINVAL, "pool_kernel (%d) must be in [1, block_size], pool_stride (%d) >= 1", p->pool_kernel,
                p->pool_stride);
  if (p->k_blocks < 1 || p->kq_blocks < 0 || p->sink_blocks < 0 || p->window_blocks < 1)
    return fail(NOSA_EINVAL, "need k_blocks >= 1, kq_blocks >= 0, sink_blocks >= 0, window_blocks >= 1");
  if (p->sink_blocks + p->window_blocks + p->kq_blocks > p->k_blocks)
    return fail(NOSA_ESHAPE, "budget: sink (%d) + window (%d) + kq (%d) exceeds k_blocks (%d)", p->sink_blocks,
                p->window_blocks, p->kq_blocks, p->k_blocks);
  if (p->k_blocks > nosa::kMaxSelBlocks) return fail(NOSA_ESHAPE, "k_blocks %d > %d", p->k_blocks, nosa::kMaxSelBlocks);
  if (p->gpu_slots < p->k_blocks) return fail(NOSA_ESHAPE, "gpu_slots (%d) < k_blocks (%d)", p->gpu_slots, p->k_blocks);
  if (p->victim_policy == 1 && p->gpu_slots > nosa::kMaxSelectBlocks)
    return fail(NOSA_ESHAPE, "victim_policy 1 supports at most %d gpu_slots", nosa::kMaxSelectBlocks);
  if (p->max_blocks < 1 || p->max_blocks > nosa::kMaxSelectBlocks)
    return fail(NOSA_ESHAPE, "max_blocks %d not in [1, %d]", p->max_blocks, nosa::kMaxSelectBlocks);
  if (p->n_sub_max < 0) return fail(NOSA_EINVAL, "n_sub_max < 0");
  {
    // every sub-block index that can be complete within max_blocks must fit the pooled arrays
    const long long tmax = 1LL * p->max_blocks * p->block_size;
    const long long need = tmax < p->pool_kernel ? 0 : (tmax - p->pool_kernel) / p->pool_stride + 1;
    if (p->n_sub_max > need) return fail(NOSA_EINVAL, "n_sub_max %d exceeds the %lld sub-blocks of max_blocks", p->n_sub_max, need);
  }
  if (!(p->softmax_scale == p->softmax_scale) || std::isinf(p->softmax_scale)) return fail(NOSA_EINVAL, "softmax_scale is not finite");
  if (msg && len) msg[0] = 0;
  return NOSA_OK;
#undef fail
}

extern "C" {

int nosa_validate_params(const nosa_params* p, char* msg, size_t msg_len) { return validate(p, msg, msg_len); }

const char* nosa_last_error(const nosa_ctx* ctx) { return ctx ? ctx->err : g_err; }

size_t nosa_workspace_bytes(const nosa_params* p) {
  if (validate(p, nullptr, 0) != NOSA_OK) return 0;
  const size_t units = (size_t)p->batch * p->n_kv_heads;
  const size_t g = p->n_q_heads / p->n_kv_heads;
  // two partitions (resident, fetched) x NOSA_MAX_SPLITS partial results per unit: O[g][d], (m, l)[g]
  const size_t per_part = g * (size_t)(p->head_dim + 2) * sizeof(float);
  const size_t counters = ((units * sizeof(int32_t)) + 255) & ~(size_t)255;   // one arrival counter per unit
  return counters + units * 2 * NOSA_MAX_SPLITS * per_part + 256;
}

int nosa_create(nosa_ctx** out, const nosa_params* p, void* main_stream) {
  if (!out) return set_error(nullptr, NOSA_EINVAL, "out is NULL");
  *out = nullptr;
  char msg[256];
  int rc = validate(p, msg, sizeof msg);
  if (rc != NOSA_OK) return set_error(nullptr, rc, "%s", msg);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
    return set_error(nullptr, NOSA_EHIP, "no HIP device available: libnosa has no CPU fallback");
  nosa_ctx* ctx = new (std::nothrow) nosa_ctx();
  if (!ctx) return set_error(nullptr, NOSA_EINVAL, "out of host memory");
  ctx->p = *p;
  ctx->group = p->n_q_heads / p->n_kv_heads;
  ctx->units = p->batch * p->n_kv_heads;
  ctx->scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
  ctx->main = (hipStream_t)main_stream;
  ctx->splits = nosa::decode_default_splits(*p);
  {
    // The gather beside the attention costs a fixed ~28 us of cross-stream waits and a second attention launch
    // per step and hides the attention over the resident blocks: it pays once that attention streams for longer
    // (from about 320 MB of selected keys and values per step on).  nosa_set_overlap overrides.
    const double kv_bytes = 2.0 * ctx->units * p->k_blocks * p->block_size * p->head_dim * (p->dtype == NOSA_DTYPE_F32 ? 4 : 2);
    ctx->overlap = kv_bytes >= 320e6 ? 1 : 0;
  }
  auto bail = [&](const char* what, hipError_t e) {
    set_error(nullptr, NOSA_EHIP, "%s failed: %s", what, hipGetErrorString(e));
    nosa_destroy(ctx);
    return NOSA_EHIP;
  };
  hipError_t e;
  if ((e = hipGetDevice(&ctx->device)) != hipSuccess) return bail("hipGetDevice", e);
  if (nosa::decode_static_scratch(nullptr, ctx->device, &ctx->static_scratch) != NOSA_OK) {
    nosa_destroy(ctx);
    return NOSA_EHIP;
  }
  if ((e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking)) != hipSuccess) return bail("hipStreamCreateWithFlags", e);
  if ((e = hipEventCreateWithFlags(&ctx->ev_select, hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
  if ((e = hipEventCreateWithFlags(&ctx->ev_fetch, hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
  for (int k = 0; k < NOSA_KERNEL_COUNT; ++k) {
    ctx->timed[k].start = new (std::nothrow) hipEvent_t[nosa::kMaxTimed]();
    ctx->timed[k].stop = new (std::nothrow) hipEvent_t[nosa::kMaxTimed]();
    if (!ctx->timed[k].start || !ctx->timed[k].stop) {
      nosa_destroy(ctx);
      return set_error(nullptr, NOSA_EINVAL, "out of host memory");
    }
  }
  *out = ctx;
  return NOSA_OK;
}

int nosa_destroy(nosa_ctx* ctx) {
  if (!ctx) return NOSA_OK;
  if (ctx->side) (void)hipStreamSynchronize(ctx->side);
  (void)hipStreamSynchronize(ctx->main);
  for (int k = 0; k < NOSA_KERNEL_COUNT; ++k) {
    nosa::Timing& t = ctx->timed[k];
    for (int i = 0; i < nosa::kMaxTimed; ++i) {
      if (t.start && t.start[i]) (void)hipEventDestroy(t.start[i]);
      if (t.stop && t.stop[i]) (void)hipEventDestroy(t.stop[i]);
    }
    delete[] t.start;
    delete[] t.stop;
  }
  if (ctx->ev_select) (void)hipEventDestroy(ctx->ev_select);
  if (ctx->ev_fetch) (void)hipEventDestroy(ctx->ev_fetch);
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  delete ctx;
  return NOSA_OK;
}

int nosa_set_workspace(nosa_ctx* ctx, void* dev_ws, size_t bytes) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, dev_ws, NOSA_EINVAL, "workspace is NULL");
  NOSA_REQUIRE(ctx, ((uintptr_t)dev_ws & 255) == 0, NOSA_EINVAL, "workspace must be 256-byte aligned");
  NOSA_REQUIRE(ctx, bytes >= nosa_workspace_bytes(&ctx->p), NOSA_EINVAL, "workspace too small: %zu < %zu", bytes,
               nosa_workspace_bytes(&ctx->p));
  ctx->ws = dev_ws;
  ctx->ws_bytes = bytes;
  return nosa::decode_zero_counters(ctx, dev_ws);
}

int nosa_set_attention_kernel(nosa_ctx* ctx, int which) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, which >= 0 && which <= 2, NOSA_EINVAL, "nosa_set_attention_kernel: %d not in {0, 1, 2}", which);
  ctx->attention_kernel = which;
  return NOSA_OK;
}

int nosa_set_merge_in_kernel(nosa_ctx* ctx, int on) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  ctx->merge_in_kernel = on ? 1 : 0;
  return NOSA_OK;
}

int nosa_set_splits(nosa_ctx* ctx, int splits) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, splits >= 1 && splits <= NOSA_MAX_SPLITS, NOSA_EINVAL, "splits %d not in [1, %d]", splits, NOSA_MAX_SPLITS);
  ctx->splits = splits;
  return NOSA_OK;
}

int nosa_get_splits(const nosa_ctx* ctx) { return ctx ? ctx->splits : NOSA_EINVAL; }

int nosa_set_fetch_workgroups(nosa_ctx* ctx, int workgroups) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, workgroups >= 1 && workgroups <= 65535, NOSA_EINVAL, "workgroups %d not in [1, 65535]", workgroups);
  ctx->fetch_wgs = workgroups;
  return NOSA_OK;
}

int nosa_set_fused_select(nosa_ctx* ctx, int on) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  ctx->fuse_stage1 = on ? 1 : 0;
  return NOSA_OK;
}

int nosa_set_overlap(nosa_ctx* ctx, int overlap) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  // a fetch in flight on the side stream must land before the ordering model changes
  if (ctx->fetch_pending) {
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, ctx->ev_fetch, 0));
    ctx->fetch_pending = false;
  }
  ctx->overlap = overlap ? 1 : 0;
  return NOSA_OK;
}

int nosa_block_score(nosa_ctx* ctx, const void* q, const void* k_pooled, const float* se_pooled,
                     const int32_t* n_tokens, float* sq_blk, float* se_blk) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, q && n_tokens && sq_blk && se_blk, NOSA_EINVAL, "nosa_block_score: NULL argument");
  NOSA_REQUIRE(ctx, ctx->p.n_sub_max == 0 || (k_pooled && se_pooled), NOSA_EINVAL,
               "nosa_block_score: k_pooled / se_pooled is NULL");
  return nosa::launch_block_score(ctx, q, k_pooled, se_pooled, n_tokens, sq_blk, se_blk);
}

int nosa_select(nosa_ctx* ctx, const float* sq_blk, const float* se_blk, const int32_t* n_tokens,
                int32_t* sel_idx, int32_t* n_sel, int32_t* slot_of_block, int32_t* block_of_slot,
                int32_t* load_list, int32_t* n_load) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, sq_blk && se_blk && n_tokens && sel_idx && n_sel && slot_of_block && block_of_slot && load_list && n_load,
               NOSA_EINVAL, "nosa_select: NULL argument");
  // The maps and the pool slots they describe may still be read by the previous step's fetch.
  if (ctx->fetch_pending) {
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, ctx->ev_fetch, 0));
    ctx->fetch_pending = false;
  }
  int rc = nosa::launch_select(ctx, sq_blk, se_blk, n_tokens, sel_idx, n_sel, slot_of_block, block_of_slot, load_list, n_load);
  if (rc != NOSA_OK) return rc;
  NOSA_HIP(ctx, hipEventRecord(ctx->ev_select, ctx->main));
  ctx->select_recorded = true;
  return NOSA_OK;
}

static int prefill_check(nosa_ctx* ctx, const char* who, int p0, int lq) {
  const nosa_params& p = ctx->p;
  NOSA_REQUIRE(ctx, p.dtype == NOSA_DTYPE_BF16, NOSA_ESHAPE, "%s: the prefill path is bf16 only", who);
  NOSA_REQUIRE(ctx, p.gpu_slots == p.max_blocks, NOSA_ESHAPE,
               "%s: the cache is addressed by block, gpu_slots (%d) must equal max_blocks (%d)", who, p.gpu_slots,
               p.max_blocks);
  NOSA_REQUIRE(ctx, p0 >= 0 && lq > 0 && p0 % p.block_size == 0 && lq % p.block_size == 0, NOSA_ESHAPE,
               "%s: p0 (%d) and lq (%d) must be multiples of the block size, lq > 0", who, p0, lq);
  NOSA_REQUIRE(ctx, (long long)p0 + lq <= (long long)p.max_blocks * p.block_size, NOSA_ESHAPE,
               "%s: p0 + lq = %lld exceeds the cache (%lld tokens)", who, (long long)p0 + lq,
               (long long)p.max_blocks * p.block_size);
  // one pooled key per block: the selection reads se_pooled and the score scratch by block index
  NOSA_REQUIRE(ctx, !(p.pool_kernel == p.block_size && p.pool_stride == p.block_size) ||
                        (long long)p.n_sub_max * p.block_size >= (long long)p0 + lq,
               NOSA_ESHAPE, "%s: n_sub_max (%d) pooled keys do not cover the %lld blocks of the prefix", who, p.n_sub_max,
               ((long long)p0 + lq) / p.block_size);
  NOSA_REQUIRE(ctx, (long long)p.batch * lq * p.n_kv_heads <= (1 << 24), NOSA_ESHAPE,
               "%s: B * lq * Hkv = %lld exceeds %d positions x KV heads per call: split the chunk", who,
               (long long)p.batch * lq * p.n_kv_heads, 1 << 24);
  return NOSA_OK;
}

int nosa_prefill_select(nosa_ctx* ctx, const void* q_chunk, const void* k_pooled, const float* se_pooled,
                        int32_t p0, int32_t lq, int32_t* n_tok_scratch, float* sq_scratch, float* se_scratch,
                        int32_t* sel_idx, int32_t* n_sel) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, q_chunk && k_pooled && se_pooled && n_tok_scratch && sq_scratch && se_scratch && sel_idx && n_sel,
               NOSA_EINVAL, "nosa_prefill_select: NULL argument");
  int rc = prefill_check(ctx, "nosa_prefill_select", p0, lq);
  if (rc != NOSA_OK) return rc;
  // every position is a batch element of its own that shares the pooled keys of its sequence
  rc = nosa::launch_prefill_positions(ctx, n_tok_scratch, p0, lq);
  if (rc != NOSA_OK) return rc;
  const nosa_params& p = ctx->p;
  if (p.pool_kernel == p.block_size && p.pool_stride == p.block_size) {
    // one pooled key per block: scores as one matrix product per unit; the block-level importance of a
    // complete block is its pooled importance, so the selection reads se_pooled itself
    rc = nosa::launch_prefill_score(ctx, q_chunk, k_pooled, sq_scratch, p0, lq);
    if (rc != NOSA_OK) return rc;
    return nosa::launch_select(ctx, sq_scratch, se_pooled, n_tok_scratch, sel_idx, n_sel, nullptr, nullptr, nullptr,
                               nullptr, lq, lq, p.n_sub_max);
  }
  rc = nosa::launch_block_score(ctx, q_chunk, k_pooled, se_pooled, n_tok_scratch, sq_scratch, se_scratch, lq);
  if (rc != NOSA_OK) return rc;
  return nosa::launch_select(ctx, sq_scratch, se_scratch, n_tok_scratch, sel_idx, n_sel, nullptr, nullptr, nullptr,
                             nullptr, lq);
}

int nosa_prefill_attend(nosa_ctx* ctx, const void* q_chunk, const void* cache_k, const void* cache_v,
                        const float* cache_bias, const int32_t* sel_idx, const int32_t* n_sel, int32_t p0,
                        int32_t lq, void* out, float* lse) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, q_chunk && cache_k && cache_v && cache_bias && sel_idx && n_sel && out && lse, NOSA_EINVAL,
               "nosa_prefill_attend: NULL argument");
  int rc = prefill_check(ctx, "nosa_prefill_attend", p0, lq);
  if (rc != NOSA_OK) return rc;
  return nosa::launch_prefill_attend(ctx, q_chunk, cache_k, cache_v, cache_bias, sel_idx, n_sel, p0, lq, out, lse);
}

int nosa_fetch(nosa_ctx* ctx, const void* host_k, const void* host_v, const float* host_bias,
               void* pool_k, void* pool_v, float* pool_bias, const int32_t* load_list, const int32_t* n_load) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, host_k && host_v && pool_k && pool_v && load_list && n_load, NOSA_EINVAL, "nosa_fetch: NULL argument");
  NOSA_REQUIRE(ctx, (host_bias == nullptr) == (pool_bias == nullptr), NOSA_EINVAL,
               "nosa_fetch: host_bias and pool_bias must both be given or both be NULL");
  // The gather kernel dereferences the host pointers on the GPU: they must be page-locked and mapped.
  // The query of the runtime is made once per pointer: a step that passes the same pools again pays nothing.
  const void* hp[3] = {host_k, host_v, host_bias};
  for (int i = 0; i < 3; ++i) {
    if (!hp[i] || hp[i] == ctx->host_ok[i]) continue;
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, hp[i]);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      return set_error(ctx, NOSA_EINVAL, "nosa_fetch: host pointer %d is not known to HIP (must be pinned or device memory)", i);
    }
    NOSA_REQUIRE(ctx, at.type == hipMemoryTypeHost || at.type == hipMemoryTypeDevice || at.type == hipMemoryTypeManaged,
                 NOSA_EINVAL, "nosa_fetch: host pointer %d is pageable host memory", i);
    ctx->host_ok[i] = hp[i];
  }
  hipStream_t s = ctx->main;
  if (ctx->overlap) {
    NOSA_REQUIRE(ctx, ctx->select_recorded, NOSA_EINVAL, "nosa_fetch called before any nosa_select");
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_select, 0));
    s = ctx->side;
  }
  int rc = nosa::launch_fetch(ctx, s, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, load_list, n_load);
  if (rc != NOSA_OK) return rc;
  if (ctx->overlap) {
    NOSA_HIP(ctx, hipEventRecord(ctx->ev_fetch, ctx->side));
    ctx->fetch_pending = true;
    ctx->pending_load_list = load_list;
    ctx->pending_n_load = n_load;
  }
  return NOSA_OK;
}

int nosa_fetch_tokens(nosa_ctx* ctx, const void* host_k, const void* host_v, const float* host_bias, void* pool_k,
                      void* pool_v, float* pool_bias, const int32_t* token_list, const int32_t* n_list, int32_t max_list) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, host_k && host_v && pool_k && pool_v && token_list && n_list && max_list >= 0, NOSA_EINVAL,
               "nosa_fetch_tokens: bad argument");
  NOSA_REQUIRE(ctx, (host_bias == nullptr) == (pool_bias == nullptr), NOSA_EINVAL,
               "nosa_fetch_tokens: host_bias and pool_bias must both be given or both be NULL");
  return nosa::launch_fetch_tokens(ctx, ctx->main, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, token_list, n_list,
                                   max_list);
}

static int sparse_decode(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v, const float* pool_bias,
                         const int32_t* sel_idx, const int32_t* n_sel, const int32_t* slot_of_block,
                         const int32_t* n_tokens, void* out, float* lse, void* ws, size_t counter_bytes) {
  // A gather in flight: the blocks it is writing are the ones in its load list; everything else in
  // the selection is already in place, so that part of the attention does not wait for it.
  hipEvent_t wait = nullptr;
  const int32_t *ll = nullptr, *nl = nullptr;
  if (ctx->fetch_pending) {
    wait = ctx->ev_fetch;
    ll = ctx->pending_load_list;
    nl = ctx->pending_n_load;
    ctx->fetch_pending = false;
  }
  return nosa::launch_decode(ctx, q, pool_k, pool_v, pool_bias, sel_idx, n_sel, slot_of_block, n_tokens, out, lse, wait, ll, nl, ws,
                             counter_bytes);
}

int nosa_sparse_decode(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v,
                       const float* pool_bias, const int32_t* sel_idx, const int32_t* n_sel,
                       const int32_t* slot_of_block, const int32_t* n_tokens, void* out, float* lse) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, q && pool_k && pool_v && sel_idx && n_sel && slot_of_block && n_tokens && out, NOSA_EINVAL,
               "nosa_sparse_decode: NULL argument");
  NOSA_REQUIRE(ctx, ctx->splits == 1 || ctx->ws, NOSA_EINVAL, "nosa_sparse_decode: no workspace set (nosa_set_workspace)");
  return sparse_decode(ctx, q, pool_k, pool_v, pool_bias, sel_idx, n_sel, slot_of_block, n_tokens, out, lse, ctx->ws,
                       nosa::decode_counter_bytes(ctx));
}

int nosa_sparse_decode_static(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v,
                              const float* pool_bias, const int32_t* sel_idx, const int32_t* n_sel,
                              const int32_t* slot_of_block, const int32_t* n_tokens, void* out, float* lse) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, q && pool_k && pool_v && sel_idx && n_sel && slot_of_block && n_tokens && out, NOSA_EINVAL,
               "nosa_sparse_decode_static: NULL argument");
  NOSA_REQUIRE(ctx, ctx->units <= NOSA_STATIC_SCRATCH_UNITS, NOSA_ESHAPE,
               "nosa_sparse_decode_static: %d units, the static scratch keeps arrival counters for %d", ctx->units,
               NOSA_STATIC_SCRATCH_UNITS);
  const size_t need = nosa::decode_static_counter_bytes() + nosa::decode_partial_bytes(ctx);
  NOSA_REQUIRE(ctx, need <= (size_t)NOSA_STATIC_SCRATCH_BYTES, NOSA_ESHAPE,
               "nosa_sparse_decode_static: %d units x %d splits x %d heads need %zu bytes of partial results, the static "
               "scratch holds %zu (use fewer splits, or nosa_sparse_decode with a workspace)",
               ctx->units, ctx->splits, ctx->group, need, (size_t)NOSA_STATIC_SCRATCH_BYTES);
  NOSA_REQUIRE(ctx, ctx->static_scratch, NOSA_EINVAL, "nosa_sparse_decode_static: the context has no static scratch");
  return sparse_decode(ctx, q, pool_k, pool_v, pool_bias, sel_idx, n_sel, slot_of_block, n_tokens, out, lse,
                       ctx->static_scratch, nosa::decode_static_counter_bytes());
}

// Stage 1 of the step in one launch: scores stay on chip between the score and the selection.
static int score_select(nosa_ctx* ctx, const nosa_step_args* a) {
  NOSA_REQUIRE(ctx, a->q && a->n_tokens && a->sel_idx && a->n_sel && a->slot_of_block && a->block_of_slot && a->load_list &&
                        a->n_load,
               NOSA_EINVAL, "nosa_decode_step: NULL argument");
  NOSA_REQUIRE(ctx, ctx->p.n_sub_max == 0 || (a->k_pooled && a->se_pooled), NOSA_EINVAL,
               "nosa_decode_step: k_pooled / se_pooled is NULL");
  if (ctx->fetch_pending) {   // the maps and the slots may still be in use by the previous step's fetch
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, ctx->ev_fetch, 0));
    ctx->fetch_pending = false;
  }
  int rc = nosa::launch_score_select(ctx, a->q, a->k_pooled, a->se_pooled, a->n_tokens, a->sq_blk, a->se_blk, a->sel_idx,
                                     a->n_sel, a->slot_of_block, a->block_of_slot, a->load_list, a->n_load);
  if (rc != NOSA_OK) return rc;
  NOSA_HIP(ctx, hipEventRecord(ctx->ev_select, ctx->main));
  ctx->select_recorded = true;
  return NOSA_OK;
}

static int run_step(nosa_ctx* ctx, const nosa_step_args* a) {
  int rc;
  if (ctx->fuse_stage1 && nosa::score_select_supported(ctx->p)) {
    rc = score_select(ctx, a);
    if (rc != NOSA_OK) return rc;
  } else {
    NOSA_REQUIRE(ctx, a->sq_blk && a->se_blk, NOSA_EINVAL,
                 "nosa_decode_step: sq_blk / se_blk may only be NULL when scores and selection run as one kernel");
    rc = nosa_block_score(ctx, a->q, a->k_pooled, a->se_pooled, a->n_tokens, a->sq_blk, a->se_blk);
    if (rc != NOSA_OK) return rc;
    rc = nosa_select(ctx, a->sq_blk, a->se_blk, a->n_tokens, a->sel_idx, a->n_sel, a->slot_of_block, a->block_of_slot,
                     a->load_list, a->n_load);
    if (rc != NOSA_OK) return rc;
  }
  rc = nosa_fetch(ctx, a->host_k, a->host_v, a->host_bias, a->pool_k, a->pool_v, a->pool_bias, a->load_list, a->n_load);
  if (rc != NOSA_OK) return rc;
  return nosa_sparse_decode(ctx, a->q, a->pool_k, a->pool_v, a->pool_bias, a->sel_idx, a->n_sel, a->slot_of_block,
                            a->n_tokens, a->out, a->lse);
}

int nosa_decode_step(nosa_ctx* ctx, const nosa_step_args* args) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, args, NOSA_EINVAL, "nosa_decode_step: args is NULL");
  return run_step(ctx, args);
}

struct nosa_graph {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

int nosa_graph_begin(nosa_ctx* ctx) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, ctx->main != nullptr, NOSA_EINVAL, "nosa_graph_begin: the default (NULL) stream cannot be captured");
  NOSA_REQUIRE(ctx, !ctx->capturing, NOSA_EINVAL, "nosa_graph_begin: a capture is already open on this context");
  if (ctx->fetch_pending) {   // nothing from before the capture may be waited on inside it
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, ctx->ev_fetch, 0));
    ctx->fetch_pending = false;
  }
  NOSA_HIP(ctx, hipStreamBeginCapture(ctx->main, hipStreamCaptureModeRelaxed));
  ctx->timing_before_capture = ctx->timing;
  ctx->timing = false;        // event pairs around kernels are not recorded into graphs
  ctx->capturing = true;
  return NOSA_OK;
}

int nosa_graph_end(nosa_ctx* ctx, nosa_graph** out) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, out, NOSA_EINVAL, "nosa_graph_end: out is NULL");
  *out = nullptr;
  NOSA_REQUIRE(ctx, ctx->capturing, NOSA_EINVAL, "nosa_graph_end without nosa_graph_begin");
  hipGraph_t graph = nullptr;
  const hipError_t e = hipStreamEndCapture(ctx->main, &graph);
  ctx->capturing = false;
  ctx->timing = ctx->timing_before_capture;
  ctx->fetch_pending = false;
  if (e != hipSuccess) {
    if (graph) (void)hipGraphDestroy(graph);
    return set_error(ctx, NOSA_EHIP, "hipStreamEndCapture failed: %s (a fetch without the attention call that joins it?)",
                     hipGetErrorString(e));
  }
  nosa_graph* g = new (std::nothrow) nosa_graph();
  if (!g) {
    (void)hipGraphDestroy(graph);
    return set_error(ctx, NOSA_EINVAL, "out of host memory");
  }
  g->graph = graph;
  const hipError_t ei = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
  if (ei != hipSuccess) {
    (void)hipGraphDestroy(g->graph);
    delete g;
    return set_error(ctx, NOSA_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(ei));
  }
  *out = g;
  return NOSA_OK;
}

int nosa_graph_create(nosa_ctx* ctx, const nosa_step_args* args, nosa_graph** out) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, args && out, NOSA_EINVAL, "nosa_graph_create: NULL argument");
  *out = nullptr;
  int rc = nosa_graph_begin(ctx);
  if (rc != NOSA_OK) return rc;
  rc = run_step(ctx, args);
  if (rc != NOSA_OK) {          // close the capture, keep the step's error message
    char keep[512];
    memcpy(keep, ctx->err, sizeof keep);
    nosa_graph* dropped = nullptr;
    (void)nosa_graph_end(ctx, &dropped);
    (void)nosa_graph_destroy(dropped);
    memcpy(ctx->err, keep, sizeof keep);
    return rc;
  }
  return nosa_graph_end(ctx, out);
}

int nosa_graph_launch(nosa_ctx* ctx, nosa_graph* graph) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, graph && graph->exec, NOSA_EINVAL, "nosa_graph_launch: no graph");
  if (ctx->fetch_pending) {
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, ctx->ev_fetch, 0));
    ctx->fetch_pending = false;
  }
  NOSA_HIP(ctx, hipGraphLaunch(graph->exec, ctx->main));
  return NOSA_OK;
}

int nosa_graph_destroy(nosa_graph* graph) {
  if (!graph) return NOSA_OK;
  if (graph->exec) (void)hipGraphExecDestroy(graph->exec);
  if (graph->graph) (void)hipGraphDestroy(graph->graph);
  delete graph;
  return NOSA_OK;
}

int nosa_pool_blocks(nosa_ctx* ctx, const void* keys, const float* bias, const int32_t* n_tokens,
                     void* k_pooled, float* se_pooled) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, keys && bias && n_tokens && k_pooled && se_pooled, NOSA_EINVAL, "nosa_pool_blocks: NULL argument");
  return nosa::launch_pool_blocks(ctx, keys, bias, n_tokens, k_pooled, se_pooled);
}

int nosa_split_qkv_evict(nosa_ctx* ctx, const void* qkv, const float* w1, const float* w2, int mode, void* q_out,
                         void* k_new, void* v_new, float* b_new) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, qkv && w1 && w2 && q_out && k_new && v_new && b_new, NOSA_EINVAL, "nosa_split_qkv_evict: NULL argument");
  NOSA_REQUIRE(ctx, mode == 0 || mode == 1, NOSA_EINVAL, "nosa_split_qkv_evict: mode %d not in {0, 1}", mode);
  return nosa::launch_split_qkv_evict(ctx, qkv, w1, w2, mode, q_out, k_new, v_new, b_new);
}

int nosa_append(nosa_ctx* ctx, const void* k_new, const void* v_new, const float* b_new, void* pool_k, void* pool_v,
                float* pool_bias, void* host_k, void* host_v, float* host_bias, void* k_pooled, float* se_pooled,
                const float* se_blk, int32_t* n_tokens, int32_t* slot_of_block, int32_t* block_of_slot) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, k_new && v_new && b_new && pool_k && pool_v && pool_bias && host_k && host_v && host_bias && se_blk &&
                        n_tokens && slot_of_block && block_of_slot,
               NOSA_EINVAL, "nosa_append: NULL argument");
  NOSA_REQUIRE(ctx, ctx->p.n_sub_max == 0 || (k_pooled && se_pooled), NOSA_EINVAL, "nosa_append: k_pooled / se_pooled is NULL");
  if (ctx->fetch_pending) {   // the gather of the previous step may still be writing slots
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, ctx->ev_fetch, 0));
    ctx->fetch_pending = false;
  }
  return nosa::launch_append(ctx, k_new, v_new, b_new, pool_k, pool_v, pool_bias, host_k, host_v, host_bias, k_pooled,
                             se_pooled, se_blk, n_tokens, slot_of_block, block_of_slot);
}

int nosa_set_trace(nosa_ctx* ctx, uint64_t* dev_buf, int32_t capacity_workgroups) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, capacity_workgroups >= 0 && (dev_buf || capacity_workgroups == 0), NOSA_EINVAL,
               "nosa_set_trace: a buffer is needed for a capacity of %d workgroups", capacity_workgroups);
  ctx->trace = (unsigned long long*)dev_buf;
  ctx->trace_capacity = dev_buf ? capacity_workgroups : 0;
  return NOSA_OK;
}

int nosa_timing_enable(nosa_ctx* ctx, int on) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  ctx->timing = on != 0;
  return NOSA_OK;
}

int nosa_timing_read(nosa_ctx* ctx, int kernel, double* total_ms, int32_t* launches) {
  NOSA_REQUIRE(ctx, ctx, NOSA_EINVAL, "ctx is NULL");
  NOSA_REQUIRE(ctx, kernel >= 0 && kernel < NOSA_KERNEL_COUNT && total_ms && launches, NOSA_EINVAL, "nosa_timing_read: bad argument");
  nosa::Timing& t = ctx->timed[kernel];
  double sum = 0.0;
  for (int i = 0; i < t.n; ++i) {
    NOSA_HIP(ctx, hipEventSynchronize(t.stop[i]));
    float ms = 0.f;
    NOSA_HIP(ctx, hipEventElapsedTime(&ms, t.start[i], t.stop[i]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = t.n;
  t.n = 0;
  return NOSA_OK;
}

}  // extern "C"
