// Internal declarations shared by the translation units of libnosa (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "../../include/nosa.h"

namespace nosa {

constexpr int kWave = 64;            // CDNA wavefront
constexpr int kBlockTokens = 64;     // n_b supported by this build
constexpr int kMaxTimed = 4096;      // launches kept per kernel between timing reads
constexpr int kMaxSelBlocks = 256;   // K limit of the decode kernel's slot table
constexpr int kMaxSelectBlocks = 4096;  // max_blocks limit of the selection kernel (LDS-resident keys)

struct Timing {
  hipEvent_t* start = nullptr;
  hipEvent_t* stop = nullptr;
  int n = 0;
};

}  // namespace nosa

struct nosa_ctx {
  nosa_params p;
  int group = 1;            // G = Hq / Hkv
  int units = 0;            // B * Hkv
  float scale = 0.f;        // softmax scale actually used
  int device = 0;
  hipStream_t main = nullptr;
  hipStream_t side = nullptr;
  hipEvent_t ev_select = nullptr;   // recorded on main after the selection kernel
  hipEvent_t ev_fetch = nullptr;    // recorded on side after the gather kernel
  bool select_recorded = false;
  bool fetch_pending = false;
  const int32_t* pending_load_list = nullptr;   // arguments of the fetch in flight (caller-owned, dev)
  const int32_t* pending_n_load = nullptr;
  int overlap = 1;
  int attention_kernel = 0; // 0 chosen from the shape, 1 vector-ALU kernel, 2 matrix-core kernel (bf16, G in {4,6,8,12,16})
  int merge_in_kernel = 1;  // split attention: the last workgroup of a unit merges (0: a separate combine launch)
  int fuse_stage1 = 1;      // nosa_decode_step runs scores + selection as one kernel when the shape allows
  int splits = 1;
  int fetch_wgs = 512;      // workgroups of the gather kernel (capped by the number of units)
  void* ws = nullptr;
  size_t ws_bytes = 0;
  void* static_scratch = nullptr;   // this device's copy of the library's static scratch array
  unsigned long long* trace = nullptr;   // nosa_set_trace: per-workgroup time stamps of the attention kernel (dev)
  int trace_capacity = 0;                // workgroups the trace buffer holds
  bool timing = false;
  bool capturing = false;             // between nosa_graph_begin and nosa_graph_end
  bool timing_before_capture = false;
  bool prefill_score_lds_set = false;    // dynamic-LDS limit of the prefill kernels raised (done once)
  bool prefill_attend_lds_set = false;
  const void* host_ok[3] = {nullptr, nullptr, nullptr};   // host pool pointers nosa_fetch has already vetted
  nosa::Timing timed[NOSA_KERNEL_COUNT];
  char err[512] = {0};
};

namespace nosa {

int set_error(nosa_ctx* ctx, int code, const char* fmt, ...);

// Brackets one kernel launch with events when timing is on.
struct TimedLaunch {
  nosa_ctx* ctx;
  int kernel;
  hipStream_t stream;
  int slot = -1;
  TimedLaunch(nosa_ctx* c, int k, hipStream_t s);
  ~TimedLaunch();
};

#define NOSA_HIP(ctx, call)                                                                   \
  do {                                                                                        \
    hipError_t e__ = (call);                                                                  \
    if (e__ != hipSuccess)                                                                    \
      return nosa::set_error((ctx), NOSA_EHIP, "%s failed: %s (%s:%d)", #call,                \
                             hipGetErrorString(e__), __FILE__, __LINE__);                     \
  } while (0)

#define NOSA_REQUIRE(ctx, cond, code, ...)                                                    \
  do {                                                                                        \
    if (!(cond)) return nosa::set_error((ctx), (code), __VA_ARGS__);                          \
  } while (0)

// kernel launchers (one per translation unit); all validate nothing: callers have done so
int launch_block_score(nosa_ctx* ctx, const void* q, const void* k_pooled, const float* se_pooled,
                       const int32_t* n_tokens, float* sq_blk, float* se_blk, int batch_div = 1);
int launch_select(nosa_ctx* ctx, const float* sq_blk, const float* se_blk, const int32_t* n_tokens,
                  int32_t* sel_idx, int32_t* n_sel, int32_t* slot_of_block, int32_t* block_of_slot,
                  int32_t* load_list, int32_t* n_load, int batch_mul = 1, int se_unit_div = 1,
                  int se_stride = 0);
int launch_score_select(nosa_ctx* ctx, const void* q, const void* k_pooled, const float* se_pooled,
                        const int32_t* n_tokens, float* sq_blk, float* se_blk, int32_t* sel_idx, int32_t* n_sel,
                        int32_t* slot_of_block, int32_t* block_of_slot, int32_t* load_list, int32_t* n_load);
bool score_select_supported(const nosa_params& p);
int launch_prefill_score(nosa_ctx* ctx, const void* q_chunk, const void* k_pooled, float* sq, int p0, int lq);
int launch_prefill_positions(nosa_ctx* ctx, int32_t* n_tok_virtual, int p0, int lq);
int launch_prefill_attend(nosa_ctx* ctx, const void* q_chunk, const void* cache_k, const void* cache_v,
                          const float* cache_bias, const int32_t* sel_idx, const int32_t* n_sel, int p0, int lq,
                          void* out, float* lse);
int launch_fetch(nosa_ctx* ctx, hipStream_t stream, const void* host_k, const void* host_v,
                 const float* host_bias, void* pool_k, void* pool_v, float* pool_bias,
                 const int32_t* load_list, const int32_t* n_load);
int launch_decode(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v,
                  const float* pool_bias, const int32_t* sel_idx, const int32_t* n_sel,
                  const int32_t* slot_of_block, const int32_t* n_tokens, void* out, float* lse,
                  hipEvent_t wait_fetch, const int32_t* load_list, const int32_t* n_load, void* ws,
                  size_t counter_bytes);
size_t decode_static_counter_bytes();
int decode_static_scratch(nosa_ctx* ctx, int device, void** out);
size_t decode_partial_bytes(const nosa_ctx* ctx);
size_t decode_counter_bytes(const nosa_ctx* ctx);
int decode_zero_counters(nosa_ctx* ctx, void* ws);
int launch_pool_blocks(nosa_ctx* ctx, const void* keys, const float* bias, const int32_t* n_tokens,
                       void* k_pooled, float* se_pooled);
int launch_append(nosa_ctx* ctx, const void* k_new, const void* v_new, const float* b_new, void* pool_k, void* pool_v,
                  float* pool_bias, void* host_k, void* host_v, float* host_bias, void* k_pooled, float* se_pooled,
                  const float* se_blk, int32_t* n_tokens, int32_t* slot_of_block, int32_t* block_of_slot);
int launch_split_qkv_evict(nosa_ctx* ctx, const void* qkv, const float* w1, const float* w2, int mode, void* q_out,
                           void* k_new, void* v_new, float* b_new);
int launch_fetch_tokens(nosa_ctx* ctx, hipStream_t stream, const void* host_k, const void* host_v, const float* host_bias,
                        void* pool_k, void* pool_v, float* pool_bias, const int32_t* token_list, const int32_t* n_list,
                        int max_list);
bool decode_supports_group(int g, int dtype);
int decode_default_splits(const nosa_params& p);

}  // namespace nosa
