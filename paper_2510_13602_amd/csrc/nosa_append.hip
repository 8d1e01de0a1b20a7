// Growing context (Alg. 1: cache update, update_compressed_k, update_importance_score): append the
// current token of every unit, give a newly opened block a slot, refresh the pooled arrays of the
// sub-blocks the token completes, advance n_tokens.  Three small launches, none on the timed path.
#include <cmath>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

struct AppendArgs {
  const void* k_new;
  const void* v_new;
  const float* b_new;
  void* pool_k;
  void* pool_v;
  float* pool_bias;
  void* host_k;
  void* host_v;
  float* host_bias;
  void* k_pooled;
  float* se_pooled;
  const float* se_blk;
  int32_t* n_tokens;
  int32_t* slot_of_block;
  int32_t* block_of_slot;
  int batch, n_kv_heads, head_dim, max_blocks, n_sub_max, gpu_slots, sink_blocks, window_blocks, pool_kernel, pool_stride, dtype;
};

using dev::f64_to_bf16;
using dev::order_key;

// one wavefront per unit
__global__ __launch_bounds__(kWave) void append_kernel(const AppendArgs a) {
  const int unit = blockIdx.x, lane = threadIdx.x;
  const int b = unit / a.n_kv_heads;
  const int t = a.n_tokens[b];
  if (t < 0 || t >= a.max_blocks * kBlockTokens) return;
  const int J = t / kBlockTokens, row = t % kBlockTokens;
  int32_t* sob = a.slot_of_block + (size_t)unit * a.max_blocks;
  int32_t* bos = a.block_of_slot + (size_t)unit * a.gpu_slots;
  const int es = a.dtype == NOSA_DTYPE_F32 ? 4 : 2;
  const int row_words = a.head_dim * es / 4;          // 32-bit words per row
  const uint32_t* ks = (const uint32_t*)a.k_new + (size_t)unit * row_words;
  const uint32_t* vs = (const uint32_t*)a.v_new + (size_t)unit * row_words;

  // host pool (device-initiated writes over the host link)
  const size_t hrow = ((size_t)unit * a.max_blocks + J) * kBlockTokens + row;
  for (int i = lane; i < row_words; i += kWave) {
    ((uint32_t*)a.host_k)[hrow * row_words + i] = ks[i];
    ((uint32_t*)a.host_v)[hrow * row_words + i] = vs[i];
  }
  if (lane == 0) a.host_bias[hrow] = a.b_new[unit];

  int slot = sob[J];
  if (row == 0 && slot < 0) {
    // lowest empty slot, else the least important resident candidate (ties: lower slot)
    const int protect = a.window_blocks;   // blocks J-Nw+1 .. J-1 stay in the window; J-Nw leaves it and may go
    const float* se = a.se_blk + (size_t)unit * a.max_blocks;
    unsigned long long best = ~0ull;
    for (int s = lane; s < a.gpu_slots; s += kWave)
      if (bos[s] < 0) best = min(best, (unsigned long long)s);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) best = min(best, (unsigned long long)__shfl_xor(best, off));
    if (best == ~0ull) {
      for (int s = lane; s < a.gpu_slots; s += kWave) {
        const int Jp = bos[s];
        if (Jp >= a.sink_blocks && Jp <= J - protect && Jp < a.max_blocks)
          best = min(best, ((unsigned long long)order_key(se[Jp]) << 32) | (unsigned long long)s);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) best = min(best, (unsigned long long)__shfl_xor(best, off));
    }
    if (best != ~0ull) {
      slot = (int)(best & 0xffffffffull);
      if (lane == 0) {
        const int old = bos[slot];
        if (old >= 0 && old < a.max_blocks) sob[old] = -1;
        bos[slot] = J;
        sob[J] = slot;
      }
    }
  }
  if (slot >= 0 && slot < a.gpu_slots) {
    const size_t prow = ((size_t)unit * a.gpu_slots + slot) * kBlockTokens + row;
    for (int i = lane; i < row_words; i += kWave) {
      ((uint32_t*)a.pool_k)[prow * row_words + i] = ks[i];
      ((uint32_t*)a.pool_v)[prow * row_words + i] = vs[i];
    }
    if (lane == 0) a.pool_bias[prow] = a.b_new[unit];
  }
}


// Pooled key / importance of the sub-block (if any) that ends with the token just appended.
// A sub-block j ends at token t iff t + 1 == j*ls + lk.  One workgroup of d threads per unit.
__global__ void append_pool_kernel(const AppendArgs a) {
  const int unit = blockIdx.x, e = threadIdx.x;
  const int b = unit / a.n_kv_heads;
  const int t = a.n_tokens[b];
  if (t < 0 || t >= a.max_blocks * kBlockTokens) return;
  const int lk = a.pool_kernel, ls = a.pool_stride, d = a.head_dim;
  const int end = t + 1;
  if (end < lk || (end - lk) % ls != 0) return;
  const int j = (end - lk) / ls;
  if (j >= a.n_sub_max) return;
  const size_t tok0 = (size_t)unit * a.max_blocks * kBlockTokens + (size_t)j * ls;
  const size_t out = ((size_t)unit * a.n_sub_max + j) * d + e;
  double s = 0.0;
  if (a.dtype == NOSA_DTYPE_F32) {
    const float* k = (const float*)a.host_k;
    for (int i = 0; i < lk; ++i) s += (double)k[(tok0 + i) * d + e];
    ((float*)a.k_pooled)[out] = (float)(s / (double)lk);
  } else {
    const uint16_t* k = (const uint16_t*)a.host_k;
    for (int i = 0; i < lk; ++i) s += (double)__uint_as_float((uint32_t)k[(tok0 + i) * d + e] << 16);
    ((uint16_t*)a.k_pooled)[out] = f64_to_bf16(s / (double)lk);
  }
  if (e == 0) {
    double sb = 0.0;
    for (int i = 0; i < lk; ++i) sb += (double)a.host_bias[tok0 + i];
    a.se_pooled[(size_t)unit * a.n_sub_max + j] = (float)(sb / (double)lk);
  }
}

__global__ void append_bump_kernel(int32_t* n_tokens, int batch, int cap) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < batch && n_tokens[b] >= 0 && n_tokens[b] < cap) n_tokens[b] += 1;
}

}  // namespace

int launch_append(nosa_ctx* ctx, const void* k_new, const void* v_new, const float* b_new, void* pool_k, void* pool_v,
                  float* pool_bias, void* host_k, void* host_v, float* host_bias, void* k_pooled, float* se_pooled,
                  const float* se_blk, int32_t* n_tokens, int32_t* slot_of_block, int32_t* block_of_slot) {
  const nosa_params& p = ctx->p;
  AppendArgs a{k_new, v_new, b_new, pool_k, pool_v, pool_bias, host_k, host_v, host_bias, k_pooled, se_pooled, se_blk,
               n_tokens, slot_of_block, block_of_slot, p.batch, p.n_kv_heads, p.head_dim, p.max_blocks, p.n_sub_max,
               p.gpu_slots, p.sink_blocks, p.window_blocks, p.pool_kernel, p.pool_stride, p.dtype};
  TimedLaunch tl(ctx, NOSA_KERNEL_APPEND, ctx->main);
  hipLaunchKernelGGL(append_kernel, dim3(ctx->units), dim3(kWave), 0, ctx->main, a);
  NOSA_HIP(ctx, hipGetLastError());
  if (p.n_sub_max > 0) {
    hipLaunchKernelGGL(append_pool_kernel, dim3(ctx->units), dim3(p.head_dim), 0, ctx->main, a);
    NOSA_HIP(ctx, hipGetLastError());
  }
  hipLaunchKernelGGL(append_bump_kernel, dim3((p.batch + 63) / 64), dim3(64), 0, ctx->main, n_tokens, p.batch,
                     p.max_blocks * p.block_size);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
