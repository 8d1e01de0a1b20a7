// Split of the fused QKV activation of the current token and the eviction head on its value
// (importance-score Eq. of Sec. 3.1; ED-DMA: b = softplus(v W1) (.) W2 with no final exp; fused with
// the QKV split as in Sec. 4 "Kernel Fusion").  One wavefront per (batch element, head row): query and
// key rows are copied, value rows are copied and reduced against W1.  The work is a few hundred KiB:
// the point of the fusion is one launch instead of several.
#include <cmath>

#include "nosa_internal.h"

namespace nosa {
namespace {

struct EvictArgs {
  const void* qkv;
  const float* w1;   // [d, Hkv]
  const float* w2;   // [Hkv]
  void* q_out;
  void* k_new;
  void* v_new;
  float* b_new;
  int n_q_heads, n_kv_heads, head_dim, dtype, mode;
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

__device__ __forceinline__ float softplus(float x) { return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x))); }

__global__ __launch_bounds__(kWave) void split_qkv_evict_kernel(const EvictArgs a) {
  const int rows = a.n_q_heads + 2 * a.n_kv_heads;
  const int b = blockIdx.x / rows, row = blockIdx.x % rows;
  const int lane = threadIdx.x, d = a.head_dim, Hq = a.n_q_heads, H = a.n_kv_heads;
  const size_t src = ((size_t)b * rows + row) * d;
  void* dst;
  size_t dst_off;
  if (row < Hq) { dst = a.q_out; dst_off = ((size_t)b * Hq + row) * d; }
  else if (row < Hq + H) { dst = a.k_new; dst_off = ((size_t)b * H + (row - Hq)) * d; }
  else { dst = a.v_new; dst_off = ((size_t)b * H + (row - Hq - H)) * d; }
  const bool is_v = row >= Hq + H;
  const int h = row - Hq - H;
  float part[16];   // partial dots against the columns of W1 this row needs (Hkv <= 16 in mode 1)
#pragma unroll
  for (int m = 0; m < 16; ++m) part[m] = 0.f;
  for (int e = lane; e < d; e += kWave) {
    float x;
    if (a.dtype == NOSA_DTYPE_F32) {
      x = ((const float*)a.qkv)[src + e];
      ((float*)dst)[dst_off + e] = x;
    } else {
      const uint16_t u = ((const uint16_t*)a.qkv)[src + e];
      ((uint16_t*)dst)[dst_off + e] = u;
      x = __uint_as_float((uint32_t)u << 16);
    }
    if (is_v) {
      if (a.mode == 0) {
        part[0] = fmaf(x, a.w1[(size_t)e * H + h], part[0]);
      } else {
#pragma unroll
        for (int m = 0; m < 16; ++m)
          if (m < H) part[m] = fmaf(x, a.w1[(size_t)e * H + m], part[m]);
      }
    }
  }
  if (!is_v) return;
  float acc;
  if (a.mode == 0) {
    acc = softplus(wave_sum(part[0])) * a.w2[h];
  } else {
    acc = 0.f;
#pragma unroll
    for (int m = 0; m < 16; ++m)
      if (m < H) acc = fmaf(softplus(wave_sum(part[m])), a.w2[m], acc);
  }
  if (lane == 0) a.b_new[(size_t)b * H + h] = acc;
}

}  // namespace

int launch_split_qkv_evict(nosa_ctx* ctx, const void* qkv, const float* w1, const float* w2, int mode, void* q_out,
                           void* k_new, void* v_new, float* b_new) {
  const nosa_params& p = ctx->p;
  NOSA_REQUIRE(ctx, mode == 0 || p.n_kv_heads <= 16, NOSA_ESHAPE, "eviction head mode 1 supports at most 16 KV heads");
  EvictArgs a{qkv, w1, w2, q_out, k_new, v_new, b_new, p.n_q_heads, p.n_kv_heads, p.head_dim, p.dtype, mode};
  const int rows = p.n_q_heads + 2 * p.n_kv_heads;
  TimedLaunch tl(ctx, NOSA_KERNEL_EVICT, ctx->main);
  hipLaunchKernelGGL(split_qkv_evict_kernel, dim3(p.batch * rows), dim3(kWave), 0, ctx->main, a);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
