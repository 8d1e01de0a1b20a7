// Block scores (Alg. 1 Stage 1: S_c^q = Q K_c^T followed by the fused block-level max pooling of
// the query-aware and the query-agnostic score; Sec. 3.1 mean- and max-pooling Eqs.).
//
// The G query heads of a KV head are combined by summing their raw scores, and a sum of dot
// products with one pooled key is the dot product with the summed query: the kernel adds the G
// query vectors once (fp32) and streams the pooled keys a single time, so the step is a
// matrix-vector product bound by reading K_c from HBM.  Same lane mapping as the attention
// kernel: LPR adjacent lanes hold one pooled key, partial dot products are added with DPP.
#include <cmath>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

constexpr int kThreads = 256;
constexpr int kBlocksPerWg = 64;

using dev::row_sum;
using dev::u32x4;
using dev::widen16;

struct ScoreArgs {
  const void* q;
  const void* k_pooled;
  const float* se_pooled;
  const int32_t* n_tokens;
  float* sq_blk;
  float* se_blk;
  int n_kv_heads, group, max_blocks, n_sub_max, pool_kernel, pool_stride;
  int batch_div;   // virtual batch elements (query positions of a prefill chunk) per cache batch element; 1 in decode
  int n_units;     // (virtual batch element, KV head) pairs; they are folded over grid y and z
};

template <int DT, int D>
__global__ __launch_bounds__(kThreads) void block_score_kernel(const ScoreArgs a) {
  constexpr int EPL = DT == NOSA_DTYPE_BF16 ? 8 : 4;
  constexpr int ES = DT == NOSA_DTYPE_BF16 ? 2 : 4;
  constexpr int LPR = D / EPL;
  constexpr int RPW = kWave / LPR;
  constexpr int GROUPS = (kThreads / kWave) * RPW;   // row-groups per workgroup
  constexpr int ITERS = kBlocksPerWg / GROUPS;

  const int unit = blockIdx.z * gridDim.y + blockIdx.y;         // (virtual batch element, KV head)
  if (unit >= a.n_units) return;
  const int b = unit / a.n_kv_heads, h = unit % a.n_kv_heads;
  const int cache_unit = (b / a.batch_div) * a.n_kv_heads + h;    // where its pooled keys live
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r = lane / LPR, c = lane % LPR;
  const int T = a.n_tokens[b];
  const int lk = a.pool_kernel, ls = a.pool_stride;
  int nsub = T < lk ? 0 : (T - lk) / ls + 1;
  nsub = min(nsub, a.n_sub_max);

  // summed query slice of this lane
  float qs[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qs[e] = 0.f;
  {
    const uint4* qp = (const uint4*)((const char*)a.q + ((size_t)b * a.n_kv_heads + h) * a.group * D * ES);
    for (int g = 0; g < a.group; ++g) {
      float f[EPL];
      widen16<DT>(qp[g * LPR + c], f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qs[e] += f[e];
    }
  }

  const uint4* kc = (const uint4*)((const char*)a.k_pooled + (size_t)cache_unit * a.n_sub_max * D * ES);
  const float* sec = a.se_pooled + (size_t)cache_unit * a.n_sub_max;
  const int J0 = blockIdx.x * kBlocksPerWg;

#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int J = J0 + it * GROUPS + wave * RPW + r;
    if (J >= a.max_blocks) continue;
    // sub-blocks wholly inside block J: J*nb <= j*ls and j*ls + lk <= (J+1)*nb, and complete (j < nsub)
    const int lo_tok = J * kBlockTokens, hi_tok = lo_tok + kBlockTokens;
    int j_lo = (lo_tok + ls - 1) / ls;
    int j_hi = hi_tok >= lk ? (hi_tok - lk) / ls : -1;   // inclusive
    j_hi = min(j_hi, nsub - 1);
    float best_q = -INFINITY, best_e = -INFINITY;
    for (int j = j_lo; j <= j_hi; ++j) {
      float f[EPL];
      widen16<DT>(kc[(size_t)j * LPR + c], f);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(f[e], qs[e], d);
      d = row_sum<LPR>(d);
      best_q = fmaxf(best_q, d);
      best_e = fmaxf(best_e, sec[j]);
    }
    if (c == 0) {
      a.sq_blk[(size_t)unit * a.max_blocks + J] = best_q;
      a.se_blk[(size_t)unit * a.max_blocks + J] = best_e;
    }
  }
}


// Fast path for one pooled key per block (pool_kernel == pool_stride == block size): sub-block j is
// block j, the block max is the identity.  A workgroup streams 128 pooled keys; every lane issues its
// 8 non-temporal 16-byte loads before the first dot product.
constexpr int kFastBlocksPerWg = 128;

template <int DT, int D>
__global__ __launch_bounds__(kThreads) void block_score_simple_kernel(const ScoreArgs a) {
  constexpr int EPL = DT == NOSA_DTYPE_BF16 ? 8 : 4;
  constexpr int ES = DT == NOSA_DTYPE_BF16 ? 2 : 4;
  constexpr int LPR = D / EPL;
  constexpr int RPW = kWave / LPR;
  constexpr int GROUPS = (kThreads / kWave) * RPW;
  constexpr int ITERS = kFastBlocksPerWg / GROUPS;

  const int unit = blockIdx.z * gridDim.y + blockIdx.y;         // (virtual batch element, KV head)
  if (unit >= a.n_units) return;
  const int b = unit / a.n_kv_heads, h = unit % a.n_kv_heads;
  const int cache_unit = (b / a.batch_div) * a.n_kv_heads + h;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r = lane / LPR, c = lane % LPR;
  const int nsub = min(a.n_tokens[b] / kBlockTokens, a.n_sub_max);   // complete blocks
  const int J0 = blockIdx.x * kFastBlocksPerWg + wave * RPW + r;     // this lane's row in round 0

  const u32x4* kc = (const u32x4*)((const char*)a.k_pooled + (size_t)cache_unit * a.n_sub_max * D * ES);
  const float* sec = a.se_pooled + (size_t)cache_unit * a.n_sub_max;
  u32x4 kv[ITERS];
  float sev[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int J = J0 + it * GROUPS;
    kv[it] = u32x4{0u, 0u, 0u, 0u};
    sev[it] = -INFINITY;
    if (J < nsub) {
      kv[it] = __builtin_nontemporal_load(kc + (size_t)J * LPR + c);
      if (c == 0) sev[it] = __builtin_nontemporal_load(sec + J);
    }
  }

  float qs[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qs[e] = 0.f;
  {
    const uint4* qp = (const uint4*)((const char*)a.q + ((size_t)b * a.n_kv_heads + h) * a.group * D * ES);
    for (int g = 0; g < a.group; ++g) {
      float f[EPL];
      widen16<DT>(qp[g * LPR + c], f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qs[e] += f[e];
    }
  }

#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int J = J0 + it * GROUPS;
    float f[EPL];
    widen16<DT>(make_uint4(kv[it].x, kv[it].y, kv[it].z, kv[it].w), f);
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) d = fmaf(f[e], qs[e], d);
    d = row_sum<LPR>(d);
    if (c == 0 && J < a.max_blocks) {
      a.sq_blk[(size_t)unit * a.max_blocks + J] = J < nsub ? d : -INFINITY;
      a.se_blk[(size_t)unit * a.max_blocks + J] = sev[it];
    }
  }
}

}  // namespace

int launch_block_score(nosa_ctx* ctx, const void* q, const void* k_pooled, const float* se_pooled,
                       const int32_t* n_tokens, float* sq_blk, float* se_blk, int batch_div) {
  const nosa_params& p = ctx->p;
  ScoreArgs a{q, k_pooled, se_pooled, n_tokens, sq_blk, se_blk, p.n_kv_heads, ctx->group,
              p.max_blocks, p.n_sub_max, p.pool_kernel, p.pool_stride, batch_div, ctx->units * batch_div};
  const int gz = (a.n_units + 32767) / 32768, gy = (a.n_units + gz - 1) / gz;   // grid y and z stay below 65536
  TimedLaunch tl(ctx, NOSA_KERNEL_SCORE, ctx->main);
  if (p.pool_kernel == p.block_size && p.pool_stride == p.block_size) {
    const dim3 fgrid((p.max_blocks + kFastBlocksPerWg - 1) / kFastBlocksPerWg, gy, gz);
    if (p.dtype == NOSA_DTYPE_BF16) {
      if (p.head_dim == 128) hipLaunchKernelGGL((block_score_simple_kernel<NOSA_DTYPE_BF16, 128>), fgrid, dim3(kThreads), 0, ctx->main, a);
      else hipLaunchKernelGGL((block_score_simple_kernel<NOSA_DTYPE_BF16, 64>), fgrid, dim3(kThreads), 0, ctx->main, a);
    } else {
      if (p.head_dim == 128) hipLaunchKernelGGL((block_score_simple_kernel<NOSA_DTYPE_F32, 128>), fgrid, dim3(kThreads), 0, ctx->main, a);
      else hipLaunchKernelGGL((block_score_simple_kernel<NOSA_DTYPE_F32, 64>), fgrid, dim3(kThreads), 0, ctx->main, a);
    }
    NOSA_HIP(ctx, hipGetLastError());
    return NOSA_OK;
  }
  const dim3 grid((p.max_blocks + kBlocksPerWg - 1) / kBlocksPerWg, gy, gz);
  if (p.dtype == NOSA_DTYPE_BF16) {
    if (p.head_dim == 128) hipLaunchKernelGGL((block_score_kernel<NOSA_DTYPE_BF16, 128>), grid, dim3(kThreads), 0, ctx->main, a);
    else hipLaunchKernelGGL((block_score_kernel<NOSA_DTYPE_BF16, 64>), grid, dim3(kThreads), 0, ctx->main, a);
  } else {
    if (p.head_dim == 128) hipLaunchKernelGGL((block_score_kernel<NOSA_DTYPE_F32, 128>), grid, dim3(kThreads), 0, ctx->main, a);
    else hipLaunchKernelGGL((block_score_kernel<NOSA_DTYPE_F32, 64>), grid, dim3(kThreads), 0, ctx->main, a);
  }
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
