// Cache maintenance outside the timed path (Alg. 1 update_compressed_k / update_importance_score):
// pooled keys K_c[j] = mean of the keys of sub-block j (block compression f_c of Sec. 2.1 realised
// as the mean of the mean-pooling Eq., Sec. 3.1) and pooled importance S_c^e[j] = mean of b over it.
// Sums run in fp64 in token order, so the stored K_c is the correctly rounded mean.
#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

using dev::f64_to_bf16;

struct PoolArgs {
  const void* keys;
  const float* bias;
  const int32_t* n_tokens;
  void* k_pooled;
  float* se_pooled;
  int n_kv_heads, head_dim, max_blocks, n_sub_max, pool_kernel, pool_stride, dtype;
};

__global__ void pool_blocks_kernel(const PoolArgs a) {
  const int j = blockIdx.x, unit = blockIdx.y, e = threadIdx.x;
  const int b = unit / a.n_kv_heads;
  const int d = a.head_dim, lk = a.pool_kernel, ls = a.pool_stride;
  const int T = a.n_tokens[b];
  const int nsub = T < lk ? 0 : (T - lk) / ls + 1;
  const size_t out = ((size_t)unit * a.n_sub_max + j) * d + e;
  if (j >= nsub) {
    if (a.dtype == NOSA_DTYPE_F32) ((float*)a.k_pooled)[out] = 0.f;
    else ((uint16_t*)a.k_pooled)[out] = 0;
    if (e == 0) a.se_pooled[(size_t)unit * a.n_sub_max + j] = 0.f;
    return;
  }
  const size_t tok0 = (size_t)unit * a.max_blocks * kBlockTokens + (size_t)j * ls;
  double s = 0.0;
  if (a.dtype == NOSA_DTYPE_F32) {
    const float* k = (const float*)a.keys;
    for (int t = 0; t < lk; ++t) s += (double)k[(tok0 + t) * d + e];
    ((float*)a.k_pooled)[out] = (float)(s / (double)lk);
  } else {
    const uint16_t* k = (const uint16_t*)a.keys;
    for (int t = 0; t < lk; ++t) s += (double)__uint_as_float((uint32_t)k[(tok0 + t) * d + e] << 16);
    ((uint16_t*)a.k_pooled)[out] = f64_to_bf16(s / (double)lk);
  }
  if (e == 0) {
    double sb = 0.0;
    for (int t = 0; t < lk; ++t) sb += (double)a.bias[tok0 + t];
    a.se_pooled[(size_t)unit * a.n_sub_max + j] = (float)(sb / (double)lk);
  }
}

}  // namespace

int launch_pool_blocks(nosa_ctx* ctx, const void* keys, const float* bias, const int32_t* n_tokens,
                       void* k_pooled, float* se_pooled) {
  const nosa_params& p = ctx->p;
  if (p.n_sub_max == 0) return NOSA_OK;
  PoolArgs a{keys, bias, n_tokens, k_pooled, se_pooled, p.n_kv_heads, p.head_dim, p.max_blocks,
             p.n_sub_max, p.pool_kernel, p.pool_stride, p.dtype};
  hipLaunchKernelGGL(pool_blocks_kernel, dim3(p.n_sub_max, ctx->units), dim3(p.head_dim), 0, ctx->main, a);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
