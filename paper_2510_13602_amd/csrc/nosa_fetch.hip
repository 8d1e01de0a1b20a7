// Host-to-device transfer of the missed blocks (Sec. 4 "Offloading Communication"; Alg. 1
// host_to_device_communication): a gather kernel whose lanes read 16 bytes each straight from
// pinned host memory (the GPU addresses it over the host link) and write the block's slot in the
// paged pool.  A block's keys and values are contiguous 8-32 KiB pieces, so every wave-load is a
// 1 KiB contiguous read; all loads of a piece are issued before the first store so that many
// requests are in flight on the link.  The list length lives on the device: the grid is sized for
// the per-step bound (Kq blocks per unit, Theorem 1) and loops when a cold start needs more.
#include "nosa_internal.h"

namespace nosa {
namespace {

constexpr int kThreads = 256;
constexpr int kInFlight = 4;   // 16-byte loads per lane before the stores start
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct FetchArgs {
  const u32x4* host_k;
  const u32x4* host_v;
  const u32x4* host_bias;
  u32x4* pool_k;
  u32x4* pool_v;
  u32x4* pool_bias;
  const int32_t* load_list;
  const int32_t* n_load;
  int k_blocks, gpu_slots, max_blocks;
  int block_vec;   // 16-byte vectors per K (or V) block
  int bias_vec;    // 16-byte vectors per bias block
};

__device__ __forceinline__ void copy_piece(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int nvec, int tid) {
  for (int base = 0; base < nvec; base += kThreads * kInFlight) {
    u32x4 buf[kInFlight];
#pragma unroll
    for (int i = 0; i < kInFlight; ++i) {
      const int x = base + i * kThreads + tid;
      if (x < nvec) buf[i] = __builtin_nontemporal_load(src + x);
    }
#pragma unroll
    for (int i = 0; i < kInFlight; ++i) {
      const int x = base + i * kThreads + tid;
      if (x < nvec) dst[x] = buf[i];
    }
  }
}

__global__ __launch_bounds__(kThreads) void fetch_kernel(const FetchArgs a) {
  const int unit = blockIdx.y;
  const int n = min(a.n_load[unit], a.k_blocks);
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const int J = a.load_list[((size_t)unit * a.k_blocks + i) * 2];
    const int s = a.load_list[((size_t)unit * a.k_blocks + i) * 2 + 1];
    if (J < 0 || J >= a.max_blocks || s < 0 || s >= a.gpu_slots) continue;   // malformed entry: skip, never fault
    const size_t src = (size_t)unit * a.max_blocks + J;
    const size_t dst = (size_t)unit * a.gpu_slots + s;
    copy_piece(a.host_k + src * a.block_vec, a.pool_k + dst * a.block_vec, a.block_vec, threadIdx.x);
    copy_piece(a.host_v + src * a.block_vec, a.pool_v + dst * a.block_vec, a.block_vec, threadIdx.x);
    if (a.host_bias) copy_piece(a.host_bias + src * a.bias_vec, a.pool_bias + dst * a.bias_vec, a.bias_vec, threadIdx.x);
  }
}

}  // namespace

int launch_fetch(nosa_ctx* ctx, hipStream_t stream, const void* host_k, const void* host_v, const float* host_bias,
                 void* pool_k, void* pool_v, float* pool_bias, const int32_t* load_list, const int32_t* n_load) {
  const nosa_params& p = ctx->p;
  const int es = p.dtype == NOSA_DTYPE_F32 ? 4 : 2;
  FetchArgs a{(const u32x4*)host_k, (const u32x4*)host_v, (const u32x4*)host_bias, (u32x4*)pool_k, (u32x4*)pool_v,
              (u32x4*)pool_bias, load_list, n_load, p.k_blocks, p.gpu_slots, p.max_blocks,
              p.block_size * p.head_dim * es / 16, p.block_size * 4 / 16};
  int per_unit = p.kq_blocks > 0 ? p.kq_blocks : 1;
  if (per_unit > p.k_blocks) per_unit = p.k_blocks;
  const dim3 grid(per_unit, ctx->units);
  TimedLaunch tl(ctx, NOSA_KERNEL_FETCH, stream);
  hipLaunchKernelGGL(fetch_kernel, grid, dim3(kThreads), 0, stream, a);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
