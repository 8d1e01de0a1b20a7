// Host-to-device transfer of the missed blocks (Sec. 4 "Offloading Communication"; Alg. 1
// host_to_device_communication): a gather kernel whose lanes read 16 bytes each straight from
// pinned host memory (the GPU addresses it over the host link) and write the block's slot in the
// paged pool.  A block's keys and values are contiguous 8-32 KiB pieces, so every wave-load is a
// 1 KiB contiguous read.  The list lengths live on the device; nothing is read back.
// Two regimes.  Every unit misses several blocks (pool = budget): with 256 workgroups or more the link is
// saturated by their number alone, each with one 16-byte load per lane in flight (4 KiB per workgroup; four
// loads per lane measured the same rate at best and 1-3 % less in most runs); fewer workgroups (small batches)
// keep four loads per lane in flight.  A unit misses one block (pool with room to spare):
// the gather is a handful of blocks and its duration is latency, so that block's keys, values and bias are
// requested together, one round trip instead of nine.
// The stores into the pool are non-temporal: written normally, the 80 MB of a step at the 8B shape stay
// behind as dirty lines in the L2s and the memory-side cache, and their write-back then competes with the
// reads of the attention kernel that follows (measured: 179 us instead of 163 us for that kernel).
#include <algorithm>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

#ifndef NOSA_FETCH_THREADS
#define NOSA_FETCH_THREADS 256
#endif
constexpr int kThreads = NOSA_FETCH_THREADS;
constexpr int kInFlight = 4;   // 16-byte loads per lane before the stores start
using dev::u32x4;

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
  int use_lone;    // a unit's lone block as one request: only when the gather has the GPU to itself
};

// A contiguous piece, DEPTH 16-byte loads per lane in flight.  Whole passes carry no per-lane conditions, so
// nothing separates their loads.
template <int DEPTH>
__device__ __forceinline__ void copy_piece(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int nvec, int tid) {
  int base = 0;
  if constexpr (DEPTH > 1) {
    for (; base + kThreads * DEPTH <= nvec; base += kThreads * DEPTH) {
      u32x4 buf[DEPTH];
#pragma unroll
      for (int i = 0; i < DEPTH; ++i) buf[i] = __builtin_nontemporal_load(src + base + i * kThreads + tid);
#pragma unroll
      for (int i = 0; i < DEPTH; ++i) __builtin_nontemporal_store(buf[i], dst + base + i * kThreads + tid);
    }
  }
  for (int x = base + tid; x < nvec; x += kThreads) __builtin_nontemporal_store(__builtin_nontemporal_load(src + x), dst + x);
}

// One block, keys, values and bias together: all its loads are issued before the first store (32 KiB and the
// bias in flight for d = 128 bf16 rows).  Whole passes only (the caller checks the shape).  Measured at the 8B
// shape with 96 slots, where a step fetches 3 blocks in all: 7.9 us for the launch instead of 14.1 us.  Used
// only when the gather runs on the main stream: beside an attention launch the deeper requests cost that launch
// more than they save (long generation, 68 blocks: 0.173 instead of 0.162 ms per step).
template <int N>   // 16-byte loads per lane, for K and again for V, before the stores start
__device__ __forceinline__ void copy_block(const FetchArgs& a, size_t src, size_t dst, int tid) {
  const u32x4* __restrict__ sk = a.host_k + src * a.block_vec;
  const u32x4* __restrict__ sv = a.host_v + src * a.block_vec;
  u32x4* __restrict__ dk = a.pool_k + dst * a.block_vec;
  u32x4* __restrict__ dv = a.pool_v + dst * a.block_vec;
  const bool has_bias = a.host_bias != nullptr && tid < a.bias_vec;
  u32x4 bb = {0u, 0u, 0u, 0u};
  if (has_bias) bb = __builtin_nontemporal_load(a.host_bias + src * a.bias_vec + tid);
  for (int base = 0; base < a.block_vec; base += kThreads * N) {
    u32x4 kb[N], vb[N];
#pragma unroll
    for (int i = 0; i < N; ++i) kb[i] = __builtin_nontemporal_load(sk + base + i * kThreads + tid);
#pragma unroll
    for (int i = 0; i < N; ++i) vb[i] = __builtin_nontemporal_load(sv + base + i * kThreads + tid);
#pragma unroll
    for (int i = 0; i < N; ++i) __builtin_nontemporal_store(kb[i], dk + base + i * kThreads + tid);
#pragma unroll
    for (int i = 0; i < N; ++i) __builtin_nontemporal_store(vb[i], dv + base + i * kThreads + tid);
  }
  if (has_bias) __builtin_nontemporal_store(bb, a.pool_bias + dst * a.bias_vec + tid);
}

// A persistent grid: workgroup w takes units w, w + gridDim.x, ... and copies each unit's listed
// blocks in turn.  Measured on MI355X (PCIe Gen5 x16): 16 workgroups
// reach 36 GB/s, 64 reach 52 GB/s, 512 reach 56 GB/s (read latency under load is several microseconds,
// so about 1 MiB has to be in flight).  Host reads in flight slow HBM reads of kernels running at
// the same time (global, not per CU or per XCD): the attention over resident blocks that overlaps the
// gather runs 1.3x slower at 64 workgroups and ~8x slower at 512 -- but it still ends before the
// gather does, so the step time is lowest with the widest gather.
// With fewer than 256 units a unit's list is shared by `share` workgroups (entry i goes to workgroup
// i % share of the unit), so that small batches still put enough requests on the link (1B shape, 32 units:
// 76 -> 72 us); beyond about 256 workgroups more of them only slow the attention launch running beside.  More requests per
// workgroup instead (four loads per lane, or whole blocks at once) measured 5-10 % slower at every shape: the
// link wants many shallow streams.
template <int DEPTH>
__global__ __launch_bounds__(kThreads) void fetch_kernel(const FetchArgs a, int units, int share) {
  for (int item = blockIdx.x; item < units * share; item += gridDim.x) {
    const int unit = item / share, part = item % share;
    const int n = min(a.n_load[unit], a.k_blocks);
    // A lone block travels as one request only when misses are rare around it (at most 2 of the 64 units this
    // one sits among fetch anything): with a lone block in every second or third unit the deeper requests
    // lower the link's rate instead (8B shape with 80 slots, 0.42 blocks per unit and step: 152 against 129 us).
    bool lone = false;
    if (n == 1 && a.use_lone && a.block_vec % (kThreads * 2) == 0 && a.bias_vec <= kThreads) {
      const int u = (unit & ~(kWave - 1)) + (int)(threadIdx.x % kWave);
      const bool busy = u < units && a.n_load[u] > 0;
      lone = __popcll(__ballot(busy)) <= 2;
    }
    for (int i = part; i < n; i += share) {
      const int J = a.load_list[((size_t)unit * a.k_blocks + i) * 2];
      const int s = a.load_list[((size_t)unit * a.k_blocks + i) * 2 + 1];
      if (J < 0 || J >= a.max_blocks || s < 0 || s >= a.gpu_slots) continue;   // malformed entry: skip, never fault
      const size_t src = (size_t)unit * a.max_blocks + J;
      const size_t dst = (size_t)unit * a.gpu_slots + s;
      if (lone) {
        if (a.block_vec % (kThreads * 4) == 0) copy_block<4>(a, src, dst, threadIdx.x);
        else copy_block<2>(a, src, dst, threadIdx.x);   // d = 64 in bf16
        continue;
      }
      copy_piece<DEPTH>(a.host_k + src * a.block_vec, a.pool_k + dst * a.block_vec, a.block_vec, threadIdx.x);
      copy_piece<DEPTH>(a.host_v + src * a.block_vec, a.pool_v + dst * a.block_vec, a.block_vec, threadIdx.x);
      if (a.host_bias) copy_piece<DEPTH>(a.host_bias + src * a.bias_vec, a.pool_bias + dst * a.bias_vec, a.bias_vec, threadIdx.x);
    }
  }
}

// Element-wise counterpart (Sec. 3.2 "Comparison with DMA"): single token rows instead of blocks.
// A row of K (or V) is d*es bytes = 8..32 lanes of 16 bytes; a workgroup copies 256*16/row_bytes rows
// per pass, several passes in flight.  Same persistent grid as the block-wise gather.
struct TokenFetchArgs {
  const u32x4* host_k;
  const u32x4* host_v;
  const float* host_bias;
  u32x4* pool_k;
  u32x4* pool_v;
  float* pool_bias;
  const int32_t* token_list;   // [units][max_list][2] (host token, pool row)
  const int32_t* n_list;
  int max_list, gpu_rows, host_rows;
  int row_vec;                 // 16-byte vectors per row
};

__global__ __launch_bounds__(kThreads) void fetch_tokens_kernel(const TokenFetchArgs a, int units) {
  const int lpr = a.row_vec;                       // lanes per row
  const int rows_per_pass = kThreads / lpr;
  const int rr = threadIdx.x / lpr, cc = threadIdx.x % lpr;
  for (int unit = blockIdx.x; unit < units; unit += gridDim.x) {
    const int n = min(a.n_list[unit], a.max_list);
    const int32_t* tl = a.token_list + (size_t)unit * a.max_list * 2;
    for (int base = 0; base < n; base += rows_per_pass * kInFlight) {
      u32x4 kb[kInFlight], vb[kInFlight];
      float bb[kInFlight];
      int dst[kInFlight];
#pragma unroll
      for (int i = 0; i < kInFlight; ++i) {
        const int e = base + i * rows_per_pass + rr;
        dst[i] = -1;
        if (e < n) {
          const int t = tl[2 * e], r = tl[2 * e + 1];
          if (t >= 0 && t < a.host_rows && r >= 0 && r < a.gpu_rows) {
            dst[i] = r;
            const size_t src = ((size_t)unit * a.host_rows + t);
            kb[i] = __builtin_nontemporal_load(a.host_k + src * lpr + cc);
            vb[i] = __builtin_nontemporal_load(a.host_v + src * lpr + cc);
            if (a.host_bias && cc == 0) bb[i] = __builtin_nontemporal_load(a.host_bias + src);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < kInFlight; ++i) {
        if (dst[i] < 0) continue;
        const size_t d = ((size_t)unit * a.gpu_rows + dst[i]);
        __builtin_nontemporal_store(kb[i], a.pool_k + d * lpr + cc);
        __builtin_nontemporal_store(vb[i], a.pool_v + d * lpr + cc);
        if (a.host_bias && cc == 0) a.pool_bias[d] = bb[i];
      }
    }
  }
}

}  // namespace

int launch_fetch(nosa_ctx* ctx, hipStream_t stream, const void* host_k, const void* host_v, const float* host_bias,
                 void* pool_k, void* pool_v, float* pool_bias, const int32_t* load_list, const int32_t* n_load) {
  const nosa_params& p = ctx->p;
  const int es = p.dtype == NOSA_DTYPE_F32 ? 4 : 2;
  FetchArgs a{(const u32x4*)host_k, (const u32x4*)host_v, (const u32x4*)host_bias, (u32x4*)pool_k, (u32x4*)pool_v,
              (u32x4*)pool_bias, load_list, n_load, p.k_blocks, p.gpu_slots, p.max_blocks,
              p.block_size * p.head_dim * es / 16, p.block_size * 4 / 16, stream == ctx->main ? 1 : 0};
  int share = 1;
  if (ctx->units < 256 && ctx->fetch_wgs >= 256) share = std::max(1, std::min(256 / ctx->units, std::max(1, p.kq_blocks)));
  const int items = ctx->units * share;
  const int wgs = ctx->fetch_wgs < items ? ctx->fetch_wgs : items;
  const int depth = wgs >= 256 ? 1 : 4;
  TimedLaunch tl(ctx, NOSA_KERNEL_FETCH, stream);
  // few workgroups: each has to keep more of the link's latency covered by itself
  if (depth == 1) hipLaunchKernelGGL(fetch_kernel<1>, dim3(wgs), dim3(kThreads), 0, stream, a, ctx->units, share);
  else if (a.block_vec % (kThreads * 4) == 0) hipLaunchKernelGGL(fetch_kernel<4>, dim3(wgs), dim3(kThreads), 0, stream, a, ctx->units, share);
  else hipLaunchKernelGGL(fetch_kernel<2>, dim3(wgs), dim3(kThreads), 0, stream, a, ctx->units, share);   // d = 64 in bf16: 8 KiB pieces
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa

namespace nosa {
int launch_fetch_tokens(nosa_ctx* ctx, hipStream_t stream, const void* host_k, const void* host_v, const float* host_bias,
                        void* pool_k, void* pool_v, float* pool_bias, const int32_t* token_list, const int32_t* n_list,
                        int max_list) {
  const nosa_params& p = ctx->p;
  const int es = p.dtype == NOSA_DTYPE_F32 ? 4 : 2;
  TokenFetchArgs a{(const u32x4*)host_k, (const u32x4*)host_v, host_bias, (u32x4*)pool_k, (u32x4*)pool_v, pool_bias,
                   token_list, n_list, max_list, p.gpu_slots * p.block_size, p.max_blocks * p.block_size,
                   p.head_dim * es / 16};
  const int wgs = ctx->fetch_wgs < ctx->units ? ctx->fetch_wgs : ctx->units;
  TimedLaunch tl(ctx, NOSA_KERNEL_FETCH, stream);
  hipLaunchKernelGGL(fetch_tokens_kernel, dim3(wgs), dim3(kThreads), 0, stream, a, ctx->units);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}
}  // namespace nosa
