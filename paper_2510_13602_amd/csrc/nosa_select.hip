// Constrained block selection (selection Eq. of Sec. 3.1; Alg. 1 select_topk_indices) and the load
// positions (Sec. 4 "Memory Layout and Block Selection"; Alg. 1 generate_load_positions), one
// wavefront per unit, one launch for both, nothing read back by the host.
//
// Exact top-k without sorting: scores are mapped to order-preserving 32-bit keys held in registers
// (block r*64 + lane in register r of a lane), and the k-th largest key is found by a bitwise
// binary search (32 rounds of "how many keys >= x", counted with wave ballots on the scalar unit).
// Keys above the threshold are taken; ties at the threshold are taken in ascending block order, which realises "the lower index wins".  The query-aware pass runs
// first, its winners are removed, then the query-agnostic pass fills the rest of the budget.
// Gamma(t) is emitted in ascending order by a ballot prefix scan over the selection flags; the
// same scan yields the missed blocks, a second one over the slots yields the victims.
#include <cmath>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

using dev::order_key;

__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
  return __popcll(mask & ((1ull << lane) - 1ull));
}

// Marks the `want` largest eligible keys (key != 0) held in registers -- lane `lane`, register r
// holds block r*64 + lane -- in flags[] with `tag`, ties to the lower block index, and zeroes the
// winners in `other` so that the next pass skips them.  All lanes of the wave call this with the
// same arguments.  Returns the number taken.
template <int R, bool HAS_OTHER>
__device__ __forceinline__ int take_top(uint32_t (&keys)[R], uint32_t (&other)[R], uint8_t* flags, int want,
                                        int n_eligible, uint8_t tag, int lane) {
  if (want <= 0 || n_eligible <= 0) return 0;
  uint32_t thr = 1;   // every eligible key is >= thr
  if (want < n_eligible) {
    uint32_t prefix = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = prefix | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int r = 0; r < R; ++r) cnt += (int)__popcll(__ballot(keys[r] >= cand));
      if (cnt >= want) prefix = cand;
      if (cnt == want) break;   // exactly the keys >= cand win: the threshold's lower bits do not matter
    }
    thr = prefix;   // the want-th largest key, or a bound with exactly `want` keys at or above it
  } else {
    want = n_eligible;
  }
  int above = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) above += (int)__popcll(__ballot(keys[r] > thr));
  int ties_left = want - above;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const uint32_t k = keys[r];
    const bool gt = k > thr;            // thr >= 1, so ineligible keys (0) never pass
    const bool eq = k == thr;
    const uint64_t eqm = __ballot(eq);
    const bool take = gt || (eq && lanes_below(eqm, lane) < ties_left);
    ties_left -= min(ties_left, (int)__popcll(eqm));
    if (take) {
      flags[r * kWave + lane] = tag;
      if constexpr (HAS_OTHER) other[r] = 0u;
    }
  }
  return want;
}

struct SelectArgs {
  const float* sq_blk;
  const float* se_blk;
  const int32_t* n_tokens;
  int32_t* sel_idx;
  int32_t* n_sel;
  int32_t* slot_of_block;
  int32_t* block_of_slot;
  int32_t* load_list;
  int32_t* n_load;
  int n_kv_heads, max_blocks, k_blocks, kq_blocks, sink_blocks, window_blocks, gpu_slots, victim_policy;
  int se_unit_div, se_stride;   // row of se_blk a unit reads: ((b / se_unit_div) * Hkv + h) * se_stride
};

// R = ceil(max_blocks / 64): candidate keys per lane, register resident.
template <int R>
__global__ __launch_bounds__(kWave) void select_kernel(const SelectArgs a) {
  extern __shared__ unsigned char smem[];
  int32_t* miss = (int32_t*)smem;                       // [K]
  int32_t* victim = miss + a.k_blocks;                  // [K]
  uint8_t* flags = (uint8_t*)(victim + a.k_blocks);     // [R*64] 0 none, 1 forced, 2 query-aware, 3 query-agnostic
  uint8_t* vflags = flags + R * kWave;                  // [R*64] victim_policy 1: slots chosen as victims

  const int unit = blockIdx.x;
  const int b = unit / a.n_kv_heads;
  const int lane = threadIdx.x;
  const int K = a.k_blocks;
  int T = a.n_tokens[b];
  T = max(0, min(T, a.max_blocks * kBlockTokens));
  const int N = (T + kBlockTokens - 1) / kBlockTokens;
  const int Nc = T / kBlockTokens;
  const float* sq = a.sq_blk + (size_t)unit * a.max_blocks;
  const float* se = a.se_blk + ((size_t)(b / a.se_unit_div) * a.n_kv_heads + unit % a.n_kv_heads) * a.se_stride;

  // forced blocks and candidate keys
  const int win_lo = N - a.window_blocks;
  uint32_t key_q[R], key_e[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int J = r * kWave + lane;
    const bool forced = J < N && (J < a.sink_blocks || J >= win_lo);
    const bool cand = !forced && J < Nc;
    flags[J] = forced ? 1 : 0;
    key_q[r] = cand ? order_key(sq[J]) : 0u;
    key_e[r] = cand ? order_key(se[J]) : 0u;
  }
  const int nF = min(N, a.sink_blocks + a.window_blocks);
  const int nD = max(0, min(Nc, win_lo) - a.sink_blocks);

  const int kq = take_top<R, true>(key_q, key_e, flags, a.kq_blocks, nD, 2, lane);
  int ke = K - nF - a.kq_blocks;
  ke = max(0, min(ke, nD - kq));
  take_top<R, false>(key_e, key_e, flags, ke, nD - kq, 3, lane);
  __syncthreads();

  // Gamma(t) ascending; misses = selected blocks without a slot
  int32_t* sel = a.sel_idx + (size_t)unit * K;
  if (a.slot_of_block == nullptr) {   // selection only (prefill: every block is resident)
    int n_on = 0;
    for (int base = 0; base < N; base += kWave) {
      const int J = base + lane;
      const bool on = J < N && flags[J] != 0;
      const uint64_t m = __ballot(on);
      const int pos = n_on + lanes_below(m, lane);
      if (on && pos < K) sel[pos] = J;
      n_on += (int)__popcll(m);
    }
    n_on = min(n_on, K);
    for (int i = n_on + lane; i < K; i += kWave) sel[i] = -1;
    if (lane == 0) a.n_sel[unit] = n_on;
    return;
  }
  int32_t* sob = a.slot_of_block + (size_t)unit * a.max_blocks;
  int32_t* bos = a.block_of_slot + (size_t)unit * a.gpu_slots;
  int n_sel = 0, n_miss = 0;
  for (int base = 0; base < N; base += kWave) {
    const int J = base + lane;
    const bool on = J < N && flags[J] != 0;
    const uint64_t m = __ballot(on);
    const int pos = n_sel + lanes_below(m, lane);
    const bool is_miss = on && pos < K && sob[J] < 0;
    if (on && pos < K) sel[pos] = J;
    const uint64_t mm = __ballot(is_miss);
    if (is_miss) miss[n_miss + lanes_below(mm, lane)] = J;
    n_sel += (int)__popcll(m);
    n_miss += (int)__popcll(mm);
  }
  n_sel = min(n_sel, K);
  for (int i = n_sel + lane; i < K; i += kWave) sel[i] = -1;

  // victim_policy 1: of the free slots keep the n_miss "cheapest": empty ones, then the ones whose
  // block has the smallest importance (largest inverted key), ties to the lower slot
  const bool ranked = a.victim_policy == 1 && n_miss > 0;
  if (ranked) {
    uint32_t vkey[R];
    int n_free = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int s = r * kWave + lane;
      uint32_t key = 0u;
      if (s < a.gpu_slots) {
        const int blk = bos[s];
        if (blk < 0 || blk >= N) key = 0xffffffffu;
        else if (flags[blk] == 0) key = ~order_key(se[blk]);
      }
      vkey[r] = key;
      vflags[s] = 0;
      n_free += (int)__popcll(__ballot(key != 0u));
    }
    take_top<R, false>(vkey, vkey, vflags, min(n_miss, n_free), n_free, 1, lane);
    __syncthreads();
  }

  // victims: slots (ascending) that are empty or hold a block outside Gamma(t); the first n_miss are used
  int n_vict = 0;
  for (int base = 0; base < a.gpu_slots && n_vict < n_miss; base += kWave) {
    const int s = base + lane;
    bool free_slot = false;
    if (s < a.gpu_slots) {
      const int blk = bos[s];
      free_slot = ranked ? vflags[s] != 0 : (blk < 0 || blk >= N || flags[blk] == 0);
    }
    const uint64_t m = __ballot(free_slot);
    const int pos = n_vict + lanes_below(m, lane);
    if (free_slot && pos < n_miss) victim[pos] = s;
    n_vict += (int)__popcll(m);
  }
  __syncthreads();
  const int n_load = min(n_miss, n_vict);   // == n_miss whenever C >= K
  int32_t* ll = a.load_list + (size_t)unit * K * 2;
  for (int i = lane; i < K; i += kWave) {
    if (i < n_load) {
      const int J = miss[i], s = victim[i];
      const int old = bos[s];
      if (old >= 0 && old < a.max_blocks) sob[old] = -1;
      bos[s] = J;
      sob[J] = s;
      ll[2 * i] = J;
      ll[2 * i + 1] = s;
    } else {
      ll[2 * i] = -1;
      ll[2 * i + 1] = -1;
    }
  }
  if (lane == 0) {
    a.n_sel[unit] = n_sel;
    a.n_load[unit] = n_load;
  }
}

}  // namespace

int launch_select(nosa_ctx* ctx, const float* sq_blk, const float* se_blk, const int32_t* n_tokens,
                  int32_t* sel_idx, int32_t* n_sel, int32_t* slot_of_block, int32_t* block_of_slot,
                  int32_t* load_list, int32_t* n_load, int batch_mul, int se_unit_div, int se_stride) {
  const nosa_params& p = ctx->p;
  SelectArgs a{sq_blk, se_blk, n_tokens, sel_idx, n_sel, slot_of_block, block_of_slot, load_list, n_load,
               p.n_kv_heads, p.max_blocks, p.k_blocks, p.kq_blocks, p.sink_blocks, p.window_blocks, p.gpu_slots,
               p.victim_policy, se_unit_div, se_stride > 0 ? se_stride : p.max_blocks};
  int regs = (p.max_blocks + kWave - 1) / kWave;
  if (p.victim_policy == 1 && (p.gpu_slots + kWave - 1) / kWave > regs) regs = (p.gpu_slots + kWave - 1) / kWave;
  const int R = regs <= 8 ? 8 : regs <= 16 ? 16 : regs <= 32 ? 32 : 64;
  NOSA_REQUIRE(ctx, regs <= 64, NOSA_ESHAPE, "selection supports at most %d blocks per unit", kMaxSelectBlocks);
  const size_t smem = (size_t)p.k_blocks * 8 + 2 * (size_t)R * kWave;
  const dim3 grid(ctx->units * batch_mul), block(kWave);   // batch_mul > 1: one virtual batch element per query position
  TimedLaunch tl(ctx, NOSA_KERNEL_SELECT, ctx->main);
  switch (R) {
    case 8: hipLaunchKernelGGL(select_kernel<8>, grid, block, smem, ctx->main, a); break;
    case 16: hipLaunchKernelGGL(select_kernel<16>, grid, block, smem, ctx->main, a); break;
    case 32: hipLaunchKernelGGL(select_kernel<32>, grid, block, smem, ctx->main, a); break;
    default: hipLaunchKernelGGL(select_kernel<64>, grid, block, smem, ctx->main, a); break;
  }
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
