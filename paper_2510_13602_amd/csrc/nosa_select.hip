// Constrained block selection (selection Eq. of Sec. 3.1; Alg. 1 select_topk_indices) and the load
// positions (Sec. 4 "Memory Layout and Block Selection"; Alg. 1 generate_load_positions), one
// wavefront per unit, one launch for both, nothing read back by the host.
//
// Exact top-k without sorting: scores are mapped to order-preserving 32-bit keys held in registers
// (block r*64 + lane in register r of a lane), and the k-th largest key is found by a bitwise
// binary search (at most 32 rounds of "how many keys >= x", counted with wave ballots on the scalar unit; it
// stops once exactly k keys pass, after ~14 rounds for scores of order one).
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

// Orders the LDS traffic of the one wavefront that runs the selection.  When that wavefront is a whole
// workgroup this is the ordinary barrier; when it is one wave of a larger workgroup (the fused score +
// selection kernel) the other waves are not part of the exchange, so a fence plus a scheduling barrier
// for the wave does the same job without a workgroup barrier.
template <bool ONE_WAVE_OF_MANY>
__device__ __forceinline__ void select_sync() {
  if constexpr (ONE_WAVE_OF_MANY) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  } else {
    __syncthreads();
  }
}

// The selection and the load positions of one unit, run by one wavefront (`lane` = 0..63).
// sq / se: the unit's block-level scores, indexed by block (global memory or LDS).
// R = ceil(max_blocks / 64): candidate keys per lane, register resident.
template <int R, bool ONE_WAVE_OF_MANY>
__device__ __forceinline__ void select_unit(const SelectArgs& a, const int unit, const int lane, const int n_tok,
                                            const float* sq, const float* se, unsigned char* smem) {
  int32_t* miss = (int32_t*)smem;                       // [K]
  int32_t* victim = miss + a.k_blocks;                  // [K]
  uint8_t* flags = (uint8_t*)(victim + a.k_blocks);     // [R*64] 0 none, 1 forced, 2 query-aware, 3 query-agnostic
  uint8_t* vflags = flags + R * kWave;                  // [R*64] victim_policy 1: slots chosen as victims

  const int K = a.k_blocks;
  const int T = max(0, min(n_tok, a.max_blocks * kBlockTokens));
  const int N = (T + kBlockTokens - 1) / kBlockTokens;
  const int Nc = T / kBlockTokens;

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

  // The residency of every block and the occupant of the first 64 slots are requested now, in one go, so
  // that their memory latency passes during the searches below instead of once per 64 blocks afterwards.
  int32_t* const sob = a.slot_of_block ? a.slot_of_block + (size_t)unit * a.max_blocks : nullptr;
  int32_t* const bos = a.block_of_slot ? a.block_of_slot + (size_t)unit * a.gpu_slots : nullptr;
  int slot_r[R];
  int bos_first = -1;
  if (sob) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int J = r * kWave + lane;
      slot_r[r] = J < N ? sob[J] : -1;
    }
    if (lane < a.gpu_slots) bos_first = bos[lane];
  }

  const int kq = take_top<R, true>(key_q, key_e, flags, a.kq_blocks, nD, 2, lane);
  int ke = K - nF - a.kq_blocks;
  ke = max(0, min(ke, nD - kq));
  take_top<R, false>(key_e, key_e, flags, ke, nD - kq, 3, lane);
  select_sync<ONE_WAVE_OF_MANY>();

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
  int n_sel = 0, n_miss = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int J = r * kWave + lane;
    const bool on = J < N && flags[J] != 0;
    const uint64_t m = __ballot(on);
    const int pos = n_sel + lanes_below(m, lane);
    const bool is_miss = on && pos < K && slot_r[r] < 0;
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
    select_sync<ONE_WAVE_OF_MANY>();
  }

  // victims: slots (ascending) that are empty or hold a block outside Gamma(t); the first n_miss are used
  int n_vict = 0;
  for (int base = 0; base < a.gpu_slots && n_vict < n_miss; base += kWave) {
    const int s = base + lane;
    bool free_slot = false;
    if (s < a.gpu_slots) {
      const int blk = base == 0 ? bos_first : bos[s];
      free_slot = ranked ? vflags[s] != 0 : (blk < 0 || blk >= N || flags[blk] == 0);
    }
    const uint64_t m = __ballot(free_slot);
    const int pos = n_vict + lanes_below(m, lane);
    if (free_slot && pos < n_miss) victim[pos] = s;
    n_vict += (int)__popcll(m);
  }
  select_sync<ONE_WAVE_OF_MANY>();
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

template <int R>
__global__ __launch_bounds__(kWave) void select_kernel(const SelectArgs a) {
  extern __shared__ unsigned char smem[];
  const int unit = blockIdx.x;
  const int b = unit / a.n_kv_heads;
  const float* sq = a.sq_blk + (size_t)unit * a.max_blocks;
  const float* se = a.se_blk + ((size_t)(b / a.se_unit_div) * a.n_kv_heads + unit % a.n_kv_heads) * a.se_stride;
  select_unit<R, false>(a, unit, threadIdx.x, a.n_tokens[b], sq, se, smem);
}

// ---- scores + selection + load positions in one launch (Alg. 1 Stage 1 as a whole) ---------------
// For one pooled key per block (pool_kernel == pool_stride == block size).  One workgroup of four
// wavefronts per unit: all four stream the unit's pooled keys once (the same arithmetic, in the same
// order, as the stand-alone score kernel: group-summed query, fp32 FMA dot, DPP row sum) and leave
// the block scores in LDS; then the first wavefront runs the selection on them.  The scores never
// travel through HBM unless the caller wants them (sq_out / se_out non-NULL).
constexpr int kFusedThreads = 256;

struct ScoreSelectArgs {
  SelectArgs sel;
  const void* q;
  const void* k_pooled;
  const float* se_pooled;
  float* sq_out;   // may be NULL
  float* se_out;   // may be NULL
  int group, n_sub_max;
};

template <int DT, int D, int R>
__global__ __launch_bounds__(kFusedThreads) void score_select_kernel(const ScoreSelectArgs a) {
  constexpr int EPL = DT == NOSA_DTYPE_BF16 ? 8 : 4;
  constexpr int ES = DT == NOSA_DTYPE_BF16 ? 2 : 4;
  constexpr int LPR = D / EPL;                           // lanes per pooled key
  constexpr int RPW = kWave / LPR;
  constexpr int GROUPS = (kFusedThreads / kWave) * RPW;  // pooled keys per round of the workgroup
  constexpr int INFL = 8;                                // 16-byte loads in flight per lane
  extern __shared__ unsigned char smem[];
  const int max_blocks = a.sel.max_blocks;
  float* s_sq = (float*)smem;                            // [max_blocks]
  float* s_se = s_sq + max_blocks;                       // [max_blocks]
  unsigned char* sel_smem = (unsigned char*)(s_se + max_blocks);

  const int unit = blockIdx.x;
  const int b = unit / a.sel.n_kv_heads, h = unit % a.sel.n_kv_heads;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r = lane / LPR, c = lane % LPR;
  int T = a.sel.n_tokens[b];
  T = max(0, min(T, max_blocks * kBlockTokens));
  const int nsub = min(T / kBlockTokens, a.n_sub_max);   // complete blocks that have a pooled key

  float qs[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qs[e] = 0.f;
  {
    const uint4* qp = (const uint4*)((const char*)a.q + ((size_t)b * a.sel.n_kv_heads + h) * a.group * D * ES);
    for (int g = 0; g < a.group; ++g) {
      float f[EPL];
      dev::widen16<DT>(qp[g * LPR + c], f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qs[e] += f[e];
    }
  }
  const dev::u32x4* kc = (const dev::u32x4*)((const char*)a.k_pooled + (size_t)unit * a.n_sub_max * D * ES);
  const float* sec = a.se_pooled + (size_t)unit * a.n_sub_max;
  float* gq = a.sq_out ? a.sq_out + (size_t)unit * max_blocks : nullptr;
  float* ge = a.se_out ? a.se_out + (size_t)unit * max_blocks : nullptr;

  for (int base = 0; base < max_blocks; base += INFL * GROUPS) {
    dev::u32x4 kv[INFL];
    float sev[INFL];
#pragma unroll
    for (int it = 0; it < INFL; ++it) {
      const int J = base + it * GROUPS + wave * RPW + r;
      kv[it] = dev::u32x4{0u, 0u, 0u, 0u};
      sev[it] = -INFINITY;
      if (J < nsub) {
        kv[it] = __builtin_nontemporal_load(kc + (size_t)J * LPR + c);
        if (c == 0) sev[it] = __builtin_nontemporal_load(sec + J);
      }
    }
#pragma unroll
    for (int it = 0; it < INFL; ++it) {
      const int J = base + it * GROUPS + wave * RPW + r;
      float f[EPL];
      dev::widen16<DT>(make_uint4(kv[it].x, kv[it].y, kv[it].z, kv[it].w), f);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(f[e], qs[e], d);
      d = dev::row_sum<LPR>(d);
      if (c == 0 && J < max_blocks) {
        const float vq = J < nsub ? d : -INFINITY;
        s_sq[J] = vq;
        s_se[J] = sev[it];
        if (gq) gq[J] = vq;
        if (ge) ge[J] = sev[it];
      }
    }
  }
  __syncthreads();                       // every wavefront is still here: the scores are complete
  if (wave != 0) return;
  select_unit<R, true>(a.sel, unit, lane, T, s_sq, s_se, sel_smem);
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
  const int R = regs <= 2 ? 2 : regs <= 4 ? 4 : regs <= 8 ? 8 : regs <= 16 ? 16 : regs <= 32 ? 32 : 64;
  NOSA_REQUIRE(ctx, regs <= 64, NOSA_ESHAPE, "selection supports at most %d blocks per unit", kMaxSelectBlocks);
  const size_t smem = (size_t)p.k_blocks * 8 + 2 * (size_t)R * kWave;
  const dim3 grid(ctx->units * batch_mul), block(kWave);   // batch_mul > 1: one virtual batch element per query position
  TimedLaunch tl(ctx, NOSA_KERNEL_SELECT, ctx->main);
  switch (R) {
    case 2: hipLaunchKernelGGL(select_kernel<2>, grid, block, smem, ctx->main, a); break;
    case 4: hipLaunchKernelGGL(select_kernel<4>, grid, block, smem, ctx->main, a); break;
    case 8: hipLaunchKernelGGL(select_kernel<8>, grid, block, smem, ctx->main, a); break;
    case 16: hipLaunchKernelGGL(select_kernel<16>, grid, block, smem, ctx->main, a); break;
    case 32: hipLaunchKernelGGL(select_kernel<32>, grid, block, smem, ctx->main, a); break;
    default: hipLaunchKernelGGL(select_kernel<64>, grid, block, smem, ctx->main, a); break;
  }
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

// Scores, selection and load positions of a step in one launch (one pooled key per block only).
int launch_score_select(nosa_ctx* ctx, const void* q, const void* k_pooled, const float* se_pooled,
                        const int32_t* n_tokens, float* sq_blk, float* se_blk, int32_t* sel_idx, int32_t* n_sel,
                        int32_t* slot_of_block, int32_t* block_of_slot, int32_t* load_list, int32_t* n_load) {
  const nosa_params& p = ctx->p;
  ScoreSelectArgs a;
  a.sel = SelectArgs{nullptr, nullptr, n_tokens, sel_idx, n_sel, slot_of_block, block_of_slot, load_list, n_load,
                     p.n_kv_heads, p.max_blocks, p.k_blocks, p.kq_blocks, p.sink_blocks, p.window_blocks, p.gpu_slots,
                     p.victim_policy, 1, p.max_blocks};
  a.q = q; a.k_pooled = k_pooled; a.se_pooled = se_pooled; a.sq_out = sq_blk; a.se_out = se_blk;
  a.group = ctx->group; a.n_sub_max = p.n_sub_max;
  int regs = (p.max_blocks + kWave - 1) / kWave;
  if (p.victim_policy == 1 && (p.gpu_slots + kWave - 1) / kWave > regs) regs = (p.gpu_slots + kWave - 1) / kWave;
  NOSA_REQUIRE(ctx, regs <= 16, NOSA_ESHAPE, "fused score + selection supports at most 1024 blocks per unit");
  const int R = regs <= 2 ? 2 : regs <= 4 ? 4 : regs <= 8 ? 8 : 16;
  const size_t smem = 2 * (size_t)p.max_blocks * sizeof(float) + (size_t)p.k_blocks * 8 + 2 * (size_t)R * kWave;
  const dim3 grid(ctx->units), block(kFusedThreads);
  TimedLaunch tl(ctx, NOSA_KERNEL_SELECT, ctx->main);
#define NOSA_SS(DT, DD)                                                                                        \
  do {                                                                                                         \
    if (R == 2) hipLaunchKernelGGL((score_select_kernel<DT, DD, 2>), grid, block, smem, ctx->main, a);          \
    else if (R == 4) hipLaunchKernelGGL((score_select_kernel<DT, DD, 4>), grid, block, smem, ctx->main, a);     \
    else if (R == 8) hipLaunchKernelGGL((score_select_kernel<DT, DD, 8>), grid, block, smem, ctx->main, a);     \
    else hipLaunchKernelGGL((score_select_kernel<DT, DD, 16>), grid, block, smem, ctx->main, a);                \
  } while (0)
  if (p.dtype == NOSA_DTYPE_BF16) {
    if (p.head_dim == 128) NOSA_SS(NOSA_DTYPE_BF16, 128); else NOSA_SS(NOSA_DTYPE_BF16, 64);
  } else {
    if (p.head_dim == 128) NOSA_SS(NOSA_DTYPE_F32, 128); else NOSA_SS(NOSA_DTYPE_F32, 64);
  }
#undef NOSA_SS
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

bool score_select_supported(const nosa_params& p) {
  int regs = (p.max_blocks + kWave - 1) / kWave;
  if (p.victim_policy == 1 && (p.gpu_slots + kWave - 1) / kWave > regs) regs = (p.gpu_slots + kWave - 1) / kWave;
  return p.pool_kernel == p.block_size && p.pool_stride == p.block_size && regs <= 16;
}

}  // namespace nosa
