// Block-sparse decode attention over the selected blocks of the paged GPU pool
// (output Eq. of Sec. 3.1 "Attention Calculation"; Alg. 1 Stage 2).
//
// The work is a stream over K and V rows, each read once: the bound is HBM.  Two kernels share the
// launch geometry, the block table, the split bookkeeping and the merge (decode_work_table,
// decode_finish):
//
//  * decode_mfma_kernel (bf16, the default there).  Per byte of K and V there are 4 G flops (G = query
//    heads per KV head); from G = 6 on the vector ALUs cannot keep up with HBM, and the paper's own 3B
//    and 8B models have G = 16.  The heads of a group are one dimension of v_mfma_f32_16x16x32_bf16,
//    so the cost of the two products no longer depends on G and the kernel streams at the same rate
//    for every group size.  Described at the kernel.
//  * decode_partial_kernel (fp32 and bf16), vector ALUs only, described next.
//
// Mapping.  One workgroup (4 wavefronts) handles one (unit, split): a contiguous range of the
// unit's tiles.  In the vector kernel a tile is 8 wave-loads (8 KiB) of K and as many of V from one
// selected block.  In a wave-load every lane reads 16 bytes; 8 adjacent lanes cover one 128-byte line
// of a token row, so one instruction reads whole lines of 8 rows, and VPL = row_bytes / 128
// instructions read the 8 rows completely ("a step").  A lane keeps the slices of q it needs in
// registers (all G heads of the group), forms partial dot products, and the 8 lanes of a row add them
// up with three DPP row operations (no LDS).  The row's scores then sit in exactly the lanes that hold
// the matching slices of the V row, so the P.V update needs no data movement either.  Each of the 8
// row-groups of lanes carries its own online-softmax state (m, l, acc[G][slices]); states are
// merged once at the end: across row-groups by lane exchange, across waves through LDS, across
// splits by the last workgroup of the unit to finish (or by the combine kernel).
//
// Logits are kept in the log2 domain: z' = (scale*log2 e) q.k + b*log2 e, p = 2^(z' - m').
#include <cmath>
#include <mutex>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {

namespace {

using dev::row_sum;
using dev::u32x4;

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
#ifndef NOSA_DECODE_LOADS
#define NOSA_DECODE_LOADS 8
#endif
constexpr int kLoads = NOSA_DECODE_LOADS;   // 16-byte loads of K (and of V) per lane and tile
constexpr int kLPR = 8;     // lanes per row: 8 x 16 B = one 128-byte line
constexpr int kRPW = kWave / kLPR;   // rows per step

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// K/V rows are read exactly once per step: stream them past the caches (non-temporal).
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

struct DecodeArgs {
  const void* q;
  const void* pool_k;
  const void* pool_v;
  const float* pool_bias;
  const int32_t* sel_idx;
  const int32_t* n_sel;
  const int32_t* slot_of_block;
  const int32_t* n_tokens;
  float* part_o;   // [units][splits][G][D] un-normalised
  float* part_ml;  // [units][splits][G][2]  (m in log2 domain, l)
  int32_t* arrived;   // [units] workgroups of a unit that have written their partial result (zero between launches)
  unsigned long long* trace;   // diagnostics (nosa_set_trace), else NULL: 4 words per workgroup
  void* out;
  float* lse;
  const int32_t* load_list;   // phases 1 and 2: the (block, slot) pairs of the fetch in flight
  const int32_t* n_load;
  int n_kv_heads, group, gpu_slots, k_blocks, max_blocks, splits;
  int phase;         // 0: all selected blocks; 1: only blocks not in load_list; 2: only load_list, then merge
  int merge_splits;  // phase 2: number of phase-1 partial results per unit to merge into the output
  float scale_log2e;
};


__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int DT>
struct Vec;  // 16 bytes of one row as seen by one lane

template <>
struct Vec<NOSA_DTYPE_BF16> {
  static constexpr int kElems = 8;
  static constexpr int kBytes = 2;
  uint4 raw;
  __device__ __forceinline__ float dot(const Vec& o) const {
    float d = 0.f;
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, raw.x), __builtin_bit_cast(bf16x2_t, o.raw.x), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, raw.y), __builtin_bit_cast(bf16x2_t, o.raw.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, raw.z), __builtin_bit_cast(bf16x2_t, o.raw.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, raw.w), __builtin_bit_cast(bf16x2_t, o.raw.w), d, false);
    return d;
  }
  __device__ __forceinline__ void widen(float (&f)[8]) const {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <>
struct Vec<NOSA_DTYPE_F32> {
  static constexpr int kElems = 4;
  static constexpr int kBytes = 4;
  uint4 raw;
  __device__ __forceinline__ float dot(const Vec& o) const {
    float d = __uint_as_float(raw.x) * __uint_as_float(o.raw.x);
    d = fmaf(__uint_as_float(raw.y), __uint_as_float(o.raw.y), d);
    d = fmaf(__uint_as_float(raw.z), __uint_as_float(o.raw.z), d);
    d = fmaf(__uint_as_float(raw.w), __uint_as_float(o.raw.w), d);
    return d;
  }
  __device__ __forceinline__ void widen(float (&f)[4]) const {
    f[0] = __uint_as_float(raw.x);
    f[1] = __uint_as_float(raw.y);
    f[2] = __uint_as_float(raw.z);
    f[3] = __uint_as_float(raw.w);
  }
};

__device__ __forceinline__ void store_out(void* out, size_t idx, float v, int dt) {
  if (dt == NOSA_DTYPE_F32) {
    ((float*)out)[idx] = v;
  } else {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
      u = (u >> 16) | 0x40;
    } else {
      u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
      u >>= 16;
    }
    ((uint16_t*)out)[idx] = (uint16_t)u;
  }
}

// Partial results that are exchanged between workgroups of ONE launch travel as relaxed device-scope
// atomics: such stores are written through the XCD's L2 and such loads do not hit lines that another
// XCD may have made stale, so the data is coherent across the chip's eight L2 caches without the
// whole-cache write-back and invalidate that a device-scope fence costs (measured: those fences, one per
// workgroup, tripled the kernel's duration).  Ordering is then a matter of waiting for the stores to be
// acknowledged before the arrival counter is bumped.
template <bool COHERENT>
__device__ __forceinline__ float part_load(const float* p) {
  if constexpr (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}
template <bool COHERENT>
__device__ __forceinline__ void part_store(float* p, float v) {
  if constexpr (COHERENT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
__device__ __forceinline__ void wait_vector_memory() {   // s_waitcnt vmcnt(0): this wave's loads and stores are done
  __builtin_amdgcn_s_waitcnt(0 | (0x7 << 4) | (0xf << 8));
}

// Log-sum-exp merge of the `splits` partial results of one unit into the output, by one workgroup.
// Used by the stand-alone combine kernel (COHERENT = false: a kernel boundary lies between writers and
// reader) and by the last workgroup of a unit inside the attention kernel (COHERENT = true): the same
// arithmetic in the same order, so both give the same bits.
template <int DT, bool COHERENT>
__device__ __forceinline__ void combine_unit(const float* part_o, const float* part_ml, void* out, float* lse, int unit,
                                             int n_kv_heads, int G, int D, int splits) {
  const int b = unit / n_kv_heads, h = unit % n_kv_heads;
  for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
    const int g = idx / D, e = idx % D;
    const size_t p0 = ((size_t)unit * splits) * G + g;
    float M = -INFINITY;
    for (int s = 0; s < splits; ++s) M = fmaxf(M, part_load<COHERENT>(part_ml + (p0 + (size_t)s * G) * 2));
    float L = 0.f, O = 0.f;
    for (int s = 0; s < splits; ++s) {
      const size_t pi = p0 + (size_t)s * G;
      const float ms = part_load<COHERENT>(part_ml + pi * 2);
      const float sc = (ms == -INFINITY) ? 0.f : fast_exp2(ms - M);
      L = fmaf(part_load<COHERENT>(part_ml + pi * 2 + 1), sc, L);
      O = fmaf(part_load<COHERENT>(part_o + pi * D + e), sc, O);
    }
    const size_t o = ((size_t)b * n_kv_heads * G + (size_t)h * G + g) * D + e;
    store_out(out, o, L > 0.f ? O / L : 0.f, DT);
    if (lse && e == 0) lse[(size_t)b * n_kv_heads * G + h * G + g] = L > 0.f ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
  }
}

// The merge as done by the last workgroup of a unit inside the attention kernel: the arithmetic of
// combine_unit in the same order (so the same bits), but every partial value a lane needs -- up to SMAX
// splits for each of its output elements -- is requested before the first one is used, so the merge pays
// one round trip to memory instead of one per split.  Splits beyond `splits` contribute m = -inf, l = 0:
// a term of weight zero.
template <int DT, int D, int NI, int SMAX>
__device__ __forceinline__ void merge_arrived(const float* part_o, const float* part_ml, void* out, float* lse, int unit,
                                              int n_kv_heads, int G, int splits) {
  const int b = unit / n_kv_heads, h = unit % n_kv_heads;
  float ms[NI][SMAX], ls[NI][SMAX], os[NI][SMAX];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int idx = threadIdx.x + i * kThreads;
    const bool ok = idx < G * D;
    const int g = ok ? idx / D : 0, e = idx % D;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
      const bool live = ok && s < splits;
      const size_t pi = ((size_t)unit * splits + (live ? s : 0)) * G + g;
      ms[i][s] = live ? part_load<true>(part_ml + pi * 2) : -INFINITY;
      ls[i][s] = live ? part_load<true>(part_ml + pi * 2 + 1) : 0.f;
      os[i][s] = live ? part_load<true>(part_o + pi * D + e) : 0.f;
    }
  }
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int idx = threadIdx.x + i * kThreads;
    if (idx >= G * D) continue;
    const int g = idx / D, e = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) M = fmaxf(M, ms[i][s]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
      const float sc = (ms[i][s] == -INFINITY) ? 0.f : fast_exp2(ms[i][s] - M);
      L = fmaf(ls[i][s], sc, L);
      O = fmaf(os[i][s], sc, O);
    }
    const size_t o = ((size_t)b * n_kv_heads * G + (size_t)h * G + g) * D + e;
    store_out(out, o, L > 0.f ? O / L : 0.f, DT);
    if (lse && e == 0) lse[(size_t)b * n_kv_heads * G + h * G + g] = L > 0.f ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
  }
}

// Resolves the blocks a workgroup attends into (slot, valid tokens) pairs in LDS, once per workgroup.
// phase 0: the whole selection; phase 1: the selection minus the blocks of the fetch in flight; phase 2: only
// those blocks.  Returns the number of table entries.  Followed by a barrier in the caller.
template <bool OVERLAP>
__device__ __forceinline__ int decode_work_table(const DecodeArgs& a, const int phase, const int unit, const int tid,
                                                 const int T, int* s_slot, int* s_valid) {
  int n_sel;
  if (phase == 2) {
    // the blocks that were fetched for this step: (block, slot) pairs of the load list
    n_sel = min(a.n_load[unit], a.k_blocks);
    const int32_t* ll = a.load_list + (size_t)unit * a.k_blocks * 2;
    const int n_all = min(a.n_sel[unit], a.k_blocks);
    const int32_t* sel = a.sel_idx + (size_t)unit * a.k_blocks;
    for (int i = tid; i < n_sel; i += kThreads) {
      const int J = ll[2 * i], slot = ll[2 * i + 1];
      int valid = (J >= 0 && J < a.max_blocks) ? min(kBlockTokens, T - J * kBlockTokens) : 0;
      if (slot < 0 || slot >= a.gpu_slots) valid = 0;
      // only blocks of the selection are attended (the selection is ascending)
      int lo = 0, hi = n_all;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (sel[mid] < J) lo = mid + 1; else hi = mid;
      }
      if (!(lo < n_all && sel[lo] == J)) valid = 0;
      s_slot[i] = slot;
      s_valid[i] = valid;
    }
  } else {
    n_sel = min(a.n_sel[unit], a.k_blocks);
    const int n_ld = phase == 1 ? min(a.n_load[unit], a.k_blocks) : 0;
    const int32_t* ll = a.load_list + (size_t)unit * a.k_blocks * 2;
    for (int i = tid; i < n_sel; i += kThreads) {
      const int J = a.sel_idx[(size_t)unit * a.k_blocks + i];
      int slot = -1, valid = 0;
      if (J >= 0 && J < a.max_blocks) {
        slot = a.slot_of_block[(size_t)unit * a.max_blocks + J];
        valid = min(kBlockTokens, T - J * kBlockTokens);
      }
      if (slot < 0 || slot >= a.gpu_slots) valid = 0;   // never dereference a bad slot
      if (n_ld > 0) {   // phase 1: leave out the blocks still in flight (load list is ascending by block)
        int lo = 0, hi = n_ld;
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (ll[2 * mid] < J) lo = mid + 1; else hi = mid;
        }
        if (lo < n_ld && ll[2 * lo] == J) valid = 0;
      }
      s_slot[i] = slot;
      s_valid[i] = valid;
    }
  }
  return n_sel;
}

// Last part of an attention workgroup: the per-wave states (m in the log2 domain, l, un-normalised O) that the
// waves left in LDS are merged; the result is the output (one split, or phase 2, which also folds in the
// phase-1 partial results), or a partial result, which the last workgroup of the unit to arrive merges.
// GS = heads the LDS arrays are laid out for (row stride), G = heads of the group (<= GS; a compile-time constant
// at the vector kernel's call site, a kernel argument at the matrix-core kernel's).
template <int DT, int D, int GS, bool OVERLAP>
__device__ __forceinline__ void decode_finish(const DecodeArgs& a, const int phase, const int unit, const int split,
                                              const int b, const int h, const int tid, const int G,
                                              const float (*s_m)[GS], const float (*s_l)[GS], const float (*s_acc)[GS][D],
                                              const unsigned long long t_start) {
  constexpr float NEG_INF = -INFINITY;
  // ---- merge the waves; write the partial result (or the output when there is one split) ----
  for (int idx = tid; idx < G * D; idx += kThreads) {
    const int g = idx / D, e = idx % D;
    float M = s_m[0][g];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w][g]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float sc = (s_m[w][g] == NEG_INF) ? 0.f : fast_exp2(s_m[w][g] - M);
      L = fmaf(s_l[w][g], sc, L);
      O = fmaf(s_acc[w][g][e], sc, O);
    }
    if (phase == 2) {
      // fold in the partial results of the resident blocks (written by the phase-1 launch)
      const size_t p0 = ((size_t)unit * a.merge_splits) * G + g;
      float M2 = M;
      for (int sp = 0; sp < a.merge_splits; ++sp) M2 = fmaxf(M2, a.part_ml[(p0 + (size_t)sp * G) * 2]);
      const float sc0 = (M == NEG_INF) ? 0.f : fast_exp2(M - M2);
      L *= sc0;
      O *= sc0;
      for (int sp = 0; sp < a.merge_splits; ++sp) {
        const size_t pi = p0 + (size_t)sp * G;
        const float ms = a.part_ml[pi * 2];
        const float sc = (ms == NEG_INF) ? 0.f : fast_exp2(ms - M2);
        L = fmaf(a.part_ml[pi * 2 + 1], sc, L);
        O = fmaf(a.part_o[pi * D + e], sc, O);
      }
      M = M2;
    }
    if (phase == 2 || (a.splits == 1 && phase == 0)) {
      const size_t o = ((size_t)b * a.n_kv_heads * G + (size_t)h * G + g) * D + e;
      store_out(a.out, o, L > 0.f ? O / L : 0.f, DT);
      if (a.lse && e == 0) a.lse[(size_t)b * a.n_kv_heads * G + h * G + g] = L > 0.f ? (M + log2f(L)) * 0.6931471805599453f : NEG_INF;
    } else {
      const size_t pidx = ((size_t)unit * a.splits + split) * G + g;
      if (!OVERLAP && a.arrived) {       // read by another workgroup of this very launch
        part_store<true>(a.part_o + pidx * D + e, O);
        if (e == 0) {
          part_store<true>(a.part_ml + pidx * 2, M);
          part_store<true>(a.part_ml + pidx * 2 + 1, L);
        }
      } else {
        a.part_o[pidx * D + e] = O;
        if (e == 0) {
          a.part_ml[pidx * 2] = M;
          a.part_ml[pidx * 2 + 1] = L;
        }
      }
    }
  }
  if constexpr (!OVERLAP) {
    // Several splits and a counter array: the workgroup that finds all the others of its unit done merges
    // their partial results into the output, which saves the separate combine launch.  Every lane waits
    // until its partial-result stores are acknowledged, the workgroup meets, one lane bumps the unit's
    // counter; whoever reads splits - 1 there is the last arrival and does the merge.  Nobody waits for
    // anybody else.  The last arrival puts the counter back to zero for the next launch.
    if (a.splits > 1 && a.arrived != nullptr) {
      __shared__ int s_last;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      wait_vector_memory();
      __syncthreads();
      if (tid == 0) {
        const int before = __hip_atomic_fetch_add(a.arrived + unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = before == a.splits - 1;
      }
      __syncthreads();
      if (s_last) {
        wait_vector_memory();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        // all partial values in flight at once while that fits the registers: (outputs per lane) x (splits) x 3
        constexpr int kPerLaneMax = (GS * D + kThreads - 1) / kThreads;
        constexpr int kPerLane8 = kPerLaneMax < 8 ? kPerLaneMax : 8, kPerLane4 = kPerLaneMax < 4 ? kPerLaneMax : 4;
        const int per_lane = (G * D + kThreads - 1) / kThreads;
        if (a.splits <= 4 && per_lane <= kPerLane8)
          merge_arrived<DT, D, kPerLane8, 4>(a.part_o, a.part_ml, a.out, a.lse, unit, a.n_kv_heads, G, a.splits);
        else if (a.splits <= 8 && per_lane <= kPerLane4)
          merge_arrived<DT, D, kPerLane4, 8>(a.part_o, a.part_ml, a.out, a.lse, unit, a.n_kv_heads, G, a.splits);
        else
          combine_unit<DT, true>(a.part_o, a.part_ml, a.out, a.lse, unit, a.n_kv_heads, G, D, a.splits);
        if (tid == 0) __hip_atomic_store(a.arrived + unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    if (a.trace && tid == 0) {   // when and where this workgroup ran: start, end, XCD (hardware register XCC_ID), its index
      unsigned long long* t = a.trace + (size_t)blockIdx.x * 4;
      t[0] = t_start;
      t[1] = __builtin_amdgcn_s_memrealtime();
      t[2] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 0xfu;
      t[3] = blockIdx.x;
    }
  }
}

// OVERLAP = false: the plain kernel (phase 0).  OVERLAP = true: the two launches that bracket a
// gather in flight (phase 1: resident blocks only; phase 2: fetched blocks, then the merge); a
// separate instantiation so that profiles list the stand-alone kernel on its own.
template <int DT, int D, int G, bool OVERLAP>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(const DecodeArgs a) {
  const int phase = OVERLAP ? a.phase : 0;
  const bool has_bias = a.pool_bias != nullptr;
  using V = Vec<DT>;
  constexpr int EPL = V::kElems;                 // elements per 16-byte load
  constexpr int RP = D / EPL;                    // row pitch in 16-byte vectors
  constexpr int VPL = RP / kLPR;                 // loads per lane and row (row_bytes / 128)
  constexpr int STEPS = kLoads / VPL;            // steps (of 8 rows) per tile
  constexpr int TILE = kRPW * STEPS;             // tokens per tile
  constexpr int TPB = kBlockTokens / TILE;       // tiles per block
  constexpr int LE = VPL * EPL;                  // elements of a row held by one lane
  static_assert(VPL >= 1 && STEPS >= 1 && TPB >= 1 && TPB * TILE == kBlockTokens, "tile must divide the block");
  constexpr float NEG_INF = -INFINITY;

  __shared__ int s_slot[kMaxSelBlocks];
  __shared__ int s_valid[kMaxSelBlocks];
  __shared__ float s_m[kWaves][G];
  __shared__ float s_l[kWaves][G];
  __shared__ float s_acc[kWaves][G][D];

  const int unit = blockIdx.x / a.splits;
  const int split = blockIdx.x % a.splits;
  const int b = unit / a.n_kv_heads;
  const int h = unit % a.n_kv_heads;
  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;
  const int r = lane / kLPR;   // row-group within the wave
  const int c = lane % kLPR;   // 16-byte slice of a 128-byte line

  unsigned long long t_start = 0;
  if (!OVERLAP && a.trace && tid == 0) t_start = __builtin_amdgcn_s_memrealtime();   // 100 MHz real-time counter

  const int T = a.n_tokens[b];
  const int n_sel = decode_work_table<OVERLAP>(a, phase, unit, tid, T, s_slot, s_valid);   // entries of the work table

  // q slices of this lane for all heads of the group: line v of the row, 16-byte slice c
  V qv[G][VPL];
  {
    const uint4* qp = (const uint4*)((const char*)a.q + ((size_t)b * a.n_kv_heads * G + (size_t)h * G) * D * V::kBytes);
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int v = 0; v < VPL; ++v) qv[g][v].raw = qp[g * RP + v * kLPR + c];
  }

  float m[G], l[G], acc[G][LE];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = NEG_INF;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < LE; ++e) acc[g][e] = 0.f;
  }
  __syncthreads();

  const int total_tiles = n_sel * TPB;
  const int t_begin = (int)(((long long)split * total_tiles) / a.splits);
  const int t_end = (int)(((long long)(split + 1) * total_tiles) / a.splits);
  constexpr size_t kBlockBytes = (size_t)kBlockTokens * D * V::kBytes;

  for (int t = t_begin + wave; t < t_end; t += kWaves) {
    const int i_blk = t / TPB;
    const int part = t % TPB;
    const int nvalid = s_valid[i_blk] - part * TILE;
    if (nvalid <= 0) continue;
    const size_t slot_lin = (size_t)unit * a.gpu_slots + s_slot[i_blk];
    const size_t row0 = (size_t)part * TILE + r;
    const uint4* kp = (const uint4*)((const char*)a.pool_k + slot_lin * kBlockBytes) + row0 * RP + c;
    const uint4* vp = (const uint4*)((const char*)a.pool_v + slot_lin * kBlockBytes) + row0 * RP + c;

    V kx[STEPS][VPL], vx[STEPS][VPL];
    float bx[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
#pragma unroll
      for (int v = 0; v < VPL; ++v) kx[i][v].raw = load_stream(kp + i * (kRPW * RP) + v * kLPR);
    if (has_bias) {
      const float* bp = a.pool_bias + slot_lin * kBlockTokens + row0;
#pragma unroll
      for (int i = 0; i < STEPS; ++i) bx[i] = __builtin_nontemporal_load(bp + i * kRPW) * 1.4426950408889634f;
    } else {
#pragma unroll
      for (int i = 0; i < STEPS; ++i) bx[i] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
#pragma unroll
      for (int v = 0; v < VPL; ++v) vx[i][v].raw = load_stream(vp + i * (kRPW * RP) + v * kLPR);

    float s[G][STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
      const float bl = bx[i];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = kx[i][0].dot(qv[g][0]);
#pragma unroll
        for (int v = 1; v < VPL; ++v) d += kx[i][v].dot(qv[g][v]);
        s[g][i] = fmaf(row_sum<kLPR>(d), a.scale_log2e, bl);
      }
    }

    const bool masked = nvalid < TILE;   // wave-uniform: only the partial tail block takes this path
    if (masked) {
#pragma unroll
      for (int i = 0; i < STEPS; ++i) {
        const bool ok = (i * kRPW + r) < nvalid;
#pragma unroll
        for (int g = 0; g < G; ++g) s[g][i] = ok ? s[g][i] : NEG_INF;
        if (!ok) {   // stale bytes beyond T must not reach the sum
#pragma unroll
          for (int v = 0; v < VPL; ++v) vx[i][v].raw = make_uint4(0, 0, 0, 0);
        }
      }
    }

    // New running maxima.  When no lane of the wave sees one move (the usual case once a few tiles have
    // passed), every rescale factor is exactly 1 and the multiplications are skipped: same bits, fewer
    // instructions.
    float m_new[G];
    bool moved = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mt = s[g][0];
#pragma unroll
      for (int i = 1; i < STEPS; ++i) mt = fmaxf(mt, s[g][i]);
      m_new[g] = fmaxf(m[g], mt);
      moved |= m_new[g] != m[g];
    }
    if (__builtin_amdgcn_ballot_w64(moved) != 0ull) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float m_use = (m_new[g] == NEG_INF) ? 0.f : m_new[g];
        const float alpha = fast_exp2(m[g] - m_use);
        m[g] = m_new[g];
        l[g] *= alpha;
#pragma unroll
        for (int e = 0; e < LE; ++e) acc[g][e] *= alpha;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m_use = (m[g] == NEG_INF) ? 0.f : m[g];
#pragma unroll
      for (int i = 0; i < STEPS; ++i) s[g][i] = fast_exp2(s[g][i] - m_use);
    }
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
#pragma unroll
      for (int g = 0; g < G; ++g) l[g] += s[g][i];
#pragma unroll
      for (int i = 0; i < STEPS; ++i) {
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          float vf[EPL];
          vx[i][v].widen(vf);
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const float p = s[g][i];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][v * EPL + e] = fmaf(p, vf[e], acc[g][v * EPL + e]);
          }
        }
      }
  }

  // ---- merge the 8 row-group states of this wave (lane exchange) ----
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float M = m[g];
#pragma unroll
    for (int off = kLPR; off < kWave; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float sc = (m[g] == NEG_INF) ? 0.f : fast_exp2(m[g] - M);
    float lg = l[g] * sc;
#pragma unroll
    for (int off = kLPR; off < kWave; off <<= 1) lg += __shfl_xor(lg, off);
#pragma unroll
    for (int e = 0; e < LE; ++e) {
      float x = acc[g][e] * sc;
#pragma unroll
      for (int off = kLPR; off < kWave; off <<= 1) x += __shfl_xor(x, off);
      acc[g][e] = x;
    }
    m[g] = M;
    l[g] = lg;
  }
  if (r == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int v = 0; v < VPL; ++v)
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_acc[wave][g][(v * kLPR + c) * EPL + e] = acc[g][v * EPL + e];
      if (c == 0) {
        s_m[wave][g] = m[g];
        s_l[wave][g] = l[g];
      }
    }
  }
  __syncthreads();

  decode_finish<DT, D, G, OVERLAP>(a, phase, unit, split, b, h, tid, G, s_m, s_l, s_acc, t_start);
}

// ---- the same attention on the matrix cores, for large query groups ------------------------------------
// With G query heads per KV head the vector kernel above does 4 G flops per byte: at G = 8 it is bound by
// its arithmetic and registers, at G = 16 (the paper's own 3B and 8B models: 32 query / 2 KV heads) it
// spills.  A group of up to 16 heads is exactly one N dimension of v_mfma_f32_16x16x32_bf16, so this
// kernel (bf16 only) computes, per tile of 32 tokens and per wave,
//   S^T = K Q^T    A = 16 token rows of K straight from global memory in operand order (lane = token row
//                  l % 16, 16-byte slice l / 16 of a 64-byte piece of the row), B = Q^T in registers for the
//                  whole kernel (lane = head l % 16, zero for l % 16 >= G).  In the C layout a lane owns one
//                  head (column l % 16) and 4 tokens per 16-token tile.
//   O^T += V^T P^T A = V^T from this wave's private LDS tile, B = P^T = the lane's own 8 weights (bf16).
//                  In the C layout a lane owns one head again, so the running maximum, the sum and the
//                  rescale of O all stay in the lane; only the tile maximum is exchanged between the four
//                  lanes of a head (two shuffles per tile).
// V arrives in full 128-byte lines as [token][d] and is transposed on its way into LDS: two tokens of one
// column share a 32-bit word (byte permute), the words go to row d of a [d][32 positions] tile whose 16-byte
// chunks are XOR-swizzled.  The position of a token inside a row is chosen so that the 8 weights a lane
// holds after the score product are 8 consecutive positions (a sum over tokens does not care about their
// order).  LDS is private to a wave: its loads and stores execute in order, no barrier inside the loop.
// Weights are rounded to bf16 (nearest even) for the second product; the row sums use the unrounded ones.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {   // round to nearest even
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// x of lanes l, l ^ 16, l ^ 32, l ^ 48 combined: the four lanes that hold one head
__device__ __forceinline__ float head_max(float x) {
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}

constexpr int kHeadTile = 16;   // heads per matrix-core tile: the largest group the kernel takes

template <int D, bool OVERLAP>
__global__ __launch_bounds__(kThreads) void decode_mfma_kernel(const DecodeArgs a) {
  constexpr int DT = NOSA_DTYPE_BF16;
  const int G = a.group;                 // 1 .. 16 heads per KV head
  constexpr int KC = D / 32;             // k-steps of the score product
  constexpr int NDT = D / 16;            // 16-row tiles of O^T
  constexpr int ROWB = D * 2;            // bytes per K or V row
  constexpr int VPL = ROWB / 128;        // 128-byte lines per row
  constexpr int TILE = 32;               // tokens per tile
  constexpr int TPB = kBlockTokens / TILE;
  constexpr int kVt = D * 64;            // bytes of one wave's V^T tile: D rows x 32 positions x 2 B
  constexpr float NEG_INF = -INFINITY;
  constexpr float kLog2e = 1.4426950408889634f;
  const int phase = OVERLAP ? a.phase : 0;

  __shared__ int s_slot[kMaxSelBlocks];
  __shared__ int s_valid[kMaxSelBlocks];
  __shared__ float s_m[kWaves][kHeadTile];
  __shared__ float s_l[kWaves][kHeadTile];
  __shared__ __align__(16) unsigned char s_buf[kWaves * kVt];   // V^T tiles in the loop, the waves' O afterwards
  static_assert(sizeof(float) * kWaves * kHeadTile * D <= sizeof(s_buf), "the per-wave results must fit the tile buffer");
  float (*s_acc)[kHeadTile][D] = reinterpret_cast<float (*)[kHeadTile][D]>(s_buf);

  const int unit = blockIdx.x / a.splits;
  const int split = blockIdx.x % a.splits;
  const int b = unit / a.n_kv_heads;
  const int h = unit % a.n_kv_heads;
  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;
  const int l16 = lane % 16, g4 = lane / 16;   // operand / accumulator coordinates
  const int r8 = lane / 8, c8 = lane % 8;      // coordinates of the V loads: row pair, 16-byte slice of a line

  unsigned long long t_start = 0;
  if (!OVERLAP && a.trace && tid == 0) t_start = __builtin_amdgcn_s_memrealtime();

  const int T = a.n_tokens[b];
  const int n_sel = decode_work_table<OVERLAP>(a, phase, unit, tid, T, s_slot, s_valid);

  // Q^T: head l16 (zero beyond the group), d = 32 kc + 8 g4 .. + 7
  bf16x8_t qb[KC];
  {
    const char* qp = (const char*)a.q + ((size_t)b * a.n_kv_heads * G + (size_t)h * G + (l16 < G ? l16 : 0)) * ROWB;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (l16 < G) v = *(const u32x4*)(qp + kc * 64 + g4 * 16);
      qb[kc] = __builtin_bit_cast(bf16x8_t, v);
    }
  }
  f32x4_t ot[NDT];
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt) ot[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = NEG_INF, l_run = 0.f;   // head l16; l_run covers this lane's tokens only

  // V^T tile of this wave.  Token 16 m + 4 q + j of a tile sits at position 8 q + 4 m + j of a row; the lane
  // (r8, c8) holds tokens 2 r8 and 2 r8 + 1 (+ 16 m) of slice c8: one word at byte 16 (r8 / 2) + 8 m + 4 (r8 % 2)
  // of row d, chunk index XORed with (d / 8) % 4 = c8 % 4.  Lanes with odd c8 write their odd column first,
  // so that one store instruction touches rows of both parities (all 32 banks).
  unsigned char* vt = s_buf + wave * kVt;
  const int vchunk = ((r8 >> 1) ^ (c8 & 3)) * 16 + 4 * (r8 & 1);
  unsigned char* vw_first = vt + (8 * c8 + (c8 & 1)) * 64 + vchunk;
  unsigned char* vw_second = vt + (8 * c8 + 1 - (c8 & 1)) * 64 + vchunk;
  const uint32_t sel_first = (c8 & 1) ? 0x07060302u : 0x05040100u;    // high (odd column) or low halves of two words
  const uint32_t sel_second = (c8 & 1) ? 0x05040100u : 0x07060302u;
  // operand reads: row d = 16 dt + l16, positions 8 g4 .. + 7 = chunk g4 ^ ((d / 8) % 4)
  const unsigned char* vr0 = vt + l16 * 64 + ((g4 ^ (l16 >> 3)) * 16);          // tiles with (2 dt) % 4 == 0
  const unsigned char* vr2 = vt + l16 * 64 + ((g4 ^ (l16 >> 3) ^ 2) * 16);      // tiles with (2 dt) % 4 == 2
  __syncthreads();

  const int total_tiles = n_sel * TPB;
  const int t_begin = (int)(((long long)split * total_tiles) / a.splits);
  const int t_end = (int)(((long long)(split + 1) * total_tiles) / a.splits);
  constexpr size_t kBlockBytes = (size_t)kBlockTokens * ROWB;

  for (int t = t_begin + wave; t < t_end; t += kWaves) {
    const int i_blk = t / TPB;
    const int part = t % TPB;
    const int nvalid = s_valid[i_blk] - part * TILE;
    if (nvalid <= 0) continue;
    const size_t slot_lin = (size_t)unit * a.gpu_slots + s_slot[i_blk];
    const char* kp = (const char*)a.pool_k + slot_lin * kBlockBytes + (size_t)(part * TILE + l16) * ROWB + g4 * 16;
    const char* vp = (const char*)a.pool_v + slot_lin * kBlockBytes + (size_t)(part * TILE + 2 * r8) * ROWB + c8 * 16;

    u32x4 kx[2][KC], vx[4][VPL];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int kc = 0; kc < KC; ++kc)
        kx[m][kc] = __builtin_nontemporal_load((const u32x4*)(kp + (size_t)m * 16 * ROWB + kc * 64));
    f32x4_t bz[2] = {f32x4_t{0.f, 0.f, 0.f, 0.f}, f32x4_t{0.f, 0.f, 0.f, 0.f}};
    if (a.pool_bias != nullptr) {
      const float* bp = a.pool_bias + slot_lin * kBlockTokens + part * TILE + 4 * g4;
      bz[0] = __builtin_nontemporal_load((const f32x4_t*)bp);
      bz[1] = __builtin_nontemporal_load((const f32x4_t*)(bp + 16));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)     // token 2 r8 + (i & 1) + 16 (i >> 1)
#pragma unroll
      for (int v = 0; v < VPL; ++v)
        vx[i][v] = __builtin_nontemporal_load((const u32x4*)(vp + (size_t)((i & 1) + 16 * (i >> 1)) * ROWB + v * 128));

    // scores: st[m][j] = token 16 m + 4 g4 + j, head l16
    f32x4_t st[2] = {f32x4_t{0.f, 0.f, 0.f, 0.f}, f32x4_t{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int kc = 0; kc < KC; ++kc)
#pragma unroll
      for (int m = 0; m < 2; ++m)
        st[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx[m][kc]), qb[kc], st[m], 0, 0, 0);

    float z[2][4];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int j = 0; j < 4; ++j) z[m][j] = fmaf(st[m][j], a.scale_log2e, bz[m][j] * kLog2e);
    const bool masked = nvalid < TILE;   // wave-uniform: only the partial tail block takes this path
    if (masked) {
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (16 * m + 4 * g4 + j >= nvalid) z[m][j] = NEG_INF;
#pragma unroll
      for (int i = 0; i < 4; ++i)        // stale bytes beyond T must not reach the sum
        if (2 * r8 + (i & 1) + 16 * (i >> 1) >= nvalid)
#pragma unroll
          for (int v = 0; v < VPL; ++v) vx[i][v] = u32x4{0u, 0u, 0u, 0u};
    }
    float mt = fmaxf(fmaxf(fmaxf(z[0][0], z[0][1]), fmaxf(z[0][2], z[0][3])),
                     fmaxf(fmaxf(z[1][0], z[1][1]), fmaxf(z[1][2], z[1][3])));
    mt = head_max(mt);
    const float m_new = fmaxf(m_run, mt);
    if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0ull) {
      const float m_use = (m_new == NEG_INF) ? 0.f : m_new;
      const float alpha = fast_exp2(m_run - m_use);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt) ot[dt] *= alpha;
    }
    const float m_use = (m_run == NEG_INF) ? 0.f : m_run;
    float p[2][4];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        p[m][j] = fast_exp2(z[m][j] - m_use);
        l_run += p[m][j];
      }
    const u32x4 pw = {pack2_bf16(p[0][0], p[0][1]), pack2_bf16(p[0][2], p[0][3]), pack2_bf16(p[1][0], p[1][1]),
                      pack2_bf16(p[1][2], p[1][3])};   // positions 8 g4 + 4 m + j
    const bf16x8_t pb = __builtin_bit_cast(bf16x8_t, pw);

    // V^T into LDS
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int v = 0; v < VPL; ++v)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t lo = vx[2 * m][v][w], hi = vx[2 * m + 1][v][w];   // tokens t and t + 1, columns 2 w and 2 w + 1 of the slice
          const int off = (64 * v + 2 * w) * 64 + 8 * m;
          *(uint32_t*)(vw_first + off) = __builtin_amdgcn_perm(hi, lo, sel_first);
          *(uint32_t*)(vw_second + off) = __builtin_amdgcn_perm(hi, lo, sel_second);
        }
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) {
      const unsigned char* rp = ((2 * dt) & 2) ? vr2 : vr0;
      const bf16x8_t av = *(const bf16x8_t*)(rp + dt * 16 * 64);
      ot[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb, ot[dt], 0, 0, 0);
    }
  }

  // the wave's result: O^T values are complete sums; only l is spread over the four lanes of a head
  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  __syncthreads();     // every wave is done with its V^T tile: the buffer now takes the waves' O
  if (l16 < G) {
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
      *(f32x4_t*)(&s_acc[wave][l16][16 * dt + 4 * g4]) = ot[dt];
    if (g4 == 0) {
      s_m[wave][l16] = m_run;
      s_l[wave][l16] = l_tot;
    }
  }
  __syncthreads();
  decode_finish<DT, D, kHeadTile, OVERLAP>(a, phase, unit, split, b, h, tid, G, s_m, s_l, s_acc, t_start);
}

// One workgroup per unit: merges the split partial results with log-sum-exp weights.
template <int DT>
__global__ __launch_bounds__(kThreads) void decode_combine_kernel(const float* __restrict__ part_o,
                                                                  const float* __restrict__ part_ml, void* out,
                                                                  float* lse, int n_kv_heads, int G, int D, int splits) {
  combine_unit<DT, false>(part_o, part_ml, out, lse, blockIdx.x, n_kv_heads, G, D, splits);
}

template <int D, bool OVERLAP>
bool dispatch_mfma(int g, const DecodeArgs& a, dim3 grid, hipStream_t s) {
  if (g < 1 || g > kHeadTile) return false;
  hipLaunchKernelGGL((decode_mfma_kernel<D, OVERLAP>), grid, dim3(kThreads), 0, s, a);
  return true;
}

template <int DT, int D, bool OVERLAP>
bool dispatch_group(int g, const DecodeArgs& a, dim3 grid, hipStream_t s) {
#define NOSA_CASE(GG)                                                                                       \
  case GG:                                                                                                  \
    hipLaunchKernelGGL((decode_partial_kernel<DT, D, GG, OVERLAP>), grid, dim3(kThreads), 0, s, a);         \
    return true;
  switch (g) {
    NOSA_CASE(1) NOSA_CASE(2) NOSA_CASE(3) NOSA_CASE(4) NOSA_CASE(6) NOSA_CASE(8) NOSA_CASE(12) NOSA_CASE(16)
    default: return false;
  }
#undef NOSA_CASE
}

}  // namespace

// Scratch of the allocation-free entry point (nosa_sparse_decode_static): one array per GPU, part of the
// loaded code object, alive until the process ends.  In host code the array's name is only a handle of
// the symbol, not a device address: the address on a given GPU comes from hipGetSymbolAddress with that
// GPU current, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[NOSA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};   // address of `scratch` on each device, looked up once
}  // namespace

// Address of the static scratch on `device`, which must be the current device.
int decode_static_scratch(nosa_ctx* ctx, int device, void** out) {
  NOSA_REQUIRE(ctx, device >= 0 && device < kMaxDevices, NOSA_ESHAPE, "device %d: the static scratch is kept for devices 0..%d",
               device, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    NOSA_HIP(ctx, hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    NOSA_REQUIRE(ctx, ptr != nullptr && ((uintptr_t)ptr & 255) == 0, NOSA_EHIP,
                 "hipGetSymbolAddress returned %p for the static scratch", ptr);
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return NOSA_OK;
}

// The scratch of a decode call starts with one arrival counter per unit.  In a caller's workspace, which belongs
// to one context, the counters take units * 4 bytes rounded up to 256 ...
size_t decode_counter_bytes(const nosa_ctx* ctx) { return (((size_t)ctx->units * sizeof(int32_t)) + 255) & ~(size_t)255; }

// ... in the static array, which contexts of any shape share one after the other, they take a fixed region
// (NOSA_STATIC_SCRATCH_UNITS counters): no context ever writes partial results where another keeps counters,
// so the counters stay zero between launches whatever ran before.
size_t decode_static_counter_bytes() { return (size_t)NOSA_STATIC_SCRATCH_UNITS * sizeof(int32_t); }

// The counters are followed by the split partial results: O[G][D] and (m, l)[G] per (unit, split).
size_t decode_partial_bytes(const nosa_ctx* ctx) {
  return (size_t)ctx->units * ctx->splits * ctx->group * (size_t)(ctx->p.head_dim + 2) * sizeof(float);
}

namespace {
__global__ void zero_counters_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}
}  // namespace

// Arrival counters of a workspace the caller has just handed over must start at zero (a fill kernel, not a
// memset, so that the call may also sit inside a stream capture).
int decode_zero_counters(nosa_ctx* ctx, void* ws) {
  hipLaunchKernelGGL(zero_counters_kernel, dim3((ctx->units + 255) / 256), dim3(256), 0, ctx->main, (int32_t*)ws, ctx->units);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

static bool vector_kernel_has_group(int g) {
  return g == 1 || g == 2 || g == 3 || g == 4 || g == 6 || g == 8 || g == 12 || g == 16;
}

// bf16: any group of 1..16 heads (matrix-core kernel); fp32: the groups the vector kernel is instantiated for
bool decode_supports_group(int g, int dtype) {
  return dtype == NOSA_DTYPE_BF16 ? (g >= 1 && g <= kHeadTile) : vector_kernel_has_group(g);
}

int decode_default_splits(const nosa_params& p) {
  const int units = p.batch * p.n_kv_heads;
  const int row_bytes = p.head_dim * (p.dtype == NOSA_DTYPE_F32 ? 4 : 2);
  const int tile_tokens = kRPW * (kLoads / (row_bytes / 128));
  const int tiles = p.k_blocks * (kBlockTokens / tile_tokens);
  // 512 workgroups (two per CU) keep HBM busy.  What a split count is worth: how full the rounds of 512 are,
  // less a charge per extra partial result to merge and per extra round.  Fitted to measurements at the 3B
  // shape (HIP events, us): 96 units 5 splits 41 (4: 46, 6: 52); 128 units 4: 49 (2: 51, 3: 57, 8: 58);
  // 160 units 3: 61 (2: 77, 4: 78); 320 units 3: 118 (1: 138, 2: 139); 400 units 1: 146 (2: 156, 3: 157).
  const int cap0 = tiles / kWaves > 1 ? tiles / kWaves : 1;   // at least one tile per wave
  const int cap = cap0 < NOSA_MAX_SPLITS ? cap0 : NOSA_MAX_SPLITS;
  if (units > 512) return 1;
  if (units * cap <= 512) return cap;     // few units: as many workgroups as the tiles allow
  int best = 1;
  double best_score = -1e9;
  for (int s = 1; s <= cap; ++s) {
    const int wgs = units * s, rounds = (wgs + 511) / 512;
    const double score = (double)wgs / (512.0 * rounds) - 0.03 * (s - 1) - 0.05 * (rounds - 1);
    if (score > best_score + 1e-9) {
      best_score = score;
      best = s;
    }
  }
  return best;
}

namespace {

template <int DT, bool OVERLAP>
bool dispatch_dim(int D, int G, const DecodeArgs& a, dim3 grid, hipStream_t s) {
  return D == 128 ? dispatch_group<DT, 128, OVERLAP>(G, a, grid, s) : dispatch_group<DT, 64, OVERLAP>(G, a, grid, s);
}

// Which kernel attends: the matrix-core one for bf16 unless the context asks for the vector kernel
// (attention_kernel 1); the vector kernel for fp32.
bool decode_uses_matrix_cores(const nosa_ctx* ctx) {
  if (ctx->p.dtype != NOSA_DTYPE_BF16) return false;
  return ctx->attention_kernel != 1 || !vector_kernel_has_group(ctx->group);   // odd groups exist on the matrix cores only
}

template <bool OVERLAP>
bool dispatch(const nosa_ctx* ctx, int G, const DecodeArgs& a, dim3 grid, hipStream_t s) {
  const nosa_params& p = ctx->p;
  if (decode_uses_matrix_cores(ctx))
    return p.head_dim == 128 ? dispatch_mfma<128, OVERLAP>(G, a, grid, s) : dispatch_mfma<64, OVERLAP>(G, a, grid, s);
  return p.dtype == NOSA_DTYPE_BF16 ? dispatch_dim<NOSA_DTYPE_BF16, OVERLAP>(p.head_dim, G, a, grid, s)
                                    : dispatch_dim<NOSA_DTYPE_F32, OVERLAP>(p.head_dim, G, a, grid, s);
}

}  // namespace

// Attention over the selected blocks.  When `wait_fetch` names an event, the blocks that were
// already resident are processed first (they do not depend on the gather in flight), then the
// stream waits for the gather and a second launch processes the fetched blocks and merges both.
int launch_decode(nosa_ctx* ctx, const void* q, const void* pool_k, const void* pool_v, const float* pool_bias,
                  const int32_t* sel_idx, const int32_t* n_sel, const int32_t* slot_of_block,
                  const int32_t* n_tokens, void* out, float* lse, hipEvent_t wait_fetch,
                  const int32_t* load_list, const int32_t* n_load, void* ws, size_t counter_bytes) {
  const nosa_params& p = ctx->p;
  const int G = ctx->group, D = p.head_dim, S = ctx->splits;
  DecodeArgs a;
  a.q = q; a.pool_k = pool_k; a.pool_v = pool_v; a.pool_bias = pool_bias;
  a.sel_idx = sel_idx; a.n_sel = n_sel; a.slot_of_block = slot_of_block; a.n_tokens = n_tokens;
  // scratch (the caller's workspace or the static array): [arrival counters][partial O][partial (m, l)]
  a.arrived = ctx->merge_in_kernel ? (int32_t*)ws : nullptr;
  a.part_o = ws ? (float*)((char*)ws + counter_bytes) : nullptr;
  a.part_ml = a.part_o ? a.part_o + (size_t)ctx->units * S * G * D : nullptr;
  a.trace = (ctx->trace && ctx->trace_capacity >= S * ctx->units) ? ctx->trace : nullptr;
  a.out = out; a.lse = lse;
  a.load_list = load_list; a.n_load = n_load;
  a.n_kv_heads = p.n_kv_heads; a.group = G; a.gpu_slots = p.gpu_slots; a.k_blocks = p.k_blocks; a.max_blocks = p.max_blocks;
  a.splits = S;
  a.phase = 0;
  a.merge_splits = 0;
  a.scale_log2e = ctx->scale * 1.4426950408889634f;
  if (wait_fetch && load_list && n_load && a.part_o) {
    a.phase = 1;
    {
      TimedLaunch tl(ctx, NOSA_KERNEL_DECODE, ctx->main);
      NOSA_REQUIRE(ctx, dispatch<true>(ctx, G, a, dim3(S * ctx->units), ctx->main), NOSA_ESHAPE, "GQA group %d unsupported", G);
    }
    NOSA_HIP(ctx, hipGetLastError());
    NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, wait_fetch, 0));
    a.phase = 2;
    a.merge_splits = S;
    a.splits = 1;
    {
      TimedLaunch tl(ctx, NOSA_KERNEL_COMBINE, ctx->main);
      NOSA_REQUIRE(ctx, dispatch<true>(ctx, G, a, dim3(ctx->units), ctx->main), NOSA_ESHAPE, "GQA group %d unsupported", G);
    }
    NOSA_HIP(ctx, hipGetLastError());
    return NOSA_OK;
  }
  if (wait_fetch) NOSA_HIP(ctx, hipStreamWaitEvent(ctx->main, wait_fetch, 0));
  {
    TimedLaunch tl(ctx, NOSA_KERNEL_DECODE, ctx->main);
    NOSA_REQUIRE(ctx, dispatch<false>(ctx, G, a, dim3(S * ctx->units), ctx->main), NOSA_ESHAPE, "GQA group %d unsupported", G);
  }
  NOSA_HIP(ctx, hipGetLastError());
  if (S > 1 && !a.arrived) {
    TimedLaunch tl(ctx, NOSA_KERNEL_COMBINE, ctx->main);
    if (p.dtype == NOSA_DTYPE_BF16)
      hipLaunchKernelGGL((decode_combine_kernel<NOSA_DTYPE_BF16>), dim3(ctx->units), dim3(kThreads), 0, ctx->main,
                         a.part_o, a.part_ml, out, lse, p.n_kv_heads, G, D, S);
    else
      hipLaunchKernelGGL((decode_combine_kernel<NOSA_DTYPE_F32>), dim3(ctx->units), dim3(kThreads), 0, ctx->main,
                         a.part_o, a.part_ml, out, lse, p.n_kv_heads, G, D, S);
    NOSA_HIP(ctx, hipGetLastError());
  }
  return NOSA_OK;
}

}  // namespace nosa
