// Sparse prefill (the variant that uses sparse attention in both stages; results Table, "Sparse
// Prefill" rows): every query position of a chunk runs the decode-step selection over its own
// causal prefix (selection Eq. of Sec. 3.1) and attends, with the eviction-head bias (Sec. 3.2),
// to the tokens of its selected blocks that are not in its future.
//
// Unlike the decode step this is a dense contraction per selected block (64 positions x G heads
// of queries against 64 keys), so it runs on the matrix cores: v_mfma_f32_32x32x16_bf16, fp32
// accumulation, flash-style online softmax.
//
// One workgroup = 64 consecutive query positions of one (batch element, KV head) and up to four
// query heads of its group; 8 waves, a wave = one query head x 32 positions (groups larger than
// four take several workgroups).  256 registers per lane, so a SIMD holds two waves.  Positions
// that are neighbours select mostly the same blocks, so the workgroup walks the UNION of their
// selections once; a 64-bit membership word per block (built with LDS atomics from sel_idx, then
// compacted into an ascending list by one wave) says which positions take part, the others get
// p = 0.  Per visited block:
//   S^T = K Q^T        A = K tile from LDS, B = Q^T held in registers for the whole kernel.
//                      In the C layout a lane owns ONE query (column) and 16 keys per 32x32 tile,
//                      so row max / row sum are in-lane plus one exchange with lane ^ 32.
//   O^T += V^T P^T     A = V^T from LDS, B = P^T built in registers from the S^T accumulators.
//                      The keys a lane holds in C order are not the ones the B operand wants in
//                      k order; since a sum over keys does not care about their order, V^T is
//                      stored with the matching key permutation (bits 2 and 3 of the key index
//                      swapped) and no cross-lane traffic is needed.
// V arrives from HBM as [key][d]; it is transposed on its way into LDS (two keys packed per
// 32-bit store).  Both LDS tiles are XOR-swizzled in 16-byte chunks so that the 16-byte operand
// reads of neighbouring lanes fall into different bank groups.  Two tile buffers: the next block's
// rows are fetched into registers while the current block is being multiplied (one barrier per block).
//
// Workgroups are numbered so that the ones that run together on one XCD (32 CUs) are
// neighbouring query tiles of the same (batch element, KV head): they share most of their
// blocks (the query-agnostic picks and overlapping windows), which then come from that XCD's L2.
#include <cmath>
#include <type_traits>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
using dev::u32x4;

constexpr int kThreads = 512;     // attention kernel: 8 waves
constexpr int kQ = 64;            // query positions per workgroup
constexpr int kHeadsPerWg = 4;    // two waves each (32 positions per wave)
constexpr int kXcds = 8;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kMaxLds = 160 * 1024;   // LDS of one CU

struct PrefillArgs {
  const void* q;             // [B, Lq, Hq, d]
  const void* cache_k;       // [B, Hkv, max_blocks, 64, d]
  const void* cache_v;
  const float* cache_bias;   // [B, Hkv, max_blocks, 64]
  const int32_t* sel_idx;    // [B, Lq, Hkv, K]
  const int32_t* n_sel;      // [B, Lq, Hkv]
  void* out;                 // [B, Lq, Hq, d]
  float* lse;                // [B, Lq, Hq]
  int n_kv_heads, group, n_q_heads, max_blocks, k_blocks, p0, lq;
  int units, n_qt, n_hz, list_cap;   // B*Hkv, query tiles per unit, head quads per KV head, LDS list capacity
  float scale;
};

__global__ void prefill_positions_kernel(int32_t* n_tok, int p0, int lq, int total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) n_tok[i] = p0 + i % lq + 1;   // position t of a chunk sees p0 + t + 1 tokens
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // round to nearest even (v_cvt_pk_bf16_f32)
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Lanes i and i + 32 hold the two halves of one query's keys: v_permlane32_swap exchanges the upper half
// of one operand with the lower half of the other (no LDS round trip as with a shuffle).
__device__ __forceinline__ float pair_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void prefill_attend_kernel(const PrefillArgs a) {
  constexpr int CH = D / 8;     // 16-byte chunks per key row
  constexpr int KC = D / 16;    // k-steps of the score product
  constexpr int RD = D / 32;    // 32-row tiles of O^T
  constexpr int kRowK = D * 2;  // bytes per row of the K tile
  constexpr int kRowV = 128;    // bytes per row of the V^T tile (64 keys)
  constexpr int kTile = 64 * kRowK + D * kRowV + 64 * 4;   // K tile, V^T tile, bias: one buffer
  constexpr int KR = kBlockTokens * CH / kThreads;                 // 16-byte K loads per thread and tile (2 or 1)
  constexpr int kPairs = (kBlockTokens / 2) * CH;                  // (key pair, chunk) tasks of the V tile: 512 or 256
  // 16-byte chunk c of key row `key` sits at chunk c ^ kswz(key): the rows that one operand read touches
  // (16 neighbouring keys at a time) then fall into 16 different 16-byte bank groups (256 bytes per clock)
  auto kswz = [](int key) { return D == 128 ? (key & 15) : ((key >> 1) & 7); };
  extern __shared__ __align__(16) unsigned char smem[];
  // two tile buffers, then the lists
  int* n_list_s = (int*)(smem + 2 * kTile);                       // [4] (one used)
  unsigned long long* memb = (unsigned long long*)(n_list_s + 4); // [list_cap] bit t: position t selected the block
  unsigned long long* list_m = memb + a.list_cap;                 // [list_cap] membership words of the visited blocks
  int* list_j = (int*)(list_m + a.list_cap);                      // [list_cap] visited blocks, ascending

  // workgroup -> (unit, query tile, head quad): id % 8 is the XCD the hardware dispatches to
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int hz = slot % a.n_hz, qt = (slot / a.n_hz) % a.n_qt;
  const int unit = xcd + kXcds * (slot / (a.n_hz * a.n_qt));   // b * Hkv + h
  if (unit >= a.units) return;                                 // before any barrier
  const int b = unit / a.n_kv_heads, h = unit % a.n_kv_heads;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int g = hz * kHeadsPerWg + (wave & 3);
  const int ct = wave >> 2;             // which half of the 64 positions
  const bool active = g < a.group;      // wave-uniform
  const int hq = h * a.group + (active ? g : 0);
  const int l32 = lane % 32, hb = lane / 32;
  const int t0 = qt * kQ;                              // first chunk position of this tile
  const int tq = ct * 32 + l32;                        // this lane's position in the tile = its row in the diagonal block
  const int diag = (a.p0 + t0) / kBlockTokens;         // the block these positions live in
  const int nblk = diag + 1;
  const float scale2 = a.scale * kLog2e;      // logits are kept unscaled; 2^(scale2 * x) = e^(scale * x)
  const float inv_scale = 1.f / a.scale;

  for (int J = tid; J < nblk; J += kThreads) memb[J] = 0ull;
  __syncthreads();
  {
    const int K = a.k_blocks;
    for (int idx = tid; idx < kQ * K; idx += kThreads) {
      const int t = idx / K, k = idx - t * K;
      const size_t vu = ((size_t)b * a.lq + t0 + t) * a.n_kv_heads + h;
      if (k < a.n_sel[vu]) {
        const int J = a.sel_idx[vu * K + k];
        if (J >= 0 && J < nblk) atomicOr(&memb[J], 1ull << t);
      }
    }
  }

  // Q^T operand, resident for the whole kernel: lane = (query l32 of this wave's half, k half hb)
  bf16x8 qreg[KC];
  {
    const size_t row = ((size_t)b * a.lq + t0 + tq) * a.n_q_heads + hq;
    const u32x4* qp = (const u32x4*)((const char*)a.q + row * (size_t)(D * 2));
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qreg[kc] = __builtin_bit_cast(bf16x8, qp[2 * kc + hb]);
  }
  __syncthreads();
  if (wave == 0) {   // the visited blocks, ascending
    int n = 0;
    for (int base = 0; base < nblk; base += kWave) {
      const int J = base + lane;
      const unsigned long long m = J < nblk ? memb[J] : 0ull;
      const uint64_t bal = __ballot(m != 0ull);
      if (m != 0ull) {
        const int pos = n + (int)__popcll(bal & ((1ull << lane) - 1ull));
        list_j[pos] = J;
        list_m[pos] = m;
      }
      n += (int)__popcll(bal);
    }
    if (lane == 0) n_list_s[0] = n;
  }
  __syncthreads();
  const int n_list = n_list_s[0];

  f32x16 o[RD];
#pragma unroll
  for (int rd = 0; rd < RD; ++rd)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[rd][i] = 0.f;
  float m_run = -INFINITY;   // running max of the unscaled logits q.k + bias / scale
  float l_run = 0.f;         // this lane's share of the running sum

  const size_t unit_blk = (size_t)unit * a.max_blocks;
  // two tiles travel from global memory through registers at any time (tile j uses set j & 1)
  struct Pre { u32x4 k[KR], v0, v1; float b; } pre[2];
  pre[0].b = pre[1].b = 0.f;
  auto fetch_tile = [&](int J, Pre& R) {   // global -> registers
    const size_t blk = unit_blk + J;
    const char* kg = (const char*)a.cache_k + blk * (size_t)(kBlockTokens * kRowK);
    const char* vg = (const char*)a.cache_v + blk * (size_t)(kBlockTokens * kRowK);
#pragma unroll
    for (int r = 0; r < KR; ++r) R.k[r] = *(const u32x4*)(kg + (size_t)(tid + r * kThreads) * 16);
    if (tid < kPairs) {
      const int key = 2 * (tid / CH), e = tid % CH;
      R.v0 = *(const u32x4*)(vg + ((size_t)key * CH + e) * 16);
      R.v1 = *(const u32x4*)(vg + ((size_t)(key + 1) * CH + e) * 16);
    }
    if (tid < kBlockTokens) R.b = a.cache_bias[blk * kBlockTokens + tid];
  };
  auto stage_tile = [&](unsigned char* buf, const Pre& R) {   // registers -> LDS (K swizzled, V transposed and swizzled)
    unsigned char* Ks = buf;
    unsigned char* Vt = buf + 64 * kRowK;
    float* bias_s = (float*)(Vt + D * kRowV);   // [64] bias / scale
#pragma unroll
    for (int r = 0; r < KR; ++r) {
      const int i = tid + r * kThreads;
      const int key = i / CH, c = i % CH;
      *(u32x4*)(Ks + key * kRowK + ((c ^ kswz(key)) * 16)) = R.k[r];
    }
    if (tid < kPairs) {
      const int key = 2 * (tid / CH), e = tid % CH;
      const int pos = (key & ~0xC) | ((key & 8) >> 1) | ((key & 4) << 1);   // even; key + 1 sits at pos + 1
      const int chunk = (pos >> 3) ^ (e & 7);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t a0 = R.v0[w], a1 = R.v1[w];
        const int dd = 8 * e + 2 * w;
        *(uint32_t*)(Vt + dd * kRowV + ((chunk ^ (dd & 7)) * 16) + (pos & 7) * 2) = (a0 & 0xffffu) | (a1 << 16);
        *(uint32_t*)(Vt + (dd + 1) * kRowV + ((chunk ^ ((dd + 1) & 7)) * 16) + (pos & 7) * 2) =
            (a0 >> 16) | (a1 & 0xffff0000u);
      }
    }
    if (tid < kBlockTokens) bias_s[tid] = R.b * inv_scale;
  };

  // tile it is multiplied out of buffer it & 1 while tile it + 1 is written into the other buffer
  // and tiles it + 2, it + 3 travel from global memory into registers: one barrier per tile
  int J_next = 0;
  unsigned long long mb_next = 0ull;
  if (n_list > 0) {
    fetch_tile(list_j[0], pre[0]);
    stage_tile(smem, pre[0]);
    if (n_list > 1) fetch_tile(list_j[1], pre[1]);
    if (n_list > 2) fetch_tile(list_j[2], pre[0]);
    J_next = list_j[0];
    mb_next = list_m[0];
  }
  __syncthreads();
  // one visited block; PAR = it & 1 is a compile-time constant so that the buffer offsets fold into the
  // LDS instructions' immediate fields (the loop below is unrolled by two)
  auto pass = [&](int it, auto par) {
    constexpr int PAR = decltype(par)::value;
    const int J = J_next;                      // read one pass ahead: no LDS round trip at the top of a pass
    const unsigned long long mb = mb_next;
    if (it + 1 < n_list) {
      J_next = list_j[it + 1];
      mb_next = list_m[it + 1];
    }
    const unsigned char* Ks = smem + PAR * kTile;
    const unsigned char* Vt = Ks + 64 * kRowK;
    const float* bias_s = (const float*)(Vt + D * kRowV);

    // a wave whose 32 positions all left this block out only helps with the staging
    const bool busy = active && ((mb >> (ct * 32)) & 0xffffffffull) != 0ull;
    f32x16 s[2];   // two tiles of 32 keys
    if (busy) {
      // accumulator i of key tile rk is key rk*32 + 8*(i/4) + 4*hb + i%4; it starts at that key's
      // bias / scale, so that scale * S is the biased logit without a separate addition
#pragma unroll
      for (int rk = 0; rk < 2; ++rk)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const float4 bz = *(const float4*)(bias_s + rk * 32 + 8 * i4 + 4 * hb);
          s[rk][4 * i4 + 0] = bz.x;
          s[rk][4 * i4 + 1] = bz.y;
          s[rk][4 * i4 + 2] = bz.z;
          s[rk][4 * i4 + 3] = bz.w;
        }
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
#pragma unroll
        for (int rk = 0; rk < 2; ++rk) {
          const int key = rk * 32 + l32;
          const bf16x8 ak = *(const bf16x8*)(Ks + key * kRowK + (((2 * kc + hb) ^ kswz(key)) * 16));
          s[rk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qreg[kc], s[rk], 0, 0, 0);
        }
      }
    }

    if (it + 1 < n_list) {
      stage_tile(smem + (PAR ^ 1) * kTile, pre[PAR ^ 1]);
      if (it + 3 < n_list) fetch_tile(list_j[it + 3], pre[PAR ^ 1]);
    }

    if (busy) {
      if (J == diag) {   // the future
#pragma unroll
        for (int rk = 0; rk < 2; ++rk)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (rk * 32 + 8 * (i / 4) + 4 * hb + (i % 4) > tq) s[rk][i] = -INFINITY;
      }
      const bool member = (mb >> tq) & 1ull;
      float mx = -INFINITY;
#pragma unroll
      for (int rk = 0; rk < 2; ++rk)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[rk][i]);
      if (!member) mx = -INFINITY;
      mx = pair_max(mx);
      const bool raise = mx > m_run;
      if (__any(raise)) {
        const float alpha = (raise && m_run != -INFINITY) ? __builtin_amdgcn_exp2f((m_run - mx) * scale2) : 1.f;
        if (raise) m_run = mx;
        l_run *= alpha;
#pragma unroll
        for (int rd = 0; rd < RD; ++rd)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[rd][i] *= alpha;
      }
      // p = 2^(scale2 * (S - m)); positions outside the block's membership, and ones that have seen
      // nothing yet, add zeros
      const float off = (member && m_run != -INFINITY) ? -m_run * scale2 : -INFINITY;
      float psum = 0.f;
      uint32_t packed[16];
#pragma unroll
      for (int rk = 0; rk < 2; ++rk) {
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[rk][i], scale2, off));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[rk][i + 1], scale2, off));
          psum += p0 + p1;
          packed[rk * 8 + i / 2] = pack_bf16(p0, p1);
        }
      }
      l_run += psum;
#pragma unroll
      for (int kc = 0; kc < 4; ++kc) {
        const u32x4 w = {packed[4 * kc], packed[4 * kc + 1], packed[4 * kc + 2], packed[4 * kc + 3]};
        const bf16x8 pb = __builtin_bit_cast(bf16x8, w);
#pragma unroll
        for (int rd = 0; rd < RD; ++rd) {
          const int dd = rd * 32 + l32;
          const bf16x8 av =
              *(const bf16x8*)(Vt + dd * kRowV + ((((2 * kc + hb) ^ ((dd >> 3) & 7)) ^ (dd & 7)) * 16));
          o[rd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb, o[rd], 0, 0, 0);
        }
      }
    }
    __syncthreads();   // tile it has been consumed, tile it + 1 is in place
  };
  for (int it = 0; it < n_list; it += 2) {
    pass(it, std::integral_constant<int, 0>{});
    if (it + 1 < n_list) pass(it + 1, std::integral_constant<int, 1>{});
  }

  if (active) {
    float l = l_run;
    l = pair_sum(l);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const size_t row = ((size_t)b * a.lq + t0 + tq) * a.n_q_heads + hq;
    char* op = (char*)a.out + row * (size_t)(D * 2);
#pragma unroll
    for (int rd = 0; rd < RD; ++rd) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int dd = rd * 32 + 8 * i4 + 4 * hb;   // accumulators 4*i4 .. 4*i4+3 are dd .. dd+3
        uint2 w;
        w.x = pack_bf16(o[rd][4 * i4] * inv, o[rd][4 * i4 + 1] * inv);
        w.y = pack_bf16(o[rd][4 * i4 + 2] * inv, o[rd][4 * i4 + 3] * inv);
        *(uint2*)(op + dd * 2) = w;
      }
    }
    if (hb == 0) a.lse[row] = l > 0.f ? m_run * a.scale + logf(l) : -INFINITY;
  }
}

// Block scores of a whole chunk as one matrix product per (batch element, KV head), for one pooled
// key per block (Alg. 1 Stage 1 with pool kernel = stride = block size): sq[t, J] = sum over the G
// query heads of q_{t,g} . kc_J.  The group sum is folded into the contraction (k runs over g and
// d), so every product is an exact bf16 x bf16 product accumulated in fp32, as in the decode path.
// A = Q rows from LDS (staged once per workgroup), B = pooled keys straight from global memory: both
// have the contraction index contiguous, nothing is transposed.  A workgroup = 32 positions x up to
// 512 blocks (one wave per 128); only the entries the selection reads (complete blocks of the
// position's prefix) are computed and written.
struct PrefillScoreArgs {
  const void* q;          // [B, Lq, Hq, d]
  const void* k_pooled;   // [B, Hkv, n_sub_max, d]
  float* sq;              // [B, Lq, Hkv, max_blocks]
  int n_kv_heads, group, n_q_heads, max_blocks, n_sub_max, p0, lq;
};

constexpr int kScoreThreads = 256;

template <int D>
__global__ __launch_bounds__(kScoreThreads) void prefill_score_kernel(const PrefillScoreArgs a) {
  constexpr int CH = D / 8, KC = D / 16, kRow = D * 2;
  extern __shared__ __align__(16) unsigned char smem[];   // [G][32 positions][D] swizzled
  const int tt = blockIdx.x, unit = blockIdx.y;
  const int b = unit / a.n_kv_heads, h = unit % a.n_kv_heads;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int l32 = lane % 32, hb = lane / 32;
  const int t0 = tt * 32;
  const int n_hi = min((a.p0 + t0 + 32) / kBlockTokens, a.n_sub_max);   // complete blocks seen by the tile's last position
  if ((int)blockIdx.z * 512 >= n_hi) return;                            // whole workgroup: nothing to score

  const int rows = a.group * 32;
  for (int i = tid; i < rows * CH; i += kScoreThreads) {
    const int r = i / CH, c = i % CH;          // r = g * 32 + position
    const int g = r / 32, tl = r % 32;
    const size_t row = ((size_t)b * a.lq + t0 + tl) * a.n_q_heads + h * a.group + g;
    *(u32x4*)(smem + r * kRow + ((c ^ (r & 7)) * 16)) = *(const u32x4*)((const char*)a.q + row * (size_t)kRow + c * 16);
  }
  __syncthreads();

  const int J0 = (blockIdx.z * 4 + wave) * 128;
  if (J0 >= n_hi) return;                      // no barrier below
  const char* kc = (const char*)a.k_pooled + (size_t)unit * a.n_sub_max * kRow;
  f32x16 acc[4];
#pragma unroll
  for (int jt = 0; jt < 4; ++jt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[jt][i] = 0.f;
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    if (J0 + jt * 32 >= n_hi) break;           // wave-uniform
    const int J = J0 + jt * 32 + l32;
    bf16x8 kb[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (J < n_hi) v = *(const u32x4*)(kc + (size_t)J * kRow + (2 * k + hb) * 16);
      kb[k] = __builtin_bit_cast(bf16x8, v);
    }
    for (int g = 0; g < a.group; ++g) {
      const int r = g * 32 + l32;
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const bf16x8 qa = *(const bf16x8*)(smem + r * kRow + (((2 * k + hb) ^ (r & 7)) * 16));
        acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kb[k], acc[jt], 0, 0, 0);
      }
    }
  }
  // accumulator i: position 8*(i/4) + 4*hb + i%4 of the tile, block = this lane's column
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    const int J = J0 + jt * 32 + l32;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int tl = 8 * (i / 4) + 4 * hb + (i % 4);
      const int nsub = min((a.p0 + t0 + tl + 1) / kBlockTokens, a.n_sub_max);
      if (J < nsub)
        a.sq[(((size_t)b * a.lq + t0 + tl) * a.n_kv_heads + h) * a.max_blocks + J] = acc[jt][i];
    }
  }
}

}  // namespace

int launch_prefill_positions(nosa_ctx* ctx, int32_t* n_tok_virtual, int p0, int lq) {
  const int total = ctx->p.batch * lq;
  hipLaunchKernelGGL(prefill_positions_kernel, dim3((total + 255) / 256), dim3(256), 0, ctx->main, n_tok_virtual, p0,
                     lq, total);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

int launch_prefill_score(nosa_ctx* ctx, const void* q_chunk, const void* k_pooled, float* sq, int p0, int lq) {
  const nosa_params& p = ctx->p;
  PrefillScoreArgs a{q_chunk, k_pooled, sq, p.n_kv_heads, ctx->group, p.n_q_heads, p.max_blocks, p.n_sub_max, p0, lq};
  const int n_hi = (p0 + lq) / kBlockTokens;
  const dim3 grid(lq / 32, ctx->units, (n_hi + 511) / 512);
  const size_t smem = (size_t)ctx->group * 32 * p.head_dim * 2;
  NOSA_REQUIRE(ctx, smem <= (size_t)kMaxLds, NOSA_ESHAPE, "prefill: %d query heads per KV head need %zu bytes of LDS (limit 163840)",
               ctx->group, smem);
  if (smem > 64 * 1024 && !ctx->prefill_score_lds_set) {   // once per context: raise the kernel's LDS limit to the CU's
    if (p.head_dim == 128)
      NOSA_HIP(ctx, hipFuncSetAttribute((const void*)prefill_score_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds));
    else
      NOSA_HIP(ctx, hipFuncSetAttribute((const void*)prefill_score_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds));
    ctx->prefill_score_lds_set = true;
  }
  NOSA_REQUIRE(ctx, ctx->units <= 65535 && grid.z <= 65535, NOSA_ESHAPE, "prefill: B * Hkv = %d exceeds 65535", ctx->units);
  TimedLaunch tl(ctx, NOSA_KERNEL_SCORE, ctx->main);
  if (p.head_dim == 128) hipLaunchKernelGGL(prefill_score_kernel<128>, grid, dim3(kScoreThreads), smem, ctx->main, a);
  else hipLaunchKernelGGL(prefill_score_kernel<64>, grid, dim3(kScoreThreads), smem, ctx->main, a);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

int launch_prefill_attend(nosa_ctx* ctx, const void* q_chunk, const void* cache_k, const void* cache_v,
                          const float* cache_bias, const int32_t* sel_idx, const int32_t* n_sel, int p0, int lq,
                          void* out, float* lse) {
  const nosa_params& p = ctx->p;
  const int n_qt = lq / kQ, n_hz = (ctx->group + kHeadsPerWg - 1) / kHeadsPerWg;
  const int list_cap = (p0 + lq) / kBlockTokens;
  PrefillArgs a{q_chunk, cache_k, cache_v, cache_bias, sel_idx, n_sel, out, lse, p.n_kv_heads, ctx->group,
                p.n_q_heads, p.max_blocks, p.k_blocks, p0, lq, ctx->units, n_qt, n_hz, list_cap, ctx->scale};
  const size_t tile = (size_t)kBlockTokens * p.head_dim * 2 + (size_t)p.head_dim * 128 + 64 * sizeof(float);
  const size_t smem = 2 * tile + 16 + (size_t)list_cap * 20;
  NOSA_REQUIRE(ctx, smem <= (size_t)kMaxLds, NOSA_ESHAPE, "prefill: %d blocks of context need %zu bytes of LDS (limit 163840)",
               list_cap, smem);
  if (smem > 64 * 1024 && !ctx->prefill_attend_lds_set) {
    if (p.head_dim == 128)
      NOSA_HIP(ctx, hipFuncSetAttribute((const void*)prefill_attend_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds));
    else
      NOSA_HIP(ctx, hipFuncSetAttribute((const void*)prefill_attend_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds));
    ctx->prefill_attend_lds_set = true;
  }
  const long long wgs = (long long)kXcds * ((ctx->units + kXcds - 1) / kXcds) * n_qt * n_hz;
  NOSA_REQUIRE(ctx, wgs <= 0x7fffffffLL, NOSA_ESHAPE, "prefill: too many workgroups (%lld)", wgs);
  const dim3 grid((unsigned)wgs);
  TimedLaunch tl(ctx, NOSA_KERNEL_PREFILL, ctx->main);
  if (p.head_dim == 128) hipLaunchKernelGGL(prefill_attend_kernel<128>, grid, dim3(kThreads), smem, ctx->main, a);
  else hipLaunchKernelGGL(prefill_attend_kernel<64>, grid, dim3(kThreads), smem, ctx->main, a);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
