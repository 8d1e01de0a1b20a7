// Sparse prefill (the variant that uses sparse attention in both stages; results Table, "Sparse
// Prefill" rows): every query position of a chunk runs the decode-step selection over its own
// causal prefix (selection Eq. of Sec. 3.1) and attends, with the eviction-head bias (Sec. 3.2),
// to the tokens of its selected blocks that are not in its future.
//
// Unlike the decode step this is a dense contraction per selected block (64 positions x G heads
// of queries against 64 keys), so it runs on the matrix cores: v_mfma_f32_32x32x16_bf16, fp32
// accumulation, flash-style online softmax.
//
// One workgroup = 64 consecutive query positions of one (batch element, KV head), one wave = one
// query head.  Positions that are neighbours select mostly the same blocks, so the workgroup walks
// the UNION of their selections once; a 64-bit membership word per block says which positions
// take part.  Per visited block:
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
// reads of eight neighbouring lanes fall into different banks.
#include <cmath>

#include "nosa_device.h"
#include "nosa_internal.h"

namespace nosa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
using dev::u32x4;

constexpr int kThreads = 256;
constexpr int kQ = 64;            // query positions per workgroup
constexpr int kHeadsPerWg = 4;    // one wave each
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

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
  float scale;
};

__global__ void prefill_positions_kernel(int32_t* n_tok, int p0, int lq, int total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) n_tok[i] = p0 + i % lq + 1;   // position t of a chunk sees p0 + t + 1 tokens
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // round to nearest even; finite inputs
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7fffu + ((a >> 16) & 1u);
  b += 0x7fffu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xffff0000u);
}

template <int D>
__global__ __launch_bounds__(kThreads) void prefill_attend_kernel(const PrefillArgs a) {
  constexpr int CH = D / 8;     // 16-byte chunks per key row
  constexpr int KC = D / 16;    // k-steps of the score product
  constexpr int RD = D / 32;    // 32-row tiles of O^T
  constexpr int kRowK = D * 2;  // bytes per row of the K tile
  constexpr int kRowV = 128;    // bytes per row of the V^T tile (64 keys)
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Ks = smem;                                   // [64 keys][D] swizzled
  unsigned char* Vt = Ks + 64 * kRowK;                        // [D][64 key positions] swizzled
  float* bias_s = (float*)(Vt + D * kRowV);                   // [64], already times log2(e)
  unsigned long long* memb = (unsigned long long*)(bias_s + 64);   // [blocks up to the diagonal]

  const int qb = blockIdx.x;
  const int unit = blockIdx.y;   // b * Hkv + h
  const int b = unit / a.n_kv_heads, h = unit % a.n_kv_heads;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int g = blockIdx.z * kHeadsPerWg + wave;
  const bool active = g < a.group;      // wave-uniform
  const int hq = h * a.group + (active ? g : 0);
  const int l32 = lane % 32, hb = lane / 32;
  const int diag = a.p0 / kBlockTokens + qb;   // the block these 64 positions live in
  const int nblk = diag + 1;
  const float scale2 = a.scale * kLog2e;

  // membership words: bit t of memb[J] = position t of this workgroup selected block J
  for (int J = tid; J < nblk; J += kThreads) memb[J] = 0ull;
  __syncthreads();
  {
    const int K = a.k_blocks;
    for (int idx = tid; idx < kQ * K; idx += kThreads) {
      const int t = idx / K, k = idx - t * K;
      const size_t vu = ((size_t)b * a.lq + qb * kQ + t) * a.n_kv_heads + h;
      if (k < a.n_sel[vu]) {
        const int J = a.sel_idx[vu * K + k];
        if (J >= 0 && J < nblk) atomicOr(&memb[J], 1ull << t);
      }
    }
  }

  // Q^T operands, resident for the whole kernel: lane = (query l32 of column tile ct, k half hb)
  bf16x8 qreg[2][KC];
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) {
    const size_t row = ((size_t)b * a.lq + qb * kQ + ct * 32 + l32) * a.n_q_heads + hq;
    const u32x4* qp = (const u32x4*)((const char*)a.q + row * (size_t)(D * 2));
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qreg[ct][kc] = __builtin_bit_cast(bf16x8, qp[2 * kc + hb]);
  }

  f32x16 o[RD][2];
#pragma unroll
  for (int rd = 0; rd < RD; ++rd)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[rd][ct][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};   // running max, in log2 units
  float l_run[2] = {0.f, 0.f};               // this lane's share of the running sum
  __syncthreads();

  for (int J = 0; J < nblk; ++J) {
    const unsigned long long mb = memb[J];   // same word for every thread: uniform branch
    if (mb == 0ull) continue;
    __syncthreads();                         // the previous tile has been consumed

    const size_t blk = (size_t)unit * a.max_blocks + J;
    const char* kg = (const char*)a.cache_k + blk * (size_t)(kBlockTokens * kRowK);
    const char* vg = (const char*)a.cache_v + blk * (size_t)(kBlockTokens * kRowK);
    for (int i = tid; i < kBlockTokens * CH; i += kThreads) {
      const int key = i / CH, c = i % CH;
      const u32x4 v = *(const u32x4*)(kg + (size_t)i * 16);
      *(u32x4*)(Ks + key * kRowK + ((c ^ (key & 7)) * 16)) = v;
    }
    for (int i = tid; i < (kBlockTokens / 2) * CH; i += kThreads) {
      const int pr = i / CH, e = i % CH;
      const int key = 2 * pr;
      const u32x4 v0 = *(const u32x4*)(vg + ((size_t)key * CH + e) * 16);
      const u32x4 v1 = *(const u32x4*)(vg + ((size_t)(key + 1) * CH + e) * 16);
      const int pos = (key & ~0xC) | ((key & 8) >> 1) | ((key & 4) << 1);   // even; key + 1 sits at pos + 1
      const int chunk = (pos >> 3) ^ (e & 7);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t a0 = v0[w], a1 = v1[w];
        const int dd = 8 * e + 2 * w;
        *(uint32_t*)(Vt + dd * kRowV + ((chunk ^ (dd & 7)) * 16) + (pos & 7) * 2) = (a0 & 0xffffu) | (a1 << 16);
        *(uint32_t*)(Vt + (dd + 1) * kRowV + ((chunk ^ ((dd + 1) & 7)) * 16) + (pos & 7) * 2) =
            (a0 >> 16) | (a1 & 0xffff0000u);
      }
    }
    if (tid < kBlockTokens) bias_s[tid] = a.cache_bias[blk * kBlockTokens + tid] * kLog2e;
    __syncthreads();

    if (active) {
      f32x16 s[2][2];   // [key tile][query tile]
#pragma unroll
      for (int rk = 0; rk < 2; ++rk)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[rk][ct][i] = 0.f;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
#pragma unroll
        for (int rk = 0; rk < 2; ++rk) {
          const int key = rk * 32 + l32;
          const bf16x8 ak = *(const bf16x8*)(Ks + key * kRowK + (((2 * kc + hb) ^ (key & 7)) * 16));
          s[rk][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qreg[0][kc], s[rk][0], 0, 0, 0);
          s[rk][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qreg[1][kc], s[rk][1], 0, 0, 0);
        }
      }

      const bool is_diag = J == diag;
      bf16x8 pb[2][4];   // P^T operands [query tile][k-step of 16 keys]
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        const int t = ct * 32 + l32;
        const bool member = (mb >> t) & 1ull;
        float mx = -INFINITY;
#pragma unroll
        for (int rk = 0; rk < 2; ++rk) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int kidx = rk * 32 + 8 * (i / 4) + 4 * hb + (i % 4);   // key of accumulator i
            float z = fmaf(s[rk][ct][i], scale2, bias_s[kidx]);
            if (is_diag && kidx > t) z = -INFINITY;                     // the future
            s[rk][ct][i] = z;
            mx = fmaxf(mx, z);
          }
        }
        if (!member) mx = -INFINITY;
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run[ct], mx);
        // positions outside the block's membership, and ones that have seen nothing yet, add zeros
        const float sub = (member && m_new != -INFINITY) ? m_new : INFINITY;
        const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run[ct] - m_new);
        float psum = 0.f;
        uint32_t packed[16];
#pragma unroll
        for (int rk = 0; rk < 2; ++rk) {
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            const float p0 = __builtin_amdgcn_exp2f(s[rk][ct][i] - sub);
            const float p1 = __builtin_amdgcn_exp2f(s[rk][ct][i + 1] - sub);
            psum += p0 + p1;
            packed[rk * 8 + i / 2] = pack_bf16(p0, p1);
          }
        }
        l_run[ct] = l_run[ct] * alpha + psum;
        m_run[ct] = m_new;
#pragma unroll
        for (int rd = 0; rd < RD; ++rd)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[rd][ct][i] *= alpha;
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
          const u32x4 w = {packed[4 * kc], packed[4 * kc + 1], packed[4 * kc + 2], packed[4 * kc + 3]};
          pb[ct][kc] = __builtin_bit_cast(bf16x8, w);
        }
      }

#pragma unroll
      for (int kc = 0; kc < 4; ++kc) {
#pragma unroll
        for (int rd = 0; rd < RD; ++rd) {
          const int dd = rd * 32 + l32;
          const bf16x8 av =
              *(const bf16x8*)(Vt + dd * kRowV + ((((2 * kc + hb) ^ ((dd >> 3) & 7)) ^ (dd & 7)) * 16));
          o[rd][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[0][kc], o[rd][0], 0, 0, 0);
          o[rd][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[1][kc], o[rd][1], 0, 0, 0);
        }
      }
    }
  }

  if (active) {
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      float l = l_run[ct];
      l += __shfl_xor(l, 32);
      const float inv = l > 0.f ? 1.f / l : 0.f;
      const size_t row = ((size_t)b * a.lq + qb * kQ + ct * 32 + l32) * a.n_q_heads + hq;
      char* op = (char*)a.out + row * (size_t)(D * 2);
#pragma unroll
      for (int rd = 0; rd < RD; ++rd) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const int dd = rd * 32 + 8 * i4 + 4 * hb;   // accumulators 4*i4 .. 4*i4+3 are dd .. dd+3
          uint2 w;
          w.x = pack_bf16(o[rd][ct][4 * i4] * inv, o[rd][ct][4 * i4 + 1] * inv);
          w.y = pack_bf16(o[rd][ct][4 * i4 + 2] * inv, o[rd][ct][4 * i4 + 3] * inv);
          *(uint2*)(op + dd * 2) = w;
        }
      }
      if (hb == 0) a.lse[row] = l > 0.f ? m_run[ct] * kLn2 + logf(l) : -INFINITY;
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

int launch_prefill_attend(nosa_ctx* ctx, const void* q_chunk, const void* cache_k, const void* cache_v,
                          const float* cache_bias, const int32_t* sel_idx, const int32_t* n_sel, int p0, int lq,
                          void* out, float* lse) {
  const nosa_params& p = ctx->p;
  PrefillArgs a{q_chunk, cache_k, cache_v, cache_bias, sel_idx, n_sel, out, lse, p.n_kv_heads, ctx->group,
                p.n_q_heads, p.max_blocks, p.k_blocks, p0, lq, ctx->scale};
  const int nblk_max = (p0 + lq) / kBlockTokens;
  const size_t smem = (size_t)kBlockTokens * p.head_dim * 2 + (size_t)p.head_dim * 128 + 64 * sizeof(float) +
                      (size_t)nblk_max * sizeof(unsigned long long);
  NOSA_REQUIRE(ctx, smem <= 64 * 1024, NOSA_ESHAPE, "prefill: %d blocks of context need %zu bytes of LDS (limit 65536)",
               nblk_max, smem);
  const dim3 grid(lq / kQ, ctx->units, (ctx->group + kHeadsPerWg - 1) / kHeadsPerWg);
  TimedLaunch tl(ctx, NOSA_KERNEL_PREFILL, ctx->main);
  if (p.head_dim == 128) hipLaunchKernelGGL(prefill_attend_kernel<128>, grid, dim3(kThreads), smem, ctx->main, a);
  else hipLaunchKernelGGL(prefill_attend_kernel<64>, grid, dim3(kThreads), smem, ctx->main, a);
  NOSA_HIP(ctx, hipGetLastError());
  return NOSA_OK;
}

}  // namespace nosa
