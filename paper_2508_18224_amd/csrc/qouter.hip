// Forward selected-block attention in QUERY-OUTER loop order: the order of the original NSA kernel that the paper
// argues against (Sec. 2.2 / 3.1; App. C gives its traffic, a K/V block re-loaded for every (token, KV head,
// selected block)).  Kept as the dispatch target the paper's fallback asks for (App. E: with many query heads per
// group the orders converge) and as the in-library comparison that shows what the KV-outer order buys on this chip.
//
// One wavefront owns one (token, KV head): its g query rows are the valid columns of a 32-column MFMA operand
// (32 / g of the matrix work is padding: the cost of this order for small g), and it walks the row's kept blocks
// with an online softmax: K_i fragments straight from memory into registers, V_i row-major into a wave-private LDS
// tile read back with transposing reads, S^T = K_i Q^T, running (max, sum) per row, O^T += V_i^T P^T.  No partial
// buffers and no merge pass; every block costs 32 KB of loads for g rows of work.  64-token blocks, no window.
#include "common.h"

namespace nsa {

constexpr int kQoPitch = 152;   // bf16 per LDS row of the V tile (128 + 24 pad), as in the 128-key forward kernel
constexpr int kQoWaves = 4;

__device__ __forceinline__ bf16x4 lds_read_tr_q(const bf16_t* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)(uint32_t)(uintptr_t)p);
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ void wave_sync_q() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ void __launch_bounds__(64 * kQoWaves, 2)
k_fwd_query_outer(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                  const int32_t* __restrict__ idx, const int32_t* __restrict__ cu, bf16_t* __restrict__ O,
                  float* __restrict__ LSE) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_q[];   // kQoWaves V tiles
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t pair = (int64_t)blockIdx.x * kQoWaves + wave;
  if (pair >= (int64_t)P.T * P.hkv) return;   // the whole wavefront leaves; no block-wide barrier is used below
  const int t = (int)(pair / P.hkv), j = (int)(pair - (int64_t)t * P.hkv);
  const int col = lane & 31, qh = lane >> 5;
  bf16_t* Vs = reinterpret_cast<bf16_t*>(smem_q) + wave * (kBlock * kQoPitch);
  int s, c0, c1;
  seq_bounds(cu, P.nseq, P.T, t, s, c0, c1);
  const int cur = (t - c0) / kBlock, b_s = (c1 - c0 + kBlock - 1) / kBlock;

  // kept columns of the row: in range, not in the future when causal, first occurrence only (lane m holds column m)
  const int my = lane < P.topk ? idx[((size_t)t * P.hkv + j) * P.topk + lane] : -1;
  const bool ok = lane < P.topk && my >= 0 && my < b_s && (!P.causal || my <= cur);
  uint64_t okm = __builtin_amdgcn_ballot_w64(ok);
  uint64_t keep = 0;
  for (int m = 0; m < P.topk; ++m) {
    if (!((okm >> m) & 1)) continue;
    const int x = __builtin_amdgcn_readlane(my, m);
    const uint64_t same = __builtin_amdgcn_ballot_w64(ok && my == x) & ((1ull << m) - 1ull);
    if (same == 0) keep |= 1ull << m;
  }

  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  bf16x8 qf[8];   // B operand of S^T: column `col` = query head j g + col, zero past the group
  {
    const bf16_t* src = Q + ((size_t)t * P.hq + j * P.g + col) * kD + 8 * qh;
#pragma unroll
    for (int s2 = 0; s2 < 8; ++s2) qf[s2] = col < P.g ? *reinterpret_cast<const bf16x8*>(src + 16 * s2) : zero8;
  }
  const float c2 = P.scale * 1.4426950408889634f;
  const int grp = lane >> 4, sl = lane & 15;
  const int tr_v = ((sl >> 2) + 4 * (grp >> 1)) * kQoPitch + 16 * (grp & 1) + 4 * (sl & 3);

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;   // per row (= per column `col`), in the raw-score domain

  for (int m = 0; m < P.topk; ++m) {
    if (!((keep >> m) & 1)) continue;      // wave-uniform
    const int x = __builtin_amdgcn_readlane(my, m);
    const int tok0 = c0 + x * kBlock;
    const int blen = min(kBlock, c1 - tok0);
    bf16x8 kf[2][8];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const int key = 32 * mb + col;
      const bf16_t* src = K + ((size_t)(tok0 + key) * P.hkv + j) * kD + 8 * qh;
#pragma unroll
      for (int s2 = 0; s2 < 8; ++s2) kf[mb][s2] = key < blen ? *reinterpret_cast<const bf16x8*>(src + 16 * s2) : zero8;
    }
    {  // V_i -> this wave's LDS tile, row-major: lane = key
      const bf16_t* src = V + ((size_t)(tok0 + lane) * P.hkv + j) * kD;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        *reinterpret_cast<bf16x8*>(&Vs[lane * kQoPitch + 8 * i]) =
            lane < blen ? *reinterpret_cast<const bf16x8*>(src + 8 * i) : zero8;
    }
    wave_sync_q();

    f32x16 sacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[mb][v] = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < 8; ++s2)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][s2], qf[s2], sacc[mb], 0, 0, 0);

    const int lim = P.causal ? min(blen, t - tok0 + 1) : blen;   // >= 1: the block was kept
    float mb_max = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
        const float xv = key < lim ? sacc[mb][v] : -INFINITY;
        sacc[mb][v] = xv;
        mb_max = fmaxf(mb_max, xv);
      }
    mb_max = fmaxf(mb_max, __shfl_xor(mb_max, 32));
    const float m_new = fmaxf(m_run, mb_max);                    // finite: at least one key is visible
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);   // 0 on the first block (m_run = -inf)
    float lsum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f((sacc[mb][v] - m_new) * c2);
        lsum += p;
        pf[2 * mb + (v >> 3)][v & 7] = (bf16_t)p;
      }
    lsum += __shfl_xor(lsum, 32);
    l_run = l_run * alpha + lsum;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
#pragma unroll
    for (int sp = 0; sp < 4; ++sp) {
      const int k0 = 32 * (sp >> 1) + 16 * (sp & 1);
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x4 a0 = lds_read_tr_q(&Vs[k0 * kQoPitch + tr_v + 32 * db]);
        const bf16x4 a1 = lds_read_tr_q(&Vs[(k0 + 8) * kQoPitch + tr_v + 32 * db]);
        const bf16x8 vf = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], oacc[db], 0, 0, 0);
      }
    }
    wave_sync_q();   // the tile is overwritten by the next block
  }

  if (col < P.g) {
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;   // no kept block: O = 0, LSE = -inf
    bf16_t* dst = O + ((size_t)t * P.hq + j * P.g + col) * kD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w;
        w.x = pack_bf16x2(oacc[db][4 * a + 0] * inv, oacc[db][4 * a + 1] * inv);
        w.y = pack_bf16x2(oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv);
        *reinterpret_cast<uint2*>(dst + 32 * db + 8 * a + 4 * qh) = w;
      }
    if (qh == 0)
      LSE[(size_t)t * P.hq + j * P.g + col] =
          l_run > 0.f ? (m_run * c2 + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
  }
}

hipError_t launch_fwd_query_outer(const Problem& P, const void* Q, const void* K, const void* V, const int32_t* idx,
                                  const int32_t* cu, void* O, float* LSE, hipStream_t st) {
  const int64_t pairs = (int64_t)P.T * P.hkv;
  constexpr int kLds = kQoWaves * kBlock * kQoPitch * 2;   // 76 KB: two workgroups per CU
  static std::atomic<uint64_t> ready;
  hipError_t e = allow_dynamic_lds((const void*)k_fwd_query_outer, kLds, ready);
  if (e != hipSuccess) return e;
  ProfScope ps(KID_FWD_QUERY_OUTER, st);
  hipLaunchKernelGGL(k_fwd_query_outer, dim3((unsigned)((pairs + kQoWaves - 1) / kQoWaves)), dim3(64 * kQoWaves), kLds, st, P,
                     (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, idx, cu, (bf16_t*)O, LSE);
  return hipGetLastError();
}

}  // namespace nsa
