// Forward selected-block attention for gfx950 (paper Sec. 3.2, the KV-outer "token selection" step and the
// reduction step; Eq. (2), c = sel).
//
// k_fwd_main: one work unit = (kv head j, KV block i, up to kFwdUnit entries of the block's query list).
//   The block's K_i and V_i stay in registers for the whole unit (K as the A operand of S^T = K_i Q^T, V^T as
//   the A operand of O^T = V_i^T P^T), so the inner loop touches no LDS: each wavefront walks tiles of 32
//   query rows (row = (list entry, head of the group), flattened so any g packs densely), gathers the rows
//   of Q straight into the B-operand layout, runs 16 + 16 MFMA 32x32x16 bf16, and does the softmax of the
//   64 scores of a row inside the accumulator layout (a lane holds 32 keys of one query; one cross-lane
//   exchange with lane ^ 32 completes max and sum).  Because S^T leaves each lane holding keys of ONE query,
//   the probabilities are already in B-operand layout for the PV product; no transposition of P is needed.
//   The result of a (token, head, block) triple is a partial output normalised by its own sum, plus the
//   log-sum-exp of its 64 scores; both go to the slot of the workspace given by the entry's idx column.
// k_fwd_merge: per (token, head) combines the kept slots: LSE = ln sum_s exp(lse_s), O = sum_s exp(lse_s-LSE) O_s.
//   This replaces the paper's separate statistics pre-pass: per-slot (max, sum) make the merge exact.
#include "common.h"

namespace nsa {

constexpr int kVtStride = 72;  // bf16 per row of the transposed V tile in LDS: 64 keys + 8 pad

// Place of a key in the contraction order of the PV product.  The accumulator of a 32x32 MFMA gives lane
// (col, q) the rows 8a + 4q + c (a, c in 0..3) of each 32-key half mb; contraction step s' = 2 mb + a / 2 takes
// element e = 4 (a & 1) + c from lane group q.
__device__ __forceinline__ int key_pos(int key) {
  const int mb = key >> 5, a = (key >> 3) & 3, q = (key >> 2) & 1, c = key & 3;
  return 16 * (2 * mb + (a >> 1)) + 8 * q + 4 * (a & 1) + c;
}

__global__ void __launch_bounds__(256)
k_fwd_main(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
           const int32_t* __restrict__ hdr, const int32_t* __restrict__ u_list, const int32_t* __restrict__ u_start,
           const int32_t* __restrict__ off, const int32_t* __restrict__ blk_tok0, const int32_t* __restrict__ blk_len,
           const int32_t* __restrict__ qlist, const int32_t* __restrict__ qslot, bf16_t* __restrict__ opart,
           float* __restrict__ lse_part) {
  __shared__ __attribute__((aligned(16))) bf16_t Vt[kD * kVtStride];
  const int u = blockIdx.x;
  if (u >= hdr[HDR_FUNITS]) return;
  const int L = u_list[u];
  const int j = L / P.b_cap;
  const int gb = L - j * P.b_cap;
  const int e0 = u_start[u];
  const int ne = min(kFwdUnit, off[L + 1] - e0);
  const int tok0 = blk_tok0[gb], blen = blk_len[gb];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, qh = lane >> 5;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  {  // V_i -> LDS, transposed and key-permuted
    const int key = tid >> 2, d0 = (tid & 3) * 32, pos = key_pos(key);
    const bf16_t* src = V + ((size_t)(tok0 + key) * P.hkv + j) * kD + d0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x8 v = key < blen ? *reinterpret_cast<const bf16x8*>(src + 8 * i) : zero8;
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(d0 + 8 * i + e) * kVtStride + pos] = v[e];
    }
  }
  bf16x8 kf[2][8];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int key = 32 * mb + col;
    const bf16_t* src = K + ((size_t)(tok0 + key) * P.hkv + j) * kD + 8 * qh;
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[mb][s] = key < blen ? *reinterpret_cast<const bf16x8*>(src + 16 * s) : zero8;
  }
  __syncthreads();
  bf16x8 vf[4][4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int sp = 0; sp < 4; ++sp)
      vf[db][sp] = *reinterpret_cast<const bf16x8*>(&Vt[(32 * db + col) * kVtStride + 16 * sp + 8 * qh]);

  const int rows_total = ne * P.g;
  const float c2 = P.scale * 1.4426950408889634f;  // scores in the log2 domain
  for (int tile = wave; tile * 32 < rows_total; tile += 4) {
    const int r = tile * 32 + col;
    const bool valid = r < rows_total;
    const int e = valid ? r / P.g : 0;
    const int hh = valid ? r - e * P.g : 0;
    const int t = qlist[e0 + e];
    const int slot = qslot[e0 + e];
    const int h = j * P.g + hh;
    const bf16_t* qrow = Q + ((size_t)t * P.hq + h) * kD + 8 * qh;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = valid ? *reinterpret_cast<const bf16x8*>(qrow + 16 * s) : zero8;

    f32x16 sacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[mb][v] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][s], qf[s], sacc[mb], 0, 0, 0);

    // keys [0, lim) of the block are visible to this row
    int lim = P.causal ? min(blen, t - tok0 + 1) : blen;
    if (!valid) lim = 0;
    float m = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
        const float x = key < lim ? sacc[mb][v] * c2 : -INFINITY;
        sacc[mb][v] = x;
        m = fmaxf(m, x);
      }
    m = fmaxf(m, __shfl_xor(m, 32));
    const float msafe = (m == -INFINITY) ? 0.f : m;
    float l = 0.f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(sacc[mb][v] - msafe);
        sacc[mb][v] = p;
        l += p;
      }
    l += __shfl_xor(l, 32);

    bf16x8 pf[4];
#pragma unroll
    for (int sp = 0; sp < 4; ++sp)
#pragma unroll
      for (int e2 = 0; e2 < 8; ++e2) pf[sp][e2] = (bf16_t)sacc[sp >> 1][8 * (sp & 1) + e2];

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
#pragma unroll
    for (int sp = 0; sp < 4; ++sp)
#pragma unroll
      for (int db = 0; db < 4; ++db)
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][sp], pf[sp], oacc[db], 0, 0, 0);

    if (valid) {
      const float inv = 1.f / l;
      const size_t prow = ((size_t)t * P.hq + h) * P.topk + slot;
      bf16_t* dst = opart + prow * kD + 4 * qh;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          uint2 w;
          w.x = pack_bf16x2(oacc[db][4 * a + 0] * inv, oacc[db][4 * a + 1] * inv);
          w.y = pack_bf16x2(oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv);
          *reinterpret_cast<uint2*>(dst + 32 * db + 8 * a) = w;
        }
      if (qh == 0) lse_part[prow] = (m + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    }
  }
}

// 16 lanes per (token, head) row, 8 output channels per lane.
__global__ void __launch_bounds__(256)
k_fwd_merge(Problem P, const bf16_t* __restrict__ opart, const float* __restrict__ lse_part,
            const uint32_t* __restrict__ vmask, bf16_t* __restrict__ O, float* __restrict__ LSE) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  if (row >= (int64_t)P.T * P.hq) return;
  const int t = (int)(row / P.hq);
  const int h = (int)(row - (int64_t)t * P.hq);
  const uint32_t vm = vmask[(size_t)t * P.hkv + h / P.g];
  bf16_t* orow = O + row * kD + 8 * sub;
  if (vm == 0u) {
    *reinterpret_cast<uint4*>(orow) = make_uint4(0, 0, 0, 0);
    if (sub == 0) LSE[row] = -INFINITY;
    return;
  }
  const float* lp = lse_part + row * P.topk;
  float M = -INFINITY;
  for (int m = 0; m < P.topk; ++m)
    if ((vm >> m) & 1u) M = fmaxf(M, lp[m]);
  float Ls = 0.f;
  for (int m = 0; m < P.topk; ++m)
    if ((vm >> m) & 1u) Ls += __expf(lp[m] - M);
  const float lse = M + __logf(Ls);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const bf16_t* prow = opart + row * P.topk * kD + 8 * sub;
  for (int m = 0; m < P.topk; ++m)
    if ((vm >> m) & 1u) {
      const float w = __expf(lp[m] - lse);
      const uint4 x = *reinterpret_cast<const uint4*>(prow + (size_t)m * kD);
      acc[0] += w * bf16_lo(x.x); acc[1] += w * bf16_hi(x.x);
      acc[2] += w * bf16_lo(x.y); acc[3] += w * bf16_hi(x.y);
      acc[4] += w * bf16_lo(x.z); acc[5] += w * bf16_hi(x.z);
      acc[6] += w * bf16_lo(x.w); acc[7] += w * bf16_hi(x.w);
    }
  uint4 o;
  o.x = pack_bf16x2(acc[0], acc[1]);
  o.y = pack_bf16x2(acc[2], acc[3]);
  o.z = pack_bf16x2(acc[4], acc[5]);
  o.w = pack_bf16x2(acc[6], acc[7]);
  *reinterpret_cast<uint4*>(orow) = o;
  if (sub == 0) LSE[row] = lse;
}

hipError_t launch_fwd(const Problem& P, const IndexLayout& L, const void* Q, const void* K, const void* V,
                      const void* index_ws, void* opart, float* lse_part, void* O, float* LSE, hipStream_t st) {
  IndexPtrs p = index_ptrs(L, const_cast<void*>(index_ws));
  { ProfScope ps(KID_FWD_MAIN, st);
  hipLaunchKernelGGL(k_fwd_main, dim3(L.fwd_units_max), dim3(256), 0, st, P, (const bf16_t*)Q, (const bf16_t*)K,
                     (const bf16_t*)V, p.hdr, p.f_list, p.f_start, p.off, p.blk_tok0, p.blk_len, p.qlist, p.qslot,
                     (bf16_t*)opart, lse_part); }
  const int64_t rows = (int64_t)P.T * P.hq;
  ProfScope ps(KID_FWD_MERGE, st);
  hipLaunchKernelGGL(k_fwd_merge, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, P, (const bf16_t*)opart,
                     (const float*)lse_part, p.vmask, (bf16_t*)O, LSE);
  return hipGetLastError();
}

}  // namespace nsa
