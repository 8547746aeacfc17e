// Backward selected-block attention for gfx950.  The paper (Sec. 3.2) only says that the backward pass follows
// the forward's KV-outer logic, gathers the queries again through the cached index tensors and stores
// intermediate query gradients to a buffer that a reduction kernel sums; dK/dV accumulation is not described.
// This file is that pass, with dK/dV accumulated without atomics:
//
//   k_bwd_delta       delta[t,h] = <dO[t,h], O[t,h]>
//   k_bwd_main        one work unit = (kv head j, KV block i, up to kBwdUnit list entries).  The four wavefronts
//                     of a workgroup share tiles of 128 gathered rows.  Wave w owns rows 32w..32w+31 for
//                     S^T = K_i Q^T, dP^T = V_i dO^T, P = exp(S - LSE), dS = P (dP - delta) scale and
//                     dQ^T = K_i^T dS^T (its probabilities leave the MFMA already in B-operand layout), and it
//                     owns channels 32w..32w+31 of the dK_i / dV_i accumulators, which stay in registers for
//                     the whole unit: dV_i += P^T dO, dK_i += dS^T Q contract over the 128 rows of the tile
//                     through LDS copies of P^T, dS^T, Q and dO.  Partial dQ rows go to the (token, head, slot)
//                     workspace; the unit's dK_i, dV_i go to a per-unit fp32 buffer.
//   k_bwd_dq_reduce   dQ[t,h] = sum over kept slots of the partial rows
//   k_bwd_dkv_reduce  dK_i, dV_i = sum over the list's units in unit order (fixed order: bit-reproducible)
#include "common.h"

namespace nsa {

constexpr int kKtStride = 72;    // bf16 per row of K^T in LDS (64 keys + 8 pad)
constexpr int kRowStride = 136;  // bf16 per row of the Q / dO / P^T / dS^T tiles in LDS (128 + 8 pad)
constexpr int kTileRows = 128;

constexpr int kLdsKt = 0;
constexpr int kLdsQ = kLdsKt + kD * kKtStride * 2;
constexpr int kLdsDO = kLdsQ + kTileRows * kRowStride * 2;
constexpr int kLdsPt = kLdsDO + kTileRows * kRowStride * 2;
constexpr int kLdsDSt = kLdsPt + kBlock * kRowStride * 2;
constexpr int kLdsBwdBytes = kLdsDSt + kBlock * kRowStride * 2;  // 122880

__device__ __forceinline__ int key_pos_bwd(int key) {  // same contraction order as the forward's PV product
  const int mb = key >> 5, a = (key >> 3) & 3, q = (key >> 2) & 1, c = key & 3;
  return 16 * (2 * mb + (a >> 1)) + 8 * q + 4 * (a & 1) + c;
}

__global__ void __launch_bounds__(256)
k_bwd_delta(int64_t rows, const bf16_t* __restrict__ O, const bf16_t* __restrict__ dO, float* __restrict__ delta) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  float acc = 0.f;
  if (row < rows) {
    const uint4 a = *reinterpret_cast<const uint4*>(O + row * kD + 8 * sub);
    const uint4 b = *reinterpret_cast<const uint4*>(dO + row * kD + 8 * sub);
    acc = bf16_lo(a.x) * bf16_lo(b.x) + bf16_hi(a.x) * bf16_hi(b.x) + bf16_lo(a.y) * bf16_lo(b.y) +
          bf16_hi(a.y) * bf16_hi(b.y) + bf16_lo(a.z) * bf16_lo(b.z) + bf16_hi(a.z) * bf16_hi(b.z) +
          bf16_lo(a.w) * bf16_lo(b.w) + bf16_hi(a.w) * bf16_hi(b.w);
  }
  acc += __shfl_xor(acc, 8);
  acc += __shfl_xor(acc, 4);
  acc += __shfl_xor(acc, 2);
  acc += __shfl_xor(acc, 1);
  if (row < rows && sub == 0) delta[row] = acc;
}

__global__ void __launch_bounds__(256)
k_bwd_main(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
           const bf16_t* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
           const int32_t* __restrict__ hdr, const int32_t* __restrict__ u_list, const int32_t* __restrict__ u_start,
           const int32_t* __restrict__ off, const int32_t* __restrict__ blk_tok0, const int32_t* __restrict__ blk_len,
           const int32_t* __restrict__ qlist, const int32_t* __restrict__ qslot, bf16_t* __restrict__ dqpart,
           float* __restrict__ dkv_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Kt = reinterpret_cast<bf16_t*>(smem + kLdsKt);
  bf16_t* Qs = reinterpret_cast<bf16_t*>(smem + kLdsQ);
  bf16_t* dOs = reinterpret_cast<bf16_t*>(smem + kLdsDO);
  bf16_t* Pt = reinterpret_cast<bf16_t*>(smem + kLdsPt);
  bf16_t* dSt = reinterpret_cast<bf16_t*>(smem + kLdsDSt);

  const int u = blockIdx.x;
  if (u >= hdr[HDR_BUNITS]) return;
  const int L = u_list[u];
  const int j = L / P.b_cap;
  const int gb = L - j * P.b_cap;
  const int e0 = u_start[u];
  const int ne = min(kBwdUnit, off[L + 1] - e0);
  const int tok0 = blk_tok0[gb], blen = blk_len[gb];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, qh = lane >> 5;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  {  // K_i -> LDS, transposed and key-permuted (A operand of dQ^T = K^T dS^T)
    const int key = tid >> 2, d0 = (tid & 3) * 32, pos = key_pos_bwd(key);
    const bf16_t* src = K + ((size_t)(tok0 + key) * P.hkv + j) * kD + d0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x8 v = key < blen ? *reinterpret_cast<const bf16x8*>(src + 8 * i) : zero8;
#pragma unroll
      for (int e = 0; e < 8; ++e) Kt[(d0 + 8 * i + e) * kKtStride + pos] = v[e];
    }
  }
  bf16x8 kf[2][8], vf[2][8];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int key = 32 * mb + col;
    const size_t o = ((size_t)(tok0 + key) * P.hkv + j) * kD + 8 * qh;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      kf[mb][s] = key < blen ? *reinterpret_cast<const bf16x8*>(K + o + 16 * s) : zero8;
      vf[mb][s] = key < blen ? *reinterpret_cast<const bf16x8*>(V + o + 16 * s) : zero8;
    }
  }
  f32x16 dkacc[2], dvacc[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      dkacc[mb][v] = 0.f;
      dvacc[mb][v] = 0.f;
    }
  __syncthreads();

  const int rows_total = ne * P.g;
  const float c2 = P.scale * 1.4426950408889634f;
  for (int tile0 = 0; tile0 < rows_total; tile0 += kTileRows) {
    const int r = tile0 + 32 * wave + col;
    const bool valid = r < rows_total;
    const int e = valid ? r / P.g : 0;
    const int hh = valid ? r - e * P.g : 0;
    const int t = qlist[e0 + e];
    const int slot = qslot[e0 + e];
    const int h = j * P.g + hh;
    const size_t grow = (size_t)t * P.hq + h;
    bf16x8 qf[8], dof[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      qf[s] = valid ? *reinterpret_cast<const bf16x8*>(Q + grow * kD + 16 * s + 8 * qh) : zero8;
      dof[s] = valid ? *reinterpret_cast<const bf16x8*>(dO + grow * kD + 16 * s + 8 * qh) : zero8;
    }
    const float lse2 = valid ? LSE[grow] * 1.4426950408889634f : 0.f;
    const float dl = valid ? delta[grow] : 0.f;
    {
      bf16_t* qdst = Qs + (32 * wave + col) * kRowStride + 8 * qh;
      bf16_t* ddst = dOs + (32 * wave + col) * kRowStride + 8 * qh;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        *reinterpret_cast<bf16x8*>(qdst + 16 * s) = qf[s];
        *reinterpret_cast<bf16x8*>(ddst + 16 * s) = dof[s];
      }
    }
    f32x16 sacc[2], dpacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        sacc[mb][v] = 0.f;
        dpacc[mb][v] = 0.f;
      }
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][s], qf[s], sacc[mb], 0, 0, 0);
        dpacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mb][s], dof[s], dpacc[mb], 0, 0, 0);
      }
    int lim = P.causal ? min(blen, t - tok0 + 1) : blen;
    if (!valid) lim = 0;
    // P and dS (scaled) of this wave's 32 rows; P^T, dS^T to LDS for the dK/dV products
    bf16_t* pdst = Pt + 32 * wave + col;
    bf16_t* sdst = dSt + 32 * wave + col;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
        const float p = key < lim ? __builtin_amdgcn_exp2f(sacc[mb][v] * c2 - lse2) : 0.f;
        const float ds = p * (dpacc[mb][v] - dl) * P.scale;
        sacc[mb][v] = ds;
        pdst[key * kRowStride] = (bf16_t)p;
        sdst[key * kRowStride] = (bf16_t)ds;
      }
    bf16x8 dsf[4];
#pragma unroll
    for (int sp = 0; sp < 4; ++sp)
#pragma unroll
      for (int e2 = 0; e2 < 8; ++e2) dsf[sp][e2] = (bf16_t)sacc[sp >> 1][8 * (sp & 1) + e2];
    f32x16 dqacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) dqacc[db][v] = 0.f;
#pragma unroll
    for (int sp = 0; sp < 4; ++sp)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x8 ktf = *reinterpret_cast<const bf16x8*>(&Kt[(32 * db + col) * kKtStride + 16 * sp + 8 * qh]);
        dqacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf[sp], dqacc[db], 0, 0, 0);
      }
    if (valid) {
      bf16_t* dst = dqpart + ((size_t)e0 * P.g + r) * kD + 4 * qh;  // compact: list position * g + head
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          uint2 w;
          w.x = pack_bf16x2(dqacc[db][4 * a + 0], dqacc[db][4 * a + 1]);
          w.y = pack_bf16x2(dqacc[db][4 * a + 2], dqacc[db][4 * a + 3]);
          *reinterpret_cast<uint2*>(dst + 32 * db + 8 * a) = w;
        }
    }
    __syncthreads();
    // dV_i[:, 32w..32w+31] += P^T dO,  dK_i[:, 32w..32w+31] += dS^T Q  over the tile's 128 rows
    const int dcol = 32 * wave + col;
#pragma unroll
    for (int qs = 0; qs < 8; ++qs) {
      bf16x8 dob, qb;
#pragma unroll
      for (int e2 = 0; e2 < 8; ++e2) {
        dob[e2] = dOs[(16 * qs + 8 * qh + e2) * kRowStride + dcol];
        qb[e2] = Qs[(16 * qs + 8 * qh + e2) * kRowStride + dcol];
      }
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const bf16x8 pa = *reinterpret_cast<const bf16x8*>(&Pt[(32 * mb + col) * kRowStride + 16 * qs + 8 * qh]);
        const bf16x8 sa = *reinterpret_cast<const bf16x8*>(&dSt[(32 * mb + col) * kRowStride + 16 * qs + 8 * qh]);
        dvacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa, dob, dvacc[mb], 0, 0, 0);
        dkacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa, qb, dkacc[mb], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  // unit partial: [u][0 = dK, 1 = dV][key][d] fp32
  float* outk = dkv_part + (size_t)u * 2 * kBlock * kD + 32 * wave + col;
  float* outv = outk + kBlock * kD;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
      outk[key * kD] = dkacc[mb][v];
      outv[key * kD] = dvacc[mb][v];
    }
}

__global__ void __launch_bounds__(256)
k_bwd_dq_reduce(Problem P, const bf16_t* __restrict__ dqpart, const uint32_t* __restrict__ vmask,
                const int32_t* __restrict__ slotpos, bf16_t* __restrict__ dQ) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  if (row >= (int64_t)P.T * P.hq) return;
  const int t = (int)(row / P.hq);
  const int h = (int)(row - (int64_t)t * P.hq);
  const int j = h / P.g, hh = h - j * P.g;
  const uint32_t vm = vmask[(size_t)t * P.hkv + j];
  const int32_t* sp = slotpos + ((size_t)t * P.hkv + j) * P.topk;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int m0 = 0; m0 < P.topk; m0 += 16) {  // 16 independent 256-byte gathers in flight per row
    uint4 x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = m0 + i;
      const bool on = m < P.topk && ((vm >> m) & 1u);
      x[i] = on ? *reinterpret_cast<const uint4*>(dqpart + ((size_t)sp[on ? m : 0] * P.g + hh) * kD + 8 * sub)
                : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      acc[0] += bf16_lo(x[i].x); acc[1] += bf16_hi(x[i].x);
      acc[2] += bf16_lo(x[i].y); acc[3] += bf16_hi(x[i].y);
      acc[4] += bf16_lo(x[i].z); acc[5] += bf16_hi(x[i].z);
      acc[6] += bf16_lo(x[i].w); acc[7] += bf16_hi(x[i].w);
    }
  }
  uint4 o;
  o.x = pack_bf16x2(acc[0], acc[1]);
  o.y = pack_bf16x2(acc[2], acc[3]);
  o.z = pack_bf16x2(acc[4], acc[5]);
  o.w = pack_bf16x2(acc[6], acc[7]);
  *reinterpret_cast<uint4*>(dQ + row * kD + 8 * sub) = o;
}

// grid (n_lists, 2): y = 0 -> dK, 1 -> dV.  Thread handles 4 consecutive channels of 8 keys.
__global__ void __launch_bounds__(256)
k_bwd_dkv_reduce(Problem P, const int32_t* __restrict__ nu_scan, const int32_t* __restrict__ blk_tok0,
                 const int32_t* __restrict__ blk_len, const float* __restrict__ dkv_part, bf16_t* __restrict__ dK,
                 bf16_t* __restrict__ dV) {
  const int L = blockIdx.x, which = blockIdx.y;
  const int j = L / P.b_cap, gb = L - j * P.b_cap;
  const int blen = blk_len[gb];
  if (blen == 0) return;
  const int tok0 = blk_tok0[gb];
  const int u0 = nu_scan[L], u1 = nu_scan[L + 1];
  bf16_t* out = which ? dV : dK;
  const int d4 = (threadIdx.x & 31) * 4;
  for (int key = threadIdx.x >> 5; key < blen; key += 8) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int u = u0; u < u1; ++u) {
      const float4 x =
          *reinterpret_cast<const float4*>(dkv_part + ((size_t)u * 2 + which) * kBlock * kD + key * kD + d4);
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    uint2 w;
    w.x = pack_bf16x2(acc.x, acc.y);
    w.y = pack_bf16x2(acc.z, acc.w);
    *reinterpret_cast<uint2*>(out + ((size_t)(tok0 + key) * P.hkv + j) * kD + d4) = w;
  }
}

hipError_t launch_bwd(const Problem& P, const IndexLayout& L, const void* Q, const void* K, const void* V,
                      const void* O, const float* LSE, const void* dO, const void* index_ws, void* dqpart,
                      float* delta, float* dkv_part, void* dQ, void* dK, void* dV, hipStream_t st) {
  IndexPtrs p = index_ptrs(L, const_cast<void*>(index_ws));
  {
    hipError_t e =
        hipFuncSetAttribute((const void*)k_bwd_main, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBwdBytes);
    if (e != hipSuccess) return e;
  }
  const int64_t rows = (int64_t)P.T * P.hq;
  const unsigned row_blocks = (unsigned)((rows + 15) / 16);
  { ProfScope ps(KID_BWD_DELTA, st);
  hipLaunchKernelGGL(k_bwd_delta, dim3(row_blocks), dim3(256), 0, st, rows, (const bf16_t*)O, (const bf16_t*)dO, delta); }
  { ProfScope ps(KID_BWD_MAIN, st);
  hipLaunchKernelGGL(k_bwd_main, dim3(L.bwd_units_max), dim3(256), kLdsBwdBytes, st, P, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, LSE, (const float*)delta, p.hdr, p.b_list,
                     p.b_start, p.off, p.blk_tok0, p.blk_len, p.qlist, p.qslot, (bf16_t*)dqpart, dkv_part); }
  { ProfScope ps(KID_BWD_DQ_REDUCE, st);
  hipLaunchKernelGGL(k_bwd_dq_reduce, dim3(row_blocks), dim3(256), 0, st, P, (const bf16_t*)dqpart, p.vmask,
                     p.slotpos, (bf16_t*)dQ); }
  ProfScope ps(KID_BWD_DKV_REDUCE, st);
  hipLaunchKernelGGL(k_bwd_dkv_reduce, dim3(L.n_lists, 2), dim3(256), 0, st, P, p.b_nu, p.blk_tok0, p.blk_len,
                     (const float*)dkv_part, (bf16_t*)dK, (bf16_t*)dV);
  return hipGetLastError();
}

}  // namespace nsa
