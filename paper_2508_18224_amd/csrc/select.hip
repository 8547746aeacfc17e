// Block selection in front of the attention path: per (token, KV head) the forced sink / most-recent blocks and
// then the visible blocks with the highest scores (see nsa_sel_select_blocks in nsa_sel.h for the rule).
//
// One wavefront owns one row.  The visible scores of up to 1024 blocks sit in 16 registers per lane as order-
// preserving unsigned keys (0 = not a candidate); a pick is two wave-wide 32-bit reductions (largest key, then the
// smallest block id holding it) after which the winner's key is cleared.  Rows with more than 1024 visible blocks
// are handled 1024 at a time: the picks of every chunk go to a small LDS list that one more selection of the same
// kind reduces to the final picks.  HBM-bound: each visible score is read once, with 16-byte loads when the rows
// are 16-byte aligned.
#include "common.h"

namespace nsa {
namespace {

constexpr int kSelWaves = 4;                  // rows per workgroup
constexpr int kChunkBlocks = 1024;            // blocks examined at a time: 16 keys per lane
constexpr int kKeys = kChunkBlocks / 64;
constexpr int kMaxChunks = 16;                // rows of up to 16384 blocks
constexpr int kCandPerLane = kMaxChunks * kMaxTopk / 64;   // chunk picks each lane holds in the final selection

// All four steps stay inside a row of 16 lanes (quad swaps, then mirrors of 8 and of 16 lanes), after which every
// lane of a row holds the row's result; the four rows are combined on the scalar unit.
template <bool kMax>
__device__ __forceinline__ uint32_t wave_reduce(uint32_t v) {
  auto comb = [](uint32_t a, uint32_t b) { return kMax ? (a > b ? a : b) : (a < b ? a : b); };
  v = comb(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, false));   // lanes ^ 1
  v = comb(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, false));   // lanes ^ 2
  v = comb(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xF, 0xF, false));  // mirror of 8
  v = comb(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xF, 0xF, false));  // mirror of 16
  const uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
  return comb(comb(a, b), comb(c, d));
}

// fp32 bits -> unsigned key with the same order as the values; NaN ranks with -infinity, -0 with +0, and every
// key is > 0 so that 0 can mean "no candidate".
__device__ __forceinline__ uint32_t order_key(uint32_t u) {
  if ((u & 0x7fffffffu) > 0x7f800000u) u = 0xff800000u;   // NaN -> -inf
  if (u == 0x80000000u) u = 0u;                            // -0 -> +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Picks up to `want` candidates in descending (key, then ascending block) order.  key[e] belongs to block
// blk_of(e), which must ascend with e inside a lane; ne bounds the e that can hold candidates (wave-uniform).
// emit(i, block, key) is called wave-uniformly for the i-th pick.  Returns the number of picks.
template <int E, class BlkOf, class Emit>
__device__ __forceinline__ int pick_rounds(uint32_t (&key)[E], int ne, int want, BlkOf blk_of, Emit emit) {
  int got = 0;
  for (; got < want; ++got) {
    uint32_t best = 0, bblk = 0x7fffffffu;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (e < ne) {
        const bool up = key[e] > best;      // strict: of equal keys the lane keeps its smallest block
        best = up ? key[e] : best;
        bblk = up ? (uint32_t)blk_of(e) : bblk;
      }
    }
    const uint32_t m = wave_reduce<true>(best);
    if (m == 0) break;                      // no candidate left
    const uint32_t wb = wave_reduce<false>(best == m ? bblk : 0x7fffffffu);
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (e < ne) key[e] = ((uint32_t)blk_of(e) == wb) ? 0u : key[e];   // block ids are unique: clears the winner only
    }
    emit(got, (int)wb, m);
  }
  return got;
}

template <bool kVec>
__global__ void __launch_bounds__(64 * kSelWaves)
k_select_blocks(const float* __restrict__ scores, int64_t stride, const int32_t* __restrict__ cu, int T, int nseq,
                int hkv, int bk, int topk, int causal, int n_sink, int n_local, int32_t* __restrict__ idx) {
  __shared__ uint32_t cand_key[kSelWaves][kMaxChunks * kMaxTopk];
  __shared__ int32_t cand_blk[kSelWaves][kMaxChunks * kMaxTopk];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row = (int64_t)blockIdx.x * kSelWaves + w;
  if (row >= (int64_t)T * hkv) return;     // whole wavefront leaves together
  const int t = (int)(row / hkv);
  int s, c0, c1;
  seq_bounds(cu, nseq, T, t, s, c0, c1);
  const int cur = (t - c0) / bk;
  const int b_s = (c1 - c0 + bk - 1) / bk;
  int b_vis = causal ? (cur + 1 < b_s ? cur + 1 : b_s) : b_s;
  if ((int64_t)b_vis > stride) b_vis = (int)stride;   // never read past a row, whatever cu says
  // forced blocks: sinks 0 .. ns-1, then cur - r0, cur - r0 - 1, ... (nl of them, all >= ns and < b_vis)
  const int ns = n_sink < b_vis ? n_sink : b_vis;
  const int r0 = cur - b_vis + 1 > 0 ? cur - b_vis + 1 : 0;
  int r_last = n_local - 1 < cur - ns ? n_local - 1 : cur - ns;
  const int nl = r_last - r0 + 1 > 0 ? r_last - r0 + 1 : 0;
  const int loc_hi = cur - r0, loc_lo = loc_hi - nl + 1;    // local forced blocks are [loc_lo, loc_hi] when nl > 0
  const int n_forced = ns + nl < topk ? ns + nl : topk;
  const int want = topk - n_forced;                          // picks by score
  const float* __restrict__ srow = scores + row * stride;

  int mine = -1;                           // lane i ends up holding column i of the output row
  if (lane < n_forced) mine = lane < ns ? lane : loc_hi - (lane - ns);

  const int n_chunks = (b_vis + kChunkBlocks - 1) / kChunkBlocks;
  int n_cand = 0;                          // chunk picks parked in the LDS (only when n_chunks > 1)
  for (int c = 0; c < n_chunks && want > 0; ++c) {
    const int base = c * kChunkBlocks;
    const int left = b_vis - base;                                   // > 0
    const int ne = left >= kChunkBlocks ? kKeys : (kVec ? ((left + 255) >> 8) << 2 : (left + 63) >> 6);
    // element e of a lane is block base + blk_in(e): four consecutive blocks per 16-byte load, or one per load
    auto blk_of = [&](int e) { return kVec ? base + ((e >> 2) << 8) + (lane << 2) + (e & 3) : base + (e << 6) + lane; };
    uint32_t key[kKeys];
    if (kVec) {
#pragma unroll
      for (int q = 0; q < kKeys / 4; ++q) {
        u32x4 x = {0u, 0u, 0u, 0u};
        const int b = base + (q << 8) + (lane << 2);
        if (q * 4 < ne && b < b_vis) x = *reinterpret_cast<const u32x4*>(srow + b);   // b + 3 < stride: both multiples of 4
#pragma unroll
        for (int i = 0; i < 4; ++i) key[q * 4 + i] = x[i];
      }
    } else {
#pragma unroll
      for (int e = 0; e < kKeys; ++e) {
        const int b = base + (e << 6) + lane;
        key[e] = (e < ne && b < b_vis) ? __builtin_bit_cast(uint32_t, srow[b]) : 0u;
      }
    }
#pragma unroll
    for (int e = 0; e < kKeys; ++e) {
      const int b = blk_of(e);
      const bool forced = b < ns || (nl > 0 && b >= loc_lo && b <= loc_hi);
      key[e] = (e < ne && b < b_vis && !forced) ? order_key(key[e]) : 0u;
    }
    if (n_chunks == 1) {
      pick_rounds<kKeys>(key, ne, want, blk_of, [&](int i, int blk, uint32_t) {
        if (lane == n_forced + i) mine = blk;
      });
    } else {
      const int got = pick_rounds<kKeys>(key, ne, want, blk_of, [&](int i, int blk, uint32_t k) {
        if (lane == 0) {
          cand_key[w][n_cand + i] = k;
          cand_blk[w][n_cand + i] = blk;
        }
      });
      n_cand += got;
    }
  }
  if (n_chunks > 1 && want > 0) {
    // final selection over the chunk picks (written by lane 0 of this wavefront, read by all of its lanes)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t key[kCandPerLane];
    int32_t blk[kCandPerLane];
#pragma unroll
    for (int e = 0; e < kCandPerLane; ++e) {
      const int q = (e << 6) + lane;
      key[e] = q < n_cand ? cand_key[w][q] : 0u;
      blk[e] = q < n_cand ? cand_blk[w][q] : 0x7fffffff;
    }
    // within a lane the candidates of later chunks have larger block ids, so blocks ascend with e as required
    pick_rounds<kCandPerLane>(key, (n_cand + 63) >> 6, want, [&](int e) { return blk[e]; },
                              [&](int i, int b, uint32_t) {
                                if (lane == n_forced + i) mine = b;
                              });
  }
  if (lane < topk) idx[row * topk + lane] = mine;
}

}  // namespace
}  // namespace nsa

using namespace nsa;

extern "C" int nsa_sel_select_blocks(const nsa_sel_shape* shape, const float* scores, int64_t score_stride,
                                     const int32_t* cu_seqlens, int32_t n_sink, int32_t n_local, int32_t* idx,
                                     void* stream) {
  if (!shape) return NSA_SEL_EINVAL;
  if (shape->total_tokens < 0 || shape->nseq < 1 || shape->hkv < 1 || n_sink < 0 || n_local < 0) return NSA_SEL_EINVAL;
  if (shape->block != kBlock && shape->block != 2 * kBlock) return NSA_SEL_EUNSUPPORTED;
  if (shape->topk < 1 || shape->topk > kMaxTopk) return NSA_SEL_EUNSUPPORTED;
  if (score_stride < 1 || score_stride > (int64_t)kMaxChunks * kChunkBlocks) return NSA_SEL_EUNSUPPORTED;
  if (!scores || !idx || ((uintptr_t)scores & 3) || ((uintptr_t)idx & 3)) return NSA_SEL_EINVAL;
  if (!cu_seqlens && shape->nseq != 1) return NSA_SEL_EINVAL;
  const int64_t rows = (int64_t)shape->total_tokens * shape->hkv;
  if (rows == 0) return NSA_SEL_OK;
  if (rows * shape->topk >= ((int64_t)1 << 31)) return NSA_SEL_EUNSUPPORTED;
  const int64_t grid = (rows + kSelWaves - 1) / kSelWaves;
  if (grid >= ((int64_t)1 << 31)) return NSA_SEL_EUNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof(KID_SELECT_BLOCKS, st);
  const bool vec = (score_stride & 3) == 0 && ((uintptr_t)scores & 15) == 0;
  auto kern = vec ? k_select_blocks<true> : k_select_blocks<false>;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * kSelWaves), 0, st, scores, score_stride, cu_seqlens,
                     shape->total_tokens, shape->nseq, shape->hkv, shape->block, shape->topk, shape->causal ? 1 : 0,
                     (int)n_sink, (int)n_local, idx);
  return hipGetLastError() == hipSuccess ? NSA_SEL_OK : NSA_SEL_EHIP;
}
