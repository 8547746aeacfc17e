// Block selection in front of the attention path: per (token, KV head) the forced sink / most-recent blocks and
// then the visible blocks with the highest scores (see nsa_sel_select_blocks in nsa_sel.h for the rule).
//
// One wavefront owns one row and looks at it in chunks of up to 1024 blocks, 16 scores per lane held in registers
// as order-preserving unsigned keys.  The fast method (select_by_threshold) bounds the picks from below with the
// r-th largest lane maximum, compacts the few elements above that bound into the LDS and ranks them against each
// other: ~400 instructions per row.  Rows where too many scores tie at the bound fall back to the general method
// (select_by_rounds): one pick per round, each round two wave-wide reductions.  Each visible score is read from
// HBM once, with 16-byte loads when the rows are 16-byte aligned.
#include "common.h"

namespace nsa {
namespace {

constexpr int kSelWaves = 4;                  // rows per workgroup
constexpr int kChunkBlocks = 1024;            // blocks examined at a time: 16 keys per lane
constexpr int kKeys = kChunkBlocks / 64;
constexpr int kMaxChunks = 16;                // rows of up to 16384 blocks
constexpr int kCandPerLane = kMaxChunks * kMaxTopk / 64;   // chunk picks each lane holds in the final selection
constexpr int kTauLowBit = 16;                // the bound is searched on the upper 16 bits of the keys (looser, still a bound)
constexpr int kMaxSurv = 128;                 // survivors the fast method ranks; rows with more take the general one

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

// What one row needs to know about itself.
struct RowInfo {
  const float* srow;  // the row's scores
  int b_vis;          // visible blocks are [0, b_vis)
  int ns;             // forced sinks are [0, ns)
  int nl, loc_lo, loc_hi;   // forced local blocks are [loc_lo, loc_hi] when nl > 0
  int n_forced;       // columns taken by forced blocks
  int want;           // columns to fill by score
  __device__ __forceinline__ bool forced(int b) const { return b < ns || (nl > 0 && b >= loc_lo && b <= loc_hi); }
};

// Block of element e of a lane in the chunk that starts at `base`: four consecutive blocks per 16-byte load, or
// one block per 4-byte load.  Ascends with e inside a lane in both layouts.
template <bool kVec>
__device__ __forceinline__ int blk_of(int base, int lane, int e) {
  return kVec ? base + ((e >> 2) << 8) + (lane << 2) + (e & 3) : base + (e << 6) + lane;
}

// Raw score bits of E elements per lane; what lies at or past b_vis in a lane's FIRST element is not loaded and
// reads as `fill` (a 16-byte load may bring up to three blocks past b_vis along; callers deal with those).
template <bool kVec, int E>
__device__ __forceinline__ void load_bits(const RowInfo& R, int base, int lane, uint32_t fill, uint32_t (&x)[E]) {
  if (kVec) {
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      const int b = base + (q << 8) + (lane << 2);
      u32x4 v = {fill, fill, fill, fill};
      if (b < R.b_vis) v = *reinterpret_cast<const u32x4*>(R.srow + b);   // b + 3 < stride: both multiples of 4
#pragma unroll
      for (int i = 0; i < 4; ++i) x[q * 4 + i] = v[i];
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int b = base + (e << 6) + lane;
      x[e] = b < R.b_vis ? __builtin_bit_cast(uint32_t, R.srow[b]) : fill;
    }
  }
}

// ---- the general method: `want` rounds of "take the largest remaining key".  Exact for any input, also when
// most scores are equal; ~150 instructions per pick, so it only serves rows the fast method hands over.
template <bool kVec>
__device__ __forceinline__ int select_by_rounds(const RowInfo& R, int lane, uint32_t* lds_wave, int mine) {
  uint32_t* cand_key = lds_wave;
  int32_t* cand_blk = reinterpret_cast<int32_t*>(lds_wave + kMaxChunks * kMaxTopk);
  const int n_chunks = (R.b_vis + kChunkBlocks - 1) / kChunkBlocks;
  int n_cand = 0;                          // chunk picks parked in the LDS (only when n_chunks > 1)
  for (int c = 0; c < n_chunks; ++c) {
    const int base = c * kChunkBlocks;
    const int left = R.b_vis - base;       // > 0
    const int ne = left >= kChunkBlocks ? kKeys : (kVec ? ((left + 255) >> 8) << 2 : (left + 63) >> 6);
    uint32_t key[kKeys];
    load_bits<kVec, kKeys>(R, base, lane, 0u, key);
#pragma unroll
    for (int e = 0; e < kKeys; ++e) {
      const int b = blk_of<kVec>(base, lane, e);
      key[e] = (b < R.b_vis && !R.forced(b)) ? order_key(key[e]) : 0u;
    }
    auto blk = [&](int e) { return blk_of<kVec>(base, lane, e); };
    if (n_chunks == 1) {
      pick_rounds<kKeys>(key, ne, R.want, blk, [&](int i, int b, uint32_t) {
        if (lane == R.n_forced + i) mine = b;
      });
    } else {
      const int got = pick_rounds<kKeys>(key, ne, R.want, blk, [&](int i, int b, uint32_t k) {
        if (lane == 0) {
          cand_key[n_cand + i] = k;
          cand_blk[n_cand + i] = b;
        }
      });
      n_cand += got;
    }
  }
  if (n_chunks > 1) {
    // final selection over the chunk picks (written by lane 0 of this wavefront, read by all of its lanes)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t key[kCandPerLane];
    int32_t blk[kCandPerLane];
#pragma unroll
    for (int e = 0; e < kCandPerLane; ++e) {
      const int q = (e << 6) + lane;
      key[e] = q < n_cand ? cand_key[q] : 0u;
      blk[e] = q < n_cand ? cand_blk[q] : 0x7fffffff;
    }
    // within a lane the candidates of later chunks have larger block ids, so blocks ascend with e as required
    pick_rounds<kCandPerLane>(key, (n_cand + 63) >> 6, R.want, [&](int e) { return blk[e]; },
                              [&](int i, int b, uint32_t) {
                                if (lane == R.n_forced + i) mine = b;
                              });
  }
  return mine;
}

// ---- the fast method.  Per chunk of up to 1024 blocks:
//   1. every lane takes the largest of its keys; tau = the r-th largest of the 64 lane maxima, found bit by bit
//      with ballots (scalar work).  r = want + (forced blocks) + 3, so at least `want` selectable blocks of the
//      chunk have a key >= tau (forced blocks and the up to three blocks a 16-byte load brings along past b_vis
//      are not masked beforehand: they are dropped in step 3), hence no block with a key < tau can be a pick;
//   2. the elements with key >= tau ("survivors", a few more than r unless many scores tie) are compacted into
//      an LDS list of (key, ~block) pairs;
//   3. after all chunks every survivor counts the survivors that beat it; that rank is its output column.
// Returns false, having written nothing, when the survivors do not fit the list.
template <bool kVec, int E>
__device__ __forceinline__ void chunk_survivors(const RowInfo& R, int base, int lane, int r, uint64_t* surv, int& n_surv) {
  uint32_t key[E];
  load_bits<kVec, E>(R, base, lane, 0u, key);
  uint32_t lmax = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    // +0 turns -0 into +0 and max(., -inf) turns a NaN into -inf, as the order of the scores demands; then the
    // sign-magnitude bits become an unsigned key of the same order (always > 0).  What was not loaded gets key 0,
    // "nothing here".
    const bool hole = blk_of<kVec>(base, lane, kVec ? (e & ~3) : e) >= R.b_vis;   // not loaded
    float f = __builtin_bit_cast(float, key[e]) + 0.0f;
    f = __builtin_fmaxf(f, -__builtin_inff());
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    const uint32_t k = u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
    key[e] = hole ? 0u : k;
    lmax = key[e] > lmax ? key[e] : lmax;
  }
  uint32_t tau = 0;
  for (int bit = 31; bit >= kTauLowBit; --bit) {
    const uint32_t trial = tau | (1u << bit);
    const int c = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lmax >= trial));
    tau = c >= r ? trial : tau;
  }
  const uint32_t thr = tau ? tau : 1u;     // fewer than r lanes hold anything: every loaded element survives
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const bool sv = key[e] >= thr;
    const uint64_t m = __builtin_amdgcn_ballot_w64(sv);
    if (m != 0) {
      const int pos = n_surv + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
      if (sv && pos < kMaxSurv)
        surv[pos] = ((uint64_t)key[e] << 32) | (uint32_t)~(uint32_t)blk_of<kVec>(base, lane, e);
      n_surv += __builtin_popcountll(m);
    }
  }
}

template <bool kVec>
__device__ __forceinline__ bool select_by_threshold(const RowInfo& R, int lane, uint64_t* surv, int32_t* out_row) {
  const int r = R.want + R.ns + R.nl + 3;   // <= topk + 3 whenever want > 0
  const int n_chunks = (R.b_vis + kChunkBlocks - 1) / kChunkBlocks;
  int n_surv = 0;
  for (int c = 0; c < n_chunks; ++c) {
    const int base = c * kChunkBlocks;
    const int nq = (R.b_vis - base + 255) >> 8;   // quarter chunks with visible blocks (>= 1)
    if (nq >= 4) chunk_survivors<kVec, 16>(R, base, lane, r, surv, n_surv);
    else if (nq == 3) chunk_survivors<kVec, 12>(R, base, lane, r, surv, n_surv);
    else if (nq == 2) chunk_survivors<kVec, 8>(R, base, lane, r, surv, n_surv);
    else chunk_survivors<kVec, 4>(R, base, lane, r, surv, n_surv);
    if (n_surv > kMaxSurv) return false;
  }
  // drop what may not be picked: forced blocks and blocks past the visible range
  for (int q = lane; q < n_surv; q += 64) {
    const int b = (int)~(uint32_t)surv[q];
    if (b >= R.b_vis || R.forced(b)) surv[q] = 0;
  }
  for (int q0 = 0; q0 < n_surv; q0 += 64) {
    const int q = q0 + lane;
    const uint64_t my = q < n_surv ? surv[q] : 0;
    int rank = 0;
#pragma unroll 4
    for (int s = 0; s < n_surv; ++s) rank += surv[s] > my ? 1 : 0;   // same address in every lane: a broadcast
    if (my != 0 && rank < R.want) out_row[R.n_forced + rank] = (int32_t)~(uint32_t)my;
  }
  return true;
}

}  // namespace

template <bool kVec>
__global__ void __launch_bounds__(64 * kSelWaves)
k_select_blocks(const float* __restrict__ scores, int64_t stride, const int32_t* __restrict__ cu, int T, int nseq,
                int hkv, int bk, int topk, int causal, int n_sink, int n_local, int32_t* __restrict__ idx) {
  // per wavefront: the survivor list of the fast method, or the chunk picks of the general one
  __shared__ uint64_t lds[kSelWaves][kMaxChunks * kMaxTopk];
  static_assert(kMaxSurv <= kMaxChunks * kMaxTopk, "survivor list must fit");
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row = (int64_t)blockIdx.x * kSelWaves + w;
  if (row >= (int64_t)T * hkv) return;     // whole wavefront leaves together
  const int t = (int)(row / hkv);
  int s, c0, c1;
  seq_bounds(cu, nseq, T, t, s, c0, c1);
  const int cur = (t - c0) / bk;
  const int b_s = (c1 - c0 + bk - 1) / bk;
  RowInfo R;
  R.b_vis = causal ? (cur + 1 < b_s ? cur + 1 : b_s) : b_s;
  if ((int64_t)R.b_vis > stride) R.b_vis = (int)stride;   // never read past a row, whatever cu says
  // forced blocks: sinks 0 .. ns-1, then cur - r0, cur - r0 - 1, ... (nl of them, all >= ns and < b_vis)
  R.ns = n_sink < R.b_vis ? n_sink : R.b_vis;
  const int r0 = cur - R.b_vis + 1 > 0 ? cur - R.b_vis + 1 : 0;
  const int r_last = n_local - 1 < cur - R.ns ? n_local - 1 : cur - R.ns;
  R.nl = r_last - r0 + 1 > 0 ? r_last - r0 + 1 : 0;
  R.loc_hi = cur - r0;
  R.loc_lo = R.loc_hi - R.nl + 1;
  R.n_forced = R.ns + R.nl < topk ? R.ns + R.nl : topk;
  R.want = topk - R.n_forced;
  R.srow = scores + row * stride;
  int32_t* out_row = idx + row * topk;

  int mine = -1;                           // lane i holds column i of the output row: forced blocks, then -1
  if (lane < R.n_forced) mine = lane < R.ns ? lane : R.loc_hi - (lane - R.ns);
  const int n_free = R.b_vis - R.ns - R.nl;                  // selectable blocks
  int n_picks = R.want < n_free ? R.want : n_free;           // columns the selection fills
  bool by_rank = true;                     // pick columns already written, each by the lane that ranked there
  if (n_picks > 0 && scores == nullptr) {
    n_picks = 0;                           // forced blocks only: the rest of the row is padding
  }
  if (n_picks > 0) {
    by_rank = select_by_threshold<kVec>(R, lane, lds[w], out_row);
    if (!by_rank) mine = select_by_rounds<kVec>(R, lane, reinterpret_cast<uint32_t*>(lds[w]), mine);
  }
  if (lane < topk && (!by_rank || lane < R.n_forced || lane >= R.n_forced + n_picks)) out_row[lane] = mine;
}

}  // namespace nsa

using namespace nsa;

extern "C" int nsa_sel_select_blocks(const nsa_sel_shape* shape, const float* scores, int64_t score_stride,
                                     const int32_t* cu_seqlens, int32_t n_sink, int32_t n_local, int32_t* idx,
                                     void* stream) {
  if (!shape) return NSA_SEL_EINVAL;
  if (shape->total_tokens < 0 || shape->nseq < 1 || shape->hkv < 1 || n_sink < 0 || n_local < 0) return NSA_SEL_EINVAL;
  if (shape->block != kBlock && shape->block != 2 * kBlock) return NSA_SEL_EUNSUPPORTED;
  if (shape->topk < 1 || shape->topk > kMaxTopk) return NSA_SEL_EUNSUPPORTED;
  if (!scores) score_stride = (int64_t)kMaxChunks * kChunkBlocks;   // no rows to stay inside
  if (score_stride < 1 || score_stride > (int64_t)kMaxChunks * kChunkBlocks) return NSA_SEL_EUNSUPPORTED;
  if (!idx || ((uintptr_t)scores & 3) || ((uintptr_t)idx & 3)) return NSA_SEL_EINVAL;   // scores may be NULL
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
