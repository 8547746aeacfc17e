// Forward selected-block attention for gfx950 (paper Sec. 3.2, the KV-outer token-selection step and the
// reduction step; Eq. (2), c = sel).
//
// k_fwd_main (B_K = 64): one work unit = (kv head j, KV block i, up to P.unit entries of the block's query list).
//   The block's K_i stays in registers for the whole unit (the A operand of S^T = K_i Q^T) and V_i^T sits in LDS,
//   transposed and key-permuted once per unit (the A operand of O^T = V_i^T P^T), so the inner loop reads no K/V
//   from memory: each wavefront walks tiles of 32 query rows (row = (list entry, head of the group), flattened so
//   any g packs densely).  The kernel is held to 256 registers per wavefront so that TWO workgroups share a CU:
//   one's unit prologue, gather waits and softmax overlap the other's MFMA and stores (with V_i^T in registers too
//   only one workgroup fitted and the kernel ran 30 % slower).  The rows of Q are gathered coalesced (16 lanes x 16
//   bytes per row) one tile ahead and re-laid out into the B-operand layout
//   through a wave-private LDS tile; 16 + 16 MFMA 32x32x16 bf16 per tile; the softmax of the 64 scores of a row
//   runs inside the accumulator layout (a lane holds 32 keys of one query; one cross-lane exchange with
//   lane ^ 32 completes max and sum).  Because S^T leaves each lane holding keys of ONE query, the probabilities
//   are already in B-operand layout for the PV product; no transposition of P is needed.
//   The result of a (token, head, block) triple is a partial output normalised by its own sum, plus the
//   log-sum-exp of its 64 scores; both are stored at the entry's own position in the list order (the compact
//   buffer the paper addresses through O_i), so a tile's 32 rows are one contiguous 8 KB (non-temporal) write.
// k_fwd_main128 (B_K = 128): see the comment above it.
// k_fwd_merge: per (token, head) combines the kept slots: LSE = ln sum_s exp(lse_s), O = sum_s exp(lse_s-LSE) O_s.
//   This replaces the paper's separate statistics pre-pass: per-slot log-sum-exps make the merge exact.
#include "common.h"

namespace nsa {

constexpr int kVtStride = 72;     // bf16 per row of the transposed V tile in LDS: 64 keys + 8 pad
constexpr int kTileStride = 136;  // bf16 per row of a wave's private 32-row tile in LDS: 128 + 8 pad

// Place of a key in the contraction order of the PV product.  The accumulator of a 32x32 MFMA gives lane
// (col, q) the rows 8a + 4q + c (a, c in 0..3) of each 32-key half mb; contraction step s' = 2 mb + a / 2 takes
// element e = 4 (a & 1) + c from lane group q.
__device__ __forceinline__ int key_pos(int key) {
  const int mb = key >> 5, a = (key >> 3) & 3, q = (key >> 2) & 1, c = key & 3;
  return 16 * (2 * mb + (a >> 1)) + 8 * q + 4 * (a & 1) + c;
}

// Orders a wavefront's own LDS traffic (no cross-wave meaning): a wave-private tile is written by some lanes and
// read by others of the same wave.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}


// Tokens of a work unit's list entries that take the gather route, compacted into `ent`, with each one's index
// inside the unit in `epos` (its partial rows live at the entry's list position, dense entries leave holes there).
// Entries of dense (tile, block) pairs carry the sign bit in their column (see k_scatter) and are skipped.  Block-wide:
// every thread takes entries i0 + tid of up to kMaxUnit / kThreads rounds, a round's survivors of a wavefront are
// ranked by ballot, and the (round, wavefront) counts are prefix-summed through `cnts`.  Returns the number of
// entries kept; ends with a barrier.
template <int kThreads>
__device__ __forceinline__ int load_sparse_entries(const int2* __restrict__ qent, int e0, int ne, int32_t* ent,
                                                   uint16_t* epos, int32_t* cnts) {
  constexpr int kRounds = kMaxUnit / kThreads, kWaves = kThreads / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int tok[kRounds];
  unsigned long long keep[kRounds];
#pragma unroll
  for (int r = 0; r < kRounds; ++r) {
    const int i = r * kThreads + tid;
    int2 e = make_int2(0, -1);
    if (i < ne) e = qent[e0 + i];
    tok[r] = e.x;
    keep[r] = __builtin_amdgcn_ballot_w64(e.y >= 0);
    if (lane == 0) cnts[r * kWaves + wave] = __popcll(keep[r]);
  }
  __syncthreads();
  int run = 0;
#pragma unroll
  for (int r = 0; r < kRounds; ++r) {
    int before = 0;  // survivors of earlier rounds and of the lower wavefronts of this round
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if (w == wave) before = run;
      run += cnts[r * kWaves + w];
    }
    if ((keep[r] >> lane) & 1ull) {
      const int pos = before + __popcll(keep[r] & ((1ull << lane) - 1ull));
      ent[pos] = tok[r];
      epos[pos] = (uint16_t)(r * kThreads + tid);
    }
  }
  __syncthreads();
  return run;
}

// LDS of k_fwd_main (dynamic: 66 KB, two workgroups per CU)
constexpr int kF64Vt = 0;
constexpr int kF64Tiles = kF64Vt + kD * kVtStride * 2;
constexpr int kF64Ent = kF64Tiles + 4 * 32 * kTileStride * 2;
constexpr int kF64Epos = kF64Ent + kMaxUnit * 4;
constexpr int kF64Cnts = kF64Epos + kMaxUnit * 2;
constexpr int kF64Rowpos = kF64Cnts + (kMaxUnit / 64) * 4;
constexpr int kF64Bytes = kF64Rowpos + 4 * 32 * 8;
static_assert(2 * kF64Bytes <= 160 * 1024, "two workgroups of the 64-key forward must fit one CU's LDS");

__global__ void __launch_bounds__(256, 2)  // two workgroups per CU: 256 registers per wavefront
k_fwd_main(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
           const int32_t* __restrict__ nu_scan, const int32_t* __restrict__ u_list, const int32_t* __restrict__ u_start,
           const int32_t* __restrict__ off, const int32_t* __restrict__ blk_tok0, const int32_t* __restrict__ blk_len,
           const int2* __restrict__ qent, bf16_t* __restrict__ opart,
           float* __restrict__ lse_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Vt = reinterpret_cast<bf16_t*>(smem + kF64Vt);
  int32_t* ent = reinterpret_cast<int32_t*>(smem + kF64Ent);     // tokens of the unit's list entries that take this route
  uint16_t* epos = reinterpret_cast<uint16_t*>(smem + kF64Epos);  // and their index inside the unit
  int32_t* cnts = reinterpret_cast<int32_t*>(smem + kF64Cnts);
  // units of this pass's KV heads [j0, j0 + nj); nu_scan is the exclusive scan of units per list
  const int u = nu_scan[P.j0 * P.b_cap] + blockIdx.x;
  if (u >= nu_scan[(P.j0 + P.nj) * P.b_cap]) return;
  const int L = u_list[u];
  const int j = L / P.b_cap;
  const int gb = L - j * P.b_cap;
  const int e0 = u_start[u];
  const int pos0 = off[P.j0 * P.b_cap];  // first list position of the pass: partial rows are relative to it
  const int ne_all = min(P.unit, off[L + 1] - e0);
  const int tok0 = blk_tok0[gb], blen = blk_len[gb];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, qh = lane >> 5;
  const int crow = lane >> 4, cchunk = (lane & 15) * 8;  // coalesced layout: 16 lanes per row, 4 rows per access
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  // entries of dense (tile, block) pairs are the dense kernel's: a unit made of them only (the sink block's) ends here
  const int ne = load_sparse_entries<256>(qent, e0, ne_all, ent, epos, cnts);
  if (ne == 0) return;

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
  const bf16_t* vbase = &Vt[col * kVtStride + 8 * qh];  // this lane's V^T fragments: + 32 db rows, + 16 sp keys

  const int rows_total = ne * P.g;
  const int n_tiles = (rows_total + 31) >> 5;
  if (wave >= n_tiles) return;  // no block-wide barrier below this point
  const float c2 = P.scale * 1.4426950408889634f;  // scores in the log2 domain
  bf16_t* tile_lds = reinterpret_cast<bf16_t*>(smem + kF64Tiles) + wave * 32 * kTileStride;
  // per wavefront: the partial-buffer row of each of the tile's 32 rows
  int64_t* rowpos = reinterpret_cast<int64_t*>(smem + kF64Rowpos) + 32 * wave;
  const int hbase = j * P.g;

  // gather the 32 rows of Q of a tile in coalesced form (a row = 16 lanes x 16 bytes, 4 rows per access)
  auto issue_q = [&](int tile, u32x4 (&qc)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // rows past the end of the list re-read the last row: they are masked out below and never stored
      const int r = min(tile * 32 + 4 * i + crow, rows_total - 1);
      const int e = div_g(r, P.g, P.g_magic);
      // (token, head) row index in 32 bits (total_tokens * hq < 2^31 is checked on the host), widened once
      const uint32_t grow = (uint32_t)ent[e] * (uint32_t)P.hq + (uint32_t)(hbase + (r - e * P.g));
      qc[i] = *reinterpret_cast<const u32x4*>(Q + ((size_t)grow * kD + cchunk));
    }
  };

  auto do_tile = [&](int tile, u32x4 (&qc)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4*>(&tile_lds[(4 * i + crow) * kTileStride + cchunk]) = qc[i];
    // this wave's next tile: its rows fly during the compute (issued before anything waits on the LDS)
    if (tile + 4 < n_tiles) issue_q(tile + 4, qc);
    wave_sync();
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
      qf[s] = *reinterpret_cast<const bf16x8*>(&tile_lds[col * kTileStride + 16 * s + 8 * qh]);

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
    const int r = tile * 32 + col;
    const bool valid = r < rows_total;
    const int ecol = div_g(min(r, rows_total - 1), P.g, P.g_magic);
    const int t = valid ? ent[ecol] : -1;
    int lim = P.causal ? min(blen, t - tok0 + 1) : blen;
    if (!valid) lim = 0;
    const int lo = P.window > 0 ? t - P.window + 1 - tok0 : 0;  // with a window, keys before lo are hidden (<= 0: none)
    // Only tiles with a row in the block itself (causal diagonal), a ragged block end or a window edge need the
    // key mask; the test is wave-uniform.  The maximum is taken over the raw scores (the scale is positive) and the scale is
    // folded into the exponent: p = 2^(s c2 - m c2).
    float m = -INFINITY;
    if (__builtin_amdgcn_ballot_w64(lim < kBlock || lo > 0) == 0) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, sacc[mb][v]);
    } else {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
          const float x = (key < lim && key >= lo) ? sacc[mb][v] : -INFINITY;
          sacc[mb][v] = x;
          m = fmaxf(m, x);
        }
    }
    m = fmaxf(m, __shfl_xor(m, 32));
    const float mc = (m == -INFINITY) ? 0.f : m * c2;  // row maximum in the log2 domain
    float l = 0.f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][v], c2, -mc));
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
      for (int db = 0; db < 4; ++db) {
        const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vbase + 32 * db * kVtStride + 16 * sp);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], oacc[db], 0, 0, 0);
      }

    // normalised partial rows -> wave tile in LDS -> coalesced 256-byte row stores
    const float inv = valid ? 1.f / l : 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w;
        w.x = pack_bf16x2(oacc[db][4 * a + 0] * inv, oacc[db][4 * a + 1] * inv);
        w.y = pack_bf16x2(oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv);
        *reinterpret_cast<uint2*>(&tile_lds[col * kTileStride + 32 * db + 8 * a + 4 * qh]) = w;
      }
    // this row's place in the partial buffers, published for the lanes that store it
    const int64_t prow = (int64_t)(e0 - pos0 + epos[ecol]) * P.g + (r - ecol * P.g);
    if (qh == 0) rowpos[col] = prow;
    wave_sync();
    // partial rows live at the list position of their entry (row = position * g + head): consecutive entries of the
    // unit give one contiguous run, broken only where a dense pair's entries were left out
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 4 * i + crow;
      if (tile * 32 + row < rows_total)
        store_streaming(opart + (size_t)rowpos[row] * kD + cchunk,
                        *reinterpret_cast<const uint4*>(&tile_lds[row * kTileStride + cchunk]));
    }
    if (valid && qh == 0) lse_part[prow] = (mc + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    wave_sync();
  };

  u32x4 qa[8];
  issue_q(wave, qa);
  for (int tile = wave; tile < n_tiles; tile += 4) do_tile(tile, qa);
}

// ---- B_K = 128 -----------------------------------------------------------------------------------------------
// Same work split, but a 128-key block does not fit the register file next to the tile state, so K_i and V_i sit
// row-major in LDS: K fragments are plain 16-byte reads, V^T fragments are LDS transpose reads (no transposed
// copy).  A tile computes S^T for all 128 keys (4 x 8 MFMA), one softmax over the 128 scores of a row, and
// O^T = V_i^T P^T (8 x 4 MFMA); one partial row and one log-sum-exp per (token, head, selected 128-block).
constexpr int kPitch128 = 152;  // bf16 per LDS row of K / V (128 + 24 pad): conflict-free operand and transpose reads
constexpr int kWaves128 = 8;    // two wavefronts per SIMD: one wave's LDS / memory waits are covered by the other
constexpr int kF128K = 0;
constexpr int kF128V = kF128K + 128 * kPitch128 * 2;
constexpr int kF128Tiles = kF128V + 128 * kPitch128 * 2;
constexpr int kF128Ent = kF128Tiles + kWaves128 * 32 * kTileStride * 2;
constexpr int kF128Epos = kF128Ent + kMaxUnit * 4;
constexpr int kF128Cnts = kF128Epos + kMaxUnit * 2;
constexpr int kF128Rowpos = kF128Cnts + (kMaxUnit / 64) * 4;
constexpr int kF128Bytes = kF128Rowpos + kWaves128 * 32 * 8;
static_assert(kF128Bytes <= 160 * 1024, "forward 128-key tile set must fit the CU's LDS");

// ds_read_b64_tr_b16: every lane passes the address of 8 bytes (four 16-bit elements); within each group of 16
// lanes, lane i receives element (i % 4) of the 8 bytes addressed by lanes 4e + i / 4, e = 0..3.
__device__ __forceinline__ bf16x4 lds_read_tr_f(const bf16_t* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)(uint32_t)(uintptr_t)p);
  return __builtin_bit_cast(bf16x4, v);
}

__global__ void __launch_bounds__(64 * kWaves128)
k_fwd_main128(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
              const int32_t* __restrict__ nu_scan, const int32_t* __restrict__ u_list,
              const int32_t* __restrict__ u_start, const int32_t* __restrict__ off,
              const int32_t* __restrict__ blk_tok0, const int32_t* __restrict__ blk_len,
              const int2* __restrict__ qent, bf16_t* __restrict__ opart,
              float* __restrict__ lse_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem + kF128K);
  bf16_t* Vs = reinterpret_cast<bf16_t*>(smem + kF128V);
  int32_t* ent = reinterpret_cast<int32_t*>(smem + kF128Ent);
  uint16_t* epos = reinterpret_cast<uint16_t*>(smem + kF128Epos);
  int32_t* cnts = reinterpret_cast<int32_t*>(smem + kF128Cnts);
  int64_t* rowpos = reinterpret_cast<int64_t*>(smem + kF128Rowpos) + 32 * (threadIdx.x >> 6);
  // units of this pass's KV heads [j0, j0 + nj); nu_scan is the exclusive scan of units per list
  const int u = nu_scan[P.j0 * P.b_cap] + blockIdx.x;
  if (u >= nu_scan[(P.j0 + P.nj) * P.b_cap]) return;
  const int L = u_list[u];
  const int j = L / P.b_cap;
  const int gb = L - j * P.b_cap;
  const int e0 = u_start[u];
  const int pos0 = off[P.j0 * P.b_cap];  // first list position of the pass: partial rows are relative to it
  const int ne_all = min(P.unit, off[L + 1] - e0);
  const int tok0 = blk_tok0[gb], blen = blk_len[gb];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int col = lane & 31, qh = lane >> 5;                 // not const: see the top of the tile loop
  int crow = lane >> 4, cchunk = (lane & 15) * 8;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  bf16_t* tile_lds = reinterpret_cast<bf16_t*>(smem + kF128Tiles) + wave * 32 * kTileStride;
  // entries of dense (tile, block) pairs belong to the dense kernel (see load_sparse_entries)
  const int ne = load_sparse_entries<64 * kWaves128>(qent, e0, ne_all, ent, epos, cnts);
  if (ne == 0) return;

  {  // K_i, V_i -> LDS, row-major (rows past the end of a ragged block are zero)
    const int key = tid >> 2, d0 = (tid & 3) * 32;
    const size_t o = ((size_t)(tok0 + key) * P.hkv + j) * kD + d0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<bf16x8*>(&Ks[key * kPitch128 + d0 + 8 * i]) =
          key < blen ? *reinterpret_cast<const bf16x8*>(K + o + 8 * i) : zero8;
      *reinterpret_cast<bf16x8*>(&Vs[key * kPitch128 + d0 + 8 * i]) =
          key < blen ? *reinterpret_cast<const bf16x8*>(V + o + 8 * i) : zero8;
    }
  }
  __syncthreads();

  const int rows_total = ne * P.g;
  const int n_tiles = (rows_total + 31) >> 5;
  if (wave >= n_tiles) return;  // no block-wide barrier below this point
  const float c2 = P.scale * 1.4426950408889634f;
  const int hbase = j * P.g;
  // this lane's share of a transposing read of four key rows x 16 channels; lane half qh = grp / 2 holds keys
  // k0 + 4 qh + {0..3} (first read) and the same + 8 (second read) of contraction step sp, k0 = 32 (sp/2) + 16 (sp&1)
  const int grp = lane >> 4, sl = lane & 15;
  int tr_v = ((sl >> 2) + 4 * (grp >> 1)) * kPitch128 + 16 * (grp & 1) + 4 * (sl & 3);

  u32x4 qc[8];
  auto issue_q = [&](int tile) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // rows past the end of the list re-read the last row: they are masked out below and never stored
      const int r = min(tile * 32 + 4 * i + crow, rows_total - 1);
      const int e = div_g(r, P.g, P.g_magic);
      // (token, head) row index in 32 bits (total_tokens * hq < 2^31 is checked on the host), widened once
      const uint32_t grow = (uint32_t)ent[e] * (uint32_t)P.hq + (uint32_t)(hbase + (r - e * P.g));
      qc[i] = *reinterpret_cast<const u32x4*>(Q + ((size_t)grow * kD + cchunk));
    }
  };
  issue_q(wave);

  for (int tile = wave; tile < n_tiles; tile += kWaves128) {
    // register budget (256 per wave): keep the lane-derived LDS addresses from being precomputed across the loop
    asm volatile("" : "+v"(col), "+v"(qh), "+v"(crow), "+v"(cchunk), "+v"(tr_v));
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4*>(&tile_lds[(4 * i + crow) * kTileStride + cchunk]) = qc[i];
    if (tile + kWaves128 < n_tiles) issue_q(tile + kWaves128);  // next rows fly during this tile's compute
    wave_sync();
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
      qf[s] = *reinterpret_cast<const bf16x8*>(&tile_lds[col * kTileStride + 16 * s + 8 * qh]);

    f32x16 sacc[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[mb][v] = 0.f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[(32 * mb + col) * kPitch128 + 16 * s + 8 * qh]);
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[mb], 0, 0, 0);
      }

    const int r = tile * 32 + col;
    const bool valid = r < rows_total;
    const int ecol = div_g(min(r, rows_total - 1), P.g, P.g_magic);
    const int t = valid ? ent[ecol] : -1;
    int lim = P.causal ? min(blen, t - tok0 + 1) : blen;
    if (!valid) lim = 0;
    const int lo = P.window > 0 ? t - P.window + 1 - tok0 : 0;  // with a window, keys before lo are hidden
    // key mask only where a row lies in the block itself, the block is ragged or a window edge falls into it (wave-uniform test); maximum over
    // the raw scores, scale folded into the exponent
    float m = -INFINITY;
    if (__builtin_amdgcn_ballot_w64(lim < 2 * kBlock || lo > 0) == 0) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, sacc[mb][v]);
    } else {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
          const float x = (key < lim && key >= lo) ? sacc[mb][v] : -INFINITY;
          sacc[mb][v] = x;
          m = fmaxf(m, x);
        }
    }
    m = fmaxf(m, __shfl_xor(m, 32));
    const float mc = (m == -INFINITY) ? 0.f : m * c2;  // row maximum in the log2 domain
    float l = 0.f;
    bf16x8 pf[8];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][v], c2, -mc));
        l += p;
        pf[2 * mb + (v >> 3)][v & 7] = (bf16_t)p;
      }
    l += __shfl_xor(l, 32);

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
#pragma unroll
    for (int sp = 0; sp < 8; ++sp) {
      const int k0 = 32 * (sp >> 1) + 16 * (sp & 1);
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x4 a0 = lds_read_tr_f(&Vs[k0 * kPitch128 + tr_v + 32 * db]);
        const bf16x4 a1 = lds_read_tr_f(&Vs[(k0 + 8) * kPitch128 + tr_v + 32 * db]);
        const bf16x8 vf = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], oacc[db], 0, 0, 0);
      }
    }

    const float inv = valid ? 1.f / l : 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w;
        w.x = pack_bf16x2(oacc[db][4 * a + 0] * inv, oacc[db][4 * a + 1] * inv);
        w.y = pack_bf16x2(oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv);
        *reinterpret_cast<uint2*>(&tile_lds[col * kTileStride + 32 * db + 8 * a + 4 * qh]) = w;
      }
    // this row's place in the partial buffers, published for the lanes that store it
    const int64_t prow = (int64_t)(e0 - pos0 + epos[ecol]) * P.g + (r - ecol * P.g);
    if (qh == 0) rowpos[col] = prow;
    wave_sync();
    // partial rows live at the list position of their entry (see k_fwd_main)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 4 * i + crow;
      if (tile * 32 + row < rows_total)
        store_streaming(opart + (size_t)rowpos[row] * kD + cchunk,
                        *reinterpret_cast<const uint4*>(&tile_lds[row * kTileStride + cchunk]));
    }
    if (valid && qh == 0) lse_part[prow] = (mc + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    wave_sync();
  }
}


// ---- dense (query-tile-outer) forward, fused with the merge ---------------------------------------------------------
// The (query tile, KV block) pairs the index marked dense - blocks that at least half of the tile's 64 tokens keep:
// the attention-sink block and the tokens' own and neighbouring blocks (App. E, the paragraph on the attention sink;
// the whole band of the sliding-window term of Eq. (2)) - are contiguous token ranges on both sides, so they need no
// gather and no partial row in memory at all.  One workgroup takes 128 rows (row = (token of the tile, head of the
// group)) of one (tile, kv head):
//   phase 1  keeps the rows' Q fragments in registers and walks the tile's dense blocks, 64 keys at a time (the index
//            lists them as pieces) through LDS, with a running (max, sum) per row and the output accumulated in
//            registers across the pieces.  The 64-bit mask of a piece says which tokens of the tile keep its block;
//            the others see none of its keys.  S^T = K Q^T and O^T = V^T P^T as in the kernels above (K fragments
//            are 16-byte LDS reads, V^T fragments LDS transpose reads); the next piece is fetched into registers while
//            the current one computes.  The result, normalised, goes to a wave-private LDS tile with its log-sum-exp.
//   phase 2  is the reduction step of Sec. 3.2 for the same rows: 16 lanes per row gather the partial rows the gather
//            route left for the row's other kept columns (two rows and eight columns at a time per lane: the few
//            wavefronts of this kernel need that many loads in flight) and combine them, together with the row of
//            phase 1, by their log-sum-exps; O, LSE and the optional gated sum of Eq. (2) are written once.  The
//            rows' kept-column masks and slot positions are fetched at the very start of the kernel and parked in
//            the wave's LDS tile (free between the Q staging and the end), so that phase 2 starts with its addresses
//            known and the only memory latency left in it is that of the gathers themselves.
// Tiles without a dense piece skip phase 1, so with the dense route on this kernel is the merge of every row.
constexpr int kDnPitch = 152;                                  // bf16 per LDS row of the K / V tiles
constexpr int kDnK = 0;
constexpr int kDnV = kDnK + 64 * kDnPitch * 2;
constexpr int kDnTiles = kDnV + 64 * kDnPitch * 2;
constexpr int kDnLse = kDnTiles + 4 * 32 * kTileStride * 2;
constexpr int kDnBytes = kDnLse + 4 * 32 * 4;                  // 74240: two workgroups per CU
static_assert(4 * 32 * kTileStride * 2 <= kDnTiles, "phase 1's result must fit the K / V area");
static_assert((kMaxTopk + 2) * 32 * 4 <= 32 * kTileStride * 2, "a wavefront's index data must fit its LDS tile");
constexpr int kMergeBatch = 8;                                 // columns of a row gathered at a time in phase 2
static_assert(2 * kDnBytes <= 160 * 1024, "two workgroups of the dense forward must fit one CU's LDS");

__global__ void __launch_bounds__(256, 2)
k_fwd_dense_merge(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                  const int32_t* __restrict__ tile_tok0, const int32_t* __restrict__ tile_len,
                  const int32_t* __restrict__ d_cnt, const int2* __restrict__ d_piece,
                  const unsigned long long* __restrict__ d_mask, const bf16_t* __restrict__ opart,
                  const float* __restrict__ lse_part, const uint32_t* __restrict__ vmask,
                  const uint32_t* __restrict__ dmask, const int32_t* __restrict__ slotpos,
                  const int32_t* __restrict__ off, bf16_t* __restrict__ O, float* __restrict__ LSE,
                  const float* __restrict__ gate, const bf16_t* Oacc, bf16_t* Oout) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem + kDnK);
  bf16_t* Vs = reinterpret_cast<bf16_t*>(smem + kDnV);
  const int chunks = (kTileTokens * P.g + 127) >> 7;  // 128-row chunks of a tile's rows
  // Workgroups are handed to the chip's 8 XCDs (each with its own L2) round-robin by their index; the work is
  // ordered kv head -> tile -> chunk, and every XCD takes one contiguous eighth of that order, so that the
  // workgroups running side by side on an XCD share K / V pieces (neighbouring tiles of one head, the sink block).
  const int total = P.nj * P.t_cap * chunks, per = (total + 7) >> 3;
  const int lid = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if (lid >= total) return;
  const int chunk = lid % chunks, qt = (lid / chunks) % P.t_cap;
  const int j = P.j0 + lid / (chunks * P.t_cap);
  const size_t slot = (size_t)qt * P.hkv + j;
  // everything the prologue needs from the tables is requested at once (the first piece's slot exists even when the
  // tile has no dense piece)
  const int nd = d_cnt[slot];
  const int tlen = tile_len[qt];
  const int ttok0 = tile_tok0[qt];
  const int2 piece0 = d_piece[slot * kDenseMax];
  const int rows_total = tlen * P.g;
  if (chunk * 128 >= rows_total) return;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, qh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: what derives from it stays out of the VGPRs
  const int crow = lane >> 4, cchunk = (lane & 15) * 8;
  bf16_t* tile_lds = reinterpret_cast<bf16_t*>(smem + kDnTiles) + wave * 32 * kTileStride;
  float* lse_lds = reinterpret_cast<float*>(smem + kDnLse) + wave * 32;
  bf16_t* od_lds = Ks + wave * 32 * kTileStride;   // phase 1's result for phase 2 (the K / V area after the last piece)
  const int row0 = chunk * 128 + wave * 32;        // first row of this wavefront
  const bool wave_on = row0 < rows_total;          // idle wavefronts still help to stage K / V
  const int hbase = j * P.g;

  // Phase 2's index data for this wavefront's tokens: per token (kept columns, dense columns, slot positions).
  // Requested now (up to 4 words per lane in registers, the rest - many tokens per wave, long rows - later), stored to
  // the wave's LDS tile once the Q fragments have left it.
  const int e_lo = div_g(min(row0, rows_total - 1), P.g, P.g_magic);
  const int e_hi = div_g(min(row0 + 31, rows_total - 1), P.g, P.g_magic);
  const int mstride = P.topk + 2;
  const int mwords = wave_on ? (e_hi - e_lo + 1) * mstride : 0;
  int32_t* meta = reinterpret_cast<int32_t*>(tile_lds);
  auto meta_word = [&](int i) -> int32_t {
    const int tk = i / mstride, c = i - tk * mstride;
    const size_t tj = (size_t)(ttok0 + e_lo + tk) * P.hkv + j;
    return c == 0 ? (int32_t)vmask[tj] : c == 1 ? (int32_t)dmask[tj] : slotpos[tj * P.topk + (c - 2)];
  };
  int32_t mreg[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) mreg[q] = lane + 64 * q < mwords ? meta_word(lane + 64 * q) : 0;
  auto park_meta = [&]() {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (lane + 64 * q < mwords) meta[lane + 64 * q] = mreg[q];
    for (int i = lane + 256; i < mwords; i += 64) meta[i] = meta_word(i);
    wave_sync();
  };

  if (nd > 0) {  // ---------------------------------------------------------------------------------- phase 1
    const float c2 = P.scale * 1.4426950408889634f;
    // staging of 64 keys: thread = (key, 32 channels), four 16-byte pieces of K and of V
    const int skey = tid >> 2, sd0 = (tid & 3) * 32;
    u32x4 kreg[4], vreg[4];
    auto fetch = [&](int2 piece) {  // (first key, number of keys)
      const bool on = skey < piece.y;
      const size_t o = ((size_t)(piece.x + (on ? skey : 0)) * P.hkv + j) * kD + sd0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        kreg[i] = *reinterpret_cast<const u32x4*>(K + o + 8 * i);
        vreg[i] = *reinterpret_cast<const u32x4*>(V + o + 8 * i);
        if (!on) {  // rows past the end of a ragged block are zero
          kreg[i] = u32x4{0, 0, 0, 0};
          vreg[i] = u32x4{0, 0, 0, 0};
        }
      }
    };
    // this wavefront's 32 rows of Q (coalesced loads) and the first piece are requested together
    u32x4 qc[8];
    if (wave_on) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = min(row0 + 4 * i + crow, rows_total - 1);
        const int e = div_g(r, P.g, P.g_magic);
        const uint32_t grow = (uint32_t)(ttok0 + e) * (uint32_t)P.hq + (uint32_t)(hbase + (r - e * P.g));
        qc[i] = *reinterpret_cast<const u32x4*>(Q + ((size_t)grow * kD + cchunk));
      }
    }
    fetch(piece0);
    // Q rows -> wave tile -> B-operand fragments, kept for the whole tile
    bf16x8 qf[8];
    if (wave_on) {
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(&tile_lds[(4 * i + crow) * kTileStride + cchunk]) = qc[i];
      wave_sync();
#pragma unroll
      for (int s = 0; s < 8; ++s)
        qf[s] = *reinterpret_cast<const bf16x8*>(&tile_lds[col * kTileStride + 16 * s + 8 * qh]);
      wave_sync();
      park_meta();  // the tile is free until phase 2
    }
    const int r = row0 + col;                        // this lane's row
    const bool valid = r < rows_total;
    const int e_row = div_g(min(r, rows_total - 1), P.g, P.g_magic);
    const int t = ttok0 + e_row;

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;            // running maximum (raw scores) and sum of the row
    const int grp = lane >> 4, sl = lane & 15;
    const int tr_v = ((sl >> 2) + 4 * (grp >> 1)) * kDnPitch + 16 * (grp & 1) + 4 * (sl & 3);

    for (int step = 0; step < nd; ++step) {
      __syncthreads();  // the previous piece is no longer read
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4*>(&Ks[skey * kDnPitch + sd0 + 8 * i]) = kreg[i];
        *reinterpret_cast<u32x4*>(&Vs[skey * kDnPitch + sd0 + 8 * i]) = vreg[i];
      }
      const int2 piece = d_piece[slot * kDenseMax + step];
      const unsigned long long members = d_mask[slot * kDenseMax + step];
      const int ktok0 = piece.x, klen = piece.y;                // first key of the piece and its number of keys
      if (step + 1 < nd) fetch(d_piece[slot * kDenseMax + step + 1]);  // flies during the compute
      __syncthreads();  // K, V of the piece staged
      if (!wave_on) continue;

      f32x16 sacc[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[mb][v] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[(32 * mb + col) * kDnPitch + 16 * s + 8 * qh]);
          sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[mb], 0, 0, 0);
        }
      // keys [lo, lim) of the piece are visible to this row: none if the token does not keep the block
      int lim = P.causal ? min(klen, t - ktok0 + 1) : klen;
      if (!valid || !((members >> e_row) & 1ull)) lim = 0;
      const int lo = P.window > 0 ? t - P.window + 1 - ktok0 : 0;
      float m = -INFINITY;
      if (__builtin_amdgcn_ballot_w64(lim < 64 || lo > 0) == 0) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int v = 0; v < 16; ++v) m = fmaxf(m, sacc[mb][v]);
      } else {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = 32 * mb + 8 * (v >> 2) + 4 * qh + (v & 3);
            const float x = (key < lim && key >= lo) ? sacc[mb][v] : -INFINITY;
            sacc[mb][v] = x;
            m = fmaxf(m, x);
          }
      }
      m = fmaxf(m, __shfl_xor(m, 32));
      // online softmax: new running maximum, rescale of what has been accumulated
      const float m_new = fmaxf(m_run, m);
      const float mc = (m_new == -INFINITY) ? 0.f : m_new * c2;
      const float alpha = __builtin_amdgcn_exp2f(fmaf(m_run, c2, -mc));  // exp2(-inf) = 0 on the first visible piece
      m_run = m_new;
      float l = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][v], c2, -mc));
          sacc[mb][v] = p;
          l += p;
        }
      l += __shfl_xor(l, 32);
      l_run = l_run * alpha + l;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;

      bf16x8 pf[4];
#pragma unroll
      for (int sp = 0; sp < 4; ++sp)
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) pf[sp][e2] = (bf16_t)sacc[sp >> 1][8 * (sp & 1) + e2];
#pragma unroll
      for (int sp = 0; sp < 4; ++sp)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const bf16x4 a0 = lds_read_tr_f(&Vs[16 * sp * kDnPitch + tr_v + 32 * db]);
          const bf16x4 a1 = lds_read_tr_f(&Vs[(16 * sp + 8) * kDnPitch + tr_v + 32 * db]);
          const bf16x8 vf = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], oacc[db], 0, 0, 0);
        }
    }
    __syncthreads();  // every wavefront is done with the last piece: the K / V area is free
    if (!wave_on) return;
    // the rows' dense result, normalised, and its log-sum-exp (natural log; -inf for a row that keeps none of the
    // tile's dense blocks) -> this wavefront's quarter of the K / V area, where phase 2 picks them up in its own
    // lane layout
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w;
        w.x = pack_bf16x2(oacc[db][4 * a + 0] * inv, oacc[db][4 * a + 1] * inv);
        w.y = pack_bf16x2(oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv);
        *reinterpret_cast<uint2*>(&od_lds[col * kTileStride + 32 * db + 8 * a + 4 * qh]) = w;
      }
    if (qh == 0) {
      const float mcf = (m_run == -INFINITY) ? 0.f : m_run * c2;
      lse_lds[col] = l_run > 0.f ? (mcf + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
    }
    wave_sync();
  }
  if (!wave_on) return;

  // ------------------------------------------------------------------------------------------------ phase 2
  if (nd == 0) park_meta();
  // lane-derived indices of this phase, recomputed here so that they do not occupy registers during phase 1
  int lane_b = threadIdx.x & 63;
  asm volatile("" : "+v"(lane_b));
  const int sub = lane_b & 15, crow_b = lane_b >> 4;
  const int pos0 = off[P.j0 * P.b_cap];  // first list position of the pass: partial rows are relative to it
  for (int pass = 0; pass < 4; ++pass) {
    // two rows per lane group: wave rows 4 pass + crow and 16 more
    bool ok[2];
    int hh[2];
    int64_t grow[2];
    uint32_t vm_all[2], vm[2];
    const int32_t* sp[2];  // the row's slot positions (LDS)
    float acc[2][8], M[2], Ls[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int wrow = 4 * pass + crow_b + 16 * x;
      const int rr = row0 + wrow;
      ok[x] = rr < rows_total;
      const int rc = min(rr, rows_total - 1);
      const int e = div_g(rc, P.g, P.g_magic);
      hh[x] = rc - e * P.g;
      grow[x] = (int64_t)(ttok0 + e) * P.hq + hbase + hh[x];
      const int32_t* mrow = meta + (e - e_lo) * mstride;
      vm_all[x] = ok[x] ? (uint32_t)mrow[0] : 0u;
      const uint32_t dm = ok[x] ? (uint32_t)mrow[1] : 0u;
      vm[x] = vm_all[x] & ~dm;
      sp[x] = mrow + 2;
      M[x] = -INFINITY;
      Ls[x] = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[x][c] = 0.f;
      if (dm != 0u && nd > 0) {  // the row of phase 1 starts the sum
        const float ls = lse_lds[wrow];
        if (ls > -INFINITY) {
          const uint4 v = *reinterpret_cast<const uint4*>(&od_lds[wrow * kTileStride + 8 * sub]);
          M[x] = ls;
          Ls[x] = 1.f;
          acc[x][0] = bf16_lo(v.x); acc[x][1] = bf16_hi(v.x); acc[x][2] = bf16_lo(v.y); acc[x][3] = bf16_hi(v.y);
          acc[x][4] = bf16_lo(v.z); acc[x][5] = bf16_hi(v.z); acc[x][6] = bf16_lo(v.w); acc[x][7] = bf16_hi(v.w);
        }
      }
    }
    for (int m0 = 0; m0 < P.topk; m0 += kMergeBatch) {
      if (((vm[0] | vm[1]) >> m0) == 0u) break;  // no kept column left in either row
      uint4 xv[2][kMergeBatch];
      float ls[2][kMergeBatch];
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int i = 0; i < kMergeBatch; ++i) {
          const int m = m0 + i;
          const bool on = m < P.topk && ((vm[x] >> m) & 1u);
          const size_t pr = on ? (size_t)(sp[x][m] - pos0) * P.g + hh[x] : (size_t)0;
          xv[x][i] = on ? *reinterpret_cast<const uint4*>(opart + pr * kD + 8 * sub) : make_uint4(0, 0, 0, 0);
          ls[x][i] = on ? lse_part[pr] : -INFINITY;
        }
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        float Mb = M[x];
#pragma unroll
        for (int i = 0; i < kMergeBatch; ++i) Mb = fmaxf(Mb, ls[x][i]);
        if (Mb == -INFINITY) continue;  // no kept column in this batch or before it
        const float rescale = __expf(M[x] - Mb);  // 0 on the first non-empty batch
        Ls[x] *= rescale;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[x][c] *= rescale;
        M[x] = Mb;
#pragma unroll
        for (int i = 0; i < kMergeBatch; ++i) {
          const float w = __expf(ls[x][i] - Mb);  // exp(-inf) = 0 for columns that are off
          Ls[x] += w;
          acc[x][0] += w * bf16_lo(xv[x][i].x); acc[x][1] += w * bf16_hi(xv[x][i].x);
          acc[x][2] += w * bf16_lo(xv[x][i].y); acc[x][3] += w * bf16_hi(xv[x][i].y);
          acc[x][4] += w * bf16_lo(xv[x][i].z); acc[x][5] += w * bf16_hi(xv[x][i].z);
          acc[x][6] += w * bf16_lo(xv[x][i].w); acc[x][7] += w * bf16_hi(xv[x][i].w);
        }
      }
    }
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      if (!ok[x]) continue;
      bf16_t* orow = O + grow[x] * kD + 8 * sub;
      if (vm_all[x] == 0u) {  // nothing visible: O = 0, LSE = -inf, and the gated sum is what the other branches gave
        *reinterpret_cast<uint4*>(orow) = make_uint4(0, 0, 0, 0);
        if (sub == 0) LSE[grow[x]] = -INFINITY;
        if (gate != nullptr)
          *reinterpret_cast<uint4*>(Oout + grow[x] * kD + 8 * sub) =
              Oacc != nullptr ? *reinterpret_cast<const uint4*>(Oacc + grow[x] * kD + 8 * sub) : make_uint4(0, 0, 0, 0);
        continue;
      }
      const float inv = 1.f / Ls[x];
      uint4 o;
      o.x = pack_bf16x2(acc[x][0] * inv, acc[x][1] * inv);
      o.y = pack_bf16x2(acc[x][2] * inv, acc[x][3] * inv);
      o.z = pack_bf16x2(acc[x][4] * inv, acc[x][5] * inv);
      o.w = pack_bf16x2(acc[x][6] * inv, acc[x][7] * inv);
      *reinterpret_cast<uint4*>(orow) = o;
      if (sub == 0) LSE[grow[x]] = M[x] + __logf(Ls[x]);
      if (gate != nullptr) {
        // Eq. (2): O_out = O_acc + gate * O, from the fp32 result (Oout may be the buffer Oacc points to: every lane
        // reads its own 16 bytes before it writes them)
        const float tau = gate[grow[x]] * inv;
        uint4 a = make_uint4(0, 0, 0, 0);
        if (Oacc != nullptr) a = *reinterpret_cast<const uint4*>(Oacc + grow[x] * kD + 8 * sub);
        o.x = pack_bf16x2(bf16_lo(a.x) + tau * acc[x][0], bf16_hi(a.x) + tau * acc[x][1]);
        o.y = pack_bf16x2(bf16_lo(a.y) + tau * acc[x][2], bf16_hi(a.y) + tau * acc[x][3]);
        o.z = pack_bf16x2(bf16_lo(a.z) + tau * acc[x][4], bf16_hi(a.z) + tau * acc[x][5]);
        o.w = pack_bf16x2(bf16_lo(a.w) + tau * acc[x][6], bf16_hi(a.w) + tau * acc[x][7]);
        *reinterpret_cast<uint4*>(Oout + grow[x] * kD + 8 * sub) = o;
      }
    }
  }
}

// 16 lanes per (token, head) row, 8 output channels per lane.  Slots are taken kSlotBatch at a time: positions,
// partial log-sum-exps and partial rows of a batch are all requested before any of them is used; batches are chained
// by the usual running-max rescale.  Small batches keep the register count low, and the many resident waves that
// result hide the gather latency better than long batches did (16 -> 4: 1.87 -> 1.80 ms at the headline shape).
__global__ void __launch_bounds__(256)
k_fwd_merge(Problem P, const bf16_t* __restrict__ opart, const float* __restrict__ lse_part,
            const uint32_t* __restrict__ vmask, const int32_t* __restrict__ slotpos,
            const int32_t* __restrict__ off, bf16_t* __restrict__ O,
            float* __restrict__ LSE, const float* __restrict__ gate, const bf16_t* Oacc, bf16_t* Oout) {
  // rows of the pass: (token, head of the KV heads [j0, j0 + nj))
  const int hp = P.nj * P.g;
  const int64_t prow = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  if (prow >= (int64_t)P.T * hp) return;
  const int t = (int)(prow / hp);
  const int h = P.j0 * P.g + (int)(prow - (int64_t)t * hp);
  const int64_t row = (int64_t)t * P.hq + h;
  const int j = h / P.g, hh = h - j * P.g;
  const int pos0 = off[P.j0 * P.b_cap];
  const uint32_t vm = vmask[(size_t)t * P.hkv + j];
  bf16_t* orow = O + row * kD + 8 * sub;
  if (vm == 0u) {
    *reinterpret_cast<uint4*>(orow) = make_uint4(0, 0, 0, 0);
    if (sub == 0) LSE[row] = -INFINITY;
    if (gate != nullptr)  // nothing to add: the gated sum is what the other branches gave
      *reinterpret_cast<uint4*>(Oout + row * kD + 8 * sub) =
          Oacc != nullptr ? *reinterpret_cast<const uint4*>(Oacc + row * kD + 8 * sub) : make_uint4(0, 0, 0, 0);
    return;
  }
  const int32_t* sp = slotpos + ((size_t)t * P.hkv + j) * P.topk;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  float M = -INFINITY, Ls = 0.f;
  for (int m0 = 0; m0 < P.topk; m0 += kSlotBatch) {
    size_t pr[kSlotBatch];
    uint4 x[kSlotBatch];
    float ls[kSlotBatch];
#pragma unroll
    for (int i = 0; i < kSlotBatch; ++i) {
      const int m = m0 + i;
      const bool on = m < P.topk && ((vm >> m) & 1u);
      pr[i] = on ? (size_t)(sp[m] - pos0) * P.g + hh : (size_t)0;
    }
#pragma unroll
    for (int i = 0; i < kSlotBatch; ++i) {
      const int m = m0 + i;
      const bool on = m < P.topk && ((vm >> m) & 1u);
      x[i] = on ? *reinterpret_cast<const uint4*>(opart + pr[i] * kD + 8 * sub) : make_uint4(0, 0, 0, 0);
      ls[i] = on ? lse_part[pr[i]] : -INFINITY;
    }
    float Mb = M;
#pragma unroll
    for (int i = 0; i < kSlotBatch; ++i) Mb = fmaxf(Mb, ls[i]);
    if (Mb == -INFINITY) continue;  // no kept slot in this batch or before it
    const float rescale = __expf(M - Mb);  // 0 on the first non-empty batch
    Ls *= rescale;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] *= rescale;
    M = Mb;
#pragma unroll
    for (int i = 0; i < kSlotBatch; ++i) {
      const float w = __expf(ls[i] - M);  // exp(-inf) = 0 for slots that are off
      Ls += w;
      acc[0] += w * bf16_lo(x[i].x); acc[1] += w * bf16_hi(x[i].x);
      acc[2] += w * bf16_lo(x[i].y); acc[3] += w * bf16_hi(x[i].y);
      acc[4] += w * bf16_lo(x[i].z); acc[5] += w * bf16_hi(x[i].z);
      acc[6] += w * bf16_lo(x[i].w); acc[7] += w * bf16_hi(x[i].w);
    }
  }
  const float inv = 1.f / Ls;
  uint4 o;
  o.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
  o.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
  o.z = pack_bf16x2(acc[4] * inv, acc[5] * inv);
  o.w = pack_bf16x2(acc[6] * inv, acc[7] * inv);
  *reinterpret_cast<uint4*>(orow) = o;
  if (sub == 0) LSE[row] = M + __logf(Ls);
  if (gate != nullptr) {
    // Eq. (2): O_out = O_acc + gate * O, from the fp32 result (Oout may be the buffer Oacc points to: every lane
    // reads its own 16 bytes before it writes them)
    const float tau = gate[row] * inv;
    uint4 a = make_uint4(0, 0, 0, 0);
    if (Oacc != nullptr) a = *reinterpret_cast<const uint4*>(Oacc + row * kD + 8 * sub);
    o.x = pack_bf16x2(bf16_lo(a.x) + tau * acc[0], bf16_hi(a.x) + tau * acc[1]);
    o.y = pack_bf16x2(bf16_lo(a.y) + tau * acc[2], bf16_hi(a.y) + tau * acc[3]);
    o.z = pack_bf16x2(bf16_lo(a.z) + tau * acc[4], bf16_hi(a.z) + tau * acc[5]);
    o.w = pack_bf16x2(bf16_lo(a.w) + tau * acc[6], bf16_hi(a.w) + tau * acc[7]);
    *reinterpret_cast<uint4*>(Oout + row * kD + 8 * sub) = o;
  }
}

hipError_t launch_fwd(const Problem& P0, const IndexLayout& L, int heads_per_pass, const void* Q, const void* K,
                      const void* V, const void* index_ws, void* opart, float* lse_part, void* O, float* LSE,
                      const GateArgs& G, hipStream_t st) {
  IndexPtrs p = index_ptrs(L, const_cast<void*>(index_ws));
  if (P0.dense) {
    static std::atomic<uint64_t> ready_dense;
    hipError_t e = allow_dynamic_lds((const void*)k_fwd_dense_merge, kDnBytes, ready_dense);
    if (e != hipSuccess) return e;
  }
  {
    static std::atomic<uint64_t> ready[2];
    hipError_t e = P0.bk == 128 ? allow_dynamic_lds((const void*)k_fwd_main128, kF128Bytes, ready[1])
                                : allow_dynamic_lds((const void*)k_fwd_main, kF64Bytes, ready[0]);
    if (e != hipSuccess) return e;
  }
  // KV heads are processed heads_per_pass at a time; every pass reuses the same partial buffers (the lists of
  // one KV head are contiguous in list-position order, so a pass owns a contiguous range of positions).
  for (int j0 = 0; j0 < P0.hkv; j0 += heads_per_pass) {
    Problem P = P0;
    P.j0 = j0;
    P.nj = min(heads_per_pass, P0.hkv - j0);
    // upper bound of the work units of the pass (the real count is only known on the device)
    const unsigned units_max = (unsigned)units_bound(P.nj, P.b_cap, P.T, P.topk, P.unit);
    if (P.bk == 128) {
      ProfScope ps(KID_FWD_MAIN, st);
      hipLaunchKernelGGL(k_fwd_main128, dim3(units_max), dim3(64 * kWaves128), kF128Bytes, st, P, (const bf16_t*)Q,
                         (const bf16_t*)K, (const bf16_t*)V, p.u_nu, p.u_list, p.u_start, p.off, p.blk_tok0,
                         p.blk_len, p.qent, (bf16_t*)opart, lse_part);
    } else {
      ProfScope ps(KID_FWD_MAIN, st);
      hipLaunchKernelGGL(k_fwd_main, dim3(units_max), dim3(256), kF64Bytes, st, P, (const bf16_t*)Q, (const bf16_t*)K,
                         (const bf16_t*)V, p.u_nu, p.u_list, p.u_start, p.off, p.blk_tok0, p.blk_len, p.qent,
                         (bf16_t*)opart, lse_part);
    }
    if (P.dense) {
      // dense pairs and the reduction step in one kernel (every row of the pass's heads)
      const int chunks = (kTileTokens * P.g + 127) / 128;
      const int per = (P.nj * P.t_cap * chunks + 7) / 8;
      ProfScope ps(KID_FWD_DENSE, st);
      hipLaunchKernelGGL(k_fwd_dense_merge, dim3((unsigned)(8 * per)), dim3(256), kDnBytes, st, P, (const bf16_t*)Q,
                         (const bf16_t*)K, (const bf16_t*)V, p.tile_tok0, p.tile_len, p.d_cnt, p.d_piece, p.d_mask,
                         (const bf16_t*)opart, (const float*)lse_part, p.vmask, p.dmask, p.slotpos, p.off, (bf16_t*)O,
                         LSE, G.gate, (const bf16_t*)G.o_acc, (bf16_t*)G.o_out);
    } else {
      const int64_t rows = (int64_t)P.T * P.nj * P.g;
      ProfScope ps(KID_FWD_MERGE, st);
      hipLaunchKernelGGL(k_fwd_merge, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, P, (const bf16_t*)opart,
                         (const float*)lse_part, p.vmask, p.slotpos, p.off, (bf16_t*)O, LSE, G.gate,
                         (const bf16_t*)G.o_acc, (bf16_t*)G.o_out);
    }
  }
  return hipGetLastError();
}

}  // namespace nsa
