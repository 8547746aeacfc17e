// Index inversion for selected-block attention: from the selection table idx[token, kv head, column] build, for
// every (kv head, KV block), the ascending list of query tokens that select it (the paper's index tensor I_i,
// Sec. 3.2, the paragraph on the token-selection kernel) together with the column each entry came from, and, per kept
// (token, kv head, column), the entry's position in its list, which is where its partial result lives in the
// compact partial buffers (the role of the paper's O_i), plus the work-unit tables of the attention kernels.
// Pipeline: per-(kv head, token chunk, block) histogram -> prefix over the chunks of every list -> exclusive scan
// of the list lengths -> ordered scatter.  The counters are stored chunk-major, [kv head][chunk][block], so that
// the histogram and the scatter of one (chunk, kv head) touch one contiguous row.
// The scatter is deterministic: a chunk is walked by one wavefront in rounds of 64 tokens, and a token's rank
// inside a round is a popcount over a 64-bit membership mask, so no ordering depends on atomics.
#include "common.h"

namespace nsa {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;  // 4096

// ------------------------------------------------------------------------------------------------ prep
// blk_base[s] = number of blocks (of bk = B_K tokens) of sequences < s; per global block its first token and its
// key count.
__global__ void k_prep(const int32_t* __restrict__ cu, int nseq, int T, int bk, int b_cap,
                       int32_t* __restrict__ blk_base,
                       int32_t* __restrict__ blk_tok0, int32_t* __restrict__ blk_len, int32_t* __restrict__ hdr_slot) {
  __shared__ int s_btot;
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int s = 0; s < nseq; ++s) {
      int c0 = cu ? cu[s] : 0, c1 = cu ? cu[s + 1] : T;
      blk_base[s] = acc;
      acc += (c1 - c0 + bk - 1) / bk;
    }
    blk_base[nseq] = acc;
    s_btot = acc;
    *hdr_slot = acc;
  }
  __threadfence_block();
  __syncthreads();
  const int b_tot = s_btot;
  for (int gb = threadIdx.x; gb < b_cap; gb += blockDim.x) {
    int tok0 = 0, len = 0;
    if (gb < b_tot) {
      int lo = 0, hi = nseq;  // blk_base[lo] <= gb < blk_base[hi]
      while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blk_base[mid] <= gb) lo = mid; else hi = mid;
      }
      int c0 = cu ? cu[lo] : 0, c1 = cu ? cu[lo + 1] : T;
      tok0 = c0 + (gb - blk_base[lo]) * bk;
      len = min(bk, c1 - tok0);
    }
    blk_tok0[gb] = tok0;
    blk_len[gb] = len;
  }
}

// Bit m of the result is set when column m of the row is a kept selection: in range for the sequence, not in
// the token's future when causal, not wholly before the token's window (first_blk = the block of the oldest
// visible key, 0 without a window), and not a repeat of an earlier column.
__device__ __forceinline__ uint32_t kept_columns(const int32_t* row, int k, int b_s, int cur, int causal,
                                                 int first_blk) {
  uint32_t vm = 0;
  for (int m = 0; m < k; ++m) {
    int x = row[m];
    const bool ok = x >= first_blk && x < b_s && (!causal || x <= cur);
    bool dup = false;  // no early exit: the reads of the earlier columns are independent and overlap
    for (int mp = 0; mp < m; ++mp) dup |= row[mp] == x;
    if (ok && !dup) vm |= 1u << m;
  }
  return vm;
}

// Window of global blocks a token chunk can touch: the blocks of the sequences it overlaps, and under the
// causal rule none past the block of the chunk's last token.
__device__ __forceinline__ void chunk_window(const int32_t* cu, const int32_t* blk_base, int nseq, int T, int t0,
                                             int t1, int bk, int causal, int& gb_lo, int& gb_hi) {
  int s0, s1, a, b, c0;
  seq_bounds(cu, nseq, T, t0, s0, a, b);
  seq_bounds(cu, nseq, T, t1 - 1, s1, c0, b);
  gb_lo = blk_base[s0];
  gb_hi = blk_base[s1 + 1];
  if (causal) gb_hi = min(gb_hi, blk_base[s1] + (t1 - 1 - c0) / bk + 1);
}

// ------------------------------------------------------------------------------------------------ histogram
// grid (n_chunks, hkv), 256 threads.  counters[(j*n_chunks + chunk)*b_cap + gb] = number of tokens of the
// chunk that keep block gb for kv head j; the whole row is written (zeros outside the chunk's window), so the
// array needs no clearing.  Dynamic LDS: b_cap ints + 256*(k+1) ints.
__global__ void __launch_bounds__(256) k_hist(const int32_t* __restrict__ idx, const int32_t* __restrict__ cu,
                                              const int32_t* __restrict__ blk_base, int nseq, int T, int hkv, int k,
                                              int bk, int causal, int window, int b_cap, int n_chunks,
                                              int32_t* __restrict__ counters, uint32_t* __restrict__ vmask) {
  extern __shared__ int32_t lds[];
  int32_t* hist = lds;
  int32_t* rows = lds + b_cap;
  const int chunk = blockIdx.x, j = blockIdx.y;
  const int t0 = chunk * kChunkTokens, t1 = min(t0 + kChunkTokens, T);
  int gb_lo, gb_hi;
  chunk_window(cu, blk_base, nseq, T, t0, t1, bk, causal, gb_lo, gb_hi);
  const int win = gb_hi - gb_lo;
  for (int i = threadIdx.x; i < win; i += blockDim.x) hist[i] = 0;
  __syncthreads();
  int32_t* row = rows + threadIdx.x * (k + 1);
  for (int t = t0 + threadIdx.x; t < t1; t += blockDim.x) {
    int s, c0, c1;
    seq_bounds(cu, nseq, T, t, s, c0, c1);
    const int32_t* src = idx + ((size_t)t * hkv + j) * k;
    for (int m = 0; m < k; ++m) row[m] = src[m];
    const int b_s = (c1 - c0 + bk - 1) / bk;
    const int cur = (t - c0) / bk;
    // oldest key a window of `window` tokens shows to this token: position p - window + 1 of its sequence
    const int first_blk = window > 0 ? max(t - c0 - window + 1, 0) / bk : 0;
    const uint32_t vm = kept_columns(row, k, b_s, cur, causal, first_blk);
    vmask[(size_t)t * hkv + j] = vm;
    const int base = blk_base[s] - gb_lo;
    for (int m = 0; m < k; ++m)
      if ((vm >> m) & 1u) atomicAdd(&hist[base + row[m]], 1);
  }
  __syncthreads();
  int32_t* out = counters + ((size_t)j * n_chunks + chunk) * b_cap;
  for (int i = threadIdx.x; i < b_cap; i += blockDim.x) out[i] = (i >= gb_lo && i < gb_hi) ? hist[i - gb_lo] : 0;
}

// ------------------------------------------------------------------------------------------------ chunk prefix
// For every list (kv head j, block gb): counters[j][chunk][gb] becomes the number of entries the list gets from
// earlier chunks, and cnt / len_scan receive the list's length.  A workgroup owns 64 consecutive blocks of one kv
// head; its four wavefronts take a quarter of the chunks each (sum, exchange through LDS, then prefix), so the
// column walk is a handful of coalesced row accesses per thread.  grid (ceil(b_cap / 64), hkv), 256 threads.
__global__ void __launch_bounds__(256) k_chunk_prefix(int32_t* __restrict__ counters, int b_cap, int n_chunks,
                                                      int n_lists, int32_t* __restrict__ cnt,
                                                      int32_t* __restrict__ len_scan) {
  __shared__ int32_t part[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6, j = blockIdx.y;
  const int gb = blockIdx.x * 64 + lane;
  const bool live = gb < b_cap;
  const int per = (n_chunks + 3) / 4;
  const int c0 = min(q * per, n_chunks), c1 = min(c0 + per, n_chunks);
  int32_t* col = counters + (size_t)j * n_chunks * b_cap + (live ? gb : 0);
  int32_t sum = 0;
  if (live) {
    int c = c0;
    for (; c + 8 <= c1; c += 8) {
      int32_t v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = col[(size_t)(c + i) * b_cap];
#pragma unroll
      for (int i = 0; i < 8; ++i) sum += v[i];
    }
    for (; c < c1; ++c) sum += col[(size_t)c * b_cap];
  }
  part[q][lane] = sum;
  __syncthreads();
  int32_t run = 0;
  for (int w = 0; w < q; ++w) run += part[w][lane];
  if (live) {
    int c = c0;
    for (; c + 8 <= c1; c += 8) {
      int32_t v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = col[(size_t)(c + i) * b_cap];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        col[(size_t)(c + i) * b_cap] = run;
        run += v[i];
      }
    }
    for (; c < c1; ++c) {
      const int32_t v = col[(size_t)c * b_cap];
      col[(size_t)c * b_cap] = run;
      run += v;
    }
    if (q == 3) {
      const int L = j * b_cap + gb;
      cnt[L] = run;
      len_scan[L] = run;
    }
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) len_scan[n_lists] = 0;
}

// ------------------------------------------------------------------------------------------------ dense detection
// Dense forward path: which (query tile, KV block) pairs skip the gather route.  A query tile is kTileTokens
// consecutive tokens of one sequence.  One wavefront per (tile, kv head), lane = token: a KV block that at least
// `need` = half of the tile's tokens keep (the attention-sink block, the tokens' own block and the blocks next to it
// are kept by all of them) becomes a dense pair: the forward computes it for the whole tile with the query tile read
// once and the output accumulated on chip, a 64-bit mask saying which tokens really keep it.  The tokens' columns
// that hold such a block are recorded in dmask; the scatter flags their list entries, and the gather route of the
// forward skips them.  Nothing here is assumed about the selection: pairs come from counting, and any pair may take
// either route.  Candidates are the kept blocks of three tokens of the tile (first, middle, last); a block that
// qualifies but is kept by none of the three simply stays on the gather route.  A per-wavefront table of counters
// (block id modulo kDenseHash, LDS atomics: counts are order-free) tells which candidates can reach `need`: lane m
// looks up column m of the proposing token, so only the few that pass get the exact count (a ballot).
// The dense table lists 64-key pieces (a 128-token block gives two) by first key and key count, in the order found;
// pieces no token of the tile can see (wholly in the future, or wholly before every token's window) are left out.
// grid (ceil(t_cap / 4), hkv), 256 threads.  Dynamic LDS: 4 * (kDenseHash + 64 * (k + 1)) ints.
__global__ void __launch_bounds__(256) k_dense_detect(const int32_t* __restrict__ idx, const int32_t* __restrict__ cu,
                                                      const int32_t* __restrict__ tile_tok0,
                                                      const int32_t* __restrict__ tile_len, int nseq, int T, int hkv,
                                                      int k, int bk, int causal, int window, int t_cap, int on,
                                                      const uint32_t* __restrict__ vmask,
                                                      uint32_t* __restrict__ dmask, int32_t* __restrict__ d_cnt,
                                                      int2* __restrict__ d_piece,
                                                      unsigned long long* __restrict__ d_mask) {
  extern __shared__ int32_t lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, j = blockIdx.y;
  const int qt = blockIdx.x * 4 + wave;
  if (qt >= t_cap) return;  // no block-wide barrier below
  int32_t* hash = lds + wave * (kDenseHash + 64 * (k + 1));
  int32_t* rows = hash + kDenseHash;
  const int tlen = tile_len[qt], ttok0 = tile_tok0[qt];
  const size_t slot = (size_t)qt * hkv + j;
  if (tlen == 0 || !on) {
    if (lane == 0) d_cnt[slot] = 0;
    if (lane < tlen) dmask[(size_t)(ttok0 + lane) * hkv + j] = 0u;
    return;
  }
  const int t = ttok0 + lane;
  const bool live = lane < tlen;
  int s, c0, c1;
  seq_bounds(cu, nseq, T, ttok0, s, c0, c1);  // a tile lies in one sequence
  for (int i = lane; i < kDenseHash; i += 64) hash[i] = 0;
  int32_t* row = rows + lane * (k + 1);
  const uint32_t vm = live ? vmask[(size_t)t * hkv + j] : 0u;
  if ((k & 3) == 0 && (reinterpret_cast<uintptr_t>(idx) & 15) == 0) {
    // the tile's rows of idx, 16 bytes per lane: k / 4 lanes cover a row, 256 / k rows per access
    const int lpr = k >> 2, rpa = 64 / lpr;
    const int sub = lane % lpr, r0 = lane / lpr;
    for (int rr = r0; rr < tlen; rr += rpa) {
      const int4 x = *reinterpret_cast<const int4*>(idx + ((size_t)(ttok0 + rr) * hkv + j) * k + 4 * sub);
      int32_t* dst = rows + rr * (k + 1) + 4 * sub;
      dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
    }
  } else if (live) {
    const int32_t* src = idx + ((size_t)t * hkv + j) * k;
    for (int m = 0; m < k; ++m) row[m] = src[m];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  for (int m = 0; m < k; ++m)
    if ((vm >> m) & 1u) atomicAdd(&hash[row[m] & (kDenseHash - 1)], 1);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // this token's kept block ids in registers (-1 where the column is not kept: no candidate matches it)
  int kept[kMaxTopk];
#pragma unroll
  for (int m = 0; m < kMaxTopk; ++m) kept[m] = (m < k && ((vm >> m) & 1u)) ? row[m] : -1;
  const int need = (tlen + 1) >> 1;
  const int prop[3] = {0, tlen >> 1, tlen - 1};
  int nd = 0;
  uint32_t dm = 0;
  for (int pi = 0; pi < 3; ++pi) {
    const int p = prop[pi];
    if ((pi == 1 && p == prop[0]) || (pi == 2 && (p == prop[0] || p == prop[1]))) continue;
    const uint32_t pvm = (uint32_t)__builtin_amdgcn_readlane((int)vm, p);
    // lane m: could column m of token p's row reach `need`?
    const bool mine = lane < k && ((pvm >> lane) & 1u);
    const int cand_blk = mine ? rows[p * (k + 1) + lane] : 0;
    const int cand_cnt = mine ? hash[cand_blk & (kDenseHash - 1)] : 0;
    unsigned long long cand = __builtin_amdgcn_ballot_w64(cand_cnt >= need);
    while (cand != 0ull) {
      const int m = __builtin_ctzll(cand);
      cand &= cand - 1ull;
      const int c = __builtin_amdgcn_readlane(cand_blk, m);
      int mycol = -1;
#pragma unroll
      for (int mm = kMaxTopk - 1; mm >= 0; --mm) mycol = kept[mm] == c ? mm : mycol;
      const unsigned long long members = __builtin_amdgcn_ballot_w64(mycol >= 0);
      // an earlier proposer that keeps c has already dealt with it
      bool seen = false;
      for (int pj = 0; pj < pi; ++pj) seen |= ((members >> prop[pj]) & 1ull) != 0ull;
      if (seen || __popcll(members) < need) continue;
      // the block's 64-key pieces some token of the tile can see
      const int btok0 = c0 + c * bk, blen = min(bk, c1 - btok0);
      int np = 0, ptok[2], plen[2];
      for (int sub = 0; sub < (bk >> 6); ++sub) {
        const int pt = btok0 + 64 * sub, pl = min(64, blen - 64 * sub);
        if (pl <= 0) continue;
        if (causal && pt > ttok0 + tlen - 1) continue;
        if (window > 0 && pt + pl - 1 < ttok0 - window + 1) continue;
        ptok[np] = pt;
        plen[np] = pl;
        ++np;
      }
      if (nd + np > kDenseMax) continue;
      if (lane == 0)
        for (int q = 0; q < np; ++q) {
          d_piece[slot * kDenseMax + nd + q] = make_int2(ptok[q], plen[q]);
          d_mask[slot * kDenseMax + nd + q] = members;
        }
      if (mycol >= 0) dm |= 1u << mycol;  // also when no piece is visible: the pair then contributes nothing
      nd += np;
    }
  }
  if (lane == 0) d_cnt[slot] = nd;
  if (live) dmask[(size_t)t * hkv + j] = dm;
}

// ------------------------------------------------------------------------------------------------ scan
__global__ void __launch_bounds__(kScanThreads) k_scan_reduce(const int32_t* __restrict__ a, int64_t n,
                                                              int32_t* __restrict__ sums) {
  __shared__ int32_t part[kScanThreads];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int32_t acc = 0;
  for (int i = 0; i < kScanItems; ++i)
    if (base + i < n) acc += a[base + i];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kScanThreads / 2; s > 0; s >>= 1) {
    if (threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) sums[blockIdx.x] = part[0];
}

// In-place exclusive scan of one 4096-item tile, plus offsets[blockIdx.x] when given.
__global__ void __launch_bounds__(kScanThreads) k_scan_tile(int32_t* __restrict__ a, int64_t n,
                                                            const int32_t* __restrict__ offsets) {
  __shared__ int32_t part[2][kScanThreads];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int32_t v[kScanItems];
  int32_t acc = 0;
  for (int i = 0; i < kScanItems; ++i) {
    v[i] = (base + i < n) ? a[base + i] : 0;
    acc += v[i];
  }
  int cur = 0;
  part[0][threadIdx.x] = acc;
  __syncthreads();
  for (int s = 1; s < kScanThreads; s <<= 1) {  // Hillis-Steele inclusive scan of the thread totals
    int32_t x = part[cur][threadIdx.x];
    if ((int)threadIdx.x >= s) x += part[cur][threadIdx.x - s];
    part[cur ^ 1][threadIdx.x] = x;
    cur ^= 1;
    __syncthreads();
  }
  int32_t run = part[cur][threadIdx.x] - acc + (offsets ? offsets[blockIdx.x] : 0);
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < n) a[base + i] = run;
    run += v[i];
  }
}

static int64_t scan_tmp_ints(int64_t n) {
  int64_t total = 0;
  while (n > kScanTile) {
    n = (n + kScanTile - 1) / kScanTile;
    total += (n + 63) / 64 * 64;
  }
  return total + 64;
}

static void scan_exclusive(int32_t* a, int64_t n, int32_t* tmp, hipStream_t st) {
  const int64_t nb = (n + kScanTile - 1) / kScanTile;
  if (nb <= 1) {
    hipLaunchKernelGGL(k_scan_tile, dim3(1), dim3(kScanThreads), 0, st, a, n, (const int32_t*)nullptr);
    return;
  }
  hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)nb), dim3(kScanThreads), 0, st, a, n, tmp);
  scan_exclusive(tmp, nb, tmp + (nb + 63) / 64 * 64, st);
  hipLaunchKernelGGL(k_scan_tile, dim3((unsigned)nb), dim3(kScanThreads), 0, st, a, n, (const int32_t*)tmp);
}

// ------------------------------------------------------------------------------------------------ scatter
// grid (n_chunks, hkv), ONE wavefront per group.  off[list] + chunk_off[kv head][chunk][block] is the position in
// qent where the chunk's tokens of that list start.  Every kept column costs one
// scattered 8-byte store (the list entry); the positions of a token's columns are collected in LDS and leave
// as one contiguous row of slotpos.  Dynamic LDS: b_cap u64 masks + b_cap int cursors + 2 * 64*(k+1) ints.
__global__ void __launch_bounds__(64) k_scatter(const int32_t* __restrict__ idx, const int32_t* __restrict__ cu,
                                                const int32_t* __restrict__ blk_base, int nseq, int T, int hkv, int k,
                                                int bk, int causal, int b_cap, int n_chunks,
                                                const int32_t* __restrict__ chunk_off,
                                                const int32_t* __restrict__ off, int2* __restrict__ qent,
                                                const uint32_t* __restrict__ vmask,
                                                const uint32_t* __restrict__ dmask, int32_t* __restrict__ slotpos) {
  extern __shared__ int32_t lds[];
  unsigned long long* mask = reinterpret_cast<unsigned long long*>(lds);
  int32_t* cursor = lds + 2 * b_cap;
  int32_t* rows = cursor + b_cap;
  int32_t* prows = rows + 64 * (k + 1);
  const int chunk = blockIdx.x, j = blockIdx.y, lane = threadIdx.x;
  const int t0 = chunk * kChunkTokens, t1 = min(t0 + kChunkTokens, T);
  int gb_lo, gb_hi;
  chunk_window(cu, blk_base, nseq, T, t0, t1, bk, causal, gb_lo, gb_hi);
  const int win = gb_hi - gb_lo;
  for (int i = lane; i < win; i += 64) {
    mask[i] = 0ull;
    cursor[i] = off[j * b_cap + gb_lo + i] + chunk_off[((size_t)j * n_chunks + chunk) * b_cap + gb_lo + i];
  }
  __syncthreads();
  int32_t* row = rows + lane * (k + 1);
  int32_t* prow = prows + lane * (k + 1);
  const unsigned long long below = (1ull << lane) - 1ull;
  const bool vec4 = (k & 3) == 0 && ((reinterpret_cast<uintptr_t>(idx) | reinterpret_cast<uintptr_t>(slotpos)) & 15) == 0;
  for (int r0 = t0; r0 < t1; r0 += 64) {
    const int t = r0 + lane;
    uint32_t vm = 0, dm = 0;
    int base = 0;
    if (t < t1) {
      int s, c0, c1;
      seq_bounds(cu, nseq, T, t, s, c0, c1);
      const int32_t* src = idx + ((size_t)t * hkv + j) * k;
      if (vec4) {
        for (int m = 0; m < k; m += 4) {
          const int4 x = *reinterpret_cast<const int4*>(src + m);
          row[m] = x.x; row[m + 1] = x.y; row[m + 2] = x.z; row[m + 3] = x.w;
        }
      } else {
        for (int m = 0; m < k; ++m) row[m] = src[m];
      }
      vm = vmask[(size_t)t * hkv + j];  // kept columns, decided by the histogram pass
      dm = dmask[(size_t)t * hkv + j];  // those of them the dense forward path takes over
      base = blk_base[s] - gb_lo;
    }
    // A: mark membership of this round's tokens in every block they keep
    for (int m = 0; m < k; ++m)
      if ((vm >> m) & 1u) atomicOr(&mask[base + row[m]], 1ull << lane);
    __syncthreads();
    // B: rank among the lower tokens of the round gives the position; lists come out ascending.  Four columns
    // per step so that their LDS reads are in flight together.
    for (int m0 = 0; m0 < k; m0 += 4) {
      int w[4], c[4];
      unsigned long long mk[4];
      bool on[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        on[u] = m0 + u < k && ((vm >> (m0 + u)) & 1u);
        w[u] = on[u] ? base + row[m0 + u] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        c[u] = cursor[w[u]];
        mk[u] = mask[w[u]];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int pos = on[u] ? c[u] + __popcll(mk[u] & below) : -1;
        // the sign bit of the column flags an entry of a dense (tile, block) pair: the forward's gather route skips
        // it, the backward (which walks whole lists) ignores the flag
        if (on[u]) qent[pos] = make_int2(t, (m0 + u) | (int)(((dm >> (m0 + u)) & 1u) << 31));
        if (m0 + u < k) prow[m0 + u] = pos;
      }
    }
    if (t < t1) {
      int32_t* dst = slotpos + ((size_t)t * hkv + j) * k;
      if (vec4) {
        for (int m = 0; m < k; m += 4)
          *reinterpret_cast<int4*>(dst + m) = make_int4(prow[m], prow[m + 1], prow[m + 2], prow[m + 3]);
      } else {
        for (int m = 0; m < k; ++m) dst[m] = prow[m];
      }
    }
    __syncthreads();
    // C: the lowest member of each touched block advances its cursor and clears the mask
    for (int m0 = 0; m0 < k; m0 += 4) {
      int w[4];
      unsigned long long mk[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool on = m0 + u < k && ((vm >> (m0 + u)) & 1u);
        w[u] = on ? base + row[m0 + u] : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) mk[u] = w[u] >= 0 ? mask[w[u]] : 0ull;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (mk[u] != 0ull && (mk[u] & below) == 0ull) {
          cursor[w[u]] += __popcll(mk[u]);
          mask[w[u]] = 0ull;
        }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------ finalize
// number of work units per list (off is the scanned list lengths, n_lists + 1 entries)
__global__ void k_finalize(const int32_t* __restrict__ cnt, const int32_t* __restrict__ off, int n_lists, int unit,
                           int32_t* __restrict__ u_nu, int32_t* __restrict__ hdr) {
  const int L = blockIdx.x * blockDim.x + threadIdx.x;
  if (L > n_lists) return;
  if (L == n_lists) {
    hdr[HDR_NPAIRS] = off[n_lists];
    u_nu[L] = 0;
    return;
  }
  const int32_t c = cnt[L];
  u_nu[L] = (c + unit - 1) / unit;
}

// nu_scan is the exclusive scan of units per list (n_lists + 1 entries).
__global__ void k_units(const int32_t* __restrict__ nu_scan, const int32_t* __restrict__ off, int n_lists, int unit,
                        int32_t* __restrict__ u_list, int32_t* __restrict__ u_start, int32_t* __restrict__ hdr_slot) {
  const int L = blockIdx.x * blockDim.x + threadIdx.x;
  if (L >= n_lists) return;
  const int u0 = nu_scan[L], u1 = nu_scan[L + 1];
  for (int u = u0; u < u1; ++u) {
    u_list[u] = L;
    u_start[u] = off[L] + (u - u0) * unit;
  }
  if (L == n_lists - 1) *hdr_slot = u1;
}

hipError_t launch_build_index(const IndexLayout& L, const int32_t* idx, const int32_t* cu, void* index_ws,
                              hipStream_t st) {
  IndexPtrs p = index_ptrs(L, index_ws);
  const size_t lds_hist = (size_t)L.b_cap * 4 + 256 * (size_t)(L.topk + 1) * 4;
  const size_t lds_scat = (size_t)L.b_cap * 12 + 2 * 64 * (size_t)(L.topk + 1) * 4;
  if (lds_hist > 64 * 1024 || lds_scat > 64 * 1024) {  // long sequences: block tables beyond the default 64 KB
    static std::atomic<uint64_t> ready_hist, ready_scat;
    hipError_t e = allow_dynamic_lds((const void*)k_hist, 160 * 1024, ready_hist);
    if (e == hipSuccess) e = allow_dynamic_lds((const void*)k_scatter, 160 * 1024, ready_scat);
    if (e != hipSuccess) return e;
  }
  { ProfScope ps(KID_INDEX_PREP, st);
  hipLaunchKernelGGL(k_prep, dim3(1), dim3(256), 0, st, cu, L.nseq, L.T, L.bk, L.b_cap, p.blk_base, p.blk_tok0, p.blk_len,
                     p.hdr + HDR_BTOT);
  // the query tiles of the dense forward path: the same table for blocks of kTileTokens tokens
  hipLaunchKernelGGL(k_prep, dim3(1), dim3(256), 0, st, cu, L.nseq, L.T, kTileTokens, L.t_cap, p.tile_base, p.tile_tok0,
                     p.tile_len, p.hdr + HDR_NTILES); }
  { ProfScope ps(KID_INDEX_HIST, st);
  hipLaunchKernelGGL(k_hist, dim3(L.n_chunks, L.hkv), dim3(256), lds_hist, st, idx, cu, p.blk_base, L.nseq, L.T, L.hkv,
                     L.topk, L.bk, L.causal, L.window, L.b_cap, L.n_chunks, p.chunk_off, p.vmask); }
  const int nl1 = L.n_lists + 1;
  { ProfScope ps(KID_INDEX_CHUNK_PREFIX, st);
  hipLaunchKernelGGL(k_chunk_prefix, dim3((L.b_cap + 63) / 64, L.hkv), dim3(256), 0, st, p.chunk_off, L.b_cap, L.n_chunks,
                     L.n_lists, p.cnt, p.off); }
  { ProfScope ps(KID_INDEX_SCAN, st);
  scan_exclusive(p.off, nl1, p.scan_tmp, st); }
  { ProfScope ps(KID_INDEX_DENSE, st);
  const size_t lds_dense = 4 * (size_t)(kDenseHash + 64 * (L.topk + 1)) * 4;
  hipLaunchKernelGGL(k_dense_detect, dim3((L.t_cap + 3) / 4, L.hkv), dim3(256), lds_dense, st, idx, cu, p.tile_tok0,
                     p.tile_len, L.nseq, L.T, L.hkv, L.topk, L.bk, L.causal, L.window, L.t_cap,
                     L.dense, p.vmask,
                     p.dmask, p.d_cnt, p.d_piece, p.d_mask); }
  { ProfScope ps(KID_INDEX_SCATTER, st);
  hipLaunchKernelGGL(k_scatter, dim3(L.n_chunks, L.hkv), dim3(64), lds_scat, st, idx, cu, p.blk_base, L.nseq, L.T,
                     L.hkv, L.topk, L.bk, L.causal, L.b_cap, L.n_chunks, p.chunk_off, p.off, p.qent, p.vmask, p.dmask,
                     p.slotpos); }
  { ProfScope ps(KID_INDEX_FINALIZE, st);
  hipLaunchKernelGGL(k_finalize, dim3((nl1 + 255) / 256), dim3(256), 0, st, p.cnt, p.off, L.n_lists, L.unit, p.u_nu,
                     p.hdr); }
  { ProfScope ps(KID_INDEX_SCAN, st);
  scan_exclusive(p.u_nu, nl1, p.scan_tmp, st); }
  { ProfScope ps(KID_INDEX_UNITS, st);
  hipLaunchKernelGGL(k_units, dim3((L.n_lists + 255) / 256), dim3(256), 0, st, p.u_nu, p.off, L.n_lists, L.unit,
                     p.u_list, p.u_start, p.hdr + HDR_UNITS); }
  return hipGetLastError();
}

// scratch of the scans: the longest scanned array has one entry per list plus one
int64_t index_scan_tmp_ints(int64_t n_lists) { return scan_tmp_ints(n_lists + 1); }

}  // namespace nsa
