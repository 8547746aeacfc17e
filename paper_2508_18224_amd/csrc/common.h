// Shared declarations of the gfx950 selected-attention library: workspace layout, launch prototypes and
// small device helpers.  Everything here is internal; the public surface is include/nsa_sel.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <atomic>

#include "../../include/nsa_sel.h"

namespace nsa {

constexpr int kBlock = 64;         // tokens of the smaller of the two block sizes (B_K = 64 or 2 * 64)
constexpr int kD = 128;            // head dimension
constexpr int kChunkTokens = 512;  // token chunk of the inversion histogram / scatter
constexpr int kMaxUnit = 2048;     // most list entries of one work unit (the size used for long inputs)
constexpr int kMinUnit = 256;
constexpr int kMaxTopk = 32;
constexpr int kSlotBatch = 4;      // slots of a row the two reduction kernels gather at a time
constexpr int kTileTokens = 64;    // query tokens of a tile of the dense forward path (whatever B_K is)
constexpr int kDenseMax = 32;      // most 64-key pieces one (query tile, kv head) routes through the dense path
constexpr int kDenseHash = 1024;   // per-wavefront counters of the detection pass (block id modulo this)

// Host-computed description of the index workspace (byte offsets from its base, all 256-aligned).
struct IndexLayout {
  int32_t T, nseq, hkv, topk, causal;
  int32_t window;       // 0 or the sliding-window length in tokens
  int32_t bk;           // B_K: tokens per KV block, 64 or 128
  int32_t b_cap;        // list stride: T / bk + nseq  (>= real number of blocks)
  int32_t n_lists;      // hkv * b_cap
  int32_t n_chunks;     // ceil(T / kChunkTokens)
  int64_t n_counters;   // n_lists * n_chunks
  int64_t p_max;        // T * hkv * topk
  int32_t unit;         // list entries per work unit of the attention kernels (see work_unit_entries)
  int32_t units_max;    // upper bound of the number of work units
  int32_t dense;        // 1: (query tile, KV block) pairs most of the tile's tokens keep go through the dense path
  int32_t t_cap;        // query tiles of kTileTokens tokens: T / kTileTokens + nseq (>= real number of tiles)
  size_t hdr, blk_base, blk_tok0, blk_len, chunk_off, cnt, off, qent, vmask, slotpos;
  size_t u_nu, u_list, u_start, scan_tmp;
  size_t tile_base, tile_tok0, tile_len, dmask, d_cnt, d_piece, d_mask;
  size_t total;
};

// hdr words
enum { HDR_BTOT = 0, HDR_NPAIRS = 1, HDR_UNITS = 2, HDR_NTILES = 3 };

struct IndexPtrs {
  int32_t* hdr;
  int32_t* blk_base;
  int32_t* blk_tok0;
  int32_t* blk_len;
  int32_t* chunk_off;  // [hkv][n_chunks][b_cap]: entries a list receives from the chunks before this one
  int32_t* cnt;        // [n_lists] list lengths
  int32_t* off;        // [n_lists + 1] exclusive scan of cnt: first position of every list in qent
  int2* qent;        // list entries: (token, column of idx it came from)
  uint32_t* vmask;
  int32_t* slotpos;  // [T, hkv, topk]: position in qent of the entry a kept column produced
  // work units (shared by forward and backward): scanned units per list, and per unit its list and first entry
  int32_t *u_nu, *u_list, *u_start;
  int32_t* scan_tmp;
  // dense forward path: query tiles (kTileTokens consecutive tokens of one sequence) and, per (tile, kv head), the
  // 64-key pieces of the KV blocks at least half of the tile's tokens keep, each with the 64-bit mask of the tokens
  // that keep its block
  int32_t *tile_base, *tile_tok0, *tile_len;
  uint32_t* dmask;     // [T, hkv]: columns of idx the dense path takes over (a subset of vmask)
  int32_t* d_cnt;      // [t_cap, hkv]
  int2* d_piece;       // [t_cap, hkv, kDenseMax] (first key token, number of keys <= 64)
  unsigned long long* d_mask;  // [t_cap, hkv, kDenseMax]
};

inline IndexPtrs index_ptrs(const IndexLayout& L, void* base) {
  char* p = static_cast<char*>(base);
  IndexPtrs r;
  r.hdr = (int32_t*)(p + L.hdr);
  r.blk_base = (int32_t*)(p + L.blk_base);
  r.blk_tok0 = (int32_t*)(p + L.blk_tok0);
  r.blk_len = (int32_t*)(p + L.blk_len);
  r.chunk_off = (int32_t*)(p + L.chunk_off);
  r.cnt = (int32_t*)(p + L.cnt);
  r.off = (int32_t*)(p + L.off);
  r.qent = (int2*)(p + L.qent);
  r.vmask = (uint32_t*)(p + L.vmask);
  r.slotpos = (int32_t*)(p + L.slotpos);
  r.u_nu = (int32_t*)(p + L.u_nu);
  r.u_list = (int32_t*)(p + L.u_list);
  r.u_start = (int32_t*)(p + L.u_start);
  r.scan_tmp = (int32_t*)(p + L.scan_tmp);
  r.tile_base = (int32_t*)(p + L.tile_base);
  r.tile_tok0 = (int32_t*)(p + L.tile_tok0);
  r.tile_len = (int32_t*)(p + L.tile_len);
  r.dmask = (uint32_t*)(p + L.dmask);
  r.d_cnt = (int32_t*)(p + L.d_cnt);
  r.d_piece = (int2*)(p + L.d_piece);
  r.d_mask = (unsigned long long*)(p + L.d_mask);
  return r;
}

// Problem description handed to the attention kernels.
struct Problem {
  int32_t T, nseq, hq, hkv, g, topk, causal, b_cap, bk;
  int32_t window;    // 0, or: key u is visible to token t only if u > t - window
  uint32_t g_magic;  // floor(2^32 / g) + 1, or 0 when g == 1: row / g as one multiply-high (see div_g)
  int32_t unit;    // list entries per work unit
  int32_t dense;   // 1: the dense forward path is on (the index carries dense flags and tables)
  int32_t t_cap;   // stride of the per-(tile, kv head) dense tables
  int32_t j0, nj;  // KV heads [j0, j0 + nj) handled by this launch (all of them unless the workspace is capped)
  float scale;
};

// List entries per work unit.  Long inputs use kMaxUnit (splitting lists further only adds dK/dV partial sums);
// short inputs use smaller units so that the ~512 workgroup slots of the chip each get several units and the sink
// block's list (every token) does not become one slot's whole share.  Sizes swept on the paper's 8K .. 64K grid.
inline int work_unit_entries(int64_t total_pairs) {
  int u = kMinUnit;
  while (u < kMaxUnit && (int64_t)u * 2 * 2048 <= total_pairs) u *= 2;  // largest power of two <= pairs / 2048
  return u;
}

// Upper bound of the work units of nj KV heads (one per non-empty list plus one per full unit of entries); the
// real count is only known on the device.
inline int64_t units_bound(int nj, int b_cap, int T, int topk, int unit) {
  return (int64_t)nj * b_cap + (int64_t)nj * T * topk / unit + 1;
}

// ---- optional per-kernel timing (off unless nsa_sel_profile_enable was called) ---------------------------
enum KernelId {
  KID_INDEX_PREP = 0, KID_INDEX_CHUNK_PREFIX, KID_INDEX_HIST, KID_INDEX_SCAN, KID_INDEX_SCATTER, KID_INDEX_FINALIZE,
  KID_INDEX_UNITS, KID_FWD_MAIN, KID_FWD_MERGE, KID_BWD_DELTA, KID_BWD_MAIN, KID_BWD_DQ_REDUCE, KID_BWD_DKV_REDUCE,
  KID_SELECT_BLOCKS, KID_FWD_QUERY_OUTER, KID_INDEX_DENSE, KID_FWD_DENSE, KID_COUNT
};
// Records a HIP event on `st` at construction and destruction when profiling is on; does nothing otherwise.
struct ProfScope {
  int slot;
  hipStream_t st;
  ProfScope(int kid, hipStream_t stream);
  ~ProfScope();
};

// Raises a kernel's dynamic-LDS limit to `bytes`, once per device (`done` holds one bit per device id), so that
// later launches - also those recorded into a HIP graph - make no attribute call at all.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Optional gated combination with the other attention branches (Eq. (2)); all null for the plain entry points.
struct GateArgs {
  const float* gate;  // [T, hq]
  const void* o_acc;  // bf16 [T, hq, d] or null
  void* o_out;        // bf16 [T, hq, d]
  float* dgate;       // [T, hq] (backward)
};

// ---- launchers (each enqueues on `st` and returns hipGetLastError()) -------------------------------------
hipError_t launch_build_index(const IndexLayout& L, const int32_t* idx, const int32_t* cu, void* index_ws,
                              hipStream_t st);
// heads_per_pass: KV heads whose partial results the workspace can hold at once (1 .. hkv)
hipError_t launch_fwd(const Problem& P, const IndexLayout& L, int heads_per_pass, const void* Q, const void* K,
                      const void* V, const void* index_ws, void* opart, float* lse_part, void* O, float* LSE,
                      const GateArgs& G, hipStream_t st);
// the same forward in query-outer loop order (no workspaces, no index): see qouter.hip
hipError_t launch_fwd_query_outer(const Problem& P, const void* Q, const void* K, const void* V, const int32_t* idx,
                                  const int32_t* cu, void* O, float* LSE, hipStream_t st);
hipError_t launch_bwd(const Problem& P, const IndexLayout& L, int heads_per_pass, const void* Q, const void* K,
                      const void* V, const void* O, const float* LSE, const void* dO, const void* index_ws,
                      void* dqpart, float* delta, float* dkv_part, void* dQ, void* dK, void* dV, const GateArgs& G,
                      hipStream_t st);

// ---- device helpers ------------------------------------------------------------------------------------
#if defined(__HIPCC__)
typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // 16 bytes in flight as a plain vector (rows being gathered)
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// r / g for 0 <= r < 2^20 and g in [1, 8] without an integer division: the error of the rounded-up reciprocal,
// r (magic - 2^32 / g) < r, stays far below 2^32 / g, so the high word of the product is the exact quotient.
// g = 1 has no 32-bit reciprocal; its magic is 0 and r is added instead (a select, not a branch).
__device__ __forceinline__ int div_g(int r, int g, uint32_t g_magic) {
  return (int)(((uint64_t)(uint32_t)r * g_magic) >> 32) + (g == 1 ? r : 0);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// 16-byte store with the non-temporal hint: partial rows are written once and read once much later, so they
// should not displace the gathered Q / dO rows from the caches.
__device__ __forceinline__ void store_streaming(bf16_t* dst, uint4 v) {
  u32x4 x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<u32x4*>(dst));
}

// Sequence bounds of token t in a packed batch (cu may be null for a single sequence).
__device__ __forceinline__ void seq_bounds(const int32_t* cu, int nseq, int T, int t, int& s, int& c0, int& c1) {
  if (cu == nullptr || nseq == 1) {
    s = 0;
    c0 = 0;
    c1 = T;
    return;
  }
  int lo = 0, hi = nseq;  // invariant: cu[lo] <= t < cu[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  s = lo;
  c0 = cu[lo];
  c1 = cu[lo + 1];
}
#endif

}  // namespace nsa
