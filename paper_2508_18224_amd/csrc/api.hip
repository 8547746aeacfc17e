// C ABI of the library (see include/nsa_sel.h): argument validation, workspace layout, launch sequencing.
#include "common.h"

namespace nsa {
int64_t index_scan_tmp_ints(int64_t n_lists);

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Tensors are moved with 16-byte accesses and the workspaces are carved at 256-byte offsets.
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

static int check_shape(const nsa_sel_shape* s) {
  if (!s) return NSA_SEL_EINVAL;
  if (s->total_tokens < 0 || s->nseq < 1 || s->hq < 1 || s->hkv < 1) return NSA_SEL_EINVAL;
  if (s->hq % s->hkv != 0) return NSA_SEL_EINVAL;
  const int g = s->hq / s->hkv;
  if (g < 1 || g > 8) return NSA_SEL_EINVAL;
  if (s->window < 0 || (s->window > 0 && !s->causal)) return NSA_SEL_EINVAL;
  if (s->unit != 0 && (s->unit < kMinUnit || s->unit > kMaxUnit || (s->unit & (s->unit - 1)) != 0)) return NSA_SEL_EINVAL;
  if (s->dense < -1 || s->dense > 1) return NSA_SEL_EINVAL;
  if (s->d != kD || (s->block != kBlock && s->block != 2 * kBlock)) return NSA_SEL_EUNSUPPORTED;
  if (s->topk < 1 || s->topk > kMaxTopk) return NSA_SEL_EUNSUPPORTED;
  if (s->nseq > (1 << 20)) return NSA_SEL_EUNSUPPORTED;
  if ((int64_t)s->total_tokens * s->hq >= ((int64_t)1 << 31)) return NSA_SEL_EUNSUPPORTED;  // 32-bit row indices
  const int64_t b_cap = (int64_t)s->total_tokens / s->block + s->nseq;
  // LDS tables of the inversion (12 bytes per block) must fit in one CU's 160 KB
  if (b_cap * 12 + 2 * 64 * (int64_t)(s->topk + 1) * 4 > 160 * 1024) return NSA_SEL_EUNSUPPORTED;
  const int64_t p_max = (int64_t)s->total_tokens * s->hkv * s->topk;
  if (p_max >= ((int64_t)1 << 31) - 4096) return NSA_SEL_EUNSUPPORTED;
  const int64_t n_chunks = ((int64_t)s->total_tokens + kChunkTokens - 1) / kChunkTokens;
  if (b_cap * s->hkv * (n_chunks > 0 ? n_chunks : 1) >= ((int64_t)1 << 31) - 4096) return NSA_SEL_EUNSUPPORTED;
  return NSA_SEL_OK;
}

static IndexLayout make_layout(const nsa_sel_shape* s) {
  IndexLayout L;
  L.T = s->total_tokens;
  L.nseq = s->nseq;
  L.hkv = s->hkv;
  L.topk = s->topk;
  L.bk = s->block;
  L.causal = s->causal ? 1 : 0;
  L.window = s->window;
  L.b_cap = s->total_tokens / s->block + s->nseq;
  L.n_lists = s->hkv * L.b_cap;
  L.n_chunks = (s->total_tokens + kChunkTokens - 1) / kChunkTokens;
  if (L.n_chunks < 1) L.n_chunks = 1;
  L.n_counters = (int64_t)L.n_lists * L.n_chunks;
  L.p_max = (int64_t)s->total_tokens * s->hkv * L.topk;
  L.unit = s->unit != 0 ? s->unit : work_unit_entries(L.p_max);
  L.units_max = (int32_t)units_bound(L.hkv, L.b_cap, L.T, L.topk, L.unit);
  // dense route: on request, or by default where it pays: with g = 1 a (tile, kv head) has only 64 rows to share a
  // K / V piece, which costs more than the gather route saves (measured: +4 % per step at g = 1, -1 % .. -8 % at
  // g = 4 .. 8), unless the call is the sliding-window branch, where every pair is dense
  // (and not for inputs so small that the step is a few launch latencies: below 2^18 (token, kv head, column) triples)
  L.dense = s->dense == 1 || (s->dense == 0 && L.p_max >= (1 << 18) && (s->hq / s->hkv >= 2 || s->window > 0)) ? 1 : 0;
  L.t_cap = s->total_tokens / kTileTokens + s->nseq;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align256(o + bytes); return at; };
  L.hdr = take(64);
  L.blk_base = take(4 * (size_t)(L.nseq + 1));
  L.blk_tok0 = take(4 * (size_t)L.b_cap);
  L.blk_len = take(4 * (size_t)L.b_cap);
  L.chunk_off = take(4 * (size_t)(L.n_counters + 1));
  L.cnt = take(4 * (size_t)L.n_lists);
  L.off = take(4 * (size_t)(L.n_lists + 1));
  L.qent = take(8 * (size_t)(L.p_max + 1));
  L.vmask = take(4 * ((size_t)L.T * L.hkv + 1));
  L.slotpos = take(4 * (size_t)(L.p_max + 1));
  L.u_nu = take(4 * (size_t)(L.n_lists + 1));
  L.u_list = take(4 * (size_t)(L.units_max + 1));
  L.u_start = take(4 * (size_t)(L.units_max + 1));
  L.scan_tmp = take(4 * (size_t)index_scan_tmp_ints(L.n_lists));
  L.tile_base = take(4 * (size_t)(L.nseq + 1));
  L.tile_tok0 = take(4 * (size_t)L.t_cap);
  L.tile_len = take(4 * (size_t)L.t_cap);
  L.dmask = take(4 * ((size_t)L.T * L.hkv + 1));
  L.d_cnt = take(4 * (size_t)L.t_cap * L.hkv);
  L.d_piece = take(8 * (size_t)L.t_cap * L.hkv * kDenseMax);
  L.d_mask = take(8 * (size_t)L.t_cap * L.hkv * kDenseMax);
  L.total = o;
  return L;
}

static Problem make_problem(const nsa_sel_shape* s, const IndexLayout& L) {
  Problem P;
  P.T = s->total_tokens;
  P.nseq = s->nseq;
  P.hq = s->hq;
  P.hkv = s->hkv;
  P.g = s->hq / s->hkv;
  P.topk = L.topk;
  P.causal = s->causal ? 1 : 0;
  P.window = s->window;
  P.b_cap = L.b_cap;
  P.bk = L.bk;
  P.unit = L.unit;
  P.dense = L.dense;
  P.t_cap = L.t_cap;
  P.g_magic = P.g == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / (uint64_t)P.g + 1);
  P.j0 = 0;
  P.nj = s->hkv;
  P.scale = s->scale > 0.f ? s->scale : 0.08838834764831845f;  // 1/sqrt(128)
  return P;
}

// Partial rows of nj KV heads: one per (token, query head of those KV heads, selected block).
static size_t partial_rows(const nsa_sel_shape* s, int nj) {
  return (size_t)s->total_tokens * nj * (s->hq / s->hkv) * s->topk;
}

// Workspaces that hold the partial results of nj KV heads at once (nj = hkv: everything in one pass).
static size_t fwd_ws_bytes(const nsa_sel_shape* s, int nj) {
  const size_t rows = partial_rows(s, nj);
  return align256(rows * kD * 2) + align256(rows * 4);
}

static size_t bwd_ws_bytes(const nsa_sel_shape* s, const IndexLayout& L, int nj) {
  const size_t rows = partial_rows(s, nj);
  return align256(rows * kD * 2) + align256((size_t)s->total_tokens * s->hq * 8) +
         align256((size_t)units_bound(nj, L.b_cap, L.T, L.topk, L.unit) * 2 * L.bk * kD * 4);
}

// Largest number of KV heads per pass that `bytes` can hold; 0 when not even one fits.
template <class F>
static int heads_that_fit(int hkv, size_t bytes, F need) {
  int nj = hkv;
  while (nj > 0 && need(nj) > bytes) --nj;
  return nj;
}
}  // namespace nsa

using namespace nsa;

extern "C" {

int nsa_sel_workspace_bytes(const nsa_sel_shape* shape, size_t* fwd_bytes, size_t* bwd_bytes, size_t* index_bytes) {
  int rc = check_shape(shape);
  if (rc) return rc;
  IndexLayout L = make_layout(shape);
  if (fwd_bytes) *fwd_bytes = fwd_ws_bytes(shape, shape->hkv);
  if (bwd_bytes) *bwd_bytes = bwd_ws_bytes(shape, L, shape->hkv);
  if (index_bytes) *index_bytes = L.total;
  return NSA_SEL_OK;
}

int nsa_sel_workspace_bytes_min(const nsa_sel_shape* shape, size_t* fwd_bytes, size_t* bwd_bytes) {
  int rc = check_shape(shape);
  if (rc) return rc;
  IndexLayout L = make_layout(shape);
  if (fwd_bytes) *fwd_bytes = fwd_ws_bytes(shape, 1);
  if (bwd_bytes) *bwd_bytes = bwd_ws_bytes(shape, L, 1);
  return NSA_SEL_OK;
}

int nsa_sel_build_index(const nsa_sel_shape* shape, const int32_t* idx, const int32_t* cu_seqlens, void* index_ws,
                        size_t index_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (shape->total_tokens == 0) return NSA_SEL_OK;
  if (!idx || !index_ws || !aligned16(index_ws)) return NSA_SEL_EINVAL;
  if (!cu_seqlens && shape->nseq != 1) return NSA_SEL_EINVAL;
  IndexLayout L = make_layout(shape);
  if (index_bytes < L.total) return NSA_SEL_EWORKSPACE;
  if (shape->total_tokens == 0) return NSA_SEL_OK;
  return launch_build_index(L, idx, cu_seqlens, index_ws, (hipStream_t)stream) == hipSuccess ? NSA_SEL_OK
                                                                                            : NSA_SEL_EHIP;
}

int nsa_sel_index_view(const nsa_sel_shape* shape, const void* index_ws, const int32_t** cnt, const int32_t** off,
                       const int32_t** qent, const uint32_t** vmask, int32_t* b_cap) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!index_ws) return NSA_SEL_EINVAL;
  IndexLayout L = make_layout(shape);
  IndexPtrs p = index_ptrs(L, const_cast<void*>(index_ws));
  if (cnt) *cnt = p.cnt;
  if (off) *off = p.off;
  if (qent) *qent = (const int32_t*)p.qent;
  if (vmask) *vmask = p.vmask;
  if (b_cap) *b_cap = L.b_cap;
  return NSA_SEL_OK;
}

// Pointer checks of the forward entry points (everything but the workspace).
static int check_fwd_pointers(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V,
                              const int32_t* idx, const int32_t* cu_seqlens, int rebuild_index, const void* index_ws,
                              const void* O, const float* LSE) {
  if (!Q || !K || !V || !index_ws || !O || !LSE) return NSA_SEL_EINVAL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(index_ws)) return NSA_SEL_EINVAL;
  if (rebuild_index && !idx) return NSA_SEL_EINVAL;
  if (!cu_seqlens && shape->nseq != 1) return NSA_SEL_EINVAL;
  return NSA_SEL_OK;
}

static int fwd_impl(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                    const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O,
                    float* LSE, const GateArgs& G, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (shape->total_tokens == 0) return NSA_SEL_OK;  // nothing to do: zero-sized tensors may have no address
  rc = check_fwd_pointers(shape, Q, K, V, idx, cu_seqlens, rebuild_index, index_ws, O, LSE);
  if (rc) return rc;
  if (!ws || !aligned16(ws)) return NSA_SEL_EINVAL;
  IndexLayout L = make_layout(shape);
  const int hpp = heads_that_fit(shape->hkv, ws_bytes, [&](int nj) { return fwd_ws_bytes(shape, nj); });
  if (index_bytes < L.total || hpp < 1) return NSA_SEL_EWORKSPACE;
  if (shape->total_tokens == 0) return NSA_SEL_OK;
  hipStream_t st = (hipStream_t)stream;
  if (rebuild_index && launch_build_index(L, idx, cu_seqlens, index_ws, st) != hipSuccess) return NSA_SEL_EHIP;
  Problem P = make_problem(shape, L);
  const size_t rows = partial_rows(shape, hpp);
  void* opart = ws;
  float* lse_part = (float*)((char*)ws + align256(rows * kD * 2));
  return launch_fwd(P, L, hpp, Q, K, V, index_ws, opart, lse_part, O, LSE, G, st) == hipSuccess ? NSA_SEL_OK
                                                                                                 : NSA_SEL_EHIP;
}

int nsa_sel_fwd(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O, float* LSE,
                void* ws, size_t ws_bytes, void* stream) {
  return fwd_impl(shape, Q, K, V, idx, cu_seqlens, rebuild_index, index_ws, index_bytes, O, LSE,
                  GateArgs{nullptr, nullptr, nullptr, nullptr}, ws, ws_bytes, stream);
}

// ---- nsa_sel_fwd_static: the forward with its partial buffers in a device array of the library -------------------
// In host code the array's name is only a stand-in for the symbol: the address kernels can use comes from
// hipGetSymbolAddress, once per device (every GPU holds its own copy of the array at its own address).
static __device__ __align__(256) unsigned char scratch[NSA_SEL_STATIC_WS_BYTES];
static constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return NSA_SEL_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return NSA_SEL_EUNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return NSA_SEL_EHIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return NSA_SEL_OK;
}

int nsa_sel_fwd_static(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                       const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O,
                       float* LSE, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (shape->total_tokens == 0) return NSA_SEL_OK;
  // sizes first: a shape whose partial results of one KV head exceed the array is refused before anything else
  if (fwd_ws_bytes(shape, 1) > (size_t)NSA_SEL_STATIC_WS_BYTES) return NSA_SEL_ESTATIC;
  rc = check_fwd_pointers(shape, Q, K, V, idx, cu_seqlens, rebuild_index, index_ws, O, LSE);
  if (rc) return rc;
  if (index_bytes < make_layout(shape).total) return NSA_SEL_EWORKSPACE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // Nothing in the array has to start at zero: the merge reads exactly the partial rows the main kernel of the same
  // call wrote (those of kept selections), whatever an earlier call left behind.
  return fwd_impl(shape, Q, K, V, idx, cu_seqlens, rebuild_index, index_ws, index_bytes, O, LSE,
                  GateArgs{nullptr, nullptr, nullptr, nullptr}, ws, (size_t)NSA_SEL_STATIC_WS_BYTES, stream);
}

int nsa_sel_fwd_query_outer(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                            const int32_t* cu_seqlens, void* O, float* LSE, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (shape->block != kBlock || shape->window != 0) return NSA_SEL_EUNSUPPORTED;
  if (shape->total_tokens == 0) return NSA_SEL_OK;
  if (!Q || !K || !V || !idx || !O || !LSE) return NSA_SEL_EINVAL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return NSA_SEL_EINVAL;
  if (!cu_seqlens && shape->nseq != 1) return NSA_SEL_EINVAL;
  IndexLayout L = make_layout(shape);
  Problem P = make_problem(shape, L);
  return launch_fwd_query_outer(P, Q, K, V, idx, cu_seqlens, O, LSE, (hipStream_t)stream) == hipSuccess ? NSA_SEL_OK
                                                                                                         : NSA_SEL_EHIP;
}

int nsa_sel_fwd_gated(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                      const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O,
                      float* LSE, const float* gate, const void* O_acc, void* O_out, void* ws, size_t ws_bytes,
                      void* stream) {
  // O_out == O would overwrite the ungated result the backward needs; O_acc == O would be read after O is written
  if (!gate || !O_out || !aligned16(O_out) || (O_acc && !aligned16(O_acc)) || ((uintptr_t)gate & 3) || O_out == O ||
      (O_acc && O_acc == O))
    return NSA_SEL_EINVAL;
  return fwd_impl(shape, Q, K, V, idx, cu_seqlens, rebuild_index, index_ws, index_bytes, O, LSE,
                  GateArgs{gate, O_acc, O_out, nullptr}, ws, ws_bytes, stream);
}

static int bwd_impl(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const void* O,
                    const float* LSE, const void* dO, const int32_t* cu_seqlens, const void* index_ws,
                    size_t index_bytes, void* dQ, void* dK, void* dV, const GateArgs& G, void* ws, size_t ws_bytes,
                    void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (shape->total_tokens == 0) return NSA_SEL_OK;  // nothing to do: zero-sized tensors may have no address
  if (!Q || !K || !V || !O || !LSE || !dO || !index_ws || !dQ || !dK || !dV || !ws) return NSA_SEL_EINVAL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(dQ) ||
      !aligned16(dK) || !aligned16(dV) || !aligned16(ws) || !aligned16(index_ws))
    return NSA_SEL_EINVAL;
  if (!cu_seqlens && shape->nseq != 1) return NSA_SEL_EINVAL;
  IndexLayout L = make_layout(shape);
  const int hpp = heads_that_fit(shape->hkv, ws_bytes, [&](int nj) { return bwd_ws_bytes(shape, L, nj); });
  if (index_bytes < L.total || hpp < 1) return NSA_SEL_EWORKSPACE;
  if (shape->total_tokens == 0) return NSA_SEL_OK;
  Problem P = make_problem(shape, L);
  const size_t rows = partial_rows(shape, hpp);
  char* w = (char*)ws;
  void* dqpart = w;
  float* delta = (float*)(w + align256(rows * kD * 2));
  float* dkv_part = (float*)((char*)delta + align256((size_t)shape->total_tokens * shape->hq * 8));
  return launch_bwd(P, L, hpp, Q, K, V, O, LSE, dO, index_ws, dqpart, delta, dkv_part, dQ, dK, dV, G,
                    (hipStream_t)stream) == hipSuccess
             ? NSA_SEL_OK
             : NSA_SEL_EHIP;
}

int nsa_sel_bwd(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const void* O,
                const float* LSE, const void* dO, const int32_t* cu_seqlens, const void* index_ws, size_t index_bytes,
                void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, void* stream) {
  return bwd_impl(shape, Q, K, V, O, LSE, dO, cu_seqlens, index_ws, index_bytes, dQ, dK, dV,
                  GateArgs{nullptr, nullptr, nullptr, nullptr}, ws, ws_bytes, stream);
}

int nsa_sel_bwd_gated(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const void* O,
                      const float* LSE, const void* dO_out, const float* gate, const int32_t* cu_seqlens,
                      const void* index_ws, size_t index_bytes, void* dQ, void* dK, void* dV, float* dgate, void* ws,
                      size_t ws_bytes, void* stream) {
  if (!gate || !dgate || ((uintptr_t)gate & 3) || ((uintptr_t)dgate & 3)) return NSA_SEL_EINVAL;
  return bwd_impl(shape, Q, K, V, O, LSE, dO_out, cu_seqlens, index_ws, index_bytes, dQ, dK, dV,
                  GateArgs{gate, nullptr, nullptr, dgate}, ws, ws_bytes, stream);
}

const char* nsa_sel_strerror(int code) {
  switch (code) {
    case NSA_SEL_OK: return "ok";
    case NSA_SEL_EINVAL: return "invalid argument (null or misaligned pointer, head counts, nseq)";
    case NSA_SEL_EUNSUPPORTED: return "unsupported shape (d must be 128, block 64 or 128, topk 1..32, size limits)";
    case NSA_SEL_EWORKSPACE: return "workspace too small (see nsa_sel_workspace_bytes / nsa_sel_workspace_bytes_min)";
    case NSA_SEL_EHIP: return "HIP runtime error at launch";
    case NSA_SEL_ESTATIC:
      return "shape too large for nsa_sel_fwd_static: the partial results of one KV head (total_tokens * g * topk * "
             "260 bytes) exceed NSA_SEL_STATIC_WS_BYTES; use nsa_sel_fwd with a caller-owned workspace";
    default: return "unknown nsa_sel error code";
  }
}

}  // extern "C"
