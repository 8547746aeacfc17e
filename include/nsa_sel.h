/*
 * nsa_sel.h — C ABI of the MI355X (gfx950) selected-block attention library.
 *
 * The operation is the `sel` branch of Native Sparse Attention as stated in the FSA paper (arXiv 2508.18224),
 * Sec. 2.2 Eq. (2): every query token attends only to the keys/values of its own T selected KV blocks of
 * B_K contiguous tokens (64 or 128), shared by the g = hq/hkv query heads of a GQA group.  The library groups the
 * queries per selected KV block (the paper's KV-outer loop order, Sec. 3.1-3.2) so that the QK^T and PV
 * products are dense MFMA tiles with no padding of small query tiles.
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers; `shape` and the size_t outputs are HOST pointers.  Q, K, V, O, dO,
 *     dQ, dK, dV and the workspaces must be 16-byte aligned (NSA_SEL_EINVAL otherwise).
 *   - The library never allocates, frees or synchronises: every buffer, including workspaces, belongs to
 *     the caller, and all work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream).
 *   - Layouts are token-major and contiguous: Q, O, dO, dQ are bf16 [total_tokens, hq, d]; K, V, dK, dV are
 *     bf16 [total_tokens, hkv, d]; LSE is fp32 [total_tokens, hq] (natural log); query head h uses KV head
 *     h / g (contiguous groups).
 *   - idx is int32 [total_tokens, hkv, topk]: block ids LOCAL to the token's sequence.  Ids that are negative
 *     (padding), >= the sequence's block count, in the future of the token when causal, or a repeat of an
 *     earlier column of the same row are ignored (set semantics); they are data, not errors.
 *   - cu_seqlens is int32 [nseq + 1] (device), cumulative sequence starts, cu_seqlens[nseq] == total_tokens;
 *     it may be NULL when nseq == 1.  Sequences need not be multiples of 64; the last block is ragged.
 *   - A row with no visible key gets O = 0, LSE = -inf and contributes no gradient.
 *   - total_tokens == 0 is valid: the calls return NSA_SEL_OK without looking at the tensor pointers.
 *   - ws_bytes may lie anywhere between nsa_sel_workspace_bytes_min and nsa_sel_workspace_bytes (more is ignored).
 *   - Return value: 0 on success, a negative NSA_SEL_E* code otherwise.  Arguments are validated on the host
 *     before anything is launched; on error nothing has been enqueued (except NSA_SEL_EHIP, a launch failure).
 */
#ifndef NSA_SEL_H
#define NSA_SEL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NSA_SEL_OK            0
#define NSA_SEL_EINVAL       -1   /* null/misaligned pointer, g not in [1,8], hq % hkv != 0, nseq < 1, negative size,
                                     window < 0 or window without causal, unit not 0 or a power of two in range,
                                     dense outside [-1, 1] */
#define NSA_SEL_EUNSUPPORTED -2   /* d != 128, block not 64 or 128, topk outside [1,32], too many tokens      */
#define NSA_SEL_EWORKSPACE   -3   /* index workspace too small, or ws below nsa_sel_workspace_bytes_min       */
#define NSA_SEL_EHIP         -4   /* the HIP runtime refused a launch or attribute                            */
#define NSA_SEL_ESTATIC      -5   /* nsa_sel_fwd_static: shape beyond the library's built-in scratch array    */

/* Size of the device array nsa_sel_fwd_static keeps its partial results in (each GPU the library runs on holds one
 * copy until the process ends). */
#define NSA_SEL_STATIC_WS_BYTES (64u << 20)

typedef struct {
  int32_t total_tokens;   /* sum of sequence lengths (N when nseq == 1)                                      */
  int32_t nseq;           /* number of packed sequences, >= 1                                                */
  int32_t hq, hkv;        /* query / KV heads; g = hq / hkv must be an integer in [1, 8]                     */
  int32_t d;              /* head dimension; 128 only (every experiment of the paper uses d = 128)           */
  int32_t block;          /* B_K; 64 or 128 (the paper's two settings, Sec. 4.1)                             */
  int32_t topk;           /* T, selected blocks per (token, KV head); 1..32                                  */
  int32_t causal;         /* 1: key u visible to token t only if u <= t (per sequence); 0: no mask           */
  float   scale;          /* softmax scale; <= 0 selects 1/sqrt(d) (Eq. (1))                                 */
  int32_t max_seqlen;     /* upper bound of the longest sequence; informational, may be 0                    */
  int32_t window;         /* 0: none.  w > 0 (needs causal = 1): key u is visible to token t only if u > t - w;
                             a selected block wholly before the window is ignored like a future one.  With idx
                             listing the blocks a window can touch (the token's own and the ceil((w-1)/block)
                             before it; nsa_sel_select_blocks with scores = NULL writes that table) the path
                             computes the sliding-window term of Eq. (2), softmax over the last w tokens       */
  int32_t unit;           /* 0: the library picks.  Else the list entries one workgroup works through (a work
                             unit; the knob that corresponds to the paper's query batch size B_Q, App. E, which
                             it picks by online profiling): a power of two in [256, 2048].  It changes speed and
                             the workspace sizes, not results (dK/dV only in their fp32 summation order)      */
  int32_t dense;          /* Routing of the forward.  1: (query tile of 64 tokens, KV block) pairs that at least half
                             of the tile's tokens keep - found by counting, e.g. the attention-sink block (App. E) and
                             the tokens' own and neighbouring blocks - go through a query-tile-outer kernel, fused
                             with the reduction step, that needs no gather and no partial row.  -1: every pair
                             takes the gather route.  0: the library picks (the dense route when hq / hkv >= 2 or a
                             window is set, and total_tokens * hkv * topk >= 2^18).  Same results up to
                             rounding; an index workspace built for one routing must not be used with the
                             other                                                                             */
} nsa_sel_shape;

/* Bytes of the three caller-owned workspaces for `shape` (any of the outputs may be NULL).
 *   index_bytes: query lists and work-unit tables, written by nsa_sel_build_index / nsa_sel_fwd(rebuild_index=1)
 *                and read by nsa_sel_fwd / nsa_sel_bwd (the paper's index tensors I_i, O_i, which its
 *                backward pass reuses from the forward, Sec. 3.2);
 *   fwd_bytes:   per-(token, head, slot) partial outputs and log-sum-exps (the paper's O_buf, Sec. 3.2);
 *   bwd_bytes:   partial dQ, delta, and per-work-unit dK/dV partial sums. */
int nsa_sel_workspace_bytes(const nsa_sel_shape* shape, size_t* fwd_bytes, size_t* bwd_bytes, size_t* index_bytes);

/* Buffer reuse over head subsets (App. E, the paragraph on implementation details): nsa_sel_fwd / nsa_sel_bwd
 * also accept a ws smaller than the sizes above, down to the minima reported here (the partial results of ONE KV
 * head with its g query heads; for the backward plus the per-row statistics of all heads).  The library then
 * works through the KV heads in groups of as many heads as ws_bytes holds, one group after the other on the
 * stream, reusing the buffers; results are bit-identical to the single-pass ones.  Either output may be NULL. */
int nsa_sel_workspace_bytes_min(const nsa_sel_shape* shape, size_t* fwd_bytes, size_t* bwd_bytes);

/* Index inversion (Sec. 3.2: the index tensors are computed from the selection tensor T before the attention kernels run):
 * histogram -> exclusive scan -> ordered scatter.  For every list L = kv_head * b_cap + global_block
 * (b_cap = total_tokens / block + nseq; global blocks number the blocks of the packed sequences consecutively;
 * lists past the real block count are empty) the result holds the ascending tokens that validly select the
 * block and, per entry, the column of idx of the first occurrence.  Deterministic and bit-reproducible. */
int nsa_sel_build_index(const nsa_sel_shape* shape, const int32_t* idx, const int32_t* cu_seqlens,
                        void* index_ws, size_t index_bytes, void* stream);

/* Device pointers into a built index workspace (for inspection and tests): cnt int32 [hkv * b_cap],
 * off int32 [hkv * b_cap + 1] (exclusive prefix of cnt), qent int32 [off[last]][2] list entries as (token id,
 * column of idx) pairs, vmask uint32 [total_tokens * hkv] (bit m set: column m of the row was kept).
 * *b_cap receives the list stride.  Any output pointer may be NULL. */
int nsa_sel_index_view(const nsa_sel_shape* shape, const void* index_ws, const int32_t** cnt, const int32_t** off,
                       const int32_t** qent, const uint32_t** vmask, int32_t* b_cap);

/* Forward (Eq. (2), c = sel): O and LSE from Q, K, V, idx.  With rebuild_index != 0 the index workspace is
 * (re)built from idx first; with 0 it must hold the result of an earlier build for the same idx/shape. */
int nsa_sel_fwd(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O,
                float* LSE, void* ws, size_t ws_bytes, void* stream);

/* Backward of the above (Sec. 3.2, the closing sentences of the token-selection paragraph: the backward pass follows
 * the forward's KV-outer logic, takes the index tensors from the forward's cache and stores intermediate query
 * gradients to a buffer that a reduction kernel sums; the formulas are the derivative of Eq. (2), c = sel):
 * dQ, dK, dV from dO, the forward's O and LSE and the cached index workspace (the call takes no idx: the index
 * workspace written by nsa_sel_fwd / nsa_sel_build_index for the same idx and shape is its only view of the
 * selection).  dK/dV are accumulated without atomics (per-work-unit partial sums reduced in a fixed order), so
 * results are bit-reproducible.  ws: at least the backward size of nsa_sel_workspace_bytes_min. */
int nsa_sel_bwd(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const void* O,
                const float* LSE, const void* dO, const int32_t* cu_seqlens, const void* index_ws,
                size_t index_bytes, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, void* stream);

/* nsa_sel_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as nsa_sel_fwd (bit for bit)
 * minus ws / ws_bytes: the partial outputs and log-sum-exps live in a file-scope device array of the library of
 * NSA_SEL_STATIC_WS_BYTES (64 MiB).  The call allocates and frees nothing.  The partial results of ONE KV head,
 * total_tokens * (hq / hkv) * topk * 260 bytes (+ up to 512 bytes of alignment), must fit the array - e.g. 4032 tokens
 * at g = 4, topk = 16 - otherwise NSA_SEL_ESTATIC is returned and nothing is enqueued; when several KV heads fit they
 * share a pass, as with a capped ws.  The index workspace is still the caller's (it is an output the backward reads).
 * Every call on a GPU uses that GPU's one array and leaves its partial rows behind; nothing needs clearing between
 * calls, but two calls in flight on the same GPU at once (two streams, two threads) race on it and give wrong
 * results: serialise them.  The first call on a device looks up the array's address (hipGetSymbolAddress) and must
 * therefore be made outside graph capture; later calls only launch kernels. */
int nsa_sel_fwd_static(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                       const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O,
                       float* LSE, void* stream);

/* The same forward in QUERY-OUTER loop order, the order of the original NSA kernel (Sec. 2.2, 3.1; App. C): one
 * wavefront per (token, KV head) walks the row's selected blocks with an online softmax, re-loading a K/V block for
 * every (token, KV head, block).  The paper's fallback for many query heads per group (App. E) would dispatch to
 * this order; on this chip it does not win for any g <= 8, and the entry point exists for that comparison.  Needs no
 * workspace and no index; same O and LSE as nsa_sel_fwd up to rounding (fp32 accumulation over all blocks instead
 * of bf16 partial rows).  block must be 64 and window 0 (NSA_SEL_EUNSUPPORTED otherwise).  Forward only. */
int nsa_sel_fwd_query_outer(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                            const int32_t* cu_seqlens, void* O, float* LSE, void* stream);

/* Gated combination with the other attention branches, fused into the forward's merge kernel (the step after the
 * path; Eq. (2): the layer output is the sum over the branches c of tau^c_t times the branch's attention output).
 * Like nsa_sel_fwd, and in addition  O_out[t,h,:] = O_acc[t,h,:] + gate[t,h] * O[t,h,:],  formed from the fp32 result
 * before it is rounded.  gate is DEVICE fp32 [total_tokens, hq] (the paper's per-token gate broadcast over heads, or
 * per-head gates); O_acc is DEVICE bf16 [total_tokens, hq, d], the gated sum of the other branches, or NULL for
 * zero; O_out is DEVICE bf16 of the same shape and may be the buffer O_acc points to, but not O; O_acc must not be O
 * either (NSA_SEL_EINVAL).  O and LSE are still written ungated: the backward needs them. */
int nsa_sel_fwd_gated(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const int32_t* idx,
                      const int32_t* cu_seqlens, int rebuild_index, void* index_ws, size_t index_bytes, void* O,
                      float* LSE, const float* gate, const void* O_acc, void* O_out, void* ws, size_t ws_bytes,
                      void* stream);

/* Backward of nsa_sel_fwd_gated with respect to Q, K, V and gate: dO_out is the gradient of O_out (it is also the
 * gradient of O_acc, which this call does not touch), O and LSE are the forward's ungated outputs.  Writes dQ, dK,
 * dV as nsa_sel_bwd would for dO = gate * dO_out, and dgate[t,h] = <dO_out[t,h,:], O[t,h,:]> (DEVICE fp32
 * [total_tokens, hq]).  Gates must be >= 0 (the paper's lie in [0, 1]); a zero gate gives zero gradients for the row.
 * The gate costs no extra pass: it is folded into the per-row log-sum-exp the main kernel already gathers. */
int nsa_sel_bwd_gated(const nsa_sel_shape* shape, const void* Q, const void* K, const void* V, const void* O,
                      const float* LSE, const void* dO_out, const float* gate, const int32_t* cu_seqlens,
                      const void* index_ws, size_t index_bytes, void* dQ, void* dK, void* dV, float* dgate, void* ws,
                      size_t ws_bytes, void* stream);

/* The step in front of the path: block scores -> selection tensor, on the device, so that nsa_sel_build_index /
 * nsa_sel_fwd can consume idx without a host round trip.  The paper takes the selection tensor T as given
 * (Sec. 2.2) and notes only that block 0, the attention sink, is selected by every token (App. E); the rule used
 * here is: for token t (own block cur, sequence of b_s blocks) and KV head j,
 *   visible = blocks b < b_s, and b <= cur when shape->causal;
 *   forced  = the first n_sink blocks, then the n_local most recent ones (cur, cur - 1, ...), each once and only
 *             if visible;
 *   idx[t, j, :] = forced, then the other visible blocks by descending score (equal scores: smaller id first;
 *             NaN ranks as -infinity), cut to shape->topk columns, padded with -1.
 * scores is DEVICE fp32 [total_tokens, hkv, score_stride], column b = score of block b of the token's own sequence;
 * score_stride (floats, 1 .. 16384) must be at least the block count of the longest sequence; only visible,
 * non-forced columns are read.  scores may be NULL: then only the forced blocks are written (with n_sink = 0 and
 * n_local = topk = ceil((w - 1) / block) + 1 that is the block table of a sliding window of w tokens).  idx is DEVICE int32 [total_tokens, hkv, topk], fully overwritten.  Uses
 * shape->total_tokens, nseq, hkv, block, topk and causal; the other fields are ignored.  Exact: scores are only
 * compared, never altered.  16-byte loads are used when scores is 16-byte aligned and score_stride % 4 == 0. */
int nsa_sel_select_blocks(const nsa_sel_shape* shape, const float* scores, int64_t score_stride,
                          const int32_t* cu_seqlens, int32_t n_sink, int32_t n_local, int32_t* idx, void* stream);

/* Optional per-kernel timing for benchmarks (not part of the paper's method).  After
 * nsa_sel_profile_enable(capacity > 0) every kernel launch of the calls above is bracketed by a pair of HIP
 * events on the caller's stream, up to `capacity` launches (later ones are not recorded); capacity <= 0 turns
 * it off and frees the events.  nsa_sel_profile_collect waits for the recorded events, writes per kernel kind
 * its name, the summed milliseconds and the number of launches into the HOST arrays (each of max_kernels
 * entries), clears the record and returns the number of kinds written (or a negative code).  Launches of a group
 * that consists of several small kernels (the scans) are timed as one.
 * RESTRICTION: the record is one process-wide table (host memory; the event objects are created by enable and
 * destroyed by enable(0)).  While profiling is on, the library must be driven from ONE host thread on ONE stream:
 * calls from a second thread race on the table, and launches on a second stream would interleave their records
 * with the first's.  With profiling off (the default) the attention entry points touch no shared state. */
int nsa_sel_profile_enable(int capacity);
/* Restricts the recording to some kernel kinds: bit i of `mask` stands for the i-th name nsa_sel_profile_collect
 * reports (all bits set by default).  An event pair costs a few microseconds on the stream, so a benchmark that
 * times whole steps records only the kernels it needs inside its timed region. */
int nsa_sel_profile_select(unsigned mask);
int nsa_sel_profile_collect(int max_kernels, const char** names, float* total_ms, int* calls);

/* Measurement aid: a plain streaming copy kernel (k_calib_copy) that reads `bytes` and writes `bytes`
 * (device pointers, bytes a multiple of 16).  Hardware HBM byte counters of the attention kernels are scaled
 * by what the same counters report for this kernel of known traffic. */
int nsa_sel_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement aid: a register-resident loop of independent bf16 MFMA chains on every CU (no memory traffic).
 * Launches it with `iters` rounds per wavefront on `stream`; *flops (HOST, may be NULL) receives the number of
 * floating-point operations the launch performs, so that FLOPs / elapsed time is the matrix-core rate reachable
 * on the chip.  `sink` is a DEVICE float the kernel may write (never read back). */
int nsa_sel_mfma_probe(int iters, float* sink, double* flops, void* stream);

/* Static text for a return code. */
const char* nsa_sel_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* NSA_SEL_H */
