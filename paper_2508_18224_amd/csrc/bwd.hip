// Backward selected-block attention for gfx950.  The paper (Sec. 3.2) only says that the backward pass follows
// the forward's KV-outer logic, gathers the queries again through the cached index tensors and stores
// intermediate query gradients to a buffer that a reduction kernel sums; dK/dV accumulation is not described.
// This file is that pass, with dK/dV accumulated without atomics:
//
//   k_bwd_delta       delta[t,h] = <dO[t,h], O[t,h]>, stored next to LSE[t,h] log2(e) as one 8-byte pair so that the
//                     main kernel fetches both row statistics with one gather
//   k_bwd_tiled<NKB>  the main kernel for B_K = 64 (NKB = B_K / 32 = 2).  One work unit = (kv head j, KV block i, up to
//                     P.unit list entries): four wavefronts and half of a CU's LDS, so two workgroups share a CU and
//                     cover each other's barriers and waits.  The waves share tiles of 64 gathered rows and take three
//                     roles per tile (see the comment above the kernel): S = Q K_i^T, dP = dO V_i^T,
//                     P = exp(S - LSE), dS = P (dP - delta) scale; then dV_i += P^T dO and dK_i += dS^T Q
//                     (accumulators in registers for the whole unit) and dQ^T = K_i^T dS^T.  Operands are row-major
//                     tiles in LDS; "lane = column" operands are LDS transpose reads.  Partial dQ rows go to the
//                     compact buffer at the rows' list position; the unit's dK_i, dV_i go out as bf16 (list fitted
//                     the unit) or to a per-unit fp32 buffer.
//   k_bwd_pipe128     the main kernel for B_K = 128, same work units and outputs.  The fp32 dK_i / dV_i accumulators
//                     of a 128-key block fill the registers of four wavefronts, so one eight-wave workgroup owns the
//                     CU; its waves specialise (four compute P / dS of tile n, four accumulate tile n - 1) instead
//                     of all stepping through the same phases (see the comment above the kernel).
//   k_bwd_dq_reduce   dQ[t,h] = sum over kept slots of the partial rows
//   k_bwd_dkv_reduce  dK_i, dV_i = sum over the list's units in unit order (fixed order: bit-reproducible); a list
//                     that fitted one unit was already written by that unit, a list with no entry gets zeros
#include "common.h"
#include <type_traits>

namespace nsa {

// bf16 per row of the K / Q / dO tiles in LDS: 128 + 24 pad.  A 304-byte row pitch puts the rows
// of both access shapes used here (16-byte operand reads down a column of rows, and the 4-row x 32-byte footprint
// of a transposing read) on disjoint banks; with 128 + 8 the transposing reads conflicted two-way (measured:
// 45 % of LDS cycles were bank conflicts, 8 % kernel time).
constexpr int kRowStride = 152;

// ds_read_b64_tr_b16: every lane passes the address of 8 bytes (four 16-bit elements); within each group of
// 16 lanes, lane i receives element (i % 4) of the 8 bytes addressed by lanes 4e + i / 4, for e = 0..3.  With
// lane s of a group pointing at row (s / 4), columns 4 (s % 4).. of a row-major tile, lane i gets column i of
// four consecutive rows: the MFMA operand layout (lane = column, elements = rows) without a transposed copy.
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)(uint32_t)(uintptr_t)p);
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ void wave_sync_bwd() {  // orders a wavefront's own LDS traffic
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ void __launch_bounds__(256)
k_bwd_delta(int64_t rows, const bf16_t* __restrict__ O, const bf16_t* __restrict__ dO, const float* __restrict__ LSE,
            float2* __restrict__ stats, const float* __restrict__ gate, float* __restrict__ dgate) {
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
  if (row < rows && sub == 0) {
    float lse2 = LSE[row] * 1.4426950408889634f;
    if (gate != nullptr) {
      // Gated output (Eq. (2)): the gradient that reaches this branch is gate * dO.  Every place the main kernel
      // uses it carries a factor P = exp2(s - lse2) (dV += P^T dO, dS = P (dP - delta)), so the gate is folded into
      // the row's log-sum-exp, lse2 - log2(gate), and dO and delta stay as they are; a zero gate gives +inf, P = 0.
      // d(loss)/d(gate) is the same <dO, O> as delta.
      if (lse2 > -INFINITY) lse2 -= log2f(gate[row]);
      dgate[row] = acc;
    }
    stats[row] = make_float2(lse2, acc);
  }
}

// ---- the tiled backward main kernel ----------------------------------------------------------------------------
// NKB = B_K / 32 key blocks, 2 NKB wavefronts per workgroup, tiles of 64 gathered rows.
// With B_K = 64 (NKB = 2) a workgroup is four wavefronts (256 registers each) and half of a CU's LDS, so TWO
// workgroups share a CU and run out of phase: one's barriers, gather waits, unit prologue and LDS-bound phases are
// covered by the other's MFMA work (with one eight-wave workgroup per CU all waves sat in the same phase, and LDS,
// MFMA and VALU time simply added up).  The kernel is written for any NKB, but only NKB = 2 is built: with B_K = 128 the
// fp32 dK/dV accumulators leave room for one workgroup per CU only, and k_bwd_pipe128 below serves that case.
// Per tile, wave w takes three roles in turn:
//   rows/keys   (rb = w / NKB, kb = w % NKB): S = Q K_i^T, dP = dO V_i^T, P, dS for rows 32 rb.. and keys 32 kb..; K_i
//               fragments from LDS, V_i fragments of the wave's 32 keys held in registers for the whole unit (only this
//               role uses V_i).  The products are taken with lane = key, so that a lane holds four consecutive rows of
//               P^T / dS^T per register quad (one 8-byte LDS store); the rows' statistics come from a record per row
//               that the staging waves leave in LDS
//   keys/chans  (kb2 = w / 2, hf = w % 2): dV_i, dK_i accumulators for keys 32 kb2.. and channels 64 hf.. (two
//               32-channel blocks share every P^T / dS^T operand read)
//   rows/chans  (rb = w / NKB, part = w % NKB): dQ^T for rows 32 rb.. and the 128 / NKB channels of `part`; the same
//               wave stages / prefetches that part of the Q and dO tiles and stores that part of dQ
// K_i, Q, dO (304-byte pitch) and P^T, dS^T (144-byte pitch) are row-major tiles in LDS; "lane = column" operands
// are LDS transpose reads.  The list's token ids are kept in LDS 1024 entries at a time.
constexpr int kTile = 64;      // rows per tile
constexpr int kPStride = 72;   // bf16 per row of the P^T / dS^T tiles: 64 rows + 8 pad
constexpr int kEntSeg = 1024;  // list entries whose token ids are resident in LDS

template <int NKB>
struct BwdLds {
  static constexpr int kKeys = 32 * NKB;
  static constexpr int K = 0;
  static constexpr int Q = K + kKeys * kRowStride * 2;
  static constexpr int DO = Q + kTile * kRowStride * 2;
  static constexpr int Pt = DO + kTile * kRowStride * 2;
  static constexpr int DSt = Pt + kKeys * kPStride * 2;
  static constexpr int Ent = DSt + kKeys * kPStride * 2;
  static constexpr int Rec = Ent + kEntSeg * 4;    // per row of the tile: LSE (log2 domain), delta * scale, visible keys
  static constexpr int Bytes = Rec + 3 * kTile * 4;  // 81664 (NKB = 2)
};
static_assert(2 * BwdLds<2>::Bytes <= 160 * 1024, "two workgroups of the 64-key backward must fit one CU's LDS");

template <int NKB, bool kWin>
__global__ void __launch_bounds__(128 * NKB, NKB == 2 ? 2 : 1)
k_bwd_tiled(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
            const bf16_t* __restrict__ dO, const float2* __restrict__ stats, const int32_t* __restrict__ u_list,
            const int32_t* __restrict__ u_start, const int32_t* __restrict__ off,
            const int32_t* __restrict__ blk_tok0, const int32_t* __restrict__ blk_len,
            const int2* __restrict__ qent, const int32_t* __restrict__ nu_scan, bf16_t* __restrict__ dqpart,
            float* __restrict__ dkv_part, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV) {
  using Lds = BwdLds<NKB>;
  constexpr int kKeys = 32 * NKB;      // B_K
  constexpr int kThreads = 128 * NKB;
  constexpr int kCW = 128 / NKB;       // channels of the rows/chans part of a wave: 64 or 32
  constexpr int kNDB = kCW / 32;       // its 32-channel accumulator blocks: 2 or 1
  constexpr int kLPR = kCW / 8;        // lanes (16 bytes each) that cover the part's channels of one row: 8 or 4
  constexpr int kRPP = 64 / kLPR;      // rows staged per access: 8 or 16
  constexpr int kNP = 32 / kRPP;       // accesses per tile and tensor: 4 or 2
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem + Lds::K);
  bf16_t* Qs = reinterpret_cast<bf16_t*>(smem + Lds::Q);
  bf16_t* dOs = reinterpret_cast<bf16_t*>(smem + Lds::DO);
  bf16_t* Pt = reinterpret_cast<bf16_t*>(smem + Lds::Pt);
  bf16_t* dSt = reinterpret_cast<bf16_t*>(smem + Lds::DSt);
  int32_t* ent = reinterpret_cast<int32_t*>(smem + Lds::Ent);

  const int ubase = nu_scan[P.j0 * P.b_cap];
  const int u = ubase + blockIdx.x;
  if (u >= nu_scan[(P.j0 + P.nj) * P.b_cap]) return;
  const int L = u_list[u];
  const int j = L / P.b_cap;
  const int gb = L - j * P.b_cap;
  const int e0 = u_start[u];
  const int pos0 = off[P.j0 * P.b_cap];
  const int ne = min(P.unit, off[L + 1] - e0);
  const int tok0 = blk_tok0[gb], blen = blk_len[gb];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int col = lane & 31, qh = lane >> 5;  // not const: made opaque at the top of the tile loop
  const int rb = wave / NKB, kb = wave % NKB;   // rows/keys role; rows/chans role uses (rb, part = kb)
  const int kb2 = wave >> 1, hf = wave & 1;     // keys/chans role
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  {  // K_i -> LDS, row-major; rows past the end of a ragged block are zero
    const int key = tid >> 2, d0 = (tid & 3) * 32;
    const bf16_t* src = K + ((size_t)(tok0 + key) * P.hkv + j) * kD + d0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<bf16x8*>(&Ks[key * kRowStride + d0 + 8 * i]) =
          key < blen ? *reinterpret_cast<const bf16x8*>(src + 8 * i) : zero8;
  }
  bf16x8 vf[8];  // V_i fragments of keys 32 kb.. (A operand of dP^T = V_i dO^T)
  {
    const int key = 32 * kb + col;
    const bf16_t* src = V + ((size_t)(tok0 + key) * P.hkv + j) * kD + 8 * qh;
#pragma unroll
    for (int s = 0; s < 8; ++s) vf[s] = key < blen ? *reinterpret_cast<const bf16x8*>(src + 16 * s) : zero8;
  }
  f32x16 dkacc[2], dvacc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      dkacc[cb][v] = 0.f;
      dvacc[cb][v] = 0.f;
    }

  const float c2 = P.scale * 1.4426950408889634f;
  const int hbase = j * P.g;
  const int grp = lane >> 4, sl = lane & 15;
  // this lane's share of a transposing read of four rows x 16 columns (see lds_read_tr), for the two row pitches
  int tr_lane = ((sl >> 2) + 8 * (grp >> 1)) * kRowStride + 16 * (grp & 1) + 4 * (sl & 3);
  int tr_lane_p = ((sl >> 2) + 8 * (grp >> 1)) * kPStride + 16 * (grp & 1) + 4 * (sl & 3);
  // staging layout of this wave's part: kLPR lanes x 16 B cover its channels of a row, kRPP rows per access
  int srow = lane / kLPR, schunk = kCW * kb + (lane % kLPR) * 8;
  bf16_t* Qmine = Qs + (32 * rb) * kRowStride;
  bf16_t* dOmine = dOs + (32 * rb) * kRowStride;

  u32x4 qc[kNP], dc[kNP];
  float lse2_n, dl_n;
  int seg0 = 0;  // first list entry whose token id is in `ent`
  int rows_end = 0;
  auto issue_rows = [&](int tile0) {
    // rows past the end of the list re-read its last row: their P and dS are forced to zero (lim = 0) and their
    // dQ is never stored, so no branch and no zero fill is needed
#pragma unroll
    for (int i = 0; i < kNP; ++i) {
      const int r = min(tile0 + 32 * rb + kRPP * i + srow, rows_end - 1);
      const int e = div_g(r, P.g, P.g_magic);
      // (token, head) row index in 32 bits (total_tokens * hq < 2^31 is checked on the host), widened once
      const uint32_t grow = (uint32_t)ent[e - seg0] * (uint32_t)P.hq + (uint32_t)(hbase + (r - e * P.g));
      const size_t o = (size_t)grow * kD + schunk;
      qc[i] = *reinterpret_cast<const u32x4*>(Q + o);
      dc[i] = *reinterpret_cast<const u32x4*>(dO + o);
    }
    const int rc = min(tile0 + 32 * rb + col, rows_end - 1);
    const int ec = div_g(rc, P.g, P.g_magic);
    const float2 st = stats[(uint32_t)ent[ec - seg0] * (uint32_t)P.hq + (uint32_t)(hbase + (rc - ec * P.g))];  // (LSE in log2 domain, delta)
    lse2_n = st.x;
    dl_n = st.y;
  };

  for (seg0 = 0; seg0 < ne; seg0 += kEntSeg) {
    const int seg_n = min(kEntSeg, ne - seg0);
    __syncthreads();  // the previous segment's ids are no longer read
    for (int i = tid; i < seg_n; i += kThreads) ent[i] = qent[e0 + seg0 + i].x;
    __syncthreads();  // ids (and K_i on the first pass) visible
    rows_end = (seg0 + seg_n) * P.g;
    issue_rows(seg0 * P.g);

    for (int tile0 = seg0 * P.g; tile0 < rows_end; tile0 += kTile) {
      // keep the lane-derived LDS addresses from being precomputed and held across the loop (register budget)
      asm volatile("" : "+v"(col), "+v"(qh), "+v"(tr_lane), "+v"(tr_lane_p), "+v"(srow), "+v"(schunk));
#pragma unroll
      for (int i = 0; i < kNP; ++i) {
        *reinterpret_cast<u32x4*>(&Qmine[(kRPP * i + srow) * kRowStride + schunk]) = qc[i];
        *reinterpret_cast<u32x4*>(&dOmine[(kRPP * i + srow) * kRowStride + schunk]) = dc[i];
      }
      const float lse2 = lse2_n, dl = dl_n;
      const bool more = tile0 + kTile < rows_end;
      if (more) issue_rows(tile0 + kTile);  // the next tile's rows fly while this one computes
      const int r = tile0 + 32 * rb + col;
      const bool valid = r < rows_end;
      const int t = valid ? ent[div_g(r, P.g, P.g_magic) - seg0] : -1;
      int lim = P.causal ? min(blen, t - tok0 + 1) : blen;  // keys [0, lim) of the block are visible to this row
      if (!valid) lim = 0;
      // kWin: the kernel variant for a sliding window, whose rows also hide the keys before lo
      const int lo = kWin ? min(max(t - P.window + 1 - tok0, 0), kKeys) : 0;
      if (kb == 0 && qh == 0) {  // this row's record, for the lanes of the rows/keys role (which hold keys, not rows)
        float* rec = reinterpret_cast<float*>(smem + Lds::Rec) + 32 * rb + col;
        rec[0] = lse2;
        rec[kTile] = dl * P.scale;
        reinterpret_cast<uint32_t*>(rec)[2 * kTile] = (uint32_t)(lo | (max(lim - lo, 0) << 16));  // keys [lo, lo + span)
      }
      __syncthreads();  // Q / dO tile and the row records staged by all waves

      {  // role rows/keys: S = Q K_i^T, dP = dO V_i^T for rows 32 rb.. x keys 32 kb..: lane = key, register v = row
         // 8 (v >> 2) + 4 qh + (v & 3), so four consecutive rows of P^T / dS^T leave each lane as one 8-byte LDS store
        f32x16 sacc, dpacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          sacc[v] = 0.f;
          dpacc[v] = 0.f;
        }
        const bf16_t* qrow = Qmine + col * kRowStride + 8 * qh;
        const bf16_t* drow = dOmine + col * kRowStride + 8 * qh;
        const bf16_t* krow = Ks + (32 * kb + col) * kRowStride + 8 * qh;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qrow + 16 * s);
          const bf16x8 dof = *reinterpret_cast<const bf16x8*>(drow + 16 * s);
          const bf16x8 kfa = *reinterpret_cast<const bf16x8*>(krow + 16 * s);
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kfa, sacc, 0, 0, 0);
          dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dof, vf[s], dpacc, 0, 0, 0);
        }
        const float* rec = reinterpret_cast<const float*>(smem + Lds::Rec);
        const int key = 32 * kb + col;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const int r4 = 32 * rb + 8 * a + 4 * qh;
          const f32x4 lse4 = *reinterpret_cast<const f32x4*>(rec + r4);
          const f32x4 dls4 = *reinterpret_cast<const f32x4*>(rec + kTile + r4);
          const u32x4 vis4 = *reinterpret_cast<const u32x4*>(rec + 2 * kTile + r4);
          float p[4], ds[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const bool seen = (uint32_t)key - (vis4[c] & 0xffffu) < (vis4[c] >> 16);
            p[c] = seen ? __builtin_amdgcn_exp2f(fmaf(sacc[4 * a + c], c2, -lse4[c])) : 0.f;
            ds[c] = p[c] * fmaf(dpacc[4 * a + c], P.scale, -dls4[c]);  // P (dP - delta) scale
          }
          uint2 pw, sw2;
          pw.x = pack_bf16x2(p[0], p[1]);
          pw.y = pack_bf16x2(p[2], p[3]);
          sw2.x = pack_bf16x2(ds[0], ds[1]);
          sw2.y = pack_bf16x2(ds[2], ds[3]);
          *reinterpret_cast<uint2*>(&Pt[key * kPStride + r4]) = pw;
          *reinterpret_cast<uint2*>(&dSt[key * kPStride + r4]) = sw2;
        }
      }
      __syncthreads();  // P^T, dS^T complete
      {  // role keys/chans: dV_i += P^T dO, dK_i += dS^T Q for keys 32 kb2.., channels 64 hf + 32 cb..
        int tr_row = tr_lane + 64 * hf;
        asm volatile("" : "+v"(tr_row));
        const bf16_t* do_tr = dOs + tr_row;  // one base per tile: the reads below differ by immediate offsets only
        const bf16_t* q_tr = Qs + tr_row;
        const bf16_t* parow = Pt + (32 * kb2 + col) * kPStride + 8 * qh;
        const bf16_t* sarow = dSt + (32 * kb2 + col) * kPStride + 8 * qh;
#pragma unroll
        for (int qs = 0; qs < 4; ++qs) {
          const bf16x8 pa = *reinterpret_cast<const bf16x8*>(parow + 16 * qs);
          const bf16x8 sa = *reinterpret_cast<const bf16x8*>(sarow + 16 * qs);
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) {
            const bf16x4 d0 = lds_read_tr(do_tr + (16 * qs * kRowStride + 32 * cb));
            const bf16x4 d1 = lds_read_tr(do_tr + ((16 * qs + 4) * kRowStride + 32 * cb));
            const bf16x4 q0 = lds_read_tr(q_tr + (16 * qs * kRowStride + 32 * cb));
            const bf16x4 q1 = lds_read_tr(q_tr + ((16 * qs + 4) * kRowStride + 32 * cb));
            const bf16x8 dob = __builtin_shufflevector(d0, d1, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 qb = __builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7);
            dvacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa, dob, dvacc[cb], 0, 0, 0);
            dkacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa, qb, dkacc[cb], 0, 0, 0);
          }
        }
      }
      f32x16 dqacc[kNDB];
      {  // role rows/chans: dQ^T[kCW kb.., 32 rb..] = K_i^T dS^T over the block's keys
#pragma unroll
        for (int db = 0; db < kNDB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) dqacc[db][v] = 0.f;
        int tr_key = tr_lane + kCW * kb;
        int tr_ds = tr_lane_p + 32 * rb;
        asm volatile("" : "+v"(tr_key), "+v"(tr_ds));
        const bf16_t* k_tr = Ks + tr_key;
        const bf16_t* ds_tr = dSt + tr_ds;
#pragma unroll
        for (int sp = 0; sp < kKeys / 16; ++sp) {
          const bf16x4 b0 = lds_read_tr(ds_tr + 16 * sp * kPStride);
          const bf16x4 b1 = lds_read_tr(ds_tr + (16 * sp + 4) * kPStride);
          const bf16x8 dsb = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
          for (int db = 0; db < kNDB; ++db) {
            const bf16x4 a0 = lds_read_tr(k_tr + (16 * sp * kRowStride + 32 * db));
            const bf16x4 a1 = lds_read_tr(k_tr + ((16 * sp + 4) * kRowStride + 32 * db));
            const bf16x8 ktf = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
            dqacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsb, dqacc[db], 0, 0, 0);
          }
        }
      }
      __syncthreads();  // every wave is done reading the Q / dO / P^T / dS^T tiles
      // dQ rows (32 rows x kCW channels) -> the part of the Q tile this wave staged -> contiguous row segments
#pragma unroll
      for (int db = 0; db < kNDB; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          uint2 w;
          w.x = pack_bf16x2(dqacc[db][4 * a + 0], dqacc[db][4 * a + 1]);
          w.y = pack_bf16x2(dqacc[db][4 * a + 2], dqacc[db][4 * a + 3]);
          *reinterpret_cast<uint2*>(&Qmine[col * kRowStride + kCW * kb + 32 * db + 8 * a + 4 * qh]) = w;
        }
      wave_sync_bwd();
      const size_t prow0 = (size_t)(e0 - pos0) * P.g + (size_t)(tile0 + 32 * rb);
#pragma unroll
      for (int i = 0; i < kNP; ++i) {
        const int row = kRPP * i + srow;
        if (tile0 + 32 * rb + row < rows_end)
          store_streaming(dqpart + (prow0 + row) * kD + schunk,
                          *reinterpret_cast<const uint4*>(&Qmine[row * kRowStride + schunk]));
      }
      wave_sync_bwd();
    }
  }

  if (nu_scan[L + 1] - nu_scan[L] == 1) {
    // the whole list fitted this unit: dK_i, dV_i are final, write them as bf16 (keys of a ragged tail excluded)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      bf16_t* outk = dK + ((size_t)tok0 * P.hkv + j) * kD + 64 * hf + 32 * cb + col;
      bf16_t* outv = dV + ((size_t)tok0 * P.hkv + j) * kD + 64 * hf + 32 * cb + col;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * kb2 + 8 * (v >> 2) + 4 * qh + (v & 3);
        if (key < blen) {
          outk[(size_t)key * P.hkv * kD] = (bf16_t)dkacc[cb][v];
          outv[(size_t)key * P.hkv * kD] = (bf16_t)dvacc[cb][v];
        }
      }
    }
    return;
  }
  // unit partial: [u][0 = dK, 1 = dV][key][d] fp32, summed by k_bwd_dkv_reduce in unit order
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    float* outk = dkv_part + (size_t)(u - ubase) * 2 * kKeys * kD + 64 * hf + 32 * cb + col;
    float* outv = outk + kKeys * kD;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 32 * kb2 + 8 * (v >> 2) + 4 * qh + (v & 3);
      outk[key * kD] = dkacc[cb][v];
      outv[key * kD] = dvacc[cb][v];
    }
  }
}

// ---- pipelined backward main kernel for 128-key blocks -----------------------------------------------------------
// With B_K = 128 the fp32 dK / dV accumulators of a block (128 KB) need the registers of four wavefronts and leave room
// for one eight-wave workgroup per CU.  If all eight waves step through the same phases of a tile (products, exponentials,
// accumulation), MFMA, VALU and LDS time add up and every LDS read waits out its latency: two waves per SIMD cannot
// cover each other.  Here the waves specialise and work one tile apart:
//   waves 0-3 (S-waves, one per SIMD): wave w keeps the K and V fragments of keys 32 w.. in registers and computes, for
//       the 64 rows of tile n, S = Q K^T, dP = dO V^T, P = exp(S - LSE), dS = P (dP - delta) scale, and writes
//       P^T, dS^T (bf16, [key][row]) to LDS; they also request and stage the gathered Q / dO rows;
//   waves 4-7 (A-waves, the other wave of each SIMD): wave a keeps the fp32 dK, dV accumulators of keys 32 a.. (all 128
//       channels) and the K^T fragments of channels 32 a.., and for tile n - 1 computes dV += P^T dO, then
//       dQ^T = K^T dS^T (channels 32 a.., all 128 keys; its 64-byte slice of every dQ row is stored at once), then
//       dK += dS^T Q; they also work out the row addresses of tile n + 3 for the S-waves.
// Q / dO tiles and P^T / dS^T tiles are double-buffered in LDS (154 KB in all), so the S-waves' MFMA and exponential work
// on tile n runs beside the A-waves' LDS-bound products on tile n - 1 on the same SIMD; two block-wide barriers per
// tile order the hand-over.  Rows are requested three tiles ahead into two register sets and staged after the second
// barrier.  Measured at 65536 tokens, g = 4, (128, 8): 3.5 ms against 4.1 ms for the eight-waves-in-step kernel.
struct PipeLds {
  static constexpr int QB = kTile * kRowStride * 2;   // one Q or dO tile: 19456 bytes
  static constexpr int PB = 128 * kPStride * 2;       // one P^T or dS^T tile: 18432 bytes
  static constexpr int Q0 = 0;
  static constexpr int DO0 = Q0 + 2 * QB;
  static constexpr int Pt0 = DO0 + 2 * QB;
  static constexpr int DSt0 = Pt0 + 2 * PB;
  static constexpr int Ent = DSt0 + 2 * PB;
  static constexpr int St0 = Ent + kEntSeg * 4;       // per-row records of a staged tile, two buffers: three arrays
  static constexpr int SB = 3 * kTile * 4;            // of 64: LSE (log2 domain), delta * scale, visible key range
  static constexpr int Tb0 = St0 + 2 * SB;            // per row of the tile to request next: (row index into Q / dO /
  static constexpr int Bytes = Tb0 + kTile * 8;       // stats, visible key range); 157696 in all
};
static_assert(PipeLds::Bytes <= 160 * 1024, "the pipelined 128-key backward must fit one CU's LDS");
constexpr int kDqPitch = 36;  // bf16 per row of an A-wave's dQ staging (64 rows x 32 channels + pad = 4608 bytes)
static_assert(64 * kDqPitch <= 32 * kPStride, "dQ staging must fit the wave's 32 rows of a P^T tile");

// Built with -DNSA_PIPE_TIMING the pipelined kernel adds up, per role, the clocks its waves spend waiting at the two
// barriers, computing, and between them (a measuring build only: the stamps drain the LDS queue and cost a few percent).
#ifdef NSA_PIPE_TIMING
__device__ unsigned long long g_pipe_t[2][8];
#define PT_STAMP(k) { const unsigned long long now_ = clock64(); pt[k] += now_ - pt_last; pt_last = now_; }
#else
#define PT_STAMP(k)
#endif
// f(integral_constant<int, I>) for I = kBegin .. kEnd - 1, every index a compile-time constant
template <int kBegin, int kEnd, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (kBegin < kEnd) {
    f(std::integral_constant<int, kBegin>{});
    static_for<kBegin + 1, kEnd>(f);
  }
}

// What one workgroup of k_bwd_pipe128 works on.
struct PipeUnit {
  int u, ubase, L, j, e0, pos0, ne, tok0, blen;
};

// One role of the pipeline (kS: an S-wave, else an A-wave).  Both roles run this same skeleton, so they execute the same
// sequence of block-wide barriers: every loop bound below depends only on the unit, never on the role or the lane.
template <bool kWin, bool kS>
__device__ __forceinline__ void
pipe_role(const Problem& P, const PipeUnit& U, unsigned char* smem, const int sw, const bf16_t* __restrict__ Q,
          const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO,
          const float2* __restrict__ stats, const int2* __restrict__ qent, const int32_t* __restrict__ nu_scan,
          bf16_t* __restrict__ dqpart, float* __restrict__ dkv_part, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV) {
  int32_t* ent = reinterpret_cast<int32_t*>(smem + PipeLds::Ent);
  const int tid = threadIdx.x, lane = tid & 63;
  int col = lane & 31, qh = lane >> 5;
  const int j = U.j, tok0 = U.tok0, blen = U.blen;
  const float c2 = P.scale * 1.4426950408889634f;
  const int hbase = j * P.g;
  const int grp = lane >> 4, sl = lane & 15;
  int tr_lane = ((sl >> 2) + 8 * (grp >> 1)) * kRowStride + 16 * (grp & 1) + 4 * (sl & 3);
  int tr_lane_p = ((sl >> 2) + 8 * (grp >> 1)) * kPStride + 16 * (grp & 1) + 4 * (sl & 3);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  // register-resident operands.  S-wave: kf = K_i, vf = V_i fragments of keys 32 sw.. (A operands of S^T and dP^T).
  // A-wave: kf = K_i^T fragments of channels 32 sw.. (A operand of dQ^T; element e of step sp = key 16 sp + 8 qh + e).
  bf16x8 kf[8], vf[kS ? 8 : 1];
  if constexpr (kS) {
    const int key = 32 * sw + col;
    const size_t o = ((size_t)(tok0 + min(key, blen - 1)) * P.hkv + j) * kD + 8 * qh;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 kk = *reinterpret_cast<const bf16x8*>(K + o + 16 * s);
      const bf16x8 vv = *reinterpret_cast<const bf16x8*>(V + o + 16 * s);
      kf[s] = key < blen ? kk : zero8;
      vf[s] = key < blen ? vv : zero8;
    }
  } else {
    const bf16_t* src = K + ((size_t)tok0 * P.hkv + j) * kD + 32 * sw + col;
#pragma unroll
    for (int sp = 0; sp < 8; ++sp)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = 16 * sp + 8 * qh + e;
        const bf16_t kk = src[(size_t)min(key, blen - 1) * P.hkv * kD];
        kf[sp][e] = key < blen ? kk : (bf16_t)0.f;
      }
  }
  f32x16 dkacc[kS ? 1 : 4], dvacc[kS ? 1 : 4];  // A-wave: keys 32 sw.., by 32-channel block
  if constexpr (!kS) {
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        dkacc[cb][v] = 0.f;
        dvacc[cb][v] = 0.f;
      }
  }

  // S-waves stage the 64-row tiles: access i of thread t covers row 16 i + (t >> 4), 16 bytes at channel 8 (t & 15).
  // Rows are requested three tiles ahead of the S-waves' own use into two register sets (tile parity), so two tiles
  // (64 KB per CU) are in flight while one is computed: one tile in flight leaves the loop waiting on HBM latency.
  const int srow = (tid & 255) >> 4, schunk = (tid & 15) * 8;
  u32x4 qc[kS ? 2 : 1][kS ? 4 : 1], dc[kS ? 2 : 1][kS ? 4 : 1];
  // row record of row (t >> 2) of a requested tile, staged like the rows: (LSE in the log2 domain, delta) and the
  // block's keys the row sees, [lo, lo + span), as lo | span << 16
  float2 st_set[2];
  int vis_set[2];
  int seg0 = 0, rows_end = 0;
  // The row table of a tile: for each of its 64 rows the (token, head) row index into Q / dO / stats and the block's
  // keys the row sees.  It is worked out one phase before the loads are issued, by whichever waves have the time
  // (all of them before the pipeline starts, the A-waves inside it) and handed over in LDS, so that the S-waves carry
  // no addresses through their products and issue the loads right after the barrier that frees the registers.
  uint2* row_table = reinterpret_cast<uint2*>(smem + PipeLds::Tb0);
  auto prepare_rows = [&](int tile0) __attribute__((always_inline)) {
    // rows past the end of the list re-read its last row: their P and dS are forced to zero and their dQ is never stored
    const int rr = tile0 + ((tid & 255) >> 2);
    const int rc = min(rr, rows_end - 1);
    const int ec = div_g(rc, P.g, P.g_magic);
    const int t = ent[ec - seg0];
    int lim = P.causal ? min(blen, t - tok0 + 1) : blen;  // keys [lo, lim) of the block are visible to this row
    if (rr >= rows_end) lim = 0;
    const int lo = kWin ? min(max(t - P.window + 1 - tok0, 0), 128) : 0;
    if ((tid & 3) == 0)
      row_table[(tid & 255) >> 2] = make_uint2((uint32_t)t * (uint32_t)P.hq + (uint32_t)(hbase + (rc - ec * P.g)),
                                               (uint32_t)(lo | (max(lim - lo, 0) << 16)));
  };
  auto issue_rows = [&](auto setc) __attribute__((always_inline)) {
    constexpr int set = kS ? decltype(setc)::value : 0;
    uint32_t grow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) grow[i] = row_table[16 * i + srow].x;
    const uint2 mine = row_table[(tid & 255) >> 2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const size_t o = (size_t)grow[i] * kD + schunk;
      qc[set][i] = *reinterpret_cast<const u32x4*>(Q + o);
      dc[set][i] = *reinterpret_cast<const u32x4*>(dO + o);
    }
    st_set[set] = stats[mine.x];
    vis_set[set] = (int)mine.y;
  };
  auto stage_rows = [&](int buf, auto setc) __attribute__((always_inline)) {
    constexpr int set = kS ? decltype(setc)::value : 0;
    bf16_t* Qs = reinterpret_cast<bf16_t*>(smem + PipeLds::Q0 + buf * PipeLds::QB);
    bf16_t* dOs = reinterpret_cast<bf16_t*>(smem + PipeLds::DO0 + buf * PipeLds::QB);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<u32x4*>(&Qs[(16 * i + srow) * kRowStride + schunk]) = qc[set][i];
      *reinterpret_cast<u32x4*>(&dOs[(16 * i + srow) * kRowStride + schunk]) = dc[set][i];
    }
    if ((tid & 3) == 0) {
      float* rec = reinterpret_cast<float*>(smem + PipeLds::St0 + buf * PipeLds::SB) + ((tid & 255) >> 2);
      rec[0] = st_set[set].x;
      rec[kTile] = st_set[set].y * P.scale;
      reinterpret_cast<int*>(rec)[2 * kTile] = vis_set[set];
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;

#ifdef NSA_PIPE_TIMING
  unsigned long long pt[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pt_last = clock64();
#endif
  for (seg0 = 0; seg0 < U.ne; seg0 += kEntSeg) {
    const int seg_n = min(kEntSeg, U.ne - seg0);
    __syncthreads();  // the previous segment's ids and tiles are no longer read
    for (int i = tid; i < seg_n; i += 512) ent[i] = qent[U.e0 + seg0 + i].x;
    __syncthreads();
    const int row_first = seg0 * P.g;
    rows_end = (seg0 + seg_n) * P.g;
    const int ntiles = (rows_end - row_first + kTile - 1) / kTile;
    // start of the pipeline: tiles 0, 1, 2 requested, tile 0 staged (one table, so a barrier pair per tile)
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      if constexpr (kS) prepare_rows(row_first + k * kTile);
      __syncthreads();
      if constexpr (kS) {
        if (k == 0) {
          issue_rows(Set0{});
          stage_rows(0, Set0{});
        } else if (k == 1) {
          issue_rows(Set1{});
        } else {
          issue_rows(Set0{});
        }
      }
      __syncthreads();
    }

    // one pipeline step: S-waves work on tile `it`, A-waves on tile `it - 1`; `par` = parity of `it`
    auto step = [&](const int it, auto par) __attribute__((always_inline)) {
      using Other = std::integral_constant<int, 1 - decltype(par)::value>;
      asm volatile("" : "+v"(col), "+v"(qh), "+v"(tr_lane), "+v"(tr_lane_p));
      PT_STAMP(3)
      __syncthreads();  // tile `it` staged; P^T / dS^T of tile `it - 1` complete
      PT_STAMP(0)
      if constexpr (kS) {
        if (it < ntiles) {  // ---- S, dP, P, dS of tile `it`: keys 32 sw.., all 64 rows
          const int buf = it & 1, tile0 = row_first + it * kTile;
          const bf16_t* Qs = reinterpret_cast<const bf16_t*>(smem + PipeLds::Q0 + buf * PipeLds::QB);
          const bf16_t* dOs = reinterpret_cast<const bf16_t*>(smem + PipeLds::DO0 + buf * PipeLds::QB);
          bf16_t* Pt = reinterpret_cast<bf16_t*>(smem + PipeLds::Pt0 + buf * PipeLds::PB);
          bf16_t* dSt = reinterpret_cast<bf16_t*>(smem + PipeLds::DSt0 + buf * PipeLds::PB);
          // S = Q K_i^T, dP = dO V_i^T for rows 32 rb.. x keys 32 sw..: lane = key, register v = row 8 (v >> 2) + 4 qh
          // + (v & 3), so four consecutive rows of P^T / dS^T leave each lane as one 8-byte LDS store.
          // Issue order, fixed by hand: a wave issues in order and only two waves share a SIMD, so an LDS read that
          // is waited for right before its MFMA exposes the whole LDS latency each time.  The four products (S, dP of
          // two row blocks) run as one software pipeline over a ring of eight fragment registers: step s issues the
          // MFMA on fragment s, refills that register with fragment s of the NEXT product, and does one eighth of the
          // elementwise work on the PREVIOUS product's result.
          f32x16 sacc[2], dpacc[2];
          float pv[2][16];
          bf16x8 fr[8];
          const float* rec = reinterpret_cast<const float*>(smem + PipeLds::St0 + buf * PipeLds::SB);
          const int key = 32 * sw + col;
          const bf16_t* q0 = Qs + col * kRowStride + 8 * qh;
          const bf16_t* d0 = dOs + col * kRowStride + 8 * qh;
          f32x4 lse4, dls4;
          u32x4 vis4;
          auto probs = [&](int rb, int st) __attribute__((always_inline)) {  // P = exp(S scale - LSE) on visible keys
            const int a = st >> 1, r4 = 32 * rb + 8 * a + 4 * qh;
            if ((st & 1) == 0) {
              lse4 = *reinterpret_cast<const f32x4*>(rec + r4);
              vis4 = *reinterpret_cast<const u32x4*>(rec + 2 * kTile + r4);
            }
#pragma unroll
            for (int c = 2 * (st & 1); c < 2 * (st & 1) + 2; ++c) {
              const bool seen = (uint32_t)key - (vis4[c] & 0xffffu) < (vis4[c] >> 16);
              pv[rb][4 * a + c] = seen ? __builtin_amdgcn_exp2f(fmaf(sacc[rb][4 * a + c], c2, -lse4[c])) : 0.f;
            }
          };
          auto emit = [&](int rb, int st) __attribute__((always_inline)) {  // dS = P (dP - delta) scale; bf16 to LDS
            const int a = st >> 1, r4 = 32 * rb + 8 * a + 4 * qh;
            if ((st & 1) == 0) {
              dls4 = *reinterpret_cast<const f32x4*>(rec + kTile + r4);
              uint2 pw;
              pw.x = pack_bf16x2(pv[rb][4 * a + 0], pv[rb][4 * a + 1]);
              pw.y = pack_bf16x2(pv[rb][4 * a + 2], pv[rb][4 * a + 3]);
              *reinterpret_cast<uint2*>(&Pt[key * kPStride + r4]) = pw;
            } else {
              float ds[4];
#pragma unroll
              for (int c = 0; c < 4; ++c) ds[c] = pv[rb][4 * a + c] * fmaf(dpacc[rb][4 * a + c], P.scale, -dls4[c]);
              uint2 sw2;
              sw2.x = pack_bf16x2(ds[0], ds[1]);
              sw2.y = pack_bf16x2(ds[2], ds[3]);
              *reinterpret_cast<uint2*>(&dSt[key * kPStride + r4]) = sw2;
            }
          };
#pragma unroll
          for (int v = 0; v < 16; ++v) sacc[0][v] = dpacc[0][v] = sacc[1][v] = dpacc[1][v] = 0.f;
#pragma unroll
          for (int st = 0; st < 8; ++st) fr[st] = *reinterpret_cast<const bf16x8*>(q0 + 16 * st);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int st = 0; st < 8; ++st) {  // S, rows 0..31; refill with dO, rows 0..31
            sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st], kf[st], sacc[0], 0, 0, 0);
            fr[st] = *reinterpret_cast<const bf16x8*>(d0 + 16 * st);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int st = 0; st < 8; ++st) {  // dP, rows 0..31; refill with Q, rows 32..63; P of rows 0..31
            dpacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st], vf[st], dpacc[0], 0, 0, 0);
            fr[st] = *reinterpret_cast<const bf16x8*>(q0 + 32 * kRowStride + 16 * st);
            probs(0, st);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int st = 0; st < 8; ++st) {  // S, rows 32..63; refill with dO, rows 32..63; dS of rows 0..31
            sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st], kf[st], sacc[1], 0, 0, 0);
            fr[st] = *reinterpret_cast<const bf16x8*>(d0 + 32 * kRowStride + 16 * st);
            emit(0, st);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int st = 0; st < 8; ++st) {  // dP, rows 32..63; P of rows 32..63
            dpacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st], vf[st], dpacc[1], 0, 0, 0);
            probs(1, st);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int st = 0; st < 8; ++st) emit(1, st);
        }
        PT_STAMP(1)
        __syncthreads();  // every wave is done with the tiles of `it - 1`: stage tile `it + 1` there, request `it + 2`
        PT_STAMP(2)
        // unconditional (tiles past the end re-read the list's last row and are never used): with no branch around
        // the loads the compiler's wait counts stay exact and the newer set's loads are left in flight here
        stage_rows((it + 1) & 1, Other{});
        issue_rows(Other{});
      } else {
        const int buf = (it - 1) & 1;
        prepare_rows(row_first + (it + 3) * kTile);  // read by the S-waves after this step's second barrier
        if (it >= 1 && it <= ntiles) {  // ---- tile `it - 1`
          const bf16_t* Qs = reinterpret_cast<const bf16_t*>(smem + PipeLds::Q0 + buf * PipeLds::QB);
          const bf16_t* dOs = reinterpret_cast<const bf16_t*>(smem + PipeLds::DO0 + buf * PipeLds::QB);
          const bf16_t* Pt = reinterpret_cast<const bf16_t*>(smem + PipeLds::Pt0 + buf * PipeLds::PB);
          const bf16_t* dSt = reinterpret_cast<const bf16_t*>(smem + PipeLds::DSt0 + buf * PipeLds::PB);
          // Three products of 16 MFMAs each, in this order:
          //   ops  0..15  dV_i += P^T dO          (op = 4 qs + cb: rows 16 qs.., channels 32 cb..)
          //   ops 16..31  dQ^T  = K_i^T dS^T      (op = 16 + 2 sp + rb: keys 16 sp.., rows 32 rb..)
          //   ops 32..47  dK_i += dS^T Q          (as the first, with Q)
          // Every op's "lane = column" operand is a pair of transposing LDS reads.  As in the S-waves the issue order
          // is fixed by hand: the operands run through a ring of kRing registers, op i issues its MFMA and refills its
          // slot with the operand of op i + kRing, across the product boundaries, so only the first kRing reads of a
          // tile are waited for at full LDS latency.  The dQ slices are stored between the second and third product.
          constexpr int kRing = 4;
          const bf16_t* parow = Pt + (32 * sw + col) * kPStride + 8 * qh;   // rows 32 sw.. of P^T: read by this wave only
          const bf16_t* sarow = dSt + (32 * sw + col) * kPStride + 8 * qh;
          const bf16_t* do_tr = dOs + tr_lane;
          const bf16_t* q_tr = Qs + tr_lane;
          const bf16_t* ds_tr = dSt + tr_lane_p;
          auto operand = [&](auto opc) __attribute__((always_inline)) {
            constexpr int op = decltype(opc)::value;
            const bf16_t* p0;
            constexpr int step = (op >= 16 && op < 32) ? 4 * kPStride : 4 * kRowStride;
            if constexpr (op < 16)
              p0 = do_tr + (16 * (op >> 2) * kRowStride + 32 * (op & 3));
            else if constexpr (op < 32)
              p0 = ds_tr + (16 * ((op - 16) >> 1) * kPStride + 32 * (op & 1));
            else
              p0 = q_tr + (16 * ((op - 32) >> 2) * kRowStride + 32 * (op & 3));
            const bf16x4 lo4 = lds_read_tr(p0);
            const bf16x4 hi4 = lds_read_tr(p0 + step);
            return __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
          };
          bf16x8 ring[kRing], af[4];  // af: the "lane = row of the result" operand of the first / third product
          f32x16 dqacc[2];
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) dqacc[rb][v] = 0.f;
#pragma unroll
          for (int qs = 0; qs < 4; ++qs) af[qs] = *reinterpret_cast<const bf16x8*>(parow + 16 * qs);
          static_for<0, kRing>([&](auto opc) { ring[decltype(opc)::value] = operand(opc); });
          __builtin_amdgcn_sched_barrier(0);
          static_for<0, 48>([&](auto opc) __attribute__((always_inline)) {
            constexpr int op = decltype(opc)::value;
            if constexpr (op < 16)
              dvacc[op & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[op >> 2], ring[op % kRing], dvacc[op & 3], 0, 0, 0);
            else if constexpr (op < 32)
              dqacc[op & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[(op - 16) >> 1], ring[op % kRing],
                                                                      dqacc[op & 1], 0, 0, 0);
            else
              dkacc[op & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[(op - 32) >> 2], ring[op % kRing],
                                                                      dkacc[op & 3], 0, 0, 0);
            if constexpr (op + kRing < 48) ring[op % kRing] = operand(std::integral_constant<int, op + kRing>{});
            if constexpr (op >= 24 && op < 28)  // the first product is done with af: refill it for the third
              af[op - 24] = *reinterpret_cast<const bf16x8*>(sarow + 16 * (op - 24));
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (op == 31) {
              // this wave's 64-byte slice of the tile's dQ rows: accumulator layout (lane = row) -> rows 32 sw.. of
              // the P^T tile, which this wave has finished reading and the S-waves rewrite only after the next
              // barrier -> 16-byte row pieces
              bf16_t* stg = reinterpret_cast<bf16_t*>(smem + PipeLds::Pt0 + buf * PipeLds::PB) + 32 * sw * kPStride;
#pragma unroll
              for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                  uint2 w;
                  w.x = pack_bf16x2(dqacc[rb][4 * a + 0], dqacc[rb][4 * a + 1]);
                  w.y = pack_bf16x2(dqacc[rb][4 * a + 2], dqacc[rb][4 * a + 3]);
                  *reinterpret_cast<uint2*>(&stg[(32 * rb + col) * kDqPitch + 8 * a + 4 * qh]) = w;
                }
              wave_sync_bwd();
              const int tile0 = row_first + (it - 1) * kTile;
              const size_t prow0 = (size_t)(U.e0 - U.pos0) * P.g + (size_t)tile0;
              int ln = lane;
              asm volatile("" : "+v"(ln));  // keeps the row addresses from being precomputed and held (register budget)
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const int row = 16 * i + (ln >> 2), piece = (ln & 3) * 8;
                if (tile0 + row < rows_end) {
                  const uint2 lo2 = *reinterpret_cast<const uint2*>(&stg[row * kDqPitch + piece]);
                  const uint2 hi2 = *reinterpret_cast<const uint2*>(&stg[row * kDqPitch + piece + 4]);
                  store_streaming(dqpart + (prow0 + row) * kD + 32 * sw + piece,
                                  make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
                }
              }
              __builtin_amdgcn_sched_barrier(0);
            }
          });
        }
        PT_STAMP(1)
        __syncthreads();  // every wave is done with the tiles of `it - 1`
        PT_STAMP(2)
      }
    };
    // both roles take the same number of steps: the barriers inside `step` pair up across the roles
    // (an even number of steps; a last step past the end computes nothing)
    for (int it = 0; it <= ntiles; it += 2) {
      step(it, Set0{});
      step(it + 1, Set1{});
    }
  }

#ifdef NSA_PIPE_TIMING
  if (lane == 0)
    for (int k = 0; k < 8; ++k)
      if (k != 4) atomicAdd(&g_pipe_t[kS ? 0 : 1][k], pt[k]);
  if (lane == 0) atomicAdd(&g_pipe_t[kS ? 0 : 1][4], 1ull);
#endif
  if constexpr (!kS) {
    if (nu_scan[U.L + 1] - nu_scan[U.L] == 1) {
      // the whole list fitted this unit: dK_i, dV_i are final, write them as bf16 (keys of a ragged tail excluded)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        bf16_t* outk = dK + ((size_t)tok0 * P.hkv + j) * kD + 32 * cb + col;
        bf16_t* outv = dV + ((size_t)tok0 * P.hkv + j) * kD + 32 * cb + col;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 32 * sw + 8 * (v >> 2) + 4 * qh + (v & 3);
          if (key < blen) {
            outk[(size_t)key * P.hkv * kD] = (bf16_t)dkacc[cb][v];
            outv[(size_t)key * P.hkv * kD] = (bf16_t)dvacc[cb][v];
          }
        }
      }
      return;
    }
    // unit partial: [u][0 = dK, 1 = dV][key][d] fp32, summed by k_bwd_dkv_reduce in unit order
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      float* outk = dkv_part + (size_t)(U.u - U.ubase) * 2 * 128 * kD + 32 * cb + col;
      float* outv = outk + 128 * kD;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * sw + 8 * (v >> 2) + 4 * qh + (v & 3);
        outk[key * kD] = dkacc[cb][v];
        outv[key * kD] = dvacc[cb][v];
      }
    }
  }
}

template <bool kWin>
__global__ void __launch_bounds__(512, 1)
k_bwd_pipe128(Problem P, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
              const bf16_t* __restrict__ dO, const float2* __restrict__ stats, const int32_t* __restrict__ u_list,
              const int32_t* __restrict__ u_start, const int32_t* __restrict__ off,
              const int32_t* __restrict__ blk_tok0, const int32_t* __restrict__ blk_len,
              const int2* __restrict__ qent, const int32_t* __restrict__ nu_scan, bf16_t* __restrict__ dqpart,
              float* __restrict__ dkv_part, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  PipeUnit U;
  U.ubase = nu_scan[P.j0 * P.b_cap];
  U.u = U.ubase + blockIdx.x;
  if (U.u >= nu_scan[(P.j0 + P.nj) * P.b_cap]) return;
  U.L = u_list[U.u];
  U.j = U.L / P.b_cap;
  const int gb = U.L - U.j * P.b_cap;
  U.e0 = u_start[U.u];
  U.pos0 = off[P.j0 * P.b_cap];
  U.ne = min(P.unit, off[U.L + 1] - U.e0);
  U.tok0 = blk_tok0[gb];
  U.blen = blk_len[gb];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave < 4)
    pipe_role<kWin, true>(P, U, smem, wave, Q, K, V, dO, stats, qent, nu_scan, dqpart, dkv_part, dK, dV);
  else
    pipe_role<kWin, false>(P, U, smem, wave - 4, Q, K, V, dO, stats, qent, nu_scan, dqpart, dkv_part, dK, dV);
}

__global__ void __launch_bounds__(256)
k_bwd_dq_reduce(Problem P, const bf16_t* __restrict__ dqpart, const uint32_t* __restrict__ vmask,
                const int32_t* __restrict__ slotpos, const int32_t* __restrict__ off, bf16_t* __restrict__ dQ) {
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
  const int32_t* sp = slotpos + ((size_t)t * P.hkv + j) * P.topk;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int m0 = 0; m0 < P.topk; m0 += kSlotBatch) {  // kSlotBatch independent 256-byte gathers in flight per row
    uint4 x[kSlotBatch];
#pragma unroll
    for (int i = 0; i < kSlotBatch; ++i) {
      const int m = m0 + i;
      const bool on = m < P.topk && ((vm >> m) & 1u);
      x[i] = on ? *reinterpret_cast<const uint4*>(dqpart + ((size_t)(sp[on ? m : 0] - pos0) * P.g + hh) * kD + 8 * sub)
                : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kSlotBatch; ++i) {
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

// grid (n_lists, 2, B_K / 8): y = 0 -> dK, 1 -> dV; z = group of 8 keys, so that the units of a long list (the sink
// block's list has 32 of them) are walked by B_K / 8 workgroups side by side.  Thread = 4 consecutive channels of
// one key; the sum runs in unit order.
__global__ void __launch_bounds__(256)
k_bwd_dkv_reduce(Problem P, const int32_t* __restrict__ nu_scan, const int32_t* __restrict__ blk_tok0,
                 const int32_t* __restrict__ blk_len, const float* __restrict__ dkv_part, bf16_t* __restrict__ dK,
                 bf16_t* __restrict__ dV) {
  const int L = P.j0 * P.b_cap + blockIdx.x, which = blockIdx.y;  // lists of the pass's KV heads
  const int ubase = nu_scan[P.j0 * P.b_cap];
  const int j = L / P.b_cap, gb = L - j * P.b_cap;
  const int blen = blk_len[gb];
  if (blen == 0) return;
  const int tok0 = blk_tok0[gb];
  const int u0 = nu_scan[L], u1 = nu_scan[L + 1];
  if (u1 - u0 == 1) return;  // a single unit wrote the final values itself
  bf16_t* out = which ? dV : dK;
  const int d4 = (threadIdx.x & 31) * 4;
  const int key = 8 * blockIdx.z + (threadIdx.x >> 5);
  if (key < blen) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int u = u0; u < u1; ++u) {
      const float4 x =
          *reinterpret_cast<const float4*>(dkv_part + ((size_t)(u - ubase) * 2 + which) * P.bk * kD + key * kD + d4);
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    uint2 w;
    w.x = pack_bf16x2(acc.x, acc.y);
    w.y = pack_bf16x2(acc.z, acc.w);
    *reinterpret_cast<uint2*>(out + ((size_t)(tok0 + key) * P.hkv + j) * kD + d4) = w;
  }
}

#ifdef NSA_PIPE_TIMING
// Measuring build only: copies the 2 x 8 counters (role x {phase 0..3 clocks, waves counted, unused}) to the host `out`
// (synchronous, on the current device) and, with `reset`, zeroes them.  Returns 0, or -1 if a HIP call failed.
extern "C" int nsa_sel_pipe_timing_read(unsigned long long* out, int reset) {
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(g_pipe_t), sizeof(unsigned long long) * 16) != hipSuccess) return -1;
  if (reset) {
    unsigned long long z[16] = {};
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_pipe_t), z, sizeof(z)) != hipSuccess) return -1;
  }
  return 0;
}
#endif
hipError_t launch_bwd(const Problem& P0, const IndexLayout& L, int heads_per_pass, const void* Q, const void* K,
                      const void* V, const void* O, const float* LSE, const void* dO, const void* index_ws,
                      void* dqpart, float* delta, float* dkv_part, void* dQ, void* dK, void* dV, const GateArgs& G,
                      hipStream_t st) {
  IndexPtrs p = index_ptrs(L, const_cast<void*>(index_ws));
  // 64-token blocks: four waves, two workgroups per CU; 128-token blocks: eight waves, one workgroup per CU
  const bool b128 = P0.bk == 128;
  const bool win = P0.window > 0;
  auto* main_kernel = b128 ? (win ? k_bwd_pipe128<true> : k_bwd_pipe128<false>)
                           : (win ? k_bwd_tiled<2, true> : k_bwd_tiled<2, false>);
  const int main_threads = b128 ? 512 : 256;
  const int main_lds = b128 ? PipeLds::Bytes : BwdLds<2>::Bytes;
  {
    static std::atomic<uint64_t> ready[4];
    hipError_t e = allow_dynamic_lds((const void*)main_kernel, main_lds, ready[2 * win + b128]);
    if (e != hipSuccess) return e;
  }
  {
    const int64_t rows = (int64_t)P0.T * P0.hq;
    ProfScope ps(KID_BWD_DELTA, st);
    hipLaunchKernelGGL(k_bwd_delta, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, rows, (const bf16_t*)O,
                       (const bf16_t*)dO, LSE, (float2*)delta, G.gate, G.dgate);
  }
  // KV heads are processed heads_per_pass at a time, every pass reusing the partial-dQ and unit-partial buffers
  for (int j0 = 0; j0 < P0.hkv; j0 += heads_per_pass) {
    Problem P = P0;
    P.j0 = j0;
    P.nj = min(heads_per_pass, P0.hkv - j0);
    const unsigned units_max = (unsigned)units_bound(P.nj, P.b_cap, P.T, P.topk, P.unit);
    const int64_t rows = (int64_t)P.T * P.nj * P.g;
    { ProfScope ps(KID_BWD_MAIN, st);
    hipLaunchKernelGGL(main_kernel, dim3(units_max), dim3(main_threads), main_lds, st, P, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, (const float2*)delta, p.u_list,
                       p.u_start, p.off, p.blk_tok0, p.blk_len, p.qent, p.u_nu, (bf16_t*)dqpart, dkv_part,
                       (bf16_t*)dK, (bf16_t*)dV); }
    { ProfScope ps(KID_BWD_DQ_REDUCE, st);
    hipLaunchKernelGGL(k_bwd_dq_reduce, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, P,
                       (const bf16_t*)dqpart, p.vmask, p.slotpos, p.off, (bf16_t*)dQ); }
    ProfScope ps(KID_BWD_DKV_REDUCE, st);
    hipLaunchKernelGGL(k_bwd_dkv_reduce, dim3(P.nj * P.b_cap, 2, P.bk / 8), dim3(256), 0, st, P, p.u_nu, p.blk_tok0, p.blk_len,
                       (const float*)dkv_part, (bf16_t*)dK, (bf16_t*)dV);
  }
  return hipGetLastError();
}

}  // namespace nsa
