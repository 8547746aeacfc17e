// Backward selected-block attention for gfx950.  The paper (Sec. 3.2) only says that the backward pass follows
// the forward's KV-outer logic, gathers the queries again through the cached index tensors and stores
// intermediate query gradients to a buffer that a reduction kernel sums; dK/dV accumulation is not described.
// This file is that pass, with dK/dV accumulated without atomics:
//
//   k_bwd_delta       delta[t,h] = <dO[t,h], O[t,h]>, stored next to LSE[t,h] log2(e) as one 8-byte pair so that the
//                     main kernel fetches both row statistics with one gather
//   k_bwd_tiled<NKB>  one work unit = (kv head j, KV block i, up to P.unit list entries); NKB = B_K / 32.  With
//                     B_K = 64: four wavefronts and half of a CU's LDS, so two workgroups share a CU and cover each
//                     other's barriers and waits; with B_K = 128: eight wavefronts, one workgroup per CU.  The waves
//                     share tiles of 64 gathered rows and take three roles per tile (see the comment above the
//                     kernel): S^T = K_i Q^T, dP^T = V_i dO^T, P = exp(S - LSE), dS = P (dP - delta) scale; then
//                     dV_i += P^T dO and dK_i += dS^T Q (accumulators in registers for the whole unit) and
//                     dQ^T = K_i^T dS^T.  Operands are row-major tiles in LDS; "lane = column" operands are LDS
//                     transpose reads.  Partial dQ rows go to the compact buffer at the rows' list position; the
//                     unit's dK_i, dV_i go out as bf16 (list fitted the unit) or to a per-unit fp32 buffer.
//   k_bwd_dq_reduce   dQ[t,h] = sum over kept slots of the partial rows
//   k_bwd_dkv_reduce  dK_i, dV_i = sum over the list's units in unit order (fixed order: bit-reproducible); a list
//                     that fitted one unit was already written by that unit, a list with no entry gets zeros
#include "common.h"

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
// MFMA and VALU time simply added up).  With B_K = 128 (NKB = 4) the fp32 dK/dV accumulators of the block need eight
// waves' registers and there is one workgroup per CU.
// Per tile, wave w takes three roles in turn:
//   rows/keys   (rb = w / NKB, kb = w % NKB): S^T, dP^T, P, dS for rows 32 rb.. and keys 32 kb..; K_i fragments from
//               LDS, V_i fragments of the wave's 32 keys held in registers for the whole unit (only this role uses V_i)
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
  static constexpr int Bytes = Ent + kEntSeg * 4;  // 80896 (NKB = 2), 118784 (NKB = 4)
};
static_assert(2 * BwdLds<2>::Bytes <= 160 * 1024, "two workgroups of the 64-key backward must fit one CU's LDS");
static_assert(BwdLds<4>::Bytes <= 160 * 1024, "the 128-key backward must fit one CU's LDS");

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
      const int lo = kWin ? t - P.window + 1 - tok0 : 0;
      __syncthreads();  // Q / dO tile staged by all waves

      {  // role rows/keys
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
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfa, qf, sacc, 0, 0, 0);
          dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], dof, dpacc, 0, 0, 0);
        }
        bf16_t* pdst = Pt + 32 * rb + col;
        bf16_t* sdst = dSt + 32 * rb + col;
        const float dls = dl * P.scale;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 32 * kb + 8 * (v >> 2) + 4 * qh + (v & 3);
          const float p = (key < lim && (!kWin || key >= lo)) ? __builtin_amdgcn_exp2f(fmaf(sacc[v], c2, -lse2)) : 0.f;
          const float ds = p * fmaf(dpacc[v], P.scale, -dls);  // P (dP - delta) scale
          pdst[key * kPStride] = (bf16_t)p;
          sdst[key * kPStride] = (bf16_t)ds;
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

hipError_t launch_bwd(const Problem& P0, const IndexLayout& L, int heads_per_pass, const void* Q, const void* K,
                      const void* V, const void* O, const float* LSE, const void* dO, const void* index_ws,
                      void* dqpart, float* delta, float* dkv_part, void* dQ, void* dK, void* dV, const GateArgs& G,
                      hipStream_t st) {
  IndexPtrs p = index_ptrs(L, const_cast<void*>(index_ws));
  // 64-token blocks: four waves, two workgroups per CU; 128-token blocks: eight waves, one workgroup per CU
  const bool b128 = P0.bk == 128;
  const bool win = P0.window > 0;
  auto* main_kernel = b128 ? (win ? k_bwd_tiled<4, true> : k_bwd_tiled<4, false>)
                           : (win ? k_bwd_tiled<2, true> : k_bwd_tiled<2, false>);
  const int main_threads = b128 ? 512 : 256;
  const int main_lds = b128 ? BwdLds<4>::Bytes : BwdLds<2>::Bytes;
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
