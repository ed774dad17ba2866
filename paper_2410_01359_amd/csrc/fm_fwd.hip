// Forward tile loop (Algorithm 1) for gfx950.
//
// One workgroup (4 waves) per (batch, head, block of 128 query rows).  Each wave
// owns 32 query rows for the whole kernel and walks the key blocks that the
// min/max tables do not prove fully masked.  Scores are computed transposed,
// S^T = K Q^T, so that after the MFMA every lane holds ONE query column: row
// max / row sum are per-lane loops plus one exchange with the lane 32 away, the
// running rescale of O is a per-lane scalar, and P^T is already in the
// B-operand layout of the second product O^T += V^T P^T.  K tiles are read
// from LDS as A operands (128-bit reads), V tiles through the LDS transpose
// read.  Q stays in registers.
//
// The loop is software-pipelined over key tiles: while the exp / row-sum
// arithmetic of tile t runs on the vector unit, the matrix unit already computes
// the scores of tile t+1 into a second accumulator set, so a wave keeps both
// units busy by itself instead of relying on the other resident wave being in
// the complementary phase.  K and V therefore travel in separate two-deep LDS
// rings: iteration t reads K(t+1) and V(t) while K(t+2) and V(t+1) are in flight.
#include "fm_common.h"
#include "fm_kernels.h"

namespace fm {

#ifndef FM_FWD_EXP_A
#define FM_FWD_EXP_A 20
#endif

template <int D>
struct FwdCfg {
  static constexpr int KT = FM_FWD_BC;          // keys per tile
  static constexpr int BR = FM_FWD_BR;          // query rows per workgroup
  using L = TileLayout<D>;
  static constexpr int K_BYTES = KT * L::RS;
  static constexpr int V_BYTES = KT * L::RS;
  static constexpr int BND_BYTES = 4 * KT * 4;  // LTS, LTE, UTS, UTE slices of one tile, kept behind its V tile
  static constexpr int VSTAGE = V_BYTES + BND_BYTES;
  static constexpr int LIST_CAP = 1024;         // key blocks classified per pass
  static constexpr int LIST_OFF = 0;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int K_OFF = CNT_OFF + 64;
  static constexpr int V_OFF = K_OFF + 2 * K_BYTES;
  static constexpr int LDS_BYTES = V_OFF + 2 * VSTAGE;
};

// Per-wave constants of the tile loop.
template <int D>
struct FwdWave {
  int a_off;               // operand rows: row c, bytes 16 g (slice kk adds 32 kk through TileLayout::add_col)
  int t_off[2];            // transpose reads: row 4 g + i16/4 (+8), bytes 32 half + 8 (i16 & 3) (d block db adds 64 db)
  int row;                 // this lane's query row
  int g;
  float sc;                // scale * log2(e)
};

// One pipeline step: exp / row-sum arithmetic and O^T += V^T P^T of the tile whose raw scores
// are in `cur` (masked first if `masked` != 0), and the raw scores of the NEXT tile (K tile at
// k_next) into `nxt`.
template <int D>
__device__ __forceinline__ void fwd_step(f32x16 (&cur)[2], f32x16 (&nxt)[2], f32x16 (&oacc)[D / 32],
                                         const bf16x8 (&qreg)[D / 16], float& m_run, float& l_run,
                                         const char* k_next, const char* vs, const int* bnd, int masked,
                                         const FwdWave<D>& w) {
  using C = FwdCfg<D>;
  constexpr int KT = C::KT, NKB = KT / 32, NDB = D / 32, NKK = D / 16;
  static_assert(NKB == 2, "two 32-key blocks per tile");
  constexpr float kRescaleGap = 8.f;
  // per-lane LDS offsets, made opaque once per tile so that what is derived from them is
  // recomputed (one vector op each) instead of being hoisted out of the tile loop into registers
  const int a_b = opaque(w.a_off), t_b0 = opaque(w.t_off[0]), t_b1 = opaque(w.t_off[1]);

  if (masked) {
    const int* bnd_g = (const int*)((const char*)bnd + opaque(16 * w.g));
    // A sub-tile that Equation 4 proves fully masked for this wave takes the same path and ends
    // with every score at -inf.  `masked` says which pairs the workgroup's tile needs (1 = LT,
    // 2 = UT, 3 = both; 5, 6 = one pair that a single comparison decides, see entry_mask_mode):
    // a pair that is not needed masks no element of the tile, so leaving it
    // out is exact -- and most partially masked tiles (a causal diagonal, a window edge, a
    // document boundary) need only one.
    if (masked == 3) {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int kx = kb * 32 + 8 * rq;
          const i32x4 bl = *(const i32x4*)(bnd_g + 0 * KT + kx);
          const i32x4 be = *(const i32x4*)(bnd_g + 1 * KT + kx);
          const i32x4 bu = *(const i32x4*)(bnd_g + 2 * KT + kx);
          const i32x4 bv = *(const i32x4*)(bnd_g + 3 * KT + kx);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool hit = ((w.row >= bl[e]) & (w.row < be[e])) | ((w.row >= bu[e]) & (w.row < bv[e]));
            if (hit) cur[kb][rq * 4 + e] = -INFINITY;
          }
          __builtin_amdgcn_sched_barrier(0);  // keep the bound reads of later steps from piling up in registers
        }
    } else if (masked & 4) {
      // one pair, decided by one comparison per element (5: row >= LTS, 6: row < UTE): one bound per key
      const int* b_one = bnd_g + (masked == 5 ? 0 : 3 * KT);
      if (masked == 5) {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const i32x4 bs = *(const i32x4*)(b_one + kb * 32 + 8 * rq);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (w.row >= bs[e]) cur[kb][rq * 4 + e] = -INFINITY;
            __builtin_amdgcn_sched_barrier(0);
          }
      } else {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const i32x4 be = *(const i32x4*)(b_one + kb * 32 + 8 * rq);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (w.row < be[e]) cur[kb][rq * 4 + e] = -INFINITY;
            __builtin_amdgcn_sched_barrier(0);
          }
      }
    } else {
      const int* b_lo = bnd_g + (masked == 2 ? 2 * KT : 0);   // starts of the one pair that is needed
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int kx = kb * 32 + 8 * rq;
          const i32x4 bs = *(const i32x4*)(b_lo + kx);
          const i32x4 be = *(const i32x4*)(b_lo + KT + kx);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool hit = (w.row >= bs[e]) & (w.row < be[e]);
            if (hit) cur[kb][rq * 4 + e] = -INFINITY;
          }
          __builtin_amdgcn_sched_barrier(0);
        }
    }
  }

  // ---- stream A: S^T(next) = K Q^T on the matrix unit, softmax(cur) on the vector unit.
  // MFMA step n: chain kb = n % 2, slice kk = n / 2 (the two accumulation chains alternate);
  // its K operand is fetched RS steps ahead into a small register ring.
  constexpr int NS = NKB * NKK, RS = 4;
  constexpr int NMAX = 4;                          // steps that carry the running max (8 elements each)
  constexpr int NEXP = NS - NMAX - 1;              // steps that carry exponentials
  // The exponentials of the first EXP_A elements (of 32 per lane) ride along with these score
  // MFMAs, the rest with the first half of the second product below (which only needs the first
  // 16): one product's shadow alone is too short for all of them.
  constexpr int EXP_A = FM_FWD_EXP_A;
  constexpr int EPS = (EXP_A + NEXP - 1) / NEXP;   // elements per such step
  bf16x8 kring[RS];
  auto k_operand = [&](int n) __attribute__((always_inline)) {
    return *(const bf16x8*)(k_next + (n % NKB) * 32 * C::L::RS + C::L::add_col(a_b, (n / NKB) * 32));
  };
  const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int n = 0; n < RS; ++n) kring[n] = k_operand(n);
  __builtin_amdgcn_sched_barrier(0);
  float mx = -INFINITY, neg_m = 0.f, rs = 0.f;
#pragma unroll
  for (int n = 0; n < NS; ++n) {
    nxt[n % NKB] = mfma32(kring[n % RS], qreg[n / NKB], n < NKB ? zero : nxt[n % NKB]);
    if (n + RS < NS) kring[n % RS] = k_operand(n + RS);
    if (n < NMAX) {
#pragma unroll
      for (int e = 8 * n; e < 8 * n + 8; ++e) mx = fmaxf(mx, cur[e / 16][e % 16]);
    } else if (n == NMAX) {
      mx = fmaxf(mx, partner32(mx)) * w.sc;
      const bool grow = mx > m_run + kRescaleGap;   // also true on the first finite maximum
      if (__any(grow)) {
        // The reference maximum only moves when a tile's maximum exceeds it by more than the
        // gap (log2 units), so this rescale of O and l is rare; any reference is a valid one,
        // P just grows up to 2^gap.
        const float m_new = grow ? mx : m_run;
        const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
      }
      neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
    } else {
      const int j = n - NMAX - 1;
#pragma unroll
      for (int e = j * EPS; e < (j + 1) * EPS && e < EXP_A; ++e) {
        const float p = fast_exp2(__builtin_fmaf(cur[e / 16][e % 16], w.sc, neg_m));
        cur[e / 16][e % 16] = p;
        rs += p;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }

  // ---- stream B: O^T += V^T P^T, step n = (16-key group n / NDB, d block n % NDB)
  constexpr int NP = NKB * 2 * NDB, RP = 4;
  bf16x8 vring[RP];
  auto v_operand = [&](int n) __attribute__((always_inline)) {
    const char* vrow = vs + ((n / NDB) * 16) * C::L::RS;   // group n / NDB = (kb, h): 16 keys each
    return cat4(lds_read_tr16(vrow + C::L::add_col(t_b0, (n % NDB) * 64)),
                lds_read_tr16(vrow + C::L::add_col(t_b1, (n % NDB) * 64)));
  };
#pragma unroll
  for (int n = 0; n < RP; ++n) vring[n] = v_operand(n);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int n = 0; n < NP; ++n) {
    const int grp = n / NDB, kb = grp / 2, h = grp % 2, db = n % NDB;
    bf16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) pb[e] = (__bf16)cur[kb][8 * h + e];
    oacc[db] = mfma32(vring[n % RP], pb, oacc[db]);
    if (n + RP < NP) vring[n % RP] = v_operand(n + RP);
    if (n < NP / 2) {   // the remaining exponentials (second 32-key block), beside the first block's MFMAs
      constexpr int EPB = (32 - EXP_A + NP / 2 - 1) / (NP / 2);
#pragma unroll
      for (int e = EXP_A + n * EPB; e < EXP_A + (n + 1) * EPB && e < 32; ++e) {
        const float p = fast_exp2(__builtin_fmaf(cur[e / 16][e % 16], w.sc, neg_m));
        cur[e / 16][e % 16] = p;
        rs += p;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  l_run += rs;
}

// RAGGED: the sequence length is not a multiple of 128.  The loops then run at the padded length
// Np (tables, lists and the padded bound vectors are built for it; the padding columns are masked
// for every row), tile copies that reach past row N clamp their source rows, and rows >= N are
// computed but not stored.
// GEN: tensors with caller-given strides and fewer K/V heads than query heads (see FmFwdArgs).
template <int D, bool RAGGED, bool GEN>
__global__ __launch_bounds__(256, D == 64 ? 3 : 2) void fwd_kernel(FmFwdArgs a) {
  using C = FwdCfg<D>;
  constexpr int KT = C::KT, NKB = KT / 32, NDB = D / 32, NKK = D / 16;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const i32x4 rec = queue_take(a.order, a.slots, (int*)(smem + C::CNT_OFF) + 8);
  const int unit = rec[0], j_lo = rec[1], j_hi = rec[2];
  if (unit < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int N = a.Np, H = a.H;            // padded length: what the loops and tables see
  const int Nr = RAGGED ? a.N : a.Np;     // rows the tensors really have
  const int t_r = N / C::BR, t_c = N / KT;
  const int bh = unit / t_r, i_blk = unit - bh * t_r, b = bh / H;
  const int q0 = i_blk * C::BR;
  const int qw0 = q0 + wave * 32;

  const int h = bh - b * H, hk = GEN ? h / (H / a.Hk) : h, Hk = GEN ? a.Hk : H;
  const __bf16* qp = slice_ptr<D, GEN>(a.q, a.sq, b, h, H, Nr);
  const __bf16* kp = slice_ptr<D, GEN>(a.k, a.sk, b, hk, Hk, Nr);
  const __bf16* vp = slice_ptr<D, GEN>(a.v, a.sv, b, hk, Hk, Nr);
  const int q_rs = row_stride<D, GEN>(a.sq), k_rs = row_stride<D, GEN>(a.sk), v_rs = row_stride<D, GEN>(a.sv);
  const int* table = a.minmax + (size_t)b * 8 * t_c;
  // lanes of wave 0 copy the four bound slices of a partially masked tile: lane l moves
  // 16 bytes of vector l / 16
  const int* my_bvec;
  {
    const int which = lane >> 4;
    const int* p = a.lts;
    if (which == 1) p = a.lte;
    if (which == 2) p = a.uts;
    if (which == 3) p = a.ute;
    my_bvec = p + (size_t)b * N + (lane & 15) * 4;
  }
  CopyLanes<D> copy_lanes, copy_lanes_v_;
  copy_lanes.init(lane, 2 * k_rs);
  if (GEN) copy_lanes_v_.init(lane, 2 * v_rs);
  const CopyLanes<D>& copy_lanes_v = GEN ? copy_lanes_v_ : copy_lanes;

  // Q fragments (B operand of S^T = K Q^T): lane holds Q[row c][16 kk + 8 g ..+7].
  bf16x8 qreg[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk)
    qreg[kk] = *(const bf16x8*)(qp + (size_t)(RAGGED ? min(qw0 + c, Nr - 1) : qw0 + c) * q_rs + kk * 16 + 8 * g);
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) settle(qreg[kk]);

  f32x16 oacc[NDB];
  float m_run = -INFINITY, l_run = 0.f;   // log2 domain
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;

  int* list = (int*)(smem + C::LIST_OFF);
  int* wave_cnt = (int*)(smem + C::CNT_OFF);
  FwdWave<D> w;
  w.sc = a.scale * kLog2e;  // > 0 (checked on the host): scores stay raw, exp2(s*sc - m) is one fma + one exp
  w.row = qw0 + c;
  w.g = g;
  {
    const int i16 = lane & 15, half = (lane >> 4) & 1;
    w.a_off = C::L::off(c, 16 * g);
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) w.t_off[hi] = C::L::off(4 * g + (i16 >> 2) + 8 * hi, (16 * half + 4 * (i16 & 3)) * 2);
  }

  // Asynchronous copies of list entry ENTRY: its K tile into K stage KBUF / its V tile (and, if the
  // workgroup's tile is partially masked, its bound slices) into V stage VBUF.
#define FM_LOAD_K(ENTRY, KBUF)                                                                   \
  {                                                                                              \
    const int j_ = entry_block(ENTRY, chunk);                                                    \
    char* st_ = smem + C::K_OFF + (KBUF) * C::K_BYTES;                                           \
    if (RAGGED && (j_ + 1) * KT > Nr)                                                            \
      tile_load_async_clamped<D>(kp, j_ * KT, Nr, st_, wave, lane, 2 * k_rs);                    \
    else                                                                                         \
      tile_load_async<D>(kp + (size_t)j_ * KT * k_rs, copy_lanes, st_, wave, 2 * k_rs);          \
  }
#define FM_LOAD_V(ENTRY, VBUF)                                                                   \
  {                                                                                              \
    const int j_ = entry_block(ENTRY, chunk);                                                    \
    char* st_ = smem + C::V_OFF + (VBUF) * C::VSTAGE;                                            \
    if (RAGGED && (j_ + 1) * KT > Nr)                                                            \
      tile_load_async_clamped<D>(vp, j_ * KT, Nr, st_, wave, lane, 2 * v_rs);                    \
    else                                                                                         \
      tile_load_async<D>(vp + (size_t)j_ * KT * v_rs, copy_lanes_v, st_, wave, 2 * v_rs);        \
    if (entry_tile_class(ENTRY) == T_PARTIAL && wave == 0)                                       \
      async_copy16(my_bvec + j_ * KT, lds_address(st_ + C::V_BYTES));                            \
  }
  // One iteration: tile T with scores in CUR, scores of tile T + 1 into NXT.  Entries past the
  // end of the list are clamped to the last one: nothing is copied for them, and the scores the last
  // step computes from the stale K stage are never used.
#define FM_STEP(T, CUR, NXT)                                                                     \
  {                                                                                              \
    /* the list entry that joins the window at the next step: read now, picked up behind the  */ \
    /* step's barrier, so that no step starts by waiting for LDS                               */ \
    const int v_3 = list[min((T) + 3, n_live - 1)];                                              \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    if ((T) + 2 < n_live) FM_LOAD_K(e_2, (T) & 1);                                               \
    if ((T) + 1 < n_live) FM_LOAD_V(e_1, ((T) + 1) & 1);                                         \
    const char* vs_ = smem + C::V_OFF + ((T) & 1) * C::VSTAGE;                                   \
    fwd_step<D>(CUR, NXT, oacc, qreg, m_run, l_run, smem + C::K_OFF + (((T) + 1) & 1) * C::K_BYTES, vs_, \
                (const int*)(vs_ + C::V_BYTES),                                                  \
                entry_wave_class(e_t, wave) != T_UNMASKED ? entry_mask_mode(e_t) : 0, w);        \
    async_wait<0>();   /* K(T+2) and V(T+1) have landed ... */                                   \
    barrier_nofence(); /* ... for every wave, and every wave is done with K(T+1) and V(T) */     \
    e_t = e_1;                                                                                   \
    e_1 = e_2;                                                                                   \
    e_2 = __builtin_amdgcn_readfirstlane(v_3);                                                   \
  }

  // only the key blocks [j_lo, j_hi) can be live for this row block (found by the work pre-pass)
  for (int chunk = j_lo; chunk < j_hi; chunk += C::LIST_CAP) {
    const int n_live = build_live_key_blocks(table, t_c, chunk, min(chunk + C::LIST_CAP, j_hi), q0, min(q0 + C::BR, N),
                                             C::BR / 4, list, wave_cnt);
    if (n_live == 0) continue;
    // the entries of tiles T, T + 1, T + 2 of the step about to run (clamped to the last one)
    int e_t = __builtin_amdgcn_readfirstlane(list[0]);
    int e_1 = __builtin_amdgcn_readfirstlane(list[min(1, n_live - 1)]);
    int e_2 = __builtin_amdgcn_readfirstlane(list[min(2, n_live - 1)]);
    {
      FM_LOAD_K(e_t, 0);
      FM_LOAD_V(e_t, 0);
      FM_LOAD_K(e_1, 1);
      async_wait<0>();
      barrier_nofence();
    }
    // scores of the first tile
    f32x16 s0[NKB], s1[NKB];
    {
      const char* ks = smem + C::K_OFF;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s0[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
          s0[kb] = mfma32(*(const bf16x8*)(ks + kb * 32 * C::L::RS + C::L::add_col(w.a_off, kk * 32)), qreg[kk], s0[kb]);
      barrier_nofence();   // the first iteration refills this K stage: every wave must have read it
    }
    for (int t = 0; t < n_live; t += 2) {
      FM_STEP(t, s0, s1)
      if (t + 1 < n_live) FM_STEP(t + 1, s1, s0)
    }
    __syncthreads();     // the list is rebuilt by the next pass
  }
#undef FM_STEP
#undef FM_LOAD_K
#undef FM_LOAD_V

  // epilogue: O / l, lse = m + log(l)   (m, l in the log2 domain)
  __bf16* op = (__bf16*)slice_ptr<D, GEN>(a.out, a.so, b, h, H, Nr);
  const int o_rs = row_stride<D, GEN>(a.so);
  float* lp = a.lse + (size_t)bh * Nr;
  {
    const float lt = l_run + partner32(l_run);
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const int row = qw0 + c;
    // every wave is past its last tile and nothing is in flight into the K / V stages (the barrier that
    // ends a pass over the list): their first bytes serve as the waves' store staging
    using RSt = RowStage<D>;
    static_assert(4 * RSt::BYTES <= C::LDS_BYTES - C::K_OFF, "store staging fits the K / V stages");
    char* stage = smem + C::K_OFF + wave * RSt::BYTES;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][rq * 4 + e] * inv);
        RSt::put(stage, c, g, db, rq, o4);
      }
    RSt::flush(stage, op + (size_t)qw0 * o_rs, o_rs, lane, RAGGED ? min(32, Nr - qw0) : 32);
    if ((!RAGGED || row < Nr) && g == 0) lp[row] = lt > 0.f ? (m_run + fast_log2(lt)) * kLn2 : -INFINITY;
  }
}

}  // namespace fm

using namespace fm;

template <int D, bool RAGGED, bool GEN>
static hipError_t launch_fwd_t(const FmFwdArgs& a, hipStream_t stream) {
  using C = FwdCfg<D>;
  static bool allowed[FM_MAX_DEVICES] = {};
  if (hipError_t e = fm_allow_lds((const void*)fwd_kernel<D, RAGGED, GEN>, C::LDS_BYTES, allowed); e != hipSuccess) return e;
  hipLaunchKernelGGL((fwd_kernel<D, RAGGED, GEN>), dim3(fm_launch_grid(a.slots)), dim3(256), C::LDS_BYTES, stream, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_fwd_d(const FmFwdArgs& a, hipStream_t stream) {
  const bool ragged = a.Np != a.N;
  if (a.general) return ragged ? launch_fwd_t<D, true, true>(a, stream) : launch_fwd_t<D, false, true>(a, stream);
  return ragged ? launch_fwd_t<D, true, false>(a, stream) : launch_fwd_t<D, false, false>(a, stream);
}

hipError_t fm_launch_fwd(const FmFwdArgs& a, hipStream_t stream) {
  static_assert(FM_FWD_BR == 128, "forward row block");
  return a.d == 128 ? launch_fwd_d<128>(a, stream) : launch_fwd_d<64>(a, stream);
}
