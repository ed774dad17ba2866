// Backward pass (Algorithm 2) for gfx950, as two kernels:
//
//   dq_kernel     row-parallel loop over query blocks i, run first: its prologue is Algorithm 2's D
//                 pre-pass, D_i = sum_c dO_ic O_ic (left in the workspace for the other loop); then
//                 S, P = exp(S - L), dP, dS per tile and dQ_i += dS K_j, accumulated in registers in a
//                 fixed order.
//   dkdv_kernel   column-parallel loop over key blocks j: recompute S and
//                 P = exp(S - L), dV_j += P^T dO_i, dP = dO_i V_j^T,
//                 dS = P o (dP - D_i), dK_j += dS^T Q_i           (Algorithm 2 main loop)
//
// Algorithm 2 adds every tile's dS K_j into dQ_i in HBM from the column-parallel
// loop.  On this chip fp32 atomic adds sustain about 1.4 TB/s, which would cap
// the backward far below the matrix-core rate, so dQ gets its own row-parallel
// pass instead (two extra products per tile, no atomics, bit-reproducible).
#include "fm_common.h"
#include "fm_kernels.h"

namespace fm {

// ---------------------------------------------------------------------------
// dQ: row-parallel, same transposed-score layout as the forward kernel.
// ---------------------------------------------------------------------------
template <int D>
struct DqCfg {
  static constexpr int KT = fm_dq_bc(D);
  static constexpr int BR = FM_DQ_BR;
  using L = TileLayout<D>;
  static constexpr int K_BYTES = KT * L::RS;
  static constexpr int V_BYTES = KT * L::RS;
  static constexpr int BND_BYTES = 4 * KT * 4;
  static constexpr int STAGE = K_BYTES + V_BYTES + BND_BYTES;
  static constexpr int LIST_CAP = 1024;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int STAGE_OFF = CNT_OFF + 256;   // stages start at multiples of 256 bytes (see the operand reads)
  static constexpr int LDS_BYTES = STAGE_OFF + 2 * STAGE;
  static_assert(STAGE % 256 == 0 && STAGE_OFF % 256 == 0 && K_BYTES % 256 == 0, "XOR after add");
};

// RAGGED: see the forward kernel -- loops at the padded length, clamped tile copies, guarded stores.
template <int D, bool RAGGED, bool GEN>
__global__ __launch_bounds__(256, 2) void dq_kernel(FmBwdArgs a) {
  using C = DqCfg<D>;
  constexpr int KT = C::KT, NKB = KT / 32, NDB = D / 32, NKK = D / 16;
  extern __shared__ __attribute__((aligned(256))) char smem[];   // the operand reads rely on the alignment

  const i32x4 rec = queue_take(a.order_dq, a.slots_dq, (int*)(smem + C::CNT_OFF) + 8);
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
  const int row = qw0 + c;  // this lane's query row
  const int row_ld = RAGGED ? min(row, Nr - 1) : row;

  const int h = bh - b * H, hk = GEN ? h / (H / a.Hk) : h, Hk = GEN ? a.Hk : H;
  const __bf16* qp = slice_ptr<D, GEN>(a.q, a.sq, b, h, H, Nr);
  const __bf16* kp = slice_ptr<D, GEN>(a.k, a.sk, b, hk, Hk, Nr);
  const __bf16* vp = slice_ptr<D, GEN>(a.v, a.sv, b, hk, Hk, Nr);
  const __bf16* dop = slice_ptr<D, GEN>(a.dout, a.sdo, b, h, H, Nr);
  const int q_rs = row_stride<D, GEN>(a.sq), k_rs = row_stride<D, GEN>(a.sk), v_rs = row_stride<D, GEN>(a.sv);
  const int do_rs = row_stride<D, GEN>(a.sdo);
  const int* table = a.minmax_dq + (size_t)b * 8 * t_c;
  // The four bound slices of a partially masked tile (KT ints each, one after the other in LDS) are copied by the
  // first BND_WAVES waves, 1 KB each: a lane moves 16 bytes of vector (64 * wave + lane) / (KT / 4).
  constexpr int BND_LPV = KT / 4, BND_WAVES = 4 * BND_LPV / 64;
  const int* my_bvec;
  {
    const int which = (64 * wave + lane) / BND_LPV;
    const int* p = a.lts;
    if (which == 1) p = a.lte;
    if (which == 2) p = a.uts;
    if (which == 3) p = a.ute;
    my_bvec = p + (size_t)b * N + (lane % BND_LPV) * 4;
  }
  CopyLanes<D> copy_lanes, copy_lanes_v_;
  copy_lanes.init(lane, 2 * k_rs);
  if (GEN) copy_lanes_v_.init(lane, 2 * v_rs);
  const CopyLanes<D>& copy_lanes_v = GEN ? copy_lanes_v_ : copy_lanes;

  bf16x8 qreg[NKK], doreg[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    qreg[kk] = *(const bf16x8*)(qp + (size_t)row_ld * q_rs + kk * 16 + 8 * g);
    doreg[kk] = *(const bf16x8*)(dop + (size_t)row_ld * do_rs + kk * 16 + 8 * g);
  }
  // Algorithm 2's D pre-pass, folded into this loop's prologue (the dO fragments are at hand; the O
  // fragments are loaded in the same layout): D_i = sum_c dO_ic O_ic of this lane's row, a partial sum
  // per lane and one exchange with the lane that holds the other half of the row.  -D and the log2-domain
  // lse (+inf for a row with no visible key and for padding rows, so that P = 0 there) also go to the
  // workspace, where the dK/dV loop, which runs after this one, picks them up per tile.
  const bool real_row = !RAGGED || row < Nr;
  float lse2 = real_row ? a.lse[(size_t)bh * Nr + row] : -INFINITY;
  float dneg = 0.f;
  {
    const __bf16* outp = slice_ptr<D, GEN>(a.out, a.so, b, h, H, Nr);
    const int o_rs = row_stride<D, GEN>(a.so);
    bf16x8 oreg[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) oreg[kk] = *(const bf16x8*)(outp + (size_t)row_ld * o_rs + kk * 16 + 8 * g);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e) dneg -= (float)oreg[kk][e] * (float)doreg[kk][e];
    dneg += partner32(dneg);
    if (!real_row) dneg = 0.f;
  }
  lse2 = (lse2 == -INFINITY) ? INFINITY : lse2 * kLog2e;
  if (g == 0) {
    a.dvec[(size_t)bh * N + row] = dneg;
    a.lse2[(size_t)bh * N + row] = lse2;
  }
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    settle(qreg[kk]);
    settle(doreg[kk]);
  }
  settle(lse2);
  settle(dneg);

  f32x16 dqacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[db][r] = 0.f;

  int* list = (int*)smem;
  int* wave_cnt = (int*)(smem + C::CNT_OFF);
  const float sc = a.scale * kLog2e;
  // lane-dependent LDS offsets inside a tile (row block 0, first column group)
  const int i16 = lane & 15, half = (lane >> 4) & 1;
  const int a_base = C::L::off(c, 16 * g);
  const int t_base0 = C::L::off(4 * g + (i16 >> 2), (16 * half + 4 * (i16 & 3)) * 2);
  const int t_base1 = C::L::off(4 * g + (i16 >> 2) + 8, (16 * half + 4 * (i16 & 3)) * 2);

#define FM_LOAD_TILE(ENTRY, BUF)                                                               \
  {                                                                                            \
    const int j_ = entry_block(ENTRY, chunk);                                                  \
    char* st_ = smem + C::STAGE_OFF + (BUF) * C::STAGE;                                        \
    _Pragma("unroll") for (int sub = 0; sub < KT / 64; ++sub) {   /* 64 keys per copy call */  \
      const int r_ = j_ * KT + sub * 64;                                                       \
      char* ks_ = st_ + sub * 64 * C::L::RS;                                                   \
      if (RAGGED && r_ + 64 > Nr) {                                                            \
        tile_load_async_clamped<D>(kp, r_, Nr, ks_, wave, lane, 2 * k_rs);                     \
        tile_load_async_clamped<D>(vp, r_, Nr, ks_ + C::K_BYTES, wave, lane, 2 * v_rs);        \
      } else {                                                                                 \
        tile_load_async<D>(kp + (size_t)r_ * k_rs, copy_lanes, ks_, wave, 2 * k_rs);           \
        tile_load_async<D>(vp + (size_t)r_ * v_rs, copy_lanes_v, ks_ + C::K_BYTES, wave, 2 * v_rs); \
      }                                                                                        \
    }                                                                                          \
    if (entry_tile_class(ENTRY) == T_PARTIAL && wave < BND_WAVES)                              \
      async_copy16(my_bvec + j_ * KT, lds_address(st_ + C::K_BYTES + C::V_BYTES) + wave * 1024); \
  }

  // only the key blocks [j_lo, j_hi) can be live for this row block (found by the work pre-pass)
  for (int chunk = j_lo; chunk < j_hi; chunk += C::LIST_CAP) {
    const int n_live = build_live_key_blocks(table, t_c, chunk, min(chunk + C::LIST_CAP, j_hi), q0, min(q0 + C::BR, N),
                                             C::BR / 4, list, wave_cnt);
    if (n_live == 0) continue;
    // the entries of tiles t and t + 1 travel in scalar registers; the one that joins them at the next tile is
    // read from the list at the top of a tile and picked up behind the tile's barrier, so that no tile starts by
    // waiting for LDS
    int entry = __builtin_amdgcn_readfirstlane(list[0]);
    int next_entry = __builtin_amdgcn_readfirstlane(list[min(1, n_live - 1)]);
    FM_LOAD_TILE(entry, 0);
    async_wait<0>();
    barrier_nofence();

    for (int t = 0; t < n_live; ++t) {
      const int v_after = list[min(t + 2, n_live - 1)];
      __builtin_amdgcn_sched_barrier(0);
      if (t + 1 < n_live) FM_LOAD_TILE(next_entry, (t + 1) & 1);

      const char* st = smem + C::STAGE_OFF + (t & 1) * C::STAGE;
      const int* bnd = (const int*)(st + C::K_BYTES + C::V_BYTES);

      const int wcls = entry_wave_class(entry, wave);   // Equation 4 on this wave's own rows
      if (wcls != T_FULLY) {
        // Operand addresses: (stage address + lane part) XOR column offset, + constants.  The stage
        // address is a multiple of 256 bytes, so the sum keeps the lane part's low byte and the XOR
        // lands where lane part XOR column offset would put it: one instruction per read, and no
        // per-(pattern, column) register that lives across tiles.
        const unsigned st_a = lds_address(st);
        const unsigned a_s = st_a + (unsigned)a_base, t_s0 = st_a + (unsigned)t_base0, t_s1 = st_a + (unsigned)t_base1;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
          f32x16 sacc, dpacc;
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
          // S^T = K Q^T, then dP^T = V dO^T, for 32 keys x 32 queries: 2*NKK MFMA steps; the LDS
          // operand of a step is fetched RS steps ahead into a small register ring.  The S chain
          // goes first, so that the exponentials P = exp(S - L) can ride along with the dP chain.
          constexpr int NS = 2 * NKK, RS = 3, NT = 2 * NDB, RT = 3;
          constexpr int EXPS = (16 + NKK - 2) / (NKK - 1);   // exponentials next to each of the last NKK - 1 dP steps
          auto s_operand = [&](int n) __attribute__((always_inline)) {
            return lds_read_row16((a_s ^ (unsigned)((n % NKK) * 32)) + (n >= NKK ? C::K_BYTES : 0) + kb * 32 * C::L::RS);
          };
          auto t_operand = [&](int n) __attribute__((always_inline)) {
            const unsigned krow = (kb * 32 + 16 * (n / NDB)) * C::L::RS;
            return cat4(lds_read_tr16_at((t_s0 ^ (unsigned)((n % NDB) * 64)) + krow),
                        lds_read_tr16_at((t_s1 ^ (unsigned)((n % NDB) * 64)) + krow));
          };
          bf16x8 ring[RS];
#pragma unroll
          for (int n = 0; n < RS; ++n) ring[n] = s_operand(n);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int n = 0; n <= NKK; ++n) {   // the S chain and the first dP step
            if (n < NKK) {
              sacc = mfma32(ring[n % RS], qreg[n], sacc);
            } else {
              // the dP accumulator starts from -D of this lane's row, so it ends as dP - D
#pragma unroll
              for (int r = 0; r < 16; ++r) dpacc[r] = dneg;
              dpacc = mfma32(ring[n % RS], doreg[0], dpacc);
            }
            if (n + RS < NS) ring[n % RS] = s_operand(n + RS);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (wcls & T_PARTIAL) {
            // which pairs the workgroup's tile needs (1 = LT, 2 = UT, 3 = both): a pair that is not needed masks
            // no element of the tile, and most partially masked tiles need only one
            const int need = entry_need_pairs(entry);
            if (need == 3) {
#pragma unroll
              for (int rq = 0; rq < 4; ++rq) {
                const int kx = kb * 32 + 8 * rq + 4 * g;
                const i32x4 bl = *(const i32x4*)(bnd + 0 * KT + kx);
                const i32x4 be = *(const i32x4*)(bnd + 1 * KT + kx);
                const i32x4 bu = *(const i32x4*)(bnd + 2 * KT + kx);
                const i32x4 bv = *(const i32x4*)(bnd + 3 * KT + kx);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const bool masked = ((row >= bl[e]) & (row < be[e])) | ((row >= bu[e]) & (row < bv[e]));
                  if (masked) sacc[rq * 4 + e] = -INFINITY;
                }
              }
            } else {
              const int* b_lo = bnd + (need == 2 ? 2 * KT : 0);
#pragma unroll
              for (int rq = 0; rq < 4; ++rq) {
                const int kx = kb * 32 + 8 * rq + 4 * g;
                const i32x4 bs = *(const i32x4*)(b_lo + kx);
                const i32x4 be = *(const i32x4*)(b_lo + KT + kx);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const bool masked = (row >= bs[e]) & (row < be[e]);
                  if (masked) sacc[rq * 4 + e] = -INFINITY;
                }
              }
            }
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int n = NKK + 1; n < NS; ++n) {   // the rest of the dP chain, P = exp(S - L) beside it
            dpacc = mfma32(ring[n % RS], doreg[n - NKK], dpacc);
            if (n + RS < NS) ring[n % RS] = s_operand(n + RS);
#pragma unroll
            for (int r = (n - NKK - 1) * EXPS; r < (n - NKK) * EXPS && r < 16; ++r)
              sacc[r] = fast_exp2(__builtin_fmaf(sacc[r], sc, -lse2));
            __builtin_amdgcn_sched_barrier(0);
          }
          // K^T operands of the dQ product do not depend on dS: fetch the first ones now
          bf16x8 tring[RT];
#pragma unroll
          for (int n = 0; n < RT; ++n) tring[n] = t_operand(n);
          __builtin_amdgcn_sched_barrier(0);
          // dS = P o (dP - D): the first 16-key half before the dQ product, the second half spread
          // over the product's first NDB steps (which only need the first)
          auto ds_elems = [&](int r0, int r1) __attribute__((always_inline)) {
#pragma unroll
            for (int r = r0; r < r1; ++r) sacc[r] *= dpacc[r];
          };
          ds_elems(0, 8);
          __builtin_amdgcn_sched_barrier(0);
          // dQ^T += K^T dS^T, step n = (16-key half n / NDB, d block n % NDB)
          bf16x8 dsb;
#pragma unroll
          for (int n = 0; n < NT; ++n) {
            if (n % NDB == 0) {
#pragma unroll
              for (int e = 0; e < 8; ++e) dsb[e] = (__bf16)sacc[8 * (n / NDB) + e];
            }
            dqacc[n % NDB] = mfma32(tring[n % RT], dsb, dqacc[n % NDB]);
            if (n + RT < NT) tring[n % RT] = t_operand(n + RT);
            if (n < NDB) ds_elems(8 + n * (8 / NDB), 8 + (n + 1) * (8 / NDB));
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }

      async_wait<0>();   // the next tile has landed ...
      barrier_nofence(); // ... for every wave, and every wave is done reading this one
      entry = next_entry;
      next_entry = __builtin_amdgcn_readfirstlane(v_after);
    }
    __syncthreads();     // the list is rebuilt by the next pass
  }
#undef FM_LOAD_TILE

  __bf16* dqp = (__bf16*)slice_ptr<D, GEN>(a.dq, a.sdq, b, h, H, Nr);
  const int dq_rs = row_stride<D, GEN>(a.sdq);
  // every wave is past its last tile and nothing is in flight into the stages (the barrier that ends a
  // pass over the list): their first bytes serve as the waves' store staging
  using RSt = RowStage<D>;
  static_assert(4 * RSt::BYTES <= 2 * C::STAGE, "store staging fits the stages");
  char* stage = smem + C::STAGE_OFF + wave * RSt::BYTES;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(dqacc[db][rq * 4 + e] * a.scale);
      RSt::put(stage, c, g, db, rq, o4);
    }
  RSt::flush(stage, dqp + (size_t)qw0 * dq_rs, dq_rs, lane, RAGGED ? min(32, Nr - qw0) : 32);
}

// ---------------------------------------------------------------------------
// dK, dV: column-parallel.  A workgroup owns FM_DKDV_BC = 128 keys (32 per
// wave, K and V fragments resident in registers) and walks the row blocks of
// FM_DKDV_BR = 64 queries that are not fully masked for its keys.  Scores are
// NOT transposed here (S = Q K^T): every lane then holds one KEY column, so the
// four bounds of that key sit in four registers for the whole kernel and P^T,
// dS^T are already A operands of dV += P^T dO and dK += dS^T Q.
//
// One wave per SIMD at d = 128 (the accumulators alone take 128 registers; at d = 64 they take 64 and
// two workgroups share a CU), so the overlap of matrix and vector work is arranged inside the wave: a 64-row tile
// is two 32-row blocks, and the instruction stream is
//   S0,dP0 | S1,dP1 with the exp/dS arithmetic of block 0 between the MFMAs |
//   dV,dK of block 0 with the arithmetic of block 1 between the MFMAs | dV,dK of block 1
// with every LDS operand fetched a fixed number of steps ahead of its MFMA.
// Scheduling fences pin that order.
// ---------------------------------------------------------------------------
template <int D>
struct DkdvCfg {
  static constexpr int QT = FM_DKDV_BR;    // query rows per step
  static constexpr int BC = FM_DKDV_BC;    // keys per workgroup
  using L = TileLayout<D>;
  static constexpr int Q_BYTES = QT * L::RS;
  static constexpr int DO_BYTES = QT * L::RS;
  static constexpr int VEC_BYTES = 2 * QT * 4;  // lse (log2 domain, +inf for dead rows) and D of the rows
  static constexpr int STAGE = Q_BYTES + DO_BYTES + VEC_BYTES;
  static constexpr int LIST_CAP = 2048;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int STAGE_OFF = CNT_OFF + 256;   // stages start at multiples of 256 bytes (dkdv_operand)
  // One workgroup per CU: a tile's math takes about a microsecond, less than a
  // trip to L2/HBM, so tiles are copied three steps ahead into a ring of four.
  static constexpr int NSTAGE = 4;
  static constexpr int LDS_BYTES = STAGE_OFF + NSTAGE * STAGE;
  // async copy instructions one wave issues per tile: COPIES for its quarter of Q and dO plus
  // one for its quarter of the lse / D slice.  Every wave issues the same number for every
  // tile, so "tile landed" is a constant outstanding-copy count.
  static constexpr int COPIES = 2 * (QT / (64 / L::CPR) / 4);
  static constexpr int NC = COPIES + 1;
  // MFMA operand fetch distance in steps; divides the steps per tile, so ring slots line up across tiles
  static constexpr int RD = 8;
};

// lse / D slice of a tile in LDS: wave w copies rows 16w..16w+15 as 128 contiguous bytes,
// 64 bytes of lse then 64 bytes of D.  Float offset of row r (r % 4 == 0 for the 16-byte reads):
__device__ __forceinline__ constexpr int dkdv_vec_off(int r, bool d_part) {
  return (r >> 4) * 32 + (d_part ? 16 : 0) + (r & 15);
}

#define FM_FENCE() __builtin_amdgcn_sched_barrier(0)
// Steps between the last MFMA of a block's S / dP chains and the first vector instruction that reads their
// result: with none, that instruction waits out the MFMA's passes with the wave idle (one wave per SIMD).
#ifndef FM_DKDV_VSHIFT
#define FM_DKDV_VSHIFT 1
#endif

// exp / dS arithmetic of elements [e0, e0 + cnt) of one 32x32 block held in the
// MFMA output layout: register r is query row 8*(r/4) + 4*g + r%4 of the block.
// The exp / dS arithmetic of one score element, cut into three stages that the
// tile loop issues in three consecutive steps, so that a step never holds two
// dependent vector instructions of the same element (one wave per SIMD: nothing
// else hides the latency of v_exp_f32 and of the AGPR reads):
//   A: t = s*sc - lse2 (with the element mask)     B: p = exp2(t)     C: dS = p * (dP - D)
// (dP - D comes straight out of the MFMA: its accumulator starts from the -D values of the rows)
// Register r of a block is query row 8*(r/4) + 4*g + r%4.
// The element mask of a lane's key is two row intervals [s, e): row q is masked by one iff
// (unsigned)(q - s) < (unsigned)max(e - s, 0), one subtraction and one compare per element with the interval's
// length formed once per unit (off_a, off_b: first row of the block's registers - s).
template <bool MASK>
__device__ __forceinline__ void dkdv_stage_a(const f32x16& s, const f32x16& dp, float (&t)[16],
                                             float (&u)[16], const f32x4 (&l4)[4], int e0,
                                             int cnt, float sc, int off_a, unsigned len_a, int off_b, unsigned len_b) {
#pragma unroll
  for (int r = e0; r < e0 + cnt; ++r) {
    float x = s[r];
    if (MASK) {
      const int dr = 8 * (r >> 2) + (r & 3);   // register r is row 8*(r/4) + 4*g + r%4 of the block; 4*g is in the offsets
      const bool hit = ((unsigned)(off_a + dr) < len_a) | ((unsigned)(off_b + dr) < len_b);
      if (hit) x = -INFINITY;
    }
    t[r] = __builtin_fmaf(x, sc, -l4[r >> 2][r & 3]);
    u[r] = dp[r];   // dP - D: the dP accumulator was started from -D
  }
}

// What the tail of a tile's stream does for the tiles that follow it.
struct DkdvAhead {
  const char* nqs;        // LDS: stage of the next list entry (its Q tile; dO follows), for the operand prefetch
  int v_copy;             // list entry (still in a vector register) of the tile NSTAGE - 1 ahead, to be copied
  const char* q_base;     // global Q / dO of this (batch, head), already advanced to this wave's 16-row block
  const char* do_base;    // of a tile, and this lane's lse2 / D source
  const float* vec_src;
  int q_rs2, do_rs2;      // bytes between consecutive rows of Q / dO in global memory
  unsigned lds_ring;      // LDS address of stage 0
  unsigned stage_copy;    // index of the stage that receives the copy
  int n_real, lane;       // ragged sequences: rows the tensors really have, and this thread's lane
  CopyLanes<128> lanes;   // per-lane source offsets of the copy instructions of Q (the first D/32 entries are used)
  CopyLanes<128> lanes_do;   // ... and of dO
  int wave;
};

// Copy number K (of NC) of the tile whose 64-row base offsets are given.  RAGGED: a tile that
// reaches past the last real row (i_copy is its index) clamps every lane's source row instead.
template <int D, int K, bool RAGGED>
__device__ __forceinline__ void dkdv_issue_copy(const DkdvAhead& ah, const char* q_src, const char* do_src,
                                                const float* vec_src, unsigned lds_stage, int i_copy) {
  using C = DkdvCfg<D>;
  constexpr int HALF = C::COPIES / 2;
  constexpr int WB = 16 * C::L::RS;   // bytes of a wave's 16-row block
  if (RAGGED && K < C::COPIES && (i_copy + 1) * C::QT > ah.n_real) {
    constexpr int RPI = 64 / C::L::CPR, S = K % HALF;
    const int row = ah.wave * 16 + S * RPI + ah.lane / C::L::CPR;
    const int grow = min(i_copy * C::QT + row, ah.n_real - 1);
    const char* base = K < HALF ? ah.q_base : ah.do_base;
    const long long rel = (long long)(grow - ah.wave * 16) * (K < HALF ? ah.q_rs2 : ah.do_rs2);   // the bases are this wave's
    const char* src = base + rel + (((ah.lane % C::L::CPR) ^ C::L::swz(row)) << 4);
    async_copy16(src, lds_stage + (K < HALF ? 0 : C::Q_BYTES) + ah.wave * WB + S * 1024);
    return;
  }
  if (K < HALF) {
    if (K == 0 || RAGGED) async_window(lds_stage + ah.wave * WB);
    async_copy16_window<(K % HALF) * 1024>(q_src, ah.lanes.v[K % HALF]);
  } else if (K < C::COPIES) {
    if (K == HALF || RAGGED) async_window(lds_stage + C::Q_BYTES + ah.wave * WB);
    async_copy16_window<(K % HALF) * 1024>(do_src, ah.lanes_do.v[K % HALF]);
  } else {
    async_copy16_lanes8(vec_src, lds_stage + C::Q_BYTES + C::DO_BYTES + ah.wave * 128);
  }
}

// Order of the 2*NKK score MFMAs of one 32-row block (step y): the S chain leads by NKK/2
// steps, so the -D values the dP chain starts from have time to arrive from LDS:
//   y < H: S   |   H <= y < 3H: dP, S alternating   |   y >= 3H: dP          (H = NKK / 2)
template <int D>
__device__ __forceinline__ constexpr bool dkdv_is_s(int y) {
  constexpr int H = D / 32;
  return y < H || (y < 3 * H && ((y - H) & 1));
}
template <int D>
__device__ __forceinline__ constexpr int dkdv_kk(int y) {
  constexpr int H = D / 32;
  if (y < H) return y;
  if (y < 3 * H) return ((y - H) & 1) ? H + (y - H - 1) / 2 : (y - H) / 2;
  return H + (y - 3 * H);
}

// Per-lane LDS addresses of a list entry's stage: the stage's address plus the lane-dependent part of
// the three read patterns (row reads; transpose reads of rows 0-7 and 8-15 of a 16-row group).  A
// step's column offset is XORed into the sum -- stage addresses are multiples of 256 bytes, so the sum
// keeps the lane part's low byte -- which costs one instruction per read and no register that lives
// across tiles; XORing into the lane part first would either keep every (pattern, column) pair in a
// register for the whole loop or take two instructions per read.
struct DkdvBases {
  unsigned a, t0, t1;
};
__device__ __forceinline__ DkdvBases dkdv_bases(const char* qs, int a_base, int t_base0, int t_base1) {
  const unsigned s = lds_address(qs);
  return DkdvBases{s + (unsigned)a_base, s + (unsigned)t_base0, s + (unsigned)t_base1};
}
// LDS operand of step x of the list entry whose stage addresses are bs (Q tile, dO tile right behind it)
template <int D>
__device__ __forceinline__ bf16x8 dkdv_operand(const DkdvBases& bs, int x) {
  using L = TileLayout<D>;
  constexpr int NKK = D / 16, NDB = D / 32, NST = 2 * NKK;
  constexpr unsigned DO = DkdvCfg<D>::Q_BYTES;
  static_assert(DkdvCfg<D>::STAGE % 256 == 0 && DkdvCfg<D>::STAGE_OFF % 256 == 0 && DO % 256 == 0, "XOR after add");
  if (x < 2 * NST) {             // row reads: Q or dO rows of block x / NST as MFMA A operand
    const int qb = x / NST;
    const unsigned tile = dkdv_is_s<D>(x % NST) ? 0u : DO;
    return lds_read_row16((bs.a ^ (unsigned)(dkdv_kk<D>(x % NST) * 32)) + tile + qb * 32 * L::RS);
  }
  // transpose reads: dO (even step, dV) or Q (odd step, dK) as MFMA B operand
  const int u = x - 2 * NST, qb = u / NST, w = u % NST, h = w / (2 * NDB), db = (w % (2 * NDB)) / 2;
  const unsigned rows = ((u & 1) ? 0u : DO) + (qb * 32 + 16 * h) * L::RS;
  return cat4(lds_read_tr16_at((bs.t0 ^ (unsigned)(db * 64)) + rows), lds_read_tr16_at((bs.t1 ^ (unsigned)(db * 64)) + rows));
}

// The workgroup-level step that every wave takes once per list entry, in the middle of the
// entry's stream : wait for this wave's part of the
// NEXT entry's tile, meet the other waves (so the next tile is complete in LDS and nobody
// still reads the previous one), then the caller refills the previous tile's stage.
template <int D>
__device__ __forceinline__ void dkdv_sync() {
  async_wait<DkdvCfg<D>::NC>();   // copies complete in order: only the tile after the next may be in flight
  // The operand ring has reads of this entry's and the next entry's stages in flight here.  The stage
  // refilled after the barrier is the PREVIOUS entry's: its last read fed an MFMA a whole tile of
  // steps ago, in program order, so it has long returned.
  barrier_reads_in_flight();
}

// One 64-row tile = two 32-row blocks.  The tile's 8*NKK MFMAs form one stream
//   [S0 | dP0 | S1 | dP1 | dV,dK of block 0 | dV,dK of block 1]      (NKK = D/16 MFMAs per bar, 2*NKK for dV,dK)
// each taking one operand from LDS (a 128-bit row read for the first four
// groups, a transpose read for the rest) that is fetched RD steps ahead into a
// small register ring.  The exp / dS arithmetic of block 0 is spread over the
// steps of S1 and dP1, that of block 1 over the dV,dK steps of block 0, so the
// vector work always has matrix work in flight beside it.  The stream runs on
// into the next list entry: near its end the wave takes the workgroup step
// (dkdv_sync), issues the copies of the tile NSTAGE - 1 entries ahead one per
// step, and its last RD operand fetches already read the next entry's tile, so
// the MFMA pipe does not drain between tiles.  On entry `op` holds the operands
// of steps 0..RD-1 of this tile, on exit those of the next one.
template <int D, bool MASK, bool RAGGED>
__device__ __forceinline__ void dkdv_tile(const char* qs, const float* vec_s, const DkdvAhead& ah,
                                          bf16x8 (&op)[DkdvCfg<D>::RD], const bf16x8 (&kreg)[D / 16],
                                          const bf16x8 (&vreg)[D / 16], f32x16 (&dkacc)[D / 32],
                                          f32x16 (&dvacc)[D / 32], int a_base, int t_base0, int t_base1, int r0,
                                          int g, float sc, int s_a, unsigned len_a, int s_b, unsigned len_b) {
  using C = DkdvCfg<D>;
  constexpr int NKK = D / 16, NDB = D / 32;
  constexpr int NST = 2 * NKK;     // MFMAs per block and product pair
  constexpr int EPS = 16 / NST;    // elements handled next to one MFMA (D = 128: 1, D = 64: 2)
  constexpr int NX = 4 * NST;      // MFMAs per tile
  constexpr int RD = C::RD;
  constexpr int XS = NX - (C::NC > RD ? C::NC : RD);   // step of the workgroup sync; the copies follow one per step
  static_assert(NX % RD == 0 && XS > 0, "ring layout");
  const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  const DkdvBases bs_cur = dkdv_bases(qs, a_base, t_base0, t_base1);
  const DkdvBases bs_next = dkdv_bases(ah.nqs, a_base, t_base0, t_base1);

  f32x16 sb[2], pb[2];             // S then P, dP then dS, of the two blocks
  bf16x8 pa[2][2], dsa[2][2];      // bf16 P^T and dS^T, [block][16-row half]
  f32x4 l4[2][4];                  // lse (log2 domain) of the blocks' rows, fetched one group of 4 rows ahead
  float tq[2][16], uq[2][16];      // per element: exponent then P, and dP - D then dS
  auto vec_group = [&](int qb, int grp) __attribute__((always_inline)) {
    const int row = qb * 32 + 8 * grp + 4 * g;
    l4[qb][grp] = *(const f32x4*)(vec_s + dkdv_vec_off(row, false));
  };
  const char* q_src = nullptr;
  const char* do_src = nullptr;
  const float* vec_src = nullptr;
  unsigned lds_stage = 0;
  int i_copy = 0;

#pragma unroll
  for (int x = 0; x < NX; ++x) {
    // --- the MFMA of this step
    if (x < 2 * NST) {
      const int qb = x / NST, y = x % NST, kk = dkdv_kk<D>(y);   // two independent accumulation chains
      if (y == 0) {   // the dP accumulator starts from -D of the block's rows (register r: row 8*(r/4) + 4*g + r%4)
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
          const f32x4 dn = *(const f32x4*)(vec_s + dkdv_vec_off(qb * 32 + 8 * grp + 4 * g, true));
#pragma unroll
          for (int i = 0; i < 4; ++i) pb[qb][4 * grp + i] = dn[i];
        }
      }
      if (dkdv_is_s<D>(y))
        sb[qb] = mfma32(op[x % RD], kreg[kk], kk == 0 ? zero : sb[qb]);
      else
        pb[qb] = mfma32(op[x % RD], vreg[kk], pb[qb]);
    } else {
      const int u = x - 2 * NST, qb = u / NST, w = u % NST, h = w / (2 * NDB), db = (w % (2 * NDB)) / 2;
      if (D == 64) {
        // d = 64: the accumulators are half as many and two workgroups share a CU (two waves per SIMD,
        // 256 registers each), so they stay ordinary compiler-managed registers
        if (u & 1)
          dkacc[db] = mfma32(op[x % RD], dsa[qb][h], dkacc[db]);
        else
          dvacc[db] = mfma32(op[x % RD], pa[qb][h], dvacc[db]);
      } else if (u & 1) {
        // dsa[qb][h] / pa[qb][h] were converted several steps ago (the vector work of a block ends before the
        // block's dV, dK steps begin), so no idle instruction is needed in front of their first reader
        mfma32_acc(dkacc[db], op[x % RD], dsa[qb][h], false);
      } else {
        mfma32_acc(dvacc[db], op[x % RD], pa[qb][h], false);
      }
    }
    // --- the workgroup step and the copies behind it
    if (x == XS) {
      dkdv_sync<D>();
      i_copy = __builtin_amdgcn_readfirstlane(ah.v_copy) & 0xFFFFFF;
      q_src = ah.q_base + (size_t)i_copy * C::QT * ah.q_rs2;
      do_src = ah.do_base + (size_t)i_copy * C::QT * ah.do_rs2;
      vec_src = ah.vec_src + i_copy * C::QT;
      lds_stage = ah.lds_ring + ah.stage_copy * C::STAGE;
    }
    if (x >= XS && x < XS + C::NC) {
      switch (x - XS) {
        case 0: dkdv_issue_copy<D, 0, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 1: dkdv_issue_copy<D, 1, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 2: dkdv_issue_copy<D, 2, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 3: dkdv_issue_copy<D, 3, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 4: dkdv_issue_copy<D, 4, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 5: dkdv_issue_copy<D, 5, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 6: dkdv_issue_copy<D, 6, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        case 7: dkdv_issue_copy<D, 7, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
        default: dkdv_issue_copy<D, 8, RAGGED>(ah, q_src, do_src, vec_src, lds_stage, i_copy); break;
      }
    }
    // --- fetch the operand of step x + RD (of the next tile once this one is used up)
    if (x + RD < NX)
      op[x % RD] = dkdv_operand<D>(bs_cur, x + RD);
    else
      op[x % RD] = dkdv_operand<D>(bs_next, x + RD - NX);
    // --- vector work riding along.  Vector step j handles EPS elements of
    //     block j / NST: stage A at x, stage B one step later, stage C two steps later
    //     (j = x - NST - FM_DKDV_VSHIFT - stage).
    if (x == NST - 1) vec_group(0, 0);
#pragma unroll
    for (int stage = 2; stage >= 0; --stage) {
      const int j = x - NST - FM_DKDV_VSHIFT - stage;
      if (j >= 0 && j < 2 * NST) {
        const int qb = j / NST, e0 = (j % NST) * EPS;
        if (stage == 0) {
          if (e0 % 4 == 0 && e0 / 4 + 1 < 4) vec_group(qb, e0 / 4 + 1);
          if (qb == 0 && e0 + EPS == 16) vec_group(1, 0);
          dkdv_stage_a<MASK>(sb[qb], pb[qb], tq[qb], uq[qb], l4[qb], e0, EPS, sc, r0 + 32 * qb + 4 * g - s_a, len_a,
                             r0 + 32 * qb + 4 * g - s_b, len_b);
        } else if (stage == 1) {
#pragma unroll
          for (int r = e0; r < e0 + EPS; ++r) tq[qb][r] = fast_exp2(tq[qb][r]);
        } else {
#pragma unroll
          for (int r = e0; r < e0 + EPS; ++r) uq[qb][r] *= tq[qb][r];
          if ((e0 + EPS) % 8 == 0) {   // a 16-row half of P^T and dS^T is complete: convert it to bf16 operands
            const int hh = (e0 + EPS) / 8 - 1;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              pa[qb][hh][e] = (__bf16)tq[qb][8 * hh + e];
              dsa[qb][hh][e] = (__bf16)uq[qb][8 * hh + e];
            }
          }
        }
      }
    }
    FM_FENCE();
  }
}

// RAGGED: see the forward kernel -- loops at the padded length, clamped tile copies and fragment
// loads, guarded stores; the padding rows carry lse = +inf (P = 0), the padding keys are masked.
// GEN: tensors with caller-given strides; a workgroup then owns 128 keys of one K/V head and
// walks the query heads that share it one after the other (same list of live row blocks: the
// mask does not depend on the head), accumulating dK and dV over all of them.
template <int D, bool RAGGED, bool GEN>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1) void dkdv_kernel(FmBwdArgs a) {
  using C = DkdvCfg<D>;
  constexpr int QT = C::QT, NDB = D / 32, NKK = D / 16;
  static_assert(QT == 64, "the tile loop is written for two 32-row blocks per tile");
  extern __shared__ __attribute__((aligned(256))) char smem[];   // dkdv_operand relies on the alignment

  // hand-off words of the unit queue: int 8 = slot of the first take, ints 12..15 = record of the next unit
  int* qwords = (int*)(smem + C::CNT_OFF);
  i32x4 rec = queue_take(a.order_dkdv, a.slots_dkdv, qwords + 8);
  if (rec[0] < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int N = a.Np, H = a.H;            // padded length: what the loops and tables see
  const int Hk = GEN ? a.Hk : H, G = GEN ? H / Hk : 1;   // K/V heads, query heads per K/V head
  const int Nr = RAGGED ? a.N : a.Np;     // rows the tensors really have
  const int t_r = N / QT, t_c = N / C::BC;
  const int q_rs = row_stride<D, GEN>(a.sq), k_rs = row_stride<D, GEN>(a.sk), v_rs = row_stride<D, GEN>(a.sv);
  const int do_rs = row_stride<D, GEN>(a.sdo);
  int* list = (int*)smem;
  int* wave_cnt = (int*)(smem + C::CNT_OFF);
  const float sc = a.scale * kLog2e;
  // lane-dependent LDS offsets inside a tile (row block 0, first column group)
  const int i16 = lane & 15, half = (lane >> 4) & 1;
  const int a_base = C::L::off(c, 16 * g);
  const int t_base0 = C::L::off(4 * g + (i16 >> 2), (16 * half + 4 * (i16 & 3)) * 2);
  const int t_base1 = C::L::off(4 * g + (i16 >> 2) + 8, (16 * half + 4 * (i16 & 3)) * 2);
  CopyLanes<D> copy_lanes, copy_lanes_do_;
  copy_lanes.init(lane, 2 * q_rs);
  if (GEN) copy_lanes_do_.init(lane, 2 * do_rs);
  const CopyLanes<D>& copy_lanes_do = GEN ? copy_lanes_do_ : copy_lanes;
  const unsigned lds_ring = lds_address(smem + C::STAGE_OFF);

  DkdvAhead ah;
  ah.q_rs2 = 2 * q_rs;
  ah.do_rs2 = 2 * do_rs;
  ah.lds_ring = lds_ring;
#pragma unroll
  for (int s = 0; s < CopyLanes<D>::NINST; ++s) {
    ah.lanes.v[s] = copy_lanes.v[s];
    ah.lanes_do.v[s] = copy_lanes_do.v[s];
  }
  ah.wave = wave;
  ah.n_real = Nr;
  ah.lane = lane;
  bf16x8 op[C::RD];

  // One pass of the tile loop over list entries [T0, T1) with the element mask compiled in or
  // out.  Tiles that need no element mask are listed first and run through the mask-free
  // instantiation, partially masked ones (for the workgroup's 128 keys) through the other;
  // keeping the two instantiations in separate loops keeps the 128 accumulator registers where
  // they are (merged into one loop, the compiler shuffled all of them every tile; a third loop for
  // tiles that need only one of the two intervals made it spill inside the mask-free one).
  // Entries past the end of the list are clamped to the last one: the copies and operand
  // fetches made for them are never used, and every entry costs the same number of copies.
#define FM_TILE_LOOP(T0, T1, MASK)                                                                     \
  for (int t = (T0); t < (T1); ++t) {                                                                  \
    const int v_next = list[min(t + 1, n_live - 1)];                                                   \
    ah.v_copy = list[min(t + C::NSTAGE - 1, n_live - 1)];                                              \
    ah.nqs = smem + C::STAGE_OFF + ((t + 1) % C::NSTAGE) * C::STAGE;                                   \
    ah.stage_copy = (t + C::NSTAGE - 1) % C::NSTAGE;                                                   \
    const char* st = smem + C::STAGE_OFF + (t % C::NSTAGE) * C::STAGE;                                 \
    const int r0 = (e_cur & 0xFFFFFF) * QT;                                                            \
    dkdv_tile<D, MASK, RAGGED>(st, (const float*)(st + C::Q_BYTES + C::DO_BYTES), ah, op, kreg, vreg, dkacc, dvacc, \
                         a_base, t_base0, t_base1, r0, g, sc, b_lts, len_lt, b_uts, len_ut);           \
    e_cur = __builtin_amdgcn_readfirstlane(v_next);                                                    \
  }

  // the first unit's min/max values (Section 4.2's table); the later units' arrive with their records
  MinMax8 gmm;
  {
    const int bh0 = rec[0] / t_c;
    gmm = load_minmax(a.minmax_dkdv + (size_t)(bh0 / Hk) * 8 * t_c, t_c, rec[0] - bh0 * t_c);
    // into scalar registers here, once: left in vector registers, every unit's list build would wait for
    // "these loads" again, i.e. for everything the workgroup has in flight, the previous unit's result
    // stores included
#pragma unroll
    for (int e = 0; e < 8; ++e) gmm.v[e] = __builtin_amdgcn_readfirstlane(gmm.v[e]);
  }

  // A workgroup works units off until the queues are empty: the launch holds as many workgroups as the
  // chip runs at once, and the next unit's ticket, record and min/max values are fetched while the first
  // tile copies of the current unit are in flight.
  while (true) {
  const int unit = rec[0], i_lo = rec[1], i_hi = rec[2];
  const int bh = unit / t_c, j_blk = unit - bh * t_c, b = bh / Hk, hk = bh - b * Hk;   // bh counts K/V heads
  const int k0 = j_blk * C::BC;
  const int kw0 = k0 + wave * 32;
  const int key = kw0 + c;  // this lane's key column
  const int key_ld = RAGGED ? min(key, Nr - 1) : key;

  const __bf16* kp = slice_ptr<D, GEN>(a.k, a.sk, b, hk, Hk, Nr);
  const __bf16* vp = slice_ptr<D, GEN>(a.v, a.sv, b, hk, Hk, Nr);

  // K and V fragments of this wave's 32 keys (B operands of S = Q K^T, dP = dO V^T) and the four
  // bounds of this lane's key, which stay in registers (Algorithm 2 loads them once per key
  // block).  They are only waited for after the first tile copies have been issued.
  bf16x8 kreg[NKK], vreg[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    kreg[kk] = *(const bf16x8*)(kp + (size_t)key_ld * k_rs + kk * 16 + 8 * g);
    vreg[kk] = *(const bf16x8*)(vp + (size_t)key_ld * v_rs + kk * 16 + 8 * g);
  }
  int b_lts = a.lts[(size_t)b * N + key], b_lte = a.lte[(size_t)b * N + key];
  int b_uts = a.uts[(size_t)b * N + key], b_ute = a.ute[(size_t)b * N + key];

  f32x16 dkacc[NDB], dvacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dkacc[db][r] = 0.f;
      dvacc[db][r] = 0.f;
    }
  bool drawn = false;   // the next unit's ticket has been drawn (uniform over the workgroup)

  // only the row blocks [i_lo, i_hi) can be live for this key block (found by the work pre-pass)
  for (int chunk = i_lo; chunk < i_hi; chunk += C::LIST_CAP) {
    int n_plain = 0;
    const int n_live = build_live_row_blocks(gmm, N, QT, chunk, min(chunk + C::LIST_CAP, i_hi), list, wave_cnt, n_plain);
    if (n_live == 0) continue;
    // the query heads that share this K/V head, one after the other (one pass if there is no sharing)
    for (int hq = 0; hq < (GEN ? G : 1); ++hq) {
    const int h = hk * G + hq;
    const __bf16* qp = slice_ptr<D, GEN>(a.q, a.sq, b, h, H, Nr);
    const __bf16* dop = slice_ptr<D, GEN>(a.dout, a.sdo, b, h, H, Nr);
    // every wave copies its 16 rows of a tile's lse and D slices with lanes 0..7:
    // lanes 0-3 lse, lanes 4-7 D, 16 bytes each
    const float* my_vec = ((lane & 4) ? a.dvec : a.lse2) + (size_t)(b * H + h) * N + wave * 16 + (lane & 3) * 4;
    ah.q_base = (const char*)qp + (size_t)(wave * 16) * ah.q_rs2;
    ah.do_base = (const char*)dop + (size_t)(wave * 16) * ah.do_rs2;
    ah.vec_src = my_vec;
    // prologue: copies of the first NSTAGE - 1 tiles, then the first tile's first operands
#pragma unroll
    for (int p = 0; p < C::NSTAGE - 1; ++p) {
      const int i_p = __builtin_amdgcn_readfirstlane(list[min(p, n_live - 1)]) & 0xFFFFFF;
      char* st_ = smem + C::STAGE_OFF + p * C::STAGE;
      if (RAGGED && (i_p + 1) * QT > Nr) {
        tile_load_async_clamped<D>(qp, i_p * QT, Nr, st_, wave, lane, 2 * q_rs);
        tile_load_async_clamped<D>(dop, i_p * QT, Nr, st_ + C::Q_BYTES, wave, lane, 2 * do_rs);
      } else {
        tile_load_async<D>(qp + (size_t)i_p * QT * q_rs, copy_lanes, st_, wave, 2 * q_rs);
        tile_load_async<D>(dop + (size_t)i_p * QT * do_rs, copy_lanes_do, st_ + C::Q_BYTES, wave, 2 * do_rs);
      }
      async_copy16_lanes8(my_vec + i_p * QT, lds_address(st_ + C::Q_BYTES + C::DO_BYTES) + wave * 128);
    }
    // the next unit's ticket and record, while these copies are in flight
    if (!drawn) {
      if (tid == 0) queue_prefetch_key_block(a.order_dkdv, a.slots_dkdv, qwords + 12, a.minmax_dkdv, t_c, Hk);
      drawn = true;
    }
    // The fragment and bound loads must be complete, and known complete to the compiler, before
    // the tile loops: a compiler-inserted wait for them inside a loop would also drain the
    // copies in flight there.  (No-op after the first chunk.)
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      settle(kreg[kk]);
      settle(vreg[kk]);
    }
    settle(b_lts);
    settle(b_lte);
    settle(b_uts);
    settle(b_ute);
    // lengths of the key's two masked row intervals (0 for an empty one), for the element mask's compare
    const unsigned len_lt = (unsigned)max(b_lte - b_lts, 0), len_ut = (unsigned)max(b_ute - b_uts, 0);
    async_wait<(C::NSTAGE - 2) * C::NC>();
    barrier_nofence();
    int e_cur = __builtin_amdgcn_readfirstlane(list[0]);
#pragma unroll
    for (int x = 0; x < C::RD; ++x)
      op[x] = dkdv_operand<D>(dkdv_bases(smem + C::STAGE_OFF, a_base, t_base0, t_base1), x);
    FM_TILE_LOOP(0, n_plain, false)
    FM_TILE_LOOP(n_plain, n_live, true)
    mfma_acc_drain();  // dkacc / dvacc are read by ordinary code after the loops over heads and chunks
    async_wait<0>();   // the copies made for entries past the end must not outlive the list / the workgroup
    __syncthreads();   // the ring is refilled by the next head, the list rebuilt by the next chunk
    }  // query heads
  }
  if (!drawn) {   // a unit without a live tile: nothing was in flight to hide the draw behind
    if (tid == 0) queue_prefetch_key_block(a.order_dkdv, a.slots_dkdv, qwords + 12, a.minmax_dkdv, t_c, Hk);
  }

  // accumulators (dK^T, dV^T): register r of block db holds [d = db*32 + 8*(r/4) + 4*g + r%4][key kw0 + c].
  // Nothing is in flight into the ring here and every wave is past its last tile (the barrier that ends the
  // loop over heads and chunks), so the ring's first bytes serve as the waves' store staging.
  __bf16* dkp = (__bf16*)slice_ptr<D, GEN>(a.dk, a.sdk, b, hk, Hk, Nr);
  __bf16* dvp_out = (__bf16*)slice_ptr<D, GEN>(a.dv, a.sdv, b, hk, Hk, Nr);
  const int dk_rs = row_stride<D, GEN>(a.sdk), dv_rs = row_stride<D, GEN>(a.sdv);
  {
    using RSt = RowStage<D>;
    static_assert(8 * RSt::BYTES <= C::NSTAGE * C::STAGE, "store staging fits the ring");
    char* stage_k = smem + C::STAGE_OFF + (2 * wave) * RSt::BYTES;
    char* stage_v = stage_k + RSt::BYTES;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        bf16x4 k4, v4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          k4[e] = (__bf16)(dkacc[db][4 * q + e] * a.scale);
          v4[e] = (__bf16)dvacc[db][4 * q + e];
        }
        RSt::put(stage_k, c, g, db, q, k4);
        RSt::put(stage_v, c, g, db, q, v4);
      }
    const int n_rows = RAGGED ? min(32, Nr - kw0) : 32;
    RSt::flush(stage_k, dkp + (size_t)kw0 * dk_rs, dk_rs, lane, n_rows);
    RSt::flush(stage_v, dvp_out + (size_t)kw0 * dv_rs, dv_rs, lane, n_rows);
  }
  __syncthreads();                       // the next record is in LDS (written before the tile loops, or just above)
  rec = queue_next_record(qwords + 12);
  if (rec[0] < 0) break;
#pragma unroll
  for (int e = 0; e < 8; ++e) gmm.v[e] = __builtin_amdgcn_readfirstlane(qwords[16 + e]);
  __syncthreads();                       // everyone has read it before the next unit's draw overwrites it
  }
#undef FM_TILE_LOOP
}

}  // namespace fm

using namespace fm;

template <int D, bool RAGGED, bool GEN>
static hipError_t launch_dq_t(const FmBwdArgs& a, hipStream_t stream) {
  using C = DqCfg<D>;
  static bool allowed[FM_MAX_DEVICES] = {};
  if (hipError_t e = fm_allow_lds((const void*)dq_kernel<D, RAGGED, GEN>, C::LDS_BYTES, allowed); e != hipSuccess) return e;
  hipLaunchKernelGGL((dq_kernel<D, RAGGED, GEN>), dim3(fm_launch_grid(a.slots_dq)), dim3(256), C::LDS_BYTES, stream, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_dq_d(const FmBwdArgs& a, hipStream_t stream) {
  const bool ragged = a.Np != a.N;
  if (a.general) return ragged ? launch_dq_t<D, true, true>(a, stream) : launch_dq_t<D, false, true>(a, stream);
  return ragged ? launch_dq_t<D, true, false>(a, stream) : launch_dq_t<D, false, false>(a, stream);
}

hipError_t fm_launch_bwd_dq(const FmBwdArgs& a, hipStream_t stream) {
  return a.d == 128 ? launch_dq_d<128>(a, stream) : launch_dq_d<64>(a, stream);
}

template <int D, bool RAGGED, bool GEN>
static hipError_t launch_dkdv_t(const FmBwdArgs& a, hipStream_t stream) {
  using C = DkdvCfg<D>;
  static bool allowed[FM_MAX_DEVICES] = {};
  if (hipError_t e = fm_allow_lds((const void*)dkdv_kernel<D, RAGGED, GEN>, C::LDS_BYTES, allowed); e != hipSuccess) return e;
  // persistent: as many workgroups as the chip holds at once (one per CU at d = 128, two at d = 64)
  const int grid = fm_persistent_grid(a.slots_dkdv, D == 64 ? 2 : 1);
  hipLaunchKernelGGL((dkdv_kernel<D, RAGGED, GEN>), dim3(grid), dim3(256), C::LDS_BYTES, stream, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_dkdv_d(const FmBwdArgs& a, hipStream_t stream) {
  const bool ragged = a.Np != a.N;
  if (a.general) return ragged ? launch_dkdv_t<D, true, true>(a, stream) : launch_dkdv_t<D, false, true>(a, stream);
  return ragged ? launch_dkdv_t<D, true, false>(a, stream) : launch_dkdv_t<D, false, false>(a, stream);
}

hipError_t fm_launch_bwd_dkdv(const FmBwdArgs& a, hipStream_t stream) {
  return a.d == 128 ? launch_dkdv_d<128>(a, stream) : launch_dkdv_d<64>(a, stream);
}
