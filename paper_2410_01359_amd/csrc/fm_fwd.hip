// Forward tile loop (Algorithm 1) for gfx950.
//
// One workgroup (4 waves) per (batch, head, block of BR query rows).  Each wave
// owns 32*QB query rows for the whole kernel and walks the key blocks that the
// min/max tables do not prove fully masked.  Scores are computed transposed,
// S^T = K Q^T, so that after the MFMA every lane holds ONE query column: row
// max / row sum are per-lane loops plus one exchange with the lane 32 away, the
// running rescale of O is a per-lane scalar, and P^T is already in the
// B-operand layout of the second product O^T += V^T P^T.  K tiles are read
// from LDS as A operands (128-bit reads), V tiles through the LDS transpose
// read.  Q stays in registers.
#include "fm_common.h"
#include "fm_kernels.h"

namespace fm {

template <int D, int QB>
struct FwdCfg {
  static constexpr int KT = FM_FWD_BC;          // keys per tile
  static constexpr int BR = 128 * QB;           // query rows per workgroup
  using L = TileLayout<D>;                      // swizzled / padded LDS rows
  static constexpr int K_BYTES = KT * L::RS;
  static constexpr int V_BYTES = KT * L::RS;
  static constexpr int BND_BYTES = 4 * KT * 4;  // LTS, LTE, UTS, UTE slices of one tile
  static constexpr int STAGE = K_BYTES + V_BYTES + BND_BYTES;
  static constexpr int LIST_CAP = 1024;         // key blocks classified per pass
  static constexpr int LIST_OFF = 0;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int STAGE_OFF = CNT_OFF + 64;
  static constexpr int LDS_BYTES = STAGE_OFF + 2 * STAGE;
};

template <int D, int QB>
__global__ __launch_bounds__(256, QB == 1 ? 2 : 1) void fwd_kernel(FmFwdArgs a) {
  using C = FwdCfg<D, QB>;
  constexpr int KT = C::KT, NKB = KT / 32, NDB = D / 32, NKK = D / 16;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int unit = a.order[blockIdx.x];
  if (unit < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int N = a.N, H = a.H;
  const int t_r = N / C::BR, t_c = N / KT;
  const int bh = unit / t_r, i_blk = unit - bh * t_r, b = bh / H;
  const int q0 = i_blk * C::BR;
  const int qw0 = q0 + wave * 32 * QB;

  const __bf16* qp = (const __bf16*)a.q + (size_t)bh * N * D;
  const __bf16* kp = (const __bf16*)a.k + (size_t)bh * N * D;
  const __bf16* vp = (const __bf16*)a.v + (size_t)bh * N * D;
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
  CopyLanes<D> copy_lanes;
  copy_lanes.init(lane);

  // Q fragments (B operand of S^T = K Q^T): lane holds Q[row c][16 kk + 8 g ..+7].
  bf16x8 qreg[QB][NKK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
      qreg[qb][kk] = *(const bf16x8*)(qp + (size_t)(qw0 + qb * 32 + c) * D + kk * 16 + 8 * g);
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) settle(qreg[qb][kk]);

  f32x16 oacc[NDB][QB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
  }

  int* list = (int*)(smem + C::LIST_OFF);
  int* wave_cnt = (int*)(smem + C::CNT_OFF);
  const float sc = a.scale * kLog2e;  // > 0 (checked on the host)
  // Scores stay raw; exp2(s*sc - m) is one fma + one exp.  The reference
  // maximum m only moves when a tile's maximum exceeds it by more than
  // kRescaleGap (log2 units), so the rescale of O and l is rare; any m is a
  // valid softmax reference, P just grows up to 2^kRescaleGap.
  constexpr float kRescaleGap = 8.f;

  // lane-dependent LDS offsets inside a tile (row block 0)
  const int i16 = lane & 15, half = (lane >> 4) & 1;
  int a_off[NKK];       // operand rows: row c, bytes (16 kk + 8 g) * 2
  int t_off[2][NDB];    // transpose reads: row 4 g + i16/4 (+8), bytes (32 db + 16 half + 4 (i16 & 3)) * 2
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) a_off[kk] = C::L::off(c, (kk * 16 + 8 * g) * 2);
#pragma unroll
  for (int hi = 0; hi < 2; ++hi)
#pragma unroll
    for (int db = 0; db < NDB; ++db)
      t_off[hi][db] = C::L::off(4 * g + (i16 >> 2) + 8 * hi, (db * 32 + 16 * half + 4 * (i16 & 3)) * 2);

  // Asynchronous copy of one live tile (K, V and, if partially masked, its bound slices)
  // into stage buffer BUF; awaited by async_wait<0>() in front of the next barrier.
#define FM_LOAD_TILE(ENTRY, BUF)                                                               \
  {                                                                                            \
    const int j_ = entry_block(ENTRY, chunk);                                                  \
    char* st_ = smem + C::STAGE_OFF + (BUF) * C::STAGE;                                        \
    tile_load_async<D>(kp + (size_t)j_ * KT * D, copy_lanes, st_, wave);                     \
    tile_load_async<D>(vp + (size_t)j_ * KT * D, copy_lanes, st_ + C::K_BYTES, wave);        \
    if (entry_tile_class(ENTRY) == T_PARTIAL && wave == 0)                                     \
      async_copy16(my_bvec + j_ * KT, lds_address(st_ + C::K_BYTES + C::V_BYTES));             \
  }

  for (int chunk = 0; chunk < t_c; chunk += C::LIST_CAP) {
    const int n_live = build_live_key_blocks(table, t_c, chunk, min(chunk + C::LIST_CAP, t_c), q0, min(q0 + C::BR, N),
                                             C::BR / 4, list, wave_cnt);
    if (n_live == 0) continue;
    const int first_entry = __builtin_amdgcn_readfirstlane(list[0]);
    FM_LOAD_TILE(first_entry, 0);
    async_wait<0>();
    barrier_nofence();

    for (int t = 0; t < n_live; ++t) {
      const int entry = __builtin_amdgcn_readfirstlane(list[t]);
      const int next_entry = __builtin_amdgcn_readfirstlane((t + 1 < n_live) ? list[t + 1] : 0);
      if (t + 1 < n_live) FM_LOAD_TILE(next_entry, (t + 1) & 1);

      const char* st = smem + C::STAGE_OFF + (t & 1) * C::STAGE;
      const char* ks = st;
      const char* vs = st + C::K_BYTES;
      const int* bnd = (const int*)(st + C::K_BYTES + C::V_BYTES);

      const int wcls = entry_wave_class(entry, wave);   // Equation 4 on this wave's own rows
      if (wcls != T_FULLY) {
        f32x16 sacc[NKB][QB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][qb][r] = 0.f;
        // S^T = K Q^T.  The K operand of step n (chain kb = n % NKB, slice kk = n / NKB: the
        // accumulation chains alternate) is fetched RS steps ahead into a small register ring,
        // so an MFMA never waits for a read issued just before it.
        constexpr int NS = NKB * NKK, RS = 6;
        bf16x8 kring[RS];
        auto k_operand = [&](int n) __attribute__((always_inline)) {
          return *(const bf16x8*)(ks + (n % NKB) * 32 * C::L::RS + a_off[n / NKB]);
        };
#pragma unroll
        for (int n = 0; n < RS; ++n) kring[n] = k_operand(n);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NS; ++n) {
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            sacc[n % NKB][qb] = mfma32(kring[n % RS], qreg[qb][n / NKB], sacc[n % NKB][qb]);
          if (n + RS < NS) kring[n % RS] = k_operand(n + RS);
          __builtin_amdgcn_sched_barrier(0);
        }
        // The V operands of the second product do not depend on the scores: start fetching them
        // now, so they arrive while the softmax arithmetic runs.
        constexpr int NP = NKB * 2 * NDB, RP = 4;
        bf16x8 vring[RP];
        auto v_operand = [&](int n) __attribute__((always_inline)) {
          const char* vrow = vs + ((n / NDB) * 16) * C::L::RS;   // group n / NDB = (kb, h): 16 keys each
          return cat4(lds_read_tr16(vrow + t_off[0][n % NDB]), lds_read_tr16(vrow + t_off[1][n % NDB]));
        };
#pragma unroll
        for (int n = 0; n < RP; ++n) vring[n] = v_operand(n);
        __builtin_amdgcn_sched_barrier(0);
        if (wcls & T_PARTIAL) {
          // Both pairs are applied whenever the tile is partial: a pair whose
          // NEED bit is clear masks no element of this tile, so this is exact,
          // and branch-free code here keeps the register allocation sane.
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
              const int kx = kb * 32 + 8 * rq + 4 * g;
              const i32x4 bl = *(const i32x4*)(bnd + 0 * KT + kx);
              const i32x4 be = *(const i32x4*)(bnd + 1 * KT + kx);
              const i32x4 bu = *(const i32x4*)(bnd + 2 * KT + kx);
              const i32x4 bv = *(const i32x4*)(bnd + 3 * KT + kx);
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) {
                const int row = qw0 + qb * 32 + c;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const bool masked = ((row >= bl[e]) & (row < be[e])) | ((row >= bu[e]) & (row < bv[e]));
                  if (masked) sacc[kb][qb][rq * 4 + e] = -INFINITY;
                }
              }
              __builtin_amdgcn_sched_barrier(0);  // keep the bound reads of later steps from piling up in registers
            }
        }

        // online softmax (per lane = per query column)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          float mx = -INFINITY;
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][qb][r]);
          mx = fmaxf(mx, partner32(mx)) * sc;
          const bool grow = mx > m_run[qb] + kRescaleGap;   // also true on the first finite maximum
          if (__any(grow)) {
            const float m_new = grow ? mx : m_run[qb];
            const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_run[qb] - m_new);
            m_run[qb] = m_new;
            l_run[qb] *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
              for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= alpha;
          }
          const float neg_m = (m_run[qb] == -INFINITY) ? 0.f : -m_run[qb];
          float rs = 0.f;
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float p = fast_exp2(__builtin_fmaf(sacc[kb][qb][r], sc, neg_m));
              sacc[kb][qb][r] = p;
              rs += p;
            }
          l_run[qb] += rs;
        }

        __builtin_amdgcn_sched_barrier(0);
        // O^T += V^T P^T, step n = (16-key group n / NDB, d block n % NDB)
#pragma unroll
        for (int n = 0; n < NP; ++n) {
          const int grp = n / NDB, kb = grp / 2, h = grp % 2, db = n % NDB;
          bf16x8 pb[QB];
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int e = 0; e < 8; ++e) pb[qb][e] = (__bf16)sacc[kb][qb][8 * h + e];
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) oacc[db][qb] = mfma32(vring[n % RP], pb[qb], oacc[db][qb]);
          if (n + RP < NP) vring[n % RP] = v_operand(n + RP);
          __builtin_amdgcn_sched_barrier(0);
        }
      }

      async_wait<0>();   // the next tile has landed ...
      barrier_nofence(); // ... for every wave, and every wave is done reading this one
    }
    __syncthreads();     // the list is rebuilt by the next pass
  }

  // epilogue: O / l, lse = m + log(l)   (m, l in the log2 domain)
  __bf16* op = (__bf16*)a.out + (size_t)bh * N * D;
  float* lp = a.lse + (size_t)bh * N;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float lt = l_run[qb] + partner32(l_run[qb]);
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const int row = qw0 + qb * 32 + c;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][qb][rq * 4 + e] * inv);
        *(bf16x4*)(op + (size_t)row * D + db * 32 + 8 * rq + 4 * g) = o4;
      }
    if (g == 0) lp[row] = lt > 0.f ? (m_run[qb] + fast_log2(lt)) * kLn2 : -INFINITY;
  }
}

#undef FM_LOAD_TILE

}  // namespace fm

using namespace fm;

template <int D, int QB>
static hipError_t launch_fwd_t(const FmFwdArgs& a, hipStream_t stream) {
  using C = FwdCfg<D, QB>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)fwd_kernel<D, QB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_kernel<D, QB>), dim3(a.slots), dim3(256), C::LDS_BYTES, stream, a);
  return hipGetLastError();
}

hipError_t fm_launch_fwd(const FmFwdArgs& a, hipStream_t stream) {
  static_assert(FM_FWD_BR == 128, "forward row block");
  if (a.d == 128) return launch_fwd_t<128, 1>(a, stream);
  return launch_fwd_t<64, 1>(a, stream);
}
