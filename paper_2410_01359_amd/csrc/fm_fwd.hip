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
  static constexpr int RSK = D * 2 + 16;        // K row stride in LDS (bytes)
  static constexpr int RSV = D * 2 + 32;        // V row stride in LDS (bytes)
  static constexpr int K_BYTES = KT * RSK;
  static constexpr int V_BYTES = KT * RSV;
  static constexpr int BND_BYTES = 4 * KT * 4;  // LTS, LTE, UTS, UTE slices of one tile
  static constexpr int STAGE = K_BYTES + V_BYTES + BND_BYTES;
  static constexpr int LIST_CAP = 1024;         // key blocks classified per pass
  static constexpr int LIST_OFF = 0;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int STAGE_OFF = CNT_OFF + 64;
  static constexpr int LDS_BYTES = STAGE_OFF + 2 * STAGE;
  static constexpr int NCH = KT * D / 8 / 256;  // 16-byte chunks per thread per matrix
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
  const int *bvec0 = a.lts + (size_t)b * N, *bvec1 = a.lte + (size_t)b * N, *bvec2 = a.uts + (size_t)b * N,
            *bvec3 = a.ute + (size_t)b * N;

  // Q fragments (B operand of S^T = K Q^T): lane holds Q[row c][16 kk + 8 g ..+7].
  bf16x8 qreg[QB][NKK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
      qreg[qb][kk] = *(const bf16x8*)(qp + (size_t)(qw0 + qb * 32 + c) * D + kk * 16 + 8 * g);

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
  const float sc = a.scale * kLog2e;

  // Register staging of the next tile: global loads are issued before the
  // current tile's math and written to the other LDS buffer after it.
  u32x4 kst[C::NCH], vst[C::NCH], bst[4];
#define FM_ISSUE_LOADS(ENTRY)                                               \
  {                                                                         \
    const int j_ = (ENTRY) & 0xFFFFFF;                                      \
    _Pragma("unroll") for (int s = 0; s < C::NCH; ++s) {                    \
      const int ch = tid + 256 * s;                                         \
      const int row = ch / (D / 8), col = ch % (D / 8);                     \
      const size_t off = (size_t)(j_ * KT + row) * D + col * 8;             \
      kst[s] = ldg16(kp + off);                                             \
      vst[s] = ldg16(vp + off);                                             \
    }                                                                       \
    if ((((ENTRY) >> 24) & T_PARTIAL) && tid < KT / 4) {                    \
      bst[0] = ldg16(bvec0 + j_ * KT + tid * 4);                            \
      bst[1] = ldg16(bvec1 + j_ * KT + tid * 4);                            \
      bst[2] = ldg16(bvec2 + j_ * KT + tid * 4);                            \
      bst[3] = ldg16(bvec3 + j_ * KT + tid * 4);                            \
    }                                                                       \
  }
#define FM_STORE_STAGE(ENTRY, BUF)                                          \
  {                                                                         \
    char* st_ = smem + C::STAGE_OFF + (BUF) * C::STAGE;                     \
    _Pragma("unroll") for (int s = 0; s < C::NCH; ++s) {                    \
      const int ch = tid + 256 * s;                                         \
      const int row = ch / (D / 8), col = ch % (D / 8);                     \
      *(u32x4*)(st_ + row * C::RSK + col * 16) = kst[s];                    \
      *(u32x4*)(st_ + C::K_BYTES + row * C::RSV + col * 16) = vst[s];       \
    }                                                                       \
    if ((((ENTRY) >> 24) & T_PARTIAL) && tid < KT / 4) {                    \
      _Pragma("unroll") for (int v_ = 0; v_ < 4; ++v_)                      \
          *(u32x4*)(st_ + C::K_BYTES + C::V_BYTES + v_ * KT * 4 + tid * 16) = bst[v_]; \
    }                                                                       \
  }

  for (int chunk = 0; chunk < t_c; chunk += C::LIST_CAP) {
    const int n_live = build_live_key_blocks(table, t_c, chunk, min(chunk + C::LIST_CAP, t_c), q0, min(q0 + C::BR, N),
                                             list, wave_cnt);
    if (n_live == 0) continue;
    const int first_entry = __builtin_amdgcn_readfirstlane(list[0]);
    FM_ISSUE_LOADS(first_entry);
    FM_STORE_STAGE(first_entry, 0);
    __syncthreads();

    for (int t = 0; t < n_live; ++t) {
      const int entry = __builtin_amdgcn_readfirstlane(list[t]);
      const int j = entry & 0xFFFFFF;
      const int next_entry = __builtin_amdgcn_readfirstlane((t + 1 < n_live) ? list[t + 1] : 0);
      if (t + 1 < n_live) FM_ISSUE_LOADS(next_entry);

      const char* st = smem + C::STAGE_OFF + (t & 1) * C::STAGE;
      const char* ks = st;
      const char* vs = st + C::K_BYTES;
      const int* bnd = (const int*)(st + C::K_BYTES + C::V_BYTES);

      // this wave's own rows against the same table entry (Equation 4 on a sub-block)
      const int wcls = classify_tile(qw0, qw0 + 32 * QB, load_minmax(table, t_c, j));
      if (wcls != T_FULLY) {
        f32x16 sacc[NKB][QB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][qb][r] = 0.f;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int kk = 0; kk < NKK; ++kk) {
            const bf16x8 ka = *(const bf16x8*)(ks + (kb * 32 + c) * C::RSK + (kk * 16 + 8 * g) * 2);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) sacc[kb][qb] = mfma32(ka, qreg[qb][kk], sacc[kb][qb]);
          }
        __builtin_amdgcn_sched_barrier(0);
        // scaled scores in the log2 domain
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][qb][r] *= sc;

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
          mx = fmaxf(mx, partner32(mx));
          const float m_new = fmaxf(m_run[qb], mx);
          const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
          const float alpha = fast_exp2(m_run[qb] - m_use);
          m_run[qb] = m_new;
          float rs = 0.f;
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float p = fast_exp2(sacc[kb][qb][r] - m_use);
              sacc[kb][qb][r] = p;
              rs += p;
            }
          l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
          for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= alpha;
        }

        __builtin_amdgcn_sched_barrier(0);
        // O^T += V^T P^T
        const int i16 = lane & 15, half = (lane >> 4) & 1;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            bf16x8 pb[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
              for (int e = 0; e < 8; ++e) pb[qb][e] = (__bf16)sacc[kb][qb][8 * h + e];
            __builtin_amdgcn_sched_barrier(0);
            const int row0 = kb * 32 + 16 * h + 4 * g + (i16 >> 2);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
              const int col = db * 32 + 16 * half + 4 * (i16 & 3);
              const bf16x4 lo = lds_read_tr16(vs + row0 * C::RSV + col * 2);
              const bf16x4 hi = lds_read_tr16(vs + (row0 + 8) * C::RSV + col * 2);
              const bf16x8 va = cat4(lo, hi);
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) oacc[db][qb] = mfma32(va, pb[qb], oacc[db][qb]);
            }
          }
      }

      if (t + 1 < n_live) FM_STORE_STAGE(next_entry, (t + 1) & 1);
      __syncthreads();
    }
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

#undef FM_ISSUE_LOADS
#undef FM_STORE_STAGE

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
