// Backward pass (Algorithm 2) for gfx950, as three kernels:
//
//   dvec_kernel   D_i = sum_c dO_ic O_ic                       (Algorithm 2, D pre-pass)
//   dkdv_kernel   column-parallel loop over key blocks j: recompute S and
//                 P = exp(S - L), dV_j += P^T dO_i, dP = dO_i V_j^T,
//                 dS = P o (dP - D_i), dK_j += dS^T Q_i           (Algorithm 2 main loop)
//   dq_kernel     row-parallel loop over query blocks i: the same S, P, dP, dS
//                 and dQ_i += dS K_j, accumulated in registers in a fixed order.
//
// Algorithm 2 adds every tile's dS K_j into dQ_i in HBM from the column-parallel
// loop.  On this chip fp32 atomic adds sustain about 1.4 TB/s, which would cap
// the backward far below the matrix-core rate, so dQ gets its own row-parallel
// pass instead (two extra products per tile, no atomics, bit-reproducible).
#include "fm_common.h"
#include "fm_kernels.h"

namespace fm {

// ---------------------------------------------------------------------------
// D pre-pass.  One row per 16 (d = 128) or 8 (d = 64) lanes, 16 bytes per lane.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void dvec_kernel(const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                                                   float* __restrict__ dvec, long long rows) {
  constexpr int LPR = D / 8;  // lanes per row
  const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = gid / LPR;
  const int part = (int)(gid % LPR);
  float acc = 0.f;
  if (row < rows) {
    const bf16x8 o = *(const bf16x8*)(out + row * D + part * 8);
    const bf16x8 g = *(const bf16x8*)(dout + row * D + part * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)o[e] * (float)g[e];
  }
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (row < rows && part == 0) dvec[row] = acc;
}

// ---------------------------------------------------------------------------
// dQ: row-parallel, same transposed-score layout as the forward kernel.
// ---------------------------------------------------------------------------
template <int D>
struct DqCfg {
  static constexpr int KT = FM_DQ_BC;
  static constexpr int BR = FM_DQ_BR;
  static constexpr int RS = D * 2 + 16;  // K and V row stride in LDS (bytes)
  static constexpr int K_BYTES = KT * RS;
  static constexpr int V_BYTES = KT * RS;
  static constexpr int BND_BYTES = 4 * KT * 4;
  static constexpr int STAGE = K_BYTES + V_BYTES + BND_BYTES;
  static constexpr int LIST_CAP = 1024;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int STAGE_OFF = CNT_OFF + 64;
  static constexpr int LDS_BYTES = STAGE_OFF + 2 * STAGE;
  static constexpr int NCH = KT * D / 8 / 256;
};

template <int D>
__global__ __launch_bounds__(256, 2) void dq_kernel(FmBwdArgs a) {
  using C = DqCfg<D>;
  constexpr int KT = C::KT, NKB = KT / 32, NDB = D / 32, NKK = D / 16;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int unit = a.order_dq[blockIdx.x];
  if (unit < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int N = a.N, H = a.H;
  const int t_r = N / C::BR, t_c = N / KT;
  const int bh = unit / t_r, i_blk = unit - bh * t_r, b = bh / H;
  const int q0 = i_blk * C::BR;
  const int qw0 = q0 + wave * 32;
  const int row = qw0 + c;  // this lane's query row

  const __bf16* qp = (const __bf16*)a.q + (size_t)bh * N * D;
  const __bf16* kp = (const __bf16*)a.k + (size_t)bh * N * D;
  const __bf16* vp = (const __bf16*)a.v + (size_t)bh * N * D;
  const __bf16* dop = (const __bf16*)a.dout + (size_t)bh * N * D;
  const int* table = a.minmax_dq + (size_t)b * 8 * t_c;
  const int *bvec0 = a.lts + (size_t)b * N, *bvec1 = a.lte + (size_t)b * N, *bvec2 = a.uts + (size_t)b * N,
            *bvec3 = a.ute + (size_t)b * N;

  bf16x8 qreg[NKK], doreg[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    qreg[kk] = *(const bf16x8*)(qp + (size_t)row * D + kk * 16 + 8 * g);
    doreg[kk] = *(const bf16x8*)(dop + (size_t)row * D + kk * 16 + 8 * g);
  }
  // lse in the log2 domain; a row with no visible key (lse = -inf) must give P = 0
  const float lse_raw = a.lse[(size_t)bh * N + row];
  const float lse2 = (lse_raw == -INFINITY) ? INFINITY : lse_raw * kLog2e;
  const float dsum = a.dvec[(size_t)bh * N + row];

  f32x16 dqacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[db][r] = 0.f;

  int* list = (int*)smem;
  int* wave_cnt = (int*)(smem + C::CNT_OFF);
  const float sc = a.scale * kLog2e;

  u32x4 kst[C::NCH], vst[C::NCH], bst[4];
#define FM_ISSUE_LOADS(ENTRY)                                               \
  {                                                                         \
    const int j_ = (ENTRY) & 0xFFFFFF;                                      \
    _Pragma("unroll") for (int s = 0; s < C::NCH; ++s) {                    \
      const int ch = tid + 256 * s;                                         \
      const int rw = ch / (D / 8), col = ch % (D / 8);                      \
      const size_t off = (size_t)(j_ * KT + rw) * D + col * 8;              \
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
      const int rw = ch / (D / 8), col = ch % (D / 8);                      \
      *(u32x4*)(st_ + rw * C::RS + col * 16) = kst[s];                      \
      *(u32x4*)(st_ + C::K_BYTES + rw * C::RS + col * 16) = vst[s];         \
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

      const int wcls = classify_tile(qw0, qw0 + 32, load_minmax(table, t_c, j));
      if (wcls != T_FULLY) {
        const int i16 = lane & 15, half = (lane >> 4) & 1;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
          f32x16 sacc, dpacc;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            sacc[r] = 0.f;
            dpacc[r] = 0.f;
          }
          // S^T = K Q^T and dP^T = V dO^T for 32 keys x 32 queries
#pragma unroll
          for (int kk = 0; kk < NKK; ++kk) {
            const bf16x8 ka = *(const bf16x8*)(ks + (kb * 32 + c) * C::RS + (kk * 16 + 8 * g) * 2);
            sacc = mfma32(ka, qreg[kk], sacc);
            const bf16x8 va = *(const bf16x8*)(vs + (kb * 32 + c) * C::RS + (kk * 16 + 8 * g) * 2);
            dpacc = mfma32(va, doreg[kk], dpacc);
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[r] *= sc;
          if (wcls & T_PARTIAL) {
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
          }
          // P = exp(S - L), dS = P o (dP - D)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = fast_exp2(sacc[r] - lse2);
            sacc[r] = p * (dpacc[r] - dsum);
          }
          __builtin_amdgcn_sched_barrier(0);
          // dQ^T += K^T dS^T
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            bf16x8 dsb;
#pragma unroll
            for (int e = 0; e < 8; ++e) dsb[e] = (__bf16)sacc[8 * h + e];
            const int row0 = kb * 32 + 16 * h + 4 * g + (i16 >> 2);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
              const int col = db * 32 + 16 * half + 4 * (i16 & 3);
              const bf16x4 lo = lds_read_tr16(ks + row0 * C::RS + col * 2);
              const bf16x4 hi = lds_read_tr16(ks + (row0 + 8) * C::RS + col * 2);
              dqacc[db] = mfma32(cat4(lo, hi), dsb, dqacc[db]);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }

      if (t + 1 < n_live) FM_STORE_STAGE(next_entry, (t + 1) & 1);
      __syncthreads();
    }
  }
#undef FM_ISSUE_LOADS
#undef FM_STORE_STAGE

  __bf16* dqp = (__bf16*)a.dq + (size_t)bh * N * D;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(dqacc[db][rq * 4 + e] * a.scale);
      *(bf16x4*)(dqp + (size_t)row * D + db * 32 + 8 * rq + 4 * g) = o4;
    }
}

// ---------------------------------------------------------------------------
// dK, dV: column-parallel.  A workgroup owns FM_DKDV_BC = 128 keys (32 per
// wave, K and V fragments resident in registers) and walks the row blocks of
// FM_DKDV_BR = 64 queries that are not fully masked for its keys.  Scores are
// NOT transposed here (S = Q K^T): every lane then holds one KEY column, so the
// four bounds of that key sit in four registers for the whole kernel and P^T,
// dS^T are already A operands of dV += P^T dO and dK += dS^T Q.
// ---------------------------------------------------------------------------
template <int D>
struct DkdvCfg {
  static constexpr int QT = FM_DKDV_BR;    // query rows per step
  static constexpr int BC = FM_DKDV_BC;    // keys per workgroup
  static constexpr int RS = D * 2 + 16;    // Q and dO row stride in LDS (bytes)
  static constexpr int Q_BYTES = QT * RS;
  static constexpr int DO_BYTES = QT * RS;
  static constexpr int VEC_BYTES = 2 * QT * 4;  // lse (log2 domain) and D of the rows
  static constexpr int STAGE = Q_BYTES + DO_BYTES + VEC_BYTES;
  static constexpr int LIST_CAP = 2048;
  static constexpr int CNT_OFF = LIST_CAP * 4;
  static constexpr int STAGE_OFF = CNT_OFF + 64;
  static constexpr int LDS_BYTES = STAGE_OFF + 2 * STAGE;
  static constexpr int NCH = QT * D / 8 / 256;
};

template <int D>
__global__ __launch_bounds__(256, 1) void dkdv_kernel(FmBwdArgs a) {
  using C = DkdvCfg<D>;
  constexpr int QT = C::QT, NQB = QT / 32, NDB = D / 32, NKK = D / 16;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int unit = a.order_dkdv[blockIdx.x];
  if (unit < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int N = a.N, H = a.H;
  const int t_r = N / QT, t_c = N / C::BC;
  const int bh = unit / t_c, j_blk = unit - bh * t_c, b = bh / H;
  const int k0 = j_blk * C::BC;
  const int kw0 = k0 + wave * 32;
  const int key = kw0 + c;  // this lane's key column

  const __bf16* qp = (const __bf16*)a.q + (size_t)bh * N * D;
  const __bf16* kp = (const __bf16*)a.k + (size_t)bh * N * D;
  const __bf16* vp = (const __bf16*)a.v + (size_t)bh * N * D;
  const __bf16* dop = (const __bf16*)a.dout + (size_t)bh * N * D;
  const float* lsep = a.lse + (size_t)bh * N;
  const float* dvp = a.dvec + (size_t)bh * N;

  // K and V fragments of this wave's 32 keys (B operands of S = Q K^T, dP = dO V^T)
  bf16x8 kreg[NKK], vreg[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    kreg[kk] = *(const bf16x8*)(kp + (size_t)key * D + kk * 16 + 8 * g);
    vreg[kk] = *(const bf16x8*)(vp + (size_t)key * D + kk * 16 + 8 * g);
  }
  // the four bounds of this lane's key stay in registers (Algorithm 2 loads them once per key block)
  const int b_lts = a.lts[(size_t)b * N + key], b_lte = a.lte[(size_t)b * N + key];
  const int b_uts = a.uts[(size_t)b * N + key], b_ute = a.ute[(size_t)b * N + key];
  // min/max over this wave's 32 keys, for the wave-level tile class
  MinMax8 wmm;
  {
    int mx[4] = {b_lts, b_lte, b_uts, b_ute}, mn[4] = {b_lts, b_lte, b_uts, b_ute};
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        mx[v] = max(mx[v], __shfl_xor(mx[v], off, 64));
        mn[v] = min(mn[v], __shfl_xor(mn[v], off, 64));
      }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      wmm.v[2 * v] = __builtin_amdgcn_readfirstlane(mx[v]);
      wmm.v[2 * v + 1] = __builtin_amdgcn_readfirstlane(mn[v]);
    }
  }
  const MinMax8 gmm = load_minmax(a.minmax_dkdv + (size_t)b * 8 * t_c, t_c, j_blk);

  f32x16 dkacc[NDB], dvacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dkacc[db][r] = 0.f;
      dvacc[db][r] = 0.f;
    }

  int* list = (int*)smem;
  int* wave_cnt = (int*)(smem + C::CNT_OFF);
  const float sc = a.scale * kLog2e;

  u32x4 qst[C::NCH], dost[C::NCH];
  float vecst = 0.f;
#define FM_ISSUE_LOADS(ENTRY)                                               \
  {                                                                         \
    const int i_ = (ENTRY) & 0xFFFFFF;                                      \
    _Pragma("unroll") for (int s = 0; s < C::NCH; ++s) {                    \
      const int ch = tid + 256 * s;                                         \
      const int rw = ch / (D / 8), col = ch % (D / 8);                      \
      const size_t off = (size_t)(i_ * QT + rw) * D + col * 8;              \
      qst[s] = ldg16(qp + off);                                             \
      dost[s] = ldg16(dop + off);                                           \
    }                                                                       \
    if (tid < QT) {                                                         \
      const float x = lsep[i_ * QT + tid];                                  \
      vecst = (x == -INFINITY) ? INFINITY : x * kLog2e;                     \
    } else if (tid < 2 * QT) {                                              \
      vecst = dvp[i_ * QT + tid - QT];                                      \
    }                                                                       \
  }
#define FM_STORE_STAGE(BUF)                                                 \
  {                                                                         \
    char* st_ = smem + C::STAGE_OFF + (BUF) * C::STAGE;                     \
    _Pragma("unroll") for (int s = 0; s < C::NCH; ++s) {                    \
      const int ch = tid + 256 * s;                                         \
      const int rw = ch / (D / 8), col = ch % (D / 8);                      \
      *(u32x4*)(st_ + rw * C::RS + col * 16) = qst[s];                      \
      *(u32x4*)(st_ + C::Q_BYTES + rw * C::RS + col * 16) = dost[s];        \
    }                                                                       \
    if (tid < 2 * QT) *(float*)(st_ + C::Q_BYTES + C::DO_BYTES + tid * 4) = vecst; \
  }

  for (int chunk = 0; chunk < t_r; chunk += C::LIST_CAP) {
    const int n_live = build_live_row_blocks(gmm, N, QT, chunk, min(chunk + C::LIST_CAP, t_r), list, wave_cnt);
    if (n_live == 0) continue;
    const int first_entry = __builtin_amdgcn_readfirstlane(list[0]);
    FM_ISSUE_LOADS(first_entry);
    FM_STORE_STAGE(0);
    __syncthreads();

    for (int t = 0; t < n_live; ++t) {
      const int entry = __builtin_amdgcn_readfirstlane(list[t]);
      const int i_blk = entry & 0xFFFFFF;
      const int next_entry = __builtin_amdgcn_readfirstlane((t + 1 < n_live) ? list[t + 1] : 0);
      if (t + 1 < n_live) FM_ISSUE_LOADS(next_entry);

      const char* st = smem + C::STAGE_OFF + (t & 1) * C::STAGE;
      const char* qs = st;
      const char* dos = st + C::Q_BYTES;
      const float* lse_s = (const float*)(st + C::Q_BYTES + C::DO_BYTES);
      const float* dv_s = lse_s + QT;
      const int r0 = i_blk * QT;

      const int wcls = classify_tile(r0, min(r0 + QT, N), wmm);
      if (wcls != T_FULLY) {
        const int i16 = lane & 15, half = (lane >> 4) & 1;
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          f32x16 sacc, dpacc;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            sacc[r] = 0.f;
            dpacc[r] = 0.f;
          }
          // S = Q K^T, dP = dO V^T for 32 queries x 32 keys
#pragma unroll
          for (int kk = 0; kk < NKK; ++kk) {
            const bf16x8 qa = *(const bf16x8*)(qs + (qb * 32 + c) * C::RS + (kk * 16 + 8 * g) * 2);
            sacc = mfma32(qa, kreg[kk], sacc);
            const bf16x8 da = *(const bf16x8*)(dos + (qb * 32 + c) * C::RS + (kk * 16 + 8 * g) * 2);
            dpacc = mfma32(da, vreg[kk], dpacc);
          }
          // register r holds query row qb*32 + 8*(r/4) + 4*g + r%4 of this tile
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const int rl = qb * 32 + 8 * rq + 4 * g;
            const f32x4 l4 = *(const f32x4*)(lse_s + rl);
            const f32x4 d4 = *(const f32x4*)(dv_s + rl);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int r = rq * 4 + e;
              const int qrow = r0 + rl + e;
              float s = sacc[r] * sc;
              if (wcls & T_PARTIAL) {
                const bool masked = ((qrow >= b_lts) & (qrow < b_lte)) | ((qrow >= b_uts) & (qrow < b_ute));
                if (masked) s = -INFINITY;
              }
              const float p = fast_exp2(s - l4[e]);
              sacc[r] = p;
              dpacc[r] = p * (dpacc[r] - d4[e]);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
          // dV += P^T dO, dK += dS^T Q
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            bf16x8 pa, dsa;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              pa[e] = (__bf16)sacc[8 * h + e];
              dsa[e] = (__bf16)dpacc[8 * h + e];
            }
            const int row0 = qb * 32 + 16 * h + 4 * g + (i16 >> 2);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
              const int col = db * 32 + 16 * half + 4 * (i16 & 3);
              const bf16x4 dlo = lds_read_tr16(dos + row0 * C::RS + col * 2);
              const bf16x4 dhi = lds_read_tr16(dos + (row0 + 8) * C::RS + col * 2);
              dvacc[db] = mfma32(pa, cat4(dlo, dhi), dvacc[db]);
              const bf16x4 qlo = lds_read_tr16(qs + row0 * C::RS + col * 2);
              const bf16x4 qhi = lds_read_tr16(qs + (row0 + 8) * C::RS + col * 2);
              dkacc[db] = mfma32(dsa, cat4(qlo, qhi), dkacc[db]);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }

      if (t + 1 < n_live) FM_STORE_STAGE((t + 1) & 1);
      __syncthreads();
    }
  }
#undef FM_ISSUE_LOADS
#undef FM_STORE_STAGE

  // accumulators: register r of block db holds [key kw0 + 8*(r/4) + 4*g + r%4][d = db*32 + c]
  __bf16* dkp = (__bf16*)a.dk + (size_t)bh * N * D;
  __bf16* dvp_out = (__bf16*)a.dv + (size_t)bh * N * D;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int krow = kw0 + 8 * (r >> 2) + 4 * g + (r & 3);
      dkp[(size_t)krow * D + db * 32 + c] = (__bf16)(dkacc[db][r] * a.scale);
      dvp_out[(size_t)krow * D + db * 32 + c] = (__bf16)dvacc[db][r];
    }
}

}  // namespace fm

using namespace fm;

hipError_t fm_launch_dvec(const FmBwdArgs& a, hipStream_t stream) {
  const long long rows = (long long)a.B * a.H * a.N;
  const long long threads = rows * (a.d / 8);
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  if (a.d == 128)
    hipLaunchKernelGGL(dvec_kernel<128>, dim3(blocks), dim3(256), 0, stream, (const __bf16*)a.out,
                       (const __bf16*)a.dout, a.dvec, rows);
  else
    hipLaunchKernelGGL(dvec_kernel<64>, dim3(blocks), dim3(256), 0, stream, (const __bf16*)a.out,
                       (const __bf16*)a.dout, a.dvec, rows);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_dq_t(const FmBwdArgs& a, hipStream_t stream) {
  using C = DqCfg<D>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e =
        hipFuncSetAttribute((const void*)dq_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((dq_kernel<D>), dim3(a.slots_dq), dim3(256), C::LDS_BYTES, stream, a);
  return hipGetLastError();
}

hipError_t fm_launch_bwd_dq(const FmBwdArgs& a, hipStream_t stream) {
  return a.d == 128 ? launch_dq_t<128>(a, stream) : launch_dq_t<64>(a, stream);
}

template <int D>
static hipError_t launch_dkdv_t(const FmBwdArgs& a, hipStream_t stream) {
  using C = DkdvCfg<D>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e =
        hipFuncSetAttribute((const void*)dkdv_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((dkdv_kernel<D>), dim3(a.slots_dkdv), dim3(256), C::LDS_BYTES, stream, a);
  return hipGetLastError();
}

hipError_t fm_launch_bwd_dkdv(const FmBwdArgs& a, hipStream_t stream) {
  return a.d == 128 ? launch_dkdv_t<128>(a, stream) : launch_dkdv_t<64>(a, stream);
}
