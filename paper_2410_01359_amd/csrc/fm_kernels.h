// Host-side launchers of the gfx950 FlashMask kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Number of launch slots for `units` work units: 8 interleaved groups.
inline int fm_order_slots(int units) { return ((units + 7) / 8) * 8; }

struct FmShape {
  int B, H, N, d;
};

// Tile shapes (rows x key columns) each pass classifies at.
constexpr int FM_FWD_BR = 128, FM_FWD_BC = 64;
constexpr int FM_DQ_BR = 128, FM_DQ_BC = 64;
constexpr int FM_DKDV_BR = 64, FM_DKDV_BC = 128;

hipError_t fm_launch_preprocess(const int* lts, const int* lte, const int* uts, const int* ute, int B, int N,
                                int block_c, int* minmax, hipStream_t stream);
// Padded copies of the four bound vectors: [4][B][Np], columns >= N masked for every row.
hipError_t fm_launch_pad_bounds(const int* lts, const int* lte, const int* uts, const int* ute, int B, int N, int Np,
                                int* padded, hipStream_t stream);
hipError_t fm_launch_classify(const int* minmax, int B, int N, int block_r, int block_c, uint8_t* cls,
                              hipStream_t stream);
// work: int[B * T_r] (resp. B * T_c); range: int[2 * B * T] = first live block and one past the
// last live block of every unit (0, 0 if none); order: int[fm_order_slots(B*H*T)].
hipError_t fm_launch_row_order(const int* minmax, int B, int H, int N, int block_r, int block_c, int* work,
                               int* range, int* order, hipStream_t stream);
hipError_t fm_launch_col_order(const int* minmax, int B, int H, int N, int block_r, int block_c, int* work,
                               int* range, int* order, hipStream_t stream);

// N is the true sequence length (stride of the tensors), Np = N rounded up to a multiple of 128: the
// length the tile loops and the tables work at.  When Np > N the bound vectors are the library's
// padded copies [B][Np] whose extra columns are masked for every row.
struct FmFwdArgs {
  const void *q, *k, *v;
  const int *lts, *lte, *uts, *ute;   // [B][Np]
  const int* minmax;  // [B][8][T_c] at FM_FWD_BC
  const int* order;   // launch slots -> unit (b*H + h)*T_r + i, or -1
  const int* range;   // [B][T_r][2]: key blocks [first, last) outside of which the row block is fully masked
  void* out;
  float* lse;
  float scale;
  int B, H, N, Np, d;
  int slots;
};
hipError_t fm_launch_fwd(const FmFwdArgs& a, hipStream_t stream);

struct FmBwdArgs {
  const void *q, *k, *v, *out, *dout;
  const float* lse;
  const int *lts, *lte, *uts, *ute;
  const int* minmax_dq;    // [B][8][T_c] at FM_DQ_BC
  const int* order_dq;
  const int* range_dq;     // [B][T_r][2] key-block range of each row block
  const int* minmax_dkdv;  // [B][8][T_c] at FM_DKDV_BC
  const int* order_dkdv;
  const int* range_dkdv;   // [B][T_c][2] row-block range of each key block
  float* dvec;             // -D = -rowsum(dO o O), [B,H,Np] (stored negated; 0 in the padding)
  float* lse2;             // lse * log2(e), +inf where lse = -inf and in the padding, [B,H,Np]
  void *dq, *dk, *dv;
  float scale;
  int B, H, N, Np, d;
  int slots_dq, slots_dkdv;
};
hipError_t fm_launch_dvec(const FmBwdArgs& a, hipStream_t stream);
hipError_t fm_launch_bwd_dq(const FmBwdArgs& a, hipStream_t stream);
hipError_t fm_launch_bwd_dkdv(const FmBwdArgs& a, hipStream_t stream);
