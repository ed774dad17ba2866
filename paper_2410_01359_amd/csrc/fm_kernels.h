// Host-side launchers of the gfx950 FlashMask kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// The tile loops draw their work units from FM_QUEUES interleaved queues (one per XCD).
constexpr int FM_QUEUES = 8;
// Number of queue slots for `units` work units.
// Slices (batch row, head) of a queue that are ranked together, longest first; a queue works its
// groups off one after the other.
constexpr int FM_QUEUE_CHUNK = 2;
// Slots of a pass's queues: FM_QUEUES x the longest queue.  Slices that do not fill a round of
// 8 queues are shared between 2, 4 or 8 queues block by block, which can make a queue up to 3 units
// longer than an eighth of all units.
inline int fm_order_slots(int units) { return ((units + FM_QUEUES - 1) / FM_QUEUES + 3) * FM_QUEUES; }
// Bytes of a pass's queue area: one 16-byte record per slot, then the FM_QUEUES queue counters.
inline size_t fm_order_bytes(int units) { return (size_t)fm_order_slots(units) * 16 + FM_QUEUES * 4; }
// Raise a tile-loop kernel's dynamic LDS limit once per device (the attribute belongs to the device's
// copy of the kernel); `done` is the launcher's own flag array, one flag per device.
constexpr int FM_MAX_DEVICES = 64;
inline hipError_t fm_allow_lds(const void* kernel, int bytes, bool (&done)[FM_MAX_DEVICES]) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  // The flags are shared by every host thread that calls the library: atomic accesses; two threads
  // that both find a flag clear both set the attribute, which is harmless (same value).
  if (dev >= 0 && dev < FM_MAX_DEVICES && __atomic_load_n(&done[dev], __ATOMIC_ACQUIRE)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev >= 0 && dev < FM_MAX_DEVICES) __atomic_store_n(&done[dev], true, __ATOMIC_RELEASE);
  return e;
}
// Workgroups of a tile-loop launch: one per slot plus a reserve of one eighth, through which the
// XCDs that finish their own queue early take units from the others (a workgroup that finds
// every queue empty ends at once).
inline int fm_launch_grid(int slots) { return slots + fm_order_slots(slots / 8); }
// Compute units of the current device (looked up once per device), 0 on failure.
inline int fm_compute_units() {
  static int cached[FM_MAX_DEVICES] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= FM_MAX_DEVICES) return 0;
  int n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
  }
  return n;
}
// Workgroups of a persistent tile-loop launch (every workgroup works units off until the queues are
// empty): what the chip holds at once, `per_cu` workgroups on each compute unit, rounded up to whole
// rounds of the FM_QUEUES queues; never more than the one-unit-per-workgroup launch would have.
inline int fm_persistent_grid(int slots, int per_cu) {
  const int cus = fm_compute_units();
  if (cus <= 0) return fm_launch_grid(slots);
  const int g = (cus * per_cu + FM_QUEUES - 1) / FM_QUEUES * FM_QUEUES;
  return g < fm_launch_grid(slots) ? g : fm_launch_grid(slots);
}
// Tile shapes (rows x key columns) each pass classifies at.
constexpr int FM_FWD_BR = 128, FM_FWD_BC = 64;
constexpr int FM_DQ_BR = 128;
// Key columns per tile of the dQ pass: at d = 64 a 128-key tile has the bytes (and the MFMAs) of a 64-key tile at
// d = 128, so that a tile's fixed work (copies' set-up, list entry, wait, barrier) is spread over as much math.
constexpr int fm_dq_bc(int d) { return d == 64 ? 128 : 64; }
constexpr int FM_DKDV_BR = 64, FM_DKDV_BC = 128;

// One pass's setup buffers (in the workspace) and tile shape.
struct FmSetup {
  int block_r, block_c;
  int* minmax;
  int* work;
  int* range;
  int* order;
};
// The backward's whole setup (tables, work pre-passes and unit queues of the dQ pass `rows` and of the
// dK/dV pass `cols`, whose units count K/V heads) in three launches.
hipError_t fm_launch_bwd_setup(const int* lts, const int* lte, const int* uts, const int* ute, int B, int H, int Hk,
                               int N, const FmSetup& rows, const FmSetup& cols, hipStream_t stream);
hipError_t fm_launch_preprocess(const int* lts, const int* lte, const int* uts, const int* ute, int B, int N,
                                int block_c, int* minmax, hipStream_t stream);
// Padded copies of the four bound vectors: [4][B][Np], columns >= N masked for every row.
hipError_t fm_launch_pad_bounds(const int* lts, const int* lte, const int* uts, const int* ute, int B, int N, int Np,
                                int* padded, hipStream_t stream);
hipError_t fm_launch_classify(const int* minmax, int B, int N, int block_r, int block_c, uint8_t* cls,
                              hipStream_t stream);
// work: int[B * T_r] (resp. B * T_c); range: int[2 * B * T] = first live block and one past the
// last live block of every unit (0, 0 if none); order: fm_order_bytes(B*H*T) bytes = the slot
// records {unit, first, last, 0} followed by the queue counters (zeroed here).
hipError_t fm_launch_row_order(const int* minmax, int B, int H, int Hk, int N, int block_r, int block_c, int* work,
                               int* range, int* order, hipStream_t stream);
hipError_t fm_launch_col_order(const int* minmax, int B, int H, int N, int block_r, int block_c, int* work,
                               int* range, int* order, hipStream_t stream);

// Measurement aid (fm_probe.hip): `workgroups` x 4 waves each issue iters x fm_mfma_ceiling_ops_per_iter()
// MFMA slots (shape 0: one 32x32x16 bf16 instruction; 1: two of the 16x16x32 shape, the same floating-point
// operations; 2: shape 0 plus the forward loop's side work per MFMA) on the operands given
// (2 * 8 * 64 * 16 bytes), one float per thread into sink.
hipError_t fm_launch_mfma_ceiling(const void* operands, float* sink, int workgroups, int iters, int shape,
                                  hipStream_t stream);
int fm_mfma_ceiling_ops_per_iter();
// Measurement aid: `workgroups` workgroups each add `tiles` 64 x 128 fp32 tiles into acc
// ([heads][n_tiles][64][128] floats) with no-return atomic adds.
hipError_t fm_launch_atomic_ceiling(float* acc, int n_tiles, int tiles, int heads, int workgroups, hipStream_t stream);

// Element strides of a bf16 tensor indexed [batch][head][row][d] (d contiguous).
struct FmStride {
  long long b, h, n;
};

// `general` selects the kernel instantiations that honour the stride fields and Hk (number of
// K/V heads, H % Hk == 0: query head h reads K/V head h / (H / Hk)); otherwise every tensor is
// contiguous [B,H,N,d], Hk == H, and the strides are compile-time constants of the kernels.
// N is the true sequence length (stride of the tensors), Np = N rounded up to a multiple of 128: the
// length the tile loops and the tables work at.  When Np > N the bound vectors are the library's
// padded copies [B][Np] whose extra columns are masked for every row.
struct FmFwdArgs {
  const void *q, *k, *v;
  const int *lts, *lte, *uts, *ute;   // [B][Np]
  const int* minmax;  // [B][8][T_c] at FM_FWD_BC
  int* order;         // queue slots {unit (b*H + h)*T_r + i or -1, first live key block, last + 1, 0}, then the
                      // queue counters; a row block is fully masked outside [first, last)
  void* out;
  float* lse;
  float scale;
  int B, H, N, Np, d;
  int slots;
  bool general;
  int Hk;
  FmStride sq, sk, sv, so;
};
hipError_t fm_launch_fwd(const FmFwdArgs& a, hipStream_t stream);

struct FmBwdArgs {
  const void *q, *k, *v, *out, *dout;
  const float* lse;
  const int *lts, *lte, *uts, *ute;
  const int* minmax_dq;    // [B][8][T_c] at fm_dq_bc(d)
  int* order_dq;           // queue slots and counters of the dQ pass (live key-block range per row block)
  const int* minmax_dkdv;  // [B][8][T_c] at FM_DKDV_BC
  int* order_dkdv;         // queue slots and counters of the dK/dV pass (live row-block range per key block)
  float* dvec;             // -D = -rowsum(dO o O), [B,H,Np] (stored negated; 0 in the padding): written by the
                           // dQ loop's prologue, read by the dK/dV loop
  float* lse2;             // lse * log2(e), +inf where lse = -inf and in the padding, [B,H,Np]: likewise
  void *dq, *dk, *dv;
  float scale;
  int B, H, N, Np, d;
  int slots_dq, slots_dkdv;
  bool general;
  int Hk;
  FmStride sq, sk, sv, so, sdo, sdq, sdk, sdv;
};
hipError_t fm_launch_bwd_dq(const FmBwdArgs& a, hipStream_t stream);
hipError_t fm_launch_bwd_dkdv(const FmBwdArgs& a, hipStream_t stream);
