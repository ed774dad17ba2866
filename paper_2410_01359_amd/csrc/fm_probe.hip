// Measurement aid: the matrix-core ceiling this chip reaches on its own.
//
// A kernel that does nothing but v_mfma_f32_32x32x16_bf16 on caller-given (random) operands, in the
// launch shape of the tile loops (256-thread workgroups, the whole chip filled), so that a benchmark
// can put the tile loops' rate next to what the matrix cores deliver under their own power draw and
// clock, not only next to the data-sheet peak.
#include "fm_common.h"
#include "fm_kernels.h"

namespace fm {

// Every wave keeps CHAINS independent accumulators going (the tile loops have two to four) and rotates
// through NOPS operand pairs held in registers.  `operands`: 2 * NOPS * 64 lanes * 16 bytes, read once;
// `sink`: one float per thread, written once, so that nothing is optimised away.
// SMALL: the 16x16x32 shape instead (half the floating-point operations per instruction, so two per slot).
// MIX: every slot also carries what the forward loop carries per MFMA, in independent instructions the
// hardware can overlap freely -- one 128-bit LDS operand read, four fp32 multiply-adds, one exponential --
// so the result is the rate of that instruction mix under perfect scheduling.
template <int CHAINS, int NOPS, bool SMALL, bool MIX>
__global__ __launch_bounds__(256, 2) void mfma_ceiling_kernel(const bf16x8* __restrict__ operands, float* __restrict__ sink,
                                                              int iters) {
  __shared__ __attribute__((aligned(16))) char lds[MIX ? 32768 : 16];
  const int lane = threadIdx.x & 63;
  if (MIX) {
    for (int i = threadIdx.x; i < 2048; i += 256) ((bf16x8*)lds)[i] = operands[i & 1023];
    __syncthreads();
  }
  float v[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = lane * 0.001f + j * 0.37f;
  const unsigned laddr = lds_address(lds) + lane * 16;
  bf16x8 a[NOPS], b[NOPS];
#pragma unroll
  for (int i = 0; i < NOPS; ++i) {
    a[i] = operands[(2 * i) * 64 + lane];
    b[i] = operands[(2 * i + 1) * 64 + lane];
  }
  f32x16 acc[CHAINS];
  f32x4 acc4[2 * CHAINS];
#pragma unroll
  for (int c = 0; c < CHAINS; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
#pragma unroll
  for (int c = 0; c < 2 * CHAINS; ++c)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc4[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NOPS; ++i)
#pragma unroll
      for (int c = 0; c < CHAINS; ++c) {
        if (SMALL) {
          acc4[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(i + c) % NOPS], b[i], acc4[2 * c], 0, 0, 0);
          acc4[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(i + c + 3) % NOPS], b[i], acc4[2 * c + 1], 0, 0, 0);
        } else {
          acc[c] = mfma32(a[(i + c) % NOPS], b[i], acc[c]);
        }
        if (MIX) {
          const int s = i * CHAINS + c;
          a[(i + c + 4) % NOPS] = lds_read_row16(laddr + (s * 1024 & 32767));   // lane * 16 + s * 1024 < 32768
          v[s % 16] = fast_exp2(v[s % 16] * 0.001f);
          v[(s + 9) % 16] = __builtin_fmaf(v[(s + 9) % 16], 0.9999f, 0.02f);
          v[(s + 13) % 16] = __builtin_fmaf(v[(s + 13) % 16], 1.0001f, -0.02f);
          v[(s + 1) % 16] = __builtin_fmaf(v[(s + 1) % 16], 0.9999f, 0.01f);
          v[(s + 5) % 16] = __builtin_fmaf(v[(s + 5) % 16], 1.0001f, -0.01f);
        }
        // keep the slots in source order: consecutive MFMAs then always belong to different accumulation
        // chains (left to itself the scheduler may group a chain's dependent MFMAs, which stall each other)
        __builtin_amdgcn_sched_barrier(0);
      }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += v[j];
#pragma unroll
  for (int i = 0; i < NOPS; ++i) s += (float)a[i][0];
#pragma unroll
  for (int c = 0; c < CHAINS; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[c][r];
#pragma unroll
  for (int c = 0; c < 2 * CHAINS; ++c)
#pragma unroll
    for (int r = 0; r < 4; ++r) s += acc4[c][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// What accumulating dQ from the column-parallel loop, as Algorithm 2 writes it, would cost on this chip:
// every workgroup adds `tiles` tiles of 64 x 128 fp32 (one per 64-row x 128-key tile of the dK/dV loop) into
// a [heads][n_tiles][64][128] accumulator with no-return fp32 atomic adds, in the register layout the dK/dV
// loop would hold such a tile in (32 adds of 64 lanes per wave and tile).  A head's adds all come from
// workgroups of one XCD (workgroup x works on head x % heads), as the unit queues would arrange it.
__global__ __launch_bounds__(256) void atomic_ceiling_kernel(float* __restrict__ acc, int n_tiles, int tiles, int heads) {
  const int x = blockIdx.x, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 31, g = lane >> 5;
  float* base = acc + (size_t)(x % heads) * n_tiles * 64 * 128;
  for (int t = 0; t < tiles; ++t) {
    float* tp = base + (size_t)(((x / 8) * 2 + t) % n_tiles) * 64 * 128;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * (w & 1) + 8 * (r >> 2) + 4 * g + (r & 3);
        const int col = 64 * (w >> 1) + 32 * db + c;
        unsafeAtomicAdd(tp + row * 128 + col, (float)(r + db));
      }
  }
}

}  // namespace fm

hipError_t fm_launch_atomic_ceiling(float* acc, int n_tiles, int tiles, int heads, int workgroups, hipStream_t stream) {
  hipLaunchKernelGGL(fm::atomic_ceiling_kernel, dim3(workgroups), dim3(256), 0, stream, acc, n_tiles, tiles, heads);
  return hipGetLastError();
}

// MFMAs one wave issues per loop iteration.
constexpr int kChains = 4, kOps = 8;

hipError_t fm_launch_mfma_ceiling(const void* operands, float* sink, int workgroups, int iters, int shape,
                                  hipStream_t stream) {
  const fm::bf16x8* ops = (const fm::bf16x8*)operands;
  if (shape == 1)
    hipLaunchKernelGGL((fm::mfma_ceiling_kernel<kChains, kOps, true, false>), dim3(workgroups), dim3(256), 0, stream, ops, sink, iters);
  else if (shape == 2)
    hipLaunchKernelGGL((fm::mfma_ceiling_kernel<kChains, kOps, false, true>), dim3(workgroups), dim3(256), 0, stream, ops, sink, iters);
  else
    hipLaunchKernelGGL((fm::mfma_ceiling_kernel<kChains, kOps, false, false>), dim3(workgroups), dim3(256), 0, stream, ops, sink, iters);
  return hipGetLastError();
}
int fm_mfma_ceiling_ops_per_iter() { return kChains * kOps; }
